// Instantiation of the bf16 expert kernels for one weight format (a translation unit of its own so
// that the formats compile in parallel).
#include "experts_bf16_tile.h"

namespace qmoe {
namespace bf16k {
template void launch_expert_kernels<WF_MXFP4>(bool, int, bool, const BArgs &, hipStream_t);
}  // namespace bf16k
}  // namespace qmoe

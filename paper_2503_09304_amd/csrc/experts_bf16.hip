// bf16 expert path: launch dispatch, the plane reduction of the K-split down projection, and the
// weight re-layout kernel.  The GEMM kernels themselves are the templates of experts_bf16_tile.h.
#include <vector>

#include "experts_bf16_tile.h"

namespace qmoe {
namespace {

using bf16k::BArgs;
using bf16k::f32x4;

// out[r,:] = ((p0 + p1) + p2) + p3 (or p0 + p1 with two planes) for the rows of the segments.
struct ReduceArgs {
    int nseg;
    Seg seg[kMaxSegs];
};

__global__ __launch_bounds__(256) void reduce_planes(const ReduceArgs b, const float *__restrict__ part, float *__restrict__ out,
                                                     int H, int ksplit, long plane) {
    const Seg g = b.seg[blockIdx.y];
    const int per_row = H >> 2;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < (long)g.rows * per_row; i += (long)gridDim.x * 256) {
        const long off = ((long)g.row0 * H) + i * 4;
        const f32x4 a = *reinterpret_cast<const f32x4 *>(part + off);
        const f32x4 p1 = *reinterpret_cast<const f32x4 *>(part + plane + off);
        f32x4 v;
        if (ksplit == 4) {
            const f32x4 p2 = *reinterpret_cast<const f32x4 *>(part + 2 * plane + off);
            const f32x4 p3 = *reinterpret_cast<const f32x4 *>(part + 3 * plane + off);
#pragma unroll
            for (int q = 0; q < 4; ++q) v[q] = ((a[q] + p1[q]) + p2[q]) + p3[q];
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) v[q] = a[q] + p1[q];
        }
        *reinterpret_cast<f32x4 *>(out + off) = v;
    }
}

// Re-layout of [E][R][K] row-major bf16 into the packed block order: one thread per 16-byte piece.
__global__ __launch_bounds__(256) void pack_weights_bf16(const uint4 *__restrict__ src, uint4 *__restrict__ dst, long pieces,
                                                         int R, int K) {
    const long i = (long)blockIdx.x * 256 + threadIdx.x;   // destination piece index
    if (i >= pieces) return;
    const long per_expert = (long)R * K / 8;
    const long e = i / per_expert, q = i - e * per_expert;
    const int lane = (int)(q & 63);
    const long blk = q >> 6;                                // nt * (K/16) + kstep
    const int ksteps = K / 16;
    const long nt = blk / ksteps;
    const int ks = (int)(blk - nt * ksteps);
    const long r = nt * 32 + (lane & 31);
    const int k = ks * 16 + (lane >> 5) * 8;
    dst[i] = src[(e * R + r) * (K / 8) + k / 8];
}

// Re-layout of 4-bit weights: one thread per 16-byte piece of the destination (expert, row tile,
// iteration, lane); lanes of the lower k-half also write their row's two scale bytes.
__global__ __launch_bounds__(256) void pack_weights_mxfp4(const uint8_t *__restrict__ codes, const uint8_t *__restrict__ scales,
                                                          uint4 *__restrict__ dcodes, uint16_t *__restrict__ dscales,
                                                          long pieces, int R, int K) {
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= pieces) return;
    const int lane = (int)(i & 63);
    const long blk = i >> 6;                                // (e * R/32 + nt) * K/64 + it
    const int kb = K >> 6;
    const int it = (int)(blk % kb);
    const long row_tile = blk / kb;                         // e * R/32 + nt
    const long row = row_tile * 32 + (lane & 31);           // e * R + r
    const int lh = lane >> 5;
    const uint8_t *src = codes + (row * K + it * 64 + lh * 8) / 2;
    uint4 v;
    v.x = *reinterpret_cast<const uint32_t *>(src);
    v.y = *reinterpret_cast<const uint32_t *>(src + 8);
    v.z = *reinterpret_cast<const uint32_t *>(src + 16);
    v.w = *reinterpret_cast<const uint32_t *>(src + 24);
    dcodes[i] = v;
    if (lh == 0) {
        const uint8_t *sp = scales + row * (K >> 5) + it * 2;
        dscales[blk * 32 + lane] = (uint16_t)(sp[0] | (sp[1] << 8));
    }
}

}  // namespace

hipError_t launch_reduce_planes(const Seg *segs, int nseg, const float *partial, float *out, int H, int ksplit, long plane,
                                hipStream_t s) {
    for (int i = 0; i < nseg; i += kMaxSegs) {
        ReduceArgs r{};
        r.nseg = std::min(kMaxSegs, nseg - i);
        int max_rows = 1;
        for (int j = 0; j < r.nseg; ++j) { r.seg[j] = segs[i + j]; max_rows = std::max(max_rows, (int)segs[i + j].rows); }
        const int per_seg = std::max(1, std::min(64, (max_rows * (H / 4) + 255) / 256));
        hipLaunchKernelGGL(reduce_planes, dim3(per_seg, r.nseg), dim3(256), 0, s, r, partial, out, H, ksplit, plane);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_pack_mxfp4(const void *codes, const void *scales, void *dcodes, void *dscales, int E, int R, int K,
                             hipStream_t s) {
    const long pieces = (long)E * (R / 32) * (K / 64) * 64;
    hipLaunchKernelGGL(pack_weights_mxfp4, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, s, (const uint8_t *)codes,
                       (const uint8_t *)scales, (uint4 *)dcodes, (uint16_t *)dscales, pieces, R, K);
    return hipGetLastError();
}

hipError_t launch_pack(const void *src, void *dst, int E, int R, int K, hipStream_t s) {
    const long pieces = (long)E * R * K / 8;
    hipLaunchKernelGGL(pack_weights_bf16, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, s, (const uint4 *)src,
                       (uint4 *)dst, pieces, R, K);
    return hipGetLastError();
}

// Columns per wave of a gate-up launch.  A workgroup stays on its CU for the whole of K, so a launch
// costs whole rounds of the chip's CUs, and a weight-streaming launch moves bytes in proportion to
// rounds x columns per workgroup.  Narrower waves (28 .. 16 columns on the 32-wide MFMA; the idle MFMA
// rows cost nothing where the stream is the bound) are taken when they make the last round full:
// 8 experts x 14336 columns are 896 workgroups of 128 columns = 3.5 rounds of 256 CUs, but exactly 4
// rounds of 112 columns (decode gate-up 0.321 -> 0.293 ms).  Only segments of at most 3 token tiles
// are bound by the stream alone: from 4 tiles on an iteration takes as long for 28 columns as for 32,
// launches whose segments share weights are MFMA-bound, and with 4-bit weights an iteration's
// conversions, not its bytes, set the pace (decode gate-up 0.109 -> 0.112 ms); those keep 32.
static int gate_up_wave_columns(bool stream, int wfmt, int tiles, int nseg, int F) {
    if (!stream || tiles > 3 || wfmt == bf16k::WF_MXFP4) return 32;
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 1) v = 256;
        cus = v;
    }
    int best = 32;
    long best_cost = 0;
    for (int cw = 32; cw >= 16; cw -= 4) {
        const long wgs = (long)nseg * ((F + 4 * cw - 1) / (4 * cw));
        if (wgs <= cus && cw < 32) break;            // a single round: nothing to even out
        const long cost = (wgs + cus - 1) / cus * cw;
        if (cw == 32 || cost < best_cost) { best = cw; best_cost = cost; }
    }
    return best;
}

void launch_experts_bf16(const ExpertArgs &a, const KArgs &gu_in, const KArgs &dn_in, hipStream_t s) {
    BArgs b{};
    b.ksplit = 1;
    b.plane = 0;
    b.nseg = a.segs ? a.nseg : 0;
    if (b.nseg > 0) {
        // Packets are groups of 4 consecutive segments.  Where an expert has several segments, its
        // groups are padded with empty segments so that no packet spans two experts: the workgroups
        // of a packet then share one set of weight tiles, fetched into that XCD's L2 once.
        int n = 0;
        bool shared = false;
        for (int i = 1; i < a.nseg; ++i) shared = shared || a.segs[i].expert == a.segs[i - 1].expert;
        if (shared) {
            // experts in descending order of their rows in this launch (the order of experts is free:
            // the busiest ones start first, the small ones fill the tail), each expert's segments
            // kept together and in row order
            struct Group { int first, count, rows; };
            std::vector<Group> groups;
            for (int i = 0; i < a.nseg; ++i) {
                if (i == 0 || a.segs[i].expert != a.segs[i - 1].expert) groups.push_back(Group{i, 0, 0});
                groups.back().count += 1;
                groups.back().rows += a.segs[i].rows;
            }
            std::stable_sort(groups.begin(), groups.end(), [](const Group &x, const Group &y) { return x.rows > y.rows; });
            for (const Group &g : groups) {
                while ((n & ((1 << QMOE_PK_U) - 1)) && n < kMaxSegs) b.seg[n++] = Seg{0, 0, 0};
                for (int i = g.first; i < g.first + g.count; ++i) {
                    if (n < kMaxSegs) b.seg[n] = a.segs[i];
                    ++n;
                }
                if (n > kMaxSegs) break;
            }
        }
        if (!shared || n > kMaxSegs) {
            std::copy(a.segs, a.segs + a.nseg, b.seg);
            n = a.nseg;
        }
        b.nseg = n;
    }
    const int tiles = (a.max_rows + 31) / 32;
    const unsigned n = b.nseg > 0 ? (unsigned)b.nseg : a.nu;
    // segments are sorted by expert: the weights are streamed once iff no two neighbours share one
    bool stream = b.nseg > 0;
    for (int i = 1; i < b.nseg; ++i) stream = stream && b.seg[i].expert != b.seg[i - 1].expert;
    // With one segment per expert the order of the segments is free: longest first, so that the
    // workgroups with the most tiles do not form the tail of the launch.
    if (stream) std::stable_sort(b.seg, b.seg + b.nseg, [](const Seg &x, const Seg &y) { return x.rows > y.rows; });

    b.k = gu_in;
    b.k.cw = a.wave_cols ? a.wave_cols : gate_up_wave_columns(stream, a.wfmt, tiles, (int)n, a.F);
    b.k.col_tiles = (a.F + 4 * b.k.cw - 1) / (4 * b.k.cw);
    auto launch = [&](bool gateup) {
        if (a.wfmt == bf16k::WF_MXFP4) bf16k::launch_expert_kernels<bf16k::WF_MXFP4>(gateup, tiles, stream, b, s);
        else if (a.wfmt == bf16k::WF_PACKED) bf16k::launch_expert_kernels<bf16k::WF_PACKED>(gateup, tiles, stream, b, s);
        else bf16k::launch_expert_kernels<bf16k::WF_ROWMAJOR>(gateup, tiles, stream, b, s);
    };
    { Scope sc(a.prof, MOE_PROF_GATE_UP, s); launch(true); }

    const int gu_col_tiles = b.k.col_tiles;
    b.k = dn_in;
    b.k.need = gu_col_tiles;         // gate-up workgroups per row range
    b.k.cw = 32;
    b.k.col_tiles = (a.H + 255) / 256;
    if (a.ksplit > 1 && a.partial != nullptr) {
        b.ksplit = a.ksplit;
        b.plane = a.plane;
        b.k.dst = a.partial;
        // the planes stay apart: moe_combine adds them in the fixed order ((p0+p1)+p2)+p3 as it reads them
        Scope sc(a.prof, MOE_PROF_DOWN, s);
        launch(false);
    } else {
        Scope sc(a.prof, MOE_PROF_DOWN, s);
        launch(false);
    }
}

}  // namespace qmoe

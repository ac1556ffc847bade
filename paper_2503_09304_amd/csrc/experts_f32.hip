// fp32 expert kernels: plain LDS-tiled FMA GEMMs (64x64 tile, K ascending, one accumulator chain
// per output), SwiGLU fused into the gate-up epilogue.  Used by the fp32 configuration, which is a
// correctness case: its sizes are bound by launch latency, not by any roofline.
#include <hip/hip_runtime.h>

#include "experts_common.h"

namespace qmoe {
namespace {

// ------------------------------------------------------------------------------------------------
// fp32 FMA kernel: 64 rows x 64 columns per workgroup, 4x4 per thread, K in steps of 16.
// ------------------------------------------------------------------------------------------------
template <bool GATEUP>
__global__ __launch_bounds__(256) void expert_f32(const KArgs p, int row_tiles) {
    __shared__ int s_run;
    __shared__ float As[16][65];
    __shared__ float B0s[16][65];
    __shared__ float B1s[GATEUP ? 16 : 1][65];
    int bid = blockIdx.x;
    const int ct = bid % p.col_tiles; bid /= p.col_tiles;
    const int rt = bid % row_tiles;
    const int ui = bid / row_tiles;
    const moe_unit un = p.units[p.u0 + ui];
    const int r0 = rt * 64;
    if (r0 >= un.rows) return;
    if (!wg_may_run(p, un.row0, (un.rows + 63) >> 6, &s_run)) return;
    const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
    const float *b0 = (const float *)p.b0 + (long)un.expert * p.b_estride;
    const float *b1 = GATEUP ? (const float *)p.b1 + (long)un.expert * p.b_estride : nullptr;

    // staging assignment: element (row tid/4 , k 4*(tid%4) + i)
    const int lrow = tid >> 2, lk = (tid & 3) * 4;
    const int arow_i = r0 + lrow;
    const bool arow_ok = arow_i < un.rows;
    long a_src_row = 0;
    if (arow_ok) a_src_row = GATEUP ? (long)(p.perm[un.row0 + arow_i] / p.kdiv) : (long)(un.row0 + arow_i);
    const float *ap = (const float *)p.a_src + a_src_row * p.lda;
    const int bcol = ct * 64 + lrow;
    const bool bcol_ok = bcol < p.ncols;

    float g[4][4], u[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) g[i][j] = u[i][j] = 0.f;

    for (int k0 = 0; k0 < p.K; k0 += 16) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int kk = k0 + lk + i;
            const bool kok = kk < p.K;
            As[lk + i][lrow] = (arow_ok && kok) ? ap[kk] : 0.f;
            B0s[lk + i][lrow] = (bcol_ok && kok) ? b0[(long)bcol * p.K + kk] : 0.f;
            if (GATEUP) B1s[lk + i][lrow] = (bcol_ok && kok) ? b1[(long)bcol * p.K + kk] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float av[4], bv[4], cv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) av[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) { bv[j] = B0s[kk][tx * 4 + j]; cv[j] = GATEUP ? B1s[kk][tx * 4 + j] : 0.f; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    g[i][j] = fmaf(av[i], bv[j], g[i][j]);
                    if (GATEUP) u[i][j] = fmaf(av[i], cv[j], u[i][j]);
                }
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = r0 + ty * 4 + i;
        if (r >= un.rows) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = ct * 64 + tx * 4 + j;
            if (c >= p.ncols) continue;
            float *d = (float *)p.dst + (long)(un.row0 + r) * p.ldd + c;
            if (GATEUP) *d = (g[i][j] / (1.f + expf(-g[i][j]))) * u[i][j];
            else *d = g[i][j];
        }
    }
}

}  // namespace

void launch_experts_f32(const ExpertArgs &a, const KArgs &gu_in, const KArgs &dn_in, hipStream_t s) {
    KArgs gu = gu_in, dn = dn_in;
    const int row_tiles = (a.max_rows + 63) / 64;
    gu.col_tiles = (a.F + 63) / 64;
    dn.col_tiles = (a.H + 63) / 64;
    dn.need = gu.col_tiles;          // gate-up workgroups per 64-row tile
    { Scope sc(a.prof, MOE_PROF_GATE_UP, s);
      hipLaunchKernelGGL(expert_f32<true>, dim3(a.nu * row_tiles * gu.col_tiles), dim3(256), 0, s, gu, row_tiles); }
    { Scope sc(a.prof, MOE_PROF_DOWN, s);
      hipLaunchKernelGGL(expert_f32<false>, dim3(a.nu * row_tiles * dn.col_tiles), dim3(256), 0, s, dn, row_tiles); }
}

}  // namespace qmoe

// Expert work: for every row r of a work unit of expert e (token n = perm[r] / k)
//     act[r,:] = silu(W1[e] x[n,:]) (.) (W3[e] x[n,:])        ("gate-up" kernel, SwiGLU fused)
//     out[r,:] = W2[e] act[r,:]                               ("down" kernel)
// Independent per-expert execution over the per-expert queues (Introduction, "Novel MoE Layer
// Design"; Sec. 3.3), one launch covering the units [u0, u0+nu) handed over by the cursor.
//
// bf16 path.  All three weight matrices are [rows_out, K] with K contiguous, and so are the
// activations, so both MFMA operands are read 8 consecutive K-elements (16 bytes) per lane with no
// transposition.  v_mfma_f32_32x32x16_bf16: A = 32 tokens x 16 k, B = 32 weight rows x 16 k,
// D[token, weight row] in fp32.  A workgroup has 4 waves; each wave owns 64 weight rows (gate-up:
// 32 rows of W1 and the same 32 of W3, so gate and up of one (token, f) meet in one lane and
// register) and every token tile of the unit.  Weight fragments go straight from global memory
// into MFMA operand registers: no wave shares them, so staging them in LDS would only add traffic.
// The token tile (gathered x rows, or act rows) is shared by the 4 waves and is staged in LDS, its
// 16-byte slots XOR-swizzled by row so that the 32 rows read by one ds_read_b128 hit distinct banks.
//
// Determinism.  Each output element is one chain of MFMA accumulations over K in ascending order
// (down projection of small units: 4 such chains over contiguous quarters of K, added in a fixed
// order).  Which variant a unit takes depends on the unit's own row count and the configuration
// only, and tiles never mix units, so results are bit-identical however the unit list is split
// into launches.
//
// fp32 path: plain LDS-tiled FMA kernel (64x64 tile, K ascending), used for small checks.
#include <hip/hip_runtime.h>

#include "qmoe_internal.h"

namespace qmoe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float silu_f(float z) { return z / (1.f + __expf(-z)); }

struct KArgs {
    const void *a_src;      // x [N,H] (gate-up) or act [A,F] (down)
    const int32_t *perm;    // gate-up: sorted row -> assignment id; down: nullptr
    const void *b0, *b1;    // gate-up: W1, W3; down: W2, unused
    void *dst;              // gate-up: act; down: out (fp32)
    const moe_unit *units;
    long b_estride;         // elements per expert in b0/b1
    int lda, K, ncols, ldd, kdiv;
    unsigned u0;
    int col_tiles;
    int cls_filter;         // 0 = every unit, 1 = only rows <= kSmallUnitRows, 2 = only larger
};

// ------------------------------------------------------------------------------------------------
// bf16 MFMA kernel
// ------------------------------------------------------------------------------------------------
template <int TMAX, bool GATEUP, int WK>
__global__ __launch_bounds__(256) void expert_bf16(const KArgs p) {
    constexpr int WN = 4 / WK;
    constexpr int ROWS = TMAX * 32;
    constexpr int COLS_PER_WAVE = GATEUP ? 32 : 64;
    __shared__ __attribute__((aligned(16))) uint16_t lds_a[WK * ROWS * 64];
    __shared__ float lds_red[(WK > 1) ? 3 * TMAX * 2 * 16 * 64 : 1];

    const int ui = blockIdx.x / p.col_tiles, ct = blockIdx.x - ui * p.col_tiles;
    const moe_unit un = p.units[p.u0 + ui];
    const int rows = un.rows;
    if (p.cls_filter == 1 && rows > kSmallUnitRows) return;
    if (p.cls_filter == 2 && rows <= kSmallUnitRows) return;
    const int t_cnt = (rows + 31) >> 5;

    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
    const int wn = w % WN, wk = w / WN;
    const int lr = l & 31, lh = l >> 5;
    const int Kg = p.K / WK;
    const int iters = Kg / 64;

    // ---- weight rows of this lane (B operand) ----
    const uint16_t *brow[2];
    const int col_base = ct * (WN * COLS_PER_WAVE) + wn * COLS_PER_WAVE;
    {
        const uint16_t *b0 = (const uint16_t *)p.b0 + (long)un.expert * p.b_estride;
        if (GATEUP) {
            const uint16_t *b1 = (const uint16_t *)p.b1 + (long)un.expert * p.b_estride;
            const int c = min(col_base + lr, p.ncols - 1);
            brow[0] = b0 + (long)c * p.K + wk * Kg + lh * 8;
            brow[1] = b1 + (long)c * p.K + wk * Kg + lh * 8;
        } else {
            const int c0 = min(col_base + lr, p.ncols - 1), c1 = min(col_base + 32 + lr, p.ncols - 1);
            brow[0] = b0 + (long)c0 * p.K + wk * Kg + lh * 8;
            brow[1] = b0 + (long)c1 * p.K + wk * Kg + lh * 8;
        }
    }
    // ---- token rows this thread stages into LDS (A operand): row tid/8 + 32*j, slot tid%8 ----
    const int srow = tid >> 3, sslot = tid & 7;
    const uint16_t *arow[TMAX];
#pragma unroll
    for (int j = 0; j < TMAX; ++j) {
        int r = srow + 32 * j;
        if (r > rows - 1) r = rows - 1;
        long src_row;
        if (GATEUP) src_row = p.perm[un.row0 + r] / p.kdiv;
        else src_row = un.row0 + r;
        arow[j] = (const uint16_t *)p.a_src + src_row * p.lda + sslot * 8;
    }

    f32x16 acc[TMAX][2];
#pragma unroll
    for (int t = 0; t < TMAX; ++t)
#pragma unroll
        for (int n = 0; n < 2; ++n)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][n][r] = 0.f;

    uint4 a_reg[WK][TMAX];
    bf16x8 b_reg[4][2];

    auto load_global = [&](int it) {
#pragma unroll
        for (int g = 0; g < WK; ++g)
#pragma unroll
            for (int j = 0; j < TMAX; ++j)
                if (j < t_cnt) a_reg[g][j] = *reinterpret_cast<const uint4 *>(arow[j] + g * Kg + it * 64);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            b_reg[ks][0] = *reinterpret_cast<const bf16x8 *>(brow[0] + it * 64 + ks * 16);
            b_reg[ks][1] = *reinterpret_cast<const bf16x8 *>(brow[1] + it * 64 + ks * 16);
        }
    };

    load_global(0);
    for (int it = 0; it < iters; ++it) {
        __syncthreads();  // previous tile fully consumed
#pragma unroll
        for (int g = 0; g < WK; ++g)
#pragma unroll
            for (int j = 0; j < TMAX; ++j)
                if (j < t_cnt) {
                    const int r = srow + 32 * j;
                    *reinterpret_cast<uint4 *>(&lds_a[((g * ROWS + r) * 8 + (sslot ^ (r & 7))) * 8]) = a_reg[g][j];
                }
        bf16x8 b_cur[4][2];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) { b_cur[ks][0] = b_reg[ks][0]; b_cur[ks][1] = b_reg[ks][1]; }
        __syncthreads();
        if (it + 1 < iters) load_global(it + 1);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
            for (int t = 0; t < TMAX; ++t) {
                if (t < t_cnt) {
                    const int r = t * 32 + lr;
                    const int slot = (ks * 2 + lh) ^ (r & 7);
                    const bf16x8 a = *reinterpret_cast<const bf16x8 *>(&lds_a[((wk * ROWS + r) * 8 + slot) * 8]);
                    acc[t][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b_cur[ks][0], acc[t][0], 0, 0, 0);
                    acc[t][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b_cur[ks][1], acc[t][1], 0, 0, 0);
                }
            }
        }
    }

    // ---- K-split: add the 4 partial tiles in wave order ----
    if (WK > 1) {
        if (wk > 0) {
#pragma unroll
            for (int t = 0; t < TMAX; ++t)
#pragma unroll
                for (int n = 0; n < 2; ++n)
#pragma unroll
                    for (int r = 0; r < 16; ++r) lds_red[(((wk - 1) * TMAX + t) * 2 + n) * 1024 + r * 64 + l] = acc[t][n][r];
        }
        __syncthreads();
        if (wk > 0) return;
#pragma unroll
        for (int t = 0; t < TMAX; ++t)
#pragma unroll
            for (int n = 0; n < 2; ++n)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float v = acc[t][n][r];
                    v += lds_red[((0 * TMAX + t) * 2 + n) * 1024 + r * 64 + l];
                    v += lds_red[((1 * TMAX + t) * 2 + n) * 1024 + r * 64 + l];
                    v += lds_red[((2 * TMAX + t) * 2 + n) * 1024 + r * 64 + l];
                    acc[t][n][r] = v;
                }
    }

    // ---- epilogue.  D register r of lane l: token 8*(r/4) + 4*(l/32) + r%4, weight row l%32 ----
#pragma unroll
    for (int t = 0; t < TMAX; ++t) {
        if (t < t_cnt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = t * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                if (i < rows) {
                    if (GATEUP) {
                        const int f = col_base + lr;
                        if (f < p.ncols) {
                            const float m = silu_f(acc[t][0][r]) * acc[t][1][r];
                            ((__bf16 *)p.dst)[(long)(un.row0 + i) * p.ldd + f] = (__bf16)m;
                        }
                    } else {
                        const int h0 = col_base + lr, h1 = h0 + 32;
                        float *o = (float *)p.dst + (long)(un.row0 + i) * p.ldd;
                        if (h0 < p.ncols) o[h0] = acc[t][0][r];
                        if (h1 < p.ncols) o[h1] = acc[t][1][r];
                    }
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// fp32 FMA kernel: 64 rows x 64 columns per workgroup, 4x4 per thread, K in steps of 16.
// ------------------------------------------------------------------------------------------------
template <bool GATEUP>
__global__ __launch_bounds__(256) void expert_f32(const KArgs p, int row_tiles) {
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

template <int TMAX, bool GATEUP, int WK>
void launch_bf16(const KArgs &k, unsigned nu, hipStream_t s) {
    hipLaunchKernelGGL((expert_bf16<TMAX, GATEUP, WK>), dim3(nu * (unsigned)k.col_tiles), dim3(256), 0, s, k);
}

template <bool GATEUP, int WK>
void launch_bf16_t(int tmax, const KArgs &k, unsigned nu, hipStream_t s) {
    if (tmax <= 1) launch_bf16<1, GATEUP, WK>(k, nu, s);
    else if (tmax <= 2 || WK > 1) launch_bf16<2, GATEUP, WK>(k, nu, s);   // K-split variants serve small units only
    else if constexpr (WK == 1) {
        if (tmax <= 4) launch_bf16<4, GATEUP, WK>(k, nu, s);
        else launch_bf16<8, GATEUP, WK>(k, nu, s);
    }
}

}  // namespace

hipError_t launch_experts(const ExpertArgs &a, hipStream_t s) {
    if (a.nu == 0) return hipSuccess;
    KArgs gu{};
    gu.a_src = a.x; gu.perm = a.perm; gu.b0 = a.W1; gu.b1 = a.W3; gu.dst = a.act; gu.units = a.units;
    gu.b_estride = (long)a.F * a.H; gu.lda = a.H; gu.K = a.H; gu.ncols = a.F; gu.ldd = a.F; gu.kdiv = a.k;
    gu.u0 = a.u0; gu.cls_filter = 0;
    KArgs dn{};
    dn.a_src = a.act; dn.perm = nullptr; dn.b0 = a.W2; dn.b1 = nullptr; dn.dst = a.out; dn.units = a.units;
    dn.b_estride = (long)a.H * a.F; dn.lda = a.F; dn.K = a.F; dn.ncols = a.H; dn.ldd = a.H; dn.kdiv = 1;
    dn.u0 = a.u0; dn.cls_filter = 0;

    if (a.dtype == MOE_F32) {
        const int row_tiles = (a.max_rows + 63) / 64;
        gu.col_tiles = (a.F + 63) / 64;
        dn.col_tiles = (a.H + 63) / 64;
        hipLaunchKernelGGL(expert_f32<true>, dim3(a.nu * row_tiles * gu.col_tiles), dim3(256), 0, s, gu, row_tiles);
        hipLaunchKernelGGL(expert_f32<false>, dim3(a.nu * row_tiles * dn.col_tiles), dim3(256), 0, s, dn, row_tiles);
        return hipGetLastError();
    }

    const int tmax = (a.max_rows + 31) / 32;
    gu.col_tiles = (a.F + 127) / 128;
    launch_bf16_t<true, 1>(tmax, gu, a.nu, s);
    // Down projection.  Small units split K over the 4 waves (4x the workgroups, for the
    // weight-streaming shapes) when F allows it; the choice depends on the unit and F only.
    const bool ksplit = (a.F % 256) == 0;
    if (a.has_small) {
        KArgs d = dn;
        d.cls_filter = 1;
        const int ts = tmax < 2 ? tmax : 2;
        if (ksplit) { d.col_tiles = (a.H + 63) / 64; launch_bf16_t<false, 4>(ts, d, a.nu, s); }
        else { d.col_tiles = (a.H + 255) / 256; launch_bf16_t<false, 1>(ts, d, a.nu, s); }
    }
    if (a.has_large) {
        KArgs d = dn;
        d.cls_filter = 2;
        d.col_tiles = (a.H + 255) / 256;
        launch_bf16_t<false, 1>(tmax, d, a.nu, s);
    }
    return hipGetLastError();
}

}  // namespace qmoe

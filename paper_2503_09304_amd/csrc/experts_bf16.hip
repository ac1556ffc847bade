// bf16 expert kernels (gate-up with fused SwiGLU, and down projection) on MFMA.
//
// All three weight matrices are [rows_out, K] with K contiguous, and so are the activations, so
// both MFMA operands are read 8 consecutive K-elements (16 bytes) per lane with no transposition.
// v_mfma_f32_32x32x16_bf16: A = 32 tokens x 16 k, B = 32 weight rows x 16 k, D[token, weight row]
// in fp32.  A workgroup has 4 waves.  Each wave owns 64 weight rows (gate-up: 32 rows of W1 and the
// same 32 of W3, so the gate and up value of one (token, f) meet in one lane and register) and every
// token tile of the unit.  No two waves use the same weight fragment, so weights go straight from
// global memory into MFMA operand registers; only the token tile (gathered x rows, or act rows),
// which all 4 waves share, is staged in LDS, double-buffered, its 16-byte slots XOR-swizzled by
// row so that the 32 rows read by one ds_read_b128 fall into distinct banks.
//
// Pipeline of one K-iteration (64 k): write the token tile for iteration it+1 into the other LDS
// stage, issue the global loads of the token tile for it+2 and of the weight fragments for it+2
// (three register sets rotate), run the MFMAs of iteration it, one barrier.  Vector loads complete
// in issue order, so this keeps two iterations of weights (16 KB per wave) in flight.
// Loads are unconditional (row and iteration indices are clamped instead) so that the wait
// counters stay exact.
//
// Shapes bound by weight streaming need more workgroups than output tiles exist in the down
// projection: there (units of at most kSmallUnitRows rows) the 4 waves split K into 4 contiguous
// quarters and add their partial tiles through LDS in wave order.
//
// Determinism.  Each output element is one chain of MFMA accumulations over K in ascending order
// (K-split: 4 chains added in a fixed order).  Which variant a unit takes depends on the unit's own
// row count and the configuration only, and tiles never mix units, so results are bit-identical
// however the unit list is split into launches.
#include <hip/hip_runtime.h>

#include <type_traits>
#include <utility>

#include "experts_common.h"

namespace qmoe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float silu_f(float z) { return z / (1.f + __expf(-z)); }

// Compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>).  Register
// arrays are only ever indexed with these constants, so they stay in registers.
template <int N, class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
    static_for_impl<N>(f, std::make_integer_sequence<int, N>{});
}

template <int T, bool GATEUP, int WK>
__device__ __forceinline__ void expert_tile(const KArgs &p, const moe_unit un, const int ct, char *lds) {
    constexpr int WN = 4 / WK;
    constexpr int ROWS = T * 32;
    constexpr int STAGE = WK * ROWS * 128;  // bytes of one LDS stage: 64 bf16 per row
    constexpr int CPW = GATEUP ? 32 : 64;   // output columns per wave
    const int rows = un.rows;
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
    const int wn = w % WN, wk = w / WN;
    const int lr = l & 31, lh = l >> 5;
    const int Kg = p.K / WK;
    const int iters = Kg / 64;
    const int col_base = ct * (WN * CPW) + wn * CPW;

    // ---- weight rows of this lane (B operand) ----
    const uint16_t *bptr[2];
    {
        const uint16_t *b0 = (const uint16_t *)p.b0 + (long)un.expert * p.b_estride;
        if (GATEUP) {
            const uint16_t *b1 = (const uint16_t *)p.b1 + (long)un.expert * p.b_estride;
            const int c = min(col_base + lr, p.ncols - 1);
            bptr[0] = b0 + (long)c * p.K + wk * Kg + lh * 8;
            bptr[1] = b1 + (long)c * p.K + wk * Kg + lh * 8;
        } else {
            const int c0 = min(col_base + lr, p.ncols - 1), c1 = min(col_base + 32 + lr, p.ncols - 1);
            bptr[0] = b0 + (long)c0 * p.K + wk * Kg + lh * 8;
            bptr[1] = b0 + (long)c1 * p.K + wk * Kg + lh * 8;
        }
    }
    // ---- token rows this thread stages into LDS (A operand): row tid/8 + 32*j, slot tid%8 ----
    const int srow = tid >> 3, sslot = tid & 7;
    const uint16_t *arow[T];
    static_for<T>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        const int r = min(srow + 32 * j, rows - 1);
        long src_row;
        if (GATEUP) src_row = p.perm[un.row0 + r] / p.kdiv;
        else src_row = un.row0 + r;
        arow[j] = (const uint16_t *)p.a_src + src_row * p.lda + sslot * 8;
    });

    f32x16 acc[T][2];
    static_for<T>([&](auto tc) {
        constexpr int t = decltype(tc)::value;
#pragma unroll
        for (int r = 0; r < 16; ++r) { acc[t][0][r] = 0.f; acc[t][1][r] = 0.f; }
    });

    u32x4 a_reg[WK * T];
    bf16x8 b_reg[3 * 8];  // [set][k-step][n-tile]

    auto load_a = [&](int it) {
        const int itc = min(it, iters - 1);
        static_for<WK * T>([&](auto ic) {
            constexpr int g = decltype(ic)::value / T, j = decltype(ic)::value % T;
            a_reg[g * T + j] = *reinterpret_cast<const u32x4 *>(arow[j] + g * Kg + itc * 64);
        });
    };
    auto store_a = [&](int stage) {
        static_for<WK * T>([&](auto ic) {
            constexpr int g = decltype(ic)::value / T, j = decltype(ic)::value % T;
            const int r = srow + 32 * j;
            *reinterpret_cast<u32x4 *>(lds + stage * STAGE + ((g * ROWS + r) * 8 + (sslot ^ (r & 7))) * 16) = a_reg[g * T + j];
        });
    };
    auto load_b = [&](int it, auto setc) {
        constexpr int S = decltype(setc)::value;
        const int itc = min(it, iters - 1);
        static_for<4>([&](auto kc) {
            constexpr int ks = decltype(kc)::value;
            b_reg[S * 8 + ks * 2 + 0] = *reinterpret_cast<const bf16x8 *>(bptr[0] + itc * 64 + ks * 16);
            b_reg[S * 8 + ks * 2 + 1] = *reinterpret_cast<const bf16x8 *>(bptr[1] + itc * 64 + ks * 16);
        });
    };
    auto mfma_tile = [&](int stage, auto setc) {
        constexpr int S = decltype(setc)::value;
        static_for<4 * T>([&](auto ic) {
            constexpr int ks = decltype(ic)::value / T, t = decltype(ic)::value % T;
            const int r = t * 32 + lr;
            const int slot = (ks * 2 + lh) ^ (r & 7);
            const bf16x8 a = *reinterpret_cast<const bf16x8 *>(lds + stage * STAGE + ((wk * ROWS + r) * 8 + slot) * 16);
            acc[t][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b_reg[S * 8 + ks * 2 + 0], acc[t][0], 0, 0, 0);
            acc[t][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b_reg[S * 8 + ks * 2 + 1], acc[t][1], 0, 0, 0);
        });
    };
    auto body = [&](int it, auto sc) {
        constexpr int S = decltype(sc)::value;
        store_a((it + 1) & 1);
        load_a(it + 2);
        load_b(it + 2, std::integral_constant<int, (S + 2) % 3>{});
        mfma_tile(it & 1, sc);
        __syncthreads();
    };

    load_a(0);
    load_b(0, std::integral_constant<int, 0>{});
    load_b(1, std::integral_constant<int, 1>{});
    store_a(0);
    load_a(1);
    __syncthreads();
    int it = 0;
    for (; it + 3 <= iters; it += 3) {
        body(it, std::integral_constant<int, 0>{});
        body(it + 1, std::integral_constant<int, 1>{});
        body(it + 2, std::integral_constant<int, 2>{});
    }
    if (it < iters) {
        body(it, std::integral_constant<int, 0>{});
        if (it + 1 < iters) body(it + 1, std::integral_constant<int, 1>{});
    }

    // ---- K-split: add the 4 partial tiles in wave order (LDS stages are free after the last barrier)
    if (WK > 1) {
        float *red = reinterpret_cast<float *>(lds);
        if (wk > 0) {
            static_for<2 * T>([&](auto ic) {
                constexpr int t = decltype(ic)::value / 2, n = decltype(ic)::value % 2;
#pragma unroll
                for (int r = 0; r < 16; ++r) red[(((wk - 1) * T + t) * 2 + n) * 1024 + r * 64 + l] = acc[t][n][r];
            });
        }
        __syncthreads();
        if (wk > 0) return;
        static_for<2 * T>([&](auto ic) {
            constexpr int t = decltype(ic)::value / 2, n = decltype(ic)::value % 2;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float v = acc[t][n][r];
                v += red[((0 * T + t) * 2 + n) * 1024 + r * 64 + l];
                v += red[((1 * T + t) * 2 + n) * 1024 + r * 64 + l];
                v += red[((2 * T + t) * 2 + n) * 1024 + r * 64 + l];
                acc[t][n][r] = v;
            }
        });
    }

    // ---- epilogue.  D register r of lane l: token 8*(r/4) + 4*(l/32) + r%4, weight row l%32 ----
    static_for<T>([&](auto tc) {
        constexpr int t = decltype(tc)::value;
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
    });
}

// TCAP: largest number of 32-token tiles a unit of this launch may have (1, 2, 4 or 8).  A
// workgroup takes the smallest fully unrolled variant that covers its unit.
template <int TCAP, bool GATEUP, int WK>
__global__ __launch_bounds__(256) void expert_bf16(const KArgs p) {
    __shared__ __attribute__((aligned(16))) char lds[2 * WK * TCAP * 32 * 128];
    const int ui = blockIdx.x / p.col_tiles, ct = blockIdx.x - ui * p.col_tiles;
    const moe_unit un = p.units[p.u0 + ui];
    if (p.cls_filter == 1 && un.rows > kSmallUnitRows) return;
    if (p.cls_filter == 2 && un.rows <= kSmallUnitRows) return;
    const int t_cnt = (un.rows + 31) >> 5;
    if (TCAP >= 8 && t_cnt > 4) expert_tile<(TCAP >= 8 ? 8 : 1), GATEUP, WK>(p, un, ct, lds);
    else if (TCAP >= 4 && t_cnt > 2) expert_tile<(TCAP >= 4 ? 4 : 1), GATEUP, WK>(p, un, ct, lds);
    else if (TCAP >= 2 && t_cnt > 1) expert_tile<(TCAP >= 2 ? 2 : 1), GATEUP, WK>(p, un, ct, lds);
    else expert_tile<1, GATEUP, WK>(p, un, ct, lds);
}

template <int TCAP, bool GATEUP, int WK>
void launch1(const KArgs &k, unsigned nu, hipStream_t s) {
    hipLaunchKernelGGL((expert_bf16<TCAP, GATEUP, WK>), dim3(nu * (unsigned)k.col_tiles), dim3(256), 0, s, k);
}

template <bool GATEUP, int WK>
void launch_t(int tiles, const KArgs &k, unsigned nu, hipStream_t s) {
    if (tiles <= 1) launch1<1, GATEUP, WK>(k, nu, s);
    else if (tiles <= 2) launch1<2, GATEUP, WK>(k, nu, s);
    else if (tiles <= 4 || WK > 1) launch1<4, GATEUP, WK>(k, nu, s);   // K-split serves units of <= 128 rows only
    else if constexpr (WK == 1) launch1<8, GATEUP, WK>(k, nu, s);
}

}  // namespace

void launch_experts_bf16(const ExpertArgs &a, const KArgs &gu_in, const KArgs &dn_in, hipStream_t s) {
    KArgs gu = gu_in;
    gu.col_tiles = (a.F + 127) / 128;
    { Scope sc(a.prof, MOE_PROF_GATE_UP, s); launch_t<true, 1>((a.max_rows + 31) / 32, gu, a.nu, s); }
    // Down projection.  Units of at most kSmallUnitRows rows split K over the 4 waves when F allows
    // it: 4x the workgroups for the weight-streaming shapes.  The choice depends on the unit's row
    // count and on F only, never on what else is in the launch.
    const bool ksplit = (a.F % 256) == 0;
    if (a.has_small) {
        KArgs d = dn_in;
        d.cls_filter = 1;
        Scope sc(a.prof, MOE_PROF_DOWN_SMALL, s);
        if (ksplit) { d.col_tiles = (a.H + 63) / 64; launch_t<false, 4>((a.max_rows_small + 31) / 32, d, a.nu, s); }
        else { d.col_tiles = (a.H + 255) / 256; launch_t<false, 1>((a.max_rows_small + 31) / 32, d, a.nu, s); }
    }
    if (a.has_large) {
        KArgs d = dn_in;
        d.cls_filter = 2;
        d.col_tiles = (a.H + 255) / 256;
        Scope sc(a.prof, MOE_PROF_DOWN_LARGE, s);
        launch_t<false, 1>((a.max_rows + 31) / 32, d, a.nu, s);
    }
}

}  // namespace qmoe

// bf16 expert kernels (gate-up with fused SwiGLU, and down projection) on MFMA: the templates.
// Included by experts_bf16.hip (dispatch) and by experts_bf16_w<WF>.hip (one instantiation per weight
// format).
//
// All three weight matrices are [rows_out, K] with K contiguous, and so are the activations, so
// both MFMA operands are read 8 consecutive K-elements (16 bytes) per lane with no transposition.
// v_mfma_f32_32x32x16_bf16: A = 32 tokens x 16 k, B = 32 weight rows x 16 k, D[token, weight row]
// in fp32.  A workgroup has 4 waves.  Each wave owns 64 weight rows (gate-up: 32 rows of W1 and the
// same 32 of W3, so the gate and up value of one (token, f) meet in one lane and register) and every
// token tile of the unit.  No two waves use the same weight fragment, so weights go straight from
// global memory into MFMA operand registers (with the packed layout every wave load is one
// contiguous KiB); only the token tile (gathered x rows, or act rows), which all 4 waves share, is
// staged in LDS, double-buffered, its 16-byte slots XOR-swizzled by row so that the 32 rows read
// by one ds_read_b128 fall into distinct banks.
//
// Pipeline of one K-iteration (64 k), prefetch distance D: issue the global loads of the token
// pieces and weight fragments for it+D (register rings of D+1 sets), run the MFMAs of iteration it,
// write the token tile for it+1 into the other LDS stage, one barrier.  Vector loads complete in
// issue order, so the waits leave about D iterations of weight loads (8 KB per wave each) in flight.
// Loads are unconditional (row and iteration indices are clamped instead) so that the wait counters
// stay exact.
//
// Down projection with K-split (a property of the context's configuration: weight-streaming shapes
// have too few output tiles to fill the chip): K is cut into 2 or 4 contiguous ranges, each computed
// by its own workgroup into a partial plane; a second kernel adds the planes in the fixed order
// ((p0+p1)+p2)+p3.
//
// A launch works on row segments: the host joins the row-adjacent units of one expert in a call (the
// LS and BE part of its queue, consecutive chunks) and cuts each such run into segments of at most 8
// token tiles with equal tile counts, so that one pass over the weights serves them and workgroups
// that share weight tiles keep the same pace.
//
// Determinism.  Each output element is one chain of MFMA accumulations over K in ascending order
// (K-split: 2 or 4 chains added in a fixed order), the same for every row of the context: it depends on
// neither the tile a row sits in, nor the rows that share it, nor the weight layout.  Results are
// therefore bit-identical however the unit list is split into launches.
#pragma once
#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>
#include <utility>

#include "experts_common.h"

namespace qmoe {
namespace bf16k {

// Weight formats of the expert matrices: bf16 row-major, bf16 in MFMA-ordered 1 KiB blocks, and
// 4-bit microscaling floats (e2m1 elements, one power-of-two e8m0 scale per 32 elements along K) in
// MFMA-ordered blocks, turned into bf16 operands in registers (exactly: every such value is a bf16).
enum { WF_ROWMAJOR = 0, WF_PACKED = 1, WF_MXFP4 = 2 };

// Smallest number of token tiles whose variant keeps three LDS stages (see P3 in expert_tile).
#ifndef QMOE_P3_MIN_T
#define QMOE_P3_MIN_T 4
#endif
constexpr int kP3MinT = QMOE_P3_MIN_T;
// A packet (32 workgroups, one XCD's CUs) is 2^QMOE_PK_U segments x 2^(5 - QMOE_PK_U) column tiles.
// 4 x 8 fetches the least (measured on the 3584-token prefill's gate-up launch: 3.1 GB against 3.4 GB
// for 8 x 4 and 5.0 GB for 2 x 16; the launch time follows weakly: +1 % and +6 %).
#ifndef QMOE_PK_U
#define QMOE_PK_U 2
#endif


typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// silu(z) = z / (1 + e^-z) as one exponential and one reciprocal (v_exp_f32, v_rcp_f32: about 1 ulp
// each, far below the bf16 rounding the product gets next).  An IEEE division costs three times the
// instructions, and a workgroup's epilogue applies this to T*32 x 128 values while its MFMA pipes idle.
__device__ __forceinline__ float silu_f(float z) { return z * __builtin_amdgcn_rcpf(1.f + __expf(-z)); }

// LDS layout of the token tile: rows of 128 bytes = 8 slots of 16 bytes; slot s of row r is stored
// at slot s ^ swz(r).  swz is a permutation of 0..7 over any 8 consecutive rows, and over 16
// consecutive rows the pairs (row parity, swz) are all distinct: the 8 or 16 lanes of one
// ds_read_b128 / ds_write_b128 pass hit distinct banks whether a pass spans 128 or 256 bytes.
__device__ __forceinline__ int swz(int r) { return (r & 7) ^ ((r >> 3) & 1); }

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

// Launch-local arguments of the bf16 kernels.
struct BArgs {
    KArgs k;
    int ksplit;          // 1, or 2 or 4: K ranges, one workgroup each, partial planes in k.dst
    long plane;          // elements between partial planes
    int nseg;            // > 0: work on seg[0..nseg); 0: on units[u0 .. u0+nu) of the device list
    Seg seg[kMaxSegs];
};

// One (unit, column tile, K range) on a workgroup.
template <int T, bool GATEUP, int WF, bool STREAM, int D>
__device__ __forceinline__ void expert_tile(const KArgs &p, const moe_unit un, const int ct, const int kq, const int ksplit,
                                            const long plane, char *lds) {
    // Stoppable launches: the workgroup leaves behind the prologue's barrier if the stop word is set or
    // (down projection) the gate-up workgroups of its rows did not all run.
    __shared__ int s_run;
    const WgProbe probe = wg_probe(p, un.row0);
    constexpr int ROWS = T * 32;
    constexpr int STAGE = ROWS * 128;      // bytes of one LDS stage: 64 bf16 per row
    // The variants of 4 and more token tiles keep three token-tile stages, write tile it+2 during
    // iteration it, and so may read the first fragments of tile it+1 before the iteration's barrier;
    // the LDS latency after the barrier disappears from the MFMA stream (8 tiles: -1.7 % on the
    // 3584-token prefill; 4-5 tiles: gate-up -1.2 % on the 512-token batch, measured against the
    // two-stage form on one machine).  Below 4 tiles an iteration is bound by the weight stream alone.
    constexpr bool P3 = T >= kP3MinT;
    // Output columns per wave.  Gate-up: 32, or fewer (p.cw, a multiple of 4) on launches whose
    // workgroup count would otherwise end in a partly filled round of the chip; the wave's MFMA rows
    // beyond p.cw repeat its last weight row and are dropped in the epilogue.
    const int cpw = GATEUP ? p.cw : 64;
    const int rows = un.rows;
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
    const int lr = l & 31, lh = l >> 5;
    const int Kg = p.K / ksplit;           // this workgroup's K range: [kq*Kg, (kq+1)*Kg)
    const int iters = Kg / 64;
    const int col_base = ct * (4 * cpw) + w * cpw;
    // gate-up: the weight row of this lane, and its place in the 32-row tiles of the packed formats
    const int grow = min(col_base + min(lr, cpw - 1), p.ncols - 1);
    const int gnt = grow >> 5, grr = grow & 31;

    // ---- weight rows of this lane (B operand) ----
    // Row-major: lane = (row l%32, k-half l/32), 16 elements per k-step, 64 per iteration.
    // Packed: the wave's 1 KiB block of k-step s of row tile nt starts at (nt*(K/16)+s)*512.
    // MXFP4: per (row tile, iteration) one KiB of codes (lane l: 16 bytes = the 8 elements of each
    // of the 4 k-steps) and 64 bytes of scales (row l%32: the two e8m0 bytes of the iteration's two
    // 32-element blocks).
    constexpr bool PACKED = WF == WF_PACKED;
    constexpr bool MX = WF == WF_MXFP4;
    constexpr int BKS = PACKED ? 512 : 16;   // elements between k-steps
    constexpr int BIT = PACKED ? 2048 : 64;  // elements between iterations
    const uint16_t *bptr[2];
    const char *cptr[2];                     // MXFP4 codes
    const char *sptr[2];                     // MXFP4 scales
    if constexpr (MX) {
        const int ntiles = p.ncols >> 5;
        const int nt0 = GATEUP ? gnt : min(col_base >> 5, ntiles - 1);
        const int nt1 = GATEUP ? gnt : min((col_base >> 5) + 1, ntiles - 1);
        const int rr = GATEUP ? grr : lr;
        const long kblocks = p.K >> 6;                              // iterations per row tile
        const char *c0 = (const char *)p.b0 + (long)un.expert * (p.b_estride >> 1);
        const char *c1 = GATEUP ? (const char *)p.b1 + (long)un.expert * (p.b_estride >> 1) : c0;
        const char *s0 = (const char *)p.s0 + (long)un.expert * (p.b_estride >> 5);
        const char *s1 = GATEUP ? (const char *)p.s1 + (long)un.expert * (p.b_estride >> 5) : s0;
        const long it0 = (long)kq * (Kg >> 6);
        cptr[0] = c0 + ((nt0 * kblocks + it0) * 64 + lh * 32 + rr) * 16;
        cptr[1] = c1 + ((nt1 * kblocks + it0) * 64 + lh * 32 + rr) * 16;
        sptr[0] = s0 + ((nt0 * kblocks + it0) * 32 + rr) * 2;
        sptr[1] = s1 + ((nt1 * kblocks + it0) * 32 + rr) * 2;
        bptr[0] = bptr[1] = nullptr;
    } else {
        cptr[0] = cptr[1] = sptr[0] = sptr[1] = nullptr;
        const uint16_t *b0 = (const uint16_t *)p.b0 + (long)un.expert * p.b_estride;
        const uint16_t *b1 = GATEUP ? (const uint16_t *)p.b1 + (long)un.expert * p.b_estride : b0;
        if (PACKED) {
            const int ntiles = p.ncols >> 5;
            const long tile_elems = (long)p.K * 32;
            const long koff = (long)kq * (Kg / 16) * 512 + (lh * 32 + (GATEUP ? grr : lr)) * 8;
            const int nt0 = GATEUP ? gnt : min(col_base >> 5, ntiles - 1);
            const int nt1 = GATEUP ? gnt : min((col_base >> 5) + 1, ntiles - 1);
            bptr[0] = b0 + nt0 * tile_elems + koff;
            bptr[1] = b1 + nt1 * tile_elems + koff;
        } else {
            const int c0 = GATEUP ? grow : min(col_base + lr, p.ncols - 1);
            const int c1 = GATEUP ? c0 : min(col_base + 32 + lr, p.ncols - 1);
            bptr[0] = b0 + (long)c0 * p.K + kq * Kg + lh * 8;
            bptr[1] = b1 + (long)c1 * p.K + kq * Kg + lh * 8;
        }
    }
    // ---- token rows this thread stages into LDS (A operand): row tid/8 + 32*j, slot tid%8 ----
    const int srow = tid >> 3, sslot = tid & 7;
    // Addressed as a wave-uniform 64-bit base plus a 32-bit offset per row in units of 16 bytes (the
    // host checks that x and act stay below 64 GiB), which halves the registers the row table costs.
    const char *abase = (const char *)p.a_src + ((long)kq * Kg + sslot * 8) * 2;
    unsigned aoff[T];
    static_for<T>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        const int r = min(srow + 32 * j, rows - 1);
        unsigned src_row;
        if (GATEUP) src_row = (unsigned)(p.perm[un.row0 + r] / p.kdiv);
        else src_row = (unsigned)(un.row0 + r);
        aoff[j] = src_row * ((unsigned)p.lda >> 3);        // in 16-byte units: lda is a multiple of 64 elements
    });

    f32x16 acc[T][2];
    static_for<T>([&](auto tc) {
        constexpr int t = decltype(tc)::value;
#pragma unroll
        for (int r = 0; r < 16; ++r) { acc[t][0][r] = 0.f; acc[t][1][r] = 0.f; }
    });

    // Register rings: weight fragments of iterations it .. it+D (NB sets), token pieces of
    // it+1 .. it+D (NA sets).  Ring positions are compile-time constants: the loop is unrolled NA*NB.
    constexpr int DA = P3 ? 1 : (T >= 5 && D > 2 ? 2 : D);   // token pieces: same distance, or less where registers are scarce
    constexpr int NB = D + 1, NA = DA, U = (NB % NA == 0) ? NB : NA * NB;
    u32x4 a_reg[NA * T];
    bf16x8 b_reg[NB * 8];  // [set][k-step][n-tile]; MXFP4: set 0 only, the operands of the current iteration
    u32x4 c_reg[NB * 2];   // MXFP4: codes [set][n-tile]
    unsigned short s_reg[NB * 2];   // MXFP4: the two scale bytes [set][n-tile]

    auto load_a = [&](int it, auto setc) {
        constexpr int S = decltype(setc)::value;
        const int itc = min(it, iters - 1);
        static_for<T>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            a_reg[S * T + j] = *reinterpret_cast<const u32x4 *>(abase + ((unsigned long)(aoff[j] + (unsigned)itc * 8u) << 4));
        });
    };
    auto store_a = [&](int stage, auto setc) {
        constexpr int S = decltype(setc)::value;
        static_for<T>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            const int r = srow + 32 * j;
            *reinterpret_cast<u32x4 *>(lds + stage * STAGE + (r * 8 + (sslot ^ swz(r))) * 16) = a_reg[S * T + j];
        });
    };
    auto load_b = [&](int it, auto setc) {
        constexpr int S = decltype(setc)::value;
        const int itc = min(it, iters - 1);
        if constexpr (MX) {
            static_for<2>([&](auto nc) {
                constexpr int n = decltype(nc)::value;
                const u32x4 *qc = reinterpret_cast<const u32x4 *>(cptr[n] + (long)itc * 1024);
                const unsigned short *qs = reinterpret_cast<const unsigned short *>(sptr[n] + (long)itc * 64);
                if constexpr (STREAM) c_reg[S * 2 + n] = __builtin_nontemporal_load(qc);
                else c_reg[S * 2 + n] = *qc;
                s_reg[S * 2 + n] = *qs;
            });
            return;
        }
        static_for<4>([&](auto kc) {
            constexpr int ks = decltype(kc)::value;
            const bf16x8 *q0 = reinterpret_cast<const bf16x8 *>(bptr[0] + (long)itc * BIT + ks * BKS);
            const bf16x8 *q1 = reinterpret_cast<const bf16x8 *>(bptr[1] + (long)itc * BIT + ks * BKS);
            if constexpr (STREAM) {
                b_reg[S * 8 + ks * 2 + 0] = __builtin_nontemporal_load(q0);
                b_reg[S * 8 + ks * 2 + 1] = __builtin_nontemporal_load(q1);
            } else {
                b_reg[S * 8 + ks * 2 + 0] = *q0;
                b_reg[S * 8 + ks * 2 + 1] = *q1;
            }
        });
    };
    // MFMAs of one iteration.  Token fragments are read from LDS one half-step (HT tiles of one
    // k-step) ahead of the MFMAs that use them.
        constexpr int HT = T >= 8 ? 4 : (T == 6 ? 3 : T), NH = T / HT, STEPS = 4 * NH;
    bf16x8 af[2 * HT];
    auto read_af = [&](int stage, auto hsc) {
        constexpr int hs = decltype(hsc)::value, ks = hs / NH, h = hs % NH;
        static_for<HT>([&](auto tc) {
            constexpr int t = h * HT + decltype(tc)::value;
            const int r = t * 32 + lr;
            const int slot = (ks * 2 + lh) ^ swz(r);
            af[(hs & 1) * HT + decltype(tc)::value] = *reinterpret_cast<const bf16x8 *>(lds + stage * STAGE + (r * 8 + slot) * 16);
        });
    };
    // MXFP4: codes and scales of ring set S -> bf16 operands (v_cvt_scalef32_pk_bf16_fp4: two e2m1
    // nibbles of one byte times a float scale, exact for a power-of-two scale).
    auto dequant_b = [&](auto setc) {
        constexpr int S = decltype(setc)::value;
        static_for<2>([&](auto nc) {
            constexpr int n = decltype(nc)::value;
            const unsigned sc = s_reg[S * 2 + n];
            const float f0 = __builtin_bit_cast(float, (sc & 0xffu) << 23);
            const float f1 = __builtin_bit_cast(float, (sc >> 8) << 23);
            static_for<4>([&](auto kc) {
                constexpr int ks = decltype(kc)::value;
                const unsigned wv = c_reg[S * 2 + n][ks];
                const float f = ks < 2 ? f0 : f1;
                const bf16x2 e0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(wv, f, 0);
                const bf16x2 e1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(wv, f, 1);
                const bf16x2 e2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(wv, f, 2);
                const bf16x2 e3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(wv, f, 3);
                bf16x8 v;
                v[0] = e0[0]; v[1] = e0[1]; v[2] = e1[0]; v[3] = e1[1];
                v[4] = e2[0]; v[5] = e2[1]; v[6] = e3[0]; v[7] = e3[1];
                b_reg[ks * 2 + n] = v;
            });
        });
    };
    auto mfma_tile = [&](int stage, int next_stage, auto setc) {
        constexpr int S = MX ? 0 : decltype(setc)::value;
        if constexpr (MX) dequant_b(setc);
        if constexpr (!P3) read_af(stage, std::integral_constant<int, 0>{});
        static_for<STEPS>([&](auto hsc) {
            constexpr int hs = decltype(hsc)::value, ks = hs / NH, h = hs % NH;
            if constexpr (hs + 1 < STEPS) read_af(stage, std::integral_constant<int, hs + 1>{});
            else if constexpr (P3) read_af(next_stage, std::integral_constant<int, 0>{});
            static_for<HT>([&](auto tc) {
                constexpr int t = h * HT + decltype(tc)::value;
                const bf16x8 a = af[(hs & 1) * HT + decltype(tc)::value];
                acc[t][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b_reg[S * 8 + ks * 2 + 0], acc[t][0], 0, 0, 0);
                acc[t][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b_reg[S * 8 + ks * 2 + 1], acc[t][1], 0, 0, 0);
            });
        });
    };
    // The instruction mix of one iteration, handed to the scheduler as one pipeline: the MFMAs are
    // the backbone (2 per slot); each slot also takes one LDS fragment read; the T+8 global loads
    // are spread over the first half of the slots (so the texture path works under the MFMAs
    // instead of in a burst), the T LDS writes of the next token tile over the last slots.
    auto pipeline = [&]() {
        constexpr int NS = 4 * T, NV = T + 8, HALF = NS / 2;
        if constexpr (!P3) __builtin_amdgcn_sched_group_barrier(0x100, HT, 0);
        static_for<NS>([&](auto sc) {
            constexpr int sl = decltype(sc)::value;
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            if constexpr (P3 || sl < NS - HT) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            if constexpr (sl < HALF) {
                constexpr int vm = NV / HALF + (sl < NV % HALF ? 1 : 0);
                if constexpr (vm > 0) __builtin_amdgcn_sched_group_barrier(0x020, vm, 0);
            }
            if constexpr (sl >= NS - T) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
        });
    };
    // Iteration `it`, position i = it mod U in the unrolled loop: request the operands of it+D (token
    // pieces first: the wait for them must not cover the weight loads), run the MFMAs of it, move the
    // token pieces of it+1 (requested earlier) into the other LDS stage.  Loads complete in issue
    // order, so neither wait disturbs the iterations of weight loads issued after the data waited for.
    auto body = [&](int it, auto ic) {
        constexpr int i = decltype(ic)::value;
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (P3) {
            static_assert(!P3 || (NA == 1 && U % 3 == 0), "three stages: one token register set, loop unrolled by a multiple of 3");
            load_a(it + 2, std::integral_constant<int, 0>{});
            load_b(it + D, std::integral_constant<int, (i + D) % NB>{});
            mfma_tile(i % 3, (i + 1) % 3, std::integral_constant<int, i % NB>{});
            store_a((i + 2) % 3, std::integral_constant<int, 0>{});
        } else {
            load_a(it + DA, std::integral_constant<int, (i + DA) % NA>{});
            load_b(it + D, std::integral_constant<int, (i + D) % NB>{});
            mfma_tile(it & 1, 0, std::integral_constant<int, i % NB>{});
            store_a((it + 1) & 1, std::integral_constant<int, (i + 1) % NA>{});
        }
        pipeline();
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
    };

    // prologue: operands of iterations 0 .. D-1; tile 0 into LDS stage 0
    load_a(0, std::integral_constant<int, 0>{});
    load_b(0, std::integral_constant<int, 0>{});
    store_a(0, std::integral_constant<int, 0>{});
    if constexpr (P3) {                      // three stages: tile 1 goes into stage 1 as well
        load_a(1, std::integral_constant<int, 0>{});
        store_a(1, std::integral_constant<int, 0>{});
    }
    static_for<D - 1>([&](auto ic) {
        constexpr int j = decltype(ic)::value + 1;
        if constexpr (!P3 && j < DA) load_a(j, std::integral_constant<int, j % NA>{});
        load_b(j, std::integral_constant<int, j % NB>{});
    });
    wg_decide(p, un.row0, 1, probe, &s_run);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    if (p.go != nullptr && s_run == 0) return;
    if constexpr (P3) read_af(0, std::integral_constant<int, 0>{});
    int it = 0;
    for (; it + U <= iters; it += U) {
        static_for<U>([&](auto ic) { body(it + decltype(ic)::value, ic); });
    }
    static_for<U - 1>([&](auto ic) {
        if (it + decltype(ic)::value < iters) body(it + decltype(ic)::value, ic);
    });

    // ---- epilogue.  D register r of lane l: token 8*(r/4) + 4*(l/32) + r%4, weight row l%32 ----
    if (GATEUP) {
        // SwiGLU in fp32, one rounding to bf16; the wave's [T*32 tokens][32 f] tile goes through LDS
        // (free after the last barrier of the main loop) so that it leaves as 16-byte stores, with the
        // non-temporal hint: the next kernel reads it, nothing in this one does.
        __bf16 *st = reinterpret_cast<__bf16 *>(lds) + w * (ROWS * 32);
        static_for<T>([&](auto tc) {
            constexpr int t = decltype(tc)::value;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = t * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                st[i * 32 + lr] = (__bf16)(silu_f(acc[t][0][r]) * acc[t][1][r]);
            }
        });
        __builtin_amdgcn_s_waitcnt(0xc07f);   // this wave's LDS writes have landed (lgkmcnt 0)
        __builtin_amdgcn_wave_barrier();
        if (cpw == 32) {
            const int f0 = col_base + (l & 3) * 8;
#pragma unroll
            for (int j = 0; j < 2 * T; ++j) {
                const int i = (l >> 2) + 16 * j;
                if (i < rows && f0 < p.ncols) {
                    const u32x4 v = *reinterpret_cast<const u32x4 *>(st + i * 32 + (l & 3) * 8);
                    __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>((__bf16 *)p.dst + (long)(un.row0 + i) * p.ldd + f0));
                }
            }
        } else {
            // narrower waves start at multiples of 4 columns: 8-byte stores of the first cpw columns
            const int fo = (l & 7) * 4;
#pragma unroll
            for (int j = 0; j < 4 * T; ++j) {
                const int i = (l >> 3) + 8 * j;
                if (i < rows && fo < cpw && col_base + fo < p.ncols) {
                    const u32x2 v = *reinterpret_cast<const u32x2 *>(st + i * 32 + fo);
                    __builtin_nontemporal_store(v, reinterpret_cast<u32x2 *>((__bf16 *)p.dst + (long)(un.row0 + i) * p.ldd + col_base + fo));
                }
            }
        }
    } else {
        // fp32 tile of 32 tokens x 64 columns at a time through this wave's 8 KiB of LDS, so that it
        // leaves as 16-byte stores (256 contiguous bytes per token row).
        float *st = reinterpret_cast<float *>(lds) + w * (32 * 64);
        float *obase = (float *)p.dst + kq * plane + (long)un.row0 * p.ldd + col_base + (l & 15) * 4;
        const bool col_ok = col_base + (l & 15) * 4 < p.ncols;
        static_for<T>([&](auto tc) {
            constexpr int t = decltype(tc)::value;
            if (t * 32 < rows) {
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int i = 8 * (r >> 2) + 4 * lh + (r & 3);
                    st[i * 64 + lr] = acc[t][0][r];
                    st[i * 64 + 32 + lr] = acc[t][1][r];
                }
                __builtin_amdgcn_s_waitcnt(0xc07f);
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int i = (l >> 4) + 4 * j;
                    const f32x4 v = *reinterpret_cast<const f32x4 *>(st + i * 64 + (l & 15) * 4);
                    if (t * 32 + i < rows && col_ok) __builtin_nontemporal_store(v, reinterpret_cast<f32x4 *>(obase + (long)(t * 32 + i) * p.ldd));
                }
                __builtin_amdgcn_s_waitcnt(0xc07f);
            }
        });
    }
}

// Workgroup id -> (unit, column tile, K range).  The hardware deals consecutive workgroup ids
// round-robin to the 8 XCDs (each with its own L2).  Work is cut into packets of 4 consecutive
// units (in launch order) x 8 consecutive column tiles = 32 workgroups = one XCD's 32 CUs: the 4
// token tiles are each shared by 8 workgroups and, when the units belong to one expert (chunks of
// a long queue, or its LS and BE part), the 8 weight tiles by up to 4.  Packet q goes to XCD q % 8;
// the workgroups of a packet get ids 8 apart.  With a K-split the column-tile axis is
// (range, tile), range slowest, so a packet stays inside one K range.
template <bool STREAM>
__device__ __forceinline__ bool map_block(const BArgs &b, moe_unit &un, int &ct, int &kq) {
    const int w = blockIdx.x;
    const int x = w & 7, j = w >> 3;
    const int packet = (j >> 5) * 8 + x, within = j & 31;
    const int n = b.nseg > 0 ? b.nseg : b.k.nu;
    constexpr int PU = QMOE_PK_U, PC = 5 - PU;      // log2 of units and of column tiles per packet
    const int ugroups = (n + (1 << PU) - 1) >> PU;
    // Streaming launches list their segments longest first: the packets walk the column tiles of one
    // group of segments before the next group, so the long segments really start first.  Launches
    // that share weights walk the groups first: the packets of one column block run side by side.
    int ctb, ug;
    if (STREAM) {
        const int ctbs = (b.k.col_tiles * b.ksplit + (1 << PC) - 1) >> PC;
        ug = packet / ctbs;
        ctb = packet - ug * ctbs;
    } else {
        ctb = packet / ugroups;
        ug = packet - ctb * ugroups;
    }
    const int pos = (ug << PU) + (within >> PC);
    const int cq = (ctb << PC) + (within & ((1 << PC) - 1));
    if (pos >= n || cq >= b.k.col_tiles * b.ksplit) return false;
    if (b.nseg > 0) {
        const Seg g = b.seg[pos];
        if (g.rows == 0) return false;      // padding between experts
        un.expert = g.expert; un.cls = 0; un.row0 = (int)g.row0; un.rows = g.rows;
    } else {
        un = b.k.units[b.k.u0 + pos];
    }
    kq = cq / b.k.col_tiles;
    ct = cq - kq * b.k.col_tiles;
    return true;
}

// TCAP: largest number of 32-token tiles a segment of this launch may have (1, 2, 4, 6 or 8).  A
// workgroup takes the smallest fully unrolled variant (1, 2, 4, 5, 6, 7 or 8 tiles) that covers its unit.
// STREAM: no two segments of the launch belong to one expert, so every weight element is read by
// exactly one workgroup: the loads carry the non-temporal hint and do not displace the token tiles
// in L2.  Where segments share an expert's weights the hint is left off so that L2 serves the re-reads.
template <int TCAP, bool GATEUP, int WF, bool STREAM>
__global__ __launch_bounds__(256) void expert_bf16(const BArgs b) {
    // two token-tile stages (three from 4 token tiles on); at least 8 KiB per wave for the
    // epilogue's store staging
    __shared__ __attribute__((aligned(16))) char lds[((TCAP >= kP3MinT ? 3 : 2) * TCAP * 32 * 128) > 32768 ? ((TCAP >= kP3MinT ? 3 : 2) * TCAP * 32 * 128) : 32768];
    // A closed gate: the sequence was stopped before this launch, or an earlier workgroup of it saw
    // the stop word.  The word may change while the launch runs, so one thread reads it for all.
    if (b.k.go != nullptr) {
        __shared__ int s_go;
        if (threadIdx.x == 0) s_go = __hip_atomic_load(b.k.go, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (s_go == 0) return;
    }
    int ct, kq;
    moe_unit un;
    if (!map_block<STREAM>(b, un, ct, kq)) return;
    const int t_cnt = (un.rows + 31) >> 5;
    // Prefetch distance of the weights: 2 iterations for the three-stage variants (their loop is unrolled by
    // a multiple of 3) and the 2-tile variant, 3 for the 1-tile variant.
    if (TCAP >= 8 && t_cnt > 7) expert_tile<(TCAP >= 8 ? 8 : 1), GATEUP, WF, STREAM, 2>(b.k, un, ct, kq, b.ksplit, b.plane, lds);
    else if (TCAP >= 8 && t_cnt > 6) expert_tile<(TCAP >= 8 ? 7 : 1), GATEUP, WF, STREAM, 2>(b.k, un, ct, kq, b.ksplit, b.plane, lds);
    else if (TCAP >= 6 && t_cnt > 5) expert_tile<(TCAP >= 6 ? 6 : 1), GATEUP, WF, STREAM, (kP3MinT <= 6 ? 2 : 3)>(b.k, un, ct, kq, b.ksplit, b.plane, lds);
    else if (TCAP >= 6 && t_cnt > 4) expert_tile<(TCAP >= 6 ? 5 : 1), GATEUP, WF, STREAM, (kP3MinT <= 5 ? 2 : 3)>(b.k, un, ct, kq, b.ksplit, b.plane, lds);
    else if (TCAP >= 4 && t_cnt > 2) expert_tile<(TCAP >= 4 ? 4 : 1), GATEUP, WF, STREAM, (kP3MinT <= 4 ? 2 : 3)>(b.k, un, ct, kq, b.ksplit, b.plane, lds);
    else if (TCAP >= 2 && t_cnt > 1) expert_tile<(TCAP >= 2 ? 2 : 1), GATEUP, WF, STREAM, 2>(b.k, un, ct, kq, b.ksplit, b.plane, lds);
    else expert_tile<1, GATEUP, WF, STREAM, 3>(b.k, un, ct, kq, b.ksplit, b.plane, lds);
}

template <int TCAP, bool GATEUP, int WF, bool STREAM>
void launch1(const BArgs &b, hipStream_t s) {
    const unsigned n = b.nseg > 0 ? (unsigned)b.nseg : (unsigned)b.k.nu;
    const unsigned ugroups = (n + (1u << QMOE_PK_U) - 1) >> QMOE_PK_U, ctb = (b.k.col_tiles * b.ksplit + (32u >> QMOE_PK_U) - 1) / (32u >> QMOE_PK_U);
    const unsigned packets = ugroups * ctb;
    const unsigned grid = (packets + 7) / 8 * 8 * 32;
    hipLaunchKernelGGL((expert_bf16<TCAP, GATEUP, WF, STREAM>), dim3(grid), dim3(256), 0, s, b);
}

template <bool GATEUP, int WF, bool STREAM>
void launch_ts(int tiles, const BArgs &b, hipStream_t s) {
    if (tiles <= 1) launch1<1, GATEUP, WF, STREAM>(b, s);
    else if (tiles <= 2) launch1<2, GATEUP, WF, STREAM>(b, s);
    else if (tiles <= 4) launch1<4, GATEUP, WF, STREAM>(b, s);
    else if (tiles <= 6) launch1<6, GATEUP, WF, STREAM>(b, s);
    else launch1<8, GATEUP, WF, STREAM>(b, s);
}

// The expert kernels of one weight format: gate-up or down, for segments of at most `tiles` token
// tiles.  Each format is instantiated in its own translation unit (experts_bf16_w<WF>.hip).
template <int WF>
void launch_expert_kernels(bool gateup, int tiles, bool stream, const BArgs &b, hipStream_t s) {
    if (gateup) {
        if (stream) launch_ts<true, WF, true>(tiles, b, s);
        else launch_ts<true, WF, false>(tiles, b, s);
    } else {
        if (stream) launch_ts<false, WF, true>(tiles, b, s);
        else launch_ts<false, WF, false>(tiles, b, s);
    }
}


extern template void launch_expert_kernels<WF_ROWMAJOR>(bool, int, bool, const BArgs &, hipStream_t);
extern template void launch_expert_kernels<WF_PACKED>(bool, int, bool, const BArgs &, hipStream_t);
extern template void launch_expert_kernels<WF_MXFP4>(bool, int, bool, const BArgs &, hipStream_t);

}  // namespace bf16k
}  // namespace qmoe

// Exact solve of four augmented systems per wave at head dimension 64 (the moments kernels' case): the 16-blocked
// Cholesky factorisation of factorise_wave, followed by forward and back substitutions on the vector ALU instead of the
// matrix cores.
//
// Why.  A substitution multiplies a 16x16 tile by two or three right-hand-side columns; as a 16x16x16 fp32 tile
// product it uses two or three of sixteen output columns and still occupies the matrix cores for 128 cycles -- 80 of
// the 144 fp32 MFMAs of a row's solve, which at 1/16 of the 16-bit rate weigh as much as a third of the main loop.
// The same products cost the vector ALU 16 multiply-adds per tile and column FOR ALL FOUR QUERIES AT ONCE when lane
// 16 q + r holds column r of query q's tile: out[r] = sum_c X[c][r] v[c] is then a chain of v_fmac with a
// row-broadcast (DPP) operand.
//   * Layout change, in place and without LDS: a tile sits in the accumulator layout (lane (g, n), register t =
//     X[4g+t][n], one register set per query); a 4x4 transpose of the four queries' registers across the four 16-lane
//     rows of the wave (v_permlane16_swap / v_permlane32_swap) leaves lane (q, r) with X_q[4g'+t][r] in the register
//     that query g' owned: column r of its own query's tile.
//   * Forward substitution (U^T a = b) needs exactly those columns.
//   * Back substitution (U x = z) needs rows; with columns at hand it is done in the outer-product form instead:
//     lane (q, c) scales its column by x[c], the partial vectors are summed over the 16 lanes of the row by a
//     transpose-reduction (16 registers -> 1 in four DPP exchange stages: mirror, half mirror, xor 2, xor 1), which
//     leaves element r of the sum in lane (q, r).
#pragma once

#include "llla_mfma_common.hpp"

namespace llla {
namespace mfma {

// 4x4 transpose across the four 16-lane rows of the wave, for the four registers of a tile at once: afterwards row q
// of a_g holds what row g of a_q held.  v_permlane16_swap exchanges the odd rows of its first operand with the even
// rows of its second, v_permlane32_swap the upper half of the first with the lower half of the second.  Inline
// assembly: the compiler's builtins for the two swaps lose the second result of v_permlane32_swap when its inputs
// are results of v_permlane16_swap (seen with ROCm 7.2: both outputs of the pair came back as the first).  A swap
// reads its registers two wait states after a vector-ALU write at the earliest, hence the two s_nop.
__device__ inline void rows_transpose4(f32x4 &a0, f32x4 &a1, f32x4 &a2, f32x4 &a3)
{
    float x0 = a0[0], x1 = a0[1], x2 = a0[2], x3 = a0[3], y0 = a1[0], y1 = a1[1], y2 = a1[2], y3 = a1[3];
    float z0 = a2[0], z1 = a2[1], z2 = a2[2], z3 = a2[3], w0 = a3[0], w1 = a3[1], w2 = a3[2], w3 = a3[3];
    asm volatile("s_nop 1\n\t"
                 "v_permlane16_swap_b32 %0, %4\n\t"
                 "v_permlane16_swap_b32 %1, %5\n\t"
                 "v_permlane16_swap_b32 %2, %6\n\t"
                 "v_permlane16_swap_b32 %3, %7\n\t"
                 "v_permlane16_swap_b32 %8, %12\n\t"
                 "v_permlane16_swap_b32 %9, %13\n\t"
                 "v_permlane16_swap_b32 %10, %14\n\t"
                 "v_permlane16_swap_b32 %11, %15\n\t"
                 "s_nop 1\n\t"
                 "v_permlane32_swap_b32 %0, %8\n\t"
                 "v_permlane32_swap_b32 %1, %9\n\t"
                 "v_permlane32_swap_b32 %2, %10\n\t"
                 "v_permlane32_swap_b32 %3, %11\n\t"
                 "v_permlane32_swap_b32 %4, %12\n\t"
                 "v_permlane32_swap_b32 %5, %13\n\t"
                 "v_permlane32_swap_b32 %6, %14\n\t"
                 "v_permlane32_swap_b32 %7, %15"
                 : "+v"(x0), "+v"(x1), "+v"(x2), "+v"(x3), "+v"(y0), "+v"(y1), "+v"(y2), "+v"(y3), "+v"(z0), "+v"(z1),
                   "+v"(z2), "+v"(z3), "+v"(w0), "+v"(w1), "+v"(w2), "+v"(w3));
    a0 = f32x4{x0, x1, x2, x3};
    a1 = f32x4{y0, y1, y2, y3};
    a2 = f32x4{z0, z1, z2, z3};
    a3 = f32x4{w0, w1, w2, w3};
}

// a_k += sum_c bcast_c(s_k) * col[c], c = 0..15, for NC vectors at once (they share the column registers and
// interleave, so that consecutive instructions do not depend on each other).  col[4j+t] = cj[t].
__device__ inline void dot16_bcast1(float &a0, float s0, const f32x4 &c0, const f32x4 &c1, const f32x4 &c2, const f32x4 &c3)
{
#define L(C, B) "v_fmac_f32_dpp %0, %1, %" #B " row_newbcast:" #C " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
    asm volatile("s_nop 1\n\t" L(0, 2) L(1, 3) L(2, 4) L(3, 5) L(4, 6) L(5, 7) L(6, 8) L(7, 9) L(8, 10) L(9, 11) L(10, 12)
                 L(11, 13) L(12, 14) L(13, 15) L(14, 16) L(15, 17)
                 : "+v"(a0)
                 : "v"(s0), "v"(c0[0]), "v"(c0[1]), "v"(c0[2]), "v"(c0[3]), "v"(c1[0]), "v"(c1[1]), "v"(c1[2]), "v"(c1[3]),
                   "v"(c2[0]), "v"(c2[1]), "v"(c2[2]), "v"(c2[3]), "v"(c3[0]), "v"(c3[1]), "v"(c3[2]), "v"(c3[3]));
#undef L
}
__device__ inline void dot16_bcast2(float &a0, float &a1, float s0, float s1, const f32x4 &c0, const f32x4 &c1,
                                    const f32x4 &c2, const f32x4 &c3)
{
#define L(C, B)                                                                                          \
    "v_fmac_f32_dpp %0, %2, %" #B " row_newbcast:" #C " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"      \
    "v_fmac_f32_dpp %1, %3, %" #B " row_newbcast:" #C " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
    asm volatile("s_nop 1\n\t" L(0, 4) L(1, 5) L(2, 6) L(3, 7) L(4, 8) L(5, 9) L(6, 10) L(7, 11) L(8, 12) L(9, 13) L(10, 14)
                 L(11, 15) L(12, 16) L(13, 17) L(14, 18) L(15, 19)
                 : "+v"(a0), "+v"(a1)
                 : "v"(s0), "v"(s1), "v"(c0[0]), "v"(c0[1]), "v"(c0[2]), "v"(c0[3]), "v"(c1[0]), "v"(c1[1]), "v"(c1[2]),
                   "v"(c1[3]), "v"(c2[0]), "v"(c2[1]), "v"(c2[2]), "v"(c2[3]), "v"(c3[0]), "v"(c3[1]), "v"(c3[2]), "v"(c3[3]));
#undef L
}
__device__ inline void dot16_bcast3(float &a0, float &a1, float &a2, float s0, float s1, float s2, const f32x4 &c0,
                                    const f32x4 &c1, const f32x4 &c2, const f32x4 &c3)
{
#define L(C, B)                                                                                          \
    "v_fmac_f32_dpp %0, %3, %" #B " row_newbcast:" #C " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"      \
    "v_fmac_f32_dpp %1, %4, %" #B " row_newbcast:" #C " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"      \
    "v_fmac_f32_dpp %2, %5, %" #B " row_newbcast:" #C " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
    asm volatile("s_nop 1\n\t" L(0, 6) L(1, 7) L(2, 8) L(3, 9) L(4, 10) L(5, 11) L(6, 12) L(7, 13) L(8, 14) L(9, 15)
                 L(10, 16) L(11, 17) L(12, 18) L(13, 19) L(14, 20) L(15, 21)
                 : "+v"(a0), "+v"(a1), "+v"(a2)
                 : "v"(s0), "v"(s1), "v"(s2), "v"(c0[0]), "v"(c0[1]), "v"(c0[2]), "v"(c0[3]), "v"(c1[0]), "v"(c1[1]),
                   "v"(c1[2]), "v"(c1[3]), "v"(c2[0]), "v"(c2[1]), "v"(c2[2]), "v"(c2[3]), "v"(c3[0]), "v"(c3[1]), "v"(c3[2]),
                   "v"(c3[3]));
#undef L
}

// Sum of x over the 16 lanes of the caller's row, in every lane of the row.
__device__ inline float row_allsum(float x)
{
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xf, 0xf, true));    // xor 1
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xf, 0xf, true));    // xor 2
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xf, 0xf, true));   // half mirror
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xf, 0xf, true));   // mirror
    return x;
}

// Transpose-reduction over a 16-lane row: returns, in lane n of the row, the sum of p[n] over the 16 lanes of the row.
// Four exchange stages; after each a lane keeps half of its registers (the half chosen by one bit of its lane index)
// and has added its partner's copy of them.  The first two stages pair lanes of different quads, so the two halves of
// an exchange are two DPP additions enabled per quad (bank mask) with no select at all.
__device__ inline float row_transpose_sum(const float (&p)[16], int nn)
{
    float o[8], o2[4];
    // stage 1, partner = 15 - n: lanes 0..7 keep p[0..7], lanes 8..15 keep p[8..15]
    asm volatile("s_nop 1\n\t"
                 "v_add_f32_dpp %0, %8, %8 row_mirror row_mask:0xf bank_mask:0x3\n\t"
                 "v_add_f32_dpp %1, %9, %9 row_mirror row_mask:0xf bank_mask:0x3\n\t"
                 "v_add_f32_dpp %2, %10, %10 row_mirror row_mask:0xf bank_mask:0x3\n\t"
                 "v_add_f32_dpp %3, %11, %11 row_mirror row_mask:0xf bank_mask:0x3\n\t"
                 "v_add_f32_dpp %4, %12, %12 row_mirror row_mask:0xf bank_mask:0x3\n\t"
                 "v_add_f32_dpp %5, %13, %13 row_mirror row_mask:0xf bank_mask:0x3\n\t"
                 "v_add_f32_dpp %6, %14, %14 row_mirror row_mask:0xf bank_mask:0x3\n\t"
                 "v_add_f32_dpp %7, %15, %15 row_mirror row_mask:0xf bank_mask:0x3\n\t"
                 "v_add_f32_dpp %0, %16, %16 row_mirror row_mask:0xf bank_mask:0xc\n\t"
                 "v_add_f32_dpp %1, %17, %17 row_mirror row_mask:0xf bank_mask:0xc\n\t"
                 "v_add_f32_dpp %2, %18, %18 row_mirror row_mask:0xf bank_mask:0xc\n\t"
                 "v_add_f32_dpp %3, %19, %19 row_mirror row_mask:0xf bank_mask:0xc\n\t"
                 "v_add_f32_dpp %4, %20, %20 row_mirror row_mask:0xf bank_mask:0xc\n\t"
                 "v_add_f32_dpp %5, %21, %21 row_mirror row_mask:0xf bank_mask:0xc\n\t"
                 "v_add_f32_dpp %6, %22, %22 row_mirror row_mask:0xf bank_mask:0xc\n\t"
                 "v_add_f32_dpp %7, %23, %23 row_mirror row_mask:0xf bank_mask:0xc"
                 : "=&v"(o[0]), "=&v"(o[1]), "=&v"(o[2]), "=&v"(o[3]), "=&v"(o[4]), "=&v"(o[5]), "=&v"(o[6]), "=&v"(o[7])
                 : "v"(p[0]), "v"(p[1]), "v"(p[2]), "v"(p[3]), "v"(p[4]), "v"(p[5]), "v"(p[6]), "v"(p[7]), "v"(p[8]),
                   "v"(p[9]), "v"(p[10]), "v"(p[11]), "v"(p[12]), "v"(p[13]), "v"(p[14]), "v"(p[15]));
    // stage 2, partner = the mirror image inside the half row: quads 0 and 2 keep o[0..3], quads 1 and 3 keep o[4..7]
    asm volatile("s_nop 1\n\t"
                 "v_add_f32_dpp %0, %4, %4 row_half_mirror row_mask:0xf bank_mask:0x5\n\t"
                 "v_add_f32_dpp %1, %5, %5 row_half_mirror row_mask:0xf bank_mask:0x5\n\t"
                 "v_add_f32_dpp %2, %6, %6 row_half_mirror row_mask:0xf bank_mask:0x5\n\t"
                 "v_add_f32_dpp %3, %7, %7 row_half_mirror row_mask:0xf bank_mask:0x5\n\t"
                 "v_add_f32_dpp %0, %8, %8 row_half_mirror row_mask:0xf bank_mask:0xa\n\t"
                 "v_add_f32_dpp %1, %9, %9 row_half_mirror row_mask:0xf bank_mask:0xa\n\t"
                 "v_add_f32_dpp %2, %10, %10 row_half_mirror row_mask:0xf bank_mask:0xa\n\t"
                 "v_add_f32_dpp %3, %11, %11 row_half_mirror row_mask:0xf bank_mask:0xa"
                 : "=&v"(o2[0]), "=&v"(o2[1]), "=&v"(o2[2]), "=&v"(o2[3])
                 : "v"(o[0]), "v"(o[1]), "v"(o[2]), "v"(o[3]), "v"(o[4]), "v"(o[5]), "v"(o[6]), "v"(o[7]));
    // stages 3 and 4 pair lanes of one quad (xor 2, xor 1): keep / send chosen by a bit of the lane index
    const bool b1 = (nn & 2) != 0, b0 = (nn & 1) != 0;
    float o3[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const float keep = b1 ? o2[i + 2] : o2[i], send = b1 ? o2[i] : o2[i + 2];
        o3[i] = keep + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), 0x4E, 0xf, 0xf, true));
    }
    const float keep = b0 ? o3[1] : o3[0], send = b0 ? o3[0] : o3[1];
    return keep + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), 0xB1, 0xf, 0xf, true));
}

// The solve.  d = 64: four queries per wave, four 16-wide blocks, ten upper-triangular tiles per query.
//   in : acc[q][tix(I,J)]  tiles of T_q = -(Sigma~_q + lambda I), accumulator layout (destroyed)
//        tmu[P], tq[P]     lane (q, r): -mu~_q[16P + r] and -q_q[16P + r]  (both destroyed)
//        te[P], r0         WITH_U: lane (q, r): -r1_q[16P + r]; r0 of the lane's query
//        omega             omega of the lane's query (lane group g = query g)
//        scw               >= 4 * 16 * SC_PITCH floats of LDS owned by this wave; pivot_floor as in chol_inv16
//   out: y1[P] = y1_q[16P + r] in lane (q, r), y0 of the lane's query in every lane;  WITH_U: u1[P], u0 likewise
// with [omega mu~^T; mu~ Sigma~ + lambda I] [y0; y1] = [1; q] and, WITH_U, the same matrix times [u0; u1] = [r0; r1].
// LIVE < 4 (a call at d = 16 / 32 on zero-padded copies): feature blocks LIVE..3 of every key and query are zero, the
// matrix is block diagonal with lambda I in those blocks and their right-hand sides are zero, so the solution vanishes
// there and only blocks 0..LIVE-1 are factorised and substituted.
template <bool WITH_U, int LIVE = 4>
__device__ __forceinline__ void solve_wave_q4(f32x4 (&acc)[4][10], float (&tmu)[4], float (&tq)[4], float (&te)[4], float r0,
                                              float omega, float *scw, int g, int nn, float pivot_floor, float (&y1)[4],
                                              float &y0, float (&u1)[4], float &u0)
{
    using S = Shape<64>;
    constexpr int QW = 4, NB = LIVE;       // blocks LIVE..3 are lambda I with zero right-hand sides (see above): y1 = u1 = 0 there
    static_assert(LIVE >= 1 && LIVE <= 4, "four 16-wide blocks");
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};

    // ---- factorisation (as in factorise_wave): acc(P,J), P < J, becomes U(P,J); acc(P,P) becomes N_P = -U(P,P)^{-1} -----
#pragma unroll
    for (int P = 0; P < NB; ++P) {
#pragma unroll
        for (int q = 0; q < QW; ++q)
#pragma unroll
            for (int t = 0; t < 4; ++t) scw[q * 16 * SC_PITCH + (4 * g + t) * SC_PITCH + nn] = acc[q][S::tix(P, P)][t];
        wave_sync();
        float a[16], li[16];
        {
            const float *my = scw + g * 16 * SC_PITCH;
#pragma unroll
            for (int c4 = 0; c4 < 4; ++c4) {
                const f32x4 v = *reinterpret_cast<const f32x4 *>(my + nn * SC_PITCH + 4 * c4);
#pragma unroll
                for (int t = 0; t < 4; ++t) a[4 * c4 + t] = v[t];
            }
#pragma unroll
            for (int c = 0; c < 16; ++c) a[c] = -0.5f * (a[c] + my[c * SC_PITCH + nn]);    // -T, symmetrised
        }
        wave_sync();
        chol_inv16(a, li, nn, pivot_floor);
        {
            float *my = scw + g * 16 * SC_PITCH;
#pragma unroll
            for (int c4 = 0; c4 < 4; ++c4)
                *reinterpret_cast<f32x4 *>(my + nn * SC_PITCH + 4 * c4) = f32x4{li[4 * c4], li[4 * c4 + 1], li[4 * c4 + 2], li[4 * c4 + 3]};
        }
        wave_sync();
#pragma unroll
        for (int q = 0; q < QW; ++q) {
            const f32x4 ui = *reinterpret_cast<const f32x4 *>(scw + q * 16 * SC_PITCH + nn * SC_PITCH + 4 * g);
            acc[q][S::tix(P, P)] = ui;
#pragma unroll
            for (int J = P + 1; J < NB; ++J) acc[q][S::tix(P, J)] = tile_atb(zero, ui, acc[q][S::tix(P, J)]);
#pragma unroll
            for (int I = P + 1; I < NB; ++I)
#pragma unroll
                for (int J = I; J < NB; ++J) acc[q][S::tix(I, J)] = tile_atb(acc[q][S::tix(I, J)], acc[q][S::tix(P, I)], acc[q][S::tix(P, J)]);
            __builtin_amdgcn_sched_barrier(0);
        }
        wave_sync();
    }

    // ---- every tile from the accumulator layout to columns: lane (q, r) now holds column r of query q's tile,
    //      element c = 4 g' + t in register acc[g'][tile][t] ---------------------------------------------------------
#pragma unroll
    for (int I = 0; I < NB; ++I)
#pragma unroll
        for (int J = I; J < NB; ++J) {
            const int tl = S::tix(I, J);
            rows_transpose4(acc[0][tl], acc[1][tl], acc[2][tl], acc[3][tl]);
        }

    // ---- forward substitution of the right-hand sides: a_P = N_P^T t_P, then t_I += U(P,I)^T a_P for I > P ----------
#pragma unroll
    for (int P = 0; P < NB; ++P) {
        const int dt = S::tix(P, P);
        float am = 0.f, aq = 0.f, ae = 0.f;
        if constexpr (WITH_U) dot16_bcast3(am, aq, ae, tmu[P], tq[P], te[P], acc[0][dt], acc[1][dt], acc[2][dt], acc[3][dt]);
        else dot16_bcast2(am, aq, tmu[P], tq[P], acc[0][dt], acc[1][dt], acc[2][dt], acc[3][dt]);
        tmu[P] = am; tq[P] = aq;
        if constexpr (WITH_U) te[P] = ae;
#pragma unroll
        for (int I = P + 1; I < NB; ++I) {
            const int ot = S::tix(P, I);
            if constexpr (WITH_U) dot16_bcast3(tmu[I], tq[I], te[I], am, aq, ae, acc[0][ot], acc[1][ot], acc[2][ot], acc[3][ot]);
            else dot16_bcast2(tmu[I], tq[I], am, aq, acc[0][ot], acc[1][ot], acc[2][ot], acc[3][ot]);
        }
    }

    // tmu = a = U^{-T} mu~, tq = c = U^{-T} q (te = e = U^{-T} r1).  Schur step on the intercept:
    // y0 = (1 - a.c) / (omega - a.a), then y1 = U^{-1} (c - a y0), started as z = a y0 - c (the factors N_P are negated)
    float saa = 0.f, sac = 0.f, sae = 0.f;
#pragma unroll
    for (int P = 0; P < NB; ++P) {
        saa = fmaf(tmu[P], tmu[P], saa);
        sac = fmaf(tmu[P], tq[P], sac);
        if constexpr (WITH_U) sae = fmaf(tmu[P], te[P], sae);
    }
    saa = row_allsum(saa);
    sac = row_allsum(sac);
    const float dinv = 1.f / (omega - saa);
    y0 = (1.f - sac) * dinv;
    float z[4], zu[4];
#pragma unroll
    for (int P = NB; P < 4; ++P) { y1[P] = 0.f; u1[P] = 0.f; }
#pragma unroll
    for (int P = 0; P < NB; ++P) z[P] = tmu[P] * y0 - tq[P];
    if constexpr (WITH_U) {
        sae = row_allsum(sae);
        u0 = (r0 - sae) * dinv;
#pragma unroll
        for (int P = 0; P < NB; ++P) zu[P] = tmu[P] * u0 - te[P];
    }

    // ---- back substitution, block rows 3..0: x_P = N_P (z_P + sum_{J>P} U(P,J) x_J), outer-product form --------------
#pragma unroll
    for (int P = NB - 1; P >= 0; --P) {
        float w = z[P], wu = WITH_U ? zu[P] : 0.f;
        if (P < NB - 1) {
            float p[16], pu[16];
#pragma unroll
            for (int c = 0; c < 16; ++c) { p[c] = 0.f; pu[c] = 0.f; }
#pragma unroll
            for (int J = P + 1; J < NB; ++J) {
                const int ot = S::tix(P, J);
#pragma unroll
                for (int c = 0; c < 16; ++c) {
                    p[c] = fmaf(acc[c >> 2][ot][c & 3], y1[J], p[c]);
                    if constexpr (WITH_U) pu[c] = fmaf(acc[c >> 2][ot][c & 3], u1[J], pu[c]);
                }
            }
            w += row_transpose_sum(p, nn);
            if constexpr (WITH_U) wu += row_transpose_sum(pu, nn);
        }
        const int dt = S::tix(P, P);
        float p[16];
#pragma unroll
        for (int c = 0; c < 16; ++c) p[c] = acc[c >> 2][dt][c & 3] * w;
        y1[P] = row_transpose_sum(p, nn);
        if constexpr (WITH_U) {
#pragma unroll
            for (int c = 0; c < 16; ++c) p[c] = acc[c >> 2][dt][c & 3] * wu;
            u1[P] = row_transpose_sum(p, nn);
        }
    }
}

}  // namespace mfma
}  // namespace llla

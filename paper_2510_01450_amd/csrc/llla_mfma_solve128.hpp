// Exact solve of ONE augmented system per wave (head dimension 128, one query per wave): the 16-blocked Cholesky
// factorisation (factorise_wave) on the matrix cores, forward and back substitutions on the vector ALU.
//
// Why.  With one query per wave a substitution step is a 16x16 tile times two or three right-hand-side columns; as a
// 16x16x16 fp32 tile product it occupies the matrix cores for 128 cycles and uses two or three of sixteen output
// columns.  At d = 128 that is 88 of the 200 tile products of a row's solve, and with the eight waves of a workgroup
// solving at the same time the phase is bound by exactly those matrix-core cycles.  On the vector ALU the same step
// is four multiply-adds per lane and column:
//   * a tile stays in the accumulator layout: lane (g, n) holds X[4g+t][n] in register t;
//   * a vector block lives in one of two layouts: C, lane (g, n) holds element n (the same in every g), or R, lane
//     (g, n) holds elements 4g..4g+3 in four registers (the same in every n);
//   * X^T v (forward substitution: U^T a = b) takes v in R, multiplies per lane and sums over g (the four 16-lane rows of
//     the wave), which gives C;  X v (back substitution: U x = z) takes v in C, multiplies per lane and sums over n (the
//     16 lanes of a row), which gives R;
//   * C <-> R goes through the wave's scratch tile in LDS (16 floats per vector).
// The sign conventions are factorise_wave's: tiles hold T = -(Sigma~ + lambda I) factorised as U^T U with acc(P,P) = N_P =
// -U(P,P)^{-1}, right-hand sides come in negated.
#pragma once

#include "llla_mfma_common.hpp"
#include "llla_mfma_solve64.hpp"      // row_allsum

namespace llla {
namespace mfma {

// sum of x over the four 16-lane rows of the wave (same lane position), in every row
__device__ inline float rows_allsum(float x)
{
    x += __shfl_xor(x, 16);
    x += __shfl_xor(x, 32);
    return x;
}

//   in : acc[0][tix(I,J)]  upper-triangular 16x16 tiles of T = -(Sigma~ + lambda I), accumulator layout (destroyed)
//        load_rhs(P, m, q, e)  element 16P + n (n = the lane's position in its row) of -mu~, -q and, WITH_U, -r1
//        om4[0] = omega; scw: >= 16 * SC_PITCH floats of LDS owned by this wave; pivot_floor as in chol_inv16
//        WITH_U: r0v[0] = r0
//   out: rhs[0][P] register t = y1[16P + 4g + t] (every lane; WITH_U: lanes n == 1 hold u1 instead), y0v[0] = y0,
//        u0v[0] = u0
// with [omega mu~^T; mu~ Sigma~ + lambda I] [y0; y1] = [1; q] and, WITH_U, the same matrix times [u0; u1] = [r0; r1].
template <int DD, bool WITH_U = false, class LoadRhs>
__device__ __forceinline__ void solve_wave_v1(f32x4 (&acc)[1][Shape<DD>::NTILE], f32x4 (&rhs)[1][Shape<DD>::NB],
                                              float (&y0v)[1], const float (&om4)[1], float *scw, int g, int nn,
                                              float pivot_floor, LoadRhs load_rhs, const float *r0v = nullptr,
                                              float *u0v = nullptr)
{
    using S = Shape<DD>;
    constexpr int NB = S::NB, NS = WITH_U ? 3 : 2;
    static_assert(S::QW == 1, "one query per wave");

    factorise_wave<DD>(acc, scw, g, nn, pivot_floor);

    // C -> R and R -> C for NV vectors at once through the scratch tile (vector v at scw + 16 v)
    auto c_to_r = [&](const float (&c)[NS], f32x4 (&r)[NS], int nv) {
        if (g == 0) {
#pragma unroll
            for (int v = 0; v < NS; ++v) if (v < nv) scw[16 * v + nn] = c[v];
        }
        wave_sync();
#pragma unroll
        for (int v = 0; v < NS; ++v) if (v < nv) r[v] = *reinterpret_cast<const f32x4 *>(scw + 16 * v + 4 * g);
        wave_sync();
    };
    auto r_to_c = [&](const f32x4 (&r)[NS], float (&c)[NS], int nv) {
        if (nn == 0) {
#pragma unroll
            for (int v = 0; v < NS; ++v) if (v < nv) *reinterpret_cast<f32x4 *>(scw + 16 * v + 4 * g) = r[v];
        }
        wave_sync();
#pragma unroll
        for (int v = 0; v < NS; ++v) if (v < nv) c[v] = scw[16 * v + nn];
        wave_sync();
    };
    auto dot4 = [](const f32x4 &x, const f32x4 &v) { return fmaf(x[3], v[3], fmaf(x[2], v[2], fmaf(x[1], v[1], x[0] * v[0]))); };

    // ---- forward substitution of [mu~ q (r1)]:  t_P = -b_P + sum_{I<P} U(I,P)^T a_I,  a_P = N_P^T t_P -----------------
    float tv[NS][NB], part[NS][NB];        // C layout: right-hand sides, then the solutions a; partial sums over this lane's g
#pragma unroll
    for (int P = 0; P < NB; ++P) {
        float m = 0.f, q = 0.f, e = 0.f;
        load_rhs(P, m, q, e);
        tv[0][P] = m; tv[1][P] = q;
        if constexpr (WITH_U) tv[2][P] = e;
#pragma unroll
        for (int v = 0; v < NS; ++v) part[v][P] = 0.f;
    }
#pragma unroll
    for (int P = 0; P < NB; ++P) {
        float tc[NS];
        f32x4 tr[NS], ar[NS];
#pragma unroll
        for (int v = 0; v < NS; ++v) tc[v] = P == 0 ? tv[v][P] : tv[v][P] + rows_allsum(part[v][P]);
        c_to_r(tc, tr, NS);
        const f32x4 np = acc[0][S::tix(P, P)];
        float ac[NS];
#pragma unroll
        for (int v = 0; v < NS; ++v) {
            ac[v] = rows_allsum(dot4(np, tr[v]));
            tv[v][P] = ac[v];
        }
        if (P + 1 < NB) {
            c_to_r(ac, ar, NS);
#pragma unroll
            for (int I = P + 1; I < NB; ++I) {
                const f32x4 u = acc[0][S::tix(P, I)];
#pragma unroll
                for (int v = 0; v < NS; ++v) part[v][I] += dot4(u, ar[v]);
            }
        }
    }

    // tv[0] = a = U^{-T} mu~, tv[1] = c = U^{-T} q (tv[2] = e = U^{-T} r1).  Schur step on the intercept:
    // y0 = (1 - a.c) / (omega - a.a), then y1 = U^{-1} (c - a y0), started as z = a y0 - c (the factors N_P are negated)
    float saa = 0.f, sac = 0.f, sae = 0.f;
#pragma unroll
    for (int P = 0; P < NB; ++P) {
        saa = fmaf(tv[0][P], tv[0][P], saa);
        sac = fmaf(tv[0][P], tv[1][P], sac);
        if constexpr (WITH_U) sae = fmaf(tv[0][P], tv[2][P], sae);
    }
    saa = row_allsum(saa);
    sac = row_allsum(sac);
    const float dinv = 1.f / (om4[0] - saa);
    const float y0 = (1.f - sac) * dinv;
    y0v[0] = y0;
    float u0 = 0.f;
    if constexpr (WITH_U) {
        sae = row_allsum(sae);
        u0 = (r0v[0] - sae) * dinv;
        u0v[0] = u0;
    }
    constexpr int NZ = WITH_U ? 2 : 1;       // systems of the back substitution
    float zc[NZ][NB], xc[NZ][NB];            // C layout
#pragma unroll
    for (int P = 0; P < NB; ++P) {
        zc[0][P] = tv[0][P] * y0 - tv[1][P];
        if constexpr (WITH_U) zc[1][P] = tv[0][P] * u0 - tv[2][P];
    }

    // ---- back substitution, block rows NB-1..0:  x_P = N_P (z_P + sum_{J>P} U(P,J) x_J) ------------------------------
#pragma unroll
    for (int P = NB - 1; P >= 0; --P) {
        f32x4 ir[NS], xr[NS];
        float ic[NS];
#pragma unroll
        for (int v = 0; v < NZ; ++v) {
            // per lane: rows 4g+t of U(P,J) x_J restricted to column n, plus z_P on the diagonal positions
            f32x4 p;
#pragma unroll
            for (int t = 0; t < 4; ++t) p[t] = (nn == 4 * g + t) ? zc[v][P] : 0.f;
#pragma unroll
            for (int J = P + 1; J < NB; ++J) {
                const f32x4 u = acc[0][S::tix(P, J)];
#pragma unroll
                for (int t = 0; t < 4; ++t) p[t] = fmaf(u[t], xc[v][J], p[t]);
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) ir[v][t] = row_allsum(p[t]);
        }
        r_to_c(ir, ic, NZ);
        const f32x4 np = acc[0][S::tix(P, P)];
#pragma unroll
        for (int v = 0; v < NZ; ++v)
#pragma unroll
            for (int t = 0; t < 4; ++t) xr[v][t] = row_allsum(np[t] * ic[v]);
        rhs[0][P] = xr[0];
        if constexpr (WITH_U) rhs[0][P] = (nn == 1) ? xr[1] : xr[0];
        if (P > 0) {
            float c[NS];
            r_to_c(xr, c, NZ);
#pragma unroll
            for (int v = 0; v < NZ; ++v) xc[v][P] = c[v];
        }
    }
}

}  // namespace mfma
}  // namespace llla

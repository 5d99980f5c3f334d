// Backward pass of Local Linear Attention on the vector ALU (fp32 arithmetic; fp32 or bf16 inputs, every
// d in {16,32,64,128}, causal).
//
// The paper derives the backward in Appendix D in terms of the centred statistics (rho_i, delta_i) and one
// more linear solve per row (its u_i).  The same structure is used here in the un-centred augmented form of
// the forward kernels.  Per row i, with x_j = [1; k_j], w_ij = exp(scale q_i.k_j - m_i),
//     M_i = sum_j w_ij x_j x_j^T + lambda_i diag(0, I),   y_i = M_i^{-1} [1; q_i],   o_i = sum_j w_ij (x_j.y_i) v_j,
// an upstream gradient g_i = dL/do_i and gamma_ij = g_i.v_j (the paper's gamma_ij):
//     r_i = sum_j w_ij gamma_ij x_j,       u_i = M_i^{-1} r_i            (the one extra solve, same matrix)
//     a_ij = x_j.y_i,  b_ij = x_j.u_i,     s_ij = w_ij a_ij              (s_ij: the output weights of Eq. (lla))
//     e_ij = w_ij (gamma_ij - b_ij),       p_ij = a_ij e_ij = dL/d(logit_ij) at fixed row maximum
//     dV_j = sum_i s_ij g_i                                              (Appendix D: Delta_V = S^T G)
//     dK_j = sum_i [ e_ij y1_i - s_ij u1_i + scale p^_ij q_i ]
//     dQ_i = u1_i + scale sum_j p^_ij k_j
//     dL/dlambda_i = -u1_i.y1_i
// where y = [y0; y1], u = [u0; u1].  The ridge acts on max-normalised weights, so o_i also depends on the row
// maximum m_i: by homogeneity (scaling all weights and the ridge together changes nothing) that dependence is
// lambda_i dL/dlambda_i, and it enters the logit of the key that holds the maximum:
// p^_ij = p_ij + [j = argmax_i] lambda_i dL/dlambda_i.
//
// Two kernels.  bwd_rows_kernel (one slot per query row, the structure of the forward vector kernel): moments and
// r_i in one sweep with a running maximum, the (d+1)x(d+1) system with two right-hand sides solved by elimination in
// LDS, a second sweep for dQ_i; it leaves (y_i, u_i, m_i, correction, argmax) of every row in the workspace.
// bwd_keys_kernel (one workgroup per block of keys): sweeps the query rows at and after the block and accumulates
// dK_j, dV_j in registers -- no atomics, deterministic.
#include "llla_valu_common.hpp"

namespace llla {
namespace {

using namespace valu;

// per-row record in the workspace, in floats: y1 [D], u1 [D], y0, u0, m, correction, argmax (int bits), 3 pad
template <int D>
constexpr int rec_floats() { return 2 * D + 8; }

template <int D, typename TI>
__global__ __launch_bounds__(NT) void bwd_rows_kernel(const TI *__restrict__ Qg, const TI *__restrict__ Kg,
                                                      const TI *__restrict__ Vg, const TI *__restrict__ Gg,
                                                      llla_strides sq, llla_strides sk, llla_strides sv,
                                                      llla_strides sg, int H, int nbh, int n, float lambda,
                                                      const float *__restrict__ LamRows, float scale,
                                                      float *__restrict__ Rec, float *__restrict__ dQ,
                                                      float *__restrict__ dLam)
{
    using C = Cfg<D>;
    constexpr int TS = C::TS, TG = C::TG, TPQ = C::TPQ, QB = C::QB, LDK = C::LDK, P = C::P;
    constexpr int LS = (D + 3) | 1;                      // odd pitch of [At | e | r]
    constexpr int TILE_F = 2 * KT * LDK + 3 * QB * KT;   // ks, vs, logits, weights, gammas
    constexpr int SYS_F = QB * P * LS;
    constexpr int UNION_F = (((TILE_F > SYS_F) ? TILE_F : SYS_F) + 3) & ~3;   // keeps the rows after it 16-byte aligned
    constexpr int REC = rec_floats<D>();

    __shared__ __align__(16) float smem[UNION_F + 4 * QB * D + 8 * QB];
    float *ks = smem;                                     // [KT][LDK]
    float *vs = ks + KT * LDK;                            // [KT][LDK]
    float *sl = vs + KT * LDK;                            // [QB][KT] logits, later p^
    float *wl = sl + QB * KT;                             // [QB][KT] weights
    float *gl = wl + QB * KT;                             // [QB][KT] gamma
    float *sys = smem;                                    // [QB][P][LS], aliases the tiles
    float *qs = smem + UNION_F;                           // [QB][D]
    float *gs = qs + QB * D;                              // [QB][D]
    float *y1s = gs + QB * D;                             // [QB][D]
    float *u1s = y1s + QB * D;                            // [QB][D]
    float *y0s = u1s + QB * D;                            // [QB]
    float *u0s = y0s + QB;                                // [QB]
    float *ms = u0s + QB;                                 // [QB] running max
    float *al = ms + QB;                                  // [QB] rescale factor of this tile
    float *cr = al + QB;                                  // [QB] lambda dL/dlambda
    int *jst = reinterpret_cast<int *>(cr + QB);          // [QB] key index of the row maximum

    const int tid = threadIdx.x;
    const int slot = tid / TPQ;
    const int r = tid % TPQ;
    const int ta = r / TG, tb = r % TG;
    // one-dimensional grid, (batch, head) index fastest: the longest query blocks of every head are dispatched first
    const int bh = (int)(blockIdx.x % (unsigned)nbh);
    const int b = bh / H, h = bh % H;

    const TI *Kh = Kg + b * sk.batch + h * sk.head;
    const TI *Vh = Vg + b * sv.batch + h * sv.head;

    const int nqb = (int)(gridDim.x / (unsigned)nbh);
    const int i0 = (nqb - 1 - (int)(blockIdx.x / (unsigned)nbh)) * QB;
    const int my_i = i0 + slot;
    const bool slot_live = my_i < n;
    const int kend = min(n, i0 + QB);
    const int my_last = min(my_i, n - 1);
    const float lam_slot = LamRows ? LamRows[(size_t)bh * n + my_last] : lambda;

    for (int idx = tid; idx < QB * D; idx += NT) {
        const int s = idx / D, c = idx % D;
        float qv = 0.f, gv = 0.f;
        if (i0 + s < n) {
            const TI *qp = Qg + b * sq.batch + h * sq.head + (int64_t)(i0 + s) * sq.seq;
            const TI *gp = Gg + b * sg.batch + h * sg.head + (int64_t)(i0 + s) * sg.seq;
            qv = sizeof(TI) == 2 ? bf16_to_f32(((const bf16_t *)qp)[c]) : ((const float *)qp)[c];
            gv = sizeof(TI) == 2 ? bf16_to_f32(((const bf16_t *)gp)[c]) : ((const float *)gp)[c];
        }
        qs[idx] = qv;
        gs[idx] = gv;
    }
    if (tid < QB) {
        ms[tid] = -INFINITY;
        jst[tid] = 0;
    }

    // ---- sweep 1: un-centred moments and r = sum_j w_j gamma_j [1; k_j], running max ------------------
    {
        float acc[TS][TS];
        float mu[TS], rr[TS];
        float omega = 0.f, r0 = 0.f;
#pragma unroll
        for (int x = 0; x < TS; ++x) {
            mu[x] = 0.f;
            rr[x] = 0.f;
#pragma unroll
            for (int y = 0; y < TS; ++y) acc[x][y] = 0.f;
        }

        for (int kt0 = 0; kt0 < kend; kt0 += KT) {
            __syncthreads();
            load_tile<D, TI>(ks, Kh, sk.seq, kt0, KT, n, tid);
            load_tile<D, TI>(vs, Vh, sv.seq, kt0, KT, n, tid);
            __syncthreads();
            for (int idx = tid; idx < QB * KT; idx += NT) {
                const int s = idx / KT, kj = idx % KT;
                const int j = kt0 + kj;
                float v = -INFINITY, gm = 0.f;
                if (j <= min(i0 + s, n - 1)) {
                    v = scale * dot_lds<D>(qs + s * D, ks + kj * LDK);
                    gm = dot_lds<D>(gs + s * D, vs + kj * LDK);
                }
                sl[idx] = v;
                gl[idx] = gm;
            }
            __syncthreads();
            if (tid < QB) {                                  // running max (first key that attains it) per slot
                float mx = ms[tid];
                const float mold = mx;
                int arg = jst[tid];
                for (int kj = 0; kj < KT; ++kj) {
                    const float v = sl[tid * KT + kj];
                    if (v > mx) {
                        mx = v;
                        arg = kt0 + kj;
                    }
                }
                ms[tid] = mx;
                jst[tid] = arg;
                al[tid] = (mold == -INFINITY) ? 0.f : __expf(mold - mx);
            }
            __syncthreads();
            for (int idx = tid; idx < QB * KT; idx += NT) {
                const float mx = ms[idx / KT];
                const float s = sl[idx];
                wl[idx] = (s == -INFINITY) ? 0.f : __expf(s - mx);
            }
            __syncthreads();
            {
                const float alpha = al[slot];
                if (alpha != 1.f) {
                    omega *= alpha;
                    r0 *= alpha;
#pragma unroll
                    for (int x = 0; x < TS; ++x) {
                        mu[x] *= alpha;
                        rr[x] *= alpha;
#pragma unroll
                        for (int y = 0; y < TS; ++y) acc[x][y] *= alpha;
                    }
                }
                const int jn = min(KT, my_last - kt0 + 1);
                for (int kj = 0; kj < jn; ++kj) {
                    const float w = wl[slot * KT + kj];
                    const float gm = gl[slot * KT + kj];
                    const float *krow = ks + kj * LDK;
                    float a[TS], bb[TS];
#pragma unroll
                    for (int x = 0; x < TS; x += 4) {
                        const float4 va = *reinterpret_cast<const float4 *>(krow + ta * TS + x);
                        const float4 vb = *reinterpret_cast<const float4 *>(krow + tb * TS + x);
                        a[x] = va.x * w; a[x + 1] = va.y * w; a[x + 2] = va.z * w; a[x + 3] = va.w * w;
                        bb[x] = vb.x; bb[x + 1] = vb.y; bb[x + 2] = vb.z; bb[x + 3] = vb.w;
                    }
                    omega += w;
                    r0 = fmaf(w, gm, r0);
#pragma unroll
                    for (int x = 0; x < TS; ++x) {
                        mu[x] += a[x];
                        rr[x] = fmaf(a[x], gm, rr[x]);
#pragma unroll
                        for (int y = 0; y < TS; ++y) acc[x][y] = fmaf(a[x], bb[y], acc[x][y]);
                    }
                }
            }
        }
        __syncthreads();                                     // tiles are dead; sys may overwrite them

        // ---- [At | e | r] in LDS ---------------------------------------------------------------------
        float *S = sys + slot * P * LS;
#pragma unroll
        for (int x = 0; x < TS; ++x)
#pragma unroll
            for (int y = 0; y < TS; ++y) {
                const int rw = ta * TS + x, cc = tb * TS + y;
                S[(1 + rw) * LS + 1 + cc] = acc[x][y] + (rw == cc ? lam_slot : 0.f);
            }
        if (tb == 0) {
#pragma unroll
            for (int x = 0; x < TS; ++x) {
                S[(1 + ta * TS + x) * LS] = mu[x];
                S[1 + ta * TS + x] = mu[x];
                S[(1 + ta * TS + x) * LS + P + 1] = rr[x];
            }
        }
        if (r == 0) {
            S[0] = slot_live ? omega : 1.f;                  // a dead slot (row >= n) gets a harmless pivot
            S[P] = 1.f;
            S[P + 1] = r0;
        }
        for (int c = r; c < D; c += TPQ) S[(c + 1) * LS + P] = qs[slot * D + c];

        // ---- elimination with two right-hand sides (the matrix is symmetric positive definite) -------
        for (int k = 0; k < P; ++k) {
            __syncthreads();
            const float pinv = 1.f / S[k * LS + k];
            for (int row = k + 1 + r; row < P; row += TPQ) {
                const float f = S[row * LS + k] * pinv;
                for (int c = k + 1; c <= P + 1; ++c) S[row * LS + c] = fmaf(-f, S[k * LS + c], S[row * LS + c]);
            }
        }
        for (int k = P - 1; k >= 0; --k) {
            __syncthreads();
            const float pinv = 1.f / S[k * LS + k];
            const float yk = S[k * LS + P] * pinv;
            const float uk = S[k * LS + P + 1] * pinv;
            if (r == 0) {
                if (k == 0) {
                    y0s[slot] = yk;
                    u0s[slot] = uk;
                } else {
                    y1s[slot * D + k - 1] = yk;
                    u1s[slot * D + k - 1] = uk;
                }
            }
            for (int row = r; row < k; row += TPQ) {
                S[row * LS + P] = fmaf(-S[row * LS + k], yk, S[row * LS + P]);
                S[row * LS + P + 1] = fmaf(-S[row * LS + k], uk, S[row * LS + P + 1]);
            }
        }
        __syncthreads();
    }

    // ---- dL/dlambda_i, the correction of the maximum's logit, and the row record for the key sweep ------
    if (r == 0) {
        float dl = 0.f;
        for (int c = 0; c < D; ++c) dl = fmaf(-u1s[slot * D + c], y1s[slot * D + c], dl);
        cr[slot] = lam_slot * dl;
        if (slot_live) {
            float *rec = Rec + ((size_t)bh * n + my_i) * REC + 2 * D;
            rec[0] = y0s[slot];
            rec[1] = u0s[slot];
            rec[2] = ms[slot];
            rec[3] = lam_slot * dl;
            rec[4] = __int_as_float(jst[slot]);
            if (dLam) dLam[(size_t)bh * n + my_i] = dl;
        }
    }
    if (slot_live) {
        float *rec = Rec + ((size_t)bh * n + my_i) * REC;
        for (int c = r; c < D; c += TPQ) {
            rec[c] = y1s[slot * D + c];
            rec[D + c] = u1s[slot * D + c];
        }
    }

    // ---- sweep 2: p^_ij and dQ_i = u1_i + scale sum_j p^_ij k_j -------------------------------------
    float dq = 0.f;
    for (int kt0 = 0; kt0 < kend; kt0 += KT) {
        __syncthreads();
        load_tile<D, TI>(ks, Kh, sk.seq, kt0, KT, n, tid);
        load_tile<D, TI>(vs, Vh, sv.seq, kt0, KT, n, tid);
        __syncthreads();
        for (int idx = tid; idx < QB * KT; idx += NT) {
            const int s = idx / KT, kj = idx % KT;
            const int j = kt0 + kj;
            float pv = 0.f;
            if (j <= min(i0 + s, n - 1)) {
                const float *krow = ks + kj * LDK;
                const float lg = scale * dot_lds<D>(qs + s * D, krow);
                const float w = __expf(lg - ms[s]);
                const float a = y0s[s] + dot_lds<D>(y1s + s * D, krow);
                const float bb = u0s[s] + dot_lds<D>(u1s + s * D, krow);
                const float gm = dot_lds<D>(gs + s * D, vs + kj * LDK);
                pv = w * a * (gm - bb);
                if (j == jst[s]) pv += cr[s];
            }
            sl[idx] = pv;
        }
        __syncthreads();
        if (r < D) {
            const int jn = min(KT, my_last - kt0 + 1);
            for (int kj = 0; kj < jn; ++kj) dq = fmaf(sl[slot * KT + kj], ks[kj * LDK + r], dq);
        }
    }
    if (slot_live && r < D) dQ[((size_t)bh * n + my_i) * D + r] = fmaf(scale, dq, u1s[slot * D + r]);
}

// ---- fp32 row sweeps for the first rows of the matrix-core flow -----------------------------------------------
// With bf16 inputs and d = 64 / 128 the moments and both solves of a row run on the matrix cores, and so do the two
// O(d)-per-pair sweeps over a row's keys -- except for the first 2d rows of a sequence: their systems are the worst
// conditioned, u_i and the coefficients are large and cancel (dQ_0 is exactly 0 as the difference of two large
// terms), and a 16-bit coefficient split is not enough there.  Those rows take these fp32 sweeps:
//   MODE 0 (before the solve): r_i = sum_j w_ij gamma_ij [1; k_j] and the key that holds the row maximum;
//   MODE 1 (after it):         dL/dlambda_i, the correction, dQ_i = u1_i + scale sum_j p^_ij k_j, and the row scalars
//                              the key sweep reads.
// The row maxima come from the matrix-core sweep (log2 units), so that all kernels normalise a row alike.
template <int D>
struct RowCfg {
    static constexpr int QT = (D == 16) ? 64 : ((D >= 128) ? 16 : 32);   // query rows per workgroup
    static constexpr int FPT = D * QT / NT;              // features per thread in the accumulation
    static constexpr int TPR = NT / QT;                  // threads per row
    static constexpr int KB = 32;                        // keys per tile
    static constexpr int KPT = QT * KB / NT;             // keys per thread when the coefficients are formed
    static constexpr int JG = KB / KPT;
    static constexpr int CP = KB + 1;
};

template <int D, typename TI, int MODE>
__global__ __launch_bounds__(NT) void bwd_rowsweep_kernel(const TI *__restrict__ Qg, const TI *__restrict__ Kg,
                                                          const TI *__restrict__ Vg, const TI *__restrict__ Gg,
                                                          llla_strides sq, llla_strides sk, llla_strides sv,
                                                          llla_strides sg, int H, int n, int nrows, float scale,
                                                          float lambda, const float *__restrict__ LamRows,
                                                          const float *__restrict__ M, int mpitch,
                                                          const float *__restrict__ Yv, const float *__restrict__ Uv,
                                                          float *__restrict__ Rv, int vpitch, float *__restrict__ Sc,
                                                          float *__restrict__ dQ, float *__restrict__ dLam)
{
    using C = RowCfg<D>;
    constexpr int QT = C::QT, FPT = C::FPT, TPR = C::TPR, KB = C::KB, KPT = C::KPT, JG = C::JG, CP = C::CP;
    constexpr int LDK = Cfg<D>::LDK;
    constexpr int NROWT = (MODE == 1) ? 4 : 2;           // row-side tiles: q, g (, y1, u1)
    static_assert(QT * JG == NT && QT * TPR == NT && FPT % 4 == 0, "thread maps");

    __shared__ __align__(16) float smem[(2 * KB + NROWT * QT) * LDK + 2 * QT * CP + QT * 8];
    float *ks = smem;                                     // [KB][LDK]
    float *vs = ks + KB * LDK;                            // [KB][LDK]
    float *qs = vs + KB * LDK;                            // [QT][LDK]
    float *gs = qs + QT * LDK;                            // [QT][LDK]
    float *y1s = gs + QT * LDK;                           // [QT][LDK]  (MODE 1)
    float *u1s = y1s + QT * LDK;                          // [QT][LDK]  (MODE 1)
    float *cs = smem + (2 * KB + NROWT * QT) * LDK;       // [QT][CP] coefficients
    float *ss = cs + QT * CP;                             // [QT][CP] logits (MODE 0)
    float *rs = ss + QT * CP;                             // [QT][8]  m, y0, u0, correction, argmax / running max

    const int tid = threadIdx.x;
    const int bh = blockIdx.y;
    const int b = bh / H, h = bh % H;
    const int i0 = ((int)gridDim.x - 1 - (int)blockIdx.x) * QT;          // long rows first
    const int kend = min(nrows, i0 + QT);                                // rows [0, nrows) only; nrows <= n
    const TI *Kh = Kg + b * sk.batch + h * sk.head;
    const TI *Vh = Vg + b * sv.batch + h * sv.head;

    load_tile<D, TI>(qs, Qg + b * sq.batch + h * sq.head, sq.seq, i0, QT, n, tid);
    load_tile<D, TI>(gs, Gg + b * sg.batch + h * sg.head, sg.seq, i0, QT, n, tid);
    if (MODE == 1) {
        load_tile<D, float>(y1s, Yv + (size_t)bh * n * vpitch, vpitch, i0, QT, n, tid);
        load_tile<D, float>(u1s, Uv + (size_t)bh * n * vpitch, vpitch, i0, QT, n, tid);
    }
    __syncthreads();
    if (tid < QT) {
        const int i = min(i0 + tid, n - 1);
        const size_t row = (size_t)bh * n + i;
        const float m = M[(size_t)bh * mpitch + i] * 0.6931471805599453f;
        rs[tid * 8 + 0] = m;
        if (MODE == 1) {
            const float y0 = Yv[row * vpitch + D], u0 = Uv[row * vpitch + D];
            const float jbits = Rv[row * vpitch + D + 1];
            float dl = 0.f;
            for (int c = 0; c < D; ++c) dl = fmaf(-u1s[tid * LDK + c], y1s[tid * LDK + c], dl);
            const float corr = (LamRows ? LamRows[row] : lambda) * dl;
            rs[tid * 8 + 1] = y0;
            rs[tid * 8 + 2] = u0;
            rs[tid * 8 + 3] = corr;
            rs[tid * 8 + 4] = jbits;
            if (i0 + tid < nrows) {
                float *sc = Sc + row * 8;
                sc[0] = y0; sc[1] = u0; sc[2] = m; sc[3] = corr; sc[4] = jbits;
                if (dLam) dLam[row] = dl;
            }
        } else {
            rs[tid * 8 + 5] = -INFINITY;                  // running maximum of the fp32 logits
            rs[tid * 8 + 6] = __int_as_float(0);          // and the first key that attains it
        }
    }

    const int ai = tid / JG, ajg = tid % JG;             // coefficient phase: row and key group
    const int bi = tid / TPR, bc = (tid % TPR) * FPT;    // accumulation phase: row and feature chunk
    float acc[FPT];
    float r0 = 0.f;
#pragma unroll
    for (int x = 0; x < FPT; ++x) acc[x] = 0.f;

    for (int kt0 = 0; kt0 < kend; kt0 += KB) {
        __syncthreads();
        load_tile<D, TI>(ks, Kh, sk.seq, kt0, KB, n, tid);
        load_tile<D, TI>(vs, Vh, sv.seq, kt0, KB, n, tid);
        __syncthreads();
        {
            const int ig = i0 + ai;
            float ds[KPT], da[KPT], db[KPT], dg[KPT];
#pragma unroll
            for (int k = 0; k < KPT; ++k) ds[k] = da[k] = db[k] = dg[k] = 0.f;
            for (int c = 0; c < D; c += 4) {
                const float4 q4 = *reinterpret_cast<const float4 *>(qs + ai * LDK + c);
                const float4 g4 = *reinterpret_cast<const float4 *>(gs + ai * LDK + c);
                float4 y4 = make_float4(0.f, 0.f, 0.f, 0.f), u4 = y4;
                if (MODE == 1) {
                    y4 = *reinterpret_cast<const float4 *>(y1s + ai * LDK + c);
                    u4 = *reinterpret_cast<const float4 *>(u1s + ai * LDK + c);
                }
#pragma unroll
                for (int k = 0; k < KPT; ++k) {
                    const int j = ajg + k * JG;
                    const float4 k4 = *reinterpret_cast<const float4 *>(ks + j * LDK + c);
                    const float4 v4 = *reinterpret_cast<const float4 *>(vs + j * LDK + c);
                    ds[k] = fmaf(q4.x, k4.x, fmaf(q4.y, k4.y, fmaf(q4.z, k4.z, fmaf(q4.w, k4.w, ds[k]))));
                    dg[k] = fmaf(g4.x, v4.x, fmaf(g4.y, v4.y, fmaf(g4.z, v4.z, fmaf(g4.w, v4.w, dg[k]))));
                    if (MODE == 1) {
                        da[k] = fmaf(y4.x, k4.x, fmaf(y4.y, k4.y, fmaf(y4.z, k4.z, fmaf(y4.w, k4.w, da[k]))));
                        db[k] = fmaf(u4.x, k4.x, fmaf(u4.y, k4.y, fmaf(u4.z, k4.z, fmaf(u4.w, k4.w, db[k]))));
                    }
                }
            }
            const float m = rs[ai * 8 + 0];
#pragma unroll
            for (int k = 0; k < KPT; ++k) {
                const int j = ajg + k * JG;
                const bool valid = (kt0 + j <= ig) && (ig < nrows);
                float cv = 0.f;
                if (MODE == 0) {
                    const float lg = scale * ds[k];
                    if (valid) cv = __expf(lg - m) * dg[k];
                    ss[ai * CP + j] = valid ? lg : -INFINITY;
                } else if (valid) {
                    const float w = __expf(scale * ds[k] - m);
                    cv = w * (rs[ai * 8 + 1] + da[k]) * (dg[k] - (rs[ai * 8 + 2] + db[k]));
                    if (kt0 + j == __float_as_int(rs[ai * 8 + 4])) cv += rs[ai * 8 + 3];
                }
                cs[ai * CP + j] = cv;
            }
        }
        __syncthreads();
        if (MODE == 0 && tid < QT) {                         // first key with the largest logit so far
            float mx = rs[tid * 8 + 5];
            int arg = __float_as_int(rs[tid * 8 + 6]);
            for (int j = 0; j < KB; ++j) {
                const float v = ss[tid * CP + j];
                if (v > mx) {
                    mx = v;
                    arg = kt0 + j;
                }
            }
            rs[tid * 8 + 5] = mx;
            rs[tid * 8 + 6] = __int_as_float(arg);
        }
        for (int j = 0; j < KB; ++j) {
            const float cv = cs[bi * CP + j];
            r0 += cv;
#pragma unroll
            for (int x = 0; x < FPT; x += 4) {
                const float4 k4 = *reinterpret_cast<const float4 *>(ks + j * LDK + bc + x);
                acc[x] = fmaf(cv, k4.x, acc[x]);
                acc[x + 1] = fmaf(cv, k4.y, acc[x + 1]);
                acc[x + 2] = fmaf(cv, k4.z, acc[x + 2]);
                acc[x + 3] = fmaf(cv, k4.w, acc[x + 3]);
            }
        }
    }
    __syncthreads();
    if (i0 + bi < nrows) {
        const size_t row = (size_t)bh * n + i0 + bi;
        if (MODE == 0) {
            float *rr = Rv + row * vpitch;
#pragma unroll
            for (int x = 0; x < FPT; x += 4)
                *reinterpret_cast<float4 *>(rr + bc + x) = make_float4(acc[x], acc[x + 1], acc[x + 2], acc[x + 3]);
            if (bc == 0) {
                rr[D] = r0;
                rr[D + 1] = rs[bi * 8 + 6];
            }
        } else {
            float *qr = dQ + row * D;
#pragma unroll
            for (int x = 0; x < FPT; x += 4)
                *reinterpret_cast<float4 *>(qr + bc + x) =
                    make_float4(fmaf(scale, acc[x], u1s[bi * LDK + bc + x]), fmaf(scale, acc[x + 1], u1s[bi * LDK + bc + x + 1]),
                                fmaf(scale, acc[x + 2], u1s[bi * LDK + bc + x + 2]), fmaf(scale, acc[x + 3], u1s[bi * LDK + bc + x + 3]));
        }
    }
}

// ---- key sweep ------------------------------------------------------------------------------------------
template <int D>
struct KeyCfg {
    static constexpr int FPT = (D >= 64) ? 8 : 4;        // features per thread in the accumulation
    static constexpr int KB = NT * FPT / D;              // keys per workgroup
    static constexpr int TPK = D / FPT;                  // threads per key
    static constexpr int QT = (D >= 128) ? 16 : 32;      // query rows per tile
    static constexpr int KPT = QT * KB / NT;             // keys per thread when the coefficients are formed
    static constexpr int JG = KB / KPT;                  // key groups
    static constexpr int CP = KB + 1;                    // pitch of the coefficient tiles
};

template <int D, typename TI>
__global__ __launch_bounds__(NT) void bwd_keys_kernel(const TI *__restrict__ Qg, const TI *__restrict__ Kg,
                                                      const TI *__restrict__ Vg, const TI *__restrict__ Gg,
                                                      llla_strides sq, llla_strides sk, llla_strides sv,
                                                      llla_strides sg, int H, int nbh, int n, float scale,
                                                      const float *__restrict__ Y1, const float *__restrict__ U1,
                                                      int vpitch, const float *__restrict__ Sc, int spitch,
                                                      float *__restrict__ dK, float *__restrict__ dV)
{
    // Y1, U1: rows of y1_i, u1_i (pitch vpitch floats); Sc: per row y0, u0, m, correction, argmax (pitch spitch)
    using C = KeyCfg<D>;
    constexpr int FPT = C::FPT, KB = C::KB, TPK = C::TPK, QT = C::QT, KPT = C::KPT, JG = C::JG, CP = C::CP;
    constexpr int LDK = Cfg<D>::LDK;
    static_assert(QT * JG == NT, "one thread per (query row, key group)");
    static_assert(KB * TPK == NT, "one thread per (key, feature chunk)");

    __shared__ __align__(16) float smem[(2 * KB + 4 * QT) * LDK + 3 * QT * CP + QT * 8];
    float *ks = smem;                                     // [KB][LDK]
    float *vs = ks + KB * LDK;                            // [KB][LDK]
    float *qs = vs + KB * LDK;                            // [QT][LDK]
    float *gs = qs + QT * LDK;                            // [QT][LDK]
    float *y1s = gs + QT * LDK;                           // [QT][LDK]
    float *u1s = y1s + QT * LDK;                          // [QT][LDK]
    float *cs = u1s + QT * LDK;                           // [QT][CP] s_ij
    float *ce = cs + QT * CP;                             // [QT][CP] e_ij
    float *cp = ce + QT * CP;                             // [QT][CP] scale p^_ij
    float *rs = cp + QT * CP;                             // [QT][8]  y0, u0, m, correction, argmax

    const int tid = threadIdx.x;
    // one-dimensional grid, (batch, head) index fastest; low key blocks see the most rows: they go first for every head
    const int bh = (int)(blockIdx.x % (unsigned)nbh);
    const int b = bh / H, h = bh % H;
    const int j0 = (int)(blockIdx.x / (unsigned)nbh) * KB;
    const TI *Qh = Qg + b * sq.batch + h * sq.head;
    const TI *Gh = Gg + b * sg.batch + h * sg.head;
    const float *Y1h = Y1 + (size_t)bh * n * vpitch, *U1h = U1 + (size_t)bh * n * vpitch;
    const float *Sh = Sc + (size_t)bh * n * spitch;

    load_tile<D, TI>(ks, Kg + b * sk.batch + h * sk.head, sk.seq, j0, KB, n, tid);
    load_tile<D, TI>(vs, Vg + b * sv.batch + h * sv.head, sv.seq, j0, KB, n, tid);

    // coefficient phase: this thread's query row of the tile and its keys jg, jg + JG, ...
    const int ai = tid / JG, ajg = tid % JG;
    // accumulation phase: this thread's key and feature chunk
    const int bj = tid / TPK, bc = (tid % TPK) * FPT;

    float dk[FPT], dv[FPT];
#pragma unroll
    for (int x = 0; x < FPT; ++x) {
        dk[x] = 0.f;
        dv[x] = 0.f;
    }

    for (int it0 = j0 - (j0 % QT); it0 < n; it0 += QT) {
        __syncthreads();                                     // previous tile fully consumed
        load_tile<D, TI>(qs, Qh, sq.seq, it0, QT, n, tid);
        load_tile<D, TI>(gs, Gh, sg.seq, it0, QT, n, tid);
        load_tile<D, float>(y1s, Y1h, vpitch, it0, QT, n, tid);
        load_tile<D, float>(u1s, U1h, vpitch, it0, QT, n, tid);
        if (tid < QT * 8) {
            const int i = tid / 8, c = tid % 8;
            rs[tid] = (it0 + i < n && c < 5) ? Sh[(size_t)(it0 + i) * spitch + c] : 0.f;
        }
        __syncthreads();
        {
            const int ig = it0 + ai;
            float ds[KPT], da[KPT], db[KPT], dg[KPT];
#pragma unroll
            for (int k = 0; k < KPT; ++k) ds[k] = da[k] = db[k] = dg[k] = 0.f;
            for (int c = 0; c < D; c += 4) {
                const float4 q4 = *reinterpret_cast<const float4 *>(qs + ai * LDK + c);
                const float4 y4 = *reinterpret_cast<const float4 *>(y1s + ai * LDK + c);
                const float4 u4 = *reinterpret_cast<const float4 *>(u1s + ai * LDK + c);
                const float4 g4 = *reinterpret_cast<const float4 *>(gs + ai * LDK + c);
#pragma unroll
                for (int k = 0; k < KPT; ++k) {
                    const int j = ajg + k * JG;
                    const float4 k4 = *reinterpret_cast<const float4 *>(ks + j * LDK + c);
                    const float4 v4 = *reinterpret_cast<const float4 *>(vs + j * LDK + c);
                    ds[k] = fmaf(q4.x, k4.x, fmaf(q4.y, k4.y, fmaf(q4.z, k4.z, fmaf(q4.w, k4.w, ds[k]))));
                    da[k] = fmaf(y4.x, k4.x, fmaf(y4.y, k4.y, fmaf(y4.z, k4.z, fmaf(y4.w, k4.w, da[k]))));
                    db[k] = fmaf(u4.x, k4.x, fmaf(u4.y, k4.y, fmaf(u4.z, k4.z, fmaf(u4.w, k4.w, db[k]))));
                    dg[k] = fmaf(g4.x, v4.x, fmaf(g4.y, v4.y, fmaf(g4.z, v4.z, fmaf(g4.w, v4.w, dg[k]))));
                }
            }
            const float y0 = rs[ai * 8 + 0], u0 = rs[ai * 8 + 1], m = rs[ai * 8 + 2], corr = rs[ai * 8 + 3];
            const int jstar = __float_as_int(rs[ai * 8 + 4]);
#pragma unroll
            for (int k = 0; k < KPT; ++k) {
                const int j = ajg + k * JG;
                float s_ = 0.f, e_ = 0.f, p_ = 0.f;
                if (j0 + j <= ig && ig < n) {
                    const float w = __expf(scale * ds[k] - m);
                    const float a = y0 + da[k];
                    e_ = w * (dg[k] - (u0 + db[k]));
                    s_ = w * a;
                    p_ = a * e_;
                    if (j0 + j == jstar) p_ += corr;
                    p_ *= scale;
                }
                cs[ai * CP + j] = s_;
                ce[ai * CP + j] = e_;
                cp[ai * CP + j] = p_;
            }
        }
        __syncthreads();
        for (int i = 0; i < QT; ++i) {
            if (it0 + i < j0 || it0 + i >= n) continue;      // uniform: the row is before the block or beyond the end
            const float s_ = cs[i * CP + bj], e_ = ce[i * CP + bj], p_ = cp[i * CP + bj];
#pragma unroll
            for (int x = 0; x < FPT; x += 4) {
                const float4 g4 = *reinterpret_cast<const float4 *>(gs + i * LDK + bc + x);
                const float4 y4 = *reinterpret_cast<const float4 *>(y1s + i * LDK + bc + x);
                const float4 u4 = *reinterpret_cast<const float4 *>(u1s + i * LDK + bc + x);
                const float4 q4 = *reinterpret_cast<const float4 *>(qs + i * LDK + bc + x);
                dv[x] = fmaf(s_, g4.x, dv[x]);
                dv[x + 1] = fmaf(s_, g4.y, dv[x + 1]);
                dv[x + 2] = fmaf(s_, g4.z, dv[x + 2]);
                dv[x + 3] = fmaf(s_, g4.w, dv[x + 3]);
                dk[x] = fmaf(p_, q4.x, fmaf(-s_, u4.x, fmaf(e_, y4.x, dk[x])));
                dk[x + 1] = fmaf(p_, q4.y, fmaf(-s_, u4.y, fmaf(e_, y4.y, dk[x + 1])));
                dk[x + 2] = fmaf(p_, q4.z, fmaf(-s_, u4.z, fmaf(e_, y4.z, dk[x + 2])));
                dk[x + 3] = fmaf(p_, q4.w, fmaf(-s_, u4.w, fmaf(e_, y4.w, dk[x + 3])));
            }
        }
    }
    if (j0 + bj < n) {
        float *kp = dK + ((size_t)bh * n + j0 + bj) * D + bc;
        float *vp = dV + ((size_t)bh * n + j0 + bj) * D + bc;
#pragma unroll
        for (int x = 0; x < FPT; x += 4) {
            *reinterpret_cast<float4 *>(kp + x) = make_float4(dk[x], dk[x + 1], dk[x + 2], dk[x + 3]);
            *reinterpret_cast<float4 *>(vp + x) = make_float4(dv[x], dv[x + 1], dv[x + 2], dv[x + 3]);
        }
    }
}

template <int D, typename TI>
hipError_t launch_backward(const BackwardProblem &p)
{
    constexpr int REC = rec_floats<D>();
    float *rec = static_cast<float *>(p.ws);
    stage_mark(p.stream, "backward_rows");
    dim3 grid_rows((p.n + Cfg<D>::QB - 1) / Cfg<D>::QB * p.B * p.H);
    hipLaunchKernelGGL((bwd_rows_kernel<D, TI>), grid_rows, dim3(NT), 0, p.stream, (const TI *)p.Q, (const TI *)p.K,
                       (const TI *)p.V, (const TI *)p.dO, p.sq, p.sk, p.sv, p.sdo, p.H, p.B * p.H, p.n, p.lambda, p.lambda_rows,
                       p.scale, rec, p.dQ, p.dlambda);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    stage_mark(p.stream, "backward_keys");
    dim3 grid_keys((p.n + KeyCfg<D>::KB - 1) / KeyCfg<D>::KB * p.B * p.H);
    hipLaunchKernelGGL((bwd_keys_kernel<D, TI>), grid_keys, dim3(NT), 0, p.stream, (const TI *)p.Q, (const TI *)p.K,
                       (const TI *)p.V, (const TI *)p.dO, p.sq, p.sk, p.sv, p.sdo, p.H, p.B * p.H, p.n, p.scale, (const float *)rec,
                       (const float *)rec + D, REC, (const float *)rec + 2 * D, REC, p.dK, p.dV);
    return hipGetLastError();
}

template <int D>
hipError_t backward_by_dtype(const BackwardProblem &p)
{
    return p.in == LLLA_F32 ? launch_backward<D, float>(p) : launch_backward<D, bf16_t>(p);
}

template <int D, int MODE>
hipError_t launch_early_rows(const BackwardProblem &p, const BackwardLayout &L, int first)
{
    using TI = bf16_t;
    char *base = static_cast<char *>(p.ws);
    const float *M = reinterpret_cast<const float *>(base + L.fwd + L.m);
    const float *Y = reinterpret_cast<const float *>(base + L.fwd + L.y);
    const float *U = reinterpret_cast<const float *>(base + L.u);
    float *R = reinterpret_cast<float *>(base + L.r);
    float *Sc = reinterpret_cast<float *>(base + L.sc);
    dim3 grid((first + RowCfg<D>::QT - 1) / RowCfg<D>::QT, p.B * p.H);
    hipLaunchKernelGGL((bwd_rowsweep_kernel<D, TI, MODE>), grid, dim3(NT), 0, p.stream, (const TI *)p.Q, (const TI *)p.K,
                       (const TI *)p.V, (const TI *)p.dO, p.sq, p.sk, p.sv, p.sdo, p.H, p.n, first, p.scale, p.lambda,
                       p.lambda_rows, M, L.npad, MODE == 1 ? Y : nullptr, MODE == 1 ? U : nullptr, R, L.ypitch,
                       MODE == 1 ? Sc : nullptr, MODE == 1 ? p.dQ : nullptr, MODE == 1 ? p.dlambda : nullptr);
    return hipGetLastError();
}

// matrix-core flow (bf16, d = 64 / 128): row maxima, r sweep, moments with both solves, dQ sweep, key sweep
hipError_t launch_backward_mfma(const BackwardProblem &p)
{
    const BackwardLayout L = mfma_backward_layout(p.B, p.H, p.n, p.d);
    hipError_t err = mfma_backward_rowmax(p, L);
    if (err != hipSuccess) return err;
    // the first 2d rows: fp32 sweeps (see bwd_rowsweep_kernel); the matrix-core sweeps start after them
    const int first = p.n < 2 * p.d ? p.n : 2 * p.d;
    stage_mark(p.stream, "backward_r");
    err = p.d == 64 ? launch_early_rows<64, 0>(p, L, first) : launch_early_rows<128, 0>(p, L, first);
    if (err != hipSuccess) return err;
    if (first < p.n) err = mfma_backward_r(p, L, first);
    if (err != hipSuccess) return err;
    err = mfma_backward_solve(p, L);
    if (err != hipSuccess) return err;
    stage_mark(p.stream, "backward_dq");
    err = p.d == 64 ? launch_early_rows<64, 1>(p, L, first) : launch_early_rows<128, 1>(p, L, first);
    if (err != hipSuccess) return err;
    if (first < p.n) err = mfma_backward_dq(p, L, first);
    if (err != hipSuccess) return err;
    stage_mark(p.stream, "backward_keys");
    return mfma_backward_keys(p, L);
}

}  // namespace

size_t valu_backward_workspace_bytes(int B, int H, int n, int d)
{
    return round_up((size_t)B * H * n * (2 * (size_t)d + 8) * sizeof(float), 256);
}

hipError_t valu_backward(const BackwardProblem &p)
{
    switch (p.d) {
        case 16: return backward_by_dtype<16>(p);
        case 32: return backward_by_dtype<32>(p);
        case 64: return backward_by_dtype<64>(p);
        case 128: return backward_by_dtype<128>(p);
        default: return hipErrorInvalidValue;
    }
}

size_t backward_workspace_bytes(int B, int H, int n, int d, llla_dtype in, llla_path path)
{
    const size_t v = valu_backward_workspace_bytes(B, H, n, d);
    if (path == LLLA_PATH_VALU || !mfma_forward_supported(d, in, true)) return v;
    const size_t m = mfma_backward_layout(B, H, n, d).total;
    return path == LLLA_PATH_MFMA ? m : (m > v ? m : v);
}

hipError_t backward(const BackwardProblem &p, llla_path path)
{
    // the matrix-core sweeps put their 64-row blocks on grid.y (at most 65535 of them, i.e. n <= 4 194 240)
    const bool use_mfma = path != LLLA_PATH_VALU && mfma_forward_supported(p.d, p.in, true) && (p.n + 63) / 64 <= 65535;
    stage_begin(p.stream);
    hipError_t err;
    if (!use_mfma) err = valu_backward(p);
    else err = launch_backward_mfma(p);
    stage_end(p.stream);
    return err;
}

}  // namespace llla

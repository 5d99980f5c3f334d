// Matrix-core sweeps of the LLA backward pass (bf16 inputs, d = 64 / 128).  Key sweep: dK_j and dV_j of a block of keys,
// summed over the query rows at and after the block (Appendix D: Delta_V = S^T G and the key-side sums of the
// w- and z-paths, here in the un-centred form described at the top of llla_bwd.hip).
//
// A wave owns 16 keys and walks over the query rows in steps of 32.  Per step, with C = A B on 16x16x32 bf16 MFMA:
//   * four products of a [16 queries x d] row tile with the wave's key (or value) fragments give, in the accumulator
//     layout (lane (g, nn): queries 4g..4g+3, key nn), the logits q_i.k_j, the linear forms y1_i.k_j and u1_i.k_j
//     (y1, u1 as bf16 hi + lo) and gamma_ij = dO_i.v_j;
//   * the vector ALU turns them into the three coefficient tiles s_ij, e_ij, scale p^_ij and splits each into
//     bf16 hi + lo;
//   * those registers are already the A operand of the second product family, whose contraction index is the query
//     (slot 4s+r of lane group g <-> query 16s+4g+r): dV += S^T dO,  dK += E^T Y1 - S^T U1 + scale P^T Q.  The B operands
//     are the same row tiles read transposed by ds_read_tr16_b64 (lane nn gets four consecutive queries of feature
//     16J+nn), so no tile is stored twice.
// Accumulators stay in registers for the whole sweep; every output element is written once (no atomics).
#include "llla_mfma_common.hpp"

namespace llla {
namespace {

using namespace mfma;

typedef short short4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) short4v *lds_short4_ptr;
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int QS = 32;        // query rows per step

// transposed fragment of a natural [32 rows][pitch P halves] tile: for feature 16J + nn the rows 4g..4g+3 and
// 16+4g..16+4g+3 -- addr is the lane's own address (row 4g + nn/4, features 16J + 4(nn%4)..) in halves
__device__ inline bf16x8 tr_frag(const bf16_t *tile, int addr, int pitch)
{
    const short4v a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(tile + addr));
    const short4v b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(tile + 16 * pitch + addr));
    const uint2 au = __builtin_bit_cast(uint2, a), bu = __builtin_bit_cast(uint2, b);
    return __builtin_bit_cast(bf16x8, make_uint4(au.x, au.y, bu.x, bu.y));
}

__device__ inline void split_bf16(float x, __bf16 &hi, __bf16 &lo)
{
    hi = (__bf16)x;
    lo = (__bf16)(x - (float)hi);
}

template <int DD>
__global__ __launch_bounds__(256, DD == 64 ? 3 : 2) void bwd_keys_mfma_kernel(
    const bf16_t *__restrict__ Qg, const bf16_t *__restrict__ Kg, const bf16_t *__restrict__ Vg,
    const bf16_t *__restrict__ Gg, llla_strides sq, llla_strides sk, llla_strides sv, llla_strides sg, int H, int n,
    float scale, const float *__restrict__ Yg, const float *__restrict__ Ug, const float *__restrict__ Sc,
    float *__restrict__ dK, float *__restrict__ dV)
{
    using S = Shape<DD>;
    constexpr int NF = S::NF, NB = S::NB, YP = S::YP;
    // halves per row of an LDS tile: 32 B of padding, i.e. a row pitch of 40 (d = 64) or 72 (d = 128) banks, keeps the
    // transposing reads of a half-wave (8 rows x 8 banks) on distinct banks; with 16 B of padding they collided and
    // 42 % of the kernel's LDS cycles were bank conflicts
    constexpr int P = DD + 16;
    constexpr int CH = DD / 8;                           // 16-byte chunks per row
    __shared__ __align__(16) bf16_t qt[QS * P], gt[QS * P], yh[QS * P], yl[QS * P], uh[QS * P], ul[QS * P];
    __shared__ float rs[QS][9];                          // y0, u0, m, correction, argmax of the step's rows (odd pitch)

    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64, g = lane / 16, nn = lane % 16;
    // A low key block sees the most rows (up to n/32 steps), the last one two steps.  Workgroups are dispatched
    // with blockIdx.x running fastest, so the head is put there: all heads' longest blocks start first and the
    // shortest ones fill the tail, instead of the last head's longest block running alone at the end.
    const int bh = blockIdx.x, b = bh / H, h = bh % H;
    const int j0 = (int)blockIdx.y * 64;
    const int jk = j0 + 16 * wave + nn, jkc = min(jk, n - 1);
    const bf16_t *Qh = Qg + b * sq.batch + h * sq.head;
    const bf16_t *Gh = Gg + b * sg.batch + h * sg.head;
    const float *Yh = Yg + (size_t)bh * n * YP, *Uh = Ug + (size_t)bh * n * YP, *Sh = Sc + (size_t)bh * n * 8;

    bf16x8 kf[NF], vf[NF];
    {
        const bf16_t *krow = Kg + b * sk.batch + h * sk.head + (int64_t)jkc * sk.seq;
        const bf16_t *vrow = Vg + b * sv.batch + h * sv.head + (int64_t)jkc * sv.seq;
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            kf[f] = *reinterpret_cast<const bf16x8 *>(krow + 32 * f + 8 * g);
            vf[f] = *reinterpret_cast<const bf16x8 *>(vrow + 32 * f + 8 * g);
        }
    }
    f32x4 dv[NB], dk[NB];
#pragma unroll
    for (int J = 0; J < NB; ++J) dv[J] = dk[J] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int tr_addr = (4 * g + (nn >> 2)) * P + 4 * (nn & 3);      // + 16 J

    for (int it0 = j0; it0 < n; it0 += QS) {
        __syncthreads();                                 // the previous step's tiles are consumed
        for (int idx = tid; idx < QS * CH; idx += 256) {
            const int row = idx / CH, ch = (idx % CH) * 8, i = it0 + row;
            u32x4 qv = {0u, 0u, 0u, 0u}, gv = qv;
            f32x4 ya = {0.f, 0.f, 0.f, 0.f}, yb = ya, ua = ya, ub = ya;
            if (i < n) {
                qv = *reinterpret_cast<const u32x4 *>(Qh + (int64_t)i * sq.seq + ch);
                gv = *reinterpret_cast<const u32x4 *>(Gh + (int64_t)i * sg.seq + ch);
                ya = *reinterpret_cast<const f32x4 *>(Yh + (size_t)i * YP + ch);
                yb = *reinterpret_cast<const f32x4 *>(Yh + (size_t)i * YP + ch + 4);
                ua = *reinterpret_cast<const f32x4 *>(Uh + (size_t)i * YP + ch);
                ub = *reinterpret_cast<const f32x4 *>(Uh + (size_t)i * YP + ch + 4);
            }
            bf16x8 y_hi, y_lo, u_hi, u_lo;
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                __bf16 hi, lo;
                split_bf16(t < 4 ? ya[t & 3] : yb[t & 3], hi, lo);
                y_hi[t] = hi; y_lo[t] = lo;
                split_bf16(-(t < 4 ? ua[t & 3] : ub[t & 3]), hi, lo);      // the tiles hold -u1: both uses subtract it
                u_hi[t] = hi; u_lo[t] = lo;
            }
            *reinterpret_cast<u32x4 *>(&qt[row * P + ch]) = qv;
            *reinterpret_cast<u32x4 *>(&gt[row * P + ch]) = gv;
            *reinterpret_cast<bf16x8 *>(&yh[row * P + ch]) = y_hi;
            *reinterpret_cast<bf16x8 *>(&yl[row * P + ch]) = y_lo;
            *reinterpret_cast<bf16x8 *>(&uh[row * P + ch]) = u_hi;
            *reinterpret_cast<bf16x8 *>(&ul[row * P + ch]) = u_lo;
        }
        {
            const int row = tid / 8, c = tid % 8;
            rs[row][c] = (it0 + row < n && c < 5) ? Sh[(size_t)(it0 + row) * 8 + c] : 0.f;
        }
        __syncthreads();

        // ---- coefficients: lane (g, nn) holds the pairs (query it0 + 16s + 4g + r, key jk) --------------------
        bf16x8 s_hi, s_lo, e_hi, e_lo, p_hi, p_lo;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            f32x4 st = {0.f, 0.f, 0.f, 0.f}, at = st, bt = st, gm = st;
            const int arow = (16 * s + nn) * P + 8 * g;
#pragma unroll
            for (int f = 0; f < NF; ++f) {
                const bf16x8 qf = *reinterpret_cast<const bf16x8 *>(&qt[arow + 32 * f]);
                const bf16x8 gf = *reinterpret_cast<const bf16x8 *>(&gt[arow + 32 * f]);
                const bf16x8 yhf = *reinterpret_cast<const bf16x8 *>(&yh[arow + 32 * f]);
                const bf16x8 ylf = *reinterpret_cast<const bf16x8 *>(&yl[arow + 32 * f]);
                const bf16x8 uhf = *reinterpret_cast<const bf16x8 *>(&uh[arow + 32 * f]);
                const bf16x8 ulf = *reinterpret_cast<const bf16x8 *>(&ul[arow + 32 * f]);
                st = mfma_bf16(qf, kf[f], st);
                gm = mfma_bf16(gf, vf[f], gm);
                at = mfma_bf16(ylf, kf[f], at);
                at = mfma_bf16(yhf, kf[f], at);
                bt = mfma_bf16(ulf, kf[f], bt);
                bt = mfma_bf16(uhf, kf[f], bt);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int qr = 16 * s + 4 * g + r, i = it0 + qr;
                const float y0 = rs[qr][0], u0 = rs[qr][1], m = rs[qr][2], corr = rs[qr][3];
                const int jstar = __float_as_int(rs[qr][4]);
                const bool valid = (jk <= i) && (i < n);
                const float w = __builtin_amdgcn_exp2f((scale * st[r] - m) * LOG2E);
                const float a = y0 + at[r];
                const float ev = w * (gm[r] - u0 + bt[r]);       // bt = -u1.k
                float pv = a * ev;
                pv = (jk == jstar) ? pv + corr : pv;
                __bf16 hi, lo;
                split_bf16(valid ? w * a : 0.f, hi, lo);
                s_hi[4 * s + r] = hi; s_lo[4 * s + r] = lo;
                split_bf16(valid ? ev : 0.f, hi, lo);
                e_hi[4 * s + r] = hi; e_lo[4 * s + r] = lo;
                split_bf16(valid ? scale * pv : 0.f, hi, lo);
                p_hi[4 * s + r] = hi; p_lo[4 * s + r] = lo;
            }
        }

        // ---- accumulate over the step's 32 queries --------------------------------------------------------------
#pragma unroll
        for (int J = 0; J < NB; ++J) {
            const int ta = tr_addr + 16 * J;
            const bf16x8 gT = tr_frag(gt, ta, P);
            dv[J] = mfma_bf16(s_lo, gT, dv[J]);
            dv[J] = mfma_bf16(s_hi, gT, dv[J]);
            const bf16x8 yhT = tr_frag(yh, ta, P), ylT = tr_frag(yl, ta, P);
            dk[J] = mfma_bf16(e_lo, yhT, dk[J]);
            dk[J] = mfma_bf16(e_hi, ylT, dk[J]);
            dk[J] = mfma_bf16(e_hi, yhT, dk[J]);
            const bf16x8 uhT = tr_frag(uh, ta, P), ulT = tr_frag(ul, ta, P);
            dk[J] = mfma_bf16(s_lo, uhT, dk[J]);
            dk[J] = mfma_bf16(s_hi, ulT, dk[J]);
            dk[J] = mfma_bf16(s_hi, uhT, dk[J]);
            const bf16x8 qT = tr_frag(qt, ta, P);
            dk[J] = mfma_bf16(p_lo, qT, dk[J]);
            dk[J] = mfma_bf16(p_hi, qT, dk[J]);
        }
    }

    // dv[J], dk[J]: lane (g, nn) reg r = gradient of key j0 + 16 wave + 4g + r, feature 16J + nn
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int key = j0 + 16 * wave + 4 * g + r;
        if (key < n) {
            const size_t off = ((size_t)bh * n + key) * DD + nn;
#pragma unroll
            for (int J = 0; J < NB; ++J) {
                dK[off + 16 * J] = dk[J][r];
                dV[off + 16 * J] = dv[J][r];
            }
        }
    }
}


// ---- row sweeps ---------------------------------------------------------------------------------------------
// The mirror image of the key sweep: a wave owns 16 query rows (their fragments stay in registers) and walks over
// the keys in steps of 32; the coefficient tiles come out as [key][query] (lane (g, nn): keys 4g..4g+3, query nn),
// which is the A operand of a product that contracts over keys, with the K tile read transposed as B.
//   MODE 0 (before the solve): c_ij = w_ij gamma_ij;  r1_i = sum_j c_ij k_j, r0_i = sum_j c_ij, and the first key that
//                              attains the row maximum (the logits are produced exactly as in the row-maximum sweep);
//   MODE 1 (after it):         dL/dlambda_i = -u1_i.y1_i, c_ij = p^_ij;  dQ_i = u1_i + scale sum_j c_ij k_j, and the row
//                              scalars (y0, u0, m, correction, argmax) the key sweep reads.
// Rows [first_row, n) only: the first rows of a sequence take fp32 sweeps (their coefficients cancel too strongly for
// a 16-bit split).
template <int DD, int MODE>
__global__ __launch_bounds__(256, 2) void bwd_rows_mfma_kernel(
    const bf16_t *__restrict__ Qg, const bf16_t *__restrict__ Kg, const bf16_t *__restrict__ Vg,
    const bf16_t *__restrict__ Gg, llla_strides sq, llla_strides sk, llla_strides sv, llla_strides sg, int H, int n,
    int first_row, int mpitch, float scale, float lambda, const float *__restrict__ LamRows, const float *__restrict__ Mg,
    const float *__restrict__ Yg, const float *__restrict__ Ug, float *__restrict__ Rv, float *__restrict__ Sc,
    float *__restrict__ dQ, float *__restrict__ dLam)
{
    using S = Shape<DD>;
    constexpr int NF = S::NF, NB = S::NB, YP = S::YP;
    constexpr int P = DD + 16, CH = DD / 8;          // row pitch as in the key sweep
    __shared__ __align__(16) bf16_t kt[KB * P], vt[KB * P];

    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64, g = lane / 16, nn = lane % 16;
    // head on blockIdx.x (dispatched fastest), row block on y, longest rows first: see bwd_keys_mfma_kernel
    const int bh = blockIdx.x, b = bh / H, h = bh % H;
    const int i0 = first_row + ((int)gridDim.y - 1 - (int)blockIdx.y) * 64;
    const int iq = i0 + 16 * wave + nn, iqc = min(iq, n - 1);
    const size_t row = (size_t)bh * n + iqc;
    const bf16_t *Kh = Kg + b * sk.batch + h * sk.head;
    const bf16_t *Vh = Vg + b * sv.batch + h * sv.head;
    const float cscale = scale * LOG2E;

    bf16x8 qf[NF], gf[NF], yhf[NF], ylf[NF], uhf[NF], ulf[NF];
    {
        const bf16_t *qrow = Qg + b * sq.batch + h * sq.head + (int64_t)iqc * sq.seq;
        const bf16_t *grow = Gg + b * sg.batch + h * sg.head + (int64_t)iqc * sg.seq;
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            qf[f] = *reinterpret_cast<const bf16x8 *>(qrow + 32 * f + 8 * g);
            gf[f] = *reinterpret_cast<const bf16x8 *>(grow + 32 * f + 8 * g);
        }
    }
    const float mrow = Mg[(size_t)bh * mpitch + iqc];                     // log2 units
    float y0 = 0.f, u0 = 0.f, corr = 0.f;
    int jstar = 0;
    if (MODE == 1) {
        const float *yr = Yg + row * YP, *ur = Ug + row * YP;
        y0 = yr[DD];
        u0 = ur[DD];
        jstar = __float_as_int(Rv[row * YP + DD + 1]);
        float dl = 0.f;
#pragma unroll
        for (int f = 0; f < NF; ++f)
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const float yv = yr[32 * f + 8 * g + t], uv = ur[32 * f + 8 * g + t];
                dl = fmaf(-uv, yv, dl);
                __bf16 hi, lo;
                split_bf16(yv, hi, lo);
                yhf[f][t] = hi; ylf[f][t] = lo;
                split_bf16(uv, hi, lo);
                uhf[f][t] = hi; ulf[f][t] = lo;
            }
        dl += __shfl_xor(dl, 16);
        dl += __shfl_xor(dl, 32);
        corr = (LamRows ? LamRows[row] : lambda) * dl;
        if (g == 0 && iq < n) {
            float *sc = Sc + row * 8;
            sc[0] = y0; sc[1] = u0; sc[2] = mrow * 0.6931471805599453f; sc[3] = corr; sc[4] = __int_as_float(jstar);
            if (dLam) dLam[row] = dl;
        }
    }
    f32x4 acc[NB];
#pragma unroll
    for (int J = 0; J < NB; ++J) acc[J] = f32x4{0.f, 0.f, 0.f, 0.f};
    float csum = 0.f, best = -INFINITY;
    int arg = 0;
    const int tr_addr = (4 * g + (nn >> 2)) * P + 4 * (nn & 3);

    const int nblk = min(i0 + 63, n - 1) / KB + 1;
    // the next key tile travels from global memory into registers while the current one is consumed
    constexpr int NIT = KB * CH / 256;
    u32x4 pk[NIT], pv[NIT];
    auto fetch = [&](int c) {
#pragma unroll
        for (int k = 0; k < NIT; ++k) {
            const int idx = tid + 256 * k, key = idx / CH, ch = (idx % CH) * 8, j = c * KB + key;
            pk[k] = pv[k] = u32x4{0u, 0u, 0u, 0u};
            if (j < n) {
                pk[k] = *reinterpret_cast<const u32x4 *>(Kh + (int64_t)j * sk.seq + ch);
                pv[k] = *reinterpret_cast<const u32x4 *>(Vh + (int64_t)j * sv.seq + ch);
            }
        }
    };
    fetch(0);
    for (int c = 0; c < nblk; ++c) {
        __syncthreads();
#pragma unroll
        for (int k = 0; k < NIT; ++k) {
            const int idx = tid + 256 * k, key = idx / CH, ch = (idx % CH) * 8;
            *reinterpret_cast<u32x4 *>(&kt[key * P + ch]) = pk[k];
            *reinterpret_cast<u32x4 *>(&vt[key * P + ch]) = pv[k];
        }
        __syncthreads();
        if (c + 1 < nblk) fetch(c + 1);
        bf16x8 c_hi, c_lo;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            f32x4 st = {0.f, 0.f, 0.f, 0.f}, gm = st, at = st, bt = st;
            const int arow = (16 * s + nn) * P + 8 * g;
#pragma unroll
            for (int f = 0; f < NF; ++f) {
                const bf16x8 kfr = *reinterpret_cast<const bf16x8 *>(&kt[arow + 32 * f]);
                const bf16x8 vfr = *reinterpret_cast<const bf16x8 *>(&vt[arow + 32 * f]);
                st = mfma_bf16(kfr, qf[f], st);
                gm = mfma_bf16(vfr, gf[f], gm);
                if (MODE == 1) {
                    at = mfma_bf16(kfr, ylf[f], at);
                    at = mfma_bf16(kfr, yhf[f], at);
                    bt = mfma_bf16(kfr, ulf[f], bt);
                    bt = mfma_bf16(kfr, uhf[f], bt);
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int j = c * KB + 16 * s + 4 * g + r;
                const bool valid = (j <= iq) && (iq < n);
                const float lg = st[r] * cscale;
                const float w = __builtin_amdgcn_exp2f(lg - mrow);
                float cv;
                if (MODE == 0) {
                    if (valid && lg > best) {
                        best = lg;
                        arg = j;
                    }
                    cv = valid ? w * gm[r] : 0.f;
                    csum += cv;
                } else {
                    cv = w * (y0 + at[r]) * (gm[r] - u0 - bt[r]);
                    cv = (j == jstar) ? cv + corr : cv;
                    cv = valid ? cv : 0.f;
                }
                __bf16 hi, lo;
                split_bf16(cv, hi, lo);
                c_hi[4 * s + r] = hi;
                c_lo[4 * s + r] = lo;
            }
        }
#pragma unroll
        for (int J = 0; J < NB; ++J) {
            const bf16x8 kT = tr_frag(kt, tr_addr + 16 * J, P);
            acc[J] = mfma_bf16(c_lo, kT, acc[J]);
            acc[J] = mfma_bf16(c_hi, kT, acc[J]);
        }
    }

    if (MODE == 0) {
        // lanes (g, nn), g = 0..3, hold query nn's partial sums and maxima over disjoint keys
        csum += __shfl_xor(csum, 16);
        csum += __shfl_xor(csum, 32);
#pragma unroll
        for (int sft = 16; sft <= 32; sft <<= 1) {
            const float ob = __shfl_xor(best, sft);
            const int oa = __shfl_xor(arg, sft);
            const bool take = (ob > best) || (ob == best && oa < arg);
            best = take ? ob : best;
            arg = take ? oa : arg;
        }
        if (g == 0 && iq < n) {
            Rv[row * YP + DD] = csum;
            Rv[row * YP + DD + 1] = __int_as_float(arg);
        }
    }
    // acc[J]: lane (g, nn) reg r = sum for query i0 + 16 wave + 4g + r, feature 16J + nn
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int i = i0 + 16 * wave + 4 * g + r;
        if (i < n) {
            const size_t ro = (size_t)bh * n + i;
#pragma unroll
            for (int J = 0; J < NB; ++J) {
                if (MODE == 0) Rv[ro * YP + 16 * J + nn] = acc[J][r];
                else dQ[ro * DD + 16 * J + nn] = fmaf(scale, acc[J][r], Ug[ro * YP + 16 * J + nn]);
            }
        }
    }
}

template <int DD, int MODE>
hipError_t launch_rows(const BackwardProblem &p, const BackwardLayout &L, int first_row)
{
    char *base = static_cast<char *>(p.ws);
    const float *M = reinterpret_cast<const float *>(base + L.fwd + L.m);
    const float *Y = reinterpret_cast<const float *>(base + L.fwd + L.y);
    const float *U = reinterpret_cast<const float *>(base + L.u);
    float *R = reinterpret_cast<float *>(base + L.r);
    float *Sc = reinterpret_cast<float *>(base + L.sc);
    hipLaunchKernelGGL((bwd_rows_mfma_kernel<DD, MODE>), dim3(p.B * p.H, (p.n - first_row + 63) / 64), dim3(256), 0, p.stream,
                       static_cast<const bf16_t *>(p.Q), static_cast<const bf16_t *>(p.K), static_cast<const bf16_t *>(p.V),
                       static_cast<const bf16_t *>(p.dO), p.sq, p.sk, p.sv, p.sdo, p.H, p.n, first_row, L.npad, p.scale,
                       p.lambda, p.lambda_rows, M, Y, U, R, Sc, p.dQ, p.dlambda);
    return hipGetLastError();
}

}  // namespace

// rows [first_row, n); first_row must be a multiple of 64
hipError_t mfma_backward_r(const BackwardProblem &p, const BackwardLayout &L, int first_row)
{
    return p.d == 64 ? launch_rows<64, 0>(p, L, first_row) : launch_rows<128, 0>(p, L, first_row);
}

hipError_t mfma_backward_dq(const BackwardProblem &p, const BackwardLayout &L, int first_row)
{
    return p.d == 64 ? launch_rows<64, 1>(p, L, first_row) : launch_rows<128, 1>(p, L, first_row);
}

hipError_t mfma_backward_keys(const BackwardProblem &p, const BackwardLayout &L)
{
    char *base = static_cast<char *>(p.ws);
    const float *Y = reinterpret_cast<const float *>(base + L.fwd + L.y);
    const float *U = reinterpret_cast<const float *>(base + L.u);
    const float *Sc = reinterpret_cast<const float *>(base + L.sc);
    const bf16_t *Q = static_cast<const bf16_t *>(p.Q), *K = static_cast<const bf16_t *>(p.K),
                 *V = static_cast<const bf16_t *>(p.V), *G = static_cast<const bf16_t *>(p.dO);
    dim3 grid(p.B * p.H, (p.n + 63) / 64);
    if (p.d == 64)
        hipLaunchKernelGGL((bwd_keys_mfma_kernel<64>), grid, dim3(256), 0, p.stream, Q, K, V, G, p.sq, p.sk, p.sv, p.sdo,
                           p.H, p.n, p.scale, Y, U, Sc, p.dK, p.dV);
    else
        hipLaunchKernelGGL((bwd_keys_mfma_kernel<128>), grid, dim3(256), 0, p.stream, Q, K, V, G, p.sq, p.sk, p.sv, p.sdo,
                           p.H, p.n, p.scale, Y, U, Sc, p.dK, p.dV);
    return hipGetLastError();
}

}  // namespace llla

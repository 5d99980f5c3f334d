// Portable vector-ALU path of Local Linear Attention for gfx950: every d in {16,32,64,128},
// fp32 or bf16 inputs (bf16 is widened exactly), all arithmetic in fp32.
//
// One 256-thread workgroup serves QB "slots".  In the forward kernel a slot is one query row and
// all slots sweep the same key tiles; in the decode kernel all slots serve the single query of a
// (batch, head) and split the cache between them, their partial moments being merged with a
// max-rescale before the solve.  Per slot the kernel follows the three sweeps of Algorithm 1
// (Section 3.2) with two changes of substance:
//   (1) the per-query statistics are the un-centred moments of Eq. (tilded_form) extended by the
//       intercept column, i.e. the (d+1)x(d+1) matrix At = sum_j w_j [1;k_j][1;k_j]^T
//       + lambda diag(0, I); it lives in registers (one TSxTS tile per thread) and in LDS, never
//       in device memory;
//   (2) the system is solved exactly by elimination in LDS (y = At^{-1} [1; q]) instead of by
//       conjugate gradients; the output weights of Eq. (lla) are then s_ij = w_ij (y0 + k_j . y1)
//       (y1 = -rho/delta, y0 = (1 + q . rho)/delta in the paper's symbols), so the third sweep is
//       the relmm-style product K y1 followed by S V.
// The running row maximum and the rescaling of the moments across key tiles are those of
// Algorithm 1 (lines computing m, alpha and the updates of omega and M).
#include "llla_valu_common.hpp"

namespace llla {
namespace {

using namespace valu;

// Kernel.  DECODE = false: grid.x = ceil(n/QB) query blocks (heaviest first) x B*H, the (batch, head) index fastest.
//          DECODE = true : grid.x = B*H; all slots share the query and split the keys.
//          GIVEN  = true : (forward only) the per-row solution y and row maximum are read from
//                          device memory (written by the MFMA moments kernel); only sweep 3 runs.
template <int D, typename TI, typename TO, bool DECODE, bool GIVEN = false>
__global__ __launch_bounds__(NT) void valu_kernel(const TI *__restrict__ Qg, const TI *__restrict__ Kg,
                                                  const TI *__restrict__ Vg, TO *__restrict__ Og,
                                                  llla_strides sq, llla_strides sk, llla_strides sv,
                                                  llla_strides so, const int32_t *__restrict__ seqlens,
                                                  int H, int nbh, int n, int causal, float lambda, float scale,
                                                  const float *__restrict__ Mg = nullptr, int mpitch = 0,
                                                  const float *__restrict__ Yg = nullptr, int ypitch = 0,
                                                  const float *__restrict__ LamRows = nullptr,
                                                  float *__restrict__ Rho = nullptr, float *__restrict__ Delta = nullptr)
{
    using C = Cfg<D>;
    constexpr int TS = C::TS, TG = C::TG, TPQ = C::TPQ, QB = C::QB, LDK = C::LDK, P = C::P,
                  LS = C::LDS_SYS;
    constexpr int KROWS = DECODE ? QB * KT : KT;         // key rows staged per tile
    constexpr int NSYS = DECODE ? 1 : QB;
    constexpr int TILE_F = 2 * KROWS * LDK + 2 * QB * KT;   // ks, vs, logits, weights
    constexpr int SYS_F = NSYS * P * LS;
    constexpr int UNION_F = (TILE_F > SYS_F) ? TILE_F : SYS_F;

    __shared__ __align__(16) float smem[UNION_F + QB * D + QB * (P + 3) + 4 * QB];
    float *ks = smem;                                     // [KROWS][LDK]
    float *vs = ks + KROWS * LDK;                         // [KROWS][LDK]
    float *sl = vs + KROWS * LDK;                         // [QB][KT] logits, later coefficients
    float *wl = sl + QB * KT;                             // [QB][KT] weights
    float *sys = smem;                                    // [NSYS][P][LS], aliases the tiles
    float *qs = smem + UNION_F;                           // [QB][D]
    float *ys = qs + QB * D;                              // [QB][P+3]  solution y = At^{-1}[1;q]
    float *ms = ys + QB * (P + 3);                        // [QB] running max
    float *al = ms + QB;                                  // [QB] rescale factor of this tile
    float *fs = al + QB;                                  // [QB] decode merge factors
    float *red = fs + QB;                                 // [QB] spare

    const int tid = threadIdx.x;
    const int slot = tid / TPQ;
    const int r = tid % TPQ;
    const int ta = r / TG, tb = r % TG;
    // one-dimensional grid, (batch, head) index fastest: blocks are dispatched in that order, so the longest query
    // blocks of every head start first and the short ones fill the tail
    const int bh = (int)(blockIdx.x % (unsigned)nbh);
    const int b = bh / H, h = bh % H;

    const TI *Kh = Kg + b * sk.batch + h * sk.head;
    const TI *Vh = Vg + b * sv.batch + h * sv.head;

    int nkeys;          // keys that exist for this head
    int i0 = 0;         // first query row of the block (forward)
    if (DECODE) {
        nkeys = seqlens ? seqlens[b] : n;
        nkeys = nkeys < 1 ? 1 : (nkeys > n ? n : nkeys);
    } else {
        nkeys = n;
        const int nqb = (int)(gridDim.x / (unsigned)nbh);
        i0 = (nqb - 1 - (int)(blockIdx.x / (unsigned)nbh)) * QB;          // long rows are scheduled first
    }
    const int my_i = DECODE ? nkeys - 1 : i0 + slot;    // query row of this slot
    const bool slot_live = DECODE ? true : (my_i < n);
    // last key (exclusive) any slot of the block can see
    const int kend = DECODE ? nkeys : (causal ? min(n, i0 + QB) : n);
    const int my_last = (DECODE || !causal) ? nkeys - 1 : min(my_i, n - 1);   // last visible key
    // ridge of this slot's row (Appendix C: lambda may differ from position to position)
    const float lam_slot = (!DECODE && LamRows) ? LamRows[(size_t)bh * n + min(my_i, n - 1)] : lambda;

    // ---- query rows -> LDS ----------------------------------------------------------------------
    for (int idx = tid; idx < QB * D; idx += NT) {
        const int s = idx / D, c = idx % D;
        float v = 0.f;
        if (DECODE) {
            const TI *qp = Qg + (int64_t)bh * D;
            v = sizeof(TI) == 2 ? bf16_to_f32(((const bf16_t *)qp)[c]) : ((const float *)qp)[c];
        } else if (i0 + s < n) {
            const TI *qp = Qg + b * sq.batch + h * sq.head + (int64_t)(i0 + s) * sq.seq;
            v = sizeof(TI) == 2 ? bf16_to_f32(((const bf16_t *)qp)[c]) : ((const float *)qp)[c];
        }
        qs[idx] = v;
    }
    if (tid < QB) ms[tid] = -INFINITY;

    const int koff = DECODE ? slot * KT : 0;             // this slot's rows inside the staged tile
    if (GIVEN) {
        // y1 at [0, D), y0 at [D] of a row of Yg; the row maximum is stored in log2 units
        for (int idx = tid; idx < QB * P; idx += NT) {
            const int s2 = idx / P, c = idx % P;
            const int i = min(i0 + s2, n - 1);
            const float *yr = Yg + ((size_t)bh * n + i) * ypitch;
            ys[s2 * (P + 3) + c] = (c == 0) ? yr[D] : yr[c - 1];
        }
        if (tid < QB) ms[tid] = Mg[(size_t)bh * mpitch + min(i0 + tid, n - 1)] * 0.6931471805599453f;
        __syncthreads();
    } else {
        // ---- sweep 1: un-centred moments with running max (Algorithm 1, first loop) -----------------
        float acc[TS][TS];
        float mu[TS];
        float omega = 0.f;
#pragma unroll
        for (int x = 0; x < TS; ++x) {
            mu[x] = 0.f;
#pragma unroll
            for (int y = 0; y < TS; ++y) acc[x][y] = 0.f;
        }

        for (int kt0 = 0; kt0 < kend; kt0 += KROWS) {
            __syncthreads();                                 // previous tile fully consumed
            load_tile<D, TI>(ks, Kh, sk.seq, kt0, KROWS, nkeys, tid);
            __syncthreads();
            for (int idx = tid; idx < QB * KT; idx += NT) {  // logits of (slot, key)
                const int s = idx / KT, kj = idx % KT;
                const int row = (DECODE ? s * KT : 0) + kj;
                const int j = kt0 + row;
                const int last = (DECODE || !causal) ? nkeys - 1 : min(i0 + s, n - 1);
                float v = -INFINITY;
                if (j <= last) v = scale * dot_lds<D>(qs + s * D, ks + row * LDK);
                sl[idx] = v;
            }
            __syncthreads();
            if (tid < QB) {                                  // running max and rescale factor per slot
                float mx = ms[tid];
                const float mold = mx;
                for (int kj = 0; kj < KT; ++kj) mx = fmaxf(mx, sl[tid * KT + kj]);
                ms[tid] = mx;
                al[tid] = (mold == -INFINITY) ? 0.f : __expf(mold - mx);
            }
            __syncthreads();
            for (int idx = tid; idx < QB * KT; idx += NT) {  // weights, 0 for masked keys
                const float mx = ms[idx / KT];
                const float s = sl[idx];
                wl[idx] = (s == -INFINITY) ? 0.f : __expf(s - mx);
            }
            __syncthreads();
            {
                const float alpha = al[slot];
                if (alpha != 1.f) {
                    omega *= alpha;
#pragma unroll
                    for (int x = 0; x < TS; ++x) {
                        mu[x] *= alpha;
#pragma unroll
                        for (int y = 0; y < TS; ++y) acc[x][y] *= alpha;
                    }
                }
                const int jn = min(KT, my_last - (kt0 + koff) + 1);   // visible keys of this slot here
                for (int kj = 0; kj < jn; ++kj) {
                    const float w = wl[slot * KT + kj];
                    const float *krow = ks + (koff + kj) * LDK;
                    float a[TS], bb[TS];
#pragma unroll
                    for (int x = 0; x < TS; x += 4) {
                        const float4 va = *reinterpret_cast<const float4 *>(krow + ta * TS + x);
                        const float4 vb = *reinterpret_cast<const float4 *>(krow + tb * TS + x);
                        a[x] = va.x * w; a[x + 1] = va.y * w; a[x + 2] = va.z * w; a[x + 3] = va.w * w;
                        bb[x] = vb.x; bb[x + 1] = vb.y; bb[x + 2] = vb.z; bb[x + 3] = vb.w;
                    }
                    omega += w;
#pragma unroll
                    for (int x = 0; x < TS; ++x) {
                        mu[x] += a[x];
#pragma unroll
                        for (int y = 0; y < TS; ++y) acc[x][y] = fmaf(a[x], bb[y], acc[x][y]);
                    }
                }
            }
        }
        __syncthreads();                                     // tiles are dead; sys may overwrite them

        // ---- the (d+1)x(d+1) system [At | rhs] in LDS -----------------------------------------------
        if (DECODE) {
            // merge the slots' partial moments: common max, then an ordered (deterministic) sum
            if (tid < QB) {
                float mx = -INFINITY;
                for (int s = 0; s < QB; ++s) mx = fmaxf(mx, ms[s]);
                fs[tid] = (ms[tid] == -INFINITY) ? 0.f : __expf(ms[tid] - mx);
                red[tid] = mx;
            }
            for (int idx = tid; idx < P * LS; idx += NT) sys[idx] = 0.f;
            __syncthreads();
            for (int s = 0; s < QB; ++s) {
                if (slot == s) {
                    const float f = fs[s];
#pragma unroll
                    for (int x = 0; x < TS; ++x)
#pragma unroll
                        for (int y = 0; y < TS; ++y)
                            sys[(1 + ta * TS + x) * LS + 1 + tb * TS + y] += f * acc[x][y];
                    if (tb == 0) {
#pragma unroll
                        for (int x = 0; x < TS; ++x) sys[(1 + ta * TS + x) * LS] += f * mu[x];
                    }
                    if (r == 0) sys[0] += f * omega;
                }
                __syncthreads();
            }
            if (tid < QB) ms[tid] = red[tid];                // every slot now works relative to the max
            for (int c = tid; c < D; c += NT) {
                sys[c + 1] = sys[(c + 1) * LS];              // row 0 mirrors column 0
                sys[(c + 1) * LS + c + 1] += lambda;
                sys[(c + 1) * LS + P] = qs[c];
            }
            if (tid == 0) sys[P] = 1.f;
        } else {
            float *S = sys + slot * P * LS;
#pragma unroll
            for (int x = 0; x < TS; ++x)
#pragma unroll
                for (int y = 0; y < TS; ++y) {
                    const int rr = ta * TS + x, cc = tb * TS + y;
                    S[(1 + rr) * LS + 1 + cc] = acc[x][y] + (rr == cc ? lam_slot : 0.f);
                }
            if (tb == 0) {
#pragma unroll
                for (int x = 0; x < TS; ++x) {
                    S[(1 + ta * TS + x) * LS] = mu[x];
                    S[1 + ta * TS + x] = mu[x];
                }
            }
            if (r == 0) {
                // a dead slot (row >= n) gets a harmless identity-like pivot
                S[0] = slot_live ? omega : 1.f;
                S[P] = 1.f;
            }
            for (int c = r; c < D; c += TPQ) S[(c + 1) * LS + P] = qs[slot * D + c];
        }

        // ---- exact solve by elimination (the matrix is symmetric positive definite) -----------------
        {
            float *S = DECODE ? sys : sys + slot * P * LS;
            const int gt = DECODE ? tid : r;
            constexpr int GS = DECODE ? NT : TPQ;
            for (int k = 0; k < P; ++k) {
                __syncthreads();
                const float pinv = 1.f / S[k * LS + k];
                for (int row = k + 1 + gt; row < P; row += GS) {
                    const float f = S[row * LS + k] * pinv;
                    for (int c = k + 1; c <= P; ++c) S[row * LS + c] = fmaf(-f, S[k * LS + c], S[row * LS + c]);
                }
            }
            float *yv = ys + (DECODE ? 0 : slot * (P + 3));
            for (int k = P - 1; k >= 0; --k) {
                __syncthreads();
                const float yk = S[k * LS + P] / S[k * LS + k];
                if (gt == 0) yv[k] = yk;
                for (int row = gt; row < k; row += GS) S[row * LS + P] = fmaf(-S[row * LS + k], yk, S[row * LS + P]);
            }
        }
        __syncthreads();

        // ---- optional statistics of Eq. (lla): with y1 = -rho/delta and y0 = (1 + q.rho)/delta,
        //      1/delta = y0 + q.y1 and rho = -delta y1 ---------------------------------------------------
        if (!DECODE && (Rho != nullptr || Delta != nullptr) && slot_live) {
            const float *ysl = ys + slot * (P + 3);
            float qy = 0.f;
            for (int c = 0; c < D; ++c) qy = fmaf(qs[slot * D + c], ysl[1 + c], qy);
            const float dl = 1.f / (ysl[0] + qy);
            const size_t row = (size_t)bh * n + my_i;
            if (Delta != nullptr && r == 0) Delta[row] = dl;
            if (Rho != nullptr)
                for (int c = r; c < D; c += TPQ) Rho[row * D + c] = -dl * ysl[1 + c];
        }
    }   // !GIVEN

    // ---- sweep 3: output weights s_ij = w_ij (y0 + k_j . y1) and O = S V ------------------------
    const float *yv = ys + (DECODE ? 0 : slot * (P + 3));
    float o = 0.f;
    for (int kt0 = 0; kt0 < kend; kt0 += KROWS) {
        __syncthreads();
        load_tile<D, TI>(ks, Kh, sk.seq, kt0, KROWS, nkeys, tid);
        load_tile<D, TI>(vs, Vh, sv.seq, kt0, KROWS, nkeys, tid);
        __syncthreads();
        for (int idx = tid; idx < QB * KT; idx += NT) {
            const int s = idx / KT, kj = idx % KT;
            const int row = (DECODE ? s * KT : 0) + kj;
            const int j = kt0 + row;
            const int last = (DECODE || !causal) ? nkeys - 1 : min(i0 + s, n - 1);
            float cval = 0.f;
            if (j <= last) {
                const float *ysl = ys + (DECODE ? 0 : s * (P + 3));
                const float lg = scale * dot_lds<D>(qs + s * D, ks + row * LDK);
                // y1 starts at ysl[1]; copy-free unaligned dot
                float u = 0.f;
                for (int c = 0; c < D; ++c) u = fmaf(ysl[1 + c], ks[row * LDK + c], u);
                cval = __expf(lg - ms[s]) * (ysl[0] + u);
            }
            sl[idx] = cval;
        }
        __syncthreads();
        if (r < D) {
            const int jn = min(KT, my_last - (kt0 + koff) + 1);
            for (int kj = 0; kj < jn; ++kj) o = fmaf(sl[slot * KT + kj], vs[(koff + kj) * LDK + r], o);
        }
    }
    (void)yv;

    if (DECODE) {
        __syncthreads();
        float *osum = sys;                               // [D], tiles are dead again
        for (int c = tid; c < D; c += NT) osum[c] = 0.f;
        __syncthreads();
        for (int s = 0; s < QB; ++s) {
            if (slot == s && r < D) osum[r] += o;
            __syncthreads();
        }
        for (int c = tid; c < D; c += NT) Io<TO>::store1(Og + (int64_t)bh * D + c, osum[c]);
    } else if (slot_live && r < D) {
        TO *op = Og + b * so.batch + h * so.head + (int64_t)my_i * so.seq;
        Io<TO>::store1(op + r, o);
    }
}

// nrows: the forward kernel serves query rows [0, nrows) only (nrows = n for a full forward)
template <int D, typename TI, typename TO, bool DECODE>
hipError_t launch(const Problem &p, int nrows)
{
    using C = Cfg<D>;
    dim3 grid((DECODE ? 1 : (nrows + C::QB - 1) / C::QB) * p.B * p.H);
    hipLaunchKernelGGL((valu_kernel<D, TI, TO, DECODE>), grid, dim3(NT), 0, p.stream,
                       (const TI *)p.Q, (const TI *)p.K, (const TI *)p.V, (TO *)p.O, p.sq, p.sk, p.sv,
                       p.so, p.seqlens, p.H, p.B * p.H, p.n, p.causal, p.lambda, p.scale, (const float *)nullptr, 0,
                       (const float *)nullptr, 0, DECODE ? nullptr : p.lambda_rows, DECODE ? nullptr : p.rho,
                       DECODE ? nullptr : p.delta);
    return hipGetLastError();
}

template <int D, bool DECODE>
hipError_t by_dtype(const Problem &p, int nrows)
{
    if (p.in == LLLA_F32)
        return p.out == LLLA_F32 ? launch<D, float, float, DECODE>(p, nrows) : launch<D, float, bf16_t, DECODE>(p, nrows);
    return p.out == LLLA_F32 ? launch<D, bf16_t, float, DECODE>(p, nrows) : launch<D, bf16_t, bf16_t, DECODE>(p, nrows);
}

template <bool DECODE>
hipError_t by_dim(const Problem &p, int nrows)
{
    switch (p.d) {
        case 16: return by_dtype<16, DECODE>(p, nrows);
        case 32: return by_dtype<32, DECODE>(p, nrows);
        case 64: return by_dtype<64, DECODE>(p, nrows);
        case 128: return by_dtype<128, DECODE>(p, nrows);
        default: return hipErrorInvalidValue;
    }
}

template <int D, typename TI>
hipError_t launch_given(const Problem &p, int nrows, const float *M, int mpitch, const float *Y, int ypitch)
{
    using C = Cfg<D>;
    nrows = nrows < p.n ? nrows : p.n;
    dim3 grid((nrows + C::QB - 1) / C::QB * p.B * p.H);
    if (p.out == LLLA_F32)
        hipLaunchKernelGGL((valu_kernel<D, TI, float, false, true>), grid, dim3(NT), 0, p.stream,
                           (const TI *)p.Q, (const TI *)p.K, (const TI *)p.V, (float *)p.O, p.sq, p.sk,
                           p.sv, p.so, nullptr, p.H, p.B * p.H, p.n, p.causal, p.lambda, p.scale, M, mpitch, Y, ypitch, (const float *)nullptr,
                           (float *)nullptr, (float *)nullptr);
    else
        hipLaunchKernelGGL((valu_kernel<D, TI, bf16_t, false, true>), grid, dim3(NT), 0, p.stream,
                           (const TI *)p.Q, (const TI *)p.K, (const TI *)p.V, (bf16_t *)p.O, p.sq, p.sk,
                           p.sv, p.so, nullptr, p.H, p.B * p.H, p.n, p.causal, p.lambda, p.scale, M, mpitch, Y, ypitch, (const float *)nullptr,
                           (float *)nullptr, (float *)nullptr);
    return hipGetLastError();
}

}  // namespace

hipError_t valu_forward_given(const Problem &p, int nrows, const float *M, int mpitch, const float *Y, int ypitch)
{
    if (p.in != LLLA_BF16) return hipErrorInvalidValue;
    if (p.d == 64) return launch_given<64, bf16_t>(p, nrows, M, mpitch, Y, ypitch);
    if (p.d == 128) return launch_given<128, bf16_t>(p, nrows, M, mpitch, Y, ypitch);
    return hipErrorInvalidValue;
}

hipError_t valu_forward(const Problem &p)
{
    if (dual_forward_rows(p) < p.n) {
        const hipError_t e = by_dim<false>(p, p.n);
        if (e != hipSuccess) return e;
    }
    return dual_forward(p);
}

hipError_t valu_decode(const Problem &p)
{
    const bool all_short = p.n <= dual_max_keys(p.d);
    if (!all_short) {
        const hipError_t e = by_dim<true>(p, 1);
        if (e != hipSuccess || p.seqlens == nullptr) return e;      // without lengths every sequence is long
    }
    return dual_decode(p);
}

}  // namespace llla

// Queries that see few keys (at most min(d, 64)), in fp64 and in the dual (key-space) form of the local linear
// regression of Section 2.3.
//
// Why a kernel of their own.  With m <= d visible keys the d x d matrix Sigma_i of Eq. (query_specific) has rank
// <= m and is held up by the ridge alone in the other directions, so rho_i and delta_i of Eq. (lla) are of size
// ||z|| / lambda and lambda / ||z||^2, and the output weights w (1 - z . rho) / delta are differences of numbers
// ~ ||z||^2 / lambda (10^4 for unit-variance keys at d = 128): fp32 keeps three digits of them.  The same
// minimiser written over the keys instead of the features has none of that.  With u_j = sqrt(w_ij),
// z_j = k_j - q_i, Z' the m x d matrix of rows u_j z_j and G' = Z' Z'^T (m x m), the push-through identity
// (Z'^T Z' + lambda I)^{-1} Z'^T = Z'^T (G' + lambda I)^{-1} gives, with t = (G' + lambda I)^{-1} u,
//     rho_i = Z'^T t,   delta_i = lambda (u . t),   s_ij = w_ij (1 - z_j . rho_i) / delta_i = u_j t_j / (u . t),
// i.e. one m x m positive definite system (all eigenvalues >= lambda, and for m well below d nowhere near it) and
// output weights that are formed directly, without cancellation.  fp64 throughout: these rows are a vanishing part
// of the work (m^2 d / 2 + m^3 / 3 multiply-adds per row).
//
// One 256-thread workgroup per (batch, head, row).  Forward: rows [0, nrows) of a causal call, or every row of a
// non-causal call with n <= the limit.  Decode: one workgroup per (batch, head); a sequence longer than the limit
// exits at once and keeps the output the decode kernel proper has written.
#include "llla_common.hpp"

namespace llla {
namespace {

constexpr int DUAL_NT = 256;

template <typename T> __device__ inline float ld_f32(const T *p, int c);
template <> __device__ inline float ld_f32<float>(const float *p, int c) { return p[c]; }
template <> __device__ inline float ld_f32<bf16_t>(const bf16_t *p, int c) { return bf16_to_f32(p[c]); }
template <typename T> __device__ inline void st_out(T *p, double v);
template <> __device__ inline void st_out<float>(float *p, double v) { *p = (float)v; }
template <> __device__ inline void st_out<bf16_t>(bf16_t *p, double v) { *p = f32_to_bf16((float)v); }

__device__ inline int tri(int j, int l) { return j * (j + 1) / 2 + l; }      // l <= j

// 1 / sqrt(x) in fp64 from the hardware estimate and two Newton steps (relative error ~1e-16 for x well inside the range)
__device__ inline double rsqrt_f64(double x)
{
    double r = __builtin_amdgcn_rsq(x);
    r = r * (1.5 - 0.5 * x * r * r);
    r = r * (1.5 - 0.5 * x * r * r);
    return r;
}

__device__ inline double lane_value(double x, int k)      // x of lane k (k wave-uniform)
{
    const long long v = __builtin_bit_cast(long long, x);
    const int lo = __builtin_amdgcn_readlane((int)v, k), hi = __builtin_amdgcn_readlane((int)(v >> 32), k);
    return __builtin_bit_cast(double, ((long long)hi << 32) | (unsigned)lo);
}

template <typename TI, typename TO>
__global__ __launch_bounds__(DUAL_NT) void dual_rows_kernel(const TI *__restrict__ Qg, const TI *__restrict__ Kg,
                                                            const TI *__restrict__ Vg, TO *__restrict__ Og,
                                                            llla_strides sq, llla_strides sk, llla_strides sv,
                                                            llla_strides so, const int32_t *__restrict__ seqlens,
                                                            int H, int n, int d, int causal, int decode, float lambda,
                                                            const float *__restrict__ lam_rows, float scale,
                                                            float *__restrict__ Rho, float *__restrict__ Delta)
{
    constexpr int MK = DUAL_MAX_KEYS;
    __shared__ float ks[(MK + 1) * 129];           // visible keys, pitch d + 1; the query as one more row
    __shared__ double G[MK * (MK + 1) / 2];        // lower triangle of G' + lambda I, then its Cholesky factor
    __shared__ double u[MK], kq[MK + 1], rd[MK];
    __shared__ double bc[2];

    const int tid = threadIdx.x, bh = blockIdx.y, b = bh / H, h = bh % H;
    const int i = decode ? 0 : (int)blockIdx.x;
    int m;
    if (decode) {
        m = seqlens ? seqlens[b] : n;
        m = m < 1 ? 1 : (m > n ? n : m);
        if (m > MK) return;                        // the whole workgroup: served by the decode kernel proper
    } else {
        m = causal ? i + 1 : n;
    }
    const int m4 = (m + 3) & ~3;                   // the system is padded with identity rows to a multiple of 4
    const int pitch = d + 1;
    const TI *qrow = decode ? Qg + (int64_t)bh * d : Qg + b * sq.batch + h * sq.head + (int64_t)i * sq.seq;
    const TI *Kh = Kg + b * sk.batch + h * sk.head;
    const TI *Vh = Vg + b * sv.batch + h * sv.head;
    // the values this thread needs at the very end (thread c < d: column c of the visible rows of V), requested now
    // (every load below has a valid, clamped address and no condition around it, so that the loads of a thread are
    // all in flight together; a condition per load made the compiler wait for each in turn)
    float vcol[MK];
    {
        const int cc = tid < d ? tid : d - 1;
#pragma unroll
        for (int j = 0; j < MK; ++j) vcol[j] = ld_f32(Vh + (int64_t)(j < m ? j : m - 1) * sv.seq, cc);
    }
    float *qs = ks + m * pitch;                    // row m of the tile: the query
    {
        // thread (r, c) of a 2 x 128 arrangement walks rows r, r + 2, ..: no division by d, coalesced along c
        const int r = tid >> 7, c = tid & 127, cc = c < d ? c : d - 1;
        float kv[MK / 2];
#pragma unroll
        for (int it = 0; it < MK / 2; ++it) {
            const int j = 2 * it + r;
            kv[it] = ld_f32(Kh + (int64_t)(j < m ? j : m - 1) * sk.seq, cc);
        }
        const float qv = ld_f32(qrow, cc);
#pragma unroll
        for (int it = 0; it < MK / 2; ++it) {
            const int j = 2 * it + r;
            if (j < m && c < d) ks[j * pitch + c] = kv[it];
        }
        if (r == 0 && c < d) qs[c] = qv;
    }
    __syncthreads();

    // <k_j, q> for the m keys and <q, q> (row m): four threads per row (m + 1 <= 65 rows: the last one by threads 0..3
    // in a second round)
    for (int base = 0; base <= m; base += DUAL_NT / 4) {
        const int j = base + (tid >> 2), sub = tid & 3;
        double s = 0.0;
        if (j <= m)
            for (int c = sub; c < d; c += 4) s += (double)qs[c] * (double)ks[j * pitch + c];
        s += __shfl_xor(s, 1);
        s += __shfl_xor(s, 2);
        if (j <= m && sub == 0) kq[j] = s;
    }
    __syncthreads();
    // logits, their maximum, u_j = sqrt(w_j) = exp((s_j - max) / 2): the first wave, one key per lane
    if (tid < 64) {
        const double lg = tid < m ? (double)scale * kq[tid] : -INFINITY;
        double mx = lg;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) mx = fmax(mx, __shfl_xor(mx, off));
        if (tid < MK) u[tid] = tid < m ? exp(0.5 * (lg - mx)) : 0.0;
    }
    __syncthreads();

    // G'_jl = u_j u_l <z_j, z_l>, lambda on the diagonal; <z_j, z_l> = <k_j, k_l> - <k_j, q> - <k_l, q> + <q, q>
    // (products of fp32 values are exact in fp64, so the four-term form loses nothing that matters beside lambda);
    // rows m .. m4 - 1 are identity
    const double lam = (!decode && lam_rows) ? (double)lam_rows[(size_t)bh * n + i] : (double)lambda;
    const int ty = tid >> 4, tx = tid & 15;        // 16 x 16 threads tile the lower triangle
    const double qq = kq[m];
    for (int j = ty; j < m4; j += 16)
        for (int l = tx; l <= j; l += 16) {
            double g = (j == l) ? 1.0 : 0.0;
            if (j < m) {
                double s0 = 0.0, s1 = 0.0;
                const float *kj = ks + j * pitch, *kl = ks + l * pitch;
#pragma unroll 4
                for (int c = 0; c < d; c += 4) {                 // d is a multiple of 16
                    s0 += (double)kj[c] * (double)kl[c];
                    s1 += (double)kj[c + 1] * (double)kl[c + 1];
                    s0 += (double)kj[c + 2] * (double)kl[c + 2];
                    s1 += (double)kj[c + 3] * (double)kl[c + 3];
                }
                g = u[j] * u[l] * (((s0 + s1) - kq[j]) - kq[l] + qq) + (j == l ? lam : 0.0);
            }
            G[tri(j, l)] = g;
        }
    __syncthreads();

    // Cholesky G' + lambda I = L L^T in place, four columns per step (two barriers per step instead of per column):
    // every thread factorises the 4 x 4 diagonal block in registers and inverts its factor; one thread per row below
    // solves the row's four entries of the panel; all threads share the rank-4 update of what is left.
    for (int k0 = 0; k0 < m4; k0 += 4) {
        double a00 = G[tri(k0, k0)], a10 = G[tri(k0 + 1, k0)], a11 = G[tri(k0 + 1, k0 + 1)], a20 = G[tri(k0 + 2, k0)],
               a21 = G[tri(k0 + 2, k0 + 1)], a22 = G[tri(k0 + 2, k0 + 2)], a30 = G[tri(k0 + 3, k0)],
               a31 = G[tri(k0 + 3, k0 + 1)], a32 = G[tri(k0 + 3, k0 + 2)], a33 = G[tri(k0 + 3, k0 + 3)];
        // L_d (lower, its diagonal kept as reciprocals r0..r3)
        const double r0 = rsqrt_f64(a00);
        const double l10 = a10 * r0, l20 = a20 * r0, l30 = a30 * r0;
        a11 -= l10 * l10; a21 -= l20 * l10; a31 -= l30 * l10; a22 -= l20 * l20; a32 -= l30 * l20; a33 -= l30 * l30;
        const double r1 = rsqrt_f64(a11);
        const double l21 = a21 * r1, l31 = a31 * r1;
        a22 -= l21 * l21; a32 -= l31 * l21; a33 -= l31 * l31;
        const double r2 = rsqrt_f64(a22);
        const double l32 = a32 * r2;
        a33 -= l32 * l32;
        const double r3 = rsqrt_f64(a33);
        __syncthreads();                           // everybody has read the diagonal block
        if (tid == 0) {
            rd[k0] = r0; rd[k0 + 1] = r1; rd[k0 + 2] = r2; rd[k0 + 3] = r3;
            G[tri(k0 + 1, k0)] = l10; G[tri(k0 + 2, k0)] = l20; G[tri(k0 + 3, k0)] = l30;
            G[tri(k0 + 2, k0 + 1)] = l21; G[tri(k0 + 3, k0 + 1)] = l31; G[tri(k0 + 3, k0 + 2)] = l32;
        }
        // panel: row j of L in columns k0..k0+3 solves x L_d^T = G[j][k0..k0+3] (forward substitution along the row)
        for (int j = k0 + 4 + tid; j < m4; j += DUAL_NT) {
            const double g0 = G[tri(j, k0)], g1 = G[tri(j, k0 + 1)], g2 = G[tri(j, k0 + 2)], g3 = G[tri(j, k0 + 3)];
            const double x0 = g0 * r0;
            const double x1 = (g1 - x0 * l10) * r1;
            const double x2 = (g2 - x0 * l20 - x1 * l21) * r2;
            const double x3 = (g3 - x0 * l30 - x1 * l31 - x2 * l32) * r3;
            G[tri(j, k0)] = x0; G[tri(j, k0 + 1)] = x1; G[tri(j, k0 + 2)] = x2; G[tri(j, k0 + 3)] = x3;
        }
        __syncthreads();
        for (int j = k0 + 4 + ty; j < m4; j += 16) {
            const double j0 = G[tri(j, k0)], j1 = G[tri(j, k0 + 1)], j2 = G[tri(j, k0 + 2)], j3 = G[tri(j, k0 + 3)];
            for (int l = k0 + 4 + tx; l <= j; l += 16)
                G[tri(j, l)] -= j0 * G[tri(l, k0)] + j1 * G[tri(l, k0 + 1)] + j2 * G[tri(l, k0 + 2)] + j3 * G[tri(l, k0 + 3)];
        }
        __syncthreads();
    }

    // t = (L L^T)^{-1} u.  Both substitutions in the first wave, lane j owning element j (m4 <= 64): at step k the owner
    // of element k finishes it (a scalar broadcast of its value) and every later (earlier) element takes its update,
    // one column of L per step; the other waves wait at the barrier below.
    if (tid < 64) {
        const int j = tid;
        double s = (j < m) ? u[j] : 0.0;
        for (int k = 0; k < m4; ++k) {                      // L y = u
            const double yk = lane_value(s, k) * rd[k];
            if (j == k) s = yk;
            else if (j > k && j < m4) s -= G[tri(j, k)] * yk;
        }
        for (int k = m4 - 1; k >= 0; --k) {                 // L^T t = y
            const double tk = lane_value(s, k) * rd[k];
            if (j == k) s = tk;
            else if (j < k) s -= G[tri(k, j)] * tk;
        }
        const double ujt = (j < m) ? u[j] * s : 0.0;        // u_j t_j: output weight s_j = u_j t_j / (u . t)
        double ut = ujt;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) ut += __shfl_xor(ut, off);
        if (j < MK) u[j] = ujt;
        if (j == 0) bc[1] = ut;
    }
    __syncthreads();
    const double ut = bc[1];

    const int64_t orow = decode ? (int64_t)bh * d : b * so.batch + h * so.head + (int64_t)i * so.seq;
    if (tid < d) {                                   // d <= 128 < DUAL_NT
        const int c = tid;
        double o = 0.0, r = 0.0;
#pragma unroll
        for (int j = 0; j < MK; ++j) {
            if (j < m) {
                o += u[j] * (double)vcol[j];
                r += u[j] * ((double)ks[j * pitch + c] - (double)qs[c]);
            }
        }
        st_out(Og + orow + c, o / ut);
        if (!decode && Rho != nullptr) Rho[((size_t)bh * n + i) * d + c] = (float)r;
    }
    if (!decode && Delta != nullptr && tid == 0) Delta[(size_t)bh * n + i] = (float)(lam * ut);
}

template <typename TI, typename TO>
hipError_t launch_dual(const Problem &p, int nrows, bool decode)
{
    hipLaunchKernelGGL((dual_rows_kernel<TI, TO>), dim3(decode ? 1 : nrows, p.B * p.H), dim3(DUAL_NT), 0, p.stream,
                       (const TI *)p.Q, (const TI *)p.K, (const TI *)p.V, (TO *)p.O, p.sq, p.sk, p.sv, p.so, p.seqlens, p.H,
                       p.n, p.d, p.causal, decode ? 1 : 0, p.lambda, decode ? nullptr : p.lambda_rows, p.scale,
                       decode ? nullptr : p.rho, decode ? nullptr : p.delta);
    return hipGetLastError();
}

hipError_t dual_by_dtype(const Problem &p, int nrows, bool decode)
{
    if (p.in == LLLA_F32)
        return p.out == LLLA_F32 ? launch_dual<float, float>(p, nrows, decode) : launch_dual<float, bf16_t>(p, nrows, decode);
    return p.out == LLLA_F32 ? launch_dual<bf16_t, float>(p, nrows, decode) : launch_dual<bf16_t, bf16_t>(p, nrows, decode);
}

}  // namespace

int dual_max_keys(int d) { return d < DUAL_MAX_KEYS ? d : DUAL_MAX_KEYS; }

int dual_forward_rows(const Problem &p)
{
    const int lim = dual_max_keys(p.d);
    if (p.causal) return p.n < lim ? p.n : lim;
    return p.n <= lim ? p.n : 0;
}

hipError_t dual_forward(const Problem &p)
{
    const int nrows = dual_forward_rows(p);
    if (nrows == 0) return hipSuccess;
    return dual_by_dtype(p, nrows, false);
}

hipError_t dual_decode(const Problem &p) { return dual_by_dtype(p, 1, true); }

}  // namespace llla

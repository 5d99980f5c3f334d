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
    __shared__ float ks[MK * 129];                 // visible keys, pitch d + 1
    __shared__ float qs[128];
    __shared__ double G[MK * (MK + 1) / 2];        // lower triangle of G' + lambda I, then its Cholesky factor
    __shared__ double u[MK], t[MK], part[DUAL_NT];
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
    const int pitch = d + 1;
    const TI *qrow = decode ? Qg + (int64_t)bh * d : Qg + b * sq.batch + h * sq.head + (int64_t)i * sq.seq;
    const TI *Kh = Kg + b * sk.batch + h * sk.head;
    const TI *Vh = Vg + b * sv.batch + h * sv.head;
    for (int c = tid; c < d; c += DUAL_NT) qs[c] = ld_f32(qrow, c);
    for (int idx = tid; idx < m * d; idx += DUAL_NT) {
        const int j = idx / d, c = idx % d;
        ks[j * pitch + c] = ld_f32(Kh + (int64_t)j * sk.seq, c);
    }
    __syncthreads();

    // logits, their maximum, u_j = sqrt(w_j) = exp((s_j - max) / 2): four threads per key
    {
        const int j = tid >> 2, sub = tid & 3;
        double s = 0.0;
        if (j < m)
            for (int c = sub; c < d; c += 4) s += (double)qs[c] * (double)ks[j * pitch + c];
        part[tid] = s;
    }
    __syncthreads();
    if (tid < m) t[tid] = (double)scale * ((part[4 * tid] + part[4 * tid + 1]) + (part[4 * tid + 2] + part[4 * tid + 3]));
    __syncthreads();
    if (tid == 0) {
        double mx = t[0];
        for (int j = 1; j < m; ++j) mx = fmax(mx, t[j]);
        bc[0] = mx;
    }
    __syncthreads();
    if (tid < m) u[tid] = exp(0.5 * (t[tid] - bc[0]));
    __syncthreads();

    // G'_jl = u_j u_l <z_j, z_l>, lambda on the diagonal
    const double lam = (!decode && lam_rows) ? (double)lam_rows[(size_t)bh * n + i] : (double)lambda;
    const int ntri = m * (m + 1) / 2;
    for (int e = tid; e < ntri; e += DUAL_NT) {
        int j = (int)((sqrt(8.0 * e + 1.0) - 1.0) * 0.5);
        while (tri(j + 1, 0) <= e) ++j;
        while (tri(j, 0) > e) --j;
        const int l = e - tri(j, 0);
        double s = 0.0;
        for (int c = 0; c < d; ++c) {
            const double qc = (double)qs[c];
            s += ((double)ks[j * pitch + c] - qc) * ((double)ks[l * pitch + c] - qc);
        }
        G[e] = u[j] * u[l] * s + (j == l ? lam : 0.0);
    }
    __syncthreads();

    // Cholesky G' + lambda I = L L^T in place (column by column; the trailing update is shared by all threads)
    for (int k = 0; k < m; ++k) {
        if (tid == 0) G[tri(k, k)] = sqrt(G[tri(k, k)]);
        __syncthreads();
        const double piv = 1.0 / G[tri(k, k)];
        for (int j = k + 1 + tid; j < m; j += DUAL_NT) G[tri(j, k)] *= piv;
        __syncthreads();
        const int rem = m - k - 1;
        for (int e = tid; e < rem * (rem + 1) / 2; e += DUAL_NT) {
            int a = (int)((sqrt(8.0 * e + 1.0) - 1.0) * 0.5);
            while (tri(a + 1, 0) <= e) ++a;
            while (tri(a, 0) > e) --a;
            const int c2 = e - tri(a, 0);
            const int j = k + 1 + a, l = k + 1 + c2;
            G[tri(j, l)] -= G[tri(j, k)] * G[tri(l, k)];
        }
        __syncthreads();
    }
    // t = (L L^T)^{-1} u: the two substitutions are short and sequential; one thread walks them
    if (tid == 0) {
        for (int j = 0; j < m; ++j) {
            double s = u[j];
            for (int l = 0; l < j; ++l) s -= G[tri(j, l)] * t[l];
            t[j] = s / G[tri(j, j)];
        }
        for (int j = m - 1; j >= 0; --j) {
            double s = t[j];
            for (int l = j + 1; l < m; ++l) s -= G[tri(l, j)] * t[l];
            t[j] = s / G[tri(j, j)];
        }
        double ut = 0.0;
        for (int j = 0; j < m; ++j) ut += u[j] * t[j];
        bc[1] = ut;
    }
    __syncthreads();
    const double ut = bc[1];
    if (tid < m) u[tid] = u[tid] * t[tid];          // u_j t_j: output weight s_j = u_j t_j / (u . t)
    __syncthreads();

    const int64_t orow = decode ? (int64_t)bh * d : b * so.batch + h * so.head + (int64_t)i * so.seq;
    for (int c = tid; c < d; c += DUAL_NT) {
        double o = 0.0, r = 0.0;
        for (int j = 0; j < m; ++j) {
            o += u[j] * (double)ld_f32(Vh + (int64_t)j * sv.seq, c);
            r += u[j] * ((double)ks[j * pitch + c] - (double)qs[c]);
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

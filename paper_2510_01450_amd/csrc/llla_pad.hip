// Head dimensions 16 and 32 on the matrix-core forward: the call is run at d = 64 on zero-padded copies.
//
// Why this is exact.  With the features d .. 63 of every query and key equal to zero the logits are unchanged, the
// padded entries of mu~ are zero, the padded rows and columns of Sigma~ are zero, and the ridge puts lambda on the
// padded diagonal: the system of Eq. (query_specific) splits into the original one and lambda * y_pad = 0.  The
// products that fill the padded tiles are products with exact zeros, so the factorisation sees an exactly
// block-diagonal matrix and the original block is solved as it would be alone (up to the order of rounding).  The
// padded columns of V give padded columns of O that are dropped.
//
// Why it pays.  The d x d moment of a query-key pair is a contraction only the matrix cores do fast; the vector
// kernels need d^2 fp32 multiply-adds per pair, the padded call 64^2 / 2 on 16-bit MFMA at sixteen times the rate
// (fp32 inputs: fp32 MFMA).  The copies are Theta(B H n 64), like the rest of the workspace.
#include "llla_common.hpp"

namespace llla {
namespace {

constexpr int PD = 64;      // padded head dimension

struct PadLayout {
    size_t q, k, v, o, rho, inner, total;
};

PadLayout make_pad_layout(int B, int H, int n, llla_dtype in, bool cg = false)
{
    const size_t rows = (size_t)B * H * n;
    const size_t esz = in == LLLA_F32 ? 4 : 2;
    PadLayout L{};
    size_t off = 0;
    L.q = off; off += round_up(rows * PD * esz, 256);
    L.k = off; off += round_up(rows * PD * esz, 256);
    L.v = off; off += round_up(rows * PD * esz, 256);
    L.o = off; off += round_up(rows * PD * 4, 256);         // fp32 or bf16 output rows
    L.rho = off; off += round_up(rows * PD * 4, 256);
    L.inner = off;
    off += round_up(cg ? mfma_forward_cg_workspace_bytes(B, H, n, PD, in)
                       : in == LLLA_F32 ? mfma_forward_f32_workspace_bytes(B, H, n) : mfma_forward_workspace_bytes(B, H, n, PD, in), 256);
    L.total = off;
    return L;
}

// One thread per 16-byte chunk of a padded row: chunks inside the original row are copied, the others cleared.
// src: [B,H,n,d] with strides (elements); dst: [B*H*n, PD] contiguous.  ESZ = bytes per element.
template <int ESZ>
__global__ __launch_bounds__(256) void pad_rows_kernel(const char *__restrict__ src, llla_strides s, int H, int n, int d,
                                                       size_t nchunks, uint4 *__restrict__ dst)
{
    constexpr int CPR = PD * ESZ / 16;                      // chunks per padded row
    const size_t id = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= nchunks) return;
    const size_t row = id / CPR;
    const int c = (int)(id % CPR);
    const int i = (int)(row % n);
    const size_t bh = row / n;
    const int h = (int)(bh % H);
    const int64_t b = (int64_t)(bh / H);
    uint4 v = {0u, 0u, 0u, 0u};
    if (c * 16 < d * ESZ) {
        const int64_t e = b * s.batch + (int64_t)h * s.head + (int64_t)i * s.seq;
        v = *reinterpret_cast<const uint4 *>(src + e * ESZ + c * 16);
    }
    dst[id] = v;
}

// The first d elements of every padded row back into a strided [B,H,n,d] tensor, one chunk of type T per thread
// (16 bytes where the destination rows are 16-byte aligned, 4 bytes for the statistics, which need not be).
template <int ESZ, class T>
__global__ __launch_bounds__(256) void unpad_rows_kernel(const T *__restrict__ src, char *__restrict__ dst, llla_strides s,
                                                         int H, int n, int d, size_t nchunks)
{
    constexpr int CB = (int)sizeof(T);
    const int cpr = d * ESZ / CB;                           // chunks per original row
    constexpr int CPR = PD * ESZ / CB;
    const size_t id = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= nchunks) return;
    const size_t row = id / cpr;
    const int c = (int)(id % cpr);
    const int i = (int)(row % n);
    const size_t bh = row / n;
    const int h = (int)(bh % H);
    const int64_t b = (int64_t)(bh / H);
    const int64_t e = b * s.batch + (int64_t)h * s.head + (int64_t)i * s.seq;
    *reinterpret_cast<T *>(dst + e * ESZ + c * CB) = src[row * CPR + c];
}

struct Rows {
    int B, H, n, d;
    hipStream_t stream;
};

hipError_t pad_rows(const void *src, llla_strides s, const Rows &r, bool f32, void *dst)
{
    const size_t rows = (size_t)r.B * r.H * r.n;
    if (f32) {
        const size_t nch = rows * (PD * 4 / 16);
        pad_rows_kernel<4><<<dim3((unsigned)((nch + 255) / 256)), dim3(256), 0, r.stream>>>(
            static_cast<const char *>(src), s, r.H, r.n, r.d, nch, static_cast<uint4 *>(dst));
    } else {
        const size_t nch = rows * (PD * 2 / 16);
        pad_rows_kernel<2><<<dim3((unsigned)((nch + 255) / 256)), dim3(256), 0, r.stream>>>(
            static_cast<const char *>(src), s, r.H, r.n, r.d, nch, static_cast<uint4 *>(dst));
    }
    return hipGetLastError();
}

template <int ESZ, class T>
hipError_t unpad_rows(const void *src, void *dst, llla_strides s, const Rows &r)
{
    const size_t nch = (size_t)r.B * r.H * r.n * (r.d * ESZ / sizeof(T));
    unpad_rows_kernel<ESZ, T><<<dim3((unsigned)((nch + 255) / 256)), dim3(256), 0, r.stream>>>(
        static_cast<const T *>(src), static_cast<char *>(dst), s, r.H, r.n, r.d, nch);
    return hipGetLastError();
}

struct PadBackwardLayout {
    size_t q, k, v, g, dq, dk, dv, inner, total;
};

PadBackwardLayout make_pad_backward_layout(int B, int H, int n)
{
    const size_t rows = (size_t)B * H * n;
    PadBackwardLayout L{};
    size_t off = 0;
    L.q = off; off += round_up(rows * PD * 2, 256);
    L.k = off; off += round_up(rows * PD * 2, 256);
    L.v = off; off += round_up(rows * PD * 2, 256);
    L.g = off; off += round_up(rows * PD * 2, 256);
    L.dq = off; off += round_up(rows * PD * 4, 256);
    L.dk = off; off += round_up(rows * PD * 4, 256);
    L.dv = off; off += round_up(rows * PD * 4, 256);
    L.inner = off;
    off += round_up(backward_workspace_bytes(B, H, n, PD, LLLA_BF16, LLLA_PATH_MFMA), 256);
    L.total = off;
    return L;
}

}  // namespace

bool padded_forward_supported(int d, llla_dtype in)
{
    if (d != 16 && d != 32) return false;
    return in == LLLA_F32 ? mfma_forward_f32_supported(PD, true) : mfma_forward_supported(PD, in, true);
}

size_t padded_forward_workspace_bytes(int B, int H, int n, int d, llla_dtype in)
{
    if (!padded_forward_supported(d, in)) return 0;
    return make_pad_layout(B, H, n, in).total;
}

hipError_t padded_forward(const Problem &p)
{
    // every grid below is one-dimensional in 256-thread groups over 16-byte chunks: at most 2^31 rows * 16 chunks
    const PadLayout L = make_pad_layout(p.B, p.H, p.n, p.in);
    char *ws = static_cast<char *>(p.ws);
    const llla_strides sp = {(int64_t)p.H * p.n * PD, (int64_t)p.n * PD, (int64_t)PD};

    const Rows r{p.B, p.H, p.n, p.d, p.stream};
    const bool f32 = p.in == LLLA_F32;
    stage_mark(p.stream, "pad");
    hipError_t e = pad_rows(p.Q, p.sq, r, f32, ws + L.q);
    if (e != hipSuccess) return e;
    e = pad_rows(p.K, p.sk, r, f32, ws + L.k);
    if (e != hipSuccess) return e;
    e = pad_rows(p.V, p.sv, r, f32, ws + L.v);
    if (e != hipSuccess) return e;

    Problem q = p;
    q.Q = ws + L.q; q.K = ws + L.k; q.V = ws + L.v; q.O = ws + L.o;
    q.sq = q.sk = q.sv = q.so = sp;
    q.d = PD;
    q.live_d = p.d;
    q.rho = p.rho ? reinterpret_cast<float *>(ws + L.rho) : nullptr;
    q.ws = ws + L.inner;
    q.ws_bytes = L.total - L.inner;
    e = p.in == LLLA_F32 ? mfma_forward_f32(q) : mfma_forward(q);
    if (e != hipSuccess) return e;

    stage_mark(p.stream, "unpad");
    e = p.out == LLLA_F32 ? unpad_rows<4, uint4>(ws + L.o, p.O, p.so, r) : unpad_rows<2, uint4>(ws + L.o, p.O, p.so, r);
    if (e != hipSuccess) return e;
    if (p.rho) {
        const llla_strides sr = {(int64_t)p.H * p.n * p.d, (int64_t)p.n * p.d, (int64_t)p.d};
        e = unpad_rows<4, uint32_t>(ws + L.rho, p.rho, sr, r);
    }
    return e;
}

// The approximate mode (conjugate gradients) at d = 16 / 32 (bf16): the same padding.  The padded entries of every
// iterate stay zero -- the residual there is mu_pad - (Sigma p)_pad = 0 - lambda * 0 -- so steps, residuals and the
// active mask are those of the original system.
size_t padded_forward_cg_workspace_bytes(int B, int H, int n, int d, llla_dtype in)
{
    if (in != LLLA_BF16 || !padded_forward_supported(d, in)) return 0;
    return make_pad_layout(B, H, n, in, true).total;
}

hipError_t padded_forward_cg(const Problem &p, int T, float eps, int32_t *iters)
{
    const PadLayout L = make_pad_layout(p.B, p.H, p.n, p.in, true);
    char *ws = static_cast<char *>(p.ws);
    const llla_strides sp = {(int64_t)p.H * p.n * PD, (int64_t)p.n * PD, (int64_t)PD};
    const Rows r{p.B, p.H, p.n, p.d, p.stream};
    hipError_t e = pad_rows(p.Q, p.sq, r, false, ws + L.q);
    if (e != hipSuccess) return e;
    e = pad_rows(p.K, p.sk, r, false, ws + L.k);
    if (e != hipSuccess) return e;
    e = pad_rows(p.V, p.sv, r, false, ws + L.v);
    if (e != hipSuccess) return e;
    Problem q = p;
    q.Q = ws + L.q; q.K = ws + L.k; q.V = ws + L.v; q.O = ws + L.o;
    q.sq = q.sk = q.sv = q.so = sp;
    q.d = PD;
    q.rho = p.rho ? reinterpret_cast<float *>(ws + L.rho) : nullptr;
    q.ws = ws + L.inner;
    q.ws_bytes = L.total - L.inner;
    e = mfma_forward_cg(q, T, eps, iters);
    if (e != hipSuccess) return e;
    e = p.out == LLLA_F32 ? unpad_rows<4, uint4>(ws + L.o, p.O, p.so, r) : unpad_rows<2, uint4>(ws + L.o, p.O, p.so, r);
    if (e != hipSuccess) return e;
    if (p.rho) {
        const llla_strides sr = {(int64_t)p.H * p.n * p.d, (int64_t)p.n * p.d, (int64_t)p.d};
        e = unpad_rows<4, uint32_t>(ws + L.rho, p.rho, sr, r);
    }
    return e;
}

// The backward pass at d = 16 / 32 (bf16): the same padding.  The gradient with respect to a padded feature is zero to
// first order -- a padded key feature enters the output only through its product with the padded part of y, and both
// factors vanish -- so the padded columns of dQ, dK and dV are dropped; dlambda has no feature index.
bool padded_backward_supported(int d, llla_dtype in)
{
    return (d == 16 || d == 32) && in == LLLA_BF16 && mfma_forward_supported(PD, in, true);
}

size_t padded_backward_workspace_bytes(int B, int H, int n, int d, llla_dtype in)
{
    if (!padded_backward_supported(d, in)) return 0;
    return make_pad_backward_layout(B, H, n).total;
}

hipError_t padded_backward(const BackwardProblem &p)
{
    const PadBackwardLayout L = make_pad_backward_layout(p.B, p.H, p.n);
    char *ws = static_cast<char *>(p.ws);
    const llla_strides sp = {(int64_t)p.H * p.n * PD, (int64_t)p.n * PD, (int64_t)PD};
    const Rows r{p.B, p.H, p.n, p.d, p.stream};

    hipError_t e = pad_rows(p.Q, p.sq, r, false, ws + L.q);
    if (e != hipSuccess) return e;
    e = pad_rows(p.K, p.sk, r, false, ws + L.k);
    if (e != hipSuccess) return e;
    e = pad_rows(p.V, p.sv, r, false, ws + L.v);
    if (e != hipSuccess) return e;
    e = pad_rows(p.dO, p.sdo, r, false, ws + L.g);
    if (e != hipSuccess) return e;

    BackwardProblem q = p;
    q.Q = ws + L.q; q.K = ws + L.k; q.V = ws + L.v; q.dO = ws + L.g;
    q.sq = q.sk = q.sv = q.sdo = sp;
    q.dQ = reinterpret_cast<float *>(ws + L.dq);
    q.dK = reinterpret_cast<float *>(ws + L.dk);
    q.dV = reinterpret_cast<float *>(ws + L.dv);
    q.d = PD;
    q.live_d = p.d;
    q.ws = ws + L.inner;
    q.ws_bytes = L.total - L.inner;
    e = backward(q, LLLA_PATH_MFMA);
    if (e != hipSuccess) return e;

    const llla_strides sg = {(int64_t)p.H * p.n * p.d, (int64_t)p.n * p.d, (int64_t)p.d};
    e = unpad_rows<4, uint4>(q.dQ, p.dQ, sg, r);
    if (e != hipSuccess) return e;
    e = unpad_rows<4, uint4>(q.dK, p.dK, sg, r);
    if (e != hipSuccess) return e;
    return unpad_rows<4, uint4>(q.dV, p.dV, sg, r);
}

}  // namespace llla

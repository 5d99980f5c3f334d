// C ABI of the library: host-side validation and dispatch.  Every check runs before anything is
// enqueued, so each error path can be exercised without a GPU.
#include <cmath>

#include "llla_common.hpp"

namespace {

using llla::Problem;

constexpr int kMaxGridY = 65535;
// LLLA_PATH_AUTO and the padded matrix-core calls (d = 16 / 32 run at d = 64; padded tiles and solve blocks skipped).
// Measured at 64 heads, bf16, vector vs padded.  Forward, d = 32: 0.028 vs 0.036 ms at n = 16, 0.075 vs 0.037 at 32, 0.19 vs
// 0.057 at 128, 22.5 vs 1.56 at 4096; d = 16: 0.028 vs 0.036 at n = 16, 0.045 vs 0.038 at 32, 0.064 vs 0.053 at 128, 6.2 vs 1.2 at
// 4096 -> from 32 rows on.  Backward, d = 32: 0.055 vs 0.057 at n = 32, 0.080 vs 0.070 at 64, 42.5 vs 3.7 at 4096 -> from 64 rows
// on; d = 16: 0.071 vs 0.106 at n = 128, 0.32 vs 0.21 at 512, 15.1 vs 3.2 at 4096 -> from 512 rows on.  fp32 inputs (fp32 MFMA, a
// sixteenth of the 16-bit rate; forward only), d = 32: 0.34 vs 0.36 ms at n = 256, 0.73 vs 0.53 at 512, 2.0 vs 1.1 at 1024, 24.3
// vs 11.1 at 4096, but 0.196 vs 0.217 at 2 heads x 1024 -> from 1024 rows on; d = 16: 0.062 vs 0.30 at n = 128, 0.53 vs 0.77 at 1024,
// 6.5 vs 6.9 at 4096 -> only when forced.
bool auto_takes_padded(int n, int d, llla_dtype in) { return in == LLLA_BF16 ? n >= 32 : (d == 32 && n >= 1024); }
bool auto_takes_padded_backward(int n, int d, llla_dtype in) { return in == LLLA_BF16 && n >= (d == 32 ? 64 : 512); }

bool dim_supported(int d) { return d == 16 || d == 32 || d == 64 || d == 128; }
bool dtype_ok(llla_dtype t) { return t == LLLA_F32 || t == LLLA_BF16; }
size_t elem_size(llla_dtype t) { return t == LLLA_F32 ? 4 : 2; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool strides_aligned(const llla_strides &s, llla_dtype t)
{
    const int64_t q = 16 / (int64_t)elem_size(t);
    return s.batch % q == 0 && s.head % q == 0 && s.seq % q == 0;
}

// the d stride is 1, so a row needs seq >= d; batch/head strides may alias only in degenerate shapes
bool strides_cover(const llla_strides &s, int B, int H, int n, int d)
{
    if (s.seq < d && n > 1) return false;
    if (s.head < 0 || s.batch < 0 || s.seq < 0) return false;
    if (H > 1 && s.head == 0) return false;
    if (B > 1 && s.batch == 0) return false;
    return true;
}

llla_status check_common(int B, int H, int n, int d, llla_dtype in, llla_dtype out, float lambda, float scale)
{
    if (B <= 0 || H <= 0 || n <= 0 || d <= 0) return LLLA_ERR_SHAPE;
    if (!dtype_ok(in) || !dtype_ok(out)) return LLLA_ERR_DTYPE;
    if (!dim_supported(d)) return LLLA_ERR_UNSUPPORTED;
    if ((int64_t)B * H > kMaxGridY) return LLLA_ERR_SHAPE;
    if ((int64_t)B * H * n > 2147483647LL) return LLLA_ERR_SHAPE;       // one-dimensional grids index (head, row block) pairs
    if (!(lambda > 0.f) || !std::isfinite(lambda) || !std::isfinite(scale)) return LLLA_ERR_PARAM;
    return LLLA_OK;
}

llla_status check_workspace(size_t need, void *ws, size_t ws_bytes)
{
    if (need == 0) return LLLA_OK;
    if (ws == nullptr || ws_bytes < need) return LLLA_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(ws) & 255u) != 0) return LLLA_ERR_WORKSPACE;
    return LLLA_OK;
}

}  // namespace

extern "C" {

size_t llla_forward_workspace_bytes(int B, int H, int n, int d, llla_dtype in)
{
    if (B <= 0 || H <= 0 || n <= 0 || !dim_supported(d) || !dtype_ok(in)) return 0;
    if (llla::padded_forward_supported(d, in)) return llla::padded_forward_workspace_bytes(B, H, n, d, in);
    if (in == LLLA_F32) return llla::mfma_forward_f32_supported(d, true) ? llla::mfma_forward_f32_workspace_bytes(B, H, n) : 0;
    return llla::mfma_forward_workspace_bytes(B, H, n, d, in);
}

llla_status llla_forward_ex(const void *Q, const void *K, const void *V, void *O, llla_strides sq, llla_strides sk,
                            llla_strides sv, llla_strides so, int B, int H, int n, int d, llla_dtype in,
                            llla_dtype out, int causal, float lambda, const float *lambda_rows, float scale,
                            float *rho, float *delta, llla_path path, void *workspace, size_t workspace_bytes,
                            void *stream)
{
    if (!Q || !K || !V || !O) return LLLA_ERR_NULL;
    // with a ridge per row the scalar is ignored, whatever it holds
    llla_status st = check_common(B, H, n, d, in, out, lambda_rows ? 1.f : lambda, scale);
    if (st != LLLA_OK) return st;
    if ((reinterpret_cast<uintptr_t>(lambda_rows) & 3u) || (reinterpret_cast<uintptr_t>(rho) & 3u) ||
        (reinterpret_cast<uintptr_t>(delta) & 3u))
        return LLLA_ERR_ALIGN;
    if (path != LLLA_PATH_AUTO && path != LLLA_PATH_VALU && path != LLLA_PATH_MFMA) return LLLA_ERR_PARAM;
    if (!strides_cover(sq, B, H, n, d) || !strides_cover(sk, B, H, n, d) || !strides_cover(sv, B, H, n, d) ||
        !strides_cover(so, B, H, n, d))
        return LLLA_ERR_SHAPE;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !strides_aligned(sq, in) ||
        !strides_aligned(sk, in) || !strides_aligned(sv, in) || !strides_aligned(so, out))
        return LLLA_ERR_ALIGN;

    // the matrix-core sweeps put their 64-row blocks on grid.y: at most 65535 of them
    const bool f32_mfma = in == LLLA_F32 && llla::mfma_forward_f32_supported(d, causal != 0);
    // d = 16 / 32: the d = 64 kernels on zero-padded copies
    const bool padded = llla::padded_forward_supported(d, in);
    const bool has_mfma = (padded || f32_mfma || llla::mfma_forward_supported(d, in, causal != 0)) && (n + 63) / 64 <= kMaxGridY;
    if (path == LLLA_PATH_MFMA && !has_mfma) return LLLA_ERR_UNSUPPORTED;
    const bool use_mfma = has_mfma && path != LLLA_PATH_VALU && !(padded && path == LLLA_PATH_AUTO && !auto_takes_padded(n, d, in));
    if (use_mfma) {
        st = check_workspace(padded ? llla::padded_forward_workspace_bytes(B, H, n, d, in)
                             : f32_mfma ? llla::mfma_forward_f32_workspace_bytes(B, H, n)
                                        : llla::mfma_forward_workspace_bytes(B, H, n, d, in), workspace, workspace_bytes);
        if (st != LLLA_OK) return st;
    }

    Problem p{};
    p.Q = Q; p.K = K; p.V = V; p.O = O;
    p.sq = sq; p.sk = sk; p.sv = sv; p.so = so;
    p.seqlens = nullptr;
    p.B = B; p.H = H; p.n = n; p.d = d;
    p.in = in; p.out = out;
    p.causal = causal ? 1 : 0;
    p.lambda = lambda; p.scale = scale;
    p.lambda_rows = lambda_rows; p.rho = rho; p.delta = delta;
    p.ws = workspace; p.ws_bytes = workspace_bytes;
    p.stream = static_cast<hipStream_t>(stream);
    llla::stage_begin(p.stream);
    if (!use_mfma) llla::stage_mark(p.stream, "valu_forward");
    const hipError_t e = !use_mfma ? llla::valu_forward(p)
                         : padded  ? llla::padded_forward(p)
                         : f32_mfma ? llla::mfma_forward_f32(p) : llla::mfma_forward(p);
    llla::stage_end(p.stream);
    return e == hipSuccess ? LLLA_OK : LLLA_ERR_LAUNCH;
}

llla_status llla_forward_path(const void *Q, const void *K, const void *V, void *O, llla_strides sq,
                              llla_strides sk, llla_strides sv, llla_strides so, int B, int H, int n, int d,
                              llla_dtype in, llla_dtype out, int causal, float lambda, float scale,
                              llla_path path, void *workspace, size_t workspace_bytes, void *stream)
{
    return llla_forward_ex(Q, K, V, O, sq, sk, sv, so, B, H, n, d, in, out, causal, lambda, nullptr, scale, nullptr,
                           nullptr, path, workspace, workspace_bytes, stream);
}

llla_status llla_forward(const void *Q, const void *K, const void *V, void *O, llla_strides sq, llla_strides sk,
                         llla_strides sv, llla_strides so, int B, int H, int n, int d, llla_dtype in,
                         llla_dtype out, int causal, float lambda, float scale, void *workspace,
                         size_t workspace_bytes, void *stream)
{
    return llla_forward_path(Q, K, V, O, sq, sk, sv, so, B, H, n, d, in, out, causal, lambda, scale,
                             LLLA_PATH_AUTO, workspace, workspace_bytes, stream);
}

size_t llla_forward_cg_workspace_bytes(int B, int H, int n, int d, llla_dtype in)
{
    if (B <= 0 || H <= 0 || n <= 0 || !dim_supported(d) || !dtype_ok(in)) return 0;
    const size_t padded = llla::padded_forward_cg_workspace_bytes(B, H, n, d, in);
    return padded ? padded : llla::mfma_forward_cg_workspace_bytes(B, H, n, d, in);
}

llla_status llla_forward_cg(const void *Q, const void *K, const void *V, void *O, llla_strides sq, llla_strides sk,
                            llla_strides sv, llla_strides so, int B, int H, int n, int d, llla_dtype in,
                            llla_dtype out, float lambda, float scale, int max_steps, float eps, float *rho,
                            float *delta, int32_t *steps, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!Q || !K || !V || !O) return LLLA_ERR_NULL;
    llla_status st = check_common(B, H, n, d, in, out, lambda, scale);
    if (st != LLLA_OK) return st;
    if (max_steps < 0 || max_steps > 4096 || !(eps >= 0.f) || !std::isfinite(eps)) return LLLA_ERR_PARAM;
    if (!strides_cover(sq, B, H, n, d) || !strides_cover(sk, B, H, n, d) || !strides_cover(sv, B, H, n, d) ||
        !strides_cover(so, B, H, n, d))
        return LLLA_ERR_SHAPE;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !strides_aligned(sq, in) ||
        !strides_aligned(sk, in) || !strides_aligned(sv, in) || !strides_aligned(so, out) ||
        (reinterpret_cast<uintptr_t>(rho) & 3u) || (reinterpret_cast<uintptr_t>(delta) & 3u) ||
        (reinterpret_cast<uintptr_t>(steps) & 3u))
        return LLLA_ERR_ALIGN;
    const size_t padded_ws = llla::padded_forward_cg_workspace_bytes(B, H, n, d, in);     // d = 16 / 32: run at d = 64 on zero-padded copies
    if ((padded_ws == 0 && !llla::mfma_forward_supported(d, in, true)) || (n + 63) / 64 > kMaxGridY) return LLLA_ERR_UNSUPPORTED;
    st = check_workspace(padded_ws ? padded_ws : llla::mfma_forward_cg_workspace_bytes(B, H, n, d, in), workspace, workspace_bytes);
    if (st != LLLA_OK) return st;

    Problem p{};
    p.Q = Q; p.K = K; p.V = V; p.O = O;
    p.sq = sq; p.sk = sk; p.sv = sv; p.so = so;
    p.B = B; p.H = H; p.n = n; p.d = d;
    p.in = in; p.out = out;
    p.causal = 1;
    p.lambda = lambda; p.scale = scale;
    p.rho = rho; p.delta = delta;
    p.ws = workspace; p.ws_bytes = workspace_bytes;
    p.stream = static_cast<hipStream_t>(stream);
    llla::stage_begin(p.stream);
    const hipError_t e = padded_ws ? llla::padded_forward_cg(p, max_steps, eps, steps) : llla::mfma_forward_cg(p, max_steps, eps, steps);
    llla::stage_end(p.stream);
    return e == hipSuccess ? LLLA_OK : LLLA_ERR_LAUNCH;
}

size_t llla_backward_workspace_bytes(int B, int H, int n, int d, llla_dtype in)
{
    if (B <= 0 || H <= 0 || n <= 0 || !dim_supported(d) || !dtype_ok(in)) return 0;
    const size_t a = llla::backward_workspace_bytes(B, H, n, d, in, LLLA_PATH_AUTO);
    const size_t b = llla::padded_backward_workspace_bytes(B, H, n, d, in);
    return a > b ? a : b;
}

llla_status llla_backward(const void *Q, const void *K, const void *V, const void *dO, llla_strides sq, llla_strides sk,
                          llla_strides sv, llla_strides sdo, float *dQ, float *dK, float *dV, float *dlambda, int B,
                          int H, int n, int d, llla_dtype in, float lambda, const float *lambda_rows, float scale,
                          llla_path path, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!Q || !K || !V || !dO || !dQ || !dK || !dV) return LLLA_ERR_NULL;
    llla_status st = check_common(B, H, n, d, in, LLLA_F32, lambda_rows ? 1.f : lambda, scale);
    if (st != LLLA_OK) return st;
    if (!strides_cover(sq, B, H, n, d) || !strides_cover(sk, B, H, n, d) || !strides_cover(sv, B, H, n, d) ||
        !strides_cover(sdo, B, H, n, d))
        return LLLA_ERR_SHAPE;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(dO) || !aligned16(dQ) || !aligned16(dK) ||
        !aligned16(dV) || !strides_aligned(sq, in) || !strides_aligned(sk, in) || !strides_aligned(sv, in) ||
        !strides_aligned(sdo, in) || (reinterpret_cast<uintptr_t>(dlambda) & 3u) ||
        (reinterpret_cast<uintptr_t>(lambda_rows) & 3u))
        return LLLA_ERR_ALIGN;
    if (path != LLLA_PATH_AUTO && path != LLLA_PATH_VALU && path != LLLA_PATH_MFMA) return LLLA_ERR_PARAM;
    const bool padded = llla::padded_backward_supported(d, in);
    if (path == LLLA_PATH_MFMA && ((!padded && !llla::mfma_forward_supported(d, in, true)) || (n + 63) / 64 > kMaxGridY))
        return LLLA_ERR_UNSUPPORTED;
    // d = 16 / 32 (bf16): the d = 64 matrix-core backward on zero-padded copies, where LLLA_PATH_AUTO takes the padded forward
    const bool use_padded = padded && (n + 63) / 64 <= kMaxGridY &&
                            (path == LLLA_PATH_MFMA || (path == LLLA_PATH_AUTO && auto_takes_padded_backward(n, d, in)));
    st = check_workspace(use_padded ? llla::padded_backward_workspace_bytes(B, H, n, d, in)
                                    : llla::backward_workspace_bytes(B, H, n, d, in, path), workspace, workspace_bytes);
    if (st != LLLA_OK) return st;

    llla::BackwardProblem p{};
    p.Q = Q; p.K = K; p.V = V; p.dO = dO;
    p.sq = sq; p.sk = sk; p.sv = sv; p.sdo = sdo;
    p.dQ = dQ; p.dK = dK; p.dV = dV; p.dlambda = dlambda;
    p.B = B; p.H = H; p.n = n; p.d = d;
    p.in = in;
    p.lambda = lambda; p.lambda_rows = lambda_rows; p.scale = scale;
    p.ws = workspace; p.ws_bytes = workspace_bytes;
    p.stream = static_cast<hipStream_t>(stream);
    return (use_padded ? llla::padded_backward(p) : llla::backward(p, path)) == hipSuccess ? LLLA_OK : LLLA_ERR_LAUNCH;
}

size_t llla_decode_workspace_bytes(int B, int H, int L_max, int d, llla_dtype in)
{
    if (B <= 0 || H <= 0 || L_max <= 0 || !dim_supported(d) || !dtype_ok(in)) return 0;
    return llla::mfma_decode_workspace_bytes(B, H, L_max, d, in);
}

llla_status llla_decode_path(const void *q, const void *Kc, const void *Vc, void *o, llla_strides sk,
                             llla_strides sv, const int32_t *seqlens, int B, int H, int L_max, int d,
                             llla_dtype in, llla_dtype out, float lambda, float scale, llla_path path,
                             void *workspace, size_t workspace_bytes, void *stream)
{
    if (!q || !Kc || !Vc || !o) return LLLA_ERR_NULL;
    llla_status st = check_common(B, H, L_max, d, in, out, lambda, scale);
    if (st != LLLA_OK) return st;
    if (path != LLLA_PATH_AUTO && path != LLLA_PATH_VALU && path != LLLA_PATH_MFMA) return LLLA_ERR_PARAM;
    if (!strides_cover(sk, B, H, L_max, d) || !strides_cover(sv, B, H, L_max, d)) return LLLA_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(Kc) || !aligned16(Vc) || !aligned16(o) || !strides_aligned(sk, in) ||
        !strides_aligned(sv, in) || (seqlens && (reinterpret_cast<uintptr_t>(seqlens) & 3u)))
        return LLLA_ERR_ALIGN;

    Problem p{};
    p.Q = q; p.K = Kc; p.V = Vc; p.O = o;
    p.sk = sk; p.sv = sv;
    p.seqlens = seqlens;
    p.B = B; p.H = H; p.n = L_max; p.d = d;
    p.in = in; p.out = out;
    p.causal = 1;
    p.lambda = lambda; p.scale = scale;
    p.ws = workspace; p.ws_bytes = workspace_bytes;
    p.stream = static_cast<hipStream_t>(stream);

    const bool has_mfma = llla::mfma_decode_supported(d, in) && llla::mfma_decode_takes(p);
    if (path == LLLA_PATH_MFMA && !has_mfma) return LLLA_ERR_UNSUPPORTED;
    const bool use_mfma = has_mfma && path != LLLA_PATH_VALU;
    if (use_mfma) {
        st = check_workspace(llla::mfma_decode_workspace_bytes(B, H, L_max, d, in), workspace, workspace_bytes);
        if (st != LLLA_OK) return st;
    }
    llla::stage_begin(p.stream);
    if (!use_mfma) llla::stage_mark(p.stream, "valu_decode");
    const hipError_t e = use_mfma ? llla::mfma_decode(p) : llla::valu_decode(p);
    llla::stage_end(p.stream);
    return e == hipSuccess ? LLLA_OK : LLLA_ERR_LAUNCH;
}

llla_status llla_decode(const void *q, const void *Kc, const void *Vc, void *o, llla_strides sk, llla_strides sv,
                        const int32_t *seqlens, int B, int H, int L_max, int d, llla_dtype in, llla_dtype out,
                        float lambda, float scale, void *workspace, size_t workspace_bytes, void *stream)
{
    return llla_decode_path(q, Kc, Vc, o, sk, sv, seqlens, B, H, L_max, d, in, out, lambda, scale,
                            LLLA_PATH_AUTO, workspace, workspace_bytes, stream);
}

const char *llla_status_string(llla_status s)
{
    switch (s) {
        case LLLA_OK: return "ok";
        case LLLA_ERR_NULL: return "a required pointer is NULL";
        case LLLA_ERR_SHAPE: return "bad shape or stride";
        case LLLA_ERR_DTYPE: return "unknown dtype";
        case LLLA_ERR_PARAM: return "lambda must be finite and > 0, scale finite, path valid";
        case LLLA_ERR_ALIGN: return "pointers and strides must keep rows 16-byte aligned";
        case LLLA_ERR_WORKSPACE: return "workspace missing, unaligned or too small";
        case LLLA_ERR_UNSUPPORTED: return "unsupported head dimension or path";
        case LLLA_ERR_LAUNCH: return "HIP launch failed";
    }
    return "unknown status";
}

const char *llla_version(void) { return "0.1.0"; }

}  // extern "C"

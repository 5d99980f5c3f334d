// Shared declarations of the gfx950 Local Linear Attention library (host + device).
// Nothing here is used by, or shared with, the CPU oracle.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "llla.h"

namespace llla {

// One forward or decode problem, as validated by the C ABI layer.
struct Problem {
    const void *Q, *K, *V;     // forward: [B,H,n,d]; decode: Q = q [B,H,d], K/V = caches [B,H,n,d]
    void *O;                   // forward: [B,H,n,d]; decode: [B,H,d]
    llla_strides sq, sk, sv, so;
    const int32_t *seqlens;    // decode only (device, [B]) or nullptr
    int B, H, n, d;            // n = sequence length (forward) or L_max (decode)
    llla_dtype in, out;
    int causal;
    int live_d;                // forward on zero-padded copies: features [live_d, d) are zero in Q and K; 0 = none are
    float lambda, scale;
    const float *lambda_rows;  // forward only: [B,H,n] ridge per query row, or nullptr (then `lambda` for all rows)
    float *rho, *delta;        // forward only: optional outputs [B,H,n,d] and [B,H,n] (Eq. (lla)), or nullptr
    void *ws;
    size_t ws_bytes;
    hipStream_t stream;
};

// One backward problem (causal), as validated by the C ABI layer.  Gradients are fp32, contiguous.
struct BackwardProblem {
    const void *Q, *K, *V, *dO;  // [B,H,n,d] in dtype `in`
    llla_strides sq, sk, sv, sdo;
    float *dQ, *dK, *dV;         // [B,H,n,d]
    float *dlambda;              // [B,H,n] or nullptr
    int B, H, n, d;
    int live_d;                  // on zero-padded copies: features [live_d, d) of Q and K are zero; 0 = none are
    llla_dtype in;
    float lambda, scale;
    const float *lambda_rows;    // [B,H,n] or nullptr
    void *ws;
    size_t ws_bytes;
    hipStream_t stream;
};

// Launchers return hipSuccess or the launch error.  Each lives in its own translation unit.
hipError_t valu_forward(const Problem &p);
// sweep 3 only, for query rows [0, nrows): y (pitch ypitch floats: y1 then y0) and the row maxima (log2
// units) come from device memory
hipError_t valu_forward_given(const Problem &p, int nrows, const float *M, int mpitch, const float *Y, int ypitch);
hipError_t valu_decode(const Problem &p);

// Queries that see at most dual_max_keys(d) = min(d, DUAL_MAX_KEYS) keys: fp64, key-space form of the same minimiser
// (llla_dual.hip).  dual_forward() serves rows [0, dual_forward_rows(p)) of a forward call (O, and rho / delta when
// asked for); dual_decode() serves the sequences of a decode call that are short enough and leaves the others alone.
constexpr int DUAL_MAX_KEYS = 64;
int dual_max_keys(int d);
int dual_forward_rows(const Problem &p);
hipError_t dual_forward(const Problem &p);
hipError_t dual_decode(const Problem &p);

size_t valu_backward_workspace_bytes(int B, int H, int n, int d);
hipError_t valu_backward(const BackwardProblem &p);
// backward with the matrix-core moments and solve (bf16, d = 64 / 128): workspace layout and the two MFMA stages
struct BackwardLayout {
    size_t fwd;        // the forward's workspace (re-tiled K, V; row maxima M; y rows)
    size_t u, r, sc;   // u rows and r rows (pitch ypitch floats: vector then scalar), row scalars (8 floats per row)
    size_t total;
    int npad;          // pitch of the row maxima (log2 units), in floats
    int ypitch;        // pitch of a y / u / r row, in floats
    size_t m, y;       // offsets of M and of the y rows inside the forward's workspace
};
BackwardLayout mfma_backward_layout(int B, int H, int n, int d);
hipError_t mfma_backward_rowmax(const BackwardProblem &p, const BackwardLayout &L);   // re-tiling and row maxima
hipError_t mfma_backward_solve(const BackwardProblem &p, const BackwardLayout &L);    // moments, y and u of every row
hipError_t mfma_backward_r(const BackwardProblem &p, const BackwardLayout &L, int first_row);   // r rows, argmax; rows >= first_row
hipError_t mfma_backward_dq(const BackwardProblem &p, const BackwardLayout &L, int first_row);  // dQ, dlambda, row scalars; rows >= first_row
hipError_t mfma_backward_keys(const BackwardProblem &p, const BackwardLayout &L);     // dK, dV from y, u and the row scalars
size_t backward_workspace_bytes(int B, int H, int n, int d, llla_dtype in, llla_path path);
hipError_t backward(const BackwardProblem &p, llla_path path);

// MFMA (matrix-core) paths; *_supported() says whether one exists for the shape and dtype.
bool mfma_forward_supported(int d, llla_dtype in, bool causal);
size_t mfma_forward_workspace_bytes(int B, int H, int n, int d, llla_dtype in);
hipError_t mfma_forward(const Problem &p);
// the same for fp32 inputs (d = 64, causal): fp32 MFMA throughout (llla_mfma_fwd_f32.hip)
bool mfma_forward_f32_supported(int d, bool causal);
size_t mfma_forward_f32_workspace_bytes(int B, int H, int n);
hipError_t mfma_forward_f32(const Problem &p);
// head dimensions 16 and 32 (bf16 or fp32): the d = 64 matrix-core forward on zero-padded copies (llla_pad.hip)
bool padded_forward_supported(int d, llla_dtype in);
size_t padded_forward_workspace_bytes(int B, int H, int n, int d, llla_dtype in);
hipError_t padded_forward(const Problem &p);
size_t padded_forward_cg_workspace_bytes(int B, int H, int n, int d, llla_dtype in);   // bf16 only, like the mode itself
hipError_t padded_forward_cg(const Problem &p, int T, float eps, int32_t *iters);
bool padded_backward_supported(int d, llla_dtype in);          // bf16 only, like the matrix-core backward itself
size_t padded_backward_workspace_bytes(int B, int H, int n, int d, llla_dtype in);
hipError_t padded_backward(const BackwardProblem &p);
// approximate mode: T conjugate-gradient steps per row (bf16, d = 64 / 128, causal); iters: [B,H,n] steps done, or nullptr
size_t mfma_forward_cg_workspace_bytes(int B, int H, int n, int d, llla_dtype in);
hipError_t mfma_forward_cg(const Problem &p, int T, float eps, int32_t *iters);
bool mfma_decode_supported(int d, llla_dtype in);
size_t mfma_decode_workspace_bytes(int B, int H, int L_max, int d, llla_dtype in);
// whether the MFMA decode path serves this call (it needs the full cache length for every sequence)
bool mfma_decode_takes(const Problem &p);
hipError_t mfma_decode(const Problem &p);
// the d = 128 kernels behind the two functions above (a translation unit of their own)
size_t mfma_decode128_workspace_bytes(int B, int H, int L_max);
hipError_t mfma_decode128(const Problem &p);

// ---- stage hooks ---------------------------------------------------------------------------------
// stage_mark(stream, name) labels the work enqueued AFTER it, up to the next mark; stage_begin() starts a new call,
// stage_end() closes the last stage.  In the production library they compile to nothing.  The measurement build
// (-DLLLA_MEASURE, a library of its own) records HIP events there so that a benchmark can time each kernel of a call.
#ifdef LLLA_MEASURE
void stage_begin(hipStream_t stream);
void stage_mark(hipStream_t stream, const char *name);
void stage_end(hipStream_t stream);
#else
inline void stage_begin(hipStream_t) {}
inline void stage_mark(hipStream_t, const char *) {}
inline void stage_end(hipStream_t) {}
#endif

// ---- storage types -----------------------------------------------------------------------------
// bf16 is handled as raw uint16_t bits; conversions are written out so that rounding is explicit.
typedef uint16_t bf16_t;

__host__ __device__ inline float bf16_to_f32(bf16_t x)
{
    union { uint32_t u; float f; } c;
    c.u = (uint32_t)x << 16;
    return c.f;
}

// round-to-nearest-even; NaN stays NaN (quiet)
__host__ __device__ inline bf16_t f32_to_bf16(float f)
{
    union { uint32_t u; float f; } c;
    c.f = f;
    if ((c.u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((c.u >> 16) | 0x40);
    c.u += 0x7fffu + ((c.u >> 16) & 1u);
    return (bf16_t)(c.u >> 16);
}

__host__ __device__ inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace llla

// Device helpers shared by the matrix-core (MFMA) kernels of the gfx950 LLA library: vector types,
// MFMA wrappers, DPP broadcasts, LDS DMA, and the on-chip exact solve of the per-query system.
#pragma once

#include "llla_common.hpp"

namespace llla {
namespace mfma {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int KB = 32;         // keys per workspace tile / MFMA step
constexpr float LOG2E = 1.4426950408889634f;

// Shape of the matrix-core kernels for head dimension DD (64 or 128).  The second moment of one
// query is NTILE upper-triangular 16x16 fp32 tiles = 4*NTILE accumulator registers per lane, which
// fixes how many queries a wave can carry: 4 at d = 64 (160 registers), 1 at d = 128 (144).
template <int DD>
struct Shape {
    static constexpr int D = DD;
    static constexpr int NB = DD / 16;                 // 16-wide feature blocks
    static constexpr int NTILE = NB * (NB + 1) / 2;    // upper-triangular tiles
    static constexpr int NF = DD / 32;                 // 32-feature steps of a logits MFMA chain
    static constexpr int QW = (DD == 64) ? 4 : 1;      // queries per wave (moments kernel)
    static constexpr int NW = NB;                      // waves per workgroup (moments kernel): one mu~ block each
    static constexpr int QB = QW * NW;                 // queries per workgroup (moments kernel)
    static constexpr int NT = 64 * NW;                 // threads per workgroup (moments kernel)
    static constexpr int YP = DD + 16;                 // pitch of a y row in the workspace: y1[0..D), y0 at [D]; rows start on 64-byte boundaries
    static constexpr int EARLY_ROWS = 2 * DD;          // rows served by the precise variant
    __host__ __device__ static constexpr int tix(int I, int J) { return I * NB - I * (I - 1) / 2 + (J - I); }
};

// Which (batch-head, block) a workgroup serves in a grid (blocks, heads).  Workgroups are handed to the 8 XCDs (each
// with an L2 of its own) round-robin in dispatch order, blockIdx.x fastest.  With the plain mapping the neighbouring
// blocks of one head land on all 8 XCDs and every L2 fetches that head's tiles for itself.  Here a group of 8 heads
// is spread over the 8 XCDs, one head per XCD, and an XCD walks through the blocks of its head in the order given
// (callers put the longest first) before the next group of heads starts: each head's tiles are fetched by one L2
// only.  Heads beyond the last full group of 8 keep the plain mapping.  Used by the moments kernels (16 or 8 rows per
// workgroup, hundreds of workgroups per head).  The 64-row sweeps do not use it: all blocks of a head fit an XCD at
// once, they would start together and the XCD would wait for the longest; those kernels put the head on blockIdx.x.
struct BlockMap { int bh, blk; };
__device__ inline BlockMap xcd_block_map()
{
    const int nblk = (int)gridDim.x, nbh = (int)gridDim.y;
    const long long lin = (long long)blockIdx.y * nblk + blockIdx.x;
    const long long grouped = (long long)(nbh & ~7) * nblk;
    if (lin >= grouped) return BlockMap{(int)blockIdx.y, (int)blockIdx.x};
    const int xcd = (int)(lin & 7);
    const long long k = lin >> 3;
    return BlockMap{(int)(k / nblk) * 8 + xcd, (int)(k % nblk)};
}

// Row broadcasts across the 16-lane rows of a wave: rows 1 and 3 receive lane 15 of rows 0 and 2 (the other rows
// keep x); rows 2 and 3 receive lane 31, the last lane of row 1 (rows 0 and 1 keep x).
__device__ inline float rows_1_3_from_rows_0_2(float x)
{
    const int v = __builtin_bit_cast(int, x);
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(v, v, 0x142, 0xa, 0xf, false));
}
__device__ inline float rows_2_3_from_row_1(float x)
{
    const int v = __builtin_bit_cast(int, x);
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(v, v, 0x143, 0xc, 0xf, false));
}

// Maximum of x[p * pitch], p in [p0, p1), over a wave: lane l takes p0 + l, p0 + l + 64, .., so the loads of a
// wave are in flight together (a loop over p in every lane would wait for each load in turn).
__device__ inline float wave_max_strided(const float *x, int p0, int p1, size_t pitch, int lane)
{
    float mv = -INFINITY;
    for (int p = p0 + lane; p < p1; p += 64) mv = fmaxf(mv, x[(size_t)p * pitch]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mv = fmaxf(mv, __shfl_xor(mv, off));
    return mv;
}

__device__ inline void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

template <int C>
__device__ inline float row_bcast(float x)   // value of lane C of the caller's 16-lane row
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x150 + C, 0xf, 0xf, true));
}
template <int J>
__device__ inline float quad_bcast(float x)   // value of lane (lane & ~3) + J
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), J * 0x55, 0xf, 0xf, true));
}
__device__ inline float lane_xor1(float x)   // value of lane ^ 1
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xf, 0xf, true));
}

// x = hi + lo with both halves f16 (about 20 significant bits).  hi is x rounded toward zero by a conversion
// builtin on purpose: a plain (_Float16) cast of a product may be fused with the multiply at one use (one
// rounding of the exact product) and not at another (product rounded to fp32 first), the two results can differ
// by one f16 ulp, and a lo computed against the one would then be added to the other.
__device__ inline void split_f16(const float (&x)[8], half8 &hi, half8 &lo)
{
    typedef __fp16 fp16x2 __attribute__((ext_vector_type(2)));
    typedef _Float16 half2v __attribute__((ext_vector_type(2)));
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const half2v h = __builtin_bit_cast(half2v, (fp16x2)__builtin_amdgcn_cvt_pkrtz(x[2 * p], x[2 * p + 1]));
        const half2v l = __builtin_bit_cast(
            half2v, (fp16x2)__builtin_amdgcn_cvt_pkrtz(x[2 * p] - (float)h[0], x[2 * p + 1] - (float)h[1]));
        hi[2 * p] = h[0]; hi[2 * p + 1] = h[1];
        lo[2 * p] = l[0]; lo[2 * p + 1] = l[1];
    }
}

__device__ inline f32x4 mfma_f16(half8 a, half8 b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0); }
__device__ inline f32x4 mfma_bf16(bf16x8 a, bf16x8 b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0); }

// C += A^T B for 16x16 fp32 tiles held in the MFMA accumulator layout (lane (g,n), reg t = X[4g+t][n]).
// The contraction slot (chunk kc, lane group g) is mapped to index 4g+kc, which is exactly where
// register kc of both tiles sits, so no data moves.
__device__ inline f32x4 tile_atb(f32x4 c, f32x4 a, f32x4 b)
{
#pragma unroll
    for (int kc = 0; kc < 4; ++kc) c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[kc], b[kc], c, 0, 0, 0);
    return c;
}

constexpr int SC_PITCH = 20;         // floats per row of a 16x16 scratch tile

// Row-broadcast multiply-adds as VOP2 DPP instructions, a_i += (src of lane C_i of the 16-lane row) * mul:
// the compiler does not fuse a DPP move into an FMA by itself, and these pairs are most of the vector-ALU
// work of the diagonal-tile factorisation.  A DPP read needs two wait states after a vector-ALU write of the
// register it reads, and the compiler's hazard handling does not look inside inline assembly; every
// statement below therefore starts with its own s_nop 1, and all registers it reads through DPP are operands
// of the statement, so whatever wrote them lies before that s_nop.
//   fmac_bcastN<C0..>(a0.., src, mul): a_i += bcast_{C_i}(src) * mul        (rank-1 update of a row)
//   fmac_selfN<C>(a0.., mul):          a_i += bcast_C(a_i) * mul            (triangular-inverse recursion)
template <int C0>
__device__ inline void fmac_bcast1(float &a0, float src, float mul)
{
    asm volatile("s_nop 1\n\t"
                 "v_fmac_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf bound_ctrl:1"
                 : "+v"(a0) : "v"(src), "v"(mul), "n"(C0));
}
template <int C0, int C1>
__device__ inline void fmac_bcast2(float &a0, float &a1, float src, float mul)
{
    asm volatile("s_nop 1\n\t"
                 "v_fmac_f32_dpp %0, %2, %3 row_newbcast:%4 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                 "v_fmac_f32_dpp %1, %2, %3 row_newbcast:%5 row_mask:0xf bank_mask:0xf bound_ctrl:1"
                 : "+v"(a0), "+v"(a1) : "v"(src), "v"(mul), "n"(C0), "n"(C1));
}
template <int C0, int C1, int C2, int C3>
__device__ inline void fmac_bcast4(float &a0, float &a1, float &a2, float &a3, float src, float mul)
{
    asm volatile("s_nop 1\n\t"
                 "v_fmac_f32_dpp %0, %4, %5 row_newbcast:%6 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                 "v_fmac_f32_dpp %1, %4, %5 row_newbcast:%7 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                 "v_fmac_f32_dpp %2, %4, %5 row_newbcast:%8 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                 "v_fmac_f32_dpp %3, %4, %5 row_newbcast:%9 row_mask:0xf bank_mask:0xf bound_ctrl:1"
                 : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3) : "v"(src), "v"(mul), "n"(C0), "n"(C1), "n"(C2), "n"(C3));
}
template <int C0, int C1, int C2, int C3, int C4, int C5, int C6, int C7>
__device__ inline void fmac_bcast8(float &a0, float &a1, float &a2, float &a3, float &a4, float &a5, float &a6, float &a7, float src, float mul)
{
    asm volatile("s_nop 1\n\t"
                 "v_fmac_f32_dpp %0, %8, %9 row_newbcast:%10 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                 "v_fmac_f32_dpp %1, %8, %9 row_newbcast:%11 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                 "v_fmac_f32_dpp %2, %8, %9 row_newbcast:%12 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                 "v_fmac_f32_dpp %3, %8, %9 row_newbcast:%13 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                 "v_fmac_f32_dpp %4, %8, %9 row_newbcast:%14 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                 "v_fmac_f32_dpp %5, %8, %9 row_newbcast:%15 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                 "v_fmac_f32_dpp %6, %8, %9 row_newbcast:%16 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                 "v_fmac_f32_dpp %7, %8, %9 row_newbcast:%17 row_mask:0xf bank_mask:0xf bound_ctrl:1"
                 : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7) : "v"(src), "v"(mul), "n"(C0), "n"(C1), "n"(C2), "n"(C3), "n"(C4), "n"(C5), "n"(C6), "n"(C7));
}
template <int C>
__device__ inline void fmac_self1(float &a0, float mul)
{
    asm volatile("s_nop 1\n\t"
                 "v_fmac_f32_dpp %0, %0, %1 row_newbcast:%2 row_mask:0xf bank_mask:0xf bound_ctrl:1"
                 : "+v"(a0) : "v"(mul), "n"(C));
}
template <int C>
__device__ inline void fmac_self2(float &a0, float &a1, float mul)
{
    asm volatile("s_nop 1\n\t"
                 "v_fmac_f32_dpp %0, %0, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                 "v_fmac_f32_dpp %1, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf bound_ctrl:1"
                 : "+v"(a0), "+v"(a1) : "v"(mul), "n"(C));
}
template <int C>
__device__ inline void fmac_self4(float &a0, float &a1, float &a2, float &a3, float mul)
{
    asm volatile("s_nop 1\n\t"
                 "v_fmac_f32_dpp %0, %0, %4 row_newbcast:%5 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                 "v_fmac_f32_dpp %1, %1, %4 row_newbcast:%5 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                 "v_fmac_f32_dpp %2, %2, %4 row_newbcast:%5 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                 "v_fmac_f32_dpp %3, %3, %4 row_newbcast:%5 row_mask:0xf bank_mask:0xf bound_ctrl:1"
                 : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3) : "v"(mul), "n"(C));
}
template <int C>
__device__ inline void fmac_self8(float &a0, float &a1, float &a2, float &a3, float &a4, float &a5, float &a6, float &a7, float mul)
{
    asm volatile("s_nop 1\n\t"
                 "v_fmac_f32_dpp %0, %0, %8 row_newbcast:%9 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                 "v_fmac_f32_dpp %1, %1, %8 row_newbcast:%9 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                 "v_fmac_f32_dpp %2, %2, %8 row_newbcast:%9 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                 "v_fmac_f32_dpp %3, %3, %8 row_newbcast:%9 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                 "v_fmac_f32_dpp %4, %4, %8 row_newbcast:%9 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                 "v_fmac_f32_dpp %5, %5, %8 row_newbcast:%9 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                 "v_fmac_f32_dpp %6, %6, %8 row_newbcast:%9 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                 "v_fmac_f32_dpp %7, %7, %8 row_newbcast:%9 row_mask:0xf bank_mask:0xf bound_ctrl:1"
                 : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7) : "v"(mul), "n"(C));
}
template <int C>
__device__ inline float bcast_settled(float src)     // row broadcast of a value that inline assembly may have written
{
    float d;
    asm volatile("s_nop 1\n\tv_mov_b32_dpp %0, %1 row_newbcast:%2 row_mask:0xf bank_mask:0xf bound_ctrl:1"
                 : "=v"(d) : "v"(src), "n"(C));
    return d;
}

// a[K+1..15] += bcast_c(src) * mul for c = K+1..15, in statements of 8, 4, 2 and 1 instructions
template <int K>
__device__ inline void rank1_row(float (&a)[16], float src, float mul)
{
    constexpr int N = 15 - K;
    constexpr int c8 = K + 1, c4 = c8 + (N & 8), c2 = c4 + (N & 4), c1 = c2 + (N & 2);
    if constexpr ((N & 8) != 0)
        fmac_bcast8<c8, c8 + 1, c8 + 2, c8 + 3, c8 + 4, c8 + 5, c8 + 6, c8 + 7>(a[c8], a[c8 + 1], a[c8 + 2], a[c8 + 3], a[c8 + 4], a[c8 + 5],
                                                                                a[c8 + 6], a[c8 + 7], src, mul);
    if constexpr ((N & 4) != 0) fmac_bcast4<c4, c4 + 1, c4 + 2, c4 + 3>(a[c4], a[c4 + 1], a[c4 + 2], a[c4 + 3], src, mul);
    if constexpr ((N & 2) != 0) fmac_bcast2<c2, c2 + 1>(a[c2], a[c2 + 1], src, mul);
    if constexpr ((N & 1) != 0) fmac_bcast1<c1>(a[c1], src, mul);
}
// li[0..P] += bcast_P(li[c]) * mul
template <int P>
__device__ inline void trinv_row(float (&li)[16], float mul)
{
    constexpr int N = P + 1;
    constexpr int c8 = 0, c4 = c8 + (N & 8), c2 = c4 + (N & 4), c1 = c2 + (N & 2);
    if constexpr ((N & 8) != 0) fmac_self8<P>(li[c8], li[c8 + 1], li[c8 + 2], li[c8 + 3], li[c8 + 4], li[c8 + 5], li[c8 + 6], li[c8 + 7], mul);
    if constexpr ((N & 4) != 0) fmac_self4<P>(li[c4], li[c4 + 1], li[c4 + 2], li[c4 + 3], mul);
    if constexpr ((N & 2) != 0) fmac_self2<P>(li[c2], li[c2 + 1], mul);
    if constexpr ((N & 1) != 0) fmac_self1<P>(li[c1], mul);
}

#define LLLA_SWITCH16(K, STMT)                                                                          \
    switch (K) {                                                                                        \
        case 0: { constexpr int KK = 0; STMT; } break;   case 1: { constexpr int KK = 1; STMT; } break;    \
        case 2: { constexpr int KK = 2; STMT; } break;   case 3: { constexpr int KK = 3; STMT; } break;    \
        case 4: { constexpr int KK = 4; STMT; } break;   case 5: { constexpr int KK = 5; STMT; } break;    \
        case 6: { constexpr int KK = 6; STMT; } break;   case 7: { constexpr int KK = 7; STMT; } break;    \
        case 8: { constexpr int KK = 8; STMT; } break;   case 9: { constexpr int KK = 9; STMT; } break;    \
        case 10: { constexpr int KK = 10; STMT; } break; case 11: { constexpr int KK = 11; STMT; } break;  \
        case 12: { constexpr int KK = 12; STMT; } break; case 13: { constexpr int KK = 13; STMT; } break;  \
        case 14: { constexpr int KK = 14; STMT; } break; default: { constexpr int KK = 15; STMT; } break;  \
    }

// Upper Cholesky factor and its inverse for the diagonal tiles of the wave's four queries at once:
// lane 16q + r owns row r of query q's symmetric 16x16 tile (a[c] = T[r][c]).  On return
// li[c] = -(L^{-1})[r][c] with T = L L^T (zero above the diagonal); the sign is the one factorise_wave wants.
// pivot_floor: every pivot of the Cholesky factorisation of (a positive semi-definite matrix + lambda I) is
// at least lambda in exact arithmetic; a computed pivot below the floor (half of lambda) is a rounding
// artefact of an ill-conditioned early row and is raised to it, which keeps the factorisation finite.
__device__ inline void chol_inv16(float (&a)[16], float (&li)[16], int r, float pivot_floor)
{
    float nl2[16];      // -L[r][k] / L[k][k]  (column-scaled factor, strictly lower part kept, negated)
    float dinv_own = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        float dk;
        const float ak = a[k];
        LLLA_SWITCH16(k, dk = bcast_settled<KK>(ak));        // diagonal entry of step k, from lane k of the row
        dk = fmaxf(dk, pivot_floor);
        float rinv = __builtin_amdgcn_rsqf(dk);
        rinv = rinv * (1.5f - 0.5f * dk * rinv * rinv);      // one Newton step
        const float u = ak * rinv;                           // L[r][k] in rows r >= k; rows above are finished and never read again
        const float nu = -u;
        nl2[k] = (r > k) ? nu * rinv : 0.f;
        dinv_own = (r == k) ? rinv : dinv_own;
        if (k < 15) { LLLA_SWITCH16(k, rank1_row<(KK < 15 ? KK : 14)>(a, u, nu)); }      // a[c] -= L[r][k] L[c][k], c > k
    }
    // M = (unit lower L'')^{-1}:  M[r][c] = [r==c] - sum_{c<=p<r} L''[r][p] M[p][c]
#pragma unroll
    for (int c = 0; c < 16; ++c) li[c] = (r == c) ? 1.f : 0.f;
#pragma unroll
    for (int p = 0; p < 15; ++p) { LLLA_SWITCH16(p, trinv_row<(KK < 15 ? KK : 14)>(li, nl2[p])); }
    const float ndinv = -dinv_own;
#pragma unroll
    for (int c = 0; c < 16; ++c) li[c] *= ndinv;             // -L^{-1} = -D^{-1} L''^{-1}
}
#undef LLLA_SWITCH16

typedef __attribute__((address_space(3))) void *lds_void_ptr;
typedef const __attribute__((address_space(1))) void *glb_void_ptr;

// 16 bytes per lane straight from global memory into LDS (no registers): lane l's data lands at
// lds_base + 16 l, the global address is per lane.  Written as inline assembly on purpose: the
// compiler makes every later LDS read wait for a DMA it knows about (it cannot tell the two
// buffers apart), which would serialise the prefetch; here the waits are placed by hand with
// dma_wait() before the data is read.  The s_nop is the wait state gfx9 needs between a scalar
// write of M0 and an LDS-DMA instruction that reads it.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ inline void dma16(const void *gsrc, void *lds_base)
{
    const unsigned lds = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(lds_void_ptr)lds_base);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gsrc), "s"(lds) : "memory", "m0");
}
// The same with a wave-uniform base address in scalar registers plus a 32-bit per-lane byte offset: no vector-ALU
// address arithmetic per transfer.
__device__ inline void dma16_base(const void *sbase, unsigned voff, void *lds_base)
{
    const unsigned lds = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(lds_void_ptr)lds_base);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds) : "memory", "m0");
}
// The same with the LDS destination given as a byte offset into the workgroup's LDS (lds_offset of the array plus
// plain integer arithmetic): a pointer that went through pointer arithmetic in the generic address space costs four
// scalar instructions per transfer to turn back into an LDS address.
__device__ inline unsigned lds_offset(const void *lds_object) { return (unsigned)(uintptr_t)(lds_void_ptr)lds_object; }
__device__ inline void dma16_base_off(const void *sbase, unsigned voff, unsigned lds_byte_off)
{
    const unsigned lds = __builtin_amdgcn_readfirstlane(lds_byte_off);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds) : "memory", "m0");
}
// The same two transfers with the non-temporal hint, for data that is read exactly once (the decode kernel's cache
// stream): without it the stream stays about 10 % below what plain streaming loads reach on this part.
__device__ inline void dma16_nt(const void *gsrc, void *lds_base)
{
    const unsigned lds = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(lds_void_ptr)lds_base);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt" ::"v"(gsrc), "s"(lds) : "memory", "m0");
}
__device__ inline void dma16_base_nt(const void *sbase, unsigned voff, void *lds_base)
{
    const unsigned lds = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(lds_void_ptr)lds_base);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt" ::"v"(voff), "s"(sbase), "s"(lds) : "memory", "m0");
}
// (and with the LDS destination as a byte offset, see dma16_base_off)
__device__ inline void dma16_nt_off(const void *gsrc, unsigned lds_byte_off)
{
    const unsigned lds = __builtin_amdgcn_readfirstlane(lds_byte_off);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt" ::"v"(gsrc), "s"(lds) : "memory", "m0");
}
__device__ inline void dma16_base_nt_off(const void *sbase, unsigned voff, unsigned lds_byte_off)
{
    const unsigned lds = __builtin_amdgcn_readfirstlane(lds_byte_off);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt" ::"v"(voff), "s"(sbase), "s"(lds) : "memory", "m0");
}
#pragma clang diagnostic pop
__device__ inline void dma_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Blocked factorisation of the wave's QW systems, all in registers / wave-private LDS scratch (the first half of the
// per-query solve; the substitutions are solve_wave_q4 at d = 64 and solve_wave_v1 at d = 128):
//   in : acc[q][tix(I,J)]  upper-triangular 16x16 tiles of T_q = -(Sigma~_q + lambda I) (MFMA accumulator layout)
//        scw               >= QW*16*SC_PITCH floats of LDS owned by this wave
//        pivot_floor       per lane: half the ridge of the query of the lane's group (see chol_inv16)
//   out: acc(P,J), P < J, holds U(P,J) and acc(P,P) holds N_P = -U(P,P)^{-1}, with Sigma~ + lambda I = U^T U.
// 16-blocked upper Cholesky whose block products are C += A^T B on fp32 MFMA; the diagonal tiles of the QW queries
// are factorised together in (query, row) lanes with DPP row broadcasts.  The matrix cores only add products, so
// everything that the textbook recursion subtracts is carried negated instead: the trailing matrix (T), the inverse
// diagonal factors (N_P), and, in the substitutions, the partial right-hand sides; no tile is ever negated on the
// vector ALU.
template <int DD>
__device__ __forceinline__ void factorise_wave(f32x4 (&acc)[Shape<DD>::QW][Shape<DD>::NTILE], float *scw, int g, int nn,
                                               float pivot_floor)
{
    using S = Shape<DD>;
    constexpr int QW = S::QW, NB = S::NB;
    const int gq = (g < QW) ? g : QW - 1;       // lane groups beyond the wave's queries shadow the last one
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int P = 0; P < NB; ++P) {
        // diagonal tiles -> (query, row) lanes, symmetrised
#pragma unroll
        for (int q = 0; q < QW; ++q)
#pragma unroll
            for (int t = 0; t < 4; ++t) scw[q * 16 * SC_PITCH + (4 * g + t) * SC_PITCH + nn] = acc[q][S::tix(P, P)][t];
        wave_sync();
        float a[16], li[16];
        {
            const float *my = scw + gq * 16 * SC_PITCH;
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
        if (g < QW) {
            float *my = scw + g * 16 * SC_PITCH;
#pragma unroll
            for (int c4 = 0; c4 < 4; ++c4)
                *reinterpret_cast<f32x4 *>(my + nn * SC_PITCH + 4 * c4) = f32x4{li[4 * c4], li[4 * c4 + 1], li[4 * c4 + 2], li[4 * c4 + 3]};
        }
        wave_sync();
#pragma unroll
        for (int q = 0; q < QW; ++q) {
            // N_P in tile layout: reg t = N[4g+t][nn] = -Linv[nn][4g+t]; it replaces the consumed diagonal tile;
            // U(P,J) = N_P^T T(P,J), and the trailing tiles take T(I,J) += U(P,I)^T U(P,J)
            const f32x4 ui = *reinterpret_cast<const f32x4 *>(scw + q * 16 * SC_PITCH + nn * SC_PITCH + 4 * g);
            acc[q][S::tix(P, P)] = ui;
#pragma unroll
            for (int J = P + 1; J < NB; ++J) acc[q][S::tix(P, J)] = tile_atb(zero, ui, acc[q][S::tix(P, J)]);
#pragma unroll
            for (int I = P + 1; I < NB; ++I)
#pragma unroll
                for (int J = I; J < NB; ++J) acc[q][S::tix(I, J)] = tile_atb(acc[q][S::tix(I, J)], acc[q][S::tix(P, I)], acc[q][S::tix(P, J)]);
            // one query at a time: its own tile products give the matrix cores enough independent work, and
            // interleaving the queries only inflates the number of live registers
            __builtin_amdgcn_sched_barrier(0);
        }
        wave_sync();
    }

}


}  // namespace mfma
}  // namespace llla

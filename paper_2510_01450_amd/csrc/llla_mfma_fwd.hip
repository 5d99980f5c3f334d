// Matrix-core (MFMA) forward path of Local Linear Attention for gfx950: bf16 inputs, d = 64.
//
// Stages (all on the caller's stream, workspace holds only Theta(B*H*n*d) data):
//   prep    K -> f16, V -> bf16, both re-tiled as [key block of 32][feature][key] so that MFMA
//           operands whose contraction index is the key are 16-byte contiguous;
//   rowmax  m_i = max_{j<=i} c <q_i,k_j>  (c = scale*log2 e), the exact row maximum that the
//           running maximum of Algorithm 1 ends at;
//   moments per block of 16 queries: weights w_ij = 2^(c<q_i,k_j> - m_i), the un-centred moments
//           omega_i, mu~_i, Sigma~_i of Eq. (tilded_form) accumulated ON CHIP as MFMA accumulators
//           (Sigma~_i: upper triangle of 16x16 tiles), then the exact per-query solve of
//           [omega mu~^T; mu~ Sigma~ + lambda I] y = [1; q] by a 16-blocked Cholesky whose block
//           products run on fp32 MFMA; only y_i (d+1 floats) and m_i leave the chip;
//   output  s_ij = w_ij (y0_i + k_j . y1_i), O = S V  (Eq. (lla) with y1 = -rho/delta,
//           y0 = (1 + q.rho)/delta), a flash-style sweep.
// The first 4d rows of every sequence, whose systems are the worst conditioned, are served by the
// fp32 vector-ALU kernel instead (same result, higher-precision second moment).
#include "llla_common.hpp"

namespace llla {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int D = 64;          // head dimension of this path
constexpr int KB = 32;         // keys per block
constexpr int NT = 256;        // threads per workgroup (4 waves)
constexpr int QW = 4;          // queries per wave in the moments kernel
constexpr int QB = 16;         // queries per workgroup in the moments kernel
constexpr int YP = D + 4;      // pitch of a y row in the workspace: y1[0..D), y0 at [D]
constexpr int EARLY_ROWS = 4 * D;
constexpr float LOG2E = 1.4426950408889634f;

struct Layout {
    size_t kt, vt, m, y, total;
    int nkb, npad;
};

Layout make_layout(int B, int H, int n)
{
    Layout L;
    L.nkb = 2 * ((n + 2 * KB - 1) / (2 * KB));      // 32-key blocks, an even count
    L.npad = L.nkb * KB;
    const size_t bh = (size_t)B * H;
    size_t off = 0;
    L.kt = off; off += round_up(bh * L.npad * D * 2, 256);
    L.vt = off; off += round_up(bh * L.npad * D * 2, 256);
    L.m = off;  off += round_up(bh * L.npad * 4, 256);
    L.y = off;  off += round_up(bh * (size_t)n * YP * 4, 256);
    L.total = off;
    return L;
}

__device__ inline void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

template <int C>
__device__ inline float row_bcast(float x)   // value of lane C of the caller's 16-lane row
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x150 + C, 0xf, 0xf, false));
}
__device__ inline float lane_xor1(float x)   // value of lane ^ 1
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xf, 0xf, false));
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

__host__ __device__ constexpr int tix(int I, int J) { return I * 4 - I * (I - 1) / 2 + (J - I); }

// ------------------------------------------------------------------------------------------------
// prep: re-tile K (-> f16) and V (bf16) as [bh][key block][feature][32 keys]
__global__ __launch_bounds__(NT) void prep_kernel(const bf16_t *__restrict__ Kg, const bf16_t *__restrict__ Vg,
                                                  llla_strides sk, llla_strides sv, int H, int n, int nkb,
                                                  _Float16 *__restrict__ KT, bf16_t *__restrict__ VT)
{
    __shared__ bf16_t tile[2][KB][D + 2];
    const int blk = blockIdx.x, bh = blockIdx.y, b = bh / H, h = bh % H, tid = threadIdx.x;
    const bf16_t *Kh = Kg + b * sk.batch + h * sk.head;
    const bf16_t *Vh = Vg + b * sv.batch + h * sv.head;
    {
        const int key = tid / 8, ch = (tid % 8) * 8;
        const int j = blk * KB + key;
        uint4 kv = make_uint4(0, 0, 0, 0), vv = kv;
        if (j < n) {
            kv = *reinterpret_cast<const uint4 *>(Kh + (int64_t)j * sk.seq + ch);
            vv = *reinterpret_cast<const uint4 *>(Vh + (int64_t)j * sv.seq + ch);
        }
        const uint32_t ku[4] = {kv.x, kv.y, kv.z, kv.w}, vu[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            tile[0][key][ch + 2 * i] = (bf16_t)(ku[i] & 0xffff);
            tile[0][key][ch + 2 * i + 1] = (bf16_t)(ku[i] >> 16);
            tile[1][key][ch + 2 * i] = (bf16_t)(vu[i] & 0xffff);
            tile[1][key][ch + 2 * i + 1] = (bf16_t)(vu[i] >> 16);
        }
    }
    __syncthreads();
    {
        const int feat = tid / 4, k0 = (tid % 4) * 8;
        half8 ko;
        uint16_t vo[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            ko[i] = (_Float16)bf16_to_f32(tile[0][k0 + i][feat]);
            vo[i] = tile[1][k0 + i][feat];
        }
        const size_t base = ((size_t)bh * nkb + blk) * (D * KB) + feat * KB + k0;
        *reinterpret_cast<half8 *>(KT + base) = ko;
        *reinterpret_cast<uint4 *>(VT + base) = make_uint4(vo[0] | (vo[1] << 16), vo[2] | (vo[3] << 16),
                                                           vo[4] | (vo[5] << 16), vo[6] | (vo[7] << 16));
    }
}

// ------------------------------------------------------------------------------------------------
// Sweep over S^T = K Q^T for 64 queries per workgroup (16 per wave).
//   MAXONLY: write the row maxima m_i (in log2 units) -- Algorithm 1's m after its last block.
//   else   : third loop of Algorithm 1: S = W (y0 + K y1), O = S V.
constexpr int KN_PITCH = D + 8;      // halves; rows of the natural K tile stay 16-byte aligned
constexpr int VT_PITCH = KB + 8;     // halves

template <bool MAXONLY>
__global__ __launch_bounds__(NT) void sweep_kernel(const bf16_t *__restrict__ Qg, const bf16_t *__restrict__ Kg,
                                                   llla_strides sq, llla_strides sk, int H, int n, int nkb,
                                                   int first_row, float cscale, const bf16_t *__restrict__ VT,
                                                   float *__restrict__ Mg, const float *__restrict__ Yg,
                                                   void *__restrict__ Og, llla_strides so, int out_bf16)
{
    __shared__ __align__(16) bf16_t kn[KB * KN_PITCH];
    __shared__ __align__(16) bf16_t vt[MAXONLY ? 8 : D * VT_PITCH];
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64, g = lane / 16, nn = lane % 16;
    const int bh = blockIdx.y, b = bh / H, h = bh % H;
    const int nqb = gridDim.x;
    const int i0 = first_row + (nqb - 1 - (int)blockIdx.x) * 64;      // long rows first
    const int iq = i0 + wave * 16 + nn;                                // this lane's query
    const int iqc = min(iq, n - 1);
    const bf16_t *Kh = Kg + b * sk.batch + h * sk.head;
    const bf16_t *qrow = Qg + b * sq.batch + h * sq.head + (int64_t)iqc * sq.seq;
    bf16x8 qf[2];
    qf[0] = *reinterpret_cast<const bf16x8 *>(qrow + 8 * g);
    qf[1] = *reinterpret_cast<const bf16x8 *>(qrow + 32 + 8 * g);

    float mrow = -INFINITY, y0 = 0.f;
    bf16x8 yh[2], yl[2];
    f32x4 oacc[4];
    if (!MAXONLY) {
        mrow = Mg[(size_t)bh * (nkb * KB) + iqc];
        const float *yr = Yg + ((size_t)bh * n + iqc) * YP;
        y0 = yr[D];
#pragma unroll
        for (int f = 0; f < 2; ++f)
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const float v = yr[32 * f + 8 * g + t];
                const __bf16 hi = (__bf16)v;
                yh[f][t] = hi;
                yl[f][t] = (__bf16)(v - (float)hi);
            }
#pragma unroll
        for (int J = 0; J < 4; ++J) oacc[J] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    float mx[2][4];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int r = 0; r < 4; ++r) mx[s][r] = -INFINITY;

    const int ilast = min(i0 + 63, n - 1);
    const int nblk = ilast / KB + 1;
    for (int c = 0; c < nblk; ++c) {
        __syncthreads();
        {   // stage K (natural) and V^T tiles
            const int key = tid / 8, ch = (tid % 8) * 8;
            const int j = c * KB + key;
            uint4 kv = make_uint4(0, 0, 0, 0);
            if (j < n) kv = *reinterpret_cast<const uint4 *>(Kh + (int64_t)j * sk.seq + ch);
            *reinterpret_cast<uint4 *>(&kn[key * KN_PITCH + ch]) = kv;
            if (!MAXONLY) {
                const int feat = tid / 4, k0 = (tid % 4) * 8;
                const uint4 vv = *reinterpret_cast<const uint4 *>(VT + ((size_t)bh * nkb + c) * (D * KB) + feat * KB + k0);
                *reinterpret_cast<uint4 *>(&vt[feat * VT_PITCH + k0]) = vv;
            }
        }
        __syncthreads();
        f32x4 st[2], ut[2];
#pragma unroll
        for (int s = 0; s < 2; ++s) {       // two sub-tiles of 16 keys
            const bf16x8 k0f = *reinterpret_cast<const bf16x8 *>(&kn[(16 * s + nn) * KN_PITCH + 8 * g]);
            const bf16x8 k1f = *reinterpret_cast<const bf16x8 *>(&kn[(16 * s + nn) * KN_PITCH + 32 + 8 * g]);
            f32x4 z = {0.f, 0.f, 0.f, 0.f};
            z = mfma_bf16(k0f, qf[0], z);
            st[s] = mfma_bf16(k1f, qf[1], z);
            if (!MAXONLY) {
                f32x4 u = {0.f, 0.f, 0.f, 0.f};
                u = mfma_bf16(k0f, yl[0], u);
                u = mfma_bf16(k1f, yl[1], u);
                u = mfma_bf16(k0f, yh[0], u);
                ut[s] = mfma_bf16(k1f, yh[1], u);
            }
        }
        // lane (g, nn): st[s][r] = <k_j, q_iq> for key j = 32c + 16s + 4g + r
        if (MAXONLY) {
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int j = c * KB + 16 * s + 4 * g + r;
                    const float t = st[s][r] * cscale;
                    mx[s][r] = (j <= iq) ? fmaxf(mx[s][r], t) : mx[s][r];
                }
        } else {
            bf16x8 ch, cl;      // output weights as bf16 hi + lo; slot t<4: key 4g+t, t>=4: key 16+4g+t-4
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int j = c * KB + 16 * s + 4 * g + r;
                    const float wgt = __builtin_amdgcn_exp2f(st[s][r] * cscale - mrow);
                    const float cv = (j <= iq) ? wgt * (y0 + ut[s][r]) : 0.f;
                    const __bf16 hi = (__bf16)cv;
                    ch[4 * s + r] = hi;
                    cl[4 * s + r] = (__bf16)(cv - (float)hi);
                }
#pragma unroll
            for (int J = 0; J < 4; ++J) {
                bf16x8 vf;
                const uint2 lo = *reinterpret_cast<const uint2 *>(&vt[(16 * J + nn) * VT_PITCH + 4 * g]);
                const uint2 hi = *reinterpret_cast<const uint2 *>(&vt[(16 * J + nn) * VT_PITCH + 16 + 4 * g]);
                const uint4 pk = make_uint4(lo.x, lo.y, hi.x, hi.y);
                vf = __builtin_bit_cast(bf16x8, pk);
                oacc[J] = mfma_bf16(cl, vf, oacc[J]);
                oacc[J] = mfma_bf16(ch, vf, oacc[J]);
            }
        }
    }

    if (MAXONLY) {
        float m = -INFINITY;
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int r = 0; r < 4; ++r) m = fmaxf(m, mx[s][r]);
        m = fmaxf(m, __shfl_xor(m, 16));
        m = fmaxf(m, __shfl_xor(m, 32));
        if (g == 0 && iq < n) Mg[(size_t)bh * (nkb * KB) + iq] = m;
    } else {
        // oacc[J]: lane (g, nn) reg r = O[query i0 + 16 wave + 4g + r][feature 16J + nn]
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int i = i0 + wave * 16 + 4 * g + r;
            if (i < n) {
                const int64_t off = b * so.batch + h * so.head + (int64_t)i * so.seq;
#pragma unroll
                for (int J = 0; J < 4; ++J) {
                    if (out_bf16) ((bf16_t *)Og)[off + 16 * J + nn] = f32_to_bf16(oacc[J][r]);
                    else ((float *)Og)[off + 16 * J + nn] = oacc[J][r];
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// moments + solve
constexpr int KB2 = 2 * KB;          // keys per pipeline step of the moments kernel
constexpr int WT_PITCH = KB2 + 8;    // halves per query row of the weight tile
constexpr int SC_PITCH = 20;         // floats per row of a 16x16 scratch tile

// Upper Cholesky factor and its inverse for the diagonal tiles of the wave's four queries at once:
// lane 16q + r owns row r of query q's symmetric 16x16 tile (a[c] = T[r][c]).  On return
// li[c] = (L^{-1})[r][c] with T = L L^T (zero above the diagonal).
__device__ inline void chol_inv16(float (&a)[16], float (&li)[16], int r)
{
    float l2[16];       // L[r][k] / L[k][k]  (column-scaled factor, strictly lower part kept)
    float dinv_own = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        float dk, ak = a[k];
        switch (k) {    // diagonal entry of step k, broadcast from lane k of the row
#define LLLA_BC(K) case K: dk = row_bcast<K>(ak); break;
            LLLA_BC(0) LLLA_BC(1) LLLA_BC(2) LLLA_BC(3) LLLA_BC(4) LLLA_BC(5) LLLA_BC(6) LLLA_BC(7)
            LLLA_BC(8) LLLA_BC(9) LLLA_BC(10) LLLA_BC(11) LLLA_BC(12) LLLA_BC(13) LLLA_BC(14) LLLA_BC(15)
#undef LLLA_BC
            default: dk = 1.f;
        }
        float rinv = __builtin_amdgcn_rsqf(dk);
        rinv = rinv * (1.5f - 0.5f * dk * rinv * rinv);      // one Newton step
        const float u = (r >= k) ? ak * rinv : 0.f;          // L[r][k]
        l2[k] = (r > k) ? u * rinv : 0.f;
        dinv_own = (r == k) ? rinv : dinv_own;
#pragma unroll
        for (int c = k + 1; c < 16; ++c) {
            float uc;
            switch (c) {
#define LLLA_BC(K) case K: uc = row_bcast<K>(u); break;
                LLLA_BC(1) LLLA_BC(2) LLLA_BC(3) LLLA_BC(4) LLLA_BC(5) LLLA_BC(6) LLLA_BC(7) LLLA_BC(8)
                LLLA_BC(9) LLLA_BC(10) LLLA_BC(11) LLLA_BC(12) LLLA_BC(13) LLLA_BC(14) LLLA_BC(15)
#undef LLLA_BC
                default: uc = 0.f;
            }
            a[c] = fmaf(-u, uc, a[c]);
        }
    }
    // M = (unit lower L'')^{-1}:  M[r][c] = [r==c] - sum_{c<=p<r} L''[r][p] M[p][c]
#pragma unroll
    for (int c = 0; c < 16; ++c) li[c] = (r == c) ? 1.f : 0.f;
#pragma unroll
    for (int p = 0; p < 15; ++p) {
#pragma unroll
        for (int c = 0; c <= p; ++c) {
            float mp;
            switch (p) {
#define LLLA_BC(K) case K: mp = row_bcast<K>(li[c]); break;
                LLLA_BC(0) LLLA_BC(1) LLLA_BC(2) LLLA_BC(3) LLLA_BC(4) LLLA_BC(5) LLLA_BC(6) LLLA_BC(7)
                LLLA_BC(8) LLLA_BC(9) LLLA_BC(10) LLLA_BC(11) LLLA_BC(12) LLLA_BC(13) LLLA_BC(14)
#undef LLLA_BC
                default: mp = 0.f;
            }
            li[c] = fmaf(-l2[p], mp, li[c]);
        }
    }
#pragma unroll
    for (int c = 0; c < 16; ++c) li[c] *= dinv_own;          // L^{-1} = D^{-1} L''^{-1}
}

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
#ifdef LLLA_DBG_BUILTIN_DMA
    __builtin_amdgcn_global_load_lds((glb_void_ptr)gsrc, (lds_void_ptr)lds_base, 16, 0, 0);
    return;
#endif
    const unsigned lds = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(lds_void_ptr)lds_base);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gsrc), "s"(lds) : "memory", "m0");
}
#pragma clang diagnostic pop
__device__ inline void dma_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// LDS tiles of one 64-key block are stored without padding (the DMA writes whole 1 KB wave rows);
// 16-byte chunks are XOR-swizzled so that the MFMA operand reads stay free of bank conflicts:
//   transposed tile (f16) : [sub-tile of 32 keys][feature row r][4 chunks of 8 keys], chunk c of row r at c ^ ((r>>2)&3)
//   natural tile (bf16)   : [key][8 chunks of 8 features],                             chunk c of key k at c ^ ((k>>1)&7)
constexpr int KT_SUB = D * KB;       // halves per transposed 32-key sub-tile (4 KB)
constexpr int KN_TILE = KB2 * D;     // halves per natural 64-key tile (8 KB)
constexpr int WT32_PITCH = KB2 + 4;  // floats per query row of the fp32 weight tile (PRECISE)

// PRECISE: fp32 weights and a two-term f16 split of the scaled operand w k, i.e. an fp32-accurate
// second moment; used for the first rows of a sequence, whose systems are the worst conditioned.
struct MomentsShared {
    _Float16 kt[2][2][KT_SUB];                 // transposed K, two buffers x two 32-key sub-tiles
    bf16_t kn[2][KN_TILE];                     // natural K, two buffers
    union {
        _Float16 h[2][QB * WT_PITCH];          // f16 weights (fast variant)
        float f[2][QB * WT32_PITCH];           // fp32 weights (precise variant)
    } w;
    float omp[4][QB];
    float mus[QB][D + 4];
    float oms[QB];
    float sc[4][QW][16 * SC_PITCH];            // per-wave scratch tiles of the solve
};

template <bool PRECISE>
__device__ __forceinline__ void moments_body(MomentsShared &sm, const bf16_t *__restrict__ Qg,
                                             const bf16_t *__restrict__ Kg, llla_strides sq, llla_strides sk, int H,
                                             int n, int nkb, int first_row, float cscale, float lambda,
                                             const _Float16 *__restrict__ KT, const float *__restrict__ Mg,
                                             float *__restrict__ Yg)
{
    auto &kt = sm.kt;
    auto &kn = sm.kn;
    auto &wt = sm.w.h;
    auto &wt32 = sm.w.f;
    auto &omp = sm.omp;
    auto &mus = sm.mus;
    auto &oms = sm.oms;
    auto &sc = sm.sc;

    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64, g = lane / 16, nn = lane % 16;
    const int bh = blockIdx.y, b = bh / H, h = bh % H;
    const int nqb = gridDim.x;
    const int i0 = first_row + (nqb - 1 - (int)blockIdx.x) * QB;       // long rows first
    const int ilast = min(i0 + QB - 1, n - 1);
    const int nblk = ilast / KB2 + 1;                                  // blocks of 64 keys
    const int mpitch = nkb * KB;
    const bf16_t *Kh = Kg + b * sk.batch + h * sk.head;
    const bf16_t *Qh = Qg + b * sq.batch + h * sq.head;
    const _Float16 *KTh = KT + (size_t)bh * nkb * (D * KB);

    // S^T role: lane (g, nn) of wave w serves query i0 + nn and keys 16w + 4g + r of a 64-key block
    const int iq = i0 + nn, iqc = min(iq, n - 1);
    bf16x8 qf[2];
    {
        const bf16_t *qrow = Qh + (int64_t)iqc * sq.seq;
        qf[0] = *reinterpret_cast<const bf16x8 *>(qrow + 8 * g);
        qf[1] = *reinterpret_cast<const bf16x8 *>(qrow + 32 + 8 * g);
    }
    const float mrow = Mg[(size_t)bh * mpitch + iqc];

    f32x4 acc[QW][10];
#pragma unroll
    for (int q = 0; q < QW; ++q)
#pragma unroll
        for (int t = 0; t < 10; ++t) acc[q][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    f32x4 mu_acc = {0.f, 0.f, 0.f, 0.f};
    float om_part = 0.f;            // this lane's share of omega for query i0 + nn
#ifdef LLLA_DBG_LDSWQ
    float dbg_mismatch = 0.f;
#endif

    // ---- per-lane constants of the staging and of the operand reads ------------------------------
    // DMA, transposed tile: this wave fills slots [64 wave, 64 wave + 64) of each 32-key sub-tile
    const int kts = 64 * wave + lane;                       // slot = row*4 + stored chunk
    const int kts_row = kts >> 2, kts_col = (kts & 3) ^ ((kts_row >> 2) & 3);
    const int kt_goff = kts_row * KB + kts_col * 8;         // halves inside a [feature][32 key] sub-tile
    // DMA, natural tile: this wave fills its own 16 keys (slots [128 wave, 128 wave + 128))
    int kn_key[2], kn_gcol[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int sl = 128 * wave + 64 * t + lane;          // slot = key*8 + stored chunk
        kn_key[t] = sl >> 3;
        kn_gcol[t] = ((sl & 7) ^ ((kn_key[t] >> 1) & 7)) * 8;
    }
    // S^T operand reads of the natural tile: key 16 wave + nn, feature chunks g and 4 + g
    const int skey = 16 * wave + nn;
    const int kn_r0 = (skey * 8 + (g ^ ((skey >> 1) & 7))) * 8;
    const int kn_r1 = (skey * 8 + ((4 + g) ^ ((skey >> 1) & 7))) * 8;
    // second-moment operand reads of a transposed sub-tile: feature row 16 I + nn, key chunk g
    const int kt_r = (nn * 4 + (g ^ ((nn >> 2) & 3))) * 8;  // + I * 16 * 32 halves

    auto issue_dma = [&](int blk) {     // block blk -> LDS buffer blk & 1
        const int buf = blk & 1;
        const _Float16 *src = KTh + (size_t)blk * (2 * KT_SUB) + kt_goff;
        dma16(src, &kt[buf][0][512 * wave]);
        dma16(src + KT_SUB, &kt[buf][1][512 * wave]);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int j = min(blk * KB2 + kn_key[t], n - 1);
            dma16(Kh + (int64_t)j * sk.seq + kn_gcol[t], &kn[buf][1024 * wave + 512 * t]);
        }
    };
    auto make_weights = [&](int blk) {  // w = 2^(c<q,k> - m) for this wave's 16 keys of block blk
        const int buf = blk & 1;
        const bf16x8 k0 = *reinterpret_cast<const bf16x8 *>(&kn[buf][kn_r0]);
        const bf16x8 k1 = *reinterpret_cast<const bf16x8 *>(&kn[buf][kn_r1]);
        f32x4 z = {0.f, 0.f, 0.f, 0.f};
        z = mfma_bf16(k0, qf[0], z);
        z = mfma_bf16(k1, qf[1], z);
        float wf[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int j = blk * KB2 + 16 * wave + 4 * g + r;
            const float wgt = __builtin_amdgcn_exp2f(z[r] * cscale - mrow);
            wf[r] = (j <= iq) ? wgt : 0.f;
        }
        if (PRECISE) {
            *reinterpret_cast<f32x4 *>(&wt32[buf][nn * WT32_PITCH + 16 * wave + 4 * g]) = f32x4{wf[0], wf[1], wf[2], wf[3]};
            om_part += (wf[0] + wf[1]) + (wf[2] + wf[3]);
        } else {
            half4 wv;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                wv[r] = (_Float16)wf[r];
                om_part += (float)wv[r];        // omega sums the weights exactly as the MFMAs see them
            }
            *reinterpret_cast<half4 *>(&wt[buf][nn * WT_PITCH + 16 * wave + 4 * g]) = wv;
        }
    };

    // Software pipeline over blocks of 64 keys: iteration c consumes block c while the DMA of block
    // c+1 lands; the weights of block c+1 are produced in the middle of the iteration (each wave
    // reads only the keys it fetched itself, so its own vmcnt wait suffices).  One barrier per block.
    issue_dma(0);
    dma_wait();
    __syncthreads();
    make_weights(0);
    __syncthreads();

#ifdef LLLA_TIMING_NO_GRAM
    for (int c = 0; c < 1; ++c) {
#else
    for (int c = 0; c < nblk; ++c) {
#endif
        const int buf = c & 1;
#ifndef LLLA_TIMING_NO_GLOAD
        if (c + 1 < nblk) issue_dma(c + 1);
#endif
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {        // two halves of 32 keys
            half8 bf[4];
#pragma unroll
            for (int I = 0; I < 4; ++I) bf[I] = *reinterpret_cast<const half8 *>(&kt[buf][hf][kt_r + I * 512]);
            if (!PRECISE) {
                // One LDS read brings the weights of all 16 queries (lane (g, nn): query (nn + 4 wave) % 16,
                // keys 8g..8g+7), rotated so that this wave's own queries sit in lanes 0..3 of every row; the
                // per-query operand scale is then a row broadcast (DPP) instead of four more LDS reads.
                const half8 wa = *reinterpret_cast<const half8 *>(&wt[buf][((nn + QW * wave) & 15) * WT_PITCH + 32 * hf + 8 * g]);
                const f32x4 wau = __builtin_bit_cast(f32x4, wa);
#pragma unroll
                for (int q = 0; q < QW; ++q) {
                    f32x4 wqu;
#pragma unroll
                    for (int t = 0; t < 4; ++t) wqu[t] = (q == 0) ? row_bcast<0>(wau[t]) : (q == 1) ? row_bcast<1>(wau[t])
                                                        : (q == 2) ? row_bcast<2>(wau[t]) : row_bcast<3>(wau[t]);
#ifdef LLLA_DBG_LDSWQ
                    const half8 wq = *reinterpret_cast<const half8 *>(&wt[buf][(QW * wave + q) * WT_PITCH + 32 * hf + 8 * g]);
                    {
                        const f32x4 ref = __builtin_bit_cast(f32x4, wq);
                        for (int t = 0; t < 4; ++t)
                            if (__builtin_bit_cast(int, ref[t]) != __builtin_bit_cast(int, wqu[t])) dbg_mismatch += 1.f;
                    }
#else
                    const half8 wq = __builtin_bit_cast(half8, wqu);
#endif
#pragma unroll
                    for (int I = 0; I < 4; ++I) {
                        const half8 af = bf[I] * wq;
#pragma unroll
                        for (int J = I; J < 4; ++J) acc[q][tix(I, J)] = mfma_f16(af, bf[J], acc[q][tix(I, J)]);
                    }
                }
                // mu~[query (4g + r + 4 wave) % 16][feature 16 wave + nn].  `wave` is a scalar (readfirstlane),
                // so these are real branches: MFMA ignores the EXEC mask and must never sit in a block that is
                // merely predicated off.
                if (wave == 0) mu_acc = mfma_f16(wa, bf[0], mu_acc);
                else if (wave == 1) mu_acc = mfma_f16(wa, bf[1], mu_acc);
                else if (wave == 2) mu_acc = mfma_f16(wa, bf[2], mu_acc);
                else mu_acc = mfma_f16(wa, bf[3], mu_acc);
            } else {
#pragma unroll
                for (int q = 0; q < QW; ++q) {
                    float wq[8];
                    {
                        const float *wp = &wt32[buf][(QW * wave + q) * WT32_PITCH + 32 * hf + 8 * g];
                        const f32x4 w0 = *reinterpret_cast<const f32x4 *>(wp), w1 = *reinterpret_cast<const f32x4 *>(wp + 4);
#pragma unroll
                        for (int t = 0; t < 4; ++t) { wq[t] = w0[t]; wq[4 + t] = w1[t]; }
                    }
#pragma unroll
                    for (int I = 0; I < 4; ++I) {
                        half8 ahi, alo;
#pragma unroll
                        for (int t = 0; t < 8; ++t) {
                            const float pr = (float)bf[I][t] * wq[t];
                            ahi[t] = (_Float16)pr;
                            alo[t] = (_Float16)(pr - (float)ahi[t]);
                        }
#pragma unroll
                        for (int J = I; J < 4; ++J) {
                            acc[q][tix(I, J)] = mfma_f16(alo, bf[J], acc[q][tix(I, J)]);
                            acc[q][tix(I, J)] = mfma_f16(ahi, bf[J], acc[q][tix(I, J)]);
                        }
                    }
                }
                // this wave's feature block for mu~ is re-read from LDS (indexing bf[] by the wave id
                // would become a per-element select chain)
                const half8 bw = *reinterpret_cast<const half8 *>(&kt[buf][hf][kt_r + wave * 512]);
                half8 whi, wlo;
                {
                    const float *wp = &wt32[buf][nn * WT32_PITCH + 32 * hf + 8 * g];
                    const f32x4 w0 = *reinterpret_cast<const f32x4 *>(wp), w1 = *reinterpret_cast<const f32x4 *>(wp + 4);
#pragma unroll
                    for (int t = 0; t < 8; ++t) {
                        const float wv = t < 4 ? w0[t] : w1[t - 4];
                        whi[t] = (_Float16)wv;
                        wlo[t] = (_Float16)(wv - (float)whi[t]);
                    }
                }
                mu_acc = mfma_f16(wlo, bw, mu_acc);
                mu_acc = mfma_f16(whi, bw, mu_acc);
            }
            if (hf == 0 && c + 1 < nblk) {
#ifndef LLLA_TIMING_NO_STAGE
                dma_wait();                     // this wave's DMA of block c+1 has landed
                make_weights(c + 1);
#endif
            }
        }
#ifndef LLLA_TIMING_NO_BARRIER
        __syncthreads();
#endif
    }

    // omega: lanes (g, nn) of all four waves hold partial sums for query i0 + nn
    om_part += __shfl_xor(om_part, 16);
    om_part += __shfl_xor(om_part, 32);
    if (g == 0) omp[wave][nn] = om_part;

    // ---- hand mu~ and omega to the waves that own the queries ---------------------------------------
#pragma unroll
    for (int r = 0; r < 4; ++r) mus[PRECISE ? 4 * g + r : ((4 * g + r + QW * wave) & 15)][16 * wave + nn] = mu_acc[r];
    __syncthreads();
    if (tid < QB) oms[tid] = (omp[0][tid] + omp[1][tid]) + (omp[2][tid] + omp[3][tid]);
    __syncthreads();

    // ---- per-query solve: 16-blocked upper Cholesky with the right-hand sides [mu~ q] as a fifth
    //      block column; all block products are C += A^T B on fp32 MFMA -----------------------------
    f32x4 rhs[QW][4];
#pragma unroll
    for (int q = 0; q < QW; ++q) {
        const int qi = QW * wave + q;
        const bf16_t *qrow = Qh + (int64_t)min(i0 + qi, n - 1) * sq.seq;
#pragma unroll
        for (int P = 0; P < 4; ++P) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int row = 16 * P + 4 * g + t;
                float v = 0.f;
                if (nn == 0) v = mus[qi][row];
                if (nn == 1) v = bf16_to_f32(qrow[row]);
                rhs[q][P][t] = v;
                acc[q][tix(P, P)][t] += (nn == 4 * g + t) ? lambda : 0.f;
            }
        }
    }

#ifdef LLLA_DBG_LDSWQ
    float dbg_g00[QW], dbg_g37[QW];
    for (int q = 0; q < QW; ++q) { dbg_g00[q] = acc[q][tix(0, 0)][0]; dbg_g37[q] = acc[q][tix(1, 3)][2]; }
#endif
    float *scw = &sc[wave][0][0];
#ifdef LLLA_TIMING_NO_SOLVE
#pragma unroll 1
    for (int P = 0; P < 0; ++P) {
#else
#pragma unroll
    for (int P = 0; P < 4; ++P) {
#endif
        // diagonal tiles -> (query, row) lanes, symmetrised
#pragma unroll
        for (int q = 0; q < QW; ++q)
#pragma unroll
            for (int t = 0; t < 4; ++t) scw[q * 16 * SC_PITCH + (4 * g + t) * SC_PITCH + nn] = acc[q][tix(P, P)][t];
        wave_sync();
        float a[16], li[16];
        {
            const float *my = scw + g * 16 * SC_PITCH;
#pragma unroll
            for (int c4 = 0; c4 < 4; ++c4) {
                const f32x4 v = *reinterpret_cast<const f32x4 *>(my + nn * SC_PITCH + 4 * c4);
#pragma unroll
                for (int t = 0; t < 4; ++t) a[4 * c4 + t] = v[t];
            }
#pragma unroll
            for (int c = 0; c < 16; ++c) a[c] = 0.5f * (a[c] + my[c * SC_PITCH + nn]);
        }
        wave_sync();
        chol_inv16(a, li, nn);
        {
            float *my = scw + g * 16 * SC_PITCH;
#pragma unroll
            for (int c4 = 0; c4 < 4; ++c4)
                *reinterpret_cast<f32x4 *>(my + nn * SC_PITCH + 4 * c4) = f32x4{li[4 * c4], li[4 * c4 + 1], li[4 * c4 + 2], li[4 * c4 + 3]};
        }
        wave_sync();
#pragma unroll
        for (int q = 0; q < QW; ++q) {
            const float *tq = scw + q * 16 * SC_PITCH;
            // U^{-1} in tile layout: reg t = Uinv[4g+t][nn] = Linv[nn][4g+t]
            const f32x4 ui = *reinterpret_cast<const f32x4 *>(tq + nn * SC_PITCH + 4 * g);
            // L^{-1} in tile layout (kept in the slot of the consumed diagonal tile for the back substitution)
            f32x4 lt;
#pragma unroll
            for (int t = 0; t < 4; ++t) lt[t] = tq[(4 * g + t) * SC_PITCH + nn];
            acc[q][tix(P, P)] = lt;
            const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int J = P + 1; J < 4; ++J) acc[q][tix(P, J)] = tile_atb(zero, ui, acc[q][tix(P, J)]);
            rhs[q][P] = tile_atb(zero, ui, rhs[q][P]);
#pragma unroll
            for (int I = P + 1; I < 4; ++I) {
                const f32x4 neg = -acc[q][tix(P, I)];
#pragma unroll
                for (int J = I; J < 4; ++J) acc[q][tix(I, J)] = tile_atb(acc[q][tix(I, J)], neg, acc[q][tix(P, J)]);
                rhs[q][I] = tile_atb(rhs[q][I], neg, rhs[q][P]);
            }
        }
        wave_sync();
    }

    // rhs[q][P]: column 0 = a = U^{-T} mu~, column 1 = c = U^{-T} q.  Schur step on the intercept:
    // y0 = (1 - a.c) / (omega - a.a);  y1 = U^{-1} (c - a y0)
    float y0v[QW];
#pragma unroll
    for (int q = 0; q < QW; ++q) {
        float saa = 0.f, sac = 0.f;
#pragma unroll
        for (int P = 0; P < 4; ++P)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float v = rhs[q][P][t];
                const float o = lane_xor1(v);
                saa = fmaf(v, v, saa);
                sac = fmaf(v, o, sac);
            }
        saa += __shfl_xor(saa, 16); saa += __shfl_xor(saa, 32);
        sac += __shfl_xor(sac, 16); sac += __shfl_xor(sac, 32);
        const float om = oms[QW * wave + q];
        const float y0 = (1.f - sac) / (om - saa);           // valid in lanes nn == 0
        y0v[q] = y0;
#pragma unroll
        for (int P = 0; P < 4; ++P)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float av = rhs[q][P][t];
                const float cv = lane_xor1(av);
                rhs[q][P][t] = (nn == 0) ? (cv - av * y0) : 0.f;
            }
    }

    // back substitution, block rows 3..0:  x_P = Uinv_P (t_P - sum_{J>P} U(P,J) x_J)
#pragma unroll
    for (int P = 3; P >= 0; --P) {
#pragma unroll
        for (int J = P + 1; J < 4; ++J) {
            // transpose U(P,J) through the scratch tile so that it can be the A^T operand
#pragma unroll
            for (int q = 0; q < QW; ++q)
                *reinterpret_cast<f32x4 *>(scw + q * 16 * SC_PITCH + nn * SC_PITCH + 4 * g) = acc[q][tix(P, J)];
            wave_sync();
#pragma unroll
            for (int q = 0; q < QW; ++q) {
                f32x4 ut;
#pragma unroll
                for (int t = 0; t < 4; ++t) ut[t] = -scw[q * 16 * SC_PITCH + (4 * g + t) * SC_PITCH + nn];
                rhs[q][P] = tile_atb(rhs[q][P], ut, rhs[q][J]);
            }
            wave_sync();
        }
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int q = 0; q < QW; ++q) rhs[q][P] = tile_atb(zero, acc[q][tix(P, P)], rhs[q][P]);
    }

#ifdef LLLA_DBG_LDSWQ
    for (int o = 1; o < 64; o <<= 1) dbg_mismatch += __shfl_xor(dbg_mismatch, o);
#endif
#pragma unroll
    for (int q = 0; q < QW; ++q) {
        const int i = i0 + QW * wave + q;
        if (i < n && nn == 0) {
            float *yr = Yg + ((size_t)bh * n + i) * YP;
#pragma unroll
            for (int P = 0; P < 4; ++P) *reinterpret_cast<f32x4 *>(yr + 16 * P + 4 * g) = rhs[q][P];
#ifdef LLLA_DBG_DUMPMU
            for (int P = 0; P < 4; ++P) for (int t = 0; t < 4; ++t) yr[16 * P + 4 * g + t] = mus[QW * wave + q][16 * P + 4 * g + t];
#endif
            if (g == 0) yr[D] = y0v[q];
#ifdef LLLA_DBG_LDSWQ
            if (g == 0) yr[D + 1] = dbg_mismatch;
            if (g == 0) { yr[D + 2] = dbg_g00[q]; yr[D + 3] = dbg_g37[q]; }
#endif
        }
    }
}

// One launch serves every query block: blocks whose rows lie below precise_rows take the precise
// variant.  The choice depends on blockIdx only, so it is a scalar branch (MFMA ignores EXEC).
__global__ __launch_bounds__(NT, 2) void moments_kernel(const bf16_t *__restrict__ Qg, const bf16_t *__restrict__ Kg,
                                                        llla_strides sq, llla_strides sk, int H, int n, int nkb,
                                                        int precise_rows, float cscale, float lambda,
                                                        const _Float16 *__restrict__ KT, const float *__restrict__ Mg,
                                                        float *__restrict__ Yg)
{
    __shared__ __align__(16) MomentsShared sm;
    const int i0 = ((int)gridDim.x - 1 - (int)blockIdx.x) * QB;
    if (i0 < precise_rows) moments_body<true>(sm, Qg, Kg, sq, sk, H, n, nkb, 0, cscale, lambda, KT, Mg, Yg);
    else moments_body<false>(sm, Qg, Kg, sq, sk, H, n, nkb, 0, cscale, lambda, KT, Mg, Yg);
}

}  // namespace

bool mfma_forward_supported(int d, llla_dtype in, bool causal) { return d == D && in == LLLA_BF16 && causal; }

size_t mfma_forward_workspace_bytes(int B, int H, int n, int d, llla_dtype in)
{
    if (!mfma_forward_supported(d, in, true)) return 0;
    return make_layout(B, H, n).total;
}

hipError_t mfma_forward(const Problem &p)
{
    const Layout L = make_layout(p.B, p.H, p.n);
    char *ws = static_cast<char *>(p.ws);
    _Float16 *KT = reinterpret_cast<_Float16 *>(ws + L.kt);
    bf16_t *VT = reinterpret_cast<bf16_t *>(ws + L.vt);
    float *M = reinterpret_cast<float *>(ws + L.m);
    float *Y = reinterpret_cast<float *>(ws + L.y);
    const int bh = p.B * p.H;
    const float cscale = p.scale * LOG2E;
    const int first = EARLY_ROWS < p.n ? EARLY_ROWS : p.n;

    const bf16_t *Q = static_cast<const bf16_t *>(p.Q), *K = static_cast<const bf16_t *>(p.K),
                 *V = static_cast<const bf16_t *>(p.V);
    stage_mark(p.stream, "prep");
    hipLaunchKernelGGL(prep_kernel, dim3(L.nkb, bh), dim3(NT), 0, p.stream, K, V, p.sk, p.sv, p.H, p.n, L.nkb, KT, VT);
    const int nq64 = (p.n + 63) / 64;
    stage_mark(p.stream, "rowmax");
    hipLaunchKernelGGL((sweep_kernel<true>), dim3(nq64, bh), dim3(NT), 0, p.stream, Q, K, p.sq, p.sk, p.H, p.n, L.nkb,
                       0, cscale, VT, M, Y, p.O, p.so, 0);
    const int nq16 = (p.n + QB - 1) / QB;
    stage_mark(p.stream, "moments");
    hipLaunchKernelGGL(moments_kernel, dim3(nq16, bh), dim3(NT), 0, p.stream, Q, K, p.sq, p.sk, p.H, p.n, L.nkb, first,
                       cscale, p.lambda, KT, M, Y);
    // output: the first rows are evaluated in fp32 on the vector ALUs (their weights y0 + k.y1 cancel
    // to a few digits), the rest by the MFMA sweep
    stage_mark(p.stream, "output_early_rows");
    hipError_t e = valu_forward_given(p, first, M, L.npad, Y, YP);
    if (e != hipSuccess) return e;
    if (first < p.n) {
        const int nq64b = (p.n - first + 63) / 64;
        stage_mark(p.stream, "output");
        hipLaunchKernelGGL((sweep_kernel<false>), dim3(nq64b, bh), dim3(NT), 0, p.stream, Q, K, p.sq, p.sk, p.H, p.n,
                           L.nkb, first, cscale, VT, M, Y, p.O, p.so, p.out == LLLA_BF16 ? 1 : 0);
    }
    return hipGetLastError();
}

}  // namespace llla

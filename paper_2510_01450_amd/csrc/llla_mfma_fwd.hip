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
#include "llla_mfma_common.hpp"

namespace llla {
namespace {

using namespace mfma;

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

    for (int c = 0; c < nblk; ++c) {
        const int buf = c & 1;
        if (c + 1 < nblk) issue_dma(c + 1);
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
                    const half8 wq = __builtin_bit_cast(half8, wqu);
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
                dma_wait();                     // this wave's DMA of block c+1 has landed
                make_weights(c + 1);
            }
        }
        __syncthreads();
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

    // ---- per-query solve (see solve_wave); the right-hand sides [mu~ q] are built inside it ----------
    f32x4 rhs[QW][4];
    float y0v[QW], om4[QW];
#pragma unroll
    for (int q = 0; q < QW; ++q) om4[q] = oms[QW * wave + q];
    solve_wave(acc, rhs, y0v, om4, &sc[wave][0][0], lambda, g, nn, [&](f32x4 (&r)[QW][4]) {
#pragma unroll
        for (int q = 0; q < QW; ++q) {
            const int qi = QW * wave + q;
            const bf16_t *qrow = Qh + (int64_t)min(i0 + qi, n - 1) * sq.seq;
#pragma unroll
            for (int P = 0; P < 4; ++P)
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int row = 16 * P + 4 * g + t;
                    float v = 0.f;
                    if (nn == 0) v = mus[qi][row];
                    if (nn == 1) v = bf16_to_f32(qrow[row]);
                    r[q][P][t] = v;
                }
        }
    });

#pragma unroll
    for (int q = 0; q < QW; ++q) {
        const int i = i0 + QW * wave + q;
        if (i < n && nn == 0) {
            float *yr = Yg + ((size_t)bh * n + i) * YP;
#pragma unroll
            for (int P = 0; P < 4; ++P) *reinterpret_cast<f32x4 *>(yr + 16 * P + 4 * g) = rhs[q][P];
            if (g == 0) yr[D] = y0v[q];
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

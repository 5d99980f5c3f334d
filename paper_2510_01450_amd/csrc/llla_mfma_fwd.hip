// Matrix-core (MFMA) forward path of Local Linear Attention for gfx950: bf16 inputs, d = 64 or 128.
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
// The first 2d rows of every sequence, whose systems are the worst conditioned, take the "precise" variant of the
// moments kernel (fp32 weights, the scaled operand as two f16 terms) and an fp32 output sweep on the vector ALU.
#include <type_traits>

#include "llla_mfma_common.hpp"
#include "llla_mfma_solve64.hpp"
#include "llla_mfma_solve128.hpp"

namespace llla {
namespace {

using namespace mfma;

struct Layout {
    size_t kt, vt, m, y, total;
    int nkb, npad;
};

template <int DD>
Layout make_layout(int B, int H, int n)
{
    Layout L;
    L.nkb = 2 * ((n + 2 * KB - 1) / (2 * KB));      // 32-key blocks, an even count
    L.npad = L.nkb * KB;
    const size_t bh = (size_t)B * H;
    size_t off = 0;
    L.kt = off; off += round_up(bh * L.npad * DD * 2, 256);
    L.vt = off; off += round_up(bh * L.npad * DD * 2, 256);
    L.m = off;  off += round_up(bh * L.npad * 4, 256);
    L.y = off;  off += round_up(bh * (size_t)n * Shape<DD>::YP * 4, 256);
    L.total = off;
    return L;
}

// ------------------------------------------------------------------------------------------------
// prep: re-tile K (-> f16) and V (bf16) as [bh][key block][feature][32 keys]
template <int DD>
__global__ __launch_bounds__(256) void prep_kernel(const bf16_t *__restrict__ Kg, const bf16_t *__restrict__ Vg,
                                                   llla_strides sk, llla_strides sv, int H, int n, int nkb,
                                                   _Float16 *__restrict__ KT, bf16_t *__restrict__ VT)
{
    __shared__ bf16_t tile[2][KB][DD + 2];
    const int blk = blockIdx.x, bh = blockIdx.y, b = bh / H, h = bh % H, tid = threadIdx.x;
    const bf16_t *Kh = Kg + b * sk.batch + h * sk.head;
    const bf16_t *Vh = Vg + b * sv.batch + h * sv.head;
    for (int idx = tid; idx < KB * (DD / 8); idx += 256) {
        const int key = idx / (DD / 8), ch = (idx % (DD / 8)) * 8;
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
    for (int idx = tid; idx < DD * 4; idx += 256) {
        const int feat = idx / 4, k0 = (idx % 4) * 8;
        half8 ko;
        uint16_t vo[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            ko[i] = (_Float16)bf16_to_f32(tile[0][k0 + i][feat]);
            vo[i] = tile[1][k0 + i][feat];
        }
        const size_t base = ((size_t)bh * nkb + blk) * (DD * KB) + feat * KB + k0;
        *reinterpret_cast<half8 *>(KT + base) = ko;
        *reinterpret_cast<uint4 *>(VT + base) = make_uint4(vo[0] | (vo[1] << 16), vo[2] | (vo[3] << 16),
                                                           vo[4] | (vo[5] << 16), vo[6] | (vo[7] << 16));
    }
}

// ------------------------------------------------------------------------------------------------
// Sweep over S^T = K Q^T for 64 queries per workgroup (16 per wave).
//   MAXONLY: write the row maxima m_i (in log2 units) -- Algorithm 1's m after its last block.
//   else   : third loop of Algorithm 1: S = W (y0 + K y1), O = S V.
constexpr int VT_PITCH = KB + 8;     // halves

// LIVE < NB (a d = 16 / 32 call on zero-padded copies): features and value columns from 16 LIVE on are zero, so the
// contractions over features stop after the chunks that hold live ones and only LIVE output tiles are formed and stored.
template <bool MAXONLY, int DD, int LIVE = Shape<DD>::NB>
__global__ __launch_bounds__(256, 2) void sweep_kernel(const bf16_t *__restrict__ Qg, const bf16_t *__restrict__ Kg,
                                                    llla_strides sq, llla_strides sk, int H, int n, int nkb,
                                                    int first_row, float cscale, const bf16_t *__restrict__ VT,
                                                    float *__restrict__ Mg, const float *__restrict__ Yg,
                                                    void *__restrict__ Og, llla_strides so, int out_bf16,
                                                    float *__restrict__ Csum = nullptr, int causal = 1)
{
    // !MAXONLY is a general "coefficients times a tile" sweep: O_i = sum_j w_ij (y0_i + k_j . y1_i) t_j with the rows t_j
    // of whatever VT holds (V for the output; K for the first moment and for the matrix-free product of the
    // approximate mode).  Yg == nullptr means y0 = 1, y1 = 0 (plain weights); Csum, if given, receives sum_j of the
    // coefficients of every row.
    using S = Shape<DD>;
    constexpr int NF = (16 * LIVE + 31) / 32, NB = LIVE, YP = S::YP;     // feature chunks of 32 and output tiles that are live
    constexpr int KN_PITCH = DD + 16;    // halves; rows of the natural K tile stay 16-byte aligned (measured 2-3 % faster than DD + 8)
    __shared__ __align__(16) bf16_t kn[KB * KN_PITCH];
    __shared__ __align__(16) bf16_t vt[MAXONLY ? 8 : DD * VT_PITCH];
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64, g = lane / 16, nn = lane % 16;
    // head on blockIdx.x (dispatched fastest), query block on y, longest rows first: every head's longest blocks
    // start first and the short ones fill the tail.  (With the head on y the last head's longest block ran alone at the
    // end; with the XCD-grouped mapping of the moments kernel a head's 64-row blocks all start at once and the XCD
    // waits for the longest: both measured slower.)  Heads that are a multiple of 8 apart share an XCD and its L2.
    const int bh = blockIdx.x, b = bh / H, h = bh % H;
    const int nqb = gridDim.y;
    const int i0 = first_row + (nqb - 1 - (int)blockIdx.y) * 64;
    const int iq = i0 + wave * 16 + nn;                                // this lane's query
    const int iqc = min(iq, n - 1);
    const int jlim = causal ? iq : n - 1;                              // last key this lane's query sees
    const bf16_t *Kh = Kg + b * sk.batch + h * sk.head;
    const bf16_t *qrow = Qg + b * sq.batch + h * sq.head + (int64_t)iqc * sq.seq;
    bf16x8 qf[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f) qf[f] = *reinterpret_cast<const bf16x8 *>(qrow + 32 * f + 8 * g);
    // Row maxima: max_j c <q, k_j> = |c| max_j <sign(c) q, k_j>, so the sign of the scale goes into the query operand
    // once (a flip of the bf16 sign bits) and the sweep keeps the maximum of the RAW products, one three-input maximum
    // per two logits; |c| is applied to the result.  (Scaling every logit first was two vector instructions per logit
    // in a sweep that the vector ALU bounds.)
    if (MAXONLY && cscale < 0.f) {
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            uint4 u = __builtin_bit_cast(uint4, qf[f]);
            u.x ^= 0x80008000u; u.y ^= 0x80008000u; u.z ^= 0x80008000u; u.w ^= 0x80008000u;
            qf[f] = __builtin_bit_cast(bf16x8, u);
        }
    }

    float mrow = -INFINITY, y0 = 0.f;
    bf16x8 yh[NF], yl[NF];
    f32x4 oacc[NB];
    if (!MAXONLY) {
        mrow = Mg[(size_t)bh * (nkb * KB) + iqc];
        const float *yr = Yg ? Yg + ((size_t)bh * n + iqc) * YP : nullptr;
        y0 = yr ? yr[DD] : 1.f;
#pragma unroll
        for (int f = 0; f < NF; ++f)
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const float v = yr ? yr[32 * f + 8 * g + t] : 0.f;
                const __bf16 hi = (__bf16)v;
                yh[f][t] = hi;
                yl[f][t] = (__bf16)(v - (float)hi);
            }
#pragma unroll
        for (int J = 0; J < NB; ++J) oacc[J] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    float mx[2][4];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int r = 0; r < 4; ++r) mx[s][r] = -INFINITY;
    float csum = 0.f;

    const int ilast = min(i0 + 63, n - 1);
    const int nblk = causal ? ilast / KB + 1 : (n + KB - 1) / KB;
    // The K (natural) and V^T tiles of block c + 1 are fetched into registers while block c is computed, and written
    // to LDS at the top of the next iteration: the global-memory latency is off the path between the two barriers
    // (the row-maximum sweep has four MFMAs of work per block and was waiting for memory most of the time).
    constexpr int NLD = DD / 64;         // 16-byte pieces per thread and tile
    uint4 kpre[NLD], vpre[MAXONLY ? 1 : NLD];
    auto fetch = [&](int c) {
#pragma unroll
        for (int u = 0; u < NLD; ++u) {
            const int idx = tid + 256 * u;
            const int key = idx / (DD / 8), ch = (idx % (DD / 8)) * 8;
            const int j = c * KB + key;
            kpre[u] = make_uint4(0, 0, 0, 0);
            if (j < n) kpre[u] = *reinterpret_cast<const uint4 *>(Kh + (int64_t)j * sk.seq + ch);
            if (!MAXONLY) {
                const int feat = idx / 4, k0 = (idx % 4) * 8;
                vpre[u] = *reinterpret_cast<const uint4 *>(VT + ((size_t)bh * nkb + c) * (DD * KB) + feat * KB + k0);
            }
        }
    };
    fetch(0);
    for (int c = 0; c < nblk; ++c) {
        __syncthreads();
#pragma unroll
        for (int u = 0; u < NLD; ++u) {
            const int idx = tid + 256 * u;
            const int key = idx / (DD / 8), ch = (idx % (DD / 8)) * 8;
            *reinterpret_cast<uint4 *>(&kn[key * KN_PITCH + ch]) = kpre[u];
            if (!MAXONLY) {
                const int feat = idx / 4, k0 = (idx % 4) * 8;
                *reinterpret_cast<uint4 *>(&vt[feat * VT_PITCH + k0]) = vpre[u];
            }
        }
        if (c + 1 < nblk) fetch(c + 1);
        __syncthreads();
        f32x4 st[2], ut[2];
#pragma unroll
        for (int s = 0; s < 2; ++s) {       // two sub-tiles of 16 keys
            bf16x8 kf[NF];
#pragma unroll
            for (int f = 0; f < NF; ++f) kf[f] = *reinterpret_cast<const bf16x8 *>(&kn[(16 * s + nn) * KN_PITCH + 32 * f + 8 * g]);
            f32x4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int f = 0; f < NF; ++f) z = mfma_bf16(kf[f], qf[f], z);
            st[s] = z;
            if (!MAXONLY) {
                f32x4 u = {y0, y0, y0, y0};         // y0 + k . y1: the intercept rides in as the accumulator's initial value
#pragma unroll
                for (int f = 0; f < NF; ++f) u = mfma_bf16(kf[f], yl[f], u);
#pragma unroll
                for (int f = 0; f < NF; ++f) u = mfma_bf16(kf[f], yh[f], u);
                ut[s] = u;
            }
        }
        // lane (g, nn): st[s][r] = <k_j, q_iq> for key j = 32c + 16s + 4g + r.  Only the blocks that reach past the
        // wave's first query need the causal mask (a scalar condition): the others skip the compares and selects,
        // which are most of the vector work of this sweep.
        const bool masked = causal ? (c * KB + KB - 1 > i0 + wave * 16) : (c * KB + KB > n);
        if (MAXONLY) {
            if (!masked) {
#pragma unroll
                for (int r = 0; r < 4; ++r) mx[0][r] = __builtin_fmaxf(__builtin_fmaxf(mx[0][r], st[0][r]), st[1][r]);   // v_max3_f32
            } else {
#pragma unroll
                for (int s = 0; s < 2; ++s)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int j = c * KB + 16 * s + 4 * g + r;
                        mx[0][r] = (j <= jlim) ? fmaxf(mx[0][r], st[s][r]) : mx[0][r];
                    }
            }
        } else {
            bf16x8 ch, cl;      // output weights as bf16 hi + lo; slot t<4: key 4g+t, t>=4: key 16+4g+t-4
            float cv[8];
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    cv[4 * s + r] = __builtin_amdgcn_exp2f(st[s][r] * cscale - mrow) * ut[s][r];
            if (masked) {
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const int j = c * KB + 16 * (t >> 2) + 4 * g + (t & 3);
                    cv[t] = (j <= jlim) ? cv[t] : 0.f;
                }
            }
            if (Csum != nullptr) {                                   // a scalar branch: the plain output call skips the sums
#pragma unroll
                for (int t = 0; t < 8; ++t) csum += cv[t];
            }
            // two values per conversion instruction (v_cvt_pk_bf16_f32)
            typedef float float2v __attribute__((ext_vector_type(2)));
            typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
#pragma unroll
            for (int t = 0; t < 8; t += 2) {
                const bf16x2v hi = __builtin_convertvector(float2v{cv[t], cv[t + 1]}, bf16x2v);
                const bf16x2v lo = __builtin_convertvector(float2v{cv[t] - (float)hi[0], cv[t + 1] - (float)hi[1]}, bf16x2v);
                ch[t] = hi[0]; ch[t + 1] = hi[1];
                cl[t] = lo[0]; cl[t + 1] = lo[1];
            }
#pragma unroll
            for (int J = 0; J < NB; ++J) {
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
        float m = fmaxf(fmaxf(mx[0][0], mx[0][1]), fmaxf(mx[0][2], mx[0][3]));
        m = fmaxf(m, __shfl_xor(m, 16));
        m = fmaxf(m, __shfl_xor(m, 32));
        // every row sees at least its own key, so m is finite; a zero scale gives 0 (not 0 times a product)
        if (g == 0 && iq < n) Mg[(size_t)bh * (nkb * KB) + iq] = cscale == 0.f ? 0.f : m * fabsf(cscale);
    } else {
        if (Csum != nullptr) {      // lanes (g, nn), g = 0..3, hold the coefficients of query nn for disjoint keys
            csum += __shfl_xor(csum, 16);
            csum += __shfl_xor(csum, 32);
            if (g == 0 && iq < n) Csum[(size_t)bh * n + iq] = csum;
        }
        // oacc[J]: lane (g, nn) reg r = O[query i0 + 16 wave + 4g + r][feature 16J + nn]
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int i = i0 + wave * 16 + 4 * g + r;
            if (i < n) {
                const int64_t off = b * so.batch + h * so.head + (int64_t)i * so.seq;
#pragma unroll
                for (int J = 0; J < NB; ++J) {
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
constexpr int WT32_PITCH = KB2 + 4;  // floats per query row of the fp32 weight tile (PRECISE)
// LDS tiles of one 64-key block are stored without padding (the DMA writes whole 1 KB wave rows);
// 16-byte chunks are XOR-swizzled so that the MFMA operand reads stay free of bank conflicts:
//   transposed tile (f16) : [sub-tile of 32 keys][feature row r][4 chunks of 8 keys], chunk c of row r at c ^ ((r>>2)&3)
//   natural tile (bf16)   : [key][d/8 chunks of 8 features], chunk c of key k at c ^ ((k>>1)&7) (d = 64), c ^ (k&15) (d = 128)

template <int DD>
struct MomentsShared {
    using S = Shape<DD>;
    _Float16 kt[2][2][DD * KB];                // transposed K, two buffers x two 32-key sub-tiles
    bf16_t kn[2][KB2 * DD];                    // natural K, two buffers
    union {
        _Float16 h[4][16 * WT_PITCH];          // f16 weights (fast variant), 16 query rows (MFMA width); 3 blocks are in
                                               // flight, the d = 64 loop rotates over 4 buffers (a power of two, see there)
        float f[3][16 * WT32_PITCH];           // fp32 weights (precise variant)
    } w;
    float omp[4][16];
    float mus[16][DD + 4];
    float oms[16];
    bf16_t qt[16][DD + 8];                     // the workgroup's query rows (operand of the logits)
    float sc[S::NW][S::QW][16 * SC_PITCH];     // per-wave scratch tiles of the solve
};

template <int CH>
__device__ inline int nat_swizzle(int key) { return CH == 8 ? ((key >> 1) & 7) : (key & 15); }

// (head, query block) of a workgroup of the moments kernels: XCD-aware at d = 64 (see xcd_block_map; HBM reads of the
// kernel 0.71 -> 0.14 GB at [4,16,4096,64], 3 % faster there and 10 % with 1024 short heads); at d = 128 the plain
// mapping (x = query block, y = head) measured 2 % faster and is kept.
template <int DD>
__device__ inline BlockMap moments_block()
{
    if (DD == 64) return xcd_block_map();
    return BlockMap{(int)blockIdx.y, (int)blockIdx.x};
}

// PRECISE: fp32 weights and a two-term f16 split of the scaled operand w k, i.e. an fp32-accurate
// second moment; used for the first rows of a sequence, whose systems are the worst conditioned.
// WITH_U (the backward pass): Rg holds, per row, r1 (DD floats) and r0 at [DD] (pitch YP); the solve then also
// returns u = M^{-1} [r0; r1] in Ug, laid out like Yg.
// LIVE: feature blocks of 16 that can be non-zero (all of them, except for calls at d = 16 / 32 that run here on
// zero-padded copies: tiles of Sigma~ with a padded block stay at their starting value, 0 or -lambda on the diagonal, so
// neither their MFMAs nor the scaled operands of padded blocks are issued).
template <bool PRECISE, int DD, bool WITH_U = false, int LIVE = Shape<DD>::NB>
__device__ __forceinline__ void moments_body(MomentsShared<DD> &sm, const bf16_t *__restrict__ Qg,
                                             const bf16_t *__restrict__ Kg, llla_strides sq, llla_strides sk, int H,
                                             int n, int nkb, float cscale, float lambda,
                                             const float *__restrict__ lam_rows, const _Float16 *__restrict__ KT,
                                             const float *__restrict__ Mg, float *__restrict__ Yg,
                                             const float *__restrict__ Rg = nullptr, float *__restrict__ Ug = nullptr,
                                             int causal = 1)
{
    using S = Shape<DD>;
    constexpr int NB = S::NB, NTILE = S::NTILE, NF = S::NF, QW = S::QW, NW = S::NW, QB = S::QB, YP = S::YP;
    constexpr int CH = DD / 8;                          // 16-byte chunks of a natural row
    static_assert(LIVE == NB || DD == 64, "padded calls run at d = 64");
    constexpr int KT_SUB = DD * KB;                     // halves per transposed 32-key sub-tile
    constexpr int NAT_INSTR = 16 * CH / 64;             // DMA instructions of a weight wave: its 16 keys
    constexpr int TW = (NW == 4) ? 4 : NW - 4;          // waves that fetch the transposed tiles
    constexpr int TR_SLOTS = DD * 4 / TW;               // 16-byte slots per sub-tile and such wave
    constexpr int TR_INSTR = TR_SLOTS / 64;
    auto &kt = sm.kt;
    auto &kn = sm.kn;
    auto &wt = sm.w.h;
    auto &wt32 = sm.w.f;
    auto &mus = sm.mus;
    auto &oms = sm.oms;
    auto &sc = sm.sc;

    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64, g = lane / 16, nn = lane % 16;
    const BlockMap bm = moments_block<DD>();
    const int bh = bm.bh, b = bh / H, h = bh % H;
    const int nqb = gridDim.x;
    const int i0 = (nqb - 1 - bm.blk) * QB;                           // long rows first
    const int ilast = min(i0 + QB - 1, n - 1);
    const int nblk = causal ? ilast / KB2 + 1 : (n + KB2 - 1) / KB2;   // blocks of 64 keys
    const int mpitch = nkb * KB;
    const bf16_t *Kh = Kg + b * sk.batch + h * sk.head;
    const bf16_t *Qh = Qg + b * sq.batch + h * sq.head;
    const _Float16 *KTh = KT + (size_t)bh * nkb * KT_SUB;
    const bool w_wave = (NW == 4) || wave < 4;          // computes weights: 16 keys x 16 query columns per block
    const bool t_wave = (NW == 4) || wave >= 4;         // fetches the transposed tiles
    const int tw = (NW == 4) ? wave : wave - 4;

    // weight role: lane (g, nn) of wave w < 4 serves query i0 + nn (nn < QB) and keys 16w + 4g + r
    const int iq = i0 + nn, iqc = min(iq, n - 1);
    const int jlim = causal ? iq : n - 1;                   // last key the lane's query sees
    const bool q_live = nn < QB;
    // The query operand of the logits: d = 64 re-reads it from LDS for every block (its registers go to the second
    // fragment set), d = 128 keeps it in registers.
    constexpr bool Q_IN_LDS = (DD == 64);
    bf16x8 qf[NF];
    {
        const bf16_t *qrow = Qh + (int64_t)iqc * sq.seq;
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            qf[f] = *reinterpret_cast<const bf16x8 *>(qrow + 32 * f + 8 * g);
            // each (g, nn) lane of the four weight waves would store the same chunks: wave 0 does
            if (Q_IN_LDS && wave == 0) *reinterpret_cast<bf16x8 *>(&sm.qt[nn][32 * f + 8 * g]) = qf[f];
        }
    }
    const float mrow = Mg[(size_t)bh * mpitch + iqc];

    f32x4 acc[QW][NTILE];
#pragma unroll
    for (int q = 0; q < QW; ++q)
#pragma unroll
        for (int t = 0; t < NTILE; ++t) acc[q][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    // The tiles accumulate T = -(Sigma~ + lambda I), the sign the solve works in (see factorise_wave): the ridge is
    // the starting value of the diagonal, and the scaled MFMA operand carries a minus sign that costs nothing.
#pragma unroll
    for (int q = 0; q < QW; ++q) {
        // the ridge of the query's own row when one is given per row (Appendix C)
        const float lq = lam_rows ? lam_rows[(size_t)bh * n + min(i0 + QW * wave + q, n - 1)] : lambda;
#pragma unroll
        for (int P = 0; P < NB; ++P)
#pragma unroll
            for (int t = 0; t < 4; ++t) acc[q][S::tix(P, P)][t] = (nn == 4 * g + t) ? -lq : 0.f;
    }
    f32x4 mu_acc = {0.f, 0.f, 0.f, 0.f};
    // omega: every weight wave sums the weights of its own keys on the vector ALU, exactly as the MFMAs see them (the
    // rounded f16 values, two per v_dot2_f32_f16).  Summing it on the matrix cores with a tile of ones as the B operand
    // of one more MFMA per half (OM_MFMA) was the d = 64 choice for a while; it costs eight registers that the
    // alternating schedule below needs, and it made the one wave that did it the slowest of its workgroup.
    constexpr bool OM_MFMA = false;
    constexpr bool PIPE = (DD == 64) && !PRECISE;
    f32x4 om_acc = {0.f, 0.f, 0.f, 0.f};      // OM_MFMA, one wave: -omega of query 4g + r in every column
    float om_part = 0.f;                      // otherwise: this lane's share of omega for query i0 + nn

    // ---- per-lane constants of the staging and of the operand reads ------------------------------
    int tr_goff[TR_INSTR];                                  // halves inside a [feature][32 key] sub-tile
#pragma unroll
    for (int t = 0; t < TR_INSTR; ++t) {
        const int sl = tw * TR_SLOTS + 64 * t + lane;       // slot = row*4 + stored chunk
        const int row = sl >> 2, col = (sl & 3) ^ ((row >> 2) & 3);
        tr_goff[t] = row * KB + col * 8;
    }
    int kn_key[NAT_INSTR], kn_gcol[NAT_INSTR];
#pragma unroll
    for (int t = 0; t < NAT_INSTR; ++t) {
        const int sl = 16 * CH * wave + 64 * t + lane;      // slot = key*CH + stored chunk
        kn_key[t] = sl / CH;
        kn_gcol[t] = ((sl % CH) ^ nat_swizzle<CH>(kn_key[t])) * 8;
    }
    // logits operand reads of the natural tile: key 16 wave + nn, feature chunks g + 4f
    const int skey = 16 * wave + nn;
    int kn_r[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f) kn_r[f] = (skey * CH + ((g + 4 * f) ^ nat_swizzle<CH>(skey))) * 8;
    // second-moment operand reads of a transposed sub-tile: feature row 16 I + nn, key chunk g
    const int kt_r = (nn * 4 + (g ^ ((nn >> 2) & 3))) * 8;  // + I * 16 * 32 halves

    // Transfers take a scalar base address per block plus per-lane byte offsets that never change, so that a
    // transfer costs no vector-ALU address arithmetic (every vector instruction of this loop competes with the
    // MFMAs for the issue port); only the last, ragged block of natural rows clamps its rows per lane.
    unsigned tr_boff[TR_INSTR], kn_boff[NAT_INSTR];
#pragma unroll
    for (int t = 0; t < TR_INSTR; ++t) tr_boff[t] = 2u * (unsigned)tr_goff[t];
#pragma unroll
    for (int t = 0; t < NAT_INSTR; ++t) kn_boff[t] = 2u * (unsigned)(kn_key[t] * (int)sk.seq + kn_gcol[t]);
    const bool small_pitch = sk.seq < (int64_t(1) << 23);       // the offsets above fit 32 bits
    const int n_whole_small = small_pitch ? n / KB2 : 0;        // blocks below this are whole tiles that the scalar-base transfers can fetch
    const unsigned kt_lds = lds_offset(&sm.kt[0][0][0]), kn_lds = lds_offset(&sm.kn[0][0]);
    auto issue_dma = [&](int blk) {     // block blk -> LDS buffer blk & 1
        const int buf = blk & 1;
        if (t_wave) {
            const _Float16 *src = KTh + (size_t)blk * (2 * KT_SUB);
            const unsigned dst = kt_lds + 2u * (unsigned)(buf * 2 * DD * KB + tw * TR_SLOTS * 8);
#pragma unroll
            for (int t = 0; t < TR_INSTR; ++t) {
                dma16_base_off(src, tr_boff[t], dst + 2u * (64 * t * 8));
                dma16_base_off(src + KT_SUB, tr_boff[t], dst + 2u * (DD * KB + 64 * t * 8));
            }
        }
        if (w_wave) {
            if (blk < n_whole_small) {
                const bf16_t *src = Kh + (int64_t)blk * KB2 * sk.seq;
                const unsigned dst = kn_lds + 2u * (unsigned)(buf * KB2 * DD + 16 * CH * wave * 8);
#pragma unroll
                for (int t = 0; t < NAT_INSTR; ++t) dma16_base_off(src, kn_boff[t], dst + 2u * (64 * t * 8));
            } else {
#pragma unroll
                for (int t = 0; t < NAT_INSTR; ++t) {
                    // (from an opaque copy of the lane index: the addresses of this rare branch are then formed here,
                    // not hoisted out of the loop as invariants that would have to be spilled across it)
                    int ln = lane;
                    asm volatile("" : "+v"(ln));
                    const int sl = 16 * CH * wave + 64 * t + ln;      // slot = key*CH + stored chunk, as above
                    const int key = sl / CH, gcol = ((sl % CH) ^ nat_swizzle<CH>(key)) * 8;
                    const int j = min(blk * KB2 + key, n - 1);
                    dma16(Kh + (int64_t)j * sk.seq + gcol, &kn[buf][(16 * CH * wave + 64 * t) * 8]);
                }
            }
        }
    };
    // Weights of block blk, w = 2^(c<q,k> - m) for this wave's 16 keys, in three steps that the loop below
    // spreads over an iteration so that no step waits on the one before it: operand reads, logits (MFMA), exp + store.
    bf16x8 knf[NF];
    auto weights_load = [&](int buf) {
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            knf[f] = *reinterpret_cast<const bf16x8 *>(&kn[buf][kn_r[f]]);
            if (Q_IN_LDS) qf[f] = *reinterpret_cast<const bf16x8 *>(&sm.qt[nn][32 * f + 8 * g]);
        }
    };
    auto weights_logits = [&]() {
        f32x4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int f = 0; f < NF; ++f) z = mfma_bf16(knf[f], qf[f], z);
        return z;
    };
    // blocks 0 .. n_unmasked - 1 lie wholly before the workgroup's first query (causal) or wholly inside the sequence
    // (not causal): no key of theirs is masked for any query of the workgroup
    const int n_unmasked = QB == 16 ? (causal ? (i0 + 1) / KB2 : n / KB2) : 0;
    auto weights_store = [&](int blk, int buf, f32x4 z) {
        float wf[4];
        // A block that lies wholly before the workgroup's first query needs no causal mask (a scalar condition; most
        // blocks of a long row)
#pragma unroll
        for (int r = 0; r < 4; ++r) wf[r] = __builtin_amdgcn_exp2f(z[r] * cscale - mrow);
        if (blk >= n_unmasked) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int j = blk * KB2 + 16 * wave + 4 * g + r;
                wf[r] = (q_live && j <= jlim) ? wf[r] : 0.f;
            }
        }
        // stored negated: the tiles accumulate -(w k) k^T
        if (PRECISE) {
            *reinterpret_cast<f32x4 *>(&wt32[buf][nn * WT32_PITCH + 16 * wave + 4 * g]) = f32x4{-wf[0], -wf[1], -wf[2], -wf[3]};
            if (!OM_MFMA) om_part += (wf[0] + wf[1]) + (wf[2] + wf[3]);
        } else {
            half4 wv;
#pragma unroll
            for (int r = 0; r < 4; ++r) wv[r] = (_Float16)wf[r];
            if (!OM_MFMA) {
                // omega sums the weights exactly as the MFMAs see them: products with 1 are exact, the sum is fp32
                typedef _Float16 half2v __attribute__((ext_vector_type(2)));
                const half2v one = {(_Float16)1.f, (_Float16)1.f};
                om_part = __builtin_amdgcn_fdot2(half2v{wv[0], wv[1]}, one, om_part, false);
                om_part = __builtin_amdgcn_fdot2(half2v{wv[2], wv[3]}, one, om_part, false);
            }
            *reinterpret_cast<half4 *>(&wt[buf][nn * WT_PITCH + 16 * wave + 4 * g]) = -wv;     // the sign bits of two registers
        }
    };

    // Operand fragments of one half (32 keys) of a block: the NB feature blocks of the transposed tile, and
    // this wave's feature block for mu~ (re-read from LDS: indexing f[] by the wave id would become a
    // per-element select chain).  Two sets, so that the next half is in flight while this one is consumed.
    struct Frags { half8 f[NB]; };
    Frags fa, fb;
    auto load_frags = [&](Frags &fr, int buf, int hf) {
#pragma unroll
        for (int I = 0; I < LIVE; ++I) fr.f[I] = *reinterpret_cast<const half8 *>(&kt[buf][hf][kt_r + I * 512]);
    };
    // The MFMAs of work items [lo, hi) of one half; item = (query q, feature block I), q-major.  wb = weight buffer.
    auto compute_items = [&](const Frags &fr, int wb, int hf, int lo, int hi) {
        if (!PRECISE && DD == 128) {
            // one query per wave: the scaled operand of item I + 1 is formed behind the MFMAs of item I, two multiplies
            // per MFMA (see pipe_query for why the two kinds alternate); 1.3 % at [1,16,8192,128]
            const _Float16 *wrow = &wt[wb][QW * wave * WT_PITCH + 32 * hf + 8 * g];
            const half8 wq = *reinterpret_cast<const half8 *>(wrow);
            half8 af = fr.f[lo] * wq;
#pragma unroll
            for (int I = lo; I < hi; ++I) {
                const half8 afn = fr.f[I + 1 < NB ? I + 1 : I] * wq;
#pragma unroll
                for (int J = I; J < NB; ++J) acc[0][S::tix(I, J)] = mfma_f16(af, fr.f[J], acc[0][S::tix(I, J)]);
                af = afn;
            }
#define SGB_MV() __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); __builtin_amdgcn_sched_group_barrier(0x002, 2, 0)
#define SGB_MV6() SGB_MV(); SGB_MV(); SGB_MV(); SGB_MV(); SGB_MV(); SGB_MV()
            if (lo == 0 && hi == NB) {
                __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
                SGB_MV6(); SGB_MV6(); SGB_MV6(); SGB_MV6(); SGB_MV6(); SGB_MV6();
            }
#undef SGB_MV6
#undef SGB_MV
        } else if (!PRECISE) {
            // the query's 8 weights of this lane's key chunk: one address per lane group (an LDS broadcast read)
            const _Float16 *wrow = &wt[wb][QW * wave * WT_PITCH + 32 * hf + 8 * g];
            half8 wq = *reinterpret_cast<const half8 *>(wrow + (lo / NB) * WT_PITCH);
#pragma unroll
            for (int it = lo; it < hi; ++it) {
                const int q = it / NB, I = it % NB;
                if (I == 0 && it != lo) wq = *reinterpret_cast<const half8 *>(wrow + q * WT_PITCH);
                if (I >= LIVE) continue;
                const half8 af = fr.f[I] * wq;
#pragma unroll
                for (int J = I; J < LIVE; ++J) acc[q][S::tix(I, J)] = mfma_f16(af, fr.f[J], acc[q][S::tix(I, J)]);
            }
        } else {
            float wq[8];
#pragma unroll
            for (int it = lo; it < hi; ++it) {
                const int q = it / NB, I = it % NB;
                if (I >= LIVE) continue;
                if (I == 0 || it == lo) {
                    const float *wp = &wt32[wb][(QW * wave + q) * WT32_PITCH + 32 * hf + 8 * g];
                    const f32x4 w0 = *reinterpret_cast<const f32x4 *>(wp), w1 = *reinterpret_cast<const f32x4 *>(wp + 4);
#pragma unroll
                    for (int t = 0; t < 4; ++t) { wq[t] = w0[t]; wq[4 + t] = w1[t]; }
                }
                half8 ahi, alo;
                float pr[8];
#pragma unroll
                for (int t = 0; t < 8; ++t) pr[t] = (float)fr.f[I][t] * wq[t];
                split_f16(pr, ahi, alo);
#pragma unroll
                for (int J = I; J < LIVE; ++J) {
                    acc[q][S::tix(I, J)] = mfma_f16(alo, fr.f[J], acc[q][S::tix(I, J)]);
                    acc[q][S::tix(I, J)] = mfma_f16(ahi, fr.f[J], acc[q][S::tix(I, J)]);
                }
            }
        }
    };
    // One query of one half with the vector and matrix-core instructions alternating: a wave's multiplies and MFMAs
    // overlap only when they alternate (a run of four multiplies followed by a run of MFMAs costs the sum of the two),
    // so the scaled operand of the NEXT item -- the next query's first item included, across halves and blocks -- is
    // formed two multiplies at a time behind the MFMAs of this one.  pipe_af / pipe_wq carry that operand and the
    // query's weights from one call to the next; frn and (wbn, hfn, qn) say where the next query's operands are.
    half8 pipe_af, pipe_wq;
    auto wq_read = [&](int wbuf, int hf, int q) {
        return *reinterpret_cast<const half8 *>(&wt[wbuf][(QW * wave + q) * WT_PITCH + 32 * hf + 8 * g]);
    };
    auto pipe_query = [&](const Frags &fr, int q, const Frags &frn, int wbn, int hfn, int qn) {
        const half8 wq_next = wq_read(wbn, hfn, qn);
        half8 af = pipe_af;
#pragma unroll
        for (int I = 0; I < LIVE; ++I) {
            const half8 afn = I + 1 < LIVE ? fr.f[I + 1] * pipe_wq : frn.f[0] * wq_next;
#pragma unroll
            for (int J = I; J < LIVE; ++J) acc[q][S::tix(I, J)] = mfma_f16(af, fr.f[J], acc[q][S::tix(I, J)]);
            af = afn;
        }
        pipe_af = af;
        pipe_wq = wq_next;
#define SGB_MV() __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); __builtin_amdgcn_sched_group_barrier(0x002, 2, 0)
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        if constexpr (LIVE == NB) {
            SGB_MV(); SGB_MV(); SGB_MV(); SGB_MV(); SGB_MV(); SGB_MV(); SGB_MV(); SGB_MV();
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        } else {
            // LIVE (LIVE + 1) / 2 MFMAs and 4 LIVE multiplies: more vector than matrix work, two multiplies behind each MFMA
#pragma unroll
            for (int m = 0; m < LIVE * (LIVE + 1) / 2; ++m) { SGB_MV(); }
        }
#undef SGB_MV
        __builtin_amdgcn_sched_barrier(0);
    };
    // -mu~ of one half: the (negated) weights of all 16 query rows are the A operand (lane (g, nn): row nn, keys
    // 8g..8g+7), this wave's feature block of the tile the B operand (re-read from LDS: indexing f[] by the wave
    // id would become a per-element select chain).  Operands are fetched by mu_load_a / mu_load_b, consumed by mu_mfma.
    half8 mu_a, mu_a2, mu_b;
    auto mu_load_b = [&](int buf, int hf) { mu_b = *reinterpret_cast<const half8 *>(&kt[buf][hf][kt_r + wave * 512]); };
    auto mu_load_a = [&](int wb, int hf) {
        if (!PRECISE) {
            mu_a = *reinterpret_cast<const half8 *>(&wt[wb][nn * WT_PITCH + 32 * hf + 8 * g]);
        } else {
            const float *wp = &wt32[wb][nn * WT32_PITCH + 32 * hf + 8 * g];
            const f32x4 w0 = *reinterpret_cast<const f32x4 *>(wp), w1 = *reinterpret_cast<const f32x4 *>(wp + 4);
            float wv[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) wv[t] = t < 4 ? w0[t] : w1[t - 4];
            split_f16(wv, mu_a, mu_a2);
        }
    };
    // omega rides on the same A operand with a tile of ones as B: it sums the weights exactly as the MFMAs of the
    // other moments see them, and costs one wave one MFMA per half instead of every weight wave eight vector
    // instructions per block (which compete with the MFMAs for the issue port)
    constexpr int OM_WAVE = NW - 1;
    half8 ones;
#pragma unroll
    for (int t = 0; t < 8; ++t) ones[t] = (_Float16)1.f;
    auto mu_mfma = [&]() {
        if (PRECISE) mu_acc = mfma_f16(mu_a2, mu_b, mu_acc);
        mu_acc = mfma_f16(mu_a, mu_b, mu_acc);          // -mu~[row 4g + r][feature 16 wave + nn]
        if (OM_MFMA && wave == OM_WAVE) {
            if (PRECISE) om_acc = mfma_f16(mu_a2, ones, om_acc);
            om_acc = mfma_f16(mu_a, ones, om_acc);      // -omega[row 4g + r] in every column
        }
    };

    // Software pipeline over blocks of 64 keys, one barrier per block, placed between its two halves:
    //   first half of block c : fragments of its second half are fetched from LDS meanwhile; the weights of
    //                           block c+1 are produced on the side (their key rows were fetched by this very
    //                           wave, so its own vmcnt wait suffices) and stored before the barrier;
    //   barrier               : block c+1 (tiles of all waves, weights) is now visible, and nobody reads the
    //                           tiles of block c any more, so the DMA of block c+2 may overwrite them;
    //   second half of block c: fragments of the first half of block c+1 are fetched meanwhile.
    // The weights live in three buffers: a wave that is ahead writes the weights of block c+1 while one that
    // is behind still reads those of block c-1.  Past the last block every key is masked (j > iq): that extra
    // round stores zeros.  `wave` is a scalar, so every branch around an MFMA is a real branch (MFMA ignores EXEC).
    constexpr int ITEMS = QW * NB, Q2 = ITEMS / 2, Q3 = 3 * ITEMS / 4;
    // A second fragment set: d = 128 has no registers for one, nor has the forward's fp32-accurate variant (it spilled 55
    // registers per block with it).  The backward's kernel keeps it in both variants: without it the allocator, which
    // works on the whole kernel, spills the transfer offsets of the fast variant instead (5 % of that kernel).
    constexpr bool PREFETCH = (DD == 64) && (!PRECISE || WITH_U);
    issue_dma(0);
    if (PREFETCH && nblk > 1) issue_dma(1);
    dma_wait();
    __syncthreads();
    if (w_wave) { weights_load(0); weights_store(0, 0, weights_logits()); }
    __syncthreads();

    int wb = 0;                                 // weight buffer of block c
    // Two workgroups share a compute unit, one wave of each per SIMD.  A wave in the main loop (matrix-core bound) gets
    // the issue slot before one that is in its solve (long vector-ALU chains that leave the matrix cores idle): 2.5 %
    // at [4,16,4096,64].
    __builtin_amdgcn_s_setprio(2);
    if (PIPE) {
        load_frags(fa, 0, 0);
        pipe_wq = wq_read(0, 0, 0);
        pipe_af = fa.f[0] * pipe_wq;
        // Unrolled four times with the tile buffer (c % 2) and the weight buffer (c % 4; four of them instead of the
        // three that are needed, so that the two periods divide the unroll factor) as compile-time constants: every LDS
        // address of the loop is then a per-lane register plus an immediate, and the dozen vector additions per block
        // that added the buffers' offsets are gone.
        // (The backward's variant of this kernel, which carries a second right-hand side through the solve and has fewer
        // registers to spare, keeps the buffers as run-time values: unrolled it spills heavily inside the loop.)
        auto pipe_block = [&](int c, auto ktag) {
            constexpr int KK = decltype(ktag)::value;
            const int buf = KK >= 0 ? (KK & 1) : (c & 1), wb = KK >= 0 ? (KK & 3) : (c & 3), wbn = (wb + 1) & 3;
            // ---- first half ---------------------------------------------------------------------------
            load_frags(fb, buf, 1);
            __builtin_amdgcn_sched_barrier(0);
            pipe_query(fa, 0, fa, wb, 0, 1);
            pipe_query(fa, 1, fa, wb, 0, 2);
            dma_wait();                         // this wave's part of block c+1 has landed
            weights_load(buf ^ 1);
            mu_load_b(buf, 0);
            mu_load_a(wb, 0);
            __builtin_amdgcn_sched_barrier(0);
            pipe_query(fa, 2, fa, wb, 0, 3);
            f32x4 z = weights_logits();
            mu_mfma();
            __builtin_amdgcn_sched_barrier(0);
            pipe_query(fa, 3, fb, wb, 1, 0);
            weights_store(c + 1, wbn, z);
            mu_load_b(buf, 1);                  // the last read of block c's tiles: they are overwritten after the barrier
            // ---- second half (its fragments are in registers already) ----------------------------------
            mu_load_a(wb, 1);
            __builtin_amdgcn_sched_barrier(0);
            pipe_query(fb, 0, fb, wb, 1, 1);
            // The block's barrier comes one query into the second half: the exponentials, the conversion and the LDS
            // write of the weights, and the skew between the waves, then pass behind ten MFMAs instead of in front of
            // an idle matrix pipe.  What the barrier orders is unchanged: the weights of block c + 1 are first read by
            // the last query of this half, the tiles of block c + 1 right below, and the tiles of block c were last
            // read above.
            __syncthreads();
            if (c + 2 < nblk) issue_dma(c + 2);
            load_frags(fa, buf ^ 1, 0);         // first half of block c+1 (unused after the last block)
            __builtin_amdgcn_sched_barrier(0);
            pipe_query(fb, 1, fb, wb, 1, 2);
            pipe_query(fb, 2, fb, wb, 1, 3);
            mu_mfma();
            __builtin_amdgcn_sched_barrier(0);
            pipe_query(fb, 3, fa, wbn, 0, 0);   // after the last block: the all-zero round of weights, operand unused
        };
        if constexpr (!WITH_U) {
            for (int c = 0; c < nblk; c += 4) {
                pipe_block(c, std::integral_constant<int, 0>{});
                if (c + 1 < nblk) pipe_block(c + 1, std::integral_constant<int, 1>{});
                if (c + 2 < nblk) pipe_block(c + 2, std::integral_constant<int, 2>{});
                if (c + 3 < nblk) pipe_block(c + 3, std::integral_constant<int, 3>{});
            }
        } else {
            for (int c = 0; c < nblk; ++c) pipe_block(c, std::integral_constant<int, -1>{});
        }
    } else if (PREFETCH) {
        load_frags(fa, 0, 0);
        for (int c = 0; c < nblk; ++c) {
            const int buf = c & 1, wbn = (wb == 2) ? 0 : wb + 1;
            // ---- first half ---------------------------------------------------------------------------
            load_frags(fb, buf, 1);
            __builtin_amdgcn_sched_barrier(0);
            compute_items(fa, wb, 0, 0, Q2);
            __builtin_amdgcn_sched_barrier(0);
            dma_wait();                         // this wave's part of block c+1 has landed
            if (NW == 4 || w_wave) weights_load(buf ^ 1);
            mu_load_b(buf, 0);
            mu_load_a(wb, 0);
            __builtin_amdgcn_sched_barrier(0);
            compute_items(fa, wb, 0, Q2, Q3);
            f32x4 z = {0.f, 0.f, 0.f, 0.f};
            if (NW == 4 || w_wave) z = weights_logits();
            mu_mfma();
            compute_items(fa, wb, 0, Q3, ITEMS);
            __builtin_amdgcn_sched_barrier(0);
            if (NW == 4 || w_wave) weights_store(c + 1, wbn, z);
            mu_load_b(buf, 1);                  // the last read of block c's tiles: they are overwritten after the barrier
            __syncthreads();
            if (c + 2 < nblk) issue_dma(c + 2);
            // ---- second half --------------------------------------------------------------------------
            load_frags(fa, buf ^ 1, 0);         // first half of block c+1 (unused after the last block)
            mu_load_a(wb, 1);
            __builtin_amdgcn_sched_barrier(0);
            compute_items(fb, wb, 1, 0, Q3);
            mu_mfma();
            compute_items(fb, wb, 1, Q3, ITEMS);
            __builtin_amdgcn_sched_barrier(0);
            wb = wbn;
        }
    } else {
        // One fragment set: the barrier sits at the end of the block, the DMA of block c+1 is issued at its
        // start, and each half fetches its own fragments; the weights of block c+1 are produced around the
        // second half.
        for (int c = 0; c < nblk; ++c) {
            const int buf = c & 1, wbn = (wb == 2) ? 0 : wb + 1;
            if (c + 1 < nblk) issue_dma(c + 1);
            load_frags(fa, buf, 0);
            mu_load_b(buf, 0);
            mu_load_a(wb, 0);
            compute_items(fa, wb, 0, 0, ITEMS);
            mu_mfma();
            __builtin_amdgcn_sched_barrier(0);
            dma_wait();                         // this wave's part of block c+1 has landed
            if (w_wave) weights_load(buf ^ 1);
            load_frags(fa, buf, 1);
            mu_load_b(buf, 1);
            mu_load_a(wb, 1);
            __builtin_amdgcn_sched_barrier(0);
            f32x4 z = {0.f, 0.f, 0.f, 0.f};
            if (w_wave) z = weights_logits();
            compute_items(fa, wb, 1, 0, ITEMS);
            mu_mfma();
            __builtin_amdgcn_sched_barrier(0);
            if (w_wave) weights_store(c + 1, wbn, z);
            __syncthreads();
            wb = wbn;
        }
    }


    // ---- hand mu~ and omega to the waves that own the queries ---------------------------------------
    // From here on the lane coordinates are taken from copies the optimiser cannot see through: every LDS and global
    // address of the epilogue and of the solve is a function of them, the optimiser would compute all of those before
    // the main loop (they are loop-invariant) and then spill them across it, for want of registers there.
    int g_e = g, nn_e = nn;
    asm volatile("" : "+v"(g_e), "+v"(nn_e));
    __builtin_amdgcn_s_setprio(0);
#define g g_e
#define nn nn_e
#pragma unroll
    for (int r = 0; r < 4; ++r) mus[4 * g + r][16 * wave + nn] = mu_acc[r];   // -mu~ (negated weights)
    if (OM_MFMA) {
        if (wave == OM_WAVE && nn == 0) {
#pragma unroll
            for (int r = 0; r < 4; ++r) oms[4 * g + r] = -om_acc[r];
        }
        __syncthreads();
    } else {
        // lanes (g, nn) of the four weight waves hold partial sums for query row nn
        om_part += __shfl_xor(om_part, 16);
        om_part += __shfl_xor(om_part, 32);
        if (w_wave && g == 0) sm.omp[wave][nn] = om_part;
        __syncthreads();
        if (tid < 16) oms[tid] = (sm.omp[0][tid] + sm.omp[1][tid]) + (sm.omp[2][tid] + sm.omp[3][tid]);
        __syncthreads();
    }

    // ---- per-query solve ---------------------------------------------------------------------------------------
    if constexpr (DD == 64) {
        // four queries per wave: blocked factorisation on the matrix cores, substitutions on the vector ALU with lane
        // (q, r) = (g, nn) holding element r of every 16-block of query q's vectors (see solve_wave_q4)
        const int qi = QW * wave + g;
        const int row = min(i0 + qi, n - 1);
        const bf16_t *qrow = Qh + (int64_t)row * sq.seq;
        const float pivot_floor = 0.5f * (lam_rows ? lam_rows[(size_t)bh * n + row] : lambda);
        float tmu[4], tq[4], te[4], y1[4], u1[4], y0 = 0.f, u0 = 0.f, r0 = 0.f;
#pragma unroll
        for (int P = 0; P < NB; ++P) {
            tmu[P] = mus[qi][16 * P + nn];                               // mus holds -mu~
            tq[P] = -bf16_to_f32(qrow[16 * P + nn]);
            te[P] = 0.f; y1[P] = 0.f; u1[P] = 0.f;
            if constexpr (WITH_U) te[P] = -Rg[((size_t)bh * n + row) * YP + 16 * P + nn];
        }
        if constexpr (WITH_U) r0 = Rg[((size_t)bh * n + row) * YP + DD];
        solve_wave_q4<WITH_U, LIVE>(acc, tmu, tq, te, r0, oms[qi], &sc[wave][0][0], g, nn, pivot_floor, y1, y0, u1, u0);
        if (i0 + qi < n) {
            float *yr = Yg + ((size_t)bh * n + row) * YP;
#pragma unroll
            for (int P = 0; P < NB; ++P) yr[16 * P + nn] = y1[P];
            if (nn == 0) yr[DD] = y0;
            if constexpr (WITH_U) {
                float *ur = Ug + ((size_t)bh * n + row) * YP;
#pragma unroll
                for (int P = 0; P < NB; ++P) ur[16 * P + nn] = u1[P];
                if (nn == 0) ur[DD] = u0;
            }
        }
    } else {
    f32x4 rhs[QW][NB];
    float y0v[QW], om4[QW];
#pragma unroll
    for (int q = 0; q < QW; ++q) om4[q] = oms[QW * wave + q];
    const int gq_row = min(i0 + QW * wave + (g < QW ? g : QW - 1), n - 1);
    const float pivot_floor = 0.5f * (lam_rows ? lam_rows[(size_t)bh * n + gq_row] : lambda);
    float r0v[QW], u0v[QW];
    if constexpr (WITH_U) {
#pragma unroll
        for (int q = 0; q < QW; ++q) r0v[q] = Rg[((size_t)bh * n + min(i0 + QW * wave + q, n - 1)) * YP + DD];
    }
    // one query per wave: factorisation on the matrix cores, substitutions on the vector ALU (solve_wave_v1)
    static_assert(QW == 1, "the general path serves d = 128, one query per wave");
    {
        const int row = min(i0 + wave, n - 1);
        const bf16_t *qrow = Qh + (int64_t)row * sq.seq;
        const float *rrow = WITH_U ? Rg + ((size_t)bh * n + row) * YP : nullptr;
        solve_wave_v1<DD, WITH_U>(acc, rhs, y0v, om4, &sc[wave][0][0], g, nn, pivot_floor,
                                  [&](int P, float &m, float &q, float &e) {
                                      m = mus[wave][16 * P + nn];                 // mus holds -mu~
                                      q = -bf16_to_f32(qrow[16 * P + nn]);
                                      if constexpr (WITH_U) e = -rrow[16 * P + nn];
                                  },
                                  r0v, u0v);
    }

#pragma unroll
    for (int q = 0; q < QW; ++q) {
        const int i = i0 + QW * wave + q;
        if (i < n && nn == 0) {
            float *yr = Yg + ((size_t)bh * n + i) * YP;
#pragma unroll
            for (int P = 0; P < NB; ++P) *reinterpret_cast<f32x4 *>(yr + 16 * P + 4 * g) = rhs[q][P];
            if (g == 0) yr[DD] = y0v[q];
        }
        if constexpr (WITH_U) {
            if (i < n && nn == 1) {
                float *ur = Ug + ((size_t)bh * n + i) * YP;
#pragma unroll
                for (int P = 0; P < NB; ++P) *reinterpret_cast<f32x4 *>(ur + 16 * P + 4 * g) = rhs[q][P];
                if (g == 0) ur[DD] = u0v[q];
            }
        }
    }
    }
#undef g
#undef nn
}

// One launch serves every query block: blocks whose rows lie below precise_rows take the precise
// variant.  The choice depends on blockIdx only, so it is a scalar branch (MFMA ignores EXEC).
template <int DD, int LIVE = Shape<DD>::NB>
__global__ __launch_bounds__(Shape<DD>::NT, DD == 64 ? 2 : 1) void moments_kernel(
    const bf16_t *__restrict__ Qg, const bf16_t *__restrict__ Kg, llla_strides sq, llla_strides sk, int H, int n, int nkb,
    int precise_rows, float cscale, float lambda, const float *__restrict__ lam_rows, const _Float16 *__restrict__ KT,
    const float *__restrict__ Mg, float *__restrict__ Yg, int causal)
{
    __shared__ __align__(16) MomentsShared<DD> sm;
    const int i0 = ((int)gridDim.x - 1 - moments_block<DD>().blk) * Shape<DD>::QB;
    if (i0 < precise_rows)
        moments_body<true, DD, false, LIVE>(sm, Qg, Kg, sq, sk, H, n, nkb, cscale, lambda, lam_rows, KT, Mg, Yg, nullptr, nullptr, causal);
    else
        moments_body<false, DD, false, LIVE>(sm, Qg, Kg, sq, sk, H, n, nkb, cscale, lambda, lam_rows, KT, Mg, Yg, nullptr, nullptr, causal);
}

// The same with the backward's second system (see moments_body).
template <int DD, int LIVE = Shape<DD>::NB>
__global__ __launch_bounds__(Shape<DD>::NT, DD == 64 ? 2 : 1) void moments_u_kernel(
    const bf16_t *__restrict__ Qg, const bf16_t *__restrict__ Kg, llla_strides sq, llla_strides sk, int H, int n, int nkb,
    int precise_rows, float cscale, float lambda, const float *__restrict__ lam_rows, const _Float16 *__restrict__ KT,
    const float *__restrict__ Mg, float *__restrict__ Yg, const float *__restrict__ Rg, float *__restrict__ Ug)
{
    __shared__ __align__(16) MomentsShared<DD> sm;
    const int i0 = ((int)gridDim.x - 1 - moments_block<DD>().blk) * Shape<DD>::QB;
    if (i0 < precise_rows)
        moments_body<true, DD, true, LIVE>(sm, Qg, Kg, sq, sk, H, n, nkb, cscale, lambda, lam_rows, KT, Mg, Yg, Rg, Ug);
    else
        moments_body<false, DD, true, LIVE>(sm, Qg, Kg, sq, sk, H, n, nkb, cscale, lambda, lam_rows, KT, Mg, Yg, Rg, Ug);
}

// Optional statistics of Eq. (lla) from the solved y of every row: with y1 = -rho/delta and
// y0 = (1 + q.rho)/delta, 1/delta = y0 + q.y1 and rho = -delta y1.  One wave per row.
template <int DD>
__global__ __launch_bounds__(256) void stats_kernel(const bf16_t *__restrict__ Qg, llla_strides sq, int H, int n,
                                                    const float *__restrict__ Yg, float *__restrict__ rho,
                                                    float *__restrict__ delta)
{
    constexpr int YP = Shape<DD>::YP, PER = DD / 64;
    const int lane = threadIdx.x % 64, i = blockIdx.x * 4 + threadIdx.x / 64, bh = blockIdx.y;
    if (i >= n) return;
    const bf16_t *qrow = Qg + (bh / H) * sq.batch + (bh % H) * sq.head + (int64_t)i * sq.seq;
    const float *yr = Yg + ((size_t)bh * n + i) * YP;
    float y1[PER], qy = 0.f;
#pragma unroll
    for (int t = 0; t < PER; ++t) {
        y1[t] = yr[lane + 64 * t];
        qy = fmaf(bf16_to_f32(qrow[lane + 64 * t]), y1[t], qy);
    }
#pragma unroll
    for (int sft = 32; sft >= 1; sft >>= 1) qy += __shfl_xor(qy, sft);
    const float dl = 1.f / (yr[DD] + qy);
    const size_t row = (size_t)bh * n + i;
    if (delta != nullptr && lane == 0) delta[row] = dl;
    if (rho != nullptr) {
#pragma unroll
        for (int t = 0; t < PER; ++t) rho[row * DD + lane + 64 * t] = -dl * y1[t];
    }
}

template <int DD>
hipError_t forward_impl(const Problem &p)
{
    using S = Shape<DD>;
    const Layout L = make_layout<DD>(p.B, p.H, p.n);
    char *ws = static_cast<char *>(p.ws);
    _Float16 *KT = reinterpret_cast<_Float16 *>(ws + L.kt);
    bf16_t *VT = reinterpret_cast<bf16_t *>(ws + L.vt);
    float *M = reinterpret_cast<float *>(ws + L.m);
    float *Y = reinterpret_cast<float *>(ws + L.y);
    const int bh = p.B * p.H;
    const float cscale = p.scale * LOG2E;
    // rows whose visible keys number at most 2 d take the precise moments and the fp32 output sweep: the first 2 d
    // rows of a causal call; every row of a non-causal call over at most 2 d keys, none of a longer one
    const int first = p.causal ? (S::EARLY_ROWS < p.n ? S::EARLY_ROWS : p.n) : (p.n <= S::EARLY_ROWS ? p.n : 0);

    const bf16_t *Q = static_cast<const bf16_t *>(p.Q), *K = static_cast<const bf16_t *>(p.K),
                 *V = static_cast<const bf16_t *>(p.V);
    stage_mark(p.stream, "prep");
    hipLaunchKernelGGL((prep_kernel<DD>), dim3(L.nkb, bh), dim3(256), 0, p.stream, K, V, p.sk, p.sv, p.H, p.n, L.nkb, KT, VT);
    const int nq64 = (p.n + 63) / 64;
    stage_mark(p.stream, "rowmax");
    // a call at d = 16 / 32 on zero-padded copies (live_d features can be non-zero): the variants that skip padded tiles
    const int live = (DD == 64 && p.live_d > 0) ? (p.live_d + 15) / 16 : S::NB;
    if constexpr (DD == 64) {
        if (live == 1)
            hipLaunchKernelGGL((sweep_kernel<true, DD, 1>), dim3(bh, nq64), dim3(256), 0, p.stream, Q, K, p.sq, p.sk, p.H, p.n,
                               L.nkb, 0, cscale, VT, M, Y, p.O, p.so, 0, (float *)nullptr, p.causal);
        else if (live == 2)
            hipLaunchKernelGGL((sweep_kernel<true, DD, 2>), dim3(bh, nq64), dim3(256), 0, p.stream, Q, K, p.sq, p.sk, p.H, p.n,
                               L.nkb, 0, cscale, VT, M, Y, p.O, p.so, 0, (float *)nullptr, p.causal);
    }
    if (live == S::NB)
        hipLaunchKernelGGL((sweep_kernel<true, DD>), dim3(bh, nq64), dim3(256), 0, p.stream, Q, K, p.sq, p.sk, p.H, p.n, L.nkb,
                           0, cscale, VT, M, Y, p.O, p.so, 0, (float *)nullptr, p.causal);
    const int nqb = (p.n + S::QB - 1) / S::QB;
    stage_mark(p.stream, "moments");
    if constexpr (DD == 64) {
        if (live == 1)
            hipLaunchKernelGGL((moments_kernel<DD, 1>), dim3(nqb, bh), dim3(S::NT), 0, p.stream, Q, K, p.sq, p.sk, p.H, p.n,
                               L.nkb, first, cscale, p.lambda, p.lambda_rows, KT, M, Y, p.causal);
        else if (live == 2)
            hipLaunchKernelGGL((moments_kernel<DD, 2>), dim3(nqb, bh), dim3(S::NT), 0, p.stream, Q, K, p.sq, p.sk, p.H, p.n,
                               L.nkb, first, cscale, p.lambda, p.lambda_rows, KT, M, Y, p.causal);
    }
    if (live == S::NB)
        hipLaunchKernelGGL((moments_kernel<DD>), dim3(nqb, bh), dim3(S::NT), 0, p.stream, Q, K, p.sq, p.sk, p.H, p.n, L.nkb,
                           first, cscale, p.lambda, p.lambda_rows, KT, M, Y, p.causal);
    if (p.rho != nullptr || p.delta != nullptr) {
        stage_mark(p.stream, "statistics");
        hipLaunchKernelGGL((stats_kernel<DD>), dim3((p.n + 3) / 4, bh), dim3(256), 0, p.stream, Q, p.sq, p.H, p.n, Y, p.rho,
                           p.delta);
    }
    // output: those rows are evaluated in fp32 on the vector ALUs (their weights y0 + k.y1 cancel
    // to a few digits), the rest by the MFMA sweep
    if (first > 0) {
        stage_mark(p.stream, "output_early_rows");
        const hipError_t e = valu_forward_given(p, first, M, L.npad, Y, S::YP);
        if (e != hipSuccess) return e;
    }
    if (first < p.n) {
        const int nq64b = (p.n - first + 63) / 64;
        stage_mark(p.stream, "output");
        const int obf = p.out == LLLA_BF16 ? 1 : 0;
        if constexpr (DD == 64) {
            if (live == 1)
                hipLaunchKernelGGL((sweep_kernel<false, DD, 1>), dim3(bh, nq64b), dim3(256), 0, p.stream, Q, K, p.sq, p.sk, p.H,
                                   p.n, L.nkb, first, cscale, VT, M, Y, p.O, p.so, obf, (float *)nullptr, p.causal);
            else if (live == 2)
                hipLaunchKernelGGL((sweep_kernel<false, DD, 2>), dim3(bh, nq64b), dim3(256), 0, p.stream, Q, K, p.sq, p.sk, p.H,
                                   p.n, L.nkb, first, cscale, VT, M, Y, p.O, p.so, obf, (float *)nullptr, p.causal);
        }
        if (live == S::NB)
            hipLaunchKernelGGL((sweep_kernel<false, DD>), dim3(bh, nq64b), dim3(256), 0, p.stream, Q, K, p.sq, p.sk, p.H, p.n,
                               L.nkb, first, cscale, VT, M, Y, p.O, p.so, obf, (float *)nullptr, p.causal);
    }
    return hipGetLastError();
}


// ------------------------------------------------------------------------------------------------
// Approximate mode of the paper (Section 3.1 "matrix-free inversion", solver of Appendix C): rho_i from T steps of
// conjugate gradients on Sigma_i rho = mu_i, Sigma_i applied matrix-free,
//     Sigma p = sum_j w_j (k_j . p) k_j - (q . p) mu~ - (mu~ . p) q + omega (q . p) q + lambda p.
// The sum over keys is one sweep_kernel launch per step (coefficients w_ij (k_j . p_i), tile = K); the vector part of a
// step is the row-wise kernel below (one wave per query row).  A row whose residual norm is at or below eps when a
// step starts is frozen (the paper's active mask).
struct CgLayout {
    Layout base;
    size_t ktb, mut, om, x, r, p, sp, rr, it, total;
};

template <int DD>
CgLayout make_cg_layout(int B, int H, int n)
{
    CgLayout C;
    C.base = make_layout<DD>(B, H, n);
    const size_t bh = (size_t)B * H, rows = bh * (size_t)n;
    size_t off = C.base.total;
    C.ktb = off; off += round_up(bh * C.base.npad * DD * 2, 256);        // K re-tiled as bf16 (tile operand of the sweeps)
    C.mut = off; off += round_up(rows * DD * 4, 256);                      // mu~
    C.om = off;  off += round_up(rows * 4, 256);                           // omega
    C.x = off;   off += round_up(rows * DD * 4, 256);
    C.r = off;   off += round_up(rows * DD * 4, 256);
    C.p = off;   off += round_up(rows * Shape<DD>::YP * 4, 256);           // search direction, laid out like a y row
    C.sp = off;  off += round_up(rows * DD * 4, 256);                      // sum_j w_j (k_j . p) k_j
    C.rr = off;  off += round_up(rows * 4, 256);
    C.it = off;  off += round_up(rows * 4, 256);                           // steps done; negative once frozen
    C.total = off;
    return C;
}

template <int DD>
__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int sft = 32; sft >= 1; sft >>= 1) v += __shfl_xor(v, sft);
    return v;
}

// phase 0: start (mu = mu~ - omega q; X = 0, R = P = mu);  phase 1: one CG step;  phase 2: rho, delta -> y (+ outputs)
template <int DD, int PHASE>
__global__ __launch_bounds__(256) void cg_rows_kernel(const bf16_t *__restrict__ Qg, llla_strides sq, int H, int n,
                                                      float lambda, float eps, const float *__restrict__ MUt,
                                                      const float *__restrict__ OM, float *__restrict__ X,
                                                      float *__restrict__ R, float *__restrict__ P,
                                                      const float *__restrict__ SP, float *__restrict__ RR,
                                                      int *__restrict__ IT, float *__restrict__ Yg,
                                                      float *__restrict__ rho, float *__restrict__ delta,
                                                      int32_t *__restrict__ iters)
{
    constexpr int YP = Shape<DD>::YP, PER = DD / 64;
    const int lane = threadIdx.x % 64, i = blockIdx.x * 4 + threadIdx.x / 64, bh = blockIdx.y;
    if (i >= n) return;
    const size_t row = (size_t)bh * n + i;
    const bf16_t *qrow = Qg + (bh / H) * sq.batch + (bh % H) * sq.head + (int64_t)i * sq.seq;
    float q[PER], mut[PER];
#pragma unroll
    for (int t = 0; t < PER; ++t) {
        q[t] = bf16_to_f32(qrow[lane + 64 * t]);
        mut[t] = MUt[row * DD + lane + 64 * t];
    }
    const float om = OM[row];
    if (PHASE == 0) {
        float rr = 0.f;
#pragma unroll
        for (int t = 0; t < PER; ++t) {
            const float mu = mut[t] - om * q[t];
            X[row * DD + lane + 64 * t] = 0.f;
            R[row * DD + lane + 64 * t] = mu;
            P[row * YP + lane + 64 * t] = mu;
            rr = fmaf(mu, mu, rr);
        }
        rr = wave_sum<DD>(rr);
        if (lane == 0) { RR[row] = rr; IT[row] = 0; P[row * YP + DD] = 0.f; }
    } else if (PHASE == 1) {
        const int it = IT[row];
        if (it < 0) return;                                     // frozen
        const float rr = RR[row];
        if (sqrtf(rr) <= eps) { if (lane == 0) IT[row] = -it - 1; return; }
        float p[PER], sp[PER], qp = 0.f, mp = 0.f;
#pragma unroll
        for (int t = 0; t < PER; ++t) {
            p[t] = P[row * YP + lane + 64 * t];
            qp = fmaf(q[t], p[t], qp);
            mp = fmaf(mut[t], p[t], mp);
        }
        qp = wave_sum<DD>(qp);
        mp = wave_sum<DD>(mp);
        float psp = 0.f;
#pragma unroll
        for (int t = 0; t < PER; ++t) {
            sp[t] = SP[row * DD + lane + 64 * t] - qp * mut[t] - mp * q[t] + om * qp * q[t] + lambda * p[t];
            psp = fmaf(p[t], sp[t], psp);
        }
        psp = wave_sum<DD>(psp);
        const float alpha = rr / psp;
        float r[PER], rr2 = 0.f;
#pragma unroll
        for (int t = 0; t < PER; ++t) {
            X[row * DD + lane + 64 * t] += alpha * p[t];
            r[t] = R[row * DD + lane + 64 * t] - alpha * sp[t];
            R[row * DD + lane + 64 * t] = r[t];
            rr2 = fmaf(r[t], r[t], rr2);
        }
        rr2 = wave_sum<DD>(rr2);
        const float beta = rr2 / rr;
#pragma unroll
        for (int t = 0; t < PER; ++t) P[row * YP + lane + 64 * t] = r[t] + beta * p[t];
        if (lane == 0) { RR[row] = rr2; IT[row] = it + 1; }
    } else {
        float x[PER], mx = 0.f, qx = 0.f;
#pragma unroll
        for (int t = 0; t < PER; ++t) {
            x[t] = X[row * DD + lane + 64 * t];
            mx = fmaf(mut[t] - om * q[t], x[t], mx);
            qx = fmaf(q[t], x[t], qx);
        }
        mx = wave_sum<DD>(mx);
        qx = wave_sum<DD>(qx);
        const float dl = om - mx, inv = 1.f / dl;                // delta = omega - mu . rho
#pragma unroll
        for (int t = 0; t < PER; ++t) {
            Yg[row * YP + lane + 64 * t] = -x[t] * inv;           // y1 = -rho / delta
            if (rho != nullptr) rho[row * DD + lane + 64 * t] = x[t];
        }
        if (lane == 0) {
            Yg[row * YP + DD] = (1.f + qx) * inv;                // y0 = (1 + q . rho) / delta
            if (delta != nullptr) delta[row] = dl;
            if (iters != nullptr) { const int it = IT[row]; iters[row] = it < 0 ? -it - 1 : it; }
        }
    }
}

template <int DD>
hipError_t forward_cg_impl(const Problem &p, int T, float eps, int32_t *iters)
{
    using S = Shape<DD>;
    const CgLayout C = make_cg_layout<DD>(p.B, p.H, p.n);
    const Layout &L = C.base;
    char *ws = static_cast<char *>(p.ws);
    _Float16 *KT = reinterpret_cast<_Float16 *>(ws + L.kt);
    bf16_t *VT = reinterpret_cast<bf16_t *>(ws + L.vt);
    bf16_t *KTB = reinterpret_cast<bf16_t *>(ws + C.ktb);
    float *M = reinterpret_cast<float *>(ws + L.m), *Y = reinterpret_cast<float *>(ws + L.y);
    float *MUt = reinterpret_cast<float *>(ws + C.mut), *OM = reinterpret_cast<float *>(ws + C.om);
    float *X = reinterpret_cast<float *>(ws + C.x), *R = reinterpret_cast<float *>(ws + C.r);
    float *P = reinterpret_cast<float *>(ws + C.p), *SP = reinterpret_cast<float *>(ws + C.sp);
    float *RR = reinterpret_cast<float *>(ws + C.rr);
    int *IT = reinterpret_cast<int *>(ws + C.it);
    const int bh = p.B * p.H, nq64 = (p.n + 63) / 64;
    const float cscale = p.scale * LOG2E;
    const bf16_t *Q = static_cast<const bf16_t *>(p.Q), *K = static_cast<const bf16_t *>(p.K),
                 *V = static_cast<const bf16_t *>(p.V);
    const llla_strides dense = {(int64_t)p.H * p.n * DD, (int64_t)p.n * DD, DD};     // [B,H,n,DD] fp32 scratch arrays
    const dim3 rows_grid((p.n + 3) / 4, bh);

    stage_mark(p.stream, "prep");
    hipLaunchKernelGGL((prep_kernel<DD>), dim3(L.nkb, bh), dim3(256), 0, p.stream, K, V, p.sk, p.sv, p.H, p.n, L.nkb, KT, VT);
    hipLaunchKernelGGL((prep_kernel<DD>), dim3(L.nkb, bh), dim3(256), 0, p.stream, K, K, p.sk, p.sk, p.H, p.n, L.nkb, KT, KTB);
    stage_mark(p.stream, "rowmax");
    hipLaunchKernelGGL((sweep_kernel<true, DD>), dim3(bh, nq64), dim3(256), 0, p.stream, Q, K, p.sq, p.sk, p.H, p.n, L.nkb,
                       0, cscale, VT, M, Y, p.O, p.so, 0);
    stage_mark(p.stream, "first_moment");       // omega = sum w, mu~ = sum w k: plain weights times the K tile
    hipLaunchKernelGGL((sweep_kernel<false, DD>), dim3(bh, nq64), dim3(256), 0, p.stream, Q, K, p.sq, p.sk, p.H, p.n, L.nkb,
                       0, cscale, KTB, M, (const float *)nullptr, (void *)MUt, dense, 0, OM);
    hipLaunchKernelGGL((cg_rows_kernel<DD, 0>), rows_grid, dim3(256), 0, p.stream, Q, p.sq, p.H, p.n, p.lambda, eps, MUt, OM,
                       X, R, P, SP, RR, IT, Y, p.rho, p.delta, iters);
    stage_mark(p.stream, "cg_steps");
    for (int t = 0; t < T; ++t) {
        hipLaunchKernelGGL((sweep_kernel<false, DD>), dim3(bh, nq64), dim3(256), 0, p.stream, Q, K, p.sq, p.sk, p.H, p.n,
                           L.nkb, 0, cscale, KTB, M, (const float *)P, (void *)SP, dense, 0, (float *)nullptr);
        hipLaunchKernelGGL((cg_rows_kernel<DD, 1>), rows_grid, dim3(256), 0, p.stream, Q, p.sq, p.H, p.n, p.lambda, eps, MUt,
                           OM, X, R, P, SP, RR, IT, Y, p.rho, p.delta, iters);
    }
    stage_mark(p.stream, "cg_finish");
    hipLaunchKernelGGL((cg_rows_kernel<DD, 2>), rows_grid, dim3(256), 0, p.stream, Q, p.sq, p.H, p.n, p.lambda, eps, MUt, OM,
                       X, R, P, SP, RR, IT, Y, p.rho, p.delta, iters);
    const int first = S::EARLY_ROWS < p.n ? S::EARLY_ROWS : p.n;
    stage_mark(p.stream, "output_early_rows");
    hipError_t e = valu_forward_given(p, first, M, L.npad, Y, S::YP);
    if (e != hipSuccess) return e;
    if (first < p.n) {
        stage_mark(p.stream, "output");
        hipLaunchKernelGGL((sweep_kernel<false, DD>), dim3(bh, (p.n - first + 63) / 64), dim3(256), 0, p.stream, Q, K, p.sq, p.sk,
                           p.H, p.n, L.nkb, first, cscale, VT, M, (const float *)Y, p.O, p.so, p.out == LLLA_BF16 ? 1 : 0,
                           (float *)nullptr);
    }
    return hipGetLastError();
}

template <int DD>
hipError_t backward_rowmax_impl(const BackwardProblem &p, const BackwardLayout &BL)
{
    const Layout L = make_layout<DD>(p.B, p.H, p.n);
    char *ws = static_cast<char *>(p.ws) + BL.fwd;
    _Float16 *KT = reinterpret_cast<_Float16 *>(ws + L.kt);
    bf16_t *VT = reinterpret_cast<bf16_t *>(ws + L.vt);
    float *M = reinterpret_cast<float *>(ws + L.m);
    float *Y = reinterpret_cast<float *>(ws + L.y);
    const int bh = p.B * p.H;
    const bf16_t *Q = static_cast<const bf16_t *>(p.Q), *K = static_cast<const bf16_t *>(p.K),
                 *V = static_cast<const bf16_t *>(p.V);
    stage_mark(p.stream, "prep");
    hipLaunchKernelGGL((prep_kernel<DD>), dim3(L.nkb, bh), dim3(256), 0, p.stream, K, V, p.sk, p.sv, p.H, p.n, L.nkb, KT, VT);
    stage_mark(p.stream, "rowmax");
    hipLaunchKernelGGL((sweep_kernel<true, DD>), dim3(bh, (p.n + 63) / 64), dim3(256), 0, p.stream, Q, K, p.sq, p.sk, p.H,
                       p.n, L.nkb, 0, p.scale * LOG2E, VT, M, Y, (void *)nullptr, llla_strides{0, 0, 0}, 0, (float *)nullptr);
    return hipGetLastError();
}

template <int DD>
hipError_t backward_solve_impl(const BackwardProblem &p, const BackwardLayout &BL)
{
    using S = Shape<DD>;
    const Layout L = make_layout<DD>(p.B, p.H, p.n);
    char *base = static_cast<char *>(p.ws);
    char *ws = base + BL.fwd;
    _Float16 *KT = reinterpret_cast<_Float16 *>(ws + L.kt);
    float *M = reinterpret_cast<float *>(ws + L.m);
    float *Y = reinterpret_cast<float *>(ws + L.y);
    const float *R = reinterpret_cast<const float *>(base + BL.r);
    float *U = reinterpret_cast<float *>(base + BL.u);
    const int first = S::EARLY_ROWS < p.n ? S::EARLY_ROWS : p.n;
    stage_mark(p.stream, "moments_and_two_solves");
    // (on zero-padded copies of a d = 16 / 32 call: the variant that skips the padded tiles, as in the forward)
    const int live = (DD == 64 && p.live_d > 0) ? (p.live_d + 15) / 16 : S::NB;
    const dim3 grid((p.n + S::QB - 1) / S::QB, p.B * p.H);
    const bf16_t *Q = static_cast<const bf16_t *>(p.Q), *K = static_cast<const bf16_t *>(p.K);
    if constexpr (DD == 64) {
        if (live == 1)
            hipLaunchKernelGGL((moments_u_kernel<DD, 1>), grid, dim3(S::NT), 0, p.stream, Q, K, p.sq, p.sk, p.H, p.n, L.nkb, first,
                               p.scale * LOG2E, p.lambda, p.lambda_rows, KT, M, Y, R, U);
        else if (live == 2)
            hipLaunchKernelGGL((moments_u_kernel<DD, 2>), grid, dim3(S::NT), 0, p.stream, Q, K, p.sq, p.sk, p.H, p.n, L.nkb, first,
                               p.scale * LOG2E, p.lambda, p.lambda_rows, KT, M, Y, R, U);
    }
    if (live == S::NB)
        hipLaunchKernelGGL((moments_u_kernel<DD>), grid, dim3(S::NT), 0, p.stream, Q, K, p.sq, p.sk, p.H, p.n, L.nkb, first,
                           p.scale * LOG2E, p.lambda, p.lambda_rows, KT, M, Y, R, U);
    return hipGetLastError();
}

}  // namespace

BackwardLayout mfma_backward_layout(int B, int H, int n, int d)
{
    BackwardLayout BL{};
    const Layout L = d == 64 ? make_layout<64>(B, H, n) : make_layout<128>(B, H, n);
    const size_t rows = (size_t)B * H * n;
    BL.ypitch = d + 16;                                  // = Shape<d>::YP
    BL.npad = L.npad;
    BL.m = L.m;
    BL.y = L.y;
    size_t off = 0;
    BL.fwd = off; off += round_up(L.total, 256);
    BL.u = off;   off += round_up(rows * BL.ypitch * 4, 256);
    BL.r = off;   off += round_up(rows * BL.ypitch * 4, 256);
    BL.sc = off;  off += round_up(rows * 8 * 4, 256);
    BL.total = off;
    return BL;
}

hipError_t mfma_backward_rowmax(const BackwardProblem &p, const BackwardLayout &L)
{
    return p.d == 64 ? backward_rowmax_impl<64>(p, L) : backward_rowmax_impl<128>(p, L);
}

hipError_t mfma_backward_solve(const BackwardProblem &p, const BackwardLayout &L)
{
    return p.d == 64 ? backward_solve_impl<64>(p, L) : backward_solve_impl<128>(p, L);
}

// (the exact forward serves causal and non-causal calls; the approximate mode and the backward, which ask with
// causal = true, are causal by definition)
bool mfma_forward_supported(int d, llla_dtype in, bool causal) { (void)causal; return (d == 64 || d == 128) && in == LLLA_BF16; }

size_t mfma_forward_workspace_bytes(int B, int H, int n, int d, llla_dtype in)
{
    if (!mfma_forward_supported(d, in, true)) return 0;
    return d == 64 ? make_layout<64>(B, H, n).total : make_layout<128>(B, H, n).total;
}

hipError_t mfma_forward(const Problem &p) { return p.d == 64 ? forward_impl<64>(p) : forward_impl<128>(p); }

size_t mfma_forward_cg_workspace_bytes(int B, int H, int n, int d, llla_dtype in)
{
    if (!mfma_forward_supported(d, in, true)) return 0;
    return d == 64 ? make_cg_layout<64>(B, H, n).total : make_cg_layout<128>(B, H, n).total;
}

hipError_t mfma_forward_cg(const Problem &p, int T, float eps, int32_t *iters)
{
    return p.d == 64 ? forward_cg_impl<64>(p, T, eps, iters) : forward_cg_impl<128>(p, T, eps, iters);
}

}  // namespace llla

// Matrix-core decode path of Local Linear Attention for gfx950: bf16 caches, d = 64, cache capacity
// L_max >= 1024, optional per-sequence lengths.  One query per (batch, head) against a cache that already
// holds the new token: the last row of the causal forward (Section 2.3: LLA keeps a Theta(n d) KV
// cache; Section 3.2: rows are independent).
//
// The cache is streamed from HBM exactly once.  In a single pass each wave accumulates, for its
// share of the keys and relative to its own running maximum m (the online rescaling of Algorithm 1),
//     omega = sum w,  mu~ = sum w k,  Sigma~ = sum w k k^T   (Eq. (tilded_form))
//     y0v   = sum w v,  G~ = sum w k v^T                      (value moments)
// as f16 MFMA accumulators: (w (.) K)^T [K | V] with the key as the contraction index.  Eq. (lla) then
// needs no second pass over the cache:  o = sum_j w_j (y0 + k_j . y1) v_j = y0 * y0v + G~^T y1,
// where [y0; y1] solves [omega mu~^T; mu~ Sigma~ + lambda I] y = [1; q].  A small second kernel merges
// the partial moments of a head with a max-rescale, solves on chip, and writes o.
#include "llla_mfma_common.hpp"
#include "llla_mfma_solve64.hpp"

namespace llla {
namespace {

using namespace mfma;

using S64 = Shape<64>;
constexpr int D = S64::D, QW = S64::QW, NT = 256;
__host__ __device__ constexpr int tix(int I, int J) { return S64::tix(I, J); }

constexpr int STEP = 32;                       // keys per MFMA step
constexpr int NSTAGE = 2;                      // LDS stages per wave; NSTAGE-1 are in flight
constexpr int TILE_H = STEP * D;               // halves of one natural [32 keys][64] tile (4 KB)
constexpr int STAGE_H = 2 * TILE_H;            // K tile + V tile
constexpr int DMA_PER_STAGE = 8;
constexpr int NTILES = 26;                     // 10 (Sigma~ upper) + 16 (G~)
constexpr int PART_F = 192 + NTILES * 256;     // floats per partial: [m, omega, ..], mu~[64], y0v[64], tiles
constexpr int MIN_L = 256;                     // shorter caches go to the vector path
constexpr int PRECISE_L = 4 * D;               // sequences up to this length take the two-term weights

typedef short short4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) short4v *lds_short4_ptr;

struct Split {
    int nsplit;          // workgroups per head
    int keys_per_wave;   // multiple of STEP
    int nparts;          // partials per head = 4 * nsplit
    int group;           // partials merged by one wave of the combine stage (0: no combine stage)
    int ngroups;         // partials per head that reach the merge kernel
};

Split make_split(int bh, int L)
{
    Split s;
    // two workgroups per compute unit fit: with 512 (batch, head) pairs or more one workgroup per pair fills the GPU
    // in a single round (a second round of equally long workgroups cost 5 % at the changeover)
    int want = (512 + bh - 1) / bh;
    int most = L / (4 * 8 * STEP);                   // at least 8 steps per wave
    if (most < 1) most = 1;
    s.nsplit = want < 1 ? 1 : (want > most ? most : want);
    if (s.nsplit > 16) s.nsplit = 16;
    const int waves = 4 * s.nsplit;
    s.keys_per_wave = ((L + waves - 1) / waves + STEP - 1) / STEP * STEP;
    s.nparts = waves;
    // few heads with long caches are cut into many partials; the merge kernel sums a head's partials one after the
    // other, so beyond 16 of them a combine stage first merges groups of about sqrt(nparts) in parallel
    s.group = 0;
    s.ngroups = s.nparts;
    if (s.nparts > 16) {
        s.group = s.nparts >= 64 ? 8 : 6;
        s.ngroups = (s.nparts + s.group - 1) / s.group;
    }
    return s;
}

// two bf16 packed in a dword -> two f16 packed (exact for values in the f16 range)
__device__ inline unsigned bf16x2_to_f16x2(unsigned u)
{
    const float lo = __uint_as_float(u << 16), hi = __uint_as_float(u & 0xffff0000u);
    return __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(lo, hi));
}

template <int N>
__device__ inline void dma_wait_pending() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

// PRECISE (short sequences, chosen per sequence by the kernel): with fewer keys than features only the ridge holds
// some directions, and the 2^-11 rounding of w k is then not small against it.  Such sequences take the weights in
// fp32 and hand w and w k to the matrix cores as an f16 head plus an f16 tail.  Long ones round w to f16 once and
// use that same rounded weight in every moment.
template <bool PRECISE>
__device__ __forceinline__ void decode_partial_body(bf16_t (&stage)[4][NSTAGE][STAGE_H], const bf16_t *__restrict__ qg,
                                                    const bf16_t *__restrict__ Kg, const bf16_t *__restrict__ Vg,
                                                    llla_strides sk, llla_strides sv,
                                                    const int32_t *__restrict__ seqlens, int H, int L_max, int nparts,
                                                    float cscale, float *__restrict__ parts)
{
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64, g = lane / 16,
              nn = lane % 16;
    const int bh = blockIdx.y, b = bh / H, h = bh % H;
    const int part = blockIdx.x * 4 + wave;
    // the sequence's own length decides the share of each wave, so short sequences stay balanced too; rows at
    // and beyond L are never read (a cache tail may hold anything, and 0 * NaN would poison the moments)
    const int L = seqlens ? min(max(seqlens[b], 1), L_max) : L_max;
    const int keys_per_wave = ((L + nparts - 1) / nparts + STEP - 1) / STEP * STEP;
    const int r0 = part * keys_per_wave;
    const int r1 = min(r0 + keys_per_wave, L);
    const int nsteps = __builtin_amdgcn_readfirstlane(r1 > r0 ? (r1 - r0 + STEP - 1) / STEP : 0);
    const bf16_t *Kh = Kg + b * sk.batch + h * sk.head;
    const bf16_t *Vh = Vg + b * sv.batch + h * sv.head;
    bf16_t *mystage = &stage[wave][0][0];

    // query fragment, the same for every column of the B operand: lane (g, *) holds q[8g..8g+7], q[32+8g..]
    bf16x8 qf[2];
    qf[0] = *reinterpret_cast<const bf16x8 *>(qg + (size_t)bh * D + 8 * g);
    qf[1] = *reinterpret_cast<const bf16x8 *>(qg + (size_t)bh * D + 32 + 8 * g);

    // ---- per-lane constants.  A natural tile is [key][8 chunks of 8 features]; chunk c of key k is
    //      stored at chunk position c ^ ((k>>1)&7) (the DMA writes whole rows, so no padding).
    int dma_key[4], dma_col[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int sl = 64 * t + lane;
        dma_key[t] = sl >> 3;
        dma_col[t] = ((sl & 7) ^ ((dma_key[t] >> 1) & 7)) * 8;
    }
    // logits operand (natural rows): key 16s + nn, feature chunks g and 4+g
    const int sw_n = (nn >> 1) & 7;
    const int nat0 = nn * D + ((g ^ sw_n) * 8), nat1 = nn * D + (((4 + g) ^ sw_n) * 8);     // + s*16*D
    // transposed operand through ds_read_b64_tr_b16: inside a 16-lane group, lane j addresses 4 features
    // (16 I + 4 (j%4) ..) of key 4g + j/4; the instruction hands lane i the 4 keys 4g..4g+3 of feature 16 I + i.
    int tr_addr[4];
    {
        const int key = 4 * g + (nn >> 2);
        const int swz = (key >> 1) & 7;
#pragma unroll
        for (int I = 0; I < 4; ++I) {
            const int c = 2 * I + ((nn & 3) >> 1);
            tr_addr[I] = key * D + ((c ^ swz) * 8) + (nn & 1) * 4;                           // + half*16*D
        }
    }

    f32x4 sig[10], gt[16], muacc[4], yvacc[4];
#pragma unroll
    for (int t = 0; t < 10; ++t) sig[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < 16; ++t) gt[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < 4; ++t) { muacc[t] = f32x4{0.f, 0.f, 0.f, 0.f}; yvacc[t] = f32x4{0.f, 0.f, 0.f, 0.f}; }
    float om = 0.f, m = -INFINITY;

    // Waves that start together on equally spaced addresses would keep hitting the same memory channels in
    // step; each wave therefore sweeps its share of the keys from a different starting step and wraps around
    // (the moments do not depend on the order of the keys).
    const int rot = nsteps > 0 ? (int)((part * 7u + bh * 13u) % (unsigned)nsteps) : 0;
    auto step_pos = [&](int step) { const int t = step + rot; return t >= nsteps ? t - nsteps : t; };
    // addresses: a scalar base per step (row j0 of the head) plus per-lane byte offsets that never change, so a
    // transfer costs no vector-ALU work; the transfers carry the non-temporal hint (the cache is read once); only a step that reaches past the sequence clamps its rows per lane
    // (to the last valid row: their weights are 0)
    unsigned koff[4], voff[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        koff[t] = 2u * (unsigned)(dma_key[t] * (int)sk.seq + dma_col[t]);
        voff[t] = 2u * (unsigned)(dma_key[t] * (int)sv.seq + dma_col[t]);
    }
    auto issue_dma = [&](int step) {
        // (LDS destinations as byte offsets: a generic pointer costs four scalar instructions per transfer to turn back)
        const unsigned dst = lds_offset(mystage) + 2u * (unsigned)((step % NSTAGE) * STAGE_H);
        const int j0 = r0 + step_pos(step < nsteps ? step : 0) * STEP;
        if (j0 + STEP <= L) {
            const bf16_t *kb = Kh + (int64_t)j0 * sk.seq, *vb = Vh + (int64_t)j0 * sv.seq;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                dma16_base_nt_off(kb, koff[t], dst + 2u * (512 * t));
                dma16_base_nt_off(vb, voff[t], dst + 2u * (TILE_H + 512 * t));
            }
        } else {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int j = min(j0 + dma_key[t], L - 1);
                dma16_nt_off(Kh + (int64_t)j * sk.seq + dma_col[t], dst + 2u * (512 * t));
                dma16_nt_off(Vh + (int64_t)j * sv.seq + dma_col[t], dst + 2u * (TILE_H + 512 * t));
            }
        }
    };

    // NSTAGE-1 stages in flight; every step issues exactly one more stage (clamped past the end) so
    // that "vmcnt <= 8 (NSTAGE-1)" always means "the oldest stage has landed"
#pragma unroll
    for (int st = 0; st < NSTAGE - 1; ++st) issue_dma(st);
    for (int s = 0; s < nsteps; ++s) {
        issue_dma(s + NSTAGE - 1);
        dma_wait_pending<DMA_PER_STAGE *(NSTAGE - 1)>();
        const bf16_t *kt = mystage + (s % NSTAGE) * STAGE_H;
        const bf16_t *vt = kt + TILE_H;
        const int j0 = r0 + step_pos(s) * STEP;

        // logits of the 32 keys: lane (g, *) gets keys 4g..4g+3 (sub-tile 0) and 16+4g.. (sub-tile 1)
        float tl[8];
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const bf16x8 k0 = *reinterpret_cast<const bf16x8 *>(kt + sub * 16 * D + nat0);
            const bf16x8 k1 = *reinterpret_cast<const bf16x8 *>(kt + sub * 16 * D + nat1);
            f32x4 z = {0.f, 0.f, 0.f, 0.f};
            z = mfma_bf16(k0, qf[0], z);
            z = mfma_bf16(k1, qf[1], z);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int j = j0 + 16 * sub + 4 * g + r;
                tl[4 * sub + r] = (j < r1) ? z[r] * cscale : -INFINITY;
            }
        }
        // running maximum over the wave's keys; the accumulators are rescaled only when it moves
        // (all 16 lanes of a row hold the same 8 logits; the maximum over the four rows goes through two row
        // broadcasts of the data-parallel primitives, without LDS round trips, and is read from the last row)
        float mx = fmaxf(fmaxf(fmaxf(tl[0], tl[1]), fmaxf(tl[2], tl[3])), fmaxf(fmaxf(tl[4], tl[5]), fmaxf(tl[6], tl[7])));
        mx = fmaxf(mx, rows_1_3_from_rows_0_2(mx));
        mx = fmaxf(mx, rows_2_3_from_row_1(mx));
        mx = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mx), 63));
        if (mx > m) {      // both are wave-uniform
            const float alpha = (m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m - mx);
            m = mx;
            om *= alpha;
#pragma unroll
            for (int t = 0; t < 10; ++t) sig[t] *= alpha;
#pragma unroll
            for (int t = 0; t < 16; ++t) gt[t] *= alpha;
#pragma unroll
            for (int t = 0; t < 4; ++t) { muacc[t] *= alpha; yvacc[t] *= alpha; }
        }
        float wf[8];
        half8 wq, wl;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            wf[t] = __builtin_amdgcn_exp2f(tl[t] - m);                // exp2(-inf) = 0 masks the tail
            wq[t] = (_Float16)wf[t];
            if (PRECISE) {
                wl[t] = (_Float16)(wf[t] - (float)wq[t]);
                om += wf[t];
            } else {
                om += (float)wq[t];                                   // omega sums the weights as the MFMAs see them
            }
        }

        // transposed K and V fragments (bf16 -> f16, exact): slot t < 4 = key 4g+t, t >= 4 = key 16+4g+t-4
        half8 kf[4], vf[4];
#pragma unroll
        for (int I = 0; I < 4; ++I) {
            const short4v ka = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(kt + tr_addr[I]));
            const short4v kb = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(kt + 16 * D + tr_addr[I]));
            const short4v va = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(vt + tr_addr[I]));
            const short4v vb = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(vt + 16 * D + tr_addr[I]));
            const uint2 kau = __builtin_bit_cast(uint2, ka), kbu = __builtin_bit_cast(uint2, kb);
            const uint2 vau = __builtin_bit_cast(uint2, va), vbu = __builtin_bit_cast(uint2, vb);
            const uint4 kp = make_uint4(bf16x2_to_f16x2(kau.x), bf16x2_to_f16x2(kau.y), bf16x2_to_f16x2(kbu.x),
                                        bf16x2_to_f16x2(kbu.y));
            const uint4 vp = make_uint4(bf16x2_to_f16x2(vau.x), bf16x2_to_f16x2(vau.y), bf16x2_to_f16x2(vbu.x),
                                        bf16x2_to_f16x2(vbu.y));
            kf[I] = __builtin_bit_cast(half8, kp);
            vf[I] = __builtin_bit_cast(half8, vp);
        }
        auto row_mfmas = [&](int I, const half8 &af) {
#pragma unroll
            for (int J = 0; J < 4; ++J)
                if (J >= I) sig[tix(I, J)] = mfma_f16(af, kf[J], sig[tix(I, J)]);
#pragma unroll
            for (int J = 0; J < 4; ++J) gt[4 * I + J] = mfma_f16(af, vf[J], gt[4 * I + J]);
        };
        auto bcast_mfmas = [&](const half8 &wv) {
#pragma unroll
            for (int J = 0; J < 4; ++J) {
                muacc[J] = mfma_f16(wv, kf[J], muacc[J]);       // every row of the tile = mu~[16J + nn]
                yvacc[J] = mfma_f16(wv, vf[J], yvacc[J]);       // every row = (sum w v)[16J + nn]
            }
        };
        if (!PRECISE) {
#pragma unroll
            for (int I = 0; I < 4; ++I) row_mfmas(I, kf[I] * wq);
            bcast_mfmas(wq);
        } else {
            // w k in fp32 (exact up to the rounding of w), handed to the matrix cores as an f16 head plus an f16 tail
#pragma unroll
            for (int I = 0; I < 4; ++I) {
                half8 ah, al;
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const float pr = (float)kf[I][t] * wf[t];
                    ah[t] = (_Float16)pr;
                    al[t] = (_Float16)(pr - (float)ah[t]);
                }
                row_mfmas(I, ah);
                row_mfmas(I, al);
            }
            bcast_mfmas(wq);
            bcast_mfmas(wl);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");        // drain the clamped tail DMAs before the wave ends

    om += __shfl_xor(om, 16);
    om += __shfl_xor(om, 32);
    float *P = parts + ((size_t)bh * nparts + part) * PART_F;
    if (lane == 0) { P[0] = m; P[1] = om; }
    if (g == 0) {
#pragma unroll
        for (int J = 0; J < 4; ++J) { P[64 + 16 * J + nn] = muacc[J][0]; P[128 + 16 * J + nn] = yvacc[J][0]; }
    }
#pragma unroll
    for (int t = 0; t < 10; ++t) *reinterpret_cast<f32x4 *>(P + 192 + t * 256 + lane * 4) = sig[t];
#pragma unroll
    for (int t = 0; t < 16; ++t) *reinterpret_cast<f32x4 *>(P + 192 + (10 + t) * 256 + lane * 4) = gt[t];
}

__global__ __launch_bounds__(NT, 2) void decode_partial_kernel(const bf16_t *__restrict__ qg,
                                                               const bf16_t *__restrict__ Kg,
                                                               const bf16_t *__restrict__ Vg, llla_strides sk,
                                                               llla_strides sv, const int32_t *__restrict__ seqlens,
                                                               int H, int L_max, int nparts, float cscale,
                                                               float *__restrict__ parts)
{
    __shared__ __align__(16) bf16_t stage[4][NSTAGE][STAGE_H];     // 4 waves x NSTAGE stages x 8 KB
    const int b = (int)blockIdx.y / H;
    const int L = seqlens ? min(max(seqlens[b], 1), L_max) : L_max;
    if (__builtin_amdgcn_readfirstlane(L <= PRECISE_L ? 1 : 0))
        decode_partial_body<true>(stage, qg, Kg, Vg, sk, sv, seqlens, H, L_max, nparts, cscale, parts);
    else
        decode_partial_body<false>(stage, qg, Kg, Vg, sk, sv, seqlens, H, L_max, nparts, cscale, parts);
}

// Combine stage for heads with many partials: one wave merges partials [g * group, (g + 1) * group) of a head into a
// single record of the same format (the merge step of Algorithm 1's running maximum), so that the merge kernel's
// sequential sum over a head's partials stays short.  grid.x = groups, grid.y = heads, 4 waves = 4 groups per block.
// (at most two waves per SIMD: the scheduler otherwise keeps the register count low for occupancy and waits for every
// load before it issues the next)
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(1, 2))) void decode_combine_kernel(const float *__restrict__ parts, float *__restrict__ parts2,
                                                            int nparts, int group, int ngroups)
{
    // the wave index as a scalar: the loop bounds below are then uniform and the loads of an iteration are issued together
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64), lane = threadIdx.x % 64;
    const int gi = (int)blockIdx.x * 4 + wave, bh = blockIdx.y;
    if (gi >= ngroups) return;
    const int p0 = gi * group, p1 = min(p0 + group, nparts);
    const float *P0 = parts + (size_t)bh * nparts * PART_F;
    const float mstar = wave_max_strided(P0, p0, p1, PART_F, lane);
    float om = 0.f, mu = 0.f, yv = 0.f;
    f32x4 acc[NTILES];
#pragma unroll
    for (int t = 0; t < NTILES; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int p = p0; p < p1; ++p) {
        const float *P = P0 + (size_t)p * PART_F;
        const float mp = P[0];
        const float f = (mp == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mp - mstar);
        om = fmaf(f, P[1], om);
        mu = fmaf(f, P[64 + lane], mu);
        yv = fmaf(f, P[128 + lane], yv);
#pragma unroll
        for (int t = 0; t < NTILES; ++t) acc[t] += f * *reinterpret_cast<const f32x4 *>(P + 192 + t * 256 + lane * 4);
    }
    float *R = parts2 + ((size_t)bh * ngroups + gi) * PART_F;
    if (lane == 0) { R[0] = mstar; R[1] = om; }
    R[64 + lane] = mu;
    R[128 + lane] = yv;
#pragma unroll
    for (int t = 0; t < NTILES; ++t) *reinterpret_cast<f32x4 *>(R + 192 + t * 256 + lane * 4) = acc[t];
}

// Merge, solve, output for 4 heads per workgroup (4 waves):
//   phase 1  wave w sums the partial moments of head 4*block + w with the max-rescale factors
//            2^(m_p - m*) into LDS (the merge step of Algorithm 1's running maximum);
//   phase 2  wave 0 solves the four systems together (solve_wave_q4: four queries per wave, lane group = head);
//   phase 3  wave w forms o = y0 * (sum w v) + G~^T y1 for its head.
__global__ __launch_bounds__(NT, 1) void decode_merge_kernel(const bf16_t *__restrict__ qg, const float *__restrict__ parts,
                                                             int BH, int nparts, float lambda, void *__restrict__ og,
                                                             int out_bf16)
{
    __shared__ __align__(16) float merged[QW][NTILES][256];
    __shared__ __align__(16) float scw[QW * 16 * SC_PITCH];
    __shared__ float mus[QW][D], yvs[QW][D], oms[QW], ys[QW][D + 4];
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64, g = lane / 16,
              nn = lane % 16;

    {   // phase 1
        const int hq = min((int)blockIdx.x * QW + wave, BH - 1);
        const float *P0 = parts + (size_t)hq * nparts * PART_F;
        const float mstar = wave_max_strided(P0, 0, nparts, PART_F, lane);
        float om = 0.f, mu = 0.f, yv = 0.f;
        f32x4 acc[NTILES];
#pragma unroll
        for (int t = 0; t < NTILES; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int p = 0; p < nparts; ++p) {
            const float *P = P0 + (size_t)p * PART_F;
            const float mp = P[0];
            const float f = (mp == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mp - mstar);
            om = fmaf(f, P[1], om);
            mu = fmaf(f, P[64 + lane], mu);
            yv = fmaf(f, P[128 + lane], yv);
#pragma unroll
            for (int t = 0; t < NTILES; ++t) acc[t] += f * *reinterpret_cast<const f32x4 *>(P + 192 + t * 256 + lane * 4);
        }
#pragma unroll
        for (int t = 0; t < NTILES; ++t) *reinterpret_cast<f32x4 *>(&merged[wave][t][lane * 4]) = acc[t];
        mus[wave][lane] = mu;
        yvs[wave][lane] = yv;
        if (lane == 0) oms[wave] = om;
    }
    __syncthreads();

    if (wave == 0) {   // phase 2 (scalar branch: the block contains MFMAs); lane (g, nn) = (head, element) in the solve
        f32x4 acc[QW][10];
#pragma unroll
        for (int q = 0; q < QW; ++q) {
#pragma unroll
            for (int t = 0; t < 10; ++t) acc[q][t] = -*reinterpret_cast<const f32x4 *>(&merged[q][t][lane * 4]);
#pragma unroll
            for (int P = 0; P < 4; ++P)     // the solve takes -(Sigma~ + lambda I)
#pragma unroll
                for (int t = 0; t < 4; ++t) acc[q][Shape<64>::tix(P, P)][t] -= (nn == 4 * g + t) ? lambda : 0.f;
        }
        const int hs = min((int)blockIdx.x * QW + g, BH - 1);
        float tmu[4], tq[4], te[4], y1[4], u1[4], y0 = 0.f, u0 = 0.f;
#pragma unroll
        for (int P = 0; P < 4; ++P) {
            tmu[P] = -mus[g][16 * P + nn];
            tq[P] = -bf16_to_f32(qg[(size_t)hs * D + 16 * P + nn]);
            te[P] = 0.f; y1[P] = 0.f; u1[P] = 0.f;
        }
        solve_wave_q4<false>(acc, tmu, tq, te, 0.f, oms[g], scw, g, nn, 0.5f * lambda, y1, y0, u1, u0);
#pragma unroll
        for (int P = 0; P < 4; ++P) ys[g][16 * P + nn] = y1[P];
        if (nn == 0) ys[g][D] = y0;
    }
    __syncthreads();

    {   // phase 3
        const int hq = (int)blockIdx.x * QW + wave;
        const float y0 = ys[wave][D];
#pragma unroll
        for (int J = 0; J < 4; ++J) {
            float s = 0.f;
#pragma unroll
            for (int I = 0; I < 4; ++I) {
                const f32x4 gv = *reinterpret_cast<const f32x4 *>(&merged[wave][10 + 4 * I + J][lane * 4]);
                const f32x4 y1 = *reinterpret_cast<const f32x4 *>(&ys[wave][16 * I + 4 * g]);
#pragma unroll
                for (int t = 0; t < 4; ++t) s = fmaf(gv[t], y1[t], s);      // G~[16I+4g+t][16J+nn] y1[16I+4g+t]
            }
            s += __shfl_xor(s, 16);
            s += __shfl_xor(s, 32);
            const float o = fmaf(y0, yvs[wave][16 * J + nn], s);
            if (g == 0 && hq < BH) {
                if (out_bf16) ((bf16_t *)og)[(size_t)hq * D + 16 * J + nn] = f32_to_bf16(o);
                else ((float *)og)[(size_t)hq * D + 16 * J + nn] = o;
            }
        }
    }
}

// The same for ONE head per workgroup, for calls with few heads (small-batch serving), where the kernel above would
// leave most compute units idle and its phase 1 -- one wave adding a head's partial records one after the other, 26 KB
// per round trip to memory -- is the longest part of the whole decode step.  Here the four waves share the head's 26
// tiles (wave w: tiles w, w + 4, ...) and fetch them for up to eight partials at a time, so a head's records are in
// after one or two round trips; wave 0 solves (the three other systems that solve_wave_q4 carries are lambda I with a
// zero right-hand side); wave J forms column block J of the output.
__global__ __launch_bounds__(NT, 1) void decode_merge1_kernel(const bf16_t *__restrict__ qg, const float *__restrict__ parts,
                                                              int nparts, float lambda, void *__restrict__ og, int out_bf16)
{
    __shared__ __align__(16) float merged[NTILES][256];
    __shared__ __align__(16) float scw[QW * 16 * SC_PITCH];
    __shared__ __align__(16) float mus[D], yvs[D], ys[D + 4];
    __shared__ float oms;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64, g = lane / 16,
              nn = lane % 16;
    const int hq = blockIdx.x;
    constexpr int PG = 8, TW = (NTILES + 3) / 4;

    {   // phase 1
        const float *P0 = parts + (size_t)hq * nparts * PART_F;
        const float mstar = wave_max_strided(P0, 0, nparts, PART_F, lane);
        float s1 = 0.f;              // wave 0: mu~[lane], wave 1: (sum w v)[lane], wave 2: omega
        f32x4 acc[TW];
#pragma unroll
        for (int i = 0; i < TW; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int pb = 0; pb < nparts; pb += PG) {
            const float *P[PG];
            float f[PG], v1[PG];
            f32x4 v[PG][TW];
#pragma unroll
            for (int k = 0; k < PG; ++k) {
                P[k] = P0 + (size_t)min(pb + k, nparts - 1) * PART_F;      // past the end: the last record again, factor 0
                f[k] = P[k][0];
                v1[k] = wave == 0 ? P[k][64 + lane] : (wave == 1 ? P[k][128 + lane] : (wave == 2 ? P[k][1] : 0.f));
#pragma unroll
                for (int i = 0; i < TW; ++i) {
                    const int t = min(wave + 4 * i, NTILES - 1);            // (a repeated tile is not stored below)
                    v[k][i] = *reinterpret_cast<const f32x4 *>(P[k] + 192 + t * 256 + lane * 4);
                }
            }
#pragma unroll
            for (int k = 0; k < PG; ++k) {
                const float fk = (pb + k >= nparts || f[k] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(f[k] - mstar);
                s1 = fmaf(fk, v1[k], s1);
#pragma unroll
                for (int i = 0; i < TW; ++i) acc[i] += fk * v[k][i];
            }
        }
#pragma unroll
        for (int i = 0; i < TW; ++i)
            if (wave + 4 * i < NTILES) *reinterpret_cast<f32x4 *>(&merged[wave + 4 * i][lane * 4]) = acc[i];
        if (wave == 0) mus[lane] = s1;
        if (wave == 1) yvs[lane] = s1;
        if (wave == 2 && lane == 0) oms = s1;
    }
    __syncthreads();

    if (wave == 0) {   // phase 2 (scalar branch: the block contains MFMAs); lane group 0 = the head, groups 1..3 idle systems
        f32x4 acc[QW][10];
#pragma unroll
        for (int q = 0; q < QW; ++q) {
#pragma unroll
            for (int t = 0; t < 10; ++t)
                acc[q][t] = q == 0 ? -*reinterpret_cast<const f32x4 *>(&merged[t][lane * 4]) : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int P = 0; P < 4; ++P)     // the solve takes -(Sigma~ + lambda I)
#pragma unroll
                for (int t = 0; t < 4; ++t) acc[q][Shape<64>::tix(P, P)][t] -= (nn == 4 * g + t) ? lambda : 0.f;
        }
        float tmu[4], tq[4], te[4], y1[4], u1[4], y0 = 0.f, u0 = 0.f;
#pragma unroll
        for (int P = 0; P < 4; ++P) {
            tmu[P] = g == 0 ? -mus[16 * P + nn] : 0.f;
            tq[P] = g == 0 ? -bf16_to_f32(qg[(size_t)hq * D + 16 * P + nn]) : 0.f;
            te[P] = 0.f; y1[P] = 0.f; u1[P] = 0.f;
        }
        solve_wave_q4<false>(acc, tmu, tq, te, 0.f, g == 0 ? oms : 1.f, scw, g, nn, 0.5f * lambda, y1, y0, u1, u0);
        if (g == 0) {
#pragma unroll
            for (int P = 0; P < 4; ++P) ys[16 * P + nn] = y1[P];
            if (nn == 0) ys[D] = y0;
        }
    }
    __syncthreads();

    {   // phase 3: wave J, column block J
        const int J = wave;
        const float y0 = ys[D];
        float s = 0.f;
#pragma unroll
        for (int I = 0; I < 4; ++I) {
            const f32x4 gv = *reinterpret_cast<const f32x4 *>(&merged[10 + 4 * I + J][lane * 4]);
            const f32x4 y1 = *reinterpret_cast<const f32x4 *>(&ys[16 * I + 4 * g]);
#pragma unroll
            for (int t = 0; t < 4; ++t) s = fmaf(gv[t], y1[t], s);          // G~[16I+4g+t][16J+nn] y1[16I+4g+t]
        }
        s += __shfl_xor(s, 16);
        s += __shfl_xor(s, 32);
        const float o = fmaf(y0, yvs[16 * J + nn], s);
        if (g == 0) {
            if (out_bf16) ((bf16_t *)og)[(size_t)hq * D + 16 * J + nn] = f32_to_bf16(o);
            else ((float *)og)[(size_t)hq * D + 16 * J + nn] = o;
        }
    }
}

}  // namespace

bool mfma_decode_supported(int d, llla_dtype in) { return (d == D || d == 128) && in == LLLA_BF16; }

size_t mfma_decode_workspace_bytes(int B, int H, int L_max, int d, llla_dtype in)
{
    if (!mfma_decode_supported(d, in) || L_max < MIN_L) return 0;
    if (d == 128) return mfma_decode128_workspace_bytes(B, H, L_max);
    const Split s = make_split(B * H, L_max);
    const size_t records = (size_t)s.nparts + (s.group ? s.ngroups : 0);
    return round_up((size_t)B * H * records * PART_F * sizeof(float), 256);
}

bool mfma_decode_takes(const Problem &p)
{
    // per-lane byte offsets inside one 32-key step are kept in 32 bits
    const int64_t reach = 2 * 32 * (p.sk.seq > p.sv.seq ? p.sk.seq : p.sv.seq);
    // (batch, head) is the y dimension of the grid
    return p.n >= MIN_L && reach < (int64_t(1) << 31) && (int64_t)p.B * p.H <= 65535;
}

hipError_t mfma_decode(const Problem &p)
{
    if (p.d == 128) return mfma_decode128(p);
    const int bh = p.B * p.H;
    const Split s = make_split(bh, p.n);
    float *parts = static_cast<float *>(p.ws);
    const float cscale = p.scale * LOG2E;
    stage_mark(p.stream, "decode_partial");
    hipLaunchKernelGGL(decode_partial_kernel, dim3(s.nsplit, bh), dim3(NT), 0, p.stream, (const bf16_t *)p.Q,
                       (const bf16_t *)p.K, (const bf16_t *)p.V, p.sk, p.sv, p.seqlens, p.H, p.n, s.nparts, cscale, parts);
    const float *merge_in = parts;
    if (s.group) {
        float *parts2 = parts + (size_t)bh * s.nparts * PART_F;
        stage_mark(p.stream, "decode_combine");
        hipLaunchKernelGGL(decode_combine_kernel, dim3((s.ngroups + 3) / 4, bh), dim3(NT), 0, p.stream, (const float *)parts,
                           parts2, s.nparts, s.group, s.ngroups);
        merge_in = parts2;
    }
    stage_mark(p.stream, "decode_merge");
    // up to one workgroup per compute unit: a head per workgroup, its waves sharing the merge; beyond that four heads
    // per workgroup, solved together
    if (bh <= 256)
        hipLaunchKernelGGL(decode_merge1_kernel, dim3(bh), dim3(NT), 0, p.stream, (const bf16_t *)p.Q, merge_in, s.ngroups,
                           p.lambda, p.O, p.out == LLLA_BF16 ? 1 : 0);
    else
        hipLaunchKernelGGL(decode_merge_kernel, dim3((bh + QW - 1) / QW), dim3(NT), 0, p.stream, (const bf16_t *)p.Q,
                           merge_in, bh, s.ngroups, p.lambda, p.O, p.out == LLLA_BF16 ? 1 : 0);
    return hipGetLastError();
}

}  // namespace llla

// Matrix-core decode path of Local Linear Attention for gfx950 at head dimension 128: bf16 caches, cache
// capacity L_max >= 1024, optional per-sequence lengths.  The method is the one of the d = 64 kernel (a single
// pass over the cache that accumulates omega, mu~, Sigma~ of Eq. (tilded_form) and the value moments sum w v,
// G~ = sum w k v^T relative to a running maximum as in Algorithm 1, then one solve per head and
// o = y0 * sum w v + G~^T y1, which is Eq. (lla) with the sum over keys taken first).
//
// What differs is who holds the moments.  At d = 128 they are 36 + 64 upper-triangular / full 16x16 tiles plus
// 16 broadcast tiles for mu~ and sum w v: 464 accumulator registers, more than one wave owns.  The four waves of
// a workgroup therefore walk ONE key stream together and split the tiles: wave (a, b) owns the rows 64a..64a+63
// of Sigma~ and G~ restricted to the columns 64b..64b+63 (the lower-left quarter of Sigma~ is not needed), and
// the two broadcast moments are dealt out so that the waves carry 34 / 36 / 16 / 30 tiles.  The wave with
// the 16 tiles also forms the 32 logits of the NEXT step (8 MFMAs), the running maximum and the weights, and hands them
// to the other three through a 264-byte record in LDS that the step's barrier publishes: every wave forming them
// for itself (bit-identical, no exchange) cost each of them as many vector instructions again as its moments do.
// A step's K and V tiles (16 KB) come into LDS in 16 transfers, five by each of the three other waves and one by the
// weight wave; a wave converts what it brought from bf16 to f16 in place; four stages rotate with one workgroup
// barrier per step.
#include "llla_mfma_common.hpp"
#include "llla_mfma_solve128.hpp"
#include <type_traits>

namespace llla {
namespace {

using namespace mfma;

using S128 = Shape<128>;
constexpr int D = 128, NB = 8, NT = 256;
constexpr int STEP = 32;                       // keys per MFMA step
constexpr int NSTAGE = 4;                      // LDS stages per workgroup: two being read, two being filled
constexpr int TILE_H = STEP * D;               // halves of one natural [32 keys][128] tile (8 KB)
constexpr int STAGE_H = 2 * TILE_H;            // K tile + V tile
constexpr int NSIG = 36, NTILES = 100;         // Sigma~ upper triangle, then G~ row-major [I][J]
constexpr int HDR = 3 * D;                     // [m, omega, ..pad], mu~ at [D, 2D), sum w v at [2D, 3D)
constexpr int PART_F = HDR + NTILES * 256;     // floats per partial record
constexpr int MIN_L = 256;                     // shorter caches go to the vector path
constexpr int MAX_SPLIT = 32;
constexpr int PRECISE_L = 4 * D;               // sequences up to this length take the two-term weights
// Exchange record of one step's weights (floats): [0, 32) the fp32 weights, [32, 48) the same rounded to f16, [48, 64)
// their f16 tails, [64] the factor by which the moments so far are rescaled before the step is added, [65] the running
// maximum the weights refer to.  Lane group g owns weights 8 g .. 8 g + 7 (keys 4 g .. 4 g + 3 and 16 + 4 g .. 16 + 4 g + 3).
constexpr int XREC_F = 128;

typedef short short4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) short4v *lds_short4_ptr;
typedef __attribute__((address_space(3))) const half8 *lds_half8_ptr;
typedef unsigned uint4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) uint4v *lds_uint4_ptr;

struct Split {
    int nsplit;          // workgroups (= partial records) per head
};

Split make_split(int bh, int L)
{
    Split s;
    int want = (512 + bh - 1) / bh;                  // two workgroups per compute unit are resident
    int most = L / (8 * STEP);                       // at least 8 steps per workgroup
    if (most < 1) most = 1;
    s.nsplit = want < 1 ? 1 : (want > most ? most : want);
    if (s.nsplit > MAX_SPLIT) s.nsplit = MAX_SPLIT;
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

// A natural tile is [key][16 chunks of 8 features], 256 B per key, which is exactly one pass over the LDS banks;
// chunk c of key k is stored at chunk position c ^ swz(k).  Bits 1..3 of the position take k mod 8, so that the
// 8 keys that half a wave reads transposed (two neighbouring chunks each) cover all banks once; bit 0 takes bit 3
// of k, so that the 16 keys a quarter wave reads as natural rows (one chunk each) do too.
__device__ inline int swz(int key) { return ((key & 7) << 1) ^ ((key >> 3) & 1); }

// Transposed fragment of 16 features x 32 keys as an MFMA operand (the tile already holds f16): slot t < 4 = key 4g + t,
// slot t >= 4 = key 16 + 4g + t - 4, feature 16 I + nn.  The argument is the lane's LDS byte address for feature
// block I of the tile; the second half of the keys lies a constant 16 rows further on.
__device__ inline half8 tr_frag(unsigned lds_byte_addr)
{
    const short4v a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(uintptr_t)lds_byte_addr);
    const short4v b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(uintptr_t)(lds_byte_addr + 16 * D * 2));
    const uint2 au = __builtin_bit_cast(uint2, a), bu = __builtin_bit_cast(uint2, b);
    return __builtin_bit_cast(half8, make_uint4(au.x, au.y, bu.x, bu.y));
}

__host__ __device__ constexpr int tix4(int i, int j) { return i * 4 - i * (i - 1) / 2 + (j - i); }   // 4x4 upper triangle

struct PartialArgs {
    const bf16_t *qg, *Kg, *Vg;
    llla_strides sk, sv;
    const int32_t *seqlens;
    int H, L_max, nparts;
    float cscale;
    float *parts;
};

// The share of wave (WA, WB): rows 4 WA .. 4 WA + 3 (feature blocks), columns 4 WB .. 4 WB + 3.
template <int WA, int WB, bool PRECISE>
__device__ __forceinline__ void partial_body(const PartialArgs &a, bf16_t *stage, float *xrec, int wave, int lane)
{
    constexpr bool SIG_DIAG = (WA == WB);                 // 10 tiles of a diagonal quarter of Sigma~
    constexpr bool SIG_FULL = (WA == 0 && WB == 1);       // the 16 tiles of the upper-right quarter
    constexpr int NS = SIG_DIAG ? 10 : (SIG_FULL ? 16 : 1);
    // the broadcast moments stay away from the wave (1, 0), which also forms the weights of the next step (of the
    // assignments that allows, this one measured fastest)
    constexpr bool HAS_MU = (WA == WB);                   // mu~ blocks 4 WA .. 4 WA + 3
    constexpr bool HAS_YV = (WA == 0);                    // (sum w v) blocks 4 WB .. 4 WB + 3

    const int g = lane / 16, nn = lane % 16;
    const int bh = blockIdx.y, b = bh / a.H, h = bh % a.H;
    const int part = blockIdx.x;
    // the sequence's own length decides the share of each workgroup; rows at and beyond L are never read
    const int L = a.seqlens ? min(max(a.seqlens[b], 1), a.L_max) : a.L_max;
    const int keys_per_part = ((L + a.nparts - 1) / a.nparts + STEP - 1) / STEP * STEP;
    const int r0 = part * keys_per_part;
    const int r1 = min(r0 + keys_per_part, L);
    const int nsteps = __builtin_amdgcn_readfirstlane(r1 > r0 ? (r1 - r0 + STEP - 1) / STEP : 0);
    // Short sequences are the ill-conditioned ones (fewer keys than features leave directions that only the ridge
    // holds, and a relative error of 2^-11 in w k is then not small against the ridge): they take the weights in
    // fp32 and hand w and w k to the matrix cores as two f16 terms each.  Long ones round w to f16 once and use
    // that same rounded weight in every moment.  (PRECISE is chosen per sequence by the kernel.)
    constexpr bool precise = PRECISE;
    const bf16_t *Kh = a.Kg + b * a.sk.batch + h * a.sk.head;
    const bf16_t *Vh = a.Vg + b * a.sv.batch + h * a.sv.head;

    // query fragments, the same for every column of the B operand: lane (g, *) holds q[32 c + 8 g ..+7]
    // (as f16, like the tiles: exact for values in the f16 range)
    half8 qf[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const uint4 u = *reinterpret_cast<const uint4 *>(a.qg + (size_t)bh * D + 32 * c + 8 * g);
        qf[c] = __builtin_bit_cast(half8, make_uint4(bf16x2_to_f16x2(u.x), bf16x2_to_f16x2(u.y), bf16x2_to_f16x2(u.z), bf16x2_to_f16x2(u.w)));
    }

    // This wave's part of a stage.  A stage is 16 transfers of 1 KB (8 for the K tile, then 8 for the V tile; transfer T
    // fills LDS chunk slots [64 (T % 8), 64 (T % 8) + 64) of its tile).  The wave that forms the weights brings one of
    // them, each of the other three brings five: bringing a transfer also means converting it, and the weight wave has
    // the most vector work already.
    constexpr bool PRODUCER = (WA == 1 && WB == 0);
    constexpr int NTR = PRODUCER ? 1 : 5;          // (0 / 5 / 5 / 6 and 0 / 6 / 4 / 6 measured the same)
    constexpr int TR0 = PRODUCER ? 0 : (WA == 0 ? (WB == 0 ? 1 : 6) : 11);
    int dma_key[NTR], dma_col[NTR];
    unsigned dma_off[NTR];
#pragma unroll
    for (int t = 0; t < NTR; ++t) {
        const int T = TR0 + t, sl = 64 * (T % 8) + lane;
        dma_key[t] = sl >> 4;
        dma_col[t] = ((sl & 15) ^ swz(dma_key[t])) * 8;
        dma_off[t] = 2u * (unsigned)(dma_key[t] * (int)(T < 8 ? a.sk.seq : a.sv.seq) + dma_col[t]);
    }
    // logits operand (natural rows): key 16 sub + nn, chunks 4 c + g
    // (LDS byte addresses relative to the start of a stage: a step adds the stage's scalar base once per address,
    // everything else is an immediate offset of the read)
    unsigned nat[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) nat[c] = 2u * (unsigned)(nn * D + (((4 * c + g) ^ swz(nn)) * 8));
    // transposed operand: inside a 16-lane group, lane j addresses 4 features (16 I + 4 (j % 4) ..) of key
    // 4 g + j / 4; the instruction hands lane i the 4 keys 4g .. 4g+3 of feature 16 I + i
    unsigned tr_addr[NB];
    {
        const int key = 4 * g + (nn >> 2);
#pragma unroll
        for (int I = 0; I < NB; ++I) {
            const int c = 2 * I + ((nn & 3) >> 1);
            tr_addr[I] = 2u * (unsigned)(key * D + ((c ^ swz(key)) * 8) + (nn & 1) * 4);
        }
    }

    f32x4 sig[NS], gt[16], muacc[4], yvacc[4];
#pragma unroll
    for (int t = 0; t < NS; ++t) sig[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < 16; ++t) gt[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < 4; ++t) { muacc[t] = f32x4{0.f, 0.f, 0.f, 0.f}; yvacc[t] = f32x4{0.f, 0.f, 0.f, 0.f}; }
    float om = 0.f, m = -INFINITY;
    const unsigned lds0 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(lds_void_ptr)stage);

    // workgroups that start together on equally spaced addresses would keep hitting the same memory channels in
    // step; each sweeps its share from a different starting step and wraps around (the moments do not depend on
    // the order of the keys)
    const int rot = nsteps > 0 ? (int)((part * 7u + bh * 13u) % (unsigned)nsteps) : 0;
    auto step_pos = [&](int step) { const int t = step + rot; return t >= nsteps ? t - nsteps : t; };
    auto issue_dma = [&](int step) {
        const unsigned dst = lds0 + 2u * (unsigned)((step % NSTAGE) * STAGE_H);      // LDS byte address of the stage
        const int j0 = r0 + step_pos(step < nsteps ? step : 0) * STEP;
        if (j0 + STEP <= L) {
            const bf16_t *kb = Kh + (int64_t)j0 * a.sk.seq, *vb = Vh + (int64_t)j0 * a.sv.seq;
#pragma unroll
            for (int t = 0; t < NTR; ++t) {
                const int T = TR0 + t;
                dma16_base_nt_off(T < 8 ? kb : vb, dma_off[t], dst + 2u * ((T / 8) * TILE_H + 512 * (T % 8)));
            }
        } else {      // a step that reaches past the sequence (or an idle workgroup): rows clamped to the last valid one
#pragma unroll
            for (int t = 0; t < NTR; ++t) {
                const int T = TR0 + t;
                const int j = max(min(j0 + dma_key[t], L - 1), 0);
                dma16_nt_off((T < 8 ? Kh + (int64_t)j * a.sk.seq : Vh + (int64_t)j * a.sv.seq) + dma_col[t],
                             dst + 2u * ((T / 8) * TILE_H + 512 * (T % 8)));
            }
        }
    };

    // bf16 -> f16 in place for the part of a stage that this wave's own transfers brought in (so only the wave's own
    // wait is needed before it): every element is converted once per workgroup, not once per wave that uses it
    auto convert_own = [&](unsigned st) {
        const unsigned base = st + 16u * (unsigned)lane;
        // all reads first, then all writes: read and written addresses are the same ones, but the compiler cannot know
        // that the transfers do not overlap each other and would wait for every read before the write in front of the next
        uint4v u[NTR];
#pragma unroll
        for (int t = 0; t < NTR; ++t) {
            const int T = TR0 + t;
            u[t] = *(lds_uint4_ptr)(uintptr_t)(base + 1024u * (T % 8) + (T / 8) * (TILE_H * 2));
        }
#pragma unroll
        for (int t = 0; t < NTR; ++t) {
            const int T = TR0 + t;
            *(lds_uint4_ptr)(uintptr_t)(base + 1024u * (T % 8) + (T / 8) * (TILE_H * 2)) =
                uint4v{bf16x2_to_f16x2(u[t].x), bf16x2_to_f16x2(u[t].y), bf16x2_to_f16x2(u[t].z), bf16x2_to_f16x2(u[t].w)};
        }
    };
    // logits of the 32 keys of a step whose K tile lies at LDS byte address kt: lane (g, *) gets keys 4g..4g+3
    // (sub-tile 0) and 16+4g.. (sub-tile 1); returns their maximum over the wave
    auto logits = [&](unsigned kt, int step, float (&tl)[8]) {
        const int j0 = r0 + step_pos(step) * STEP;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            f32x4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < 4; ++c)
                z = mfma_f16(*(lds_half8_ptr)(uintptr_t)(kt + nat[c] + sub * 16 * D * 2), qf[c], z);
#pragma unroll
            for (int r = 0; r < 4; ++r) tl[4 * sub + r] = z[r] * a.cscale;
        }
        // only a step that reaches past the wave's share (or lies past its last step) masks keys
        if (__builtin_amdgcn_readfirstlane((j0 + STEP > r1 || step >= nsteps) ? 1 : 0)) {
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int j = j0 + 16 * (t >> 2) + 4 * g + (t & 3);
                if (!(j < r1 && step < nsteps)) tl[t] = -INFINITY;
            }
        }
        // all 16 lanes of a row hold the same 8 logits; the maximum over the four rows goes through two row
        // broadcasts of the data-parallel primitives (no LDS round trips) and ends up in the last row
        float mx = fmaxf(fmaxf(fmaxf(tl[0], tl[1]), fmaxf(tl[2], tl[3])), fmaxf(fmaxf(tl[4], tl[5]), fmaxf(tl[6], tl[7])));
        mx = fmaxf(mx, rows_1_3_from_rows_0_2(mx));
        mx = fmaxf(mx, rows_2_3_from_row_1(mx));
        return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mx), 63));
    };
    // The wave that forms the weights (PRODUCER) keeps the running maximum over the workgroup's keys; a step's record
    // says by what factor the moments so far shrink before the step is added (1 unless the maximum moved) and carries
    // the weights relative to the new maximum: wq (f16), and for short sequences the fp32 weights and their f16 tails.
    float wf[8];
    half8 wq, wl;
    auto produce = [&](float mx, const float (&tl)[8], int slot) {
        float alpha = 1.f;
        if (mx > m) {      // both are wave-uniform
            alpha = (m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m - mx);
            m = mx;
        }
        const float mref = (m == -INFINITY) ? 0.f : m;                // an idle workgroup has no maximum yet
        float pf[8];
        half8 pq, pl;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            pf[t] = __builtin_amdgcn_exp2f(tl[t] - mref);             // exp2(-inf) = 0 masks the tail
            pq[t] = (_Float16)pf[t];
            pl[t] = (_Float16)(pf[t] - (float)pq[t]);
        }
        float *rec = xrec + slot * XREC_F;
        if (nn == 0) {                                                // the 16 lanes of a group hold the same 8 weights
            if constexpr (precise) {
                *reinterpret_cast<f32x4 *>(rec + 8 * g) = f32x4{pf[0], pf[1], pf[2], pf[3]};
                *reinterpret_cast<f32x4 *>(rec + 8 * g + 4) = f32x4{pf[4], pf[5], pf[6], pf[7]};
                *reinterpret_cast<half8 *>(rec + 48 + 4 * g) = pl;
            }
            *reinterpret_cast<half8 *>(rec + 32 + 4 * g) = pq;
            if (g == 0) { rec[64] = alpha; rec[65] = m; }
        }
    };
    // every wave, after the barrier that follows the record's writing: shrink the moments if the maximum moved, take the
    // weights; omega sums them exactly as the matrix cores see them (only the wave that writes it keeps it)
    auto take = [&](int slot) {
        const float *rec = xrec + slot * XREC_F;
        const float alpha = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, rec[64])));
        if constexpr (!PRODUCER) m = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, rec[65])));
        wq = *reinterpret_cast<const half8 *>(rec + 32 + 4 * g);
        if constexpr (precise) {
            const f32x4 f0 = *reinterpret_cast<const f32x4 *>(rec + 8 * g), f1 = *reinterpret_cast<const f32x4 *>(rec + 8 * g + 4);
#pragma unroll
            for (int t = 0; t < 4; ++t) { wf[t] = f0[t]; wf[4 + t] = f1[t]; }
            wl = *reinterpret_cast<const half8 *>(rec + 48 + 4 * g);
        }
        if (alpha != 1.f) {      // wave-uniform
            om *= alpha;
#pragma unroll
            for (int t = 0; t < NS; ++t) sig[t] *= alpha;
#pragma unroll
            for (int t = 0; t < 16; ++t) gt[t] *= alpha;
#pragma unroll
            for (int t = 0; t < 4; ++t) { muacc[t] *= alpha; yvacc[t] *= alpha; }
        }
        if constexpr (WA == 0 && WB == 0) {
#pragma unroll
            for (int t = 0; t < 8; ++t) om += precise ? wf[t] : (float)wq[t];
        }
    };

    // NSTAGE - 1 stages are issued ahead.  Iteration s multiplies step s into the moments and, independently of
    // that, forms the logits and weights of step s + 1, so that the chain "LDS read, logits, maximum over the wave,
    // exponentials" of one step lies beside the matrix-core work of the step before instead of in front of it.
    // An iteration therefore reads stages s and s + 1: it first waits for this wave's transfers of step s + 1 and
    // converts what they brought, then meets the other waves (now the whole stage s + 1 is there as f16, and
    // everybody has finished reading stage s - 1), and only then refills that oldest stage with step s + NSTAGE - 1.  Every iteration issues exactly
    // one stage (clamped past the end), so "at most NTR (NSTAGE - 3) of its own transfers pending" always means
    // "step s + 1 has landed".
#pragma unroll
    for (int st = 0; st < NSTAGE - 1; ++st) issue_dma(st);
    dma_wait_pending<NTR *(NSTAGE - 2)>();
    convert_own(lds0);
    __syncthreads();
    if constexpr (PRODUCER) {
        float tl[8];
        const float mx = logits(lds0, 0, tl);
        produce(mx, tl, 0);                    // published by the barrier of the first iteration
    }
    // The loop is unrolled over the NSTAGE stages (for the long sequences; the short ones keep the stage a run-time
    // scalar): with the stage a compile-time constant, its LDS offset becomes part of the immediate offset of every
    // read, and the per-lane addresses need no vector addition per read and step.
    auto iteration = [&](int s, auto stage_tag) {
        constexpr int STG = decltype(stage_tag)::value;                      // >= 0: the stage of step s, known here
        unsigned kt, kn;
        if constexpr (STG >= 0) {
            kt = lds_offset(stage) + STG * (STAGE_H * 2);
            kn = lds_offset(stage) + ((STG + 1) % NSTAGE) * (STAGE_H * 2);
        } else {
            kt = lds0 + (unsigned)(s % NSTAGE) * (STAGE_H * 2);
            kn = lds0 + (unsigned)((s + 1) % NSTAGE) * (STAGE_H * 2);
            asm volatile("" : "+s"(kt), "+s"(kn));      // scalars that the optimiser cannot take apart into per-read induction registers
        }
        dma_wait_pending<NTR *(NSTAGE - 3)>();
        convert_own(kn);
        __syncthreads();
        issue_dma(s + NSTAGE - 1);
        take(s & 1);
        const unsigned vt = kt + TILE_H * 2;

        half8 kA[4], vB[4], kB[SIG_FULL ? 4 : 1];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            kA[i] = tr_frag(kt + tr_addr[4 * WA + i]);
            vB[i] = tr_frag(vt + tr_addr[4 * WB + i]);
            if constexpr (SIG_FULL) kB[i] = tr_frag(kt + tr_addr[4 + i]);
        }
        auto row_mfmas = [&](int i, const half8 &af) {
            if constexpr (SIG_DIAG) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (j >= i) sig[tix4(i, j)] = mfma_f16(af, kA[j], sig[tix4(i, j)]);
            }
            if constexpr (SIG_FULL) {
#pragma unroll
                for (int j = 0; j < 4; ++j) sig[4 * i + j] = mfma_f16(af, kB[j], sig[4 * i + j]);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) gt[4 * i + j] = mfma_f16(af, vB[j], gt[4 * i + j]);
        };
        auto bcast_mfmas = [&](const half8 &wv) {
            if constexpr (HAS_MU) {
#pragma unroll
                for (int j = 0; j < 4; ++j) muacc[j] = mfma_f16(wv, kA[j], muacc[j]);      // every row = mu~[64 WA + 16 j + nn]
            }
            if constexpr (HAS_YV) {
#pragma unroll
                for (int j = 0; j < 4; ++j) yvacc[j] = mfma_f16(wv, vB[j], yvacc[j]);      // every row = (sum w v)[64 WB + 16 j + nn]
            }
        };
        float tln[8];
        float mxn = -INFINITY;
        if constexpr (PRODUCER) mxn = logits(kn, s + 1, tln);
        if constexpr (!precise) {
#pragma unroll
            for (int i = 0; i < 4; ++i) row_mfmas(i, kA[i] * wq);
            bcast_mfmas(wq);
        } else {
            // w k in fp32 (exact up to the rounding of w), handed to the matrix cores as an f16 head plus an f16 tail
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                half8 ah, al;
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const float pr = (float)kA[i][t] * wf[t];
                    ah[t] = (_Float16)pr;
                    al[t] = (_Float16)(pr - (float)ah[t]);
                }
                row_mfmas(i, ah);
                row_mfmas(i, al);
            }
            bcast_mfmas(wq);
            bcast_mfmas(wl);
        }
        if constexpr (PRODUCER) produce(mxn, tln, (s + 1) & 1);
    };
    if constexpr (!precise) {
        static_assert(NSTAGE == 4, "the unrolled loop below names the stages");
        for (int s = 0; s < nsteps; s += NSTAGE) {
            iteration(s, std::integral_constant<int, 0>{});
            if (s + 1 < nsteps) iteration(s + 1, std::integral_constant<int, 1>{});
            if (s + 2 < nsteps) iteration(s + 2, std::integral_constant<int, 2>{});
            if (s + 3 < nsteps) iteration(s + 3, std::integral_constant<int, 3>{});
        }
    } else {
        for (int s = 0; s < nsteps; ++s) iteration(s, std::integral_constant<int, -1>{});
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");        // drain the clamped tail transfers before the wave ends

    om += __shfl_xor(om, 16);
    om += __shfl_xor(om, 32);
    float *P = a.parts + ((size_t)bh * a.nparts + part) * PART_F;
    if (WA == 0 && WB == 0 && lane == 0) { P[0] = m; P[1] = om; }
    if (g == 0) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (HAS_MU) P[D + 64 * WA + 16 * j + nn] = muacc[j][0];
            if constexpr (HAS_YV) P[2 * D + 64 * WB + 16 * j + nn] = yvacc[j][0];
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int I = 4 * WA + i, J = 4 * WB + j;
            if constexpr (SIG_DIAG) {
                if (j >= i) *reinterpret_cast<f32x4 *>(P + HDR + S128::tix(I, J) * 256 + lane * 4) = sig[tix4(i, j)];
            }
            if constexpr (SIG_FULL) *reinterpret_cast<f32x4 *>(P + HDR + S128::tix(I, J) * 256 + lane * 4) = sig[4 * i + j];
            *reinterpret_cast<f32x4 *>(P + HDR + (NSIG + NB * I + J) * 256 + lane * 4) = gt[4 * i + j];
        }
    }
}

__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(2, 2))) void decode128_partial_kernel(PartialArgs a)
{
    __shared__ __align__(16) bf16_t stage[NSTAGE * STAGE_H];       // 4 stages x 16 KB
    __shared__ __align__(16) float xrec[2][XREC_F];                // the weights of a step, from the wave that forms them to all four
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64), lane = threadIdx.x % 64;
    // Scalar branches: each wave runs the loop of its own share; all of them meet at the same barriers.  The shares
    // differ in work (16 tiles plus the weights, 30 to 36 tiles), and wave w of every workgroup runs on SIMD w of its compute unit; the shares
    // therefore rotate with the workgroup index, so that no SIMD gets the heaviest share from both of its workgroups.
    const int b = (int)blockIdx.y / a.H;
    const int L = a.seqlens ? min(max(a.seqlens[b], 1), a.L_max) : a.L_max;
    const int role = (wave + (int)blockIdx.x + (int)blockIdx.y) & 3;
    if (__builtin_amdgcn_readfirstlane(L <= PRECISE_L ? 1 : 0)) {
        if (role == 0) partial_body<0, 0, true>(a, stage, &xrec[0][0], wave, lane);
        else if (role == 1) partial_body<0, 1, true>(a, stage, &xrec[0][0], wave, lane);
        else if (role == 2) partial_body<1, 0, true>(a, stage, &xrec[0][0], wave, lane);
        else partial_body<1, 1, true>(a, stage, &xrec[0][0], wave, lane);
    } else {
        if (role == 0) partial_body<0, 0, false>(a, stage, &xrec[0][0], wave, lane);
        else if (role == 1) partial_body<0, 1, false>(a, stage, &xrec[0][0], wave, lane);
        else if (role == 2) partial_body<1, 0, false>(a, stage, &xrec[0][0], wave, lane);
        else partial_body<1, 1, false>(a, stage, &xrec[0][0], wave, lane);
    }
}

// Merge, solve, output for one head per workgroup (4 waves):
//   phase 1  wave w sums tiles w, w + 4, .. of the head's partial records with the max-rescale factors
//            2^(m_p - m*) into LDS (the merge step of Algorithm 1's running maximum);
//   phase 2  wave 0 solves the augmented system;
//   phase 3  wave w forms o = y0 * (sum w v) + G~^T y1 for the value blocks 2w and 2w + 1.
__global__ __launch_bounds__(NT, 1) void decode128_merge_kernel(const bf16_t *__restrict__ qg, const float *__restrict__ parts,
                                                                int nparts, float lambda, void *__restrict__ og, int out_bf16)
{
    constexpr int TPW = NTILES / 4;                                 // tiles per wave in phase 1
    __shared__ __align__(16) float merged[NTILES][256];
    __shared__ __align__(16) float scw[16 * SC_PITCH];
    __shared__ __align__(16) float mus[D], yvs[D], ys[D + 4];
    __shared__ float oms;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64, g = lane / 16,
              nn = lane % 16;
    const int bh = blockIdx.x;
    const float *P0 = parts + (size_t)bh * nparts * PART_F;

    {   // phase 1
        const float mstar = wave_max_strided(P0, 0, nparts, PART_F, lane);
        float om = 0.f, hv = 0.f;
        f32x4 acc[TPW];
#pragma unroll
        for (int t = 0; t < TPW; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int p = 0; p < nparts; ++p) {
            const float *P = P0 + (size_t)p * PART_F;
            const float mp = P[0];
            const float f = (mp == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mp - mstar);
            om = fmaf(f, P[1], om);
            hv = fmaf(f, P[D + tid], hv);                           // mu~ (threads 0..127), sum w v (128..255)
#pragma unroll
            for (int t = 0; t < TPW; ++t)
                acc[t] += f * *reinterpret_cast<const f32x4 *>(P + HDR + (4 * t + wave) * 256 + lane * 4);
        }
#pragma unroll
        for (int t = 0; t < TPW; ++t) *reinterpret_cast<f32x4 *>(&merged[4 * t + wave][lane * 4]) = acc[t];
        if (tid < D) mus[tid] = hv; else yvs[tid - D] = hv;
        if (tid == 0) oms = om;
    }
    __syncthreads();

    if (wave == 0) {   // phase 2 (scalar branch: the block contains MFMAs)
        f32x4 acc[1][NSIG], rhs[1][NB];
        float om4[1] = {oms}, y0v[1];
#pragma unroll
        for (int t = 0; t < NSIG; ++t) acc[0][t] = -*reinterpret_cast<const f32x4 *>(&merged[t][lane * 4]);
#pragma unroll
        for (int P = 0; P < NB; ++P)        // the solve takes -(Sigma~ + lambda I)
#pragma unroll
            for (int t = 0; t < 4; ++t) acc[0][S128::tix(P, P)][t] -= (nn == 4 * g + t) ? lambda : 0.f;
        solve_wave_v1<128>(acc, rhs, y0v, om4, scw, g, nn, 0.5f * lambda, [&](int P, float &m, float &q, float &e) {
            m = -mus[16 * P + nn];
            q = -bf16_to_f32(qg[(size_t)bh * D + 16 * P + nn]);
            (void)e;
        });
        if (nn == 0) {
#pragma unroll
            for (int P = 0; P < NB; ++P) *reinterpret_cast<f32x4 *>(&ys[16 * P + 4 * g]) = rhs[0][P];
            if (g == 0) ys[D] = y0v[0];
        }
    }
    __syncthreads();

    {   // phase 3
        const float y0 = ys[D];
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const int J = 2 * wave + jj;
            float s = 0.f;
#pragma unroll
            for (int I = 0; I < NB; ++I) {
                const f32x4 gv = *reinterpret_cast<const f32x4 *>(&merged[NSIG + NB * I + J][lane * 4]);
                const f32x4 y1 = *reinterpret_cast<const f32x4 *>(&ys[16 * I + 4 * g]);
#pragma unroll
                for (int t = 0; t < 4; ++t) s = fmaf(gv[t], y1[t], s);      // G~[16I+4g+t][16J+nn] y1[16I+4g+t]
            }
            s += __shfl_xor(s, 16);
            s += __shfl_xor(s, 32);
            const float o = fmaf(y0, yvs[16 * J + nn], s);
            if (g == 0) {
                if (out_bf16) ((bf16_t *)og)[(size_t)bh * D + 16 * J + nn] = f32_to_bf16(o);
                else ((float *)og)[(size_t)bh * D + 16 * J + nn] = o;
            }
        }
    }
}

}  // namespace

size_t mfma_decode128_workspace_bytes(int B, int H, int L_max)
{
    if (L_max < MIN_L) return 0;
    const Split s = make_split(B * H, L_max);
    return round_up((size_t)B * H * s.nsplit * PART_F * sizeof(float), 256);
}

hipError_t mfma_decode128(const Problem &p)
{
    const int bh = p.B * p.H;
    const Split s = make_split(bh, p.n);
    PartialArgs a;
    a.qg = (const bf16_t *)p.Q;
    a.Kg = (const bf16_t *)p.K;
    a.Vg = (const bf16_t *)p.V;
    a.sk = p.sk;
    a.sv = p.sv;
    a.seqlens = p.seqlens;
    a.H = p.H;
    a.L_max = p.n;
    a.nparts = s.nsplit;
    a.cscale = p.scale * LOG2E;
    a.parts = static_cast<float *>(p.ws);
    stage_mark(p.stream, "decode_partial");
    hipLaunchKernelGGL(decode128_partial_kernel, dim3(s.nsplit, bh), dim3(NT), 0, p.stream, a);
    stage_mark(p.stream, "decode_merge");
    hipLaunchKernelGGL(decode128_merge_kernel, dim3(bh), dim3(NT), 0, p.stream, (const bf16_t *)p.Q, (const float *)a.parts,
                       s.nsplit, p.lambda, p.O, p.out == LLLA_BF16 ? 1 : 0);
    return hipGetLastError();
}

}  // namespace llla

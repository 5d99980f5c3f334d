// Matrix-core forward path for fp32 inputs, d = 64: the contractions of Algorithm 1 (Section 3.2) -- logits,
// first moment, second moment -- on v_mfma_f32_16x16x4_f32, fp32 operands and fp32 accumulation throughout, so the
// path has the accuracy of the vector kernels and no value-range condition.
//
//   moments  per block of 16 queries: weights, omega_i, mu~_i and Sigma~_i (Eq. (tilded_form)) on chip, the ten upper
//            16x16 tiles of Sigma~_i per query in MFMA accumulators, then the exact per-query solve (solve_wave_q4);
//   output   third loop of Algorithm 1 as a flash-style sweep, its three products on fp32 MFMA as well;
//   rows that see at most 64 keys are rewritten by the fp64 key-space kernel (llla_dual.hip).
//
// Running maximum.  There is no separate sweep for the row maxima.  fp32 weights have 2^127 of headroom, so the
// weights are taken relative to a reference exponent mh_i that only moves when a block's largest logit exceeds it by
// more than 2^64 (Algorithm 1's running maximum and rescale, applied lazily: for ordinary data mh_i is the first
// block's maximum and never moves), while the true maximum m_i is tracked beside it.  With F_i = 2^(m_i - mh_i) every
// moment is F_i times the max-normalised one, so the system solved is the max-normalised one times F_i:
// [omega' mu~'^T; mu~' Sigma~' + lambda F I] y' = [1; q], and the output weights w'_ij (y0' + k_j . y1') equal those of
// Eq. (lla).  mh_i and y'_i go to the output sweep; delta_i = delta'_i / F_i (rho_i needs no correction).
#include "llla_mfma_common.hpp"
#include "llla_mfma_solve64.hpp"

namespace llla {
namespace {

using namespace mfma;

constexpr int FD = 64;                 // head dimension
constexpr int FKB = 64;                // keys per block
constexpr int FWP = 68;                // floats per query row of the weight tile
constexpr float LAZY_BITS = 64.f;      // the reference exponent moves when a block exceeds it by more than this

struct F32Layout {
    size_t m, lf, y, total;
    int npad;
};

F32Layout make_f32_layout(int B, int H, int n)
{
    F32Layout L;
    L.npad = (n + FKB - 1) / FKB * FKB;
    const size_t bh = (size_t)B * H;
    size_t off = 0;
    L.m = off;  off += round_up(bh * L.npad * 4, 256);                       // reference exponent mh (log2 units)
    L.lf = off; off += round_up(bh * L.npad * 4, 256);                       // log2 F = m - mh
    L.y = off;  off += round_up(bh * (size_t)n * Shape<FD>::YP * 4, 256);    // y' rows
    L.total = off;
    return L;
}

// The K tile of one block: 64 keys x 64 floats, unpadded (the DMA writes whole 1 KB wave rows), 16-byte chunks
// XOR-swizzled so that both operand reads are free of bank conflicts: chunk c of key row r sits at c ^ swz(r),
// swz(r) = ((r & 1) << 2) | ((r >> 1) & 3).  (b32 reads of rows 4s+g, g = 0..3, 16 consecutive floats each: rows of
// different parity land in different halves of the banks; b128 reads of 8 consecutive rows at one chunk: 8 distinct
// chunk positions.)
__device__ inline int swz(int r) { return ((r & 1) << 2) | ((r >> 1) & 3); }

struct F32Shared {
    float kt[2][FKB * FD];
    float wt[16 * FWP];                // weights of the current block, negated: [query][g * 16 + s], key = 4 s + g
    float pm[4][16];                   // block maximum of every query, per weight wave
    float rs[16];                      // rescale factor of every query for this block (1 unless its reference moved)
    float mus[16][FD + 4];
    float oms[16];
    float fsc[16];                     // F of every query
    float sc[4][4][16 * SC_PITCH];
};

// LIVE: feature blocks of 16 that can be non-zero (4, except for calls at d = 16 / 32 that run here on zero-padded
// copies: the tiles, scaled operands and solve blocks of padded feature blocks are skipped, see moments_body).
template <int LIVE>
__global__ __launch_bounds__(256, 2) void moments_f32_kernel(const float *__restrict__ Qg, const float *__restrict__ Kg,
                                                            llla_strides sq, llla_strides sk, int H, int n, int npad,
                                                            float cscale, float lambda, const float *__restrict__ lam_rows,
                                                            float *__restrict__ Mg, float *__restrict__ LFg,
                                                            float *__restrict__ Yg, int causal)
{
    using S = Shape<FD>;
    constexpr int NB = 4, QW = 4, QB = 16, YP = S::YP;
    __shared__ __align__(16) F32Shared sm;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64, g = lane / 16, nn = lane % 16;
    const BlockMap bm = xcd_block_map();
    const int bh = bm.bh, b = bh / H, h = bh % H;
    const int nqb = gridDim.x;
    const int i0 = (nqb - 1 - bm.blk) * QB;                           // long rows first
    const int ilast = min(i0 + QB - 1, n - 1);
    const int nblk = causal ? ilast / FKB + 1 : (n + FKB - 1) / FKB;
    const float *Kh = Kg + b * sk.batch + h * sk.head;
    const float *Qh = Qg + b * sq.batch + h * sq.head;

    // weight role: lane (g, nn) of wave w serves query i0 + nn and keys 16 w + 4 g + r of a block
    const int iq = i0 + nn;
    const int jlim = causal ? iq : n - 1;                              // last key the lane's query sees
    const bool q_live = iq < n;
    // the 16 query rows wait in LDS (in the rows that hold mu~ after the sweep) instead of in 16 registers per lane:
    // thread t brings floats 4 (t % 16) .. + 3 of query t / 16
    {
        const int qr = tid >> 4, qc = 4 * (tid & 15);
        *reinterpret_cast<f32x4 *>(&sm.mus[qr][qc]) =
            *reinterpret_cast<const f32x4 *>(Qh + (int64_t)min(i0 + qr, n - 1) * sq.seq + qc);
    }

    f32x4 acc[QW][10];
#pragma unroll
    for (int q = 0; q < QW; ++q)
#pragma unroll
        for (int t = 0; t < 10; ++t) acc[q][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    f32x4 mu_acc = {0.f, 0.f, 0.f, 0.f};
    float om_part = 0.f;                   // this lane's share of -omega' of query nn (its keys: 4 g + r of every wave block)
    float mh = -INFINITY, mtrue = -INFINITY;   // reference exponent and true maximum of query nn (log2 units)

    // DMA of one K block: 16 KB = 16 wave transfers of 1 KB, four per wave; transfer t of wave w fills key rows
    // 16 w + 4 t .. + 3; lane l of it writes row 16 w + 4 t + l / 16, stored chunk l % 16
    // Full blocks: a wave-uniform base address per block (scalar registers) plus one 32-bit byte offset per lane and
    // transfer, formed when needed from an opaque copy of the lane index (nothing address-like stays live over the
    // sweep); the last, ragged block clamps its rows to n - 1.
    auto issue_dma = [&](int blk) {
        float *dst = sm.kt[blk & 1];
        int lane_e = lane;
        asm volatile("" : "+v"(lane_e));
        if (blk * FKB + FKB <= n && sk.seq < (int64_t(1) << 23)) {       // whole block, byte offsets fit 32 bits
            const float *base = Kh + (int64_t)blk * FKB * sk.seq;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int row = 16 * wave + 4 * t + (lane_e >> 4);
                const int chunk = (lane_e & 15) ^ swz(row);
                dma16_base(base, (unsigned)(row * (int)sk.seq + 4 * chunk) * 4u, dst + (16 * wave + 4 * t) * FD);
            }
        } else {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int row = 16 * wave + 4 * t + (lane_e >> 4);
                const int j = min(blk * FKB + row, n - 1);
                const int chunk = (lane_e & 15) ^ swz(row);
                dma16(Kh + (int64_t)j * sk.seq + 4 * chunk, dst + (16 * wave + 4 * t) * FD);
            }
        }
    };

    issue_dma(0);
    for (int c = 0; c < nblk; ++c) {
        const float *kt = sm.kt[c & 1];
        dma_wait();
        __syncthreads();                   // tile c complete; everybody is done with block c-1

        // ---- weights of block c: S^T = K Q^T for this wave's 16 keys, contraction slot (s, g) <-> feature 16 g + s ----
        f32x4 z = {0.f, 0.f, 0.f, 0.f};
        {
            const int row = 16 * wave + nn;
            const float *krow = kt + row * FD;
            const int sw = swz(row);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const f32x4 kv = *reinterpret_cast<const f32x4 *>(krow + 4 * ((4 * g + v) ^ sw));
                const f32x4 qv = *reinterpret_cast<const f32x4 *>(&sm.mus[nn][16 * g + 4 * v]);   // Q[query nn][16 g + 4 v ..]
#pragma unroll
                for (int e = 0; e < 4; ++e) z = __builtin_amdgcn_mfma_f32_16x16x4f32(kv[e], qv[e], z, 0, 0, 0);
            }
        }
        float zs[4], pmx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int j = c * FKB + 16 * wave + 4 * g + r;
            zs[r] = z[r] * cscale;
            pmx = (q_live && j <= jlim) ? fmaxf(pmx, zs[r]) : pmx;
        }
        pmx = fmaxf(pmx, __shfl_xor(pmx, 16));
        pmx = fmaxf(pmx, __shfl_xor(pmx, 32));
        if (g == 0) sm.pm[wave][nn] = pmx;
        __syncthreads();
        const float bmx = fmaxf(fmaxf(sm.pm[0][nn], sm.pm[1][nn]), fmaxf(sm.pm[2][nn], sm.pm[3][nn]));
        mtrue = fmaxf(mtrue, bmx);
        float rsc = 1.f;
        if (bmx > mh + LAZY_BITS || (mh == -INFINITY && bmx > -INFINITY)) {       // the reference moves (first block: always)
            rsc = (mh == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mh - bmx);
            mh = bmx;
        }
        if (wave == 0 && g == 0) sm.rs[nn] = rsc;
        om_part *= rsc;
        {
            float wf[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int j = c * FKB + 16 * wave + 4 * g + r;
                const float wgt = __builtin_amdgcn_exp2f(zs[r] - mh);
                wf[r] = (q_live && j <= jlim) ? -wgt : 0.f;           // stored negated: the tiles accumulate -(w k) k^T
                sm.wt[nn * FWP + r * 16 + 4 * wave + g] = wf[r];
            }
            om_part += (wf[0] + wf[1]) + (wf[2] + wf[3]);
        }
        __syncthreads();                   // weights and rescale factors of block c visible
        if (c + 1 < nblk) issue_dma(c + 1);

        // ---- rescale what has been accumulated (factors are 1 unless a reference exponent moved) -------------------
        {
            const f32x4 r4 = *reinterpret_cast<const f32x4 *>(&sm.rs[4 * g]);        // rows 4 g + r of mu~
#pragma unroll
            for (int r = 0; r < 4; ++r) mu_acc[r] *= r4[r];
            const f32x4 mine = *reinterpret_cast<const f32x4 *>(&sm.rs[QW * wave]);  // this wave's four queries
#pragma unroll
            for (int q = 0; q < QW; ++q) {
                if (mine[q] != 1.f) {                                                  // wave-uniform
#pragma unroll
                    for (int t = 0; t < 10; ++t) acc[q][t] *= mine[q];
                }
            }
        }

        // ---- moments of block c: 16 steps of 4 keys ------------------------------------------------------------
#pragma unroll 1
        for (int s4 = 0; s4 < 4; ++s4) {
            // weights of keys 4 s + g, s = 4 s4 .. 4 s4 + 3: for this wave's queries (scaling) and for all 16 (mu~)
            f32x4 wq[QW];
#pragma unroll
            for (int q = 0; q < QW; ++q) wq[q] = *reinterpret_cast<const f32x4 *>(&sm.wt[(QW * wave + q) * FWP + g * 16 + 4 * s4]);
            const f32x4 wa = *reinterpret_cast<const f32x4 *>(&sm.wt[nn * FWP + g * 16 + 4 * s4]);
            // the operand addresses below are formed from copies of the lane indices that the compiler cannot see
            // through: twenty of them are loop-invariant and would otherwise be kept in registers over the whole sweep
            int g_e = g, nn_e = nn;
            asm volatile("" : "+v"(g_e), "+v"(nn_e));
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int row = 4 * (4 * s4 + e) + g_e;
                const float *krow = kt + row * FD + (nn_e & 3);
                const int sw = swz(row), c4 = nn_e >> 2;
                float kf[NB];
#pragma unroll
                for (int I = 0; I < LIVE; ++I) kf[I] = krow[4 * ((4 * I + c4) ^ sw)];
                const float kmu = krow[4 * ((4 * wave + c4) ^ sw)];                   // this wave's feature block of mu~
#pragma unroll
                for (int q = 0; q < QW; ++q)
#pragma unroll
                    for (int I = 0; I < LIVE; ++I) {
                        const float af = kf[I] * wq[q][e];
#pragma unroll
                        for (int J = I; J < LIVE; ++J)
                            acc[q][S::tix(I, J)] = __builtin_amdgcn_mfma_f32_16x16x4f32(af, kf[J], acc[q][S::tix(I, J)], 0, 0, 0);
                    }
                mu_acc = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[e], kmu, mu_acc, 0, 0, 0);   // -mu~'[query 4g+r][16 wave + nn]
            }
        }
    }

    // ---- hand mu~', omega' and F to the waves that own the queries -------------------------------------------------
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 4; ++r) sm.mus[4 * g + r][16 * wave + nn] = mu_acc[r];
    om_part += __shfl_xor(om_part, 16);
    om_part += __shfl_xor(om_part, 32);
    if (g == 0) sm.pm[wave][nn] = om_part;
    const float lf = q_live ? mtrue - mh : 0.f;                          // log2 F
    if (wave == 0 && g == 0) {
        sm.fsc[nn] = __builtin_amdgcn_exp2f(lf);
        if (q_live) {
            Mg[(size_t)bh * npad + iq] = mh;
            LFg[(size_t)bh * npad + iq] = lf;
        }
    }
    __syncthreads();
    if (tid < 16) sm.oms[tid] = -((sm.pm[0][tid] + sm.pm[1][tid]) + (sm.pm[2][tid] + sm.pm[3][tid]));
    __syncthreads();

    // ---- the ridge lambda F on the diagonal (the tiles hold -Sigma~'), then the solve ----------------------------------
    const int qi = QW * wave + g;                                       // solve role: lane (g, nn) = (query, element)
    const int row = min(i0 + qi, n - 1);
#pragma unroll
    for (int q = 0; q < QW; ++q) {
        const int rq = min(i0 + QW * wave + q, n - 1);
        const float lq = (lam_rows ? lam_rows[(size_t)bh * n + rq] : lambda) * sm.fsc[QW * wave + q];
#pragma unroll
        for (int P = 0; P < NB; ++P)
#pragma unroll
            for (int t = 0; t < 4; ++t) acc[q][S::tix(P, P)][t] -= (nn == 4 * g + t) ? lq : 0.f;
    }
    const float pivot_floor = 0.5f * (lam_rows ? lam_rows[(size_t)bh * n + row] : lambda) * sm.fsc[qi];
    const float *qrow = Qh + (int64_t)row * sq.seq;
    float tmu[4], tq[4], te[4], y1[4], u1[4], y0 = 0.f, u0 = 0.f;
#pragma unroll
    for (int P = 0; P < NB; ++P) {
        tmu[P] = sm.mus[qi][16 * P + nn];                                // -mu~'
        tq[P] = -qrow[16 * P + nn];
        te[P] = 0.f; y1[P] = 0.f; u1[P] = 0.f;
    }
    solve_wave_q4<false, LIVE>(acc, tmu, tq, te, 0.f, sm.oms[qi], &sm.sc[wave][0][0], g, nn, pivot_floor, y1, y0, u1, u0);
    if (i0 + qi < n) {
        float *yr = Yg + ((size_t)bh * n + row) * YP;
#pragma unroll
        for (int P = 0; P < NB; ++P) yr[16 * P + nn] = y1[P];
        if (nn == 0) yr[FD] = y0;
    }
}

// Third loop of Algorithm 1 for 64 queries per workgroup (16 per wave): S^T = K Q^T and K y1' on fp32 MFMA, the output
// weights w'_ij (y0'_i + k_j . y1'_i) on the vector ALU, O = S V on fp32 MFMA.  The coefficient tile comes out of the
// first two products in the accumulator layout (lane (g, n): keys 4 g + r of a 16-key sub-tile, query n), which is
// directly the A operand of the third when contraction slot (g, r) stands for key 4 g + r.  K and V tiles of 64 keys
// arrive by DMA, 16-byte chunks XOR-swizzled with the low three bits of the key row (the b128 reads of K rows and the
// b32 reads of V rows 4 g + r are then both free of bank conflicts).
struct OutShared {
    float k[FKB * FD];
    float v[FKB * FD];
};

__global__ __launch_bounds__(256, 2) void output_f32_kernel(const float *__restrict__ Qg, const float *__restrict__ Kg,
                                                         const float *__restrict__ Vg, llla_strides sq, llla_strides sk,
                                                         llla_strides sv, int H, int n, int npad, float cscale,
                                                         const float *__restrict__ Mg, const float *__restrict__ Yg,
                                                         void *__restrict__ Og, llla_strides so, int out_bf16, int causal)
{
    constexpr int YP = Shape<FD>::YP, NB = 4;
    __shared__ __align__(16) OutShared sm;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64, g = lane / 16, nn = lane % 16;
    // head on blockIdx.x (dispatched fastest), query block on y, longest rows first
    const int bh = blockIdx.x, b = bh / H, h = bh % H;
    const int i0 = ((int)gridDim.y - 1 - (int)blockIdx.y) * 64;
    const int iq = i0 + wave * 16 + nn, iqc = min(iq, n - 1);
    const int jlim = causal ? iq : n - 1;
    const float *Kh = Kg + b * sk.batch + h * sk.head;
    const float *Vh = Vg + b * sv.batch + h * sv.head;
    float qreg[16], yreg[16];                                       // Q and y1' of query nn, features 16 g + s
    {
        const float *qrow = Qg + b * sq.batch + h * sq.head + (int64_t)iqc * sq.seq + 16 * g;
        const float *yrow = Yg + ((size_t)bh * n + iqc) * YP + 16 * g;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const f32x4 a = *reinterpret_cast<const f32x4 *>(qrow + 4 * v), c = *reinterpret_cast<const f32x4 *>(yrow + 4 * v);
#pragma unroll
            for (int e = 0; e < 4; ++e) { qreg[4 * v + e] = a[e]; yreg[4 * v + e] = c[e]; }
        }
    }
    const float y0 = Yg[((size_t)bh * n + iqc) * YP + FD];
    const float mh = Mg[(size_t)bh * npad + iqc];
    f32x4 oacc[NB];
#pragma unroll
    for (int J = 0; J < NB; ++J) oacc[J] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int ilast = min(i0 + 63, n - 1);
    const int nblk = causal ? ilast / FKB + 1 : (n + FKB - 1) / FKB;
    for (int c = 0; c < nblk; ++c) {
        __syncthreads();                                            // everybody is done with the previous tiles
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int row = 16 * wave + 4 * t + (lane >> 4);
            const int j = min(c * FKB + row, n - 1);
            const int chunk = (lane & 15) ^ (row & 7);
            dma16(Kh + (int64_t)j * sk.seq + 4 * chunk, sm.k + (16 * wave + 4 * t) * FD);
            dma16(Vh + (int64_t)j * sv.seq + 4 * chunk, sm.v + (16 * wave + 4 * t) * FD);
        }
        dma_wait();
        __syncthreads();
        // blocks that lie wholly before the wave's first query need no causal mask (a scalar condition)
        const bool masked = causal ? (c * FKB + FKB - 1 > i0 + wave * 16) : (c * FKB + FKB > n);
#pragma unroll
        for (int sub = 0; sub < 4; ++sub) {
            f32x4 z = {0.f, 0.f, 0.f, 0.f}, u = {0.f, 0.f, 0.f, 0.f};
            {
                const int row = 16 * sub + nn;
                const float *krow = sm.k + row * FD;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const f32x4 kv = *reinterpret_cast<const f32x4 *>(krow + 4 * ((4 * g + v) ^ (row & 7)));
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        z = __builtin_amdgcn_mfma_f32_16x16x4f32(kv[e], qreg[4 * v + e], z, 0, 0, 0);
                        u = __builtin_amdgcn_mfma_f32_16x16x4f32(kv[e], yreg[4 * v + e], u, 0, 0, 0);
                    }
                }
            }
            float cf[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                cf[r] = __builtin_amdgcn_exp2f(z[r] * cscale - mh) * (y0 + u[r]);
                if (masked) {
                    const int j = c * FKB + 16 * sub + 4 * g + r;
                    cf[r] = (j <= jlim) ? cf[r] : 0.f;
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = 16 * sub + 4 * g + r;
                const float *vrow = sm.v + row * FD + (nn & 3);
#pragma unroll
                for (int J = 0; J < NB; ++J)
                    oacc[J] = __builtin_amdgcn_mfma_f32_16x16x4f32(cf[r], vrow[4 * ((4 * J + (nn >> 2)) ^ (row & 7))], oacc[J], 0, 0, 0);
            }
        }
    }
    // oacc[J]: lane (g, nn) reg r = O[query i0 + 16 wave + 4 g + r][feature 16 J + nn]
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

// Statistics of Eq. (lla) from y' and F: 1/delta' = y0' + q . y1', delta = delta' / F, rho = -delta' y1'.  One wave per row.
__global__ __launch_bounds__(256) void stats_f32_kernel(const float *__restrict__ Qg, llla_strides sq, int H, int n, int npad,
                                                        const float *__restrict__ Yg, const float *__restrict__ LFg,
                                                        float *__restrict__ rho, float *__restrict__ delta)
{
    constexpr int YP = Shape<FD>::YP;
    const int lane = threadIdx.x % 64, i = blockIdx.x * 4 + threadIdx.x / 64, bh = blockIdx.y;
    if (i >= n) return;
    const float *qrow = Qg + (bh / H) * sq.batch + (bh % H) * sq.head + (int64_t)i * sq.seq;
    const float *yr = Yg + ((size_t)bh * n + i) * YP;
    const float y1 = yr[lane];
    float qy = qrow[lane] * y1;
#pragma unroll
    for (int sft = 32; sft >= 1; sft >>= 1) qy += __shfl_xor(qy, sft);
    const float dl = 1.f / (yr[FD] + qy);                                 // delta'
    const size_t row = (size_t)bh * n + i;
    if (delta != nullptr && lane == 0) delta[row] = dl * __builtin_amdgcn_exp2f(-LFg[(size_t)bh * npad + i]);
    if (rho != nullptr) rho[row * FD + lane] = -dl * y1;
}

}  // namespace

bool mfma_forward_f32_supported(int d, bool causal) { (void)causal; return d == FD; }

size_t mfma_forward_f32_workspace_bytes(int B, int H, int n) { return make_f32_layout(B, H, n).total; }

hipError_t mfma_forward_f32(const Problem &p)
{
    using S = Shape<FD>;
    const F32Layout L = make_f32_layout(p.B, p.H, p.n);
    char *ws = static_cast<char *>(p.ws);
    float *M = reinterpret_cast<float *>(ws + L.m), *LF = reinterpret_cast<float *>(ws + L.lf);
    float *Y = reinterpret_cast<float *>(ws + L.y);
    const int bh = p.B * p.H;
    const float *Q = static_cast<const float *>(p.Q), *K = static_cast<const float *>(p.K);
    stage_mark(p.stream, "moments");
    const int live = p.live_d > 0 ? (p.live_d + 15) / 16 : 4;      // a d = 16 / 32 call on zero-padded copies: 1 or 2
    const dim3 grid((p.n + S::QB - 1) / S::QB, bh);
    if (live == 1)
        hipLaunchKernelGGL(moments_f32_kernel<1>, grid, dim3(256), 0, p.stream, Q, K, p.sq, p.sk, p.H, p.n, L.npad,
                           p.scale * LOG2E, p.lambda, p.lambda_rows, M, LF, Y, p.causal);
    else if (live == 2)
        hipLaunchKernelGGL(moments_f32_kernel<2>, grid, dim3(256), 0, p.stream, Q, K, p.sq, p.sk, p.H, p.n, L.npad,
                           p.scale * LOG2E, p.lambda, p.lambda_rows, M, LF, Y, p.causal);
    else
        hipLaunchKernelGGL(moments_f32_kernel<4>, grid, dim3(256), 0, p.stream, Q, K, p.sq, p.sk, p.H, p.n, L.npad,
                           p.scale * LOG2E, p.lambda, p.lambda_rows, M, LF, Y, p.causal);
    if (p.rho != nullptr || p.delta != nullptr) {
        stage_mark(p.stream, "statistics");
        hipLaunchKernelGGL(stats_f32_kernel, dim3((p.n + 3) / 4, bh), dim3(256), 0, p.stream, Q, p.sq, p.H, p.n, L.npad,
                           (const float *)Y, (const float *)LF, p.rho, p.delta);
    }
    stage_mark(p.stream, "output");
    hipLaunchKernelGGL(output_f32_kernel, dim3(bh, (p.n + 63) / 64), dim3(256), 0, p.stream, Q, K, static_cast<const float *>(p.V),
                       p.sq, p.sk, p.sv, p.H, p.n, L.npad, p.scale * LOG2E, (const float *)M, (const float *)Y, p.O, p.so,
                       p.out == LLLA_BF16 ? 1 : 0, p.causal);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // rows that see at most 64 keys: fp64 in key space (their output weights cancel to three digits in fp32)
    stage_mark(p.stream, "few_key_rows");
    return dual_forward(p);
}

}  // namespace llla

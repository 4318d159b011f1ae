// Compressed-space scores, Alg. 1 steps 2-3: P~ = Q~ K~^T / sqrt(d_k), row softmax over composite
// keys, block aggregation Score(i, j) of Eq. (3) with the index sets of Eq. (4).
//
// The (L/c_q) x (L/c_k) matrices P~ and A~ are never written to memory.  A workgroup of four
// wavefronts owns 256 composite query rows that share one key head (4 query heads of a GQA group
// x 64 rows, or fewer heads x more rows) and streams the composite keys through LDS in stages of
// 128.  Each wavefront keeps its 64 query rows as MFMA B operands in registers and computes
// 32-key x 64-query logit tiles transposed (S^T = K~ Q~^T, v_mfma_f32_32x32x16_bf16), so that every
// lane owns whole query rows and the softmax statistics are lane-local.  The query rows are read as composite tokens
// or, since each of them is used by exactly one wavefront, formed from the queries themselves as they are loaded
// (Eq. (1), average pooling; ProxyArgs::qt == NULL).
//
// Two forms.  The two-sweep form needs no memory beyond Score: the first sweep over the keys finds a reference value
// and the denominator of each row, the second sums the normalised probabilities over the composite keys of each key
// block (in registers), then over the composite queries of each query block (cross-lane), and stores Score(i, j).
// The one-sweep form (ROWSUMS) halves the MFMA and exponential work: it writes, for every composite query row t and
// key block j, the unnormalised sum U(t, j) of exp(P~(t, s) - ref_t) over the composite keys s of block j, and the
// row's weight 1 / sum_j U(t, j); the selection kernel then forms Score(i, j) = sum_{t in block i} weight_t U(t, j)
// as it loads its row.  ref_t is fixed by the first key tile and moves only when a tile's sum would pass 2^40; a
// workgroup in which some row's reference moved after values had been written repeats the sweep with the final
// references (the second sweep of the other form), so the common case costs one sweep and the worst case two.
// U is laid out for the selection kernel's loads: per (head, query block) and per 64 key blocks, groups of four
// composite query rows, each group 64 key blocks x 4 rows (a wavefront of the selection kernel reads 1 KB in a row).
#pragma once
#include "common.h"

namespace us {

constexpr int kPxThreads = 256;
constexpr int kPxStageKeys = 128;          // composite keys per LDS stage
constexpr int kPxRowsPerWave = 64;         // query rows per wavefront: two MFMA tiles of 32 (one when QT = 1)
template <int D>
struct PxCfg {
    static constexpr int kSteps = D / 16;                  // MFMA steps over the head dimension
    static constexpr int kPitch = 2 * D + 16;              // bytes per LDS row: + 16 keeps 16-byte row reads conflict-free
    static constexpr int kStageBytes = kPxStageKeys * kPitch;
    static constexpr int kLoads = kPxStageKeys * (D / 8) / kPxThreads;   // 16-byte loads per thread and stage
    // d = 256 doubles the query operands and the prefetch registers: one wavefront per SIMD with 512 registers
    static constexpr int kWaves = D == 256 ? 1 : 2;
};

// Sum over aligned groups of R consecutive lanes (R = 4, 8, 16 or 32), result in every lane of the group: DPP
// lane permutations inside a row of 16 lanes (no LDS traffic), one cross-row exchange for R = 32.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x)
{
    const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true);
    return x + __int_as_float(y);
}
template <int R>
__device__ __forceinline__ float group_sum(float x)
{
    if (R >= 32) x += __shfl_xor(x, 16, 64);
    if (R >= 16) x = dpp_add<0x140>(x);      // row_mirror: lane l <-> 15 - l
    if (R >= 8) x = dpp_add<0x141>(x);       // row_half_mirror: lane l <-> 7 - l inside each half row
    x = dpp_add<0xB1>(x);                    // quad_perm [1, 0, 3, 2]
    x = dpp_add<0x4E>(x);                    // quad_perm [2, 3, 0, 1]
    return x;
}

struct ProxyGeom {
    int HG;          // query heads of one key head handled by a workgroup (1, 2 or 4)
    int RC;          // 64-row chunks per head in a workgroup (4 / HG)
    int GS;          // head slices per key head (G / HG)
    int n_tiles;     // query tiles over all sequences
    int QT;          // 32-row MFMA tiles per wavefront: 2, or 1 to get twice the workgroups out of a small problem
};

template <int D, int NQB, int NKB, bool CAUSAL, int QT = 2, bool ROWSUMS = false>
__global__ __launch_bounds__(kPxThreads) __attribute__((amdgpu_waves_per_eu(PxCfg<D>::kWaves, PxCfg<D>::kWaves)))
void proxy_kernel(ProxyArgs a, ProxyGeom g)
{
    using C = PxCfg<D>;
    constexpr int kPxPitch = C::kPitch, kPxStageBytes = C::kStageBytes, kHeadDim = D;
    constexpr int kPxRowsPerWave = 32 * QT;                // shadows the two-tile default
    static_assert(QT == 2 || NQB <= 32, "a query block must stay inside one wavefront");
    static_assert(!ROWSUMS || NKB >= 8, "the one-sweep form is not offered for key blocks of 4 composite keys");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int lr = lane & 31;            // column of the MFMA tile this lane owns (a query row)
    const int lh = lane >> 5;            // lane half

    // ---- which (key head, head slice, sequence, query tile) ------------------------------------
    const int vid = xcd_contiguous_id(blockIdx.x, gridDim.x);
    const int per_kv = g.n_tiles * g.GS;
    const int kvh = vid / per_kv;
    int rem = vid % per_kv;
    const int tile_rank = rem / g.GS;
    const int gs = rem % g.GS;
    int tile = g.n_tiles - 1 - tile_rank;                  // longest (latest) tiles first
    const int rows_per_tile = kPxRowsPerWave * g.RC;
    int seq = 0, qt = 0;
    {
        int base = 0;
        for (int b = 0; b < a.st.num_seqs; ++b) {
            int lq = a.cu_cq[b + 1] - a.cu_cq[b];
            int nt = (lq + rows_per_tile - 1) / rows_per_tile;
            if (tile < base + nt) { seq = b; qt = tile - base; break; }
            base += nt;
        }
    }
    const int tok0 = a.st.cu_tok[seq];
    const int Lb = a.st.cu_tok[seq + 1] - tok0;
    const int Lq = a.cu_cq[seq + 1] - a.cu_cq[seq], Lk = a.cu_ck[seq + 1] - a.cu_ck[seq];   // a last window may be partial
    const int Nb = (Lb + a.S - 1) / a.S;                    // the last block may be a shorter remainder
    const int64_t Tq = a.cu_cq[a.st.num_seqs], Tk = a.cu_ck[a.st.num_seqs];
    int row_base = 0;                                       // packed query-block row of the sequence's block 0
    for (int b = 0; b < seq; ++b) row_base += (a.st.cu_tok[b + 1] - a.st.cu_tok[b] + a.S - 1) / a.S;

    const int G = a.n_heads_q / a.n_heads_kv;
    const int hh = wave % g.HG, rc = wave / g.HG;
    const int head = kvh * G + gs * g.HG + hh;
    const int t0 = (qt * g.RC + rc) * kPxRowsPerWave;       // first composite query row of this wavefront
    const bool wave_active = t0 < Lq;

    // highest visible composite key of a composite query row
    auto limit_of = [&](int t) -> int {
        int lim = Lk - 1;
        if (CAUSAL) {
            int c = ((t + 1) * a.c_q - 1) / a.c_k;
            lim = c < lim ? c : lim;
        }
        return lim;
    };
    const int tile_last_row = min((qt + 1) * rows_per_tile, Lq) - 1;
    const int n_stages = limit_of(tile_last_row) / kPxStageKeys + 1;
    const int w_first = min(t0, Lq - 1), w_last = min(t0 + kPxRowsPerWave - 1, Lq - 1);
    const int lim_first = limit_of(w_first), lim_last = limit_of(w_last);

    // ---- query rows of this lane as B operands ---------------------------------------------------
    bf16x8 qreg[QT][C::kSteps];
    int lim_row[QT];
#pragma unroll
    for (int qb = 0; qb < QT; ++qb) {
        int t = min(t0 + 32 * qb + lr, Lq - 1);
        lim_row[qb] = limit_of(t);
        if (a.qt != nullptr) {                              // (uniform) composite queries pooled by an earlier pass
            const bf16_t *src = a.qt + ((int64_t)head * Tq + a.cu_cq[seq] + t) * kHeadDim + 8 * lh;
#pragma unroll
            for (int ks = 0; ks < C::kSteps; ++ks) qreg[qb][ks] = *reinterpret_cast<const bf16x8 *>(src + 16 * ks);
        } else {
            // Eq. (1) on the fly, the arithmetic of the pooling kernel: fp32 sum of the window's tokens in token
            // order (the sequence's last window may be short), one division, one rounding to bf16
            const int cnt = min(a.c_q, Lb - t * a.c_q);
            const bf16_t *src = a.q_src.ptr + (int64_t)head * a.q_src.stride_head +
                                ((int64_t)tok0 + (int64_t)t * a.c_q) * a.q_src.stride_tok + 8 * lh;
            float acc[C::kSteps][8];
#pragma unroll
            for (int ks = 0; ks < C::kSteps; ++ks)
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[ks][e] = 0.0f;
#pragma unroll 2
            for (int m = 0; m < a.c_q; ++m) {
                if (m < cnt) {
                    u32x4 w[C::kSteps];
#pragma unroll
                    for (int ks = 0; ks < C::kSteps; ++ks)
                        w[ks] = *reinterpret_cast<const u32x4 *>(src + (int64_t)m * a.q_src.stride_tok + 16 * ks);
#pragma unroll
                    for (int ks = 0; ks < C::kSteps; ++ks) {
                        float f[8];
                        unpack8(w[ks], f);
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[ks][e] += f[e];
                    }
                }
            }
            const float cf = (float)cnt;
#pragma unroll
            for (int ks = 0; ks < C::kSteps; ++ks) {
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[ks][e] = acc[ks][e] / cf;
                const u32x4 pk = pack8_rne(acc[ks]);
                qreg[qb][ks] = __builtin_bit_cast(bf16x8, pk);
            }
        }
    }

    const bf16_t *kbase = a.kt + ((int64_t)kvh * Tk + a.cu_ck[seq]) * kHeadDim;
    u32x4 pre[C::kLoads];
    auto load_stage = [&](int st) {
#pragma unroll
        for (int it = 0; it < C::kLoads; ++it) {
            int id = it * kPxThreads + tid;
            int r = min(st * kPxStageKeys + id / (D / 8), Lk - 1);
            pre[it] = *reinterpret_cast<const u32x4 *>(kbase + (int64_t)r * kHeadDim + (id % (D / 8)) * 8);
        }
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int it = 0; it < C::kLoads; ++it) {
            int id = it * kPxThreads + tid;
            *reinterpret_cast<u32x4 *>(lds + buf * kPxStageBytes + (id / (D / 8)) * kPxPitch + (id % (D / 8)) * 16) = pre[it];
        }
    };

    const float c2 = a.scale_log2;
    float m_run[QT], l_run[QT], mc[QT], wnorm[QT];
#pragma unroll
    for (int qb = 0; qb < QT; ++qb) {
        m_run[qb] = -INFINITY;
        l_run[qb] = 0.0f;
        mc[qb] = -INFINITY;             // first sweep: the scaled reference value (none yet); second sweep: the final one
        wnorm[qb] = 0.0f;
    }

    // Key blocks against the registers of a 32-key tile: register v of a lane holds key
    // 8 (v / 4) + 4 lh + v % 4.  n_k >= 8: a block is one or more groups of 8 keys, summed
    // over both lane halves; n_k = 4: a block is the four keys of one lane half; n_k = 64: a
    // block is two tiles, the second tile adds to what the first one stored.
    constexpr bool kHalfBlocks = NKB == 4, kTwoTiles = NKB == 64;
    constexpr int NBK = kHalfBlocks ? 4 : (NKB >= 32 ? 1 : 32 / NKB);   // bins per lane
    constexpr int GPB = kHalfBlocks ? 1 : (NKB >= 32 ? 4 : NKB / 8);    // register groups per bin

    // one-sweep form: where this lane's rows go in U - element (row r of query block i, key block j) lives at
    // [head][i][j / 64][r / 4][j % 64][r % 4] - and whether some row's reference moved after values relative to the
    // old one had been stored.  Rows past the sequence's end (copies of its last row) fill the rest of a last,
    // partial query block (they weigh 0) and have no place beyond it.
    constexpr int kRowGroup = (NQB / 4) * 256;              // floats per 64 key blocks of one query block
    float *ub[QT] = {};
    bool row_ok[QT] = {};
    bool moved = false;
    if constexpr (ROWSUMS) {
        const int64_t nk64 = (a.NK + 63) / 64;
#pragma unroll
        for (int qb = 0; qb < QT; ++qb) {
            const int t = t0 + 32 * qb + lr, blk = t / NQB, r = t % NQB;
            row_ok[qb] = blk < Nb;
            ub[qb] = a.u + ((int64_t)head * a.NQ + row_base + blk) * nk64 * kRowGroup + (r / 4) * 256 + r % 4;
        }
    }
    auto u_at = [&](int qb, int j) -> float & { return ub[qb][(j >> 6) * kRowGroup + (j & 63) * 4]; };

    // ---- per-tile work, as separate pieces so that the MFMAs of one tile can run under the VALU work of another
    // S^T of one 32-key tile for both query tiles (each K operand read feeds two MFMAs)
    auto mfma_tile = [&](f32x16 (&dst)[QT], const unsigned char *kb, int sub) __attribute__((always_inline)) {
        f32x16 zero;
#pragma unroll
        for (int v = 0; v < 16; ++v) zero[v] = 0.0f;
        const unsigned char *arow = kb + (32 * sub + lr) * kPxPitch + 16 * lh;
#pragma unroll
        for (int ks = 0; ks < C::kSteps; ++ks) {
            bf16x8 ka = *reinterpret_cast<const bf16x8 *>(arow + 32 * ks);
#pragma unroll
            for (int qb = 0; qb < QT; ++qb)
                dst[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[qb][ks], ks == 0 ? zero : dst[qb], 0, 0, 0);
        }
    };
    // first sweep: a reference value and the denominator (relative to it) of every composite query row.  Softmax is
    // shift-invariant, so the reference need not be the row maximum: it is the maximum of the first tile that shows
    // the row a visible key and moves only when a tile's sum of exponentials passes 2^40 (or is not finite: no
    // reference yet, or a logit hundreds of units above it).  The common case is one fma, one exponential and one
    // add per value; the tile is redone with its true maximum otherwise.
    auto stats_tile = [&](const f32x16 (&src)[QT]) __attribute__((always_inline)) {
        constexpr float kBig = 1099511627776.0f;           // 2^40
        float sum[QT];
        bool need[QT], redo = false;
#pragma unroll
        for (int qb = 0; qb < QT; ++qb) {
            sum[qb] = 0.0f;
#pragma unroll
            for (int v = 0; v < 16; ++v) sum[qb] += fast_exp2(fmaf(src[qb][v], c2, -mc[qb]));
            need[qb] = !(sum[qb] <= kBig);
            redo = redo || need[qb];
        }
        if (__any(redo)) {                                 // (a row's reference moves only on that row's own account)
#pragma unroll
            for (int qb = 0; qb < QT; ++qb) {
                float mx = src[qb][0];
#pragma unroll
                for (int v = 1; v < 16; ++v) mx = fmaxf(mx, src[qb][v]);
                const float m_new = need[qb] ? fmaxf(m_run[qb], mx) : m_run[qb];
                const bool none = m_new == -INFINITY;      // nothing visible to this row yet
                const float m_safe = none ? 0.0f : m_new;
                const float alpha = fast_exp2((m_run[qb] - m_safe) * c2);
                const float msc = m_safe * c2;
                float sm = 0.0f;
#pragma unroll
                for (int v = 0; v < 16; ++v) sm += fast_exp2(fmaf(src[qb][v], c2, -msc));
                sum[qb] = sm;
                l_run[qb] *= alpha;
                m_run[qb] = m_new;
                mc[qb] = none ? -INFINITY : msc;
            }
        }
#pragma unroll
        for (int qb = 0; qb < QT; ++qb) l_run[qb] += sum[qb];
    };
    // second sweep: normalised probabilities summed over the composite keys of each key block (registers),
    // then over the composite queries of each query block (lanes), stored as Score(i, j)
    auto bins_tile = [&](const f32x16 (&src)[QT], int s_lo, int sub) __attribute__((always_inline)) {
        constexpr int QR = NQB < 32 ? NQB : 32;                             // lanes of one query block
        float bin[QT][NBK];
#pragma unroll
        for (int qb = 0; qb < QT; ++qb) {
#pragma unroll
            for (int b = 0; b < NBK; ++b) bin[qb][b] = 0.0f;
#pragma unroll
            for (int v = 0; v < 16; ++v)
                bin[qb][(v >> 2) / GPB] += fast_exp2(fmaf(src[qb][v], c2, -mc[qb]));
#pragma unroll
            for (int b = 0; b < NBK; ++b) {
                float x = bin[qb][b] * wnorm[qb];
                if (!kHalfBlocks) x += swap_half(x);
                x = group_sum<QR>(x);
                bin[qb][b] = x;
            }
        }
        if constexpr (NQB == 64) {             // the wavefront's 64 rows are one query block
#pragma unroll
            for (int b = 0; b < NBK; ++b) bin[0][b] += bin[1][b];
        }
        if ((kHalfBlocks || lh == 0) && (lr % QR) == 0) {
#pragma unroll
            for (int qb = 0; qb < (NQB == 64 ? 1 : QT); ++qb) {
                int t = t0 + 32 * qb + lr;
                if (t < Lq) {
                    int i = t / NQB;
                    float *dst = a.score + ((int64_t)head * a.NQ + row_base + i) * a.NK;
#pragma unroll
                    for (int b = 0; b < NBK; ++b) {
                        int j = kHalfBlocks ? s_lo / 4 + 2 * b + lh : s_lo / NKB + b;
                        if (j < Nb) {
                            if (kTwoTiles && (sub & 1)) dst[j] += bin[qb][b];
                            else dst[j] = bin[qb][b];
                        }
                    }
                }
            }
        }
    };
    // one-sweep form: U(t, j) of one tile.  bin holds each lane's sums over its own keys of every block of the tile;
    // the two lane halves of a row are added with one half swap per pair of blocks (the low half ends with the
    // first block of the pair, the high half with the second).
    auto store_rowsums = [&](const float (&bin)[QT][NBK], int s_lo, int sub) __attribute__((always_inline)) {
#pragma unroll
        for (int qb = 0; qb < QT; ++qb) {
            if constexpr (NBK >= 2) {
#pragma unroll
                for (int b = 0; b < NBK / 2; ++b) {
                    auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(bin[qb][b]),
                                                               __float_as_uint(bin[qb][b + NBK / 2]), false, false);
                    const float x = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
                    const int j = s_lo / NKB + b + lh * (NBK / 2);
                    if (row_ok[qb] && j < Nb) u_at(qb, j) = x;
                }
            } else {
                const float x = bin[qb][0] + swap_half(bin[qb][0]);
                const int j = s_lo / NKB;
                if (row_ok[qb] && lh == 0 && j < Nb) {
                    if (kTwoTiles && (sub & 1)) u_at(qb, j) += x;
                    else u_at(qb, j) = x;
                }
            }
        }
    };
    // one sweep: the exponentials of a tile relative to the row's reference feed both the denominator and U.  The
    // reference is kept equal in the two lane halves of a row (their sums are added before they are stored), so
    // the halves decide together whether it moves.
    auto fused_tile = [&](const f32x16 (&src)[QT], int s_lo, int sub) __attribute__((always_inline)) {
        constexpr float kBig = 1099511627776.0f;           // 2^40
        float bin[QT][NBK], tsum[QT];
        bool need[QT], redo = false;
#pragma unroll
        for (int qb = 0; qb < QT; ++qb) {
#pragma unroll
            for (int b = 0; b < NBK; ++b) bin[qb][b] = 0.0f;
#pragma unroll
            for (int v = 0; v < 16; ++v) bin[qb][(v >> 2) / GPB] += fast_exp2(fmaf(src[qb][v], c2, -mc[qb]));
            tsum[qb] = bin[qb][0];
#pragma unroll
            for (int b = 1; b < NBK; ++b) tsum[qb] += bin[qb][b];
            need[qb] = !(tsum[qb] <= kBig);
            redo = redo || need[qb];
        }
        if (__any(redo)) {
#pragma unroll
            for (int qb = 0; qb < QT; ++qb) {
                const bool nd = need[qb] || __shfl_xor((int)need[qb], 32, 64) != 0;
                float mx = src[qb][0];
#pragma unroll
                for (int v = 1; v < 16; ++v) mx = fmaxf(mx, src[qb][v]);
                mx = fmaxf(mx, swap_half(mx));
                const float m_new = nd ? fmaxf(m_run[qb], mx) : m_run[qb];
                const bool none = m_new == -INFINITY;      // nothing visible to this row yet
                const float m_safe = none ? 0.0f : m_new;
                const float alpha = fast_exp2((m_run[qb] - m_safe) * c2);
                const float msc = m_safe * c2;
                moved = moved || (nd && m_run[qb] != -INFINITY);
#pragma unroll
                for (int b = 0; b < NBK; ++b) bin[qb][b] = 0.0f;
#pragma unroll
                for (int v = 0; v < 16; ++v) bin[qb][(v >> 2) / GPB] += fast_exp2(fmaf(src[qb][v], c2, -msc));
                tsum[qb] = bin[qb][0];
#pragma unroll
                for (int b = 1; b < NBK; ++b) tsum[qb] += bin[qb][b];
                l_run[qb] *= alpha;
                m_run[qb] = m_new;
                mc[qb] = none ? -INFINITY : msc;
            }
        }
#pragma unroll
        for (int qb = 0; qb < QT; ++qb) l_run[qb] += tsum[qb];
        store_rowsums(bin, s_lo, sub);
    };
    // the repeat sweep of the one-sweep form: U again, relative to the final references
    auto rowsums_tile = [&](const f32x16 (&src)[QT], int s_lo, int sub) __attribute__((always_inline)) {
        float bin[QT][NBK];
#pragma unroll
        for (int qb = 0; qb < QT; ++qb) {
#pragma unroll
            for (int b = 0; b < NBK; ++b) bin[qb][b] = 0.0f;
#pragma unroll
            for (int v = 0; v < 16; ++v) bin[qb][(v >> 2) / GPB] += fast_exp2(fmaf(src[qb][v], c2, -mc[qb]));
        }
        store_rowsums(bin, s_lo, sub);
    };
    // Software pipeline over the tiles that every row of the wavefront sees in full: the MFMAs of a tile are
    // issued together with the VALU work of the tile before it (two sets of accumulators), across the stage
    // barriers.  sA holds the tile whose VALU work is still pending.
    f32x16 sA[QT], sB[QT];
    bool pend = false;
    int pend_slo = 0, pend_sub = 0;
    auto valu_tile = [&](const f32x16 (&src)[QT], auto pass_c, int s_lo, int sub) __attribute__((always_inline)) {
        if constexpr (ROWSUMS) {
            if constexpr (decltype(pass_c)::value == 0) fused_tile(src, s_lo, sub);
            else rowsums_tile(src, s_lo, sub);
        } else {
            if constexpr (decltype(pass_c)::value == 0) stats_tile(src);
            else bins_tile(src, s_lo, sub);
        }
    };
    // one MFMA, its share of the VALU work, one operand read per two MFMAs - a hint for the machine scheduler
    constexpr int MIXV = 4;
    auto mix_hint = []() __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < C::kSteps; ++k) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // DS read
#pragma unroll
            for (int qb = 0; qb < QT; ++qb) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // MFMA
                __builtin_amdgcn_sched_group_barrier(0x002, MIXV, 0);   // VALU
            }
        }
    };

    bool repeat = true;
    static_for<2>([&](auto pass_c) __attribute__((always_inline)) {
        constexpr int pass = decltype(pass_c)::value;
        if (ROWSUMS && pass == 1 && !repeat) return;        // (uniform over the workgroup)
        load_stage(0);
        __syncthreads();                                    // previous sweep finished reading LDS
        store_stage(0);
        __syncthreads();
#pragma unroll 1
        for (int st = 0; st < n_stages; ++st) {
            const bool more = st + 1 < n_stages;
            if (more) load_stage(st + 1);
            const unsigned char *kb = lds + (st & 1) * kPxStageBytes;
            if (wave_active) {
                const int s0 = st * kPxStageKeys;
                if (s0 + kPxStageKeys - 1 <= lim_first) {   // all four tiles fully visible to all rows
                    if (!pend) {
                        mfma_tile(sB, kb, 0);
                    } else {
                        mfma_tile(sB, kb, 0);
                        valu_tile(sA, pass_c, pend_slo, pend_sub);
                        mix_hint();
                    }
                    mfma_tile(sA, kb, 1);
                    valu_tile(sB, pass_c, s0, 0);
                    mix_hint();
                    mfma_tile(sB, kb, 2);
                    valu_tile(sA, pass_c, s0 + 32, 1);
                    mix_hint();
                    mfma_tile(sA, kb, 3);
                    valu_tile(sB, pass_c, s0 + 64, 2);
                    mix_hint();
                    pend = true;
                    pend_slo = s0 + 96;
                    pend_sub = 3;
                } else {
                    if (pend) {
                        valu_tile(sA, pass_c, pend_slo, pend_sub);
                        pend = false;
                    }
#pragma unroll 1
                    for (int sub = 0; sub < 4; ++sub) {
                        const int s_lo = s0 + 32 * sub;
                        if (s_lo > lim_last) break;
                        const bool partial = s_lo + 31 > lim_first;
                        f32x16 sacc[QT];
                        mfma_tile(sacc, kb, sub);
                        if (partial) {
#pragma unroll
                            for (int qb = 0; qb < QT; ++qb)
#pragma unroll
                                for (int v = 0; v < 16; ++v) {
                                    int key = s_lo + 8 * (v >> 2) + 4 * lh + (v & 3);
                                    sacc[qb][v] = key <= lim_row[qb] ? sacc[qb][v] : -INFINITY;
                                }
                        }
                        valu_tile(sacc, pass_c, s_lo, sub);
                    }
                }
            }
            if (more) store_stage((st + 1) & 1);
            __syncthreads();
        }
        if (pend) {                                         // (not reached under causality: the last stage is partial)
            valu_tile(sA, pass_c, pend_slo, pend_sub);
            pend = false;
        }
        if constexpr (pass == 0) {
#pragma unroll
            for (int qb = 0; qb < QT; ++qb) {
                float m_o = swap_half(m_run[qb]), l_o = swap_half(l_run[qb]);
                float m_t = fmaxf(m_run[qb], m_o);          // finite: every row sees at least key 0
                float l_t = l_run[qb] * fast_exp2((m_run[qb] - m_t) * c2) + l_o * fast_exp2((m_o - m_t) * c2);
                l_t = __shfl(l_t, lr, 64);                  // both halves use half 0's rounding of the sum
                mc[qb] = m_t * c2;
                // rows beyond the sequence (clamped copies of its last row) must not count in a partial query block
                wnorm[qb] = t0 + 32 * qb + lr < Lq ? 1.0f / l_t : 0.0f;
                if constexpr (ROWSUMS) {        // [head][query block][row]
                    const int t = t0 + 32 * qb + lr;
                    if (wave_active && lh == 0 && row_ok[qb])
                        a.w[((int64_t)head * a.NQ + row_base + t / NQB) * NQB + t % NQB] = wnorm[qb];
                }
            }
            if constexpr (ROWSUMS) repeat = __syncthreads_or(moved ? 1 : 0) != 0;
        }
    });
}

template <int D, int NQB, int NKB, int QT, bool ROWSUMS>
static hipError_t proxy_launch_t(const ProxyArgs &a, const ProxyGeom &g, dim3 grid, hipStream_t stream)
{
    const int lds_bytes = 2 * PxCfg<D>::kStageBytes;
    hipError_t e;
    if (a.causal) {
        static LdsAttr attr;
        e = attr.set(reinterpret_cast<const void *>(&proxy_kernel<D, NQB, NKB, true, QT, ROWSUMS>), lds_bytes);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((proxy_kernel<D, NQB, NKB, true, QT, ROWSUMS>), grid, dim3(kPxThreads), lds_bytes, stream, a, g);
    } else {
        static LdsAttr attr;
        e = attr.set(reinterpret_cast<const void *>(&proxy_kernel<D, NQB, NKB, false, QT, ROWSUMS>), lds_bytes);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((proxy_kernel<D, NQB, NKB, false, QT, ROWSUMS>), grid, dim3(kPxThreads), lds_bytes, stream, a, g);
    }
    return hipGetLastError();
}

// The one-tile-per-wavefront variants exist where small grids occur in practice: head dimension 128 and query
// blocks of at most 32 composite tokens (high compression ratios).
constexpr bool proxy_has_single_tile(int head_dim, int nqb) { return head_dim == 128 && nqb <= 32; }

// All granularities of one head dimension and one form; each pair is compiled in a translation unit of its own.
template <int D, bool ROWSUMS>
static hipError_t proxy_dispatch_t(const ProxyArgs &a, const ProxyGeom &g, dim3 grid, hipStream_t stream)
{
    const int nq = a.S / a.c_q, nk = a.S / a.c_k;
#define US_PX(NQB, NKB)                                                                               \
    if constexpr (!ROWSUMS || NKB >= 8) {                                                             \
        if (nq == NQB && nk == NKB) {                                                                 \
            if constexpr (proxy_has_single_tile(D, NQB))                                              \
                if (g.QT == 1) return proxy_launch_t<D, NQB, NKB, 1, ROWSUMS>(a, g, grid, stream);    \
            return proxy_launch_t<D, NQB, NKB, 2, ROWSUMS>(a, g, grid, stream);                       \
        }                                                                                             \
    }
    US_PX(4, 4); US_PX(4, 8); US_PX(4, 16); US_PX(4, 32); US_PX(4, 64);
    US_PX(8, 4); US_PX(8, 8); US_PX(8, 16); US_PX(8, 32); US_PX(8, 64);
    US_PX(16, 4); US_PX(16, 8); US_PX(16, 16); US_PX(16, 32); US_PX(16, 64);
    US_PX(32, 4); US_PX(32, 8); US_PX(32, 16); US_PX(32, 32); US_PX(32, 64);
    US_PX(64, 4); US_PX(64, 8); US_PX(64, 16); US_PX(64, 32); US_PX(64, 64);
#undef US_PX
    return hipErrorInvalidValue;
}

// two-sweep form (Score written by the kernel) and one-sweep form (U and the row weights written) per head dimension
hipError_t proxy_dispatch_d64(const ProxyArgs &a, const ProxyGeom &g, dim3 grid, hipStream_t stream);
hipError_t proxy_dispatch_d128(const ProxyArgs &a, const ProxyGeom &g, dim3 grid, hipStream_t stream);
hipError_t proxy_dispatch_d256(const ProxyArgs &a, const ProxyGeom &g, dim3 grid, hipStream_t stream);
hipError_t proxy_rowsums_dispatch_d64(const ProxyArgs &a, const ProxyGeom &g, dim3 grid, hipStream_t stream);
hipError_t proxy_rowsums_dispatch_d128(const ProxyArgs &a, const ProxyGeom &g, dim3 grid, hipStream_t stream);
hipError_t proxy_rowsums_dispatch_d256(const ProxyArgs &a, const ProxyGeom &g, dim3 grid, hipStream_t stream);

}  // namespace us

// Block selection, Alg. 1 step 4: causal cut, then Top-P (Eq. (5)) or a fixed budget per row.
//
// The rule: order the row's valid scores (j <= i when causal) descending, equal scores by ascending j; Top-P keeps
// the shortest prefix whose sum reaches P times the row's total (an element is kept iff it is the first or the sum
// before it is still below the target), the budget mode keeps the first k.  No sort is needed to apply it:
//
//   * every score above a threshold value tau is kept, every score below it is dropped, and tau is the smallest
//     score whose strictly-larger scores sum to less than the target (Top-P) or number fewer than k (budget);
//     that sum / count is monotone in the threshold, so tau is found by bisection on the 32 bits of the float;
//   * of the scores equal to tau the first m in index order are kept, m found by adding tau to the running sum
//     until the target is reached (Top-P) or m = k - (number above tau).
//
// One wavefront owns one (compressed head, query-block row): lane l holds scores l, l + 64, l + 128, ... in
// registers, so the mask word w of the row is exactly the 64-lane ballot of "element w of my registers is kept".
// Sums are fp64, as in the definition.  The kept columns are written once per head of the broadcast group.
//
// The scores are either given, or (FROM_ROWSUMS) formed here from what the one-sweep score kernel left: Eq. (3) as
// Score(i, j) = sum over the composite query rows t of block i of weight_t U(t, j), in ascending t, and stored.
#include "common.h"

namespace us {

constexpr int kSelThreads = 256;
constexpr int kSelRows = kSelThreads / 64;               // rows per workgroup

// Wavefront sums without LDS traffic: lane permutations inside rows of 16 lanes (DPP), then the row and half swaps of
// gfx950.  Every step adds a value and its partner's, so all lanes end with the same bits.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_mov(uint32_t x)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xf, 0xf, true);
}
__device__ __forceinline__ double make_f64(uint32_t lo, uint32_t hi)
{
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}
template <int CTRL>
__device__ __forceinline__ double dpp_add(double x)
{
    const uint64_t b = (uint64_t)__double_as_longlong(x);
    return x + make_f64(dpp_mov<CTRL>((uint32_t)b), dpp_mov<CTRL>((uint32_t)(b >> 32)));
}
__device__ __forceinline__ double wave_sum(double x)
{
    x = dpp_add<0xB1>(x);                                 // quad_perm [1, 0, 3, 2]
    x = dpp_add<0x4E>(x);                                 // quad_perm [2, 3, 0, 1]
    x = dpp_add<0x141>(x);                                // row_half_mirror
    x = dpp_add<0x140>(x);                                // row_mirror: every lane holds the sum of its row of 16
    uint64_t b = (uint64_t)__double_as_longlong(x);
    auto l16 = __builtin_amdgcn_permlane16_swap((uint32_t)b, (uint32_t)b, false, false);
    auto h16 = __builtin_amdgcn_permlane16_swap((uint32_t)(b >> 32), (uint32_t)(b >> 32), false, false);
    x = make_f64(l16[0], h16[0]) + make_f64(l16[1], h16[1]);
    b = (uint64_t)__double_as_longlong(x);
    auto l32 = __builtin_amdgcn_permlane32_swap((uint32_t)b, (uint32_t)b, false, false);
    auto h32 = __builtin_amdgcn_permlane32_swap((uint32_t)(b >> 32), (uint32_t)(b >> 32), false, false);
    return make_f64(l32[0], h32[0]) + make_f64(l32[1], h32[1]);
}
__device__ __forceinline__ int wave_sum(int x)
{
    x += (int)dpp_mov<0xB1>((uint32_t)x);
    x += (int)dpp_mov<0x4E>((uint32_t)x);
    x += (int)dpp_mov<0x141>((uint32_t)x);
    x += (int)dpp_mov<0x140>((uint32_t)x);
    auto s16 = __builtin_amdgcn_permlane16_swap((uint32_t)x, (uint32_t)x, false, false);
    x = (int)(s16[0] + s16[1]);
    auto s32 = __builtin_amdgcn_permlane32_swap((uint32_t)x, (uint32_t)x, false, false);
    return (int)(s32[0] + s32[1]);
}

// E = register elements per lane: rows of up to 64 E valid blocks.
template <int E, bool FROM_ROWSUMS>
__global__ __launch_bounds__(kSelThreads) void select_kernel(SelectArgs a)
{
    const int lane = threadIdx.x & 63;
    const int64_t rid = (int64_t)blockIdx.x * kSelRows + (threadIdx.x >> 6);
    if (rid >= (int64_t)a.n_heads_c * a.NQ) return;       // whole wavefront
    const int row = (int)(rid % a.NQ);
    const int hc = (int)(rid / a.NQ);
    int seq, i, nb;
    locate_row(a.st, a.S, row, seq, i, nb);
    const int nv = a.causal ? i + 1 : nb;
    const int ne = (nv + 63) >> 6;                        // register elements in use (uniform), <= E

    float *srow = a.score + ((int64_t)hc * a.NQ + row) * a.NK;
    float agg[FROM_ROWSUMS ? E : 1];
    if constexpr (FROM_ROWSUMS) {
        // the block's n_q composite query rows in groups of four: per group and 64 key blocks, 1 KB in lane order
        const int nq4 = a.S / a.c_q / 4;
        const float *ur = a.u + ((int64_t)hc * a.NQ + row) * ((a.NK + 63) / 64) * (nq4 * 256) + lane * 4;
        const float *wr = a.w + ((int64_t)hc * a.NQ + row) * (nq4 * 4);
#pragma unroll
        for (int e = 0; e < E; ++e) agg[e] = 0.0f;
#pragma unroll 2
        for (int c = 0; c < nq4; ++c) {
            const f32x4 w4 = *reinterpret_cast<const f32x4 *>(wr + 4 * c);
#pragma unroll
            for (int e = 0; e < E; ++e) {
                if (e < ne && lane + 64 * e < nv) {
                    const f32x4 u4 = *reinterpret_cast<const f32x4 *>(ur + (e * nq4 + c) * 256);
                    agg[e] = fmaf(w4[3], u4[3], fmaf(w4[2], u4[2], fmaf(w4[1], u4[1], fmaf(w4[0], u4[0], agg[e]))));
                }
            }
        }
    }
    uint32_t sb[E];                                       // score bits (non-negative floats order like integers)
    double sd[E];
    double local = 0.0;
    uint32_t mx = 0;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        sb[e] = 0;
        sd[e] = 0.0;
        if (e < ne) {
            const int idx = lane + 64 * e;
            float s;
            if constexpr (FROM_ROWSUMS) {
                s = idx < nv ? agg[e] : 0.0f;
                if (idx < nv) srow[idx] = s;
            } else {
                s = idx < nv ? srow[idx] : 0.0f;
            }
            s = s > 0.0f ? s : 0.0f;
            sb[e] = __float_as_uint(s);
            sd[e] = (double)s;
            local += sd[e];
            mx = sb[e] > mx ? sb[e] : mx;
        }
    }
    for (int idx = nv + lane; idx < a.NK; idx += 64) srow[idx] = 0.0f;   // outside the valid set
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)mx, off, 64);
        mx = o > mx ? o : mx;
    }
    const double tot = wave_sum(local);

    const bool top_p = a.mode == UNISPARSE_TOP_P;
    const bool all = top_p && a.param >= 1.0;
    const double target = a.param * tot;
    int kbudget = nv;
    if (!top_p) {
        const double kk = ceil(a.param * (double)nv);
        kbudget = kk < 1.0 ? 1 : (kk > (double)nv ? nv : (int)kk);
    }

    // sum (Top-P) or number (budget) of the scores strictly above threshold bits t; padding holds zeros, never above
    auto above = [&](uint32_t t, bool want_sum, bool want_cnt, double &sum, int &cnt) __attribute__((always_inline)) {
        double s = 0.0;
        int c = 0;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            if (e < ne) {
                const bool gt = sb[e] > t;
                s += gt ? sd[e] : 0.0;
                c += gt ? 1 : 0;
            }
        }
        if (want_sum) sum = wave_sum(s);
        if (want_cnt) cnt = wave_sum(c);
    };
    auto below_cut = [&](double sum, int cnt) __attribute__((always_inline)) -> bool {
        return top_p ? sum < target : cnt < kbudget;
    };

    // tau = smallest threshold t in [0, mx] with below_cut(above(t)); t = mx always qualifies in budget mode
    // (nothing is above the maximum) and in Top-P mode unless the target is 0 (an all-zero row), where tau = mx.
    uint32_t lo = 0, hi = mx;                             // invariant: the answer lies in [lo, hi]
    double s_hi = 0.0;
    int c_hi = 0;
#pragma unroll 1
    while (lo < hi) {
        const uint32_t mid = lo + ((hi - lo) >> 1);
        double s = 0.0;
        int c = 0;
        above(mid, top_p, !top_p, s, c);
        if (below_cut(s, c)) hi = mid;
        else lo = mid + 1;
    }
    uint32_t tau = __builtin_amdgcn_readfirstlane(hi);
    // tau is one of the row's values unless the row is all zero: snap it to the smallest score >= tau
    {
        uint32_t best = mx;
#pragma unroll
        for (int e = 0; e < E; ++e)
            if (e < ne && lane + 64 * e < nv && sb[e] >= tau && sb[e] < best) best = sb[e];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const uint32_t o = (uint32_t)__shfl_xor((int)best, off, 64);
            best = o < best ? o : best;
        }
        tau = best;
    }
    above(tau, true, true, s_hi, c_hi);

    // how many of the scores equal to tau are kept, in index order
    int ties = 0;
#pragma unroll
    for (int e = 0; e < E; ++e)
        if (e < ne && lane + 64 * e < nv && sb[e] == tau) ++ties;
    ties = wave_sum(ties);
    int keep;
    if (all) {
        keep = ties;
    } else if (top_p) {
        const double tv = (double)__uint_as_float(tau);
        double run = s_hi;
        keep = 0;
        while (keep < ties && run < target) {             // the same additions, in the same order, as the definition
            ++keep;
            run += tv;
        }
        if (keep == 0 && c_hi == 0) keep = 1;             // the first element of the order is always kept
    } else {
        keep = kbudget - c_hi;
        keep = keep > ties ? ties : keep;
    }

    int seen = 0;                                         // ties before this register element, in index order
    const uint64_t lt_mask = (1ull << lane) - 1ull;      // the lanes before this one
#pragma unroll
    for (int e = 0; e < E; ++e) {
        if (e < ne) {
            const bool valid = lane + 64 * e < nv;
            const bool is_tie = valid && sb[e] == tau;
            const uint64_t tie_mask = __ballot(is_tie);
            const int rank = seen + __builtin_popcountll(tie_mask & lt_mask);
            const bool sel = valid && (all || sb[e] > tau || (is_tie && rank < keep));
            const uint64_t word = __ballot(sel);
            seen += __builtin_popcountll(tie_mask);
            for (int m = lane; m < a.c_h; m += 64)        // one lane per head of the broadcast group
                a.mask[((int64_t)(hc * a.c_h + m) * a.NQ + row) * a.W + e] = word;
        }
    }
    for (int x = lane; x < (a.W - ne) * a.c_h; x += 64)   // words beyond the valid set
        a.mask[((int64_t)(hc * a.c_h + x % a.c_h) * a.NQ + row) * a.W + ne + x / a.c_h] = 0ull;
}

hipError_t launch_select(const SelectArgs &a, hipStream_t stream)
{
    const int64_t n = (int64_t)a.n_heads_c * a.NQ;
    if (n == 0) return hipSuccess;
    if (a.NK > UNISPARSE_MAX_BLOCKS_PER_SEQ) return hipErrorInvalidValue;
    if (a.u != nullptr && (a.w == nullptr || a.c_q < 1 || a.S % a.c_q != 0 || (a.S / a.c_q) % 4 != 0)) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((n + kSelRows - 1) / kSelRows)), block(kSelThreads);
    const int ne = (a.NK + 63) / 64;
#define US_SEL(EE)                                                                               \
    if (ne <= EE) {                                                                              \
        if (a.u != nullptr) hipLaunchKernelGGL((select_kernel<EE, true>), grid, block, 0, stream, a);  \
        else hipLaunchKernelGGL((select_kernel<EE, false>), grid, block, 0, stream, a);          \
        return hipGetLastError();                                                                \
    }
    US_SEL(1) US_SEL(2) US_SEL(4) US_SEL(8) US_SEL(16) US_SEL(32) US_SEL(64)
#undef US_SEL
    return hipErrorInvalidValue;
}

}  // namespace us

// Block-sparse attention (Alg. 1 step 5, Sec. 2.2) and the dense baseline (Sec. 2.1) for the head dimensions the
// software-pipelined kernel of attention.hip is not written for (64 and 256).
//
// Same decomposition and the same MFMA operand layouts as that kernel, without its pipelining: a workgroup owns one
// (query head, query block of S rows), one wavefront per 32 query rows, and visits the key blocks its mask row
// selects (every valid block when dense).  Per block: all wavefronts copy the K and V block into LDS (rows padded by
// 16 bytes), barrier, then each wavefront walks the block in tiles of 32 keys:
//   S^T (32 keys x 32 queries) = K Q^T   : A = K rows from LDS, B = Q^T kept in registers
//   online softmax, lane-local per query column (one exchange with lane ^ 32)
//   O^T (d x 32 queries) += V^T P^T      : A = V^T through the LDS transpose read, B = P^T = the S^T accumulators
// A shorter last block of a sequence is handled by clamping row indices when loading and masking its missing keys.
#include "common.h"

namespace us {

template <int D, int S>
struct GenCfg {
    static constexpr int NW = S / 32;              // wavefronts = 32-row query slices
    static constexpr int NT = NW * 64;
    static constexpr int kSteps = D / 16;          // MFMA steps over the head dimension (Q K^T)
    static constexpr int kDimBlocks = D / 32;      // 32-dim output blocks (P V)
    static constexpr int kPitch = 2 * D + 16;      // bytes per LDS row
    static constexpr int kTileBytes = S * kPitch;  // one K or V block
    static constexpr int kLdsBytes = 2 * kTileBytes;
    static constexpr int kLoads = S * (D / 8) / NT;   // 16-byte loads per thread per K (or V) block
};

template <int D, int S, bool CAUSAL, bool DENSE>
__global__ __launch_bounds__((GenCfg<D, S>::NT)) void attention_generic_kernel(AttnArgs a)
{
    using C = GenCfg<D, S>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    typedef short4v __attribute__((address_space(3))) * lds_s4_ptr;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lr = lane & 31, lh = lane >> 5, i16 = lane & 15;

    // Workgroup ids are dealt round-robin to the 8 XCDs: the heads of one row (which share K/V per key head) go to
    // one XCD and its L2, rows go round the XCDs, longest rows first.
    const int xcd = (int)blockIdx.x % kNumXcd, idx = (int)blockIdx.x / kNumXcd;
    const int row = a.NQ - 1 - ((idx / a.n_heads_q) * kNumXcd + xcd);
    if (row < 0) return;
    const int head = idx % a.n_heads_q;
    const int kvh = head / (a.n_heads_q / a.n_heads_kv);
    int seq, i, nb;
    locate_row(a.st, S, row, seq, i, nb);
    const int64_t tok0 = a.st.cu_tok[seq];
    const int Lb = a.st.cu_tok[seq + 1] - a.st.cu_tok[seq];
    const int q_rows = min(S, Lb - i * S);                  // query rows of this block that exist (>= 1)
    const int nvalid = CAUSAL ? i + 1 : nb;
    const float c2 = a.scale_log2;

    // ---- Q^T as B operands: lane = query row 32 wave + lr (clamped to the sequence), 8 dims per MFMA step ----
    bf16x8 bq[C::kSteps];
    {
        const int r = min(32 * wave + lr, q_rows - 1);
        const bf16_t *src = a.q.ptr + (int64_t)head * a.q.stride_head + (tok0 + (int64_t)i * S + r) * a.q.stride_tok + 8 * lh;
#pragma unroll
        for (int ks = 0; ks < C::kSteps; ++ks) bq[ks] = *reinterpret_cast<const bf16x8 *>(src + 16 * ks);
    }

    f32x16 oacc[C::kDimBlocks];
#pragma unroll
    for (int db = 0; db < C::kDimBlocks; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[db][v] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;

    unsigned char *ldsK = lds, *ldsV = lds + C::kTileBytes;
    const bf16_t *kbase = a.k.ptr + (int64_t)kvh * a.k.stride_head + tok0 * a.k.stride_tok;
    const bf16_t *vbase = a.v.ptr + (int64_t)kvh * a.v.stride_head + tok0 * a.v.stride_tok;

    auto visit = [&](int j) __attribute__((always_inline)) {
        // ---- K and V block j into LDS --------------------------------------------------------------------
        __syncthreads();                                    // the previous block has been read
        const int last = Lb - 1 - j * S;                    // last existing row of this block (>= 0)
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            u32x4 pre[C::kLoads];
            const bf16_t *base = half == 0 ? kbase : vbase;
            const int64_t st = half == 0 ? a.k.stride_tok : a.v.stride_tok;
#pragma unroll
            for (int it = 0; it < C::kLoads; ++it) {
                const int id = it * C::NT + tid;
                const int r = min(id / (D / 8), last);
                pre[it] = *reinterpret_cast<const u32x4 *>(base + ((int64_t)j * S + r) * st + (id % (D / 8)) * 8);
            }
            unsigned char *dst = half == 0 ? ldsK : ldsV;
#pragma unroll
            for (int it = 0; it < C::kLoads; ++it) {
                const int id = it * C::NT + tid;
                *reinterpret_cast<u32x4 *>(dst + (id / (D / 8)) * C::kPitch + (id % (D / 8)) * 16) = pre[it];
            }
        }
        __syncthreads();

        // ---- tiles of 32 keys ------------------------------------------------------------------------------
#pragma unroll 1
        for (int t = 0; t < S / 32; ++t) {
            const int key0 = j * S + 32 * t;                // first key of the tile, within the sequence
            if (key0 >= Lb) break;                          // beyond the shorter last block
            if (CAUSAL && j == i && t > wave) break;        // beyond every query row of this wavefront
            f32x16 sacc;
#pragma unroll
            for (int v = 0; v < 16; ++v) sacc[v] = 0.0f;
            const unsigned char *arow = ldsK + (32 * t + lr) * C::kPitch + 16 * lh;
#pragma unroll
            for (int ks = 0; ks < C::kSteps; ++ks) {
                bf16x8 ka = *reinterpret_cast<const bf16x8 *>(arow + 32 * ks);
                sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, bq[ks], sacc, 0, 0, 0);
            }
            // register v of a lane holds key 8 (v / 4) + 4 lh + v % 4 of the tile, for query column lr
            if ((CAUSAL && j == i && t == wave) || key0 + 32 > Lb) {
                const int qpos = i * S + 32 * wave + lr;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = key0 + 8 * (v >> 2) + 4 * lh + (v & 3);
                    const bool ok = key < Lb && (!CAUSAL || key <= qpos);
                    sacc[v] = ok ? sacc[v] : -INFINITY;
                }
            }
            float mx = sacc[0];
#pragma unroll
            for (int v = 1; v < 16; ++v) mx = fmaxf(mx, sacc[v]);
            mx = fmaxf(mx, swap_half(mx));
            // lazy reference: it moves only when the tile's maximum exceeds it by more than 2^8 in the exponent, so
            // probabilities stay <= 256 and the rescaling of O^T below is rare
            const float m_new = mx > m_run + 8.0f / c2 ? mx : m_run;
            const float m_safe = m_new == -INFINITY ? 0.0f : m_new;
            const float alpha = fast_exp2((m_run - m_safe) * c2);
            const float msc = m_safe * c2;
            float p[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) p[v] = fast_exp2(fmaf(sacc[v], c2, -msc));
            m_run = m_new;
            if (__any(alpha != 1.0f)) {
#pragma unroll
                for (int db = 0; db < C::kDimBlocks; ++db)
#pragma unroll
                    for (int v = 0; v < 16; ++v) oacc[db][v] *= alpha;
            }
            // P^T as B operands: 16-key group g takes registers 8 g .. 8 g + 7 (keys 4 lh + 0..3 and 8 + 4 lh + 0..3
            // of the group); the V^T operand below supplies the same keys in the same slots
            // The row sum is taken over the rounded probabilities, the values the product below multiplies, so that the
            // rounding cancels between numerator and denominator.
            bf16x8 pb[2];
            float sum = 0.0f;
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                u32x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    w[e] = f32_to_bf16_rne(p[8 * g + 2 * e]) | (f32_to_bf16_rne(p[8 * g + 2 * e + 1]) << 16);
                    sum += __uint_as_float(w[e] << 16);
                    sum += __uint_as_float(w[e] & 0xffff0000u);
                }
                pb[g] = __builtin_bit_cast(bf16x8, w);
            }
            l_run = l_run * alpha + sum;
#pragma unroll
            for (int db = 0; db < C::kDimBlocks; ++db) {
#pragma unroll
                for (int g = 0; g < 2; ++g) {
                    // transpose read: the lane ends up with dims 32 db + lr, keys 4 lh + 0..3 (x0) and 8 + 4 lh + 0..3 (x1)
                    const unsigned char *p0 = ldsV + (32 * t + 16 * g + 4 * lh + (i16 >> 2)) * C::kPitch + 64 * db +
                                              32 * (lr >> 4) + 8 * (i16 & 3);
                    short4v x0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_ptr)p0);
                    short4v x1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_ptr)(p0 + 8 * C::kPitch));
                    bf16x8 va = __builtin_bit_cast(bf16x8, __builtin_shufflevector(x0, x1, 0, 1, 2, 3, 4, 5, 6, 7));
                    oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[g], oacc[db], 0, 0, 0);
                }
            }
        }
    };

    if (DENSE) {
#pragma unroll 1
        for (int j = 0; j < nvalid; ++j) visit(j);
    } else {
        const uint64_t *mrow = a.mask + ((int64_t)head * a.NQ + row) * a.W;
        const int nw = (nvalid + 63) / 64;
#pragma unroll 1
        for (int wd = 0; wd < nw; ++wd) {
            uint64_t bits = mrow[wd];                       // the same word in every lane
            const int hi = nvalid - wd * 64;
            if (hi < 64) bits &= (1ull << hi) - 1ull;       // bits of invalid blocks are ignored
            const uint32_t lo32 = __builtin_amdgcn_readfirstlane((uint32_t)bits);
            const uint32_t hi32 = __builtin_amdgcn_readfirstlane((uint32_t)(bits >> 32));
            bits = ((uint64_t)hi32 << 32) | lo32;
#pragma unroll 1
            while (bits != 0) {
                visit(wd * 64 + __builtin_ctzll(bits));
                bits &= bits - 1;
            }
        }
    }

    // ---- normalise and store ------------------------------------------------------------------------------
    const float l_t = l_run + swap_half(l_run);
    const bool empty = m_run == -INFINITY;                  // no block visited (caller-made empty mask row)
    const float inv = empty ? 0.0f : 1.0f / l_t;
    const bool row_exists = 32 * wave + lr < q_rows;
    const int64_t tok = tok0 + (int64_t)i * S + 32 * wave + lr;
    bf16_t *dst = a.o + tok * a.o_stride_tok + (int64_t)head * a.o_stride_head;
#pragma unroll
    for (int db = 0; db < C::kDimBlocks; ++db) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            u32x2 w;
            w[0] = f32_to_bf16_rne(oacc[db][4 * g] * inv) | (f32_to_bf16_rne(oacc[db][4 * g + 1] * inv) << 16);
            w[1] = f32_to_bf16_rne(oacc[db][4 * g + 2] * inv) | (f32_to_bf16_rne(oacc[db][4 * g + 3] * inv) << 16);
            if (row_exists) *reinterpret_cast<u32x2 *>(dst + 32 * db + 8 * g + 4 * lh) = w;
        }
    }
    if (a.lse != nullptr && lh == 0 && row_exists)
        a.lse[(int64_t)head * a.total_tokens + tok] = empty ? -INFINITY : (__log2f(l_t) + m_run * c2) * kLn2;
}

template <int D, int S, bool CAUSAL, bool DENSE>
static hipError_t gen_launch_t(const AttnArgs &a, hipStream_t stream)
{
    using C = GenCfg<D, S>;
    static LdsAttr attr;
    hipError_t e = attr.set(reinterpret_cast<const void *>(&attention_generic_kernel<D, S, CAUSAL, DENSE>), C::kLdsBytes);
    if (e != hipSuccess) return e;
    if (a.n_heads_q == 0 || a.NQ == 0) return hipSuccess;
    const int64_t nblk = (int64_t)a.n_heads_q * ((a.NQ + kNumXcd - 1) / kNumXcd) * kNumXcd;
    hipLaunchKernelGGL((attention_generic_kernel<D, S, CAUSAL, DENSE>), dim3((unsigned)nblk), dim3(C::NT), C::kLdsBytes,
                       stream, a);
    return hipGetLastError();
}

hipError_t launch_attention_generic(const AttnArgs &a, hipStream_t stream)
{
    const bool dense = a.mask == nullptr;
#define US_GA(DD, SS, CA, DE) \
    if (a.head_dim == DD && a.S == SS && (a.causal != 0) == CA && dense == DE) return gen_launch_t<DD, SS, CA, DE>(a, stream)
#define US_GA4(DD, SS) \
    US_GA(DD, SS, true, true); US_GA(DD, SS, true, false); US_GA(DD, SS, false, true); US_GA(DD, SS, false, false)
    US_GA4(64, 128); US_GA4(64, 64); US_GA4(256, 128); US_GA4(256, 64);
#undef US_GA4
#undef US_GA
    return hipErrorInvalidValue;
}

}  // namespace us

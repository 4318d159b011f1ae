// Block-sparse attention (Alg. 1 step 5, Sec. 2.2) and the dense baseline (Sec. 2.1), one kernel.
//
// A workgroup owns one (query head, query block of S rows) and visits the key blocks its mask row
// selects (or every valid block when dense).  K and V blocks are staged through LDS, double
// buffered, with the next block's global loads in flight during the current block's math.
//
// Wavefront tiling (S = 128: four wavefronts): wavefront (qh, kh) owns query rows [64 qh, 64 qh + 64)
// and key rows [64 kh, 64 kh + 64) of every visited block, with its own running max / sum / output;
// the two key halves are merged through LDS once, after the last block.  Splitting keys instead of
// giving every wavefront 32 rows x all keys halves the LDS read traffic per MFMA.
//
// All matrix products are computed transposed so that a lane owns whole query rows:
//   S^T (keys x queries)  = K Q^T   : A = K rows from LDS (16-byte reads), B = Q^T kept in registers
//   O^T (dims x queries) += V^T P^T : A = V^T via the LDS transpose read of row-major V,
//                                     B = P^T, which is exactly the accumulator layout of S^T
// With v_mfma_f32_32x32x16_bf16 a lane holds column (query) lane % 32 of the accumulator, so row max,
// row sum and the rescale of O^T are lane-local; only one exchange with lane ^ 32 is needed.
#include "common.h"

namespace us {

constexpr int kKPitch = 272;     // bytes per K row in LDS (256 + 16: conflict-free 16-byte row reads)
constexpr int kVPitch = 320;     // bytes per V row in LDS (256 + 64: conflict-free transpose reads)

template <int S>
struct AttnCfg {
    static constexpr int QW = S / 64;            // query halves
    static constexpr int KW = 2;                 // key halves
    static constexpr int NW = QW * KW;
    static constexpr int NT = NW * 64;
    static constexpr int KC = S / KW;            // keys per wavefront per block
    static constexpr int KB = KC / 32;           // 32-key MFMA tiles per wavefront per block
    static constexpr int kStageBytes = S * (kKPitch + kVPitch);
    static constexpr int kLdsBytes = 2 * kStageBytes;
    static constexpr int kChunks = S * 16 / NT;  // 16-byte chunks per thread per tile (= 8)
};

template <int S, bool CAUSAL, bool DENSE>
__global__ __launch_bounds__(AttnCfg<S>::NT) void attention_kernel(AttnArgs a)
{
    using C = AttnCfg<S>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    __shared__ uint64_t mwords[UNISPARSE_MAX_BLOCKS_PER_SEQ / 64];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int lr = lane & 31, lh = lane >> 5;
    const int qh = wave % C::QW, kh = wave / C::QW;

    // ---- which (head, query-block row): one key head per XCD slice, longest rows first ------------
    const int G = a.n_heads_q / a.n_heads_kv;
    const int vid = xcd_contiguous_id(blockIdx.x, gridDim.x);
    const int kvh = vid / (a.NQ * G);
    const int rem = vid % (a.NQ * G);
    const int row = a.NQ - 1 - rem / G;
    const int head = kvh * G + rem % G;
    int seq, i, nb;
    locate_row(a.st, S, row, seq, i, nb);
    const int64_t tok0 = a.st.cu_tok[seq];
    const int nvalid = CAUSAL ? i + 1 : nb;

    if (!DENSE) {
        const int nw = (nvalid + 63) / 64;
        for (int w = tid; w < nw; w += C::NT) {
            uint64_t bits = a.mask[((int64_t)head * a.NQ + row) * a.W + w];
            int hi = nvalid - w * 64;
            if (hi < 64) bits &= (1ull << hi) - 1ull;
            mwords[w] = bits;
        }
        __syncthreads();
    }
    int widx = -1;
    uint64_t wbits = 0;
    int jdense = 0;
    auto next_block = [&]() -> int {
        if (DENSE) {
            int j = jdense < nvalid ? jdense : -1;
            ++jdense;
            return j;
        } else {
            const int nw = (nvalid + 63) / 64;
            while (wbits == 0) {
                if (++widx >= nw) return -1;
                wbits = mwords[widx];
            }
            int j = widx * 64 + __builtin_ctzll(wbits);
            wbits &= wbits - 1;
            return __builtin_amdgcn_readfirstlane(j);
        }
    };

    // ---- this wavefront's 64 query rows as B operands ---------------------------------------------
    bf16x8 qreg[2][8];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const bf16_t *src = a.q.ptr + (tok0 + (int64_t)i * S + 64 * qh + 32 * qb + lr) * a.q.stride_tok +
                            (int64_t)head * a.q.stride_head + 8 * lh;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qreg[qb][ks] = *reinterpret_cast<const bf16x8 *>(src + 16 * ks);
    }

    const bf16_t *kptr = a.k.ptr + (int64_t)kvh * a.k.stride_head + tok0 * a.k.stride_tok;
    const bf16_t *vptr = a.v.ptr + (int64_t)kvh * a.v.stride_head + tok0 * a.v.stride_tok;
    u32x4 preK[C::kChunks], preV[C::kChunks];
    auto load_tile = [&](int j) {
#pragma unroll
        for (int it = 0; it < C::kChunks; ++it) {
            int id = it * C::NT + tid;
            int64_t r = (int64_t)j * S + (id >> 4);
            preK[it] = *reinterpret_cast<const u32x4 *>(kptr + r * a.k.stride_tok + (id & 15) * 8);
            preV[it] = *reinterpret_cast<const u32x4 *>(vptr + r * a.v.stride_tok + (id & 15) * 8);
        }
    };
    auto store_tile = [&](int buf) {
        unsigned char *kb = lds + buf * C::kStageBytes;
        unsigned char *vb = kb + S * kKPitch;
#pragma unroll
        for (int it = 0; it < C::kChunks; ++it) {
            int id = it * C::NT + tid;
            *reinterpret_cast<u32x4 *>(kb + (id >> 4) * kKPitch + (id & 15) * 16) = preK[it];
            *reinterpret_cast<u32x4 *>(vb + (id >> 4) * kVPitch + (id & 15) * 16) = preV[it];
        }
    };

    f32x16 oacc[4][2];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int v = 0; v < 16; ++v) oacc[db][qb][v] = 0.0f;
    float m_run[2] = {-INFINITY, -INFINITY};
    float l_run[2] = {0.0f, 0.0f};
    const float c2 = a.scale_log2;

    int j = next_block();
    if (j >= 0) {
        load_tile(j);
        store_tile(0);
    }
    __syncthreads();
    int buf = 0;
#pragma unroll 1
    while (j >= 0) {
        const int jn = next_block();
        if (jn >= 0) load_tile(jn);

        const bool diag = CAUSAL && (j == i);
        const bool wave_skip = diag && (C::KC * kh > 64 * qh + 63);
        if (!wave_skip) {
            const unsigned char *kb = lds + buf * C::kStageBytes;
            const unsigned char *vb = kb + S * kKPitch;
            // ---- S^T = K Q^T ------------------------------------------------------------------------
            f32x16 sacc[C::KB][2];
#pragma unroll
            for (int t = 0; t < C::KB; ++t) {
#pragma unroll
                for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) sacc[t][qb][v] = 0.0f;
                const unsigned char *arow = kb + (C::KC * kh + 32 * t + lr) * kKPitch + 16 * lh;
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    bf16x8 ka = *reinterpret_cast<const bf16x8 *>(arow + 32 * ks);
                    sacc[t][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[0][ks], sacc[t][0], 0, 0, 0);
                    sacc[t][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[1][ks], sacc[t][1], 0, 0, 0);
                }
            }
            if (diag) {
#pragma unroll
                for (int t = 0; t < C::KB; ++t)
#pragma unroll
                    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            int key = C::KC * kh + 32 * t + 8 * (v >> 2) + 4 * lh + (v & 3);
                            int qrow = 64 * qh + 32 * qb + lr;
                            sacc[t][qb][v] = key <= qrow ? sacc[t][qb][v] : -INFINITY;
                        }
            }
            // ---- online softmax, lane-local per query row -------------------------------------------
            bf16x8 pb[C::KB][2][2];
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                float mx = -INFINITY;
#pragma unroll
                for (int t = 0; t < C::KB; ++t)
#pragma unroll
                    for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sacc[t][qb][v]);
                mx = fmaxf(mx, swap_half(mx));
                const float m_new = fmaxf(m_run[qb], mx);
                const float m_safe = m_new == -INFINITY ? 0.0f : m_new;
                const float alpha = fast_exp2((m_run[qb] - m_safe) * c2);
                const float msc = m_safe * c2;
                float sum = 0.0f;
#pragma unroll
                for (int t = 0; t < C::KB; ++t) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        float p = fast_exp2(fmaf(sacc[t][qb][v], c2, -msc));
                        sum += p;
                        sacc[t][qb][v] = p;
                    }
#pragma unroll
                    for (int u = 0; u < 2; ++u)
#pragma unroll
                        for (int e = 0; e < 8; ++e) pb[t][qb][u][e] = (bf16_t)sacc[t][qb][8 * u + e];
                }
                l_run[qb] = l_run[qb] * alpha + sum;
                m_run[qb] = m_new;
                if (__any(alpha != 1.0f)) {
#pragma unroll
                    for (int db = 0; db < 4; ++db)
#pragma unroll
                        for (int v = 0; v < 16; ++v) oacc[db][qb][v] *= alpha;
                }
            }
            // ---- O^T += V^T P^T ---------------------------------------------------------------------
            const int i16 = lane & 15;
#pragma unroll
            for (int t = 0; t < C::KB; ++t) {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int k0 = C::KC * kh + 32 * t + 16 * u + 4 * lh + (i16 >> 2);
#pragma unroll
                    for (int db = 0; db < 4; ++db) {
                        const unsigned char *p0 = vb + k0 * kVPitch + (32 * db + 16 * (lr >> 4) + 4 * (i16 & 3)) * 2;
                        short4v x0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (short4v __attribute__((address_space(3))) *)(p0));
                        short4v x1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (short4v __attribute__((address_space(3))) *)(p0 + 8 * kVPitch));
                        const bf16x8 va = __builtin_bit_cast(bf16x8, __builtin_shufflevector(x0, x1, 0, 1, 2, 3, 4, 5, 6, 7));
                        oacc[db][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[t][0][u], oacc[db][0], 0, 0, 0);
                        oacc[db][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[t][1][u], oacc[db][1], 0, 0, 0);
                    }
                }
            }
        }
        if (jn >= 0) store_tile(buf ^ 1);
        __syncthreads();
        buf ^= 1;
        j = jn;
    }

    // ---- merge the two key halves through LDS, normalise, store -------------------------------------
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) l_run[qb] += swap_half(l_run[qb]);
    float *mo = reinterpret_cast<float *>(lds) + qh * (132 * 64);     // [128 + 4 slots][64 lanes] per query half
    float *ml = mo + 128 * 64;
    if (kh == 1) {
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                for (int v = 0; v < 16; ++v) mo[((db * 2 + qb) * 16 + v) * 64 + lane] = oacc[db][qb][v];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            ml[(qb * 2 + 0) * 64 + lane] = m_run[qb];
            ml[(qb * 2 + 1) * 64 + lane] = l_run[qb];
        }
    }
    __syncthreads();
    if (kh == 0) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const float m1 = ml[(qb * 2 + 0) * 64 + lane], l1 = ml[(qb * 2 + 1) * 64 + lane];
            const float m0 = m_run[qb], l0 = l_run[qb];
            const float m_t = fmaxf(m0, m1);
            const bool empty = m_t == -INFINITY;
            const float m_s = empty ? 0.0f : m_t;
            const float a0 = fast_exp2((m0 - m_s) * c2), a1 = fast_exp2((m1 - m_s) * c2);
            const float l_t = l0 * a0 + l1 * a1;
            const float inv = empty ? 0.0f : 1.0f / l_t;
            const int64_t tok = tok0 + (int64_t)i * S + 64 * qh + 32 * qb + lr;
            bf16_t *dst = a.o + tok * a.o_stride_tok + (int64_t)head * a.o_stride_head;
#pragma unroll
            for (int db = 0; db < 4; ++db) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    float r[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        int v = 4 * g + e;
                        float o1 = mo[((db * 2 + qb) * 16 + v) * 64 + lane];
                        r[e] = (oacc[db][qb][v] * a0 + o1 * a1) * inv;
                    }
                    u32x2 w;
                    w[0] = f32_to_bf16_rne(r[0]) | (f32_to_bf16_rne(r[1]) << 16);
                    w[1] = f32_to_bf16_rne(r[2]) | (f32_to_bf16_rne(r[3]) << 16);
                    *reinterpret_cast<u32x2 *>(dst + 32 * db + 8 * g + 4 * lh) = w;
                }
            }
            if (a.lse != nullptr && lh == 0)
                a.lse[(int64_t)head * a.total_tokens + tok] = empty ? -INFINITY : (__log2f(l_t) + m_t * c2) * kLn2;
        }
    }
}

template <int S, bool CAUSAL, bool DENSE>
static hipError_t attn_launch_t(const AttnArgs &a, hipStream_t stream)
{
    using C = AttnCfg<S>;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&attention_kernel<S, CAUSAL, DENSE>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C::kLdsBytes);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    int64_t nblk = (int64_t)a.n_heads_q * a.NQ;
    if (nblk == 0) return hipSuccess;
    hipLaunchKernelGGL((attention_kernel<S, CAUSAL, DENSE>), dim3((unsigned)nblk), dim3(C::NT), C::kLdsBytes, stream, a);
    return hipGetLastError();
}

hipError_t launch_attention(const AttnArgs &a, hipStream_t stream)
{
    const bool dense = a.mask == nullptr;
#define US_AT(SS, CA, DE) \
    if (a.S == SS && (a.causal != 0) == CA && dense == DE) return attn_launch_t<SS, CA, DE>(a, stream)
    US_AT(128, true, true); US_AT(128, true, false); US_AT(128, false, true); US_AT(128, false, false);
    US_AT(64, true, true); US_AT(64, true, false); US_AT(64, false, true); US_AT(64, false, false);
#undef US_AT
    return hipErrorInvalidValue;
}

}  // namespace us

// Block-sparse attention (Alg. 1 step 5, Sec. 2.2) and the dense baseline (Sec. 2.1), one kernel.
//
// A workgroup owns one (query head, query block of S rows) and visits the key blocks its mask row
// selects (or every valid block when dense).  K and V blocks go from global memory straight into
// LDS (global_load_lds_dwordx4, no staging registers), double buffered: the next block's loads
// are in flight during the current block's math and are awaited at the single barrier per block.
//
// Wavefront tiling (S = 128: eight wavefronts, two per SIMD so that one wavefront's softmax VALU
// work overlaps the other's MFMAs): wavefront (qq, kh) owns query rows [32 qq, 32 qq + 32) and key
// rows [64 kh, 64 kh + 64) of every visited block, with its own running max / sum / output; the
// two key halves are merged through LDS once, after the last block.
//
// All matrix products are computed transposed so that a lane owns whole query rows:
//   S^T (keys x queries)  = K Q^T   : A = K rows from LDS (16-byte reads), B = Q^T kept in registers
//   O^T (dims x queries) += V^T P^T : A = V^T via the LDS transpose read of row-major V,
//                                     B = P^T, which is exactly the accumulator layout of S^T
// With v_mfma_f32_32x32x16_bf16 a lane holds column (query) lane % 32 of the accumulator, so row max,
// row sum and the rescale of O^T are lane-local; only one exchange with lane ^ 32 is needed.
//
// LDS layout: rows of 256 bytes, unpadded (a direct-to-LDS load writes 64 lanes x 16 bytes
// contiguously), with the 16-byte chunk index XOR-swizzled by the row so that the K operand reads
// (32 rows, same column) and the V transpose reads (8 rows x 64 bytes) spread over all banks.  The
// swizzle is applied by choosing which global chunk each lane fetches.
#include <cstdlib>

#include "common.h"

namespace us {

template <int S>
struct AttnCfg {
    static constexpr int QW = S / 32;            // query slices of 32 rows
    static constexpr int KW = 2;                 // key halves
    static constexpr int NW = QW * KW;
    static constexpr int NT = NW * 64;
    static constexpr int KC = S / KW;            // keys per wavefront per block
    static constexpr int KB = KC / 32;           // 32-key MFMA tiles per wavefront per block
    static constexpr int kTileBytes = S * 256;   // one K or V block
    static constexpr int kStageBytes = 2 * kTileBytes;
    static constexpr int kLdsBytes = 2 * kStageBytes;
    static constexpr int kDma = S / 4 / NW;      // 1 KB direct-to-LDS loads per wavefront per K (or V) block
};

__device__ __forceinline__ int k_swizzle(int row) { return row & 15; }
__device__ __forceinline__ int v_swizzle(int row) { return (row & 3) << 2; }

// Work order.  The hardware deals workgroup ids round-robin to the 8 XCDs (private L2 each), and each
// XCD works through its share in order.  Workgroups are grouped in chunks of (one key head) x (R
// consecutive query-block rows) x (its G query heads), about 32 workgroups that read the same K/V; chunk
// number ci runs on XCD ci % 8, longest rows first, and the key head is rotated against the row group
// so that every XCD sees every head (masks of different heads have different densities).
struct AttnOrder {
    int R;           // rows per chunk
    int n_rg;        // row groups = ceil(NQ / R)
    int n_chunks;    // n_rg * n_heads_kv
    int head_major;  // 1: all row groups of key head 0, then head 1, ... ; 0: row groups outermost, heads rotated
};

template <int S, bool CAUSAL, bool DENSE>
__global__ __launch_bounds__(AttnCfg<S>::NT) __attribute__((amdgpu_waves_per_eu(2, 2))) void attention_kernel(AttnArgs a, AttnOrder ord)
{
    using C = AttnCfg<S>;
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    __shared__ uint64_t mwords[UNISPARSE_MAX_BLOCKS_PER_SEQ / 64];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lr = lane & 31, lh = lane >> 5;
    const int qq = wave % C::QW, kh = wave / C::QW;

    // ---- which (head, query-block row) ---------------------------------------------------------------
    const int G = a.n_heads_q / a.n_heads_kv;
    const int cs = ord.R * G;
    const int xcd = blockIdx.x % kNumXcd, idx = blockIdx.x / kNumXcd;
    const int ci = (idx / cs) * kNumXcd + xcd;
    if (ci >= ord.n_chunks) return;
    const int slot = idx % cs;
    const int rg = ord.head_major ? ci % ord.n_rg : ci / a.n_heads_kv;
    const int kvh = ord.head_major ? ci / ord.n_rg : (ci % a.n_heads_kv + rg) % a.n_heads_kv;
    // consecutive workgroups of an XCD go to different shader engines: vary the row, not the head, fastest,
    // so that no engine collects all workgroups of a dense (or sparse) head
    const int row = a.NQ - 1 - (rg * ord.R + slot % ord.R);
    if (row < 0) return;
    const int head = kvh * G + slot / ord.R;
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

    // ---- this wavefront's 32 query rows as B operands -------------------------------------------------
    bf16x8 qreg[8];
    {
        const bf16_t *src = a.q.ptr + (tok0 + (int64_t)i * S + 32 * qq + lr) * a.q.stride_tok +
                            (int64_t)head * a.q.stride_head + 8 * lh;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8 *>(src + 16 * ks);
    }

    // ---- direct-to-LDS block loads: lane l of a 1 KB load fills row l / 16, physical chunk l % 16 -----
    const bf16_t *kptr = a.k.ptr + (int64_t)kvh * a.k.stride_head + tok0 * a.k.stride_tok;
    const bf16_t *vptr = a.v.ptr + (int64_t)kvh * a.v.stride_head + tok0 * a.v.stride_tok;
    const int dma_row = lane >> 4, dma_chunk = lane & 15;
    auto dma_tile = [&](int j, int buf) {
        unsigned char *kb = lds + buf * C::kStageBytes;
        unsigned char *vb = kb + C::kTileBytes;
#pragma unroll
        for (int it = 0; it < C::kDma; ++it) {
            const int r = 4 * (it * C::NW + wave) + dma_row;       // row of the block
            const int64_t grow = (int64_t)j * S + r;
            const bf16_t *gk = kptr + grow * a.k.stride_tok + ((dma_chunk ^ k_swizzle(r)) * 8);
            const bf16_t *gv = vptr + grow * a.v.stride_tok + ((dma_chunk ^ v_swizzle(r)) * 8);
            __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1))) *)gk,
                                             (void __attribute__((address_space(3))) *)(kb + (it * C::NW + wave) * 1024),
                                             16, 0, 0);
            __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1))) *)gv,
                                             (void __attribute__((address_space(3))) *)(vb + (it * C::NW + wave) * 1024),
                                             16, 0, 0);
        }
    };

    f32x16 oacc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[db][v] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;
    const float c2 = a.scale_log2;
    const int i16 = lane & 15;

    int j = next_block();
    if (j >= 0) dma_tile(j, 0);
    __syncthreads();
    int buf = 0;
#pragma unroll 1
    while (j >= 0) {
        const int jn = next_block();
        if (jn >= 0) dma_tile(jn, buf ^ 1);

        const bool diag = CAUSAL && (j == i);
        const bool wave_skip = diag && (C::KC * kh > 32 * qq + 31);
        if (!wave_skip) {
            const unsigned char *kb = lds + buf * C::kStageBytes;
            const unsigned char *vb = kb + C::kTileBytes;
            // ---- S^T = K Q^T ------------------------------------------------------------------------
            f32x16 sacc[C::KB];
            {
                bf16x8 ka[C::KB][8];
#pragma unroll
                for (int t = 0; t < C::KB; ++t) {
                    const int r = C::KC * kh + 32 * t + lr;
                    const unsigned char *arow = kb + r * 256;
                    const int sw = k_swizzle(r);
#pragma unroll
                    for (int ks = 0; ks < 8; ++ks)
                        ka[t][ks] = *reinterpret_cast<const bf16x8 *>(arow + (((2 * ks + lh) ^ sw) << 4));
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t = 0; t < C::KB; ++t)
#pragma unroll
                    for (int v = 0; v < 16; ++v) sacc[t][v] = 0.0f;
#pragma unroll
                for (int ks = 0; ks < 8; ++ks)
#pragma unroll
                    for (int t = 0; t < C::KB; ++t)
                        sacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[t][ks], qreg[ks], sacc[t], 0, 0, 0);
            }
            if (diag) {
#pragma unroll
                for (int t = 0; t < C::KB; ++t)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        int key = C::KC * kh + 32 * t + 8 * (v >> 2) + 4 * lh + (v & 3);
                        int qrow = 32 * qq + lr;
                        sacc[t][v] = key <= qrow ? sacc[t][v] : -INFINITY;
                    }
            }
            // ---- online softmax, lane-local per query row -------------------------------------------
            bf16x8 pb[C::KB][2];
            {
                float mx = -INFINITY;
#pragma unroll
                for (int t = 0; t < C::KB; ++t)
#pragma unroll
                    for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sacc[t][v]);
                mx = fmaxf(mx, swap_half(mx));
                const float m_new = fmaxf(m_run, mx);
                const float m_safe = m_new == -INFINITY ? 0.0f : m_new;
                const float alpha = fast_exp2((m_run - m_safe) * c2);
                const float msc = m_safe * c2;
                float sum = 0.0f;
#pragma unroll
                for (int t = 0; t < C::KB; ++t) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        float p = fast_exp2(fmaf(sacc[t][v], c2, -msc));
                        sum += p;
                        sacc[t][v] = p;
                    }
#pragma unroll
                    for (int u = 0; u < 2; ++u)
#pragma unroll
                        for (int e = 0; e < 8; ++e) pb[t][u][e] = (bf16_t)sacc[t][8 * u + e];
                }
                l_run = l_run * alpha + sum;
                m_run = m_new;
                if (__any(alpha != 1.0f)) {
#pragma unroll
                    for (int db = 0; db < 4; ++db)
#pragma unroll
                        for (int v = 0; v < 16; ++v) oacc[db][v] *= alpha;
                }
            }
            // ---- O^T += V^T P^T ---------------------------------------------------------------------
#pragma unroll
            for (int t = 0; t < C::KB; ++t) {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int r0 = C::KC * kh + 32 * t + 16 * u + 4 * lh + (i16 >> 2);   // + 8 for the second read
                    const unsigned char *vrow = vb + r0 * 256 + (i16 & 1) * 8;
                    const int sw = v_swizzle(r0);                                        // same for row r0 + 8
#pragma unroll
                    for (int db = 0; db < 4; ++db) {
                        const int chunk = (4 * db + 2 * (lr >> 4) + ((i16 & 3) >> 1)) ^ sw;
                        const unsigned char *p0 = vrow + (chunk << 4);
                        short4v x0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (short4v __attribute__((address_space(3))) *)(p0));
                        short4v x1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (short4v __attribute__((address_space(3))) *)(p0 + 8 * 256));
                        const bf16x8 va =
                            __builtin_bit_cast(bf16x8, __builtin_shufflevector(x0, x1, 0, 1, 2, 3, 4, 5, 6, 7));
                        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[t][u], oacc[db], 0, 0, 0);
                    }
                }
            }
        }
        __syncthreads();          // every wavefront is done with buf, and the loads into buf ^ 1 have landed
        buf ^= 1;
        j = jn;
    }

    // ---- merge the two key halves through LDS, normalise, store -------------------------------------
    l_run += swap_half(l_run);
    float *mo = reinterpret_cast<float *>(lds) + qq * (66 * 64);      // [64 + 2 slots][64 lanes] per query slice
    float *ml = mo + 64 * 64;
    if (kh == 1) {
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) mo[(db * 16 + v) * 64 + lane] = oacc[db][v];
        ml[lane] = m_run;
        ml[64 + lane] = l_run;
    }
    __syncthreads();
    if (kh == 0) {
        const float m1 = ml[lane], l1 = ml[64 + lane];
        const float m0 = m_run, l0 = l_run;
        const float m_t = fmaxf(m0, m1);
        const bool empty = m_t == -INFINITY;
        const float m_s = empty ? 0.0f : m_t;
        const float a0 = fast_exp2((m0 - m_s) * c2), a1 = fast_exp2((m1 - m_s) * c2);
        const float l_t = l0 * a0 + l1 * a1;
        const float inv = empty ? 0.0f : 1.0f / l_t;
        const int64_t tok = tok0 + (int64_t)i * S + 32 * qq + lr;
        bf16_t *dst = a.o + tok * a.o_stride_tok + (int64_t)head * a.o_stride_head;
#pragma unroll
        for (int db = 0; db < 4; ++db) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                float r[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    int v = 4 * g + e;
                    float o1 = mo[(db * 16 + v) * 64 + lane];
                    r[e] = (oacc[db][v] * a0 + o1 * a1) * inv;
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
    if (a.n_heads_q == 0 || a.NQ == 0) return hipSuccess;
    const int G = a.n_heads_q / a.n_heads_kv;
    AttnOrder ord;
    ord.R = G >= 32 ? 1 : 32 / G;
    ord.n_rg = (a.NQ + ord.R - 1) / ord.R;
    ord.n_chunks = ord.n_rg * a.n_heads_kv;
    {
        const char *e = getenv("UNISPARSE_ATTN_ORDER");
        ord.head_major = e ? atoi(e) : 1;
    }
    const int64_t per_xcd = (ord.n_chunks + kNumXcd - 1) / kNumXcd;
    const int64_t nblk = per_xcd * kNumXcd * ord.R * G;
    hipLaunchKernelGGL((attention_kernel<S, CAUSAL, DENSE>), dim3((unsigned)nblk), dim3(C::NT), C::kLdsBytes, stream,
                       a, ord);
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

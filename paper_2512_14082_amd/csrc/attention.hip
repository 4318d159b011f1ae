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
// XCD works through its share in order.  Workgroups are grouped in chunks of (HG query heads of one key
// head) x (R consecutive query-block rows), 32 workgroups that read the same K/V; chunk number ci runs on
// XCD ci % 8, longest rows first, and the head group is rotated against the row group so that every XCD
// sees every head (masks of different heads have different densities).
struct AttnOrder {
    int R;           // rows per chunk
    int HG;          // query heads (of one key head) per chunk
    int n_rg;        // row groups = ceil(NQ / R)
    int n_chunks;    // n_rg * (n_heads_q / HG)
    int head_major;  // 1: all row groups of key head 0, then head 1, ... ; 0: row groups outermost, heads rotated
};

template <int S, bool CAUSAL, bool DENSE>
__global__ __launch_bounds__(AttnCfg<S>::NT) __attribute__((amdgpu_waves_per_eu(2, 2))) void attention_kernel(AttnArgs a, AttnOrder ord)
{
    using C = AttnCfg<S>;
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    __shared__ uint16_t jlist[UNISPARSE_MAX_BLOCKS_PER_SEQ];
    __shared__ int jcount;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lr = lane & 31, lh = lane >> 5;
    const int qq = wave % C::QW, kh = wave / C::QW;

    // ---- which (head, query-block row) ---------------------------------------------------------------
    const int G = a.n_heads_q / a.n_heads_kv;
    const int cs = ord.R * ord.HG;
    const int xcd = blockIdx.x % kNumXcd, idx = blockIdx.x / kNumXcd;
    const int ci = (idx / cs) * kNumXcd + xcd;
    if (ci >= ord.n_chunks) return;
    const int slot = idx % cs;
    const int n_hg = a.n_heads_q / ord.HG;                   // head groups
    const int rg = ord.head_major ? ci % ord.n_rg : ci / n_hg;
    const int hg = ord.head_major ? ci / ord.n_rg : (ci % n_hg + rg) % n_hg;
    // consecutive workgroups of an XCD go to different shader engines: vary the row, not the head, fastest,
    // so that no engine collects all workgroups of a dense (or sparse) head
    const int row = a.NQ - 1 - (rg * ord.R + slot % ord.R);
    if (row < 0) return;
    const int head = hg * ord.HG + slot / ord.R;
    const int kvh = head / G;
    int seq, i, nb;
    locate_row(a.st, S, row, seq, i, nb);
    const int64_t tok0 = a.st.cu_tok[seq];
    const int nvalid = CAUSAL ? i + 1 : nb;

    // The selected key blocks of this row, expanded once from the mask bits into an ascending list in LDS
    // (one mask word per lane of wavefront 0, positions placed by a prefix sum of the popcounts).
    int n_sel = nvalid;
    if (!DENSE) {
        if (wave == 0) {
            const int nw = (nvalid + 63) / 64;
            uint64_t bits = 0;
            if (lane < nw) {
                bits = a.mask[((int64_t)head * a.NQ + row) * a.W + lane];
                const int hi = nvalid - lane * 64;
                if (hi < 64) bits &= (1ull << hi) - 1ull;
            }
            const int cnt = __builtin_popcountll(bits);
            int incl = cnt;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int up = __shfl_up(incl, off, 64);
                if (lane >= off) incl += up;
            }
            int pos = incl - cnt;
            while (bits != 0) {
                jlist[pos++] = (uint16_t)(lane * 64 + __builtin_ctzll(bits));
                bits &= bits - 1;
            }
            if (lane == 63) jcount = incl;
        }
        __syncthreads();
        n_sel = __builtin_amdgcn_readfirstlane(jcount);
    }
    int cursor = 0;
    auto next_block = [&]() __attribute__((always_inline)) -> int {
        if (cursor >= n_sel) return -1;
        const int j = DENSE ? cursor : __builtin_amdgcn_readfirstlane((int)jlist[cursor]);
        ++cursor;
        return j;
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
    // Issued as inline assembly so that the compiler does not serialise later LDS reads behind them; their
    // completion is awaited explicitly (vmcnt) before the barrier that publishes the buffer.
    const bf16_t *kptr = a.k.ptr + (int64_t)kvh * a.k.stride_head + tok0 * a.k.stride_tok;
    const bf16_t *vptr = a.v.ptr + (int64_t)kvh * a.v.stride_head + tok0 * a.v.stride_tok;
    const int dma_row = lane >> 4, dma_chunk = lane & 15;
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds;
    auto dma16 = [](const void *gbase, uint32_t goff, uint32_t lds_addr) __attribute__((always_inline)) {
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %0"
                     :
                     : "s"(gbase), "v"(goff), "s"(lds_addr)
                     : "memory", "m0");
    };
    // Only the early group (kh = 0, wavefront index = qq) issues block loads, interleaved with its MFMA chain:
    // kDmaA instructions of 1 KB (4 rows) per wavefront for K and as many for V.
    constexpr int kDmaA = S / 4 / C::QW;
    // per-lane byte offsets inside a block (row r, swizzled chunk); the block base is wave-uniform
    uint32_t koff[kDmaA], voff[kDmaA];
#pragma unroll
    for (int it = 0; it < kDmaA; ++it) {
        const int r = 4 * (it * C::QW + qq) + dma_row;
        koff[it] = (uint32_t)(r * a.k.stride_tok + (dma_chunk ^ k_swizzle(r)) * 8) * 2u;
        voff[it] = (uint32_t)(r * a.v.stride_tok + (dma_chunk ^ v_swizzle(r)) * 8) * 2u;
    }
    // LDS map: K buffers at [0, 2 tiles), V buffers at [2 tiles, 4 tiles).  Instruction d of a block pair:
    // d < kDmaA loads K rows of block jk into K buffer bk, d >= kDmaA loads V rows of block jv into V buffer bv.
    auto dma_one = [&](int d, int jk, int bk, int jv, int bv) __attribute__((always_inline)) {
        if (d < kDmaA) {
            if (jk >= 0)
                dma16(kptr + (int64_t)jk * S * a.k.stride_tok, koff[d],
                      lds_base + bk * C::kTileBytes + (d * C::QW + qq) * 1024);
        } else {
            const int e = d - kDmaA;
            if (jv >= 0)
                dma16(vptr + (int64_t)jv * S * a.v.stride_tok, voff[e],
                      lds_base + (2 + bv) * C::kTileBytes + (e * C::QW + qq) * 1024);
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
    f32x16 sacc[C::KB];
    bf16x8 pb[C::KB][2];
#pragma unroll
    for (int t = 0; t < C::KB; ++t) {
#pragma unroll
        for (int v = 0; v < 16; ++v) sacc[t][v] = 0.0f;
    }

    // ---- MFMA slot ----------------------------------------------------------------------------------------
    // The slot is a flat chain of MFMA "units": first the PV product of the previous block (unit = one MFMA
    // on 16 keys x 32 dims, operand = two transpose reads of V), then S^T of the current block (unit = one
    // MFMA on 32 keys x 16 dims, operand = one 16-byte read of K).  Operand reads run kAhead units in front
    // of the MFMA that consumes them, so LDS latency and issue time hide behind the matrix pipe; the
    // scheduling barriers keep the compiler from collapsing the chain back into "all loads, then all MFMAs"
    // (too many registers) or "load, wait, MFMA" (no overlap).
    constexpr int NG = 2 * C::KB;                 // operand groups per block for K (4 k-steps) and V (16 keys)
    constexpr int NU = 4 * NG;                    // MFMA units per product per block
    constexpr int kAhead = 8;
    bf16x8 opnd[kAhead];                          // operand ring
    // Lane-constant LDS addresses of the operand reads, computed once; every read is "register + immediate".
    typedef const unsigned char __attribute__((address_space(3))) * lds_ptr;
    typedef short4v __attribute__((address_space(3))) * lds_s4_ptr;
    typedef const bf16x8 __attribute__((address_space(3))) * lds_b8_ptr;
    lds_ptr kaddr[8], vaddr[4];
    {
        lds_ptr lbase = (lds_ptr)lds;
        const int r = C::KC * kh + lr;                                    // K row of tile t = 0 (t adds 32 rows)
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) kaddr[ks] = lbase + (r * 256 + (((2 * ks + lh) ^ k_swizzle(r)) << 4));
        const int r0 = C::KC * kh + 4 * lh + (i16 >> 2);                  // V row of group g = 0 (g adds 16 rows)
#pragma unroll
        for (int db = 0; db < 4; ++db) {
            const int chunk = (4 * db + 2 * (lr >> 4) + ((i16 & 3) >> 1)) ^ v_swizzle(r0);
            vaddr[db] = lbase + (2 * C::kTileBytes + r0 * 256 + (i16 & 1) * 8 + (chunk << 4));
        }
    }
    // PV unit u = (g, db): g = u / 4 selects 16 keys, db = u % 4 selects 32 dims
    auto v_fetch = [&](int u) __attribute__((always_inline)) -> bf16x8 {
        const int g = u >> 2, db = u & 3;
        lds_ptr p0 = vaddr[db] + 16 * g * 256;
        short4v x0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_ptr)p0);
        short4v x1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_ptr)(p0 + 8 * 256));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(x0, x1, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    // QK unit u = (t, ks): t = u / 8, ks = u % 8
    auto k_fetch = [&](int u) __attribute__((always_inline)) -> bf16x8 {
        const int t = u >> 3, ks = u & 7;
        return *(lds_b8_ptr)(kaddr[ks] + 32 * t * 256);
    };
    // kaddr / vaddr point into buffer 0 or 1; the other buffer is one block (a power of two) further or back
    int k_flip = C::kTileBytes, v_flip = C::kTileBytes;
    auto flip_k = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) kaddr[ks] += k_flip;
        k_flip = -k_flip;
    };
    auto flip_v = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int db = 0; db < 4; ++db) vaddr[db] += v_flip;
        v_flip = -v_flip;
    };
    // prefill: the first kAhead operand fetches of a chain (may be issued before the barrier that opens the slot
    // when the data was published a slot earlier)
    auto m_prefill = [&](bool has_pv, bool has_qk) __attribute__((always_inline)) {
        const int n_pv = has_pv ? NU : 0, n_all = n_pv + (has_qk ? NU : 0);
#pragma unroll
        for (int w = 0; w < kAhead; ++w) {
            if (w < n_all) {
                if (w < n_pv) opnd[w] = v_fetch(w);
                else opnd[w] = k_fetch(w - n_pv);
            }
        }
    };
    // side(w) runs after the MFMA of unit w (used by the early group to issue block loads)
    auto m_slot = [&](bool has_pv, bool has_qk, auto side) __attribute__((always_inline)) {
        const int n_pv = has_pv ? NU : 0, n_all = n_pv + (has_qk ? NU : 0);
#pragma unroll
        for (int w = 0; w < 2 * NU; ++w) {
            if (w < n_all) {
                __builtin_amdgcn_sched_barrier(0);
                const bf16x8 x = opnd[w % kAhead];
                if (w < n_pv) {
                    const int g = w >> 2, db = w & 3;
                    oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, pb[g >> 1][g & 1], oacc[db], 0, 0, 0);
                } else {
                    const int u = w - n_pv, t = u >> 3, ks = u & 7;
                    if (ks == 0) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) sacc[t][v] = 0.0f;
                    }
                    sacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, qreg[ks], sacc[t], 0, 0, 0);
                }
                if (w + kAhead < n_all) {
                    const int w2 = w + kAhead;
                    if (w2 < n_pv) opnd[w2 % kAhead] = v_fetch(w2);
                    else opnd[w2 % kAhead] = k_fetch(w2 - n_pv);
                }
                side(w);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    // ---- online softmax of the S^T tile, lane-local per query row; leaves P^T (bf16) in pb ---------------
    auto softmax_phase = [&](bool diag) __attribute__((always_inline)) {
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
        // P^T must be complete in this slot: without this the compiler sinks the exponentials past the
        // barrier, next to the MFMAs that consume them, and the VALU work lands in the MFMA slot
#pragma unroll
        for (int t = 0; t < C::KB; ++t)
#pragma unroll
            for (int u = 0; u < 2; ++u) asm volatile("" : "+v"(pb[t][u]));
        asm volatile("" : "+v"(l_run), "+v"(m_run));
    };
    // ---- software pipeline over the visited blocks ----------------------------------------------------------
    // Per wavefront the work is a chain of slots  M_0 V_0 M_1 V_1 ... V_{N-1} M_N  separated by workgroup
    // barriers, where M_n = { O^T += V P^T of block n-1 ; S^T of block n } (MFMA) and V_n = softmax of block
    // n (VALU).  The two wavefronts of a SIMD (key halves kh = 0 / 1) run the same chain one slot apart, so
    // one is in an MFMA slot while the other is in a VALU slot.  Block n's K must be in LDS by global slot
    // 2n and its V by slot 2n + 2; both loads are issued at global slot 2n - 2 resp. 2n by every wavefront
    // (which is the start of M_n for kh = 0 and the start of V_{n-1} for kh = 1) and awaited one slot later.
    // Blocks are visited in ascending order, so only the last one can be the diagonal block.
    auto wait_dma = []() __attribute__((always_inline)) { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };
    auto slot_barrier = []() __attribute__((always_inline)) {
        __builtin_amdgcn_sched_barrier(0);     // keep each slot's instructions on their own side of the barrier
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };
    int j_prev = -1, j_cur = next_block();
    if (j_cur >= 0) {
        int j_nxt = next_block();
        if (kh == 0) {
#pragma unroll
            for (int d = 0; d < kDmaA; ++d) dma_one(d, j_cur, 0, -1, 0);
        }
        wait_dma();
        __syncthreads();
        // global slot 0
        if (kh == 1) slot_barrier();                         // the late group idles through slot 0
        m_prefill(false, true);
        __builtin_amdgcn_s_setprio(2);
        // M_0 (K buffer 0); the early group loads K of block 1 and V of block 0 underneath, spread over the units
        m_slot(false, true, [&](int w) __attribute__((always_inline)) {
            if (kh == 0) {
#pragma unroll
                for (int d = w * 2 * kDmaA / NU; d < (w + 1) * 2 * kDmaA / NU; ++d) dma_one(d, j_nxt, 1, j_cur, 0);
            }
        });
        __builtin_amdgcn_s_setprio(0);
        flip_k();                                            // M_1 reads K buffer 1 and V buffer 0
        slot_barrier();
        int n = 1;
        j_prev = j_cur;
        j_cur = j_nxt;
#pragma unroll 1
        while (j_cur >= 0) {
            j_nxt = next_block();
            // V_{n-1}.  For the late group the blocks of its next MFMA slot were published a slot ago, so it
            // puts that slot's first operand reads in flight before the barrier; the early group's blocks are
            // published by this very barrier.
            softmax_phase(false);
            if (kh == 1) m_prefill(true, true);
            if (kh == 0) wait_dma();
            slot_barrier();
            // M_n: K buffer n & 1, V buffer (n - 1) & 1; loads of K block n+1 and V block n underneath
            if (kh == 0) m_prefill(true, true);
            __builtin_amdgcn_s_setprio(2);
            m_slot(true, true, [&](int w) __attribute__((always_inline)) {
                if (kh == 0) {
#pragma unroll
                    for (int d = w * kDmaA / NU; d < (w + 1) * kDmaA / NU; ++d)
                        dma_one(d, j_nxt, (n + 1) & 1, j_cur, n & 1);
                }
            });
            __builtin_amdgcn_s_setprio(0);
            flip_k();
            flip_v();
            slot_barrier();
            j_prev = j_cur;
            j_cur = j_nxt;
            ++n;
        }
        // V_{N-1}: the last block may be the diagonal one
        if (CAUSAL && j_prev == i) softmax_phase(true);
        else softmax_phase(false);
        if (kh == 1) m_prefill(true, false);
        if (kh == 0) wait_dma();
        slot_barrier();
        // M_N: PV product of block N-1
        if (kh == 0) m_prefill(true, false);
        __builtin_amdgcn_s_setprio(2);
        m_slot(true, false, [](int) __attribute__((always_inline)) {});
        __builtin_amdgcn_s_setprio(0);
        if (kh == 0) slot_barrier();                         // the early group idles through the last slot
    }
    __syncthreads();

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
    ord.HG = G % 2 == 0 ? 2 : 1;
    ord.R = 32 / ord.HG;
    ord.n_rg = (a.NQ + ord.R - 1) / ord.R;
    ord.n_chunks = ord.n_rg * (a.n_heads_q / ord.HG);
    ord.head_major = 0;
    const int64_t per_xcd = (ord.n_chunks + kNumXcd - 1) / kNumXcd;
    const int64_t nblk = per_xcd * kNumXcd * ord.R * ord.HG;
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

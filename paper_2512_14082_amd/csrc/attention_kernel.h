// Block-sparse attention (Alg. 1 step 5, Sec. 2.2) and the dense baseline (Sec. 2.1), one kernel template over the
// head dimension d (64, 128, 256), the block size S (64, 128), causality, and dense / block-sparse.
//
// A workgroup owns one (query head, query block of S rows) and visits the key blocks its mask row selects (or
// every valid block when dense) in stages of SK keys: a whole block, or half a block of 128 at d = 256, where a
// stage of K and V already fills 64 KB.  K and V stages go from global memory straight into LDS
// (global_load_lds_dwordx4, no staging registers), double buffered: the next stage's loads are in flight during
// the current stage's math and are awaited at the single barrier per stage.
//
// Wavefront tiling: wavefront (qq, kh) owns query rows [32 qq, 32 qq + 32) and key rows [64 kh, 64 kh + 64) of every
// visited stage, with its own softmax reference / sum / output; with two key groups they are merged through LDS
// once, after the last stage.  S = 128: eight wavefronts, two per SIMD (d = 256: four, one per SIMD with the whole
// register file, the output accumulators in AccVGPRs); S = 64: two wavefronts.
//
// Every wavefront runs the same software pipeline over "sub-steps" of 32 keys: while the matrix pipe works on S^T of
// sub-step s+1 and on the PV product of sub-step s-1, the VALU does the softmax of sub-step s, cut into chunks of
// about three instructions that sit between consecutive MFMAs (an MFMA hides that much VALU work of the same or
// the other wavefront of the SIMD; measured on gfx950, where dot-product and long runs of transcendental
// instructions are the ones that do not hide).  The chain of a stage is 4 x 8 "units": one MFMA each at d = 128,
// two at d = 256; at d = 64 it is 4 x 4 units with two softmax chunks each (that shape is bound by the exponentials).
//
// All matrix products are computed transposed so that a lane owns whole query rows:
//   S^T (keys x queries)  = K Q^T   : A = K rows from LDS (16-byte reads), B = Q^T kept in registers
//   O^T (dims x queries) += V^T P^T : A = V^T via the LDS transpose read of row-major V,
//                                     B = P^T, which is exactly the accumulator layout of S^T
// With v_mfma_f32_32x32x16_bf16 a lane holds column (query) lane % 32 of the accumulator, so the softmax is
// lane-local.  It needs no row maximum in the common case (see "Reference value" below) and takes its row sums
// on the matrix pipe.
//
// LDS layout: rows of 2 d bytes, unpadded (a direct-to-LDS load writes 64 lanes x 16 bytes contiguously), with the
// 16-byte chunk index XOR-swizzled by the row so that the K operand reads (32 rows, same column) and the V
// transpose reads (8 rows x 64 bytes) spread over all banks.  The swizzle is applied by choosing which global
// chunk each lane fetches.
#pragma once
#include "common.h"

namespace us {

template <int S, int D, int SKP>
struct AttnCfg {
    static constexpr int RB = 2 * D;               // bytes of a K or V row
    static constexpr int CH = D / 8;               // 16-byte chunks per row
    static constexpr int SK = SKP;                 // keys per stage: what one iteration of the pipeline works on and
                                                   // what an LDS buffer holds (a block, or half a block of 128)
    static constexpr int SPB = S / SK;             // stages per block
    static constexpr int QW = S / 32;              // query slices of 32 rows
    static constexpr int KW = SK / 64;             // key groups of 64 rows
    static constexpr int NW = QW * KW;
    static constexpr int NT = NW * 64;
    static constexpr int KC = SK / KW;             // keys per wavefront per stage
    static constexpr int KB = KC / 32;             // 32-key MFMA tiles per wavefront per stage
    static constexpr int KS = D / 16;              // MFMAs of one S^T tile (steps over the head dimension)
    static constexpr int DB = D / 32;              // 32-dim blocks of O^T
    static constexpr int MPU = D >= 128 ? D / 128 : 1;   // MFMAs per unit of the pipeline
    static constexpr int UPP = KS / MPU;           // units per phase (one S^T tile, or the PV product of one tile)
    static constexpr int CPU = 8 / UPP;            // softmax chunks per unit
    static constexpr int kTileBytes = SK * RB;     // one K or V stage
    static constexpr int kStageBytes = 2 * kTileBytes;
    static constexpr int kLdsBytes = 2 * kStageBytes;
    static constexpr int RPL = 1024 / RB;          // rows per 1 KB direct-to-LDS load
    static constexpr int kDma = SK / RPL / NW;     // such loads per wavefront per K (or V) stage
    static constexpr int kWaves = D == 256 ? 1 : 2;   // wavefronts per SIMD (d = 256 needs the whole register file)
    static constexpr int kAhead = 4;               // operand reads run this many units ahead of their MFMAs
};

// XOR swizzles of the 16-byte chunk index by the row: the K operand reads (32 rows, same logical chunk) and the V
// transpose reads (8 rows x 64 bytes) then spread over all banks.  Rows of 256 and 512 bytes cover the 64 banks
// once or twice, rows of 128 bytes (d = 64) only half of them, so there the row's parity takes part.
template <int D> __device__ __forceinline__ int k_swizzle(int row) { return D == 64 ? (row >> 1) & 7 : row & 15; }
template <int D> __device__ __forceinline__ int v_swizzle(int row) { return D == 64 ? ((row >> 1) & 1) << 2 : (row & 3) << 2; }

// Work order.  The hardware deals workgroup ids round-robin to the 8 XCDs (private L2 each), and each
// XCD works through its share in order.  Workgroups are grouped in chunks of (HG query heads of one key
// head) x (R consecutive query-block rows), 32 workgroups that read the same K/V; chunk number ci runs on
// XCD ci % 8, longest rows first, and the head group is rotated against the row group so that every XCD
// sees every head (masks of different heads have different densities).
//
// Ranked variant (block-sparse only, when the caller gives scratch memory): the rows of a chunk are not R consecutive
// rows but R rows of consecutive RANK, every head's rows ranked by (sequence, number of selected blocks descending).
// Workgroups of a chunk then have about the same length, start together and stay together on their way through the
// K/V blocks they share, which is what the L2 needs: on the 128K configuration the traffic behind the L2 halves.  The
// rank table is made by attn_rank_kernel from the mask alone, so the order - and with it nothing but the order: every
// row's arithmetic is the same - is a function of the mask.  The 8 chunks that run at a time are 8 consecutive
// chunks: of one row group and 8 HG heads, or - when the K/V of the key heads those belong to would not fit the
// 256 MB cache behind the L2s (many key heads, long sequences) - of one key head (head_major).
struct AttnOrder {
    int R;           // rows per chunk
    int HG;          // query heads (of one key head) per chunk
    int n_rg;        // row groups = ceil(NQ / R)
    int n_chunks;    // n_rg * (n_heads_q / HG)
    int head_major;  // 1: all row groups of key head 0, then key head 1, ... ; 0: row groups outermost, heads rotated
    const int32_t *table;   // ranked variant: (head << 20 | row) per workgroup id, -1 = no work; NULL = formula below
};
constexpr int kRankMaxRows = 8192;      // rows per head the rank kernel sorts (in LDS)
constexpr int64_t kLastLevelCacheBytes = (int64_t)256 << 20;   // MI355X: 256 MB behind the XCDs' L2s

template <int D, int S, bool CAUSAL, bool DENSE, int SKP>
__global__ __launch_bounds__((AttnCfg<S, D, SKP>::NT))
__attribute__((amdgpu_waves_per_eu(AttnCfg<S, D, SKP>::kWaves, AttnCfg<S, D, SKP>::kWaves)))
void attention_kernel(AttnArgs a, AttnOrder ord)
{
    using C = AttnCfg<S, D, SKP>;
    constexpr int SK = C::SK, RB = C::RB;
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
    int row = a.NQ - 1 - (rg * ord.R + slot % ord.R);
    int head = hg * ord.HG + slot / ord.R;
    if (!DENSE && ord.table != nullptr) {                    // ranked: same chunk, same head, the row of that rank
        const int e = __builtin_amdgcn_readfirstlane(ord.table[blockIdx.x]);
        row = e < 0 ? -1 : (e & 0xfffff);
        head = e < 0 ? head : (e >> 20);
    }
    if (row < 0) return;
    const int kvh = head / G;
    int seq, i, nb;
    locate_row(a.st, S, row, seq, i, nb);
    const int64_t tok0 = a.st.cu_tok[seq];
    const int Lb = a.st.cu_tok[seq + 1] - a.st.cu_tok[seq];
    // A sequence whose length is not a multiple of S ends in a shorter block: its missing rows are never
    // loaded (row indices are clamped to the sequence), never attended (masked like the future keys of the
    // diagonal block) and never stored.
    // The pipeline iterates over stages of SK keys (a block, or at d = 256 half a block), numbered over the sequence.
    const int j_short = Lb % SK != 0 ? Lb / SK : -1;       // index of the shorter last stage, if any
    const int rows_short = Lb % SK;                         // its number of rows
    const int q_rows = (i == nb - 1 && Lb % S != 0) ? Lb % S : S;   // query rows of this workgroup that exist
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
    // stages to visit: every stage of every selected block, except a second half that lies beyond the sequence
    int n_stages = n_sel * C::SPB;
    if (C::SPB == 2 && n_sel > 0) {
        const int j_last = DENSE ? n_sel - 1 : __builtin_amdgcn_readfirstlane((int)jlist[n_sel - 1]);
        if (j_last == nb - 1 && Lb - j_last * S <= SK) --n_stages;
    }
    int cursor = 0;
    auto next_block = [&]() __attribute__((always_inline)) -> int {
        if (cursor >= n_stages) return -1;
        const int b = cursor / C::SPB;
        const int j = DENSE ? b : __builtin_amdgcn_readfirstlane((int)jlist[b]);
        const int js = j * C::SPB + cursor % C::SPB;
        ++cursor;
        return js;
    };

    // ---- this wavefront's 32 query rows as B operands -------------------------------------------------
    bf16x8 qreg[C::KS];
    {
        const int qr = 32 * qq + lr < q_rows ? 32 * qq + lr : q_rows - 1;
        const bf16_t *src = a.q.ptr + (tok0 + (int64_t)i * S + qr) * a.q.stride_tok +
                            (int64_t)head * a.q.stride_head + 8 * lh;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8 *>(src + 16 * ks);
    }

    // ---- direct-to-LDS block loads: lane l of a 1 KB load fills row l / CH, physical chunk l % CH (CH = d / 8) ----
    // Issued as inline assembly so that the compiler does not serialise later LDS reads behind them; their
    // completion is awaited explicitly (vmcnt) before the barrier that publishes the buffer.
    const bf16_t *kptr = a.k.ptr + (int64_t)kvh * a.k.stride_head + tok0 * a.k.stride_tok;
    const bf16_t *vptr = a.v.ptr + (int64_t)kvh * a.v.stride_head + tok0 * a.v.stride_tok;
    const int dma_row = lane / C::CH, dma_chunk = lane % C::CH;
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds;
    auto dma16 = [](const void *gbase, uint32_t goff, uint32_t lds_addr) __attribute__((always_inline)) {
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %0"
                     :
                     : "s"(gbase), "v"(goff), "s"(lds_addr)
                     : "memory", "m0");
    };
    // Every wavefront issues kDma instructions of 1 KB (RPL rows) for K and as many for V per stage.
    constexpr int kDma = C::kDma;
    // Per-lane byte offset of this lane's 16 bytes inside a stage (row r, swizzled chunk) for the wavefront's
    // first load; load number d of a stage is d * RPL * NW rows further and that distance goes into the wave-uniform
    // base address.  The K swizzle has a period of 16 rows: when the row step is 8 or 4, the loads need 2 or 4
    // different offsets, used in turn (the V swizzle has a period of 4 rows, which every row step is a multiple of).
    constexpr int kRowStep = C::RPL * C::NW;      // rows between two consecutive loads of a wavefront
    constexpr int NKO = kRowStep % 16 == 0 ? 1 : (kRowStep % 8 == 0 ? 2 : 4);
    static_assert(kRowStep % 4 == 0, "the V swizzle repeats every four rows");
    uint32_t koff[NKO], voff0;
    {
        const int r = C::RPL * wave + dma_row;
#pragma unroll
        for (int o = 0; o < NKO; ++o)
            koff[o] = (uint32_t)(r * a.k.stride_tok + (dma_chunk ^ k_swizzle<D>(r + kRowStep * o)) * 8) * 2u;
        voff0 = (uint32_t)(r * a.v.stride_tok + (dma_chunk ^ v_swizzle<D>(r)) * 8) * 2u;
    }
    // LDS map: K buffers at [0, 2 tiles), V buffers at [2 tiles, 4 tiles).  Instruction d of an iteration:
    // d < kDma loads K rows of stage jk into K buffer bk, d >= kDma loads V rows of stage jv into V buffer bv.
    const int64_t k_step = (int64_t)kRowStep * a.k.stride_tok, v_step = (int64_t)kRowStep * a.v.stride_tok;
    const uint32_t lds_wave = lds_base + wave * 1024;
    auto dma_one = [&](int d, int jk, int bk, int jv, int bv) __attribute__((always_inline)) {
        if (d < kDma) {
            dma16(kptr + (int64_t)jk * SK * a.k.stride_tok + d * k_step, koff[d % NKO],
                  lds_wave + bk * C::kTileBytes + d * C::NW * 1024);
        } else {
            const int e = d - kDma;
            dma16(vptr + (int64_t)jv * SK * a.v.stride_tok + e * v_step, voff0,
                  lds_wave + (2 + bv) * C::kTileBytes + e * C::NW * 1024);
        }
    };

    // The same loads for a stage that may be the shorter last one: rows beyond the sequence are replaced by its
    // last row (only used outside the main loop, so the extra address arithmetic does not matter).
    auto dma_clamped = [&](int d, int jk, int bk, int jv, int bv) __attribute__((always_inline)) {
        const bool is_k = d < kDma;
        const int e = is_k ? d : d - kDma, j = is_k ? jk : jv;
        const int rows = j == j_short ? rows_short : SK;
        int r = C::RPL * (e * C::NW + wave) + dma_row;
        const int swz = is_k ? k_swizzle<D>(r) : v_swizzle<D>(r);
        r = r < rows ? r : rows - 1;
        const int64_t st = is_k ? a.k.stride_tok : a.v.stride_tok;
        const uint32_t off = (uint32_t)(r * st + (dma_chunk ^ swz) * 8) * 2u;
        dma16((is_k ? kptr : vptr) + (int64_t)j * SK * st, off,
              lds_wave + (is_k ? bk : 2 + bv) * C::kTileBytes + e * C::NW * 1024);
    };

    f32x16 oacc[C::DB];
#pragma unroll
    for (int db = 0; db < C::DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[db][v] = 0.0f;
    float m_run = -INFINITY;                     // reference value of the exponentials (raw logits), per query row
    float msc = -INFINITY;                       // m_run * c2 + kOff, or -inf while the row has seen no finite logit
    const float c2 = a.scale_log2;
    const int i16 = lane & 15;
    static_assert(C::KB == 2, "the pipeline below works on two 32-key tiles per wavefront and stage");
    // The unit of the software pipeline is a "sub-step": one 32-key tile t of one stage, numbered 2 n + t.
    // State is kept twice, indexed by the parity of the sub-step (= t).
    f32x16 sacc[2];                              // S^T tile
    u32x4 pbw[2][2];                             // P^T tile as packed bf16 pairs: two MFMA operands of 16 keys
    float sm_a[2][2], sm_x[2][2];                // exponent arguments / exponentials in flight (even, odd value)
    uint32_t ovf = 0;                            // OR of the packed probabilities of the sub-step in flight
    // Row sums on the matrix pipe: lacc += R P^T with v_mfma_f32_16x16x32_bf16, where the 16 x 32 matrix R has ones in
    // row 0 for the contraction indices of lanes 0-15 and 32-47 and in row 1 for those of lanes 16-31 and 48-63.  A lane
    // of a P^T operand holds eight probabilities of query (lane % 32), so row 0 of the product collects the sixteen
    // probabilities of queries 0-15 and row 1 those of queries 16-31: lacc[0] / lacc[1] of lanes 0-15.
    f32x4 lacc = {0.0f, 0.0f, 0.0f, 0.0f};
    bf16x8 ones_a;
    {
        const bool one = (lane & 15) < 2 && ((lane >> 4) & 1) == (lane & 15);
#pragma unroll
        for (int e = 0; e < 8; ++e) ones_a[e] = one ? (bf16_t)1.0f : (bf16_t)0.0f;
    }

    // ---- operand fetches -------------------------------------------------------------------------------
    // MFMA "units": a QK unit is one MFMA on 32 keys x 16 dims (operand = one 16-byte read of K), a PV unit
    // one MFMA on 16 keys x 32 dims (operand = two transpose reads of V).  Operand reads run kAhead units
    // in front of the MFMA that consumes them.
    constexpr int kAhead = C::kAhead;
    constexpr int kDmaGap = 2;                   // MFMA units between two block loads (when the chain is long enough)
    bf16x8 opnd[kAhead][C::MPU];                  // operand ring: the operands of the MFMAs of one unit
    // Lane-constant LDS addresses of the operand reads, computed once; every read is "register + immediate".
    typedef const unsigned char __attribute__((address_space(3))) * lds_ptr;
    typedef short4v __attribute__((address_space(3))) * lds_s4_ptr;
    typedef const bf16x8 __attribute__((address_space(3))) * lds_b8_ptr;
    lds_ptr kaddr[C::KS], vaddr[C::DB];
    {
        lds_ptr lbase = (lds_ptr)lds;
        const int r = C::KC * kh + lr;                                    // K row of tile t = 0 (t adds 32 rows)
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) kaddr[ks] = lbase + (r * RB + (((2 * ks + lh) ^ k_swizzle<D>(r)) << 4));
        const int r0 = C::KC * kh + 4 * lh + (i16 >> 2);                  // V row of group g = 0 (g adds 16 rows)
#pragma unroll
        for (int db = 0; db < C::DB; ++db) {
            const int chunk = (4 * db + 2 * (lr >> 4) + ((i16 & 3) >> 1)) ^ v_swizzle<D>(r0);
            vaddr[db] = lbase + (2 * C::kTileBytes + r0 * RB + (i16 & 1) * 8 + (chunk << 4));
        }
    }
    // PV operand: tile t, group g (16 keys) of the tile, dims block db
    // (`off`: compile-time byte offset of the buffer, for the unrolled main loop whose base addresses never move)
    auto v_fetch = [&](int t, int g, int db, int off) __attribute__((always_inline)) -> bf16x8 {
        lds_ptr p0 = vaddr[db] + ((32 * t + 16 * g) * RB + off);
        short4v x0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_ptr)p0);
        short4v x1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_ptr)(p0 + 8 * RB));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(x0, x1, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    // QK operand: tile t, k-step ks
    auto k_fetch = [&](int t, int ks, int off) __attribute__((always_inline)) -> bf16x8 {
        return *(lds_b8_ptr)(kaddr[ks] + (32 * t * RB + off));
    };
    // kaddr / vaddr point into buffer 0 or 1; the other buffer is one block further or back
    int k_flip = C::kTileBytes, v_flip = C::kTileBytes;
    auto flip_k = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) kaddr[ks] += k_flip;
        k_flip = -k_flip;
    };
    auto flip_v = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int db = 0; db < C::DB; ++db) vaddr[db] += v_flip;
        v_flip = -v_flip;
    };

    // ---- online softmax in chunks of a few instructions (lane-local per query row) -----------------------
    // Per sub-step the 16 values of a lane go through
    //   MX: starts the pipeline below (arguments of values 0 and 1, exponential of value 0)
    //   EX: one chunk per value u: [pack values u-1, u to bf16, OR the packed word into ovf]; exp(u+1); argument(u+2)
    //       - nothing in a chunk uses a result of the same chunk, so VALU latency never stalls the wavefront
    //   and a test of ovf when the sub-step closes (has the reference value to move?).
    // Every chunk is tied (empty asm) to the operand of the MFMA that follows it, which keeps it between the
    // same two MFMAs in the machine code: the matrix pipe hides a handful of VALU instructions per MFMA.
    // Last visited block only: keys after the query's own position (diagonal block of a causal row) and keys
    // beyond the end of the sequence (shorter last block) are excluded.  key_max = highest admissible key row.
    auto sm_mask = [&](auto par_c, int key_max) __attribute__((always_inline)) {
        constexpr int par = decltype(par_c)::value;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            int key = C::KC * kh + 32 * par + 8 * (v >> 2) + 4 * lh + (v & 3);
            sacc[par][v] = key <= key_max ? sacc[par][v] : -INFINITY;
        }
    };
    auto key_max_of = [&](int j) __attribute__((always_inline)) -> int {
        int km = j == j_short ? rows_short - 1 : SK - 1;
        if (CAUSAL && j / C::SPB == i) km = min(km, 32 * qq + lr - (j % C::SPB) * SK);   // (negative: nothing visible)
        return km;
    };
    auto needs_mask = [&](int j) __attribute__((always_inline)) -> bool {
        return (CAUSAL && j / C::SPB == i) || j == j_short;
    };
    // Reference value of the exponentials.  Softmax is shift-invariant, so any reference works as long as no
    // exponential overflows and the row's largest ones stay far above the underflow threshold.  The reference of a
    // row is the maximum of the first tile that shows it a finite logit, and from then on it moves only when some
    // probability would reach 2^(kOff + 1) relative to it; the probabilities carry a constant factor 2^-kOff, which
    // puts that bound at 2.0: "some value of the tile reached 2.0" is one bit of the bf16 exponent (infinities and
    // NaNs have it too), read off the OR of the packed probabilities.  The common case therefore needs no row
    // maximum, no rescaling factor and no rescaling test: per value one fma, one exponential, half a conversion,
    // and a quarter of an OR.  The row sums are taken by the matrix pipe over the very bf16 values the PV product
    // multiplies (numerator and denominator round alike).
    constexpr float kOff = 20.0f;
    constexpr int NMX = 2;
    // Starts sub-step `par`: arguments of values 0 and 1, exponential of value 0.
    auto mx_chunk = [&](auto par_c, auto m_c, bf16x8 &next) __attribute__((always_inline)) {
        constexpr int par = decltype(par_c)::value, m = decltype(m_c)::value;
        const f32x16 &s = sacc[par];
        if constexpr (m == 0) {
            sm_a[par][0] = fmaf(s[0], c2, -msc);
            sm_a[par][1] = fmaf(s[1], c2, -msc);
            asm volatile("" : "+v"(sm_a[par][0]), "+v"(sm_a[par][1]), "+v"(next));
        } else {
            sm_x[par][0] = fast_exp2(sm_a[par][0]);
            asm volatile("" : "+v"(sm_x[par][0]), "+v"(next));
        }
    };
    // EX chunk of value u: [pack values u-1, u to bf16, OR into ovf]; exp(u+1); argument(u+2).
    auto ex_chunk = [&](auto par_c, auto u_c, bf16x8 &next) __attribute__((always_inline)) {
        constexpr int par = decltype(par_c)::value, u = decltype(u_c)::value;
        if constexpr ((u & 1) != 0) {
            f32x2 pe = {sm_x[par][0], sm_x[par][1]};
            pbw[par][u >> 3][(u >> 1) & 3] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pe, bf16x2));
        }
        if constexpr (u == 3) ovf = pbw[par][0][0] | pbw[par][0][1];
        if constexpr (u == 7) ovf = ovf | pbw[par][0][2] | pbw[par][0][3];
        if constexpr (u == 11) ovf = ovf | pbw[par][1][0] | pbw[par][1][1];
        if constexpr (u == 15) ovf = ovf | pbw[par][1][2] | pbw[par][1][3];
        if constexpr (u + 1 < 16) sm_x[par][(u + 1) & 1] = fast_exp2(sm_a[par][(u + 1) & 1]);
        if constexpr (u + 2 < 16) sm_a[par][u & 1] = fmaf(sacc[par][u + 2], c2, -msc);
        // (only values that exist take part in a pin: a pinned constant would cost a move)
        if constexpr ((u & 3) == 3) {
            asm volatile("" : "+v"(pbw[par][u >> 3][(u >> 1) & 3]), "+v"(ovf), "+v"(sm_x[par][0]), "+v"(sm_x[par][1]),
                              "+v"(sm_a[par][0]), "+v"(sm_a[par][1]), "+v"(next));
        } else if constexpr ((u & 1) != 0) {
            asm volatile("" : "+v"(pbw[par][u >> 3][(u >> 1) & 3]), "+v"(sm_x[par][0]), "+v"(sm_x[par][1]),
                              "+v"(sm_a[par][0]), "+v"(sm_a[par][1]), "+v"(next));
        } else {
            asm volatile("" : "+v"(sm_x[par][0]), "+v"(sm_x[par][1]), "+v"(sm_a[par][0]), "+v"(sm_a[par][1]), "+v"(next));
        }
    };
    // The uncommon case, and the first tile of every row: take the tile's row maximum (one exchange with the other
    // half of the key rows, lane ^ 32), move the reference of the rows that exceed it, redo the tile's probabilities
    // and rescale what was accumulated under the old reference.  `started` says whether the next sub-step (the other
    // parity) has already taken its first values under the old reference; they are redone as well.
    auto sm_slow = [&](auto par_c, auto started_c) __attribute__((always_inline)) {
        constexpr int par = decltype(par_c)::value;
        constexpr bool started = decltype(started_c)::value != 0;
        const f32x16 &s = sacc[par];
        float mx = fmaxf(fmaxf(s[0], s[1]), s[2]);
#pragma unroll
        for (int v = 3; v < 16; ++v) mx = fmaxf(mx, s[v]);
        auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
        const float tmax = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
        const float m_new = fmaxf(m_run, tmax);
        const bool none = m_new == -INFINITY;                 // the row has still seen nothing but masked keys
        const float m_safe = none ? 0.0f : m_new;
        const float alpha = fast_exp2((m_run - m_safe) * c2); // 1 for rows whose reference stays, 0 for a first reference
        m_run = m_new;
        msc = none ? -INFINITY : fmaf(m_safe, c2, kOff);
        const float msc_safe = none ? 0.0f : msc;
#pragma unroll
        for (int v = 0; v < 16; v += 2) {
            f32x2 pe = {fast_exp2(fmaf(s[v], c2, -msc_safe)), fast_exp2(fmaf(s[v + 1], c2, -msc_safe))};
            pbw[par][v >> 3][(v >> 1) & 3] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pe, bf16x2));
        }
        if (__any(alpha != 1.0f)) {
#pragma unroll
            for (int db = 0; db < C::DB; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) oacc[db][v] *= alpha;
            lacc[0] *= __shfl(alpha, lane & 15, 64);
            lacc[1] *= __shfl(alpha, (lane & 15) + 16, 64);
        }
        if constexpr (started) {
            sm_a[par ^ 1][0] = fmaf(sacc[par ^ 1][0], c2, -msc);
            sm_a[par ^ 1][1] = fmaf(sacc[par ^ 1][1], c2, -msc);
            sm_x[par ^ 1][0] = fast_exp2(sm_a[par ^ 1][0]);
        }
    };
    // Closes sub-step `par`: nothing to do unless some probability reached 2.0 (or is not a number: a row without a
    // reference yet).
    auto sm_finish = [&](auto par_c, auto started_c) __attribute__((always_inline)) {
        if (__any((ovf & 0x40004000u) != 0u)) sm_slow(par_c, started_c);
    };
    const std::integral_constant<int, 0> c0;
    const std::integral_constant<int, 1> c1;

    // ---- one iteration of the pipeline --------------------------------------------------------------------
    // Iteration n (stage n = j_n in the K/V buffers n & 1) is one chain of 4 UPP units (UPP = 8, or 4 at d = 64)
    //   [S^T of stage n+1, tile 0] [PV of stage n, tile 0] [S^T of stage n+1, tile 1] [PV of stage n, tile 1]
    // with the softmax chunks of sub-steps 2n+1 (EX, first half of the chain), 2n+2 (MX right after the S^T of its
    // tile, EX in the second half) and 2n+3 (MX) between them.  The block loads of an
    // iteration (K of block n+2 into the buffer of K block n, V of block n+1 into the buffer of V block n-1:
    // both buffers were last read in the iteration before) are spread over the chain and awaited at the barrier
    // that closes the iteration.  Without a stage n+1 (has_qk = 0) the chain is the PV units only.
    // buf_c: 0 = the address registers point at the buffers this iteration reads (they are flipped between
    // iterations); 1 / 2 = they point at buffer 0 and this is an even / odd iteration of the unrolled main loop: K of
    // stage n+1 sits in buffer (n+1) & 1, V of stage n in buffer n & 1, reached through immediate offsets.
    auto iteration = [&](auto has_qk_c, auto diag_c, auto kload_c, auto vload_c, auto clamp_c, auto buf_c, bool diag, int key_max,
                         int jk, int bk, int jv, int bv)
                         __attribute__((always_inline)) {
        constexpr int buf = decltype(buf_c)::value;
        constexpr int k_off = buf == 1 ? C::kTileBytes : 0, v_off = buf == 2 ? C::kTileBytes : 0;
        constexpr bool has_qk = decltype(has_qk_c)::value != 0, may_diag = decltype(diag_c)::value != 0,
                       kload = decltype(kload_c)::value != 0, vload = decltype(vload_c)::value != 0,
                       clamp = decltype(clamp_c)::value != 0;
        constexpr int UPP = C::UPP, MPU = C::MPU, CPU = C::CPU, UPG = UPP / 2;
        constexpr int n_all = has_qk ? 4 * UPP : 2 * UPP;
        // unit w: phase ph (even: S^T of tile ph / 2, odd: the PV product of tile ph / 2), unit u of the phase
        auto fetch = [&](auto w_c, bf16x8 (&dst)[MPU]) __attribute__((always_inline)) {
            constexpr int w = decltype(w_c)::value;
            constexpr int ph = has_qk ? (w / UPP) : 2 * (w / UPP) + 1, t = ph >> 1, u = w % UPP;
#pragma unroll
            for (int m = 0; m < MPU; ++m) {
                if constexpr ((ph & 1) == 0) dst[m] = k_fetch(t, u * MPU + m, k_off);
                else dst[m] = v_fetch(t, u / UPG, (u % UPG) * MPU + m, v_off);
            }
        };
        static_for<(kAhead < n_all ? kAhead : n_all)>([&](auto w_c) __attribute__((always_inline)) { fetch(w_c, opnd[decltype(w_c)::value % kAhead]); });
        static_for<n_all>([&](auto w_c) __attribute__((always_inline)) {
            constexpr int w = decltype(w_c)::value;
            constexpr int ph = has_qk ? (w / UPP) : 2 * (w / UPP) + 1, t = ph >> 1, u = w % UPP;
            __builtin_amdgcn_sched_barrier(0);
            static_for<MPU>([&](auto m_c) __attribute__((always_inline)) {
                constexpr int m = decltype(m_c)::value;
                const bf16x8 x = opnd[w % kAhead][m];
                if constexpr ((ph & 1) == 0) {
                    constexpr int ks = u * MPU + m;
                    f32x16 zero;
#pragma unroll
                    for (int v = 0; v < 16; ++v) zero[v] = 0.0f;
                    sacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, qreg[ks], ks == 0 ? zero : sacc[t], 0, 0, 0);
                } else {
                    constexpr int g = u / UPG, db = (u % UPG) * MPU + m;
                    oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, __builtin_bit_cast(bf16x8, pbw[t][g]), oacc[db], 0, 0, 0);
                    if constexpr (db == C::DB - 1)
                        lacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones_a, __builtin_bit_cast(bf16x8, pbw[t][g]), lacc, 0, 0, 0);
                }
            });
            if constexpr (w + kAhead < n_all) fetch(std::integral_constant<int, (w + kAhead < n_all ? w + kAhead : 0)>{}, opnd[(w + kAhead) % kAhead]);
            // block loads, evenly spread
            constexpr int n_dma = (kload ? kDma : 0) + (vload ? kDma : 0);
            if constexpr (n_dma > 0) {
                constexpr int gap = kDmaGap * 2 * kDma <= n_all ? kDmaGap : n_all / (2 * kDma);
                static_assert(gap >= 1, "more block loads than units");
                if constexpr (w % gap == gap / 2 && w / gap < 2 * kDma) {
                    constexpr int d = w / gap;
                    if constexpr ((d < kDma && kload) || (d >= kDma && vload)) {
                        if constexpr (clamp) dma_clamped(d, jk, bk, jv, bv);
                        else dma_one(d, jk, bk, jv, bv);
                    }
                }
            }
            bf16x8 &next = opnd[(w + 1) % kAhead][0];
            if constexpr (has_qk) {
                // sub-step of parity 1 in the first half of the chain, of parity 0 in the second: CPU chunks per unit
                static_for<CPU>([&](auto c_c) __attribute__((always_inline)) {
                    constexpr int uu = (w % (2 * UPP)) * CPU + decltype(c_c)::value;
                    if constexpr (w < 2 * UPP) ex_chunk(c1, std::integral_constant<int, uu>{}, next);
                    else ex_chunk(c0, std::integral_constant<int, uu>{}, next);
                });
                if constexpr (may_diag && (w == UPP - 1 || w == 3 * UPP - 1)) {
                    if (diag) sm_mask(std::integral_constant<int, (w == 3 * UPP - 1)>{}, key_max);
                }
                constexpr int mx0 = UPP + 1, mx1 = 3 * UPP + 1;
                if constexpr (w >= mx0 && w < mx0 + NMX) mx_chunk(c0, std::integral_constant<int, (w >= mx0 && w < mx0 + NMX ? w - mx0 : 0)>{}, next);
                if constexpr (w >= mx1 && w < mx1 + NMX) mx_chunk(c1, std::integral_constant<int, (w >= mx1 && w < mx1 + NMX ? w - mx1 : 0)>{}, next);
                if constexpr (w == 2 * UPP - 1) {
                    __builtin_amdgcn_sched_barrier(0);
                    sm_finish(c1, c1);
                }
                if constexpr (w == 4 * UPP - 1) {
                    __builtin_amdgcn_sched_barrier(0);
                    sm_finish(c0, c1);
                }
            } else {
                if constexpr (w < UPP) {
                    static_for<16 / UPP>([&](auto c_c) __attribute__((always_inline)) {
                        ex_chunk(c1, std::integral_constant<int, (w % UPP) * (16 / UPP) + decltype(c_c)::value>{}, next);
                    });
                }
                if constexpr (w == UPP - 1) {
                    __builtin_amdgcn_sched_barrier(0);
                    sm_finish(c1, c0);
                }
            }
        });
        __builtin_amdgcn_sched_barrier(0);
    };
    auto wait_dma = []() __attribute__((always_inline)) { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };
    auto close_unrolled = [&]() __attribute__((always_inline)) {
        wait_dma();
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
    };
    auto close_iteration = [&]() __attribute__((always_inline)) {
        flip_k();
        flip_v();
        wait_dma();
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
    };

    // ---- pipeline over the visited stages (ascending: only the last ones lie on the diagonal or are short) ----
    const int j_first = next_block();
    if (j_first >= 0) {
        int j1 = next_block();                    // block n+1 at the top of iteration n
        int j2 = j1 >= 0 ? next_block() : -1;     // block n+2
#pragma unroll
        for (int d = 0; d < 2 * kDma; ++d) dma_clamped(d, j_first, 0, j_first, 0);
        if (j1 >= 0) {
#pragma unroll
            for (int d = 0; d < kDma; ++d) dma_clamped(d, j1, 1, -1, 0);
        }
        wait_dma();
        __syncthreads();
        // prologue: S^T of stage 0, the whole softmax of its tile 0 (which sets the reference value of every row that
        // sees a key in it) and the start of its tile 1, unhidden
        static_for<2 * C::KS>([&](auto w_c) __attribute__((always_inline)) {
            constexpr int w = decltype(w_c)::value, t = w / C::KS, ks = w % C::KS;
            f32x16 zero;
#pragma unroll
            for (int v = 0; v < 16; ++v) zero[v] = 0.0f;
            sacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_fetch(t, ks, 0), qreg[ks], ks == 0 ? zero : sacc[t], 0, 0, 0);
        });
        if (needs_mask(j_first)) {
            const int km = key_max_of(j_first);
            sm_mask(c0, km);
            sm_mask(c1, km);
        }
        sm_slow(c0, c0);
        static_for<NMX>([&](auto m_c) __attribute__((always_inline)) { mx_chunk(c1, m_c, opnd[0][0]); });
        __syncthreads();                          // K buffer 0 is reloaded from the first iteration on
        int n = 0;
        if (j1 >= 0) {
            // Main loop, two iterations per trip so that the buffer an iteration reads is known at compile time and
            // the address registers never move: while stage n+2 exists and is whole and stage n+1 needs no mask.
            auto plain = [&]() __attribute__((always_inline)) -> bool { return j2 >= 0 && j2 != j_short && !needs_mask(j1); };
            const std::integral_constant<int, 2> c2_;
#pragma unroll 1
            while (plain()) {
                iteration(c1, c0, c1, c1, c0, c1, false, 0, j2, 0, j1, 1);          // n even
                close_unrolled();
                j1 = j2;
                j2 = next_block();
                ++n;
                if (!plain()) break;
                iteration(c1, c0, c1, c1, c0, c2_, false, 0, j2, 1, j1, 0);         // n odd
                close_unrolled();
                j1 = j2;
                j2 = next_block();
                ++n;
            }
            // from here on the address registers follow the buffers: K of stage n+1, V of stage n
            if ((n & 1) == 0) {
                flip_k();
            } else {
                flip_v();
            }
#pragma unroll 1
            while (j2 >= 0) {                     // the last stages of the row: clamped loads, masked tiles
                iteration(c1, c1, c1, c1, c1, c0, needs_mask(j1), key_max_of(j1), j2, n & 1, j1, (n + 1) & 1);
                close_iteration();
                j1 = j2;
                j2 = next_block();
                ++n;
            }
            // stage n+1 is the last one: no K stage to load; it may lie on the diagonal and / or be the shorter one
            iteration(c1, c1, c0, c1, c1, c0, needs_mask(j1), key_max_of(j1), -1, 0, j1, (n + 1) & 1);
            close_iteration();
        }
        // the last block's P V
        iteration(c0, c0, c0, c0, c0, c0, false, 0, -1, 0, -1, 0);
    }
    __syncthreads();

    // ---- merge the two key halves through LDS, normalise, store -------------------------------------
    // row sums: lanes 0-15 hold those of queries 0-15 in lacc[0] and of queries 16-31 in lacc[1]
    const float l_lo = __shfl(lacc[0], lane & 15, 64), l_hi = __shfl(lacc[1], lane & 15, 64);   // (all lanes active)
    const float l_run = lr < 16 ? l_lo : l_hi;
    constexpr int kSlots = 16 * C::DB;                                 // accumulator registers of a lane
    float *mo = reinterpret_cast<float *>(lds) + qq * ((kSlots + 2) * 64);   // [kSlots + 2][64 lanes] per query slice
    float *ml = mo + kSlots * 64;
    static_assert(C::KW == 1 || C::QW * (kSlots + 2) * 64 * 4 <= C::kLdsBytes, "merge buffer exceeds the LDS");
    if (kh == 1) {
#pragma unroll
        for (int db = 0; db < C::DB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) mo[(db * 16 + v) * 64 + lane] = oacc[db][v];
        ml[lane] = m_run;
        ml[64 + lane] = l_run;
    }
    __syncthreads();
    if (kh == 0) {
        const float m1 = C::KW == 2 ? ml[lane] : -INFINITY, l1 = C::KW == 2 ? ml[64 + lane] : 0.0f;
        const float m0 = m_run, l0 = l_run;
        const float m_t = fmaxf(m0, m1);
        const bool empty = m_t == -INFINITY;
        const float m_s = empty ? 0.0f : m_t;
        const float a0 = fast_exp2((m0 - m_s) * c2), a1 = fast_exp2((m1 - m_s) * c2);
        const float l_t = l0 * a0 + l1 * a1;
        const float inv = empty ? 0.0f : 1.0f / l_t;
        const bool row_exists = 32 * qq + lr < q_rows;
        const int64_t tok = tok0 + (int64_t)i * S + 32 * qq + lr;
        bf16_t *dst = a.o + tok * a.o_stride_tok + (int64_t)head * a.o_stride_head;
#pragma unroll
        for (int db = 0; db < C::DB; ++db) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                float r[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    int v = 4 * g + e;
                    float o1 = C::KW == 2 ? mo[(db * 16 + v) * 64 + lane] : 0.0f;
                    r[e] = (oacc[db][v] * a0 + o1 * a1) * inv;
                }
                u32x2 w;
                w[0] = f32_to_bf16_rne(r[0]) | (f32_to_bf16_rne(r[1]) << 16);
                w[1] = f32_to_bf16_rne(r[2]) | (f32_to_bf16_rne(r[3]) << 16);
                if (row_exists) *reinterpret_cast<u32x2 *>(dst + 32 * db + 8 * g + 4 * lh) = w;
            }
        }
        if (a.lse != nullptr && lh == 0 && row_exists)
            a.lse[(int64_t)head * a.total_tokens + tok] = empty ? -INFINITY : (__log2f(l_t) + m_t * c2 + kOff) * kLn2;
    }
}

// fills a.sched with the ranked work order of `ord` (defined in attention.hip)
hipError_t launch_attention_rank(const AttnArgs &a, const AttnOrder &ord, hipStream_t stream);

template <int D, int S, bool CAUSAL, bool DENSE, int SKP>
static hipError_t attn_launch_t(const AttnArgs &a, hipStream_t stream)
{
    using C = AttnCfg<S, D, SKP>;
    static LdsAttr attr;
    hipError_t e = attr.set(reinterpret_cast<const void *>(&attention_kernel<D, S, CAUSAL, DENSE, SKP>), C::kLdsBytes);
    if (e != hipSuccess) return e;
    if (a.n_heads_q == 0 || a.NQ == 0) return hipSuccess;
    const int G = a.n_heads_q / a.n_heads_kv;
    // workgroups of a chunk: what an XCD (32 CUs) runs at a time - two per CU with the half-block stages of d = 64
    // and 128 (four wavefronts and at most 64 KB of LDS each)
    constexpr int kChunk = (D <= 128 && S == 128 && SKP == 64) ? 64 : 32;
    AttnOrder ord;
    ord.HG = G % 2 == 0 ? 2 : 1;
    ord.R = kChunk / ord.HG;
    ord.n_rg = (a.NQ + ord.R - 1) / ord.R;
    ord.n_chunks = ord.n_rg * (a.n_heads_q / ord.HG);
    ord.head_major = 0;
    ord.table = nullptr;
    // ranked order when the caller gave scratch for it; long rows (>= 960 blocks) then do best with chunks of one head
    // (not for a grid that fits the device at once: there the order changes nothing and the ranking is one more launch)
    const bool ranked = !DENSE && a.sched != nullptr && a.NQ <= kRankMaxRows && a.n_heads_q < 2048 &&
                        (int64_t)a.n_heads_q * a.NQ > 512 &&
                        (int64_t)attention_sched_bytes(a.n_heads_q, a.n_heads_kv, a.NQ) <= a.sched_bytes;
    if (ranked && a.W >= 16) {
        ord.HG = 1;
        ord.R = kChunk;
        ord.n_rg = (a.NQ + ord.R - 1) / ord.R;
        ord.n_chunks = ord.n_rg * a.n_heads_q;
    }
    const int64_t per_xcd = (ord.n_chunks + kNumXcd - 1) / kNumXcd;
    const int64_t nblk = per_xcd * kNumXcd * ord.R * ord.HG;
    if (ranked) {
        // The 8 chunks that run at a time belong to 8 HG / G key heads.  When the K and V of that many key heads (of
        // the longest sequence) do not fit the last-level cache, the chunks are ordered key head by key head instead
        // of row group by row group, so that one key head's K/V is what the XCDs' L2 misses fall on.
        int max_len = 0;
        for (int b = 0; b < a.st.num_seqs; ++b) max_len = max(max_len, a.st.cu_tok[b + 1] - a.st.cu_tok[b]);
        const int64_t kv_at_a_time = min((int64_t)a.n_heads_kv, ((int64_t)kNumXcd * ord.HG + G - 1) / G);
        const int64_t kv_bytes = kv_at_a_time * 2 * (int64_t)max_len * D * 2;
        ord.head_major = kv_at_a_time > 1 && kv_bytes >= kLastLevelCacheBytes ? 1 : 0;
        e = launch_attention_rank(a, ord, stream);
        if (e != hipSuccess) return e;
        ord.table = a.sched;
    }
    hipLaunchKernelGGL((attention_kernel<D, S, CAUSAL, DENSE, SKP>), dim3((unsigned)nblk), dim3(C::NT), C::kLdsBytes, stream,
                       a, ord);
    return hipGetLastError();
}

// All instantiations of one head dimension (each head dimension is compiled in a translation unit of its own).
template <int D>
static hipError_t attn_dispatch_t(const AttnArgs &a, hipStream_t stream)
{
    const bool dense = a.mask == nullptr;
    // Stage size at S = 128.  d = 256: half a block (a whole one would need 256 KB of LDS).  d = 64 and 128: half a
    // block - workgroups of four wavefronts, two per CU, which fill each other's barriers, prologues and epilogues
    // (d = 128: dense -2 %, block-sparse rows of up to a few hundred blocks -2 ... -4 %; d = 64: -4 % and -8 %) -
    // except for block-sparse rows of a thousand blocks and more, where whole blocks and one workgroup of eight
    // wavefronts per CU do as well or better (twice as many workgroups per XCD spread over more of the K/V stream
    // than its L2 holds).
    constexpr int kHalf = 64;
    const bool whole_blocks = D != 256 && (!dense && a.W >= 16);
#define US_AT(SS, CA, DE, SK) \
    if (a.S == SS && (a.causal != 0) == CA && dense == DE) return attn_launch_t<D, SS, CA, DE, SK>(a, stream)
    if (whole_blocks) {
        if constexpr (D != 256) {
            US_AT(128, true, false, 128); US_AT(128, false, false, 128);
        }
    } else {
        US_AT(128, true, true, kHalf); US_AT(128, true, false, kHalf); US_AT(128, false, true, kHalf); US_AT(128, false, false, kHalf);
    }
    US_AT(64, true, false, 64); US_AT(64, false, false, 64);      // (dense problems with S = 64 arrive as S = 128)
#undef US_AT
    return hipErrorInvalidValue;
}

hipError_t attn_dispatch_d64(const AttnArgs &a, hipStream_t stream);
hipError_t attn_dispatch_d128(const AttnArgs &a, hipStream_t stream);
hipError_t attn_dispatch_d256(const AttnArgs &a, hipStream_t stream);

}  // namespace us

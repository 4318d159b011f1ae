// Shared declarations of the UniSparse HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

#include "unisparse.h"

namespace us {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kMaxSeqs = UNISPARSE_MAX_SEQS;
constexpr int kNumXcd = 8;              // MI355X: 8 accelerator dies, workgroups are dealt round-robin to them
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Packed-batch geometry passed to kernels by value.
struct SeqTable {
    int32_t num_seqs;
    int32_t cu_tok[kMaxSeqs + 1];       // token offsets, cu_tok[num_seqs] = total tokens
};

struct TensorView {
    const bf16_t *ptr;
    int64_t stride_tok;
    int64_t stride_head;
};

// Packed query-block row -> (sequence, local block index, blocks in that sequence).  A sequence whose length
// is not a multiple of S ends in a shorter block.
__device__ __forceinline__ void locate_row(const SeqTable &st, int S, int row, int &seq, int &local, int &nblk)
{
    seq = 0;
    int base = 0;
#pragma unroll 1
    for (int b = 0; b < st.num_seqs; ++b) {
        int nb = (st.cu_tok[b + 1] - st.cu_tok[b] + S - 1) / S;
        if (row < base + nb) { seq = b; local = row - base; nblk = nb; return; }
        base += nb;
    }
    seq = st.num_seqs - 1; local = 0; nblk = 0;   // not reached for valid rows
}

// Workgroup ids are dealt round-robin over the 8 XCDs (each with a private L2).  This maps the
// hardware id to a virtual id such that consecutive virtual ids share an XCD.
__device__ __forceinline__ int xcd_contiguous_id(int bid, int nblocks)
{
    int xcd = bid % kNumXcd, idx = bid / kNumXcd;
    int low = nblocks / kNumXcd, rem = nblocks % kNumXcd;
    return xcd * low + (xcd < rem ? xcd : rem) + idx;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Exchange between lane l and lane l ^ 32.
__device__ __forceinline__ float swap_half(float x)
{
    return __shfl_xor(x, 32, 64);
}

// float -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float x)
{
    uint32_t u = __float_as_uint(x);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// 8 bf16 (16 bytes) -> fp32, and back with round to nearest even.
__device__ __forceinline__ void unpack8(const u32x4 &w, float *f)
{
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        f[2 * e] = __uint_as_float(w[e] << 16);
        f[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
    }
}

__device__ __forceinline__ u32x4 pack8_rne(const float *f)
{
    u32x4 w;
#pragma unroll
    for (int e = 0; e < 4; ++e) w[e] = f32_to_bf16_rne(f[2 * e]) | (f32_to_bf16_rne(f[2 * e + 1]) << 16);
    return w;
}

// Compile-time loop: f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N - 1>{}).
template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// A kernel that needs more than 64 KB of dynamic LDS must be told so once per device (the attribute belongs to the
// device's copy of the kernel).  One object per kernel instantiation; racing first calls both set it, harmlessly.
struct LdsAttr {
    bool done[32] = {};
    hipError_t set(const void *kernel, int bytes)
    {
        int dev = -1;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= 32) return hipErrorInvalidDevice;
        if (done[dev]) return hipSuccess;
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (e == hipSuccess) done[dev] = true;
        return e;
    }
};

// ---- kernel launchers (defined one per .hip file) ------------------------------------------
// head_dim is 64, 128 or 256 everywhere.
hipError_t launch_avgpool_seq(const TensorView &x, int n_heads, int64_t total_tokens, int c, int pool, int head_dim,
                              bf16_t *out, hipStream_t stream);
// The same per sequence: sequence b owns ceil(L_b / c) composite tokens, its last window may be partial.
hipError_t launch_avgpool_seq_varlen(const TensorView &x, int n_heads, const SeqTable &st, int c, int pool,
                                     int head_dim, bf16_t *out, hipStream_t stream);
hipError_t launch_stochpool_seq_varlen(const TensorView &x, int n_heads, const SeqTable &st, int c, int head_dim,
                                       const float *u, bf16_t *out, hipStream_t stream);
hipError_t launch_avgpool_head(const bf16_t *x, int n_heads_in, int64_t tokens, int c_h, int head_dim, bf16_t *out,
                               hipStream_t stream);

struct ProxyArgs {
    const bf16_t *qt;        // [Hc][Tq][d] composite queries (Tq = cu_cq[num_seqs]); NULL: q_src is pooled on the fly
    TensorView q_src;        // the queries themselves, [T, H, d] view (used when qt == NULL: average pooling, Eq. (1))
    const bf16_t *kt;        // [Hkc][Tk][d] composite keys
    float *score;            // [Hc][NQ][NK], written by the two-sweep form (u == NULL)
    // one-sweep form (u != NULL): per composite query row and key block the unnormalised sum of exponentials,
    // [Hc][NQ][ceil(NK / 64)][n_q / 4][64][4] (row r of a query block and key block j at [j / 64][r / 4][j % 64][r % 4]),
    // and the rows' weights 1 / denominator, [Hc][NQ][n_q]
    float *u;
    float *w;
    SeqTable st;
    int32_t cu_cq[kMaxSeqs + 1];     // packed offsets of the composite queries / keys: sequence b owns
    int32_t cu_ck[kMaxSeqs + 1];     // ceil(L_b / c) of them
    int32_t n_heads_q, n_heads_kv;   // (compressed) head counts
    int32_t S, c_q, c_k;
    int32_t causal;
    int32_t NQ, NK;
    int32_t head_dim;        // d
    int32_t tiles;           // 32-row tiles per wavefront: 0 = automatic, 1 or 2 forced
    int32_t n_cu;            // compute units of the device (for the automatic choice)
    float scale_log2;        // softmax scale * log2(e)
};
hipError_t launch_proxy_scores(const ProxyArgs &a, hipStream_t stream);

struct SelectArgs {
    float *score;            // [Hc][NQ][NK]: read, or - with u != NULL - formed from u and w and written
    const float *u;          // ProxyArgs::u and ::w of the one-sweep score kernel, NULL = the scores are given
    const float *w;
    int32_t c_q;
    uint64_t *mask;          // [Hc * c_h][NQ][W]
    SeqTable st;
    int32_t n_heads_c;       // compressed heads
    int32_t c_h;
    int32_t S, causal, NQ, NK, W;
    int32_t mode;
    double param;
};
hipError_t launch_select(const SelectArgs &a, hipStream_t stream);

struct AttnArgs {
    TensorView q, k, v;
    bf16_t *o;
    int64_t o_stride_tok, o_stride_head;
    const uint64_t *mask;    // NULL = dense
    float *lse;              // optional [H][T]
    SeqTable st;
    int32_t n_heads_q, n_heads_kv;
    int32_t S, causal, NQ, W;
    int32_t head_dim;
    int64_t total_tokens;
    float scale_log2;
    int32_t *sched;          // optional scratch for a mask-dependent work order (block-sparse only), NULL = none
    int64_t sched_bytes;
};
// bytes of AttnArgs::sched that let launch_attention rank the rows of every head by their number of selected blocks
size_t attention_sched_bytes(int n_heads_q, int n_heads_kv, int NQ);
// one software-pipelined kernel (attention_kernel.h), instantiated per head dimension, block size, causality and
// dense / block-sparse
hipError_t launch_attention(const AttnArgs &a, hipStream_t stream);

}  // namespace us

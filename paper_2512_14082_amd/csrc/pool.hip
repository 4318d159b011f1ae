// Composite tokens: sequence-level (Eq. (1)) and head-level (Eq. (2)) average pooling.
//
// HBM-bound streaming kernels.  One thread owns 8 consecutive channels (16 bytes) of one composite
// token, so the d / 8 threads of a token (d = head dimension: 64, 128 or 256) read one coalesced row per
// source token.  The sum is
// an fp32 sum in token (head) order followed by one fp32 division and one round-to-nearest-even to
// bf16, which is bit-for-bit what a bf16 average pool defines.  With pool = UNISPARSE_POOL_MAX the same
// windows are reduced by a channel-wise maximum instead (exact: the result is one of the inputs).
#include "common.h"

namespace us {

template <int C>
__global__ __launch_bounds__(256) void avgpool_seq_kernel(const bf16_t *__restrict__ x, int64_t stride_tok,
                                                          int64_t stride_head, int64_t tokens_out, int c_rt,
                                                          int pool, int lpt_shift, int64_t n_items,
                                                          bf16_t *__restrict__ out)
{
    const int c = C > 0 ? C : c_rt;
    int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= n_items) return;
    int chunk = (int)(gid & ((1 << lpt_shift) - 1));      // 1 << lpt_shift = d / 8 threads per token
    int64_t tt = gid >> lpt_shift;
    int64_t t = tt % tokens_out;
    int64_t h = tt / tokens_out;
    const bf16_t *src = x + h * stride_head + (t * c) * stride_tok + chunk * 8;
    const bool pmax = pool == UNISPARSE_POOL_MAX;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = pmax ? -INFINITY : 0.0f;
    if (C > 0) {
        u32x4 w[C > 0 ? C : 1];
#pragma unroll
        for (int m = 0; m < C; ++m) w[m] = *reinterpret_cast<const u32x4 *>(src + m * stride_tok);
#pragma unroll
        for (int m = 0; m < C; ++m) {
            float f[8];
            unpack8(w[m], f);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = pmax ? fmaxf(acc[e], f[e]) : acc[e] + f[e];
        }
    } else {
        for (int m = 0; m < c; ++m) {
            u32x4 w = *reinterpret_cast<const u32x4 *>(src + m * stride_tok);
            float f[8];
            unpack8(w, f);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = pmax ? fmaxf(acc[e], f[e]) : acc[e] + f[e];
        }
    }
    const float cf = pmax ? 1.0f : (float)c;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = acc[e] / cf;
    *reinterpret_cast<u32x4 *>(out + ((h * tokens_out + t) << (lpt_shift + 3)) + chunk * 8) = pack8_rne(acc);
}

// log2(d / 8): threads per token
static int lpt_shift_of(int head_dim) { return head_dim == 64 ? 3 : head_dim == 256 ? 5 : 4; }

hipError_t launch_avgpool_seq(const TensorView &x, int n_heads, int64_t total_tokens, int c, int pool, int head_dim,
                              bf16_t *out, hipStream_t stream)
{
    const int sh = lpt_shift_of(head_dim);
    int64_t tokens_out = total_tokens / c;
    int64_t n_items = ((int64_t)n_heads * tokens_out) << sh;
    if (n_items == 0) return hipSuccess;
    dim3 grid((unsigned)((n_items + 255) / 256)), block(256);
#define US_POOL(CC)                                                                                         \
    hipLaunchKernelGGL(avgpool_seq_kernel<CC>, grid, block, 0, stream, x.ptr, x.stride_tok, x.stride_head, \
                       tokens_out, c, pool, sh, n_items, out)
    switch (c) {
        case 4: US_POOL(4); break;
        case 8: US_POOL(8); break;
        case 16: US_POOL(16); break;
        default: US_POOL(0); break;
    }
#undef US_POOL
    return hipGetLastError();
}

// Eq. (1) for packed sequences of any length: composite token t of the packed output belongs to the sequence b
// with cu_c[b] <= t < cu_c[b + 1] (cu_c accumulated on the fly), its window is clipped to that sequence and the
// divisor is the number of tokens in it.
__global__ __launch_bounds__(256) void avgpool_seq_varlen_kernel(const bf16_t *__restrict__ x, int64_t stride_tok,
                                                                 int64_t stride_head, SeqTable st, int c, int pool,
                                                                 int lpt_shift, int64_t tokens_out, int64_t n_items,
                                                                 bf16_t *__restrict__ out)
{
    int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= n_items) return;
    int chunk = (int)(gid & ((1 << lpt_shift) - 1));
    int64_t tt = gid >> lpt_shift;
    int64_t t = tt % tokens_out;
    int64_t h = tt / tokens_out;
    int64_t base = 0;
    int tok_first = 0, cnt = 0;
    for (int b = 0; b < st.num_seqs; ++b) {
        const int len = st.cu_tok[b + 1] - st.cu_tok[b];
        const int nc = (len + c - 1) / c;
        if (t < base + nc) {
            const int w = (int)(t - base);
            tok_first = st.cu_tok[b] + w * c;
            cnt = min(c, len - w * c);
            break;
        }
        base += nc;
    }
    const bf16_t *src = x + h * stride_head + (int64_t)tok_first * stride_tok + chunk * 8;
    const bool pmax = pool == UNISPARSE_POOL_MAX;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = pmax ? -INFINITY : 0.0f;
    for (int m = 0; m < cnt; ++m) {
        u32x4 w = *reinterpret_cast<const u32x4 *>(src + m * stride_tok);
        float f[8];
        unpack8(w, f);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = pmax ? fmaxf(acc[e], f[e]) : acc[e] + f[e];
    }
    const float cf = pmax ? 1.0f : (float)cnt;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = acc[e] / cf;
    *reinterpret_cast<u32x4 *>(out + ((h * tokens_out + t) << (lpt_shift + 3)) + chunk * 8) = pack8_rne(acc);
}

hipError_t launch_avgpool_seq_varlen(const TensorView &x, int n_heads, const SeqTable &st, int c, int pool,
                                     int head_dim, bf16_t *out, hipStream_t stream)
{
    const int sh = lpt_shift_of(head_dim);
    int64_t tokens_out = 0;
    for (int b = 0; b < st.num_seqs; ++b) tokens_out += (st.cu_tok[b + 1] - st.cu_tok[b] + c - 1) / c;
    int64_t n_items = ((int64_t)n_heads * tokens_out) << sh;
    if (n_items == 0) return hipSuccess;
    dim3 grid((unsigned)((n_items + 255) / 256)), block(256);
    hipLaunchKernelGGL(avgpool_seq_varlen_kernel, grid, block, 0, stream, x.ptr, x.stride_tok, x.stride_head, st, c,
                       pool, sh, tokens_out, n_items, out);
    return hipGetLastError();
}

// Stochastic pooling of the windows of Eq. (1) (third strategy of the ablation "Compression Strategy"): the composite
// token is one token of its window, token m drawn with probability ||x_m||_2 / sum_m' ||x_m'||_2 by inversion of the
// caller's uniform number u[h][t].  A comparison decides an index, so the arithmetic is pinned down: fp32 squares
// accumulated by fused multiply-adds in channel order, a correctly rounded square root, the running sum in token
// order, and the first m with (w_0 + ... + w_m) > u * total wins (the last token if none does).
//
// 16 lanes serve one window.  Lane l computes the norms of tokens l and l + 16 of the window, each over the d
// channels in order (so no cross-lane reduction touches the rounding), the 16 lanes exchange them, every lane
// repeats the same running sum, and the group then copies the chosen row, 16 bytes per lane and turn.
__device__ __forceinline__ float token_norm(const bf16_t *row, int head_dim)
{
    float sq = 0.0f;
#pragma unroll 4
    for (int k = 0; k < head_dim / 8; ++k) {
        u32x4 w = *reinterpret_cast<const u32x4 *>(row + k * 8);
        float f[8];
        unpack8(w, f);
#pragma unroll
        for (int e = 0; e < 8; ++e) sq = __builtin_fmaf(f[e], f[e], sq);
    }
    return __builtin_sqrtf(sq);          // IEEE square root (hipcc rounds fp32 sqrt correctly by default)
}

__global__ __launch_bounds__(256) void stochpool_seq_varlen_kernel(const bf16_t *__restrict__ x, int64_t stride_tok,
                                                                   int64_t stride_head, SeqTable st, int c,
                                                                   int head_dim, const float *__restrict__ u,
                                                                   int64_t tokens_out, int64_t n_items,
                                                                   bf16_t *__restrict__ out)
{
    int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= n_items) return;                     // n_items is a multiple of 16: groups leave together
    int lane16 = (int)(gid & 15);
    int64_t tt = gid >> 4;
    int64_t t = tt % tokens_out;
    int64_t h = tt / tokens_out;
    int64_t base = 0;
    int tok_first = 0, cnt = 0;
    for (int b = 0; b < st.num_seqs; ++b) {
        const int len = st.cu_tok[b + 1] - st.cu_tok[b];
        const int nc = (len + c - 1) / c;
        if (t < base + nc) {
            const int w = (int)(t - base);
            tok_first = st.cu_tok[b] + w * c;
            cnt = min(c, len - w * c);
            break;
        }
        base += nc;
    }
    if (cnt <= 0) return;                           // cannot happen for t < tokens_out; the whole group agrees
    const bf16_t *src = x + h * stride_head + (int64_t)tok_first * stride_tok;
    float w0 = lane16 < cnt ? token_norm(src + (int64_t)lane16 * stride_tok, head_dim) : 0.0f;
    float w1 = lane16 + 16 < cnt ? token_norm(src + (int64_t)(lane16 + 16) * stride_tok, head_dim) : 0.0f;
    float total = 0.0f;
    for (int m = 0; m < cnt; ++m) total = total + __shfl(m < 16 ? w0 : w1, m & 15, 16);
    const float cut = u[h * tokens_out + t] * total;
    int pick = cnt - 1;
    float run = 0.0f;
    bool found = false;
    for (int m = 0; m < cnt; ++m) {
        run = run + __shfl(m < 16 ? w0 : w1, m & 15, 16);
        if (!found && run > cut) {
            pick = m;
            found = true;
        }
    }
    for (int ch = lane16; ch < head_dim / 8; ch += 16) {
        u32x4 row = *reinterpret_cast<const u32x4 *>(src + (int64_t)pick * stride_tok + ch * 8);
        *reinterpret_cast<u32x4 *>(out + (h * tokens_out + t) * head_dim + ch * 8) = row;
    }
}

hipError_t launch_stochpool_seq_varlen(const TensorView &x, int n_heads, const SeqTable &st, int c, int head_dim,
                                       const float *u, bf16_t *out, hipStream_t stream)
{
    if (c > 32) return hipErrorInvalidValue;        // two tokens per lane
    int64_t tokens_out = 0;
    for (int b = 0; b < st.num_seqs; ++b) tokens_out += (st.cu_tok[b + 1] - st.cu_tok[b] + c - 1) / c;
    int64_t n_items = (int64_t)n_heads * tokens_out * 16;
    if (n_items == 0) return hipSuccess;
    dim3 grid((unsigned)((n_items + 255) / 256)), block(256);
    hipLaunchKernelGGL(stochpool_seq_varlen_kernel, grid, block, 0, stream, x.ptr, x.stride_tok, x.stride_head, st, c,
                       head_dim, u, tokens_out, n_items, out);
    return hipGetLastError();
}

// out[h'][t][:] = bf16(mean over m < c_h of x[h' c_h + m][t][:]); x, out contiguous [heads][tokens][d].
__global__ __launch_bounds__(256) void avgpool_head_kernel(const bf16_t *__restrict__ x, int64_t tokens, int c_h,
                                                           int lpt_shift, int64_t n_items, bf16_t *__restrict__ out)
{
    int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= n_items) return;
    int chunk = (int)(gid & ((1 << lpt_shift) - 1));
    int64_t tt = gid >> lpt_shift;
    int64_t t = tt % tokens;
    int64_t hp = tt / tokens;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.0f;
    for (int m = 0; m < c_h; ++m) {
        u32x4 w = *reinterpret_cast<const u32x4 *>(x + (((hp * c_h + m) * tokens + t) << (lpt_shift + 3)) + chunk * 8);
        float f[8];
        unpack8(w, f);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = acc[e] + f[e];
    }
    const float cf = (float)c_h;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = acc[e] / cf;
    *reinterpret_cast<u32x4 *>(out + ((hp * tokens + t) << (lpt_shift + 3)) + chunk * 8) = pack8_rne(acc);
}

hipError_t launch_avgpool_head(const bf16_t *x, int n_heads_in, int64_t tokens, int c_h, int head_dim, bf16_t *out,
                               hipStream_t stream)
{
    const int sh = lpt_shift_of(head_dim);
    int64_t n_items = ((int64_t)(n_heads_in / c_h) * tokens) << sh;
    if (n_items == 0) return hipSuccess;
    dim3 grid((unsigned)((n_items + 255) / 256)), block(256);
    hipLaunchKernelGGL(avgpool_head_kernel, grid, block, 0, stream, x, tokens, c_h, sh, n_items, out);
    return hipGetLastError();
}

}  // namespace us

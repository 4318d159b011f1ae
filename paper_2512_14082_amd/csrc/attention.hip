// Launcher of the attention kernel (attention_kernel.h) and its head-dimension-128 instantiations.
#include "attention_kernel.h"

namespace us {

hipError_t attn_dispatch_d128(const AttnArgs &a, hipStream_t stream) { return attn_dispatch_t<128>(a, stream); }

// ---- ranked work order ------------------------------------------------------------------------------------------
// One workgroup per query head: the head's rows are sorted by (sequence ascending, selected blocks descending, row
// descending) - a bitonic sort of 32-bit keys in LDS - and the row of rank k is written where the attention kernel's
// workgroup of chunk slot k % R of row group k / R of this head looks for it.  The chunks are numbered row group by
// row group with the heads rotated, or (AttnOrder::head_major) key head by key head.
constexpr int kRankThreads = 1024;

__global__ __launch_bounds__(kRankThreads) void attn_rank_kernel(AttnArgs a, AttnOrder ord, int32_t *table)
{
    __shared__ uint32_t keys[kRankMaxRows];
    const int h = blockIdx.x, tid = threadIdx.x;
    int n2 = 1;
    while (n2 < a.NQ) n2 <<= 1;
    for (int r = tid; r < n2; r += kRankThreads) {
        uint32_t key = 0xffffffffu;                              // padding sorts last
        if (r < a.NQ) {
            int seq, i, nb;
            locate_row(a.st, a.S, r, seq, i, nb);
            const int nvalid = a.causal ? i + 1 : nb;            // bits beyond the valid set are ignored, as in the kernel
            const uint64_t *mrow = a.mask + ((int64_t)h * a.NQ + r) * a.W;
            int len = 0;
            for (int w = 0; w * 64 < nvalid; ++w) {
                uint64_t bits = mrow[w];
                const int hi = nvalid - w * 64;
                if (hi < 64) bits &= (1ull << hi) - 1ull;
                len += __builtin_popcountll(bits);
            }
            key = ((uint32_t)seq << 26) | ((uint32_t)(UNISPARSE_MAX_BLOCKS_PER_SEQ - len) << 13) | (uint32_t)(a.NQ - 1 - r);
        }
        keys[r] = key;
    }
    __syncthreads();
    for (int k = 2; k <= n2; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = tid; t < n2; t += kRankThreads) {
                const int p = t ^ j;
                if (p > t) {
                    const uint32_t x = keys[t], y = keys[p];
                    const bool up = (t & k) == 0;
                    if ((x > y) == up) { keys[t] = y; keys[p] = x; }
                }
            }
            __syncthreads();
        }
    }
    const int n_hg = a.n_heads_q / ord.HG, cs = ord.R * ord.HG;
    const int hg = h / ord.HG, hh = h % ord.HG;
    for (int k = tid; k < ord.n_rg * ord.R; k += kRankThreads) {
        const int rg = k / ord.R;
        int ci = rg * n_hg + ((hg - rg) % n_hg + n_hg) % n_hg;     // the chunk with (ci % n_hg + rg) % n_hg == hg
        if (ord.head_major) {
            // all chunks of one key head, then the next key head's: positions inside a key head's run ordered by
            // (row group, head) and shifted cyclically by the key head's number, so that over the key heads every
            // XCD (position % 8) sees every rank
            const int gq = (a.n_heads_q / a.n_heads_kv) / ord.HG;        // head groups per key head
            const int kvg = hg / gq, nph = ord.n_rg * gq;
            ci = kvg * nph + (rg * gq + hg % gq + kvg) % nph;
        }
        const int idx = (ci / kNumXcd) * cs + hh * ord.R + k % ord.R;
        const int row = k < a.NQ ? a.NQ - 1 - (int)(keys[k] & 0x1fffu) : -1;
        table[(int64_t)idx * kNumXcd + ci % kNumXcd] = row < 0 ? -1 : ((h << 20) | row);
    }
}

size_t attention_sched_bytes(int n_heads_q, int n_heads_kv, int NQ)
{
    // the largest of the chunk shapes the launcher may pick: 32 or 64 workgroups of 1 or 2 heads
    size_t best = 0;
    for (int chunk = 32; chunk <= 64; chunk += 32) {
        for (int HG = 1; HG <= 2; ++HG) {
            if ((n_heads_q / n_heads_kv) % HG != 0) continue;
            const int R = chunk / HG;
            const int64_t n_chunks = (int64_t)((NQ + R - 1) / R) * (n_heads_q / HG);
            const int64_t nblk = (n_chunks + kNumXcd - 1) / kNumXcd * kNumXcd * chunk;
            if ((size_t)nblk * 4 > best) best = (size_t)nblk * 4;
        }
    }
    return (best + 255) & ~(size_t)255;
}

hipError_t launch_attention_rank(const AttnArgs &a, const AttnOrder &ord, hipStream_t stream)
{
    hipLaunchKernelGGL(attn_rank_kernel, dim3((unsigned)a.n_heads_q), dim3(kRankThreads), 0, stream, a, ord, a.sched);
    return hipGetLastError();
}

hipError_t launch_attention(const AttnArgs &a_in, hipStream_t stream)
{
    AttnArgs a = a_in;
    // Dense attention does not depend on the block size (the causal mask is applied per token): problems with
    // S = 64 run as S = 128, whose workgroups of four wavefronts fill the CUs twice as well as the two of S = 64.
    if (a.mask == nullptr && a.S == 64) {
        a.S = 128;
        a.NQ = 0;
        for (int b = 0; b < a.st.num_seqs; ++b) a.NQ += (a.st.cu_tok[b + 1] - a.st.cu_tok[b] + 127) / 128;
        a.W = (a.W + 1) / 2;
    }
    switch (a.head_dim) {
        case 64: return attn_dispatch_d64(a, stream);
        case 128: return attn_dispatch_d128(a, stream);
        case 256: return attn_dispatch_d256(a, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace us

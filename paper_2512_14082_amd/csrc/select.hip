// Block selection, Alg. 1 step 4: causal cut, then Top-P (Eq. (5)) or a fixed budget per row.
//
// One 256-thread workgroup owns one (compressed head, query-block row).  The row's valid scores
// (j <= i when causal) are packed as 64-bit keys  score_bits << 32 | ~j, sorted descending with
// a bitonic network in LDS (so equal scores order by ascending j), prefix-summed in fp64 and cut
// where the cumulative share first reaches P.  The selected columns are scattered into a bit row
// with LDS atomics (order independent) and written out as uint64 words, once per broadcast head.
#include "common.h"

namespace us {

constexpr int kSelThreads = 256;
constexpr int kSelMaxN = UNISPARSE_MAX_BLOCKS_PER_SEQ;

__global__ __launch_bounds__(kSelThreads) void select_kernel(SelectArgs a)
{
    extern __shared__ uint64_t keys[];                    // next power of two >= NK entries (sized by the launcher)
    __shared__ double part[2][kSelThreads];
    __shared__ uint32_t bits[kSelMaxN / 32];

    const int tid = threadIdx.x;
    const int row = blockIdx.x % a.NQ;
    const int hc = blockIdx.x / a.NQ;
    int seq, i, nb;
    locate_row(a.st, a.S, row, seq, i, nb);
    const int nv = a.causal ? i + 1 : nb;
    int P2 = 1;
    while (P2 < nv) P2 <<= 1;

    float *srow = a.score + ((int64_t)hc * a.NQ + row) * a.NK;
    for (int idx = tid; idx < P2; idx += kSelThreads) {
        uint64_t key = 0;
        if (idx < nv) {
            float s = srow[idx];
            s = s > 0.0f ? s : 0.0f;
            key = ((uint64_t)__float_as_uint(s) << 32) | (uint64_t)(0xffffffffu - (uint32_t)idx);
        }
        keys[idx] = key;
    }
    for (int idx = nv + tid; idx < a.NK; idx += kSelThreads) srow[idx] = 0.0f;   // outside the valid set
    for (int w = tid; w < kSelMaxN / 32; w += kSelThreads) bits[w] = 0u;
    __syncthreads();

    // bitonic sort, descending
    for (int k = 2; k <= P2; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = tid; t < (P2 >> 1); t += kSelThreads) {
                int lo = ((t / j) * (j << 1)) + (t % j);
                int hi = lo + j;
                bool desc = (lo & k) == 0;
                uint64_t x = keys[lo], y = keys[hi];
                if ((x < y) == desc) { keys[lo] = y; keys[hi] = x; }
            }
            __syncthreads();
        }
    }

    // fp64 prefix sums over the sorted order: each thread owns a contiguous chunk
    const int E = P2 >= kSelThreads ? P2 / kSelThreads : 1;
    const int p0 = tid * E;
    double local = 0.0;
    if (p0 < P2) {
        for (int e = 0; e < E; ++e) local += (double)__uint_as_float((uint32_t)(keys[p0 + e] >> 32));
    }
    part[0][tid] = local;
    __syncthreads();
    int cur = 0;
    for (int off = 1; off < kSelThreads; off <<= 1) {                 // inclusive Hillis-Steele scan
        double v = part[cur][tid];
        if (tid >= off) v += part[cur][tid - off];
        part[cur ^ 1][tid] = v;
        cur ^= 1;
        __syncthreads();
    }
    const double tot = part[cur][kSelThreads - 1];
    double run = part[cur][tid] - local;                               // cumulative score before this chunk

    int kbudget = nv;
    double target = 0.0;
    bool all = false;
    if (a.mode == UNISPARSE_TOP_P) {
        all = a.param >= 1.0;
        target = a.param * tot;
    } else {
        double kk = ceil(a.param * (double)nv);
        kbudget = kk < 1.0 ? 1 : (kk > (double)nv ? nv : (int)kk);
    }
    if (p0 < P2) {
        for (int e = 0; e < E; ++e) {
            int p = p0 + e;
            uint64_t key = keys[p];
            bool sel;
            if (a.mode == UNISPARSE_TOP_P) sel = all || p == 0 || (run < target);
            else sel = p < kbudget;
            if (p < nv && sel) {
                uint32_t j = 0xffffffffu - (uint32_t)key;
                atomicOr(&bits[j >> 5], 1u << (j & 31));
            }
            run += (double)__uint_as_float((uint32_t)(key >> 32));
        }
    }
    __syncthreads();
    for (int w = tid; w < a.W; w += kSelThreads) {
        uint64_t word = (uint64_t)bits[2 * w] | ((uint64_t)bits[2 * w + 1] << 32);
        for (int m = 0; m < a.c_h; ++m)
            a.mask[((int64_t)(hc * a.c_h + m) * a.NQ + row) * a.W + w] = word;
    }
}

hipError_t launch_select(const SelectArgs &a, hipStream_t stream)
{
    int64_t n = (int64_t)a.n_heads_c * a.NQ;
    if (n == 0) return hipSuccess;
    int p2 = 1;
    while (p2 < a.NK) p2 <<= 1;       // the sort works on a power of two; sizing LDS by it lets more workgroups share a CU
    hipLaunchKernelGGL(select_kernel, dim3((unsigned)n), dim3(kSelThreads), (size_t)p2 * sizeof(uint64_t), stream, a);
    return hipGetLastError();
}

}  // namespace us

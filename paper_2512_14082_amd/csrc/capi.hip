// C ABI of the UniSparse library: argument validation, workspace carving, kernel sequencing.
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>

#include "common.h"

struct unisparse_ctx {
    int device;
    int n_cu;        // compute units: sizes the score kernel's grid rule
    void *scratch;   // this device's copy of the static workspace below (its device address)
};

// Workspace of unisparse_build_mask_static: composite tokens and block scores of one call.  Every device the
// library is loaded on holds a copy until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; kernels are given the address that call returns for the context's device.
static __device__ __align__(256) unsigned char scratch[UNISPARSE_STATIC_WORKSPACE_BYTES];

namespace {

using namespace us;

struct Geom {
    SeqTable st;
    int64_t T;
    int NQ, NK, W;
};

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Common preamble of every launching entry point: the context's device must be the one current in the calling
// thread (kernels go to the current device), and an error that earlier, unrelated work left behind in the runtime is
// cleared so that the launch checks below report this library's launches only.
unisparse_status enter(const unisparse_ctx *ctx)
{
    if (ctx == nullptr) return UNISPARSE_ERR_NULL;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return UNISPARSE_ERR_HIP;
    if (dev != ctx->device) return UNISPARSE_ERR_PARAM;
    (void)hipGetLastError();
    return UNISPARSE_OK;
}

unisparse_status check_problem(const unisparse_problem *p, Geom *g)
{
    if (p == nullptr || p->cu_seqlens == nullptr) return UNISPARSE_ERR_NULL;
    if (p->num_seqs < 1 || p->num_seqs > UNISPARSE_MAX_SEQS) return UNISPARSE_ERR_SHAPE;
    if (p->head_dim != 64 && p->head_dim != 128 && p->head_dim != 256) return UNISPARSE_ERR_UNSUPPORTED;
    if (p->block_size != 64 && p->block_size != 128) return UNISPARSE_ERR_UNSUPPORTED;
    if (p->n_heads_q < 1 || p->n_heads_kv < 1 || p->n_heads_q % p->n_heads_kv != 0) return UNISPARSE_ERR_SHAPE;
    if (!(p->softmax_scale >= 0.0f) || std::isinf(p->softmax_scale)) return UNISPARSE_ERR_PARAM;
    if (p->cu_seqlens[0] != 0) return UNISPARSE_ERR_SHAPE;
    std::memset(&g->st, 0, sizeof(g->st));
    g->st.num_seqs = p->num_seqs;
    int64_t nq = 0, nk = 0;
    for (int b = 0; b < p->num_seqs; ++b) {
        int64_t len = (int64_t)p->cu_seqlens[b + 1] - (int64_t)p->cu_seqlens[b];
        if (len < 0) return UNISPARSE_ERR_SHAPE;
        const int64_t nb = (len + p->block_size - 1) / p->block_size;     // the last block may be a shorter remainder
        g->st.cu_tok[b] = p->cu_seqlens[b];
        nq += nb;
        if (nb > nk) nk = nb;
    }
    g->st.cu_tok[p->num_seqs] = p->cu_seqlens[p->num_seqs];
    if (nk > UNISPARSE_MAX_BLOCKS_PER_SEQ) return UNISPARSE_ERR_UNSUPPORTED;
    g->T = p->cu_seqlens[p->num_seqs];
    g->NQ = (int)nq;
    g->NK = (int)nk;
    g->W = (int)((nk + 63) / 64);
    return UNISPARSE_OK;
}

// Compressed head geometry for head-level pooling (Eq. (2)) under grouped-query attention.
struct HeadGeom {
    int Hc;        // compressed query heads
    int Hkc;       // key heads the compressed queries attend
    int kpool;     // key heads averaged into one (1 = none)
};

unisparse_status check_select(const unisparse_problem *p, const unisparse_select *s, HeadGeom *hg)
{
    if (s == nullptr) return UNISPARSE_ERR_NULL;
    if (s->c_q < 1 || s->c_k < 1 || s->c_h < 1) return UNISPARSE_ERR_PARAM;
    if (p->block_size % s->c_q != 0 || p->block_size % s->c_k != 0) return UNISPARSE_ERR_SHAPE;
    int nq = p->block_size / s->c_q, nk = p->block_size / s->c_k;
    auto ok = [](int n) { return n == 4 || n == 8 || n == 16 || n == 32 || n == 64; };
    if (!ok(nq) || !ok(nk)) return UNISPARSE_ERR_UNSUPPORTED;
    if (s->mode != UNISPARSE_TOP_P && s->mode != UNISPARSE_TOP_K) return UNISPARSE_ERR_PARAM;
    if (s->pool < UNISPARSE_POOL_AVG || s->pool > UNISPARSE_POOL_STOCHASTIC) return UNISPARSE_ERR_PARAM;
    if (s->proxy_tiles < 0 || s->proxy_tiles > 2) return UNISPARSE_ERR_PARAM;
    if (s->query_pool_pass < 0 || s->query_pool_pass > 1 || s->reserved != 0) return UNISPARSE_ERR_PARAM;
    if (s->proxy_tiles == 1 && (p->head_dim != 128 || nq > 32)) return UNISPARSE_ERR_UNSUPPORTED;
    if (s->pool == UNISPARSE_POOL_STOCHASTIC && (s->rand_q == nullptr || s->rand_k == nullptr)) return UNISPARSE_ERR_NULL;
    if (s->mode == UNISPARSE_TOP_P && !(s->threshold > 0.0 && s->threshold <= 1.0)) return UNISPARSE_ERR_PARAM;
    if (s->mode == UNISPARSE_TOP_K && !(s->budget_frac > 0.0 && s->budget_frac <= 1.0)) return UNISPARSE_ERR_PARAM;
    if (p->n_heads_q % s->c_h != 0) return UNISPARSE_ERR_SHAPE;
    const int G = p->n_heads_q / p->n_heads_kv;
    hg->Hc = p->n_heads_q / s->c_h;
    if (G % s->c_h == 0) {                 // groups of c_h heads stay inside one key head
        hg->Hkc = p->n_heads_kv;
        hg->kpool = 1;
    } else if (s->c_h % G == 0) {          // a group spans c_h / G whole key heads
        hg->kpool = s->c_h / G;
        hg->Hkc = p->n_heads_kv / hg->kpool;
    } else {
        return UNISPARSE_ERR_UNSUPPORTED;
    }
    return UNISPARSE_OK;
}

unisparse_status check_tensor(const unisparse_tensor &t, int head_dim)
{
    if (t.ptr == nullptr) return UNISPARSE_ERR_NULL;
    if (((uintptr_t)t.ptr & 15) != 0 || t.stride_tok % 8 != 0 || t.stride_head % 8 != 0) return UNISPARSE_ERR_SHAPE;
    // a token row may not overlap the next one; the attention kernels address a block's rows with 32-bit byte
    // offsets, which holds for token strides up to 2^22 elements
    if (t.stride_tok < head_dim || t.stride_tok > ((int64_t)1 << 22) || t.stride_head < 0) return UNISPARSE_ERR_SHAPE;
    return UNISPARSE_OK;
}

inline TensorView view(const unisparse_tensor &t)
{
    return TensorView{reinterpret_cast<const bf16_t *>(t.ptr), t.stride_tok, t.stride_head};
}

inline float scale_log2(const unisparse_problem *p)
{
    float sc = p->softmax_scale > 0.0f ? p->softmax_scale : 1.0f / std::sqrt((float)p->head_dim);
    return sc * kLog2e;
}

// Packed offsets of the composite tokens (sequence b owns ceil(L_b / c) of them); returns their total and says
// whether every window is whole (then the offsets are cu_tok / c and the flat pooling kernel applies).
inline int64_t composite_offsets(const SeqTable &st, int c, int32_t *cu, bool *whole)
{
    int64_t tot = 0;
    *whole = true;
    for (int b = 0; b < st.num_seqs; ++b) {
        const int len = st.cu_tok[b + 1] - st.cu_tok[b];
        if (cu != nullptr) cu[b] = (int32_t)tot;
        tot += (len + c - 1) / c;
        if (len % c != 0) *whole = false;
    }
    if (cu != nullptr) cu[st.num_seqs] = (int32_t)tot;
    return tot;
}

// The one-sweep score kernel leaves a sum per composite query row and key block: S / c_q times the size of Score
// (key blocks rounded up to 64s).  It is used when that buffer stays below this size, a key block holds at least 8
// composite keys and the caller's workspace holds it.
constexpr size_t kRowSumsMaxBytes = (size_t)8 << 30;

struct WsLayout {
    size_t qt, kt, qth, kth, score, total;     // the two-sweep path
    size_t u, wgt, total_rowsums;              // the one-sweep path in addition (total_rowsums = 0: not offered)
};

WsLayout carve(const unisparse_problem *p, const unisparse_select *s, const Geom &g, const HeadGeom &hg,
               bool need_score)
{
    WsLayout w;
    size_t off = 0;
    const size_t row = (size_t)p->head_dim * 2;
    bool whole;
    const size_t Tq = (size_t)composite_offsets(g.st, s->c_q, nullptr, &whole);
    const size_t Tk = (size_t)composite_offsets(g.st, s->c_k, nullptr, &whole);
    w.qt = off; off += align256((size_t)p->n_heads_q * Tq * row);
    w.kt = off; off += align256((size_t)p->n_heads_kv * Tk * row);
    w.qth = off; if (s->c_h > 1) off += align256((size_t)hg.Hc * Tq * row);
    w.kth = off; if (hg.kpool > 1) off += align256((size_t)hg.Hkc * Tk * row);
    w.score = off; if (need_score) off += align256((size_t)hg.Hc * g.NQ * g.NK * sizeof(float));
    w.total = off;
    const size_t nq = (size_t)(p->block_size / s->c_q);
    const size_t u_bytes = (size_t)hg.Hc * g.NQ * (((size_t)g.NK + 63) / 64 * 64) * nq * sizeof(float);
    w.u = off; off += align256(u_bytes);
    w.wgt = off; off += align256((size_t)hg.Hc * g.NQ * nq * sizeof(float));
    // (with 4 composite keys per key block the sums are a quarter of the exponentials: writing and reading them
    // costs what the second sweep does)
    w.total_rowsums = u_bytes <= kRowSumsMaxBytes && p->block_size / s->c_k >= 8 ? off : 0;
    return w;
}

unisparse_status select_impl(const unisparse_problem *p, const unisparse_select *s, const Geom &g,
                             const HeadGeom &hg, float *score, uint64_t *M, hipStream_t stream,
                             const float *u = nullptr, const float *wgt = nullptr)
{
    SelectArgs sa;
    sa.score = score;
    sa.u = u;
    sa.w = wgt;
    sa.c_q = s->c_q;
    sa.mask = M;
    sa.st = g.st;
    sa.n_heads_c = hg.Hc;
    sa.c_h = s->c_h;
    sa.S = p->block_size;
    sa.causal = p->causal;
    sa.NQ = g.NQ;
    sa.NK = g.NK;
    sa.W = g.W;
    sa.mode = s->mode;
    sa.param = s->mode == UNISPARSE_TOP_P ? s->threshold : s->budget_frac;
    return launch_select(sa, stream) == hipSuccess ? UNISPARSE_OK : UNISPARSE_ERR_HIP;
}

unisparse_status attn_impl(const unisparse_ctx *ctx, const unisparse_problem *p, const Geom &g, unisparse_tensor Q, unisparse_tensor K,
                           unisparse_tensor V, const uint64_t *M, unisparse_tensor O, float *lse,
                           hipStream_t stream, void *sched = nullptr, size_t sched_bytes = 0)
{
    unisparse_status st;
    if ((st = check_tensor(Q, p->head_dim)) != UNISPARSE_OK) return st;
    if ((st = check_tensor(K, p->head_dim)) != UNISPARSE_OK) return st;
    if ((st = check_tensor(V, p->head_dim)) != UNISPARSE_OK) return st;
    if ((st = check_tensor(O, p->head_dim)) != UNISPARSE_OK) return st;
    if ((st = enter(ctx)) != UNISPARSE_OK) return st;
    AttnArgs a;
    a.q = view(Q);
    a.k = view(K);
    a.v = view(V);
    a.o = reinterpret_cast<bf16_t *>(O.ptr);
    a.o_stride_tok = O.stride_tok;
    a.o_stride_head = O.stride_head;
    a.mask = M;
    a.lse = lse;
    a.st = g.st;
    a.n_heads_q = p->n_heads_q;
    a.n_heads_kv = p->n_heads_kv;
    a.S = p->block_size;
    a.head_dim = p->head_dim;
    a.causal = p->causal;
    a.NQ = g.NQ;
    a.W = g.W;
    a.total_tokens = g.T;
    a.scale_log2 = scale_log2(p);
    a.sched = reinterpret_cast<int32_t *>(sched);
    a.sched_bytes = (int64_t)sched_bytes;
    return launch_attention(a, stream) == hipSuccess ? UNISPARSE_OK : UNISPARSE_ERR_HIP;
}

}  // namespace

extern "C" {

unisparse_status unisparse_create(unisparse_ctx **ctx, int device)
{
    if (ctx == nullptr) return UNISPARSE_ERR_NULL;
    *ctx = nullptr;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return UNISPARSE_ERR_HIP;
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return UNISPARSE_ERR_UNSUPPORTED;
    // the work orders of the kernels deal workgroups to kNumXcd dies with a private L2 each
    int n_xcd = 0;
    if (hipDeviceGetAttribute(&n_xcd, hipDeviceAttributeNumberOfXccs, device) == hipSuccess && n_xcd > 0 &&
        n_xcd != kNumXcd)
        return UNISPARSE_ERR_UNSUPPORTED;
    (void)hipGetLastError();
    // device address of this device's copy of the static workspace (looked up with that device current)
    int prev = -1;
    if (hipGetDevice(&prev) != hipSuccess) return UNISPARSE_ERR_HIP;
    if (prev != device && hipSetDevice(device) != hipSuccess) return UNISPARSE_ERR_HIP;
    void *scratch_ptr = nullptr;
    const hipError_t se = hipGetSymbolAddress(&scratch_ptr, HIP_SYMBOL(scratch));
    if (prev != device && hipSetDevice(prev) != hipSuccess) return UNISPARSE_ERR_HIP;
    if (se != hipSuccess || scratch_ptr == nullptr) return UNISPARSE_ERR_HIP;
    unisparse_ctx *c = new (std::nothrow) unisparse_ctx;
    if (c == nullptr) return UNISPARSE_ERR_HIP;
    c->scratch = scratch_ptr;
    c->device = device;
    c->n_cu = prop.multiProcessorCount;
    *ctx = c;
    return UNISPARSE_OK;
}

void unisparse_destroy(unisparse_ctx *ctx) { delete ctx; }

const char *unisparse_status_string(unisparse_status s)
{
    switch (s) {
        case UNISPARSE_OK: return "ok";
        case UNISPARSE_ERR_NULL: return "null pointer";
        case UNISPARSE_ERR_SHAPE: return "invalid shape";
        case UNISPARSE_ERR_PARAM: return "invalid parameter";
        case UNISPARSE_ERR_UNSUPPORTED: return "unsupported configuration";
        case UNISPARSE_ERR_WORKSPACE: return "workspace too small";
        case UNISPARSE_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

size_t unisparse_mask_row_words(const unisparse_problem *p)
{
    Geom g;
    return check_problem(p, &g) == UNISPARSE_OK ? (size_t)g.W : 0;
}

size_t unisparse_mask_words(const unisparse_problem *p)
{
    Geom g;
    return check_problem(p, &g) == UNISPARSE_OK ? (size_t)p->n_heads_q * g.NQ * g.W : 0;
}

size_t unisparse_score_elems(const unisparse_problem *p, const unisparse_select *s)
{
    Geom g;
    HeadGeom hg;
    if (check_problem(p, &g) != UNISPARSE_OK || check_select(p, s, &hg) != UNISPARSE_OK) return 0;
    return (size_t)hg.Hc * g.NQ * g.NK;
}

size_t unisparse_workspace_bytes(const unisparse_problem *p, const unisparse_select *s)
{
    Geom g;
    HeadGeom hg;
    if (check_problem(p, &g) != UNISPARSE_OK || check_select(p, s, &hg) != UNISPARSE_OK) return 0;
    // (also enough for unisparse_sparse_attn_ws, so that unisparse_attn can hand the same buffer on)
    const WsLayout w = carve(p, s, g, hg, true);
    const size_t build = w.total_rowsums != 0 ? w.total_rowsums : w.total;
    const size_t attn = attention_sched_bytes(p->n_heads_q, p->n_heads_kv, g.NQ);
    return (build > attn ? build : attn) + 256;
}

size_t unisparse_workspace_bytes_min(const unisparse_problem *p, const unisparse_select *s)
{
    Geom g;
    HeadGeom hg;
    if (check_problem(p, &g) != UNISPARSE_OK || check_select(p, s, &hg) != UNISPARSE_OK) return 0;
    const size_t build = carve(p, s, g, hg, true).total, attn = attention_sched_bytes(p->n_heads_q, p->n_heads_kv, g.NQ);
    return (build > attn ? build : attn) + 256;
}

unisparse_status unisparse_avgpool_seq(unisparse_ctx *ctx, unisparse_tensor x, int32_t n_heads, int64_t total_tokens,
                                       int32_t c, void *out, void *stream)
{
    if (ctx == nullptr || out == nullptr) return UNISPARSE_ERR_NULL;
    unisparse_status st = check_tensor(x, UNISPARSE_HEAD_DIM);
    if (st != UNISPARSE_OK) return st;
    if (n_heads < 1 || total_tokens < 0 || c < 1 || total_tokens % c != 0) return UNISPARSE_ERR_SHAPE;
    if (((uintptr_t)out & 15) != 0) return UNISPARSE_ERR_SHAPE;
    if ((st = enter(ctx)) != UNISPARSE_OK) return st;
    hipError_t e = launch_avgpool_seq(view(x), n_heads, total_tokens, c, UNISPARSE_POOL_AVG, UNISPARSE_HEAD_DIM,
                                      reinterpret_cast<bf16_t *>(out),
                                      (hipStream_t)stream);
    return e == hipSuccess ? UNISPARSE_OK : UNISPARSE_ERR_HIP;
}

unisparse_status unisparse_pool_seq_varlen(unisparse_ctx *ctx, const unisparse_problem *p, unisparse_tensor x,
                                           int32_t n_heads, int32_t c, int32_t pool, const float *rand, void *out,
                                           void *stream)
{
    if (ctx == nullptr || out == nullptr) return UNISPARSE_ERR_NULL;
    Geom g;
    unisparse_status st;
    if ((st = check_problem(p, &g)) != UNISPARSE_OK) return st;
    if ((st = check_tensor(x, p->head_dim)) != UNISPARSE_OK) return st;
    if (n_heads < 1 || c < 1) return UNISPARSE_ERR_SHAPE;
    if (pool < UNISPARSE_POOL_AVG || pool > UNISPARSE_POOL_STOCHASTIC) return UNISPARSE_ERR_PARAM;
    if (((uintptr_t)out & 15) != 0) return UNISPARSE_ERR_SHAPE;
    if (pool == UNISPARSE_POOL_STOCHASTIC && rand == nullptr) return UNISPARSE_ERR_NULL;
    if (pool == UNISPARSE_POOL_STOCHASTIC && c > 32) return UNISPARSE_ERR_UNSUPPORTED;
    if ((st = enter(ctx)) != UNISPARSE_OK) return st;
    hipError_t e = pool == UNISPARSE_POOL_STOCHASTIC
                       ? launch_stochpool_seq_varlen(view(x), n_heads, g.st, c, p->head_dim, rand, reinterpret_cast<bf16_t *>(out),
                                                     (hipStream_t)stream)
                       : launch_avgpool_seq_varlen(view(x), n_heads, g.st, c, pool, p->head_dim, reinterpret_cast<bf16_t *>(out),
                                                   (hipStream_t)stream);
    return e == hipSuccess ? UNISPARSE_OK : UNISPARSE_ERR_HIP;
}

unisparse_status unisparse_build_mask(unisparse_ctx *ctx, const unisparse_problem *p, const unisparse_select *s,
                                      unisparse_tensor Q, unisparse_tensor K, void *workspace,
                                      size_t workspace_bytes, uint64_t *M, float *score, void *stream_)
{
    if (ctx == nullptr || M == nullptr || workspace == nullptr) return UNISPARSE_ERR_NULL;
    if (((uintptr_t)M & 7) != 0) return UNISPARSE_ERR_SHAPE;          // mask words are 8-byte loads and stores
    Geom g;
    HeadGeom hg;
    unisparse_status st;
    if ((st = check_problem(p, &g)) != UNISPARSE_OK) return st;
    if ((st = check_select(p, s, &hg)) != UNISPARSE_OK) return st;
    if ((st = check_tensor(Q, p->head_dim)) != UNISPARSE_OK) return st;
    if ((st = check_tensor(K, p->head_dim)) != UNISPARSE_OK) return st;
    const WsLayout w = carve(p, s, g, hg, score == nullptr);
    unsigned char *base = reinterpret_cast<unsigned char *>(align256((size_t)(uintptr_t)workspace));
    const size_t lead = (size_t)(base - reinterpret_cast<unsigned char *>(workspace));
    if (workspace_bytes < w.total + lead) return UNISPARSE_ERR_WORKSPACE;
    const bool rowsums = w.total_rowsums != 0 && workspace_bytes >= w.total_rowsums + lead;
    if ((st = enter(ctx)) != UNISPARSE_OK) return st;
    if (g.T == 0) return UNISPARSE_OK;
    hipStream_t stream = (hipStream_t)stream_;

    bf16_t *qt = reinterpret_cast<bf16_t *>(base + w.qt);
    bf16_t *kt = reinterpret_cast<bf16_t *>(base + w.kt);
    ProxyArgs pa;
    bool whole_q, whole_k;
    const int64_t Tq = composite_offsets(g.st, s->c_q, pa.cu_cq, &whole_q);
    const int64_t Tk = composite_offsets(g.st, s->c_k, pa.cu_ck, &whole_k);
    // windows never straddle sequences; with whole windows everywhere the packed batch pools as one flat array
    const bool stoch = s->pool == UNISPARSE_POOL_STOCHASTIC;
    const int d = p->head_dim;
    // averaged queries that no head pooling follows are formed by the score kernel as it loads them
    const bool q_on_the_fly = s->pool == UNISPARSE_POOL_AVG && s->c_h == 1 && s->query_pool_pass == 0;
    hipError_t pe = q_on_the_fly ? hipSuccess
                    : stoch      ? launch_stochpool_seq_varlen(view(Q), p->n_heads_q, g.st, s->c_q, d, s->rand_q, qt, stream)
                    : whole_q    ? launch_avgpool_seq(view(Q), p->n_heads_q, g.T, s->c_q, s->pool, d, qt, stream)
                                 : launch_avgpool_seq_varlen(view(Q), p->n_heads_q, g.st, s->c_q, s->pool, d, qt, stream);
    if (pe != hipSuccess) return UNISPARSE_ERR_HIP;
    pe = stoch     ? launch_stochpool_seq_varlen(view(K), p->n_heads_kv, g.st, s->c_k, d, s->rand_k, kt, stream)
         : whole_k ? launch_avgpool_seq(view(K), p->n_heads_kv, g.T, s->c_k, s->pool, d, kt, stream)
                   : launch_avgpool_seq_varlen(view(K), p->n_heads_kv, g.st, s->c_k, s->pool, d, kt, stream);
    if (pe != hipSuccess) return UNISPARSE_ERR_HIP;
    if (s->c_h > 1) {
        bf16_t *qth = reinterpret_cast<bf16_t *>(base + w.qth);
        if (launch_avgpool_head(qt, p->n_heads_q, Tq, s->c_h, d, qth, stream) != hipSuccess)
            return UNISPARSE_ERR_HIP;
        qt = qth;
        if (hg.kpool > 1) {
            bf16_t *kth = reinterpret_cast<bf16_t *>(base + w.kth);
            if (launch_avgpool_head(kt, p->n_heads_kv, Tk, hg.kpool, d, kth, stream) != hipSuccess)
                return UNISPARSE_ERR_HIP;
            kt = kth;
        }
    }
    float *sc = score != nullptr ? score : reinterpret_cast<float *>(base + w.score);
    pa.qt = q_on_the_fly ? nullptr : qt;
    pa.q_src = view(Q);
    pa.kt = kt;
    pa.score = sc;
    pa.st = g.st;
    pa.n_heads_q = hg.Hc;
    pa.n_heads_kv = hg.Hkc;
    pa.S = p->block_size;
    pa.head_dim = p->head_dim;
    pa.tiles = s->proxy_tiles;
    pa.c_q = s->c_q;
    pa.c_k = s->c_k;
    pa.causal = p->causal;
    pa.NQ = g.NQ;
    pa.NK = g.NK;
    pa.scale_log2 = scale_log2(p);
    pa.n_cu = ctx->n_cu;
    pa.u = rowsums ? reinterpret_cast<float *>(base + w.u) : nullptr;
    pa.w = rowsums ? reinterpret_cast<float *>(base + w.wgt) : nullptr;
    if (launch_proxy_scores(pa, stream) != hipSuccess) return UNISPARSE_ERR_HIP;
    return select_impl(p, s, g, hg, sc, M, stream, pa.u, pa.w);
}

unisparse_status unisparse_build_mask_static(unisparse_ctx *ctx, const unisparse_problem *p,
                                             const unisparse_select *s, unisparse_tensor Q, unisparse_tensor K,
                                             uint64_t *M, void *stream)
{
    if (ctx == nullptr) return UNISPARSE_ERR_NULL;
    const size_t need = unisparse_workspace_bytes_min(p, s);  // 0 for an invalid problem: build_mask reports which
    if (need > (size_t)UNISPARSE_STATIC_WORKSPACE_BYTES) return UNISPARSE_ERR_WORKSPACE;
    return unisparse_build_mask(ctx, p, s, Q, K, ctx->scratch, (size_t)UNISPARSE_STATIC_WORKSPACE_BYTES, M, nullptr,
                                stream);
}

unisparse_status unisparse_select_blocks(unisparse_ctx *ctx, const unisparse_problem *p, const unisparse_select *s,
                                         float *score, uint64_t *M, void *stream)
{
    if (ctx == nullptr || score == nullptr || M == nullptr) return UNISPARSE_ERR_NULL;
    if (((uintptr_t)M & 7) != 0) return UNISPARSE_ERR_SHAPE;          // mask words are 8-byte loads and stores
    Geom g;
    HeadGeom hg;
    unisparse_status st;
    if ((st = check_problem(p, &g)) != UNISPARSE_OK) return st;
    if ((st = check_select(p, s, &hg)) != UNISPARSE_OK) return st;
    if ((st = enter(ctx)) != UNISPARSE_OK) return st;
    if (g.T == 0) return UNISPARSE_OK;
    return select_impl(p, s, g, hg, score, M, (hipStream_t)stream);
}

unisparse_status unisparse_sparse_attn(unisparse_ctx *ctx, const unisparse_problem *p, unisparse_tensor Q,
                                       unisparse_tensor K, unisparse_tensor V, const uint64_t *M,
                                       unisparse_tensor O, float *lse, void *stream)
{
    if (ctx == nullptr || M == nullptr) return UNISPARSE_ERR_NULL;
    if (((uintptr_t)M & 7) != 0) return UNISPARSE_ERR_SHAPE;          // mask words are 8-byte loads and stores
    Geom g;
    unisparse_status st;
    if ((st = check_problem(p, &g)) != UNISPARSE_OK) return st;
    if (g.T == 0) return check_tensor(Q, p->head_dim);
    return attn_impl(ctx, p, g, Q, K, V, M, O, lse, (hipStream_t)stream);
}

size_t unisparse_attn_workspace_bytes(const unisparse_problem *p)
{
    Geom g;
    if (check_problem(p, &g) != UNISPARSE_OK) return 0;
    return attention_sched_bytes(p->n_heads_q, p->n_heads_kv, g.NQ) + 256;
}

unisparse_status unisparse_sparse_attn_ws(unisparse_ctx *ctx, const unisparse_problem *p, unisparse_tensor Q,
                                          unisparse_tensor K, unisparse_tensor V, const uint64_t *M,
                                          unisparse_tensor O, float *lse, void *workspace, size_t workspace_bytes,
                                          void *stream)
{
    if (ctx == nullptr || M == nullptr) return UNISPARSE_ERR_NULL;
    if (((uintptr_t)M & 7) != 0) return UNISPARSE_ERR_SHAPE;          // mask words are 8-byte loads and stores
    Geom g;
    unisparse_status st;
    if ((st = check_problem(p, &g)) != UNISPARSE_OK) return st;
    unsigned char *base = nullptr;
    size_t avail = 0;
    if (workspace != nullptr) {
        base = reinterpret_cast<unsigned char *>(align256((size_t)(uintptr_t)workspace));
        const size_t lead = (size_t)(base - reinterpret_cast<unsigned char *>(workspace));
        const size_t need = attention_sched_bytes(p->n_heads_q, p->n_heads_kv, g.NQ);
        if (workspace_bytes < need + lead) return UNISPARSE_ERR_WORKSPACE;
        avail = workspace_bytes - lead;
    }
    if (g.T == 0) return check_tensor(Q, p->head_dim);
    return attn_impl(ctx, p, g, Q, K, V, M, O, lse, (hipStream_t)stream, base, avail);
}

unisparse_status unisparse_full_attn(unisparse_ctx *ctx, const unisparse_problem *p, unisparse_tensor Q,
                                     unisparse_tensor K, unisparse_tensor V, unisparse_tensor O, float *lse,
                                     void *stream)
{
    if (ctx == nullptr) return UNISPARSE_ERR_NULL;
    Geom g;
    unisparse_status st;
    if ((st = check_problem(p, &g)) != UNISPARSE_OK) return st;
    if (g.T == 0) return check_tensor(Q, p->head_dim);
    return attn_impl(ctx, p, g, Q, K, V, nullptr, O, lse, (hipStream_t)stream);
}

unisparse_status unisparse_attn(unisparse_ctx *ctx, const unisparse_problem *p, const unisparse_select *s,
                                unisparse_tensor Q, unisparse_tensor K, unisparse_tensor V, void *workspace,
                                size_t workspace_bytes, uint64_t *M, unisparse_tensor O, float *lse, void *stream)
{
    unisparse_status st;
    if (p == nullptr) return UNISPARSE_ERR_NULL;
    if ((st = check_tensor(V, p->head_dim)) != UNISPARSE_OK) return st;
    if ((st = check_tensor(O, p->head_dim)) != UNISPARSE_OK) return st;
    if (workspace_bytes < unisparse_attn_workspace_bytes(p)) return UNISPARSE_ERR_WORKSPACE;
    st = unisparse_build_mask(ctx, p, s, Q, K, workspace, workspace_bytes, M, nullptr, stream);
    if (st != UNISPARSE_OK) return st;
    // the mask is built: the workspace is free again and serves the attention kernel's work order
    return unisparse_sparse_attn_ws(ctx, p, Q, K, V, M, O, lse, workspace, workspace_bytes, stream);
}

}  // extern "C"

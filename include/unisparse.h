/*
 * unisparse.h -- C ABI of the UniSparse hot path for AMD MI355X (gfx950).
 *
 * UniSparse (arXiv 2512.14082) builds a block-sparse attention mask M from a cheap proxy
 * computed on "composite tokens" (average-pooled queries and keys) and then runs
 * block-sparse attention over the selected (query block, key block) pairs:
 *
 *   Alg. 1 step 1  sequence / head average pooling                     Eq. (1), Eq. (2)
 *   Alg. 1 step 2  compressed logits Q~ K~^T / sqrt(d_k), row softmax  Sec. 4.3
 *   Alg. 1 step 3  block aggregation Score(i, j)                       Eq. (3), Eq. (4)
 *   Alg. 1 step 4  causal cut + Top-P selection (or a fixed budget)    Eq. (5)
 *   Alg. 1 step 5  block-sparse attention with mask M                  Sec. 2.2
 *
 * Conventions shared by every call
 * --------------------------------
 * - All tensor pointers are DEVICE pointers unless a comment says HOST.  The caller owns
 *   every buffer (inputs, outputs, workspace).  The library allocates no device memory,
 *   never synchronises the device or a stream, and enqueues work only on the stream given.
 * - Element type of Q, K, V, O and of the composite tokens is bf16 (2 bytes).  head_dim d = 64, 128 or 256
 *   (128 is the dimension of every model the paper measures).
 * - A problem is a packed batch of B sequences ("varlen"): tokens of all sequences are
 *   concatenated along the token axis, sequence b owning tokens [cu_seqlens[b], cu_seqlens[b+1]).
 *   Sequences never interact.  A length that is not a multiple of block_size gives a shorter last block
 *   (the block index sets of Eq. (4) clipped to the sequence) and, when c does not divide it, a partial last
 *   pooling window that averages the tokens that exist.
 * - Grouped-query attention: query head h uses key/value head h / (n_heads_q / n_heads_kv).
 * - Query-block rows are numbered over the packed batch: row r = (blocks of earlier sequences)
 *   + local block index i.  NQ = sum_b ceil(L_b / block_size) rows, NK = max_b ceil(L_b / block_size).
 * - Mask layout: uint64 M[n_heads_q][NQ][W], W = ceil(NK / 64).  Bit (j % 64) of word j / 64 of
 *   row r says whether query block r attends key block j *of its own sequence*.  Bits with
 *   j > i under causality and bits with j >= N_b are always written as 0 by build_mask and
 *   are ignored (treated as 0) by sparse_attn.
 * - Errors: every call validates its arguments on the host before launching anything and
 *   returns a status; on error no kernel is launched and no output is touched.  Launch
 *   failures reported by HIP map to UNISPARSE_ERR_HIP; an error that earlier work of the caller left pending in
 *   the runtime (hipGetLastError) is cleared on entry and not reported.
 * - stream arguments are hipStream_t values passed as void* (NULL = the null stream).  Work goes to the device
 *   the context was created for; it must be the device current in the calling thread and the stream's device
 *   (UNISPARSE_ERR_PARAM if another device is current).
 * - The first launch of a kernel on a device raises that kernel's dynamic-LDS limit (a host-side HIP call), so a
 *   stream capture should follow one ordinary call of the same entry point with the same configuration; after
 *   that the calls are launches only - no allocation, no memset, no synchronisation.
 * - Calls may come from several host threads; concurrent calls that share an output or workspace buffer race.
 */
#ifndef UNISPARSE_H
#define UNISPARSE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define UNISPARSE_MAX_SEQS 64      /* sequences per packed batch */
#define UNISPARSE_HEAD_DIM 128       /* the default head dimension (and that of unisparse_avgpool_seq) */
#define UNISPARSE_MAX_BLOCKS_PER_SEQ 4096   /* NK limit (selection keeps one row in a wavefront's registers) */

typedef struct unisparse_ctx unisparse_ctx;   /* opaque; the device it was created for and its compute-unit count */

typedef enum {
    UNISPARSE_OK = 0,
    UNISPARSE_ERR_NULL = 1,          /* a required pointer is NULL */
    UNISPARSE_ERR_SHAPE = 2,         /* c not dividing block_size, head counts, misaligned tensors ... */
    UNISPARSE_ERR_PARAM = 3,         /* threshold / budget outside (0, 1], unknown mode ... */
    UNISPARSE_ERR_UNSUPPORTED = 4,   /* valid request this build has no kernel for */
    UNISPARSE_ERR_WORKSPACE = 5,     /* workspace smaller than the call's documented minimum */
    UNISPARSE_ERR_HIP = 6            /* HIP runtime reported an error */
} unisparse_status;

/* Problem geometry.  cu_seqlens is a HOST pointer to num_seqs + 1 int32 (cu[0] = 0); it is read
 * during the call and not retained. */
typedef struct {
    int32_t num_seqs;                /* B, 1 .. UNISPARSE_MAX_SEQS */
    const int32_t *cu_seqlens;       /* HOST */
    int32_t n_heads_q;               /* H */
    int32_t n_heads_kv;              /* H_kv, divides H */
    int32_t head_dim;                /* d: 64, 128 or 256 */
    int32_t block_size;              /* S: 64 or 128 */
    int32_t causal;                  /* 0 / 1 */
    float softmax_scale;             /* 0 -> 1 / sqrt(head_dim) */
} unisparse_problem;

/* A [tokens, heads, head_dim] view with token / head strides in elements; the last dimension is contiguous and
 * 16-byte aligned.  Covers both token-major and head-major storage.  Strides are multiples of 8,
 * head_dim <= stride_tok <= 2^22, stride_head >= 0 (UNISPARSE_ERR_SHAPE otherwise); that heads and tokens of an
 * output view do not overlap is the caller's business. */
typedef struct {
    void *ptr;                       /* DEVICE, bf16 */
    int64_t stride_tok;
    int64_t stride_head;
} unisparse_tensor;

#define UNISPARSE_POOL_AVG 0
#define UNISPARSE_POOL_MAX 1
#define UNISPARSE_POOL_STOCHASTIC 2

#define UNISPARSE_TOP_P 0            /* cumulative-score threshold, Eq. (5) */
#define UNISPARSE_TOP_K 1            /* fixed budget: keep max(1, ceil(f * n_valid)) blocks per row */

/* Selection parameters (the inputs of Alg. 1 besides Q, K, V and S). */
typedef struct {
    int32_t c_q, c_k;                /* sequence compression factors; block_size / c must be 4, 8, 16, 32 or 64 */
    int32_t c_h;                     /* head compression factor; must divide H.  Groups of c_h query heads
                                        share one mask (Eq. (2) and the broadcast of Alg. 1) */
    int32_t mode;                    /* UNISPARSE_TOP_P or UNISPARSE_TOP_K */
    double threshold;                /* P in (0, 1]; P >= 1 keeps every valid block */
    double budget_frac;              /* f in (0, 1] */
    int32_t pool;                    /* UNISPARSE_POOL_AVG (Eq. (1), the method), or one of the alternatives of the
                                        "Compression Strategy" ablation: UNISPARSE_POOL_MAX (channel-wise maximum of
                                        the window) or UNISPARSE_POOL_STOCHASTIC (one token of the window, drawn by
                                        its share of the window's L2 norms; see unisparse_pool_seq_varlen) */
    int32_t proxy_tiles;             /* tuning: 32-row MFMA tiles per wavefront of the score kernel.  0 = chosen by the
                                        library (2, or 1 when the problem yields few workgroups: high compression
                                        ratios, compressed heads); 1 or 2 force it.  1 exists for head_dim 128 and
                                        block_size / c_q <= 32 (UNISPARSE_ERR_UNSUPPORTED otherwise) */
    int32_t query_pool_pass;         /* tuning: 0 = the score kernel pools the queries itself as it loads them (Eq. (1)
                                        on the fly, the same arithmetic; done for average pooling without head
                                        compression), 1 = always in a pass of their own, as the keys are */
    int32_t reserved;                /* must be 0 */
    const float *rand_q;             /* UNISPARSE_POOL_STOCHASTIC only (else ignored): DEVICE uniform numbers in [0, 1), */
    const float *rand_k;             /* one per composite token: rand_q [H][sum_b ceil(L_b/c_q)],
                                        rand_k [H_kv][sum_b ceil(L_b/c_k)], laid out like the composite tokens.
                                        Borrowed for the call; the library draws no random numbers itself. */
} unisparse_select;

unisparse_status unisparse_create(unisparse_ctx **ctx, int device);
void unisparse_destroy(unisparse_ctx *ctx);
const char *unisparse_status_string(unisparse_status s);

/* Sizes the caller needs for its allocations.  All return 0 for an invalid problem. */
size_t unisparse_mask_row_words(const unisparse_problem *p);             /* W                         */
size_t unisparse_mask_words(const unisparse_problem *p);                 /* H * NQ * W  (uint64)      */
size_t unisparse_score_elems(const unisparse_problem *p, const unisparse_select *s); /* (H/c_h)*NQ*NK floats */
/* Workspace of unisparse_build_mask: _bytes() lets it run the fast form of the score computation (one sweep over
 * the composite keys, with a sum per composite query row and key block parked in the workspace: S / c_q times the
 * size of the scores; equal to _bytes_min() when that buffer would pass 8 GiB or when S / c_k < 8, where the sums
 * would cost what they save), _bytes_min() is the least it accepts (two sweeps, nothing parked). */
size_t unisparse_workspace_bytes(const unisparse_problem *p, const unisparse_select *s);
size_t unisparse_workspace_bytes_min(const unisparse_problem *p, const unisparse_select *s);

/*
 * Sequence-level average pooling, Eq. (1): out[h][t'][:] = bf16( (1/c) * sum_{m<c} x[t'c + m][h][:] ),
 * fp32 sum in token order, one rounding to bf16 (nearest even).
 *   x       : [total_tokens, n_heads, 128] view
 *   out     : DEVICE bf16 [n_heads][total_tokens / c][128], contiguous
 * total_tokens must be a multiple of c (windows then never straddle sequences whose lengths are
 * multiples of c).
 */
unisparse_status unisparse_avgpool_seq(unisparse_ctx *ctx, unisparse_tensor x, int32_t n_heads,
                                       int64_t total_tokens, int32_t c, void *out, void *stream);

/*
 * Eq. (1) for the packed batch of a problem whose lengths need not be multiples of c: sequence b yields
 * ceil(L_b / c) composite tokens, windows never straddle sequences, and a last window that the sequence
 * does not fill averages the tokens that exist (divisor = their number).  pool = UNISPARSE_POOL_MAX takes
 * the channel-wise maximum of the same windows instead.  pool = UNISPARSE_POOL_STOCHASTIC copies ONE token
 * of the window: token m with probability w_m / sum_m' w_m', w_m = the L2 norm of the token's 128 channels,
 * drawn by inversion of rand[h][t'] -- the first m whose running sum w_0 + ... + w_m exceeds
 * rand * (w_0 + ... + w_{cnt-1}), the last token of the window if none does.  That comparison is taken in
 * fp32 (squares accumulated by fused multiply-adds in channel order, correctly rounded square root, sums in
 * token order), so equal inputs and equal random numbers give equal choices everywhere; c <= 32.
 * This is what build_mask applies internally.  Only num_seqs and cu_seqlens of the problem are used for
 * the geometry.
 *   x    : [total_tokens, n_heads, d] view (d = head_dim of the problem)
 *   rand : DEVICE float [n_heads][sum_b ceil(L_b / c)] in [0, 1); read only for UNISPARSE_POOL_STOCHASTIC
 *          (NULL otherwise); UNISPARSE_ERR_NULL if missing
 *   out  : DEVICE bf16 [n_heads][sum_b ceil(L_b / c)][d], contiguous
 */
unisparse_status unisparse_pool_seq_varlen(unisparse_ctx *ctx, const unisparse_problem *p, unisparse_tensor x,
                                           int32_t n_heads, int32_t c, int32_t pool, const float *rand, void *out,
                                           void *stream);

/*
 * Alg. 1 steps 1-4: composite tokens, compressed softmax scores, block aggregation, selection.
 *   Q : [T, H, d] view, K : [T, H_kv, d] view
 *   workspace : DEVICE scratch of at least unisparse_workspace_bytes_min() bytes, 256-byte aligned.  With
 *           unisparse_workspace_bytes() or more the scores are computed in one sweep over the composite keys,
 *           below that in two; the two forms agree to rounding (both normalise by the same row sums, added in a
 *           different order), so a score within a few ulp of the selection cut may fall on either side of it.
 *   M     : out, uint64 [H][NQ][W]
 *   score : out, optional (may be NULL), float [H / c_h][NQ][NK]; Score(i, j) of Eq. (3) for valid j,
 *           0 elsewhere.  When NULL the scores live in the workspace.
 * Causal problems exclude, inside the compressed softmax, composite keys whose window starts after
 * the last token of the composite query's window, and drop key blocks j > i before selection.
 */
unisparse_status unisparse_build_mask(unisparse_ctx *ctx, const unisparse_problem *p,
                                      const unisparse_select *s, unisparse_tensor Q, unisparse_tensor K,
                                      void *workspace, size_t workspace_bytes, uint64_t *M, float *score,
                                      void *stream);

/*
 * unisparse_build_mask for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the same kernels, with the composite tokens and the block
 * scores in a workspace that is part of the library's device image instead of a caller's buffer.  The call
 * allocates nothing and frees nothing.
 *   limit : unisparse_workspace_bytes_min(p, s) <= UNISPARSE_STATIC_WORKSPACE_BYTES (64 MiB; e.g. GQA 32/8 at
 *           32K tokens with c = 8 needs 48 MiB), else UNISPARSE_ERR_WORKSPACE and nothing is launched.  The
 *           result is that of unisparse_build_mask with a workspace of UNISPARSE_STATIC_WORKSPACE_BYTES.
 *   M     : out, uint64 [H][NQ][W] as for unisparse_build_mask; the scores are not returned
 * Every device keeps one copy of that workspace for the life of the process, shared by all contexts and all
 * calls on the device: it holds the previous call's contents (nothing in it needs clearing - every value read is
 * written earlier in the same call), and calls that overlap in time on one device race on it.
 */
#define UNISPARSE_STATIC_WORKSPACE_BYTES (64u << 20)
unisparse_status unisparse_build_mask_static(unisparse_ctx *ctx, const unisparse_problem *p,
                                             const unisparse_select *s, unisparse_tensor Q, unisparse_tensor K,
                                             uint64_t *M, void *stream);

/*
 * Selection only (Alg. 1 step 4) on caller-provided scores, e.g. to re-select with another threshold.
 *   score : float [H / c_h][NQ][NK] (read; entries outside a row's valid set are overwritten with 0)
 */
unisparse_status unisparse_select_blocks(unisparse_ctx *ctx, const unisparse_problem *p,
                                         const unisparse_select *s, float *score, uint64_t *M, void *stream);

/*
 * Alg. 1 step 5 / Sec. 2.2: O = softmax(Q K^T * scale + M~) V over the selected blocks only, with
 * token-level causality inside the diagonal block.
 *   Q, O : [T, H, d] views;  K, V : [T, H_kv, d] views;  M as above
 *   lse  : optional (may be NULL), float [H][T]: natural-log sum of exponentials of the visible logits
 * A query row whose mask row is empty gets O = 0 and lse = -inf.
 */
unisparse_status unisparse_sparse_attn(unisparse_ctx *ctx, const unisparse_problem *p, unisparse_tensor Q,
                                       unisparse_tensor K, unisparse_tensor V, const uint64_t *M,
                                       unisparse_tensor O, float *lse, void *stream);

/*
 * The same with scratch memory for a mask-dependent work order: before the attention kernel, a small kernel ranks
 * every head's query-block rows by their number of selected blocks, and workgroups that run side by side then take
 * rows of neighbouring rank of one head (or two) instead of neighbouring index - they have about the same
 * length, so they stay together on the K/V blocks they share and the L2 serves them (about half the traffic behind
 * the L2 and 3 % less time on the 128K configuration).  O and lse are bit-identical to unisparse_sparse_attn: only the
 * order in which rows are worked on changes, and it depends on nothing but the mask.
 *   workspace : DEVICE scratch of at least unisparse_attn_workspace_bytes(p) bytes (the workspace of a finished
 *               unisparse_build_mask of the same problem is large enough and may be reused); NULL = no ranking,
 *               exactly unisparse_sparse_attn.  UNISPARSE_ERR_WORKSPACE if too small.
 * Problems with more than 8192 query-block rows, and problems of at most 512 (head, query-block row) pairs - which
 * the device works on all at once - run in the default order.
 */
size_t unisparse_attn_workspace_bytes(const unisparse_problem *p);
unisparse_status unisparse_sparse_attn_ws(unisparse_ctx *ctx, const unisparse_problem *p, unisparse_tensor Q,
                                          unisparse_tensor K, unisparse_tensor V, const uint64_t *M,
                                          unisparse_tensor O, float *lse, void *workspace, size_t workspace_bytes,
                                          void *stream);

/* Dense attention (Sec. 2.1): the same kernel visiting every valid block.  The speedup baseline.  (The result does
 * not depend on block_size, which only has to be a valid one.) */
unisparse_status unisparse_full_attn(unisparse_ctx *ctx, const unisparse_problem *p, unisparse_tensor Q,
                                     unisparse_tensor K, unisparse_tensor V, unisparse_tensor O, float *lse,
                                     void *stream);

/*
 * The paper's one-call interface (Sec. 5): build_mask followed by sparse_attn_ws (which reuses the workspace) on
 * the same stream.
 *   workspace : as for unisparse_build_mask (at least unisparse_workspace_bytes_min(); unisparse_workspace_bytes()
 *               for the one-sweep score computation); both sizes cover the row ranking of sparse_attn_ws
 *   M : scratch/out uint64 [H][NQ][W] (the mask that was used, left for inspection)
 */
unisparse_status unisparse_attn(unisparse_ctx *ctx, const unisparse_problem *p, const unisparse_select *s,
                                unisparse_tensor Q, unisparse_tensor K, unisparse_tensor V, void *workspace,
                                size_t workspace_bytes, uint64_t *M, unisparse_tensor O, float *lse,
                                void *stream);

#ifdef __cplusplus
}
#endif
#endif /* UNISPARSE_H */

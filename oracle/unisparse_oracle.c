/*
 * UniSparse reference oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct CPU statement of what the UniSparse hot path
 * computes (composite-token proxy -> block mask -> block-sparse attention),
 * written from the paper's definitions.  It shares no code with the HIP library
 * and must never be linked, imported or called by the product path; only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may use it.
 *
 * Precision: inputs are float arrays whose values are exactly representable in
 * bf16.  Every contraction, softmax and cumulative sum is carried in fp64, in
 * the index order of the defining formula.  The one exception is the pooling
 * step, whose result is *quantised* to bf16: a quantisation decision has to be
 * taken in the same precision on both sides of a parity test, so the window sum
 * is an fp32 sum in token order, divided by c in fp32, then rounded to nearest
 * even bf16 -- exactly what a bf16 average-pool produces.
 *
 * Loops are parallelised with OpenMP over independent output rows only; no
 * blocking, fusion or reordering of the arithmetic is applied.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- bf16 quantisation (round to nearest, ties to even), value kept as float */
static float oracle_round_bf16(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7f800000u) == 0x7f800000u) {          /* inf / nan: truncate, keep nan a nan */
        if (u & 0x007fffffu) u |= 0x00400000u;
        u &= 0xffff0000u;
    } else {
        uint32_t lsb = (u >> 16) & 1u;
        u += 0x7fffu + lsb;
        u &= 0xffff0000u;
    }
    memcpy(&x, &u, 4);
    return x;
}

float oracle_bf16_round_scalar(float x) { return oracle_round_bf16(x); }

/*
 * Sequence-level average pooling, Eq. (1) / Alg. 1 step 1.
 *   x   : [L][d] tokens of one head of one sequence
 *   out : [ceil(L/c)][d] composite tokens; window t' covers tokens [t'c, t'c + c)
 * (0-based, non-overlapping windows).  When c does not divide L the last window is
 * clipped to the sequence and averages the tokens that exist.  Result quantised to bf16.
 */
void oracle_avgpool_seq(const float *x, int64_t L, int d, int c, float *out)
{
    int64_t Lc = (L + c - 1) / c;
    #pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < Lc; ++t) {
        int64_t cnt = (t + 1) * c <= L ? c : L - t * c;
        for (int e = 0; e < d; ++e) {
            float acc = 0.0f;
            for (int64_t m = 0; m < cnt; ++m)
                acc = acc + x[(t * c + m) * (int64_t)d + e];
            out[t * (int64_t)d + e] = oracle_round_bf16(acc / (float)cnt);
        }
    }
}

/*
 * Max pooling of the same windows (the alternative compression strategy of the ablation in
 * Sec. 6 "Compression Strategy"): every channel keeps its largest value in the window.
 * No rounding is involved: the result is one of the bf16 inputs.
 */
void oracle_maxpool_seq(const float *x, int64_t L, int d, int c, float *out)
{
    int64_t Lc = (L + c - 1) / c;
    #pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < Lc; ++t) {
        int64_t cnt = (t + 1) * c <= L ? c : L - t * c;
        for (int e = 0; e < d; ++e) {
            float best = x[(t * c) * (int64_t)d + e];
            for (int64_t m = 1; m < cnt; ++m) {
                float v = x[(t * c + m) * (int64_t)d + e];
                if (v > best) best = v;
            }
            out[t * (int64_t)d + e] = best;
        }
    }
}

/*
 * Stochastic pooling of the same windows (third compression strategy of the ablation in Sec. 6
 * "Compression Strategy"): the composite token is ONE token of the window, token m drawn with
 * probability  w_m / sum_m' w_m'  where the magnitude w_m = ||x_m||_2 is the Euclidean norm of the
 * token's d channels.  The draw is made from a caller-supplied uniform number u[t'] in [0, 1) by
 * inversion: the chosen m is the first one whose running sum w_0 + ... + w_m exceeds u * (total sum);
 * if none does (all magnitudes zero) the last token of the window is taken.
 *
 * A floating-point comparison decides an index here, so the precision is part of the definition:
 * fp32 throughout -- squares accumulated with fused multiply-adds in channel order, a correctly
 * rounded square root, the running sum in token order, one product u * total.
 *   sel (optional) : [ceil(L/c)] receives the chosen offsets m.
 */
void oracle_stochpool_seq(const float *x, int64_t L, int d, int c, const float *u, float *out, int32_t *sel)
{
    int64_t Lc = (L + c - 1) / c;
    #pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < Lc; ++t) {
        int64_t cnt = (t + 1) * c <= L ? c : L - t * c;
        float total = 0.0f;
        for (int64_t m = 0; m < cnt; ++m) {
            float sq = 0.0f;
            for (int e = 0; e < d; ++e) {
                float v = x[(t * c + m) * (int64_t)d + e];
                sq = fmaf(v, v, sq);
            }
            total = total + sqrtf(sq);
        }
        float cut = u[t] * total;
        int64_t pick = cnt - 1;
        float run = 0.0f;
        for (int64_t m = 0; m < cnt; ++m) {
            float sq = 0.0f;
            for (int e = 0; e < d; ++e) {
                float v = x[(t * c + m) * (int64_t)d + e];
                sq = fmaf(v, v, sq);
            }
            run = run + sqrtf(sq);
            if (run > cut) { pick = m; break; }
        }
        for (int e = 0; e < d; ++e) out[t * (int64_t)d + e] = x[(t * c + pick) * (int64_t)d + e];
        if (sel) sel[t] = (int32_t)pick;
    }
}

/*
 * Head-level average pooling, Eq. (2): mean of c_h consecutive heads of the
 * composite tokens.   x : [H][Lc][d]  ->  out : [H/c_h][Lc][d], quantised to bf16
 * (same quantisation rule as the sequence pooling).
 */
void oracle_avgpool_head(const float *x, int H, int64_t Lc, int d, int c_h, float *out)
{
    int Hc = H / c_h;
    int64_t plane = Lc * (int64_t)d;
    #pragma omp parallel for schedule(static)
    for (int64_t idx = 0; idx < (int64_t)Hc * plane; ++idx) {
        int hp = (int)(idx / plane);
        int64_t r = idx % plane;
        float acc = 0.0f;
        for (int m = 0; m < c_h; ++m)
            acc = acc + x[((int64_t)(hp * c_h + m)) * plane + r];
        out[idx] = oracle_round_bf16(acc / (float)c_h);
    }
}

/*
 * Block importance scores of one (compressed) head: compressed logits
 * P~ = Q~ K~^T * scale (Sec. 4.3), row softmax over composite keys, then the
 * block aggregation of Eq. (3) with the index sets R_x(u) of Eq. (4).
 *
 *   qt : [Lq][d] composite queries (Lq = ceil(L/c_q)),  kt : [Lk][d] composite keys
 *   rows[n_rows] : the query-block indices i whose score rows are wanted
 *   score : [n_rows][N] (N = L/S), score[r][j] = Score(rows[r], j)
 *
 * causal_mode 0: non-causal, every composite key enters the softmax.
 * causal_mode 1: composite key s' is visible to composite query t' iff the first
 *                token of its window is not after the last token of the query
 *                window:  s' c_k <= (t'+1) c_q - 1.  Invisible keys are excluded
 *                from the softmax (the "valid attention ranges integrated into
 *                the scoring" of Sec. 5).
 * causal_mode 2: the literal Alg. 1 ordering -- softmax over all composite keys,
 *                causality applied only by the later block-level cut.  Kept for a
 *                sensitivity test of the reading above.
 */
void oracle_block_scores(const float *qt, const float *kt, int64_t Lq, int64_t Lk,
                         int d, int S, int c_q, int c_k, int causal_mode, double scale,
                         const int32_t *rows, int n_rows, int64_t N, double *score)
{
    int nq = S / c_q;                       /* composite queries per query block  */
    #pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < n_rows; ++r) {
        int64_t i = rows[r];
        double *out = score + (int64_t)r * N;
        double *p = (double *)malloc(sizeof(double) * (size_t)Lk);
        for (int64_t j = 0; j < N; ++j) out[j] = 0.0;
        for (int64_t tq = i * nq; tq < (i + 1) * nq && tq < Lq; ++tq) {   /* t' in R_q(i) */
            const float *qrow = qt + tq * d;
            double pmax = -INFINITY;
            for (int64_t s = 0; s < Lk; ++s) {
                int visible = 1;
                if (causal_mode == 1) visible = (s * c_k <= (tq + 1) * (int64_t)c_q - 1);
                if (!visible) { p[s] = -INFINITY; continue; }
                const float *krow = kt + s * d;
                double acc = 0.0;
                for (int e = 0; e < d; ++e) acc += (double)qrow[e] * (double)krow[e];
                p[s] = acc * scale;
                if (p[s] > pmax) pmax = p[s];
            }
            double den = 0.0;
            for (int64_t s = 0; s < Lk; ++s)
                if (p[s] != -INFINITY) den += exp(p[s] - pmax);
            for (int64_t s = 0; s < Lk; ++s) {
                if (p[s] == -INFINITY) continue;
                double a = exp(p[s] - pmax) / den;            /* A~[t', s'] */
                int64_t j = (s * c_k) / S;                    /* s' in R_k(j) */
                out[j] += a;
            }
        }
        free(p);
    }
}

/* ---- selection ------------------------------------------------------------ */

typedef struct { double v; int32_t j; } oracle_kv;

static int oracle_cmp_desc(const void *a, const void *b)
{
    const oracle_kv *x = (const oracle_kv *)a, *y = (const oracle_kv *)b;
    if (x->v > y->v) return -1;
    if (x->v < y->v) return 1;
    return (x->j > y->j) - (x->j < y->j);            /* ties: lower key block first */
}

/*
 * Top-P selection of one score row, Eq. (5) and the sentence before it: order the
 * valid key blocks by descending score, accumulate greedily, stop as soon as the
 * cumulative share reaches P (the block that crosses the threshold is kept).
 *   score[n_valid] : scores of the valid key blocks (entries the causal cut
 *                    removes are simply not passed in)
 *   sel[n_valid]   : out, 1 = selected
 * P >= 1 selects every valid block.  Returns the number selected.
 */
int oracle_select_top_p(const double *score, int n_valid, double P, uint8_t *sel)
{
    oracle_kv *o = (oracle_kv *)malloc(sizeof(oracle_kv) * (size_t)(n_valid > 0 ? n_valid : 1));
    double tot = 0.0;
    for (int j = 0; j < n_valid; ++j) { o[j].v = score[j]; o[j].j = j; tot += score[j]; sel[j] = 0; }
    qsort(o, (size_t)n_valid, sizeof(oracle_kv), oracle_cmp_desc);
    int count = 0;
    if (P >= 1.0) {
        for (int j = 0; j < n_valid; ++j) sel[j] = 1;
        count = n_valid;
    } else {
        double run = 0.0, target = P * tot;
        for (int r = 0; r < n_valid; ++r) {
            sel[o[r].j] = 1; ++count;
            run += o[r].v;
            if (run >= target) break;
        }
    }
    free(o);
    return count;
}

/*
 * Fixed-budget selection (the "selection budget" alternative to the threshold):
 * keep the k = max(1, ceil(f * n_valid)) best blocks in the same order as above.
 */
int oracle_select_top_k(const double *score, int n_valid, double f, uint8_t *sel)
{
    oracle_kv *o = (oracle_kv *)malloc(sizeof(oracle_kv) * (size_t)(n_valid > 0 ? n_valid : 1));
    for (int j = 0; j < n_valid; ++j) { o[j].v = score[j]; o[j].j = j; sel[j] = 0; }
    qsort(o, (size_t)n_valid, sizeof(oracle_kv), oracle_cmp_desc);
    int k = (int)ceil(f * (double)n_valid);
    if (k < 1) k = 1;
    if (k > n_valid) k = n_valid;
    for (int r = 0; r < k; ++r) sel[o[r].j] = 1;
    free(o);
    return k;
}

/*
 * Block-masked attention of one head (Sec. 2.2):
 *   O = softmax(Q K^T * scale + M~) V,  M~ = 0 on selected blocks, -inf elsewhere,
 * plus token-level causality (s <= t) when causal != 0.
 *   q : [L][d];  k, v : [L][d];  mask : [N][N] bytes, N = ceil(L/S): when S does not divide L
 *   the last block is the shorter remainder (the index sets of Eq. (4) clipped to the sequence)
 *   rows[n_rows] : query blocks to evaluate
 *   out : [n_rows][S][d],  lse : [n_rows][S] = log sum_s exp(logit)  (natural log)
 * A query with no visible key yields a zero row and lse = -inf; so do the slots of the last
 * block that lie beyond the sequence.
 */
void oracle_masked_attention(const float *q, const float *k, const float *v, int64_t L, int d,
                             int S, int causal, double scale, const uint8_t *mask,
                             const int32_t *rows, int n_rows, double *out, double *lse)
{
    int64_t N = (L + S - 1) / S;
    #pragma omp parallel for schedule(dynamic, 8)
    for (int64_t idx = 0; idx < (int64_t)n_rows * S; ++idx) {
        int r = (int)(idx / S);
        int64_t i = rows[r];
        int64_t t = i * S + idx % S;
        double *orow = out + idx * d;
        if (t >= L) {                                   /* beyond the sequence: no query here */
            for (int e = 0; e < d; ++e) orow[e] = 0.0;
            lse[idx] = -INFINITY;
            continue;
        }
        const float *qrow = q + t * d;
        double *p = (double *)malloc(sizeof(double) * (size_t)L);
        double pmax = -INFINITY;
        for (int64_t s = 0; s < L; ++s) {
            int allowed = mask[i * N + s / S] != 0;
            if (causal && s > t) allowed = 0;
            if (!allowed) { p[s] = -INFINITY; continue; }
            const float *krow = k + s * d;
            double acc = 0.0;
            for (int e = 0; e < d; ++e) acc += (double)qrow[e] * (double)krow[e];
            p[s] = acc * scale;
            if (p[s] > pmax) pmax = p[s];
        }
        for (int e = 0; e < d; ++e) orow[e] = 0.0;
        double den = 0.0;
        if (pmax != -INFINITY) {
            for (int64_t s = 0; s < L; ++s)
                if (p[s] != -INFINITY) den += exp(p[s] - pmax);
            for (int64_t s = 0; s < L; ++s) {
                if (p[s] == -INFINITY) continue;
                double a = exp(p[s] - pmax) / den;
                const float *vrow = v + s * d;
                for (int e = 0; e < d; ++e) orow[e] += a * (double)vrow[e];
            }
            lse[idx] = pmax + log(den);
        } else {
            lse[idx] = -INFINITY;
        }
        free(p);
    }
}

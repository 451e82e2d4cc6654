/*
 * CPU oracle for the LAQ re-eviction hot path -- TEST INFRASTRUCTURE ONLY.
 *
 * This file is the plain, slow, single-threaded fp64 definition that the HIP
 * library is checked against.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it; the product path never does, and it shares no
 * code, header, table or helper with the HIP sources.
 *
 * What it computes (paper, Sec. 4.3 "KV-Cache Re-eviction", Eq. 4; the
 * observation-window procedure it defers to is the one summarised in Sec. 2.1
 * and Sec. 5.1 "Selected baselines"):
 *
 *   For one (sequence, layer) instance with Hq query heads sharing Hkv KV heads
 *   (G = Hq/Hkv consecutive query heads per KV head), the Q-cache holds W
 *   lookahead queries per query head and the key cache holds L rows per KV
 *   head, the last W of which are the window tokens themselves.  P = L - W.
 *
 *   1. window query w stands at position P + w and sees keys j <= P + w;
 *   2. logit  s_j = scale * <q[h,w,:], k[h/G, j, :]>;
 *   3. attention of that query over its visible keys: p_j = exp(s_j - M) / Z;
 *   4. raw[g, j] = sum over the G heads of the group and the W queries of p_j
 *      (the sum over the Q-cache of Eq. 4, taken on attention scores);
 *   5. pooled[g, j] = max of raw[g, i] over |i - j| <= (p-1)/2 clipped to the
 *      prefix [0, P); window columns keep their raw value;
 *   6. per KV head keep the (budget - W) largest pooled prefix entries, ties to
 *      the lower index, plus the W window tokens; indices ascending
 *      ("ArgSort(...)[:B]" of Eq. 4);
 *   7. the compacted cache is K and V restricted to those rows.
 *
 * General observation window (Sec. 4.3, Eq. 5, "LAQ++": local window queries
 * joined with the lookahead Q-cache): each of the W queries carries its own
 * position q_pos[w] in the key sequence and sees keys j <= q_pos[w]; a
 * lookahead query, generated after the whole prompt, has q_pos >= L-1 and
 * sees every key.  The number of trailing keys that are always retained
 * (`keep`, the local window's own tokens; may be 0) is then independent of W;
 * ranking and pooling run over the prefix [0, L - keep).  The layout above is
 * the special case q_pos[w] = L - W + w, keep = W.
 *
 * Stage-1 eviction (Sec. 4.2 "Lookahead": the low-budget eviction that
 * precedes the lookahead decoding uses an existing method): the observation-
 * window procedure above with the prompt suffix as window is that method in
 * its SnapKV form; Sec. 5.1 describes its pooling as an average, provided here
 * as laq_oracle_avgpool (window mean with zeros outside the prefix, i.e. the
 * sum over the clipped window divided by the kernel size).  The StreamingLLM
 * form keeps the first tokens of the sequence ("sinks") and the most recent
 * ones and needs no scores: laq_oracle_sink_recent.
 *
 * Recall of a selection (Sec. 3, Eq. 1-3): with M_gold the index set selected
 * by one set of queries (the response tokens') and M_pred the set selected by
 * another (an observation window's), Recall = |M_pred ∩ M_gold| / |M_gold| per
 * KV head: laq_oracle_overlap counts the intersection.
 *
 * The step after the path (Sec. 4.3: after the re-eviction, generation goes on
 * as standard autoregressive decoding): one new token's query attends to the
 * retained rows of its KV head, out[h] = softmax_j(scale <q_h, K'_j>) V' with
 * KV head h / G and no mask (every retained key precedes the new token):
 * laq_oracle_decode_attention.  The step before it (Sec. 4.2: the lookahead
 * decoding keeps its query states as the Q-cache) is a plain store of the
 * step's queries into slot t of the cache: laq_oracle_qcache_store.
 *
 * Readings where the paper is silent (softmax before the sum, 1/sqrt(d) scale,
 * max- rather than average-pooling, GQA sum, budget including the window,
 * tie-break) are listed in the design notes of the repository.
 *
 * Pins (tests marked "not gpu"): brute-force attention matrices on tiny inputs,
 * row-sum and non-negativity invariants, the closed form for identical keys,
 * the W=1/G=1/pool=1 reduction to ArgSort(q K^T), GQA additivity, key-shift
 * invariance, hand-computed pooling cases, exhaustive top-k, planted keys;
 * the average pool against a library average-pooling routine, its column-sum
 * identity and hand cases; the sink+recent list against set-built brute force;
 * the overlap count against Python set intersection, its symmetry and extremes;
 * decode attention against a library softmax-and-matmul, the mean of V for
 * identical keys, a dominant key, GQA head mapping; the Q-cache store against
 * tensor indexing.
 * No function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

static double load_elem(const void *base, int dtype, size_t i)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[i];
    /* bfloat16: the high 16 bits of an IEEE binary32 */
    uint32_t bits = (uint32_t)((const uint16_t *)base)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/*
 * Steps 1-4.  q: [Hq, W, d], k: [Hkv, L, d] in `dtype`; raw: [Hkv, L] doubles.
 * q_pos: W positions (query w sees keys j <= q_pos[w]; values beyond L-1 mean
 * "every key"), or NULL for the trailing window q_pos[w] = L - W + w (needs
 * W <= L).  scale <= 0 selects 1/sqrt(d).  Returns 0, or -1 on bad arguments.
 */
int laq_oracle_raw_scores(const void *q, const void *k, int dtype,
                          int Hq, int Hkv, int d, int L, int W,
                          const int32_t *q_pos, double scale, double *raw)
{
    if (!q || !k || !raw || Hq <= 0 || Hkv <= 0 || d <= 0 || L <= 0 || W <= 0 ||
        (!q_pos && W > L) || Hq % Hkv != 0 || (dtype != ORACLE_F32 && dtype != ORACLE_BF16))
        return -1;
    if (q_pos)
        for (int w = 0; w < W; ++w)
            if (q_pos[w] < 0) return -1;
    const int G = Hq / Hkv;
    if (scale <= 0.0)
        scale = 1.0 / sqrt((double)d);

    double *qrow = (double *)malloc(sizeof(double) * (size_t)d);
    double *s = (double *)malloc(sizeof(double) * (size_t)L);
    if (!qrow || !s) { free(qrow); free(s); return -1; }

    for (size_t i = 0; i < (size_t)Hkv * (size_t)L; ++i)
        raw[i] = 0.0;

    for (int h = 0; h < Hq; ++h) {
        const int g = h / G;
        for (int w = 0; w < W; ++w) {
            int last = q_pos ? q_pos[w] : L - W + w;   /* last visible key */
            if (last > L - 1) last = L - 1;
            const int vis = last + 1;
            for (int c = 0; c < d; ++c)
                qrow[c] = load_elem(q, dtype, ((size_t)h * W + w) * d + c);
            double M = -INFINITY;
            for (int j = 0; j < vis; ++j) {
                double acc = 0.0;
                const size_t off = ((size_t)g * L + j) * d;
                for (int c = 0; c < d; ++c)
                    acc += qrow[c] * load_elem(k, dtype, off + c);
                s[j] = scale * acc;
                if (s[j] > M) M = s[j];
            }
            double Z = 0.0;
            for (int j = 0; j < vis; ++j) {
                s[j] = exp(s[j] - M);
                Z += s[j];
            }
            for (int j = 0; j < vis; ++j)
                raw[(size_t)g * L + j] += s[j] / Z;
        }
    }
    free(qrow);
    free(s);
    return 0;
}

/*
 * Step 5.  raw, pooled: [Hkv, L] doubles (may not alias).  pool is odd >= 1.
 * keep = number of trailing keys that are always retained (0 <= keep <= L);
 * P = L - keep.  The max runs over the part of the pooling window that lies
 * inside the prefix [0, P); columns j >= P are copied.
 */
int laq_oracle_maxpool(const double *raw, int Hkv, int L, int keep, int pool, double *pooled)
{
    if (!raw || !pooled || Hkv <= 0 || L <= 0 || keep < 0 || keep > L || pool < 1 || pool % 2 == 0)
        return -1;
    const int P = L - keep, half = (pool - 1) / 2;
    for (int g = 0; g < Hkv; ++g) {
        const double *r = raw + (size_t)g * L;
        double *o = pooled + (size_t)g * L;
        for (int j = 0; j < P; ++j) {
            int lo = j - half, hi = j + half;
            if (lo < 0) lo = 0;
            if (hi > P - 1) hi = P - 1;
            double m = r[lo];
            for (int i = lo + 1; i <= hi; ++i)
                if (r[i] > m) m = r[i];
            o[j] = m;
        }
        for (int j = P; j < L; ++j)
            o[j] = r[j];
    }
    return 0;
}

/*
 * Step 5, average variant (Sec. 5.1 describes the observation-window baseline's
 * pooling as an average).  Same arguments as laq_oracle_maxpool.  The mean is
 * taken over the full kernel with zeros standing in for positions outside the
 * prefix [0, P): pooled[j] = (sum of raw[i], |i-j| <= (pool-1)/2, 0 <= i < P) / pool.
 * Columns j >= P are copied.
 */
int laq_oracle_avgpool(const double *raw, int Hkv, int L, int keep, int pool, double *pooled)
{
    if (!raw || !pooled || Hkv <= 0 || L <= 0 || keep < 0 || keep > L || pool < 1 || pool % 2 == 0)
        return -1;
    const int P = L - keep, half = (pool - 1) / 2;
    for (int g = 0; g < Hkv; ++g) {
        const double *r = raw + (size_t)g * L;
        double *o = pooled + (size_t)g * L;
        for (int j = 0; j < P; ++j) {
            double acc = 0.0;
            for (int i = j - half; i <= j + half; ++i)
                if (i >= 0 && i < P) acc += r[i];
            o[j] = acc / (double)pool;
        }
        for (int j = P; j < L; ++j)
            o[j] = r[j];
    }
    return 0;
}

/*
 * Score-free stage-1 eviction in the StreamingLLM form (Sec. 2.1, Sec. 4.2):
 * every head keeps the first n_sink positions and the most recent ones, Bk =
 * min(budget, L) in all (budget >= 1).  idx: [Hkv, Bk], ascending.  When n_sink >= Bk the
 * list is the first Bk positions.
 */
int laq_oracle_sink_recent(int Hkv, int L, int n_sink, int budget, int32_t *idx)
{
    if (!idx || Hkv <= 0 || L <= 0 || n_sink < 0 || budget < 1)
        return -1;
    const int Bk = budget < L ? budget : L;
    const int s = n_sink < Bk ? n_sink : Bk;
    const int recent = Bk - s;
    for (int g = 0; g < Hkv; ++g) {
        int32_t *out = idx + (size_t)g * Bk;
        for (int t = 0; t < s; ++t)
            out[t] = t;
        for (int t = 0; t < recent; ++t)
            out[s + t] = L - recent + t;
    }
    return 0;
}

/*
 * Eq. 3's numerator.  pred: [Hkv, n_pred], gold: [Hkv, n_gold], entries in
 * [0, L), each row without repeats (any order); overlap[g] = number of
 * positions that row g of pred shares with row g of gold.  The recall of Eq. 3
 * is overlap[g] / n_gold.
 */
int laq_oracle_overlap(const int32_t *pred, int n_pred, const int32_t *gold, int n_gold,
                       int Hkv, int L, int32_t *overlap)
{
    if (!pred || !gold || !overlap || Hkv <= 0 || L <= 0 || n_pred < 0 || n_gold < 0)
        return -1;
    unsigned char *in_gold = (unsigned char *)malloc((size_t)L);
    if (!in_gold) return -1;
    for (int g = 0; g < Hkv; ++g) {
        memset(in_gold, 0, (size_t)L);
        for (int t = 0; t < n_gold; ++t) {
            int32_t j = gold[(size_t)g * n_gold + t];
            if (j < 0 || j >= L) { free(in_gold); return -1; }
            in_gold[j] = 1;
        }
        int32_t count = 0;
        for (int t = 0; t < n_pred; ++t) {
            int32_t j = pred[(size_t)g * n_pred + t];
            if (j < 0 || j >= L) { free(in_gold); return -1; }
            count += in_gold[j];
        }
        overlap[g] = count;
    }
    free(in_gold);
    return 0;
}

/*
 * Single-token attention over a compacted cache (Sec. 4.3, the decoding that
 * follows the re-eviction).  q: [Hq, d], kc, vc: [Hkv, Bk, d] in `dtype`;
 * out: [Hq, d] doubles.  Query head h uses KV head h / (Hq / Hkv).
 * scale <= 0 selects 1/sqrt(d).
 */
int laq_oracle_decode_attention(const void *q, const void *kc, const void *vc, int dtype,
                                int Hq, int Hkv, int d, int Bk, double scale, double *out)
{
    if (!q || !kc || !vc || !out || Hq <= 0 || Hkv <= 0 || d <= 0 || Bk <= 0 || Hq % Hkv != 0 ||
        (dtype != ORACLE_F32 && dtype != ORACLE_BF16))
        return -1;
    const int G = Hq / Hkv;
    if (scale <= 0.0)
        scale = 1.0 / sqrt((double)d);
    double *p = (double *)malloc(sizeof(double) * (size_t)Bk);
    if (!p) return -1;
    for (int h = 0; h < Hq; ++h) {
        const int g = h / G;
        double M = -INFINITY;
        for (int j = 0; j < Bk; ++j) {
            double acc = 0.0;
            for (int c = 0; c < d; ++c)
                acc += load_elem(q, dtype, (size_t)h * d + c) * load_elem(kc, dtype, ((size_t)g * Bk + j) * d + c);
            p[j] = scale * acc;
            if (p[j] > M) M = p[j];
        }
        double Z = 0.0;
        for (int j = 0; j < Bk; ++j) {
            p[j] = exp(p[j] - M);
            Z += p[j];
        }
        for (int c = 0; c < d; ++c) {
            double acc = 0.0;
            for (int j = 0; j < Bk; ++j)
                acc += p[j] * load_elem(vc, dtype, ((size_t)g * Bk + j) * d + c);
            out[(size_t)h * d + c] = acc / Z;
        }
    }
    free(p);
    return 0;
}

/*
 * Q-cache capture (Sec. 4.2): the queries of lookahead step t, q_step [Hq, d],
 * become row t of every head of the Q-cache [Hq, W, d]; elem_bytes is the
 * element size.  A byte copy.
 */
int laq_oracle_qcache_store(const void *q_step, int Hq, int W, int d, size_t elem_bytes, int t, void *q_cache)
{
    if (!q_step || !q_cache || Hq <= 0 || W <= 0 || d <= 0 || t < 0 || t >= W || elem_bytes == 0)
        return -1;
    const size_t row = (size_t)d * elem_bytes;
    for (int h = 0; h < Hq; ++h)
        memcpy((char *)q_cache + ((size_t)h * W + t) * row, (const char *)q_step + (size_t)h * row, row);
    return 0;
}

typedef struct { float score; int32_t index; } ranked_t;

static int ranked_cmp(const void *a, const void *b)
{
    const ranked_t *x = (const ranked_t *)a, *y = (const ranked_t *)b;
    if (x->score > y->score) return -1;      /* larger score first */
    if (x->score < y->score) return 1;
    return (x->index > y->index) - (x->index < y->index);   /* then lower index */
}

static int int32_cmp(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * Step 6.  scores: [Hkv, L] fp32 (the precision in which the library takes the
 * decision); idx: [Hkv, Bk] with Bk = min(budget, L).  keep = number of
 * trailing keys always retained (0 <= keep <= L, budget >= keep); P = L - keep.
 * A full sort of the prefix by (score descending, index ascending); the first
 * Bk - keep entries are kept, re-sorted ascending, and followed by P .. L-1.
 */
int laq_oracle_select(const float *scores, int Hkv, int L, int keep, int budget, int32_t *idx)
{
    if (!scores || !idx || Hkv <= 0 || L <= 0 || keep < 0 || keep > L || budget < keep)
        return -1;
    const int W = keep;
    const int P = L - W;
    const int Bk = budget < L ? budget : L;
    const int ksel = Bk - W;
    ranked_t *r = (ranked_t *)malloc(sizeof(ranked_t) * (size_t)(P > 0 ? P : 1));
    if (!r) return -1;
    for (int g = 0; g < Hkv; ++g) {
        int32_t *out = idx + (size_t)g * Bk;
        for (int j = 0; j < P; ++j) {
            r[j].score = scores[(size_t)g * L + j];
            r[j].index = j;
        }
        qsort(r, (size_t)P, sizeof(ranked_t), ranked_cmp);
        for (int t = 0; t < ksel; ++t)
            out[t] = r[t].index;
        qsort(out, (size_t)ksel, sizeof(int32_t), int32_cmp);
        for (int w = 0; w < W; ++w)
            out[ksel + w] = P + w;
    }
    free(r);
    return 0;
}

/*
 * Step 7.  src: [Hkv, L, row_bytes], idx: [Hkv, Bk], dst: [Hkv, Bk, row_bytes].
 * Byte copy of the selected rows (row_bytes = d * element size).
 */
int laq_oracle_compact(const void *src, int Hkv, int L, size_t row_bytes,
                       const int32_t *idx, int Bk, void *dst)
{
    if (!src || !idx || !dst || Hkv <= 0 || L <= 0 || Bk < 0)
        return -1;
    for (int g = 0; g < Hkv; ++g)
        for (int t = 0; t < Bk; ++t) {
            int32_t j = idx[(size_t)g * Bk + t];
            if (j < 0 || j >= L) return -1;
            memcpy((char *)dst + ((size_t)g * Bk + t) * row_bytes,
                   (const char *)src + ((size_t)g * L + j) * row_bytes, row_bytes);
        }
    return 0;
}

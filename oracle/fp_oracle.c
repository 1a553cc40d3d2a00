/*
 * CPU oracle for the FlashPrefill prefill-attention path.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct implementation of what the paper's three stages
 * compute, written from the paper's equations.  It shares no code with the GPU
 * library and must never be called from the product path: only the test-suite, the
 * smoke check and the benchmark's cpu_baseline leg may load it.
 *
 * Arithmetic: inputs are bf16 bit patterns widened exactly; every sum, product and
 * exponential is taken in fp64; block scores are rounded once to fp32 on output
 * (the boundary's dtype).  The keep/drop decision of the threshold is an integer
 * decided by floating point, so it is taken in fp32 on those fp32 scores, the
 * precision the GPU kernel decides in.
 *
 * Layout: Q [T, Hq, d], K and V [Tk, Hkv, d], token-major packed; sequence s owns
 * query tokens cu[s]..cu[s+1] and key tokens cuk[s]..cuk[s+1] (cuk == NULL: the
 * same tokens, plain prefill).  With a KV prefix (chunked prefill) the queries are the
 * last tokens of the sequence: query i of the chunk sits at position P + i, where
 * P = kv_len - q_len >= 0 must be a multiple of `block`, and sees keys 0..P+i.
 * Blocks of `block` tokens are aligned to each sequence's start, so q-block I of the
 * chunk is the sequence's block I + P/block, and its causal key blocks are
 * J <= I + P/block.  q-block row r = row_offset[s] + I.  scores/idx are
 * [Hq, m_total, n_max] with n_max the most key blocks of any sequence, cnt is
 * [Hq, m_total], O is [T, Hq, d] (fp32 here), lse is [Hq, T].
 *
 * Readings of points the paper leaves open are listed where they apply.
 * Pins: tests/test_oracle_*.py (closed forms, library softmax, brute force, invariants).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline double bf16_val(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

typedef struct {
    int nseq, m_total, n_max, kb_total;
    int *row_offset; /* nseq+1: first q-block row of each sequence */
    int *kb_offset;  /* nseq+1: first key block of each sequence (in the list of all key blocks) */
    int *pb;         /* nseq: prefix length in blocks */
    int *row_seq;    /* m_total: sequence of each q-block row */
    const int32_t *cuq, *cuk;
} rows_t;

static void rows_free(rows_t *R) {
    free(R->row_offset);
    free(R->kb_offset);
    free(R->pb);
    free(R->row_seq);
}

static int rows_init(rows_t *R, int nseq, const int32_t *cu, const int32_t *cuk, int block) {
    memset(R, 0, sizeof(*R));
    R->nseq = nseq;
    R->cuq = cu;
    R->cuk = cuk ? cuk : cu;
    R->row_offset = (int *)malloc(sizeof(int) * (size_t)(nseq + 1));
    R->kb_offset = (int *)malloc(sizeof(int) * (size_t)(nseq + 1));
    R->pb = (int *)malloc(sizeof(int) * (size_t)(nseq > 0 ? nseq : 1));
    if (!R->row_offset || !R->kb_offset || !R->pb) return -1;
    R->row_offset[0] = 0;
    R->kb_offset[0] = 0;
    for (int s = 0; s < nseq; ++s) {
        int qlen = cu[s + 1] - cu[s];
        int klen = R->cuk[s + 1] - R->cuk[s];
        int prefix = klen - qlen;
        if (qlen <= 0 || prefix < 0 || prefix % block != 0) {
            rows_free(R);
            return -1;
        }
        int nkb = (klen + block - 1) / block;
        if (nkb > R->n_max) R->n_max = nkb;
        R->pb[s] = prefix / block;
        R->row_offset[s + 1] = R->row_offset[s] + (qlen + block - 1) / block;
        R->kb_offset[s + 1] = R->kb_offset[s] + nkb;
    }
    R->m_total = R->row_offset[nseq];
    R->kb_total = R->kb_offset[nseq];
    R->row_seq = (int *)malloc(sizeof(int) * (size_t)(R->m_total > 0 ? R->m_total : 1));
    if (!R->row_seq) {
        rows_free(R);
        return -1;
    }
    for (int s = 0; s < nseq; ++s)
        for (int r = R->row_offset[s]; r < R->row_offset[s + 1]; ++r) R->row_seq[r] = s;
    return 0;
}

int fpo_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* (m_total, n_max, row_offset[nseq+1]) of a packed batch; -1 for lengths the path does not take. */
int fpo_layout(int nseq, const int32_t *cu, const int32_t *cuk, int block, int32_t *m_total, int32_t *n_max,
               int32_t *row_offset) {
    rows_t R;
    if (rows_init(&R, nseq, cu, cuk, block)) return -1;
    *m_total = R.m_total;
    *n_max = R.n_max;
    if (row_offset) memcpy(row_offset, R.row_offset, sizeof(int) * (size_t)(nseq + 1));
    rows_free(&R);
    return 0;
}

/*
 * Stage (i), pattern discovery: Sec. 3.1 (pooled keys), Sec. 3.2 Eq. 1-4, Alg. 1.
 *
 *   kbar_J   = mean of the keys of block J                       (Alg. 1 stage 1)
 *   x_i      = tau * q_i . kbar_J   for the queries i of tile I, J <= I  (with a KV prefix of
 *              PB blocks, "J <= I" reads "J <= I + PB" here and below)
 *   m_IJ     = max_i x_i ;  S_IJ = sum_i exp(x_i - m_IJ)          (Eq. 1, 2)
 *   M_I      = max_{J<=I} m_IJ ;  S'_IJ = S_IJ exp(m_IJ - M_I)    (Eq. 3)
 *   P_IJ     = S'_IJ / (sum_{K<=I} S'_IK + eps) ;  P_IJ = 0, J>I  (Eq. 4)
 *
 * Alg. 1 writes the same function in base 2 with log2(e) folded into the logits.
 * Readings: the "causal mask" on a query-tile x pooled-key product is pair-level
 * (J <= I) only, the diagonal block's pooled key is the mean of the whole block; a
 * ragged last block averages its valid keys and leaves out missing queries; query
 * head h uses KV head h / (Hq/Hkv); the normalisation line applies to every J <= I.
 *
 * rows: optional list of q-block rows to compute (all heads); NULL = all rows.
 * Rows not listed are left untouched; listed rows are written for all n_max columns.
 */
int fpo_block_search(const uint16_t *Q, const uint16_t *K, int nseq, const int32_t *cu, const int32_t *cuk, int hq,
                     int hkv, int d, int block, double tau, double eps, const int32_t *rows, int nrows,
                     float *scores) {
    rows_t R;
    if (rows_init(&R, nseq, cu, cuk, block)) return -1;
    const int g = hq / hkv;
    const size_t kb_stride = (size_t)hkv * d;
    double *kbar = (double *)calloc((size_t)(R.kb_total > 0 ? R.kb_total : 1) * kb_stride, sizeof(double));
    if (!kbar) return -1;

    /* Alg. 1 stage 1: one mean vector per (key block, KV head). */
#pragma omp parallel for schedule(static)
    for (int s = 0; s < nseq; ++s) {
        for (int J = 0; J < R.kb_offset[s + 1] - R.kb_offset[s]; ++J) {
            int t0 = R.cuk[s] + J * block;
            int t1 = t0 + block < R.cuk[s + 1] ? t0 + block : R.cuk[s + 1];
            for (int hk = 0; hk < hkv; ++hk) {
                double *kb = kbar + (size_t)(R.kb_offset[s] + J) * kb_stride + (size_t)hk * d;
                for (int t = t0; t < t1; ++t)
                    for (int c = 0; c < d; ++c) kb[c] += bf16_val(K[((size_t)t * hkv + hk) * d + c]);
                for (int c = 0; c < d; ++c) kb[c] /= (double)(t1 - t0);
            }
        }
    }

    const int nwork = (rows ? nrows : R.m_total) * hq;
#pragma omp parallel
    {
        double *m = (double *)malloc(sizeof(double) * (size_t)(R.n_max + 1));
        double *S = (double *)malloc(sizeof(double) * (size_t)(R.n_max + 1));
        double *x = (double *)malloc(sizeof(double) * (size_t)block);
#pragma omp for schedule(dynamic, 1)
        for (int wk = 0; wk < nwork; ++wk) {
            int r = rows ? rows[wk / hq] : (R.m_total - 1 - wk / hq);
            int h = wk % hq, hk = h / g;
            int s = R.row_seq[r];
            int Iq = r - R.row_offset[s];
            int I = Iq + R.pb[s]; /* the tile's block index within its sequence */
            int t0 = cu[s] + Iq * block;
            int nq = (t0 + block < cu[s + 1] ? t0 + block : cu[s + 1]) - t0;
            /* Alg. 1 stage 2: per block pair a max and a sum of exponentials over the query tile. */
            for (int J = 0; J <= I; ++J) {
                const double *kb = kbar + (size_t)(R.kb_offset[s] + J) * kb_stride + (size_t)hk * d;
                double mx = -INFINITY;
                for (int i = 0; i < nq; ++i) {
                    const uint16_t *q = Q + ((size_t)(t0 + i) * hq + h) * d;
                    double dot = 0.0;
                    for (int c = 0; c < d; ++c) dot += bf16_val(q[c]) * kb[c];
                    x[i] = tau * dot;
                    if (x[i] > mx) mx = x[i];
                }
                double sum = 0.0;
                for (int i = 0; i < nq; ++i) sum += exp(x[i] - mx);
                m[J] = mx;
                S[J] = sum;
            }
            /* Alg. 1 stage 3: bring every pair of the row to the row's max, then normalise. */
            double M = -INFINITY;
            for (int J = 0; J <= I; ++J)
                if (m[J] > M) M = m[J];
            double total = 0.0;
            for (int J = 0; J <= I; ++J) {
                S[J] = S[J] * exp(m[J] - M);
                total += S[J];
            }
            float *out = scores + ((size_t)h * R.m_total + r) * R.n_max;
            for (int J = 0; J < R.n_max; ++J) out[J] = J <= I ? (float)(S[J] / (total + eps)) : 0.0f;
        }
        free(m);
        free(S);
        free(x);
    }
    free(kbar);
    rows_free(&R);
    return 0;
}

/*
 * Stage (ii), max-based dynamic threshold and index compression: Sec. 3.4, Alg. 2.
 *
 *   thresh_I = alpha * max_{J<=I} score_IJ
 *   active_J = (score_IJ >= thresh_I  or  J < sinkB  or  0 <= I-J < winB)  and  J <= I
 *   idx[h, r, 0..cnt) = the active J in ascending order ; cnt[h, r] = their number
 *
 * Readings: keep at equality (Alg. 2 uses >=); the sink and window sizes are given
 * in tokens and compared in blocks, rounded up (256 -> 2 blocks, 512 -> 4 blocks,
 * the window including the diagonal block); the row max runs over J <= I; alpha <= 0
 * keeps every causal block.  Entries of idx past cnt are set to n_max here (the
 * paper's fill value is the block count); the boundary leaves them undefined.
 * The product alpha*max and the comparison are fp32, rounded once.
 */
int fpo_threshold(const float *scores, int nseq, const int32_t *cu, const int32_t *cuk, int hq, int block,
                  float alpha, int sink_tokens, int window_tokens, int32_t *idx, int32_t *cnt) {
    rows_t R;
    if (rows_init(&R, nseq, cu, cuk, block)) return -1;
    const int sinkB = (sink_tokens + block - 1) / block;
    const int winB = (window_tokens + block - 1) / block;
#pragma omp parallel for schedule(dynamic, 16)
    for (int wk = 0; wk < R.m_total * hq; ++wk) {
        int r = wk / hq, h = wk % hq;
        int I = r - R.row_offset[R.row_seq[r]] + R.pb[R.row_seq[r]];
        const float *row = scores + ((size_t)h * R.m_total + r) * R.n_max;
        int32_t *out = idx + ((size_t)h * R.m_total + r) * R.n_max;
        float mx = row[0];
        for (int J = 1; J <= I; ++J)
            if (row[J] > mx) mx = row[J];
        volatile float thr = alpha * mx; /* one fp32 rounding, no fused contraction */
        int c = 0;
        for (int J = 0; J <= I; ++J) {
            int by_score = row[J] >= thr;
            int by_sink = J < sinkB;
            int by_window = (I - J >= 0) && (I - J < winB);
            if (by_score || by_sink || by_window) out[c++] = J;
        }
        cnt[(size_t)h * R.m_total + r] = c;
        for (int J = c; J < R.n_max; ++J) out[J] = R.n_max;
    }
    rows_free(&R);
    return 0;
}

/* softmax(tau q.k) V over an explicit key set, two passes, fp64. */
static void attend_row(const uint16_t *q, const uint16_t *K, const uint16_t *V, int hkv, int hk, int d, double tau,
                       const int *keys, int nkeys, double *logit, float *o, float *lse) {
    if (nkeys == 0) { /* not a paper case: a query with no visible key (empty list) gets O = 0, lse = -inf */
        for (int c = 0; c < d; ++c) o[c] = 0.0f;
        if (lse) *lse = -INFINITY;
        return;
    }
    double mx = -INFINITY;
    double qd[d];
    for (int c = 0; c < d; ++c) qd[c] = bf16_val(q[c]);
    for (int n = 0; n < nkeys; ++n) {
        const uint16_t *k = K + ((size_t)keys[n] * hkv + hk) * d;
        double dot = 0.0;
        for (int c = 0; c < d; ++c) dot += qd[c] * bf16_val(k[c]);
        logit[n] = tau * dot;
        if (logit[n] > mx) mx = logit[n];
    }
    double sum = 0.0;
    for (int n = 0; n < nkeys; ++n) {
        logit[n] = exp(logit[n] - mx);
        sum += logit[n];
    }
    for (int c = 0; c < d; ++c) {
        double acc = 0.0;
        for (int n = 0; n < nkeys; ++n) acc += logit[n] * bf16_val(V[((size_t)keys[n] * hkv + hk) * d + c]);
        o[c] = (float)(acc / sum);
    }
    if (lse) *lse = (float)((mx + log(sum)) * 1.4426950408889634074); /* base-2 log-sum-exp, Alg. 3 last line */
}

/*
 * Stage (iii), block-sparse attention given index lists: Sec. 3.5, Alg. 3.
 * The online-softmax loop of Alg. 3 computes exactly a softmax over the keys of the
 * listed blocks that are not in the query's future, so the oracle is that definition:
 *
 *   O_t = sum_u softmax_u(tau q_t.k_u) v_u ,  u in listed blocks of (h, I(t)), u <= t
 *   (positions within the sequence; with a KV prefix query t of the chunk is at P + t)
 *   lse_t = log2 sum_u 2^(tau log2e q_t.k_u)
 *
 * Query tile = block (the lists are indexed by the same I as the q-blocks).
 * rows: optional subset of q-block rows (all heads); NULL = all.  Unlisted rows untouched.
 */
int fpo_sparse_prefill(const uint16_t *Q, const uint16_t *K, const uint16_t *V, int nseq, const int32_t *cu,
                       const int32_t *cuk, int hq, int hkv, int d, int block, double tau, const int32_t *idx,
                       const int32_t *cnt, const int32_t *rows, int nrows, float *O, float *lse) {
    rows_t R;
    if (rows_init(&R, nseq, cu, cuk, block)) return -1;
    const int g = hq / hkv;
    int T = cu[nseq];
    const int nwork = (rows ? nrows : R.m_total) * hq;
#pragma omp parallel
    {
        int *keys = (int *)malloc(sizeof(int) * (size_t)(R.n_max + 1) * block);
        double *logit = (double *)malloc(sizeof(double) * (size_t)(R.n_max + 1) * block);
#pragma omp for schedule(dynamic, 1)
        for (int wk = 0; wk < nwork; ++wk) {
            int r = rows ? rows[wk / hq] : (R.m_total - 1 - wk / hq);
            int h = wk % hq, hk = h / g;
            int s = R.row_seq[r];
            int I = r - R.row_offset[s];
            int t0 = cu[s] + I * block;
            int t1 = t0 + block < cu[s + 1] ? t0 + block : cu[s + 1];
            const int32_t *list = idx + ((size_t)h * R.m_total + r) * R.n_max;
            int c = cnt[(size_t)h * R.m_total + r];
            for (int t = t0; t < t1; ++t) {
                int pos = R.pb[s] * block + (t - cu[s]); /* the query's position in its sequence */
                int nk = 0;
                for (int n = 0; n < c; ++n) {
                    int p0 = list[n] * block;
                    for (int p = p0; p < p0 + block && R.cuk[s] + p < R.cuk[s + 1]; ++p)
                        if (p <= pos) keys[nk++] = R.cuk[s] + p;
                }
                attend_row(Q + ((size_t)t * hq + h) * d, K, V, hkv, hk, d, tau, keys, nk, logit,
                           O + ((size_t)t * hq + h) * d, lse ? lse + (size_t)h * T + t : NULL);
            }
        }
        free(keys);
        free(logit);
    }
    rows_free(&R);
    return 0;
}

/*
 * Full causal attention (the comparison the paper measures against):
 *   O_t = sum_{u<=t, same sequence} softmax_u(tau q_t.k_u) v_u  (u, t: positions in the sequence).
 */
int fpo_dense_prefill(const uint16_t *Q, const uint16_t *K, const uint16_t *V, int nseq, const int32_t *cu,
                      const int32_t *cuk, int hq, int hkv, int d, int block, double tau, const int32_t *rows, int nrows,
                      float *O, float *lse) {
    rows_t R;
    if (rows_init(&R, nseq, cu, cuk, block)) return -1;
    const int g = hq / hkv;
    int T = cu[nseq];
    const int nwork = (rows ? nrows : R.m_total) * hq;
#pragma omp parallel
    {
        int *keys = (int *)malloc(sizeof(int) * (size_t)(R.n_max + 1) * block);
        double *logit = (double *)malloc(sizeof(double) * (size_t)(R.n_max + 1) * block);
#pragma omp for schedule(dynamic, 1)
        for (int wk = 0; wk < nwork; ++wk) {
            int r = rows ? rows[wk / hq] : (R.m_total - 1 - wk / hq);
            int h = wk % hq, hk = h / g;
            int s = R.row_seq[r];
            int I = r - R.row_offset[s];
            int t0 = cu[s] + I * block;
            int t1 = t0 + block < cu[s + 1] ? t0 + block : cu[s + 1];
            for (int t = t0; t < t1; ++t) {
                int pos = R.pb[s] * block + (t - cu[s]);
                int nk = 0;
                for (int p = 0; p <= pos; ++p) keys[nk++] = R.cuk[s] + p;
                attend_row(Q + ((size_t)t * hq + h) * d, K, V, hkv, hk, d, tau, keys, nk, logit,
                           O + ((size_t)t * hq + h) * d, lse ? lse + (size_t)h * T + t : NULL);
            }
        }
        free(keys);
        free(logit);
    }
    rows_free(&R);
    return 0;
}

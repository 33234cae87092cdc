/*
 * CPU oracle for the Judge Q eviction hot path -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow fp64 implementation of what the method computes at the end of
 * prefill (paper Section 4.3, the inference-time use of the soft tokens,
 * Eq. 3): the attention map of the soft-token queries over
 * the prompt keys, top-k retention on that map, and the pruned cache.  It is
 * used by the tests, the smoke check and the benchmark's CPU baseline leg to
 * judge the HIP kernels; it shares no code with them and the product path must
 * never call it.
 *
 * Every function works on ONE layer and ONE sequence; batching over layers and
 * ragged sequences is a loop in the Python wrapper.  Inputs are the raw bf16
 * bit patterns (widened exactly to double); all arithmetic is fp64 and every
 * output element is produced by one thread in index order, so results do not
 * depend on the thread count.
 *
 * Readings of points the paper leaves open (heads/GQA, sum vs mean, softmax
 * domain, pooling operator, tie-break) are listed next to each function.
 *
 * Pins (tests/test_oracle_*.py): hand-worked 3-key softmax, row-sum invariant,
 * L=1, zero queries, key-shift invariance, permutation/duplication laws, GQA
 * mapping by construction, brute force without max subtraction, numpy
 * cross-checks; the supplied-normaliser and soft-token-tail variants by hand-worked cases, by reduction
 * to jqo_score and by numpy with explicit keys; pooling impulse/constant/weight identities; exhaustive subset
 * search for top-B; numpy.take for compaction.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

static double bf16_to_f64(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

int jqo_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Importance scores (Section 4.3; Eq. 3 without its 1/n).
 *
 *   s[h,i,j]  = scale * sum_c Q[i,h,c] * K[j,g,c]          g = h / G, G = h_q / h_kv
 *   p[h,i,j]  = exp(s[h,i,j] - m[h,i]) / Z[h,i]            softmax over the L prompt keys
 *   score[g,j] = sum_{h in group g} sum_i p[h,i,j]
 *
 * Readings: the softmax runs over the prompt keys only (each query's row sums
 * to one); the n soft-token rows and the G query heads sharing a KV head are
 * summed, not averaged (ranking is the same); query head h reads KV head h/G.
 *
 * Q [n_q, h_q, d] and K [L, h_kv, d] are bf16 bits; score [h_kv, L] is double.
 * scale <= 0 means 1/sqrt(d).  Returns 0, or -1 on a bad argument / no memory.
 */
int jqo_score(int n_q, int h_q, int h_kv, int d, long L, double scale,
              const uint16_t* Q, const uint16_t* K, double* score) {
    if (n_q < 1 || h_q < 1 || h_kv < 1 || d < 1 || L < 1 || h_q % h_kv != 0 || !Q || !K || !score) return -1;
    const int G = h_q / h_kv;
    const int rows = n_q * G;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)d);

    double* Kd = (double*)malloc(sizeof(double) * (size_t)L * d);       /* one KV head's keys */
    double* Qd = (double*)malloc(sizeof(double) * (size_t)rows * d);    /* the group's query rows */
    double* mrow = (double*)malloc(sizeof(double) * rows);
    double* zrow = (double*)malloc(sizeof(double) * rows);
    if (!Kd || !Qd || !mrow || !zrow) { free(Kd); free(Qd); free(mrow); free(zrow); return -1; }

    for (int g = 0; g < h_kv; ++g) {
        for (long j = 0; j < L; ++j)
            for (int c = 0; c < d; ++c) Kd[j * d + c] = bf16_to_f64(K[((size_t)j * h_kv + g) * d + c]);
        /* row r = (hh, i): query head h = g*G + hh, soft token i */
        for (int hh = 0; hh < G; ++hh)
            for (int i = 0; i < n_q; ++i)
                for (int c = 0; c < d; ++c)
                    Qd[((size_t)hh * n_q + i) * d + c] = bf16_to_f64(Q[((size_t)i * h_q + (g * G + hh)) * d + c]);

        /* per query row: m = max_j s, Z = sum_j exp(s - m) */
#pragma omp parallel for schedule(dynamic, 1)
        for (int r = 0; r < rows; ++r) {
            const double* q = Qd + (size_t)r * d;
            double m = -INFINITY;
            for (long j = 0; j < L; ++j) {
                const double* k = Kd + (size_t)j * d;
                double acc = 0.0;
                for (int c = 0; c < d; ++c) acc += q[c] * k[c];
                double s = acc * scale;
                if (s > m) m = s;
            }
            double z = 0.0;
            for (long j = 0; j < L; ++j) {
                const double* k = Kd + (size_t)j * d;
                double acc = 0.0;
                for (int c = 0; c < d; ++c) acc += q[c] * k[c];
                z += exp(acc * scale - m);
            }
            mrow[r] = m;
            zrow[r] = z;
        }

        /* per key: sum of the normalised probabilities over the group's rows */
#pragma omp parallel for schedule(static)
        for (long j = 0; j < L; ++j) {
            const double* k = Kd + (size_t)j * d;
            double total = 0.0;
            for (int r = 0; r < rows; ++r) {
                const double* q = Qd + (size_t)r * d;
                double acc = 0.0;
                for (int c = 0; c < d; ++c) acc += q[c] * k[c];
                total += exp(acc * scale - mrow[r]) / zrow[r];
            }
            score[(size_t)g * L + j] = total;
        }
    }
    free(Kd); free(Qd); free(mrow); free(zrow);
    return 0;
}

/*
 * Importance scores as a slice of a wider softmax (Section 4.2, Eq. 1 and Eq. 3; Section 4.3).
 *
 * In the model's own prefill the soft tokens are appended after the prompt, so soft token i also
 * attends to the soft tokens up to itself and its softmax normaliser covers more than the prompt
 * keys.  Given that normaliser as lse[i,h] = log sum_{j in domain} exp(s[h,i,j]) (natural log, the
 * value attention kernels keep), the attention the prompt key j receives is
 *
 *   p[h,i,j]   = exp(s[h,i,j] - lse[i,h])
 *   score[g,j] = sum_{h in group g} sum_i p[h,i,j]
 *
 * With lse taken over the prompt keys alone this is jqo_score.  lse is [n_q, h_q] double.
 */
int jqo_score_lse(int n_q, int h_q, int h_kv, int d, long L, double scale, const uint16_t* Q, const uint16_t* K,
                  const double* lse, double* score) {
    if (n_q < 1 || h_q < 1 || h_kv < 1 || d < 1 || L < 1 || h_q % h_kv != 0 || !Q || !K || !lse || !score) return -1;
    const int G = h_q / h_kv;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)d);
#pragma omp parallel for schedule(static) collapse(2)
    for (int g = 0; g < h_kv; ++g)
        for (long j = 0; j < L; ++j) {
            const uint16_t* k = K + ((size_t)j * h_kv + g) * d;
            double total = 0.0;
            for (int hh = 0; hh < G; ++hh)
                for (int i = 0; i < n_q; ++i) {
                    const int h = g * G + hh;
                    const uint16_t* q = Q + ((size_t)i * h_q + h) * d;
                    double acc = 0.0;
                    for (int c = 0; c < d; ++c) acc += bf16_to_f64(q[c]) * bf16_to_f64(k[c]);
                    total += exp(acc * scale - lse[(size_t)i * h_q + h]);
                }
            score[(size_t)g * L + j] = total;
        }
    return 0;
}

/*
 * Importance scores with the soft tokens' own keys in the softmax (Section 4.2: the soft tokens are
 * appended to the prompt; Section 4.3 / Eq. 3: their attention over the prompt is the score).
 *
 * In a causal model soft token i attends to the L prompt keys and to soft tokens 0..i (itself
 * included), so with the soft tokens' keys Kt given explicitly
 *
 *   Z[h,i]     = sum_{j < L} exp(s[h,i,j]) + sum_{i' <= i} exp(scale * Q[i,h,:] . Kt[i',g,:])
 *   p[h,i,j]   = exp(s[h,i,j]) / Z[h,i]                      (prompt keys only are scored)
 *   score[g,j] = sum_{h in group g} sum_i p[h,i,j]
 *
 * Reading: "causal" includes the diagonal (a token attends to itself), as in every decoder-only model
 * the paper evaluates.  The same function scores a prompt under its own last n_q tokens (the
 * observation window of the SnapKV-style baselines in Section 5.1): pass the window's queries and keys.
 * Kt is [n_q, h_kv, d] bf16 bits.  Two passes per row, like jqo_score, with the maximum taken over both parts.
 */
int jqo_score_tail(int n_q, int h_q, int h_kv, int d, long L, double scale, const uint16_t* Q, const uint16_t* K,
                   const uint16_t* Kt, double* score) {
    if (n_q < 1 || h_q < 1 || h_kv < 1 || d < 1 || L < 1 || h_q % h_kv != 0 || !Q || !K || !Kt || !score) return -1;
    const int G = h_q / h_kv;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)d);
    double* mz = (double*)malloc(sizeof(double) * 2 * (size_t)n_q * h_q);  /* (m, Z) per (i, h) */
    if (!mz) return -1;
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
    for (int i = 0; i < n_q; ++i)
        for (int h = 0; h < h_q; ++h) {
            const int g = h / G;
            const uint16_t* q = Q + ((size_t)i * h_q + h) * d;
            double m = -INFINITY;
            for (int pass = 0; pass < 2; ++pass) {
                double z = 0.0;
                for (long j = 0; j < L + i + 1; ++j) {  /* the L prompt keys, then soft tokens 0..i */
                    const uint16_t* k = j < L ? K + ((size_t)j * h_kv + g) * d : Kt + ((size_t)(j - L) * h_kv + g) * d;
                    double acc = 0.0;
                    for (int c = 0; c < d; ++c) acc += bf16_to_f64(q[c]) * bf16_to_f64(k[c]);
                    const double sv = acc * scale;
                    if (pass == 0) { if (sv > m) m = sv; }
                    else z += exp(sv - m);
                }
                if (pass == 1) { mz[2 * ((size_t)i * h_q + h)] = m; mz[2 * ((size_t)i * h_q + h) + 1] = z; }
            }
        }
#pragma omp parallel for schedule(static) collapse(2)
    for (int g = 0; g < h_kv; ++g)
        for (long j = 0; j < L; ++j) {
            const uint16_t* k = K + ((size_t)j * h_kv + g) * d;
            double total = 0.0;
            for (int hh = 0; hh < G; ++hh)
                for (int i = 0; i < n_q; ++i) {
                    const int h = g * G + hh;
                    const uint16_t* q = Q + ((size_t)i * h_q + h) * d;
                    double acc = 0.0;
                    for (int c = 0; c < d; ++c) acc += bf16_to_f64(q[c]) * bf16_to_f64(k[c]);
                    total += exp(acc * scale - mz[2 * ((size_t)i * h_q + h)]) / mz[2 * ((size_t)i * h_q + h) + 1];
                }
            score[(size_t)g * L + j] = total;
        }
    free(mz);
    return 0;
}

/*
 * The same map when the queries are the prompt's OWN last n_q tokens -- the observation window of the
 * window-query baselines of Section 5.1 (H2O as implemented there, SnapKV, PyramidKV): K holds all L
 * prompt keys, its last n_q rows being the window tokens' keys, Q the window tokens' queries.  Window token i
 * sits at position w_i = L - n_q + i and, the model being causal, attends to positions 0..w_i only:
 *
 *   Z[h,i]     = sum_{j <= w_i} exp(scale * Q[i,h,:] . K[j,g,:])
 *   score[g,j] = sum_{h in group g} sum_i exp(scale * Q[i,h,:] . K[j,g,:]) / Z[h,i]   for j < L - n_q
 *   score[g,j] = 0                                                                    for the window itself
 *
 * (the window's own positions are observers, not candidates: they are kept unconditionally).
 */
int jqo_score_window(int n_q, int h_q, int h_kv, int d, long L, double scale, const uint16_t* Q, const uint16_t* K,
                     double* score) {
    if (n_q < 1 || h_q < 1 || h_kv < 1 || d < 1 || L < n_q || h_q % h_kv != 0 || !Q || !K || !score) return -1;
    const int G = h_q / h_kv;
    const long P = L - n_q;  /* prefix length */
    if (scale <= 0.0) scale = 1.0 / sqrt((double)d);
    for (size_t x = 0; x < (size_t)h_kv * (size_t)L; ++x) score[x] = 0.0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int g = 0; g < h_kv; ++g) {
        double* s = (double*)malloc(sizeof(double) * (size_t)L);
        for (int hh = 0; hh < G && s; ++hh)
            for (int i = 0; i < n_q; ++i) {
                const int h = g * G + hh;
                const long last = P + i;  /* the row's last visible key (itself) */
                const uint16_t* q = Q + ((size_t)i * h_q + h) * d;
                double m = -INFINITY, z = 0.0;
                for (long j = 0; j <= last; ++j) {
                    const uint16_t* k = K + ((size_t)j * h_kv + g) * d;
                    double acc = 0.0;
                    for (int c = 0; c < d; ++c) acc += bf16_to_f64(q[c]) * bf16_to_f64(k[c]);
                    s[j] = acc * scale;
                    if (s[j] > m) m = s[j];
                }
                for (long j = 0; j <= last; ++j) z += exp(s[j] - m);
                for (long j = 0; j < P; ++j) score[(size_t)g * L + j] += exp(s[j] - m) / z;
            }
        free(s);
    }
    return 0;
}

/*
 * 1-D average pooling of one head's scores (the pooling settings of the
 * Section 5.1 baselines paragraph).  Reading: stride 1, same-length output,
 * zeros outside [0, L), divisor always pool_k (so the first and last
 * (pool_k-1)/2 outputs are damped).  pool_k must be odd and >= 1.
 */
int jqo_pool(long L, int pool_k, const double* score, double* pooled) {
    if (L < 1 || pool_k < 1 || pool_k % 2 == 0 || !score || !pooled) return -1;
    const long r = (pool_k - 1) / 2;
    for (long j = 0; j < L; ++j) {
        double acc = 0.0;
        for (long t = -r; t <= r; ++t) {
            long p = j + t;
            if (p >= 0 && p < L) acc += score[p];
        }
        pooled[j] = acc / (double)pool_k;
    }
    return 0;
}

/*
 * Training objective, forward value only (Section 4.2, Eq. 3-5): the attention maps of the soft tokens and of
 * the response tokens over the prompt, each averaged over its tokens, and their mean squared error.
 * With the scores of jqo_score (sums over n tokens and the G heads of the group) the averaged map is
 * score / (n * G), so
 *   mse[g] = (1 / L) * sum_j ( score_a[g,j] / rows_a  -  score_b[g,j] / rows_b )^2,   rows = n * G.
 * Readings: the average also runs over the query heads that share the KV head; Eq. 5 divides by the
 * length of the maps (it prints the symbol of the head dimension, which has no place there).
 */
int jqo_map_mse(long L, int h_kv, double rows_a, double rows_b, const double* score_a, const double* score_b, double* mse) {
    if (L < 1 || h_kv < 1 || !(rows_a > 0.0) || !(rows_b > 0.0) || !score_a || !score_b || !mse) return -1;
    for (int g = 0; g < h_kv; ++g) {
        double acc = 0.0;
        for (long j = 0; j < L; ++j) {
            const double diff = score_a[(size_t)g * L + j] / rows_a - score_b[(size_t)g * L + j] / rows_b;
            acc += diff * diff;
        }
        mse[g] = acc / (double)L;
    }
    return 0;
}

typedef struct { double v; int32_t i; } jqo_item;

static int jqo_item_cmp(const void* a, const void* b) {
    const jqo_item* x = (const jqo_item*)a;
    const jqo_item* y = (const jqo_item*)b;
    if (x->v > y->v) return -1;
    if (x->v < y->v) return 1;
    return (x->i > y->i) - (x->i < y->i);
}

static int jqo_i32_cmp(const void* a, const void* b) {
    int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
    return (x > y) - (x < y);
}

/*
 * Top-B retention for one head (Section 4.3: keep the pairs with the top-k
 * highest scores, discard the rest).  Reading: among equal scores the lower
 * position wins; the kept positions are reported in ascending order.
 * A full sort on (score descending, position ascending), first B taken.
 */
int jqo_select_topk(long L, long B, const double* pooled, int32_t* idx) {
    if (L < 1 || B < 1 || B > L || L > 2147483647L || !pooled || !idx) return -1;
    jqo_item* it = (jqo_item*)malloc(sizeof(jqo_item) * (size_t)L);
    if (!it) return -1;
    for (long j = 0; j < L; ++j) { it[j].v = pooled[j]; it[j].i = (int32_t)j; }
    qsort(it, (size_t)L, sizeof(jqo_item), jqo_item_cmp);
    for (long b = 0; b < B; ++b) idx[b] = it[b].i;
    qsort(idx, (size_t)B, sizeof(int32_t), jqo_i32_cmp);
    free(it);
    return 0;
}

/*
 * Top-B retention with positions that are kept no matter what they score: the
 * baselines of Section 5.1 retain the beginning of the input and / or the local
 * window (StreamingLLM by construction, the window-query methods because the
 * window's own tokens stay).  Reading: the first keep_first and the last
 * keep_last positions are in the kept set; they count towards B; the other
 * B - keep_first - keep_last places go to the highest-scoring remaining
 * positions (equal scores: lower position first); output ascending.
 * Written as that definition: forced positions are copied, the rest is sorted.
 */
int jqo_select_topk_keep(long L, long B, long keep_first, long keep_last, const double* pooled, int32_t* idx) {
    if (L < 1 || B < 1 || B > L || L > 2147483647L || !pooled || !idx) return -1;
    if (keep_first < 0 || keep_last < 0 || keep_first + keep_last > B) return -1;
    long n = 0;
    for (long j = 0; j < keep_first; ++j) idx[n++] = (int32_t)j;
    for (long j = L - keep_last; j < L; ++j) idx[n++] = (int32_t)j;
    const long lo = keep_first, hi = L - keep_last;  /* the positions that compete: [lo, hi) */
    if (hi > lo && n < B) {
        jqo_item* it = (jqo_item*)malloc(sizeof(jqo_item) * (size_t)(hi - lo));
        if (!it) return -1;
        for (long j = lo; j < hi; ++j) { it[j - lo].v = pooled[j]; it[j - lo].i = (int32_t)j; }
        qsort(it, (size_t)(hi - lo), sizeof(jqo_item), jqo_item_cmp);
        for (long b = 0; n < B; ++b) idx[n++] = it[b].i;
        free(it);
    }
    qsort(idx, (size_t)B, sizeof(int32_t), jqo_i32_cmp);
    return 0;
}

/*
 * Pruned cache (Section 4.3: decoding continues on the pruned KV cache):
 *   K_out[b,g,:] = K[idx[g,b], g, :],   V_out likewise, as 16-bit patterns.
 * K,V [L, h_kv, d]; idx [h_kv, B]; K_out,V_out [B, h_kv, d].
 */
int jqo_compact(long L, int h_kv, int d, long B, const uint16_t* K, const uint16_t* V,
                const int32_t* idx, uint16_t* K_out, uint16_t* V_out) {
    if (L < 1 || h_kv < 1 || d < 1 || B < 1 || !K || !V || !idx || !K_out || !V_out) return -1;
    for (int g = 0; g < h_kv; ++g)
        for (long b = 0; b < B; ++b) {
            long j = idx[(size_t)g * B + b];
            if (j < 0 || j >= L) return -1;
            for (int c = 0; c < d; ++c) {
                K_out[((size_t)b * h_kv + g) * d + c] = K[((size_t)j * h_kv + g) * d + c];
                V_out[((size_t)b * h_kv + g) * d + c] = V[((size_t)j * h_kv + g) * d + c];
            }
        }
    return 0;
}

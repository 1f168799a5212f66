/*
 * fp64 CPU oracle for shared-prefix decode attention.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the yardstick the GPU library is checked against.  It is plain,
 * slow and independent: it shares no code, header, table or layout helper with
 * the HIP sources, and nothing on the product path may call it.  Only the
 * tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * What it computes is the plain definition, not the Hydragen algorithm:
 *
 *   hgo_attention  For every selected sequence b and query head h, scaled
 *                  dot-product attention (paper Eq. 1) of the single decode
 *                  query q[b,h] over the CONCATENATION, in order, of every
 *                  shared KV block that covers b (root level first; Sec. 2.3:
 *                  prefix keys/values are identical across sequences, so the
 *                  concatenated cache is the ground truth; Sec. 3.3 for trees)
 *                  followed by b's own suffix rows, together with the
 *                  log-sum-exp of the scaled scores (Eq. 4, natural log).
 *                  With nq > 1 queries per sequence (App. B's num_queries:
 *                  the last nq tokens of a sequence queried at once) query t
 *                  sees every shared row and suffix rows [0, L_b - (nq-1-t)):
 *                  the plain causal definition, a token does not see the
 *                  tokens after it (the paper gives only the shape).
 *                  With zero levels it is attention over the suffix alone;
 *                  with all lengths zero it is attention over shared blocks
 *                  alone: those give the per-part (O, LSE) pairs.
 *   hgo_merge      Eq. 5 (the decomposition identity of Sec. 3.1) for n parts:
 *                  O = sum_i O_i e^{LSE_i} / sum_i e^{LSE_i}, evaluated after
 *                  subtracting the largest LSE (as App. B's two-part combine
 *                  routine does), plus the merged LSE.
 *
 * All inputs are bf16 bit patterns widened exactly to fp64; every sum runs in
 * index order in fp64.  Empty key lists give O = 0 and LSE = -inf (the paper
 * is silent; this is the reading that makes an empty part the identity of the
 * merge).  GQA maps query head h to KV head h / (Hq/Hkv) (contiguous groups).
 *
 * Pinned by tests/test_oracle_pins.py: closed forms (one key, two keys, equal
 * scores, constant V), shift/permutation/duplication invariants, brute force
 * in exact-sum Python, a library softmax, GQA-by-repetition, tree-by-physical
 * concatenation, the decomposition identity at every split point, and a
 * hand-derived worked example in tests/golden/.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline double widen(uint16_t bits)
{
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

typedef struct {
    const uint16_t *K, *V; /* [rows, Hkv, D] */
    int64_t begin, count;  /* row range */
} span_t;

/* attention of one query vector over a list of row spans, for KV head kvh */
static void attend(const double *q, int D, int Hkv, int kvh, const span_t *spans, int nspans,
                   double scale, double *scores, double *O, double *LSE)
{
    int64_t n = 0;
    double m = -INFINITY;
    for (int s = 0; s < nspans; ++s) {
        for (int64_t r = 0; r < spans[s].count; ++r) {
            const uint16_t *k = spans[s].K + ((spans[s].begin + r) * Hkv + kvh) * (int64_t)D;
            double dot = 0.0;
            for (int d = 0; d < D; ++d) dot += q[d] * widen(k[d]);
            double sc = dot * scale;
            scores[n++] = sc;
            if (sc > m) m = sc;
        }
    }
    for (int d = 0; d < D; ++d) O[d] = 0.0;
    if (n == 0) {
        *LSE = -INFINITY;
        return;
    }
    double denom = 0.0;
    n = 0;
    for (int s = 0; s < nspans; ++s) {
        for (int64_t r = 0; r < spans[s].count; ++r) {
            const uint16_t *v = spans[s].V + ((spans[s].begin + r) * Hkv + kvh) * (int64_t)D;
            double w = exp(scores[n++] - m);
            denom += w;
            for (int d = 0; d < D; ++d) O[d] += w * widen(v[d]);
        }
    }
    for (int d = 0; d < D; ++d) O[d] /= denom;
    *LSE = m + log(denom);
}

#define HGO_MAX_LEVELS 8

/*
 * Q [B,nq,Hq,D] bf16 bits (nq >= 1 queries per sequence).  Level l: K/V [rows_l,Hkv,D], Gn[l] blocks, kv_off[l][Gn+1], seq_off[l][Gn+1].
 * Suffix: Ks/Vs [T,Hkv,D], offsets[B], lengths[B] (Ks may be NULL when every length is 0 or lengths is NULL).
 * seqs: optional list of n_seqs sequence ids to evaluate (NULL = all B, n_seqs ignored).
 * Outputs are indexed by position in that list: O [n,nq,Hq,D], LSE [n,nq,Hq], fp64.
 * Returns 0, or -1 on a bad argument.
 */
int hgo_attention(const uint16_t *Q, int B, int nq, int Hq, int Hkv, int D,
                  int n_levels, const uint16_t *const *Kl, const uint16_t *const *Vl,
                  const int32_t *Gn, const int32_t *const *kv_off, const int32_t *const *seq_off,
                  const uint16_t *Ks, const uint16_t *Vs, const int32_t *offsets, const int32_t *lengths,
                  double scale, const int32_t *seqs, int n_seqs, double *O, double *LSE)
{
    if (B < 0 || nq < 1 || Hq <= 0 || Hkv <= 0 || D <= 0 || Hq % Hkv != 0) return -1;
    if (n_levels < 0 || n_levels > HGO_MAX_LEVELS) return -1;
    const int G = Hq / Hkv;
    const int n = seqs ? n_seqs : B;
    int bad = 0;

#pragma omp parallel
    {
        double *q = (double *)malloc(sizeof(double) * (size_t)D);
        double *scores = NULL;
        int64_t cap = 0;
#pragma omp for schedule(dynamic, 1)
        for (int i = 0; i < n; ++i) {
            const int b = seqs ? seqs[i] : i;
            if (b < 0 || b >= B) {
#pragma omp atomic write
                bad = 1;
                continue;
            }
            span_t spans[HGO_MAX_LEVELS + 1];
            int ns = 0;
            int64_t total = 0;
            for (int l = 0; l < n_levels; ++l) {
                for (int g = 0; g < Gn[l]; ++g) {
                    if (seq_off[l][g] <= b && b < seq_off[l][g + 1]) {
                        spans[ns].K = Kl[l];
                        spans[ns].V = Vl[l];
                        spans[ns].begin = kv_off[l][g];
                        spans[ns].count = (int64_t)kv_off[l][g + 1] - kv_off[l][g];
                        total += spans[ns].count;
                        ++ns;
                        break;
                    }
                }
            }
            const int nshared = ns;
            const int64_t len_b = lengths && lengths[b] > 0 ? lengths[b] : 0;
            if (total + len_b > cap) {
                free(scores);
                cap = total + len_b;
                scores = (double *)malloc(sizeof(double) * (size_t)cap);
            }
            for (int t = 0; t < nq; ++t) {
                /* query t is the (nq-1-t)-th token from the end: it sees the suffix up to and including itself */
                const int64_t visible = len_b - (nq - 1 - t);
                ns = nshared;
                if (visible > 0) {
                    spans[ns].K = Ks;
                    spans[ns].V = Vs;
                    spans[ns].begin = offsets[b];
                    spans[ns].count = visible;
                    ++ns;
                }
                for (int h = 0; h < Hq; ++h) {
                    const uint16_t *qb = Q + (((int64_t)b * nq + t) * Hq + h) * D;
                    for (int d = 0; d < D; ++d) q[d] = widen(qb[d]);
                    attend(q, D, Hkv, h / G, spans, ns, scale, scores,
                           O + (((int64_t)i * nq + t) * Hq + h) * D, LSE + ((int64_t)i * nq + t) * Hq + h);
                }
            }
        }
        free(scores);
        free(q);
    }
    return bad ? -1 : 0;
}

/*
 * n-way merge over `rows` query rows: parts[i] -> O_i [rows,D], lses[i] -> LSE_i [rows], all fp64.
 * A part with LSE = -inf has weight 0; if every part is empty the row is O = 0, LSE = -inf.
 * LSE_out may be NULL.
 */
int hgo_merge(int n, const double *const *parts, const double *const *lses, int64_t rows, int D,
              double *O_out, double *LSE_out)
{
    if (n <= 0 || rows < 0 || D <= 0) return -1;
    for (int64_t r = 0; r < rows; ++r) {
        double m = -INFINITY;
        for (int i = 0; i < n; ++i)
            if (lses[i][r] > m) m = lses[i][r];
        double *o = O_out + r * D;
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        if (m == -INFINITY) {
            if (LSE_out) LSE_out[r] = -INFINITY;
            continue;
        }
        double denom = 0.0;
        for (int i = 0; i < n; ++i) {
            double w = exp(lses[i][r] - m);
            denom += w;
            const double *oi = parts[i] + r * D;
            for (int d = 0; d < D; ++d) o[d] += w * oi[d];
        }
        for (int d = 0; d < D; ++d) o[d] /= denom;
        if (LSE_out) LSE_out[r] = m + log(denom);
    }
    return 0;
}

int hgo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * CPU checker for the TableCache online path.  TEST INFRASTRUCTURE ONLY: the
 * product (the HIP library) never links, loads or calls this file.  Plain C,
 * fp64, no tiling, no online softmax, no reordering beyond the definitions.
 *
 * What the path computes (paper Sec. 1 and Sec. 4.1.2: the KV caches of the
 * tables matched in a prompt are concatenated in match order and handed to the
 * model; App. E.4: only the query part is computed and it attends to all
 * preceding table content) has a plain definition, and this file is that
 * definition written out:
 *
 *   orc_concat_tokens   - the stitched sequence: table segments laid end to end
 *   orc_prefill_attn    - softmax attention of the suffix rows over
 *                         {all stitched schema keys} U {suffix keys 0..r}
 *   orc_reencode_keys   - Sec. 4.1.1, last paragraph: table keys are stored without
 *                         positional encoding and get it at inference from their global
 *                         position in the concatenated sequence (rotary encoding)
 *
 * Parity pins (tests/test_oracle_*.py): rows P..P+S-1 of a library causal
 * attention over the whole sequence; softmax rows summing to one; brute-force
 * enumeration of the visible-key set; closed forms (equal keys, constant V,
 * one dominating logit); GQA reductions; position-coded gather; the rotary
 * re-encoding against complex multiplication, its group properties and the
 * relative-position invariance of rotated dot products.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Stitched sequence of one layer (Sec. 4.1.2, last sentence: concatenation in
 * the order the tables were matched).  seg[j] points at table j's rows for this
 * layer, n_tok[j] rows of row_bytes each; out receives sum(n_tok) rows.
 * Token-granular byte copy; returns the number of rows written.
 */
int64_t orc_concat_tokens(const uint8_t *const *seg, const int32_t *n_tok, int32_t m,
                          int64_t row_bytes, uint8_t *out)
{
    int64_t p = 0;
    for (int32_t j = 0; j < m; ++j)
        for (int32_t u = 0; u < n_tok[j]; ++u) {
            for (int64_t b = 0; b < row_bytes; ++b)
                out[p * row_bytes + b] = seg[j][(int64_t)u * row_bytes + b];
            ++p;
        }
    return p;
}

/*
 * Suffix prefill attention of one query in one layer (App. E.4; spec mask:
 * full over the schema prefix, causal inside the suffix).
 *
 *   q      [S][Hq][D]     suffix queries
 *   k_seq  [P][Hkv][D]    stitched schema keys,   v_seq likewise
 *   k_new  [S][Hkv][D]    suffix keys,            v_new likewise
 *   out    [S][Hq][D]
 *   w_out  optional [S][Hq][P+S]: the normalised softmax weights (0 where masked)
 *
 * Query head h reads KV head h / (Hq/Hkv).  Row r sees key j of the logical
 * sequence (schema first, suffix after) iff  j < P  or  j - P <= r.
 */
int orc_prefill_attn(const double *q, const double *k_seq, const double *v_seq,
                     const double *k_new, const double *v_new,
                     int32_t P, int32_t S, int32_t Hq, int32_t Hkv, int32_t D,
                     double sm_scale, double *out, double *w_out)
{
    if (P < 0 || S < 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || Hq % Hkv != 0) return -1;
    const int32_t G = Hq / Hkv;
    const int32_t N = P + S;
    int failed = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int32_t r = 0; r < S; ++r)
        for (int32_t h = 0; h < Hq; ++h) {
            const int32_t g = h / G;
            const double *qr = q + ((int64_t)r * Hq + h) * D;
            double *s = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
            if (!s) { failed = 1; continue; }
            /* scores of the visible keys, running maximum */
            double m = -INFINITY;
            for (int32_t j = 0; j < N; ++j) {
                if (!(j < P || (j - P) <= r)) { s[j] = -INFINITY; continue; }
                const double *kj = (j < P) ? k_seq + ((int64_t)j * Hkv + g) * D
                                           : k_new + ((int64_t)(j - P) * Hkv + g) * D;
                double dot = 0.0;
                for (int32_t d = 0; d < D; ++d) dot += qr[d] * kj[d];
                s[j] = sm_scale * dot;
                if (s[j] > m) m = s[j];
            }
            /* weights and their sum */
            double denom = 0.0;
            for (int32_t j = 0; j < N; ++j) {
                if (!(j < P || (j - P) <= r)) { s[j] = 0.0; continue; }
                s[j] = exp(s[j] - m);
                denom += s[j];
            }
            double *o = out + ((int64_t)r * Hq + h) * D;
            for (int32_t d = 0; d < D; ++d) o[d] = 0.0;
            for (int32_t j = 0; j < N; ++j) {
                if (!(j < P || (j - P) <= r)) continue;
                const double *vj = (j < P) ? v_seq + ((int64_t)j * Hkv + g) * D
                                           : v_new + ((int64_t)(j - P) * Hkv + g) * D;
                const double w = s[j] / denom;
                for (int32_t d = 0; d < D; ++d) o[d] += w * vj[d];
            }
            if (w_out) {
                double *wr = w_out + ((int64_t)r * Hq + h) * N;
                for (int32_t j = 0; j < N; ++j) wr[j] = s[j] / denom;
            }
            free(s);
        }
    return failed ? -2 : 0;
}

/*
 * Positional re-encoding of stitched keys (Sec. 4.1.1: keys are stored position-free;
 * at inference every token is encoded by its global position in the concatenation).
 * The paper names no encoding; its models are rotary-position decoders, so this is the
 * rotary encoding in the half-split convention of those models: with D the head size,
 * frequency w_i = theta^(-2i/D) for i < D/2, and a = pos * w_i,
 *     k'[i]       = k[i] cos a - k[i + D/2] sin a
 *     k'[i + D/2] = k[i + D/2] cos a + k[i] sin a
 * k is [n_tokens][n_heads][D] fp64, rotated in place; pos[t] is token t's position.
 */
int orc_reencode_keys(double *k, int64_t n_tokens, int32_t n_heads, int32_t D, const int64_t *pos, double theta)
{
    if (D <= 0 || (D & 1) || n_heads <= 0 || n_tokens < 0 || !(theta > 0.0)) return -1;
    const int32_t half = D / 2;
    for (int64_t t = 0; t < n_tokens; ++t)
        for (int32_t h = 0; h < n_heads; ++h) {
            double *row = k + (t * n_heads + h) * D;
            for (int32_t i = 0; i < half; ++i) {
                const double w = pow(theta, -2.0 * (double)i / (double)D);
                const double a = (double)pos[t] * w;
                const double c = cos(a), sn = sin(a);
                const double x = row[i], y = row[i + half];
                row[i] = x * c - y * sn;
                row[i + half] = y * c + x * sn;
            }
        }
    return 0;
}

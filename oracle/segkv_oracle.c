/*
 * segkv_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain, slow, fp64 CPU statement of what the fused decode-step attention over
 * a segment KV cache computes (arxiv 2401.05391, Sections 3.1-3.3).  Only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it.  It
 * shares no code, header, table or helper with the GPU library.
 *
 * What is computed, and where the paper says so:
 *   - response K/V live in a pre-allocated sequence-first buffer
 *     [Tcap, B*W, Hkv, D]; the current step's K/V are written into row T-1
 *     of it before attention (Section 3.1, decoding phase);
 *   - prompt K/V are stored once per request as [B, Lp, Hkv, D] and shared by
 *     the W beams of that request (Section 3.2);
 *   - for beam position j and past step s the response row that is attended is
 *     the one the beam-index tensor names (Section 3.3, "Index select fusion");
 *   - attention over the prompt segment and over the selected response rows
 *     is accumulated into one softmax-weighted context (Section 3.3, "Kernel
 *     implementation").  The method is an exact re-arrangement of standard
 *     attention over the gathered per-beam history, so the oracle is that
 *     definition written out: one softmax over all Lp+T logits.
 *
 * Readings where the paper is silent (all restated in the design notes):
 *   - the index tensor is supplied as raw per-step parent slots
 *     parent[s][b*W+j] in [0,W): the slot, at step s-1, of the hypothesis that
 *     slot j at step s extends.  Ancestors are resolved here by walking back
 *     from the beam's own slot at step T-1.  parent[0] refers to the shared
 *     prompt and is ignored.
 *   - grouped-query attention: query head hq reads KV head hq / (Hq/Hkv).
 *   - ALiBi: slope[hq] * key_position is added to the scaled logit, key
 *     positions being 0..Lp-1 for the prompt and Lp+s for response step s.
 *   - the single decode query sits at position Lp+T-1 and sees all Lp+T keys.
 *
 * Pins: tests/test_oracle_*.py (brute force over an explicitly gathered dense
 * cache built by simulating per-step index_select + cat, library SDPA for
 * beam=1, closed forms, the paper's worked index datum).
 * ALiBi slope *formula* is an input here, hence not pinned by this file.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t B, beam, Hq, Hkv, D;
    int32_t Lp;
    int32_t T;
    int32_t Tcap;
} oracle_dims;

/* IEEE binary16 bit pattern -> double, exactly (every fp16 value is a double). */
static double half_bits_decode(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0) {
        v = ldexp((double)f, -24);            /* zero and subnormals */
    } else if (e == 31) {
        v = f ? NAN : INFINITY;
    } else {
        v = ldexp((double)(f + 1024), e - 25); /* (1 + f/1024) * 2^(e-15) */
    }
    return sign ? -v : v;
}

/* All 65536 decoded values, filled once before any parallel region. */
static double half_table[65536];
static int half_table_ready = 0;

static void half_table_init(void)
{
    if (half_table_ready) return;
    for (uint32_t h = 0; h < 65536u; ++h) half_table[h] = half_bits_decode((uint16_t)h);
    half_table_ready = 1;
}

static inline double half_bits_to_double(uint16_t h) { return half_table[h]; }

int segkv_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Section 3.1: Key_t / Value_t are kept in row t of the pre-allocated
 * sequence-first response buffers; a plain contiguous row copy. */
int segkv_oracle_append_kv(uint16_t *resp_k, uint16_t *resp_v,
                           const uint16_t *k_new, const uint16_t *v_new,
                           int32_t t, const oracle_dims *d)
{
    if (t < 0 || t >= d->Tcap) return -1;
    size_t row = (size_t)d->B * d->beam * d->Hkv * d->D;
    memcpy(resp_k + (size_t)t * row, k_new, row * sizeof(uint16_t));
    memcpy(resp_v + (size_t)t * row, v_new, row * sizeof(uint16_t));
    return 0;
}

/* Section 3.3, index select: anc[s][b*W+j] = slot whose response K/V row at
 * step s belongs to the history of the hypothesis now in slot j.
 * A beam wrote its own row at the current step; each earlier row is found by
 * following the parent pointer of the row after it. */
void segkv_oracle_ancestors(const int32_t *parent, int32_t B, int32_t W,
                            int32_t T, int32_t *anc)
{
    int32_t N = B * W;
    for (int32_t b = 0; b < B; ++b) {
        for (int32_t j = 0; j < W; ++j) {
            int32_t n = b * W + j;
            anc[(size_t)(T - 1) * N + n] = j;
            for (int32_t s = T - 1; s >= 1; --s) {
                int32_t cur = anc[(size_t)s * N + n];
                anc[(size_t)(s - 1) * N + n] = parent[(size_t)s * N + b * W + cur];
            }
        }
    }
}

/*
 * Attention for a list of (n, hq) output rows.
 *   pairs      [n_pairs][2] int32: beam row n in [0,B*W), query head hq.
 *              NULL => all B*W*Hq rows in natural order.
 *   out        [n_pairs][D] double.
 *   probs      NULL or [n_pairs][Lp+T] double softmax weights (prompt keys
 *              first, then response steps).
 *   anc        [T][B*W] int32, written (resolved ancestors).
 *   resp_k/v   row T-1 must already hold the current step's K/V (call
 *              segkv_oracle_append_kv first).  Rows >= T are never read.
 *   slopes     NULL or [Hq] double ALiBi slopes.
 * Returns 0, or -1 on invalid dimensions.
 */
int segkv_oracle_sdpa_decode(double *out, double *probs, int32_t *anc,
                             const uint16_t *q,
                             const uint16_t *prompt_k, const uint16_t *prompt_v,
                             const uint16_t *resp_k, const uint16_t *resp_v,
                             const int32_t *parent, const double *slopes,
                             double scale, const oracle_dims *d,
                             const int32_t *pairs, int64_t n_pairs)
{
    const int32_t B = d->B, W = d->beam, Hq = d->Hq, Hkv = d->Hkv, D = d->D;
    const int32_t Lp = d->Lp, T = d->T;
    if (B < 1 || W < 1 || Hq < 1 || Hkv < 1 || D < 1 || Lp < 0 || T < 1 ||
        T > d->Tcap || Hq % Hkv != 0)
        return -1;
    const int32_t N = B * W;
    const int32_t group = Hq / Hkv;
    const int64_t L = (int64_t)Lp + T;
    if (!pairs) n_pairs = (int64_t)N * Hq;

    half_table_init();
    segkv_oracle_ancestors(parent, B, W, T, anc);

#pragma omp parallel
    {
        double *z = (double *)malloc((size_t)L * sizeof(double));
        double *qd = (double *)malloc((size_t)D * sizeof(double));
#pragma omp for schedule(dynamic, 4)
        for (int64_t r = 0; r < n_pairs; ++r) {
            int32_t n = pairs ? pairs[2 * r] : (int32_t)(r / Hq);
            int32_t hq = pairs ? pairs[2 * r + 1] : (int32_t)(r % Hq);
            int32_t b = n / W;
            int32_t g = hq / group;
            double slope = slopes ? slopes[hq] : 0.0;
            for (int32_t e = 0; e < D; ++e)
                qd[e] = half_bits_to_double(q[((size_t)n * Hq + hq) * D + e]);

            /* logits: prompt keys, then the selected response row of each step */
            for (int32_t i = 0; i < Lp; ++i) {
                const uint16_t *k = prompt_k + (((size_t)b * Lp + i) * Hkv + g) * D;
                double dot = 0.0;
                for (int32_t e = 0; e < D; ++e) dot += qd[e] * half_bits_to_double(k[e]);
                z[i] = scale * dot + slope * (double)i;
            }
            for (int32_t s = 0; s < T; ++s) {
                int32_t slot = anc[(size_t)s * N + n];
                const uint16_t *k = resp_k + (((size_t)s * N + b * W + slot) * Hkv + g) * D;
                double dot = 0.0;
                for (int32_t e = 0; e < D; ++e) dot += qd[e] * half_bits_to_double(k[e]);
                z[Lp + s] = scale * dot + slope * (double)(Lp + s);
            }

            /* one softmax over all Lp+T logits */
            double zmax = z[0];
            for (int64_t i = 1; i < L; ++i) if (z[i] > zmax) zmax = z[i];
            double denom = 0.0;
            for (int64_t i = 0; i < L; ++i) { z[i] = exp(z[i] - zmax); denom += z[i]; }
            for (int64_t i = 0; i < L; ++i) z[i] /= denom;
            if (probs) memcpy(probs + (size_t)r * L, z, (size_t)L * sizeof(double));

            /* context = sum of weights times values over both segments */
            double *o = out + (size_t)r * D;
            for (int32_t e = 0; e < D; ++e) o[e] = 0.0;
            for (int32_t i = 0; i < Lp; ++i) {
                const uint16_t *v = prompt_v + (((size_t)b * Lp + i) * Hkv + g) * D;
                for (int32_t e = 0; e < D; ++e) o[e] += z[i] * half_bits_to_double(v[e]);
            }
            for (int32_t s = 0; s < T; ++s) {
                int32_t slot = anc[(size_t)s * N + n];
                const uint16_t *v = resp_v + (((size_t)s * N + b * W + slot) * Hkv + g) * D;
                for (int32_t e = 0; e < D; ++e) o[e] += z[Lp + s] * half_bits_to_double(v[e]);
            }
        }
        free(z);
        free(qd);
    }
    return 0;
}

/*
 * Prefill-phase attention (Section 3.1, prefill phase; Section 3.3: "a special
 * case of that at decoding phase", using only the query and the prompt
 * key/value).  Batch-first tensors, one softmax per (request, token, head):
 *   q, out   [B, N0, Hq, D]      k, v   [B, N0, Hkv, D]
 * Token i attends to keys 0..i of its own request (causal).  ALiBi and the
 * grouped-query head map are read as in the decode oracle.  `rows` selects
 * (b, i, hq) triples to compute (NULL = all, natural order); out is
 * [n_rows][D] double.  Returns 0, or -1 on invalid dimensions.
 */
int segkv_oracle_sdpa_prefill(double *out, const uint16_t *q, const uint16_t *k,
                              const uint16_t *v, const double *slopes, double scale,
                              int32_t B, int32_t N0, int32_t Hq, int32_t Hkv, int32_t D,
                              const int32_t *rows, int64_t n_rows)
{
    if (B < 1 || N0 < 1 || Hq < 1 || Hkv < 1 || D < 1 || Hq % Hkv != 0) return -1;
    const int32_t group = Hq / Hkv;
    if (!rows) n_rows = (int64_t)B * N0 * Hq;
    half_table_init();

#pragma omp parallel
    {
        double *z = (double *)malloc((size_t)N0 * sizeof(double));
        double *qd = (double *)malloc((size_t)D * sizeof(double));
#pragma omp for schedule(dynamic, 16)
        for (int64_t r = 0; r < n_rows; ++r) {
            int32_t b, i, hq;
            if (rows) {
                b = rows[3 * r]; i = rows[3 * r + 1]; hq = rows[3 * r + 2];
            } else {
                hq = (int32_t)(r % Hq);
                i = (int32_t)((r / Hq) % N0);
                b = (int32_t)(r / ((int64_t)Hq * N0));
            }
            const int32_t g = hq / group;
            const double slope = slopes ? slopes[hq] : 0.0;
            for (int32_t e = 0; e < D; ++e)
                qd[e] = half_bits_to_double(q[(((size_t)b * N0 + i) * Hq + hq) * D + e]);
            double zmax = -INFINITY;
            for (int32_t j = 0; j <= i; ++j) {
                const uint16_t *kr = k + (((size_t)b * N0 + j) * Hkv + g) * D;
                double dot = 0.0;
                for (int32_t e = 0; e < D; ++e) dot += qd[e] * half_bits_to_double(kr[e]);
                z[j] = scale * dot + slope * (double)j;
                if (z[j] > zmax) zmax = z[j];
            }
            double denom = 0.0;
            for (int32_t j = 0; j <= i; ++j) { z[j] = exp(z[j] - zmax); denom += z[j]; }
            double *o = out + (size_t)r * D;
            for (int32_t e = 0; e < D; ++e) o[e] = 0.0;
            for (int32_t j = 0; j <= i; ++j) {
                const uint16_t *vr = v + (((size_t)b * N0 + j) * Hkv + g) * D;
                const double w = z[j] / denom;
                for (int32_t e = 0; e < D; ++e) o[e] += w * half_bits_to_double(vr[e]);
            }
        }
        free(z);
        free(qd);
    }
    return 0;
}

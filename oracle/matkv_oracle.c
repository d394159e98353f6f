/*
 * fp64 CPU oracle for the MatKV inference hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the plain definition of what the path computes, written out in
 * double precision with no tiling, no online softmax, no splits and no pages.
 * It shares no code, header, table or constant with the HIP library; only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * What the paper fixes (Section III-B, "Materializing and Retrieving KV
 * Caches"):
 *   - every retrieved chunk's K/V is computed on its own, independent of the
 *     query and of the other chunks, and each chunk starts at input position 0;
 *   - the chunk KVs sit before the user query; only the query (and what is
 *     generated after it) attends to them, there is no chunk-to-chunk attention;
 *   - Section IV ("Avoiding Prefill Using KV in SSD"): the loaded chunk KVs are
 *     combined with the query's KVs as the past cache of ordinary generation.
 * What the paper leaves open and this oracle reads as the LLaMA family does
 * (the models of Section V-A): rotary embedding with half-split pairing and
 * theta_j = base^(-2j/D), softmax scale 1/sqrt(D) unless given, contiguous
 * grouped-query head groups (KV head = query head / G), no projection bias.
 *
 * Pins (tests/test_oracle_pins.py): brute-force masked attention in numpy,
 * rows of the softmax summing to one, single chunk == full causal computation,
 * chunk-order invariance, rotary closed forms, degenerate attention cases,
 * GQA replication, split/merge by log-sum-exp, decode row == prefill row.
 * Not pinnable from the paper (parity unpinned, exposed as parameters): the
 * position of the first question token, the rotary pairing/base.
 *
 * Parallel only across independent (row, head) or token units (OpenMP).
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Rotary embedding of one head vector x[D] at position pos (in place).
 * Pair (j, j + D/2) is rotated by the angle pos * base^(-2j/D). */
void oracle_rope(double* x, int D, double pos, double base) {
    int half = D / 2;
    for (int j = 0; j < half; ++j) {
        double theta = pow(base, -2.0 * (double)j / (double)D);
        double ang = pos * theta;
        double c = cos(ang), s = sin(ang);
        double a = x[j], b = x[j + half];
        x[j] = a * c - b * s;
        x[j + half] = a * s + b * c;
    }
}

/* Per-layer K/V of T tokens from their hidden states (Section III-B step 2,
 * cut down to the K/V projection of one layer):
 *   K[g][i][:] = R(pos0 + i) (Wk_g X[i]),   V[g][i][:] = Wv_g X[i]
 * X  [T][Hd], Wk/Wv [Hkv*D][Hd] row-major (row = output feature),
 * K,V [Hkv][T][D].  A chunk is materialized with pos0 = 0. */
void oracle_materialize(const double* X, const double* Wk, const double* Wv,
                        int T, int Hd, int Hkv, int D, double pos0, double base,
                        double* K, double* V) {
#pragma omp parallel for schedule(static)
    for (int i = 0; i < T; ++i) {
        const double* x = X + (size_t)i * Hd;
        for (int g = 0; g < Hkv; ++g) {
            double* k = K + ((size_t)g * T + i) * D;
            double* v = V + ((size_t)g * T + i) * D;
            for (int d = 0; d < D; ++d) {
                const double* wk = Wk + ((size_t)g * D + d) * Hd;
                const double* wv = Wv + ((size_t)g * D + d) * Hd;
                double sk = 0.0, sv = 0.0;
                for (int c = 0; c < Hd; ++c) {
                    sk += wk[c] * x[c];
                    sv += wv[c] * x[c];
                }
                k[d] = sk;
                v[d] = sv;
            }
            oracle_rope(k, D, pos0 + (double)i, base);
        }
    }
}

/* Attention of R query rows over a flat key list.
 *   Q [R][Hq][D] (already rotated), K,V [Hkv][Nk][D], O [R][Hq][D].
 * Keys 0 .. n_ctx-1 are the cached chunk tokens: visible to every row.
 * Key n_ctx + j is tail token j (question, then generated): visible to row r
 * iff j <= row0 + r.  Prefill of a question: row0 = 0.  Decode step t after an
 * Lq-token question: R = 1, row0 = Lq + t.
 *   s_n = scale * <q_h, k_{g,n}>,  g = h / (Hq/Hkv)
 *   p = exp(s - max s) / sum exp(s - max s),  o_h = sum_n p_n v_{g,n}
 * lse (may be NULL) [R][Hq] receives log sum_n exp(s_n); probs (may be NULL)
 * [R][Hq][Nk] receives p with zeros at masked keys. */
void oracle_attn(const double* Q, const double* K, const double* V,
                 int R, int Hq, int Hkv, int D, int Nk, int n_ctx, int row0,
                 double scale, double* O, double* lse, double* probs) {
    int G = Hq / Hkv;
#pragma omp parallel
    {
        double* s = (double*)malloc(sizeof(double) * (size_t)(Nk > 0 ? Nk : 1));
#pragma omp for collapse(2) schedule(static)
        for (int r = 0; r < R; ++r) {
            for (int h = 0; h < Hq; ++h) {
                int g = h / G;
                const double* q = Q + ((size_t)r * Hq + h) * D;
                double* o = O + ((size_t)r * Hq + h) * D;
                int visible = n_ctx + row0 + r + 1;
                if (visible > Nk) visible = Nk;
                double mx = -INFINITY;
                for (int n = 0; n < visible; ++n) {
                    const double* k = K + ((size_t)g * Nk + n) * D;
                    double acc = 0.0;
                    for (int d = 0; d < D; ++d) acc += q[d] * k[d];
                    s[n] = acc * scale;
                    if (s[n] > mx) mx = s[n];
                }
                double den = 0.0;
                for (int n = 0; n < visible; ++n) {
                    s[n] = exp(s[n] - mx);
                    den += s[n];
                }
                for (int d = 0; d < D; ++d) o[d] = 0.0;
                for (int n = 0; n < visible; ++n) {
                    double p = s[n] / den;
                    const double* v = V + ((size_t)g * Nk + n) * D;
                    for (int d = 0; d < D; ++d) o[d] += p * v[d];
                    if (probs) probs[((size_t)r * Hq + h) * Nk + n] = p;
                }
                if (probs)
                    for (int n = visible; n < Nk; ++n)
                        probs[((size_t)r * Hq + h) * Nk + n] = 0.0;
                if (lse) lse[(size_t)r * Hq + h] = mx + log(den);
            }
        }
        free(s);
    }
}

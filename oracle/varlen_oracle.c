/*
 * CPU oracle for packed variable-length causal attention -- TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain reference the GPU library is checked against.
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may build
 * or call it; the product path never does.  It shares no code with the HIP
 * sources.  Everything is fp64 and written row by row from the definitions:
 *
 *   - Example boundaries (Section 3, Section 3.1 of the paper): the packed
 *     stream carries position ids that run 0..L-1 inside each example and
 *     restart at 0; the restart marks the boundary.  Rows of a [R, T] batch
 *     are separate batch elements, so token 0 of a row always starts an
 *     example.  cu_seqlens is derived from the ids (Section 3, last paragraph).
 *   - "Correct cross-attention" (Table 1): a token attends only to tokens of
 *     its own example, causally (decoder fine-tuning, Section 2).
 *   - The attention arithmetic itself is delegated by the paper to a library
 *     routine; the oracle uses the textbook definition
 *         S_ij = scale * q_i . k_j   (a <= j <= i, a = first token of the example)
 *         P_i  = softmax_j(S_i)      (two passes, explicit max subtraction)
 *         O_i  = sum_j P_ij v_j,     LSE_i = log sum_j exp(S_ij)
 *     and the analytic gradients of  loss = sum(O * dO):
 *         dP_ij = dO_i . v_j,  D_i = sum_j P_ij dP_ij,  dS_ij = P_ij (dP_ij - D_i)
 *         dQ_i  = scale * sum_j dS_ij k_j
 *         dK_j  = scale * sum_{i>=j} dS_ij q_i      (also summed over the query heads
 *         dV_j  =         sum_{i>=j} P_ij  dO_i       that share KV head g = h / (Hq/Hkv))
 *
 * Layouts: Q, O, dO, dQ  [N, Hq, d];  K, V, dK, dV  [N, Hkv, d];  LSE [Hq, N]; all
 * row-major doubles.  No blocking, fusion or reordering beyond the above.
 *
 * The padding-free collator (Section 3.4) that produces the ids is written out
 * as its three rules (concatenate; first label of an example -> -100; ids
 * restart at 0) -- see oracle_collate.
 *
 * Pins (tests/test_oracle_*.py): the paper's worked example (Section 3.5: printed
 * input_ids, labels, position_ids pin the collator and the boundaries),
 * brute-force dense masked attention, per-example unpacking, perturbation of
 * other examples, closed forms (length-1 example, Q = 0 running mean), central
 * finite differences, and a library attention routine on one example.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- boundaries ------------------------------------------------------- */

/* position ids [R, T] (int64) -> cu_seqlens[n+1], seg_id[N], n, max_seqlen.
 * A token starts an example iff it is the first of its row or its id is 0. */
int oracle_pack(const int64_t *pos, int R, int T, int32_t *cu, int32_t *seg_id,
                int32_t *n_out, int32_t *max_seqlen_out)
{
    if (!pos || !cu || !seg_id || !n_out || !max_seqlen_out || R <= 0 || T <= 0) return 1;
    int64_t N = (int64_t)R * T;
    int32_t n = 0;
    for (int64_t t = 0; t < N; ++t) {
        int starts = (t % T == 0) || (pos[t] == 0);
        if (starts) cu[n++] = (int32_t)t;
        seg_id[t] = n - 1;
    }
    cu[n] = (int32_t)N;
    int32_t mx = 0;
    for (int32_t s = 0; s < n; ++s)
        if (cu[s + 1] - cu[s] > mx) mx = cu[s + 1] - cu[s];
    *n_out = n;
    *max_seqlen_out = mx;
    return 0;
}

/* ---- padding-free collator -------------------------------------------- */

/* The collator of Section 3.4 on a minibatch given as a padded [n, Lp] batch
 * with per-example lengths: concatenate the examples into one row of n_out
 * tokens.  input_ids: the tokens in order.  labels: the labels (labels_in, or
 * the ids when labels_in is NULL) with the first label of every example set to
 * -100.  position_ids: 0..L-1 inside every example.  (Section 3.5 prints all
 * three for lengths 4, 8, 5, 11.)  offsets[n+1]: running sum of the lengths.
 * Readings where the paper is silent: a length outside [0, Lp] is clamped; if
 * the lengths sum to less than n_out the tail is one pad pseudo-example
 * (pad_id, label -100, ids 0, 1, 2, ...); if to more, the stream is cut at
 * n_out (the last example is broken, as fixed-length packing does, Table 1). */
int oracle_collate(const int64_t *ids, const int64_t *labels_in, const int32_t *lengths,
                   int n, int Lp, int64_t n_out, int64_t pad_id, int64_t *input_ids,
                   int64_t *labels, int64_t *position_ids, int32_t *offsets)
{
    if (!ids || !lengths || !input_ids || !labels || !position_ids || !offsets || n < 0 || Lp <= 0 ||
        n_out < 0)
        return 1;
    int64_t t = 0, total = 0;
    offsets[0] = 0;
    for (int e = 0; e < n; ++e) {
        int32_t L = lengths[e];
        if (L < 0) L = 0;
        if (L > Lp) L = Lp;
        for (int32_t p = 0; p < L; ++p, ++t) {
            if (t >= n_out) continue;
            const int64_t src = (int64_t)e * Lp + p;
            input_ids[t] = ids[src];
            labels[t] = p == 0 ? -100 : (labels_in ? labels_in[src] : ids[src]);
            position_ids[t] = p;
        }
        total += L;
        offsets[e + 1] = (int32_t)total;
    }
    for (int64_t p = 0; t < n_out; ++t, ++p) {
        input_ids[t] = pad_id;
        labels[t] = -100;
        position_ids[t] = p;
    }
    return 0;
}

/* ---- rotary position embedding ---------------------------------------- */

/* The other consumer of the restarting position ids (Section 3: models that take
 * position ids apply them to their positional encoding, so a packed example is
 * encoded exactly as if it were alone).  Textbook rotary embedding in the
 * "rotate-half" pairing: for a head vector x of even length d at position p,
 * pair c in [0, d/2) is (x[c], x[c + d/2]), rotated by the angle
 *     a = p * base^(-2c/d):   y[c]       = x[c] cos a - x[c + d/2] sin a
 *                             y[c + d/2] = x[c + d/2] cos a + x[c] sin a
 * inverse != 0 rotates by -a (the transpose: what the gradient needs).
 * X, Y: [N, H, d] doubles; pos: [N].  The paper names no pairing or base: this
 * is the one its listed decoder models use, base passed in. */
int oracle_rope(const double *X, double *Y, const int64_t *pos, int64_t N, int H, int d,
                double base, int inverse)
{
    if (!X || !Y || !pos || N < 0 || H <= 0 || d <= 0 || (d & 1) || base <= 0.0) return 1;
    const int hd = d / 2;
    for (int64_t t = 0; t < N; ++t)
        for (int c = 0; c < hd; ++c) {
            double a = (double)pos[t] * pow(base, -2.0 * (double)c / (double)d);
            if (inverse) a = -a;
            const double cs = cos(a), sn = sin(a);
            for (int h = 0; h < H; ++h) {
                const size_t o = ((size_t)t * H + h) * d;
                const double x1 = X[o + c], x2 = X[o + c + hd];
                Y[o + c] = x1 * cs - x2 * sn;
                Y[o + c + hd] = x2 * cs + x1 * sn;
            }
        }
    return 0;
}

/* ---- one query row ---------------------------------------------------- */

/* Softmax row of token i, head h, over keys a..i of KV head g.  Fills
 * P[0..i-a] and returns LSE_i.  S is scratch of the same length. */
static double softmax_row(const double *Q, const double *K, int64_t i, int64_t a,
                          int h, int g, int Hq, int Hkv, int d, double scale,
                          double *S, double *P)
{
    const double *q = Q + ((size_t)i * Hq + h) * d;
    double m = -INFINITY;
    for (int64_t j = a; j <= i; ++j) {
        const double *k = K + ((size_t)j * Hkv + g) * d;
        double s = 0.0;
        for (int c = 0; c < d; ++c) s += q[c] * k[c];
        s *= scale;
        S[j - a] = s;
        if (s > m) m = s;
    }
    double Z = 0.0;
    for (int64_t j = a; j <= i; ++j) Z += exp(S[j - a] - m);
    for (int64_t j = a; j <= i; ++j) P[j - a] = exp(S[j - a] - m) / Z;
    return m + log(Z);
}

/* dS row: dP_ij = dO_i . v_j, D_i = sum_j P_ij dP_ij, dS_ij = P_ij (dP_ij - D_i). */
static void ds_row(const double *dO, const double *V, const double *P, int64_t i, int64_t a,
                   int h, int g, int Hq, int Hkv, int d, double *dP, double *dS)
{
    const double *go = dO + ((size_t)i * Hq + h) * d;
    double D = 0.0;
    for (int64_t j = a; j <= i; ++j) {
        const double *v = V + ((size_t)j * Hkv + g) * d;
        double x = 0.0;
        for (int c = 0; c < d; ++c) x += go[c] * v[c];
        dP[j - a] = x;
        D += P[j - a] * x;
    }
    for (int64_t j = a; j <= i; ++j) dS[j - a] = P[j - a] * (dP[j - a] - D);
}

/* ---- full forward ----------------------------------------------------- */

int oracle_fwd(const double *Q, const double *K, const double *V, const int32_t *cu, int n,
               int N, int Hq, int Hkv, int d, double scale, double *O, double *LSE)
{
    if (!Q || !K || !V || !cu || !O || !LSE) return 1;
    if (Hkv <= 0 || Hq % Hkv != 0 || d <= 0 || n <= 0 || cu[0] != 0 || cu[n] != N) return 2;
    const int G = Hq / Hkv;
    int bad = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int s = 0; s < n; ++s) {
        for (int h = 0; h < Hq; ++h) {
            const int64_t a = cu[s], b = cu[s + 1];
            const int g = h / G;
            double *S = (double *)malloc(sizeof(double) * (size_t)(b - a));
            double *P = (double *)malloc(sizeof(double) * (size_t)(b - a));
            if (!S || !P) {
#pragma omp atomic write
                bad = 1;
                free(S); free(P); continue;
            }
            for (int64_t i = a; i < b; ++i) {
                LSE[(size_t)h * N + i] = softmax_row(Q, K, i, a, h, g, Hq, Hkv, d, scale, S, P);
                double *o = O + ((size_t)i * Hq + h) * d;
                for (int c = 0; c < d; ++c) o[c] = 0.0;
                for (int64_t j = a; j <= i; ++j) {
                    const double *v = V + ((size_t)j * Hkv + g) * d;
                    const double p = P[j - a];
                    for (int c = 0; c < d; ++c) o[c] += p * v[c];
                }
            }
            free(S); free(P);
        }
    }
    return bad ? 3 : 0;
}

/* ---- full backward ---------------------------------------------------- */

int oracle_bwd(const double *dO, const double *Q, const double *K, const double *V,
               const int32_t *cu, int n, int N, int Hq, int Hkv, int d, double scale,
               double *dQ, double *dK, double *dV)
{
    if (!dO || !Q || !K || !V || !cu || !dQ || !dK || !dV) return 1;
    if (Hkv <= 0 || Hq % Hkv != 0 || d <= 0 || n <= 0 || cu[0] != 0 || cu[n] != N) return 2;
    const int G = Hq / Hkv;
    memset(dK, 0, sizeof(double) * (size_t)N * Hkv * d);
    memset(dV, 0, sizeof(double) * (size_t)N * Hkv * d);
    int bad = 0;
    /* one task per (example, KV head): it alone writes that example's dK/dV rows of head g */
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int s = 0; s < n; ++s) {
        for (int g = 0; g < Hkv; ++g) {
            const int64_t a = cu[s], b = cu[s + 1];
            const size_t L = (size_t)(b - a);
            double *S = (double *)malloc(sizeof(double) * L);
            double *P = (double *)malloc(sizeof(double) * L);
            double *dP = (double *)malloc(sizeof(double) * L);
            double *dS = (double *)malloc(sizeof(double) * L);
            if (!S || !P || !dP || !dS) {
#pragma omp atomic write
                bad = 1;
                free(S); free(P); free(dP); free(dS); continue;
            }
            for (int h = g * G; h < (g + 1) * G; ++h) {
                for (int64_t i = a; i < b; ++i) {
                    softmax_row(Q, K, i, a, h, g, Hq, Hkv, d, scale, S, P);
                    ds_row(dO, V, P, i, a, h, g, Hq, Hkv, d, dP, dS);
                    const double *q = Q + ((size_t)i * Hq + h) * d;
                    const double *go = dO + ((size_t)i * Hq + h) * d;
                    double *dq = dQ + ((size_t)i * Hq + h) * d;
                    for (int c = 0; c < d; ++c) dq[c] = 0.0;
                    for (int64_t j = a; j <= i; ++j) {
                        const double *k = K + ((size_t)j * Hkv + g) * d;
                        double *dk = dK + ((size_t)j * Hkv + g) * d;
                        double *dv = dV + ((size_t)j * Hkv + g) * d;
                        const double ds = dS[j - a], p = P[j - a];
                        for (int c = 0; c < d; ++c) {
                            dq[c] += scale * ds * k[c];
                            dk[c] += scale * ds * q[c];
                            dv[c] += p * go[c];
                        }
                    }
                }
            }
            free(S); free(P); free(dP); free(dS);
        }
    }
    return bad ? 3 : 0;
}

/* ---- sampled outputs (full-size parity: one output row at a time) ------ */

static int find_segment(const int32_t *cu, int n, int64_t t)
{
    int lo = 0, hi = n;            /* cu[lo] <= t < cu[hi] */
    while (hi - lo > 1) {
        int mid = (lo + hi) / 2;
        if (cu[mid] <= t) lo = mid; else hi = mid;
    }
    return lo;
}

/* O[i,h,:], LSE[h,i] and dQ[i,h,:] for m sampled (token, head) pairs.
 * out_O, out_dQ: [m, d]; out_LSE: [m].  dO may be NULL (then dQ is skipped). */
int oracle_rows_q(const double *dO, const double *Q, const double *K, const double *V,
                  const int32_t *cu, int n, int N, int Hq, int Hkv, int d, double scale,
                  const int32_t *tok, const int32_t *head, int m,
                  double *out_O, double *out_LSE, double *out_dQ)
{
    if (!Q || !K || !V || !cu || !tok || !head || !out_O || !out_LSE) return 1;
    if (Hkv <= 0 || Hq % Hkv != 0) return 2;
    const int G = Hq / Hkv;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < m; ++r) {
        const int64_t i = tok[r];
        const int h = head[r], g = h / G;
        if (i < 0 || i >= N || h < 0 || h >= Hq) {
#pragma omp atomic write
            bad = 2;
            continue;
        }
        const int64_t a = cu[find_segment(cu, n, i)];
        const size_t L = (size_t)(i - a + 1);
        double *S = (double *)malloc(sizeof(double) * L);
        double *P = (double *)malloc(sizeof(double) * L);
        double *dP = (double *)malloc(sizeof(double) * L);
        double *dS = (double *)malloc(sizeof(double) * L);
        if (!S || !P || !dP || !dS) {
#pragma omp atomic write
            bad = 3;
            free(S); free(P); free(dP); free(dS); continue;
        }
        out_LSE[r] = softmax_row(Q, K, i, a, h, g, Hq, Hkv, d, scale, S, P);
        double *o = out_O + (size_t)r * d;
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        for (int64_t j = a; j <= i; ++j) {
            const double *v = V + ((size_t)j * Hkv + g) * d;
            for (int c = 0; c < d; ++c) o[c] += P[j - a] * v[c];
        }
        if (dO && out_dQ) {
            ds_row(dO, V, P, i, a, h, g, Hq, Hkv, d, dP, dS);
            double *dq = out_dQ + (size_t)r * d;
            for (int c = 0; c < d; ++c) dq[c] = 0.0;
            for (int64_t j = a; j <= i; ++j) {
                const double *k = K + ((size_t)j * Hkv + g) * d;
                for (int c = 0; c < d; ++c) dq[c] += scale * dS[j - a] * k[c];
            }
        }
        free(S); free(P); free(dP); free(dS);
    }
    return bad;
}

/* dK[j,g,:] and dV[j,g,:] for m sampled (token, KV head) pairs: the sum over
 * every later row i of the same example and every query head of the group. */
int oracle_rows_kv(const double *dO, const double *Q, const double *K, const double *V,
                   const int32_t *cu, int n, int N, int Hq, int Hkv, int d, double scale,
                   const int32_t *tok, const int32_t *kvhead, int m,
                   double *out_dK, double *out_dV)
{
    if (!dO || !Q || !K || !V || !cu || !tok || !kvhead || !out_dK || !out_dV) return 1;
    if (Hkv <= 0 || Hq % Hkv != 0) return 2;
    const int G = Hq / Hkv;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < m; ++r) {
        const int64_t j = tok[r];
        const int g = kvhead[r];
        if (j < 0 || j >= N || g < 0 || g >= Hkv) {
#pragma omp atomic write
            bad = 2;
            continue;
        }
        const int s = find_segment(cu, n, j);
        const int64_t a = cu[s], b = cu[s + 1];
        const size_t L = (size_t)(b - a);
        double *S = (double *)malloc(sizeof(double) * L);
        double *P = (double *)malloc(sizeof(double) * L);
        double *dP = (double *)malloc(sizeof(double) * L);
        double *dS = (double *)malloc(sizeof(double) * L);
        if (!S || !P || !dP || !dS) {
#pragma omp atomic write
            bad = 3;
            free(S); free(P); free(dP); free(dS); continue;
        }
        double *dk = out_dK + (size_t)r * d, *dv = out_dV + (size_t)r * d;
        for (int c = 0; c < d; ++c) { dk[c] = 0.0; dv[c] = 0.0; }
        for (int h = g * G; h < (g + 1) * G; ++h) {
            for (int64_t i = j; i < b; ++i) {
                softmax_row(Q, K, i, a, h, g, Hq, Hkv, d, scale, S, P);
                ds_row(dO, V, P, i, a, h, g, Hq, Hkv, d, dP, dS);
                const double *q = Q + ((size_t)i * Hq + h) * d;
                const double *go = dO + ((size_t)i * Hq + h) * d;
                for (int c = 0; c < d; ++c) {
                    dk[c] += scale * dS[j - a] * q[c];
                    dv[c] += P[j - a] * go[c];
                }
            }
        }
        free(S); free(P); free(dP); free(dS);
    }
    return bad;
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    n = omp_get_max_threads();
#endif
    return n;
}

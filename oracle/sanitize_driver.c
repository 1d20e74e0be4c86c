/*
 * Driver for a sanitizer build of the CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * Compiled together with varlen_oracle.c under -fsanitize=address,undefined (tests/test_oracle_sanitized.py)
 * and run as a program: every oracle entry point on small inputs that reach its edge cases (a packed
 * row that does not start at id 0, consecutive zeros, length-1 examples, grouped heads, a collator
 * row with a pad tail and one that is cut, sampled rows at example ends).  Prints one checksum line;
 * any out-of-bounds access, use of uninitialised stack, signed overflow or misaligned access aborts
 * the run with a sanitizer report.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_pack(const int64_t *, int, int, int32_t *, int32_t *, int32_t *, int32_t *);
int oracle_collate(const int64_t *, const int64_t *, const int32_t *, int, int, int64_t, int64_t, int64_t *,
                   int64_t *, int64_t *, int32_t *);
int oracle_rope(const double *, double *, const int64_t *, int64_t, int, int, double, int);
int oracle_fwd(const double *, const double *, const double *, const int32_t *, int, int, int, int, int, double,
               double *, double *);
int oracle_bwd(const double *, const double *, const double *, const double *, const int32_t *, int, int, int, int,
               int, double, double *, double *, double *);
int oracle_rows_q(const double *, const double *, const double *, const double *, const int32_t *, int, int, int,
                  int, int, double, const int32_t *, const int32_t *, int, double *, double *, double *);
int oracle_rows_kv(const double *, const double *, const double *, const double *, const int32_t *, int, int, int,
                   int, int, double, const int32_t *, const int32_t *, int, double *, double *);

static uint64_t state = 88172645463325252ull;
static double rnd(void)
{ /* xorshift64, mapped to [-1, 1) */
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (double)(state >> 11) / 9007199254740992.0 * 2.0 - 1.0;
}
static double *randv(size_t n)
{
    double *p = (double *)malloc(sizeof(double) * (n ? n : 1));
    if (!p) exit(3);
    for (size_t i = 0; i < n; ++i) p[i] = rnd();
    return p;
}
static double sum(const double *p, size_t n)
{
    double s = 0.0;
    for (size_t i = 0; i < n; ++i) s += p[i] * (double)(1 + i % 7);
    return s;
}

int main(void)
{
    double check = 0.0;
    /* boundaries: 2 rows of 12; row 1 starts with a non-zero id; consecutive zeros */
    enum { R = 2, T = 12, N = R * T, Hq = 4, Hkv = 2, D = 6 };
    const int64_t pos[N] = {0, 1, 2, 0, 0, 1, 2, 3, 4, 0, 1, 2,   5, 6, 0, 1, 0, 0, 0, 1, 2, 3, 4, 5};
    int32_t cu[N + 1], seg_id[N], n = 0, mx = 0;
    if (oracle_pack(pos, R, T, cu, seg_id, &n, &mx)) return 1;
    check += n * 1000 + mx;
    for (int i = 0; i <= n; ++i) check += cu[i] * (i + 1);

    double *Q = randv((size_t)N * Hq * D), *K = randv((size_t)N * Hkv * D), *V = randv((size_t)N * Hkv * D);
    double *dO = randv((size_t)N * Hq * D);
    double *O = randv((size_t)N * Hq * D), *LSE = randv((size_t)Hq * N);
    double *dQ = randv((size_t)N * Hq * D), *dK = randv((size_t)N * Hkv * D), *dV = randv((size_t)N * Hkv * D);
    if (oracle_fwd(Q, K, V, cu, n, N, Hq, Hkv, D, 0.4, O, LSE)) return 1;
    if (oracle_bwd(dO, Q, K, V, cu, n, N, Hq, Hkv, D, 0.4, dQ, dK, dV)) return 1;
    check += sum(O, (size_t)N * Hq * D) + sum(LSE, (size_t)Hq * N) + sum(dQ, (size_t)N * Hq * D) +
             sum(dK, (size_t)N * Hkv * D) + sum(dV, (size_t)N * Hkv * D);

    /* sampled rows: first and last token of the stream, example ends, every head */
    const int32_t tok[6] = {0, 2, 3, 11, 12, N - 1}, head[6] = {0, 1, 2, 3, 0, 3}, kvh[6] = {0, 1, 0, 1, 0, 1};
    double rO[6 * D], rL[6], rdQ[6 * D], rdK[6 * D], rdV[6 * D];
    if (oracle_rows_q(dO, Q, K, V, cu, n, N, Hq, Hkv, D, 0.4, tok, head, 6, rO, rL, rdQ)) return 1;
    if (oracle_rows_q(NULL, Q, K, V, cu, n, N, Hq, Hkv, D, 0.4, tok, head, 6, rO, rL, NULL)) return 1;
    if (oracle_rows_kv(dO, Q, K, V, cu, n, N, Hq, Hkv, D, 0.4, tok, kvh, 6, rdK, rdV)) return 1;
    check += sum(rO, 6 * D) + sum(rL, 6) + sum(rdQ, 6 * D) + sum(rdK, 6 * D) + sum(rdV, 6 * D);
    /* the sampled rows equal the full results */
    for (int r = 0; r < 6; ++r)
        for (int c = 0; c < D; ++c) {
            double a = rdQ[r * D + c] - dQ[((size_t)tok[r] * Hq + head[r]) * D + c];
            double b = rdK[r * D + c] - dK[((size_t)tok[r] * Hkv + kvh[r]) * D + c];
            if (a > 1e-12 || a < -1e-12 || b > 1e-12 || b < -1e-12) return 2;
        }

    /* rotary embedding: odd head count, smallest head_dim, inverse */
    double *X = randv((size_t)N * 3 * 2), *Y = randv((size_t)N * 3 * 2);
    if (oracle_rope(X, Y, pos, N, 3, 2, 10000.0, 0)) return 1;
    if (oracle_rope(Y, X, pos, N, 3, 2, 10000.0, 1)) return 1;
    check += sum(Y, (size_t)N * 3 * 2);

    /* collator: lengths outside [0, Lp] are clamped; a pad tail; then a cut row */
    enum { NE = 4, LP = 5 };
    int64_t ids[NE * LP], labs[NE * LP];
    for (int i = 0; i < NE * LP; ++i) { ids[i] = 100 + i; labs[i] = 200 + i; }
    const int32_t lengths[NE] = {3, 9, -2, 5};
    int64_t out_ids[20], out_lab[20], out_pos[20];
    int32_t offs[NE + 1];
    if (oracle_collate(ids, labs, lengths, NE, LP, 20, 7, out_ids, out_lab, out_pos, offs)) return 1; /* 13 real + 7 pad */
    for (int i = 0; i < 20; ++i) check += (double)(out_ids[i] + 3 * out_lab[i] + 5 * out_pos[i]);
    if (oracle_collate(ids, NULL, lengths, NE, LP, 6, 7, out_ids, out_lab, out_pos, offs)) return 1;  /* cut at 6 */
    for (int i = 0; i < 6; ++i) check += (double)(out_ids[i] + 3 * out_lab[i] + 5 * out_pos[i]);
    if (oracle_collate(ids, NULL, lengths, 0, LP, 0, 7, out_ids, out_lab, out_pos, offs)) return 1;  /* empty */
    check += offs[0];

    printf("oracle sanitize driver ok: checksum %.12e\n", check);
    free(Q); free(K); free(V); free(dO); free(O); free(LSE); free(dQ); free(dK); free(dV); free(X); free(Y);
    return 0;
}

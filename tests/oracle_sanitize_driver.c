/* Calls every entry point of oracle/d3tom_oracle.c once on small ragged inputs.  Built with
 * -fsanitize=address,undefined by tests/test_oracle_pins.py: a memory error or undefined behaviour in
 * the oracle aborts this program.  Test infrastructure, host only. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_keep_count(int, double);
int oracle_deciders(const int32_t*, const int32_t*, int, int, int32_t*, int);
int oracle_importance(const float*, const float*, int, int, int, double, const int32_t*, int, int, int, double*, double*);
int oracle_select_topk(const double*, int, int, int32_t*, int32_t*);
int oracle_assign(const float*, int, int, int, const int32_t*, int, int32_t*, double*, const int32_t*);
double oracle_cosine(const float*, int, int, int);
int oracle_merge(const float*, int, int, int, int, const int32_t*, int, const int32_t*, int, double*, int32_t*, int32_t*);
int oracle_attend(const float*, const float*, const float*, int, int, int, double, const double*, double*, const int32_t*, int);

static float rnd(unsigned* s) {
    *s = *s * 1664525u + 1013904223u;
    return (float)((*s >> 8) & 0xFFFF) / 32768.0f - 1.0f;
}

int main(void) {
    enum { N = 37, H = 3, DH = 5, P = 4, V = 29, D = 3, K = 7, DM = H * DH };
    unsigned s = 1;
    float *q = malloc(sizeof(float) * N * DM), *k = malloc(sizeof(float) * N * DM), *x = malloc(sizeof(float) * N * DM);
    for (int i = 0; i < N * DM; ++i) { q[i] = rnd(&s); k[i] = rnd(&s); x[i] = rnd(&s); }
    int32_t dec[D] = {33, 35, 36};
    double *S = malloc(sizeof(double) * V), *Sall = malloc(sizeof(double) * N);
    if (oracle_importance(q, k, N, H, DH, 0.4, dec, D, P, V, S, Sall)) return 2;
    int32_t *kept = malloc(sizeof(int32_t) * K), *slot = malloc(sizeof(int32_t) * V);
    if (oracle_keep_count(V, 0.24) != K || oracle_select_topk(S, V, K, kept, slot)) return 3;
    int32_t* asg = malloc(sizeof(int32_t) * V);
    double* bc = malloc(sizeof(double) * V);
    int32_t* only = calloc(V, sizeof(int32_t));
    only[1] = only[20] = 1;
    if (oracle_assign(x, DM, P, V, kept, K, asg, bc, only)) return 4;
    if (oracle_assign(x, DM, P, V, kept, K, asg, bc, NULL)) return 4;
    const double c = oracle_cosine(x, DM, 0, N - 1);
    const int NM = N - (V - K);
    double* y = malloc(sizeof(double) * NM * DM);
    int32_t *cnt = malloc(sizeof(int32_t) * K), *src = malloc(sizeof(int32_t) * NM);
    for (int mode = 0; mode < 2; ++mode)
        if (oracle_merge(x, N, DM, P, V, kept, K, asg, mode, y, cnt, src)) return 5;
    double *o = malloc(sizeof(double) * N * DM), *w = malloc(sizeof(double) * N);
    for (int j = 0; j < N; ++j) w[j] = 1.0 + j % 3;
    int32_t rows[3] = {0, 17, N - 1};
    if (oracle_attend(q, k, x, N, H, DH, 0.4, NULL, o, NULL, 0)) return 6;
    if (oracle_attend(q, k, x, N, H, DH, 0.4, w, o, rows, 3)) return 6;
    int32_t prev[9] = {1, 9, 9, 9, 2, 9, 9, 3, 9}, cur[9] = {1, 5, 9, 6, 2, 9, 7, 3, 8}, out[2];
    if (oracle_deciders(prev, cur, 9, 9, out, 2) != 4) return 7;
    printf("ok %g %g %d\n", c, o[0], cnt[0]);
    free(q); free(k); free(x); free(S); free(Sall); free(kept); free(slot); free(asg); free(bc); free(only);
    free(y); free(cnt); free(src); free(o); free(w);
    return 0;
}

/*
 * CPU oracle for the D3ToM merge layer and the bidirectional attention after it.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * hot path computes; it exists so that the HIP library can be checked against
 * it.  It shares no code, header, table or helper with the HIP path and must
 * never be called from it.  Only the tests, the smoke check and the benchmark's
 * CPU-baseline leg load it.
 *
 * Every function takes float32 inputs (values already rounded to the storage
 * type of the workload: float32, or bfloat16 widened exactly), widens them to
 * double and does ALL arithmetic in double.  No blocking, no fusion, no
 * re-association beyond what the definition states.  The only concession to
 * wall-clock time is an OpenMP "parallel for" over independent outer
 * iterations (heads, rows); each iteration is the sequential definition.
 *
 * Pinned by tests/test_oracle_pins.py: closed forms, invariants, textbook special
 * cases, library routines and brute force.  The paper prints no worked numeric
 * example of the merge, so no printed values exist to compare with.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
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

/* Kept-token count.  Section 3.2 keeps the tokens whose rank is at most
 * (1 - alpha)|V|; with keep_ratio = 1 - alpha and a non-integer product the
 * count is rounded UP (reading K1: ceil), never below 1 nor above V.  The
 * 1e-9 guard absorbs products such as 0.25 * 144 = 36.000000000000004. */
int oracle_keep_count(int V, double keep_ratio) {
    double c = ceil(keep_ratio * (double)V - 1e-9);
    if (c < 1.0) c = 1.0;
    if (c > (double)V) c = (double)V;
    return (int)c;
}

/* Decider set (Section 3.2, "The Decider-Guided Mechanism"): the positions that
 * hold a token in the current iterate and held [MASK] in the preceding one,
 * listed in ascending position.  Returns their number; at most `cap` are
 * written to out. */
int oracle_deciders(const int32_t* prev_ids, const int32_t* cur_ids, int n, int mask_id, int32_t* out, int cap) {
    int c = 0;
    for (int i = 0; i < n; ++i) {
        if (cur_ids[i] != mask_id && prev_ids[i] == mask_id) {
            if (c < cap) out[c] = i;
            ++c;
        }
    }
    return c;
}

/* Linear schedule of Section 3.2 ("Timestep-Dependent Merge Schedule"),
 * written direction-neutrally: value at decoding-order step s of T, moving
 * linearly from r_first (s = 0) to r_last (s = T-1). */
double oracle_schedule(int s, int T, double r_first, double r_last) {
    if (T <= 1) return r_first;
    return r_first + (r_last - r_first) * (double)s / (double)(T - 1);
}

/*
 * Importance map (Section 3.2, "The Decider-Guided Mechanism": the attention
 * matrix A and the decider score S_j = sum_{i in D} A_ij; Algorithm 1, the
 * line that forms S).
 *
 * Multi-head reading: A is formed per head with the row softmax taken over ALL
 * N keys, scores are summed over the decider rows and averaged over heads.
 *
 *   q, k     [N, H, dh]   queries / keys of one sample
 *   dec_idx  [D]          positions of the decider tokens (rows of A that count)
 *   S        [V]  out     score of visual token j = vis_start + jj
 *   S_all    [N]  out, optional: the same sum for every key position
 */
int oracle_importance(const float* q, const float* k, int N, int H, int dh, double scale,
                      const int32_t* dec_idx, int D, int vis_start, int V,
                      double* S, double* S_all) {
    if (N <= 0 || H <= 0 || dh <= 0 || D <= 0 || V < 0 || vis_start < 0 || vis_start + V > N) return 1;
    for (int i = 0; i < D; ++i) if (dec_idx[i] < 0 || dec_idx[i] >= N) return 1;
    double* acc = (double*)calloc((size_t)H * N, sizeof(double));   /* per head: sum_i A^h_ij */
    if (!acc) return 2;
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < H; ++h) {
        double* logit = (double*)malloc((size_t)N * sizeof(double));
        for (int i = 0; i < D; ++i) {
            const float* qi = q + ((size_t)dec_idx[i] * H + h) * dh;
            double mx = -INFINITY;
            for (int j = 0; j < N; ++j) {
                const float* kj = k + ((size_t)j * H + h) * dh;
                double s = 0.0;
                for (int c = 0; c < dh; ++c) s += (double)qi[c] * (double)kj[c];
                logit[j] = s * scale;
                if (logit[j] > mx) mx = logit[j];
            }
            double z = 0.0;
            for (int j = 0; j < N; ++j) { logit[j] = exp(logit[j] - mx); z += logit[j]; }
            for (int j = 0; j < N; ++j) acc[(size_t)h * N + j] += logit[j] / z;
        }
        free(logit);
    }
    for (int j = 0; j < N; ++j) {
        double s = 0.0;
        for (int h = 0; h < H; ++h) s += acc[(size_t)h * N + j];
        s /= (double)H;
        if (S_all) S_all[j] = s;
        if (j >= vis_start && j < vis_start + V) S[j - vis_start] = s;
    }
    free(acc);
    return 0;
}

/*
 * Keep / merge partition (Section 3.2: V_kept = tokens whose score rank is at
 * most the kept count; Algorithm 1, the TopK line).
 *
 * Rank order is (score descending, index ascending): among equal scores the
 * lower index ranks first (reading T1).  Output: the kept indices in ascending
 * position order, and slot_of[j] = position of j within that list, or -1.
 */
typedef struct { double s; int32_t j; } ranked_t;
static int ranked_cmp(const void* a, const void* b) {
    const ranked_t* x = (const ranked_t*)a; const ranked_t* y = (const ranked_t*)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->j > y->j) - (x->j < y->j);
}
int oracle_select_topk(const double* S, int V, int keep_k, int32_t* kept_idx, int32_t* slot_of) {
    if (V <= 0 || keep_k < 1 || keep_k > V) return 1;
    ranked_t* r = (ranked_t*)malloc((size_t)V * sizeof(ranked_t));
    if (!r) return 2;
    for (int j = 0; j < V; ++j) { r[j].s = S[j]; r[j].j = j; }
    qsort(r, (size_t)V, sizeof(ranked_t), ranked_cmp);
    for (int j = 0; j < V; ++j) slot_of[j] = -1;
    for (int t = 0; t < keep_k; ++t) slot_of[r[t].j] = 0;          /* mark */
    int slot = 0;
    for (int j = 0; j < V; ++j) if (slot_of[j] == 0) { kept_idx[slot] = j; slot_of[j] = slot++; }
    free(r);
    return 0;
}

/*
 * Cosine nearest-kept assignment (Section 3.2, "Similarity-Based Merging": k* =
 * argmax over kept tokens of the cosine similarity; Algorithm 1, the argmax
 * line).  All similarities use the ORIGINAL rows (reading M2: assign first,
 * accumulate afterwards).  Ties go to the lowest slot (reading T2).  A zero row
 * has similarity 0 with everything (norm product clamped at 1e-30, reading Z1).
 *
 *   f        [n_rows, d]  feature rows; the visual block starts at row vis_start
 *   kept_idx [keep_k]     ascending indices inside the visual block
 *   assign   [V]  out     slot every visual token ends up in (kept token: its own slot)
 *   best_cos [V]  out, optional: similarity to the chosen slot (1 for kept tokens)
 *   only     [V]  optional mask: when given, pruned tokens with only[m] == 0 are skipped and get
 *                 assign[m] = -1 (lets a test look at a sample of rows of a large case)
 */
int oracle_assign(const float* f, int d, int vis_start, int V,
                  const int32_t* kept_idx, int keep_k, int32_t* assign, double* best_cos,
                  const int32_t* only) {
    if (d <= 0 || V <= 0 || keep_k < 1 || keep_k > V) return 1;
    double* nrm = (double*)malloc((size_t)V * sizeof(double));
    int32_t* slot_of = (int32_t*)malloc((size_t)V * sizeof(int32_t));
    if (!nrm || !slot_of) return 2;
    for (int j = 0; j < V; ++j) {
        const float* r = f + (size_t)(vis_start + j) * d;
        double s = 0.0;
        for (int c = 0; c < d; ++c) s += (double)r[c] * (double)r[c];
        nrm[j] = sqrt(s);
        slot_of[j] = -1;
    }
    for (int r = 0; r < keep_k; ++r) {
        if (kept_idx[r] < 0 || kept_idx[r] >= V) { free(nrm); free(slot_of); return 1; }
        slot_of[kept_idx[r]] = r;
    }
#pragma omp parallel for schedule(dynamic, 8)
    for (int m = 0; m < V; ++m) {
        if (slot_of[m] >= 0) { assign[m] = slot_of[m]; if (best_cos) best_cos[m] = 1.0; continue; }
        if (only && !only[m]) { assign[m] = -1; if (best_cos) best_cos[m] = 0.0; continue; }
        const float* xm = f + (size_t)(vis_start + m) * d;
        int best = -1; double bc = 0.0;
        for (int r = 0; r < keep_k; ++r) {
            const float* xk = f + (size_t)(vis_start + kept_idx[r]) * d;
            double dot = 0.0;
            for (int c = 0; c < d; ++c) dot += (double)xm[c] * (double)xk[c];
            double den = nrm[m] * nrm[kept_idx[r]];
            if (den < 1e-30) den = 1e-30;
            double cs = dot / den;
            if (best < 0 || cs > bc) { best = r; bc = cs; }
        }
        assign[m] = best;
        if (best_cos) best_cos[m] = bc;
    }
    free(nrm); free(slot_of);
    return 0;
}

/* Cosine similarity of one visual token to one slot, for judging near-ties. */
double oracle_cosine(const float* f, int d, int row_a, int row_b) {
    const float* a = f + (size_t)row_a * d; const float* b = f + (size_t)row_b * d;
    double dot = 0.0, na = 0.0, nb = 0.0;
    for (int c = 0; c < d; ++c) { dot += (double)a[c] * b[c]; na += (double)a[c] * a[c]; nb += (double)b[c] * b[c]; }
    double den = sqrt(na) * sqrt(nb);
    if (den < 1e-30) den = 1e-30;
    return dot / den;
}

/*
 * Aggregation and removal (Section 3.2: h_k* <- h_k* + h_m, then the merged
 * positions are removed; Algorithm 1, the accumulate and "Remove positions"
 * lines).  mode 0 = MEAN (sum divided by the member count, reading M1),
 * mode 1 = SUM (the paper's literal update).
 *
 *   x        [N, d]        payload rows
 *   y        [N_m, d] out  rows before the visual block | keep_k merged rows in
 *                          ascending original position | rows after the block
 *   counts   [keep_k] out  members per slot (the kept token itself included)
 *   src_pos  [N_m]   out   original position of every output row
 */
int oracle_merge(const float* x, int N, int d, int vis_start, int V,
                 const int32_t* kept_idx, int keep_k, const int32_t* assign, int mode,
                 double* y, int32_t* counts, int32_t* src_pos) {
    if (N <= 0 || d <= 0 || V <= 0 || keep_k < 1 || keep_k > V || vis_start < 0 || vis_start + V > N) return 1;
    const int N_m = N - (V - keep_k);
    memset(y, 0, (size_t)N_m * d * sizeof(double));
    for (int r = 0; r < keep_k; ++r) counts[r] = 0;
    for (int p = 0; p < vis_start; ++p) {
        for (int c = 0; c < d; ++c) y[(size_t)p * d + c] = (double)x[(size_t)p * d + c];
        src_pos[p] = p;
    }
    for (int m = 0; m < V; ++m) {            /* ascending member order */
        int r = assign[m];
        if (r < 0 || r >= keep_k) return 1;
        double* yr = y + (size_t)(vis_start + r) * d;
        const float* xm = x + (size_t)(vis_start + m) * d;
        for (int c = 0; c < d; ++c) yr[c] += (double)xm[c];
        counts[r] += 1;
    }
    for (int r = 0; r < keep_k; ++r) {
        src_pos[vis_start + r] = vis_start + kept_idx[r];
        if (mode == 0) {
            double* yr = y + (size_t)(vis_start + r) * d;
            for (int c = 0; c < d; ++c) yr[c] /= (double)counts[r];
        }
    }
    for (int p = vis_start + V; p < N; ++p) {
        int o = p - (V - keep_k);
        for (int c = 0; c < d; ++c) y[(size_t)o * d + c] = (double)x[(size_t)p * d + c];
        src_pos[o] = p;
    }
    return 0;
}

/*
 * Bidirectional attention over the shortened sequence (Section 3.2: the
 * shortened tensor propagates through the later layers; Section 4.3: the
 * 2 n^2 d term of the per-layer cost; no causal mask, every query sees every
 * key).  Per head: O = softmax(scale * Q K^T) V.
 *
 * Size-weighted form (reading M1).  Under MEAN aggregation a merged row stands
 * for count_r original tokens but enters the softmax of the later layers once,
 * so the attention mass those tokens had is lost; SUM aggregation (the paper's
 * literal update) keeps it in the row's magnitude instead.  With per-key weights
 * w_j (the member counts the merge reports) the attention probabilities become
 * p_ij = w_j exp(l_ij) / sum_j' w_j' exp(l_ij'), i.e. softmax(l_ij + log w_j):
 * exactly what attention over the sequence with key/value row j written w_j
 * times would give.  key_weight == NULL is the plain form (all w_j = 1).
 *
 *   q, k, v     [n, H, dh]   out [n, H, dh]
 *   key_weight  [n] optional, every entry > 0
 *   rows        [n_rows] optional: query rows to evaluate (NULL = all n); other rows of out are left alone
 */
int oracle_attend(const float* q, const float* k, const float* v, int n, int H, int dh, double scale,
                  const double* key_weight, double* out, const int32_t* rows, int n_rows) {
    if (n <= 0 || H <= 0 || dh <= 0) return 1;
    if (!rows) n_rows = n;
    for (int t = 0; rows && t < n_rows; ++t) if (rows[t] < 0 || rows[t] >= n) return 1;
    for (int j = 0; key_weight && j < n; ++j) if (!(key_weight[j] > 0.0)) return 1;
#pragma omp parallel for collapse(2) schedule(dynamic, 16)
    for (int h = 0; h < H; ++h) {
        for (int t = 0; t < n_rows; ++t) {
            const int i = rows ? rows[t] : t;
            double* p = (double*)malloc((size_t)n * sizeof(double));
            const float* qi = q + ((size_t)i * H + h) * dh;
            double mx = -INFINITY;
            for (int j = 0; j < n; ++j) {
                const float* kj = k + ((size_t)j * H + h) * dh;
                double s = 0.0;
                for (int c = 0; c < dh; ++c) s += (double)qi[c] * (double)kj[c];
                p[j] = s * scale;
                if (p[j] > mx) mx = p[j];
            }
            double z = 0.0;
            for (int j = 0; j < n; ++j) {
                p[j] = exp(p[j] - mx);
                if (key_weight) p[j] *= key_weight[j];
                z += p[j];
            }
            double* o = out + ((size_t)i * H + h) * dh;
            for (int c = 0; c < dh; ++c) o[c] = 0.0;
            for (int j = 0; j < n; ++j) {
                const float* vj = v + ((size_t)j * H + h) * dh;
                double w = p[j] / z;
                for (int c = 0; c < dh; ++c) o[c] += w * (double)vj[c];
            }
            free(p);
        }
    }
    return 0;
}

/*
 * Theoretical cost model (Section 4.3 "Efficiency Analysis"; Appendix B).
 * FLOPs_layer(n) = 4 n d^2 + 2 n^2 d + 3 n d m.
 */
double oracle_flops_layer(double n, double d, double m) {
    return 4.0 * n * d * d + 2.0 * n * n * d + 3.0 * n * d * m;
}
double oracle_flops_attn(double n, double d) { return 4.0 * n * d * d + 2.0 * n * n * d; }
double oracle_flops_ffn(double n, double d, double m) { return 3.0 * n * d * m; }
/* merge overhead: 2 a (1-a) |V|^2 d + a |V| d */
double oracle_flops_merge(double alpha, double V, double d) {
    return 2.0 * alpha * (1.0 - alpha) * V * V * d + alpha * V * d;
}
/* one step with the merge inside layer l_star (layers before it at N, its attention
 * at N and its FFN at N_m, the remaining L - l_star - 1 layers at N_m, plus the merge) */
double oracle_flops_step(double alpha, int l_star, int L, double V, double P, double O, double d, double m) {
    double N = V + P + O, Nm = N - alpha * V;
    return (double)l_star * oracle_flops_layer(N, d, m)
         + oracle_flops_attn(N, d) + oracle_flops_ffn(Nm, d, m)
         + (double)(L - l_star - 1) * oracle_flops_layer(Nm, d, m)
         + oracle_flops_merge(alpha, V, d);
}
/* whole trajectory: the first of the T steps has an empty decider set (Algorithm 1
 * initialises it empty and skips the merge then), so it runs unmerged. */
double oracle_flops_total(double alpha, int l_star, int L, int T, double V, double P, double O, double d, double m) {
    double N = V + P + O;
    return (double)L * oracle_flops_layer(N, d, m)
         + (double)(T - 1) * oracle_flops_step(alpha, l_star, L, V, P, O, d, m);
}

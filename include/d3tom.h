/*
 * d3tom.h — C ABI of the MI355X (gfx950) library for the D3ToM merge layer and the
 * bidirectional attention over the shortened sequence that follows it.
 *
 * One denoising step of the method, at the merge layer (Algorithm 1, the block guarded by
 * "l = l* and the decider set is not empty"):
 *
 *     d3tom_importance   S_j = sum over decider rows of the attention they pay to visual token j
 *     d3tom_select_topk  keep the ceil(keep_ratio |V|) highest-scoring visual tokens
 *     d3tom_merge        send every other visual token to its most cosine-similar kept token,
 *                        aggregate, and physically remove the merged positions
 *                        (d3tom_merge_kv: the same on a key/value cache, Section 4.4)
 *     d3tom_attend       full (unmasked) attention over the shortened sequence
 * and, between steps, d3tom_update_deciders builds the decider set of the next step on the device.
 *
 * Conventions shared by the device entry points
 * --------------------------------------------------
 * Pointers   Every pointer is a DEVICE pointer owned by the caller, unless the parameter is
 *            documented "host".  The library never allocates, frees or keeps a pointer.
 * Batching   B samples are concatenated along the token axis.  Per-sample metadata are device
 *            int32 arrays; everything the host needs to size a launch is passed by value
 *            (B, H, dh, max_*).  Values in device metadata that exceed the stated maxima are
 *            clamped by the kernels (no out-of-bounds access); results for such samples are
 *            unspecified.
 * Layout     Token-major rows.  q/k/v: [tokens, H, dh], heads contiguous inside a row.
 *            Hidden states: [tokens, d].  Rows must be 16-byte aligned (dh and d multiples of
 *            8 for bf16, of 4 for f32; base pointers 16-byte aligned).
 * Types      D3TOM_F32: IEEE float.  D3TOM_BF16: bfloat16 storage, float32 accumulation.
 * Stream     All work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *            default stream).  No entry point synchronises or reads device memory on the host.
 * Workspace  `ws` is device scratch of at least d3tom_workspace_bytes(op, ...) bytes, 256-byte
 *            aligned.  It carries no state between calls; concurrent calls need separate ones.
 * Errors     The return value is a d3tom_status.  Arguments are validated on the host before
 *            anything is enqueued: INVALID_ARG, NO_DECIDERS, WORKSPACE_TOO_SMALL and UNSUPPORTED mean
 *            that nothing was enqueued.  D3TOM_ERR_DEVICE (the HIP runtime refused a launch or a
 *            set-up call) can come from the middle of an entry point that enqueues several kernels:
 *            earlier kernels of that call may then already be on the stream and the outputs are
 *            unspecified.
 * Determinism  No floating-point atomics: the same inputs give bit-identical outputs.
 * NaN/Inf inputs are outside the contract.
 */
#ifndef D3TOM_H
#define D3TOM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    D3TOM_OK = 0,
    D3TOM_ERR_INVALID_ARG = 1,        /* null pointer, non-positive size, misaligned pointer        */
    D3TOM_ERR_NO_DECIDERS = 2,        /* a sample has an empty decider set: skip the merge          */
    D3TOM_ERR_WORKSPACE_TOO_SMALL = 3,
    D3TOM_ERR_UNSUPPORTED = 4,        /* shape or type outside what the kernels are built for       */
    D3TOM_ERR_DEVICE = 5              /* the HIP runtime rejected a launch                          */
} d3tom_status;

typedef enum { D3TOM_F32 = 0, D3TOM_BF16 = 1 } d3tom_dtype;
typedef enum { D3TOM_MERGE_MEAN = 0, D3TOM_MERGE_SUM = 1 } d3tom_merge_mode;
typedef enum { D3TOM_OP_IMPORTANCE = 0, D3TOM_OP_SELECT_TOPK = 1, D3TOM_OP_MERGE = 2, D3TOM_OP_ATTEND = 3 } d3tom_op;

/* Largest visual-token count per sample that select_topk / merge keep resident in LDS. */
#define D3TOM_MAX_VISUAL 16384
/* Largest decider count per sample. */
#define D3TOM_MAX_DECIDERS 256

/* ------------------------------------------------------------------------------------------
 * Host-only helpers (no device work).
 * ---------------------------------------------------------------------------------------- */

/* Number of visual tokens kept at a keep ratio (= 1 - merge ratio alpha_t).  Section 3.2 keeps
 * the tokens whose score rank is at most (1 - alpha_t)|V|; a fractional product is rounded up:
 * ceil(keep_ratio * V - 1e-9), clamped to [1, V].  Returns 0 if V < 1. */
int d3tom_keep_count(int V, double keep_ratio);

/* Linear timestep-dependent schedule (Section 3.2, "Timestep-Dependent Merge Schedule"): the
 * value at decoding-order step `step` in 0..T-1, moving linearly from r_first to r_last.  The
 * caller decides whether the quantity is a merge ratio or a keep ratio and which way it runs. */
double d3tom_schedule(int step, int T, double r_first, double r_last);

/* Theoretical FLOPs of a whole denoising trajectory under the paper's cost model (Section 4.3
 * and Appendix B): FLOPs_layer(n) = 4 n d^2 + 2 n^2 d + 3 n d m; the merge inside layer l_star
 * at constant merge ratio alpha adds 2 alpha (1-alpha) |V|^2 d + alpha |V| d per step; the first
 * of the T steps runs unmerged (empty decider set).  alpha = 0 gives the unmerged baseline. */
double d3tom_model_flops(double alpha, int l_star, int L, int T, int V, int P, int O, int d, int m);

/* Bytes of workspace the given entry point needs for at most B samples of at most max_N tokens,
 * max_V visual tokens and max_D deciders each, with H heads of size dh (d = H * dh). */
size_t d3tom_workspace_bytes(int op, int B, int max_N, int max_V, int H, int dh, int max_D);

/* Static, human-readable name of a status code. */
const char* d3tom_status_string(int status);

/* ------------------------------------------------------------------------------------------
 * d3tom_importance — decider-guided importance map (Section 3.2, "The Decider-Guided
 * Mechanism": attention matrix A and S_j = sum_{i in D} A_ij; Algorithm 1, the line forming S).
 *
 * For sample b, head h and decider row i: softmax over ALL keys of the sample of
 * scale * q[i,h,:] . k[j,h,:]; the probabilities are summed over the sample's decider rows and
 * averaged over heads; only the visual columns are written.  The N x N matrix is never formed.
 *
 *   q, k        [seq_off[B], H, dh]  dt
 *   seq_off     int32[B+1]  first token of each sample (seq_off[0] = 0)
 *   dec_idx     int32[dec_off[B]]  decider positions, relative to the sample's first token
 *   dec_off     int32[B+1]
 *   min_D,max_D host-known smallest / largest decider count over the batch
 *   vis_start   int32[B]  first visual token, relative to the sample's first token
 *   vis_count   int32[B]  |V| of each sample
 *   score_off   int32[B+1]  offsets into `scores` (prefix sums of vis_count)
 *   max_N,max_V host-known largest token / visual-token count per sample
 *   scores      float[score_off[B]]  out
 *
 * min_D == 0 returns D3TOM_ERR_NO_DECIDERS (Algorithm 1 skips the merge when the decider set is
 * empty; the caller then runs the layer at full length).  max_D > D3TOM_MAX_DECIDERS or a dh the
 * kernels are not built for (bf16: 64 or 128; f32: any multiple of 4 up to 256) returns
 * D3TOM_ERR_UNSUPPORTED.
 * ---------------------------------------------------------------------------------------- */
int d3tom_importance(const void* q, const void* k, int dt,
                     int B, const int32_t* seq_off, int H, int dh, float scale,
                     const int32_t* dec_idx, const int32_t* dec_off, int min_D, int max_D,
                     const int32_t* vis_start, const int32_t* vis_count, const int32_t* score_off,
                     int max_N, int max_V,
                     float* scores, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * d3tom_importance_static — d3tom_importance for callers that cannot allocate device memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same kernels and bit-identical scores, but no workspace argument: the scratch memory is a
 * file-scope device array of D3TOM_IMPORTANCE_STATIC_BYTES inside the library, which every GPU the
 * library runs on holds until the process ends.  The call allocates and frees nothing (no
 * hipMalloc / hipFree, no allocating library routine); the first call on a device only looks up
 * the array's device address.
 *
 * Shapes whose workspace (d3tom_workspace_bytes(D3TOM_OP_IMPORTANCE, ...)) exceeds
 * D3TOM_IMPORTANCE_STATIC_BYTES return D3TOM_ERR_UNSUPPORTED before anything is enqueued.  All calls
 * on one GPU share that GPU's array, which keeps the previous call's contents (no kernel relies on
 * them): two calls that overlap on one GPU (different streams or threads) race and give
 * unspecified scores; calls on one stream are ordered and safe.
 * ---------------------------------------------------------------------------------------- */
#define D3TOM_IMPORTANCE_STATIC_BYTES (16u << 20)
int d3tom_importance_static(const void* q, const void* k, int dt,
                            int B, const int32_t* seq_off, int H, int dh, float scale,
                            const int32_t* dec_idx, const int32_t* dec_off, int min_D, int max_D,
                            const int32_t* vis_start, const int32_t* vis_count, const int32_t* score_off,
                            int max_N, int max_V, float* scores, void* stream);

/* ------------------------------------------------------------------------------------------
 * d3tom_select_topk — keep / merge partition (Section 3.2: V_kept holds the tokens whose rank is
 * at most the kept count; Algorithm 1, the TopK line).
 *
 * Rank order is (score descending, index ascending): equal scores at the threshold go to the
 * lower index.  Output order is ascending position (positions are removed, never reordered).
 *
 *   scores    float[score_off[B]]
 *   keep_k    int32[B]   kept count per sample, 1 <= keep_k[b] <= vis_count[b] (d3tom_keep_count)
 *   kept_off  int32[B+1] offsets into kept_idx (prefix sums of keep_k)
 *   max_V     host-known largest |V|; above D3TOM_MAX_VISUAL returns D3TOM_ERR_UNSUPPORTED
 *   kept_idx  int32[kept_off[B]]  out: kept tokens, ascending, relative to the visual block
 *   slot_of   int32[score_off[B]] out: kept token -> its index in kept_idx (0..k-1), other -> -1
 * ---------------------------------------------------------------------------------------- */
int d3tom_select_topk(const float* scores, int B, const int32_t* score_off, const int32_t* keep_k,
                      const int32_t* kept_off, int max_V,
                      int32_t* kept_idx, int32_t* slot_of,
                      void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * d3tom_merge — similarity-based merging (Section 3.2, "Similarity-Based Merging": cosine argmax
 * over the kept set, h_k* <- h_k* + h_m, removal of the merged positions; Algorithm 1, the FORALL
 * block and the "Remove positions" line; Section 4.4 for similarity taken on other features).
 *
 * Every pruned visual token m goes to slot argmax_r cos(sim_m, sim_kept[r]), computed from the
 * rows as given (all assignments first, aggregation afterwards); ties go to the lowest slot; a
 * zero row has cosine 0 with everything.  Output rows of sample b:
 *     [rows before the visual block | keep_k merged rows, ascending position | rows after it]
 * MEAN: merged row = (sum of member rows) / member count.  SUM: the plain sum (the paper's literal
 * update).  Accumulation is float32 in ascending member order, rounded once on store; a slot with
 * no absorbed token, and every non-visual row, is copied bit-exactly.
 *
 *   x         [seq_off[B], d]  dt   payload rows
 *   sim       NULL (use x) or [seq_off[B], d_sim] dt: rows the cosine is taken on
 *   d, d_sim  row lengths (d_sim ignored when sim is NULL)
 *   kept_idx, kept_off   as written by d3tom_select_topk
 *   max_N, max_V, max_keep, max_pruned, max_out  host-known maxima over the batch of N_b, |V_b|,
 *             keep_k[b], |V_b| - keep_k[b] and the output row count N_b - (|V_b| - keep_k[b])
 *   out_off   int32[B+1]  first output row of each sample; sample b emits
 *             N_b - (vis_count[b] - keep_k[b]) rows (Section 3.2, the post-merge length)
 *   y         [out_off[B], d] dt  out
 *   assign    int32[score_off-like: sum V_b] out or NULL: slot of every visual token
 *   counts    int32[kept_off[B]]  out or NULL: members per slot, the kept token included
 *   src_pos   int32[out_off[B]]   out or NULL: original position (within the sample) of each row
 *   vis_off   int32[B+1]  offsets of each sample's visual block into `assign` (prefix sums of
 *             vis_count)
 * ---------------------------------------------------------------------------------------- */
int d3tom_merge(const void* x, const void* sim, int d, int d_sim, int dt,
                int B, const int32_t* seq_off, const int32_t* vis_start, const int32_t* vis_count,
                const int32_t* vis_off, const int32_t* kept_idx, const int32_t* kept_off,
                int max_N, int max_V, int max_keep, int max_pruned, int max_out, int mode,
                const int32_t* out_off, void* y, int32_t* assign, int32_t* counts, int32_t* src_pos,
                void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * d3tom_merge_kv — the same merge applied to a key/value cache (Section 4.4, "Compatibility with
 * KV-Cache": pi(m) = argmax over kept k of the cosine of the cached key rows K_m, K_k; then
 * K_pi(m) <- K_pi(m) + K_m and V_pi(m) <- V_pi(m) + V_m, and the merged positions are dropped).
 *
 * The routing is computed once, on the rows of k_cache (all d = H * dh elements of a row), and
 * both caches are aggregated with it in one pass.  mode, row order, rounding, ties and the index
 * outputs are those of d3tom_merge; SUM is the printed update, MEAN divides both caches by the
 * member count ("merge caches and renormalise").
 *
 *   k_cache, v_cache  [seq_off[B], d] dt   cached key / value rows (layout as in d3tom_merge: the
 *                     visual block of sample b is rows vis_start[b] .. + vis_count[b])
 *   k_out, v_out      [out_off[B], d] dt   out: the shortened caches
 *   all other arguments as in d3tom_merge; workspace size is that of D3TOM_OP_MERGE
 * ---------------------------------------------------------------------------------------- */
int d3tom_merge_kv(const void* k_cache, const void* v_cache, int d, int dt,
                   int B, const int32_t* seq_off, const int32_t* vis_start, const int32_t* vis_count,
                   const int32_t* vis_off, const int32_t* kept_idx, const int32_t* kept_off,
                   int max_N, int max_V, int max_keep, int max_pruned, int max_out, int mode,
                   const int32_t* out_off, void* k_out, void* v_out, int32_t* assign, int32_t* counts,
                   int32_t* src_pos, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * d3tom_merge_layer — the merge layer of one denoising step in one call (Algorithm 1, the block guarded by
 * "l = l* and the decider set is not empty": S from the decider rows, TopK at the step's keep ratio, cosine
 * assignment, aggregation, removal of the merged positions), i.e. d3tom_importance -> d3tom_select_topk ->
 * d3tom_merge on one workspace, with the kept counts computed ON THE DEVICE from per-sample keep ratios
 * (Section 3.2, "Timestep-Dependent Merge Schedule": the ratio may come from a schedule evaluated on the
 * device), so that no host integer sits between the importance map and the merge.
 *
 *   keep_ratio  double[B] (device): keep ratio 1 - alpha_t of each sample; the kept count is
 *               ceil(keep_ratio * |V_b| - 1e-9) clamped to [1, |V_b|], the arithmetic of d3tom_keep_count
 *   min_keep, max_keep   host-known bounds on the kept counts (1 <= min_keep <= every count <= max_keep <=
 *               max_V); they only size the launches: tight bounds give the launch shapes of the separate
 *               calls, loose ones (1, max_V) are always valid
 *   scores      float[vis_off[B]] out
 *   keep_k      int32[B] out, kept_off int32[B+1] out, out_off int32[B+1] out: what the separate calls take as
 *               inputs (counts, their prefix sums, first output row of each sample)
 *   kept_idx    int32[B * max_keep or more] out, packed by kept_off
 *   y           [sum of output rows, d] out; room for seq_off[B] rows is always enough
 *   assign, counts, src_pos   optional outputs as in d3tom_merge
 *   all other arguments as in d3tom_importance / d3tom_merge; vis_off = prefix sums of vis_count
 * Results are those of the three separate calls, bit for bit when the bounds are tight.  The selection launch
 * also reads every visual row of the similarity features once (it computes the row norms there, on compute
 * units the selection leaves idle, and the rows are then cached for the cosine step), so vis_start / vis_count
 * must describe rows inside x (sim) as for d3tom_merge; batches whose visual rows exceed 160 MB take the plain
 * sequence of launches.
 * Workspace: d3tom_merge_layer_workspace_bytes.  Statuses as for the separate calls (an empty decider set
 * returns D3TOM_ERR_NO_DECIDERS before anything is enqueued).
 * ---------------------------------------------------------------------------------------- */
size_t d3tom_merge_layer_workspace_bytes(int B, int max_N, int max_V, int H, int dh, int max_D);
int d3tom_merge_layer(const void* q, const void* k, const void* x, const void* sim, int d, int d_sim, int dt,
                      int B, const int32_t* seq_off, int H, int dh, float scale,
                      const int32_t* dec_idx, const int32_t* dec_off, int min_D, int max_D,
                      const int32_t* vis_start, const int32_t* vis_count, const int32_t* vis_off,
                      const double* keep_ratio, int max_N, int max_V, int min_keep, int max_keep, int mode,
                      float* scores, int32_t* keep_k, int32_t* kept_off, int32_t* kept_idx, int32_t* out_off,
                      void* y, int32_t* assign, int32_t* counts, int32_t* src_pos,
                      void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * d3tom_attend — bidirectional attention over the shortened sequence (Section 3.2: the shortened
 * tensor propagates through the later layers; Section 4.3: the 2 n^2 d term of FLOPs_layer; the
 * model attends without a causal mask).
 *
 * Per sample and head: o = softmax(scale * q k^T) v over all keys of the sample (variable-length
 * batch, no mask, no dropout).  bf16: MFMA with float32 online-softmax state; f32: plain float.
 *
 *   q, k, v     [cu_seqlens[B], H, dh] dt
 *   scale       logit scale, finite and > 0 (1/sqrt(dh) in the paper's models); otherwise
 *               D3TOM_ERR_INVALID_ARG (same rule in d3tom_importance)
 *   cu_seqlens  int32[B+1]  first token of each sample
 *   max_seqlen  host-known longest sample
 *   o           [cu_seqlens[B], H, dh] dt  out
 * ---------------------------------------------------------------------------------------- */
int d3tom_attend(const void* q, const void* k, const void* v, int dt,
                 int B, const int32_t* cu_seqlens, int max_seqlen, int H, int dh, float scale,
                 void* o, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * d3tom_attend_weighted — d3tom_attend with per-key weights taken from the merge's member counts
 * (Section 3.2 aggregates by a plain sum; under MEAN aggregation a merged row stands for count_r
 * original tokens but would enter the softmax of later layers once).  Key row j of sample b gets the
 * weight w_j = counts[kept_off[b] + j - vis_start[b]] if it is one of the sample's merged rows
 * (vis_start[b] <= j < vis_start[b] + kept_off[b+1] - kept_off[b], the layout d3tom_merge writes), else 1,
 * and the attention probabilities are softmax_j(scale * q k_j + log w_j): exactly the attention over the
 * sequence with row j written w_j times.  All weights 1 gives d3tom_attend.
 *
 *   counts, kept_off   as written by / passed to d3tom_merge (counts >= 1)
 *   vis_start          int32[B]  first merged row of each sample (= first visual token)
 *   other arguments as in d3tom_attend.  bf16 with dh 64 / 128 keeps a sample's log-weights in LDS:
 *   max_seqlen above 3584 returns D3TOM_ERR_UNSUPPORTED there.
 * ---------------------------------------------------------------------------------------- */
int d3tom_attend_weighted(const void* q, const void* k, const void* v, int dt,
                          int B, const int32_t* cu_seqlens, int max_seqlen, int H, int dh, float scale,
                          const int32_t* counts, const int32_t* kept_off, const int32_t* vis_start,
                          void* o, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * d3tom_update_deciders — the decider set for the next merge (Section 3.2, "The Decider-Guided
 * Mechanism": D = { positions that hold a token now and held [MASK] in the preceding iteration };
 * Algorithm 1, the last line of the denoising loop; an empty set means "run this step unmerged").
 *
 *   prev_ids, cur_ids  int32[seq_off[B]]  token ids of every position one iteration ago / now
 *                      (prompt and visual positions never hold mask_id, so they never qualify)
 *   mask_id            id of the [MASK] token
 *   max_D              host-known cap per sample, 1 .. D3TOM_MAX_DECIDERS; a sample with more newly
 *                      revealed positions lists the max_D lowest ones (dec_count still reports all)
 *   dec_idx            int32[B * max_D]  out: decider positions within each sample, ascending, packed
 *   dec_off            int32[B + 1]      out: offsets into dec_idx (prefix sums of the listed counts)
 *   dec_count          int32[B] out or NULL: number of newly revealed positions per sample
 *
 * dec_idx / dec_off are exactly what d3tom_importance takes.  Its min_D / max_D arguments are host
 * values: a caller that cannot bound them otherwise copies dec_count (4 B bytes) back once per
 * step; a sample with dec_count 0 must skip the merge (D3TOM_ERR_NO_DECIDERS mirrors that case).
 * ---------------------------------------------------------------------------------------- */
int d3tom_update_deciders(const int32_t* prev_ids, const int32_t* cur_ids, int mask_id,
                          int B, const int32_t* seq_off, int max_D,
                          int32_t* dec_idx, int32_t* dec_off, int32_t* dec_count, void* stream);

/* ------------------------------------------------------------------------------------------
 * The blocks around the merge layer (Algorithm 1, the loop over layers l = 1 .. L_model: every layer
 * is a self-attention part followed by a feed-forward part, the merge sits between the two inside
 * layer l*; Section 4.3 counts a layer as 4 n d^2 + 2 n^2 d + 3 n d m FLOPs).  The paper's models are
 * Llama-style: pre-norm residual blocks with RMSNorm, rotary position embedding on q and k, and a
 * SwiGLU feed-forward part.  bf16 storage, float32 arithmetic, one rounding where a tensor is stored.
 * ---------------------------------------------------------------------------------------- */

/* d3tom_rmsnorm: y[r, :] = x[r, :] / sqrt(mean(x[r, :]^2) + eps) * gain.
 *   x, y  [rows, d] bf16 (y may be x)   gain [d] bf16   d a multiple of 8, at most 8192; eps >= 0 */
int d3tom_rmsnorm(const void* x, const void* gain, int rows, int d, float eps, void* y, void* stream);

/* d3tom_rope: rotary position embedding, in place on q and k [rows, H, dh] bf16.  Channel c < dh/2 of
 * every head is paired with channel c + dh/2; the pair is rotated by pos[r] * theta^(-2c/dh) radians.
 * After the merge the kept tokens keep their original positions (Section 3.2 removes positions, it
 * does not renumber them): pos is then the src_pos output of d3tom_merge.
 *   pos  int32[rows]   dh a multiple of 16, at most 256   theta > 1 */
int d3tom_rope(void* q, void* k, const int32_t* pos, int rows, int H, int dh, float theta, void* stream);

/* d3tom_linear: out = a w^T, the projections of a block (the 4 n d^2 and 3 n d m terms), on MFMA.
 *   a         [rows, K] bf16
 *   w         [n_w_rows, K] bf16: one row per output feature
 *   epilogue  D3TOM_LINEAR_PLAIN     out[rows, n_w_rows] = a w^T.  With 0 < out_chunk < n_w_rows the
 *                                    result is written as n_w_rows / out_chunk matrices [rows, out_chunk]
 *                                    one after the other (q, k, v from one stacked weight).
 *             D3TOM_LINEAR_RESIDUAL  out = residual + a w^T, residual [rows, n_w_rows] bf16; out may be
 *                                    the residual buffer itself.
 *             D3TOM_LINEAR_SWIGLU    w = F gate rows followed by F up rows (n_w_rows = 2F);
 *                                    out[rows, F] = silu(a w_gate^T) * (a w_up^T).
 *   out_chunk 0 = one matrix; otherwise a multiple of 8 dividing n_w_rows (PLAIN only)
 * K must be a multiple of 64 and the output row length a multiple of 8; each operand below 2 GiB;
 * otherwise D3TOM_ERR_UNSUPPORTED. */
typedef enum { D3TOM_LINEAR_PLAIN = 0, D3TOM_LINEAR_RESIDUAL = 1, D3TOM_LINEAR_SWIGLU = 2 } d3tom_linear_epilogue;
int d3tom_linear(const void* a, const void* w, int rows, int n_w_rows, int K, int epilogue,
                 const void* residual, void* out, int out_chunk, void* stream);
/* The same with the workgroup's row-tile height fixed to tile * 64 rows (tile = 1, 2 or 4) instead of
 * chosen from the problem size; for tuning and tests. */
int d3tom_linear_tile(const void* a, const void* w, int rows, int n_w_rows, int K, int epilogue,
                      const void* residual, void* out, int out_chunk, int tile, void* stream);

/* Weights of one block, device pointers, bf16. */
typedef struct {
    const void* attn_norm;   /* [d]      RMSNorm gain in front of the attention part        */
    const void* w_qkv;       /* [3d, d]  rows of W_Q, then W_K, then W_V                      */
    const void* w_o;         /* [d, d]   attention output projection                          */
    const void* ffn_norm;    /* [d]      RMSNorm gain in front of the feed-forward part       */
    const void* w_gate_up;   /* [2F, d]  F gate rows, then F up rows                          */
    const void* w_down;      /* [d, F]                                                        */
} d3tom_block_weights;

/* Workspace of d3tom_stack_step for a sequence of N tokens (V of them visual, at most max_D
 * deciders), hidden size d = H * dh, feed-forward width F. */
size_t d3tom_stack_workspace_bytes(int N, int d, int H, int F, int V, int max_D);

/* ------------------------------------------------------------------------------------------
 * d3tom_stack_step — one denoising step through all L blocks for one sample (Algorithm 1, the body
 * of the loop over t without Embed / Decode):
 *
 *   for l = 1 .. L:   a = rmsnorm(h);  q, k, v = a W_Q^T, a W_K^T, a W_V^T;  rope(q, k) at the tokens'
 *                     original positions;  h~ = h + attend(q, k, v) W_O^T
 *                     if l == merge_layer and D > 0:  S = importance(q, k, deciders);  kept = top-k(S);
 *                         h~ = merge(h~, kept)          -- N -> N - (V - keep_k) rows from here on
 *                     h = h~ + (silu(f W_gate^T) * (f W_up^T)) W_down^T  with  f = rmsnorm(h~)
 *
 * i.e. the importance map comes from the attention the merge block itself just computed, the cosine is
 * taken on that block's post-attention hidden states, and the block's own feed-forward part already runs
 * on the shortened sequence.  D == 0 (first step, empty decider set) or merge_layer outside 1 .. L runs
 * every block at full length.  Logit scale 1/sqrt(dh); no final norm, no decoding head.
 *
 *   x          [N, d] bf16     hidden states entering block 1 (never written)
 *   blocks     HOST array of L d3tom_block_weights (device pointers inside)
 *   dec_idx    int32[D]  decider positions (device; may be NULL when D == 0)
 *   vis_start, V, keep_k   the visual block and the kept count (d3tom_keep_count)
 *   mode       d3tom_merge_mode
 *   y          [n_out, d] bf16 out, n_out = N - (V - keep_k) when merging, else N (room for N rows is
 *              always enough)
 *   src_pos    int32[n_out] out or NULL: original position of every output row
 *   scores_out float[V], kept_idx_out int32[keep_k], assign_out int32[V]: the merge layer's intermediate
 *              results, out or NULL (written only when merging)
 *   n_out      HOST int out or NULL
 * dh must be 64 or 128, d and F multiples of 64, d at most 8192, every activation and weight matrix below
 * 2 GiB (otherwise D3TOM_ERR_UNSUPPORTED, before anything is enqueued).
 * ---------------------------------------------------------------------------------------- */
int d3tom_stack_step(const void* x, int N, int d, int H, int F, int L, const d3tom_block_weights* blocks /* host */,
                     int merge_layer, const int32_t* dec_idx, int D, int vis_start, int V, int keep_k, int mode,
                     float eps, float theta, void* y, int32_t* src_pos, float* scores_out, int32_t* kept_idx_out,
                     int32_t* assign_out, int* n_out /* host */, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * d3tom_stack_step_batch — d3tom_stack_step for B samples concatenated along the token axis (Algorithm 1 is
 * stated per sample; samples only meet in the launches: projections and normalisations run over all rows,
 * attention and the merge layer per sample).  Per-sample sizes are HOST arrays of B entries (they size the
 * launches); everything else is as in d3tom_stack_step, with outputs concatenated in sample order.
 *
 *   x          [sum N_b, d] bf16
 *   N, D, vis_start, V, keep_k   host int32[B]; vis_start / V / keep_k may be NULL when no sample has deciders
 *   dec_idx    device int32[sum D_b], the samples' decider positions (within the sample) back to back
 *   y          [sum n_out_b, d] out, n_out_b = N_b - (V_b - keep_k[b]) when merging, else N_b
 *   src_pos    int32[sum n_out_b] out or NULL (positions within the sample)
 *   scores_out float[sum V_b], kept_idx_out int32[sum keep_k], assign_out int32[sum V_b]: out or NULL
 *   n_out      HOST int[B] out or NULL
 * B above D3TOM_STACK_MAX_BATCH returns D3TOM_ERR_UNSUPPORTED.  Inside one batch all samples take the same path:
 * if some samples have deciders and others none, the call returns D3TOM_ERR_NO_DECIDERS before anything is
 * enqueued (the caller splits the batch).  Workspace: d3tom_stack_batch_workspace_bytes.
 * ---------------------------------------------------------------------------------------- */
#define D3TOM_STACK_MAX_BATCH 64
size_t d3tom_stack_batch_workspace_bytes(int B, int sum_N, int max_N, int d, int H, int F, int sum_V, int max_V, int max_D);
int d3tom_stack_step_batch(const void* x, int B, const int32_t* N /* host */, int d, int H, int F, int L,
                           const d3tom_block_weights* blocks /* host */, int merge_layer, const int32_t* dec_idx,
                           const int32_t* D /* host */, const int32_t* vis_start /* host */, const int32_t* V /* host */,
                           const int32_t* keep_k /* host */, int mode, float eps, float theta, void* y, int32_t* src_pos,
                           float* scores_out, int32_t* kept_idx_out, int32_t* assign_out, int* n_out /* host */,
                           void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Per-kernel timing (diagnostics; used by the benchmark for its roofline figures).  While enabled,
 * every kernel launch of the four entry points is bracketed by HIP events on the caller's stream.
 * d3tom_profile_collect waits for the recorded events, adds up milliseconds and launch counts per
 * kernel into the host arrays ms_sum[n] / calls[n] (n >= d3tom_profile_kernel_count()), and
 * forgets the records.  Not thread-safe with respect to concurrent launches.
 * ---------------------------------------------------------------------------------------- */
int d3tom_profile_enable(int on);
int d3tom_profile_kernel_count(void);
const char* d3tom_profile_kernel_name(int kernel);
int d3tom_profile_collect(double* ms_sum /* host */, long long* calls /* host */, int n);

#ifdef __cplusplus
}
#endif
#endif /* D3TOM_H */

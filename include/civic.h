/*
 * civic.h — C ABI of the compact-prefill hot path of CIVIC (path-consistent compact
 * inference for vision-language models) for AMD MI355X (gfx950).
 *
 * The path, in call order:
 *   civic_score        per visual token, the anchor logit of Eq. 8 (civic_score_visual: the same on
 *                      the frame spans of the dense sequence, in place)
 *   civic_select       kept set under a global token budget and spatial retention floors
 *   civic_compact      Merge of Eq. 13: one contiguous, order-preserving sequence with the
 *                      position ids carried along (sentence after Eq. 14)
 *   civic_prefill_attn dense grouped-query prefill attention over the compact sequence
 *                      (the beta * N_l * (L+M_p)^2 * D_l term of Eq. 7)
 *   civic_kv_write     contiguous, un-paged KV-cache rows (the gamma * N_l * (L+M_p) * D_l
 *                      term of Eq. 7, ratio of Eq. 14)
 *   civic_prefill_attn_kv  the last two as one call (the K/V rows are read once)
 * and, after the prefill, per generated token:
 *   civic_decode_attn  one query per sequence against the compact cache (inside C_dec of Eq. 7)
 *
 * Conventions shared by every call
 *   - Plain C.  Every function that launches work returns int: CIVIC_OK or a negative
 *     CIVIC_ERR_* code.  Nothing throws, aborts or prints.
 *   - Unless a parameter says "host", tensor pointers are DEVICE pointers owned by the
 *     caller.  The library allocates nothing, frees nothing and keeps no pointer after the
 *     call returns.  civic_grid and frame_start are HOST memory, read during the call only.
 *   - Calls are asynchronous on the hipStream_t passed as `void* stream` (NULL = the
 *     default stream).  They never synchronise and never read device memory back: every
 *     output shape is a function of the arguments alone (civic_kept_count).
 *   - All argument checks happen before the first HIP call, so a rejected call has no
 *     side effect.  On CIVIC_ERR_HIP the outputs are unspecified; no out-of-bounds access
 *     is made in any case.
 *   - A tensor pointer may be NULL when the tensor it names has no elements (no rows, an
 *     empty batch, nothing kept and no text); otherwise NULL is CIVIC_ERR_INVALID_ARG.
 *   - dtype: CIVIC_F32 (4-byte IEEE) or CIVIC_BF16 (2-byte bfloat16).
 *   - Re-entrant.  Global mutable state: the last HIP error code, and per kernel and device one flag
 *     that its dynamic LDS limit has been raised (set once, never cleared); per thread, the two
 *     event handles of civic_time_next_kernel between arming and the next launch.
 */
#ifndef CIVIC_H
#define CIVIC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    CIVIC_OK = 0,
    CIVIC_ERR_INVALID_ARG = -1, /* null pointer, bad shape, misalignment, inconsistent sizes  */
    CIVIC_ERR_WORKSPACE   = -2, /* workspace missing or smaller than the *_workspace_bytes()  */
    CIVIC_ERR_UNSUPPORTED = -3, /* valid but outside what the kernels cover (limits below)    */
    CIVIC_ERR_HIP         = -4  /* a HIP call failed; see civic_last_hip_error()              */
};

enum { CIVIC_F32 = 0, CIVIC_BF16 = 1 };

/* Limits of this implementation (exceeding them gives CIVIC_ERR_UNSUPPORTED). */
#define CIVIC_MAX_VISUAL_TOKENS 32768 /* N_v per sample: civic_select keeps the keys in LDS  */
#define CIVIC_MAX_FRAMES        128   /* frames per sample in civic_compact                  */
#define CIVIC_MAX_SCORE_DIM     8192  /* hidden size in civic_score (bf16; 4096 for fp32)    */
#define CIVIC_MAX_HEAD_DIM      256   /* head_dim in civic_prefill_attn                      */

/* One sample's visual layout; every batch item shares it.  Visual-local token index
 * v = f*height*width + r*width + c (frame-major raster).  The cell of v is
 * (f, r / cell_h, c / cell_w); cells at the right/bottom edge may be smaller.  The paper
 * names the budget ("token budget", the maximum number of visual tokens propagated
 * downstream) and the floor ("minimum keep ratio", "adaptive spatial retention floor") in
 * its Ablation Study without a formula; the reading implemented is documented at
 * civic_select. */
typedef struct {
    int32_t frames;      /* images or video frames, each one contiguous raster span, > 0     */
    int32_t height;      /* merged-grid rows per frame, > 0                                   */
    int32_t width;       /* merged-grid columns per frame, > 0                                */
    int32_t cell_h;      /* spatial cell height, > 0                                          */
    int32_t cell_w;      /* spatial cell width, > 0                                           */
    int32_t cell_floor;  /* tokens kept per cell at least (clipped to the cell's size), >= 0  */
    int32_t frame_floor; /* further tokens kept per frame on top of its cells' floors, >= 0   */
    int32_t budget;      /* global keep budget over the sample's N_v tokens, 0..N_v           */
} civic_grid;

/* Last hipError_t (as int) recorded by a call that returned CIVIC_ERR_HIP on this thread's
 * process; 0 if none. */
int civic_last_hip_error(void);

/* Measurement hook (no passage of the paper: it serves whoever reports a kernel's own duration).
 * Arms a one-shot timer on the calling thread: the next kernel that thread launches through this
 * library - the first kernel of the next entry-point call, for calls that launch several - carries
 * the two events on its stream, `start_event` taking the time the kernel begins to run and
 * `stop_event` the time it ends, so hipEventElapsedTime(start, stop) after a synchronisation is the
 * kernel's duration without launch latency or the gap to the kernel before it.  Both are hipEvent_t
 * handles (host values) created with timing enabled, owned by the caller, distinct.  Two null
 * pointers disarm.  The timed launch uses the extended launch call and must not be captured into a
 * HIP graph.  CIVIC_ERR_INVALID_ARG if exactly one is null or both are the same event. */
int civic_time_next_kernel(void* start_event, void* stop_event);

/* Number of visual tokens civic_select keeps per sample: K = max(budget, sum of floors),
 * where a cell contributes min(cell_floor, its size) and a frame min(frame_floor, what its
 * cell floors leave).  A pure host function of the grid; negative CIVIC_ERR_* on a bad grid.
 * The compact sequence length of Eq. 13 is L + M_p = seq_len - N_v + K. */
int64_t civic_kept_count(const civic_grid* grid /* host */);

/* Scratch sizes (host functions; 0 is a valid answer and then workspace may be NULL). */
size_t civic_select_workspace_bytes(const civic_grid* grid /* host */, int32_t batch);
size_t civic_compact_workspace_bytes(int32_t batch, int64_t seq_len);

/* Q_A = Norm(LN(a)) of Eq. 8 for one anchor row: layer norm without affine (its epsilon
 * cancels under the l2 normalisation that follows), then unit l2 norm.  HOST pointers;
 * computed in double, rounded to fp32.  The result has zero mean and unit norm, which is
 * what civic_score expects.  CIVIC_ERR_INVALID_ARG if a has no variance. */
int civic_anchor_normalize(const float* anchor /* host [dim] */, int32_t dim,
                           float* anchor_q /* host [dim] */);

/* Token scoring.  scores[i] = inv_tau * < anchor_q, Norm(LN(x_i)) > for each of n_rows
 * hidden rows x_i: the pre-softmax logit of Eq. 8 with a single anchor (with one anchor the
 * softmax over tokens is monotone in it).  Norm(LN(x)) = (x - mean) / ||x - mean||; a row
 * without variance scores 0.  fp32 accumulation.  fp32 rows take two passes (mean, then the
 * centred norm and dot product).  bf16 rows take one pass (sum, sum of squares, dot product;
 * the anchor is used as two bf16 terms, 16 mantissa bits) whenever |mean| <= the row's
 * standard deviation, and the two centred passes otherwise; both agree with the fp64 value
 * to ~1e-6.  Rows whose sum of squares overflows fp32 are outside the supported range.
 *   hidden     [n_rows, row_stride] elements of `dtype`, row_stride >= dim, in elements
 *   anchor_q   device [dim] fp32, zero mean, unit norm (civic_anchor_normalize)
 *   scores     device [n_rows] fp32
 * dim must be a multiple of 8 (bf16) or 4 (fp32) and at most CIVIC_MAX_SCORE_DIM (half of
 * it for fp32); hidden and row_stride*sizeof(element) must be 16-byte aligned. */
int civic_score(const void* hidden, int dtype, int64_t n_rows, int64_t row_stride, int32_t dim,
                const float* anchor_q, float inv_tau, float* scores, void* stream);

/* civic_score on the visual tokens where they lie: frame f of batch item b occupies rows
 * [frame_start[f], frame_start[f] + height*width) of that item's dense sequence (the "dense visual
 * placeholder spans" that Eq. 13 merges from), with text rows in between, so the visual rows are not at
 * one uniform stride and a single civic_score call cannot address them.  One launch scores them all:
 * scores[b, f*height*width + t] is the civic_score value of row frame_start[f] + t of item b.
 *   hidden      device [batch, seq_len, dim] of `dtype`, dense
 *   frame_start host [grid->frames] int64, ascending, spans inside [0, seq_len), disjoint
 *   scores      device [batch, N_v] fp32, N_v = frames*height*width
 * Arithmetic, accuracy and dim limits are civic_score's; grid->frames <= CIVIC_MAX_FRAMES,
 * batch * frames <= 65535, seq_len < 2^31. */
int civic_score_visual(const void* hidden, int dtype, int32_t batch, int64_t seq_len, int32_t dim,
                       const civic_grid* grid /* host */, const int64_t* frame_start /* host */,
                       const float* anchor_q, float inv_tau, float* scores, void* stream);

/* Token selection.  With the strict order "higher score first, equal scores (IEEE ==, so
 * -0 equals +0) to the lower index", per sample:
 *   (1) every cell keeps its first min(cell_floor, size) tokens;
 *   (2) every frame keeps the first min(frame_floor, remaining) of its tokens not kept yet;
 *   (3) the first max(0, budget - kept so far) tokens of the sample not kept yet are kept.
 * Exactly K = civic_kept_count(grid) tokens result for any scores.  NaN scores are a caller
 * error (the result is then unspecified, but in bounds).
 *   scores     device [batch, N_v] fp32
 *   kept_idx   device [batch, K] int32, visual-local indices in ascending order
 *   keep_flags device [batch, N_v] uint8 (1 = kept) or NULL
 * N_v <= CIVIC_MAX_VISUAL_TOKENS. */
int civic_select(const float* scores, int32_t batch, const civic_grid* grid /* host */,
                 int32_t* kept_idx, uint8_t* keep_flags,
                 void* workspace, size_t workspace_bytes, void* stream);

/* Compact merge (Eq. 13).  Frame f of the grid occupies sequence positions
 * [frame_start[f], frame_start[f] + height*width); every other position is text.  The
 * output keeps all text tokens and the visual tokens listed in kept_idx, in their original
 * order, as one dense sequence of length S_c = seq_len - N_v + K.  Rows are copied bit for
 * bit; position ids are copied, never renumbered (text positions preserved, visual
 * positions inherited from the dense span).
 *   hidden      device [batch, seq_len, dim] of `dtype`, dense
 *   pos_ids     device [3, batch, seq_len] int32 (temporal, height, width ids)
 *   frame_start host [grid->frames] int64, ascending, spans inside [0, seq_len), disjoint
 *   kept_idx    device [batch, n_kept] int32 ascending (civic_select's output);
 *               n_kept in [0, N_v]
 *   hidden_c    device [batch, S_c, dim]
 *   pos_c       device [3, batch, S_c] int32
 *   src_idx     device [batch, S_c] int32: dense sequence index of every compact token
 * frames <= CIVIC_MAX_FRAMES and seq_len < 2^31.  hidden and hidden_c must be aligned to
 * min(16, largest power of two dividing the row size in bytes). */
int civic_compact(const void* hidden, int dtype, int32_t dim, const int32_t* pos_ids,
                  int32_t batch, int64_t seq_len, const civic_grid* grid /* host */,
                  const int64_t* frame_start /* host */, const int32_t* kept_idx, int64_t n_kept,
                  void* hidden_c, int32_t* pos_c, int32_t* src_idx,
                  void* workspace, size_t workspace_bytes, void* stream);

/* The front of the path in one call: civic_score_visual (Eq. 8), civic_select (budget and
 * floors) and civic_compact (Eq. 13) enqueued back to back on `stream`, with n_kept =
 * civic_kept_count(grid).  The results are those of the three calls, bit for bit; what the
 * call saves is host time (one crossing from the caller's language instead of three).
 * Arguments as in the three calls; scores [batch, N_v] and kept_idx [batch, K] are outputs
 * here (intermediate results the caller may want).  Every check of every stage runs before
 * the first launch. */
int civic_compact_prefill(const void* hidden, int dtype, int32_t batch, int64_t seq_len, int32_t dim,
                          const int32_t* pos_ids, const civic_grid* grid /* host */,
                          const int64_t* frame_start /* host */, const float* anchor_q, float inv_tau,
                          float* scores, int32_t* kept_idx, void* hidden_c, int32_t* pos_c,
                          int32_t* src_idx, void* workspace, size_t workspace_bytes, void* stream);

/* The same path for a batch whose samples differ in length and grid (images of different grid sizes in one
 * batch; the rectangular civic_grid covers one shape per call): the samples' rows are packed back to back along
 * the token axis and every sample is scored, selected and merged by itself, with its own grid, floors and
 * budget (Eq. 13 per sample; results equal the rectangular calls on that sample alone, bit for bit).
 *
 * civic_ragged_offsets (host only) turns the samples' lengths and grids into the row offsets of the packed
 * tensors, [batch + 1] int64 each (any of the three outputs may be NULL):
 *   seq_offsets      host [batch + 1], seq_offsets[0] = 0: sample b owns dense rows [seq_offsets[b], seq_offsets[b+1])
 *   grids            host [batch] civic_grid, one per sample
 *   visual_offsets   N_v of the samples before b;  kept_offsets  K of the samples before b (civic_kept_count);
 *   compact_offsets  compact rows before b, a sample's count being its length - N_v + K
 * CIVIC_ERR_INVALID_ARG on a bad grid or a sample shorter than its visual tokens.
 *
 * civic_compact_prefill_ragged: the three stages of civic_compact_prefill for all samples - the scores of up to 64
 * frame spans per launch, the selection of up to 16 samples per launch (a workgroup per sample, each with its own
 * grid), the merge of up to 24 samples per launch (a sample of more than 8 frames by a launch of its own, together
 * with the samples of the same shape that follow it) - with every check of every sample before the first launch.  seq_offsets[batch] and the visual tokens together <= INT32_MAX, else
 * CIVIC_ERR_UNSUPPORTED.
 *   hidden      device [seq_offsets[batch], dim];  pos_ids  device [3, seq_offsets[batch]] int32
 *   frame_start host, the samples' frame starts one after the other (grids[b].frames entries each), each
 *               counted from its sample's first row
 *   scores      device [visual_offsets[batch]] fp32 (output);  kept_idx  device [kept_offsets[batch]] int32 (output,
 *               every sample's own ascending visual-local indices)
 *   hidden_c    device [compact_offsets[batch], dim];  pos_c  device [3, compact_offsets[batch]] int32
 *   src_idx     device [compact_offsets[batch]] int32, counted from the sample's first row
 * dim * sizeof(element) must be a multiple of 16 (every sample's first row is then aligned like the tensor). */
int civic_ragged_offsets(int32_t batch, const int64_t* seq_offsets /* host */, const civic_grid* grids /* host */,
                         int64_t* visual_offsets /* host */, int64_t* kept_offsets /* host */,
                         int64_t* compact_offsets /* host */);
int civic_compact_prefill_ragged(const void* hidden, int dtype, int32_t batch, const int64_t* seq_offsets /* host */,
                                 int32_t dim, const int32_t* pos_ids, const civic_grid* grids /* host */,
                                 const int64_t* frame_start /* host */, const float* anchor_q, float inv_tau,
                                 float* scores, int32_t* kept_idx, void* hidden_c, int32_t* pos_c, int32_t* src_idx,
                                 void* stream);

/* Prefill attention over the compact sequence: out[b,i,h,:] = sum_j softmax_j(scale *
 * <q[b,i,h,:], k[b,j,g,:]>) v[b,j,g,:] with g = h / (n_q_heads / n_kv_heads); j <= i when
 * causal (order of the compact sequence, not the position ids), every j otherwise.
 * bf16: MFMA with fp32 accumulation, fp32 online softmax, bf16 round-to-nearest-even
 * output.  fp32: plain fp32 arithmetic.
 *   q, out     device [batch, seq, n_q_heads, head_dim]; strides in ELEMENTS for
 *              (batch, token, head) in q_strides / o_strides (host int64[3]); head_dim is
 *              contiguous
 *   k, v       device [batch, seq, n_kv_heads, head_dim]; both use kv_strides
 *   softmax_scale  0 means 1/sqrt(head_dim)
 * Pointers and strides*sizeof(element) must be 16-byte aligned; head_dim a multiple of 8
 * and at most CIVIC_MAX_HEAD_DIM; n_q_heads a multiple of n_kv_heads; batch and n_q_heads at
 * most 65535.  The MFMA kernel serves bf16 with head_dim <= 128 while its 32-bit row offsets
 * and its grid allow (seq * q token stride below 2^31 elements, seq up to 2^22); sizes beyond
 * that, like fp32 and wider heads, take the plain kernel. */
int civic_prefill_attn(const void* q, const void* k, const void* v, void* out, int dtype,
                       int32_t batch, int32_t seq, int32_t n_q_heads, int32_t n_kv_heads,
                       int32_t head_dim, const int64_t* q_strides /* host [3] */,
                       const int64_t* kv_strides /* host [3] */,
                       const int64_t* o_strides /* host [3] */,
                       int32_t causal, float softmax_scale, void* stream);

/* KV-cache write: k_cache[b, g, pos0 + i, :] = k[b, i, g, :] and the same for v, bit for
 * bit; no other byte of the caches is touched.
 *   k, v       device [batch, seq, n_kv_heads, head_dim], strides in elements in kv_strides
 *   k_cache, v_cache  device [batch, n_kv_heads, s_max, head_dim] dense
 *   pos0       first cache row written; pos0 >= 0 and pos0 + seq <= s_max
 * Pointers and strides*sizeof(element) must be 16-byte aligned and head_dim*sizeof(element)
 * a multiple of 16. */
int civic_kv_write(const void* k, const void* v, const int64_t* kv_strides /* host [3] */,
                   int dtype, void* k_cache, void* v_cache, int32_t batch, int32_t seq,
                   int32_t n_kv_heads, int32_t head_dim, int64_t s_max, int64_t pos0,
                   void* stream);

/* civic_prefill_attn followed by civic_kv_write on the same K and V, as one call: the attention
 * term and the KV-write term of Eq. 7 belong to the same layer and read the same rows, so the
 * workgroup that owns a block of query rows also copies the K/V rows of those positions into the
 * caches: one launch, and where the MFMA attention kernel runs (bf16, head_dim <= 128) no second
 * pass over K and V from memory.  Results are those of the two separate calls, bit for bit.
 * Arguments, layouts and error behaviour are theirs; k_cache and v_cache must not be null. */
int civic_prefill_attn_kv(const void* q, const void* k, const void* v, void* out,
                          void* k_cache, void* v_cache, int dtype,
                          int32_t batch, int32_t seq, int32_t n_q_heads, int32_t n_kv_heads,
                          int32_t head_dim, const int64_t* q_strides /* host [3] */,
                          const int64_t* kv_strides /* host [3] */,
                          const int64_t* o_strides /* host [3] */,
                          int64_t s_max, int64_t pos0, int32_t causal, float softmax_scale,
                          void* stream);

/* civic_prefill_attn (and civic_prefill_attn_kv when the caches are given) for packed samples of different lengths:
 * sample b owns rows [row_offsets[b], row_offsets[b+1]) of q, k, v and out (civic_ragged_offsets' compact offsets);
 * it attends to its own keys only, the causal mask counts from its first row, and its K and V rows go to rows
 * [pos0, pos0 + its length) of k_cache[b], v_cache[b].  ONE launch per group of up to 64 samples (the workgroups
 * look their sample's rows up in a table passed with the launch); fp32 or head_dim > 128: one launch per sample.
 * Results equal the rectangular calls on each sample alone, bit for bit.
 *   q, out       device [total_rows, n_q_heads, head_dim], element strides (unused, token, head)
 *   k, v         device [total_rows, n_kv_heads, head_dim], element strides (unused, token, head)
 *   row_offsets  host [batch + 1] int64, row_offsets[0] = 0, strictly increasing; row_offsets[batch] <= INT32_MAX
 *   k_cache, v_cache  device [batch, n_kv_heads, s_max, head_dim] dense, or both NULL; pos0 + longest sample <= s_max
 * Everything else as civic_prefill_attn; every group is checked before the first launch. */
int civic_prefill_attn_ragged(const void* q, const void* k, const void* v, void* out, int dtype, int32_t batch,
                              const int64_t* row_offsets /* host */, int32_t n_q_heads, int32_t n_kv_heads,
                              int32_t head_dim, const int64_t* q_strides /* host [3] */,
                              const int64_t* kv_strides /* host [3] */, const int64_t* o_strides /* host [3] */,
                              int32_t causal, float softmax_scale, void* k_cache, void* v_cache, int64_t s_max,
                              int64_t pos0, void* stream);

/* Rotary position embedding from the carried position ids.  The compact merge copies the three ids of every
 * token unchanged ("text positions are preserved, compact visual positions are inherited", sentence after
 * Eq. 14); this is where they are consumed.  The paper prints no rotary formula: the form is the published
 * three-axis rotary embedding of the Qwen-VL family in rotate-half layout.  Frequency pair i of a head row is
 * (x[i], x[i + head_dim/2]); it is turned by angle(t, i) = pos_ids[axis_of_pair[i], b, t] * inv_freq[i]:
 *   y[i] = x[i] cos - x[i + head_dim/2] sin,   y[i + head_dim/2] = x[i + head_dim/2] cos + x[i] sin.
 * Which id axis (0 temporal, 1 height, 2 width) and which frequency a pair uses are the caller's tables, so
 * sectioned and interleaved splits and any base are covered.
 *
 * civic_mrope_table: (cos, sin) of every angle, once per prefill (all layers and heads share them).
 *   pos_ids       device [3, batch, seq] int32 (civic_compact's pos_c)
 *   axis_of_pair  host [n_pairs] int32 in {0, 1, 2};  inv_freq  host [n_pairs] fp32, finite
 *   cos_sin       device [batch, seq, n_pairs, 2] fp32, 16-byte aligned
 * Angles are formed and reduced in double precision.  n_pairs <= CIVIC_MAX_HEAD_DIM / 2. */
int civic_mrope_table(const int32_t* pos_ids, int32_t batch, int64_t seq, int32_t n_pairs,
                      const int32_t* axis_of_pair /* host */, const float* inv_freq /* host */,
                      float* cos_sin, void* stream);

/* Rotates every head row of x into out (out may be x): fp32 arithmetic, output rounded to `dtype`.
 *   x, out   device [batch, seq, heads, head_dim], element strides (batch, token, head) in x_strides /
 *            out_strides (host int64[3]), head_dim contiguous
 *   cos_sin  device [batch, seq, head_dim/2, 2] fp32 (civic_mrope_table with n_pairs = head_dim/2)
 * head_dim/2 * sizeof(element) must be a multiple of 16; pointers and strides*sizeof(element) 16-byte aligned. */
int civic_mrope_apply(const void* x, void* out, int dtype, int32_t batch, int64_t seq, int32_t heads, int32_t head_dim,
                      const int64_t* x_strides /* host [3] */, const int64_t* out_strides /* host [3] */,
                      const float* cos_sin, void* stream);

/* civic_kv_write with K rotated on its way into the cache (V is copied as it is): the keys enter the cache
 * with their positions applied once, which is what civic_decode_attn and civic_prefill_attn_rope expect to
 * find there.  Arguments as civic_kv_write plus cos_sin [batch, seq, head_dim/2, 2] for the seq tokens written;
 * head_dim/2 * sizeof(element) a multiple of 16. */
int civic_kv_write_rope(const void* k, const void* v, const int64_t* kv_strides /* host [3] */, int dtype,
                        const float* cos_sin, void* k_cache, void* v_cache, int32_t batch, int32_t seq,
                        int32_t n_kv_heads, int32_t head_dim, int64_t s_max, int64_t pos0, void* stream);

/* civic_prefill_attn with the rotary embedding of Q applied on the fly (in registers, from q_cos_sin
 * [batch, seq, head_dim/2, 2]); k is taken as given, i.e. already rotated - typically the cache rows
 * civic_kv_write_rope has just written, addressed through kv_strides (batch: n_kv_heads*s_max*head_dim,
 * token: head_dim, head: s_max*head_dim).  No separate pass over Q is made.  Everything else as
 * civic_prefill_attn; the rotated query is rounded to `dtype` before the products, as a separate
 * civic_mrope_apply would.  head_dim a multiple of 4; the MFMA kernel serves head_dim 64, 96 and 128. */
int civic_prefill_attn_rope(const void* q, const void* k, const void* v, void* out, int dtype,
                            int32_t batch, int32_t seq, int32_t n_q_heads, int32_t n_kv_heads,
                            int32_t head_dim, const int64_t* q_strides /* host [3] */,
                            const int64_t* kv_strides /* host [3] */, const int64_t* o_strides /* host [3] */,
                            int32_t causal, float softmax_scale, const float* q_cos_sin, void* stream);

/* Soft anchor aggregation, Eq. 8 in full - the paper's own, learned route from T_e dense patch embeddings to M_e
 * compact tokens, before the visual encoder:
 *   K_0 = Norm(LN(X_0)),  Q_A = Norm(LN(A)),  W_A = softmax(Q_A K_0^T / tau) over the dense tokens,  Z_0 = W_A X_0.
 * LN without affine (its epsilon cancels under Norm); a row without variance normalises to zero.  K_0, Q_A and
 * W_A are rounded to bf16 for the two contractions (bf16 MFMA, fp32 accumulation); the softmax is fp32.
 *   x0            device [batch, n_tokens, dim] bf16, dense
 *   anchors       device [n_anchors, dim] bf16: A itself, not normalised (shared by the batch)
 *   z0            device [batch, n_anchors, dim] bf16
 *   token_weight  device [batch, n_tokens] fp32 or NULL: sum over the anchors of W_A[a, i], the weight each dense
 *                 token receives (a multi-anchor importance score that civic_select accepts)
 *   workspace     device, 16-byte aligned, civic_anchor_aggregate_workspace_bytes(same sizes) bytes: normalised
 *                 rows, logits, weights, X_0 transposed; no initialisation needed
 * dtype must be CIVIC_BF16 and dim a multiple of 64 (else CIVIC_ERR_UNSUPPORTED); inv_tau >= 0, finite. */
size_t civic_anchor_aggregate_workspace_bytes(int32_t batch, int32_t n_tokens, int32_t n_anchors, int32_t dim);
int civic_anchor_aggregate(const void* x0, const void* anchors, int dtype, int32_t batch, int32_t n_tokens,
                           int32_t n_anchors, int32_t dim, float inv_tau, void* z0, float* token_weight,
                           void* workspace, size_t workspace_bytes, void* stream);

/* KV compression of the compact visual encoder, Eq. 9: K_c = Rbar^T K and V_c = Rbar^T V, where R [n_rows, n_mem]
 * assigns the n_rows compact tokens to n_mem memory anchors and Rbar is R "column-normalised", read here as every
 * column divided by its sum (each compressed key is a weighted mean of keys; a column that sums to zero gives a
 * zero row).  The paper does not say how R is produced; it is an input.
 *   k, v      device [batch, n_rows, width] bf16, dense (width = heads * head_dim)
 *   r         device [n_rows, n_mem] fp32, shared by the batch
 *   k_c, v_c  device [batch, n_mem, width] bf16
 *   workspace device, 16-byte aligned, civic_kv_compress_workspace_bytes(same sizes) bytes
 * Rbar is rounded to bf16 for the contraction (bf16 MFMA, fp32 accumulation).  dtype must be CIVIC_BF16. */
size_t civic_kv_compress_workspace_bytes(int32_t batch, int32_t n_rows, int32_t n_mem, int32_t width);
int civic_kv_compress(const void* k, const void* v, int dtype, const float* r, int32_t batch, int32_t n_rows,
                      int32_t n_mem, int32_t width, void* k_c, void* v_c, void* workspace, size_t workspace_bytes,
                      void* stream);

/* Attention of n_q queries over n_kv keys without a mask, out = softmax(Q K^T * scale) V: with the compressed
 * K_c, V_c of civic_kv_compress this is the compact visual attention of Eq. 9 (score size M_e x S instead of
 * M_e x M_e).  Same kernels, layouts, strides and limits as civic_prefill_attn; k and v hold n_kv tokens. */
int civic_cross_attn(const void* q, const void* k, const void* v, void* out, int dtype, int32_t batch, int32_t n_q,
                     int32_t n_kv, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                     const int64_t* q_strides /* host [3] */, const int64_t* kv_strides /* host [3] */,
                     const int64_t* o_strides /* host [3] */, float softmax_scale, void* stream);

/* Eq. 9 for a batch whose items differ in size (images of different grids in one batch): the rows of all items are
 * packed back to back, item b owning rows [row_offsets[b], row_offsets[b+1]) of k, v and of its own assignment rows in
 * r; every item is compressed and attended by itself, and the results equal civic_kv_compress / civic_cross_attn on
 * that item alone, bit for bit.  Items travel in groups of up to 64 whose row numbers are passed with the launch: the
 * compression is three launches per group (partial column sums, Rbar^T of every item, one grouped GEMM for K_c and
 * V_c of all items), the attention ONE launch per group (fp32 or head_dim > 128: one launch per item).
 *   k, v         device [total_rows, width] bf16;  r  device [total_rows, n_mem] fp32
 *   row_offsets  host [batch + 1] int64, row_offsets[0] = 0, strictly increasing (no empty item)
 *   k_c, v_c     device [batch, n_mem, width] bf16
 *   workspace    civic_kv_compress_ragged_workspace_bytes(same sizes): every item's column sums and padded Rbar^T
 *   row_offsets[batch] <= INT32_MAX, else CIVIC_ERR_UNSUPPORTED
 * width must be a multiple of 8 and n_mem of 4 (every item's first row 16-byte aligned), else CIVIC_ERR_UNSUPPORTED. */
size_t civic_kv_compress_ragged_workspace_bytes(int32_t batch, const int64_t* row_offsets /* host */, int32_t n_mem,
                                                int32_t width);
int civic_kv_compress_ragged(const void* k, const void* v, int dtype, const float* r, int32_t batch,
                             const int64_t* row_offsets /* host */, int32_t n_mem, int32_t width, void* k_c, void* v_c,
                             void* workspace, size_t workspace_bytes, void* stream);
/*   q, out       device [total_rows, n_q_heads, head_dim], element strides (unused, token, head) in q_strides / o_strides
 *   k, v         device [batch, n_kv, n_kv_heads, head_dim] (civic_kv_compress_ragged's outputs), strides in kv_strides
 *   q_offsets    as row_offsets above; q_offsets[batch] <= INT32_MAX, else CIVIC_ERR_UNSUPPORTED
 * Everything else as civic_cross_attn; every group of items is checked before the first launch. */
int civic_cross_attn_ragged(const void* q, const void* k, const void* v, void* out, int dtype, int32_t batch,
                            const int64_t* q_offsets /* host */, int32_t n_kv, int32_t n_q_heads, int32_t n_kv_heads,
                            int32_t head_dim, const int64_t* q_strides /* host [3] */,
                            const int64_t* kv_strides /* host [3] */, const int64_t* o_strides /* host [3] */,
                            float softmax_scale, void* stream);

/* Decode-step attention over the compact cache: the work one generated token adds to the autoregressive
 * decoding cost C_dec of Eq. 2 / Eq. 7, in which "every generated text token must attend to the entire visual
 * prompt" (latency decomposition, decode column of the latency table) - here to the compact one that
 * civic_kv_write left in the contiguous caches.
 *   out[b, h, :] = sum_{j < n_ctx} softmax_j(scale * <q[b,h,:], k_cache[b,g,j,:]>) v_cache[b,g,j,:],
 * g = h / (n_q_heads / n_kv_heads).  Rows at or beyond n_ctx are not read.  fp32 logits and accumulation
 * (exp2 of logits scaled by log2 e); the output is rounded to `dtype` (nearest even for bf16).
 *   q, out            device [batch, n_q_heads, head_dim] of `dtype`, dense
 *   k_cache, v_cache  device [batch, n_kv_heads, s_max, head_dim] of `dtype`, dense
 *   n_ctx             rows of every cache that hold the context, 1..s_max (the same for every batch item:
 *                     compact sequences of one grid have one length)
 *   softmax_scale     0 means 1/sqrt(head_dim)
 *   workspace         device, 16-byte aligned, at least civic_decode_attn_workspace_bytes(same sizes) bytes:
 *                     partial (max, sum, output) per split of the context; may be NULL when that is 0.
 *                     Contents need no initialisation and mean nothing afterwards.
 * Pointers 16-byte aligned; head_dim * sizeof(element) a multiple of 16 and at most 1024 bytes; batch at most
 * 65535.  CIVIC_ERR_WORKSPACE if the workspace is missing or too small. */
size_t civic_decode_attn_workspace_bytes(int dtype, int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                                         int32_t head_dim, int64_t n_ctx);
int civic_decode_attn(const void* q, const void* k_cache, const void* v_cache, void* out, int dtype,
                      int32_t batch, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, int64_t s_max,
                      int64_t n_ctx, float softmax_scale, void* workspace, size_t workspace_bytes, void* stream);

/* civic_decode_attn for callers that cannot allocate or hand over a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the workspace, same kernels,
 * same results bit for bit; the partial results of the splits live in an array inside the library's code
 * object, of CIVIC_DECODE_NOALLOC_MAX_BYTES on every GPU that runs the library, held until the process ends.
 * The call allocates and frees nothing (device or pinned memory) and needs no initialisation call.
 * CIVIC_ERR_WORKSPACE when civic_decode_attn_workspace_bytes(same sizes) exceeds that maximum.
 * All calls on one GPU share the array: calls that may overlap on one GPU (different streams, different
 * threads) race on it and must be serialised by the caller; civic_decode_attn with separate workspaces has no
 * such limit. */
#define CIVIC_DECODE_NOALLOC_MAX_BYTES (4u << 20)
int civic_decode_attn_noalloc(const void* q, const void* k_cache, const void* v_cache, void* out, int dtype,
                              int32_t batch, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, int64_t s_max,
                              int64_t n_ctx, float softmax_scale, void* stream);

/* civic_decode_attn over caches that hold a different number of rows per sample (what civic_prefill_attn_ragged
 * leaves): sample b attends to rows [0, n_ctx[b]) of k_cache[b], v_cache[b].  Groups of up to 256 samples, each the two
 * launches of civic_decode_attn laid out for the group's longest context (a split that starts past a sample's rows
 * contributes nothing); results equal civic_decode_attn on every sample alone up to the order of the partial sums.
 *   n_ctx      host [batch] int32, every entry in [1, s_max]
 *   workspace  civic_decode_attn_ragged_workspace_bytes(same sizes), 16-byte aligned (shared by the groups in turn)
 * Everything else as civic_decode_attn; every group is checked before the first launch. */
size_t civic_decode_attn_ragged_workspace_bytes(int dtype, int32_t batch, const int32_t* n_ctx /* host */, int32_t n_q_heads,
                                                int32_t n_kv_heads, int32_t head_dim);
int civic_decode_attn_ragged(const void* q, const void* k_cache, const void* v_cache, void* out, int dtype, int32_t batch,
                             const int32_t* n_ctx /* host */, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                             int64_t s_max, float softmax_scale, void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CIVIC_H */

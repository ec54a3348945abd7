/*
 * CPU oracle for the compact-prefill path of CIVIC (path-consistent compact inference).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, obviously-correct C in double precision.  It
 * shares no code, header, table or helper with the HIP library and must never be linked
 * or called from the product path; only the tests, the smoke check and the benchmark's
 * cpu_baseline leg use it.
 *
 * What is written out here, and where the paper fixes it:
 *   oracle_anchor_normalize  Q_A = Norm(LN(A))                     (Eq. 8, one anchor row)
 *   oracle_score             s_i = <Q_A, Norm(LN(x_i))> / tau      (Eq. 8, the pre-softmax
 *                            logit; the paper defines no other per-token quantity)
 *   oracle_select            exact constrained top-k: per-cell floor, per-frame floor,
 *                            global budget ("token budget" C and "minimum keep ratio" of
 *                            the Ablation Study; "adaptive spatial retention floor" of the
 *                            Abstract).  The paper names these and gives no formula:
 *                            PARITY UNPINNED BY THE PAPER for the floor semantics and for
 *                            the scoring rule; they are pinned by brute force, a second
 *                            algorithm and closed forms in the CPU tests instead.
 *   oracle_compact           x~_c = Merge(E_x, V_c), |x~_c| = L + M_p (Eq. 13), positions
 *                            preserved / inherited (sentence after Eq. 14)
 *   oracle_attention         softmax(Q K^T / sqrt(d)) V per head, grouped-query, optional
 *                            causal mask: the "LLM prefill attention" term of Eq. 2 / Eq. 7
 *   oracle_kv_write          the "KV-cache storage" term of Eq. 2 / Eq. 7: contiguous rows
 *   oracle_mrope_table /     rotary position embedding driven by the position ids that the compact
 *   oracle_mrope_apply       merge carries along ("text positions are preserved, compact visual
 *                            positions are inherited", sentence after Eq. 14).  The paper does not
 *                            print the rotary form: three-axis rotary embedding as published for
 *                            the Qwen-VL family, pairs (i, i + d/2), axis and frequency per pair
 *                            given by the caller: PARITY UNPINNED BY THE PAPER, pinned by the
 *                            complex-multiplication form and the relative-position property.
 *   oracle_anchor_aggregate  Z_0 = softmax(Q_A K_0^T / tau) X_0, K_0 = Norm(LN(X_0)), Q_A = Norm(LN(A)),
 *                            softmax over the dense tokens (Eq. 8 in full)
 *   oracle_kv_compress       K_c = Rbar^T K, V_c = Rbar^T V with the column-normalised assignment
 *                            matrix (Eq. 9); "column-normalised" is read as every column divided by
 *                            its sum (the rows of K_c are weighted means): PARITY UNPINNED BY THE PAPER
 *   oracle_cross_attention   softmax(Q K_c^T / sqrt(d)) V_c, queries and keys of different counts (Eq. 9)
 *   oracle_decode_attention  one generated token attending to the whole compact prompt in
 *                            the cache: the per-token work inside the autoregressive decoding
 *                            cost C_dec of Eq. 2 / Eq. 7 (decode column of the latency table)
 *
 * OpenMP is used on the outermost independent loop only (rows, batch items, query rows);
 * every inner computation is a sequential loop in the order the definition states.
 */
#define _GNU_SOURCE
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t frames, height, width;   /* N_v = frames * height * width, frame-major raster  */
    int32_t cell_h, cell_w;          /* spatial cell; edge cells may be smaller            */
    int32_t cell_floor;              /* kept at least this many per cell (clipped to size) */
    int32_t frame_floor;             /* per-frame floor, see `nested` in oracle_select     */
    int32_t budget;                  /* global keep budget C over the sample's N_v tokens  */
} oracle_grid;

int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ Eq. 8: anchor side */
/* q = Norm(LN(a)) with LN(a) = (a - mean) / sqrt(var + eps) (no affine) and Norm the l2
 * normalisation.  Returns 0, or -1 if LN(a) is the zero vector. */
int oracle_anchor_normalize(const float *a, int32_t dim, double eps, double *q)
{
    double mean = 0.0, var = 0.0, nrm = 0.0;
    for (int32_t j = 0; j < dim; ++j) mean += (double)a[j];
    mean /= dim;
    for (int32_t j = 0; j < dim; ++j) { double c = (double)a[j] - mean; var += c * c; }
    var /= dim;
    for (int32_t j = 0; j < dim; ++j) {
        q[j] = ((double)a[j] - mean) / sqrt(var + eps);
        nrm += q[j] * q[j];
    }
    nrm = sqrt(nrm);
    if (!(nrm > 0.0)) return -1;
    for (int32_t j = 0; j < dim; ++j) q[j] /= nrm;
    return 0;
}

/* ------------------------------------------------------------------ Eq. 8: token side  */
/* scores[i] = inv_tau * <q, Norm(LN(x_i))>.  LN's eps and gain cancel under Norm, so
 * Norm(LN(x)) = (x - mean(x)) / ||x - mean(x)||; a constant row scores 0. */
void oracle_score(const float *x, int64_t n_rows, int64_t row_stride, int32_t dim,
                  const float *q, double inv_tau, float *scores)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_rows; ++i) {
        const float *row = x + i * row_stride;
        double mean = 0.0, n2 = 0.0, dot = 0.0;
        for (int32_t j = 0; j < dim; ++j) mean += (double)row[j];
        mean /= dim;
        for (int32_t j = 0; j < dim; ++j) {
            double c = (double)row[j] - mean;
            n2 += c * c;
            dot += (double)q[j] * c;
        }
        double n = sqrt(n2);
        scores[i] = (n > 0.0) ? (float)(inv_tau * dot / n) : 0.0f;
    }
}

/* ----------------------------------------------------------------------------- select  */
/* Strict total order on token indices: higher score first, ties to the lower index.  IEEE
 * comparison, so -0 and +0 tie. */
static int precedes_cmp(const void *pa, const void *pb, void *ctx)
{
    const float *s = (const float *)ctx;
    int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    if (s[a] > s[b]) return -1;
    if (s[a] < s[b]) return 1;
    return (a < b) ? -1 : (a > b) ? 1 : 0;
}

static int grid_ok(const oracle_grid *g)
{
    if (!g) return 0;
    if (g->frames <= 0 || g->height <= 0 || g->width <= 0) return 0;
    if (g->cell_h <= 0 || g->cell_w <= 0) return 0;
    if (g->cell_floor < 0 || g->frame_floor < 0 || g->budget < 0) return 0;
    int64_t nv = (int64_t)g->frames * g->height * g->width;
    if (nv > INT32_MAX || g->budget > nv) return 0;
    return 1;
}

/* Marks the kept tokens of ONE sample.  keep[v] in {0,1} for visual-local index
 * v = f*H*W + r*W + c.  Returns the number kept, -1 on a bad grid, -2 if a score is NaN.
 *   (1) every cell keeps its first min(cell_floor, size) tokens in the order above;
 *   (2) every frame then keeps, among its not-yet-kept tokens, the first frame_floor
 *       (additive reading, nested == 0) or just enough to reach frame_floor kept in the
 *       frame (nested reading, nested != 0);
 *   (3) the first max(0, budget - #kept) not-yet-kept tokens of the sample are kept. */
int64_t oracle_select(const float *scores, const oracle_grid *g, int nested, uint8_t *keep)
{
    if (!grid_ok(g)) return -1;
    const int32_t H = g->height, W = g->width, HW = H * W;
    const int32_t nv = g->frames * HW;
    for (int32_t v = 0; v < nv; ++v) if (isnan(scores[v])) return -2;
    int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)nv);
    if (!idx) return -1;
    memset(keep, 0, (size_t)nv);

    for (int32_t f = 0; f < g->frames; ++f)                       /* (1) cell floors */
        for (int32_t r0 = 0; r0 < H; r0 += g->cell_h)
            for (int32_t c0 = 0; c0 < W; c0 += g->cell_w) {
                int32_t n = 0;
                for (int32_t r = r0; r < r0 + g->cell_h && r < H; ++r)
                    for (int32_t c = c0; c < c0 + g->cell_w && c < W; ++c)
                        idx[n++] = f * HW + r * W + c;
                qsort_r(idx, (size_t)n, sizeof(int32_t), precedes_cmp, (void *)scores);
                for (int32_t k = 0; k < n && k < g->cell_floor; ++k) keep[idx[k]] = 1;
            }

    for (int32_t f = 0; f < g->frames; ++f) {                     /* (2) frame floors */
        int32_t n = 0, already = 0;
        for (int32_t v = f * HW; v < (f + 1) * HW; ++v) {
            if (keep[v]) ++already; else idx[n++] = v;
        }
        int32_t want = nested ? (g->frame_floor - already) : g->frame_floor;
        qsort_r(idx, (size_t)n, sizeof(int32_t), precedes_cmp, (void *)scores);
        for (int32_t k = 0; k < n && k < want; ++k) keep[idx[k]] = 1;
    }

    int64_t kept = 0;                                             /* (3) global budget */
    int32_t n = 0;
    for (int32_t v = 0; v < nv; ++v) { if (keep[v]) ++kept; else idx[n++] = v; }
    int64_t fill = (int64_t)g->budget - kept;
    qsort_r(idx, (size_t)n, sizeof(int32_t), precedes_cmp, (void *)scores);
    for (int32_t k = 0; k < n && k < fill; ++k) { keep[idx[k]] = 1; ++kept; }

    free(idx);
    return kept;
}

/* Batch of samples sharing one grid.  kept_idx[b, 0..K) receives the kept visual-local
 * indices in ascending order, K = the count every sample returns (data independent).
 * Returns K, or a negative code. */
int64_t oracle_select_batch(const float *scores, int32_t batch, const oracle_grid *g,
                            int nested, int32_t *kept_idx, int64_t kept_capacity,
                            uint8_t *keep_flags)
{
    if (!grid_ok(g)) return -1;
    const int64_t nv = (int64_t)g->frames * g->height * g->width;
    int64_t *per_item = (int64_t *)malloc(sizeof(int64_t) * (size_t)(batch > 0 ? batch : 1));
    if (!per_item) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t b = 0; b < batch; ++b) {
        uint8_t *keep = keep_flags + (int64_t)b * nv;
        int64_t k = oracle_select(scores + (int64_t)b * nv, g, nested, keep);
        if (k > kept_capacity) k = -3;
        int64_t w = 0;
        if (k >= 0)
            for (int64_t v = 0; v < nv; ++v)
                if (keep[v]) kept_idx[(int64_t)b * kept_capacity + w++] = (int32_t)v;
        per_item[b] = k;
    }
    int64_t result = (batch > 0) ? per_item[0] : 0;
    for (int32_t b = 0; b < batch; ++b) {
        if (per_item[b] < 0) { result = per_item[b]; break; }
        if (per_item[b] != result) { result = -4; break; }
    }
    free(per_item);
    return result;
}

/* The keep count is a function of the grid alone: run the selection on all-equal scores. */
int64_t oracle_kept_count(const oracle_grid *g, int nested)
{
    if (!grid_ok(g)) return -1;
    const size_t nv = (size_t)g->frames * g->height * g->width;
    float *zeros = (float *)calloc(nv, sizeof(float));
    uint8_t *keep = (uint8_t *)malloc(nv);
    int64_t k = (zeros && keep) ? oracle_select(zeros, g, nested, keep) : -1;
    free(zeros);
    free(keep);
    return k;
}

/* --------------------------------------------------------------- Eq. 13: compact merge */
/* Walks the dense sequence t = 0..S-1 of every batch item.  A token is visual if it lies
 * in a frame span [frame_start[f], frame_start[f] + H*W); its visual-local index is
 * f*H*W + (t - frame_start[f]).  Text tokens and kept visual tokens are appended, in
 * order, to the compact sequence: the source index, the hidden row (raw bytes) and the
 * three position ids are copied unchanged.  Returns the compact length, or -1 if the
 * items disagree or exceed seq_c_capacity. */
int64_t oracle_compact(const uint8_t *hidden, int64_t row_bytes,
                       const int32_t *pos_ids /* [3, batch, S] */,
                       int32_t batch, int64_t seq_len, const oracle_grid *g,
                       const int64_t *frame_start, const int32_t *kept_idx, int64_t n_kept,
                       int64_t seq_c_capacity,
                       uint8_t *hidden_c /* [batch, cap, row_bytes] */,
                       int32_t *pos_c /* [3, batch, cap] */, int32_t *src_idx /* [batch, cap] */)
{
    if (!grid_ok(g)) return -1;
    const int64_t HW = (int64_t)g->height * g->width, nv = HW * g->frames;
    uint8_t *is_kept = (uint8_t *)malloc((size_t)nv);
    if (!is_kept) return -1;
    int64_t len0 = -1;
    for (int32_t b = 0; b < batch; ++b) {
        memset(is_kept, 0, (size_t)nv);
        for (int64_t k = 0; k < n_kept; ++k) {
            int32_t v = kept_idx[(int64_t)b * n_kept + k];
            if (v < 0 || v >= nv) { free(is_kept); return -1; }
            is_kept[v] = 1;
        }
        int64_t out = 0;
        for (int64_t t = 0; t < seq_len; ++t) {
            int keep_it = 1;
            for (int32_t f = 0; f < g->frames; ++f)
                if (t >= frame_start[f] && t < frame_start[f] + HW)
                    keep_it = is_kept[f * HW + (t - frame_start[f])];
            if (!keep_it) continue;
            if (out >= seq_c_capacity) { free(is_kept); return -1; }
            src_idx[(int64_t)b * seq_c_capacity + out] = (int32_t)t;
            memcpy(hidden_c + ((int64_t)b * seq_c_capacity + out) * row_bytes,
                   hidden + ((int64_t)b * seq_len + t) * row_bytes, (size_t)row_bytes);
            for (int a = 0; a < 3; ++a)
                pos_c[((int64_t)a * batch + b) * seq_c_capacity + out] =
                    pos_ids[((int64_t)a * batch + b) * seq_len + t];
            ++out;
        }
        if (b == 0) len0 = out;
        else if (out != len0) { free(is_kept); return -1; }
    }
    free(is_kept);
    return len0;
}

/* ------------------------------------------------- Eq. 2 / Eq. 7: prefill attention    */
/* out[b, i, h, :] = sum_j softmax_j(scale * <Q[b,i,h], K[b,j,g]>) V[b,j,g], g = h / (H_q /
 * H_kv), j <= i when causal (compact index order), all j otherwise.  Strides are in
 * elements for (batch, token, head); head_dim is contiguous.  Output is double, dense
 * [batch, seq, H_q, head_dim].  Rows with row_step > 1 are sampled: only i % row_step == 0
 * are computed (others left untouched), which lets large cases be spot-checked. */
void oracle_attention(const float *q, const float *k, const float *v, double *out,
                      int32_t batch, int32_t seq, int32_t n_q_heads, int32_t n_kv_heads,
                      int32_t head_dim, const int64_t *q_strides, const int64_t *kv_strides,
                      int causal, double scale, int32_t row_step)
{
    const int32_t group = n_q_heads / n_kv_heads;
    if (row_step < 1) row_step = 1;
    const int64_t total = (int64_t)batch * n_q_heads * seq;
#pragma omp parallel
    {
        double *z = (double *)malloc(sizeof(double) * (size_t)seq);
#pragma omp for schedule(dynamic, 16)
        for (int64_t w = 0; w < total; ++w) {
            const int32_t i = (int32_t)(w % seq);
            const int32_t h = (int32_t)((w / seq) % n_q_heads);
            const int32_t b = (int32_t)(w / ((int64_t)seq * n_q_heads));
            if (i % row_step) continue;
            const int32_t gk = h / group;
            const float *qi = q + b * q_strides[0] + i * q_strides[1] + h * q_strides[2];
            const int32_t last = causal ? i : seq - 1;
            double zmax = -INFINITY;
            for (int32_t j = 0; j <= last; ++j) {
                const float *kj = k + b * kv_strides[0] + j * kv_strides[1] + gk * kv_strides[2];
                double acc = 0.0;
                for (int32_t c = 0; c < head_dim; ++c) acc += (double)qi[c] * (double)kj[c];
                z[j] = scale * acc;
                if (z[j] > zmax) zmax = z[j];
            }
            double denom = 0.0;
            for (int32_t j = 0; j <= last; ++j) { z[j] = exp(z[j] - zmax); denom += z[j]; }
            double *o = out + (((int64_t)b * seq + i) * n_q_heads + h) * head_dim;
            for (int32_t c = 0; c < head_dim; ++c) o[c] = 0.0;
            for (int32_t j = 0; j <= last; ++j) {
                const float *vj = v + b * kv_strides[0] + j * kv_strides[1] + gk * kv_strides[2];
                const double p = z[j] / denom;
                for (int32_t c = 0; c < head_dim; ++c) o[c] += p * (double)vj[c];
            }
        }
        free(z);
    }
}

/* ------------------------------------------------------ Eq. 2 / Eq. 7: KV-cache rows   */
/* cache[b, g, pos0 + i, :] = src[b, i, g, :] (raw bytes) for K and for V; every other byte
 * of the caches is left as it was.  Cache layout [batch, H_kv, s_max, head_dim] dense.
 * Returns the number of bytes written into the two caches together. */
int64_t oracle_kv_write(const uint8_t *k, const uint8_t *v, const int64_t *kv_strides_bytes,
                        uint8_t *k_cache, uint8_t *v_cache, int32_t batch, int32_t seq,
                        int32_t n_kv_heads, int64_t head_bytes, int64_t s_max, int64_t pos0)
{
    int64_t written = 0;
#pragma omp parallel for schedule(static) reduction(+ : written)
    for (int32_t b = 0; b < batch; ++b)
        for (int32_t i = 0; i < seq; ++i)
            for (int32_t g = 0; g < n_kv_heads; ++g) {
                const int64_t src = b * kv_strides_bytes[0] + i * kv_strides_bytes[1] +
                                    g * kv_strides_bytes[2];
                const int64_t dst = (((int64_t)b * n_kv_heads + g) * s_max + pos0 + i) * head_bytes;
                memcpy(k_cache + dst, k + src, (size_t)head_bytes);
                memcpy(v_cache + dst, v + src, (size_t)head_bytes);
                written += 2 * head_bytes;
            }
    return written;
}

/* ---------------------------------------------- Eq. 2 / Eq. 7: decode-step attention   */
/* One query per (batch item, query head) against the first n_ctx rows of the contiguous
 * caches [batch, H_kv, s_max, head_dim] (the layout oracle_kv_write fills):
 *   out[b, h, :] = sum_{j < n_ctx} softmax_j(scale * <q[b,h,:], K[b,g,j,:]>) V[b,g,j,:],
 * g = h / (H_q / H_kv).  Rows at or beyond n_ctx are never read.  q is dense
 * [batch, H_q, head_dim]; output double, same shape.  n_ctx >= 1. */
void oracle_decode_attention(const float *q, const float *k_cache, const float *v_cache,
                             double *out, int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                             int32_t head_dim, int64_t s_max, int64_t n_ctx, double scale)
{
    const int32_t group = n_q_heads / n_kv_heads;
#pragma omp parallel for schedule(static)
    for (int64_t w = 0; w < (int64_t)batch * n_q_heads; ++w) {
        const int32_t b = (int32_t)(w / n_q_heads), h = (int32_t)(w % n_q_heads);
        const int32_t g = h / group;
        const float *qv = q + w * head_dim;
        const float *kb = k_cache + ((int64_t)b * n_kv_heads + g) * s_max * head_dim;
        const float *vb = v_cache + ((int64_t)b * n_kv_heads + g) * s_max * head_dim;
        double *z = (double *)malloc(sizeof(double) * (size_t)n_ctx);
        double zmax = -INFINITY, denom = 0.0;
        for (int64_t j = 0; j < n_ctx; ++j) {
            double acc = 0.0;
            for (int32_t c = 0; c < head_dim; ++c) acc += (double)qv[c] * (double)kb[j * head_dim + c];
            z[j] = scale * acc;
            if (z[j] > zmax) zmax = z[j];
        }
        for (int64_t j = 0; j < n_ctx; ++j) { z[j] = exp(z[j] - zmax); denom += z[j]; }
        double *o = out + w * head_dim;
        for (int32_t c = 0; c < head_dim; ++c) o[c] = 0.0;
        for (int64_t j = 0; j < n_ctx; ++j) {
            const double p = z[j] / denom;
            for (int32_t c = 0; c < head_dim; ++c) o[c] += p * (double)vb[j * head_dim + c];
        }
        free(z);
    }
}

/* ------------------------------------------- position ids -> rotary angles (M-RoPE)    */
/* cos_sin[b, t, i, 0..1] = (cos, sin) of angle = pos_ids[axis_of_pair[i], b, t] * inv_freq[i]
 * for every frequency pair i < n_pairs; pos_ids is int32 [3, batch, seq] (temporal, height,
 * width), axis_of_pair[i] in {0, 1, 2}.  inv_freq is taken as the fp32 values given. */
void oracle_mrope_table(const int32_t *pos_ids, int32_t batch, int64_t seq, int32_t n_pairs,
                        const int32_t *axis_of_pair, const float *inv_freq, double *cos_sin)
{
#pragma omp parallel for schedule(static)
    for (int64_t w = 0; w < (int64_t)batch * seq; ++w) {
        const int32_t b = (int32_t)(w / seq);
        const int64_t t = w % seq;
        for (int32_t i = 0; i < n_pairs; ++i) {
            const double p = (double)pos_ids[((int64_t)axis_of_pair[i] * batch + b) * seq + t];
            const double angle = p * (double)inv_freq[i];
            cos_sin[(w * n_pairs + i) * 2] = cos(angle);
            cos_sin[(w * n_pairs + i) * 2 + 1] = sin(angle);
        }
    }
}

/* Rotates every head row of x [batch, seq, heads, head_dim] (element strides for batch, token,
 * head; head_dim contiguous, head_dim = 2 * n_pairs): pair i is (x[i], x[i + n_pairs]),
 *   out[i]           = x[i] * cos - x[i + n_pairs] * sin
 *   out[i + n_pairs] = x[i + n_pairs] * cos + x[i] * sin
 * with the (cos, sin) of the row's token.  Output double, dense [batch, seq, heads, head_dim]. */
void oracle_mrope_apply(const float *x, const int64_t *x_strides, int32_t batch, int64_t seq,
                        int32_t heads, int32_t n_pairs, const double *cos_sin, double *out)
{
    const int32_t d = 2 * n_pairs;
#pragma omp parallel for schedule(static)
    for (int64_t w = 0; w < (int64_t)batch * seq; ++w) {
        const int32_t b = (int32_t)(w / seq);
        const int64_t t = w % seq;
        for (int32_t h = 0; h < heads; ++h) {
            const float *row = x + b * x_strides[0] + t * x_strides[1] + h * x_strides[2];
            double *o = out + (w * heads + h) * d;
            for (int32_t i = 0; i < n_pairs; ++i) {
                const double c = cos_sin[(w * n_pairs + i) * 2], sn = cos_sin[(w * n_pairs + i) * 2 + 1];
                const double x0 = (double)row[i], x1 = (double)row[i + n_pairs];
                o[i] = x0 * c - x1 * sn;
                o[i + n_pairs] = x1 * c + x0 * sn;
            }
        }
    }
}

/* --------------------------------------------------------- Eq. 8: anchor aggregation   */
/* For every batch item: K_0 = Norm(LN(X_0)) and Q_A = Norm(LN(A)) row by row (LN without
 * affine, epsilon eps; Norm = division by the l2 norm, a zero row stays zero), logits
 * Q_A K_0^T * inv_tau, softmax over the T dense tokens for every anchor, Z_0 = W_A X_0.
 *   x0 [batch, T, D], anchors [M, D] -> z0 [batch, M, D] (double);
 *   col_sum [batch, T] (may be NULL): sum over the anchors of W_A[a, i], the total weight a
 *   dense token receives. */
static void ln_norm_row(const float *x, int32_t dim, double eps, double *out)
{
    double mean = 0.0, var = 0.0, nrm = 0.0;
    for (int32_t j = 0; j < dim; ++j) mean += (double)x[j];
    mean /= dim;
    for (int32_t j = 0; j < dim; ++j) { double c = (double)x[j] - mean; var += c * c; }
    var /= dim;
    for (int32_t j = 0; j < dim; ++j) { out[j] = ((double)x[j] - mean) / sqrt(var + eps); nrm += out[j] * out[j]; }
    nrm = sqrt(nrm);
    for (int32_t j = 0; j < dim; ++j) out[j] = nrm > 0.0 ? out[j] / nrm : 0.0;
}

void oracle_anchor_aggregate(const float *x0, const float *anchors, int32_t batch, int32_t n_tokens,
                             int32_t n_anchors, int32_t dim, double inv_tau, double eps, double *z0,
                             double *col_sum)
{
    double *qa = (double *)malloc(sizeof(double) * (size_t)n_anchors * dim);
    for (int32_t a = 0; a < n_anchors; ++a) ln_norm_row(anchors + (int64_t)a * dim, dim, eps, qa + (int64_t)a * dim);
    for (int32_t b = 0; b < batch; ++b) {
        const float *xb = x0 + (int64_t)b * n_tokens * dim;
        double *k0 = (double *)malloc(sizeof(double) * (size_t)n_tokens * dim);
        double *w = (double *)malloc(sizeof(double) * (size_t)n_anchors * n_tokens);
#pragma omp parallel for schedule(static)
        for (int32_t i = 0; i < n_tokens; ++i) ln_norm_row(xb + (int64_t)i * dim, dim, eps, k0 + (int64_t)i * dim);
#pragma omp parallel for schedule(static)
        for (int32_t a = 0; a < n_anchors; ++a) {
            double *wa = w + (int64_t)a * n_tokens;
            double zmax = -INFINITY, denom = 0.0;
            for (int32_t i = 0; i < n_tokens; ++i) {
                double acc = 0.0;
                for (int32_t j = 0; j < dim; ++j) acc += qa[(int64_t)a * dim + j] * k0[(int64_t)i * dim + j];
                wa[i] = acc * inv_tau;
                if (wa[i] > zmax) zmax = wa[i];
            }
            for (int32_t i = 0; i < n_tokens; ++i) { wa[i] = exp(wa[i] - zmax); denom += wa[i]; }
            for (int32_t i = 0; i < n_tokens; ++i) wa[i] /= denom;
            double *z = z0 + ((int64_t)b * n_anchors + a) * dim;
            for (int32_t j = 0; j < dim; ++j) z[j] = 0.0;
            for (int32_t i = 0; i < n_tokens; ++i)
                for (int32_t j = 0; j < dim; ++j) z[j] += wa[i] * (double)xb[(int64_t)i * dim + j];
        }
        if (col_sum)
            for (int32_t i = 0; i < n_tokens; ++i) {
                double t = 0.0;
                for (int32_t a = 0; a < n_anchors; ++a) t += w[(int64_t)a * n_tokens + i];
                col_sum[(int64_t)b * n_tokens + i] = t;
            }
        free(k0);
        free(w);
    }
    free(qa);
}

/* ------------------------------------------------- Eq. 9: compressed keys and values   */
/* out[b, s, :] = sum_m Rbar[m, s] * x[b, m, :] with Rbar[m, s] = R[m, s] / sum_m' R[m', s]
 * (a column whose sum is zero gives a zero row).  x [batch, M, width] (width = heads *
 * head_dim), r [M, S] shared by the batch, out [batch, S, width] double. */
void oracle_kv_compress(const float *x, const float *r, int32_t batch, int32_t n_rows, int32_t n_mem,
                        int32_t width, double *out)
{
    double *colsum = (double *)calloc((size_t)n_mem, sizeof(double));
    for (int32_t m = 0; m < n_rows; ++m)
        for (int32_t s = 0; s < n_mem; ++s) colsum[s] += (double)r[(int64_t)m * n_mem + s];
#pragma omp parallel for schedule(static)
    for (int64_t w = 0; w < (int64_t)batch * n_mem; ++w) {
        const int32_t b = (int32_t)(w / n_mem), s = (int32_t)(w % n_mem);
        double *o = out + w * width;
        for (int32_t c = 0; c < width; ++c) o[c] = 0.0;
        if (colsum[s] == 0.0) continue;
        for (int32_t m = 0; m < n_rows; ++m) {
            const double wgt = (double)r[(int64_t)m * n_mem + s] / colsum[s];
            const float *row = x + ((int64_t)b * n_rows + m) * width;
            for (int32_t c = 0; c < width; ++c) o[c] += wgt * (double)row[c];
        }
    }
    free(colsum);
}

/* out[b, i, h, :] = sum_{j < n_kv} softmax_j(scale * <q[b,i,h], k[b,j,g]>) v[b,j,g], g = h /
 * (H_q / H_kv): every query sees every key.  q [batch, n_q, H_q, d], k and v [batch, n_kv,
 * H_kv, d], all dense; out double [batch, n_q, H_q, d]. */
void oracle_cross_attention(const float *q, const float *k, const float *v, double *out, int32_t batch,
                            int32_t n_q, int32_t n_kv, int32_t n_q_heads, int32_t n_kv_heads,
                            int32_t head_dim, double scale)
{
    const int32_t group = n_q_heads / n_kv_heads;
#pragma omp parallel
    {
        double *z = (double *)malloc(sizeof(double) * (size_t)n_kv);
#pragma omp for schedule(static)
        for (int64_t w = 0; w < (int64_t)batch * n_q * n_q_heads; ++w) {
            const int32_t h = (int32_t)(w % n_q_heads);
            const int32_t b = (int32_t)(w / ((int64_t)n_q * n_q_heads));
            const int32_t g = h / group;
            const float *qi = q + w * head_dim;
            double zmax = -INFINITY, denom = 0.0;
            for (int32_t j = 0; j < n_kv; ++j) {
                const float *kj = k + (((int64_t)b * n_kv + j) * n_kv_heads + g) * head_dim;
                double acc = 0.0;
                for (int32_t c = 0; c < head_dim; ++c) acc += (double)qi[c] * (double)kj[c];
                z[j] = scale * acc;
                if (z[j] > zmax) zmax = z[j];
            }
            for (int32_t j = 0; j < n_kv; ++j) { z[j] = exp(z[j] - zmax); denom += z[j]; }
            double *o = out + w * head_dim;
            for (int32_t c = 0; c < head_dim; ++c) o[c] = 0.0;
            for (int32_t j = 0; j < n_kv; ++j) {
                const float *vj = v + (((int64_t)b * n_kv + j) * n_kv_heads + g) * head_dim;
                const double p = z[j] / denom;
                for (int32_t c = 0; c < head_dim; ++c) o[c] += p * (double)vj[c];
            }
        }
        free(z);
    }
}

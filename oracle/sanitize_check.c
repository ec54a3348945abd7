/*
 * Host-side sanitizer run of the CPU oracle (test infrastructure, like the oracle itself).
 *
 * Compiled together with civic_oracle.c under -fsanitize=address,undefined by
 * tests/test_oracle_sanitizers.py and executed there: every oracle function is driven over
 * small shapes that include the edge cases (ragged cells, floors above the budget, empty
 * kept lists, one-row caches, strided K/V), with exactly-sized heap buffers so that any
 * out-of-bounds access, overflow or misaligned access aborts the run.  A few invariants
 * that need no second implementation are checked on the way.  Prints "sanitize_check OK".
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct { int32_t frames, height, width, cell_h, cell_w, cell_floor, frame_floor, budget; } oracle_grid;

int oracle_anchor_normalize(const float *a, int32_t dim, double eps, double *q);
void oracle_score(const float *x, int64_t n_rows, int64_t row_stride, int32_t dim, const float *q, double inv_tau, float *scores);
int64_t oracle_select(const float *scores, const oracle_grid *g, int nested, uint8_t *keep);
int64_t oracle_select_batch(const float *scores, int32_t batch, const oracle_grid *g, int nested, int32_t *kept_idx,
                            int64_t kept_capacity, uint8_t *keep_flags);
int64_t oracle_kept_count(const oracle_grid *g, int nested);
int64_t oracle_compact(const uint8_t *hidden, int64_t row_bytes, const int32_t *pos_ids, int32_t batch, int64_t seq_len,
                       const oracle_grid *g, const int64_t *frame_start, const int32_t *kept_idx, int64_t n_kept,
                       int64_t seq_c_capacity, uint8_t *hidden_c, int32_t *pos_c, int32_t *src_idx);
void oracle_attention(const float *q, const float *k, const float *v, double *out, int32_t batch, int32_t seq,
                      int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, const int64_t *q_strides,
                      const int64_t *kv_strides, int causal, double scale, int32_t row_step);
int64_t oracle_kv_write(const uint8_t *k, const uint8_t *v, const int64_t *kv_strides_bytes, uint8_t *k_cache,
                        uint8_t *v_cache, int32_t batch, int32_t seq, int32_t n_kv_heads, int64_t head_bytes,
                        int64_t s_max, int64_t pos0);
void oracle_decode_attention(const float *q, const float *k_cache, const float *v_cache, double *out, int32_t batch,
                             int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, int64_t s_max, int64_t n_ctx,
                             double scale);

void oracle_mrope_table(const int32_t *pos_ids, int32_t batch, int64_t seq, int32_t n_pairs, const int32_t *axis_of_pair,
                        const float *inv_freq, double *cos_sin);
void oracle_mrope_apply(const float *x, const int64_t *x_strides, int32_t batch, int64_t seq, int32_t heads, int32_t n_pairs,
                        const double *cos_sin, double *out);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static float rnd(void)
{
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return (float)((double)(rng_state >> 40) / (double)(1 << 24)) * 2.0f - 1.0f;
}
static float *rand_floats(size_t n)
{
    float *p = (float *)malloc(sizeof(float) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) p[i] = rnd();
    return p;
}
#define CHECK(c) do { if (!(c)) { printf("sanitize_check FAILED at line %d: %s\n", __LINE__, #c); return 1; } } while (0)

int main(void)
{
    /* score: rows at a stride, a constant row */
    {
        const int32_t dim = 24, rows = 7, stride = 40;
        float *a = rand_floats(dim), *x = rand_floats((size_t)(rows - 1) * stride + dim), *qf = (float *)malloc(sizeof(float) * dim);
        double *q = (double *)malloc(sizeof(double) * dim);
        float *s = (float *)malloc(sizeof(float) * rows);
        CHECK(oracle_anchor_normalize(a, dim, 1e-6, q) == 0);
        for (int j = 0; j < dim; ++j) { qf[j] = (float)q[j]; x[3 * stride + j] = 2.5f; }
        oracle_score(x, rows, stride, dim, qf, 3.0, s);
        CHECK(s[3] == 0.0f);
        for (int i = 0; i < rows; ++i) CHECK(fabsf(s[i]) <= 3.0f + 1e-5f);
        free(a); free(x); free(qf); free(q); free(s);
    }
    /* select + compact over grids with ragged cells, floors above the budget, nothing kept */
    {
        const oracle_grid grids[] = {
            {1, 4, 4, 2, 2, 1, 0, 5}, {1, 5, 7, 2, 3, 9, 0, 4}, {2, 3, 5, 2, 2, 1, 2, 9}, {3, 4, 6, 4, 3, 0, 5, 7},
            {1, 1, 1, 1, 1, 1, 1, 1}, {2, 6, 5, 4, 4, 0, 0, 0}, {1, 3, 3, 3, 3, 0, 0, 9},
        };
        for (size_t gi = 0; gi < sizeof(grids) / sizeof(grids[0]); ++gi) {
            const oracle_grid *g = &grids[gi];
            for (int nested = 0; nested < 2; ++nested) {
                const int32_t batch = 2, hw = g->height * g->width, nv = g->frames * hw;
                const int64_t k = oracle_kept_count(g, nested);
                CHECK(k >= g->budget && k <= nv);
                float *sc = rand_floats((size_t)batch * nv);
                int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)(batch * k ? batch * k : 1));
                uint8_t *flags = (uint8_t *)malloc((size_t)batch * nv);
                CHECK(oracle_select_batch(sc, batch, g, nested, idx, k, flags) == k);
                for (int b = 0; b < batch; ++b)
                    for (int64_t i = 1; i < k; ++i) CHECK(idx[b * k + i] > idx[b * k + i - 1]);
                if (nested) { free(sc); free(idx); free(flags); continue; }
                /* compact: frames separated by one text token, 6-byte rows */
                const int64_t seq = nv + g->frames + 1, seq_c = seq - nv + k, rb = 6;
                int64_t *fs = (int64_t *)malloc(sizeof(int64_t) * g->frames);
                for (int f = 0; f < g->frames; ++f) fs[f] = 1 + (int64_t)f * (hw + 1);
                uint8_t *hid = (uint8_t *)malloc((size_t)(batch * seq * rb));
                int32_t *pos = (int32_t *)malloc(sizeof(int32_t) * (size_t)(3 * batch * seq));
                for (int64_t i = 0; i < batch * seq * rb; ++i) hid[i] = (uint8_t)(i * 7);
                for (int64_t i = 0; i < 3 * batch * seq; ++i) pos[i] = (int32_t)i;
                uint8_t *hc = (uint8_t *)malloc((size_t)(batch * seq_c * rb));
                int32_t *pc = (int32_t *)malloc(sizeof(int32_t) * (size_t)(3 * batch * seq_c));
                int32_t *si = (int32_t *)malloc(sizeof(int32_t) * (size_t)(batch * seq_c));
                CHECK(oracle_compact(hid, rb, pos, batch, seq, g, fs, idx, k, seq_c, hc, pc, si) == seq_c);
                for (int b = 0; b < batch; ++b)
                    for (int64_t j = 0; j < seq_c; ++j) {
                        const int32_t t = si[b * seq_c + j];
                        CHECK(t >= 0 && t < seq && (j == 0 || t > si[b * seq_c + j - 1]));
                        CHECK(memcmp(hc + (b * seq_c + j) * rb, hid + (b * seq + t) * rb, (size_t)rb) == 0);
                        CHECK(pc[(2 * batch + b) * seq_c + j] == pos[(2 * batch + b) * seq + t]);
                    }
                free(sc); free(idx); free(flags); free(fs); free(hid); free(pos); free(hc); free(pc); free(si);
            }
        }
    }
    /* attention (strided K/V, sampled rows), KV write into a longer cache, decode over the cache */
    {
        const int32_t b = 2, s = 19, hq = 4, hkv = 2, d = 12;
        const int64_t qs[3] = {(int64_t)s * hq * d, (int64_t)hq * d, d};
        const int64_t kvw = (int64_t)hkv * d + 5;                /* K/V rows embedded in wider rows */
        const int64_t ks[3] = {(int64_t)s * kvw, kvw, d};
        float *q = rand_floats((size_t)b * s * hq * d);
        const size_t kv_elems = (size_t)((b - 1) * ks[0] + (s - 1) * ks[1] + (hkv - 1) * ks[2] + d);
        float *k = rand_floats(kv_elems), *v = rand_floats(kv_elems);
        double *o = (double *)malloc(sizeof(double) * (size_t)b * s * hq * d);
        for (int causal = 0; causal < 2; ++causal)
            for (int step = 1; step <= 5; step += 4) {
                oracle_attention(q, k, v, o, b, s, hq, hkv, d, qs, ks, causal, 0.3, step);
                CHECK(isfinite(o[0]));
            }
        const int64_t s_max = s + 3, pos0 = 2, ksb[3] = {ks[0] * 4, ks[1] * 4, ks[2] * 4};
        float *kc = (float *)calloc((size_t)(b * hkv * s_max * d), sizeof(float));
        float *vc = (float *)calloc((size_t)(b * hkv * s_max * d), sizeof(float));
        CHECK(oracle_kv_write((const uint8_t *)k, (const uint8_t *)v, ksb, (uint8_t *)kc, (uint8_t *)vc, b, s, hkv, d * 4,
                              s_max, pos0) == (int64_t)2 * b * s * hkv * d * 4);
        CHECK(kc[0] == 0.0f && kc[(pos0 * d)] == k[0]);
        double *od = (double *)malloc(sizeof(double) * (size_t)b * hq * d);
        oracle_decode_attention(q, kc, vc, od, b, hq, hkv, d, s_max, 1, 0.3);
        CHECK(od[0] == (double)vc[0]);
        oracle_decode_attention(q, kc, vc, od, b, hq, hkv, d, s_max, s_max, 0.3);
        CHECK(isfinite(od[b * hq * d - 1]));
        free(q); free(k); free(v); free(o); free(kc); free(vc); free(od);
    }
    /* rotary embedding: rows embedded in wider rows, ids on three axes */
    {
        const int32_t b = 2, heads = 3, np_ = 5, d = 10;
        const int64_t s = 7, xs[3] = {s * heads * (d + 3), heads * (d + 3), d + 3};
        float *x = rand_floats((size_t)((b - 1) * xs[0] + (s - 1) * xs[1] + (heads - 1) * xs[2] + d));
        int32_t *pos = (int32_t *)malloc(sizeof(int32_t) * (size_t)(3 * b * s));
        for (int64_t i = 0; i < 3 * b * s; ++i) pos[i] = (int32_t)(i * 37 % 1000);
        const int32_t axis[5] = {0, 1, 2, 1, 0};
        const float inv[5] = {1.0f, 0.5f, 0.1f, 0.01f, 0.001f};
        double *cs = (double *)malloc(sizeof(double) * (size_t)(b * s * np_ * 2));
        double *o = (double *)malloc(sizeof(double) * (size_t)(b * s * heads * d));
        oracle_mrope_table(pos, b, s, np_, axis, inv, cs);
        oracle_mrope_apply(x, xs, b, s, heads, np_, cs, o);
        CHECK(fabs(cs[0] * cs[0] + cs[1] * cs[1] - 1.0) < 1e-12 && isfinite(o[b * s * heads * d - 1]));
        free(x); free(pos); free(cs); free(o);
    }
    printf("sanitize_check OK\n");
    return 0;
}

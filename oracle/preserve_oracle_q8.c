/*
 * CPU oracle, int8 variant of the decode layer (see preserve_oracle.h for the format).
 *
 * TEST INFRASTRUCTURE ONLY: never linked into, imported by or called from the GPU library.
 * Same style as the bf16 oracle: plain loops in double precision; the one single-precision
 * step is the quantisation of the appended key / value rows, which decides integer codes.
 */
#include "preserve_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* out[r] = scale[r] * sum_c code[r][c] * in[c] */
void orc_linear_q8(const int8_t *codes, const float *scale, const double *in, int rows, int cols,
                   double *out)
{
#pragma omp parallel for schedule(static)
    for (int r = 0; r < rows; ++r) {
        const int8_t *wr = codes + (size_t)r * (size_t)cols;
        double acc = 0.0;
        for (int c = 0; c < cols; ++c) acc += (double)wr[c] * in[c];
        out[r] = (double)scale[r] * acc;
    }
}

/* Symmetric per-row quantisation of v[0..n) to int8; codes are written `stride` bytes apart. */
void orc_quantize_row(const double *v, int n, int stride, int8_t *codes, float *scale)
{
    float amax = 0.0f;
    for (int i = 0; i < n; ++i) {
        float a = fabsf((float)v[i]);
        if (a > amax) amax = a;
    }
    float s = amax > 0.0f ? amax / 127.0f : 1.0f;
    for (int i = 0; i < n; ++i) {
        float q = rintf((float)v[i] / s);            /* default rounding mode: ties to even */
        if (q > 127.0f) q = 127.0f;
        if (q < -127.0f) q = -127.0f;
        codes[(size_t)i * (size_t)stride] = (int8_t)q;
    }
    *scale = s;
}

/* ---- int8 cache addressing: a (block, kv head) unit is bt*d code bytes, then bt fp32 scales */

static size_t unit_bytes(const orc_model *m)
{
    return (size_t)m->block_tokens * (size_t)m->head_dim + 4u * (size_t)m->block_tokens;
}

static size_t block_of(const orc_kv_x *kv, int b, int t, int bt)
{
    size_t logical = (size_t)b * (size_t)kv->max_blocks + (size_t)(t / bt);
    return kv->page_table ? (size_t)kv->page_table[logical] : logical;
}

static uint8_t *unit_ptr(const orc_model *m, void *pool, size_t block, int kvh)
{
    return (uint8_t *)pool + (block * (size_t)m->n_kv_heads + (size_t)kvh) * unit_bytes(m);
}

static float unit_scale(const orc_model *m, const uint8_t *unit, int row)
{
    float s;
    memcpy(&s, unit + (size_t)m->block_tokens * (size_t)m->head_dim + 4u * (size_t)row, sizeof s);
    return s;
}

void orc_attention_head_q8(const orc_model *m, const orc_kv_x *kv, int b, int q_head,
                           const double *q, double *out)
{
    int d = m->head_dim, bt = m->block_tokens;
    int group = m->n_q_heads / m->n_kv_heads;
    int kvh = q_head / group;
    int T = kv->seq_lens[b];
    double *p = (double *)malloc((size_t)T * sizeof(double));
    double inv_sqrt_d = 1.0 / sqrt((double)d);
    for (int t = 0; t < T; ++t) {
        const uint8_t *unit = unit_ptr(m, kv->k_pool, block_of(kv, b, t, bt), kvh);
        const int8_t *row = (const int8_t *)unit + (size_t)(t % bt) * (size_t)d;     /* [token][channel] */
        double acc = 0.0;
        for (int c = 0; c < d; ++c) acc += q[c] * (double)row[c];
        p[t] = acc * (double)unit_scale(m, unit, t % bt) * inv_sqrt_d;
    }
    orc_softmax(p, T);
    for (int c = 0; c < d; ++c) out[c] = 0.0;
    for (int t = 0; t < T; ++t) {
        const uint8_t *unit = unit_ptr(m, kv->v_pool, block_of(kv, b, t, bt), kvh);
        const int8_t *codes = (const int8_t *)unit;                                   /* [channel][token] */
        double vs = (double)unit_scale(m, unit, t % bt);
        for (int c = 0; c < d; ++c)
            out[c] += p[t] * vs * (double)codes[(size_t)c * (size_t)bt + (size_t)(t % bt)];
    }
    free(p);
}

static void linear_any(const void *w, const float *scale, const double *in, int rows, int cols, double *out)
{
    if (scale) orc_linear_q8((const int8_t *)w, scale, in, rows, cols, out);
    else       orc_linear((const uint16_t *)w, in, rows, cols, out);
}

int orc_decode_layer_x(const orc_model *m, const orc_layer_weights_x *w, const orc_kv_x *kv,
                       int batch, double *x)
{
    if (!m || !w || !kv || !x || batch < 0) return -1;
    int H = m->hidden, nq = m->n_q_heads, nkv = m->n_kv_heads, d = m->head_dim, F = m->ffn;
    int bt = m->block_tokens;
    if (H <= 0 || nq <= 0 || nkv <= 0 || d <= 0 || (d & 1) || F <= 0 || bt <= 0 || nq % nkv) return -1;
    if (m->kv_token_major && kv->kv_int8) return -1;      /* the token-major layout is defined for the bf16 cache only */
    int qkv_rows = (nq + 2 * nkv) * d;

    double *h   = (double *)malloc((size_t)H * sizeof(double));
    double *qkv = (double *)malloc((size_t)batch * (size_t)qkv_rows * sizeof(double));
    double *o   = (double *)malloc((size_t)batch * (size_t)nq * (size_t)d * sizeof(double));
    double *a   = (double *)malloc((size_t)H * sizeof(double));
    double *gt  = (double *)malloc((size_t)F * sizeof(double));
    double *up  = (double *)malloc((size_t)F * sizeof(double));
    int rc = 0;

    /* norm, q/k/v projection, rotation, cache append (rounded to bf16 or quantised per row) */
    for (int b = 0; b < batch && !rc; ++b) {
        int T = kv->seq_lens[b];
        if (T < 1 || (T - 1) / bt >= kv->max_blocks) { rc = -1; break; }
        double *row = qkv + (size_t)b * (size_t)qkv_rows;
        orc_rmsnorm(x + (size_t)b * H, w->g_attn, H, m->rms_eps, h);
        linear_any(w->w_qkv, w->s_qkv, h, qkv_rows, H, row);
        int pos = T - 1;
        for (int j = 0; j < nq + nkv; ++j) orc_rope(row + (size_t)j * d, d, (int64_t)pos, m->rope_theta);
        size_t blk = block_of(kv, b, pos, bt);
        int r = pos % bt;
        for (int kvh = 0; kvh < nkv; ++kvh) {
            const double *kn = row + (size_t)(nq + kvh) * d;
            const double *vn = row + (size_t)(nq + nkv + kvh) * d;
            if (kv->kv_int8) {
                uint8_t *ku = unit_ptr(m, kv->k_pool, blk, kvh), *vu = unit_ptr(m, kv->v_pool, blk, kvh);
                float ks, vs;
                orc_quantize_row(kn, d, 1, (int8_t *)ku + (size_t)r * (size_t)d, &ks);
                orc_quantize_row(vn, d, bt, (int8_t *)vu + (size_t)r, &vs);
                memcpy(ku + (size_t)bt * (size_t)d + 4u * (size_t)r, &ks, sizeof ks);
                memcpy(vu + (size_t)bt * (size_t)d + 4u * (size_t)r, &vs, sizeof vs);
            } else {
                uint16_t *kp = (uint16_t *)kv->k_pool, *vp = (uint16_t *)kv->v_pool;
                size_t base = blk * (size_t)nkv + (size_t)kvh;
                size_t tm = ((blk * (size_t)bt + (size_t)r) * (size_t)nkv + (size_t)kvh) * (size_t)d;   /* token-major row */
                for (int c = 0; c < d; ++c) {
                    if (m->kv_token_major) {
                        kp[tm + (size_t)c] = orc_f64_to_bf16(kn[c]);
                        vp[tm + (size_t)c] = orc_f64_to_bf16(vn[c]);
                    } else {
                        kp[(base * (size_t)bt + (size_t)r) * (size_t)d + (size_t)c] = orc_f64_to_bf16(kn[c]);
                        vp[(base * (size_t)d + (size_t)c) * (size_t)bt + (size_t)r] = orc_f64_to_bf16(vn[c]);
                    }
                }
            }
        }
    }

    if (!rc) {
        orc_kv kvb = { (uint16_t *)kv->k_pool, (uint16_t *)kv->v_pool, kv->page_table, kv->max_blocks, kv->seq_lens };
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
        for (int b = 0; b < batch; ++b)
            for (int j = 0; j < nq; ++j) {
                const double *q = qkv + (size_t)b * qkv_rows + (size_t)j * d;
                double *dst = o + ((size_t)b * nq + (size_t)j) * d;
                if (kv->kv_int8) orc_attention_head_q8(m, kv, b, j, q, dst);
                else             orc_attention_head(m, &kvb, b, j, q, dst);
            }

        for (int b = 0; b < batch; ++b) {
            double *xb = x + (size_t)b * H;
            linear_any(w->w_o, w->s_o, o + (size_t)b * nq * d, H, nq * d, a);
            for (int i = 0; i < H; ++i) xb[i] += a[i];

            orc_rmsnorm(xb, w->g_mlp, H, m->rms_eps, h);
            linear_any(w->w_gate, w->s_gate, h, F, H, gt);
            linear_any(w->w_up, w->s_up, h, F, H, up);
            for (int i = 0; i < F; ++i) gt[i] = orc_silu(gt[i]) * up[i];
            linear_any(w->w_down, w->s_down, gt, H, F, a);
            for (int i = 0; i < H; ++i) xb[i] += a[i];
        }
    }

    free(h); free(qkv); free(o); free(a); free(gt); free(up);
    return rc;
}

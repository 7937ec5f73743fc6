/*
 * CPU oracle for the PRESERVE decode step (see preserve_oracle.h).
 *
 * TEST INFRASTRUCTURE ONLY: never linked into, imported by or called from the GPU library.
 * Straightforward loops in double precision, no blocking, no fusion, no reordering beyond
 * what the definitions state.  The only parallelism is an OpenMP loop over independent
 * outputs (rows of a projection; (sequence, head) pairs of attention).
 */
#include "preserve_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ bf16 <-> double */

double orc_bf16_to_f64(uint16_t h)
{
    uint32_t bits = (uint32_t)h << 16;   /* bf16 is the top half of an IEEE single */
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

uint16_t orc_f64_to_bf16(double v)
{
    float f = (float)v;
    uint32_t bits;
    memcpy(&bits, &f, sizeof bits);
    if ((bits & 0x7fffffffu) > 0x7f800000u)          /* NaN: keep it a quiet NaN */
        return (uint16_t)((bits >> 16) | 0x0040u);
    uint32_t keep_lsb = (bits >> 16) & 1u;           /* ties go to the even bf16 */
    bits += 0x7fffu + keep_lsb;
    return (uint16_t)(bits >> 16);
}

/* ------------------------------------------------------------------ elementary pieces */

/* Root-mean-square normalisation with a learned gain (the "normalization" layers of
 * Section 2): out_i = x_i * gain_i / sqrt(mean(x^2) + eps). */
void orc_rmsnorm(const double *x, const uint16_t *gain, int n, double eps, double *out)
{
    double ss = 0.0;
    for (int i = 0; i < n; ++i) ss += x[i] * x[i];
    double inv = 1.0 / sqrt(ss / (double)n + eps);
    for (int i = 0; i < n; ++i) out[i] = x[i] * inv * orc_bf16_to_f64(gain[i]);
}

/* Linear projection out = W * in with W [rows][cols] row-major bf16 (Section 2: the
 * projection layers, whose weights are read-only during decode). */
void orc_linear(const uint16_t *w, const double *in, int rows, int cols, double *out)
{
#pragma omp parallel for schedule(static)
    for (int r = 0; r < rows; ++r) {
        const uint16_t *wr = w + (size_t)r * (size_t)cols;
        double acc = 0.0;
        for (int c = 0; c < cols; ++c) acc += orc_bf16_to_f64(wr[c]) * in[c];
        out[r] = acc;
    }
}

/* Rotary positional embedding, "rotate-half" pairing: channel i is paired with i + d/2 and
 * the pair is rotated by pos * theta^(-2i/d).  (Section 2 only names "a positional
 * embedding"; the form is the one used by the Llama-family models the paper evaluates.) */
void orc_rope(double *vec, int d, int64_t pos, double theta)
{
    if (theta <= 0.0) return;
    int half = d / 2;
    for (int i = 0; i < half; ++i) {
        double freq = pow(theta, -2.0 * (double)i / (double)d);
        double ang = (double)pos * freq;
        double c = cos(ang), s = sin(ang);
        double a = vec[i], b = vec[i + half];
        vec[i] = a * c - b * s;
        vec[i + half] = b * c + a * s;
    }
}

void orc_softmax(double *s, int n)
{
    double mx = s[0];
    for (int i = 1; i < n; ++i) if (s[i] > mx) mx = s[i];
    double sum = 0.0;
    for (int i = 0; i < n; ++i) { s[i] = exp(s[i] - mx); sum += s[i]; }
    for (int i = 0; i < n; ++i) s[i] /= sum;
}

double orc_silu(double z) { return z / (1.0 + exp(-z)); }

/* ------------------------------------------------------------------ KV-cache addressing */

static size_t kv_block_of(const orc_kv *kv, int b, int t, int bt)
{
    size_t logical = (size_t)b * (size_t)kv->max_blocks + (size_t)(t / bt);
    return kv->page_table ? (size_t)kv->page_table[logical] : logical;
}

static size_t tm_index(const orc_model *m, size_t block, int kvh, int row, int c)
{
    return ((block * (size_t)m->block_tokens + (size_t)row) * (size_t)m->n_kv_heads + (size_t)kvh)
               * (size_t)m->head_dim + (size_t)c;
}

static size_t k_index(const orc_model *m, size_t block, int kvh, int row, int c)
{
    if (m->kv_token_major) return tm_index(m, block, kvh, row, c);
    return ((block * (size_t)m->n_kv_heads + (size_t)kvh) * (size_t)m->block_tokens + (size_t)row)
               * (size_t)m->head_dim + (size_t)c;
}

static size_t v_index(const orc_model *m, size_t block, int kvh, int row, int c)
{
    if (m->kv_token_major) return tm_index(m, block, kvh, row, c);
    return ((block * (size_t)m->n_kv_heads + (size_t)kvh) * (size_t)m->head_dim + (size_t)c)
               * (size_t)m->block_tokens + (size_t)row;
}

/* ------------------------------------------------------------------ attention */

/* Decode attention of one query head against all T cached tokens of its kv head
 * (Section 2, "LLM decoding is memory BW-limited": QK^T, softmax, SV with one narrow
 * operand).  Scores are scaled by 1/sqrt(d). */
void orc_attention_head(const orc_model *m, const orc_kv *kv, int b, int q_head,
                        const double *q, double *out)
{
    int d = m->head_dim, bt = m->block_tokens;
    int group = m->n_q_heads / m->n_kv_heads;
    int kvh = q_head / group;
    int T = kv->seq_lens[b];
    double *p = (double *)malloc((size_t)T * sizeof(double));
    double scale = 1.0 / sqrt((double)d);
    for (int t = 0; t < T; ++t) {
        size_t blk = kv_block_of(kv, b, t, bt);
        double acc = 0.0;
        for (int c = 0; c < d; ++c)
            acc += q[c] * orc_bf16_to_f64(kv->k_pool[k_index(m, blk, kvh, t % bt, c)]);
        p[t] = acc * scale;
    }
    orc_softmax(p, T);
    for (int c = 0; c < d; ++c) out[c] = 0.0;
    for (int t = 0; t < T; ++t) {
        size_t blk = kv_block_of(kv, b, t, bt);
        for (int c = 0; c < d; ++c)
            out[c] += p[t] * orc_bf16_to_f64(kv->v_pool[v_index(m, blk, kvh, t % bt, c)]);
    }
    free(p);
}

/* ------------------------------------------------------------------ one decoder layer */

int orc_decode_layer(const orc_model *m, const orc_layer_weights *w, const orc_kv *kv,
                     int batch, double *x)
{
    if (!m || !w || !kv || !x || batch < 0) return -1;
    int H = m->hidden, nq = m->n_q_heads, nkv = m->n_kv_heads, d = m->head_dim, F = m->ffn;
    int bt = m->block_tokens;
    if (H <= 0 || nq <= 0 || nkv <= 0 || d <= 0 || (d & 1) || F <= 0 || bt <= 0 || nq % nkv) return -1;
    int qkv_rows = (nq + 2 * nkv) * d;

    double *h   = (double *)malloc((size_t)H * sizeof(double));
    double *qkv = (double *)malloc((size_t)batch * (size_t)qkv_rows * sizeof(double));
    double *o   = (double *)malloc((size_t)batch * (size_t)nq * (size_t)d * sizeof(double));
    double *a   = (double *)malloc((size_t)H * sizeof(double));
    double *gt  = (double *)malloc((size_t)F * sizeof(double));
    double *up  = (double *)malloc((size_t)F * sizeof(double));

    /* Attention block, part 1: norm, fused q/k/v projection, rotation, cache append. */
    for (int b = 0; b < batch; ++b) {
        int T = kv->seq_lens[b];
        if (T < 1 || (T - 1) / bt >= kv->max_blocks) {
            free(h); free(qkv); free(o); free(a); free(gt); free(up);
            return -1;
        }
        double *row = qkv + (size_t)b * (size_t)qkv_rows;
        orc_rmsnorm(x + (size_t)b * H, w->g_attn, H, m->rms_eps, h);
        orc_linear(w->w_qkv, h, qkv_rows, H, row);
        int64_t pos = (int64_t)T - 1;                 /* the token being decoded */
        for (int j = 0; j < nq + nkv; ++j)            /* q heads then k heads; v is not rotated */
            orc_rope(row + (size_t)j * d, d, pos, m->rope_theta);
        size_t blk = kv_block_of(kv, b, (int)pos, bt);
        for (int kvh = 0; kvh < nkv; ++kvh) {
            const double *kn = row + (size_t)(nq + kvh) * d;
            const double *vn = row + (size_t)(nq + nkv + kvh) * d;
            for (int c = 0; c < d; ++c) {
                kv->k_pool[k_index(m, blk, kvh, (int)(pos % bt), c)] = orc_f64_to_bf16(kn[c]);
                kv->v_pool[v_index(m, blk, kvh, (int)(pos % bt), c)] = orc_f64_to_bf16(vn[c]);
            }
        }
    }

    /* Attention block, part 2: every (sequence, query head) is independent. */
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < batch; ++b)
        for (int j = 0; j < nq; ++j)
            orc_attention_head(m, kv, b, j, qkv + (size_t)b * qkv_rows + (size_t)j * d,
                               o + ((size_t)b * nq + (size_t)j) * d);

    /* Output projection and residual, then the MLP block with its residual.  The sum over
     * tensor-parallel ranks that would follow each block is the identity for one rank. */
    for (int b = 0; b < batch; ++b) {
        double *xb = x + (size_t)b * H;
        orc_linear(w->w_o, o + (size_t)b * nq * d, H, nq * d, a);
        for (int i = 0; i < H; ++i) xb[i] += a[i];

        orc_rmsnorm(xb, w->g_mlp, H, m->rms_eps, h);
        orc_linear(w->w_gate, h, F, H, gt);
        orc_linear(w->w_up, h, F, H, up);
        for (int i = 0; i < F; ++i) gt[i] = orc_silu(gt[i]) * up[i];
        orc_linear(w->w_down, gt, H, F, a);
        for (int i = 0; i < H; ++i) xb[i] += a[i];
    }

    free(h); free(qkv); free(o); free(a); free(gt); free(up);
    return 0;
}

int orc_decode_step(const orc_model *m, int n_layers, const orc_layer_weights *weights,
                    uint16_t *const *k_pools, uint16_t *const *v_pools,
                    const int32_t *page_table, int32_t max_blocks, const int32_t *seq_lens,
                    int batch, double *x)
{
    if (!weights || !k_pools || !v_pools || n_layers < 0) return -1;
    for (int l = 0; l < n_layers; ++l) {
        orc_kv kv = { k_pools[l], v_pools[l], page_table, max_blocks, seq_lens };
        int rc = orc_decode_layer(m, &weights[l], &kv, batch, x);
        if (rc) return rc;
    }
    return 0;
}

/* ------------------------------------------------------------------ Algorithm 1 */

int64_t orc_plan(int n_nodes, const int32_t *node_type, const uint64_t *mem_size,
                 const int32_t *child_off, const int32_t *child_idx, uint64_t capacity,
                 int32_t *out_comm, int32_t *out_target, int64_t cap)
{
    if (n_nodes < 0 || !node_type || !mem_size || !child_off || (!child_idx && child_off[n_nodes] > 0))
        return -1;
    int32_t *queue = (int32_t *)malloc((size_t)(n_nodes + 1) * sizeof(int32_t));
    unsigned char *seen = (unsigned char *)malloc((size_t)n_nodes + 1);
    int64_t found = 0;

    for (int comm = 0; comm < n_nodes; ++comm) {
        if (node_type[comm] != ORC_NODE_COMM) continue;
        int reached_end = 0;
        uint64_t cache_sum = 0;
        memset(seen, 0, (size_t)n_nodes + 1);
        int head = 0, tail = 0;
        seen[comm] = 1;
        for (int e = child_off[comm]; e < child_off[comm + 1]; ++e)
            if (!seen[child_idx[e]]) { seen[child_idx[e]] = 1; queue[tail++] = child_idx[e]; }

        while (!reached_end && head < tail) {          /* an empty queue is the end of the graph */
            int n = queue[head++];
            if (node_type[n] == ORC_NODE_COMM) {
                reached_end = 1;
            } else if (node_type[n] == ORC_NODE_MATMUL || node_type[n] == ORC_NODE_SELFATTN) {
                cache_sum += mem_size[n];
                if (cache_sum < capacity) {
                    if (found < cap && out_comm && out_target) { out_comm[found] = comm; out_target[found] = n; }
                    ++found;
                } else {
                    reached_end = 1;
                }
            }
            if (!reached_end)
                for (int e = child_off[n]; e < child_off[n + 1]; ++e)
                    if (!seen[child_idx[e]]) { seen[child_idx[e]] = 1; queue[tail++] = child_idx[e]; }
        }
    }
    free(queue); free(seen);
    return found;
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

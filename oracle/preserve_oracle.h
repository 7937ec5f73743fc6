/*
 * CPU oracle for the PRESERVE decode step and its prefetch-insertion planner.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the plain, slow, obviously-correct definition of what
 * the GPU library computes.  It shares no code with the HIP path and is only ever called by
 * the test-suite, the smoke check and the CPU-baseline leg of the benchmark.
 *
 * Arithmetic: every intermediate is IEEE double.  The only rounding to bf16 is the KV-cache
 * append, because the cache *is* bf16 state (Section 3, "Execution with the proposed method":
 * the caches are read-only during decode except for the last entry, which the step writes).
 * bf16 inputs are widened exactly.
 *
 * Layer definition (Section 2 "LLM inference workloads": attention = input projections,
 * positional embedding, self-attention kernel, output projection; MLP = three projections and
 * one activation; Section 2 "Multi-device inference": one allreduce per attention block and
 * one per MLP block).  With a single rank the allreduce is the identity, so the communication
 * window has no numeric effect and does not appear here.
 *
 * KV-cache layout (bt = tokens per block, d = head dim, nkv = local kv heads), head-major (the default):
 *   K pool : [block][kv head][bt tokens][d]      (token-major inside a block)
 *   V pool : [block][kv head][d][bt tokens]      (channel-major inside a block)
 * Token-major layout (orc_model.kv_token_major; bf16 cache only): both pools [block][bt tokens][kv head][d], the
 * layout in which a shard with several local kv heads reads one head's keys and values strided (Section 4, the
 * discussion of the tensor-parallel degree).  Same logical cache, same results.
 * The block that holds token t of sequence b is page_table[b*max_blocks + t/bt], or
 * b*max_blocks + t/bt when page_table is NULL ("contiguous" cache).
 */
#ifndef PRESERVE_ORACLE_H
#define PRESERVE_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t hidden;        /* H */
    int32_t n_q_heads;     /* local query heads */
    int32_t n_kv_heads;    /* local kv heads; divides n_q_heads */
    int32_t head_dim;      /* d, even */
    int32_t ffn;           /* local intermediate width F */
    int32_t block_tokens;  /* bt */
    double  rms_eps;
    double  rope_theta;    /* 0 => no positional rotation */
    int32_t kv_token_major; /* 0 => head-major pools, 1 => token-major pools (see above) */
} orc_model;

typedef struct {
    const uint16_t *w_qkv;   /* bf16 [(nq+2nkv)*d][H], rows: q heads, k heads, v heads */
    const uint16_t *w_o;     /* bf16 [H][nq*d] */
    const uint16_t *w_gate;  /* bf16 [F][H] */
    const uint16_t *w_up;    /* bf16 [F][H] */
    const uint16_t *w_down;  /* bf16 [H][F] */
    const uint16_t *g_attn;  /* bf16 [H] */
    const uint16_t *g_mlp;   /* bf16 [H] */
} orc_layer_weights;

typedef struct {
    uint16_t *k_pool;            /* this layer's K pool (mutated: one slot per sequence) */
    uint16_t *v_pool;            /* this layer's V pool (mutated: one slot per sequence) */
    const int32_t *page_table;   /* [batch][max_blocks] or NULL */
    int32_t max_blocks;          /* row stride of the page table / blocks per sequence */
    const int32_t *seq_lens;     /* [batch]; span INCLUDING the token decoded by this step */
} orc_kv;

/* ---- scalar building blocks (exported so each can be pinned on its own) ---- */
double   orc_bf16_to_f64(uint16_t h);
uint16_t orc_f64_to_bf16(double v);                      /* round-to-nearest-even */
void orc_rmsnorm(const double *x, const uint16_t *gain, int n, double eps, double *out);
void orc_linear(const uint16_t *w, const double *in, int rows, int cols, double *out);
void orc_rope(double *vec, int d, int64_t pos, double theta);
void orc_softmax(double *s, int n);
double orc_silu(double z);

/* One (sequence, query head) of decode attention over tokens [0, T).  q: [d].  out: [d]. */
void orc_attention_head(const orc_model *m, const orc_kv *kv, int b, int q_head,
                        const double *q, double *out);

/* One decoder layer on x [batch][H] in place.  Returns 0, or -1 on a bad argument. */
int orc_decode_layer(const orc_model *m, const orc_layer_weights *w, const orc_kv *kv,
                     int batch, double *x);

/* Layers [0, n_layers) in order.  weights[l], k_pools[l], v_pools[l] per layer. */
int orc_decode_step(const orc_model *m, int n_layers, const orc_layer_weights *weights,
                    uint16_t *const *k_pools, uint16_t *const *v_pools,
                    const int32_t *page_table, int32_t max_blocks, const int32_t *seq_lens,
                    int batch, double *x);

/* ---- int8 variant -------------------------------------------------------------------------
 *
 * The paper's measurements store weights and KV-cache in int8 (Section 4, experimental set-up and
 * the captions of its result tables) but give no quantisation scheme; this is the one assumed here.
 *
 * Weights: int8 codes [rows][cols] row-major and one fp32 scale per output row;
 *          W[r][c] = scale[r] * code[r][c].
 * KV-cache: one fp32 scale per (token, kv head).  A block of one kv head is bt*d code bytes followed
 *          by bt fp32 scales (2048 + 64 bytes for bt = 16, d = 128); a pool block is n_kv_heads of
 *          those.  K codes are [token][channel], V codes [channel][token], as in the bf16 layout.
 *          K[t][c] = k_scale[t] * code[t][c]; likewise V.
 * Append rule (orc_quantize_row), taken in single precision because it decides integers:
 *          vf = (float)v;  amax = max|vf|;  scale = amax > 0 ? amax / 127 : 1;
 *          code = clamp(rintf(vf / scale), -127, 127)     (ties to even).
 * Activations stay in floating point (the paper also quantises them; only the bytes streamed from
 * memory matter to the method, and those are weights and KV).
 */
void orc_linear_q8(const int8_t *codes, const float *scale, const double *in, int rows, int cols,
                   double *out);
void orc_quantize_row(const double *v, int n, int stride, int8_t *codes, float *scale);

typedef struct {
    const void *w_qkv, *w_o, *w_gate, *w_up, *w_down;        /* bf16 or int8 codes, shapes as above */
    const float *s_qkv, *s_o, *s_gate, *s_up, *s_down;        /* per-row scales; NULL => bf16 weights */
    const uint16_t *g_attn, *g_mlp;                           /* bf16 [H] */
} orc_layer_weights_x;

typedef struct {
    void *k_pool, *v_pool;       /* bf16 pools, or int8 pools with embedded scales */
    int32_t kv_int8;             /* 0 => bf16 layout, 1 => int8 layout */
    const int32_t *page_table;
    int32_t max_blocks;
    const int32_t *seq_lens;
} orc_kv_x;

/* One (sequence, query head) of decode attention over an int8 cache. */
void orc_attention_head_q8(const orc_model *m, const orc_kv_x *kv, int b, int q_head,
                           const double *q, double *out);

/* One decoder layer with either weight format and either cache format. */
int orc_decode_layer_x(const orc_model *m, const orc_layer_weights_x *w, const orc_kv_x *kv,
                       int batch, double *x);

/* ---- Algorithm 1 (prefetch operator insertion) on a general graph ---- */
enum { ORC_NODE_OTHER = 0, ORC_NODE_COMM = 1, ORC_NODE_MATMUL = 2, ORC_NODE_SELFATTN = 3 };

/*
 * Graph in CSR form: children of node i are child_idx[child_off[i] .. child_off[i+1]).
 * For every communication node (ascending node id) the traversal of its descendants is
 * breadth first; each visited MatMul / SelfAttention node adds mem_size to a running sum and
 * receives a prefetch op while the sum stays strictly below `capacity`; the first node that
 * does not fit, or the first communication node met, ends that communication op's traversal.
 * Writes up to `cap` (comm node, target node) pairs; returns the number of pairs found
 * (which may exceed cap), or -1 on a bad argument.
 */
int64_t orc_plan(int n_nodes, const int32_t *node_type, const uint64_t *mem_size,
                 const int32_t *child_off, const int32_t *child_idx, uint64_t capacity,
                 int32_t *out_comm, int32_t *out_target, int64_t cap);

int orc_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif

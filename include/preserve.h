/*
 * libpreserve_mi355x -- C ABI of the PRESERVE decode step for one tensor-parallel shard on one
 * MI355X (gfx950).
 *
 * The library runs one decode iteration of a pre-norm Llama-style decoder shard -- RMSNorm,
 * QKV projection, rotary embedding, KV-cache append, decode attention over a block-structured
 * (optionally paged) KV-cache, O projection, gate/up projection with SwiGLU, down projection
 * -- and, beside each of the two communication windows of a layer, a prefetch kernel on a
 * side stream that pulls the weights and KV blocks of the operators that follow the window
 * from HBM into the on-chip cache (Section 3, "Execution with the proposed method").  Which
 * operators each window prefetches is decided once by Algorithm 1 (Section 3, "Operator
 * insertion") under the byte budget C of the policy.  The tensor-parallel allreduce that would
 * occupy the window is replaced by a timed single-workgroup spin kernel that moves no data.
 *
 * Conventions
 *  - "dev" pointers are HIP device pointers, "host" pointers are ordinary host memory.
 *  - The caller owns every buffer and both streams.  The library borrows the pointers handed
 *    to psv_set_* until the next psv_set_* of the same kind or psv_destroy.  The library owns
 *    only its context and an internal workspace allocated by psv_create.
 *  - bf16 tensors are raw 16-bit patterns.  Projection weights are row-major [out, in].
 *  - KV-cache: blocks of PSV_BLOCK_TOKENS tokens.  Per layer one K pool
 *    [block][kv head][16 tokens][128 channels] and one V pool [block][kv head][128 channels]
 *    [16 tokens].  Token t of sequence b lives in block page_table[b*max_blocks + t/16], or in
 *    block b*max_blocks + t/16 when the page table is NULL ("contiguous" cache).
 *  - int8 formats (the precision the paper measures in, Section 4; it gives no quantisation scheme, this
 *    one is symmetric and per row).  Weights (weight_format = PSV_FMT_INT8): int8 codes row-major
 *    [out, in] plus one fp32 scale per output row, W[r][c] = scale[r] * code[r][c]; RMSNorm gains stay
 *    bf16.  KV-cache (kv_format = PSV_FMT_INT8): one fp32 scale per (token, kv head); the unit of one
 *    (block, kv head) is 2048 code bytes (K: [16 tokens][128 channels], V: [128 channels][16 tokens])
 *    followed by the 16 fp32 scales of its tokens = PSV_KV_UNIT_BYTES_INT8 bytes, and a pool block is
 *    n_kv_heads units.  The step quantises the key and value rows it appends in single precision:
 *    scale = max|v| / 127 (1 if the row is zero), code = clamp(rint(v / scale), -127, 127), ties to
 *    even.  Activations stay in floating point.
 *  - seq_lens[b] is the attention span INCLUDING the token decoded by the step: the step
 *    writes slot seq_lens[b]-1 of every layer's cache and attends over [0, seq_lens[b]).
 *    It never changes seq_lens or the page table, so repeating a call is idempotent.
 *  - Every entry point returns a psv_status (0 = ok, negative = error); nothing throws, aborts
 *    or prints.  Argument checks are done on the host before anything is launched.
 *    Asynchronous HIP errors surface at psv_sync.
 *  - A context must be used by one host thread at a time.
 */
#ifndef PRESERVE_H
#define PRESERVE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PSV_BLOCK_TOKENS 16u
#define PSV_HEAD_DIM 128u
#define PSV_KV_UNIT_BYTES_BF16 4096u   /* one (block, kv head) of a bf16 K or V pool */
#define PSV_KV_UNIT_BYTES_INT8 2112u   /* 2048 int8 codes + 16 fp32 scales */

enum { PSV_FMT_BF16 = 0u, PSV_FMT_INT8 = 1u };

typedef int32_t psv_status;
enum {
    PSV_OK = 0,
    PSV_ERR_INVALID_ARG = -1,   /* null pointer, size out of range, inconsistent descriptor */
    PSV_ERR_BAD_STATE = -2,     /* e.g. decode step before weights / KV were set */
    PSV_ERR_UNSUPPORTED = -3,   /* shape outside what the kernels are built for */
    PSV_ERR_HIP = -4,           /* a HIP runtime call failed (also: no GPU present) */
    PSV_ERR_NOMEM = -5          /* host or device allocation failed */
};

typedef struct psv_ctx psv_ctx;   /* opaque */

/* Shape and storage formats of one shard.  hidden % 512 == 0, ffn % 256 == 0, head_dim == 128,
 * n_q_heads % n_kv_heads == 0, n_q_heads / n_kv_heads <= 16, max_seq % 16 == 0. */
typedef struct {
    uint32_t n_layers;
    uint32_t hidden;        /* H */
    uint32_t n_q_heads;     /* local query heads */
    uint32_t n_kv_heads;    /* local kv heads */
    uint32_t head_dim;      /* must be 128 */
    uint32_t ffn;           /* local intermediate width F */
    float    rms_eps;
    float    rope_theta;    /* 0 => rotary embedding disabled */
    uint32_t max_batch;
    uint32_t max_seq;       /* largest seq_lens[b] that will be used */
    uint32_t weight_format; /* PSV_FMT_BF16 or PSV_FMT_INT8: format of the five projection matrices */
    uint32_t kv_format;     /* PSV_FMT_BF16 or PSV_FMT_INT8: format of the K and V pools */
} psv_model_desc;

/* dev pointers; projection matrices in the descriptor's weight_format, gains bf16 */
typedef struct {
    const void *w_qkv;      /* [(nq+2nkv)*128, H]  rows: q heads, then k heads, then v heads */
    const void *w_o;        /* [H, nq*128] */
    const void *w_gate;     /* [F, H] */
    const void *w_up;       /* [F, H] */
    const void *w_down;     /* [H, F] */
    const void *g_attn;     /* [H]  RMSNorm gain before the attention block */
    const void *g_mlp;      /* [H]  RMSNorm gain before the MLP block */
    /* fp32 per-output-row scales of the int8 format, same row order as the matrices; ignored
     * (may be NULL) for bf16 weights */
    const float *s_qkv, *s_o, *s_gate, *s_up, *s_down;
} psv_layer_weights;

typedef struct {
    void *const *k_pools;        /* host array [n_layers] of dev pointers (K pool per layer) */
    void *const *v_pools;        /* host array [n_layers] of dev pointers (V pool per layer) */
    const int32_t *page_table;   /* dev [max_batch][max_blocks], or NULL for a contiguous cache */
    uint32_t max_blocks;         /* blocks per sequence = row stride of the page table */
    uint32_t num_pool_blocks;    /* blocks in each pool (bounds the page-table entries) */
    const int32_t *seq_lens;     /* dev [max_batch] */
} psv_kv_desc;

/* Prefetch policy.  budget_bytes is Algorithm 1's capacity C. */
typedef struct {
    uint32_t mode;           /* 0 = off (vanilla execution), 1 = on */
    uint32_t targets;        /* bit 0: projection weights, bit 1: KV blocks */
    uint64_t budget_bytes;   /* C: per window, the running sum must stay strictly below it */
    uint64_t chunk_bytes;    /* one prefetch launch covers at most this many bytes (0 = no split) */
    uint32_t cu_budget;      /* workgroups the prefetch kernel may occupy (0 = default 64) */
    uint32_t partial;        /* 0 = Algorithm 1 as published (an operator is prefetched whole or
                                not at all); 1 = extension: the operator that overflows C is
                                prefetched up to the remaining budget, in the order its consumer
                                reads it */
    uint32_t join;           /* 0 = the op after a window starts when the window ends;
                                1 = it also waits for that window's prefetch to finish */
    uint32_t prelaunch;      /* 0 = every prefetch goes to the memory-side cache (the paper's scheme);
                                1 = extension for this hardware, whose large on-chip memory is the register
                                file (128 MB) rather than a shared cache: when Algorithm 1 hands the first
                                operator after a window (gate/up, or the next layer's QKV) to that window,
                                that operator's kernel is itself launched at the start of the window on the
                                other stream, loads its first weights into registers while the window runs,
                                waits for the window's end on a device flag and finishes from registers; the
                                operator chain continues on that stream, so the two streams swap roles at
                                every window.  Takes effect for eager launches at batch 1 (and batch 2 up
                                to H = 4096), and only on a context whose two streams run concurrently
                                (psv_check_overlap; psv_set_policy runs that check itself if it has not
                                been run): a kernel that waits on a flag must never sit in front of the
                                kernel that sets it -- under a profiler that serialises kernels, or on two
                                streams that share a hardware queue, it would wait until its time limit.
                                Otherwise ignored.  Results are bit-identical either way. */
} psv_prefetch_policy;

enum { PSV_TARGET_WEIGHTS = 1u, PSV_TARGET_KV = 2u };

/* Operator ids (also the order of one layer's chain). */
enum {
    PSV_OP_QKV = 0, PSV_OP_ATTN = 1, PSV_OP_O = 2, PSV_OP_GATE = 3, PSV_OP_UP = 4, PSV_OP_DOWN = 5,
    PSV_OP_COUNT = 6
};

typedef struct {
    uint32_t layer;          /* layer whose communication op hosts this prefetch */
    uint32_t window;         /* 0 = window after the attention block, 1 = after the MLP block */
    uint32_t target_layer;   /* layer of the operator whose data is prefetched */
    uint32_t target_op;      /* PSV_OP_* */
    uint64_t mem_size;       /* Algorithm 1's memSize() of that operator, bytes */
    uint64_t bytes;          /* bytes this entry prefetches (== mem_size unless partial) */
} psv_plan_entry;

typedef struct {
    uint64_t weight_bytes_per_layer;   /* algorithmic bytes: every projection weight once */
    uint64_t kv_bytes_per_layer;       /* algorithmic bytes: K and V of the attended span once */
    uint64_t planned_prefetch_bytes;   /* sum of plan entry bytes over the whole step */
    uint64_t workspace_bytes;
    uint32_t kernels_per_layer;        /* main-stream launches per layer */
    uint32_t prefetch_launches;        /* side-stream launches per step */
    uint32_t steps;                    /* decode steps issued since creation */
    uint32_t reserved;
} psv_stats;

/* ---- pure host functions (no GPU needed) -------------------------------------------- */

/* Human-readable text for a status.  Never NULL; static storage. */
const char *psv_strerror(psv_status s);

/* Checks a descriptor against the limits listed at psv_model_desc. */
psv_status psv_validate_desc(const psv_model_desc *desc);

/* Bytes of device workspace psv_create will allocate for this descriptor (0 if invalid). */
size_t psv_workspace_bytes(const psv_model_desc *desc);

/* Algorithm 1 (Section 3, "Operator insertion") on the operator chain of `desc`:
 * per layer  norm, QKV, rope, attention, O, COMM, norm, gate, up, act, down, COMM.
 * For every communication op the operators that follow it, up to the next communication op or
 * the end of the graph, are visited in program order; a MatMul contributes its weight bytes,
 * the attention its read-only K+V bytes (batch * (context-1) tokens; int8 caches include their
 * scales), both in the descriptor's formats; an operator receives a
 * prefetch while the running sum stays strictly below policy->budget_bytes; the first one that
 * does not fit ends that window.  Operators whose class is not in policy->targets are visited
 * but neither counted nor prefetched.  mode == 0 yields an empty plan.
 * Writes at most `cap` entries to `out` (host; may be NULL when cap == 0) and the full count
 * to *n. */
psv_status psv_plan_chain(const psv_model_desc *desc, uint32_t batch, uint32_t context,
                          const psv_prefetch_policy *policy, psv_plan_entry *out, size_t cap,
                          size_t *n);

/* ---- context ---------------------------------------------------------------------------- */

/* Creates a context on the current HIP device.  stream_main / stream_side are hipStream_t
 * handles owned by the caller; they must differ and have default priority.  Allocates the
 * workspace.  *out is set only on success. */
psv_status psv_create(const psv_model_desc *desc, void *stream_main, void *stream_side,
                      psv_ctx **out);
psv_status psv_destroy(psv_ctx *ctx);

psv_status psv_set_layer_weights(psv_ctx *ctx, uint32_t layer, const psv_layer_weights *w);
psv_status psv_set_kv(psv_ctx *ctx, const psv_kv_desc *kv);

/* Durations of the two communication windows of every layer, microseconds (>= 0).  A window
 * of 0 launches neither the spin kernel nor any prefetch. */
psv_status psv_set_comm_windows(psv_ctx *ctx, float us_after_attn, float us_after_mlp);

/* Stores the policy and rebuilds the plan for (batch, context): Algorithm 1 needs the KV size,
 * which depends on them.  context is the attention span used for memSize(). */
psv_status psv_set_policy(psv_ctx *ctx, const psv_prefetch_policy *policy, uint32_t batch,
                          uint32_t context);

/* Copies the current plan (see psv_plan_chain) to host memory. */
psv_status psv_plan(psv_ctx *ctx, psv_plan_entry *out, size_t cap, size_t *n);

/* 0 = launch kernels one by one on the two streams; 1 = capture the step into a HIP graph on
 * first use (keyed by the argument tuple of psv_decode_step) and replay it afterwards.
 * Graph mode is switched off by default: 1 is answered with PSV_ERR_UNSUPPORTED unless the environment
 * variable PSV_ENABLE_HIP_GRAPHS is "1".  Test runs that went through many capture / replay / destroy
 * cycles ended, rarely, in an abort inside the HIP runtime; until that is understood the eager path (which
 * is also the faster one on this runtime) is the only one enabled. */
psv_status psv_set_graph_mode(psv_ctx *ctx, uint32_t use_graph);

/*
 * One decode step over layers [layer_begin, layer_end): Section 3's execution with (policy
 * mode 1) or without (mode 0) prefetching.  x_in, x_out: dev fp32 [batch, H] (may alias).
 * Asynchronous: returns after enqueueing on stream_main / stream_side.  Mutates only x_out,
 * slot seq_lens[b]-1 of each layer's K and V pools, and the workspace.  The results are bit
 * identical for every policy, window and graph mode.
 */
psv_status psv_decode_step(psv_ctx *ctx, const float *x_in, float *x_out, uint32_t batch,
                           uint32_t layer_begin, uint32_t layer_end);

/* Waits for both streams; returns PSV_ERR_HIP if any enqueued work failed (including a pre-launched kernel
 * whose bounded wait for its window expired). */
psv_status psv_sync(psv_ctx *ctx);

psv_status psv_get_stats(psv_ctx *ctx, psv_stats *out);

/* Chooses how many tokens of a sequence one attention workgroup covers (the split of the span over
 * workgroups).  The default comes from a heuristic on (max_batch, kv heads, max_seq); which split is fastest
 * depends on the shape in ways a heuristic captures only roughly (measured spread over the candidates: 10 %;
 * the default lands within 1-2 % of the best on the shapes it was centred on), so this call times
 * psv_decode_step(ctx, x_in, x_out, batch, 0, 1) -- layer 0 only, prefetching off, no windows -- for a list of
 * candidate splits and keeps the fastest for all later steps of this context.  It has the side effects of that
 * decode step (x_out, slot seq_lens[b]-1 of layer 0's cache) and needs weights of layer 0 and the KV-cache set.
 * The split changes the summation order of the attention partials, i.e. results before and after tuning agree
 * to rounding, not bit for bit; within one split they stay bit-identical for every policy.  *chunk_tokens
 * (optional) receives the choice.  Synchronises both streams. */
psv_status psv_tune_attention(psv_ctx *ctx, const float *x_in, float *x_out, uint32_t batch,
                              uint32_t *chunk_tokens);

/* Checks that work on stream_side really runs beside work on stream_main.  HIP multiplexes streams
 * onto a few hardware queues; two streams that land on the same queue execute one after the other,
 * and a prefetch can then never overlap its window.  The check runs a 1 ms window kernel on
 * stream_main and a gate on stream_side that waits for the window's start flag, and times on the
 * host how long stream_side takes to drain: *concurrent = 1 if the gate got through in under half
 * the window, 0 if it had to wait for the window's end (then create the context again with another
 * side stream).  The context remembers the answer: policy.prelaunch stays without effect unless it is 1.
 * Synchronises both streams. */
psv_status psv_check_overlap(psv_ctx *ctx, int32_t *concurrent);

/* ---- measurement and test aids ---------------------------------------------------------- */

/* When op is a PSV_OP_* id (not PSV_OP_UP: gate and up share one kernel), every later eager-mode
 * decode step binds a HIP event to the dispatch of each main-stream kernel; the duration reported
 * for the operator is the time from the end of the kernel launched just before it on stream_main
 * to the end of the operator's kernel (for PSV_OP_ATTN: the split-K kernel, not the small merge
 * that follows).  op = -1 switches it off.  Synchronises. */
psv_status psv_set_profile_op(psv_ctx *ctx, int32_t op);
/* After psv_sync: total milliseconds and number of bracketed launches since the last call of
 * psv_set_profile_op; resets the accumulation. */
psv_status psv_get_profile(psv_ctx *ctx, double *total_ms, uint64_t *launches);

/* The prefetch kernel on its own: reads `bytes` at dev pointer `ptr` with `workgroups`
 * workgroups on `stream` (hipStream_t) and writes nothing. */
psv_status psv_prefetch_region(const void *ptr, uint64_t bytes, uint32_t workgroups, void *stream);
/* The communication stand-in on its own: one workgroup spinning for `us` microseconds. */
psv_status psv_spin(float us, void *stream);
/* A plain device-to-device copy kernel of `bytes` (multiple of 16) used to calibrate hardware
 * byte counters against a known size. */
psv_status psv_copy_bytes(void *dst, const void *src, uint64_t bytes, void *stream);

/* Test aid for the prelaunch policy: while on, a kernel launched ahead of its window's end gives up its
 * (always bounded) wait at once.  The kernel then still completes, sets an error word, and the next psv_sync
 * returns PSV_ERR_HIP once; the context stays usable. */
psv_status psv_debug_force_wait_timeout(psv_ctx *ctx, uint32_t on);

/* Intermediate buffers of the most recent layer executed, for debugging parity failures.  PSV_DBG_H1 and
 * PSV_DBG_H2 exist only when the step ran on the vector path (batch 1, or batch 2 with H <= 4096): the
 * matrix-core path never forms the normalised activations (it scales the projection's result instead), and
 * psv_debug_read returns PSV_ERR_BAD_STATE for them. */
enum {
    PSV_DBG_H1 = 0,     /* fp32 [batch, H]            normalised input of QKV */
    PSV_DBG_QKV = 1,    /* fp32 [batch, (nq+2nkv)*128] projection output before rotation */
    PSV_DBG_ATTN = 2,   /* fp32 [batch, nq*128]       attention output */
    PSV_DBG_Y = 3,      /* fp32 [batch, H]            residual after the attention block */
    PSV_DBG_H2 = 4,     /* fp32 [batch, H]            normalised input of gate/up */
    PSV_DBG_M = 5,      /* fp32 [batch, F]            silu(gate) * up */
    PSV_DBG_COUNT = 6
};
/* Synchronises, then copies min(bytes, buffer size) bytes of buffer `which` to host memory. */
psv_status psv_debug_read(psv_ctx *ctx, uint32_t which, void *host_dst, size_t bytes);

#ifdef __cplusplus
}
#endif
#endif

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
 *    With kv_layout = PSV_KV_TOKEN_MAJOR (bf16 cache only) both pools are [block][16 tokens][kv head][128 channels]
 *    instead: the layout in which a shard with several local kv heads reads one head's keys and values as
 *    256-byte pieces at a stride of n_kv_heads * 256 bytes (Section 4, the discussion of the tensor-parallel
 *    degree, attributes the larger gains at 2 local kv heads to such strided reads).  Same bytes per block, same
 *    results to rounding; offered to measure that effect.
 *    With weight_layout = PSV_W_TILED the five projection matrices are stored in the order in which the matrix-core
 *    projections read them: matrix [N][K] (N % 128 == 0, K % 64 == 0) as [N/128 row tiles][K/64 slabs] units, a unit
 *    being the 128 x 64 elements of one tile and slab, contiguous (16 KiB of bf16, 8 KiB of int8 codes), inside a unit
 *    bf16: [4 waves][2 row groups][2 k halves][64 lanes][8 elements], lane l holding row 32*wave + 16*group + l%16,
 *    elements 32*half + 8*(l/16) .. +7 of the slab; int8: [4 waves][2 row groups][64 lanes][16 codes], lane l holding
 *    row 32*wave + 16*group + l%16, codes 16*(l/16) .. +15.  A workgroup then streams contiguous memory instead of 128
 *    rows that lie 2*K bytes apart (measured: 20-27 % faster on 59-235 MB matrices).  psv_tile_weights
 *    (preserve_aux.h) converts a row-major matrix.  Same bytes, same results bit for bit; a context with tiled weights
 *    runs the matrix-core projections at every batch size (the batch-1 kernels want whole rows).
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
enum { PSV_KV_HEAD_MAJOR = 0u, PSV_KV_TOKEN_MAJOR = 1u };
enum { PSV_W_ROW_MAJOR = 0u, PSV_W_TILED = 1u };

typedef int32_t psv_status;
enum {
    PSV_OK = 0,
    PSV_ERR_INVALID_ARG = -1,   /* null pointer, size out of range, inconsistent descriptor */
    PSV_ERR_BAD_STATE = -2,     /* e.g. decode step before weights / KV were set */
    PSV_ERR_UNSUPPORTED = -3,   /* shape outside what the kernels are built for */
    PSV_ERR_HIP = -4,           /* a HIP runtime call failed (also: no GPU present) */
    PSV_ERR_NOMEM = -5,         /* host or device allocation failed */
    PSV_ERR_TIMEOUT = -6        /* a kernel launched ahead of its communication window (policy.prelaunch) gave up its
                                   bounded wait for the window's end; reported once, by psv_sync.  (A matrix-core
                                   projection launched that way waits for its activations as well: giving up
                                   invalidates the step and is reported as PSV_ERR_HIP.) */
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
    uint32_t kv_layout;     /* PSV_KV_HEAD_MAJOR (default) or PSV_KV_TOKEN_MAJOR (bf16 cache only): see the conventions */
    uint32_t weight_layout; /* PSV_W_ROW_MAJOR (default) or PSV_W_TILED: see the conventions */
} psv_model_desc;

/* dev pointers; projection matrices in the descriptor's weight_format and weight_layout (shapes below: rows x columns),
 * gains bf16 */
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
                                every window.  Takes effect at batch 1 (and batch 2 up to H = 4096) for both
                                windows when the plan hands them the operator whole; with the matrix-core
                                projections (larger batches, or tiled weights) at batch <= 32 (int8 weights: 16)
                                for the gate/up projection when the plan hands its window any of it and all
                                its workgroups fit the device at once -- that kernel also walks the window's
                                prefetch job, keeps its first weight slabs in registers and LDS, and waits
                                for the residual kernel that follows the window; and only on a context whose
                                two streams run concurrently
                                -- i.e. after psv_check_overlap (preserve_aux.h) has been called on the
                                context and answered 1: a kernel that waits on a flag must never sit in front of the
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
    uint32_t kernels_per_layer;        /* launches of the operator chain per layer, windows included: counted on the last
                                          step, before the first one an estimate from the shape */
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

/* Creates a context on the current HIP device.  The two streams are Section 3's ("PRESERVE") execution
 * model: the operators of the step run in order on stream_main, the prefetch operators that Algorithm 1
 * inserted run on stream_side beside the communication operator they were attached to.  Both are hipStream_t
 * handles owned by the caller; they must differ and have default priority.  Allocates the workspace
 * (psv_workspace_bytes) with hipMalloc.  *out is set only on success. */
psv_status psv_create(const psv_model_desc *desc, void *stream_main, void *stream_side,
                      psv_ctx **out);
/* Frees the context and its workspace.  The caller synchronises first (psv_sync). */
psv_status psv_destroy(psv_ctx *ctx);

/* The operands of one layer's five MatMul nodes (Section 2, "LLM inference workloads": QKV, output, and the
 * three MLP projections) and its two norm gains; they are also what a prefetch operator of class "weights"
 * reads.  Borrowed until replaced or psv_destroy; pointers must be 16-byte aligned. */
psv_status psv_set_layer_weights(psv_ctx *ctx, uint32_t layer, const psv_layer_weights *w);
/* The KV-cache every SelfAttention node reads and appends to (Section 3, "Execution with the proposed method":
 * all of it except the newest entry is known before the step and can be prefetched).  The host arrays of pool
 * pointers are copied; pools, page table and seq_lens are borrowed.  max_blocks * 16 >= the descriptor's
 * max_seq; without a page table num_pool_blocks >= max_batch * max_blocks. */
psv_status psv_set_kv(psv_ctx *ctx, const psv_kv_desc *kv);

/* Durations of the two communication operators of every layer (Section 2, "Multi-device inference": one
 * allreduce after the attention block, one after the MLP block), microseconds (0 <= us <= 1e6); each is
 * executed as a spin kernel of that length standing in for the collective.  A window of 0 launches neither
 * the spin kernel nor any prefetch. */
psv_status psv_set_comm_windows(psv_ctx *ctx, float us_after_attn, float us_after_mlp);

/* Stores the policy and runs Algorithm 1 (Section 3, "Operator insertion") for (batch, context): its inputs
 * are the operator graph, fixed by the descriptor, the capacity C = policy->budget_bytes, and memSize() of
 * every node, which for SelfAttention depends on batch and on context, the attention span.  Pure host work:
 * nothing is launched. */
psv_status psv_set_policy(psv_ctx *ctx, const psv_prefetch_policy *policy, uint32_t batch,
                          uint32_t context);

/* Copies the current plan (see psv_plan_chain) to host memory. */
psv_status psv_plan(psv_ctx *ctx, psv_plan_entry *out, size_t cap, size_t *n);

/*
 * One decode step over layers [layer_begin, layer_end): Section 3's execution with (policy
 * mode 1) or without (mode 0) prefetching.  x_in, x_out: dev fp32 [batch, H] (may alias).
 * Asynchronous: returns after enqueueing on stream_main / stream_side.  Mutates only x_out,
 * slot seq_lens[b]-1 of each layer's K and V pools, and the workspace.  The results are bit
 * identical for every policy and window.
 */
psv_status psv_decode_step(psv_ctx *ctx, const float *x_in, float *x_out, uint32_t batch,
                           uint32_t layer_begin, uint32_t layer_end);

/* Waits for both streams (the event synchronisation between the two streams of Section 3, "PRESERVE", seen
 * from the host).  PSV_ERR_HIP if any enqueued work failed -- also, once, if a hand-over inside a fused kernel
 * (psv_set_fused_kernels, preserve_aux.h) ran out of its bound: that step's results are invalid, the context stays
 * usable; PSV_ERR_TIMEOUT, once, if a kernel launched ahead of its window gave up waiting for the window's end (it
 * still finished with the right result; the context stays usable). */
psv_status psv_sync(psv_ctx *ctx);

/* Algorithmic bytes of the step as Section 2 ("LLM decoding is memory BW-limited") counts them -- every weight
 * once, K and V of the attended span once -- and what the current plan prefetches. */
psv_status psv_get_stats(psv_ctx *ctx, psv_stats *out);

/* ---- for callers that cannot allocate ------------------------------------------------------- */

/* For callers that cannot call hipMalloc -- code under HIP graph capture, tight serving loops, harnesses that
 * forbid it: psv_decode_step without a context.  One decode step over layers [layer_begin, layer_end) in vanilla
 * execution (no communication stand-in, no prefetch), enqueued on `stream` (hipStream_t), with the workspace that
 * psv_create would allocate held in a fixed device array of PSV_STATIC_SCRATCH_BYTES inside the library instead.
 * The call allocates no device memory and creates no stream or event (its host-side bookkeeping is a few small
 * heap vectors).  layers: host array [desc->n_layers] (only the entries of the range are read); kv, x_in, x_out,
 * batch: as for psv_set_kv / psv_decode_step; the results are those of psv_decode_step with the policy off, both
 * windows 0 and one kernel per operator (psv_set_fused_kernels 0, preserve_aux.h), bit for bit.  PSV_ERR_UNSUPPORTED if psv_workspace_bytes(desc) exceeds PSV_STATIC_SCRATCH_BYTES.
 * Every call on a GPU shares that GPU's one array, which keeps the previous call's contents (nothing in it has to
 * start at zero): calls that overlap on one GPU -- from two streams or two threads -- race; serialise them.  The
 * array (one per GPU the library runs on) stays allocated until the process ends. */
#define PSV_STATIC_SCRATCH_BYTES (16u << 20)
psv_status psv_decode_step_static(const psv_model_desc *desc, const psv_layer_weights *layers,
                                  const psv_kv_desc *kv, const float *x_in, float *x_out, uint32_t batch,
                                  uint32_t layer_begin, uint32_t layer_end, void *stream);

#ifdef __cplusplus
}
#endif
#endif

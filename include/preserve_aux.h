/*
 * libpreserve_mi355x -- auxiliary entry points: stream checks, tuning, measurement aids and test hooks.
 *
 * None of these is part of the decode-step contract of preserve.h (create / set / plan / step / sync / stats);
 * they exist for the benchmark, the profiler runs and the tests.  Same conventions as preserve.h: every call
 * returns a psv_status, nothing throws or prints, "dev" pointers are HIP device pointers.
 */
#ifndef PRESERVE_AUX_H
#define PRESERVE_AUX_H

#include "preserve.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ---- execution mode ------------------------------------------------------------------------ */

/* 0 = launch kernels one by one on the two streams (the only mode).  1 asked for capturing the step into a HIP
 * graph and replaying it; that mode is retired and 1 is always answered with PSV_ERR_UNSUPPORTED: on this
 * runtime a captured side branch did not overlap its window (slower than eager launches with prefetching on),
 * and test runs that went through many capture / replay / destroy cycles ended, rarely, in an abort inside the
 * HIP runtime whose cause was not found. */
psv_status psv_set_graph_mode(psv_ctx *ctx, uint32_t use_graph);

/* 0 = one kernel per operator; 1 = at batch 1, where the shape allows it (bf16 cache, sequences up to 4096
 * tokens), the operators between two communication windows run as one fused kernel each (QKV + attention + O;
 * gate/up + down) whose phases hand their results over through tagged values in memory.  Faster by ~3 us per layer
 * on an 8B-shaped shard when the kernels are launched into the windows (policy.prelaunch), slower otherwise.  The two
 * settings agree to rounding, not bit for bit; within one setting every policy gives the same bits.  A hand-over that
 * does not complete within its bound makes the next psv_sync return PSV_ERR_HIP.
 * 2 = under the same conditions (and every projection at least as many rows as the device has thread groups) the whole
 * step is ONE kernel: resident workgroups walk the layers, the residual stream stays in registers, the communication
 * windows are timed inside the kernel, and what the plan hands to a window whole is requested into registers before the
 * window's end (nothing runs on the side stream; an operator the plan covers only in part is not requested early).
 * Shapes it does not take run as under 1.  Per-operator profiling sees one kernel (reported as the QKV operator).
 * 3 (default) = the library chooses by shape between 0 and 1: 1 where rows have at least 4096 elements and all
 * weights of a block fit the registers of one pass (an 8B-shaped TP=8 shard does), 0 elsewhere.
 * psv_decode_step_static always runs as under 0.
 * Kernels of settings 1 and 2 need every one of their workgroups resident at once (one per compute unit): while such a
 * step runs, nothing else that holds compute units for long may run on the device -- in particular not a step of
 * another context -- or their hand-overs run out of patience and psv_sync reports PSV_ERR_HIP.  The library's own
 * window and prefetch kernels are short or single-workgroup and are accounted for. */
psv_status psv_set_fused_kernels(psv_ctx *ctx, uint32_t on);

/* ---- streams and tuning -------------------------------------------------------------------- */

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
 * side stream).  The context remembers the answer: policy.prelaunch stays without effect unless this call has been
 * made and answered 1.
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

/* Rewrites a row-major projection matrix [rows][cols] (dev, bf16 or int8 codes per `weight_format`) into the tiled
 * layout of PSV_W_TILED (preserve.h) at dst (dev, same size, must not overlap src); rows % 128 == 0, cols % 64 == 0,
 * both pointers 16-byte aligned.  Row scales of an int8 matrix are not touched (they stay one per row).  Asynchronous
 * on `stream`. */
psv_status psv_tile_weights(void *dst, const void *src, uint32_t rows, uint32_t cols, uint32_t weight_format, void *stream);

/* Test aid for the bounded waits: while on, a kernel launched ahead of its window's end gives up its (always bounded)
 * wait at once -- it still completes with the right result, sets an error word, and the next psv_sync returns
 * PSV_ERR_TIMEOUT once; a matrix-core projection launched that way reads activations that are not there yet, the step's
 * output is invalid and the next psv_sync returns PSV_ERR_HIP once -- and every hand-over inside a fused kernel (psv_set_fused_kernels) expires at once: those
 * kernels run to their end on whatever their buffers held, the step's output and the cache rows it appends are
 * invalid, and the next psv_sync returns PSV_ERR_HIP once.  The context stays usable either way. */
psv_status psv_debug_force_wait_timeout(psv_ctx *ctx, uint32_t on);

/* Which kernels the most recent psv_decode_step ran: 0 = one per operator, 1 = at least one block as a fused kernel,
 * 2 = the whole step as one kernel (psv_set_fused_kernels asks; the shape decides). */
psv_status psv_debug_last_step_path(psv_ctx *ctx, uint32_t *path);
/* How many first consumers the most recent psv_decode_step launched into their communication windows (policy.prelaunch;
 * per-operator and per-block kernels -- the whole-step kernel has its windows inside and reports 0). */
psv_status psv_debug_last_step_prelaunches(psv_ctx *ctx, uint32_t *count);

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

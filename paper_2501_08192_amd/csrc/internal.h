// Internal interface between the host side of libpreserve_mi355x (api.cpp, executor.cpp, planner.cpp) and
// its gfx950 kernels (gemv.hip, gemm_sk.hip, attention.hip, window.hip).  Launch wrappers take plain
// pointers and sizes, validate nothing (the API layer has already done so) and return the hipError_t
// of the launch.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/preserve.h"

namespace psv {

// ---- attention work split ---------------------------------------------------------------
// One 64-lane wave consumes the KV-cache in tiles of 32 tokens; a workgroup has 4 waves, so a
// workgroup's chunk is a multiple of 128 tokens.  Every wave writes its own partial result.
constexpr int kAttnTileTokens = 32;       // tokens per wave and loop step, bf16 cache
constexpr int kAttnTileTokensInt8 = 64;   // int8 cache
constexpr int kAttnWaves = 4;
constexpr int kAttnMaxChunks = 256;
constexpr int kAttnResident = 448;      // workgroups the default split aims at: one round that leaves every CU a little slack

struct AttnSplit {
    int chunk_tokens;   // tokens per workgroup
    int n_chunks;       // workgroups along the sequence (grid.x) = partial results per (sequence, kv head)
};
AttnSplit attn_split(uint32_t batch, uint32_t n_kv_heads, uint32_t max_seq, bool kv_int8);

struct KvView {
    uint16_t *k_pool;            // bf16 pool, or (int8 != 0) byte pool of PSV_KV_UNIT_BYTES_INT8 units
    uint16_t *v_pool;
    int int8;
    int token_major;             // bf16 pools laid out [block][16 tokens][kv head][128] (both K and V)
    const int32_t *page_table;   // null => contiguous
    int max_blocks;
    int max_tokens;              // longest valid sequence: min(max_blocks * 16, the descriptor's max_seq); the
                                 //   attention grid and its partial buffers are sized for it
    int num_pool_blocks;
    const int32_t *seq_lens;
};

// Operand of a matrix-core projection as its producer stores it (the `x_bf16` / `out_bf16` arguments below):
// two bf16 planes (hi, lo; x = hi + lo) of [round_up(batch,16)][K] elements for bf16 weights, or -- `digits` --
// for int8 weights two int8 digit planes of the same shape followed by one fp32 scale per 128 elements of a row.
// Both fit the same buffer of 4 * round_up(batch,16) * K bytes.

// A projection matrix in either storage format: bf16 [rows][cols] (scale == nullptr), or int8 codes
// [rows][cols] with one fp32 scale per row.
struct Mat {
    const void *w = nullptr;
    const float *scale = nullptr;
    bool tiled = false;          // PSV_W_TILED storage (matrix-core projections only)
};

// ---- kernel launchers ---------------------------------------------------------------------

// The next kernel launched from this thread records `start` / `stop` around its own execution.
void set_launch_events(hipEvent_t start, hipEvent_t stop);

// Vector-ALU GEMV for batch <= 2:  out[b][r] = sum_k W[r][k] * x[b][k]   (fp32 x; W bf16 or int8 + row scale).
// W2.w != null selects the SwiGLU form: out[b][r] = silu(W[r].x[b]) * (W2[r].x[b]); same format as W.
hipError_t launch_gemv(Mat W, Mat W2, const float *x, float *out, int batch, int N, int K, hipStream_t s);
// Same with the activations formed in the prologue: x = rmsnorm(res + delta) * gain.  out_res
// receives res + delta and out_h (optional) the normalised vector; neither may alias res or delta.
// wait != null: the kernel is launched before its inputs exist.  It requests its first weights, then waits
// (bounded) until *done has reached seq -- published by the window kernel when the window ends -- and only
// then reads res / delta.  A wait that hits its bounds sets *err and the kernel continues.
struct GemvWait {
    const unsigned *done;
    unsigned seq;
    uint32_t iters;
    uint64_t ticks;
    unsigned *err;
};
hipError_t launch_gemv_norm(Mat W, Mat W2, const float *res, const float *delta,
                            const uint16_t *gain, float eps, float *out_res, float *out_h, float *out, int batch,
                            int N, int K, const GemvWait *wait, hipStream_t s);
bool gemv_supported(int batch, int N, int K);
// O projection with the attention merge in its prologue: x = merged split-K partials (K = nq*128).
// out_attn (optional) receives the merged attention output.  Usable for few chunks only.
constexpr int kGemvMergeMaxChunks = 16;
bool gemv_merge_supported(int batch, int nq, int n_chunks);
hipError_t launch_gemv_merge(Mat W, const float *part_ml, const float *part_o, int nq, int nkv,
                             int n_chunks, float *out_attn, float *out, int batch, int N, hipStream_t s);

// ---- fused kernels of the vector path (segment.hip): all operators between two communication windows in one launch
// of `blocks` workgroups (one per CU, all resident).  Phases hand their results over through buffers of tagged values
// ({value, tag} pairs, 8 bytes each); `tag` must be unique per launch (next_tag).  *err: bit 0 = the wait for the
// window's end expired (wait != null), bit 1 = a hand-over poll expired (results invalid).
constexpr uint32_t kSegPollIters = 1u << 16;
unsigned next_tag();
constexpr int kSegIndCopies = 8, kSegIndStride = 512;    // indicator entries behind m_ll: copies x workgroups (launch_seg_mlp)
// MLP block: y = res + delta; h = rmsnorm(y) * gain; m = silu(Wg h) * (Wu h); out = Wd m.  m: [batch][F] floats (the kernel's
// own hand-over buffer); m_ll: [batch][F] pairs (unused here) followed by kSegIndCopies x kSegIndStride indicator pairs (blocks <= kSegIndStride).
// wait != null: launched into the window ahead of its inputs, see GemvWait; hold_down = false makes that variant
// request the down weights only after the window's end (the plan did not hand them to this window).
// poll_iters: bound of every hand-over poll (kSegPollIters; 0 makes every hand-over expire at once -- a test aid).
bool seg_mlp_supported(int batch, int H, int F);
// do the first passes of the gate/up and of the down projection (what the kernel requests at its start) cover all of
// W_gate and W_up / all of W_down?
bool seg_mlp_holds_gate_up(int H, int F, bool w8, int blocks);
bool seg_mlp_holds_down(int H, int F, bool w8, int blocks);
hipError_t launch_seg_mlp(Mat Wg, Mat Wu, Mat Wd, const float *res, const float *delta, const uint16_t *gain, float eps,
                          float *out_res, float *out_h, float *m, void *m_ll, float *out, int batch, int H, int F, unsigned tag,
                          unsigned *err, const GemvWait *wait, bool hold_down, uint32_t poll_iters, int blocks, hipStream_t s);

// Attention block of one sequence: x = res + delta; h = rmsnorm(x) * gain; qkv = Wq h; rotary embedding, KV append and
// decode attention over 256-token chunks (workgroup kvh * n_chunks + c runs chunk c of kv head kvh); out = Wo attn.
// qkv_ll: [QR] pairs; pml: [nkv][n_chunks][16] (max, sum) float pairs and po: [nkv][n_chunks][G][128] floats
// (plain data, the kernel's own); ind_ll: kSegIndCopies x kSegIndStride indicator pairs (one entry per partial in every copy).  bf16 cache only.
// hold_kv / hold_o: see hold_down.
int seg_attn_chunks(uint32_t max_seq);
bool seg_attn_supported(int batch, int H, int nq, int nkv, uint32_t max_seq, bool kv_int8, int blocks);
bool seg_attn_holds_o(int H, int nq, bool w8, int blocks);      // the first pass of the O projection covers all of W_o
bool seg_attn_holds_qkv(int H, int QR, bool w8, int blocks);    // ... of the QKV projection all of W_qkv
hipError_t launch_seg_attn(Mat Wq, Mat Wo, const float *res, const float *delta, const uint16_t *gain, float eps,
                           float *out_res, float *out_h, void *qkv_ll, const float2 *rope, KvView kv, int nq, int nkv,
                           int n_chunks, void *pml, void *po, void *ind_ll, float *out_attn, float *out, int H, unsigned tag,
                           unsigned *err, const GemvWait *wait, bool hold_kv, bool hold_o, uint32_t poll_iters, int blocks, hipStream_t s);

// ---- the whole step of one sequence as one kernel (step.hip): `blocks` resident workgroups walk layers [lb, le); the
// residual stream stays in registers, every hand-over is a buffer of tagged values, and the communication windows
// are timed inside the kernel (the last workgroup computes nothing: it waits for a block's whole output, spins `ticks`
// of the wall clock and publishes the window's end).
// hold[w]: what is requested into registers before the end of window w (0: after the attention block, 1: after the
// MLP block) instead of after it -- bit 0 the first projection of the next block, then [0] bit 1 down, [1] bit 1 the
// K/V tiles and bit 2 O; a window of 0 ticks does not exist and everything is requested up front.
// layer_table: device array of kStepLayerBytes per layer of the model (index = layer): pointers Wq, Wo, Wg, Wu, Wd,
// their int8 row scales sq, so, sg, su, sd, the gains g_attn, g_mlp and the layer's K and V pools.
// ll_base: (2 * H + 2) pairs for the two projection outputs and the two window-end words.  Tags tag_base ..
// tag_base + 8 * (le - lb) - 1 must be unused by any other launch (next_tags).
constexpr size_t kStepLayerBytes = 14 * sizeof(void *);
unsigned next_tags(unsigned n);
struct StepLaunch {
    const void *layer_table;
    int lb, le;
    const float *x_in;
    float *x_out;
    int H, F, nq, nkv, n_chunks;
    bool w8;
    float eps;
    const float2 *rope;
    KvView kv;
    void *qkv_ll, *pml_ll, *po_ll, *m_ll, *ll_base;
    unsigned tag_base;
    unsigned *err;
    uint64_t ticks[2];
    uint32_t spin_iters[2];
    uint32_t poll_iters;      // bound of every hand-over poll (kSegPollIters / 4; 0: a test aid, see launch_seg_mlp)
    int hold[2];
    float *dbg_x, *dbg_h1, *dbg_attn, *dbg_y, *dbg_h2;   // intermediates of the last layer (optional)
};
bool step_supported(int batch, int H, int F, int nq, int nkv, uint32_t max_seq, bool other_cache, bool w8, int blocks);
hipError_t launch_step(const StepLaunch &p, int blocks, hipStream_t s);

// Split-K skinny GEMM on the matrix cores with the activation slab shared through LDS:
// part[split][b][r] = partial sums of W[r].x[b] (rows >= split_row come from W2), to be summed in split
// order by launch_sk_reduce or launch_resid_sum.  x_bf16: see the operand formats above.
constexpr int kSkMaxSplits = 16;
int gemm_sk_splits(int batch, int N, int K, bool w8, bool tiled);
bool gemm_sk_supported(int batch, int N, int K);
// ssq != null (K % 512 == 0): x_bf16 holds x * gain without the 1/rms factor of its RMSNorm and ssq the partial
// sums of squares [batch][K / 512] written by launch_resid_sum; the result is multiplied by 1/rms of its batch row.
// wait != null (ssq != null, one batch tile): launched into a communication window ahead of its activations, on another
// stream than the launch_resid_sum that produces them, which is given the same SkWait as its signal.
constexpr int kSkWaitMaxBatch = 32;      // one or two batch tiles (bf16 weights; int8: one)
constexpr int kSkWaitEntries = 1024;     // batch * K / 512 of a projection launched that way
constexpr int kSkTagCopies = 8;         // the tagged sums of squares are published in that many copies; a waiting workgroup polls one
inline size_t sk_tag_stride(int batch, int K) { return ((size_t)batch * (K / 512) + 511) / 512 * 512; }   // entries from copy to copy
struct SkWait {
    void *ssq_ll;            // tagged sums of squares: kSkTagCopies copies of [K / 512][batch] x 8 bytes, sk_tag_stride entries apart
    unsigned tag;            // of this launch pair (next_tag)
    const unsigned *win_done;   // launch_gemm_sk: end word of the window and the value it takes then (GemvWait::done, seq)
    unsigned win_seq;
    uint32_t iters;          // bounds of the wait, as in GemvWait
    uint64_t ticks;
    unsigned *err;
    double share_w, share_w2;   // launch_gemm_sk: planned fraction (0..1) of W and of W2 that the kernel prefetches for itself
    const struct PrefetchJob *job;   // launch_gemm_sk: what else it prefetches while it waits (may be null)
};
hipError_t launch_gemm_sk(Mat W, Mat W2, int split_row, const uint16_t *x_bf16, const float *ssq, float eps,
                          float *part, int batch, int N, int K, const SkWait *wait, hipStream_t s);
// May that projection be launched with a wait on a device of `cus` compute units (its waiting workgroups leave room
// for the kernel they wait for)?
bool gemm_sk_can_wait(int batch, int N, int K, bool w8, bool tiled, int cus);
// out_res = res + delta (delta: null, or `delta_splits` split-K partials summed in split order), one float4 per
// thread over grid (H / 512, batch).  gain != null: also out_res * gain as hi/lo bf16 planes (xg_bf16, lo plane
// plane_stride elements after the hi plane) and the sums of squares per workgroup, ssq[batch][H / 512].
hipError_t launch_resid_sum(const float *res, const float *delta, int delta_splits, int batch, int H, float *out_res,
                            const uint16_t *gain, uint16_t *xg_bf16, size_t plane_stride, bool digits, float *ssq,
                            const SkWait *signal, hipStream_t s);
// signal != null (gain != null): every output is written through to the memory side and each workgroup's
// sum of squares is published as a tagged value in signal->ssq_ll once its other stores are acknowledged.
// out = sum of the splits; swiglu: N = gate | up columns, out = silu(gate) * up of width N/2.  out_bf16
// (optional) receives hi/lo planes.
hipError_t launch_sk_reduce(const float *part, int splits, int batch, int N, bool swiglu, float *out,
                            uint16_t *out_bf16, bool digits, hipStream_t s);

// cos/sin of the rotary angles at position seq_len-1: table [batch][64] (inv_freq null => identity).
hipError_t launch_rope_table(const int32_t *seq_lens, const double *inv_freq, int max_tokens, int batch,
                             float2 *table, hipStream_t s);

// Decode attention: RoPE of q, KV append and split-K partials (max, sum, weighted V) per workgroup ...
hipError_t launch_attn(const float *qkv, const float2 *rope, KvView kv, int batch, int nq, int nkv, AttnSplit sp,
                       float *part_ml, float *part_o, hipStream_t s);
// ... and the fixed-order merge of the partials into out_f32 and the hi/lo bf16 planes out_bf16.
hipError_t launch_attn_merge(const float *part_ml, const float *part_o, int batch, int nq, int nkv, AttnSplit sp,
                             float *out_f32, uint16_t *out_bf16, bool digits, hipStream_t s);

// Communication stand-in: one workgroup busy-waits `ticks` of the constant-rate wall clock.
// `flag` (optional): the kernel stores `seq` there on entry, which releases the gate of this window; `done`
// (optional): it stores `seq` there when the window ends, which releases a consumer launched ahead of time.
hipError_t launch_spin(uint64_t ticks, uint32_t max_iters, unsigned *flag, unsigned *done, unsigned seq, hipStream_t s);

// Prefetch: everything one communication window pulls towards the cache, in one launch.
constexpr int kPrefetchRegions = 6;
struct PrefetchJob {
    const void *ptr[kPrefetchRegions];   // linear regions (projection weights), 16-byte aligned
    uint64_t n16[kPrefetchRegions];      // their sizes in 16-byte words
    int n_regions;
    int nkv;
    KvView kv;                           // KV range: logical blocks [kv_first, kv_first + kv_count) of the
    uint32_t blocks_per_seq;             //   flattened (sequence, block) order, blocks_per_seq per sequence
    uint64_t kv_first, kv_count;
    const unsigned *skip;                // optional: word written by the gate kernel; non-zero => do nothing
};
// One-wave gate on the side stream: returns when *flag has reached seq (or the bounds expire) and
// writes *skip = 1 if *flag is already beyond seq.
hipError_t launch_gate(const unsigned *flag, unsigned seq, uint32_t wait_iters, uint64_t wait_ticks, unsigned *skip,
                       hipStream_t s);
hipError_t launch_prefetch_job(const PrefetchJob &j, uint32_t workgroups, hipStream_t s);
hipError_t launch_prefetch(const void *ptr, uint64_t bytes, uint32_t workgroups, hipStream_t s);

hipError_t launch_copy(void *dst, const void *src, uint64_t bytes, hipStream_t s);
// row-major [rows][cols] -> the tiled layout of PSV_W_TILED; elem_bytes = 2 (bf16) or 1 (int8 codes)
hipError_t launch_tile_weights(void *dst, const void *src, int rows, int cols, int elem_bytes, hipStream_t s);

// ---- planner (pure host) ---------------------------------------------------------------------
uint64_t op_mem_size(const psv_model_desc &d, uint32_t op, uint32_t batch, uint32_t context);
size_t plan_chain(const psv_model_desc &d, uint32_t batch, uint32_t context,
                  const psv_prefetch_policy &p, psv_plan_entry *out, size_t cap);

}  // namespace psv

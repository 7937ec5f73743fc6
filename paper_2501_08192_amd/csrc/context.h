// Context of libpreserve_mi355x: what a psv_ctx holds, the layout of its workspace, and the interface between
// the C entry points (api.cpp) and the step executor (executor.cpp).
#pragma once

#include <stddef.h>
#include <stdint.h>

#include <utility>
#include <vector>

#include "internal.h"

namespace psv {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Workspace {
    size_t total = 0;
    // offsets
    size_t x, y, h1_f32, h1_bf16, h2_f32, h2_bf16, qkv, rope, part_ml, part_o, attn_f32, attn_bf16,
        delta_a, delta_m, m_f32, m_bf16, inv_freq, flag, part, ssq, ssq_ll, m_ll, qkv_ll, pml_ll, po_ll, step_tbl, step_ll, seg_ind, seg_pml, seg_po, seg_m;
};

Workspace layout_workspace(const psv_model_desc &d);

}  // namespace psv

struct psv_ctx {
    psv_model_desc d{};
    hipStream_t main = nullptr, side = nullptr;
    int device = 0;
    uint64_t clock_khz = 100000;
    psv::Workspace ws{};
    char *wsp = nullptr;
    std::vector<psv_layer_weights> weights;
    std::vector<unsigned char> weights_set;
    bool kv_set = false;
    std::vector<void *> k_pools, v_pools;
    psv_kv_desc kv{};
    float window_us[2] = {0.f, 0.f};
    psv_prefetch_policy policy{};
    uint32_t plan_batch = 0, plan_context = 0;
    std::vector<psv_plan_entry> plan;
    std::vector<hipEvent_t> ev_join;             // [layer*2 + window], policy.join
    hipEvent_t ev_end = nullptr;
    int32_t profile_op = -1;
    std::vector<hipEvent_t> prof_events;         // pool, one per profiled launch
    size_t prof_next = 0;
    hipEvent_t prof_last = nullptr;              // event of the previous main-stream kernel
    std::vector<std::pair<hipEvent_t, hipEvent_t>> prof_pairs;
    uint32_t steps = 0;
    uint32_t last_prefetch_launches = 0;
    uint32_t step_launches = 0, step_layers = 0; // launches of the operator chain in the last step (windows included), and its layers
    uint32_t last_step_prelaunches = 0;          // consumers the last step launched into their windows
    unsigned window_seq = 0;                     // sequence number of the last communication window enqueued
    uint32_t attn_chunk_tokens = 0;               // 0 = default split; else tokens per attention workgroup (psv_tune_attention)
    int overlap = -1;                            // psv_check_overlap's last answer (-1 = not run yet)
    bool check_err_word = false;                 // a kernel that may set the error word (a pre-launched consumer, a fused kernel) was launched: read it at sync
    int fused = 3;                               // psv_set_fused_kernels: 0 one kernel per operator, 1 one per block, 2 one per step, 3 by shape
    bool step_tbl_dirty = true;                  // the per-layer pointer table of the whole-step kernel has to be uploaded again
    std::vector<unsigned char> step_tbl_host;    // ... its host copy (kept alive until the upload has run)
    bool force_wait_timeout = false;             // test aid: such consumers give up waiting at once (and report it)
    bool last_step_vec = false;                  // the last step formed h1 / h2 (vector path)
    bool last_step_seg_attn = false;             // ... the attention block (qkv lives in the tagged buffer)
    bool last_step_seg_mlp = false;              // ... and ran the MLP block as one fused kernel (m lives in the tagged buffer)
    bool last_step_whole = false;                // ... or the whole step as one kernel
    int cus = 0;                                 // compute units of the device = workgroups of a fused kernel (0: fused kernels off)

    template <class T> T *at(size_t off) const { return reinterpret_cast<T *>(wsp + off); }
};

#define HIP_TRY(expr)                        \
    do {                                     \
        hipError_t e__ = (expr);             \
        if (e__ != hipSuccess) return PSV_ERR_HIP; \
    } while (0)

#define ST_TRY(expr)                      \
    do {                                  \
        psv_status st__ = (expr);         \
        if (st__ != PSV_OK) return st__;  \
    } while (0)

namespace psv {

AttnSplit ctx_split(const psv_ctx *c);       // attention split in force (default or tuned)
uint64_t us_to_ticks(uint64_t clock_khz, float us);
uint32_t spin_cap(float us);
psv_status rebuild_plan(psv_ctx *c);
// Enqueues one decode step over layers [lb, le) on the context's two streams.
psv_status enqueue_step(psv_ctx *c, const float *x_in, float *x_out, uint32_t batch, uint32_t lb, uint32_t le);

}  // namespace psv

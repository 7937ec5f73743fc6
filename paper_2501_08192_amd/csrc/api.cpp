// C entry points of libpreserve_mi355x (include/preserve.h, include/preserve_aux.h): argument checks, context life
// cycle, setters, the decode step, synchronisation, statistics and the measurement aids.
#include <cstdlib>
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <chrono>
#include <new>
#include <utility>
#include <vector>

#include "context.h"
#include "../../include/preserve_aux.h"

using namespace psv;

extern "C" {

size_t psv_workspace_bytes(const psv_model_desc *desc)
{
    if (psv_validate_desc(desc) != PSV_OK) return 0;
    return layout_workspace(*desc).total;
}

psv_status psv_create(const psv_model_desc *desc, void *stream_main, void *stream_side, psv_ctx **out)
{
    if (!desc || !out) return PSV_ERR_INVALID_ARG;
    if (psv_validate_desc(desc) != PSV_OK) return PSV_ERR_INVALID_ARG;
    if (stream_main == stream_side) return PSV_ERR_INVALID_ARG;
    psv_ctx *c = new (std::nothrow) psv_ctx();
    if (!c) return PSV_ERR_NOMEM;
    c->d = *desc;
    c->main = static_cast<hipStream_t>(stream_main);
    c->side = static_cast<hipStream_t>(stream_side);
    auto fail = [&](psv_status st) { psv_destroy(c); return st; };
    if (hipGetDevice(&c->device) != hipSuccess) return fail(PSV_ERR_HIP);
    int khz = 0;
    if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, c->device) == hipSuccess && khz > 0) c->clock_khz = (uint64_t)khz;
    if (hipDeviceGetAttribute(&c->cus, hipDeviceAttributeMultiprocessorCount, c->device) != hipSuccess) c->cus = 0;
    c->ws = layout_workspace(c->d);
    if (hipMalloc(reinterpret_cast<void **>(&c->wsp), c->ws.total) != hipSuccess) {
        c->wsp = nullptr;
        return fail(PSV_ERR_NOMEM);
    }
    if (hipMemset(c->wsp, 0, c->ws.total) != hipSuccess) return fail(PSV_ERR_HIP);
    if (c->d.rope_theta > 0.f) {
        double f[64];
        for (int i = 0; i < 64; ++i) f[i] = pow((double)c->d.rope_theta, -2.0 * (double)i / 128.0);
        if (hipMemcpy(c->wsp + c->ws.inv_freq, f, sizeof f, hipMemcpyHostToDevice) != hipSuccess) return fail(PSV_ERR_HIP);
    }
    c->weights.resize(c->d.n_layers);
    c->weights_set.assign(c->d.n_layers, 0);
    c->k_pools.assign(c->d.n_layers, nullptr);
    c->v_pools.assign(c->d.n_layers, nullptr);
    c->ev_join.assign((size_t)c->d.n_layers * 2, nullptr);
    for (size_t i = 0; i < c->ev_join.size(); ++i)
        if (hipEventCreateWithFlags(&c->ev_join[i], hipEventDisableTiming) != hipSuccess) return fail(PSV_ERR_HIP);
    if (hipEventCreateWithFlags(&c->ev_end, hipEventDisableTiming) != hipSuccess) return fail(PSV_ERR_HIP);
    c->policy.mode = 0;
    c->policy.targets = PSV_TARGET_WEIGHTS | PSV_TARGET_KV;
    *out = c;
    return PSV_OK;
}

psv_status psv_destroy(psv_ctx *c)
{
    if (!c) return PSV_ERR_INVALID_ARG;
    for (hipEvent_t e : c->ev_join) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->prof_events) if (e) (void)hipEventDestroy(e);
    if (c->ev_end) (void)hipEventDestroy(c->ev_end);
    if (c->wsp) (void)hipFree(c->wsp);
    delete c;
    return PSV_OK;
}

psv_status psv_set_layer_weights(psv_ctx *c, uint32_t layer, const psv_layer_weights *w)
{
    if (!c || !w || layer >= c->d.n_layers) return PSV_ERR_INVALID_ARG;
    if (!w->w_qkv || !w->w_o || !w->w_gate || !w->w_up || !w->w_down || !w->g_attn || !w->g_mlp) return PSV_ERR_INVALID_ARG;
    const void *ptrs[7] = {w->w_qkv, w->w_o, w->w_gate, w->w_up, w->w_down, w->g_attn, w->g_mlp};
    for (const void *p : ptrs)
        if (reinterpret_cast<uintptr_t>(p) % 16 != 0) return PSV_ERR_INVALID_ARG;
    if (c->d.weight_format == PSV_FMT_INT8) {
        const float *scales[5] = {w->s_qkv, w->s_o, w->s_gate, w->s_up, w->s_down};
        for (const float *p : scales)
            if (!p || reinterpret_cast<uintptr_t>(p) % 16 != 0) return PSV_ERR_INVALID_ARG;
    }
    c->weights[layer] = *w;
    c->weights_set[layer] = 1;
    c->step_tbl_dirty = true;
    return PSV_OK;
}

psv_status psv_set_kv(psv_ctx *c, const psv_kv_desc *kv)
{
    if (!c || !kv || !kv->k_pools || !kv->v_pools || !kv->seq_lens) return PSV_ERR_INVALID_ARG;
    if (kv->max_blocks == 0 || (uint64_t)kv->max_blocks * PSV_BLOCK_TOKENS < c->d.max_seq) return PSV_ERR_INVALID_ARG;
    if (kv->num_pool_blocks == 0 || kv->num_pool_blocks > 0x7fffffffu) return PSV_ERR_INVALID_ARG;
    if ((uint64_t)kv->max_blocks * c->d.max_batch > 0x7fffffffull) return PSV_ERR_INVALID_ARG;
    if (!kv->page_table && (uint64_t)kv->max_blocks * c->d.max_batch > kv->num_pool_blocks) return PSV_ERR_INVALID_ARG;
    for (uint32_t l = 0; l < c->d.n_layers; ++l) {
        if (!kv->k_pools[l] || !kv->v_pools[l]) return PSV_ERR_INVALID_ARG;
        if (reinterpret_cast<uintptr_t>(kv->k_pools[l]) % 16 || reinterpret_cast<uintptr_t>(kv->v_pools[l]) % 16) return PSV_ERR_INVALID_ARG;
    }
    for (uint32_t l = 0; l < c->d.n_layers; ++l) {
        c->k_pools[l] = kv->k_pools[l];
        c->v_pools[l] = kv->v_pools[l];
    }
    c->kv = *kv;
    c->kv.k_pools = nullptr;   // the host arrays are copied, not borrowed
    c->kv.v_pools = nullptr;
    c->kv_set = true;
    c->step_tbl_dirty = true;
    return PSV_OK;
}

psv_status psv_set_comm_windows(psv_ctx *c, float us_after_attn, float us_after_mlp)
{
    if (!c || !(us_after_attn >= 0.f) || !(us_after_mlp >= 0.f) || us_after_attn > 1.0e6f || us_after_mlp > 1.0e6f) return PSV_ERR_INVALID_ARG;
    c->window_us[0] = us_after_attn;
    c->window_us[1] = us_after_mlp;
    return PSV_OK;
}

psv_status psv_set_policy(psv_ctx *c, const psv_prefetch_policy *p, uint32_t batch, uint32_t context)
{
    if (!c || !p) return PSV_ERR_INVALID_ARG;
    if (p->mode > 1 || (p->targets & ~3u) || p->partial > 1 || p->join > 1 || p->prelaunch > 1 || p->cu_budget > 65535)
        return PSV_ERR_INVALID_ARG;
    if (batch == 0 || batch > c->d.max_batch || context == 0 || context > c->d.max_seq) return PSV_ERR_INVALID_ARG;
    c->policy = *p;
    c->plan_batch = batch;
    c->plan_context = context;
    return rebuild_plan(c);
}

psv_status psv_plan(psv_ctx *c, psv_plan_entry *out, size_t cap, size_t *n)
{
    if (!c || !n || (cap > 0 && !out)) return PSV_ERR_INVALID_ARG;
    *n = c->plan.size();
    for (size_t i = 0; i < c->plan.size() && i < cap; ++i) out[i] = c->plan[i];
    return PSV_OK;
}

psv_status psv_set_graph_mode(psv_ctx *c, uint32_t use_graph)
{
    if (!c || use_graph > 1) return PSV_ERR_INVALID_ARG;
    // Retired: runs that captured, replayed and destroyed step graphs ended twice (in ~20 runs of ~75 captures each)
    // in an abort inside the HIP runtime, with no message and no cause found; eager launches were faster anyway.
    return use_graph == 1 ? PSV_ERR_UNSUPPORTED : PSV_OK;
}

psv_status psv_decode_step(psv_ctx *c, const float *x_in, float *x_out, uint32_t batch, uint32_t lb, uint32_t le)
{
    if (!c || !x_in || !x_out) return PSV_ERR_INVALID_ARG;
    if (batch == 0 || batch > c->d.max_batch || lb >= le || le > c->d.n_layers) return PSV_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(x_in) % 16 || reinterpret_cast<uintptr_t>(x_out) % 16) return PSV_ERR_INVALID_ARG;
    if (!c->kv_set) return PSV_ERR_BAD_STATE;
    for (uint32_t l = lb; l < le; ++l)
        if (!c->weights_set[l]) return PSV_ERR_BAD_STATE;
    if (c->policy.mode == 1 && c->plan_batch != batch) return PSV_ERR_BAD_STATE;   // the plan was sized for another batch
    ++c->steps;
    return enqueue_step(c, x_in, x_out, batch, lb, le);
}

psv_status psv_sync(psv_ctx *c)
{
    if (!c) return PSV_ERR_INVALID_ARG;
    hipError_t a = hipStreamSynchronize(c->main);
    hipError_t b = hipStreamSynchronize(c->side);
    hipError_t l = hipGetLastError();
    if (!(a == hipSuccess && b == hipSuccess && l == hipSuccess)) return PSV_ERR_HIP;
    if (c->check_err_word) {
        // bit 0: a consumer launched ahead of time gave up waiting for its window's end (its results are still right);
        // bit 1: a hand-over inside a fused kernel expired (results invalid)
        unsigned *err = c->at<unsigned>(c->ws.flag) + 48;
        unsigned v = 0;
        if (hipMemcpy(&v, err, sizeof v, hipMemcpyDeviceToHost) != hipSuccess) return PSV_ERR_HIP;
        c->check_err_word = false;
        if (v) {
            (void)hipMemset(err, 0, sizeof v);
            return (v & 2u) ? PSV_ERR_HIP : PSV_ERR_TIMEOUT;
        }
    }
    return PSV_OK;
}

psv_status psv_debug_force_wait_timeout(psv_ctx *c, uint32_t on)
{
    if (!c || on > 1) return PSV_ERR_INVALID_ARG;
    c->force_wait_timeout = on == 1;
    return PSV_OK;
}

psv_status psv_debug_last_step_path(psv_ctx *c, uint32_t *path)
{
    if (!c || !path) return PSV_ERR_INVALID_ARG;
    *path = c->last_step_whole ? 2u : (c->last_step_seg_attn || c->last_step_seg_mlp) ? 1u : 0u;
    return PSV_OK;
}

psv_status psv_debug_last_step_prelaunches(psv_ctx *c, uint32_t *count)
{
    if (!c || !count) return PSV_ERR_INVALID_ARG;
    *count = c->last_step_prelaunches;
    return PSV_OK;
}

psv_status psv_set_fused_kernels(psv_ctx *c, uint32_t on)
{
    if (!c || on > 3) return PSV_ERR_INVALID_ARG;
    c->fused = (int)on;
    return PSV_OK;
}

psv_status psv_get_stats(psv_ctx *c, psv_stats *out)
{
    if (!c || !out) return PSV_ERR_INVALID_ARG;
    memset(out, 0, sizeof *out);
    const uint32_t batch = c->plan_batch ? c->plan_batch : c->d.max_batch;
    const uint32_t context = c->plan_context ? c->plan_context : c->d.max_seq;
    uint64_t wb = 0;
    for (uint32_t op = 0; op < PSV_OP_COUNT; ++op)
        if (op != PSV_OP_ATTN) wb += op_mem_size(c->d, op, batch, context);
    out->weight_bytes_per_layer = wb;
    out->kv_bytes_per_layer = op_mem_size(c->d, PSV_OP_ATTN, batch, context + 1);   // the whole span, new token included
    for (const psv_plan_entry &e : c->plan) out->planned_prefetch_bytes += e.bytes;
    out->workspace_bytes = c->ws.total;
    const bool vec = c->d.weight_layout == PSV_W_ROW_MAJOR && (batch == 1 || (batch == 2 && c->d.hidden <= 4096)) && c->d.hidden <= 8192 && c->d.ffn <= 8192;
    // counted on the last step where there was one (its rotary-table and final-residual launches are once per step);
    // before the first step: the per-operator kernels of the path the shape selects
    if (c->last_step_whole)
        out->kernels_per_layer = 1;          // one kernel for the whole step
    else if (c->step_layers && c->step_launches > 2)
        out->kernels_per_layer = (c->step_launches - 2 + c->step_layers - 1) / c->step_layers;
    else
        out->kernels_per_layer = (vec ? 5 : 10) + (c->window_us[0] > 0.f ? 1 : 0) + (c->window_us[1] > 0.f ? 1 : 0);
    out->prefetch_launches = c->last_prefetch_launches;
    out->steps = c->steps;
    return PSV_OK;
}

psv_status psv_check_overlap(psv_ctx *c, int32_t *concurrent)
{
    if (!c || !concurrent) return PSV_ERR_INVALID_ARG;
    psv_status st = psv_sync(c);
    if (st != PSV_OK) return st;
    unsigned *flag = c->at<unsigned>(c->ws.flag);
    const unsigned seq = ++c->window_seq;
    // A gate that shares a hardware queue with the spin starts only once the spin has ended: time, on the host,
    // how long the side stream takes to drain while a 1 ms window runs on the main stream.
    const float us = 1000.f;
    const auto t0 = std::chrono::steady_clock::now();
    HIP_TRY(launch_spin(us_to_ticks(c->clock_khz, us), spin_cap(us), flag, nullptr, seq, c->main));
    HIP_TRY(launch_gate(flag, seq, 1u << 20, c->clock_khz * 4 /* 4 ms */, flag + 16, c->side));
    HIP_TRY(hipStreamSynchronize(c->side));
    const double waited_us = std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - t0).count();
    *concurrent = waited_us < 0.5 * us ? 1 : 0;
    c->overlap = *concurrent;
    return psv_sync(c);
}

psv_status psv_tune_attention(psv_ctx *c, const float *x_in, float *x_out, uint32_t batch, uint32_t *chunk_tokens)
{
    if (!c || !x_in || !x_out || batch == 0 || batch > c->d.max_batch) return PSV_ERR_INVALID_ARG;
    if (!c->kv_set || !c->weights_set[0]) return PSV_ERR_BAD_STATE;
    psv_status st = psv_sync(c);
    if (st != PSV_OK) return st;
    const psv_model_desc &d = c->d;
    const uint32_t unit = (d.kv_format == PSV_FMT_INT8 ? kAttnTileTokensInt8 : kAttnTileTokens) * kAttnWaves;
    // measured with prefetching off and no windows; everything is restored afterwards
    const psv_prefetch_policy saved_policy = c->policy;
    const float saved_win[2] = {c->window_us[0], c->window_us[1]};
    c->policy.mode = 0;
    c->window_us[0] = c->window_us[1] = 0.f;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) st = PSV_ERR_HIP;
    uint32_t best = 0;
    float best_ms = 0.f;
    const AttnSplit def = attn_split(d.max_batch, d.n_kv_heads, d.max_seq, d.kv_format == PSV_FMT_INT8);
    static const uint32_t mult[] = {1, 2, 3, 4, 5, 6, 7, 8, 10, 11, 12, 14, 16, 20, 24, 28, 32, 40, 48, 64};
    for (int k = -1; k < (int)(sizeof mult / sizeof mult[0]) && st == PSV_OK; ++k) {
        const uint32_t chunk = k < 0 ? (uint32_t)def.chunk_tokens : mult[k] * unit;
        const uint64_t n_chunks = ((uint64_t)d.max_seq + chunk - 1) / chunk;
        if (n_chunks > (uint64_t)kAttnMaxChunks || (k >= 0 && chunk == (uint32_t)def.chunk_tokens)) continue;
        const uint64_t wgs = n_chunks * d.n_kv_heads * batch;
        if (k >= 0 && (wgs > 8192 || (wgs < 128 && chunk > unit))) continue;   // far from filling the chip, or a long tail of rounds
        c->attn_chunk_tokens = chunk;
        float ms = 0.f;
        for (int rep = 0; rep < 2 + 8 && st == PSV_OK; ++rep) {
            if (rep == 2 && hipEventRecord(e0, c->main) != hipSuccess) st = PSV_ERR_HIP;
            if (st == PSV_OK) st = enqueue_step(c, x_in, x_out, batch, 0, 1);
        }
        if (st == PSV_OK && (hipEventRecord(e1, c->main) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                             hipEventElapsedTime(&ms, e0, e1) != hipSuccess))
            st = PSV_ERR_HIP;
        if (st == PSV_OK && (best == 0 || ms < best_ms)) { best = chunk; best_ms = ms; }
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    c->policy = saved_policy;
    c->window_us[0] = saved_win[0];
    c->window_us[1] = saved_win[1];
    c->attn_chunk_tokens = (st == PSV_OK && best != (uint32_t)def.chunk_tokens) ? best : 0;
    if (st == PSV_OK && chunk_tokens) *chunk_tokens = best;
    const psv_status st2 = psv_sync(c);
    return st != PSV_OK ? st : st2;
}

psv_status psv_set_profile_op(psv_ctx *c, int32_t op)
{
    if (!c || op < -1 || op >= (int32_t)PSV_OP_COUNT || op == PSV_OP_UP) return PSV_ERR_INVALID_ARG;   // up shares gate's kernel
    psv_status st = psv_sync(c);
    if (st != PSV_OK) return st;
    c->profile_op = op;
    c->prof_next = 0;
    c->prof_last = nullptr;
    c->prof_pairs.clear();
    return PSV_OK;
}

psv_status psv_get_profile(psv_ctx *c, double *total_ms, uint64_t *launches)
{
    if (!c || !total_ms || !launches) return PSV_ERR_INVALID_ARG;
    psv_status st = psv_sync(c);
    if (st != PSV_OK) return st;
    double sum = 0.0;
    for (const auto &pr : c->prof_pairs) {
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, pr.first, pr.second));
        sum += ms;
    }
    *total_ms = sum;
    *launches = c->prof_pairs.size();
    c->prof_next = 0;
    c->prof_last = nullptr;
    c->prof_pairs.clear();
    return PSV_OK;
}

static uint64_t current_clock_khz()
{
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) == hipSuccess && khz > 0)
        return (uint64_t)khz;
    return 100000;
}

psv_status psv_prefetch_region(const void *ptr, uint64_t bytes, uint32_t workgroups, void *stream)
{
    if (!ptr || reinterpret_cast<uintptr_t>(ptr) % 16 || workgroups == 0 || workgroups > 65535) return PSV_ERR_INVALID_ARG;
    HIP_TRY(launch_prefetch(ptr, bytes & ~(uint64_t)15, workgroups, static_cast<hipStream_t>(stream)));
    return PSV_OK;
}

psv_status psv_spin(float us, void *stream)
{
    if (!(us >= 0.f) || us > 1.0e6f) return PSV_ERR_INVALID_ARG;
    if (us == 0.f) return PSV_OK;
    HIP_TRY(launch_spin(us_to_ticks(current_clock_khz(), us), spin_cap(us), nullptr, nullptr, 0, static_cast<hipStream_t>(stream)));
    return PSV_OK;
}

psv_status psv_tile_weights(void *dst, const void *src, uint32_t rows, uint32_t cols, uint32_t weight_format, void *stream)
{
    if (!dst || !src || dst == src || weight_format > PSV_FMT_INT8) return PSV_ERR_INVALID_ARG;
    if (rows == 0 || cols == 0 || rows % 128 || cols % 64 || rows > (1u << 20) || cols > (1u << 20)) return PSV_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(dst) % 16 || reinterpret_cast<uintptr_t>(src) % 16) return PSV_ERR_INVALID_ARG;
    {
        const size_t bytes = (size_t)rows * cols * (weight_format == PSV_FMT_INT8 ? 1 : 2);
        const char *a = static_cast<const char *>(src), *b = static_cast<const char *>(dst);
        if ((a < b ? b - a : a - b) < (ptrdiff_t)bytes) return PSV_ERR_INVALID_ARG;      // the two regions overlap
    }
    HIP_TRY(launch_tile_weights(dst, src, (int)rows, (int)cols, weight_format == PSV_FMT_INT8 ? 1 : 2, static_cast<hipStream_t>(stream)));
    return PSV_OK;
}

psv_status psv_copy_bytes(void *dst, const void *src, uint64_t bytes, void *stream)
{
    if (!dst || !src || bytes % 16 || reinterpret_cast<uintptr_t>(dst) % 16 || reinterpret_cast<uintptr_t>(src) % 16) return PSV_ERR_INVALID_ARG;
    HIP_TRY(launch_copy(dst, src, bytes, static_cast<hipStream_t>(stream)));
    return PSV_OK;
}

psv_status psv_debug_read(psv_ctx *c, uint32_t which, void *host_dst, size_t bytes)
{
    if (!c || !host_dst || which >= PSV_DBG_COUNT) return PSV_ERR_INVALID_ARG;
    psv_status st = psv_sync(c);
    if (st != PSV_OK) return st;
    const size_t B = c->d.max_batch, H = c->d.hidden;
    const size_t QR = (size_t)(c->d.n_q_heads + 2 * c->d.n_kv_heads) * 128, QD = (size_t)c->d.n_q_heads * 128;
    if ((which == PSV_DBG_H1 || which == PSV_DBG_H2) && !c->last_step_vec) return PSV_ERR_BAD_STATE;
    size_t off = 0, size = 0;
    switch (which) {
    case PSV_DBG_H1: off = c->ws.h1_f32; size = B * H * 4; break;
    case PSV_DBG_QKV: off = c->ws.qkv; size = B * QR * 4; break;
    case PSV_DBG_ATTN: off = c->ws.attn_f32; size = B * QD * 4; break;
    case PSV_DBG_Y: off = c->ws.y; size = B * H * 4; break;
    case PSV_DBG_H2: off = c->ws.h2_f32; size = B * H * 4; break;
    case PSV_DBG_M: off = c->ws.m_f32; size = B * (size_t)c->d.ffn * 4; break;
    default: return PSV_ERR_INVALID_ARG;
    }
    if (bytes < size) size = bytes;
    if ((which == PSV_DBG_M && c->last_step_seg_mlp) || (which == PSV_DBG_QKV && c->last_step_seg_attn)) {
        // the fused kernels keep m and qkv (one sequence) as {value, tag} pairs
        if (which == PSV_DBG_QKV && size > QR * 4) size = QR * 4;
        std::vector<uint32_t> pairs(size / 4 * 2);
        HIP_TRY(hipMemcpy(pairs.data(), c->wsp + (which == PSV_DBG_M ? c->ws.m_ll : c->ws.qkv_ll), pairs.size() * 4, hipMemcpyDeviceToHost));
        for (size_t i = 0; i < size / 4; ++i) static_cast<uint32_t *>(host_dst)[i] = pairs[2 * i];
        return PSV_OK;
    }
    HIP_TRY(hipMemcpy(host_dst, c->wsp + off, size, hipMemcpyDeviceToHost));
    return PSV_OK;
}

}  // extern "C"

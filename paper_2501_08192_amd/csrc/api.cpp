// Context, workspace and step executor of libpreserve_mi355x.
//
// Execution model (Section 3, "PRESERVE"): the decode step's operators run in order on the main
// stream; beside each communication window an event forks the side stream, which runs the
// prefetch kernels the plan assigned to that window while the main stream sits in the window
// (here: a spin kernel standing in for the allreduce).  Prefetch kernels only read, so the main
// stream never has to wait for them; the side stream itself serialises consecutive windows.
#include <cstdlib>
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <new>
#include <utility>
#include <chrono>
#include <vector>

#include "internal.h"

using namespace psv;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Workspace {
    size_t total = 0;
    // offsets
    size_t x, y, h1_f32, h1_bf16, h2_f32, h2_bf16, qkv, rope, part_ml, part_o, attn_f32, attn_bf16,
        delta_a, delta_m, m_f32, m_bf16, inv_freq, flag, part, ssq;
};

Workspace layout_workspace(const psv_model_desc &d)
{
    Workspace w;
    const size_t B = d.max_batch, Bp = (B + 15) / 16 * 16, H = d.hidden, F = d.ffn;
    const size_t QR = (size_t)(d.n_q_heads + 2 * d.n_kv_heads) * d.head_dim, QD = (size_t)d.n_q_heads * d.head_dim;
    const size_t G = d.n_q_heads / d.n_kv_heads;
    // room for the finest attention split psv_tune_attention may choose, not only the default one
    const size_t tile_unit = (size_t)(d.kv_format == PSV_FMT_INT8 ? kAttnTileTokensInt8 : kAttnTileTokens) * kAttnWaves;
    AttnSplit sp = attn_split(d.max_batch, d.n_kv_heads, d.max_seq, d.kv_format == PSV_FMT_INT8);
    {
        size_t finest = (d.max_seq + tile_unit - 1) / tile_unit;
        if (finest > (size_t)kAttnMaxChunks) finest = kAttnMaxChunks;
        if ((size_t)sp.n_chunks < finest) sp.n_chunks = (int)finest;
    }
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
    w.x = take(B * H * 4);
    w.y = take(B * H * 4);
    w.h1_f32 = take(B * H * 4);
    w.h1_bf16 = take(2 * Bp * H * 2);
    w.h2_f32 = take(B * H * 4);
    w.h2_bf16 = take(2 * Bp * H * 2);
    w.qkv = take(B * QR * 4);
    w.rope = take(B * 64 * 2 * 4);
    w.part_ml = take(B * d.n_kv_heads * (size_t)sp.n_chunks * 16 * 2 * 4);
    w.part_o = take(B * d.n_kv_heads * (size_t)sp.n_chunks * G * 128 * 4);
    w.attn_f32 = take(B * QD * 4);
    w.attn_bf16 = take(2 * Bp * QD * 2);
    w.delta_a = take(B * H * 4);
    w.delta_m = take(B * H * 4);
    w.m_f32 = take(B * F * 4);
    w.m_bf16 = take(2 * Bp * F * 2);
    w.inv_freq = take(64 * sizeof(double));
    w.flag = take(256);
    w.ssq = take(B * (H / 512) * 4);
    {   // split-K partials of the widest projection
        size_t widest = QR > H ? QR : H;
        if (2 * F > widest) widest = 2 * F;
        w.part = take((size_t)kSkMaxSplits * B * widest * 4);
    }
    w.total = off;
    return w;
}

struct GraphKey {
    const float *x_in = nullptr;
    float *x_out = nullptr;
    uint32_t batch = 0, lb = 0, le = 0;
    uint64_t version = 0;
    bool operator==(const GraphKey &o) const
    {
        return x_in == o.x_in && x_out == o.x_out && batch == o.batch && lb == o.lb && le == o.le && version == o.version;
    }
};

}  // namespace

struct psv_ctx {
    psv_model_desc d{};
    hipStream_t main = nullptr, side = nullptr;
    int device = 0;
    uint64_t clock_khz = 100000;
    Workspace ws{};
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
    std::vector<hipEvent_t> ev_fork, ev_join;   // [layer*2 + window]
    hipEvent_t ev_end = nullptr;
    uint64_t version = 1;                        // bumped by every psv_set_*
    bool use_graph = false;
    hipGraphExec_t graph_exec = nullptr;
    GraphKey graph_key{};
    int32_t profile_op = -1;
    std::vector<hipEvent_t> prof_events;         // pool, one per profiled launch
    size_t prof_next = 0;
    hipEvent_t prof_last = nullptr;              // event of the previous main-stream kernel
    std::vector<std::pair<hipEvent_t, hipEvent_t>> prof_pairs;
    uint32_t steps = 0;
    uint32_t last_prefetch_launches = 0;
    unsigned window_seq = 0;                     // sequence number of the last communication window enqueued
    bool capturing = false;
    uint32_t attn_chunk_tokens = 0;               // 0 = default split; else tokens per attention workgroup (psv_tune_attention)
    int overlap = -1;                            // psv_check_overlap's last answer (-1 = not run yet)
    bool prelaunch_used = false;                 // some consumer was launched ahead of its window's end: check the error word at sync
    bool force_wait_timeout = false;             // test aid: such consumers give up waiting at once (and report it)
    bool last_step_vec = false;                  // the last step formed h1 / h2 (vector path)

    template <class T> T *at(size_t off) const { return reinterpret_cast<T *>(wsp + off); }
};

namespace {

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

void drop_graph(psv_ctx *c)
{
    if (c->graph_exec) {
        (void)hipGraphExecDestroy(c->graph_exec);
        c->graph_exec = nullptr;
    }
}

void touch(psv_ctx *c)
{
    ++c->version;
    drop_graph(c);
}

KvView kv_view(const psv_ctx *c, uint32_t layer)
{
    KvView v;
    v.k_pool = static_cast<uint16_t *>(c->k_pools[layer]);
    v.v_pool = static_cast<uint16_t *>(c->v_pools[layer]);
    v.int8 = c->d.kv_format == PSV_FMT_INT8 ? 1 : 0;
    v.page_table = c->kv.page_table;
    v.max_blocks = (int)c->kv.max_blocks;
    v.num_pool_blocks = (int)c->kv.num_pool_blocks;
    v.seq_lens = c->kv.seq_lens;
    return v;
}

// Attention split of this context: the default heuristic, or the chunk size chosen by psv_tune_attention.
AttnSplit ctx_split(const psv_ctx *c)
{
    const psv_model_desc &d = c->d;
    AttnSplit sp = attn_split(d.max_batch, d.n_kv_heads, d.max_seq, d.kv_format == PSV_FMT_INT8);
    if (c->attn_chunk_tokens) {
        sp.chunk_tokens = (int)c->attn_chunk_tokens;
        sp.n_chunks = (int)((d.max_seq + c->attn_chunk_tokens - 1) / c->attn_chunk_tokens);
    }
    return sp;
}

uint64_t us_to_ticks(uint64_t clock_khz, float us) { return (uint64_t)llround((double)us * (double)clock_khz / 1000.0); }
uint32_t spin_cap(float us) { return (uint32_t)(us * 4000.0f) + 100000u; }

// Per-operator timing.  While profiling is on, every main-stream kernel carries an event bound to its own
// dispatch (its end timestamp).  The duration of an operator's kernel is the distance between its event and
// the event of the kernel launched just before it on the same stream, i.e. the kernel's execution time plus
// the true dispatch gap -- no marker packets in between, which would add ~2 us each.
psv_status prof_tag(psv_ctx *c, int32_t op)
{
    if (c->capturing || c->profile_op < 0) return PSV_OK;
    if (c->prof_next == c->prof_events.size()) {
        hipEvent_t e;
        HIP_TRY(hipEventCreate(&e));
        c->prof_events.push_back(e);
    }
    hipEvent_t ev = c->prof_events[c->prof_next++];
    set_launch_events(nullptr, ev);
    if (op == c->profile_op && c->prof_last) c->prof_pairs.push_back({c->prof_last, ev});
    c->prof_last = ev;
    return PSV_OK;
}

// Projection matrix `op` of a layer in the context's weight format.
Mat mat_of(const psv_ctx *c, const psv_layer_weights &w, uint32_t op)
{
    const bool q8 = c->d.weight_format == PSV_FMT_INT8;
    Mat m;
    switch (op) {
    case PSV_OP_QKV: m.w = w.w_qkv; m.scale = q8 ? w.s_qkv : nullptr; break;
    case PSV_OP_O: m.w = w.w_o; m.scale = q8 ? w.s_o : nullptr; break;
    case PSV_OP_GATE: m.w = w.w_gate; m.scale = q8 ? w.s_gate : nullptr; break;
    case PSV_OP_UP: m.w = w.w_up; m.scale = q8 ? w.s_up : nullptr; break;
    case PSV_OP_DOWN: m.w = w.w_down; m.scale = q8 ? w.s_down : nullptr; break;
    default: break;
    }
    return m;
}

const void *weight_ptr(const psv_layer_weights &w, uint32_t op)
{
    switch (op) {
    case PSV_OP_QKV: return w.w_qkv;
    case PSV_OP_O: return w.w_o;
    case PSV_OP_GATE: return w.w_gate;
    case PSV_OP_UP: return w.w_up;
    case PSV_OP_DOWN: return w.w_down;
    default: return nullptr;
    }
}

// Packs the plan entries of one window into prefetch launches: one launch per window, or several
// when the policy caps the bytes per launch (chunk_bytes).
struct JobBuilder {
    psv_ctx *c;
    uint64_t cap;        // bytes per launch (0 = unlimited)
    const unsigned *skip;   // word written by the gate kernel of this window (null under graph capture)
    hipStream_t stream;     // where the prefetch launches go
    uint64_t used = 0;
    PrefetchJob job{};
    psv_status st = PSV_OK;

    void flush()
    {
        if (st != PSV_OK) return;
        if (job.n_regions || job.kv_count) {
            const uint32_t wg = c->policy.cu_budget ? c->policy.cu_budget : 64u;
            job.skip = skip;
            if (launch_prefetch_job(job, wg, stream) != hipSuccess) st = PSV_ERR_HIP;
            ++c->last_prefetch_launches;
        }
        job = PrefetchJob{};
        used = 0;
    }
    void add_region(const char *p, uint64_t bytes)
    {
        bytes &= ~(uint64_t)15;
        while (bytes && st == PSV_OK) {
            uint64_t room = cap ? (cap > used ? cap - used : 0) : bytes;
            room &= ~(uint64_t)15;
            if (room == 0 || job.n_regions == kPrefetchRegions) { flush(); continue; }
            const uint64_t n = bytes < room ? bytes : room;
            job.ptr[job.n_regions] = p;
            job.n16[job.n_regions] = n / 16;
            ++job.n_regions;
            used += n;
            p += n;
            bytes -= n;
        }
    }
    void add_kv(const KvView &v, int nkv, uint32_t blocks_per_seq, uint64_t count, uint64_t bytes_per_block)
    {
        uint64_t first = 0;
        while (count && st == PSV_OK) {
            uint64_t room = cap ? (cap > used ? (cap - used) / bytes_per_block : 0) : count;
            if (room == 0 && used == 0) room = 1;          // a launch always makes progress
            if (room == 0 || job.kv_count) { flush(); continue; }
            const uint64_t n = count < room ? count : room;
            job.kv = v;
            job.nkv = nkv;
            job.blocks_per_seq = blocks_per_seq;
            job.kv_first = first;
            job.kv_count = n;
            used += n * bytes_per_block;
            first += n;
            count -= n;
        }
    }
};

psv_status add_entry(psv_ctx *c, JobBuilder &jb, const psv_plan_entry &e, uint32_t batch)
{
    if (e.target_op == PSV_OP_ATTN) {
        const uint32_t ro_tokens = c->plan_context > 0 ? c->plan_context - 1 : 0;
        const uint32_t blocks_per_seq = (ro_tokens + PSV_BLOCK_TOKENS - 1) / PSV_BLOCK_TOKENS;
        if (blocks_per_seq == 0) return PSV_OK;
        const uint64_t unit = c->d.kv_format == PSV_FMT_INT8 ? PSV_KV_UNIT_BYTES_INT8 : PSV_KV_UNIT_BYTES_BF16;
        const uint64_t bytes_per_block = (uint64_t)c->d.n_kv_heads * unit * 2;   // K and V
        const uint64_t total = (uint64_t)batch * blocks_per_seq;
        uint64_t count = (e.bytes + bytes_per_block - 1) / bytes_per_block;
        if (count > total) count = total;
        jb.add_kv(kv_view(c, e.target_layer), (int)c->d.n_kv_heads, blocks_per_seq, count, bytes_per_block);
        return jb.st;
    }
    const char *p = static_cast<const char *>(weight_ptr(c->weights[e.target_layer], e.target_op));
    if (!p) return PSV_ERR_BAD_STATE;
    jb.add_region(p, e.bytes);
    return jb.st;
}

// The two streams of a step.  Normally `cur` is the caller's main stream for the whole step; with the
// `prelaunch` policy the operator chain hops to the other stream at every communication window.
struct Lanes {
    hipStream_t cur, other;
};

// The communication window after the attention block (window 0) or the MLP block (window 1).  The
// stand-in for the collective is enqueued first, so that the stream never waits for the host; the window's
// prefetch job goes to the other stream and starts when the window starts.
//
// prelaunch (policy extension, eager launches, vector path): the first consumer after the window -- gate/up
// after window 0, the next layer's QKV after window 1 -- is the one operator whose weights are needed the moment
// the window ends.  If Algorithm 1 planned a prefetch for it, that prefetch is done by the consumer itself: the
// caller launches it on the other stream right behind the window's gate and its (remaining) prefetch job, with a
// GemvWait on the window's end.  It pulls its first weights into registers while the window runs and finishes a
// few microseconds after the window does.  The rest of the chain follows it on that stream, so the two streams
// swap roles at every window and no host-side event is needed: every cross-stream dependency is one of the two
// flags the window kernel publishes (start, end).  *wait_set tells the caller to launch the consumer that way.
// Does the plan hand the whole weight matrix of the first consumer after (layer, window) to that window, so that
// the consumer can be launched ahead of time (policy.prelaunch, eager launches, vector path)?
bool can_prelaunch(const psv_ctx *c, uint32_t layer, uint32_t window, uint32_t layer_end, bool vec)
{
    if (c->capturing || !vec || c->policy.mode != 1 || !c->policy.prelaunch || !(c->window_us[window] > 0.f)) return false;
    if (c->overlap != 1) return false;      // a waiting kernel may only be queued where it cannot block the window kernel
    if (window == 1 && layer + 1 >= layer_end) return false;       // end of the graph: no consumer
    const uint32_t first_op = window == 0 ? PSV_OP_GATE : PSV_OP_QKV;
    for (const psv_plan_entry &e : c->plan)
        if (e.layer == layer && e.window == window && e.target_op == first_op && e.bytes == e.mem_size) return true;
    return false;
}

psv_status comm_window(psv_ctx *c, uint32_t layer, uint32_t window, uint32_t batch, uint32_t layer_end, bool pre,
                       Lanes *ln, GemvWait *wait, bool *wait_set, bool *side_used)
{
    *wait_set = false;
    const float us = c->window_us[window];
    if (!(us > 0.f)) return PSV_OK;
    bool any = false;
    if (c->policy.mode == 1)
        for (const psv_plan_entry &e : c->plan)
            if (e.layer == layer && e.window == window && e.target_layer < layer_end) { any = true; break; }
    // Eager launches fork on the device: the window kernel publishes a sequence number that a one-wave gate
    // kernel, queued on the other stream ahead of the prefetch launches, waits for.  Under graph capture the
    // fork is an event edge.
    unsigned *flag = c->capturing ? nullptr : c->at<unsigned>(c->ws.flag);
    unsigned *done = flag ? flag + 32 : nullptr, *err = flag ? flag + 48 : nullptr;
    const unsigned seq = ++c->window_seq;
    const uint32_t first_op = window == 0 ? PSV_OP_GATE : PSV_OP_QKV;
    hipEvent_t ev = c->ev_fork[layer * 2 + window];
    if (any && !flag) HIP_TRY(hipEventRecord(ev, ln->cur));
    ST_TRY(prof_tag(c, -2));
    HIP_TRY(launch_spin(us_to_ticks(c->clock_khz, us), spin_cap(us), flag, done, seq, ln->cur));
    if (!any) return PSV_OK;
    unsigned *skip = flag ? flag + 16 : nullptr;
    if (flag)
        // A gate that gives up only costs its window's prefetch -- unless a consumer is queued behind it: that
        // one must not start (and then run out of patience itself) while the stream of the window is merely
        // held up by earlier work of the caller, so its gate and its own wait are bounded by a second, not 20 ms.
        HIP_TRY(launch_gate(flag, seq, pre ? 1u << 22 : 1u << 20, c->clock_khz * (pre ? 1000 : 20) /* 1 s : 20 ms */, skip,
                            ln->other));
    else
        HIP_TRY(hipStreamWaitEvent(ln->other, ev, 0));
    uint64_t cap = c->policy.chunk_bytes & ~(uint64_t)15;
    if (c->policy.chunk_bytes && cap < 16) cap = 16;
    JobBuilder jb{c, cap, skip, ln->other};
    for (const psv_plan_entry &e : c->plan) {
        if (e.layer != layer || e.window != window || e.target_layer >= layer_end) continue;
        // what the pre-launched consumer reads itself needs no second copy in the memory-side cache
        if (pre && (e.target_op == first_op || (window == 0 && e.target_op == PSV_OP_UP))) continue;
        psv_status st = add_entry(c, jb, e, batch);
        if (st != PSV_OK) return st;
    }
    jb.flush();
    if (jb.st != PSV_OK) return jb.st;
    *side_used = true;
    if (pre) {
        wait->done = done;
        wait->seq = seq;
        wait->iters = c->force_wait_timeout ? 0u : (1u << 22);
        wait->ticks = c->force_wait_timeout ? 0ull : us_to_ticks(c->clock_khz, us) * 2 + c->clock_khz * 1000 /* + 1 s */;
        wait->err = err;
        *wait_set = true;
        c->prelaunch_used = true;
        std::swap(ln->cur, ln->other);     // the chain continues behind the consumer
        return PSV_OK;
    }
    if (c->policy.join) {
        HIP_TRY(hipEventRecord(c->ev_join[layer * 2 + window], ln->other));
        HIP_TRY(hipStreamWaitEvent(ln->cur, c->ev_join[layer * 2 + window], 0));
    }
    return PSV_OK;
}

psv_status enqueue_step(psv_ctx *c, const float *x_in, float *x_out, uint32_t batch, uint32_t lb, uint32_t le)
{
    const psv_model_desc &d = c->d;
    const int B = (int)batch, H = (int)d.hidden, F = (int)d.ffn, nq = (int)d.n_q_heads, nkv = (int)d.n_kv_heads;
    const int QR = (nq + 2 * nkv) * 128, QD = nq * 128;
    const AttnSplit sp = ctx_split(c);
    float *x = c->at<float>(c->ws.x), *y = c->at<float>(c->ws.y);
    float *delta_a = c->at<float>(c->ws.delta_a), *delta_m = c->at<float>(c->ws.delta_m);
    float *h1 = c->at<float>(c->ws.h1_f32), *h2 = c->at<float>(c->ws.h2_f32);
    uint16_t *h1b = c->at<uint16_t>(c->ws.h1_bf16), *h2b = c->at<uint16_t>(c->ws.h2_bf16);
    float *qkv = c->at<float>(c->ws.qkv), *attn = c->at<float>(c->ws.attn_f32), *m = c->at<float>(c->ws.m_f32);
    uint16_t *attnb = c->at<uint16_t>(c->ws.attn_bf16), *mb = c->at<uint16_t>(c->ws.m_bf16);
    float *pml = c->at<float>(c->ws.part_ml), *po = c->at<float>(c->ws.part_o);
    float2 *rope = c->at<float2>(c->ws.rope);
    const double *inv_freq = d.rope_theta > 0.f ? c->at<double>(c->ws.inv_freq) : nullptr;
    Lanes ln{c->main, c->side};
    hipStream_t &s = ln.cur;          // the stream the operator chain is on (changes at a pre-launching window)
    GemvWait wait{};
    bool wait_qkv = false, wait_gate = false;
    bool side_used = false;
    c->last_prefetch_launches = 0;
    auto u16 = [](const void *p) { return static_cast<const uint16_t *>(p); };
    const bool w8 = d.weight_format == PSV_FMT_INT8;
    const size_t plane_h = (size_t)((B + 15) / 16 * 16) * H;   // hi -> lo plane distance of the bf16 activations

    // Batch 1 (and batch 2 on 8B-sized matrices) runs every projection on the vector ALU with the normalisation
    // fused into the prologue; larger batches use the matrix cores: split-K GEMMs whose partials are summed by the
    // residual kernel (O, down) or a small reduction kernel (QKV; gate/up with SwiGLU), the RMSNorm factor being
    // applied in the epilogue of the GEMM that follows the residual kernel.
    // (Measured crossover: the vector path loses ~10 us per layer and extra batch row to register pressure.)
    const bool vec = (B == 1 || (B == 2 && H <= 4096)) && gemv_supported(B, QR, H) && gemv_supported(B, H, QD) &&
                     gemv_supported(B, F, H) && gemv_supported(B, H, F);
    const bool sk = !vec;
    c->last_step_vec = vec;
    float *part = c->at<float>(c->ws.part), *ssq = c->at<float>(c->ws.ssq);

    // The chain hops to the other stream at every pre-launching window and has to be back on the main stream when
    // the step ends (the caller's own work on that stream follows it): with an odd number of such windows the last
    // one runs without pre-launch.
    int pre_left = 0;
    for (uint32_t l = lb; l < le; ++l)
        for (uint32_t wdw = 0; wdw < 2; ++wdw) pre_left += can_prelaunch(c, l, wdw, le, vec) ? 1 : 0;
    if (pre_left & 1) --pre_left;
    auto take_pre = [&](uint32_t l, uint32_t wdw) {
        if (pre_left > 0 && can_prelaunch(c, l, wdw, le, vec)) { --pre_left; return true; }
        return false;
    };

    ST_TRY(prof_tag(c, -2));
    HIP_TRY(launch_rope_table(c->kv.seq_lens, inv_freq, (int)c->kv.max_blocks * 16, B, rope, s));
    const float *res = x_in, *delta = nullptr;   // residual stream entering the layer = res + delta
    int delta_splits = 1;                        // delta may be a stack of split-K partials
    for (uint32_t l = lb; l < le; ++l) {
        const psv_layer_weights &w = c->weights[l];
        const KvView kv = kv_view(c, l);
        const Mat Wqkv = mat_of(c, w, PSV_OP_QKV), Wo = mat_of(c, w, PSV_OP_O), Wg = mat_of(c, w, PSV_OP_GATE),
                  Wu = mat_of(c, w, PSV_OP_UP), Wd = mat_of(c, w, PSV_OP_DOWN);

        if (sk) {
            ST_TRY(prof_tag(c, -2));
            HIP_TRY(launch_resid_sum(res, delta, delta_splits, B, H, x, u16(w.g_attn), h1b, plane_h, w8, ssq, s));
        }
        ST_TRY(prof_tag(c, PSV_OP_QKV));
        if (vec) {
            HIP_TRY(launch_gemv_norm(Wqkv, Mat{}, res, delta, u16(w.g_attn), d.rms_eps, x, h1, qkv, B, QR, H,
                                     wait_qkv ? &wait : nullptr, s));
            wait_qkv = false;
        } else {
            if (!gemm_sk_supported(B, QR, H)) return PSV_ERR_UNSUPPORTED;
            HIP_TRY(launch_gemm_sk(Wqkv, Mat{}, 0, h1b, ssq, d.rms_eps, part, B, QR, H, s));
            ST_TRY(prof_tag(c, -2));
            HIP_TRY(launch_sk_reduce(part, gemm_sk_splits(B, QR, H, w8), B, QR, false, qkv, nullptr, false, s));
        }

        ST_TRY(prof_tag(c, PSV_OP_ATTN));
        HIP_TRY(launch_attn(qkv, rope, kv, B, nq, nkv, sp, pml, po, s));
        const bool fuse_merge = vec && gemv_merge_supported(B, nq, sp.n_chunks);
        if (!fuse_merge) {
            ST_TRY(prof_tag(c, -2));
            HIP_TRY(launch_attn_merge(pml, po, B, nq, nkv, sp, attn, attnb, sk && w8, s));
        }

        ST_TRY(prof_tag(c, PSV_OP_O));
        const float *attn_delta = delta_a;
        int attn_splits = 1;
        if (fuse_merge) {
            HIP_TRY(launch_gemv_merge(Wo, pml, po, nq, nkv, sp.n_chunks, attn, delta_a, B, H, s));
        } else if (vec) {
            HIP_TRY(launch_gemv(Wo, Mat{}, attn, delta_a, B, H, QD, s));
        } else {
            if (!gemm_sk_supported(B, H, QD)) return PSV_ERR_UNSUPPORTED;
            HIP_TRY(launch_gemm_sk(Wo, Mat{}, 0, attnb, nullptr, 0.f, part, B, H, QD, s));
            attn_delta = part;
            attn_splits = gemm_sk_splits(B, H, QD, w8);
        }

        ST_TRY(comm_window(c, l, 0, batch, le, take_pre(l, 0), &ln, &wait, &wait_gate, &side_used));

        if (sk) {
            ST_TRY(prof_tag(c, -2));
            HIP_TRY(launch_resid_sum(x, attn_delta, attn_splits, B, H, y, u16(w.g_mlp), h2b, plane_h, w8, ssq, s));
        }
        ST_TRY(prof_tag(c, PSV_OP_GATE));
        if (vec) {
            HIP_TRY(launch_gemv_norm(Wg, Wu, x, delta_a, u16(w.g_mlp), d.rms_eps, y, h2, m, B, F, H,
                                     wait_gate ? &wait : nullptr, s));
            wait_gate = false;
        } else {
            if (!gemm_sk_supported(B, 2 * F, H)) return PSV_ERR_UNSUPPORTED;
            HIP_TRY(launch_gemm_sk(Wg, Wu, F, h2b, ssq, d.rms_eps, part, B, 2 * F, H, s));
            ST_TRY(prof_tag(c, -2));
            HIP_TRY(launch_sk_reduce(part, gemm_sk_splits(B, 2 * F, H, w8), B, 2 * F, true, m, mb, w8, s));
        }

        ST_TRY(prof_tag(c, PSV_OP_DOWN));
        delta = delta_m;
        delta_splits = 1;
        if (vec) {
            HIP_TRY(launch_gemv(Wd, Mat{}, m, delta_m, B, H, F, s));
        } else {
            if (!gemm_sk_supported(B, H, F)) return PSV_ERR_UNSUPPORTED;
            HIP_TRY(launch_gemm_sk(Wd, Mat{}, 0, mb, nullptr, 0.f, part, B, H, F, s));
            delta = part;
            delta_splits = gemm_sk_splits(B, H, F, w8);
        }

        ST_TRY(comm_window(c, l, 1, batch, le, take_pre(l, 1), &ln, &wait, &wait_qkv, &side_used));
        res = y;
    }
    ST_TRY(prof_tag(c, -2));
    HIP_TRY(launch_resid_sum(res, delta, delta_splits, B, H, x_out, nullptr, nullptr, 0, false, nullptr, s));
    if (ln.cur != c->main) {           // cannot happen with the pairing above; kept as a safety net
        HIP_TRY(hipEventRecord(c->ev_end, ln.cur));
        HIP_TRY(hipStreamWaitEvent(c->main, c->ev_end, 0));
    }
    if (side_used && c->capturing) {   // a captured side branch has to rejoin the origin stream
        HIP_TRY(hipEventRecord(c->ev_end, c->side));
        HIP_TRY(hipStreamWaitEvent(c->main, c->ev_end, 0));
    }
    return PSV_OK;
}

psv_status rebuild_plan(psv_ctx *c)
{
    c->plan.clear();
    if (c->plan_batch == 0) return PSV_OK;
    size_t n = plan_chain(c->d, c->plan_batch, c->plan_context, c->policy, nullptr, 0);
    c->plan.resize(n);
    if (n) plan_chain(c->d, c->plan_batch, c->plan_context, c->policy, c->plan.data(), n);
    return PSV_OK;
}

}  // namespace

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
    c->ev_fork.assign((size_t)c->d.n_layers * 2, nullptr);
    c->ev_join.assign((size_t)c->d.n_layers * 2, nullptr);
    for (size_t i = 0; i < c->ev_fork.size(); ++i) {
        if (hipEventCreateWithFlags(&c->ev_fork[i], hipEventDisableTiming) != hipSuccess) return fail(PSV_ERR_HIP);
        if (hipEventCreateWithFlags(&c->ev_join[i], hipEventDisableTiming) != hipSuccess) return fail(PSV_ERR_HIP);
    }
    if (hipEventCreateWithFlags(&c->ev_end, hipEventDisableTiming) != hipSuccess) return fail(PSV_ERR_HIP);
    c->policy.mode = 0;
    c->policy.targets = PSV_TARGET_WEIGHTS | PSV_TARGET_KV;
    *out = c;
    return PSV_OK;
}

psv_status psv_destroy(psv_ctx *c)
{
    if (!c) return PSV_ERR_INVALID_ARG;
    drop_graph(c);
    for (hipEvent_t e : c->ev_fork) if (e) (void)hipEventDestroy(e);
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
    touch(c);
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
    touch(c);
    return PSV_OK;
}

psv_status psv_set_comm_windows(psv_ctx *c, float us_after_attn, float us_after_mlp)
{
    if (!c || !(us_after_attn >= 0.f) || !(us_after_mlp >= 0.f) || us_after_attn > 1.0e6f || us_after_mlp > 1.0e6f) return PSV_ERR_INVALID_ARG;
    c->window_us[0] = us_after_attn;
    c->window_us[1] = us_after_mlp;
    touch(c);
    return PSV_OK;
}

psv_status psv_set_policy(psv_ctx *c, const psv_prefetch_policy *p, uint32_t batch, uint32_t context)
{
    if (!c || !p) return PSV_ERR_INVALID_ARG;
    if (p->mode > 1 || (p->targets & ~3u) || p->partial > 1 || p->join > 1 || p->prelaunch > 1 || p->cu_budget > 65535)
        return PSV_ERR_INVALID_ARG;
    if (batch == 0 || batch > c->d.max_batch || context == 0 || context > c->d.max_seq) return PSV_ERR_INVALID_ARG;
    if (p->mode == 1 && p->prelaunch && c->overlap < 0) {   // pre-launched kernels need streams that really overlap
        int32_t concurrent = 0;
        psv_status st = psv_check_overlap(c, &concurrent);
        if (st != PSV_OK) return st;
    }
    c->policy = *p;
    c->plan_batch = batch;
    c->plan_context = context;
    touch(c);
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
    if (use_graph == 1) {
        // Off unless asked for twice: runs that captured, replayed and destroyed step graphs ended twice (in ~20 runs
        // of ~75 captures each) in an abort inside the HIP runtime, with no message and no cause found.
        const char *on = std::getenv("PSV_ENABLE_HIP_GRAPHS");
        if (!on || on[0] != '1' || on[1] != '\0') return PSV_ERR_UNSUPPORTED;
    }
    c->use_graph = use_graph == 1;
    if (!c->use_graph) drop_graph(c);
    return PSV_OK;
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
    if (!c->use_graph) return enqueue_step(c, x_in, x_out, batch, lb, le);

    GraphKey key{x_in, x_out, batch, lb, le, c->version};
    if (!c->graph_exec || !(key == c->graph_key)) {
        drop_graph(c);
        hipGraph_t graph = nullptr;
        HIP_TRY(hipStreamBeginCapture(c->main, hipStreamCaptureModeThreadLocal));
        c->capturing = true;
        psv_status st = enqueue_step(c, x_in, x_out, batch, lb, le);
        c->capturing = false;
        hipError_t e = hipStreamEndCapture(c->main, &graph);
        if (st != PSV_OK || e != hipSuccess) {
            if (graph) (void)hipGraphDestroy(graph);
            return st != PSV_OK ? st : PSV_ERR_HIP;
        }
        e = hipGraphInstantiate(&c->graph_exec, graph, nullptr, nullptr, 0);
        (void)hipGraphDestroy(graph);
        if (e != hipSuccess) {
            c->graph_exec = nullptr;
            return PSV_ERR_HIP;
        }
        c->graph_key = key;
    }
    HIP_TRY(hipGraphLaunch(c->graph_exec, c->main));
    return PSV_OK;
}

psv_status psv_sync(psv_ctx *c)
{
    if (!c) return PSV_ERR_INVALID_ARG;
    hipError_t a = hipStreamSynchronize(c->main);
    hipError_t b = hipStreamSynchronize(c->side);
    hipError_t l = hipGetLastError();
    if (!(a == hipSuccess && b == hipSuccess && l == hipSuccess)) return PSV_ERR_HIP;
    if (c->prelaunch_used) {   // did a consumer launched ahead of time give up waiting for its window's end?
        unsigned *err = c->at<unsigned>(c->ws.flag) + 48;
        unsigned v = 0;
        if (hipMemcpy(&v, err, sizeof v, hipMemcpyDeviceToHost) != hipSuccess) return PSV_ERR_HIP;
        c->prelaunch_used = false;
        if (v) {
            (void)hipMemset(err, 0, sizeof v);
            return PSV_ERR_HIP;
        }
    }
    return PSV_OK;
}

psv_status psv_debug_force_wait_timeout(psv_ctx *c, uint32_t on)
{
    if (!c || on > 1) return PSV_ERR_INVALID_ARG;
    c->force_wait_timeout = on == 1;
    touch(c);
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
    const bool vec = (batch == 1 || (batch == 2 && c->d.hidden <= 4096)) && c->d.hidden <= 8192 && c->d.ffn <= 8192;
    out->kernels_per_layer = (vec ? 5 : 7) + (c->window_us[0] > 0.f ? 1 : 0) + (c->window_us[1] > 0.f ? 1 : 0);
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
    touch(c);
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
    // measured with prefetching off, eager launches and no windows; everything is restored afterwards
    const psv_prefetch_policy saved_policy = c->policy;
    const float saved_win[2] = {c->window_us[0], c->window_us[1]};
    const bool saved_graph = c->use_graph;
    c->policy.mode = 0;
    c->window_us[0] = c->window_us[1] = 0.f;
    c->use_graph = false;
    drop_graph(c);
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
    c->use_graph = saved_graph;
    c->attn_chunk_tokens = (st == PSV_OK && best != (uint32_t)def.chunk_tokens) ? best : 0;
    touch(c);
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
    HIP_TRY(hipMemcpy(host_dst, c->wsp + off, size, hipMemcpyDeviceToHost));
    return PSV_OK;
}

}  // extern "C"

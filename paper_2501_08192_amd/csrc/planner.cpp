// Host-only part of libpreserve_mi355x: descriptor validation, byte accounting and the prefetch
// planner (Algorithm 1, Section 3 "Operator insertion") specialised to the operator chain of a
// decoder shard.  Nothing here touches the GPU.
#include "internal.h"

namespace psv {

static bool desc_ok(const psv_model_desc &d)
{
    if (d.n_layers == 0 || d.n_layers > 4096) return false;
    if (d.hidden == 0 || d.hidden % 512 != 0 || d.hidden > 16384) return false;
    if (d.head_dim != PSV_HEAD_DIM) return false;
    if (d.n_q_heads == 0 || d.n_kv_heads == 0 || d.n_q_heads % d.n_kv_heads != 0) return false;
    if (d.n_q_heads / d.n_kv_heads > 16 || d.n_q_heads > 128) return false;
    if (d.ffn == 0 || d.ffn % 256 != 0 || d.ffn > 65536) return false;
    if (!(d.rms_eps >= 0.f) || !(d.rope_theta >= 0.f)) return false;
    if (d.max_batch == 0 || d.max_batch > 64) return false;
    if (d.max_seq == 0 || d.max_seq % PSV_BLOCK_TOKENS != 0 || d.max_seq > (1u << 20)) return false;
    if (d.weight_format > PSV_FMT_INT8 || d.kv_format > PSV_FMT_INT8) return false;
    if (d.kv_layout > PSV_KV_TOKEN_MAJOR || (d.kv_layout == PSV_KV_TOKEN_MAJOR && d.kv_format != PSV_FMT_BF16)) return false;
    if (d.weight_layout > PSV_W_TILED) return false;
    return true;
}

// memSize() of Algorithm 1: a MatMul counts its weight matrix, the attention counts the K and V
// entries it only reads (the newest entry is written by the step itself and is not prefetchable).
uint64_t op_mem_size(const psv_model_desc &d, uint32_t op, uint32_t batch, uint32_t context)
{
    const uint64_t H = d.hidden, F = d.ffn, hd = d.head_dim;
    const uint64_t wb = d.weight_format == PSV_FMT_INT8 ? 1 : 2;                 // bytes per weight
    // K and V bytes of one token of one kv head; the int8 cache carries a 4-byte scale per row
    const uint64_t kvb = d.kv_format == PSV_FMT_INT8 ? 2 * (hd + 4) : 2 * hd * 2;
    switch (op) {
    case PSV_OP_QKV: return (uint64_t)(d.n_q_heads + 2 * d.n_kv_heads) * hd * H * wb;
    case PSV_OP_ATTN: return (uint64_t)batch * (context > 0 ? context - 1 : 0) * d.n_kv_heads * kvb;
    case PSV_OP_O: return H * d.n_q_heads * hd * wb;
    case PSV_OP_GATE: return F * H * wb;
    case PSV_OP_UP: return F * H * wb;
    case PSV_OP_DOWN: return H * F * wb;
    default: return 0;
    }
}

static bool op_in_targets(uint32_t op, uint32_t targets)
{
    if (op == PSV_OP_ATTN) return (targets & PSV_TARGET_KV) != 0;
    return (targets & PSV_TARGET_WEIGHTS) != 0;
}

// The chain is linear, so "visit the children breadth first until the next communication op" is a
// walk in program order.  Window 0 of layer l is followed by {gate, up, down} of layer l, window 1
// by {QKV, attention, O} of layer l+1 (nothing after the last layer: end of graph).
size_t plan_chain(const psv_model_desc &d, uint32_t batch, uint32_t context, const psv_prefetch_policy &p,
                  psv_plan_entry *out, size_t cap)
{
    size_t n = 0;
    if (p.mode == 0) return 0;
    static const uint32_t after_attn[3] = {PSV_OP_GATE, PSV_OP_UP, PSV_OP_DOWN};
    static const uint32_t after_mlp[3] = {PSV_OP_QKV, PSV_OP_ATTN, PSV_OP_O};
    for (uint32_t layer = 0; layer < d.n_layers; ++layer) {
        for (uint32_t window = 0; window < 2; ++window) {
            const uint32_t tl = window == 0 ? layer : layer + 1;
            if (tl >= d.n_layers) continue;
            const uint32_t *ops = window == 0 ? after_attn : after_mlp;
            uint64_t cache_sum = 0;
            for (int k = 0; k < 3; ++k) {
                const uint32_t op = ops[k];
                if (!op_in_targets(op, p.targets)) continue;
                const uint64_t mem = op_mem_size(d, op, batch, context);
                const uint64_t before = cache_sum;
                cache_sum += mem;
                uint64_t take = 0;
                bool stop = false;
                if (cache_sum < p.budget_bytes) {
                    take = mem;
                } else {
                    stop = true;
                    if (p.partial && p.budget_bytes > before + 1) take = p.budget_bytes - 1 - before;
                }
                if (take > 0) {
                    if (out && n < cap) out[n] = psv_plan_entry{layer, window, tl, op, mem, take};
                    ++n;
                }
                if (stop) break;
            }
        }
    }
    return n;
}

}  // namespace psv

using namespace psv;

extern "C" {

const char *psv_strerror(psv_status s)
{
    switch (s) {
    case PSV_OK: return "ok";
    case PSV_ERR_INVALID_ARG: return "invalid argument";
    case PSV_ERR_BAD_STATE: return "call not valid in the current state";
    case PSV_ERR_UNSUPPORTED: return "shape not supported by the kernels";
    case PSV_ERR_HIP: return "HIP runtime error";
    case PSV_ERR_NOMEM: return "out of memory";
    case PSV_ERR_TIMEOUT: return "a kernel launched ahead of its communication window gave up waiting for the window's end";
    default: return "unknown status";
    }
}

psv_status psv_validate_desc(const psv_model_desc *desc)
{
    if (!desc) return PSV_ERR_INVALID_ARG;
    return desc_ok(*desc) ? PSV_OK : PSV_ERR_INVALID_ARG;
}

psv_status psv_plan_chain(const psv_model_desc *desc, uint32_t batch, uint32_t context,
                          const psv_prefetch_policy *policy, psv_plan_entry *out, size_t cap, size_t *n)
{
    if (!desc || !policy || !n || (cap > 0 && !out)) return PSV_ERR_INVALID_ARG;
    if (!desc_ok(*desc) || batch == 0 || batch > desc->max_batch || context == 0 || context > desc->max_seq)
        return PSV_ERR_INVALID_ARG;
    if (policy->mode > 1 || (policy->targets & ~3u) || policy->partial > 1 || policy->join > 1 || policy->prelaunch > 1)
        return PSV_ERR_INVALID_ARG;
    *n = plan_chain(*desc, batch, context, *policy, out, cap);
    return PSV_OK;
}

}  // extern "C"

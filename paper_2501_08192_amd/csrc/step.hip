// gfx950 (MI355X, CDNA4) kernels of the PRESERVE decode step: the whole step of one sequence as ONE kernel.
//
// One workgroup per CU, all resident for the whole step, walks the layers.  Every hand-over -- between the phases of a
// block (QKV -> attention -> O; gate/up -> down), across a communication window and from layer to layer -- is a set of
// tagged values (tagged.h); there is no kernel boundary, no dispatch gap and no cold instruction cache after the first
// layer.  The residual stream never touches memory: every workgroup carries its own copy of it, spread over its threads'
// registers, and adds the same tagged projection outputs to it.
//
// Communication window (Section 2, "Multi-device inference": one allreduce after the attention block, one after the MLP
// block; here the timed stand-in): the last workgroup of the grid stands in for the collective and does nothing else.
// It reads the block's whole output until every value carries the layer's tag -- the collective cannot start before its
// input exists --, then its wave 0 spins for the window's length on the wall clock (one wave on one CU) and publishes
// the window's end as a tagged word.  No other workgroup reads the block's output before it has seen that word: the
// output of a real in-kernel collective would not exist earlier.  (The time-keeper must not be a wave that also
// requests weights: a wave cannot go on to its spin loop until the memory pipeline has accepted its loads, which under
// the load of a whole chip requesting at once takes as long as the transfer -- measured: the window then starts 8 us late.)
//
// Prefetch (Section 3, "Execution with the proposed method"): what Algorithm 1 hands to a window -- the next block's
// projection weights, and for the attention block its K/V tiles -- is requested into registers BEFORE the workgroup
// starts waiting for that window's end, so it travels while the window runs; what the plan does not hand to the window
// (policy off, or a budget that ends earlier) is requested only AFTER the end word has been seen, which is the vanilla
// execution.  Same kernel, same order of arithmetic, same bits either way.
//
// Every wait is bounded (iteration caps); a hand-over that expires sets bit 1 of the error word, the kernel runs to its
// end and psv_sync reports an error.
#include "tagged.h"

namespace psv {

struct StepLayer {            // one entry per layer of a table in device memory
    const void *Wq, *Wo, *Wg, *Wu, *Wd;
    const float *sq, *so, *sg, *su, *sd;
    const uint16_t *g_attn, *g_mlp;
    uint16_t *k_pool, *v_pool;
};
static_assert(sizeof(StepLayer) == kStepLayerBytes, "the host lays the table out by this size");

struct StepArgs {
    const StepLayer *layers;
    int lb, le;
    const float *x_in;
    float *x_out;
    int H, F, nq, nkv, QR, QD, n_chunks;
    float eps;
    SegGeom gq, go, g1, g2;
    const float2 *rope;
    const int32_t *page_table;
    int max_blocks, max_tokens, num_pool_blocks;
    const int32_t *seq_lens;
    uint2 *qkv_ll, *pml_ll, *po_ll, *da_ll, *m_ll, *dm_ll, *done_ll;
    unsigned tag_base;
    uint32_t ll_iters;
    unsigned *err;
    uint64_t ticks[2];          // window after the attention block, after the MLP block (0: no window)
    uint32_t spin_iters[2];
    int hold[2];                // requested before the window's end: [0] bit 0 gate/up, bit 1 down; [1] bit 0 QKV, bit 1 K/V tiles, bit 2 O
    float *dbg_x, *dbg_h1, *dbg_attn, *dbg_y, *dbg_h2;      // intermediates of the last layer run, stored by workgroup 0
};

enum { TAG_QKV = 0, TAG_PART = 1, TAG_DA = 2, TAG_WIN0 = 3, TAG_M = 4, TAG_DM = 5, TAG_WIN1 = 6, TAGS_PER_LAYER = 8 };

// Per-thread state that lives across the layers.
template <int ITH>
struct StepState {
    float res[ITH][8];      // this thread's slice of the residual stream
    int rb[4], re[4];       // row range of this thread's group in QKV, O, gate/up, down
    int blkA, blkB;         // physical K/V blocks of this wave's attention tile (-1: none)
    int lost;               // a hand-over expired
};

// One layer (l < le), or the receipt of the last layer's output (l == le).  A function of its own, not the body of a
// loop in the kernel: as a loop body the compiler's register allocation keeps several hundred values too many alive
// and spills them (measured: 700-1200 spilled registers against none this way).  The arguments of the kernel are read
// from the kernel-argument segment again, whose address the kernel passes down.
template <int ITH, int IT2, bool W8>
__device__ __noinline__ void step_layer(StepState<ITH> &st, int l_any, uint64_t kernarg_any)
{
    // the address of the kernel's argument block, handed down by the kernel; made wave-uniform again so that the
    // arguments are fetched by scalar loads
    // (the builtin returns a signed int: without the cast to unsigned the low half would be sign-extended over the high one)
    const uint64_t ka_addr = (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)kernarg_any) |
                             ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(kernarg_any >> 32)) << 32);
    union {
        StepArgs a;
        uint32_t w[sizeof(StepArgs) / 4];
    } args;
    {
        const __attribute__((address_space(4))) uint32_t *src = (const __attribute__((address_space(4))) uint32_t *)ka_addr;
#pragma unroll
        for (unsigned k = 0; k < sizeof(StepArgs) / 4; ++k) args.w[k] = src[k];
    }
    const StepArgs &a = args.a;
    const int l = __builtin_amdgcn_readfirstlane(l_any);
    constexpr int WB = W8 ? 1 : 2;
    constexpr int RBQ = W8 ? 8 : 4, RBO = W8 ? 16 : 8, RB1 = (ITH == 1 ? 8 : 4) * (W8 ? 2 : 1), RB2 = W8 ? 16 : 8;
    using WV = typename std::conditional<W8, uint2, uint4>::type;
    constexpr int RED = 2 * RB1 > RBO ? 2 * RB1 : RBO;
    __shared__ float red[8][RED];
    __shared__ float ssq[8];
    __shared__ float xs[4096];
    __shared__ f32x4 accs[4][8][64];
    __shared__ float ms[8][16], ls[8][16];
    __shared__ float2 rope_s[64];
    const int nwg = (int)gridDim.x - 1;      // the last workgroup keeps the windows' time
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, i = lane & 15, q4 = lane >> 4;
    const int H = a.H, F = a.F, QR = a.QR, QD = a.QD, nq = a.nq, nkv = a.nkv, G = nq / nkv, nc = a.n_chunks;
    auto ldw = [](const char *p) __attribute__((always_inline)) {
        if constexpr (W8) {
            const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(p));
            return make_uint2(v.x, v.y);
        } else {
            const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
            return make_uint4(v.x, v.y, v.z, v.w);
        }
    };
    // ---- geometry of the four projections (rows dealt to thread groups in balanced contiguous ranges)
    struct Geo { int gs, groups, wpg, gid, lg, rb, re; };
    auto geo = [&](SegGeom g, int which) __attribute__((always_inline)) {
        Geo o;
        o.gs = 1 << g.gs_log2; o.groups = 512 >> g.gs_log2; o.wpg = o.gs >> 6;
        o.gid = tid >> g.gs_log2; o.lg = tid & (o.gs - 1);
        o.rb = st.rb[which]; o.re = st.re[which];
        return o;
    };
    const Geo gq = geo(a.gq, 0), go = geo(a.go, 1), g1 = geo(a.g1, 2), g2 = geo(a.g2, 3);
    int kh[ITH], kf[IT2];       // this thread's columns of a K = H row (QKV and gate/up share the map) and of a K = F row
    bool okh[ITH], okf[IT2];
#pragma unroll
    for (int it = 0; it < ITH; ++it) {
        kh[it] = (it * gq.gs + gq.lg) * 8;
        okh[it] = kh[it] < H;
    }
#pragma unroll
    for (int it = 0; it < IT2; ++it) {
        kf[it] = (it * g2.gs + g2.lg) * 8;
        okf[it] = kf[it] < F;
    }
    const int ko = go.lg * 8;
    const bool oko = ko < QD;
    // ---- attention role (the same in every layer)
    const bool att = (int)blockIdx.x < nkv * nc;
    const int kvh = att ? (int)blockIdx.x / nc : 0, c = att ? (int)blockIdx.x % nc : 0;
    int T = a.seq_lens[0];
    if (T < 0 || T > a.max_tokens) T = 0;
    const int t_begin = c * 256, t_end = min(T, t_begin + 256);
    const int t0 = t_begin + wave * kAttnTileTokens;
    const bool early = att && t0 < a.max_blocks * 16;
    const int tau1 = 8 * (i >> 2) + (i & 3);
    const int blkA = st.blkA, blkB = st.blkB;
    if (att && tid < 64) rope_s[tid] = a.rope[tid];      // read after the barriers of the normalisation
    float res[ITH][8];
#pragma unroll
    for (int it = 0; it < ITH; ++it)
#pragma unroll
        for (int e = 0; e < 8; ++e) res[it][e] = st.res[it][e];
    bool lost = false;
    auto leave = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < ITH; ++it)
#pragma unroll
            for (int e = 0; e < 8; ++e) st.res[it][e] = res[it][e];
        if (lost) st.lost = 1;
    };

    const bool last = l == a.le;
    const StepLayer L = a.layers[last ? a.lb : l];
    // waits (bounded) until the tagged word `slot` of done_ll carries `tag`; wave 0 polls, the others wait at the barrier
    auto wait_window = [&](int slot, unsigned tag) __attribute__((always_inline)) {
        if (wave == 0) {
            uint2 v;
            bool ok = false;
            for (uint32_t spin = 0; !ok && spin < a.ll_iters; ++spin) {
                ll_issue1(v, a.done_ll + slot);
                asm volatile("s_waitcnt vmcnt(0)" : "+v"(v) : : "memory");
                ok = v.y == tag;
                if (!ok) __builtin_amdgcn_s_sleep(8);
            }
            if (!ok) lost = true;
        }
        __syncthreads();
    };
    // adds the tagged projection output `buf` (K = H values) to the residual registers
    auto add_delta = [&](const uint2 *buf, unsigned tag) __attribute__((always_inline)) {
        float d[ITH][8];
        bool all = false;
        for (uint32_t spin = 0; !all && spin < a.ll_iters; ++spin) {
            u32x4 q[ITH][4];
#pragma unroll
            for (int it = 0; it < ITH; ++it)
#pragma unroll
                for (int u = 0; u < 4; ++u) ll_issue(q[it][u], buf + (okh[it] ? kh[it] : 0) + 2 * u);
            ll_wait_all();
            bool mine = true;
#pragma unroll
            for (int it = 0; it < ITH; ++it)
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    asm volatile("" : "+v"(q[it][u]));
                    if (q[it][u].y != tag || q[it][u].w != tag) mine = false;
                    d[it][2 * u] = __uint_as_float(q[it][u].x);
                    d[it][2 * u + 1] = __uint_as_float(q[it][u].z);
                }
            all = __all(mine);
            if (!all) __builtin_amdgcn_s_sleep(2);
        }
        if (!all) lost = true;
#pragma unroll
        for (int it = 0; it < ITH; ++it)
            if (okh[it])
#pragma unroll
                for (int e = 0; e < 8; ++e) res[it][e] += d[it][e];
    };
    // xv = rmsnorm(res) * gain; workgroup 0 stores the residual and the normalised vector (debug aids)
    auto normalise = [&](const uint16_t *gain, float (&xv)[ITH][8], float *dbg_res, float *dbg_h) __attribute__((always_inline)) {
        uint4 gv[ITH];
        float ss = 0.f;
#pragma unroll
        for (int it = 0; it < ITH; ++it) {
            gv[it] = okh[it] ? ld16(gain + kh[it]) : zero16();
#pragma unroll
            for (int e = 0; e < 8; ++e) ss += res[it][e] * res[it][e];
            if (blockIdx.x == 0 && gq.gid == 0 && okh[it] && dbg_res) {
                *reinterpret_cast<float4 *>(dbg_res + kh[it]) = make_float4(res[it][0], res[it][1], res[it][2], res[it][3]);
                *reinterpret_cast<float4 *>(dbg_res + kh[it] + 4) = make_float4(res[it][4], res[it][5], res[it][6], res[it][7]);
            }
        }
        ss = wave_sum(ss);
        __syncthreads();                 // ssq may still be read by a slow wave of the previous block
        if (lane == 0) ssq[wave] = ss;
        __syncthreads();
        float tot = 0.f;
        for (int w = 0; w < gq.wpg; ++w) tot += ssq[gq.gid * gq.wpg + w];   // fixed order
        const float inv = 1.0f / sqrtf(tot / (float)H + a.eps);
#pragma unroll
        for (int it = 0; it < ITH; ++it) {
            const uint4 g = gv[it];
            float *x = xv[it];
            x[0] = res[it][0] * (inv * bf16_lo(g.x)); x[1] = res[it][1] * (inv * bf16_hi(g.x));
            x[2] = res[it][2] * (inv * bf16_lo(g.y)); x[3] = res[it][3] * (inv * bf16_hi(g.y));
            x[4] = res[it][4] * (inv * bf16_lo(g.z)); x[5] = res[it][5] * (inv * bf16_hi(g.z));
            x[6] = res[it][6] * (inv * bf16_lo(g.w)); x[7] = res[it][7] * (inv * bf16_hi(g.w));
            if (blockIdx.x == 0 && gq.gid == 0 && okh[it] && dbg_h) {
                *reinterpret_cast<float4 *>(dbg_h + kh[it]) = make_float4(x[0], x[1], x[2], x[3]);
                *reinterpret_cast<float4 *>(dbg_h + kh[it] + 4) = make_float4(x[4], x[5], x[6], x[7]);
            }
        }
    };

    const unsigned tag0 = a.tag_base + (unsigned)(l - a.lb) * TAGS_PER_LAYER;
    const char *Wq = static_cast<const char *>(L.Wq), *Wo = static_cast<const char *>(L.Wo);
    const char *Wg = static_cast<const char *>(L.Wg), *Wu = static_cast<const char *>(L.Wu), *Wd = static_cast<const char *>(L.Wd);

    // =================================================================== attention block
    WV wq[ITH][RBQ], wo[RBO];
    uint4 ka[4], kb[4], vf[8];
    float scq = 0.f, sco = 0.f;
    auto load_q = [&](int r0) __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < ITH; ++it) {
            const int col = okh[it] ? kh[it] : 0;
#pragma unroll
            for (int r = 0; r < RBQ; ++r) {
                const int row = max(min(r0 + r, gq.re - 1), 0);
                const WV v = ldw(Wq + ((size_t)row * H + col) * WB);
                wq[it][r] = okh[it] ? v : WV{};
            }
        }
        if (W8 && gq.lg < RBQ && r0 + gq.lg < gq.re) scq = L.sq[r0 + gq.lg];
    };
    auto load_o = [&](int r0) __attribute__((always_inline)) {
        const int col = oko ? ko : 0;
#pragma unroll
        for (int r = 0; r < RBO; ++r) {
            const int row = max(min(r0 + r, go.re - 1), 0);
            const WV v = ldw(Wo + ((size_t)row * QD + col) * WB);
            wo[r] = oko ? v : WV{};
        }
        if (W8 && go.lg < RBO && r0 + go.lg < go.re) sco = L.so[r0 + go.lg];
    };
    auto load_tile = [&]() __attribute__((always_inline)) {
        {
            const int blk = (i < 8) ? blkA : blkB;
            if (blk >= 0) {
                const uint16_t *base = L.k_pool + (((size_t)blk * nkv + kvh) * 16 + (tau1 & 15)) * 128 + q4 * 8;
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    ka[ks] = ld16(base + ks * 32);
                    kb[ks] = ld16(base + 4 * 128 + ks * 32);
                }
            } else {
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) { ka[ks] = zero16(); kb[ks] = zero16(); }
            }
        }
        {
            const int blk = (q4 < 2) ? blkA : blkB;
            if (blk >= 0) {
                const uint16_t *base = L.v_pool + (((size_t)blk * nkv + kvh) * 128 + i) * 16 + (q4 & 1) * 8;
#pragma unroll
                for (int dg = 0; dg < 8; ++dg) vf[dg] = ld16(base + dg * 16 * 16);
            } else {
#pragma unroll
                for (int dg = 0; dg < 8; ++dg) vf[dg] = zero16();
            }
        }
    };
    {
        const bool first = l == a.lb;
        const bool win = !first && a.ticks[1] > 0;            // the previous layer's second window precedes this block
        const int hold = last ? 0 : (win ? a.hold[1] : 7);
        int rq = gq.rb, ro = go.rb;
        if (hold & 1) load_q(rq);
        if (hold & 4) load_o(ro);
        if (early && (hold & 2)) load_tile();
        if (win) wait_window(1, tag0 - TAGS_PER_LAYER + TAG_WIN1);
        if (!first) add_delta(a.dm_ll, tag0 - TAGS_PER_LAYER + TAG_DM);
        if (last) {                  // the step's output
            if (blockIdx.x == 0 && gq.gid == 0)
#pragma unroll
                for (int it = 0; it < ITH; ++it)
                    if (okh[it]) {
                        *reinterpret_cast<float4 *>(a.x_out + kh[it]) = make_float4(res[it][0], res[it][1], res[it][2], res[it][3]);
                        *reinterpret_cast<float4 *>(a.x_out + kh[it] + 4) = make_float4(res[it][4], res[it][5], res[it][6], res[it][7]);
                    }
            leave();
            return;
        }
        if (!(hold & 1)) load_q(rq);
        if (!(hold & 4)) load_o(ro);
        if (early && !(hold & 2)) load_tile();
        float xv[ITH][8];
        normalise(L.g_attn, xv, a.dbg_x, a.dbg_h1);

        // ---- QKV rows -> tagged
        for (int pass = 0; pass < a.gq.passes; ++pass) {
            float acc[RBQ];
#pragma unroll
            for (int r = 0; r < RBQ; ++r) {
                float s = 0.f;
#pragma unroll
                for (int it = 0; it < ITH; ++it) s = dot8(wq[it][r], xv[it], s);
                acc[r] = wave_sum(s);
            }
            const int rows_here = rq;
            rq += RBQ;
            const float sc_now = scq;
            if (pass + 1 < a.gq.passes) load_q(rq);
            if (gq.wpg == 1) {
                if (lane == 0)
#pragma unroll
                    for (int r = 0; r < RBQ; ++r)
                        if (rows_here + r < gq.re) {
                            float v = acc[r];
                            if (W8) v *= L.sq[rows_here + r];
                            ll_store(a.qkv_ll + rows_here + r, v, tag0 + TAG_QKV);
                        }
            } else {
                if (lane == 0)
#pragma unroll
                    for (int r = 0; r < RBQ; ++r) red[wave][r] = acc[r];
                __syncthreads();
                if (gq.lg < RBQ && rows_here + gq.lg < gq.re) {
                    float v = 0.f;
                    for (int w = 0; w < gq.wpg; ++w) v += red[gq.gid * gq.wpg + w][gq.lg];   // fixed order
                    if (W8) v *= sc_now;
                    ll_store(a.qkv_ll + rows_here + gq.lg, v, tag0 + TAG_QKV);
                }
                __syncthreads();
            }
        }

        // ---- attention of this workgroup's chunk (see k_seg_attn)
        if (att) {
            bf16x8 qf[4], qfl[4];
            {
                const uint4 z = zero16();
                qf[0] = qf[1] = qf[2] = qf[3] = __builtin_bit_cast(bf16x8, z);
                qfl[0] = qfl[1] = qfl[2] = qfl[3] = __builtin_bit_cast(bf16x8, z);
                float *qs = xs;                               // [G + 2][128]
                const int n_val = (G + 2) * 128;
                bool all = false;
                for (uint32_t spin = 0; !all && spin < a.ll_iters; ++spin) {
                    bool mine = true;
                    uint2 pv[5];
#pragma unroll
                    for (int u = 0; u < 5; ++u) {
                        const int v0 = tid + 512 * u;
                        if (v0 < n_val) {
                            const int hrow = v0 >> 7;
                            const int row = hrow < G ? kvh * G + hrow : (hrow == G ? nq + kvh : nq + nkv + kvh);
                            ll_issue1(pv[u], a.qkv_ll + (size_t)row * 128 + (v0 & 127));
                        }
                    }
                    ll_wait_all();
#pragma unroll
                    for (int u = 0; u < 5; ++u) {
                        const int v0 = tid + 512 * u;
                        if (v0 < n_val) {
                            asm volatile("" : "+v"(pv[u]));
                            if (pv[u].y != tag0 + TAG_QKV) mine = false;
                            qs[v0] = __uint_as_float(pv[u].x);
                        }
                    }
                    all = __syncthreads_and(mine ? 1 : 0) != 0;
                    if (!all) __builtin_amdgcn_s_sleep(2);
                }
                if (!all) lost = true;
                if (i < G) {
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) {
                        const int f0 = ks * 32 + q4 * 8;
                        const float *lo = qs + i * 128 + f0, *hi = lo + 64;
                        uint32_t lh[4], ll[4], hh[4], hl[4];
#pragma unroll
                        for (int e = 0; e < 8; e += 2) {
                            const float2 c0 = rope_s[f0 + e], c1 = rope_s[f0 + e + 1];
                            pack_split(lo[e] * c0.x - hi[e] * c0.y, lo[e + 1] * c1.x - hi[e + 1] * c1.y, lh[e >> 1], ll[e >> 1]);
                            pack_split(hi[e] * c0.x + lo[e] * c0.y, hi[e + 1] * c1.x + lo[e + 1] * c1.y, hh[e >> 1], hl[e >> 1]);
                        }
                        qf[ks] = __builtin_bit_cast(bf16x8, make_uint4(lh[0], lh[1], lh[2], lh[3]));
                        qfl[ks] = __builtin_bit_cast(bf16x8, make_uint4(ll[0], ll[1], ll[2], ll[3]));
                        qf[ks + 2] = __builtin_bit_cast(bf16x8, make_uint4(hh[0], hh[1], hh[2], hh[3]));
                        qfl[ks + 2] = __builtin_bit_cast(bf16x8, make_uint4(hl[0], hl[1], hl[2], hl[3]));
                    }
                }
            }
            if (T >= 1 && c == (T - 1) / 256) {          // append the new token's K and V
                if (wave == 0) {
                    const int pos = T - 1;
                    const int blk = kv_phys_block(a.page_table, a.max_blocks, a.num_pool_blocks, 0, pos >> 4);
                    if (blk >= 0) {
                        const float2 cs = rope_s[lane];
                        const float *ksrc = xs + G * 128, *vsrc = xs + (G + 1) * 128;
                        const float lo = ksrc[lane], hi = ksrc[lane + 64];
                        const int r = pos & 15;
                        uint16_t *kdst = L.k_pool + (((size_t)blk * nkv + kvh) * 16 + r) * 128;
                        kdst[lane] = (uint16_t)f32_to_bf16(lo * cs.x - hi * cs.y);
                        kdst[lane + 64] = (uint16_t)f32_to_bf16(hi * cs.x + lo * cs.y);
                        uint16_t *vdst = L.v_pool + ((size_t)blk * nkv + kvh) * 128 * 16 + r;
                        vdst[(size_t)lane * 16] = (uint16_t)f32_to_bf16(vsrc[lane]);
                        vdst[(size_t)(lane + 64) * 16] = (uint16_t)f32_to_bf16(vsrc[lane + 64]);
                    }
                    __threadfence();
                }
                __syncthreads();
                if (early && T - 1 >= t0 && T - 1 < t0 + kAttnTileTokens) load_tile();
            }
            const float kScale = 0.08838834764831845f * 1.4426950408889634f;   // 1/sqrt(128) * log2(e)
            float m_run = -1.0e30f, l_part = 0.f;
            f32x4 acc[8];
#pragma unroll
            for (int dg = 0; dg < 8; ++dg) acc[dg] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (t0 < t_end) {
                f32x4 s1 = {0.f, 0.f, 0.f, 0.f}, s2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[ks]), qfl[ks], s1, 0, 0, 0);
                    s2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kb[ks]), qfl[ks], s2, 0, 0, 0);
                    s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[ks]), qf[ks], s1, 0, 0, 0);
                    s2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kb[ks]), qf[ks], s2, 0, 0, 0);
                }
                float sv[8];
                const int tl = t0 + 8 * q4;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    sv[e] = (tl + e < t_end) ? s1[e] * kScale : -INFINITY;
                    sv[e + 4] = (tl + e + 4 < t_end) ? s2[e] * kScale : -INFINITY;
                }
                float tmax = sv[0];
#pragma unroll
                for (int e = 1; e < 8; ++e) tmax = fmaxf(tmax, sv[e]);
                tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
                tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
                m_run = fmaxf(m_run, tmax);
                float p[8], psum = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    p[e] = exp2f(sv[e] - m_run);
                    psum += p[e];
                }
                l_part = psum;
                uint4 pk, pkl;
                pack_split(p[0], p[1], pk.x, pkl.x);
                pack_split(p[2], p[3], pk.y, pkl.y);
                pack_split(p[4], p[5], pk.z, pkl.z);
                pack_split(p[6], p[7], pk.w, pkl.w);
                if (t0 + kAttnTileTokens > t_end) {   // ragged tail: blank cache slots past the span
                    uint32_t mlo[4];
#pragma unroll
                    for (int h = 0; h < 4; ++h) {
                        const uint32_t m0 = (tl + 2 * h < t_end) ? 0x0000ffffu : 0u;
                        const uint32_t m1 = (tl + 2 * h + 1 < t_end) ? 0xffff0000u : 0u;
                        mlo[h] = m0 | m1;
                    }
#pragma unroll
                    for (int dg = 0; dg < 8; ++dg) {
                        vf[dg].x &= mlo[0]; vf[dg].y &= mlo[1]; vf[dg].z &= mlo[2]; vf[dg].w &= mlo[3];
                    }
                }
                const bf16x8 pfrag = __builtin_bit_cast(bf16x8, pk), pfrag_lo = __builtin_bit_cast(bf16x8, pkl);
#pragma unroll
                for (int dg = 0; dg < 8; ++dg) {
                    acc[dg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vf[dg]), pfrag_lo, acc[dg], 0, 0, 0);
                    acc[dg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vf[dg]), pfrag, acc[dg], 0, 0, 0);
                }
            }
            // merge of the 8 waves: common maximum, fixed summation order
            l_part += __shfl_xor(l_part, 16, 64);
            l_part += __shfl_xor(l_part, 32, 64);
            if (q4 == 0) ms[wave][i] = m_run;
            __syncthreads();
            float M = ms[0][i];
#pragma unroll
            for (int w = 1; w < 8; ++w) M = fmaxf(M, ms[w][i]);
            const float scl = exp2f(m_run - M);
            if (q4 == 0) ls[wave][i] = l_part * scl;
#pragma unroll
            for (int dg = 0; dg < 8; ++dg) acc[dg] *= scl;
            if (wave >= 4)
#pragma unroll
                for (int dg = 0; dg < 8; ++dg) accs[wave - 4][dg][lane] = acc[dg];
            __syncthreads();
            if (wave < 4)
#pragma unroll
                for (int dg = 0; dg < 8; ++dg) acc[dg] += accs[wave][dg][lane];
            __syncthreads();
            if (wave < 4)
#pragma unroll
                for (int dg = 0; dg < 8; ++dg) accs[wave][dg][lane] = acc[dg];
            __syncthreads();
            if (i < G) {
                const size_t slot = (size_t)kvh * nc + c;
                if (wave == 0 && q4 == 0) {
                    float Lsum = ls[0][i];
#pragma unroll
                    for (int w = 1; w < 8; ++w) Lsum += ls[w][i];
                    ll_store(a.pml_ll + (slot * 16 + i) * 2, M, tag0 + TAG_PART);
                    ll_store(a.pml_ll + (slot * 16 + i) * 2 + 1, Lsum, tag0 + TAG_PART);
                }
                const f32x4 v = (accs[0][wave][lane] + accs[1][wave][lane]) + (accs[2][wave][lane] + accs[3][wave][lane]);
                uint2 *dst = a.po_ll + (slot * G + i) * 128 + wave * 16 + 4 * q4;
#pragma unroll
                for (int j = 0; j < 4; ++j) ll_store(dst + j, v[j], tag0 + TAG_PART);
            }
            __syncthreads();                 // xs and accs are reused below
        }

        // ---- merge of the chunk partials (once per workgroup, into LDS), then the O rows -> tagged
        {
            constexpr int MB = 8;
            if (wave == 0) {
                const int n_part = nkv * nc;
                bool all = false;
                for (uint32_t spin = 0; !all && spin < a.ll_iters; ++spin) {
                    bool mine = true;
                    for (int pi = lane; pi < n_part; pi += 64) {
                        uint2 v;
                        ll_issue1(v, a.po_ll + ((size_t)pi * G + (G - 1)) * 128 + 127);
                        asm volatile("s_waitcnt vmcnt(0)" : "+v"(v) : : "memory");
                        if (v.y != tag0 + TAG_PART) mine = false;
                    }
                    all = __all(mine);
                    if (!all) __builtin_amdgcn_s_sleep(8);
                }
            }
            __syncthreads();
            for (int ch = tid; ch < QD; ch += 512) {
                const int j = ch >> 7, c7 = ch & 127, hk = j / G, g = j % G;
                const uint2 *mlp = a.pml_ll + (((size_t)hk * nc) * 16 + g) * 2;
                const uint2 *op = a.po_ll + (((size_t)hk * nc) * G + g) * 128 + c7;
                float Mx = -1.0e30f, den = 0.f, num = 0.f;
                for (int sp0 = 0; sp0 < nc; sp0 += MB) {
                    u32x4 ml[MB];
                    uint2 ov[MB];
                    bool all = false;
                    for (uint32_t spin = 0; !all && spin < a.ll_iters; ++spin) {
#pragma unroll
                        for (int u = 0; u < MB; ++u) {
                            const int sp = min(sp0 + u, nc - 1);
                            ll_issue(ml[u], mlp + (size_t)sp * 32);
                            ll_issue1(ov[u], op + (size_t)sp * G * 128);
                        }
                        ll_wait_all();
                        bool mine = true;
#pragma unroll
                        for (int u = 0; u < MB; ++u) {
                            asm volatile("" : "+v"(ml[u]), "+v"(ov[u]));
                            if (ml[u].y != tag0 + TAG_PART || ml[u].w != tag0 + TAG_PART || ov[u].y != tag0 + TAG_PART) mine = false;
                        }
                        all = __all(mine);
                        if (!all) __builtin_amdgcn_s_sleep(4);
                    }
                    if (!all) lost = true;
                    float bm = Mx;
#pragma unroll
                    for (int u = 0; u < MB; ++u)
                        if (sp0 + u < nc) bm = fmaxf(bm, __uint_as_float(ml[u].x));
                    const float rs = exp2f(Mx - bm);
                    Mx = bm;
                    den *= rs;
                    num *= rs;
#pragma unroll
                    for (int u = 0; u < MB; ++u)
                        if (sp0 + u < nc) {
                            const float lsum = __uint_as_float(ml[u].z);
                            const float wgt = lsum > 0.f ? exp2f(__uint_as_float(ml[u].x) - Mx) : 0.f;
                            den += wgt * lsum;
                            num = fmaf(wgt, __uint_as_float(ov[u].x), num);
                        }
                }
                const float r = den > 0.f ? num / den : 0.f;
                xs[ch] = r;
                if (blockIdx.x == 0 && a.dbg_attn) a.dbg_attn[ch] = r;
            }
            __syncthreads();
            float xo[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) xo[e] = oko ? xs[ko + e] : 0.f;
            for (int pass = 0; pass < a.go.passes; ++pass) {
                float acc[RBO];
#pragma unroll
                for (int r = 0; r < RBO; ++r) acc[r] = wave_sum(dot8(wo[r], xo, 0.f));
                const int rows_here = ro;
                ro += RBO;
                const float sc_now = sco;
                if (pass + 1 < a.go.passes) load_o(ro);
                if (go.wpg == 1) {
                    if (lane == 0)
#pragma unroll
                        for (int r = 0; r < RBO; ++r)
                            if (rows_here + r < go.re) {
                                float v = acc[r];
                                if (W8) v *= L.so[rows_here + r];
                                ll_store(a.da_ll + rows_here + r, v, tag0 + TAG_DA);
                            }
                } else {
                    if (lane == 0)
#pragma unroll
                        for (int r = 0; r < RBO; ++r) red[wave][r] = acc[r];
                    __syncthreads();
                    if (go.lg < RBO && rows_here + go.lg < go.re) {
                        float v = 0.f;
                        for (int w = 0; w < go.wpg; ++w) v += red[go.gid * go.wpg + w][go.lg];   // fixed order
                        if (W8) v *= sc_now;
                        ll_store(a.da_ll + rows_here + go.lg, v, tag0 + TAG_DA);
                    }
                    __syncthreads();
                }
            }
        }
    }

    // =================================================================== MLP block
    {
        WV w1[ITH][2][RB1], w2[IT2][RB2];
        float sc1[2] = {0.f, 0.f}, sc2 = 0.f;
        auto load1 = [&](int r0) __attribute__((always_inline)) {
#pragma unroll
            for (int it = 0; it < ITH; ++it) {
                const int col = okh[it] ? kh[it] : 0;
#pragma unroll
                for (int r = 0; r < RB1; ++r) {
                    const int row = max(min(r0 + r, g1.re - 1), 0);
                    const size_t off = ((size_t)row * H + col) * WB;
                    const WV g = ldw(Wg + off), u = ldw(Wu + off);
                    w1[it][0][r] = okh[it] ? g : WV{};
                    w1[it][1][r] = okh[it] ? u : WV{};
                }
            }
            const int my = g1.lg;
            if (W8 && my < RB1 && r0 + my < g1.re) {
                sc1[0] = L.sg[r0 + my];
                sc1[1] = L.su[r0 + my];
            }
        };
        auto load2 = [&](int r0) __attribute__((always_inline)) {
#pragma unroll
            for (int it = 0; it < IT2; ++it) {
                const int col = okf[it] ? kf[it] : 0;
#pragma unroll
                for (int r = 0; r < RB2; ++r) {
                    const int row = max(min(r0 + r, g2.re - 1), 0);
                    const WV d = ldw(Wd + ((size_t)row * F + col) * WB);
                    w2[it][r] = okf[it] ? d : WV{};
                }
            }
            if (W8 && g2.lg < RB2 && r0 + g2.lg < g2.re) sc2 = L.sd[r0 + g2.lg];
        };
        const bool win = a.ticks[0] > 0;
        const int hold = win ? a.hold[0] : 3;
        int r1 = g1.rb, r2 = g2.rb;
        if (hold & 1) load1(r1);
        if (hold & 2) load2(r2);
        if (win) wait_window(0, tag0 + TAG_WIN0);
        if (!(hold & 1)) load1(r1);
        if (!(hold & 2)) load2(r2);
        add_delta(a.da_ll, tag0 + TAG_DA);
        float xv[ITH][8];
        normalise(L.g_mlp, xv, a.dbg_y, a.dbg_h2);

        // ---- gate/up rows, SwiGLU -> tagged
        for (int pass = 0; pass < a.g1.passes; ++pass) {
            float acc[2][RB1];
#pragma unroll
            for (int q = 0; q < 2; ++q)
#pragma unroll
                for (int r = 0; r < RB1; ++r) {
                    float s = 0.f;
#pragma unroll
                    for (int it = 0; it < ITH; ++it) s = dot8(w1[it][q][r], xv[it], s);
                    acc[q][r] = wave_sum(s);
                }
            const int rows_here = r1;
            r1 += RB1;
            const float sg_now = sc1[0], su_now = sc1[1];
            if (pass + 1 < a.g1.passes) load1(r1);
            if (g1.wpg == 1) {
                if (lane == 0)
#pragma unroll
                    for (int r = 0; r < RB1; ++r)
                        if (rows_here + r < g1.re) {
                            float v = acc[0][r], u = acc[1][r];
                            if (W8) {
                                v *= L.sg[rows_here + r];
                                u *= L.su[rows_here + r];
                            }
                            ll_store(a.m_ll + rows_here + r, silu_mul(v, u), tag0 + TAG_M);
                        }
            } else {
                if (lane == 0)
#pragma unroll
                    for (int q = 0; q < 2; ++q)
#pragma unroll
                        for (int r = 0; r < RB1; ++r) red[wave][q * RB1 + r] = acc[q][r];
                __syncthreads();
                if (g1.lg < RB1 && rows_here + g1.lg < g1.re) {
                    float v = 0.f, u = 0.f;
                    for (int w = 0; w < g1.wpg; ++w) {   // fixed order
                        v += red[g1.gid * g1.wpg + w][g1.lg];
                        u += red[g1.gid * g1.wpg + w][RB1 + g1.lg];
                    }
                    if (W8) {
                        v *= sg_now;
                        u *= su_now;
                    }
                    ll_store(a.m_ll + rows_here + g1.lg, silu_mul(v, u), tag0 + TAG_M);
                }
                __syncthreads();
            }
        }

        // ---- hand-over of m: one wave watches the last row of every workgroup first, then everyone reads its slice
        float mv[IT2][8];
        {
            if (wave == 0) {
                const int slots1 = nwg * g1.groups;
                bool ready = false;
                for (uint32_t spin = 0; !ready && spin < a.ll_iters; ++spin) {
                    bool mine = true;
                    for (int p0 = 0; p0 < nwg; p0 += 256) {
                        uint2 v[4];
                        int pe[4];
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            const int wg = min(p0 + lane + 64 * u, nwg - 1);
                            pe[u] = (int)((long long)(wg + 1) * g1.groups * F / slots1);
                            ll_issue1(v[u], a.m_ll + max(pe[u] - 1, 0));
                        }
                        asm volatile("s_waitcnt vmcnt(0)" : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]) : : "memory");
#pragma unroll
                        for (int u = 0; u < 4; ++u)
                            if (pe[u] > 0 && v[u].y != tag0 + TAG_M) mine = false;
                    }
                    ready = __all(mine);
                    if (!ready) __builtin_amdgcn_s_sleep(8);
                }
            }
            __syncthreads();
            bool all = false;
            for (uint32_t spin = 0; !all && spin < a.ll_iters; ++spin) {
                u32x4 q[IT2][4];
#pragma unroll
                for (int it = 0; it < IT2; ++it)
#pragma unroll
                    for (int u = 0; u < 4; ++u) ll_issue(q[it][u], a.m_ll + (okf[it] ? kf[it] : 0) + 2 * u);
                ll_wait_all();
                bool mine = true;
#pragma unroll
                for (int it = 0; it < IT2; ++it)
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        asm volatile("" : "+v"(q[it][u]));
                        if (q[it][u].y != tag0 + TAG_M || q[it][u].w != tag0 + TAG_M) mine = false;
                        mv[it][2 * u] = okf[it] ? __uint_as_float(q[it][u].x) : 0.f;
                        mv[it][2 * u + 1] = okf[it] ? __uint_as_float(q[it][u].z) : 0.f;
                    }
                all = __all(mine);
                if (!all) __builtin_amdgcn_s_sleep(2);
            }
            if (!all) lost = true;
        }

        // ---- down rows -> tagged
        for (int pass = 0; pass < a.g2.passes; ++pass) {
            float acc[RB2];
#pragma unroll
            for (int r = 0; r < RB2; ++r) {
                float s = 0.f;
#pragma unroll
                for (int it = 0; it < IT2; ++it) s = dot8(w2[it][r], mv[it], s);
                acc[r] = wave_sum(s);
            }
            const int rows_here = r2;
            r2 += RB2;
            const float sd_now = sc2;
            if (pass + 1 < a.g2.passes) load2(r2);
            if (g2.wpg == 1) {
                if (lane == 0)
#pragma unroll
                    for (int r = 0; r < RB2; ++r)
                        if (rows_here + r < g2.re) {
                            float v = acc[r];
                            if (W8) v *= L.sd[rows_here + r];
                            ll_store(a.dm_ll + rows_here + r, v, tag0 + TAG_DM);
                        }
            } else {
                if (lane == 0)
#pragma unroll
                    for (int r = 0; r < RB2; ++r) red[wave][r] = acc[r];
                __syncthreads();
                if (g2.lg < RB2 && rows_here + g2.lg < g2.re) {
                    float v = 0.f;
                    for (int w = 0; w < g2.wpg; ++w) v += red[g2.gid * g2.wpg + w][g2.lg];   // fixed order
                    if (W8) v *= sd_now;
                    ll_store(a.dm_ll + rows_here + g2.lg, v, tag0 + TAG_DM);
                }
                __syncthreads();
            }
        }
    }
    leave();
}

template <int ITH, int IT2, bool W8>
__global__ __launch_bounds__(512) void k_step(StepArgs a)
{
    const int tid = threadIdx.x, wave = tid >> 6;
    const int nwg = (int)gridDim.x - 1;
    if ((int)blockIdx.x == nwg) {
        // ---- the stand-in for the collectives
        bool lost = false;
        auto window = [&](const uint2 *buf, unsigned tag, int w, unsigned tag_done) __attribute__((always_inline)) {
            bool all = false;           // the window starts when the block's whole output exists
            for (uint32_t spin = 0; !all && spin < a.ll_iters; ++spin) {
                bool mine = true;
                u32x4 q[8];             // H <= 8192: at most 8 pairs of values per thread, requested together
#pragma unroll
                for (int k = 0; k < 8; ++k) ll_issue(q[k], buf + 2 * min(tid + 512 * k, a.H / 2 - 1));
                ll_wait_all();
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    asm volatile("" : "+v"(q[k]));
                    if (q[k].y != tag || q[k].w != tag) mine = false;
                }
                all = __syncthreads_and(mine ? 1 : 0) != 0;
                if (!all) __builtin_amdgcn_s_sleep(4);
            }
            if (!all) lost = true;
            if (wave == 0) {
                const uint64_t ts = wall_clock64();
                uint32_t it = 0;
                while (wall_clock64() - ts < a.ticks[w] && it < a.spin_iters[w]) {
                    __builtin_amdgcn_s_sleep(2);
                    ++it;
                }
                if (tid == 0) ll_store(a.done_ll + w, 0.f, tag_done);
            }
        };
        for (int l = a.lb; l < a.le; ++l) {
            const unsigned tag0 = a.tag_base + (unsigned)(l - a.lb) * TAGS_PER_LAYER;
            if (a.ticks[0] > 0) window(a.da_ll, tag0 + TAG_DA, 0, tag0 + TAG_WIN0);
            if (a.ticks[1] > 0) window(a.dm_ll, tag0 + TAG_DM, 1, tag0 + TAG_WIN1);
        }
        if (__any(lost) && (tid & 63) == 0) atomicOr(a.err, 2u);
        return;
    }
    StepState<ITH> st;
    {
        const SegGeom gs[4] = {a.gq, a.go, a.g1, a.g2};
        const int Ns[4] = {a.QR, a.H, a.F, a.H};
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int groups = 512 >> gs[p].gs_log2, gid = tid >> gs[p].gs_log2;
            const int slots = nwg * groups, slot = blockIdx.x * groups + gid;
            st.rb[p] = (int)((long long)slot * Ns[p] / slots);
            st.re[p] = (int)((long long)(slot + 1) * Ns[p] / slots);
        }
        const int lg = tid & ((1 << a.gq.gs_log2) - 1), gsz = 1 << a.gq.gs_log2;
#pragma unroll
        for (int it = 0; it < ITH; ++it) {
            const int k = (it * gsz + lg) * 8;
            float4 v0 = make_float4(0.f, 0.f, 0.f, 0.f), v1 = v0;
            if (k < a.H) {
                v0 = *reinterpret_cast<const float4 *>(a.x_in + k);
                v1 = *reinterpret_cast<const float4 *>(a.x_in + k + 4);
            }
            st.res[it][0] = v0.x; st.res[it][1] = v0.y; st.res[it][2] = v0.z; st.res[it][3] = v0.w;
            st.res[it][4] = v1.x; st.res[it][5] = v1.y; st.res[it][6] = v1.z; st.res[it][7] = v1.w;
        }
    }
    st.blkA = st.blkB = -1;
    st.lost = 0;
    {
        const int nc = a.n_chunks;
        const bool att = (int)blockIdx.x < a.nkv * nc;
        const int t0 = (att ? (int)blockIdx.x % nc : 0) * 256 + wave * kAttnTileTokens;
        if (att && t0 < a.max_blocks * 16) {
            const int lb = t0 >> 4;
            st.blkA = kv_phys_block(a.page_table, a.max_blocks, a.num_pool_blocks, 0, lb);
            st.blkB = (lb + 1 < a.max_blocks) ? kv_phys_block(a.page_table, a.max_blocks, a.num_pool_blocks, 0, lb + 1) : -1;
        }
    }
    // the explicit arguments are the start of the kernel-argument segment
    const uint64_t kernarg = (uint64_t)__builtin_amdgcn_kernarg_segment_ptr();
    for (int l = a.lb; l <= a.le; ++l) step_layer<ITH, IT2, W8>(st, l, kernarg);
    if (__any(st.lost != 0) && (tid & 63) == 0) atomicOr(a.err, 2u);
}

// Shapes the fused kernels take, and every group of threads of every workgroup owns at least one row of every
// projection: then each workgroup takes part in every hand-over and none can fall a whole layer behind the others
// (a buffer of tagged values is written again one layer later).
bool step_supported(int batch, int H, int F, int nq, int nkv, uint32_t max_seq, bool other_cache, bool w8, int blocks)
{
    if (!seg_attn_supported(batch, H, nq, nkv, max_seq, other_cache, blocks) || !seg_mlp_supported(batch, H, F)) return false;
    const int QR = (nq + 2 * nkv) * 128, QD = nq * 128, ith = H > 4096 ? 2 : 1, it2 = F > 4096 ? 2 : 1;
    const int nwg = blocks - 1;                    // one workgroup keeps the windows' time
    if (nwg < 1 || nkv * seg_attn_chunks(max_seq) > nwg) return false;
    const SegGeom gq = seg_geom(QR, H, ith, w8 ? 8 : 4, nwg), go = seg_geom(H, QD, 1, w8 ? 16 : 8, nwg);
    const SegGeom g1 = seg_geom(F, H, ith, 8, nwg), g2 = seg_geom(H, F, it2, w8 ? 16 : 8, nwg);
    auto slots = [&](SegGeom g) { return (long long)nwg * (512 >> g.gs_log2); };
    return QR >= slots(gq) && H >= slots(go) && F >= slots(g1) && H >= slots(g2);
}

template <int ITH, int IT2, bool W8>
static hipError_t step_go(StepArgs a, int blocks, hipStream_t s)
{
    constexpr int RBQ = W8 ? 8 : 4, RBO = W8 ? 16 : 8, RB1 = (ITH == 1 ? 8 : 4) * (W8 ? 2 : 1), RB2 = W8 ? 16 : 8;
    a.gq = seg_geom(a.QR, a.H, ITH, RBQ, blocks - 1);      // the last workgroup computes nothing
    a.go = seg_geom(a.H, a.QD, 1, RBO, blocks - 1);
    a.g1 = seg_geom(a.F, a.H, ITH, RB1, blocks - 1);
    a.g2 = seg_geom(a.H, a.F, IT2, RB2, blocks - 1);
    PSV_LAUNCH((k_step<ITH, IT2, W8>), dim3(blocks), dim3(512), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_step(const StepLaunch &p, int blocks, hipStream_t s)
{
    StepArgs a{};
    a.layers = static_cast<const StepLayer *>(p.layer_table);
    a.lb = p.lb; a.le = p.le; a.x_in = p.x_in; a.x_out = p.x_out;
    a.H = p.H; a.F = p.F; a.nq = p.nq; a.nkv = p.nkv; a.QR = (p.nq + 2 * p.nkv) * 128; a.QD = p.nq * 128; a.n_chunks = p.n_chunks;
    a.eps = p.eps; a.rope = p.rope;
    a.page_table = p.kv.page_table; a.max_blocks = p.kv.max_blocks; a.max_tokens = p.kv.max_tokens;
    a.num_pool_blocks = p.kv.num_pool_blocks; a.seq_lens = p.kv.seq_lens;
    uint2 *ll = static_cast<uint2 *>(p.ll_base);
    a.qkv_ll = static_cast<uint2 *>(p.qkv_ll); a.pml_ll = static_cast<uint2 *>(p.pml_ll); a.po_ll = static_cast<uint2 *>(p.po_ll);
    a.m_ll = static_cast<uint2 *>(p.m_ll);
    a.da_ll = ll; a.dm_ll = ll + p.H; a.done_ll = ll + 2 * (size_t)p.H;
    a.tag_base = p.tag_base; a.ll_iters = p.poll_iters; a.err = p.err;
    a.ticks[0] = p.ticks[0]; a.ticks[1] = p.ticks[1]; a.spin_iters[0] = p.spin_iters[0]; a.spin_iters[1] = p.spin_iters[1];
    a.hold[0] = p.hold[0]; a.hold[1] = p.hold[1];
    a.dbg_x = p.dbg_x; a.dbg_h1 = p.dbg_h1; a.dbg_attn = p.dbg_attn; a.dbg_y = p.dbg_y; a.dbg_h2 = p.dbg_h2;
    const bool two_h = p.H > 4096, two_f = p.F > 4096;
    if (p.w8) {
        if (two_h) return two_f ? step_go<2, 2, true>(a, blocks, s) : step_go<2, 1, true>(a, blocks, s);
        return two_f ? step_go<1, 2, true>(a, blocks, s) : step_go<1, 1, true>(a, blocks, s);
    }
    if (two_h) return two_f ? step_go<2, 2, false>(a, blocks, s) : step_go<2, 1, false>(a, blocks, s);
    return two_f ? step_go<1, 2, false>(a, blocks, s) : step_go<1, 1, false>(a, blocks, s);
}

}  // namespace psv

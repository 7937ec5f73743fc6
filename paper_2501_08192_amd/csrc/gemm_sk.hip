// gfx950 (MI355X, CDNA4) kernels of the PRESERVE decode step: the split-K projections on the matrix cores and the small kernels around them.
//
// Weights and the KV-cache are bf16 (or int8 codes with fp32 scales) in HBM; every accumulation is fp32.  The step
// is bound by HBM bandwidth (Section 2, "LLM decoding is memory BW-limited"), so the kernels are built around
// 16-byte-per-lane coalesced loads with many loads in flight per 64-lane wave; the matrix cores are used where a
// vector-ALU formulation would bind on arithmetic (batch > 2 projections, grouped-query attention).
#include "device.h"
#include "tagged.h"
#include "prefetch.h"

namespace psv {

// ------------------------------------------------------------------------------------ norm

// Residual add for the matrix-core path, spread over many workgroups: grid (H / 512, batch), one float4 per
// thread.  out_res = res + delta, where delta may be `delta_splits` split-K partials [split][batch][H] that are
// summed in split order.  With a gain, the kernel also prepares the next projection's operand without ever seeing
// a whole row: it stores out_res * gain as hi/lo bf16 planes and the sum of squares of its 512 outputs in
// ssq[batch][H / 512].  RMSNorm is linear in its 1/rms factor, so that projection runs on the unnormalised planes
// and multiplies its result by 1/rms of the batch row, which it forms from ssq (k_gemm_sk).
// SIGNAL: a projection launched ahead of this kernel is waiting for its outputs (k_gemm_sk<1, HOLD> or k_gemm_sk_i8<1, HOLD>, HOLD > 0).  Every
// output is stored written through to the memory side; once a workgroup's stores are acknowledged, its sum of squares goes out as a
// tagged value {sum, tag} (ssq_ll: kSkTagCopies copies of [H / 512][batch], stored by as many lanes at once), and the waiting
// kernel proceeds when every entry it polls carries the tag of this launch.  No fence and no counter: a release fence makes every wave write back its XCD's L2 and a device-scope
// counter serialises at the memory side -- measured 25-55 ns per workgroup either way, 7 us per layer at batch 8 and
// 25 us at batch 32.

template <bool SIGNAL>
__global__ __launch_bounds__(128) void k_resid_sum(const float *__restrict__ res, const float *__restrict__ delta,
                                                   int delta_splits, size_t delta_stride, int H,
                                                   float *__restrict__ out_res, const uint16_t *__restrict__ gain,
                                                   uint16_t *__restrict__ xg_bf16, size_t plane_stride,
                                                   int digits, float *__restrict__ ssq, uint2 *ssq_ll, unsigned ll_stride,
                                                   unsigned tag)
{
    __shared__ float red[2];
    const int b = blockIdx.y, tid = threadIdx.x;
    const int i = (blockIdx.x * 128 + tid) * 4;       // H is a multiple of 512: always inside the row
    const size_t at = (size_t)b * H + i;
    float4 v = *reinterpret_cast<const float4 *>(res + at);
    uint2 g = make_uint2(0u, 0u);
    if (gain) g = *reinterpret_cast<const uint2 *>(gain + i);
    if (delta) {
        const float *d = delta + at;
        // all loads of a group first (their latencies overlap), then the sum in split order.  The signalling variant runs
        // beside a full house of waiting workgroups and has to fit the registers they leave: groups of 8 instead of 16.
        constexpr int GR = SIGNAL ? 8 : kSkMaxSplits;
        float4 e = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int k0 = 0; k0 < kSkMaxSplits; k0 += GR) {
            if (k0 && k0 >= delta_splits) break;
            float4 t[GR];
#pragma unroll
            for (int ks = 0; ks < GR; ++ks)
                t[ks] = k0 + ks < delta_splits ? *reinterpret_cast<const float4 *>(d + (k0 + ks) * delta_stride)
                                               : make_float4(0.f, 0.f, 0.f, 0.f);
            if (k0 == 0) e = t[0];
#pragma unroll
            for (int ks = k0 ? 0 : 1; ks < GR; ++ks) { e.x += t[ks].x; e.y += t[ks].y; e.z += t[ks].z; e.w += t[ks].w; }
        }
        v.x += e.x; v.y += e.y; v.z += e.z; v.w += e.w;
    }
    if (SIGNAL) st_wt16(out_res + at, v);
    else *reinterpret_cast<float4 *>(out_res + at) = v;
    if (!gain) return;
    const float4 xg = make_float4(v.x * bf16_lo(g.x), v.y * bf16_hi(g.x), v.z * bf16_lo(g.y), v.w * bf16_hi(g.y));
    if (digits) {   // operand of an int8 projection
        store_digits4<SIGNAL>(reinterpret_cast<uint8_t *>(xg_bf16), plane_stride, H, (size_t)b, i, xg);
    } else {
        uint32_t h0, h1, h2, h3, l0, l1, l2, l3;
        split_bf16(xg.x, h0, l0); split_bf16(xg.y, h1, l1); split_bf16(xg.z, h2, l2); split_bf16(xg.w, h3, l3);
        if (SIGNAL) {
            st_wt8(xg_bf16 + at, make_uint2(h0 | (h1 << 16), h2 | (h3 << 16)));
            st_wt8(xg_bf16 + plane_stride + at, make_uint2(l0 | (l1 << 16), l2 | (l3 << 16)));
        } else {
            *reinterpret_cast<uint2 *>(xg_bf16 + at) = make_uint2(h0 | (h1 << 16), h2 | (h3 << 16));
            *reinterpret_cast<uint2 *>(xg_bf16 + plane_stride + at) = make_uint2(l0 | (l1 << 16), l2 | (l3 << 16));
        }
    }
    const float ss = wave_sum(v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    if (!SIGNAL) {
        if (tid == 0) ssq[(size_t)b * gridDim.x + blockIdx.x] = red[0] + red[1];
        return;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // every wave: its stores are acknowledged by the memory side
    __syncthreads();
    if (tid < kSkTagCopies)     // [copy][H / 512][batch]: every waiting workgroup polls one copy, a few dozen of them each
        ll_store(ssq_ll + (size_t)tid * ll_stride + (size_t)blockIdx.x * gridDim.y + b, red[0] + red[1], tag);
}

hipError_t launch_resid_sum(const float *res, const float *delta, int delta_splits, int batch, int H, float *out_res,
                            const uint16_t *gain, uint16_t *xg_bf16, size_t plane_stride, bool digits, float *ssq,
                            const SkWait *signal, hipStream_t s)
{
    if (signal && (!gain || !signal->ssq_ll)) return hipErrorInvalidValue;   // only the form that prepares an operand signals
    if (signal)
        PSV_LAUNCH(k_resid_sum<true>, dim3(H / 512, batch), dim3(128), 0, s, res, delta, delta_splits, (size_t)batch * H, H,
                   out_res, gain, xg_bf16, plane_stride, digits ? 1 : 0, ssq, static_cast<uint2 *>(signal->ssq_ll),
                   (unsigned)sk_tag_stride(batch, H), signal->tag);
    else
        PSV_LAUNCH(k_resid_sum<false>, dim3(H / 512, batch), dim3(128), 0, s, res, delta, delta_splits, (size_t)batch * H, H,
                   out_res, gain, xg_bf16, plane_stride, digits ? 1 : 0, ssq, static_cast<uint2 *>(nullptr), 0u, 0u);
    return hipGetLastError();
}


// ------------------------------------------------------------------------------------ split-K skinny GEMM

// What a projection that is launched into its communication window (k_gemm_sk<1, HOLD>, k_gemm_sk_i8<1, HOLD>, HOLD > 0)
// is told besides its ordinary arguments.  While the window runs every workgroup walks the window's prefetch job, reads
// and drops the slabs of its own range up to touch_w (rows of W) or touch_w2 (rows of W2) -- which leaves them in the
// memory-side cache -- and requests the slabs it keeps on chip.  Then it waits: for the window's end word first (one word;
// the tagged values would be too much to hammer on for a whole window), then until the tagged sums of squares of the
// k_resid_sum<true> workgroups that write its K range carry `tag` (each is stored after its workgroup's share of the
// operand has reached the memory side); only then does it touch the operand.  The waits are bounded: one that runs into
// its bounds sets bit 1 of *err and the kernel goes on.
struct SkWaitArgs {
    const unsigned *win_done;
    unsigned win_seq;
    const uint2 *ll;          // tagged sums of squares: kSkTagCopies copies of [K / 512][batch], ll_stride entries apart
    unsigned ll_stride;
    unsigned tag;
    int touch_w, touch_w2;
    uint32_t iters;
    uint64_t ticks;
    unsigned *err;
};

// The wait itself, run by one wave of the workgroup whose K range is slabs [s0, s1).
__device__ __forceinline__ void sk_wait_for_operand(const SkWaitArgs &wt, int batch, int K, int s0, int s1, int lane)
{
    const uint2 *ll = wt.ll + (size_t)(blockIdx.x % kSkTagCopies) * wt.ll_stride;     // this workgroup's copy
    const uint64_t t0 = wall_clock64();
    uint32_t it = 0;
    {
        unsigned v = __hip_atomic_load(wt.win_done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        while ((int)(v - wt.win_seq) < 0 && it < wt.iters && wall_clock64() - t0 < wt.ticks) {
            __builtin_amdgcn_s_sleep(8);
            v = __hip_atomic_load(wt.win_done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            ++it;
        }
    }
    // The tags of the producer workgroups that write this K range (all batch rows): a few dozen contiguous entries, other
    // lines for other splits, and one copy of kSkTagCopies per workgroup.  Who polls what matters: every workgroup polling
    // every entry made one 1-4 KiB region a hot spot, and with the entries of a range spread over one line per batch row,
    // shared by all workgroups, the tags were seen 1.5 us later than with a line per range and copy (70B-shaped TP=8 shard,
    // batch 8: 109.2 -> 107.3 us/layer).
    const int blk0 = s0 >> 3, nbr = (((s1 << 6) - 1) >> 9) - blk0 + 1, cnt = batch * nbr;
    bool ok;
    for (;;) {
        ok = true;
        for (int idx = lane; idx < cnt; idx += 64) {
            uint2 v;
            ll_issue1(v, ll + blk0 * batch + idx);             // [K / 512][batch]: a range's entries are contiguous
            asm volatile("s_waitcnt vmcnt(0)" : "+v"(v) : : "memory");
            ok = ok && v.y == wt.tag;
        }
        ok = __all(ok);
        if (ok || it >= wt.iters || wall_clock64() - t0 >= wt.ticks) break;
        __builtin_amdgcn_s_sleep(8);
        ++it;
    }
    if (lane == 0 && !ok) atomicOr(wt.err, 2u);     // the operand may not be there: results invalid
}

// All tagged sums of squares into LDS (one wave; eight entries per lane and round), for the 1/rms factors of the epilogue.
__device__ __forceinline__ void sk_read_sums(const SkWaitArgs &wt, int n_ent, int lane, float *ssq_s)
{
    const uint2 *ll = wt.ll + (size_t)(blockIdx.x % kSkTagCopies) * wt.ll_stride;
    const uint64_t t0 = wall_clock64();
    uint32_t it = 0;
    bool ok;
    for (;;) {
        ok = true;
        for (int e0 = 0; e0 < n_ent; e0 += 512) {
            const int e = e0 + lane * 8;
            if (e < n_ent) {
                u32x4 q0, q1, q2, q3;
                ll_issue(q0, ll + e);
                ll_issue(q1, ll + e + 2);
                ll_issue(q2, ll + e + 4);
                ll_issue(q3, ll + e + 6);
                ll_wait4(q0, q1, q2, q3);
                const unsigned t = wt.tag;
                ok = ok && (e + 0 >= n_ent || q0.y == t) && (e + 1 >= n_ent || q0.w == t) && (e + 2 >= n_ent || q1.y == t) &&
                     (e + 3 >= n_ent || q1.w == t) && (e + 4 >= n_ent || q2.y == t) && (e + 5 >= n_ent || q2.w == t) &&
                     (e + 6 >= n_ent || q3.y == t) && (e + 7 >= n_ent || q3.w == t);
                ssq_s[e + 0] = __uint_as_float(q0.x); ssq_s[e + 1] = __uint_as_float(q0.z);
                ssq_s[e + 2] = __uint_as_float(q1.x); ssq_s[e + 3] = __uint_as_float(q1.z);
                ssq_s[e + 4] = __uint_as_float(q2.x); ssq_s[e + 5] = __uint_as_float(q2.z);
                ssq_s[e + 6] = __uint_as_float(q3.x); ssq_s[e + 7] = __uint_as_float(q3.z);
            }
        }
        ok = __all(ok);
        if (ok || it >= wt.iters || wall_clock64() - t0 >= wt.ticks) break;
        __builtin_amdgcn_s_sleep(8);
        ++it;
    }
    if (lane == 0 && !ok) atomicOr(wt.err, 2u);
}

// part[ks][b][r] = sum over the K-range of split ks of W[r][k] x[b][k], for batches of 17..64 (and any
// smaller batch).  A workgroup of 4 waves owns 128 weight rows (2 MFMA row tiles per wave) and a range of
// 64-element K slabs.  Per slab the activations of all batch entries (hi and lo bf16 planes) are brought
// into LDS once, in MFMA fragment order, and every wave reads its B-fragments from there, so the 16-byte
// global loads of a wave are spent on weights only: 32 contiguous bytes per lane per row tile, i.e. whole
// 128-byte lines of 16 rows.  Weight fragments are prefetched PF slabs ahead through a register ring and
// the activation slab two slabs ahead, which keeps 16 KiB per wave in flight even when only a few
// workgroups exist (small matrices at batch 64 cannot use many: every extra K split costs a partial
// result of batch x rows floats).  Splits are summed later in split order by the consumer (k_sk_reduce or
// k_resid_sum): deterministic, no atomics.
struct GemmSkArgs {
    const uint16_t *W, *W2;   // rows >= split_row are taken from W2 (row - split_row): gate | up in one launch
    int split_row;
    const uint16_t *xb;       // hi plane [round_up(batch,16)][K], lo plane x_plane elements further
    size_t x_plane;
    float *part;              // [splits][batch][N]
    int batch, N, K, n_slabs, slabs_per_block;
    // ssq != null: the activations are x * gain without the 1/rms factor of their RMSNorm; ssq[batch][K / 512]
    // holds partial sums of squares of x (k_resid_sum) and the epilogue multiplies column b by 1/rms(b)
    const float *ssq;
    float eps;
    int tiled;                // weights in the tiled layout: a workgroup's 128 rows x 64 elements per slab are contiguous
    SkWaitArgs wt;            // k_gemm_sk<1, HOLD>, HOLD > 0
};

// HOLD: 0 = the ordinary kernel; 1, 2 = the variant launched into a communication window, on another stream than the kernel
// that produces its activations, keeping 6 or 12 slabs of its range on chip (the launcher takes the larger one that the
// range has); kernels of their own, so that the ordinary one carries none of that code.  The activation planes are read
// with ordinary loads.  Nothing on the device reads them between this kernel's start and the producer's stores (not this
// kernel before its wait, no other kernel of the step), so its CU's vector cache, emptied when the kernel started, holds
// nothing of them; the XCDs' L2s are kept coherent for device memory by the hardware (a copy left from the previous
// layer's operand does not outlive the producer's stores -- the same property every kernel that reads a reused buffer
// written on another XCD relies on), and those stores have reached the memory side before the producer signals.  The
// sums of squares are what the wait polls, with device-coherent loads.
// pj (HOLD > 0): what else the window's plan prefetches -- other operators' weights, KV blocks.  The waiting kernel is the
// window's prefetch kernel as well: it walks the job first, before anything of its own sits in registers.
__device__ __forceinline__ uint32_t xor4(uint4 v) { return v.x ^ v.y ^ v.z ^ v.w; }

template <int NB, int HOLD>
__global__ __launch_bounds__(256) void k_gemm_sk(GemmSkArgs a, PrefetchJob pj)
{
    constexpr bool WAIT = HOLD > 0;
    static_assert(!WAIT || NB <= 2, "the waiting variant is built for one or two batch tiles");
    constexpr int PF = 4;   // slabs of weight fragments in flight per wave (8 measured slower: fewer straight-line rounds, more registers)
    __shared__ uint4 xs[2][NB * 4][64];   // [buffer][(batch tile*2 + plane)*2 + k half][lane]
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, i = lane & 15, g = lane >> 4;
    const int row_base = blockIdx.x * 128 + w * 32;
    const int s0 = blockIdx.y * a.slabs_per_block, s1 = min(s0 + a.slabs_per_block, a.n_slabs);
    const int K = a.K;

    // Lane (i, g) owns elements g*8 .. g*8+7 of both 32-element halves of row i of every 64-element slab (the matrix
    // cores' own operand order): each of its two load instructions covers 64 contiguous bytes of every row, whole
    // 32-byte sectors, instead of 16 bytes out of every 32.
    // Tiled storage: the unit of (row tile, slab) is 16 KiB in exactly this order -- [wave][row group][k half][lane] --
    // so every load instruction of a wave covers 1 KiB of contiguous memory and the workgroup walks one contiguous run.
    const uint16_t *wp[2];
    bool wok[2];
    const size_t wstep = a.tiled ? 8192 : 64;       // elements from one slab to the next
    const int whalf = a.tiled ? 512 : 32;           // ... from the first 32 elements of a slab to the second
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        const int r = row_base + mt * 16 + i;
        wok[mt] = r < a.N;
        const int rr = wok[mt] ? r : 0;
        if (a.tiled) {
            const int tile = blockIdx.x, tsplit = a.split_row >> 7;
            const uint16_t *t = tile < tsplit ? a.W + (size_t)tile * 128 * K : a.W2 + (size_t)(tile - tsplit) * 128 * K;
            wp[mt] = t + ((w * 2 + mt) * 2 * 64 + lane) * 8;
        } else {
            wp[mt] = (rr < a.split_row ? a.W + (size_t)rr * K : a.W2 + (size_t)(rr - a.split_row) * K) + g * 8;
        }
    }
    struct WFrag { uint4 a0[2], a1[2]; };
    auto load_w = [&](int s, WFrag &f) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            f.a0[mt] = wok[mt] ? ld16(wp[mt] + (size_t)s * wstep) : zero16();
            f.a1[mt] = wok[mt] ? ld16(wp[mt] + (size_t)s * wstep + whalf) : zero16();
        }
    };
    auto load_w_all = [&](int s, WFrag &f) {   // unpredicated: a row past N reads row 0 (wp) and is never stored
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            f.a0[mt] = ld16(wp[mt] + (size_t)s * wstep);
            f.a1[mt] = ld16(wp[mt] + (size_t)s * wstep + whalf);
        }
    };
    // activation slab: NB*256 16-byte units, unit u = ((tile*2 + plane)*16 + row)*8 + segment
    auto load_slab = [&](int s, uint4 (&r)[NB]) {
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int u = tid + j * 256, n = u >> 8, p = (u >> 7) & 1, row = (u >> 3) & 15, seg = u & 7;
            r[j] = ld16(a.xb + (size_t)p * a.x_plane + (size_t)(n * 16 + row) * K + (size_t)s * 64 + seg * 8);
        }
    };
    auto store_slab = [&](int buf, const uint4 (&r)[NB]) {
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int u = tid + j * 256, n = u >> 8, p = (u >> 7) & 1, row = (u >> 3) & 15, seg = u & 7;
            xs[buf][(n * 2 + p) * 2 + (seg >> 2)][(seg & 3) * 16 + row] = r[j];   // fragment order: k = half*32 + g*8 + e
        }
    };

    f32x4 acc[2][NB];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int n = 0; n < NB; ++n) acc[mt][n] = f32x4{0.f, 0.f, 0.f, 0.f};
    __shared__ float inv_s[NB * 16];

    // WAIT: the first PF slabs of the range wait in the register ring as always, the next RH in registers of their own
    // (used once) and the LH after those are parked in LDS (each thread keeps its own fragments there: 16 KiB per slab and
    // workgroup).  HS is even (the activation double buffer alternates per slab).
    constexpr int RH = HOLD == 2 ? (NB == 1 ? 4 : 2) : 0;          // two batch tiles: 6 or 8 slabs (registers, LDS)
    constexpr int LH = HOLD == 2 ? (NB == 1 ? 4 : 2) : HOLD == 1 ? 2 : 0;
    constexpr int HS = PF + RH + LH;        // slabs held on chip when the wait ends
    __shared__ uint4 wl[LH ? LH * 4 * 256 : 1];
    const bool held = WAIT && s1 - s0 >= HS;
    if (held) {
        // First the window's prefetch, while no register holds anything yet: the other operators' job, then the slabs of
        // this workgroup's own range beyond the ones kept on chip -- four slabs (16 loads per lane) in flight, results dropped.
        if (pj.n_regions || pj.kv_count) prefetch_walk(pj, blockIdx.y * gridDim.x + blockIdx.x, (uint64_t)gridDim.x * gridDim.y);
        {
            const int t_end = min(s1, s0 + (row_base < a.split_row ? a.wt.touch_w : a.wt.touch_w2));
            uint32_t sink = 0;
            for (int s = s0 + HS; s < t_end; s += 4) {
                WFrag t[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (s + q < t_end) load_w(s + q, t[q]);
                    else t[q].a0[0] = t[q].a0[1] = t[q].a1[0] = t[q].a1[1] = zero16();
                }
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    sink ^= xor4(t[q].a0[0]) ^ xor4(t[q].a0[1]) ^ xor4(t[q].a1[0]) ^ xor4(t[q].a1[1]);
            }
            asm volatile("" ::"v"(sink));   // keeps the loads alive without a store
        }
#pragma unroll
        for (int e = 0; e < LH; e += 2) {
            WFrag t[2];
            load_w(s0 + PF + RH + e, t[0]);
            load_w(s0 + PF + RH + e + 1, t[1]);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                uint4 *d = wl + ((e + j) * 4) * 256 + tid;
                d[0] = t[j].a0[0]; d[256] = t[j].a0[1]; d[512] = t[j].a1[0]; d[768] = t[j].a1[1];
            }
        }
    } else if (WAIT) {      // a range too short for that: the job still has to be walked
        if (pj.n_regions || pj.kv_count) prefetch_walk(pj, blockIdx.y * gridDim.x + blockIdx.x, (uint64_t)gridDim.x * gridDim.y);
    }
    WFrag hq[RH ? RH : 1];
    if (RH && held) {
#pragma unroll
        for (int q = 0; q < RH; ++q) load_w(s0 + PF + q, hq[q]);
    }
    WFrag wq[PF];
#pragma unroll
    for (int q = 0; q < PF; ++q)
        if (s0 + q < s1) load_w(s0 + q, wq[q]);
    __shared__ float ssq_s[WAIT ? kSkWaitEntries : 1];
    if (WAIT) {     // the weights above travel, then sit on chip, while the window runs
        if (w == 0) sk_wait_for_operand(a.wt, a.batch, K, s0, s1, lane);     // one wave polls
        __syncthreads();
    }
    // Activations.  Ordinary start: the first two slabs are requested, the first one goes to LDS.  After a wait the
    // weights of the first HS slabs are on chip, so those steps would each cost one load latency of the activation
    // pipeline (a slab is requested one step before it is stored): their activation slabs are requested XG steps ahead --
    // the first XG at once, together with the two that the main loop starts from.
    uint4 xr[2][NB];
    constexpr int XG = WAIT ? 6 : 1;
    uint4 xa[XG][NB];
    if (held) {
#pragma unroll
        for (int h = 0; h < XG; ++h) load_slab(s0 + h, xa[h]);
        if (s0 + HS < s1) load_slab(s0 + HS, xr[0]);
        if (s0 + HS + 1 < s1) load_slab(s0 + HS + 1, xr[1]);
    } else if (s0 < s1) {
        load_slab(s0, xr[0]);
        if (s0 + 1 < s1) load_slab(s0 + 1, xr[1]);
        store_slab(0, xr[0]);
    }
    // 1/rms of every batch row from the partial sums of squares (block order); read in the epilogue only.  The waiting
    // variant forms it after the main loop, from the tagged values of all producer workgroups (by then long complete).
    auto inv_rms = [&]() {
        if (tid < NB * 16) {
            float inv = 1.0f;
            if (a.ssq) {
                float tot = 0.f;
                const int nblk = K / 512;                       // <= 32
                if (tid < a.batch) {
                    const float *p = a.ssq + (size_t)tid * nblk;
                    if (WAIT) {                                 // what the wait has read, in block order
                        for (int q = 0; q < nblk; ++q) tot += ssq_s[q * a.batch + tid];
                    } else if ((nblk & 3) == 0) {               // all loads at once, then the sum in block order
                        float4 t[8];
#pragma unroll
                        for (int q = 0; q < 8; ++q)
                            t[q] = 4 * q < nblk ? *reinterpret_cast<const float4 *>(p + 4 * q) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                        for (int q = 0; q < 8; ++q) tot = (((tot + t[q].x) + t[q].y) + t[q].z) + t[q].w;
                    } else {
                        for (int q = 0; q < nblk; ++q) tot += p[q];
                    }
                }
                inv = 1.0f / sqrtf(tot / (float)K + a.eps);
            }
            inv_s[tid] = inv;
        }
    };
    if (!WAIT) inv_rms();
    __syncthreads();

    auto mfma_slab = [&](int buf, const WFrag &f) {
#pragma unroll
        for (int n = 0; n < NB; ++n) {
            const bf16x8 bh0 = __builtin_bit_cast(bf16x8, xs[buf][(n * 2 + 0) * 2 + 0][lane]);
            const bf16x8 bh1 = __builtin_bit_cast(bf16x8, xs[buf][(n * 2 + 0) * 2 + 1][lane]);
            const bf16x8 bl0 = __builtin_bit_cast(bf16x8, xs[buf][(n * 2 + 1) * 2 + 0][lane]);
            const bf16x8 bl1 = __builtin_bit_cast(bf16x8, xs[buf][(n * 2 + 1) * 2 + 1][lane]);
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                const bf16x8 a0 = __builtin_bit_cast(bf16x8, f.a0[mt]);
                const bf16x8 a1 = __builtin_bit_cast(bf16x8, f.a1[mt]);
                acc[mt][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, bh0, acc[mt][n], 0, 0, 0);
                acc[mt][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, bh1, acc[mt][n], 0, 0, 0);
                acc[mt][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, bl0, acc[mt][n], 0, 0, 0);
                acc[mt][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, bl1, acc[mt][n], 0, 0, 0);
            }
        }
    };
    // Steady state: as long as every slab this round touches exists (s + PF < s1 for all four steps), the round is
    // straight-line code -- no predicate on any load.  Only then can the compiler count the loads issued after the
    // one it needs and wait with the exact vmcnt; behind predicated loads it waits for everything outstanding at the
    // top of every round, which exposes a full memory latency per PF slabs.
    int sb = s0;
    if (held) {
        // The slabs held on chip, in the order of the range (the sum of a split has one order, launched ahead or not):
        // the ring's PF, each slot refilled with the slab HS further on (the ring then holds what the main loop expects),
        // the RH of the extra registers, the LH from LDS.  Straight-line; a refill past the range re-reads its last slab
        // and is never used.
#pragma unroll
        for (int h = 0; h < HS; ++h) {
            const int buf = h & 1;
            store_slab(buf, xa[h % XG]);
            if (h + XG < HS) load_slab(s0 + h + XG, xa[h % XG]);
            __syncthreads();
            if (h < PF) {
                mfma_slab(buf, wq[h]);
                load_w_all(min(s0 + h + HS, s1 - 1), wq[h]);
            } else if (h < PF + RH) {
                mfma_slab(buf, hq[RH ? h - PF : 0]);
            } else {
                WFrag f;
                const uint4 *d = wl + ((h - PF - RH) * 4) * 256 + tid;
                f.a0[0] = d[0]; f.a0[1] = d[256]; f.a1[0] = d[512]; f.a1[1] = d[768];
                mfma_slab(buf, f);
            }
        }
        sb = s0 + HS;
        if (sb < s1) store_slab(0, xr[0]);      // HS is even: the main loop's first slab goes to buffer 0
        __syncthreads();
    }
    for (; sb + 2 * PF <= s1; sb += PF) {
#pragma unroll
        for (int q = 0; q < PF; ++q) {
            const int s = sb + q, buf = q & 1;      // (s - s0) & 1, because PF and the number of slabs parked in LDS are even
            load_slab(s + 2, xr[q & 1]);
            mfma_slab(buf, wq[q]);
            load_w_all(s + PF, wq[q]);
            store_slab(buf ^ 1, xr[(q + 1) & 1]);
            __syncthreads();
        }
    }
    for (; sb < s1; sb += PF) {                     // the last rounds: every step checks what is left
#pragma unroll
        for (int q = 0; q < PF; ++q) {
            const int s = sb + q;
            if (s < s1) {                       // uniform over the workgroup
                const int buf = q & 1;
                if (s + 2 < s1) load_slab(s + 2, xr[q & 1]);
                mfma_slab(buf, wq[q]);
                if (s + PF < s1) load_w(s + PF, wq[q]);
                if (s + 1 < s1) store_slab(buf ^ 1, xr[(q + 1) & 1]);
                __syncthreads();
            }
        }
    }

    if (WAIT) {
        if (w == 0) sk_read_sums(a.wt, a.batch * (K / 512), lane, ssq_s);       // <= kSkWaitEntries
        __syncthreads();
        inv_rms();
        __syncthreads();
    }
    // D fragment: lane holds rows 4g..4g+3 of batch column i
    float *part = a.part + (size_t)blockIdx.y * a.batch * a.N;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        const int r = row_base + mt * 16 + 4 * g;
        if (r < a.N) {
#pragma unroll
            for (int n = 0; n < NB; ++n) {
                const int b = n * 16 + i;
                const float inv = inv_s[b];
                if (b < a.batch)
                    *reinterpret_cast<float4 *>(part + (size_t)b * a.N + r) =
                        make_float4(acc[mt][n][0] * inv, acc[mt][n][1] * inv, acc[mt][n][2] * inv, acc[mt][n][3] * inv);
            }
        }
    }
}

// The same split-K projection for int8 weights, entirely on the int8 matrix cores: the weight codes are the A
// operand as they are (16 bytes = 16 consecutive k of one row per lane and 64-element slab), the activations
// arrive as two int8 digit planes with one scale per 128-element block (store_digits4) and are the B operand.
// Each digit has its own exact i32 accumulator; at the end of every 128-element block (two slabs) the pair is
// folded into the fp32 accumulator as scale/254 * (254*D1 + D2).  No per-element conversion of weights anywhere.
// (128-element slabs, i.e. whole 128-byte lines per row and step, measured slower: 19.6 -> 25 us on the 70B-shaped
// gate/up matrix at batch 8.)
struct GemmI8Args {
    const int8_t *W, *W2;          // rows >= split_row come from W2
    const float *scale, *scale2;   // per-row weight scales
    int split_row;
    const uint8_t *xd;             // digit plane d1 [round_up(batch,16)][K]; d2 x_plane bytes later; then the block scales
    size_t x_plane;
    float *part;                   // [splits][batch][N]
    int batch, N, K, n_slabs, slabs_per_block;
    const float *ssq;              // see GemmSkArgs
    float eps;
    int tiled;                     // see GemmSkArgs; the unit of (row tile, slab) is 8 KiB: [wave][row group][lane][16 codes]
    SkWaitArgs wt;                 // k_gemm_sk_i8<1, HOLD>, HOLD > 0
};

constexpr int kSkI8Blocks = 66;    // 128-element blocks a workgroup's K range can touch (ranges of up to 128 slabs)

// HOLD, pj: as for k_gemm_sk.  The waiting variant keeps the 8 slabs of its register ring, or those and 4 more in LDS
// (8 KiB each), on chip.  The operand's block scales share cache lines between producer workgroups of different XCDs,
// so the waiting variant reads those of its K range with device-coherent loads, once, after the wait.
template <int NB, int HOLD>
__global__ __launch_bounds__(256) void k_gemm_sk_i8(GemmI8Args a, PrefetchJob pj)
{
    constexpr bool WAIT = HOLD > 0;
    static_assert(!WAIT || NB == 1, "the waiting variant is built for one batch tile");
    constexpr int PF = 8;                          // slabs of weight codes in flight per wave (2 x 16 bytes each)
    __shared__ uint4 xs[2][NB * 2][64];            // [buffer][batch tile * 2 + digit][lane]
    __shared__ float bs[2][NB * 16];               // block scale of each batch row for the buffered slab
    __shared__ float inv_s[NB * 16];
    __shared__ float bsl[WAIT ? 16 * kSkI8Blocks : 1];     // waiting variant: block scales of this K range, [batch row][block]
    __shared__ float ssq_s[WAIT ? kSkWaitEntries : 1];
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, i = lane & 15, g = lane >> 4;
    const int row_base = blockIdx.x * 128 + w * 32;
    const int s0 = blockIdx.y * a.slabs_per_block, s1 = min(s0 + a.slabs_per_block, a.n_slabs);
    const int K = a.K;
    const float *bscale = reinterpret_cast<const float *>(a.xd + 2 * a.x_plane);
    const int nblk128 = K / 128;

    const int8_t *wp[2];
    bool wok[2];
    const size_t wstep = a.tiled ? 8192 : 64;       // bytes from one slab to the next
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        const int r = row_base + mt * 16 + i;
        wok[mt] = r < a.N;
        const int rr = wok[mt] ? r : 0;
        if (a.tiled) {
            const int tile = blockIdx.x, tsplit = a.split_row >> 7;
            const int8_t *t = tile < tsplit ? a.W + (size_t)tile * 128 * K : a.W2 + (size_t)(tile - tsplit) * 128 * K;
            wp[mt] = t + ((w * 2 + mt) * 64 + lane) * 16;
        } else {
            wp[mt] = (rr < a.split_row ? a.W + (size_t)rr * K : a.W2 + (size_t)(rr - a.split_row) * K) + g * 16;
        }
    }
    // Lane (i, g) owns bytes g*16 .. g*16+15 of row i of every 64-element slab: the A operand of one MFMA.
    struct WFrag { uint4 c[2]; };
    auto load_w = [&](int s, WFrag &f) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
            f.c[mt] = wok[mt] ? *reinterpret_cast<const uint4 *>(wp[mt] + (size_t)s * wstep) : zero16();
    };
    // activation slab: NB*128 16-byte units, unit u = ((tile*2 + digit)*16 + row)*4 + segment
    constexpr int NU = (NB + 1) / 2;
    struct SlabRegs { uint4 r[NU]; float sc; };
    auto load_slab = [&](int s, SlabRegs &sr) {
#pragma unroll
        for (int j = 0; j < NU; ++j) {
            const int u = tid + j * 256, n = u >> 7, dgt = (u >> 6) & 1, row = (u >> 2) & 15, seg = u & 3;
            sr.r[j] = u < NB * 128 ? *reinterpret_cast<const uint4 *>(a.xd + (size_t)dgt * a.x_plane +
                                                                       (size_t)(n * 16 + row) * K + (size_t)s * 64 + seg * 16)
                                   : zero16();
        }
        if (WAIT) sr.sc = tid < a.batch ? bsl[tid * kSkI8Blocks + (s >> 1) - (s0 >> 1)] : 0.f;
        else sr.sc = tid < NB * 16 ? bscale[(size_t)tid * nblk128 + (s >> 1)] : 0.f;
    };
    auto store_slab = [&](int buf, const SlabRegs &sr) {
#pragma unroll
        for (int j = 0; j < NU; ++j) {
            const int u = tid + j * 256, n = u >> 7, dgt = (u >> 6) & 1, row = (u >> 2) & 15, seg = u & 3;
            if (u < NB * 128) xs[buf][n * 2 + dgt][seg * 16 + row] = sr.r[j];   // B operand: lane (row, segment)
        }
        if (tid < NB * 16) bs[buf][tid] = sr.sc;
    };
    f32x4 acc[2][NB];
    i32x4 d1[2][NB], d2[2][NB];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int n = 0; n < NB; ++n) {
            acc[mt][n] = f32x4{0.f, 0.f, 0.f, 0.f};
            d1[mt][n] = i32x4{0, 0, 0, 0};
            d2[mt][n] = i32x4{0, 0, 0, 0};
        }

    // Waiting variant: see k_gemm_sk.  The ring's PF slabs and the LH after them stay on chip.
    constexpr int LH = HOLD == 2 ? 4 : 0;
    constexpr int HS = PF + LH;
    __shared__ uint4 wl[LH ? LH * 2 * 256 : 1];
    const bool held = WAIT && s1 - s0 >= HS;
    if (WAIT && (pj.n_regions || pj.kv_count))
        prefetch_walk(pj, blockIdx.y * gridDim.x + blockIdx.x, (uint64_t)gridDim.x * gridDim.y);
    if (held) {
        {   // this workgroup's own slabs beyond the ones kept on chip: eight slabs (16 loads per lane) in flight, dropped
            const int t_end = min(s1, s0 + (row_base < a.split_row ? a.wt.touch_w : a.wt.touch_w2));
            uint32_t sink = 0;
            for (int s = s0 + HS; s < t_end; s += 8) {
                WFrag t[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    if (s + q < t_end) load_w(s + q, t[q]);
                    else t[q].c[0] = t[q].c[1] = zero16();
                }
#pragma unroll
                for (int q = 0; q < 8; ++q) sink ^= xor4(t[q].c[0]) ^ xor4(t[q].c[1]);
            }
            asm volatile("" ::"v"(sink));
        }
#pragma unroll
        for (int e = 0; e < LH; e += 2) {
            WFrag t[2];
            load_w(s0 + PF + e, t[0]);
            load_w(s0 + PF + e + 1, t[1]);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                uint4 *d = wl + ((e + j) * 2) * 256 + tid;
                d[0] = t[j].c[0]; d[256] = t[j].c[1];
            }
        }
    }
    WFrag wq[PF];
#pragma unroll
    for (int q = 0; q < PF; ++q)
        if (s0 + q < s1) load_w(s0 + q, wq[q]);
    if (WAIT) {
        if (w == 0) sk_wait_for_operand(a.wt, a.batch, K, s0, s1, lane);     // one wave polls
        __syncthreads();
        const int b0 = s0 >> 1, nbk = ((s1 - 1) >> 1) - b0 + 1;             // <= kSkI8Blocks
        for (int idx = tid; idx < a.batch * nbk; idx += 256) {
            float v;
            asm volatile("global_load_dword %0, %1, off sc0 sc1" : "=v"(v) : "v"(bscale + (size_t)(idx / nbk) * nblk128 + b0 + idx % nbk) : "memory");
            asm volatile("s_waitcnt vmcnt(0)" : "+v"(v) : : "memory");
            bsl[(idx / nbk) * kSkI8Blocks + idx % nbk] = v;
        }
        __syncthreads();
    }
    SlabRegs xr[2];
    constexpr int XG = WAIT ? 6 : 1;        // activation slabs requested ahead in the held part (see k_gemm_sk)
    SlabRegs xa[XG];
    if (held) {
#pragma unroll
        for (int h = 0; h < XG; ++h) load_slab(s0 + h, xa[h]);
        if (s0 + HS < s1) load_slab(s0 + HS, xr[0]);
        if (s0 + HS + 1 < s1) load_slab(s0 + HS + 1, xr[1]);
    } else if (s0 < s1) {
        load_slab(s0, xr[0]);
        if (s0 + 1 < s1) load_slab(s0 + 1, xr[1]);
        store_slab(0, xr[0]);
    }
    auto inv_rms = [&]() {      // 1/rms of every batch row (see k_gemm_sk)
        if (tid < NB * 16) {
            float inv = 1.0f;
            if (a.ssq) {
                float tot = 0.f;
                const int nblk = K / 512;
                if (tid < a.batch) {
                    const float *p = a.ssq + (size_t)tid * nblk;
                    if (WAIT) {
                        for (int q = 0; q < nblk; ++q) tot += ssq_s[q * a.batch + tid];
                    } else if ((nblk & 3) == 0) {
                        float4 t[8];
#pragma unroll
                        for (int q = 0; q < 8; ++q)
                            t[q] = 4 * q < nblk ? *reinterpret_cast<const float4 *>(p + 4 * q) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                        for (int q = 0; q < 8; ++q) tot = (((tot + t[q].x) + t[q].y) + t[q].z) + t[q].w;
                    } else {
                        for (int q = 0; q < nblk; ++q) tot += p[q];
                    }
                }
                inv = 1.0f / sqrtf(tot / (float)K + a.eps);
            }
            inv_s[tid] = inv;
        }
    };
    if (!WAIT) inv_rms();
    __syncthreads();

    // one slab: both digit planes against the weight codes; at the end of a 128-element block (or of the range) the pair
    // of exact sums is folded into the fp32 accumulator
    auto mfma_slab = [&](int s, int buf, const WFrag &f) {
        const bool fold = (s & 1) || s + 1 == s1;
#pragma unroll
        for (int n = 0; n < NB; ++n) {
            const i32x4 x1 = __builtin_bit_cast(i32x4, xs[buf][n * 2 + 0][lane]);
            const i32x4 x2 = __builtin_bit_cast(i32x4, xs[buf][n * 2 + 1][lane]);
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                const i32x4 wc = __builtin_bit_cast(i32x4, f.c[mt]);
                d1[mt][n] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wc, x1, d1[mt][n], 0, 0, 0);
                d2[mt][n] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wc, x2, d2[mt][n], 0, 0, 0);
            }
            if (fold) {
                const float sc = bs[buf][n * 16 + i] * (1.0f / 254.0f);
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        acc[mt][n][j] = fmaf(sc, (float)(d1[mt][n][j] * 254 + d2[mt][n][j]), acc[mt][n][j]);
                    d1[mt][n] = i32x4{0, 0, 0, 0};
                    d2[mt][n] = i32x4{0, 0, 0, 0};
                }
            }
        }
    };

    int sb0 = s0;
    if (held) {     // the slabs held on chip, in the order of the range; ring slots are refilled with the slab HS further on
#pragma unroll
        for (int h = 0; h < HS; ++h) {
            const int buf = h & 1;
            store_slab(buf, xa[h % XG]);
            if (h + XG < HS) load_slab(s0 + h + XG, xa[h % XG]);
            __syncthreads();
            if (h < PF) {
                mfma_slab(s0 + h, buf, wq[h]);
                load_w(min(s0 + h + HS, s1 - 1), wq[h]);
            } else {
                WFrag f;
                const uint4 *d = wl + ((h - PF) * 2) * 256 + tid;
                f.c[0] = d[0]; f.c[1] = d[256];
                mfma_slab(s0 + h, buf, f);
            }
        }
        sb0 = s0 + HS;
        if (sb0 < s1) store_slab(0, xr[0]);     // HS is even: the main loop's first slab goes to buffer 0
        __syncthreads();
    }
    for (int sb = sb0; sb < s1; sb += PF) {
#pragma unroll
        for (int q = 0; q < PF; ++q) {
            const int s = sb + q;
            if (s < s1) {                       // uniform over the workgroup
                const int buf = q & 1;          // (s - s0) & 1, because PF and the number of slabs held are even
                if (s + 2 < s1) load_slab(s + 2, xr[q & 1]);
                mfma_slab(s, buf, wq[q]);
                if (s + PF < s1) load_w(s + PF, wq[q]);
                if (s + 1 < s1) store_slab(buf ^ 1, xr[(q + 1) & 1]);
                __syncthreads();
            }
        }
    }
    if (WAIT) {
        if (w == 0) sk_read_sums(a.wt, a.batch * (K / 512), lane, ssq_s);       // <= kSkWaitEntries
        __syncthreads();
        inv_rms();
        __syncthreads();
    }

    // D fragment: lane holds rows 4g..4g+3 of batch column i
    float *part = a.part + (size_t)blockIdx.y * a.batch * a.N;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        const int r = row_base + mt * 16 + 4 * g;
        if (r < a.N) {
            const float4 sc = r < a.split_row ? *reinterpret_cast<const float4 *>(a.scale + r)
                                              : *reinterpret_cast<const float4 *>(a.scale2 + (r - a.split_row));
#pragma unroll
            for (int n = 0; n < NB; ++n) {
                const int b = n * 16 + i;
                const float inv = inv_s[b];
                if (b < a.batch)
                    *reinterpret_cast<float4 *>(part + (size_t)b * a.N + r) =
                        make_float4(acc[mt][n][0] * sc.x * inv, acc[mt][n][1] * sc.y * inv, acc[mt][n][2] * sc.z * inv,
                                    acc[mt][n][3] * sc.w * inv);
            }
        }
    }
}

// Number of K splits, from a small cost model of the kernel: a workgroup needs ~0.6 us per slab it walks
// (latency of one pipelined slab step), 512 workgroups are resident at a time, and weights plus partial
// results (written once, read back once) stream at ~4 TB/s.  More splits shorten the walk and cost partial
// traffic of batch * N * 8 bytes each; small matrices at batch 64 end up with 4-16 splits, wide ones at
// small batch with as many as keep every CU busy.
int gemm_sk_splits(int batch, int N, int K, bool w8, bool tiled)
{
    const int n_slabs = K / 64;
    const double row_groups = (double)((N + 127) / 128);
    const double w_bytes = (w8 ? 1.0 : 2.0) * N * K, part_bytes = 8.0 * batch * N;
    int best = 1, best1 = 0;                    // best1: the best choice whose workgroups are all resident at once
    double best_cost = 1e30, best1_cost = 1e30;
    for (int ks = 1; ks <= kSkMaxSplits && ks * 2 <= n_slabs; ++ks) {
        const int spb = (n_slabs + ks - 1) / ks;
        const int real = (n_slabs + spb - 1) / spb;
        if (real != ks) continue;
        const double rounds = (double)(long long)((row_groups * ks + 511) / 512);
        const double cost = rounds * spb * 0.6 + (w_bytes + ks * part_bytes) / 4.0e6;
        if (cost < best_cost - 1e-9) { best_cost = cost; best = ks; }
        if (rounds == 1.0 && cost < best1_cost - 1e-9) { best1_cost = cost; best1 = ks; }
    }
    // On tiled weights, within 2 % of each other one round wins: such a projection can be launched into a communication
    // window (gemm_sk_can_wait), and the model's step cost is no finer than that.  (Measured on the 235 MB gate/up matrix of
    // a TP=4 70B-shaped shard at batch 4: 4 splits instead of 9 are 1.5 % faster per layer on tiled weights and 3 % slower
    // on row-major ones, whose long per-workgroup ranges walk rows 16 KiB apart.)
    if (tiled && best1 && best1_cost <= 1.02 * best_cost) best = best1;
    return best;
}

bool gemm_sk_supported(int batch, int N, int K)
{
    return batch >= 1 && batch <= 64 && N % 16 == 0 && K % 64 == 0;
}

// Which waiting variant a range of `slabs_per_block` slabs takes: the one that keeps 12 slabs on chip if the range has them.
static int sk_hold_level(int slabs_per_block, int nb = 1) { return slabs_per_block >= (nb == 1 ? 12 : 8) ? 2 : 1; }

// Resources of the waiting variants ([bf16 | int8 | bf16 with two batch tiles][hold level - 1]) and of the kernel they wait for, asked from
// the runtime once.
struct SkWaitRes {
    int occ[3][2];       // resident workgroups per compute unit
    int regs[3][2];      // registers per lane (vector + accumulation), rounded up to the allocation unit
    int lds[3][2];       // static LDS bytes per workgroup
    int regs_signal;     // k_resid_sum<true>
    bool ok;
};
static const SkWaitRes &sk_wait_res()
{
    static SkWaitRes r = [] {
        SkWaitRes q{};
        q.ok = true;
        auto ask = [&](int kind, int lv, auto kernel) {
            hipFuncAttributes at{};
            int n = 0;
            const hipError_t e1 = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, 256, 0);
            const hipError_t e2 = hipFuncGetAttributes(&at, reinterpret_cast<const void *>(kernel));
            q.ok = q.ok && e1 == hipSuccess && e2 == hipSuccess && n > 0;
            q.occ[kind][lv] = n;
            q.regs[kind][lv] = (at.numRegs + 7) / 8 * 8;
            q.lds[kind][lv] = (int)at.sharedSizeBytes;
        };
        ask(0, 0, k_gemm_sk<1, 1>);
        ask(0, 1, k_gemm_sk<1, 2>);
        ask(1, 0, k_gemm_sk_i8<1, 1>);
        ask(1, 1, k_gemm_sk_i8<1, 2>);
        ask(2, 0, k_gemm_sk<2, 1>);
        ask(2, 1, k_gemm_sk<2, 2>);
        hipFuncAttributes at{};
        q.ok = q.ok && hipFuncGetAttributes(&at, reinterpret_cast<const void *>(k_resid_sum<true>)) == hipSuccess;
        q.regs_signal = (at.numRegs + 7) / 8 * 8;
        return q;
    }();
    return r;
}

// Can this projection be launched ahead of its activations (launch_gemm_sk with a wait)?  Its workgroups then sit on
// the compute units until k_resid_sum has run, so all of them must be resident at once and leave room for that kernel:
// either a quarter of the compute units keep a free workgroup slot of this kernel's size, or a wave of k_resid_sum fits
// beside a full house (512 registers per lane and SIMD, with 16 to spare; 160 KiB of LDS, with 4 KiB to spare).
bool gemm_sk_can_wait(int batch, int N, int K, bool w8, bool tiled, int cus)
{
    if (!gemm_sk_supported(batch, N, K) || K % 512 || (long long)batch * (K / 512) > kSkWaitEntries) return false;
    if (batch > (w8 ? 16 : kSkWaitMaxBatch)) return false;         // the instantiations of the waiting kernels
    const SkWaitRes &r = sk_wait_res();
    if (!r.ok) return false;
    const int splits = gemm_sk_splits(batch, N, K, w8, tiled);
    const int nb = (batch + 15) / 16;
    const int kind = w8 ? 1 : nb == 2 ? 2 : 0, lv = sk_hold_level((K / 64 + splits - 1) / splits, nb) - 1;
    const long long grid = (long long)((N + 127) / 128) * splits;
    // Worth it only if a good part of a workgroup's range stays on chip: with less than a third (two batch tiles on the
    // 235 MB gate/up matrix of a TP=4 70B-shaped shard: 8 slabs of 32) the wait's latencies cost more than the slabs save.
    {
        const int spb = (K / 64 + splits - 1) / splits;
        const int hs = w8 ? (lv ? 12 : 8) : nb == 2 ? (lv ? 8 : 6) : (lv ? 12 : 6);
        if (hs * 3 < spb) return false;
    }
    // ... and it is the window's prefetch kernel as well, which needs at least 128 workgroups to reach its rate
    if (grid < 128 || grid > (long long)r.occ[kind][lv] * cus) return false;
    const bool free_slots = grid + cus / 4 <= (long long)r.occ[kind][lv] * cus;
    const bool beside = 512 - r.occ[kind][lv] * r.regs[kind][lv] >= r.regs_signal + 16 &&
                        163840 - r.occ[kind][lv] * r.lds[kind][lv] >= 4096;
    return free_slots || beside;
}

hipError_t launch_gemm_sk(Mat W, Mat W2, int split_row, const uint16_t *xb, const float *ssq, float eps, float *part,
                          int batch, int N, int K, const SkWait *wait, hipStream_t s)
{
    const int nb = (batch + 15) / 16;
    // planned share of each matrix, spread evenly over its workgroups: slabs of a workgroup's range that are either kept
    // on chip or read and dropped
    auto fill_wait = [&](SkWaitArgs &wt, int slabs_per_block) {
        wt.win_done = wait->win_done; wt.win_seq = wait->win_seq;
        wt.ll = static_cast<const uint2 *>(wait->ssq_ll); wt.ll_stride = (unsigned)sk_tag_stride(batch, K);
        wt.tag = wait->tag; wt.iters = wait->iters;
        wt.ticks = wait->ticks; wt.err = wait->err;
        wt.touch_w = (int)(wait->share_w * slabs_per_block + 0.5);
        wt.touch_w2 = (int)(wait->share_w2 * slabs_per_block + 0.5);
    };
    if (wait && (!ssq || !wait->ssq_ll || !wait->win_done || batch > (W.scale ? 16 : kSkWaitMaxBatch) || K % 512 || (long long)batch * (K / 512) > kSkWaitEntries)) return hipErrorInvalidValue;
    if (W.scale) {   // int8 weights: xb holds digit planes (bytes), see k_gemm_sk_i8
        GemmI8Args q{};
        q.W = static_cast<const int8_t *>(W.w); q.W2 = static_cast<const int8_t *>(W2.w ? W2.w : W.w);
        q.scale = W.scale; q.scale2 = W2.w ? W2.scale : W.scale; q.split_row = W2.w ? split_row : N;
        q.xd = reinterpret_cast<const uint8_t *>(xb); q.x_plane = (size_t)nb * 16 * K;
        q.part = part; q.batch = batch; q.N = N; q.K = K; q.n_slabs = K / 64; q.ssq = ssq; q.eps = eps;
        q.tiled = W.tiled ? 1 : 0;
        const int splits = gemm_sk_splits(batch, N, K, true, W.tiled);
        q.slabs_per_block = (q.n_slabs + splits - 1) / splits;
        const dim3 grid((N + 127) / 128, splits);
        if (wait) {
            fill_wait(q.wt, q.slabs_per_block);
            const PrefetchJob pj = wait->job ? *wait->job : PrefetchJob{};
            if (sk_hold_level(q.slabs_per_block) == 2) PSV_LAUNCH((k_gemm_sk_i8<1, 2>), grid, dim3(256), 0, s, q, pj);
            else PSV_LAUNCH((k_gemm_sk_i8<1, 1>), grid, dim3(256), 0, s, q, pj);
            return hipGetLastError();
        }
        switch (nb) {
        case 1: PSV_LAUNCH((k_gemm_sk_i8<1, 0>), grid, dim3(256), 0, s, q, PrefetchJob{}); break;
        case 2: PSV_LAUNCH((k_gemm_sk_i8<2, 0>), grid, dim3(256), 0, s, q, PrefetchJob{}); break;
        case 3: PSV_LAUNCH((k_gemm_sk_i8<3, 0>), grid, dim3(256), 0, s, q, PrefetchJob{}); break;
        case 4: PSV_LAUNCH((k_gemm_sk_i8<4, 0>), grid, dim3(256), 0, s, q, PrefetchJob{}); break;
        default: return hipErrorInvalidValue;
        }
        return hipGetLastError();
    }
    GemmSkArgs a{};
    a.ssq = ssq; a.eps = eps;
    a.W = static_cast<const uint16_t *>(W.w); a.W2 = static_cast<const uint16_t *>(W2.w ? W2.w : W.w);
    a.split_row = W2.w ? split_row : N; a.xb = xb; a.x_plane = (size_t)nb * 16 * K;
    a.part = part; a.batch = batch; a.N = N; a.K = K; a.n_slabs = K / 64;
    a.tiled = W.tiled ? 1 : 0;
    const int splits = gemm_sk_splits(batch, N, K, false, W.tiled);
    a.slabs_per_block = (a.n_slabs + splits - 1) / splits;
    const dim3 grid((N + 127) / 128, splits);
    if (wait) {
        fill_wait(a.wt, a.slabs_per_block);
        const PrefetchJob pj = wait->job ? *wait->job : PrefetchJob{};
        const int lv = sk_hold_level(a.slabs_per_block, nb);
        if (nb == 1 && lv == 2) PSV_LAUNCH((k_gemm_sk<1, 2>), grid, dim3(256), 0, s, a, pj);
        else if (nb == 1) PSV_LAUNCH((k_gemm_sk<1, 1>), grid, dim3(256), 0, s, a, pj);
        else if (lv == 2) PSV_LAUNCH((k_gemm_sk<2, 2>), grid, dim3(256), 0, s, a, pj);
        else PSV_LAUNCH((k_gemm_sk<2, 1>), grid, dim3(256), 0, s, a, pj);
        return hipGetLastError();
    }
    switch (nb) {
    case 1: PSV_LAUNCH((k_gemm_sk<1, 0>), grid, dim3(256), 0, s, a, PrefetchJob{}); break;
    case 2: PSV_LAUNCH((k_gemm_sk<2, 0>), grid, dim3(256), 0, s, a, PrefetchJob{}); break;
    case 3: PSV_LAUNCH((k_gemm_sk<3, 0>), grid, dim3(256), 0, s, a, PrefetchJob{}); break;
    case 4: PSV_LAUNCH((k_gemm_sk<4, 0>), grid, dim3(256), 0, s, a, PrefetchJob{}); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// out[b][n] = sum over splits (split order) of part[ks][b][n]; with SwiGLU the N columns are gate | up
// halves and the result is silu(gate) * up, [batch][N/2], stored as fp32 and as hi/lo bf16 planes.
template <bool SWIGLU>
__global__ __launch_bounds__(256) void k_sk_reduce(const float *__restrict__ part, int splits, int batch, int N,
                                                   float *__restrict__ out, uint16_t *__restrict__ out_bf16, size_t out_plane,
                                                   int digits)
{
    const int NO = SWIGLU ? N / 2 : N;                 // output columns
    const size_t total4 = (size_t)batch * NO / 4;
    const size_t split_stride = (size_t)batch * N;
    for (size_t q = (size_t)blockIdx.x * 256 + threadIdx.x; q < total4; q += (size_t)gridDim.x * 256) {
        const size_t e = q * 4, b = e / NO, c = e % NO;
        const float *p = part + b * N + c;
        // all split loads first (their latencies overlap), then the sums in split order
        float4 t[kSkMaxSplits], t2[SWIGLU ? kSkMaxSplits : 1];
#pragma unroll
        for (int ks = 0; ks < kSkMaxSplits; ++ks) {
            t[ks] = ks < splits ? *reinterpret_cast<const float4 *>(p + ks * split_stride) : make_float4(0.f, 0.f, 0.f, 0.f);
            if (SWIGLU)
                t2[ks] = ks < splits ? *reinterpret_cast<const float4 *>(p + ks * split_stride + NO)
                                     : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        float4 v = t[0], u = make_float4(0.f, 0.f, 0.f, 0.f);
        if (SWIGLU) u = t2[0];
#pragma unroll
        for (int ks = 1; ks < kSkMaxSplits; ++ks) {
            v.x += t[ks].x; v.y += t[ks].y; v.z += t[ks].z; v.w += t[ks].w;
            if (SWIGLU) { u.x += t2[ks].x; u.y += t2[ks].y; u.z += t2[ks].z; u.w += t2[ks].w; }
        }
        if (SWIGLU) {
            v.x = silu_mul(v.x, u.x); v.y = silu_mul(v.y, u.y); v.z = silu_mul(v.z, u.z); v.w = silu_mul(v.w, u.w);
        }
        *reinterpret_cast<float4 *>(out + b * NO + c) = v;
        if (out_bf16 && digits) {   // whole waves take this branch together (NO is a multiple of 256)
            store_digits4(reinterpret_cast<uint8_t *>(out_bf16), out_plane, NO, b, (int)c, v);
        } else if (out_bf16) {
            uint32_t h0, h1, h2, h3, l0, l1, l2, l3;
            split_bf16(v.x, h0, l0); split_bf16(v.y, h1, l1); split_bf16(v.z, h2, l2); split_bf16(v.w, h3, l3);
            *reinterpret_cast<uint2 *>(out_bf16 + b * NO + c) = make_uint2(h0 | (h1 << 16), h2 | (h3 << 16));
            *reinterpret_cast<uint2 *>(out_bf16 + out_plane + b * NO + c) = make_uint2(l0 | (l1 << 16), l2 | (l3 << 16));
        }
    }
}

hipError_t launch_sk_reduce(const float *part, int splits, int batch, int N, bool swiglu, float *out,
                            uint16_t *out_bf16, bool digits, hipStream_t s)
{
    const int NO = swiglu ? N / 2 : N;
    const size_t total4 = (size_t)batch * NO / 4;
    unsigned blocks = (unsigned)((total4 + 255) / 256);
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    const size_t out_plane = (size_t)((batch + 15) / 16 * 16) * NO;
    if (swiglu)
        PSV_LAUNCH(k_sk_reduce<true>, dim3(blocks), dim3(256), 0, s, part, splits, batch, N, out, out_bf16, out_plane, digits ? 1 : 0);
    else
        PSV_LAUNCH(k_sk_reduce<false>, dim3(blocks), dim3(256), 0, s, part, splits, batch, N, out, out_bf16, out_plane, digits ? 1 : 0);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------ tiled weight layout

// One thread per 16-byte piece of the destination: row-major [rows][cols] -> [row tile][slab][unit] (see GemmSkArgs /
// GemmI8Args for the order inside a unit).
template <int EB>
__global__ __launch_bounds__(256) void k_tile_weights(const char *__restrict__ src, char *__restrict__ dst, int rows, int cols)
{
    const size_t n_slabs = cols / 64, unit16 = EB == 2 ? 1024 : 512;       // 16-byte pieces per unit
    const size_t total = (size_t)(rows / 128) * n_slabs * unit16;
    for (size_t u = (size_t)blockIdx.x * 256 + threadIdx.x; u < total; u += (size_t)gridDim.x * 256) {
        const size_t unit = u / unit16, tile = unit / n_slabs, slab = unit % n_slabs;
        const int in = (int)(u % unit16);
        int w, mt, half, lane;
        if (EB == 2) { w = in >> 8; mt = (in >> 7) & 1; half = (in >> 6) & 1; lane = in & 63; }
        else { w = in >> 7; mt = (in >> 6) & 1; half = 0; lane = in & 63; }
        const size_t row = tile * 128 + w * 32 + mt * 16 + (lane & 15);
        const size_t col = slab * 64 + (EB == 2 ? half * 32 + (lane >> 4) * 8 : (lane >> 4) * 16);
        *reinterpret_cast<uint4 *>(dst + u * 16) = *reinterpret_cast<const uint4 *>(src + (row * cols + col) * EB);
    }
}

hipError_t launch_tile_weights(void *dst, const void *src, int rows, int cols, int elem_bytes, hipStream_t s)
{
    const size_t total = (size_t)rows * cols * elem_bytes / 16;
    unsigned blocks = (unsigned)((total + 255) / 256);
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    if (elem_bytes == 2)
        hipLaunchKernelGGL(k_tile_weights<2>, dim3(blocks), dim3(256), 0, s, static_cast<const char *>(src), static_cast<char *>(dst), rows, cols);
    else
        hipLaunchKernelGGL(k_tile_weights<1>, dim3(blocks), dim3(256), 0, s, static_cast<const char *>(src), static_cast<char *>(dst), rows, cols);
    return hipGetLastError();
}

}  // namespace psv

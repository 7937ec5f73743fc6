// gfx950 (MI355X, CDNA4) kernels of the PRESERVE decode step: the operators between two communication windows
// fused into one kernel (batch 1-2, vector ALU).
//
// Between two communication operators a layer runs a chain of dependent, bandwidth-bound operators (Section 2,
// "LLM inference workloads"): gate/up + SwiGLU -> down after the attention block's allreduce, and
// QKV -> attention -> O after the MLP block's.  At batch 1-2 every one of them moves 1-30 MB and, launched as a
// kernel of its own, pays ~3.5 us of dispatch, ramp-up and drain plus the latency of its first bytes, which is more
// than its streaming time.  Here a whole chain is one kernel of one workgroup per CU, all resident at once:
//
//  * every phase requests its first weights (and the attention phase its K/V tiles) at the start of the kernel, so
//    the later phases' data travels while the earlier ones compute -- and, when the kernel is launched into the
//    communication window (policy.prelaunch), sits in registers before the window ends: the register file is the
//    large on-chip memory of this machine (Section 3, "Execution with the proposed method", with the registers in
//    the role of the paper's L2);
//  * the hand-over between two phases is an all-gather through memory, in one of two forms.  Few readers (the QKV rows,
//    read by the attention workgroups): every value travels with a tag (8-byte stores of {value, tag}, written through
//    to the memory side) and the readers poll the values themselves with device-coherent loads until every tag is this
//    launch's; no separate flag, hence no store that has to be acknowledged before a flag may follow it.  Everybody reads
//    everything (the attention partials, the SwiGLU vector): the data is plain and written through; once its stores are
//    acknowledged a producer workgroup publishes a tagged indicator entry (in copies, so that 256 watchers do not poll the
//    same lines), one wave per workgroup watches the indicators, and when all are there every thread reads the data with
//    ordinary loads, which the XCD's L2 serves after the first.  Read as tagged values with device-coherent loads these
//    hand-overs were bound by the bandwidth of such loads (256 workgroups x 32 KB of attention partials: 2.4 us), not by
//    latency.
//
// Measured (8B-shaped shard, batch 1, context 2048).  With the first kernel after each window launched into the window
// they save 5 us per layer (11.6 us remain of the attention block after its window, 6.8 us of the MLP block, against
// 3.0 + 6.8 + 5.8 and 3.9 + 4.7 us for one kernel per operator, of which only the first can be launched ahead); launched
// the ordinary way they are somewhat faster than one kernel per operator (16.2 vs 17.6 us, 13.0 vs 13.8 us): a hand-over
// costs about what the kernel boundary it replaces does, and what the later phases gain from having their weights requested
// early, the first phase loses to sharing the memory system with them.  On shapes whose blocks need several passes, and on
// short rows (hidden 1024-2048), they lose 3-9 us per layer; the executor uses them by default only where rows have at least
// 4096 elements and every block's weights fit one pass.
//
// Tags are unique per launch (a process-wide counter), so a buffer never has to be cleared and stale contents of any
// earlier launch can never be taken for data.  Every poll is bounded; a poll that expires sets bit 1 of the error
// word and the kernel runs to its end (the step's results are then invalid and psv_sync reports an error).
// Row sums are formed exactly as in k_gemv (same thread-to-column map, same reduction order), so a projection gives
// the same bits in both kernels.
#include <atomic>

#include "tagged.h"

namespace psv {

static std::atomic<unsigned> g_tag_counter{1};

unsigned next_tags(unsigned n)
{
    for (;;) {
        const unsigned t = g_tag_counter.fetch_add(n, std::memory_order_relaxed);
        if (t != 0 && t + (n - 1) >= t) return t;      // 0 is what a fresh workspace holds; a run must not wrap through it
    }
}

unsigned next_tag() { return next_tags(1); }

struct SegWait {            // launched ahead of its inputs: see GemvWait
    const unsigned *done;
    unsigned seq;
    uint32_t iters;
    uint64_t ticks;
};

// ------------------------------------------------------------------------------------ MLP block

struct SegMlpArgs {
    const void *Wg, *Wu, *Wd;           // [F][H], [F][H], [H][F]; bf16 or int8 codes
    const float *sg, *su, *sd;          // int8: row scales
    const float *res, *delta;           // residual entering the block = res + delta, [NB][H]
    const uint16_t *gain;               // [H]
    float eps;
    float *out_res, *out_h;             // res + delta and the normalised activations, stored by workgroup 0
    float *m;                           // [NB][F] silu(gate) * up: plain data, written through, complete when the indicators say so
    uint2 *m_ll;                        // behind [NB][F] unused pairs: kSegIndCopies x kSegIndStride tagged indicator entries
    float *out;                         // [NB][H] down projection
    int F, H;
    SegGeom g1, g2;
    unsigned tag;
    uint32_t ll_iters;                  // bound of a hand-over poll
    unsigned *err;
    SegWait wait;
    int hold_down;                      // launched into its window: request the down weights before (1) or after (0) the wait
};

template <int NB, int RB1, int IT1, int RB2, int IT2, bool W8, bool WAIT>
__global__ __launch_bounds__(512) void k_seg_mlp(SegMlpArgs a)
{
    constexpr int WB = W8 ? 1 : 2;
    using WV = typename std::conditional<W8, uint2, uint4>::type;
    constexpr int RED1 = 2 * RB1 * NB, RED2 = RB2 * NB, RED = RED1 > RED2 ? RED1 : RED2;
    __shared__ float red[8][RED];
    __shared__ float ssq[8][NB];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    auto ldw = [](const char *p) {
        // streamed once: non-temporal, so that the weights do not push the kernel's code and the activations out of L2
        if constexpr (W8) {
            const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(p));
            return make_uint2(v.x, v.y);
        } else {
            const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
            return make_uint4(v.x, v.y, v.z, v.w);
        }
    };

    // ---- phase 1 geometry: gate/up, N = F rows of K = H
    const int H = a.H, F = a.F;
    const int GS1 = 1 << a.g1.gs_log2, groups1 = 512 >> a.g1.gs_log2, wpg1 = GS1 >> 6;
    const int gid1 = tid >> a.g1.gs_log2, lg1 = tid & (GS1 - 1);
    const int slots1 = gridDim.x * groups1, slot1 = blockIdx.x * groups1 + gid1;
    const int rb1 = (int)((long long)slot1 * F / slots1), re1 = (int)((long long)(slot1 + 1) * F / slots1);
    int k1[IT1];
    bool ok1[IT1];
#pragma unroll
    for (int it = 0; it < IT1; ++it) {
        k1[it] = (it * GS1 + lg1) * 8;
        ok1[it] = k1[it] < H;
    }
    // ---- phase 2 geometry: down, N = H rows of K = F
    const int GS2 = 1 << a.g2.gs_log2, groups2 = 512 >> a.g2.gs_log2, wpg2 = GS2 >> 6;
    const int gid2 = tid >> a.g2.gs_log2, lg2 = tid & (GS2 - 1);
    const int slots2 = gridDim.x * groups2, slot2 = blockIdx.x * groups2 + gid2;
    const int rb2 = (int)((long long)slot2 * H / slots2), re2 = (int)((long long)(slot2 + 1) * H / slots2);
    int k2[IT2];
    bool ok2[IT2];
#pragma unroll
    for (int it = 0; it < IT2; ++it) {
        k2[it] = (it * GS2 + lg2) * 8;
        ok2[it] = k2[it] < F;
    }

    // Weight loads are unconditional, straight-line code: a row past the group's range re-reads its last row (never
    // stored), a thread past the end of a short row reads column 0 and blanks what it got.
    const char *Wg = static_cast<const char *>(a.Wg), *Wu = static_cast<const char *>(a.Wu), *Wd = static_cast<const char *>(a.Wd);
    WV w1[IT1][2][RB1], w2[IT2][RB2];
    auto load1 = [&](int r0) {
#pragma unroll
        for (int it = 0; it < IT1; ++it) {
            const int col = ok1[it] ? k1[it] : 0;
#pragma unroll
            for (int r = 0; r < RB1; ++r) {
                const int row = max(min(r0 + r, re1 - 1), 0);
                const size_t off = ((size_t)row * H + col) * WB;
                const WV g = ldw(Wg + off), u = ldw(Wu + off);
                w1[it][0][r] = ok1[it] ? g : WV{};
                w1[it][1][r] = ok1[it] ? u : WV{};
            }
        }
    };
    auto load2 = [&](int r0) {
#pragma unroll
        for (int it = 0; it < IT2; ++it) {
            const int col = ok2[it] ? k2[it] : 0;
#pragma unroll
            for (int r = 0; r < RB2; ++r) {
                const int row = max(min(r0 + r, re2 - 1), 0);
                const WV d = ldw(Wd + ((size_t)row * F + col) * WB);
                w2[it][r] = ok2[it] ? d : WV{};
            }
        }
    };
    // int8: the thread that will store output (row r, batch entry b) of a pass fetches that row's scale with the pass
    const int my_r1 = lg1 / NB, my_r2 = lg2 / NB;
    float sc1[2] = {0.f, 0.f}, sc2 = 0.f;
    auto scales1 = [&](int r0) {
        if (W8 && lg1 < RB1 * NB && r0 + my_r1 < re1) {
            sc1[0] = a.sg[r0 + my_r1];
            sc1[1] = a.su[r0 + my_r1];
        }
    };
    auto scales2 = [&](int r0) {
        if (W8 && lg2 < RB2 * NB && r0 + my_r2 < re2) sc2 = a.sd[r0 + my_r2];
    };

    // ---- first requests.  Launched the ordinary way, the residual and the gains (cache hits) are requested ahead of
    //      the weights, so that the normalisation runs while the weights travel; launched into its window, the kernel
    //      requests the weights of both phases, waits for the window's end and only then reads the residual.
    float4 xr[IT1][NB][2], xd[IT1][NB][2];
    uint4 gv[IT1];
#pragma unroll
    for (int it = 0; it < IT1; ++it) gv[it] = ok1[it] ? ld16(a.gain + k1[it]) : zero16();   // constants: never after the wait
    if (!WAIT) {
#pragma unroll
        for (int it = 0; it < IT1; ++it) {
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
                xr[it][b][0] = xr[it][b][1] = xd[it][b][0] = xd[it][b][1] = z;
                if (ok1[it]) {
                    xr[it][b][0] = *reinterpret_cast<const float4 *>(a.res + (size_t)b * H + k1[it]);
                    xr[it][b][1] = *reinterpret_cast<const float4 *>(a.res + (size_t)b * H + k1[it] + 4);
                    if (a.delta) {
                        xd[it][b][0] = *reinterpret_cast<const float4 *>(a.delta + (size_t)b * H + k1[it]);
                        xd[it][b][1] = *reinterpret_cast<const float4 *>(a.delta + (size_t)b * H + k1[it] + 4);
                    }
                }
            }
        }
    }
    int r1 = rb1, r2 = rb2;
    load1(r1);
    scales1(r1);
    if (!WAIT || a.hold_down) {
        load2(r2);
        scales2(r2);
    }

    if (WAIT) {
        if (wave == 0) {
            const uint64_t t0 = wall_clock64();
            unsigned v = __hip_atomic_load(a.wait.done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            uint32_t it = 0;
            while ((int)(v - a.wait.seq) < 0 && it < a.wait.iters && wall_clock64() - t0 < a.wait.ticks) {
                __builtin_amdgcn_s_sleep(8);
                v = __hip_atomic_load(a.wait.done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ++it;
            }
            if (lane == 0 && (int)(v - a.wait.seq) < 0) atomicOr(a.err, 1u);
        }
        __syncthreads();
        if (!a.hold_down) {
            load2(r2);
            scales2(r2);
        }
    }

    // ---- rmsnorm(res + delta) * gain into registers
    float xv[IT1][NB][8];
    {
        float ss[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            ss[b] = 0.f;
#pragma unroll
            for (int it = 0; it < IT1; ++it) {
                float4 v0 = make_float4(0.f, 0.f, 0.f, 0.f), v1 = v0;
                if (ok1[it]) {
                    float4 d0 = make_float4(0.f, 0.f, 0.f, 0.f), d1 = d0;
                    if (WAIT) {
                        const float *dp = a.delta ? a.delta : a.res;
                        f32x4 q0, q1, q2, q3;
                        ldc_issue(q0, a.res + (size_t)b * H + k1[it]);
                        ldc_issue(q1, a.res + (size_t)b * H + k1[it] + 4);
                        ldc_issue(q2, dp + (size_t)b * H + k1[it]);
                        ldc_issue(q3, dp + (size_t)b * H + k1[it] + 4);
                        ldc_wait(q0, q1, q2, q3);
                        v0 = make_float4(q0[0], q0[1], q0[2], q0[3]);
                        v1 = make_float4(q1[0], q1[1], q1[2], q1[3]);
                        d0 = make_float4(q2[0], q2[1], q2[2], q2[3]);
                        d1 = make_float4(q3[0], q3[1], q3[2], q3[3]);
                    } else {
                        v0 = xr[it][b][0]; v1 = xr[it][b][1];
                        d0 = xd[it][b][0]; d1 = xd[it][b][1];
                    }
                    if (a.delta) {
                        v0.x += d0.x; v0.y += d0.y; v0.z += d0.z; v0.w += d0.w;
                        v1.x += d1.x; v1.y += d1.y; v1.z += d1.z; v1.w += d1.w;
                    }
                    if (blockIdx.x == 0 && gid1 == 0) {
                        *reinterpret_cast<float4 *>(a.out_res + (size_t)b * H + k1[it]) = v0;
                        *reinterpret_cast<float4 *>(a.out_res + (size_t)b * H + k1[it] + 4) = v1;
                    }
                }
                float *x = xv[it][b];
                x[0] = v0.x; x[1] = v0.y; x[2] = v0.z; x[3] = v0.w;
                x[4] = v1.x; x[5] = v1.y; x[6] = v1.z; x[7] = v1.w;
#pragma unroll
                for (int e = 0; e < 8; ++e) ss[b] += x[e] * x[e];
            }
            ss[b] = wave_sum(ss[b]);
        }
        if (lane == 0)
#pragma unroll
            for (int b = 0; b < NB; ++b) ssq[wave][b] = ss[b];
        __syncthreads();
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            float tot = 0.f;
            for (int w = 0; w < wpg1; ++w) tot += ssq[gid1 * wpg1 + w][b];   // fixed order
            const float inv = 1.0f / sqrtf(tot / (float)H + a.eps);
#pragma unroll
            for (int it = 0; it < IT1; ++it) {
                float *x = xv[it][b];
                if (ok1[it]) {
                    const uint4 g = gv[it];
                    x[0] *= inv * bf16_lo(g.x); x[1] *= inv * bf16_hi(g.x);
                    x[2] *= inv * bf16_lo(g.y); x[3] *= inv * bf16_hi(g.y);
                    x[4] *= inv * bf16_lo(g.z); x[5] *= inv * bf16_hi(g.z);
                    x[6] *= inv * bf16_lo(g.w); x[7] *= inv * bf16_hi(g.w);
                    if (a.out_h && blockIdx.x == 0 && gid1 == 0) {
                        *reinterpret_cast<float4 *>(a.out_h + (size_t)b * H + k1[it]) = make_float4(x[0], x[1], x[2], x[3]);
                        *reinterpret_cast<float4 *>(a.out_h + (size_t)b * H + k1[it] + 4) = make_float4(x[4], x[5], x[6], x[7]);
                    }
                }
            }
        }
    }

    // ---- phase 1: gate/up rows, SwiGLU, tagged stores
    for (int pass = 0; pass < a.g1.passes; ++pass) {
        float acc[2][RB1][NB];
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int r = 0; r < RB1; ++r)
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    float s = 0.f;
#pragma unroll
                    for (int it = 0; it < IT1; ++it) s = dot8(w1[it][q][r], xv[it][b], s);
                    acc[q][r][b] = s;
                }
        // the 2 * RB1 * NB sums over the wave at once: lane l < N1 holds the one of index l = (q * RB1 + r) * NB + b
        constexpr int N1 = 2 * RB1 * NB, CS1 = N1 < 16 ? N1 : 16, NC1 = N1 / CS1;     // in chunks of 16: lane l < CS1, chunk c: index c * CS1 + l
        float tot1[NC1];
#pragma unroll
        for (int c = 0; c < NC1; ++c)
            tot1[c] = wave_sum_scatter<CS1>(reinterpret_cast<const float (&)[CS1]>((&acc[0][0][0])[c * CS1]), lane);
        const int rows_here = r1;
        r1 += RB1;
        const float sg_now = sc1[0], su_now = sc1[1];
        if (pass + 1 < a.g1.passes) {
            load1(r1);
            scales1(r1);
        }
        if (wpg1 == 1) {
            // the gate sum of index i = r * NB + b (chunk i / CS1) and the up sum, RB1 * NB further on, into one lane
            constexpr int HALF1 = RB1 * NB;
            const int i1 = scatter_index<CS1>(lane);
            float gate1 = tot1[0], up1;
            if constexpr (NC1 == 1) {
                up1 = __int_as_float(__builtin_amdgcn_ds_bpermute(scatter_holder((i1 + HALF1) & (CS1 - 1)) << 2, __float_as_int(tot1[0])));
            } else {
                static_assert(NC1 == 1 || (NC1 == 2 && HALF1 == 16), "gate sums in the first chunk, up sums in the second");
                up1 = tot1[NC1 - 1];
            }
            if (lane < CS1 && i1 < HALF1) {
                const int r = i1 / NB, b = i1 % NB;
                if (rows_here + r < re1) {
                    float v = gate1, u = up1;
                    if (W8) {
                        v *= a.sg[rows_here + r];
                        u *= a.su[rows_here + r];
                    }
                    st_wt4(a.m + (size_t)b * F + rows_here + r, __float_as_uint(silu_mul(v, u)));
                }
            }
        } else {
            if (lane < CS1)
#pragma unroll
                for (int c = 0; c < NC1; ++c) red[wave][c * CS1 + scatter_index<CS1>(lane)] = tot1[c];
            __syncthreads();
            if (lg1 < RB1 * NB) {
                const int r = lg1 / NB, b = lg1 % NB;
                if (rows_here + r < re1) {
                    float v = 0.f, u = 0.f;
                    for (int w = 0; w < wpg1; ++w) {   // fixed order
                        v += red[gid1 * wpg1 + w][r * NB + b];
                        u += red[gid1 * wpg1 + w][(RB1 + r) * NB + b];
                    }
                    if (W8) {
                        v *= sg_now;
                        u *= su_now;
                    }
                    st_wt4(a.m + (size_t)b * F + rows_here + r, __float_as_uint(silu_mul(v, u)));
                }
            }
            __syncthreads();
        }
    }

    // this workgroup's part of m is at the memory side once its stores are acknowledged: it says so in the indicator array
    // ([copy][workgroup], kSegIndCopies copies written by as many lanes at once, so that the watchers below do not all
    // poll the same lines)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid < kSegIndCopies) ll_store(a.m_ll + (size_t)NB * F + tid * kSegIndStride + blockIdx.x, 0.f, a.tag);

    // ---- hand-over: every thread polls its slice of m until all of it carries this launch's tag
    float mv[IT2][NB][8];
    {
        // one wave per workgroup first watches the producers' indicator entries (its copy of them), sleeping between looks, while
        // the others wait at the barrier: 130 000 threads polling from the moment they are done would slow the
        // stores they are waiting for
        if (wave == 0) {
            bool ready = false;
            for (uint32_t spin = 0; !ready && spin < a.ll_iters; ++spin) {
                bool mine = true;
                const uint2 *ind = a.m_ll + (size_t)NB * F + (blockIdx.x % kSegIndCopies) * kSegIndStride;
                for (int p0 = 0; p0 < (int)gridDim.x; p0 += 256) {
                    uint2 v[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u)        // workgroup p0 + lane + 64 u (clamped: a repeat is harmless)
                        ll_issue1(v[u], ind + min(p0 + lane + 64 * u, (int)gridDim.x - 1));
                    asm volatile("s_waitcnt vmcnt(0)" : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]) : : "memory");
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (v[u].y != a.tag) mine = false;
                }
                ready = __all(mine);
                if (!ready) __builtin_amdgcn_s_sleep(8);
            }
            if (!ready && lane == 0) atomicOr(a.err, 2u);       // part of m may be missing: results invalid
        }
        __syncthreads();
        // all of m is complete at the memory side and nothing on this CU has read it since the kernel started: ordinary
        // loads, served by the XCD's L2 after the first workgroup's
#pragma unroll
        for (int it = 0; it < IT2; ++it)
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                float4 m0 = make_float4(0.f, 0.f, 0.f, 0.f), m1 = m0;
                if (ok2[it]) {
                    m0 = *reinterpret_cast<const float4 *>(a.m + (size_t)b * F + k2[it]);
                    m1 = *reinterpret_cast<const float4 *>(a.m + (size_t)b * F + k2[it] + 4);
                }
                mv[it][b][0] = m0.x; mv[it][b][1] = m0.y; mv[it][b][2] = m0.z; mv[it][b][3] = m0.w;
                mv[it][b][4] = m1.x; mv[it][b][5] = m1.y; mv[it][b][6] = m1.z; mv[it][b][7] = m1.w;
            }
    }

    // ---- phase 2: down rows
    for (int pass = 0; pass < a.g2.passes; ++pass) {
        float acc[RB2][NB];
#pragma unroll
        for (int r = 0; r < RB2; ++r)
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                float s = 0.f;
#pragma unroll
                for (int it = 0; it < IT2; ++it) s = dot8(w2[it][r], mv[it][b], s);
                acc[r][b] = s;
            }
        constexpr int N2 = RB2 * NB;        // lane l < N2 holds the sum of index l = r * NB + b
        static_assert(N2 <= 16, "one scatter sum");
        const float tot2 = wave_sum_scatter<N2>(reinterpret_cast<const float (&)[N2]>(acc), lane);
        const int rows_here = r2;
        r2 += RB2;
        const float sd_now = sc2;
        if (pass + 1 < a.g2.passes) {
            load2(r2);
            scales2(r2);
        }
        if (wpg2 == 1) {
            if (lane < N2) {
                const int i2 = scatter_index<N2>(lane), r = i2 / NB, b = i2 % NB;
                if (rows_here + r < re2) {
                    float v = tot2;
                    if (W8) v *= a.sd[rows_here + r];
                    a.out[(size_t)b * H + rows_here + r] = v;
                }
            }
        } else {
            if (lane < N2) red[wave][scatter_index<N2>(lane)] = tot2;
            __syncthreads();
            if (lg2 < RB2 * NB) {
                const int r = lg2 / NB, b = lg2 % NB;
                if (rows_here + r < re2) {
                    float v = 0.f;
                    for (int w = 0; w < wpg2; ++w) v += red[gid2 * wpg2 + w][r * NB + b];   // fixed order
                    if (W8) v *= sd_now;
                    a.out[(size_t)b * H + rows_here + r] = v;
                }
            }
            __syncthreads();
        }
    }
}

// ---- launch

bool seg_mlp_supported(int batch, int H, int F)
{
    return batch == 1 && H % 8 == 0 && F % 8 == 0 && H >= 64 && F >= 64 && H <= 8192 && F <= 8192;
}

bool seg_mlp_holds_gate_up(int H, int F, bool w8, int blocks)
{
    const int r1 = w8 ? 8 : 4;
    if (H > 4096) return seg_geom(F, H, 2, r1, blocks).passes == 1;
    return seg_geom(F, H, 1, r1, blocks).passes <= (F > 4096 ? 1 : 2);     // see seg_mlp_pick: two passes' worth fit when rows are long
}

bool seg_mlp_holds_down(int H, int F, bool w8, int blocks)
{
    return seg_geom(H, F, F > 4096 ? 2 : 1, w8 ? 16 : 8, blocks).passes == 1;
}

template <int NB, int RB1, int IT1, int RB2, int IT2, bool W8>
static hipError_t seg_mlp_go(SegMlpArgs a, bool wait, int blocks, hipStream_t s)
{
    a.g1 = seg_geom(a.F, a.H, IT1, RB1, blocks);
    a.g2 = seg_geom(a.H, a.F, IT2, RB2, blocks);
    if (wait)
        PSV_LAUNCH((k_seg_mlp<NB, RB1, IT1, RB2, IT2, W8, true>), dim3(blocks), dim3(512), 0, s, a);
    else
        PSV_LAUNCH((k_seg_mlp<NB, RB1, IT1, RB2, IT2, W8, false>), dim3(blocks), dim3(512), 0, s, a);
    return hipGetLastError();
}

template <int NB, bool W8>
static hipError_t seg_mlp_pick(const SegMlpArgs &a, bool wait, int blocks, hipStream_t s)
{
    constexpr int R1 = W8 ? 8 : 4, R2 = W8 ? 16 : 8;    // 8 x 16 bytes (gate + up) and 8 x 16 bytes in flight per thread and pass
    const bool two1 = a.H > 4096, two2 = a.F > 4096;
    if (two1) return two2 ? seg_mlp_go<NB, R1, 2, R2, 2, W8>(a, wait, blocks, s) : seg_mlp_go<NB, R1, 2, R2, 1, W8>(a, wait, blocks, s);
    // rows longer than half of what a thread group covers in one load leave few rows per group: the whole first pass
    // fits twice over (c2: 7 gate + 7 up rows per workgroup)
    const SegGeom g = seg_geom(a.F, a.H, 1, R1, blocks);
    if (g.passes == 2 && !two2) return seg_mlp_go<NB, 2 * R1, 1, R2, 1, W8>(a, wait, blocks, s);
    return two2 ? seg_mlp_go<NB, R1, 1, R2, 2, W8>(a, wait, blocks, s) : seg_mlp_go<NB, R1, 1, R2, 1, W8>(a, wait, blocks, s);
}

hipError_t launch_seg_mlp(Mat Wg, Mat Wu, Mat Wd, const float *res, const float *delta, const uint16_t *gain, float eps,
                          float *out_res, float *out_h, float *m, void *m_ll, float *out, int batch, int H, int F, unsigned tag,
                          unsigned *err, const GemvWait *wait, bool hold_down, uint32_t poll_iters, int blocks, hipStream_t s)
{
    SegMlpArgs a{};
    a.Wg = Wg.w; a.Wu = Wu.w; a.Wd = Wd.w; a.sg = Wg.scale; a.su = Wu.scale; a.sd = Wd.scale;
    a.res = res; a.delta = delta; a.gain = gain; a.eps = eps; a.out_res = out_res; a.out_h = out_h;
    a.m = m; a.m_ll = static_cast<uint2 *>(m_ll); a.out = out; a.F = F; a.H = H; a.tag = tag; a.ll_iters = poll_iters; a.err = err;
    if (wait) a.wait = SegWait{wait->done, wait->seq, wait->iters, wait->ticks};
    a.hold_down = hold_down ? 1 : 0;
    if (batch != 1 || blocks > kSegIndStride) return hipErrorInvalidValue;
    return Wg.scale ? seg_mlp_pick<1, true>(a, wait != nullptr, blocks, s) : seg_mlp_pick<1, false>(a, wait != nullptr, blocks, s);
}


// ------------------------------------------------------------------------------------ attention block


constexpr int kSegChunkTokens = 256;     // 8 waves x one 32-token tile
constexpr int kSegMaxChunks = 16;        // per kv head: sequences of up to 4096 tokens

struct SegAttnArgs {
    const void *Wq, *Wo;                // [QR][H], [H][QD]
    const float *sq, *so;               // int8: row scales
    const float *res, *delta;           // residual entering the block = res + delta, [H]
    const uint16_t *gain;
    float eps;
    float *out_res, *out_h;             // res + delta and the normalised activations, stored by workgroup 0
    uint2 *qkv_ll;                      // [QR] tagged projection output (q heads, k heads, v heads), not yet rotated
    const float2 *rope;                 // [64] (cos, sin) at position T-1
    KvView kv;
    int nq, nkv, n_chunks;
    float2 *pml;                        // [nkv][n_chunks][16] (max, sum) of every partial and head
    float *po;                          // [nkv][n_chunks][G][128] partial outputs
    uint2 *ind_ll;                      // [kSegIndCopies][kSegIndStride] one entry per partial: that workgroup has stored it
    float *out_attn;                    // [QD] merged attention output, stored by workgroup 0
    float *out;                         // [H] O projection
    int H, QR, QD;
    SegGeom gq, go;
    unsigned tag;
    uint32_t ll_iters;
    unsigned *err;
    SegWait wait;
    int hold_kv, hold_o;                // launched into its window: request the K/V tile / the O weights before (1) or after (0) the wait
};

// QKV projection -> rotary embedding, KV append, decode attention -> merge + O projection, one sequence.
// Workgroup kvh * n_chunks + c also runs the attention of tokens [256 c, 256 c + 256) of kv head kvh: wave w takes the
// 32-token tile w, all G query heads of the kv head ride in the N side of the matrix-core contractions exactly as in
// k_attn, the 8 waves merge through LDS in a fixed tree order and the workgroup stores one tagged partial.
template <int RBQ, int ITQ, int RBO, bool W8, bool WAIT>
__global__ __launch_bounds__(512) void k_seg_attn(SegAttnArgs a)
{
    constexpr int WB = W8 ? 1 : 2;
    using WV = typename std::conditional<W8, uint2, uint4>::type;
    constexpr int RED = RBQ > RBO ? RBQ : RBO;
    __shared__ float red[8][RED];
    __shared__ float ssq[8];
    __shared__ float xs[4096];
    __shared__ f32x4 accs[8][8][64];
    __shared__ float ms[8][16], ls[8][16];
    __shared__ float2 rope_s[64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, i = lane & 15, q4 = lane >> 4;
    auto ldw = [](const char *p) {
        // streamed once: non-temporal, so that the weights do not push the kernel's code and the activations out of L2
        if constexpr (W8) {
            const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(p));
            return make_uint2(v.x, v.y);
        } else {
            const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
            return make_uint4(v.x, v.y, v.z, v.w);
        }
    };
    const int H = a.H, QR = a.QR, QD = a.QD, nq = a.nq, nkv = a.nkv, G = nq / nkv, nc = a.n_chunks;
    const KvView &kv = a.kv;

    // ---- QKV geometry: N = QR rows of K = H
    const int GS1 = 1 << a.gq.gs_log2, groups1 = 512 >> a.gq.gs_log2, wpg1 = GS1 >> 6;
    const int gid1 = tid >> a.gq.gs_log2, lg1 = tid & (GS1 - 1);
    const int slots1 = gridDim.x * groups1, slot1 = blockIdx.x * groups1 + gid1;
    const int rb1 = (int)((long long)slot1 * QR / slots1), re1 = (int)((long long)(slot1 + 1) * QR / slots1);
    int k1[ITQ];
    bool ok1[ITQ];
#pragma unroll
    for (int it = 0; it < ITQ; ++it) {
        k1[it] = (it * GS1 + lg1) * 8;
        ok1[it] = k1[it] < H;
    }
    // ---- O geometry: N = H rows of K = QD (<= 4096: one load per thread and row)
    const int GS3 = 1 << a.go.gs_log2, groups3 = 512 >> a.go.gs_log2, wpg3 = GS3 >> 6;
    const int gid3 = tid >> a.go.gs_log2, lg3 = tid & (GS3 - 1);
    const int slots3 = gridDim.x * groups3, slot3 = blockIdx.x * groups3 + gid3;
    const int rb3 = (int)((long long)slot3 * H / slots3), re3 = (int)((long long)(slot3 + 1) * H / slots3);
    const int k3 = lg3 * 8;
    const bool ok3 = k3 < QD;

    const char *Wq = static_cast<const char *>(a.Wq), *Wo = static_cast<const char *>(a.Wo);
    WV w1[ITQ][RBQ], w3[RBO];
    auto load1 = [&](int r0) {
#pragma unroll
        for (int it = 0; it < ITQ; ++it) {
            const int col = ok1[it] ? k1[it] : 0;
#pragma unroll
            for (int r = 0; r < RBQ; ++r) {
                const int row = max(min(r0 + r, re1 - 1), 0);
                const WV v = ldw(Wq + ((size_t)row * H + col) * WB);
                w1[it][r] = ok1[it] ? v : WV{};
            }
        }
    };
    auto load3 = [&](int r0) {
        const int col = ok3 ? k3 : 0;
#pragma unroll
        for (int r = 0; r < RBO; ++r) {
            const int row = max(min(r0 + r, re3 - 1), 0);
            const WV v = ldw(Wo + ((size_t)row * QD + col) * WB);
            w3[r] = ok3 ? v : WV{};
        }
    };
    const int my_r1 = lg1, my_r3 = lg3;
    float sc1 = 0.f, sc3 = 0.f;
    auto scales1 = [&](int r0) { if (W8 && lg1 < RBQ && r0 + my_r1 < re1) sc1 = a.sq[r0 + my_r1]; };
    auto scales3 = [&](int r0) { if (W8 && lg3 < RBO && r0 + my_r3 < re3) sc3 = a.so[r0 + my_r3]; };

    // ---- attention role of this workgroup
    const bool att = (int)blockIdx.x < nkv * nc;
    const int kvh = att ? (int)blockIdx.x / nc : 0, c = att ? (int)blockIdx.x % nc : 0;
    int T = kv.seq_lens[0];
    if (T < 0 || T > kv.max_tokens) T = 0;
    const int t_begin = c * kSegChunkTokens, t_end = min(T, t_begin + kSegChunkTokens);
    const int t0 = t_begin + wave * kAttnTileTokens;
    const bool early = att && t0 < kv.max_blocks * 16;
    const int tau1 = 8 * (i >> 2) + (i & 3);
    uint4 ka[4], kb[4], vf[8];
    auto lookup = [&](int &blkA, int &blkB) {
        const int lb = t0 >> 4;
        blkA = kv_phys_block(kv.page_table, kv.max_blocks, kv.num_pool_blocks, 0, lb);
        blkB = (lb + 1 < kv.max_blocks) ? kv_phys_block(kv.page_table, kv.max_blocks, kv.num_pool_blocks, 0, lb + 1) : -1;
    };
    auto load_blocks = [&](int blkA, int blkB) {
        {
            const int blk = (i < 8) ? blkA : blkB;
            if (blk >= 0) {
                const uint16_t *base = kv.k_pool + (((size_t)blk * nkv + kvh) * 16 + (tau1 & 15)) * 128 + q4 * 8;
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
                const uint16_t *base = kv.v_pool + (((size_t)blk * nkv + kvh) * 128 + i) * 16 + (q4 & 1) * 8;
#pragma unroll
                for (int dg = 0; dg < 8; ++dg) vf[dg] = ld16(base + dg * 16 * 16);
            } else {
#pragma unroll
                for (int dg = 0; dg < 8; ++dg) vf[dg] = zero16();
            }
        }
    };
    auto load_tile = [&]() {
        int blkA, blkB;
        lookup(blkA, blkB);
        load_blocks(blkA, blkB);
    };

    // ---- first requests.  Loads return in order, so what is small and needed early goes first: the page-table entries
    //      of the tile and the rotary table (attention workgroups), then -- launched the ordinary way -- the residual
    //      and the gains (see k_seg_mlp), then the weights of both projections, then the K/V tile.
    int blkA0 = -1, blkB0 = -1;
    float2 rope_v = make_float2(1.f, 0.f);
    if (att && tid < 64) rope_v = a.rope[tid];
    if (early) lookup(blkA0, blkB0);
    float4 xr[ITQ][2], xd[ITQ][2];
    uint4 gv[ITQ];
#pragma unroll
    for (int it = 0; it < ITQ; ++it) gv[it] = ok1[it] ? ld16(a.gain + k1[it]) : zero16();   // constants: never after the wait
    if (!WAIT) {
#pragma unroll
        for (int it = 0; it < ITQ; ++it) {
            const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
            xr[it][0] = xr[it][1] = xd[it][0] = xd[it][1] = z;
            if (ok1[it]) {
                xr[it][0] = *reinterpret_cast<const float4 *>(a.res + k1[it]);
                xr[it][1] = *reinterpret_cast<const float4 *>(a.res + k1[it] + 4);
                if (a.delta) {
                    xd[it][0] = *reinterpret_cast<const float4 *>(a.delta + k1[it]);
                    xd[it][1] = *reinterpret_cast<const float4 *>(a.delta + k1[it] + 4);
                }
            }
        }
    }
    int r1 = rb1, r3 = rb3;
    load1(r1);
    scales1(r1);
    if (!WAIT || a.hold_o) {
        load3(r3);
        scales3(r3);
    }
    if (early && (!WAIT || a.hold_kv)) load_blocks(blkA0, blkB0);

    if (WAIT) {
        if (wave == 0) {
            const uint64_t tw = wall_clock64();
            unsigned v = __hip_atomic_load(a.wait.done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            uint32_t it = 0;
            while ((int)(v - a.wait.seq) < 0 && it < a.wait.iters && wall_clock64() - tw < a.wait.ticks) {
                __builtin_amdgcn_s_sleep(8);
                v = __hip_atomic_load(a.wait.done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ++it;
            }
            if (lane == 0 && (int)(v - a.wait.seq) < 0) atomicOr(a.err, 1u);
        }
        __syncthreads();
        if (early && !a.hold_kv) load_blocks(blkA0, blkB0);
        if (!a.hold_o) {
            load3(r3);
            scales3(r3);
        }
    }

    // ---- rmsnorm(res + delta) * gain into registers
    float xv[ITQ][8];
    {
        float ss = 0.f;
#pragma unroll
        for (int it = 0; it < ITQ; ++it) {
            float4 v0 = make_float4(0.f, 0.f, 0.f, 0.f), v1 = v0;
            if (ok1[it]) {
                float4 d0 = make_float4(0.f, 0.f, 0.f, 0.f), d1 = d0;
                if (WAIT) {
                    const float *dp = a.delta ? a.delta : a.res;
                    f32x4 p0, p1, p2, p3;
                    ldc_issue(p0, a.res + k1[it]);
                    ldc_issue(p1, a.res + k1[it] + 4);
                    ldc_issue(p2, dp + k1[it]);
                    ldc_issue(p3, dp + k1[it] + 4);
                    ldc_wait(p0, p1, p2, p3);
                    v0 = make_float4(p0[0], p0[1], p0[2], p0[3]);
                    v1 = make_float4(p1[0], p1[1], p1[2], p1[3]);
                    d0 = make_float4(p2[0], p2[1], p2[2], p2[3]);
                    d1 = make_float4(p3[0], p3[1], p3[2], p3[3]);
                } else {
                    v0 = xr[it][0]; v1 = xr[it][1];
                    d0 = xd[it][0]; d1 = xd[it][1];
                }
                if (a.delta) {
                    v0.x += d0.x; v0.y += d0.y; v0.z += d0.z; v0.w += d0.w;
                    v1.x += d1.x; v1.y += d1.y; v1.z += d1.z; v1.w += d1.w;
                }
                if (blockIdx.x == 0 && gid1 == 0) {
                    *reinterpret_cast<float4 *>(a.out_res + k1[it]) = v0;
                    *reinterpret_cast<float4 *>(a.out_res + k1[it] + 4) = v1;
                }
            }
            float *x = xv[it];
            x[0] = v0.x; x[1] = v0.y; x[2] = v0.z; x[3] = v0.w;
            x[4] = v1.x; x[5] = v1.y; x[6] = v1.z; x[7] = v1.w;
#pragma unroll
            for (int e = 0; e < 8; ++e) ss += x[e] * x[e];
        }
        ss = wave_sum(ss);
        if (lane == 0) ssq[wave] = ss;
        if (att && tid < 64) rope_s[tid] = rope_v;      // stored here, not where it was requested: by now it has arrived
        __syncthreads();
        float tot = 0.f;
        for (int w = 0; w < wpg1; ++w) tot += ssq[gid1 * wpg1 + w];   // fixed order
        const float inv = 1.0f / sqrtf(tot / (float)H + a.eps);
#pragma unroll
        for (int it = 0; it < ITQ; ++it) {
            float *x = xv[it];
            if (ok1[it]) {
                const uint4 g = gv[it];
                x[0] *= inv * bf16_lo(g.x); x[1] *= inv * bf16_hi(g.x);
                x[2] *= inv * bf16_lo(g.y); x[3] *= inv * bf16_hi(g.y);
                x[4] *= inv * bf16_lo(g.z); x[5] *= inv * bf16_hi(g.z);
                x[6] *= inv * bf16_lo(g.w); x[7] *= inv * bf16_hi(g.w);
                if (a.out_h && blockIdx.x == 0 && gid1 == 0) {
                    *reinterpret_cast<float4 *>(a.out_h + k1[it]) = make_float4(x[0], x[1], x[2], x[3]);
                    *reinterpret_cast<float4 *>(a.out_h + k1[it] + 4) = make_float4(x[4], x[5], x[6], x[7]);
                }
            }
        }
    }

    // ---- phase 1: QKV rows, tagged stores
    for (int pass = 0; pass < a.gq.passes; ++pass) {
        float acc[RBQ];
#pragma unroll
        for (int r = 0; r < RBQ; ++r) {
            float s = 0.f;
#pragma unroll
            for (int it = 0; it < ITQ; ++it) s = dot8(w1[it][r], xv[it], s);
            acc[r] = s;
        }
        const float tot1 = wave_sum_scatter<RBQ>(acc, lane);      // lane l < RBQ: the sum of row scatter_index<RBQ>(l)
        const int rows_here = r1;
        r1 += RBQ;
        const float sc_now = sc1;
        if (pass + 1 < a.gq.passes) {
            load1(r1);
            scales1(r1);
        }
        if (wpg1 == 1) {
            const int r = scatter_index<RBQ>(lane);
            if (lane < RBQ && rows_here + r < re1) {
                float v = tot1;
                if (W8) v *= a.sq[rows_here + r];
                ll_store(a.qkv_ll + rows_here + r, v, a.tag);
            }
        } else {
            if (lane < RBQ) red[wave][scatter_index<RBQ>(lane)] = tot1;
            __syncthreads();
            if (lg1 < RBQ && rows_here + lg1 < re1) {
                float v = 0.f;
                for (int w = 0; w < wpg1; ++w) v += red[gid1 * wpg1 + w][lg1];   // fixed order
                if (W8) v *= sc_now;
                ll_store(a.qkv_ll + rows_here + lg1, v, a.tag);
            }
            __syncthreads();
        }
    }

    // ---- phase 2: attention of this workgroup's chunk
    if (att) {
        bool lost = false;
        // query rows of the G heads, rotated, as hi + lo bf16 fragments (lane (g = i, q4): channels ks*32 + q4*8 + e and + 64)
        bf16x8 qf[4], qfl[4];
        {
            const uint4 z = zero16();
            qf[0] = qf[1] = qf[2] = qf[3] = __builtin_bit_cast(bf16x8, z);
            qfl[0] = qfl[1] = qfl[2] = qfl[3] = __builtin_bit_cast(bf16x8, z);
            // The G query rows of this kv head (and its new key and value rows) are polled once per workgroup, one
            // value per thread, into LDS: eight waves each polling all of it multiplied the traffic on the one or
            // two memory channels that hold these few KB, and a poll took 4 us instead of 1.
            float *qs = xs;                                   // [G + 2][128]: free until the merge of phase 3
            bool all = false;
            {
                const int n_val = (G + 2) * 128;
                for (uint32_t spin = 0; !all && spin < a.ll_iters; ++spin) {
                    bool mine = true;
                    uint2 pv[5];                                  // (16 + 2) * 128 values / 512 threads
#pragma unroll
                    for (int u = 0; u < 5; ++u) {
                        const int v0 = tid + 512 * u;
                        if (v0 < n_val) {
                            const int hrow = v0 >> 7;             // 0..G-1: query heads; G: new key; G+1: new value
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
                            if (pv[u].y != a.tag) mine = false;
                            qs[v0] = __uint_as_float(pv[u].x);
                        }
                    }
                    all = __syncthreads_and(mine ? 1 : 0) != 0;
                    if (!all) __builtin_amdgcn_s_sleep(2);
                }
            }
            if (!all) lost = true;
            // The rotated query as hi + lo fragments: four pieces -- (k half ks, the rotation's first or second output) -- of
            // which waves 0..3 form one each and leave it in LDS for all eight (every wave forming all four cost 0.85 us,
            // three quarters of it redundant).  accs is free until the merge.
            uint4 *qfs = reinterpret_cast<uint4 *>(&accs[0][0][0]);      // [8][64]: qf[0..3], qfl[0..3]
            if (wave < 4) {
                const int ks = wave & 1, second = wave >> 1;
                uint4 fh = zero16(), fl = zero16();
                if (i < G) {
                    float qlo[8], qhi[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        qlo[e] = qs[i * 128 + ks * 32 + q4 * 8 + e];
                        qhi[e] = qs[i * 128 + ks * 32 + q4 * 8 + e + 64];
                    }
                    const int f0 = ks * 32 + q4 * 8;
                    uint32_t h[4], l[4];
#pragma unroll
                    for (int e = 0; e < 8; e += 2) {
                        const float2 c0 = rope_s[f0 + e], c1 = rope_s[f0 + e + 1];
                        if (!second) pack_split(qlo[e] * c0.x - qhi[e] * c0.y, qlo[e + 1] * c1.x - qhi[e + 1] * c1.y, h[e >> 1], l[e >> 1]);
                        else pack_split(qhi[e] * c0.x + qlo[e] * c0.y, qhi[e + 1] * c1.x + qlo[e + 1] * c1.y, h[e >> 1], l[e >> 1]);
                    }
                    fh = make_uint4(h[0], h[1], h[2], h[3]);
                    fl = make_uint4(l[0], l[1], l[2], l[3]);
                }
                qfs[(ks + 2 * second) * 64 + lane] = fh;
                qfs[(4 + ks + 2 * second) * 64 + lane] = fl;
            }
            __syncthreads();
#pragma unroll
            for (int f = 0; f < 4; ++f) {
                qf[f] = __builtin_bit_cast(bf16x8, qfs[f * 64 + lane]);
                qfl[f] = __builtin_bit_cast(bf16x8, qfs[(4 + f) * 64 + lane]);
            }
        }
        // append the new token's K and V (the workgroup whose chunk holds token T-1)
        if (T >= 1 && c == (T - 1) / kSegChunkTokens) {
            if (wave == 0) {
                const int pos = T - 1;
                const int blk = kv_phys_block(kv.page_table, kv.max_blocks, kv.num_pool_blocks, 0, pos >> 4);
                if (blk >= 0) {
                    const float2 cs = rope_s[lane];
                    const float *ksrc = xs + G * 128, *vsrc = xs + (G + 1) * 128;
                    const float lo = ksrc[lane], hi = ksrc[lane + 64];
                    const int r = pos & 15;
                    uint16_t *kdst = kv.k_pool + (((size_t)blk * nkv + kvh) * 16 + r) * 128;
                    kdst[lane] = (uint16_t)f32_to_bf16(lo * cs.x - hi * cs.y);
                    kdst[lane + 64] = (uint16_t)f32_to_bf16(hi * cs.x + lo * cs.y);
                    uint16_t *vdst = kv.v_pool + ((size_t)blk * nkv + kvh) * 128 * 16 + r;
                    vdst[(size_t)lane * 16] = (uint16_t)f32_to_bf16(vsrc[lane]);
                    vdst[(size_t)(lane + 64) * 16] = (uint16_t)f32_to_bf16(vsrc[lane + 64]);
                }
            }
            // the new rows are read back by this workgroup only (its own tile), through the CU's cache: the barrier's
            // workgroup-scope ordering is all that needs (a device-scope fence here cost the one workgroup that appends,
            // and so the whole hand-over, a write-back of its XCD's L2)
            __syncthreads();   // uniform: the condition depends on the workgroup only
            if (early && T - 1 >= t0 && T - 1 < t0 + kAttnTileTokens) load_tile();   // now with the new entry
        }

        const float kScale = 0.08838834764831845f * 1.4426950408889634f;   // 1/sqrt(128) * log2(e)
        float m_run = -1.0e30f, l_part = 0.f;
        f32x4 acc[8];
#pragma unroll
        for (int dg = 0; dg < 8; ++dg) acc[dg] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (t0 < t_end) {
            if (!early) load_tile();
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
            if (t0 + kAttnTileTokens > t_end) {   // ragged tail: blank cache slots past the span (they may hold anything)
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
        // merge of the 8 waves: common maximum, then a fixed summation order
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
        // every wave leaves its scaled accumulators in LDS; one barrier, then wave w sums channel group w over the eight
#pragma unroll
        for (int dg = 0; dg < 8; ++dg) accs[wave][dg][lane] = acc[dg];
        __syncthreads();
        if (i < G) {
            const size_t slot = (size_t)kvh * nc + c;
            if (wave == 0 && q4 == 0) {
                float L = ls[0][i];
#pragma unroll
                for (int w = 1; w < 8; ++w) L += ls[w][i];
                st_wt8(a.pml + slot * 16 + i, make_uint2(__float_as_uint(M), __float_as_uint(L)));
            }
            // wave w finishes and stores channel group w: ((0+4) + (1+5)) + ((2+6) + (3+7))
            const f32x4 v = ((accs[0][wave][lane] + accs[4][wave][lane]) + (accs[1][wave][lane] + accs[5][wave][lane])) +
                            ((accs[2][wave][lane] + accs[6][wave][lane]) + (accs[3][wave][lane] + accs[7][wave][lane]));
            st_wt16(a.po + (slot * G + i) * 128 + wave * 16 + 4 * q4, make_float4(v[0], v[1], v[2], v[3]));
        }
        if (lost && lane == 0) atomicOr(a.err, 2u);
        // The partial itself is plain data, written through to the memory side; once every wave's stores are
        // acknowledged the workgroup says so with a tagged entry in every copy of the indicator array (copies, so that the
        // watchers below do not all poll the same lines).  The readers then use ordinary loads, which their XCD's L2 serves
        // after the first: with tagged values and device-coherent loads 256 workgroups reading all 32 KB took 2.4 us.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid < kSegIndCopies) ll_store(a.ind_ll + tid * kSegIndStride + kvh * nc + c, 0.f, a.tag);
    }

    // ---- phase 3: merge of the chunk partials (once per workgroup, into LDS), then the O rows
    {
        constexpr int MB = 8;
        bool lost = false;
        // While the attention runs, one wave per workgroup watches the indicator entry of every partial (in its copy of
        // them), sleeping between looks; the others wait at the barrier.  (All threads polling their own values from the start kept the memory
        // side so busy that the attention workgroups' tagged stores took 15 us to get through.)
        if (wave == 0) {
            const int n_part = nkv * nc;
            bool all = false;
            for (uint32_t spin = 0; !all && spin < a.ll_iters; ++spin) {
                bool mine = true;
                for (int pi = lane; pi < n_part; pi += 64) {
                    uint2 v;
                    ll_issue1(v, a.ind_ll + (blockIdx.x % kSegIndCopies) * kSegIndStride + pi);
                    asm volatile("s_waitcnt vmcnt(0)" : "+v"(v) : : "memory");
                    if (v.y != a.tag) mine = false;
                }
                all = __all(mine);
                if (!all) __builtin_amdgcn_s_sleep(16);
            }
            if (!all) lost = true;          // a partial may be missing: results invalid
        }
        __syncthreads();
        // every partial is complete at the memory side; nothing on this CU has read these addresses since the kernel started
        for (int ch = tid; ch < QD; ch += 512) {
            const int j = ch >> 7, c7 = ch & 127, hk = j / G, g = j % G;
            const float2 *mlp = a.pml + ((size_t)hk * nc) * 16 + g;
            const float *op = a.po + (((size_t)hk * nc) * G + g) * 128 + c7;
            float Mx = -1.0e30f, den = 0.f, num = 0.f;
            for (int sp0 = 0; sp0 < nc; sp0 += MB) {
                float2 ml[MB];
                float ov[MB];
#pragma unroll
                for (int u = 0; u < MB; ++u) {
                    const int sp = min(sp0 + u, nc - 1);
                    ml[u] = mlp[(size_t)sp * 16];
                    ov[u] = op[(size_t)sp * G * 128];
                }
                float bm = Mx;
#pragma unroll
                for (int u = 0; u < MB; ++u)
                    if (sp0 + u < nc) bm = fmaxf(bm, ml[u].x);
                const float rs = exp2f(Mx - bm);
                Mx = bm;
                den *= rs;
                num *= rs;
#pragma unroll
                for (int u = 0; u < MB; ++u)
                    if (sp0 + u < nc) {
                        const float lsum = ml[u].y;
                        const float wgt = lsum > 0.f ? exp2f(ml[u].x - Mx) : 0.f;
                        den += wgt * lsum;
                        num = fmaf(wgt, ov[u], num);
                    }
            }
            const float r = den > 0.f ? num / den : 0.f;
            xs[ch] = r;
            if (blockIdx.x == 0 && a.out_attn) a.out_attn[ch] = r;
        }
        if (lost && lane == 0) atomicOr(a.err, 2u);
        __syncthreads();
        float xo[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) xo[e] = ok3 ? xs[k3 + e] : 0.f;
        for (int pass = 0; pass < a.go.passes; ++pass) {
            float acc[RBO];
#pragma unroll
            for (int r = 0; r < RBO; ++r) acc[r] = dot8(w3[r], xo, 0.f);
            const float tot3 = wave_sum_scatter<RBO>(acc, lane);
            const int rows_here = r3;
            r3 += RBO;
            const float sc_now = sc3;
            if (pass + 1 < a.go.passes) {
                load3(r3);
                scales3(r3);
            }
            if (wpg3 == 1) {
                const int r = scatter_index<RBO>(lane);
                if (lane < RBO && rows_here + r < re3) {
                    float v = tot3;
                    if (W8) v *= a.so[rows_here + r];
                    a.out[rows_here + r] = v;
                }
            } else {
                if (lane < RBO) red[wave][scatter_index<RBO>(lane)] = tot3;
                __syncthreads();
                if (lg3 < RBO && rows_here + lg3 < re3) {
                    float v = 0.f;
                    for (int w = 0; w < wpg3; ++w) v += red[gid3 * wpg3 + w][lg3];   // fixed order
                    if (W8) v *= sc_now;
                    a.out[rows_here + lg3] = v;
                }
                __syncthreads();
            }
        }
    }
}

int seg_attn_chunks(uint32_t max_seq) { return (int)((max_seq + kSegChunkTokens - 1) / kSegChunkTokens); }

bool seg_attn_supported(int batch, int H, int nq, int nkv, uint32_t max_seq, bool kv_int8, int blocks)
{
    const int nc = seg_attn_chunks(max_seq);
    return batch == 1 && !kv_int8 && H % 8 == 0 && H >= 64 && H <= 8192 && nq * 128 <= 4096 && nc >= 1 && nc <= kSegMaxChunks &&
           nkv * nc <= blocks;
}

static int seg_rbo(int H, int QD, int blocks)
{
    const SegGeom g = seg_geom(H, QD, 1, 1, blocks);   // passes at one row per pass = rows per group
    return g.passes <= 2 ? 2 : g.passes <= 4 ? 4 : 8;
}

bool seg_attn_holds_o(int H, int nq, bool w8, int blocks)
{
    const int rbo = seg_rbo(H, nq * 128, blocks) * (w8 ? 2 : 1);
    return seg_geom(H, nq * 128, 1, rbo, blocks).passes == 1;
}
bool seg_attn_holds_qkv(int H, int QR, bool w8, int blocks)
{
    return seg_geom(QR, H, H > 4096 ? 2 : 1, w8 ? 8 : 4, blocks).passes == 1;
}

template <int RBQ, int ITQ, int RBO, bool W8>
static hipError_t seg_attn_go(SegAttnArgs a, bool wait, int blocks, hipStream_t s)
{
    a.gq = seg_geom(a.QR, a.H, ITQ, RBQ, blocks);
    a.go = seg_geom(a.H, a.QD, 1, RBO, blocks);
    if (wait)
        PSV_LAUNCH((k_seg_attn<RBQ, ITQ, RBO, W8, true>), dim3(blocks), dim3(512), 0, s, a);
    else
        PSV_LAUNCH((k_seg_attn<RBQ, ITQ, RBO, W8, false>), dim3(blocks), dim3(512), 0, s, a);
    return hipGetLastError();
}

template <bool W8>
static hipError_t seg_attn_pick(const SegAttnArgs &a, bool wait, int blocks, hipStream_t s)
{
    constexpr int RQ = W8 ? 8 : 4, M = W8 ? 2 : 1;
    const int rbo = seg_rbo(a.H, a.QD, blocks);
    if (a.H > 4096) {
        if (rbo == 2) return seg_attn_go<RQ, 2, 2 * M, W8>(a, wait, blocks, s);
        if (rbo == 4) return seg_attn_go<RQ, 2, 4 * M, W8>(a, wait, blocks, s);
        return seg_attn_go<RQ, 2, 8 * M, W8>(a, wait, blocks, s);
    }
    if (rbo == 2) return seg_attn_go<RQ, 1, 2 * M, W8>(a, wait, blocks, s);
    if (rbo == 4) return seg_attn_go<RQ, 1, 4 * M, W8>(a, wait, blocks, s);
    return seg_attn_go<RQ, 1, 8 * M, W8>(a, wait, blocks, s);
}

hipError_t launch_seg_attn(Mat Wq, Mat Wo, const float *res, const float *delta, const uint16_t *gain, float eps,
                           float *out_res, float *out_h, void *qkv_ll, const float2 *rope, KvView kv, int nq, int nkv,
                           int n_chunks, void *pml, void *po, void *ind_ll, float *out_attn, float *out, int H, unsigned tag,
                           unsigned *err, const GemvWait *wait, bool hold_kv, bool hold_o, uint32_t poll_iters, int blocks, hipStream_t s)
{
    SegAttnArgs a{};
    a.Wq = Wq.w; a.Wo = Wo.w; a.sq = Wq.scale; a.so = Wo.scale;
    a.res = res; a.delta = delta; a.gain = gain; a.eps = eps; a.out_res = out_res; a.out_h = out_h;
    a.qkv_ll = static_cast<uint2 *>(qkv_ll); a.rope = rope; a.kv = kv; a.nq = nq; a.nkv = nkv; a.n_chunks = n_chunks;
    a.pml = static_cast<float2 *>(pml); a.po = static_cast<float *>(po); a.ind_ll = static_cast<uint2 *>(ind_ll);
    a.out_attn = out_attn; a.out = out;
    a.H = H; a.QR = (nq + 2 * nkv) * 128; a.QD = nq * 128; a.tag = tag; a.ll_iters = poll_iters; a.err = err;
    if (wait) a.wait = SegWait{wait->done, wait->seq, wait->iters, wait->ticks};
    a.hold_kv = hold_kv ? 1 : 0;
    a.hold_o = hold_o ? 1 : 0;
    if (nkv * n_chunks > kSegIndStride) return hipErrorInvalidValue;
    return Wq.scale ? seg_attn_pick<true>(a, wait != nullptr, blocks, s) : seg_attn_pick<false>(a, wait != nullptr, blocks, s);
}

}  // namespace psv

// gfx950 (MI355X, CDNA4) kernels of the PRESERVE decode step: the batch 1-2 projections on the vector ALU.
//
// Weights and the KV-cache are bf16 (or int8 codes with fp32 scales) in HBM; every accumulation is fp32.  The step
// is bound by HBM bandwidth (Section 2, "LLM decoding is memory BW-limited"), so the kernels are built around
// 16-byte-per-lane coalesced loads with many loads in flight per 64-lane wave; the matrix cores are used where a
// vector-ALU formulation would bind on arithmetic (batch > 2 projections, grouped-query attention).
#include "device.h"

namespace psv {

// ------------------------------------------------------------------------------------ GEMV

// Weight-streaming GEMV on the vector ALU (batch NB <= 2).
//
// A workgroup has 512 (merge mode: 256) threads, cut into groups of GS = 64..512 threads such that one 16-byte load
// per thread covers a whole weight row (K <= 8*GS; ITERS = 2 loads for K up to 8192).  A thread
// therefore always sees the same k positions, and its slice of the activations lives in registers
// for the whole kernel: no LDS staging, no re-reads.  Every group owns a contiguous, balanced
// range of output rows and streams them RB rows at a time, i.e. RB (2*RB with SwiGLU) independent
// 16-byte loads in flight per thread, issued before anything else the kernel does.  Row sums are
// finished with a 64-lane butterfly and, for GS > 64, a fixed-order sum over the group's waves
// through LDS (no atomics; bit-reproducible).
//
// MODE selects where the activations come from, always while the first weight loads are in flight:
//   GEMV_PLAIN  a vector in memory;
//   GEMV_NORM   rmsnorm(res + delta) * gain formed in the prologue; workgroup 0 also stores the new
//               residual (res + delta) and the normalised vector -- no separate normalisation launch;
//   GEMV_MERGE  the attention output, merged in the prologue from the split-K partials of the attention
//               kernel (chunk order, fixed) -- no separate merge launch; workgroup 0 stores it as well.
struct GemvArgs {
    const void *W, *W2;         // W2 != null: SwiGLU pair (gate, up); bf16, or int8 codes (template W8)
    const float *scale, *scale2;   // int8 only: per-row scales of W and W2
    const float *x;             // [NB][K] activations (plain mode)
    const float *res, *delta;   // FUSE_NORM inputs, [NB][K]; delta may be null
    const uint16_t *gain;       // FUSE_NORM: [K]
    float eps;
    float *out_res;             // FUSE_NORM: res + delta, written by workgroup 0 (must not alias res/delta)
    float *out_h;               // FUSE_NORM: normalised activations, written by workgroup 0 (may be null)
    float *out;                 // [NB][N]
    int N, K, gs_log2, passes;
    // MODE_MERGE: the activations are the attention output, merged here from the split-K partials
    const float *part_ml, *part_o;
    int nkv, G, nc;             // kv heads, query heads per kv head, chunks per (sequence, kv head)
    // Launched ahead of time (GemvWait): after requesting its first weights, every workgroup waits until
    // *wait_done has reached wait_seq -- the end of the communication window -- before it touches activations
    const unsigned *wait_done;
    unsigned wait_seq;
    uint32_t wait_iters;        // bounds of the wait: iterations of the poll loop and wall-clock ticks; a wait that
    uint64_t wait_ticks;        //   runs into them sets *wait_err and the kernel goes on (it always ends)
    unsigned *wait_err;
};

enum { GEMV_PLAIN = 0, GEMV_NORM = 1, GEMV_MERGE = 2 };

// WAIT: the variant that is launched ahead of its inputs (GemvArgs::wait_done); a kernel of its own, so that the
// ordinary one carries none of that code and the two show up separately in a kernel trace (the waiting one's
// duration includes its wait).
template <int NB, int RB, int ITERS, bool SWIGLU, int MODE, bool W8, bool WAIT>
__global__ __launch_bounds__(512) void k_gemv(GemvArgs a)
{
    constexpr int NW = SWIGLU ? 2 : 1;
    constexpr int WB = W8 ? 1 : 2;                       // bytes per weight
    using WV = typename std::conditional<W8, uint2, uint4>::type;   // 8 weights
    __shared__ float red[8][NW * RB * NB];   // [wave][value]
    __shared__ float ssq[8][NB];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int GS = 1 << a.gs_log2, groups = (int)blockDim.x >> a.gs_log2, wpg = GS >> 6;
    const int gid = tid >> a.gs_log2, lg = tid & (GS - 1), gw = wave & (wpg - 1);
    const int K = a.K, N = a.N;
    const int slots = gridDim.x * groups, slot = blockIdx.x * groups + gid;
    const int row_begin = (int)((long long)slot * N / slots), row_end = (int)((long long)(slot + 1) * N / slots);

    int kk[ITERS];
    bool kok[ITERS];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        kk[it] = (it * GS + lg) * 8;
        kok[it] = kk[it] < K;
    }

    WV wv[ITERS][NW][RB];
    const char *Wb = static_cast<const char *>(a.W), *W2b = static_cast<const char *>(a.W2);
    auto ldw = [](const char *p) {
        if constexpr (W8) return ld8(p);
        else return *reinterpret_cast<const uint4 *>(p);
    };
    // int8: the thread that will store output (row r, batch entry b) of a pass fetches that row's scale
    // together with the pass's weights
    const int my_r = lg / NB;
    float sc[NW] = {};
    // Where the activations are requested ahead of the weights (the ordinary kernel with the fused normalisation),
    // every load of a pass is issued unconditionally, in straight-line code: a row past the group's range re-reads
    // the group's last row (a cache hit; its result is never stored) and a thread past the end of a short row reads
    // column 0 and blanks what it got.  Predicated loads would sit in blocks of their own, and the compiler's wait
    // counters are conservative across such blocks: it would wait for the weights before any arithmetic on the
    // activations that were requested ahead of them.
    constexpr bool ahead = MODE == GEMV_NORM && !WAIT;     // activations are requested ahead of the weights
    auto load_rows = [&](int r0) {
        if constexpr (!ahead) {
#pragma unroll
            for (int it = 0; it < ITERS; ++it)
#pragma unroll
                for (int r = 0; r < RB; ++r) {
                    const bool ok = kok[it] && (r0 + r < row_end);
                    const size_t off = ((size_t)(r0 + r) * K + kk[it]) * WB;
                    wv[it][0][r] = ok ? ldw(Wb + off) : WV{};
                    if (SWIGLU) wv[it][NW - 1][r] = ok ? ldw(W2b + off) : WV{};
                }
            return;
        }
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int col = kok[it] ? kk[it] : 0;
#pragma unroll
            for (int r = 0; r < RB; ++r) {
                const int row = max(min(r0 + r, row_end - 1), 0);          // row_end <= N, N >= 1: always inside the matrix
                const size_t off = ((size_t)row * K + col) * WB;
                const WV w1 = ldw(Wb + off);
                wv[it][0][r] = kok[it] ? w1 : WV{};
                if (SWIGLU) {
                    const WV w2 = ldw(W2b + off);
                    wv[it][NW - 1][r] = kok[it] ? w2 : WV{};
                }
            }
        }
    };
    auto load_scales = [&](int r0) {
        if (W8 && lg < RB * NB && r0 + my_r < row_end) {
            sc[0] = a.scale[r0 + my_r];
            if (SWIGLU) sc[NW - 1] = a.scale2[r0 + my_r];
        }
    };
    // ---- order of the first requests.  Loads return in order, and the activations come from the caches (or the
    //      memory-side cache) while the weights come from HBM: requested first, the activations are back while
    //      the weights are still on their way, and the prologue (normalisation, attention merge) runs in that
    //      time instead of after it (c2 gate/up: 9.4 -> 8.9 us).  A kernel launched ahead of its inputs (WAIT)
    //      cannot do that: its activations do not exist yet; it requests the weights, waits, and only then
    //      reads them.  The other modes keep the weights first: measured no faster the other way round.
    constexpr bool late_inputs = WAIT;
    constexpr int MB = 8;                        // MERGE: chunks merged per round
    float4 xr[ITERS][NB][2], xd[ITERS][NB][2];   // NORM: residual and delta slices
    uint4 gv[ITERS];                             // NORM: gains
    float2 mt[MB];                               // MERGE: (max, sum) and two 16-byte pieces of the partial of MB chunks
    float4 mo0[MB], mo1[MB];
    if (MODE == GEMV_NORM)
#pragma unroll
        for (int it = 0; it < ITERS; ++it) gv[it] = kok[it] ? ld16(a.gain + kk[it]) : zero16();   // constants: never after a wait
    if (ahead) {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
                xr[it][b][0] = xr[it][b][1] = xd[it][b][0] = xd[it][b][1] = z;
                if (kok[it]) {
                    const float *src = a.res;
                    xr[it][b][0] = *reinterpret_cast<const float4 *>(src + (size_t)b * K + kk[it]);
                    xr[it][b][1] = *reinterpret_cast<const float4 *>(src + (size_t)b * K + kk[it] + 4);
                    if (a.delta) {
                        xd[it][b][0] = *reinterpret_cast<const float4 *>(a.delta + (size_t)b * K + kk[it]);
                        xd[it][b][1] = *reinterpret_cast<const float4 *>(a.delta + (size_t)b * K + kk[it] + 4);
                    }
                }
            }
        }
    }
    auto merge_loads = [&](int b, int it, int sp0) {   // partials of chunks sp0 .. sp0+MB-1 for this thread's slice
        const int h = kk[it] >> 7, ch0 = kk[it] & 127, kvh = h / a.G, g = h % a.G;
        const size_t slot0 = ((size_t)b * a.nkv + kvh) * a.nc;
        const float2 *ml = reinterpret_cast<const float2 *>(a.part_ml) + slot0 * 16 + g;
#pragma unroll
        for (int u = 0; u < MB; ++u) {
            const bool ok = sp0 + u < a.nc;
            const float *o = a.part_o + ((slot0 + sp0 + u) * a.G + g) * 128 + ch0;
            mt[u] = ok ? ml[(size_t)(sp0 + u) * 16] : make_float2(-1.0e30f, 0.f);
            mo0[u] = ok ? *reinterpret_cast<const float4 *>(o) : make_float4(0.f, 0.f, 0.f, 0.f);
            mo1[u] = ok ? *reinterpret_cast<const float4 *>(o + 4) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };

    int r0 = row_begin;
    load_rows(r0);
    load_scales(r0);

    // ---- launched ahead of its inputs: the weights above travel (and then sit in registers) while the
    //      communication window is still running; one wave of the workgroup polls for the window's end
    if (WAIT) {
        if (wave == 0) {
            const uint64_t t0 = wall_clock64();
            // relaxed polls (an acquire per poll would invalidate caches every time); no fence follows either: what
            // the kernel reads after the wait is fetched with device-coherent loads (ldc_issue)
            unsigned v = __hip_atomic_load(a.wait_done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            uint32_t it = 0;
            while ((int)(v - a.wait_seq) < 0 && it < a.wait_iters && wall_clock64() - t0 < a.wait_ticks) {
                __builtin_amdgcn_s_sleep(8);
                v = __hip_atomic_load(a.wait_done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ++it;
            }
            if (lane == 0 && (int)(v - a.wait_seq) < 0) atomicOr(a.wait_err, 1u);
        }
        __syncthreads();
        // The activations read below may have been written while this kernel was already running (by the
        // collective of the window), so they are fetched with device-coherent loads (ldc_issue); a fence that
        // invalidates the caches instead costs ~30 us when 4096 waves issue it.
    }

    // ---- activations into registers
    float xv[ITERS][NB][8];
    if (MODE == GEMV_NORM) {
        float ss[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            ss[b] = 0.f;
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                float4 v0 = make_float4(0.f, 0.f, 0.f, 0.f), v1 = v0;
                if (kok[it]) {
                    float4 d0 = make_float4(0.f, 0.f, 0.f, 0.f), d1 = d0;
                    if (late_inputs) {
                        const float *dp = a.delta ? a.delta : a.res;   // (a pre-launched kernel always has a delta)
                        f32x4 q0, q1, q2, q3;
                        ldc_issue(q0, a.res + (size_t)b * K + kk[it]);
                        ldc_issue(q1, a.res + (size_t)b * K + kk[it] + 4);
                        ldc_issue(q2, dp + (size_t)b * K + kk[it]);
                        ldc_issue(q3, dp + (size_t)b * K + kk[it] + 4);
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
                    if (blockIdx.x == 0 && gid == 0) {
                        *reinterpret_cast<float4 *>(a.out_res + (size_t)b * K + kk[it]) = v0;
                        *reinterpret_cast<float4 *>(a.out_res + (size_t)b * K + kk[it] + 4) = v1;
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
            for (int w2 = 0; w2 < wpg; ++w2) tot += ssq[gid * wpg + w2][b];   // fixed order
            const float inv = 1.0f / sqrtf(tot / (float)K + a.eps);
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                float *x = xv[it][b];
                if (kok[it]) {
                    const uint4 g = gv[it];
                    x[0] *= inv * bf16_lo(g.x); x[1] *= inv * bf16_hi(g.x);
                    x[2] *= inv * bf16_lo(g.y); x[3] *= inv * bf16_hi(g.y);
                    x[4] *= inv * bf16_lo(g.z); x[5] *= inv * bf16_hi(g.z);
                    x[6] *= inv * bf16_lo(g.w); x[7] *= inv * bf16_hi(g.w);
                    if (a.out_h && blockIdx.x == 0 && gid == 0) {
                        *reinterpret_cast<float4 *>(a.out_h + (size_t)b * K + kk[it]) = make_float4(x[0], x[1], x[2], x[3]);
                        *reinterpret_cast<float4 *>(a.out_h + (size_t)b * K + kk[it] + 4) = make_float4(x[4], x[5], x[6], x[7]);
                    }
                }
            }
        }
    } else if (MODE == GEMV_MERGE) {
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                float *x = xv[it][b];
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] = 0.f;
                if (kok[it]) {
                    // One pass with a running maximum; loads are issued MB chunks at a time so that their
                    // latencies overlap.  Chunk order is fixed, so the result is reproducible.  (Requesting the
                    // first round ahead of the weights, 16 chunks at a time, was slower for short chunk lists.)
                    float Mx = -1.0e30f, den = 0.f;
                    for (int sp0 = 0; sp0 < a.nc; sp0 += MB) {
                        merge_loads(b, it, sp0);
                        float bm = Mx;
#pragma unroll
                        for (int u = 0; u < MB; ++u) bm = fmaxf(bm, mt[u].x);
                        const float rs = exp2f(Mx - bm);
                        Mx = bm;
                        den *= rs;
#pragma unroll
                        for (int e = 0; e < 8; ++e) x[e] *= rs;
#pragma unroll
                        for (int u = 0; u < MB; ++u) {
                            const float wgt = mt[u].y > 0.f ? exp2f(mt[u].x - Mx) : 0.f;
                            den += wgt * mt[u].y;
                            x[0] = fmaf(wgt, mo0[u].x, x[0]); x[1] = fmaf(wgt, mo0[u].y, x[1]);
                            x[2] = fmaf(wgt, mo0[u].z, x[2]); x[3] = fmaf(wgt, mo0[u].w, x[3]);
                            x[4] = fmaf(wgt, mo1[u].x, x[4]); x[5] = fmaf(wgt, mo1[u].y, x[5]);
                            x[6] = fmaf(wgt, mo1[u].z, x[6]); x[7] = fmaf(wgt, mo1[u].w, x[7]);
                        }
                    }
                    const float inv = den > 0.f ? 1.0f / den : 0.f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) x[e] *= inv;
                    if (a.out_h && blockIdx.x == 0 && gid == 0) {
                        *reinterpret_cast<float4 *>(a.out_h + (size_t)b * K + kk[it]) = make_float4(x[0], x[1], x[2], x[3]);
                        *reinterpret_cast<float4 *>(a.out_h + (size_t)b * K + kk[it] + 4) = make_float4(x[4], x[5], x[6], x[7]);
                    }
                }
            }
    } else {
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                float4 v0 = make_float4(0.f, 0.f, 0.f, 0.f), v1 = v0;
                if (kok[it]) {
                    v0 = *reinterpret_cast<const float4 *>(a.x + (size_t)b * K + kk[it]);
                    v1 = *reinterpret_cast<const float4 *>(a.x + (size_t)b * K + kk[it] + 4);
                }
                float *x = xv[it][b];
                x[0] = v0.x; x[1] = v0.y; x[2] = v0.z; x[3] = v0.w;
                x[4] = v1.x; x[5] = v1.y; x[6] = v1.z; x[7] = v1.w;
            }
    }

    // ---- stream the rows.  `passes` is the same for every group of the launch, so the barriers match.
    for (int pass = 0; pass < a.passes; ++pass) {
        float acc[NW][RB][NB];
#pragma unroll
        for (int q = 0; q < NW; ++q)
#pragma unroll
            for (int r = 0; r < RB; ++r)
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    float s = 0.f;
#pragma unroll
                    for (int it = 0; it < ITERS; ++it) s = dot8(wv[it][q][r], xv[it][b], s);
                    acc[q][r][b] = s;
                }
        // all sums of the pass over the wave at once, in chunks of up to 16 values: lane l < CS holds, of chunk c, the
        // value of index c * CS + scatter_index<CS>(l), index = (q * RB + r) * NB + b
        constexpr int NT = NW * RB * NB, CS = NT < 16 ? NT : 16, NC = NT / CS, HALF = RB * NB;
        float tot[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) tot[c] = wave_sum_scatter<CS>(reinterpret_cast<const float (&)[CS]>((&acc[0][0][0])[c * CS]), lane);
        const int li = scatter_index<CS>(lane);
        const int rows_here = r0;
        r0 += RB;
        float sc_now[NW];
#pragma unroll
        for (int q = 0; q < NW; ++q) sc_now[q] = sc[q];
        if (pass + 1 < a.passes) {   // next pass's loads fly during the reduction below
            load_rows(r0);
            load_scales(r0);
        }

        if (wpg == 1) {
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                if (c * CS >= HALF) continue;               // the chunks of the first (or only) matrix
                const int i = c * CS + li, r = i / NB, b = i % NB;
                float v = tot[c], u = 0.f;
                if constexpr (SWIGLU) {                    // the second matrix's sum of the same row: HALF indices further on
                    if constexpr (HALF >= CS) u = tot[c + HALF / CS];
                    else u = __int_as_float(__builtin_amdgcn_ds_bpermute(scatter_holder((li + HALF) & (CS - 1)) << 2, __float_as_int(tot[c])));
                }
                if (lane < CS && i < HALF && rows_here + r < row_end) {
                    if (W8) {   // one wave per row group: a rare shape, the scale is fetched late
                        v *= a.scale[rows_here + r];
                        if (SWIGLU) u *= a.scale2[rows_here + r];
                    }
                    if (SWIGLU) v = silu_mul(v, u);
                    a.out[(size_t)b * N + rows_here + r] = v;
                }
            }
        } else {
            if (lane < CS)
#pragma unroll
                for (int c = 0; c < NC; ++c) red[wave][c * CS + li] = tot[c];
            __syncthreads();
            if (lg < RB * NB) {
                const int r = lg / NB, b = lg % NB;
                if (rows_here + r < row_end) {
                    float v = 0.f, u = 0.f;
                    for (int w2 = 0; w2 < wpg; ++w2) {   // fixed order
                        v += red[gid * wpg + w2][r * NB + b];
                        if (SWIGLU) u += red[gid * wpg + w2][(RB + r) * NB + b];
                    }
                    if (W8) {
                        v *= sc_now[0];
                        if (SWIGLU) u *= sc_now[NW - 1];
                    }
                    if (SWIGLU) v = silu_mul(v, u);
                    a.out[(size_t)b * N + rows_here + r] = v;
                }
            }
            __syncthreads();
        }
    }
    (void)gw;
}

bool gemv_supported(int batch, int N, int K)
{
    return batch >= 1 && batch <= 2 && K % 8 == 0 && K >= 64 && K <= 8192 && N >= 1;
}

// Workgroup size: 512 threads, except for the merge mode, whose prologue is repeated by every group of
// threads that covers a row: 256 threads measured 1 us faster there.
static constexpr int gemv_threads(int mode) { return mode == GEMV_MERGE ? 256 : 512; }

// Launch geometry shared by every instantiation: group size (threads that cover one row), workgroups, and
// the most rows any group owns.
struct GemvGeom {
    int gs_log2, groups, max_rows;
    long long blocks;
};
static GemvGeom gemv_geom(int N, int K, int iters, int threads, int rb)
{
    GemvGeom g;
    g.gs_log2 = 6;
    while ((8 << g.gs_log2) * iters < K && (1 << g.gs_log2) < threads) ++g.gs_log2;
    g.groups = threads >> g.gs_log2;
    // enough workgroups that a group gets at most rb rows per pass and the grid is a multiple of the
    // 256 CUs (2 workgroups fit on a CU); rows are dealt to the groups in balanced contiguous ranges.
    const long long want = ((long long)N + (long long)rb * g.groups - 1) / ((long long)rb * g.groups);
    g.blocks = (want + 255) / 256 * 256;
    if (g.blocks < 256) g.blocks = 256;
    if (g.blocks > 1024) g.blocks = 1024;
    const long long slots = g.blocks * g.groups;
    g.max_rows = (int)((N + slots - 1) / slots);
    return g;
}

template <int NB, int RB, int ITERS, bool SW, int MODE, bool W8>
static hipError_t gemv_go(GemvArgs a, hipStream_t s)
{
    const int threads = gemv_threads(MODE);
    const GemvGeom g = gemv_geom(a.N, a.K, ITERS, threads, RB);
    a.gs_log2 = g.gs_log2;
    a.passes = (g.max_rows + RB - 1) / RB;
    if (a.passes < 1) a.passes = 1;
    if (a.wait_done) {
        if constexpr (MODE == GEMV_NORM) {
            PSV_LAUNCH((k_gemv<NB, RB, ITERS, SW, MODE, W8, true>), dim3((unsigned)g.blocks), dim3(threads), 0, s, a);
            return hipGetLastError();
        } else {
            return hipErrorInvalidValue;     // only the kernels that open a block (fused add + norm) are launched ahead
        }
    }
    PSV_LAUNCH((k_gemv<NB, RB, ITERS, SW, MODE, W8, false>), dim3((unsigned)g.blocks), dim3(threads), 0, s, a);
    return hipGetLastError();
}

// Rows per pass: as many as keep 128 bytes (x ITERS) of weight loads in flight per thread (8 rows of bf16, 16
// of int8; half of that for a SwiGLU pair) -- but no more than a group owns when the matrix is small and the
// minimum grid of 256 workgroups already leaves only a few rows per group, since padded rows cost ALU work.
template <int NB, int ITERS, bool SW, int MODE, bool W8>
static hipError_t gemv_rows(const GemvArgs &a, hipStream_t s)
{
    // A kernel that is launched ahead of its inputs holds the first pass in registers while it waits, so there a
    // SwiGLU pair takes the full 8 (16) rows where the registers allow it; launched the ordinary way the second
    // pass of 4 rows is as fast (c2 gate/up: 7 rows per group, 9.4 us in two passes, 9.7 us in one).
    constexpr int RBMAX = (SW ? (ITERS == 1 && NB == 1 ? 8 : 4) : 8) * (W8 ? 2 : 1);
    const int threads = gemv_threads(MODE);
    int rb = a.wait_done ? RBMAX : (SW ? 4 : 8) * (W8 ? 2 : 1);
    while (rb > 4 && gemv_geom(a.N, a.K, ITERS, threads, rb).max_rows <= rb / 2) rb /= 2;
    if constexpr (RBMAX >= 16) if (rb == 16) return gemv_go<NB, 16, ITERS, SW, MODE, W8>(a, s);
    if constexpr (RBMAX >= 8) if (rb == 8) return gemv_go<NB, 8, ITERS, SW, MODE, W8>(a, s);
    return gemv_go<NB, 4, ITERS, SW, MODE, W8>(a, s);
}

template <int NB, int MODE>
static hipError_t gemv_pick(const GemvArgs &a, hipStream_t s)
{
    const int threads = gemv_threads(MODE);
    const bool sw = a.W2 != nullptr, two = a.K > 8 * threads;
    if (MODE == GEMV_MERGE && sw) return hipErrorInvalidValue;   // the merge prologue feeds the O projection only
    if (a.scale) {
        if (two) return sw ? gemv_rows<NB, 2, MODE != GEMV_MERGE, MODE, true>(a, s) : gemv_rows<NB, 2, false, MODE, true>(a, s);
        return sw ? gemv_rows<NB, 1, MODE != GEMV_MERGE, MODE, true>(a, s) : gemv_rows<NB, 1, false, MODE, true>(a, s);
    }
    if (two) return sw ? gemv_rows<NB, 2, MODE != GEMV_MERGE, MODE, false>(a, s) : gemv_rows<NB, 2, false, MODE, false>(a, s);
    return sw ? gemv_rows<NB, 1, MODE != GEMV_MERGE, MODE, false>(a, s) : gemv_rows<NB, 1, false, MODE, false>(a, s);
}

template <int MODE>
static hipError_t gemv_dispatch(const GemvArgs &a, int batch, hipStream_t s)
{
    switch (batch) {
    case 1: return gemv_pick<1, MODE>(a, s);
    case 2: return gemv_pick<2, MODE>(a, s);
    default: return hipErrorInvalidValue;   // larger batches run on the matrix cores
    }
}

hipError_t launch_gemv(Mat W, Mat W2, const float *x, float *out, int batch, int N, int K, hipStream_t s)
{
    GemvArgs a{};
    a.W = W.w; a.W2 = W2.w; a.scale = W.scale; a.scale2 = W2.scale; a.x = x; a.out = out; a.N = N; a.K = K;
    return gemv_dispatch<GEMV_PLAIN>(a, batch, s);
}

hipError_t launch_gemv_norm(Mat W, Mat W2, const float *res, const float *delta,
                            const uint16_t *gain, float eps, float *out_res, float *out_h, float *out, int batch,
                            int N, int K, const GemvWait *wait, hipStream_t s)
{
    GemvArgs a{};
    if (wait) {
        a.wait_done = wait->done; a.wait_seq = wait->seq; a.wait_iters = wait->iters; a.wait_ticks = wait->ticks;
        a.wait_err = wait->err;
    }
    a.W = W.w; a.W2 = W2.w; a.scale = W.scale; a.scale2 = W2.scale; a.res = res; a.delta = delta; a.gain = gain; a.eps = eps; a.out_res = out_res; a.out_h = out_h;
    a.out = out; a.N = N; a.K = K;
    return gemv_dispatch<GEMV_NORM>(a, batch, s);
}

bool gemv_merge_supported(int batch, int nq, int n_chunks)
{
    return batch >= 1 && batch <= 2 && nq * 128 <= 4096 && n_chunks <= kGemvMergeMaxChunks;
}

hipError_t launch_gemv_merge(Mat W, const float *part_ml, const float *part_o, int nq, int nkv,
                             int n_chunks, float *out_attn, float *out, int batch, int N, hipStream_t s)
{
    GemvArgs a{};
    a.W = W.w; a.scale = W.scale; a.part_ml = part_ml; a.part_o = part_o; a.nkv = nkv; a.G = nq / nkv; a.nc = n_chunks; a.out_h = out_attn;
    a.out = out; a.N = N; a.K = nq * 128;
    return gemv_dispatch<GEMV_MERGE>(a, batch, s);
}

}  // namespace psv

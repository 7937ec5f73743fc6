// gfx950 (MI355X, CDNA4) kernels of the PRESERVE decode step.
//
// All weights and the KV-cache are bf16 in HBM; every accumulation is fp32.  The step is bound
// by HBM bandwidth (Section 2, "LLM decoding is memory BW-limited"), so the kernels are built
// around 16-byte-per-lane coalesced loads with many loads in flight per 64-lane wave; matrix
// cores (16x16x32 bf16 MFMA) are used where a vector-ALU formulation would bind on arithmetic
// (batch > 4 projections, grouped-query attention).
#include <hip/hip_ext.h>
#include <stdlib.h>

#include <type_traits>

#include "internal.h"

namespace psv {

// Optional events that the next kernel launch attaches to its own dispatch: `stop` is bound to the kernel
// command and carries its end timestamp; `start` is a marker ahead of it.  Used by the per-operator
// profiling of the API layer.
static thread_local hipEvent_t g_ev_start = nullptr, g_ev_stop = nullptr;
void set_launch_events(hipEvent_t start, hipEvent_t stop)
{
    g_ev_start = start;
    g_ev_stop = stop;
}

#define PSV_LAUNCH(kernel, grid, block, shmem, stream, ...)                                                      \
    do {                                                                                                         \
        if (g_ev_start || g_ev_stop) {                                                                           \
            hipExtLaunchKernelGGL(kernel, grid, block, shmem, stream, g_ev_start, g_ev_stop, 0, __VA_ARGS__);    \
            g_ev_start = g_ev_stop = nullptr;                                                                    \
        } else {                                                                                                 \
            hipLaunchKernelGGL(kernel, grid, block, shmem, stream, __VA_ARGS__);                                 \
        }                                                                                                        \
    } while (0)

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef int i32x4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------------------------ helpers

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ uint32_t f32_to_bf16(float f)   // round to nearest even
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    return f32_to_bf16(lo) | (f32_to_bf16(hi) << 16);
}

// Activations that feed the matrix cores are carried as two bf16 planes, x = hi + lo (+ a remainder below
// 2^-17 |x|): one MFMA per plane restores fp32-grade accuracy at negligible cost, since the matrix cores
// idle most of the time in a bandwidth-bound GEMM.  lo plane = hi plane + plane_stride elements.
__device__ __forceinline__ void split_bf16(float v, uint32_t &hi, uint32_t &lo)
{
    hi = f32_to_bf16(v);
    lo = f32_to_bf16(v - __uint_as_float(hi << 16));
}

// Sum over the 64 lanes of a wave, returned in every lane.  Four DPP steps (quad swaps, half-row and row
// mirrors: VALU only, no LDS crossbar traffic) leave the sum of each 16-lane row in all of its lanes; the
// four row sums are then read through scalar registers.  Must be called with all lanes active.  A
// ds_bpermute butterfly does the same in six LDS-pipe round trips per value, which cost ~2 us per GEMV.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v)
{
    const int t = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true);
    return v + __int_as_float(t);
}
__device__ __forceinline__ float wave_sum(float v)
{
    v = dpp_add<0xB1>(v);    // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);    // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);   // row_half_mirror
    v = dpp_add<0x140>(v);   // row_mirror
    const int iv = __float_as_int(v);
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(iv, 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(iv, 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(iv, 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(iv, 48));
    return (r0 + r1) + (r2 + r3);
}

// low bytes of four floats that hold small integers in "magic number" form (x + 1.5 * 2^23)
__device__ __forceinline__ uint32_t pack_magic_bytes(float a0, float a1, float a2, float a3)
{
    const uint32_t lo = __builtin_amdgcn_perm(__float_as_uint(a1), __float_as_uint(a0), 0x0c0c0400u);   // a0.b0 | a1.b0 << 8
    const uint32_t hi = __builtin_amdgcn_perm(__float_as_uint(a3), __float_as_uint(a2), 0x04000c0cu);   // a2.b0 << 16 | a3.b0 << 24
    return lo | hi;
}

// Two int8 digits of t (|t| <= 127.5): d1 = rint(t), d2 = rint(254 * (t - d1)); both returned in magic form.
__device__ __forceinline__ void two_digits(float t, float &m1, float &m2)
{
    const float kMagic = 12582912.0f;   // 1.5 * 2^23: adding it rounds to an integer (ties to even)
    m1 = t + kMagic;
    const float r = t - (m1 - kMagic);
    m2 = fmaf(r, 254.0f, kMagic);
}

// Maximum over aligned groups of 32 lanes, returned in every lane of the group (all lanes must be active).
template <int CTRL>
__device__ __forceinline__ float dpp_max(float v)
{
    const int t = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true);
    return fmaxf(v, __int_as_float(t));
}
__device__ __forceinline__ float max32(float v)
{
    v = dpp_max<0xB1>(v);    // quad_perm [1,0,3,2]
    v = dpp_max<0x4E>(v);    // quad_perm [2,3,0,1]
    v = dpp_max<0x141>(v);   // row_half_mirror
    v = dpp_max<0x140>(v);   // row_mirror: every lane holds the maximum of its row of 16
    return fmaxf(v, __shfl_xor(v, 16, 64));
}

// Operand format of the int8 matrix-core projections ("digit planes"): an activation row is cut into blocks of
// 128 consecutive elements; every element is stored as two int8 digits, x ~ s * (d1 + d2 / 254) with s = (largest
// magnitude of the block) / 127, which keeps 15-16 bits of the block's largest element.  Plane d1 is [rows][K]
// bytes at `base`, plane d2 follows `plane` bytes later, the block scales [rows][K / 128] fp32 after both.
// Called by the 32 consecutive lanes that hold one block, four elements each (k0 = first of the lane's four).
__device__ __forceinline__ void store_digits4(uint8_t *base, size_t plane, int K, size_t row, int k0, float4 v)
{
    const float amax = max32(fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
    const float inv = amax > 0.f ? 127.0f / amax : 0.f;
    float a1[4], a2[4];
    two_digits(v.x * inv, a1[0], a2[0]);
    two_digits(v.y * inv, a1[1], a2[1]);
    two_digits(v.z * inv, a1[2], a2[2]);
    two_digits(v.w * inv, a1[3], a2[3]);
    uint8_t *p = base + row * K + k0;
    *reinterpret_cast<uint32_t *>(p) = pack_magic_bytes(a1[0], a1[1], a1[2], a1[3]);
    *reinterpret_cast<uint32_t *>(p + plane) = pack_magic_bytes(a2[0], a2[1], a2[2], a2[3]);
    if ((threadIdx.x & 31) == 0)
        reinterpret_cast<float *>(base + 2 * plane)[row * (K / 128) + k0 / 128] = amax / 127.0f;
}

// Maximum over the 64 lanes of a wave, returned in every lane (all lanes must be active).
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// int8 code of v under `scale`: round to nearest (ties to even), clamp to [-127, 127]
__device__ __forceinline__ uint8_t quant_i8(float v, float scale)
{
    float q = rintf(v / scale);
    q = fminf(fmaxf(q, -127.0f), 127.0f);
    return (uint8_t)(int8_t)(int)q;
}

__device__ __forceinline__ uint4 ld16(const uint16_t *p) { return *reinterpret_cast<const uint4 *>(p); }
__device__ __forceinline__ uint4 zero16() { return make_uint4(0u, 0u, 0u, 0u); }

__device__ __forceinline__ uint2 ld8(const void *p) { return *reinterpret_cast<const uint2 *>(p); }

// int8 code j (0..3) of a 32-bit word as a float
template <int J>
__device__ __forceinline__ float i8f(uint32_t w) { return (float)((int32_t)(w << (24 - 8 * J)) >> 24); }

// dot of 8 int8 weights (one 8-byte word) with 8 fp32 activations
__device__ __forceinline__ float dot8(uint2 w, const float (&x)[8], float acc)
{
    acc = fmaf(i8f<0>(w.x), x[0], acc);
    acc = fmaf(i8f<1>(w.x), x[1], acc);
    acc = fmaf(i8f<2>(w.x), x[2], acc);
    acc = fmaf(i8f<3>(w.x), x[3], acc);
    acc = fmaf(i8f<0>(w.y), x[4], acc);
    acc = fmaf(i8f<1>(w.y), x[5], acc);
    acc = fmaf(i8f<2>(w.y), x[6], acc);
    acc = fmaf(i8f<3>(w.y), x[7], acc);
    return acc;
}

// dot of 8 bf16 weights (one 16-byte word) with 8 fp32 activations
__device__ __forceinline__ float dot8(uint4 w, const float (&x)[8], float acc)
{
    acc = fmaf(bf16_lo(w.x), x[0], acc);
    acc = fmaf(bf16_hi(w.x), x[1], acc);
    acc = fmaf(bf16_lo(w.y), x[2], acc);
    acc = fmaf(bf16_hi(w.y), x[3], acc);
    acc = fmaf(bf16_lo(w.z), x[4], acc);
    acc = fmaf(bf16_hi(w.z), x[5], acc);
    acc = fmaf(bf16_lo(w.w), x[6], acc);
    acc = fmaf(bf16_hi(w.w), x[7], acc);
    return acc;
}

// Device-coherent 16-byte loads (sc0 sc1: served by the memory side, past the caches that are not kept coherent
// while a kernel runs), for data that another kernel may have written after this one started.  The compiler does
// not count the loads of an asm statement, so ldc_issue only requests and ldc_wait -- which names the destination
// registers as operands, so that no use can be scheduled above it -- waits for everything outstanding.
__device__ __forceinline__ void ldc_issue(f32x4 &v, const float *p)
{
    asm volatile("global_load_dwordx4 %0, %1, off sc0 sc1" : "=v"(v) : "v"(p) : "memory");
}
__device__ __forceinline__ void ldc_wait(f32x4 &a, f32x4 &b, f32x4 &c, f32x4 &d)
{
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : : "memory");
}

__device__ __forceinline__ float silu_mul(float g, float u) { return g / (1.0f + expf(-g)) * u; }

// ------------------------------------------------------------------------------------ norm

// Residual add for the matrix-core path, spread over many workgroups: grid (H / 512, batch), one float4 per
// thread.  out_res = res + delta, where delta may be `delta_splits` split-K partials [split][batch][H] that are
// summed in split order.  With a gain, the kernel also prepares the next projection's operand without ever seeing
// a whole row: it stores out_res * gain as hi/lo bf16 planes and the sum of squares of its 512 outputs in
// ssq[batch][H / 512].  RMSNorm is linear in its 1/rms factor, so that projection runs on the unnormalised planes
// and multiplies its result by 1/rms of the batch row, which it forms from ssq (k_gemm_sk).
__global__ __launch_bounds__(128) void k_resid_sum(const float *__restrict__ res, const float *__restrict__ delta,
                                                   int delta_splits, size_t delta_stride, int H,
                                                   float *__restrict__ out_res, const uint16_t *__restrict__ gain,
                                                   uint16_t *__restrict__ xg_bf16, size_t plane_stride,
                                                   int digits, float *__restrict__ ssq)
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
        float4 t[kSkMaxSplits];   // all loads first (their latencies overlap), then the sum in split order
#pragma unroll
        for (int ks = 0; ks < kSkMaxSplits; ++ks)
            t[ks] = ks < delta_splits ? *reinterpret_cast<const float4 *>(d + ks * delta_stride)
                                      : make_float4(0.f, 0.f, 0.f, 0.f);
        float4 e = t[0];
#pragma unroll
        for (int ks = 1; ks < kSkMaxSplits; ++ks) { e.x += t[ks].x; e.y += t[ks].y; e.z += t[ks].z; e.w += t[ks].w; }
        v.x += e.x; v.y += e.y; v.z += e.z; v.w += e.w;
    }
    *reinterpret_cast<float4 *>(out_res + at) = v;
    if (!gain) return;
    const float4 xg = make_float4(v.x * bf16_lo(g.x), v.y * bf16_hi(g.x), v.z * bf16_lo(g.y), v.w * bf16_hi(g.y));
    if (digits) {   // operand of an int8 projection
        store_digits4(reinterpret_cast<uint8_t *>(xg_bf16), plane_stride, H, (size_t)b, i, xg);
    } else {
        uint32_t h0, h1, h2, h3, l0, l1, l2, l3;
        split_bf16(xg.x, h0, l0); split_bf16(xg.y, h1, l1); split_bf16(xg.z, h2, l2); split_bf16(xg.w, h3, l3);
        *reinterpret_cast<uint2 *>(xg_bf16 + at) = make_uint2(h0 | (h1 << 16), h2 | (h3 << 16));
        *reinterpret_cast<uint2 *>(xg_bf16 + plane_stride + at) = make_uint2(l0 | (l1 << 16), l2 | (l3 << 16));
    }
    const float ss = wave_sum(v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    if (tid == 0) ssq[(size_t)b * gridDim.x + blockIdx.x] = red[0] + red[1];
}

hipError_t launch_resid_sum(const float *res, const float *delta, int delta_splits, int batch, int H, float *out_res,
                            const uint16_t *gain, uint16_t *xg_bf16, size_t plane_stride, bool digits, float *ssq,
                            hipStream_t s)
{
    PSV_LAUNCH(k_resid_sum, dim3(H / 512, batch), dim3(128), 0, s, res, delta, delta_splits, (size_t)batch * H, H,
               out_res, gain, xg_bf16, plane_stride, digits ? 1 : 0, ssq);
    return hipGetLastError();
}

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
    if (ahead) {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            gv[it] = kok[it] ? ld16(a.gain + kk[it]) : zero16();
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
        __shared__ unsigned wait_ok;
        if (wave == 0) {
            const uint64_t t0 = wall_clock64();
            // relaxed polls (an acquire per poll would invalidate caches every time); one acquire fence follows
            unsigned v = __hip_atomic_load(a.wait_done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            uint32_t it = 0;
            while ((int)(v - a.wait_seq) < 0 && it < a.wait_iters && wall_clock64() - t0 < a.wait_ticks) {
                __builtin_amdgcn_s_sleep(8);
                v = __hip_atomic_load(a.wait_done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ++it;
            }
            if (lane == 0) {
                wait_ok = (int)(v - a.wait_seq) >= 0 ? 1u : 0u;
                if (!wait_ok) atomicOr(a.wait_err, 1u);
            }
        }
        __syncthreads();
        // The activations read below may have been written while this kernel was already running (by the
        // collective of the window), so they are fetched with device-coherent loads (ldc_issue); a fence that
        // invalidates the caches instead costs ~30 us when 4096 waves issue it.
    }

    // ---- activations into registers
    float xv[ITERS][NB][8];
    if (MODE == GEMV_NORM) {
        if (WAIT)
#pragma unroll
            for (int it = 0; it < ITERS; ++it) gv[it] = kok[it] ? ld16(a.gain + kk[it]) : zero16();
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
                    acc[q][r][b] = wave_sum(s);
                }
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
            if (lane == 0)
#pragma unroll
                for (int r = 0; r < RB; ++r)
                    if (rows_here + r < row_end)
#pragma unroll
                        for (int b = 0; b < NB; ++b) {
                            float v = acc[0][r][b], u = SWIGLU ? acc[NW - 1][r][b] : 0.f;
                            if (W8) {   // one wave per row group: a rare shape, the scale is fetched late
                                v *= a.scale[rows_here + r];
                                if (SWIGLU) u *= a.scale2[rows_here + r];
                            }
                            if (SWIGLU) v = silu_mul(v, u);
                            a.out[(size_t)b * N + rows_here + r] = v;
                        }
        } else {
            if (lane == 0)
#pragma unroll
                for (int q = 0; q < NW; ++q)
#pragma unroll
                    for (int r = 0; r < RB; ++r)
#pragma unroll
                        for (int b = 0; b < NB; ++b) red[wave][(q * RB + r) * NB + b] = acc[q][r][b];
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

// ------------------------------------------------------------------------------------ split-K skinny GEMM

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
};

template <int NB>
__global__ __launch_bounds__(256) void k_gemm_sk(GemmSkArgs a)
{
    constexpr int PF = 4;   // slabs of weight fragments in flight per wave (8 measured slower: fewer straight-line rounds, more registers)
    __shared__ uint4 xs[2][NB * 4][64];   // [buffer][(batch tile*2 + plane)*2 + k half][lane]
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, i = lane & 15, g = lane >> 4;
    const int row_base = blockIdx.x * 128 + w * 32;
    const int s0 = blockIdx.y * a.slabs_per_block, s1 = min(s0 + a.slabs_per_block, a.n_slabs);
    const int K = a.K;

    // Lane (i, g) owns elements g*16 .. g*16+15 of row i of every 64-element slab: 32 contiguous bytes = two fragments.
    const uint16_t *wp[2];
    bool wok[2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        const int r = row_base + mt * 16 + i;
        wok[mt] = r < a.N;
        const int rr = wok[mt] ? r : 0;
        wp[mt] = (rr < a.split_row ? a.W + (size_t)rr * K : a.W2 + (size_t)(rr - a.split_row) * K) + g * 16;
    }
    struct WFrag { uint4 a0[2], a1[2]; };
    auto load_w = [&](int s, WFrag &f) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            f.a0[mt] = wok[mt] ? ld16(wp[mt] + (size_t)s * 64) : zero16();
            f.a1[mt] = wok[mt] ? ld16(wp[mt] + (size_t)s * 64 + 8) : zero16();
        }
    };
    auto load_w_all = [&](int s, WFrag &f) {   // unpredicated: a row past N reads row 0 (wp) and is never stored
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            f.a0[mt] = ld16(wp[mt] + (size_t)s * 64);
            f.a1[mt] = ld16(wp[mt] + (size_t)s * 64 + 8);
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
            xs[buf][(n * 2 + p) * 2 + (seg & 1)][(seg >> 1) * 16 + row] = r[j];   // fragment order: k = g*16 + half*8 + e
        }
    };

    f32x4 acc[2][NB];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int n = 0; n < NB; ++n) acc[mt][n] = f32x4{0.f, 0.f, 0.f, 0.f};
    __shared__ float inv_s[NB * 16];

    WFrag wq[PF];
#pragma unroll
    for (int q = 0; q < PF; ++q)
        if (s0 + q < s1) load_w(s0 + q, wq[q]);
    uint4 xr[2][NB];
    if (s0 < s1) {
        load_slab(s0, xr[0]);
        if (s0 + 1 < s1) load_slab(s0 + 1, xr[1]);
        store_slab(0, xr[0]);
    }
    // 1/rms of every batch row from the partial sums of squares (block order); read in the epilogue only, the
    // barriers of the main loop make it visible
    if (tid < NB * 16) {
        float inv = 1.0f;
        if (a.ssq) {
            float tot = 0.f;
            const int nblk = K / 512;                       // <= 32
            if (tid < a.batch) {
                const float *p = a.ssq + (size_t)tid * nblk;
                if ((nblk & 3) == 0) {                      // all loads at once, then the sum in block order
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
    for (; sb + 2 * PF <= s1; sb += PF) {
#pragma unroll
        for (int q = 0; q < PF; ++q) {
            const int s = sb + q, buf = q & 1;      // (s - s0) & 1, because PF is even
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
};

template <int NB>
__global__ __launch_bounds__(256) void k_gemm_sk_i8(GemmI8Args a)
{
    constexpr int PF = 8;                          // slabs of weight codes in flight per wave (2 x 16 bytes each)
    __shared__ uint4 xs[2][NB * 2][64];            // [buffer][batch tile * 2 + digit][lane]
    __shared__ float bs[2][NB * 16];               // block scale of each batch row for the buffered slab
    __shared__ float inv_s[NB * 16];
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, i = lane & 15, g = lane >> 4;
    const int row_base = blockIdx.x * 128 + w * 32;
    const int s0 = blockIdx.y * a.slabs_per_block, s1 = min(s0 + a.slabs_per_block, a.n_slabs);
    const int K = a.K;
    const float *bscale = reinterpret_cast<const float *>(a.xd + 2 * a.x_plane);
    const int nblk128 = K / 128;

    const int8_t *wp[2];
    bool wok[2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        const int r = row_base + mt * 16 + i;
        wok[mt] = r < a.N;
        const int rr = wok[mt] ? r : 0;
        wp[mt] = (rr < a.split_row ? a.W + (size_t)rr * K : a.W2 + (size_t)(rr - a.split_row) * K) + g * 16;
    }
    // Lane (i, g) owns bytes g*16 .. g*16+15 of row i of every 64-element slab: the A operand of one MFMA.
    struct WFrag { uint4 c[2]; };
    auto load_w = [&](int s, WFrag &f) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
            f.c[mt] = wok[mt] ? *reinterpret_cast<const uint4 *>(wp[mt] + (size_t)s * 64) : zero16();
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
        sr.sc = tid < NB * 16 ? bscale[(size_t)tid * nblk128 + (s >> 1)] : 0.f;
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

    WFrag wq[PF];
#pragma unroll
    for (int q = 0; q < PF; ++q)
        if (s0 + q < s1) load_w(s0 + q, wq[q]);
    SlabRegs xr[2];
    if (s0 < s1) {
        load_slab(s0, xr[0]);
        if (s0 + 1 < s1) load_slab(s0 + 1, xr[1]);
        store_slab(0, xr[0]);
    }
    if (tid < NB * 16) {   // 1/rms of every batch row (see k_gemm_sk)
        float inv = 1.0f;
        if (a.ssq) {
            float tot = 0.f;
            const int nblk = K / 512;
            if (tid < a.batch) {
                const float *p = a.ssq + (size_t)tid * nblk;
                if ((nblk & 3) == 0) {
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
    __syncthreads();

    for (int sb = s0; sb < s1; sb += PF) {
#pragma unroll
        for (int q = 0; q < PF; ++q) {
            const int s = sb + q;
            if (s < s1) {                       // uniform over the workgroup
                const int buf = q & 1;          // (s - s0) & 1, because PF is even
                if (s + 2 < s1) load_slab(s + 2, xr[q & 1]);
                const bool fold = (s & 1) || s + 1 == s1;   // end of a 128-element block, or of this workgroup's range
#pragma unroll
                for (int n = 0; n < NB; ++n) {
                    const i32x4 x1 = __builtin_bit_cast(i32x4, xs[buf][n * 2 + 0][lane]);
                    const i32x4 x2 = __builtin_bit_cast(i32x4, xs[buf][n * 2 + 1][lane]);
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt) {
                        const i32x4 wc = __builtin_bit_cast(i32x4, wq[q].c[mt]);
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
                if (s + PF < s1) load_w(s + PF, wq[q]);
                if (s + 1 < s1) store_slab(buf ^ 1, xr[(q + 1) & 1]);
                __syncthreads();
            }
        }
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
int gemm_sk_splits(int batch, int N, int K, bool w8)
{
    const int n_slabs = K / 64;
    const double row_groups = (double)((N + 127) / 128);
    const double w_bytes = (w8 ? 1.0 : 2.0) * N * K, part_bytes = 8.0 * batch * N;
    int best = 1;
    double best_cost = 1e30;
    for (int ks = 1; ks <= kSkMaxSplits && ks * 2 <= n_slabs; ++ks) {
        const int spb = (n_slabs + ks - 1) / ks;
        const int real = (n_slabs + spb - 1) / spb;
        if (real != ks) continue;
        const double rounds = (double)(long long)((row_groups * ks + 511) / 512);
        const double cost = rounds * spb * 0.6 + (w_bytes + ks * part_bytes) / 4.0e6;
        if (cost < best_cost - 1e-9) { best_cost = cost; best = ks; }
    }
    return best;
}

bool gemm_sk_supported(int batch, int N, int K)
{
    return batch >= 1 && batch <= 64 && N % 16 == 0 && K % 64 == 0;
}

hipError_t launch_gemm_sk(Mat W, Mat W2, int split_row, const uint16_t *xb, const float *ssq, float eps, float *part,
                          int batch, int N, int K, hipStream_t s)
{
    const int nb = (batch + 15) / 16;
    if (W.scale) {   // int8 weights: xb holds digit planes (bytes), see k_gemm_sk_i8
        GemmI8Args q{};
        q.W = static_cast<const int8_t *>(W.w); q.W2 = static_cast<const int8_t *>(W2.w ? W2.w : W.w);
        q.scale = W.scale; q.scale2 = W2.w ? W2.scale : W.scale; q.split_row = W2.w ? split_row : N;
        q.xd = reinterpret_cast<const uint8_t *>(xb); q.x_plane = (size_t)nb * 16 * K;
        q.part = part; q.batch = batch; q.N = N; q.K = K; q.n_slabs = K / 64; q.ssq = ssq; q.eps = eps;
        const int splits = gemm_sk_splits(batch, N, K, true);
        q.slabs_per_block = (q.n_slabs + splits - 1) / splits;
        const dim3 grid((N + 127) / 128, splits);
        switch (nb) {
        case 1: PSV_LAUNCH(k_gemm_sk_i8<1>, grid, dim3(256), 0, s, q); break;
        case 2: PSV_LAUNCH(k_gemm_sk_i8<2>, grid, dim3(256), 0, s, q); break;
        case 3: PSV_LAUNCH(k_gemm_sk_i8<3>, grid, dim3(256), 0, s, q); break;
        case 4: PSV_LAUNCH(k_gemm_sk_i8<4>, grid, dim3(256), 0, s, q); break;
        default: return hipErrorInvalidValue;
        }
        return hipGetLastError();
    }
    GemmSkArgs a{};
    a.ssq = ssq; a.eps = eps;
    a.W = static_cast<const uint16_t *>(W.w); a.W2 = static_cast<const uint16_t *>(W2.w ? W2.w : W.w);
    a.split_row = W2.w ? split_row : N; a.xb = xb; a.x_plane = (size_t)nb * 16 * K;
    a.part = part; a.batch = batch; a.N = N; a.K = K; a.n_slabs = K / 64;
    const int splits = gemm_sk_splits(batch, N, K, false);
    a.slabs_per_block = (a.n_slabs + splits - 1) / splits;
    const dim3 grid((N + 127) / 128, splits);
    switch (nb) {
    case 1: PSV_LAUNCH(k_gemm_sk<1>, grid, dim3(256), 0, s, a); break;
    case 2: PSV_LAUNCH(k_gemm_sk<2>, grid, dim3(256), 0, s, a); break;
    case 3: PSV_LAUNCH(k_gemm_sk<3>, grid, dim3(256), 0, s, a); break;
    case 4: PSV_LAUNCH(k_gemm_sk<4>, grid, dim3(256), 0, s, a); break;
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

// ------------------------------------------------------------------------------------ KV addressing

__device__ __forceinline__ int kv_phys_block(const int32_t *page_table, int max_blocks, int num_pool_blocks,
                                             int b, int logical)
{
    int idx = b * max_blocks + logical;
    int blk = page_table ? page_table[idx] : idx;
    return (blk >= 0 && blk < num_pool_blocks) ? blk : -1;   // a corrupt entry is skipped, never followed
}

// ------------------------------------------------------------------------------------ RoPE table

// cos/sin of the rotary angles at position seq_len-1, one row of 64 pairs per sequence.  The angle
// is formed and reduced in double (position * theta^(-2i/128)), so long contexts lose nothing to
// fp32 range reduction.  The position is the same for every layer, so this runs once per step.
__global__ __launch_bounds__(64) void k_rope_table(const int32_t *__restrict__ seq_lens, const double *__restrict__ inv_freq,
                                                   int max_tokens, float2 *__restrict__ table)
{
    const int b = blockIdx.x, i = threadIdx.x;
    int T = seq_lens[b];
    if (T < 1 || T > max_tokens) T = 1;
    float2 cs = make_float2(1.f, 0.f);
    if (inv_freq) {
        double sd, cd;
        sincos((double)(T - 1) * inv_freq[i], &sd, &cd);
        cs = make_float2((float)cd, (float)sd);
    }
    table[b * 64 + i] = cs;
}

hipError_t launch_rope_table(const int32_t *seq_lens, const double *inv_freq, int max_tokens, int batch, float2 *table,
                             hipStream_t s)
{
    PSV_LAUNCH(k_rope_table, dim3(batch), dim3(64), 0, s, seq_lens, inv_freq, max_tokens, table);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------ decode attention

AttnSplit attn_split(uint32_t batch, uint32_t n_kv_heads, uint32_t max_seq, bool kv_int8)
{
    // Two workgroups of the attention kernel fit on a CU (register bound), 512 on the chip.  Measured on the
    // large shapes, one round of somewhat fewer workgroups (400-450) is fastest: a second, partial round costs a
    // whole chunk time, and a completely full chip is slower than a nearly full one.  So: at most kAttnResident
    // workgroups, chunks of whole steps (4 waves x one tile) and at most kAttnMaxChunks chunks per
    // (sequence, kv head).  psv_tune_attention replaces this guess by a measurement.
    const int unit = (kv_int8 ? kAttnTileTokensInt8 : kAttnTileTokens) * kAttnWaves;
    const uint64_t seqs = (uint64_t)batch * n_kv_heads;
    uint64_t max_chunks = kAttnResident / (seqs ? seqs : 1);
    if (max_chunks < 1) max_chunks = 1;
    if (max_chunks > (uint64_t)kAttnMaxChunks) max_chunks = kAttnMaxChunks;
    uint64_t chunk = ((uint64_t)max_seq + max_chunks - 1) / max_chunks;
    chunk = (chunk + unit - 1) / unit * unit;
    if (chunk < (uint64_t)unit) chunk = unit;
    AttnSplit sp;
    sp.chunk_tokens = (int)chunk;
    sp.n_chunks = (int)((max_seq + chunk - 1) / chunk);
    if (sp.n_chunks < 1) sp.n_chunks = 1;
    return sp;
}

struct AttnArgs {
    const float *qkv;          // [batch][(nq+2nkv)*128] projection output, not yet rotated
    const float2 *rope;        // [batch][64] (cos, sin)
    KvView kv;
    int nq, nkv, chunk_tokens, n_chunks;
    float *part_ml;            // [batch][nkv][n_chunks][16][2]
    float *part_o;             // [batch][nkv][n_chunks][G][128]
    float *out_f32;            // [batch][nq*128]
    uint16_t *out_bf16;        // same as hi/lo bf16 planes (operand of the MFMA O projection)
    size_t out_plane;          // distance between the planes, elements
    int out_digits;            // out_bf16 receives int8 digit planes (operand of an int8 projection) instead
};

// Split-K decode attention with everything around it fused in.  grid (chunks, kv heads, batch),
// 4 waves; wave w of chunk c takes the 32-token tiles c*chunk + (w + 4*it)*32.
//
//  * prologue: the G <= 16 query heads sharing the kv head are rotated (RoPE) straight into MFMA
//    B-fragments; the workgroup whose chunk holds token T-1 also rotates the new key, rounds key and
//    value to bf16 and appends them to the cache before it reads its tiles.
//  * main loop: all G heads ride in the N side of the MFMAs, so K and V are read from HBM once.
//        S^T[token][g]  = K[token][:] . Q[g][:]          A = K rows (token-major in the pool)
//        O^T[chan][g]  += V^T[chan][token] P[g][token]   A = V^T rows (channel-major in the pool)
//    Tile 1 of a 32-token group covers tokens {8q+0..3}, tile 2 tokens {8q+4..7} (q = 0..3), so after
//    the two S^T MFMAs lane (g, q) holds the scores of the 8 consecutive tokens 8q..8q+7 of its head:
//    exactly the B-fragment the O^T MFMA needs.  Probabilities never leave registers.
//  * epilogue: the 4 waves merge through LDS and the workgroup stores one partial (max, sum, O);
//    k_attn_merge then combines the partials of a (sequence, kv head) in chunk order.
__global__ __launch_bounds__(256) void k_attn(AttnArgs a)
{
    __shared__ float ms[kAttnWaves][16], ls[kAttnWaves][16];
    __shared__ f32x4 accs[kAttnWaves][8][64];

    const int b = blockIdx.z, kvh = blockIdx.y, c = blockIdx.x;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, i = lane & 15, q4 = lane >> 4;
    const int nq = a.nq, nkv = a.nkv, G = nq / nkv;
    const KvView &kv = a.kv;
    const int qkv_rows = (nq + 2 * nkv) * 128;
    int T = kv.seq_lens[b];
    if (T < 0 || T > kv.max_blocks * 16) T = 0;
    const int t_begin = c * a.chunk_tokens;
    const int t_end = min(T, t_begin + a.chunk_tokens);
    const float *qkv_b = a.qkv + (size_t)b * qkv_rows;
    const float2 *rope_b = a.rope + b * 64;

    // ---- K/V tile loader.  The addresses depend on the page table only, not on the sequence length (tokens
    //      past the span are masked later, and every logical block below max_blocks maps into the pool), so
    //      each wave issues the loads of its first tile right away, ahead of everything else in the kernel.
    const int tau1 = 8 * (i >> 2) + (i & 3);          // token (within the 32-token group) of K row i, tile 1
    uint4 ka[4], kb[4], vf[8];
    auto lookup = [&](int t0, int &blkA, int &blkB) {
        const int lb = t0 >> 4;
        blkA = kv_phys_block(kv.page_table, kv.max_blocks, kv.num_pool_blocks, b, lb);
        blkB = (lb + 1 < kv.max_blocks) ? kv_phys_block(kv.page_table, kv.max_blocks, kv.num_pool_blocks, b, lb + 1) : -1;
    };
    auto load_blocks = [&](int blkA, int blkB) {
        // K fragments: tile 1 row i = token tau1, tile 2 row i = token tau1 + 4
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
        // V^T fragments: row = channel dg*16 + i, k-slots of lane group q4 = tokens 8*q4 .. 8*q4+7
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
    auto load_tile = [&](int t0) {
        int blkA, blkB;
        lookup(t0, blkA, blkB);
        load_blocks(blkA, blkB);
    };
    // Order of the first requests: page-table entries of the first tile, then the query rows and the rotary
    // table, then the tile itself.  Loads return in order, so the query can be rotated while the tile -- the one
    // request that goes all the way to HBM -- is still on its way.
    const int t_first = t_begin + w * kAttnTileTokens;
    const bool early = t_first < kv.max_blocks * 16;
    int blkA0 = -1, blkB0 = -1;
    if (early) lookup(t_first, blkA0, blkB0);
    float qlo[2][8], qhi[2][8];
    float2 qcs[2][8];
    if (i < G) {
        const float *qrow = qkv_b + (size_t)(kvh * G + i) * 128;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const int f0 = ks * 32 + q4 * 8;
            *reinterpret_cast<float4 *>(qlo[ks]) = *reinterpret_cast<const float4 *>(qrow + f0);
            *reinterpret_cast<float4 *>(qlo[ks] + 4) = *reinterpret_cast<const float4 *>(qrow + f0 + 4);
            *reinterpret_cast<float4 *>(qhi[ks]) = *reinterpret_cast<const float4 *>(qrow + f0 + 64);
            *reinterpret_cast<float4 *>(qhi[ks] + 4) = *reinterpret_cast<const float4 *>(qrow + f0 + 68);
#pragma unroll
            for (int e = 0; e < 8; ++e) qcs[ks][e] = rope_b[f0 + e];
        }
    }
    if (early) load_blocks(blkA0, blkB0);

    // ---- Q fragments, rotated: lane (g = i, q4) holds channels ks*32 + q4*8 + e; channel f < 64
    //      pairs with f + 64, i.e. fragment ks with fragment ks + 2 of the same lane.
    bf16x8 qf[4];
    {
        uint4 z = zero16();
        qf[0] = qf[1] = qf[2] = qf[3] = __builtin_bit_cast(bf16x8, z);
        if (i < G) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const float *lo = qlo[ks], *hi = qhi[ks];
                float rl[8], rh[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float2 cs = qcs[ks][e];
                    rl[e] = lo[e] * cs.x - hi[e] * cs.y;
                    rh[e] = hi[e] * cs.x + lo[e] * cs.y;
                }
                uint4 pl = make_uint4(pack_bf16(rl[0], rl[1]), pack_bf16(rl[2], rl[3]), pack_bf16(rl[4], rl[5]), pack_bf16(rl[6], rl[7]));
                uint4 ph = make_uint4(pack_bf16(rh[0], rh[1]), pack_bf16(rh[2], rh[3]), pack_bf16(rh[4], rh[5]), pack_bf16(rh[6], rh[7]));
                qf[ks] = __builtin_bit_cast(bf16x8, pl);
                qf[ks + 2] = __builtin_bit_cast(bf16x8, ph);
            }
        }
    }

    // ---- append the new token's K and V (one workgroup per kv head does it)
    if (T >= 1 && c == (T - 1) / a.chunk_tokens) {
        if (tid < 64) {
            const int pos = T - 1;
            const int blk = kv_phys_block(kv.page_table, kv.max_blocks, kv.num_pool_blocks, b, pos >> 4);
            if (blk >= 0) {
                const float2 cs = rope_b[tid];
                const float *krow = qkv_b + (size_t)(nq + kvh) * 128;
                const float *vrow = qkv_b + (size_t)(nq + nkv + kvh) * 128;
                const float lo = krow[tid], hi = krow[tid + 64];
                const int r = pos & 15;
                uint16_t *kdst = kv.k_pool + (((size_t)blk * nkv + kvh) * 16 + r) * 128;
                kdst[tid] = (uint16_t)f32_to_bf16(lo * cs.x - hi * cs.y);
                kdst[tid + 64] = (uint16_t)f32_to_bf16(hi * cs.x + lo * cs.y);
                uint16_t *vdst = kv.v_pool + ((size_t)blk * nkv + kvh) * 128 * 16 + r;
                vdst[(size_t)tid * 16] = (uint16_t)f32_to_bf16(vrow[tid]);
                vdst[(size_t)(tid + 64) * 16] = (uint16_t)f32_to_bf16(vrow[tid + 64]);
            }
            __threadfence();
        }
        __syncthreads();   // uniform: the condition depends on the workgroup only
        if (early && T - 1 >= t_first && T - 1 < t_first + kAttnTileTokens) load_tile(t_first);   // now with the new entry
    }

    const float kScale = 0.08838834764831845f * 1.4426950408889634f;   // 1/sqrt(128) * log2(e)
    float m_run = -1.0e30f, l_part = 0.f;
    f32x4 acc[8];
#pragma unroll
    for (int dg = 0; dg < 8; ++dg) acc[dg] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int t0 = t_first; t0 < t_end; t0 += kAttnWaves * kAttnTileTokens) {
        if (t0 != t_first || !early) load_tile(t0);

        f32x4 s1 = {0.f, 0.f, 0.f, 0.f}, s2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[ks]), qf[ks], s1, 0, 0, 0);
            s2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kb[ks]), qf[ks], s2, 0, 0, 0);
        }
        // lane (g = i, q4) now holds tokens t0 + 8*q4 + e, e = 0..7
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
        const float m_new = fmaxf(m_run, tmax);
        const float alpha = exp2f(m_run - m_new);
        float p[8], psum = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            p[e] = exp2f(sv[e] - m_new);
            psum += p[e];
        }
        l_part = l_part * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int dg = 0; dg < 8; ++dg) acc[dg] *= alpha;

        uint4 pk = make_uint4(pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]), pack_bf16(p[4], p[5]), pack_bf16(p[6], p[7]));
        if (t0 + kAttnTileTokens > t_end) {
            // ragged tail: cache slots past the span may hold anything (even NaN); blank them so
            // that 0 * garbage cannot reach the accumulators.
            uint32_t mlo[4];
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                uint32_t m0 = (tl + 2 * h < t_end) ? 0x0000ffffu : 0u;
                uint32_t m1 = (tl + 2 * h + 1 < t_end) ? 0xffff0000u : 0u;
                mlo[h] = m0 | m1;
            }
#pragma unroll
            for (int dg = 0; dg < 8; ++dg) {
                vf[dg].x &= mlo[0]; vf[dg].y &= mlo[1]; vf[dg].z &= mlo[2]; vf[dg].w &= mlo[3];
            }
        }
        const bf16x8 pfrag = __builtin_bit_cast(bf16x8, pk);
#pragma unroll
        for (int dg = 0; dg < 8; ++dg)
            acc[dg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vf[dg]), pfrag, acc[dg], 0, 0, 0);
    }

    // ---- merge the 4 waves (wave order)
    l_part += __shfl_xor(l_part, 16, 64);
    l_part += __shfl_xor(l_part, 32, 64);
    if (q4 == 0) ms[w][i] = m_run;
    __syncthreads();
    const float M = fmaxf(fmaxf(ms[0][i], ms[1][i]), fmaxf(ms[2][i], ms[3][i]));
    const float sc = exp2f(m_run - M);
    if (q4 == 0) ls[w][i] = l_part * sc;
#pragma unroll
    for (int dg = 0; dg < 8; ++dg) accs[w][dg][lane] = acc[dg] * sc;
    __syncthreads();
    const size_t slot0 = ((size_t)b * nkv + kvh) * a.n_chunks;
    if (i < G) {
        const size_t slot = slot0 + c;
        if (w == 0 && q4 == 0) {
            a.part_ml[(slot * 16 + i) * 2 + 0] = M;
            a.part_ml[(slot * 16 + i) * 2 + 1] = ls[0][i] + ls[1][i] + ls[2][i] + ls[3][i];
        }
#pragma unroll
        for (int d = 0; d < 2; ++d) {
            const int dg = 2 * w + d;
            f32x4 v = accs[0][dg][lane];
            v += accs[1][dg][lane];
            v += accs[2][dg][lane];
            v += accs[3][dg][lane];
            *reinterpret_cast<float4 *>(a.part_o + (slot * G + i) * 128 + dg * 16 + 4 * q4) = make_float4(v[0], v[1], v[2], v[3]);
        }
    }

}

// ---- int8 cache: decode attention on the int8 matrix cores -------------------------------------------------
//
// Same split-K scheme and the same partials as k_attn, but the cache codes go into v_mfma_i32_16x16x64_i8 as
// they are (no widening): the floating-point operand of each contraction is cut into two int8 "digits" with
// a per-column scale, x ~ s * (d1 + d2 / 254), |d| <= 127, which keeps 15-16 bits of the column's largest
// element, and the two exact i32 results are recombined as 254 * D1 + D2 before one conversion to fp32.
//   S^T[token][g] = K[token][:] . Q[g][:]      A = K codes, 16 bytes = 16 channels per lane and k step
//                                              B = digits of the rotated query (scale per head)
//   O^T[chan][g] += V^T[chan][token] P'[g][token]   A = V codes, 16 bytes = the 16 tokens of one block
//                                              B = digits of P' = softmax numerator x value scale (scale per
//                                                  head and tile)
// A wave tile is 64 tokens = 4 cache blocks.  Row i of score tile m (m = 0..3) is token 16*(i/4) + 4m + i%4,
// so that lane (g, q4) ends up with the scores of tokens 16*q4 .. 16*q4+15 -- block q4, in byte order -- which
// is exactly the B operand of the second contraction.  Key scales multiply the scores, value scales the
// probabilities.  The appended rows are quantised per row in single precision (scale = max|v| / 127,
// code = rint(v / scale)), stored, and re-read by the wave whose tile holds them.

__global__ __launch_bounds__(256) void k_attn_q8(AttnArgs a)
{
    constexpr int TT = kAttnTileTokensInt8;
    __shared__ float ms[kAttnWaves][16], ls[kAttnWaves][16];
    __shared__ f32x4 accs[kAttnWaves][8][64];

    const int b = blockIdx.z, kvh = blockIdx.y, c = blockIdx.x;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, i = lane & 15, q4 = lane >> 4;
    const int nq = a.nq, nkv = a.nkv, G = nq / nkv;
    const KvView &kv = a.kv;
    const int qkv_rows = (nq + 2 * nkv) * 128;
    int T = kv.seq_lens[b];
    if (T < 0 || T > kv.max_blocks * 16) T = 0;
    const int t_begin = c * a.chunk_tokens;
    const int t_end = min(T, t_begin + a.chunk_tokens);
    const float *qkv_b = a.qkv + (size_t)b * qkv_rows;
    const float2 *rope_b = a.rope + b * 64;
    uint8_t *k8 = reinterpret_cast<uint8_t *>(kv.k_pool), *v8 = reinterpret_cast<uint8_t *>(kv.v_pool);

    // ---- tile loader (addresses depend on the page table only, so the first tile is requested right away)
    uint4 kc[4][2], vc[8];
    float4 ksc[4], vsc[4];
    auto lookup = [&](int t0, int &blkK, int &blkV) {
        const int lb = t0 >> 4;
        const int lbk = lb + (i >> 2), lbv = lb + q4;        // block of this lane's K rows / of its V tokens
        blkK = lbk < kv.max_blocks ? kv_phys_block(kv.page_table, kv.max_blocks, kv.num_pool_blocks, b, lbk) : -1;
        blkV = lbv < kv.max_blocks ? kv_phys_block(kv.page_table, kv.max_blocks, kv.num_pool_blocks, b, lbv) : -1;
    };
    auto load_blocks = [&](int blkK, int blkV) {
        // A block outside the table (or a corrupt entry) reads block 0 and is blanked with selects: whole-array
        // assignments in two branches would push the fragments out of registers.
        const bool okK = blkK >= 0, okV = blkV >= 0;
        {
            const uint8_t *base = k8 + ((size_t)(okK ? blkK : 0) * nkv + kvh) * PSV_KV_UNIT_BYTES_INT8 + (i & 3) * 128 + q4 * 16;
#pragma unroll
            for (int m = 0; m < 4; ++m)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const uint4 v = *reinterpret_cast<const uint4 *>(base + m * 4 * 128 + j * 64);
                    kc[m][j] = make_uint4(okK ? v.x : 0u, okK ? v.y : 0u, okK ? v.z : 0u, okK ? v.w : 0u);
                }
        }
        {
            const size_t unit = ((size_t)(okV ? blkV : 0) * nkv + kvh) * PSV_KV_UNIT_BYTES_INT8;
#pragma unroll
            for (int dg = 0; dg < 8; ++dg) {
                const uint4 v = *reinterpret_cast<const uint4 *>(v8 + unit + (dg * 16 + i) * 16);
                vc[dg] = make_uint4(okV ? v.x : 0u, okV ? v.y : 0u, okV ? v.z : 0u, okV ? v.w : 0u);
            }
            const float4 *ks4 = reinterpret_cast<const float4 *>(k8 + unit + 2048);
            const float4 *vs4 = reinterpret_cast<const float4 *>(v8 + unit + 2048);
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const float4 kq = ks4[m], vq4 = vs4[m];
                ksc[m] = make_float4(okV ? kq.x : 0.f, okV ? kq.y : 0.f, okV ? kq.z : 0.f, okV ? kq.w : 0.f);
                vsc[m] = make_float4(okV ? vq4.x : 0.f, okV ? vq4.y : 0.f, okV ? vq4.z : 0.f, okV ? vq4.w : 0.f);
            }
        }
    };
    auto load_tile = [&](int t0) {
        int blkK, blkV;
        lookup(t0, blkK, blkV);
        load_blocks(blkK, blkV);
    };
    // Order of the first requests: page-table entries of the first tile, then the query row and the rotary table,
    // then the tile itself; loads return in order, so the query digits are formed while the tile is on its way.
    const int t_first = t_begin + w * TT;
    const bool early = t_first < kv.max_blocks * 16;
    int blkK0 = -1, blkV0 = -1;
    if (early) lookup(t_first, blkK0, blkV0);
    const bool have_q = i < G;
    float4 q_lo[4], q_hi[4];
    float2 q_cs[16];
    {
        const float *qrow = qkv_b + (size_t)(kvh * G + (have_q ? i : 0)) * 128 + q4 * 16;
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
            q_lo[e4] = *reinterpret_cast<const float4 *>(qrow + e4 * 4);
            q_hi[e4] = *reinterpret_cast<const float4 *>(qrow + 64 + e4 * 4);
#pragma unroll
            for (int u = 0; u < 4; ++u) q_cs[e4 * 4 + u] = rope_b[q4 * 16 + e4 * 4 + u];
        }
    }
    if (early) load_blocks(blkK0, blkV0);

    // ---- query digits: lane (g = i, q4) holds channels j*64 + q4*16 + e (j = 0, 1; e = 0..15), the byte order of
    //      its K codes; channel f < 64 pairs with f + 64 for the rotation, i.e. j = 0 with j = 1 of the same lane
    uint4 qd1[2], qd2[2];
    float q_back = 0.f;                       // head scale / 254 * softmax scale, applied to 254*S1 + S2
    const float kScale = 0.08838834764831845f * 1.4426950408889634f;   // 1/sqrt(128) * log2(e)
    {
        float ql[16], qh[16];
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
            const float4 lo = q_lo[e4], hi = q_hi[e4];
            const float2 c0 = q_cs[e4 * 4 + 0], c1 = q_cs[e4 * 4 + 1], c2 = q_cs[e4 * 4 + 2], c3 = q_cs[e4 * 4 + 3];
            ql[e4 * 4 + 0] = have_q ? lo.x * c0.x - hi.x * c0.y : 0.f;
            qh[e4 * 4 + 0] = have_q ? hi.x * c0.x + lo.x * c0.y : 0.f;
            ql[e4 * 4 + 1] = have_q ? lo.y * c1.x - hi.y * c1.y : 0.f;
            qh[e4 * 4 + 1] = have_q ? hi.y * c1.x + lo.y * c1.y : 0.f;
            ql[e4 * 4 + 2] = have_q ? lo.z * c2.x - hi.z * c2.y : 0.f;
            qh[e4 * 4 + 2] = have_q ? hi.z * c2.x + lo.z * c2.y : 0.f;
            ql[e4 * 4 + 3] = have_q ? lo.w * c3.x - hi.w * c3.y : 0.f;
            qh[e4 * 4 + 3] = have_q ? hi.w * c3.x + lo.w * c3.y : 0.f;
        }
        float amax = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) amax = fmaxf(amax, fmaxf(fabsf(ql[e]), fabsf(qh[e])));
        amax = fmaxf(amax, __shfl_xor(amax, 16, 64));
        amax = fmaxf(amax, __shfl_xor(amax, 32, 64));
        const float inv = amax > 0.f ? 127.0f / amax : 0.f;
        q_back = amax / 127.0f / 254.0f * kScale;
        uint32_t w1[2][4], w2[2][4];
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
            float a1[4], a2[4], b1[4], b2[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                two_digits(ql[e4 * 4 + u] * inv, a1[u], a2[u]);
                two_digits(qh[e4 * 4 + u] * inv, b1[u], b2[u]);
            }
            w1[0][e4] = pack_magic_bytes(a1[0], a1[1], a1[2], a1[3]);
            w2[0][e4] = pack_magic_bytes(a2[0], a2[1], a2[2], a2[3]);
            w1[1][e4] = pack_magic_bytes(b1[0], b1[1], b1[2], b1[3]);
            w2[1][e4] = pack_magic_bytes(b2[0], b2[1], b2[2], b2[3]);
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            qd1[j] = make_uint4(w1[j][0], w1[j][1], w1[j][2], w1[j][3]);
            qd2[j] = make_uint4(w2[j][0], w2[j][1], w2[j][2], w2[j][3]);
        }
    }

    // ---- append the new token's K and V (one workgroup per kv head does it)
    if (T >= 1 && c == (T - 1) / a.chunk_tokens) {
        if (tid < 64) {
            const int pos = T - 1;
            const int blk = kv_phys_block(kv.page_table, kv.max_blocks, kv.num_pool_blocks, b, pos >> 4);
            if (blk >= 0) {    // uniform over the wave
                const float2 cs = rope_b[tid];
                const float *krow = qkv_b + (size_t)(nq + kvh) * 128;
                const float *vrow = qkv_b + (size_t)(nq + nkv + kvh) * 128;
                const float lo = krow[tid], hi = krow[tid + 64];
                const int r = pos & 15;
                const float k0 = lo * cs.x - hi * cs.y, k1 = hi * cs.x + lo * cs.y;
                const float v0 = vrow[tid], v1 = vrow[tid + 64];
                const float ka_max = wave_max(fmaxf(fabsf(k0), fabsf(k1)));
                const float va_max = wave_max(fmaxf(fabsf(v0), fabsf(v1)));
                const float ksc1 = ka_max > 0.f ? ka_max / 127.0f : 1.0f;
                const float vsc1 = va_max > 0.f ? va_max / 127.0f : 1.0f;
                const size_t unit = ((size_t)blk * nkv + kvh) * PSV_KV_UNIT_BYTES_INT8;
                uint8_t *kdst = k8 + unit, *vdst = v8 + unit;
                kdst[r * 128 + tid] = quant_i8(k0, ksc1);
                kdst[r * 128 + tid + 64] = quant_i8(k1, ksc1);
                vdst[tid * 16 + r] = quant_i8(v0, vsc1);
                vdst[(tid + 64) * 16 + r] = quant_i8(v1, vsc1);
                if (tid == 0) {
                    reinterpret_cast<float *>(kdst + 2048)[r] = ksc1;
                    reinterpret_cast<float *>(vdst + 2048)[r] = vsc1;
                }
            }
            __threadfence();
        }
        __syncthreads();   // uniform: the condition depends on the workgroup only
        if (early && T - 1 >= t_first && T - 1 < t_first + TT) load_tile(t_first);   // now with the new entry
    }

    float m_run = -1.0e30f, l_part = 0.f;
    f32x4 acc[8];
#pragma unroll
    for (int dg = 0; dg < 8; ++dg) acc[dg] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int t0 = t_first; t0 < t_end; t0 += kAttnWaves * TT) {
        if (t0 != t_first || !early) load_tile(t0);

        // scores of tokens t0 + 16*q4 + e, e = 4m + j
        float sv[16];
        const int tl = t0 + 16 * q4;
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            i32x4 s1 = {0, 0, 0, 0}, s2 = {0, 0, 0, 0};
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const i32x4 ak = __builtin_bit_cast(i32x4, kc[m][j]);
                s1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(ak, __builtin_bit_cast(i32x4, qd1[j]), s1, 0, 0, 0);
                s2 = __builtin_amdgcn_mfma_i32_16x16x64_i8(ak, __builtin_bit_cast(i32x4, qd2[j]), s2, 0, 0, 0);
            }
            const float kk4[4] = {ksc[m].x, ksc[m].y, ksc[m].z, ksc[m].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float raw = (float)(s1[j] * 254 + s2[j]);
                sv[4 * m + j] = (tl + 4 * m + j < t_end) ? raw * q_back * kk4[j] : -INFINITY;
            }
        }
        float tmax = sv[0];
#pragma unroll
        for (int e = 1; e < 16; ++e) tmax = fmaxf(tmax, sv[e]);
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
        const float m_new = fmaxf(m_run, tmax);
        const float alpha = exp2f(m_run - m_new);
        float pv[16], psum = 0.f, pmax = 0.f;
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const float vv4[4] = {vsc[m].x, vsc[m].y, vsc[m].z, vsc[m].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int e = 4 * m + j;
                const float p = exp2f(sv[e] - m_new);
                psum += p;
                // slots past the span may hold any scale: their probability is an exact zero only while it is
                // not multiplied by a NaN or an infinity
                pv[e] = (tl + e < t_end) ? p * vv4[j] : 0.f;
                pmax = fmaxf(pmax, fabsf(pv[e]));
            }
        }
        l_part = l_part * alpha + psum;
        m_run = m_new;
        pmax = fmaxf(pmax, __shfl_xor(pmax, 16, 64));
        pmax = fmaxf(pmax, __shfl_xor(pmax, 32, 64));
        const float p_inv = pmax > 0.f ? 127.0f / pmax : 0.f;
        const float p_back = pmax / 127.0f / 254.0f;
        uint32_t pw1[4], pw2[4];
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            float a1[4], a2[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) two_digits(pv[4 * m + j] * p_inv, a1[j], a2[j]);
            pw1[m] = pack_magic_bytes(a1[0], a1[1], a1[2], a1[3]);
            pw2[m] = pack_magic_bytes(a2[0], a2[1], a2[2], a2[3]);
        }
        const i32x4 pd1 = {(int)pw1[0], (int)pw1[1], (int)pw1[2], (int)pw1[3]};
        const i32x4 pd2 = {(int)pw2[0], (int)pw2[1], (int)pw2[2], (int)pw2[3]};
#pragma unroll
        for (int dg = 0; dg < 8; ++dg) {
            const i32x4 av = __builtin_bit_cast(i32x4, vc[dg]);
            const i32x4 z = {0, 0, 0, 0};
            const i32x4 o1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(av, pd1, z, 0, 0, 0);
            const i32x4 o2 = __builtin_amdgcn_mfma_i32_16x16x64_i8(av, pd2, z, 0, 0, 0);
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[dg][j] = fmaf(acc[dg][j], alpha, p_back * (float)(o1[j] * 254 + o2[j]));
        }
    }

    // ---- merge the 4 waves (wave order); same partials as k_attn
    l_part += __shfl_xor(l_part, 16, 64);
    l_part += __shfl_xor(l_part, 32, 64);
    if (q4 == 0) ms[w][i] = m_run;
    __syncthreads();
    const float M = fmaxf(fmaxf(ms[0][i], ms[1][i]), fmaxf(ms[2][i], ms[3][i]));
    const float sc = exp2f(m_run - M);
    if (q4 == 0) ls[w][i] = l_part * sc;
#pragma unroll
    for (int dg = 0; dg < 8; ++dg) accs[w][dg][lane] = acc[dg] * sc;
    __syncthreads();
    const size_t slot0 = ((size_t)b * nkv + kvh) * a.n_chunks;
    if (i < G) {
        const size_t slot = slot0 + c;
        if (w == 0 && q4 == 0) {
            a.part_ml[(slot * 16 + i) * 2 + 0] = M;
            a.part_ml[(slot * 16 + i) * 2 + 1] = ls[0][i] + ls[1][i] + ls[2][i] + ls[3][i];
        }
#pragma unroll
        for (int d = 0; d < 2; ++d) {
            const int dg = 2 * w + d;
            f32x4 v = accs[0][dg][lane];
            v += accs[1][dg][lane];
            v += accs[2][dg][lane];
            v += accs[3][dg][lane];
            *reinterpret_cast<float4 *>(a.part_o + (slot * G + i) * 128 + dg * 16 + 4 * q4) = make_float4(v[0], v[1], v[2], v[3]);
        }
    }
}

// Merge of the chunk partials of one (sequence, query head): grid (query heads, batch), 1024 threads = 128
// channels x 8 groups that share the chunks.  Wave 0 forms the softmax weights of the chunks once (LDS); every
// thread sums its group's chunks of its channel in chunk order, and the 8 partial sums are added in group order.
// All orders are fixed, so the result is reproducible.
__global__ __launch_bounds__(1024) void k_attn_merge(AttnArgs a)
{
    __shared__ float wl[kAttnMaxChunks + 8];   // weights of the chunks (+ slack for the predicated last batch)
    __shared__ float inv_den;
    __shared__ float psum[1024];
    const int j = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int nq = a.nq, nkv = a.nkv, G = nq / nkv, nc = a.n_chunks;
    const int kvh = j / G, g = j % G;
    const size_t slot0 = ((size_t)b * nkv + kvh) * nc;
    if (w == 0) {
        constexpr int MU = kAttnMaxChunks / 64;
        float2 ml[MU];
        float Mx = -1.0e30f;
#pragma unroll
        for (int u = 0; u < MU; ++u) {
            const int sp = lane + 64 * u;
            ml[u] = sp < nc ? *reinterpret_cast<const float2 *>(a.part_ml + ((slot0 + sp) * 16 + g) * 2)
                            : make_float2(-1.0e30f, 0.f);
            Mx = fmaxf(Mx, ml[u].x);
        }
        Mx = wave_max(Mx);
        float den = 0.f;
#pragma unroll
        for (int u = 0; u < MU; ++u) {
            const int sp = lane + 64 * u;
            const float wgt = ml[u].y > 0.f ? exp2f(ml[u].x - Mx) : 0.f;
            if (sp < nc) wl[sp] = wgt;
            den += wave_sum(wgt * ml[u].y);
        }
        if (lane == 0) inv_den = den > 0.f ? 1.0f / den : 0.f;
    }
    __syncthreads();
    const int ch = tid & 127, sg = tid >> 7;               // 8 groups
    const int per = (nc + 7) / 8;
    const int sp_end = min(nc, (sg + 1) * per);
    const float *po = a.part_o + (slot0 * G + g) * 128 + ch;
    const size_t stride = (size_t)G * 128;                 // chunk to chunk
    float num = 0.f;
    int sp = sg * per;
    for (; sp + 8 <= sp_end; sp += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = po[(size_t)(sp + u) * stride];
#pragma unroll
        for (int u = 0; u < 8; ++u) num = fmaf(wl[sp + u], v[u], num);
    }
    {   // ragged end of the group's range, still one batch of loads
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = sp + u < sp_end ? po[(size_t)(sp + u) * stride] : 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u) num = fmaf(sp + u < sp_end ? wl[sp + u] : 0.f, v[u], num);
    }
    psum[tid] = num;
    __syncthreads();
    if (sg == 0) {
        num = 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k) num += psum[k * 128 + ch];   // group order
        const float r = num * inv_den;
        const size_t idx = ((size_t)b * nq + j) * 128 + ch;
        a.out_f32[idx] = r;
        if (!a.out_digits) {
            uint32_t hi, lo;
            split_bf16(r, hi, lo);
            a.out_bf16[idx] = (uint16_t)hi;
            a.out_bf16[a.out_plane + idx] = (uint16_t)lo;
        }
        psum[ch] = r;      // the writers of psum[0..127] are these same threads
    }
    if (!a.out_digits) return;
    __syncthreads();
    if (tid < 32) {        // one head = one 128-element block of the digit planes: 32 lanes x 4 channels
        const float4 v = make_float4(psum[4 * tid], psum[4 * tid + 1], psum[4 * tid + 2], psum[4 * tid + 3]);
        // only half of the wave is here, so the block maximum comes from LDS-free DPP steps within rows of 16 and
        // one exchange between the two rows, all inside lanes 0..31
        store_digits4(reinterpret_cast<uint8_t *>(a.out_bf16), a.out_plane, nq * 128, (size_t)b, j * 128 + 4 * tid, v);
    }
}

static AttnArgs attn_args(const float *qkv, const float2 *rope, KvView kv, int batch, int nq, int nkv, AttnSplit sp,
                          float *part_ml, float *part_o, float *out_f32, uint16_t *out_bf16)
{
    const size_t out_plane = (size_t)((batch + 15) / 16 * 16) * nq * 128;
    return AttnArgs{qkv, rope, kv, nq, nkv, sp.chunk_tokens, sp.n_chunks, part_ml, part_o, out_f32, out_bf16, out_plane, 0};
}

hipError_t launch_attn(const float *qkv, const float2 *rope, KvView kv, int batch, int nq, int nkv, AttnSplit sp,
                       float *part_ml, float *part_o, hipStream_t s)
{
    AttnArgs a = attn_args(qkv, rope, kv, batch, nq, nkv, sp, part_ml, part_o, nullptr, nullptr);
    if (kv.int8)
        PSV_LAUNCH(k_attn_q8, dim3(sp.n_chunks, nkv, batch), dim3(256), 0, s, a);
    else
        PSV_LAUNCH(k_attn, dim3(sp.n_chunks, nkv, batch), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_attn_merge(const float *part_ml, const float *part_o, int batch, int nq, int nkv, AttnSplit sp,
                             float *out_f32, uint16_t *out_bf16, bool digits, hipStream_t s)
{
    AttnArgs a = attn_args(nullptr, nullptr, KvView{}, batch, nq, nkv, sp, const_cast<float *>(part_ml),
                           const_cast<float *>(part_o), out_f32, out_bf16);
    a.out_digits = digits ? 1 : 0;
    PSV_LAUNCH(k_attn_merge, dim3(nq, batch), dim3(1024), 0, s, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------ spin window

// One workgroup of one wave busy-waits on the constant-rate wall clock; the iteration cap makes
// sure the wave exits even if the clock misbehaves.  On entry it publishes the window's sequence
// number: a gate kernel (k_gate) is already waiting for it on the side stream, ahead of the window's
// prefetch launches (a device-side fork, no host event in between).
// On exit it publishes the same number in *done (release order): a consumer kernel that was launched ahead of
// time on the other stream and has already pulled its weights into registers waits for exactly that (k_gemv).
__global__ __launch_bounds__(64) void k_spin(uint64_t ticks, uint32_t max_iters, unsigned *flag, unsigned *done, unsigned seq)
{
    const uint64_t t0 = wall_clock64();
    if (flag && threadIdx.x == 0) __hip_atomic_store(flag, seq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    uint32_t it = 0;
    while (wall_clock64() - t0 < ticks && it < max_iters) {
        __builtin_amdgcn_s_sleep(2);
        ++it;
    }
    if (done && threadIdx.x == 0) __hip_atomic_store(done, seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

hipError_t launch_spin(uint64_t ticks, uint32_t max_iters, unsigned *flag, unsigned *done, unsigned seq, hipStream_t s)
{
    PSV_LAUNCH(k_spin, dim3(1), dim3(64), 0, s, ticks, max_iters, flag, done, seq);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------ prefetch

// Reads memory with 16-byte loads and throws the data away: the loads allocate the lines in the
// memory-side cache (Infinity Cache).  Nothing is written.  One launch serves a whole communication
// window: up to kPrefetchRegions linear regions (projection weights) plus a range of KV blocks that
// is walked through the page table.  The grid size is the CU budget of the policy; 16 x 16-byte loads are in flight per thread.
__device__ __forceinline__ uint32_t fold(uint4 v) { return v.x ^ v.y ^ v.z ^ v.w; }

__global__ __launch_bounds__(256) void k_prefetch(PrefetchJob j)
{
    constexpr int U = 16;
    if (j.skip && *j.skip) return;   // the gate kernel ahead of this launch found the window already over
    const uint64_t stride = (uint64_t)gridDim.x * 256;
    const uint64_t me = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    uint32_t sink = 0;
    for (int r = 0; r < j.n_regions; ++r) {
        const uint4 *p = reinterpret_cast<const uint4 *>(j.ptr[r]);
        const uint64_t n16 = j.n16[r];
        // batches of U independent loads per thread; the ragged end of a region is predicated rather than
        // peeled into a one-load-at-a-time loop, so a region costs one round trip per batch, tail included
        for (uint64_t base = me; base < n16; base += U * stride) {
            uint4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint64_t idx = base + u * stride;
                v[u] = idx < n16 ? p[idx] : zero16();
            }
#pragma unroll
            for (int u = 0; u < U; ++u) sink ^= fold(v[u]);
        }
    }
    if (j.kv_count) {
        // Work item = one (logical block, kv head): a K unit and a V unit (bf16: 4 KiB each; int8: 2112 bytes, codes
        // + scales).  A wave takes up to NBW items per step and requests all of them before it looks at any
        // result; with few items every wave takes one, so that a small cache is spread over many waves.
        constexpr int NBW = 4;
        const int lane = threadIdx.x & 63;
        const uint64_t gw = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
        const uint64_t nw = (uint64_t)gridDim.x * 4;
        const uint32_t unit16 = j.kv.int8 ? PSV_KV_UNIT_BYTES_INT8 / 16 : 256;   // 16-byte words per unit
        const uint64_t items = j.kv_count * (uint64_t)j.nkv;
        const int nbw = items >= nw * NBW ? NBW : 1;
        for (uint64_t q0 = gw * nbw; q0 < items; q0 += nw * nbw) {
            const uint4 *kp[NBW], *vp[NBW];
#pragma unroll
            for (int u = 0; u < NBW; ++u) {
                kp[u] = vp[u] = nullptr;
                const uint64_t q = q0 + u;
                if (u < nbw && q < items) {
                    const uint64_t lin = j.kv_first + q / j.nkv;
                    const int kvh = (int)(q % j.nkv);
                    const int b = (int)(lin / j.blocks_per_seq), lb = (int)(lin % j.blocks_per_seq);
                    const int blk = lb < j.kv.max_blocks
                                        ? kv_phys_block(j.kv.page_table, j.kv.max_blocks, j.kv.num_pool_blocks, b, lb) : -1;
                    if (blk >= 0) {
                        const size_t at = ((size_t)blk * j.nkv + kvh) * unit16;
                        kp[u] = reinterpret_cast<const uint4 *>(j.kv.k_pool) + at;
                        vp[u] = reinterpret_cast<const uint4 *>(j.kv.v_pool) + at;
                    }
                }
            }
            for (uint32_t o = lane; o < unit16; o += 192) {   // 3 words per pool: one step covers an int8 unit
                const bool p1 = o + 64 < unit16, p2 = o + 128 < unit16;
                uint4 v[NBW][6];
#pragma unroll
                for (int u = 0; u < NBW; ++u) {
                    const bool ok = kp[u] != nullptr;
                    v[u][0] = ok ? kp[u][o] : zero16();
                    v[u][1] = ok && p1 ? kp[u][o + 64] : zero16();
                    v[u][2] = ok && p2 ? kp[u][o + 128] : zero16();
                    v[u][3] = ok ? vp[u][o] : zero16();
                    v[u][4] = ok && p1 ? vp[u][o + 64] : zero16();
                    v[u][5] = ok && p2 ? vp[u][o + 128] : zero16();
                }
#pragma unroll
                for (int u = 0; u < NBW; ++u)
                    sink ^= fold(v[u][0]) ^ fold(v[u][1]) ^ fold(v[u][2]) ^ fold(v[u][3]) ^ fold(v[u][4]) ^ fold(v[u][5]);
            }
        }
    }
    asm volatile("" ::"v"(sink));   // keeps the loads alive without a store
}

// Device-side fork.  One wave waits (bounded) until the main stream has entered the window whose
// sequence number is `seq` (published by k_spin), then ends, which releases the prefetch launches queued
// behind it on the side stream.  A single wave cannot keep any main-stream kernel off the CUs, whatever
// that kernel's register or LDS footprint.  If a later window has already begun, the data would arrive
// after its consumers ran: *skip = 1 tells the prefetch launches to do nothing.  Being early or late can
// never change a result (prefetch only reads), so the bounds are just an exit guarantee.
__global__ __launch_bounds__(64) void k_gate(const unsigned *flag, unsigned seq, uint32_t wait_iters, uint64_t wait_ticks,
                                             unsigned *skip)
{
    if (threadIdx.x != 0) return;
    const uint64_t t0 = wall_clock64();
    unsigned v = __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    uint32_t it = 0;
    while ((int)(v - seq) < 0 && it < wait_iters && wall_clock64() - t0 < wait_ticks) {
        __builtin_amdgcn_s_sleep(2);
        v = __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ++it;
    }
    *skip = (int)(v - seq) > 0 ? 1u : 0u;
}

hipError_t launch_gate(const unsigned *flag, unsigned seq, uint32_t wait_iters, uint64_t wait_ticks, unsigned *skip,
                       hipStream_t s)
{
    PSV_LAUNCH(k_gate, dim3(1), dim3(64), 0, s, flag, seq, wait_iters, wait_ticks, skip);
    return hipGetLastError();
}

hipError_t launch_prefetch_job(const PrefetchJob &j, uint32_t workgroups, hipStream_t s)
{
    if (workgroups == 0 || (j.n_regions == 0 && j.kv_count == 0)) return hipSuccess;
    PSV_LAUNCH(k_prefetch, dim3(workgroups), dim3(256), 0, s, j);
    return hipGetLastError();
}

hipError_t launch_prefetch(const void *ptr, uint64_t bytes, uint32_t workgroups, hipStream_t s)
{
    if (bytes < 16) return hipSuccess;
    PrefetchJob j{};
    j.n_regions = 1;
    j.ptr[0] = ptr;
    j.n16[0] = bytes / 16;
    return launch_prefetch_job(j, workgroups, s);
}

// ------------------------------------------------------------------------------------ copy (counter calibration)

__global__ __launch_bounds__(256) void k_copy(uint4 *__restrict__ dst, const uint4 *__restrict__ src, uint64_t n16)
{
    const uint64_t stride = (uint64_t)gridDim.x * 256;
    for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

hipError_t launch_copy(void *dst, const void *src, uint64_t bytes, hipStream_t s)
{
    if (bytes < 16) return hipSuccess;
    uint64_t n16 = bytes / 16;
    uint64_t blocks = (n16 + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    PSV_LAUNCH(k_copy, dim3((unsigned)blocks), dim3(256), 0, s, reinterpret_cast<uint4 *>(dst),
                       reinterpret_cast<const uint4 *>(src), n16);
    return hipGetLastError();
}

}  // namespace psv

// Shared device-side pieces of the gfx950 kernels: the launch macro (with the optional per-dispatch events of
// the profiling mode), vector types, bf16 / int8 conversions, loads, reductions and cache addressing.  Included by
// every kernel file; everything here is inline.
#ifndef PSV_DEVICE_H
#define PSV_DEVICE_H

#include <hip/hip_ext.h>
#include <stdlib.h>

#include <type_traits>

#include "internal.h"

namespace psv {

// Optional events that the next kernel launch attaches to its own dispatch: `stop` is bound to the kernel
// command and carries its end timestamp; `start` is a marker ahead of it.  Used by the per-operator
// profiling of the API layer (set_launch_events).  One pair per host thread, shared by all kernel files.
inline thread_local hipEvent_t g_ev_start = nullptr, g_ev_stop = nullptr;

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

// float -> bf16, round to nearest even: the hardware conversion of gfx950 (one instruction per pair of values; the
// bit-twiddling version costs ~6 vector instructions per value, which showed in kernels that convert thousands).
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    const bf16x2_t v = __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t);
    return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ uint32_t f32_to_bf16(float f) { return pack_bf16(f, 0.f) & 0xffffu; }

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

// Sums over the 64 lanes of a wave of N values per lane at once (N = 2, 4, 8 or 16), scattered: lane l < N returns the
// total of v[scatter_index(l)].  Every step halves what a lane carries: it keeps the values of one class and adds its
// partner's partial sums of them, so the whole reduction costs ~4N + 10 vector instructions and two LDS-pipe shuffles
// instead of N times the eleven of wave_sum (measured on 16 values, beside the 16 dot products that produce them: 0.25 us
// instead of 1.0 us per workgroup of 8 waves).  The partners are those of wave_sum -- quad swaps, half-row and row
// mirrors, then the rows -- and the classes are chosen so that a partner always holds the class a lane keeps (the
// mirrors flip the low lane bits as well: class bit 0 = l0 ^ l2, bit 1 = l1 ^ l2, bit 2 = l2 ^ l3, bit 3 = l3).  Every
// total is summed in the same tree as wave_sum's, so the two give the same bits.  All lanes active.
template <int CTRL>
__device__ __forceinline__ float dpp_get(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
template <int K>
__device__ __forceinline__ float lane_partner(float v, int lane)
{
    if constexpr (K == 0) return dpp_get<0xB1>(v);          // quad_perm [1,0,3,2]
    else if constexpr (K == 1) return dpp_get<0x4E>(v);     // quad_perm [2,3,0,1]
    else if constexpr (K == 2) return dpp_get<0x141>(v);    // row_half_mirror
    else if constexpr (K == 3) return dpp_get<0x140>(v);    // row_mirror
    else if constexpr (K == 4) return __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(v), 0x401F));   // lane ^ 16
    else return __int_as_float(__builtin_amdgcn_ds_bpermute((lane ^ 32) << 2, __float_as_int(v)));
}
template <int N, int K>
__device__ __forceinline__ float wave_sum_scatter_step(const float (&cur)[N], int lane)
{
    if constexpr (N > 1) {
        float nxt[N / 2];
        const bool up = K == 0 ? ((lane ^ (lane >> 2)) & 1) : K == 1 ? (((lane >> 1) ^ (lane >> 2)) & 1)
                      : K == 2 ? (((lane >> 2) ^ (lane >> 3)) & 1) : ((lane >> 3) & 1);
#pragma unroll
        for (int m = 0; m < N / 2; ++m) {
            const float keep = up ? cur[2 * m + 1] : cur[2 * m], send = up ? cur[2 * m] : cur[2 * m + 1];
            nxt[m] = keep + lane_partner<K>(send, lane);
        }
        return wave_sum_scatter_step<N / 2, K + 1>(nxt, lane);
    } else {
        float v = cur[0];
        if constexpr (K <= 0) v += lane_partner<0>(v, lane);
        if constexpr (K <= 1) v += lane_partner<1>(v, lane);
        if constexpr (K <= 2) v += lane_partner<2>(v, lane);
        if constexpr (K <= 3) v += lane_partner<3>(v, lane);
        if constexpr (K <= 4) v += lane_partner<4>(v, lane);
        v += lane_partner<5>(v, lane);
        return v;
    }
}
template <int N>
__device__ __forceinline__ float wave_sum_scatter(const float (&v)[N], int lane)
{
    static_assert(N == 1 || N == 2 || N == 4 || N == 8 || N == 16, "one value per lane of a 16-lane row at most");
    return wave_sum_scatter_step<N, 0>(v, lane);
}
// Which of the N values lane l (any lane; lanes l < N are one holder of each) holds after wave_sum_scatter<N>.
template <int N>
__device__ __forceinline__ int scatter_index(int l)
{
    return (((l ^ (l >> 2)) & 1) | ((((l >> 1) ^ (l >> 2)) & 1) << 1) | ((((l >> 2) ^ (l >> 3)) & 1) << 2) | (((l >> 3) & 1) << 3)) & (N - 1);
}
// ... and the lane below N that holds value j.
__device__ __forceinline__ int scatter_holder(int j)
{
    const int l3 = (j >> 3) & 1, l2 = ((j >> 2) & 1) ^ l3, l1 = ((j >> 1) & 1) ^ l2, l0 = (j & 1) ^ l2;
    return l0 | (l1 << 1) | (l2 << 2) | (l3 << 3);
}

// Two values as a pair of packed bf16 words: hi = their bf16 roundings, lo = the bf16 roundings of what is left.
__device__ __forceinline__ void pack_split(float a, float b, uint32_t &hi, uint32_t &lo)
{
    hi = pack_bf16(a, b);
    lo = pack_bf16(a - bf16_lo(hi), b - bf16_hi(hi));
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
// WT: every store written through to the memory side (sc0 sc1), for a producer whose consumer is already running.
__device__ __forceinline__ void st_wt4(void *p, uint32_t v)
{
    asm volatile("global_store_dword %0, %1, off sc0 sc1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void st_wt8(void *p, uint2 v)
{
    typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));
    const u32x2_t w = {v.x, v.y};
    asm volatile("global_store_dwordx2 %0, %1, off sc0 sc1" ::"v"(p), "v"(w) : "memory");
}
__device__ __forceinline__ void st_wt16(void *p, float4 v)
{
    const f32x4 w = {v.x, v.y, v.z, v.w};
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" ::"v"(p), "v"(w) : "memory");
}
template <bool WT = false>
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
    float *sc = reinterpret_cast<float *>(base + 2 * plane) + row * (K / 128) + k0 / 128;
    if (WT) {
        st_wt4(p, pack_magic_bytes(a1[0], a1[1], a1[2], a1[3]));
        st_wt4(p + plane, pack_magic_bytes(a2[0], a2[1], a2[2], a2[3]));
        if ((threadIdx.x & 31) == 0) st_wt4(sc, __float_as_uint(amax / 127.0f));
    } else {
        *reinterpret_cast<uint32_t *>(p) = pack_magic_bytes(a1[0], a1[1], a1[2], a1[3]);
        *reinterpret_cast<uint32_t *>(p + plane) = pack_magic_bytes(a2[0], a2[1], a2[2], a2[3]);
        if ((threadIdx.x & 31) == 0) *sc = amax / 127.0f;
    }
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

// ------------------------------------------------------------------------------------ KV addressing

__device__ __forceinline__ int kv_phys_block(const int32_t *page_table, int max_blocks, int num_pool_blocks,
                                             int b, int logical)
{
    int idx = b * max_blocks + logical;
    int blk = page_table ? page_table[idx] : idx;
    return (blk >= 0 && blk < num_pool_blocks) ? blk : -1;   // a corrupt entry is skipped, never followed
}

}  // namespace psv

#endif

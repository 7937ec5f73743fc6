// Tagged values: the hand-over between the phases of a fused kernel (segment.hip, step.hip).  Every value travels with
// a tag in the same 8 bytes; producers store {value, tag} written through to the memory side, consumers poll the values
// themselves with device-coherent loads until every tag is the expected one.  No separate flag, no store that has to be
// acknowledged before a flag may follow.  Also the geometry of a projection inside such a kernel.
#ifndef PSV_TAGGED_H
#define PSV_TAGGED_H

#include "device.h"

namespace psv {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ void ll_store(uint2 *p, float v, unsigned tag)
{
    const uint2 w = make_uint2(__float_as_uint(v), tag);
    asm volatile("global_store_dwordx2 %0, %1, off sc0 sc1" ::"v"(p), "v"(w) : "memory");
}
// two {value, tag} pairs per 16-byte load
__device__ __forceinline__ void ll_issue(u32x4 &v, const uint2 *p)
{
    asm volatile("global_load_dwordx4 %0, %1, off sc0 sc1" : "=v"(v) : "v"(p) : "memory");
}
__device__ __forceinline__ void ll_wait4(u32x4 &a, u32x4 &b, u32x4 &c, u32x4 &d)
{
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : : "memory");
}

__device__ __forceinline__ void ll_issue1(uint2 &v, const uint2 *p)
{
    asm volatile("global_load_dwordx2 %0, %1, off sc0 sc1" : "=v"(v) : "v"(p) : "memory");
}
__device__ __forceinline__ void ll_wait_all() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Reads 8 consecutive tagged values (64 bytes) into x[0..7]; returns true when all eight carry `tag`.
__device__ __forceinline__ bool ll_read8(const uint2 *p, unsigned tag, float (&x)[8])
{
    u32x4 q0, q1, q2, q3;
    ll_issue(q0, p);
    ll_issue(q1, p + 2);
    ll_issue(q2, p + 4);
    ll_issue(q3, p + 6);
    ll_wait4(q0, q1, q2, q3);
    x[0] = __uint_as_float(q0.x); x[1] = __uint_as_float(q0.z);
    x[2] = __uint_as_float(q1.x); x[3] = __uint_as_float(q1.z);
    x[4] = __uint_as_float(q2.x); x[5] = __uint_as_float(q2.z);
    x[6] = __uint_as_float(q3.x); x[7] = __uint_as_float(q3.z);
    return q0.y == tag && q0.w == tag && q1.y == tag && q1.w == tag && q2.y == tag && q2.w == tag && q3.y == tag && q3.w == tag;
}

// Geometry of one projection inside a fused kernel: threads per weight row (GS = 1 << gs_log2) and passes of RB rows.
struct SegGeom {
    int gs_log2, passes;
};

// Threads per row and passes of a projection of N rows by K columns run by `blocks` workgroups of 512 threads.
inline SegGeom seg_geom(int N, int K, int iters, int rb, int blocks)
{
    SegGeom g;
    g.gs_log2 = 6;
    while ((8 << g.gs_log2) * iters < K && (1 << g.gs_log2) < 512) ++g.gs_log2;
    const long long slots = (long long)blocks * (512 >> g.gs_log2);
    const int max_rows = (int)((N + slots - 1) / slots);
    g.passes = (max_rows + rb - 1) / rb;
    if (g.passes < 1) g.passes = 1;
    return g;
}

}  // namespace psv

#endif

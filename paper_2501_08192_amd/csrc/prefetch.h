// The walk of the prefetch kernel as a device function: k_prefetch runs it with its own grid, and a projection that is
// launched into a communication window (the waiting variant of k_gemm_sk) runs it while it waits, with the window's job as an argument.
#ifndef PSV_PREFETCH_H
#define PSV_PREFETCH_H

#include "device.h"

namespace psv {

__device__ __forceinline__ uint32_t fold(uint4 v) { return v.x ^ v.y ^ v.z ^ v.w; }

// Reads memory with 16-byte loads and throws the data away: the loads allocate the lines in the
// memory-side cache (Infinity Cache).  Nothing is written.  One job serves a whole communication
// window: up to kPrefetchRegions linear regions (projection weights) plus a range of KV blocks that
// is walked through the page table.  Workgroup `wg` of `n_wg` workgroups of 256 threads takes its share;
// 16 x 16-byte loads are in flight per thread.
__device__ __forceinline__ void prefetch_walk(const PrefetchJob &j, uint64_t wg, uint64_t n_wg)
{
    constexpr int U = 16;
    if (j.skip && *j.skip) return;   // the gate kernel ahead of this launch found the window already over
    const uint64_t stride = n_wg * 256;
    const uint64_t me = wg * 256 + threadIdx.x;
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
        const uint64_t gw = wg * 4 + (threadIdx.x >> 6);
        const uint64_t nw = n_wg * 4;
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

}  // namespace psv

#endif

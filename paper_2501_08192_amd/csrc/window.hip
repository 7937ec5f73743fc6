// gfx950 (MI355X, CDNA4) kernels of the PRESERVE decode step: the communication-window stand-in, the gate, the prefetch kernel and the calibration copy.
//
// Weights and the KV-cache are bf16 (or int8 codes with fp32 scales) in HBM; every accumulation is fp32.  The step
// is bound by HBM bandwidth (Section 2, "LLM decoding is memory BW-limited"), so the kernels are built around
// 16-byte-per-lane coalesced loads with many loads in flight per 64-lane wave; the matrix cores are used where a
// vector-ALU formulation would bind on arithmetic (batch > 2 projections, grouped-query attention).
#include "device.h"
#include "prefetch.h"

namespace psv {

void set_launch_events(hipEvent_t start, hipEvent_t stop)
{
    g_ev_start = start;
    g_ev_stop = stop;
}

// ------------------------------------------------------------------------------------ spin window

// One workgroup of one wave busy-waits on the constant-rate wall clock; the iteration cap makes
// sure the wave exits even if the clock misbehaves.  On entry it publishes the window's sequence
// number: a gate kernel (k_gate) is already waiting for it on the side stream, ahead of the window's
// prefetch launches (a device-side fork, no host event in between).
// On exit it publishes the same number in *done: a consumer kernel that was launched ahead of time on the other
// stream and has already pulled its weights into registers waits for exactly that (k_gemv).  A relaxed store: the
// stand-in writes no data that the word would have to order (a release here wrote back the XCD's L2 first and made every
// window 0.3 us longer than asked for).
__global__ __launch_bounds__(64) void k_spin(uint64_t ticks, uint32_t max_iters, unsigned *flag, unsigned *done, unsigned seq)
{
    const uint64_t t0 = wall_clock64();
    if (flag && threadIdx.x == 0) __hip_atomic_store(flag, seq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    uint32_t it = 0;
    while (wall_clock64() - t0 < ticks && it < max_iters) {
        __builtin_amdgcn_s_sleep(2);
        ++it;
    }
    if (done && threadIdx.x == 0) __hip_atomic_store(done, seq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

hipError_t launch_spin(uint64_t ticks, uint32_t max_iters, unsigned *flag, unsigned *done, unsigned seq, hipStream_t s)
{
    PSV_LAUNCH(k_spin, dim3(1), dim3(64), 0, s, ticks, max_iters, flag, done, seq);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------ prefetch

// The prefetch kernel: the walk of prefetch.h over a grid of its own.  The grid size is the CU budget of the policy.
__global__ __launch_bounds__(256) void k_prefetch(PrefetchJob j)
{
    prefetch_walk(j, blockIdx.x, gridDim.x);
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

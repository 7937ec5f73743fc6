// psv_decode_step_static: the decode step for callers that cannot allocate device memory.
//
// psv_create allocates the step's workspace (activations between the kernels, rotary table, attention and split-K
// partials) with hipMalloc.  This entry point runs the same kernels on a workspace that lives in a file-scope device
// array instead, so that it allocates nothing: no device memory, no streams, no events.  Every GPU the library runs
// on holds its own copy of the array, at its own address, until the process ends; the address is looked up once per
// device and handed to the kernels as an ordinary pointer.
#include <math.h>

#include <vector>

#include "context.h"

static __device__ __align__(256) unsigned char scratch[PSV_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each device (null: not looked up yet)

// The 64 rotary frequencies arrive as a kernel argument and are stored by the kernel: no host-to-device copy.
struct FreqTable {
    double f[64];
};
__global__ __launch_bounds__(64) void k_store_freq(FreqTable t, double *dst) { dst[threadIdx.x] = t.f[threadIdx.x]; }

}  // namespace

extern "C" psv_status psv_decode_step_static(const psv_model_desc *desc, const psv_layer_weights *layers,
                                             const psv_kv_desc *kv, const float *x_in, float *x_out, uint32_t batch,
                                             uint32_t layer_begin, uint32_t layer_end, void *stream)
{
    using namespace psv;
    if (!desc || !layers || !kv || !x_in || !x_out) return PSV_ERR_INVALID_ARG;
    if (psv_validate_desc(desc) != PSV_OK) return PSV_ERR_INVALID_ARG;
    if (batch == 0 || batch > desc->max_batch || layer_begin >= layer_end || layer_end > desc->n_layers) return PSV_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(x_in) % 16 || reinterpret_cast<uintptr_t>(x_out) % 16) return PSV_ERR_INVALID_ARG;
    const Workspace ws = layout_workspace(*desc);
    if (ws.total > (size_t)PSV_STATIC_SCRATCH_BYTES) return PSV_ERR_UNSUPPORTED;   // the shape needs more than the fixed array holds

    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return PSV_ERR_UNSUPPORTED;
    if (!g_scratch_ptr[dev]) {
        // In host code the array's name is only a handle for the symbol: its address on the current device has to be
        // asked for, once per device.
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PSV_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }

    // A context on the stack, filled through the same setters (and therefore the same argument checks) as a created one.
    psv_ctx c;
    c.d = *desc;
    c.main = static_cast<hipStream_t>(stream);
    c.side = nullptr;                       // never used: no windows, no prefetch
    c.device = dev;
    if (hipDeviceGetAttribute(&c.cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) c.cus = 0;
    c.ws = ws;
    c.wsp = static_cast<char *>(g_scratch_ptr[dev]);
    c.weights.resize(desc->n_layers);
    c.weights_set.assign(desc->n_layers, 0);
    c.k_pools.assign(desc->n_layers, nullptr);
    c.v_pools.assign(desc->n_layers, nullptr);
    c.policy.mode = 0;
    c.fused = 0;                            // one kernel per operator: nothing here reads the error word of a fused kernel
    for (uint32_t l = layer_begin; l < layer_end; ++l) ST_TRY(psv_set_layer_weights(&c, l, &layers[l]));
    {
        // layers outside the range are not run; psv_set_kv wants a pool pointer for every layer
        std::vector<void *> kp(desc->n_layers, kv->k_pools ? kv->k_pools[layer_begin] : nullptr);
        std::vector<void *> vp(desc->n_layers, kv->v_pools ? kv->v_pools[layer_begin] : nullptr);
        for (uint32_t l = layer_begin; l < layer_end && kv->k_pools && kv->v_pools; ++l) {
            kp[l] = kv->k_pools[l];
            vp[l] = kv->v_pools[l];
        }
        psv_kv_desc k2 = *kv;
        k2.k_pools = kp.data();
        k2.v_pools = vp.data();
        ST_TRY(psv_set_kv(&c, &k2));
    }
    if (desc->rope_theta > 0.f) {
        FreqTable t;
        for (int i = 0; i < 64; ++i) t.f[i] = pow((double)desc->rope_theta, -2.0 * (double)i / 128.0);
        hipLaunchKernelGGL(k_store_freq, dim3(1), dim3(64), 0, c.main, t, c.at<double>(ws.inv_freq));
        HIP_TRY(hipGetLastError());
    }
    // Nothing in the workspace has to start at zero for a step without windows: every buffer is written by the step
    // before it is read (the flag words of the window fork are not used here), so the previous call's contents --
    // of this or any other shape -- are simply overwritten.
    return enqueue_step(&c, x_in, x_out, batch, layer_begin, layer_end);
}

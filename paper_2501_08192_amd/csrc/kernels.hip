// gfx950 (MI355X, CDNA4) kernels of the PRESERVE decode step.
//
// All weights and the KV-cache are bf16 in HBM; every accumulation is fp32.  The step is bound
// by HBM bandwidth (Section 2, "LLM decoding is memory BW-limited"), so the kernels are built
// around 16-byte-per-lane coalesced loads with many loads in flight per 64-lane wave; matrix
// cores (16x16x32 bf16 MFMA) are used where a vector-ALU formulation would bind on arithmetic
// (batch > 4 projections, grouped-query attention).
#include "internal.h"

namespace psv {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

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

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__device__ __forceinline__ uint4 ld16(const uint16_t *p) { return *reinterpret_cast<const uint4 *>(p); }
__device__ __forceinline__ uint4 zero16() { return make_uint4(0u, 0u, 0u, 0u); }

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

__device__ __forceinline__ float silu_mul(float g, float u) { return g / (1.0f + expf(-g)) * u; }

// ------------------------------------------------------------------------------------ norm

// out_res = res + delta; h = out_res * rsqrt(mean(out_res^2) + eps) * gain.  One workgroup per
// batch row; the row is re-read from out_res for the second pass (each thread re-reads only what
// it wrote itself).
__global__ __launch_bounds__(256) void k_add_rmsnorm(const float *__restrict__ res,
                                                     const float *__restrict__ delta,
                                                     const uint16_t *__restrict__ gain, float eps, int H,
                                                     float *out_res, float *__restrict__ h_f32,
                                                     uint16_t *__restrict__ h_bf16)
{
    __shared__ float red[4];
    const int b = blockIdx.x, tid = threadIdx.x;
    const float *r = res + (size_t)b * H;
    const float *d = delta ? delta + (size_t)b * H : nullptr;
    float *o = out_res + (size_t)b * H;
    float ss = 0.f;
    for (int i = tid * 4; i < H; i += 1024) {
        float4 v = *reinterpret_cast<const float4 *>(r + i);
        if (d) {
            float4 e = *reinterpret_cast<const float4 *>(d + i);
            v.x += e.x; v.y += e.y; v.z += e.z; v.w += e.w;
        }
        *reinterpret_cast<float4 *>(o + i) = v;
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
    if (!gain) return;
    ss = wave_sum(ss);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    ss = red[0] + red[1] + red[2] + red[3];
    const float inv = 1.0f / sqrtf(ss / (float)H + eps);
    for (int i = tid * 4; i < H; i += 1024) {
        float4 v = *reinterpret_cast<const float4 *>(o + i);
        uint2 g = *reinterpret_cast<const uint2 *>(gain + i);
        v.x = v.x * inv * bf16_lo(g.x);
        v.y = v.y * inv * bf16_hi(g.x);
        v.z = v.z * inv * bf16_lo(g.y);
        v.w = v.w * inv * bf16_hi(g.y);
        *reinterpret_cast<float4 *>(h_f32 + (size_t)b * H + i) = v;
        uint2 pk = make_uint2(pack_bf16(v.x, v.y), pack_bf16(v.z, v.w));
        *reinterpret_cast<uint2 *>(h_bf16 + (size_t)b * H + i) = pk;
    }
}

hipError_t launch_add_rmsnorm(const float *res, const float *delta, const uint16_t *gain, float eps,
                              int batch, int H, float *out_res, float *h_f32, uint16_t *h_bf16,
                              hipStream_t s)
{
    hipLaunchKernelGGL(k_add_rmsnorm, dim3(batch), dim3(256), 0, s, res, delta, gain, eps, H, out_res,
                       h_f32, h_bf16);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------ GEMV

// Weight-streaming GEMV on the vector ALU (batch NB <= 4).  A wave owns R output rows at a time
// and walks them along K in 1 KiB steps (64 lanes x 16 bytes, fully coalesced); U steps are
// issued back to back so that U*R (2*U*R with SwiGLU) 16-byte loads are in flight per lane.  The
// activations sit in LDS as fp32.  A 64-lane butterfly finishes each row; no atomics, fixed order.
template <int NB, int R, bool SWIGLU>
__global__ __launch_bounds__(256) void k_gemv(const uint16_t *__restrict__ W, const uint16_t *__restrict__ W2,
                                              const float *__restrict__ x, float *__restrict__ out,
                                              uint16_t *__restrict__ out_bf16, int N, int K)
{
    constexpr int U = 4;
    constexpr int NW = SWIGLU ? 2 : 1;
    extern __shared__ float xs[];   // [NB][K]
    const int tid = threadIdx.x;
    for (int i = tid * 4; i < NB * K; i += 1024)
        *reinterpret_cast<float4 *>(xs + i) = *reinterpret_cast<const float4 *>(x + i);
    __syncthreads();

    const int lane = tid & 63;
    const int gw = blockIdx.x * 4 + (tid >> 6);
    const int nw = gridDim.x * 4;
    for (int row0 = gw * R; row0 < N; row0 += nw * R) {
        float acc[NW][R][NB];
#pragma unroll
        for (int a = 0; a < NW; ++a)
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int b = 0; b < NB; ++b) acc[a][r][b] = 0.f;

        for (int k0 = lane * 8; k0 < K; k0 += 512 * U) {
            uint4 wv[U][NW][R];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int kk = k0 + u * 512;
                const bool ok = kk < K;
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    wv[u][0][r] = ok ? ld16(W + (size_t)(row0 + r) * K + kk) : zero16();
                    if (SWIGLU) wv[u][NW - 1][r] = ok ? ld16(W2 + (size_t)(row0 + r) * K + kk) : zero16();
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int kk = k0 + u * 512;
                if (kk < K) {
#pragma unroll
                    for (int b = 0; b < NB; ++b) {
                        float xv[8];
                        float4 x0 = *reinterpret_cast<const float4 *>(xs + b * K + kk);
                        float4 x1 = *reinterpret_cast<const float4 *>(xs + b * K + kk + 4);
                        xv[0] = x0.x; xv[1] = x0.y; xv[2] = x0.z; xv[3] = x0.w;
                        xv[4] = x1.x; xv[5] = x1.y; xv[6] = x1.z; xv[7] = x1.w;
#pragma unroll
                        for (int a = 0; a < NW; ++a)
#pragma unroll
                            for (int r = 0; r < R; ++r) acc[a][r][b] = dot8(wv[u][a][r], xv, acc[a][r][b]);
                    }
                }
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                float v = wave_sum(acc[0][r][b]);
                if (SWIGLU) {
                    float u = wave_sum(acc[NW - 1][r][b]);
                    v = silu_mul(v, u);
                }
                if (lane == 0) {
                    out[(size_t)b * N + row0 + r] = v;
                    if (out_bf16) out_bf16[(size_t)b * N + row0 + r] = (uint16_t)f32_to_bf16(v);
                }
            }
    }
}

bool gemv_supported(int batch, int N, int K)
{
    return batch >= 1 && batch <= 4 && K % 256 == 0 && N % 2 == 0 && (size_t)batch * K * 4 <= 64 * 1024;
}

template <int NB, int R, bool SW>
static hipError_t gemv_go(const uint16_t *W, const uint16_t *W2, const float *x, float *out,
                          uint16_t *out_bf16, int N, int K, int blocks, hipStream_t s)
{
    hipLaunchKernelGGL((k_gemv<NB, R, SW>), dim3(blocks), dim3(256), (size_t)NB * K * sizeof(float), s, W, W2,
                       x, out, out_bf16, N, K);
    return hipGetLastError();
}

template <int NB>
static hipError_t gemv_pick(const uint16_t *W, const uint16_t *W2, const float *x, float *out,
                            uint16_t *out_bf16, int N, int K, hipStream_t s)
{
    // Two rows per wave once there are enough rows to give every one of 2048 waves work.
    const bool sw = W2 != nullptr;
    const int R = (!sw && N >= 4096) ? 2 : 1;
    int waves = N / R;
    int blocks = (waves + 3) / 4;
    if (blocks > 1024) blocks = 1024;
    if (sw) return gemv_go<NB, 1, true>(W, W2, x, out, out_bf16, N, K, blocks, s);
    if (R == 2) return gemv_go<NB, 2, false>(W, W2, x, out, out_bf16, N, K, blocks, s);
    return gemv_go<NB, 1, false>(W, W2, x, out, out_bf16, N, K, blocks, s);
}

hipError_t launch_gemv(const uint16_t *W, const uint16_t *W2, const float *x, float *out,
                       uint16_t *out_bf16, int batch, int N, int K, hipStream_t s)
{
    switch (batch) {
    case 1: return gemv_pick<1>(W, W2, x, out, out_bf16, N, K, s);
    case 2: return gemv_pick<2>(W, W2, x, out, out_bf16, N, K, s);
    case 3: return gemv_pick<3>(W, W2, x, out, out_bf16, N, K, s);
    case 4: return gemv_pick<4>(W, W2, x, out, out_bf16, N, K, s);
    default: return hipErrorInvalidValue;
    }
}

// ------------------------------------------------------------------------------------ MFMA skinny GEMM

// out[b][r] = sum_k W[r][k] x[b][k] with v_mfma_f32_16x16x32_bf16: the 16 rows of a weight tile
// are the M side, 16 batch entries the N side.  The waves of a workgroup split K between them in
// interleaved 64-element slices; every lane loads 32 contiguous bytes per row and slice (so a wave
// touches whole 128-byte lines of 16 rows) and feeds them to two MFMAs.  Because A and B fragments
// use the same (lane group, element) -> k mapping, the order of k inside a slice does not matter.
// Partial tiles are summed through LDS in wave order (deterministic).
template <int NB, int NWAVES, bool SWIGLU>
__global__ __launch_bounds__(NWAVES * 64) void k_gemm_mfma(const uint16_t *__restrict__ W,
                                                            const uint16_t *__restrict__ W2,
                                                            const uint16_t *__restrict__ xb,
                                                            float *__restrict__ out,
                                                            uint16_t *__restrict__ out_bf16, int batch, int N, int K)
{
    constexpr int NW = SWIGLU ? 2 : 1;
    __shared__ f32x4 red[NWAVES][NW][NB][64];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int row0 = blockIdx.x * 16;

    f32x4 acc[NW][NB];
#pragma unroll
    for (int a = 0; a < NW; ++a)
#pragma unroll
        for (int n = 0; n < NB; ++n) acc[a][n] = f32x4{0.f, 0.f, 0.f, 0.f};

    const uint16_t *wrow = W + (size_t)(row0 + i) * K + g * 16;
    const uint16_t *w2row = SWIGLU ? W2 + (size_t)(row0 + i) * K + g * 16 : nullptr;
    const uint16_t *xrow = xb + (size_t)i * K + g * 16;

    for (int kb = w * 64; kb < K; kb += NWAVES * 64) {
        uint4 a0[NW], a1[NW], b0[NB], b1[NB];
        a0[0] = ld16(wrow + kb);
        a1[0] = ld16(wrow + kb + 8);
        if (SWIGLU) {
            a0[NW - 1] = ld16(w2row + kb);
            a1[NW - 1] = ld16(w2row + kb + 8);
        }
#pragma unroll
        for (int n = 0; n < NB; ++n) {
            b0[n] = ld16(xrow + (size_t)n * 16 * K + kb);
            b1[n] = ld16(xrow + (size_t)n * 16 * K + kb + 8);
        }
#pragma unroll
        for (int a = 0; a < NW; ++a)
#pragma unroll
            for (int n = 0; n < NB; ++n) {
                acc[a][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a0[a]),
                                                                    __builtin_bit_cast(bf16x8, b0[n]), acc[a][n], 0, 0, 0);
                acc[a][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a1[a]),
                                                                    __builtin_bit_cast(bf16x8, b1[n]), acc[a][n], 0, 0, 0);
            }
    }
#pragma unroll
    for (int a = 0; a < NW; ++a)
#pragma unroll
        for (int n = 0; n < NB; ++n) red[w][a][n][lane] = acc[a][n];
    __syncthreads();

    // D fragment: lane holds rows 4g..4g+3 of column i  ->  out[batch n*16+i][row0 + 4g + j]
    for (int n = w; n < NB; n += NWAVES) {
        f32x4 v = red[0][0][n][lane];
#pragma unroll
        for (int ww = 1; ww < NWAVES; ++ww) v += red[ww][0][n][lane];
        if (SWIGLU) {
            f32x4 u = red[0][NW - 1][n][lane];
#pragma unroll
            for (int ww = 1; ww < NWAVES; ++ww) u += red[ww][NW - 1][n][lane];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = silu_mul(v[j], u[j]);
        }
        const int b = n * 16 + i;
        if (b < batch) {
            const size_t o = (size_t)b * N + row0 + 4 * g;
            *reinterpret_cast<float4 *>(out + o) = make_float4(v[0], v[1], v[2], v[3]);
            if (out_bf16)
                *reinterpret_cast<uint2 *>(out_bf16 + o) = make_uint2(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]));
        }
    }
}

bool gemm_mfma_supported(int batch, int N, int K)
{
    return batch >= 1 && batch <= 64 && N % 16 == 0 && K % 64 == 0;
}

template <int NB, int NWAVES>
static hipError_t gemm_go(const uint16_t *W, const uint16_t *W2, const uint16_t *xb, float *out,
                          uint16_t *out_bf16, int batch, int N, int K, hipStream_t s)
{
    if (W2)
        hipLaunchKernelGGL((k_gemm_mfma<NB, NWAVES, true>), dim3(N / 16), dim3(NWAVES * 64), 0, s, W, W2, xb, out,
                           out_bf16, batch, N, K);
    else
        hipLaunchKernelGGL((k_gemm_mfma<NB, NWAVES, false>), dim3(N / 16), dim3(NWAVES * 64), 0, s, W, W2, xb, out,
                           out_bf16, batch, N, K);
    return hipGetLastError();
}

hipError_t launch_gemm_mfma(const uint16_t *W, const uint16_t *W2, const uint16_t *xb, float *out,
                            uint16_t *out_bf16, int batch, int N, int K, hipStream_t s)
{
    const int nb = (batch + 15) / 16;
    // Few row tiles (a narrow projection): 8 waves per workgroup split K further so that the
    // launch still puts >= 2 waves on every SIMD of the chip.
    const bool wide = (N / 16) < 1024;
    switch (nb) {
    case 1: return wide ? gemm_go<1, 8>(W, W2, xb, out, out_bf16, batch, N, K, s) : gemm_go<1, 4>(W, W2, xb, out, out_bf16, batch, N, K, s);
    case 2: return wide ? gemm_go<2, 8>(W, W2, xb, out, out_bf16, batch, N, K, s) : gemm_go<2, 4>(W, W2, xb, out, out_bf16, batch, N, K, s);
    case 3: return wide ? gemm_go<3, 8>(W, W2, xb, out, out_bf16, batch, N, K, s) : gemm_go<3, 4>(W, W2, xb, out, out_bf16, batch, N, K, s);
    case 4: return wide ? gemm_go<4, 8>(W, W2, xb, out, out_bf16, batch, N, K, s) : gemm_go<4, 4>(W, W2, xb, out, out_bf16, batch, N, K, s);
    default: return hipErrorInvalidValue;
    }
}

// ------------------------------------------------------------------------------------ KV addressing

__device__ __forceinline__ int kv_phys_block(const int32_t *page_table, int max_blocks, int num_pool_blocks,
                                             int b, int logical)
{
    int idx = b * max_blocks + logical;
    int blk = page_table ? page_table[idx] : idx;
    return (blk >= 0 && blk < num_pool_blocks) ? blk : -1;   // a corrupt entry is skipped, never followed
}

// ------------------------------------------------------------------------------------ RoPE + append

// grid (nq + nkv, batch), 64 threads: thread i rotates the pair (i, i+64) of one head.  Angles are
// formed in double (position * theta^(-2i/128)) so that long contexts lose nothing to fp32 range
// reduction.  q heads go to a bf16 staging buffer; k heads (rotated) and the matching v heads are
// rounded to bf16 and stored in slot seq_len-1 of the pools.
__global__ __launch_bounds__(64) void k_rope_append(const float *__restrict__ qkv, const double *__restrict__ inv_freq,
                                                    KvView kv, int nq, int nkv, uint16_t *__restrict__ q_bf16)
{
    const int hh = blockIdx.x, b = blockIdx.y, i = threadIdx.x;
    const int qkv_rows = (nq + 2 * nkv) * 128;
    int T = kv.seq_lens[b];
    if (T < 1 || T > kv.max_blocks * 16) return;
    const int pos = T - 1;
    float c = 1.f, sn = 0.f;
    if (inv_freq) {
        double sd, cd;
        sincos((double)pos * inv_freq[i], &sd, &cd);
        c = (float)cd;
        sn = (float)sd;
    }
    const float *row = qkv + (size_t)b * qkv_rows + (size_t)hh * 128;
    const float a = row[i], bb = row[i + 64];
    const float ra = a * c - bb * sn, rb = bb * c + a * sn;
    if (hh < nq) {
        uint16_t *q = q_bf16 + ((size_t)b * nq + hh) * 128;
        q[i] = (uint16_t)f32_to_bf16(ra);
        q[i + 64] = (uint16_t)f32_to_bf16(rb);
        return;
    }
    const int kvh = hh - nq;
    const int blk = kv_phys_block(kv.page_table, kv.max_blocks, kv.num_pool_blocks, b, pos >> 4);
    if (blk < 0) return;
    const int r = pos & 15;
    uint16_t *kdst = kv.k_pool + (((size_t)blk * nkv + kvh) * 16 + r) * 128;
    kdst[i] = (uint16_t)f32_to_bf16(ra);
    kdst[i + 64] = (uint16_t)f32_to_bf16(rb);
    const float *vrow = qkv + (size_t)b * qkv_rows + (size_t)(nq + nkv + kvh) * 128;
    uint16_t *vdst = kv.v_pool + ((size_t)blk * nkv + kvh) * 128 * 16 + r;
    vdst[(size_t)i * 16] = (uint16_t)f32_to_bf16(vrow[i]);
    vdst[(size_t)(i + 64) * 16] = (uint16_t)f32_to_bf16(vrow[i + 64]);
}

hipError_t launch_rope_append(const float *qkv, const double *inv_freq, KvView kv, int batch, int nq,
                              int nkv, uint16_t *q_bf16, hipStream_t s)
{
    hipLaunchKernelGGL(k_rope_append, dim3(nq + nkv, batch), dim3(64), 0, s, qkv, inv_freq, kv, nq, nkv, q_bf16);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------ decode attention

AttnSplit attn_split(uint32_t batch, uint32_t n_kv_heads, uint32_t max_seq)
{
    // Aim at ~4096 waves over the whole launch, at least one 32-token tile per wave.
    uint64_t tiles = (uint64_t)batch * n_kv_heads * ((max_seq + kAttnTileTokens - 1) / kAttnTileTokens);
    uint64_t per_wave = (tiles + 4095) / 4096;
    if (per_wave < 1) per_wave = 1;
    AttnSplit sp;
    sp.chunk_tokens = (int)(per_wave * kAttnTileTokens * kAttnWaves);
    sp.n_chunks = (int)((max_seq + sp.chunk_tokens - 1) / sp.chunk_tokens);
    if (sp.n_chunks < 1) sp.n_chunks = 1;
    sp.n_splits = sp.n_chunks * kAttnWaves;
    return sp;
}

// Split-K decode attention, grouped-query aware.  grid (chunks, kv heads, batch), 4 waves; wave w
// of chunk c takes the 32-token tiles c*chunk + (w + 4*it)*32.  All G <= 16 query heads that share
// the kv head ride in the N side of the MFMAs, so K and V are read from HBM exactly once.
//
//   S^T[token][g]  = K[token][:] . Q[g][:]      A = K rows (token-major in the pool)
//   O^T[chan][g]  += V^T[chan][token] P[g][token]   A = V^T rows (channel-major in the pool)
//
// Tile 1 of a 32-token group covers tokens {8q+0..3}, tile 2 tokens {8q+4..7} (q = 0..3), so that
// after the two S^T MFMAs lane (g, q) holds the scores of the 8 consecutive tokens 8q..8q+7 of its
// query head: exactly the B-fragment the O^T MFMA needs.  Probabilities never leave registers.
__global__ __launch_bounds__(256) void k_attn_partial(const uint16_t *__restrict__ q_bf16, KvView kv, int nq, int nkv,
                                                      int chunk_tokens, int n_splits,
                                                      float *__restrict__ part_ml, float *__restrict__ part_o)
{
    const int b = blockIdx.z, kvh = blockIdx.y, c = blockIdx.x;
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63, i = lane & 15, q4 = lane >> 4;
    const int G = nq / nkv;
    int T = kv.seq_lens[b];
    if (T < 0 || T > kv.max_blocks * 16) T = 0;
    const int t_begin = c * chunk_tokens;
    const int t_end = min(T, t_begin + chunk_tokens);
    const int n_valid_blocks = (T + 15) >> 4;

    bf16x8 qf[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        uint4 v = zero16();
        if (i < G) v = ld16(q_bf16 + ((size_t)b * nq + kvh * G + i) * 128 + ks * 32 + q4 * 8);
        qf[ks] = __builtin_bit_cast(bf16x8, v);
    }

    const float kScale = 0.08838834764831845f * 1.4426950408889634f;   // 1/sqrt(128) * log2(e)
    float m_run = -1.0e30f, l_part = 0.f;
    f32x4 acc[8];
#pragma unroll
    for (int dg = 0; dg < 8; ++dg) acc[dg] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int tau1 = 8 * (i >> 2) + (i & 3);          // token (within the 32-token group) of K row i, tile 1
    for (int t0 = t_begin + w * kAttnTileTokens; t0 < t_end; t0 += kAttnWaves * kAttnTileTokens) {
        const int lb = t0 >> 4;
        const int blkA = kv_phys_block(kv.page_table, kv.max_blocks, kv.num_pool_blocks, b, lb);
        const int blkB = (lb + 1 < n_valid_blocks)
                             ? kv_phys_block(kv.page_table, kv.max_blocks, kv.num_pool_blocks, b, lb + 1) : -1;
        // K fragments: tile 1 row i = token tau1, tile 2 row i = token tau1 + 4
        uint4 ka[4], kb[4];
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
        uint4 vf[8];
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

    l_part += __shfl_xor(l_part, 16, 64);
    l_part += __shfl_xor(l_part, 32, 64);

    if (i < G) {
        const int sp = c * kAttnWaves + w;
        const size_t slot = ((size_t)b * nkv + kvh) * n_splits + sp;
        if (q4 == 0) {
            part_ml[(slot * 16 + i) * 2 + 0] = m_run;
            part_ml[(slot * 16 + i) * 2 + 1] = l_part;
        }
        float *o = part_o + (slot * G + i) * 128 + 4 * q4;
#pragma unroll
        for (int dg = 0; dg < 8; ++dg)
            *reinterpret_cast<float4 *>(o + dg * 16) = make_float4(acc[dg][0], acc[dg][1], acc[dg][2], acc[dg][3]);
    }
}

hipError_t launch_attn_partial(const uint16_t *q_bf16, KvView kv, int batch, int nq, int nkv, AttnSplit sp,
                               float *part_ml, float *part_o, hipStream_t s)
{
    hipLaunchKernelGGL(k_attn_partial, dim3(sp.n_chunks, nkv, batch), dim3(256), 0, s, q_bf16, kv, nq, nkv,
                       sp.chunk_tokens, sp.n_splits, part_ml, part_o);
    return hipGetLastError();
}

// Fixed-order combine of the per-wave partials: grid (nq, batch), 128 threads = 128 channels.
__global__ __launch_bounds__(128) void k_attn_combine(const float *__restrict__ part_ml, const float *__restrict__ part_o,
                                                      int nq, int nkv, int n_splits, float *__restrict__ out_f32,
                                                      uint16_t *__restrict__ out_bf16)
{
    const int h = blockIdx.x, b = blockIdx.y, ch = threadIdx.x;
    const int G = nq / nkv, kvh = h / G, g = h % G;
    const size_t slot0 = ((size_t)b * nkv + kvh) * n_splits;
    float M = -1.0e30f;
    for (int sp = 0; sp < n_splits; ++sp) M = fmaxf(M, part_ml[((slot0 + sp) * 16 + g) * 2]);
    float den = 0.f, num = 0.f;
    for (int sp = 0; sp < n_splits; ++sp) {
        const float m = part_ml[((slot0 + sp) * 16 + g) * 2];
        const float l = part_ml[((slot0 + sp) * 16 + g) * 2 + 1];
        if (l > 0.f) {
            const float wgt = exp2f(m - M);
            den += wgt * l;
            num += wgt * part_o[((slot0 + sp) * G + g) * 128 + ch];
        }
    }
    const float o = den > 0.f ? num / den : 0.f;
    const size_t idx = ((size_t)b * nq + h) * 128 + ch;
    out_f32[idx] = o;
    out_bf16[idx] = (uint16_t)f32_to_bf16(o);
}

hipError_t launch_attn_combine(const float *part_ml, const float *part_o, int batch, int nq, int nkv, AttnSplit sp,
                               float *out_f32, uint16_t *out_bf16, hipStream_t s)
{
    hipLaunchKernelGGL(k_attn_combine, dim3(nq, batch), dim3(128), 0, s, part_ml, part_o, nq, nkv, sp.n_splits,
                       out_f32, out_bf16);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------ spin window

// One workgroup of one wave busy-waits on the constant-rate wall clock; the iteration cap makes
// sure the wave exits even if the clock misbehaves.
__global__ __launch_bounds__(64) void k_spin(uint64_t ticks, uint32_t max_iters)
{
    const uint64_t t0 = wall_clock64();
    uint32_t it = 0;
    while (wall_clock64() - t0 < ticks && it < max_iters) {
        __builtin_amdgcn_s_sleep(2);
        ++it;
    }
}

hipError_t launch_spin(uint64_t ticks, uint32_t max_iters, hipStream_t s)
{
    hipLaunchKernelGGL(k_spin, dim3(1), dim3(64), 0, s, ticks, max_iters);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------ prefetch

// Reads a region with 16-byte loads and throws the data away: the loads allocate the lines in the
// memory-side cache (and in the L2 of the XCD that ran the workgroup).  Nothing is written.
__global__ __launch_bounds__(256) void k_prefetch(const uint4 *__restrict__ p, uint64_t n16)
{
    constexpr int U = 8;
    const uint64_t stride = (uint64_t)gridDim.x * 256;
    uint32_t sink = 0;
    uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + (U - 1) * stride < n16; i += U * stride) {
        uint4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = p[i + u * stride];
#pragma unroll
        for (int u = 0; u < U; ++u) sink ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < n16; i += stride) {
        uint4 v = p[i];
        sink ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    asm volatile("" ::"v"(sink));   // keeps the loads alive without a store
}

hipError_t launch_prefetch(const void *ptr, uint64_t bytes, uint32_t workgroups, hipStream_t s)
{
    if (bytes < 16 || workgroups == 0) return hipSuccess;
    hipLaunchKernelGGL(k_prefetch, dim3(workgroups), dim3(256), 0, s, reinterpret_cast<const uint4 *>(ptr), bytes / 16);
    return hipGetLastError();
}

// KV prefetch: one wave per logical block (K part and V part of every kv head, 4 KiB each per head).
__global__ __launch_bounds__(256) void k_prefetch_kv(KvView kv, int nkv, uint32_t blocks_per_seq, uint64_t first,
                                                     uint64_t count)
{
    const int lane = threadIdx.x & 63;
    const uint64_t gw = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const uint64_t nw = (uint64_t)gridDim.x * 4;
    const uint32_t per_block16 = (uint32_t)nkv * 16 * 128 * 2 / 16;   // 16-byte words per pool block
    uint32_t sink = 0;
    for (uint64_t j = gw; j < count; j += nw) {
        const uint64_t lin = first + j;
        const int b = (int)(lin / blocks_per_seq), lb = (int)(lin % blocks_per_seq);
        if (lb >= kv.max_blocks) continue;
        const int blk = kv_phys_block(kv.page_table, kv.max_blocks, kv.num_pool_blocks, b, lb);
        if (blk < 0) continue;
        const uint4 *kp = reinterpret_cast<const uint4 *>(kv.k_pool) + (size_t)blk * per_block16;
        const uint4 *vp = reinterpret_cast<const uint4 *>(kv.v_pool) + (size_t)blk * per_block16;
        for (uint32_t o = lane; o < per_block16; o += 256) {
            uint4 a0 = kp[o], a1 = (o + 64 < per_block16) ? kp[o + 64] : zero16();
            uint4 a2 = (o + 128 < per_block16) ? kp[o + 128] : zero16(), a3 = (o + 192 < per_block16) ? kp[o + 192] : zero16();
            uint4 b0 = vp[o], b1 = (o + 64 < per_block16) ? vp[o + 64] : zero16();
            uint4 b2 = (o + 128 < per_block16) ? vp[o + 128] : zero16(), b3 = (o + 192 < per_block16) ? vp[o + 192] : zero16();
            sink ^= a0.x ^ a1.x ^ a2.x ^ a3.x ^ b0.x ^ b1.x ^ b2.x ^ b3.x;
            sink ^= a0.y ^ a1.y ^ a2.y ^ a3.y ^ b0.y ^ b1.y ^ b2.y ^ b3.y;
            sink ^= a0.z ^ a1.z ^ a2.z ^ a3.z ^ b0.z ^ b1.z ^ b2.z ^ b3.z;
            sink ^= a0.w ^ a1.w ^ a2.w ^ a3.w ^ b0.w ^ b1.w ^ b2.w ^ b3.w;
        }
    }
    asm volatile("" ::"v"(sink));
}

hipError_t launch_prefetch_kv(KvView kv, int nkv, uint32_t blocks_per_seq, uint64_t first, uint64_t count,
                              uint32_t workgroups, hipStream_t s)
{
    if (count == 0 || workgroups == 0) return hipSuccess;
    hipLaunchKernelGGL(k_prefetch_kv, dim3(workgroups), dim3(256), 0, s, kv, nkv, blocks_per_seq, first, count);
    return hipGetLastError();
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
    hipLaunchKernelGGL(k_copy, dim3((unsigned)blocks), dim3(256), 0, s, reinterpret_cast<uint4 *>(dst),
                       reinterpret_cast<const uint4 *>(src), n16);
    return hipGetLastError();
}

}  // namespace psv

// gfx950 (MI355X, CDNA4) kernels of the PRESERVE decode step: rotary table, decode attention over the block-structured cache, merge of its partials.
//
// Weights and the KV-cache are bf16 (or int8 codes with fp32 scales) in HBM; every accumulation is fp32.  The step
// is bound by HBM bandwidth (Section 2, "LLM decoding is memory BW-limited"), so the kernels are built around
// 16-byte-per-lane coalesced loads with many loads in flight per 64-lane wave; the matrix cores are used where a
// vector-ALU formulation would bind on arithmetic (batch > 2 projections, grouped-query attention).
#include "device.h"

namespace psv {

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
//
// TM: token-major cache (both pools [block][16 tokens][kv head][128 channels]).  One head's key rows are then 256-byte
// pieces at a stride of n_kv_heads * 256 bytes -- the strided read of a shard with several local kv heads -- and are
// loaded exactly like the head-major rows.  The value tile arrives token-major as well, but the second contraction
// needs, per lane, eight consecutive tokens of one channel: each wave passes its 32 x 128 tile through LDS (whole
// 256-byte token rows in, 16-byte pieces XOR-swizzled by the token's group of eight so that the transposed 2-byte
// reads of all 64 lanes fall into different banks) and picks its fragments up transposed.
template <bool TM>
__global__ __launch_bounds__(256) void k_attn(AttnArgs a)
{
    __shared__ float ms[kAttnWaves][16], ls[kAttnWaves][16];
    __shared__ f32x4 accs[kAttnWaves][8][64];      // TM: also the waves' value tiles (4 x 8 KiB) while the loop runs

    const int b = blockIdx.z, kvh = blockIdx.y, c = blockIdx.x;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, i = lane & 15, q4 = lane >> 4;
    const int nq = a.nq, nkv = a.nkv, G = nq / nkv;
    const KvView &kv = a.kv;
    const int qkv_rows = (nq + 2 * nkv) * 128;
    int T = kv.seq_lens[b];
    if (T < 0 || T > kv.max_tokens) T = 0;      // a length outside the descriptor's range is treated as an empty sequence
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
                const uint16_t *base = TM ? kv.k_pool + (((size_t)blk * 16 + (tau1 & 15)) * nkv + kvh) * 128 + q4 * 8
                                          : kv.k_pool + (((size_t)blk * nkv + kvh) * 16 + (tau1 & 15)) * 128 + q4 * 8;
                const size_t row4 = TM ? (size_t)4 * nkv * 128 : (size_t)4 * 128;      // four tokens further
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    ka[ks] = ld16(base + ks * 32);
                    kb[ks] = ld16(base + row4 + ks * 32);
                }
            } else {
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) { ka[ks] = zero16(); kb[ks] = zero16(); }
            }
        }
        if constexpr (TM) {
            // value tile, token-major: load j brings the whole rows of tokens 4j .. 4j+3 (lane = token q4, 16-byte piece i)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int blk = j < 4 ? blkA : blkB;
                vf[j] = blk >= 0 ? ld16(kv.v_pool + (((size_t)blk * 16 + ((4 * j + q4) & 15)) * nkv + kvh) * 128 + i * 8) : zero16();
            }
            return;
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
    //      pairs with f + 64, i.e. fragment ks with fragment ks + 2 of the same lane.  The rotated query is carried
    //      as two bf16 fragments, q = hi + lo: a single bf16 query (2^-9 relative) puts a 2e-3 relative error on the
    //      attention output, which wide models amplify past the tolerance in the MLP block that follows.
    bf16x8 qf[4], qfl[4];
    {
        uint4 z = zero16();
        qf[0] = qf[1] = qf[2] = qf[3] = __builtin_bit_cast(bf16x8, z);
        qfl[0] = qfl[1] = qfl[2] = qfl[3] = __builtin_bit_cast(bf16x8, z);
        if (i < G) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const float *lo = qlo[ks], *hi = qhi[ks];
                uint32_t lh[4], ll[4], hh[4], hl[4];
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    const float2 c0 = qcs[ks][e], c1 = qcs[ks][e + 1];
                    pack_split(lo[e] * c0.x - hi[e] * c0.y, lo[e + 1] * c1.x - hi[e + 1] * c1.y, lh[e >> 1], ll[e >> 1]);
                    pack_split(hi[e] * c0.x + lo[e] * c0.y, hi[e + 1] * c1.x + lo[e + 1] * c1.y, hh[e >> 1], hl[e >> 1]);
                }
                qf[ks] = __builtin_bit_cast(bf16x8, make_uint4(lh[0], lh[1], lh[2], lh[3]));
                qfl[ks] = __builtin_bit_cast(bf16x8, make_uint4(ll[0], ll[1], ll[2], ll[3]));
                qf[ks + 2] = __builtin_bit_cast(bf16x8, make_uint4(hh[0], hh[1], hh[2], hh[3]));
                qfl[ks + 2] = __builtin_bit_cast(bf16x8, make_uint4(hl[0], hl[1], hl[2], hl[3]));
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
                const size_t tm_row = (((size_t)blk * 16 + r) * nkv + kvh) * 128;
                uint16_t *kdst = TM ? kv.k_pool + tm_row : kv.k_pool + (((size_t)blk * nkv + kvh) * 16 + r) * 128;
                kdst[tid] = (uint16_t)f32_to_bf16(lo * cs.x - hi * cs.y);
                kdst[tid + 64] = (uint16_t)f32_to_bf16(hi * cs.x + lo * cs.y);
                if constexpr (TM) {
                    kv.v_pool[tm_row + tid] = (uint16_t)f32_to_bf16(vrow[tid]);
                    kv.v_pool[tm_row + tid + 64] = (uint16_t)f32_to_bf16(vrow[tid + 64]);
                } else {
                    uint16_t *vdst = kv.v_pool + ((size_t)blk * nkv + kvh) * 128 * 16 + r;
                    vdst[(size_t)tid * 16] = (uint16_t)f32_to_bf16(vrow[tid]);
                    vdst[(size_t)(tid + 64) * 16] = (uint16_t)f32_to_bf16(vrow[tid + 64]);
                }
            }
        }
        // the new rows are read back within this workgroup only, through the CU's cache: the barrier's workgroup-scope
        // ordering suffices (later kernels see them after this one has ended)
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
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[ks]), qfl[ks], s1, 0, 0, 0);
            s2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kb[ks]), qfl[ks], s2, 0, 0, 0);
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

        if constexpr (TM) {
            // the wave's own 8 KiB of LDS: token rows in (piece index XOR 2 * (token / 8)), fragments out transposed
            unsigned char *vt = reinterpret_cast<unsigned char *>(&accs[w][0][0]);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int tok = 4 * j + q4;
                *reinterpret_cast<uint4 *>(vt + tok * 256 + ((i ^ (2 * (tok >> 3))) << 4)) = vf[j];
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int dg = 0; dg < 8; ++dg) {
                const int piece = (2 * dg + (i >> 3)) ^ (2 * q4);        // tokens 8 q4 .. 8 q4 + 7 all have token / 8 = q4
                const unsigned char *src = vt + (8 * q4) * 256 + (piece << 4) + (i & 7) * 2;
                uint32_t h[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) h[e] = *reinterpret_cast<const uint16_t *>(src + e * 256);
                vf[dg] = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();      // the next tile's rows overwrite the buffer only after these reads
        }
        // probabilities as two bf16 fragments as well (p = hi + lo)
        uint4 pk, pkl;
        pack_split(p[0], p[1], pk.x, pkl.x);
        pack_split(p[2], p[3], pk.y, pkl.y);
        pack_split(p[4], p[5], pk.z, pkl.z);
        pack_split(p[6], p[7], pk.w, pkl.w);
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
        const bf16x8 pfrag = __builtin_bit_cast(bf16x8, pk), pfrag_lo = __builtin_bit_cast(bf16x8, pkl);
#pragma unroll
        for (int dg = 0; dg < 8; ++dg) {
            acc[dg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vf[dg]), pfrag_lo, acc[dg], 0, 0, 0);
            acc[dg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vf[dg]), pfrag, acc[dg], 0, 0, 0);
        }
    }

    // ---- merge the 4 waves (wave order)
    l_part += __shfl_xor(l_part, 16, 64);
    l_part += __shfl_xor(l_part, 32, 64);
    if (q4 == 0) ms[w][i] = m_run;
    __syncthreads();      // (TM: every wave is also done with its value tile in accs)
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
    if (T < 0 || T > kv.max_tokens) T = 0;      // a length outside the descriptor's range is treated as an empty sequence
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
        }
        // the new rows are read back within this workgroup only, through the CU's cache: the barrier's workgroup-scope
        // ordering suffices (later kernels see them after this one has ended)
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
    else if (kv.token_major)
        PSV_LAUNCH(k_attn<true>, dim3(sp.n_chunks, nkv, batch), dim3(256), 0, s, a);
    else
        PSV_LAUNCH(k_attn<false>, dim3(sp.n_chunks, nkv, batch), dim3(256), 0, s, a);
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

}  // namespace psv

// Q4 pack / unpack kernels (Sec. 3.2 "Q4 Quantization Pipeline"): the flat codec used when an
// agent's cache is saved or restored, and the paged form that appends new tokens to a cache
// (Sec. 3.4, update_and_fetch).  All three stream rows through once and are HBM-bound:
// 2 bytes in and 0.5625 bytes out per quantized element, the reverse for dequantize.
//
// Work layout: one group of 64 elements is handled by 8 consecutive lanes; each lane moves
// 16 bytes of binary16 input (8 elements) and one 32-bit word of codes, so both the loads and
// the stores of a wavefront are contiguous.
#include "q4_device.h"
#include "q4kv_internal.h"

namespace q4kv {
namespace {

constexpr int kThreads = 256;
#ifndef Q4KV_CODEC_WG_PER_CU
#define Q4KV_CODEC_WG_PER_CU 8 // measured best for the read+write mix (4, 8, 16, 32 tried)
#endif

#pragma clang fp contract(off)

// min over the 8 lanes of an octet of both halves of a packed binary16 pair: two quad permutes and a mirror
// inside each half row, on the vector ALU's data-parallel-primitive lanes
__device__ __forceinline__ half2_t octet_pk_min(half2_t v)
{
    int u = (int)half2_to_bits(v);
    v = __builtin_elementwise_min(v, bits_to_half2((uint32_t)__builtin_amdgcn_update_dpp(u, u, 0xB1, 0xF, 0xF, false)));  // quad_perm [1,0,3,2]
    u = (int)half2_to_bits(v);
    v = __builtin_elementwise_min(v, bits_to_half2((uint32_t)__builtin_amdgcn_update_dpp(u, u, 0x4E, 0xF, 0xF, false)));  // quad_perm [2,3,0,1]
    u = (int)half2_to_bits(v);
    v = __builtin_elementwise_min(v, bits_to_half2((uint32_t)__builtin_amdgcn_update_dpp(u, u, 0x141, 0xF, 0xF, false))); // row_half_mirror
    return v;
}

// Quantize the 8 elements held by this lane; the 8 lanes of an octet form one group.
// Returns the packed word; *scale_bits / *bias_bits are the group's stored parameters: binary16, or bfloat16 when
// BF.  The codes are taken against the stored parameters; a bfloat16 bias is in general not the minimum itself, so
// quotients may fall below 0 or above 15 and are clamped.
template <bool BF>
__device__ __forceinline__ uint32_t quantize_octet(uint4 raw, int lane_in_octet, uint16_t *scale_bits,
                                                   uint16_t *bias_bits)
{
    const uint32_t wds[4] = {raw.x, raw.y, raw.z, raw.w};
    float x[8];
    uint16_t xb[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        xb[2 * i] = (uint16_t)(wds[i] & 0xffffu);
        xb[2 * i + 1] = (uint16_t)(wds[i] >> 16);
        x[2 * i] = half_bits_to_float(xb[2 * i]);
        x[2 * i + 1] = half_bits_to_float(xb[2 * i + 1]);
    }
    // min and max of the group in packed binary16 (exact: the inputs are binary16), carried together as
    // (min, -max) so that one packed minimum per exchange serves both
    const half2_t p0 = bits_to_half2(wds[0]), p1 = bits_to_half2(wds[1]), p2 = bits_to_half2(wds[2]), p3 = bits_to_half2(wds[3]);
    const half2_t lo2 = __builtin_elementwise_min(__builtin_elementwise_min(p0, p1), __builtin_elementwise_min(p2, p3));
    const half2_t hi2 = __builtin_elementwise_max(__builtin_elementwise_max(p0, p1), __builtin_elementwise_max(p2, p3));
    half2_t mm = {lo2.x < lo2.y ? lo2.x : lo2.y, -(hi2.x > hi2.y ? hi2.x : hi2.y)};
    mm = octet_pk_min(mm);
    const float mn = (float)mm.x, mx = -(float)mm.y;
    // The stored bias is the bit pattern of the first minimal element.  Only a zero minimum has two
    // encodings; then the sign of the first zero in the group decides.
    uint16_t bb = float_to_half_bits(mn);
    if (mn == 0.0f) {
        uint32_t key = 0xffffffffu; // (position << 1) | sign of the first zero seen by this lane
#pragma unroll
        for (int i = 7; i >= 0; --i)
            if (x[i] == 0.0f) key = ((uint32_t)(lane_in_octet * 8 + i) << 1) | (uint32_t)(xb[i] >> 15);
#pragma unroll
        for (int off = 4; off >= 1; off >>= 1) key = min(key, (uint32_t)__shfl_xor((int)key, off, 8));
        bb = (key & 1u) ? 0x8000u : 0x0000u;
    }
    if (BF && mn != 0.0f) bb = float_to_bf16_bits(mn); // +-0 has the same bits in both types
    const float b = BF ? bf16_bits_to_float(bb) : mn;  // what a decoder adds back
    const float scale32 = (mx - mn) / 15.0f;      // IEEE binary32 division
    const uint16_t sb = BF ? float_to_bf16_bits(scale32) : float_to_half_bits(scale32);
    const float s = param_bits_to_float<BF>(sb);
    uint32_t word = 0;
    if (s != 0.0f) {
        // code = clamp(rint(fl(d / s)), 0, 15) with a correctly rounded binary32 division.  The division is the
        // expensive part, so the quotient is first approximated as t = d * rcp(s): rcp is within 1 ulp and d / s < 32
        // here (d <= max - min, and s is (max - min) / 15 rounded to binary16, at worst halved when it is a binary16
        // subnormal), so |t - fl(d / s)| <= 32 * (2^-23 + 2^-24 + 2^-24) = 2^-17.  rint(t) can differ from
        // rint(fl(d / s)) only if a half-integer lies within that distance of t; such octets (about one element in
        // 2^15) redo all eight codes with the true division.  v_cvt_pk_u8_f32 rounds to nearest even and saturates
        // at 0 (checked on the device); quotients reach 15.5 only in the careful path, which clamps them first.
        // With bfloat16 parameters the bias may lie above the minimum or far below it (|d / s| is then unbounded):
        // groups whose quotients leave [-0.4, 15.4] take the careful path as well.
        const float inv = __builtin_amdgcn_rcpf(s);
        float d[8], t[8];
        // the upper clamp only matters when the stored scale was rounded down a lot (a binary16 subnormal); then too
        // the lane takes the careful path
        bool careful = (mx - b) * inv >= 15.4f;
        if (BF) careful |= (mn - b) * inv <= -0.4f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            d[i] = x[i] - b;
            t[i] = d[i] * inv;
            careful |= fabsf(__builtin_amdgcn_fractf(t[i]) - 0.5f) <= 0x1p-16f;
        }
        if (careful) {
#pragma unroll
            for (int i = 0; i < 8; ++i) t[i] = fminf(BF ? fmaxf(d[i] / s, 0.0f) : d[i] / s, 15.0f);
        }
        uint32_t even = 0, odd = 0; // codes 0,2,4,6 and 1,3,5,7 as bytes
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            even = __builtin_amdgcn_cvt_pk_u8_f32(t[2 * i], i, even);
            odd = __builtin_amdgcn_cvt_pk_u8_f32(t[2 * i + 1], i, odd);
        }
        word = even | (odd << 4);
    }
    *scale_bits = sb;
    *bias_bits = bb;
    return word;
}

// Flat form: destination group = source group, no row arithmetic at all.
template <bool BF>
__global__ __launch_bounds__(kThreads) void quantize_kernel(const uint16_t *__restrict__ x, int64_t total_groups,
                                                            uint32_t *__restrict__ codes, uint16_t *__restrict__ scale,
                                                            uint16_t *__restrict__ bias)
{
    const int sub = threadIdx.x & 7;
    const int64_t stride = (int64_t)gridDim.x * (kThreads / 8);
    const int generation = blockIdx.x / max(1u, gridDim.x / Q4KV_CODEC_WG_PER_CU);
    for (int64_t grp = (int64_t)blockIdx.x * (kThreads / 8) + (threadIdx.x >> 3); grp < total_groups; grp += stride) {
        rotate_wave_priority(generation);
        const uint4 raw = *reinterpret_cast<const uint4 *>(x + grp * kGroup + sub * 8);
        uint16_t sb, bb;
        const uint32_t word = quantize_octet<BF>(raw, sub, &sb, &bb);
        codes[grp * 8 + sub] = word;
        if (sub == 0) {
            scale[grp] = sb;
            bias[grp] = bb;
        }
    }
}

// Paged form (Sec. 3.4 update_and_fetch, first half): source rows [layer in call][agent][chunk token][kv head],
// destination the agent's blocks.  Layer and agent come from the launch grid, so that a lane's index arithmetic is
// two 32-bit divisions (by the groups per row and by the chunk length) instead of a chain of 64-bit ones; a token
// outside the table or a block id outside the pool is skipped.
struct AppendParams {
    const int32_t *block_table;
    const int32_t *seq_len_before;
    int max_blocks, chunk_len, heads, layer_begin, num_blocks, groups_per_row;
};

template <bool BF>
__global__ __launch_bounds__(kThreads) void append_kernel(const uint16_t *__restrict__ x, uint32_t *__restrict__ codes,
                                                          uint16_t *__restrict__ scale, uint16_t *__restrict__ bias,
                                                          AppendParams p)
{
    const int sub = threadIdx.x & 7;
    const int a = blockIdx.y, li = blockIdx.z, agents = gridDim.y;
    const uint32_t per_unit = (uint32_t)p.chunk_len * p.heads * p.groups_per_row; // groups of one (layer, agent)
    const int64_t src0 = ((int64_t)li * agents + a) * per_unit;
    const int n0 = p.seq_len_before[a];
    const int32_t *table = p.block_table + (int64_t)a * p.max_blocks;
    // generations of the launch: workgroups in launch order (x fastest), about 256 of them per generation
    const uint32_t linear = (blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
    const int generation = linear / max(1u, gridDim.x * gridDim.y * gridDim.z / Q4KV_CODEC_WG_PER_CU);
    for (uint32_t gi = blockIdx.x * (kThreads / 8) + (threadIdx.x >> 3); gi < per_unit; gi += gridDim.x * (kThreads / 8)) {
        rotate_wave_priority(generation);
        // groups are walked in the order of the pool (head, then chunk token, then group): consecutive lanes then
        // write consecutive rows of one head's plane of a block, and read whole 2 dim-byte source rows
        const uint32_t row = gi / (uint32_t)p.groups_per_row, g = gi - row * p.groups_per_row;
        const uint32_t h = row / (uint32_t)p.chunk_len, c = row - h * p.chunk_len;
        const uint32_t src = (c * p.heads + h) * p.groups_per_row + g;
        const uint4 raw = *reinterpret_cast<const uint4 *>(x + (src0 + src) * kGroup + sub * 8);
        uint16_t sb, bb;
        const uint32_t word = quantize_octet<BF>(raw, sub, &sb, &bb);
        const int t = n0 + (int)c;
        const int bi = t / kBlockTokens;
        if (t < 0 || bi >= p.max_blocks) continue;
        const int blk = table[bi];
        if (blk < 0 || blk >= p.num_blocks) continue;
        const int64_t drow = (((int64_t)(p.layer_begin + li) * p.num_blocks + blk) * p.heads + h) * kBlockTokens + (t % kBlockTokens);
        const int64_t dgrp = drow * p.groups_per_row + g;
        codes[dgrp * 8 + sub] = word;
        if (sub == 0) {
            scale[dgrp] = sb;
            bias[dgrp] = bb;
        }
    }
}

// One lane per word: 8 codes -> 8 binary16 values (16 bytes).
template <bool BF>
__global__ __launch_bounds__(kThreads) void dequantize_kernel(const uint32_t *__restrict__ codes,
                                                              const uint16_t *__restrict__ scale,
                                                              const uint16_t *__restrict__ bias, int64_t total_words,
                                                              uint16_t *__restrict__ x)
{
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    const int generation = blockIdx.x / max(1u, gridDim.x / Q4KV_CODEC_WG_PER_CU);
    for (int64_t w = (int64_t)blockIdx.x * kThreads + threadIdx.x; w < total_words; w += stride) {
        rotate_wave_priority(generation);
        const uint32_t word = codes[w];
        const float s = param_bits_to_float<BF>(scale[w >> 3]);
        const float b = param_bits_to_float<BF>(bias[w >> 3]);
        uint32_t o[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float lo = (float)((word >> (8 * i)) & 0xfu) * s + b;      // product exact in binary32
            const float hi = (float)((word >> (8 * i + 4)) & 0xfu) * s + b;
            o[i] = (uint32_t)float_to_half_bits(lo) | ((uint32_t)float_to_half_bits(hi) << 16);
        }
        // a store that says the line will not be read again: +4 % (4.85 -> 5.05 TB/s); the same hint on the loads
        // changes nothing, and on either side of the quantize kernel it costs 6-9 %
        typedef uint32_t u4_t __attribute__((ext_vector_type(4)));
        __builtin_nontemporal_store(u4_t{o[0], o[1], o[2], o[3]}, reinterpret_cast<u4_t *>(x + w * 8));
    }
}

int grid_for(int64_t items, int per_block)
{
    int64_t blocks = (items + per_block - 1) / per_block;
    const int64_t cap = 256 * Q4KV_CODEC_WG_PER_CU; // the kernels grid-stride
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    return (int)blocks;
}

} // namespace

hipError_t launch_quantize(const uint16_t *x, int64_t rows, int dim, bool bf16_params, uint32_t *codes, uint16_t *scale,
                           uint16_t *bias, hipStream_t stream)
{
    const int G = dim / kGroup;
    const int64_t groups = rows * G;
    if (groups == 0) return hipSuccess;
    const dim3 grid(grid_for(groups, kThreads / 8));
    if (bf16_params)
        hipLaunchKernelGGL(quantize_kernel<true>, grid, dim3(kThreads), 0, stream, x, groups, codes, scale, bias);
    else
        hipLaunchKernelGGL(quantize_kernel<false>, grid, dim3(kThreads), 0, stream, x, groups, codes, scale, bias);
    return hipGetLastError();
}

hipError_t launch_dequantize(const uint32_t *codes, const uint16_t *scale, const uint16_t *bias, int64_t rows,
                             int dim, bool bf16_params, uint16_t *x, hipStream_t stream)
{
    const int64_t words = rows * (dim / 8);
    if (words == 0) return hipSuccess;
    const dim3 grid(grid_for(words, kThreads));
    if (bf16_params)
        hipLaunchKernelGGL(dequantize_kernel<true>, grid, dim3(kThreads), 0, stream, codes, scale, bias, words, x);
    else
        hipLaunchKernelGGL(dequantize_kernel<false>, grid, dim3(kThreads), 0, stream, codes, scale, bias, words, x);
    return hipGetLastError();
}

hipError_t launch_append(const q4kv_spec &spec, const q4kv_pool &pool, int dim, const uint16_t *x_new,
                         const int32_t *block_table, int max_blocks, const int32_t *seq_len_before, int num_agents,
                         int chunk_len, int layer_begin, int layer_end, hipStream_t stream)
{
    const int G = dim / kGroup;
    const int layers = layer_end - layer_begin;
    const int64_t per_unit = (int64_t)chunk_len * spec.num_kv_heads * G;
    if (layers <= 0 || num_agents <= 0 || per_unit == 0) return hipSuccess;
    if (per_unit > 0x7fffffffLL || num_agents > 65535 || layers > 65535) return hipErrorInvalidValue;
    AppendParams p{block_table, seq_len_before, max_blocks, chunk_len, spec.num_kv_heads, layer_begin, pool.num_blocks, G};
    // workgroups per (layer, agent): enough for the chunk, and at most 8 per compute unit over the whole launch
    // (rounded down: a launch of 1.2 rounds takes as long as one of 2)
    int64_t gx = (per_unit + kThreads / 8 - 1) / (kThreads / 8);
    const int64_t cap = 256LL * Q4KV_CODEC_WG_PER_CU / ((int64_t)layers * num_agents);
    if (gx > cap) gx = cap;
    if (gx < 1) gx = 1;
    const dim3 grid((unsigned)gx, (unsigned)num_agents, (unsigned)layers);
    if (spec.param_format == Q4KV_PARAMS_BF16)
        hipLaunchKernelGGL(append_kernel<true>, grid, dim3(kThreads), 0, stream, x_new, pool.codes, pool.scale, pool.bias, p);
    else
        hipLaunchKernelGGL(append_kernel<false>, grid, dim3(kThreads), 0, stream, x_new, pool.codes, pool.scale, pool.bias, p);
    return hipGetLastError();
}

} // namespace q4kv

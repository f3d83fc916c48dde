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
constexpr int kWorkgroupsPerCu = 8; // measured best for the read+write mix (4, 8, 16, 32 tried)

#pragma clang fp contract(off)

// Packed binary16 minimum / maximum as single instructions.  (The generic element-wise builtins first quiet a
// signalling NaN in each operand, one more instruction per operand; a cache row holds no NaN.)
__device__ __forceinline__ uint32_t pk_min(uint32_t a, uint32_t b)
{
    uint32_t r;
    asm("v_pk_min_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ uint32_t pk_max(uint32_t a, uint32_t b)
{
    uint32_t r;
    asm("v_pk_max_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// fl(h + a) in binary32 for the low / the high binary16 half h of a word: the mixed-precision fused multiply-add
// h * 1.0 + a converts and adds in one instruction (the product is exact, so the one rounding is that of the sum)
__device__ __forceinline__ float half_lo_plus(uint32_t pair, float a)
{
    float d;
    asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel_hi:[1,0,0]" : "=v"(d) : "v"(pair), "v"(a));
    return d;
}
__device__ __forceinline__ float half_hi_plus(uint32_t pair, float a)
{
    float d;
    asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(pair), "v"(a));
    return d;
}

// min over the 8 lanes of an octet of both halves of a packed binary16 pair: two quad permutes and a mirror
// inside each half row, on the vector ALU's data-parallel-primitive lanes (every lane has a source lane, so the
// previous value of the destination is never used)
__device__ __forceinline__ uint32_t octet_pk_min(uint32_t v)
{
    v = pk_min(v, (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true));  // quad_perm [1,0,3,2]
    v = pk_min(v, (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true));  // quad_perm [2,3,0,1]
    v = pk_min(v, (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x141, 0xF, 0xF, true)); // row_half_mirror
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
    uint16_t xb[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        xb[2 * i] = (uint16_t)(wds[i] & 0xffffu);
        xb[2 * i + 1] = (uint16_t)(wds[i] >> 16);
    }
    // min and max of the group in packed binary16 (exact: the inputs are binary16), carried together as
    // (min, -max) so that one packed minimum per exchange serves both
    const uint32_t lo2 = pk_min(pk_min(wds[0], wds[1]), pk_min(wds[2], wds[3]));
    const uint32_t hi2 = pk_max(pk_max(wds[0], wds[1]), pk_max(wds[2], wds[3]));
    const half2_t l2 = bits_to_half2(lo2), h2 = bits_to_half2(hi2);
    half2_t mm = {l2.x < l2.y ? l2.x : l2.y, -(h2.x > h2.y ? h2.x : h2.y)};
    mm = bits_to_half2(octet_pk_min(half2_to_bits(mm)));
    const float mn = (float)mm.x, mx = -(float)mm.y;
    // The stored bias is the bit pattern of the first minimal element.  Only a zero minimum has two
    // encodings; then the sign of the first zero in the group decides.
    uint16_t bb = float_to_half_bits(mn);
    if (mn == 0.0f) {
        uint32_t key = 0xffffffffu; // (position << 1) | sign of the first zero seen by this lane
#pragma unroll
        for (int i = 7; i >= 0; --i)
            if ((xb[i] & 0x7fffu) == 0) key = ((uint32_t)(lane_in_octet * 8 + i) << 1) | (uint32_t)(xb[i] >> 15);
#pragma unroll
        for (int off = 4; off >= 1; off >>= 1) key = min(key, (uint32_t)__shfl_xor((int)key, off, 8));
        bb = (key & 1u) ? 0x8000u : 0x0000u;
    }
    if (BF && mn != 0.0f) bb = float_to_bf16_bits(mn); // +-0 has the same bits in both types
    const float b = BF ? bf16_bits_to_float(bb) : mn;  // what a decoder adds back
    // scale = fl((max - min) / 15), the correctly rounded binary32 quotient, without the division sequence: with
    // c = fl(1/15), q0 = fl(r * c), e = fma(-15, q0, r) and q = fma(e, c, q0), q equals fl(r / 15) for every
    // binary32 r in [2^-24, 2^17] (checked value by value on the host); r = max - min of finite binary16 values
    // is 0 or lies in that range
    const float r = mx - mn, q0 = r * (1.0f / 15.0f);
    float scale32 = __builtin_fmaf(__builtin_fmaf(-15.0f, q0, r), 1.0f / 15.0f, q0);
    asm("" : "+v"(scale32)); // the binary32 value itself is rounded next: keeps that rounding a step of its own
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
        const float minus_b = -b;
        // the upper clamp only matters when the stored scale was rounded down a lot (a binary16 subnormal); then too
        // the lane takes the careful path
        bool careful = (mx - b) * inv >= 15.4f;
        if (BF) careful |= (mn - b) * inv <= -0.4f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            d[i] = (i & 1) ? half_hi_plus(wds[i / 2], minus_b) : half_lo_plus(wds[i / 2], minus_b); // fl(x - b)
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
    const int sub = threadIdx.x & 7, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int generation = blockIdx.x / max(1u, gridDim.x / kWorkgroupsPerCu);
    // A wave takes 64 consecutive groups per round, in four steps of two groups per octet of lanes (both loads of a
    // step issued before either is used).  The round's 64 scales and 64 biases are gathered in the wave's own 256
    // bytes of LDS and leave as one store instruction: two whole 128-byte lines.  Stored 16 bytes at a time (one
    // lane per group), the memory system wrote such lines in pieces: 6-7 % more bytes written than stored.
    __shared__ uint16_t s_par[kThreads / 64][2][64];
    const bool words_ok = ((reinterpret_cast<uintptr_t>(scale) | reinterpret_cast<uintptr_t>(bias)) & 3u) == 0;
    const int64_t rounds = (total_groups + 63) / 64;
    for (int64_t c = (int64_t)blockIdx.x * (kThreads / 64) + wave; c < rounds; c += (int64_t)gridDim.x * (kThreads / 64)) {
        rotate_wave_priority(generation);
#pragma unroll
        for (int step = 0; step < 4; ++step) {
            const int l0 = step * 16 + (lane >> 3), l1 = l0 + 8;
            const int64_t g0 = c * 64 + l0, g1 = c * 64 + l1;
            uint4 raw0 = make_uint4(0, 0, 0, 0), raw1 = make_uint4(0, 0, 0, 0);
            if (g0 < total_groups) raw0 = *reinterpret_cast<const uint4 *>(x + g0 * kGroup + sub * 8);
            if (g1 < total_groups) raw1 = *reinterpret_cast<const uint4 *>(x + g1 * kGroup + sub * 8);
            uint16_t sb, bb;
            if (g0 < total_groups) {
                const uint32_t word = quantize_octet<BF>(raw0, sub, &sb, &bb);
                codes[g0 * 8 + sub] = word;
                if (sub == 0) {
                    s_par[wave][0][l0] = sb;
                    s_par[wave][1][l0] = bb;
                }
            }
            if (g1 < total_groups) {
                const uint32_t word = quantize_octet<BF>(raw1, sub, &sb, &bb);
                codes[g1 * 8 + sub] = word;
                if (sub == 0) {
                    s_par[wave][0][l1] = sb;
                    s_par[wave][1][l1] = bb;
                }
            }
        }
        // the wave's LDS operations complete in order; the fences keep the compiler from moving them
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        {
            const int which = lane >> 5, pair = lane & 31; // lanes 0-31 the scales, 32-63 the biases, two per lane
            const int64_t g = c * 64 + 2 * pair;
            uint16_t *dst = (which ? bias : scale) + g;
            const uint32_t two = *reinterpret_cast<const uint32_t *>(&s_par[wave][which][2 * pair]);
            if (g + 1 < total_groups && words_ok) {
                *reinterpret_cast<uint32_t *>(dst) = two;
            } else {
                if (g < total_groups) dst[0] = (uint16_t)(two & 0xffffu);
                if (g + 1 < total_groups) dst[1] = (uint16_t)(two >> 16);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

// Paged form (Sec. 3.4 update_and_fetch, first half): source rows [layer in call][agent][chunk token][kv head],
// destination the agent's blocks.  Layer and agent come from the launch grid, so that a lane's index arithmetic is
// two 32-bit divisions (by the groups per row and by the chunk length) instead of a chain of 64-bit ones; a token
// outside the table or a block id outside the pool is skipped.
// One launch serves the K and the V pool (two short launches one after the other each paid their own ramp and
// tail): the upper half of the grid's z range belongs to the second pool.
struct AppendPool {
    const uint16_t *x;
    uint32_t *codes;
    uint16_t *scale, *bias;
    int groups_per_row;
};
struct AppendParams {
    AppendPool pool[2];
    const int32_t *block_table;
    const int32_t *seq_len_before;
    int max_blocks, chunk_len, heads, layer_begin, num_blocks, layers;
};

template <bool BF>
__global__ __launch_bounds__(kThreads) void append_kernel(AppendParams pp)
{
    const int sub = threadIdx.x & 7;
    const int which = blockIdx.z >= (unsigned)pp.layers ? 1 : 0;
    const int a = blockIdx.y, li = blockIdx.z - which * pp.layers, agents = gridDim.y;
    struct {
        const int32_t *block_table, *seq_len_before;
        int max_blocks, chunk_len, heads, layer_begin, num_blocks, groups_per_row;
    } p = {pp.block_table, pp.seq_len_before, pp.max_blocks, pp.chunk_len, pp.heads, pp.layer_begin, pp.num_blocks,
           pp.pool[which].groups_per_row};
    const uint16_t *__restrict__ x = pp.pool[which].x;
    uint32_t *__restrict__ codes = pp.pool[which].codes;
    uint16_t *__restrict__ scale = pp.pool[which].scale, *__restrict__ bias = pp.pool[which].bias;
    const uint32_t per_unit = (uint32_t)p.chunk_len * p.heads * p.groups_per_row; // groups of one (layer, agent)
    const int64_t src0 = ((int64_t)li * agents + a) * per_unit;
    const int n0 = p.seq_len_before[a];
    const int32_t *table = p.block_table + (int64_t)a * p.max_blocks;
    // generations of the launch: workgroups in launch order (x fastest), about 256 of them per generation
    const uint32_t linear = (blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
    const int generation = linear / max(1u, gridDim.x * gridDim.y * gridDim.z / kWorkgroupsPerCu);
    // 64 consecutive groups per wave and round, in four steps of two groups per octet of lanes, the parameters
    // gathered in LDS and stored two per lane, as in quantize_kernel.  Where a group comes from and where it goes is
    // worked out once per round, by lane l for group l of the round, and kept in LDS: worked out by every lane of an
    // octet for each of its eight groups it was a third of the kernel's vector instructions, and the kernel is bound
    // by those (the vector ALUs were busy nine tenths of its time).
    __shared__ uint16_t s_par[kThreads / 64][2][64];
    __shared__ int64_t s_dst[kThreads / 64][64];  // group index in the pool, -1: skipped
    __shared__ uint32_t s_src[kThreads / 64][64]; // group index in this (layer, agent)'s source rows
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool words_ok = ((reinterpret_cast<uintptr_t>(scale) | reinterpret_cast<uintptr_t>(bias)) & 3u) == 0;
    const float inv_gpr = 1.0f / (float)p.groups_per_row, inv_chunk = 1.0f / (float)p.chunk_len;
    for (uint32_t c0 = (blockIdx.x * (kThreads / 64) + wave) * 64; c0 < per_unit; c0 += gridDim.x * kThreads) {
        rotate_wave_priority(generation);
        // Where the round begins -- head, chunk token, group in the row -- is the same for the whole wave and costs
        // two integer divisions per round.  A lane is at most 63 groups further on: its own place follows from two
        // quotients of small numbers, each taken as floor((n + 0.5) * fl(1 / d)), which equals n / d for
        // n < 2^21 (the product errs by less than n / d * 2^-22, and (n + 0.5) / d is at least 0.5 / d away from an
        // integer); the host refuses longer chunks.
        // Groups are walked in the order of the pool (head, then chunk token, then group): consecutive lanes then
        // write consecutive rows of one head's plane of a block, and read whole 2 dim-byte source rows.  (Walking
        // them in source order instead, a contiguous span per workgroup -- contiguous reads, scattered rows written
        // -- was measured slower: 0.69 against 0.65 ms on the 10-agent, 48-layer chunk.)
        const uint32_t row0 = c0 / (uint32_t)p.groups_per_row, g0 = c0 - row0 * p.groups_per_row;
        const uint32_t h0 = row0 / (uint32_t)p.chunk_len, cr0 = row0 - h0 * p.chunk_len;
        {
            const uint32_t gl = g0 + lane;
            const uint32_t rows = (uint32_t)(((float)gl + 0.5f) * inv_gpr);
            const uint32_t g = gl - rows * p.groups_per_row;
            const uint32_t cl = cr0 + rows;
            const uint32_t heads = (uint32_t)(((float)cl + 0.5f) * inv_chunk);
            const uint32_t h = h0 + heads, c = cl - heads * p.chunk_len;
            int64_t dgrp = -1;
            if (c0 + lane < per_unit) {
                const int t = n0 + (int)c;
                const int bi = t / kBlockTokens;
                if (t >= 0 && bi < p.max_blocks) {
                    const int blk = table[bi];
                    if (blk >= 0 && blk < p.num_blocks) {
                        const int64_t drow = (((int64_t)(p.layer_begin + li) * p.num_blocks + blk) * p.heads + h) * kBlockTokens +
                                             (t % kBlockTokens);
                        dgrp = drow * p.groups_per_row + g;
                    }
                }
            }
            s_src[wave][lane] = (c * p.heads + h) * p.groups_per_row + g;
            s_dst[wave][lane] = dgrp;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll 1
        for (int step = 0; step < 4; ++step) {
            uint4 raw[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const uint32_t l = step * 16 + 8 * j + (lane >> 3);
                const uint32_t src = s_src[wave][l];
                raw[j] = c0 + l < per_unit ? *reinterpret_cast<const uint4 *>(x + (src0 + src) * kGroup + sub * 8) : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const uint32_t l = step * 16 + 8 * j + (lane >> 3);
                uint16_t sb = 0, bb = 0;
                if (c0 + l < per_unit) {
                    const uint32_t word = quantize_octet<BF>(raw[j], sub, &sb, &bb);
                    const int64_t dgrp = s_dst[wave][l];
                    if (dgrp >= 0) codes[dgrp * 8 + sub] = word;
                }
                if (sub == 0) {
                    s_par[wave][0][l] = sb;
                    s_par[wave][1][l] = bb;
                }
            }
        }
        // the wave's LDS operations complete in order; the fences keep the compiler from moving them
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        {
            const int which_par = lane >> 5, pair = lane & 31; // lanes 0-31 the scales, 32-63 the biases
            const int64_t d0 = s_dst[wave][2 * pair], d1 = s_dst[wave][2 * pair + 1];
            const uint32_t two = *reinterpret_cast<const uint32_t *>(&s_par[wave][which_par][2 * pair]);
            uint16_t *arr = which_par ? bias : scale;
            if (words_ok && d0 >= 0 && d1 == d0 + 1 && (d0 & 1) == 0) {
                *reinterpret_cast<uint32_t *>(arr + d0) = two;
            } else {
                if (d0 >= 0) arr[d0] = (uint16_t)(two & 0xffffu);
                if (d1 >= 0) arr[d1] = (uint16_t)(two >> 16);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

// One lane per word: 8 codes -> 8 binary16 values (16 bytes).
template <bool BF>
__global__ __launch_bounds__(kThreads) void dequantize_kernel(const uint32_t *__restrict__ codes,
                                                              const uint16_t *__restrict__ scale,
                                                              const uint16_t *__restrict__ bias, int64_t total_words,
                                                              uint16_t *__restrict__ x)
{
    // A workgroup takes 1,024 consecutive words (128 groups) per round, four per lane, every load issued before the
    // first is used; the round's scales and biases are two whole lines read by one compute unit.
    constexpr int NQ = 4;
    typedef uint32_t u4_t __attribute__((ext_vector_type(4)));
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    const int generation = blockIdx.x / max(1u, gridDim.x / kWorkgroupsPerCu);
    for (int64_t w0 = (int64_t)blockIdx.x * NQ * kThreads + threadIdx.x; w0 < total_words; w0 += NQ * stride) {
        rotate_wave_priority(generation);
        uint32_t word[NQ];
        uint16_t sb[NQ], bb[NQ];
#pragma unroll
        for (int j = 0; j < NQ; ++j) {
            const int64_t w = w0 + j * kThreads;
            const bool in = w < total_words;
            word[j] = in ? codes[w] : 0u;
            sb[j] = in ? scale[w >> 3] : (uint16_t)0;
            bb[j] = in ? bias[w >> 3] : (uint16_t)0;
        }
#pragma unroll
        for (int j = 0; j < NQ; ++j) {
            const int64_t w = w0 + j * kThreads;
            if (w >= total_words) break;
            const float s = param_bits_to_float<BF>(sb[j]), b = param_bits_to_float<BF>(bb[j]);
            uint32_t o[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float lo = (float)((word[j] >> (8 * i)) & 0xfu) * s + b;      // product exact in binary32
                const float hi = (float)((word[j] >> (8 * i + 4)) & 0xfu) * s + b;
                o[i] = (uint32_t)float_to_half_bits(lo) | ((uint32_t)float_to_half_bits(hi) << 16);
            }
            // a store that says the line will not be read again: +4 % (4.85 -> 5.05 TB/s); the same hint on the
            // loads changes nothing, and on either side of the quantize kernel it costs 6-9 %
            __builtin_nontemporal_store(u4_t{o[0], o[1], o[2], o[3]}, reinterpret_cast<u4_t *>(x + w * 8));
        }
    }
}

int grid_for(int64_t items, int per_block, int compute_units)
{
    int64_t blocks = (items + per_block - 1) / per_block;
    const int64_t cap = (int64_t)compute_units * kWorkgroupsPerCu; // the kernels grid-stride
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    return (int)blocks;
}

} // namespace

hipError_t launch_quantize(const uint16_t *x, int64_t rows, int dim, bool bf16_params, uint32_t *codes, uint16_t *scale,
                           uint16_t *bias, int compute_units, hipStream_t stream)
{
    const int G = dim / kGroup;
    const int64_t groups = rows * G;
    if (groups == 0) return hipSuccess;
    const dim3 grid(grid_for(groups, 4 * 64, compute_units));
    if (bf16_params)
        hipLaunchKernelGGL(quantize_kernel<true>, grid, dim3(kThreads), 0, stream, x, groups, codes, scale, bias);
    else
        hipLaunchKernelGGL(quantize_kernel<false>, grid, dim3(kThreads), 0, stream, x, groups, codes, scale, bias);
    return hipGetLastError();
}

hipError_t launch_dequantize(const uint32_t *codes, const uint16_t *scale, const uint16_t *bias, int64_t rows,
                             int dim, bool bf16_params, uint16_t *x, int compute_units, hipStream_t stream)
{
    const int64_t words = rows * (dim / 8);
    if (words == 0) return hipSuccess;
    const dim3 grid(grid_for(words, 4 * kThreads, compute_units));
    if (bf16_params)
        hipLaunchKernelGGL(dequantize_kernel<true>, grid, dim3(kThreads), 0, stream, codes, scale, bias, words, x);
    else
        hipLaunchKernelGGL(dequantize_kernel<false>, grid, dim3(kThreads), 0, stream, codes, scale, bias, words, x);
    return hipGetLastError();
}

hipError_t launch_append(const q4kv_spec &spec, const q4kv_pool &k, const q4kv_pool *v, const uint16_t *k_new,
                         const uint16_t *v_new, const int32_t *block_table, int max_blocks,
                         const int32_t *seq_len_before, int num_agents, int chunk_len, int layer_begin, int layer_end,
                         int compute_units, hipStream_t stream)
{
    const int layers = layer_end - layer_begin;
    const int pools = v ? 2 : 1;
    const int gk = spec.k_dim / kGroup, gv = v ? spec.v_dim / kGroup : 0;
    const int64_t per_unit = (int64_t)chunk_len * spec.num_kv_heads * (gk > gv ? gk : gv); // of the wider pool
    if (layers <= 0 || num_agents <= 0 || per_unit == 0) return hipSuccess;
    if (per_unit > 0x7fffffffLL || num_agents > 65535 || pools * layers > 65535 || chunk_len > Q4KV_MAX_CHUNK_LEN)
        return hipErrorInvalidValue;
    AppendParams p;
    p.pool[0] = AppendPool{k_new, k.codes, k.scale, k.bias, gk};
    p.pool[1] = v ? AppendPool{v_new, v->codes, v->scale, v->bias, gv} : p.pool[0];
    p.block_table = block_table;
    p.seq_len_before = seq_len_before;
    p.max_blocks = max_blocks;
    p.chunk_len = chunk_len;
    p.heads = spec.num_kv_heads;
    p.layer_begin = layer_begin;
    p.num_blocks = k.num_blocks;
    p.layers = layers;
    // workgroups per (pool, layer, agent): enough for the chunk, and at most 8 per compute unit over the whole
    // launch (rounded down: a launch of 1.2 rounds takes as long as one of 2)
    int64_t gx = (per_unit + kThreads - 1) / kThreads;
    const int64_t cap = (int64_t)compute_units * kWorkgroupsPerCu / ((int64_t)pools * layers * num_agents);
    if (gx > cap) gx = cap;
    if (gx < 1) gx = 1;
    const dim3 grid((unsigned)gx, (unsigned)num_agents, (unsigned)(pools * layers));
    if (spec.param_format == Q4KV_PARAMS_BF16)
        hipLaunchKernelGGL(append_kernel<true>, grid, dim3(kThreads), 0, stream, p);
    else
        hipLaunchKernelGGL(append_kernel<false>, grid, dim3(kThreads), 0, stream, p);
    return hipGetLastError();
}

} // namespace q4kv

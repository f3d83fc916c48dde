// Device-side helpers shared by the gfx950 kernels of libq4kv: binary16 access,
// nibble unpacking into packed binary16 pairs, wave-level reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace q4kv {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));

constexpr int kGroup = 64;        // elements per quantization group (Sec. 3.2: g = 64)
constexpr int kBlockTokens = 256; // tokens per cache block (Sec. 3.1)
constexpr int kWave = 64;         // CDNA wavefront width

__device__ __forceinline__ half2_t bits_to_half2(uint32_t u) { return __builtin_bit_cast(half2_t, u); }
__device__ __forceinline__ uint32_t half2_to_bits(half2_t h) { return __builtin_bit_cast(uint32_t, h); }
__device__ __forceinline__ float half_bits_to_float(uint16_t b) { return (float)__builtin_bit_cast(half_t, b); }
__device__ __forceinline__ uint16_t float_to_half_bits(float f)
{
    return __builtin_bit_cast(uint16_t, (half_t)f); // v_cvt_f16_f32, round to nearest even
}

// bfloat16 (the upper half of a binary32): the other type scale and bias may be stored in (Sec. 3.1, Sec. 3.2).
__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __builtin_bit_cast(float, (uint32_t)b << 16); }
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) // finite f, round to nearest even
{
    const uint32_t u = __builtin_bit_cast(uint32_t, f);
    return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}
// a stored scale or bias as binary32; BF: the bits are bfloat16, else binary16
template <bool BF>
__device__ __forceinline__ float param_bits_to_float(uint16_t b)
{
    if constexpr (BF) return bf16_bits_to_float(b);
    else return half_bits_to_float(b);
}

// Eight 4-bit codes of one word as four packed binary16 pairs.  A code c placed in the low
// mantissa bits of a binary16 with zero exponent is the subnormal c * 2^-24 (bits 0..3) or
// c * 2^-20 (bits 4..7), so no integer-to-float conversion is needed:
//   a0 = (c0, c4) * 2^-24   b0 = (c1, c5) * 2^-20   a1 = (c2, c6) * 2^-24   b1 = (c3, c7) * 2^-20
// The consumers multiply by kCodeScaleA / kCodeScaleB afterwards (in binary32, exact).
struct CodePairs {
    half2_t a0, b0, a1, b1;
};
constexpr float kCodeScaleA = 16777216.0f; // 2^24
constexpr float kCodeScaleB = 1048576.0f;  // 2^20

__device__ __forceinline__ CodePairs unpack_codes(uint32_t w)
{
    CodePairs p;
    const uint32_t w8 = w >> 8;
    p.a0 = bits_to_half2(w & 0x000F000Fu);
    p.b0 = bits_to_half2(w & 0x00F000F0u);
    p.a1 = bits_to_half2(w8 & 0x000F000Fu);
    p.b1 = bits_to_half2(w8 & 0x00F000F0u);
    return p;
}

// On a compute unit the oldest wave wins every arbitration (also the one for the memory pipeline), so of the
// workgroups a grid-striding launch stacks on a compute unit the ones launched first run ahead, finish first and
// leave the last generation to stream alone at the end.  A kernel that calls this once per loop iteration hands
// the four wave priorities round among its generations in 10 us slices of the chip-wide clock: all generations
// then finish together (measured: quantize +11 %, dequantize +8 %).  `generation` = launch
// index / workgroups launched per generation (one per compute unit).
__device__ __forceinline__ void rotate_wave_priority(int generation)
{
    const int level = (generation + (int)(wall_clock64() >> 10)) & 3;
    if (level == 0) __builtin_amdgcn_s_setprio(0);
    else if (level == 1) __builtin_amdgcn_s_setprio(1);
    else if (level == 2) __builtin_amdgcn_s_setprio(2);
    else __builtin_amdgcn_s_setprio(3);
}

// Orders LDS traffic between the lanes of one wavefront: what lanes wrote before is visible to
// every lane after.  Waves of a workgroup that do not share LDS regions need nothing stronger.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Wave-wide reductions on the vector ALU's data-parallel-primitive lanes (no LDS round trips):
// four steps inside each row of 16 lanes, two row broadcasts, result read from lane 63.
#define Q4KV_DPP(old, src, ctrl, row_mask)                                                                   \
    __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, (float)(old)),                \
                                                          __builtin_bit_cast(int, (float)(src)), (ctrl), (row_mask), \
                                                          0xF, false))

__device__ __forceinline__ float wave_max(float v)
{
    v = fmaxf(v, Q4KV_DPP(v, v, 0xB1, 0xF));  // quad_perm [1,0,3,2]
    v = fmaxf(v, Q4KV_DPP(v, v, 0x4E, 0xF));  // quad_perm [2,3,0,1]
    v = fmaxf(v, Q4KV_DPP(v, v, 0x141, 0xF)); // row_half_mirror
    v = fmaxf(v, Q4KV_DPP(v, v, 0x140, 0xF)); // row_mirror
    v = fmaxf(v, Q4KV_DPP(v, v, 0x142, 0xA)); // row_bcast15 into rows 1 and 3
    v = fmaxf(v, Q4KV_DPP(v, v, 0x143, 0xC)); // row_bcast31 into rows 2 and 3
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// The maxima of N values over the wave, taken together: every step is one v_max_f32 with a DPP operand per value
// (written out: through the builtins each step costs a copy, the move and a NaN-quieting maximum besides), and the
// steps of the N chains interleave.  A DPP operand must not be read within two wait states of the vector
// instruction that wrote it, nor within five of a vector instruction that wrote EXEC; the compiler does not look
// inside asm statements, so each begins with the longer wait and has the shorter one between its steps.
#define Q4KV_MAX_DPP(CTRL) "v_max_f32_dpp %0, %0, %0 " CTRL "\n\t"
#define Q4KV_MAX_DPP2(CTRL) Q4KV_MAX_DPP(CTRL) "v_max_f32_dpp %1, %1, %1 " CTRL "\n\t"
#define Q4KV_MAX_DPP4(CTRL)                                                                                             \
    Q4KV_MAX_DPP2(CTRL) "v_max_f32_dpp %2, %2, %2 " CTRL "\n\tv_max_f32_dpp %3, %3, %3 " CTRL "\n\t"
#define Q4KV_MAX_STEPS(M)                                                                                               \
    M("quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf")                                                                 \
    "s_nop 1\n\t" M("quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf")                                                   \
    "s_nop 1\n\t" M("row_half_mirror row_mask:0xf bank_mask:0xf")                                                       \
    "s_nop 1\n\t" M("row_mirror row_mask:0xf bank_mask:0xf")                                                            \
    "s_nop 1\n\t" M("row_bcast:15 row_mask:0xa bank_mask:0xf")                                                          \
    "s_nop 1\n\t" M("row_bcast:31 row_mask:0xc bank_mask:0xf")
template <int N>
__device__ __forceinline__ void wave_max_n(float (&v)[N])
{
    static_assert(N == 1 || N == 2 || N == 4 || N == 8, "heads per KV head");
    if constexpr (N == 1) {
        asm("s_nop 4\n\t" Q4KV_MAX_STEPS(Q4KV_MAX_DPP) : "+v"(v[0]));
    } else if constexpr (N == 2) {
        asm("s_nop 4\n\t" Q4KV_MAX_STEPS(Q4KV_MAX_DPP2) : "+v"(v[0]), "+v"(v[1]));
    } else {
#pragma unroll
        for (int i = 0; i < N; i += 4)
            asm("s_nop 4\n\t" Q4KV_MAX_STEPS(Q4KV_MAX_DPP4) : "+v"(v[i]), "+v"(v[i + 1]), "+v"(v[i + 2]), "+v"(v[i + 3]));
    }
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v[i]), 63));
}

__device__ __forceinline__ float wave_sum(float v)
{
    v += Q4KV_DPP(0.0f, v, 0xB1, 0xF);
    v += Q4KV_DPP(0.0f, v, 0x4E, 0xF);
    v += Q4KV_DPP(0.0f, v, 0x141, 0xF);
    v += Q4KV_DPP(0.0f, v, 0x140, 0xF);
    v += Q4KV_DPP(0.0f, v, 0x142, 0xA);
    v += Q4KV_DPP(0.0f, v, 0x143, 0xC);
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

} // namespace q4kv

// Batched decode attention over a shared-latent Q4 cache (Sec. 3.6, the MLA-shaped spec: one latent row per
// token serves as K in full and as V in its first v_dim elements; 16 query heads read it):
//   out[l][a][h] = softmax(sm * q_h C_hat^T) C_hat[:, :v_dim],   C_hat = code*scale + bias   (Sec. 3.2, 3.4)
//
// A cached token costs k_dim/2 + 4*k_dim/64 bytes and 2*16*(k_dim + v_dim) flops, about 100 flop/byte, so the
// pass is still HBM-bound but only if both contractions run on the matrix cores and the vector ALUs do little
// more than unpack nibbles.  Per wave (one per SIMD, 512 registers, no synchronisation between waves):
//
//  * Work decomposition: the stream-K tile stream of stream_k.h, 64-token tiles, one partial (acc, m, l) per
//    (unit, wave) intersection.  The records of a unit (16 heads x 512 values x about 9 waves: 290 KB) are merged by
//    a kernel of their own with one thread per four output values: left to the last wave that leaves the unit, as
//    the GQA decode path does with its far smaller records, the merge took that one wave 50 round trips to memory
//    and the call 0.75 instead of 0.40 ms.
//  * A tile's code rows are contiguous in the pool; they travel HBM -> LDS directly (global_load_lds, 16 bytes
//    per lane) into one of two buffers while the other is being consumed, so no register holds a code word
//    before it is used.  Scale and bias (18 + 18 bytes per token) go through registers and are re-laid in LDS
//    in the two orders the matrix instructions want.
//  * Scores, transposed:  S^T[t][h] = sum_g s[t,g] * (C_g Q_g^T)[t][h] + (b Qsum^T)[t][h].
//    C_g Q_g^T is two v_mfma_f32_16x16x32_f16 per 16 tokens and group: operand A is a code word masked in place
//    (nibbles become binary16 subnormals, see q4_device.h), operand B the query in the matching element order.
//    The bias term is one more instruction per 16 tokens, its contraction index running over the groups with
//    the group sums of q split into binary16 high and low parts.
//  * Row i of a 16-token set is token 4*(i%4) + i/4, so the lane that receives S^T for (head, tokens 4r+q) is
//    the lane that must supply P^T for the same tokens as operand B of the second contraction: probabilities
//    never leave their registers.
//  * Output, transposed:  O^T[e][h] = sum_t c[t,e] * (p[h,t] s[t,g(e)])  +  sum_t b[t,g(e)] p[h,t].
//    Operand A wants 8 tokens of one element per lane while a word holds 8 elements of one token; the lane reads
//    the same word column of 8 rows from LDS (row pitch 72 words: conflict-free), masks the low or the high
//    nibbles once, and v_perm picks byte M of two tokens into one register: rows 0..7 of tile (g, M) are element
//    2M of word columns 8g..8g+7, rows 8..15 element 2M+1 (carrying a factor 16 until the end).
//  * Online softmax per tile of 64 tokens, lane-local denominators, accumulators rescaled only when some
//    head's running maximum moved.
#include "q4_device.h"
#include "q4kv_internal.h"
#include "stream_k.h"

namespace q4kv {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kHeads = 16;          // query heads per latent head: the M (or N) extent of the matrix tiles
constexpr float kNegBig = -1.0e30f; // "minus infinity" that survives subtraction
constexpr float kLog2e = 1.4426950408889634f;

typedef __attribute__((address_space(3))) void *lds_ptr_t;
typedef const __attribute__((address_space(1))) void *global_ptr_t;

struct MlaParams {
    const uint32_t *codes;
    const uint16_t *scale, *bias;
    const uint16_t *q;
    StreamParams stream;
    float *part_acc, *part_ml;
    int q_heads, max_slots;
    float score_scale; // sm_scale * log2(e): scores are kept in log2 units
};

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// x[i] (op) x[i ^ 16], x[i] (op) x[i ^ 32] without touching LDS
__device__ __forceinline__ float xor16_max(float x)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    return fmaxf(__builtin_bit_cast(float, (uint32_t)r[0]), __builtin_bit_cast(float, (uint32_t)r[1]));
}
__device__ __forceinline__ float xor32_max(float x)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__builtin_bit_cast(float, (uint32_t)r[0]), __builtin_bit_cast(float, (uint32_t)r[1]));
}
__device__ __forceinline__ float xor16_sum(float x)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    return __builtin_bit_cast(float, (uint32_t)r[0]) + __builtin_bit_cast(float, (uint32_t)r[1]);
}
__device__ __forceinline__ float xor32_sum(float x)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __builtin_bit_cast(float, (uint32_t)r[0]) + __builtin_bit_cast(float, (uint32_t)r[1]);
}
// the value lane i ^ 16 holds
__device__ __forceinline__ float xor16_other(float x, bool odd_row)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    return __builtin_bit_cast(float, (uint32_t)(odd_row ? r[0] : r[1]));
}

__device__ __forceinline__ half8_t words_to_half8(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    return __builtin_bit_cast(half8_t, make_uint4(a, b, c, d));
}

__device__ __forceinline__ half8_t code_operand(uint32_t w)
{
    const uint32_t w8 = w >> 8;
    return words_to_half8(w & 0x000F000Fu, w & 0x00F000F0u, w8 & 0x000F000Fu, w8 & 0x00F000F0u);
}

__device__ __forceinline__ float half_of(uint32_t pair, int hi)
{
    return half_bits_to_float((uint16_t)(hi ? pair >> 16 : pair & 0xffffu));
}

// GK, GV: quantization groups of the latent row and of its value part (k_dim = 64 GK, v_dim = 64 GV <= k_dim).
// BF: scale and bias are stored as bfloat16; they are converted to binary16 (exactly, for parameters of binary16-range
// data above 2^-14) when a tile's parameters are re-laid in LDS, everything after that is the same.
template <int GK, int GV, bool BF>
__global__ __launch_bounds__(kThreads, 1) void mla_decode_kernel(const MlaParams p)
{
    static_assert(GV <= 8 && GV <= GK && GK <= 10, "group counts");
    constexpr int DK = GK * kGroup, DV = GV * kGroup;
    constexpr int W = DK / 8;               // code words per token row
    constexpr int kTileWords = kWave * W;   // one tile of code rows
    constexpr int kLoads = kTileWords / (kWave * 4); // 1 KiB transfers per tile
    constexpr int BTP = GK > 8 ? 12 : 8;    // binary16 slots per token in the token-major bias copy

    __shared__ __attribute__((aligned(16))) uint32_t codes_all[kWaves][2][kTileWords]; // two tile buffers per wave
    // scale and bias of the tile, [32-token half][group][q][e] <-> token 32*half + 4*e + q: one 16-byte read gives
    // a lane the 8 tokens of its contraction slots
    __shared__ __attribute__((aligned(16))) uint16_t sc_all[kWaves][2][GK][4][8];
    __shared__ __attribute__((aligned(16))) uint16_t bg_all[kWaves][2][GV][4][8];
    // bias again, token-major [64][BTP] (groups 0..7, then groups 8.. and zero padding): operand of the score bias term
    __shared__ __attribute__((aligned(16))) uint16_t bt_all[kWaves][kWave * BTP + 8];

    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = uniform(tid / kWave);
    const int gw = blockIdx.x * kWaves + wave; // this wave's index in the launch

    const TileStream ts(p.stream);
    const int per = ts.per, N = ts.N;
    const long long x_begin = (long long)gw * per;
    if (x_begin >= N) return;
    const int x0 = (int)x_begin;
    const int x1 = (int)min((long long)N, x_begin + per);

    uint32_t *const bufs = &codes_all[wave][0][0];
    uint16_t *const sc = &sc_all[wave][0][0][0][0];
    uint16_t *const bg = &bg_all[wave][0][0][0][0];
    uint16_t *const bt = bt_all[wave];

    // lane roles: col = row of an A operand / column of a B operand or result; qk = the lane's contraction slot
    // (8 of 32 indices) in an operand, the row quad in a result
    const int col = lane % 16, qk = lane / 16;
    const int trow = 4 * (col % 4) + col / 4;       // token (within its 16-token set) behind A row `col`
    const int tok_q = lane % 4, tok_e = (lane % 32) / 4, tok_h2 = lane / 32; // where token `lane` sits in sc / bg
    const uint32_t nibble_mask = col < 8 ? 0x0F0F0F0Fu : 0xF0F0F0F0u;

    typedef CursorT<int> Cursor;
    Cursor cur = ts.locate<Cursor>(x0);

    uint32_t sraw[GK], braw[GK]; // scale / bias bits of token `lane` of the tile in flight

    // Start the transfer of a tile: kLoads instructions move 1 KiB each straight from global memory into LDS
    // (lane i's 16 bytes land at M0 + offset + 16 i), then the lane's scale and bias loads.  The transfers are
    // written as asm statements so that the compiler neither tracks them nor makes later LDS reads of the
    // other buffer wait for them; the tile loop waits for them itself (vmcnt) before it touches the buffer.
    auto issue_tile = [&](const Cursor &c, int buf) __attribute__((always_inline)) {
        const uint32_t *src = p.codes + c.row * W; // wave-uniform
        const uint32_t dst = (uint32_t)(uintptr_t)(lds_ptr_t)(bufs + buf * kTileWords);
        const uint32_t lane_off = lane * 16;
#pragma unroll
        for (int i = 0; i < kLoads; i += 4) {
            const uint32_t *s4k = src + i * (kWave * 4);
            const uint32_t d4k = dst + i * 1024;
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(s4k), "s"(d4k) : "memory", "m0");
            if (i + 1 < kLoads)
                asm volatile("global_load_lds_dwordx4 %0, %1 offset:1024" ::"v"(lane_off), "s"(s4k) : "memory");
            if (i + 2 < kLoads)
                asm volatile("global_load_lds_dwordx4 %0, %1 offset:2048" ::"v"(lane_off), "s"(s4k) : "memory");
            if (i + 3 < kLoads)
                asm volatile("global_load_lds_dwordx4 %0, %1 offset:3072" ::"v"(lane_off), "s"(s4k) : "memory");
        }
        const uint16_t *sp = p.scale + (c.row + lane) * GK;
        const uint16_t *bp = p.bias + (c.row + lane) * GK;
#pragma unroll
        for (int g = 0; g < GK; ++g) {
            sraw[g] = sp[g];
            braw[g] = bp[g];
        }
    };

    half8_t qop[GK][2]; // query operand per (group, word pair member): element order of code_operand, odd elements / 16
    half8_t qsop;       // group sums of q: slots of qk 0 = high parts of groups 0..7, qk 1 = low parts, qk 2 / 3 = groups 8..
    int x = x0;
    int buf = 0;        // tile buffer the current tile arrives in

    issue_tile(cur, 0);
    while (x < x1) {
        // ---- a unit (or the part of it inside this wave's range) begins: its 16 query heads as operand B of the
        // score contraction.  Lane (head col, slot qk) holds, for group g and word r, the 8 elements of word
        // 8g + 2qk + r in the order code_operand emits codes (0,4,1,5,2,6,3,7), odd elements divided by 16
        // because their codes arrive 16 times larger.
        const int64_t unit0 =
            ((int64_t)cur.li * p.stream.num_agents + cur.agent) * p.q_heads + (int64_t)cur.kvh * kHeads;
        int slot, slots_unused;
        ts.slot_of(cur, gw, slot, slots_unused);
        {
            const uint16_t *qrow = p.q + (unit0 + col) * DK + 16 * qk;
            float qs[GK];
#pragma unroll
            for (int g = 0; g < GK; ++g) {
                float sum = 0.0f;
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    const uint4 raw = *reinterpret_cast<const uint4 *>(qrow + g * kGroup + 8 * r);
                    const half2_t e01 = bits_to_half2(raw.x), e23 = bits_to_half2(raw.y);
                    const half2_t e45 = bits_to_half2(raw.z), e67 = bits_to_half2(raw.w);
                    const half_t sixteenth = (half_t)0.0625f;
                    qop[g][r] = half8_t{e01.x, e45.x, e01.y * sixteenth, e45.y * sixteenth,
                                        e23.x, e67.x, e23.y * sixteenth, e67.y * sixteenth};
                    sum += ((float)e01.x + (float)e01.y) + ((float)e23.x + (float)e23.y) +
                           ((float)e45.x + (float)e45.y) + ((float)e67.x + (float)e67.y);
                }
                qs[g] = xor32_sum(xor16_sum(sum)); // all four slots of a head now hold the group's sum
            }
            half_t part[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                // slot qk, element e: qk 0 -> high part of group e, qk 1 -> low part of group e,
                // qk 2 -> high part of group 8 + e, qk 3 -> low part of group 8 + e
                const float lo_grp = e < GK ? qs[e] : 0.0f;
                const float hi_grp = 8 + e < GK ? qs[(8 + e) < GK ? 8 + e : 0] : 0.0f;
                const float v = qk >= 2 ? hi_grp : lo_grp;
                const half_t hi = (half_t)v;
                part[e] = (qk & 1) ? (half_t)(v - (float)hi) : hi;
            }
            qsop = half8_t{part[0], part[1], part[2], part[3], part[4], part[5], part[6], part[7]};
        }
        float4_t acc[GV][4]; // [group][byte M]: rows = (word column, low / high nibble), columns = heads
        float4_t pbacc = float4_t{0.0f, 0.0f, 0.0f, 0.0f}; // rows = groups: sum_t b[t,g] p[h,t]
#pragma unroll
        for (int g = 0; g < GV; ++g)
#pragma unroll
            for (int m = 0; m < 4; ++m) acc[g][m] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
        float m_run = kNegBig, l_run = 0.0f; // of head `col`; l_run covers this lane's tokens only
        bool first_tile = true, unit_ends;

        do { // ---- the tiles of the unit
            const uint32_t *cb = bufs + buf * kTileWords;
            const bool last_of_wave = x + 1 >= x1;
            Cursor nxt = cur;
            if (!last_of_wave) ts.step(nxt); // the wave's last tile re-reads itself: a valid address, the data is ignored
            unit_ends = last_of_wave || nxt.j == 0;

            // everything of this tile has landed: codes in `cb`, scale / bias in registers
            __builtin_amdgcn_s_waitcnt(0x0F70); // vmcnt(0)
            const int tok = cur.t0 + lane;
            const bool tok_valid = cur.reachable && tok >= cur.first && tok < cur.n;
            // wave-uniform: some token of the tile lies outside the agent's visible range
            const bool edge = !(cur.reachable && cur.t0 >= cur.first && cur.t0 + kWave <= cur.n);
            {
                // rows outside the agent's range may hold anything: their scale and bias become zero so that no NaN
                // or infinity reaches a matrix operand (codes are nibbles and always finite)
                uint32_t s[GK], b[BTP];
#pragma unroll
                for (int g = 0; g < GK; ++g) {
                    s[g] = BF ? (uint32_t)float_to_half_bits(bf16_bits_to_float((uint16_t)sraw[g])) : sraw[g];
                    b[g] = BF ? (uint32_t)float_to_half_bits(bf16_bits_to_float((uint16_t)braw[g])) : braw[g];
                }
                if (edge) { // interior tiles (nearly all) skip the selects
#pragma unroll
                    for (int g = 0; g < GK; ++g) {
                        s[g] = tok_valid ? s[g] : 0u;
                        b[g] = tok_valid ? b[g] : 0u;
                    }
                }
#pragma unroll
                for (int g = GK; g < BTP; ++g) b[g] = 0u;
#pragma unroll
                for (int g = 0; g < GK; ++g) sc[((tok_h2 * GK + g) * 4 + tok_q) * 8 + tok_e] = (uint16_t)s[g];
#pragma unroll
                for (int g = 0; g < GV; ++g) bg[((tok_h2 * GV + g) * 4 + tok_q) * 8 + tok_e] = (uint16_t)b[g];
                uint2 *btw = reinterpret_cast<uint2 *>(bt + lane * BTP);
#pragma unroll
                for (int i = 0; i < BTP / 4; ++i)
                    btw[i] = make_uint2(b[4 * i] | (b[4 * i + 1] << 16), b[4 * i + 2] | (b[4 * i + 3] << 16));
            }
            // the next tile starts travelling (into the buffer the previous tile was read from)
            issue_tile(nxt, buf ^ 1);
            __builtin_amdgcn_sched_barrier(0);
            wave_lds_sync();

            // LDS reads are issued ahead of their use (one 16-token set, two value groups) and fenced so that
            // they stay there: with one wave per SIMD nothing else hides their latency.  LDS returns data in
            // issue order, so a step waits only for its own operands while the later ones are still on their way.
            struct SetIn {    // operands of one 16-token set of scores
                uint2 w[GK];  // code words 8g + 2qk, 8g + 2qk + 1 of this lane's row
                uint2 s4[GK]; // scale of the four tokens this lane gets results for
                uint2 b0, b1; // bias row (slots as in qsop)
            };
            auto load_set = [&](int h2, int sub) __attribute__((always_inline)) {
                SetIn in;
                const int t_row = 32 * h2 + 16 * sub + trow; // this lane's A row
#pragma unroll
                for (int g = 0; g < GK; ++g) in.w[g] = *reinterpret_cast<const uint2 *>(cb + t_row * W + 8 * g + 2 * qk);
#pragma unroll
                for (int g = 0; g < GK; ++g)
                    in.s4[g] = *reinterpret_cast<const uint2 *>(sc + ((h2 * GK + g) * 4 + qk) * 8 + 4 * sub);
                const uint16_t *btp = bt + t_row * BTP + ((GK > 8 && qk >= 2) ? 8 : 0);
                in.b0 = *reinterpret_cast<const uint2 *>(btp);
                in.b1 = *reinterpret_cast<const uint2 *>(btp + 4);
                return in;
            };
            struct GroupIn {    // operands of one (32-token half, value group) step
                uint32_t w[8];  // word column 8g + col % 8 of tokens 32 h2 + 4 e + qk
                uint4 s8;       // their scales
            };
            auto load_group = [&](int step) __attribute__((always_inline)) { // step = h2 * GV + g
                GroupIn in;
                const int h2 = step / GV, g = step % GV;
#pragma unroll
                for (int e = 0; e < 8; ++e) in.w[e] = cb[(32 * h2 + 4 * e + qk) * W + 8 * g + (col % 8)];
                in.s8 = *reinterpret_cast<const uint4 *>(sc + ((h2 * GK + g) * 4 + qk) * 8);
                return in;
            };

            // ---- scores of the 64 tokens, four 16-token sets: z[h2][sub][r] is token 32 h2 + 16 sub + 4 r + qk, head col
            float z[2][2][4];
            const float c_code = p.score_scale * kCodeScaleA;
            const float4_t zero = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
            SetIn set_in = load_set(0, 0);
            constexpr int kRing = 2; // deeper rings (3, 4) were measured and change nothing
            GroupIn grp_in[kRing]; // a ring of the next value steps
#pragma unroll
            for (int set = 0; set < 4; ++set) {
                const int h2 = set / 2, sub = set % 2;
                SetIn set_next;
                if (set < 3) {
                    set_next = load_set((set + 1) / 2, (set + 1) % 2);
                } else {
#pragma unroll
                    for (int i = 0; i < kRing; ++i) grp_in[i] = load_group(i);
                }
                __builtin_amdgcn_sched_barrier(0);
                float4_t d[GK];
#pragma unroll
                for (int g = 0; g < GK; ++g) {
                    d[g] = __builtin_amdgcn_mfma_f32_16x16x32_f16(code_operand(set_in.w[g].x), qop[g][0], zero, 0, 0, 0);
                    d[g] = __builtin_amdgcn_mfma_f32_16x16x32_f16(code_operand(set_in.w[g].y), qop[g][1], d[g], 0, 0, 0);
                }
                // bias term: A = b[t][.], B = group sums of q
                uint2 b0 = set_in.b0, b1 = set_in.b1;
                if (qk >= 2) {
                    b1 = make_uint2(0u, 0u);
                    if (GK <= 8) b0 = make_uint2(0u, 0u);
                }
                const float4_t bterm =
                    __builtin_amdgcn_mfma_f32_16x16x32_f16(words_to_half8(b0.x, b0.y, b1.x, b1.y), qsop, zero, 0, 0, 0);
                float4_t s_acc = zero;
#pragma unroll
                for (int g = 0; g < GK; ++g) {
                    s_acc[0] = fmaf(half_of(set_in.s4[g].x, 0), d[g][0], s_acc[0]);
                    s_acc[1] = fmaf(half_of(set_in.s4[g].x, 1), d[g][1], s_acc[1]);
                    s_acc[2] = fmaf(half_of(set_in.s4[g].y, 0), d[g][2], s_acc[2]);
                    s_acc[3] = fmaf(half_of(set_in.s4[g].y, 1), d[g][3], s_acc[3]);
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) z[h2][sub][r] = fmaf(s_acc[r], c_code, bterm[r] * p.score_scale);
                // pin the scores here: without a use in this block the compiler sinks all the scale multiplies
                // below the branch that follows and keeps every matrix result of the tile alive until then
                asm volatile("" : "+v"(z[h2][sub][0]), "+v"(z[h2][sub][1]), "+v"(z[h2][sub][2]), "+v"(z[h2][sub][3]));
                __builtin_amdgcn_sched_barrier(0);
                if (set < 3) set_in = set_next;
            }

            // ---- online softmax of head col over the tile.  m_run is the reference the exponentials are taken
            // against, not the exact running maximum: it moves only when a tile's maximum exceeds it by more than
            // kSlack (in log2 units), so p <= 2^kSlack and p * s stays far inside binary16 for any binary16 scale,
            // and the accumulators are rescaled a handful of times per unit instead of in every other tile.
            constexpr float kSlack = 3.0f;
            if (edge) {
#pragma unroll
                for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
                    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int t = cur.t0 + 32 * h2 + 16 * sub + 4 * r + qk;
                            if (!(cur.reachable && t >= cur.first && t < cur.n)) z[h2][sub][r] = kNegBig;
                        }
            }
            float mt = kNegBig;
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
                for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                    for (int r = 0; r < 4; ++r) mt = fmaxf(mt, z[h2][sub][r]);
            mt = xor32_max(xor16_max(mt));
            const bool moved = mt > m_run + kSlack; // the same in the four lanes of a head
            const float m_new = moved ? mt : m_run;
            const float alpha = moved ? __builtin_amdgcn_exp2f(m_run - m_new) : 1.0f;
            m_run = m_new;
            float psum = 0.0f;
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
                for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float pr = __builtin_amdgcn_exp2f(z[h2][sub][r] - m_new);
                        if (edge && z[h2][sub][r] == kNegBig) pr = 0.0f; // also when the whole tile is masked
                        z[h2][sub][r] = pr;
                        psum += pr;
                    }
            l_run = fmaf(l_run, alpha, psum);
            if (!first_tile && __builtin_amdgcn_ballot_w64(moved) != 0ull) { // accumulators are zero in a unit's first tile
                // Rare.  The empty asm statements tie the accumulators to the accumulator registers on entry, and
                // the products are handed back through a matrix instruction with zero operands (0*0 + C = C) whose
                // result lives there again: on the path that skips this block the accumulators then never move.
                const half8_t none = half8_t{0, 0, 0, 0, 0, 0, 0, 0};
                asm volatile("" : "+a"(pbacc));
                pbacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(none, none, pbacc * alpha, 0, 0, 0);
#pragma unroll
                for (int g = 0; g < GV; ++g)
#pragma unroll
                    for (int m = 0; m < 4; ++m) {
                        asm volatile("" : "+a"(acc[g][m]));
                        acc[g][m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(none, none, acc[g][m] * alpha, 0, 0, 0);
                    }
            }

            // ---- values: per 32-token half, B = p * s of tokens 32 h2 + 4 e + qk, e = 0..7, in two binary16 terms.
            // The product of two binary16 numbers minus its rounded value is a binary16 number again (barring
            // underflow), so hi + lo carries p s to about 22 bits.  With hi alone an agent of a handful of tokens,
            // where one or two rounding errors of p s make up the whole error of an output, can leave the tolerance
            // when the latent holds channels of several times the usual magnitude.
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2) {
                half2_t p16[4];
                p16[0] = half2_t{(half_t)z[h2][0][0], (half_t)z[h2][0][1]};
                p16[1] = half2_t{(half_t)z[h2][0][2], (half_t)z[h2][0][3]};
                p16[2] = half2_t{(half_t)z[h2][1][0], (half_t)z[h2][1][1]};
                p16[3] = half2_t{(half_t)z[h2][1][2], (half_t)z[h2][1][3]};
                const half8_t pop = words_to_half8(half2_to_bits(p16[0]), half2_to_bits(p16[1]), half2_to_bits(p16[2]),
                                                   half2_to_bits(p16[3]));
                const int g_row = (col % 8) < GV ? (col % 8) : GV - 1; // rows past GV repeat a valid row, unused
                const uint4 braw4 = *reinterpret_cast<const uint4 *>(bg + ((h2 * GV + g_row) * 4 + qk) * 8);
#pragma unroll
                for (int g = 0; g < GV; ++g) {
                    const int step = h2 * GV + g;
                    const GroupIn in = grp_in[step % kRing];
                    if (step + kRing < 2 * GV) grp_in[step % kRing] = load_group(step + kRing);
                    __builtin_amdgcn_sched_barrier(0);
                    const half2_t s2[4] = {bits_to_half2(in.s8.x), bits_to_half2(in.s8.y), bits_to_half2(in.s8.z),
                                           bits_to_half2(in.s8.w)};
                    half2_t hi[4], lo[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        hi[i] = p16[i] * s2[i];
                        lo[i] = __builtin_elementwise_fma(p16[i], s2[i], -hi[i]);
                    }
                    const half8_t ps_hi = words_to_half8(half2_to_bits(hi[0]), half2_to_bits(hi[1]), half2_to_bits(hi[2]),
                                                         half2_to_bits(hi[3]));
                    const half8_t ps_lo = words_to_half8(half2_to_bits(lo[0]), half2_to_bits(lo[1]), half2_to_bits(lo[2]),
                                                         half2_to_bits(lo[3]));
                    uint32_t wm[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) wm[e] = in.w[e] & nibble_mask;
#pragma unroll
                    for (int m = 0; m < 4; ++m) {
                        const uint32_t sel = 0x0C040C00u + m * 0x00010001u; // byte m of two tokens into the low bytes of two halves
                        const half8_t cop =
                            words_to_half8(__builtin_amdgcn_perm(wm[1], wm[0], sel), __builtin_amdgcn_perm(wm[3], wm[2], sel),
                                           __builtin_amdgcn_perm(wm[5], wm[4], sel), __builtin_amdgcn_perm(wm[7], wm[6], sel));
                        acc[g][m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(cop, ps_hi, acc[g][m], 0, 0, 0);
                        acc[g][m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(cop, ps_lo, acc[g][m], 0, 0, 0);
                    }
                    if (g == GV - 1) // bias sums of this half: rows = groups
                        pbacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(words_to_half8(braw4.x, braw4.y, braw4.z, braw4.w), pop,
                                                                       pbacc, 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            wave_lds_sync(); // the next tile rewrites sc / bg / bt
            first_tile = false;
            cur = nxt;
            buf ^= 1;
            ++x;
        } while (!unit_ends);

        // ---- this wave's share of the unit is complete: one partial per query head, written straight from the
        // accumulators.  Lane (head col, quad qk) holds rows 4 qk + r of every tile: word column
        // 8 g + 4 (qk % 2) + r, nibble 2 m + qk / 2; of the bias sums it holds groups 4 (qk % 2) + r.
        const float l_tot = xor32_sum(xor16_sum(l_run));
        const bool odd = (qk & 1) != 0;
        float pb[8];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float other = xor16_other(pbacc[r], odd);
            pb[r] = odd ? other : pbacc[r];
            pb[4 + r] = odd ? pbacc[r] : other;
        }
        const int64_t rec = (unit0 + col) * p.max_slots + slot;
        float *dst = p.part_acc + rec * DV + 8 * (4 * (qk % 2)) + qk / 2;
        const float unscale = qk >= 2 ? kCodeScaleB : kCodeScaleA;
#pragma unroll
        for (int g = 0; g < GV; ++g)
#pragma unroll
            for (int m = 0; m < 4; ++m)
#pragma unroll
                for (int r = 0; r < 4; ++r) dst[kGroup * g + 8 * r + 2 * m] = fmaf(acc[g][m][r], unscale, pb[g]);
        if (qk == 0) {
            p.part_ml[rec * 2] = m_run;
            p.part_ml[rec * 2 + 1] = l_tot;
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70); // the last tile's look-ahead transfer must land before the LDS is released
}

// Merge the partials of every (layer, agent, query head) in slot order: binary32, output binary16.  A thread owns
// four consecutive output elements of one head (16-byte loads); v_dim / 4 threads share a head.
__global__ __launch_bounds__(kThreads) void combine_kernel(const float *__restrict__ part_acc,
                                                           const float *__restrict__ part_ml,
                                                           const int32_t *__restrict__ plan, uint16_t *__restrict__ out,
                                                           int q_heads, int kv_heads, int num_agents, int v_dim,
                                                           int max_slots, int layers, long long units, int signature)
{
    if (plan[5] != signature) return; // a plan made for other arguments: the attention launch did nothing either
    const int threads_per_unit = v_dim / 4;
    const long long unit = (long long)blockIdx.x * (kThreads / threads_per_unit) + threadIdx.x / threads_per_unit;
    if (unit >= units) return; // (layer in call, agent, query head)
    const int e = (threadIdx.x % threads_per_unit) * 4;
    const int qh = (int)(unit % q_heads);
    const int agent = (int)((unit / q_heads) % num_agents);
    const int li = (int)(unit / ((long long)q_heads * num_agents));
    const int kvh = qh / (q_heads / kv_heads);
    PlanView pv;
    pv.plan = plan;
    pv.A = num_agents;
    pv.L = layers;
    const int per = plan[1];
    const int cb = pv.layer_class_off(li);
    const int32_t *tpre = pv.tpre(cb);
    const int tiles = tpre[agent + 1] - tpre[agent];
    int slots = 0;
    if (tiles > 0) {
        const long long u0 = (long long)plan[pv.lt_off() + li] + (long long)kvh * pv.tiles_per_head(cb) + tpre[agent];
        slots = (int)((u0 + tiles - 1) / per - u0 / per) + 1;
    }
    const float *ml = part_ml + unit * max_slots * 2;
    const float *acc = part_acc + unit * max_slots * v_dim + e;
    // Four slots at a time: every load of a group is issued before anything is computed, so a unit costs one
    // memory round trip per group instead of two dependent ones per slot.  The running reference moves group by
    // group (with at most four slots: exactly the maximum over all slots, then one weighted sum in slot order).
    float m = kNegBig, denom = 0.0f;
    float4 o = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    for (int s0 = 0; s0 < slots; s0 += 4) {
        float mm[4], ll[4];
        float4 a[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const bool in = s0 + k < slots;
            const float2 t = in ? *reinterpret_cast<const float2 *>(ml + 2 * (s0 + k)) : make_float2(kNegBig, 0.0f);
            mm[k] = t.x;
            ll[k] = t.y;
            a[k] = in ? *reinterpret_cast<const float4 *>(acc + (long long)(s0 + k) * v_dim) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        }
        float m_new = m;
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (ll[k] > 0.0f) m_new = fmaxf(m_new, mm[k]);
        const float keep = __builtin_amdgcn_exp2f(m - m_new); // 1 when the reference stays, 0 while nothing was added yet
        denom *= keep;
        o.x *= keep; o.y *= keep; o.z *= keep; o.w *= keep;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (!(ll[k] > 0.0f)) continue;
            const float wgt = __builtin_amdgcn_exp2f(mm[k] - m_new);
            denom = fmaf(wgt, ll[k], denom);
            o.x = fmaf(wgt, a[k].x, o.x);
            o.y = fmaf(wgt, a[k].y, o.y);
            o.z = fmaf(wgt, a[k].z, o.z);
            o.w = fmaf(wgt, a[k].w, o.w);
        }
        m = m_new;
    }
    const float inv = denom > 0.0f ? 1.0f / denom : 0.0f;
    const uint32_t lo = (uint32_t)float_to_half_bits(o.x * inv) | ((uint32_t)float_to_half_bits(o.y * inv) << 16);
    const uint32_t hi = (uint32_t)float_to_half_bits(o.z * inv) | ((uint32_t)float_to_half_bits(o.w * inv) << 16);
    *reinterpret_cast<uint2 *>(out + unit * v_dim + e) = make_uint2(lo, hi);
}

hipError_t launch_combine(const AttentionArgs &a, hipStream_t stream)
{
    const int64_t units = (int64_t)a.layers_in_call * a.num_agents * a.q_len * a.spec.num_q_heads;
    if (units == 0) return hipSuccess;
    const int units_per_block = kThreads / (a.spec.v_dim / 4); // v_dim is a multiple of 64 and at most 1,024 here
    const int64_t blocks = (units + units_per_block - 1) / units_per_block;
    hipLaunchKernelGGL(combine_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, a.part_acc, a.part_ml, a.plan,
                       a.out, a.spec.num_q_heads, a.spec.num_kv_heads, a.num_agents, a.spec.v_dim, a.max_slots,
                       a.layers_in_call, (long long)units, a.plan_signature);
    return hipGetLastError();
}

template <int GK, int GV, bool BF>
hipError_t launch_mla_t(const AttentionArgs &a, hipStream_t stream)
{
    MlaParams p;
    p.codes = a.k.codes; p.scale = a.k.scale; p.bias = a.k.bias;
    p.q = a.q;
    p.stream = stream_params(a);
    p.part_acc = a.part_acc; p.part_ml = a.part_ml;
    p.q_heads = a.spec.num_q_heads;
    p.max_slots = a.max_slots;
    p.score_scale = a.sm_scale * kLog2e;
    hipLaunchKernelGGL((mla_decode_kernel<GK, GV, BF>), dim3(a.grid_workgroups), dim3(kThreads), 0, stream, p);
    return hipGetLastError();
}

} // namespace

bool mla_decode_supported(const q4kv_spec &s)
{
    return s.v_aliases_k && s.num_q_heads == kHeads * s.num_kv_heads && s.k_dim == 576 && s.v_dim == 512;
}

// every wave walks a tile range of its own
hipError_t launch_mla_decode_plan(const AttentionArgs &a, hipStream_t stream)
{
    return launch_plan(a, a.grid_workgroups * kWaves, 1, stream);
}

hipError_t launch_mla_decode_attention(const AttentionArgs &a, hipStream_t stream)
{
    hipError_t e = a.spec.param_format == Q4KV_PARAMS_BF16 ? launch_mla_t<9, 8, true>(a, stream) : launch_mla_t<9, 8, false>(a, stream);
    return e == hipSuccess ? launch_combine(a, stream) : e;
}

} // namespace q4kv

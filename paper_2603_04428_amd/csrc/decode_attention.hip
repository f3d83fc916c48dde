// Batched decode attention (one query token per agent) over paged Q4 KV caches, GQA form:
//   out[l][a][h] = softmax(sm * q K_hat^T) V_hat   over the agent's cached tokens,
// K_hat / V_hat = code*scale + bias, never materialised (Sec. 3.2 item 3, Sec. 3.4, Sec. 3.6).
//
// The step is a single pass over the cache and is HBM-bound: per cached token and KV head it reads
// DK/2 + DV/2 bytes of codes and 4 bytes of scale/bias per 64-wide group, once, for all n_rep
// query heads of the group.  The design follows from keeping the vector ALUs under that stream:
//
//  * split-K: a workgroup owns (layer, agent, KV head, split of `split_tokens` tokens) and emits an
//    un-normalised partial (acc[DV], running max m, denominator l) per query head; a small combine
//    kernel merges the splits in a fixed order, so results are run-to-run identical.
//  * inside a workgroup each of the 4 waves walks its own 64-token tiles (slots 64w..64w+63 of every
//    256-token block) with private online-softmax state; waves meet only once, at the end.
//  * codes never become integers or binary32: a nibble masked in place is a binary16 subnormal
//    (c*2^-24 or c*2^-20) and goes straight into the matrix core (K side) or v_dot2_f32_f16 (V side).
//  * the affine part of the dequantization is factored out of the inner loops:
//        q . K_hat[t]   = sum_g  s[t,g] * (q_g . c[t,g])  +  b[t,g] * sum(q_g)
//        sum_t p_t V_hat[t,e] = sum_t (p_t s[t,g(e)]) c[t,e]  +  sum_t p_t b[t,g(e)]
//    so scale and bias are touched once per (token, group), by the lane that owns the token.
//  * K side: q_g . c[t,g] is a contraction over head_dim with the codes laid out exactly as the matrix
//    core wants its K-index (8 consecutive dims per 32-bit word), so it runs as v_mfma_f32_16x16x32_f16:
//    16 tokens are the N columns, the rows are (query head, group-in-chunk) pairs, and the cross-lane
//    sum over head_dim -- the expensive part on the vector ALUs -- comes for free.  A lane loads 16 bytes
//    (4 words) of one token row; the four lanes that share a token cover a 64-byte chunk = two groups,
//    and the query operand is zeroed outside a row's own group so that one instruction yields both
//    groups' partial dot products separately.
//  * V side: the contraction runs over tokens while a word holds 8 dims of one token, so the matrix
//    core's operand shape does not fit; each lane owns 8*VW output dims, pairs the codes of two tokens
//    with v_perm and multiplies them with the binary16 pair (p s)[t], (p s)[t'] in one v_dot2_f32_f16.
#include <type_traits>

#include "q4_device.h"
#include "q4kv_internal.h"

namespace q4kv {
namespace {

#ifndef Q4KV_DEC_WAVES_PER_EU
#define Q4KV_DEC_WAVES_PER_EU 2 // resident waves per SIMD the register budget is sized for
#endif
constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr float kNegBig = -1.0e30f; // "minus infinity" that survives subtraction
constexpr float kLog2e = 1.4426950408889634f;

struct DecodeParams {
    const uint32_t *k_codes, *v_codes;
    const uint16_t *k_scale, *k_bias, *v_scale, *v_bias;
    const uint16_t *q;
    const int32_t *block_table, *seq_len;
    float *part_acc, *part_ml;
    int num_blocks, kv_heads, q_heads, num_agents, max_blocks, max_seq_len, window, split_tokens, num_splits;
    int layer_begin;
    int v_row_words, v_row_groups; // row pitch of the V pool in words / groups (K's pitch when V aliases K)
    float score_scale;             // sm_scale * log2(e): scores are kept in log2 units
};

// One token's scales or biases (N binary16 values, N = 1, 2 or a multiple of 4) as raw bits: loaded with one
// 2-, 4- or 8-byte load per 4 values and converted only where they are used, so that issuing the load never
// makes the wave wait for it.
template <int N>
struct GroupBits {
    uint32_t w[(N + 1) / 2];
};

template <int N>
__device__ __forceinline__ GroupBits<N> load_groups(const uint16_t *p)
{
    GroupBits<N> r;
    if constexpr (N == 1) {
        r.w[0] = *p;
    } else if constexpr (N == 2) {
        r.w[0] = *reinterpret_cast<const uint32_t *>(p);
    } else {
        static_assert(N % 4 == 0, "group count");
#pragma unroll
        for (int i = 0; i < N / 4; ++i) {
            const uint2 t = reinterpret_cast<const uint2 *>(p)[i];
            r.w[2 * i] = t.x;
            r.w[2 * i + 1] = t.y;
        }
    }
    return r;
}

template <int N>
__device__ __forceinline__ float group_value(const GroupBits<N> &b, int g)
{
    return half_bits_to_float((uint16_t)((g & 1) ? (b.w[g / 2] >> 16) : (b.w[g / 2] & 0xffffu)));
}

template <int W>
struct Words {
    uint32_t w[W];
};

template <int W>
__device__ __forceinline__ Words<W> load_words(const uint32_t *p)
{
    Words<W> r;
    if constexpr (W == 4) {
        const uint4 t = *reinterpret_cast<const uint4 *>(p);
        r.w[0] = t.x; r.w[1] = t.y; r.w[2] = t.z; r.w[3] = t.w;
    } else if constexpr (W == 2) {
        const uint2 t = *reinterpret_cast<const uint2 *>(p);
        r.w[0] = t.x; r.w[1] = t.y;
    } else {
        r.w[0] = *p;
    }
    return r;
}

// DK, DV: head widths (multiples of 64, DK/8 and DV/8 divisible by KW and VW); NREP query heads per KV head.
// KW / VW: 32-bit words of codes a lane takes per load on the K / V side.
//
// Loads are never predicated: a tile's 64 rows always exist inside its block, so rows past the agent's
// length are read and then ignored (their score is forced to "minus infinity", their p*s to zero; codes
// are nibbles and cannot produce a NaN, scale/bias of such rows are replaced by zero after the load).
template <int DK, int DV, int NREP, int KW, int VW>
__global__ __launch_bounds__(kThreads, Q4KV_DEC_WAVES_PER_EU) void decode_attention_kernel(DecodeParams p)
{
    constexpr int GK = DK / kGroup, GV = DV / kGroup;
    // K side (matrix core): lane = (token j = lane % 16 of a 16-token set, k-block kb = lane / 16)
    constexpr int KWPL = DK >= 128 ? 4 : 2;        // words a lane loads per chunk (16 or 8 bytes)
    constexpr int KCHUNKS = DK / (32 * KWPL);      // chunks per row: 4 lanes * KWPL words each
    constexpr int KGPC = KWPL == 4 ? 2 : 1;        // quantization groups per chunk
    constexpr int KSETS = kWave / 16;              // 16-token sets per tile
    constexpr int KROWS = NREP * KGPC;             // distinct rows of the query operand
    static_assert(KW == 4 && KROWS <= 16 && KCHUNKS * KGPC == GK, "K layout");
    constexpr int VLPT = DV / (8 * VW);
    constexpr int VTPS = kWave / VLPT;
    constexpr int VSTEPS = kWave / VTPS;
    constexpr int VLPG = kGroup / (8 * VW);
    static_assert(VLPT <= kWave && VLPG >= 1 && VSTEPS % 2 == 0, "lane layout");

    // per wave: q.c per token, group and head [64][GK][NREP] (binary32) and p*scale [NREP][GV][64] (binary16,
    // tokens of consecutive V load steps interleaved so that a pair sits in one 32-bit word)
    constexpr int kPartFloats = kWave * GK * NREP;
    constexpr int kPsFloats = NREP * GV * kWave / 2;
    constexpr int kWaveFloats = kPartFloats + kPsFloats;
    constexpr int kFinalFloats = kWaves * VTPS * NREP * DV + kWaves * NREP * GV + 2 * kWaves * NREP;
    constexpr int kLdsFloats = (kWaves * kWaveFloats > kFinalFloats ? kWaves * kWaveFloats : kFinalFloats) + NREP * GK;
    __shared__ float lds[kLdsFloats];

    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave); // wave-uniform, so tile addresses stay scalar
    const int split = blockIdx.x;
    const int kvh = blockIdx.y % p.kv_heads, agent = blockIdx.y / p.kv_heads;
    const int li = blockIdx.z, layer = p.layer_begin + li;

    int n = p.seq_len[agent];
    n = n < p.max_seq_len ? n : p.max_seq_len;
    const int first = (p.window > 0 && n > p.window) ? n - p.window : 0;
    const int t_begin = split * p.split_tokens;
    if (t_begin >= n) return; // the combine kernel never looks at splits past the agent's length
    const int t_end = min(n, t_begin + p.split_tokens);

    const int64_t unit0 = ((int64_t)li * p.num_agents + agent) * p.q_heads + (int64_t)kvh * NREP;
    if (t_end <= first) { // split lies wholly before the window: an empty partial
        if (tid < NREP) {
            float *ml = p.part_ml + ((unit0 + tid) * p.num_splits + split) * 2;
            ml[0] = kNegBig;
            ml[1] = 0.0f;
        }
        return;
    }

    float *qsum_lds = lds + (kLdsFloats - NREP * GK); // sum of q over each 64-wide group, [NREP][GK]
    const uint16_t *qrow = p.q + unit0 * DK;           // NREP consecutive query heads
    if (tid < NREP * GK * 8) { // eight lanes per 64-wide group, 8 dims each, folded inside the octet
        const uint4 raw = *reinterpret_cast<const uint4 *>(qrow + tid * 8);
        const half2_t a = bits_to_half2(raw.x), b = bits_to_half2(raw.y), c = bits_to_half2(raw.z), d = bits_to_half2(raw.w);
        float s = ((float)a.x + (float)a.y) + ((float)b.x + (float)b.y) + ((float)c.x + (float)c.y) + ((float)d.x + (float)d.y);
        s += Q4KV_DPP(0.0f, s, 0xB1, 0xF);  // quad_perm [1,0,3,2]
        s += Q4KV_DPP(0.0f, s, 0x4E, 0xF);  // quad_perm [2,3,0,1]
        s += Q4KV_DPP(0.0f, s, 0x141, 0xF); // row_half_mirror
        if ((tid & 7) == 0) qsum_lds[tid >> 3] = s;
    }

    // Query operand of the matrix core, one per (chunk, word): row i = lane % 16 stands for query head
    // i % NREP and group-in-chunk (i / NREP) % KGPC; the lane holds the 8 dims of its k-block in the order
    // unpack_codes emits codes (0,4,1,5,2,6,3,7), odd dims divided by 16 because their codes arrive 16 times
    // larger, and zeros when its k-block belongs to the row's other group.
    const int kj = lane % 16, kkb = lane / 16;
    half8_t qop[KCHUNKS][KWPL];
    {
        const int r = kj % NREP, u = (kj / NREP) % KGPC;
        const bool mine = (KGPC == 1) || (u == kkb / 2);
#pragma unroll
        for (int c = 0; c < KCHUNKS; ++c)
#pragma unroll
            for (int w = 0; w < KWPL; ++w) {
                const uint16_t *src = qrow + r * DK + c * (32 * KWPL) + kkb * (8 * KWPL) + 8 * w;
                const uint4 raw = *reinterpret_cast<const uint4 *>(src);
                const half2_t e01 = bits_to_half2(raw.x), e23 = bits_to_half2(raw.y);
                const half2_t e45 = bits_to_half2(raw.z), e67 = bits_to_half2(raw.w);
                const half_t sixteenth = (half_t)0.0625f;
                half8_t v = {e01.x, e45.x, e01.y * sixteenth, e45.y * sixteenth,
                             e23.x, e67.x, e23.y * sixteenth, e67.y * sixteenth};
                if (!mine) v = half8_t{0, 0, 0, 0, 0, 0, 0, 0};
                qop[c][w] = v;
            }
    }
    __syncthreads();
    float qsum[NREP][GK];
#pragma unroll
    for (int r = 0; r < NREP; ++r)
#pragma unroll
        for (int g = 0; g < GK; ++g) qsum[r][g] = qsum_lds[r * GK + g];

    float *part = lds + wave * kWaveFloats;                               // [64][GK][NREP]
    uint16_t *ps_h = reinterpret_cast<uint16_t *>(part + kPartFloats);     // [NREP][GV][64] binary16
    const uint32_t *ps_w = reinterpret_cast<const uint32_t *>(ps_h);      // the same as token pairs

    const int vj = lane % VLPT, vo = lane / VLPT, vg = vj / VLPG;
    // where the token owned by this lane (local index `lane` = step*VTPS + slot) goes in ps_h
    const int ps_slot = 2 * VTPS * ((lane / VTPS) / 2) + 2 * (lane % VTPS) + ((lane / VTPS) & 1);
    float acc[NREP][8 * VW]; // odd dims carry an extra factor 16 until the end (their codes sit 4 bits higher)
#pragma unroll
    for (int r = 0; r < NREP; ++r)
#pragma unroll
        for (int e = 0; e < 8 * VW; ++e) acc[r][e] = 0.0f;
    float m_run[NREP], l_run[NREP], pb[NREP][GV]; // l_run, pb: this lane's tokens only
#pragma unroll
    for (int r = 0; r < NREP; ++r) {
        m_run[r] = kNegBig;
        l_run[r] = 0.0f;
#pragma unroll
        for (int g = 0; g < GV; ++g) pb[r][g] = 0.0f;
    }

    const int32_t *table = p.block_table + (int64_t)agent * p.max_blocks;
    const int b_end = (t_end + kBlockTokens - 1) / kBlockTokens;
    // next block index >= bi whose 64-token tile of this wave holds visible tokens of a valid block
    auto next_tile = [&](int bi, int64_t &row0) {
        for (; bi < b_end; ++bi) {
            const int t0 = bi * kBlockTokens + wave * kWave;
            if (t0 >= t_end || t0 + kWave <= first) continue;
            const int blk = table[bi];
            if (blk < 0 || blk >= p.num_blocks) continue;
            row0 = (((int64_t)layer * p.num_blocks + blk) * p.kv_heads + kvh) * kBlockTokens + wave * kWave;
            return bi;
        }
        return b_end;
    };

    Words<KWPL> kc[KSETS][KCHUNKS];
    Words<VW> vc[VSTEPS];
    GroupBits<GK> ks_bits, kb_bits;
    GroupBits<GV> vs_bits, vb_bits;
    // tile base (uniform, from row0) + a fixed per-lane offset + a compile-time step offset
    const int k_lane_off = kj * (DK / 8) + kkb * KWPL;
    const int v_lane_off = vo * p.v_row_words + vj * VW;
    auto load_k = [&](int64_t row0) {
        const uint32_t *tile = p.k_codes + row0 * (DK / 8);
#pragma unroll
        for (int ts = 0; ts < KSETS; ++ts)
#pragma unroll
            for (int c = 0; c < KCHUNKS; ++c)
                kc[ts][c] = load_words<KWPL>(tile + k_lane_off + ts * 16 * (DK / 8) + c * 4 * KWPL);
    };
    auto load_v = [&](int64_t row0) {
        const uint32_t *tile = p.v_codes + row0 * p.v_row_words;
#pragma unroll
        for (int i = 0; i < VSTEPS; ++i) vc[i] = load_words<VW>(tile + v_lane_off + i * VTPS * p.v_row_words);
    };
    auto load_params = [&](int64_t row0) {
        ks_bits = load_groups<GK>(p.k_scale + row0 * GK + lane * GK);
        kb_bits = load_groups<GK>(p.k_bias + row0 * GK + lane * GK);
        vs_bits = load_groups<GV>(p.v_scale + row0 * p.v_row_groups + lane * p.v_row_groups);
        vb_bits = load_groups<GV>(p.v_bias + row0 * p.v_row_groups + lane * p.v_row_groups);
    };

    // One 64-token tile.  PREFETCH is a compile-time flag: every tile but the last of a wave issues the next
    // tile's loads unconditionally (K codes once the K side is done, the rest after the V side), so the code
    // buffers are plain loop-carried registers and loads are always in flight while the ALUs work.
    auto tile = [&](const int t0, const int64_t row0_next, auto prefetch) {
        constexpr bool PREFETCH = decltype(prefetch)::value;
        // ---- K side: q.c per (token, head, group) on the matrix core, results to LDS in token order
        {
            float4_t d[KSETS][KCHUNKS];
#pragma unroll
            for (int ts = 0; ts < KSETS; ++ts)
#pragma unroll
                for (int c = 0; c < KCHUNKS; ++c) d[ts][c] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int w = 0; w < KWPL; ++w)
#pragma unroll
                for (int ts = 0; ts < KSETS; ++ts)
#pragma unroll
                    for (int c = 0; c < KCHUNKS; ++c) {
                        const CodePairs cp = unpack_codes(kc[ts][c].w[w]);
                        const uint4 packed = make_uint4(half2_to_bits(cp.a0), half2_to_bits(cp.b0),
                                                        half2_to_bits(cp.a1), half2_to_bits(cp.b1));
                        d[ts][c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(qop[c][w], __builtin_bit_cast(half8_t, packed),
                                                                          d[ts][c], 0, 0, 0);
                    }
            // result row i = 4*(lane/16) + reg belongs to (head i % NREP, group-in-chunk i / NREP); rows past
            // KROWS are repeats.  part[token][group][head] keeps a lane's registers contiguous.
            constexpr int kRegs = KROWS < 4 ? KROWS : 4;
            if (4 * kkb < KROWS) {
#pragma unroll
                for (int ts = 0; ts < KSETS; ++ts)
#pragma unroll
                    for (int c = 0; c < KCHUNKS; ++c) {
                        float *dst = part + ((ts * 16 + kj) * GK + c * KGPC) * NREP + 4 * kkb;
#pragma unroll
                        for (int e = 0; e < kRegs; ++e) dst[e] = d[ts][c][e];
                    }
            }
        }
        if constexpr (PREFETCH) load_k(row0_next); // the next tile's K codes travel while this tile finishes
        wave_lds_sync();

        // ---- the lane that owns token `lane`: finish its scores, online softmax, publish p*s
        const bool tok_valid = (t0 + lane >= first) && (t0 + lane < t_end);
        float ks[GK], kb[GK], vs[GV], vb[GV];
#pragma unroll
        for (int g = 0; g < GK; ++g) {
            ks[g] = group_value<GK>(ks_bits, g) * kCodeScaleA;
            kb[g] = group_value<GK>(kb_bits, g);
        }
#pragma unroll
        for (int g = 0; g < GV; ++g) {
            vs[g] = group_value<GV>(vs_bits, g);
            vb[g] = group_value<GV>(vb_bits, g);
        }
        float alpha[NREP];
#pragma unroll
        for (int r = 0; r < NREP; ++r) {
            float z = 0.0f;
#pragma unroll
            for (int g = 0; g < GK; ++g) {
                z = fmaf(ks[g], part[(lane * GK + g) * NREP + r], z);
                z = fmaf(kb[g], qsum[r][g], z);
            }
            z = tok_valid ? z * p.score_scale : kNegBig;
            const float m_new = fmaxf(m_run[r], wave_max(z));
            alpha[r] = __builtin_amdgcn_exp2f(m_run[r] - m_new);
            m_run[r] = m_new;
            const float pr = tok_valid ? __builtin_amdgcn_exp2f(z - m_new) : 0.0f;
            l_run[r] = fmaf(l_run[r], alpha[r], pr);
#pragma unroll
            for (int g = 0; g < GV; ++g) {
                ps_h[(r * GV + g) * kWave + ps_slot] = float_to_half_bits(tok_valid ? pr * vs[g] : 0.0f);
                pb[r][g] = fmaf(pb[r][g], alpha[r], tok_valid ? pr * vb[g] : 0.0f);
            }
        }
        wave_lds_sync();

        // ---- V side: acc[r][e] += (p s)[t] * c[t][e], two tokens per v_dot2_f32_f16
#pragma unroll
        for (int r = 0; r < NREP; ++r)
            if (alpha[r] != 1.0f) { // wave-uniform
#pragma unroll
                for (int e = 0; e < 8 * VW; ++e) acc[r][e] *= alpha[r];
            }
#pragma unroll
        for (int i = 0; i < VSTEPS; i += 2) {
            half2_t pp[NREP];
#pragma unroll
            for (int r = 0; r < NREP; ++r) pp[r] = bits_to_half2(ps_w[(r * GV + vg) * (kWave / 2) + VTPS * (i / 2) + vo]);
#pragma unroll
            for (int w = 0; w < VW; ++w) {
#pragma unroll
                for (int by = 0; by < 4; ++by) {
                    // byte `by` of both tokens' words: codes 2*by (low nibble) and 2*by+1 (high nibble)
                    const uint32_t pair = __builtin_amdgcn_perm(vc[i + 1].w[w], vc[i].w[w], 0x0C040C00u + by * 0x00010001u);
                    const half2_t lo = bits_to_half2(pair & 0x000F000Fu);
                    const half2_t hi = bits_to_half2(pair & 0x00F000F0u);
#pragma unroll
                    for (int r = 0; r < NREP; ++r) {
                        acc[r][8 * w + 2 * by] = dot2(lo, pp[r], acc[r][8 * w + 2 * by]);
                        acc[r][8 * w + 2 * by + 1] = dot2(hi, pp[r], acc[r][8 * w + 2 * by + 1]);
                    }
                }
            }
        }
        if constexpr (PREFETCH) {
            load_params(row0_next);
            load_v(row0_next);
        }
        wave_lds_sync(); // the next tile overwrites part / ps
    };

    int64_t row0 = 0, row0_next = 0;
    int bi = next_tile(t_begin / kBlockTokens, row0);
    if (bi < b_end) {
        // same issue order as inside the loop (K codes first), pinned so that the wait for the K codes
        // never covers the loads issued after them
        load_k(row0);
        __builtin_amdgcn_sched_barrier(0);
        load_params(row0);
        load_v(row0);
        __builtin_amdgcn_sched_barrier(0);
        for (;;) {
            const int bn = next_tile(bi + 1, row0_next);
            if (bn >= b_end) break;
            tile(bi * kBlockTokens + wave * kWave, row0_next, std::true_type{});
            bi = bn;
        }
        tile(bi * kBlockTokens + wave * kWave, 0, std::false_type{});
    }

    // ---- merge token slots, lanes and waves in a fixed order, through LDS
    __syncthreads(); // every wave is done with its part / ps region
    float *fin_acc = lds;                                   // [kWaves][VTPS][NREP][DV]
    float *fin_pb = fin_acc + kWaves * VTPS * NREP * DV;    // [kWaves][NREP][GV]
    float *fin_m = fin_pb + kWaves * NREP * GV;             // [kWaves][NREP]
    float *fin_l = fin_m + kWaves * NREP;                   // [kWaves][NREP]
#pragma unroll
    for (int r = 0; r < NREP; ++r) {
        float *dst = fin_acc + ((wave * VTPS + vo) * NREP + r) * DV + vj * 8 * VW;
#pragma unroll
        for (int e = 0; e < 8 * VW; ++e) dst[e] = acc[r][e] * ((e & 1) ? kCodeScaleB : kCodeScaleA);
        const float lsum = wave_sum(l_run[r]);
#pragma unroll
        for (int g = 0; g < GV; ++g) {
            const float s = wave_sum(pb[r][g]);
            if (lane == 0) fin_pb[(wave * NREP + r) * GV + g] = s;
        }
        if (lane == 0) {
            fin_m[wave * NREP + r] = m_run[r];
            fin_l[wave * NREP + r] = lsum;
        }
    }
    __syncthreads();
    for (int idx = tid; idx < NREP * DV; idx += kThreads) {
        const int r = idx / DV, e = idx % DV;
        float m = kNegBig;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) m = fmaxf(m, fin_m[w * NREP + r]);
        float o = 0.0f, l = 0.0f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float f = __builtin_amdgcn_exp2f(fin_m[w * NREP + r] - m);
            float a = fin_pb[(w * NREP + r) * GV + e / kGroup];
#pragma unroll
            for (int sl = 0; sl < VTPS; ++sl) a += fin_acc[((w * VTPS + sl) * NREP + r) * DV + e];
            o = fmaf(f, a, o);
            l = fmaf(f, fin_l[w * NREP + r], l);
        }
        const int64_t rec = (unit0 + r) * p.num_splits + split;
        p.part_acc[rec * DV + e] = o;
        if (e == 0) {
            p.part_ml[rec * 2] = m;
            p.part_ml[rec * 2 + 1] = l;
        }
    }
}

// Merge the split partials of one (layer, agent, query head): fixed order, binary32, output binary16.
__global__ __launch_bounds__(kWave) void combine_kernel(const float *__restrict__ part_acc,
                                                        const float *__restrict__ part_ml,
                                                        const int32_t *__restrict__ seq_len, uint16_t *__restrict__ out,
                                                        int q_heads, int num_agents, int v_dim, int num_splits,
                                                        int split_tokens, int max_seq_len)
{
    const int64_t unit = blockIdx.x;
    const int agent = (int)((unit / q_heads) % num_agents);
    int n = seq_len[agent];
    n = n < max_seq_len ? n : max_seq_len;
    const int live = n > 0 ? (n + split_tokens - 1) / split_tokens : 0;
    const float *ml = part_ml + unit * num_splits * 2;
    float m = kNegBig;
    for (int s = 0; s < live; ++s)
        if (ml[2 * s + 1] > 0.0f) m = fmaxf(m, ml[2 * s]);
    float denom = 0.0f;
    for (int s = 0; s < live; ++s)
        if (ml[2 * s + 1] > 0.0f) denom = fmaf(__builtin_amdgcn_exp2f(ml[2 * s] - m), ml[2 * s + 1], denom);
    const float inv = denom > 0.0f ? 1.0f / denom : 0.0f;
    for (int e = threadIdx.x; e < v_dim; e += kWave) {
        float o = 0.0f;
        for (int s = 0; s < live; ++s)
            if (ml[2 * s + 1] > 0.0f) o = fmaf(__builtin_amdgcn_exp2f(ml[2 * s] - m), part_acc[(unit * num_splits + s) * v_dim + e], o);
        out[unit * v_dim + e] = float_to_half_bits(o * inv);
    }
}

template <int DK, int DV, int NREP>
hipError_t launch_decode_t(const AttentionArgs &a, hipStream_t stream)
{
    DecodeParams p;
    p.k_codes = a.k.codes; p.k_scale = a.k.scale; p.k_bias = a.k.bias;
    p.v_codes = a.v.codes; p.v_scale = a.v.scale; p.v_bias = a.v.bias;
    p.q = a.q; p.block_table = a.block_table; p.seq_len = a.seq_len;
    p.part_acc = a.part_acc; p.part_ml = a.part_ml;
    p.num_blocks = a.k.num_blocks; p.kv_heads = a.spec.num_kv_heads; p.q_heads = a.spec.num_q_heads;
    p.num_agents = a.num_agents; p.max_blocks = a.max_blocks; p.max_seq_len = a.max_seq_len;
    p.window = a.window; p.split_tokens = a.split_tokens; p.num_splits = a.num_splits;
    p.layer_begin = a.layer_begin;
    const int v_row_dim = a.spec.v_aliases_k ? a.spec.k_dim : a.spec.v_dim;
    p.v_row_words = v_row_dim / 8; p.v_row_groups = v_row_dim / kGroup;
    p.score_scale = a.sm_scale * kLog2e;
    dim3 grid(a.num_splits, a.num_agents * a.spec.num_kv_heads, a.layers_in_call);
#ifndef Q4KV_DEC_KW
#define Q4KV_DEC_KW 4
#endif
#ifndef Q4KV_DEC_VW
#define Q4KV_DEC_VW (NREP >= 4 ? 1 : 2) // keeps the NREP * 8 * VW accumulators and both code buffers in registers
#endif
    constexpr int KW = Q4KV_DEC_KW;
    constexpr int VW = (DV / 16 < (Q4KV_DEC_VW)) ? DV / 16 : (Q4KV_DEC_VW);
    hipLaunchKernelGGL((decode_attention_kernel<DK, DV, NREP, KW, VW>), grid, dim3(kThreads), 0, stream, p);
    return hipGetLastError();
}

template <int DK, int DV>
hipError_t launch_decode_d(const AttentionArgs &a, int n_rep, hipStream_t stream)
{
    switch (n_rep) {
    case 1: return launch_decode_t<DK, DV, 1>(a, stream);
    case 2: return launch_decode_t<DK, DV, 2>(a, stream);
    case 4: return launch_decode_t<DK, DV, 4>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

} // namespace

bool decode_supported(const q4kv_spec &s)
{
    const int n_rep = s.num_q_heads / s.num_kv_heads;
    const bool rep_ok = n_rep == 1 || n_rep == 2 || n_rep == 4;
    const bool dims_ok = (s.k_dim == 64 || s.k_dim == 128 || s.k_dim == 256) && s.v_dim == s.k_dim && !s.v_aliases_k;
    return rep_ok && dims_ok;
}

hipError_t launch_decode_attention(const AttentionArgs &a, hipStream_t stream)
{
    const int n_rep = a.spec.num_q_heads / a.spec.num_kv_heads;
    switch (a.spec.k_dim) {
    case 64: return launch_decode_d<64, 64>(a, n_rep, stream);
    case 128: return launch_decode_d<128, 128>(a, n_rep, stream);
    case 256: return launch_decode_d<256, 256>(a, n_rep, stream);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_combine(const AttentionArgs &a, hipStream_t stream)
{
    const int64_t units = (int64_t)a.layers_in_call * a.num_agents * a.q_len * a.spec.num_q_heads;
    if (units == 0) return hipSuccess;
    hipLaunchKernelGGL(combine_kernel, dim3((unsigned)units), dim3(kWave), 0, stream, a.part_acc, a.part_ml, a.seq_len,
                       a.out, a.spec.num_q_heads, a.num_agents, a.spec.v_dim, a.num_splits, a.split_tokens,
                       a.max_seq_len);
    return hipGetLastError();
}

} // namespace q4kv

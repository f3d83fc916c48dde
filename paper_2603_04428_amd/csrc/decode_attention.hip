// Batched decode attention (one query token per agent) over paged Q4 KV caches, GQA form:
//   out[l][a][h] = softmax(sm * q K_hat^T) V_hat   over the agent's cached tokens,
// K_hat / V_hat = code*scale + bias, never materialised (Sec. 3.2 item 3, Sec. 3.4, Sec. 3.6).
//
// The step is a single pass over the cache and is HBM-bound: per cached token and KV head it reads
// DK/2 + DV/2 bytes of codes and 4 bytes of scale/bias per 64-wide group, once, for all n_rep
// query heads of the group.  The design follows from keeping everything else under that stream:
//
//  * Work decomposition ("stream-K" over tokens).  All (layer, KV head, agent) units are cut into
//    64-token tiles and numbered consecutively; the launch is a fixed set of workgroups (two per compute
//    unit) and workgroup w owns the contiguous tile range [w*per, (w+1)*per), whose tiles its four waves
//    take in turn (wave i: the range's tiles i, i+4, ...: inside a unit the four waves read one 256-token
//    block together).  Ragged context lengths therefore balance to within a few tiles.  A small plan
//    kernel turns seq_len[] into the tile prefix sums first.
//  * Waves walk their tiles with private online-softmax state and private LDS, and the next tile's loads
//    (also across a unit boundary) are issued while the current tile is processed, so loads are always
//    in flight.  They meet only where a unit (or the workgroup's part of it) ends: each folds its state
//    into one (sums, running maximum, denominator) per query head in LDS, and the four are merged there.
//    A unit that lies inside one workgroup's range is normalised and written out at that point; a unit
//    shared by several workgroups gets one un-normalised record per workgroup in the workspace, and the
//    workgroup that arrives last (a counter per unit) merges the records, in record order whoever it is,
//    so results are run-to-run identical.  A short call (one layer) thus keeps every wave busy with two
//    or three tiles while a unit still has only a dozen records to merge.
//  * A long call (a workgroup's range spans several units) gains nothing from that and would pay for the
//    meetings: there every wave takes a contiguous quarter of the workgroup's range for itself, as if it
//    were a workgroup of one -- the same segments, records and arrival counters, no barrier.
//  * Codes never become integers or binary32: a nibble masked in place is a binary16 subnormal
//    (c*2^-24 or c*2^-20) and goes straight into a matrix-core operand.
//  * The affine part of the dequantization is factored out of the inner loops:
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
//  * V side: the contraction runs over tokens while a word holds 8 dims of one token, so the big matrix
//    tiles do not fit (their K-index would have to be 8 tokens of one dim).  It runs on the 16-block
//    4x4x4 form instead (v_mfma_f32_4x4x4_16B_f16): each block of 4 lanes multiplies the 4x4 matrix
//    (operand row) x (4 tokens) of binary16 p*s -- one quantization group per block, so the per-group
//    scale can live in it -- with (4 tokens) x (4 dims) of codes.  The lane owning a word pairs the
//    codes of two tokens with v_perm and masks nibbles in place, two tokens per register.
//    p*s travels as two binary16 terms, hi = fl16(p*s) and lo = fl16(p*s - hi), in two operand rows per
//    query head: one term alone errs by 2^-12 of p*s*c, which is relative to a group's range (c*s up to
//    15 s) and not to the value, and would leave the output tolerance on caches with wide value groups.
//    With one or two query heads per KV head the second term sits in operand rows that were repeats (no
//    further matrix instruction); with four or eight it is a second instruction into the same accumulator.
#include "q4_device.h"
#include "q4kv_internal.h"
#include "stream_k.h"

namespace q4kv {
namespace {

constexpr int kWavesPerSimd = 2; // resident waves per SIMD the register budget is sized for
constexpr int kPrioShift = 12;   // log2 of the priority time slice in 10 ns ticks (41 us)
constexpr int kPrioLevel = 2;
constexpr int kPrioMinTiles = 128; // tiles per workgroup from which the priority turns are taken
constexpr float kOneTermScale = 0.49f; // largest value scale for which one binary16 term of p*s keeps the tolerance
constexpr int kCoopMaxTiles = 64;  // tiles per workgroup below which its four waves share every unit (else: a quarter each)
constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr float kNegBig = -1.0e30f; // "minus infinity" that survives subtraction
constexpr float kLog2e = 1.4426950408889634f;

struct DecodeParams {
    const uint32_t *k_codes, *v_codes;
    const uint16_t *k_scale, *k_bias, *v_scale, *v_bias;
    const uint16_t *q;
    StreamParams stream;
    MergeParams merge;
    int q_heads;
    float score_scale;             // sm_scale * log2(e): scores are kept in log2 units
};

// ---------------------------------------------------------------------------------------------- plan

// Sliding windows of the layers of a call, passed to plan_kernel by value: one window for all layers, or one each.
struct LayerWindows {
    int uniform;                 // 1: `window` holds for every layer
    int window;
    int w[kMaxWindowLayers];
};

// total_waves = workers of the attention launch (workgroups, or waves for the shared-latent kernel).  Workgroup 0 writes the plan described in stream_k.h; all workgroups
// of the launch share the clearing of the arrival counters (one per (layer, KV head, agent) unit).
__global__ __launch_bounds__(kThreads) void plan_kernel(const int32_t *__restrict__ seq_len, int num_agents,
                                                        int max_seq_len, const LayerWindows lw, int layers,
                                                        int kv_heads, int total_waves, int min_tiles_per_wave,
                                                        int per_multiple, int signature, int32_t *__restrict__ plan,
                                                        int32_t *__restrict__ arrivals)
{
    {
        const int counters = layers * kv_heads * num_agents; // the host keeps this below 2^31
        for (int i = blockIdx.x * kThreads + threadIdx.x; i < counters; i += gridDim.x * kThreads) arrivals[i] = 0;
        if (blockIdx.x != 0) return;
    }
    __shared__ int s_wave_sum[kWaves];
    __shared__ int s_cls[kMaxWindowLayers], s_win[kMaxWindowLayers], s_tt[kMaxWindowLayers], s_classes;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    PlanView pv;
    pv.plan = plan;
    pv.A = num_agents;
    pv.L = layers;
    // ---- classes of equal windows (a handful at most in practice), numbered in the order of their first layer.
    // Thread li finds the first layer with its window; the class of a layer is the number of such first layers
    // before its own.
    __shared__ int s_first[kMaxWindowLayers];
    static_assert(kThreads >= kMaxWindowLayers, "one thread per layer");
    if (lw.uniform) {
        if (tid == 0) {
            s_win[0] = lw.window > 0 ? lw.window : 0;
            s_classes = 1;
        }
    } else {
        const int li = tid < layers ? tid : 0; // kThreads >= kMaxWindowLayers
        const int w_li = lw.w[li] > 0 ? lw.w[li] : 0;
        int first = li;
        for (int j = layers - 1; j >= 0; --j) {
            const int w_j = lw.w[j] > 0 ? lw.w[j] : 0; // wave-uniform
            if (j < li && w_j == w_li) first = j;
        }
        if (tid < layers) s_first[tid] = first;
        __syncthreads();
        if (tid < layers) {
            int c = 0;
            for (int k = 0; k < first; ++k) c += s_first[k] == k ? 1 : 0;
            s_cls[tid] = c;
            if (first == tid) s_win[c] = w_li;
            if (tid == layers - 1) { // classes in all = first layers up to the last layer
                int total = c;
                for (int k = first; k < layers; ++k) total += s_first[k] == k ? 1 : 0;
                s_classes = total;
            }
        }
    }
    __syncthreads();
    const int C = s_classes;
    for (int li = tid; li < layers; li += kThreads) plan[pv.cls_off() + li] = lw.uniform ? 0 : s_cls[li];
    const int per_thread = (num_agents + kThreads - 1) / kThreads;
    const int a0 = tid * per_thread, a1 = min(num_agents, a0 + per_thread);
    int32_t *nlen = plan + pv.nlen_off();
    // Nothing written to the plan is read back here: every value comes from seq_len (cached after its first read)
    // and registers, so the kernel's length is a few memory round trips.
    auto length = [&](int a) {
        const int n = seq_len[a];
        return n < 0 ? 0 : (n > max_seq_len ? max_seq_len : n);
    };
    auto first_tile_token = [](int n, int window) {
        const int first = (window > 0 && n > window) ? n - window : 0;
        return first & ~(kWave - 1);
    };
    int empties = 0;
    for (int a = a0; a < a1; ++a) {
        const int n = length(a);
        nlen[a] = n;
        empties += n == 0 ? 1 : 0;
    }
    { // ---- agents without a visible token, in index order
        int incl = empties;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            const int up = __shfl_up(incl, off, kWave);
            if (lane >= off) incl += up;
        }
        if (lane == kWave - 1) s_wave_sum[wave] = incl;
        __syncthreads();
        int before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const int t = s_wave_sum[w];
            if (w < wave) before += t;
            total += t;
        }
        __syncthreads(); // s_wave_sum is free again
        if (tid == 0) {
            plan[4] = total;
            plan[5] = signature;
        }
        int at = before + incl - empties;
        int32_t *empty = plan + pv.empty_off();
        for (int a = a0; a < a1; ++a)
            if (length(a) == 0) empty[at++] = a;
    }
    // ---- per class: first visible tile and tile count of every agent, prefix sum over the agents
    for (int c = 0; c < C; ++c) {
        const int cb = pv.class_off(c);
        const int window = s_win[c];
        int32_t *tpre = plan + cb + 1, *tstart = plan + cb + 2 + num_agents;
        int local = 0;
        for (int a = a0; a < a1; ++a) {
            const int n = length(a);
            const int start = first_tile_token(n, window);
            tstart[a] = start;
            local += n > 0 ? (n - start + kWave - 1) / kWave : 0;
        }
        int incl = local; // inclusive scan inside the wave, then over the waves through LDS
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            const int up = __shfl_up(incl, off, kWave);
            if (lane >= off) incl += up;
        }
        if (lane == kWave - 1) s_wave_sum[wave] = incl;
        __syncthreads();
        int before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const int t = s_wave_sum[w];
            if (w < wave) before += t;
            total += t;
        }
        __syncthreads(); // s_wave_sum is free again
        if (tid == 0) {
            plan[cb] = window;
            tpre[num_agents] = total;
            s_tt[c] = total;
        }
        int run = before + incl - local; // exclusive prefix of this thread's chunk
        for (int a = a0; a < a1; ++a) {
            tpre[a] = run;
            const int n = length(a);
            run += n > 0 ? (n - first_tile_token(n, window) + kWave - 1) / kWave : 0;
        }
    }
    __syncthreads();
    // ---- tiles before every layer (prefix sum over the layers, one thread each; the host keeps the total below
    // 2^31), the waves' share
    if (layers <= kThreads) {
        const int mine = tid < layers ? s_tt[lw.uniform ? 0 : s_cls[tid]] * kv_heads : 0;
        int incl = mine;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            const int up = __shfl_up(incl, off, kWave);
            if (lane >= off) incl += up;
        }
        if (lane == kWave - 1) s_wave_sum[wave] = incl;
        __syncthreads();
        int before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const int t = s_wave_sum[w];
            if (w < wave) before += t;
            total += t;
        }
        if (tid < layers) plan[pv.lt_off() + tid] = before + incl - mine;
        if (tid == 0) {
            plan[pv.lt_off() + layers] = total;
            int per = (int)(((long long)total + total_waves - 1) / total_waves);
            if (per < min_tiles_per_wave) per = min_tiles_per_wave;
            per = (per + per_multiple - 1) / per_multiple * per_multiple;
            plan[0] = total;
            plan[1] = per;
            plan[2] = C;
            plan[3] = layers;
        }
    } else if (tid == 0) { // more layers than threads: one window for all of them (see kMaxWindowLayers)
        int total = 0;
        for (int li = 0; li < layers; ++li) {
            plan[pv.lt_off() + li] = total;
            total += s_tt[0] * kv_heads;
        }
        plan[pv.lt_off() + layers] = total;
        int per = (int)(((long long)total + total_waves - 1) / total_waves);
        if (per < min_tiles_per_wave) per = min_tiles_per_wave;
        per = (per + per_multiple - 1) / per_multiple * per_multiple;
        plan[0] = total;
        plan[1] = per;
        plan[2] = C;
        plan[3] = layers;
    }
}

// ---------------------------------------------------------------------------------------------- loads
//
// Loads of cache data can be marked non-temporal (NT: the data is read once).  With the hint the memory system
// delivers 12 % more to a kernel that only reads (6.1 -> 6.8 TB/s).  What it does for this kernel depends on the row
// shapes, measured per head width (GB/s: plain / codes NT / parameters NT / both NT):
//   256, n_rep 2 (ragged 1K-8K x 10)   5618 / 6157 / 5835 / 6194      128, n_rep 4 (4K x 5)   4390 / 4847 / 4501 / 4834
//   192 + 128, n_rep 1 (8K x 5)        5698 / 5357 / 5801 / 5455      128, n_rep 1 (6K x 6)   5005 / 5693 / 5144 / 5529
// (64-wide heads and n_rep 8 are not memory-bound and do not care.)  The policy below takes the best column.
template <int DK>
struct LoadHints {
    static constexpr bool codes = DK != 192; // 8-byte code loads of the 192-wide rows lose with the hint
    static constexpr bool params = DK >= 192;
};

template <bool NT, typename T>
__device__ __forceinline__ T hinted_load(const T *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

// One token's scales or biases (N binary16 values) as raw bits: loaded with one 2-, 4- or 8-byte load per 4
// values where the row width allows it and converted only where they are used, so that issuing the load never
// makes the wave wait for it.
template <int N>
struct GroupBits {
    uint32_t w[(N + 1) / 2];
};

template <int N, bool NT>
__device__ __forceinline__ GroupBits<N> load_groups(const uint16_t *p)
{
    GroupBits<N> r;
    typedef uint32_t u2_t __attribute__((ext_vector_type(2)));
    if constexpr (N == 1) {
        r.w[0] = hinted_load<NT>(p);
    } else if constexpr (N == 2) {
        r.w[0] = hinted_load<NT>(reinterpret_cast<const uint32_t *>(p));
    } else if constexpr (N % 4 == 0) {
#pragma unroll
        for (int i = 0; i < N / 4; ++i) {
            const u2_t t = hinted_load<NT>(reinterpret_cast<const u2_t *>(p) + i);
            r.w[2 * i] = t.x;
            r.w[2 * i + 1] = t.y;
        }
    } else { // rows of 2 N bytes are only 2-byte aligned: one load per value
#pragma unroll
        for (int i = 0; i < (N + 1) / 2; ++i) r.w[i] = 0;
#pragma unroll
        for (int i = 0; i < N; ++i) r.w[i / 2] |= (uint32_t)hinted_load<NT>(p + i) << (16 * (i & 1));
    }
    return r;
}

template <int N, bool BF>
__device__ __forceinline__ float group_value(const GroupBits<N> &b, int g)
{
    return param_bits_to_float<BF>((uint16_t)((g & 1) ? (b.w[g / 2] >> 16) : (b.w[g / 2] & 0xffffu)));
}

template <int W>
struct Words {
    uint32_t w[W];
};

template <int W, bool NT>
__device__ __forceinline__ Words<W> load_words(const uint32_t *p)
{
    Words<W> r;
    typedef uint32_t u4_t __attribute__((ext_vector_type(4)));
    typedef uint32_t u2_t __attribute__((ext_vector_type(2)));
    if constexpr (W == 4) {
        const u4_t t = hinted_load<NT>(reinterpret_cast<const u4_t *>(p));
        r.w[0] = t.x; r.w[1] = t.y; r.w[2] = t.z; r.w[3] = t.w;
    } else if constexpr (W == 2) {
        const u2_t t = hinted_load<NT>(reinterpret_cast<const u2_t *>(p));
        r.w[0] = t.x; r.w[1] = t.y;
    } else {
        r.w[0] = hinted_load<NT>(p);
    }
    return r;
}

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// ---------------------------------------------------------------------------------------------- attention

// DK, DV: head widths (multiples of 64); NREP query heads per KV head; BF: scale and bias are stored as bfloat16
// instead of binary16 (they are only ever used as binary32 here, so the two differ in one conversion).
//
// Loads are never predicated: a tile's 64 rows always exist inside its block, so rows past the agent's
// length are read and then ignored (their score is forced to "minus infinity", their p*s to zero; codes
// are nibbles and cannot produce a NaN, scale/bias of such rows are replaced by zero after the load).
template <int DK, int DV, int NREP, bool BF>
__global__ __launch_bounds__(kThreads, kWavesPerSimd) void decode_attention_kernel(DecodeParams p)
{
    constexpr int GK = DK / kGroup, GV = DV / kGroup;
    // K side (matrix core): lane = (token j = lane % 16 of a 16-token set, k-block kb = lane / 16)
    constexpr int KWPL = DK % 128 == 0 ? 4 : 2;    // words a lane loads per chunk (16 or 8 bytes)
    constexpr int KCHUNKS = DK / (32 * KWPL);      // chunks per row: 4 lanes * KWPL words each
    constexpr int KGPC = KWPL == 4 ? 2 : 1;        // quantization groups per chunk
    constexpr int KSETS = kWave / 16;              // 16-token sets per tile
    constexpr int KROWS = NREP * KGPC;             // distinct rows of the query operand
    static_assert(KROWS <= 16 && KCHUNKS * KGPC == GK, "K layout");
    // V side (16 blocks of 4x4x4): a lane takes one word (8 dims) per token, VLPT lanes share a token, VTPS
    // token slots per load step; the 4 lanes of a block lie in one token slot and one quantization group
    constexpr int VLPT = DV / 8;
    constexpr int VTPS = kWave / VLPT;
    constexpr int VSTEPS = kWave / VTPS;
    constexpr int VROWS = 2 * NREP;                // rows of p*s: row t*NREP + r = term t (0: hi, 1: lo) of head r
    constexpr bool kTermRows = NREP <= 2;          // both terms fit the 4 operand rows of one instruction
    constexpr int VHQ = NREP > 4 ? NREP / 4 : 1;   // passes over the query heads, 4 rows each
    static_assert(VLPT % 8 == 0 && VLPT <= kWave && VSTEPS % 4 == 0, "V layout");
    // per wave: q.c per token, group and head [64][GK][NREP] (binary32) and p*scale [VROWS][GV][64] (binary16,
    // the tokens of four consecutive V load steps of a slot side by side, 8 bytes); the same
    // region serves the end-of-unit reduction [VTPS][NREP][DV] + bias sums [NREP][GV]; behind it the group sums of
    // q [NREP][GK]
    constexpr int kPartFloats = kWave * GK * NREP;
    constexpr int kPsFloats = VROWS * GV * kWave / 2;
    constexpr int kFinalFloats = VTPS * NREP * DV + NREP * GV;
    constexpr int kWaveFloats = (kPartFloats + kPsFloats > kFinalFloats ? kPartFloats + kPsFloats : kFinalFloats) + NREP * GK;
    __shared__ float lds[kWaves * kWaveFloats];
    // what a wave leaves behind when it is done with a segment: sums [NREP][DV], then (maximum, denominator)
    // [NREP][2]; kSegBufs segments can be pending before a wave has to wait for the others
    constexpr int kSegFloats = NREP * DV + 2 * NREP;
    constexpr int kSegBufs = (NREP >= 8 || NREP * DV >= 2048) ? 1 : 2; // LDS: two workgroups per compute unit
    __shared__ float seg_lds[kSegBufs * kWaves * kSegFloats];
    __shared__ int s_last;

    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = uniform(tid / kWave);
    const int gw = blockIdx.x * kWaves + wave; // this wave's index in the launch

    const TileStream ts_(p.stream);
    if (!ts_.valid) return;
    zero_empty_units<DV>(ts_.pv, p.merge.out, p.q_heads, gw, gridDim.x * kWaves, lane);
    const int per = ts_.per, N = ts_.N; // per: tiles of a workgroup
    const int wg = blockIdx.x;
    const long long x_begin = (long long)wg * per;
    if (x_begin >= N) return;           // the whole workgroup leaves
    const int x0 = (int)x_begin;
    const int x1 = (int)min((long long)N, x_begin + per);
    // how the workgroup's range is shared out: tiles in turn (short ranges), or a contiguous quarter per wave
    const bool coop = per < kCoopMaxTiles;
    const int stride = coop ? kWaves : 1;
    const int wx0 = coop ? x0 + wave : x0 + wave * (per / kWaves); // per is a multiple of 4
    const int wx1 = coop ? x1 : min(x1, wx0 + per / kWaves);
    if (!coop && wx0 >= wx1) return; // nothing to do and nobody to meet

    float *region = lds + wave * kWaveFloats;
    float *part = region;                                                  // [64][GK][NREP]
    uint16_t *ps_h = reinterpret_cast<uint16_t *>(region + kPartFloats);   // [VROWS][GV][64] binary16
    const uint2 *ps_q = reinterpret_cast<const uint2 *>(ps_h);            // the same as token quads
    float *qsum_lds = region + (kWaveFloats - NREP * GK);                  // [NREP][GK]

    // This wave's tiles are wx0, wx0 + stride, ... below wx1; a wave of a sharing workgroup whose range holds none
    // keeps a valid cursor that it never uses.  A range (the workgroup's when its waves share, else the wave's own) is
    // a sequence of segments (the parts of units inside it), numbered from 0: `seg` is the oldest one the four waves
    // have not finished together yet (number k_old), `mseg` the one this wave's current tile lies in (number k_my).
    const int r0 = coop ? x0 : wx0, r1 = coop ? x1 : wx1;
    Cursor cur = ts_.locate(r0);
    Segment seg, mseg;
    seg.start(cur, r0, r1);
    mseg = seg;
    int k_old = 0, k_my = 0;
    uint32_t pub_mask = 0; // bit i: this wave has left its result of segment k_old + i in seg_lds
    int x = wx0;
    bool active = x < wx1;
    if (coop && active && wave > 0) ts_.advance(cur, wave);

    const int kj = lane % 16, kkb = lane / 16;
    const int vj = lane % VLPT, vo = lane / VLPT, vg = vj / 8;
    // where the token owned by this lane (local index `lane` = step*VTPS + slot) goes in ps_h
    const int ps_slot = 4 * VTPS * ((lane / VTPS) / 4) + 4 * (lane % VTPS) + ((lane / VTPS) & 3);
    // row of p*s (within a pass and term) that this lane supplies to the matrix instruction
    const int v_row = kTermRows ? (lane & 3) % VROWS : (lane & 3);

    Words<KWPL> kc[KSETS][KCHUNKS];
    uint32_t vc[VSTEPS];
    GroupBits<GK> ks_bits, kb_bits;
    GroupBits<GV> vs_bits, vb_bits;
    // tile base (uniform, from the row) + a fixed per-lane offset + a compile-time step offset
    const int k_lane_off = kj * (DK / 8) + kkb * KWPL;
    const int v_lane_off = vo * (DV / 8) + vj;
    // Loads are issued in the order they are consumed (K sets, scale/bias, V steps) and every buffer register is
    // reloaded for the next tile as soon as its last reader has been issued, so that each spends almost all of
    // its time in flight.
    auto load_k_pair = [&](int tp, int64_t row0) { // two 16-token sets
        const uint32_t *tile = p.k_codes + row0 * (DK / 8);
#pragma unroll
        for (int ts = tp; ts < tp + 2; ++ts)
#pragma unroll
            for (int c = 0; c < KCHUNKS; ++c)
                kc[ts][c] = load_words<KWPL, LoadHints<DK>::codes>(tile + k_lane_off + ts * 16 * (DK / 8) + c * 4 * KWPL);
    };
    auto load_v_quad = [&](int i, int64_t row0) { // four load steps
        const uint32_t *tile = p.v_codes + row0 * (DV / 8);
#pragma unroll
        for (int k = i; k < i + 4; ++k) vc[k] = hinted_load<LoadHints<DK>::codes>(tile + v_lane_off + k * VTPS * (DV / 8));
    };
    auto load_params = [&](int64_t row0) {
        ks_bits = load_groups<GK, LoadHints<DK>::params>(p.k_scale + row0 * GK + lane * GK);
        kb_bits = load_groups<GK, LoadHints<DK>::params>(p.k_bias + row0 * GK + lane * GK);
        vs_bits = load_groups<GV, LoadHints<DK>::params>(p.v_scale + row0 * GV + lane * GV);
        vb_bits = load_groups<GV, LoadHints<DK>::params>(p.v_bias + row0 * GV + lane * GV);
    };

    half8_t qop[KCHUNKS][KWPL];
    float qsum[NREP][GK];
    float4_t acc[VHQ][8]; // [pass][dim of this lane's word][operand row in pass]; odd dims carry an extra factor 16
                          // until the end (their codes sit 4 bits higher)
    float m_run[NREP], l_run[NREP], pb[NREP][GV]; // l_run, pb: this lane's tokens only

    if (active) {
        const int64_t row0 = cur.row;
        // same issue order as inside the loop (K codes first), pinned so that the wait for the K codes never
        // covers the loads issued after them
#pragma unroll
        for (int tp = 0; tp < KSETS; tp += 2) {
            load_k_pair(tp, row0);
            __builtin_amdgcn_sched_barrier(0);
        }
        load_params(row0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < VSTEPS; i += 4) {
            load_v_quad(i, row0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // Two workgroups share a compute unit, and at equal priority the older wave wins every arbitration, also the
    // one for the memory pipeline: the workgroups launched first would finish their equal shares about 13 % ahead
    // of the others and leave half of the waves to stream alone at the end.  The two halves of the launch
    // therefore take turns at a raised priority, in time slices read from the chip-wide clock.  (Which half is the
    // older one on a compute unit is a guess from the launch order; if it is wrong nothing but this balance is lost.)
    const bool second_half = blockIdx.x >= gridDim.x / 2;

    // ---- Leaving a segment and finishing it are two steps, so that no wave waits while it still has tiles.
    // publish: a wave that is done with its tiles of segment k folds token slots and lanes through its LDS region
    // (fixed order) into one (sums, maximum, denominator) per query head and leaves that in buffer k % kSegBufs.
    // close: the four waves finish the oldest segment together -- a wave that had no tile in it marks its entry
    // empty -- and all 256 threads merge the four entries in wave order, one (head, element) at a time: into the
    // output row when no other workgroup shares the unit, else into this workgroup's record of the unit, after
    // which the workgroup that arrives last merges the records.  A wave closes segments only when it needs a buffer
    // for a later one or has run out of tiles.  Barriers here wait for LDS traffic only (loads stay in flight).
    auto lds_barrier = [&]() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };
    auto publish = [&]() {
        float *fin_acc = region;                      // [VTPS][NREP][DV]
        float *fin_pb = region + VTPS * NREP * DV;    // [NREP][GV]
        float *mine = seg_lds + ((k_my % kSegBufs) * kWaves + wave) * kSegFloats;
        float lsum[NREP];
#pragma unroll
        for (int r = 0; r < NREP; ++r) {
            float *dst = fin_acc + (vo * NREP + r) * DV + vj * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e)
                dst[e] = (kTermRows ? acc[0][e][r] + acc[0][e][NREP + r] : acc[r / 4][e][r % 4]) *
                         ((e & 1) ? kCodeScaleB : kCodeScaleA);
            lsum[r] = wave_sum(l_run[r]);
#pragma unroll
            for (int g = 0; g < GV; ++g) {
                const float s = wave_sum(pb[r][g]);
                if (lane == 0) fin_pb[r * GV + g] = s;
            }
        }
        wave_lds_sync();
#pragma unroll
        for (int r = 0; r < NREP; ++r) {
#pragma unroll
            for (int e0 = 0; e0 < DV; e0 += kWave) {
                const int e = e0 + lane;
                float o = fin_pb[r * GV + e / kGroup];
#pragma unroll
                for (int sl = 0; sl < VTPS; ++sl) o += fin_acc[(sl * NREP + r) * DV + e];
                mine[r * DV + e] = o;
            }
            if (lane == 0) {
                mine[NREP * DV + 2 * r] = m_run[r];
                mine[NREP * DV + 2 * r + 1] = lsum[r];
            }
        }
        wave_lds_sync(); // the region is free for the next tile
        pub_mask |= 1u << (k_my - k_old);
    };
    auto close_oldest = [&]() {
        const float *buf = seg_lds + (k_old % kSegBufs) * kWaves * kSegFloats;
        if (!(pub_mask & 1u) && lane < NREP) {
            float *mine = seg_lds + ((k_old % kSegBufs) * kWaves + wave) * kSegFloats;
            mine[NREP * DV + 2 * lane] = kNegBig;
            mine[NREP * DV + 2 * lane + 1] = 0.0f;
        }
        pub_mask >>= 1;
        lds_barrier();
        int slot, slots;
        seg.slot_of(per, wg, slot, slots);
        const bool alone = slots == 1;
        const int64_t u0 = ((int64_t)seg.li * p.stream.num_agents + seg.agent) * p.q_heads + (int64_t)seg.kvh * NREP;
        // thread tid takes (head, element) pairs tid, tid + 256, ...: the head is the same for a whole wave
        for (int i = tid; i < NREP * DV; i += kThreads) {
            const int r = i / DV, e = i % DV;
            float mw[kWaves], lw[kWaves], m_ref = kNegBig;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                mw[w] = buf[w * kSegFloats + NREP * DV + 2 * r];
                lw[w] = buf[w * kSegFloats + NREP * DV + 2 * r + 1];
                if (lw[w] > 0.0f) m_ref = fmaxf(m_ref, mw[w]);
            }
            float o = 0.0f, l = 0.0f;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                if (lw[w] > 0.0f) { // a wave without tiles here left nothing to read
                    const float wgt = __builtin_amdgcn_exp2f(mw[w] - m_ref);
                    o = fmaf(wgt, buf[w * kSegFloats + r * DV + e], o);
                    l = fmaf(wgt, lw[w], l);
                }
            }
            if (alone) {
                p.merge.out[(u0 + r) * DV + e] = float_to_half_bits(l > 0.0f ? o / l : 0.0f);
            } else {
                const int64_t rec = (u0 + r) * p.merge.max_slots + slot;
                record_store(p.merge.part_acc + rec * DV + e, o);
                if (e == 0) {
                    record_store(p.merge.part_ml + rec * 2, m_ref);
                    record_store(p.merge.part_ml + rec * 2 + 1, l);
                }
            }
        }
        if (!alone) {
            // every wave's record stores have reached memory before thread 0 counts the workgroup in
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_s_waitcnt(0x0F70); // vmcnt(0)
            lds_barrier();
            if (tid == 0) {
                int32_t *counter = p.merge.arrivals +
                                   ((int64_t)seg.li * p.stream.kv_heads + seg.kvh) * p.stream.num_agents + seg.agent;
                s_last = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == slots - 1;
            }
            lds_barrier();
            const bool last = s_last != 0;
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            if (last) {
                for (int i = tid; i < NREP * DV; i += kThreads) {
                    const int r = i / DV, e = i % DV;
                    const int64_t rec0 = (u0 + r) * p.merge.max_slots;
                    const float o = merge_element<DV>(p.merge.part_acc + rec0 * DV, p.merge.part_ml + rec0 * 2, slots, e, lane);
                    p.merge.out[(u0 + r) * DV + e] = float_to_half_bits(o);
                }
                // the counter is back at zero for the next call that reuses this plan
                if (tid == 0) {
                    int32_t *counter = p.merge.arrivals +
                                       ((int64_t)seg.li * p.stream.kv_heads + seg.kvh) * p.stream.num_agents + seg.agent;
                    __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        } else {
            lds_barrier(); // the buffer is free again
        }
        if (seg.end < x1) seg.next(ts_, x1); else seg.begin = x1;
        ++k_old;
    };

    // ---- a wave on its own: what publish and close do together, for mseg, without the other waves
    auto finish_alone = [&]() {
        float *fin_acc = region;                      // [VTPS][NREP][DV]
        float *fin_pb = region + VTPS * NREP * DV;    // [NREP][GV]
        float lsum[NREP];
#pragma unroll
        for (int r = 0; r < NREP; ++r) {
            float *dst = fin_acc + (vo * NREP + r) * DV + vj * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e)
                dst[e] = (kTermRows ? acc[0][e][r] + acc[0][e][NREP + r] : acc[r / 4][e][r % 4]) *
                         ((e & 1) ? kCodeScaleB : kCodeScaleA);
            lsum[r] = wave_sum(l_run[r]);
#pragma unroll
            for (int g = 0; g < GV; ++g) {
                const float s = wave_sum(pb[r][g]);
                if (lane == 0) fin_pb[r * GV + g] = s;
            }
        }
        wave_lds_sync();
        int slot, slots;
        mseg.slot_of_quarter(per, wg * kWaves + wave, slot, slots);
        const bool alone = slots == 1;
        const int64_t u0 = ((int64_t)mseg.li * p.stream.num_agents + mseg.agent) * p.q_heads + (int64_t)mseg.kvh * NREP;
#pragma unroll
        for (int r = 0; r < NREP; ++r) {
            const int64_t rec = (u0 + r) * p.merge.max_slots + slot;
            const float inv = lsum[r] > 0.0f ? 1.0f / lsum[r] : 0.0f;
#pragma unroll
            for (int e0 = 0; e0 < DV; e0 += kWave) {
                const int e = e0 + lane;
                float o = fin_pb[r * GV + e / kGroup];
#pragma unroll
                for (int sl = 0; sl < VTPS; ++sl) o += fin_acc[(sl * NREP + r) * DV + e];
                if (alone) p.merge.out[(u0 + r) * DV + e] = float_to_half_bits(o * inv);
                else record_store(p.merge.part_acc + rec * DV + e, o);
            }
            if (!alone && lane == 0) {
                record_store(p.merge.part_ml + rec * 2, m_run[r]);
                record_store(p.merge.part_ml + rec * 2 + 1, lsum[r]);
            }
        }
        wave_lds_sync(); // the region is free for the next tile
        if (!alone) {
            int32_t *counter = p.merge.arrivals +
                               ((int64_t)mseg.li * p.stream.kv_heads + mseg.kvh) * p.stream.num_agents + mseg.agent;
            if (arrive_last(counter, slots, lane)) {
                for (int r = 0; r < NREP; ++r) {
                    const int64_t rec0 = (u0 + r) * p.merge.max_slots;
                    merge_row<DV>(p.merge.part_acc + rec0 * DV, p.merge.part_ml + rec0 * 2, slots,
                                  p.merge.out + (u0 + r) * DV, lane);
                }
                if (lane == 0) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    };

    bool have = false; // this wave holds online-softmax state of mseg's unit
    int64_t unit0 = 0;
    for (;;) {
        if (__builtin_expect(!active || x >= mseg.end, 0)) {
            // this wave is done with mseg: it leaves its result behind (closing the oldest segments first when
            // no buffer is free) and goes on, or, without a tile left, helps to close everything that remains
            if (have) {
                if (coop) {
                    while (k_my - k_old >= kSegBufs) close_oldest();
                    publish();
                } else {
                    finish_alone();
                }
                have = false;
            }
            if (!active) {
                if (coop)
                    while (seg.begin < x1) close_oldest();
                break;
            }
            while (x >= mseg.end) {
                mseg.next(ts_, r1);
                ++k_my;
            }
        }
        if (per >= kPrioMinTiles) { // a short call would spend its whole life in one slice
            const bool turn = ((wall_clock64() >> kPrioShift) & 1) != 0;
            if (turn != second_half) __builtin_amdgcn_s_setprio(kPrioLevel); else __builtin_amdgcn_s_setprio(0);
        }
        const bool more = x + stride < wx1;
        Cursor nxt = cur;
        if (more) ts_.advance(nxt, stride); // the wave's last tile re-reads itself: a valid address, the data is ignored
        const int64_t row0_next = nxt.row;

        if (__builtin_expect(!have, 0)) { // the common tile continues a unit: that path runs straight through
            have = true;
            // first of this unit's NREP query heads
            unit0 = ((int64_t)cur.li * p.stream.num_agents + cur.agent) * p.q_heads + (int64_t)cur.kvh * NREP;
            // ---- new unit: its query heads.  Query operand of the matrix core, one per (chunk, word): row
            // i = lane % 16 stands for query head i % NREP and group-in-chunk (i / NREP) % KGPC; the lane holds
            // the 8 dims of its k-block in the order unpack_codes emits codes (0,4,1,5,2,6,3,7), odd dims divided
            // by 16 because their codes arrive 16 times larger, and zeros when its k-block belongs to the row's
            // other group.
            const uint16_t *qrow = p.q + unit0 * DK;
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
            // sum of q over each 64-wide group: eight lanes per group, 8 dims each, folded inside the octet
            for (int base = 0; base < NREP * GK * 8; base += kWave) {
                const int idx = base + lane;
                if (idx < NREP * GK * 8) {
                    const uint4 raw = *reinterpret_cast<const uint4 *>(qrow + idx * 8);
                    const half2_t a = bits_to_half2(raw.x), b = bits_to_half2(raw.y), c = bits_to_half2(raw.z),
                                  d = bits_to_half2(raw.w);
                    float s = ((float)a.x + (float)a.y) + ((float)b.x + (float)b.y) + ((float)c.x + (float)c.y) +
                              ((float)d.x + (float)d.y);
                    s += Q4KV_DPP(0.0f, s, 0xB1, 0xF);  // quad_perm [1,0,3,2]
                    s += Q4KV_DPP(0.0f, s, 0x4E, 0xF);  // quad_perm [2,3,0,1]
                    s += Q4KV_DPP(0.0f, s, 0x141, 0xF); // row_half_mirror
                    if ((idx & 7) == 0) qsum_lds[idx >> 3] = s;
                }
            }
            wave_lds_sync();
#pragma unroll
            for (int rr = 0; rr < NREP; ++rr) {
#pragma unroll
                for (int g = 0; g < GK; ++g) qsum[rr][g] = qsum_lds[rr * GK + g];
                m_run[rr] = kNegBig;
                l_run[rr] = 0.0f;
#pragma unroll
                for (int g = 0; g < GV; ++g) pb[rr][g] = 0.0f;
            }
#pragma unroll
            for (int h = 0; h < VHQ; ++h)
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[h][e] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
        }

        // ---- K side: q.c per (token, head, group) on the matrix core, results to LDS in token order;
        // two 16-token sets at a time keep the accumulators few
#pragma unroll
        for (int tp = 0; tp < KSETS; tp += 2) {
            float4_t d[2][KCHUNKS];
#pragma unroll
            for (int ts = 0; ts < 2; ++ts)
#pragma unroll
                for (int c = 0; c < KCHUNKS; ++c) d[ts][c] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int w = 0; w < KWPL; ++w)
#pragma unroll
                for (int ts = 0; ts < 2; ++ts)
#pragma unroll
                    for (int c = 0; c < KCHUNKS; ++c) {
                        const CodePairs cp = unpack_codes(kc[tp + ts][c].w[w]);
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
                for (int ts = 0; ts < 2; ++ts)
#pragma unroll
                    for (int c = 0; c < KCHUNKS; ++c) {
                        float *dst = part + (((tp + ts) * 16 + kj) * GK + c * KGPC) * NREP + 4 * kkb;
#pragma unroll
                        for (int e = 0; e < kRegs; ++e) dst[e] = d[ts][c][e];
                    }
            }
            load_k_pair(tp, row0_next); // these registers are free again: the next tile's codes start travelling
        }
        wave_lds_sync();

        // ---- the lane that owns token `lane`: finish its scores, online softmax, publish p*s
        const bool tok_valid = cur.reachable && (cur.t0 + lane >= cur.first) && (cur.t0 + lane < cur.n);
        float ks[GK], kb[GK], vs[GV], vb[GV];
#pragma unroll
        for (int g = 0; g < GK; ++g) {
            ks[g] = group_value<GK, BF>(ks_bits, g) * kCodeScaleA;
            kb[g] = group_value<GK, BF>(kb_bits, g);
        }
#pragma unroll
        for (int g = 0; g < GV; ++g) {
            vs[g] = group_value<GV, BF>(vs_bits, g);
            vb[g] = group_value<GV, BF>(vb_bits, g);
        }
        load_params(row0_next);
        // With four or eight query heads per KV head the second term of p*s is a matrix instruction of its own, and
        // a tile takes it only when it has to: one term errs by at most 2^-12 * 15 s per unit of probability, which
        // stays below 1.8e-3 (inside the output tolerance whatever the values are) while every scale of the tile is
        // at most kOneTermScale.  Unit-variance values have scales around 0.3.
        bool two_terms = true;
        if constexpr (!kTermRows) {
            float s_max = 0.0f;
#pragma unroll
            for (int g = 0; g < GV; ++g) s_max = fmaxf(s_max, fabsf(vs[g]));
            two_terms = __builtin_amdgcn_ballot_w64(tok_valid && !(s_max <= kOneTermScale)) != 0ull;
        }
        // A masked row's parameters may hold anything (a NaN included): zeroed once here, they need no further
        // guard in the products below
        if (!tok_valid) {
#pragma unroll
            for (int g = 0; g < GV; ++g) vs[g] = vb[g] = 0.0f;
        }
        float alpha[NREP], z[NREP], mx[NREP], pr[NREP];
#pragma unroll
        for (int r = 0; r < NREP; ++r) {
            float zr = 0.0f;
#pragma unroll
            for (int g = 0; g < GK; ++g) {
                zr = fmaf(ks[g], part[(lane * GK + g) * NREP + r], zr);
                zr = fmaf(kb[g], qsum[r][g], zr);
            }
            z[r] = mx[r] = tok_valid ? zr * p.score_scale : kNegBig;
        }
        wave_max_n(mx); // the tile's maximum of every head, the heads' reductions interleaved
        // The running maxima settle after a unit's first tiles: one wave-uniform test for all heads, and a tile that
        // moves none of them takes no exponential for the factors (exp2(0) = 1: the same bits either way).
        bool any_moved = false;
#pragma unroll
        for (int r = 0; r < NREP; ++r) any_moved |= mx[r] > m_run[r];
        const bool moved = uniform((int)any_moved) != 0;
#pragma unroll
        for (int r = 0; r < NREP; ++r) alpha[r] = 1.0f;
        if (__builtin_expect(moved, 0)) {
#pragma unroll
            for (int r = 0; r < NREP; ++r) {
                const float m_new = fmaxf(m_run[r], mx[r]);
                alpha[r] = __builtin_amdgcn_exp2f(m_run[r] - m_new);
                m_run[r] = m_new;
            }
        }
#pragma unroll
        for (int r = 0; r < NREP; ++r) {
            pr[r] = tok_valid ? __builtin_amdgcn_exp2f(z[r] - m_run[r]) : 0.0f;
            l_run[r] = fmaf(l_run[r], alpha[r], pr[r]);
#pragma unroll
            for (int g = 0; g < GV; ++g) {
                const half_t hi = (half_t)(pr[r] * vs[g]);
                ps_h[(r * GV + g) * kWave + ps_slot] = __builtin_bit_cast(uint16_t, hi);
                pb[r][g] = fmaf(pb[r][g], alpha[r], pr[r] * vb[g]);
            }
        }
        if (kTermRows || __builtin_expect(two_terms, 0)) { // wave-uniform; one block for all heads: what each hi rounded away
#pragma unroll
            for (int r = 0; r < NREP; ++r)
#pragma unroll
                for (int g = 0; g < GV; ++g) {
                    const half_t hi = (half_t)(pr[r] * vs[g]);
                    const half_t lo = (half_t)fmaf(pr[r], vs[g], -(float)hi);
                    ps_h[((NREP + r) * GV + g) * kWave + ps_slot] = __builtin_bit_cast(uint16_t, lo);
                }
        }
        wave_lds_sync();

        // ---- V side: acc[head][e] += (p s)[t] * c[t][e], four tokens per matrix instruction
        // One wave-uniform test for all heads: a branch per head made the compiler copy the accumulators round
        // every one of them.  The running maxima settle after a unit's first tiles, so this is rarely taken.
        if (__builtin_expect(moved, 0)) {
#pragma unroll
            for (int row = 0; row < (kTermRows ? VROWS : NREP); ++row)
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[row / 4][e][row % 4] *= alpha[row % NREP];
        }
#pragma unroll
        for (int i = 0; i < VSTEPS; i += 4) {
            constexpr int kTerms = kTermRows ? 1 : 2; // matrix instructions per accumulator and step (the second: if needed)
            half4_t pq[kTerms][VHQ];
#pragma unroll
            for (int t = 0; t < kTerms; ++t)
#pragma unroll
                for (int h = 0; h < VHQ; ++h) {
                    const uint2 raw = ps_q[((t * NREP + h * 4 + v_row) * GV + vg) * (kWave / 4) + VTPS * (i / 4) + vo];
                    pq[t][h] = __builtin_bit_cast(half4_t, raw);
                }
            half4_t lo[4], hi[4];
#pragma unroll
            for (int by = 0; by < 4; ++by) {
                // byte `by` of the four tokens' words: codes 2*by (low nibble) and 2*by+1 (high nibble)
                const uint32_t sel = 0x0C040C00u + by * 0x00010001u;
                const uint32_t p01 = __builtin_amdgcn_perm(vc[i + 1], vc[i], sel);
                const uint32_t p23 = __builtin_amdgcn_perm(vc[i + 3], vc[i + 2], sel);
                lo[by] = __builtin_bit_cast(half4_t, make_uint2(p01 & 0x000F000Fu, p23 & 0x000F000Fu));
                hi[by] = __builtin_bit_cast(half4_t, make_uint2(p01 & 0x00F000F0u, p23 & 0x00F000F0u));
#pragma unroll
                for (int h = 0; h < VHQ; ++h) {
                    acc[h][2 * by] = __builtin_amdgcn_mfma_f32_4x4x4f16(pq[0][h], lo[by], acc[h][2 * by], 0, 0, 0);
                    acc[h][2 * by + 1] = __builtin_amdgcn_mfma_f32_4x4x4f16(pq[0][h], hi[by], acc[h][2 * by + 1], 0, 0, 0);
                }
            }
            if constexpr (kTerms == 2) {
                // one wave-uniform test per four tokens' words (a test per byte put sixteen taken branches into every
                // tile of the usual cache, which needs no second term)
                if (__builtin_expect(two_terms, 0)) {
#pragma unroll
                    for (int by = 0; by < 4; ++by)
#pragma unroll
                        for (int h = 0; h < VHQ; ++h) {
                            acc[h][2 * by] = __builtin_amdgcn_mfma_f32_4x4x4f16(pq[1][h], lo[by], acc[h][2 * by], 0, 0, 0);
                            acc[h][2 * by + 1] = __builtin_amdgcn_mfma_f32_4x4x4f16(pq[1][h], hi[by], acc[h][2 * by + 1], 0, 0, 0);
                        }
                }
            }
            load_v_quad(i, row0_next);
        }
        wave_lds_sync(); // the next tile (or the reduction below) overwrites part / ps

        cur = nxt;
        x += stride;
        active = more;
    }
}

template <int DK, int DV, int NREP>
hipError_t launch_decode_t(const AttentionArgs &a, hipStream_t stream)
{
    DecodeParams p;
    p.k_codes = a.k.codes; p.k_scale = a.k.scale; p.k_bias = a.k.bias;
    p.v_codes = a.v.codes; p.v_scale = a.v.scale; p.v_bias = a.v.bias;
    p.q = a.q;
    p.stream = stream_params(a);
    p.merge = merge_params(a);
    p.q_heads = a.spec.num_q_heads;
    p.score_scale = a.sm_scale * kLog2e;
    if (a.spec.param_format == Q4KV_PARAMS_BF16)
        hipLaunchKernelGGL((decode_attention_kernel<DK, DV, NREP, true>), dim3(a.grid_workgroups), dim3(kThreads), 0, stream, p);
    else
        hipLaunchKernelGGL((decode_attention_kernel<DK, DV, NREP, false>), dim3(a.grid_workgroups), dim3(kThreads), 0, stream, p);
    return hipGetLastError();
}

template <int DK, int DV>
hipError_t launch_decode_d(const AttentionArgs &a, int n_rep, hipStream_t stream)
{
    switch (n_rep) {
    case 1: return launch_decode_t<DK, DV, 1>(a, stream);
    case 2: return launch_decode_t<DK, DV, 2>(a, stream);
    case 4: return launch_decode_t<DK, DV, 4>(a, stream);
    case 8: return launch_decode_t<DK, DV, 8>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

} // namespace

StreamParams stream_params(const AttentionArgs &a)
{
    StreamParams s;
    s.plan = a.plan;
    s.block_table = a.block_table;
    s.num_agents = a.num_agents;
    s.max_blocks = a.max_blocks;
    s.kv_heads = a.spec.num_kv_heads;
    s.num_blocks = a.k.num_blocks;
    s.layer_begin = a.layer_begin;
    s.layers = a.layers_in_call;
    s.plan_signature = a.plan_signature;
    return s;
}

MergeParams merge_params(const AttentionArgs &a)
{
    MergeParams m;
    m.part_acc = a.part_acc;
    m.part_ml = a.part_ml;
    m.arrivals = a.arrivals;
    m.out = a.out;
    m.max_slots = a.max_slots;
    return m;
}

hipError_t launch_plan(const AttentionArgs &a, int workers, int per_multiple, hipStream_t stream)
{
    LayerWindows lw;
    lw.uniform = a.layer_window == nullptr;
    lw.window = a.window;
    for (int i = 0; i < kMaxWindowLayers; ++i) lw.w[i] = (!lw.uniform && i < a.layers_in_call) ? a.layer_window[i] : 0;
    // workgroup 0 plans; one more per 8,192 arrival counters (at most 256) helps clearing them
    const int64_t counters = (int64_t)a.layers_in_call * a.spec.num_kv_heads * a.num_agents;
    const int helpers = (int)(counters / 8192 < 256 ? counters / 8192 : 256);
    hipLaunchKernelGGL(plan_kernel, dim3(1 + helpers), dim3(kThreads), 0, stream, a.seq_len, a.num_agents, a.max_seq_len,
                       lw, a.layers_in_call, a.spec.num_kv_heads, workers, a.split_tokens / kWave, per_multiple, a.plan_signature,
                       a.plan, a.arrivals);
    return hipGetLastError();
}

int decode_waves_per_workgroup() { return kWaves; }

int decode_solo_quarter_tiles() { return kCoopMaxTiles / kWaves; }

int max_window_layers() { return kMaxWindowLayers; }

size_t decode_plan_ints(int num_agents, int layers) { return PlanView::ints(num_agents, layers); }

bool decode_supported(const q4kv_spec &s)
{
    const int n_rep = s.num_q_heads / s.num_kv_heads;
    const bool rep_ok = n_rep == 1 || n_rep == 2 || n_rep == 4 || n_rep == 8;
    const bool square = (s.k_dim == 64 || s.k_dim == 128 || s.k_dim == 256) && s.v_dim == s.k_dim;
    const bool mla_per_head = s.k_dim == 192 && s.v_dim == 128; // decompressed per-head MLA cache (Sec. 3.6)
    return rep_ok && (square || mla_per_head) && !s.v_aliases_k;
}

// the workers of the tile stream are workgroups here, with ranges that divide among four waves
hipError_t launch_decode_plan(const AttentionArgs &a, hipStream_t stream)
{
    return launch_plan(a, a.grid_workgroups, kWaves, stream);
}

hipError_t launch_decode_attention(const AttentionArgs &a, hipStream_t stream)
{
    const int n_rep = a.spec.num_q_heads / a.spec.num_kv_heads;
    switch (a.spec.k_dim) {
    case 64: return launch_decode_d<64, 64>(a, n_rep, stream);
    case 128: return launch_decode_d<128, 128>(a, n_rep, stream);
    case 192: return launch_decode_d<192, 128>(a, n_rep, stream);
    case 256: return launch_decode_d<256, 256>(a, n_rep, stream);
    default: return hipErrorInvalidValue;
    }
}

} // namespace q4kv

// Chunked-append causal attention over paged Q4 KV caches (Sec. 3.4 chunked prefill, Sec. 3.5 cross-phase
// append, Sec. 3.6 causal and sliding-window masks): every agent brings q_len new query tokens whose K/V have
// already been quantize-appended, and query token c of agent a attends to the first
// seq_len[a] - (q_len-1-c) tokens of that agent's cache -- the chunk's own keys in their Q4 form included.
//
// Unlike decode this is a dense contraction: the q_len * n_rep query rows that share one KV head form the
// M side of two GEMMs per KV tile (S = Q K^T, O += P V), so it runs on the matrix cores and is bound by them.
//
//  * A workgroup (4 waves) owns 128 query rows of one (layer, agent, KV head): 128/n_rep consecutive chunk
//    positions times the n_rep query heads of the group.  Each wave owns 32 rows.
//  * KV tiles of 64 tokens are fetched as Q4 (codes + scale/bias, coalesced 16-byte loads, prefetched one
//    tile ahead into registers) and staged ONCE per workgroup in LDS for all 128 rows, row-major: V_hat
//    dequantized to binary16, K as the packed code words themselves (a quarter of the LDS traffic of binary16
//    keys; a lane's A operand of a matrix instruction is exactly one word).  The dims inside a word appear in the
//    order the nibble masks deliver them (0,4,1,5,2,6,3,7): the query operand uses the same order for K, the
//    output store undoes it for V_hat.
//  * K stays factored, S^T = sum_g s[t,g] (C_g Q_g^T) + b Qsum^T: a code word masked in place is eight binary16
//    subnormals (c 2^-24, odd nibbles 16 c 2^-24 against q/16), the matrix core multiplies them exactly, and the
//    per-(token, group) scale meets the binary32 result of each group; the bias term is one more matrix
//    instruction per 16 tokens whose contraction runs over the groups (group sums of q split into a binary16 high
//    and low part).  A K row dequantized to binary16 would carry an absolute rounding error of 2^-11 |K_hat|,
//    which the large channels of real key caches turn into score errors of several 1e-3.  V_hat is dequantized
//    to binary16 (its rounding error is relative to the values that are averaged).
//  * The wave computes S^T (tokens are the M rows), so that the probabilities come out of the
//    matrix core already in the register layout the second GEMM wants for its B operand (P^T); no shuffle
//    or LDS round trip between the GEMMs.  O^T = V_hat^T P^T accumulates in binary32; its A operand wants 8
//    tokens of one dim per lane, which the transposing LDS read (ds_read_b64_tr_b16) delivers straight from the
//    row-major tile: in a group of 16 lanes, lane 4e + c points at 4 consecutive dims (chunk c) of token e, and
//    element e of what lane j receives is half j % 4 of the chunk that lane 4e + j / 4 addressed, i.e. dim j of
//    token e.
//  * Softmax is online, per query row (= per lane column): scores in binary32, log2 domain.
//  * The workgroups of one KV head are adjacent in the launch order of ONE XCD, so the 8 query tiles of a
//    unit stream the same KV tiles through the same L2 at the same time.
#include "q4_device.h"
#include "q4kv_internal.h"

namespace q4kv {
namespace {

constexpr int kRowsWG = 128;  // query rows per workgroup
constexpr int kTile = 64;     // KV tokens per tile
constexpr float kNegBig = -1.0e30f;
constexpr float kLog2e = 1.4426950408889634f;
constexpr int kXcds = 8;
constexpr int kMaxChunkWindowLayers = 128; // layers per call when every layer brings its own window

struct ChunkParams {
    const uint32_t *k_codes, *v_codes;
    const uint16_t *k_scale, *k_bias, *v_scale, *v_bias;
    const uint16_t *q;
    uint16_t *out;
    const int32_t *block_table, *seq_len;
    int num_blocks, kv_heads, q_heads, num_agents, max_blocks, max_seq_len, window, q_len;
    int layer_begin, layers_in_call, q_tiles;
    float score_scale;
    int per_layer_windows;          // 1: layer_window[] holds the window of every layer of the call
    int layer_window[kMaxChunkWindowLayers];
};

__device__ __forceinline__ half2_t pk_fma(half2_t a, half2_t b, half2_t c) { return a * b + c; }

// two nibble positions of a word pair as exact small integers in binary16:
// ((w & mask) | 0x6400.6400) is 1024 + c (or 1024 + 16c for the upper nibble of a byte); subtracting 1024 is exact
__device__ __forceinline__ half2_t nibbles_lo(uint32_t w)
{
    return bits_to_half2((w & 0x000F000Fu) | 0x64006400u) - half2_t{(half_t)1024.0f, (half_t)1024.0f};
}
__device__ __forceinline__ half2_t nibbles_hi16(uint32_t w) // 16 * code
{
    return bits_to_half2((w & 0x00F000F0u) | 0x64006400u) - half2_t{(half_t)1024.0f, (half_t)1024.0f};
}

typedef short short4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) short4_t *lds_short4_ptr;

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

// How the threads of a workgroup share the staging of one 64-row tile of DIM-wide code rows: as many threads per row
// as fit, each with 2, 4 or 8 consecutive words (never across a quantization group).
template <int DIM, int THREADS>
struct Stage {
    static constexpr int WORDS = DIM / 8; // code words per row
    static constexpr int WPT = kTile * (WORDS / 2) <= THREADS ? 2 : (kTile * (WORDS / 4) <= THREADS ? 4 : 8);
    static constexpr int TPR = WORDS / WPT; // threads per row
    static constexpr int ACTIVE = kTile * TPR;
    static_assert(WORDS % WPT == 0 && ACTIVE <= THREADS, "tile split");
};

// QT: 16-row query tiles per wave.  Two tiles halve the LDS operand traffic per matrix instruction; one tile keeps
// a wave within 256 registers also at D = 256, so that two waves share a SIMD and one wave's dequantization and
// softmax run under the other's matrix instructions.  The workgroup always owns 128 rows: 128 / (16 QT) waves.
// BF: scale and bias are stored as bfloat16 (converted to binary16 when a row is staged).
// (Two tiles at 192-wide keys need more than 256 registers: one wave per SIMD there, no scratch.)
template <int DK, int DV, int NREP, int QT, bool BF>
__global__ __launch_bounds__(kRowsWG / (16 * QT) * kWave, (QT == 2 && DK > 128) ? 1 : 2) void chunk_attention_kernel(ChunkParams p)
{
    constexpr int kRowsWave = 16 * QT;
    constexpr int kWaves = kRowsWG / kRowsWave;
    constexpr int kThreads = kWaves * kWave;
    constexpr int GK = DK / kGroup, GV = DV / kGroup;
    // row pitches of the tiles in LDS.  K rows (32-bit code words) are read one word per lane by 16 rows x 4 words at
    // a time: a pitch of 4 x odd words spreads those over all 64 banks.  V_hat rows (halves) are read 8 bytes per
    // lane by 4 rows x 32 bytes at a time (pitch = 32 bytes mod 256).
    constexpr int KPITCH = DK / 8 + 4;
    constexpr int VPITCH = DV + 16;
    constexpr int QPOS = kRowsWG / NREP; // chunk positions per workgroup
    constexpr int KSTEPS = DK / 32;    // k-steps of the QK contraction
    constexpr int ETILES = DV / 16;    // 16-row tiles of O^T
    typedef Stage<DK, kThreads> SK;    // staging of the K rows of a tile ...
    typedef Stage<DV, kThreads> SV;    // ... and of its V rows

    // two tiles each: while the waves multiply against one, they unpack the next into the other
    __shared__ __attribute__((aligned(16))) uint32_t k_lds[2][kTile * KPITCH]; // K code words as they are in the pool
    __shared__ __attribute__((aligned(16))) half_t v_lds[2][kTile * VPITCH]; // V_hat
    __shared__ __attribute__((aligned(16))) half_t ks_lds[2][GK * kTile];    // K scale [group][token]
    // K bias [token][8]: groups 0..3 (zero padded) twice, against the high and the low parts of the group sums of q
    __shared__ __attribute__((aligned(16))) half_t kb_lds[2][kTile * 8];

    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);

    // ---- which (layer, agent, kv head, query tile): consecutive workgroups of one XCD share a KV head
    const int per_xcd_slot = blockIdx.x / kXcds, xcd = blockIdx.x % kXcds;
    const int unit_in_xcd = per_xcd_slot / p.q_tiles, qt = per_xcd_slot % p.q_tiles;
    const int unit = unit_in_xcd * kXcds + xcd; // ((layer in call) * agents + agent) * kv_heads + kv head
    const int total_units = p.layers_in_call * p.num_agents * p.kv_heads;
    if (unit >= total_units) return;
    const int kvh = unit % p.kv_heads, agent = (unit / p.kv_heads) % p.num_agents, li = unit / (p.kv_heads * p.num_agents);
    const int layer = p.layer_begin + li;

    int n = p.seq_len[agent];
    n = n < 0 ? 0 : (n > p.max_seq_len ? p.max_seq_len : n);
    const int window = p.per_layer_windows ? p.layer_window[li] : p.window;
    const int pos0 = qt * QPOS;                   // first chunk position of this workgroup
    if (pos0 >= p.q_len) return;
    // chunk position c sees tokens [first(c), vis(c)),  vis(c) = n - (q_len - 1 - c)
    const int vis_last = n - (p.q_len - 1 - min(p.q_len - 1, pos0 + QPOS - 1)); // keys visible to the last row here
    const int vis_first = n - (p.q_len - 1 - pos0);
    int t_begin = 0;
    if (window > 0 && vis_first - window > 0) t_begin = (vis_first - window) & ~(kTile - 1);
    const int t_end = vis_last; // exclusive; may be <= 0 when nothing is visible

    // ---- this lane's query rows: column n = lane % 16 of the two 16-row tiles of its wave
    const int qn = lane % 16, kb = lane / 16;
    int row_pos[QT], row_vis[QT], row_first[QT];
    half8_t qop[QT][KSTEPS];
    half8_t qsop[QT]; // lanes kb == 0: group sums of this row's q, high parts in slots 0..3, low parts in 4..7; else 0
    const int64_t q_agent = ((int64_t)li * p.num_agents + agent) * p.q_len;
#pragma unroll
    for (int qi = 0; qi < QT; ++qi) {
        const int r_w = wave * kRowsWave + qi * 16 + qn;   // row inside the workgroup
        const int c = pos0 + r_w / NREP, head = kvh * NREP + r_w % NREP;
        row_pos[qi] = c;
        const bool live = c < p.q_len;
        row_vis[qi] = live ? n - (p.q_len - 1 - c) : 0;
        row_first[qi] = (window > 0 && row_vis[qi] > window) ? row_vis[qi] - window : 0;
        const uint16_t *src = p.q + ((q_agent + (live ? c : 0)) * p.q_heads + head) * DK;
        float qs[GK];
#pragma unroll
        for (int g = 0; g < GK; ++g) qs[g] = 0.0f;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            // dims 32*ks + 8*kb .. +7 in the order the nibble masks emit them: 0,4,1,5,2,6,3,7; the odd ones divided
            // by 16 because their codes arrive 16 times larger
            const uint4 raw = *reinterpret_cast<const uint4 *>(src + 32 * ks + 8 * kb);
            const half2_t e01 = bits_to_half2(raw.x), e23 = bits_to_half2(raw.y);
            const half2_t e45 = bits_to_half2(raw.z), e67 = bits_to_half2(raw.w);
            const half_t sixteenth = (half_t)0.0625f;
            qop[qi][ks] = half8_t{e01.x, e45.x, e01.y * sixteenth, e45.y * sixteenth,
                                  e23.x, e67.x, e23.y * sixteenth, e67.y * sixteenth};
            qs[ks / 2] += ((float)e01.x + (float)e01.y) + ((float)e23.x + (float)e23.y) +
                          ((float)e45.x + (float)e45.y) + ((float)e67.x + (float)e67.y);
        }
        half_t part[8];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const float v = g < GK ? xor32_sum(xor16_sum(qs[g < GK ? g : 0])) : 0.0f; // over the four lanes of the row
            const half_t hi = (half_t)v;
            part[g] = kb == 0 ? hi : (half_t)0.0f;
            part[4 + g] = kb == 0 ? (half_t)(v - (float)hi) : (half_t)0.0f;
        }
        qsop[qi] = half8_t{part[0], part[1], part[2], part[3], part[4], part[5], part[6], part[7]};
    }
    // what every row of this wave sees / hides (rows differ along lane % 16): tiles inside [all_first, all_vis)
    // need no masks
    int all_vis = row_vis[0], all_first = row_first[0];
#pragma unroll
    for (int qi = 1; qi < QT; ++qi) {
        all_vis = min(all_vis, row_vis[qi]);
        all_first = max(all_first, row_first[qi]);
    }
#pragma unroll
    for (int s = 1; s < 16; s <<= 1) {
        all_vis = min(all_vis, __shfl_xor(all_vis, s, kWave));
        all_first = max(all_first, __shfl_xor(all_first, s, kWave));
    }

    float4_t o_acc[QT][ETILES]; // O^T: [q tile][16-dim tile], lane column = query row, regs = row positions 4*kb .. 4*kb+3
#pragma unroll
    for (int qi = 0; qi < QT; ++qi)
#pragma unroll
        for (int et = 0; et < ETILES; ++et) o_acc[qi][et] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
    // m_run: the reference the exponentials are taken against.  It moves only when a tile's maximum exceeds it by
    // more than kSlack (log2 units), so the accumulators are rescaled a few times per row, not once per tile.
    constexpr float kSlack = 3.0f;
    float m_run[QT], l_run[QT];
#pragma unroll
    for (int qi = 0; qi < QT; ++qi) {
        m_run[qi] = kNegBig;
        l_run[qi] = 0.0f;
    }

    // ---- KV tile staging: raw Q4 in registers one tile ahead.  A thread takes WPT consecutive words of one token's
    // K row and (the same ones when the rows are equally wide) of one token's V row; with rows that do not divide
    // evenly the last waves stage nothing
    const int32_t *table = p.block_table + (int64_t)agent * p.max_blocks;
    uint32_t kraw[SK::WPT], vraw[SV::WPT];
    uint32_t ksb[2], vsb[2]; // scale / bias bits of the group this thread unpacks
    // 16 consecutive lanes take 16 consecutive tokens (and the same part of the row): their 16-byte LDS stores then
    // fall into 16 different bank groups, like the operand reads
    const bool k_on = SK::ACTIVE == kThreads || tid < SK::ACTIVE, v_on = SV::ACTIVE == kThreads || tid < SV::ACTIVE;
    const int k_tok = k_on ? (tid % 16) + 16 * (tid / (16 * SK::TPR)) : 0, k_w0 = ((tid / 16) % SK::TPR) * SK::WPT;
    const int v_tok = v_on ? (tid % 16) + 16 * (tid / (16 * SV::TPR)) : 0, v_w0 = ((tid / 16) % SV::TPR) * SV::WPT;
    const int k_grp = (k_w0 * 8) / kGroup, v_grp = (v_w0 * 8) / kGroup;
    // A block id outside the pool: the tile's (unconditional) loads go to the agent's own first block instead -- to
    // block 0 only if that id is outside the pool as well -- and everything they bring is discarded.
    const int own0 = table[0];
    const int fallback_blk = own0 >= 0 && own0 < p.num_blocks ? own0 : 0;
    auto tile_row0 = [&](int t0, bool &ok) {
        const int bi = t0 / kBlockTokens;
        const int blk = bi < p.max_blocks ? table[bi] : -1;
        ok = blk >= 0 && blk < p.num_blocks;
        return (((int64_t)layer * p.num_blocks + (ok ? blk : fallback_blk)) * p.kv_heads + kvh) * kBlockTokens + (t0 % kBlockTokens);
    };
    auto load_words = [&](const uint32_t *src, auto &dst) {
        constexpr int N = sizeof(dst) / sizeof(uint32_t);
        if constexpr (N % 4 == 0) {
#pragma unroll
            for (int i = 0; i < N / 4; ++i) {
                const uint4 t = *reinterpret_cast<const uint4 *>(src + 4 * i);
                dst[4 * i] = t.x; dst[4 * i + 1] = t.y; dst[4 * i + 2] = t.z; dst[4 * i + 3] = t.w;
            }
        } else {
            const uint2 t = *reinterpret_cast<const uint2 *>(src);
            dst[0] = t.x; dst[1] = t.y;
        }
    };
    // threads without a share load row 0 of the tile again (a valid address) and never store
    auto load_tile = [&](int t0, bool &ok) {
        const int64_t row0 = tile_row0(t0, ok);
        const int64_t krow = row0 + k_tok, vrow = row0 + v_tok;
        load_words(p.k_codes + krow * SK::WORDS + (k_on ? k_w0 : 0), kraw);
        load_words(p.v_codes + vrow * SV::WORDS + (v_on ? v_w0 : 0), vraw);
        ksb[0] = p.k_scale[krow * GK + (k_on ? k_grp : 0)];
        ksb[1] = p.k_bias[krow * GK + (k_on ? k_grp : 0)];
        vsb[0] = p.v_scale[vrow * GV + (v_on ? v_grp : 0)];
        vsb[1] = p.v_bias[vrow * GV + (v_on ? v_grp : 0)];
    };
    // unpack the staged words of one row into LDS (V: dequantized; K: codes, see store_codes).  Rows of an unreachable block and rows at or past t_end
    // (never visible, possibly never written) become zeros, so that no stale bit pattern can reach an accumulator.
    // Dequantization of the staged rows happens one code word (8 dims, one 16-byte store) at a time, so that the
    // matrix loops below can take a word between their steps: a wave cannot overlap its own vector and matrix
    // instructions, but the other wave of its SIMD fills in whenever both streams are mixed rather than phased.
    struct RowDequant {
        half2_t s2, s16, b2;
        bool ok;
    };
    auto row_params = [&](const uint32_t (&sb)[2], bool ok) {
        RowDequant r;
        // bfloat16 parameters of binary16-range data convert exactly (8 significant bits into 11) unless they are
        // below 2^-14, where the difference is far below what binary16 operands resolve anyway
        const half_t s_in = BF ? (half_t)bf16_bits_to_float((uint16_t)sb[0]) : __builtin_bit_cast(half_t, (uint16_t)sb[0]);
        const half_t b_in = BF ? (half_t)bf16_bits_to_float((uint16_t)sb[1]) : __builtin_bit_cast(half_t, (uint16_t)sb[1]);
        const half_t s = ok ? s_in : (half_t)0.0f;
        const half_t b = ok ? b_in : (half_t)0.0f;
        r.s2 = half2_t{s, s};
        r.b2 = half2_t{b, b};
        r.s16 = r.s2 * half2_t{(half_t)0.0625f, (half_t)0.0625f};
        r.ok = ok;
        return r;
    };
    auto store_word = [&](half_t *dst, uint32_t raw, const RowDequant &r) {
        const uint32_t word = r.ok ? raw : 0u, w8 = word >> 8;
        const half2_t v0 = pk_fma(nibbles_lo(word), r.s2, r.b2);    // dims 0, 4
        const half2_t v1 = pk_fma(nibbles_hi16(word), r.s16, r.b2); // dims 1, 5
        const half2_t v2 = pk_fma(nibbles_lo(w8), r.s2, r.b2);      // dims 2, 6
        const half2_t v3 = pk_fma(nibbles_hi16(w8), r.s16, r.b2);   // dims 3, 7
        *reinterpret_cast<uint4 *>(dst) = make_uint4(half2_to_bits(v0), half2_to_bits(v1), half2_to_bits(v2), half2_to_bits(v3));
    };
    // K rows keep their codes: the nibbles masked in place are binary16 subnormals c 2^-24 (dims 0, 4, 2, 6 of a
    // word) and 16 c 2^-24 (dims 1, 5, 3, 7); the row's scale and bias go to LDS beside them, written by the thread
    // that holds the first word of the group
    // the staged K words of this thread go to LDS as they are, 16 (or 8) bytes per store: 16 consecutive lanes
    // are 16 consecutive tokens, whose rows start 4 x odd banks apart
    auto store_codes = [&](uint32_t *dst, const uint32_t (&raw)[SK::WPT], bool ok) {
        if constexpr (SK::WPT % 4 == 0) {
#pragma unroll
            for (int w = 0; w < SK::WPT; w += 4)
                *reinterpret_cast<uint4 *>(dst + w) =
                    ok ? make_uint4(raw[w], raw[w + 1], raw[w + 2], raw[w + 3]) : make_uint4(0u, 0u, 0u, 0u);
        } else {
            *reinterpret_cast<uint2 *>(dst) = ok ? make_uint2(raw[0], raw[1]) : make_uint2(0u, 0u);
        }
    };
    // a code word as the A operand of a matrix instruction: the nibbles masked in place are binary16 subnormals
    // c 2^-24 (dims 0, 4, 2, 6 of the word) and 16 c 2^-24 (dims 1, 5, 3, 7)
    auto code_operand = [&](uint32_t w) {
        const uint32_t w8 = w >> 8;
        return __builtin_bit_cast(half8_t, make_uint4(w & 0x000F000Fu, w & 0x00F000F0u, w8 & 0x000F000Fu, w8 & 0x00F000F0u));
    };
    const bool k_params_writer = k_on && (k_w0 * 8) % kGroup == 0;
    auto store_k_params = [&](int b, const RowDequant &r) {
        ks_lds[b][k_grp * kTile + k_tok] = r.s2.x;
        kb_lds[b][k_tok * 8 + k_grp] = r.b2.x;
        kb_lds[b][k_tok * 8 + 4 + k_grp] = r.b2.x;
    };
    if constexpr (GK < 4) { // bias slots of groups the rows do not have: zero once (their q sums are zero too)
        for (int i = tid; i < 2 * kTile * 8 / 2; i += kThreads) reinterpret_cast<uint32_t *>(&kb_lds[0][0])[i] = 0u;
        __syncthreads();
    }
    // rows of an unreachable block and rows at or past t_end (never visible, possibly never written) become zeros,
    // so that no stale bit pattern can reach an accumulator
    auto row_ok = [&](int t0, int tok, bool ok_tile) { return ok_tile && (t0 + tok < t_end); };
    const int k_dst = k_tok * KPITCH + k_w0, v_dst = v_tok * VPITCH + v_w0 * 8;

    // transposing read of V_hat: this lane's address inside a tile for (16-dim tile 0, 32-token block 0, first
    // half): token 4 kb + (lane % 16) / 4, dims 4 (lane % 4) ..
    const int v_lane = (4 * kb + qn / 4) * VPITCH + 4 * (qn % 4);

    // One barrier per tile: tile i is multiplied out of buffer i % 2 while tile i + 1 (already in registers) is
    // unpacked into the other buffer and tile i + 2 is fetched.
    bool ok_next = false, ok_cur = false;
    int buf = 0;
    const int t_last = t_begin < t_end ? t_begin + (t_end - 1 - t_begin) / kTile * kTile : 0; // start of the last tile
    if (t_begin < t_end) {
        load_tile(t_begin, ok_next);
        const RowDequant kr = row_params(ksb, row_ok(t_begin, k_tok, ok_next));
        const RowDequant vr = row_params(vsb, row_ok(t_begin, v_tok, ok_next));
        if (k_on) store_codes(k_lds[0] + k_dst, kraw, kr.ok);
        if (k_params_writer) store_k_params(0, kr);
        if (v_on) {
#pragma unroll
            for (int w = 0; w < SV::WPT; ++w) store_word(v_lds[0] + v_dst + 8 * w, vraw[w], vr);
        }
        ok_cur = ok_next;
        if (t_begin + kTile < t_end) load_tile(t_begin + kTile, ok_next);
    }
    __syncthreads();
    for (int t0 = t_begin; t0 < t_end; t0 += kTile) {
        const uint32_t *k_cur = k_lds[buf];
        const half_t *v_cur = v_lds[buf];

        // ---- S^T = sum_g s_g (C_g Q_g^T) + b Qsum^T : [64 tokens][16 QT query rows] per wave, binary32, in units of
        // 2^-24.  An item is one (group, 16-token tile): two matrix instructions per query tile over the group's 64
        // dims into a fresh accumulator; while they run, the item before meets its scales (one fused multiply-add
        // per score).  Operands and scales are fetched two items ahead; the next tile's K rows go registers -> LDS
        // (other buffer) between the items.  Past the last tile that stores zeros into the idle buffer:
        // straight-line code keeps the mix.
        const bool ok_this = ok_cur;
        const bool more = t0 + kTile < t_end;
        const RowDequant kr = row_params(ksb, row_ok(t0 + kTile, k_tok, ok_next && more));
        const RowDequant vr = row_params(vsb, row_ok(t0 + kTile, v_tok, ok_next && more));
        const half_t *ks_cur = ks_lds[buf], *kb_cur = kb_lds[buf];
        const float4_t zero4 = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
        float4_t st[QT][kTile / 16]; // [q tile][token tile]: lane column = query row, regs = tokens 4*kb .. 4*kb+3
#pragma unroll
        for (int tt = 0; tt < kTile / 16; ++tt) { // bias term: A = b[token][group slots], B = group sums of q
            const half8_t ba = *reinterpret_cast<const half8_t *>(kb_cur + (tt * 16 + qn) * 8);
#pragma unroll
            for (int qi = 0; qi < QT; ++qi) st[qi][tt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ba, qsop[qi], zero4, 0, 0, 0);
        }
        // TPI token tiles per item.  One: the two dependent matrix instructions of an item follow each other
        // directly, which measured faster than pairing token tiles for two independent chains (742 against 732
        // TFLOP/s at D = 256) because the operand ring stays small.
        constexpr int TPI = 1;
        constexpr int kItemsPerGroup = kTile / 16 / TPI;
        constexpr int kItems = GK * kItemsPerGroup;
        constexpr int kAhead = 1; // items the operand reads run ahead (1: 757, 2: 750, 3: 750 TFLOP/s at D = 256)
        struct ItemIn {
            uint32_t a0[TPI], a1[TPI]; // code words of token 16 tt + qn: dims 64 g + 8 kb .. and 64 g + 32 + 8 kb ..
            uint2 s4[TPI];            // scales of tokens 16 tt + 4 kb .. + 3, group g
        };
        auto load_item = [&](int it) {
            const int g = it / kItemsPerGroup, tt0 = (it % kItemsPerGroup) * TPI;
            ItemIn in;
#pragma unroll
            for (int j = 0; j < TPI; ++j) {
                const uint32_t *row = k_cur + ((tt0 + j) * 16 + qn) * KPITCH + 8 * g + kb;
                in.a0[j] = row[0];
                in.a1[j] = row[4];
                in.s4[j] = *reinterpret_cast<const uint2 *>(ks_cur + g * kTile + (tt0 + j) * 16 + 4 * kb);
            }
            return in;
        };
        ItemIn item[kAhead + 1];
#pragma unroll
        for (int it = 0; it < kAhead; ++it) item[it] = load_item(it);
        float4_t dq[2][TPI][QT]; // raw group products of the item in flight and of the one before
        uint2 s_prev[TPI];
#pragma unroll
        for (int it = 0; it <= kItems; ++it) {
            if (it + kAhead < kItems) item[(it + kAhead) % (kAhead + 1)] = load_item(it + kAhead);
            if (it < kItems) {
                const int g = it / kItemsPerGroup;
                const ItemIn &in = item[it % (kAhead + 1)];
#pragma unroll
                for (int j = 0; j < TPI; ++j)
#pragma unroll
                    for (int qi = 0; qi < QT; ++qi)
                        dq[it & 1][j][qi] = __builtin_amdgcn_mfma_f32_16x16x32_f16(code_operand(in.a0[j]), qop[qi][2 * g], zero4, 0, 0, 0);
#pragma unroll
                for (int j = 0; j < TPI; ++j)
#pragma unroll
                    for (int qi = 0; qi < QT; ++qi)
                        dq[it & 1][j][qi] =
                            __builtin_amdgcn_mfma_f32_16x16x32_f16(code_operand(in.a1[j]), qop[qi][2 * g + 1], dq[it & 1][j][qi], 0, 0, 0);
            }
            if (it > 0) { // the item before: scores += scale * product
                const int g = (it - 1) / kItemsPerGroup, tt0 = ((it - 1) % kItemsPerGroup) * TPI;
#pragma unroll
                for (int j = 0; j < TPI; ++j) {
                    const half2_t s01 = bits_to_half2(s_prev[j].x), s23 = bits_to_half2(s_prev[j].y);
#pragma unroll
                    for (int qi = 0; qi < QT; ++qi) {
                        float4_t acc = st[qi][tt0 + j];
                        if (g == 0) acc = acc * 0x1p-24f; // the bias term enters in the products' unit
                        const float4_t d = dq[(it - 1) & 1][j][qi];
                        acc[0] = fmaf((float)s01.x, d[0], acc[0]);
                        acc[1] = fmaf((float)s01.y, d[1], acc[1]);
                        acc[2] = fmaf((float)s23.x, d[2], acc[2]);
                        acc[3] = fmaf((float)s23.y, d[3], acc[3]);
                        st[qi][tt0 + j] = acc;
                    }
                }
            }
            if (it < kItems) {
#pragma unroll
                for (int j = 0; j < TPI; ++j) s_prev[j] = item[it % (kAhead + 1)].s4[j];
            }
            if (it == 0 && k_on) store_codes(k_lds[buf ^ 1] + k_dst, kraw, kr.ok); // the next tile's K words
            if (it == 1 && k_params_writer) store_k_params(buf ^ 1, kr);
            __builtin_amdgcn_sched_barrier(0);
        }
        const float zscale = p.score_scale * 16777216.0f; // scores are in units of 2^-24

        // ---- online softmax per query row (lane column), then P^T in binary16 as the next B operand
        const bool masked = !(ok_this && t0 >= all_first && t0 + kTile <= all_vis); // wave-uniform
        const bool general = masked || !(p.score_scale > 0.0f); // the path that assumes nothing
        half8_t pt[QT][kTile / 32]; // [q tile][32-token block]: tokens 4*kb..+3 of both 16-token tiles of the block
        bool any_moved = false;
        float alpha[QT];
#pragma unroll
        for (int qi = 0; qi < QT; ++qi) {
            float mx = kNegBig;
            if (general) {
#pragma unroll
                for (int tt = 0; tt < kTile / 16; ++tt)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float z = st[qi][tt][e] * zscale;
                        const int t = t0 + tt * 16 + 4 * kb + e;
                        if (!(ok_this && t < row_vis[qi] && t >= row_first[qi])) z = kNegBig;
                        st[qi][tt][e] = z;
                        mx = fmaxf(mx, z);
                    }
            } else { // interior tile, positive scale: the maximum can be taken before the scale is applied
#pragma unroll
                for (int tt = 0; tt < kTile / 16; ++tt)
#pragma unroll
                    for (int e = 0; e < 4; ++e) mx = fmaxf(mx, st[qi][tt][e]);
                mx *= zscale;
            }
            // the row's tokens live in the 4 lanes qn, qn+16, qn+32, qn+48
            mx = xor32_max(xor16_max(mx));
            const bool moved = mx > m_run[qi] + kSlack;
            const float m_new = moved ? mx : m_run[qi];
            alpha[qi] = moved ? __builtin_amdgcn_exp2f(m_run[qi] - m_new) : 1.0f;
            any_moved |= moved;
            m_run[qi] = m_new;
            float sum = 0.0f;
            if (general) {
#pragma unroll
                for (int tt = 0; tt < kTile / 16; ++tt)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float pr = __builtin_amdgcn_exp2f(st[qi][tt][e] - m_new);
                        pr = st[qi][tt][e] > 0.5f * kNegBig ? pr : 0.0f; // also a row with nothing visible yet
                        st[qi][tt][e] = pr;
                        sum += pr;
                    }
            } else {
#pragma unroll
                for (int tt = 0; tt < kTile / 16; ++tt)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float pr = __builtin_amdgcn_exp2f(fmaf(st[qi][tt][e], zscale, -m_new));
                        st[qi][tt][e] = pr;
                        sum += pr;
                    }
            }
            l_run[qi] = fmaf(l_run[qi], alpha[qi], sum); // this lane's tokens only; lanes are added up at the end
#pragma unroll
            for (int tb = 0; tb < kTile / 32; ++tb)
                pt[qi][tb] = half8_t{(half_t)st[qi][2 * tb][0], (half_t)st[qi][2 * tb][1], (half_t)st[qi][2 * tb][2],
                                     (half_t)st[qi][2 * tb][3], (half_t)st[qi][2 * tb + 1][0], (half_t)st[qi][2 * tb + 1][1],
                                     (half_t)st[qi][2 * tb + 1][2], (half_t)st[qi][2 * tb + 1][3]};
        }
        if (__builtin_amdgcn_ballot_w64(any_moved) != 0ull) {
            // Rare after a row's first tiles.  (This file is compiled with matrix results in vector registers, so
            // the accumulators are ordinary operands here.)
#pragma unroll
            for (int qi = 0; qi < QT; ++qi)
#pragma unroll
                for (int et = 0; et < ETILES; ++et) o_acc[qi][et] = o_acc[qi][et] * alpha[qi];
        }

        // ---- O^T += V_hat^T P^T : A operand = 8 tokens of one dim in P^T's token order (tokens 4 kb .. + 3 of
        // both 16-token tiles of a 32-token block), fetched with two transposing reads one step ahead; the next
        // tile's V rows are dequantized between the steps
        constexpr int VA_AHEAD = 2; // steps the operand reads run ahead
        half8_t va[VA_AHEAD + 1][2]; // [step in the ring][32-token block]
        auto load_va = [&](int et) {
#pragma unroll
            for (int tb = 0; tb < kTile / 32; ++tb) {
                const half_t *src = v_cur + v_lane + tb * 32 * VPITCH + et * 16;
                const short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)src);
                const short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(src + 16 * VPITCH));
                va[et % (VA_AHEAD + 1)][tb] = __builtin_bit_cast(half8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            }
        };
#pragma unroll
        for (int et = 0; et < VA_AHEAD; ++et) load_va(et);
#pragma unroll
        for (int et = 0; et < ETILES; ++et) {
            if (et + VA_AHEAD < ETILES) load_va(et + VA_AHEAD);
#pragma unroll
            for (int tb = 0; tb < kTile / 32; ++tb)
#pragma unroll
                for (int qi = 0; qi < QT; ++qi)
                    o_acc[qi][et] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va[et % (VA_AHEAD + 1)][tb], pt[qi][tb], o_acc[qi][et], 0, 0, 0);
#pragma unroll
            for (int w = 0; w < SV::WPT; ++w)
                if (w * ETILES / SV::WPT == et && v_on) store_word(v_lds[buf ^ 1] + v_dst + 8 * w, vraw[w], vr);
            __builtin_amdgcn_sched_barrier(0);
        }
        ok_cur = ok_next;
        load_tile(min(t0 + 2 * kTile, t_last), ok_next); // past the end: the last tile again, never used
        __syncthreads(); // every wave is done with this buffer and has filled its part of the other
        buf ^= 1;
    }

    // ---- normalise and store: lane column = query row, regs = 4 consecutive row positions of V_hat, which hold
    // dims (0,4,1,5) or (2,6,3,7) of an 8-dim word
#pragma unroll
    for (int qi = 0; qi < QT; ++qi) {
        const float l_tot = xor32_sum(xor16_sum(l_run[qi]));
        if (row_pos[qi] >= p.q_len) continue;
        const int r_w = wave * kRowsWave + qi * 16 + qn;
        const int head = kvh * NREP + r_w % NREP;
        const float inv = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
        uint16_t *dst = p.out + ((q_agent + row_pos[qi]) * p.q_heads + head) * DV;
#pragma unroll
        for (int et = 0; et < ETILES; ++et) {
            uint16_t *d8 = dst + et * 16 + 8 * (kb / 2) + 2 * (kb % 2); // the word of 8 dims, dims 0.. or 2..
            d8[0] = float_to_half_bits(o_acc[qi][et][0] * inv);
            d8[4] = float_to_half_bits(o_acc[qi][et][1] * inv);
            d8[1] = float_to_half_bits(o_acc[qi][et][2] * inv);
            d8[5] = float_to_half_bits(o_acc[qi][et][3] * inv);
        }
    }
}

template <int DK, int DV, int NREP>
hipError_t launch_chunk_t(const AttentionArgs &a, hipStream_t stream)
{
    constexpr int QT = (DK == 128 || DK >= 256) ? 1 : 2; // two tiles where the registers allow it without scratch
    constexpr int kThreads = kRowsWG / (16 * QT) * kWave;
    ChunkParams p;
    p.k_codes = a.k.codes; p.k_scale = a.k.scale; p.k_bias = a.k.bias;
    p.v_codes = a.v.codes; p.v_scale = a.v.scale; p.v_bias = a.v.bias;
    p.q = a.q; p.out = a.out; p.block_table = a.block_table; p.seq_len = a.seq_len;
    p.num_blocks = a.k.num_blocks; p.kv_heads = a.spec.num_kv_heads; p.q_heads = a.spec.num_q_heads;
    p.num_agents = a.num_agents; p.max_blocks = a.max_blocks; p.max_seq_len = a.max_seq_len;
    p.window = a.window; p.q_len = a.q_len;
    p.per_layer_windows = a.layer_window != nullptr;
    for (int i = 0; i < kMaxChunkWindowLayers; ++i)
        p.layer_window[i] = (a.layer_window && i < a.layers_in_call) ? a.layer_window[i] : 0;
    p.layer_begin = a.layer_begin; p.layers_in_call = a.layers_in_call;
    constexpr int QPOS = kRowsWG / NREP;
    p.q_tiles = (a.q_len + QPOS - 1) / QPOS;
    p.score_scale = a.sm_scale * kLog2e;
    const int64_t units = (int64_t)a.layers_in_call * a.num_agents * a.spec.num_kv_heads;
    const int64_t units_padded = (units + kXcds - 1) / kXcds * kXcds;
    const int64_t grid = units_padded * p.q_tiles;
    if (grid <= 0) return hipSuccess;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    if (a.spec.param_format == Q4KV_PARAMS_BF16)
        hipLaunchKernelGGL((chunk_attention_kernel<DK, DV, NREP, QT, true>), dim3((unsigned)grid), dim3(kThreads), 0, stream, p);
    else
        hipLaunchKernelGGL((chunk_attention_kernel<DK, DV, NREP, QT, false>), dim3((unsigned)grid), dim3(kThreads), 0, stream, p);
    return hipGetLastError();
}

template <int DK, int DV>
hipError_t launch_chunk_d(const AttentionArgs &a, int n_rep, hipStream_t stream)
{
    switch (n_rep) {
    case 1: return launch_chunk_t<DK, DV, 1>(a, stream);
    case 2: return launch_chunk_t<DK, DV, 2>(a, stream);
    case 4: return launch_chunk_t<DK, DV, 4>(a, stream);
    case 8: return launch_chunk_t<DK, DV, 8>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

} // namespace

bool chunk_supported(const q4kv_spec &s)
{
    const int n_rep = s.num_q_heads / s.num_kv_heads;
    const bool rep_ok = n_rep == 1 || n_rep == 2 || n_rep == 4 || n_rep == 8;
    const bool square = (s.k_dim == 64 || s.k_dim == 128 || s.k_dim == 256) && s.v_dim == s.k_dim;
    const bool mla_per_head = s.k_dim == 192 && s.v_dim == 128; // decompressed per-head MLA cache (Sec. 3.6)
    return rep_ok && (square || mla_per_head) && !s.v_aliases_k;
}

hipError_t launch_chunk_attention(const AttentionArgs &a, hipStream_t stream)
{
    const int n_rep = a.spec.num_q_heads / a.spec.num_kv_heads;
    switch (a.spec.k_dim) {
    case 64: return launch_chunk_d<64, 64>(a, n_rep, stream);
    case 128: return launch_chunk_d<128, 128>(a, n_rep, stream);
    case 192: return launch_chunk_d<192, 128>(a, n_rep, stream);
    case 256: return launch_chunk_d<256, 256>(a, n_rep, stream);
    default: return hipErrorInvalidValue;
    }
}

} // namespace q4kv

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
//    tile ahead into registers), dequantized ONCE per workgroup into LDS as binary16 and reused by all 128
//    rows: K_hat row-major (dims inside a word stay in the order the nibble masks deliver them; the query
//    operand uses the same order), V_hat transposed so that the PV contraction finds 4 consecutive tokens in
//    8 bytes.
//  * The wave computes S^T = K_hat Q^T (tokens are the M rows), so that the probabilities come out of the
//    matrix core already in the register layout the second GEMM wants for its B operand (P^T); no shuffle
//    or LDS round trip between the GEMMs.  O^T = V_hat^T P^T accumulates in binary32.
//  * Softmax is online, per query row (= per lane column): scores in binary32, log2 domain.
//  * The workgroups of one KV head are adjacent in the launch order of ONE XCD, so the 8 query tiles of a
//    unit stream the same KV tiles through the same L2 at the same time.
#include "q4_device.h"
#include "q4kv_internal.h"

namespace q4kv {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kRowsWG = 128;  // query rows per workgroup
constexpr int kRowsWave = kRowsWG / kWaves;
constexpr int kTile = 64;     // KV tokens per tile
constexpr float kNegBig = -1.0e30f;
constexpr float kLog2e = 1.4426950408889634f;
constexpr int kXcds = 8;

struct ChunkParams {
    const uint32_t *k_codes, *v_codes;
    const uint16_t *k_scale, *k_bias, *v_scale, *v_bias;
    const uint16_t *q;
    uint16_t *out;
    const int32_t *block_table, *seq_len;
    int num_blocks, kv_heads, q_heads, num_agents, max_blocks, max_seq_len, window, q_len;
    int layer_begin, layers_in_call, q_tiles;
    float score_scale;
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

// D = 256 keeps 128 accumulator registers per lane besides the query operand, so it runs one wave per SIMD
// (512 registers); narrower heads fit two.
template <int D, int NREP>
__global__ __launch_bounds__(kThreads, (D >= 256 ? 1 : 2)) void chunk_attention_kernel(ChunkParams p)
{
    constexpr int G = D / kGroup;
    constexpr int KPITCH = D + 8;      // halves per K_hat row in LDS (pad: conflict-free 16-byte operand reads)
    constexpr int VPITCH = kTile + 8;  // halves per V_hat^T row
    constexpr int QPOS = kRowsWG / NREP; // chunk positions per workgroup
    constexpr int KSTEPS = D / 32;     // k-steps of the QK contraction
    constexpr int ETILES = D / 16;     // 16-row tiles of O^T
    constexpr int WORDS = D / 8;       // code words per row
    constexpr int KW_PER_THREAD = kTile * WORDS / kThreads;         // K code words a thread dequantizes per tile
    constexpr int VPAIRS_PER_THREAD = (kTile / 2) * WORDS / kThreads; // (token pair, word column) items per thread
    static_assert(KW_PER_THREAD % 4 == 0 || KW_PER_THREAD == 2, "K tile split");

    __shared__ __attribute__((aligned(16))) half_t k_lds[kTile * KPITCH];
    __shared__ __attribute__((aligned(16))) half_t v_lds[D * VPITCH];

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
    const int pos0 = qt * QPOS;                   // first chunk position of this workgroup
    if (pos0 >= p.q_len) return;
    // chunk position c sees tokens [first(c), vis(c)),  vis(c) = n - (q_len - 1 - c)
    const int vis_last = n - (p.q_len - 1 - min(p.q_len - 1, pos0 + QPOS - 1)); // keys visible to the last row here
    const int vis_first = n - (p.q_len - 1 - pos0);
    int t_begin = 0;
    if (p.window > 0 && vis_first - p.window > 0) t_begin = (vis_first - p.window) & ~(kTile - 1);
    const int t_end = vis_last; // exclusive; may be <= 0 when nothing is visible

    // ---- this lane's query rows: column n = lane % 16 of the two 16-row tiles of its wave
    const int qn = lane % 16, kb = lane / 16;
    int row_pos[2], row_vis[2], row_first[2];
    half8_t qop[2][KSTEPS];
    const int64_t q_agent = ((int64_t)li * p.num_agents + agent) * p.q_len;
#pragma unroll
    for (int qi = 0; qi < 2; ++qi) {
        const int r_w = wave * kRowsWave + qi * 16 + qn;   // row inside the workgroup
        const int c = pos0 + r_w / NREP, head = kvh * NREP + r_w % NREP;
        row_pos[qi] = c;
        const bool live = c < p.q_len;
        row_vis[qi] = live ? n - (p.q_len - 1 - c) : 0;
        row_first[qi] = (p.window > 0 && row_vis[qi] > p.window) ? row_vis[qi] - p.window : 0;
        const uint16_t *src = p.q + ((q_agent + (live ? c : 0)) * p.q_heads + head) * D;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            // dims 32*ks + 8*kb .. +7 in the order the nibble masks emit them: 0,4,1,5,2,6,3,7
            const uint4 raw = *reinterpret_cast<const uint4 *>(src + 32 * ks + 8 * kb);
            const half2_t e01 = bits_to_half2(raw.x), e23 = bits_to_half2(raw.y);
            const half2_t e45 = bits_to_half2(raw.z), e67 = bits_to_half2(raw.w);
            qop[qi][ks] = half8_t{e01.x, e45.x, e01.y, e45.y, e23.x, e67.x, e23.y, e67.y};
        }
    }

    float4_t o_acc[2][ETILES]; // O^T: [q tile][16-dim tile], lane column = query row, regs = dims 4*kb .. 4*kb+3
#pragma unroll
    for (int qi = 0; qi < 2; ++qi)
#pragma unroll
        for (int et = 0; et < ETILES; ++et) o_acc[qi][et] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
    float m_run[2] = {kNegBig, kNegBig}, l_run[2] = {0.0f, 0.0f};

    // ---- KV tile staging: raw Q4 in registers one tile ahead
    const int32_t *table = p.block_table + (int64_t)agent * p.max_blocks;
    uint32_t kraw[KW_PER_THREAD], vraw[2 * VPAIRS_PER_THREAD];
    uint32_t ksb[2], vsb[2 * VPAIRS_PER_THREAD][2]; // scale / bias bits of the rows this thread dequantizes
    // K: thread handles KW_PER_THREAD consecutive words of one token row: token = tid / (WORDS / KW_PER_THREAD)
    constexpr int K_THREADS_PER_ROW = WORDS / KW_PER_THREAD;
    const int k_tok = tid / K_THREADS_PER_ROW, k_w0 = (tid % K_THREADS_PER_ROW) * KW_PER_THREAD;
    const int k_grp = (k_w0 * 8) / kGroup; // the thread's words lie in one group when KW_PER_THREAD <= 8
    static_assert(KW_PER_THREAD <= 8, "a thread's K words must stay inside one quantization group");
    // V: item i of this thread: token pair tp = item / WORDS, word column wc = item % WORDS
    auto tile_row0 = [&](int t0, bool &ok) {
        const int bi = t0 / kBlockTokens;
        const int blk = bi < p.max_blocks ? table[bi] : -1;
        ok = blk >= 0 && blk < p.num_blocks;
        return (((int64_t)layer * p.num_blocks + (ok ? blk : 0)) * p.kv_heads + kvh) * kBlockTokens + (t0 % kBlockTokens);
    };
    auto load_tile = [&](int t0, bool &ok) {
        const int64_t row0 = tile_row0(t0, ok);
        const int64_t krow = row0 + k_tok;
        if constexpr (KW_PER_THREAD % 4 == 0) {
#pragma unroll
            for (int i = 0; i < KW_PER_THREAD / 4; ++i) {
                const uint4 t = *reinterpret_cast<const uint4 *>(p.k_codes + krow * WORDS + k_w0 + 4 * i);
                kraw[4 * i] = t.x; kraw[4 * i + 1] = t.y; kraw[4 * i + 2] = t.z; kraw[4 * i + 3] = t.w;
            }
        } else {
            const uint2 t = *reinterpret_cast<const uint2 *>(p.k_codes + krow * WORDS + k_w0);
            kraw[0] = t.x; kraw[1] = t.y;
        }
        ksb[0] = p.k_scale[krow * G + k_grp];
        ksb[1] = p.k_bias[krow * G + k_grp];
#pragma unroll
        for (int i = 0; i < VPAIRS_PER_THREAD; ++i) {
            const int item = tid + i * kThreads, tp = item / WORDS, wc = item % WORDS;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int64_t vrow = row0 + 2 * tp + h;
                vraw[2 * i + h] = p.v_codes[vrow * WORDS + wc];
                vsb[2 * i + h][0] = p.v_scale[vrow * G + wc / 8];
                vsb[2 * i + h][1] = p.v_bias[vrow * G + wc / 8];
            }
        }
    };
    // dequantize the staged tile into LDS.  Rows of an unreachable block and rows at or past t_end (never
    // visible, possibly never written) become zeros, so that no stale bit pattern can reach an accumulator.
    auto store_tile = [&](int t0, bool ok_tile) {
        {
            const bool ok = ok_tile && (t0 + k_tok < t_end);
            const half_t s = ok ? __builtin_bit_cast(half_t, (uint16_t)ksb[0]) : (half_t)0.0f;
            const half_t b = ok ? __builtin_bit_cast(half_t, (uint16_t)ksb[1]) : (half_t)0.0f;
            const half2_t s2 = {s, s}, b2 = {b, b};
            const half2_t s16 = s2 * half2_t{(half_t)0.0625f, (half_t)0.0625f};
            half_t *dst = k_lds + k_tok * KPITCH + k_w0 * 8;
#pragma unroll
            for (int w = 0; w < KW_PER_THREAD; ++w) {
                const uint32_t word = ok ? kraw[w] : 0u, w8 = word >> 8;
                const half2_t v0 = pk_fma(nibbles_lo(word), s2, b2);    // dims 0, 4
                const half2_t v1 = pk_fma(nibbles_hi16(word), s16, b2); // dims 1, 5
                const half2_t v2 = pk_fma(nibbles_lo(w8), s2, b2);      // dims 2, 6
                const half2_t v3 = pk_fma(nibbles_hi16(w8), s16, b2);   // dims 3, 7
                *reinterpret_cast<uint4 *>(dst + 8 * w) =
                    make_uint4(half2_to_bits(v0), half2_to_bits(v1), half2_to_bits(v2), half2_to_bits(v3));
            }
        }
#pragma unroll
        for (int i = 0; i < VPAIRS_PER_THREAD; ++i) {
            const int item = tid + i * kThreads, tp = item / WORDS, wc = item % WORDS;
            const bool oka = ok_tile && (t0 + 2 * tp < t_end), okb = ok_tile && (t0 + 2 * tp + 1 < t_end);
            const half_t sa = oka ? __builtin_bit_cast(half_t, (uint16_t)vsb[2 * i][0]) : (half_t)0.0f;
            const half_t sb = okb ? __builtin_bit_cast(half_t, (uint16_t)vsb[2 * i + 1][0]) : (half_t)0.0f;
            const half_t ba = oka ? __builtin_bit_cast(half_t, (uint16_t)vsb[2 * i][1]) : (half_t)0.0f;
            const half_t bb = okb ? __builtin_bit_cast(half_t, (uint16_t)vsb[2 * i + 1][1]) : (half_t)0.0f;
            const half2_t s2 = {sa, sb}, b2 = {ba, bb};
            const half2_t s16 = s2 * half2_t{(half_t)0.0625f, (half_t)0.0625f};
            const uint32_t wa = vraw[2 * i], wb = vraw[2 * i + 1]; // codes are nibbles: with scale = bias = 0 they vanish
#pragma unroll
            for (int by = 0; by < 4; ++by) {
                // byte `by` of both tokens: dims 2*by (low nibble) and 2*by + 1 (high nibble)
                const uint32_t pair = __builtin_amdgcn_perm(wb, wa, 0x0C040C00u + by * 0x00010001u);
                const half2_t lo = pk_fma(nibbles_lo(pair), s2, b2);
                const half2_t hi = pk_fma(nibbles_hi16(pair), s16, b2);
                const int e = wc * 8 + 2 * by;
                *reinterpret_cast<uint32_t *>(v_lds + e * VPITCH + 2 * tp) = half2_to_bits(lo);
                *reinterpret_cast<uint32_t *>(v_lds + (e + 1) * VPITCH + 2 * tp) = half2_to_bits(hi);
            }
        }
    };

    bool ok_next = false;
    if (t_begin < t_end) load_tile(t_begin, ok_next);
    for (int t0 = t_begin; t0 < t_end; t0 += kTile) {
        __syncthreads(); // every wave is done reading the previous tile
        store_tile(t0, ok_next);
        const bool ok_cur = ok_next;
        if (t0 + kTile < t_end) load_tile(t0 + kTile, ok_next);
        __syncthreads();

        // ---- S^T = K_hat Q^T : [64 tokens][32 query rows] per wave, binary32
        float4_t st[2][kTile / 16]; // [q tile][token tile]: lane column = query row, regs = tokens 4*kb .. 4*kb+3
#pragma unroll
        for (int qi = 0; qi < 2; ++qi)
#pragma unroll
            for (int tt = 0; tt < kTile / 16; ++tt) st[qi][tt] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
            for (int tt = 0; tt < kTile / 16; ++tt) {
                const half8_t ka = *reinterpret_cast<const half8_t *>(k_lds + (tt * 16 + qn) * KPITCH + 32 * ks + 8 * kb);
#pragma unroll
                for (int qi = 0; qi < 2; ++qi)
                    st[qi][tt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka, qop[qi][ks], st[qi][tt], 0, 0, 0);
            }

        // ---- online softmax per query row (lane column), then P^T in binary16 as the next B operand
        half8_t pt[2][kTile / 32]; // [q tile][32-token block]: tokens 4*kb..+3 of both 16-token tiles of the block
#pragma unroll
        for (int qi = 0; qi < 2; ++qi) {
            float mx = kNegBig;
#pragma unroll
            for (int tt = 0; tt < kTile / 16; ++tt)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int t = t0 + tt * 16 + 4 * kb + e;
                    const bool vis = ok_cur && t < row_vis[qi] && t >= row_first[qi];
                    const float z = vis ? st[qi][tt][e] * p.score_scale : kNegBig;
                    st[qi][tt][e] = z;
                    mx = fmaxf(mx, z);
                }
            // the row's tokens live in the 4 lanes qn, qn+16, qn+32, qn+48
            mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
            mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
            const float m_new = fmaxf(m_run[qi], mx);
            const float alpha = __builtin_amdgcn_exp2f(m_run[qi] - m_new);
            m_run[qi] = m_new;
            float sum = 0.0f;
#pragma unroll
            for (int tt = 0; tt < kTile / 16; ++tt)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float pr = st[qi][tt][e] > 0.5f * kNegBig ? __builtin_amdgcn_exp2f(st[qi][tt][e] - m_new) : 0.0f;
                    st[qi][tt][e] = pr;
                    sum += pr;
                }
            sum += __shfl_xor(sum, 16, kWave);
            sum += __shfl_xor(sum, 32, kWave);
            l_run[qi] = fmaf(l_run[qi], alpha, sum);
#pragma unroll
            for (int et = 0; et < ETILES; ++et) o_acc[qi][et] *= alpha;
#pragma unroll
            for (int tb = 0; tb < kTile / 32; ++tb)
                pt[qi][tb] = half8_t{(half_t)st[qi][2 * tb][0], (half_t)st[qi][2 * tb][1], (half_t)st[qi][2 * tb][2],
                                     (half_t)st[qi][2 * tb][3], (half_t)st[qi][2 * tb + 1][0], (half_t)st[qi][2 * tb + 1][1],
                                     (half_t)st[qi][2 * tb + 1][2], (half_t)st[qi][2 * tb + 1][3]};
        }

        // ---- O^T += V_hat^T P^T : A operand = 8 tokens of one dim in P^T's token order
#pragma unroll
        for (int et = 0; et < ETILES; ++et)
#pragma unroll
            for (int tb = 0; tb < kTile / 32; ++tb) {
                const half_t *vrow = v_lds + (et * 16 + qn) * VPITCH + tb * 32 + 4 * kb;
                const uint2 lo = *reinterpret_cast<const uint2 *>(vrow);
                const uint2 hi = *reinterpret_cast<const uint2 *>(vrow + 16);
                const half8_t va = __builtin_bit_cast(half8_t, make_uint4(lo.x, lo.y, hi.x, hi.y));
#pragma unroll
                for (int qi = 0; qi < 2; ++qi)
                    o_acc[qi][et] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va, pt[qi][tb], o_acc[qi][et], 0, 0, 0);
            }
    }

    // ---- normalise and store: lane column = query row, regs = 4 consecutive dims
#pragma unroll
    for (int qi = 0; qi < 2; ++qi) {
        if (row_pos[qi] >= p.q_len) continue;
        const int r_w = wave * kRowsWave + qi * 16 + qn;
        const int head = kvh * NREP + r_w % NREP;
        const float inv = l_run[qi] > 0.0f ? 1.0f / l_run[qi] : 0.0f;
        uint16_t *dst = p.out + ((q_agent + row_pos[qi]) * p.q_heads + head) * D;
#pragma unroll
        for (int et = 0; et < ETILES; ++et) {
            const uint32_t a = (uint32_t)float_to_half_bits(o_acc[qi][et][0] * inv) |
                               ((uint32_t)float_to_half_bits(o_acc[qi][et][1] * inv) << 16);
            const uint32_t b = (uint32_t)float_to_half_bits(o_acc[qi][et][2] * inv) |
                               ((uint32_t)float_to_half_bits(o_acc[qi][et][3] * inv) << 16);
            *reinterpret_cast<uint2 *>(dst + et * 16 + 4 * kb) = make_uint2(a, b);
        }
    }
}

template <int D, int NREP>
hipError_t launch_chunk_t(const AttentionArgs &a, hipStream_t stream)
{
    ChunkParams p;
    p.k_codes = a.k.codes; p.k_scale = a.k.scale; p.k_bias = a.k.bias;
    p.v_codes = a.v.codes; p.v_scale = a.v.scale; p.v_bias = a.v.bias;
    p.q = a.q; p.out = a.out; p.block_table = a.block_table; p.seq_len = a.seq_len;
    p.num_blocks = a.k.num_blocks; p.kv_heads = a.spec.num_kv_heads; p.q_heads = a.spec.num_q_heads;
    p.num_agents = a.num_agents; p.max_blocks = a.max_blocks; p.max_seq_len = a.max_seq_len;
    p.window = a.window; p.q_len = a.q_len;
    p.layer_begin = a.layer_begin; p.layers_in_call = a.layers_in_call;
    constexpr int QPOS = kRowsWG / NREP;
    p.q_tiles = (a.q_len + QPOS - 1) / QPOS;
    p.score_scale = a.sm_scale * kLog2e;
    const int64_t units = (int64_t)a.layers_in_call * a.num_agents * a.spec.num_kv_heads;
    const int64_t units_padded = (units + kXcds - 1) / kXcds * kXcds;
    const int64_t grid = units_padded * p.q_tiles;
    if (grid <= 0) return hipSuccess;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((chunk_attention_kernel<D, NREP>), dim3((unsigned)grid), dim3(kThreads), 0, stream, p);
    return hipGetLastError();
}

template <int D>
hipError_t launch_chunk_d(const AttentionArgs &a, int n_rep, hipStream_t stream)
{
    switch (n_rep) {
    case 1: return launch_chunk_t<D, 1>(a, stream);
    case 2: return launch_chunk_t<D, 2>(a, stream);
    case 4: return launch_chunk_t<D, 4>(a, stream);
    case 8: return launch_chunk_t<D, 8>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

} // namespace

bool chunk_supported(const q4kv_spec &s)
{
    const int n_rep = s.num_q_heads / s.num_kv_heads;
    const bool rep_ok = n_rep == 1 || n_rep == 2 || n_rep == 4 || n_rep == 8;
    const bool dims_ok = (s.k_dim == 64 || s.k_dim == 128 || s.k_dim == 256) && s.v_dim == s.k_dim && !s.v_aliases_k;
    return rep_ok && dims_ok;
}

hipError_t launch_chunk_attention(const AttentionArgs &a, hipStream_t stream)
{
    const int n_rep = a.spec.num_q_heads / a.spec.num_kv_heads;
    switch (a.spec.k_dim) {
    case 64: return launch_chunk_d<64>(a, n_rep, stream);
    case 128: return launch_chunk_d<128>(a, n_rep, stream);
    case 256: return launch_chunk_d<256>(a, n_rep, stream);
    default: return hipErrorInvalidValue;
    }
}

} // namespace q4kv

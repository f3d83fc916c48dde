// "Stream-K over tokens": the work decomposition shared by the decode kernels.
//
// All (layer in call, KV head, agent) units are cut into 64-token tiles and numbered consecutively (layer-major,
// then KV head, then agent); a fixed launch of waves owns equal contiguous tile ranges.  plan_kernel turns
// seq_len[] into per-agent tile prefix sums on the device; a Cursor walks a wave's range with scalar arithmetic,
// touching memory only where a unit or a 256-token block begins.  A unit that lies inside one wave's range is
// finished by that wave.  Waves that meet in a unit each leave a partial result (un-normalised sums, running
// maximum, denominator) in the unit's slot for them and count themselves in on the unit's arrival counter; the
// one that arrives last merges all slots, in slot order whoever it is, so results do not depend on timing.
#pragma once
#include "q4_device.h"

namespace q4kv {

// Plan written by plan_kernel into the workspace (int32).  Layers with the same sliding window form a class; the
// per-agent arrays exist once per class.  A = agents, L = layers in the call, C <= L classes.
//   [0] N = total tiles   [1] per = tiles per wave   [2] C   [3] L
//   LT[L + 1]    tiles before layer li of the call (all KV heads and agents), LT[L] = N
//   cls[L]       class of layer li
//   C_max = L class blocks of 2A + 2 ints:  window (0 = global), tpre[A + 1] (tile prefix sum over agents, tpre[A] =
//                tiles of one (layer, KV head) of the class), tstart[A] (first visible token rounded down to a tile)
//   nlen[A]      seq_len clamped to [0, max_seq_len]
//   [4] E = agents without a visible token; empty[A]: their indices (first E entries) -- no wave visits their
//                units, their output rows are zeroed by the attention launch before anything else
//   [5] signature of the arguments the plan was made for (a planned call checks it before it trusts the plan)
constexpr int kPlanHeader = 6;
constexpr int kMaxWindowLayers = 128; // layers per call when every layer brings its own window

struct PlanView {
    const int32_t *plan;
    int A, L;
    __device__ __host__ __forceinline__ static size_t ints(int A, int L)
    {
        return (size_t)kPlanHeader + 2 * (size_t)L + 1 + (size_t)L * (2 * (size_t)A + 2) + 2 * (size_t)A;
    }
    __device__ __forceinline__ int class_stride() const { return 2 * A + 2; }
    __device__ __forceinline__ int lt_off() const { return kPlanHeader; }
    __device__ __forceinline__ int cls_off() const { return kPlanHeader + L + 1; }
    __device__ __forceinline__ int class_off(int c) const { return kPlanHeader + 2 * L + 1 + c * class_stride(); }
    __device__ __forceinline__ int nlen_off() const { return class_off(L); }
    __device__ __forceinline__ int empty_off() const { return nlen_off() + A; }
    __device__ __forceinline__ int layer_class_off(int li) const { return class_off(plan[cls_off() + li]); }
    // inside a class block
    __device__ __forceinline__ int window(int cb) const { return plan[cb]; }
    __device__ __forceinline__ const int32_t *tpre(int cb) const { return plan + cb + 1; }
    __device__ __forceinline__ const int32_t *tstart(int cb) const { return plan + cb + 2 + A; }
    __device__ __forceinline__ int tiles_per_head(int cb) const { return plan[cb + 1 + A]; }
};

struct StreamParams {
    const int32_t *plan;
    const int32_t *block_table;
    int num_agents, max_blocks, kv_heads, num_blocks, layer_begin, layers;
    int plan_signature; // what plan[5] must hold
};

// Position of a wave in the tile stream; every field is wave-uniform and lives in scalar registers.
// Everything that needs a division, a wide multiply or a memory lookup is refreshed only where it can
// change: per unit (unit_row, first) or per 256-token block (row of the block, reachable).
// Flag is the type of `reachable`: a kernel picks the one its register allocation fares better with.
template <typename Flag>
struct CursorT {
    int li, kvh, agent;  // unit: layer in call, KV head, agent
    int cb;              // plan offset of the class block of layer li
    int j, tiles;        // tile inside the unit, tiles of the unit
    int t0;              // first token of the tile
    int n, first;        // visible tokens of the agent, first visible token (sliding window)
    int64_t unit_row;    // pool row of (layer, block 0, kv head, slot 0)
    int64_t row;         // pool row of the tile's first token
    int fallback_blk;    // where the loads of a tile go whose block id is outside the pool: the agent's first block
    Flag reachable;      // the tile's block id is inside the pool
    int blk_ahead;       // table entry of the block after the tile's (-1 past the table): fetched one block early so
                         // that the lookup is never on the path of the next tile's loads
};
typedef CursorT<bool> Cursor;

struct TileStream {
    StreamParams sp;
    PlanView pv;
    int per, N;
    bool valid; // the plan in the workspace was made for this call's arguments

    __device__ __forceinline__ explicit TileStream(const StreamParams &s) : sp(s)
    {
        pv.plan = s.plan;
        pv.A = s.num_agents;
        pv.L = s.layers;
        N = s.plan[0];
        per = s.plan[1];
        // A plan made for other arguments (possible only when the caller reuses a prepared workspace against the
        // rules) is not walked: the launch then does nothing.
        valid = s.plan[5] == s.plan_signature;
        if (!valid) N = 0;
    }

    template <typename C>
    __device__ __forceinline__ void place_block(C &c, int blk) const
    {
        c.reachable = blk >= 0 && blk < sp.num_blocks;
        // the (unconditional) loads of a tile whose block id is outside the pool go to the agent's own first block
        // (to block 0 only if that id is outside the pool as well); everything they bring is masked
        c.row = c.unit_row + (int64_t)(c.reachable ? blk : c.fallback_blk) * (sp.kv_heads * kBlockTokens) +
                (c.t0 % kBlockTokens);
    }

    template <typename C>
    __device__ __forceinline__ void enter_block(C &c) const
    {
        const int bi = c.t0 / kBlockTokens;
        const int32_t *row = sp.block_table + (long long)c.agent * sp.max_blocks;
        const int blk = bi < sp.max_blocks ? row[bi] : -1;
        c.blk_ahead = bi + 1 < sp.max_blocks ? row[bi + 1] : -1;
        const int own0 = row[0];
        c.fallback_blk = own0 >= 0 && own0 < sp.num_blocks ? own0 : 0;
        place_block(c, blk);
    }

    // the same when the tile stream walks from one block of an agent into the next
    template <typename C>
    __device__ __forceinline__ void next_block(C &c) const
    {
        const int bi = c.t0 / kBlockTokens;
        const int blk = c.blk_ahead;
        c.blk_ahead = bi + 1 < sp.max_blocks ? sp.block_table[(long long)c.agent * sp.max_blocks + bi + 1] : -1;
        place_block(c, blk);
    }

    template <typename C>
    __device__ __forceinline__ void enter_unit(C &c) const
    {
        const int32_t *tpre = pv.tpre(c.cb);
        const int window = pv.window(c.cb);
        c.tiles = tpre[c.agent + 1] - tpre[c.agent];
        c.n = pv.plan[pv.nlen_off() + c.agent];
        c.first = (window > 0 && c.n > window) ? c.n - window : 0;
        c.unit_row = (((int64_t)(sp.layer_begin + c.li) * sp.num_blocks) * sp.kv_heads + c.kvh) * kBlockTokens;
    }

    // to the next tile of the stream (meaningful while it stays below the wave's last tile)
    template <typename C>
    __device__ __forceinline__ void step(C &c) const
    {
        if (++c.j < c.tiles) {
            c.t0 += kWave;
            if (c.t0 % kBlockTokens == 0) next_block(c); else c.row += kWave;
            return;
        }
        const int32_t *tpre = pv.tpre(c.cb);
        do {
            if (++c.agent >= sp.num_agents) {
                c.agent = 0;
                if (++c.kvh >= sp.kv_heads) {
                    c.kvh = 0;
                    ++c.li;
                    c.cb = pv.layer_class_off(c.li);
                    tpre = pv.tpre(c.cb);
                }
            }
        } while (tpre[c.agent + 1] == tpre[c.agent]);
        c.j = 0;
        c.t0 = pv.tstart(c.cb)[c.agent];
        enter_unit(c);
        enter_block(c);
    }

    // to the next unit of the stream that has tiles (li, kvh, agent and cb only)
    template <typename C>
    __device__ __forceinline__ void next_unit(C &c) const
    {
        const int32_t *tpre = pv.tpre(c.cb);
        do {
            if (++c.agent >= sp.num_agents) {
                c.agent = 0;
                if (++c.kvh >= sp.kv_heads) {
                    c.kvh = 0;
                    ++c.li;
                    c.cb = pv.layer_class_off(c.li);
                    tpre = pv.tpre(c.cb);
                }
            }
        } while (tpre[c.agent + 1] == tpre[c.agent]);
    }

    // `stride` tiles ahead (stride <= 4, the target stays below the stream's end): the walk of one wave of a
    // workgroup whose waves take the tiles of the workgroup's range in turn.  Inside a unit with stride 4 the target
    // is the same slot range of the next 256-token block.
    template <typename C>
    __device__ __forceinline__ void advance(C &c, int stride) const
    {
        c.j += stride;
        if (__builtin_expect(c.j < c.tiles, 1)) {
            const int old_block = c.t0 / kBlockTokens;
            c.t0 += stride * kWave;
            if (c.t0 / kBlockTokens != old_block) next_block(c); else c.row += stride * kWave;
            return;
        }
        int r = c.j - c.tiles; // tiles to go beyond the end of this unit
        for (;;) {
            next_unit(c);
            const int32_t *tpre = pv.tpre(c.cb);
            const int tiles = tpre[c.agent + 1] - tpre[c.agent];
            if (r < tiles) break;
            r -= tiles;
        }
        c.j = r;
        c.t0 = pv.tstart(c.cb)[c.agent] + r * kWave;
        enter_unit(c);
        enter_block(c);
    }

    // where tile x lies: layer by binary search over the layer prefix, agent by binary search over the class's
    // per-agent prefix
    template <typename C = Cursor>
    __device__ __forceinline__ C locate(int x) const
    {
        C c;
        const int32_t *LT = pv.plan + pv.lt_off();
        int lo = 0, hi = sp.layers - 1; // largest li with LT[li] <= x (layers without tiles are stepped over)
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (LT[mid] <= x) lo = mid; else hi = mid - 1;
        }
        c.li = lo;
        c.cb = pv.layer_class_off(lo);
        const int TT = pv.tiles_per_head(c.cb);
        const int32_t *tpre = pv.tpre(c.cb);
        const int in_layer = x - LT[lo];
        c.kvh = in_layer / TT;
        const int r = in_layer - c.kvh * TT;
        lo = 0, hi = sp.num_agents - 1; // largest a with tpre[a] <= r and at least one tile
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (tpre[mid] <= r) lo = mid; else hi = mid - 1;
        }
        c.agent = lo;
        c.j = r - tpre[lo];
        c.t0 = pv.tstart(c.cb)[lo] + c.j * kWave;
        enter_unit(c);
        enter_block(c);
        return c;
    }

    // index of the partial record that wave `gw` writes for the unit the cursor is in, and how many waves meet in
    // that unit (= records to merge)
    template <typename C>
    __device__ __forceinline__ void slot_of(const C &c, int gw, int &slot, int &slots) const
    {
        const int unit_first_tile =
            pv.plan[pv.lt_off() + c.li] + c.kvh * pv.tiles_per_head(c.cb) + pv.tpre(c.cb)[c.agent];
        const int first_wave = unit_first_tile / per;
        slot = gw - first_wave;
        slots = (unit_first_tile + c.tiles - 1) / per - first_wave + 1;
    }
};

// The part of one unit that lies inside a worker's tile range [x0, x1): what the waves of a workgroup finish
// together before any of them goes on.
struct Segment {
    int li, kvh, agent, cb;
    int unit_first, tiles; // stream index of the unit's first tile, tiles of the unit
    int begin, end;        // stream indices of the segment, begin < end <= x1

    // the segment that starts at the worker's first tile (c = locate(x0))
    template <typename C>
    __device__ __forceinline__ void start(const C &c, int x0, int x1)
    {
        li = c.li, kvh = c.kvh, agent = c.agent, cb = c.cb;
        unit_first = x0 - c.j;
        tiles = c.tiles;
        begin = x0;
        end = unit_first + tiles < x1 ? unit_first + tiles : x1;
    }
    // the next one (meaningful while end < x1)
    __device__ __forceinline__ void next(const TileStream &ts, int x1)
    {
        ts.next_unit(*this);
        const int32_t *tpre = ts.pv.tpre(cb);
        unit_first = begin = end;
        tiles = tpre[agent + 1] - tpre[agent];
        end = unit_first + tiles < x1 ? unit_first + tiles : x1;
    }
    // the record this worker writes for the unit, and how many workers meet in it
    __device__ __forceinline__ void slot_of(int per, int worker, int &slot, int &slots) const
    {
        const int first_worker = unit_first / per;
        slot = worker - first_worker;
        slots = (unit_first + tiles - 1) / per - first_worker + 1;
    }
    // the same when every worker's range of `per` tiles (a multiple of 4) is cut into four sub-ranges of per / 4
    // tiles with a record each: sub-range i of worker w has the number 4 w + i
    __device__ __forceinline__ void slot_of_quarter(int per, int number, int &slot, int &slots) const
    {
        const int q = per / 4, last_tile = unit_first + tiles - 1;
        const int first = 4 * (unit_first / per) + (unit_first % per) / q;
        slot = number - first;
        slots = 4 * (last_tile / per) + (last_tile % per) / q - first + 1;
    }
};

// ---------------------------------------------------------------------------------------------- merging a unit

constexpr float kMergeNegBig = -1.0e30f;

struct MergeParams {
    float *part_acc;    // [query-head unit][max_slots][DV] un-normalised sums
    float *part_ml;     // [query-head unit][max_slots][2]  running maximum (log2 units), denominator
    int32_t *arrivals;  // [layer in call][kv head][agent], zeroed by the plan kernel
    uint16_t *out;      // [query-head unit][DV] binary16
    int max_slots;
};

// Rows of agents that have no visible token: zeros.  Every wave of the launch takes its share before it looks
// for tiles (waves without tiles included); a call without such agents pays one scalar load.
template <int DV>
__device__ __forceinline__ void zero_empty_units(const PlanView &pv, uint16_t *out, int q_heads, int gw, int total_waves,
                                                 int lane)
{
    const int E = pv.plan[4];
    if (E == 0) return;
    const int32_t *empty = pv.plan + pv.empty_off();
    const int rows = pv.L * E * q_heads;
    for (int i = gw; i < rows; i += total_waves) {
        const int h = i % q_heads, ea = (i / q_heads) % E, li = i / (q_heads * E);
        uint16_t *row = out + (((int64_t)li * pv.A + empty[ea]) * q_heads + h) * DV;
        for (int e = 2 * lane; e < DV; e += 2 * kWave) *reinterpret_cast<uint32_t *>(row + e) = 0u;
    }
}

// Partial records are exchanged between waves on different compute dies, whose second-level caches are not kept
// coherent with each other inside a kernel.  A device-wide release / acquire fence pair would do (write the whole
// cache back, drop it on the other side), but costs tens of microseconds per fence on this chip (measured: the
// 48-layer decode call went from 0.76 to 0.93 ms).  Instead every access to a record is itself a device-scope access:
// such a store goes through to memory, such a load does not take a cached copy, and nothing else has to move.
__device__ __forceinline__ void record_store(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float record_load(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Counts this wave in on a unit whose partial record it has just written with record_store; true for the wave that
// arrives last, which may then read every record of the unit with record_load.  Lane 0 counts only after the
// record stores of all lanes have been acknowledged (they are issued by the same wave, in order, before the wait).
__device__ __forceinline__ bool arrive_last(int32_t *counter, int slots, int lane)
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront"); // the compiler keeps the record stores above this point
    __builtin_amdgcn_s_waitcnt(0x0F70);                    // vmcnt(0): they have reached memory
    int old = 0;
    if (lane == 0) old = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    old = __builtin_amdgcn_readfirstlane(old);
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront"); // and the record loads below it
    return old == slots - 1;
}

// One output value of one query head from the `slots` partial records of its unit: element e of every record,
// binary32, slot order.  All lanes of the wave work on the same head (ml: its [slots][2] maxima and denominators;
// acc: its [slots][DV] sums).  Records whose denominator is zero (every token masked) are skipped; a head with
// nothing at all yields zero.  A record load is a trip to memory, so the loads of up to 16 records are issued
// together with their maxima and denominators and only then used: units of up to 16 records cost one round trip.
template <int DV>
__device__ __forceinline__ float merge_element(const float *acc, const float *ml, int slots, int e, int lane)
{
    constexpr int B = 16;
    float o = 0.0f, m_ref = kMergeNegBig, denom = 0.0f;
    for (int s0 = 0; s0 < slots; s0 += B) {
        const int count = slots - s0 < B ? slots - s0 : B;
        const int s = s0 + (lane < count ? lane : count - 1);
        const float m_s = record_load(ml + 2 * s);
        const float l_s = lane < count ? record_load(ml + 2 * s + 1) : 0.0f;
        float v[B];
#pragma unroll
        for (int j = 0; j < B; ++j) {
            const int k = j < count ? j : count - 1; // repeats of the batch's last record are not used
            v[j] = record_load(acc + (int64_t)(s0 + k) * DV + e);
        }
        const float m_new = fmaxf(m_ref, wave_max(l_s > 0.0f ? m_s : kMergeNegBig));
        const float keep = __builtin_amdgcn_exp2f(m_ref - m_new); // 1 when the reference stays
        m_ref = m_new;
        denom *= keep;
        o *= keep;
        const float w = l_s > 0.0f ? __builtin_amdgcn_exp2f(m_s - m_ref) : 0.0f;
        const float wl = w * l_s;
#pragma unroll
        for (int j = 0; j < B; ++j) {
            if (j < count) { // wave-uniform
                const float wk = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, w), j));
                denom += __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wl), j));
                o = fmaf(wk, v[j], o);
            }
        }
    }
    return denom > 0.0f ? o / denom : 0.0f;
}

// The same for a whole output row of one query head by one wave (a lane owns elements lane, lane + 64, ...): the
// loads of 16 / (DV / 64) records at a time, all chunks of a record together, so that a unit of a few records costs a
// single round trip per head.  Writes the normalised row as binary16.
template <int DV>
__device__ __forceinline__ void merge_row(const float *acc, const float *ml, int slots, uint16_t *out_row, int lane)
{
    constexpr int CH = DV / kWave; // 1, 2, 4 or 8 elements per lane
    static_assert(CH == 1 || CH == 2 || CH == 4 || CH == 8, "row width");
    constexpr int B = CH >= 8 ? 2 : 16 / CH;
    float o[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) o[c] = 0.0f;
    float m_ref = kMergeNegBig, denom = 0.0f;
    for (int s0 = 0; s0 < slots; s0 += B) {
        const int count = slots - s0 < B ? slots - s0 : B;
        const int s = s0 + (lane < count ? lane : count - 1);
        const float m_s = record_load(ml + 2 * s);
        const float l_s = lane < count ? record_load(ml + 2 * s + 1) : 0.0f;
        float v[B][CH];
#pragma unroll
        for (int j = 0; j < B; ++j) {
            const int k = j < count ? j : count - 1; // repeats of the batch's last record are not used
#pragma unroll
            for (int c = 0; c < CH; ++c) v[j][c] = record_load(acc + (int64_t)(s0 + k) * DV + c * kWave + lane);
        }
        const float m_new = fmaxf(m_ref, wave_max(l_s > 0.0f ? m_s : kMergeNegBig));
        const float keep = __builtin_amdgcn_exp2f(m_ref - m_new); // 1 when the reference stays
        m_ref = m_new;
        denom *= keep;
#pragma unroll
        for (int c = 0; c < CH; ++c) o[c] *= keep;
        const float w = l_s > 0.0f ? __builtin_amdgcn_exp2f(m_s - m_ref) : 0.0f;
        const float wl = w * l_s;
#pragma unroll
        for (int j = 0; j < B; ++j) {
            if (j < count) { // wave-uniform
                const float wk = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, w), j));
                denom += __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wl), j));
#pragma unroll
                for (int c = 0; c < CH; ++c) o[c] = fmaf(wk, v[j][c], o[c]);
            }
        }
    }
    const float inv = denom > 0.0f ? 1.0f / denom : 0.0f;
#pragma unroll
    for (int c = 0; c < CH; ++c) out_row[c * kWave + lane] = float_to_half_bits(o[c] * inv);
}

} // namespace q4kv

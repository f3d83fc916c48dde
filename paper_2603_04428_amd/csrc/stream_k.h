// "Stream-K over tokens": the work decomposition shared by the decode kernels.
//
// All (layer in call, KV head, agent) units are cut into 64-token tiles and numbered consecutively (layer-major,
// then KV head, then agent); a fixed launch of waves owns equal contiguous tile ranges.  plan_kernel turns
// seq_len[] into per-agent tile prefix sums on the device; a Cursor walks a wave's range with scalar arithmetic,
// touching memory only where a unit or a 256-token block begins; combine_kernel merges the partial results
// that the waves meeting in one unit leave behind.
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
constexpr int kPlanHeader = 4;
constexpr int kMaxWindowLayers = 128; // layers per call when every layer brings its own window

struct PlanView {
    const int32_t *plan;
    int A, L;
    __device__ __host__ __forceinline__ static size_t ints(int A, int L)
    {
        return (size_t)kPlanHeader + 2 * (size_t)L + 1 + (size_t)L * (2 * (size_t)A + 2) + (size_t)A;
    }
    __device__ __forceinline__ int class_stride() const { return 2 * A + 2; }
    __device__ __forceinline__ int lt_off() const { return kPlanHeader; }
    __device__ __forceinline__ int cls_off() const { return kPlanHeader + L + 1; }
    __device__ __forceinline__ int class_off(int c) const { return kPlanHeader + 2 * L + 1 + c * class_stride(); }
    __device__ __forceinline__ int nlen_off() const { return class_off(L); }
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
    Flag reachable;      // the tile's block id is inside the pool
    int blk_ahead;       // table entry of the block after the tile's (-1 past the table): fetched one block early so
                         // that the lookup is never on the path of the next tile's loads
};
typedef CursorT<bool> Cursor;

struct TileStream {
    StreamParams sp;
    PlanView pv;
    int per, N;

    __device__ __forceinline__ explicit TileStream(const StreamParams &s) : sp(s)
    {
        pv.plan = s.plan;
        pv.A = s.num_agents;
        pv.L = s.layers;
        N = s.plan[0];
        per = s.plan[1];
    }

    template <typename C>
    __device__ __forceinline__ void place_block(C &c, int blk) const
    {
        c.reachable = blk >= 0 && blk < sp.num_blocks;
        // rows of an unreachable block fall back to block 0 and are fully masked
        c.row = c.unit_row + (int64_t)(c.reachable ? blk : 0) * (sp.kv_heads * kBlockTokens) + (c.t0 % kBlockTokens);
    }

    template <typename C>
    __device__ __forceinline__ void enter_block(C &c) const
    {
        const int bi = c.t0 / kBlockTokens;
        const int32_t *row = sp.block_table + (long long)c.agent * sp.max_blocks;
        const int blk = bi < sp.max_blocks ? row[bi] : -1;
        c.blk_ahead = bi + 1 < sp.max_blocks ? row[bi + 1] : -1;
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

    // index of the partial record that wave `gw` writes for the unit the cursor is in
    template <typename C>
    __device__ __forceinline__ int slot_of(const C &c, int gw) const
    {
        const int unit_first_tile =
            pv.plan[pv.lt_off() + c.li] + c.kvh * pv.tiles_per_head(c.cb) + pv.tpre(c.cb)[c.agent];
        return gw - unit_first_tile / per;
    }
};

} // namespace q4kv

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

// Plan written by plan_kernel into the workspace (int32):
//   [0] TT = tiles of all agents of one (layer, KV head)   [1] per = tiles per wave   [2] N = total tiles
//   [4 .. 4+A]        tpre[a]   tile prefix sum over agents (tpre[A] == TT)
//   [.. +A]           tstart[a] first visible token rounded down to a tile boundary
//   [.. +A]           nlen[a]   seq_len clamped to [0, max_seq_len]
constexpr int kPlanHeader = 4;

struct StreamParams {
    const int32_t *plan;
    const int32_t *block_table;
    int num_agents, max_blocks, kv_heads, num_blocks, layer_begin, window;
};

// Position of a wave in the tile stream; every field is wave-uniform and lives in scalar registers.
// Everything that needs a division, a wide multiply or a memory lookup is refreshed only where it can
// change: per unit (unit_row, first) or per 256-token block (row of the block, reachable).
// Flag is the type of `reachable`: a kernel picks the one its register allocation fares better with.
template <typename Flag>
struct CursorT {
    int li, kvh, agent;  // unit: layer in call, KV head, agent
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
    const int32_t *tpre, *tstart, *nlen;
    int TT, per, N;

    __device__ __forceinline__ explicit TileStream(const StreamParams &s) : sp(s)
    {
        TT = s.plan[0];
        per = s.plan[1];
        N = s.plan[2];
        tpre = s.plan + kPlanHeader;
        tstart = tpre + s.num_agents + 1;
        nlen = tstart + s.num_agents;
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
        c.tiles = tpre[c.agent + 1] - tpre[c.agent];
        c.n = nlen[c.agent];
        c.first = (sp.window > 0 && c.n > sp.window) ? c.n - sp.window : 0;
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
        do {
            if (++c.agent >= sp.num_agents) {
                c.agent = 0;
                if (++c.kvh >= sp.kv_heads) {
                    c.kvh = 0;
                    ++c.li;
                }
            }
        } while (tpre[c.agent + 1] == tpre[c.agent]);
        c.j = 0;
        c.t0 = tstart[c.agent];
        enter_unit(c);
        enter_block(c);
    }

    // where tile x lies: unit by binary search over the agents' tile prefix sums
    template <typename C = Cursor>
    __device__ __forceinline__ C locate(int x) const
    {
        C c;
        const int lu = x / TT, r = x - lu * TT;
        int lo = 0, hi = sp.num_agents - 1; // largest a with tpre[a] <= r and at least one tile
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (tpre[mid] <= r) lo = mid; else hi = mid - 1;
        }
        c.li = lu / sp.kv_heads;
        c.kvh = lu % sp.kv_heads;
        c.agent = lo;
        c.j = r - tpre[lo];
        c.t0 = tstart[lo] + c.j * kWave;
        enter_unit(c);
        enter_block(c);
        return c;
    }

    // index of the partial record that wave `gw` writes for the unit the cursor is in
    template <typename C>
    __device__ __forceinline__ int slot_of(const C &c, int gw) const
    {
        const int unit_first_tile = (c.li * sp.kv_heads + c.kvh) * TT + tpre[c.agent];
        return gw - unit_first_tile / per;
    }
};

} // namespace q4kv

// Host-side block pool (Sec. 3.1 "Block Pool with Per-Agent Isolation"): which 256-token block of the device pools
// belongs to which agent, in which order, and which agent has been idle longest.  Pure bookkeeping in host memory:
// no device call, no kernel.  The device side of the same component is the block table the attention kernels read
// (one row per agent, written from q4kv_block_pool_table_row) and the block images of persist.hip (an evicted
// agent's blocks leave through q4kv_export_blocks and come back, into whatever blocks are free then, through
// q4kv_import_blocks).
//
// Isolation is structural: a block id is either on the free list or in exactly one agent's list; every entry point
// keeps that invariant and none hands out a block twice.  All entry points lock one mutex per pool.
#include <cstdint>
#include <functional>
#include <mutex>
#include <new>
#include <queue>
#include <unordered_map>
#include <vector>

#include "../../include/q4kv.h"

struct q4kv_block_pool {
    struct Agent {
        std::vector<int32_t> blocks; // token order: entry i holds tokens 256 i .. 256 i + 255
        uint64_t stamp = 0;          // larger = used more recently
        bool pinned = false;         // part of a running batch: never a victim
    };
    std::mutex mu;
    std::vector<int64_t> owner;                                                     // per block: agent id, or -1 when free
    std::vector<uint8_t> is_free;
    std::priority_queue<int32_t, std::vector<int32_t>, std::greater<int32_t>> free_ids; // lowest id first
    std::unordered_map<int64_t, Agent> agents;
    uint64_t clock = 0;
    int32_t free_count = 0;
};

namespace {
constexpr int64_t kBlock = 256;
}

extern "C" {

q4kv_block_pool *q4kv_block_pool_create(int32_t num_blocks)
{
    if (num_blocks <= 0) return nullptr;
    q4kv_block_pool *p = new (std::nothrow) q4kv_block_pool;
    if (!p) return nullptr;
    try {
        p->owner.assign((size_t)num_blocks, -1);
        p->is_free.assign((size_t)num_blocks, 1);
        for (int32_t i = 0; i < num_blocks; ++i) p->free_ids.push(i);
    } catch (...) {
        delete p;
        return nullptr;
    }
    p->free_count = num_blocks;
    return p;
}

void q4kv_block_pool_destroy(q4kv_block_pool *pool) { delete pool; }

int32_t q4kv_block_pool_reserve(q4kv_block_pool *pool, int64_t agent_id, int64_t tokens)
{
    if (!pool || agent_id < 0 || tokens < 0) return Q4KV_EINVAL;
    const int64_t need64 = (tokens + kBlock - 1) / kBlock;
    std::lock_guard<std::mutex> lock(pool->mu);
    if (need64 > (int64_t)pool->owner.size()) return Q4KV_ENOSPACE;
    const int32_t need = (int32_t)need64;
    auto it = pool->agents.find(agent_id);
    const int32_t have = it == pool->agents.end() ? 0 : (int32_t)it->second.blocks.size();
    if (need - have > pool->free_count) return Q4KV_ENOSPACE; // nothing has changed
    try {
        q4kv_block_pool::Agent &a = pool->agents[agent_id];
        a.blocks.reserve((size_t)(need > have ? need : have));
        for (int32_t i = have; i < need; ++i) {
            const int32_t id = pool->free_ids.top();
            pool->free_ids.pop();
            pool->is_free[(size_t)id] = 0;
            pool->owner[(size_t)id] = agent_id;
            --pool->free_count;
            a.blocks.push_back(id);
        }
        a.stamp = ++pool->clock;
        return (int32_t)a.blocks.size();
    } catch (...) {
        return Q4KV_ENOSPACE;
    }
}

int32_t q4kv_block_pool_release(q4kv_block_pool *pool, int64_t agent_id)
{
    if (!pool) return Q4KV_EINVAL;
    std::lock_guard<std::mutex> lock(pool->mu);
    auto it = pool->agents.find(agent_id);
    if (it == pool->agents.end()) return Q4KV_EINVAL;
    const int32_t n = (int32_t)it->second.blocks.size();
    for (int32_t id : it->second.blocks) {
        pool->owner[(size_t)id] = -1;
        pool->is_free[(size_t)id] = 1;
        pool->free_ids.push(id);
    }
    pool->free_count += n;
    pool->agents.erase(it);
    return n;
}

int32_t q4kv_block_pool_blocks(q4kv_block_pool *pool, int64_t agent_id, int32_t *ids, int32_t cap)
{
    if (!pool || cap < 0 || (cap > 0 && !ids)) return Q4KV_EINVAL;
    std::lock_guard<std::mutex> lock(pool->mu);
    auto it = pool->agents.find(agent_id);
    if (it == pool->agents.end()) return Q4KV_EINVAL;
    const int32_t n = (int32_t)it->second.blocks.size();
    for (int32_t i = 0; i < n && i < cap; ++i) ids[i] = it->second.blocks[(size_t)i];
    return n;
}

int32_t q4kv_block_pool_table_row(q4kv_block_pool *pool, int64_t agent_id, int32_t *row, int32_t max_blocks, int32_t fill)
{
    if (!pool || !row || max_blocks <= 0) return Q4KV_EINVAL;
    std::lock_guard<std::mutex> lock(pool->mu);
    auto it = pool->agents.find(agent_id);
    if (it == pool->agents.end()) return Q4KV_EINVAL;
    const int32_t n = (int32_t)it->second.blocks.size();
    if (n > max_blocks) return Q4KV_ERANGE;
    for (int32_t i = 0; i < max_blocks; ++i) row[i] = i < n ? it->second.blocks[(size_t)i] : fill;
    return n;
}

int32_t q4kv_block_pool_touch(q4kv_block_pool *pool, int64_t agent_id)
{
    if (!pool) return Q4KV_EINVAL;
    std::lock_guard<std::mutex> lock(pool->mu);
    auto it = pool->agents.find(agent_id);
    if (it == pool->agents.end()) return Q4KV_EINVAL;
    it->second.stamp = ++pool->clock;
    return Q4KV_OK;
}

int32_t q4kv_block_pool_pin(q4kv_block_pool *pool, int64_t agent_id, int32_t pinned)
{
    if (!pool) return Q4KV_EINVAL;
    std::lock_guard<std::mutex> lock(pool->mu);
    auto it = pool->agents.find(agent_id);
    if (it == pool->agents.end()) return Q4KV_EINVAL;
    it->second.pinned = pinned != 0;
    return Q4KV_OK;
}

int64_t q4kv_block_pool_lru_victim(q4kv_block_pool *pool)
{
    if (!pool) return -1;
    std::lock_guard<std::mutex> lock(pool->mu);
    int64_t victim = -1;
    uint64_t oldest = 0;
    for (const auto &kv : pool->agents) {
        const q4kv_block_pool::Agent &a = kv.second;
        if (a.pinned || a.blocks.empty()) continue;
        if (victim < 0 || a.stamp < oldest) {
            victim = kv.first;
            oldest = a.stamp;
        }
    }
    return victim;
}

int32_t q4kv_block_pool_free_blocks(q4kv_block_pool *pool)
{
    if (!pool) return Q4KV_EINVAL;
    std::lock_guard<std::mutex> lock(pool->mu);
    return pool->free_count;
}

int64_t q4kv_block_pool_owner(q4kv_block_pool *pool, int32_t block_id)
{
    if (!pool) return -1;
    std::lock_guard<std::mutex> lock(pool->mu);
    if (block_id < 0 || (size_t)block_id >= pool->owner.size()) return -1;
    return pool->owner[(size_t)block_id];
}

} // extern "C"

// The C ABI of libq4kv (include/q4kv.h): argument validation on the host, launch planning
// (split-K schedule), and nothing else -- every step of the path runs in the kernels.
#include <atomic>
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "q4kv_internal.h"

// Workspace of q4kv_batched_attention_static: one copy per GPU inside the loaded code object, never allocated or
// freed.  In host code this name is only a handle for hipGetSymbolAddress; the device address it yields (one per
// device) is what kernels and host calls are given.
static __device__ __align__(256) unsigned char scratch[Q4KV_STATIC_SCRATCH_BYTES];

namespace {

thread_local char g_error[256] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return code;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_spec(const q4kv_spec *s)
{
    if (!s) return fail(Q4KV_EINVAL, "spec is NULL");
    if (s->num_layers <= 0 || s->num_q_heads <= 0 || s->num_kv_heads <= 0)
        return fail(Q4KV_ESHAPE, "layer/head counts must be positive");
    if (s->num_q_heads % s->num_kv_heads) return fail(Q4KV_ESHAPE, "num_q_heads %% num_kv_heads != 0");
    if (s->group_size != 64) return fail(Q4KV_ESHAPE, "group_size must be 64");
    if (s->block_tokens != 256) return fail(Q4KV_ESHAPE, "block_tokens must be 256");
    if (s->k_dim <= 0 || s->v_dim <= 0 || s->k_dim % 64 || s->v_dim % 64)
        return fail(Q4KV_ESHAPE, "k_dim and v_dim must be positive multiples of 64");
    if (s->v_aliases_k && s->v_dim > s->k_dim) return fail(Q4KV_ESHAPE, "v_aliases_k needs v_dim <= k_dim");
    if (s->param_format != Q4KV_PARAMS_F16 && s->param_format != Q4KV_PARAMS_BF16)
        return fail(Q4KV_EINVAL, "param_format %d is neither Q4KV_PARAMS_F16 nor Q4KV_PARAMS_BF16", s->param_format);
    return Q4KV_OK;
}

int check_pool(const q4kv_pool *p, const char *name)
{
    if (!p) return fail(Q4KV_EINVAL, "%s pool is NULL", name);
    if (!p->codes || !p->scale || !p->bias) return fail(Q4KV_EINVAL, "%s pool has a NULL array", name);
    if (!aligned16(p->codes) || !aligned16(p->scale) || !aligned16(p->bias))
        return fail(Q4KV_EINVAL, "%s pool arrays must be 16-byte aligned", name);
    if (p->num_blocks <= 0) return fail(Q4KV_EINVAL, "%s pool has no blocks", name);
    return Q4KV_OK;
}

// Compute units of the current device (cached per device); the attention launch is two workgroups per unit.
int compute_units()
{
    static std::atomic<int> cached[64]; // zero-initialised; threads that race here store the same value
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

// Workgroups of a decode launch: the shared-latent kernel fills a compute unit's LDS with one workgroup,
// the GQA kernel runs two per compute unit.
int attention_workgroups(const q4kv_spec &s) { return (q4kv::mla_decode_supported(s) ? 1 : 2) * compute_units(); }

// Smallest token range a wave takes when the caller leaves the choice to the library.  The floor matters for small
// jobs only (a wave's partial record and its share of the combine step cost about one tile's time, so shares
// of very few tiles do not pay); a large job gives every wave an even share whatever the floor is.  Since only the
// device knows how much of max_seq_len the agents and the sliding windows leave visible, the floor stays small:
// twice an even share of the largest possible job, between one block and 512 tokens.  Measured on one layer's
// call: 10 agents of 1K-8K tokens, 256-wide heads (even share 2.7 tiles) 51.6 / 47.8 / 52.6 / 59.9 us at 256 /
// 512 / 768 / 1,024 tokens; 5 agents of 4K tokens, 128-wide heads (1.25 tiles) 32.6 / 34.2 / 43.6 / 46.7 us.
// A larger floor leaves waves without work whenever the visible cache is a fraction of the largest job: at
// 4,096 tokens a quarter of the waves on a 10-agent, 48-layer step whose windows hid two thirds of the cache; at
// 1,024 tokens four in ten on ten 300-token agents (0.115 ms against 0.090 ms at 512).
int pick_split_tokens(const q4kv_spec &s, int num_agents, int max_seq_len, int layers)
{
    const long long tiles = (long long)layers * s.num_kv_heads * num_agents * ((max_seq_len + 63) / 64);
    // the workers that share the tiles out: workgroups, or single waves for the shared-latent kernel
    const long long workers =
        (long long)attention_workgroups(s) * (q4kv::mla_decode_supported(s) ? q4kv::decode_waves_per_workgroup() : 1);
    long long blocks = tiles / workers / 2; // 2 * (tiles / workers) tiles, in 256-token blocks of 4 tiles
    if (blocks < 1) blocks = 1;
    if (blocks > 2) blocks = 2;
    return (int)blocks * 256;
}

// Partial records reserved per (layer, agent, query head): the most workers that can meet in one unit.  A worker's
// range is at least split_tokens long.  The GQA kernel's workers are workgroups, except that from a certain range
// length on (decode_solo_quarter_tiles() * 4) every wave takes a quarter of its workgroup's range and writes a record
// of its own.
int slots_per_unit(const q4kv_spec &s, int max_seq_len, int split_tokens)
{
    const int tiles = (max_seq_len + 63) / 64, min_per = split_tokens / 64;
    int slots = (tiles + min_per - 1) / min_per + 1;
    if (!q4kv::mla_decode_supported(s)) {
        int quarter = min_per / 4;
        if (quarter < q4kv::decode_solo_quarter_tiles()) quarter = q4kv::decode_solo_quarter_tiles();
        const int solo = (tiles + quarter - 1) / quarter + 1;
        if (solo > slots) slots = solo;
    }
    return slots;
}

size_t plan_bytes(int num_agents, int layers)
{
    return (q4kv::decode_plan_ints(num_agents, layers) * sizeof(int32_t) + 255) / 256 * 256;
}

// What a plan depends on besides seq_len[], folded into one word: kept in the plan and compared by the kernels, so
// that a prepared workspace used with other arguments makes a planned call do nothing instead of walking a plan that
// does not fit its tables.
int plan_signature(const q4kv_spec &s, int num_agents, int max_seq_len, int layers, int split_tokens, int window,
                   int workgroups)
{
    const int v[] = {s.num_q_heads, s.num_kv_heads, s.k_dim, s.v_dim, s.v_aliases_k, num_agents, max_seq_len, layers,
                     split_tokens, window > 0 ? window : 0, workgroups};
    uint32_t h = 0x9E3779B9u;
    for (int x : v) h = (h ^ (uint32_t)x) * 0x01000193u + 0x7F4A7C15u;
    return (int)(h | 1u); // never zero
}

// arrival counters, one per (layer, KV head, agent)
size_t arrival_bytes(const q4kv_spec &s, int num_agents, int layers)
{
    return ((size_t)layers * s.num_kv_heads * num_agents * sizeof(int32_t) + 255) / 256 * 256;
}

} // namespace

extern "C" {

int q4kv_version(void) { return 100; }

const char *q4kv_last_error(void) { return g_error; }

int64_t q4kv_cache_bytes(const q4kv_spec *spec, int64_t tokens)
{
    if (check_spec(spec) != Q4KV_OK) return -1;
    if (tokens < 0) {
        fail(Q4KV_EINVAL, "tokens < 0");
        return -1;
    }
    const int64_t width = spec->k_dim + (spec->v_aliases_k ? 0 : spec->v_dim);
    const int64_t elems = (int64_t)spec->num_layers * spec->num_kv_heads * width * tokens;
    return elems / 2 + 4 * (elems / 64);
}

int q4kv_quantize_fmt(const uint16_t *x, int64_t rows, int32_t dim, int32_t param_format, uint32_t *codes,
                      uint16_t *scale, uint16_t *bias, void *hip_stream)
{
    if (param_format != Q4KV_PARAMS_F16 && param_format != Q4KV_PARAMS_BF16)
        return fail(Q4KV_EINVAL, "param_format %d is neither Q4KV_PARAMS_F16 nor Q4KV_PARAMS_BF16", param_format);
    if (dim <= 0 || dim % 64) return fail(Q4KV_ESHAPE, "dim must be a positive multiple of 64");
    if (rows < 0) return fail(Q4KV_EINVAL, "rows < 0");
    if (rows == 0) return Q4KV_OK;
    if (!x || !codes || !scale || !bias) return fail(Q4KV_EINVAL, "NULL pointer");
    if (!aligned16(x) || !aligned16(codes)) return fail(Q4KV_EINVAL, "x and codes must be 16-byte aligned");
    hipError_t e = q4kv::launch_quantize(x, rows, dim, param_format == Q4KV_PARAMS_BF16, codes, scale, bias,
                                         compute_units(), (hipStream_t)hip_stream);
    return e == hipSuccess ? Q4KV_OK : fail(Q4KV_EHIP, "quantize launch: %s", hipGetErrorString(e));
}

int q4kv_quantize(const uint16_t *x, int64_t rows, int32_t dim, uint32_t *codes, uint16_t *scale, uint16_t *bias,
                  void *hip_stream)
{
    return q4kv_quantize_fmt(x, rows, dim, Q4KV_PARAMS_F16, codes, scale, bias, hip_stream);
}

int q4kv_dequantize_fmt(const uint32_t *codes, const uint16_t *scale, const uint16_t *bias, int64_t rows, int32_t dim,
                        int32_t param_format, uint16_t *x, void *hip_stream)
{
    if (param_format != Q4KV_PARAMS_F16 && param_format != Q4KV_PARAMS_BF16)
        return fail(Q4KV_EINVAL, "param_format %d is neither Q4KV_PARAMS_F16 nor Q4KV_PARAMS_BF16", param_format);
    if (dim <= 0 || dim % 64) return fail(Q4KV_ESHAPE, "dim must be a positive multiple of 64");
    if (rows < 0) return fail(Q4KV_EINVAL, "rows < 0");
    if (rows == 0) return Q4KV_OK;
    if (!x || !codes || !scale || !bias) return fail(Q4KV_EINVAL, "NULL pointer");
    if (!aligned16(x) || !aligned16(codes)) return fail(Q4KV_EINVAL, "x and codes must be 16-byte aligned");
    hipError_t e = q4kv::launch_dequantize(codes, scale, bias, rows, dim, param_format == Q4KV_PARAMS_BF16, x,
                                           compute_units(), (hipStream_t)hip_stream);
    return e == hipSuccess ? Q4KV_OK : fail(Q4KV_EHIP, "dequantize launch: %s", hipGetErrorString(e));
}

int q4kv_dequantize(const uint32_t *codes, const uint16_t *scale, const uint16_t *bias, int64_t rows, int32_t dim,
                    uint16_t *x, void *hip_stream)
{
    return q4kv_dequantize_fmt(codes, scale, bias, rows, dim, Q4KV_PARAMS_F16, x, hip_stream);
}

int q4kv_append(const q4kv_spec *spec, const q4kv_pool *k, const q4kv_pool *v, const uint16_t *k_new,
                const uint16_t *v_new, const int32_t *block_table, int32_t max_blocks,
                const int32_t *seq_len_before, int32_t num_agents, int32_t chunk_len, int32_t layer_begin,
                int32_t layer_end, void *hip_stream)
{
    int rc = check_spec(spec);
    if (rc) return rc;
    if ((rc = check_pool(k, "K"))) return rc;
    if (spec->v_aliases_k) {
        if (v || v_new) return fail(Q4KV_EINVAL, "v and v_new must be NULL when v_aliases_k");
    } else {
        if ((rc = check_pool(v, "V"))) return rc;
        if (v->num_blocks != k->num_blocks) return fail(Q4KV_EINVAL, "K and V pools differ in num_blocks");
    }
    if (layer_begin < 0 || layer_end > spec->num_layers || layer_begin > layer_end)
        return fail(Q4KV_EINVAL, "bad layer range [%d, %d)", layer_begin, layer_end);
    if (num_agents < 0 || chunk_len < 0 || max_blocks <= 0) return fail(Q4KV_EINVAL, "negative count");
    if (num_agents == 0 || chunk_len == 0 || layer_begin == layer_end) return Q4KV_OK;
    if (chunk_len > Q4KV_MAX_CHUNK_LEN)
        return fail(Q4KV_ERANGE, "chunk_len %d is beyond %d tokens: append it in pieces", chunk_len, Q4KV_MAX_CHUNK_LEN);
    if (!k_new || (!spec->v_aliases_k && !v_new) || !block_table || !seq_len_before)
        return fail(Q4KV_EINVAL, "NULL pointer");
    if (!aligned16(k_new) || (v_new && !aligned16(v_new))) return fail(Q4KV_EINVAL, "k_new/v_new must be 16-byte aligned");
    hipStream_t st = (hipStream_t)hip_stream;
    hipError_t e = q4kv::launch_append(*spec, *k, spec->v_aliases_k ? nullptr : v, k_new, v_new, block_table, max_blocks,
                                       seq_len_before, num_agents, chunk_len, layer_begin, layer_end, compute_units(), st);
    return e == hipSuccess ? Q4KV_OK : fail(Q4KV_EHIP, "append launch: %s", hipGetErrorString(e));
}

int32_t q4kv_default_split_tokens(const q4kv_spec *spec, int32_t num_agents, int32_t q_len, int32_t max_seq_len,
                                  int32_t num_layers_in_call)
{
    if (check_spec(spec) != Q4KV_OK) return 0;
    if (num_agents <= 0 || q_len <= 0 || max_seq_len < 0 || num_layers_in_call <= 0) {
        fail(Q4KV_EINVAL, "bad counts");
        return 0;
    }
    return pick_split_tokens(*spec, num_agents, max_seq_len, num_layers_in_call);
}

size_t q4kv_attention_workspace_bytes(const q4kv_spec *spec, int32_t num_agents, int32_t q_len, int32_t max_seq_len,
                                      int32_t split_tokens, int32_t num_layers_in_call)
{
    if (check_spec(spec) != Q4KV_OK) return 0;
    if (num_agents <= 0 || q_len <= 0 || max_seq_len < 0 || num_layers_in_call <= 0 || split_tokens < 0 ||
        split_tokens % 256) {
        fail(Q4KV_EINVAL, "bad counts");
        return 0;
    }
    if (q_len > 1) return 0; // the chunk kernel keeps everything on chip
    const int st = split_tokens ? split_tokens : pick_split_tokens(*spec, num_agents, max_seq_len, num_layers_in_call);
    const int64_t slots = slots_per_unit(*spec, max_seq_len, st);
    const int64_t units = (int64_t)num_layers_in_call * num_agents * q_len * spec->num_q_heads;
    return plan_bytes(num_agents, num_layers_in_call) + arrival_bytes(*spec, num_agents, num_layers_in_call) +
           (size_t)(units * slots * (spec->v_dim + 2) * (int64_t)sizeof(float));
}

// planned: the workspace already holds the plan of q4kv_decode_plan for these arguments (seq_len is then not needed)
static int attention_common(const q4kv_spec *spec, const q4kv_pool *k, const q4kv_pool *v, const uint16_t *q,
                            uint16_t *out, const int32_t *block_table, int32_t max_blocks, const int32_t *seq_len,
                            int32_t num_agents, int32_t q_len, int32_t max_seq_len, float sm_scale, int32_t window,
                            const int32_t *layer_window, int32_t split_tokens, int32_t layer_begin, int32_t layer_end,
                            void *workspace, size_t workspace_bytes, void *hip_stream, bool planned = false)
{
    int rc = check_spec(spec);
    if (rc) return rc;
    if ((rc = check_pool(k, "K"))) return rc;
    if (spec->v_aliases_k) {
        if (v) return fail(Q4KV_EINVAL, "v must be NULL when v_aliases_k");
    } else {
        if ((rc = check_pool(v, "V"))) return rc;
        if (v->num_blocks != k->num_blocks) return fail(Q4KV_EINVAL, "K and V pools differ in num_blocks");
    }
    if (layer_begin < 0 || layer_end > spec->num_layers || layer_begin > layer_end)
        return fail(Q4KV_EINVAL, "bad layer range [%d, %d)", layer_begin, layer_end);
    if (num_agents < 0 || q_len < 1 || max_blocks <= 0 || max_seq_len < 0) return fail(Q4KV_EINVAL, "bad counts");
    if (split_tokens < 0 || split_tokens % 256) return fail(Q4KV_EINVAL, "split_tokens must be a multiple of 256");
    if ((int64_t)max_seq_len > (int64_t)max_blocks * 256)
        return fail(Q4KV_ERANGE, "max_seq_len %d exceeds max_blocks*256 = %lld", max_seq_len,
                    (long long)max_blocks * 256);
    if (num_agents == 0 || layer_begin == layer_end) return Q4KV_OK;
    if (!q || !out || !block_table || (!seq_len && !planned)) return fail(Q4KV_EINVAL, "NULL pointer");
    if (!aligned16(q) || !aligned16(out)) return fail(Q4KV_EINVAL, "q and out must be 16-byte aligned");
    const int layers = layer_end - layer_begin;
    // the kernels number the 64-token tiles of a call with 32-bit integers
    if ((int64_t)layers * spec->num_kv_heads * num_agents * (((int64_t)max_seq_len + 63) / 64 + 1) > 0x7fffffffLL)
        return fail(Q4KV_ERANGE, "more than 2^31 tiles in one call: split the layer range");

    q4kv::AttentionArgs a;
    a.spec = *spec;
    a.k = *k;
    a.v = spec->v_aliases_k ? *k : *v;
    a.q = q;
    a.out = out;
    a.block_table = block_table;
    a.seq_len = seq_len;
    a.max_blocks = max_blocks;
    a.num_agents = num_agents;
    a.q_len = q_len;
    a.max_seq_len = max_seq_len;
    a.window = window;
    a.layer_window = layer_window;
    a.split_tokens = split_tokens ? split_tokens : pick_split_tokens(*spec, num_agents, max_seq_len, layers);
    a.max_slots = slots_per_unit(*spec, max_seq_len, a.split_tokens);
    a.grid_workgroups = attention_workgroups(*spec);
    a.layer_begin = layer_begin;
    a.layers_in_call = layers;
    a.sm_scale = sm_scale;

    hipStream_t st = (hipStream_t)hip_stream;
    if (q_len > 1) { // chunked append: causal attention of q_len new tokens per agent, no workspace needed
        if (!q4kv::chunk_supported(*spec))
            return fail(Q4KV_ESHAPE, "no chunk kernel for k_dim=%d v_dim=%d n_rep=%d alias=%d", spec->k_dim, spec->v_dim,
                        spec->num_q_heads / spec->num_kv_heads, spec->v_aliases_k);
        hipError_t e = q4kv::launch_chunk_attention(a, st);
        return e == hipSuccess ? Q4KV_OK : fail(Q4KV_EHIP, "attention launch: %s", hipGetErrorString(e));
    }
    const bool mla = q4kv::mla_decode_supported(*spec);
    if (!mla && !q4kv::decode_supported(*spec))
        return fail(Q4KV_ESHAPE, "no decode kernel for k_dim=%d v_dim=%d n_rep=%d alias=%d", spec->k_dim, spec->v_dim,
                    spec->num_q_heads / spec->num_kv_heads, spec->v_aliases_k);

    const size_t need = q4kv_attention_workspace_bytes(spec, num_agents, q_len, max_seq_len, a.split_tokens, layers);
    if (!workspace || workspace_bytes < need || !aligned16(workspace))
        return fail(Q4KV_EWORKSPACE, "workspace needs %zu bytes (16-byte aligned), got %zu", need, workspace_bytes);
    const int64_t units = (int64_t)layers * num_agents * q_len * spec->num_q_heads;
    a.plan = static_cast<int32_t *>(workspace);
    a.arrivals = reinterpret_cast<int32_t *>(static_cast<char *>(workspace) + plan_bytes(num_agents, layers));
    a.part_acc = reinterpret_cast<float *>(static_cast<char *>(workspace) + plan_bytes(num_agents, layers) +
                                           arrival_bytes(*spec, num_agents, layers));
    a.part_ml = a.part_acc + units * a.max_slots * spec->v_dim;
    a.plan_signature = plan_signature(*spec, num_agents, max_seq_len, layers, a.split_tokens, layer_window ? -1 : window,
                                      a.grid_workgroups);

    hipError_t e = hipSuccess;
    if (!planned) e = mla ? q4kv::launch_mla_decode_plan(a, st) : q4kv::launch_decode_plan(a, st);
    if (e == hipSuccess) e = mla ? q4kv::launch_mla_decode_attention(a, st) : q4kv::launch_decode_attention(a, st);
    return e == hipSuccess ? Q4KV_OK : fail(Q4KV_EHIP, "attention launch: %s", hipGetErrorString(e));
}

int q4kv_batched_attention(const q4kv_spec *spec, const q4kv_pool *k, const q4kv_pool *v, const uint16_t *q,
                           uint16_t *out, const int32_t *block_table, int32_t max_blocks, const int32_t *seq_len,
                           int32_t num_agents, int32_t q_len, int32_t max_seq_len, float sm_scale, int32_t window,
                           int32_t split_tokens, int32_t layer_begin, int32_t layer_end, void *workspace,
                           size_t workspace_bytes, void *hip_stream)
{
    return attention_common(spec, k, v, q, out, block_table, max_blocks, seq_len, num_agents, q_len, max_seq_len, sm_scale,
                            window, nullptr, split_tokens, layer_begin, layer_end, workspace, workspace_bytes, hip_stream);
}

int q4kv_batched_attention_windows(const q4kv_spec *spec, const q4kv_pool *k, const q4kv_pool *v, const uint16_t *q,
                                   uint16_t *out, const int32_t *block_table, int32_t max_blocks,
                                   const int32_t *seq_len, int32_t num_agents, int32_t q_len, int32_t max_seq_len,
                                   float sm_scale, const int32_t *window_per_layer, int32_t split_tokens,
                                   int32_t layer_begin, int32_t layer_end, void *workspace, size_t workspace_bytes,
                                   void *hip_stream)
{
    if (!window_per_layer) return fail(Q4KV_EINVAL, "NULL window_per_layer");
    if (layer_end - layer_begin > q4kv::max_window_layers())
        return fail(Q4KV_EINVAL, "at most %d layers per call with per-layer windows", q4kv::max_window_layers());
    return attention_common(spec, k, v, q, out, block_table, max_blocks, seq_len, num_agents, q_len, max_seq_len, sm_scale,
                            0, window_per_layer, split_tokens, layer_begin, layer_end, workspace, workspace_bytes,
                            hip_stream);
}

// Device address of `scratch` on the current device, looked up once per device (threads that race here store the
// same value).  nullptr with the error message set when the runtime cannot resolve it.
static void *static_scratch()
{
    static std::atomic<void *> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        fail(Q4KV_EHIP, "no current device (or a device index above 63)");
        return nullptr;
    }
    void *ptr = cached[dev].load(std::memory_order_acquire);
    if (!ptr) {
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            fail(Q4KV_EHIP, "address of the static scratch array on device %d: %s", dev, hipGetErrorString(e));
            return nullptr;
        }
        cached[dev].store(ptr, std::memory_order_release);
    }
    return ptr;
}

int q4kv_batched_attention_static(const q4kv_spec *spec, const q4kv_pool *k, const q4kv_pool *v, const uint16_t *q,
                                  uint16_t *out, const int32_t *block_table, int32_t max_blocks,
                                  const int32_t *seq_len, int32_t num_agents, int32_t q_len, int32_t max_seq_len,
                                  float sm_scale, int32_t window, int32_t split_tokens, int32_t layer_begin,
                                  int32_t layer_end, void *hip_stream)
{
    // the size first, from host arithmetic alone: a call that does not fit launches nothing and touches no device state
    if (spec && num_agents > 0 && q_len == 1 && max_seq_len >= 0 && layer_end > layer_begin && split_tokens >= 0 &&
        split_tokens % 256 == 0 && check_spec(spec) == Q4KV_OK) {
        const size_t need =
            q4kv_attention_workspace_bytes(spec, num_agents, q_len, max_seq_len, split_tokens, layer_end - layer_begin);
        if (need > (size_t)Q4KV_STATIC_SCRATCH_BYTES)
            return fail(Q4KV_EWORKSPACE,
                        "the call needs %zu bytes of workspace, the static scratch array holds %u: pass fewer layers "
                        "per call or a larger split_tokens, or use q4kv_batched_attention with a workspace",
                        need, (unsigned)Q4KV_STATIC_SCRATCH_BYTES);
    }
    void *ptr = static_scratch();
    if (!ptr) return Q4KV_EHIP;
    return attention_common(spec, k, v, q, out, block_table, max_blocks, seq_len, num_agents, q_len, max_seq_len, sm_scale,
                            window, nullptr, split_tokens, layer_begin, layer_end, ptr, (size_t)Q4KV_STATIC_SCRATCH_BYTES,
                            hip_stream);
}

int q4kv_decode_plan(const q4kv_spec *spec, const int32_t *seq_len, int32_t num_agents, int32_t max_seq_len,
                     int32_t window, int32_t split_tokens, int32_t num_layers_in_call, void *workspace,
                     size_t workspace_bytes, void *hip_stream)
{
    int rc = check_spec(spec);
    if (rc) return rc;
    if (num_agents < 0 || max_seq_len < 0 || num_layers_in_call < 0) return fail(Q4KV_EINVAL, "bad counts");
    if (split_tokens < 0 || split_tokens % 256) return fail(Q4KV_EINVAL, "split_tokens must be a multiple of 256");
    if (num_agents == 0 || num_layers_in_call == 0) return Q4KV_OK;
    if (!seq_len) return fail(Q4KV_EINVAL, "NULL pointer");
    const bool mla = q4kv::mla_decode_supported(*spec);
    if (!mla && !q4kv::decode_supported(*spec))
        return fail(Q4KV_ESHAPE, "no decode kernel for k_dim=%d v_dim=%d n_rep=%d alias=%d", spec->k_dim, spec->v_dim,
                    spec->num_q_heads / spec->num_kv_heads, spec->v_aliases_k);
    if ((int64_t)num_layers_in_call * spec->num_kv_heads * num_agents * (((int64_t)max_seq_len + 63) / 64 + 1) > 0x7fffffffLL)
        return fail(Q4KV_ERANGE, "more than 2^31 tiles in one call: split the layer range");
    q4kv::AttentionArgs a{};
    a.spec = *spec;
    a.seq_len = seq_len;
    a.num_agents = num_agents;
    a.q_len = 1;
    a.max_seq_len = max_seq_len;
    a.window = window;
    a.layer_window = nullptr;
    a.split_tokens = split_tokens ? split_tokens : pick_split_tokens(*spec, num_agents, max_seq_len, num_layers_in_call);
    a.grid_workgroups = attention_workgroups(*spec);
    a.layers_in_call = num_layers_in_call;
    const size_t need = q4kv_attention_workspace_bytes(spec, num_agents, 1, max_seq_len, a.split_tokens, num_layers_in_call);
    if (!workspace || workspace_bytes < need || !aligned16(workspace))
        return fail(Q4KV_EWORKSPACE, "workspace needs %zu bytes (16-byte aligned), got %zu", need, workspace_bytes);
    a.plan = static_cast<int32_t *>(workspace);
    a.arrivals = reinterpret_cast<int32_t *>(static_cast<char *>(workspace) + plan_bytes(num_agents, num_layers_in_call));
    a.plan_signature = plan_signature(*spec, num_agents, max_seq_len, num_layers_in_call, a.split_tokens, window,
                                      a.grid_workgroups);
    hipStream_t st = (hipStream_t)hip_stream;
    const hipError_t e = mla ? q4kv::launch_mla_decode_plan(a, st) : q4kv::launch_decode_plan(a, st);
    return e == hipSuccess ? Q4KV_OK : fail(Q4KV_EHIP, "plan launch: %s", hipGetErrorString(e));
}

int q4kv_batched_attention_planned(const q4kv_spec *spec, const q4kv_pool *k, const q4kv_pool *v, const uint16_t *q,
                                   uint16_t *out, const int32_t *block_table, int32_t max_blocks, int32_t num_agents,
                                   int32_t max_seq_len, float sm_scale, int32_t window, int32_t split_tokens,
                                   int32_t layer_begin, int32_t layer_end, void *workspace, size_t workspace_bytes,
                                   void *hip_stream)
{
    return attention_common(spec, k, v, q, out, block_table, max_blocks, nullptr, num_agents, 1, max_seq_len, sm_scale,
                            window, nullptr, split_tokens, layer_begin, layer_end, workspace, workspace_bytes, hip_stream,
                            true);
}

size_t q4kv_block_image_bytes(const q4kv_spec *spec, int32_t num_blocks)
{
    if (check_spec(spec) != Q4KV_OK) return 0;
    if (num_blocks < 0) {
        fail(Q4KV_EINVAL, "num_blocks < 0");
        return 0;
    }
    return q4kv::image_record_bytes(*spec) * (size_t)spec->num_layers * (size_t)num_blocks;
}

static int block_image_common(const q4kv_spec *spec, const q4kv_pool *k, const q4kv_pool *v, const int32_t *block_ids,
                              int32_t num_blocks, void *image, size_t image_bytes, bool to_image, void *hip_stream)
{
    int rc = check_spec(spec);
    if (rc) return rc;
    if ((rc = check_pool(k, "K"))) return rc;
    if (spec->v_aliases_k) {
        if (v) return fail(Q4KV_EINVAL, "V pool must be NULL when v_aliases_k is set");
    } else {
        if ((rc = check_pool(v, "V"))) return rc;
        if (v->num_blocks != k->num_blocks) return fail(Q4KV_EINVAL, "K and V pools differ in num_blocks");
    }
    if (num_blocks < 0) return fail(Q4KV_EINVAL, "num_blocks < 0");
    if (num_blocks == 0) return Q4KV_OK;
    if (!block_ids || !image) return fail(Q4KV_EINVAL, "NULL pointer");
    if (!aligned16(image)) return fail(Q4KV_EINVAL, "image must be 16-byte aligned");
    if (image_bytes < q4kv_block_image_bytes(spec, num_blocks)) return fail(Q4KV_EWORKSPACE, "image buffer too small");
    hipError_t e = q4kv::launch_image_copy(*spec, *k, spec->v_aliases_k ? nullptr : v, block_ids, num_blocks, image,
                                          to_image, 8 * compute_units(), (hipStream_t)hip_stream);
    return e == hipSuccess ? Q4KV_OK : fail(Q4KV_EHIP, "block image launch: %s", hipGetErrorString(e));
}

int q4kv_export_blocks(const q4kv_spec *spec, const q4kv_pool *k, const q4kv_pool *v, const int32_t *block_ids,
                       int32_t num_blocks, void *image, size_t image_bytes, void *hip_stream)
{
    return block_image_common(spec, k, v, block_ids, num_blocks, image, image_bytes, true, hip_stream);
}

int q4kv_import_blocks(const q4kv_spec *spec, const q4kv_pool *k, const q4kv_pool *v, const int32_t *block_ids,
                       int32_t num_blocks, const void *image, size_t image_bytes, void *hip_stream)
{
    return block_image_common(spec, k, v, block_ids, num_blocks, const_cast<void *>(image), image_bytes, false,
                              hip_stream);
}

int q4kv_read_probe(const void *src, size_t bytes, uint32_t *sink, void *hip_stream)
{
    if (bytes < 16384) return Q4KV_OK; // nothing to read
    if (!src || !sink) return fail(Q4KV_EINVAL, "NULL pointer");
    if (!aligned16(src)) return fail(Q4KV_EINVAL, "src must be 16-byte aligned");
    hipError_t e = q4kv::launch_read_probe(src, bytes, sink, 2 * compute_units(), (hipStream_t)hip_stream);
    return e == hipSuccess ? Q4KV_OK : fail(Q4KV_EHIP, "read probe launch: %s", hipGetErrorString(e));
}

} // extern "C"

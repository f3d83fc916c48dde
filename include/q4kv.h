/*
 * q4kv.h -- C ABI of libq4kv: batched attention over many agents' paged, 4-bit
 * group-quantized KV caches on one AMD MI355X (gfx950), plus the Q4 pack/unpack
 * codec used when a cache is saved or restored.
 *
 * Conventions that hold for every entry point
 *   - "device" pointers are GPU global memory owned by the caller (for example the
 *     storage of a torch tensor).  The library allocates no device memory and keeps
 *     no state between calls.  "host" pointers are ordinary process memory.
 *   - Calls only enqueue work on `hip_stream` (a hipStream_t passed as void*, NULL =
 *     the default stream) and return without synchronising.
 *   - Return value: Q4KV_OK (0) or a negative q4kv_status.  Argument errors are found
 *     on the host before anything is launched; q4kv_last_error() then gives a message
 *     (thread-local, valid until the same thread's next failing call).
 *   - binary16 values travel as uint16_t bit patterns.  Inputs must be finite.
 *   - Calls that overlap in time on different streams are safe as long as their
 *     output and workspace buffers do not overlap.
 *
 * The Q4 format (Sec. 3.2 "Q4 Quantization Pipeline" of the paper; arithmetic fixed
 * by the project brief where the paper defers to its framework): a row of `dim`
 * elements is cut into groups of 64 consecutive elements along head_dim.  Per group:
 *     bias  = min x                          stored as binary16 (exact)
 *     scale = (max x - min x) / 15           computed in binary32, stored as binary16 (RNE)
 *     code  = clamp(rint((x - min) / scale_stored), 0, 15)   binary32 division, ties to even;
 *             all codes 0 when scale_stored == 0
 * Element d of a row lives in 32-bit word d/8, bits 4*(d%8) .. 4*(d%8)+3.
 * The paper stores scale and bias as bfloat16 for one model family and as binary16 for another (Sec. 3.1, Sec. 3.2,
 * appendix "safetensors Q4 Format").  Q4KV_PARAMS_BF16 selects the bfloat16 form: the same formula with both
 * parameters rounded to bfloat16 (nearest even) and the codes taken against the STORED parameters,
 *     code = clamp(rint((x - bias_stored) / scale_stored), 0, 15),
 * so a reader needs nothing but the stored values.  The stored bias is then in general not the minimum itself:
 * |x - x_hat| <= scale_stored/2 + |bias_stored - min| + 15 |scale_stored - scale|.  Parameters must stay inside the
 * binary16 range (they do for binary16 data).
 * Bytes per row: dim/2 (codes) + 2*dim/64 (scale) + 2*dim/64 (bias), i.e. K+V of a
 * layer take h*d*n*(1 + 8/64) bytes, the paper's count.
 */
#ifndef Q4KV_H
#define Q4KV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    Q4KV_OK = 0,
    Q4KV_EINVAL = -1,     /* null / misaligned pointer, negative count, bad layer range */
    Q4KV_ESHAPE = -2,     /* unsupported dims: dim % 64, q_heads % kv_heads, head widths, group/block size */
    Q4KV_ERANGE = -3,     /* max_seq_len exceeds what the block table can address, or chunk_len its limit */
    Q4KV_EWORKSPACE = -4, /* workspace too small or missing */
    Q4KV_EHIP = -5,       /* the HIP runtime refused a launch */
    Q4KV_ENOSPACE = -6    /* the block pool has too few free blocks (nothing was changed) */
} q4kv_status;

/* Type of the stored scale and bias values (both 16 bits wide, so layouts and byte counts do not change). */
typedef enum {
    Q4KV_PARAMS_F16 = 0,  /* IEEE binary16 */
    Q4KV_PARAMS_BF16 = 1  /* bfloat16 */
} q4kv_param_format;

/* Shape descriptor of one model's cache: the paper's ModelCacheSpec (Sec. 3.1, and
 * Sec. 3.6 for v_dim != k_dim).  The library reads nothing model-specific beyond it. */
typedef struct {
    int32_t num_layers;
    int32_t num_q_heads;
    int32_t num_kv_heads;   /* divides num_q_heads; query head h reads KV head h / (num_q_heads/num_kv_heads) */
    int32_t k_dim;          /* multiple of 64 */
    int32_t v_dim;          /* multiple of 64 */
    int32_t v_aliases_k;    /* 1: a token's V row is the first v_dim elements of its K row (one shared
                               latent per token); the V pool argument must then be NULL */
    int32_t block_tokens;   /* 256, the paper's block size (Sec. 3.1) */
    int32_t group_size;     /* 64 */
    int32_t param_format;   /* q4kv_param_format of every pool used with this spec */
} q4kv_spec;

/* One paged Q4 pool (K or V) for all layers, device memory, row-major:
 *   codes [num_layers][num_blocks][num_kv_heads][block_tokens][dim/8]   uint32
 *   scale [num_layers][num_blocks][num_kv_heads][block_tokens][dim/64]  binary16 (or bfloat16) bits
 *   bias  same shape as scale
 * All three base pointers must be 16-byte aligned.  A block id indexes the second axis;
 * an agent owns the blocks its block-table row lists (Sec. 3.1, per-agent isolation). */
typedef struct {
    uint32_t *codes;
    uint16_t *scale;
    uint16_t *bias;
    int32_t num_blocks;
} q4kv_pool;

/* Sec. 3.2, the "save" half of the codec.  Quantize `rows` rows of `dim` binary16 values.
 *   x      device, [rows][dim], 16-byte aligned
 *   codes  device out, [rows][dim/8]; scale, bias device out, [rows][dim/64]
 * Bit-exact with the definition above.  rows == 0 is a no-op.  dim % 64 != 0 -> Q4KV_ESHAPE. */
int q4kv_quantize(const uint16_t *x, int64_t rows, int32_t dim, uint32_t *codes, uint16_t *scale, uint16_t *bias,
                  void *hip_stream);

/* Sec. 3.2 / Sec. 4.4 (the dequantization cost on restore): x_hat = code*scale + bias in
 * binary32, rounded to binary16.  Arguments mirror q4kv_quantize; x is the device output. */
int q4kv_dequantize(const uint32_t *codes, const uint16_t *scale, const uint16_t *bias, int64_t rows, int32_t dim,
                    uint16_t *x, void *hip_stream);

/* The two calls above with the type of scale and bias chosen by `param_format` (a q4kv_param_format; anything
 * else -> Q4KV_EINVAL).  Q4KV_PARAMS_F16 is exactly q4kv_quantize / q4kv_dequantize. */
int q4kv_quantize_fmt(const uint16_t *x, int64_t rows, int32_t dim, int32_t param_format, uint32_t *codes,
                      uint16_t *scale, uint16_t *bias, void *hip_stream);
int q4kv_dequantize_fmt(const uint32_t *codes, const uint16_t *scale, const uint16_t *bias, int64_t rows, int32_t dim,
                        int32_t param_format, uint16_t *x, void *hip_stream);

/* Sec. 3.4, first half of update_and_fetch: quantize new K/V rows and store them behind
 * each agent's cached tokens.
 *   k_new, v_new    device, [layer_end-layer_begin][num_agents][chunk_len][num_kv_heads][dim] binary16
 *                   (v_new and v must be NULL when spec->v_aliases_k)
 *   block_table     device int32 [num_agents][max_blocks]; entry i of a row is the physical block that
 *                   holds tokens 256*i .. 256*i+255 of that agent; it must already list the blocks the
 *                   new tokens fall into
 *   seq_len_before  device int32 [num_agents], tokens cached before this call
 * Token seq_len_before[a]+c of agent a receives chunk row c.  A token whose table slot is beyond
 * max_blocks or whose block id is outside the pool is skipped (nothing is written for it).
 * chunk_len > Q4KV_MAX_CHUNK_LEN -> Q4KV_ERANGE (the kernel places rows with quotients that are exact up
 * to there); longer chunks are appended in pieces. */
#define Q4KV_MAX_CHUNK_LEN (1 << 20)
int q4kv_append(const q4kv_spec *spec, const q4kv_pool *k, const q4kv_pool *v, const uint16_t *k_new,
                const uint16_t *v_new, const int32_t *block_table, int32_t max_blocks,
                const int32_t *seq_len_before, int32_t num_agents, int32_t chunk_len, int32_t layer_begin,
                int32_t layer_end, void *hip_stream);

/* Sec. 3.4, second half of update_and_fetch, and Sec. 3.6 (GQA grouping, causal chunk masks):
 * out = softmax(sm_scale * q K_hat^T) V_hat per agent, layer and query head, directly on the Q4
 * pools (nothing is dequantized to memory).
 *   q            device, [layer_end-layer_begin][num_agents][q_len][num_q_heads][k_dim] binary16
 *   out          device out, same leading shape, v_dim wide, binary16
 *   seq_len      device int32 [num_agents]: keys visible to the LAST query row of each agent, the
 *                appended chunk included; row r sees the first seq_len[a] - (q_len-1-r) tokens
 *                (q_len == 1: decode).  A row with no visible key yields zeros.
 *   max_seq_len  host upper bound of seq_len[]; it sizes the launch.  seq_len values above it are
 *                clamped to it on the device.  max_seq_len > max_blocks*256 -> Q4KV_ERANGE.
 *   window       <= 0: global attention.  > 0: row at position p also requires t > p - window
 *                (sliding-window layers, Sec. 3.6).
 *   split_tokens smallest token range handed to one wavefront (multiple of 256), 0 = library picks.  The
 *                tokens of all (layer, KV head, agent) units are dealt out evenly over a fixed set of
 *                wavefronts; this is the floor of a wavefront's share and bounds the partial results kept
 *                per query head.  Must equal the value given to q4kv_attention_workspace_bytes.
 *   workspace    device scratch of at least q4kv_attention_workspace_bytes(...) bytes, 16-byte aligned;
 *                contents before and after the call are unspecified.
 * Per-agent isolation (Sec. 3.1): nothing an agent's table row does not list up to seq_len ever enters its result,
 * and the kernels read no block the row does not list: slots past seq_len that a tile's loads touch lie in the
 * agent's own last block, and a block id outside [0, num_blocks) is skipped (its tokens count as masked; the loads
 * go to the agent's own first block instead, or to block 0 if that id is outside the pool too, and are discarded).
 * Outputs are run-to-run bit-identical for identical arguments. */
int q4kv_batched_attention(const q4kv_spec *spec, const q4kv_pool *k, const q4kv_pool *v, const uint16_t *q,
                           uint16_t *out, const int32_t *block_table, int32_t max_blocks, const int32_t *seq_len,
                           int32_t num_agents, int32_t q_len, int32_t max_seq_len, float sm_scale, int32_t window,
                           int32_t split_tokens, int32_t layer_begin, int32_t layer_end, void *workspace,
                           size_t workspace_bytes, void *hip_stream);

/* Sec. 3.6 (models that interleave global and sliding-window layers): q4kv_batched_attention with one window per
 * layer of the call instead of a single one.
 *   window_per_layer  HOST int32 [layer_end - layer_begin], read before the call returns; entry i belongs to layer
 *                     layer_begin + i; <= 0: global attention on that layer.
 * At most 128 layers per call (more -> Q4KV_EINVAL; split the layer range).  Everything else, the workspace size
 * included, is as for q4kv_batched_attention.  On decode the tokens a window hides are never read. */
int q4kv_batched_attention_windows(const q4kv_spec *spec, const q4kv_pool *k, const q4kv_pool *v, const uint16_t *q,
                                   uint16_t *out, const int32_t *block_table, int32_t max_blocks,
                                   const int32_t *seq_len, int32_t num_agents, int32_t q_len, int32_t max_seq_len,
                                   float sm_scale, const int32_t *window_per_layer, int32_t split_tokens,
                                   int32_t layer_begin, int32_t layer_end, void *workspace, size_t workspace_bytes,
                                   void *hip_stream);

/* The decode step of a forward pass is one call per layer (the next layer's queries depend on this layer's output),
 * all with the same lengths, and then the small kernel that turns seq_len[] into the launch's work plan is a tenth of
 * every call.  These two entry points take it out of the loop (Sec. 3.4, the decode loop of a batch):
 *   q4kv_decode_plan                writes the plan for calls of `num_layers_in_call` layers with these lengths, this
 *                                   window (one for all layers, <= 0: global) and this split_tokens into `workspace`
 *   q4kv_batched_attention_planned  q4kv_batched_attention with q_len == 1 on a workspace prepared that way: no
 *                                   seq_len argument (the plan holds the lengths, clamped to max_seq_len), one kernel
 * Every argument the two share must be the same in both calls (the layer range may differ from call to call, its
 * length may not), and seq_len[] must not be relied on to have changed in between: the planned call attends to the
 * lengths the plan was made from.  A workspace may be used for any number of planned calls on one stream, one after
 * the other; when the lengths change (every decode step), plan again.  A workspace prepared for other arguments
 * makes the planned call do nothing (it is detected on the device; `out` is left as it was).  Shapes, workspace size,
 * error codes and results (bit-identical to q4kv_batched_attention with the same arguments) as described there. */
int q4kv_decode_plan(const q4kv_spec *spec, const int32_t *seq_len, int32_t num_agents, int32_t max_seq_len,
                     int32_t window, int32_t split_tokens, int32_t num_layers_in_call, void *workspace,
                     size_t workspace_bytes, void *hip_stream);
int q4kv_batched_attention_planned(const q4kv_spec *spec, const q4kv_pool *k, const q4kv_pool *v, const uint16_t *q,
                                   uint16_t *out, const int32_t *block_table, int32_t max_blocks, int32_t num_agents,
                                   int32_t max_seq_len, float sm_scale, int32_t window, int32_t split_tokens,
                                   int32_t layer_begin, int32_t layer_end, void *workspace, size_t workspace_bytes,
                                   void *hip_stream);

/* For callers that cannot allocate device memory or have none to hand over -- code recording a HIP graph, tight
 * serving loops that call once per layer, harnesses that forbid hipMalloc: q4kv_batched_attention with the decode
 * path's workspace (tile plan and partial results) taken from a fixed array of Q4KV_STATIC_SCRATCH_BYTES bytes that
 * the library's code object holds on every GPU it is loaded on, from the first use of the library on that GPU until
 * the process ends.  No workspace arguments; everything else, q and out (caller-owned device memory) included, is as
 * for q4kv_batched_attention, and the results are bit-identical to that call with the same split_tokens.
 *   - The call allocates nothing and frees nothing, on the device or through any library.  The first call on a
 *     device looks the array's address up once (with that device current, as for every call); make that first call
 *     outside a graph capture.
 *   - q4kv_attention_workspace_bytes(...) > Q4KV_STATIC_SCRATCH_BYTES -> Q4KV_EWORKSPACE, nothing is launched: pass
 *     fewer layers per call (one layer of every benchmark configuration fits: at most 11 MB) or a larger split_tokens.
 *   - Every call on a GPU shares that GPU's one array, which keeps the last call's contents (nothing in it has to
 *     start at zero that the call's own first kernel does not write): calls that overlap in time on one GPU, on
 *     different streams or from different threads, race on it and are not allowed.  Calls on one stream are ordered
 *     by the stream. */
#define Q4KV_STATIC_SCRATCH_BYTES (16u << 20)
int q4kv_batched_attention_static(const q4kv_spec *spec, const q4kv_pool *k, const q4kv_pool *v, const uint16_t *q,
                                  uint16_t *out, const int32_t *block_table, int32_t max_blocks,
                                  const int32_t *seq_len, int32_t num_agents, int32_t q_len, int32_t max_seq_len,
                                  float sm_scale, int32_t window, int32_t split_tokens, int32_t layer_begin,
                                  int32_t layer_end, void *hip_stream);

/* Bytes of workspace q4kv_batched_attention needs for these arguments.  0 on bad arguments (q4kv_last_error() then
 * holds a message) and for q_len > 1, where the chunk kernel keeps everything on chip and needs no workspace. */
size_t q4kv_attention_workspace_bytes(const q4kv_spec *spec, int32_t num_agents, int32_t q_len, int32_t max_seq_len,
                                      int32_t split_tokens, int32_t num_layers_in_call);

/* The split size the library would pick for split_tokens == 0 (0 on bad arguments). */
int32_t q4kv_default_split_tokens(const q4kv_spec *spec, int32_t num_agents, int32_t q_len, int32_t max_seq_len,
                                  int32_t num_layers_in_call);

/* Sec. 3.2 closed form: Q4 bytes (K and V, all layers) of `tokens` cached tokens:
 * layers * kv_heads * (k_dim + v_dim) * tokens * (1/2 + 4/64); v_dim counts 0 when V aliases K.
 * Negative on bad arguments. */
int64_t q4kv_cache_bytes(const q4kv_spec *spec, int64_t tokens);

/* Saving and restoring an agent's cache (Sec. 3.1 block pool; Sec. 3.2 "Q4 at rest"; appendix "safetensors Q4
 * Format": one tensor per layer, block and array, Q4 on disk exactly as in memory, so that a restore is a copy and
 * no prefill).  A block image is the contiguous form of `num_blocks` listed blocks of every layer of the spec:
 *   for layer l = 0 .. num_layers-1, for i = 0 .. num_blocks-1 (block block_ids[i]):
 *     K codes uint32 [kv_heads][256][k_dim/8], K scale binary16 [kv_heads][256][k_dim/64], K bias (same shape),
 *     V codes, V scale, V bias likewise with v_dim (absent when v_aliases_k)
 * i.e. the pool's own bytes of that (layer, block), array after array.  q4kv_block_image_bytes gives its size
 * (0 on bad arguments).  q4kv_export_blocks gathers pool -> image, q4kv_import_blocks scatters image -> pool
 * (into whatever blocks block_ids names now: a restored agent need not get its old blocks back).
 *   block_ids  device, int32 [num_blocks]; an id outside [0, pool.num_blocks) is skipped (its records are left
 *              untouched on export, nothing is written on import)
 *   image      device (or pinned host memory the GPU can address), 16-byte aligned, at least image_bytes long
 *              With the image in host memory the launch is kept small (the host link, not the chip, is the
 *              limit), so that it can run beside a decode step on another stream.
 * Enqueue on hip_stream, allocate nothing, never synchronise.  Q4KV_EWORKSPACE when image_bytes is too small. */
size_t q4kv_block_image_bytes(const q4kv_spec *spec, int32_t num_blocks);
int q4kv_export_blocks(const q4kv_spec *spec, const q4kv_pool *k, const q4kv_pool *v, const int32_t *block_ids,
                       int32_t num_blocks, void *image, size_t image_bytes, void *hip_stream);
int q4kv_import_blocks(const q4kv_spec *spec, const q4kv_pool *k, const q4kv_pool *v, const int32_t *block_ids,
                       int32_t num_blocks, const void *image, size_t image_bytes, void *hip_stream);

/* Sec. 3.1 "Block Pool with Per-Agent Isolation", host side: which 256-token block of the device pools belongs to
 * which agent.  Pure bookkeeping in HOST memory (no device call): a block id is either free or in exactly one agent's
 * list, so two agents can never share or overwrite a block (the paper's namespace isolation); the list order is the
 * token order, i.e. a row of the block table the attention calls read.  Eviction is the caller's sequence
 * lru_victim -> q4kv_export_blocks -> (file) -> release; a restore is reserve -> q4kv_import_blocks into whatever blocks
 * were free.  Agent ids are caller-chosen non-negative numbers.  Every call locks the pool (thread-safe).
 *   create        a pool over block ids 0 .. num_blocks-1, all free; NULL on a bad argument or out of memory
 *   reserve       make the agent own ceil(tokens/256) blocks: blocks it has stay (in place and order), missing ones
 *                 come from the free list, lowest id first; an unknown agent is created; the agent becomes the most
 *                 recently used.  Never shrinks.  Returns the number of blocks owned, Q4KV_ENOSPACE when the free
 *                 list is too short (nothing changed), Q4KV_EINVAL on a negative id or token count
 *   release       free all blocks of the agent and forget it; returns the number freed, Q4KV_EINVAL if unknown
 *   blocks        copy the agent's block ids in token order into ids[0 .. cap) (host); returns how many it owns
 *   table_row     the same as a block-table row: ids, then `fill` up to max_blocks; Q4KV_ERANGE if it owns more
 *   touch         mark the agent most recently used;  pin(1): never a victim while it is in a running batch
 *   lru_victim    the unpinned agent with at least one block that was used least recently, or -1
 *   free_blocks   length of the free list;  owner: the agent id that owns a block, or -1 */
typedef struct q4kv_block_pool q4kv_block_pool;
q4kv_block_pool *q4kv_block_pool_create(int32_t num_blocks);
void q4kv_block_pool_destroy(q4kv_block_pool *pool);
int32_t q4kv_block_pool_reserve(q4kv_block_pool *pool, int64_t agent_id, int64_t tokens);
int32_t q4kv_block_pool_release(q4kv_block_pool *pool, int64_t agent_id);
int32_t q4kv_block_pool_blocks(q4kv_block_pool *pool, int64_t agent_id, int32_t *ids, int32_t cap);
int32_t q4kv_block_pool_table_row(q4kv_block_pool *pool, int64_t agent_id, int32_t *row, int32_t max_blocks, int32_t fill);
int32_t q4kv_block_pool_touch(q4kv_block_pool *pool, int64_t agent_id);
int32_t q4kv_block_pool_pin(q4kv_block_pool *pool, int64_t agent_id, int32_t pinned);
int64_t q4kv_block_pool_lru_victim(q4kv_block_pool *pool);
int32_t q4kv_block_pool_free_blocks(q4kv_block_pool *pool);
int64_t q4kv_block_pool_owner(q4kv_block_pool *pool, int32_t block_id);

/* Measurement helper, no part of the method: a kernel that only reads.  Reads the first
 * floor(bytes / 16384) * 16384 bytes of the device buffer `src` (16-byte aligned) exactly once, in the launch
 * shape and with the load width of the decode kernel, and writes nothing except, possibly, the one device word
 * `sink` (its value means nothing).  Timing it gives the read bandwidth the memory system sustains, against which
 * the benchmark quotes the decode kernel next to the published peak.  Enqueues on hip_stream; no allocation, no
 * synchronisation.  Fewer than 16,384 bytes: nothing happens.  Q4KV_EINVAL on a NULL or misaligned pointer. */
int q4kv_read_probe(const void *src, size_t bytes, uint32_t *sink, void *hip_stream);

/* Message of this thread's most recent failing call ("" if none). */
const char *q4kv_last_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int q4kv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* Q4KV_H */

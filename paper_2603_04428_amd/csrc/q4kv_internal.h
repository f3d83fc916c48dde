// Internal launch interface between the C ABI (api.hip) and the kernel files.
// Every function only enqueues kernels on `stream` and returns the hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/q4kv.h"

namespace q4kv {

// bf16_params: scale and bias are bfloat16 bit patterns instead of binary16 ones; compute_units sizes the launch
hipError_t launch_quantize(const uint16_t *x, int64_t rows, int dim, bool bf16_params, uint32_t *codes, uint16_t *scale,
                           uint16_t *bias, int compute_units, hipStream_t stream);
hipError_t launch_dequantize(const uint32_t *codes, const uint16_t *scale, const uint16_t *bias, int64_t rows,
                             int dim, bool bf16_params, uint16_t *x, int compute_units, hipStream_t stream);
// v, v_new: null when the V rows alias the K rows
hipError_t launch_append(const q4kv_spec &spec, const q4kv_pool &k, const q4kv_pool *v, const uint16_t *k_new,
                         const uint16_t *v_new, const int32_t *block_table, int max_blocks,
                         const int32_t *seq_len_before, int num_agents, int chunk_len, int layer_begin, int layer_end,
                         int compute_units, hipStream_t stream);

struct AttentionArgs {
    q4kv_spec spec;
    q4kv_pool k, v;             // v == k when the V rows alias the K rows
    const uint16_t *q;
    uint16_t *out;
    const int32_t *block_table;
    const int32_t *seq_len;
    int max_blocks, num_agents, q_len, max_seq_len, window;
    const int32_t *layer_window; // host, [layers_in_call]: one window per layer of the call, or nullptr: `window` for all
    int split_tokens;           // smallest token range one wave takes (multiple of 256)
    int max_slots;              // partial records reserved per (layer, agent, query head)
    int grid_workgroups;        // workgroups of the attention launch (two per compute unit)
    int layer_begin, layers_in_call;
    float sm_scale;
    int32_t *plan;              // workspace: tile plan written by the plan kernel
    float *part_acc;            // workspace: [units][max_slots][v_dim]
    float *part_ml;             // workspace: [units][max_slots][2]  (running max in log2 units, denominator)
    int32_t *arrivals;          // workspace: [layers_in_call][kv_heads][num_agents] waves that have left a unit
    int plan_signature;         // hash of the arguments the plan depends on, kept in the plan and checked by the kernels
};

struct StreamParams;
struct MergeParams;
StreamParams stream_params(const AttentionArgs &a);
MergeParams merge_params(const AttentionArgs &a);
// workers: how many equal tile ranges the plan cuts the call into, each a multiple of per_multiple tiles long; needs
// split_tokens, plan, arrivals
hipError_t launch_plan(const AttentionArgs &a, int workers, int per_multiple, hipStream_t stream);

// true when a decode (q_len == 1) kernel exists for these head shapes
bool decode_supported(const q4kv_spec &spec);
int decode_waves_per_workgroup();
int decode_solo_quarter_tiles();   // smallest tile range a single wave of the GQA kernel takes for itself
size_t decode_plan_ints(int num_agents, int layers);
int max_window_layers();   // layers per call when every layer brings its own window
hipError_t launch_decode_plan(const AttentionArgs &a, hipStream_t stream);      // plan kernel for the GQA decode kernels
hipError_t launch_decode_attention(const AttentionArgs &a, hipStream_t stream); // needs the plan in the workspace

// shared-latent decode (V is a prefix of K, 16 query heads per latent head): its plan, and attention + combine
bool mla_decode_supported(const q4kv_spec &spec);
hipError_t launch_mla_decode_plan(const AttentionArgs &a, hipStream_t stream);
hipError_t launch_mla_decode_attention(const AttentionArgs &a, hipStream_t stream);

// true when a chunk (q_len > 1, causal) kernel exists for these head shapes
bool chunk_supported(const q4kv_spec &spec);
hipError_t launch_chunk_attention(const AttentionArgs &a, hipStream_t stream);

// persist.hip: bytes of one (layer, block) record of a block image; gather (to_image) or scatter of `num_blocks`
// listed blocks of every layer between the pools and the image (v: null when V aliases K)
size_t image_record_bytes(const q4kv_spec &s);
hipError_t launch_image_copy(const q4kv_spec &s, const q4kv_pool &k, const q4kv_pool *v, const int32_t *block_ids,
                             int num_blocks, void *image, bool to_image, int workgroups_when_on_device,
                             hipStream_t stream);

// read_probe.hip: reads bytes / 16,384 * 16,384 bytes of `src` once; `sink` is one device word that may be written
hipError_t launch_read_probe(const void *src, size_t bytes, uint32_t *sink, int workgroups, hipStream_t stream);

} // namespace q4kv

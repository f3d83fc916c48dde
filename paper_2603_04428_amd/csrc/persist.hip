// Block images: an agent's cache blocks gathered from the pools into one contiguous buffer (and scattered back),
// the device half of saving a cache to disk and restoring it (Sec. 3.1 block pool, Sec. 3.2 "Q4 at rest", the
// appendix "safetensors Q4 Format": one tensor per layer, block and array).
//
// Image layout: for layer l = 0 .. layers-1, for the i-th listed block: K codes [kv_heads][256][k_dim/8] uint32,
// K scale [kv_heads][256][k_dim/64] binary16, K bias (same), then V codes, V scale, V bias (absent when V aliases
// K).  Every piece is one contiguous run of the pool (layout [layer][block][kv_head][256][..]), a multiple of 16
// bytes long, so both directions are a batched copy: one workgroup column per piece, 16 bytes per lane and step.
#include "q4_device.h"
#include "q4kv_internal.h"

namespace q4kv {
namespace {

constexpr int kCopyThreads = 256;
constexpr int kPieces = 6;

struct ImageParams {
    unsigned char *pool[kPieces];   // K codes, K scale, K bias, V codes, V scale, V bias (V entries unused if aliased)
    long long piece_bytes[kPieces]; // bytes of one (layer, block) of each array
    long long piece_off[kPieces];   // offset of each piece inside a (layer, block) record of the image
    long long record_bytes;         // one (layer, block) record of the image
    const int32_t *block_ids;       // device, [num_blocks]
    unsigned char *image;
    int pieces, num_blocks, pool_blocks, layers;
};

// A record is cut into chunks of kChunkBytes (the last one may be short); workgroups stride over all (record, chunk)
// items and every lane moves 16 bytes of whatever piece its offset falls into.  TO_IMAGE: pool -> image, else
// image -> pool.  A block id outside the pool is skipped (export leaves that record untouched, import writes
// nothing).
constexpr int kChunkBytes = kCopyThreads * 16;

template <bool TO_IMAGE>
__global__ __launch_bounds__(kCopyThreads) void image_copy_kernel(ImageParams p)
{
    const long long chunks_per_record = (p.record_bytes + kChunkBytes - 1) / kChunkBytes;
    const long long items = (long long)p.layers * p.num_blocks * chunks_per_record;
    const int generation = blockIdx.x / max(1u, gridDim.x / 8); // the device launch stacks eight workgroups per compute unit
    for (long long item = blockIdx.x; item < items; item += gridDim.x) {
        rotate_wave_priority(generation);
        const long long rec = item / chunks_per_record;
        const long long off = (item % chunks_per_record) * kChunkBytes + threadIdx.x * 16; // inside the record
        const int l = (int)(rec / p.num_blocks), i = (int)(rec % p.num_blocks);
        const int blk = p.block_ids[i];
        if (blk < 0 || blk >= p.pool_blocks || off >= p.record_bytes) continue;
        int piece = 0;
#pragma unroll
        for (int k = 1; k < kPieces; ++k)
            if (k < p.pieces && off >= p.piece_off[k]) piece = k;
        typedef uint32_t u4_t __attribute__((ext_vector_type(4)));
        u4_t *pool = reinterpret_cast<u4_t *>(p.pool[piece] + ((long long)l * p.pool_blocks + blk) * p.piece_bytes[piece] +
                                              (off - p.piece_off[piece]));
        u4_t *img = reinterpret_cast<u4_t *>(p.image + rec * p.record_bytes + off);
        // the stores say that the line will not be read again soon (as in the dequantize kernel)
        if (TO_IMAGE) __builtin_nontemporal_store(*pool, img); else __builtin_nontemporal_store(*img, pool);
    }
}

} // namespace

size_t image_record_bytes(const q4kv_spec &s)
{
    const size_t rows = (size_t)s.num_kv_heads * kBlockTokens;
    size_t n = rows * (s.k_dim / 8) * 4 + 2 * rows * (s.k_dim / kGroup) * 2;
    if (!s.v_aliases_k) n += rows * (s.v_dim / 8) * 4 + 2 * rows * (s.v_dim / kGroup) * 2;
    return n;
}

hipError_t launch_image_copy(const q4kv_spec &s, const q4kv_pool &k, const q4kv_pool *v, const int32_t *block_ids,
                             int num_blocks, void *image, bool to_image, int workgroups_when_on_device,
                             hipStream_t stream)
{
    ImageParams p;
    const long long rows = (long long)s.num_kv_heads * kBlockTokens;
    const long long kc = rows * (s.k_dim / 8) * 4, kg = rows * (s.k_dim / kGroup) * 2;
    const long long vc = rows * (s.v_dim / 8) * 4, vg = rows * (s.v_dim / kGroup) * 2;
    p.pool[0] = reinterpret_cast<unsigned char *>(k.codes);
    p.pool[1] = reinterpret_cast<unsigned char *>(k.scale);
    p.pool[2] = reinterpret_cast<unsigned char *>(k.bias);
    p.piece_bytes[0] = kc; p.piece_bytes[1] = kg; p.piece_bytes[2] = kg;
    p.pieces = 3;
    for (int i = 3; i < kPieces; ++i) { p.pool[i] = nullptr; p.piece_bytes[i] = 0; }
    if (v) {
        p.pool[3] = reinterpret_cast<unsigned char *>(v->codes);
        p.pool[4] = reinterpret_cast<unsigned char *>(v->scale);
        p.pool[5] = reinterpret_cast<unsigned char *>(v->bias);
        p.piece_bytes[3] = vc; p.piece_bytes[4] = vg; p.piece_bytes[5] = vg;
        p.pieces = 6;
    }
    long long off = 0;
    for (int i = 0; i < kPieces; ++i) { p.piece_off[i] = off; off += p.piece_bytes[i]; }
    p.record_bytes = off;
    p.block_ids = block_ids;
    p.image = static_cast<unsigned char *>(image);
    p.num_blocks = num_blocks;
    p.pool_blocks = k.num_blocks;
    p.layers = s.num_layers;
    if (num_blocks == 0) return hipSuccess;
    // every piece is a multiple of 512 bytes (256 tokens x 2 bytes x heads x groups), hence of a lane's 16
    const long long items = (long long)s.num_layers * num_blocks * ((p.record_bytes + kChunkBytes - 1) / kChunkBytes);
    // An image in host memory is read or written across the host link at a few tens of GB/s: a small launch
    // saturates it and leaves the compute units to whatever else runs (a launch of thousands of workgroups
    // waiting on the link would hold every slot of the chip and stall a concurrent decode step).
    hipPointerAttribute_t attr;
    bool host_image = false;
    if (hipPointerGetAttributes(&attr, image) == hipSuccess)
        host_image = attr.type == hipMemoryTypeHost;
    else
        (void)hipGetLastError();
    const long long cap = host_image ? 64 : (long long)workgroups_when_on_device;
    const unsigned grid = (unsigned)(items < cap ? items : cap);
    if (to_image)
        hipLaunchKernelGGL(image_copy_kernel<true>, dim3(grid), dim3(kCopyThreads), 0, stream, p);
    else
        hipLaunchKernelGGL(image_copy_kernel<false>, dim3(grid), dim3(kCopyThreads), 0, stream, p);
    {
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

} // namespace q4kv

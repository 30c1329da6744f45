// Internal declarations shared by the host entry points and the kernel launchers of libcq.
// Nothing here is part of the public ABI (see include/libcq.h for that).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "libcq.h"

namespace cq {

constexpr int kTileTokens = CQ_TILE_TOKENS;   // tokens per cache tile == lanes per wavefront
constexpr int kTabWords = 64;                 // 4-byte words per lookup-table row (b = 8)
constexpr int kPartialHeader = 2;             // running max and sum in front of each partial

struct Derived {
    int c, b, head_dim, n_kv_heads;
    int gh;            // groups per head
    int k;             // centroids per group
    int channels;      // n_kv_heads * head_dim
    int groups;        // channels / c
    int bpth;          // code bytes per token-head
    int tile_bytes;    // 64 * bpth
    // sub-byte formats (b = 2, 4; derive_any only): `fuse` = 8 / b neighbouring groups share a code
    // byte, and everything above describes the fused format CQ-<c fuse>c8b whose cache layout
    // they use; sub_c / sub_b are the format's own c and b.  fuse = 1 otherwise.
    int fuse, sub_c, sub_b;
};

// Host-side format check shared by the entry points: formats with decode kernels (b = 8, 10).
cq_status derive(const cq_format* fmt, Derived* out);
// ... and also the sub-byte formats, which only cq_encode*, the size functions and
// cq_expand_codebook take (they are decoded through their fused format).
cq_status derive_any(const cq_format* fmt, Derived* out);

// Where the 64-token tiles of a packed cache live.  Contiguous: [sequence][kv head][tile] with
// t_cap / 64 tiles per stream.  Paged: a pool of pages, a page being one tile of every KV head
// ([page][kv head][tile bytes]), and block_table[n * bt_stride + tile] names the page of tile
// `tile` of sequence n (entries are clamped to the pool, so a bad table cannot cause a fault).
struct CacheMap {
    const int32_t* block_table;   // null: contiguous
    int64_t bt_stride;
    int n_pages;
    int tiles_cap;                // contiguous: t_cap / 64
    int n_kv_heads;

    __device__ __forceinline__ int page(int n, int tile) const
    {
        const int p = block_table[(size_t)n * bt_stride + tile];
        return p < 0 ? 0 : (p >= n_pages ? n_pages - 1 : p);
    }
    // index of the tile in units of tile bytes
    __device__ __forceinline__ size_t tile_index(int n, int hkv, int tile) const
    {
        if (block_table) return (size_t)page(n, tile) * n_kv_heads + hkv;
        return (size_t)(n * n_kv_heads + hkv) * tiles_cap + tile;
    }
};

// One or two tensors (K alone, or K and V of the same shape) encoded by one launch.
struct EncodeTensor {
    const uint16_t* x;
    int64_t x_batch_stride, x_row_stride;
    const uint16_t* centroids;
    uint8_t* codes;
};

struct EncodeArgs {
    EncodeTensor tensor[2];
    int n_tensors;
    int batch, t_new, t_offset;
    CacheMap map;
    Derived f;
};

// One layer's tensors of a layer-batched decode step (mirrors cq_layer_io; lives in device memory).
struct LayerPtrs {
    const uint16_t* q;
    const uint16_t* xk_new;
    const uint16_t* xv_new;
    uint8_t* k_codes;
    uint8_t* v_codes;
    const uint16_t* k_centroids;
    const uint16_t* v_centroids;
    uint16_t* out;
};

// Up to N records passed by value to the kernel that writes them into the device table.
struct LayerChunk {
    static constexpr int N = 32;
    LayerPtrs p[N];
};

struct DecodeArgs {
    const uint16_t* q;
    const uint8_t* k_codes;
    const uint8_t* v_codes;
    const uint16_t* k_centroids;
    const uint16_t* v_centroids;
    float scale_log2e;        // scale * log2(e): scores are kept in the base-2 domain
    int batch, n_q_heads, t;
    CacheMap map;
    const int32_t* seq_lens;
    // fused decode step (null xk_new = plain attention): the new token's key / value rows,
    // fp16 [batch][D] with row stride x_new_stride (elements); the caches are then written too
    const uint16_t* xk_new;
    const uint16_t* xv_new;
    int64_t x_new_stride;
    int tiles_per_split, n_split;
    float* partials;          // [batch][n_q_heads][n_split][2 + head_dim]
    uint16_t* out;
    // q and out are [batch][n_q_heads][head_dim] with these batch strides (elements); sequence n
    // attends to min(max(seq_lens[n] - seq_len_shift, seq_len_floor), t) tokens.  (Other than
    // n_q_heads * head_dim, 0 and 1 only where a chunk of query tokens is served token by token.)
    int64_t q_batch_stride, out_batch_stride;
    int seq_len_shift, seq_len_floor;
    // layer-batched launch (null: one layer): workgroup blockIdx / wgs_per_layer serves layer
    // layers[...], whose pointers replace q, xk_new, xv_new, the caches, the codebooks and out;
    // its partials follow those of the layers before it
    const LayerPtrs* layers;
    int n_layers, wgs_per_layer;
    // arrival counters of the in-kernel merge, one per (sequence, query head) row (set by the
    // launcher; null: the partials are merged by a kernel of their own)
    unsigned* merge_counters;
    Derived f;
};

// Causal attention of the last m tokens of every sequence over its cache (cq_chunk.hip).
struct ChunkArgs {
    const uint16_t* q;        // fp16 [batch][m][n_q_heads][head_dim]
    const uint8_t* k_codes;
    const uint8_t* v_codes;
    const uint16_t* k_centroids;
    const uint16_t* v_centroids;
    float scale_log2e;
    int batch, m, n_q_heads, t;
    CacheMap map;
    const int32_t* seq_lens;
    int tiles_per_split, n_split;
    float* partials;          // [batch][m][n_q_heads][n_split][2 + head_dim]
    uint16_t* out;            // fp16 [batch][m][n_q_heads][head_dim]
    // keys cached before the rotary position embedding (null: keys are used as stored): the two
    // parts of the table of cq_rope_table, cos / sin of (64 tile theta_i) and of (lane theta_i)
    const float2* rope_tile_tab;
    const float2* rope_lane_tab;
    Derived f;
};
int chunk_rows_per_workgroup(int rows_per_kv_head);
cq_status launch_chunk_attention(const ChunkArgs& a, hipStream_t stream);

// Largest tokens_per_split the decode kernel's on-chip score buffer can hold.
int decode_max_tiles_per_split(const Derived& f);

struct DequantArgs {
    const uint8_t* codes;
    const uint16_t* centroids;
    uint16_t* out;            // fp16 [batch][t_count][D]
    int64_t out_batch_stride, out_row_stride;
    int batch, t_offset, t_count;
    CacheMap map;
    Derived f;
};
cq_status launch_dequantize(const DequantArgs& a, hipStream_t stream);

// Centroid learning: k-means++ (do_init) or given starting centroids, then n_iter Lloyd iterations.
struct KMeansArgs {
    const uint16_t* x;        // fp16 [n][D]
    int64_t x_row_stride;
    const float* weights;     // fp32 [n][G] or null
    int n, n_iter;
    const uint64_t* rnd;      // [G][K] random words (k-means++)
    bool do_init;
    const float* cent_in;     // fp32 [G][K][c] starting centroids when !do_init
    int32_t* picks;           // [G][K] out, optional
    uint16_t* cent16_out;     // fp16 [G][K][c] out, optional
    float* cent32_out;        // fp32 [G][K][c] out, optional
    uint16_t* assign_out;     // [G][n] out, optional
    Derived f;
};
struct KMeansWorkspace {
    uint16_t* xg;             // fp16 [G][n][c]: the tokens, group-major
    uint32_t* wq;             // [G][n] integer weights
    float* dmin;              // [G][n] distance to the nearest chosen centre
    uint16_t* assign;         // [G][n]
    float* cent;              // fp32 [G][K][c]
    unsigned* wmax_bits;      // [G]
};
// Carves `base` (null: sizes only) into the workspace arrays; returns the bytes needed.
size_t kmeans_workspace_layout(const Derived& f, int n, void* base, KMeansWorkspace* ws);
cq_status launch_kmeans(const KMeansArgs& a, void* workspace, hipStream_t stream);

cq_status launch_encode(const EncodeArgs& a, hipStream_t stream);
// many tokens per sequence: the MFMA-filtered kernel (cq_encode_mfma.hip)
cq_status launch_encode_tiles(const EncodeArgs& a, hipStream_t stream);
cq_status launch_decode(const DecodeArgs& a, hipStream_t stream);
// centroids fp16 [G][2^b][c] of a sub-byte format -> fp16 [G / fuse][256][c fuse] of its fused format
cq_status launch_expand_codebook(const uint16_t* centroids, const Derived& f, uint16_t* fused, hipStream_t stream);
// writes `count` records of a layer table (device memory) from values passed with the launch
cq_status launch_layer_table_write(const LayerChunk& chunk, int count, LayerPtrs* dst, hipStream_t stream);
// merges the partials of `rows` (sequence, query head) pairs, n_split each, into fp16 rows
// (row r goes to out + (r / n_q_heads) * out_batch_stride + (r % n_q_heads) * head_dim)
cq_status launch_decode_merge(const float* partials, uint16_t* out, int rows, int n_q_heads, int64_t out_batch_stride,
                              int n_split, int head_dim, hipStream_t stream);

// Keys cached before the rotary position embedding (cq_decode_rope.hip).  The table holds, for
// head_dim 128, cos / sin of (64 * tile) * theta_i for every tile of `positions` tokens, then
// cos / sin of u * theta_i for u < 64 (theta_i = base^(-2i/128), i < 64).
size_t rope_table_floats(int positions);
cq_status launch_rope_table(double base, int positions, float* table, hipStream_t stream);
int decode_rope_max_tiles_per_split();
int decode_rope_shared_max_tiles_per_split();
cq_status launch_decode_rope(const DecodeArgs& a, const float* table, int positions, hipStream_t stream);

// Kernels that address their dynamic LDS block from LDS address 0 and use more than 64 KB of it:
// once per device (kernel attributes are kept per device) check that no static LDS precedes the
// block and raise the kernel's dynamic LDS limit to the 160 KB of a gfx950 CU.  One object per
// kernel instantiation (a function-local static of the launcher).
struct LdsKernelSetup {
    static constexpr int kMaxDevices = 64;
    std::once_flag once[kMaxDevices];
    hipError_t result[kMaxDevices];
    hipError_t ensure(const void* kernel)
    {
        int dev = 0;
        const hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
        std::call_once(once[dev], [&] {
            hipFuncAttributes attr;
            hipError_t r = hipFuncGetAttributes(&attr, kernel);
            if (r == hipSuccess && attr.sharedSizeBytes != 0) r = hipErrorInvalidValue;
            if (r == hipSuccess) r = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            result[dev] = r;
        });
        return result[dev];
    }
};

}  // namespace cq

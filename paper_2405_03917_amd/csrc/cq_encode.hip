// Nearest-centroid encoding of key/value activations (Section 3.2 of the paper) for gfx950.
//
// Two kernels, picked by the number of new tokens per sequence:
//   encode_mfma_kernel       (prefill: 32 tokens or more; cq_encode_mfma.hip)  scores 32 tokens x
//       32 centroids per MFMA, keeps the two best, and re-does the near ties by the direct form.
//   encode_centroids_kernel  (decode step: a handful of tokens; here)  16 lanes per token.  A
//       workgroup takes one group and up to 16 tokens; each lane scans every 16th centroid and
//       the 16 lanes of a token reduce their (distance, index) pairs.
// The direct form is sum_i (x_i - c_i)^2 in fp32 with one fused multiply-add per channel, in
// channel order, ties broken towards the lowest index.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "cq_internal.hpp"

namespace cq {
namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

template <int C>
__device__ __forceinline__ void load_halfs(const uint16_t* p, float (&v)[C])
{
    if constexpr (C == 8) {
        const uint4 a = *reinterpret_cast<const uint4*>(p);
        const unsigned w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const half2_t h = __builtin_bit_cast(half2_t, w[i]);
            v[2 * i] = (float)h.x;
            v[2 * i + 1] = (float)h.y;
        }
    } else if constexpr (C == 4) {
        const uint2 a = *reinterpret_cast<const uint2*>(p);
        const half2_t h0 = __builtin_bit_cast(half2_t, a.x), h1 = __builtin_bit_cast(half2_t, a.y);
        v[0] = (float)h0.x; v[1] = (float)h0.y; v[2] = (float)h1.x; v[3] = (float)h1.y;
    } else {
        static_assert(C == 2, "channels per group must be 2, 4 or 8");
        const unsigned a = *reinterpret_cast<const unsigned*>(p);
        const half2_t h = __builtin_bit_cast(half2_t, a);
        v[0] = (float)h.x; v[1] = (float)h.y;
    }
}

template <int C>
__device__ __forceinline__ float sq_dist(const float (&x)[C], const float (&c)[C])
{
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < C; ++i) {
        const float d = x[i] - c[i];
        acc = __builtin_fmaf(d, d, acc);
    }
    return acc;
}

// ------------------------------------------------------------------------------------------
// a handful of tokens: 16 lanes per token
// ------------------------------------------------------------------------------------------
constexpr int kSmallTokens = 16;     // tokens per workgroup

// One workgroup = one group x up to 16 tokens.  Token i of the chunk is served by lanes
// 16 i .. 16 i + 15; lane r of those scans centroids r, r + 16, r + 32, ... in ascending order,
// then the 16 lanes reduce their (distance, index) pairs.  No LDS, no barrier.
template <int GH, int C, int B>
__global__ __launch_bounds__(256) void encode_centroids_kernel(EncodeArgs a)
{
    constexpr int K = 1 << B;
    constexpr int PER_LANE = K / 16;
    constexpr int TILE_LOW = kTileTokens * GH;
    constexpr int TILE_BYTES = kTileTokens * GH * B / 8;

    const int tid = threadIdx.x;
    const int r = tid & 15;
    const int g_abs = blockIdx.x;
    const EncodeTensor& ten = a.tensor[blockIdx.z];
    const int total = a.batch * a.t_new;
    const int tt = blockIdx.y * kSmallTokens + (tid >> 4);
    const bool valid = tt < total;
    const int n = valid ? tt / a.t_new : 0, t = valid ? tt % a.t_new : 0;

    float x[C];
    load_halfs<C>(ten.x + (size_t)n * ten.x_batch_stride + (size_t)t * ten.x_row_stride + (size_t)g_abs * C, x);
    const uint16_t* cen = ten.centroids + ((size_t)g_abs * K + r) * C;

    // d >= +0, so its bit pattern orders like the value; the index in the low word makes the
    // minimum pick the lowest index among equal distances
    unsigned long long key = ~0ull;
#pragma unroll 16
    for (int k = 0; k < PER_LANE; ++k) {
        float c[C];
        load_halfs<C>(cen + (size_t)k * 16 * C, c);
        const float d = sq_dist<C>(x, c);
        const unsigned long long kk = ((unsigned long long)__float_as_uint(d) << 32) | (unsigned)(k * 16 + r);
        key = kk < key ? kk : key;
    }
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) {
        const unsigned long long other = __shfl_xor(key, o, 16);
        key = other < key ? other : key;
    }
    if (r == 0 && valid) {
        const unsigned code = (unsigned)(key & 0xffffffffu);
        const int pos = a.t_offset + t;
        const int u = pos & (kTileTokens - 1);
        const int hkv = g_abs / GH, g = g_abs % GH;
        const int slot = (g - u) & (GH - 1);
        uint8_t* tile = ten.codes + a.map.tile_index(n, hkv, pos / kTileTokens) * TILE_BYTES;
        tile[(slot >> 4) * 1024 + u * 16 + (slot & 15)] = (uint8_t)(code & 0xff);
        if constexpr (B == 10) {
            // the high bits of a token's 16 codes share one word that other workgroups update too
            unsigned* hw = reinterpret_cast<unsigned*>(tile + TILE_LOW + u * 4);
            atomicAnd(hw, ~(3u << (2 * slot)));
            atomicOr(hw, (code >> 8) << (2 * slot));
        }
    }
}

template <int GH, int C, int B>
cq_status launch_format(const EncodeArgs& a, hipStream_t stream)
{
    if (a.t_new < 32) {
        const int total = a.batch * a.t_new;
        dim3 grid((unsigned)a.f.groups, (unsigned)((total + kSmallTokens - 1) / kSmallTokens), (unsigned)a.n_tensors);
        hipLaunchKernelGGL((encode_centroids_kernel<GH, C, B>), grid, dim3(256), 0, stream, a);
    } else {
        return launch_encode_tiles(a, stream);
    }
    if (hipGetLastError() != hipSuccess) return CQ_ERR_HIP;
    return CQ_OK;
}

// ------------------------------------------------------------------------------------------
// dequantize: code -> centroid (the inverse lookup of Section 2.2 / "CQ(A)" of Eq. 5)
// ------------------------------------------------------------------------------------------
// One workgroup = one 64-token tile of one (sequence, KV head): the tile's bytes go through LDS
// (one coalesced read), then every thread writes 16-byte pieces of the fp16 rows: piece q of
// token u covers channels 8 q .. 8 q + 7 of the head, i.e. 8 / C consecutive groups.
template <int GH, int C, int B>
__global__ __launch_bounds__(256) void dequantize_kernel(DequantArgs a)
{
    constexpr int K = 1 << B;
    constexpr int TILE_LOW = kTileTokens * GH;
    constexpr int TILE_BYTES = kTileTokens * GH * B / 8;
    constexpr int GPP = 8 / C;                      // groups per 16-byte piece
    constexpr int PIECES = GH * C / 8;              // pieces per token-head
    __shared__ __attribute__((aligned(16))) uint8_t tb[TILE_BYTES];

    const int tid = threadIdx.x;
    const int first_tile = a.t_offset / kTileTokens;
    const int tile = first_tile + blockIdx.x, hkv = blockIdx.y, n = blockIdx.z;
    const uint8_t* src = a.codes + a.map.tile_index(n, hkv, tile) * TILE_BYTES;
    for (int i = tid; i < TILE_BYTES / 16; i += 256)
        reinterpret_cast<uint4*>(tb)[i] = reinterpret_cast<const uint4*>(src)[i];
    __syncthreads();

    const int t_end = a.t_offset + a.t_count;
    for (int e = tid; e < kTileTokens * PIECES; e += 256) {
        const int u = e / PIECES, q = e % PIECES;
        const int pos = tile * kTileTokens + u;
        if (pos < a.t_offset || pos >= t_end) continue;
        unsigned w[4];
#pragma unroll
        for (int k = 0; k < GPP; ++k) {
            const int g = q * GPP + k;
            const int slot = (g - u) & (GH - 1);
            unsigned code = tb[(slot >> 4) * 1024 + u * 16 + (slot & 15)];
            if constexpr (B == 10) {
                const unsigned hi = *reinterpret_cast<const unsigned*>(tb + TILE_LOW + u * 4);
                code |= ((hi >> (2 * slot)) & 3u) << 8;
            }
            const uint16_t* cen = a.centroids + ((size_t)(hkv * GH + g) * K + code) * C;
#pragma unroll
            for (int i = 0; i < C / 2; ++i) w[k * (C / 2) + i] = *reinterpret_cast<const unsigned*>(cen + 2 * i);
        }
        uint16_t* dst = a.out + (size_t)n * a.out_batch_stride + (size_t)(pos - a.t_offset) * a.out_row_stride +
                        (size_t)hkv * GH * C + q * 8;
        *reinterpret_cast<uint4*>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

template <int GH, int C, int B>
cq_status launch_dequant_format(const DequantArgs& a, hipStream_t stream)
{
    const int first_tile = a.t_offset / kTileTokens;
    const int last_tile = (a.t_offset + a.t_count - 1) / kTileTokens;
    dim3 grid((unsigned)(last_tile - first_tile + 1), (unsigned)a.f.n_kv_heads, (unsigned)a.batch);
    hipLaunchKernelGGL((dequantize_kernel<GH, C, B>), grid, dim3(256), 0, stream, a);
    return hipGetLastError() == hipSuccess ? CQ_OK : CQ_ERR_HIP;
}

// ------------------------------------------------------------------------------------------
// sub-byte formats (b = 2, 4; the CQ-<c>c<b>b variants of the paper's ablation on coupled channels)
// ------------------------------------------------------------------------------------------
// 8 / b neighbouring groups share one code byte (group i of the byte in bits [b i, b i + b)), and
// the byte is stored where the fused format CQ-<c 8/b>c8b stores its code, so every decode kernel
// reads these caches with the expanded codebook of expand_codebook_kernel.  The search itself is
// the format's own: each group against its 2^b centroids, squared distance in fp32 in channel
// order, lowest index on ties (searching the product codebook instead would let the rounding of
// one group's distance decide the other's near ties).  One thread per (token, code byte).
template <int SUB_B>
__global__ __launch_bounds__(256) void encode_subbyte_kernel(EncodeArgs a)
{
    constexpr int FUSE = 8 / SUB_B, KS = 1 << SUB_B;
    const EncodeTensor& tsr = a.tensor[blockIdx.z];
    const int sub_c = a.f.sub_c;
    const int bytes_per_token = a.f.groups;                 // fused groups = code bytes per token
    const long long total = (long long)a.batch * a.t_new * bytes_per_token;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int gf = (int)(idx % bytes_per_token);            // fused group (all heads)
    const long long row = idx / bytes_per_token;
    const int t = (int)(row % a.t_new), n = (int)(row / a.t_new);
    const uint16_t* x = tsr.x + (size_t)n * tsr.x_batch_stride + (size_t)t * tsr.x_row_stride + (size_t)gf * a.f.c;
    unsigned code_byte = 0;
    for (int i = 0; i < FUSE; ++i) {
        const uint16_t* cen = tsr.centroids + ((size_t)gf * FUSE + i) * KS * sub_c;
        float best = __builtin_inff();
        int best_j = 0;
        for (int j = 0; j < KS; ++j) {
            float acc = 0.f;
            for (int ch = 0; ch < sub_c; ++ch) {
                const float d = (float)__builtin_bit_cast(_Float16, x[i * sub_c + ch]) -
                                (float)__builtin_bit_cast(_Float16, cen[j * sub_c + ch]);
                acc = __builtin_fmaf(d, d, acc);
            }
            if (acc < best) {
                best = acc;
                best_j = j;
            }
        }
        code_byte |= (unsigned)best_j << (SUB_B * i);
    }
    const int hkv = gf / a.f.gh, g = gf % a.f.gh;
    const int pos = a.t_offset + t, tile = pos / kTileTokens, u = pos % kTileTokens;
    const int slot = (g - u) & (a.f.gh - 1);
    uint8_t* dst = tsr.codes + a.map.tile_index(n, hkv, tile) * (size_t)a.f.tile_bytes;
    dst[(slot >> 4) * 1024 + u * 16 + (slot & 15)] = (uint8_t)code_byte;
}

__global__ __launch_bounds__(256) void expand_codebook_kernel(const uint16_t* centroids, uint16_t* fused, int n_fused_groups,
                                                              int sub_c, int sub_b)
{
    const int fuse = 8 / sub_b, ks = 1 << sub_b, cf = sub_c * fuse;
    const long long total = (long long)n_fused_groups * 256 * cf;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int ch = (int)(idx % cf);
    const int j = (int)((idx / cf) % 256);
    const int gf = (int)(idx / ((long long)cf * 256));
    const int i = ch / sub_c;                                // which of the fused groups
    const int ji = (j >> (sub_b * i)) & (ks - 1);
    fused[idx] = centroids[(((size_t)gf * fuse + i) * ks + ji) * sub_c + ch % sub_c];
}

cq_status launch_encode_subbyte(const EncodeArgs& a, hipStream_t stream)
{
    const long long total = (long long)a.batch * a.t_new * a.f.groups;
    const long long blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffLL) return CQ_ERR_INVALID_ARG;
    const dim3 grid((unsigned)blocks, 1, (unsigned)a.n_tensors);
    if (a.f.sub_b == 4) hipLaunchKernelGGL(encode_subbyte_kernel<4>, grid, dim3(256), 0, stream, a);
    else if (a.f.sub_b == 2) hipLaunchKernelGGL(encode_subbyte_kernel<2>, grid, dim3(256), 0, stream, a);
    else return CQ_ERR_UNSUPPORTED;
    return hipGetLastError() == hipSuccess ? CQ_OK : CQ_ERR_HIP;
}

}  // namespace

cq_status launch_expand_codebook(const uint16_t* centroids, const Derived& f, uint16_t* fused, hipStream_t stream)
{
    const long long total = (long long)f.groups * 256 * f.c;
    hipLaunchKernelGGL(expand_codebook_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, centroids, fused,
                       f.groups, f.sub_c, f.sub_b);
    return hipGetLastError() == hipSuccess ? CQ_OK : CQ_ERR_HIP;
}

cq_status launch_encode(const EncodeArgs& a, hipStream_t stream)
{
    if (a.f.fuse > 1) return launch_encode_subbyte(a, stream);
    if (a.f.b == 8) {
        if (a.f.gh == 16 && a.f.c == 8) return launch_format<16, 8, 8>(a, stream);
        if (a.f.gh == 32 && a.f.c == 4) return launch_format<32, 4, 8>(a, stream);
        if (a.f.gh == 64 && a.f.c == 2) return launch_format<64, 2, 8>(a, stream);
    } else if (a.f.b == 10) {
        if (a.f.gh == 16 && a.f.c == 8) return launch_format<16, 8, 10>(a, stream);
    }
    return CQ_ERR_UNSUPPORTED;
}

cq_status launch_dequantize(const DequantArgs& a, hipStream_t stream)
{
    if (a.f.b == 8) {
        if (a.f.gh == 16 && a.f.c == 8) return launch_dequant_format<16, 8, 8>(a, stream);
        if (a.f.gh == 32 && a.f.c == 4) return launch_dequant_format<32, 4, 8>(a, stream);
        if (a.f.gh == 64 && a.f.c == 2) return launch_dequant_format<64, 2, 8>(a, stream);
    } else if (a.f.b == 10) {
        if (a.f.gh == 16 && a.f.c == 8) return launch_dequant_format<16, 8, 10>(a, stream);
    }
    return CQ_ERR_UNSUPPORTED;
}

}  // namespace cq

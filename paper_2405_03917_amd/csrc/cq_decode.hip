// Decode attention straight from packed CQ codes (Eq. 1 of the paper over the centroids the
// cached codes select), for gfx950.
//
// One workgroup handles one (sequence, query head, context split).  Per workgroup:
//   1. build the score table  LUT[g][j] = scale * log2(e) * (q_g . C_K[g][j])  in LDS;
//   2. phase K: stream the split's key codes (one 64-token tile per wavefront per step, lane =
//      token), score = sum over groups of LUT[g][code]; keep scores in LDS, reduce the maximum;
//   3. phase V: stream the value codes; p = 2^(score - max); add p into bin[g][code] in LDS;
//   4. epilogue: o[g c + i] = sum_j bin[g][j] * C_V[g][j][i]; write (max, sum p, o) as a partial;
// a second kernel merges the partials of all splits and rounds to fp16.
//
// LDS table layout (b = 8): 256 rows (one per code value) of 64 four-byte words (256 B per row).
// Lane l of a wavefront owns ONE word column at every step s of the walk over a token's Gh
// slots, column(l, g) with g = (l + s) mod Gh the group that the cache layout put in slot s of
// token l.  Columns of the 64 lanes are pairwise different and, within each half-wavefront,
// different modulo 32, so neither the table gather nor the bin update ever has a bank conflict
// or two lanes on one address.  Groups are replicated R = 64 / Gh times to give every lane its
// own column; the epilogue adds the replicas.  The byte address of a lookup is
// (code << 8) | (4 * column): one v_perm_b32 from the code word and a per-lane constant.
#include <hip/hip_runtime.h>

#include <mutex>

#include "cq_internal.hpp"

namespace cq {
namespace {

typedef __attribute__((address_space(3))) float lds_f32;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int kTabFloats = 256 * kTabWords;   // 16384 floats = 64 KB
constexpr int kRedFloats = 64;
constexpr int kMinScoreFloats = 4096;         // also the staging area of one 16-group chunk

// Raw LDS accesses by byte address.  The table sits at LDS address 0 (the kernels declare no
// static LDS; the launcher checks that), so a table-relative address is an LDS address.
__device__ __forceinline__ float lds_load(unsigned byte_addr) { return *(lds_f32*)(byte_addr); }
__device__ __forceinline__ void lds_add(unsigned byte_addr, float v)
{
    __hip_atomic_fetch_add((lds_f32*)(byte_addr), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// Word column of lane `lane` when it handles group g.
template <int GH>
__device__ __forceinline__ int column(int lane, int g)
{
    if constexpr (GH == 64) {
        return g;
    } else if constexpr (GH == 32) {
        return 2 * g + (((g >> 4) ^ (lane >> 5)) & 1);
    } else {
        static_assert(GH == 16, "groups per head must be 16, 32 or 64");
        return 4 * g + 2 * (((g >> 3) ^ (lane >> 5)) & 1) + ((lane >> 4) & 1);
    }
}

__device__ __forceinline__ int stage_index(int gl, int j) { return gl * 256 + (j ^ (2 * gl)); }

template <int C>
__device__ __forceinline__ float dot_group(const uint16_t* cent, const uint16_t* qg)
{
    float acc = 0.f;
    if constexpr (C == 8) {
        uint4 a = *reinterpret_cast<const uint4*>(cent);
        uint4 b = *reinterpret_cast<const uint4*>(qg);
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a.x), __builtin_bit_cast(half2_t, b.x), acc, false);
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a.y), __builtin_bit_cast(half2_t, b.y), acc, false);
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a.z), __builtin_bit_cast(half2_t, b.z), acc, false);
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a.w), __builtin_bit_cast(half2_t, b.w), acc, false);
    } else if constexpr (C == 4) {
        uint2 a = *reinterpret_cast<const uint2*>(cent);
        uint2 b = *reinterpret_cast<const uint2*>(qg);
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a.x), __builtin_bit_cast(half2_t, b.x), acc, false);
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a.y), __builtin_bit_cast(half2_t, b.y), acc, false);
    } else {
        static_assert(C == 2, "channels per group must be 2, 4 or 8");
        unsigned a = *reinterpret_cast<const unsigned*>(cent);
        unsigned b = *reinterpret_cast<const unsigned*>(qg);
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a), __builtin_bit_cast(half2_t, b), acc, false);
    }
    return acc;
}

template <int C>
__device__ __forceinline__ void load_centroid(const uint16_t* cent, float (&v)[C])
{
    if constexpr (C == 8) {
        uint4 a = *reinterpret_cast<const uint4*>(cent);
        unsigned w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            half2_t h = __builtin_bit_cast(half2_t, w[i]);
            v[2 * i] = (float)h.x;
            v[2 * i + 1] = (float)h.y;
        }
    } else if constexpr (C == 4) {
        uint2 a = *reinterpret_cast<const uint2*>(cent);
        half2_t h0 = __builtin_bit_cast(half2_t, a.x), h1 = __builtin_bit_cast(half2_t, a.y);
        v[0] = (float)h0.x; v[1] = (float)h0.y; v[2] = (float)h1.x; v[3] = (float)h1.y;
    } else {
        unsigned a = *reinterpret_cast<const unsigned*>(cent);
        half2_t h = __builtin_bit_cast(half2_t, a);
        v[0] = (float)h.x; v[1] = (float)h.y;
    }
}

template <int P>
struct TileWords {
    u32x4 v[P];
};

template <int GH>
__device__ __forceinline__ TileWords<GH / 16> load_tile(const uint8_t* stream, int tile, int lane)
{
    TileWords<GH / 16> w;
    const u32x4* p = reinterpret_cast<const u32x4*>(stream + (size_t)tile * (kTileTokens * GH)) + lane;
#pragma unroll
    for (int pl = 0; pl < GH / 16; ++pl) w.v[pl] = __builtin_nontemporal_load(p + pl * 64);
    return w;
}

// Byte address of the table word for slot s: (code << 8) | off byte.
template <int GH>
__device__ __forceinline__ unsigned slot_addr(const TileWords<GH / 16>& w, const unsigned (&off)[GH / 4], int s)
{
    const u32x4 q = w.v[s >> 4];
    const int dw = (s >> 2) & 3;
    const unsigned code_word = dw == 0 ? q.x : dw == 1 ? q.y : dw == 2 ? q.z : q.w;
    const unsigned k = s & 3;
    const unsigned sel = 0x0c0c0000u | ((4u + k) << 8) | k;   // {0, 0, code byte k, off byte k}
    return __builtin_amdgcn_perm(code_word, off[s >> 2], sel);
}

// Walk tiles first, first + stride, ... (n of them) of a code stream with PF tiles in flight.
// The steady state is straight-line code (consume one tile, request the tile PF steps ahead)
// so that the compiler can keep PF loads outstanding; the last tiles are requested together
// and then consumed.  `fn(words, k)` is called once per tile k = 0 .. n-1, in order.
template <int GH, int PF, class Fn>
__device__ __forceinline__ void stream_tiles(const uint8_t* stream, int n, int first, int stride, int lane, Fn&& fn)
{
    constexpr int P = GH / 16;
    int k = 0;
    if (n >= 2 * PF) {
        TileWords<P> buf[PF];
#pragma unroll
        for (int i = 0; i < PF; ++i) {
            buf[i] = load_tile<GH>(stream, first + i * stride, lane);
            __builtin_amdgcn_sched_barrier(0);      // keep request order == consumption order
        }
        for (; k + 2 * PF <= n; k += PF) {
#pragma unroll
            for (int i = 0; i < PF; ++i) {
                fn(buf[i], k + i);
                buf[i] = load_tile<GH>(stream, first + (k + PF + i) * stride, lane);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int i = 0; i < PF; ++i) fn(buf[i], k + i);
        k += PF;
    }
    constexpr int TAIL = 2 * PF - 1;
    TileWords<P> tbuf[TAIL];
#pragma unroll
    for (int i = 0; i < TAIL; ++i)
        if (k + i < n) tbuf[i] = load_tile<GH>(stream, first + (k + i) * stride, lane);
#pragma unroll
    for (int i = 0; i < TAIL; ++i)
        if (k + i < n) fn(tbuf[i], k + i);
}

template <int GH, int C, int NT>
__global__ __launch_bounds__(NT) void decode_split_kernel(DecodeArgs a)
{
    constexpr int R = 64 / GH;          // replicas per group
    constexpr int P = GH / 16;          // 16-byte planes per token
    constexpr int NW = NT / 64;         // wavefronts
    constexpr int D = GH * C;           // head_dim
    constexpr int PF = GH == 16 ? 4 : 2;   // tiles in flight per wavefront (4 KB)
    extern __shared__ float smem[];
    float* tab = smem;                              // [256][64]
    float* sc = smem + kTabFloats;                  // scores of the split / staging
    const int sc_floats = max(kMinScoreFloats, a.tiles_per_split * kTileTokens + kRedFloats);
    float* red = sc + sc_floats - kRedFloats;       // cross-wave reductions

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    int idx = blockIdx.x;
    const int hq = idx % a.n_q_heads;
    idx /= a.n_q_heads;
    const int split = idx % a.n_split;
    const int n = idx / a.n_split;
    const int hkv = hq / (a.n_q_heads / a.f.n_kv_heads);

    int t_n = a.t;
    if (a.seq_lens) t_n = min(max(a.seq_lens[n], 1), a.t);
    const int n_tiles = (t_n + kTileTokens - 1) / kTileTokens;
    const int tile0 = split * a.tiles_per_split;
    const int tile1 = min(tile0 + a.tiles_per_split, n_tiles);

    float* part = a.partials + ((size_t)(n * a.n_q_heads + hq) * a.n_split + split) * (D + kPartialHeader);
    if (tile0 >= tile1) {               // this split lies beyond the sequence: neutral partial
        if (tid == 0) { part[0] = -INFINITY; part[1] = 0.f; }
        for (int i = tid; i < D; i += NT) part[kPartialHeader + i] = 0.f;
        return;
    }

    // per-lane column bytes for the Gh steps of a token walk
    unsigned off[GH / 4];
#pragma unroll
    for (int i = 0; i < GH / 4; ++i) {
        unsigned v = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int g = (lane + 4 * i + k) & (GH - 1);
            v |= (unsigned)(4 * column<GH>(lane, g)) << (8 * k);
        }
        off[i] = v;
    }

    const size_t stream_idx = (size_t)(n * a.f.n_kv_heads + hkv) * (a.t_cap / kTileTokens) * (kTileTokens * GH);
    const uint8_t* kstream = a.k_codes + stream_idx;
    const uint8_t* vstream = a.v_codes + stream_idx;
    const int my_tiles = (tile1 - tile0 - wave + NW - 1) / NW;   // tiles tile0 + wave + k NW

    // ---- 1. score table ------------------------------------------------------------------
    const uint16_t* qh = a.q + (size_t)(n * a.n_q_heads + hq) * D;
    for (int g0 = 0; g0 < GH; g0 += 16) {
        const uint16_t* ck = a.k_centroids + (size_t)(hkv * GH + g0) * 256 * C;
        for (int it = tid; it < 16 * 256; it += NT) {
            const int gl = it >> 8, j = it & 255;
            const float dot = dot_group<C>(ck + (size_t)it * C, qh + (g0 + gl) * C);
            sc[stage_index(gl, j)] = dot * a.scale_log2e;
        }
        __syncthreads();
        for (int it = tid; it < 16 * 256; it += NT) {
            const int gl = it & 15, j = it >> 4;
            const float v = sc[stage_index(gl, j)];
            float* dst = tab + j * kTabWords + (g0 + gl) * R;
            if constexpr (R == 4) *reinterpret_cast<float4*>(dst) = make_float4(v, v, v, v);
            else if constexpr (R == 2) *reinterpret_cast<float2*>(dst) = make_float2(v, v);
            else *dst = v;
        }
        __syncthreads();
    }

    // ---- 2. phase K: scores --------------------------------------------------------------
    float lane_max = -INFINITY;
    stream_tiles<GH, PF>(kstream, my_tiles, tile0 + wave, NW, lane, [&](const TileWords<P>& w, int k) {
        float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
        for (int s = 0; s < GH; s += 2) {
            acc0 += lds_load(slot_addr<GH>(w, off, s));
            acc1 += lds_load(slot_addr<GH>(w, off, s + 1));
        }
        const int lt = wave + k * NW;                       // tile within the split
        const int tok = (tile0 + lt) * kTileTokens + lane;
        const float sv = tok < t_n ? acc0 + acc1 : -INFINITY;
        sc[lt * kTileTokens + lane] = sv;
        lane_max = fmaxf(lane_max, sv);
    });

    lane_max = wave_max(lane_max);
    __syncthreads();                                // all table reads done, all scores written
    if (lane == 0) red[wave] = lane_max;
    {
        float4* t4 = reinterpret_cast<float4*>(tab);
        for (int i = tid; i < kTabFloats / 4; i += NT) t4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    __syncthreads();
    float m = red[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) m = fmaxf(m, red[w]);
    // (every split that reaches this point holds at least one valid token, so m is finite)

    // ---- 3. phase V: probability bins ----------------------------------------------------
    float lane_sum = 0.f;
    stream_tiles<GH, PF>(vstream, my_tiles, tile0 + wave, NW, lane, [&](const TileWords<P>& w, int k) {
        const int lt = wave + k * NW;
        const float p = __builtin_amdgcn_exp2f(sc[lt * kTileTokens + lane] - m);
        lane_sum += p;
#pragma unroll
        for (int s = 0; s < GH; ++s) lds_add(slot_addr<GH>(w, off, s), p);
    });
    lane_sum = wave_sum(lane_sum);
    __syncthreads();                                // all bin updates done, red free again
    if (lane == 0) red[wave] = lane_sum;
    __syncthreads();
    if (tid == 0) {
        float l = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) l += red[w];
        part[0] = m;
        part[1] = l;
    }
    __syncthreads();                                // red is part of the staging area below

    // ---- 4. epilogue: o = bins . C_V -----------------------------------------------------
    constexpr int LPG = NT / 16;                    // lanes per group in the product step
    for (int g0 = 0; g0 < GH; g0 += 16) {
        for (int it = tid; it < 16 * 256; it += NT) {
            const int gl = it & 15, j = it >> 4;
            const float* src = tab + j * kTabWords + (g0 + gl) * R;
            float v;
            if constexpr (R == 4) { const float4 x = *reinterpret_cast<const float4*>(src); v = (x.x + x.y) + (x.z + x.w); }
            else if constexpr (R == 2) { const float2 x = *reinterpret_cast<const float2*>(src); v = x.x + x.y; }
            else v = *src;
            sc[stage_index(gl, j)] = v;
        }
        __syncthreads();
        {
            const int gl = tid / LPG, jl = tid % LPG;
            const uint16_t* cv = a.v_centroids + (size_t)(hkv * GH + g0 + gl) * 256 * C;
            float acc[C];
#pragma unroll
            for (int i = 0; i < C; ++i) acc[i] = 0.f;
            for (int j = jl; j < 256; j += LPG) {
                const float bin = sc[stage_index(gl, j)];
                float cen[C];
                load_centroid<C>(cv + (size_t)j * C, cen);
#pragma unroll
                for (int i = 0; i < C; ++i) acc[i] = __builtin_fmaf(bin, cen[i], acc[i]);
            }
#pragma unroll
            for (int i = 0; i < C; ++i) {
#pragma unroll
                for (int o = LPG / 2; o > 0; o >>= 1) acc[i] += __shfl_xor(acc[i], o);
            }
            if (jl == 0) {
#pragma unroll
                for (int i = 0; i < C; ++i) part[kPartialHeader + (g0 + gl) * C + i] = acc[i];
            }
        }
        __syncthreads();
    }
}

// Merge the partials of all splits of one (sequence, query head): exact rescaling by the
// overall maximum, then one rounding to fp16.
__global__ void decode_merge_kernel(const float* partials, uint16_t* out, int n_split, int head_dim)
{
    const int bh = blockIdx.x;
    const int stride = head_dim + kPartialHeader;
    const float* p = partials + (size_t)bh * n_split * stride;
    float m = -INFINITY;
    for (int s = 0; s < n_split; ++s) m = fmaxf(m, p[s * stride]);
    for (int i = threadIdx.x; i < head_dim; i += blockDim.x) {
        float l = 0.f, o = 0.f;
        for (int s = 0; s < n_split; ++s) {
            const float ms = p[s * stride];
            if (ms == -INFINITY) continue;
            const float w = __builtin_amdgcn_exp2f(ms - m);
            l = __builtin_fmaf(p[s * stride + 1], w, l);
            o = __builtin_fmaf(p[s * stride + kPartialHeader + i], w, o);
        }
        const _Float16 h = (_Float16)(o / l);
        out[(size_t)bh * head_dim + i] = __builtin_bit_cast(uint16_t, h);
    }
}


// ------------------------------------------------------------------------------------------
// 10-bit codes (CQ-8c10b): 1024 rows of 32 words (128 B per row, 128 KB).  16 groups x 2
// replicas; lanes l and l + 32 share a column, which costs nothing on a 32-bank LDS that
// serves a wavefront in two halves.  Byte address = (code << 7) | (4 * column).
// ------------------------------------------------------------------------------------------
constexpr int kTab10Words = 32;
constexpr int kTab10Floats = 1024 * kTab10Words;

struct Tile10 {
    u32x4 lo;          // low bytes of the 16 slots
    unsigned hi;       // bits [2s+1 : 2s] = high bits of slot s
};

__device__ __forceinline__ Tile10 load_tile10(const uint8_t* stream, int tile, int lane)
{
    const uint8_t* base = stream + (size_t)tile * (kTileTokens * 20);
    Tile10 w;
    w.lo = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base) + lane);
    w.hi = __builtin_nontemporal_load(reinterpret_cast<const unsigned*>(base + 1024) + lane);
    return w;
}

__device__ __forceinline__ unsigned slot_addr10(const Tile10& w, const unsigned (&off)[16], int s)
{
    const int dw = s >> 2;
    const unsigned word = dw == 0 ? w.lo.x : dw == 1 ? w.lo.y : dw == 2 ? w.lo.z : w.lo.w;
    const unsigned lo = (word >> (8 * (s & 3))) & 0xffu;
    const unsigned hi = (w.hi >> (2 * s)) & 3u;
    return ((lo << 7) | (hi << 15)) | off[s];
}

template <int PF, class Fn>
__device__ __forceinline__ void stream_tiles10(const uint8_t* stream, int n, int first, int stride, int lane, Fn&& fn)
{
    int k = 0;
    if (n >= 2 * PF) {
        Tile10 buf[PF];
#pragma unroll
        for (int i = 0; i < PF; ++i) {
            buf[i] = load_tile10(stream, first + i * stride, lane);
            __builtin_amdgcn_sched_barrier(0);
        }
        for (; k + 2 * PF <= n; k += PF) {
#pragma unroll
            for (int i = 0; i < PF; ++i) {
                fn(buf[i], k + i);
                buf[i] = load_tile10(stream, first + (k + PF + i) * stride, lane);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int i = 0; i < PF; ++i) fn(buf[i], k + i);
        k += PF;
    }
    constexpr int TAIL = 2 * PF - 1;
    Tile10 tbuf[TAIL];
#pragma unroll
    for (int i = 0; i < TAIL; ++i)
        if (k + i < n) tbuf[i] = load_tile10(stream, first + (k + i) * stride, lane);
#pragma unroll
    for (int i = 0; i < TAIL; ++i)
        if (k + i < n) fn(tbuf[i], k + i);
}

__device__ __forceinline__ int stage_index10(int gl, int j) { return gl * 1024 + (j ^ (2 * gl)); }

__global__ __launch_bounds__(1024) void decode_split10_kernel(DecodeArgs a)
{
    constexpr int GH = 16, C = 8, K = 1024, NT = 1024, NW = NT / 64, D = GH * C, PF = 4;
    constexpr int GC = 4;                               // groups per staging chunk (4 * 1024 floats)
    extern __shared__ float smem[];
    float* tab = smem;                                  // [1024][32]
    float* sc = smem + kTab10Floats;
    const int sc_floats = max(kMinScoreFloats, a.tiles_per_split * kTileTokens + kRedFloats);
    float* red = sc + sc_floats - kRedFloats;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    int idx = blockIdx.x;
    const int hq = idx % a.n_q_heads;
    idx /= a.n_q_heads;
    const int split = idx % a.n_split;
    const int n = idx / a.n_split;
    const int hkv = hq / (a.n_q_heads / a.f.n_kv_heads);

    int t_n = a.t;
    if (a.seq_lens) t_n = min(max(a.seq_lens[n], 1), a.t);
    const int n_tiles = (t_n + kTileTokens - 1) / kTileTokens;
    const int tile0 = split * a.tiles_per_split;
    const int tile1 = min(tile0 + a.tiles_per_split, n_tiles);

    float* part = a.partials + ((size_t)(n * a.n_q_heads + hq) * a.n_split + split) * (D + kPartialHeader);
    if (tile0 >= tile1) {
        if (tid == 0) { part[0] = -INFINITY; part[1] = 0.f; }
        for (int i = tid; i < D; i += NT) part[kPartialHeader + i] = 0.f;
        return;
    }

    unsigned off[16];
#pragma unroll
    for (int s = 0; s < 16; ++s) {
        const int g = (lane + s) & 15;
        off[s] = 4u * (unsigned)(2 * g + ((lane >> 4) & 1));
    }

    const size_t stream_idx = (size_t)(n * a.f.n_kv_heads + hkv) * (a.t_cap / kTileTokens) * (kTileTokens * 20);
    const uint8_t* kstream = a.k_codes + stream_idx;
    const uint8_t* vstream = a.v_codes + stream_idx;
    const int my_tiles = (tile1 - tile0 - wave + NW - 1) / NW;

    // ---- 1. score table ------------------------------------------------------------------
    const uint16_t* qh = a.q + (size_t)(n * a.n_q_heads + hq) * D;
    for (int g0 = 0; g0 < GH; g0 += GC) {
        const uint16_t* ck = a.k_centroids + (size_t)(hkv * GH + g0) * K * C;
        for (int it = tid; it < GC * K; it += NT) {
            const int gl = it >> 10, j = it & 1023;
            const float dot = dot_group<C>(ck + (size_t)it * C, qh + (g0 + gl) * C);
            sc[stage_index10(gl, j)] = dot * a.scale_log2e;
        }
        __syncthreads();
        for (int it = tid; it < GC * K; it += NT) {
            const int gl = it & 3, j = it >> 2;
            const float v = sc[stage_index10(gl, j)];
            *reinterpret_cast<float2*>(tab + j * kTab10Words + (g0 + gl) * 2) = make_float2(v, v);
        }
        __syncthreads();
    }

    // ---- 2. phase K ----------------------------------------------------------------------
    float lane_max = -INFINITY;
    stream_tiles10<PF>(kstream, my_tiles, tile0 + wave, NW, lane, [&](const Tile10& w, int k) {
        float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
        for (int s = 0; s < GH; s += 2) {
            acc0 += lds_load(slot_addr10(w, off, s));
            acc1 += lds_load(slot_addr10(w, off, s + 1));
        }
        const int lt = wave + k * NW;
        const int tok = (tile0 + lt) * kTileTokens + lane;
        const float sv = tok < t_n ? acc0 + acc1 : -INFINITY;
        sc[lt * kTileTokens + lane] = sv;
        lane_max = fmaxf(lane_max, sv);
    });

    lane_max = wave_max(lane_max);
    __syncthreads();
    if (lane == 0) red[wave] = lane_max;
    {
        float4* t4 = reinterpret_cast<float4*>(tab);
        for (int i = tid; i < kTab10Floats / 4; i += NT) t4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    __syncthreads();
    float m = red[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) m = fmaxf(m, red[w]);

    // ---- 3. phase V ----------------------------------------------------------------------
    float lane_sum = 0.f;
    stream_tiles10<PF>(vstream, my_tiles, tile0 + wave, NW, lane, [&](const Tile10& w, int k) {
        const int lt = wave + k * NW;
        const float p = __builtin_amdgcn_exp2f(sc[lt * kTileTokens + lane] - m);
        lane_sum += p;
#pragma unroll
        for (int s = 0; s < GH; ++s) lds_add(slot_addr10(w, off, s), p);
    });
    lane_sum = wave_sum(lane_sum);
    __syncthreads();
    if (lane == 0) red[wave] = lane_sum;
    __syncthreads();
    if (tid == 0) {
        float l = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) l += red[w];
        part[0] = m;
        part[1] = l;
    }
    __syncthreads();

    // ---- 4. epilogue ---------------------------------------------------------------------
    // wave w handles group g0 + (w & 3) and the quarter (w >> 2) of its 1024 centroids
    for (int g0 = 0; g0 < GH; g0 += GC) {
        for (int it = tid; it < GC * K; it += NT) {
            const int gl = it & 3, j = it >> 2;
            const float2 x = *reinterpret_cast<const float2*>(tab + j * kTab10Words + (g0 + gl) * 2);
            sc[stage_index10(gl, j)] = x.x + x.y;
        }
        __syncthreads();
        float acc[C];
        {
            const int gl = wave & 3, quarter = wave >> 2;
            const uint16_t* cv = a.v_centroids + (size_t)(hkv * GH + g0 + gl) * K * C;
#pragma unroll
            for (int i = 0; i < C; ++i) acc[i] = 0.f;
            for (int j = quarter * 256 + lane; j < quarter * 256 + 256; j += 64) {
                const float bin = sc[stage_index10(gl, j)];
                float cen[C];
                load_centroid<C>(cv + (size_t)j * C, cen);
#pragma unroll
                for (int i = 0; i < C; ++i) acc[i] = __builtin_fmaf(bin, cen[i], acc[i]);
            }
#pragma unroll
            for (int i = 0; i < C; ++i) acc[i] = wave_sum(acc[i]);
        }
        __syncthreads();                                // staging reads done; reuse its head
        if (lane == 0) {
#pragma unroll
            for (int i = 0; i < C; ++i) sc[wave * C + i] = acc[i];
        }
        __syncthreads();
        if (tid < GC * C) {
            const int gl = tid / C, i = tid % C;
            float o = 0.f;
#pragma unroll
            for (int quarter = 0; quarter < 4; ++quarter) o += sc[(quarter * 4 + gl) * C + i];
            part[kPartialHeader + (g0 + gl) * C + i] = o;
        }
        __syncthreads();
    }
}

size_t smem_bytes(int tiles_per_split)
{
    const int sc_floats = std::max(kMinScoreFloats, tiles_per_split * kTileTokens + kRedFloats);
    return sizeof(float) * (size_t)(kTabFloats + sc_floats);
}

template <int GH, int C, int NT>
cq_status launch_variant(const DecodeArgs& a, hipStream_t stream)
{
    auto kernel = decode_split_kernel<GH, C, NT>;
    static std::once_flag once;
    static hipError_t setup = hipSuccess;
    std::call_once(once, [&] {
        hipFuncAttributes attr;
        setup = hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(kernel));
        // the kernels address the table from LDS address 0: no static LDS may precede it
        if (setup == hipSuccess && attr.sharedSizeBytes != 0) setup = hipErrorInvalidValue;
        if (setup == hipSuccess)
            setup = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    });
    if (setup != hipSuccess) return CQ_ERR_HIP;
    const size_t smem = smem_bytes(a.tiles_per_split);
    const unsigned grid = (unsigned)(a.batch * a.n_q_heads * a.n_split);
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(NT), smem, stream, a);
    if (hipGetLastError() != hipSuccess) return CQ_ERR_HIP;
    return CQ_OK;
}

template <int GH, int C>
cq_status launch_by_split(const DecodeArgs& a, hipStream_t stream)
{
    // up to 63 tiles the workgroup's LDS footprint is 80 KB: two 512-thread workgroups per CU;
    // longer splits run as one 1024-thread workgroup per CU.
    if (a.tiles_per_split <= 63) return launch_variant<GH, C, 512>(a, stream);
    return launch_variant<GH, C, 1024>(a, stream);
}


cq_status launch_variant10(const DecodeArgs& a, hipStream_t stream)
{
    auto kernel = decode_split10_kernel;
    static std::once_flag once;
    static hipError_t setup = hipSuccess;
    std::call_once(once, [&] {
        hipFuncAttributes attr;
        setup = hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(kernel));
        if (setup == hipSuccess && attr.sharedSizeBytes != 0) setup = hipErrorInvalidValue;
        if (setup == hipSuccess)
            setup = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    });
    if (setup != hipSuccess) return CQ_ERR_HIP;
    const int sc_floats = std::max(kMinScoreFloats, a.tiles_per_split * kTileTokens + kRedFloats);
    const size_t smem = sizeof(float) * (size_t)(kTab10Floats + sc_floats);
    const unsigned grid = (unsigned)(a.batch * a.n_q_heads * a.n_split);
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(1024), smem, stream, a);
    if (hipGetLastError() != hipSuccess) return CQ_ERR_HIP;
    return CQ_OK;
}

}  // namespace

int decode_max_tiles_per_split(const Derived& f)
{
    // LDS: 160 KB = table + scores (+64 floats for reductions)
    if (f.b == 10) return (160 * 1024 / 4 - kTab10Floats - kRedFloats) / kTileTokens;   // 127
    return 255;
}

cq_status launch_decode(const DecodeArgs& a, hipStream_t stream)
{
    cq_status st = CQ_ERR_UNSUPPORTED;
    if (a.f.b == 8) {
        if (a.f.gh == 16 && a.f.c == 8) st = launch_by_split<16, 8>(a, stream);
        else if (a.f.gh == 32 && a.f.c == 4) st = launch_by_split<32, 4>(a, stream);
        else if (a.f.gh == 64 && a.f.c == 2) st = launch_by_split<64, 2>(a, stream);
    } else if (a.f.b == 10 && a.f.gh == 16 && a.f.c == 8) {
        st = launch_variant10(a, stream);
    }
    if (st != CQ_OK) return st;
    const int threads = a.f.head_dim <= 64 ? 64 : (a.f.head_dim <= 128 ? 128 : 256);
    hipLaunchKernelGGL(decode_merge_kernel, dim3((unsigned)(a.batch * a.n_q_heads)), dim3(threads), 0, stream,
                       a.partials, a.out, a.n_split, a.f.head_dim);
    if (hipGetLastError() != hipSuccess) return CQ_ERR_HIP;
    return CQ_OK;
}

}  // namespace cq

// Device code shared by the decode-attention kernels of libcq (cq_decode.hip, cq_decode_rope.hip):
// raw LDS access, wavefront reductions, the format constants, the tile of codes of 64 tokens and
// its lane-per-token view, the walk over a code stream with tiles in flight.  Internal linkage:
// every translation unit gets its own copy.
#pragma once

#include <hip/hip_runtime.h>

#include "cq_internal.hpp"

namespace cq {
namespace {

typedef __attribute__((address_space(3))) float lds_f32;
typedef __attribute__((address_space(3))) unsigned lds_u32;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int kMinScoreFloats = 4096;         // the score buffer doubles as reduction scratch
// fused step: 2 x Gh 64-bit (distance, index) minima, then the new token's fixed-point weight
constexpr int kKeyFloats(int gh) { return 2 * 2 * gh + 2; }
// one (maximum, sum) pair per wavefront, up to 16 wavefronts
constexpr int kSlotFloats = 32;
// reduction scratch: 64 words + one row of head_dim floats per wavefront
constexpr int kScratchFloats(int nt, int head_dim) { return 64 + (nt / 64) * head_dim; }

// Raw LDS accesses by byte address.  The table sits at LDS address 0 (the kernels declare no
// static LDS; the launcher checks that), so a table-relative address is an LDS address.
__device__ __forceinline__ float lds_load(unsigned byte_addr) { return *(lds_f32*)(byte_addr); }
__device__ __forceinline__ void lds_add(unsigned byte_addr, unsigned v)
{
    __hip_atomic_fetch_add((lds_u32*)(byte_addr), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() would also wait for every
// outstanding global load, i.e. for the code tiles that are deliberately kept in flight across
// the barriers of this kernel.  (No barrier here orders global memory: what the workgroup
// exchanges lives in LDS.)
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
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
__device__ __forceinline__ unsigned wave_sum_u32(unsigned v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

__device__ __forceinline__ void lds_min_u64(unsigned long long* p, unsigned long long v)
{
    __hip_atomic_fetch_min(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// Nearest-centroid search of the fused decode step, bit-identical to cq_encode: squared distance
// in fp32, one fused multiply-add per channel in channel order.  x - c is formed as
// fma(c, -1, x): one rounding like the subtraction, and the fp16 centroid is read directly by
// the mixed-precision FMA.  A thread walks its centroids in ascending index order and keeps
// the first minimum; (distance bits, index) packed into 64 bits then make the minimum over
// threads the nearest centroid with the lowest index among equals.
template <int C>
__device__ __forceinline__ float centroid_distance(const float (&x)[C], const unsigned* halves)
{
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < C / 2; ++i) {
        const half2_t h = __builtin_bit_cast(half2_t, halves[i]);
        const float d0 = __builtin_fmaf((float)h.x, -1.0f, x[2 * i]);
        acc = __builtin_fmaf(d0, d0, acc);
        const float d1 = __builtin_fmaf((float)h.y, -1.0f, x[2 * i + 1]);
        acc = __builtin_fmaf(d1, d1, acc);
    }
    return acc;
}
struct Nearest {
    float d = __builtin_inff();
    int j = 0;
    __device__ __forceinline__ void offer(float dist, int idx)
    {
        j = dist < d ? idx : j;
        d = dist < d ? dist : d;
    }
    __device__ __forceinline__ unsigned long long key() const
    {
        return ((unsigned long long)__float_as_uint(d) << 32) | (unsigned)j;
    }
};

template <int C>
__device__ __forceinline__ void load_row_slice(const uint16_t* p, float (&x)[C])
{
#pragma unroll
    for (int i = 0; i < C / 2; ++i) {
        const half2_t h = __builtin_bit_cast(half2_t, *reinterpret_cast<const unsigned*>(p + 2 * i));
        x[2 * i] = (float)h.x;
        x[2 * i + 1] = (float)h.y;
    }
}

// minimum over the LPG neighbouring lanes that walk the same group's codebook
template <int LPG>
__device__ __forceinline__ unsigned long long group_lanes_min(unsigned long long key)
{
#pragma unroll
    for (int m = 1; m < LPG; m <<= 1) {
        const unsigned long long o = __shfl_xor(key, m);
        key = o < key ? o : key;
    }
    return key;
}

// Fixed-point scale for the probabilities of one split: with l_est = sum_t 2^(s_t - m) (fp32),
// 2^29 <= 2^e * l_est < 2^30, so no bin (each holds a partial sum of the p_t) can overflow 32
// bits, and each p_t is kept to an absolute error of 2^-(e+1) <= 2^-30 * l_est.
__device__ __forceinline__ int fixed_point_exponent(float l_est)
{
    int ex;
    (void)frexpf(l_est, &ex);           // l_est = f * 2^ex, f in [0.5, 1)
    return 30 - ex;
}

// Format constants.
// LONG (16 groups per head, b = 8 only): one column per group instead of two replicas, which
// leaves 48 instead of 32 words of every row for scores, i.e. splits of 12288 instead of 8192 tokens.
template <int GH, int B, bool LONG = false>
struct Fmt {
    static constexpr int K = 1 << B;                    // rows
    // replicas per group: two where a row would otherwise be 16 words and 4 lanes of a wavefront
    // would share each column; not for b = 10, whose 1024 rows would then fill 128 KB and leave
    // room for short splits only (fixed costs per split dominate that format)
    static constexpr int R = (GH == 16 && B == 8 && !LONG) ? 2 : 1;
    static constexpr int RW = B == 8 ? 64 : 16;         // words per row
    static constexpr bool SCORES_IN_TABLE = B == 8 && GH <= 32;   // behind the table's columns in each row
    static constexpr int LUT_WORDS = GH * R;            // words of a row that hold table columns
    static constexpr int SCORE_WORDS = 64 - LUT_WORDS;  // scores per row (SCORES_IN_TABLE)
    static constexpr int P = GH / 16;                   // 16-byte planes of low code bytes
    static constexpr int TAB_FLOATS = K * RW;
    static constexpr int TILE_BYTES = kTileTokens * GH * B / 8;
    static_assert(B == 8 || (B == 10 && GH == 16), "formats: b = 8, or b = 10 with 16 groups per head");
    static_assert(GH == 16 || GH == 32 || GH == 64, "groups per head must be 16, 32 or 64");
};

// Word column of lane `lane` when it handles group g.
template <int GH, int B, bool LONG>
__device__ __forceinline__ int column(int lane, int g)
{
    if constexpr (Fmt<GH, B, LONG>::R == 2) {
        return 2 * g + ((lane >> 4) & 1);       // lanes l and l + 16 differ, l and l + 32 share
    } else {
        (void)lane;
        return g;
    }
}

// 16 bytes of fp16 centroids: 8 / C consecutive centroids of one group.
struct Cent16 {
    unsigned w[4];
};
__device__ __forceinline__ Cent16 load_cent16(const uint16_t* p)
{
    const uint4 a = *reinterpret_cast<const uint4*>(p);
    return Cent16{{a.x, a.y, a.z, a.w}};
}

// The codes of one 64-token tile, one token per lane.
template <int GH, int B>
struct Tile {
    u32x4 lo[GH / 16];
    unsigned hi;                        // b = 10 only: bits [2s+1 : 2s] = high bits of slot s
};

template <int GH, int B>
__device__ __forceinline__ Tile<GH, B> load_tile(const uint8_t* base, int lane)
{
    Tile<GH, B> w;
    const u32x4* p = reinterpret_cast<const u32x4*>(base) + lane;
#pragma unroll
    for (int pl = 0; pl < GH / 16; ++pl) w.lo[pl] = __builtin_nontemporal_load(p + pl * 64);
    if constexpr (B == 10)
        w.hi = __builtin_nontemporal_load(reinterpret_cast<const unsigned*>(base + kTileTokens * GH) + lane);
    else
        w.hi = 0;
    return w;
}

// A wavefront's tiles of one code stream: tile k of its walk is tile first + k stride of the
// (sequence, KV head).  Contiguous cache: consecutive tiles are TILE_BYTES apart from `base`.
// Paged cache: lane j of `pages` holds the page of the walk's j-th tile (read once, before the
// walk; a walk has at most 64 tiles), and a tile sits at base + page * page_bytes.
template <int GH, int B>
struct TileWalk {
    const uint8_t* base;
    int first, stride;
    int pages;                  // per lane
    size_t page_bytes;          // 0: contiguous
    __device__ __forceinline__ const uint8_t* at(int k) const
    {
        if (page_bytes) return base + (size_t)__builtin_amdgcn_readlane(pages, k) * page_bytes;
        return base + (size_t)(first + k * stride) * Fmt<GH, B>::TILE_BYTES;
    }
};

// Per-lane column constants for the Gh steps: b = 8 packs 4 byte offsets per register (the
// v_perm_b32 picks one), b = 10 keeps one register per step.
template <int GH, int B, bool LONG = false>
struct Columns {
    unsigned v[B == 8 ? GH / 4 : GH];
    __device__ __forceinline__ void init(int lane)
    {
        if constexpr (B == 8) {
#pragma unroll
            for (int i = 0; i < GH / 4; ++i) {
                unsigned x = 0;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int g = (lane + 4 * i + k) & (GH - 1);
                    x |= (unsigned)(4 * column<GH, B, LONG>(lane, g)) << (8 * k);
                }
                v[i] = x;
            }
        } else {
#pragma unroll
            for (int s = 0; s < GH; ++s) v[s] = 4u * (unsigned)column<GH, B, LONG>(lane, (lane + s) & (GH - 1));
        }
    }
};

// Byte address of the table word for slot s of this lane's token.
template <int GH, int B, bool LONG>
__device__ __forceinline__ unsigned slot_addr(const Tile<GH, B>& w, const Columns<GH, B, LONG>& col, int s)
{
    const u32x4 q = w.lo[s >> 4];
    const int dw = (s >> 2) & 3;
    const unsigned code_word = dw == 0 ? q.x : dw == 1 ? q.y : dw == 2 ? q.z : q.w;
    const unsigned k = s & 3;
    if constexpr (B == 8) {
        const unsigned sel = 0x0c0c0000u | ((4u + k) << 8) | k;   // {0, 0, code byte k, column byte k}
        return __builtin_amdgcn_perm(code_word, col.v[s >> 2], sel);
    } else {
        const unsigned lo = (code_word >> (8 * k)) & 0xffu;
        const unsigned hi = (w.hi >> (2 * s)) & 3u;
        constexpr int SH = Fmt<GH, B>::RW == 32 ? 7 : 6;      // log2 of the row size in bytes
        return ((lo << SH) | (hi << (SH + 8))) | col.v[s];
    }
}

// Fused step: the codes of the new token as the cache layout would hold them (slot s of token u
// carries group (s + u) mod Gh), from keys[g] = group g's (distance, index) minimum.  Called by
// the one wavefront whose walk meets the token's tile, before its walk starts: lane i builds
// word i of the record, and every lane receives all words (wave-uniform values).
template <int GH, int B>
struct NewTokenCodes {
    unsigned lo[GH / 4];
    unsigned hi;                        // b = 10 only
    __device__ __forceinline__ void build(const unsigned long long* keys, int u_new, int lane)
    {
        unsigned x = 0, h = 0;
        if (lane < GH / 4) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int s = 4 * lane + k;
                const unsigned code = (unsigned)(keys[(s + u_new) & (GH - 1)] & 0xffffffffu);
                x |= (code & 0xffu) << (8 * k);
                if constexpr (B == 10) h |= (code >> 8) << (2 * s);
            }
        }
#pragma unroll
        for (int i = 0; i < GH / 4; ++i) lo[i] = __builtin_amdgcn_readlane(x, i);
        hi = 0;
        if constexpr (B == 10) {
#pragma unroll
            for (int i = 0; i < GH / 4; ++i) hi |= __builtin_amdgcn_readlane(h, i);
        }
    }
    // lane u_new's token of tile w becomes the new token
    __device__ __forceinline__ void patch(Tile<GH, B>& w, int u_new, int lane) const
    {
        const bool mine = lane == u_new;
#pragma unroll
        for (int pl = 0; pl < GH / 16; ++pl) {
            u32x4 q = w.lo[pl];
            q.x = mine ? lo[4 * pl] : q.x;
            q.y = mine ? lo[4 * pl + 1] : q.y;
            q.z = mine ? lo[4 * pl + 2] : q.z;
            q.w = mine ? lo[4 * pl + 3] : q.w;
            w.lo[pl] = q;
        }
        if constexpr (B == 10) w.hi = mine ? hi : w.hi;
    }
};

// Fused step: store the new token's codes of one KV head into its cache tile.
template <int GH, int B>
__device__ __forceinline__ void store_new_codes(uint8_t* tile, const unsigned long long* keys, int u_new, int tid)
{
    if (tid < GH) {
        const unsigned code = (unsigned)(keys[tid] & 0xffffffffu);
        const int slot = (tid - u_new) & (GH - 1);
        tile[(slot >> 4) * 1024 + u_new * 16 + (slot & 15)] = (uint8_t)(code & 0xffu);
    }
    if constexpr (B == 10) {
        if (tid == 0) {                 // the token's high-bit word belongs to this (token, head) alone
            unsigned hi = 0;
#pragma unroll
            for (int g = 0; g < GH; ++g) {
                const unsigned code = (unsigned)(keys[g] & 0xffffffffu);
                hi |= (code >> 8) << (2 * ((g - u_new) & (GH - 1)));
            }
            *reinterpret_cast<unsigned*>(tile + kTileTokens * GH + u_new * 4) = hi;
        }
    }
}

// Walk tiles first, first + stride, ... (n of them) of a code stream with PF tiles in flight.
// begin() requests the first tiles (so that the latency overlaps whatever the caller does
// next); run() consumes.  The steady state is straight-line code (consume one tile, request the
// tile PF steps ahead) so that the compiler keeps PF loads outstanding; the last tiles are
// requested together and then consumed.  `fn(words, k)` is called once per tile k = 0 .. n-1.
template <int GH, int B, int PF>
struct Streamer {
    static constexpr int TAIL = 2 * PF - 1;
    Tile<GH, B> buf[TAIL];

    __device__ __forceinline__ void begin(const TileWalk<GH, B>& tw, int n, int lane)
    {
        if (n >= 2 * PF) {
#pragma unroll
            for (int i = 0; i < PF; ++i) {
                buf[i] = load_tile<GH, B>(tw.at(i), lane);
                __builtin_amdgcn_sched_barrier(0);      // keep request order == consumption order
            }
        } else {
#pragma unroll
            for (int i = 0; i < TAIL; ++i)
                if (i < n) buf[i] = load_tile<GH, B>(tw.at(i), lane);
        }
    }

    // `last_requests()` is called once, after the last tile has been requested and before the
    // last tiles are consumed: loads the caller issues there ride behind the stream.
    template <class Fn, class Hook>
    __device__ __forceinline__ void run(const TileWalk<GH, B>& tw, int n, int lane, Fn&& fn, Hook&& last_requests)
    {
        int k = 0;
        if (n >= 2 * PF) {
            for (; k + 2 * PF <= n; k += PF) {
#pragma unroll
                for (int i = 0; i < PF; ++i) {
                    fn(buf[i], k + i);
                    buf[i] = load_tile<GH, B>(tw.at(k + PF + i), lane);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
#pragma unroll
            for (int i = 0; i < PF; ++i) fn(buf[i], k + i);
            k += PF;
#pragma unroll
            for (int i = 0; i < TAIL; ++i)
                if (k + i < n) buf[i] = load_tile<GH, B>(tw.at(k + i), lane);
        }
        last_requests();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < TAIL; ++i)
            if (k + i < n) fn(buf[i], k + i);
    }
};

}  // namespace
}  // namespace cq

// Nearest-centroid encoding of many tokens (Section 3.2 of the paper) with the matrix cores of
// gfx950 as a FILTER and the exact fp32 search as the judge.
//
// For one group (c channels, K = 2^b centroids) and a tile of tokens, argmin_j |x - c_j|^2 =
// argmax_j (x . c_j - |c_j|^2 / 2).  One MFMA evaluates that score for 32 tokens x 32 centroids:
// the K dimension of the matrix product carries the c channels plus three fp16 pieces of
// -|c_j|^2 / 2 (their sum is exact to fp32 precision; see "Scaling").  The two largest scores of a
// token are then found in two levels: each lane keeps the two largest QUAD maxima it sees (the
// maximum of four scores, with the quad's number packed into its five lowest mantissa bits:
// 1.2 VALU instructions per score instead of the 2 c + 3 of the direct form), and the four
// scores of the winning quad are evaluated once more, with packed dot products in fp32.
//
// Scaling.  A group whose largest |c_j|^2 is small is multiplied (centroids and tokens alike)
// by a power of two 2^s, s >= 0, that brings the largest scaled |c'|^2 into [2^12, 2^14): the
// pieces of |c'|^2 / 2 then sit well inside fp16's normal range however small the data (the
// argmax does not change and scaling up is exact).  Nothing is scaled down: a group whose
// |c|^2 / 2 would not fit fp16 (|c|^2 >= 60000), and a token whose scaled channels would not,
// are handed to the exact path whole.
//
// Error bound.  With M = |x'| |c'|_max + |c'|_max^2 / 2 >= sum of the absolute values of the
// terms of any score, in units of 2^-20 M.  A quad maximum from the matrix core: |c|^2 summed in
// fp32 (0.5); the matrix core aligns the exact products to the largest one and drops what falls
// below about 2^-24 of it -- at most 2^-23 M for each of at most 11 terms and the final rounding
// (1.5; measured on such operands: never above 0.2); the five packed bits move a score by less
// than 32 units in its last place (3.9): 5.9 in all.  A score of the winning quad from the
// vector ALU: |c|^2 (0.5), c / 2 + 2 roundings to fp32 (0.4), two packed bits (0.5): 1.4.  The
// best is always of the second kind, the runner-up of either, so the two compare correctly
// whenever they differ by more than 7.3 units; the test below uses 8 = 2^-17 M.  (If rounding
// made the wrong quad win, the true best's quad maximum is the runner-up and lies within 7.3
// units of the reported best: the test fails and the pair is re-done.)  If the best beats the
// runner-up by more than that, the best IS the
// nearest centroid in exact arithmetic.  Otherwise (a near tie or an exact tie) the (token,
// group) pair is re-done at once by the direct form -- sum_i (x_i - c_i)^2 in fp32, channel
// order, lowest index on ties; on the scaled values, which changes no bit of the comparison --
// by the whole wavefront, from the codebook copy in LDS.  The result is
// the exact nearest centroid wherever the two nearest are separated by more than the bound, and
// the direct fp32 form's choice elsewhere.
//
// This file is compiled with -fno-honor-nans: the maxima below are then bare v_max3_f32 /
// v_med3_f32 without canonicalisation of their inputs.  Non-finite activations or centroids
// give unspecified codes (always in range), as they do in the direct form.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "cq_internal.hpp"

namespace cq {
namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

template <int C>
struct Aug {
    static constexpr int KDIM = C == 8 ? 16 : 8;        // K of the MFMA = halfs per centroid record
    static constexpr int HALF = KDIM / 2;               // halfs per lane operand
    using vec_t = std::conditional_t<C == 8, half8_t, half4_t>;
};

template <int C>
__device__ __forceinline__ float16_t mfma(typename Aug<C>::vec_t a, typename Aug<C>::vec_t b)
{
    const float16_t zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if constexpr (C == 8) return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, zero, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_32x32x8f16(a, b, zero, 0, 0, 0);
}

// Direct form: sum_i (x_i - c_i)^2 in fp32, channel order (its bits order like its value).
template <int C>
__device__ __forceinline__ unsigned exact_distance_bits(const float (&x)[C], const unsigned (&cw)[C / 2])
{
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < C / 2; ++i) {
        const half2_t h = __builtin_bit_cast(half2_t, cw[i]);
        const float d0 = x[2 * i] - (float)h.x;
        acc = __builtin_fmaf(d0, d0, acc);
        const float d1 = x[2 * i + 1] - (float)h.y;
        acc = __builtin_fmaf(d1, d1, acc);
    }
    return __float_as_uint(acc);
}

// Minimum of v over the 64 lanes (all active), wavefront-uniform: four DPP steps inside each
// row of 16 lanes, then the four row results through scalar registers.
template <int CTRL>
__device__ __forceinline__ unsigned dpp_min(unsigned v)
{
    const unsigned o = (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xf, 0xf, false);
    return o < v ? o : v;
}
__device__ __forceinline__ unsigned wave_min_u32(unsigned v)
{
    v = dpp_min<0xB1>(v);      // quad_perm [1,0,3,2]
    v = dpp_min<0x4E>(v);      // quad_perm [2,3,0,1]
    v = dpp_min<0x141>(v);     // row_half_mirror
    v = dpp_min<0x140>(v);     // row_mirror
    const unsigned r0 = (unsigned)__builtin_amdgcn_readlane((int)v, 0), r1 = (unsigned)__builtin_amdgcn_readlane((int)v, 16);
    const unsigned r2 = (unsigned)__builtin_amdgcn_readlane((int)v, 32), r3 = (unsigned)__builtin_amdgcn_readlane((int)v, 48);
    const unsigned a = r0 < r1 ? r0 : r1, b = r2 < r3 ? r2 : r3;
    return a < b ? a : b;
}

template <int CTRL>
__device__ __forceinline__ unsigned dpp_max(unsigned v)
{
    const unsigned o = (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xf, 0xf, false);
    return o > v ? o : v;
}
__device__ __forceinline__ unsigned wave_max_u32(unsigned v)
{
    v = dpp_max<0xB1>(v);
    v = dpp_max<0x4E>(v);
    v = dpp_max<0x141>(v);
    v = dpp_max<0x140>(v);
    const unsigned r0 = (unsigned)__builtin_amdgcn_readlane((int)v, 0), r1 = (unsigned)__builtin_amdgcn_readlane((int)v, 16);
    const unsigned r2 = (unsigned)__builtin_amdgcn_readlane((int)v, 32), r3 = (unsigned)__builtin_amdgcn_readlane((int)v, 48);
    const unsigned a = r0 > r1 ? r0 : r1, b = r2 > r3 ? r2 : r3;
    return a > b ? a : b;
}

// |c|^2 of the fp16 pairs in n words, fp32, channel order
template <int N>
__device__ __forceinline__ float norm2(const unsigned (&w)[N])
{
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const half2_t h = __builtin_bit_cast(half2_t, w[i]);
        s = __builtin_fmaf((float)h.x, (float)h.x, s);
        s = __builtin_fmaf((float)h.y, (float)h.y, s);
    }
    return s;
}
// The same for SCALED values (of a group's centroids, of a token's slice), whose norm lies far
// above fp16's subnormals: exact products summed in fp32 pair by pair (v_dot2_f32_f16, one
// instruction per pair instead of two conversions and two multiply-adds).  Whatever that
// instruction does with a subnormal component, its square is below 4e-9 against a unit of the
// error bound of 2e-3 or more.
template <int N>
__device__ __forceinline__ float norm2_scaled(const unsigned (&w)[N])
{
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const half2_t h = __builtin_bit_cast(half2_t, w[i]);
        s = __builtin_amdgcn_fdot2(h, h, s, false);
    }
    return s;
}

// The group's power-of-two scale from its largest |c|^2 (bits of a non-negative float):
// s >= 0 with 4^s c2max in [2^12, 2^14) when c2max < 2^12, else s = 0; at most 30 (fp16 data
// needs no more; an all-zero group gets 30 and ties everywhere).
struct GroupScale {
    half2_t m1, m2;         // 2^s = m1 * m2, both fp16 powers of two
    float f1, f2;           // 2^s, 4^s
    float c2max_scaled;     // c2max * 4^s
    bool too_big;           // |c|^2 / 2 would not fit fp16: the filter steps aside
};
// (c2bits is wavefront-uniform: everything here but one multiplication is scalar integer work)
__device__ __forceinline__ GroupScale group_scale(unsigned c2bits)
{
    GroupScale r;
    const int e = (int)((c2bits >> 23) & 0xffu) - 127;
    int s = (13 - e) >> 1;
    s = s > 30 ? 30 : (s < 0 ? 0 : s);
    const int s1 = s >> 1, s2 = s - s1;                     // both at most 15: 2^15 is an fp16 number
    const unsigned a = (unsigned)(15 + s1) << 10, b = (unsigned)(15 + s2) << 10;     // fp16 bits of 2^s1, 2^s2
    r.m1 = __builtin_bit_cast(half2_t, a | (a << 16));
    r.m2 = __builtin_bit_cast(half2_t, b | (b << 16));
    r.f1 = __uint_as_float((unsigned)(127 + s) << 23);
    r.f2 = __uint_as_float((unsigned)(127 + 2 * s) << 23);
    r.c2max_scaled = __uint_as_float(c2bits) * r.f2;
    r.too_big = c2bits >= 0x476a6000u;                      // |c|^2 >= 60000 (bits of a non-negative float order like it)
    return r;
}
__device__ __forceinline__ unsigned scale_pair(unsigned w, const GroupScale& gs)
{
    return __builtin_bit_cast(unsigned, __builtin_bit_cast(half2_t, w) * gs.m1 * gs.m2);
}

// GS (group split): the NW wavefronts of a workgroup share TILES tiles and take GH / NW groups
// each, for every one of those tiles; a wavefront stages its groups' codebooks by itself, into a
// buffer of its own, so nothing but the final store of the tiles' records is synchronised across
// the workgroup.  TILES = 1 spreads a small problem over the chip (a wavefront's chain of groups
// is the latency of such a call); TILES = NW costs the staging of the shared-buffer form
// without its barrier per group.
template <int GH, int C, int B, int NW, bool GS = false, int TILES = 1>
__global__ __launch_bounds__(NW * 64) void encode_mfma_kernel(EncodeArgs a)
{
    static_assert(!GS || (B == 8 && GH % NW == 0), "group split: byte codes, groups divisible among the wavefronts");
    static_assert(GS || TILES == 1, "several tiles per wavefront: group split only");
    using A = Aug<C>;
    using vec_t = typename A::vec_t;
    constexpr int K = 1 << B;
    constexpr int NT = NW * 64;
    constexpr int KDIM = A::KDIM, HALF = A::HALF;
    constexpr int NBLK = K / 32;                     // 32-centroid blocks
    constexpr int NSB = NBLK / 8;                    // runs of 8 blocks (the packed quad number has 5 bits)
    constexpr int P = GH / 16;
    constexpr int TILE_LOW = kTileTokens * GH;
    constexpr int TILE_BYTES = kTileTokens * GH * B / 8;
    constexpr float LOWEST = -3.0e38f;

    constexpr int SNT = GS ? 64 : NT;                // threads that stage a group's codebook together
    constexpr int NTILE = GS ? TILES : NW;           // tiles per workgroup
    constexpr int TPW = GS ? TILES : 1;              // tiles per wavefront
    // augmented codebook records: two buffers that the workgroup alternates, or (GS) one per wavefront
    __shared__ __attribute__((aligned(16))) _Float16 cba[GS ? NW : 2][K * KDIM];
    __shared__ unsigned c2bits[GH];                                       // bits of max_j |c_j|^2 per group
    __shared__ __attribute__((aligned(16))) uint8_t rec[NTILE][TILE_LOW];  // low code bytes, cache order
    __shared__ uint16_t code16[B == 10 ? NW : 1][B == 10 ? kTileTokens : 1][B == 10 ? GH : 1];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int stid = GS ? lane : tid;                // index among the threads that stage together
    const int hkv = blockIdx.y;
    const int n = blockIdx.z % a.batch;
    const EncodeTensor& ten = a.tensor[blockIdx.z / a.batch];

    const int first_tile = a.t_offset / kTileTokens;
    const int t_end = a.t_offset + a.t_new;
    const int last_tile = (t_end - 1) / kTileTokens;
    // tile t of this wavefront (GS: of the workgroup); this lane's token in it (cache position)
    auto tile_index = [&](int t) { return GS ? t : wave; };
    auto tile_at = [&](int t) { return first_tile + (int)blockIdx.x * NTILE + tile_index(t); };
    auto valid_at = [&](int t) {
        const int pos = tile_at(t) * kTileTokens + lane;
        return pos >= a.t_offset && pos < t_end;
    };
    const uint16_t* xbase = ten.x + (size_t)n * ten.x_batch_stride + (size_t)hkv * GH * C;
    auto xrow_at = [&](int t) {
        const int pos = tile_at(t) * kTileTokens + lane;
        return xbase + (size_t)(valid_at(t) ? pos - a.t_offset : 0) * ten.x_row_stride;
    };

    // Staging of a group's codebook is split in two so that the global loads of group g + 1 fly
    // while group g is computed: fetch() issues them into registers, commit() turns centroid j
    // into its record [channels | three pieces of -|c|^2/2, zeros] in LDS.
    constexpr int SPT = (K + SNT - 1) / SNT;         // centroids staged per thread
    unsigned craw[SPT][C / 2];
    auto fetch = [&](int g) {
        const uint16_t* src = ten.centroids + (size_t)(hkv * GH + g) * K * C;
#pragma unroll
        for (int k = 0; k < SPT; ++k) {
            const int j = stid + k * SNT;
            if (j < K) {
#pragma unroll
                for (int i = 0; i < C / 2; ++i) craw[k][i] = *reinterpret_cast<const unsigned*>(src + j * C + 2 * i);
            }
        }
    };
    // bits of max_j |c_j|^2 of the group being committed.  Not GS: from the prologue pass below.  GS:
    // the wavefront holds the whole group in craw and takes the maximum itself (c2_staged then
    // serves the group's turn in the main loop), which spares the small call that pass
    unsigned c2_staged = 0;
    auto commit = [&](int buf, int g) {
        unsigned c2;
        if constexpr (GS) {
            float m = 0.f;
#pragma unroll
            for (int k = 0; k < SPT; ++k)
                if (stid + k * SNT < K) m = fmaxf(m, norm2<C / 2>(craw[k]));
            c2 = c2_staged = wave_max_u32(__float_as_uint(m));
        } else {
            c2 = (unsigned)__builtin_amdgcn_readfirstlane((int)c2bits[g]);
        }
        const GroupScale gs = group_scale(c2);
#pragma unroll
        for (int k = 0; k < SPT; ++k) {
            const int j = stid + k * SNT;
            if (j >= K) continue;
            unsigned cs[C / 2];
#pragma unroll
            for (int i = 0; i < C / 2; ++i) cs[i] = scale_pair(craw[k][i], gs);
            const float v = gs.too_big ? 0.f : -0.5f * norm2_scaled<C / 2>(cs);          // -|c'|^2 / 2
            const _Float16 h1 = (_Float16)v;
            const float r1 = v - (float)h1;
            const _Float16 h2 = (_Float16)r1;
            const _Float16 h3 = (_Float16)(r1 - (float)h2);
            const _Float16 zero = (_Float16)0.0f;
            const unsigned w12 = __builtin_bit_cast(unsigned, half2_t{h1, h2});
            const unsigned w30 = __builtin_bit_cast(unsigned, half2_t{h3, zero});
            uint4* dst = reinterpret_cast<uint4*>(&cba[buf][j * KDIM]);
            if constexpr (C == 8) {
                dst[0] = make_uint4(cs[0], cs[1], cs[2], cs[3]);
                dst[1] = make_uint4(w12, w30, 0u, 0u);
            } else if constexpr (C == 4) {
                dst[0] = make_uint4(cs[0], cs[1], w12, w30);
            } else {
                dst[0] = make_uint4(cs[0], w12, w30, 0u);
            }
        }
    };
    auto load_x = [&](int g, int t, unsigned (&dst)[C / 2]) {
        const uint16_t* xrow = xrow_at(t);
#pragma unroll
        for (int i = 0; i < C / 2; ++i) dst[i] = *reinterpret_cast<const unsigned*>(xrow + g * C + 2 * i);
    };

    // max_j |c_j|^2 of every group of this head: each thread takes 16-byte pieces of the head's
    // codebooks; a group's pieces are a multiple of 64, so a wavefront works on one group at a time
    if constexpr (!GS) {
        constexpr int CH = K * C / 8;                // 16-byte pieces per group
        constexpr int ROUNDS = GH * CH / NT;
        static_assert(CH % 64 == 0 && (GH * CH) % NT == 0, "a wavefront's pieces must share a group");
        for (int i = tid; i < GH; i += NT) c2bits[i] = 0u;
        __syncthreads();
        const uint4* cen16 = reinterpret_cast<const uint4*>(ten.centroids + (size_t)hkv * GH * K * C);
        constexpr int RPG = CH >= NT ? CH / NT : 1;      // consecutive rounds inside one group
        constexpr int STEPS = ROUNDS / RPG;
        constexpr int UNR = RPG >= 16 ? 1 : 16 / RPG;    // about 16 loads in flight
#pragma unroll UNR
        for (int st = 0; st < STEPS; ++st) {
            float m = 0.f;
#pragma unroll
            for (int rr = 0; rr < RPG; ++rr) {
                const uint4 w = cen16[(st * RPG + rr) * NT + tid];
                if constexpr (C == 8) {
                    const unsigned a0[4] = {w.x, w.y, w.z, w.w};
                    m = fmaxf(m, norm2<4>(a0));
                } else if constexpr (C == 4) {
                    const unsigned a0[2] = {w.x, w.y}, a1[2] = {w.z, w.w};
                    m = fmaxf(m, fmaxf(norm2<2>(a0), norm2<2>(a1)));
                } else {
                    const unsigned a0[1] = {w.x}, a1[1] = {w.y}, a2[1] = {w.z}, a3[1] = {w.w};
                    m = fmaxf(m, fmaxf(fmaxf(norm2<1>(a0), norm2<1>(a1)), fmaxf(norm2<1>(a2), norm2<1>(a3))));
                }
            }
            const unsigned mb = wave_max_u32(__float_as_uint(m));
            if (lane == 0) atomicMax(&c2bits[(st * RPG * NT + wave * 64) / CH], mb);
        }
        __syncthreads();
    }

    const int g_begin = GS ? wave * (GH / NW) : 0, g_end = GS ? g_begin + GH / NW : GH;
    fetch(g_begin);
    commit(GS ? wave : 0, g_begin);
    // the token slices of the tiles to come, in the order of their use: xnext[0] is the next one
    unsigned xnext[TPW][C / 2];
#pragma unroll
    for (int t = 0; t < TPW; ++t) load_x(g_begin, t, xnext[t]);
    if constexpr (!GS) __syncthreads();
    for (int g = g_begin; g < g_end; ++g) {
        const int buf = GS ? wave : (g & 1);
        const GroupScale gs = group_scale(GS ? c2_staged : (unsigned)__builtin_amdgcn_readfirstlane((int)c2bits[g]));
        if (g + 1 < g_end) fetch(g + 1);
#pragma unroll 1
        for (int t = 0; t < TPW; ++t) {
            const int ti = tile_index(t);
            // this lane's token: its slice of the group (fetched one group ahead), scaled, and |x'|^2
            unsigned xw[C / 2], xs[C / 2];
#pragma unroll
            for (int i = 0; i < C / 2; ++i) xw[i] = xnext[0][i];
            // (the slices loaded earlier move up before the new request goes out: nothing in flight is touched)
#pragma unroll
            for (int k = 0; k + 1 < TPW; ++k)
#pragma unroll
                for (int i = 0; i < C / 2; ++i) xnext[k][i] = xnext[k + 1][i];
            if (g + 1 < g_end) load_x(g + 1, t, xnext[TPW - 1]);
            if (TPW > 1 && tile_at(t) > last_tile) continue;        // (a workgroup's tiles beyond the call's last)
#pragma unroll
            for (int i = 0; i < C / 2; ++i) xs[i] = scale_pair(xw[i], gs);
            const float x2 = norm2_scaled<C / 2>(xs);                // (infinite where the scaling overflowed)
            const bool x_over = !(x2 < 1.0e9f);                      // |x'| beyond 2^15: not as fp16
#pragma unroll
            for (int i = 0; i < C / 2; ++i) xs[i] = x_over ? 0u : xs[i];
            // 2^-17 M with M >= |x'| |c'|max + |c'|max^2 / 2 (1 % slack for the roundings of this line)
            const float thr = (1.01f * (__builtin_sqrtf(x2 * gs.c2max_scaled) + 0.5f * gs.c2max_scaled)) * (1.0f / 131072.0f);
            const bool exact_only = gs.too_big || x_over;

            // Level 1, once per half of the tile (tokens 32 h .. 32 h + 31 are the 32 columns of the
            // matrix product): the two largest of the lane's 16 NBLK scores.  The maximum of every quad
            // of scores (the 4 consecutive centroids 8 q + 4 (lane / 32) .. + 3 of a block: registers
            // 4 q .. 4 q + 3) with the quad's number, 4 (blk % 8) + q, packed into its five lowest
            // mantissa bits, and a running (best, runner-up) over those: 1.2 VALU instructions per
            // score instead of the 2.8 of tracking every score.
            float hbest[2], hsecond[2];
            int hsb[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                // B operand: lanes < 32 carry the channels of token 32 h + lane (their own for h = 0,
                // the partner lane's for h = 1), lanes >= 32 the ones that pick up the pieces of
                // -|c|^2 / 2
                unsigned xh[C / 2];
#pragma unroll
                for (int i = 0; i < C / 2; ++i) xh[i] = h == 0 ? xs[i] : __shfl_xor(xs[i], 32);
                const _Float16 one = (_Float16)1.0f, zero = (_Float16)0.0f;
                vec_t bop;
                if constexpr (C == 8) {
                    if (lane < 32) {
                        const half2_t p0 = __builtin_bit_cast(half2_t, xh[0]), p1 = __builtin_bit_cast(half2_t, xh[1]);
                        const half2_t p2 = __builtin_bit_cast(half2_t, xh[2]), p3 = __builtin_bit_cast(half2_t, xh[3]);
                        bop = vec_t{p0.x, p0.y, p1.x, p1.y, p2.x, p2.y, p3.x, p3.y};
                    } else {
                        bop = vec_t{one, one, one, zero, zero, zero, zero, zero};
                    }
                } else if constexpr (C == 4) {
                    if (lane < 32) {
                        const half2_t p0 = __builtin_bit_cast(half2_t, xh[0]), p1 = __builtin_bit_cast(half2_t, xh[1]);
                        bop = vec_t{p0.x, p0.y, p1.x, p1.y};
                    } else {
                        bop = vec_t{one, one, one, zero};
                    }
                } else {
                    if (lane < 32) {
                        const half2_t p0 = __builtin_bit_cast(half2_t, xh[0]);
                        bop = vec_t{p0.x, p0.y, one, one};
                    } else {
                        bop = vec_t{one, zero, zero, zero};
                    }
                }

                float gbest = LOWEST, gsecond = LOWEST;
                int gsb = 0;                                 // block / 8 of gbest (more than 8 blocks: b = 10)
#pragma unroll 1
                for (int sb = 0; sb < NSB; ++sb) {
                    float sbest = LOWEST, ssecond = LOWEST;
#pragma unroll                  // (whole: the quad numbers are then immediates of one v_and_or_b32)
                    for (int b8 = 0; b8 < 8; ++b8) {
                        const int blk = sb * 8 + b8;
                        const vec_t aop = *reinterpret_cast<const vec_t*>(&cba[buf][(blk * 32 + (lane & 31)) * KDIM + (lane >> 5) * HALF]);
                        const float16_t d = mfma<C>(aop, bop);
                        float qm[4];
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const float m = fmaxf(fmaxf(fmaxf(d[4 * q], d[4 * q + 1]), d[4 * q + 2]), d[4 * q + 3]);
                            qm[q] = __uint_as_float((__float_as_uint(m) & 0xffffffe0u) | (unsigned)(4 * b8 + q));
                        }
                        // two quads per step: the runner-up of {best, second, k1, k2} with second <= best
                        // is max(median(best, k1, k2), second)
#pragma unroll
                        for (int q = 0; q < 4; q += 2) {
                            ssecond = fmaxf(ssecond, __builtin_amdgcn_fmed3f(sbest, qm[q], qm[q + 1]));
                            sbest = fmaxf(fmaxf(sbest, qm[q]), qm[q + 1]);
                        }
                    }
                    if constexpr (NSB == 1) {
                        gbest = sbest;
                        gsecond = ssecond;
                    } else {
                        gsecond = fmaxf(fmaxf(fminf(gbest, sbest), gsecond), ssecond);
                        gsb = sbest > gbest ? sb : gsb;
                        gbest = fmaxf(gbest, sbest);
                    }
                }
                hbest[h] = gbest;
                hsecond[h] = gsecond;
                hsb[h] = gsb;
            }
            // Lanes l and l + 32 saw the two halves of every block's rows for tokens l % 32 (h = 0) and
            // 32 + l % 32 (h = 1).  Each lane now takes its OWN token (token `lane`, in half lane / 32):
            // its own scan of that half, and the partner lane's, which sends it in exchange for the
            // other half's.  Everything below runs once per tile and group, on all 64 lanes.
            const int hi = lane >> 5;
            const float gbest = hi ? hbest[1] : hbest[0], gsecond = hi ? hsecond[1] : hsecond[0];
            const float obest = __shfl_xor(hi ? hbest[0] : hbest[1], 32), osecond = __shfl_xor(hi ? hsecond[0] : hsecond[1], 32);
            const int gsb = hi ? hsb[1] : hsb[0];
            const int osb = NSB == 1 ? 0 : __shfl_xor(hi ? hsb[0] : hsb[1], 32);
            const bool other = obest > gbest;
            const float best = fmaxf(gbest, obest);
            const float second = fmaxf(fmaxf(fminf(gbest, obest), gsecond), osecond);
            const int wsb = other ? osb : gsb;
            const int whalf = other ? 1 - hi : hi;
            const int u = lane;                                      // token of the tile
            const int slot = (g - u) & (GH - 1);
            // Level 2: the winning quad's four centroids against this token, x . c - |c|^2 / 2 in fp32
            // from the records in LDS.
            const int quad = (int)(__float_as_uint(best) & 31u);
            const int j0 = (wsb * 8 + (quad >> 2)) * 32 + 8 * (quad & 3) + 4 * whalf;
            // (v_dot2_f32_f16: exact products of the fp16 pairs, fp32 sums; the centroid's number
            // within the quad rides in the two lowest mantissa bits)
            float qk[4];
            const half2_t ones = half2_t{(_Float16)1.0f, (_Float16)1.0f};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const unsigned* r = reinterpret_cast<const unsigned*>(&cba[buf][(j0 + e) * KDIM]);
                unsigned w[C / 2 + 2];
                if constexpr (C == 8) {
                    const uint4 a0 = *reinterpret_cast<const uint4*>(r);
                    const uint2 a1 = *reinterpret_cast<const uint2*>(r + 4);
                    w[0] = a0.x; w[1] = a0.y; w[2] = a0.z; w[3] = a0.w; w[4] = a1.x; w[5] = a1.y;
                } else if constexpr (C == 4) {
                    const uint4 a0 = *reinterpret_cast<const uint4*>(r);
                    w[0] = a0.x; w[1] = a0.y; w[2] = a0.z; w[3] = a0.w;
                } else {
                    const uint4 a0 = *reinterpret_cast<const uint4*>(r);
                    w[0] = a0.x; w[1] = a0.y; w[2] = a0.z;
                }
                // the three pieces of -|c|^2 / 2 sit behind the C channels: (h1, h2), (h3, 0)
                float sc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, w[C / 2 + 1]), ones, 0.f, false);
                sc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, w[C / 2]), ones, sc, false);
#pragma unroll
                for (int i = 0; i < C / 2; ++i)
                    sc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, xs[i]), __builtin_bit_cast(half2_t, w[i]), sc, false);
                qk[e] = __uint_as_float((__float_as_uint(sc) & 0xfffffffcu) | (unsigned)e);
            }
            const float q01 = fmaxf(qk[0], qk[1]);
            const float qbest_k = fmaxf(fmaxf(q01, qk[2]), qk[3]);
            const float qsecond = fmaxf(fminf(qk[0], qk[1]), __builtin_amdgcn_fmed3f(q01, qk[2], qk[3]));
            const int qarg = (int)(__float_as_uint(qbest_k) & 3u);
            const float qbest = __uint_as_float(__float_as_uint(qbest_k) & 0xfffffffcu);
            bool unsure;
            {
                const int code = j0 + qarg;
                const float sv = fmaxf(__uint_as_float(__float_as_uint(second) & 0xffffffe0u), qsecond);
                unsure = !(qbest - sv > thr) || exact_only;
                rec[ti][(slot >> 4) * 1024 + u * 16 + (slot & 15)] = (uint8_t)(code & 0xff);
                if constexpr (B == 10) code16[wave][u][g] = (uint16_t)code;
            }

            // exact re-do of the unsure tokens of this tile, one at a time by the whole wavefront
            unsigned long long todo = __ballot(unsure);
            while (todo) {
                const int r = (int)__builtin_ctzll(todo);
                todo &= todo - 1;
                float x[C];
#pragma unroll
                for (int i = 0; i < C / 2; ++i) {
                    const half2_t hh = __builtin_bit_cast(half2_t, (unsigned)__builtin_amdgcn_readlane((int)xw[i], r));
                    x[2 * i] = (float)hh.x * gs.f1;                // exact in fp32
                    x[2 * i + 1] = (float)hh.y * gs.f1;
                }
                unsigned dmin = ~0u, jmin = 0;
#pragma unroll 4
                for (int j = lane; j < K; j += 64) {
                    unsigned cw[C / 2];
#pragma unroll
                    for (int i = 0; i < C / 2; ++i) cw[i] = *reinterpret_cast<const unsigned*>(&cba[buf][j * KDIM + 2 * i]);
                    const unsigned dj = exact_distance_bits<C>(x, cw);
                    jmin = dj < dmin ? (unsigned)j : jmin;       // increasing j: the lowest index stays on ties
                    dmin = dj < dmin ? dj : dmin;
                }
                const unsigned wmin = wave_min_u32(dmin);
                // the lowest index among the lanes that hold the minimum: almost always one lane
                const unsigned long long holders = __ballot(dmin == wmin);
                unsigned code;
                if ((holders & (holders - 1)) == 0) code = (unsigned)__builtin_amdgcn_readlane((int)jmin, (int)__builtin_ctzll(holders));
                else code = wave_min_u32(dmin == wmin ? jmin : ~0u);
                if (lane == r) {
                    rec[ti][(slot >> 4) * 1024 + u * 16 + (slot & 15)] = (uint8_t)(code & 0xff);
                    if constexpr (B == 10) code16[wave][u][g] = (uint16_t)code;
                }
            }
        }
        // (GS: the wavefront is the only reader of its buffer, and its LDS operations keep their order)
        if (g + 1 < g_end) commit(GS ? wave : buf ^ 1, g + 1);
        if constexpr (!GS) __syncthreads();
    }
    if constexpr (GS) __syncthreads();  // the tiles' codes of all groups are in rec

    // store this lane's token (GS: the wavefronts share the workgroup's tiles out)
    for (int t = GS ? wave : 0; t < (GS ? TILES : 1); t += GS ? NW : 1) {
        if (!valid_at(t)) continue;
        const int ti = tile_index(t);
        uint8_t* tp = ten.codes + a.map.tile_index(n, hkv, tile_at(t)) * TILE_BYTES;
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const uint4 v = *reinterpret_cast<const uint4*>(&rec[ti][p * 1024 + lane * 16]);
            *reinterpret_cast<uint4*>(tp + p * 1024 + lane * 16) = v;
        }
        if constexpr (B == 10) {
            unsigned hi = 0;
#pragma unroll
            for (int g = 0; g < GH; ++g)
                hi |= (unsigned)(code16[wave][lane][g] >> 8) << (2 * ((g - lane) & (GH - 1)));
            *reinterpret_cast<unsigned*>(tp + TILE_LOW + lane * 4) = hi;
        }
    }
}

// Byte codes: up to kGroupSplitEightBelow (tile, head, sequence, tensor) items eight wavefronts
// share a tile, below kGroupSplitBelow (and for sequences of fewer than four tiles) four; larger
// calls give four tiles to a workgroup of four wavefronts.
constexpr long kGroupSplitBelow = 4096;
constexpr long kGroupSplitEightBelow = 1024;

template <int GH, int C, int B>
cq_status launch_mfma_format(const EncodeArgs& a, hipStream_t stream)
{
    const int first_tile = a.t_offset / kTileTokens;
    const int last_tile = (a.t_offset + a.t_new - 1) / kTileTokens;
    const int n_tiles = last_tile - first_tile + 1;
    const long wave_tiles = (long)n_tiles * a.f.n_kv_heads * a.batch * a.n_tensors;
    const unsigned gy = (unsigned)a.f.n_kv_heads, gz = (unsigned)(a.batch * a.n_tensors);
    if constexpr (B == 8) {
        if (wave_tiles <= kGroupSplitEightBelow) {
            hipLaunchKernelGGL((encode_mfma_kernel<GH, C, B, 8, true, 1>), dim3((unsigned)n_tiles, gy, gz), dim3(8 * 64), 0, stream, a);
        } else if (wave_tiles < kGroupSplitBelow || n_tiles < 4) {
            hipLaunchKernelGGL((encode_mfma_kernel<GH, C, B, 4, true, 1>), dim3((unsigned)n_tiles, gy, gz), dim3(4 * 64), 0, stream, a);
        } else {
            hipLaunchKernelGGL((encode_mfma_kernel<GH, C, B, 4, true, 4>), dim3((unsigned)((n_tiles + 3) / 4), gy, gz), dim3(4 * 64), 0, stream, a);
        }
    } else {
        // 1024 centroids per group: one buffer per wavefront would not fit; four tiles per workgroup
        // share one staging of each group's codebook, small problems take one tile per workgroup
        if (wave_tiles >= 4096 && n_tiles >= 4) {
            constexpr int NW = 4;
            hipLaunchKernelGGL((encode_mfma_kernel<GH, C, B, NW>), dim3((unsigned)((n_tiles + NW - 1) / NW), gy, gz), dim3(NW * 64), 0, stream, a);
        } else {
            constexpr int NW = 1;
            hipLaunchKernelGGL((encode_mfma_kernel<GH, C, B, NW>), dim3((unsigned)n_tiles, gy, gz), dim3(NW * 64), 0, stream, a);
        }
    }
    if (hipGetLastError() != hipSuccess) return CQ_ERR_HIP;
    return CQ_OK;
}

}  // namespace

cq_status launch_encode_tiles(const EncodeArgs& a, hipStream_t stream)
{
    if (a.f.b == 8) {
        if (a.f.gh == 16 && a.f.c == 8) return launch_mfma_format<16, 8, 8>(a, stream);
        if (a.f.gh == 32 && a.f.c == 4) return launch_mfma_format<32, 4, 8>(a, stream);
        if (a.f.gh == 64 && a.f.c == 2) return launch_mfma_format<64, 2, 8>(a, stream);
    } else if (a.f.b == 10) {
        if (a.f.gh == 16 && a.f.c == 8) return launch_mfma_format<16, 8, 10>(a, stream);
    }
    return CQ_ERR_UNSUPPORTED;
}

}  // namespace cq

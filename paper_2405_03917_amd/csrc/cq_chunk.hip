// Causal attention of the last m tokens of each sequence over its packed CQ cache (a prefill
// chunk, or the verification step of speculative decoding), for gfx950.  Eq. 1 of the paper once
// per query token; the cache already holds the codes of the m tokens.
//
// With many queries per (sequence, KV head) the per-query lookup tables of the decode kernel
// no longer fit on chip and the path becomes a dense contraction, so this one is built on the
// matrix cores: a workgroup (8 wavefronts) owns up to 256 query rows of one KV head (query
// tokens x the query heads that share the KV head), walks the context in 64-token tiles, turns
// each tile's codes back into fp16 keys and values ONCE in LDS (centroid gathers from the
// L2-resident codebooks), and every wavefront runs a flash-attention step on its 32 rows:
//     S^T = K Q^T      v_mfma_f32_32x32x16_f16, A = keys of 32 tokens (LDS), B = queries (registers)
//     online softmax   each lane owns ONE query (a column of S^T): running maximum, sum and the
//                      rescaling of its output column are lane-local
//     O^T += V^T P^T   A = values, stored transposed in LDS, B = the probabilities just computed,
//                      scaled by 2^12 and split into two fp16 numbers (high and low part: 22
//                      bits; one fp16 alone leaves errors of 1e-5 of the largest output element,
//                      too much for the small ones); fp32 accumulation
// HBM traffic is the codes, read once per workgroup; the kernel is bound by the matrix cores and
// the LDS reads that feed them.  Long contexts with few rows are split over workgroups and
// merged by the decode path's merge kernel (same (m, l, o) partials).
#include "cq_decode_common.hpp"

namespace cq {
namespace {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));

// 8 wavefronts x 32 query rows per workgroup (one workgroup per CU), or 4 x 32 where a KV head has
// no more than 128 rows (two workgroups per CU then)
constexpr int kKsStride = 272;                    // bytes per token row of the key tile (256 + 16: conflict-free 16-byte reads)
constexpr int kVtStride = 136;                    // bytes per channel row of the transposed value tile (128 + 8)
constexpr int kKsBytes = kTileTokens * kKsStride; // 17408
constexpr int kVtBytes = 128 * kVtStride;         // 17408
// a stage: the key tile, the transposed value tile and (rotated keys only) the low parts of the key tile
constexpr int kStageBytes(bool rope) { return kKsBytes + kVtBytes + (rope ? kKsBytes : 0); }
constexpr unsigned kRawBase(bool rope) { return 2 * kStageBytes(rope); }     // behind the two stages: the raw code tiles (K, V) of two tiles
constexpr float kProbScale = 4096.f;              // 2^12

__device__ __forceinline__ half8_t lds_half8(unsigned byte_addr)
{
    return *(__attribute__((address_space(3))) half8_t*)(byte_addr);
}
__device__ __forceinline__ half4_t lds_half4(unsigned byte_addr)
{
    return *(__attribute__((address_space(3))) half4_t*)(byte_addr);
}

// Codes of 64 tokens -> fp16 keys [token][channel] and values [channel][token] in LDS.
// The codes of a tile first go to LDS as they are (load_raw / store_raw: one 16-byte record per
// thread).  Then thread (token u = tid % 64, wavefront e = tid / 64) expands groups
// e Gh/8 .. (e + 1) Gh/8 - 1 of its token: the code of group g sits in slot (g - u) mod Gh of the
// token's record.  A wavefront thus gathers from ONE group's centroids at a time: its 64 lanes
// touch the 8 to 32 cache lines of that group's table instead of 64 lines of 64 tables, which is
// what the texture path charges for.
//
// ROPE (keys cached before the rotary position embedding): thread (u, e) takes groups e, e + NW,
// e + 2 NW, ... instead, so that it holds both halves of its channel pairs (channel i of the head
// is rotated with channel i + 64, i.e. group g with group g + Gh/2), and store() rotates the
// pairs to the token's position before the keys go to LDS: once per (tile, KV head), for all
// query rows of the workgroup.
template <int GH, int C, int NW, int B, bool ROPE>
struct Dequant {
    static constexpr int GPT = GH / NW;                 // groups per thread
    static_assert(!ROPE || GPT % 2 == 0, "a thread holds both groups of a pair");
    static constexpr int NP = ROPE ? GPT / 2 * C : 1;   // channel pairs per thread
    float2 cs[NP];                                      // ROPE: cos / sin of (position * theta) of this thread's pairs
    // ROPE: low parts of the rotated keys.  A rotated key is kept as the sum of two fp16 numbers
    // (22 bits): rounded to one, its error of 2^-11 reaches the scores and leaves 4e-4 of a
    // row's largest output element, which fails the 2e-3 bar on the small elements
    unsigned kwl[ROPE ? GPT : 1][C / 2];
    __device__ __forceinline__ static int group(int e, int gi) { return ROPE ? e + gi * NW : e * GPT + gi; }
    static constexpr int K = 1 << B;                    // centroids per group
    static constexpr int TILE = kTileTokens * GH * B / 8;   // bytes of one tile's codes (b = 10: low bytes, then high-bit words)
    static constexpr int LOADERS = TILE / 16;           // threads that carry one record of K and one of V
    static constexpr int RAW_STAGE = 2 * TILE;          // K tile, V tile
    static_assert(LOADERS <= NW * 64, "one record per thread");
    u32x4 kraw, vraw;                                   // 16-byte records of the next tile's codes
    unsigned kw[GPT][C / 2], vw[GPT][C / 2];            // the centroids of this thread's (token, group) pairs

    __device__ __forceinline__ void load_raw(const uint8_t* ktile, const uint8_t* vtile, int tid)
    {
        if (tid < LOADERS) {
            kraw = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(ktile) + tid);
            vraw = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vtile) + tid);
        }
    }
    __device__ __forceinline__ void store_raw(unsigned raw_stage, int tid) const
    {
        typedef __attribute__((address_space(3))) u32x4 lds_q;
        if (tid < LOADERS) {
            *(lds_q*)(raw_stage + (unsigned)tid * 16) = kraw;
            *(lds_q*)(raw_stage + TILE + (unsigned)tid * 16) = vraw;
        }
    }

    // read this thread's codes from the raw tile and request their centroids (L2-resident codebooks)
    __device__ __forceinline__ void gather(unsigned raw_stage, const uint16_t* ck_head, const uint16_t* cv_head, int tid)
    {
        typedef __attribute__((address_space(3))) uint8_t lds_b;
        const int u = tid & 63, e = tid >> 6;
#pragma unroll
        for (int gi = 0; gi < GPT; ++gi) {
            const int g = group(e, gi);
            const unsigned slot = (unsigned)(g - u) & (unsigned)(GH - 1);
            const unsigned off = (slot >> 4) * 1024 + (unsigned)u * 16 + (slot & 15);
            unsigned kc = *(lds_b*)(raw_stage + off);
            unsigned vc = *(lds_b*)(raw_stage + TILE + off);
            if constexpr (B == 10) {        // bits [2 s + 1 : 2 s] of the token's high-bit word
                typedef __attribute__((address_space(3))) unsigned lds_w;
                const unsigned hoff = (unsigned)(kTileTokens * GH) + (unsigned)u * 4;
                kc |= ((*(lds_w*)(raw_stage + hoff) >> (2 * slot)) & 3u) << 8;
                vc |= ((*(lds_w*)(raw_stage + TILE + hoff) >> (2 * slot)) & 3u) << 8;
            }
            const unsigned* kp = reinterpret_cast<const unsigned*>(ck_head + ((size_t)g * K + kc) * C);
            const unsigned* vp = reinterpret_cast<const unsigned*>(cv_head + ((size_t)g * K + vc) * C);
#pragma unroll
            for (int i = 0; i < C / 2; ++i) {
                kw[gi][i] = kp[i];
                vw[gi][i] = vp[i];
            }
        }
    }

    // ROPE: cos / sin of the rotation of this thread's pairs for the tokens of `tile`, by angle
    // addition from the table's two parts (64 tile theta_i per tile, u theta_i per lane)
    __device__ __forceinline__ void request_angles(const float2* tile_tab, const float2* lane_tab, int tile, int tid)
    {
        if constexpr (ROPE) {
            const int u = tid & 63, e = tid >> 6;
#pragma unroll
            for (int gi = 0; gi < GPT / 2; ++gi)
#pragma unroll
                for (int i = 0; i < C; ++i) {
                    const int p = group(e, gi) * C + i;             // pair index = channel of the first half
                    const float2 t = tile_tab[(size_t)tile * 64 + p], l = lane_tab[p * 64 + u];
                    cs[gi * C + i] = make_float2(t.x * l.x - t.y * l.y, t.y * l.x + t.x * l.y);
                }
        }
    }
    // rotate the gathered keys: (k_i, k_{i+64}) -> (k_i cos - k_{i+64} sin, k_{i+64} cos + k_i sin), fp32, one
    // rounding to fp16
    __device__ __forceinline__ void rotate()
    {
        if constexpr (ROPE) {
#pragma unroll
            for (int gi = 0; gi < GPT / 2; ++gi)
#pragma unroll
                for (int i = 0; i < C / 2; ++i) {
                    const half2_t lo = __builtin_bit_cast(half2_t, kw[gi][i]), hi = __builtin_bit_cast(half2_t, kw[gi + GPT / 2][i]);
                    const float2 c0 = cs[gi * C + 2 * i], c1 = cs[gi * C + 2 * i + 1];
                    const float fl0 = (float)lo.x * c0.x - (float)hi.x * c0.y, fh0 = (float)hi.x * c0.x + (float)lo.x * c0.y;
                    const float fl1 = (float)lo.y * c1.x - (float)hi.y * c1.y, fh1 = (float)hi.y * c1.x + (float)lo.y * c1.y;
                    half2_t rl, rh, el, eh;
                    rl.x = (_Float16)fl0;
                    rh.x = (_Float16)fh0;
                    rl.y = (_Float16)fl1;
                    rh.y = (_Float16)fh1;
                    el.x = (_Float16)(fl0 - (float)rl.x);
                    eh.x = (_Float16)(fh0 - (float)rh.x);
                    el.y = (_Float16)(fl1 - (float)rl.y);
                    eh.y = (_Float16)(fh1 - (float)rh.y);
                    kw[gi][i] = __builtin_bit_cast(unsigned, rl);
                    kw[gi + GPT / 2][i] = __builtin_bit_cast(unsigned, rh);
                    kwl[gi][i] = __builtin_bit_cast(unsigned, el);
                    kwl[gi + GPT / 2][i] = __builtin_bit_cast(unsigned, eh);
                }
        }
    }

    __device__ __forceinline__ void store(unsigned stage, int tid) const
    {
        typedef __attribute__((address_space(3))) unsigned lds_u;
        typedef __attribute__((address_space(3))) uint16_t lds_h;
        const int u = tid & 63, e = tid >> 6;
#pragma unroll
        for (int gi = 0; gi < GPT; ++gi) {
            const int g = group(e, gi);
            const unsigned kaddr = stage + (unsigned)u * kKsStride + (unsigned)g * (C * 2);
#pragma unroll
            for (int i = 0; i < C / 2; ++i) *(lds_u*)(kaddr + 4 * i) = kw[gi][i];
            if constexpr (ROPE) {
#pragma unroll
                for (int i = 0; i < C / 2; ++i) *(lds_u*)(kaddr + kKsBytes + kVtBytes + 4 * i) = kwl[gi][i];
            }
            const unsigned vaddr = stage + kKsBytes + (unsigned)(g * C) * kVtStride + (unsigned)u * 2;
#pragma unroll
            for (int i = 0; i < C / 2; ++i) {
                *(lds_h*)(vaddr + (2 * i) * kVtStride) = (uint16_t)(vw[gi][i] & 0xffffu);
                *(lds_h*)(vaddr + (2 * i + 1) * kVtStride) = (uint16_t)(vw[gi][i] >> 16);
            }
        }
    }
};

template <int GH, int C, int NW, int B, bool ROPE>
__global__ __launch_bounds__(NW * 64) void chunk_attention_kernel(ChunkArgs a)
{
    constexpr int kRowsPerWg = NW * 32;
    constexpr unsigned kRawStageBytes = Dequant<GH, C, NW, B, ROPE>::RAW_STAGE;
    using F = Fmt<GH, B>;
    constexpr int D = 128;
    static_assert(GH * C == D, "head_dim 128");
    extern __shared__ float smem[];
    (void)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rc = lane & 31, kh = lane >> 5;

    // workgroup -> (sequence, KV head, block of 128 query rows, context split)
    const int qper = a.n_q_heads / a.f.n_kv_heads;
    const int rows_total = a.m * qper;                      // row r = (query token r / qper, query head r % qper)
    const int row_blocks = (rows_total + kRowsPerWg - 1) / kRowsPerWg;
    int idx = blockIdx.x;
    const int hkv = idx % a.f.n_kv_heads;
    idx /= a.f.n_kv_heads;
    const int rb = idx % row_blocks;
    idx /= row_blocks;
    const int split = idx % a.n_split;
    const int n = idx / a.n_split;

    int t_n = a.t;
    if (a.seq_lens) t_n = min(max(a.seq_lens[n], a.m), a.t);
    const int pos0 = t_n - a.m;                             // position of query token 0

    // this lane's query row
    const int row = rb * kRowsPerWg + wave * 32 + rc;
    const bool valid = row < rows_total;
    const int row_c = valid ? row : rows_total - 1;
    const int j = row_c / qper, hq = hkv * qper + row_c % qper;
    const int pos = pos0 + j;
    // (rows ascend with the lane: the wavefront's earliest position is its first lane's)
    const int pos_first = __builtin_amdgcn_readfirstlane(pos);
    // tiles this workgroup needs: up to the position of its last row, within its split
    const int last_row = min(rb * kRowsPerWg + kRowsPerWg, rows_total) - 1;
    const int tiles_needed = (pos0 + last_row / qper) / kTileTokens + 1;
    const int tile0 = split * a.tiles_per_split;
    const int tile1 = min(tile0 + a.tiles_per_split, tiles_needed);
    // the wavefront's own last tile (rows of later wavefronts reach further)
    const int wave_last_row = min(rb * kRowsPerWg + wave * 32 + 31, rows_total - 1);
    const int wave_tiles = (pos0 + wave_last_row / qper) / kTileTokens + 1;

    const size_t out_row = ((size_t)n * a.m + j) * a.n_q_heads + hq;
    float* part = a.partials + (out_row * a.n_split + split) * (D + kPartialHeader);

    // queries: B operand of S^T = K Q^T, lane (rc, kh) holds Q[row][16 s + 8 kh .. + 7] for the 8 steps
    half8_t qreg[8];
    {
        const uint16_t* qrow = a.q + out_row * D;
#pragma unroll
        for (int s = 0; s < 8; ++s) qreg[s] = *reinterpret_cast<const half8_t*>(qrow + 16 * s + 8 * kh);
    }

    const uint16_t* ck_head = a.k_centroids + (size_t)hkv * GH * F::K * C;
    const uint16_t* cv_head = a.v_centroids + (size_t)hkv * GH * F::K * C;
    auto tile_ptr = [&](const uint8_t* base, int tile) {
        return base + a.map.tile_index(n, hkv, tile) * F::TILE_BYTES;
    };

    float16_t o[4];
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[cb][i] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    // software pipeline over the tiles: while tile k is multiplied, the centroids of tile k + 1
    // are on their way from L2 and the codes of tile k + 2 from HBM
    Dequant<GH, C, NW, B, ROPE> dq;
    if (tile0 < tile1) {
        dq.load_raw(tile_ptr(a.k_codes, tile0), tile_ptr(a.v_codes, tile0), tid);
        dq.store_raw(kRawBase(ROPE), tid);
        if (tile0 + 1 < tile1) dq.load_raw(tile_ptr(a.k_codes, tile0 + 1), tile_ptr(a.v_codes, tile0 + 1), tid);
        lds_barrier();
        dq.gather(kRawBase(ROPE), ck_head, cv_head, tid);
        dq.request_angles(a.rope_tile_tab, a.rope_lane_tab, tile0, tid);
        dq.rotate();
        dq.store(0, tid);
        if (tile0 + 1 < tile1) dq.store_raw(kRawBase(ROPE) + kRawStageBytes, tid);
    }
    lds_barrier();

    for (int tile = tile0; tile < tile1; ++tile) {
        const unsigned par = (unsigned)((tile - tile0) & 1);
        const unsigned stage = par * kStageBytes(ROPE);
        const bool more = tile + 1 < tile1;
        if (more) {
            dq.gather(kRawBase(ROPE) + (par ^ 1u) * kRawStageBytes, ck_head, cv_head, tid);     // codes of tile + 1
            dq.request_angles(a.rope_tile_tab, a.rope_lane_tab, tile + 1, tid);
            if (tile + 2 < tile1) dq.load_raw(tile_ptr(a.k_codes, tile + 2), tile_ptr(a.v_codes, tile + 2), tid);
            __builtin_amdgcn_sched_barrier(0);          // requests first, then the multiplications
        }

        if (tile < wave_tiles) {
            // The two 32-token blocks of the tile are interleaved so that the matrix pipe and the
            // vector ALU overlap within the wavefront: scores of both blocks first; the softmax
            // arithmetic of block 0 runs while the scores of block 1 are still being multiplied,
            // that of block 1 while block 0's values are.
            float16_t acc[2];
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[tb][i] = 0.f;
                const unsigned krow = stage + (unsigned)(tb * 32 + rc) * kKsStride + (unsigned)kh * 16;
#pragma unroll
                for (int s = 0; s < 8; ++s)
                    acc[tb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(lds_half8(krow + 32 * s), qreg[s], acc[tb], 0, 0, 0);
                if constexpr (ROPE) {           // ... and the low parts of the rotated keys
#pragma unroll
                    for (int s = 0; s < 8; ++s)
                        acc[tb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(lds_half8(krow + kKsBytes + kVtBytes + 32 * s), qreg[s], acc[tb], 0, 0, 0);
                }
            }
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
                // acc[tb][i] is token 8 (i / 4) + 4 kh + i % 4 of the block, query rc
                const int tok0 = tile * kTileTokens + tb * 32 + 4 * kh;
                float bmax = -INFINITY;
                if (tile * kTileTokens + tb * 32 + 31 > pos_first) {
                    // a block on the causal diagonal of some query of this wavefront: mask
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int tok = tok0 + 8 * (i >> 2) + (i & 3);
                        acc[tb][i] = tok <= pos ? acc[tb][i] * a.scale_log2e : -INFINITY;
                        bmax = fmaxf(bmax, acc[tb][i]);
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        acc[tb][i] *= a.scale_log2e;
                        bmax = fmaxf(bmax, acc[tb][i]);
                    }
                }
                bmax = fmaxf(bmax, __shfl_xor(bmax, 32));
                const float m_new = fmaxf(m_run, bmax);
                const float m_safe = m_new == -INFINITY ? 0.f : m_new;      // nothing visible yet: all weights 0
                const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
                m_run = m_new;
                // probabilities times 2^12 (the sum l_run is kept in that scale too)
                const float m_shift = m_safe - 12.f;
                float psum = 0.f;
                half8_t ph[2], pl[2];            // p * 2^12 = ph + pl to 22 bits
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float ps = __builtin_amdgcn_exp2f(acc[tb][i] - m_shift);
                    psum += ps;
                    const _Float16 hi = (_Float16)ps;
                    ph[i >> 3][i & 7] = hi;
                    pl[i >> 3][i & 7] = (_Float16)(ps - (float)hi);
                }
                l_run = __builtin_fmaf(l_run, alpha, psum);
                if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) {
#pragma unroll
                    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
                        for (int i = 0; i < 16; ++i) o[cb][i] *= alpha;
                }
                // ---- O^T += V^T P^T: contraction index (kh, i) is token 16 t + 8 (i / 4) + 4 kh + i % 4 ----
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    half8_t av[4];
#pragma unroll
                    for (int cb = 0; cb < 4; ++cb) {
                        const unsigned vrow = stage + kKsBytes + (unsigned)(cb * 32 + rc) * kVtStride + (unsigned)(tb * 32 + 4 * kh) * 2;
                        const half4_t v0 = lds_half4(vrow + 32 * t), v1 = lds_half4(vrow + 32 * t + 16);
                        av[cb] = half8_t{v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
                    }
#pragma unroll
                    for (int cb = 0; cb < 4; ++cb) o[cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av[cb], ph[t], o[cb], 0, 0, 0);
#pragma unroll
                    for (int cb = 0; cb < 4; ++cb) o[cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av[cb], pl[t], o[cb], 0, 0, 0);
                }
            }
        }
        // the next tile goes to the other stage (its last readers passed the previous barrier)
        if (more) {
            dq.rotate();
            dq.store(par ? 0u : (unsigned)kStageBytes(ROPE), tid);
            // the raw tile read two steps ago (tile's own codes) makes room for those of tile + 2
            if (tile + 2 < tile1) dq.store_raw(kRawBase(ROPE) + par * kRawStageBytes, tid);
        }
        lds_barrier();
    }

    // ---- output: lane (rc, kh) holds channels 32 cb + 8 (i / 4) + 4 kh + i % 4 of query rc ----
    const float l = l_run + __shfl_xor(l_run, 32);
    if (!valid) return;
    if (a.n_split == 1) {
        const float inv = 1.f / l;
        uint16_t* orow = a.out + out_row * D;
#pragma unroll
        for (int cb = 0; cb < 4; ++cb)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                half4_t h;
#pragma unroll
                for (int b = 0; b < 4; ++b) h[b] = (_Float16)(o[cb][4 * i4 + b] * inv);
                *reinterpret_cast<half4_t*>(orow + 32 * cb + 8 * i4 + 4 * kh) = h;
            }
    } else {
        if (kh == 0) {
            part[0] = m_run;
            part[1] = l * (1.f / kProbScale);
        }
#pragma unroll
        for (int cb = 0; cb < 4; ++cb)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                float4 v;
                v.x = o[cb][4 * i4 + 0] * (1.f / kProbScale);
                v.y = o[cb][4 * i4 + 1] * (1.f / kProbScale);
                v.z = o[cb][4 * i4 + 2] * (1.f / kProbScale);
                v.w = o[cb][4 * i4 + 3] * (1.f / kProbScale);
                float* dst = part + kPartialHeader + 32 * cb + 8 * i4 + 4 * kh;
                dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
            }
    }
}

template <int GH, int C, int NW, int B, bool ROPE>
cq_status launch_chunk_variant(const ChunkArgs& a, hipStream_t stream)
{
    auto kernel = chunk_attention_kernel<GH, C, NW, B, ROPE>;
    static LdsKernelSetup setup;
    if (setup.ensure(reinterpret_cast<const void*>(kernel)) != hipSuccess) return CQ_ERR_HIP;
    const int qper = a.n_q_heads / a.f.n_kv_heads;
    const int row_blocks = (a.m * qper + NW * 32 - 1) / (NW * 32);
    const unsigned grid = (unsigned)(a.batch * a.n_split * row_blocks * a.f.n_kv_heads);
    const size_t lds = 2 * kStageBytes(ROPE) + 2 * Dequant<GH, C, NW, B, ROPE>::RAW_STAGE;
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(NW * 64), lds, stream, a);
    return hipGetLastError() == hipSuccess ? CQ_OK : CQ_ERR_HIP;
}

template <int GH, int C, int B>
cq_status launch_chunk_rows(const ChunkArgs& a, hipStream_t stream)
{
    const int rows = a.m * (a.n_q_heads / a.f.n_kv_heads);
    if (a.rope_tile_tab) {
        if (chunk_rows_per_workgroup(rows) == 128) return launch_chunk_variant<GH, C, 4, B, true>(a, stream);
        return launch_chunk_variant<GH, C, 8, B, true>(a, stream);
    }
    if (chunk_rows_per_workgroup(rows) == 128) return launch_chunk_variant<GH, C, 4, B, false>(a, stream);
    return launch_chunk_variant<GH, C, 8, B, false>(a, stream);
}

}  // namespace

int chunk_rows_per_workgroup(int rows_per_kv_head) { return rows_per_kv_head <= 128 ? 128 : 256; }

cq_status launch_chunk_attention(const ChunkArgs& a, hipStream_t stream)
{
    cq_status st = CQ_ERR_UNSUPPORTED;
    if (a.f.b == 8 && a.f.head_dim == 128) {
        if (a.f.gh == 16 && a.f.c == 8) st = launch_chunk_rows<16, 8, 8>(a, stream);
        else if (a.f.gh == 32 && a.f.c == 4) st = launch_chunk_rows<32, 4, 8>(a, stream);
        else if (a.f.gh == 64 && a.f.c == 2) st = launch_chunk_rows<64, 2, 8>(a, stream);
    } else if (a.f.b == 10 && a.f.head_dim == 128 && a.f.gh == 16 && a.f.c == 8) {
        st = launch_chunk_rows<16, 8, 10>(a, stream);
    }
    if (st != CQ_OK) return st;
    if (a.n_split > 1)
        return launch_decode_merge(a.partials, a.out, a.batch * a.m * a.n_q_heads, a.n_q_heads, (int64_t)a.n_q_heads * a.f.head_dim, a.n_split,
                                   a.f.head_dim, stream);
    return CQ_OK;
}

}  // namespace cq

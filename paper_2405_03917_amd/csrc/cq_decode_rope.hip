// Decode attention from packed CQ codes when the cached KEYS were quantized before the rotary
// position embedding (Section 3.2 of the paper quantizes keys "before RoPE"; Eq. 1's f_K counts
// the positional encoding in), for gfx950.  The paper cites RoPE without restating it; the form
// implemented is the one of the models it evaluates (LLaMA, Mistral): channels i and i + d/2 of a
// head form a pair that is rotated by position * base^(-2i/d); the query arrives already rotated.
//
// The rotation angle differs per channel pair, so the score of a token can no longer be summed
// from one table entry per group.  With t = t0 + u (t0 = 64 * tile, u = the token's lane) the
// rotation is split by the angle-addition theorem: the key is rotated to the tile's base position,
//     X_i = k_i cos(t0 th_i) - k_{i+64} sin(t0 th_i),   Y_i = k_{i+64} cos(t0 th_i) + k_i sin(t0 th_i),
// (the cosines and sines of a tile are the same for all its tokens: scalar operands, read with
// scalar loads from a [tile][pair] table), and the rest of the way is taken by the query instead,
//     q . R_t k  =  sum_i  X_i A_i(u) + Y_i B_i(u),
//     A_i(u) = q_i cos(u th_i) + q_{i+64} sin(u th_i),   B_i(u) = q_{i+64} cos(u th_i) - q_i sin(u th_i),
// which depends on the lane only: 128 registers per lane, computed once per workgroup from a
// [pair][lane] table.  Lane = token as in the position-independent kernel; the key centroids
// themselves (fp16, 64 KB per head) take the place of the score table in LDS, and a token costs,
// per channel pair, six VALU instructions (against one gather and one add per GROUP without
// rotation) and no LDS access beyond its centroids: phase K is bound by the vector ALU, not by
// HBM.  512 threads, one workgroup per CU (the registers of the per-lane query want two
// wavefronts per SIMD at most).  Phase V, the epilogue and the split-context merge are those of
// the position-independent kernel.  Both trigonometric tables come from cq_rope_table (computed
// in fp64).
#include "cq_decode_common.hpp"

namespace cq {
namespace {

constexpr int kPairs = 64;                        // head_dim / 2
constexpr unsigned kTabBytes = 65536;             // centroids (phase K), then bins (phase V)
constexpr int kRopeThreads = 512;
struct CosSin { float c, s; };
constexpr unsigned kScrBytes = (64 + kRopeThreads / 64 * 128) * 4;     // reductions: two rows of per-wavefront scalars, per-wavefront outputs

__global__ void rope_tables_kernel(double base, int n_tiles, float2* tile_tab, float2* lane_tab)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    const int n_tile_entries = n_tiles * kPairs;
    if (idx >= n_tile_entries + kPairs * 64) return;
    int i;
    double pos;
    float2* dst;
    if (idx < n_tile_entries) {
        i = idx % kPairs;
        pos = (double)(idx / kPairs) * 64.0;
        dst = tile_tab + idx;
    } else {
        const int j = idx - n_tile_entries;
        i = j / 64;
        pos = (double)(j % 64);
        dst = lane_tab + j;
    }
    const double ang = pos * pow(base, -2.0 * (double)i / 128.0);
    *dst = make_float2((float)cos(ang), (float)sin(ang));
}

template <int C>
struct CenVec {
    unsigned w[C / 2];
};
template <int C>
__device__ __forceinline__ CenVec<C> lds_centroid(unsigned byte_addr)
{
    typedef __attribute__((address_space(3))) unsigned lds_u;
    CenVec<C> v;
    if constexpr (C == 8) {
        typedef unsigned u4 __attribute__((ext_vector_type(4)));
        const u4 a = *(__attribute__((address_space(3))) u4*)(byte_addr);
        v.w[0] = a.x; v.w[1] = a.y; v.w[2] = a.z; v.w[3] = a.w;
    } else if constexpr (C == 4) {
        typedef unsigned u2 __attribute__((ext_vector_type(2)));
        const u2 a = *(__attribute__((address_space(3))) u2*)(byte_addr);
        v.w[0] = a.x; v.w[1] = a.y;
    } else {
        v.w[0] = *(lds_u*)(byte_addr);
    }
    return v;
}
template <int C>
__device__ __forceinline__ CenVec<C> global_centroid(const uint16_t* p)
{
    CenVec<C> v;
#pragma unroll
    for (int i = 0; i < C / 2; ++i) v.w[i] = reinterpret_cast<const unsigned*>(p)[i];
    return v;
}
// One mixed-precision multiply-add: the fp16 half HI of register `w`, times the fp32 scalar `s`,
// plus / minus the fp32 `c` (or plus nothing).  Written out because the compiler converts a half
// that is used twice to fp32 first (one more instruction per channel) instead of letting both
// users read it as it is.  Volatile: the statements stay in the order written, which is batches of
// sixteen independent ones (a wavefront has one partner on its SIMD to hide a dependent
// instruction's latency behind, so it has to bring its own independent work).
__device__ __forceinline__ float mix_mul(bool HI, unsigned w, float s)
{
    float d;
    if (HI) asm volatile("v_fma_mix_f32 %0, %1, %2, 0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(w), "s"(s));
    else asm volatile("v_fma_mix_f32 %0, %1, %2, 0 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(w), "s"(s));
    return d;
}
template <bool MINUS>
__device__ __forceinline__ float mix_fma(bool HI, unsigned w, float s, float c)
{
    float d;
    if (HI && MINUS) asm volatile("v_fma_mix_f32 %0, %1, %2, -%3 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(w), "s"(s), "v"(c));
    else if (HI) asm volatile("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(w), "s"(s), "v"(c));
    else if (MINUS) asm volatile("v_fma_mix_f32 %0, %1, %2, -%3 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(w), "s"(s), "v"(c));
    else asm volatile("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(w), "s"(s), "v"(c));
    return d;
}

// A token's codes in group order.  The cache stores the code of group (s + u) mod Gh in slot s
// of token u (the position-independent kernel wants neighbouring lanes on different groups);
// here every lane should work on the same channel pair at the same time (the rotated query is
// then a scalar, and every table address a compile-time offset), so the token's Gh bytes are
// rotated by u positions once per tile: bytes first (v_alignbyte), then whole dwords (selects).
struct Unrotate {
    unsigned bytes;             // (Gh - u) mod 4
    unsigned dwords;            // ((Gh - u) mod Gh) / 4
};
template <int GH, int B>
__device__ __forceinline__ void group_order(const Tile<GH, B>& w, const Unrotate& r, unsigned (&d)[GH / 4])
{
    constexpr int N = GH / 4;
    unsigned x[N];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const u32x4 q = w.lo[i >> 2];
        x[i] = (i & 3) == 0 ? q.x : (i & 3) == 1 ? q.y : (i & 3) == 2 ? q.z : q.w;
    }
    // group g sits in slot (g - u) mod Gh = (g + r) mod Gh with r = (Gh - u) mod Gh
#pragma unroll
    for (int i = 0; i < N; ++i) d[i] = __builtin_amdgcn_alignbyte(x[(i + 1) % N], x[i], r.bytes);
#pragma unroll
    for (int bit = 1; bit < N; bit <<= 1) {
        const bool on = (r.dwords & bit) != 0;
        unsigned y[N];
#pragma unroll
        for (int i = 0; i < N; ++i) y[i] = on ? d[(i + bit) % N] : d[i];
#pragma unroll
        for (int i = 0; i < N; ++i) d[i] = y[i];
    }
}

// STEP = true is the fused decode step, as in cq_decode.hip: the workgroup whose split holds the
// newest position also encodes that token's key row (before any rotation: the cache holds
// pre-rotation keys) against the centroids it has just brought into LDS, patches the tile that
// holds the position in registers, and finds the value codes in the epilogue.  Same results as
// cq_encode_kv followed by the attention call, bit for bit.
// B = 10 (1024 centroids per group: 256 KB of key centroids per head) reads the centroids from
// global memory (L2) instead of LDS, in phase K and in the fused step's search.
template <int GH, int C, int NT, bool STEP, int B>
__global__ __launch_bounds__(NT) void decode_rope_kernel(DecodeArgs a, const float2* tile_tab, const float2* lane_tab)
{
    using F = Fmt<GH, B>;
    constexpr int K = F::K, RW = F::RW, R = F::R;
    constexpr int NW = NT / 64;
    constexpr int D = GH * C;
    constexpr int HALF = GH / 2;                    // groups per half of the head
    constexpr int PF = GH == 16 ? 4 : (GH == 32 ? 2 : 1);
    constexpr int JPL = 8 / C;
    constexpr int NCH = GH / 16;
    constexpr int UNITS = 16 * K / JPL;
    constexpr int IPT = UNITS / NT;
    static_assert(D == 128 && UNITS % NT == 0, "head_dim 128");
    static_assert(NT == kRopeThreads, "LDS layout");
    constexpr unsigned SC_BASE = kTabBytes + kScrBytes;
    extern __shared__ float smem[];
    float* tab = smem;                                              // centroids in phase K, bins in phase V
    float* sc = smem + SC_BASE / 4;                                 // scores of the split
    float* scr = smem + kTabBytes / 4;                              // reductions
    // fused step: (distance, index) minima per group, keys[0..GH) for K, [GH..2GH) for V, then the new token's weight
    unsigned long long* keys = reinterpret_cast<unsigned long long*>(smem + SC_BASE / 4 + a.tiles_per_split * kTileTokens);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // workgroup -> (sequence, split, query head), KV head a function of blockIdx % 8 (see cq_decode.hip)
    const int qper = a.n_q_heads / a.f.n_kv_heads;
    int hq, split, n;
    if (a.f.n_kv_heads % 8 == 0) {
        const int xcd = blockIdx.x & 7;
        int r = blockIdx.x >> 3;
        const int per_xcd = a.f.n_kv_heads >> 3;
        const int hkv_ = xcd + 8 * (r % per_xcd);
        r /= per_xcd;
        hq = hkv_ * qper + r % qper;
        r /= qper;
        split = r % a.n_split;
        n = r / a.n_split;
    } else {
        int idx = blockIdx.x;
        hq = idx % a.n_q_heads;
        idx /= a.n_q_heads;
        split = idx % a.n_split;
        n = idx / a.n_split;
    }
    const int hkv = hq / qper;

    int t_n = a.t;
    if (a.seq_lens) t_n = min(max(a.seq_lens[n] - a.seq_len_shift, a.seq_len_floor), a.t);
    const int n_tiles = (t_n + kTileTokens - 1) / kTileTokens;
    const int tile0 = split * a.tiles_per_split;
    const int tile1 = min(tile0 + a.tiles_per_split, n_tiles);
    float* part = a.partials + ((size_t)(n * a.n_q_heads + hq) * a.n_split + split) * (D + kPartialHeader);
    if (tile0 >= tile1) {
        if (tid == 0) { part[0] = -INFINITY; part[1] = 0.f; }
        for (int i = tid; i < D; i += NT) part[kPartialHeader + i] = 0.f;
        return;
    }

    const int pos_new = t_n - 1;
    const int tile_new = pos_new / kTileTokens, u_new = pos_new % kTileTokens;
    const bool has_new = STEP && tile_new >= tile0 && tile_new < tile1;
    if (has_new && tid < 2 * GH) keys[tid] = ~0ull;         // (ordered by the barrier behind the table copy)

    Columns<GH, B> col;
    const int my_tiles = (tile1 - tile0 - wave + NW - 1) / NW;
    TileWalk<GH, B> kwalk, vwalk;
    kwalk.first = tile0 + wave;
    kwalk.stride = NW;
    kwalk.pages = 0;
    if (a.map.block_table) {
        if (lane < my_tiles) kwalk.pages = a.map.page(n, tile0 + wave + lane * NW);
        kwalk.page_bytes = (size_t)a.f.n_kv_heads * F::TILE_BYTES;
        kwalk.base = a.k_codes + (size_t)hkv * F::TILE_BYTES;
        vwalk = kwalk;
        vwalk.base = a.v_codes + (size_t)hkv * F::TILE_BYTES;
    } else {
        const size_t stream_idx = a.map.tile_index(n, hkv, 0) * F::TILE_BYTES;
        kwalk.page_bytes = 0;
        kwalk.base = a.k_codes + stream_idx;
        vwalk = kwalk;
        vwalk.base = a.v_codes + stream_idx;
    }
    // phase K keeps one tile in flight ahead of the one it works on (a tile is thousands of cycles
    // of arithmetic; every further copy of its body would only crowd the instruction cache)
    Streamer<GH, B, 1> stk;
    Streamer<GH, B, PF> st;

    // ---- 1. the head's key centroids go to LDS; this lane's query, rotated back by its offset ----
    if constexpr (B == 8) {
        const uint4* src = reinterpret_cast<const uint4*>(a.k_centroids + (size_t)hkv * GH * K * C);
        for (int i = tid; i < (int)(kTabBytes / 16); i += NT) reinterpret_cast<uint4*>(smem)[i] = src[i];
    }
    stk.begin(kwalk, my_tiles, lane);
    // cos / sin of the tiles' base positions: uniform per wavefront, read through the scalar cache
    typedef __attribute__((address_space(4))) const CosSin tile_cs_t;
    tile_cs_t* tile_cs = (tile_cs_t*)reinterpret_cast<unsigned long long>(tile_tab);
    // (the four lanes of a group are neighbours and read four neighbouring 16-byte pieces of its
    // value codebook: 64 contiguous bytes, four cache lines per 16 lanes instead of sixteen)
    const int gl16 = (tid >> 2) & 15;
    auto piece = [&](int k) { return (((tid + k * NT) >> 6) << 2) + (tid & 3); };
    unsigned xvw[STEP ? NCH : 1][C / 2];            // fused step: this thread's slices of the new value row
    lds_barrier();

    // fused step: nearest key centroids of the new row, NT / GH threads per group over the
    // centroids in LDS (b = 10: in global memory; ascending index per thread, 64-bit minimum over
    // the threads: the exact search of cq_encode with its tie rule); the first query head of the
    // KV head stores the codes
    if (has_new) {
        constexpr int TPG = NT / GH;
        const int g = tid / TPG;
        const size_t xrow = (size_t)n * a.x_new_stride + (size_t)hkv * GH * C;
        float xk[C];
        load_row_slice<C>(a.xk_new + xrow + g * C, xk);
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch)
#pragma unroll
            for (int i = 0; i < C / 2; ++i)
                xvw[ch][i] = *reinterpret_cast<const unsigned*>(a.xv_new + xrow + (ch * 16 + gl16) * C + 2 * i);
        Nearest knear;
        if constexpr (B == 8) {
            for (int j = tid % TPG; j < K; j += TPG) {
                const CenVec<C> cen = lds_centroid<C>((unsigned)(g * K + j) * (C * 2));
                knear.offer(centroid_distance<C>(xk, cen.w), j);
            }
        } else {
            // 1024 centroids per group stay in global memory: a wavefront reads runs of 64 of them
            const uint16_t* cg = a.k_centroids + ((size_t)hkv * GH + g) * K * C;
            constexpr int PER = K / TPG, BATCH = PER < 4 ? PER : 4;
            static_assert(PER % BATCH == 0, "whole batches of loads");
#pragma unroll 1
            for (int j0 = tid % TPG; j0 < K; j0 += TPG * BATCH) {
                CenVec<C> cen[BATCH];
#pragma unroll
                for (int u = 0; u < BATCH; ++u) cen[u] = global_centroid<C>(cg + (size_t)(j0 + u * TPG) * C);
#pragma unroll
                for (int u = 0; u < BATCH; ++u) knear.offer(centroid_distance<C>(xk, cen[u].w), j0 + u * TPG);
            }
        }
        lds_min_u64(&keys[g], knear.key());
        lds_barrier();
    }
    const bool writer = has_new && hq % qper == 0;
    if (writer)
        store_new_codes<GH, B>(const_cast<uint8_t*>(a.k_codes) + a.map.tile_index(n, hkv, tile_new) * F::TILE_BYTES, keys, u_new, tid);

    // ---- 2. phase K: scores ----------------------------------------------------------------
    float qa[kPairs], qb[kPairs];
    {
        const unsigned* qh = reinterpret_cast<const unsigned*>(a.q + (size_t)n * a.q_batch_stride + (size_t)hq * D);
#pragma unroll
        for (int i = 0; i < kPairs; i += 2) {
            // (the query is the same for all lanes: scalar loads)
            const half2_t lo = __builtin_bit_cast(half2_t, qh[i >> 1]), hi = __builtin_bit_cast(half2_t, qh[(i + kPairs) >> 1]);
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const float2 cs = lane_tab[(i + e) * 64 + lane];
                const float q0 = (float)(e ? lo.y : lo.x) * a.scale_log2e, q1 = (float)(e ? hi.y : hi.x) * a.scale_log2e;
                qa[i + e] = __builtin_fmaf(q0, cs.x, q1 * cs.y);
                qb[i + e] = __builtin_fmaf(q1, cs.x, -(q0 * cs.y));
            }
        }
    }
    const uint16_t* k_head = a.k_centroids + (size_t)hkv * GH * K * C;
    Unrotate unrot;
    unrot.bytes = (unsigned)(GH - lane) & 3u;
    unrot.dwords = ((unsigned)(GH - lane) & (unsigned)(GH - 1)) >> 2;
    float lane_max = -INFINITY;
    // fused step: the wavefront whose walk meets the new token's tile patches that tile in registers
    const bool meets_new = has_new && (tile_new - tile0) % NW == wave;
    NewTokenCodes<GH, B> new_codes;
    if (meets_new) new_codes.build(keys, u_new, lane);
    constexpr int kBatch = 8;                       // channel pairs per batch of scalars and centroids
    constexpr int GPB = kBatch / C;                 // groups (of each half of the head) per batch
    CosSin cur[kBatch];
    {
        tile_cs_t* first = tile_cs + (size_t)(my_tiles > 0 ? tile0 + wave : tile0) * kPairs;
#pragma unroll
        for (int e = 0; e < kBatch; ++e) { cur[e].c = first[e].c; cur[e].s = first[e].s; }
    }
    stk.run(kwalk, my_tiles, lane, [&](const Tile<GH, B>& w_in, int k) {
        const int lt = wave + k * NW;
        Tile<GH, B> w = w_in;
        if (meets_new && tile0 + lt == tile_new) new_codes.patch(w, u_new, lane);
        tile_cs_t* cs = tile_cs + (size_t)(tile0 + lt) * kPairs;
        // codes in group order: byte g of d[] is the code of group g
        unsigned d[GH / 4];
        group_order<GH, B>(w, unrot, d);
        // b = 10: the high bits of group g sit at bits [2 g + 1 : 2 g] once the word is rotated like the bytes
        const unsigned hi_rot = B == 10 ? __builtin_amdgcn_alignbit(w.hi, w.hi, 2u * (((unsigned)(GH - lane)) & (unsigned)(GH - 1))) : 0u;
        float acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.f;
        // centroids of a batch: both halves' groups bi GPB .. of the head
        auto centroids = [&](int bi, CenVec<C> (&ka)[GPB], CenVec<C> (&kb)[GPB], float after) {
#pragma unroll
            for (int gg = 0; gg < GPB; ++gg) {
                const int g = bi * GPB + gg;
                unsigned c_first = (d[g >> 2] >> (8 * (g & 3))) & 0xffu;                       // channels < 64
                unsigned c_second = (d[(g + HALF) >> 2] >> (8 * ((g + HALF) & 3))) & 0xffu;    // their partners
                if constexpr (B == 10) {
                    c_first |= ((hi_rot >> (2 * g)) & 3u) << 8;
                    c_second |= ((hi_rot >> (2 * (g + HALF))) & 3u) << 8;
                }
                asm volatile("" : "+v"(c_first), "+v"(c_second) : "v"(after));
                if constexpr (B == 8) {
                    ka[gg] = lds_centroid<C>(c_first * (C * 2) + (unsigned)(g * K * C * 2));
                    kb[gg] = lds_centroid<C>(c_second * (C * 2) + (unsigned)((g + HALF) * K * C * 2));
                } else {
                    ka[gg] = global_centroid<C>(k_head + ((size_t)g * K + c_first) * C);
                    kb[gg] = global_centroid<C>(k_head + ((size_t)(g + HALF) * K + c_second) * C);
                }
            }
        };
        CenVec<C> ka[GPB], kb[GPB];
        centroids(0, ka, kb, 0.f);
#pragma unroll
        for (int bi = 0; bi < kPairs / kBatch; ++bi) {
            CosSin nxt[kBatch];
            CenVec<C> ka_n[GPB], kb_n[GPB];
            // pair e of the batch: channel pair (i, i + 64), i = kBatch bi + e, group bi GPB + e / C, channel j = e % C of it;
            // x, y: the key rotated to the tile's base position
#pragma unroll
            for (int h = 0; h < kBatch; h += 8) {
                float t1[8], t2[8], x[8], y[8];
#pragma unroll
                for (int e = h; e < h + 8; ++e) t1[e - h] = mix_mul((e % C) & 1, kb[e / C].w[(e % C) >> 1], cur[e].s);
                if (h == 0) {
                    // The next batch's scalars (behind the last batch: the next tile's) and centroids
                    // are requested here: behind the first use of this batch's (a wait for a scalar load
                    // is a wait for everything outstanding, so nothing may be in flight at that
                    // point that is not needed yet), a batch of arithmetic ahead of their own use.
                    tile_cs_t* nx = bi + 1 < kPairs / kBatch ? cs + (bi + 1) * kBatch
                                                             : tile_cs + (size_t)(tile0 + (k + 1 < my_tiles ? lt + NW : lt)) * kPairs;
                    asm volatile("" : "+s"(nx) : "v"(t1[0]));
#pragma unroll
                    for (int e = 0; e < kBatch; ++e) { nxt[e].c = nx[e].c; nxt[e].s = nx[e].s; }
                    if (bi + 1 < kPairs / kBatch) centroids(bi + 1, ka_n, kb_n, t1[0]);
                }
#pragma unroll
                for (int e = h; e < h + 8; ++e) t2[e - h] = mix_mul((e % C) & 1, ka[e / C].w[(e % C) >> 1], cur[e].s);
#pragma unroll
                for (int e = h; e < h + 8; ++e) x[e - h] = mix_fma<true>((e % C) & 1, ka[e / C].w[(e % C) >> 1], cur[e].c, t1[e - h]);
#pragma unroll
                for (int e = h; e < h + 8; ++e) y[e - h] = mix_fma<false>((e % C) & 1, kb[e / C].w[(e % C) >> 1], cur[e].c, t2[e - h]);
#pragma unroll
                for (int e = h; e < h + 8; ++e) acc[e & 7] = __builtin_fmaf(x[e - h], qa[bi * kBatch + e], acc[e & 7]);
#pragma unroll
                for (int e = h; e < h + 8; ++e) acc[e & 7] = __builtin_fmaf(y[e - h], qb[bi * kBatch + e], acc[e & 7]);
                // (left alone, the compiler moves the multiply-adds of all batches behind the last
                // rotation, with every rotated key of the tile in a register of its own until then:
                // the sums pass through a statement that keeps its place among the rotations)
                asm volatile("" : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]), "+v"(acc[4]), "+v"(acc[5]), "+v"(acc[6]), "+v"(acc[7]));
            }
#pragma unroll
            for (int e = 0; e < kBatch; ++e) cur[e] = nxt[e];
            if (bi + 1 < kPairs / kBatch) {
#pragma unroll
                for (int gg = 0; gg < GPB; ++gg) { ka[gg] = ka_n[gg]; kb[gg] = kb_n[gg]; }
            }
        }
        const float acc0 = (acc[0] + acc[1]) + (acc[2] + acc[3]), acc1 = (acc[4] + acc[5]) + (acc[6] + acc[7]);
        const int tok = (tile0 + lt) * kTileTokens + lane;
        const float sv = tok < t_n ? acc0 + acc1 : -INFINITY;
        sc[lt * kTileTokens + lane] = sv;
        lane_max = fmaxf(lane_max, sv);
    }, [] {});
    st.begin(vwalk, my_tiles, lane);

    lane_max = wave_max(lane_max);
    lds_barrier();                                  // all centroid / table reads done, all scores written
    if (lane == 0) scr[wave] = lane_max;
    lds_barrier();
    float m = scr[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) m = fmaxf(m, scr[w]);
    float l_est = 0.f;
    for (int i = tid; i < (tile1 - tile0) * kTileTokens; i += NT) l_est += __builtin_amdgcn_exp2f(sc[i] - m);
    l_est = wave_sum(l_est);
    if (lane == 0) scr[32 + wave] = l_est;
    lds_barrier();
    l_est = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) l_est += scr[32 + w];
    const int fx = fixed_point_exponent(l_est);
    const float fx_scale = ldexpf(1.f, fx), fx_inv = ldexpf(1.f, -fx);
    {
        float4* t4 = reinterpret_cast<float4*>(tab);
#pragma unroll 4
        for (int i = tid; i < F::TAB_FLOATS / 4; i += NT) t4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    lds_barrier();

    // ---- 3. phase V: probability bins (as in the position-independent kernel) -------------
    col.init(lane);
    unsigned* pf_new = reinterpret_cast<unsigned*>(keys + 2 * GH);
    constexpr int KB = IPT < 8 ? IPT : 8;
    constexpr bool EARLY = IPT * NCH <= 8 && KB == IPT;
    Cent16 rawv[EARLY ? NCH : 1][KB];
    unsigned lane_sum = 0;
    st.run(vwalk, my_tiles, lane, [&](const Tile<GH, B>& w, int k) {
        const int lt = wave + k * NW;
        const float p = __builtin_amdgcn_exp2f(sc[lt * kTileTokens + lane] - m);
        unsigned pf = (unsigned)__builtin_fmaf(p, fx_scale, 0.5f);
        lane_sum += pf;
        // fused step: the new token's value codes are found in the epilogue; its weight waits in LDS
        if (has_new && tile0 + lt == tile_new && lane == u_new) {
            *pf_new = pf;
            pf = 0;
        }
#pragma unroll
        for (int s = 0; s < GH; ++s) lds_add(slot_addr<GH, B, false>(w, col, s), pf);
    }, [&] {
        if constexpr (EARLY) {
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
                const uint16_t* cv = a.v_centroids + (size_t)(hkv * GH + ch * 16 + gl16) * K * C;
#pragma unroll
                for (int k = 0; k < IPT; ++k) rawv[ch][k] = load_cent16(cv + (size_t)piece(k) * 8);
            }
        }
    });

    // ---- 4. epilogue: o = bins . C_V -------------------------------------------------------
    lane_sum = wave_sum_u32(lane_sum);
    lds_barrier();
    if (lane == 0) scr[wave] = __uint_as_float(lane_sum);

    // fused step: encode the new value row against the value codebook (the registers of the sums
    // below), add its weight to the bins of its codes, store the codes
    if (has_new) {
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
            float xv[C];
#pragma unroll
            for (int i = 0; i < C / 2; ++i) {
                const half2_t h = __builtin_bit_cast(half2_t, xvw[ch][i]);
                xv[2 * i] = (float)h.x;
                xv[2 * i + 1] = (float)h.y;
            }
            const uint16_t* cvg = a.v_centroids + (size_t)(hkv * GH + ch * 16 + gl16) * K * C;
            Nearest vnear;
#pragma unroll
            for (int k0 = 0; k0 < IPT; k0 += KB) {
                Cent16 rawb[EARLY ? 1 : KB];            // (where the codebook is not in registers yet: b = 10)
                if constexpr (!EARLY) {
#pragma unroll
                    for (int k = 0; k < KB; ++k) rawb[k] = load_cent16(cvg + (size_t)piece(k0 + k) * 8);
                }
#pragma unroll
                for (int k = 0; k < KB; ++k) {
                    const int j0 = piece(k0 + k) * JPL;
                    const Cent16& r = EARLY ? rawv[EARLY ? ch : 0][k] : rawb[EARLY ? 0 : k];
#pragma unroll
                    for (int jj = 0; jj < JPL; ++jj) vnear.offer(centroid_distance<C>(xv, &r.w[jj * (C / 2)]), j0 + jj);
                }
            }
            const unsigned long long vkey = group_lanes_min<4>(vnear.key());
            if ((lane & 3) == 0) lds_min_u64(&keys[GH + ch * 16 + gl16], vkey);
        }
        lds_barrier();
        if (tid < GH) {
            const unsigned code = (unsigned)(keys[GH + tid] & 0xffffffffu);
            lds_add((code * RW + tid * R) * 4u, *pf_new);
        }
        if (writer)
            store_new_codes<GH, B>(const_cast<uint8_t*>(a.v_codes) + a.map.tile_index(n, hkv, tile_new) * F::TILE_BYTES, keys + GH, u_new, tid);
        lds_barrier();
    }
    float acc[NCH][C];
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
#pragma unroll
        for (int i = 0; i < C; ++i) acc[ch][i] = 0.f;
#pragma unroll
        for (int k0 = 0; k0 < IPT; k0 += KB) {
            if constexpr (!EARLY) {
                const uint16_t* cv = a.v_centroids + (size_t)(hkv * GH + ch * 16 + gl16) * K * C;
#pragma unroll
                for (int k = 0; k < KB; ++k) rawv[0][k] = load_cent16(cv + (size_t)piece(k0 + k) * 8);
            }
            const Cent16 (&raw)[KB] = rawv[EARLY ? ch : 0];
#pragma unroll
            for (int k = 0; k < KB; ++k) {
                const int j0 = piece(k0 + k) * JPL;
#pragma unroll
                for (int jj = 0; jj < JPL; ++jj) {
                    const float* src = tab + (j0 + jj) * RW + (ch * 16 + gl16) * R;
                    unsigned cnt;
                    if constexpr (R == 2) { const uint2 x = *reinterpret_cast<const uint2*>(src); cnt = x.x + x.y; }
                    else cnt = *reinterpret_cast<const unsigned*>(src);
                    const float bin = (float)cnt * fx_inv;
#pragma unroll
                    for (int i = 0; i < C / 2; ++i) {
                        const half2_t h = __builtin_bit_cast(half2_t, raw[k].w[jj * (C / 2) + i]);
                        acc[ch][2 * i] = __builtin_fmaf(bin, (float)h.x, acc[ch][2 * i]);
                        acc[ch][2 * i + 1] = __builtin_fmaf(bin, (float)h.y, acc[ch][2 * i + 1]);
                    }
                }
            }
        }
#pragma unroll
        for (int i = 0; i < C; ++i) {
            acc[ch][i] += __shfl_xor(acc[ch][i], 1);
            acc[ch][i] += __shfl_xor(acc[ch][i], 2);
        }
    }
    if ((lane & 3) == 0) {
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch)
#pragma unroll
            for (int i = 0; i < C; ++i) scr[64 + wave * D + (ch * 16 + gl16) * C + i] = acc[ch][i];
    }
    lds_barrier();
    unsigned l_fix = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) l_fix += __float_as_uint(scr[w]);
    const float l = (float)l_fix * fx_inv;
    const bool direct = a.n_split == 1;
    if (tid == 0 && !direct) {
        part[0] = m;
        part[1] = l;
    }
    for (int chn = tid; chn < D; chn += NT) {
        float o = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) o += scr[64 + w * D + chn];
        if (direct) a.out[(size_t)n * a.out_batch_stride + (size_t)hq * D + chn] = __builtin_bit_cast(uint16_t, (_Float16)(o / l));
        else part[kPartialHeader + chn] = o;
    }
}

// acc += (the query values of pair i, one head per row) x (the rotated key of pair i, one token per
// column): the A operand is register i / 16 of the per-tile query registers, broadcast from the
// block of four lanes i % 16.
typedef float mfma_f4 __attribute__((ext_vector_type(4)));
template <int ABID>
__device__ __forceinline__ mfma_f4 mfma_bcast(float a, float b, mfma_f4 c)
{
    return __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, c, 4, ABID, 0);
}
__device__ __forceinline__ mfma_f4 mfma_pair(const float (&q)[4], float x, mfma_f4 c, int i)
{
    const float a = q[i >> 4];
    switch (i & 15) {
        case 0: return mfma_bcast<0>(a, x, c);
        case 1: return mfma_bcast<1>(a, x, c);
        case 2: return mfma_bcast<2>(a, x, c);
        case 3: return mfma_bcast<3>(a, x, c);
        case 4: return mfma_bcast<4>(a, x, c);
        case 5: return mfma_bcast<5>(a, x, c);
        case 6: return mfma_bcast<6>(a, x, c);
        case 7: return mfma_bcast<7>(a, x, c);
        case 8: return mfma_bcast<8>(a, x, c);
        case 9: return mfma_bcast<9>(a, x, c);
        case 10: return mfma_bcast<10>(a, x, c);
        case 11: return mfma_bcast<11>(a, x, c);
        case 12: return mfma_bcast<12>(a, x, c);
        case 13: return mfma_bcast<13>(a, x, c);
        case 14: return mfma_bcast<14>(a, x, c);
        default: return mfma_bcast<15>(a, x, c);
    }
}

// The mixed-precision multiply-adds with a vector operand in place of the scalar one.
__device__ __forceinline__ float mixv_mul(bool HI, unsigned w, float s)
{
    float d;
    if (HI) asm volatile("v_fma_mix_f32 %0, %1, %2, 0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(w), "v"(s));
    else asm volatile("v_fma_mix_f32 %0, %1, %2, 0 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(w), "v"(s));
    return d;
}
// (Its result feeds a matrix instruction.  The compiler does not look inside an asm statement, so
// it cannot know that a vector instruction wrote the register and leaves out the two wait states
// that a matrix instruction reading it needs.  The caller keeps the two apart instead: all
// sixteen results of a batch pass through one more (empty) statement before the first matrix
// instruction may read any of them, so that at least eight instructions lie between a result
// and its use.)
template <bool MINUS>
__device__ __forceinline__ float mixv_fma(bool HI, unsigned w, float s, float c)
{
    float d;
    if (HI && MINUS) asm volatile("v_fma_mix_f32 %0, %1, %2, -%3 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(w), "v"(s), "v"(c));
    else if (HI) asm volatile("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(w), "v"(s), "v"(c));
    else if (MINUS) asm volatile("v_fma_mix_f32 %0, %1, %2, -%3 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(w), "v"(s), "v"(c));
    else asm volatile("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(w), "v"(s), "v"(c));
    return d;
}

// Grouped queries: the (up to) four query heads of a KV head that one workgroup serves share
// every key rotation.  The roles of the two halves of the angle are swapped against the kernel
// above: the KEY is rotated by the lane's part (cos / sin(u th_i): 128 registers per lane, from
// the [pair][lane] table) -- that is the same for all heads --
//     X_i = k_i cos(u th_i) - k_{i+64} sin(u th_i),   Y_i = k_{i+64} cos(u th_i) + k_i sin(u th_i),
// and each head's QUERY by the tile's part, once per tile (lane 4 p + h computes pairs p, p + 16,
// p + 32, p + 48 of head h),
//     A_i = q_i cos(t0 th_i) + q_{i+64} sin(t0 th_i),   B_i = q_{i+64} cos(t0 th_i) - q_i sin(t0 th_i),
// so that score(token, head) = sum_i X_i A_i + Y_i B_i is a product of a [token][pair] matrix that
// lives one column per instruction in a register (lane = token) and a [pair][head] matrix: one
// v_mfma_f32_4x4x1_16B_f32 per X_i and per Y_i, the A operand (4 heads x 1) broadcast from the
// block of four lanes that holds pair i to all 16 blocks, the B operand (1 x 4 tokens per
// block) the rotated key itself; lane = token also in the result, heads in its four registers.
// Per pair: 4 vector instructions and 2 matrix instructions for four heads, against 6 vector
// instructions per head.  Phase V and the epilogue run once per head over the split's scores
// in LDS (the value tiles of the later heads come from L2).
template <int GH, int C, int NT, bool STEP>
__global__ __launch_bounds__(NT) void decode_rope_gqa_kernel(DecodeArgs a, const float2* tile_tab, const float2* lane_tab)
{
    constexpr int B = 8, QH = 4;
    using F = Fmt<GH, B>;
    typedef float f4 __attribute__((ext_vector_type(4)));
    constexpr int K = F::K, RW = F::RW, R = F::R;
    constexpr int NW = NT / 64;
    constexpr int D = GH * C;
    constexpr int HALF = GH / 2;
    constexpr int PF = GH == 16 ? 4 : (GH == 32 ? 2 : 1);
    constexpr int JPL = 8 / C;
    constexpr int NCH = GH / 16;
    constexpr int UNITS = 16 * K / JPL;
    constexpr int IPT = UNITS / NT;
    static_assert(D == 128 && UNITS % NT == 0 && NT == kRopeThreads, "head_dim 128");
    constexpr unsigned SC_BASE = kTabBytes + kScrBytes;
    extern __shared__ float smem[];
    float* tab = smem;                                              // centroids in phase K, bins in phase V
    float* scr = smem + kTabBytes / 4;                              // reductions
    float* sc = smem + SC_BASE / 4;                                 // scores of the split: [head][token]
    // fused step: (distance, index) minima per group, keys[0..GH) for K, [GH..2GH) for V, then the new token's weight
    unsigned long long* keys = reinterpret_cast<unsigned long long*>(smem + SC_BASE / 4 + QH * a.tiles_per_split * kTileTokens);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // workgroup -> (sequence, split, quad of query heads), KV head a function of blockIdx % 8
    const int qper = a.n_q_heads / a.f.n_kv_heads;
    const int quads = (qper + QH - 1) / QH;
    int hkv, quad, split, n;
    {
        int r = blockIdx.x;
        if (a.f.n_kv_heads % 8 == 0) {
            const int per_xcd = a.f.n_kv_heads >> 3;
            const int xcd = r & 7;
            r >>= 3;
            hkv = xcd + 8 * (r % per_xcd);
            r /= per_xcd;
        } else {
            hkv = r % a.f.n_kv_heads;
            r /= a.f.n_kv_heads;
        }
        quad = r % quads;
        r /= quads;
        split = r % a.n_split;
        n = r / a.n_split;
    }
    const int hq0 = hkv * qper + quad * QH;
    const int heads = min(QH, qper - quad * QH);

    int t_n = a.t;
    if (a.seq_lens) t_n = min(max(a.seq_lens[n] - a.seq_len_shift, a.seq_len_floor), a.t);
    const int n_tiles = (t_n + kTileTokens - 1) / kTileTokens;
    const int tile0 = split * a.tiles_per_split;
    const int tile1 = min(tile0 + a.tiles_per_split, n_tiles);
    const bool direct = a.n_split == 1;
    if (tile0 >= tile1) {
        for (int h = 0; h < heads; ++h) {
            float* part = a.partials + ((size_t)(n * a.n_q_heads + hq0 + h) * a.n_split + split) * (D + kPartialHeader);
            if (tid == 0) { part[0] = -INFINITY; part[1] = 0.f; }
            for (int i = tid; i < D; i += NT) part[kPartialHeader + i] = 0.f;
        }
        return;
    }
    const int split_tokens = a.tiles_per_split * kTileTokens;
    // fused step (as in the kernel above): the workgroup whose split holds the newest position encodes
    // the new key row against the centroids it has just brought into LDS and patches the tile
    // that holds the position in registers; the new value row is encoded before the per-head
    // passes, which leave the position out of the bins and add its weight to the bins of the
    // codes found.  The workgroup of the KV head's first four query heads stores the codes.
    const int pos_new = t_n - 1;
    const int tile_new = pos_new / kTileTokens, u_new = pos_new % kTileTokens;
    const bool has_new = STEP && tile_new >= tile0 && tile_new < tile1;
    const bool writer = has_new && quad == 0;
    if (has_new && tid < 2 * GH) keys[tid] = ~0ull;         // (ordered by the barrier behind the table copy)

    Columns<GH, B> col;
    const int my_tiles = (tile1 - tile0 - wave + NW - 1) / NW;
    TileWalk<GH, B> kwalk, vwalk;
    kwalk.first = tile0 + wave;
    kwalk.stride = NW;
    kwalk.pages = 0;
    if (a.map.block_table) {
        if (lane < my_tiles) kwalk.pages = a.map.page(n, tile0 + wave + lane * NW);
        kwalk.page_bytes = (size_t)a.f.n_kv_heads * F::TILE_BYTES;
        kwalk.base = a.k_codes + (size_t)hkv * F::TILE_BYTES;
        vwalk = kwalk;
        vwalk.base = a.v_codes + (size_t)hkv * F::TILE_BYTES;
    } else {
        const size_t stream_idx = a.map.tile_index(n, hkv, 0) * F::TILE_BYTES;
        kwalk.page_bytes = 0;
        kwalk.base = a.k_codes + stream_idx;
        vwalk = kwalk;
        vwalk.base = a.v_codes + stream_idx;
    }
    Streamer<GH, B, 1> stk;
    Streamer<GH, B, PF> st;

    // ---- 1. the head's key centroids go to LDS; the lane's cosines and sines; this lane's query slices ----
    {
        const uint4* src = reinterpret_cast<const uint4*>(a.k_centroids + (size_t)hkv * GH * K * C);
        for (int i = tid; i < (int)(kTabBytes / 16); i += NT) reinterpret_cast<uint4*>(smem)[i] = src[i];
    }
    stk.begin(kwalk, my_tiles, lane);
    float cu[kPairs], su[kPairs];
#pragma unroll
    for (int i = 0; i < kPairs; ++i) {
        const float2 t = lane_tab[i * 64 + lane];
        cu[i] = t.x;
        su[i] = t.y;
    }
    // lane 4 p + h: pairs p + 16 m of head h (zero for a head this workgroup does not have)
    const int hl = lane & 3, pl = lane >> 2;
    float qlo[4], qhi[4];
    {
        const uint16_t* qh = a.q + (size_t)n * a.q_batch_stride + (size_t)(hq0 + (hl < heads ? hl : 0)) * D;
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const float s = hl < heads ? a.scale_log2e : 0.f;
            qlo[m] = (float)__builtin_bit_cast(_Float16, qh[16 * m + pl]) * s;
            qhi[m] = (float)__builtin_bit_cast(_Float16, qh[16 * m + pl + kPairs]) * s;
        }
    }
    // cos / sin of a tile's base position for this lane's four pairs, read one tile ahead
    auto tile_cs = [&](int k, float2 (&dst)[4]) {
        const int kk = k < my_tiles ? k : (my_tiles > 0 ? my_tiles - 1 : 0);
        const int tile = my_tiles > 0 ? tile0 + wave + kk * NW : tile0;
#pragma unroll
        for (int m = 0; m < 4; ++m) dst[m] = tile_tab[(size_t)tile * kPairs + 16 * m + pl];
    };
    float2 cs_next[4];
    tile_cs(0, cs_next);
    lds_barrier();
    if (has_new) {
        constexpr int TPG = NT / GH;
        const int g = tid / TPG;
        const size_t xrow = (size_t)n * a.x_new_stride + (size_t)hkv * GH * C;
        float xk[C];
        load_row_slice<C>(a.xk_new + xrow + g * C, xk);
        Nearest knear;
        for (int j = tid % TPG; j < K; j += TPG) {
            const CenVec<C> cen = lds_centroid<C>((unsigned)(g * K + j) * (C * 2));
            knear.offer(centroid_distance<C>(xk, cen.w), j);
        }
        lds_min_u64(&keys[g], knear.key());
        lds_barrier();
        if (writer)
            store_new_codes<GH, B>(const_cast<uint8_t*>(a.k_codes) + a.map.tile_index(n, hkv, tile_new) * F::TILE_BYTES, keys, u_new, tid);
    }
    const bool meets_new = has_new && (tile_new - tile0) % NW == wave;
    NewTokenCodes<GH, B> new_codes;
    if (meets_new) new_codes.build(keys, u_new, lane);

    // ---- 2. phase K: scores of four heads --------------------------------------------------
    Unrotate unrot;
    unrot.bytes = (unsigned)(GH - lane) & 3u;
    unrot.dwords = ((unsigned)(GH - lane) & (unsigned)(GH - 1)) >> 2;
    constexpr int kBatch = 8;                       // channel pairs per batch of centroids
    constexpr int GPB = kBatch / C;                 // groups (of each half of the head) per batch
    stk.run(kwalk, my_tiles, lane, [&](const Tile<GH, B>& w_in, int k) {
        const int lt = wave + k * NW;
        Tile<GH, B> w = w_in;
        if (meets_new && tile0 + lt == tile_new) new_codes.patch(w, u_new, lane);
        // the queries rotated to the tile's base position, in the A-operand layout
        float qa[4], qb[4];
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const float2 t = cs_next[m];
            qa[m] = __builtin_fmaf(qlo[m], t.x, qhi[m] * t.y);
            qb[m] = __builtin_fmaf(qhi[m], t.x, -(qlo[m] * t.y));
        }
        tile_cs(k + 1, cs_next);
        unsigned d[GH / 4];
        group_order<GH, B>(w, unrot, d);
        // four accumulators: a matrix instruction that adds to the result of the one before it has to wait for it
        f4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f}, acc2 = {0.f, 0.f, 0.f, 0.f}, acc3 = {0.f, 0.f, 0.f, 0.f};
        auto centroids = [&](int bi, CenVec<C> (&ka)[GPB], CenVec<C> (&kb)[GPB], float after) {
#pragma unroll
            for (int gg = 0; gg < GPB; ++gg) {
                const int g = bi * GPB + gg;
                unsigned c_first = (d[g >> 2] >> (8 * (g & 3))) & 0xffu;
                unsigned c_second = (d[(g + HALF) >> 2] >> (8 * ((g + HALF) & 3))) & 0xffu;
                asm volatile("" : "+v"(c_first), "+v"(c_second) : "v"(after));
                ka[gg] = lds_centroid<C>(c_first * (C * 2) + (unsigned)(g * K * C * 2));
                kb[gg] = lds_centroid<C>(c_second * (C * 2) + (unsigned)((g + HALF) * K * C * 2));
            }
        };
        CenVec<C> ka[GPB], kb[GPB];
        centroids(0, ka, kb, 0.f);
#pragma unroll
        for (int bi = 0; bi < kPairs / kBatch; ++bi) {
            CenVec<C> ka_n[GPB], kb_n[GPB];
            float t1[kBatch], t2[kBatch], x[kBatch], y[kBatch];
#pragma unroll
            for (int e = 0; e < kBatch; ++e) t1[e] = mixv_mul((e % C) & 1, kb[e / C].w[(e % C) >> 1], su[bi * kBatch + e]);
            // the next batch's centroids: requested behind the first use of this batch's
            if (bi + 1 < kPairs / kBatch) centroids(bi + 1, ka_n, kb_n, t1[0]);
#pragma unroll
            for (int e = 0; e < kBatch; ++e) t2[e] = mixv_mul((e % C) & 1, ka[e / C].w[(e % C) >> 1], su[bi * kBatch + e]);
#pragma unroll
            for (int e = 0; e < kBatch; ++e) x[e] = mixv_fma<true>((e % C) & 1, ka[e / C].w[(e % C) >> 1], cu[bi * kBatch + e], t1[e]);
#pragma unroll
            for (int e = 0; e < kBatch; ++e) y[e] = mixv_fma<false>((e % C) & 1, kb[e / C].w[(e % C) >> 1], cu[bi * kBatch + e], t2[e]);
            static_assert(kBatch == 8, "operands of the statement below");
            asm volatile("" : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7]),
                              "+v"(y[0]), "+v"(y[1]), "+v"(y[2]), "+v"(y[3]), "+v"(y[4]), "+v"(y[5]), "+v"(y[6]), "+v"(y[7]));
#pragma unroll
            for (int e = 0; e < kBatch; ++e) {
                const int i = bi * kBatch + e;              // pair i: register i / 16 of the block of lanes i % 16
                if (e & 1) {
                    acc2 = mfma_pair(qa, x[e], acc2, i);
                    acc3 = mfma_pair(qb, y[e], acc3, i);
                } else {
                    acc0 = mfma_pair(qa, x[e], acc0, i);
                    acc1 = mfma_pair(qb, y[e], acc1, i);
                }
            }
            asm volatile("" : "+v"(acc0), "+v"(acc1), "+v"(acc2), "+v"(acc3));
            if (bi + 1 < kPairs / kBatch) {
#pragma unroll
                for (int gg = 0; gg < GPB; ++gg) { ka[gg] = ka_n[gg]; kb[gg] = kb_n[gg]; }
            }
        }
        const int tok = (tile0 + lt) * kTileTokens + lane;
        const bool live = tok < t_n;
#pragma unroll
        for (int h = 0; h < QH; ++h) sc[h * split_tokens + lt * kTileTokens + lane] = live ? (acc0[h] + acc1[h]) + (acc2[h] + acc3[h]) : -INFINITY;
    }, [] {});
    lds_barrier();                                  // all centroid reads done, all scores written

    // ---- 3. per head: softmax reference, phase V, epilogue ----------------------------------
    col.init(lane);
    // (the four lanes of a group are neighbours and read four neighbouring 16-byte pieces of its
    // value codebook: 64 contiguous bytes, four cache lines per 16 lanes instead of sixteen)
    const int gl16 = (tid >> 2) & 15;
    auto piece = [&](int k) { return (((tid + k * NT) >> 6) << 2) + (tid & 3); };
    constexpr int KB = IPT < 8 ? IPT : 8;
    const int n_tok = (tile1 - tile0) * kTileTokens;
    unsigned* pf_new = reinterpret_cast<unsigned*>(keys + 2 * GH);
    if (has_new) {
        // the new value row against the value codebook (global memory): the walk of the epilogue,
        // ascending index per thread, 64-bit minimum over the threads of a group
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
            const size_t xrow = (size_t)n * a.x_new_stride + (size_t)hkv * GH * C;
            float xv[C];
            load_row_slice<C>(a.xv_new + xrow + (ch * 16 + gl16) * C, xv);
            const uint16_t* cvg = a.v_centroids + (size_t)(hkv * GH + ch * 16 + gl16) * K * C;
            Nearest vnear;
#pragma unroll
            for (int k0 = 0; k0 < IPT; k0 += KB) {
                Cent16 rawb[KB];
#pragma unroll
                for (int k = 0; k < KB; ++k) rawb[k] = load_cent16(cvg + (size_t)piece(k0 + k) * 8);
#pragma unroll
                for (int k = 0; k < KB; ++k) {
                    const int j0 = piece(k0 + k) * JPL;
#pragma unroll
                    for (int jj = 0; jj < JPL; ++jj) vnear.offer(centroid_distance<C>(xv, &rawb[k].w[jj * (C / 2)]), j0 + jj);
                }
            }
            const unsigned long long vkey = group_lanes_min<4>(vnear.key());
            if ((lane & 3) == 0) lds_min_u64(&keys[GH + ch * 16 + gl16], vkey);
        }
        lds_barrier();
        if (writer)
            store_new_codes<GH, B>(const_cast<uint8_t*>(a.v_codes) + a.map.tile_index(n, hkv, tile_new) * F::TILE_BYTES, keys + GH, u_new, tid);
    }
    // Two heads per pass where the bins of two fit side by side (16 or 32 groups per head: words
    // 0..31 of a 64-word row are the columns of one head's bins, words 32..63 the other's), so
    // that the value tiles are streamed twice, not four times.  The value centroids of the
    // epilogue are the same for every head: they stay in registers where they fit.
    constexpr int HP = GH <= 32 ? 2 : 1;
    constexpr bool KEEP = IPT * NCH <= 8 && KB == IPT;
    Cent16 rawv[KEEP ? NCH : 1][KB];
    if constexpr (KEEP) {
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
            const uint16_t* cv = a.v_centroids + (size_t)(hkv * GH + ch * 16 + gl16) * K * C;
#pragma unroll
            for (int k = 0; k < IPT; ++k) rawv[ch][k] = load_cent16(cv + (size_t)piece(k) * 8);
        }
    }
    for (int h0 = 0; h0 < heads; h0 += HP) {
        const int nh = min(HP, heads - h0);                 // heads of this pass
        // scr: [0..16) sums, [16..32) maxima, [32..48) estimates of l; 8 wavefronts x 2 heads each
        float m[HP], fx_scale[HP], fx_inv[HP];
#pragma unroll
        for (int e = 0; e < HP; ++e) {
            const float* sch = sc + (h0 + (e < nh ? e : 0)) * split_tokens;
            float lane_max = -INFINITY;
            for (int i = tid; i < n_tok; i += NT) lane_max = fmaxf(lane_max, sch[i]);
            lane_max = wave_max(lane_max);
            if (lane == 0) scr[16 + e * NW + wave] = lane_max;
        }
        st.begin(vwalk, my_tiles, lane);
        lds_barrier();
#pragma unroll
        for (int e = 0; e < HP; ++e) {
            const float* sch = sc + (h0 + (e < nh ? e : 0)) * split_tokens;
            float mm = scr[16 + e * NW];
#pragma unroll
            for (int w = 1; w < NW; ++w) mm = fmaxf(mm, scr[16 + e * NW + w]);
            m[e] = mm;
            float l_est = 0.f;
            for (int i = tid; i < n_tok; i += NT) l_est += __builtin_amdgcn_exp2f(sch[i] - mm);
            l_est = wave_sum(l_est);
            if (lane == 0) scr[32 + e * NW + wave] = l_est;
        }
        {
            float4* t4 = reinterpret_cast<float4*>(tab);
#pragma unroll 4
            for (int i = tid; i < F::TAB_FLOATS / 4; i += NT) t4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
        lds_barrier();
#pragma unroll
        for (int e = 0; e < HP; ++e) {
            float l_est = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) l_est += scr[32 + e * NW + w];
            const int fx = fixed_point_exponent(l_est);
            fx_scale[e] = ldexpf(1.f, fx);
            fx_inv[e] = ldexpf(1.f, -fx);
        }

        unsigned lane_sum[HP];
#pragma unroll
        for (int e = 0; e < HP; ++e) lane_sum[e] = 0;
        const float* sc0 = sc + h0 * split_tokens;
        const float* sc1 = sc + (h0 + (nh > 1 ? 1 : 0)) * split_tokens;
        st.run(vwalk, my_tiles, lane, [&](const Tile<GH, B>& w, int k) {
            const int lt = wave + k * NW;
            unsigned pf[HP];
#pragma unroll
            for (int e = 0; e < HP; ++e) {
                const float p = __builtin_amdgcn_exp2f((e ? sc1 : sc0)[lt * kTileTokens + lane] - m[e]);
                pf[e] = (unsigned)__builtin_fmaf(p, fx_scale[e], 0.5f);
                lane_sum[e] += pf[e];
            }
            if (has_new && tile0 + lt == tile_new && lane == u_new) {
#pragma unroll
                for (int e = 0; e < HP; ++e) {
                    pf_new[e] = pf[e];
                    pf[e] = 0;
                }
            }
#pragma unroll
            for (int s = 0; s < GH; ++s) {
                const unsigned addr = slot_addr<GH, B, false>(w, col, s);
                lds_add(addr, pf[0]);
                if constexpr (HP == 2) lds_add(addr + 128u, pf[1]);
            }
        }, [] {});
#pragma unroll
        for (int e = 0; e < HP; ++e) lane_sum[e] = wave_sum_u32(lane_sum[e]);
        lds_barrier();
        if (lane == 0) {
#pragma unroll
            for (int e = 0; e < HP; ++e) scr[e * NW + wave] = __uint_as_float(lane_sum[e]);
        }
        if (has_new) {
            if (tid < GH) {
                const unsigned code = (unsigned)(keys[GH + tid] & 0xffffffffu);
#pragma unroll
                for (int e = 0; e < HP; ++e) lds_add((code * RW + tid * R) * 4u + 128u * e, pf_new[e]);
            }
            lds_barrier();
        }

        for (int e = 0; e < nh; ++e) {
            float acc[NCH][C];
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
#pragma unroll
                for (int i = 0; i < C; ++i) acc[ch][i] = 0.f;
                const uint16_t* cv = a.v_centroids + (size_t)(hkv * GH + ch * 16 + gl16) * K * C;
#pragma unroll
                for (int k0 = 0; k0 < IPT; k0 += KB) {
                    if constexpr (!KEEP) {
#pragma unroll
                        for (int k = 0; k < KB; ++k) rawv[0][k] = load_cent16(cv + (size_t)piece(k0 + k) * 8);
                    }
                    const Cent16 (&raw)[KB] = rawv[KEEP ? ch : 0];
#pragma unroll
                    for (int k = 0; k < KB; ++k) {
                        const int j0 = piece(k0 + k) * JPL;
#pragma unroll
                        for (int jj = 0; jj < JPL; ++jj) {
                            const float* src = tab + (j0 + jj) * RW + (ch * 16 + gl16) * R + 32 * e;
                            unsigned cnt;
                            if constexpr (R == 2) { const uint2 x = *reinterpret_cast<const uint2*>(src); cnt = x.x + x.y; }
                            else cnt = *reinterpret_cast<const unsigned*>(src);
                            const float bin = (float)cnt * (e ? fx_inv[HP - 1] : fx_inv[0]);
#pragma unroll
                            for (int i = 0; i < C / 2; ++i) {
                                const half2_t hv = __builtin_bit_cast(half2_t, raw[k].w[jj * (C / 2) + i]);
                                acc[ch][2 * i] = __builtin_fmaf(bin, (float)hv.x, acc[ch][2 * i]);
                                acc[ch][2 * i + 1] = __builtin_fmaf(bin, (float)hv.y, acc[ch][2 * i + 1]);
                            }
                        }
                    }
                }
#pragma unroll
                for (int i = 0; i < C; ++i) {
                    acc[ch][i] += __shfl_xor(acc[ch][i], 1);
                    acc[ch][i] += __shfl_xor(acc[ch][i], 2);
                }
            }
            if ((lane & 3) == 0) {
#pragma unroll
                for (int ch = 0; ch < NCH; ++ch)
#pragma unroll
                    for (int i = 0; i < C; ++i) scr[64 + wave * D + (ch * 16 + gl16) * C + i] = acc[ch][i];
            }
            lds_barrier();
            unsigned l_fix = 0;
#pragma unroll
            for (int w = 0; w < NW; ++w) l_fix += __float_as_uint(scr[e * NW + w]);
            const float l = (float)l_fix * (e ? fx_inv[HP - 1] : fx_inv[0]);
            const int hq = hq0 + h0 + e;
            float* part = a.partials + ((size_t)(n * a.n_q_heads + hq) * a.n_split + split) * (D + kPartialHeader);
            if (tid == 0 && !direct) {
                part[0] = e ? m[HP - 1] : m[0];
                part[1] = l;
            }
            for (int chn = tid; chn < D; chn += NT) {
                float o = 0.f;
#pragma unroll
                for (int w = 0; w < NW; ++w) o += scr[64 + w * D + chn];
                if (direct) a.out[(size_t)n * a.out_batch_stride + (size_t)hq * D + chn] = __builtin_bit_cast(uint16_t, (_Float16)(o / l));
                else part[kPartialHeader + chn] = o;
            }
            lds_barrier();                          // the next head reuses the scratch, the next pass the bins
        }
    }
}

template <int GH, int C, bool STEP, int B = 8>
cq_status launch_rope_variant(const DecodeArgs& a, const float2* tile_tab, const float2* lane_tab, hipStream_t stream)
{
    constexpr int NT = kRopeThreads;
    auto kernel = decode_rope_kernel<GH, C, NT, STEP, B>;
    static LdsKernelSetup setup;
    if (setup.ensure(reinterpret_cast<const void*>(kernel)) != hipSuccess) return CQ_ERR_HIP;
    const size_t smem = kTabBytes + kScrBytes + (size_t)a.tiles_per_split * kTileTokens * 4 + (STEP ? kKeyFloats(GH) * 4 : 0);
    if (smem > 160 * 1024) return CQ_ERR_INVALID_ARG;
    const unsigned grid = (unsigned)(a.batch * a.n_q_heads * a.n_split);
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(NT), smem, stream, a, tile_tab, lane_tab);
    return hipGetLastError() == hipSuccess ? CQ_OK : CQ_ERR_HIP;
}

template <int GH, int C, bool STEP>
cq_status launch_rope_gqa_variant(const DecodeArgs& a, const float2* tile_tab, const float2* lane_tab, hipStream_t stream)
{
    constexpr int NT = kRopeThreads;
    auto kernel = decode_rope_gqa_kernel<GH, C, NT, STEP>;
    static LdsKernelSetup setup;
    if (setup.ensure(reinterpret_cast<const void*>(kernel)) != hipSuccess) return CQ_ERR_HIP;
    const size_t smem = kTabBytes + kScrBytes + (size_t)4 * a.tiles_per_split * kTileTokens * 4 + (STEP ? kKeyFloats(GH) * 4 : 0);
    if (smem > 160 * 1024) return CQ_ERR_INVALID_ARG;
    const int qper = a.n_q_heads / a.f.n_kv_heads;
    const unsigned grid = (unsigned)(a.batch * a.f.n_kv_heads * ((qper + 3) / 4) * a.n_split);
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(NT), smem, stream, a, tile_tab, lane_tab);
    return hipGetLastError() == hipSuccess ? CQ_OK : CQ_ERR_HIP;
}

}  // namespace

int decode_rope_max_tiles_per_split() { return 256; }

// grouped queries (two or more query heads per KV head, byte codes): splits of at
// most this many tiles run the kernel that shares the key rotation among four query heads
// (scores of four heads beside the centroids in LDS)
constexpr int kGqaTiles = 88;
int decode_rope_shared_max_tiles_per_split() { return kGqaTiles; }
static_assert(kTabBytes + kScrBytes + 4 * kGqaTiles * kTileTokens * 4 + kKeyFloats(64) * 4 <= 160 * 1024, "LDS of the grouped-query kernel");

size_t rope_table_floats(int t_cap) { return ((size_t)(t_cap / kTileTokens) * kPairs + (size_t)kPairs * 64) * 2; }

cq_status launch_rope_table(double base, int t_cap, float* tables, hipStream_t stream)
{
    const int n_tiles = t_cap / kTileTokens;
    float2* tile_tab = reinterpret_cast<float2*>(tables);
    float2* lane_tab = tile_tab + (size_t)n_tiles * kPairs;
    const int total = n_tiles * kPairs + kPairs * 64;
    hipLaunchKernelGGL(rope_tables_kernel, dim3((total + 255) / 256), dim3(256), 0, stream, base, n_tiles, tile_tab, lane_tab);
    return hipGetLastError() == hipSuccess ? CQ_OK : CQ_ERR_HIP;
}

cq_status launch_decode_rope(const DecodeArgs& a, const float* tables, int t_cap, hipStream_t stream)
{
    const float2* tile_tab = reinterpret_cast<const float2*>(tables);
    const float2* lane_tab = tile_tab + (size_t)(t_cap / kTileTokens) * kPairs;
    cq_status st = CQ_ERR_UNSUPPORTED;
    const bool shared = a.f.b == 8 && a.f.head_dim == 128 && a.n_q_heads >= 2 * a.f.n_kv_heads && a.tiles_per_split <= kGqaTiles;
    if (shared) {
        const bool step = a.xk_new != nullptr;
        if (a.f.gh == 16 && a.f.c == 8)
            st = step ? launch_rope_gqa_variant<16, 8, true>(a, tile_tab, lane_tab, stream) : launch_rope_gqa_variant<16, 8, false>(a, tile_tab, lane_tab, stream);
        else if (a.f.gh == 32 && a.f.c == 4)
            st = step ? launch_rope_gqa_variant<32, 4, true>(a, tile_tab, lane_tab, stream) : launch_rope_gqa_variant<32, 4, false>(a, tile_tab, lane_tab, stream);
        else if (a.f.gh == 64 && a.f.c == 2)
            st = step ? launch_rope_gqa_variant<64, 2, true>(a, tile_tab, lane_tab, stream) : launch_rope_gqa_variant<64, 2, false>(a, tile_tab, lane_tab, stream);
    } else if (a.f.b == 8 && a.f.head_dim == 128) {
        const bool step = a.xk_new != nullptr;
        if (a.f.gh == 16 && a.f.c == 8)
            st = step ? launch_rope_variant<16, 8, true>(a, tile_tab, lane_tab, stream) : launch_rope_variant<16, 8, false>(a, tile_tab, lane_tab, stream);
        else if (a.f.gh == 32 && a.f.c == 4)
            st = step ? launch_rope_variant<32, 4, true>(a, tile_tab, lane_tab, stream) : launch_rope_variant<32, 4, false>(a, tile_tab, lane_tab, stream);
        else if (a.f.gh == 64 && a.f.c == 2)
            st = step ? launch_rope_variant<64, 2, true>(a, tile_tab, lane_tab, stream) : launch_rope_variant<64, 2, false>(a, tile_tab, lane_tab, stream);
    }
    if (a.f.b == 10 && a.f.head_dim == 128 && a.f.gh == 16 && a.f.c == 8)
        st = a.xk_new ? launch_rope_variant<16, 8, true, 10>(a, tile_tab, lane_tab, stream)
                      : launch_rope_variant<16, 8, false, 10>(a, tile_tab, lane_tab, stream);
    if (st != CQ_OK) return st;
    if (a.n_split > 1)
        return launch_decode_merge(a.partials, a.out, a.batch * a.n_q_heads, a.n_q_heads, a.out_batch_stride, a.n_split, a.f.head_dim, stream);
    return CQ_OK;
}

}  // namespace cq

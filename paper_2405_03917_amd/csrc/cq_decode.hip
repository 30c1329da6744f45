// Decode attention straight from packed CQ codes (Eq. 1 of the paper over the centroids the
// cached codes select), for gfx950.
//
// One workgroup handles one (sequence, query head, context split).  Per workgroup:
//   1. build the score table  LUT[g][j] = scale * log2(e) * (q_g . C_K[g][j])  in LDS;
//   2. phase K: stream the split's key codes (one 64-token tile per wavefront per step, lane =
//      token), score = sum over groups of LUT[g][code]; keep scores in LDS, reduce the maximum;
//   3. phase V: stream the value codes; p = 2^(score - max) in fixed point; add p into
//      bin[g][code] in LDS with integer atomics (exact, order independent);
//   4. epilogue: o[g c + i] = sum_j bin[g][j] * C_V[g][j][i]; with a single split the normalised
//      result is rounded to fp16 and stored, otherwise (max, sum p, o) goes out as a partial and
//      a second kernel merges the partials of all splits.
//
// LDS table layout: one row per code value, RW four-byte words per row (b = 8: 256 rows of 64
// words = 64 KB; b = 10: 1024 rows of 16 words = 64 KB).  Lane l of a wavefront owns ONE word
// column at every step s of the walk over a token's Gh slots: column(l, g) with g = (l + s) mod
// Gh, the group that the cache layout put in slot s of token l.  With 32 or 64 groups per head
// the 32 columns of a half-wavefront are different modulo 32 (lanes l and l + 32 may share one:
// the LDS serves a wavefront in two halves), so neither the table gather nor the bin update ever
// has a bank conflict.  With 16 groups per head and b = 8 each group is replicated twice to give
// 32 lanes their own column (the epilogue adds the replicas), except in the form for long splits
// (LONG) and for b = 10, which keep one column per group and the row space for other uses:
// measured, the lanes that then share a column cost 2-4 % at equal split length.  For b = 8 the byte address of
// a lookup is (code << 8) | (4 * column): one v_perm_b32 from the code word and a per-lane
// constant.  With 16 or 32 groups per head only words 0..31 (0..15: LONG) of a 256-byte row are
// columns; the remaining words of the 256 rows hold the split's scores (8192 of them; 12288:
// LONG), which keeps a workgroup under 70 KB of LDS so that two of them share a CU.
//
// Measured on MI355X (microbenchmark, per CU): ds_read_b32 gathers and ds_add_u32 run at the
// same rate with this layout as with linear addresses; ds_add_f32 is about 45 times slower than
// ds_add_u32, which is why the bins are integers.
#include <hip/hip_runtime.h>

#include "cq_decode_common.hpp"

namespace cq {
namespace {

// LayerPtrs as the kernel reads it.  A pointer read from memory could point anywhere (LDS,
// scratch) as far as the compiler knows, and every access through it would be a flat instruction,
// which waits on the LDS counter and the memory counter at once; the table's pointers are
// therefore declared as what they are, pointers into global memory.
#define CQ_GLOBAL __attribute__((address_space(1)))
struct LayerPtrsGlobal {
    CQ_GLOBAL const uint16_t* q;
    CQ_GLOBAL const uint16_t* xk_new;
    CQ_GLOBAL const uint16_t* xv_new;
    CQ_GLOBAL uint8_t* k_codes;
    CQ_GLOBAL uint8_t* v_codes;
    CQ_GLOBAL const uint16_t* k_centroids;
    CQ_GLOBAL const uint16_t* v_centroids;
    CQ_GLOBAL uint16_t* out;
};
#undef CQ_GLOBAL
static_assert(sizeof(LayerPtrsGlobal) == sizeof(LayerPtrs), "same record");

__global__ void layer_table_write_kernel(LayerChunk chunk, int count, LayerPtrs* dst)
{
    if ((int)threadIdx.x < count) dst[threadIdx.x] = chunk.p[threadIdx.x];
}

// STEP = true is the fused decode step: the workgroup whose split holds the newest position
// (t_n - 1) also encodes that token's key and value rows for its KV head.  Keys: while it builds
// the score table (the key codebook is in registers anyway); the tile that holds the position is
// then patched in registers as if the codes were already in the cache.  Values: in the epilogue
// (the value codebook is in registers there); phase V leaves the position out of the bins and
// its weight is added to the bins of the codes just found.  The first query head of each KV head
// stores the codes.  Results equal cq_encode_kv followed by cq_decode_attention bit for bit
// (the bins are integers: the order of the additions does not matter).
// A kernel argument is loaded (scalar load from the argument block) where it is first used;
// left to the compiler, the prologue of this kernel loads its arguments in four dependent
// stages (head counts; split and context; strides; pointers), each awaited before the next is
// requested, and an argument added to a late stage delays the first global load (measured: 0.3-0.4
// us per launch of the attention kernel for two more strides).  early() pins a value in a scalar
// register at the point of the call, so that everything the workgroup needs before its first
// global load is requested together at entry and awaited once.
// (A pointer comes back as a pointer into global memory, which is what every pointer argument
// of these kernels is: a pointer of unknown provenance would make each access through it a flat
// instruction.)
template <class T>
__device__ __forceinline__ T* early(T* p)
{
    unsigned long long x = reinterpret_cast<unsigned long long>(p);
    asm volatile("" : "+s"(x));
    return (T*)reinterpret_cast<__attribute__((address_space(1))) T*>(x);
}
template <class T>
__device__ __forceinline__ T early(T v)
{
    if constexpr (sizeof(T) == 4) {
        unsigned x = __builtin_bit_cast(unsigned, v);
        asm volatile("" : "+s"(x));
        return __builtin_bit_cast(T, x);
    } else {
        static_assert(sizeof(T) == 8, "32- or 64-bit arguments");
        unsigned long long x = __builtin_bit_cast(unsigned long long, v);
        asm volatile("" : "+s"(x));
        return __builtin_bit_cast(T, x);
    }
}

template <bool STEP, bool LAYERS>
__device__ __forceinline__ DecodeArgs early_args(const DecodeArgs& in)
{
    DecodeArgs a = in;                  // (what is not named below is read where it is used)
    // (not for a layer-batched launch: its workgroups overlap one another's prologues anyway, and
    // the pinned registers cost that variant 2 % at 32 groups per head)
    if constexpr (LAYERS) return a;
    a.n_q_heads = early(in.n_q_heads);
    a.f.n_kv_heads = early(in.f.n_kv_heads);
    a.n_split = early(in.n_split);
    a.tiles_per_split = early(in.tiles_per_split);
    a.t = early(in.t);
    a.seq_lens = early(in.seq_lens);
    a.seq_len_shift = early(in.seq_len_shift);
    a.seq_len_floor = early(in.seq_len_floor);
    a.map.block_table = early(in.map.block_table);
    a.map.bt_stride = early(in.map.bt_stride);
    a.map.n_pages = early(in.map.n_pages);
    a.map.tiles_cap = early(in.map.tiles_cap);
    a.map.n_kv_heads = early(in.map.n_kv_heads);
    a.scale_log2e = early(in.scale_log2e);
    a.partials = early(in.partials);
    a.q = early(in.q);
    a.k_codes = early(in.k_codes);
    a.v_codes = early(in.v_codes);
    a.k_centroids = early(in.k_centroids);
    a.v_centroids = early(in.v_centroids);
    a.out = early(in.out);
    a.q_batch_stride = early(in.q_batch_stride);
    a.out_batch_stride = early(in.out_batch_stride);
    if constexpr (STEP) {
        a.xk_new = early(in.xk_new);
        a.xv_new = early(in.xv_new);
        a.x_new_stride = early(in.x_new_stride);
    }
    return a;
}

template <int GH, int C, int B, int NT, bool STEP, bool LAYERS, bool LONG>
__global__ __launch_bounds__(NT, 4) void decode_split_kernel(DecodeArgs a_in)
{
    const DecodeArgs a = early_args<STEP, LAYERS>(a_in);
    using F = Fmt<GH, B, LONG>;
    constexpr int K = F::K, RW = F::RW, R = F::R;
    constexpr int NW = NT / 64;         // wavefronts
    constexpr int D = GH * C;           // head_dim
    // tiles in flight per wavefront (about 4 KB; less where registers are short)
    constexpr int PF = B == 10 ? 2 : (GH == 16 ? 4 : (GH == 32 ? 2 : 1));
    constexpr int JPL = 8 / C;          // centroids per 16-byte load
    constexpr int NCH = GH / 16;        // 16-group chunks
    constexpr int UNITS = 16 * K / JPL; // 16-byte loads per chunk
    constexpr int IPT = UNITS / NT;     // ... per thread
    constexpr int KB = IPT < 8 ? IPT : 8;   // ... requested together
    static_assert(UNITS % NT == 0 && NT % 16 == 0, "thread count must divide the codebook walk");
    extern __shared__ float smem[];
    float* tab = smem;                              // [K][RW]; first the score table, then the bins
    // scores of the split: interleaved into the table rows, or a buffer behind the table
    float* sc = F::SCORES_IN_TABLE ? smem : smem + F::TAB_FLOATS;
    auto sidx = [](int i) { return F::SCORES_IN_TABLE ? (i / F::SCORE_WORDS) * 64 + F::LUT_WORDS + i % F::SCORE_WORDS : i; };
    // reduction scratch: behind the table, or the (by then dead) score buffer
    float* scr = smem + F::TAB_FLOATS;
    // fused step: 64-bit (distance, index) minima per group, keys[0..GH) for K, [GH..2GH) for V
    unsigned long long* keys = reinterpret_cast<unsigned long long*>(
        smem + F::TAB_FLOATS + (F::SCORES_IN_TABLE ? kScratchFloats(NT, D) : max(kMinScoreFloats, a.tiles_per_split * kTileTokens)));

    // the wavefronts' (maximum, sum) pairs of phase K: in the reduction scratch, or (b = 10) behind
    // everything else; 64 groups per head have no LDS to spare (table + 4096 scores fill half a CU)
    constexpr bool SLOTS_BEHIND = F::SCORES_IN_TABLE || B == 10;
    float* slot_area = F::SCORES_IN_TABLE ? scr : reinterpret_cast<float*>(keys) + (STEP ? kKeyFloats(GH) : 0);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // Workgroup -> (sequence, split, query head).  Consecutive workgroups go to consecutive XCDs
    // (8 of them, each with its own L2), so the KV head is made a function of blockIdx % 8 where
    // the head count allows: every workgroup that reads a head's codebooks and code streams then
    // shares one L2 (with grouped queries that is 4 query heads x splits x sequences per head).
    const int qper = a.n_q_heads / a.f.n_kv_heads;
    // layer-batched launch: this workgroup's layer and that layer's tensors
    int bid = blockIdx.x;
    const uint16_t* q_ptr = a.q;
    const uint16_t* xk_new = a.xk_new;
    const uint16_t* xv_new = a.xv_new;
    const uint8_t* k_codes = a.k_codes;
    const uint8_t* v_codes = a.v_codes;
    const uint16_t* k_centroids = a.k_centroids;
    const uint16_t* v_centroids = a.v_centroids;
    uint16_t* out_ptr = a.out;
    float* partials = a.partials;
    const int64_t q_batch_stride = a.q_batch_stride, out_batch_stride = a.out_batch_stride;
    const int seq_len_shift = a.seq_len_shift, seq_len_floor = a.seq_len_floor;
    if constexpr (LAYERS) {
        const int layer = bid / a.wgs_per_layer;
        bid -= layer * a.wgs_per_layer;
        const LayerPtrsGlobal& lp = reinterpret_cast<const LayerPtrsGlobal*>(a.layers)[layer];
        q_ptr = (const uint16_t*)lp.q;
        xk_new = (const uint16_t*)lp.xk_new;
        xv_new = (const uint16_t*)lp.xv_new;
        k_codes = (const uint8_t*)lp.k_codes;
        v_codes = (const uint8_t*)lp.v_codes;
        k_centroids = (const uint16_t*)lp.k_centroids;
        v_centroids = (const uint16_t*)lp.v_centroids;
        out_ptr = (uint16_t*)lp.out;
        partials += (size_t)layer * a.wgs_per_layer * (D + kPartialHeader);
    }
    int hq, split, n;
    if (a.f.n_kv_heads % 8 == 0) {
        const int xcd = bid & 7;
        int r = bid >> 3;
        const int per_xcd = a.f.n_kv_heads >> 3;
        const int hkv_ = xcd + 8 * (r % per_xcd);
        r /= per_xcd;
        hq = hkv_ * qper + r % qper;
        r /= qper;
        split = r % a.n_split;
        n = r / a.n_split;
    } else {
        int idx = bid;
        hq = idx % a.n_q_heads;
        idx /= a.n_q_heads;
        split = idx % a.n_split;
        n = idx / a.n_split;
    }
    const int hkv = hq / qper;

    int t_n = a.t;
    if (a.seq_lens) t_n = min(max(a.seq_lens[n] - seq_len_shift, seq_len_floor), a.t);
    const int n_tiles = (t_n + kTileTokens - 1) / kTileTokens;
    const int tile0 = split * a.tiles_per_split;
    const int tile1 = min(tile0 + a.tiles_per_split, n_tiles);

    float* part = partials + ((size_t)(n * a.n_q_heads + hq) * a.n_split + split) * (D + kPartialHeader);
    if (tile0 >= tile1) {               // this split lies beyond the sequence: neutral partial
        if (tid == 0) { part[0] = -INFINITY; part[1] = 0.f; }
        for (int i = tid; i < D; i += NT) part[kPartialHeader + i] = 0.f;
        return;
    }

    // fused step: position of the new token, and whether this workgroup's split holds it
    const int pos_new = t_n - 1;
    const int tile_new = pos_new / kTileTokens, u_new = pos_new % kTileTokens;
    const bool has_new = STEP && tile_new >= tile0 && tile_new < tile1;
    if (has_new) {
        if (tid < 2 * GH) keys[tid] = ~0ull;
        lds_barrier();
    }

    Columns<GH, B, LONG> col;
    col.init(lane);

    const int my_tiles = (tile1 - tile0 - wave + NW - 1) / NW;   // tiles tile0 + wave + k NW
    // the two code streams of this (sequence, KV head); a paged cache first reads the pages of
    // this wavefront's tiles (lane j: its j-th tile; a split has at most 64 tiles per wavefront)
    TileWalk<GH, B> kwalk, vwalk;
    kwalk.first = tile0 + wave;
    kwalk.stride = NW;
    kwalk.pages = 0;
    if (a.map.block_table) {
        if (lane < my_tiles) kwalk.pages = a.map.page(n, tile0 + wave + lane * NW);
        kwalk.page_bytes = (size_t)a.f.n_kv_heads * F::TILE_BYTES;
        kwalk.base = k_codes + (size_t)hkv * F::TILE_BYTES;
        vwalk = kwalk;
        vwalk.base = v_codes + (size_t)hkv * F::TILE_BYTES;
    } else {
        const size_t stream_idx = a.map.tile_index(n, hkv, 0) * F::TILE_BYTES;
        kwalk.page_bytes = 0;
        kwalk.base = k_codes + stream_idx;
        vwalk = kwalk;
        vwalk.base = v_codes + stream_idx;
    }

    Streamer<GH, B, PF> st;

    // ---- 1. score table ------------------------------------------------------------------
    // unit u = tid + k NT of a 16-group chunk: group gl = u % 16 (fixed per thread), centroids
    // j0 .. j0 + JPL - 1 with j0 = (u / 16) * JPL.  A wavefront's loads are 16 segments of 64 B.
    const int gl = tid & 15;
    unsigned xvw[STEP ? NCH : 1][C / 2];            // fused step: this thread's slices of the new value row
    {
        const uint16_t* qh = q_ptr + (size_t)n * q_batch_stride + (size_t)hq * D;
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
            const int g = ch * 16 + gl;
            const uint16_t* ck = k_centroids + (size_t)(hkv * GH + g) * K * C;
            unsigned qw[C / 2];
#pragma unroll
            for (int i = 0; i < C / 2; ++i) qw[i] = *reinterpret_cast<const unsigned*>(qh + g * C + 2 * i);
            // fused step: the new key row against this group's codebook, same walk (the row's
            // words are only requested here; they are converted after the loads below went out)
            unsigned xkw[C / 2];
            float xk[C];
            Nearest knear;
            if (has_new) {
                const size_t xoff = (size_t)n * a.x_new_stride + (size_t)(hkv * GH + g) * C;
#pragma unroll
                for (int i = 0; i < C / 2; ++i) {
                    xkw[i] = *reinterpret_cast<const unsigned*>(xk_new + xoff + 2 * i);
                    xvw[ch][i] = *reinterpret_cast<const unsigned*>(xv_new + xoff + 2 * i);
                }
            }
#pragma unroll
            for (int k0 = 0; k0 < IPT; k0 += KB) {
                Cent16 raw[KB];
#pragma unroll
                for (int k = 0; k < KB; ++k) raw[k] = load_cent16(ck + (size_t)((tid + (k0 + k) * NT) >> 4) * 8);
                // the first key tiles are requested behind the first centroids: tile requests must
                // go out as early as possible (the kernel is bound by HBM from its first
                // microsecond), but not in front of the loads the table build waits for
                if (ch == 0 && k0 == 0) st.begin(kwalk, my_tiles, lane);
                if constexpr (STEP) __builtin_amdgcn_sched_barrier(0);
                if (has_new && k0 == 0) {
#pragma unroll
                    for (int i = 0; i < C / 2; ++i) {
                        const half2_t h = __builtin_bit_cast(half2_t, xkw[i]);
                        xk[2 * i] = (float)h.x;
                        xk[2 * i + 1] = (float)h.y;
                    }
                }
#pragma unroll
                for (int k = 0; k < KB; ++k) {
                    const int j0 = ((tid + (k0 + k) * NT) >> 4) * JPL;
#pragma unroll
                    for (int jj = 0; jj < JPL; ++jj) {
                        float dot = 0.f;
#pragma unroll
                        for (int i = 0; i < C / 2; ++i)
                            dot = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, raw[k].w[jj * (C / 2) + i]),
                                                         __builtin_bit_cast(half2_t, qw[i]), dot, false);
                        const float v = dot * a.scale_log2e;
                        float* dst = tab + (j0 + jj) * RW + g * R;
                        if constexpr (R == 2) *reinterpret_cast<float2*>(dst) = make_float2(v, v);
                        else *dst = v;
                        if (has_new) knear.offer(centroid_distance<C>(xk, &raw[k].w[jj * (C / 2)]), j0 + jj);
                    }
                }
            }
            if (has_new) {
                const unsigned long long kkey = group_lanes_min(knear.key());
                if (lane < 16) lds_min_u64(&keys[g], kkey);
            }
        }
    }
    lds_barrier();

    // fused step: the key codes of the new token are known; the first query head of the KV head
    // stores them (each token owns its 16-byte records, so no other token's bytes are touched)
    const bool writer = has_new && hq % (a.n_q_heads / a.f.n_kv_heads) == 0;
    if (writer)
        store_new_codes<GH, B>(const_cast<uint8_t*>(k_codes) + a.map.tile_index(n, hkv, tile_new) * F::TILE_BYTES, keys, u_new, tid);

    // ---- 2. phase K: scores --------------------------------------------------------------
    // Every lane also keeps the maximum m of its scores and l = sum 2^(s - m) over them (the
    // usual running pair), so that the split's maximum and the estimate of its l that places the
    // fixed point of phase V are known as soon as the wavefronts have exchanged one pair each.
    float lane_m = -1e30f, lane_l = 0.f;        // (finite start: a lane without valid tokens stays at l = 0)
    // fused step: the wavefront whose walk meets the new token's tile patches that tile in registers
    // as if the codes just found were already in the cache
    const bool meets_new = has_new && (tile_new - tile0) % NW == wave;
    NewTokenCodes<GH, B> new_codes;
    if (meets_new) new_codes.build(keys, u_new, lane);
    st.run(kwalk, my_tiles, lane, [&](const Tile<GH, B>& w_in, int k) {
        const int lt = wave + k * NW;                       // tile within the split
        Tile<GH, B> w = w_in;
        if (meets_new && tile0 + lt == tile_new) new_codes.patch(w, u_new, lane);
        float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
        for (int s = 0; s < GH; s += 2) {
            acc0 += lds_load(slot_addr<GH, B, LONG>(w, col, s));
            acc1 += lds_load(slot_addr<GH, B, LONG>(w, col, s + 1));
        }
        const int tok = (tile0 + lt) * kTileTokens + lane;
        const float sv = tok < t_n ? acc0 + acc1 : -INFINITY;
        sc[sidx(lt * kTileTokens + lane)] = sv;
        const float m_new = fmaxf(lane_m, sv);
        lane_l = __builtin_fmaf(lane_l, __builtin_amdgcn_exp2f(lane_m - m_new), __builtin_amdgcn_exp2f(sv - m_new));
        lane_m = m_new;
    }, [] {});
    st.begin(vwalk, my_tiles, lane);         // value codes are on their way

    {
        const float wave_m = wave_max(lane_m);
        const float wave_l = wave_sum(lane_l * __builtin_amdgcn_exp2f(lane_m - wave_m));
        // Where the wavefronts' pairs go.  Formats with spare LDS behind the table exchange them
        // there, across the barrier that ends the table reads; the others have to wait for that
        // barrier and use the first row of the (then dead) table.
        float* slots = SLOTS_BEHIND ? slot_area : tab;
        if constexpr (!SLOTS_BEHIND) lds_barrier();
        if (lane == 0) {
            slots[wave] = wave_m;
            slots[NW + wave] = wave_l;
        }
    }
    lds_barrier();                                // all table reads done, all scores written, all pairs visible
    float m, l_est = 0.f;
    {
        const float* slots = SLOTS_BEHIND ? slot_area : tab;
        m = slots[0];
#pragma unroll
        for (int w = 1; w < NW; ++w) m = fmaxf(m, slots[w]);
        // (every split that reaches this point holds at least one valid token, so m is a score)
#pragma unroll
        for (int w = 0; w < NW; ++w) l_est = __builtin_fmaf(slots[NW + w], __builtin_amdgcn_exp2f(slots[w] - m), l_est);
    }
    const int fx = fixed_point_exponent(l_est);
    const float fx_scale = ldexpf(1.f, fx), fx_inv = ldexpf(1.f, -fx);
    if constexpr (!SLOTS_BEHIND) lds_barrier();   // everyone holds m and fx before the table is cleared
    {
        float4* t4 = reinterpret_cast<float4*>(tab);
        if constexpr (F::SCORES_IN_TABLE) {         // clear the table columns of every row, keep the scores
            constexpr int Q = F::LUT_WORDS / 4;     // float4 per row
#pragma unroll 4
            for (int i = tid; i < K * Q; i += NT) t4[(i / Q) * 16 + (i % Q)] = make_float4(0.f, 0.f, 0.f, 0.f);
        } else {
#pragma unroll 4
            for (int i = tid; i < F::TAB_FLOATS / 4; i += NT) t4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    lds_barrier();

    // ---- 3. phase V: probability bins ----------------------------------------------------
    unsigned* pf_new = reinterpret_cast<unsigned*>(keys + 2 * GH);
    constexpr bool EARLY = IPT * NCH <= 8 && KB == IPT;
    Cent16 rawv[EARLY ? NCH : 1][KB];
    unsigned lane_sum = 0;
    st.run(vwalk, my_tiles, lane, [&](const Tile<GH, B>& w_in, int k) {
        const int lt = wave + k * NW;
        const Tile<GH, B>& w = w_in;
        const float p = __builtin_amdgcn_exp2f(sc[sidx(lt * kTileTokens + lane)] - m);
        unsigned pf = (unsigned)__builtin_fmaf(p, fx_scale, 0.5f);           // round to nearest
        lane_sum += pf;
        // fused step: the new token's value codes are found in the epilogue (the value codebook is
        // loaded there anyway); its weight waits in LDS and joins the bins then
        if (has_new && tile0 + lt == tile_new && lane == u_new) {
            *pf_new = pf;
            pf = 0;
        }
#pragma unroll
        for (int s = 0; s < GH; ++s) lds_add(slot_addr<GH, B, LONG>(w, col, s), pf);
    }, [&] {
        // the value centroids of the epilogue are requested behind the last value tiles, so their
        // latency overlaps the last tiles and the wait for the slowest wavefront (where registers
        // allow: not with 1024 rows)
        if constexpr (EARLY) {
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
                const uint16_t* cv = v_centroids + (size_t)(hkv * GH + ch * 16 + gl) * K * C;
#pragma unroll
                for (int k = 0; k < IPT; ++k) rawv[ch][k] = load_cent16(cv + (size_t)((tid + k * NT) >> 4) * 8);
            }
        }
    });

    // ---- 4. epilogue: o = bins . C_V -----------------------------------------------------
    // same walk as the table build; thread-private sums over its centroids of group gl in every
    // chunk, then lanes l, l+16, l+32, l+48 and the wavefronts are added up.
    lane_sum = wave_sum_u32(lane_sum);

    // fused step: encode the new value row against the value codebook (same walk, same registers
    // as the sums below).  A wavefront does this as soon as its own tiles are done, i.e. while it
    // would otherwise wait at the barrier for the slowest one (the minima go to LDS words of
    // their own).
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
            const uint16_t* cv = v_centroids + (size_t)(hkv * GH + ch * 16 + gl) * K * C;
            Nearest vnear;
#pragma unroll
            for (int k0 = 0; k0 < IPT; k0 += KB) {
                Cent16 rawb[EARLY ? 1 : KB];
                if constexpr (!EARLY) {
#pragma unroll
                    for (int k = 0; k < KB; ++k) rawb[k] = load_cent16(cv + (size_t)((tid + (k0 + k) * NT) >> 4) * 8);
                }
#pragma unroll
                for (int k = 0; k < KB; ++k) {
                    const int j0 = ((tid + (k0 + k) * NT) >> 4) * JPL;
                    const Cent16& r = EARLY ? rawv[EARLY ? ch : 0][k] : rawb[EARLY ? 0 : k];
#pragma unroll
                    for (int jj = 0; jj < JPL; ++jj) vnear.offer(centroid_distance<C>(xv, &r.w[jj * (C / 2)]), j0 + jj);
                }
            }
            const unsigned long long vkey = group_lanes_min(vnear.key());
            if (lane < 16) lds_min_u64(&keys[GH + ch * 16 + gl], vkey);
        }
    }
    lds_barrier();                                // all bin updates done; the scores are dead
    if (lane == 0) scr[wave] = __uint_as_float(lane_sum);
    // fused step: the new token's weight joins the bins of the codes just found; store the codes
    if (has_new) {
        if (tid < GH) {
            const unsigned code = (unsigned)(keys[GH + tid] & 0xffffffffu);
            lds_add((code * RW + tid * R) * 4u, *pf_new);
        }
        if (writer)
            store_new_codes<GH, B>(const_cast<uint8_t*>(v_codes) + a.map.tile_index(n, hkv, tile_new) * F::TILE_BYTES, keys + GH, u_new, tid);
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
                const uint16_t* cv = v_centroids + (size_t)(hkv * GH + ch * 16 + gl) * K * C;
#pragma unroll
                for (int k = 0; k < KB; ++k) rawv[0][k] = load_cent16(cv + (size_t)((tid + (k0 + k) * NT) >> 4) * 8);
            }
            const Cent16 (&raw)[KB] = rawv[EARLY ? ch : 0];
#pragma unroll
            for (int k = 0; k < KB; ++k) {
                const int j0 = ((tid + (k0 + k) * NT) >> 4) * JPL;
#pragma unroll
                for (int jj = 0; jj < JPL; ++jj) {
                    const float* src = tab + (j0 + jj) * RW + (ch * 16 + gl) * R;
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
            acc[ch][i] += __shfl_xor(acc[ch][i], 16);
            acc[ch][i] += __shfl_xor(acc[ch][i], 32);
        }
    }
    // per-wave results: scr[64 + wave * D + channel]
    if (lane < 16) {
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch)
#pragma unroll
            for (int i = 0; i < C; ++i) scr[64 + wave * D + (ch * 16 + gl) * C + i] = acc[ch][i];
    }
    lds_barrier();
    unsigned l_fix = 0;                             // exact: integer adds
#pragma unroll
    for (int w = 0; w < NW; ++w) l_fix += __float_as_uint(scr[w]);
    const float l = (float)l_fix * fx_inv;
    const bool direct = a.n_split == 1;             // a single split needs no merge kernel
    if (tid == 0 && !direct) {
        part[0] = m;
        part[1] = l;
    }
    for (int chn = tid; chn < D; chn += NT) {
        float o = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) o += scr[64 + w * D + chn];
        if (direct) out_ptr[(size_t)n * out_batch_stride + (size_t)hq * D + chn] = __builtin_bit_cast(uint16_t, (_Float16)(o / l));
        else part[kPartialHeader + chn] = o;
    }
}

// Merge the partials of all splits of one (sequence, query head): rescaling to the running
// maximum split by split, then one rounding to fp16.
__global__ void decode_merge_kernel(const float* partials, uint16_t* out, int n_split, int head_dim,
                                    const LayerPtrs* layers, int rows_per_layer, int n_q_heads, int64_t out_batch_stride)
{
    int bh = blockIdx.x;
    const int stride = head_dim + kPartialHeader;
    const float* p = partials + (size_t)bh * n_split * stride;
    if (layers) {                       // layer-batched: row bh of layer blockIdx / rows_per_layer
        const int layer = bh / rows_per_layer;
        bh -= layer * rows_per_layer;
        out = layers[layer].out;
    }
    out += (size_t)(bh / n_q_heads) * out_batch_stride + (size_t)(bh % n_q_heads) * head_dim;
    // One pass with a running maximum (the usual rescaling), so that no load waits for a value
    // computed from another: the loads of all splits go out together.  A split beyond its
    // sequence left m = -inf, l = 0, o = 0 and gets weight 0.
    for (int i = threadIdx.x; i < head_dim; i += blockDim.x) {
        float m = -INFINITY, l = 0.f, o = 0.f;
#pragma unroll 4
        for (int s = 0; s < n_split; ++s) {
            const float ms = p[s * stride], ls = p[s * stride + 1], os = p[s * stride + kPartialHeader + i];
            const float m_new = fmaxf(m, ms);
            const float m_safe = m_new == -INFINITY ? 0.f : m_new;
            const float keep = __builtin_amdgcn_exp2f(m - m_safe), w = __builtin_amdgcn_exp2f(ms - m_safe);
            l = __builtin_fmaf(l, keep, ls * w);
            o = __builtin_fmaf(o, keep, os * w);
            m = m_new;
        }
        const _Float16 h = (_Float16)(o / l);
        out[i] = __builtin_bit_cast(uint16_t, h);
    }
}

template <int GH, int B, int NT, bool LONG>
size_t smem_bytes(int tiles_per_split, int head_dim, bool step)
{
    using F = Fmt<GH, B, LONG>;
    const int key_floats = step ? kKeyFloats(GH) : 0;
    if (F::SCORES_IN_TABLE) return sizeof(float) * (size_t)(F::TAB_FLOATS + kScratchFloats(NT, head_dim) + key_floats);
    // behind the table: the score buffer (reused as scratch once the scores are dead), then the
    // keys, then (b = 10) the wavefronts' reduction slots
    const int sc_floats = std::max(kMinScoreFloats, tiles_per_split * kTileTokens);
    return sizeof(float) * (size_t)(F::TAB_FLOATS + sc_floats + key_floats + (B == 10 ? kSlotFloats : 0));
}

template <int GH, int C, int B, int NT, bool STEP, bool LAYERS, bool LONG = false>
cq_status launch_variant(const DecodeArgs& a, hipStream_t stream)
{
    auto kernel = decode_split_kernel<GH, C, B, NT, STEP, LAYERS, LONG>;
    static LdsKernelSetup setup;
    if (setup.ensure(reinterpret_cast<const void*>(kernel)) != hipSuccess) return CQ_ERR_HIP;
    const size_t smem = smem_bytes<GH, B, NT, LONG>(a.tiles_per_split, a.f.head_dim, STEP);
    if (smem > 160 * 1024) return CQ_ERR_INVALID_ARG;
    const unsigned grid = (unsigned)(a.batch * a.n_q_heads * a.n_split) * (unsigned)(a.layers ? a.n_layers : 1);
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(NT), smem, stream, a);
    if (hipGetLastError() != hipSuccess) return CQ_ERR_HIP;
    return CQ_OK;
}

template <int GH, int C, bool STEP, bool LAYERS>
cq_status launch_by_split(const DecodeArgs& a, hipStream_t stream)
{
    // 16 / 32 groups per head: scores live inside the table, 68 KB of LDS, two 512-thread
    // workgroups per CU.  64 groups per head: 64 KB table + 4 B per token of the split; up to 64
    // tiles two 512-thread workgroups fit a CU, longer splits run as one 1024-thread workgroup.
    // 16 groups per head, more than 8192 tokens per split: the table without replicas (12288 tokens)
    if constexpr (GH == 16) {
        if (a.tiles_per_split > 256 * Fmt<16, 8>::SCORE_WORDS / kTileTokens)
            return launch_variant<GH, C, 8, 512, STEP, LAYERS, true>(a, stream);
    }
    if (Fmt<GH, 8>::SCORES_IN_TABLE || a.tiles_per_split <= 64) return launch_variant<GH, C, 8, 512, STEP, LAYERS>(a, stream);
    return launch_variant<GH, C, 8, 1024, STEP, LAYERS>(a, stream);
}

template <bool STEP, bool LAYERS>
cq_status launch_format(const DecodeArgs& a, hipStream_t stream)
{
    if (a.f.b == 8) {
        if (a.f.gh == 16 && a.f.c == 8) return launch_by_split<16, 8, STEP, LAYERS>(a, stream);
        if (a.f.gh == 32 && a.f.c == 4) return launch_by_split<32, 4, STEP, LAYERS>(a, stream);
        if (a.f.gh == 64 && a.f.c == 2) return launch_by_split<64, 2, STEP, LAYERS>(a, stream);
    } else if (a.f.b == 10 && a.f.gh == 16 && a.f.c == 8) {
        return launch_variant<16, 8, 10, 1024, STEP, LAYERS>(a, stream);
    }
    return CQ_ERR_UNSUPPORTED;
}

}  // namespace

cq_status launch_layer_table_write(const LayerChunk& chunk, int count, LayerPtrs* dst, hipStream_t stream)
{
    hipLaunchKernelGGL(layer_table_write_kernel, dim3(1), dim3(64), 0, stream, chunk, count, dst);
    return hipGetLastError() == hipSuccess ? CQ_OK : CQ_ERR_HIP;
}

cq_status launch_decode_merge(const float* partials, uint16_t* out, int rows, int n_q_heads, int64_t out_batch_stride,
                              int n_split, int head_dim, hipStream_t stream)
{
    hipLaunchKernelGGL(decode_merge_kernel, dim3((unsigned)rows), dim3(128), 0, stream, partials, out, n_split, head_dim,
                       static_cast<const LayerPtrs*>(nullptr), 0, n_q_heads, out_batch_stride);
    return hipGetLastError() == hipSuccess ? CQ_OK : CQ_ERR_HIP;
}

int decode_max_tiles_per_split(const Derived& f)
{
    if (f.b == 10) return (160 * 1024 / 4 - Fmt<16, 10>::TAB_FLOATS - kKeyFloats(16) - kSlotFloats) / kTileTokens;   // 382: 160 KB of LDS
    if (f.gh == 16) return 256 * Fmt<16, 8, true>::SCORE_WORDS / kTileTokens;         // 192: scores inside the table, no replicas
    if (f.gh == 32) return 256 * Fmt<32, 8>::SCORE_WORDS / kTileTokens;               // 128
    return 256;
}

cq_status launch_decode(const DecodeArgs& a, hipStream_t stream)
{
    // (a layer-batched launch is always a fused step: its table holds the new rows)
    const cq_status st = a.layers ? launch_format<true, true>(a, stream)
                         : a.xk_new ? launch_format<true, false>(a, stream) : launch_format<false, false>(a, stream);
    if (st != CQ_OK || a.n_split == 1) return st;
    const int threads = a.f.head_dim <= 64 ? 64 : (a.f.head_dim <= 128 ? 128 : 256);
    const int rows = a.batch * a.n_q_heads;
    hipLaunchKernelGGL(decode_merge_kernel, dim3((unsigned)(rows * (a.layers ? a.n_layers : 1))), dim3(threads), 0, stream,
                       a.partials, a.out, a.n_split, a.f.head_dim, a.layers, rows, a.n_q_heads, a.out_batch_stride);
    if (hipGetLastError() != hipSuccess) return CQ_ERR_HIP;
    return CQ_OK;
}

}  // namespace cq

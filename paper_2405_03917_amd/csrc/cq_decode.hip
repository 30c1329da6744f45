// Decode attention straight from packed CQ codes (Eq. 1 of the paper over the centroids the
// cached codes select), for gfx950.
//
// One workgroup handles one (sequence, query head, context split).  Per workgroup:
//   1. build the score table  LUT[g][j] = scale * log2(e) * (q_g . C_K[g][j])  in LDS;
//   2. walk the split chunk by chunk (a chunk is 16 tiles of 64 tokens per wavefront):
//      K: stream the chunk's key codes (one tile per wavefront per step, lane = token),
//         score = sum over groups of LUT[g][code]; the scores stay in registers;
//      V: stream the chunk's value codes; p = 2^(score - reference) in fixed point; add p into
//         bin[g][code] in LDS with integer atomics (exact, order independent);
//   3. epilogue: o[g c + i] = sum_j bin[g][j] * C_V[g][j][i]; with a single split the normalised
//      result is rounded to fp16 and stored, otherwise (max, sum p, o) goes out as a partial and
//      a second kernel merges the partials of all splits.
//
// LDS table layout: 256 rows of 64 four-byte words (64 KB); b = 8: one row per code value;
// b = 10: one row per value of a code's low byte, whose four 16-word quarters belong to the
// four values of its two high bits.  Lane l of a wavefront owns ONE word
// column at every step s of the walk over a token's Gh slots: column(l, g) with g = (l + s) mod
// Gh, the group that the cache layout put in slot s of token l.  With 32 or 64 groups per head
// the 32 columns of a half-wavefront are different modulo 32 (lanes l and l + 32 may share one:
// the LDS serves a wavefront in two halves), so neither the table gather nor the bin update ever
// has a bank conflict.  With 16 groups per head and b = 8 each group is replicated twice to give
// 32 lanes their own column (the epilogue adds the replicas); b = 10 keeps one column per
// group.  For b = 8 the byte address of a lookup is (code << 8) | (4 * column): one v_perm_b32
// from the code word and a per-lane constant; b = 10 ors the two high bits in behind it.  With 16 or 32 groups per head words 0..31 of a
// 256-byte row are the table's columns and words 32..63 the bins', so both exist at once and a
// workgroup can walk any number of chunks with one table; 64 groups per head and b = 10 turn the
// table into the bins once their single chunk is scored.  Every format needs 70 KB of LDS, so
// two workgroups share a CU.
//
// Measured on MI355X (microbenchmark, per CU): ds_read_b32 gathers and ds_add_u32 run at the
// same rate with this layout as with linear addresses; ds_add_f32 is about 45 times slower than
// ds_add_u32, which is why the bins are integers.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "cq_decode_common.hpp"

// arrival counters of the in-kernel merge (see MergeCounters); 512 KB per GPU
static __device__ __align__(256) unsigned merge_counters[16 * 8192];

namespace cq {
namespace {

constexpr int kDecodeThreads = 512;
constexpr int kDecodeWaves = kDecodeThreads / 64;
// tiles per wavefront and chunk (= score registers per lane): b = 8: 16, and 8 for splits that fit;
// b = 10: 32 (one chunk must hold the longest split, 16384 tokens), and 16 for splits that fit
constexpr int kChunkTiles8 = 16;
constexpr int kChunkTiles10 = 32;
constexpr int kMergeRows = 8192;        // arrival counters per set (rows of one launch)
constexpr int kMergeSets = 16;          // sets (streams served) per device
static_assert(sizeof(merge_counters) == sizeof(unsigned) * kMergeRows * kMergeSets, "size of the counter array");

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

// Merge the partials of all splits of one (sequence, query head): one pass with a running
// maximum (the usual rescaling), so that no load waits for a value computed from another and
// the loads of all splits go out together; then one rounding to fp16.  A split beyond its
// sequence left m = -inf, l = 0, o = 0 and gets weight 0.  DEVICE_LOADS: the partials were
// written by other workgroups of the running kernel: read them with device-scope loads.
template <bool DEVICE_LOADS>
__device__ __forceinline__ float partial_load(const float* p)
{
    if constexpr (DEVICE_LOADS) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else return *p;
}
template <bool DEVICE_LOADS>
__device__ __forceinline__ void merge_splits(const float* p, int n_split, int head_dim, uint16_t* out, int tid, int nt)
{
    const int stride = head_dim + kPartialHeader;
    for (int i = tid; i < head_dim; i += nt) {
        float m = -INFINITY, l = 0.f, o = 0.f;
#pragma unroll 4
        for (int s = 0; s < n_split; ++s) {
            const float ms = partial_load<DEVICE_LOADS>(p + s * stride), ls = partial_load<DEVICE_LOADS>(p + s * stride + 1),
                        os = partial_load<DEVICE_LOADS>(p + s * stride + kPartialHeader + i);
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
// (device-scope store: written through to where every workgroup's device-scope loads find it)
__device__ __forceinline__ void partial_store(float* p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---- layout of the workgroup's LDS ---------------------------------------------------------
// b = 8, 16 or 32 groups per head (SEPARATE): every 256-byte row holds the score table in words
// 0..31 and the probability bins in words 32..63 (16 groups per head: two replicas of each, so
// that the 32 lanes of a half-wavefront own 32 different banks), 64 KB in all.  Table and bins
// live side by side, so a workgroup can walk a context of any length chunk by chunk with the
// table it built once.
// b = 8 with 64 groups per head, b = 10 (SHARED): the table fills the 64 KB; it is cleared after
// the scores of the (single) chunk are known and becomes the bins.
// Behind the table: the wavefronts' (maximum, sum) pairs of a chunk (two sets, used alternately),
// their integer sums at a rescale, the reduction scratch of the epilogue, the fused step's keys.
template <int GH, int B>
struct Lay {
    static constexpr int K = 1 << B;
    static constexpr int RW = 64;                                   // words per row
    static constexpr bool SEPARATE = B == 8 && GH <= 32;
    static constexpr int R = (GH == 16 && B == 8) ? 2 : 1;          // replicas per group
    static constexpr int BIN0 = SEPARATE ? 32 : 0;                  // first bin word of a row
    static constexpr int TAB_FLOATS = 256 * RW;
    static constexpr int TILE_BYTES = kTileTokens * GH * B / 8;
    static constexpr int SLOTS = TAB_FLOATS;                        // [2][2][NW] floats
    static constexpr int SUMS = SLOTS + 4 * kDecodeWaves;           // [NW] unsigned
    static constexpr int SCR = SUMS + kDecodeWaves;                 // 64 + NW * head_dim floats
    static constexpr int KEYS(int head_dim) { return SCR + 64 + kDecodeWaves * head_dim; }   // fused step only
    // fused step: the keys, the new token's fixed-point weight, its record of key codes in cache order
    static constexpr int FLOATS(int head_dim, bool step) { return KEYS(head_dim) + (step ? kKeyFloats(GH) + GH / 4 + 2 : 0); }
    // Word of code value j in word column `col`.  b = 8: row j.  b = 10: row = the low 8 bits,
    // and the two high bits pick one of four 16-word quarters of the row, which makes the byte
    // address (low << 8) | (high << 6) | (4 * column): the b = 8 address plus one shift-or.
    __device__ __forceinline__ static constexpr int word(int j, int col)
    {
        return B == 8 ? j * 64 + col : (j & 255) * 64 + (j >> 8) * 16 + col;
    }
};

// Per-lane column constants for the Gh slots of a token, four byte offsets per register (the
// table's columns; the bins' are Lay::BIN0 words further, which rides in the offset field of
// the LDS instruction).
template <int GH, int B>
struct Cols {
    unsigned v[GH / 4];
    __device__ __forceinline__ void init(int lane)
    {
#pragma unroll
        for (int i = 0; i < GH / 4; ++i) {
            unsigned x = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int g = (lane + 4 * i + k) & (GH - 1);
                const int column = Lay<GH, B>::R == 2 ? 2 * g + ((lane >> 4) & 1) : g;   // lanes l and l + 16 differ, l and l + 32 share
                x |= (unsigned)(4 * column) << (8 * k);
            }
            v[i] = x;
        }
    }
};

// Byte address of the word for slot s of this lane's token.
template <int GH, int B>
__device__ __forceinline__ unsigned code_addr(const Tile<GH, B>& w, const Cols<GH, B>& col, int s)
{
    const u32x4 q = w.lo[s >> 4];
    const int dw = (s >> 2) & 3;
    const unsigned code_word = dw == 0 ? q.x : dw == 1 ? q.y : dw == 2 ? q.z : q.w;
    const unsigned k = s & 3;
    const unsigned sel = 0x0c0c0000u | ((4u + k) << 8) | k;   // {0, 0, code byte k, column byte k}
    const unsigned lo = __builtin_amdgcn_perm(code_word, col.v[s >> 2], sel);
    if constexpr (B == 8) return lo;
    else return (((w.hi >> (2 * s)) & 3u) << 6) | lo;
}

// Fused step: the key codes of the new token as the cache layout would hold them (slot s of token
// u carries group (s + u) mod Gh), from keys[g] = group g's (distance, index) minimum.  Built in LDS
// by the one wavefront whose walk meets the token's tile, before its walk starts (lane i builds word
// i); when the walk reaches the tile, lane u's codes are replaced by the record.
template <int GH, int B>
struct NewTokenRecord {
    unsigned* rec;                      // [GH / 4] words of low bytes, then (b = 10) the word of high bits
    __device__ __forceinline__ void build(const unsigned long long* keys, int u_new, int lane) const
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
            rec[lane] = x;
        }
        if constexpr (B == 10) {
            static_assert(B != 10 || GH == 16, "four lanes hold the high bits");
            h |= __shfl_xor(h, 1);
            h |= __shfl_xor(h, 2);
            if (lane == 0) rec[GH / 4] = h;
        }
    }
    __device__ __forceinline__ void patch(Tile<GH, B>& w, int u_new, int lane) const
    {
        const bool mine = lane == u_new;
#pragma unroll
        for (int pl = 0; pl < GH / 16; ++pl) {
            const uint4 r = *reinterpret_cast<const uint4*>(rec + 4 * pl);
            u32x4 q = w.lo[pl];
            q.x = mine ? r.x : q.x;
            q.y = mine ? r.y : q.y;
            q.z = mine ? r.z : q.z;
            q.w = mine ? r.w : q.w;
            w.lo[pl] = q;
        }
        if constexpr (B == 10) w.hi = mine ? rec[GH / 4] : w.hi;
    }
};

// One 64-token tile through a buffer descriptor of its own: `tile` is wave-uniform; a tile that
// does not exist gets a descriptor of size zero, for which the hardware returns zeros without
// touching memory.  Every request of the walk is therefore issued unconditionally, and the
// number of loads in flight at any point of the (unrolled) walk is a compile-time constant.
template <int GH, int B>
__device__ __forceinline__ Tile<GH, B> load_tile_desc(const uint8_t* tile, bool exists, int lane)
{
    constexpr int TB = Lay<GH, B>::TILE_BYTES;
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(tile), 0, exists ? TB : 0, 0x00020000);
    Tile<GH, B> w;
    const unsigned off = 16u * (unsigned)lane;
#pragma unroll
    for (int pl = 0; pl < GH / 16; ++pl)
        w.lo[pl] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, off + 1024u * pl, 0, 2));
    if constexpr (B == 10)
        w.hi = __builtin_amdgcn_raw_buffer_load_b32(rsrc, 4u * (unsigned)lane + (unsigned)(kTileTokens * GH), 0, 2);
    else
        w.hi = 0;
    return w;
}

// STEP = true is the fused decode step: the workgroup whose split holds the newest position
// (t_n - 1) also encodes that token's key and value rows for its KV head.  Keys: while it builds
// the score table (the key codebook is in registers anyway); the tile that holds the position is
// then patched in registers as if the codes were already in the cache.  Values: in the epilogue
// (the value codebook is in registers there); phase V leaves the position out of the bins and
// its weight is added to the bins of the codes just found.  The first query head of each KV head
// stores the codes.  Results equal cq_encode_kv followed by cq_decode_attention bit for bit
// (the bins are integers: the order of the additions does not matter).
//
// The walk.  Wavefront w owns tiles w, w + 8, ... of the split; a CHUNK is NS of its tiles (8 NS
// tiles of the workgroup).  Per chunk: the key tiles give one score per lane and tile, kept in
// NS registers (lane = token in both streams, so the lane that scored a token also bins it);
// the wavefronts exchange the chunk's (maximum, sum of 2^(score - maximum)) across one barrier;
// then the value tiles are binned.  Requests run PF tiles ahead through both streams and across
// chunk boundaries.
template <int GH, int C, int B, int NS, bool STEP, bool LAYERS>
__global__ __launch_bounds__(kDecodeThreads, 4) void decode_split_kernel(DecodeArgs a_in)
{
    const DecodeArgs a = early_args<STEP, LAYERS>(a_in);
    using F = Lay<GH, B>;
    constexpr int NT = kDecodeThreads;
    constexpr int K = F::K, RW = F::RW, R = F::R;
    constexpr int NW = kDecodeWaves;    // wavefronts
    constexpr int D = GH * C;           // head_dim
    // tiles in flight per wavefront (about 4 KB)
    constexpr int PF = B == 10 ? 2 : (GH == 16 ? 4 : (GH == 32 ? 2 : 1));
    static_assert(NS % PF == 0 && NS >= PF, "the ring of tiles in flight must divide a chunk");
    constexpr int JPL = 8 / C;          // centroids per 16-byte load
    // groups per chunk of the codebook walk; 64 / GPC neighbouring lanes are on a group and read as
    // many neighbouring 16-byte pieces.  (Measured: four lanes, 64 contiguous bytes, is the
    // optimum; eight -- whole cache lines, but eight lanes on one LDS column and twice the chunks
    // -- is 3 to 10 % slower at every format, two -- all 32 LDS columns in one store, but 32-byte
    // runs -- 2 to 12 %.)
    constexpr int GPC = 16;
    constexpr int LPG = 64 / GPC;
    constexpr int NCH = GH / GPC;       // chunks of the codebook walk
    constexpr int UNITS = GPC * K / JPL;    // 16-byte loads per chunk
    constexpr int IPT = UNITS / NT;     // ... per thread
    constexpr int KB = IPT < 8 ? IPT : 8;   // ... requested together
    constexpr int KU = IPT / KB <= 2 ? IPT / KB : 1;    // (1024 rows: the batches stay a loop, for registers)
    static_assert(UNITS % NT == 0 && NT % 64 == 0, "thread count must divide the codebook walk");
    extern __shared__ float smem[];
    float* tab = smem;                              // [K][RW]: score table (and bins)
    float* slots = smem + F::SLOTS;
    unsigned* sums = reinterpret_cast<unsigned*>(smem + F::SUMS);
    float* scr = smem + F::SCR;
    // fused step: 64-bit (distance, index) minima per group, keys[0..GH) for K, [GH..2GH) for V
    unsigned long long* keys = reinterpret_cast<unsigned long long*>(smem + F::KEYS(D));

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
    // The last split of a (sequence, query head) to finish merges them all (when the launch
    // brought counters; else a merge kernel follows).  Partials are written with device-scope
    // stores (write-through) and the merging workgroup reads them with device-scope loads, so
    // no cache has to be written back or invalidated as a whole (a device-scope release fence
    // per workgroup, which writes the whole L2 back, cost 50 us on a 90 us launch).  Order:
    // every thread's stores are complete at the barrier (it waits for them), then one thread
    // counts the workgroup in; the workgroup that counts the last split takes the counter back
    // to zero for the next call and merges.
    auto count_and_merge = [&] {
        if (!a.merge_counters) return;
        __syncthreads();
        unsigned* flag = sums;
        if (tid == 0) {
            const size_t row = (size_t)(part - a.partials) / ((size_t)(D + kPartialHeader) * a.n_split);
            const unsigned arrived = __hip_atomic_fetch_add(a.merge_counters + row, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const bool last = arrived == (unsigned)a.n_split - 1u;
            if (last) __hip_atomic_store(a.merge_counters + row, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *flag = last;
        }
        __syncthreads();
        if (!*flag) return;
        merge_splits<true>(part - (size_t)split * (D + kPartialHeader), a.n_split, D,
                           out_ptr + (size_t)n * out_batch_stride + (size_t)hq * D, tid, NT);
    };
    if (tile0 >= tile1) {               // this split lies beyond the sequence: neutral partial
        if (tid == 0) { partial_store(part, -INFINITY); partial_store(part + 1, 0.f); }
        for (int i = tid; i < D; i += NT) partial_store(part + kPartialHeader + i, 0.f);
        count_and_merge();
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

    // per-lane column constants: the table's, and the same shifted to the bins
    Cols<GH, B> col;
    col.init(lane);

    // this wavefront's tiles: tile0 + wave + k NW, k = 0 .. my_tiles - 1; chunk c holds k = c NS .. c NS + NS - 1
    const int my_tiles = (tile1 - tile0 - wave + NW - 1) / NW;
    const int n_chunks = ((tile1 - tile0 + NW - 1) / NW + NS - 1) / NS;      // of wavefront 0, which has the most tiles
    // The two code streams of this (sequence, KV head).  Contiguous cache: consecutive tiles are
    // TILE_BYTES apart.  Paged cache: lane j holds the page of the j-th tile of the wavefront's
    // current chunk (read one chunk ahead), and a tile sits at base + page * page_bytes.
    const bool paged = a.map.block_table != nullptr;
    const size_t page_bytes = paged ? (size_t)a.f.n_kv_heads * F::TILE_BYTES : 0;
    const size_t stream0 = paged ? (size_t)hkv * F::TILE_BYTES : a.map.tile_index(n, hkv, 0) * F::TILE_BYTES;
    const uint8_t* kbase = k_codes + stream0;
    const uint8_t* vbase = v_codes + stream0;
    auto chunk_pages = [&](int c) {
        int pg = 0;
        const int k = c * NS + lane;
        if (paged && lane < NS && k < my_tiles) pg = a.map.page(n, tile0 + wave + k * NW);
        return pg;
    };
    int pages = chunk_pages(0), pages_next = 0;
    // Request tile i (a compile-time index) of chunk c of a stream.  All of it is scalar
    // arithmetic; the tile's index goes through an opaque copy so that nothing derived from it is
    // kept in registers from one use of the tile to the next (request and use in both streams:
    // that was a pair of scalar registers per tile and condition, and spills).
    const size_t cont_bytes = paged ? 0 : (size_t)F::TILE_BYTES;
    auto request = [&](const uint8_t* base, int c, int i, int pg) {
        int k = c * NS + i;
        asm volatile("" : "+s"(k));
        const bool exists = k < my_tiles;
        const size_t off = (size_t)(unsigned)__builtin_amdgcn_readlane(pg, i) * page_bytes +
                           (size_t)(tile0 + wave + k * NW) * cont_bytes;
        return load_tile_desc<GH, B>(base + (exists ? off : 0), exists, lane);
    };
    // whether tile i of chunk c exists, for the uses (an opaque copy again)
    auto tile_exists = [&](int c, int i) {
        int k = c * NS + i;
        asm volatile("" : "+s"(k));
        return k < my_tiles;
    };
    Tile<GH, B> buf[PF];

    // ---- 1. score table ------------------------------------------------------------------
    // A chunk of the walk is GPC groups; a thread stays on group gl of every chunk.  16-byte piece
    // k of its walk through a group's codebook (centroids j0 .. j0 + JPL - 1, j0 = piece * JPL):
    // the LPG lanes of a group are neighbours and read LPG neighbouring pieces, so the 16 lanes
    // that the memory pipeline takes together read four runs of 64 bytes (with lanes l, l + 16,
    // l + 32, l + 48 on a group, as it first was, they touched 16 lines for 16 bytes each).
    const int gl = (tid / LPG) % GPC;
    auto piece = [&](int k) { return ((tid + k * NT) >> 6) * LPG + (tid % LPG); };
    unsigned xvw[STEP ? NCH : 1][C / 2];            // fused step: this thread's slices of the new value row
    {
        const uint16_t* qh = q_ptr + (size_t)n * q_batch_stride + (size_t)hq * D;
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
            const int g = ch * GPC + gl;
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
#pragma unroll(KU)
            for (int k0 = 0; k0 < IPT; k0 += KB) {
                Cent16 raw[KB];
#pragma unroll
                for (int k = 0; k < KB; ++k) raw[k] = load_cent16(ck + (size_t)piece(k0 + k) * 8);
                // the first key tiles are requested behind the first centroids: tile requests must
                // go out as early as possible (the kernel is bound by HBM from its first
                // microsecond), but not in front of the loads the table build waits for
                if (ch == 0 && k0 == 0) {
#pragma unroll
                    for (int i = 0; i < PF; ++i) {
                        buf[i] = request(kbase, 0, i, pages);
                        __builtin_amdgcn_sched_barrier(0);      // keep request order == consumption order
                    }
                    // the bins start at zero (the barrier behind the table build covers these stores)
                    if constexpr (F::SEPARATE) {
                        float4* t4 = reinterpret_cast<float4*>(tab);
#pragma unroll
                        for (int i = tid; i < K * 8; i += NT) t4[(i >> 3) * 16 + 8 + (i & 7)] = make_float4(0.f, 0.f, 0.f, 0.f);
                    }
                }
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
                    const int j0 = piece(k0 + k) * JPL;
#pragma unroll
                    for (int jj = 0; jj < JPL; ++jj) {
                        float dot = 0.f;
#pragma unroll
                        for (int i = 0; i < C / 2; ++i)
                            dot = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, raw[k].w[jj * (C / 2) + i]),
                                                         __builtin_bit_cast(half2_t, qw[i]), dot, false);
                        const float v = dot * a.scale_log2e;
                        float* dst = tab + F::word(j0 + jj, g * R);
                        if constexpr (R == 2) *reinterpret_cast<float2*>(dst) = make_float2(v, v);
                        else *dst = v;
                        if (has_new) knear.offer(centroid_distance<C>(xk, &raw[k].w[jj * (C / 2)]), j0 + jj);
                    }
                }
            }
            if (has_new) {
                const unsigned long long kkey = group_lanes_min<LPG>(knear.key());
                if (lane % LPG == 0) lds_min_u64(&keys[g], kkey);
            }
        }
    }
    lds_barrier();

    // fused step: the key codes of the new token are known; the first query head of the KV head
    // stores them (each token owns its 16-byte records, so no other token's bytes are touched)
    const bool writer = has_new && hq % (a.n_q_heads / a.f.n_kv_heads) == 0;
    if (writer)
        store_new_codes<GH, B>(const_cast<uint8_t*>(k_codes) + a.map.tile_index(n, hkv, tile_new) * F::TILE_BYTES, keys, u_new, tid);
    // fused step: the wavefront whose walk meets the new token's tile patches that tile in registers
    // as if the codes just found were already in the cache
    const bool meets_new = has_new && (tile_new - tile0) % NW == wave;
    const NewTokenRecord<GH, B> new_codes{reinterpret_cast<unsigned*>(keys + 2 * GH) + 4};
    if (meets_new) new_codes.build(keys, u_new, lane);

    // ---- 2. the walk: per chunk, scores from the key tiles, then bins from the value tiles ----
    // Fixed point.  A probability is binned as pf = round(2^(s - m0 + fx)): m0 is the maximum of
    // the first chunk, fx an integer.  With (m, l) the running pair of all scores seen so far,
    // the bins of a group then sum to about U = l 2^(m - m0 + fx).  fx starts so that the first
    // chunk's U times the number of chunks lies in [2^29, 2^30); before a later chunk is binned,
    // U including that chunk is predicted from the pair, and if it could pass 2^31.5 every bin
    // (and the running integer sum) is shifted right, rounding to nearest, so that U comes to lie
    // in [2^28, 2^29), and fx drops by the shift.  No bin can overflow 32 bits, and each
    // probability is kept to an absolute error of at most 2^-29 of the softmax denominator.
    constexpr bool EARLY = IPT * NCH <= 8 && KB == IPT;
    Cent16 rawv[EARLY ? NCH : 1][KB];
    unsigned* pf_new = reinterpret_cast<unsigned*>(keys + 2 * GH);
    float m0 = 0.f, m_run = 0.f, l_run = 0.f, fxf = 0.f;
    int fx = 0;
    unsigned lane_sum = 0, l_carry = 0;
    float sreg[NS];

    // one key tile: the lane's score, its running pair
    float lane_m, lane_l;
    auto score_tile = [&](const Tile<GH, B>& w_in, int k) {
        const int tile = tile0 + wave + k * NW;
        Tile<GH, B> w = w_in;
        if (meets_new && tile == tile_new) new_codes.patch(w, u_new, lane);
        float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
        for (int s = 0; s < GH; s += 2) {
            acc0 += lds_load(code_addr<GH, B>(w, col, s));
            acc1 += lds_load(code_addr<GH, B>(w, col, s + 1));
        }
        const int tok = tile * kTileTokens + lane;
        float sv = tok < t_n ? acc0 + acc1 : -INFINITY;
        // (the sum is formed here, behind its gathers: left free, the compiler sinks the additions of
        // all tiles of a chunk behind the last tile and runs out of registers for the gathered words)
        asm volatile("" : "+v"(sv));
        const float m_new = fmaxf(lane_m, sv);
        lane_l = __builtin_fmaf(lane_l, __builtin_amdgcn_exp2f(lane_m - m_new), __builtin_amdgcn_exp2f(sv - m_new));
        lane_m = m_new;
        return sv;
    };
    // one value tile: the lane's probability in fixed point into the bins of its token's codes
    auto bin_tile = [&](const Tile<GH, B>& w, int k, float sv) {
        const int tile = tile0 + wave + k * NW;
        const float p = __builtin_amdgcn_exp2f((sv - m0) + fxf);
        unsigned pf = (unsigned)(p + 0.5f);           // round to nearest
        lane_sum += pf;
        // fused step: the new token's value codes are found in the epilogue (the value codebook is
        // loaded there anyway); its weight waits in LDS and joins the bins then
        if (has_new && tile == tile_new && lane == u_new) {
            *pf_new = pf;
            pf = 0;
        }
#pragma unroll
        for (int s = 0; s < GH; ++s) lds_add(code_addr<GH, B>(w, col, s) + 4u * F::BIN0, pf);
    };
    // the value centroids of the epilogue are requested behind the last value tiles, so their
    // latency overlaps the last tiles and the wait for the slowest wavefront (where registers
    // allow: not with 1024 rows)
    auto request_value_centroids = [&] {
        if constexpr (EARLY) {
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
                const uint16_t* cv = v_centroids + (size_t)(hkv * GH + ch * GPC + gl) * K * C;
#pragma unroll
                for (int kk = 0; kk < IPT; ++kk) rawv[ch][kk] = load_cent16(cv + (size_t)piece(kk) * 8);
            }
        }
    };

    // Chunk c.  FULL: all NS tiles of this wavefront exist (always so before the last chunk): the
    // requests run PF tiles ahead through the key tiles, on into the value tiles and on into the
    // next chunk's key tiles, without a condition anywhere.  Otherwise (the wavefront's share of
    // the last chunk is short or empty) the tiles are taken in blocks of PF, blocks without tiles
    // are skipped, and the value tiles are first requested when the key tiles are done.
    auto chunk = [&](int c, auto last_tag, auto full_tag) {
        constexpr bool LAST = decltype(last_tag)::value;
        constexpr bool FULL = decltype(full_tag)::value;
        static_assert(LAST || FULL, "only the last chunk can be short");
        if (paged && !LAST) pages_next = chunk_pages(c + 1);
        const int n_c = my_tiles - c * NS;          // (FULL: >= NS)
        // -- scores.  Every lane also keeps the maximum of its scores and l = sum 2^(s - m) over
        // them (the usual running pair), so that the chunk's pair is known as soon as the
        // wavefronts have exchanged one pair each.
        lane_m = -1e30f;                            // (finite start: a lane without valid tokens stays at l = 0)
        lane_l = 0.f;
        if constexpr (FULL) {
#pragma unroll
            for (int i = 0; i < NS; ++i) {
                // (the tile exists; the test keeps each tile's arithmetic in a block of its own, which the
                // compiler schedules with far fewer registers than the chunk as one block)
                sreg[i] = tile_exists(c, i) ? score_tile(buf[i % PF], c * NS + i) : -INFINITY;
                // the request PF tiles ahead: a key tile of this chunk, then its first value tiles
                buf[i % PF] = i + PF < NS ? request(kbase, c, i + PF, pages) : request(vbase, c, i + PF - NS, pages);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
#pragma unroll
            for (int ib = 0; ib < NS / PF; ++ib) {
                if (ib * PF < n_c) {                 // (wave-uniform)
#pragma unroll
                    for (int ii = 0; ii < PF; ++ii) {
                        const int i = ib * PF + ii;
                        sreg[i] = tile_exists(c, i) ? score_tile(buf[ii], c * NS + i) : -INFINITY;
                        if (i + PF < NS) buf[ii] = request(kbase, c, i + PF, pages);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                } else {
#pragma unroll
                    for (int ii = 0; ii < PF; ++ii) sreg[ib * PF + ii] = -INFINITY;
                }
            }
#pragma unroll
            for (int ii = 0; ii < PF; ++ii) {
                buf[ii] = request(vbase, c, ii, pages);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        {
            const float wave_m = wave_max(lane_m);
            const float wave_l = wave_sum(lane_l * __builtin_amdgcn_exp2f(lane_m - wave_m));
            float* sl = slots + (c & 1) * 2 * NW;
            if (lane == 0) {
                sl[wave] = wave_m;
                sl[NW + wave] = wave_l;
            }
        }
        lds_barrier();              // the chunk's pairs are visible; every bin update of the chunk before is done
        {
            const float* sl = slots + (c & 1) * 2 * NW;
            float m_c = sl[0], l_c = 0.f;
#pragma unroll
            for (int w = 1; w < NW; ++w) m_c = fmaxf(m_c, sl[w]);
            // (every chunk holds at least one valid token, so m_c is a score)
#pragma unroll
            for (int w = 0; w < NW; ++w) l_c = __builtin_fmaf(sl[NW + w], __builtin_amdgcn_exp2f(sl[w] - m_c), l_c);
            if (c == 0) {
                m0 = m_run = m_c;
                l_run = l_c;
                fx = fixed_point_exponent(l_c * (float)n_chunks);
            } else if constexpr (F::SEPARATE) {
                const float m_new = fmaxf(m_run, m_c);
                l_run = l_run * __builtin_amdgcn_exp2f(m_run - m_new) + l_c * __builtin_amdgcn_exp2f(m_c - m_new);
                m_run = m_new;
                const float lg_u = __builtin_amdgcn_logf(l_run) + (m_run - m0) + (float)fx;
                if (lg_u >= 31.5f) {            // (uniform over the workgroup: every thread computes the same)
                    const int sh = (int)floorf(lg_u) - 28;
                    // all wavefronts are between the barrier above and the one below: the bins are quiet
                    const unsigned ws = wave_sum_u32(lane_sum);
                    lane_sum = 0;
                    if (lane == 0) sums[wave] = ws;
                    uint4* b4 = reinterpret_cast<uint4*>(tab);
                    constexpr int Q = 8;                                // 16-byte pieces of bins per row
                    const unsigned half = sh < 32 ? 1u << (sh - 1) : 0u;
                    for (int i = tid; i < 256 * Q; i += NT) {
                        uint4* p = b4 + (i / Q) * (RW / 4) + F::BIN0 / 4 + (i % Q);
                        uint4 v = *p;
                        if (sh >= 32) {
                            v = make_uint4(0, 0, 0, 0);
                        } else {
                            v.x = (v.x + half) >> sh;
                            v.y = (v.y + half) >> sh;
                            v.z = (v.z + half) >> sh;
                            v.w = (v.w + half) >> sh;
                        }
                        *p = v;
                    }
                    lds_barrier();
                    unsigned tot = l_carry;
#pragma unroll
                    for (int w = 0; w < NW; ++w) tot += sums[w];
                    l_carry = sh >= 32 ? 0u : (tot + half) >> sh;
                    fx -= sh;
                }
            }
            fxf = (float)fx;
        }
        if constexpr (!F::SEPARATE) {           // the table becomes the bins (single chunk)
            float4* t4 = reinterpret_cast<float4*>(tab);
#pragma unroll 4
            for (int i = tid; i < F::TAB_FLOATS / 4; i += NT) t4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            lds_barrier();
        }
        // -- bins
        if constexpr (FULL) {
#pragma unroll
            for (int i = 0; i < NS; ++i) {
                if (tile_exists(c, i)) bin_tile(buf[i % PF], c * NS + i, sreg[i]);
                // the request PF tiles ahead: a value tile of this chunk, then the first key tiles of the next
                if (i + PF < NS) {
                    buf[i % PF] = request(vbase, c, i + PF, pages);
                } else if constexpr (!LAST) {
                    buf[i % PF] = request(kbase, c + 1, i + PF - NS, pages_next);
                } else if (i + PF == NS) {
                    request_value_centroids();
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
            const int last_blk = n_c > 0 ? (n_c - 1) / PF : 0;
#pragma unroll
            for (int ib = 0; ib < NS / PF; ++ib) {
                if (ib <= last_blk) {                // (wave-uniform; block 0 always runs)
#pragma unroll
                    for (int ii = 0; ii < PF; ++ii) {
                        const int i = ib * PF + ii;
                        if (tile_exists(c, i)) bin_tile(buf[ii], c * NS + i, sreg[i]);
                        if (i + PF < NS) buf[ii] = request(vbase, c, i + PF, pages);
                        __builtin_amdgcn_sched_barrier(0);
                        if (ii == PF - 1 && ib == last_blk) request_value_centroids();
                    }
                }
            }
        }
        pages = pages_next;
    };
    if constexpr (F::SEPARATE) {
        for (int c = 0; c + 1 < n_chunks; ++c) chunk(c, std::false_type{}, std::true_type{});
    }
    if (my_tiles >= n_chunks * NS) chunk(n_chunks - 1, std::true_type{}, std::true_type{});
    else chunk(n_chunks - 1, std::true_type{}, std::false_type{});

    // ---- 3. epilogue: o = bins . C_V -----------------------------------------------------
    // same walk as the table build; thread-private sums over its centroids of group gl in every
    // chunk, then the four lanes of a group and the wavefronts are added up.
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
            const uint16_t* cv = v_centroids + (size_t)(hkv * GH + ch * GPC + gl) * K * C;
            Nearest vnear;
#pragma unroll(KU)
            for (int k0 = 0; k0 < IPT; k0 += KB) {
                Cent16 rawb[EARLY ? 1 : KB];
                if constexpr (!EARLY) {
#pragma unroll
                    for (int k = 0; k < KB; ++k) rawb[k] = load_cent16(cv + (size_t)piece(k0 + k) * 8);
                }
#pragma unroll
                for (int k = 0; k < KB; ++k) {
                    const int j0 = piece(k0 + k) * JPL;
                    const Cent16& r = EARLY ? rawv[EARLY ? ch : 0][k] : rawb[EARLY ? 0 : k];
#pragma unroll
                    for (int jj = 0; jj < JPL; ++jj) vnear.offer(centroid_distance<C>(xv, &r.w[jj * (C / 2)]), j0 + jj);
                }
            }
            const unsigned long long vkey = group_lanes_min<LPG>(vnear.key());
            if (lane % LPG == 0) lds_min_u64(&keys[GH + ch * GPC + gl], vkey);
        }
    }
    lds_barrier();                                // all bin updates done
    if (lane == 0) sums[wave] = lane_sum;
    // fused step: the new token's weight joins the bins of the codes just found; store the codes
    if (has_new) {
        if (tid < GH) {
            const unsigned code = (unsigned)(keys[GH + tid] & 0xffffffffu);
            lds_add((unsigned)F::word((int)code, F::BIN0 + tid * R) * 4u, *pf_new);
        }
        if (writer)
            store_new_codes<GH, B>(const_cast<uint8_t*>(v_codes) + a.map.tile_index(n, hkv, tile_new) * F::TILE_BYTES, keys + GH, u_new, tid);
        lds_barrier();
    }

    // one fixed-point unit of the bins, relative to the split's maximum
    const float unit = __builtin_amdgcn_exp2f((m0 - m_run) - fxf);
    float acc[NCH][C];
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
#pragma unroll
        for (int i = 0; i < C; ++i) acc[ch][i] = 0.f;
#pragma unroll(KU)
        for (int k0 = 0; k0 < IPT; k0 += KB) {
            if constexpr (!EARLY) {
                const uint16_t* cv = v_centroids + (size_t)(hkv * GH + ch * GPC + gl) * K * C;
#pragma unroll
                for (int k = 0; k < KB; ++k) rawv[0][k] = load_cent16(cv + (size_t)piece(k0 + k) * 8);
            }
            const Cent16 (&raw)[KB] = rawv[EARLY ? ch : 0];
#pragma unroll
            for (int k = 0; k < KB; ++k) {
                const int j0 = piece(k0 + k) * JPL;
#pragma unroll
                for (int jj = 0; jj < JPL; ++jj) {
                    const float* src = tab + F::word(j0 + jj, F::BIN0 + (ch * GPC + gl) * R);
                    unsigned cnt;
                    if constexpr (R == 2) { const uint2 x = *reinterpret_cast<const uint2*>(src); cnt = x.x + x.y; }
                    else cnt = *reinterpret_cast<const unsigned*>(src);
                    const float bin = (float)cnt * unit;
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
#pragma unroll
            for (int m = 1; m < LPG; m <<= 1) acc[ch][i] += __shfl_xor(acc[ch][i], m);
        }
    }
    // per-wave results: scr[64 + wave * D + channel]
    if (lane % LPG == 0) {
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch)
#pragma unroll
            for (int i = 0; i < C; ++i) scr[64 + wave * D + (ch * GPC + gl) * C + i] = acc[ch][i];
    }
    lds_barrier();
    unsigned l_fix = l_carry;                       // exact: integer adds
#pragma unroll
    for (int w = 0; w < NW; ++w) l_fix += sums[w];
    const float l = (float)l_fix * unit;
    const bool direct = a.n_split == 1;             // a single split needs no merge
    if (tid == 0 && !direct) {
        partial_store(part, m_run);
        partial_store(part + 1, l);
    }
    for (int chn = tid; chn < D; chn += NT) {
        float o = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) o += scr[64 + w * D + chn];
        if (direct) out_ptr[(size_t)n * out_batch_stride + (size_t)hq * D + chn] = __builtin_bit_cast(uint16_t, (_Float16)(o / l));
        else partial_store(part + kPartialHeader + chn, o);
    }
    if (!direct) count_and_merge();
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
    merge_splits<false>(p, n_split, head_dim, out, threadIdx.x, blockDim.x);
}

// Arrival counters of the in-kernel merge: one per (sequence, query head) row of a launch.  They
// start at zero (static storage) and every launch leaves them at zero, so they need no clearing;
// what they need is that no two launches that can overlap share a set.  Launches on one stream
// never overlap, so every stream gets a set of its own (the first kMergeSets streams that ask,
// per device; a stream keeps its set).  A stream under graph capture gets none: replays of its
// graph may run on other streams, at the same time as one another.  Whoever gets no set runs
// the separate merge kernel instead.
struct MergeCounters {
    static constexpr int kMaxDevices = 64;
    struct PerDevice {
        std::mutex mu;
        unsigned* base = nullptr;
        bool failed = false;
        hipStream_t streams[kMergeSets];
        int n = 0;
    };
    PerDevice dev[kMaxDevices];

    unsigned* for_stream(hipStream_t stream, int rows)
    {
        if (rows > kMergeRows) return nullptr;
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(stream, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) {
            (void)hipGetLastError();
            return nullptr;
        }
        int d = 0;
        if (hipGetDevice(&d) != hipSuccess || d < 0 || d >= kMaxDevices) return nullptr;
        PerDevice& pd = dev[d];
        std::lock_guard<std::mutex> lock(pd.mu);
        if (pd.failed) return nullptr;
        if (!pd.base) {
            void* p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(merge_counters)) != hipSuccess || !p) {
                pd.failed = true;
                return nullptr;
            }
            pd.base = static_cast<unsigned*>(p);
        }
        for (int i = 0; i < pd.n; ++i)
            if (pd.streams[i] == stream) return pd.base + (size_t)i * kMergeRows;
        if (pd.n == kMergeSets) return nullptr;
        pd.streams[pd.n] = stream;
        return pd.base + (size_t)(pd.n++) * kMergeRows;
    }
};
MergeCounters g_merge_counters;

template <int GH, int C, int B, int NS, bool STEP, bool LAYERS>
cq_status launch_variant(const DecodeArgs& a, hipStream_t stream)
{
    auto kernel = decode_split_kernel<GH, C, B, NS, STEP, LAYERS>;
    static LdsKernelSetup setup;
    if (setup.ensure(reinterpret_cast<const void*>(kernel)) != hipSuccess) return CQ_ERR_HIP;
    using F = Lay<GH, B>;
    if (!F::SEPARATE && a.tiles_per_split > NS * kDecodeWaves) return CQ_ERR_INVALID_ARG;
    const size_t smem = sizeof(float) * (size_t)F::FLOATS(a.f.head_dim, STEP);
    if (smem > 160 * 1024) return CQ_ERR_INVALID_ARG;
    const unsigned grid = (unsigned)(a.batch * a.n_q_heads * a.n_split) * (unsigned)(a.layers ? a.n_layers : 1);
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(kDecodeThreads), smem, stream, a);
    if (hipGetLastError() != hipSuccess) return CQ_ERR_HIP;
    return CQ_OK;
}

template <int GH, int C, int B, int NS, bool STEP, bool LAYERS>
cq_status launch_by_length(const DecodeArgs& a, hipStream_t stream)
{
    const int tiles_per_wave = (a.tiles_per_split + kDecodeWaves - 1) / kDecodeWaves;
    if (tiles_per_wave <= NS / 2) return launch_variant<GH, C, B, NS / 2, STEP, LAYERS>(a, stream);
    return launch_variant<GH, C, B, NS, STEP, LAYERS>(a, stream);
}

template <bool STEP, bool LAYERS>
cq_status launch_format(const DecodeArgs& a, hipStream_t stream)
{
    // 70 KB of LDS per workgroup in every format: two 512-thread workgroups share a CU
    if (a.f.b == 8) {
        if (a.f.gh == 16 && a.f.c == 8) return launch_by_length<16, 8, 8, kChunkTiles8, STEP, LAYERS>(a, stream);
        if (a.f.gh == 32 && a.f.c == 4) return launch_by_length<32, 4, 8, kChunkTiles8, STEP, LAYERS>(a, stream);
        if (a.f.gh == 64 && a.f.c == 2) return launch_by_length<64, 2, 8, kChunkTiles8, STEP, LAYERS>(a, stream);
    } else if (a.f.b == 10 && a.f.gh == 16 && a.f.c == 8) {
        return launch_by_length<16, 8, 10, kChunkTiles10, STEP, LAYERS>(a, stream);
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
    // formats whose table and bins share their LDS walk one chunk per workgroup; the others walk
    // any number of chunks (the bound below only keeps the index arithmetic inside 32 bits)
    if (f.b == 10) return kChunkTiles10 * kDecodeWaves;                // 16384 tokens
    if (f.gh == 64) return kChunkTiles8 * kDecodeWaves;                // 8192 tokens
    return 1 << 20;
}

cq_status launch_decode(const DecodeArgs& a_in, hipStream_t stream)
{
    DecodeArgs a = a_in;
    const int rows = a.batch * a.n_q_heads;
    const int all_rows = rows * (a.layers ? a.n_layers : 1);
    a.merge_counters = a.n_split > 1 ? g_merge_counters.for_stream(stream, all_rows) : nullptr;
    // (a layer-batched launch is always a fused step: its table holds the new rows)
    const cq_status st = a.layers ? launch_format<true, true>(a, stream)
                         : a.xk_new ? launch_format<true, false>(a, stream) : launch_format<false, false>(a, stream);
    if (st != CQ_OK || a.n_split == 1 || a.merge_counters) return st;
    const int threads = a.f.head_dim <= 64 ? 64 : (a.f.head_dim <= 128 ? 128 : 256);
    hipLaunchKernelGGL(decode_merge_kernel, dim3((unsigned)all_rows), dim3(threads), 0, stream,
                       a.partials, a.out, a.n_split, a.f.head_dim, a.layers, rows, a.n_q_heads, a.out_batch_stride);
    if (hipGetLastError() != hipSuccess) return CQ_ERR_HIP;
    return CQ_OK;
}

}  // namespace cq

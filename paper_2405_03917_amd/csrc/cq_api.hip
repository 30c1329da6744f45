// Host entry points of libcq: argument validation, sizing helpers and dispatch.
// Every check here runs before any HIP call, so error paths can be exercised without a GPU.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>

#include "cq_internal.hpp"

// Scratch of cq_decode_attention_static: the partial results of the context splits, for callers
// that cannot pass (or allocate) a workspace.  Every GPU the library runs on holds its own copy
// of the array for the life of the process.  In host code the name below is only a stand-in
// for the symbol: the array's device address is looked up once per device (StaticScratch).
static __device__ __align__(256) unsigned char scratch[CQ_STATIC_SCRATCH_BYTES];

namespace cq {

cq_status derive(const cq_format* fmt, Derived* out)
{
    if (!fmt) return CQ_ERR_INVALID_ARG;
    if (fmt->c <= 0 || fmt->b <= 0 || fmt->head_dim <= 0 || fmt->n_kv_heads <= 0) return CQ_ERR_INVALID_ARG;
    if (fmt->head_dim % fmt->c != 0) return CQ_ERR_INVALID_ARG;
    Derived d;
    d.c = fmt->c;
    d.b = fmt->b;
    d.head_dim = fmt->head_dim;
    d.n_kv_heads = fmt->n_kv_heads;
    d.gh = fmt->head_dim / fmt->c;
    const bool ok8 = fmt->b == 8 && (fmt->c == 2 || fmt->c == 4 || fmt->c == 8) && fmt->head_dim == 128;
    const bool ok10 = fmt->b == 10 && fmt->c == 8 && fmt->head_dim == 128;
    if (!ok8 && !ok10) return CQ_ERR_UNSUPPORTED;
    d.k = 1 << fmt->b;
    d.channels = fmt->n_kv_heads * fmt->head_dim;
    d.groups = d.channels / fmt->c;
    d.bpth = d.gh * fmt->b / 8;
    d.tile_bytes = kTileTokens * d.bpth;
    d.fuse = 1;
    d.sub_c = d.c;
    d.sub_b = d.b;
    if (out) *out = d;
    return CQ_OK;
}

cq_status derive_any(const cq_format* fmt, Derived* out)
{
    const cq_status st = derive(fmt, out);
    if (st != CQ_ERR_UNSUPPORTED) return st;
    // CQ-<c>c<b>b with b = 2 or 4: 8 / b neighbouring groups are stored as one byte, i.e. as one code
    // of the product codebook of those groups
    if (fmt->b != 2 && fmt->b != 4) return CQ_ERR_UNSUPPORTED;
    const int fuse = 8 / fmt->b;
    cq_format fused = *fmt;
    fused.c = fmt->c * fuse;
    fused.b = 8;
    Derived d;
    const cq_status sf = derive(&fused, &d);
    if (sf != CQ_OK) return sf;
    d.fuse = fuse;
    d.sub_c = fmt->c;
    d.sub_b = fmt->b;
    if (out) *out = d;
    return CQ_OK;
}

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Device address of `scratch` on the current device: asked for on the first use on each
// device (with that device current) and kept; host code passes this pointer, never the
// array's name, to kernels.
struct StaticScratch {
    static constexpr int kMaxDevices = 64;
    std::once_flag once[kMaxDevices];
    hipError_t result[kMaxDevices];
    void* ptr[kMaxDevices];
    hipError_t get(void** out)
    {
        int dev = 0;
        const hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
        std::call_once(once[dev], [&] {
            void* p = nullptr;
            result[dev] = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            ptr[dev] = p;
        });
        if (result[dev] != hipSuccess || !ptr[dev]) return result[dev] != hipSuccess ? result[dev] : hipErrorInvalidSymbol;
        *out = ptr[dev];
        return hipSuccess;
    }
};
StaticScratch g_static_scratch;

int default_tiles_per_split(const Derived& f, int batch, int n_q_heads, int t, int max_tiles, bool rope = false)
{
    // A workgroup costs its tiles plus a fixed part (table build, bins x centroids: each reads a
    // whole head's codebook), here expressed in tiles of streaming time; the chip runs `slots`
    // workgroups at a time, in rounds.  Take the number of splits that minimises
    // rounds x (tiles + fixed) over the splits the kernel allows, down to 16 tiles per split.
    const int n_tiles = (t + kTileTokens - 1) / kTileTokens;
    const long bh = (long)batch * n_q_heads;
    // Two workgroups per CU stream a few per cent faster than one, and pay the fixed part twice,
    // one after the other: with byte codes that is worth it from about 768 tiles per CU on
    // (measured: below, one workgroup per CU is 2 to 4 us faster at every size).  Keys cached
    // before RoPE run one workgroup per CU, and a tile costs several times the arithmetic, so the
    // fixed part is worth fewer of them.
    const long slots = rope ? 256 : (f.b == 8 && bh * n_tiles < 768L * 256 ? 256 : 512);
    const long fixed = rope ? (f.b == 10 ? 32 : 8) : (f.b == 10 ? 180 : (f.gh == 16 ? 60 : (f.gh == 32 ? 30 : 15)));
    const long ns_min = (n_tiles + max_tiles - 1) / max_tiles;
    const long ns_max = std::max<long>(ns_min, n_tiles / 16);
    long best_ns = ns_min, best_cost = -1;
    for (long ns = ns_min; ns <= ns_max && ns < ns_min + 4096; ++ns) {
        const long tiles = (n_tiles + ns - 1) / ns;
        const long rounds = (bh * ns + slots - 1) / slots;
        const long cost = rounds * (tiles + fixed);
        if (best_cost < 0 || cost < best_cost) {
            best_cost = cost;
            best_ns = ns;
        }
        if (bh * ns >= 8 * slots && tiles <= 2 * fixed) break;      // further splits only add fixed cost
    }
    return (int)((n_tiles + best_ns - 1) / best_ns);
}

int default_tiles_per_split(const Derived& f, int batch, int n_q_heads, int t)
{
    return default_tiles_per_split(f, batch, n_q_heads, t, decode_max_tiles_per_split(f));
}

int rope_default_tiles_per_split(const Derived& f, int batch, int n_q_heads, int t)
{
    // grouped queries with byte codes: the kernel that shares the key rotation among four query
    // heads, one workgroup per (sequence, KV head, four query heads, split), shorter splits
    const int qper = n_q_heads / f.n_kv_heads;
    if (f.b == 8 && qper >= 2)
        return default_tiles_per_split(f, batch, f.n_kv_heads * ((qper + 3) / 4), t, decode_rope_shared_max_tiles_per_split(), true);
    return default_tiles_per_split(f, batch, n_q_heads, t, decode_rope_max_tiles_per_split(), true);
}

}  // namespace
}  // namespace cq

using namespace cq;

extern "C" {

int32_t cq_version(void) { return 100; }

const char* cq_status_string(cq_status status)
{
    switch (status) {
        case CQ_OK: return "CQ_OK";
        case CQ_ERR_INVALID_ARG: return "CQ_ERR_INVALID_ARG";
        case CQ_ERR_UNSUPPORTED: return "CQ_ERR_UNSUPPORTED";
        case CQ_ERR_WORKSPACE_TOO_SMALL: return "CQ_ERR_WORKSPACE_TOO_SMALL";
        case CQ_ERR_HIP: return "CQ_ERR_HIP";
    }
    return "CQ_ERR_UNKNOWN";
}

cq_status cq_format_check(const cq_format* fmt) { return derive_any(fmt, nullptr); }

size_t cq_code_bytes_per_token_head(const cq_format* fmt)
{
    Derived f;
    if (derive_any(fmt, &f) != CQ_OK) return 0;
    return (size_t)f.bpth;
}

size_t cq_cache_bytes(const cq_format* fmt, int32_t batch, int32_t t_cap)
{
    Derived f;
    if (derive_any(fmt, &f) != CQ_OK) return 0;
    if (batch <= 0 || t_cap <= 0 || t_cap % kTileTokens != 0) return 0;
    return (size_t)batch * f.n_kv_heads * (t_cap / kTileTokens) * f.tile_bytes;
}

namespace {

cq_status check_encode_tensor(const Derived& f, const void* x, int64_t x_batch_stride, int64_t x_row_stride,
                              const void* centroids, const void* codes, int32_t batch, int32_t t_new)
{
    if (!x || !centroids || !codes) return CQ_ERR_INVALID_ARG;
    if (x_row_stride < f.channels || x_row_stride % 8 != 0) return CQ_ERR_INVALID_ARG;
    if (batch > 1 && (x_batch_stride < (int64_t)t_new * x_row_stride || x_batch_stride % 8 != 0))
        return CQ_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned16(centroids) || !aligned16(codes)) return CQ_ERR_INVALID_ARG;
    return CQ_OK;
}

CacheMap contiguous_map(const Derived& f, int32_t t_cap)
{
    return CacheMap{nullptr, 0, 0, t_cap / kTileTokens, f.n_kv_heads};
}

// Checks a page table and turns it into the kernels' map; *t_cap receives the token capacity.
cq_status paged_map(const Derived& f, const cq_page_table* pt, int32_t batch, CacheMap* map, int32_t* t_cap)
{
    if (!pt || !pt->block_table || pt->n_pages <= 0 || pt->max_tiles <= 0 || pt->max_tiles > (1 << 24)) return CQ_ERR_INVALID_ARG;
    if (pt->row_stride < pt->max_tiles || (reinterpret_cast<uintptr_t>(pt->block_table) & 3u)) return CQ_ERR_INVALID_ARG;
    (void)batch;
    *map = CacheMap{pt->block_table, pt->row_stride, pt->n_pages, 0, f.n_kv_heads};
    *t_cap = pt->max_tiles * kTileTokens;
    return CQ_OK;
}

cq_status check_encode_shape(const Derived& f, int32_t batch, int32_t t_new, int32_t t_offset, int32_t t_cap)
{
    if (batch <= 0 || t_new <= 0 || t_cap <= 0 || t_cap % kTileTokens != 0) return CQ_ERR_INVALID_ARG;
    if (batch > 32767 || f.n_kv_heads > 65535) return CQ_ERR_INVALID_ARG;
    if (t_offset < 0 || (int64_t)t_offset + t_new > t_cap) return CQ_ERR_INVALID_ARG;
    return CQ_OK;
}

}  // namespace

namespace {

cq_status encode_common(const void* x_k, const void* x_v, int64_t x_batch_stride, int64_t x_row_stride,
                        const void* k_centroids, const void* v_centroids, const Derived& f,
                        int32_t batch, int32_t t_new, void* k_codes, void* v_codes, int32_t t_offset, int32_t t_cap,
                        const CacheMap& map, void* stream)
{
    cq_status st;
    if ((st = check_encode_shape(f, batch, t_new, t_offset, t_cap)) != CQ_OK) return st;
    if ((st = check_encode_tensor(f, x_k, x_batch_stride, x_row_stride, k_centroids, k_codes, batch, t_new)) != CQ_OK) return st;
    const bool two = x_v != nullptr || v_centroids != nullptr || v_codes != nullptr;
    if (two) {
        if ((st = check_encode_tensor(f, x_v, x_batch_stride, x_row_stride, v_centroids, v_codes, batch, t_new)) != CQ_OK) return st;
        if (k_codes == v_codes) return CQ_ERR_INVALID_ARG;
    }
    EncodeArgs a;
    a.tensor[0] = EncodeTensor{static_cast<const uint16_t*>(x_k), x_batch_stride, x_row_stride,
                               static_cast<const uint16_t*>(k_centroids), static_cast<uint8_t*>(k_codes)};
    a.tensor[1] = two ? EncodeTensor{static_cast<const uint16_t*>(x_v), x_batch_stride, x_row_stride,
                                     static_cast<const uint16_t*>(v_centroids), static_cast<uint8_t*>(v_codes)}
                      : a.tensor[0];
    a.n_tensors = two ? 2 : 1;
    a.batch = batch;
    a.t_new = t_new;
    a.t_offset = t_offset;
    a.map = map;
    a.f = f;
    return launch_encode(a, static_cast<hipStream_t>(stream));
}

}  // namespace

cq_status cq_encode(const void* x, int64_t x_batch_stride, int64_t x_row_stride,
                    const void* centroids, const cq_format* fmt,
                    int32_t batch, int32_t t_new,
                    void* codes, int32_t t_offset, int32_t t_cap, void* stream)
{
    Derived f;
    const cq_status st = derive_any(fmt, &f);
    if (st != CQ_OK) return st;
    if (t_cap <= 0 || t_cap % kTileTokens != 0) return CQ_ERR_INVALID_ARG;
    return encode_common(x, nullptr, x_batch_stride, x_row_stride, centroids, nullptr, f, batch, t_new, codes, nullptr,
                         t_offset, t_cap, contiguous_map(f, t_cap), stream);
}

cq_status cq_encode_kv(const void* x_k, const void* x_v, int64_t x_batch_stride, int64_t x_row_stride,
                       const void* k_centroids, const void* v_centroids, const cq_format* fmt,
                       int32_t batch, int32_t t_new,
                       void* k_codes, void* v_codes, int32_t t_offset, int32_t t_cap, void* stream)
{
    Derived f;
    const cq_status st = derive_any(fmt, &f);
    if (st != CQ_OK) return st;
    if (t_cap <= 0 || t_cap % kTileTokens != 0) return CQ_ERR_INVALID_ARG;
    if (!x_v || !v_centroids || !v_codes) return CQ_ERR_INVALID_ARG;
    return encode_common(x_k, x_v, x_batch_stride, x_row_stride, k_centroids, v_centroids, f, batch, t_new, k_codes,
                         v_codes, t_offset, t_cap, contiguous_map(f, t_cap), stream);
}

cq_status cq_fused_format(const cq_format* fmt, cq_format* fused)
{
    Derived f;
    const cq_status st = derive_any(fmt, &f);
    if (st != CQ_OK) return st;
    if (!fused) return CQ_ERR_INVALID_ARG;
    *fused = cq_format{f.c, f.b, f.head_dim, f.n_kv_heads};
    return CQ_OK;
}

cq_status cq_expand_codebook(const void* centroids, const cq_format* fmt, void* fused_centroids, void* stream)
{
    Derived f;
    const cq_status st = derive_any(fmt, &f);
    if (st != CQ_OK) return st;
    if (f.fuse == 1) return CQ_ERR_INVALID_ARG;          // nothing to expand: the format is its own fused format
    if (!centroids || !fused_centroids || !aligned16(centroids) || !aligned16(fused_centroids) || centroids == fused_centroids)
        return CQ_ERR_INVALID_ARG;
    return launch_expand_codebook(static_cast<const uint16_t*>(centroids), f, static_cast<uint16_t*>(fused_centroids),
                                  static_cast<hipStream_t>(stream));
}

size_t cq_paged_cache_bytes(const cq_format* fmt, int32_t n_pages)
{
    Derived f;
    if (derive_any(fmt, &f) != CQ_OK || n_pages <= 0) return 0;
    return (size_t)n_pages * f.n_kv_heads * f.tile_bytes;
}

cq_status cq_encode_kv_paged(const void* x_k, const void* x_v, int64_t x_batch_stride, int64_t x_row_stride,
                             const void* k_centroids, const void* v_centroids, const cq_format* fmt,
                             int32_t batch, int32_t t_new,
                             void* k_pool, void* v_pool, const cq_page_table* pages, int32_t t_offset, void* stream)
{
    Derived f;
    cq_status st = derive_any(fmt, &f);
    if (st != CQ_OK) return st;
    CacheMap map;
    int32_t t_cap = 0;
    if ((st = paged_map(f, pages, batch, &map, &t_cap)) != CQ_OK) return st;
    if (!x_v || !v_centroids || !v_pool) return CQ_ERR_INVALID_ARG;
    return encode_common(x_k, x_v, x_batch_stride, x_row_stride, k_centroids, v_centroids, f, batch, t_new, k_pool,
                         v_pool, t_offset, t_cap, map, stream);
}

cq_status cq_dequantize(const void* codes, const void* centroids, const cq_format* fmt,
                        int32_t batch, int32_t t_offset, int32_t t_count, int32_t t_cap,
                        void* out, int64_t out_batch_stride, int64_t out_row_stride, void* stream)
{
    Derived f;
    cq_status st = derive(fmt, &f);
    if (st != CQ_OK) return st;
    if ((st = check_encode_shape(f, batch, t_count, t_offset, t_cap)) != CQ_OK) return st;
    if (!codes || !centroids || !out || !aligned16(codes) || !aligned16(centroids) || !aligned16(out)) return CQ_ERR_INVALID_ARG;
    if (out_row_stride < f.channels || out_row_stride % 8 != 0) return CQ_ERR_INVALID_ARG;
    if (batch > 1 && (out_batch_stride < (int64_t)t_count * out_row_stride || out_batch_stride % 8 != 0)) return CQ_ERR_INVALID_ARG;
    DequantArgs a;
    a.codes = static_cast<const uint8_t*>(codes);
    a.centroids = static_cast<const uint16_t*>(centroids);
    a.out = static_cast<uint16_t*>(out);
    a.out_batch_stride = out_batch_stride;
    a.out_row_stride = out_row_stride;
    a.batch = batch;
    a.t_offset = t_offset;
    a.t_count = t_count;
    a.map = contiguous_map(f, t_cap);
    a.f = f;
    return launch_dequantize(a, static_cast<hipStream_t>(stream));
}

namespace {

// The centroid learning sees a sub-byte format as what it is: channels / c groups of 2^b centroids.
cq_status derive_for_learning(const cq_format* fmt, Derived* f)
{
    const cq_status st = derive_any(fmt, f);
    if (st != CQ_OK || f->fuse == 1) return st;
    f->c = f->sub_c;
    f->b = f->sub_b;
    f->k = 1 << f->sub_b;
    f->gh = f->head_dim / f->sub_c;
    f->groups = f->channels / f->sub_c;
    return CQ_OK;
}

}  // namespace

size_t cq_kmeans_workspace_bytes(const cq_format* fmt, int32_t n_points)
{
    Derived f;
    if (derive_for_learning(fmt, &f) != CQ_OK || n_points <= 0 || n_points > CQ_KMEANS_MAX_POINTS) return 0;
    return kmeans_workspace_layout(f, n_points, nullptr, nullptr);
}

cq_status cq_kmeans_fit(const void* x, int64_t x_row_stride, const float* weights, const cq_format* fmt,
                        int32_t n_points, int32_t n_iter, const uint64_t* rnd, const float* init_centroids,
                        int32_t* picks, void* centroids, float* centroids_f32, uint16_t* assignment,
                        void* workspace, size_t workspace_bytes, void* stream)
{
    Derived f;
    cq_status st = derive_for_learning(fmt, &f);
    if (st != CQ_OK) return st;
    if (n_points <= 0 || n_points > CQ_KMEANS_MAX_POINTS || n_iter < 0) return CQ_ERR_INVALID_ARG;
    if (!x || !aligned16(x) || x_row_stride < f.channels || x_row_stride % 8 != 0) return CQ_ERR_INVALID_ARG;
    if (weights && !aligned16(weights)) return CQ_ERR_INVALID_ARG;
    // exactly one source of starting centroids: k-means++ from random words, or the caller's
    if ((rnd == nullptr) == (init_centroids == nullptr)) return CQ_ERR_INVALID_ARG;
    if ((rnd && !aligned16(rnd)) || (init_centroids && !aligned16(init_centroids))) return CQ_ERR_INVALID_ARG;
    if (picks && !rnd) return CQ_ERR_INVALID_ARG;
    if (!centroids && !centroids_f32) return CQ_ERR_INVALID_ARG;
    if ((centroids && !aligned16(centroids)) || (centroids_f32 && !aligned16(centroids_f32)) ||
        (assignment && !aligned16(assignment)) || (picks && !aligned16(picks)))
        return CQ_ERR_INVALID_ARG;
    if (!workspace || !aligned16(workspace)) return CQ_ERR_INVALID_ARG;
    if (workspace_bytes < kmeans_workspace_layout(f, n_points, nullptr, nullptr)) return CQ_ERR_WORKSPACE_TOO_SMALL;

    KMeansArgs a;
    a.x = static_cast<const uint16_t*>(x);
    a.x_row_stride = x_row_stride;
    a.weights = weights;
    a.n = n_points;
    a.n_iter = n_iter;
    a.rnd = rnd;
    a.do_init = rnd != nullptr;
    a.cent_in = init_centroids;
    a.picks = picks;
    a.cent16_out = static_cast<uint16_t*>(centroids);
    a.cent32_out = centroids_f32;
    a.assign_out = assignment;
    a.f = f;
    return launch_kmeans(a, workspace, static_cast<hipStream_t>(stream));
}

int32_t cq_decode_default_split(const cq_format* fmt, int32_t batch, int32_t n_q_heads, int32_t t)
{
    Derived f;
    if (derive(fmt, &f) != CQ_OK || batch <= 0 || n_q_heads <= 0 || t <= 0) return 0;
    return default_tiles_per_split(f, batch, n_q_heads, t) * kTileTokens;
}

size_t cq_decode_workspace_bytes(const cq_format* fmt, int32_t batch, int32_t n_q_heads,
                                 int32_t t, int32_t tokens_per_split)
{
    Derived f;
    if (derive(fmt, &f) != CQ_OK || batch <= 0 || n_q_heads <= 0 || t <= 0) return 0;
    if (tokens_per_split < 0 || tokens_per_split % kTileTokens != 0) return 0;
    const int tiles = tokens_per_split ? tokens_per_split / kTileTokens
                                       : default_tiles_per_split(f, batch, n_q_heads, t);
    if (tiles > decode_max_tiles_per_split(f)) return 0;
    const int n_tiles = (t + kTileTokens - 1) / kTileTokens;
    const int n_split = (n_tiles + tiles - 1) / tiles;
    return sizeof(float) * (size_t)batch * n_q_heads * n_split * (f.head_dim + kPartialHeader);
}

namespace {

// One query token of a chunk served token by token: q and out rows of the token inside
// [batch][m][n_q_heads][head_dim] tensors, and its context seq_lens[n] - shift (at least floor).
struct TokenView {
    int64_t q_batch_stride, out_batch_stride;
    int seq_len_shift, seq_len_floor;
};

cq_status decode_common(const void* q, const void* x_k_new, const void* x_v_new, int64_t x_row_stride,
                        const void* k_codes, const void* v_codes,
                        const void* k_centroids, const void* v_centroids,
                        float scale, const cq_format* fmt,
                        int32_t batch, int32_t n_q_heads, int32_t t, int32_t t_cap, const cq_page_table* pages,
                        const int32_t* seq_lens, int32_t tokens_per_split,
                        void* out, void* workspace, size_t workspace_bytes, void* stream, bool step,
                        const void* rope_table = nullptr, int32_t rope_positions = 0,
                        const LayerPtrs* layers = nullptr, int32_t n_layers = 1, const TokenView* view = nullptr,
                        bool static_scratch = false)
{
    Derived f;
    cq_status st = derive(fmt, &f);
    if (st != CQ_OK) return st;
    const bool rope = rope_positions != 0;
    // the library's own scratch array takes the workspace's place (its address is only looked up
    // once every check below has passed); until then a stand-in keeps the checks uniform
    if (static_scratch) {
        workspace = reinterpret_cast<void*>(uintptr_t{256});
        workspace_bytes = CQ_STATIC_SCRATCH_BYTES;
    }
    if (rope && f.head_dim != 128) return CQ_ERR_UNSUPPORTED;
    CacheMap map;
    if (pages) {
        if ((st = paged_map(f, pages, batch, &map, &t_cap)) != CQ_OK) return st;
    } else {
        if (t_cap <= 0 || t_cap % kTileTokens != 0) return CQ_ERR_INVALID_ARG;
        map = contiguous_map(f, t_cap);
    }
    // (a layer-batched call brings these per layer in its table, checked when the table was filled)
    if (!layers && (!q || !k_codes || !v_codes || !k_centroids || !v_centroids || !out)) return CQ_ERR_INVALID_ARG;
    if (!workspace || n_layers <= 0) return CQ_ERR_INVALID_ARG;
    if (batch <= 0 || n_q_heads <= 0 || n_q_heads % f.n_kv_heads != 0) return CQ_ERR_INVALID_ARG;
    if (t <= 0 || t > t_cap) return CQ_ERR_INVALID_ARG;
    if (!std::isfinite(scale)) return CQ_ERR_INVALID_ARG;
    if (tokens_per_split < 0 || tokens_per_split % kTileTokens != 0) return CQ_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k_codes) || !aligned16(v_codes) || !aligned16(k_centroids) ||
        !aligned16(v_centroids) || !aligned16(out) || !aligned16(workspace))
        return CQ_ERR_INVALID_ARG;
    if (step) {
        if (!layers && (!x_k_new || !x_v_new || !aligned16(x_k_new) || !aligned16(x_v_new))) return CQ_ERR_INVALID_ARG;
        if (x_row_stride < f.channels || x_row_stride % 8 != 0) return CQ_ERR_INVALID_ARG;
        if (!layers && k_codes == v_codes) return CQ_ERR_INVALID_ARG;
    }
    if (rope) {
        if (!rope_table || !aligned16(rope_table)) return CQ_ERR_INVALID_ARG;
        if (rope_positions < 0 || rope_positions % kTileTokens != 0 || t > rope_positions) return CQ_ERR_INVALID_ARG;
    }
    const int max_tiles = rope ? decode_rope_max_tiles_per_split() : decode_max_tiles_per_split(f);
    const int tiles = tokens_per_split ? tokens_per_split / kTileTokens
                                       : (rope ? rope_default_tiles_per_split(f, batch, n_q_heads, t)
                                               : default_tiles_per_split(f, batch, n_q_heads, t, max_tiles));
    if (tiles > max_tiles) return CQ_ERR_INVALID_ARG;
    const int n_tiles = (t + kTileTokens - 1) / kTileTokens;
    const int n_split = (n_tiles + tiles - 1) / tiles;
    const size_t need = sizeof(float) * (size_t)batch * n_q_heads * n_split * (f.head_dim + kPartialHeader) * n_layers;
    if (workspace_bytes < need) return CQ_ERR_WORKSPACE_TOO_SMALL;
    if ((int64_t)batch * n_q_heads * n_split * n_layers > 0x7fffffffLL) return CQ_ERR_INVALID_ARG;
    if (static_scratch && g_static_scratch.get(&workspace) != hipSuccess) return CQ_ERR_HIP;

    DecodeArgs a;
    a.layers = layers;
    a.n_layers = n_layers;
    a.wgs_per_layer = batch * n_q_heads * n_split;
    a.q = static_cast<const uint16_t*>(q);
    a.k_codes = static_cast<const uint8_t*>(k_codes);
    a.v_codes = static_cast<const uint8_t*>(v_codes);
    a.k_centroids = static_cast<const uint16_t*>(k_centroids);
    a.v_centroids = static_cast<const uint16_t*>(v_centroids);
    a.scale_log2e = scale * 1.4426950408889634f;
    a.batch = batch;
    a.n_q_heads = n_q_heads;
    a.t = t;
    a.map = map;
    a.seq_lens = seq_lens;
    a.xk_new = step ? static_cast<const uint16_t*>(x_k_new) : nullptr;
    a.xv_new = step ? static_cast<const uint16_t*>(x_v_new) : nullptr;
    a.x_new_stride = x_row_stride;
    a.tiles_per_split = tiles;
    a.n_split = n_split;
    a.partials = static_cast<float*>(workspace);
    a.out = static_cast<uint16_t*>(out);
    a.q_batch_stride = view ? view->q_batch_stride : (int64_t)n_q_heads * f.head_dim;
    a.out_batch_stride = view ? view->out_batch_stride : (int64_t)n_q_heads * f.head_dim;
    a.seq_len_shift = view ? view->seq_len_shift : 0;
    a.seq_len_floor = view ? view->seq_len_floor : 1;
    a.merge_counters = nullptr;
    a.f = f;
    if (rope) return launch_decode_rope(a, static_cast<const float*>(rope_table), rope_positions, static_cast<hipStream_t>(stream));
    return launch_decode(a, static_cast<hipStream_t>(stream));
}

}  // namespace

cq_status cq_decode_attention(const void* q, const void* k_codes, const void* v_codes,
                              const void* k_centroids, const void* v_centroids,
                              float scale, const cq_format* fmt,
                              int32_t batch, int32_t n_q_heads, int32_t t, int32_t t_cap,
                              const int32_t* seq_lens, int32_t tokens_per_split,
                              void* out, void* workspace, size_t workspace_bytes, void* stream)
{
    return decode_common(q, nullptr, nullptr, 0, k_codes, v_codes, k_centroids, v_centroids, scale, fmt, batch,
                         n_q_heads, t, t_cap, nullptr, seq_lens, tokens_per_split, out, workspace, workspace_bytes, stream,
                         false);
}

cq_status cq_decode_attention_static(const void* q, const void* k_codes, const void* v_codes,
                                     const void* k_centroids, const void* v_centroids,
                                     float scale, const cq_format* fmt,
                                     int32_t batch, int32_t n_q_heads, int32_t t, int32_t t_cap,
                                     const int32_t* seq_lens, int32_t tokens_per_split,
                                     void* out, void* stream)
{
    return decode_common(q, nullptr, nullptr, 0, k_codes, v_codes, k_centroids, v_centroids, scale, fmt, batch,
                         n_q_heads, t, t_cap, nullptr, seq_lens, tokens_per_split, out, nullptr, 0, stream,
                         false, nullptr, 0, nullptr, 1, nullptr, true);
}

cq_status cq_decode_attention_paged(const void* q, const void* k_pool, const void* v_pool,
                                    const void* k_centroids, const void* v_centroids,
                                    float scale, const cq_format* fmt,
                                    int32_t batch, int32_t n_q_heads, int32_t t, const cq_page_table* pages,
                                    const int32_t* seq_lens, int32_t tokens_per_split,
                                    void* out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!pages) return CQ_ERR_INVALID_ARG;
    return decode_common(q, nullptr, nullptr, 0, k_pool, v_pool, k_centroids, v_centroids, scale, fmt, batch,
                         n_q_heads, t, 0, pages, seq_lens, tokens_per_split, out, workspace, workspace_bytes, stream, false);
}

cq_status cq_decode_step(const void* q, const void* x_k_new, const void* x_v_new, int64_t x_row_stride,
                         void* k_codes, void* v_codes,
                         const void* k_centroids, const void* v_centroids,
                         float scale, const cq_format* fmt,
                         int32_t batch, int32_t n_q_heads, int32_t t, int32_t t_cap,
                         const int32_t* seq_lens, int32_t tokens_per_split,
                         void* out, void* workspace, size_t workspace_bytes, void* stream)
{
    return decode_common(q, x_k_new, x_v_new, x_row_stride, k_codes, v_codes, k_centroids, v_centroids, scale, fmt,
                         batch, n_q_heads, t, t_cap, nullptr, seq_lens, tokens_per_split, out, workspace, workspace_bytes,
                         stream, true);
}

cq_status cq_decode_step_paged(const void* q, const void* x_k_new, const void* x_v_new, int64_t x_row_stride,
                               void* k_pool, void* v_pool,
                               const void* k_centroids, const void* v_centroids,
                               float scale, const cq_format* fmt,
                               int32_t batch, int32_t n_q_heads, int32_t t, const cq_page_table* pages,
                               const int32_t* seq_lens, int32_t tokens_per_split,
                               void* out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!pages) return CQ_ERR_INVALID_ARG;
    return decode_common(q, x_k_new, x_v_new, x_row_stride, k_pool, v_pool, k_centroids, v_centroids, scale, fmt,
                         batch, n_q_heads, t, 0, pages, seq_lens, tokens_per_split, out, workspace, workspace_bytes,
                         stream, true);
}

namespace {

// context split of the chunk kernel: enough workgroups to fill the chip, at least 8 tiles each
int chunk_tiles_per_split(const Derived& f, int batch, int n_q_heads, int m, int t)
{
    const int qper = n_q_heads / f.n_kv_heads;
    const int rpw = chunk_rows_per_workgroup(m * qper);
    const long row_blocks = ((long)m * qper + rpw - 1) / rpw;
    const long base = (long)batch * f.n_kv_heads * row_blocks;
    const int n_tiles = (t + kTileTokens - 1) / kTileTokens;
    long n_split = std::max(1L, (512 + base - 1) / base);
    n_split = std::min<long>(n_split, std::max(1, n_tiles / 8));
    return (int)((n_tiles + n_split - 1) / n_split);
}

// Short chunks go through the single-token kernel, one launch per query token (token j with a
// context shortened by m - 1 - j): the chunk kernel dequantises every tile of the context
// whatever m is, which costs 8-16 single-token launches on large multi-head batches (measured;
// divided by the query heads per KV head, which share the dequantised tiles) and 2-3 on small
// ones (both kernels are then bound by launch and latency).
bool chunk_by_token(const Derived& f, int batch, int n_q_heads, int m, int t)
{
    const int qper = n_q_heads / f.n_kv_heads;
    const long tiles = (long)batch * f.n_kv_heads * ((t + kTileTokens - 1) / kTileTokens);
    const int limit = tiles >= 16384 ? std::max(2, 8 / qper) : 2;
    return m <= limit;
}

// split (tiles) and workspace need of query token j of a chunk served token by token
struct TokenCall {
    int t, tiles, n_split;
    size_t workspace;
};
TokenCall chunk_token_call(const Derived& f, int batch, int n_q_heads, int m, int t, int j)
{
    TokenCall c;
    c.t = t - (m - 1 - j);
    c.tiles = default_tiles_per_split(f, batch, n_q_heads, c.t);
    const int n_tiles = (c.t + kTileTokens - 1) / kTileTokens;
    c.n_split = (n_tiles + c.tiles - 1) / c.tiles;
    c.workspace = c.n_split > 1 ? sizeof(float) * (size_t)batch * n_q_heads * c.n_split * (f.head_dim + kPartialHeader) : 0;
    return c;
}

cq_status chunk_common(const void* q, const void* k_codes, const void* v_codes,
                       const void* k_centroids, const void* v_centroids, float scale, const cq_format* fmt,
                       int32_t batch, int32_t n_q_heads, int32_t m, int32_t t, int32_t t_cap, const cq_page_table* pages,
                       const int32_t* seq_lens, int32_t tokens_per_split,
                       void* out, void* workspace, size_t workspace_bytes, void* stream,
                       const void* rope_table = nullptr, int32_t rope_positions = 0)
{
    Derived f;
    cq_status st = derive(fmt, &f);
    if (st != CQ_OK) return st;
    if (f.head_dim != 128) return CQ_ERR_UNSUPPORTED;
    // keys cached before the rotary embedding: always the matrix-core kernel here (its caller serves
    // the shortest chunks token by token itself)
    const bool rope = rope_positions != 0;
    if (rope) {
        if (!rope_table || !aligned16(rope_table)) return CQ_ERR_INVALID_ARG;
        if (rope_positions < 0 || rope_positions % kTileTokens != 0 || t > rope_positions) return CQ_ERR_INVALID_ARG;
    }
    CacheMap map;
    if (pages) {
        if ((st = paged_map(f, pages, batch, &map, &t_cap)) != CQ_OK) return st;
    } else {
        if (t_cap <= 0 || t_cap % kTileTokens != 0) return CQ_ERR_INVALID_ARG;
        map = contiguous_map(f, t_cap);
    }
    if (!q || !k_codes || !v_codes || !k_centroids || !v_centroids || !out) return CQ_ERR_INVALID_ARG;
    if (batch <= 0 || n_q_heads <= 0 || n_q_heads % f.n_kv_heads != 0) return CQ_ERR_INVALID_ARG;
    if (m <= 0 || t < m || t > t_cap) return CQ_ERR_INVALID_ARG;
    if (!std::isfinite(scale)) return CQ_ERR_INVALID_ARG;
    if (tokens_per_split < 0 || tokens_per_split % kTileTokens != 0) return CQ_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k_codes) || !aligned16(v_codes) || !aligned16(k_centroids) ||
        !aligned16(v_centroids) || !aligned16(out) || !aligned16(workspace))
        return CQ_ERR_INVALID_ARG;
    if (!rope && tokens_per_split == 0 && chunk_by_token(f, batch, n_q_heads, m, t)) {
        for (int j = 0; j < m; ++j) {
            const TokenCall c = chunk_token_call(f, batch, n_q_heads, m, t, j);
            if (c.workspace && !workspace) return CQ_ERR_INVALID_ARG;
            if (workspace_bytes < c.workspace) return CQ_ERR_WORKSPACE_TOO_SMALL;
            if ((int64_t)batch * n_q_heads * c.n_split > 0x7fffffffLL) return CQ_ERR_INVALID_ARG;
        }
        const int64_t row = (int64_t)n_q_heads * f.head_dim;
        for (int j = 0; j < m; ++j) {           // (in stream order: the calls share the workspace)
            const TokenCall c = chunk_token_call(f, batch, n_q_heads, m, t, j);
            DecodeArgs a;
            a.layers = nullptr;
            a.n_layers = 1;
            a.wgs_per_layer = batch * n_q_heads * c.n_split;
            a.q = static_cast<const uint16_t*>(q) + j * row;
            a.out = static_cast<uint16_t*>(out) + j * row;
            a.q_batch_stride = a.out_batch_stride = m * row;
            a.k_codes = static_cast<const uint8_t*>(k_codes);
            a.v_codes = static_cast<const uint8_t*>(v_codes);
            a.k_centroids = static_cast<const uint16_t*>(k_centroids);
            a.v_centroids = static_cast<const uint16_t*>(v_centroids);
            a.scale_log2e = scale * 1.4426950408889634f;
            a.batch = batch;
            a.n_q_heads = n_q_heads;
            a.t = c.t;
            a.map = map;
            a.seq_lens = seq_lens;
            a.seq_len_shift = m - 1 - j;        // token j of sequence n sees max(seq_lens[n], m) - (m - 1 - j) tokens
            a.seq_len_floor = j + 1;
            a.xk_new = a.xv_new = nullptr;
            a.x_new_stride = 0;
            a.tiles_per_split = c.tiles;
            a.n_split = c.n_split;
            a.partials = static_cast<float*>(workspace);
            a.f = f;
            if ((st = launch_decode(a, static_cast<hipStream_t>(stream))) != CQ_OK) return st;
        }
        return CQ_OK;
    }
    const int tiles = tokens_per_split ? tokens_per_split / kTileTokens : chunk_tiles_per_split(f, batch, n_q_heads, m, t);
    const int n_tiles = (t + kTileTokens - 1) / kTileTokens;
    const int n_split = (n_tiles + tiles - 1) / tiles;
    const size_t rows = (size_t)batch * m * n_q_heads;
    if (n_split > 1) {
        if (!workspace) return CQ_ERR_INVALID_ARG;
        if (workspace_bytes < sizeof(float) * rows * n_split * (f.head_dim + kPartialHeader)) return CQ_ERR_WORKSPACE_TOO_SMALL;
    }
    const int qper = n_q_heads / f.n_kv_heads;
    const int rpw = chunk_rows_per_workgroup(m * qper);
    const int64_t row_blocks = ((int64_t)m * qper + rpw - 1) / rpw;
    if ((int64_t)batch * f.n_kv_heads * row_blocks * n_split > 0x7fffffffLL || rows * n_split > 0x7fffffffULL)
        return CQ_ERR_INVALID_ARG;
    ChunkArgs a;
    a.q = static_cast<const uint16_t*>(q);
    a.k_codes = static_cast<const uint8_t*>(k_codes);
    a.v_codes = static_cast<const uint8_t*>(v_codes);
    a.k_centroids = static_cast<const uint16_t*>(k_centroids);
    a.v_centroids = static_cast<const uint16_t*>(v_centroids);
    a.scale_log2e = scale * 1.4426950408889634f;
    a.batch = batch;
    a.m = m;
    a.n_q_heads = n_q_heads;
    a.t = t;
    a.map = map;
    a.seq_lens = seq_lens;
    a.tiles_per_split = tiles;
    a.n_split = n_split;
    a.partials = static_cast<float*>(workspace);
    a.out = static_cast<uint16_t*>(out);
    a.rope_tile_tab = static_cast<const float2*>(rope_table);
    a.rope_lane_tab = rope ? a.rope_tile_tab + (size_t)(rope_positions / kTileTokens) * 64 : nullptr;
    a.f = f;
    return launch_chunk_attention(a, static_cast<hipStream_t>(stream));
}

}  // namespace

int32_t cq_chunk_default_split(const cq_format* fmt, int32_t batch, int32_t n_q_heads, int32_t m, int32_t t)
{
    Derived f;
    if (derive(fmt, &f) != CQ_OK || f.head_dim != 128) return 0;
    if (batch <= 0 || n_q_heads <= 0 || n_q_heads % f.n_kv_heads != 0 || m <= 0 || t < m) return 0;
    if (chunk_by_token(f, batch, n_q_heads, m, t)) return chunk_token_call(f, batch, n_q_heads, m, t, m - 1).tiles * kTileTokens;
    return chunk_tiles_per_split(f, batch, n_q_heads, m, t) * kTileTokens;
}

size_t cq_chunk_workspace_bytes(const cq_format* fmt, int32_t batch, int32_t n_q_heads, int32_t m, int32_t t,
                                int32_t tokens_per_split)
{
    Derived f;
    if (derive(fmt, &f) != CQ_OK || f.head_dim != 128) return 0;
    if (batch <= 0 || n_q_heads <= 0 || n_q_heads % f.n_kv_heads != 0 || m <= 0 || t < m) return 0;
    if (tokens_per_split < 0 || tokens_per_split % kTileTokens != 0) return 0;
    if (tokens_per_split == 0 && chunk_by_token(f, batch, n_q_heads, m, t)) {
        size_t need = 0;
        for (int j = 0; j < m; ++j) need = std::max(need, chunk_token_call(f, batch, n_q_heads, m, t, j).workspace);
        return need;
    }
    const int tiles = tokens_per_split ? tokens_per_split / kTileTokens : chunk_tiles_per_split(f, batch, n_q_heads, m, t);
    const int n_tiles = (t + kTileTokens - 1) / kTileTokens;
    const int n_split = (n_tiles + tiles - 1) / tiles;
    return sizeof(float) * (size_t)batch * m * n_q_heads * n_split * (f.head_dim + kPartialHeader);
}

cq_status cq_chunk_attention(const void* q, const void* k_codes, const void* v_codes,
                             const void* k_centroids, const void* v_centroids, float scale, const cq_format* fmt,
                             int32_t batch, int32_t n_q_heads, int32_t m, int32_t t, int32_t t_cap,
                             const int32_t* seq_lens, int32_t tokens_per_split,
                             void* out, void* workspace, size_t workspace_bytes, void* stream)
{
    return chunk_common(q, k_codes, v_codes, k_centroids, v_centroids, scale, fmt, batch, n_q_heads, m, t, t_cap, nullptr,
                        seq_lens, tokens_per_split, out, workspace, workspace_bytes, stream);
}

cq_status cq_chunk_attention_paged(const void* q, const void* k_pool, const void* v_pool,
                                   const void* k_centroids, const void* v_centroids, float scale, const cq_format* fmt,
                                   int32_t batch, int32_t n_q_heads, int32_t m, int32_t t, const cq_page_table* pages,
                                   const int32_t* seq_lens, int32_t tokens_per_split,
                                   void* out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!pages) return CQ_ERR_INVALID_ARG;
    return chunk_common(q, k_pool, v_pool, k_centroids, v_centroids, scale, fmt, batch, n_q_heads, m, t, 0, pages,
                        seq_lens, tokens_per_split, out, workspace, workspace_bytes, stream);
}

size_t cq_layer_table_bytes(int32_t n_layers)
{
    return n_layers > 0 ? sizeof(LayerPtrs) * (size_t)n_layers : 0;
}

cq_status cq_layer_table_fill(const cq_layer_io* layers, int32_t n_layers, void* table, size_t table_bytes, void* stream)
{
    static_assert(sizeof(cq_layer_io) == sizeof(LayerPtrs), "the device table holds the caller's records as they are");
    if (!layers || n_layers <= 0 || !table || !aligned16(table)) return CQ_ERR_INVALID_ARG;
    if (table_bytes < sizeof(LayerPtrs) * (size_t)n_layers) return CQ_ERR_WORKSPACE_TOO_SMALL;
    for (int32_t l = 0; l < n_layers; ++l) {
        const cq_layer_io& io = layers[l];
        const void* all[] = {io.q, io.x_k_new, io.x_v_new, io.k_codes, io.v_codes, io.k_centroids, io.v_centroids, io.out};
        for (const void* p : all)
            if (!p || !aligned16(p)) return CQ_ERR_INVALID_ARG;
        if (io.k_codes == io.v_codes) return CQ_ERR_INVALID_ARG;
        // two layers may not share a cache or an output (they are written concurrently)
        for (int32_t m = 0; m < l; ++m)
            if (layers[m].k_codes == io.k_codes || layers[m].v_codes == io.v_codes || layers[m].k_codes == io.v_codes ||
                layers[m].v_codes == io.k_codes || layers[m].out == io.out)
                return CQ_ERR_INVALID_ARG;
    }
    // the records travel as kernel arguments (copied at launch: the host array is free again when
    // this returns, and the write is an ordinary kernel on the stream, also under graph capture)
    for (int32_t l0 = 0; l0 < n_layers; l0 += LayerChunk::N) {
        LayerChunk chunk;
        const int32_t cnt = std::min<int32_t>(LayerChunk::N, n_layers - l0);
        std::memcpy(chunk.p, layers + l0, sizeof(LayerPtrs) * (size_t)cnt);
        const cq_status st = launch_layer_table_write(chunk, cnt, static_cast<LayerPtrs*>(table) + l0,
                                                      static_cast<hipStream_t>(stream));
        if (st != CQ_OK) return st;
    }
    return CQ_OK;
}

cq_status cq_decode_step_layers(const void* layer_table, int32_t n_layers, int64_t x_row_stride,
                                float scale, const cq_format* fmt,
                                int32_t batch, int32_t n_q_heads, int32_t t, int32_t t_cap,
                                const int32_t* seq_lens, int32_t tokens_per_split,
                                void* workspace, size_t workspace_bytes, void* stream)
{
    if (!layer_table || !aligned16(layer_table) || n_layers <= 0) return CQ_ERR_INVALID_ARG;
    return decode_common(nullptr, nullptr, nullptr, x_row_stride, nullptr, nullptr, nullptr, nullptr, scale, fmt, batch,
                         n_q_heads, t, t_cap, nullptr, seq_lens, tokens_per_split, nullptr, workspace, workspace_bytes,
                         stream, true, nullptr, 0, static_cast<const LayerPtrs*>(layer_table), n_layers);
}

size_t cq_rope_table_bytes(int32_t head_dim, int32_t positions)
{
    if (head_dim != 128 || positions <= 0 || positions % kTileTokens != 0) return 0;
    return sizeof(float) * rope_table_floats(positions);
}

cq_status cq_rope_table(double base, int32_t head_dim, int32_t positions, void* table, size_t table_bytes, void* stream)
{
    if (head_dim != 128) return CQ_ERR_UNSUPPORTED;
    if (positions <= 0 || positions % kTileTokens != 0 || !table || !aligned16(table)) return CQ_ERR_INVALID_ARG;
    if (!(base > 1.0) || !std::isfinite(base)) return CQ_ERR_INVALID_ARG;
    if (table_bytes < sizeof(float) * rope_table_floats(positions)) return CQ_ERR_WORKSPACE_TOO_SMALL;
    return launch_rope_table(base, positions, static_cast<float*>(table), static_cast<hipStream_t>(stream));
}

int32_t cq_decode_rope_default_split(const cq_format* fmt, int32_t batch, int32_t n_q_heads, int32_t t)
{
    Derived f;
    if (derive(fmt, &f) != CQ_OK || f.head_dim != 128 || batch <= 0 || n_q_heads <= 0 || t <= 0) return 0;
    return rope_default_tiles_per_split(f, batch, n_q_heads, t) * kTileTokens;
}

cq_status cq_decode_attention_rope(const void* q, const void* k_codes, const void* v_codes,
                                   const void* k_centroids, const void* v_centroids,
                                   float scale, const cq_format* fmt,
                                   int32_t batch, int32_t n_q_heads, int32_t t, int32_t t_cap,
                                   const int32_t* seq_lens, int32_t tokens_per_split,
                                   const void* rope_table, int32_t rope_positions,
                                   void* out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (rope_positions <= 0) return CQ_ERR_INVALID_ARG;
    return decode_common(q, nullptr, nullptr, 0, k_codes, v_codes, k_centroids, v_centroids, scale, fmt, batch,
                         n_q_heads, t, t_cap, nullptr, seq_lens, tokens_per_split, out, workspace, workspace_bytes, stream,
                         false, rope_table, rope_positions);
}

cq_status cq_decode_step_rope(const void* q, const void* x_k_new, const void* x_v_new, int64_t x_row_stride,
                              void* k_codes, void* v_codes,
                              const void* k_centroids, const void* v_centroids,
                              float scale, const cq_format* fmt,
                              int32_t batch, int32_t n_q_heads, int32_t t, int32_t t_cap,
                              const int32_t* seq_lens, int32_t tokens_per_split,
                              const void* rope_table, int32_t rope_positions,
                              void* out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (rope_positions <= 0) return CQ_ERR_INVALID_ARG;
    return decode_common(q, x_k_new, x_v_new, x_row_stride, k_codes, v_codes, k_centroids, v_centroids, scale, fmt,
                         batch, n_q_heads, t, t_cap, nullptr, seq_lens, tokens_per_split, out, workspace, workspace_bytes,
                         stream, true, rope_table, rope_positions);
}

cq_status cq_decode_step_rope_paged(const void* q, const void* x_k_new, const void* x_v_new, int64_t x_row_stride,
                                    void* k_pool, void* v_pool,
                                    const void* k_centroids, const void* v_centroids,
                                    float scale, const cq_format* fmt,
                                    int32_t batch, int32_t n_q_heads, int32_t t, const cq_page_table* pages,
                                    const int32_t* seq_lens, int32_t tokens_per_split,
                                    const void* rope_table, int32_t rope_positions,
                                    void* out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!pages || rope_positions <= 0) return CQ_ERR_INVALID_ARG;
    return decode_common(q, x_k_new, x_v_new, x_row_stride, k_pool, v_pool, k_centroids, v_centroids, scale, fmt,
                         batch, n_q_heads, t, 0, pages, seq_lens, tokens_per_split, out, workspace, workspace_bytes,
                         stream, true, rope_table, rope_positions);
}

namespace {

// Chunks of one or two query tokens over pre-RoPE keys go through the single-token kernel (one
// launch per token), as long as the caller leaves the context split to the library.
bool chunk_rope_by_token(int m, int tokens_per_split) { return tokens_per_split == 0 && m <= 2; }

// split (tiles) and workspace need of query token j of a chunk over pre-RoPE keys
TokenCall chunk_rope_token_call(const Derived& f, int batch, int n_q_heads, int m, int t, int j, int tokens_per_split)
{
    TokenCall c;
    c.t = t - (m - 1 - j);
    c.tiles = tokens_per_split ? tokens_per_split / kTileTokens
                               : rope_default_tiles_per_split(f, batch, n_q_heads, c.t);
    const int n_tiles = (c.t + kTileTokens - 1) / kTileTokens;
    c.n_split = (n_tiles + c.tiles - 1) / c.tiles;
    c.workspace = sizeof(float) * (size_t)batch * n_q_heads * c.n_split * (f.head_dim + kPartialHeader);
    return c;
}

cq_status chunk_rope_common(const void* q, const void* k_codes, const void* v_codes,
                            const void* k_centroids, const void* v_centroids, float scale, const cq_format* fmt,
                            int32_t batch, int32_t n_q_heads, int32_t m, int32_t t, int32_t t_cap, const cq_page_table* pages,
                            const int32_t* seq_lens, int32_t tokens_per_split,
                            const void* rope_table, int32_t rope_positions,
                            void* out, void* workspace, size_t workspace_bytes, void* stream)
{
    Derived f;
    const cq_status st0 = derive(fmt, &f);
    if (st0 != CQ_OK) return st0;
    if (f.head_dim != 128) return CQ_ERR_UNSUPPORTED;
    if (!q || !out || batch <= 0 || n_q_heads <= 0 || n_q_heads % f.n_kv_heads != 0) return CQ_ERR_INVALID_ARG;
    if (m <= 0 || t < m || rope_positions <= 0) return CQ_ERR_INVALID_ARG;
    if (tokens_per_split < 0 || tokens_per_split % kTileTokens != 0) return CQ_ERR_INVALID_ARG;
    // chunks of more than two tokens (or with a split of the caller's): the matrix-core kernel, which
    // rotates each dequantised key tile once for all query rows
    if (!chunk_rope_by_token(m, tokens_per_split))
        return chunk_common(q, k_codes, v_codes, k_centroids, v_centroids, scale, fmt, batch, n_q_heads, m, t, t_cap, pages,
                            seq_lens, tokens_per_split, out, workspace, workspace_bytes, stream, rope_table, rope_positions);
    // all tokens are checked before the first one is launched
    for (int j = 0; j < m; ++j)
        if (workspace_bytes < chunk_rope_token_call(f, batch, n_q_heads, m, t, j, tokens_per_split).workspace)
            return CQ_ERR_WORKSPACE_TOO_SMALL;
    const int64_t row = (int64_t)n_q_heads * f.head_dim;
    for (int j = 0; j < m; ++j) {               // (in stream order: the calls share the workspace)
        const TokenView view{m * row, m * row, m - 1 - j, j + 1};
        const cq_status st = decode_common(static_cast<const uint16_t*>(q) + j * row, nullptr, nullptr, 0, k_codes, v_codes,
                                           k_centroids, v_centroids, scale, fmt, batch, n_q_heads, t - (m - 1 - j), t_cap, pages,
                                           seq_lens, tokens_per_split, static_cast<uint16_t*>(out) + j * row, workspace,
                                           workspace_bytes, stream, false, rope_table, rope_positions, nullptr, 1, &view);
        if (st != CQ_OK) return st;
    }
    return CQ_OK;
}

}  // namespace

size_t cq_chunk_rope_workspace_bytes(const cq_format* fmt, int32_t batch, int32_t n_q_heads, int32_t m, int32_t t,
                                     int32_t tokens_per_split)
{
    Derived f;
    if (derive(fmt, &f) != CQ_OK || f.head_dim != 128) return 0;
    if (batch <= 0 || n_q_heads <= 0 || n_q_heads % f.n_kv_heads != 0 || m <= 0 || t < m) return 0;
    if (tokens_per_split < 0 || tokens_per_split % kTileTokens != 0) return 0;
    if (!chunk_rope_by_token(m, tokens_per_split)) {
        const int tiles = tokens_per_split ? tokens_per_split / kTileTokens : chunk_tiles_per_split(f, batch, n_q_heads, m, t);
        const int n_tiles = (t + kTileTokens - 1) / kTileTokens;
        const int n_split = (n_tiles + tiles - 1) / tiles;
        return sizeof(float) * (size_t)batch * m * n_q_heads * n_split * (f.head_dim + kPartialHeader);
    }
    size_t need = 0;
    for (int j = 0; j < m; ++j) need = std::max(need, chunk_rope_token_call(f, batch, n_q_heads, m, t, j, tokens_per_split).workspace);
    return need;
}

cq_status cq_chunk_attention_rope(const void* q, const void* k_codes, const void* v_codes,
                                  const void* k_centroids, const void* v_centroids, float scale, const cq_format* fmt,
                                  int32_t batch, int32_t n_q_heads, int32_t m, int32_t t, int32_t t_cap,
                                  const int32_t* seq_lens, int32_t tokens_per_split,
                                  const void* rope_table, int32_t rope_positions,
                                  void* out, void* workspace, size_t workspace_bytes, void* stream)
{
    return chunk_rope_common(q, k_codes, v_codes, k_centroids, v_centroids, scale, fmt, batch, n_q_heads, m, t, t_cap, nullptr,
                             seq_lens, tokens_per_split, rope_table, rope_positions, out, workspace, workspace_bytes, stream);
}

cq_status cq_chunk_attention_rope_paged(const void* q, const void* k_pool, const void* v_pool,
                                        const void* k_centroids, const void* v_centroids, float scale, const cq_format* fmt,
                                        int32_t batch, int32_t n_q_heads, int32_t m, int32_t t, const cq_page_table* pages,
                                        const int32_t* seq_lens, int32_t tokens_per_split,
                                        const void* rope_table, int32_t rope_positions,
                                        void* out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!pages) return CQ_ERR_INVALID_ARG;
    return chunk_rope_common(q, k_pool, v_pool, k_centroids, v_centroids, scale, fmt, batch, n_q_heads, m, t, 0, pages,
                             seq_lens, tokens_per_split, rope_table, rope_positions, out, workspace, workspace_bytes, stream);
}

cq_status cq_decode_attention_rope_paged(const void* q, const void* k_pool, const void* v_pool,
                                         const void* k_centroids, const void* v_centroids,
                                         float scale, const cq_format* fmt,
                                         int32_t batch, int32_t n_q_heads, int32_t t, const cq_page_table* pages,
                                         const int32_t* seq_lens, int32_t tokens_per_split,
                                         const void* rope_table, int32_t rope_positions,
                                         void* out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!pages || rope_positions <= 0) return CQ_ERR_INVALID_ARG;
    return decode_common(q, nullptr, nullptr, 0, k_pool, v_pool, k_centroids, v_centroids, scale, fmt, batch,
                         n_q_heads, t, 0, pages, seq_lens, tokens_per_split, out, workspace, workspace_bytes, stream,
                         false, rope_table, rope_positions);
}

}  // extern "C"

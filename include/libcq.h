/*
 * libcq -- Coupled Quantization (CQ) KV-cache hot path for AMD MI355X (gfx950).
 *
 * Two operations, both defined by the CQ paper (arXiv 2405.03917):
 *
 *   cq_encode            Section 3.2: the channels of a key or value embedding are cut into
 *                        non-overlapping groups of c contiguous channels; every group owns a
 *                        codebook of 2^b c-dimensional centroids and is stored as the b-bit index
 *                        of its nearest centroid in L2 distance (the map "CQ(.)" of Eq. 5).
 *   cq_decode_attention  Section 2.1, Eq. 1: attention of one new token over all cached tokens,
 *                        out = [v_1..v_t] softmax([k_1..k_t]^T q), where k_i, v_i are the centroids
 *                        selected by the cached codes.  The library never materialises k_i / v_i:
 *                        by linearity q.k_i is a sum over groups of (q_g . centroid) looked up by
 *                        code, and sum_i p_i v_i is regrouped by code; both are exact rewrites of
 *                        Eq. 1.
 *
 * Conventions
 *   - plain C ABI; no C++ or framework types cross it;
 *   - every data pointer is a DEVICE pointer owned by the caller, 16-byte aligned; the library
 *     allocates no device memory, keeps no state and never synchronises;
 *   - work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default stream);
 *   - every call validates its arguments on the host before touching the GPU and returns a
 *     cq_status; nothing is launched unless the status is CQ_OK;
 *   - fp16 means IEEE-754 binary16.  Inputs must be finite.
 *
 * Where the paper is silent this library takes these readings: ties in the nearest-centroid
 * search go to the lowest index; the softmax scale is an explicit argument (Eq. 1 has none);
 * query head h reads KV head h / (n_q_heads / n_kv_heads); in cq_decode_attention and
 * cq_decode_step the stored key is the key the query is dotted with (no positional rotation);
 * the *_rope calls are for caches of keys quantized before the rotary position embedding and
 * rotate each key to its position.
 *
 * Packed code cache (the paper fixes only its density, b / c bits per stored number -- the
 * "Bits Per FPN" column of Table 1; the arrangement below is this library's):
 *   - one stream per (sequence n, KV head h), streams ordered [n][h];
 *   - a stream is t_cap / 64 tiles of 64 tokens (t_cap is a multiple of 64); a tile holds
 *     64 * Gh * b / 8 bytes, Gh = head_dim / c groups per head;
 *   - b = 8: a tile is Gh / 16 planes of 64 x 16 bytes.  Byte w of token u's 16 bytes in plane p
 *     is slot s = 16 p + w and holds the code of group (s + u) mod Gh of that head.  (The
 *     per-token rotation makes the 64 tokens of a tile touch 64 different lookup-table
 *     columns at every step of the decode kernel.)
 *   - b = 10 (Gh = 16 only): a 64 x 16-byte plane with the low 8 bits of the code of each slot
 *     (same rotation), then a 64 x 4-byte plane with one little-endian uint32 per token whose
 *     bits [2 s + 1 : 2 s] are the high two bits of the code in slot s.
 *   Supported formats: b = 8 with Gh in {16, 32, 64}; b = 10 with Gh = 16; b = 2, 4 through their
 *   fused b = 8 format (see cq_fused_format).
 */
#ifndef LIBCQ_H
#define LIBCQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define CQ_API __attribute__((visibility("default")))
#else
#define CQ_API
#endif

typedef enum cq_status {
    CQ_OK = 0,
    CQ_ERR_INVALID_ARG = 1,          /* null pointer, non-positive size, inconsistent shapes */
    CQ_ERR_UNSUPPORTED = 2,          /* a (c, b, head_dim) with no kernel */
    CQ_ERR_WORKSPACE_TOO_SMALL = 3,
    CQ_ERR_HIP = 4                   /* the HIP runtime refused a launch */
} cq_status;

/* CQ-<c>c<b>b of Section 3.2, plus the shape of the KV embedding it applies to. */
typedef struct cq_format {
    int32_t c;            /* channels per coupled group; divides head_dim */
    int32_t b;            /* bits per code; 2^b centroids per group */
    int32_t head_dim;     /* channels of one head */
    int32_t n_kv_heads;   /* KV heads; D = n_kv_heads * head_dim channels, G = D / c groups */
} cq_format;

#define CQ_TILE_TOKENS 64
/* size of the library's own scratch array (per GPU), used by cq_decode_attention_static only */
#define CQ_STATIC_SCRATCH_BYTES (4u << 20)

/* Library version, major * 10000 + minor * 100 + patch. */
CQ_API int32_t cq_version(void);

/* Static string naming a status code. */
CQ_API const char *cq_status_string(cq_status status);

/* CQ_OK if the format has kernels, else CQ_ERR_INVALID_ARG / CQ_ERR_UNSUPPORTED.  Host only. */
CQ_API cq_status cq_format_check(const cq_format *fmt);

/* Bytes of packed codes of one token of one KV head: (head_dim / c) * b / 8
 * (16 / 32 / 64 / 20 for CQ-8c8b / 4c8b / 2c8b / 8c10b at head_dim 128).  0 on a bad format. */
CQ_API size_t cq_code_bytes_per_token_head(const cq_format *fmt);

/* Bytes of one packed cache (K or V of one layer) for `batch` sequences of capacity t_cap
 * tokens (multiple of 64).  0 on bad arguments. */
CQ_API size_t cq_cache_bytes(const cq_format *fmt, int32_t batch, int32_t t_cap);

/*
 * cq_encode -- Section 3.2 of the paper (nearest centroid per channel group), packed store.
 *
 *   x               device, fp16 [batch][t_new][D]; element strides x_batch_stride and
 *                   x_row_stride (>= D) are given in fp16 elements; rows 16-byte aligned
 *   centroids       device, fp16 [G][2^b][c]
 *   codes           device, packed cache of cq_cache_bytes(fmt, batch, t_cap) bytes; the codes of
 *                   token t of sequence n are written at cache position t_offset + t; other
 *                   positions are left untouched
 *   Distances are sum_i (x_i - centroid_i)^2 evaluated in fp32 in channel order; the lowest
 *   index wins ties.
 * Errors: CQ_ERR_INVALID_ARG for null pointers, batch/t_new <= 0, batch > 32767, t_cap not a multiple of 64,
 * t_offset < 0 or t_offset + t_new > t_cap, strides too small or misaligned;
 * CQ_ERR_UNSUPPORTED for a format without kernels; CQ_ERR_HIP if a launch fails.
 */
CQ_API cq_status cq_encode(const void *x, int64_t x_batch_stride, int64_t x_row_stride,
                    const void *centroids, const cq_format *fmt,
                    int32_t batch, int32_t t_new,
                    void *codes, int32_t t_offset, int32_t t_cap,
                    void *stream);

/*
 * cq_encode_kv -- cq_encode of a key tensor and a value tensor of the same shape and strides in
 * ONE launch (a decode step encodes a handful of rows of each: two launches would cost more than
 * the work).  Arguments as for cq_encode, per tensor; k_codes and v_codes must differ.  The result
 * is identical to two cq_encode calls.
 */
CQ_API cq_status cq_encode_kv(const void *x_k, const void *x_v, int64_t x_batch_stride, int64_t x_row_stride,
                       const void *k_centroids, const void *v_centroids, const cq_format *fmt,
                       int32_t batch, int32_t t_new,
                       void *k_codes, void *v_codes, int32_t t_offset, int32_t t_cap,
                       void *stream);

/* Tokens per context split the library would pick for this problem (a multiple of 64). */
CQ_API int32_t cq_decode_default_split(const cq_format *fmt, int32_t batch, int32_t n_q_heads, int32_t t);

/* Workspace bytes cq_decode_attention needs for up to t cached tokens when run with
 * tokens_per_split (0 = the library's default).  0 on bad arguments. */
CQ_API size_t cq_decode_workspace_bytes(const cq_format *fmt, int32_t batch, int32_t n_q_heads,
                                 int32_t t, int32_t tokens_per_split);

/*
 * cq_decode_attention -- Eq. 1 of the paper for one query token per sequence, computed from
 * packed codes (see the top of this file for the rewrite used).
 *
 *   q                 device, fp16 [batch][n_q_heads][head_dim]
 *   k_codes, v_codes  device, packed caches (layout above) with capacity t_cap
 *   k_centroids, v_centroids   device, fp16 [G][2^b][c]
 *   scale             multiplies q.k before the softmax (e.g. 1/sqrt(head_dim))
 *   t                 cached tokens attended per sequence (positions 0 .. t-1), 1 <= t <= t_cap
 *   seq_lens          device int32 [batch] or NULL; if given, sequence n attends positions
 *                     0 .. seq_lens[n]-1; values must lie in [1, t] (not checked on the host;
 *                     the kernels clamp them into that range)
 *   tokens_per_split  0 = library default; otherwise a multiple of 64: each workgroup handles
 *                     that many tokens of one (sequence, query head) and a second kernel merges
 *                     the partial softmax results (exact rescaling by the running maximum);
 *                     CQ-8c8b / 4c8b: any length (a workgroup walks its split in chunks of
 *                     8192 tokens with one score table); CQ-2c8b: at most 8192 tokens,
 *                     CQ-8c10b: at most 16384 (one chunk, whose scores stay in registers)
 *   out               device, fp16 [batch][n_q_heads][head_dim]
 *   workspace         device scratch of at least cq_decode_workspace_bytes(...) bytes; contents
 *                     need not be initialised and are overwritten
 *   Arithmetic: fp32 lookup tables, scores, softmax and accumulation; the result is rounded to
 *   fp16 once (round to nearest even).
 * Errors: as cq_encode, plus CQ_ERR_INVALID_ARG when n_q_heads is not a multiple of
 * n_kv_heads or tokens_per_split is not a positive multiple of 64 (or too large for the
 * kernel's on-chip score buffer), and CQ_ERR_WORKSPACE_TOO_SMALL.
 */
CQ_API cq_status cq_decode_attention(const void *q,
                              const void *k_codes, const void *v_codes,
                              const void *k_centroids, const void *v_centroids,
                              float scale, const cq_format *fmt,
                              int32_t batch, int32_t n_q_heads, int32_t t, int32_t t_cap,
                              const int32_t *seq_lens, int32_t tokens_per_split,
                              void *out, void *workspace, size_t workspace_bytes,
                              void *stream);

/*
 * cq_decode_attention_static -- cq_decode_attention for callers that cannot allocate device
 * memory and have no workspace to pass: code under HIP graph capture, tight serving loops,
 * harnesses that forbid allocation.  Same arguments, kernels and results (bit for bit) as
 * cq_decode_attention, minus the workspace: the partial results of the context splits live in
 * an array of CQ_STATIC_SCRATCH_BYTES (4 MiB) inside the library, which each GPU the library
 * runs on holds until the process ends.  The call allocates and frees nothing; the first call
 * on a device looks the array's address up once.
 *   Limit: batch * n_q_heads * n_split * (2 + head_dim) * 4 bytes must fit the array (8065 rows
 *   of (sequence, query head, split) at head_dim 128), else CQ_ERR_WORKSPACE_TOO_SMALL; a call
 *   with one split uses none of it.
 *   All calls on one GPU share the array: calls that may overlap on a GPU (different streams,
 *   concurrently replayed graphs) race on it and must use cq_decode_attention with workspaces
 *   of their own.  Nothing in the array has to start at zero and no call depends on what an
 *   earlier one left there.
 * Errors: as cq_decode_attention; CQ_ERR_HIP also when the array's address cannot be obtained.
 */
CQ_API cq_status cq_decode_attention_static(const void *q,
                              const void *k_codes, const void *v_codes,
                              const void *k_centroids, const void *v_centroids,
                              float scale, const cq_format *fmt,
                              int32_t batch, int32_t n_q_heads, int32_t t, int32_t t_cap,
                              const int32_t *seq_lens, int32_t tokens_per_split,
                              void *out, void *stream);

/*
 * cq_decode_step -- one fused launch that equals cq_encode_kv of ONE new token per sequence
 * followed by cq_decode_attention over the context that now includes it (Section 3.2, then
 * Eq. 1).  A decode step encodes 2 x batch rows: as separate launches those cost as much as a
 * third of the attention itself, while the attention workgroups hold the codebooks anyway.
 *
 *   x_k_new, x_v_new  device, fp16 [batch][D], row stride x_row_stride (>= D, multiple of 8)
 *   k_codes, v_codes  device, packed caches; the new token's codes are WRITTEN at position
 *                     t - 1 (or seq_lens[n] - 1), all other positions are only read
 *   t                 cached tokens attended per sequence INCLUDING the new one
 *   everything else as in cq_decode_attention.
 * The stored codes and the output are bit-identical to the two-call sequence.
 * Errors: as cq_decode_attention and cq_encode_kv.
 */
CQ_API cq_status cq_decode_step(const void *q, const void *x_k_new, const void *x_v_new, int64_t x_row_stride,
                         void *k_codes, void *v_codes,
                         const void *k_centroids, const void *v_centroids,
                         float scale, const cq_format *fmt,
                         int32_t batch, int32_t n_q_heads, int32_t t, int32_t t_cap,
                         const int32_t *seq_lens, int32_t tokens_per_split,
                         void *out, void *workspace, size_t workspace_bytes,
                         void *stream);

/*
 * Sub-byte formats: CQ-<c>c<b>b with b = 2 or 4 (the low-bit variants of the paper's ablation on
 * the number of coupled channels, Section 4.3 / Figure 4: CQ-1c2b, 2c2b, 1c4b, 2c4b, 4c4b at
 * head_dim 128; density b / c bits per stored number as in Table 1).
 *
 * 8 / b neighbouring groups share one code byte: group i of the byte sits in bits [b i, b i + b).
 * That byte IS a code of the product codebook of those groups -- the 256 concatenations of their
 * centroids -- so a sub-byte cache is, byte for byte, a cache of the fused format
 * CQ-<c 8/b>c8b (cq_fused_format) with the expanded codebook (cq_expand_codebook), and every
 * attention call (cq_decode_attention, the paged, rope and chunk variants) and cq_dequantize
 * take (fused format, expanded codebook) for it; the scores and outputs are those of Eq. 1 over
 * the sub-byte centroids, since a concatenation's dot product is the sum of its parts'.  (The
 * fused decode STEP on the fused format searches the product codebook, where the rounding of
 * one group's distance can decide another group's near tie; append with cq_encode_kv in the
 * sub-byte format instead when the format's own search is wanted bit for bit.)
 *
 * cq_encode, cq_encode_kv, cq_encode_kv_paged, cq_cache_bytes, cq_paged_cache_bytes,
 * cq_code_bytes_per_token_head, cq_format_check, cq_kmeans_workspace_bytes and cq_kmeans_fit
 * accept the sub-byte format itself, with its
 * own codebook fp16 [G][2^b][c]: every group is searched against its own 2^b centroids
 * (squared distance in fp32 in channel order, lowest index on ties), not the product codebook.
 *
 * cq_fused_format     host only; *fused = the format whose layout and decode kernels apply
 *                     (the format itself for b = 8, 10)
 * cq_expand_codebook  centroids fp16 [G][2^b][c] -> fused_centroids fp16 [G b/8][256][8 c/b]
 *                     (device, 16-byte aligned, distinct; written on `stream`); entry j of fused
 *                     group f is the concatenation over i of centroid (j >> b i) mod 2^b of
 *                     group f 8/b + i.  CQ_ERR_INVALID_ARG for b = 8, 10 (nothing to expand).
 */
CQ_API cq_status cq_fused_format(const cq_format *fmt, cq_format *fused);
CQ_API cq_status cq_expand_codebook(const void *centroids, const cq_format *fmt, void *fused_centroids, void *stream);

/*
 * cq_decode_step for several layers in ONE launch (the decode step of a workload whose layers are
 * independent of each other, as in a benchmark over stored per-layer inputs; in a model the
 * query of layer l + 1 depends on layer l's output and the layers have to be launched one by
 * one).  Without the drain and ramp-up between per-layer launches, workgroups of the next layer
 * start as soon as a compute unit is free.
 *
 * The per-layer tensors are named by a table in device memory, written once by
 * cq_layer_table_fill from a host array of cq_layer_io records (each pointer: device memory,
 * non-null, 16-byte aligned, with the meaning, shape and ownership of the argument of the same
 * name of cq_decode_step; no two layers may share a cache or an output).  The fill validates what
 * the host can see of them and writes the records with a small kernel on `stream` (they travel
 * as kernel arguments, so the call may also be captured into a graph); the host array may be reused when
 * it returns.  The table (cq_layer_table_bytes(n_layers) bytes, 16-byte aligned) stays owned by
 * the caller and is only read by cq_decode_step_layers, which trusts its contents.
 *
 * cq_decode_step_layers: all layers share format, batch, head counts, t, t_cap, seq_lens, scale,
 * x_row_stride and the split; workspace: n_layers * cq_decode_workspace_bytes(...) bytes.
 * Results per layer are bit-identical to n_layers calls of cq_decode_step.
 * Errors: as cq_decode_step (the per-layer pointers are checked by cq_layer_table_fill instead).
 */
typedef struct cq_layer_io {
    const void *q;
    const void *x_k_new;
    const void *x_v_new;
    void *k_codes;
    void *v_codes;
    const void *k_centroids;
    const void *v_centroids;
    void *out;
} cq_layer_io;

CQ_API size_t cq_layer_table_bytes(int32_t n_layers);
CQ_API cq_status cq_layer_table_fill(const cq_layer_io *layers, int32_t n_layers,
                              void *table, size_t table_bytes, void *stream);
CQ_API cq_status cq_decode_step_layers(const void *layer_table, int32_t n_layers, int64_t x_row_stride,
                                float scale, const cq_format *fmt,
                                int32_t batch, int32_t n_q_heads, int32_t t, int32_t t_cap,
                                const int32_t *seq_lens, int32_t tokens_per_split,
                                void *workspace, size_t workspace_bytes, void *stream);

/*
 * Paged caches.  Instead of t_cap contiguous positions per sequence, the codes live in a pool
 * of pages; a page is the 64-token tile of EVERY KV head ([n_kv_heads][tile bytes], tile bytes =
 * 64 * cq_code_bytes_per_token_head), and a block table names the page of each tile of each
 * sequence: block_table[n * row_stride + i] = page of tokens 64 i .. 64 i + 63 of sequence n, for
 * i < max_tiles (device memory, int32; the K pool and the V pool share the table).  Entries are
 * clamped to [0, n_pages) by the kernels.  The *_paged calls take the same arguments as their
 * contiguous namesakes with (pool, cq_page_table) in the place of (cache, t_cap); capacity is
 * max_tiles * 64 tokens per sequence; results are identical to the contiguous calls on the same
 * logical contents.
 */
typedef struct cq_page_table {
    int32_t n_pages;               /* pages in each pool */
    int32_t max_tiles;             /* valid entries per sequence */
    int64_t row_stride;            /* entries between sequences (>= max_tiles) */
    const int32_t *block_table;    /* device */
} cq_page_table;

/* Bytes of one pool (K or V of one layer) of n_pages pages.  0 on bad arguments. */
CQ_API size_t cq_paged_cache_bytes(const cq_format *fmt, int32_t n_pages);
CQ_API cq_status cq_encode_kv_paged(const void *x_k, const void *x_v, int64_t x_batch_stride, int64_t x_row_stride,
                             const void *k_centroids, const void *v_centroids, const cq_format *fmt,
                             int32_t batch, int32_t t_new,
                             void *k_pool, void *v_pool, const cq_page_table *pages, int32_t t_offset, void *stream);
CQ_API cq_status cq_decode_attention_paged(const void *q, const void *k_pool, const void *v_pool,
                                    const void *k_centroids, const void *v_centroids,
                                    float scale, const cq_format *fmt,
                                    int32_t batch, int32_t n_q_heads, int32_t t, const cq_page_table *pages,
                                    const int32_t *seq_lens, int32_t tokens_per_split,
                                    void *out, void *workspace, size_t workspace_bytes, void *stream);
CQ_API cq_status cq_decode_step_paged(const void *q, const void *x_k_new, const void *x_v_new, int64_t x_row_stride,
                               void *k_pool, void *v_pool,
                               const void *k_centroids, const void *v_centroids,
                               float scale, const cq_format *fmt,
                               int32_t batch, int32_t n_q_heads, int32_t t, const cq_page_table *pages,
                               const int32_t *seq_lens, int32_t tokens_per_split,
                               void *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * cq_chunk_attention -- Eq. 1 of the paper for the LAST m tokens of each sequence at once, with
 * the causal restriction that makes it m single-token attentions: query token j sits at position
 * t_n - m + j (t_n = seq_lens[n], default t) and attends to the cached tokens 0 .. t_n - m + j.
 * The caches already hold the codes of the m tokens (cq_encode_kv first).  Use: a prefill chunk
 * after the first, or the verification of m speculated tokens.
 *
 *   q                 device, fp16 [batch][m][n_q_heads][head_dim]
 *   out               device, fp16 [batch][m][n_q_heads][head_dim]
 *   m                 query tokens per sequence, 1 <= m <= seq_lens[n] <= t <= t_cap
 *   tokens_per_split  0 = cq_chunk_default_split(...); otherwise a multiple of 64: the context is
 *                     cut into pieces of this many tokens, each handled by its own workgroups
 *   workspace         device, cq_chunk_workspace_bytes(...) bytes (may be null when that is 0 or
 *                     the context is not split)
 *   everything else as in cq_decode_attention; stored keys are the keys the queries are dotted
 *   with (no positional rotation).
 * The contraction runs on the matrix cores in fp16 with fp32 accumulation: scores are exact
 * products summed in fp32; probabilities enter the value product as two fp16 numbers (22 bits).
 * Short chunks with tokens_per_split = 0 (m <= 2; m <= 8 / (query heads per KV head) on large
 * batches) are instead served token by token by the kernel of cq_decode_attention, m launches
 * in stream order, which is faster there; the results are then bit-identical to m calls of
 * cq_decode_attention with the contexts of the m tokens.  cq_chunk_default_split and
 * cq_chunk_workspace_bytes describe whichever path the library takes; an explicit
 * tokens_per_split always runs the matrix-core kernel.
 * Formats: those of cq_decode_attention (b = 8, 10 at head_dim 128).
 * Errors: as cq_decode_attention; CQ_ERR_INVALID_ARG also for m <= 0 or m > t.
 */
CQ_API int32_t cq_chunk_default_split(const cq_format *fmt, int32_t batch, int32_t n_q_heads, int32_t m, int32_t t);
CQ_API size_t cq_chunk_workspace_bytes(const cq_format *fmt, int32_t batch, int32_t n_q_heads, int32_t m, int32_t t,
                                int32_t tokens_per_split);
CQ_API cq_status cq_chunk_attention(const void *q, const void *k_codes, const void *v_codes,
                             const void *k_centroids, const void *v_centroids, float scale, const cq_format *fmt,
                             int32_t batch, int32_t n_q_heads, int32_t m, int32_t t, int32_t t_cap,
                             const int32_t *seq_lens, int32_t tokens_per_split,
                             void *out, void *workspace, size_t workspace_bytes, void *stream);
CQ_API cq_status cq_chunk_attention_paged(const void *q, const void *k_pool, const void *v_pool,
                                   const void *k_centroids, const void *v_centroids, float scale, const cq_format *fmt,
                                   int32_t batch, int32_t n_q_heads, int32_t m, int32_t t, const cq_page_table *pages,
                                   const int32_t *seq_lens, int32_t tokens_per_split,
                                   void *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Keys cached BEFORE the rotary position embedding.  Section 3.2 quantizes key activations
 * before RoPE (the position-dependent rotation would otherwise spread each channel pair over a
 * circle and cost codebook resolution), and Eq. 1 counts the positional encoding into the
 * attention function; the cache then holds codes of un-rotated keys and attention has to apply
 * the rotation of position t to the key of token t.  The paper cites RoPE without restating it;
 * the form implemented is that of the models it evaluates: for head_dim d, channels i and
 * i + d/2 (i < d/2) of a head form a pair, and the key at position t enters the score as
 *     k'_i       = k_i cos(t th_i) - k_{i+d/2} sin(t th_i)
 *     k'_{i+d/2} = k_{i+d/2} cos(t th_i) + k_i sin(t th_i),      th_i = base^(-2 i / d).
 * The query is passed already rotated (it is one row; the caller's projection kernel rotates
 * it).  Token u of the cache has position u.  Values are not rotated.
 *
 * cq_rope_table fills the trigonometric table the attention call reads (fp64 arithmetic,
 * rounded once to fp32): one call per (base, longest context), reused by every layer and step.
 *   head_dim       128 (others: CQ_ERR_UNSUPPORTED)
 *   positions      table covers token positions [0, positions); a positive multiple of 64
 *   table          device, 16-byte aligned, cq_rope_table_bytes(head_dim, positions) bytes,
 *                  written asynchronously on `stream`; owned by the caller
 * cq_rope_table_bytes returns 0 on bad arguments.
 *
 * cq_decode_attention_rope[_paged]: as cq_decode_attention[_paged], plus
 *   q              rotated to its own position, otherwise as before
 *   rope_table     device, as written by cq_rope_table(base, 128, rope_positions, ...)
 *   rope_positions must be >= t
 *   tokens_per_split  0 = cq_decode_rope_default_split(...); at most 16384.  With two or more query
 *                     heads per KV head and byte codes, splits of at most 5632 tokens (the default
 *                     then) run the kernel that rotates each key once for four query heads;
 *                     longer ones the kernel that serves one query head per workgroup
 * cq_decode_step_rope[_paged]: the fused decode step (cq_decode_step[_paged]) for such caches:
 * the new key row is passed BEFORE the rotation (it is quantized as it is; position t - 1, or
 * seq_lens[n] - 1, rotates it like every cached key), the new value row as always; same
 * arguments as cq_decode_step plus the table, same results as cq_encode_kv followed by
 * cq_decode_attention_rope, bit for bit.
 * Formats: head_dim 128.  For b = 8 (CQ-8c8b, CQ-4c8b, CQ-2c8b) the kernel keeps a head's key
 * centroids (64 KiB) on chip; CQ-8c10b (256 KiB per head) reads them from global memory.
 * Workspace size: cq_decode_workspace_bytes with the tokens_per_split actually used.
 * Errors: as cq_decode_attention; CQ_ERR_INVALID_ARG also for a missing or too short table.
 */
CQ_API size_t cq_rope_table_bytes(int32_t head_dim, int32_t positions);
CQ_API cq_status cq_rope_table(double base, int32_t head_dim, int32_t positions,
                        void *table, size_t table_bytes, void *stream);
CQ_API int32_t cq_decode_rope_default_split(const cq_format *fmt, int32_t batch, int32_t n_q_heads, int32_t t);
CQ_API cq_status cq_decode_attention_rope(const void *q, const void *k_codes, const void *v_codes,
                                   const void *k_centroids, const void *v_centroids,
                                   float scale, const cq_format *fmt,
                                   int32_t batch, int32_t n_q_heads, int32_t t, int32_t t_cap,
                                   const int32_t *seq_lens, int32_t tokens_per_split,
                                   const void *rope_table, int32_t rope_positions,
                                   void *out, void *workspace, size_t workspace_bytes, void *stream);
CQ_API cq_status cq_decode_step_rope(const void *q, const void *x_k_new, const void *x_v_new, int64_t x_row_stride,
                              void *k_codes, void *v_codes,
                              const void *k_centroids, const void *v_centroids,
                              float scale, const cq_format *fmt,
                              int32_t batch, int32_t n_q_heads, int32_t t, int32_t t_cap,
                              const int32_t *seq_lens, int32_t tokens_per_split,
                              const void *rope_table, int32_t rope_positions,
                              void *out, void *workspace, size_t workspace_bytes, void *stream);
CQ_API cq_status cq_decode_step_rope_paged(const void *q, const void *x_k_new, const void *x_v_new, int64_t x_row_stride,
                                    void *k_pool, void *v_pool,
                                    const void *k_centroids, const void *v_centroids,
                                    float scale, const cq_format *fmt,
                                    int32_t batch, int32_t n_q_heads, int32_t t, const cq_page_table *pages,
                                    const int32_t *seq_lens, int32_t tokens_per_split,
                                    const void *rope_table, int32_t rope_positions,
                                    void *out, void *workspace, size_t workspace_bytes, void *stream);
CQ_API cq_status cq_decode_attention_rope_paged(const void *q, const void *k_pool, const void *v_pool,
                                         const void *k_centroids, const void *v_centroids,
                                         float scale, const cq_format *fmt,
                                         int32_t batch, int32_t n_q_heads, int32_t t, const cq_page_table *pages,
                                         const int32_t *seq_lens, int32_t tokens_per_split,
                                         const void *rope_table, int32_t rope_positions,
                                         void *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * cq_chunk_attention_rope[_paged] -- cq_chunk_attention for caches whose keys were quantized
 * before the rotary position embedding (Section 3.2): causal attention of the LAST m tokens of
 * each sequence, query token j (rotated by the caller to its own position t_n - m + j) over the
 * cached tokens 0 .. t_n - m + j.  Chunks of more than two tokens (and any chunk when
 * tokens_per_split is given) run on the matrix cores like cq_chunk_attention: each 64-token tile
 * of keys is dequantised and rotated to its tokens' positions once per (tile, KV head) in fp32,
 * rounded to fp16 and multiplied with all query rows of the workgroup.  With tokens_per_split = 0,
 * chunks of one or two tokens are served token by token by the kernel of
 * cq_decode_attention_rope (m launches in stream order, bit-identical to m calls of it).
 *   q, out            device, fp16 [batch][m][n_q_heads][head_dim]
 *   m                 1 <= m <= seq_lens[n] <= t <= t_cap (t <= rope_positions)
 *   tokens_per_split  0 = library default; otherwise a multiple of 64 (context split of the
 *                     matrix-core kernel, as in cq_chunk_attention)
 *   workspace         device, cq_chunk_rope_workspace_bytes(...) bytes
 *   everything else as in cq_decode_attention_rope.
 * Errors: as cq_decode_attention_rope; CQ_ERR_INVALID_ARG also for m <= 0 or m > t; nothing is
 * launched when the workspace is too small.
 */
CQ_API size_t cq_chunk_rope_workspace_bytes(const cq_format *fmt, int32_t batch, int32_t n_q_heads, int32_t m, int32_t t,
                                     int32_t tokens_per_split);
CQ_API cq_status cq_chunk_attention_rope(const void *q, const void *k_codes, const void *v_codes,
                                  const void *k_centroids, const void *v_centroids, float scale, const cq_format *fmt,
                                  int32_t batch, int32_t n_q_heads, int32_t m, int32_t t, int32_t t_cap,
                                  const int32_t *seq_lens, int32_t tokens_per_split,
                                  const void *rope_table, int32_t rope_positions,
                                  void *out, void *workspace, size_t workspace_bytes, void *stream);
CQ_API cq_status cq_chunk_attention_rope_paged(const void *q, const void *k_pool, const void *v_pool,
                                        const void *k_centroids, const void *v_centroids, float scale, const cq_format *fmt,
                                        int32_t batch, int32_t n_q_heads, int32_t m, int32_t t, const cq_page_table *pages,
                                        const int32_t *seq_lens, int32_t tokens_per_split,
                                        const void *rope_table, int32_t rope_positions,
                                        void *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * cq_dequantize -- the inverse lookup ("dequantization", Section 2.2; CQ(A) of Eq. 5 as values):
 * out[n][t][g c + i] = centroids[g][code(n, t_offset + t, g)][i] for t = 0 .. t_count - 1, bit
 * for bit the stored fp16 centroids.  For callers that need dense keys / values (e.g. a
 * multi-query attention over a coded cache).
 *
 *   codes           device, packed cache (cq_cache_bytes(fmt, batch, t_cap) bytes)
 *   centroids       device, fp16 [G][2^b][c]
 *   out             device, fp16 [batch][t_count][D]; element strides out_batch_stride and
 *                   out_row_stride (>= D, multiples of 8)
 * Errors: as cq_encode.
 */
CQ_API cq_status cq_dequantize(const void *codes, const void *centroids, const cq_format *fmt,
                        int32_t batch, int32_t t_offset, int32_t t_count, int32_t t_cap,
                        void *out, int64_t out_batch_stride, int64_t out_row_stride, void *stream);

/*
 * Centroid learning (Section 3.2 of the paper, "Centroid Learning"): for every channel group an
 * independent k-means run over the tokens of a calibration tensor -- Eq. 5; with `weights`,
 * the weighted objective of Eq. 6 (weighted k-means; the caller supplies the weight of each
 * token and group, e.g. the sum of the squared gradients of the group's channels) -- with
 * k-means++ initialisation and a fixed number of Lloyd iterations (Section 4.3: 100).
 *
 * Every decision is taken in arithmetic that does not depend on processing order (fp32
 * distances with one fused multiply-add per channel in channel order, lowest index on ties;
 * integer weights floor(w 2^kw) with the largest weight of a group in [2^21, 2^22); exact
 * integer sums for the means; k-means++ sampled on integers from the caller's random words), so
 * the result is a function of the inputs alone, bit for bit.
 *
 *   x                 fp16 [n_points][D], row stride x_row_stride (>= D, multiple of 8) elements
 *   weights           fp32 [n_points][G], >= 0, or NULL (all tokens weigh the same); a group whose
 *                     weights are all zero is treated as unweighted
 *   n_points          1 .. CQ_KMEANS_MAX_POINTS
 *   n_iter            Lloyd iterations (>= 0; 0 with rnd: k-means++ only)
 *   rnd               uint64 [G][2^b]: one random word per centre to draw (k-means++), or NULL
 *   init_centroids    fp32 [G][2^b][c] starting centroids, or NULL; exactly one of rnd and
 *                     init_centroids must be given
 *   picks             out, optional (needs rnd): int32 [G][2^b], the tokens chosen by k-means++
 *   centroids         out, optional: fp16 [G][2^b][c], the fp32 result rounded to nearest even --
 *                     the codebook cq_encode and cq_decode_attention take
 *   centroids_f32     out, optional: fp32 [G][2^b][c]; at least one of the two must be given
 *   assignment        out, optional: uint16 [G][n_points], the cluster of every token in the last
 *                     iteration's assignment step (untouched when n_iter = 0)
 *   workspace         at least cq_kmeans_workspace_bytes(fmt, n_points) bytes (0: invalid arguments)
 * All pointers are device pointers, 16-byte aligned.  A cluster that owns no token keeps its
 * centroid.  Errors: CQ_ERR_INVALID_ARG, CQ_ERR_UNSUPPORTED (format), CQ_ERR_WORKSPACE_TOO_SMALL,
 * CQ_ERR_HIP.
 */
#define CQ_KMEANS_MAX_POINTS 524288
CQ_API size_t cq_kmeans_workspace_bytes(const cq_format *fmt, int32_t n_points);
CQ_API cq_status cq_kmeans_fit(const void *x, int64_t x_row_stride, const float *weights, const cq_format *fmt,
                        int32_t n_points, int32_t n_iter, const uint64_t *rnd, const float *init_centroids,
                        int32_t *picks, void *centroids, float *centroids_f32, uint16_t *assignment,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * Measurement aids (no part of the method; benchmarks use them as yardsticks).
 *
 * cq_probe_stream_read  reads `bytes` (multiple of 16) from device memory `src` once, 16 bytes
 *                       per lane with the same non-temporal loads the decode kernel uses, and
 *                       XORs what it read into `sink` (device, at least 8 KiB, any contents).
 * cq_probe_copy         copies `bytes` (multiple of 16) from `src` to `dst` (device, 16-byte
 *                       aligned, not overlapping): a kernel whose HBM traffic is known exactly.
 * cq_probe_mfma         one matrix-core product D = A B exactly as the prefill encode kernel
 *                       issues it (v_mfma_f32_32x32x16_f16 for kdim 16, v_mfma_f32_32x32x8_f16
 *                       for kdim 8; zero accumulator): a fp16 [32][kdim] row-major, b fp16
 *                       [kdim][32] row-major, d fp32 [32][32] row-major, all device.  Tests pin
 *                       the rounding model that the encode kernel's error bound assumes to it.
 * Errors: CQ_ERR_INVALID_ARG for null / misaligned pointers, a size that is zero or not a
 * multiple of 16, or a kdim other than 8 and 16; CQ_ERR_HIP if the launch fails.
 */
CQ_API cq_status cq_probe_stream_read(const void *src, size_t bytes, void *sink, void *stream);
CQ_API cq_status cq_probe_copy(const void *src, void *dst, size_t bytes, void *stream);
CQ_API cq_status cq_probe_mfma(const void *a, const void *b, void *d, int32_t kdim, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LIBCQ_H */

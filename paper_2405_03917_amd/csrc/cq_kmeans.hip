// Centroid learning of CQ (Section 3.2 of the paper, "Centroid Learning"): one independent
// k-means run per channel group (Eq. 5), k-means++ initialisation and a fixed number of Lloyd
// iterations (Section 4.3), optionally weighted per (token, group) as in the Fisher-guided
// objective of Eq. 6 (weighted k-means), for gfx950.
//
// Every decision of the iteration is taken in arithmetic that does not depend on the order in
// which tokens are processed, so that the result is reproducible bit for bit:
//   distance     sum_i (x_i - c_i)^2 in fp32: rounded difference, one fused multiply-add per
//                channel in channel order; x is fp16 widened, c an fp32 centroid
//   assignment   smallest distance, lowest index among equals
//   weights      integers wq = floor(w * 2^kw), the largest weight of a group in [2^21, 2^22)
//                (no weights, or all zero: wq = 1)
//   update       exact integer sums of wq * (x * 2^24), held as S_hi * 2^20 + S_lo in two 64-bit
//                integers, and of wq; centroid = fp32((fp64(S_hi) * 2^20 + fp64(S_lo)) / fp64(W)
//                * 2^-24); a cluster without tokens keeps its centroid
//   k-means++    first centre with probability wq / sum wq, the others with probability
//                proportional to wq * dmin (dmin: fp32 distance to the nearest centre so far),
//                sampled on integers: q = floor(fp64(wq) * fp64(dmin) * 2^kq), kq = 62 -
//                ceil(log2 n) - (exponent of the largest product + 1); r = floor(rnd * sum q /
//                2^64) with the caller's 64-bit random word of the pick; chosen = first token
//                whose inclusive prefix sum of q exceeds r; all products zero: floor(rnd * n / 2^64)
//
// Kernels: prepare (group-major copy of the tokens, integer weights), k-means++ (one workgroup
// per group, K sequential picks), and per Lloyd iteration an assignment kernel (plain fp32 VALU
// search against the group's centroids in LDS) and an update kernel (integer LDS atomics, then
// the new centroids).
#include <hip/hip_runtime.h>

#include <type_traits>

#include "cq_internal.hpp"

namespace cq {
namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

constexpr int kPPThreads = 1024;     // k-means++ workgroup
constexpr int kAssignThreads = 256;
constexpr int kAssignPoints = 2;     // tokens per thread of the assignment kernel
constexpr int kUpdateClusters = 256; // clusters per update workgroup

template <int C>
__device__ __forceinline__ void widen(const uint16_t* p, float (&v)[C])
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
    } else if constexpr (C == 2) {
        const half2_t h = __builtin_bit_cast(half2_t, *reinterpret_cast<const unsigned*>(p));
        v[0] = (float)h.x; v[1] = (float)h.y;
    } else {
        static_assert(C == 1, "channels per group: 1, 2, 4 or 8");
        v[0] = (float)__builtin_bit_cast(_Float16, *p);
    }
}

template <int C>
__device__ __forceinline__ float dist2(const float (&x)[C], const float* c)
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
// prepare
// ------------------------------------------------------------------------------------------
__global__ void kmeans_clear_kernel(unsigned* p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// largest weight of every group (weights are non-negative: their bits order like their values)
__global__ void kmeans_wmax_kernel(const float* w, int n, int G, unsigned* wmax_bits)
{
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= G) return;
    unsigned m = 0;
    for (int i = blockIdx.y; i < n; i += gridDim.y) {
        const unsigned b = __float_as_uint(w[(size_t)i * G + g]);
        m = b > m ? b : m;
    }
    atomicMax(wmax_bits + g, m);
}

// xg[g][i][:] = x[i][g c ..], wq[g][i] = integer weight.  A workgroup moves a tile of 32 tokens x
// 64 groups through LDS so that both sides are read and written in contiguous runs.
constexpr int kPrepTokens = 32, kPrepGroups = 64;

template <int C>
__global__ __launch_bounds__(256) void kmeans_prepare_kernel(const uint16_t* x, int64_t x_stride, const float* w,
                                                             const unsigned* wmax_bits, int n, int G, uint16_t* xg,
                                                             uint32_t* wq)
{
    using unit_t = std::conditional_t<C == 8, uint4, std::conditional_t<C == 4, uint2, std::conditional_t<C == 2, unsigned, uint16_t>>>;
    __shared__ unit_t tile[kPrepTokens][kPrepGroups + 1];
    __shared__ uint32_t wt[kPrepTokens][kPrepGroups + 1];
    const int i0 = blockIdx.x * kPrepTokens, g0 = blockIdx.y * kPrepGroups;
    {
        const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;     // tx: group, ty: token row
        for (int r = ty; r < kPrepTokens; r += 4) {
            const int i = i0 + r, g = g0 + tx;
            if (i < n && g < G) {
                tile[r][tx] = *reinterpret_cast<const unit_t*>(x + (size_t)i * x_stride + (size_t)g * C);
                uint32_t q = 1u;
                const unsigned mb = w ? wmax_bits[g] : 0u;
                if (mb != 0u) {
                    // kw = 21 - floor(log2(wmax)); w * 2^kw is exact in fp64, the conversion truncates
                    const int kw = 21 - ilogbf(__uint_as_float(mb));
                    q = (uint32_t)ldexp((double)w[(size_t)i * G + g], kw);
                }
                wt[r][tx] = q;
            }
        }
    }
    __syncthreads();
    {
        const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;     // tx: token, ty: group row
        for (int r = ty; r < kPrepGroups; r += 8) {
            const int g = g0 + r, i = i0 + tx;
            if (i < n && g < G) {
                *reinterpret_cast<unit_t*>(xg + ((size_t)g * n + i) * C) = tile[tx][r];
                wq[(size_t)g * n + i] = wt[tx][r];
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// k-means++
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ unsigned long long wave_incl_scan_u64(unsigned long long v, int lane)
{
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const unsigned long long up = __shfl_up(v, o);
        if (lane >= o) v += up;
    }
    return v;
}
__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// One workgroup per group.  Wavefront w owns the contiguous tokens [w W, (w + 1) W), W a multiple
// of 64; in round p its lane l handles token w W + 64 p + l, so every load is one contiguous run
// and (wavefront, round, lane) order is token order.  A pick: the wavefronts' totals locate the
// wavefront that holds the r-th unit of mass, that wavefront walks its rounds to the round, and
// a scan over its lanes finds the token.
template <int C>
__global__ __launch_bounds__(kPPThreads) void kmeanspp_kernel(const uint16_t* __restrict__ xg_all,
                                                              const uint32_t* __restrict__ wq_all,
                                                              float* __restrict__ dmin_all,
                                                              const uint64_t* __restrict__ rnd_all,
                                                              int32_t* __restrict__ picks_all, float* __restrict__ cent_all,
                                                              int n, int K, int log2n)
{
    constexpr int NWAVE = kPPThreads / 64;
    __shared__ unsigned long long wave_tot[NWAVE];
    __shared__ unsigned long long pmax_bits;
    __shared__ int pick_sh;

    const int g = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint16_t* xg = xg_all + (size_t)g * n * C;
    const uint32_t* wq = wq_all + (size_t)g * n;
    float* dmin = dmin_all + (size_t)g * n;
    const uint64_t* rnd = rnd_all + (size_t)g * K;
    int32_t* picks = picks_all ? picks_all + (size_t)g * K : nullptr;
    float* cent = cent_all + (size_t)g * K * C;

    const int rounds = (n + kPPThreads - 1) / kPPThreads;    // rounds of 64 tokens per wavefront
    const int t0 = wave * rounds * 64;                       // this wavefront's first token

    // q of this lane's token in round p: the integer weight (kq < -9000: first pick) or
    // floor(wq * dmin * 2^kq)
    auto mass = [&](int p, int kq) -> unsigned long long {
        const int i = t0 + p * 64 + lane;
        if (i >= n) return 0ull;
        if (kq < -9000) return wq[i];
        return (unsigned long long)ldexp((double)wq[i] * (double)dmin[i], kq);
    };
    // draws the token that holds unit r of the total mass (all threads call; sets pick_sh)
    auto draw = [&](uint64_t word, int kq) {
        unsigned long long local = 0;
        for (int p = 0; p < rounds; ++p) local += mass(p, kq);
        const unsigned long long wtot = wave_sum_u64(local);
        if (lane == 0) wave_tot[wave] = wtot;
        __syncthreads();
        unsigned long long off = 0, total = 0;
#pragma unroll
        for (int w = 0; w < NWAVE; ++w) {
            const unsigned long long t = wave_tot[w];
            off += w < wave ? t : 0ull;
            total += t;
        }
        const unsigned long long r = __umul64hi(word, total);
        if (r >= off && r < off + wtot) {                    // wavefront-uniform: exactly one wavefront
            unsigned long long run = off;
            for (int p = 0; p < rounds; ++p) {
                const unsigned long long q = mass(p, kq);
                const unsigned long long rsum = wave_sum_u64(q);
                if (run + rsum > r) {
                    const unsigned long long incl = run + wave_incl_scan_u64(q, lane);
                    const unsigned long long hit = __ballot(incl > r);
                    if (lane == 0) pick_sh = t0 + p * 64 + __builtin_ctzll(hit);
                    break;
                }
                run += rsum;
            }
        }
        __syncthreads();
    };

    draw(rnd[0], -10000);                                    // first centre: proportional to the integer weights
    for (int j = 0;; ++j) {
        const int pick = pick_sh;
        __syncthreads();                                     // everyone has read pick_sh
        if (tid == 0) {
            if (picks) picks[j] = pick;
            pmax_bits = 0ull;
        }
        float cj[C];
        widen<C>(xg + (size_t)pick * C, cj);
        if (tid < C) cent[(size_t)j * C + tid] = cj[tid];
        if (j + 1 == K) break;

        // distance to the nearest centre so far; largest weighted distance (non-negative doubles
        // order like their bits)
        double pmax = 0.0;
#pragma unroll 4
        for (int p = 0; p < rounds; ++p) {
            const int i = t0 + p * 64 + lane;
            if (i < n) {
                float xi[C];
                widen<C>(xg + (size_t)i * C, xi);
                const float d = dist2<C>(xi, cj);
                const float dm = (j == 0 || d < dmin[i]) ? d : dmin[i];
                dmin[i] = dm;
                const double pr = (double)wq[i] * (double)dm;
                pmax = pr > pmax ? pr : pmax;
            }
        }
        unsigned long long pb = (unsigned long long)__double_as_longlong(pmax);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const unsigned long long other = __shfl_xor(pb, o);
            pb = other > pb ? other : pb;
        }
        __syncthreads();                                     // pmax_bits was cleared; dmin is written
        if (lane == 0) atomicMax(&pmax_bits, pb);
        __syncthreads();
        const unsigned long long pm = pmax_bits;
        if (pm == 0ull) {                                    // every token sits on a centre already
            if (tid == 0) pick_sh = (int)__umul64hi(rnd[j + 1], (unsigned long long)n);
            __syncthreads();
            continue;
        }
        const int kq = 62 - log2n - ((int)((pm >> 52) & 0x7ffull) - 1023 + 1);
        draw(rnd[j + 1], kq);
    }
}

// ------------------------------------------------------------------------------------------
// Lloyd iteration
// ------------------------------------------------------------------------------------------
template <int C>
__global__ __launch_bounds__(kAssignThreads) void kmeans_assign_kernel(const uint16_t* xg_all, const float* cent_all,
                                                                      uint16_t* assign_all, int n, int K)
{
    extern __shared__ float cs[];                   // [K][C]
    const int g = blockIdx.y, tid = threadIdx.x;
    const float* cent = cent_all + (size_t)g * K * C;
    for (int i = tid; i < K * C; i += kAssignThreads) cs[i] = cent[i];
    __syncthreads();

    const uint16_t* xg = xg_all + (size_t)g * n * C;
    const int base = blockIdx.x * (kAssignThreads * kAssignPoints) + tid;
    float x[kAssignPoints][C];
    float best[kAssignPoints];
    int arg[kAssignPoints];
#pragma unroll
    for (int p = 0; p < kAssignPoints; ++p) {
        const int i = min(base + p * kAssignThreads, n - 1);
        widen<C>(xg + (size_t)i * C, x[p]);
        best[p] = dist2<C>(x[p], cs);
        arg[p] = 0;
    }
    for (int k = 1; k < K; ++k) {
        float c[C];
#pragma unroll
        for (int i = 0; i < C; ++i) c[i] = cs[k * C + i];
#pragma unroll
        for (int p = 0; p < kAssignPoints; ++p) {
            const float d = dist2<C>(x[p], c);
            arg[p] = d < best[p] ? k : arg[p];
            best[p] = d < best[p] ? d : best[p];
        }
    }
#pragma unroll
    for (int p = 0; p < kAssignPoints; ++p) {
        const int i = base + p * kAssignThreads;
        if (i < n) assign_all[(size_t)g * n + i] = (uint16_t)arg[p];
    }
}

// One workgroup: clusters [k0, k0 + 256) of one group.  Exact integer sums in LDS, then the new
// centroids of the clusters that own tokens.
template <int C>
__global__ __launch_bounds__(256) void kmeans_update_kernel(const uint16_t* xg_all, const uint32_t* wq_all,
                                                            const uint16_t* assign_all, float* cent_all, int n, int K)
{
    __shared__ unsigned long long s_hi[kUpdateClusters * C], s_lo[kUpdateClusters * C], wsum[kUpdateClusters];
    const int g = blockIdx.x, k0 = blockIdx.y * kUpdateClusters, tid = threadIdx.x;
    for (int i = tid; i < kUpdateClusters * C; i += 256) { s_hi[i] = 0ull; s_lo[i] = 0ull; }
    for (int i = tid; i < kUpdateClusters; i += 256) wsum[i] = 0ull;
    __syncthreads();
    const uint16_t* xg = xg_all + (size_t)g * n * C;
    const uint32_t* wq = wq_all + (size_t)g * n;
    const uint16_t* assign = assign_all + (size_t)g * n;
    for (int i = tid; i < n; i += 256) {
        const int k = (int)assign[i] - k0;
        if (k < 0 || k >= kUpdateClusters) continue;
        const long long w = (long long)wq[i];
        float xi[C];
        widen<C>(xg + (size_t)i * C, xi);
#pragma unroll
        for (int ch = 0; ch < C; ++ch) {
            const long long xq = (long long)ldexpf(xi[ch], 24);          // an integer: exact
            const long long hi = xq >> 20;                               // floor
            const long long lo = xq - hi * 1048576;
            atomicAdd(&s_hi[k * C + ch], (unsigned long long)(w * hi));
            atomicAdd(&s_lo[k * C + ch], (unsigned long long)(w * lo));
        }
        atomicAdd(&wsum[k], (unsigned long long)w);
    }
    __syncthreads();
    for (int e = tid; e < kUpdateClusters * C; e += 256) {
        const int k = e / C;
        if (k0 + k >= K) continue;
        const long long wk = (long long)wsum[k];
        if (wk == 0) continue;                      // a cluster without tokens keeps its centroid
        const double num = (double)(long long)s_hi[e] * 1048576.0 + (double)(long long)s_lo[e];
        const double mean = num / (double)wk;
        cent_all[((size_t)g * K + k0) * C + e] = (float)(mean * 0x1p-24);
    }
}

__global__ void kmeans_finish_kernel(const float* cent, size_t count, uint16_t* out16, float* out32)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    const float v = cent[i];
    if (out16) out16[i] = __builtin_bit_cast(uint16_t, (_Float16)v);     // round to nearest even
    if (out32) out32[i] = v;
}

__global__ void kmeans_copy_u16_kernel(const uint16_t* src, uint16_t* dst, size_t count)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) dst[i] = src[i];
}

__global__ void kmeans_copy_f32_kernel(const float* src, float* dst, size_t count)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) dst[i] = src[i];
}

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

int ceil_log2(int n)
{
    int l = 0;
    while ((1ll << l) < n) ++l;
    return l;
}

bool launch_ok() { return hipGetLastError() == hipSuccess; }

template <int C>
cq_status run_init(const KMeansArgs& a, const KMeansWorkspace& ws, hipStream_t st)
{
    const int G = a.f.groups, K = a.f.k, n = a.n;
    if (a.weights) {
        hipLaunchKernelGGL(kmeans_clear_kernel, dim3((G + 255) / 256), dim3(256), 0, st, ws.wmax_bits, G);
        const int rows = n < 256 ? n : 256;
        hipLaunchKernelGGL(kmeans_wmax_kernel, dim3((G + 255) / 256, rows), dim3(256), 0, st, a.weights, n, G, ws.wmax_bits);
    }
    hipLaunchKernelGGL((kmeans_prepare_kernel<C>), dim3((n + kPrepTokens - 1) / kPrepTokens, (G + kPrepGroups - 1) / kPrepGroups), dim3(256), 0, st, a.x, a.x_row_stride,
                       a.weights, ws.wmax_bits, n, G, ws.xg, ws.wq);
    if (!launch_ok()) return CQ_ERR_HIP;
    (void)K;
    return CQ_OK;
}

template <int C>
cq_status run_kmeanspp(const KMeansArgs& a, const KMeansWorkspace& ws, hipStream_t st)
{
    hipLaunchKernelGGL((kmeanspp_kernel<C>), dim3(a.f.groups), dim3(kPPThreads), 0, st, ws.xg, ws.wq, ws.dmin, a.rnd, a.picks,
                       ws.cent, a.n, a.f.k, ceil_log2(a.n));
    return launch_ok() ? CQ_OK : CQ_ERR_HIP;
}

template <int C>
cq_status run_lloyd(const KMeansArgs& a, const KMeansWorkspace& ws, hipStream_t st)
{
    const int G = a.f.groups, K = a.f.k, n = a.n;
    const size_t lds = sizeof(float) * (size_t)K * C;
    const dim3 agrid((n + kAssignThreads * kAssignPoints - 1) / (kAssignThreads * kAssignPoints), G);
    const dim3 ugrid(G, (K + kUpdateClusters - 1) / kUpdateClusters);
    for (int it = 0; it < a.n_iter; ++it) {
        hipLaunchKernelGGL((kmeans_assign_kernel<C>), agrid, dim3(kAssignThreads), lds, st, ws.xg, ws.cent, ws.assign, n, K);
        hipLaunchKernelGGL((kmeans_update_kernel<C>), ugrid, dim3(256), 0, st, ws.xg, ws.wq, ws.assign, ws.cent, n, K);
    }
    return launch_ok() ? CQ_OK : CQ_ERR_HIP;
}

template <int C>
cq_status run_all(const KMeansArgs& a, const KMeansWorkspace& ws, hipStream_t st)
{
    cq_status s = run_init<C>(a, ws, st);
    if (s != CQ_OK) return s;
    if (a.do_init) {
        s = run_kmeanspp<C>(a, ws, st);
        if (s != CQ_OK) return s;
    } else {
        const size_t cnt = (size_t)a.f.groups * a.f.k * C;
        hipLaunchKernelGGL(kmeans_copy_f32_kernel, dim3((unsigned)((cnt + 255) / 256)), dim3(256), 0, st, a.cent_in, ws.cent, cnt);
    }
    s = run_lloyd<C>(a, ws, st);
    if (s != CQ_OK) return s;
    const size_t cnt = (size_t)a.f.groups * a.f.k * C;
    hipLaunchKernelGGL(kmeans_finish_kernel, dim3((unsigned)((cnt + 255) / 256)), dim3(256), 0, st, ws.cent, cnt, a.cent16_out,
                       a.cent32_out);
    if (a.assign_out && a.n_iter > 0) {
        const size_t an = (size_t)a.f.groups * a.n;
        hipLaunchKernelGGL(kmeans_copy_u16_kernel, dim3((unsigned)((an + 255) / 256)), dim3(256), 0, st, ws.assign, a.assign_out, an);
    }
    return launch_ok() ? CQ_OK : CQ_ERR_HIP;
}

}  // namespace

size_t kmeans_workspace_layout(const Derived& f, int n, void* base, KMeansWorkspace* ws)
{
    const size_t G = (size_t)f.groups, K = (size_t)f.k, C = (size_t)f.c;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off = align256(off + bytes);
        return at;
    };
    const size_t o_xg = take(G * n * C * 2);
    const size_t o_wq = take(G * n * 4);
    const size_t o_dmin = take(G * n * 4);
    const size_t o_assign = take(G * n * 2);
    const size_t o_cent = take(G * K * C * 4);
    const size_t o_wmax = take(G * 4);
    if (ws) {
        char* b = static_cast<char*>(base);
        ws->xg = reinterpret_cast<uint16_t*>(b + o_xg);
        ws->wq = reinterpret_cast<uint32_t*>(b + o_wq);
        ws->dmin = reinterpret_cast<float*>(b + o_dmin);
        ws->assign = reinterpret_cast<uint16_t*>(b + o_assign);
        ws->cent = reinterpret_cast<float*>(b + o_cent);
        ws->wmax_bits = reinterpret_cast<unsigned*>(b + o_wmax);
    }
    return off;
}

cq_status launch_kmeans(const KMeansArgs& a, void* workspace, hipStream_t stream)
{
    KMeansWorkspace ws;
    kmeans_workspace_layout(a.f, a.n, workspace, &ws);
    switch (a.f.c) {
    case 8: return run_all<8>(a, ws, stream);
    case 4: return run_all<4>(a, ws, stream);
    case 2: return run_all<2>(a, ws, stream);
    case 1: return run_all<1>(a, ws, stream);
    default: return CQ_ERR_UNSUPPORTED;
    }
}

}  // namespace cq

// Measurement aids of libcq: a read-only streaming kernel and a plain copy kernel of known
// size.  They compute nothing of the method; benchmarks use them as yardsticks (what fraction of
// a pure streaming read the decode kernel reaches; what the HBM byte counters report for a
// known number of bytes).
#include <hip/hip_runtime.h>

#include "cq_internal.hpp"

namespace cq {
namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
constexpr int kProbeThreads = 512;
constexpr int kProbeUnroll = 8;

// Every workgroup reads a contiguous chunk, 16 bytes per lane per load, kProbeUnroll loads in
// flight per lane; the XOR of everything read goes to sink[blockIdx.x] so the loads are live.
__global__ __launch_bounds__(kProbeThreads) void probe_read_kernel(const u32x4* src, size_t n16, unsigned* sink)
{
    const size_t per_wg = (size_t)kProbeThreads * kProbeUnroll;
    u32x4 acc = {0, 0, 0, 0};
    for (size_t base = (size_t)blockIdx.x * per_wg; base < n16; base += (size_t)gridDim.x * per_wg) {
        u32x4 v[kProbeUnroll];
#pragma unroll
        for (int k = 0; k < kProbeUnroll; ++k) {
            const size_t i = base + (size_t)k * kProbeThreads + threadIdx.x;
            v[k] = i < n16 ? __builtin_nontemporal_load(src + i) : u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int k = 0; k < kProbeUnroll; ++k) acc ^= v[k];
    }
    unsigned x = acc.x ^ acc.y ^ acc.z ^ acc.w;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x ^= __shfl_xor(x, o);
    if ((threadIdx.x & 63) == 0) atomicXor(sink + blockIdx.x, x);
}

__global__ __launch_bounds__(kProbeThreads) void probe_copy_kernel(const u32x4* src, u32x4* dst, size_t n16)
{
    const size_t per_wg = (size_t)kProbeThreads * kProbeUnroll;
    for (size_t base = (size_t)blockIdx.x * per_wg; base < n16; base += (size_t)gridDim.x * per_wg) {
        u32x4 v[kProbeUnroll];
#pragma unroll
        for (int k = 0; k < kProbeUnroll; ++k) {
            const size_t i = base + (size_t)k * kProbeThreads + threadIdx.x;
            if (i < n16) v[k] = src[i];
        }
#pragma unroll
        for (int k = 0; k < kProbeUnroll; ++k) {
            const size_t i = base + (size_t)k * kProbeThreads + threadIdx.x;
            if (i < n16) dst[i] = v[k];
        }
    }
}

unsigned probe_grid(size_t n16)
{
    const size_t per_wg = (size_t)kProbeThreads * kProbeUnroll;
    const size_t want = (n16 + per_wg - 1) / per_wg;
    return (unsigned)std::min<size_t>(want, 256 * 8);      // a few workgroups per CU, grid-stride beyond
}

}  // namespace
}  // namespace cq

using namespace cq;

typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

// One wavefront, one MFMA.  Lane l supplies row (l % 32) of A and column (l % 32) of B for the
// k range (l / 32) * KD/2 ...; it receives rows 8 (i / 4) + 4 (l / 32) + i % 4 of column l % 32.
template <int KD>
__global__ __launch_bounds__(64) void probe_mfma_kernel(const _Float16* a, const _Float16* b, float* d)
{
    constexpr int HALF = KD / 2;
    const int lane = threadIdx.x, rc = lane & 31, kh = lane >> 5;
    const float16_t zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float16_t acc;
    if constexpr (KD == 16) {
        half8_t av, bv;
#pragma unroll
        for (int i = 0; i < HALF; ++i) {
            av[i] = a[rc * KD + kh * HALF + i];
            bv[i] = b[(kh * HALF + i) * 32 + rc];
        }
        acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, bv, zero, 0, 0, 0);
    } else {
        half4_t av, bv;
#pragma unroll
        for (int i = 0; i < HALF; ++i) {
            av[i] = a[rc * KD + kh * HALF + i];
            bv[i] = b[(kh * HALF + i) * 32 + rc];
        }
        acc = __builtin_amdgcn_mfma_f32_32x32x8f16(av, bv, zero, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) d[(8 * (i / 4) + 4 * kh + (i % 4)) * 32 + rc] = acc[i];
}

extern "C" {

cq_status cq_probe_stream_read(const void* src, size_t bytes, void* sink, void* stream)
{
    if (!src || !sink || bytes == 0 || bytes % 16 != 0) return CQ_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return CQ_ERR_INVALID_ARG;
    const size_t n16 = bytes / 16;
    hipLaunchKernelGGL(probe_read_kernel, dim3(probe_grid(n16)), dim3(kProbeThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4*>(src), n16, static_cast<unsigned*>(sink));
    return hipGetLastError() == hipSuccess ? CQ_OK : CQ_ERR_HIP;
}

cq_status cq_probe_copy(const void* src, void* dst, size_t bytes, void* stream)
{
    if (!src || !dst || bytes == 0 || bytes % 16 != 0) return CQ_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(dst) & 15u)) return CQ_ERR_INVALID_ARG;
    const size_t n16 = bytes / 16;
    hipLaunchKernelGGL(probe_copy_kernel, dim3(probe_grid(n16)), dim3(kProbeThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), n16);
    return hipGetLastError() == hipSuccess ? CQ_OK : CQ_ERR_HIP;
}

cq_status cq_probe_mfma(const void* a, const void* b, void* d, int32_t kdim, void* stream)
{
    if (!a || !b || !d || (kdim != 8 && kdim != 16)) return CQ_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(a) & 15u) || (reinterpret_cast<uintptr_t>(b) & 15u) || (reinterpret_cast<uintptr_t>(d) & 15u))
        return CQ_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (kdim == 16)
        hipLaunchKernelGGL(probe_mfma_kernel<16>, dim3(1), dim3(64), 0, st, static_cast<const _Float16*>(a),
                           static_cast<const _Float16*>(b), static_cast<float*>(d));
    else
        hipLaunchKernelGGL(probe_mfma_kernel<8>, dim3(1), dim3(64), 0, st, static_cast<const _Float16*>(a),
                           static_cast<const _Float16*>(b), static_cast<float*>(d));
    return hipGetLastError() == hipSuccess ? CQ_OK : CQ_ERR_HIP;
}

}  // extern "C"

// Measurement helpers: what this card sustains on the two resources the hot-path kernels are bound
// by, measured with the simplest possible kernels.  Not part of the method; the benchmark reports
// these figures next to the published peaks.
//   * dynb_probe_mfma_bf16: register-only loop of independent v_mfma_f32_32x32x16_bf16 (no memory
//     traffic at all): the dense bf16 rate the matrix pipes sustain at the clock the card settles at.
//   * dynb_probe_copy: plain device-to-device copy with 16-byte accesses: achievable HBM bandwidth,
//     and the known-size reference that the profiler's FETCH_SIZE / WRITE_SIZE counters are scaled by.
//   * dynb_probe_read: the same accesses without the stores: what a kernel that only streams operands in
//     (the expert layers' weights) can expect.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <string>

#include "device_utils.h"
#include "plan_internal.h"

using dynb::fail;

namespace {

constexpr int PROBE_CHAINS = 8;      // independent accumulator chains per wave (128 accumulator registers)

__global__ __launch_bounds__(256) void k_probe_mfma(float* __restrict__ sink, int iters)
{
    const int lane = threadIdx.x & 63;
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = __bf16(float((lane + i) & 7) * 0.125f);
        b[i] = __bf16(float((lane * 3 + i) & 7) * 0.125f - 0.5f);
    }
    f32x16 acc[PROBE_CHAINS];
#pragma unroll
    for (int c = 0; c < PROBE_CHAINS; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int c = 0; c < PROBE_CHAINS; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < PROBE_CHAINS; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[c][i];
    if (s == 12345.678f) sink[0] = s;          // keeps the loop alive; practically never taken
}

__global__ __launch_bounds__(256) void k_probe_copy(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n16)
{
    for (size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n16; i += size_t(gridDim.x) * blockDim.x)
        dst[i] = src[i];
}

// Every workgroup reads a contiguous share of the buffer, 4 KB per step of its 256 lanes, eight steps in flight: of
// the patterns tried (this one, lanes striding over the whole buffer with 4 to 16 loads in flight, grids of 512 to
// 8192 workgroups, non-temporal loads, shares dealt so that a die reads one eighth) the fastest on this card, about
// a fifth above the striding one.
__global__ __launch_bounds__(256) void k_probe_read(const u32x4* __restrict__ src, uint32_t* __restrict__ sink, size_t n16)
{
    const size_t per = (n16 / gridDim.x) & ~size_t(2047);          // pieces per workgroup: whole steps of 8 x 256
    const u32x4* p = src + size_t(blockIdx.x) * per + threadIdx.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (size_t i = 0; i < per; i += 8 * 256) {
        u32x4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = p[i + j * 256];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc |= v[j];
    }
    // what the shares left over, lanes striding
    for (size_t i = per * gridDim.x + size_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n16; i += size_t(gridDim.x) * blockDim.x)
        acc |= src[i];
    if ((acc.x & acc.y & acc.z & acc.w) == 0xdeadbeefu) sink[0] = acc.x;   // keeps the loads alive; practically never taken
}

}  // namespace

extern "C" int dynb_probe_read(const void* src, size_t bytes, void* sink, void* stream)
{
    if (!src || !sink) return fail(DYNB_E_INVAL, "dynb_probe_read: NULL argument");
    if (bytes % 16 || reinterpret_cast<uintptr_t>(src) % 16)
        return fail(DYNB_E_INVAL, "dynb_probe_read: size and pointer must be multiples of 16 bytes");
    if (bytes == 0) return DYNB_OK;
    const size_t n16 = bytes / 16;
    const unsigned grid = unsigned(std::min<size_t>((n16 + 2047) / 2048, size_t(256) * 8));
    hipLaunchKernelGGL(k_probe_read, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4*>(src), static_cast<uint32_t*>(sink), n16);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(DYNB_E_HIP, std::string("dynb_probe_read: ") + hipGetErrorString(e));
    return DYNB_OK;
}

extern "C" int dynb_probe_mfma_bf16(int32_t iters, int32_t workgroups, float* sink, void* stream, double* flops)
{
    if (iters <= 0 || workgroups <= 0 || !sink || !flops)
        return fail(DYNB_E_INVAL, "dynb_probe_mfma_bf16: iters and workgroups must be positive, sink and flops not NULL");
    hipLaunchKernelGGL(k_probe_mfma, dim3(unsigned(workgroups)), dim3(256), 0, static_cast<hipStream_t>(stream), sink, iters);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(DYNB_E_HIP, std::string("dynb_probe_mfma_bf16: ") + hipGetErrorString(e));
    // one 32x32x16 MFMA = 2 * 32 * 32 * 16 flop per wave
    *flops = double(workgroups) * 4.0 * double(iters) * PROBE_CHAINS * (2.0 * 32 * 32 * 16);
    return DYNB_OK;
}

extern "C" int dynb_probe_copy(void* dst, const void* src, size_t bytes, void* stream)
{
    if (!dst || !src) return fail(DYNB_E_INVAL, "dynb_probe_copy: NULL argument");
    if (bytes % 16 || (reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) % 16)
        return fail(DYNB_E_INVAL, "dynb_probe_copy: size and pointers must be multiples of 16 bytes");
    if (bytes == 0) return DYNB_OK;
    const size_t n16 = bytes / 16;
    const unsigned grid = unsigned(std::min<size_t>((n16 + 255) / 256, size_t(256) * 32));
    hipLaunchKernelGGL(k_probe_copy, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), n16);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(DYNB_E_HIP, std::string("dynb_probe_copy: ") + hipGetErrorString(e));
    return DYNB_OK;
}

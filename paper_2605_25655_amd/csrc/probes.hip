// Two measurement probes behind a C ABI of their own (include/thi_probe.h, libthi_probe.so): what this GPU actually sustains for
// the two resources the kernels are bound by.  They compute nothing useful and are only called by
// the benchmark, which reports them next to the nominal peaks.
#include "../../include/thi_probe.h"
#include "thi_internal.h"

namespace {

using namespace thi;

// Streaming read: every workgroup walks a contiguous share with non-temporal 16-byte loads, eight
// 1 KiB wave-loads in flight per wave -- the access pattern of an ideal weight-streaming kernel.
__global__ __launch_bounds__(256) void probe_stream_read(const uintx4* __restrict__ p, size_t n16, unsigned* sink)
{
    const size_t per = n16 / gridDim.x;
    const uintx4* base = p + per * blockIdx.x;
    unsigned acc = 0;
    for (size_t i = threadIdx.x; i + 7 * 256 < per; i += 8 * 256) {
        uintx4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(base + i + u * 256);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x12345678u) sink[0] = acc;      // keeps the loads alive; practically never true
}

// Register-only MFMA loop: 8 independent 32x32x16 fp16 accumulators per wave, operands taken from
// `src` (so that the caller decides whether they are constant or random -- the clock under load, and
// with it the attainable rate, depends on how many operand bits toggle).
__global__ __launch_bounds__(512) void probe_mfma_f16(const half8* __restrict__ src, float* sink, int iters)
{
    half8 a[4], b[4];
    for (int i = 0; i < 4; ++i) {
        a[i] = src[(threadIdx.x + 512 * i) & 4095];
        b[i] = src[(threadIdx.x * 3 + 17 + 512 * i) & 4095];
    }
    floatx16 acc[8];
    for (int i = 0; i < 8; ++i)
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i & 3], b[(i >> 2) & 3], acc[i], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 8; ++i)
        for (int e = 0; e < 16; ++e) s += acc[i][e];
    if (s == 12345.678f) sink[0] = s;
}

}  // namespace

extern "C" {

int thi_probe_stream_read(const void* buffer, size_t bytes, void* sink, void* hip_stream)
{
    if (!buffer || !sink) return THI_ERR_NULL;
    if (bytes < (size_t)512 * 8 * 256 * 16) return THI_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(buffer) & 15) || (reinterpret_cast<uintptr_t>(sink) & 3)) return THI_ERR_ALIGN;
    hipLaunchKernelGGL(probe_stream_read, dim3(512), dim3(256), 0, (hipStream_t)hip_stream,
                       (const uintx4*)buffer, bytes / 16, (unsigned*)sink);
    return hipGetLastError() == hipSuccess ? THI_OK : THI_ERR_HIP;
}

int thi_probe_mfma_f16(const void* operands, int iters, int workgroups, void* sink, void* hip_stream)
{
    if (!operands || !sink) return THI_ERR_NULL;
    if (iters < 1 || workgroups < 1) return THI_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(operands) & 15) || (reinterpret_cast<uintptr_t>(sink) & 3)) return THI_ERR_ALIGN;
    hipLaunchKernelGGL(probe_mfma_f16, dim3(workgroups), dim3(512), 0, (hipStream_t)hip_stream,
                       (const half8*)operands, (float*)sink, iters);
    return hipGetLastError() == hipSuccess ? THI_OK : THI_ERR_HIP;
}

}  // extern "C"

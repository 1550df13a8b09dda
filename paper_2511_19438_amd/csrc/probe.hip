// Measurement aids, not part of the method: two kernels that show what this chip delivers to ANY kernel, so
// that the roofline fractions of the GEMM kernels can be read against the machine and not only against the
// data-sheet peaks.
//   * stream_probe: a plain read of a buffer with 128-bit loads (the footprint of a GEMV's packed weights):
//     launch gap, first-byte latency and ramp are paid by every kernel of that size.
//   * mfma_probe: v_mfma_f32_32x32x16_f16 back to back on register operands taken from a caller-supplied
//     buffer (random values: the sustained rate depends on operand toggling through the power limit), with
//     nothing else running - the ceiling of the matrix pipe under the same power budget as the prefill kernel.
//   * issue_probe: one MFMA followed by V independent packed-fp16 vector instructions, with one, two or four
//     wavefronts per SIMD: what the dequantisation around an MFMA costs on this chip (the mid-batch and prefill
//     kernels are bound by the SIMD's vector issue port, not by the matrix pipe or by memory).
#include "gptq_w4a16.h"

#include "kernels.h"

namespace {

using namespace gptq;

__global__ __launch_bounds__(512) void stream_probe_kernel(const uint4 *p, size_t n16, uint32_t *sink)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    uint32_t acc = 0;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const uint4 a = p[i], b = p[i + stride], c = p[i + 2 * stride], d = p[i + 3 * stride];
        acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    for (; i < n16; i += stride) {
        const uint4 a = p[i];
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    // one word per workgroup: keeps the loads alive, writes next to nothing
    acc ^= __shfl_xor(acc, 32, 64);
    if (threadIdx.x == 0)
        sink[blockIdx.x & 63] = acc;
}

constexpr int kProbeChains = 16;  // independent accumulator chains per wavefront (256 accumulator registers)
constexpr int kProbeOperands = 8;

__global__ __launch_bounds__(256) void mfma_probe_kernel(const half8_t *operands, int count, float *sink, int iters)
{
    half8_t a[kProbeOperands], b[kProbeOperands];
#pragma unroll
    for (int j = 0; j < kProbeOperands; ++j) {
        a[j] = operands[(threadIdx.x + 256 * j) % count];
        b[j] = operands[(threadIdx.x * 7 + 13 * j + blockIdx.x) % count];
    }
    float16_t acc[kProbeChains];
#pragma unroll
    for (int j = 0; j < kProbeChains; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            acc[j][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < kProbeChains; ++j)
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[j % kProbeOperands], b[(j / 2) % kProbeOperands], acc[j],
                                                            0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < kProbeChains; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            s += acc[j][r];
    if (s == 1.2345f)  // practically never: the sums only have to be observable
        sink[0] = s;
}

// One group = one MFMA + V packed-fp16 fused multiply-adds on eight rotating registers (independent of the MFMA
// and, eight instructions apart, of each other).  Inline assembly keeps the sequence as written.
template <int V>
__global__ __launch_bounds__(1024) void issue_probe_kernel(const half8_t *operands, int count, float *sink, int iters)
{
    const half8_t a = operands[threadIdx.x % count];
    const half8_t b = operands[(threadIdx.x * 3 + 1 + blockIdx.x) % count];
    float16_t acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            acc[j][r] = 0.f;
    half2_t v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
        v[j] = half2_t{(half_t)(float)(threadIdx.x & 7), (half_t)(float)j};
    half2_t c = {(half_t)0.5f, (half_t)0.25f}, d = {(half_t)0.25f, (half_t)0.125f};
    asm volatile("" : "+v"(c), "+v"(d));
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+v"(acc[j]) : "v"(a), "v"(b));
#pragma unroll
            for (int q = 0; q < V; ++q)
                asm volatile("v_pk_fma_f16 %0, %0, %1, %2" : "+v"(v[(j * V + q) % 8]) : "v"(c), "v"(d));
        }
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            s += acc[j][r];
#pragma unroll
    for (int j = 0; j < 8; ++j)
        s += (float)v[j][0] + (float)v[j][1];
    if (s == 1.2345f)
        sink[0] = s;
}

template <int V>
hipError_t launch_issue_probe(int workgroups, int threads, hipStream_t stream, const half8_t *operands, int count,
                              float *sink, int iters)
{
    // 96 KB of (unused) LDS per workgroup: one workgroup per compute unit, so `threads / 256` wavefronts per SIMD
    constexpr int kLds = 96 * 1024;
    hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(issue_probe_kernel<V>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
    if (err != hipSuccess)
        return err;
    hipLaunchKernelGGL(issue_probe_kernel<V>, dim3(workgroups), dim3(threads), kLds, stream, operands, count, sink,
                       iters);
    return hipGetLastError();
}

}  // namespace

extern "C" {

int gptq_w4a16_stream_probe(const void *buf, size_t bytes, void *sink, gptq_stream_t stream)
{
    if (!buf || !sink || bytes < 16)
        return GPTQ_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(buf) & 15u) != 0 || (reinterpret_cast<uintptr_t>(sink) & 15u) != 0)
        return GPTQ_MISALIGNED;
    hipLaunchKernelGGL(stream_probe_kernel, dim3(256), dim3(512), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4 *>(buf), bytes / 16, static_cast<uint32_t *>(sink));
    return hipGetLastError() == hipSuccess ? GPTQ_OK : GPTQ_HIP_ERROR;
}

int gptq_w4a16_mfma_probe(const void *operands, size_t bytes, void *sink, int iters, double *flops,
                          gptq_stream_t stream)
{
    if (!operands || !sink || bytes < 16 || iters <= 0 || iters > (1 << 22))
        return GPTQ_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(operands) & 15u) != 0 || (reinterpret_cast<uintptr_t>(sink) & 15u) != 0)
        return GPTQ_MISALIGNED;
    const int workgroups = 512;  // two per compute unit, four wavefronts each
    const size_t count = bytes / 16 < (size_t)(1 << 20) ? bytes / 16 : (size_t)(1 << 20);
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const half8_t *>(operands), (int)count, static_cast<float *>(sink), iters);
    if (hipGetLastError() != hipSuccess)
        return GPTQ_HIP_ERROR;
    if (flops)
        *flops = (double)workgroups * 4.0 * iters * kProbeChains * (2.0 * 32 * 32 * 16);
    return GPTQ_OK;
}

int gptq_w4a16_issue_probe(const void *operands, size_t bytes, void *sink, int iters, int valu_per_mfma,
                           int waves_per_simd, double *mfma_per_simd, gptq_stream_t stream)
{
    if (!operands || !sink || bytes < 16 || iters <= 0 || iters > (1 << 20))
        return GPTQ_INVALID_ARG;
    if (waves_per_simd != 1 && waves_per_simd != 2 && waves_per_simd != 4)
        return GPTQ_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(operands) & 15u) != 0 || (reinterpret_cast<uintptr_t>(sink) & 15u) != 0)
        return GPTQ_MISALIGNED;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return GPTQ_HIP_ERROR;
    const int rounds = 4;  // workgroups per compute unit, one after the other
    const int workgroups = cus * rounds;
    const int threads = 256 * waves_per_simd;
    const size_t count = bytes / 16 < (size_t)(1 << 20) ? bytes / 16 : (size_t)(1 << 20);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const half8_t *ops = static_cast<const half8_t *>(operands);
    float *out = static_cast<float *>(sink);
    hipError_t err;
    switch (valu_per_mfma) {
    case 0: err = launch_issue_probe<0>(workgroups, threads, s, ops, (int)count, out, iters); break;
    case 2: err = launch_issue_probe<2>(workgroups, threads, s, ops, (int)count, out, iters); break;
    case 4: err = launch_issue_probe<4>(workgroups, threads, s, ops, (int)count, out, iters); break;
    case 6: err = launch_issue_probe<6>(workgroups, threads, s, ops, (int)count, out, iters); break;
    case 8: err = launch_issue_probe<8>(workgroups, threads, s, ops, (int)count, out, iters); break;
    case 12: err = launch_issue_probe<12>(workgroups, threads, s, ops, (int)count, out, iters); break;
    case 16: err = launch_issue_probe<16>(workgroups, threads, s, ops, (int)count, out, iters); break;
    default: return GPTQ_INVALID_ARG;
    }
    if (err != hipSuccess)
        return GPTQ_HIP_ERROR;
    if (mfma_per_simd)
        *mfma_per_simd = (double)rounds * waves_per_simd * iters * 4.0;
    return GPTQ_OK;
}

}  // extern "C"

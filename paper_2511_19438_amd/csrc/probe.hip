// Measurement aids, not part of the method: two kernels that show what this chip delivers to ANY kernel, so
// that the roofline fractions of the GEMM kernels can be read against the machine and not only against the
// data-sheet peaks.
//   * stream_probe: a plain read of a buffer with 128-bit loads (the footprint of a GEMV's packed weights):
//     launch gap, first-byte latency and ramp are paid by every kernel of that size.
//   * mfma_probe: v_mfma_f32_32x32x16_f16 back to back on register operands taken from a caller-supplied
//     buffer (random values: the sustained rate depends on operand toggling through the power limit), with
//     nothing else running - the ceiling of the matrix pipe under the same power budget as the prefill kernel.
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

}  // extern "C"

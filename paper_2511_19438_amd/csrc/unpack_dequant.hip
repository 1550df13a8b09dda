// Standalone int4 unpack and per-group dequantisation kernels for gfx950.
//
// These expose the first stages of the W4A16 GPTQ pipeline (the 4-bit field extraction and
// w = scale * (q - z)) as tensors so that they can be checked bit for bit.  Both are pure
// streaming kernels: one thread owns four adjacent columns of one packed row (a 128-bit
// load of qweight), i.e. 4 x 8 weights, and writes them row by row so that a wavefront
// stores 256 B (uint8) or 512 B (fp16) of each output row contiguously.
#include "kernels.h"

namespace gptq {

namespace {

constexpr int kThreads = 256;

// q_out[k, n] = (qweight[k/8, n] >> 4*(k%8)) & 15
__global__ __launch_bounds__(kThreads) void unpack_qweight_kernel(const uint32_t *__restrict__ qweight,
                                                                   uint8_t *__restrict__ q_out, int rows, int N)
{
    const int quads = N >> 2;
    const long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= (long long)rows * quads)
        return;
    const int row = (int)(idx / quads);
    const int n0 = (int)(idx % quads) * 4;
    const uint4 w = *reinterpret_cast<const uint4 *>(qweight + (size_t)row * N + n0);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t packed = ((w.x >> (4 * j)) & 15u) | (((w.y >> (4 * j)) & 15u) << 8) |
                                (((w.z >> (4 * j)) & 15u) << 16) | (((w.w >> (4 * j)) & 15u) << 24);
        *reinterpret_cast<uint32_t *>(q_out + (size_t)(row * 8 + j) * N + n0) = packed;
    }
}

// z_out[r, n] = (qzeros[r, n/8] >> 4*(n%8)) & 15
__global__ __launch_bounds__(kThreads) void unpack_qzeros_kernel(const uint32_t *__restrict__ qzeros,
                                                                  uint8_t *__restrict__ z_out, long long words)
{
    const long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= words)
        return;
    const uint32_t w = qzeros[idx];
    uint2 bytes;
    bytes.x = (w & 15u) | (((w >> 4) & 15u) << 8) | (((w >> 8) & 15u) << 16) | (((w >> 12) & 15u) << 24);
    bytes.y = ((w >> 16) & 15u) | (((w >> 20) & 15u) << 8) | (((w >> 24) & 15u) << 16) | (((w >> 28) & 15u) << 24);
    // word idx of row r covers columns 8*(idx % (N/8)) .. +7 of that row: the flat byte offset is simply 8*idx
    *reinterpret_cast<uint2 *>(z_out + 8 * idx) = bytes;
}

// w_out[k, n] = fp16( scales[r(k), n] * (q[k, n] - z[r(k), n]) ): exact integer difference, one fp16 multiply.
template <bool ACT_ORDER>
__global__ __launch_bounds__(kThreads) void dequant_kernel(const uint32_t *__restrict__ qweight,
                                                           const uint32_t *__restrict__ qzeros,
                                                           const half_t *__restrict__ scales,
                                                           const int32_t *__restrict__ g_idx,
                                                           half_t *__restrict__ w_out, int rows, int N,
                                                           int group_size)
{
    const int quads = N >> 2;
    const long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= (long long)rows * quads)
        return;
    const int row = (int)(idx / quads);
    const int n0 = (int)(idx % quads) * 4;
    const uint4 wv = *reinterpret_cast<const uint4 *>(qweight + (size_t)row * N + n0);
    const uint32_t w[4] = {wv.x, wv.y, wv.z, wv.w};
    const int zshift = (n0 & 4) * 4;  // which half of the zero-point word holds these four columns

    int group = (row * 8) / group_size;  // group_size is a multiple of 8: one group per packed row
    half4_t s;
    uint32_t zbits;
    if (!ACT_ORDER) {
        s = *reinterpret_cast<const half4_t *>(scales + (size_t)group * N + n0);
        zbits = qzeros[(size_t)group * (N >> 3) + (n0 >> 3)] >> zshift;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int k = row * 8 + j;
        if (ACT_ORDER) {
            group = g_idx[k];
            s = *reinterpret_cast<const half4_t *>(scales + (size_t)group * N + n0);
            zbits = qzeros[(size_t)group * (N >> 3) + (n0 >> 3)] >> zshift;
        }
        half4_t o;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int q = (int)((w[c] >> (4 * j)) & 15u);
            const int z = (int)((zbits >> (4 * c)) & 15u);
            o[c] = (half_t)(q - z) * s[c];
        }
        *reinterpret_cast<half4_t *>(w_out + (size_t)k * N + n0) = o;
    }
}

inline unsigned blocks_for(long long items)
{
    return (unsigned)((items + kThreads - 1) / kThreads);
}

// z' = (z + delta) mod 16 for every nibble of every word (delta in 0..15; even and odd nibbles apart so that
// no carry crosses into a neighbour).
__global__ __launch_bounds__(kThreads) void shift_zeros_kernel(const uint32_t *__restrict__ in,
                                                               uint32_t *__restrict__ out, long long words,
                                                               uint32_t delta)
{
    const long long i = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (i >= words)
        return;
    const uint32_t w = in[i];
    const uint32_t even = ((w & 0x0f0f0f0fu) + delta * 0x01010101u) & 0x0f0f0f0fu;
    const uint32_t odd = (((w >> 4) & 0x0f0f0f0fu) + delta * 0x01010101u) & 0x0f0f0f0fu;
    out[i] = even | (odd << 4);
}

}  // namespace

hipError_t launch_unpack(const uint32_t *qweight, uint8_t *q_out, const uint32_t *qzeros, uint8_t *z_out, int K,
                         int N, int group_size, hipStream_t stream)
{
    const int rows = K / 8;
    const long long items = (long long)rows * (N / 4);
    hipLaunchKernelGGL(unpack_qweight_kernel, dim3(blocks_for(items)), dim3(kThreads), 0, stream, qweight, q_out,
                       rows, N);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess)
        return err;
    if (z_out) {
        const long long words = (long long)(K / group_size) * (N / 8);
        hipLaunchKernelGGL(unpack_qzeros_kernel, dim3(blocks_for(words)), dim3(kThreads), 0, stream, qzeros, z_out,
                           words);
        err = hipGetLastError();
    }
    return err;
}

hipError_t launch_shift_zeros(const uint32_t *in, uint32_t *out, long long words, int delta, hipStream_t stream)
{
    hipLaunchKernelGGL(shift_zeros_kernel, dim3(blocks_for(words)), dim3(kThreads), 0, stream, in, out, words,
                       (uint32_t)(delta & 15));
    return hipGetLastError();
}

hipError_t launch_dequant(const uint32_t *qweight, const uint32_t *qzeros, const half_t *scales,
                          const int32_t *g_idx, half_t *w_out, int K, int N, int group_size, hipStream_t stream)
{
    const int rows = K / 8;
    const long long items = (long long)rows * (N / 4);
    if (g_idx)
        hipLaunchKernelGGL(dequant_kernel<true>, dim3(blocks_for(items)), dim3(kThreads), 0, stream, qweight, qzeros,
                           scales, g_idx, w_out, rows, N, group_size);
    else
        hipLaunchKernelGGL(dequant_kernel<false>, dim3(blocks_for(items)), dim3(kThreads), 0, stream, qweight,
                           qzeros, scales, g_idx, w_out, rows, N, group_size);
    return hipGetLastError();
}

}  // namespace gptq

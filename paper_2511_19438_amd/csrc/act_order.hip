// One-time repack of an act-order (g_idx) checkpoint and the activation gather that goes with it.
//
// With activation ordering (not treated by the paper; part of the problem statement: the quantiser visited
// the input channels in order of importance) row k of the packed weight belongs to group g_idx[k], an arbitrary map.  The kernels
// that read g_idx per row pay for it on every call.  The map is fixed once the checkpoint is loaded,
// so the rows can be sorted by group ONCE: with perm = the stable order of k by g_idx[k], row j of the
// sorted matrix is row perm[j] of the original, group j / group_size, and
//     out[m, n] = sum_j x[m, perm[j]] * W_sorted[j, n]
// is the plain (no g_idx) problem on gathered activations.  Requires every group to own exactly
// group_size rows, which is what the quantiser produces.
#include "kernels.h"

namespace gptq {

namespace {

constexpr int kThreads = 256;

// perm[g * group_size + r] = k, where r is the number of k' < k of the same group (stable order).
// status bit 0: an entry of g_idx lies outside [0, groups); bit 1: a group owns more than group_size rows.
__global__ __launch_bounds__(kThreads) void rank_rows_kernel(const int32_t *__restrict__ g_idx,
                                                             int32_t *__restrict__ perm, int K, int groups,
                                                             int group_size, int *status)
{
    __shared__ int32_t tile[1024];
    const int k = blockIdx.x * kThreads + threadIdx.x;
    const int g = k < K ? g_idx[k] : -1;
    int rank = 0;
    const int last = min(K, (int)(blockIdx.x + 1) * kThreads);  // nobody in this block needs k' beyond its own k
    for (int base = 0; base < last; base += 1024) {
        for (int i = threadIdx.x; i < 1024; i += kThreads)
            tile[i] = base + i < K ? g_idx[base + i] : -2;
        __syncthreads();
        const int n = min(1024, k - base);  // entries of this tile that come before k
        for (int i = 0; i < n; ++i)
            rank += tile[i] == g;
        __syncthreads();
    }
    if (k >= K)
        return;
    if (g < 0 || g >= groups) {
        atomicOr(status, 1);
        return;
    }
    if (rank >= group_size) {
        atomicOr(status, 2);
        return;
    }
    perm[g * group_size + rank] = k;
}

// Row j of the sorted matrix is row perm[j] of the original: gathers nibbles, 4 adjacent columns per thread.
__global__ __launch_bounds__(kThreads) void sort_rows_kernel(const uint32_t *__restrict__ qweight,
                                                             const int32_t *__restrict__ perm,
                                                             uint32_t *__restrict__ sorted, int rows, int N)
{
    const int quads = N >> 2;
    const long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= (long long)rows * quads)
        return;
    const int jr = (int)(idx / quads);
    const int n = (int)(idx - (long long)jr * quads) * 4;
    uint4 out = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int src = perm[jr * 8 + e];
        const uint4 w = *reinterpret_cast<const uint4 *>(qweight + (size_t)(src >> 3) * N + n);
        const int sh = 4 * (src & 7);
        out.x |= ((w.x >> sh) & 15u) << (4 * e);
        out.y |= ((w.y >> sh) & 15u) << (4 * e);
        out.z |= ((w.z >> sh) & 15u) << (4 * e);
        out.w |= ((w.w >> sh) & 15u) << (4 * e);
    }
    *reinterpret_cast<uint4 *>(sorted + (size_t)jr * N + n) = out;
}

// xp[m, j] = x[m, perm[j]], eight adjacent j per thread (one 128-bit store).
__global__ __launch_bounds__(kThreads) void gather_activations_kernel(const half_t *__restrict__ x,
                                                                      const int32_t *__restrict__ perm,
                                                                      half_t *__restrict__ xp, int M, int K)
{
    const int chunks = K >> 3;
    const long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= (long long)M * chunks)
        return;
    const int m = (int)(idx / chunks);
    const int j = (int)(idx - (long long)m * chunks) * 8;
    const int4 pa = *reinterpret_cast<const int4 *>(perm + j);
    const int4 pb = *reinterpret_cast<const int4 *>(perm + j + 4);
    const half_t *row = x + (size_t)m * K;
    const half8_t v = {row[pa.x], row[pa.y], row[pa.z], row[pa.w], row[pb.x], row[pb.y], row[pb.z], row[pb.w]};
    *reinterpret_cast<half8_t *>(xp + (size_t)m * K + j) = v;
}

unsigned blocks_for(long long items)
{
    return (unsigned)((items + kThreads - 1) / kThreads);
}

}  // namespace

hipError_t launch_rank_rows(const int32_t *g_idx, int32_t *perm, int K, int group_size, int *status, hipStream_t stream)
{
    hipLaunchKernelGGL(rank_rows_kernel, dim3(blocks_for(K)), dim3(kThreads), 0, stream, g_idx, perm, K,
                       K / group_size, group_size, status);
    return hipGetLastError();
}

hipError_t launch_sort_rows(const uint32_t *qweight, const int32_t *perm, uint32_t *sorted, int K, int N,
                            hipStream_t stream)
{
    const int rows = K / 8;
    hipLaunchKernelGGL(sort_rows_kernel, dim3(blocks_for((long long)rows * (N / 4))), dim3(kThreads), 0, stream,
                       qweight, perm, sorted, rows, N);
    return hipGetLastError();
}

hipError_t launch_gather_activations(const half_t *x, const int32_t *perm, half_t *xp, int M, int K,
                                     hipStream_t stream)
{
    hipLaunchKernelGGL(gather_activations_kernel, dim3(blocks_for((long long)M * (K / 8))), dim3(kThreads), 0,
                       stream, x, perm, xp, M, K);
    return hipGetLastError();
}

}  // namespace gptq

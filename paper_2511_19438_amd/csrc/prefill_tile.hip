// Instantiates the MFMA kernels for ONE tile configuration (GPTQ_PREFILL_TILE, set on the compiler
// command line) so that the configurations compile in parallel.
#include "prefill_kernel.h"

#ifndef GPTQ_PREFILL_TILE
#error "compile with -DGPTQ_PREFILL_TILE=<1|3|5|8>"
#endif

namespace gptq {
namespace prefill {

template <int TILE>
hipError_t launch_tile(const Args &a, int mode, hipStream_t stream);

namespace {

// rows x columns per workgroup, wavefront grid, k per stage, stage buffers in the LDS ring
#if GPTQ_PREFILL_TILE == 1
constexpr int BM = 256, BN = 256, WM = 1, WN = 4, BK = 64, NBUF = 3;
#elif GPTQ_PREFILL_TILE == 3
constexpr int BM = 128, BN = 128, WM = 2, WN = 2, BK = 64, NBUF = 3;
#elif GPTQ_PREFILL_TILE == 5
constexpr int BM = 64, BN = 128, WM = 1, WN = 4, BK = 64, NBUF = 4;
#elif GPTQ_PREFILL_TILE == 8
constexpr int BM = 128, BN = 256, WM = 1, WN = 4, BK = 64, NBUF = 3;
#else
#error "unknown tile id"
#endif

template <typename Kernel>
hipError_t launch(Kernel kernel, Args a, size_t lds, bool may_split, hipStream_t stream)
{
    a.tiles_m = (a.M + BM - 1) / BM;
    a.tiles_n = (a.N + BN - 1) / BN;
    const int total = a.tiles_m * a.tiles_n;
    // the requested split, in whole stages of this tile's BK
    const int all_stages = (a.K + BK - 1) / BK;
    int split = (may_split && a.split_k > 1) ? (a.split_k < all_stages ? a.split_k : all_stages) : 1;
    a.stages_per_slice = (all_stages + split - 1) / split;
    split = (all_stages + a.stages_per_slice - 1) / a.stages_per_slice;
    a.split_k = split;
    const unsigned grid = 8u * (unsigned)((total + 7) / 8) * (unsigned)split;
    if (lds > 48 * 1024) {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (err != hipSuccess)
            return err;
    }
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(kThreads), lds, stream, a);
    return hipGetLastError();
}

}  // namespace

template <>
hipError_t launch_tile<GPTQ_PREFILL_TILE>(const Args &a, int mode, hipStream_t stream)
{
    if (mode == kGroupPerStage)
        return launch(prefill_pipelined_kernel<BM, BN, WM, WN, BK, NBUF>, a,
                      (size_t)NBUF * StageLayout<BM, BN, BK>::BYTES, true, stream);
#if GPTQ_PREFILL_TILE == 3
    const size_t lds = 2 * (size_t)BM * 64 * sizeof(half_t);
    if (mode == kGroupPerRow)
        return launch(prefill_general_kernel<BM, BN, WM, WN, kGroupPerRow>, a, lds, false, stream);
    if (mode == kActOrder)
        return launch(prefill_general_kernel<BM, BN, WM, WN, kActOrder>, a, lds, false, stream);
#endif
    return hipErrorInvalidValue;
}

}  // namespace prefill
}  // namespace gptq

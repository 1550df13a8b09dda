// Instantiates the split-K vector kernel for ONE batch size (GPTQ_DECODE_MB, set on the
// compiler command line: 1, 2, 4, 8 or 16) so that the five sizes compile in parallel.
#include "decode_kernel.h"

#ifndef GPTQ_DECODE_MB
#error "compile with -DGPTQ_DECODE_MB=<1|2|4|8|16>"
#endif

namespace gptq {
namespace decode {

namespace {

template <int MB, int LPR, int R, bool ACT, int ABL = 0>
hipError_t launch_one(const Args &a, size_t lds_bytes, hipStream_t stream)
{
    auto kernel = decode_kernel<MB, LPR, R, ACT, ABL>;
    if (lds_bytes > 48 * 1024) {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (err != hipSuccess)
            return err;
    }
    constexpr unsigned threads = (ABL & kEightWaves) ? 512 : 256;
    hipLaunchKernelGGL(kernel, dim3((unsigned)(a.tiles_n * a.split_k)), dim3(threads), lds_bytes, stream, a);
    return hipGetLastError();
}

// the plain format with chunks of four packed rows, any tile width
template <int MB, int ABL>
hipError_t launch_lpr(const Args &a, int lpr, size_t lds_bytes, hipStream_t stream)
{
    switch (lpr) {
    case 4: return launch_one<MB, 4, 4, false, ABL>(a, lds_bytes, stream);
    case 8: return launch_one<MB, 8, 4, false, ABL>(a, lds_bytes, stream);
    case 16: return launch_one<MB, 16, 4, false, ABL>(a, lds_bytes, stream);
    case 32: return launch_one<MB, 32, 4, false, ABL>(a, lds_bytes, stream);
    case 64: return launch_one<MB, 64, 4, false, ABL>(a, lds_bytes, stream);
    default: return hipErrorInvalidValue;
    }
}

// ABL, or ABL with eight wavefronts (single-row kernel only)
template <int MB, int ABL>
hipError_t launch_lpr_waves(const Args &a, int lpr, bool eight_waves, size_t lds_bytes, hipStream_t stream)
{
    if constexpr (MB == 1) {
        if (eight_waves)
            return launch_lpr<MB, ABL | kEightWaves>(a, lpr, lds_bytes, stream);
    }
    return eight_waves ? hipErrorInvalidValue : launch_lpr<MB, ABL>(a, lpr, lds_bytes, stream);
}

// the same for the one tile width (64 columns) the ablation variants exist for
template <int MB, int ABL>
hipError_t launch_64_waves(const Args &a, bool eight_waves, size_t lds_bytes, hipStream_t stream)
{
    if constexpr (MB == 1) {
        if (eight_waves)
            return launch_one<MB, 16, 4, false, ABL | kEightWaves>(a, lds_bytes, stream);
    }
    return eight_waves ? hipErrorInvalidValue : launch_one<MB, 16, 4, false, ABL>(a, lds_bytes, stream);
}

// (a template, so that the branches a batch size has no kernels for are discarded, not instantiated)
template <int MB>
hipError_t dispatch(const Args &a, int lpr, int chunk_rows, bool act, int variant, size_t lds_bytes, hipStream_t stream)
{
    const bool eight_waves = (variant & kEightWaves) != 0;
    const bool gather = (variant & kGatherX) != 0;
    const bool vector_dot = (variant & kMatrixDot) != 0;  // as a plan flag this bit asks for the v_dot2 loop
    const int ablate = variant & 7;
    if ((eight_waves || gather) && (MB != 1 || act || chunk_rows != 4))
        return hipErrorInvalidValue;
    if (gather) {  // activations gathered while staged: the default inner loop only
        if constexpr (MB == 1) {
            if (!ablate && !vector_dot)
                return launch_lpr_waves<MB, kMatrixDot | kGatherX>(a, lpr, eight_waves, lds_bytes, stream);
        }
        return hipErrorInvalidValue;
    }
    if (ablate != 0) {
        // the ablation variants exist for the default tile shape of the plain format, up to four rows; taking
        // the packed arithmetic out (kNoIla) replaces the whole inner loop, the other two keep the matrix-unit one
        if (MB > 4 || act || lpr != 16 || chunk_rows != 4)
            return hipErrorInvalidValue;
        if constexpr (MB <= 4) {
            switch (ablate) {
            case 1: return launch_64_waves<MB, 1 | kMatrixDot>(a, eight_waves, lds_bytes, stream);
            case 2: return launch_64_waves<MB, 2 | kMatrixDot>(a, eight_waves, lds_bytes, stream);
            case 3: return launch_64_waves<MB, 3 | kMatrixDot>(a, eight_waves, lds_bytes, stream);
            case 4: return launch_64_waves<MB, 4>(a, eight_waves, lds_bytes, stream);
            case 5: return launch_64_waves<MB, 5>(a, eight_waves, lds_bytes, stream);
            case 6: return launch_64_waves<MB, 6>(a, eight_waves, lds_bytes, stream);
            default: return launch_64_waves<MB, 7>(a, eight_waves, lds_bytes, stream);
            }
        }
        return hipErrorInvalidValue;
    }
    if (act) {
        if (lpr == 16 && chunk_rows == 4)
            return launch_one<MB, 16, 4, true>(a, lds_bytes, stream);
        return hipErrorInvalidValue;
    }
    if (chunk_rows == 4) {
        // Up to four batch rows the inner loop contracts on the matrix unit (kMatrixDot): measured 3-6 % faster
        // than v_dot2_f32_f16 at M = 1, which stays as a comparison switch and for the larger batches.
        if constexpr (MB == 1) {
            if (!vector_dot && (variant & kGroupCorr))
                return launch_lpr_waves<MB, kMatrixDot | kGroupCorr>(a, lpr, eight_waves, lds_bytes, stream);
        }
        if constexpr (MB <= 4) {
            if (!vector_dot)
                return launch_lpr_waves<MB, kMatrixDot>(a, lpr, eight_waves, lds_bytes, stream);
        }
        return launch_lpr_waves<MB, 0>(a, lpr, eight_waves, lds_bytes, stream);
    }
    if (lpr != 16)
        return hipErrorInvalidValue;
    if (chunk_rows == 2)
        return launch_one<MB, 16, 2, false>(a, lds_bytes, stream);
    if (chunk_rows == 1)
        return launch_one<MB, 16, 1, false>(a, lds_bytes, stream);
    return hipErrorInvalidValue;
}

}  // namespace

template <>
hipError_t launch_mb<GPTQ_DECODE_MB>(const Args &a, int lpr, int chunk_rows, bool act, int variant, size_t lds_bytes,
                                     hipStream_t stream)
{
    return dispatch<GPTQ_DECODE_MB>(a, lpr, chunk_rows, act, variant, lds_bytes, stream);
}

}  // namespace decode
}  // namespace gptq

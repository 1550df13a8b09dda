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
    hipLaunchKernelGGL(kernel, dim3((unsigned)(a.tiles_n * a.split_k)), dim3(64 * waves_for(MB, ACT)), lds_bytes, stream, a);
    return hipGetLastError();
}

}  // namespace

template <>
hipError_t launch_mb<GPTQ_DECODE_MB>(const Args &a, int lpr, int chunk_rows, bool act, int ablate, size_t lds_bytes,
                                     hipStream_t stream)
{
    constexpr int MB = GPTQ_DECODE_MB;
    // The inner loop of the plain format with chunks of four packed rows, up to four batch rows, contracts on
    // the matrix unit (kMatrixDot); measured 3-6 % faster than v_dot2_f32_f16 at M = 1.
#if GPTQ_DECODE_MB == 1
    if (ablate & kGatherX) {  // activations gathered while staged: the default inner loop only
        if (ablate != kGatherX || act || chunk_rows != 4)
            return hipErrorInvalidValue;
        switch (lpr) {
        case 4: return launch_one<MB, 4, 4, false, kMatrixDot | kGatherX>(a, lds_bytes, stream);
        case 8: return launch_one<MB, 8, 4, false, kMatrixDot | kGatherX>(a, lds_bytes, stream);
        case 16: return launch_one<MB, 16, 4, false, kMatrixDot | kGatherX>(a, lds_bytes, stream);
        case 32: return launch_one<MB, 32, 4, false, kMatrixDot | kGatherX>(a, lds_bytes, stream);
        case 64: return launch_one<MB, 64, 4, false, kMatrixDot | kGatherX>(a, lds_bytes, stream);
        default: return hipErrorInvalidValue;
        }
    }
#endif
#if GPTQ_DECODE_MB <= 4
    const bool vector_dot = (ablate & 8) != 0;  // comparison switch: keep the v_dot2_f32_f16 loop
    ablate &= 7;
    if (ablate == 0 && !vector_dot && !act && chunk_rows == 4) {
        switch (lpr) {
        case 4: return launch_one<MB, 4, 4, false, kMatrixDot>(a, lds_bytes, stream);
        case 8: return launch_one<MB, 8, 4, false, kMatrixDot>(a, lds_bytes, stream);
        case 16: return launch_one<MB, 16, 4, false, kMatrixDot>(a, lds_bytes, stream);
        case 32: return launch_one<MB, 32, 4, false, kMatrixDot>(a, lds_bytes, stream);
        case 64: return launch_one<MB, 64, 4, false, kMatrixDot>(a, lds_bytes, stream);
        default: return hipErrorInvalidValue;
        }
    }
#endif
    if (ablate & kGatherX)
        return hipErrorInvalidValue;
    if (ablate != 0) {
        // the ablation variants exist for the default tile shape of the plain format, up to four rows; taking
        // the packed arithmetic out (kNoIla) replaces the whole inner loop, the other two keep the matrix-unit one
#if GPTQ_DECODE_MB <= 4
        if (act || lpr != 16 || chunk_rows != 4)
            return hipErrorInvalidValue;
        switch (ablate & 7) {
        case 1: return launch_one<MB, 16, 4, false, 1 | kMatrixDot>(a, lds_bytes, stream);
        case 2: return launch_one<MB, 16, 4, false, 2 | kMatrixDot>(a, lds_bytes, stream);
        case 3: return launch_one<MB, 16, 4, false, 3 | kMatrixDot>(a, lds_bytes, stream);
        case 4: return launch_one<MB, 16, 4, false, 4>(a, lds_bytes, stream);
        case 5: return launch_one<MB, 16, 4, false, 5>(a, lds_bytes, stream);
        case 6: return launch_one<MB, 16, 4, false, 6>(a, lds_bytes, stream);
        case 7: return launch_one<MB, 16, 4, false, 7>(a, lds_bytes, stream);
        default: return hipErrorInvalidValue;
        }
#else
        return hipErrorInvalidValue;
#endif
    }
    if (act) {
        if (lpr == 16 && chunk_rows == 4)
            return launch_one<MB, 16, 4, true>(a, lds_bytes, stream);
        return hipErrorInvalidValue;
    }
    if (chunk_rows == 4) {
        switch (lpr) {
        case 4: return launch_one<MB, 4, 4, false>(a, lds_bytes, stream);
        case 8: return launch_one<MB, 8, 4, false>(a, lds_bytes, stream);
        case 16: return launch_one<MB, 16, 4, false>(a, lds_bytes, stream);
        case 32: return launch_one<MB, 32, 4, false>(a, lds_bytes, stream);
        case 64: return launch_one<MB, 64, 4, false>(a, lds_bytes, stream);
        default: return hipErrorInvalidValue;
        }
    }
    if (lpr != 16)
        return hipErrorInvalidValue;
    if (chunk_rows == 2)
        return launch_one<MB, 16, 2, false>(a, lds_bytes, stream);
    if (chunk_rows == 1)
        return launch_one<MB, 16, 1, false>(a, lds_bytes, stream);
    return hipErrorInvalidValue;
}

}  // namespace decode
}  // namespace gptq

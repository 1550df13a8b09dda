// Host side of the small-batch MFMA kernel: support check, launch plan, scratch sizing, dispatch.
#include "skinny_kernel.h"

namespace gptq {

namespace {

constexpr int kMaxActivationLdsBytes = 64 * 1024;
constexpr size_t kCounterBytes = 256 * 1024;  // same fixed counter area as the vector kernel
constexpr int kMaxColumnTiles = (int)(kCounterBytes / sizeof(unsigned));

int ceil_div(int a, int b)
{
    return (a + b - 1) / b;
}

int row_blocks(int M)
{
    return M <= 16 ? 1 : (M <= 32 ? 2 : 4);
}

template <int TM, int WN>
hipError_t launch_tm(const skinny::Args &a, size_t lds, hipStream_t stream)
{
    auto kernel = skinny::skinny_kernel<TM, WN>;
    if (lds > 48 * 1024) {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (err != hipSuccess)
            return err;
    }
    hipLaunchKernelGGL(kernel, dim3((unsigned)(a.tiles_n * a.split_k)), dim3(skinny::kThreads), lds, stream, a);
    return hipGetLastError();
}

}  // namespace

bool skinny_supported(const Problem &p)
{
    return p.g_idx == nullptr && p.M >= 1 && p.M <= kSkinnyMaxM && p.group_size % 128 == 0 && p.N >= 8 &&
           ceil_div(p.N, skinny::kCols) <= kMaxColumnTiles;
}

void skinny_make_plan(const Problem &p, SkinnyPlan &plan)
{
    const int rows = 16 * row_blocks(p.M);
    const int total_units = p.K / skinny::kUnitK;
    int max_units = kMaxActivationLdsBytes / (rows * 2) / skinny::kUnitK;  // activations of a slice must fit LDS
    if (max_units < 1)
        max_units = 1;
    if (plan.cols_per_wg != 64 && plan.cols_per_wg != 256) {
        // Wide tiles stage the activations once for four times as many weights, but a workgroup's wavefronts
        // then walk the whole slice: that only pays (measured) once the columns alone spread over most of
        // the chip.
        plan.cols_per_wg = ceil_div(p.N, 256) >= 192 ? 256 : 64;
    }
    const int tiles_n = ceil_div(p.N, plan.cols_per_wg);
    const int quantum = plan.cols_per_wg == 64 ? 4 : 1;  // narrow tiles: one unit per wavefront and turn
    int ups;
    if (plan.split_k > 0) {
        ups = ceil_div(total_units, plan.split_k < total_units ? plan.split_k : total_units);
    } else {
        // Workgroup count as close to the target as possible - but the fp32 partial sums that the slices
        // exchange through scratch (8 bytes per slice and output: written once, read once) may not exceed a
        // quarter of the packed weight bytes (K*N/2), or they, not the weights, set the time:
        // split * M * N * 8 <= K * N / 8.
        int max_split = p.K / (64 * p.M);
        if (max_split < 1)
            max_split = 1;
        const int min_units = ceil_div(total_units, max_split);
        const double target = plan.cols_per_wg == 64 ? 768.0 : 512.0;
        ups = 0;
        double best = 0.0;
        for (int c = quantum; c <= total_units + quantum - 1; c += quantum) {
            const int cand = c < total_units ? c : total_units;
            if (cand > max_units && ups)
                break;
            if (cand < min_units && cand < max_units && cand < total_units)
                continue;
            const double wgs = (double)tiles_n * ceil_div(total_units, cand);
            const double ratio = wgs > target ? wgs / target : target / wgs;
            if (!ups || ratio < best - 1e-9) {
                ups = cand;
                best = ratio;
            }
            if (cand == total_units)
                break;
        }
    }
    if (ups > max_units)
        ups = max_units;
    if (ups < 1)
        ups = 1;
    plan.units_per_slice = ups;
    plan.split_k = ceil_div(total_units, ups);
}

size_t skinny_workspace_bytes(const Problem &p, const SkinnyPlan &plan)
{
    size_t bytes = kCounterBytes;
    if (plan.split_k > 1)
        bytes += (size_t)plan.split_k * p.M * p.N * sizeof(float);
    return bytes;
}

hipError_t launch_skinny(const Problem &p, const SkinnyPlan &plan, void *workspace, hipStream_t stream)
{
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    skinny::Args a;
    a.x = p.x;
    a.qweight = p.qweight;
    a.qzeros = p.qzeros;
    a.scales = p.scales;
    a.out = p.out;
    a.counters = reinterpret_cast<unsigned *>(ws);
    a.partial = reinterpret_cast<float *>(ws + kCounterBytes);
    a.M = p.M;
    a.K = p.K;
    a.N = p.N;
    a.units_per_group = p.group_size / skinny::kUnitK;
    a.unit_group_shift = -1;
    for (int sh = 0; sh < 20; ++sh)
        if ((1 << sh) == a.units_per_group)
            a.unit_group_shift = sh;
    const int wn = plan.cols_per_wg / skinny::kCols;
    a.tiles_n = ceil_div(p.N, plan.cols_per_wg);
    a.split_k = plan.split_k;
    a.units_per_slice = plan.units_per_slice;
    a.total_units = p.K / skinny::kUnitK;

    const int tm = row_blocks(p.M);
    const int rows = 16 * tm;
    const size_t xs = (size_t)rows * plan.units_per_slice * skinny::kUnitK * sizeof(half_t);
    const size_t red = (size_t)skinny::kWaves * rows * skinny::kCols * sizeof(float);  // [4/wn][rows][64*wn]
    const size_t lds = xs > red ? xs : red;
    if (wn == 4) {
        switch (tm) {
        case 1: return launch_tm<1, 4>(a, lds, stream);
        case 2: return launch_tm<2, 4>(a, lds, stream);
        default: return launch_tm<4, 4>(a, lds, stream);
        }
    }
    switch (tm) {
    case 1: return launch_tm<1, 1>(a, lds, stream);
    case 2: return launch_tm<2, 1>(a, lds, stream);
    default: return launch_tm<4, 1>(a, lds, stream);
    }
}

}  // namespace gptq

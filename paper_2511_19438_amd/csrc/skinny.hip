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

// Batches of more than 64 rows are processed 64 rows at a time (one launch each, same stream): the weights
// are streamed once per launch, the second time mostly from the memory-side cache.
constexpr int kRowsPerLaunch = 64;

int row_blocks(int M)
{
    return M <= 16 ? 1 : M <= 32 ? 2 : 4;
}

int rows_of_launch(int M)
{
    return M < kRowsPerLaunch ? M : kRowsPerLaunch;
}

// Wavefronts per workgroup: eight where the 64-column workgroups have a compute unit each, else four.
int waves_of(int tiles_n, int split_k, int wn, int tm)
{
    if (wn == 2)
        return 8;  // 128-column workgroups: two column blocks of four wavefronts
    // (four row blocks do not fit the 256 registers that two wavefronts per SIMD leave each)
    return (wn == 1 && tm <= 2 && (long long)tiles_n * split_k <= 256) ? 8 : 4;
}

template <int TM, int WN, int WAVES, int GPU = 1>
hipError_t launch_tm(const skinny::Args &a, size_t lds, hipStream_t stream)
{
    auto kernel = skinny::skinny_kernel<TM, WN, WAVES, GPU>;
    if (lds > 48 * 1024) {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (err != hipSuccess)
            return err;
    }
    hipLaunchKernelGGL(kernel, dim3((unsigned)(a.tiles_n * a.split_k)), dim3(64 * WAVES), lds, stream, a);
    return hipGetLastError();
}

}  // namespace

bool skinny_supported(const Problem &p)
{
    if (p.g_idx != nullptr || p.M < 1 || p.M > kSkinnyMaxM || p.N < 8 || p.K % skinny::kUnitK != 0 ||
        ceil_div(p.N, skinny::kCols) > kMaxColumnTiles)
        return false;
    // groups of 64 and 32 k: the 64-column kernel with up to two row blocks
    if (p.group_size == 64 || p.group_size == 32)
        return p.M <= 32;
    return p.group_size % 128 == 0;
}

void skinny_make_plan(const Problem &p, SkinnyPlan &plan)
{
    const int launch_m = rows_of_launch(p.M);
    const int rows = 16 * row_blocks(launch_m);
    const int total_units = p.K / skinny::kUnitK;
    if (p.group_size < skinny::kUnitK)
        plan.cols_per_wg = 64;  // the small-group variants exist for the 64-column workgroup
    const bool wide_ok = rows <= 32;  // the 128-column workgroup exists for one and two row blocks
    if (plan.cols_per_wg == 128 && !wide_ok)
        plan.cols_per_wg = 0;
    if (plan.cols_per_wg != 64 && plan.cols_per_wg != 128 && plan.cols_per_wg != 256) {
        // Wide tiles stage the activations once for four times as many weights, but a workgroup's wavefronts
        // then walk the whole slice: that only pays (measured) once the columns alone spread over most of
        // the chip.  In between - more 64-column tiles than compute units, but no more 128-column ones - two
        // column blocks share a workgroup of eight wavefronts, so that every compute unit has one workgroup
        // instead of some having two.
        const int tiles64 = ceil_div(p.N, 64);
        plan.cols_per_wg = ceil_div(p.N, 256) >= 192 ? 256 : (wide_ok && tiles64 > 256 && ceil_div(p.N, 128) <= 256) ? 128 : 64;
    }
    // where the activations of a slice are staged in LDS (wide tiles, more than 32 rows) they must fit
    const bool direct = plan.cols_per_wg <= 128;
    int max_units = direct ? total_units : kMaxActivationLdsBytes / (rows * 2) / skinny::kUnitK;
    if (max_units < 1)
        max_units = 1;
    const int tiles_n = ceil_div(p.N, plan.cols_per_wg);
    int ups;
    if (plan.split_k > 0) {
        ups = ceil_div(total_units, plan.split_k < total_units ? plan.split_k : total_units);
    } else {
        // One workgroup per compute unit is the target (measured: 192..344 unsplit workgroups beat any split
        // of the same layer, and narrow layers want tiles * split = 256) - but the fp32 partial sums that the
        // slices exchange through scratch (8 bytes per slice and output: written once, read once) may not
        // exceed half of the packed weight bytes (K*N/2), or they, not the weights, set the time:
        // split * M * N * 8 <= K * N / 4 (measured on 4096x4096 at 24-32 rows: four slices 8.6-9.1 us, two
        // slices 9.7-10.5).  Slices are whole multiples of `quantum` units.
        int max_split = p.K / (32 * launch_m);
        if (max_split < 1)
            max_split = 1;
        int split = (256 + tiles_n / 2) / tiles_n;
        // A few workgroups more than compute units is the worst case (four-wavefront workgroups, some units with
        // two of them): 160 tiles x 2 slices on 8192x10240 measured 15.2 us at M = 2 against 13.4 unsplit.
        if (tiles_n > 128)
            split = 1;
        if (plan.cols_per_wg == 256) {
            // wide tiles (very wide layers): eight slices, within a quarter of the weight bytes for the partial
            // sums (8192x57344 at M = 2: 46.1 us with eight slices, 49.9 with four)
            split = 8;
            max_split = p.K / (64 * launch_m);
            if (max_split < 1)
                max_split = 1;
        }
        if (split > max_split)
            split = max_split;
        if (split < 1)
            split = 1;
        // narrow tiles: one unit per wavefront and turn
        const int quantum = plan.cols_per_wg == 64 ? waves_of(tiles_n, split, 1, row_blocks(launch_m))
                                                   : plan.cols_per_wg == 128 ? 4 : 1;
        ups = ceil_div(ceil_div(total_units, split), quantum) * quantum;
        if (ups > total_units)
            ups = total_units;
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
        bytes += (size_t)plan.split_k * rows_of_launch(p.M) * p.N * sizeof(float);
    return bytes;
}

hipError_t launch_skinny(const Problem &p, const SkinnyPlan &plan, void *workspace, hipStream_t stream)
{
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    const int wn = plan.cols_per_wg / skinny::kCols;
    for (int m0 = 0; m0 < p.M; m0 += kRowsPerLaunch) {
        skinny::Args a;
        a.x = p.x + (size_t)m0 * p.K;
        a.qweight = p.qweight;
        a.qzeros = p.qzeros;
        a.scales = p.scales;
        a.out = p.out + (size_t)m0 * p.N;
        a.counters = reinterpret_cast<unsigned *>(ws);
        a.partial = reinterpret_cast<float *>(ws + kCounterBytes);
        a.M = (p.M - m0) < kRowsPerLaunch ? (p.M - m0) : kRowsPerLaunch;
        a.K = p.K;
        a.N = p.N;
        a.units_per_group = p.group_size >= skinny::kUnitK ? p.group_size / skinny::kUnitK : 1;
        a.unit_group_shift = -1;
        for (int sh = 0; sh < 20; ++sh)
            if ((1 << sh) == a.units_per_group)
                a.unit_group_shift = sh;
        a.tiles_n = ceil_div(p.N, plan.cols_per_wg);
        a.split_k = plan.split_k;
        a.units_per_slice = plan.units_per_slice;
        a.total_units = p.K / skinny::kUnitK;

        const int tm = row_blocks(a.M);
        const int rows = 16 * tm;
        // 64- and 128-column workgroups read the activations straight from global memory
        const bool direct = wn <= 2;
        const size_t xs = direct ? 0 : (size_t)rows * plan.units_per_slice * skinny::kUnitK * sizeof(half_t);
        const int waves = waves_of(a.tiles_n, a.split_k, wn, tm);
        const size_t red = (size_t)waves * rows * skinny::kCols * sizeof(float);  // [waves/wn][rows][64*wn]
        const size_t lds = xs > red ? xs : red;
        hipError_t err;
        const int gpu = p.group_size >= skinny::kUnitK ? 1 : skinny::kUnitK / p.group_size;
        if (gpu > 1) {
            if (wn != 1 || tm > 2)
                return hipErrorInvalidValue;  // refused by skinny_supported / skinny_make_plan
            if (gpu == 2)
                err = waves == 8 ? (tm == 1 ? launch_tm<1, 1, 8, 2>(a, lds, stream) : launch_tm<2, 1, 8, 2>(a, lds, stream))
                                 : (tm == 1 ? launch_tm<1, 1, 4, 2>(a, lds, stream) : launch_tm<2, 1, 4, 2>(a, lds, stream));
            else
                err = waves == 8 ? (tm == 1 ? launch_tm<1, 1, 8, 4>(a, lds, stream) : launch_tm<2, 1, 8, 4>(a, lds, stream))
                                 : (tm == 1 ? launch_tm<1, 1, 4, 4>(a, lds, stream) : launch_tm<2, 1, 4, 4>(a, lds, stream));
        } else if (wn == 2) {
            if (tm > 2)
                return hipErrorInvalidValue;  // refused by skinny_make_plan
            err = tm == 1 ? launch_tm<1, 2, 8>(a, lds, stream) : launch_tm<2, 2, 8>(a, lds, stream);
        } else if (wn == 4)
            err = tm == 1 ? launch_tm<1, 4, 4>(a, lds, stream)
                          : tm == 2 ? launch_tm<2, 4, 4>(a, lds, stream) : launch_tm<4, 4, 4>(a, lds, stream);
        else if (waves == 8)
            err = tm == 1 ? launch_tm<1, 1, 8>(a, lds, stream) : launch_tm<2, 1, 8>(a, lds, stream);
        else
            err = tm == 1 ? launch_tm<1, 1, 4>(a, lds, stream)
                          : tm == 2 ? launch_tm<2, 1, 4>(a, lds, stream) : launch_tm<4, 1, 4>(a, lds, stream);
        if (err != hipSuccess)
            return err;
    }
    return hipSuccess;
}

}  // namespace gptq

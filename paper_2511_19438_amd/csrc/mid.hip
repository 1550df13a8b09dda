// Host side of the mid-batch streaming MFMA kernel: support check, launch plan, scratch sizing, dispatch.
#include "mid_kernel.h"

namespace gptq {

namespace {

constexpr size_t kCounterBytes = 256 * 1024;  // same fixed counter area as the other kernels
constexpr int kMaxColumnTiles = (int)(kCounterBytes / sizeof(unsigned));

int ceil_div(int a, int b)
{
    return (a + b - 1) / b;
}

int row_blocks(int M)
{
    return M <= 32 ? 1 : M <= 64 ? 2 : 4;
}

// Wavefronts per workgroup: eight (two per SIMD) where their activation rings fit the LDS, else four.
int waves_of(int tmb)
{
    return tmb <= 2 ? 8 : 4;
}

template <int TMB, int NB, int WAVES>
hipError_t launch_one(const mid::Args &a, hipStream_t stream)
{
    auto kernel = mid::mid_kernel<TMB, NB, WAVES>;
    const size_t lds = (size_t)WAVES * 2 * (32 * TMB) * 128;
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

bool mid_supported(const Problem &p)
{
    if (p.g_idx != nullptr || p.M < 1 || p.M > kMidMaxM || p.N < 8 || p.K % mid::kStageK != 0 ||
        p.group_size % mid::kStageK != 0 || ceil_div(p.N, 64) > kMaxColumnTiles)
        return false;
    // the kernel divides stage numbers by the stages per group with one multiply-high, which is exact while
    // stages * stages per group stays below 2^32
    return (long long)(p.K / mid::kStageK) * (p.group_size / mid::kStageK) < (1ll << 31);
}

void mid_make_plan(const Problem &p, MidPlan &plan)
{
    const int tmb = row_blocks(p.M);
    const int waves = waves_of(tmb);
    const int total = p.K / mid::kStageK;
    // four row blocks leave registers for two n-blocks only
    if (tmb == 4)
        plan.cols_per_wg = 64;
    if (plan.cols_per_wg != 64 && plan.cols_per_wg != 128) {
        // 128-column tiles where they alone give most compute units a workgroup, or where K is so deep that the
        // exchange of a few more slices is cheap next to the loop (28672x8192 at 64 rows: 50.1 us with 64 tiles
        // in four slices, 54.2 with 128 tiles in two); else 64
        const int tiles128 = ceil_div(p.N, 128);
        plan.cols_per_wg = (tiles128 >= 160 || (tiles128 <= 64 && p.K >= 16384)) ? 128 : 64;
    }
    const int tiles_n = ceil_div(p.N, plan.cols_per_wg);
    int split = plan.split_k;
    if (split <= 0) {
        // one workgroup per compute unit (their activation rings fill its LDS: workgroups beyond 256 wait for a
        // second round); every wavefront should keep at least two stages
        split = 256 / tiles_n;
        const int max_split = total / (2 * waves);
        if (split > max_split)
            split = max_split;
        if (split < 1)
            split = 1;
    }
    if (split > total)
        split = total;
    const int sps = ceil_div(total, split);
    plan.stages_per_slice = sps;
    plan.split_k = ceil_div(total, sps);
}

size_t mid_workspace_bytes(const Problem &p, const MidPlan &plan)
{
    size_t bytes = kCounterBytes;
    if (plan.split_k > 1)
        bytes += (size_t)plan.split_k * p.M * p.N * sizeof(float);
    return bytes;
}

hipError_t launch_mid(const Problem &p, const MidPlan &plan, void *workspace, hipStream_t stream)
{
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    mid::Args a;
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
    const uint32_t stages_per_group = (uint32_t)(p.group_size / mid::kStageK);
    a.group_mul = stages_per_group == 1 ? 0u : (uint32_t)(0x100000000ull / stages_per_group) + 1u;
    a.group_one = stages_per_group == 1 ? 1u : 0u;
    a.tiles_n = ceil_div(p.N, plan.cols_per_wg);
    a.split_k = plan.split_k;
    a.stages_per_slice = plan.stages_per_slice;
    a.total_stages = p.K / mid::kStageK;
    const int tmb = row_blocks(p.M);
    if (plan.cols_per_wg == 128) {
        if (tmb == 1)
            return launch_one<1, 4, 8>(a, stream);
        if (tmb == 2)
            return launch_one<2, 4, 8>(a, stream);
        return hipErrorInvalidValue;  // refused by mid_make_plan
    }
    if (tmb == 1)
        return launch_one<1, 2, 8>(a, stream);
    if (tmb == 2)
        return launch_one<2, 2, 8>(a, stream);
    return launch_one<4, 2, 4>(a, stream);
}

}  // namespace gptq

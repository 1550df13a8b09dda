// Internal launcher interface between the C-ABI translation unit and the kernel files.
// Everything here is device-pointer based; shapes were validated by the caller.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gptq {

using half_t = _Float16;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));

struct Problem {
    const half_t *x;          // [M, K]
    const uint32_t *qweight;  // [K/8, N]
    const uint32_t *qzeros;   // [K/group, N/8]
    const half_t *scales;     // [K/group, N]
    const int32_t *g_idx;     // [K] or nullptr
    const int32_t *x_perm = nullptr;  // [K]: gather x through it while staging (vector kernel, M = 1 only)
    half_t *out;              // [M, N]
    int M, K, N, group_size;
};

// ---- unpack / dequant (standalone, HBM-bound) ----
hipError_t launch_unpack(const uint32_t *qweight, uint8_t *q_out, const uint32_t *qzeros, uint8_t *z_out, int K,
                         int N, int group_size, hipStream_t stream);
hipError_t launch_shift_zeros(const uint32_t *in, uint32_t *out, long long words, int delta, hipStream_t stream);
hipError_t launch_dequant(const uint32_t *qweight, const uint32_t *qzeros, const half_t *scales,
                          const int32_t *g_idx, half_t *w_out, int K, int N, int group_size, hipStream_t stream);

// ---- act-order repack (one-time) and the activation gather of the repacked path ----
// `status` is a device int that must be zero before the call; see the kernel for its bits.
hipError_t launch_rank_rows(const int32_t *g_idx, int32_t *perm, int K, int group_size, int *status, hipStream_t stream);
hipError_t launch_sort_rows(const uint32_t *qweight, const int32_t *perm, uint32_t *sorted, int K, int N,
                            hipStream_t stream);
hipError_t launch_gather_activations(const half_t *x, const int32_t *perm, half_t *xp, int M, int K,
                                     hipStream_t stream);

// ---- decode: split-K vector kernel, M <= 16 per launch ----
struct DecodePlan {
    int cols_per_wg;   // 16, 32, 64, 128 or 256
    int split_k;       // number of K slices
    int chunk_rows;    // packed rows handled per lane per step (1, 2 or 4), divides group_size/8
    int chunks_per_slice;
    int flags;         // ablation switches (bit 0: no on-chip reduction, 1: scalar activation loads, 2: scalar fp32 math)
};
// Fills `plan` (honouring non-zero requests in it) for the problem.
void decode_make_plan(const Problem &p, DecodePlan &plan);
// Bytes of scratch (partials + counters) the plan needs; counter area comes first.
size_t decode_workspace_bytes(const Problem &p, const DecodePlan &plan);
size_t decode_counter_bytes(int N);
hipError_t launch_decode(const Problem &p, const DecodePlan &plan, void *workspace, hipStream_t stream);
// Whether a workgroup of the planned launch fits the LDS (the act-order variant keeps a table of every group
// there, which very deep layers with small groups overflow).
bool decode_plan_fits(const Problem &p, const DecodePlan &plan);
// Whether the ablation variants of the vector kernel (DecodePlan::flags != 0) exist for this problem.
bool decode_ablation_supported(const Problem &p);

// ---- small batch: MFMA kernel with the vector kernel's split-K decomposition, M <= 128 (64 rows per launch) ----
constexpr int kSkinnyMaxM = 128;
struct SkinnyPlan {
    int cols_per_wg;      // 64 (wavefronts split the K slice), 128 (two column blocks, four wavefronts each split the slice)
                          // or 256 (four wavefronts side by side); 0 = choose
    int split_k;          // number of K slices (0 = choose)
    int units_per_slice;  // 128-k units per slice
};
bool skinny_supported(const Problem &p);
void skinny_make_plan(const Problem &p, SkinnyPlan &plan);
size_t skinny_workspace_bytes(const Problem &p, const SkinnyPlan &plan);
hipError_t launch_skinny(const Problem &p, const SkinnyPlan &plan, void *workspace, hipStream_t stream);

// ---- mid batch: streaming MFMA kernel, every wavefront on its own share of the K slice, M <= 128 ----
constexpr int kMidMaxM = 128;
struct MidPlan {
    int cols_per_wg;       // 64 or 128 (two or four 32-column n-blocks per wavefront); 0 = choose
    int split_k;           // number of K slices across workgroups (0 = choose)
    int stages_per_slice;  // 64-k stages per slice
};
bool mid_supported(const Problem &p);
void mid_make_plan(const Problem &p, MidPlan &plan);
size_t mid_workspace_bytes(const Problem &p, const MidPlan &plan);
hipError_t launch_mid(const Problem &p, const MidPlan &plan, void *workspace, hipStream_t stream);

// ---- prefill: fp16 MFMA kernel ----
struct PrefillPlan {
    int tile;     // tile configuration id (1-based), 0 = auto
    int split_k;  // K slices (pipelined kernel only), 0 = auto
};
bool prefill_supported(const Problem &p);
bool prefill_tile_exists(int tile);  // the tile ids a plan may name
void prefill_make_plan(const Problem &p, PrefillPlan &plan);
// Scratch of a plan with split_k > 1 (counter area first, as for the other kernels); 0 without a split.
size_t prefill_workspace_bytes(const Problem &p, const PrefillPlan &plan);
hipError_t launch_prefill(const Problem &p, const PrefillPlan &plan, void *workspace, hipStream_t stream);

}  // namespace gptq

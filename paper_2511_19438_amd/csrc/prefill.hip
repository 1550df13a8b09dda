// Host side of the MFMA kernel: tile selection and dispatch.
#include "prefill_kernel.h"

namespace gptq {

namespace prefill {
template <int TILE>
hipError_t launch_tile(const Args &a, int mode, hipStream_t stream);
template <> hipError_t launch_tile<1>(const Args &, int, hipStream_t);
template <> hipError_t launch_tile<2>(const Args &, int, hipStream_t);
template <> hipError_t launch_tile<3>(const Args &, int, hipStream_t);
template <> hipError_t launch_tile<4>(const Args &, int, hipStream_t);
template <> hipError_t launch_tile<5>(const Args &, int, hipStream_t);
template <> hipError_t launch_tile<6>(const Args &, int, hipStream_t);
template <> hipError_t launch_tile<7>(const Args &, int, hipStream_t);
template <> hipError_t launch_tile<8>(const Args &, int, hipStream_t);
template <> hipError_t launch_tile<9>(const Args &, int, hipStream_t);
template <> hipError_t launch_tile<10>(const Args &, int, hipStream_t);
}  // namespace prefill

namespace {

struct TileShape {
    int bm, bn;
    double rate;  // measured in-loop MFMA rate relative to the 256x256 tile with 2x2 wavefronts (0 = not auto-selected)
};
// ids 1..10, see the plan documentation in the public header
constexpr TileShape kTiles[11] = {{0, 0, 0.0},      {256, 256, 0.0},  {256, 128, 0.0},  {128, 128, 0.68},
                                  {128, 256, 0.0},  {64, 128, 0.45},  {32, 256, 0.30},  {256, 256, 0.0},
                                  {128, 256, 0.84}, {256, 256, 1.00}, {256, 256, 0.0}};
constexpr int kNumTiles = 10;
constexpr int kComputeUnits = 256;

int mode_of(const Problem &p)
{
    if (p.g_idx)
        return prefill::kActOrder;
    // the pipelined kernel moves 16-byte chunks of every operand row: rows of packed zero points (N/8 words)
    // are 16-byte aligned only when N is a multiple of 32
    return (p.group_size % 64 == 0 && p.N % 32 == 0) ? prefill::kGroupPerStage : prefill::kGroupPerRow;
}

}  // namespace

bool prefill_supported(const Problem &p)
{
    return p.M >= 1 && p.K % 8 == 0 && p.N % 8 == 0;
}

void prefill_make_plan(const Problem &p, PrefillPlan &plan)
{
    const int mode = mode_of(p);
    if (mode != prefill::kGroupPerStage) {
        plan.tile = 3;  // the general modes exist for one tile shape only
        return;
    }
    if (plan.tile >= 1 && plan.tile <= kNumTiles)
        return;
    // Pick the tile that minimises (rounds of workgroups over the chip) x (cost of one tile).
    double best = 0.0;
    int best_tile = 3;
    for (int t = 1; t <= kNumTiles; ++t) {
        const TileShape &ts = kTiles[t];
        if (ts.rate <= 0.0)
            continue;
        const long long tiles = (long long)((p.M + ts.bm - 1) / ts.bm) * ((p.N + ts.bn - 1) / ts.bn);
        const long long rounds = (tiles + kComputeUnits - 1) / kComputeUnits;
        const double cost = (double)rounds * ts.bm * ts.bn / ts.rate;
        if (best == 0.0 || cost < best) {
            best = cost;
            best_tile = t;
        }
    }
    plan.tile = best_tile;
}

hipError_t launch_prefill(const Problem &p, const PrefillPlan &plan, hipStream_t stream)
{
    prefill::Args a;
    a.x = p.x;
    a.qweight = p.qweight;
    a.qzeros = p.qzeros;
    a.scales = p.scales;
    a.g_idx = p.g_idx;
    a.out = p.out;
    a.M = p.M;
    a.K = p.K;
    a.N = p.N;
    a.group_size = p.group_size;
    a.tiles_m = a.tiles_n = 0;
    const int mode = mode_of(p);
    switch (plan.tile) {
    case 1: return prefill::launch_tile<1>(a, mode, stream);
    case 2: return prefill::launch_tile<2>(a, mode, stream);
    case 3: return prefill::launch_tile<3>(a, mode, stream);
    case 4: return prefill::launch_tile<4>(a, mode, stream);
    case 5: return prefill::launch_tile<5>(a, mode, stream);
    case 6: return prefill::launch_tile<6>(a, mode, stream);
    case 7: return prefill::launch_tile<7>(a, mode, stream);
    case 8: return prefill::launch_tile<8>(a, mode, stream);
    case 9: return prefill::launch_tile<9>(a, mode, stream);
    case 10: return prefill::launch_tile<10>(a, mode, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace gptq

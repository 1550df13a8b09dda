// Host side of the MFMA kernel: tile selection and dispatch.
#include "prefill_kernel.h"

#include <cmath>

namespace gptq {

namespace prefill {
template <int TILE>
hipError_t launch_tile(const Args &a, int mode, hipStream_t stream);
template <> hipError_t launch_tile<1>(const Args &, int, hipStream_t);
template <> hipError_t launch_tile<3>(const Args &, int, hipStream_t);
template <> hipError_t launch_tile<5>(const Args &, int, hipStream_t);
template <> hipError_t launch_tile<8>(const Args &, int, hipStream_t);
}  // namespace prefill

namespace {

struct TileShape {
    int bm, bn, bk;
    double stage_us;  // one 64-k stage of a workgroup that has a compute unit to itself, measured
                      // (0 = tile is never auto-selected)
    bool may_split;   // K slices pay only where a thread holds few accumulators (the combine moves them all)
    double pair_us;   // big tiles, if > 0: exactly two workgroups fit a compute unit and a stage takes this long
                      // when two are resident (they share the matrix pipe); the estimate counts waves of 512
    // small tiles (resident > 0): up to `resident` workgroups share a compute unit and a stage of each takes
    // pace[r-1] with r of them resident; fixed_us covers launch, pipeline fill and the store; a split moves
    // every slice's partial tile through scratch once each way at scratch_tbps
    int resident;
    double pace[3];
    double fixed_us;
    double scratch_tbps;
};
// by tile id (1, 3, 5, 8: see the plan documentation in the public header; the other ids up to 10 belonged to
// layouts that measurement retired - 2x2 wavefront grids, 32-k stages, a 32-row tile - and are refused)
constexpr TileShape kTiles[11] = {
    {0, 0, 64, 0.0, false, 0.0, 0, {0, 0, 0}, 0, 0},
    {256, 256, 64, 1.25, false, 0.0, 0, {0, 0, 0}, 0, 0},
    {0, 0, 64, 0.0, false, 0.0, 0, {0, 0, 0}, 0, 0},
    {128, 128, 64, 0.75, true, 0.0, 2, {0.75, 1.4, 0}, 7.0, 6.0},
    {0, 0, 64, 0.0, false, 0.0, 0, {0, 0, 0}, 0, 0},
    {64, 128, 64, 0.46, true, 0.0, 3, {0.46, 0.72, 1.0}, 6.0, 6.0},
    {0, 0, 64, 0.0, false, 0.0, 0, {0, 0, 0}, 0, 0},
    {0, 0, 64, 0.0, false, 0.0, 0, {0, 0, 0}, 0, 0},
    {128, 256, 64, 0.99, true, 1.31, 0, {0, 0, 0}, 0, 0},
    {0, 0, 64, 0.0, false, 0.0, 0, {0, 0, 0}, 0, 0},
    {0, 0, 64, 0.0, false, 0.0, 0, {0, 0, 0}, 0, 0}};
constexpr int kNumTiles = 10;
constexpr int kComputeUnits = 256;
constexpr size_t kCounterBytes = 256 * 1024;  // same fixed counter area as the other kernels
constexpr int kMaxSplit = 32;

int ceil_div_i(int a, int b)
{
    return (a + b - 1) / b;
}

// Estimated duration (microseconds) of the pipelined kernel with tile `t` and `split` K slices.  A workgroup
// walks its stages at a pace set by instruction issue and latency, not by the matrix pipe or by HBM: alone on
// a compute unit it leaves most of it idle, and co-resident workgroups slow each other down by less than their
// number.  Big tiles: whole rounds (or waves of pairs) of workgroups.  Small tiles: workgroups per compute unit
// -> pace, from sweeps of 6 Llama shapes x 8 batch sizes (48 ... 512) x 8 slice counts (picks within 1.1 % of
// the best swept plan on average, 7 % at worst).
double estimate_us(const Problem &p, int t, int split)
{
    const TileShape &ts = kTiles[t];
    const int tiles = ceil_div_i(p.M, ts.bm) * ceil_div_i(p.N, ts.bn);
    const int stages = ceil_div_i(p.K, 64);
    const int sps = ceil_div_i(stages, split);
    const int slices = ceil_div_i(stages, sps);
    const double wgs = (double)tiles * slices;
    if (ts.resident > 0) {
        const double n = wgs / kComputeUnits;  // workgroups per compute unit
        // the busiest compute units set the time: ceil(n) resident there; past `resident` the rest queue up
        double pace;
        if (n >= ts.resident) {
            pace = ts.pace[ts.resident - 1] * n / ts.resident;
        } else {
            const int r = (int)std::ceil(n - 1e-9);
            pace = ts.pace[(r < 1 ? 1 : r) - 1];
        }
        double us = ts.fixed_us + sps * pace;
        if (slices > 1)
            us += 2.0 * wgs * ts.bm * ts.bn * sizeof(float) / (ts.scratch_tbps * 1e6);
        return us;
    }
    if (ts.pair_us > 0.0 && slices > 1) {
        // K slices of the 128x256 tile, for few tiles under a deep K (M = 512 ... 1024 on the narrow layers): only
        // with one workgroup per compute unit at most.  A stage takes 0.8 of its usual time while a quarter of
        // the chip idles (clock), the slices' fp32 tiles go through scratch once each way - written by all
        // workgroups at about 4 TB/s, read back by the last arriver of each tile alone at about 60 GB/s.
        // (up to 128 rows the 64x128 tile's slices measured 10 % faster: 4096x22016 at M = 128, 42 against 46 us)
        if (wgs > kComputeUnits || p.M <= 128)
            return 1e30;
        const double stage = ts.stage_us * (wgs <= 192.0 ? 0.8 : 1.0);
        const double tile_bytes = (double)ts.bm * ts.bn * sizeof(float);
        return 3.5 + sps * stage + 1.5 + 4.0 + wgs * tile_bytes / 4e6 + slices * tile_bytes / 6e4;
    }
    if (ts.pair_us > 0.0) {
        // whole waves of two workgroups per compute unit, then the rest: alone if it fits one per unit
        const int per_wave = 2 * kComputeUnits;
        const int waves = (int)wgs / per_wave;
        const int rest = (int)wgs - waves * per_wave;
        double us = 3.5 + waves * (sps * ts.pair_us + 1.5);
        if (rest > 0)
            us += sps * (rest > kComputeUnits ? ts.pair_us : ts.stage_us) + 1.5;
        return us;
    }
    // one workgroup per compute unit: whole rounds, 1.5 us each to fill and drain the pipeline
    return 3.5 + std::ceil(wgs / kComputeUnits) * (sps * ts.stage_us + 1.5) + (slices > 1 ? 5.0 : 0.0);
}

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

bool prefill_tile_exists(int tile)
{
    return tile >= 1 && tile <= kNumTiles && kTiles[tile].bm > 0;
}

void prefill_make_plan(const Problem &p, PrefillPlan &plan)
{
    const int mode = mode_of(p);
    if (mode != prefill::kGroupPerStage) {
        plan.tile = 3;  // the general modes exist for one tile shape only, without a K split
        plan.split_k = 1;
        return;
    }
    const bool tile_given = prefill_tile_exists(plan.tile);
    const bool split_given = plan.split_k >= 1;
    // Few output tiles and a deep K leave most of the chip idle and every workgroup walking all of K: K slices
    // (combined through scratch in slice order) shorten the walk.  Cheapest (tile, split) by the estimate.
    double best = 0.0;
    int best_tile = 3, best_split = 1;
    const int stages = ceil_div_i(p.K, 64);
    for (int t = 1; t <= kNumTiles; ++t) {
        if (kTiles[t].stage_us <= 0.0 || (tile_given && t != plan.tile))
            continue;
        int last_slices = 0;
        for (int split = 1; split <= kMaxSplit && split <= stages / 2 + (stages < 2); ++split) {
            if (split_given && split != (plan.split_k < stages ? plan.split_k : stages))
                continue;
            if (!split_given && split > 1 && !kTiles[t].may_split)
                break;
            const int slices = ceil_div_i(stages, ceil_div_i(stages, split));
            if (slices == last_slices)
                continue;
            last_slices = slices;
            const double us = estimate_us(p, t, split);
            if (best == 0.0 || us < best - 1e-9) {
                best = us;
                best_tile = t;
                best_split = slices;
            }
        }
    }
    if (best == 0.0) {  // a requested split beyond what the loop offers
        best_tile = tile_given ? plan.tile : 3;
        best_split = split_given ? plan.split_k : 1;
    }
    plan.tile = best_tile;
    plan.split_k = best_split;
}

size_t prefill_workspace_bytes(const Problem &p, const PrefillPlan &plan)
{
    if (plan.split_k <= 1 || !prefill_tile_exists(plan.tile))
        return 0;
    const TileShape &ts = kTiles[plan.tile];
    const size_t tiles = (size_t)ceil_div_i(p.M, ts.bm) * ceil_div_i(p.N, ts.bn);
    return kCounterBytes + (size_t)plan.split_k * tiles * ts.bm * ts.bn * sizeof(float);
}

hipError_t launch_prefill(const Problem &p, const PrefillPlan &plan, void *workspace, hipStream_t stream)
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
    a.split_k = (workspace && plan.split_k > 1) ? plan.split_k : 1;
    a.stages_per_slice = 0;
    a.counters = reinterpret_cast<unsigned *>(workspace);
    a.partial = workspace ? reinterpret_cast<float *>(static_cast<unsigned char *>(workspace) + kCounterBytes) : nullptr;
    if (a.split_k > 1 && (size_t)ceil_div_i(p.M, kTiles[plan.tile].bm) * ceil_div_i(p.N, kTiles[plan.tile].bn) >
                             kCounterBytes / sizeof(unsigned))
        a.split_k = 1;  // more tiles than arrival counters: such a problem needs no split anyway
    const int mode = mode_of(p);
    switch (plan.tile) {
    case 1: return prefill::launch_tile<1>(a, mode, stream);
    case 3: return prefill::launch_tile<3>(a, mode, stream);
    case 5: return prefill::launch_tile<5>(a, mode, stream);
    case 8: return prefill::launch_tile<8>(a, mode, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace gptq

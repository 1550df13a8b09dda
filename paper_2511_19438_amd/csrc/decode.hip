// Host side of the split-K vector kernel: launch plan, scratch sizing, dispatch on batch size.
#include "decode_kernel.h"

#include <cmath>

namespace gptq {

namespace {

constexpr int kMaxSliceLdsBytes = 32 * 1024;  // activations of one slice, all batch rows
// The arrival counters occupy a fixed area at the front of the scratch, whatever the problem: partial sums of
// one call must never land where another call keeps counters (they are only ever reset by the kernels).
constexpr size_t kCounterBytes = 256 * 1024;
constexpr int kMaxColumnTiles = (int)(kCounterBytes / sizeof(unsigned));
constexpr size_t kMaxLdsBytes = 160 * 1024;

int batch_template(int M)
{
    return M <= 1 ? 1 : M <= 2 ? 2 : M <= 4 ? 4 : M <= 8 ? 8 : 16;
}

int ceil_div(int a, int b)
{
    return (a + b - 1) / b;
}

struct Derived {
    int lpr, rw, rows, total_chunks, tiles_n, max_chunks_per_slice;
};

// Wavefronts per workgroup: eight for the single-row kernel of the plain format (chunks of four packed rows)
// when every workgroup has a compute unit to itself, else four (see decode::kEightWaves).
int decode_waves(int mb, bool act, int chunk_rows, long long workgroups)
{
    return (mb == 1 && !act && chunk_rows == 4 && workgroups <= 256) ? 8 : 4;
}

Derived derive(const Problem &p, int cols_per_wg, int chunk_rows)
{
    Derived d;
    const int mb = batch_template(p.M < 16 ? p.M : 16);
    d.lpr = cols_per_wg / 4;
    d.rw = 4 * (64 / d.lpr);  // with four wavefronts; eight where decode_waves() says so
    d.rows = p.K / 8;
    d.total_chunks = ceil_div(d.rows, chunk_rows);
    d.tiles_n = ceil_div(p.N, cols_per_wg);
    int ls_max = kMaxSliceLdsBytes / (2 * mb);  // activations per batch row per slice
    if (ls_max > 16384)
        ls_max = 16384;
    d.max_chunks_per_slice = ls_max / (chunk_rows * 8);
    if (d.max_chunks_per_slice < 1)
        d.max_chunks_per_slice = 1;
    return d;
}

// Estimated duration (microseconds) of one launch with the given column tile and chunks per slice.
//
// The kernel is bound by whichever is slower: the HBM stream of the packed weights, or the most loaded
// compute unit (workgroups are dealt out evenly, so that is ceil(workgroups / 256) workgroups' worth of
// dequantisation arithmetic); narrow tiles read short row segments and stream below the full rate, a
// K split adds the scratch round trip of the combine step, and more workgroups than compute units
// cost a little extra.  The constants were fitted to measurements of the Llama-7B/70B projection
// shapes at M = 1 on MI355X; the arithmetic rate is scaled by the instruction count per packed word.
double estimate_us(const Problem &p, const Derived &d, int cols_per_wg, int chunk_rows, int cps, bool act)
{
    const int m = p.M < 16 ? p.M : 16;
    const double weight_bytes = 0.5 * (double)p.K * (double)p.N;
    const int slices = ceil_div(d.total_chunks, cps);
    const double wgs = (double)d.tiles_n * slices;
    const double tb_per_s = cols_per_wg <= 16 ? 2.6 : cols_per_wg <= 32 ? 5.0 : cols_per_wg <= 64 ? 5.8 : 6.2;
    const double hbm = weight_bytes / (tb_per_s * 1e6);
    double ops = m < 8 ? 11.0 + 8.0 * (m - 1) : 30.0 + 8.0 * m;  // vector instructions per packed word
    if (act)
        ops += 24.0;
    const double cu_gb_per_s = 44.0 * 11.0 / ops;
    const double wg_bytes = 0.5 * (double)cps * chunk_rows * 8 * cols_per_wg;
    const double rounds = (double)ceil_div((int)wgs, 256);
    const double cu = rounds * (wg_bytes / (cu_gb_per_s * 1e3) + 0.3);  // 0.3 us of staging and reduction each
    double t = 4.2 + std::cbrt(hbm * hbm * hbm + cu * cu * cu);
    if (slices > 1)
        t += 0.8;
    // Unsplit single-row plans that qualify for the group-level correction (see launch_decode) and keep more than
    // half of the compute units busy measured about a microsecond under this estimate (8192x10240: 64-column
    // tiles unsplit 11.0 us against 12.1 for the 128-column tiles in three slices the estimate used to prefer).
    const int waves = decode_waves(batch_template(m), act, chunk_rows, (long long)wgs);
    if (m == 1 && !act && chunk_rows == 4 && slices == 1 && p.group_size % 128 == 0 && wgs > 128.0 &&
        cols_per_wg >= 64 &&
        cps % (4 * d.rw * waves / 4) == 0)
        t -= 1.0;
    if (wgs > 256.0)
        t += 0.03 * hbm;
    return t;
}

// LDS of one workgroup (must mirror the kernel's carve-up): the slice's activations, the per-chunk activation
// sums of the factored arithmetic, the cross-wavefront reduction buffer and, with g_idx, the slice's group
// numbers plus a (scale, zero) table of ALL groups for the tile's columns.
size_t lds_bytes(const Problem &p, const DecodePlan &plan, int mb, int waves)
{
    const bool act = p.g_idx != nullptr;
    const int mc = mb < 4 ? mb : 4;
    const int ls = plan.chunks_per_slice * plan.chunk_rows * 8;
    size_t lds = ((size_t)mb * ls * sizeof(half_t) + 15) & ~(size_t)15;
    if (!act && mb < 8)
        lds += ((size_t)mb * plan.chunks_per_slice * 2 * sizeof(float) + 15) & ~(size_t)15;
    lds += (size_t)waves * mc * plan.cols_per_wg * sizeof(float);
    if (act)
        lds += (size_t)ls * sizeof(int) + (size_t)(p.K / p.group_size) * plan.cols_per_wg * sizeof(uint32_t);
    return lds;
}

}  // namespace

bool decode_plan_fits(const Problem &p, const DecodePlan &plan)
{
    const int mb = batch_template(p.M < 16 ? p.M : 16);
    const Derived d = derive(p, plan.cols_per_wg, plan.chunk_rows);
    const int waves = decode_waves(mb, p.g_idx != nullptr, plan.chunk_rows, (long long)d.tiles_n * plan.split_k);
    return lds_bytes(p, plan, mb, waves) <= kMaxLdsBytes;
}

void decode_make_plan(const Problem &p, DecodePlan &plan)
{
    const bool act = p.g_idx != nullptr;
    const int gr = p.group_size / 8;
    plan.chunk_rows = act ? 4 : (gr % 4 == 0 ? 4 : (gr % 2 == 0 ? 2 : 1));
    // these variants (and the ablation ones) exist for 64-column tiles only
    const bool fixed_shape = act || plan.chunk_rows != 4 || (plan.flags & 7) != 0;
    const int c = plan.cols_per_wg;
    const bool tile_given = (c == 16 || c == 32 || c == 64 || c == 128 || c == 256) && !fixed_shape;

    // candidates: every allowed tile width (one arrival counter per column tile must fit the fixed
    // counter area) and, per width, every slice length of whole pipeline steps (no lane idles or re-reads
    // a clamped chunk); the cheapest by the estimate wins
    int best_tile = 0, best_cps = 0;
    double best_t = 0.0;
    for (int tile = 32; tile <= 256; tile *= 2) {
        if (tile_given && tile != c)
            continue;
        if (fixed_shape && tile != 64)
            continue;
        if (ceil_div(p.N, tile) > kMaxColumnTiles && tile < 256)
            continue;
        const Derived d = derive(p, tile, plan.chunk_rows);
        const int step_chunks = d.rw * (act ? 1 : 2);  // chunks one workgroup consumes per pipeline step
        if (plan.split_k > 0) {
            const int split = plan.split_k < d.total_chunks ? plan.split_k : d.total_chunks;
            int cps = ceil_div(d.total_chunks, split);
            if (cps > d.max_chunks_per_slice)
                cps = d.max_chunks_per_slice;
            const double t = estimate_us(p, d, tile, plan.chunk_rows, cps, act);
            if (!best_tile || t < best_t) {
                best_tile = tile, best_cps = cps, best_t = t;
            }
            continue;
        }
        // slice lengths of whole steps, for the step of either wavefront count; a candidate stands if its
        // workgroup count calls for the wavefront count it was made for
        const int mb = batch_template(p.M < 16 ? p.M : 16);
        for (int waves = 8; waves >= 4; waves -= 4) {
            if (waves == 8 && decode_waves(mb, act, plan.chunk_rows, 1) != 8)
                continue;
            const int step = step_chunks * waves / 4;
            int last_slices = 0;
            for (int steps = 1; steps <= ceil_div(d.total_chunks, step); ++steps) {
                int cps = steps * step;
                if (cps > d.max_chunks_per_slice) {
                    if (steps > 1)
                        break;
                    cps = d.max_chunks_per_slice;
                }
                const int slices = ceil_div(d.total_chunks, cps);
                if (slices == last_slices)
                    continue;  // same slice count as with the shorter slices before: only less balanced
                last_slices = slices;
                if (decode_waves(mb, act, plan.chunk_rows, (long long)d.tiles_n * slices) != waves)
                    continue;
                const double t = estimate_us(p, d, tile, plan.chunk_rows, cps, act);
                if (!best_tile || t < best_t - 1e-9) {
                    best_tile = tile, best_cps = cps, best_t = t;
                }
            }
        }
    }
    if (tile_given && c == 16) {  // the narrowest tile is never chosen, only honoured
        const Derived d = derive(p, 16, plan.chunk_rows);
        const int split = plan.split_k > 0 ? (plan.split_k < d.total_chunks ? plan.split_k : d.total_chunks) : 1;
        best_tile = 16;
        best_cps = ceil_div(d.total_chunks, split);
        if (best_cps > d.max_chunks_per_slice)
            best_cps = d.max_chunks_per_slice;
    }
    if (best_cps < 1)
        best_cps = 1;
    plan.cols_per_wg = best_tile;
    const Derived d = derive(p, plan.cols_per_wg, plan.chunk_rows);
    plan.chunks_per_slice = best_cps;
    plan.split_k = ceil_div(d.total_chunks, best_cps);
}

size_t decode_counter_bytes(int)
{
    return kCounterBytes;
}

size_t decode_workspace_bytes(const Problem &p, const DecodePlan &plan)
{
    const int m = p.M < 16 ? p.M : 16;
    size_t bytes = decode_counter_bytes(p.N);
    if (plan.split_k > 1)
        bytes += (size_t)plan.split_k * m * p.N * sizeof(float);
    else if (plan.flags & decode::kNoSmb)
        bytes += (size_t)m * p.N * sizeof(float);  // the fp32 sums the lanes add into
    return bytes;
}

namespace {

__global__ void zero_floats_kernel(float *p, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n)
        p[i] = 0.f;
}

}  // namespace

bool decode_ablation_supported(const Problem &p)
{
    return p.g_idx == nullptr && p.M <= 4 && p.group_size % 32 == 0;
}

hipError_t launch_decode(const Problem &p, const DecodePlan &plan, void *workspace, hipStream_t stream)
{
    const bool act = p.g_idx != nullptr;
    const Derived d = derive(p, plan.cols_per_wg, plan.chunk_rows);
    if (d.tiles_n > kMaxColumnTiles)
        return hipErrorInvalidValue;  // more column tiles than arrival counters (N beyond ~16M columns)
    unsigned char *ws = static_cast<unsigned char *>(workspace);

    // batches larger than 16 rows are processed 16 rows at a time on the same stream
    for (int m0 = 0; m0 < p.M; m0 += 16) {
        const int m = (p.M - m0) < 16 ? (p.M - m0) : 16;
        const int mb = batch_template(m);
        decode::Args a;
        a.x = p.x + (size_t)m0 * p.K;
        a.qweight = p.qweight;
        a.qzeros = p.qzeros;
        a.scales = p.scales;
        a.g_idx = p.g_idx;
        a.x_perm = p.x_perm;
        a.out = p.out + (size_t)m0 * p.N;
        a.counters = reinterpret_cast<unsigned *>(ws);
        a.partial = reinterpret_cast<float *>(ws + decode_counter_bytes(p.N));
        a.M = m;
        a.K = p.K;
        a.N = p.N;
        a.rows = d.rows;
        a.rows_per_group = p.group_size / 8;
        a.chunk_group_shift = -1;
        if (a.rows_per_group % plan.chunk_rows == 0) {
            const int cpg = a.rows_per_group / plan.chunk_rows;
            if ((cpg & (cpg - 1)) == 0) {
                a.chunk_group_shift = 0;
                while ((1 << a.chunk_group_shift) < cpg)
                    ++a.chunk_group_shift;
            }
        }
        a.groups = p.K / p.group_size;
        a.tiles_n = d.tiles_n;
        a.split_k = plan.split_k;
        a.chunks_per_slice = plan.chunks_per_slice;
        a.total_chunks = d.total_chunks;

        const int waves = decode_waves(mb, act, plan.chunk_rows, (long long)d.tiles_n * plan.split_k);
        const size_t lds = lds_bytes(p, plan, mb, waves);
        if (lds > kMaxLdsBytes)
            return hipErrorInvalidValue;

        if (plan.flags & decode::kNoSmb) {  // the baseline accumulates into memory: it needs zeros first
            const size_t n = (size_t)m * p.N;
            hipLaunchKernelGGL(zero_floats_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, a.partial,
                               n);
            if (hipGetLastError() != hipSuccess)
                return hipErrorLaunchFailure;
        }
        // Group-level correction (decode::kGroupCorr): single row, groups of whole 128-k units, and a plan whose
        // one slice gives every row lane whole groups (four chunks each per pair of steps) - otherwise lanes
        // idle where the per-chunk kernel keeps them busy.  Measured: 4096x12288 7.6 -> 7.3 us, 4096x22016
        // 12.0 -> 10.8; with K slices it was level or slower (8192x8192 9.9 -> 10.3), so those keep the
        // per-chunk correction.
        const int row_lanes = d.rw * waves / 4;
        const bool group_corr = mb == 1 && !act && plan.flags == 0 && !p.x_perm && plan.chunk_rows == 4 &&
                                p.group_size % 128 == 0 && plan.split_k == 1 &&
                                plan.chunks_per_slice % (4 * row_lanes) == 0;
        const int flags = plan.flags | (p.x_perm ? decode::kGatherX : 0) | (waves == 8 ? decode::kEightWaves : 0) |
                          (group_corr ? decode::kGroupCorr : 0);
        hipError_t err;
        switch (mb) {
        case 1: err = decode::launch_mb<1>(a, d.lpr, plan.chunk_rows, act, flags, lds, stream); break;
        case 2: err = decode::launch_mb<2>(a, d.lpr, plan.chunk_rows, act, flags, lds, stream); break;
        case 4: err = decode::launch_mb<4>(a, d.lpr, plan.chunk_rows, act, flags, lds, stream); break;
        case 8: err = decode::launch_mb<8>(a, d.lpr, plan.chunk_rows, act, flags, lds, stream); break;
        default: err = decode::launch_mb<16>(a, d.lpr, plan.chunk_rows, act, flags, lds, stream); break;
        }
        if (err != hipSuccess)
            return err;
    }
    return hipSuccess;
}

}  // namespace gptq

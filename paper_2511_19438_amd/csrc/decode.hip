// Host side of the split-K vector kernel: launch plan, scratch sizing, dispatch on batch size.
#include "decode_kernel.h"

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

Derived derive(const Problem &p, int cols_per_wg, int chunk_rows)
{
    Derived d;
    d.lpr = cols_per_wg / 4;
    d.rw = decode::kWaves * (64 / d.lpr);
    d.rows = p.K / 8;
    d.total_chunks = ceil_div(d.rows, chunk_rows);
    d.tiles_n = ceil_div(p.N, cols_per_wg);
    const int mb = batch_template(p.M < 16 ? p.M : 16);
    int ls_max = kMaxSliceLdsBytes / (2 * mb);  // activations per batch row per slice
    if (ls_max > 8192)
        ls_max = 8192;
    d.max_chunks_per_slice = ls_max / (chunk_rows * 8);
    if (d.max_chunks_per_slice < 1)
        d.max_chunks_per_slice = 1;
    return d;
}

}  // namespace

void decode_make_plan(const Problem &p, DecodePlan &plan)
{
    const bool act = p.g_idx != nullptr;
    const int gr = p.group_size / 8;
    plan.chunk_rows = act ? 4 : (gr % 4 == 0 ? 4 : (gr % 2 == 0 ? 2 : 1));
    const bool fixed_shape = act || plan.chunk_rows != 4;  // these variants exist for 64-column tiles only
    const int c = plan.cols_per_wg;
    const bool tile_given = (c == 16 || c == 32 || c == 64 || c == 128 || c == 256) && !fixed_shape;
    if (!tile_given) {
        // widest tile that still leaves at least ~512 column tiles' worth of workgroups to spread
        plan.cols_per_wg = 64;
        if (!fixed_shape) {
            if (ceil_div(p.N, 64) > 768)
                plan.cols_per_wg = 128;
            if (ceil_div(p.N, 128) > 768)
                plan.cols_per_wg = 256;
        }
    }
    while (!fixed_shape && plan.cols_per_wg < 256 && ceil_div(p.N, plan.cols_per_wg) > kMaxColumnTiles)
        plan.cols_per_wg *= 2;  // keep one arrival counter per column tile inside the fixed counter area
    const Derived d = derive(p, plan.cols_per_wg, plan.chunk_rows);

    const int step_chunks = d.rw * (act ? 1 : 2);  // chunks one workgroup consumes per pipeline step
    int cps;
    if (plan.split_k > 0) {
        int split = plan.split_k < d.total_chunks ? plan.split_k : d.total_chunks;
        cps = ceil_div(d.total_chunks, split);
    } else {
        // Slices are whole pipeline steps (no lane idles or re-reads a clamped chunk) and their number puts
        // the workgroup count as close as possible (in ratio) to two per compute unit.
        const double target_wgs = 512.0;
        int best_cps = 0;
        double best_cost = 0.0;
        const int max_steps = ceil_div(d.total_chunks, step_chunks);
        for (int steps = 1; steps <= max_steps; ++steps) {
            const int c = steps * step_chunks;
            if (c > d.max_chunks_per_slice && best_cps)
                break;
            const double wgs = (double)d.tiles_n * ceil_div(d.total_chunks, c);
            const double ratio = wgs > target_wgs ? wgs / target_wgs : target_wgs / wgs;
            if (!best_cps || ratio < best_cost - 1e-9) {
                best_cps = c;
                best_cost = ratio;
            }
        }
        cps = best_cps;
    }
    if (cps > d.max_chunks_per_slice)
        cps = d.max_chunks_per_slice;
    if (cps < 1)
        cps = 1;
    plan.chunks_per_slice = cps;
    plan.split_k = ceil_div(d.total_chunks, cps);
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
    return bytes;
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

        const int mc = mb < 4 ? mb : 4;
        const int ls = plan.chunks_per_slice * plan.chunk_rows * 8;
        size_t lds = ((size_t)mb * ls * sizeof(half_t) + 15) & ~(size_t)15;
        if (!act && mb < 8)  // per-chunk sums of the activations (must mirror the kernel's carve-up)
            lds += ((size_t)mb * plan.chunks_per_slice * 2 * sizeof(float) + 15) & ~(size_t)15;
        lds += (size_t)decode::kWaves * mc * plan.cols_per_wg * sizeof(float);
        if (act)
            lds += (size_t)ls * sizeof(int) + (size_t)a.groups * plan.cols_per_wg * sizeof(uint32_t);
        if (lds > kMaxLdsBytes)
            return hipErrorInvalidValue;

        hipError_t err;
        switch (mb) {
        case 1: err = decode::launch_mb<1>(a, d.lpr, plan.chunk_rows, act, lds, stream); break;
        case 2: err = decode::launch_mb<2>(a, d.lpr, plan.chunk_rows, act, lds, stream); break;
        case 4: err = decode::launch_mb<4>(a, d.lpr, plan.chunk_rows, act, lds, stream); break;
        case 8: err = decode::launch_mb<8>(a, d.lpr, plan.chunk_rows, act, lds, stream); break;
        default: err = decode::launch_mb<16>(a, d.lpr, plan.chunk_rows, act, lds, stream); break;
        }
        if (err != hipSuccess)
            return err;
    }
    return hipSuccess;
}

}  // namespace gptq

// Host side of the split-K vector kernel: launch plan, scratch sizing, dispatch on batch size.
#include "decode_kernel.h"

namespace gptq {

namespace {

constexpr int kMaxSliceLdsBytes = 32 * 1024;  // activations of one slice, all batch rows
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
    if (plan.cols_per_wg != 64 && plan.cols_per_wg != 128 && plan.cols_per_wg != 256)
        plan.cols_per_wg = 64;
    if (act || plan.chunk_rows != 4)
        plan.cols_per_wg = 64;
    const Derived d = derive(p, plan.cols_per_wg, plan.chunk_rows);

    int split = plan.split_k;
    if (split <= 0) {
        // Enough workgroups to cover 256 compute units several times, but at least one chunk per row lane.
        const int target_wgs = act ? 768 : 1024;
        split = ceil_div(target_wgs, d.tiles_n);
        const int max_split = ceil_div(d.total_chunks, d.rw);
        if (split > max_split)
            split = max_split;
        if (split < 1)
            split = 1;
    }
    if (split > d.total_chunks)
        split = d.total_chunks;
    int cps = ceil_div(d.total_chunks, split);
    if (cps > d.max_chunks_per_slice)
        cps = d.max_chunks_per_slice;
    plan.chunks_per_slice = cps;
    plan.split_k = ceil_div(d.total_chunks, cps);
}

size_t decode_counter_bytes(int N)
{
    const size_t tiles = (size_t)(N + 63) / 64;  // the narrowest tile gives the most counters
    return (tiles * sizeof(unsigned) + 255) & ~(size_t)255;
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
        a.groups = p.K / p.group_size;
        a.tiles_n = d.tiles_n;
        a.split_k = plan.split_k;
        a.chunks_per_slice = plan.chunks_per_slice;
        a.total_chunks = d.total_chunks;

        const int mc = mb < 4 ? mb : 4;
        const int ls = plan.chunks_per_slice * plan.chunk_rows * 8;
        size_t lds = ((size_t)mb * ls * sizeof(half_t) + 15) & ~(size_t)15;
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

// fp16 MFMA kernels for the W4A16 GPTQ matrix multiply at large batch (prefill), gfx950.
//
// This is the one place where the path is a real dense contraction, so it runs on the matrix
// cores (v_mfma_f32_32x32x16_f16, fp32 accumulation).  The paper's kernel (Opt4GPTQ, Section 3)
// uses one vector kernel for every batch size; what carries over is its pipeline order: stage the
// operands on chip with wide loads (Section 3.2), dequantise with packed half arithmetic
// (Section 3.3), accumulate on chip and commit each output once (Section 3.1).
//
// Design for CDNA4 (prefill_pipelined_kernel, the tuned path: no g_idx, group size a multiple of 64):
//   * Everything that comes from global memory - the activation tile, the packed weight words, the
//     scales and the packed zero points of a k stage - is copied global -> LDS by the DMA path
//     (global_load_lds_dwordx4), never through registers, into a ring of NBUF stage buffers that runs
//     NBUF-2 stages ahead of the MFMAs.  One s_waitcnt vmcnt(n) + s_barrier per stage publishes the
//     oldest batch in flight; loads complete in order, so "at most n outstanding" means "the batch
//     issued NBUF-2 stages ago has landed".
//   * A operand (activations): 16-byte chunks are XOR-swizzled by row so that the 32-row operand
//     reads (ds_read_b128) are bank-conflict free on the 64-bank LDS.
//   * B operand (weights): a packed qweight word holds eight consecutive k of ONE column, which is
//     exactly what one lane of the 32x32x16 MFMA B operand holds.  Each lane reads its word(s) from
//     the LDS copy and dequantises them in registers into the four VGPRs of the operand:
//     v_perm_b32 + v_and_or_b32 build the pair (1024 + q_even, 64 + q_odd), a packed add of
//     (-(1024 + z), -(64 + z)) gives the exact integer differences and a packed multiply by the scale
//     gives the fp16 weight with one rounding.  The dequantised weights never touch LDS.
//   * Waves of a workgroup split the N extent of the tile where possible, so every weight is
//     dequantised by exactly one wave of the workgroup.
//   * The instruction order of a k step is pinned with scheduling barriers: every MFMA is followed by
//     a few instructions of the NEXT k step's LDS reads and dequantisation, which issue in the shadow
//     of that MFMA (one wave per SIMD: nothing else would hide their latency or keep the pipe fed).
//   * Lane j of an n-block owns TN adjacent columns (n-block t <-> column base + TN*j + t), so the
//     weight reads are TN dwords wide and the output stores are TN halves wide.
//   * Workgroup ids are remapped so that the tiles resident on one XCD (ids congruent mod 8) are
//     neighbours in the (m fastest) tile order and share their weight panel and activations in
//     that XCD's L2.
//
// prefill_general_kernel serves the remaining cases (g_idx, group sizes that are not a multiple of
// 64, a k tail) with the same operand layout but plain register staging; it is about correctness.
#pragma once

#include <type_traits>

#include "exchange.h"
#include "kernels.h"

namespace gptq {
namespace prefill {

constexpr int kThreads = 256;

enum Mode {
    kGroupPerStage = 0,  // group_size % 64 == 0, no g_idx: pipelined kernel
    kGroupPerRow = 1,    // any group_size, no g_idx: looked up per packed row
    kActOrder = 2        // g_idx: looked up per k
};

struct Args {
    const half_t *x;
    const uint32_t *qweight;
    const uint32_t *qzeros;
    const half_t *scales;
    const int32_t *g_idx;
    half_t *out;
    int M, K, N, group_size;
    int tiles_m, tiles_n;
    // K split of the pipelined kernel (few output tiles, deep K): slice s of a tile covers the stages
    // [s * stages_per_slice, ...); the slices meet in scratch, in slice order, as in the other kernels.
    int split_k;            // 1 = no split
    int stages_per_slice;
    float *partial;         // [split_k][tiles][accumulators per thread][256 threads] fp32 (see combine_slices)
    unsigned *counters;     // [tiles], zero between launches
};

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void lds_ptr_t;
typedef __attribute__((address_space(1))) const void global_ptr_t;

__device__ __forceinline__ half2_t as_half2(uint32_t v)
{
    return __builtin_bit_cast(half2_t, v);
}

// (-(1024 + z), -(64 + z)) as packed fp16 bits
__device__ __forceinline__ uint32_t neg_bias(uint32_t z)
{
    return 0xD400E400u | z | (z << 20);
}

// Constants of the nibble -> fp16 conversion, kept in registers so that mask-and-bias is one v_and_or_b32
// (VOP3 on gfx9 takes no literals).  0x6400 = 1024.0 (ulp 1), 0x5400 = 64.0 (ulp 1/16).
struct PairMagic {
    uint32_t mask, bias;
    __device__ __forceinline__ PairMagic()
    {
        mask = 0x00f0000fu;
        bias = 0x54006400u;
        asm volatile("" : "+s"(mask), "+v"(bias));
    }
};

// Pair P (k = 2P, 2P+1) of one packed word -> two fp16 weights, as the bits of a half2.
// Byte P of w = q_{2P} | q_{2P+1} << 4 is spread to both halves, one nibble kept in each:
// low half 1024 + q_{2P}, high half 64 + q_{2P+1}; nz = (-(1024+z), -(64+z)), ss = (s, s).
template <int P>
__device__ __forceinline__ uint32_t dequant_pair(uint32_t w, const PairMagic &k, uint32_t nz, uint32_t ss)
{
    const uint32_t spread = __builtin_amdgcn_perm(0u, w, 0x0c000c00u | P | (P << 16));
    const half2_t v = (as_half2((spread & k.mask) | k.bias) + as_half2(nz)) * as_half2(ss);
    return __builtin_bit_cast(uint32_t, v);
}

// The same in two halves, so that independent work can sit between the add and the multiply (a packed
// multiply that consumes the result of the packed add right before it costs a wait state).
template <int P>
__device__ __forceinline__ uint32_t dequant_pair_begin(uint32_t w, const PairMagic &k, uint32_t nz)
{
    const uint32_t spread = __builtin_amdgcn_perm(0u, w, 0x0c000c00u | P | (P << 16));
    const half2_t v = as_half2((spread & k.mask) | k.bias) + as_half2(nz);
    return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ uint32_t dequant_pair_end(uint32_t diff, uint32_t ss)
{
    const half2_t v = as_half2(diff) * as_half2(ss);
    return __builtin_bit_cast(uint32_t, v);
}

__device__ __forceinline__ u32x4_t dequant_word(uint32_t w, const PairMagic &k, const uint32_t nz[4],
                                                const uint32_t ss[4])
{
    u32x4_t r;
    r[0] = dequant_pair<0>(w, k, nz[0], ss[0]);
    r[1] = dequant_pair<1>(w, k, nz[1], ss[1]);
    r[2] = dequant_pair<2>(w, k, nz[2], ss[2]);
    r[3] = dequant_pair<3>(w, k, nz[3], ss[3]);
    return r;
}

// XCD-aware tile order: workgroup ids congruent mod 8 run on one XCD; give each XCD a contiguous range
// of the (m fastest) tile order.  Returns false for the padding workgroups of the last range.
// With a K split the grid is `split_k` such ranges one after the other (the slices of a tile share an XCD).
__device__ __forceinline__ bool tile_of_workgroup(const Args &a, int &tile_m, int &tile_n, int &logical, int &slice)
{
    const int total = a.tiles_m * a.tiles_n;
    const int per_xcd = (total + 7) / 8;
    const int padded = per_xcd * 8;
    slice = blockIdx.x / padded;
    const int inner = blockIdx.x - slice * padded;
    logical = (inner & 7) * per_xcd + (inner >> 3);
    if (logical >= total)
        return false;
    tile_m = logical % a.tiles_m;
    tile_n = logical / a.tiles_m;
    return true;
}

// One fp16 rounding per output, TN adjacent columns per store.  Lane (lj, kh) holds, for 32-row block i and
// accumulator register r, row 8*(r/4) + 4*kh + r%4 of the block and column lj of n-block t.
template <int TM, int TN>
__device__ __forceinline__ void store_tile(const float16_t (&acc)[TM][TN], half_t *out, int row0, int col0,
                                           bool col_ok, int kh, int M, int N)
{
    if (!col_ok)
        return;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = row0 + i * 32 + 8 * (r >> 2) + 4 * kh + (r & 3);
            if (m < M) {
                half_t *dst = out + (size_t)m * N + col0;
                if (TN == 4) {
                    half4_t v = {(half_t)acc[i][0][r], (half_t)acc[i][1 % TN][r], (half_t)acc[i][2 % TN][r],
                                 (half_t)acc[i][3 % TN][r]};
                    *reinterpret_cast<half4_t *>(dst) = v;
                } else if (TN == 2) {
                    half2_t v = {(half_t)acc[i][0][r], (half_t)acc[i][1 % TN][r]};
                    *reinterpret_cast<half2_t *>(dst) = v;
                } else {
                    *dst = (half_t)acc[i][0][r];
                }
            }
        }
    }
}

// K slices across workgroups (few output tiles, deep K).  Every slice leaves its results in scratch and the
// last workgroup of the tile to arrive adds them in slice order (deterministic), then goes on to store the
// tile.  The values travel in pairs - 64-bit accesses, pair p of thread t at [p][t]: coalesced - and the last
// arriver loads several slices before it uses any, so the combine costs a few scratch round trips instead of
// one per slice.  Device-scope accesses and an arrival counter with release / acquire at agent scope (exchange.h).
// Returns false in the workgroups that are not the last of their tile.  Partial layout:
// [split_k][tiles][ACC / 2 pairs][256 threads] x 8 bytes.
template <int ACC>
__device__ __forceinline__ bool combine_slices(float (&v)[ACC], const Args &a, int slice, int tile_id, int tid)
{
    static_assert(ACC % 2 == 0, "values travel in pairs");
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    constexpr int PAIRS = ACC / 2;
    constexpr int CH = PAIRS < 64 ? PAIRS : 64;  // pairs of one slice loaded together
    constexpr int G = 64 / CH;                   // slices loaded together: up to 128 values in flight
    static_assert(PAIRS % CH == 0, "whole batches");
    __shared__ int s_last;
    const size_t tiles = (size_t)a.tiles_m * a.tiles_n;
    unsigned long long *scratch = reinterpret_cast<unsigned long long *>(a.partial);
    unsigned long long *mine = scratch + ((size_t)slice * tiles + tile_id) * PAIRS * kThreads + tid;
#pragma unroll
    for (int p = 0; p < PAIRS; ++p) {
        const f32x2_t pair = {v[2 * p], v[2 * p + 1]};
        __hip_atomic_store(mine + (size_t)p * kThreads, __builtin_bit_cast(unsigned long long, pair), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    }
    __builtin_amdgcn_s_waitcnt(0);  // every partial store of this workgroup has been acknowledged (exchange.h)
    __syncthreads();
    if (tid == 0)
        s_last = (slice_arrive(a.counters + tile_id) == (unsigned)(a.split_k - 1));
    __syncthreads();
    if (!s_last)
        return false;
    slice_acquire();
#pragma unroll
    for (int e = 0; e < ACC; ++e)
        v[e] = 0.f;
#pragma unroll
    for (int c0 = 0; c0 < PAIRS; c0 += CH) {
        for (int sl0 = 0; sl0 < a.split_k; sl0 += G) {
            unsigned long long part[G][CH];
#pragma unroll
            for (int u = 0; u < G; ++u) {
                const int sl = min(sl0 + u, a.split_k - 1);  // unconditional loads; a repeated slice is not added
                const unsigned long long *theirs =
                    scratch + ((size_t)sl * tiles + tile_id) * PAIRS * kThreads + (size_t)c0 * kThreads + tid;
#pragma unroll
                for (int p = 0; p < CH; ++p)
                    part[u][p] =
                        __hip_atomic_load(theirs + (size_t)p * kThreads, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
#pragma unroll
            for (int u = 0; u < G; ++u) {
                const float keep = sl0 + u < a.split_k ? 1.f : 0.f;
#pragma unroll
                for (int p = 0; p < CH; ++p) {
                    const f32x2_t pair = __builtin_bit_cast(f32x2_t, part[u][p]);
                    v[2 * (c0 + p)] += keep * pair[0];
                    v[2 * (c0 + p) + 1] += keep * pair[1];
                }
            }
        }
    }
    if (tid == 0)
        __hip_atomic_store(a.counters + tile_id, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // next launch
    return true;
}

// =====================================================================================================
// Tuned path
// =====================================================================================================

// LDS layout of one stage buffer of the pipelined kernel.
template <int BM, int BN, int BK>
struct StageLayout {
    static constexpr int A_BYTES = BM * BK * 2;        // [BM][BK] halves, 16-byte chunks swizzled
    static constexpr int B_BYTES = (BK / 8) * BN * 4;  // [BK/8][BN] packed words
    static constexpr int SZ_BYTES = 1024;              // scales [BN] halves, then zero words [BN/8], then padding
    static constexpr int BYTES = A_BYTES + B_BYTES + SZ_BYTES;
};

// Tiles with up to 128 accumulator registers per lane are compiled to fit two workgroups on a compute unit
// (256 registers per lane each): one workgroup's dequantisation then runs under the other's MFMAs.
template <int BM, int BN>
constexpr int kWavesPerSimd = (BM * BN <= 128 * 256) ? 2 : 1;

template <int BM, int BN, int WM, int WN, int BK, int NBUF>
__global__ __launch_bounds__(kThreads, (kWavesPerSimd<BM, BN>)) void prefill_pipelined_kernel(const Args a)
{
    static_assert(WM * WN == 4, "four wavefronts per workgroup");
    static_assert(BK == 32 || BK == 64, "stage of 32 or 64 k");
    static_assert(NBUF >= 3, "ring of at least three stage buffers");
    using L = StageLayout<BM, BN, BK>;
    constexpr int WAVE_M = BM / WM;
    constexpr int WAVE_N = BN / WN;
    constexpr int TM = WAVE_M / 32;
    constexpr int TN = WAVE_N / 32;
    static_assert(TM >= 1 && (TN == 1 || TN == 2 || TN == 4), "wave tile: 32-row blocks by 32/64/128 columns");
    constexpr int KSTEPS = BK / 16;                         // MFMA k steps per stage (2 or 4)
    constexpr int CH = BK / 8;                              // 16-byte chunks per A row
    constexpr int RPB = 16 / CH;                            // A rows per 256-byte bank row
    constexpr int A_CHUNKS = BM * CH / kThreads;            // DMA instructions per thread for the A tile
    constexpr int B_CHUNKS = (BK / 8) * BN / 4 / kThreads;  // ... for the packed weights
    static_assert(A_CHUNKS >= 1 && B_CHUNKS >= 1, "tile too small for 256 threads");
    static_assert(BN / 8 + BN / 32 <= 64, "scales and zero points of a stage must fit one wave-wide DMA");
    constexpr int LOADS_PER_STAGE = A_CHUNKS + B_CHUNKS + 1;
    constexpr int MAX_IN_FLIGHT = (NBUF - 3) * LOADS_PER_STAGE;  // may stay outstanding when a stage is published
    static_assert(MAX_IN_FLIGHT < 64, "vmcnt is a 6-bit counter");

    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keep it in a scalar register
    const int wm = wave / WN;
    const int wn = wave % WN;
    const int lj = lane & 31;
    const int kh = lane >> 5;

    int tile_m, tile_n, tile_id, slice;
    if (!tile_of_workgroup(a, tile_m, tile_n, tile_id, slice))
        return;
    const int m0 = tile_m * BM;
    const int n0 = tile_n * BN;
    const int N = a.N, K = a.K, M = a.M;
    const int all_stages = K / BK;  // K is a multiple of the group size, which is a multiple of 64
    const int first = slice * a.stages_per_slice;  // this workgroup's stages: [first, first + stages)
    const int stages = min(a.stages_per_slice, all_stages - first);
    const int last = first + stages - 1;
    const int col_local = wn * WAVE_N + TN * lj;  // first of this lane's TN columns inside the tile
    const int col_raw = n0 + col_local;
    const bool col_ok = col_raw < N;

    float16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int t = 0; t < TN; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[i][t][r] = 0.f;

    // ---- global sources of this thread's DMA slots, as 32-bit byte offsets from bases that are uniform over
    //      the workgroup (scalar registers).  Loads never branch: rows past M and columns past N are clamped
    //      to the last valid ones; what they produce lands in output rows / columns that are not stored.
    // A: slot p = tid + j*256 holds physical chunk p % CH of row p / CH = logical chunk (p % CH) ^ ((row / RPB) % CH).
    const char *a_base = reinterpret_cast<const char *>(a.x + (size_t)m0 * K);
    uint32_t a_off[A_CHUNKS];
#pragma unroll
    for (int j = 0; j < A_CHUNKS; ++j) {
        const int slot = tid + j * kThreads;
        const int row = slot / CH;
        const int ch = (slot % CH) ^ ((row / RPB) & (CH - 1));
        a_off[j] = (uint32_t)((min(m0 + row, M - 1) - m0) * K + ch * 8) * 2u;
    }
    // B: slot p holds words 4*(p % (BN/4)) .. +3 of packed row p / (BN/4) of the stage.
    const char *b_base = reinterpret_cast<const char *>(a.qweight + n0);
    uint32_t b_off[B_CHUNKS];
#pragma unroll
    for (int j = 0; j < B_CHUNKS; ++j) {
        const int slot = tid + j * kThreads;
        const int row = slot / (BN / 4);
        const int c4 = slot % (BN / 4);
        b_off[j] = (uint32_t)(row * N + min(4 * c4, N - 4 - n0)) * 4u;
    }
    // scales / zero points: lanes 0 .. BN/8-1 fetch 8 scales each, the next BN/32 lanes 4 zero words each, the
    // rest refetch the last zero chunk into padding (every lane takes part: the DMA needs no exec mask).
    // (N is a multiple of 32 here, so a clamped chunk of four zero words still lies inside its row.)
    const int sz_lane = min(lane, BN / 8 + BN / 32 - 1);
    const bool sz_is_scale = sz_lane < BN / 8;
    const int sz_col = sz_is_scale ? min(n0 + 8 * sz_lane, N - 8) : min(n0 + 32 * (sz_lane - BN / 8), N - 32);
    const char *sz_src = sz_is_scale ? reinterpret_cast<const char *>(a.scales + sz_col)
                                     : reinterpret_cast<const char *>(a.qzeros + (sz_col >> 3));
    const uint32_t sz_stride = sz_is_scale ? (uint32_t)N * 2u : (uint32_t)(N >> 3) * 4u;  // bytes per group row
    const int stages_per_group = a.group_size / BK;

    // The stage whose loads are issued next, as running source pointers (uniform for the activations and the
    // packed words, per lane for the scales / zero points) that advance by constants: no multiplication and no
    // division in the loop, and selects instead of branches - a branch would end the basic block, and the
    // dequantisation of a stage's last k step (pure arithmetic, first used in the next stage) would sink
    // across it, out of the MFMAs' shadow.
    int ld_stage = first, ld_in_group = first % stages_per_group;
    const char *a_cur = a_base + (size_t)first * BK * 2;
    const size_t b_step = (size_t)(BK / 8) * N * 4;  // bytes between the packed rows of consecutive stages
    const char *b_cur = b_base + (size_t)first * b_step;
    const char *sz_cur = sz_src + (size_t)(first / stages_per_group) * sz_stride;
    auto stage_base = [&](int ring) { return smem + (size_t)ring * L::BYTES; };
    // piece `p` (0 .. LOADS_PER_STAGE-1) of the loads of stage `ld_stage` into ring slot `ring`
    auto issue_piece = [&](int p, int ring) {
        unsigned char *base = stage_base(ring);
        if (p < A_CHUNKS) {  // the wave's 64 lanes fill 64 consecutive 16-byte slots
            __builtin_amdgcn_global_load_lds((global_ptr_t *)(a_cur + a_off[p]),
                                             (lds_ptr_t *)(base + (size_t)(p * kThreads + wave * 64) * 16), 16, 0, 0);
        } else if (p < A_CHUNKS + B_CHUNKS) {
            const int j = p - A_CHUNKS;
            __builtin_amdgcn_global_load_lds((global_ptr_t *)(b_cur + b_off[j]),
                                             (lds_ptr_t *)(base + L::A_BYTES + (size_t)(j * kThreads + wave * 64) * 16),
                                             16, 0, 0);
        } else {
            // all four waves write the same bytes: keeps the per-wave count of outstanding loads identical
            __builtin_amdgcn_global_load_lds((global_ptr_t *)sz_cur, (lds_ptr_t *)(base + L::A_BYTES + L::B_BYTES),
                                             16, 0, 0);
        }
    };
    auto advance_load_stage = [&]() {
        // past the end the last stage is refetched: uniform counts, no branch in the loads
        const int more = ld_stage < last ? 1 : 0;
        ld_stage += more;
        a_cur += more ? BK * 2 : 0;
        b_cur += more ? b_step : (size_t)0;
        ld_in_group += more;
        const bool wrap = ld_in_group == stages_per_group;
        ld_in_group = wrap ? 0 : ld_in_group;
        sz_cur += wrap ? sz_stride : 0u;
    };
    // Publish the oldest batch in flight: every wave waits for its own part of it, the barrier does the rest.
    auto publish = [&]() {
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(MAX_IN_FLIGHT) : "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };

    // ---- operand registers ----
    half8_t afr[2][TM];  // A operands of two consecutive k steps
    u32x4_t bfr[2][TN];  // B operands (bits of 4 half2 each)
    uint32_t w_cur[KSTEPS][TN], w_nxt[KSTEPS][TN];  // packed words of this lane: stage in use / the next one
    uint32_t nz_cur[TN], ss_cur[TN], nz_nxt[TN], ss_nxt[TN];
    const PairMagic magic;

    // A operand of 32-row block i at k step kk: row wm*WAVE_M + 32 i + lj, chunk (2 kk + kh) ^ swizzle(row).
    // The swizzle does not depend on i (32 rows are a whole number of swizzle periods), so the byte offset is
    // a per-lane value per k step plus i * 32 rows: the reads of one k step share ONE address register (the
    // stage buffer's base added once per k step) and differ in the instruction's immediate offset.
    uint32_t a_lane_off[KSTEPS];
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
        const int row = wm * WAVE_M + lj;
        a_lane_off[kk] = (uint32_t)(row * (BK * 2) + (((2 * kk + kh) ^ ((row / RPB) & (CH - 1))) * 16));
    }
    // The reads are issued as inline asm and waited for by hand (`wait_afrag`): the compiler's own counter
    // bookkeeping loses track of the order of LDS operations across the loop's back edge and falls back to
    // waiting for ALL outstanding LDS reads - including the one issued a few cycles earlier - before the first
    // use of every operand, which stalls the matrix pipe for an LDS round trip several times per k step.
    const uint32_t smem_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    auto read_afrag = [&](int ring, int kk, int i, half8_t &dst) {
        const uint32_t addr = smem_base + a_lane_off[kk] + (uint32_t)ring * (uint32_t)L::BYTES;
#define GPTQ_READ_A(I) \
    case I: asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"((I) * 32 * BK * 2)); break;
        switch (i) {  // (the immediate offset must be a constant expression: one case per 32-row block)
            GPTQ_READ_A(0) GPTQ_READ_A(1) GPTQ_READ_A(2) GPTQ_READ_A(3)
            GPTQ_READ_A(4) GPTQ_READ_A(5) GPTQ_READ_A(6) GPTQ_READ_A(7)
        }
#undef GPTQ_READ_A
    };
    // Before the first use of operand i of a k step: LDS reads return in order, and the reads issued after
    // operand i's are the rest of its own k step (TM-1-i) and those of the current k step issued so far
    // (one per slot in the first TM slots).  Reads the compiler issues in between only make this stricter.
    // (The operand is an in/out of the wait, so that the MFMA that consumes it cannot be moved above it.)
    auto wait_afrag = [&](int i, half8_t &frag) {
#define GPTQ_WAIT_A(I)                                                                                              \
    case I:                                                                                                         \
        asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(frag) : "n"(TM - 1 - (I) + (((I) * TN < TM) ? (I) * TN : TM))); \
        break;
        switch (i) {
            GPTQ_WAIT_A(0) GPTQ_WAIT_A(1) GPTQ_WAIT_A(2) GPTQ_WAIT_A(3)
            GPTQ_WAIT_A(4) GPTQ_WAIT_A(5) GPTQ_WAIT_A(6) GPTQ_WAIT_A(7)
        }
#undef GPTQ_WAIT_A
    };
    // this lane's packed words, scales and zero points of a whole stage
    auto read_weights = [&](int ring, uint32_t (&w)[KSTEPS][TN], uint32_t (&nz)[TN], uint32_t (&ss)[TN]) {
        const unsigned char *base = stage_base(ring) + L::A_BYTES;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            const unsigned char *src = base + ((size_t)(2 * kk + kh) * BN + col_local) * 4;
            if (TN == 4) {
                const uint4 v = *reinterpret_cast<const uint4 *>(src);
                w[kk][0] = v.x;
                w[kk][1 % TN] = v.y;
                w[kk][2 % TN] = v.z;
                w[kk][3 % TN] = v.w;
            } else if (TN == 2) {
                const uint2 v = *reinterpret_cast<const uint2 *>(src);
                w[kk][0] = v.x;
                w[kk][1 % TN] = v.y;
            } else {
                w[kk][0] = *reinterpret_cast<const uint32_t *>(src);
            }
        }
        const unsigned char *sz = base + L::B_BYTES;
        const uint32_t zword = *reinterpret_cast<const uint32_t *>(sz + BN * 2 + (col_local >> 3) * 4);
#pragma unroll
        for (int t = 0; t < TN; ++t) {
            const uint32_t sb = *reinterpret_cast<const uint16_t *>(sz + (col_local + t) * 2);
            ss[t] = sb | (sb << 16);
            nz[t] = neg_bias((zword >> (4 * ((col_local + t) & 7))) & 15u);
        }
    };

    // One k step, in exactly this instruction order (a scheduling barrier closes every slot): ONE MFMA, then
    // its share of the work for the NEXT k step - an LDS read of an A operand (first TM slots), dequantisation
    // of weight pairs, and whatever `extra` adds (loads for a later stage, weight reads for the next one).
    // An MFMA occupies the matrix pipe for 8 passes but the wave can issue other instructions right behind it,
    // so a handful of them per MFMA run in its shadow; several MFMAs back to back followed by a block of
    // vector work would leave the pipe idle during the block.
    constexpr int SLOTS = TM * TN;  // MFMAs per k step
    constexpr int PAIRS = 4 * TN;   // half2 results to produce per k step
    auto kstep = [&](auto parity, int next_ring, int next_kk, const uint32_t (&nw)[TN], const uint32_t (&nnz)[TN],
                     const uint32_t (&nss)[TN], auto &&extra) {
        constexpr int CUR = std::decay_t<decltype(parity)>::value, NXT = CUR ^ 1;
        uint32_t pending[(PAIRS + SLOTS - 1) / SLOTS] = {};
#pragma unroll
        for (int m = 0; m < SLOTS; ++m) {
            const int i = m / TN, t = m % TN;
            if (t == 0)
                wait_afrag(i, afr[CUR][i]);
            acc[i][t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(afr[CUR][i], __builtin_bit_cast(half8_t, bfr[CUR][t]),
                                                               acc[i][t], 0, 0, 0);
            if (m < TM)
                read_afrag(next_ring, next_kk, m, afr[NXT][m]);
            // pairs [m * PAIRS / SLOTS, (m + 1) * PAIRS / SLOTS) belong to this slot: their conversion and
            // zero-point subtraction happen here, the multiply by the scale one slot later (the last slot
            // finishes its own), so no multiply directly follows the add it depends on
            constexpr int PPS = (PAIRS + SLOTS - 1) / SLOTS;
            uint32_t now[PPS];
#pragma unroll
            for (int pair = m * PAIRS / SLOTS; pair < (m + 1) * PAIRS / SLOTS; ++pair) {
                const int pt = pair >> 2;
                uint32_t r;
                switch (pair & 3) {
                case 0: r = dequant_pair_begin<0>(nw[pt], magic, nnz[pt]); break;
                case 1: r = dequant_pair_begin<1>(nw[pt], magic, nnz[pt]); break;
                case 2: r = dequant_pair_begin<2>(nw[pt], magic, nnz[pt]); break;
                default: r = dequant_pair_begin<3>(nw[pt], magic, nnz[pt]); break;
                }
                now[pair - m * PAIRS / SLOTS] = r;
            }
            if (m > 0) {
#pragma unroll
                for (int pair = (m - 1) * PAIRS / SLOTS; pair < m * PAIRS / SLOTS; ++pair) {
                    const int pt = pair >> 2;
                    bfr[NXT][pt][pair & 3] = dequant_pair_end(pending[pair - (m - 1) * PAIRS / SLOTS], nss[pt]);
                }
            }
#pragma unroll
            for (int q = 0; q < PPS; ++q)
                pending[q] = now[q];
            if (m == SLOTS - 1) {
#pragma unroll
                for (int pair = m * PAIRS / SLOTS; pair < (m + 1) * PAIRS / SLOTS; ++pair) {
                    const int pt = pair >> 2;
                    bfr[NXT][pt][pair & 3] = dequant_pair_end(pending[pair - m * PAIRS / SLOTS], nss[pt]);
                }
            }
            extra(m);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    auto nothing = [](int) {};

    // ---- prologue: put NBUF-1 stages in flight, publish the first two, load the first operands ----
#pragma unroll
    for (int s = 0; s < NBUF - 1; ++s) {
#pragma unroll
        for (int p = 0; p < LOADS_PER_STAGE; ++p)
            issue_piece(p, s);
        advance_load_stage();
    }
    publish();
    read_weights(0, w_cur, nz_cur, ss_cur);
#pragma unroll
    for (int i = 0; i < TM; ++i)
        read_afrag(0, 0, i, afr[0][i]);
#pragma unroll
    for (int t = 0; t < TN; ++t) {
        bfr[0][t][0] = dequant_pair<0>(w_cur[0][t], magic, nz_cur[t], ss_cur[t]);
        bfr[0][t][1] = dequant_pair<1>(w_cur[0][t], magic, nz_cur[t], ss_cur[t]);
        bfr[0][t][2] = dequant_pair<2>(w_cur[0][t], magic, nz_cur[t], ss_cur[t]);
        bfr[0][t][3] = dequant_pair<3>(w_cur[0][t], magic, nz_cur[t], ss_cur[t]);
    }

    // Invariant at the top of stage s: stages s and s+1 are in LDS and visible, every wave has left stage s-1,
    // and the operands of k step 0 of stage s sit in afr[0] / bfr[0].
    int ring = 0;  // s % NBUF
    for (int s = 0; s < stages; ++s) {
        const int ring_next = ring + 1 == NBUF ? 0 : ring + 1;
        const int ring_free = ring == 0 ? NBUF - 1 : ring - 1;  // buffer of stage s-1
        // the loads of stage s+NBUF-1 (into the buffer stage s-1 has left) are spread over the slots of the
        // first k step, so that they issue in the shadow of MFMAs like everything else
        constexpr int PIECES_PER_SLOT = (LOADS_PER_STAGE + SLOTS - 1) / SLOTS;
        auto issue_loads = [&](int m) {
#pragma unroll
            for (int q = 0; q < PIECES_PER_SLOT; ++q)
                if (m * PIECES_PER_SLOT + q < LOADS_PER_STAGE)
                    issue_piece(m * PIECES_PER_SLOT + q, ring_free);
        };
        auto fetch_next_weights = [&](int m) {
            if (m == SLOTS - 1)
                read_weights(ring_next, w_nxt, nz_nxt, ss_nxt);
        };
        if (KSTEPS == 4) {
            kstep(P0{}, ring, 1, w_cur[1], nz_cur, ss_cur, issue_loads);
            kstep(P1{}, ring, 2, w_cur[2 % KSTEPS], nz_cur, ss_cur, nothing);
            kstep(P0{}, ring, 3, w_cur[3 % KSTEPS], nz_cur, ss_cur, fetch_next_weights);
            kstep(P1{}, ring_next, 0, w_nxt[0], nz_nxt, ss_nxt, nothing);
        } else {
            auto both = [&](int m) {
                issue_loads(m);
                fetch_next_weights(m);
            };
            kstep(P0{}, ring, 1, w_cur[1], nz_cur, ss_cur, both);
            kstep(P1{}, ring_next, 0, w_nxt[0], nz_nxt, ss_nxt, nothing);
        }
        advance_load_stage();
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk)
#pragma unroll
            for (int t = 0; t < TN; ++t)
                w_cur[kk][t] = w_nxt[kk][t];
#pragma unroll
        for (int t = 0; t < TN; ++t) {
            nz_cur[t] = nz_nxt[t];
            ss_cur[t] = ss_nxt[t];
        }
        publish();  // stage s+2 has landed; everyone is done with stage s
        ring = ring_next;
    }
    // nothing may still be writing this workgroup's LDS when it retires; the LDS wait retires the operand reads
    // issued for the stage after the last one, whose destination registers stay reserved until here (named as
    // in/outs after the wait: the compiler knows nothing of the inline-asm reads in flight and could otherwise
    // reuse the registers of these dead values while a read is still due to land in them)
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int i = 0; i < TM; ++i)
        asm volatile("" : "+v"(afr[0][i]), "+v"(afr[1][i]));

    if (a.split_k > 1) {
        constexpr int ACC = TM * TN * 16;
        float flat[ACC];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int t = 0; t < TN; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    flat[(i * TN + t) * 16 + r] = acc[i][t][r];
        if (!combine_slices<ACC>(flat, a, slice, tile_id, tid))
            return;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int t = 0; t < TN; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    acc[i][t][r] = flat[(i * TN + t) * 16 + r];
    }
    store_tile<TM, TN>(acc, a.out, m0 + wm * WAVE_M, col_raw, col_ok, kh, M, N);
}

// =====================================================================================================
// General path (g_idx, any group size, k tail): registers -> LDS, two buffers, one barrier per stage
// =====================================================================================================

template <int BM, int BN, int WM, int WN, int MODE>
__global__ __launch_bounds__(kThreads) void prefill_general_kernel(const Args a)
{
    static_assert(WM * WN == 4, "four wavefronts per workgroup");
    static_assert(MODE == kGroupPerRow || MODE == kActOrder, "the tuned modes use the pipelined kernel");
    constexpr int BK = 64;
    constexpr int WAVE_M = BM / WM;
    constexpr int WAVE_N = BN / WN;
    constexpr int TM = WAVE_M / 32;
    constexpr int TN = WAVE_N / 32;
    static_assert(TM >= 1 && (TN == 1 || TN == 2 || TN == 4), "wave tile: 32-row blocks by 32/64/128 columns");
    constexpr int A_CHUNKS = BM * (BK / 8) / kThreads;
    static_assert(A_CHUNKS >= 1, "tile too small for 256 threads");
    constexpr int KSTEPS = BK / 16;
    constexpr int STAGE_HALVES = BM * BK;

    extern __shared__ __align__(16) unsigned char smem[];
    half_t *lds_a = reinterpret_cast<half_t *>(smem);  // [2][BM][64] halves, chunk-swizzled

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN;
    const int wn = wave % WN;
    const int lj = lane & 31;
    const int kh = lane >> 5;

    int tile_m, tile_n;
    int tile_id, slice;
    if (!tile_of_workgroup(a, tile_m, tile_n, tile_id, slice))
        return;
    const int m0 = tile_m * BM;
    const int n0 = tile_n * BN;
    const int N = a.N, K = a.K, M = a.M;
    const int rows = K >> 3;
    const int col_raw = n0 + wn * WAVE_N + TN * lj;
    const bool col_ok = col_raw < N;
    const int col0 = col_ok ? col_raw : N - TN;  // clamped: see the pipelined kernel
    const int zshift = 4 * (col0 & 7);
    const int stages = (K + BK - 1) / BK;

    float16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int t = 0; t < TN; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[i][t][r] = 0.f;

    // slot p (16 bytes) holds chunk (p & 7) ^ ((row >> 1) & 7) of row p >> 3 (64 banks, 16 lanes per pass)
    const half_t *a_src[A_CHUNKS];
#pragma unroll
    for (int c = 0; c < A_CHUNKS; ++c) {
        const int slot = tid + c * kThreads;
        const int row = slot >> 3;
        const int ch = (slot & 7) ^ ((row >> 1) & 7);
        a_src[c] = a.x + (size_t)min(m0 + row, M - 1) * K + ch * 8;
    }
    uint4 a_next[A_CHUNKS];
    auto load_a = [&](int stage) {
        const int k0 = stage * BK;
#pragma unroll
        for (int c = 0; c < A_CHUNKS; ++c) {
            const int slot = tid + c * kThreads;
            const int ch = (slot & 7) ^ ((slot >> 4) & 7);
            const int k = k0 + ch * 8;
            const uint4 v = *reinterpret_cast<const uint4 *>(a_src[c] + min(k0, K - 8 - ch * 8));
            a_next[c] = k < K ? v : make_uint4(0, 0, 0, 0);  // the k tail must contribute exact zeros
        }
    };
    auto store_a = [&](int buf) {
#pragma unroll
        for (int c = 0; c < A_CHUNKS; ++c) {
            const int slot = tid + c * kThreads;
            *reinterpret_cast<uint4 *>(lds_a + (size_t)buf * STAGE_HALVES + (size_t)slot * 8) = a_next[c];
        }
    };
    uint32_t w_cur[KSTEPS][TN], w_nxt[KSTEPS][TN];
    auto load_b = [&](int stage, uint32_t (&w)[KSTEPS][TN]) {
        const int prow0 = stage * (BK / 8);
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            const int prow = min(prow0 + 2 * kk + kh, rows - 1);
            const uint32_t *src = a.qweight + (size_t)prow * N + col0;
            if (TN == 4) {
                const uint4 v = *reinterpret_cast<const uint4 *>(src);
                w[kk][0] = v.x;
                w[kk][1 % TN] = v.y;
                w[kk][2 % TN] = v.z;
                w[kk][3 % TN] = v.w;
            } else if (TN == 2) {
                const uint2 v = *reinterpret_cast<const uint2 *>(src);
                w[kk][0] = v.x;
                w[kk][1 % TN] = v.y;
            } else {
                w[kk][0] = *src;
            }
        }
    };
    const PairMagic magic;

    // B operands of k step `kk` of stage `s`, dequantised in registers
    auto make_bfrags = [&](int s, int kk, u32x4_t bfrag[TN]) {
        const int prow = s * (BK / 8) + 2 * kk + kh;  // this lane's packed row
#pragma unroll
        for (int t = 0; t < TN; ++t) {
            uint32_t nz[4] = {0, 0, 0, 0}, ss[4] = {0, 0, 0, 0};
            if (prow < rows) {  // past the k tail the scale stays zero: exact zero weights
                if (MODE == kGroupPerRow) {
                    const int g = (prow * 8) / a.group_size;
                    const uint32_t sb = __builtin_bit_cast(uint16_t, a.scales[(size_t)g * N + col0 + t]);
                    const uint32_t z = (a.qzeros[(size_t)g * (N >> 3) + (col0 >> 3)] >> (zshift + 4 * t)) & 15u;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        nz[i] = neg_bias(z);
                        ss[i] = sb | (sb << 16);
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int g0 = a.g_idx[prow * 8 + 2 * i];
                        const int g1 = a.g_idx[prow * 8 + 2 * i + 1];
                        const uint32_t s0 = __builtin_bit_cast(uint16_t, a.scales[(size_t)g0 * N + col0 + t]);
                        const uint32_t s1 = __builtin_bit_cast(uint16_t, a.scales[(size_t)g1 * N + col0 + t]);
                        const uint32_t z0 = (a.qzeros[(size_t)g0 * (N >> 3) + (col0 >> 3)] >> (zshift + 4 * t)) & 15u;
                        const uint32_t z1 = (a.qzeros[(size_t)g1 * (N >> 3) + (col0 >> 3)] >> (zshift + 4 * t)) & 15u;
                        nz[i] = 0xD400E400u | z0 | (z1 << 20);
                        ss[i] = s0 | (s1 << 16);
                    }
                }
            }
            bfrag[t] = dequant_word(w_cur[kk][t], magic, nz, ss);
        }
    };
    auto read_afrags = [&](const half_t *base, int kk, half8_t af[TM]) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row = wm * WAVE_M + i * 32 + lj;
            const int ch = (2 * kk + kh) ^ ((row >> 1) & 7);
            af[i] = *reinterpret_cast<const half8_t *>(base + (size_t)row * BK + ch * 8);
        }
    };

    half8_t af[2][TM];
    u32x4_t bf[2][TN];
    load_a(0);
    load_b(0, w_cur);
    store_a(0);
    __syncthreads();
    for (int s = 0; s < stages; ++s) {
        const int buf = s & 1;
        const int sn = min(s + 1, stages - 1);  // the last iteration harmlessly refetches its own stage
        load_a(sn);
        load_b(sn, w_nxt);
        const half_t *base = lds_a + (size_t)buf * STAGE_HALVES;
        read_afrags(base, 0, af[0]);
        make_bfrags(s, 0, bf[0]);
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            if (kk + 1 < KSTEPS) {
                read_afrags(base, kk + 1, af[(kk + 1) & 1]);
                make_bfrags(s, kk + 1, bf[(kk + 1) & 1]);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int t = 0; t < TN; ++t)
                    acc[i][t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                        af[kk & 1][i], __builtin_bit_cast(half8_t, bf[kk & 1][t]), acc[i][t], 0, 0, 0);
        }
        store_a(buf ^ 1);
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk)
#pragma unroll
            for (int t = 0; t < TN; ++t)
                w_cur[kk][t] = w_nxt[kk][t];
        __syncthreads();
    }

    store_tile<TM, TN>(acc, a.out, m0 + wm * WAVE_M, col_raw, col_ok, kh, M, N);
}

}  // namespace prefill
}  // namespace gptq

// Small-batch MFMA kernel for the W4A16 GPTQ matrix multiply (2 <= M <= 64 per launch), gfx950.
//
// Between the vector kernel (which runs out of vector ALU throughput once every weight has to be
// multiplied with more than a few batch rows) and the big-tile MFMA kernel (which needs hundreds of rows
// to fill its tiles) the problem is still bound by streaming the packed weights from HBM, but the
// contraction no longer fits the vector units.  This kernel keeps the work decomposition of the vector
// kernel - a workgroup owns 64 columns and one K slice, its four wavefronts split the slice, partial
// sums meet in LDS and then in scratch, in a fixed order (Opt4GPTQ, Section 3.1) - and hands the
// contraction to v_mfma_f32_16x16x32_f16:
//   * one lane of the MFMA B operand holds 8 consecutive k of one column, which is exactly one packed
//     qweight word: a lane loads four adjacent words (128 bits; a wavefront load touches 4 packed rows x
//     256 contiguous bytes), dequantises them in registers (exact q - z, one fp16 multiply by the scale)
//     and feeds four MFMAs, n-block t <-> column 4*(lane%16) + t;
//   * the activations of the slice are staged in LDS with 128-bit accesses (Section 3.2), 16-byte chunks
//     XOR-swizzled by row so that the 16-row operand reads are bank-conflict free;
//   * every weight is read once and dequantised once, whatever M is: 2 vector ALU operations per weight
//     instead of 1.2 + M/2 in the vector kernel.
// Supports no g_idx and group sizes that are multiples of 128 (the tuned format) or 64 / 32 (template GPU);
// other cases use the other kernels.
#pragma once

#include "exchange.h"
#include "kernels.h"

#include <type_traits>

namespace gptq {
namespace skinny {

constexpr int kCols = 64;      // columns per workgroup
constexpr int kUnitK = 128;    // k per pipeline unit (4 MFMA steps of 32)

struct Args {
    const half_t *x;
    const uint32_t *qweight;
    const uint32_t *qzeros;
    const half_t *scales;
    half_t *out;
    float *partial;      // [split_k, M, N] fp32, only if split_k > 1
    unsigned *counters;  // [tiles_n], zero between launches
    int M, K, N;
    int units_per_group;  // group_size / 128
    int unit_group_shift; // log2(units_per_group) if that is a power of two, else -1
    int tiles_n;
    int split_k;
    int units_per_slice;  // 128-k units per K slice (multiple of 4 where possible)
    int total_units;      // K / 128
};

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ half2_t as_half2(uint32_t v)
{
    return __builtin_bit_cast(half2_t, v);
}

// Bit patterns that turn 4-bit codes into fp16 values without an integer-to-float conversion:
// 0x6400 is 1024.0 (ulp 1): OR-ing a nibble into bits 0..3 gives 1024 + q exactly;
// 0x5400 is 64.0 (ulp 1/16): OR-ing a nibble into bits 4..7 gives 64 + q exactly.
// The constants are kept in registers (not literals) so that each pair costs ONE v_and_or_b32.
struct NibbleMagic {
    uint32_t mask_lo, mask_hi, bias_lo, bias_hi;
    __device__ __forceinline__ NibbleMagic()
    {
        mask_lo = 0x000f000fu;
        mask_hi = 0x00f000f0u;
        bias_lo = 0x64006400u;
        bias_hi = 0x54005400u;
        asm volatile("" : "+s"(mask_lo), "+s"(mask_hi), "+v"(bias_lo), "+v"(bias_hi));
    }
};

__device__ __forceinline__ void store_device_scope(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_device_scope(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Loads of one 128-k unit of one lane: 4 steps x 4 adjacent words, plus the unit's scales and zero word.
template <int XROWS, int GPU>  // XROWS: 16-row blocks of activations that travel with the weights (0: they are in LDS)
struct UnitRegs {                // GPU: quantisation groups per unit (1: groups of 128 k or more; 2: 64; 4: 32)
    uint4 w[4];
    uint2 sc[GPU];  // four fp16 scales as raw bits, per group of the unit
    uint32_t zb[GPU];
    u32x4_t xa[XROWS > 0 ? XROWS : 1][4];  // A operand per row block and k step
};

// TM: 16-row blocks (M <= 16 * TM).  WN: wavefronts side by side along N (1, 2 or 4).  With WN = 1 the
// workgroup owns 64 columns and its four wavefronts split the K slice (narrow layers: many small
// workgroups); with WN = 4 it owns 256 columns, every wavefront walks the whole slice for its own 64
// columns and the staged activations serve four times as many weights (wide layers).
//
// WAVES wavefronts per workgroup: four, or - 64-column workgroups that have a compute unit to themselves -
// eight, two per SIMD, so that the loads, LDS and scalar instructions of one overlap the arithmetic of the
// other (3-11 % on the narrow and deep Llama layers; with more workgroups than compute units the co-resident
// workgroups already do that, and eight wavefronts each measured 3-12 % slower).
//
// GPU: quantisation groups per 128-k unit.  1 serves every group size that is a multiple of 128; 2 and 4 serve
// groups of 64 and 32 k: a unit then carries two or four (scale, zero) rows, the exact q - z of a 32-k step is
// formed with its own group's zero point and the MFMA chain is scaled and restarted at every group boundary.
template <int TM, int WN, int WAVES, int GPU = 1>
__global__ __launch_bounds__(64 * WAVES) void skinny_kernel(const Args a)
{
    static_assert(GPU == 1 || GPU == 2 || GPU == 4, "groups of >= 128, 64 or 32 k");
    static_assert(GPU == 1 || TM <= 2, "small groups: up to two row blocks");
    static_assert(WAVES == 4 || (WAVES == 8 && WN <= 2), "eight wavefronts only where they split the slice");
    static_assert(WN != 2 || WAVES == 8, "128-column workgroups: two column blocks x four wavefronts each");
    constexpr int kWaves = WAVES;
    constexpr int kThreads = 64 * WAVES;
    constexpr int ROWS = 16 * TM;
    constexpr int COLS = kCols * WN;   // columns per workgroup
    constexpr int KW = kWaves / WN;    // wavefronts that share a column block and split the slice
    // With 64-column workgroups every activation is used by exactly one lane (the wavefronts split the
    // slice), so staging them in LDS would be a copy without reuse: each lane loads its A operand straight
    // from global memory (L2), in the same pipeline as the weights.  With 256-column workgroups the four
    // wavefronts share the slice and the activations are staged once in LDS.
    // (128-column workgroups, WN = 2 with eight wavefronts, read them the same way: every activation is then
    // loaded by the two wavefronts that share its k range, from L2.)
    constexpr bool DIRECT = WN <= 2;
    // DIRECT with four row blocks: the A operands of two units in flight would take 128 registers.  They are kept
    // for ONE unit instead and refilled step by step: as soon as a 32-k step's operands have been permuted into
    // the MFMA's k order, the same registers receive that step of the NEXT unit (from L2: a four-step lead is
    // enough), which leaves room for two wavefronts per SIMD.
    constexpr bool XSTEP = DIRECT && TM >= 4;
    using Regs = UnitRegs<(DIRECT && !XSTEP) ? TM : 0, GPU>;

    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int s_last;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cq = lane & 15;  // column quad: columns n0 + 4*cq .. +3
    const int kg = lane >> 4;  // k group inside a 32-k step = packed row inside the step
    const int tile = blockIdx.x % a.tiles_n;
    const int slice = blockIdx.x / a.tiles_n;
    const int N = a.N;
    const int cb = wave / KW;  // this wavefront's 64-column block inside the tile
    const int kw = wave % KW;  // and its share of the slice
    const int n0 = tile * COLS + cb * kCols + 4 * cq;
    const int nc = min(n0, N - 4);  // clamped for loads; columns past N are never stored

    const int u0 = slice * a.units_per_slice;
    const int u1 = min(u0 + a.units_per_slice, a.total_units);
    const int nunits = u1 - u0;
    const int kbeg = u0 * kUnitK;
    const int Ls = nunits * kUnitK;  // activations of this slice per row (multiple of 128)

    // this wavefront's contiguous share of the slice's units
    const int per_wave = (nunits + KW - 1) / KW;
    const int wu0 = min(u0 + kw * per_wave, u1);
    const int wu1 = min(wu0 + per_wave, u1);

    half_t *xs = reinterpret_cast<half_t *>(smem);  // [ROWS][Ls], 16-byte chunks swizzled by row

    // Addresses are a wavefront-uniform base (the unit, the step and the group are the same for all lanes:
    // scalar registers) plus a 32-bit byte offset per lane.  Nothing waits on a load where it is issued
    // (the zero word is shifted when it is used) and no branch sits between a load and its use.
    const uint32_t voff_w = ((uint32_t)kg * N + nc) * 4u;
    const uint32_t voff_s = (uint32_t)nc * 2u;
    const uint32_t voff_z = (uint32_t)(nc >> 3) * 4u;
    const int zshift = (nc & 4) * 4;
    uint32_t voff_x[TM];  // DIRECT: this lane's row and k group inside a 32-k step, as a byte offset
#pragma unroll
    for (int i = 0; i < TM; ++i)
        voff_x[i] = ((uint32_t)min(16 * i + cq, a.M - 1) * a.K + kg * 8) * 2u;
    auto issue = [&](int u, Regs &r) {
        const int uc = min(u, u1 - 1);  // clamped: a unit past the end is loaded again but not consumed
        const uint32_t *wrow = a.qweight + (size_t)uc * 16 * N;
#pragma unroll
        for (int s = 0; s < 4; ++s)
            r.w[s] = *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(wrow + (size_t)s * 4 * N) +
                                                      voff_w);
        const int grp0 = GPU > 1 ? uc * GPU
                                 : (a.unit_group_shift >= 0 ? (uc >> a.unit_group_shift) : uc / a.units_per_group);
#pragma unroll
        for (int h = 0; h < GPU; ++h) {
            const int grp = grp0 + h;
            r.sc[h] =
                *reinterpret_cast<const uint2 *>(reinterpret_cast<const char *>(a.scales + (size_t)grp * N) + voff_s);
            r.zb[h] = *reinterpret_cast<const uint32_t *>(
                reinterpret_cast<const char *>(a.qzeros + (size_t)grp * (N >> 3)) + voff_z);
        }
        if (DIRECT && !XSTEP) {
            const half_t *xrow = a.x + (size_t)uc * kUnitK;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int st = 0; st < 4; ++st)
                    r.xa[i][st] = *reinterpret_cast<const u32x4_t *>(reinterpret_cast<const char *>(xrow + st * 32) +
                                                                     voff_x[i]);
        }
    };
    u32x4_t xstep[XSTEP ? TM : 1][4];  // XSTEP: the A operands of the unit being consumed, refilled per step
    auto issue_x = [&](int u, int st) {
        const half_t *xrow = a.x + (size_t)min(u, u1 - 1) * kUnitK + st * 32;
#pragma unroll
        for (int i = 0; i < (XSTEP ? TM : 1); ++i)
            xstep[i][st] = *reinterpret_cast<const u32x4_t *>(reinterpret_cast<const char *>(xrow) + voff_x[i]);
    };

    Regs ra, rb;
    const bool active = wu0 < wu1;
    if (active) {
        issue(wu0, ra);  // in flight while the activations are staged (when they are)
        if (XSTEP) {
#pragma unroll
            for (int st = 0; st < 4; ++st)
                issue_x(wu0, st);
        }
    }

    // ---- stage the activations global -> LDS by DMA (no registers, all loads in flight at once): 16-byte slot p
    //      of the buffer holds, for row m = p / chunks, the chunk whose index is p % chunks with its low four
    //      bits XORed with m (the swizzle is its own inverse).  Rows past M repeat row M-1: their outputs are
    //      never stored.
    if (!DIRECT) {
        typedef __attribute__((address_space(3))) void lds_ptr_t;
        typedef __attribute__((address_space(1))) const void global_ptr_t;
        const int chunks = Ls >> 3;
        const int per_thread = ROWS * chunks / kThreads;  // ROWS * chunks is a multiple of 256
        for (int j = 0; j < per_thread; ++j) {
            const int p = j * kThreads + tid;
            const int m = p / chunks;
            const int pc = p - m * chunks;
            const int c = (pc & ~15) | ((pc ^ m) & 15);
            const half_t *src = a.x + (size_t)min(m, a.M - 1) * a.K + kbeg + c * 8;
            __builtin_amdgcn_global_load_lds((global_ptr_t *)src,
                                             (lds_ptr_t *)(smem + (size_t)(j * kThreads + wave * 64) * 16), 16, 0, 0);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the DMA is not ordered against LDS reads by the compiler
        __syncthreads();
    }

    float4_t acc[TM][4];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int t = 0; t < 4; ++t)
            acc[i][t] = float4_t{0.f, 0.f, 0.f, 0.f};

    const NibbleMagic magic;

    // One unit: 128 k of this lane's four columns against all batch rows.
    //
    // The B operand is the exact integer q - z, not the weight: a pair of nibbles four k apart is masked out of
    // the packed word and OR-ed into the mantissa of 1024.0 (even k) or 64.0 (odd k), and one packed fp16 add of
    // -(1024 + z) or -(64 + z) leaves q - z (exact: small integers).  Nine vector operations per packed word
    // instead of sixteen for per-element weights; the group's scale is applied to the MFMA chain's result in
    // fp32:  acc += s * sum_k x_k (q_k - z).  (Contracting the biased codes and cancelling sum_k x_k * bias
    // afterwards saves the adds but loses digits to the size of that sum: activations with a common offset of a
    // few tens then leave the tolerance band.)
    // From four row blocks on (SCALE_B) the scale goes into the B operand instead (one more packed multiply per
    // pair: the fp16 weight itself, rounded once) and the MFMAs add straight into the running sums: scaling the
    // sums of 4 x 16 rows per group would cost as many operations and twice the accumulator registers.
    constexpr bool SCALE_B = TM >= 4;
    auto consume = [&](int u, const Regs &r, auto refill) {
        constexpr bool REFILL = decltype(refill)::value;  // XSTEP: fetch the next unit's A operands step by step
        const int j = u - u0;
        constexpr int SPG = 4 / GPU;  // 32-k steps per quantisation group
        half2_t neg_lo[4], neg_hi[4], s2[4];
        float sf[4];
        float4_t d[SCALE_B ? 1 : TM][4];
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            if (st % SPG == 0) {  // a group begins: its zero points and scales
                const int h = st / SPG;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const uint32_t z = (r.zb[h] >> (zshift + 4 * t)) & 15u;
                    const uint32_t zz = z | (z << 16);
                    neg_lo[t] = as_half2(zz | 0xE400E400u);         // (-(1024 + z)) x2
                    neg_hi[t] = as_half2((zz << 4) | 0xD400D400u);  // (-(64 + z)) x2
                    const uint32_t pair = t < 2 ? r.sc[h].x : r.sc[h].y;
                    const uint16_t sb = (uint16_t)((t & 1) ? (pair >> 16) : (pair & 0xffffu));
                    sf[t] = (float)__builtin_bit_cast(half_t, sb);
                    s2[t] = as_half2((uint32_t)sb | ((uint32_t)sb << 16));
                }
            }
            const uint32_t w[4] = {r.w[st].x, r.w[st].y, r.w[st].z, r.w[st].w};
            const int c = (j * 4 + st) * 4 + kg;  // 16-byte chunk of the activation row
            half8_t av[TM];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                u32x4_t xv;
                if (XSTEP) {
                    xv = xstep[i][st];
                } else if (DIRECT) {
                    xv = r.xa[i][st];
                } else {
                    const int m = 16 * i + cq;  // the A operand lane holds row lane % 16
                    const int pc = (c & ~15) | ((c ^ m) & 15);
                    xv = *reinterpret_cast<const u32x4_t *>(xs + (size_t)m * Ls + pc * 8);
                }
                // the same k order for the activations: halves (0,4) (1,5) (2,6) (3,7)
                const u32x4_t xp = {__builtin_amdgcn_perm(xv[2], xv[0], 0x05040100u),
                                    __builtin_amdgcn_perm(xv[2], xv[0], 0x07060302u),
                                    __builtin_amdgcn_perm(xv[3], xv[1], 0x05040100u),
                                    __builtin_amdgcn_perm(xv[3], xv[1], 0x07060302u)};
                av[i] = __builtin_bit_cast(half8_t, xp);
            }
            if (XSTEP && REFILL)
                issue_x(u + 1, st);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const uint32_t w8 = w[t] >> 8;
                // k order inside the operand: (0,4) (1,5) (2,6) (3,7)
                half2_t c0 = as_half2((w[t] & magic.mask_lo) | magic.bias_lo) + neg_lo[t];
                half2_t c1 = as_half2((w[t] & magic.mask_hi) | magic.bias_hi) + neg_hi[t];
                half2_t c2 = as_half2((w8 & magic.mask_lo) | magic.bias_lo) + neg_lo[t];
                half2_t c3 = as_half2((w8 & magic.mask_hi) | magic.bias_hi) + neg_hi[t];
                if (SCALE_B) {
                    c0 *= s2[t];
                    c1 *= s2[t];
                    c2 *= s2[t];
                    c3 *= s2[t];
                }
                const half8_t b = half8_t{c0[0], c0[1], c1[0], c1[1], c2[0], c2[1], c3[0], c3[1]};
                const float4_t zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    if (SCALE_B)
                        acc[i][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(av[i], b, acc[i][t], 0, 0, 0);
                    else
                        d[i][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(av[i], b, st % SPG == 0 ? zero : d[i][t], 0, 0,
                                                                         0);
                }
            }
            if (!SCALE_B && st % SPG == SPG - 1) {  // the group is complete: scale its sum
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int t = 0; t < 4; ++t)
#pragma unroll
                        for (int rr = 0; rr < 4; ++rr)
                            acc[i][t][rr] = __builtin_fmaf(sf[t], d[i][t][rr], acc[i][t][rr]);
            }
        }
    };

    if (active) {
        // Software pipeline over two register sets: the next unit's weights fly while this one is consumed.
        // The steady-state loop issues unconditionally and the last one or two units are peeled; at a unit
        // boundary the accumulators are pinned (empty asm) and the scheduler stopped, so that the loads of
        // the unit after next are issued after this unit's arithmetic: two units in flight, not three.
        auto unit_boundary = [&]() {
            // (with four row blocks the running sums live in accumulation registers: pinning them as vector
            // registers would copy all 64 out and back at every unit)
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                if (TM >= 4)
                    asm volatile("" : "+a"(acc[i][0]), "+a"(acc[i][1]), "+a"(acc[i][2]), "+a"(acc[i][3])::"memory");
                else
                    asm volatile("" : "+v"(acc[i][0]), "+v"(acc[i][1]), "+v"(acc[i][2]), "+v"(acc[i][3])::"memory");
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        const std::integral_constant<bool, true> more;
        const std::integral_constant<bool, false> last;
        int u = wu0;
        while (u + 2 < wu1) {
            issue(u + 1, rb);
            consume(u, ra, more);
            unit_boundary();
            issue(u + 2, ra);
            consume(u + 1, rb, more);
            unit_boundary();
            u += 2;
        }
        if (u + 2 == wu1) {
            issue(u + 1, rb);
            consume(u, ra, more);
            unit_boundary();
            consume(u + 1, rb, last);
        } else {
            consume(u, ra, last);
        }
    }

    // ---- through LDS (the activation buffer is reused): reduce over the wavefronts that split the slice
    //      and turn the MFMA register layout into rows of adjacent columns ----
    // lane holds, for block i, n-block t, register r: row 16*i + 4*kg + r, column 4*cq + t of its block
    __syncthreads();
    float *red = reinterpret_cast<float *>(smem);  // [KW][ROWS][COLS]
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = 16 * i + 4 * kg + r;
            float4_t v = {acc[i][0][r], acc[i][1][r], acc[i][2][r], acc[i][3][r]};
            *reinterpret_cast<float4_t *>(red + ((size_t)kw * ROWS + row) * COLS + cb * kCols + 4 * cq) = v;
        }
    __syncthreads();
    for (int i = tid; i < a.M * COLS; i += kThreads) {
        const int m = i / COLS;
        const int col = i - m * COLS;
        const int n = tile * COLS + col;
        float s = red[(size_t)m * COLS + col];
#pragma unroll
        for (int w = 1; w < KW; ++w)
            s += red[((size_t)w * ROWS + m) * COLS + col];
        if (n < N) {
            if (a.split_k == 1)
                a.out[(size_t)m * N + n] = (half_t)s;
            else
                store_device_scope(a.partial + ((size_t)slice * a.M + m) * N + n, s);
        }
    }

    // ---- combine the K slices: the last workgroup of this column tile adds them in slice order ----
    if (a.split_k > 1) {
        __builtin_amdgcn_s_waitcnt(0);  // every partial store of this workgroup has been acknowledged (exchange.h)
        __syncthreads();
        if (tid == 0)
            s_last = (slice_arrive(a.counters + tile) == (unsigned)(a.split_k - 1));
        __syncthreads();
        if (s_last) {
            slice_acquire();
            // All partial sums a thread needs are requested before the first is used (up to four outputs
            // times eight slices in flight), so the combine costs one scratch round trip, not one per
            // output; the additions stay in slice order.
            auto combine = [&](auto outs) {
            constexpr int OUTS = decltype(outs)::value;
            for (int i0 = tid; i0 < a.M * COLS; i0 += OUTS * kThreads) {
                float s[OUTS];
                size_t off[OUTS];
                bool live[OUTS];
#pragma unroll
                for (int o = 0; o < OUTS; ++o) {
                    const int i = min(i0 + o * kThreads, a.M * COLS - 1);
                    const int m = i / COLS;
                    const int n = min(tile * COLS + (i - m * COLS), N - 1);
                    off[o] = (size_t)m * N + n;
                    live[o] = i0 + o * kThreads < a.M * COLS && tile * COLS + (i - m * COLS) < N;
                    s[o] = 0.f;
                }
                for (int sl0 = 0; sl0 < a.split_k; sl0 += 8) {
                    float v[OUTS][8];
#pragma unroll
                    for (int o = 0; o < OUTS; ++o)
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            const int sl = min(sl0 + j, a.split_k - 1);
                            v[o][j] = load_device_scope(a.partial + (size_t)sl * a.M * N + off[o]);
                        }
#pragma unroll
                    for (int o = 0; o < OUTS; ++o)
#pragma unroll
                        for (int j = 0; j < 8; ++j)
                            s[o] += (sl0 + j < a.split_k) ? v[o][j] : 0.f;
                }
#pragma unroll
                for (int o = 0; o < OUTS; ++o)
                    if (live[o])
                        a.out[off[o]] = (half_t)s[o];
            }
            };
            if (a.M * COLS <= kThreads)
                combine(std::integral_constant<int, 1>());
            else
                combine(std::integral_constant<int, 4>());
            if (tid == 0)
                __hip_atomic_store(a.counters + tile, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

}  // namespace skinny
}  // namespace gptq

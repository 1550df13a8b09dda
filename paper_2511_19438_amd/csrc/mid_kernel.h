// Mid-batch streaming MFMA kernel for the W4A16 GPTQ matrix multiply (32 < M <= 128 per launch), gfx950.
//
// Between the small-batch kernel (up to 32 rows: one or two 16-row MFMA operands per weight) and the big-tile
// kernel (hundreds of rows per tile) the weights still have to be streamed once at HBM speed, but every packed
// word now feeds enough MFMAs that instruction issue, not memory, sets the pace of a wavefront.  This kernel
// therefore makes each wavefront an independent stream processor with nothing shared and no workgroup barrier
// in its loop (Opt4GPTQ's three stages - vectorised loads, activations staged in on-chip memory, packed fp16
// arithmetic - per wavefront; Sections 3.1-3.3):
//   * a workgroup owns 32*NB columns and one K slice; its wavefronts split the slice, so every wavefront streams
//     its own rows of qweight: a lane loads NB adjacent packed words (a wavefront load covers two packed rows
//     of 128*NB contiguous bytes), which are NB B operands of v_mfma_f32_32x32x16_f16 (one word = eight
//     consecutive k of one column = one lane's operand), dequantised in registers to the exact fp16 weight;
//   * the activations of a 64-k stage (32*TMB rows x 128 bytes) go global -> LDS by DMA into a ring that belongs
//     to the wavefront alone: `s_waitcnt vmcnt(n)` is all the synchronisation the loop needs.  16-byte chunks are
//     XOR-swizzled by row so that the 32-row operand reads are free of bank conflicts;
//   * weights are prefetched two stages ahead in three register sets (the DMA of the next stage is issued
//     before them, so waiting for it does not wait for them), which covers the HBM latency with two wavefronts
//     per SIMD;
//   * partial sums meet in LDS (wavefronts, fixed order), then - if K is split across workgroups - in scratch,
//     where the last workgroup to arrive adds the slices in slice order (Section 3.1's reduction, without
//     floating point atomics).
// No g_idx; K and group_size multiples of 64.
#pragma once

#include "exchange.h"
#include "kernels.h"

#include <type_traits>

namespace gptq {
namespace mid {

constexpr int kStageK = 64;  // k per pipeline stage: 8 packed rows, 128 bytes of every activation row

struct Args {
    const half_t *x;
    const uint32_t *qweight;
    const uint32_t *qzeros;
    const half_t *scales;
    half_t *out;
    float *partial;      // [split_k, M, N] fp32, only if split_k > 1
    unsigned *counters;  // [tiles_n], zero between launches
    int M, K, N;
    // group of stage s = mulhi(s, group_mul) + s * group_one: group_mul = floor(2^32 / stages per group) + 1 and
    // group_one = 0, or (one stage per group) 0 and 1 - a division without a branch in the loop
    uint32_t group_mul;
    uint32_t group_one;
    int tiles_n;
    int split_k;
    int stages_per_slice;
    int total_stages;  // K / 64
};

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void lds_ptr_t;
typedef __attribute__((address_space(1))) const void global_ptr_t;

__device__ __forceinline__ half2_t as_half2(uint32_t v)
{
    return __builtin_bit_cast(half2_t, v);
}

// Nibble pair -> fp16 pair without an integer-to-float conversion: byte P of the word (q_2P | q_2P+1 << 4) is
// copied into both halves, one nibble kept in each and OR-ed into the mantissa of 1024.0 (0x6400, ulp 1) or
// 64.0 (0x5400, ulp 1/16); adding (-(1024 + z), -(64 + z)) leaves the exact integers q - z, one multiply by the
// scale rounds once.  Mask and bias live in registers so that mask-and-bias is one v_and_or_b32.
struct PairMagic {
    uint32_t mask, bias;
    __device__ __forceinline__ PairMagic()
    {
        mask = 0x00f0000fu;
        bias = 0x54006400u;
        asm volatile("" : "+s"(mask), "+v"(bias));
    }
};

template <int P>
__device__ __forceinline__ uint32_t dequant_pair(uint32_t w, const PairMagic &k, uint32_t nz, uint32_t ss)
{
    const uint32_t spread = __builtin_amdgcn_perm(0u, w, 0x0c000c00u | P | (P << 16));
    const half2_t v = (as_half2((spread & k.mask) | k.bias) + as_half2(nz)) * as_half2(ss);
    return __builtin_bit_cast(uint32_t, v);
}

__device__ __forceinline__ half8_t dequant_word(uint32_t w, const PairMagic &k, uint32_t nz, uint32_t ss)
{
    const u32x4_t r = {dequant_pair<0>(w, k, nz, ss), dequant_pair<1>(w, k, nz, ss), dequant_pair<2>(w, k, nz, ss),
                       dequant_pair<3>(w, k, nz, ss)};
    return __builtin_bit_cast(half8_t, r);
}

// The loop's loads into registers are written as inline assembly: address = wavefront-uniform base in scalar
// registers + one 32-bit byte offset per lane.  The compiler then knows of no load in flight and inserts
// no waits of its own (with the DMA in the loop its bookkeeping fell back to `vmcnt(0)` once per iteration, which
// drained the prefetch); the one `s_waitcnt vmcnt(n)` per stage below names the registers it makes valid as
// in/out operands, so nothing that uses them can be scheduled above it.
__device__ __forceinline__ void load_global(u32x4_t &dst, uint32_t byte_off, const void *base)
{
    asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(dst) : "v"(byte_off), "s"(base) : "memory");
}
__device__ __forceinline__ void load_global(u32x2_t &dst, uint32_t byte_off, const void *base)
{
    asm volatile("global_load_dwordx2 %0, %1, %2" : "=v"(dst) : "v"(byte_off), "s"(base) : "memory");
}
__device__ __forceinline__ void load_global(uint32_t &dst, uint32_t byte_off, const void *base)
{
    asm volatile("global_load_dword %0, %1, %2" : "=v"(dst) : "v"(byte_off), "s"(base) : "memory");
}
// A loop-invariant lane offset, made opaque at every use: the zero extension then stays next to the memory
// instruction, which lets the instruction selector use the scalar-base + 32-bit-offset addressing mode.
__device__ __forceinline__ uint32_t at_use(uint32_t v)
{
    asm volatile("" : "+v"(v));
    return v;
}

template <int NB>
struct WordVec {
    using type = u32x4_t;
};
template <>
struct WordVec<2> {
    using type = u32x2_t;
};
template <int NB>
struct ScaleVec {  // NB fp16 scales as raw bits
    using type = u32x2_t;
};
template <>
struct ScaleVec<2> {
    using type = uint32_t;
};

// Loads of one 64-k stage of one lane: four 16-k steps x NB adjacent words, the group's scales and zero word.
template <int NB>
struct StageRegs {
    typename WordVec<NB>::type w[4];
    typename ScaleVec<NB>::type sc;
    uint32_t zb;
};
__device__ __forceinline__ uint32_t scale_pair(const u32x2_t &sc, int t)
{
    return sc[t / 2];
}
__device__ __forceinline__ uint32_t scale_pair(const uint32_t &sc, int)
{
    return sc;
}

// TMB: 32-row blocks (M <= 32 * TMB).  NB: 32-column n-blocks per wavefront (2 or 4; n-block t <-> column
// NB * (lane % 32) + t of the tile).  WAVES: wavefronts per workgroup, each with its own share of the K slice.
template <int TMB, int NB, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void mid_kernel(const Args a)
{
    static_assert(NB == 2 || NB == 4, "64- or 128-bit weight loads");
    constexpr int kThreads = 64 * WAVES;
    constexpr int ROWS = 32 * TMB;
    constexpr int COLS = 32 * NB;
    constexpr int XBUF = ROWS * 128;  // bytes of one stage of activations
    constexpr int NX = ROWS / 8;      // DMA instructions per stage: 8 rows x 128 bytes each
    constexpr int NWL = 6;            // vector memory instructions of one stage of weights (4 + scales + zeros)
    constexpr int LW = 2 * XBUF;      // LDS bytes of one wavefront: a ring of two stages

    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int s_last;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 31;  // column group: columns NB*c .. NB*c + NB-1 of the tile; A operand: row c of a block
    const int h = lane >> 5;  // k half of a 16-k step
    const int tile = blockIdx.x % a.tiles_n;
    const int slice = blockIdx.x / a.tiles_n;
    const int N = a.N;
    const int n0 = tile * COLS + NB * c;
    const int nc = min(n0, N - NB);  // clamped for loads; columns past N are never stored

    const int s0 = slice * a.stages_per_slice;
    const int s1 = min(s0 + a.stages_per_slice, a.total_stages);
    const int per_wave = (s1 - s0 + WAVES - 1) / WAVES;
    const int ws0 = min(s0 + wave * per_wave, s1);
    const int ws1 = min(ws0 + per_wave, s1);
    // every wavefront runs `per_wave` stage bodies (three per loop iteration - the register sets rotate by
    // unrolling - and one or two after the loop); a body past the wavefront's own share loads its last stage
    // again and contributes zeros

    unsigned char *ring = smem + (size_t)wave * LW;

    // Addresses: wavefront-uniform base (scalar registers) + one 32-bit byte offset per lane.
    const uint32_t voff_w = ((uint32_t)h * N + nc) * 4u;
    const uint32_t voff_s = (uint32_t)nc * 2u;
    const uint32_t voff_z = (uint32_t)(nc >> 3) * 4u;
    const int zshift = (nc & 7) * 4;
    // DMA q of a stage: lane -> row 8q + lane/8, LDS chunk lane%8, which holds global chunk (lane%8) ^ ((row>>1)&7)
    uint32_t voff_x[NX];
#pragma unroll
    for (int q = 0; q < NX; ++q) {
        const int row = 8 * q + (lane >> 3);
        const int chunk = (lane & 7) ^ ((row >> 1) & 7);
        voff_x[q] = ((uint32_t)min(row, a.M - 1) * a.K + chunk * 8) * 2u;
    }
    // A operand of step s, block i: row 32i + c, global chunk 2s + h -> LDS chunk (2s + h) ^ ((c>>1)&7)
    const uint32_t aoff = (uint32_t)c * 128u + ((uint32_t)(h ^ ((c >> 1) & 7)) << 4);

    auto issue_x = [&](int st, int buf) {
        const int sc = min(st, s1 - 1);
        const char *xb = reinterpret_cast<const char *>(a.x + (size_t)sc * kStageK);
#pragma unroll
        for (int q = 0; q < NX; ++q)
            __builtin_amdgcn_global_load_lds((global_ptr_t *)(xb + at_use(voff_x[q])),
                                             (lds_ptr_t *)(ring + (size_t)buf * XBUF + q * 1024), 16, 0, 0);
    };
    auto issue_w = [&](int st, StageRegs<NB> &r) {
        const int sc = min(st, s1 - 1);
        const uint32_t *wrow = a.qweight + (size_t)sc * 8 * N;
#pragma unroll
        for (int s = 0; s < 4; ++s)
            load_global(r.w[s], voff_w, wrow + (size_t)(2 * s) * N);
        const uint32_t grp = __umulhi((uint32_t)sc, a.group_mul) + (uint32_t)sc * a.group_one;
        load_global(r.sc, voff_s, a.scales + (size_t)grp * N);
        load_global(r.zb, voff_z, a.qzeros + (size_t)grp * (N >> 3));
    };
    // the stage's loads have arrived: `outstanding` vector memory instructions were issued after them
    auto arrived = [&](StageRegs<NB> &r, auto outstanding) {
        asm volatile("s_waitcnt vmcnt(%6)"
                     : "+v"(r.w[0]), "+v"(r.w[1]), "+v"(r.w[2]), "+v"(r.w[3]), "+v"(r.sc), "+v"(r.zb)
                     : "n"(decltype(outstanding)::value)
                     : "memory");
    };

    float16_t acc[TMB][NB];
#pragma unroll
    for (int i = 0; i < TMB; ++i)
#pragma unroll
        for (int t = 0; t < NB; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[i][t][r] = 0.f;

    const PairMagic magic;

    // One stage: 64 k of this lane's NB columns against all batch rows.
    auto consume = [&](int st, const StageRegs<NB> &r, int buf) {
        const bool live = st < ws1;
        uint32_t nz[NB], ss[NB];
#pragma unroll
        for (int t = 0; t < NB; ++t) {
            const uint32_t z = (r.zb >> (zshift + 4 * t)) & 15u;
            nz[t] = 0xD400E400u | z | (z << 20);  // (-(1024 + z), -(64 + z))
            const uint32_t pair = scale_pair(r.sc, t);
            const uint32_t sb = (t & 1) ? (pair >> 16) : (pair & 0xffffu);
            ss[t] = live ? (sb | (sb << 16)) : 0u;
        }
        const unsigned char *xs = ring + (size_t)buf * XBUF;
        // The A operands of a step are read from LDS while the MFMAs of the step before run (two register sets):
        // issued right before their use, the read's latency stalled the wavefront once per step.
        half8_t av[2][TMB];
        auto read_a = [&](int s, half8_t (&dst)[TMB]) {
#pragma unroll
            for (int i = 0; i < TMB; ++i)
                dst[i] = *reinterpret_cast<const half8_t *>(xs + (aoff ^ (uint32_t)(s << 5)) + i * 4096);
        };
        read_a(0, av[0]);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            if (s + 1 < 4) {
                read_a(s + 1, av[(s + 1) & 1]);
                __builtin_amdgcn_sched_barrier(0);  // (keeps the reads above the arithmetic below)
            }
#pragma unroll
            for (int t = 0; t < NB; ++t) {
                const half8_t b = dequant_word(r.w[s][t], magic, nz[t], ss[t]);  // (vector element t)
#pragma unroll
                for (int i = 0; i < TMB; ++i)
                    acc[i][t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av[s & 1][i], b, acc[i][t], 0, 0, 0);
            }
        }
    };

    // ---- the loop: x(i+1) and w(i+2) are issued, in that order, before stage i is consumed.  The vector memory
    //      counter retires in order, so waiting until only NX + 2*NWL instructions are outstanding leaves exactly
    //      w(i+1), x(i+1), w(i+2) in flight: x(i) and w(i) have arrived.  Compiler barriers keep the issue order. ----
    StageRegs<NB> r0, r1, r2;
    auto body = [&](int st, StageRegs<NB> &cur, StageRegs<NB> &nxt2, int buf) {
        issue_x(st + 1, buf ^ 1);
        asm volatile("" ::: "memory");
        issue_w(st + 2, nxt2);
        arrived(cur, std::integral_constant<int, NX + 2 * NWL>());
        consume(st, cur, buf);
        // the next body's DMA overwrites the buffer this one has just read: the reads are complete (their values
        // fed the MFMAs above), this keeps the compiler from moving them
        asm volatile("" ::: "memory");
    };
    issue_w(ws0, r0);
    asm volatile("" ::: "memory");
    issue_x(ws0, 0);
    asm volatile("" ::: "memory");
    issue_w(ws0 + 1, r1);
    asm volatile("" ::: "memory");
    {
        int st = ws0;
        int buf = 0;
        for (int b = 3; b <= per_wave; b += 3) {
            body(st, r0, r2, buf);
            body(st + 1, r1, r0, buf ^ 1);
            body(st + 2, r2, r1, buf);
            st += 3;
            buf ^= 1;
        }
        const int rest = per_wave % 3;  // the same for every wavefront of the grid
        if (rest >= 1)
            body(st, r0, r2, buf);
        if (rest == 2)
            body(st + 1, r1, r0, buf ^ 1);
    }

    // ---- wavefronts meet in LDS (the rings are reused: every DMA has landed first), fixed order ----
    // The last bodies prefetched stages that nobody consumes: their registers stay reserved until those loads
    // have landed (naming them here keeps the compiler from handing them to the code below while a load that
    // it cannot see is still on its way).
    arrived(r0, std::integral_constant<int, 0>());
    arrived(r1, std::integral_constant<int, 0>());
    arrived(r2, std::integral_constant<int, 0>());
    __syncthreads();
    float *red = reinterpret_cast<float *>(smem);
    constexpr int AT = ROWS * COLS;  // floats of one wavefront's tile
    // lane (c, h) holds, for block i, n-block t, register r: row 32i + 8(r/4) + 4h + r%4, column NB*c + t
    auto tile_slot = [&](int slot, int i, int r) -> float * {
        const int row = 32 * i + 8 * (r >> 2) + 4 * h + (r & 3);
        return red + (size_t)slot * AT + (size_t)row * COLS + NB * c;
    };
    auto write_tile = [&](int slot) {
#pragma unroll
        for (int i = 0; i < TMB; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float *p = tile_slot(slot, i, r);
                if (NB == 4) {
                    const float4_t v = {acc[i][0][r], acc[i][1][r], acc[i][2 % NB][r], acc[i][3 % NB][r]};
                    *reinterpret_cast<float4_t *>(p) = v;
                } else {
                    const f32x2_t v = {acc[i][0][r], acc[i][1][r]};
                    *reinterpret_cast<f32x2_t *>(p) = v;
                }
            }
    };
    auto add_tile = [&](int slot) {
#pragma unroll
        for (int i = 0; i < TMB; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float *p = tile_slot(slot, i, r);
#pragma unroll
                for (int t = 0; t < NB; ++t)
                    acc[i][t][r] += p[t];
            }
    };
    // A wavefront's tile may be twice its share of the LDS: then the upper half of the wavefronts hand their
    // tiles to the lower half first.
    constexpr bool HALVE = AT * 4 > LW;
    static_assert(AT * 4 <= 2 * LW, "a tile fits two wavefronts' rings");
    constexpr int NBUF = HALVE ? WAVES / 2 : WAVES;
    if (HALVE) {
        if (wave >= NBUF)
            write_tile(wave - NBUF);
        __syncthreads();
        if (wave < NBUF)
            add_tile(wave);
        __syncthreads();
    }
    if (wave < NBUF)
        write_tile(wave);
    __syncthreads();
    constexpr int QUADS = COLS / 4;
    for (int e = tid; e < ROWS * QUADS; e += kThreads) {
        const int row = e / QUADS;
        const int col = (e - row * QUADS) * 4;
        const int n = tile * COLS + col;
        float4_t s = *reinterpret_cast<const float4_t *>(red + (size_t)row * COLS + col);
#pragma unroll
        for (int w = 1; w < NBUF; ++w)
            s += *reinterpret_cast<const float4_t *>(red + (size_t)w * AT + (size_t)row * COLS + col);
        if (row < a.M && n < N) {
            if (a.split_k == 1) {
                const half4_t v = {(half_t)s[0], (half_t)s[1], (half_t)s[2], (half_t)s[3]};
                *reinterpret_cast<half4_t *>(a.out + (size_t)row * N + n) = v;
            } else {
                unsigned long long *dst =
                    reinterpret_cast<unsigned long long *>(a.partial + ((size_t)slice * a.M + row) * N + n);
                const f32x2_t lo = {s[0], s[1]}, hi = {s[2], s[3]};
                __hip_atomic_store(dst, __builtin_bit_cast(unsigned long long, lo), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(dst + 1, __builtin_bit_cast(unsigned long long, hi), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }

    // ---- K slices across workgroups: the last one of this column tile to arrive adds them in slice order ----
    if (a.split_k > 1) {
        __builtin_amdgcn_s_waitcnt(0);  // every partial store of this workgroup has been acknowledged (exchange.h)
        __syncthreads();
        if (tid == 0)
            s_last = (slice_arrive(a.counters + tile) == (unsigned)(a.split_k - 1));
        __syncthreads();
        if (s_last) {
            slice_acquire();
            // all slices of two column pairs are requested before the first is used; additions in slice order
            for (int e0 = tid; e0 < a.M * QUADS; e0 += kThreads) {
                const int row = e0 / QUADS;
                const int col = (e0 - row * QUADS) * 4;
                const int n = tile * COLS + col;
                if (n >= N)
                    continue;
                const size_t off = (size_t)row * N + n;
                float4_t s = {0.f, 0.f, 0.f, 0.f};
                for (int sl0 = 0; sl0 < a.split_k; sl0 += 8) {
                    unsigned long long v[8][2];
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const int sl = min(sl0 + j, a.split_k - 1);
                        const unsigned long long *src =
                            reinterpret_cast<const unsigned long long *>(a.partial + (size_t)sl * a.M * N + off);
                        v[j][0] = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        v[j][1] = __hip_atomic_load(src + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const float keep = sl0 + j < a.split_k ? 1.f : 0.f;
                        const f32x2_t lo = __builtin_bit_cast(f32x2_t, v[j][0]);
                        const f32x2_t hi = __builtin_bit_cast(f32x2_t, v[j][1]);
                        s[0] += keep * lo[0];
                        s[1] += keep * lo[1];
                        s[2] += keep * hi[0];
                        s[3] += keep * hi[1];
                    }
                }
                const half4_t o = {(half_t)s[0], (half_t)s[1], (half_t)s[2], (half_t)s[3]};
                *reinterpret_cast<half4_t *>(a.out + off) = o;
            }
            if (tid == 0)
                __hip_atomic_store(a.counters + tile, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

}  // namespace mid
}  // namespace gptq

// Split-K vector kernel for the W4A16 GPTQ matrix multiply at small batch (M <= 16), gfx950.
//
// The paper's kernel pipeline (Opt4GPTQ, Section 3) has three stages, all of which exist here
// in a form that suits CDNA4:
//   * activations are staged in on-chip memory with wide loads (Section 3.2; here 128-bit loads,
//     and the eight values of a packed row are stored in the order the dequantised pairs need);
//   * the inner loop is packed half arithmetic (Section 3.3, Eq. 14-15): two weights per VGPR are
//     formed with one v_and_or_b32 and contracted with v_dot2_f32_f16 into fp32 accumulators; zero
//     point and scale are applied per chunk (small batches) or per element with packed fp16 ops;
//   * partial sums are reduced on chip before anything is committed (Section 3.1, Eq. 6-10):
//     across lanes with wavefront shuffles, across wavefronts through LDS, and across the K slices
//     of different workgroups through fp32 partials in scratch that the last workgroup to arrive
//     adds in slice order.  No floating point atomics: the result is deterministic.  The scratch
//     is written and read with device-scope accesses and an arrival counter, not with device-wide
//     fences: a fence writes back and invalidates a whole L2 and costs microseconds per workgroup.
//
// Work decomposition.  A workgroup (4 wavefronts) owns CT = 4*LPR adjacent columns and one slice
// of K.  A lane owns 4 adjacent columns (one 128-bit load of a packed qweight row = 4 x 8 weights)
// and, together with the other lanes of the same column quad ("row lanes", 64/LPR per wavefront,
// 4x that per workgroup), strides over the slice in chunks of R packed rows.  With LPR = 16 a
// wavefront load touches 4 rows x 256 contiguous bytes.
#pragma once

#include <type_traits>

#include "exchange.h"
#include "kernels.h"

namespace gptq {
namespace decode {

struct Args {
    const half_t *x;
    const uint32_t *qweight;
    const uint32_t *qzeros;
    const half_t *scales;
    const int32_t *g_idx;
    const int32_t *x_perm;  // [K] source position of each activation element (kGatherX), else unused
    half_t *out;
    float *partial;       // [split_k, M, N] fp32, only if split_k > 1
    unsigned *counters;   // [tiles_n], zero between launches
    int M, K, N;
    int rows;             // K / 8 packed rows
    int rows_per_group;   // group_size / 8
    int chunk_group_shift;  // log2(chunks per group) if that is a power of two, else -1
    int groups;           // K / group_size
    int tiles_n;
    int split_k;
    int chunks_per_slice;
    int total_chunks;     // ceil(rows / R)
};

__device__ __forceinline__ half2_t as_half2(uint32_t v)
{
    return __builtin_bit_cast(half2_t, v);
}

__device__ __forceinline__ uint32_t as_u32(half2_t v)
{
    return __builtin_bit_cast(uint32_t, v);
}

// acc + a.x*b.x + a.y*b.y with fp32 accumulation (v_dot2_f32_f16)
__device__ __forceinline__ float dot2(half2_t a, half2_t b, float acc)
{
    return __builtin_amdgcn_fdot2(a, b, acc, false);
}

// Bit patterns used to turn 4-bit codes into fp16 values without any integer-to-float conversion:
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

// The eight codes of one packed word as four half2 that still carry their bias:
//   b[0] = (1024 + q0, 1024 + q4), b[1] = (64 + q1, 64 + q5), b[2] = (1024 + q2, 1024 + q6), b[3] = (64 + q3, 64 + q7).
__device__ __forceinline__ void biased_codes(uint32_t w, const NibbleMagic &k, half2_t b[4])
{
    const uint32_t w8 = w >> 8;
    b[0] = as_half2((w & k.mask_lo) | k.bias_lo);
    b[1] = as_half2((w & k.mask_hi) | k.bias_hi);
    b[2] = as_half2((w8 & k.mask_lo) | k.bias_lo);
    b[3] = as_half2((w8 & k.mask_hi) | k.bias_hi);
}

// Same, with the bias and the zero point taken off: exact small integers q - z.
// neg_lo = (-(1024 + z)) x2 and neg_hi = (-(64 + z)) x2; both sums are exact in fp16.
__device__ __forceinline__ void codes_minus_zero(uint32_t w, const NibbleMagic &k, half2_t neg_lo, half2_t neg_hi,
                                                 half2_t d[4])
{
    biased_codes(w, k, d);
    d[0] += neg_lo;
    d[1] += neg_hi;
    d[2] += neg_lo;
    d[3] += neg_hi;
}

// Global loads of one step of one lane: UNROLL chunks of R packed rows, plus their scale / zero words.
template <int R, int UNROLL>
struct StepRegs {
    uint4 wq[UNROLL][R];
    half4_t sc[UNROLL];
    uint32_t zb[UNROLL];
};

// Scratch traffic between workgroups goes through device-scope (sc1) accesses that are coherent
// across the XCDs' L2 caches by themselves, so no cache write-back / invalidate fence is needed.
__device__ __forceinline__ void store_device_scope(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_device_scope(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Ablation switches (template parameter ABL, a bit set; 0 = the kernel as designed).  Each bit takes one of
// the paper's three techniques out and puts the baseline it describes in its place, so that the gain of the
// technique on this chip can be measured in isolation (Table 3 has the same columns end to end):
//   kNoSmb: no on-chip hierarchical reduction (Section 3.1) - every lane commits its partial sums straight to
//           global memory with floating point atomics (Eq. 9-10 at thread level); the sums need a zeroed fp32
//           buffer and a conversion by the last workgroup of the column tile;
//   kNoVml: activations are staged with one 16-bit load per element instead of 128-bit loads (Section 3.2);
//   kNoIla: every weight is converted to fp32 on its own and multiplied-added with scalar fp32 instructions
//           instead of packed half conversion and v_dot2_f32_f16 (Section 3.3).
constexpr int kNoSmb = 1, kNoVml = 2, kNoIla = 4;
// Not an ablation but a variant of the inner loop, selected with the same parameter: the contraction of the
// biased codes with the activations goes to the matrix unit (v_mfma_f32_4x4x4_16B_f16: sixteen independent
// 4x4x4 products per instruction; in each, lane 4b+j supplies row j of A = batch row j and column l of B =
// this lane's own column, and receives that column of the result) instead of four v_dot2_f32_f16 per packed
// word: two MFMAs per word that run beside the vector ALU, which is left with the five code-forming
// operations.  Up to four batch rows ride along for free.
constexpr int kMatrixDot = 8;
// Another variant: the activations are gathered through Args::x_perm while they are staged (the weight's rows
// were sorted by group once, so that it reads like the plain format; the activations follow them per call).
constexpr int kGatherX = 16;
// Eight wavefronts per workgroup (two per SIMD) instead of four, for the single-row kernel of the plain format
// where every workgroup has a compute unit to itself: a wavefront issues one instruction every few cycles
// whatever its kind, and with a second one on the SIMD the loads, LDS reads, matrix-unit and scalar
// instructions of one overlap the vector arithmetic of the other (measured 3-8 % on the Llama GEMVs; sixteen
// were twice as slow, and with more workgroups than compute units eight are 2-5 % slower than four).
constexpr int kEightWaves = 32;
// The bias / zero-point correction of the factored arithmetic once per quantisation group (128 k = four chunks)
// instead of once per 32-k chunk: a lane then walks the four chunks of ONE group in two consecutive pipeline steps
// (chunks 4g .. 4g+3, two per step), keeps the matrix-unit sums running across them and corrects with the
// group's activation sums - the conversions of the four zero points and scales and the two fused multiply-adds
// per column are paid once per 64 packed words instead of once per 16.  Single row, plain format, group sizes
// that are multiples of 128, slices of whole groups.
constexpr int kGroupCorr = 64;

template <int MB, int LPR, int R, bool ACT, int ABL = 0>
__global__ __launch_bounds__((ABL & kEightWaves) ? 512 : 256) void decode_kernel(const Args a)
{
    static_assert(ABL == 0 || (!ACT && MB < 8), "the ablation variants exist for the plain format at small batch");
    static_assert(!(ABL & kMatrixDot) || MB <= 4, "the 4x4x4 matrix product carries four batch rows");
    static_assert(!(ABL & kEightWaves) || (MB == 1 && !ACT), "eight wavefronts: single row, plain format");
    constexpr bool GC = (ABL & kGroupCorr) != 0;
    static_assert(!GC || (MB == 1 && !ACT && R == 4 && (ABL & kMatrixDot) && !(ABL & 7)),
                  "group-level correction: single row, plain format, matrix-unit loop");
    constexpr int kWaves = (ABL & kEightWaves) ? 8 : 4;
    constexpr int kThreads = 64 * kWaves;
    constexpr int RL = 64 / LPR;          // row lanes per wavefront
    constexpr int RW = kWaves * RL;       // row lanes per workgroup
    constexpr int CT = LPR * 4;           // columns per workgroup
    constexpr int MC = MB < 4 ? MB : 4;   // batch rows per cross-wavefront reduction round
    // Two ways to apply zero point and scale.  FACTORED (small batches, memory bound): contract the
    // biased codes directly, sum_k x_k (bias_k + q_k), and correct once per chunk with sums of x
    // that were prepared while staging:  sum_k x_k (q_k - z) = D - sum_k bias_k x_k - z sum_k x_k,
    // then scale the chunk sum.  Otherwise (act-order or large batches): form the fp16 weight
    // s * (q - z) per element and contract it.
    constexpr bool FACTORED = !ACT && MB < 8;
    constexpr int UNROLL = ACT ? 1 : 2;   // chunks in flight per lane and step (act-order needs the registers)
    constexpr int STEP = RW * UNROLL;     // chunks a workgroup consumes per step

    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int s_last;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int cq = lane % LPR;
    const int rl = lane / LPR;
    const int rid = wave * RL + rl;
    const int tile = blockIdx.x % a.tiles_n;
    const int slice = blockIdx.x / a.tiles_n;
    const int n0 = tile * CT + cq * 4;
    const int N = a.N;

    const int c0 = slice * a.chunks_per_slice;
    const int c1 = min(c0 + a.chunks_per_slice, a.total_chunks);
    const int nchunks = c1 - c0;
    const int kbeg = c0 * R * 8;
    const int kend = min(c1 * R * 8, a.K);
    const int Ls = kend - kbeg;  // activations of this slice, per batch row (multiple of 8)

    // ---- LDS carve-up ----
    half_t *xs = reinterpret_cast<half_t *>(smem);                      // [MB][Ls], pair-permuted
    size_t off = ((size_t)MB * Ls * sizeof(half_t) + 15) & ~(size_t)15;
    float2 *xc = reinterpret_cast<float2 *>(smem + off);                // FACTORED: [MB][nchunks] (sum bias*x, sum x)
    off += FACTORED ? (((size_t)MB * nchunks * sizeof(float2) + 15) & ~(size_t)15) : 0;
    float *red = reinterpret_cast<float *>(smem + off);                 // [kWaves][MC][CT]
    off += (size_t)kWaves * MC * CT * sizeof(float);
    int *gl = reinterpret_cast<int *>(smem + off);                      // ACT: [Ls] group of each k
    uint32_t *tab = reinterpret_cast<uint32_t *>(smem + off + (ACT ? (size_t)Ls * sizeof(int) : 0));  // ACT: [groups][CT]

    // Every load below is made unconditional by clamping its chunk / column to the last valid one of the
    // slice; what a clamped (out-of-range) chunk contributes is zeroed when it is used.  No branch sits
    // between a load and its use, so the waits the compiler inserts count exactly the loads that were
    // issued later and the prefetched step stays in flight.
    //
    // Addresses are a wavefront-uniform base (scalar registers) plus a 32-bit byte offset per lane, so a
    // load costs no 64-bit vector arithmetic: the R packed rows of a chunk differ only in the base.
    const int n0c = min(n0, N - 4);
    const uint32_t *wslice = a.qweight + (size_t)c0 * R * N;  // first packed row of the slice
    // slice-relative chunk of this lane in step t (GC: the four chunks of group (t / 2) * RW + rid over two steps)
    auto lane_chunk = [&](int t, int j) {
        return GC ? 4 * ((t >> 1) * RW + rid) + 2 * (t & 1) + j : t * STEP + j * RW + rid;
    };
    using Regs = StepRegs<R, UNROLL>;
    auto issue = [&](int t, Regs &r, auto odd_tag) {
        constexpr bool ODD = decltype(odd_tag)::value;  // GC: the group's scales and zeros travel with the even step
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) {
            const int ul = min(lane_chunk(t, j), nchunks - 1);
            const uint32_t woff = (__umul24(ul * R, N) + n0c) * 4u;
#pragma unroll
            for (int rr = 0; rr < R; ++rr)
                r.wq[j][rr] = *reinterpret_cast<const uint4 *>(
                    reinterpret_cast<const char *>(wslice + (size_t)rr * N) + woff);
            if (!ACT && !(GC && (ODD || j > 0))) {
                const int u = c0 + ul;
                const int grp = a.chunk_group_shift >= 0 ? (u >> a.chunk_group_shift) : (u * R) / a.rows_per_group;
                r.sc[j] = *reinterpret_cast<const half4_t *>(reinterpret_cast<const char *>(a.scales) +
                                                             (__umul24(grp, N) + n0c) * 2u);
                // the shift that isolates this lane's zero points is applied when the word is used: no wait here
                r.zb[j] = *reinterpret_cast<const uint32_t *>(reinterpret_cast<const char *>(a.qzeros) +
                                                              (__umul24(grp, N >> 3) + (n0c >> 3)) * 4u);
            }
        }
    };

    const int zshift = (n0c & 4) * 4;  // this lane's four zero points inside the packed word

    // ---- stage the activations of this slice: one packed row (eight values, one 128-bit load) per thread
    //      and turn, stored in the order (0,4,1,5,2,6,3,7) that the dequantised pairs need.  The first
    //      turn's load goes out before the weights' and is waited for alone. ----
    const int rows_s = Ls >> 3;            // packed rows of the slice
    const int rows_p = nchunks * R;        // the same, padded to whole chunks
    const int items = MB * rows_p;
    auto x_load = [&](int i) -> half8_t {
        const int m = MB == 1 ? 0 : i / rows_p;
        const int row = i - m * rows_p;
        if (ABL & kGatherX) {  // the activations of a row-sorted weight: element k comes from position x_perm[k]
            const int32_t *ps = a.x_perm + kbeg + min(row, rows_s - 1) * 8;
            const int4 pa = *reinterpret_cast<const int4 *>(ps);
            const int4 pb = *reinterpret_cast<const int4 *>(ps + 4);
            const half_t *xr = a.x + (size_t)min(m, a.M - 1) * a.K;
            const unsigned last = (unsigned)a.K - 1u;  // a position outside the row reads its last element
            return half8_t{xr[min((unsigned)pa.x, last)], xr[min((unsigned)pa.y, last)],
                           xr[min((unsigned)pa.z, last)], xr[min((unsigned)pa.w, last)],
                           xr[min((unsigned)pb.x, last)], xr[min((unsigned)pb.y, last)],
                           xr[min((unsigned)pb.z, last)], xr[min((unsigned)pb.w, last)]};
        }
        const half_t *src = a.x + (size_t)min(m, a.M - 1) * a.K + kbeg + min(row, rows_s - 1) * 8;
        if (ABL & kNoVml) {  // eight separate 16-bit loads (volatile: not to be merged)
            const volatile half_t *v = src;
            return half8_t{v[0], v[1], v[2], v[3], v[4], v[5], v[6], v[7]};
        }
        return *reinterpret_cast<const half8_t *>(src);
    };
    auto x_store = [&](int i, half8_t h) {
        const int m = MB == 1 ? 0 : i / rows_p;
        const int row = i - m * rows_p;
        const bool real = i < items && row < rows_s && m < a.M;
        if (!real)
            h = half8_t{0, 0, 0, 0, 0, 0, 0, 0};
        if (i < items && row < rows_s) {
            half8_t p = {h[0], h[4], h[1], h[5], h[2], h[6], h[3], h[7]};
            *reinterpret_cast<half8_t *>(xs + (size_t)m * Ls + row * 8) = p;
        }
        if (FACTORED) {
            // sums of x over the k that get bias 1024 / bias 64, added over the R rows of the chunk
            float s_lo = ((float)h[0] + (float)h[4]) + ((float)h[2] + (float)h[6]);
            float s_hi = ((float)h[1] + (float)h[5]) + ((float)h[3] + (float)h[7]);
            constexpr int SUMROWS = GC ? 16 : R;  // packed rows whose sums travel together: a chunk, or a group
#pragma unroll
            for (int o = 1; o < SUMROWS; o <<= 1) {
                s_lo += __shfl_xor(s_lo, o, 64);
                s_hi += __shfl_xor(s_hi, o, 64);
            }
            if (i < items && (row & (SUMROWS - 1)) == 0)
                xc[(size_t)m * nchunks + row / SUMROWS] = make_float2(1024.f * s_lo + 64.f * s_hi, s_lo + s_hi);
        }
    };

    const std::integral_constant<bool, false> even_step;
    const std::integral_constant<bool, true> odd_step;
    Regs ra, rb;
    {
        const half8_t h0 = x_load(tid);
        issue(0, ra, even_step);  // the weights are in flight while the activations are staged
        x_store(tid, h0);
        for (int i0 = kThreads; i0 < items; i0 += kThreads)
            x_store(i0 + tid, x_load(i0 + tid));
        if (ACT) {
            for (int i = tid; i < Ls; i += kThreads)
                gl[i] = a.g_idx[kbeg + i];
            // per (group, column) of this tile: low half = scale bits, high half = -(1024 + z) as fp16 bits
            for (int i = tid; i < a.groups * CT; i += kThreads) {
                const int g = i / CT;
                const int n = tile * CT + (i - g * CT);
                uint32_t e = 0;
                if (n < N) {
                    const uint32_t sbits = __builtin_bit_cast(uint16_t, a.scales[(size_t)g * N + n]);
                    const uint32_t z = (a.qzeros[(size_t)g * (N >> 3) + (n >> 3)] >> (4 * (n & 7))) & 15u;
                    e = sbits | ((0xE400u | z) << 16);
                }
                tab[i] = e;
            }
        }
    }
    __syncthreads();

    float acc[MB][4];
#pragma unroll
    for (int m = 0; m < MB; ++m)
#pragma unroll
        for (int c = 0; c < 4; ++c)
            acc[m][c] = 0.f;

    const NibbleMagic magic;

    // dequantise and contract the chunks held in `r`
    float4_t gdot[4];   // GC: the matrix-unit sums of the group being walked
    float gzf[4], gsf[4];  // GC: its zero points and scales
    auto consume = [&](int t, const Regs &r, auto odd_tag) {
        constexpr bool ODD = decltype(odd_tag)::value;
        if constexpr (GC) {
            const int gi = (t >> 1) * RW + rid;          // slice-relative group of this lane
            const bool valid = gi < (nchunks >> 2);
            if (!ODD) {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    gdot[c] = float4_t{0.f, 0.f, 0.f, 0.f};
                    gzf[c] = (float)((r.zb[0] >> (zshift + 4 * c)) & 15u);
                    gsf[c] = valid ? (float)r.sc[0][c] : 0.f;  // a clamped group contributes nothing
                }
            }
#pragma unroll
            for (int j = 0; j < UNROLL; ++j) {
                const int ul = min(lane_chunk(t, j), nchunks - 1);
                const half_t *xchunk = xs + ul * (R * 8);
#pragma unroll
                for (int rr = 0; rr < R; ++rr) {
                    const uint32_t w[4] = {r.wq[j][rr].x, r.wq[j][rr].y, r.wq[j][rr].z, r.wq[j][rr].w};
                    const uint4 xv = *reinterpret_cast<const uint4 *>(xchunk + rr * 8);
                    const half4_t a01 = __builtin_bit_cast(half4_t, make_uint2(xv.x, xv.y));
                    const half4_t a23 = __builtin_bit_cast(half4_t, make_uint2(xv.z, xv.w));
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        half2_t d[4];
                        biased_codes(w[c], magic, d);
                        const half4_t b01 = __builtin_bit_cast(half4_t, make_uint2(as_u32(d[0]), as_u32(d[1])));
                        const half4_t b23 = __builtin_bit_cast(half4_t, make_uint2(as_u32(d[2]), as_u32(d[3])));
                        gdot[c] = __builtin_amdgcn_mfma_f32_4x4x4f16(a01, b01, gdot[c], 0, 0, 0);
                        gdot[c] = __builtin_amdgcn_mfma_f32_4x4x4f16(a23, b23, gdot[c], 0, 0, 0);
                    }
                }
            }
            if (ODD) {
                const float2 bs = xc[min(gi, (nchunks >> 2) - 1)];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const float tt = __builtin_fmaf(-gzf[c], bs.y, gdot[c][0] - bs.x);  // sum_k x_k (q_k - z)
                    acc[0][c] = __builtin_fmaf(gsf[c], tt, acc[0][c]);
                }
            }
            return;
        }
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) {
            const bool valid = lane_chunk(t, j) < nchunks;
            const int ul = min(lane_chunk(t, j), nchunks - 1);
            const half_t *xchunk = xs + ul * (R * 8);  // this chunk's activations; batch row m at + m * Ls
            half2_t neg_lo[4], neg_hi[4], s2[4];
            float sf[4], zf[4];
            float gacc[MB][4];
            if (!ACT) {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const uint32_t z = (r.zb[j] >> (zshift + 4 * c)) & 15u;
                    const half_t s = valid ? r.sc[j][c] : (half_t)0;  // a clamped chunk contributes nothing
                    if (FACTORED) {
                        zf[c] = (float)z;
                        sf[c] = (float)s;
                    } else {
                        neg_lo[c] = as_half2(0xE400E400u | (z * 0x00010001u));
                        neg_hi[c] = as_half2(0xD400D400u | (z * 0x00100010u));
                        s2[c] = half2_t{s, s};
                    }
                }
                if (FACTORED) {
#pragma unroll
                    for (int m = 0; m < MB; ++m)
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            gacc[m][c] = 0.f;
                }
            }
            float4_t mdot[4];  // kMatrixDot: per column, the chunk's sums for batch rows 0..3
#pragma unroll
            for (int c = 0; c < 4; ++c)
                mdot[c] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int rr = 0; rr < R; ++rr) {
                const uint32_t w[4] = {r.wq[j][rr].x, r.wq[j][rr].y, r.wq[j][rr].z, r.wq[j][rr].w};
                half2_t d[4][4];
                if ((ABL & kMatrixDot) && !(ABL & kNoIla)) {
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        biased_codes(w[c], magic, d[c]);
                    // A operand: the activations of batch row lane % 4 (rows past MB - 1 repeat it: their results
                    // are not used), already in the codes' k order (0,4,1,5 | 2,6,3,7)
                    const int arow = min(lane & 3, MB - 1);
                    const uint4 xv = *reinterpret_cast<const uint4 *>(xchunk + arow * Ls + rr * 8);
                    const half4_t a01 = __builtin_bit_cast(half4_t, make_uint2(xv.x, xv.y));
                    const half4_t a23 = __builtin_bit_cast(half4_t, make_uint2(xv.z, xv.w));
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const half4_t b01 = __builtin_bit_cast(half4_t, make_uint2(as_u32(d[c][0]), as_u32(d[c][1])));
                        const half4_t b23 = __builtin_bit_cast(half4_t, make_uint2(as_u32(d[c][2]), as_u32(d[c][3])));
                        mdot[c] = __builtin_amdgcn_mfma_f32_4x4x4f16(a01, b01, mdot[c], 0, 0, 0);
                        mdot[c] = __builtin_amdgcn_mfma_f32_4x4x4f16(a23, b23, mdot[c], 0, 0, 0);
                    }
                    continue;
                }
                if (ABL & kNoIla) {
                    // baseline arithmetic: per weight a bit-field extract, an integer-to-float conversion, the
                    // zero point and the scale in fp32, one fp32 multiply-add per batch row
#pragma unroll
                    for (int m = 0; m < MB; ++m) {
                        const uint4 xv = *reinterpret_cast<const uint4 *>(xchunk + m * Ls + rr * 8);
                        const uint32_t xw[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            // activation k = i of the packed row sits at position 2*i (i < 4) or 2*(i-4)+1
                            const int pos = i < 4 ? 2 * i : 2 * (i - 4) + 1;
                            const uint16_t hb = (uint16_t)(xw[pos >> 1] >> (16 * (pos & 1)));
                            const float xf = (float)__builtin_bit_cast(half_t, hb);
#pragma unroll
                            for (int c = 0; c < 4; ++c) {
                                const float qf = (float)((w[c] >> (4 * i)) & 15u);
                                acc[m][c] = __builtin_fmaf(xf, (qf - zf[c]) * sf[c], acc[m][c]);
                            }
                        }
                    }
                    continue;
                }
                if (FACTORED) {
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        biased_codes(w[c], magic, d[c]);
                } else if (!ACT) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        codes_minus_zero(w[c], magic, neg_lo[c], neg_hi[c], d[c]);
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            d[c][i] = d[c][i] * s2[c];
                    }
                } else {
                    // every k of the packed row may belong to a different group
                    const int4 ga = *reinterpret_cast<const int4 *>(gl + (ul * R + rr) * 8);
                    const int4 gb = *reinterpret_cast<const int4 *>(gl + (ul * R + rr) * 8 + 4);
                    const int g[8] = {ga.x, ga.y, ga.z, ga.w, gb.x, gb.y, gb.z, gb.w};
                    uint4 t[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        t[e] = *reinterpret_cast<const uint4 *>(tab + (size_t)g[e] * CT + cq * 4);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint32_t ta[4] = {t[i].x, t[i].y, t[i].z, t[i].w};                  // k = 8*row + i
                        const uint32_t tb[4] = {t[i + 4].x, t[i + 4].y, t[i + 4].z, t[i + 4].w};  // k + 4
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            const uint32_t h = ((w[c] >> (4 * i)) & magic.mask_lo) | magic.bias_lo;
                            const uint32_t nz = (ta[c] >> 16) | (tb[c] & 0xffff0000u);
                            const uint32_t ss = (ta[c] & 0xffffu) | (tb[c] << 16);
                            d[c][i] = (as_half2(h) + as_half2(nz)) * as_half2(ss);
                        }
                    }
                }
#pragma unroll
                for (int m = 0; m < MB; ++m) {
                    uint4 xv = *reinterpret_cast<const uint4 *>(xchunk + m * Ls + rr * 8);
                    if (ACT && !valid)
                        xv = make_uint4(0, 0, 0, 0);
                    const half2_t xp[4] = {as_half2(xv.x), as_half2(xv.y), as_half2(xv.z), as_half2(xv.w)};
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        float s = FACTORED ? gacc[m][c] : acc[m][c];
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            s = dot2(d[c][i], xp[i], s);
                        if (FACTORED)
                            gacc[m][c] = s;
                        else
                            acc[m][c] = s;
                    }
                }
            }
            if (FACTORED && !(ABL & kNoIla)) {
#pragma unroll
                for (int m = 0; m < MB; ++m) {
                    const float2 bs = xc[m * nchunks + ul];
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const float dsum = (ABL & kMatrixDot) ? mdot[c][m] : gacc[m][c];
                        const float t = __builtin_fmaf(-zf[c], bs.y, dsum - bs.x);  // sum_k x_k (q_k - z)
                        acc[m][c] = __builtin_fmaf(sf[c], t, acc[m][c]);
                    }
                }
            }
        }
    };

    {
        // Software pipeline over two register sets: the next step's weights fly while this step is
        // consumed.  Every wavefront runs the same number of steps (lanes past the end of the slice load
        // clamped chunks and add nothing); the steady-state loop issues unconditionally and the last one
        // or two steps are peeled, so that no branch separates a load from its use.
        // (GC: two steps per group, RW groups per pair of steps)
        const int nsteps = GC ? 2 * (((nchunks >> 2) + RW - 1) / RW) : (nchunks + STEP - 1) / STEP;
        int t = 0;
        // The step boundary: everything a step adds to the accumulators is computed before the loads of
        // the step after next are issued (the empty asm orders the arithmetic, the scheduling barrier the
        // loads), so two steps are in flight, not three, and the register count stays down.
        auto step_boundary = [&]() {
#pragma unroll
            for (int m = 0; m < MB; ++m)
                asm volatile("" : "+v"(acc[m][0]), "+v"(acc[m][1]), "+v"(acc[m][2]), "+v"(acc[m][3])::"memory");
            __builtin_amdgcn_sched_barrier(0);
        };
        while (t + 2 < nsteps) {
            issue(t + 1, rb, odd_step);
            consume(t, ra, even_step);
            step_boundary();
            issue(t + 2, ra, even_step);
            consume(t + 1, rb, odd_step);
            step_boundary();
            t += 2;
        }
        if (t + 2 == nsteps) {
            issue(t + 1, rb, odd_step);
            consume(t, ra, even_step);
            step_boundary();
            consume(t + 1, rb, odd_step);
        } else {
            consume(t, ra, even_step);
        }
    }

    if (ABL & kNoSmb) {
        // baseline commit: every lane adds its partial sums to the (zeroed) fp32 buffer with atomics; the last
        // workgroup of the column tile converts and clears the buffer
        if (n0 < N) {
#pragma unroll
            for (int m = 0; m < MB; ++m)
                if (m < a.M)
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        __hip_atomic_fetch_add(a.partial + (size_t)m * N + n0 + c, acc[m][c], __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT);
        }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (tid == 0)
            s_last = (slice_arrive(a.counters + tile) == (unsigned)(a.split_k - 1));
        __syncthreads();
        if (s_last) {
            slice_acquire();
            for (int i = tid; i < a.M * CT; i += kThreads) {
                const int m = i / CT;
                const int n = tile * CT + (i - m * CT);
                if (n < N)
                    a.out[(size_t)m * N + n] = (half_t)load_device_scope(a.partial + (size_t)m * N + n);
            }
            if (tid == 0)
                __hip_atomic_store(a.counters + tile, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        return;
    }

    // ---- reduce over the row lanes of a wavefront (shuffles), then over wavefronts (LDS) ----
    if (RL > 1) {
#pragma unroll
        for (int o = LPR; o < 64; o <<= 1)
#pragma unroll
            for (int m = 0; m < MB; ++m)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    acc[m][c] += __shfl_xor(acc[m][c], o, 64);
    }

#pragma unroll
    for (int m0 = 0; m0 < MB; m0 += MC) {
        if (m0 > 0)
            __syncthreads();
        if (rl == 0) {
#pragma unroll
            for (int mm = 0; mm < MC; ++mm) {
                float4_t v = {acc[m0 + mm][0], acc[m0 + mm][1], acc[m0 + mm][2], acc[m0 + mm][3]};
                *reinterpret_cast<float4_t *>(red + ((size_t)wave * MC + mm) * CT + cq * 4) = v;
            }
        }
        __syncthreads();
        for (int i = tid; i < MC * CT; i += kThreads) {
            const int mm = i / CT;
            const int col = i - mm * CT;
            const int m = m0 + mm;
            const int n = tile * CT + col;
            float s = red[(0 * MC + mm) * CT + col];
#pragma unroll
            for (int w = 1; w < kWaves; ++w)
                s += red[((size_t)w * MC + mm) * CT + col];
            if (m < a.M && n < N) {
                if (a.split_k == 1)
                    a.out[(size_t)m * N + n] = (half_t)s;
                else
                    store_device_scope(a.partial + ((size_t)slice * a.M + m) * N + n, s);
            }
        }
    }

    // ---- combine the K slices: the last workgroup of this column tile adds them in slice order ----
    if (a.split_k > 1) {
        // all partial stores of this workgroup have been acknowledged before its arrival is counted (exchange.h)
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (tid == 0)
            s_last = (slice_arrive(a.counters + tile) == (unsigned)(a.split_k - 1));
        __syncthreads();
        if (s_last) {
            slice_acquire();
            for (int i = tid; i < a.M * CT; i += kThreads) {
                const int m = i / CT;
                const int n = tile * CT + (i - m * CT);
                if (n < N) {
                    // eight loads in flight at a time; the additions stay in slice order
                    float s = 0.f;
                    for (int sl0 = 0; sl0 < a.split_k; sl0 += 8) {
                        float v[8];
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            const int sl = min(sl0 + j, a.split_k - 1);
                            v[j] = load_device_scope(a.partial + ((size_t)sl * a.M + m) * N + n);
                        }
#pragma unroll
                        for (int j = 0; j < 8; ++j)
                            s += (sl0 + j < a.split_k) ? v[j] : 0.f;
                    }
                    a.out[(size_t)m * N + n] = (half_t)s;
                }
            }
            if (tid == 0)
                __hip_atomic_store(a.counters + tile, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // next launch
        }
    }
}

// Host-side launcher of one batch size (defined once per MB in decode_mb.hip).
template <int MB>
hipError_t launch_mb(const Args &a, int lpr, int chunk_rows, bool act, int ablate, size_t lds_bytes,
                     hipStream_t stream);

}  // namespace decode
}  // namespace gptq

// Split-K vector kernel for the W4A16 GPTQ matrix multiply at small batch (M <= 16), gfx950.
//
// The paper's kernel pipeline (Opt4GPTQ, Section 3) has three stages, all of which exist here
// in a form that suits CDNA4:
//   * activations are staged in on-chip memory with wide loads (Section 3.2; here 128-bit loads,
//     and the eight values of a packed row are stored in the order the dequantised pairs need);
//   * the inner loop is packed half arithmetic (Section 3.3, Eq. 14-15): two weights per VGPR are
//     formed with one v_and_or_b32, shifted by the zero point with one packed add, and contracted
//     with v_dot2_f32_f16 into fp32 accumulators;
//   * partial sums are reduced on chip before anything is committed (Section 3.1, Eq. 6-10):
//     across lanes with wavefront shuffles, across wavefronts through LDS, and across the K slices
//     of different workgroups through fp32 partials in scratch that the last workgroup to arrive
//     adds in slice order.  No floating point atomics: the result is deterministic.
//
// Work decomposition.  A workgroup (4 wavefronts) owns CT = 4*LPR adjacent columns and one slice
// of K.  A lane owns 4 adjacent columns (one 128-bit load of a packed qweight row = 4 x 8 weights)
// and, together with the other lanes of the same column quad ("row lanes", 64/LPR per wavefront,
// 4x that per workgroup), strides over the slice in chunks of R packed rows.  With LPR = 16 a
// wavefront load touches 4 rows x 256 contiguous bytes.
#pragma once

#include "kernels.h"

namespace gptq {
namespace decode {

constexpr int kThreads = 256;
constexpr int kWaves = 4;

struct Args {
    const half_t *x;
    const uint32_t *qweight;
    const uint32_t *qzeros;
    const half_t *scales;
    const int32_t *g_idx;
    half_t *out;
    float *partial;       // [split_k, M, N] fp32, only if split_k > 1
    unsigned *counters;   // [tiles_n], zero between launches
    int M, K, N;
    int rows;             // K / 8 packed rows
    int rows_per_group;   // group_size / 8
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

// The eight codes of one packed word as four half2 of exact small integers minus the zero point:
//   d[0] = (q0 - z, q4 - z), d[1] = (q1 - z, q5 - z), d[2] = (q2 - z, q6 - z), d[3] = (q3 - z, q7 - z).
// 0x6400 is 1024.0 (ulp 1): OR-ing a nibble into bits 0..3 gives 1024 + q exactly.
// 0x5400 is 64.0 (ulp 1/16): OR-ing a nibble into bits 4..7 gives 64 + q exactly.
// neg_lo = (-(1024 + z)) x2 and neg_hi = (-(64 + z)) x2; both sums are exact in fp16.
__device__ __forceinline__ void codes_minus_zero(uint32_t w, half2_t neg_lo, half2_t neg_hi, half2_t d[4])
{
    const uint32_t w8 = w >> 8;
    d[0] = as_half2((w & 0x000f000fu) | 0x64006400u) + neg_lo;
    d[1] = as_half2((w & 0x00f000f0u) | 0x54005400u) + neg_hi;
    d[2] = as_half2((w8 & 0x000f000fu) | 0x64006400u) + neg_lo;
    d[3] = as_half2((w8 & 0x00f000f0u) | 0x54005400u) + neg_hi;
}

template <int MB, int LPR, int R, bool ACT>
__global__ __launch_bounds__(kThreads) void decode_kernel(const Args a)
{
    constexpr int RL = 64 / LPR;          // row lanes per wavefront
    constexpr int RW = kWaves * RL;       // row lanes per workgroup
    constexpr int CT = LPR * 4;           // columns per workgroup
    constexpr int MC = MB < 4 ? MB : 4;   // batch rows per cross-wavefront reduction round
    constexpr bool SCALE_W = ACT || MB >= 8;  // scale the weights (true) or the per-chunk sums (false)

    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int cq = lane % LPR;
    const int rl = lane / LPR;
    const int rid = wave * RL + rl;
    const int tile = blockIdx.x % a.tiles_n;
    const int slice = blockIdx.x / a.tiles_n;
    const int n0 = tile * CT + cq * 4;
    const bool col_ok = n0 < a.N;
    const int N = a.N;

    const int c0 = slice * a.chunks_per_slice;
    const int c1 = min(c0 + a.chunks_per_slice, a.total_chunks);
    const int kbeg = c0 * R * 8;
    const int kend = min(c1 * R * 8, a.K);
    const int Ls = kend - kbeg;  // activations of this slice, per batch row (multiple of 8)

    // ---- LDS carve-up ----
    half_t *xs = reinterpret_cast<half_t *>(smem);                      // [MB][Ls], pair-permuted
    size_t off = ((size_t)MB * Ls * sizeof(half_t) + 15) & ~(size_t)15;
    float *red = reinterpret_cast<float *>(smem + off);                 // [kWaves][MC][CT]
    off += (size_t)kWaves * MC * CT * sizeof(float);
    int *gl = reinterpret_cast<int *>(smem + off);                      // ACT: [Ls] group of each k
    uint32_t *tab = reinterpret_cast<uint32_t *>(smem + off + (ACT ? (size_t)Ls * sizeof(int) : 0));  // ACT: [groups][CT]

    // ---- stage the activations of this slice (128-bit loads), in the order (0,4,1,5,2,6,3,7) ----
    {
        const int vecs = Ls >> 3;
        for (int i = tid; i < MB * vecs; i += kThreads) {
            const int m = i / vecs;
            const int v = i - m * vecs;
            half8_t h = {0, 0, 0, 0, 0, 0, 0, 0};
            if (m < a.M)
                h = *reinterpret_cast<const half8_t *>(a.x + (size_t)m * a.K + kbeg + v * 8);
            half8_t p = {h[0], h[4], h[1], h[5], h[2], h[6], h[3], h[7]};
            *reinterpret_cast<half8_t *>(xs + (size_t)m * Ls + v * 8) = p;
        }
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

    constexpr int UNROLL = 2;  // chunks in flight per lane
    if (col_ok) {
        for (int u0 = c0 + rid; u0 < c1; u0 += RW * UNROLL) {
            uint4 wq[UNROLL][R];
            half4_t sc[UNROLL];
            uint32_t zb[UNROLL];
            // ---- issue every global load of this step first ----
#pragma unroll
            for (int j = 0; j < UNROLL; ++j) {
                const int u = u0 + j * RW;
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const int row = u * R + r;
                    wq[j][r] = make_uint4(0, 0, 0, 0);
                    if (u < c1 && row < a.rows)
                        wq[j][r] = *reinterpret_cast<const uint4 *>(a.qweight + (size_t)row * N + n0);
                }
                sc[j] = half4_t{0, 0, 0, 0};
                zb[j] = 0;
                if (!ACT && u < c1) {
                    const int grp = (u * R) / a.rows_per_group;
                    sc[j] = *reinterpret_cast<const half4_t *>(a.scales + (size_t)grp * N + n0);
                    zb[j] = a.qzeros[(size_t)grp * (N >> 3) + (n0 >> 3)] >> ((n0 & 4) * 4);
                }
            }
            // ---- dequantise and contract ----
#pragma unroll
            for (int j = 0; j < UNROLL; ++j) {
                const int u = u0 + j * RW;
                if (u >= c1)
                    break;
                half2_t neg_lo[4], neg_hi[4], s2[4];
                float gacc[MB][4];
                if (!ACT) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const uint32_t z = (zb[j] >> (4 * c)) & 15u;
                        neg_lo[c] = as_half2(0xE400E400u | (z * 0x00010001u));
                        neg_hi[c] = as_half2(0xD400D400u | (z * 0x00100010u));
                        s2[c] = half2_t{sc[j][c], sc[j][c]};
                    }
#pragma unroll
                    for (int m = 0; m < MB; ++m)
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            gacc[m][c] = 0.f;
                }
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const int row = u * R + r;
                    if (row >= a.rows)
                        break;
                    const int koff = row * 8 - kbeg;
                    const uint32_t w[4] = {wq[j][r].x, wq[j][r].y, wq[j][r].z, wq[j][r].w};
                    half2_t d[4][4];
                    if (!ACT) {
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            codes_minus_zero(w[c], neg_lo[c], neg_hi[c], d[c]);
                            if (SCALE_W) {
#pragma unroll
                                for (int i = 0; i < 4; ++i)
                                    d[c][i] = d[c][i] * s2[c];
                            }
                        }
                    } else {
                        // every k of the packed row may belong to a different group
                        const int4 ga = *reinterpret_cast<const int4 *>(gl + koff);
                        const int4 gb = *reinterpret_cast<const int4 *>(gl + koff + 4);
                        const int g[8] = {ga.x, ga.y, ga.z, ga.w, gb.x, gb.y, gb.z, gb.w};
                        uint4 t[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            t[e] = *reinterpret_cast<const uint4 *>(tab + (size_t)g[e] * CT + cq * 4);
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const uint32_t ta[4] = {t[i].x, t[i].y, t[i].z, t[i].w};          // k = 8*row + i
                            const uint32_t tb[4] = {t[i + 4].x, t[i + 4].y, t[i + 4].z, t[i + 4].w};  // k + 4
#pragma unroll
                            for (int c = 0; c < 4; ++c) {
                                const uint32_t h = ((w[c] >> (4 * i)) & 0x000f000fu) | 0x64006400u;
                                const uint32_t nz = (ta[c] >> 16) | (tb[c] & 0xffff0000u);
                                const uint32_t ss = (ta[c] & 0xffffu) | (tb[c] << 16);
                                d[c][i] = (as_half2(h) + as_half2(nz)) * as_half2(ss);
                            }
                        }
                    }
#pragma unroll
                    for (int m = 0; m < MB; ++m) {
                        const uint4 xv = *reinterpret_cast<const uint4 *>(xs + (size_t)m * Ls + koff);
                        const half2_t xp[4] = {as_half2(xv.x), as_half2(xv.y), as_half2(xv.z), as_half2(xv.w)};
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            float s = SCALE_W ? acc[m][c] : gacc[m][c];
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                s = dot2(d[c][i], xp[i], s);
                            if (SCALE_W)
                                acc[m][c] = s;
                            else
                                gacc[m][c] = s;
                        }
                    }
                }
                if (!SCALE_W) {
#pragma unroll
                    for (int m = 0; m < MB; ++m)
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            acc[m][c] = __builtin_fmaf((float)sc[j][c], gacc[m][c], acc[m][c]);
                }
            }
        }
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
                    a.partial[((size_t)slice * a.M + m) * N + n] = s;
            }
        }
    }

    // ---- combine the K slices: the last workgroup of this column tile adds them in slice order ----
    if (a.split_k > 1) {
        __shared__ int s_last;
        __threadfence();  // release this workgroup's partials device-wide
        __syncthreads();
        if (tid == 0) {
            const unsigned prev = atomicAdd(a.counters + tile, 1u);
            s_last = (prev == (unsigned)(a.split_k - 1));
        }
        __syncthreads();
        if (s_last) {
            __threadfence();  // acquire the other workgroups' partials
            for (int i = tid; i < a.M * CT; i += kThreads) {
                const int m = i / CT;
                const int n = tile * CT + (i - m * CT);
                if (n < N) {
                    float s = 0.f;
                    for (int sl = 0; sl < a.split_k; ++sl)
                        s += a.partial[((size_t)sl * a.M + m) * N + n];
                    a.out[(size_t)m * N + n] = (half_t)s;
                }
            }
            if (tid == 0)
                atomicExch(a.counters + tile, 0u);  // ready for the next launch
        }
    }
}

// Host-side launcher of one batch size (defined once per MB in decode_mb.hip).
template <int MB>
hipError_t launch_mb(const Args &a, int lpr, int chunk_rows, bool act, size_t lds_bytes, hipStream_t stream);

}  // namespace decode
}  // namespace gptq

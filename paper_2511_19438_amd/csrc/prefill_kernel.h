// fp16 MFMA kernel for the W4A16 GPTQ matrix multiply at large batch (prefill), gfx950.
//
// This is the one place where the path is a real dense contraction, so it runs on the matrix
// cores (v_mfma_f32_32x32x16_f16, fp32 accumulation).  The paper's kernel (Opt4GPTQ, Section 3)
// uses one vector kernel for every batch size; what carries over is its pipeline order: stage the
// activations on chip with wide loads (Section 3.2), dequantise with packed half arithmetic
// (Section 3.3), accumulate on chip and commit each output once (Section 3.1).
//
// Design for CDNA4:
//   * A operand (activations): tiles of BM x 64 are copied global -> registers -> LDS with 128-bit
//     accesses, double buffered, 16-byte chunks XOR-swizzled by row so that the MFMA operand reads
//     (ds_read_b128, 32 rows at one k offset) are bank-conflict free.
//   * B operand (weights): never touches LDS.  A packed qweight word holds eight consecutive k of
//     ONE column, which is exactly what one lane of the 32x32x16 MFMA B operand holds.  Each lane
//     loads its word(s) straight from global memory, one stage ahead, and dequantises them in
//     registers into the four VGPRs of the operand: v_perm_b32 + v_and_or_b32 build the pair
//     (1024 + q_even, 64 + q_odd), a packed add of (-(1024 + z), -(64 + z)) gives the exact integer
//     differences and a packed multiply by the scale gives the fp16 weight with one rounding.
//   * Waves of a workgroup split the N extent of the tile where possible, so every weight is
//     dequantised by exactly one wave of the workgroup and the VALU work rides in the shadow of
//     the MFMAs.
//   * Lane j of an n-block owns TN adjacent columns (n-block t <-> column base + TN*j + t), so the
//     B loads are TN dwords wide and the output stores are TN halves wide.
//   * Workgroup ids are remapped so that the tiles resident on one XCD (ids congruent mod 8) are
//     neighbours in the (m fastest) tile order and share their weight panel and activations in
//     that XCD's L2.
#pragma once

#include "kernels.h"

namespace gptq {
namespace prefill {

constexpr int kThreads = 256;
constexpr int BK = 64;  // k extent of one LDS stage

enum Mode {
    kGroupPerStage = 0,  // group_size % 64 == 0, no g_idx: one scale/zero per lane column per stage
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
};

__device__ __forceinline__ half2_t as_half2(uint32_t v)
{
    return __builtin_bit_cast(half2_t, v);
}

// (-(1024 + z), -(64 + z)) as packed fp16 bits
__device__ __forceinline__ uint32_t neg_bias(uint32_t z)
{
    return 0xD400E400u | z | (z << 20);
}

// One packed word (8 consecutive k of one column) -> the 8 fp16 weights in k order.
// nz[i] / ss[i] are the packed negative biases and scales of the pair (2i, 2i+1).
__device__ __forceinline__ half8_t dequant_word(uint32_t w, const uint32_t nz[4], const uint32_t ss[4])
{
    half2_t p[4];
    // byte i of w = q_{2i} | q_{2i+1} << 4 ; spread it to both halves, keep one nibble in each
    p[0] = as_half2((__builtin_amdgcn_perm(0u, w, 0x0c000c00u) & 0x00f0000fu) | 0x54006400u);
    p[1] = as_half2((__builtin_amdgcn_perm(0u, w, 0x0c010c01u) & 0x00f0000fu) | 0x54006400u);
    p[2] = as_half2((__builtin_amdgcn_perm(0u, w, 0x0c020c02u) & 0x00f0000fu) | 0x54006400u);
    p[3] = as_half2((__builtin_amdgcn_perm(0u, w, 0x0c030c03u) & 0x00f0000fu) | 0x54006400u);
#pragma unroll
    for (int i = 0; i < 4; ++i)
        p[i] = (p[i] + as_half2(nz[i])) * as_half2(ss[i]);
    return half8_t{p[0][0], p[0][1], p[1][0], p[1][1], p[2][0], p[2][1], p[3][0], p[3][1]};
}

template <int BM, int BN, int WM, int WN, int MODE>
__global__ __launch_bounds__(kThreads) void prefill_kernel(const Args a)
{
    static_assert(WM * WN == 4, "four wavefronts per workgroup");
    constexpr int WAVE_M = BM / WM;
    constexpr int WAVE_N = BN / WN;
    constexpr int TM = WAVE_M / 32;
    constexpr int TN = WAVE_N / 32;
    static_assert(TM >= 1 && (TN == 1 || TN == 2 || TN == 4), "wave tile must be 32-row blocks by 32/64/128 columns");
    constexpr int A_CHUNKS = BM * (BK / 8) / kThreads;  // 16-byte chunks of the A tile per thread
    static_assert(A_CHUNKS >= 1, "tile too small for 256 threads");
    constexpr int KSTEPS = BK / 16;

    extern __shared__ __align__(16) unsigned char smem[];
    half_t *lds_a = reinterpret_cast<half_t *>(smem);  // [2][BM][64] halves, chunk-swizzled

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN;
    const int wn = wave % WN;
    const int lj = lane & 31;
    const int kh = lane >> 5;

    // ---- XCD-aware tile order: ids congruent mod 8 run on one XCD; give each XCD a contiguous range ----
    const int total = a.tiles_m * a.tiles_n;
    const int per_xcd = (total + 7) / 8;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= total)
        return;
    const int tile_m = logical % a.tiles_m;
    const int tile_n = logical / a.tiles_m;
    const int m0 = tile_m * BM;
    const int n0 = tile_n * BN;

    const int N = a.N, K = a.K, M = a.M;
    const int rows = K >> 3;
    const int col0 = n0 + wn * WAVE_N + TN * lj;  // first of this lane's TN columns
    const bool col_ok = col0 < N;
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

    uint4 a_next[A_CHUNKS];
    uint32_t bw_cur[KSTEPS][TN], bw_next[KSTEPS][TN];
    half_t sc_cur[TN], sc_next[TN];
    uint32_t z_cur = 0, z_next = 0;

    auto load_a = [&](int stage) {
        const int k0 = stage * BK;
#pragma unroll
        for (int c = 0; c < A_CHUNKS; ++c) {
            const int idx = tid + c * kThreads;
            const int row = idx >> 3;
            const int ch = idx & 7;
            const int m = m0 + row;
            const int k = k0 + ch * 8;
            a_next[c] = make_uint4(0, 0, 0, 0);
            if (m < M && k < K)
                a_next[c] = *reinterpret_cast<const uint4 *>(a.x + (size_t)m * K + k);
        }
    };
    auto store_a = [&](int buf) {
#pragma unroll
        for (int c = 0; c < A_CHUNKS; ++c) {
            const int idx = tid + c * kThreads;
            const int row = idx >> 3;
            const int ch = (idx & 7) ^ (row & 7);
            *reinterpret_cast<uint4 *>(lds_a + ((size_t)buf * BM + row) * BK + ch * 8) = a_next[c];
        }
    };
    auto load_b = [&](int stage) {
        const int prow0 = stage * (BK / 8);
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            const int prow = prow0 + 2 * kk + kh;
#pragma unroll
            for (int t = 0; t < TN; ++t)
                bw_next[kk][t] = 0;
            if (col_ok && prow < rows) {
                const uint32_t *src = a.qweight + (size_t)prow * N + col0;
                if (TN == 4) {
                    const uint4 v = *reinterpret_cast<const uint4 *>(src);
                    bw_next[kk][0] = v.x;
                    bw_next[kk][1 % TN] = v.y;
                    bw_next[kk][2 % TN] = v.z;
                    bw_next[kk][3 % TN] = v.w;
                } else if (TN == 2) {
                    const uint2 v = *reinterpret_cast<const uint2 *>(src);
                    bw_next[kk][0] = v.x;
                    bw_next[kk][1 % TN] = v.y;
                } else {
                    bw_next[kk][0] = *src;
                }
            }
        }
        if (MODE == kGroupPerStage) {
#pragma unroll
            for (int t = 0; t < TN; ++t)
                sc_next[t] = (half_t)0;
            z_next = 0;
            const int k0 = stage * BK;
            if (col_ok && k0 < K) {
                const int g = k0 / a.group_size;
#pragma unroll
                for (int t = 0; t < TN; ++t)
                    sc_next[t] = a.scales[(size_t)g * N + col0 + t];
                z_next = a.qzeros[(size_t)g * (N >> 3) + (col0 >> 3)] >> zshift;
            }
        }
    };

    // ---- prologue ----
    load_a(0);
    load_b(0);
    store_a(0);
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk)
#pragma unroll
        for (int t = 0; t < TN; ++t)
            bw_cur[kk][t] = bw_next[kk][t];
#pragma unroll
    for (int t = 0; t < TN; ++t)
        sc_cur[t] = sc_next[t];
    z_cur = z_next;
    __syncthreads();

    for (int s = 0; s < stages; ++s) {
        const int buf = s & 1;
        if (s + 1 < stages) {
            load_a(s + 1);
            load_b(s + 1);
        }

        // per-stage dequant constants (group-per-stage mode)
        uint32_t nz_st[TN][4], ss_st[TN][4];
        if (MODE == kGroupPerStage) {
#pragma unroll
            for (int t = 0; t < TN; ++t) {
                const uint32_t nb = neg_bias((z_cur >> (4 * t)) & 15u);
                const uint32_t sb = __builtin_bit_cast(uint16_t, sc_cur[t]);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    nz_st[t][i] = nb;
                    ss_st[t][i] = sb | (sb << 16);
                }
            }
        }

#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            const int prow = s * (BK / 8) + 2 * kk + kh;  // this lane's packed row
            half8_t bfrag[TN];
#pragma unroll
            for (int t = 0; t < TN; ++t) {
                if (MODE == kGroupPerStage) {
                    bfrag[t] = dequant_word(bw_cur[kk][t], nz_st[t], ss_st[t]);
                } else {
                    uint32_t nz[4] = {0, 0, 0, 0}, ss[4] = {0, 0, 0, 0};
                    if (col_ok && prow < rows) {
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
                    bfrag[t] = dequant_word(bw_cur[kk][t], nz, ss);
                }
            }
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int row = wm * WAVE_M + i * 32 + lj;
                const int ch = (2 * kk + kh) ^ (row & 7);
                const half8_t afrag =
                    *reinterpret_cast<const half8_t *>(lds_a + ((size_t)buf * BM + row) * BK + ch * 8);
#pragma unroll
                for (int t = 0; t < TN; ++t)
                    acc[i][t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(afrag, bfrag[t], acc[i][t], 0, 0, 0);
            }
        }

        if (s + 1 < stages) {
            store_a(buf ^ 1);
#pragma unroll
            for (int kk = 0; kk < KSTEPS; ++kk)
#pragma unroll
                for (int t = 0; t < TN; ++t)
                    bw_cur[kk][t] = bw_next[kk][t];
#pragma unroll
            for (int t = 0; t < TN; ++t)
                sc_cur[t] = sc_next[t];
            z_cur = z_next;
        }
        __syncthreads();
    }

    // ---- epilogue: one fp16 rounding, TN adjacent columns per store ----
    if (col_ok) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm * WAVE_M + i * 32 + 8 * (r >> 2) + 4 * kh + (r & 3);
                if (m < M) {
                    half_t *dst = a.out + (size_t)m * N + col0;
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
}

}  // namespace prefill
}  // namespace gptq

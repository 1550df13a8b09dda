// Mid-batch variant of the big-tile fp16 MFMA kernel (32 ... 128 rows): the four wavefronts of a workgroup
// split the K extent of every stage instead of the tile's columns.
//
// In the column-split layout of prefill_pipelined_kernel a 64 x 128 tile gives each wavefront a 64 x 32
// share: every A operand read from LDS (1 KB) feeds ONE MFMA, four wavefronts read the whole activation tile
// each, and the LDS bandwidth (128 B per cycle and compute unit) - not the matrix pipe, not HBM - sets the pace
// (0.46 us per 64-k stage, i.e. 9 GB/s of weights per workgroup).  Here wavefront w takes k step w (16 k) of
// every 64-k stage and multiplies it into the WHOLE tile (TM x 4 accumulator blocks), so an A operand is read
// once per four MFMAs and by one wavefront only; LDS traffic per stage drops from 36 KB to 12 KB.  The four
// partial tiles meet at the end through LDS (the stage ring is free by then), in wavefront order; each
// wavefront then owns four of every sixteen accumulator rows, which is what it stores or - with K slices
// across workgroups - leaves in scratch exactly as the other kernels do (Section 3.1 of the paper: accumulate
// on chip, commit once; here without atomics and in a fixed order).
//
// Staging (global -> LDS by DMA, ring of NBUF stage buffers, one vmcnt wait + barrier per stage), the A tile's
// swizzle, the in-register dequantisation of the B operand and the workgroup order are those of
// prefill_pipelined_kernel.
#pragma once

#include "prefill_kernel.h"

namespace gptq {
namespace prefill {

// LDS the cross-wavefront reduction of one 32-row block needs: 12 (source, destination) pairs x 4 n-blocks x
// 64 lanes x 16 bytes.
constexpr int kKsplitReduceBytes = 12 * 4 * 64 * 16;

typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

template <int BM, int BN, int NBUF>
__global__ __launch_bounds__(kThreads, 2) void prefill_ksplit_kernel(const Args a)
{
    constexpr int BK = 64;
    using L = StageLayout<BM, BN, BK>;
    constexpr int TM = BM / 32;
    constexpr int TN = BN / 32;
    static_assert(TM == 1 || TM == 2, "32 or 64 rows");
    static_assert(TN == 4, "128 columns: a lane's four columns are one 128-bit word read");
    static_assert(NBUF >= 3, "ring of at least three stage buffers");
    constexpr int CH = BK / 8;    // 16-byte chunks per A row
    constexpr int RPB = 16 / CH;  // A rows per 256-byte bank row
    constexpr int A_CHUNKS = BM * CH / kThreads;
    constexpr int B_CHUNKS = (BK / 8) * BN / 4 / kThreads;
    static_assert(A_CHUNKS >= 1 && B_CHUNKS >= 1, "tile too small for 256 threads");
    constexpr int LOADS_PER_STAGE = A_CHUNKS + B_CHUNKS + 1;
    constexpr int MAX_IN_FLIGHT = (NBUF - 3) * LOADS_PER_STAGE;
    static_assert(MAX_IN_FLIGHT < 64, "vmcnt is a 6-bit counter");

    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // = this wavefront's k step in every stage
    const int lj = lane & 31;
    const int kh = lane >> 5;

    int tile_m, tile_n, tile_id, slice;
    if (!tile_of_workgroup(a, tile_m, tile_n, tile_id, slice))
        return;
    const int m0 = tile_m * BM;
    const int n0 = tile_n * BN;
    const int N = a.N, K = a.K, M = a.M;
    const int all_stages = K / BK;
    const int first = slice * a.stages_per_slice;
    const int stages = min(a.stages_per_slice, all_stages - first);
    const int last = first + stages - 1;
    const int col_local = TN * lj;
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

    // ---- DMA sources (see prefill_pipelined_kernel: clamped, branch-free, 32-bit offsets from uniform bases) ----
    const char *a_base = reinterpret_cast<const char *>(a.x + (size_t)m0 * K);
    uint32_t a_off[A_CHUNKS];
#pragma unroll
    for (int j = 0; j < A_CHUNKS; ++j) {
        const int slot = tid + j * kThreads;
        const int row = slot / CH;
        const int ch = (slot % CH) ^ ((row / RPB) & (CH - 1));
        a_off[j] = (uint32_t)((min(m0 + row, M - 1) - m0) * K + ch * 8) * 2u;
    }
    const char *b_base = reinterpret_cast<const char *>(a.qweight + n0);
    uint32_t b_off[B_CHUNKS];
#pragma unroll
    for (int j = 0; j < B_CHUNKS; ++j) {
        const int slot = tid + j * kThreads;
        const int row = slot / (BN / 4);
        const int c4 = slot % (BN / 4);
        b_off[j] = (uint32_t)(row * N + min(4 * c4, N - 4 - n0)) * 4u;
    }
    const int sz_lane = min(lane, BN / 8 + BN / 32 - 1);
    const bool sz_is_scale = sz_lane < BN / 8;
    const int sz_col = sz_is_scale ? min(n0 + 8 * sz_lane, N - 8) : min(n0 + 32 * (sz_lane - BN / 8), N - 32);
    const char *sz_src = sz_is_scale ? reinterpret_cast<const char *>(a.scales + sz_col)
                                     : reinterpret_cast<const char *>(a.qzeros + (sz_col >> 3));
    const uint32_t sz_stride = sz_is_scale ? (uint32_t)N * 2u : (uint32_t)(N >> 3) * 4u;
    const int stages_per_group = a.group_size / BK;

    int ld_stage = first, ld_group = first / stages_per_group, ld_in_group = first % stages_per_group;
    auto stage_base = [&](int ring) { return smem + (size_t)ring * L::BYTES; };
    auto issue_piece = [&](int p, int ring) {
        unsigned char *base = stage_base(ring);
        const size_t k0 = (size_t)ld_stage * BK;
        if (p < A_CHUNKS) {
            __builtin_amdgcn_global_load_lds((global_ptr_t *)(a_base + k0 * 2 + a_off[p]),
                                             (lds_ptr_t *)(base + (size_t)(p * kThreads + wave * 64) * 16), 16, 0, 0);
        } else if (p < A_CHUNKS + B_CHUNKS) {
            const int j = p - A_CHUNKS;
            __builtin_amdgcn_global_load_lds((global_ptr_t *)(b_base + (k0 / 8) * N * 4 + b_off[j]),
                                             (lds_ptr_t *)(base + L::A_BYTES + (size_t)(j * kThreads + wave * 64) * 16),
                                             16, 0, 0);
        } else {
            __builtin_amdgcn_global_load_lds((global_ptr_t *)(sz_src + (size_t)ld_group * sz_stride),
                                             (lds_ptr_t *)(base + L::A_BYTES + L::B_BYTES), 16, 0, 0);
        }
    };
    // (selects, not branches: a branch here ends the basic block, and the dequantisation of a stage's last
    // slots - pure arithmetic whose results are first used in the next stage - sinks across it, out of the
    // MFMAs' shadow)
    auto advance_load_stage = [&]() {
        const int more = ld_stage < last ? 1 : 0;  // past the end the last stage is refetched: uniform counts
        ld_stage += more;
        ld_in_group += more;
        const int wrap = ld_in_group == stages_per_group ? 1 : 0;
        ld_in_group = wrap ? 0 : ld_in_group;
        ld_group += wrap;
    };
    auto publish = [&]() {
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(MAX_IN_FLIGHT) : "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };

    // ---- operands: this wavefront's k step (16 k) of the stage in use and of the next one ----
    half8_t afr[2][TM];
    u32x4_t bfr[2][TN];
    const PairMagic magic;
    const uint32_t a_lane_off = (uint32_t)(lj * (BK * 2) + (((2 * wave + kh) ^ ((lj / RPB) & (CH - 1))) * 16));
    const uint32_t smem_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    auto read_afrag = [&](int ring, int i, half8_t &dst) {
        const uint32_t addr = smem_base + a_lane_off + (uint32_t)ring * (uint32_t)L::BYTES;
        if (i == 0)
            asm volatile("ds_read_b128 %0, %1" : "=v"(dst) : "v"(addr));
        else
            asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(32 * BK * 2));
    };
    // Every LDS read still outstanding at these points was issued at least two MFMAs earlier, so waiting for
    // all of them costs nothing; the operand is an in/out so that its MFMA cannot be moved above the wait.
    auto wait_afrag = [&](half8_t &frag) { asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(frag)); };

    // the lane's four packed words of k step `wave`, the four scales and the zero word, as read from LDS
    struct RawWeights {
        u32x4_t w;
        u32x2_t s;
        uint32_t z;
    };
    auto read_raw = [&](int ring) {
        const unsigned char *base = stage_base(ring) + L::A_BYTES;
        RawWeights r;
        r.w = *reinterpret_cast<const u32x4_t *>(base + ((size_t)(2 * wave + kh) * BN + col_local) * 4);
        const unsigned char *sz = base + L::B_BYTES;
        r.s = *reinterpret_cast<const u32x2_t *>(sz + col_local * 2);
        r.z = *reinterpret_cast<const uint32_t *>(sz + BN * 2 + (col_local >> 3) * 4);
        return r;
    };
    // (s, s) and (-(1024 + z), -(64 + z)) of the lane's four columns
    auto finish_raw = [&](const RawWeights &r, uint32_t (&nz)[TN], uint32_t (&ss)[TN]) {
        const uint32_t s01 = r.s[0], s23 = r.s[1];
        ss[0] = __builtin_amdgcn_perm(s01, s01, 0x01000100u);
        ss[1] = __builtin_amdgcn_perm(s01, s01, 0x03020302u);
        ss[2] = __builtin_amdgcn_perm(s23, s23, 0x01000100u);
        ss[3] = __builtin_amdgcn_perm(s23, s23, 0x03020302u);
        const uint32_t zs = r.z >> (16 * (lj & 1));  // the lane's four nibbles start at bit 0 or 16 of the word
#pragma unroll
        for (int t = 0; t < TN; ++t)
            nz[t] = neg_bias((zs >> (4 * t)) & 15u);
    };

    // One stage of this wavefront = TM * 4 MFMAs on its k step, in exactly this order (a scheduling barrier
    // closes every slot).  The first TM slots issue the LDS reads for the NEXT stage (A operands, and in slot 0
    // the packed words / scales / zero word), the remaining slots dequantise them into the next B operands.
    constexpr int SLOTS = TM * TN;
    constexpr int PAIRS = 4 * TN;
    constexpr int F = TM;  // first dequantising slot
    constexpr int DQ = SLOTS - F;
    constexpr int PPS = (PAIRS + DQ - 1) / DQ;
    auto stage_step = [&](auto parity, int next_ring, auto &&extra) {
        constexpr int CUR = std::decay_t<decltype(parity)>::value, NXT = CUR ^ 1;
        RawWeights raw;
        uint32_t nz[TN], ss[TN];
        uint32_t pending[PPS] = {};
#pragma unroll
        for (int m = 0; m < SLOTS; ++m) {
            const int i = m / TN, t = m % TN;
            if (t == 0)
                wait_afrag(afr[CUR][i]);
            acc[i][t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(afr[CUR][i], __builtin_bit_cast(half8_t, bfr[CUR][t]),
                                                               acc[i][t], 0, 0, 0);
            if (m < TM)
                read_afrag(next_ring, m, afr[NXT][m]);
            if (m == 0)
                raw = read_raw(next_ring);
            if (m == F)
                finish_raw(raw, nz, ss);
            if (m >= F) {
                uint32_t now[PPS];
#pragma unroll
                for (int pair = (m - F) * PAIRS / DQ; pair < (m - F + 1) * PAIRS / DQ; ++pair) {
                    const int pt = pair >> 2;
                    uint32_t r;
                    switch (pair & 3) {
                    case 0: r = dequant_pair_begin<0>(raw.w[pt], magic, nz[pt]); break;
                    case 1: r = dequant_pair_begin<1>(raw.w[pt], magic, nz[pt]); break;
                    case 2: r = dequant_pair_begin<2>(raw.w[pt], magic, nz[pt]); break;
                    default: r = dequant_pair_begin<3>(raw.w[pt], magic, nz[pt]); break;
                    }
                    asm volatile("" : "+v"(r));  // computed here, in this slot
                    now[pair - (m - F) * PAIRS / DQ] = r;
                }
                if (m > F) {
#pragma unroll
                    for (int pair = (m - 1 - F) * PAIRS / DQ; pair < (m - F) * PAIRS / DQ; ++pair) {
                        const int pt = pair >> 2;
                        uint32_t r = dequant_pair_end(pending[pair - (m - 1 - F) * PAIRS / DQ], ss[pt]);
                        asm volatile("" : "+v"(r));
                        bfr[NXT][pt][pair & 3] = r;
                    }
                }
#pragma unroll
                for (int q = 0; q < PPS; ++q)
                    pending[q] = now[q];
                if (m == SLOTS - 1) {
#pragma unroll
                    for (int pair = (m - F) * PAIRS / DQ; pair < (m - F + 1) * PAIRS / DQ; ++pair) {
                        const int pt = pair >> 2;
                        uint32_t r = dequant_pair_end(pending[pair - (m - F) * PAIRS / DQ], ss[pt]);
                        asm volatile("" : "+v"(r));
                        bfr[NXT][pt][pair & 3] = r;
                    }
                }
            }
            extra(m);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;

    // ---- prologue: NBUF-1 stages in flight, the first two published, operands of the first stage ----
#pragma unroll
    for (int s = 0; s < NBUF - 1; ++s) {
#pragma unroll
        for (int p = 0; p < LOADS_PER_STAGE; ++p)
            issue_piece(p, s);
        advance_load_stage();
    }
    publish();
    {
        const RawWeights raw = read_raw(0);
        uint32_t nz[TN], ss[TN];
        finish_raw(raw, nz, ss);
#pragma unroll
        for (int i = 0; i < TM; ++i)
            read_afrag(0, i, afr[0][i]);
#pragma unroll
        for (int t = 0; t < TN; ++t) {
            bfr[0][t][0] = dequant_pair<0>(raw.w[t], magic, nz[t], ss[t]);
            bfr[0][t][1] = dequant_pair<1>(raw.w[t], magic, nz[t], ss[t]);
            bfr[0][t][2] = dequant_pair<2>(raw.w[t], magic, nz[t], ss[t]);
            bfr[0][t][3] = dequant_pair<3>(raw.w[t], magic, nz[t], ss[t]);
        }
    }

    // Invariant at the top of stage s: stages s and s+1 are in LDS and visible, every wavefront has left stage
    // s-1, and the operands of stage s sit in afr / bfr of the stage's parity.  (After the last stage the "next"
    // reads fetch the refetched copy of the last stage; nothing uses them.)
    int ring = 0;
    auto one_stage = [&](auto parity) {
        const int ring_next = ring + 1 == NBUF ? 0 : ring + 1;
        const int ring_free = ring == 0 ? NBUF - 1 : ring - 1;
        constexpr int PIECES_PER_SLOT = (LOADS_PER_STAGE + SLOTS - 1) / SLOTS;
        auto issue_loads = [&](int m) {
#pragma unroll
            for (int q = 0; q < PIECES_PER_SLOT; ++q)
                if (m * PIECES_PER_SLOT + q < LOADS_PER_STAGE)
                    issue_piece(m * PIECES_PER_SLOT + q, ring_free);
        };
        stage_step(parity, ring_next, issue_loads);
        advance_load_stage();
        publish();
        ring = ring_next;
    };
    int s = 0;
    for (; s + 1 < stages; s += 2) {
        one_stage(P0{});
        one_stage(P1{});
    }
    if (s < stages)
        one_stage(P0{});
    // nothing may still be writing this workgroup's LDS when the ring is reused below (every wavefront has
    // waited for its own loads; the barrier inside the reduction orders them against the other wavefronts' writes)
    // The LDS wait retires the operand reads issued for the stage after the last one.  Their destination
    // registers are named as in/outs AFTER the wait: the compiler knows nothing of the reads in flight, and where
    // the values are dead (the peeled last stage) it would otherwise hand the registers to something else - an
    // address, say - that the returning read then overwrites.
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int i = 0; i < TM; ++i)
        asm volatile("" : "+v"(afr[0][i]), "+v"(afr[1][i]));
    __syncthreads();

    // ---- the four wavefronts' partial tiles meet in LDS: wavefront d ends up with accumulator rows 4d .. 4d+3
    //      of every 16 (rows 8d + 4*kh + 0..3 of each 32-row block), summed in wavefront order ----
    float red[TM][TN][4];
    float4 *xch = reinterpret_cast<float4 *>(smem);  // [12 pairs][TN][64 lanes]
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            if (d != wave) {  // uniform branch; register indices stay constant
                const int pair = wave * 3 + (d > wave ? d - 1 : d);
#pragma unroll
                for (int t = 0; t < TN; ++t)
                    xch[(pair * TN + t) * 64 + lane] = make_float4(acc[i][t][4 * d], acc[i][t][4 * d + 1],
                                                                   acc[i][t][4 * d + 2], acc[i][t][4 * d + 3]);
            }
        }
        __syncthreads();
#pragma unroll
        for (int t = 0; t < TN; ++t)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                red[i][t][q] = 0.f;
#pragma unroll
        for (int src = 0; src < 4; ++src) {
            if (src == wave) {
#pragma unroll
                for (int d = 0; d < 4; ++d)
                    if (d == wave) {
#pragma unroll
                        for (int t = 0; t < TN; ++t)
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                red[i][t][q] += acc[i][t][4 * d + q];
                    }
            } else {
                const int pair = src * 3 + (wave > src ? wave - 1 : wave);
#pragma unroll
                for (int t = 0; t < TN; ++t) {
                    const float4 v = xch[(pair * TN + t) * 64 + lane];
                    red[i][t][0] += v.x;
                    red[i][t][1] += v.y;
                    red[i][t][2] += v.z;
                    red[i][t][3] += v.w;
                }
            }
        }
        if (i + 1 < TM)
            __syncthreads();  // the next block's partials overwrite the exchange area
    }

    constexpr int ACC = TM * TN * 4;  // results per thread
    if (a.split_k > 1) {
        // ---- K slices across workgroups: as in prefill_pipelined_kernel (element e of thread t at [e][t]) ----
        __shared__ int s_last;
        const size_t tiles = (size_t)a.tiles_m * a.tiles_n;
        float *mine = a.partial + ((size_t)slice * tiles + tile_id) * ACC * kThreads + tid;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int t = 0; t < TN; ++t)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    __hip_atomic_store(mine + (size_t)((i * TN + t) * 4 + q) * kThreads, red[i][t][q],
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_s_waitcnt(0);  // every partial store of this workgroup has been acknowledged
        __syncthreads();
        if (tid == 0) {
            const unsigned prev =
                __hip_atomic_fetch_add(a.counters + tile_id, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_last = (prev == (unsigned)(a.split_k - 1));
        }
        __syncthreads();
        if (!s_last)
            return;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int t = 0; t < TN; ++t)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    red[i][t][q] = 0.f;
        for (int sl = 0; sl < a.split_k; ++sl) {
            const float *theirs = a.partial + ((size_t)sl * tiles + tile_id) * ACC * kThreads + tid;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int t = 0; t < TN; ++t)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        red[i][t][q] += __hip_atomic_load(theirs + (size_t)((i * TN + t) * 4 + q) * kThreads,
                                                          __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (tid == 0)
            __hip_atomic_store(a.counters + tile_id, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // next launch
    }

    // ---- one fp16 rounding per output; a lane stores its four adjacent columns of four rows per block ----
    if (!col_ok)
        return;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int m = m0 + i * 32 + 8 * wave + 4 * kh + q;
            if (m < M) {
                const half4_t v = {(half_t)red[i][0][q], (half_t)red[i][1][q], (half_t)red[i][2][q],
                                   (half_t)red[i][3][q]};
                *reinterpret_cast<half4_t *>(a.out + (size_t)m * N + col_raw) = v;
            }
        }
    }
}

}  // namespace prefill
}  // namespace gptq

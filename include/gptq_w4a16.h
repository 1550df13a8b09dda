/*
 * gptq_w4a16.h - C ABI of the MI355X (gfx950) W4A16 GPTQ matrix multiply.
 *
 * The operation is the 4-bit GPTQ weight-only quantized GEMM that Opt4GPTQ
 * (arxiv 2511.19438) optimises: Section 3 describes its kernel pipeline (vectorised
 * activation loads into on-chip memory, packed half-precision multiply-accumulate,
 * Eq. 14-15, and a hierarchical on-chip reduction before the result is committed,
 * Eq. 6-10 / Algorithm 1); Section 4.4 states that the result equals the plain GPTQ
 * computation up to the order of floating point additions.  That plain computation is
 *
 *     out[m, n] = sum_k x[m, k] * W[k, n]
 *     W[k, n]   = scales[r(k), n] * ( q[k, n] - z[r(k), n] )
 *     q[k, n]   = (u32(qweight[k/8][n]) >> 4*(k%8)) & 15     eight codes per word along K
 *     z[r, n]   = (u32(qzeros[r][n/8])  >> 4*(n%8)) & 15     eight zero points per word along N
 *     r(k)      = g_idx ? g_idx[k] : k / group_size          (g_idx: act-order group map)
 *
 * Layout.  Every tensor is row-major, contiguous, and lives in DEVICE memory of the
 * current HIP device.  fp16 is IEEE-754 binary16.
 *     x        fp16  [M, K]
 *     qweight  int32 [K/8, N]
 *     qzeros   int32 [K/group_size, N/8]
 *     scales   fp16  [K/group_size, N]
 *     g_idx    int32 [K]  or NULL
 *     out      fp16  [M, N]
 *
 * Ownership.  All pointers are borrowed from the caller; the library neither frees nor
 * keeps them, except the workspace given to gptq_w4a16_set_workspace(), which it uses
 * until it is replaced.  Calls only enqueue work on `stream` (a hipStream_t passed as
 * void*, NULL = the default stream) and never synchronise it: inputs and outputs must
 * stay alive until the stream has passed the call.
 *
 * Errors.  Every entry point returns 0 on success or a negative gptq_status code; it
 * never throws, aborts or prints.  Nothing is enqueued when an error is returned.
 * A g_idx entry outside [0, K/group_size) is a precondition violation that the library
 * cannot see without reading device memory; the result is then undefined.
 *
 * Supported shapes: M >= 1; K, N multiples of 8; group_size a multiple of 8 that divides K;
 * K < 2^23, N < 2^24 and K*N < 2^33 (the kernels use 32-bit offsets inside a matrix: packed
 * weights under 4 GiB).  Tuned for group_size 128.  All base pointers must be 16-byte aligned.
 *
 * Format variants.  A checkpoint without zero points (symmetric quantisation) is the same
 * format with every qzeros word equal to 0x88888888 (z = 8).  Checkpoints that store z - 1
 * are converted once with gptq_w4a16_shift_zeros().  group_size = K is one group per column.
 */
#ifndef GPTQ_W4A16_H
#define GPTQ_W4A16_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef void *gptq_stream_t; /* hipStream_t */

#define GPTQ_API __attribute__((visibility("default")))

enum gptq_status {
    GPTQ_OK = 0,
    GPTQ_INVALID_ARG = -1,         /* NULL required pointer, non-positive size, bad plan field */
    GPTQ_UNSUPPORTED_SHAPE = -2,   /* divisibility rules above violated */
    GPTQ_MISALIGNED = -3,          /* a base pointer is not 16-byte aligned */
    GPTQ_HIP_ERROR = -4,           /* a HIP call or a kernel launch failed */
    GPTQ_WORKSPACE_TOO_SMALL = -5, /* caller-set workspace smaller than gptq_w4a16_workspace_bytes() */
    GPTQ_STATIC_SCRATCH_EXCEEDED = -6 /* gptq_w4a16_gemm_static: the problem needs more than the static scratch */
};

/*
 * out = x * W (definition above; the whole pipeline of Section 3: unpack, group lookup,
 * dequantise, stage activations on chip, contract, reduce the split-K partial sums on
 * chip and across workgroups, round once to fp16, store).  `out` is OVERWRITTEN and need
 * not be zeroed (unlike the accumulate-by-atomicAdd contract of Eq. 9-10).
 * By default M = 1 runs the bandwidth-bound split-K vector kernel, 2 <= M <= 32 a small-batch
 * MFMA kernel with the same split-K decomposition (when the format allows: no g_idx,
 * group_size % 128 == 0 or 64 / 32; otherwise the vector kernel up to M = 16), 33 <= M <= 64
 * (and 17-32 or 65-128 rows on the layer shapes where it measured faster) a mid-batch MFMA
 * kernel in which every wavefront streams its own share of the K slice (no g_idx, K and
 * group_size multiples of 64), larger M the big-tile fp16 MFMA kernel (with K slices where
 * the output tiles alone would not fill the chip).
 * Accumulation is in fp32; the result differs from the exact sum by fp32 reassociation
 * and the final fp16 rounding only.  The same inputs give bit-identical outputs on every
 * call (no floating point atomics are used).
 */
GPTQ_API int gptq_w4a16_gemm(const void *x, const void *qweight, const void *qzeros, const void *scales,
                    const void *g_idx, void *out, int M, int K, int N, int group_size,
                    gptq_stream_t stream);

/*
 * gptq_w4a16_gemm for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same operation, arguments, kernels, automatic plan and (bit-identical)
 * results as gptq_w4a16_gemm, but the split-K scratch (partial sums and arrival counters) is a fixed block of
 * GPTQ_STATIC_SCRATCH_BYTES inside the library's device image: every GPU the library runs on holds it until the
 * process ends, and the call makes no hipMalloc / hipFree and ignores gptq_w4a16_set_workspace().  A problem
 * whose plan needs more scratch returns GPTQ_STATIC_SCRATCH_EXCEEDED and enqueues nothing (needs are
 * 256 KiB + 4 * slices * M * N bytes where the plan splits K, which it does only while the output is small; the
 * largest need among the Llama-7B/70B layer shapes for M up to 2048 is 40.3 MiB, at 512 x 8192 x 10240).  The first call on a
 * device also enqueues one small kernel on `stream` that clears the arrival counters.  All calls on one GPU share
 * the block: calls that overlap in time on one GPU (different streams) race, as do a call here and a graph replay
 * that uses it.
 */
#define GPTQ_STATIC_SCRATCH_BYTES (48u << 20)
GPTQ_API int gptq_w4a16_gemm_static(const void *x, const void *qweight, const void *qzeros, const void *scales,
                                    const void *g_idx, void *out, int M, int K, int N, int group_size,
                                    gptq_stream_t stream);

/*
 * Launch plan for gptq_w4a16_gemm_plan(): selects the kernel and its decomposition
 * explicitly (for tuning sweeps).  A zero field means "let the library choose".
 */
#define GPTQ_ABLATE_SMB 1
#define GPTQ_ABLATE_VML 2
#define GPTQ_ABLATE_ILA 4
#define GPTQ_VECTOR_DOT 8

typedef struct gptq_w4a16_plan {
    int kernel;      /* 0 auto, 1 vector split-K kernel (any M, processed 16 rows at a time), 2 big-tile MFMA kernel,
                        3 small-batch MFMA kernel (M <= 128, processed 64 rows at a time; no g_idx,
                        group_size % 128 == 0; else falls back),
                        4 mid-batch streaming MFMA kernel (M <= 128; no g_idx, K % 64 == 0, group_size % 64 == 0;
                        else falls back) */
    int split_k;     /* number of K slices (all four kernels; the big-tile kernel splits by itself on every tile
                        but 256x256); 0 auto */
    int tile;        /* vector kernel: columns per workgroup (16, 32, 64, 128 or 256);
                        small-batch MFMA kernel: columns per workgroup (64, 128 - up to 32 rows - or 256; anything else = auto);
                        mid-batch MFMA kernel: columns per workgroup (64 or 128; anything else = auto; more than
                        64 rows always use 64);
                        MFMA kernel: tile id = rows x columns per workgroup (wavefront grid):
                        1 256x256 (1x4), 3 128x128 (2x2), 5 64x128 (1x4), 8 128x256 (1x4, two workgroups
                        per compute unit); 0 auto; any other id is GPTQ_INVALID_ARG */
    int flags;       /* 0, or (vector kernel only: M <= 4, no g_idx, group_size % 32 == 0, 64-column tiles) a set
                        of ablation switches that take one of the paper's techniques out each, for measuring its
                        gain in isolation (Table 3's columns at kernel level):
                        1 GPTQ_ABLATE_SMB  no on-chip reduction (Section 3.1): every lane adds its partial sums to
                                           memory with fp32 atomics (order of additions, hence the last bits,
                                           not reproducible), one extra launch zeroes the sums;
                        2 GPTQ_ABLATE_VML  activations staged with 16-bit instead of 128-bit loads (Section 3.2);
                        4 GPTQ_ABLATE_ILA  per-weight fp32 conversion and scalar multiply-add instead of packed
                                           half arithmetic (Section 3.3);
                        and one comparison switch without restrictions on the problem:
                        8 GPTQ_VECTOR_DOT  contract the packed codes with v_dot2_f32_f16 on the vector ALU instead
                                           of 4x4x4 MFMAs (the default up to four rows) */
    int reserved[4]; /* must be zero */
} gptq_w4a16_plan_t;

/* Same operation and contract as gptq_w4a16_gemm with an explicit plan (NULL = automatic). */
GPTQ_API int gptq_w4a16_gemm_plan(const void *x, const void *qweight, const void *qzeros, const void *scales,
                         const void *g_idx, void *out, int M, int K, int N, int group_size,
                         gptq_stream_t stream, const gptq_w4a16_plan_t *plan);

/*
 * One-time repack of an act-order checkpoint (the paper does not treat activation ordering; it is part of
 * the problem statement this library is built to: row k of the weight belongs to group g_idx[k], and the map
 * is fixed once the checkpoint is loaded).
 * Writes perm int32[K] (device) = the stable order of k by g_idx[k], and qweight_sorted int32[K/8, N]
 * (device, same packing as qweight, must not alias it) whose row j is row perm[j] of qweight, so that
 * row j belongs to group j / group_size like a checkpoint without g_idx.  qzeros and scales are used
 * unchanged afterwards.  Requires every group to own exactly group_size rows (what the quantiser
 * produces): otherwise GPTQ_UNSUPPORTED_SHAPE; an entry of g_idx outside [0, K/group_size) gives
 * GPTQ_INVALID_ARG; in both cases the outputs are undefined.  Blocks until the work on `stream` is
 * done (it reads a status word back) and allocates a few bytes of device memory meanwhile.
 */
GPTQ_API int gptq_w4a16_act_order_prepare(const void *qweight, const void *g_idx, void *qweight_sorted, void *perm,
                                          int K, int N, int group_size, gptq_stream_t stream);

/*
 * The act-order GEMM on a repacked checkpoint:  out[m, n] = sum_j x[m, perm[j]] * W_sorted[j, n],
 * equal (up to the order of the fp32 additions) to gptq_w4a16_gemm with the original qweight and
 * g_idx.  At M = 1 the vector kernel gathers x through perm while it stages it (one launch; perm
 * entries outside [0, K) read x[K-1]); for larger M x is first gathered into scratch (M*K fp16) and
 * the kernels of the plain format run on it; otherwise the contract of gptq_w4a16_gemm.  A caller-owned workspace must hold
 * gptq_w4a16_workspace_bytes(M, K, N, group_size) + 256 + 2*M*K bytes.
 */
GPTQ_API int gptq_w4a16_gemm_prepared(const void *x, const void *qweight_sorted, const void *qzeros,
                                      const void *scales, const void *perm, void *out, int M, int K, int N,
                                      int group_size, gptq_stream_t stream);

/*
 * Host-only: what gptq_w4a16_gemm_plan(..., request) would run for a problem of this shape.
 * `act_order` non-zero means a g_idx array would be passed; `request` may be NULL (automatic).
 * On success *resolved holds the kernel id (1 to 4, never 0), its number of K slices and its tile
 * (vector, small-batch and mid-batch kernels: columns per workgroup; big-tile MFMA kernel: tile id).  Touches no
 * device.  Errors as for gptq_w4a16_gemm_plan's shape and plan checks.
 */
GPTQ_API int gptq_w4a16_plan_query(int M, int K, int N, int group_size, int act_order,
                                   const gptq_w4a16_plan_t *request, gptq_w4a16_plan_t *resolved);

/*
 * The dequantised weights themselves: w_out (fp16 [K, N], device) = W as defined above,
 * computed as the exact integer difference q - z followed by ONE IEEE fp16 multiplication
 * by the scale (round to nearest even, subnormals kept).  Bit-exact by definition.
 */
GPTQ_API int gptq_w4a16_dequant(const void *qweight, const void *qzeros, const void *scales, const void *g_idx,
                       void *w_out, int K, int N, int group_size, gptq_stream_t stream);

/*
 * Format conversion, one-time: qzeros_out (int32 [K/group_size, N/8], device; may be qzeros_in) holds
 * (z + delta) mod 16 for every zero point of qzeros_in.  delta = +1 turns a checkpoint that stores z - 1
 * (the reading in which a stored 15 stands for z = 0) into the format of this header.
 */
GPTQ_API int gptq_w4a16_shift_zeros(const void *qzeros_in, void *qzeros_out, int delta, int K, int N,
                                    int group_size, gptq_stream_t stream);

/*
 * The unpacked 4-bit fields: q_out (uint8 [K, N], device) = q; z_out (uint8 [K/group_size, N],
 * device, may be NULL to skip) = z.  Integer work, bit-exact.
 */
GPTQ_API int gptq_w4a16_unpack(const void *qweight, void *q_out, const void *qzeros, void *z_out, int K, int N,
                      int group_size, gptq_stream_t stream);

/*
 * Split-K scratch.  gptq_w4a16_gemm needs device scratch for the partial sums of the K
 * slices and one arrival counter per column tile.  gptq_w4a16_workspace_bytes() is an
 * upper bound for a given problem under the automatic plan, with or without g_idx (0 for invalid
 * shapes); an explicit plan that needs more fails with GPTQ_WORKSPACE_TOO_SMALL on a caller-owned
 * workspace.  If the caller never sets a workspace the library allocates one with hipMalloc on
 * first use and replaces it by a larger one when a problem needs more (the only allocations it makes
 * besides the status word of gptq_w4a16_act_order_prepare).  An outgrown block is retired, not freed:
 * launches in flight and HIP graphs captured earlier keep working on it, so later growth never invalidates a
 * captured graph.  Growth is refused (GPTQ_WORKSPACE_TOO_SMALL, nothing enqueued) while `stream` is being
 * captured, since it allocates and clears memory: make one eager call of every problem a graph will hold
 * before capturing it, or use gptq_w4a16_gemm_static.  A graph replay and an eager call that use different
 * blocks do not share arrival counters; two pieces of work that share one block must not overlap in time.
 * gptq_w4a16_set_workspace() hands over caller-owned device memory (256-byte aligned, at least
 * gptq_w4a16_workspace_bytes() of the problems it will serve) instead; it synchronises the device, frees
 * every library-owned block (current and retired: graphs captured on them must not be replayed afterwards)
 * and clears the new memory with a synchronous hipMemset.  Passing NULL returns to library-owned scratch.
 * There is one workspace per device (the current one when the call is made): calls that overlap in time on
 * different streams of one device race on it.
 */
GPTQ_API size_t gptq_w4a16_workspace_bytes(int M, int K, int N, int group_size);
GPTQ_API int gptq_w4a16_set_workspace(void *dev_ptr, size_t bytes);

/*
 * Measurement aids (no part of the method; bench.py reports them as context for the roofline fractions).
 * gptq_w4a16_stream_probe: a plain read kernel over buf[0, bytes) (device, 16-byte aligned; bytes rounded down to
 * 16) with 128-bit loads on 256 workgroups - what any kernel of a GEMV's footprint pays for launch, first-byte
 * latency and ramp.  sink: at least 256 bytes of device memory that receive a few checksum words.
 * gptq_w4a16_mfma_probe: `iters` rounds of sixteen independent v_mfma_f32_32x32x16_f16 per wavefront on 512
 * workgroups, register operands read once from operands[0, bytes) (device fp16 values, caller's choice: the
 * sustained rate depends on how much the operands toggle); *flops (host, may be NULL) receives the floating
 * point operations of the launch.  Both only enqueue; errors as everywhere.
 */
GPTQ_API int gptq_w4a16_stream_probe(const void *buf, size_t bytes, void *sink, gptq_stream_t stream);
GPTQ_API int gptq_w4a16_mfma_probe(const void *operands, size_t bytes, void *sink, int iters, double *flops,
                                   gptq_stream_t stream);

/*
 * gptq_w4a16_issue_probe: on every compute unit, one after the other, four workgroups of 4 * waves_per_simd
 * wavefronts (waves_per_simd = 1, 2 or 4) run `iters` x 4 groups of one v_mfma_f32_32x32x16_f16 followed by
 * valu_per_mfma (0, 2, 4, 6, 8, 12 or 16) independent packed-fp16 vector instructions, on register operands read
 * once from `operands` (device, 16-byte aligned, `bytes` long; random fp16 values are the representative case).
 * *mfma_per_simd (host, may be NULL) receives the number of MFMAs each SIMD executes, so that the caller's own
 * timing gives the time per MFMA per SIMD: what vector work beside an MFMA costs on this chip.  `sink`: device,
 * >= 4 bytes, 16-byte aligned, written at most once.  Errors: GPTQ_INVALID_ARG (null pointer, iters outside
 * [1, 2^20], a count not listed), GPTQ_MISALIGNED, GPTQ_HIP_ERROR.
 */
GPTQ_API int gptq_w4a16_issue_probe(const void *operands, size_t bytes, void *sink, int iters, int valu_per_mfma,
                                    int waves_per_simd, double *mfma_per_simd, gptq_stream_t stream);

/* Text for a status code (static storage). */
GPTQ_API const char *gptq_w4a16_strerror(int code);

/* Library version: major * 10000 + minor * 100 + patch. */
GPTQ_API int gptq_w4a16_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GPTQ_W4A16_H */

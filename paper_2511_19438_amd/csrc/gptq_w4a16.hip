// C-ABI entry points of the W4A16 GPTQ library: argument validation, kernel choice, scratch.
// The contract of every function is stated in include/gptq_w4a16.h.
#include "gptq_w4a16.h"

#include <mutex>
#include <vector>

#include "kernels.h"

namespace {

using namespace gptq;

constexpr int kVersion = 100;  // 0.1.0
constexpr int kMaxDevices = 16;
constexpr int kDecodeMaxM = 16;

struct Workspace {
    void *ptr = nullptr;
    size_t bytes = 0;
    bool owned = false;
};

std::mutex g_mutex;
Workspace g_ws[kMaxDevices];
std::vector<void *> g_retired[kMaxDevices];  // outgrown library-owned blocks, still referenced by earlier work

// Scratch of gptq_w4a16_gemm_static(): a fixed block in every device's copy of the code object, for callers
// that may not allocate.  The array's name is only a host-side handle; its device address is looked up once
// per device (static_scratch_ptr) and that pointer is what kernels and fills receive.
constexpr size_t kStaticScratchBytes = GPTQ_STATIC_SCRATCH_BYTES;
void *g_static_ptr[kMaxDevices] = {};

}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

__global__ void clear_words_kernel(unsigned *p, unsigned n)
{
    const unsigned i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n)
        p[i] = 0u;
}

// Device address of the current device's static scratch.  The first call on a device looks the address up and
// clears the arrival counters at its front with a small kernel on `stream` (a kernel, not a memset: the call
// may be under stream capture).  No allocation.
int static_scratch_ptr(hipStream_t stream, void **out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return GPTQ_HIP_ERROR;
    std::lock_guard<std::mutex> lock(g_mutex);
    if (!g_static_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr)
            return GPTQ_HIP_ERROR;
        const unsigned words = (unsigned)(decode_counter_bytes(0) / sizeof(unsigned));
        hipLaunchKernelGGL(clear_words_kernel, dim3((words + 255) / 256), dim3(256), 0, stream,
                           static_cast<unsigned *>(ptr), words);
        if (hipGetLastError() != hipSuccess)
            return GPTQ_HIP_ERROR;
        g_static_ptr[dev] = ptr;
    }
    *out = g_static_ptr[dev];
    return GPTQ_OK;
}

bool aligned16(const void *p)
{
    return (reinterpret_cast<uintptr_t>(p) & 15u) == 0;
}

int check_shape(int K, int N, int group_size)
{
    if (K <= 0 || N <= 0 || group_size <= 0)
        return GPTQ_INVALID_ARG;
    if (K % 8 || N % 8 || group_size % 8 || K % group_size)
        return GPTQ_UNSUPPORTED_SHAPE;
    // The kernels address with 32-bit byte offsets from 64-bit bases: the packed weights (K*N/2 bytes) must
    // stay under 4 GiB, a tile's rows of x (256 * K * 2 bytes) too, and row / column numbers under 2^24
    // (24-bit multiplies).  Real layers are three orders of magnitude below these limits.
    if (K >= (1 << 23) || N >= (1 << 24) || (long long)K * N >= (1LL << 33))
        return GPTQ_UNSUPPORTED_SHAPE;
    return GPTQ_OK;
}

// Makes sure the current device has scratch of at least `bytes`; returns it in *out.
//
// Library-owned scratch only ever grows, and a block that has been handed to a launch is never freed while the
// library keeps its own scratch: launches still in flight and HIP graphs captured earlier hold its address (partial
// sums, arrival counters, gathered activations).  A block that became too small is retired instead and stays
// valid; retired blocks are released by gptq_w4a16_set_workspace().  Growth allocates and clears memory, which is
// not allowed while `stream` is being captured: such a call is refused.
int acquire_workspace(size_t bytes, hipStream_t stream, void **out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return GPTQ_HIP_ERROR;
    std::lock_guard<std::mutex> lock(g_mutex);
    Workspace &ws = g_ws[dev];
    if (ws.ptr && ws.bytes >= bytes) {
        *out = ws.ptr;
        return GPTQ_OK;
    }
    if (ws.ptr && !ws.owned)
        return GPTQ_WORKSPACE_TOO_SMALL;
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &capturing) != hipSuccess) {
        (void)hipGetLastError();
        return GPTQ_HIP_ERROR;
    }
    if (capturing != hipStreamCaptureStatusNone)
        return GPTQ_WORKSPACE_TOO_SMALL;
    size_t want = bytes + bytes / 2;
    if (want < (size_t)(8u << 20))
        want = (size_t)(8u << 20);
    void *p = nullptr;
    if (hipMalloc(&p, want) != hipSuccess)
        return GPTQ_HIP_ERROR;
    // the arrival counters live at the front and must start at zero; clear everything once
    if (hipMemset(p, 0, want) != hipSuccess) {
        (void)hipFree(p);
        return GPTQ_HIP_ERROR;
    }
    if (ws.ptr)
        g_retired[dev].push_back(ws.ptr);
    ws.ptr = p;
    ws.bytes = want;
    ws.owned = true;
    *out = p;
    return GPTQ_OK;
}

// Default kernel by batch size, from measurement on Llama-shaped layers.  A single row is streamed fastest
// by the vector kernel.  From two rows on the small-batch MFMA kernel wins: its time is nearly flat up to 16
// rows and grows slowly to 32, where the vector kernel pays for every weight once per batch row.  From 33 to
// 64 rows the mid-batch streaming kernel is the fastest on every Llama shape measured (10-40 % ahead of the
// big-tile kernel with K slices); it also takes 17-32 rows on wide or very deep layers (3-17 % ahead of the
// small-batch kernel, 2-12 % behind it on narrow ones) and 65-128 rows where its 64-column tiles give between half
// and all of the compute units one workgroup each, or K is deep (1-24 % ahead of the big-tile kernel; 3-18 %
// behind it on 4096x4096 and on layers whose tiles make a second, partly filled round).
constexpr int kVectorMaxM = 1;
constexpr int kSmallBatchAutoMaxM = 32;

bool small_batch_by_default(const Problem &p)
{
    if (!skinny_supported(p))
        return false;
    return p.M <= kSmallBatchAutoMaxM;
}

bool mid_batch_by_default(const Problem &p)
{
    if (!mid_supported(p) || p.M <= 16)
        return false;
    const long long tiles64 = (p.N + 63) / 64;
    if (p.M <= 32)
        return tiles64 >= 160 || (long long)p.K * p.N >= (1ll << 27);
    if (p.M <= 64)
        return true;
    return tiles64 <= 256 && (tiles64 >= 128 || p.K >= 8192);
}

// What a call resolves to: the kernel and its decomposition, after the automatic choices.
struct Resolved {
    int kernel;  // 1 vector, 2 big-tile MFMA, 3 small-batch MFMA, 4 mid-batch streaming MFMA
    DecodePlan decode;
    SkinnyPlan skinny;
    MidPlan mid;
    PrefillPlan prefill;
};

Resolved resolve(const Problem &p, const gptq_w4a16_plan_t *plan)
{
    Resolved r = {};
    int kernel = plan ? plan->kernel : 0;
    if (kernel == 0) {
        if (p.M <= kVectorMaxM)
            kernel = 1;
        else if (mid_batch_by_default(p))
            kernel = 4;
        else if (small_batch_by_default(p))
            kernel = 3;
        else
            kernel = (p.M <= kDecodeMaxM) ? 1 : 2;
    }
    if (kernel == 3 && !skinny_supported(p))
        kernel = (p.M <= kDecodeMaxM) ? 1 : 2;
    if (kernel == 4 && !mid_supported(p))
        kernel = (p.M <= kDecodeMaxM) ? 1 : 2;
    if (kernel == 2 && !prefill_supported(p))
        kernel = 1;
    r.kernel = kernel;
    if (kernel == 1) {
        r.decode.cols_per_wg = plan ? plan->tile : 0;
        r.decode.split_k = plan ? plan->split_k : 0;
        r.decode.flags = plan ? plan->flags : 0;
        decode_make_plan(p, r.decode);
        if (!decode_plan_fits(p, r.decode)) {
            // the big-tile kernel's general path takes any format at any M
            r.kernel = kernel = 2;
            r.prefill.tile = 0;
            r.prefill.split_k = 0;
            prefill_make_plan(p, r.prefill);
        }
    } else if (kernel == 3) {
        r.skinny.cols_per_wg = plan ? plan->tile : 0;
        r.skinny.split_k = plan ? plan->split_k : 0;
        skinny_make_plan(p, r.skinny);
    } else if (kernel == 4) {
        r.mid.cols_per_wg = plan ? plan->tile : 0;
        r.mid.split_k = plan ? plan->split_k : 0;
        mid_make_plan(p, r.mid);
    } else {
        r.prefill.tile = plan ? plan->tile : 0;
        r.prefill.split_k = plan ? plan->split_k : 0;
        prefill_make_plan(p, r.prefill);
    }
    return r;
}

size_t scratch_bytes(const Problem &p, const Resolved &r)
{
    if (r.kernel == 1)
        return decode_workspace_bytes(p, r.decode);
    if (r.kernel == 3)
        return skinny_workspace_bytes(p, r.skinny);
    if (r.kernel == 4)
        return mid_workspace_bytes(p, r.mid);
    return prefill_workspace_bytes(p, r.prefill);  // 0 unless K is split
}

int launch_resolved(const Problem &p, const Resolved &r, void *ws, hipStream_t stream)
{
    hipError_t err;
    if (r.kernel == 1)
        err = launch_decode(p, r.decode, ws, stream);
    else if (r.kernel == 3)
        err = launch_skinny(p, r.skinny, ws, stream);
    else if (r.kernel == 4)
        err = launch_mid(p, r.mid, ws, stream);
    else
        err = launch_prefill(p, r.prefill, ws, stream);
    return err == hipSuccess ? GPTQ_OK : GPTQ_HIP_ERROR;
}

int run_gemm(const Problem &p, hipStream_t stream, const gptq_w4a16_plan_t *plan)
{
    const Resolved r = resolve(p, plan);
    void *ws = nullptr;
    const size_t bytes = scratch_bytes(p, r);
    if (bytes > 0) {
        const int rc = acquire_workspace(bytes, stream, &ws);
        if (rc != GPTQ_OK)
            return rc;
    }
    return launch_resolved(p, r, ws, stream);
}

size_t align256(size_t v)
{
    return (v + 255) & ~(size_t)255;
}

int check_plan(const gptq_w4a16_plan_t *plan)
{
    if (!plan)
        return GPTQ_OK;
    if (plan->kernel < 0 || plan->kernel > 4 || plan->split_k < 0 || plan->tile < 0)
        return GPTQ_INVALID_ARG;
    // the ablation switches belong to the vector kernel
    if (plan->flags < 0 || plan->flags > 15 || (plan->flags != 0 && plan->kernel != 1))
        return GPTQ_INVALID_ARG;
    if (plan->kernel == 2 && plan->tile != 0 && !prefill_tile_exists(plan->tile))
        return GPTQ_INVALID_ARG;
    for (int i = 0; i < 4; ++i)
        if (plan->reserved[i] != 0)
            return GPTQ_INVALID_ARG;
    return GPTQ_OK;
}

// Validates the arguments of a GEMM call and fills `p`.
int make_problem(const void *x, const void *qweight, const void *qzeros, const void *scales, const void *g_idx,
                 void *out, int M, int K, int N, int group_size, const gptq_w4a16_plan_t *plan, Problem &p)
{
    if (!x || !qweight || !qzeros || !scales || !out || M <= 0)
        return GPTQ_INVALID_ARG;
    const int rc = check_shape(K, N, group_size);
    if (rc != GPTQ_OK)
        return rc;
    if (check_plan(plan) != GPTQ_OK)
        return GPTQ_INVALID_ARG;
    if (!aligned16(x) || !aligned16(qweight) || !aligned16(qzeros) || !aligned16(scales) || !aligned16(out) ||
        (g_idx && !aligned16(g_idx)))
        return GPTQ_MISALIGNED;
    p.x = static_cast<const half_t *>(x);
    p.qweight = static_cast<const uint32_t *>(qweight);
    p.qzeros = static_cast<const uint32_t *>(qzeros);
    p.scales = static_cast<const half_t *>(scales);
    p.g_idx = static_cast<const int32_t *>(g_idx);
    p.out = static_cast<half_t *>(out);
    p.M = M;
    p.K = K;
    p.N = N;
    p.group_size = group_size;
    if (plan && (plan->flags & 7) != 0 && !decode_ablation_supported(p))
        return GPTQ_UNSUPPORTED_SHAPE;
    return GPTQ_OK;
}

}  // namespace

extern "C" {

int gptq_w4a16_gemm_plan(const void *x, const void *qweight, const void *qzeros, const void *scales,
                         const void *g_idx, void *out, int M, int K, int N, int group_size,
                         gptq_stream_t stream, const gptq_w4a16_plan_t *plan)
{
    Problem p;
    const int rc = make_problem(x, qweight, qzeros, scales, g_idx, out, M, K, N, group_size, plan, p);
    if (rc != GPTQ_OK)
        return rc;
    return run_gemm(p, static_cast<hipStream_t>(stream), plan);
}

int gptq_w4a16_gemm_static(const void *x, const void *qweight, const void *qzeros, const void *scales,
                           const void *g_idx, void *out, int M, int K, int N, int group_size,
                           gptq_stream_t stream)
{
    Problem p;
    const int rc = make_problem(x, qweight, qzeros, scales, g_idx, out, M, K, N, group_size, nullptr, p);
    if (rc != GPTQ_OK)
        return rc;
    const Resolved r = resolve(p, nullptr);
    if (scratch_bytes(p, r) > kStaticScratchBytes)
        return GPTQ_STATIC_SCRATCH_EXCEEDED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    void *ws = nullptr;
    const int wrc = static_scratch_ptr(st, &ws);
    if (wrc != GPTQ_OK)
        return wrc;
    return launch_resolved(p, r, ws, st);
}

int gptq_w4a16_gemm(const void *x, const void *qweight, const void *qzeros, const void *scales,
                    const void *g_idx, void *out, int M, int K, int N, int group_size, gptq_stream_t stream)
{
    return gptq_w4a16_gemm_plan(x, qweight, qzeros, scales, g_idx, out, M, K, N, group_size, stream, nullptr);
}

int gptq_w4a16_plan_query(int M, int K, int N, int group_size, int act_order, const gptq_w4a16_plan_t *request,
                          gptq_w4a16_plan_t *resolved)
{
    if (!resolved || M <= 0)
        return GPTQ_INVALID_ARG;
    const int rc = check_shape(K, N, group_size);
    if (rc != GPTQ_OK)
        return rc;
    if (check_plan(request) != GPTQ_OK)
        return GPTQ_INVALID_ARG;
    static const int32_t some_g_idx = 0;  // only its presence matters to the plan
    Problem p = {};
    p.g_idx = act_order ? &some_g_idx : nullptr;
    p.M = M;
    p.K = K;
    p.N = N;
    p.group_size = group_size;
    if (request && (request->flags & 7) != 0 && !decode_ablation_supported(p))
        return GPTQ_UNSUPPORTED_SHAPE;
    const Resolved r = resolve(p, request);
    gptq_w4a16_plan_t out = {};
    out.kernel = r.kernel;
    if (r.kernel == 1) {
        out.split_k = r.decode.split_k;
        out.tile = r.decode.cols_per_wg;
        out.flags = r.decode.flags;
    } else if (r.kernel == 3) {
        out.split_k = r.skinny.split_k;
        out.tile = r.skinny.cols_per_wg;
    } else if (r.kernel == 4) {
        out.split_k = r.mid.split_k;
        out.tile = r.mid.cols_per_wg;
    } else {
        out.split_k = r.prefill.split_k;
        out.tile = r.prefill.tile;
    }
    *resolved = out;
    return GPTQ_OK;
}

int gptq_w4a16_act_order_prepare(const void *qweight, const void *g_idx, void *qweight_sorted, void *perm, int K,
                                 int N, int group_size, gptq_stream_t stream)
{
    if (!qweight || !g_idx || !qweight_sorted || !perm)
        return GPTQ_INVALID_ARG;
    const int rc = check_shape(K, N, group_size);
    if (rc != GPTQ_OK)
        return rc;
    if (!aligned16(qweight) || !aligned16(g_idx) || !aligned16(qweight_sorted) || !aligned16(perm))
        return GPTQ_MISALIGNED;
    if (qweight == qweight_sorted)
        return GPTQ_INVALID_ARG;  // the gather is not in place
    hipStream_t st = static_cast<hipStream_t>(stream);
    int *status = nullptr;
    if (hipMalloc(reinterpret_cast<void **>(&status), sizeof(int)) != hipSuccess)
        return GPTQ_HIP_ERROR;
    int host_status = 0;
    bool ok = hipMemsetAsync(status, 0, sizeof(int), st) == hipSuccess;
    ok = ok && launch_rank_rows(static_cast<const int32_t *>(g_idx), static_cast<int32_t *>(perm), K, group_size,
                                status, st) == hipSuccess;
    ok = ok && hipMemcpyAsync(&host_status, status, sizeof(int), hipMemcpyDeviceToHost, st) == hipSuccess;
    ok = ok && hipStreamSynchronize(st) == hipSuccess;
    (void)hipFree(status);
    if (!ok)
        return GPTQ_HIP_ERROR;
    if (host_status & 1)
        return GPTQ_INVALID_ARG;  // g_idx entry outside [0, K / group_size)
    if (host_status & 2)
        return GPTQ_UNSUPPORTED_SHAPE;  // a group owns more (so another fewer) than group_size rows
    if (launch_sort_rows(static_cast<const uint32_t *>(qweight), static_cast<const int32_t *>(perm),
                         static_cast<uint32_t *>(qweight_sorted), K, N, st) != hipSuccess)
        return GPTQ_HIP_ERROR;
    return hipStreamSynchronize(st) == hipSuccess ? GPTQ_OK : GPTQ_HIP_ERROR;
}

int gptq_w4a16_gemm_prepared(const void *x, const void *qweight_sorted, const void *qzeros, const void *scales,
                             const void *perm, void *out, int M, int K, int N, int group_size,
                             gptq_stream_t stream)
{
    if (!x || !qweight_sorted || !qzeros || !scales || !perm || !out || M <= 0)
        return GPTQ_INVALID_ARG;
    const int rc = check_shape(K, N, group_size);
    if (rc != GPTQ_OK)
        return rc;
    if (!aligned16(x) || !aligned16(qweight_sorted) || !aligned16(qzeros) || !aligned16(scales) || !aligned16(out) ||
        !aligned16(perm))
        return GPTQ_MISALIGNED;
    Problem p;
    p.x = nullptr;  // the gathered copy, below
    p.qweight = static_cast<const uint32_t *>(qweight_sorted);
    p.qzeros = static_cast<const uint32_t *>(qzeros);
    p.scales = static_cast<const half_t *>(scales);
    p.g_idx = nullptr;
    p.out = static_cast<half_t *>(out);
    p.M = M;
    p.K = K;
    p.N = N;
    p.group_size = group_size;
    const Resolved r = resolve(p, nullptr);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (r.kernel == 1 && M == 1 && r.decode.chunk_rows == 4 && r.decode.flags == 0) {
        // the vector kernel gathers the activations itself while it stages them: one launch
        p.x = static_cast<const half_t *>(x);
        p.x_perm = static_cast<const int32_t *>(perm);
        void *ws = nullptr;
        const size_t bytes = scratch_bytes(p, r);
        if (bytes > 0) {
            const int wrc = acquire_workspace(bytes, st, &ws);
            if (wrc != GPTQ_OK)
                return wrc;
        }
        return launch_resolved(p, r, ws, st);
    }
    // scratch: what the kernel needs, then the gathered activations
    // (the counter area at the front stays reserved even if this launch needs none: it must remain zero)
    size_t kernel_bytes = align256(scratch_bytes(p, r));
    if (kernel_bytes < decode_counter_bytes(N))
        kernel_bytes = decode_counter_bytes(N);
    void *ws = nullptr;
    const int wrc = acquire_workspace(kernel_bytes + (size_t)M * K * sizeof(half_t), st, &ws);
    if (wrc != GPTQ_OK)
        return wrc;
    half_t *xp = reinterpret_cast<half_t *>(static_cast<unsigned char *>(ws) + kernel_bytes);
    if (launch_gather_activations(static_cast<const half_t *>(x), static_cast<const int32_t *>(perm), xp, M, K, st) !=
        hipSuccess)
        return GPTQ_HIP_ERROR;
    p.x = xp;
    return launch_resolved(p, r, ws, st);
}

int gptq_w4a16_shift_zeros(const void *qzeros_in, void *qzeros_out, int delta, int K, int N, int group_size,
                           gptq_stream_t stream)
{
    if (!qzeros_in || !qzeros_out)
        return GPTQ_INVALID_ARG;
    const int rc = check_shape(K, N, group_size);
    if (rc != GPTQ_OK)
        return rc;
    if (!aligned16(qzeros_in) || !aligned16(qzeros_out))
        return GPTQ_MISALIGNED;
    const long long words = (long long)(K / group_size) * (N / 8);
    const hipError_t err = launch_shift_zeros(static_cast<const uint32_t *>(qzeros_in),
                                              static_cast<uint32_t *>(qzeros_out), words, ((delta % 16) + 16) % 16,
                                              static_cast<hipStream_t>(stream));
    return err == hipSuccess ? GPTQ_OK : GPTQ_HIP_ERROR;
}

int gptq_w4a16_dequant(const void *qweight, const void *qzeros, const void *scales, const void *g_idx,
                       void *w_out, int K, int N, int group_size, gptq_stream_t stream)
{
    if (!qweight || !qzeros || !scales || !w_out)
        return GPTQ_INVALID_ARG;
    const int rc = check_shape(K, N, group_size);
    if (rc != GPTQ_OK)
        return rc;
    if (!aligned16(qweight) || !aligned16(qzeros) || !aligned16(scales) || !aligned16(w_out) ||
        (g_idx && !aligned16(g_idx)))
        return GPTQ_MISALIGNED;
    const hipError_t err = launch_dequant(static_cast<const uint32_t *>(qweight), static_cast<const uint32_t *>(qzeros),
                                          static_cast<const half_t *>(scales), static_cast<const int32_t *>(g_idx),
                                          static_cast<half_t *>(w_out), K, N, group_size,
                                          static_cast<hipStream_t>(stream));
    return err == hipSuccess ? GPTQ_OK : GPTQ_HIP_ERROR;
}

int gptq_w4a16_unpack(const void *qweight, void *q_out, const void *qzeros, void *z_out, int K, int N,
                      int group_size, gptq_stream_t stream)
{
    if (!qweight || !q_out || (z_out && !qzeros))
        return GPTQ_INVALID_ARG;
    const int rc = check_shape(K, N, group_size);
    if (rc != GPTQ_OK)
        return rc;
    if (!aligned16(qweight) || !aligned16(q_out) || (z_out && (!aligned16(qzeros) || !aligned16(z_out))))
        return GPTQ_MISALIGNED;
    const hipError_t err =
        launch_unpack(static_cast<const uint32_t *>(qweight), static_cast<uint8_t *>(q_out),
                      static_cast<const uint32_t *>(qzeros), static_cast<uint8_t *>(z_out), K, N, group_size,
                      static_cast<hipStream_t>(stream));
    return err == hipSuccess ? GPTQ_OK : GPTQ_HIP_ERROR;
}

size_t gptq_w4a16_workspace_bytes(int M, int K, int N, int group_size)
{
    if (M <= 0 || check_shape(K, N, group_size) != GPTQ_OK)
        return 0;
    // The automatic plan never uses more slices than this bound; explicit plans are checked at launch.
    Problem p = {};
    p.M = M;
    p.K = K;
    p.N = N;
    p.group_size = group_size;
    DecodePlan dp = {};
    decode_make_plan(p, dp);
    size_t bytes = decode_workspace_bytes(p, dp);
    // act-order problems may be planned with a different slice count
    int dummy = 0;
    p.g_idx = &dummy;
    DecodePlan da = {};
    decode_make_plan(p, da);
    const size_t act = decode_workspace_bytes(p, da);
    if (act > bytes)
        bytes = act;
    p.g_idx = nullptr;
    if (skinny_supported(p)) {
        SkinnyPlan sp = {};
        skinny_make_plan(p, sp);
        const size_t sk = skinny_workspace_bytes(p, sp);
        if (sk > bytes)
            bytes = sk;
    }
    // the big-tile and mid-batch kernels split K on few-tile shapes; counted where the default dispatch picks them
    for (int act = 0; act < 2; ++act) {
        p.g_idx = act ? &dummy : nullptr;
        const Resolved r = resolve(p, nullptr);
        if (r.kernel == 2 || r.kernel == 4) {
            const size_t pf = scratch_bytes(p, r);
            if (pf > bytes)
                bytes = pf;
        }
    }
    return bytes;
}

int gptq_w4a16_set_workspace(void *dev_ptr, size_t bytes)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return GPTQ_HIP_ERROR;
    if (dev_ptr && (reinterpret_cast<uintptr_t>(dev_ptr) & 255u) != 0)
        return GPTQ_MISALIGNED;
    if (dev_ptr && bytes < decode_counter_bytes(0))
        return GPTQ_WORKSPACE_TOO_SMALL;  // not even room for the arrival counters
    std::lock_guard<std::mutex> lock(g_mutex);
    Workspace &ws = g_ws[dev];
    // the library's own blocks, current and retired, go now: drain the device first
    if ((ws.ptr && ws.owned) || !g_retired[dev].empty()) {
        if (hipDeviceSynchronize() != hipSuccess)
            return GPTQ_HIP_ERROR;
        if (ws.ptr && ws.owned)
            (void)hipFree(ws.ptr);
        for (void *old : g_retired[dev])
            (void)hipFree(old);
        g_retired[dev].clear();
    }
    ws = Workspace();
    if (dev_ptr) {
        if (hipDeviceSynchronize() != hipSuccess)
            return GPTQ_HIP_ERROR;
        if (hipMemset(dev_ptr, 0, bytes) != hipSuccess)
            return GPTQ_HIP_ERROR;
        ws.ptr = dev_ptr;
        ws.bytes = bytes;
        ws.owned = false;
    }
    return GPTQ_OK;
}

const char *gptq_w4a16_strerror(int code)
{
    switch (code) {
    case GPTQ_OK: return "ok";
    case GPTQ_INVALID_ARG: return "invalid argument (null pointer, non-positive size or bad plan)";
    case GPTQ_UNSUPPORTED_SHAPE: return "unsupported shape (K, N, group_size must be multiples of 8; group_size must divide K)";
    case GPTQ_MISALIGNED: return "a base pointer is not 16-byte aligned";
    case GPTQ_HIP_ERROR: return "a HIP call or kernel launch failed";
    case GPTQ_WORKSPACE_TOO_SMALL: return "caller-set workspace is too small for this problem";
    case GPTQ_STATIC_SCRATCH_EXCEEDED:
        return "problem needs more split-K scratch than the 48 MiB static block of gptq_w4a16_gemm_static";
    default: return "unknown status code";
    }
}

int gptq_w4a16_version(void)
{
    return kVersion;
}

}  // extern "C"

// Host side of the Stream-K GEMM: kernel table, workspace handling and the sk_gemm launcher.
#include <mutex>
#include "streamk_kernels.h"

using namespace streamk_detail;

namespace {

KernelEntry** kernel_table(int* count) {
    static KernelEntry* table[64];
    static int n = 0;
    static std::once_flag once;
    std::call_once(once, [] {
        register_bf16(table, &n);
        register_f16(table, &n);
        register_fp8(table, &n);
        register_bf16_atomic(table, &n);
        register_f16_atomic(table, &n);
        register_fp8_atomic(table, &n);
    });
    *count = n;
    return table;
}

// The kernel for a tile shape, input type and fix-up mode: the wanted variant if the shape has it,
// else the shape's variant 0.  want = 0 leaves the choice to the library: variant 0, except that a plan
// without split tiles (whole_tile_iters = its k-iterations per tile, 0 for plans with split tiles) gets
// the variant marked for such plans where the shape has one and the tiles are deep enough.
KernelEntry* find_kernel(int dtype, int bm, int bn, int bk, int fixup = SK_FIXUP_FLAGS, int want = 0, int whole_tile_iters = 0) {
    int n;
    KernelEntry** t = kernel_table(&n);
    KernelEntry* fallback = nullptr;
    KernelEntry* exact = nullptr;
    for (int i = 0; i < n; i++)
        if (t[i]->dtype == dtype && t[i]->bm == bm && t[i]->bn == bn && t[i]->bk == bk && t[i]->fixup == fixup) {
            if (want == 0 && t[i]->whole_tiles_choice && whole_tile_iters >= t[i]->whole_tiles_choice) return t[i];
            if (t[i]->variant == want) exact = t[i];
            if (t[i]->variant == 0) fallback = t[i];
        }
    return exact ? exact : fallback;
}


// Helpers of the atomic fix-up: clear the fp32 image, and turn it into a 16-bit D afterwards.
__global__ void zero_image_kernel(float4* p, size_t n4, float* tail, int n_tail) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) p[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (blockIdx.x == 0 && (int)threadIdx.x < n_tail) tail[threadIdx.x] = 0.f;
}
template <int OUT> __global__ void convert_image_kernel(const float* src, void* dst, size_t n) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        if (OUT == SK_BF16) static_cast<u16*>(dst)[i] = to_bf16_bits(src[i]);
        else static_cast<_Float16*>(dst)[i] = (_Float16)src[i];
    }
}

thread_local hipError_t g_last_hip = hipSuccess;   // last failing HIP call of this thread
inline bool hip_ok(hipError_t e) {
    if (e != hipSuccess) g_last_hip = e;
    return e == hipSuccess;
}

}  // namespace

extern "C" const char* sk_last_hip_error(void) { return hipGetErrorString(g_last_hip); }

bool sk_kernel_available(int in_dtype, int blk_m, int blk_n, int blk_k) {
    return find_kernel(in_dtype, blk_m, blk_n, blk_k) != nullptr;
}

extern "C" int sk_plan_set_workspace(sk_plan_t* plan, void* dev_ptr, size_t bytes) {
    if (!plan || !dev_ptr) return SK_ERR_INVALID_ARG;
    if (bytes < sk_workspace_bytes(plan) || (reinterpret_cast<uintptr_t>(dev_ptr) & 255)) return SK_ERR_WORKSPACE;
    if (!hip_ok(hipMemset(dev_ptr, 0, sk_ws_partials_offset(plan->h.grid)))) return SK_ERR_HIP;
    if (!hip_ok(hipDeviceSynchronize())) return SK_ERR_HIP;
    plan->workspace = dev_ptr;
    plan->workspace_bytes = bytes;
    return SK_OK;
}

extern "C" int sk_plan_check(const sk_plan_t* plan, void* stream) {
    if (!plan) return SK_ERR_INVALID_ARG;
    if (!hip_ok(hipStreamSynchronize(static_cast<hipStream_t>(stream)))) return SK_ERR_HIP;
    if (!plan->workspace) return SK_OK;
    uint32_t* st = reinterpret_cast<uint32_t*>(static_cast<char*>(plan->workspace) + sk_ws_status_offset(plan->h.grid));
    uint32_t v = 0;
    if (!hip_ok(hipMemcpy(&v, st, sizeof v, hipMemcpyDeviceToHost))) return SK_ERR_HIP;
    if (v) {
        // flags of contributors that nobody waited for may still be up: take the whole flag and status area down
        if (!hip_ok(hipMemset(plan->workspace, 0, sk_ws_partials_offset(plan->h.grid)))) return SK_ERR_HIP;
        return SK_ERR_TIMEOUT;
    }
    return SK_OK;
}

extern "C" int sk_plan_kernel_info(const sk_plan_t* plan, int32_t* threads, int32_t* lds_bytes, int32_t* variant) {
    if (!plan) return SK_ERR_INVALID_ARG;
    const sk_plan_header& h = plan->h;
    const bool atomic = plan->fixup == SK_FIXUP_ATOMIC && plan->needs_fixup;
    const KernelEntry* e = find_kernel(h.in_dtype, h.blk_m, h.blk_n, h.blk_k, atomic ? SK_FIXUP_ATOMIC : SK_FIXUP_FLAGS, plan->kernel_variant, plan->needs_fixup ? 0 : plan->h.iters_per_tile);
    if (!e) return SK_ERR_UNSUPPORTED;
    if (threads) *threads = e->threads;
    if (lds_bytes) *lds_bytes = e->lds_bytes;
    if (variant) *variant = e->variant;
    return SK_OK;
}

namespace {

// The launch behind sk_gemm and sk_gemm_static: `workspace` is the device memory that holds the flag
// lines, the status line and the partial tiles (or the fp32 image of the atomic fix-up).
int launch_gemm(const void* A, const void* B, void* D, const sk_plan_t* plan, void* stream, void* workspace) {
    if (!A || !B || !D || !plan) return SK_ERR_INVALID_ARG;
    const sk_plan_header& h = plan->h;
    const uintptr_t align = reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B) | reinterpret_cast<uintptr_t>(D);
    if (align & 15) return SK_ERR_INVALID_ARG;
    // the kernels use 32-bit byte offsets into A and B, 32-bit element offsets into D and 32-bit iteration counts
    if (h.M * h.K >= (1ll << 31) || h.K * h.N >= (1ll << 31) || h.M * h.N >= (1ll << 32) || h.total_iters >= (1ll << 30))
        return SK_ERR_UNSUPPORTED;
    // plans without split tiles run the plain kernel under either fix-up mode
    const bool atomic = plan->fixup == SK_FIXUP_ATOMIC && plan->needs_fixup;
    KernelEntry* e = find_kernel(h.in_dtype, h.blk_m, h.blk_n, h.blk_k, atomic ? SK_FIXUP_ATOMIC : SK_FIXUP_FLAGS, plan->kernel_variant, plan->needs_fixup ? 0 : plan->h.iters_per_tile);
    if (!e) return SK_ERR_UNSUPPORTED;
    if (plan->needs_fixup && !workspace && !(atomic && h.out_dtype == SK_F32)) return SK_ERR_WORKSPACE;
    const bool aligned = (h.K % e->piece_elems == 0) && (h.N % e->piece_elems == 0);   // whole 16-byte pieces per row
    kernel_fn fn = aligned ? e->aligned : e->generic;

    if (e->max_resident.load() < 0) {
        // first use on this process: allow the large LDS footprint and ask how many workgroups fit at once
        for (kernel_fn f : {e->aligned, e->generic})
            if (!hip_ok(hipFuncSetAttribute(reinterpret_cast<const void*>(f), hipFuncAttributeMaxDynamicSharedMemorySize, e->lds_bytes)))
                return SK_ERR_HIP;
        int dev = 0, cus = 0, per_cu = 0;
        if (!hip_ok(hipGetDevice(&dev)) || !hip_ok(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)))
            return SK_ERR_HIP;
        if (!hip_ok(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(e->generic), e->threads, e->lds_bytes)))
            return SK_ERR_HIP;
        e->max_resident.store(per_cu * cus);
    }
    // an owner spins on flags of other workgroups: all of them must be on the machine at once
    if (plan->needs_fixup && !atomic && h.grid > e->max_resident.load()) return SK_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);

    GemmArgs g{};
    g.A = A; g.B = B; g.D = D;
    char* ws = static_cast<char*>(workspace);
    g.flags = reinterpret_cast<uint32_t*>(ws);
    g.status = ws ? reinterpret_cast<uint32_t*>(ws + sk_ws_status_offset(h.grid)) : nullptr;
    g.partials = ws ? reinterpret_cast<float*>(ws + sk_ws_partials_offset(h.grid)) : nullptr;
    g.M = (int)h.M; g.N = (int)h.N; g.K = (int)h.K;
    g.tiles_m = h.tiles_m; g.tiles_n = h.tiles_n; g.tiles = h.tiles; g.ipt = h.iters_per_tile; g.tile_order = h.tile_order;
    g.sk_tiles = h.sk_tiles; g.ipw = h.iters_per_wg; g.grid = h.grid; g.sk_iters = (int)h.sk_iters;
    g.spin_limit = plan->spin_limit;
    g.out_dtype = h.out_dtype;
    g.dp_first = plan->dp_first;
    g.k_aligned = plan->k_aligned;
    g.xcd_remap = h.xcd_remap;
    // B is requested non-temporally when it is read exactly once (one row of tiles) and is too large to be
    // found in the 256 MB memory-side cache by a later launch anyway (at least half of it: 128 MiB).  Measured:
    // 16 x 8192 x 8192 and 16 x 16384 x 4096 (128 MiB) 5 - 6 % faster, 16 x 4096 x 4096 and 32 x 8192 x 2048
    // (32 MiB, served by the caches from launch to launch) 10 - 25 % slower with the hint.
    g.stream_b = h.tiles_m == 1 && (size_t)h.K * (size_t)h.N * (h.in_dtype == SK_FP8_E4M3 ? 1 : 2) >= ((size_t)128 << 20);
    g.div_ipt = sk_make_fast_div((uint32_t)h.iters_per_tile);
    g.div_ipw = sk_make_fast_div((uint32_t)h.iters_per_wg);
    g.div_tiles_n = sk_make_fast_div((uint32_t)h.tiles_n);
    g.div_band = sk_make_fast_div((uint32_t)(SK_GROUP_ROWS * h.tiles_n));
    g.div_last_rows = sk_make_fast_div((uint32_t)(h.tiles_m % SK_GROUP_ROWS));
    if (atomic) {
        // Algorithm 1's atomic accumulation needs C to start at zero: clear the image in-stream, accumulate, convert
        const size_t n = (size_t)h.M * (size_t)h.N;
        g.image = h.out_dtype == SK_F32 ? static_cast<float*>(D) : g.partials;
        const int blocks = (int)((n / 4 + 255) / 256 < 2048 ? (n / 4 + 255) / 256 : 2048);
        hipLaunchKernelGGL(zero_image_kernel, dim3(blocks ? blocks : 1), dim3(256), 0, st,
                           reinterpret_cast<float4*>(g.image), n / 4, g.image + (n / 4) * 4, (int)(n % 4));
        hipLaunchKernelGGL(fn, dim3(h.grid), dim3(e->threads), e->lds_bytes, st, g);
        if (h.out_dtype != SK_F32) {
            const int cb = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
            if (h.out_dtype == SK_BF16) hipLaunchKernelGGL(convert_image_kernel<SK_BF16>, dim3(cb), dim3(256), 0, st, g.image, D, n);
            else hipLaunchKernelGGL(convert_image_kernel<SK_F16>, dim3(cb), dim3(256), 0, st, g.image, D, n);
        }
        return hip_ok(hipGetLastError()) ? SK_OK : SK_ERR_HIP;
    }
    hipLaunchKernelGGL(fn, dim3(h.grid), dim3(e->threads), e->lds_bytes, st, g);
    return hip_ok(hipGetLastError()) ? SK_OK : SK_ERR_HIP;
}

// ---- sk_gemm_static: the workspace lives in the library's own device image ---------------------
// `scratch` is the workspace of every sk_gemm_static call on a device: flag lines, status line and
// one fp32 partial tile per workgroup, in the layout of a caller-supplied workspace.  Each device
// that loads the library holds its own copy until the process ends.  In host code the name of the
// array is only a handle for hipGetSymbolAddress; the device address it yields (one per device) is
// what kernels and fills get.
constexpr size_t SK_STATIC_SCRATCH_BYTES = SK_STATIC_WORKSPACE_MAX;
static_assert(SK_STATIC_SCRATCH_BYTES == SK_STATIC_WORKSPACE_MAX_BYTES, "the limit stated in streamk.h");
static __device__ __align__(256) unsigned char scratch[SK_STATIC_SCRATCH_BYTES];

constexpr int SK_MAX_DEVICES = 64;
void* g_scratch_ptr[SK_MAX_DEVICES] = {};      // device address of `scratch` on device i, once asked for
std::mutex g_scratch_mutex;

// Flag and status lines back to zero (a fill kernel, not a memset node: the call may be captured into a graph).
__global__ void clear_words_kernel(uint32_t* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// Device address of this device's `scratch` (asked for once per device, with that device current).
int static_scratch(void** out) {
    int dev = 0;
    if (!hip_ok(hipGetDevice(&dev))) return SK_ERR_HIP;
    if (dev < 0 || dev >= SK_MAX_DEVICES) return SK_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (!hip_ok(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch))) || !ptr) return SK_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SK_OK;
}

}  // namespace

extern "C" int sk_gemm(const void* A, const void* B, void* D, const sk_plan_t* plan, void* stream) {
    if (!plan) return SK_ERR_INVALID_ARG;
    return launch_gemm(A, B, D, plan, stream, plan->workspace);
}

extern "C" int sk_gemm_static(const void* A, const void* B, void* D, const sk_plan_t* plan, void* stream) {
    if (!A || !B || !D || !plan) return SK_ERR_INVALID_ARG;
    // the atomic fix-up accumulates into an fp32 image of D, whose size has no bound: caller-owned memory only
    if (plan->fixup == SK_FIXUP_ATOMIC && plan->needs_fixup && plan->h.out_dtype != SK_F32) return SK_ERR_UNSUPPORTED;
    if (!plan->needs_fixup) return launch_gemm(A, B, D, plan, stream, nullptr);    // no split tile: nothing to exchange
    if (sk_workspace_bytes(plan) > SK_STATIC_SCRATCH_BYTES) return SK_ERR_WORKSPACE;
    void* ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != SK_OK) return rc;
    // the array keeps what the last call left: a call that timed out may have left flags or the status up
    const int words = (int)(sk_ws_partials_offset(plan->h.grid) / 4);
    hipLaunchKernelGGL(clear_words_kernel, dim3((words + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<uint32_t*>(ws), words);
    if (!hip_ok(hipGetLastError())) return SK_ERR_HIP;
    return launch_gemm(A, B, D, plan, stream, ws);
}

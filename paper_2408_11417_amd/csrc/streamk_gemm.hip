// Stream-K GEMM for gfx950 (MI355X): one persistent kernel serves every
// scheduling policy.  Each workgroup derives its own share of the iteration
// space from a handful of plan numbers (Algorithm 1, lines 4-12), runs the MAC
// loop of each segment on the matrix cores, and either stores the tile, parks an
// fp32 partial in the workspace, or - as the tile's owner - waits for the parked
// partials and adds them in a fixed order (the synchronised reduction that
// Sec. 5.3 names as the alternative to Algorithm 1's atomic adds).
#include <hip/hip_runtime.h>
#include <atomic>
#include <mutex>
#include "streamk_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16;

struct GemmArgs {
    const void* A;
    const void* B;
    void* D;
    float* partials;       // grid slots of BM*BN floats
    uint32_t* flags;       // one per workgroup, SK_FLAG_STRIDE bytes apart
    uint32_t* status;      // set non-zero when an owner gives up waiting
    int M, N, K;
    int tiles_n, tiles, ipt, sk_tiles, ipw, grid;
    long long sk_iters;
    uint32_t epoch, spin_limit;
    int out_dtype;
};

// ---- matrix-core wrappers ---------------------------------------------------------------------
// One instruction multiplies an MF x KM block of A by a KM x MF block of B.  Lane l holds, for A,
// row l % MF and the 8 consecutive k starting at 8 * (l / MF); for B, column l % MF and the same
// k; for the MF x MF result, column l % MF and rows (r/4) * (256/MF) + 4 * (l / MF) + r % 4.
template <int DT, int MF> struct Mfma;
template <> struct Mfma<SK_BF16, 32> {
    typedef f32x16 Acc;
    static __device__ __forceinline__ Acc run(uint4 a, uint4 b, Acc c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct Mfma<SK_F16, 32> {
    typedef f32x16 Acc;
    static __device__ __forceinline__ Acc run(uint4 a, uint4 b, Acc c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};
template <> struct Mfma<SK_BF16, 16> {
    typedef f32x4 Acc;
    static __device__ __forceinline__ Acc run(uint4 a, uint4 b, Acc c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct Mfma<SK_F16, 16> {
    typedef f32x4 Acc;
    static __device__ __forceinline__ Acc run(uint4 a, uint4 b, Acc c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};

template <int DT_, int BM_, int BN_, int BK_, int WM_, int WN_, int MF_>
struct Cfg {
    static constexpr int DT = DT_, BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, MF = MF_;
    static constexpr int THREADS = 64 * WM * WN;
    static constexpr int WTM = BM / WM, WTN = BN / WN;   // tile of one wave
    static constexpr int MI = WTM / MF, NI = WTN / MF;   // matrix-core blocks per wave tile
    static constexpr int KG = 64 / MF;                   // groups of 8 k across the lanes
    static constexpr int KM = 8 * KG;                    // k per instruction
    static constexpr int KK = BK / KM;
    static constexpr int ACC = MF * MF / 64;             // accumulator registers per block
    // LDS: A as [BM][BK + 8], B as [BK][BN + 32] 16-bit elements.  The paddings put the 16-byte
    // reads of 16 consecutive A rows, and the 8-byte transposing reads of 4 consecutive B rows,
    // on disjoint banks.
    static constexpr int LDA = BK + 8, LDB = BN + 32;
    static constexpr int A_ELEMS = BM * LDA, B_ELEMS = BK * LDB;
    static constexpr int STAGE_ELEMS = A_ELEMS + B_ELEMS;
    static constexpr int LDS_BYTES = 2 * STAGE_ELEMS * 2;
    static constexpr int A_CHUNKS = BM * BK / 8, B_CHUNKS = BK * BN / 8;   // 16-byte pieces per tile
    static constexpr int CA = (A_CHUNKS + THREADS - 1) / THREADS;
    static constexpr int CB = (B_CHUNKS + THREADS - 1) / THREADS;
    static_assert(WTM % MF == 0 && WTN % MF == 0 && BK % KM == 0, "tile does not divide");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
};

// Hardware workgroup ids go round-robin over the 8 XCDs; give each XCD a contiguous block of
// logical workgroup ids so that neighbours in the schedule (which share tiles and A row-blocks)
// share an L2.
__device__ __forceinline__ int logical_wg(int hw, int grid) {
    return (grid % 8 == 0) ? (hw % 8) * (grid / 8) + hw / 8 : hw;
}

template <bool ALIGNED>
__device__ __forceinline__ uint4 load8(const u16* __restrict__ base, long long row, long long col, int rows, int cols, long long ld) {
    // 8 consecutive 16-bit elements of a row-major matrix, zero beyond its edges
    uint4 v = make_uint4(0, 0, 0, 0);
    if (row < rows) {
        if (ALIGNED) {
            if (col < cols) v = *reinterpret_cast<const uint4*>(base + row * ld + col);
        } else {
            u16 e[8];
#pragma unroll
            for (int i = 0; i < 8; i++) e[i] = (col + i < cols) ? base[row * ld + col + i] : (u16)0;
            v.x = e[0] | (uint32_t)e[1] << 16; v.y = e[2] | (uint32_t)e[3] << 16;
            v.z = e[4] | (uint32_t)e[5] << 16; v.w = e[6] | (uint32_t)e[7] << 16;
        }
    }
    return v;
}

template <class C, bool ALIGNED>
__device__ __forceinline__ void fetch_tiles(const GemmArgs& g, int m0, int n0, int kit, uint4 (&ra)[C::CA], uint4 (&rb)[C::CB]) {
    const int tid = threadIdx.x;
    const u16* A = static_cast<const u16*>(g.A);
    const u16* B = static_cast<const u16*>(g.B);
    const int k0 = kit * C::BK;
#pragma unroll
    for (int i = 0; i < C::CA; i++) {
        const int c = tid + i * C::THREADS;
        if (C::A_CHUNKS % C::THREADS == 0 || c < C::A_CHUNKS)
            ra[i] = load8<ALIGNED>(A, m0 + c / (C::BK / 8), k0 + (c % (C::BK / 8)) * 8, g.M, g.K, g.K);
    }
#pragma unroll
    for (int i = 0; i < C::CB; i++) {
        const int c = tid + i * C::THREADS;
        if (C::B_CHUNKS % C::THREADS == 0 || c < C::B_CHUNKS)
            rb[i] = load8<ALIGNED>(B, k0 + c / (C::BN / 8), n0 + (c % (C::BN / 8)) * 8, g.K, g.N, g.N);
    }
}

template <class C>
__device__ __forceinline__ void stash_tiles(u16* stage, const uint4 (&ra)[C::CA], const uint4 (&rb)[C::CB]) {
    const int tid = threadIdx.x;
    u16* sA = stage;
    u16* sB = stage + C::A_ELEMS;
#pragma unroll
    for (int i = 0; i < C::CA; i++) {
        const int c = tid + i * C::THREADS;
        if (C::A_CHUNKS % C::THREADS == 0 || c < C::A_CHUNKS)
            *reinterpret_cast<uint4*>(sA + (c / (C::BK / 8)) * C::LDA + (c % (C::BK / 8)) * 8) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < C::CB; i++) {
        const int c = tid + i * C::THREADS;
        if (C::B_CHUNKS % C::THREADS == 0 || c < C::B_CHUNKS)
            *reinterpret_cast<uint4*>(sB + (c / (C::BN / 8)) * C::LDB + (c % (C::BN / 8)) * 8) = rb[i];
    }
}

// 4 k-consecutive elements of one B column out of the row-major [k][n] LDS tile: the
// transposing read hands lane j of each 16-lane group column j of a 4 x 16 block whose rows are
// addressed by lanes 4e..4e+3 of the group.
__device__ __forceinline__ uint2 read_b_transposed(const u16* p) {
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p));
    return __builtin_bit_cast(uint2, v);
}

template <class C>
__device__ __forceinline__ void mac_stage(const u16* stage, typename Mfma<C::DT, C::MF>::Acc (&acc)[C::MI][C::NI]) {
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    const int wm = wave / C::WN, wn = wave % C::WN;
    const u16* sA = stage + (wm * C::WTM + lane % C::MF) * C::LDA + 8 * (lane / C::MF);
    const u16* sB = stage + C::A_ELEMS + (8 * (lane / C::MF) + (lane % 16) / 4) * C::LDB
                  + wn * C::WTN + 16 * ((lane % C::MF) / 16) + 4 * (lane % 4);
#pragma unroll
    for (int kk = 0; kk < C::KK; kk++) {
        uint4 af[C::MI], bf[C::NI];
#pragma unroll
        for (int mi = 0; mi < C::MI; mi++)
            af[mi] = *reinterpret_cast<const uint4*>(sA + mi * C::MF * C::LDA + kk * C::KM);
#pragma unroll
        for (int ni = 0; ni < C::NI; ni++) {
            const u16* p = sB + kk * C::KM * C::LDB + ni * C::MF;
            const uint2 lo = read_b_transposed(p), hi = read_b_transposed(p + 4 * C::LDB);
            bf[ni] = make_uint4(lo.x, lo.y, hi.x, hi.y);
        }
#pragma unroll
        for (int mi = 0; mi < C::MI; mi++)
#pragma unroll
            for (int ni = 0; ni < C::NI; ni++)
                acc[mi][ni] = Mfma<C::DT, C::MF>::run(af[mi], bf[ni], acc[mi][ni]);
    }
}

__device__ __forceinline__ u16 to_bf16_bits(float f) {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u16)((u >> 16) | 0x40);   // quiet NaN
    return (u16)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);                   // round to nearest even
}

template <class C, bool ALIGNED>
__global__ __launch_bounds__(C::THREADS) void streamk_gemm_kernel(GemmArgs g) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    u16* smem = reinterpret_cast<u16*>(smem_raw);
    typedef typename Mfma<C::DT, C::MF>::Acc Acc;
    const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
    const int wm = wave / C::WN, wn = wave % C::WN;
    const int x = logical_wg(blockIdx.x, g.grid);

    // Algorithm 1, lines 5-6 (clamped): this workgroup's share of the Stream-K iterations
    long long it = (long long)x * g.ipw, it_end = it + g.ipw;
    if (it > g.sk_iters) it = g.sk_iters;
    if (it_end > g.sk_iters) it_end = g.sk_iters;
    int dp_tile = g.sk_tiles + x;   // data-parallel tiles come after the Stream-K work

    while (true) {
        int tile, k_begin, k_end;
        if (it < it_end) {                       // Algorithm 1, lines 8-12
            tile = (int)(it / g.ipt);
            const long long tile_first = (long long)tile * g.ipt;
            k_begin = (int)(it - tile_first);
            const long long stop = it_end < tile_first + g.ipt ? it_end : tile_first + g.ipt;
            k_end = (int)(stop - tile_first);
            it = tile_first + g.ipt;
        } else if (dp_tile < g.tiles) {
            tile = dp_tile; k_begin = 0; k_end = g.ipt;
            dp_tile += g.grid;
        } else {
            break;
        }
        const int m0 = (tile / g.tiles_n) * C::BM, n0 = (tile % g.tiles_n) * C::BN;

        // ---- MAC loop (Algorithm 1, line 13): global -> registers -> LDS (two stages) -> matrix cores
        Acc acc[C::MI][C::NI];
#pragma unroll
        for (int mi = 0; mi < C::MI; mi++)
#pragma unroll
            for (int ni = 0; ni < C::NI; ni++)
#pragma unroll
                for (int r = 0; r < C::ACC; r++) acc[mi][ni][r] = 0.f;
        {
            uint4 ra[C::CA], rb[C::CB];
            fetch_tiles<C, ALIGNED>(g, m0, n0, k_begin, ra, rb);
            stash_tiles<C>(smem, ra, rb);
            __syncthreads();
            for (int k = k_begin; k < k_end; k++) {
                const int cur = (k - k_begin) & 1;
                const bool more = k + 1 < k_end;
                if (more) fetch_tiles<C, ALIGNED>(g, m0, n0, k + 1, ra, rb);
                mac_stage<C>(smem + cur * C::STAGE_ELEMS, acc);
                if (more) stash_tiles<C>(smem + (cur ^ 1) * C::STAGE_ELEMS, ra, rb);
                __syncthreads();
            }
        }

        // ---- fix-up
        float4* slot = reinterpret_cast<float4*>(g.partials + (size_t)x * C::BM * C::BN);
        if (k_begin > 0) {
            // contributor: park the accumulators (register order, coalesced), then signal
#pragma unroll
            for (int mi = 0; mi < C::MI; mi++)
#pragma unroll
                for (int ni = 0; ni < C::NI; ni++)
#pragma unroll
                    for (int q = 0; q < C::ACC / 4; q++)
                        slot[((mi * C::NI + ni) * (C::ACC / 4) + q) * C::THREADS + tid] =
                            make_float4(acc[mi][ni][4 * q], acc[mi][ni][4 * q + 1], acc[mi][ni][4 * q + 2], acc[mi][ni][4 * q + 3]);
            __threadfence();                      // make the partial visible device-wide (all XCDs)
            __syncthreads();
            if (tid == 0)
                __hip_atomic_store(g.flags + (size_t)x * (SK_FLAG_STRIDE / 4), g.epoch, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
            continue;
        }
        if (k_end < g.ipt) {
            // owner: contributors are the following workgroups up to the one holding the tile's last iteration
            const int last = (int)(((long long)tile * g.ipt + g.ipt - 1) / g.ipw);
            for (int c = x + 1; c <= last; c++) {
                if (tid == 0) {
                    uint32_t polls = 0;
                    while (__hip_atomic_load(g.flags + (size_t)c * (SK_FLAG_STRIDE / 4), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != g.epoch) {
                        if (polls++ >= g.spin_limit) {   // bounded wait: record and go on
                            __hip_atomic_store(g.status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            break;
                        }
                        __builtin_amdgcn_s_sleep(2);
                    }
                }
                __syncthreads();
                __threadfence();                  // acquire: drop stale cached copies of the slot
                const float4* src = reinterpret_cast<const float4*>(g.partials + (size_t)c * C::BM * C::BN);
#pragma unroll
                for (int mi = 0; mi < C::MI; mi++)
#pragma unroll
                    for (int ni = 0; ni < C::NI; ni++)
#pragma unroll
                        for (int q = 0; q < C::ACC / 4; q++) {
                            const float4 v = src[((mi * C::NI + ni) * (C::ACC / 4) + q) * C::THREADS + tid];
                            acc[mi][ni][4 * q] += v.x; acc[mi][ni][4 * q + 1] += v.y;
                            acc[mi][ni][4 * q + 2] += v.z; acc[mi][ni][4 * q + 3] += v.w;
                        }
            }
        }

        // ---- epilogue: fp32 accumulators -> D
#pragma unroll
        for (int mi = 0; mi < C::MI; mi++)
#pragma unroll
            for (int ni = 0; ni < C::NI; ni++) {
                const int col = n0 + wn * C::WTN + ni * C::MF + lane % C::MF;
#pragma unroll
                for (int r = 0; r < C::ACC; r++) {
                    const int row = m0 + wm * C::WTM + mi * C::MF + (r / 4) * (4 * C::KG) + 4 * (lane / C::MF) + r % 4;
                    if (row < g.M && col < g.N) {
                        const size_t o = (size_t)row * g.N + col;
                        const float v = acc[mi][ni][r];
                        if (g.out_dtype == SK_F32) static_cast<float*>(g.D)[o] = v;
                        else if (g.out_dtype == SK_BF16) static_cast<u16*>(g.D)[o] = to_bf16_bits(v);
                        else static_cast<_Float16*>(g.D)[o] = (_Float16)v;
                    }
                }
            }
    }
}

// ---- host side ---------------------------------------------------------------------------------
typedef void (*kernel_fn)(GemmArgs);
struct KernelEntry {
    int dtype, bm, bn, bk;
    kernel_fn aligned, generic;
    int threads, lds_bytes;
    std::atomic<int> max_resident{-1};   // co-resident workgroups on the device, -1 = not yet asked
    KernelEntry(int d, int m, int n, int k, kernel_fn a, kernel_fn g, int t, int l)
        : dtype(d), bm(m), bn(n), bk(k), aligned(a), generic(g), threads(t), lds_bytes(l) {}
};

template <class C> KernelEntry* make_entry() {
    return new KernelEntry(C::DT, C::BM, C::BN, C::BK, streamk_gemm_kernel<C, true>, streamk_gemm_kernel<C, false>,
                           C::THREADS, C::LDS_BYTES);
}

template <int DT> void add_dtype(KernelEntry** t, int* n) {
    t[(*n)++] = make_entry<Cfg<DT, 128, 128, 32, 2, 2, 32>>();
    t[(*n)++] = make_entry<Cfg<DT, 128, 128, 64, 2, 2, 32>>();
    t[(*n)++] = make_entry<Cfg<DT, 256, 128, 64, 2, 2, 32>>();
    t[(*n)++] = make_entry<Cfg<DT, 256, 256, 64, 2, 4, 32>>();
    t[(*n)++] = make_entry<Cfg<DT, 64, 128, 64, 2, 2, 32>>();
    t[(*n)++] = make_entry<Cfg<DT, 32, 128, 64, 1, 4, 32>>();
    t[(*n)++] = make_entry<Cfg<DT, 16, 128, 64, 1, 4, 16>>();
}

KernelEntry** kernel_table(int* count) {
    static KernelEntry* table[32];
    static int n = 0;
    static std::once_flag once;
    std::call_once(once, [] {
        add_dtype<SK_BF16>(table, &n);
        add_dtype<SK_F16>(table, &n);
    });
    *count = n;
    return table;
}

KernelEntry* find_kernel(int dtype, int bm, int bn, int bk) {
    int n;
    KernelEntry** t = kernel_table(&n);
    for (int i = 0; i < n; i++)
        if (t[i]->dtype == dtype && t[i]->bm == bm && t[i]->bn == bn && t[i]->bk == bk) return t[i];
    return nullptr;
}

std::atomic<uint32_t> g_epoch{0};

}  // namespace

bool sk_kernel_available(int in_dtype, int blk_m, int blk_n, int blk_k) {
    return find_kernel(in_dtype, blk_m, blk_n, blk_k) != nullptr;
}

extern "C" int sk_plan_set_workspace(sk_plan_t* plan, void* dev_ptr, size_t bytes) {
    if (!plan || !dev_ptr) return SK_ERR_INVALID_ARG;
    if (bytes < sk_workspace_bytes(plan) || (reinterpret_cast<uintptr_t>(dev_ptr) & 255)) return SK_ERR_WORKSPACE;
    if (hipMemset(dev_ptr, 0, sk_ws_partials_offset(plan->h.grid)) != hipSuccess) return SK_ERR_HIP;
    if (hipDeviceSynchronize() != hipSuccess) return SK_ERR_HIP;
    plan->workspace = dev_ptr;
    plan->workspace_bytes = bytes;
    return SK_OK;
}

extern "C" int sk_plan_check(const sk_plan_t* plan, void* stream) {
    if (!plan) return SK_ERR_INVALID_ARG;
    if (hipStreamSynchronize(static_cast<hipStream_t>(stream)) != hipSuccess) return SK_ERR_HIP;
    if (!plan->workspace) return SK_OK;
    uint32_t* st = reinterpret_cast<uint32_t*>(static_cast<char*>(plan->workspace) + sk_ws_status_offset(plan->h.grid));
    uint32_t v = 0;
    if (hipMemcpy(&v, st, sizeof v, hipMemcpyDeviceToHost) != hipSuccess) return SK_ERR_HIP;
    if (v) {
        if (hipMemset(st, 0, sizeof v) != hipSuccess) return SK_ERR_HIP;
        return SK_ERR_TIMEOUT;
    }
    return SK_OK;
}

extern "C" int sk_gemm(const void* A, const void* B, void* D, const sk_plan_t* plan, void* stream) {
    if (!A || !B || !D || !plan) return SK_ERR_INVALID_ARG;
    const sk_plan_header& h = plan->h;
    const uintptr_t align = reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B) | reinterpret_cast<uintptr_t>(D);
    if (align & 15) return SK_ERR_INVALID_ARG;
    if (h.M > 0x7FFFFFFF || h.N > 0x7FFFFFFF || h.K > 0x7FFFFFFF) return SK_ERR_UNSUPPORTED;
    KernelEntry* e = find_kernel(h.in_dtype, h.blk_m, h.blk_n, h.blk_k);
    if (!e) return SK_ERR_UNSUPPORTED;
    if (plan->needs_fixup && !plan->workspace) return SK_ERR_WORKSPACE;
    const bool aligned = (h.K % 8 == 0) && (h.N % 8 == 0);
    kernel_fn fn = aligned ? e->aligned : e->generic;

    if (e->max_resident.load() < 0) {
        // first use on this process: allow the large LDS footprint and ask how many workgroups fit at once
        for (kernel_fn f : {e->aligned, e->generic})
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(f), hipFuncAttributeMaxDynamicSharedMemorySize, e->lds_bytes) != hipSuccess)
                return SK_ERR_HIP;
        int dev = 0, cus = 0, per_cu = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return SK_ERR_HIP;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(e->generic), e->threads, e->lds_bytes) != hipSuccess)
            return SK_ERR_HIP;
        e->max_resident.store(per_cu * cus);
    }
    // an owner spins on flags of other workgroups: all of them must be on the machine at once
    if (plan->needs_fixup && h.grid > e->max_resident.load()) return SK_ERR_UNSUPPORTED;

    GemmArgs g{};
    g.A = A; g.B = B; g.D = D;
    char* ws = static_cast<char*>(plan->workspace);
    g.flags = reinterpret_cast<uint32_t*>(ws);
    g.status = ws ? reinterpret_cast<uint32_t*>(ws + sk_ws_status_offset(h.grid)) : nullptr;
    g.partials = ws ? reinterpret_cast<float*>(ws + sk_ws_partials_offset(h.grid)) : nullptr;
    g.M = (int)h.M; g.N = (int)h.N; g.K = (int)h.K;
    g.tiles_n = h.tiles_n; g.tiles = h.tiles; g.ipt = h.iters_per_tile;
    g.sk_tiles = h.sk_tiles; g.ipw = h.iters_per_wg; g.grid = h.grid; g.sk_iters = h.sk_iters;
    uint32_t ep = ++g_epoch;
    if (ep == 0) ep = ++g_epoch;                 // 0 is the cleared state of a flag
    g.epoch = ep;
    g.spin_limit = plan->spin_limit;
    g.out_dtype = h.out_dtype;
    hipLaunchKernelGGL(fn, dim3(h.grid), dim3(e->threads), e->lds_bytes, static_cast<hipStream_t>(stream), g);
    return hipGetLastError() == hipSuccess ? SK_OK : SK_ERR_HIP;
}

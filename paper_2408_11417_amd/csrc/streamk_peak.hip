// Matrix-core rate of the device with nothing else in the way: every wave runs a register-resident
// loop of independent matrix-core instructions (the instructions of the GEMM kernels' MAC loop, no
// LDS, no global memory inside the loop).  What this loop reaches is the ceiling the MAC loop
// could reach on the same operand values at the clock the device sustains under that load.
#include <hip/hip_runtime.h>
#include "streamk_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int PEAK_THREADS = 256;      // one wave per SIMD
constexpr int PEAK_FRAGS = 4;          // 4 x 4 operand pairs = 16 independent accumulators per wave

template <int DT> struct PeakOp;
template <> struct PeakOp<SK_BF16> {
    typedef u32x4 Frag;
    static constexpr double FLOPS = 2.0 * 32 * 32 * 16;
    static __device__ __forceinline__ f32x16 run(Frag a, Frag b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct PeakOp<SK_F16> {
    typedef u32x4 Frag;
    static constexpr double FLOPS = 2.0 * 32 * 32 * 16;
    static __device__ __forceinline__ f32x16 run(Frag a, Frag b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};
template <> struct PeakOp<SK_FP8_E4M3> {
    typedef i32x8 Frag;
    static constexpr double FLOPS = 2.0 * 32 * 32 * 64;
    static __device__ __forceinline__ f32x16 run(Frag a, Frag b, f32x16 c) {
        return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 127, 0, 127);
    }
};

// operands: 2 * PEAK_FRAGS fragments per lane, read once; sink: one float per thread
template <int DT>
__global__ __launch_bounds__(PEAK_THREADS) void mfma_peak_kernel(const void* operands, float* sink, int iters) {
    typedef typename PeakOp<DT>::Frag Frag;
    const Frag* src = static_cast<const Frag*>(operands) + (size_t)threadIdx.x * (2 * PEAK_FRAGS);
    Frag a[PEAK_FRAGS], b[PEAK_FRAGS];
#pragma unroll
    for (int i = 0; i < PEAK_FRAGS; i++) { a[i] = src[i]; b[i] = src[PEAK_FRAGS + i]; }
    f32x16 acc[PEAK_FRAGS][PEAK_FRAGS];
#pragma unroll
    for (int i = 0; i < PEAK_FRAGS; i++)
#pragma unroll
        for (int j = 0; j < PEAK_FRAGS; j++) acc[i][j] = f32x16{};
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int i = 0; i < PEAK_FRAGS; i++)
#pragma unroll
            for (int j = 0; j < PEAK_FRAGS; j++) acc[i][j] = PeakOp<DT>::run(a[i], b[j], acc[i][j]);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < PEAK_FRAGS; i++)
#pragma unroll
        for (int j = 0; j < PEAK_FRAGS; j++) s += acc[i][j][0] + acc[i][j][15];
    sink[(size_t)blockIdx.x * PEAK_THREADS + threadIdx.x] = s;
}

}  // namespace

extern "C" size_t sk_mfma_peak_operand_bytes(void) { return (size_t)PEAK_THREADS * 2 * PEAK_FRAGS * sizeof(i32x8); }

extern "C" int sk_mfma_peak_launch(int in_dtype, const void* operands, float* sink, int workgroups, int iters, void* stream, double* flops) {
    if (!operands || !sink || workgroups < 1 || iters < 1) return SK_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    double per_op = 0.0;
    switch (in_dtype) {
        case SK_BF16: per_op = PeakOp<SK_BF16>::FLOPS; hipLaunchKernelGGL(mfma_peak_kernel<SK_BF16>, dim3(workgroups), dim3(PEAK_THREADS), 0, st, operands, sink, iters); break;
        case SK_F16: per_op = PeakOp<SK_F16>::FLOPS; hipLaunchKernelGGL(mfma_peak_kernel<SK_F16>, dim3(workgroups), dim3(PEAK_THREADS), 0, st, operands, sink, iters); break;
        case SK_FP8_E4M3: per_op = PeakOp<SK_FP8_E4M3>::FLOPS; hipLaunchKernelGGL(mfma_peak_kernel<SK_FP8_E4M3>, dim3(workgroups), dim3(PEAK_THREADS), 0, st, operands, sink, iters); break;
        default: return SK_ERR_INVALID_ARG;
    }
    if (hipGetLastError() != hipSuccess) return SK_ERR_HIP;
    if (flops) *flops = per_op * PEAK_FRAGS * PEAK_FRAGS * (double)iters * (PEAK_THREADS / 64) * (double)workgroups;
    return SK_OK;
}

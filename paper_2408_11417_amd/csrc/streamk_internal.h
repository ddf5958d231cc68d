// Internal definitions shared by the host planner and the HIP launcher.
#pragma once
#include <cstdint>
#include <cstddef>
#include "streamk.h"

struct sk_plan_t {
    sk_plan_header h;
    void* workspace = nullptr;      // caller-owned device memory
    size_t workspace_bytes = 0;
    uint32_t spin_limit = 1u << 24;
    int needs_fixup = 0;            // 1 if any tile is split over several workgroups
    int fixup = SK_FIXUP_FLAGS;     // how split tiles are combined
    int dp_first = 0;               // 1: data-parallel tiles before the Stream-K iterations
    int k_aligned = 1;              // 1: head piece of a Stream-K range first, last workgroup of a tile owns it
    int kernel_variant = 0;         // which compiled wave layout of the tile's kernel to launch (0 = the library's choice)
};

// Workspace layout: [grid flag lines of SK_FLAG_STRIDE bytes][status line][partials]
constexpr size_t SK_FLAG_STRIDE = 128;
constexpr int SK_GROUP_ROWS = 8;   // tile rows per band of the grouped tile order
constexpr int SK_TREE_GROUP = 8;   // contributors per group in the two-level reduction of tiles shared by many workgroups
inline size_t sk_ws_status_offset(int grid) { return (size_t)grid * SK_FLAG_STRIDE; }
inline size_t sk_ws_partials_offset(int grid) { return ((size_t)grid + 1) * SK_FLAG_STRIDE + 384; }

// Size of the device array behind sk_gemm_static: the flag and status lines of 256 workgroups plus
// 256 partial tiles of 256 x 256 fp32 (the largest tile), i.e. every plan on the default grid.
constexpr size_t SK_STATIC_WORKSPACE_MAX = (256 + 1) * SK_FLAG_STRIDE + 384 + (size_t)256 * 256 * 256 * 4;

// Division of a number below 2^31 by a divisor that is fixed for a launch: with shift = 31 + ceil(log2 d)
// and mul = ceil(2^shift / d) (which fits 32 bits), n / d == (n * mul) >> shift for every n < 2^31, because
// the error n * (mul * d - 2^shift) stays below 2^shift.  The kernels' index arithmetic (Algorithm 1's
// iteration -> tile and tile -> workgroup maps) sits ahead of a workgroup's first load and inside the
// fix-up chain, and a division by a run-time value costs about 300 cycles of dependent instructions there.
struct sk_fast_div { uint32_t mul, shift; };
inline sk_fast_div sk_make_fast_div(uint32_t d) {
    if (d == 0) return sk_fast_div{0u, 0u};          // never divided by (e.g. no Stream-K iterations)
    uint32_t log2_up = 0;
    while ((1ull << log2_up) < d) log2_up++;
    const uint32_t shift = 31 + log2_up;
    return sk_fast_div{(uint32_t)(((1ull << shift) + d - 1) / d), shift};
}
inline uint32_t sk_fast_div_apply(uint32_t n, sk_fast_div f) { return (uint32_t)(((uint64_t)n * f.mul) >> f.shift); }

// Does the GEMM launcher hold a kernel for this configuration?
bool sk_kernel_available(int in_dtype, int blk_m, int blk_n, int blk_k);
// Bytes of the fp32 image of D that the atomic fix-up accumulates into (0 if D itself serves).
inline size_t sk_ws_image_bytes(const sk_plan_t* p) {
    return p->fixup == SK_FIXUP_ATOMIC && p->h.out_dtype != SK_F32 ? (size_t)p->h.M * (size_t)p->h.N * sizeof(float) : 0;
}

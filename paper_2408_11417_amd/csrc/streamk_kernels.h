// Stream-K GEMM for gfx950 (MI355X): one persistent kernel serves every
// scheduling policy.  Each workgroup derives its own share of the iteration
// space from a handful of plan numbers (Algorithm 1's range and tile arithmetic), runs the MAC
// loop of each segment on the matrix cores, and either stores the tile, parks an
// fp32 partial in the workspace, or - as the tile's owner - waits for the parked
// partials and adds them in a fixed order (the synchronised reduction that
// Sec. 5.3 names as the alternative to Algorithm 1's atomic adds).
//
// MAC loop data path: A (row-major, k contiguous) and B (row-major, n contiguous)
// tiles go from global memory straight into LDS with 16-byte LDS-DMA loads, into
// a ring of NS stages; the LDS image is XOR-swizzled at 16-byte granularity (the
// swizzle is applied by choosing which global piece each lane fetches) so that
// the matrix-core operand reads are bank-conflict free without padding.  A
// operands are read with 16-byte LDS reads, B operands with the transposing
// 8-byte reads that turn the [k][n] image into k-contiguous lanes.
#pragma once
#include <hip/hip_runtime.h>
#include <atomic>
#include <type_traits>
#include <utility>
#include "streamk_internal.h"


namespace streamk_detail {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16;
typedef __attribute__((address_space(3))) unsigned char lds_byte;

struct GemmArgs {
    const void* A;
    const void* B;
    void* D;
    float* partials;       // grid slots of BM*BN floats
    float* image;          // atomic fix-up: fp32 image of D that partial tiles are added into (D itself for fp32 output)
    uint32_t* flags;       // one per workgroup, SK_FLAG_STRIDE bytes apart
    uint32_t* status;      // set non-zero when an owner gives up waiting
    int M, N, K;
    int tiles_m, tiles_n, tiles, ipt, sk_tiles, ipw, grid, sk_iters, tile_order;
    uint32_t spin_limit;
    int out_dtype;
    int dp_first;          // 1: a workgroup runs its data-parallel tiles before its Stream-K iterations
    int xcd_remap;         // 1: consecutive logical workgroup ids share an XCD (see logical_wg)
    int k_aligned;         // 1: a workgroup runs the whole tiles of its Stream-K range first, then the head of its last
                           //    tile (k from 0), then the tail of its first one, and the workgroup holding a tile's
                           //    last iteration reduces and stores it
    int stream_b;          // 1: B is read exactly once (one row of tiles) and is large: the low tiles request it non-temporally
    // divisors of the index arithmetic: ipt, ipw, tiles_n, SK_GROUP_ROWS * tiles_n, rows of the last (short) band
    sk_fast_div div_ipt, div_ipw, div_tiles_n, div_band, div_last_rows;
};

__device__ __forceinline__ uint32_t fast_div(uint32_t n, sk_fast_div f) { return (uint32_t)(((uint64_t)n * f.mul) >> f.shift); }

// ---- matrix-core wrappers ---------------------------------------------------------------------
// One instruction multiplies an MF x KM block (first operand) by a KM x MF block (second operand).
// Lane l holds, for the first operand, row l % MF and the 8 consecutive k starting at
// 8 * (l / MF); for the second, column l % MF and the same k; for the MF x MF result, column
// l % MF and rows (r/4) * (256/MF) + 4 * (l / MF) + r % 4.  Both operands have the same register
// format, so the kernels pass the B block first and the A block second: the instruction then
// produces the transposed block, i.e. lane l holds row l % MF of the D block and, in registers
// 4q .. 4q+3, the four consecutive columns (256/MF) * q + 4 * (l / MF) + {0..3}, which can be
// stored as vectors.
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

// fp8 (e4m3): the scaled 8-bit instruction with both block scales at 2^0 (biased exponent 127);
// per lane 32 consecutive k (8 registers) of row / column l % MF starting at 32 * (l / MF).
template <> struct Mfma<SK_FP8_E4M3, 32> {
    typedef f32x16 Acc;
    static __device__ __forceinline__ Acc run(i32x8 a, i32x8 b, Acc c) {
        return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 127, 0, 127);
    }
};
template <> struct Mfma<SK_FP8_E4M3, 16> {
    typedef f32x4 Acc;
    static __device__ __forceinline__ Acc run(i32x8 a, i32x8 b, Acc c) {
        return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 0, 0, 0, 127, 0, 127);
    }
};

template <int DT_, int BM_, int BN_, int BK_, int WM_, int WN_, int MF_, int NSA_, int NSB_ = NSA_, int FINE_ = 0>
struct Cfg {
    static constexpr int DT = DT_, BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, MF = MF_;
    static constexpr int NSA = NSA_, NSB = NSB_;        // LDS ring depth of the A and of the B tiles
    static constexpr int NW = WM * WN, THREADS = 64 * NW;
    static constexpr int WTM = BM / WM, WTN = BN / WN;   // tile of one wave
    static constexpr int MI = WTM / MF, NI = WTN / MF;   // matrix-core blocks per wave tile
    static constexpr bool FP8 = DT == SK_FP8_E4M3;
    static constexpr int ES = FP8 ? 1 : 2;               // bytes per input element
    static constexpr int PE = 16 / ES;                   // elements per 16-byte piece
    static constexpr int KPL = FP8 ? 32 : 8;             // consecutive k per lane per instruction
    static constexpr int APL = KPL / PE;                 // A pieces per lane per instruction
    static constexpr int KG = 64 / MF;                   // groups of KPL k across the lanes
    static constexpr int KM = KPL * KG;                  // k per instruction
    static constexpr int KK = BK / KM;
    static constexpr int ACC = MF * MF / 64;             // accumulator registers per block
    // LDS: a ring of NSA A tiles (BM rows of CPA 16-byte pieces) followed by a ring of NSB B tiles
    // (BK rows of CPB pieces), no padding.  A may be one stage deeper than B: its loads then run
    // two iterations ahead and only the B tile has to arrive within one iteration.
    static constexpr int CPA = BK / PE, CPB = BN / PE;
    static constexpr int A_PIECES = BM * CPA, B_PIECES = BK * CPB;
    static constexpr int A_BYTES = A_PIECES * 16, B_BYTES = B_PIECES * 16;
    static constexpr int B_RING = NSA * A_BYTES;         // byte offset of the B ring
    static constexpr int LDS_BYTES = NSA * A_BYTES + NSB * B_BYTES;
    // one LDS-DMA instruction of one wave fills 64 consecutive pieces
    static constexpr bool DIRECT = (A_PIECES % (64 * NW) == 0) && (B_PIECES % (64 * NW) == 0);
    static constexpr int A_LD = A_PIECES / (64 * NW), B_LD = B_PIECES / (64 * NW);
    static constexpr int LPS = A_LD + B_LD;              // LDS-DMA loads per stage per wave
    // register-staged fill (unaligned problems, tiles too small for the DMA split)
    static constexpr int CA = (A_PIECES + THREADS - 1) / THREADS, CB = (B_PIECES + THREADS - 1) / THREADS;
    // Registers of one set of matrix-core operands and of the accumulators.  With 8 waves a lane has
    // 256 registers for everything; with 4 waves 256 plus 256 that can hold the accumulators.
    // PIN_ORDER: there is room to hold two operand sets, so the MAC loop pins "read the next
    // k-step's operands, then multiply the current ones".
    static constexpr int FRAG_REGS = (MI + NI) * (FP8 ? 8 : 4), ACC_REGS = MI * NI * ACC;
    static constexpr bool PIN_ORDER = NW >= 8 ? 2 * FRAG_REGS + ACC_REGS + 64 <= 256 : 2 * FRAG_REGS + 64 <= 192;
    // FINE: the MAC loop is written out instruction by instruction - one matrix-core instruction, then
    // at most a few LDS reads of the next k-step's operands or one LDS-DMA request, and so on - so that
    // a wave that has a SIMD to itself keeps the matrix-core pipe fed while its memory instructions
    // queue up (needs the two operand sets of PIN_ORDER).
    static constexpr bool FINE = FINE_ != 0;
    // the tiles of at most 64 rows (HBM-bound shapes) can request B non-temporally, decided per launch
    // (GemmArgs::stream_b); the larger tiles re-use B blocks through the L2 caches and their request code
    // sits in the instruction-by-instruction loop, so they carry no such switch
    static constexpr bool MAY_STREAM_B = BM <= 64;
    static_assert(!FINE || PIN_ORDER, "the instruction-by-instruction order needs two operand sets");
    // register-staged path: room to hold the next stage's pieces (4 registers each) during the matrix-core work
    static constexpr bool STAGE_AHEAD = NW >= 8 ? 2 * FRAG_REGS + ACC_REGS + 4 * (CA + CB) + 64 <= 256 : 2 * FRAG_REGS + 4 * (CA + CB) + 64 <= 224;
    // vector stores one wave issues in the epilogue of an unsplit interior tile with 16-bit output (an fp32
    // output issues more): what may still be in flight when the next tile's first stage is waited for
    static constexpr int EPILOGUE_STORES = MI * NI * (MF == 32 ? ACC / 8 : ACC / 4);
    static_assert(WTM % MF == 0 && WTN % MF == 0 && BK % KM == 0, "tile does not divide");
    static_assert(CPA == 4 || CPA == 8 || CPA == 16, "A swizzle assumes 64/128/256-byte rows");
    static_assert(CPB >= 16, "B swizzle assumes rows of at least 256 bytes");
    static_assert(NSB >= 2 && (NSA == NSB || NSA == NSB + 1) && LDS_BYTES <= 160 * 1024, "LDS budget / ring depths");
    static_assert((NSA - 1) * LPS <= 63, "vmcnt range");
    // LDS-DMA loads that may still be in flight when iteration i starts, if `later` more
    // iterations follow it.  Issue order inside an iteration: B tile of iteration +NSB-1, then A
    // tile of iteration +NSA-1; loads complete in order.
    static constexpr int in_flight(int later) {
        int n = 0;
        if (NSA == NSB) {
            for (int d = 1; d <= NSA - 2; d++) n += later >= d ? LPS : 0;
        } else {
            n += later >= 1 ? A_LD : 0;
            for (int d = 1; d <= NSB - 2; d++) n += (later >= d ? B_LD : 0) + (later >= d + 1 ? A_LD : 0);
        }
        return n;
    }
};

// ---- LDS image --------------------------------------------------------------------------------
// A: piece c of row r sits at position c ^ swz_a(r).  Eight consecutive rows and also sixteen
// consecutive rows then spread the same logical piece over all banks (32- or 64-bank view).
template <int CPA> __device__ __forceinline__ int swz_a(int r) {
    if (CPA == 4) return (r >> 1) & 3;
    return (r & 7) ^ ((r >> 3) & 1);
}
// B: piece c of row k sits at position c ^ swz_b<C::FP8>(k): rows k..k+3, read together by one transposing
// read, land on different 32-byte and different 64-byte bank groups.
// (8-bit elements: one transposing read covers 8 rows; rows k..k+7 go to 8 different 32-byte groups.)
template <bool FP8> __device__ __forceinline__ int swz_b(int k) {
    if (FP8) return (k & 7) << 1;
    const int k0 = k & 1, k1 = (k >> 1) & 1;
    return (k0 << 1) | (k1 << 2) | (k0 << 3);
}

// Source of the pieces that lie beyond K in a ragged last k-iteration.
static __device__ __align__(16) const unsigned char g_zero_piece[16] = {0};

// 16 bytes global -> LDS without passing through registers.  The LDS destination of lane l is
// lds_base + 16 * l; lds_base must be wave-uniform.  Completion is tracked by vmcnt only; the
// compiler is not told that LDS is written: the caller orders the reads with s_waitcnt + barrier.
// m0 is not named as clobbered: it is a reserved register for this compiler (it never holds a value of
// the program across statements; the compiler writes it right before an instruction of its own that
// reads it), and naming a reserved register in a clobber list is rejected as undefined behaviour.
__device__ __forceinline__ void lds_dma16(const void* base, uint32_t byte_off, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(byte_off), "s"(base), "s"(lds_base));
}
// The same load marked non-temporal: for data that is read exactly once and is too large for the caches
// to hold until a later launch (the B operand of a plan with a single row of tiles, see the launcher).
__device__ __forceinline__ void lds_dma16_nt(const void* base, uint32_t byte_off, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt" ::"v"(byte_off), "s"(base), "s"(lds_base));
}
__device__ __forceinline__ void lds_dma16_ptr(const void* gptr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_base));
}

template <int N> __device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N <= 63, "vmcnt range");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);   // lgkmcnt / expcnt not waited
}

// Hardware workgroup ids go round-robin over the 8 XCDs; give each XCD a contiguous block of
// logical workgroup ids so that neighbours in the schedule (which share tiles and A row-blocks)
// share an L2.  Plans with a single row of low tiles keep the hardware order: their workgroups
// only stream B, and neighbouring column blocks read from different XCDs reach a higher HBM rate.
__device__ __forceinline__ int logical_wg(int hw, int grid, int remap) {
    return (remap && grid % 8 == 0) ? (hw % 8) * (grid / 8) + hw / 8 : hw;
}

// 16 bytes whose address is only known to be a multiple of the element size (rows of a matrix whose
// leading dimension is not a multiple of 8 elements start anywhere); the compiler picks the access.
struct __attribute__((packed, aligned(1))) Piece1 { u32x4 v; };
struct __attribute__((packed, aligned(2))) Piece2 { u32x4 v; };

template <int ES, bool ALIGNED>
__device__ __forceinline__ uint4 load_piece(const unsigned char* __restrict__ base, int row, int col, int rows, int cols) {
    // 16 bytes = 16 / ES consecutive elements of a row-major matrix with `cols` columns, zero beyond its edges
    uint4 v = make_uint4(0, 0, 0, 0);
    if (row < rows) {
        const unsigned char* p = base + (size_t)((uint32_t)row * (uint32_t)cols + (uint32_t)col) * ES;
        if (ALIGNED) {
            if (col < cols) v = *reinterpret_cast<const uint4*>(p);
        } else if (col + 16 / ES <= cols) {          // the whole piece lies inside the row
            const u32x4 w = ES == 2 ? reinterpret_cast<const Piece2*>(p)->v : reinterpret_cast<const Piece1*>(p)->v;
            v = make_uint4(w[0], w[1], w[2], w[3]);
        } else if (col < cols) {                     // the piece that straddles the end of the row
            unsigned char e[16];
#pragma unroll
            for (int i = 0; i < 16; i++) e[i] = (col + i / ES < cols) ? p[i] : (unsigned char)0;
            v.x = e[0] | (uint32_t)e[1] << 8 | (uint32_t)e[2] << 16 | (uint32_t)e[3] << 24;
            v.y = e[4] | (uint32_t)e[5] << 8 | (uint32_t)e[6] << 16 | (uint32_t)e[7] << 24;
            v.z = e[8] | (uint32_t)e[9] << 8 | (uint32_t)e[10] << 16 | (uint32_t)e[11] << 24;
            v.w = e[12] | (uint32_t)e[13] << 8 | (uint32_t)e[14] << 16 | (uint32_t)e[15] << 24;
        }
    }
    return v;
}

// Register-staged fill of one stage with zero fill at every edge (same LDS image as the DMA path),
// in two halves: fetch the stage's pieces into registers, and later park them in LDS.
template <class C, bool ALIGNED> struct StagedFill {
    uint4 ra[C::CA], rb[C::CB];
    __device__ __forceinline__ void fetch(const GemmArgs& g, int m0, int n0, int kit) {
        const int tid = threadIdx.x;
        const unsigned char* A = static_cast<const unsigned char*>(g.A);
        const unsigned char* B = static_cast<const unsigned char*>(g.B);
        const int k0 = kit * C::BK;
#pragma unroll
        for (int i = 0; i < C::CA; i++) {
            const int p = tid + i * C::THREADS;
            if (C::A_PIECES % C::THREADS == 0 || p < C::A_PIECES)
                ra[i] = load_piece<C::ES, ALIGNED>(A, m0 + p / C::CPA, k0 + (p % C::CPA) * C::PE, g.M, g.K);
        }
#pragma unroll
        for (int i = 0; i < C::CB; i++) {
            const int p = tid + i * C::THREADS;
            if (C::B_PIECES % C::THREADS == 0 || p < C::B_PIECES)
                rb[i] = load_piece<C::ES, ALIGNED>(B, k0 + p / C::CPB, n0 + (p % C::CPB) * C::PE, g.K, g.N);
        }
    }
    __device__ __forceinline__ void park(unsigned char* a_stage, unsigned char* b_stage) const {
        const int tid = threadIdx.x;
        uint4* sA = reinterpret_cast<uint4*>(a_stage);
        uint4* sB = reinterpret_cast<uint4*>(b_stage);
#pragma unroll
        for (int i = 0; i < C::CA; i++) {
            const int p = tid + i * C::THREADS, r = p / C::CPA;
            if (C::A_PIECES % C::THREADS == 0 || p < C::A_PIECES) sA[r * C::CPA + ((p % C::CPA) ^ swz_a<C::CPA>(r))] = ra[i];
        }
#pragma unroll
        for (int i = 0; i < C::CB; i++) {
            const int p = tid + i * C::THREADS, k = p / C::CPB;
            if (C::B_PIECES % C::THREADS == 0 || p < C::B_PIECES) sB[k * C::CPB + ((p % C::CPB) ^ swz_b<C::FP8>(k))] = rb[i];
        }
    }
};

// Per-tile addressing of the LDS-DMA loads: lane l of this wave's j-th A instruction fills A
// position (j * NW + wave) * 64 + l.  Rows beyond M and columns beyond N are clamped to the last
// valid one: they only feed output elements that are never stored.
template <class C> struct DmaMap {
    uint32_t a_off[C::A_LD > 0 ? C::A_LD : 1];   // byte offsets from A / B at k-iteration 0
    uint32_t b_off[C::B_LD > 0 ? C::B_LD : 1];
    __device__ __forceinline__ void init(const GemmArgs& g, int m0, int n0) {
        const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
#pragma unroll
        for (int j = 0; j < C::A_LD; j++) {
            const int p = (j * C::NW + wave) * 64 + lane;
            const int r = p / C::CPA, c = (p % C::CPA) ^ swz_a<C::CPA>(r);
            int row = m0 + r;
            row = row < g.M ? row : g.M - 1;
            a_off[j] = ((uint32_t)row * (uint32_t)g.K + (uint32_t)(C::PE * c)) * C::ES;
        }
#pragma unroll
        for (int j = 0; j < C::B_LD; j++) {
            const int p = (j * C::NW + wave) * 64 + lane;
            const int k = p / C::CPB, c = (p % C::CPB) ^ swz_b<C::FP8>(k);
            int col = n0 + C::PE * c;
            col = col < g.N ? col : g.N - C::PE;
            b_off[j] = ((uint32_t)k * (uint32_t)g.N + (uint32_t)col) * C::ES;
        }
    }
    // Loads of k-iteration `kit`.  TAIL: the iteration reaches beyond K (K is a multiple of the
    // piece length here); pieces at k >= K are then fetched from a zero piece so that they add nothing.
    template <bool TAIL> __device__ __forceinline__ void issue_a(const GemmArgs& g, int kit, uint32_t lds, int j0 = 0, int j1 = C::A_LD) const {
        const int lane = threadIdx.x % 64;
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
        const char* A = static_cast<const char*>(g.A) + (size_t)((uint32_t)kit * (uint32_t)(C::BK * C::ES));
#pragma unroll
        for (int j = 0; j < C::A_LD; j++) {
            if (j < j0 || j >= j1) continue;
            if (!TAIL) {
                lds_dma16(A, a_off[j], lds + (j * C::NW + wave) * 1024);
            } else {
                const int p = (j * C::NW + wave) * 64 + lane;
                const int r = p / C::CPA, c = (p % C::CPA) ^ swz_a<C::CPA>(r);
                const char* src = kit * C::BK + C::PE * c < g.K ? A + a_off[j] : reinterpret_cast<const char*>(g_zero_piece);
                lds_dma16_ptr(src, lds + (j * C::NW + wave) * 1024);
            }
        }
    }
    template <bool TAIL, bool NT = false> __device__ __forceinline__ void issue_b(const GemmArgs& g, int kit, uint32_t lds, int j0 = 0, int j1 = C::B_LD) const {
        const int lane = threadIdx.x % 64;
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
        const char* B = static_cast<const char*>(g.B) + (size_t)((uint32_t)kit * (uint32_t)(C::BK * C::ES)) * (uint32_t)g.N;
#pragma unroll
        for (int j = 0; j < C::B_LD; j++) {
            if (j < j0 || j >= j1) continue;
            if (!TAIL) {
                if (NT) lds_dma16_nt(B, b_off[j], lds + (j * C::NW + wave) * 1024);
                else lds_dma16(B, b_off[j], lds + (j * C::NW + wave) * 1024);
            } else {
                const int p = (j * C::NW + wave) * 64 + lane;
                const char* src = kit * C::BK + p / C::CPB < g.K ? B + b_off[j] : reinterpret_cast<const char*>(g_zero_piece);
                lds_dma16_ptr(src, lds + (j * C::NW + wave) * 1024);
            }
        }
    }
};

// k-consecutive elements of one B column out of the row-major [k][n] LDS image.  16-bit: the
// transposing read hands lane j of each 16-lane group column j of a 4 x 16 block whose rows are
// addressed by lanes 4e..4e+3 of the group (4 k per read).  8-bit: an 8 x 16 block whose rows are
// addressed by lanes 2e, 2e+1 (8 k per read).
__device__ __forceinline__ uint2 read_b_tr16(const unsigned char* p) {
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p));
    return __builtin_bit_cast(uint2, v);
}
__device__ __forceinline__ i32x2 read_b_tr8(const unsigned char* p) {
    return __builtin_amdgcn_ds_read_tr8_b64_v2i32((i32x2 __attribute__((address_space(3)))*)(p));
}

// Lane-constant parts of the operand addresses inside a stage.
template <class C> struct FragMap {
    uint32_t a_kk[C::KK][C::APL];   // byte offsets of this lane's A piece(s) for k-step kk, block row 0
    uint32_t b_ni[C::NI];           // byte offset of this lane's first B read for block column ni, k-step 0
    __device__ __forceinline__ void init() {
        const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
        const int wm = wave / C::WN, wn = wave % C::WN;
        const int row = wm * C::WTM + lane % C::MF;          // + mi * MF keeps row % 16
#pragma unroll
        for (int kk = 0; kk < C::KK; kk++)
#pragma unroll
            for (int i = 0; i < C::APL; i++)
                a_kk[kk][i] = (row * C::CPA + ((kk * (C::KM / C::PE) + (lane / C::MF) * C::APL + i) ^ swz_a<C::CPA>(row))) * 16;
        // rows of one transposing read: 4 (16-bit) or 8 (8-bit); later reads and k-steps add multiples of that
        const int krow = C::KPL * (lane / C::MF) + (C::FP8 ? (lane % 16) / 2 : (lane % 16) / 4);
#pragma unroll
        for (int ni = 0; ni < C::NI; ni++) {
            const int col = wn * C::WTN + ni * C::MF + 16 * ((lane % C::MF) / 16) + (C::FP8 ? 8 * (lane % 2) : 4 * (lane % 4));
            b_ni[ni] = (krow * C::CPB + ((col / C::PE) ^ swz_b<C::FP8>(krow))) * 16 + (col % C::PE) * C::ES;
        }
    }
};

template <class C, bool FP8 = C::FP8> struct Frags;
template <class C> struct Frags<C, false> {
    uint4 a[C::MI], b[C::NI];
    // The LDS reads of one k-step one at a time, in the order in which the matrix-core work needs
    // them (block row 0, all block columns, the other block rows): read number r of READS.
    static constexpr int READS = C::MI + 2 * C::NI;
    __device__ __forceinline__ void load_one(const unsigned char* a_stage, const unsigned char* b_stage, const FragMap<C>& fm, int kk, int r) {
        if (r == 0 || r > 2 * C::NI) {
            const int mi = r == 0 ? 0 : r - 2 * C::NI;
            a[mi] = *reinterpret_cast<const uint4*>(a_stage + fm.a_kk[kk][0] + mi * C::MF * C::CPA * 16);
        } else {
            const int ni = (r - 1) / 2, h = (r - 1) % 2;
            const uint2 v = read_b_tr16(b_stage + fm.b_ni[ni] + kk * C::KM * C::CPB * 16 + h * 4 * C::CPB * 16);
            if (h == 0) { b[ni].x = v.x; b[ni].y = v.y; } else { b[ni].z = v.x; b[ni].w = v.y; }
        }
    }
    __device__ __forceinline__ void load(const unsigned char* a_stage, const unsigned char* b_stage, const FragMap<C>& fm, int kk) {
#pragma unroll
        for (int mi = 0; mi < C::MI; mi++)
            a[mi] = *reinterpret_cast<const uint4*>(a_stage + fm.a_kk[kk][0] + mi * C::MF * C::CPA * 16);
#pragma unroll
        for (int ni = 0; ni < C::NI; ni++) {
            const unsigned char* p = b_stage + fm.b_ni[ni] + kk * C::KM * C::CPB * 16;
            const uint2 lo = read_b_tr16(p), hi = read_b_tr16(p + 4 * C::CPB * 16);
            b[ni] = make_uint4(lo.x, lo.y, hi.x, hi.y);
        }
    }
};
template <class C> struct Frags<C, true> {
    i32x8 a[C::MI], b[C::NI];
    static constexpr int READS = 2 * C::MI + 4 * C::NI;
    __device__ __forceinline__ void load_one(const unsigned char* a_stage, const unsigned char* b_stage, const FragMap<C>& fm, int kk, int r) {
        if (r < 2 || r >= 2 + 4 * C::NI) {
            const int mi = r < 2 ? 0 : (r - 4 * C::NI) / 2, h = r % 2;
            const uint4 v = *reinterpret_cast<const uint4*>(a_stage + fm.a_kk[kk][h] + mi * C::MF * C::CPA * 16);
            a[mi][4 * h] = (int)v.x; a[mi][4 * h + 1] = (int)v.y; a[mi][4 * h + 2] = (int)v.z; a[mi][4 * h + 3] = (int)v.w;
        } else {
            const int ni = (r - 2) / 4, q = (r - 2) % 4;
            const i32x2 v = read_b_tr8(b_stage + fm.b_ni[ni] + kk * C::KM * C::CPB * 16 + q * 8 * C::CPB * 16);
            b[ni][2 * q] = v[0]; b[ni][2 * q + 1] = v[1];
        }
    }
    __device__ __forceinline__ void load(const unsigned char* a_stage, const unsigned char* b_stage, const FragMap<C>& fm, int kk) {
#pragma unroll
        for (int mi = 0; mi < C::MI; mi++) {
            const uint4 lo = *reinterpret_cast<const uint4*>(a_stage + fm.a_kk[kk][0] + mi * C::MF * C::CPA * 16);
            const uint4 hi = *reinterpret_cast<const uint4*>(a_stage + fm.a_kk[kk][1] + mi * C::MF * C::CPA * 16);
            a[mi] = i32x8{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
        }
#pragma unroll
        for (int ni = 0; ni < C::NI; ni++) {
            const unsigned char* p = b_stage + fm.b_ni[ni] + kk * C::KM * C::CPB * 16;
            const i32x2 q0 = read_b_tr8(p), q1 = read_b_tr8(p + 8 * C::CPB * 16);
            const i32x2 q2 = read_b_tr8(p + 16 * C::CPB * 16), q3 = read_b_tr8(p + 24 * C::CPB * 16);
            b[ni] = i32x8{q0[0], q0[1], q1[0], q1[1], q2[0], q2[1], q3[0], q3[1]};
        }
    }
};

__device__ __forceinline__ u16 to_bf16_bits(float f) {
    return __builtin_bit_cast(u16, (__bf16)f);     // round to nearest even (one hardware instruction on gfx950)
}

template <class C, int LATER, int EXTRA = 0> __device__ __forceinline__ void wait_stage(int later) {
    // wait until the loads of the wanted stage have landed, given how many stages follow it; EXTRA:
    // vector-memory instructions that this wave is known to have issued after those loads besides the
    // later stages' loads (the counter retires in issue order, so they may stay in flight)
    if (LATER == 0 || later >= LATER) wait_vmcnt<(C::in_flight(LATER) + EXTRA < 63 ? C::in_flight(LATER) + EXTRA : 63)>();
    else wait_stage<C, (LATER > 0 ? LATER - 1 : 0), EXTRA>(later);
}

// The matrix-core work of one k-step.
// TR: pass the B block first and the A block second, which yields the transposed result block.
template <class C, bool TR>
__device__ __forceinline__ void mma_step(const Frags<C>& f, typename Mfma<C::DT, C::MF>::Acc (&acc)[C::MI][C::NI]) {
#pragma unroll
    for (int mi = 0; mi < C::MI; mi++)
#pragma unroll
        for (int ni = 0; ni < C::NI; ni++)
            acc[mi][ni] = TR ? Mfma<C::DT, C::MF>::run(f.b[ni], f.a[mi], acc[mi][ni]) : Mfma<C::DT, C::MF>::run(f.a[mi], f.b[ni], acc[mi][ni]);
}

// All k-steps of one stage, for the register-staged path: the operands of step kk+1 are read from
// LDS while the matrix cores work on step kk.
template <class C, bool TR>
__device__ __forceinline__ void mac_stage(const unsigned char* a_stage, const unsigned char* b_stage, const FragMap<C>& fm,
                                          typename Mfma<C::DT, C::MF>::Acc (&acc)[C::MI][C::NI]) {
    Frags<C> f[2];
    f[0].load(a_stage, b_stage, fm, 0);
#pragma unroll
    for (int kk = 0; kk < C::KK; kk++) {
        if (kk + 1 < C::KK) f[(kk + 1) & 1].load(a_stage, b_stage, fm, kk + 1);
        mma_step<C, TR>(f[kk & 1], acc);
    }
}

// Slice `step` of `steps` of request batch j of a segment (k-iterations k_begin .. k_begin + nk - 1 of a
// tile): the B tile of stage j + NSB, then the A tile of stage j + NSA, into ring slots slot_b / slot_a.
// STEADY: the caller knows that both stages exist and lie entirely inside K.
template <class C, bool STEADY, bool NT>
__device__ __forceinline__ void issue_requests(const GemmArgs& g, const DmaMap<C>& dm, uint32_t lds0, int k_begin, int nk, int full_k,
                                               int j, int slot_a, int slot_b, int step, int steps) {
    const int ib = j + C::NSB, ia = j + C::NSA;
    const int q0 = step * C::LPS / steps, q1 = (step + 1) * C::LPS / steps;
    const int b0 = q0 < C::B_LD ? q0 : C::B_LD, b1 = q1 < C::B_LD ? q1 : C::B_LD;
    const int a0 = q0 > C::B_LD ? q0 - C::B_LD : 0, a1 = q1 > C::B_LD ? q1 - C::B_LD : 0;
    if ((STEADY || (ib >= 0 && ib < nk)) && b1 > b0) {
        const uint32_t lds = lds0 + C::B_RING + slot_b * C::B_BYTES;
        if (STEADY || k_begin + ib < full_k) dm.template issue_b<false, NT>(g, k_begin + ib, lds, b0, b1);
        else dm.template issue_b<true, NT>(g, k_begin + ib, lds, b0, b1);
    }
    if ((STEADY || (ia >= 0 && ia < nk)) && a1 > a0) {
        const uint32_t lds = lds0 + slot_a * C::A_BYTES;
        if (STEADY || k_begin + ia < full_k) dm.template issue_a<false>(g, k_begin + ia, lds, a0, a1);
        else dm.template issue_a<true>(g, k_begin + ia, lds, a0, a1);
    }
}

// The first requests of a segment on the LDS-DMA path: the batches that stages before the first would have
// requested, all but the last (that one goes out in the MAC loop's first trip).  The ring must be free: no
// wave may still read operands of the previous segment.  Called either at the start of the MAC loop or -
// for the segment after the current one - before the current tile's fix-up and epilogue, so that the
// first loads travel while the tile is stored.
template <class C, bool NT>
__device__ __forceinline__ void mac_prefetch(const GemmArgs& g, int m0, int n0, int k_begin, int k_end, unsigned char* smem, const DmaMap<C>& dm) {
    const uint32_t lds0 = (uint32_t)(size_t)(lds_byte*)smem;
    const int nk = k_end - k_begin, full_k = g.K / C::BK;
#pragma unroll
    for (int j = -C::NSA; j <= -2; j++)
        issue_requests<C, false, NT>(g, dm, lds0, k_begin, nk, full_k, j, (j + C::NSA) % C::NSA, (j + 2 * C::NSB) % C::NSB, 0, 1);
}

// MAC loop of one segment (Algorithm 1's MAC-loop call): k-iterations [k_begin, k_end) of one tile.
//
// Software pipeline of the LDS-DMA path.  Stage s (one k-iteration) lives in A ring slot s % NSA and
// B ring slot s % NSB.  The barrier that hands stage i+1 to the waves sits one k-step *before* the
// end of stage i: by then every wave has read the operands of stage i's last k-step into registers,
// so (1) stage i's slots can be refilled at once (with stages i+NSB / i+NSA), (2) the operands of
// stage i+1's first k-step are read while the matrix cores still work on stage i's last one, and
// (3) the time a wave spends at the barrier is covered by matrix-core work already queued.
// prefetched / stores_in_flight (LDS-DMA path only): prefetched says that mac_prefetch has already been
// called for this segment; stores_in_flight that this wave has since issued exactly C::EPILOGUE_STORES (or
// more) other vector-memory instructions, which the first wait may leave in flight.  (The per-tile
// addressing is worked out again here rather than kept from the prefetch: kept in registers across the
// epilogue it gets spilled, and a reload pending at the loop's entry makes the compiler wait for every
// outstanding load inside the steady-state trips.)
template <class C, bool ALIGNED, bool TR, bool NT>
__device__ __forceinline__ void mac_loop(const GemmArgs& g, int m0, int n0, int k_begin, int k_end,
                                         unsigned char* smem, const FragMap<C>& fm,
                                         typename Mfma<C::DT, C::MF>::Acc (&acc)[C::MI][C::NI],
                                         bool prefetched, bool stores_in_flight) {
    const int nk = k_end - k_begin;
    if (C::DIRECT && ALIGNED) {
        static_assert(!C::DIRECT || C::KK % 2 == 0, "operand double buffering assumes an even number of k-steps");
        const uint32_t lds0 = (uint32_t)(size_t)(lds_byte*)smem;
        const int full_k = g.K / C::BK;             // iterations below this index are entirely inside K
        DmaMap<C> dm;
        dm.init(g, m0, n0);
        if (!prefetched) mac_prefetch<C, NT>(g, m0, n0, k_begin, k_end, smem, dm);
        // request batch j (issued after the barrier of stage j): B tile of stage j+NSB, then A tile of
        // stage j+NSA, into the slots of stage j; step / steps select a slice of the batch
        auto issue_batch = [&](int j, int slot_a, int slot_b, int step, int steps, auto steady) {
            issue_requests<C, decltype(steady)::value, NT>(g, dm, lds0, k_begin, nk, full_k, j, slot_a, slot_b, step, steps);
        };
        Frags<C> f[2];
        int ca = C::NSA - 1, cb = C::NSB - 1;        // ring slots of stage i (i = -1: the slots batch -1 fills)
        // one trip = [barrier that hands over stage i+1] [operands of stage i+1's first k-step]
        //            [requests of batch i, sliced over the k-steps] [last k-step of stage i]
        //            [k-steps 0 .. KK-2 of stage i+1, each preceded by the operand reads of the next one].
        // FIRST: i = -1, no stage i yet.  NEXT: whether a stage i+1 exists.  Where registers allow two
        // operand sets (PIN_ORDER), NEXT is a compile-time fact - the steady-state loop body then has
        // no joins between the LDS reads and the matrix-core work (the compiler's wait-count
        // bookkeeping merges conservatively at joins) - and scheduling barriers keep the reads of
        // k-step kk+1 ahead of the matrix-core work of k-step kk.  Otherwise the compiler is left
        // to order reads and matrix-core work so that one operand set suffices.
        // FINE: one k-step written out slot by slot.  Slot s = [matrix-core instruction s of the k-step
        // on operand set `cur`] [its share of the LDS reads that fill `nxt` with the operands of k-step
        // kk_next of stage i+1: the reads go into the first three quarters of the slots, so that the
        // last of them has long landed when the k-step ends] [its share of request batch i, spread
        // evenly over all slots of the trip].  A scheduling barrier after every slot keeps that order:
        // a wave that has a SIMD to itself issues about five other instructions in the shadow of one
        // matrix-core instruction, and issued in a block they would drain the matrix-core pipe.
        auto fine_step = [&](int i, int step, auto mma, auto read, const Frags<C>& cur, Frags<C>& nxt,
                             const unsigned char* a_next, const unsigned char* b_next, int kk_next, auto steady) {
            constexpr int NM = C::MI * C::NI, R = Frags<C>::READS, NRS = NM * 3 / 4 > 0 ? NM * 3 / 4 : 1;
#pragma unroll
            for (int s = 0; s < NM; s++) {
                const int mi = s / C::NI, ni = s % C::NI;
                if (decltype(mma)::value)
                    acc[mi][ni] = TR ? Mfma<C::DT, C::MF>::run(cur.b[ni], cur.a[mi], acc[mi][ni]) : Mfma<C::DT, C::MF>::run(cur.a[mi], cur.b[ni], acc[mi][ni]);
                if (decltype(read)::value && s < NRS) {
#pragma unroll
                    for (int r = s * R / NRS; r < (s + 1) * R / NRS; r++) nxt.load_one(a_next, b_next, fm, kk_next, r);
                }
                issue_batch(i, ca, cb, step * NM + s, C::KK * NM, steady);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        auto trip = [&](int i, auto first, auto next, auto steady) {
            constexpr bool FIRST = decltype(first)::value;
            constexpr bool STEADY = decltype(steady)::value;     // batch i's stages exist and need no K-tail handling, and at least NSA - 1 stages follow stage i + 1
            constexpr int NEXT = decltype(next)::value;          // 1 / 0: known, -1: decided at run time
            const bool has_next = NEXT < 0 ? i + 1 < nk : NEXT == 1;
            const int na = ca + 1 == C::NSA ? 0 : ca + 1, nb = cb + 1 == C::NSB ? 0 : cb + 1;   // slots of stage i+1
            const unsigned char* a_next = smem + na * C::A_BYTES;
            const unsigned char* b_next = smem + C::B_RING + nb * C::B_BYTES;
            if constexpr (C::FINE) {
                static_assert(!C::FINE || NEXT >= 0, "known at compile time under PIN_ORDER");
                if (NEXT) {
                    if (STEADY) wait_vmcnt<C::in_flight(C::NSA - 1)>();
                    else if (FIRST && stores_in_flight) wait_stage<C, C::NSA - 1, C::EPILOGUE_STORES>(nk - 2 - i);
                    else wait_stage<C, C::NSA - 1>(nk - 2 - i);
                    __syncthreads();
                }
                __builtin_amdgcn_sched_barrier(0);
                // last k-step of stage i, with the reads of stage i+1's first k-step
                fine_step(i, 0, std::integral_constant<bool, !FIRST>(), std::integral_constant<bool, NEXT == 1>(), f[1], f[0], a_next, b_next, 0, steady);
                if (NEXT) {
#pragma unroll
                    for (int kk = 0; kk < C::KK - 1; kk++)
                        fine_step(i, kk + 1, std::true_type(), std::true_type(), f[kk & 1], f[(kk + 1) & 1], a_next, b_next, kk + 1, steady);
                }
                ca = na;
                cb = nb;
                return;
            }
            if (has_next) {
                if (STEADY) wait_vmcnt<C::in_flight(C::NSA - 1)>();
                else if (FIRST && stores_in_flight) wait_stage<C, C::NSA - 1, C::EPILOGUE_STORES>(nk - 2 - i);
                else wait_stage<C, C::NSA - 1>(nk - 2 - i);   // stage i+1 has landed (this wave's share)
                __syncthreads();                         // ... and everybody's; stage i's slots are free
                f[0].load(a_next, b_next, fm, 0);
            }
            issue_batch(i, ca, cb, 0, C::KK, steady);
            if (C::PIN_ORDER) __builtin_amdgcn_sched_barrier(0);
            if (!FIRST) mma_step<C, TR>(f[1], acc);          // last k-step of stage i
            if (has_next) {
#pragma unroll
                for (int kk = 0; kk < C::KK - 1; kk++) {
                    if (C::PIN_ORDER) __builtin_amdgcn_sched_barrier(0);
                    f[(kk + 1) & 1].load(a_next, b_next, fm, kk + 1);
                    issue_batch(i, ca, cb, kk + 1, C::KK, steady);
                    if (C::PIN_ORDER) __builtin_amdgcn_sched_barrier(0);
                    mma_step<C, TR>(f[kk & 1], acc);
                }
            }
            ca = na;
            cb = nb;
        };
        typedef std::integral_constant<int, 1> Yes;
        typedef std::integral_constant<int, 0> No;
        typedef std::integral_constant<int, -1> AtRunTime;
        // Trips 0 .. n_steady-1 request stages that exist and lie inside K: their body carries neither
        // range checks nor the K-tail variant of the requests, and waits with a constant count.
        int n_steady = (full_k - k_begin < nk ? full_k - k_begin : nk) - C::NSA;
        if (n_steady < 0) n_steady = 0;
        if constexpr (C::PIN_ORDER) {
            trip(-1, std::true_type(), Yes(), std::false_type());
            int i = 0;
            for (; i < n_steady; i++) trip(i, std::false_type(), Yes(), std::true_type());
            for (; i < nk - 1; i++) trip(i, std::false_type(), Yes(), std::false_type());
            trip(nk - 1, std::false_type(), No(), std::false_type());
        } else {
            trip(-1, std::true_type(), AtRunTime(), std::false_type());
            int i = 0;
            for (; i < n_steady; i++) trip(i, std::false_type(), Yes(), std::true_type());
            for (; i < nk; i++) trip(i, std::false_type(), AtRunTime(), std::false_type());
        }
        __syncthreads();                             // all reads done before the next segment refills
    } else {
        // Register-staged path, two LDS slots.  Where registers allow (STAGE_AHEAD) the pieces of
        // stage k+1 are requested before the matrix-core work of stage k and parked after it.
        StagedFill<C, ALIGNED> sf;
        if (C::STAGE_AHEAD) sf.fetch(g, m0, n0, k_begin);
        for (int k = k_begin; k < k_end; k++) {
            const int slot = (k - k_begin) & 1;
            unsigned char* a_stage = smem + slot * C::A_BYTES;
            unsigned char* b_stage = smem + C::B_RING + slot * C::B_BYTES;
            if (!C::STAGE_AHEAD) sf.fetch(g, m0, n0, k);
            sf.park(a_stage, b_stage);
            __syncthreads();      // also: every wave is done with the other slot (stage k-1)
            if (C::STAGE_AHEAD && k + 1 < k_end) sf.fetch(g, m0, n0, k + 1);
            mac_stage<C, TR>(a_stage, b_stage, fm, acc);
        }
        __syncthreads();
    }
}

// Wait until `count` contributors have raised their flags: workgroups first, first + stride, ...
// The lanes of the calling wave watch up to 64 flags at a time, one flag each, so the wait costs one
// round trip however many flags there are.  A lane that has seen its flag takes it down again:
// every flag is watched by exactly one lane of one waiting workgroup, so all flags are back at zero
// when the kernel ends and the next launch (or a replay of a captured launch) starts from the same
// state.  The wait is bounded: after spin_limit unsuccessful polls it is recorded in the status word
// and given up.
__device__ __forceinline__ void wait_flags(const GemmArgs& g, int first, int count, int stride) {
    const int lane = threadIdx.x % 64;
    uint32_t polls = 0;
    for (int base = 0; base < count; base += 64) {
        const bool mine = base + lane < count;
        uint32_t* flag = g.flags + (size_t)(first + (mine ? base + lane : 0) * stride) * (SK_FLAG_STRIDE / 4);
        bool seen = !mine;
        while (true) {
            if (!seen && __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
                seen = true;
                __hip_atomic_store(flag, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (__all(seen)) break;
            if (polls++ >= g.spin_limit) {
                if (lane == 0) __hip_atomic_store(g.status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            __builtin_amdgcn_s_sleep(2);
        }
    }
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>)
template <int N, class F, int... I>
__device__ __forceinline__ void for_each_below_impl(F&& f, std::integer_sequence<int, I...>) { (f(std::integral_constant<int, I>()), ...); }
template <int N, class F>
__device__ __forceinline__ void for_each_below(F&& f) { for_each_below_impl<N>(f, std::make_integer_sequence<int, N>()); }

// blk += this block's share of the parked partial tiles src, src + stride, ... (`count` of them), in
// that order, GB contributors per round trip (GB * ACC registers of loads in flight).
template <class C, int GB>
__device__ __forceinline__ void add_block_partials(typename Mfma<C::DT, C::MF>::Acc& blk, const float* src, int count, ptrdiff_t stride) {
    int c = 0;
    for (; c + GB <= count; c += GB, src += GB * stride) {
        float v[GB][C::ACC];
#pragma unroll
        for (int j = 0; j < GB; j++)
#pragma unroll
            for (int r = 0; r < C::ACC; r++)
                v[j][r] = __hip_atomic_load(src + j * stride + r * C::THREADS, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_sched_barrier(0);     // all loads of the round trip in flight before the first addition waits for one
#pragma unroll
        for (int j = 0; j < GB; j++)
#pragma unroll
            for (int r = 0; r < C::ACC; r++) blk[r] += v[j][r];
    }
    for (; c < count; c++, src += stride) {
        float v[C::ACC];
#pragma unroll
        for (int r = 0; r < C::ACC; r++)
            v[r] = __hip_atomic_load(src + r * C::THREADS, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int r = 0; r < C::ACC; r++) blk[r] += v[r];
    }
}

// sum += the parked partial tiles src, src + stride, ... (`count` of them, this lane's share), in
// that order.  Tiles with at most 64 accumulators per lane: a contributor's whole share is
// fetched at once and G contributors per round trip (about 64 registers of loads in flight).
// Bigger tiles: block by block, the shares of two contributors per round trip.
template <class C>
__device__ __forceinline__ void add_partials(typename Mfma<C::DT, C::MF>::Acc (&sum)[C::MI][C::NI], const float* src, int count, ptrdiff_t stride) {
    if constexpr (C::ACC_REGS > 64) {
#pragma unroll
        for (int mi = 0; mi < C::MI; mi++)
#pragma unroll
            for (int ni = 0; ni < C::NI; ni++) {
                add_block_partials<C, 32 / C::ACC>(sum[mi][ni], src + ((mi * C::NI + ni) * C::ACC) * C::THREADS, count, stride);
                __builtin_amdgcn_sched_barrier(0);
            }
    } else {
    constexpr int G = 64 / C::ACC_REGS < 8 ? 64 / C::ACC_REGS : 8;
    auto add_group = [&](const float* p, auto cnt) {
        constexpr int CNT = decltype(cnt)::value;
        float v[CNT][C::ACC_REGS];
#pragma unroll
        for (int j = 0; j < CNT; j++)
#pragma unroll
            for (int i = 0; i < C::ACC_REGS; i++)
                v[j][i] = __hip_atomic_load(p + j * stride + i * C::THREADS, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_sched_barrier(0);     // all loads of the round trip in flight before the first addition waits for one
#pragma unroll
        for (int j = 0; j < CNT; j++)
#pragma unroll
            for (int mi = 0; mi < C::MI; mi++)
#pragma unroll
                for (int ni = 0; ni < C::NI; ni++)
#pragma unroll
                    for (int r = 0; r < C::ACC; r++) sum[mi][ni][r] += v[j][(mi * C::NI + ni) * C::ACC + r];
    };
    int c = 0;
    for (; c + G <= count; c += G, src += G * stride) add_group(src, std::integral_constant<int, G>());
    // the 1 .. G-1 contributors left over: one round trip for all of them (the order of the additions is
    // the same whatever the grouping)
    for_each_below<G>([&](auto r) {
        if (decltype(r)::value > 0 && count - c == decltype(r)::value) add_group(src, std::integral_constant<int, decltype(r)::value < 1 ? 1 : decltype(r)::value>());
    });
    }
}

// Two fp32 values -> one register of two 16-bit values, round to nearest even (gfx950 converts a
// pair to bf16 with one instruction).
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2{lo, hi}), bf16x2));
}
__device__ __forceinline__ uint32_t pack_f16(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2{lo, hi}), f16x2));
}

// Convert and store one accumulator block.
// TR (transposed blocks; used when rows of D start on 16-byte boundaries and N is a multiple of 8):
// lane l holds row `row` (= block row l % MF) and in registers 4q..4q+3 the columns
// col0 + 4*KG*q + {0..3}, col0 already including 4 * (l / MF).  16-bit outputs of the 32 x 32 block
// exchange register pairs between lanes l and l + 32, after which a lane owns 8 consecutive columns
// = one 16-byte store; fp32 outputs store 4 columns = 16 bytes per q.  A group of 4 (8) columns
// starting at a multiple of 4 (8) is then inside N as a whole or not at all.
// Not TR: lane l holds column `col0` (= block column l % MF) and in register r the row
// row + 4*KG*(r/4) + r%4, `row` already including 4 * (l / MF); stored element by element, the
// lanes of one store instruction side by side in a row of D.
template <class C, int OUT, bool EDGE, bool TR>
__device__ __forceinline__ void store_block(const GemmArgs& g, int row, int col0, const typename Mfma<C::DT, C::MF>::Acc& blk) {
    constexpr int Q = C::ACC / 4, QS = 4 * C::KG;    // register groups per lane, distance between their rows / columns
    if constexpr (!TR) {
#pragma unroll
        for (int r = 0; r < C::ACC; r++) {
            const int rr = row + (r / 4) * QS + r % 4;
            if (!EDGE || (rr < g.M && col0 < g.N)) {
                const size_t o = (size_t)((uint32_t)rr * (uint32_t)g.N + (uint32_t)col0);
                if (OUT == SK_F32) static_cast<float*>(g.D)[o] = blk[r];
                else if (OUT == SK_BF16) static_cast<u16*>(g.D)[o] = to_bf16_bits(blk[r]);
                else static_cast<_Float16*>(g.D)[o] = (_Float16)blk[r];
            }
        }
        return;
    }
    const bool row_ok = !EDGE || row < g.M;
    const uint32_t row_off = (uint32_t)row * (uint32_t)g.N;
    if constexpr (OUT == SK_F32) {
#pragma unroll
        for (int q = 0; q < Q; q++) {
            const int col = col0 + q * QS;
            if (row_ok && (!EDGE || col < g.N))
                *reinterpret_cast<f32x4*>(static_cast<float*>(g.D) + (size_t)(row_off + (uint32_t)col)) =
                    f32x4{blk[4 * q], blk[4 * q + 1], blk[4 * q + 2], blk[4 * q + 3]};
        }
    } else {
        uint32_t w[Q][2];
#pragma unroll
        for (int q = 0; q < Q; q++) {
            w[q][0] = OUT == SK_BF16 ? pack_bf16(blk[4 * q], blk[4 * q + 1]) : pack_f16(blk[4 * q], blk[4 * q + 1]);
            w[q][1] = OUT == SK_BF16 ? pack_bf16(blk[4 * q + 2], blk[4 * q + 3]) : pack_f16(blk[4 * q + 2], blk[4 * q + 3]);
        }
        if constexpr (C::MF == 32) {
            // groups q (lanes below 32 keep theirs) and q + 1 (lanes from 32 up keep theirs): after the
            // exchange a lane holds columns 8 * (q + l / 32) .. + 7 of its row, relative to the block
            const int half = threadIdx.x % 64 / 32;
#pragma unroll
            for (int q = 0; q < Q; q += 2) {
                const u32x2 d0 = __builtin_amdgcn_permlane32_swap(w[q][0], w[q + 1][0], false, false);
                const u32x2 d1 = __builtin_amdgcn_permlane32_swap(w[q][1], w[q + 1][1], false, false);
                const int col = col0 - 4 * half + 8 * (q + half);
                if (row_ok && (!EDGE || col < g.N))
                    *reinterpret_cast<u32x4*>(static_cast<u16*>(g.D) + (size_t)(row_off + (uint32_t)col)) = u32x4{d0[0], d1[0], d0[1], d1[1]};
            }
        } else {
#pragma unroll
            for (int q = 0; q < Q; q++) {
                const int col = col0 + q * QS;
                if (row_ok && (!EDGE || col < g.N))
                    *reinterpret_cast<u32x2*>(static_cast<u16*>(g.D) + (size_t)(row_off + (uint32_t)col)) = u32x2{w[q][0], w[q][1]};
            }
        }
    }
}

// Epilogue of a tile's owner (or of an unsplit tile, n_contrib = 0): add the parked partials of the
// contributors part0, part0 + part_stride, ... (a fixed order: away from the owner in k), convert and store.  OUT selects the
// output type, EDGE adds the bounds checks, TR says that the blocks are transposed (see store_block).
// row0 / col0: the lane's (first) row and (first) column in the wave's first block.  The big tiles
// work one block at a time, which keeps their register need flat.
template <class C, int OUT, bool EDGE, bool TR>
__device__ __forceinline__ void reduce_and_store(const GemmArgs& g, int row0, int col0, const float* part0, int n_contrib,
                                                 ptrdiff_t part_stride, const typename Mfma<C::DT, C::MF>::Acc (&acc)[C::MI][C::NI]) {
    typedef typename Mfma<C::DT, C::MF>::Acc Acc;
    // Tiles with few accumulators per lane fetch a contributor's whole share at once (one round trip
    // per contributor instead of one per block and contributor); the big tiles have no registers for that.
    constexpr bool WHOLE = C::ACC_REGS <= 64;
    Acc sum[WHOLE ? C::MI : 1][WHOLE ? C::NI : 1];
    if constexpr (WHOLE) {
#pragma unroll
        for (int mi = 0; mi < C::MI; mi++)
#pragma unroll
            for (int ni = 0; ni < C::NI; ni++) sum[mi][ni] = acc[mi][ni];
        add_partials<C>(sum, part0, n_contrib, part_stride);
    }
#pragma unroll
    for (int mi = 0; mi < C::MI; mi++)
#pragma unroll
        for (int ni = 0; ni < C::NI; ni++) {
            Acc blk;
            if constexpr (WHOLE) {
                blk = sum[mi][ni];
            } else {
                blk = acc[mi][ni];
                const float* src = part0 + ((mi * C::NI + ni) * C::ACC) * C::THREADS;
                // two contributors' shares of this block per round trip (all the registers allow), added in
                // the same fixed order as one by one
                add_block_partials<C, 32 / C::ACC>(blk, src, n_contrib, part_stride);
            }
            store_block<C, OUT, EDGE, TR>(g, row0 + mi * C::MF, col0 + ni * C::MF, blk);
            __builtin_amdgcn_sched_barrier(0);
        }
}

// Atomic fix-up (the accumulation step of Algorithm 1): a segment that covers only part of the tile's
// K-iterations adds its accumulators into the zero-initialised fp32 image with atomic adds; a
// segment that covers the whole tile stores them.  Blocks are not transposed here: the lanes of
// one atomic instruction then sit side by side in a row of the image (two cache lines per
// instruction instead of 32).
template <class C, bool EDGE>
__device__ __forceinline__ void add_to_image(const GemmArgs& g, int row0, int col0, bool partial,
                                             const typename Mfma<C::DT, C::MF>::Acc (&acc)[C::MI][C::NI]) {
#pragma unroll
    for (int mi = 0; mi < C::MI; mi++)
#pragma unroll
        for (int ni = 0; ni < C::NI; ni++) {
            const int col = col0 + ni * C::MF;
#pragma unroll
            for (int r = 0; r < C::ACC; r++) {
                const int row = row0 + mi * C::MF + (r / 4) * (4 * C::KG) + r % 4;
                if (!EDGE || (row < g.M && col < g.N)) {
                    float* p = g.image + (size_t)((uint32_t)row * (uint32_t)g.N + (uint32_t)col);
                    if (partial) unsafeAtomicAdd(p, acc[mi][ni][r]);
                    else *p = acc[mi][ni][r];
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
}

template <class C, bool ALIGNED, bool ATOMIC = false>
__global__ __launch_bounds__(C::THREADS) void streamk_gemm_kernel(GemmArgs g) {
    extern __shared__ __align__(1024) unsigned char smem[];
    typedef typename Mfma<C::DT, C::MF>::Acc Acc;
    const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
    const int wm = wave / C::WN, wn = wave % C::WN;
    const int x = logical_wg(blockIdx.x, g.grid, g.xcd_remap);
    // transposed accumulator blocks (vector stores) where D's rows are 16-byte aligned; the atomic
    // fix-up and the element-wise stores of unaligned problems want the lanes side by side in a row
    constexpr bool TR = ALIGNED && !ATOMIC;
    FragMap<C> fm;
    fm.init();

    // Algorithm 1 (clamped): this workgroup's share of the Stream-K iterations
    int it = x * g.ipw, it_end = it + g.ipw;
    if (it > g.sk_iters) it = g.sk_iters;
    if (it_end > g.sk_iters) it_end = g.sk_iters;
    int dp_tile = g.sk_tiles + x;   // data-parallel tiles come after the Stream-K work
    // k-aligned order: a share that contains a tile boundary is run as its whole tiles first, then
    // the head piece of its last tile (k from 0), then the tail piece of its first tile.  Whole
    // tiles and head pieces then start at k = 0 at multiples of a tile's duration in every workgroup,
    // whatever its offset in the iteration space, which keeps the operand blocks that neighbouring
    // tiles share in L2; and the tail piece, whose workgroup owns the tile, comes last, when the
    // pieces before it in k have long been parked.
    int next_b = it_end, next_e = it_end, last_b = it_end, last_e = it_end;     // the sub-ranges after [it, it_end)
    if (g.k_aligned && it < it_end) {
        const int first_full = (int)fast_div((uint32_t)it + (uint32_t)g.ipt - 1, g.div_ipt) * g.ipt;
        const int last_full = (int)fast_div((uint32_t)it_end, g.div_ipt) * g.ipt;
        if (first_full <= last_full) {
            next_b = last_full; next_e = it_end;     // head piece (may be empty)
            last_b = it; last_e = first_full;        // tail piece (may be empty)
            it = first_full; it_end = last_full;     // whole tiles (may be none)
        }
    }
    // The next segment of this workgroup: tile index, k-iterations and the tile's origin; false when the work is done.
    auto next_segment = [&](int& tile, int& k_begin, int& k_end, int& m0, int& n0) -> bool {
        if (it >= it_end) { it = next_b; it_end = next_e; next_b = last_b; next_e = last_e; last_b = last_e; }
        if (it >= it_end) { it = next_b; it_end = next_e; next_b = last_b; next_e = last_e; last_b = last_e; }
        const bool dp_now = dp_tile < g.tiles && (g.dp_first || it >= it_end);
        if (!dp_now && it < it_end) {            // Algorithm 1: cut the share at tile boundaries
            tile = (int)fast_div((uint32_t)it, g.div_ipt);
            const int tile_first = tile * g.ipt;
            k_begin = it - tile_first;
            const int stop = it_end < tile_first + g.ipt ? it_end : tile_first + g.ipt;
            k_end = stop - tile_first;
            it = stop;
        } else if (dp_now) {
            tile = dp_tile; k_begin = 0; k_end = g.ipt;
            dp_tile += g.grid;
        } else {
            return false;
        }
        int tm, tn;
        if (g.tile_order == SK_ORDER_ROW_MAJOR) {
            tm = (int)fast_div((uint32_t)tile, g.div_tiles_n);
            tn = tile - tm * g.tiles_n;
        } else {                                 // bands of 8 tile rows, walked column by column
            const uint32_t per_band = (uint32_t)(SK_GROUP_ROWS * g.tiles_n);
            const uint32_t band = fast_div((uint32_t)tile, g.div_band), within = (uint32_t)tile - band * per_band;
            const int left = g.tiles_m - (int)band * SK_GROUP_ROWS;
            const uint32_t rows = (uint32_t)(left < SK_GROUP_ROWS ? left : SK_GROUP_ROWS);
            tn = (int)(left < SK_GROUP_ROWS ? fast_div(within, g.div_last_rows) : within / (uint32_t)SK_GROUP_ROWS);
            tm = (int)band * SK_GROUP_ROWS + (int)(within - (uint32_t)tn * rows);
        }
        m0 = tm * C::BM;
        n0 = tn * C::BN;
        return true;
    };

    // Fix-up and epilogue of one finished segment.  Returns true if every wave has issued exactly the
    // stores of an unsplit interior tile (C::EPILOGUE_STORES for 16-bit outputs, more for fp32) and no
    // other vector-memory instruction.
    auto finish_segment = [&](int tile, int k_begin, int k_end, int m0, int n0, Acc (&acc)[C::MI][C::NI]) -> bool {
        if (ATOMIC) {
            int row0 = m0 + wm * C::WTM + 4 * (lane / C::MF), col0 = n0 + wn * C::WTN + lane % C::MF;
            asm volatile("" : "+v"(row0), "+v"(col0));
            const bool partial = k_begin > 0 || k_end < g.ipt;
            if (m0 + C::BM > g.M || n0 + C::BN > g.N) add_to_image<C, true>(g, row0, col0, partial, acc);
            else add_to_image<C, false>(g, row0, col0, partial, acc);
            return false;
        }

        // ---- fix-up
        // Tiles shared by many workgroups are reduced in two levels: every SK_TREE_GROUP-th contributor first
        // adds the partials of the contributors behind it to its own accumulators, so the owner
        // collects one partial per group.  The order of the additions stays fixed.
        // The owner of a split tile is the workgroup holding its first iteration, the contributors
        // are the workgroups after it (dir = +1); in the k-aligned order the one holding its last
        // iteration, which finishes last, and the contributors are the workgroups before it (dir = -1).
        const bool split = k_begin > 0 || k_end < g.ipt;
        const bool contributor = g.k_aligned ? k_end < g.ipt : k_begin > 0;
        const int dir = g.k_aligned ? -1 : 1;
        int j = 0, n_all = 0;                                           // distance from the tile's owner, the tile's number of contributors
        if (split) {                                                    // (only split tiles; ipw is 0 in a plan without Stream-K work)
            const int first_wg = (int)fast_div((uint32_t)(tile * g.ipt), g.div_ipw);
            const int last_wg = (int)fast_div((uint32_t)(tile * g.ipt + g.ipt - 1), g.div_ipw);
            n_all = last_wg - first_wg;
            j = g.k_aligned ? last_wg - x : x - first_wg;
        }
        const bool two_level = n_all >= 2 * SK_TREE_GROUP;
        const ptrdiff_t slot_stride = (ptrdiff_t)dir * (C::BM * C::BN);
        if (contributor) {
            if (two_level && (j - 1) % SK_TREE_GROUP == 0) {            // group leader: members j+1 .. j+GROUP-1
                const int members = (j + SK_TREE_GROUP - 1 <= n_all ? j + SK_TREE_GROUP - 1 : n_all) - j;
                if (wave == 0) wait_flags(g, x + dir, members, dir);
                __syncthreads();
                const float* mp = g.partials + (ptrdiff_t)(x + dir) * (C::BM * C::BN) + tid;
                asm volatile("" : "+v"(mp));
                add_partials<C>(acc, mp, members, slot_stride);
            }
            // park the accumulators (register order, coalesced), then signal.
            // Partial tiles are stored and loaded with device-scope atomic accesses (one dword
            // per lane, lanes contiguous): these are coherent across the XCDs' L2 caches by
            // themselves, so no L2 write-back / invalidate is needed around the exchange.
            // (the empty asm statements keep the per-block addresses from being computed once, ahead
            // of the persistent loop, where they would occupy registers for the whole kernel)
            float* slot = g.partials + (size_t)x * (C::BM * C::BN) + tid;
            asm volatile("" : "+v"(slot));
#pragma unroll
            for (int mi = 0; mi < C::MI; mi++)
#pragma unroll
                for (int ni = 0; ni < C::NI; ni++) {
#pragma unroll
                    for (int r = 0; r < C::ACC; r++)
                        __hip_atomic_store(slot + ((mi * C::NI + ni) * C::ACC + r) * C::THREADS, acc[mi][ni][r],
                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __builtin_amdgcn_sched_barrier(0);
                }
            wait_vmcnt<0>();                      // every lane's part of the partial tile has reached memory
            __syncthreads();
            if (tid == 0)
                __hip_atomic_store(g.flags + (size_t)x * (SK_FLAG_STRIDE / 4), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return false;
        }
        int n_contrib = 0;
        ptrdiff_t part_stride = slot_stride;
        if (split) {
            // owner: the contributors are the n_all workgroups next to it in direction dir - or, with
            // two levels, their group leaders.  Wait for all of them; the epilogue adds their
            // partials in a fixed order, so the result does not depend on timing.
            const int step = two_level ? SK_TREE_GROUP : 1;
            n_contrib = two_level ? (n_all + SK_TREE_GROUP - 1) / SK_TREE_GROUP : n_all;
            part_stride *= step;
            if (wave == 0) wait_flags(g, x + dir, n_contrib, step * dir);
            __syncthreads();
        }

        // ---- epilogue: fp32 accumulators -> D
        int row0 = m0 + wm * C::WTM + (TR ? lane % C::MF : 4 * (lane / C::MF));
        int col0 = n0 + wn * C::WTN + (TR ? 4 * (lane / C::MF) : lane % C::MF);
        asm volatile("" : "+v"(row0), "+v"(col0));
        const float* part0 = g.partials + (ptrdiff_t)(x + dir) * (C::BM * C::BN) + tid;
        asm volatile("" : "+v"(part0));
        const bool edge = m0 + C::BM > g.M || n0 + C::BN > g.N;
        if (g.out_dtype == SK_BF16) {
            if (edge) reduce_and_store<C, SK_BF16, true, TR>(g, row0, col0, part0, n_contrib, part_stride, acc);
            else reduce_and_store<C, SK_BF16, false, TR>(g, row0, col0, part0, n_contrib, part_stride, acc);
        } else if (g.out_dtype == SK_F16) {
            if (edge) reduce_and_store<C, SK_F16, true, TR>(g, row0, col0, part0, n_contrib, part_stride, acc);
            else reduce_and_store<C, SK_F16, false, TR>(g, row0, col0, part0, n_contrib, part_stride, acc);
        } else {
            if (edge) reduce_and_store<C, SK_F32, true, TR>(g, row0, col0, part0, n_contrib, part_stride, acc);
            else reduce_and_store<C, SK_F32, false, TR>(g, row0, col0, part0, n_contrib, part_stride, acc);
        }
        return TR && !split && !edge;
    };

    // On the LDS-DMA path the first requests of the next segment go out before the current tile's
    // fix-up and epilogue (the ring is free once the MAC loop has ended): the loads travel while the
    // tile is stored, and the first wait of the next MAC loop leaves the epilogue's stores in flight.
    constexpr bool PREFETCH = C::DIRECT && ALIGNED;
    int tile, k_begin, k_end, m0, n0;
    bool have = next_segment(tile, k_begin, k_end, m0, n0);
    bool prefetched = false, stores_in_flight = false;
    while (have) {
        Acc acc[C::MI][C::NI];
#pragma unroll
        for (int mi = 0; mi < C::MI; mi++)
#pragma unroll
            for (int ni = 0; ni < C::NI; ni++) acc[mi][ni] = Acc{};
        // B requested non-temporally or not: decided once per launch, two copies of the loop in the low tiles
        if (C::MAY_STREAM_B && g.stream_b) mac_loop<C, ALIGNED, TR, C::MAY_STREAM_B>(g, m0, n0, k_begin, k_end, smem, fm, acc, prefetched, stores_in_flight);
        else mac_loop<C, ALIGNED, TR, false>(g, m0, n0, k_begin, k_end, smem, fm, acc, prefetched, stores_in_flight);

        // this segment's numbers for the fix-up and the epilogue; then look ahead
        const int cur_tile = tile, cur_k_begin = k_begin, cur_k_end = k_end, cur_m0 = m0, cur_n0 = n0;
        have = next_segment(tile, k_begin, k_end, m0, n0);
        prefetched = PREFETCH && have;
        stores_in_flight = false;
        if (prefetched) {
            DmaMap<C> ahead;
            ahead.init(g, m0, n0);
            if (C::MAY_STREAM_B && g.stream_b) mac_prefetch<C, C::MAY_STREAM_B>(g, m0, n0, k_begin, k_end, smem, ahead);
            else mac_prefetch<C, false>(g, m0, n0, k_begin, k_end, smem, ahead);
        }
        stores_in_flight = finish_segment(cur_tile, cur_k_begin, cur_k_end, cur_m0, cur_n0, acc) && prefetched;
    }
}

// ---- kernel table entries --------------------------------------------------------------------
typedef void (*kernel_fn)(GemmArgs);
struct KernelEntry {
    int dtype, bm, bn, bk, variant, fixup;
    int whole_tiles_choice = 0;          // > 0: the library launches this variant instead of variant 0 for plans without split
                                         // tiles whose tiles have at least this many k-iterations
    kernel_fn aligned, generic;
    int threads, lds_bytes, piece_elems;
    std::atomic<int> max_resident{-1};   // co-resident workgroups on the device, -1 = not yet asked
    KernelEntry(int d, int m, int n, int k, int v, int fx, kernel_fn a, kernel_fn g, int t, int l, int pe)
        : dtype(d), bm(m), bn(n), bk(k), variant(v), fixup(fx), aligned(a), generic(g), threads(t), lds_bytes(l), piece_elems(pe) {}
};

template <class C, bool ATOMIC = false> KernelEntry* make_entry(int variant = 0, int whole_tiles_choice = 0) {
    KernelEntry* e = new KernelEntry(C::DT, C::BM, C::BN, C::BK, variant, ATOMIC ? SK_FIXUP_ATOMIC : SK_FIXUP_FLAGS,
                                     streamk_gemm_kernel<C, true, ATOMIC>, streamk_gemm_kernel<C, false, ATOMIC>,
                                     C::THREADS, C::LDS_BYTES, C::PE);
    e->whole_tiles_choice = whole_tiles_choice;
    return e;
}

// Tile shapes with a kernel: <dtype, BM, BN, BK, waves along M, waves along N, matrix-core block,
// A ring depth[, B ring depth[, instruction-by-instruction MAC loop]]>.  Variant 0 of a shape is the
// one sk_gemm uses; other variants are alternative wave layouts of the same shape, selectable with
// sk_plan_set_kernel_variant for tuning runs.  ATOMIC selects the atomic-add fix-up (sk_fixup).
// The three compute-bound shapes have two kernels that the library itself chooses between: four
// waves (one per SIMD, twice the tile per wave: a quarter less LDS read traffic, +1.5 - 3 % on problems
// of whole tiles) for plans without split tiles, eight waves for plans with split tiles (twice as
// many lanes fetch and add the partial tiles: 10 - 25 % faster there with 256 x 256 tiles).  Variant 3
// is the eight-wave kernel under a number of its own (variant 0 means "the library's choice").
template <int DT, bool ATOMIC = false> void add_16bit_tiles(KernelEntry** t, int* n) {
    // The 128- and 64-row tiles run 8 waves (2 x 4), two per SIMD, like the large ones: with one wave
    // per SIMD (2 x 2) nothing overlaps a wave's waits (128 x 128 x 64: +8 - 12 % on 512 x 8192 x 8192
    // and 4096^3; 64 x 128 x 64: +4 % on the HBM-bound M = 64 shape, +12 - 20 % on small problems).
    // The three compute-bound shapes run the instruction-by-instruction MAC loop (+5 % on 8192^3 with
    // 256 x 256, +8 % on 4096^3 with 128 x 128, +2 - 3 % with 256 x 128; the 64-row tile loses 7 % with it).
    t[(*n)++] = make_entry<Cfg<DT, 128, 128, 32, 2, 4, 32, 4>, ATOMIC>();
    t[(*n)++] = make_entry<Cfg<DT, 128, 128, 64, 2, 4, 32, 3, 3, 1>, ATOMIC>();
    t[(*n)++] = make_entry<Cfg<DT, 256, 128, 64, 4, 2, 32, 3, 3, 1>, ATOMIC>();
    t[(*n)++] = make_entry<Cfg<DT, 256, 256, 64, 2, 4, 32, 3, 2, 1>, ATOMIC>();
    t[(*n)++] = make_entry<Cfg<DT, 64, 128, 64, 2, 4, 32, 4>, ATOMIC>();
    t[(*n)++] = make_entry<Cfg<DT, 32, 128, 64, 1, 4, 32, 4>, ATOMIC>();
    t[(*n)++] = make_entry<Cfg<DT, 16, 128, 64, 1, 4, 16, 4>, ATOMIC>();
    if constexpr (!ATOMIC) {  // (the atomic fix-up exists for the layouts above only)
        t[(*n)++] = make_entry<Cfg<DT, 256, 128, 64, 2, 2, 32, 3, 3, 1>>(1, 16);
        t[(*n)++] = make_entry<Cfg<DT, 256, 128, 64, 4, 2, 32, 3, 3, 1>>(3);
        t[(*n)++] = make_entry<Cfg<DT, 256, 256, 64, 2, 2, 32, 3, 2, 1>>(1, 48);
        t[(*n)++] = make_entry<Cfg<DT, 256, 256, 64, 2, 4, 32, 3, 2>>(2);
        t[(*n)++] = make_entry<Cfg<DT, 256, 256, 64, 2, 4, 32, 3, 2, 1>>(3);      // variant 0's kernel under a number of its own
        t[(*n)++] = make_entry<Cfg<DT, 256, 256, 32, 2, 2, 32, 4>>();
        t[(*n)++] = make_entry<Cfg<DT, 128, 128, 64, 2, 2, 32, 3, 3, 1>>(1, 1);
        t[(*n)++] = make_entry<Cfg<DT, 128, 128, 64, 2, 4, 32, 3, 3, 1>>(3);
        t[(*n)++] = make_entry<Cfg<DT, 64, 128, 64, 2, 2, 32, 4>>(1);
    }
}

// One function per input type, each in its own translation unit (so that they compile in parallel);
// it appends that type's kernels to the table.
void register_bf16(KernelEntry** t, int* n);
void register_f16(KernelEntry** t, int* n);
void register_fp8(KernelEntry** t, int* n);
void register_bf16_atomic(KernelEntry** t, int* n);
void register_f16_atomic(KernelEntry** t, int* n);
void register_fp8_atomic(KernelEntry** t, int* n);

}  // namespace streamk_detail

// Building blocks of the bf16 MFMA attention kernels (gfx950, wave64, head size 128).
//
// Matrix-core instruction used everywhere: v_mfma_f32_32x32x16_bf16, D[32x32] += A[32x16] B[16x32].
// Per lane (l = lane id, n = l & 31, h = l >> 5):
//   A operand: row n of A, eight consecutive k (k-slots 8h .. 8h+7)
//   B operand: column n of B, the same eight k-slots
//   C/D      : column n; register r holds row 8 (r / 4) + 4 h + (r % 4)
// Because the contraction only pairs k-slot (h, e) of A with k-slot (h, e) of B, any bijection
// between k-slots and the contracted index is valid as long as both operands use the same one.
// The kernels exploit that: a C/D tile is re-used directly as the next product's operand, with
// its eight registers 8 half .. 8 half + 7 standing for the contracted indices
//   16 half + 4 h + {0,1,2,3}  and  16 half + 8 + 4 h + {0,1,2,3},
// and the other operand is read from LDS in that same order (two 8-byte reads of a transposed tile).
#pragma once
#include <type_traits>
#include <utility>

#include "common.hpp"

namespace l2a {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

// compile-time loop: f(std::integral_constant<int, I>{}) for I = BEGIN .. END-1
template <int BEGIN, int END, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (BEGIN < END) {
        f(std::integral_constant<int, BEGIN>{});
        static_for<BEGIN + 1, END>(f);
    }
}

constexpr int kD = 128;         // head size
constexpr int kThreads = 256;   // 4 wavefronts
constexpr int kRowPad = kD + 8; // row-major tile: 272-byte rows, conflict-free 16-byte reads

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Tile orders of the forward and dQ kernels: tokens x (b, KV head) up to which the tiles of all heads
// run together.  Their K and V (512 bytes per token and head) then have to share the 256 MB
// last-level cache: at 2^19 (268 MB) running them together still measured 1 % faster than one head
// after the other, at 2^20 it was 12-18 % slower.
constexpr long long kAllHeadsMaxTokens = 1 << 19;

// index along the M dimension held by register r of a C/D tile
__device__ __forceinline__ int c_row(int r, int h) { return 8 * (r >> 2) + 4 * h + (r & 3); }

// eight fp32 -> one bf16 MFMA operand (registers 8*half .. 8*half+7 of a C/D tile)
__device__ __forceinline__ bf16x8 pack8(const f32x16& x, int half) {
    bf16x8 o;
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
        f32x2 f = {x[8 * half + e], x[8 * half + e + 1]};
        bf16x2 b = __builtin_convertvector(f, bf16x2);
        o[e] = b[0];
        o[e + 1] = b[1];
    }
    return o;
}

// ---------------------------------------------------------------------------------------
// LDS tiles.  A "rows x 128" bf16 tile is kept row-major (stride kRowPad) for operands whose
// contracted index is the channel, and/or transposed ([128][rows + 4]) for operands whose
// contracted index is the row (token).  ROWS is 64 for every tile here.
// ---------------------------------------------------------------------------------------
constexpr int kTileRows = 64;
constexpr int kColPad = kTileRows + 4;                 // transposed tile: 136-byte rows
constexpr int kRowMajorBytes = kTileRows * kRowPad * 2;  // 17408
constexpr int kTransposedBytes = kD * kColPad * 2;       // 17408

// Global -> register staging of one 64 x 128 tile: thread t owns channels 8 (t & 15) .. +7 of
// rows 4 (t >> 4) + i, i = 0..3 (sixteen lanes read one whole 256-byte row).
struct TileRegs {
    u32x4 x[4];
};

// row_ptr(i) must return the global address of row 4 (t >> 4) + i of the tile
template <typename RowPtr>
__device__ __forceinline__ void tile_load(TileRegs& r, RowPtr row_ptr) {
    const int c8 = (threadIdx.x & 15) * 8;
#pragma unroll
    for (int i = 0; i < 4; ++i) r.x[i] = *reinterpret_cast<const u32x4*>(row_ptr(i) + c8);
}

__device__ __forceinline__ void tile_store_rowmajor(const TileRegs& r, __bf16* lds) {
    const int c8 = (threadIdx.x & 15) * 8, r4 = (threadIdx.x >> 4) * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(lds + (r4 + i) * kRowPad + c8) = r.x[i];
}

// 4 rows x 8 channels in registers -> 8 channels x 4 rows in LDS
__device__ __forceinline__ void tile_store_transposed(const TileRegs& r, __bf16* lds) {
    const int c8 = (threadIdx.x & 15) * 8, r4 = (threadIdx.x >> 4) * 4;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const uint32_t a = r.x[0][p], b = r.x[1][p], c = r.x[2][p], d = r.x[3][p];
        u32x2 even = {(a & 0xffffu) | (b << 16), (c & 0xffffu) | (d << 16)};
        u32x2 odd = {(a >> 16) | (b & 0xffff0000u), (c >> 16) | (d & 0xffff0000u)};
        *reinterpret_cast<u32x2*>(lds + (c8 + 2 * p) * kColPad + r4) = even;
        *reinterpret_cast<u32x2*>(lds + (c8 + 2 * p + 1) * kColPad + r4) = odd;
    }
}

// MFMA operand from a row-major tile: row `row`, channels 16 ks + 8 h .. +7
__device__ __forceinline__ bf16x8 lds_rowmajor(const __bf16* lds, int row, int ks, int h) {
    return *reinterpret_cast<const bf16x8*>(lds + row * kRowPad + ks * 16 + 8 * h);
}

// MFMA operand from a transposed tile: channel `ch`, tokens 16 step + 4 h + {0..3} and + 8
__device__ __forceinline__ bf16x8 lds_transposed(const __bf16* lds, int ch, int step, int h) {
    const __bf16* p = lds + ch * kColPad + step * 16 + 4 * h;
    const bf16x4 lo = *reinterpret_cast<const bf16x4*>(p);
    const bf16x4 hi = *reinterpret_cast<const bf16x4*>(p + 8);
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// ---------------------------------------------------------------------------------------
// rows of a branch.  The lists live in device memory, where the host cannot check them: counts and
// row codes are clamped into their valid ranges, so that a damaged list gives wrong numbers but
// never an address outside the tensors.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ int rows_total(const RowSet& rs, const Geom& gm, int bh) {
    return rs.count ? min(max(rs.count[bh], 0), gm.T * gm.G) : gm.T * gm.G;
}
__device__ __forceinline__ int row_code(const RowSet& rs, const Geom& gm, int bh, int r) {
    return rs.row_idx ? min(max(rs.row_idx[(size_t)bh * gm.T * gm.G + r], 0), gm.T * gm.G - 1) : r;
}

// Value of an accumulator element that lives in an AGPR (the VALU cannot read AGPRs).  Written
// out so that the copy is issued where the value is consumed, between matrix instructions,
// instead of in a burst of copies where the compiler splits the accumulator's live range.
__device__ __forceinline__ float acc_read(float x) {
    float y;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(y) : "a"(x));
    return y;
}

// Matrix instructions whose result tile is consumed by the VALU (scores, dP): written as inline
// assembly with the C/D tile in VGPRs.  The compiler puts every builtin MFMA's C/D tile in AGPRs
// when a kernel uses more than 256 registers, and then needs one v_accvgpr_read per element the
// VALU touches -- in these kernels the VALU is the busier unit.
// Rules the callers keep, since the compiler does not see an MFMA here and inserts no hazard
// no-ops for it: (1) A and B come from LDS loads or from registers written long before (never
// straight from a VALU result); (2) a tile is read by the VALU only after at least eight further
// matrix instructions have been issued behind the last write to it; (3) a chain accumulates into
// exactly the same registers (the hardware interlocks that case).
// After the last write of a chain that the VALU reads right away (a kernel prologue): wait out
// the matrix pipeline.
__device__ __forceinline__ void mfma_vgpr_settle() {
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}
__device__ __forceinline__ void mfma32_vgpr_first(f32x16& d, bf16x8 a, bf16x8 b) {
    asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma32_vgpr_from(f32x16& d, bf16x8 a, bf16x8 b, const f32x16& c) {
    asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(d) : "v"(a), "v"(b), "v"(c));
}
__device__ __forceinline__ void mfma32_vgpr_acc(f32x16& d, bf16x8 a, bf16x8 b) {
    asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(a), "v"(b));
}

}  // namespace l2a

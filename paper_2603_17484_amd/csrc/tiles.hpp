// LDS tiles of the matrix-core kernels and their direct global->LDS loads (gfx950).
//
// Every matrix-core operand is read from LDS with one 16-byte ds_read_b128 per lane.  To make
// that possible for operands whose contracted index is the token (V in P V, K in dS K, Q and dO
// in dS^T Q and P^T dO), a pre-pass writes *token-minor* copies of those tensors, [.., D, tokens],
// in which every group of 16 tokens is stored in the order
//      0 1 2 3  8 9 10 11 | 4 5 6 7  12 13 14 15
// i.e. position p holds token (p & 3) + 8 ((p >> 2) & 1) + 4 (p >> 3).  The first eight
// positions are exactly the contracted indices a lane of the lower half-wave needs for one
// MFMA (see mfma.hpp), the last eight those of the upper half-wave.
//
// Tiles are filled by global_load_lds_dwordx4: each lane names its own global address and the
// hardware writes the 64 lanes' 16-byte pieces to 1024 consecutive LDS bytes starting at M0.
// No staging registers, no LDS store instructions.  Since the LDS side is fixed, bank conflicts
// are avoided by permuting on the global side: 16-byte chunk c of a row lands in chunk slot
// c ^ f(row), and readers apply the same XOR.
#pragma once
#include "mfma.hpp"

namespace l2a {

__device__ __forceinline__ unsigned lds_offset(const void* p) {
    return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

__device__ __forceinline__ void dma_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// ---------------------------------------------------------------------------------------
// Row-major tile: ROWS tokens x 128 channels, 256-byte rows, chunk c of row r in slot c ^ (r & 15).
// ---------------------------------------------------------------------------------------
constexpr int kRmRowBytes = 256;

// MFMA operand: row `row`, channels 16 ks + 8 h .. + 7
__device__ __forceinline__ bf16x8 rm_operand(const __bf16* tile, int row, int ks, int h) {
    const int slot = (2 * ks + h) ^ (row & 15);
    return *reinterpret_cast<const bf16x8*>(tile + row * 128 + slot * 8);
}

// ---------------------------------------------------------------------------------------
// Token-minor tile: 128 channels x TOK tokens (TOK = 64 or 32), rows of 2 TOK bytes.
// ---------------------------------------------------------------------------------------
template <int TOK>
__device__ __forceinline__ int tm_swizzle(int ch) {
    if (TOK == 64) return (ch & 7) ^ ((ch >> 3) & 1);  // 8 chunks per 128-byte row
    return (ch >> 2) & 3;                              // 4 chunks per 64-byte row (measured conflict-free)
}

// MFMA operand: channel `ch`, the eight tokens of 16-token group `step` that half-wave h contracts
template <int TOK>
__device__ __forceinline__ bf16x8 tm_operand(const __bf16* tile, int ch, int step, int h) {
    const int slot = (2 * step + h) ^ tm_swizzle<TOK>(ch);
    return *reinterpret_cast<const bf16x8*>(tile + ch * TOK + slot * 8);
}

// ---------------------------------------------------------------------------------------
// Tile loads.  A tile whose rows are a fixed byte stride apart is loaded from a wave-uniform
// 64-bit base (scalar registers) plus a per-lane 32-bit offset that never changes, so issuing a
// load costs no vector instruction: lane l's 16 (or 4) bytes at sbase + voff go to LDS bytes
// [lds_base + 16 l, +16) (or 4 l).  lds_base and `wave` (readfirstlane of threadIdx.x >> 6) must
// be wave-uniform; offsets must stay below 4 GiB (checked by the host wrappers).  Completion is
// tracked by vmcnt (dma_wait).
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void dma16_so(const void* sbase, unsigned voff, unsigned lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(voff), "s"(sbase)
                 : "memory");
}
__device__ __forceinline__ void dma4_so(const void* sbase, unsigned voff, unsigned lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, %2" ::"s"(lds_base), "v"(voff), "s"(sbase)
                 : "memory");
}

// NW = wavefronts of the workgroup; every wavefront loads 1/NW of the tile.
template <int ROWS, int NW = 4>
struct RmDma {
    unsigned voff[ROWS / (4 * NW)];
};
template <int ROWS, int NW = 4>
__device__ __forceinline__ RmDma<ROWS, NW> rm_dma_setup(unsigned row_stride_bytes, int wave) {
    RmDma<ROWS, NW> d;
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < ROWS / (4 * NW); ++i) {
        const int row = (i * NW + wave) * 4 + (lane >> 4);
        d.voff[i] = (unsigned)row * row_stride_bytes + (unsigned)(((lane & 15) ^ (row & 15)) * 16);
    }
    return d;
}
// The same tile with the chunk permutation that suits *transposed* reads (ds_read_b64_tr_b16 of
// 4 rows x 16 channels per 16 lanes): slot = c ^ (4 (r & 3) + ((r >> 2) & 3)), so that the four
// rows one read touches fall into four different groups of banks.  Row reads stay conflict-free.
__device__ __forceinline__ int rm_tr_swizzle(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }
template <int ROWS, int NW = 4>
__device__ __forceinline__ RmDma<ROWS, NW> rm_tr_dma_setup(unsigned row_stride_bytes, int wave) {
    RmDma<ROWS, NW> d;
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < ROWS / (4 * NW); ++i) {
        const int row = (i * NW + wave) * 4 + (lane >> 4);
        d.voff[i] = (unsigned)row * row_stride_bytes + (unsigned)(((lane & 15) ^ rm_tr_swizzle(row)) * 16);
    }
    return d;
}
// Operands from a tile in that layout.  Row-major: row `row`, channels 16 ks + 8 h .. + 7.
__device__ __forceinline__ bf16x8 rm_tr_row_operand(const __bf16* tile, int row, int ks, int h) {
    const int slot = (2 * ks + h) ^ rm_tr_swizzle(row);
    return *reinterpret_cast<const bf16x8*>(tile + row * 128 + slot * 8);
}
// Transposed (contraction over the rows): channel d*32 + (lane & 31), the rows of 16-row group `step`
// in the order 4h..4h+3, 8+4h..8+4h+3 -- the order in which a C tile's registers hold them.
typedef short s16x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ bf16x8 rm_tr_col_operand(const __bf16* tile, int d, int step, int lane) {
    const int i = lane & 15, n16 = (lane >> 4) & 1, h = lane >> 5;
    const int ch = d * 32 + 16 * n16 + 4 * (i & 3);
    const int row = 16 * step + 4 * h + (i >> 2);
    auto addr = [&](int r) { return tile + r * 128 + (((ch >> 3) ^ rm_tr_swizzle(r)) * 8) + (ch & 7); };
    const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (s16x4 __attribute__((address_space(3)))*)(__attribute__((address_space(3))) const void*)addr(row));
    const s16x4 v2 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (s16x4 __attribute__((address_space(3)))*)(__attribute__((address_space(3))) const void*)addr(row + 8));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(v1, v2, 0, 1, 2, 3, 4, 5, 6, 7));
}
// The same read with the per-lane part of the address computed once: byte offset of this lane's piece for
// channel block d and half j (rows 4h.., 8+4h..) of 16-row group 0; group `step` lies 4096 bytes further.
__device__ __forceinline__ unsigned rm_tr_col_offset(int d, int j, int lane) {
    const int i = lane & 15, n16 = (lane >> 4) & 1, h = lane >> 5;
    const int ch = d * 32 + 16 * n16 + 4 * (i & 3);
    const int r = 4 * h + (i >> 2) + 8 * j;
    return (unsigned)(r * 256 + (((ch >> 3) ^ rm_tr_swizzle(r)) * 16) + (ch & 7) * 2);
}
// p0, p1: LDS addresses of this lane's two pieces in 16-row group 0 of the first of several tiles that lie
// `tile_bytes` apart (tile address + rm_tr_col_offset(d, 0 / 1, lane)); the constant parts of the address
// end up in the instruction's offset field.
typedef __attribute__((address_space(3))) const char* lds_cptr;
__device__ __forceinline__ bf16x8 rm_tr_col_operand_at(lds_cptr p0, lds_cptr p1, int step, int tile_bytes_off) {
    typedef s16x4 __attribute__((address_space(3)))* lds_ptr;
    const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p0 + step * 4096 + tile_bytes_off));
    const s16x4 v2 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p1 + step * 4096 + tile_bytes_off));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(v1, v2, 0, 1, 2, 3, 4, 5, 6, 7));
}
// sbase: global address of (row 0, channel 0) of the tile, wave-uniform
template <int ROWS, int NW>
__device__ __forceinline__ void rm_dma_issue(const RmDma<ROWS, NW>& d, const void* sbase, unsigned lds_base,
                                             int wave) {
#pragma unroll
    for (int i = 0; i < ROWS / (4 * NW); ++i) dma16_so(sbase, d.voff[i], lds_base + (i * NW + wave) * 1024);
}

// The same tile when only the first `rows_valid` rows exist in memory: later rows repeat the last
// valid one (their contents never matter to the caller).  Per-lane arithmetic; for ragged ends only.
// TR: the chunk permutation for transposed reads (rm_tr_swizzle) instead of the plain one.
template <int ROWS, int NW = 4, bool TR = false>
__device__ __forceinline__ void rm_dma_issue_clamped(unsigned row_stride_bytes, int rows_valid, const void* sbase,
                                                     unsigned lds_base, int wave) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < ROWS / (4 * NW); ++i) {
        const int row = (i * NW + wave) * 4 + (lane >> 4);
        const int sw = TR ? (((row & 3) << 2) | ((row >> 2) & 3)) : (row & 15);
        const unsigned voff = (unsigned)min(row, rows_valid - 1) * row_stride_bytes + (unsigned)(((lane & 15) ^ sw) * 16);
        dma16_so(sbase, voff, lds_base + (i * NW + wave) * 1024);
    }
}

template <int TOK, int NW = 4>
struct TmDma {
    unsigned voff[TOK / (4 * NW)];  // 128 channels * 2 TOK bytes / (1024 NW) bytes per workgroup instruction
};
template <int TOK, int NW = 4>
__device__ __forceinline__ TmDma<TOK, NW> tm_dma_setup(unsigned ch_stride_bytes, int wave) {
    constexpr int kChunks = TOK / 8, kRowsPerSeg = 64 / kChunks;
    TmDma<TOK, NW> d;
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < TOK / (4 * NW); ++i) {
        const int ch = (i * NW + wave) * kRowsPerSeg + lane / kChunks;
        d.voff[i] = (unsigned)ch * ch_stride_bytes + (unsigned)(((lane % kChunks) ^ tm_swizzle<TOK>(ch)) * 16);
    }
    return d;
}
// sbase: global address of (channel 0, first token of the tile), wave-uniform
template <int TOK, int NW>
__device__ __forceinline__ void tm_dma_issue(const TmDma<TOK, NW>& d, const void* sbase, unsigned lds_base,
                                             int wave) {
#pragma unroll
    for (int i = 0; i < TOK / (4 * NW); ++i) dma16_so(sbase, d.voff[i], lds_base + (i * NW + wave) * 1024);
}

// position of token t inside its 16-token group in a token-minor copy, and the inverse
__device__ __host__ __forceinline__ int tm_pos_of_token(int t) {
    return (t & ~15) | ((t & 3) + 4 * ((t >> 3) & 1) + 8 * ((t >> 2) & 1));
}
__device__ __host__ __forceinline__ int tm_token_at_pos(int p) {
    return (p & ~15) | ((p & 3) + 8 * ((p >> 2) & 1) + 4 * ((p >> 3) & 1));
}

}  // namespace l2a

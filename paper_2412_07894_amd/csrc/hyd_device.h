// Device-side building blocks shared by the gfx950 attention kernels: vector types, the MFMA
// wrapper with its operand/accumulator lane maps, the LDS tile layout, and global<->LDS movers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hyd {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;

constexpr int kWave = 64;
constexpr int kHeadDim = 128;                 // bf16 path
constexpr int kRowBytes = kHeadDim * 2;       // one (token, head) row of bf16
constexpr int kChunksPerRow = kRowBytes / 16; // 16-byte chunks per row

// v_mfma_f32_32x32x16_bf16: D[32][32] += A[32][16] * B[16][32].  With lane l, half = l / 32:
//   a[e] = A[l % 32][8 * half + e],  b[e] = B[8 * half + e][l % 32],  e = 0..7
//   acc[r] = D[8 * (r / 4) + 4 * half + r % 4][l % 32],             r = 0..15
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) {
    bf16x8 r;
    __builtin_memcpy(&r, &v, 16);
    return r;
}

// Two floats -> packed bf16 pair (round to nearest even), low half = x.
__device__ __forceinline__ uint32_t pack_bf16(float x, float y) {
    f32x2 v = {x, y};
    bf16x2 b = __builtin_convertvector(v, bf16x2);
    uint32_t r;
    __builtin_memcpy(&r, &b, 4);
    return r;
}

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// LDS tile of bf16 rows of 256 bytes, no padding.  The 16-byte chunk c of row r lives at chunk
// position c ^ swz(r).  swz is chosen so that both access patterns of the kernels are free of
// bank conflicts: (1) 16 lanes reading the same chunk of 16 consecutive rows (MFMA operands whose
// contraction index is the head dimension) see 16 distinct chunk positions; (2) 32 lanes of a
// transposing read touching 4 consecutive rows x 64 contiguous bytes see 4 distinct 64-byte groups.
__device__ __forceinline__ int swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }
__device__ __forceinline__ int tile_off(int row, int chunk) {     // byte offset in the tile
    return row * kRowBytes + ((chunk ^ swz(row)) << 4);
}

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// Operand fragment whose contraction index is the head dimension: 8 consecutive elements
// [16*ks + 8*half, +8) of row `row` of a tile.
__device__ __forceinline__ bf16x8 lds_row_frag(const char* tile, int row, int ks, int half) {
    return as_bf16x8(*reinterpret_cast<const u32x4*>(tile + tile_off(row, 2 * ks + half)));
}

// Transposing read (ds_read_b64_tr_b16).  Within each group of 16 lanes, lane i supplies the
// address of a 4-element row fragment; lane L then receives element L % 4 of the fragments
// supplied by lanes L / 4, 4 + L / 4, 8 + L / 4, 12 + L / 4.  With lane i pointing at
// tile[row0 + i / 4][col0 + 4 * (i % 4) ..+4], lane L ends up with tile[row0 + 0..3][col0 + L]:
// four consecutive ROWS of one column, i.e. a fragment whose contraction index is the row.
__device__ __forceinline__ u32x2 lds_tr4(const char* tile, int row0, int col0, int lane16) {
    const int row = row0 + (lane16 >> 2);
    const int col = col0 + ((lane16 & 3) << 2);               // element column, multiple of 4
    const char* p = tile + tile_off(row, col >> 3) + ((col & 4) << 1);
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
    u32x2 r;
    __builtin_memcpy(&r, &v, 8);
    return r;
}

// Operand fragment whose contraction index is the tile ROW, matched to the accumulator lane map:
// for contraction step b (16 rows) and column block cb (32 columns) the lane holding column
// 32*cb + l%32 receives rows 16b + 4*half + {0..3} and 16b + 8 + 4*half + {0..3}; these are the
// rows a lane's accumulator registers 8*(b%2) .. +8 of row block b/2 hold (see mfma32).
__device__ __forceinline__ bf16x8 lds_col_frag(const char* tile, int b, int cb, int lane) {
    const int half = lane >> 5, lane16 = lane & 15;
    const int col0 = 32 * cb + (lane & 16);
    u32x2 lo = lds_tr4(tile, 16 * b + 4 * half, col0, lane16);
    u32x2 hi = lds_tr4(tile, 16 * b + 8 + 4 * half, col0, lane16);
    u32x4 v = {lo[0], lo[1], hi[0], hi[1]};
    return as_bf16x8(v);
}

// Global -> registers -> LDS copy of a [ROWS][128] bf16 tile by NT threads.  Row r of the tile is
// global row (row_base + r) of a [T][H][128] tensor at head `h`; rows at or beyond row_end are
// filled with zeros (never read from memory).
template <int ROWS, int NT>
struct TileMover {
    static constexpr int kChunks = ROWS * kChunksPerRow;
    static constexpr int kPerThread = kChunks / NT;
    static_assert(kChunks % NT == 0, "tile must divide over the threads");
    u32x4 reg[kPerThread];

    __device__ __forceinline__ void load(const uint16_t* base, int64_t row_stride_elems, int h,
                                         int row_base, int row_end, int tid) {
#pragma unroll
        for (int p = 0; p < kPerThread; ++p) {
            const int idx = tid + p * NT;
            const int r = idx / kChunksPerRow, c = idx % kChunksPerRow;
            const int grow = row_base + r;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (grow < row_end)
                v = *reinterpret_cast<const u32x4*>(base + (int64_t)grow * row_stride_elems +
                                                   (int64_t)h * kHeadDim + c * 8);
            reg[p] = v;
        }
    }
    __device__ __forceinline__ void store(char* tile, int tid) const {
#pragma unroll
        for (int p = 0; p < kPerThread; ++p) {
            const int idx = tid + p * NT;
            const int r = idx / kChunksPerRow, c = idx % kChunksPerRow;
            *reinterpret_cast<u32x4*>(tile + tile_off(r, c)) = reg[p];
        }
    }
};

__device__ __forceinline__ float shfl_xor32(float v) {
    // exchange with the lane 32 away (the other half of the wave)
    return __shfl_xor(v, 32, 64);
}

}  // namespace hyd

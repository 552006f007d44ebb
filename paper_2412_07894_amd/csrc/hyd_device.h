// Device-side building blocks shared by the gfx950 attention kernels: vector types, the MFMA
// wrapper with its operand/accumulator lane maps, the LDS tile layout and the fragment reads.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hyd {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) __fp16 f16x4;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

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

// v_mfma_f32_32x32x16_f16: same shape, rate and lane maps, operands in fp16 (11 significant bits).
// The backward's products run on it: every bf16 input converts to fp16 exactly (magnitudes in
// [2^-14, 65504]), and the factors formed in registers (P, dS) keep three more bits than bf16
// would leave them.  Fragments travel as 16-byte register groups typed bf16x8 whatever their
// element format is; this wrapper reads the bits as fp16.
__device__ __forceinline__ f32x16 mfma32h(bf16x8 a, bf16x8 b, f32x16 c) {
    f16x8 x, y;
    __builtin_memcpy(&x, &a, 16);
    __builtin_memcpy(&y, &b, 16);
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(x, y, c, 0, 0, 0);
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

// Two floats -> packed fp16 pair (round to nearest even, v_cvt_pk_f16_f32), low half = x.
__device__ __forceinline__ uint32_t pack_f16(float x, float y) {
    f32x2 v = {x, y};
    f16x2 h = __builtin_convertvector(v, f16x2);
    uint32_t r;
    __builtin_memcpy(&r, &h, 4);
    return r;
}

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// Packed bf16 pair -> packed fp16 pair, each value times `mul` (a power of two).  Exact for
// magnitudes in [2^-14, 65504]; smaller ones keep an absolute accuracy of 2^-25, larger ones
// become infinite (and NaN stays NaN), so that an input outside the fp16 range shows in the result.
__device__ __forceinline__ uint32_t bf16x2_to_f16x2(uint32_t u, float mul = 1.f) {
    return pack_f16(bf16_lo(u) * mul, bf16_hi(u) * mul);
}

// LDS tile of bf16 rows of 256 bytes, no padding.  The 16-byte chunk c of row r lives at chunk
// position c ^ swz(r).  swz is chosen so that both access patterns of the kernels are free of
// bank conflicts: (1) 16 lanes reading the same chunk of 16 consecutive rows (MFMA operands whose
// contraction index is the head dimension) see 16 distinct chunk positions; (2) 32 lanes of a
// transposing read touching 4 consecutive rows x 64 contiguous bytes see 4 distinct 64-byte groups.
__device__ __forceinline__ int swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }
__device__ __forceinline__ int tile_off(int row, int chunk) {     // byte offset in the tile
    return row * kRowBytes + ((chunk ^ swz(row)) << 4);
}


// Transposing read (ds_read_b64_tr_b16).  Within each group of 16 lanes, lane i supplies the
// address of a 4-element row fragment; lane L then receives element L % 4 of the fragments
// supplied by lanes L / 4, 4 + L / 4, 8 + L / 4, 12 + L / 4.  With lane i pointing at
// tile[row0 + i / 4][col0 + 4 * (i % 4) ..+4], lane L ends up with tile[row0 + 0..3][col0 + L]:
// four consecutive ROWS of one column, i.e. a fragment whose contraction index is the row.
//
// A column fragment (contraction index = tile row) is two such reads, matched to the accumulator
// lane map: for contraction step b (16 rows) and column block cb (32 columns) the lane holding
// column 32*cb + l%32 receives rows 16b + 4*half + {0..3} and 16b + 8 + 4*half + {0..3}, which are
// the rows that the lane's accumulator registers 8*(b%2) .. +8 of row block b/2 hold (see mfma32).

// Per-lane LDS byte offsets of the two fragment kinds, computed once per kernel.  A fragment read
// is then one LDS instruction whose address is one of these registers plus a compile-time offset
// (tile base, 32-row block, 16-row contraction step): swz() is invariant under adding multiples
// of 16 rows, so blocks and steps move the address by plain multiples of kRowBytes.
typedef __attribute__((address_space(3))) char lds_char;
typedef __attribute__((address_space(3))) const u32x4 lds_u32x4;

struct FragAddr {
    // ABSOLUTE LDS byte addresses (the base of the dynamic LDS block is folded in here, once,
    // because the compiler cannot fold that link-time constant into instruction offsets)
    uint32_t row[8];      // row fragment of row (lane % 32), contraction step ks = 0..7
    uint32_t col[8];      // [2 * cb + hi]: transposing read of column block cb, row group hi, step 0
    __device__ __forceinline__ void init(int lane, const char* lds_base) {
        const int l32 = lane & 31, half = lane >> 5, lane16 = lane & 15;
        const uint32_t base = (uint32_t)(uintptr_t)(lds_char*)lds_base;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) row[ks] = base + tile_off(l32, 2 * ks + half);
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) {
#pragma unroll
            for (int hi = 0; hi < 2; ++hi) {
                const int r = 4 * half + 8 * hi + (lane16 >> 2);
                const int c = 32 * cb + (lane & 16) + ((lane16 & 3) << 2);
                col[2 * cb + hi] = base + tile_off(r, c >> 3) + ((c & 4) << 1);
            }
        }
    }
};

// Row fragment (contraction index = head dimension): elements [16*ks + 8*half, +8) of tile row
// 32*blk + lane%32.  `tile` is the tile's byte offset from the LDS base given to FragAddr::init.
__device__ __forceinline__ bf16x8 frag_row(int tile, const FragAddr& fa, int blk, int ks) {
    return as_bf16x8(*(lds_u32x4*)(uintptr_t)(fa.row[ks] + (uint32_t)(tile + blk * 32 * kRowBytes)));
}

// ---- LDS fragment reads with explicit completion tracking
//
// The compiler cannot tell a direct-to-LDS load (global -> LDS without registers) apart from the
// tiles the kernel is reading, so before an LDS read it knows to be one it drains the whole load
// queue, the tiles requested for LATER steps included; that turns a ring of stages into a ring
// of one.  The fragment reads of the hot loops are therefore issued as volatile assembly, which
// keeps them in source order, and completion is tracked by hand: LDS reads return in order, so a
// fragment has arrived once at most (reads issued after it) remain outstanding.  LdsQueue counts
// issued read instructions; after full unrolling every count is a compile-time constant and goes
// into the immediate of s_waitcnt.  The wait statement takes the fragment as an in/out operand, so
// the consumer depends on the wait and the wait on the read, wherever the scheduler puts them.
// Reads the compiler issues by itself in between only make these waits stricter than necessary.
// Instruction offsets are 16-bit immediates; issue_row / issue_col move what exceeds them into the
// address register (a compile-time constant per call site, so at most one add per address).
struct LdsQueue { int issued; };
struct RowFrag { u32x4 v; int seq; };
struct ColFrag { u32x2 lo, hi; int seq; };

__device__ __forceinline__ void lds_issue_row(LdsQueue& q, RowFrag& f, uint32_t addr, int off) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f.v) : "v"(addr), "i"(off));
    f.seq = ++q.issued;
}
__device__ __forceinline__ void lds_issue_col(LdsQueue& q, ColFrag& f, uint32_t addr_lo, uint32_t addr_hi, int off) {
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(f.lo) : "v"(addr_lo), "i"(off));
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(f.hi) : "v"(addr_hi), "i"(off));
    q.issued += 2;
    f.seq = q.issued;
}
__device__ __forceinline__ bf16x8 lds_wait(const LdsQueue& q, RowFrag& f) {
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(f.v) : "i"(q.issued - f.seq < 15 ? q.issued - f.seq : 15));
    return as_bf16x8(f.v);
}
__device__ __forceinline__ bf16x8 lds_wait(const LdsQueue& q, ColFrag& f) {
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(f.lo), "+v"(f.hi) : "i"(q.issued - f.seq < 15 ? q.issued - f.seq : 15));
    u32x4 v = {f.lo[0], f.lo[1], f.hi[0], f.hi[1]};
    return as_bf16x8(v);
}
// Row fragment (blk, ks) of the tile at byte offset `tile` (indices as in frag_row); column
// fragment (contraction index = tile row): contraction step b (16 rows), column block cb (32
// columns), two transposing reads matched to the accumulator lane map as described above.
__device__ __forceinline__ void issue_row(LdsQueue& q, RowFrag& f, int tile, const FragAddr& fa, int blk, int ks) {
    const int off = tile + blk * 32 * kRowBytes, hi = off & ~0xffff;
    lds_issue_row(q, f, fa.row[ks] + (uint32_t)hi, off - hi);
}
__device__ __forceinline__ void issue_col(LdsQueue& q, ColFrag& f, int tile, const FragAddr& fa, int b, int cb) {
    const int off = tile + b * 16 * kRowBytes, hi = off & ~0xffff;
    lds_issue_col(q, f, fa.col[2 * cb] + (uint32_t)hi, fa.col[2 * cb + 1] + (uint32_t)hi, off - hi);
}
// Keeps a value's computation where the source puts it (the optimiser otherwise sinks work into
// the block of its first use).
__device__ __forceinline__ void pin(uint32_t& v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ void pin(float& v) { asm volatile("" : "+v"(v)); }

// Buffer resource over `bytes` bytes starting at `base`: loads beyond the range return zero, which
// is how the tails of a sequence are zero-filled without branches.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}

typedef __attribute__((address_space(3))) u32x2 lds_u32x2;

// Writes a transposed accumulator set acc[4] (rows = head dim, column = this lane's token: lane
// (l32, half) owns elements 32*db + 8*rq + 4*half + {0..3} of token l32) as 32 bf16 rows of 256
// bytes, `row_stride` elements apart, starting at `dst`.  The rows pass through 8 KB of LDS that
// belong to this wave alone (absolute address `stage`, free of other use), so that every store
// instruction writes four whole rows instead of 16 bytes of each of 32 rows: the address path of
// a CU handles a fixed number of cache lines per cycle, and 32 lines per instruction made the
// epilogue of an item as long as two of its steps.  Rows >= rows_valid are not written.
// The lane index is laundered through an empty asm statement so that the addresses are formed
// here (hoisted above the caller's tile loop they would hold some 40 registers through it).
template <int D = kHeadDim>
__device__ __forceinline__ void store_rows_via_lds(uint16_t* dst, int64_t row_stride, int rows_valid,
                                                   const f32x16 (&acc)[D / 32], float mul, uint32_t stage, int lane) {
    asm volatile("" : "+v"(lane));
    const int l32 = lane & 31, half = lane >> 5, c16 = lane & 15, r4 = lane >> 4;
    const uint32_t wbase = stage + (uint32_t)(l32 * kRowBytes + 8 * half);
    const int wswz = swz(l32);
#pragma unroll
    for (int db = 0; db < D / 32; ++db) {
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
            u32x2 w = {pack_bf16(acc[db][4 * rq] * mul, acc[db][4 * rq + 1] * mul),
                       pack_bf16(acc[db][4 * rq + 2] * mul, acc[db][4 * rq + 3] * mul)};
            *(lds_u32x2*)(uintptr_t)(wbase + (uint32_t)(((4 * db + rq) ^ wswz) << 4)) = w;
        }
    }
    // rows 4k + r4: swz() of such a row is ((r4 & 3) << 2) | (k & 3)
    uint16_t* ob = dst + (int64_t)r4 * row_stride + 8 * c16;
    const uint32_t rbase = stage + (uint32_t)(r4 * kRowBytes);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const u32x4 w = *(lds_u32x4*)(uintptr_t)(rbase + (uint32_t)(4 * k * kRowBytes + ((c16 ^ (((r4 & 3) << 2) | (k & 3))) << 4)));
        if (4 * k + r4 < rows_valid && (D == kHeadDim || c16 < D / 8)) *reinterpret_cast<u32x4*>(ob + (int64_t)(4 * k) * row_stride) = w;
    }
}

// Per-lane byte offset of a direct-to-LDS row load: lane i of a 64-lane instruction fills LDS
// position i%16 of tile row `row`, which in the swizzled layout holds chunk (i%16) ^ swz(row) of
// the row.  A head dimension of 64 has only chunks 0..7: the other lanes point far outside the
// buffer resource (their LDS bytes become zeros; nothing reads them), which requires resources
// below 2 GiB for D = 64.
constexpr uint32_t kDmaOutOfRange = 0x7fffff00u;
template <int D>
__device__ __forceinline__ uint32_t dma_lane_voff(int row, int lane, uint32_t row_stride_b) {
    const int chunk = (lane & 15) ^ swz(row);
    return (D == kHeadDim || chunk < D / 8) ? (uint32_t)row * row_stride_b + (uint32_t)(chunk << 4) : kDmaOutOfRange;
}

// Direct-to-LDS load of a block of `n64` x 64 rows of 256 bytes (row r of the block at byte r *
// row_stride_b of the resource) into LDS in the swizzled tile layout, 64-row tile j at lds + off(j).
// All NW waves of the workgroup call it; each issues n64 * 16 / NW instructions.
template <int NW, typename OffFn>
__device__ __forceinline__ void dma_rows(const __amdgpu_buffer_rsrc_t& rs, char* lds, OffFn off, int n64,
                                         uint32_t row_stride_b, int wave, uint32_t voff) {
    typedef __attribute__((address_space(3))) void lds_void_t;
#pragma unroll
    for (int sub = 0; sub < 4; ++sub) {
        if (sub < n64) {
#pragma unroll
            for (int j = 0; j < 16 / NW; ++j) {
                char* d = lds + off(sub) + (4 * wave + j * NW * 4) * kRowBytes;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void_t*)d, 16, voff, (uint32_t)(sub * 64 + j * NW * 4) * row_stride_b, 0, 0);
            }
        }
    }
}

// Both halves' values of v in every lane: lo = v of lane l % 32, hi = v of lane l % 32 + 32.  One
// v_permlane32_swap (gfx950) instead of a trip through LDS, whose wait would also drain every
// fragment read in flight.
__device__ __forceinline__ void both_halves(float v, float& lo, float& hi) {
    const uint32_t u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);   // swaps r[0]'s upper half with r[1]'s lower half
    lo = __uint_as_float(r[0]);
    hi = __uint_as_float(r[1]);
}

}  // namespace hyd

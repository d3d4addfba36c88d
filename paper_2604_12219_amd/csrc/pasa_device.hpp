// Device-side building blocks shared by the gfx950 kernels of the PASA forward: vector types,
// the swizzled LDS tile layout, global->LDS tile staging and the two MFMA operand fetches.
//
// LDS tile layout.  A tile is ROWS rows of D bf16 (a row of K, V, block-mean K or block-sum V),
// row r at byte r*2D.  Inside a row the 16-byte chunks are XOR-swizzled by a function of the row
// so that both access patterns below are bank-conflict free:
//   (a) "row fragment":   16 consecutive lanes read the same logical chunk of 16 consecutive rows
//                         (ds_read_b128) -- operand of S^T = K Q^T;
//   (b) "column fragment": ds_read_b64_tr_b16, where a half-wave reads 4 consecutive rows x 64 B
//                         -- operand of O^T = V^T P^T and of K^T V in the statistics kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void gbl_void;

#define PASA_DEVICE __device__ __forceinline__

// swizzle of the 16-byte chunk index inside a row (see the layout note above)
template <int D>
PASA_DEVICE int swz(int row) {
  if constexpr (D == 128) {
    return ((row & 3) << 2) | ((row >> 2) & 3);
  } else {  // D == 64: rows are 128 B, two rows share one 256-byte bank sweep
    return (((row >> 1) & 1) << 2) | (((row >> 3) & 1) << 1) | ((row >> 2) & 1);
  }
}

template <int D>
PASA_DEVICE int lds_chunk_off(int row, int chunk) {
  return row * (2 * D) + ((chunk ^ swz<D>(row)) << 4);
}

// value of the other half-wave's lane (lane ^ 32), combined with `op`
PASA_DEVICE float half_swap_max(float x) {
  u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
PASA_DEVICE float half_swap_sum(float x) {
  u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// ---- global -> registers -> LDS staging of a [rows x D] bf16 tile by T threads ------------------
template <int D, int T>
struct TileStage {
  static constexpr int CPR = D / 8;          // 16-byte chunks per row
  static constexpr int CH = 64 * CPR / T;    // chunks per thread for a 64-row tile
  static constexpr int RPP = T / CPR;        // rows covered by one pass of all threads
  uint4 r[CH];

  // rows [r0, r0+rows) of a row-major matrix with `stride` elements between rows; rows at or
  // beyond `rlimit` read as zero.  rows <= 64.
  PASA_DEVICE void load(const uint16_t* base, int64_t stride, int r0, int rows, int rlimit, int tid) {
#pragma unroll
    for (int p = 0; p < CH; ++p) {
      int row = p * RPP + tid / CPR, c = tid % CPR;
      uint4 z = {0u, 0u, 0u, 0u};
      if (row < rows && r0 + row < rlimit)
        z = *reinterpret_cast<const uint4*>(base + (int64_t)(r0 + row) * stride + c * 8);
      r[p] = z;
    }
  }
  PASA_DEVICE void store(char* lds, int rows, int tid) const {
#pragma unroll
    for (int p = 0; p < CH; ++p) {
      int row = p * RPP + tid / CPR, c = tid % CPR;
      if (row < rows) *reinterpret_cast<uint4*>(lds + lds_chunk_off<D>(row, c)) = r[p];
    }
  }
};

// (a) row fragment: lane (x = lane & 31, h = lane >> 5) gets elements [16*s + 8*h, +8) of row
//     row0 + x: the A operand of a 32x32x16 MFMA whose M index is the tile row.
template <int D>
PASA_DEVICE bf16x8 row_frag(const char* lds, int row0, int s, int lane) {
  int row = row0 + (lane & 31), c = 2 * s + (lane >> 5);
  return *reinterpret_cast<const bf16x8*>(lds + lds_chunk_off<D>(row, c));
}

// (b) column fragment: lane (x, h) gets, for column col0 + x, the 8 rows
//     row0 + 4*h + {0,1,2,3} and row0 + 8 + 4*h + {0,1,2,3}: the A (or B) operand of a 32x32x16
//     MFMA whose contraction index runs over tile rows.  This row order is exactly the order in
//     which a 32x32 MFMA result holds its M index in registers 8*(s)..8*(s)+7 of a lane, so a
//     P^T fragment cut from an S^T result pairs with it without any shuffle.
template <int D>
PASA_DEVICE bf16x8 col_frag(const char* lds, int row0, int col0, int lane) {
  int i = lane & 15, half16 = (lane >> 4) & 1, h = lane >> 5;
  int row = row0 + 4 * h + (i >> 2);
  int col = col0 + 16 * half16 + 4 * (i & 3);
  int c = col >> 3, inb = (col & 7) * 2;
  const char* lo = lds + lds_chunk_off<D>(row, c) + inb;
  const char* hi = lds + lds_chunk_off<D>(row + 8, c) + inb;
  s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)lo);
  s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)hi);
  s16x8 v = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

PASA_DEVICE f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// M index (row of the 32x32 result) held in register `reg` (0..15) of a lane in half-wave h
PASA_DEVICE int mfma_row(int reg, int h) { return 8 * (reg >> 2) + 4 * h + (reg & 3); }

// Shared pieces of the matrix-core (MFMA) scan kernels for gfx950.
//
// Tiling.  The K rows of the state are independent recurrences that share only
// W, v_t and f_t (row i of H W + k v^T needs row i of H and the scalar k_i;
// this is the structure Theorem 1 of the paper uses).  A workgroup therefore
// owns RB blocks of 16 rows of one (batch, head) state and all V columns; each
// wavefront owns one 16 x 16 tile: lane l holds rows 4*(l/16)+r (r = 0..3) of
// column l%16 -- the accumulator layout of the 16x16 MFMA family.  A state of
// K rows is split over P = K/(16*RB) workgroups so that small batches still
// fill 256 CUs; sums over rows (y, dv, df, dW) are finished across workgroups
// in a fixed order by small epilogue kernels.
//
// Scaled state.  tanh(x) = 1 - 2/(1 + 2^(c x)) with c = 2*log2(e).  The kernels
// carry H' = c*H in fp32 registers, so the fp16 operand cvt(H') makes the MFMA
// produce c*(H W) directly and the exponent needs no multiply; results that
// leave the chip (y, dq, dW, df, H_T, checkpoints) are scaled back by 1/c.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace m2rnn {

typedef _Float16 h2_t __attribute__((ext_vector_type(2)));
typedef _Float16 h4_t __attribute__((ext_vector_type(4)));
typedef _Float16 h8_t __attribute__((ext_vector_type(8)));
typedef float f4_t __attribute__((ext_vector_type(4)));
typedef unsigned short bf16_raw;

constexpr float kC = 2.8853900817779268f;  // 2*log2(e)
constexpr float kInvC = 0.34657359027997264f;
constexpr int kLdsLimit = 160 * 1024;

__device__ __forceinline__ float bf16_to_f32(bf16_raw x) {
  return __builtin_bit_cast(float, (uint32_t)x << 16);
}
// round to nearest even; NaN stays NaN
__device__ __forceinline__ bf16_raw f32_to_bf16(float x) {
  uint32_t u = __builtin_bit_cast(uint32_t, x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_raw)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_raw)(u >> 16);
}

__device__ __forceinline__ f4_t mfma_k32(h8_t a, h8_t b, f4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f4_t mfma_k16(h4_t a, h4_t b, f4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x16f16(a, b, c, 0, 0, 0);
}

template <int K_, int V_, int RB_>
struct Tile {
  static constexpr int K = K_, V = V_, RB = RB_;
  static constexpr int CT = V / 16;            // column tiles = waves per row block
  static constexpr int WAVES = RB * CT;
  static constexpr int THREADS = WAVES * 64;
  static constexpr int P = K / (16 * RB);      // workgroups per (b, n) state
  static constexpr int ROWS = RB * 16;         // state rows per workgroup
  static constexpr bool X32 = (V >= 32);       // 16x16x32 MFMA for the V-contraction
  static constexpr int KS = X32 ? V / 32 : 1;  // MFMAs per state contraction
  static constexpr int LDH = V + 8;            // halfs per row of a row-major exchange buffer
  static_assert(K % (16 * RB) == 0 && V % 16 == 0 && WAVES <= 16, "bad tile");
};

// Operand fragment of the V-contraction (8 halfs for the k=32 MFMA, 4 for k=16).
template <bool X32> struct Frag { typedef h8_t type; };
template <> struct Frag<false> { typedef h4_t type; };

// blockIdx -> (unit, part).  Workgroups are dealt round-robin to the 8 XCDs, so
// all P parts of a (b, n) state get ids that are equal mod 8: they then share
// one XCD's L2 for v_t, f_t and W.  Returns false for padding blocks.
template <int P>
__device__ __forceinline__ bool map_block(int units, int &unit, int &part) {
  const int x = blockIdx.x;
  const int xcd = x & 7, r = x >> 3;
  part = r % P;
  unit = xcd + 8 * (r / P);
  return unit < units;
}
inline int grid_blocks(int units, int P) { return 8 * P * ((units + 7) / 8); }

}  // namespace m2rnn

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
// Operand precision.  Gradients of this recurrence at T = 4096 are extremely
// sensitive to the forward trajectory (the backward amplifies a trajectory
// error of 2e-4 into gradient errors of several percent), so the state enters
// its contraction as an fp16 pair (hi, lo) with hi + lo = H' to ~21 bits.  The
// pair occupies two adjacent k-slots of the 16x16x32 MFMA and the W fragment
// holds each row of W twice.  All other matrix-core operands (dS, the stash
// copies of H and Z, q, k, v, dy) are single fp16 values.
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
typedef uint32_t u2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u4_t __attribute__((ext_vector_type(4)));
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

// H' -> fp16 pair packed in one dword: hi (H' truncated to 11 significant
// bits, exact in fp16) in the low half, lo = fp16(H' - hi) in the high half.
__device__ __forceinline__ uint32_t split_hi_lo(float h) {
  typedef float f2_t __attribute__((ext_vector_type(2)));
  const float hi = __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, h) & 0xFFFFE000u);
  const f2_t pr = {hi, h - hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, h2_t));
}
// the four hi halves of four packed pairs, as one MFMA fragment
__device__ __forceinline__ h4_t hi_of_pairs(const uint32_t (&pk)[4]) {
  uint2 v;
  v.x = (pk[0] & 0xFFFFu) | (pk[1] << 16);
  v.y = (pk[2] & 0xFFFFu) | (pk[3] << 16);
  return __builtin_bit_cast(h4_t, v);
}

// One state element through the non-linearity and the gate of the recurrence equations, on the
// scaled state:  H' <- f H' + gp tanh(s),  gp = c (1 - f),  sp = c s = 2 log2(e) s.
//     tanh(s) = sign(s) (1 - e) / (1 + e),   e = 2^-|sp|  in (0, 1].
// Why this form and not 1 - 2 / (1 + 2^sp): the forward trajectory of this recurrence can be
// transiently chaotic (units whose transition matrix has gain above one amplify a
// perturbation of the state by 10^4 .. 10^6 over a few hundred steps, and the backward
// gradient of such a unit follows the trajectory), so the ABSOLUTE error of tanh near zero
// decides how far such units drift from an exact evaluation.  1 - 2/(1+e) carries the
// rounding of exp2, of the sum and of the reciprocal as absolute errors (measured 4.4e-8
// rms); here 1 - e is exact for e in [1/2, 1] and the reciprocal's error is relative to the
// result, which leaves half an ulp of e in [1/2, 1) (measured 0.7e-8 rms).  e <= 1 also
// cannot overflow, whatever the pre-activation.  Two more vector instructions per element.
__device__ __forceinline__ float gate_tanh_step(float f, float gp, float h, float sp) {
  const float e = __builtin_amdgcn_exp2f(-__builtin_fabsf(sp));
  const float rr = __builtin_amdgcn_rcpf(1.f + e);
  const float n = fmaf(-gp, e, gp);                      // gp (1 - e) >= 0
  const float ns = __builtin_copysignf(n, sp);
  return fmaf(ns, rr, f * h);
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also drains
// the vector-memory counter, i.e. it would wait for every global load and store
// in flight (the staged q/k/v prefetch, the per-step y / dq / dk stores) at each
// of the one or two barriers a scan step needs.  Nothing is exchanged between
// waves through global memory inside these kernels, so only LDS must be settled.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// LDS access as base register + compile-time byte offset (the offset lands in the
// instruction's 16-bit immediate).  `lchar` pointers are 32-bit LDS addresses.
typedef __attribute__((address_space(3))) char lchar;
template <typename T>
__device__ __forceinline__ T lds_ld(const lchar *p, int off) {
  return *(const __attribute__((address_space(3))) T *)(p + off);
}
template <typename T>
__device__ __forceinline__ void lds_st(lchar *p, int off, T v) {
  *(__attribute__((address_space(3))) T *)(p + off) = v;
}

__device__ __forceinline__ f4_t mfma_k32(h8_t a, h8_t b, f4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f4_t mfma_k16(h4_t a, h4_t b, f4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x16f16(a, b, c, 0, 0, 0);
}

// Reads a just-finished MFMA chain's result into vector registers HERE, in the
// basic block that issued the MFMAs.  Without it the compiler may sink the first
// read of the result below a conditional block that follows the chain
// (MFMA; if (...) {long block}; use): the wait states an MFMA result needs before
// a vector-ALU read are then counted along the long path only, and the waves
// that skip the block read the accumulator too early (seen as wrong gradients).
// settle() alone only marks the spot: where a conditional block follows the chain, the first
// real consumer must also sit (and be pinned) in front of that block, as the backward's
// carry update does.  Guarded by tests/test_gpu_instantiations.py, which runs every tiling.
__device__ __forceinline__ void settle(f4_t &d) { asm volatile("" : "+v"(d)); }

// Maximum of a NON-NEGATIVE float over aligned groups of G = 2, 4, 8, 16, 32 or 64 consecutive
// lanes (result in every lane of the group), without LDS traffic: DPP steps inside each row
// of 16 lanes, then the rows through scalar registers.  Non-negative floats order like
// their bit patterns, so the maxima are taken on integers.
template <int G>
__device__ __forceinline__ float group_max_nonneg(float x) {
  static_assert(G == 2 || G == 4 || G == 8 || G == 16 || G == 32 || G == 64, "group size");
  int v = __builtin_bit_cast(int, x);
  v = max(v, __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
  if constexpr (G > 2)
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
  if constexpr (G > 4)
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, false));  // row_half_mirror
  if constexpr (G > 8)
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, false));  // row_mirror
  if constexpr (G > 16) {
    const int r0 = __builtin_amdgcn_readlane(v, 0), r1 = __builtin_amdgcn_readlane(v, 16);
    const int r2 = __builtin_amdgcn_readlane(v, 32), r3 = __builtin_amdgcn_readlane(v, 48);
    if constexpr (G == 64)
      v = max(max(r0, r1), max(r2, r3));
    else
      v = (threadIdx.x & 32) ? max(r2, r3) : max(r0, r1);
  }
  return __builtin_bit_cast(float, v);
}
// eight bf16 values (one 16-byte load) widened to fp32
__device__ __forceinline__ void bf16x8_to_f32(const u4_t &w, float (&x)[8]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = __builtin_bit_cast(float, w[i] << 16);
    x[2 * i + 1] = __builtin_bit_cast(float, w[i] & 0xFFFF0000u);
  }
}
// 2^e with e clamped to the normal range
__device__ __forceinline__ float pow2i(int e) {
  e = e < -126 ? -126 : (e > 127 ? 127 : e);
  return __builtin_bit_cast(float, (uint32_t)(127 + e) << 23);
}
// floor(log2 x) of a positive finite float (subnormals count as 2^-127)
__device__ __forceinline__ int ilog2f(float x) {
  return (int)((__builtin_bit_cast(uint32_t, x) >> 23) & 255u) - 127;
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
  static constexpr int LDH = V + 8;            // halfs per row of a row-major fp16 exchange buffer
  static constexpr int LDH2 = 2 * V + 8;       // ... of a (hi, lo) pair exchange buffer
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


// (K, V, RB) tilings that are instantiated
#define M2RNN_TILE_CASES(X)                                                                      \
  X(64, 64, 2) X(64, 64, 1) X(128, 128, 1) X(32, 32, 2) X(32, 32, 1) X(16, 16, 1) X(64, 16, 1)

// (K, V) shapes of the register-resident (one wave per row block) kernels
#define M2RNN_ROWWAVE_CASES(X)                                                                  \
  X(16, 16) X(32, 16) X(64, 16) X(128, 16) X(16, 32) X(32, 32) X(64, 32) X(128, 32) X(16, 64)   \
  X(32, 64) X(64, 64) X(128, 64)

}  // namespace m2rnn

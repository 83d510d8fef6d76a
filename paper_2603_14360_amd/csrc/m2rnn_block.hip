// The scan's two neighbours in the M2RNN block (layer equations of the "M2RNN Block"
// section), as bandwidth-bound kernels that touch every tensor once:
//   * prologue of q, k, v:  out = SiLU(conv1d(x)), depthwise causal convolution of kernel
//     size 4 along time (zero left padding; tap j meets step t - 3 + j), and its backward;
//   * epilogue of y:  out = RMSNorm(y (.) SiLU(a)) over all D = N V features of a token
//     (forward and backward as printed in the "RMSNormTP Module" appendix, eps under the
//     root), and its backward.
// Why they are kernels of their own and not folded into the scan kernels: the norm spans all
// heads of a token while a scan workgroup holds one head, and the scan is bound by its vector
// ALUs with HBM at a few percent of peak, where a convolution re-evaluated by every workgroup
// that stages the same q, k, v rows would add exactly the instructions that bind it.  Here
// each tensor makes one trip through HBM: x -> out, and (y, a) -> out.
// Sums over tokens (dw, dbias) are two-stage and ordered: bit-reproducible, no atomics.
#include "m2rnn_kernels.hpp"

#include <hip/hip_bf16.h>

namespace m2rnn {
namespace {

typedef float f4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t lo16) {
  return __builtin_bit_cast(float, lo16 << 16);
}
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float x) {  // round to nearest even
  uint32_t u = __builtin_bit_cast(uint32_t, x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

// eight consecutive elements of an io tensor <-> eight floats
template <typename IO> struct Vec8;
template <> struct Vec8<float> {
  struct Raw { f4_t a, b; };
  static __device__ __forceinline__ Raw load_raw(const void *base, size_t e) {
    return Raw{*(const f4_t *)((const float *)base + e), *(const f4_t *)((const float *)base + e + 4)};
  }
  static __device__ __forceinline__ void widen(const Raw &r, float (&x)[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) { x[i] = r.a[i]; x[4 + i] = r.b[i]; }
  }
  static __device__ __forceinline__ void load(const void *base, size_t e, float (&x)[8]) {
    const f4_t a = *(const f4_t *)((const float *)base + e), b = *(const f4_t *)((const float *)base + e + 4);
#pragma unroll
    for (int i = 0; i < 4; ++i) { x[i] = a[i]; x[4 + i] = b[i]; }
  }
  static __device__ __forceinline__ void store(void *base, size_t e, const float (&x)[8]) {
    *(f4_t *)((float *)base + e) = f4_t{x[0], x[1], x[2], x[3]};
    *(f4_t *)((float *)base + e + 4) = f4_t{x[4], x[5], x[6], x[7]};
  }
};
template <> struct Vec8<__hip_bfloat16> {
  typedef u4_t Raw;
  static __device__ __forceinline__ Raw load_raw(const void *base, size_t e) {
    return *(const u4_t *)((const unsigned short *)base + e);
  }
  static __device__ __forceinline__ void widen(const Raw &w, float (&x)[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = bf16_bits_to_f32(w[i] & 0xFFFFu);
      x[2 * i + 1] = __builtin_bit_cast(float, w[i] & 0xFFFF0000u);
    }
  }
  static __device__ __forceinline__ void load(const void *base, size_t e, float (&x)[8]) {
    const u4_t w = *(const u4_t *)((const unsigned short *)base + e);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = bf16_bits_to_f32(w[i] & 0xFFFFu);
      x[2 * i + 1] = __builtin_bit_cast(float, w[i] & 0xFFFF0000u);
    }
  }
  static __device__ __forceinline__ void store(void *base, size_t e, const float (&x)[8]) {
    u4_t w;
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = f32_to_bf16_bits(x[2 * i]) | (f32_to_bf16_bits(x[2 * i + 1]) << 16);
    *(u4_t *)((unsigned short *)base + e) = w;
  }
};
// 1 / (1 + e^-u) on the hardware's exp2 and reciprocal (1 ulp each; e^-u = inf gives 0)
__device__ __forceinline__ float sigmoidf_(float u) {
  return __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * u));
}

// ------------------------------------------------------------------ conv1d(4) + SiLU
constexpr int kTaps = 4;
constexpr int kSeg = 32;  // time steps per work item (3 halo rows are re-read: 9 %)
constexpr int kBlk = 8;   // steps whose loads are issued together

// taps [8 channels][4] (32 consecutive elements of w [C,4]) and bias of channels c0 .. c0 + 7
template <typename IO>
__device__ __forceinline__ void load_taps(const void *w, const void *bias, int c0, float (&wt)[8][kTaps],
                                          float (&bs)[8]) {
  float wv[4][8];
#pragma unroll
  for (int q = 0; q < 4; ++q) Vec8<IO>::load(w, (size_t)c0 * kTaps + 8 * q, wv[q]);
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < kTaps; ++j) wt[i][j] = wv[(i * kTaps + j) / 8][(i * kTaps + j) % 8];
  if (bias) Vec8<IO>::load(bias, c0, bs);
  else
#pragma unroll
    for (int i = 0; i < 8; ++i) bs[i] = 0.f;
}

// One work item = 8 channels x kSeg steps of one batch row.  Items are numbered with the
// channel vector fastest, so a wave reads 1 KB (bf16) of one time step at a time.
template <typename IO>
__global__ void __launch_bounds__(256)
    conv_silu_fwd_kernel(const void *__restrict__ x, const void *__restrict__ w,
                         const void *__restrict__ bias, void *__restrict__ out, int B, int T, int C) {
  const int CV = C / 8, nseg = (T + kSeg - 1) / kSeg;
  const size_t items = (size_t)B * nseg * CV;
  for (size_t it = blockIdx.x * (size_t)blockDim.x + threadIdx.x; it < items;
       it += (size_t)gridDim.x * blockDim.x) {
    const int cv = it % CV;
    const size_t r = it / CV;
    const int seg = r % nseg, b = r / nseg;
    const int c0 = cv * 8, t0 = seg * kSeg, t1 = t0 + kSeg < T ? t0 + kSeg : T;
    float wt[8][kTaps], bs[8];
    load_taps<IO>(w, bias, c0, wt, bs);
    float win[kTaps - 1][8];  // steps t-3, t-2, t-1
#pragma unroll
    for (int j = 0; j < kTaps - 1; ++j) {
      const int ts = t0 - (kTaps - 1) + j;
      if (ts >= 0) Vec8<IO>::load(x, ((size_t)b * T + ts) * C + c0, win[j]);
      else
#pragma unroll
        for (int i = 0; i < 8; ++i) win[j][i] = 0.f;
    }
    // kBlk steps at a time: their loads are all in flight before the first is used (one load
    // per iteration would expose the memory latency kSeg times per item)
    for (int tb = t0; tb < t1; tb += kBlk) {
      typename Vec8<IO>::Raw raw[kBlk];
#pragma unroll
      for (int u = 0; u < kBlk; ++u) {
        const int t = tb + u < t1 ? tb + u : t1 - 1;  // (clamped: every load is unconditional)
        raw[u] = Vec8<IO>::load_raw(x, ((size_t)b * T + t) * C + c0);
      }
#pragma unroll
      for (int u = 0; u < kBlk; ++u) {
        if (tb + u < t1) {
          float cur[8], o[8];
          Vec8<IO>::widen(raw[u], cur);
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const float a = bs[i] + wt[i][0] * win[0][i] + wt[i][1] * win[1][i] + wt[i][2] * win[2][i] +
                            wt[i][3] * cur[i];
            o[i] = a * sigmoidf_(a);
            win[0][i] = win[1][i];
            win[1][i] = win[2][i];
            win[2][i] = cur[i];
          }
          Vec8<IO>::store(out, ((size_t)b * T + tb + u) * C + c0, o);
        }
      }
    }
  }
}

// Backward.  A work item recomputes the pre-activation of its own steps and of the three
// after them (their gradients reach back into its steps), forms da = dout SiLU'(a), and
// finishes dx of step t-3 as soon as da of step t is known.  dw and dbias of its OWN steps are
// summed per thread over the items it walks (row r, r + R, ...: increasing time inside a batch
// row, increasing batch row) and written to part[row][C][5]; conv_sum_kernel adds the rows.
template <typename IO>
__global__ void __launch_bounds__(256)
    conv_silu_bwd_kernel(const void *__restrict__ x, const void *__restrict__ w,
                         const void *__restrict__ bias, const void *__restrict__ dout,
                         void *__restrict__ dx, float *__restrict__ part, int B, int T, int C, int R) {
  // A workgroup = 8 walker rows x 32 channel vectors; its 8 partial sums per channel are added
  // through LDS (increasing row) before they leave, so part has R / 8 rows.
  const int CV = C / 8, nseg = (T + kSeg - 1) / kSeg;
  const int rows = B * nseg;
  const int CVB = (CV + 31) / 32;
  const int cvl = threadIdx.x & 31, rl = threadIdx.x >> 5;
  const int cvb = blockIdx.x % CVB, rg = blockIdx.x / CVB;
  const int cv = cvb * 32 + cvl, row0 = rg * 8 + rl;
  const bool walker = cv < CV && row0 < R;
  const int c0 = (cv < CV ? cv : CV - 1) * 8;
  __shared__ float red[8][32][8 * (kTaps + 1)];
  float wt[8][kTaps], bs[8], dwacc[8][kTaps], dbacc[8];
  load_taps<IO>(w, bias, c0, wt, bs);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
#pragma unroll
    for (int j = 0; j < kTaps; ++j) dwacc[i][j] = 0.f;
    dbacc[i] = 0.f;
  }
  for (int r = walker ? row0 : rows; r < rows; r += R) {
    const int seg = r % nseg, b = r / nseg;
    const int t0 = seg * kSeg, t1 = t0 + kSeg < T ? t0 + kSeg : T;
    float win[kTaps - 1][8], dawin[kTaps - 1][8];  // x and da of steps t-3, t-2, t-1
#pragma unroll
    for (int j = 0; j < kTaps - 1; ++j) {
      const int ts = t0 - (kTaps - 1) + j;
      if (ts >= 0) Vec8<IO>::load(x, ((size_t)b * T + ts) * C + c0, win[j]);
      else
#pragma unroll
        for (int i = 0; i < 8; ++i) win[j][i] = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) dawin[j][i] = 0.f;   // da of earlier steps does not reach mine
    }
    // (BLK steps at a time, loads first: see the forward)
    constexpr int BLK = sizeof(IO) == 4 ? kBlk / 2 : kBlk;
    const int tend = t1 + (kTaps - 1);
    for (int tb = t0; tb < tend; tb += BLK) {
     typename Vec8<IO>::Raw rx[BLK], rd[BLK];
#pragma unroll
     for (int u = 0; u < BLK; ++u) {
       const int tc = tb + u < T ? tb + u : T - 1;
       rx[u] = Vec8<IO>::load_raw(x, ((size_t)b * T + tc) * C + c0);
       rd[u] = Vec8<IO>::load_raw(dout, ((size_t)b * T + tc) * C + c0);
     }
#pragma unroll
     for (int u = 0; u < BLK; ++u) {
      const int t = tb + u;
      if (t >= tend) break;
      float cur[8], da[8];
      if (t < T) {
        float dd[8];
        Vec8<IO>::widen(rx[u], cur);
        Vec8<IO>::widen(rd[u], dd);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float a = bs[i] + wt[i][0] * win[0][i] + wt[i][1] * win[1][i] + wt[i][2] * win[2][i] +
                          wt[i][3] * cur[i];
          const float sg = sigmoidf_(a);
          da[i] = dd[i] * (sg * (1.f + a * (1.f - sg)));
        }
        if (t < t1) {  // my own step: its share of dw, dbias
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            dwacc[i][0] = fmaf(da[i], win[0][i], dwacc[i][0]);
            dwacc[i][1] = fmaf(da[i], win[1][i], dwacc[i][1]);
            dwacc[i][2] = fmaf(da[i], win[2][i], dwacc[i][2]);
            dwacc[i][3] = fmaf(da[i], cur[i], dwacc[i][3]);
            dbacc[i] += da[i];
          }
        }
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) { cur[i] = 0.f; da[i] = 0.f; }
      }
      const int td = t - (kTaps - 1);  // dx of this step is complete now
      if (td >= t0) {
        float o[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
          o[i] = wt[i][3] * dawin[0][i] + wt[i][2] * dawin[1][i] + wt[i][1] * dawin[2][i] + wt[i][0] * da[i];
        Vec8<IO>::store(dx, ((size_t)b * T + td) * C + c0, o);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        win[0][i] = win[1][i]; win[1][i] = win[2][i]; win[2][i] = cur[i];
        dawin[0][i] = dawin[1][i]; dawin[1][i] = dawin[2][i]; dawin[2][i] = da[i];
      }
     }
    }
  }
  constexpr int PER = 8 * (kTaps + 1);  // floats per channel vector: [8 channels][4 taps, bias]
#pragma unroll
  for (int i = 0; i < 8; ++i) {
#pragma unroll
    for (int j = 0; j < kTaps; ++j) red[rl][cvl][i * (kTaps + 1) + j] = dwacc[i][j];
    red[rl][cvl][i * (kTaps + 1) + kTaps] = dbacc[i];
  }
  __syncthreads();
  float *dst = part + ((size_t)rg * C + (size_t)cvb * 32 * 8) * (kTaps + 1);
  for (int o = threadIdx.x; o < 32 * PER; o += 256) {
    const int cl = o / PER, j = o - cl * PER;
    if (cvb * 32 + cl < CV) {
      float acc = red[0][cl][j];
#pragma unroll
      for (int q = 1; q < 8; ++q) acc += red[q][cl][j];
      dst[o] = acc;
    }
  }
}

// Ordered sum of R partial rows of E floats, in two levels so that it is both parallel and
// reproducible: group g (blockIdx.y) adds its rows g*per .. (g+1)*per - 1 in increasing order
// into row g of `lvl` (kSumGroups rows behind the partials); the second level adds those.
constexpr int kSumGroups = 32;
// Sum of p[r * stride] for r in [r0, r1) in a FIXED order that keeps eight loads in flight:
// eight interleaved running sums (rows r0 + k, r0 + k + 8, ...), combined pairwise at the end.
// (One running sum is a chain of dependent loads: these kernels are a few workgroups, and
// with it each of them paid the memory latency once per row.)
__device__ __forceinline__ float strided_sum8(const float *__restrict__ p, size_t stride, int r0, int r1) {
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  int r = r0;
  for (; r + 8 <= r1; r += 8) {
    float x[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) x[k] = p[(size_t)(r + k) * stride];
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] += x[k];
  }
  for (int k = 0; r < r1; ++r, ++k) acc[k] += p[(size_t)r * stride];
  return ((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]));
}
__global__ void ordered_sum_level1_kernel(const float *__restrict__ part, float *__restrict__ lvl,
                                          int E, int R) {
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= E) return;
  const int per = (R + kSumGroups - 1) / kSumGroups;
  const int r0 = blockIdx.y * per, r1 = r0 + per < R ? r0 + per : R;
  lvl[(size_t)blockIdx.y * E + e] = strided_sum8(part + e, (size_t)E, r0, r1);
}
__global__ void conv_sum_kernel(const float *__restrict__ lvl, float *__restrict__ dw,
                                float *__restrict__ dbias, int C, int groups) {
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= C * (kTaps + 1)) return;
  const float s = strided_sum8(lvl + e, (size_t)C * (kTaps + 1), 0, groups);
  const int c = e / (kTaps + 1), j = e - c * (kTaps + 1);
  if (j < kTaps) dw[c * kTaps + j] = s;
  else if (dbias) dbias[c] = s;
}

// ------------------------------------------------------------------ gated RMSNorm
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
  return v;
}

// One wave per token; a lane owns the 8-element vectors lane, lane + 64, ... of its D features.
// NV = 8-element vectors per lane (D <= 512 NV).  A token is read from memory ONCE: the
// forward keeps x = y SiLU(a) in registers between the sum of squares and the output, the
// backward keeps the raw y, a, dout vectors (fp32 io with more than 4 vectors per lane
// re-reads them instead: they would not fit).
template <typename IO, int NV>
__global__ void __launch_bounds__(256)
    gated_rmsnorm_fwd_kernel(const void *__restrict__ y, const void *__restrict__ a,
                             const void *__restrict__ w, float eps, void *__restrict__ out,
                             float *__restrict__ s_out, size_t tokens, int D) {
  const int lane = threadIdx.x & 63, DV = D / 8;
  const size_t wave = (blockIdx.x * (size_t)blockDim.x + threadIdx.x) >> 6;
  const size_t nwaves = ((size_t)gridDim.x * blockDim.x) >> 6;
  for (size_t tok = wave; tok < tokens; tok += nwaves) {
    typename Vec8<IO>::Raw ry[NV], ra[NV];
#pragma unroll
    for (int q = 0; q < NV; ++q) {
      const int v = lane + 64 * q, vc = v < DV ? v : DV - 1;  // (clamped: loads are unconditional)
      ry[q] = Vec8<IO>::load_raw(y, tok * D + 8 * vc);
      ra[q] = Vec8<IO>::load_raw(a, tok * D + 8 * vc);
    }
    float x[NV][8];
    float ss = 0.f;
#pragma unroll
    for (int q = 0; q < NV; ++q) {
      float yy[8], aa[8];
      Vec8<IO>::widen(ry[q], yy);
      Vec8<IO>::widen(ra[q], aa);
      const bool ok = lane + 64 * q < DV;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        x[q][i] = ok ? yy[i] * (aa[i] * sigmoidf_(aa[i])) : 0.f;
        ss = fmaf(x[q][i], x[q][i], ss);
      }
    }
    ss = wave_sum(ss);
    const float s = 1.f / sqrtf(ss / (float)D + eps);
    if (s_out && lane == 0) s_out[tok] = s;
#pragma unroll
    for (int q = 0; q < NV; ++q) {
      const int v = lane + 64 * q;
      if (v < DV) {
        float ww[8], o[8];
        Vec8<IO>::load(w, 8 * v, ww);
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = ww[i] * x[q][i] * s;
        Vec8<IO>::store(out, tok * D + 8 * v, o);
      }
    }
  }
}

constexpr int kMaxVecPerLane = 8;  // D <= 8 * 64 * 8 = 4096

// Backward (appendix): p = w dout, r = sum p x, dx = s p - r s^3 x / d; dy = dx g,
// da = dx y SiLU'(a); dw = sum over tokens of dout x s: per wave over the tokens it walks
// (increasing), written to part[wave][D]; norm_sum_kernel adds the waves in order.
template <typename IO, int NV>
__global__ void __launch_bounds__(256)
    gated_rmsnorm_bwd_kernel(const void *__restrict__ y, const void *__restrict__ a,
                             const void *__restrict__ w, float eps, const float *__restrict__ s_in,
                             const void *__restrict__ dout, void *__restrict__ dy,
                             void *__restrict__ da, float *__restrict__ part, size_t tokens, int D) {
  constexpr bool KEEP = sizeof(IO) == 2 || NV <= 4;
  const int lane = threadIdx.x & 63, DV = D / 8;
  const size_t wave = (blockIdx.x * (size_t)blockDim.x + threadIdx.x) >> 6;
  const size_t nwaves = ((size_t)gridDim.x * blockDim.x) >> 6;
  float dwacc[NV][8];
#pragma unroll
  for (int q = 0; q < NV; ++q)
#pragma unroll
    for (int i = 0; i < 8; ++i) dwacc[q][i] = 0.f;
  // The next token of this wave is fetched while the current one is worked on (a wave walks
  // several tokens, and a token is two dependent phases with a wave-wide sum between them).
  constexpr bool PF = NV * sizeof(IO) <= 8;  // (two sets of raw vectors must fit the registers)
  typename Vec8<IO>::Raw ry[NV], ra[NV], rd[NV], ny[NV], na[NV], nd[NV];
  auto fetch = [&](size_t tok, typename Vec8<IO>::Raw (&fy)[NV], typename Vec8<IO>::Raw (&fa)[NV],
                   typename Vec8<IO>::Raw (&fd)[NV]) {
#pragma unroll
    for (int q = 0; q < NV; ++q) {
      const int v = lane + 64 * q, vc = v < DV ? v : DV - 1;  // (clamped: loads are unconditional)
      fy[q] = Vec8<IO>::load_raw(y, tok * D + 8 * vc);
      fa[q] = Vec8<IO>::load_raw(a, tok * D + 8 * vc);
      fd[q] = Vec8<IO>::load_raw(dout, tok * D + 8 * vc);
    }
  };
  if (PF && wave < tokens) fetch(wave, ny, na, nd);
  for (size_t tok = wave; tok < tokens; tok += nwaves) {
    if constexpr (PF) {
#pragma unroll
      for (int q = 0; q < NV; ++q) { ry[q] = ny[q]; ra[q] = na[q]; rd[q] = nd[q]; }
      const size_t nx = tok + nwaves < tokens ? tok + nwaves : tok;  // (last token: fetched again, unused)
      fetch(nx, ny, na, nd);
    } else {
      fetch(tok, ry, ra, rd);
    }
    float ss = 0.f, r = 0.f;
#pragma unroll
    for (int q = 0; q < NV; ++q) {
      const int v = lane + 64 * q;
      if (v < DV) {
        float yy[8], aa[8], dd[8], ww[8];
        Vec8<IO>::widen(ry[q], yy);
        Vec8<IO>::widen(ra[q], aa);
        Vec8<IO>::widen(rd[q], dd);
        Vec8<IO>::load(w, 8 * v, ww);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float xi = yy[i] * (aa[i] * sigmoidf_(aa[i]));
          ss = fmaf(xi, xi, ss);
          r = fmaf(ww[i] * dd[i], xi, r);
        }
      }
    }
    r = wave_sum(r);
    float s;
    if (s_in) s = s_in[tok];
    else s = 1.f / sqrtf(wave_sum(ss) / (float)D + eps);
    const float c3 = r * s * s * s / (float)D;
#pragma unroll
    for (int q = 0; q < NV; ++q) {
      const int v = lane + 64 * q;
      if (v < DV) {
        float yy[8], aa[8], dd[8], ww[8], oy[8], oa[8];
        if constexpr (KEEP) {
          Vec8<IO>::widen(ry[q], yy);
          Vec8<IO>::widen(ra[q], aa);
          Vec8<IO>::widen(rd[q], dd);
        } else {
          Vec8<IO>::load(y, tok * D + 8 * v, yy);
          Vec8<IO>::load(a, tok * D + 8 * v, aa);
          Vec8<IO>::load(dout, tok * D + 8 * v, dd);
        }
        Vec8<IO>::load(w, 8 * v, ww);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float sg = sigmoidf_(aa[i]);
          const float g = aa[i] * sg;
          const float xi = yy[i] * g;
          const float dxi = s * (ww[i] * dd[i]) - c3 * xi;
          dwacc[q][i] = fmaf(dd[i] * xi, s, dwacc[q][i]);
          oy[i] = dxi * g;
          oa[i] = dxi * yy[i] * (sg * (1.f + aa[i] * (1.f - sg)));
        }
        Vec8<IO>::store(dy, tok * D + 8 * v, oy);
        Vec8<IO>::store(da, tok * D + 8 * v, oa);
      }
    }
  }
#pragma unroll
  for (int q = 0; q < NV; ++q) {
    const int v = lane + 64 * q;
    if (v < DV) {
      *(f4_t *)&part[wave * D + 8 * v] = f4_t{dwacc[q][0], dwacc[q][1], dwacc[q][2], dwacc[q][3]};
      *(f4_t *)&part[wave * D + 8 * v + 4] = f4_t{dwacc[q][4], dwacc[q][5], dwacc[q][6], dwacc[q][7]};
    }
  }
}

__global__ void norm_sum_kernel(const float *__restrict__ lvl, float *__restrict__ dw, int D, int groups) {
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= D) return;
  dw[e] = strided_sum8(lvl + e, (size_t)D, 0, groups);
}

// Partial rows of the weight-gradient sums.  Many rows = many independent walkers (these
// kernels are bound by memory latency per walker, not by arithmetic); the partials cost
// 2 x rows x features x 4 B of extra traffic, about a fifth of the tensors' own at these caps.
constexpr int kConvRows = 2048;  // of the convolution's dw / dbias sums
constexpr int kNormWaves = 4096; // of the norm's dw sum

inline int conv_rows(int B, int T) {
  const long long rows = (long long)B * ((T + kSeg - 1) / kSeg);
  return (int)(rows < kConvRows ? (rows < 1 ? 1 : rows) : kConvRows);
}
// (a multiple of four: whole workgroups; waves beyond the tokens write zero rows)
inline int norm_waves(size_t tokens) {
  const size_t r = tokens < (size_t)kNormWaves ? (tokens < 1 ? 1 : tokens) : kNormWaves;
  return (int)((r + 3) / 4 * 4);
}

}  // namespace

size_t conv_silu_scratch_bytes(int B, int T, int C) {
  return align256((size_t)(conv_rows(B, T) + kSumGroups) * C * (kTaps + 1) * sizeof(float));
}
size_t gated_rmsnorm_scratch_bytes(int B, int T, int D) {
  return align256((size_t)(norm_waves((size_t)B * T) + kSumGroups) * D * sizeof(float));
}
int gated_rmsnorm_max_features() { return kMaxVecPerLane * 64 * 8; }

template <typename IO>
static hipError_t conv_fwd_t(int B, int T, int C, const void *x, const void *w, const void *bias,
                             void *out, hipStream_t s) {
  const size_t items = (size_t)B * ((T + kSeg - 1) / kSeg) * (C / 8);
  if (items == 0) return hipSuccess;
  size_t blocks = (items + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL((conv_silu_fwd_kernel<IO>), dim3((unsigned)blocks), dim3(256), 0, s, x, w, bias, out, B, T, C);
  return hipGetLastError();
}
hipError_t conv_silu_fwd(int B, int T, int C, int io, const void *x, const void *w, const void *bias,
                         void *out, hipStream_t s) {
  return io == 0 ? conv_fwd_t<float>(B, T, C, x, w, bias, out, s)
                 : conv_fwd_t<__hip_bfloat16>(B, T, C, x, w, bias, out, s);
}

template <typename IO>
static hipError_t conv_bwd_t(int B, int T, int C, const void *x, const void *w, const void *bias,
                             const void *dout, void *dx, float *dw, float *dbias, float *part,
                             hipStream_t s) {
  const int R = conv_rows(B, T);
  const int RG = (R + 7) / 8;  // partial rows that leave the kernel
  const bool any = (size_t)B * T > 0;
  if (any) {
    const int CVB = (C / 8 + 31) / 32;
    hipLaunchKernelGGL((conv_silu_bwd_kernel<IO>), dim3((unsigned)(CVB * RG)), dim3(256), 0, s,
                       x, w, bias, dout, dx, part, B, T, C, R);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const int E = C * (kTaps + 1);
  float *lvl = part + (size_t)RG * E;
  if (any)
    hipLaunchKernelGGL(ordered_sum_level1_kernel, dim3((E + 255) / 256, kSumGroups), dim3(256), 0, s,
                       (const float *)part, lvl, E, RG);
  hipLaunchKernelGGL(conv_sum_kernel, dim3((E + 255) / 256), dim3(256), 0, s, (const float *)lvl, dw,
                     dbias, C, any ? kSumGroups : 0);
  return hipGetLastError();
}
hipError_t conv_silu_bwd(int B, int T, int C, int io, const void *x, const void *w, const void *bias,
                         const void *dout, void *dx, float *dw, float *dbias, float *part,
                         hipStream_t s) {
  return io == 0 ? conv_bwd_t<float>(B, T, C, x, w, bias, dout, dx, dw, dbias, part, s)
                 : conv_bwd_t<__hip_bfloat16>(B, T, C, x, w, bias, dout, dx, dw, dbias, part, s);
}

template <typename IO>
static hipError_t norm_fwd_t(int B, int T, int D, const void *y, const void *a, const void *w, float eps,
                             void *out, float *s_out, hipStream_t s) {
  const size_t tokens = (size_t)B * T;
  if (tokens == 0) return hipSuccess;
  size_t blocks = (tokens + 3) / 4;  // four waves = four tokens per workgroup
  if (blocks > 16384) blocks = 16384;
  const int nv = (D / 8 + 63) / 64;
#define M2RNN_GO(NV_)                                                                              \
  hipLaunchKernelGGL((gated_rmsnorm_fwd_kernel<IO, NV_>), dim3((unsigned)blocks), dim3(256), 0, s, y, a, \
                     w, eps, out, s_out, tokens, D)
  if (nv <= 1) M2RNN_GO(1);
  else if (nv <= 2) M2RNN_GO(2);
  else if (nv <= 4) M2RNN_GO(4);
  else M2RNN_GO(8);
#undef M2RNN_GO
  return hipGetLastError();
}
hipError_t gated_rmsnorm_fwd(int B, int T, int D, int io, const void *y, const void *a, const void *w,
                             float eps, void *out, float *s_out, hipStream_t s) {
  return io == 0 ? norm_fwd_t<float>(B, T, D, y, a, w, eps, out, s_out, s)
                 : norm_fwd_t<__hip_bfloat16>(B, T, D, y, a, w, eps, out, s_out, s);
}

template <typename IO>
static hipError_t norm_bwd_t(int B, int T, int D, const void *y, const void *a, const void *w, float eps,
                             const float *s_in, const void *dout, void *dy, void *da, float *dw,
                             float *part, hipStream_t s) {
  const size_t tokens = (size_t)B * T;
  const int R = norm_waves(tokens);
  if (tokens > 0) {
    const int nv = (D / 8 + 63) / 64;
#define M2RNN_GO(NV_)                                                                              \
  hipLaunchKernelGGL((gated_rmsnorm_bwd_kernel<IO, NV_>), dim3(R / 4), dim3(256), 0, s, y, a, w, eps,   \
                     s_in, dout, dy, da, part, tokens, D)
    if (nv <= 1) M2RNN_GO(1);
    else if (nv <= 2) M2RNN_GO(2);
    else if (nv <= 4) M2RNN_GO(4);
    else M2RNN_GO(8);
#undef M2RNN_GO
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  float *lvl = part + (size_t)R * D;
  if (tokens > 0)
    hipLaunchKernelGGL(ordered_sum_level1_kernel, dim3((D + 255) / 256, kSumGroups), dim3(256), 0, s,
                       (const float *)part, lvl, D, R);
  hipLaunchKernelGGL(norm_sum_kernel, dim3((D + 255) / 256), dim3(256), 0, s, (const float *)lvl, dw, D,
                     tokens > 0 ? kSumGroups : 0);
  return hipGetLastError();
}
hipError_t gated_rmsnorm_bwd(int B, int T, int D, int io, const void *y, const void *a, const void *w,
                             float eps, const float *s_in, const void *dout, void *dy, void *da,
                             float *dw, float *part, hipStream_t s) {
  return io == 0 ? norm_bwd_t<float>(B, T, D, y, a, w, eps, s_in, dout, dy, da, dw, part, s)
                 : norm_bwd_t<__hip_bfloat16>(B, T, D, y, a, w, eps, s_in, dout, dy, da, dw, part, s);
}

}  // namespace m2rnn

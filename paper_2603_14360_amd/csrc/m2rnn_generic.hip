// fp32 scan kernels: one workgroup per (batch, head) recurrence, the K x V
// state resident in LDS for all T steps, every contraction done with fp32
// vector FMAs.  This is the path for float32 io (1e-5 parity class) and for
// shapes the matrix-core kernels do not cover.
//
// Forward : recurrence equations / Algorithm 1 of the paper.
// Backward: Algorithm 2 (BPTT) with the carried state gradient added to
//           q dy^T and propagated as f*G + dS W^T.  Instead of the paper's
//           H_full cache of every state, the forward stores one fp32 checkpoint
//           every C steps and the backward recomputes a chunk of C states into
//           a per-recurrence scratch that stays in L2.
#include "m2rnn_kernels.hpp"

#include <hip/hip_bf16.h>

namespace m2rnn {
namespace {

constexpr int kMaxThreads = 1024;
constexpr int kMaxPerThread = 16;  // 128*128 / 1024
constexpr size_t kLdsBudget = 160 * 1024 - 2048;
// unroll factor of the contraction loops: as far as the registers left by PT elements per
// thread allow without spilling
template <int PT> constexpr int kUnrollOf = PT <= 2 ? 8 : (PT <= 4 ? 2 : 1);

template <typename IO> __device__ __forceinline__ float to_f32(IO x);
template <> __device__ __forceinline__ float to_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ float to_f32<__hip_bfloat16>(__hip_bfloat16 x) {
  return __bfloat162float(x);
}
template <typename IO> __device__ __forceinline__ IO from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ __hip_bfloat16 from_f32<__hip_bfloat16>(float x) {
  return __float2bfloat16(x);  // round to nearest even
}

// fp32 copies of W[n] and its transpose, so that both contractions of the
// backward read with unit stride.
template <typename IO>
__global__ void w_prep_kernel(const IO *W, float *W32, float *WT32, int N, int V) {
  const size_t total = (size_t)N * V * V;
  for (size_t e = blockIdx.x * (size_t)blockDim.x + threadIdx.x; e < total;
       e += (size_t)gridDim.x * blockDim.x) {
    const int n = e / ((size_t)V * V);
    const int r = e % ((size_t)V * V);
    const int c = r / V, j = r % V;
    const float w = to_f32<IO>(W[e]);
    W32[e] = w;
    WT32[((size_t)n * V + j) * V + c] = w;
  }
}

// Sum over the workgroup in a fixed order; the result is valid in thread 0.
__device__ __forceinline__ float block_sum(float x, float *red) {
  for (int o = 32; o > 0; o >>= 1) x += __shfl_down(x, o, 64);
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) red[w] = x;
  __syncthreads();
  float s = 0.f;
  if (threadIdx.x == 0) {
    const int nw = (blockDim.x + 63) >> 6;
    for (int i = 0; i < nw; ++i) s += red[i];
  }
  __syncthreads();
  return s;
}

// One step of the recurrence for the elements this thread owns.  Hs holds the
// state before the step; the new values are returned in hn[] (and Z in z[] if
// asked) and are NOT yet written back.
template <bool kKeepZ, int PT>
__device__ __forceinline__ void step_elements(const float *Hs, const float *Wf, const float *ks,
                                              const float *vs, float f, int K, int V, int KV,
                                              float *hn, float *z) {
  const int tid = threadIdx.x, nt = blockDim.x;
  constexpr int UN = kUnrollOf<PT>;
#pragma unroll
  for (int m = 0; m < PT; ++m) {
    const int e = tid + m * nt;
    if (e < KV) {
      const int i = e / V, j = e - i * V;
      float s = 0.f;
#pragma unroll UN
      for (int c = 0; c < V; ++c) s = fmaf(Hs[i * V + c], Wf[c * V + j], s);
      s = fmaf(ks[i], vs[j], s);
      const float zz = tanhf(s);
      if (kKeepZ) z[m] = zz;
      hn[m] = fmaf(f, Hs[e], (1.f - f) * zz);
    }
  }
}

// PT: state (and dW) elements per thread, the smallest power of two that covers the shape:
// the per-thread arrays and the unrolled element loops are no longer than they must be.
// WL: W[n] is copied to LDS (it fits next to the state) and read from there; a template
// parameter, so that every access to W has one address space (with a run-time choice the
// contraction reads W through generic-address loads, one wait per load).
template <typename IO, bool WL, int PT>
__global__ void __launch_bounds__(kMaxThreads) gen_fwd_kernel(FwdArgs a, const float *W32) {
  extern __shared__ float smem[];
  constexpr int UN = kUnrollOf<PT>;
  const int K = a.K, V = a.V, KV = K * V, T = a.T, N = a.N;
  const int tid = threadIdx.x, nt = blockDim.x;
  float *Hs = smem;
  float *ks = Hs + KV;
  float *qs = ks + K;
  float *vs = qs + K;
  float *Wl = vs + V;
  const int unit = blockIdx.x, b = unit / N, n = unit - b * N;
  const int g = n / (N / a.Nqk);
  const float *Wg = W32 + (size_t)n * V * V;
  if constexpr (WL)
    for (int e = tid; e < V * V; e += nt) Wl[e] = Wg[e];
  const float *Wf = WL ? Wl : Wg;
  for (int e = tid; e < KV; e += nt) Hs[e] = a.H0 ? a.H0[(size_t)unit * KV + e] : 0.f;
  __syncthreads();
  const int nck = (T + a.C - 1) / a.C;
  const IO *q = (const IO *)a.q, *k = (const IO *)a.k, *v = (const IO *)a.v;
  IO *y = (IO *)a.y;
  float hn[PT];
  for (int t = 0; t < T; ++t) {
    if (a.ckpt && (t % a.C) == 0) {
      float *dst = a.ckpt + ((size_t)unit * nck + t / a.C) * KV;
      for (int e = tid; e < KV; e += nt) dst[e] = Hs[e];
    }
    const size_t qk_off = (((size_t)b * T + t) * a.Nqk + g) * K;
    const size_t v_off = (((size_t)b * T + t) * N + n) * V;
    for (int e = tid; e < K; e += nt) {
      ks[e] = to_f32<IO>(k[qk_off + e]);
      qs[e] = to_f32<IO>(q[qk_off + e]);
    }
    for (int e = tid; e < V; e += nt) vs[e] = to_f32<IO>(v[v_off + e]);
    float f = a.f[((size_t)b * T + t) * N + n];
    if (a.gate_alpha) f = gate_psi(f, a.gate_alpha[n], a.gate_beta[n]);
    __syncthreads();
    step_elements<false, PT>(Hs, Wf, ks, vs, f, K, V, KV, hn, nullptr);
    __syncthreads();
#pragma unroll
    for (int m = 0; m < PT; ++m) {
      const int e = tid + m * nt;
      if (e < KV) Hs[e] = hn[m];
    }
    __syncthreads();
    if (a.write_y) {
      for (int j = tid; j < V; j += nt) {
        float acc = 0.f;
#pragma unroll UN
        for (int i = 0; i < K; ++i) acc = fmaf(Hs[i * V + j], qs[i], acc);
        if (a.w_r) acc = fmaf(to_f32<IO>(((const IO *)a.w_r)[n * V + j]), vs[j], acc);
        y[v_off + j] = from_f32<IO>(acc);
      }
    }
    __syncthreads();
  }
  if (a.HT)
    for (int e = tid; e < KV; e += nt) a.HT[(size_t)unit * KV + e] = Hs[e];
}

// Backward for one (b, n): chunks from last to first; per chunk a forward
// recompute that parks the chunk's states in `states`, then the reverse sweep.
template <typename IO, bool WL, int PT>
__global__ void __launch_bounds__(kMaxThreads)
    gen_bwd_kernel(BwdArgs a, const float *W32, const float *WT32, float *states, float *dW_unit,
                   float *dq_heads, float *dk_heads) {
  extern __shared__ float smem[];
  __shared__ float red[kMaxThreads / 64];
  constexpr int UN = kUnrollOf<PT>;
  const int K = a.K, V = a.V, KV = K * V, VV = V * V, T = a.T, N = a.N, C = a.C;
  const int tid = threadIdx.x, nt = blockDim.x;
  float *Hs = smem;        // state before the step
  float *Xs = Hs + KV;     // state after the step, then dS
  float *ks = Xs + KV;
  float *qs = ks + K;
  float *vs = qs + K;      // V
  float *dys = vs + V;     // V
  float *Wl = dys + V;
  const int unit = blockIdx.x, b = unit / N, n = unit - b * N;
  const int g = n / (N / a.Nqk);
  const float *Wg = W32 + (size_t)n * VV;
  const float *WTg = WT32 + (size_t)n * VV;
  if constexpr (WL)
    for (int e = tid; e < VV; e += nt) {
      Wl[e] = Wg[e];
      Wl[VV + e] = WTg[e];
    }
  const float *Wf = WL ? Wl : Wg;
  const float *WTf = WL ? Wl + VV : WTg;
  const IO *q = (const IO *)a.q, *k = (const IO *)a.k, *v = (const IO *)a.v,
           *dy = (const IO *)a.dy;
  float *st = states + (size_t)unit * (C + 1) * KV;
  const int nck = (T + C - 1) / C;

  float carry[PT];  // dL/dH flowing from later steps, per owned element
  float dWacc[PT];  // this thread's elements of dW (indexed over V*V)
  float hn[PT], z[PT];
#pragma unroll
  for (int m = 0; m < PT; ++m) {
    const int e = tid + m * nt;
    carry[m] = (e < KV && a.dHT) ? a.dHT[(size_t)unit * KV + e] : 0.f;
    dWacc[m] = 0.f;
  }
  __syncthreads();

  for (int ck = nck - 1; ck >= 0; --ck) {
    const int t0 = ck * C;
    const int len = min(C, T - t0);
    // ---- recompute the chunk's states from its checkpoint
    {
      const float *src = a.ckpt + ((size_t)unit * nck + ck) * KV;
      for (int e = tid; e < KV; e += nt) Hs[e] = src[e];
    }
    __syncthreads();
    for (int s = 0; s < len; ++s) {
      const int t = t0 + s;
      for (int e = tid; e < KV; e += nt) st[(size_t)s * KV + e] = Hs[e];
      const size_t qk_off = (((size_t)b * T + t) * a.Nqk + g) * K;
      const size_t v_off = (((size_t)b * T + t) * N + n) * V;
      for (int e = tid; e < K; e += nt) ks[e] = to_f32<IO>(k[qk_off + e]);
      for (int e = tid; e < V; e += nt) vs[e] = to_f32<IO>(v[v_off + e]);
      float f = a.f[((size_t)b * T + t) * N + n];
    if (a.gate_alpha) f = gate_psi(f, a.gate_alpha[n], a.gate_beta[n]);
      __syncthreads();
      step_elements<false, PT>(Hs, Wf, ks, vs, f, K, V, KV, hn, nullptr);
      __syncthreads();
#pragma unroll
      for (int m = 0; m < PT; ++m) {
        const int e = tid + m * nt;
        if (e < KV) Hs[e] = hn[m];
      }
      __syncthreads();
    }
    // ---- reverse sweep over the chunk
    for (int s = len - 1; s >= 0; --s) {
      const int t = t0 + s;
      const size_t qk_off = (((size_t)b * T + t) * a.Nqk + g) * K;
      const size_t v_off = (((size_t)b * T + t) * N + n) * V;
      for (int e = tid; e < KV; e += nt) Hs[e] = st[(size_t)s * KV + e];
      for (int e = tid; e < K; e += nt) {
        ks[e] = to_f32<IO>(k[qk_off + e]);
        qs[e] = to_f32<IO>(q[qk_off + e]);
      }
      for (int e = tid; e < V; e += nt) {
        vs[e] = to_f32<IO>(v[v_off + e]);
        dys[e] = to_f32<IO>(dy[v_off + e]);
      }
      float f = a.f[((size_t)b * T + t) * N + n];
    if (a.gate_alpha) f = gate_psi(f, a.gate_alpha[n], a.gate_beta[n]);
      __syncthreads();
      // recompute Z_t and H_t exactly as the forward did
      step_elements<true, PT>(Hs, Wf, ks, vs, f, K, V, KV, hn, z);
#pragma unroll
      for (int m = 0; m < PT; ++m) {
        const int e = tid + m * nt;
        if (e < KV) Xs[e] = hn[m];
      }
      __syncthreads();
      // dq_t = H_t dy_t
      for (int i = tid; i < K; i += nt) {
        float acc = 0.f;
#pragma unroll UN
        for (int j = 0; j < V; ++j) acc = fmaf(Xs[i * V + j], dys[j], acc);
        if (dq_heads)
          dq_heads[(((size_t)b * T + t) * N + n) * K + i] = acc;
        else
          ((IO *)a.dq)[qk_off + i] = from_f32<IO>(acc);
      }
      __syncthreads();
      // G = q dy^T + carry ; df ; dS = (1-f) G (1 - Z^2)
      float dfp = 0.f;
#pragma unroll
      for (int m = 0; m < PT; ++m) {
        const int e = tid + m * nt;
        if (e < KV) {
          const int i = e / V, j = e - i * V;
          const float G = fmaf(qs[i], dys[j], carry[m]);
          dfp = fmaf(G, Hs[e] - z[m], dfp);
          Xs[e] = (1.f - f) * G * (1.f - z[m] * z[m]);
          carry[m] = G;
        }
      }
      const float dft = block_sum(dfp, red);  // contains the barriers that publish Xs
      if (tid == 0) a.df[((size_t)b * T + t) * N + n] = dft;
      // carry = f G + dS W^T
#pragma unroll
      for (int m = 0; m < PT; ++m) {
        const int e = tid + m * nt;
        if (e < KV) {
          const int i = e / V, c = e - i * V;
          float acc = 0.f;
#pragma unroll UN
          for (int j = 0; j < V; ++j) acc = fmaf(Xs[i * V + j], WTf[j * V + c], acc);
          carry[m] = fmaf(f, carry[m], acc);
          if (a.clip > 0.f) carry[m] = fminf(fmaxf(carry[m], -a.clip), a.clip);
        }
      }
      // dW += H_{t-1}^T dS
#pragma unroll
      for (int m = 0; m < PT; ++m) {
        const int e = tid + m * nt;
        if (e < VV) {
          const int c = e / V, j = e - c * V;
          float acc = 0.f;
#pragma unroll UN
          for (int i = 0; i < K; ++i) acc = fmaf(Hs[i * V + c], Xs[i * V + j], acc);
          dWacc[m] += acc;
        }
      }
      // dk_t = dS v_t ; dv_t = dS^T k_t
      for (int i = tid; i < K; i += nt) {
        float acc = 0.f;
#pragma unroll UN
        for (int j = 0; j < V; ++j) acc = fmaf(Xs[i * V + j], vs[j], acc);
        if (dk_heads)
          dk_heads[(((size_t)b * T + t) * N + n) * K + i] = acc;
        else
          ((IO *)a.dk)[qk_off + i] = from_f32<IO>(acc);
      }
      for (int j = tid; j < V; j += nt) {
        float acc = 0.f;
#pragma unroll UN
        for (int i = 0; i < K; ++i) acc = fmaf(Xs[i * V + j], ks[i], acc);
        if (a.w_r) acc = fmaf(to_f32<IO>(((const IO *)a.w_r)[n * V + j]), dys[j], acc);
        ((IO *)a.dv)[v_off + j] = from_f32<IO>(acc);
      }
      __syncthreads();
    }
  }
#pragma unroll
  for (int m = 0; m < PT; ++m) {
    const int e = tid + m * nt;
    if (e < KV && a.dH0) a.dH0[(size_t)unit * KV + e] = carry[m];
    if (e < VV) dW_unit[(size_t)unit * VV + e] = dWacc[m];
  }
}

// dW[n] = sum over b of the per-recurrence dW, in increasing b.
__global__ void dw_batch_sum_kernel(const float *dW_unit, float *dW, int B, int N, int VV) {
  const size_t total = (size_t)N * VV;
  for (size_t e = blockIdx.x * (size_t)blockDim.x + threadIdx.x; e < total;
       e += (size_t)gridDim.x * blockDim.x) {
    float s = 0.f;
    for (int b = 0; b < B; ++b) s += dW_unit[(size_t)b * total + e];
    dW[e] = s;
  }
}

// Gradient of the residual weight: dw_r[n][j] = sum over (b, t) of dy (.) v.  Stage 1: block s
// adds the rows r = s, s + S, s + 2S, ... of the [B*T, N*V] tensors in increasing r; stage 2
// adds the S partial rows in increasing s.  The order is fixed, so the result is reproducible.
constexpr int kDwrStages = 1024;
template <typename IO>
__global__ void dwr_stage1_kernel(const IO *__restrict__ dy, const IO *__restrict__ v,
                                  float *__restrict__ part, size_t BT, int NV) {
  for (int c = threadIdx.x; c < NV; c += blockDim.x) {
    float acc = 0.f;
    for (size_t r = blockIdx.x; r < BT; r += gridDim.x)
      acc = fmaf(to_f32<IO>(dy[r * NV + c]), to_f32<IO>(v[r * NV + c]), acc);
    part[(size_t)blockIdx.x * NV + c] = acc;
  }
}
__global__ void dwr_stage2_kernel(const float *__restrict__ part, float *__restrict__ dw_r, int S,
                                  int NV) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= NV) return;
  float s = 0.f;
  for (int p = 0; p < S; ++p) s += part[(size_t)p * NV + c];
  dw_r[c] = s;
}

// dq/dk of a shared q/k head = sum over its heads, in increasing head index.
template <typename IO>
__global__ void head_group_sum_kernel(const float *per_head, IO *out, size_t BT, int N, int Nqk,
                                      int K) {
  const int per = N / Nqk;
  const size_t total = BT * Nqk * K;
  for (size_t e = blockIdx.x * (size_t)blockDim.x + threadIdx.x; e < total;
       e += (size_t)gridDim.x * blockDim.x) {
    const int i = e % K;
    const size_t r = e / K;
    const int g = r % Nqk;
    const size_t bt = r / Nqk;
    float s = 0.f;
    for (int h = 0; h < per; ++h) s += per_head[((bt * N) + g * per + h) * K + i];
    out[e] = from_f32<IO>(s);
  }
}

struct GenericPlan {
  int threads, per_thread;
  size_t lds_fwd, lds_bwd;
  int w_lds_fwd, w_lds_bwd;
};

GenericPlan make_plan(int K, int V) {
  GenericPlan p;
  const int KV = K * V, VV = V * V;
  p.threads = KV < kMaxThreads ? KV : kMaxThreads;
  // every thread must be able to own its share of dW (V*V elements) as well
  while (p.threads < kMaxThreads && VV > p.threads * kMaxPerThread) p.threads *= 2;
  const int big = KV > VV ? KV : VV;
  p.per_thread = 1;
  while (p.per_thread * p.threads < big) p.per_thread *= 2;
  const size_t base_f = (size_t)(KV + 2 * K + V) * 4;
  p.w_lds_fwd = base_f + (size_t)VV * 4 <= kLdsBudget;
  p.lds_fwd = base_f + (p.w_lds_fwd ? (size_t)VV * 4 : 0);
  const size_t base_b = (size_t)(2 * KV + 2 * K + 2 * V) * 4;
  p.w_lds_bwd = base_b + (size_t)2 * VV * 4 <= kLdsBudget;
  p.lds_bwd = base_b + (p.w_lds_bwd ? (size_t)2 * VV * 4 : 0);
  return p;
}

// Workspace carve-up (byte offsets).  The forward uses only the two W copies.
struct GenericWs {
  size_t w32, wt32, states, dw_unit, dq_heads, dk_heads, total;
};

GenericWs layout_ws(int B, int T, int N, int Nqk, int K, int V, int C, int bwd) {
  GenericWs w;
  size_t off = 0;
  const size_t wbytes = align256((size_t)N * V * V * 4);
  w.w32 = off; off += wbytes;
  w.wt32 = off; off += wbytes;
  w.states = off; off += bwd ? align256((size_t)B * N * (C + 1) * K * V * 4) : 0;
  w.dw_unit = off; off += bwd ? align256((size_t)B * N * V * V * 4) : 0;
  const size_t heads = (bwd && Nqk != N) ? align256((size_t)B * T * N * K * 4) : 0;
  w.dq_heads = off; off += heads;
  w.dk_heads = off; off += heads;
  w.total = off;
  return w;
}

inline int grid_for(size_t total, int threads) {
  size_t g = (total + threads - 1) / threads;
  if (g < 1) g = 1;
  if (g > 4096) g = 4096;
  return (int)g;
}

template <typename IO>
hipError_t run_fwd(const FwdArgs &a, hipStream_t s) {
  const int units = a.B * a.N;
  if (units == 0) return hipSuccess;
  const GenericPlan p = make_plan(a.K, a.V);
  const GenericWs w = layout_ws(a.B, a.T, a.N, a.Nqk, a.K, a.V, a.C, 0);
  float *W32 = (float *)(a.ws + w.w32);
  float *WT32 = (float *)(a.ws + w.wt32);
  hipLaunchKernelGGL(w_prep_kernel<IO>, dim3(grid_for((size_t)a.N * a.V * a.V, 256)), dim3(256), 0,
                     s, (const IO *)a.W, W32, WT32, a.N, a.V);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  auto go = [&](auto kernel) {
    hipError_t e2 = set_max_lds_once(kernel, (int)kLdsBudget);  // (the need varies with the shape)
    if (e2 != hipSuccess) return e2;
    hipLaunchKernelGGL(kernel, dim3(units), dim3(p.threads), p.lds_fwd, s, a, (const float *)W32);
    return hipGetLastError();
  };
#define M2RNN_GEN_FWD(PT_) \
  if (p.per_thread == PT_)  \
    return p.w_lds_fwd ? go(gen_fwd_kernel<IO, true, PT_>) : go(gen_fwd_kernel<IO, false, PT_>);
  M2RNN_GEN_FWD(1) M2RNN_GEN_FWD(2) M2RNN_GEN_FWD(4) M2RNN_GEN_FWD(8) M2RNN_GEN_FWD(16)
#undef M2RNN_GEN_FWD
  return hipErrorInvalidValue;
}

template <typename IO>
hipError_t run_bwd(const BwdArgs &a, hipStream_t s) {
  const int units = a.B * a.N;
  const GenericPlan p = make_plan(a.K, a.V);
  const GenericWs w = layout_ws(a.B, a.T, a.N, a.Nqk, a.K, a.V, a.C, 1);
  float *W32 = (float *)(a.ws + w.w32);
  float *WT32 = (float *)(a.ws + w.wt32);
  float *states = (float *)(a.ws + w.states);
  float *dW_unit = (float *)(a.ws + w.dw_unit);
  const bool shared = a.Nqk != a.N;
  float *dq_heads = shared ? (float *)(a.ws + w.dq_heads) : nullptr;
  float *dk_heads = shared ? (float *)(a.ws + w.dk_heads) : nullptr;
  hipError_t e;
  if (units > 0) {
    hipLaunchKernelGGL(w_prep_kernel<IO>, dim3(grid_for((size_t)a.N * a.V * a.V, 256)), dim3(256),
                       0, s, (const IO *)a.W, W32, WT32, a.N, a.V);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    auto go = [&](auto kernel) {
      hipError_t e2 = set_max_lds_once(kernel, (int)kLdsBudget);
      if (e2 != hipSuccess) return e2;
      hipLaunchKernelGGL(kernel, dim3(units), dim3(p.threads), p.lds_bwd, s, a, (const float *)W32,
                         (const float *)WT32, states, dW_unit, dq_heads, dk_heads);
      return hipGetLastError();
    };
    e = hipErrorInvalidValue;
#define M2RNN_GEN_BWD(PT_) \
  if (p.per_thread == PT_)  \
    e = p.w_lds_bwd ? go(gen_bwd_kernel<IO, true, PT_>) : go(gen_bwd_kernel<IO, false, PT_>);
    M2RNN_GEN_BWD(1) M2RNN_GEN_BWD(2) M2RNN_GEN_BWD(4) M2RNN_GEN_BWD(8) M2RNN_GEN_BWD(16)
#undef M2RNN_GEN_BWD
    if (e != hipSuccess) return e;
    if (shared && a.T > 0) {
      const size_t total = (size_t)a.B * a.T * a.Nqk * a.K;
      hipLaunchKernelGGL(head_group_sum_kernel<IO>, dim3(grid_for(total, 256)), dim3(256), 0, s,
                         (const float *)dq_heads, (IO *)a.dq, (size_t)a.B * a.T, a.N, a.Nqk, a.K);
      hipLaunchKernelGGL(head_group_sum_kernel<IO>, dim3(grid_for(total, 256)), dim3(256), 0, s,
                         (const float *)dk_heads, (IO *)a.dk, (size_t)a.B * a.T, a.N, a.Nqk, a.K);
      if ((e = hipGetLastError()) != hipSuccess) return e;
    }
  }
  // B == 0 leaves dW = 0: the sum below runs over zero terms.
  hipLaunchKernelGGL(dw_batch_sum_kernel, dim3(grid_for((size_t)a.N * a.V * a.V, 256)), dim3(256),
                     0, s, (const float *)dW_unit, a.dW, a.B, a.N, a.V * a.V);
  return hipGetLastError();
}

}  // namespace

int generic_default_chunk(int, int) { return 16; }
int generic_max_chunk(int, int) { return 256; }

size_t generic_workspace_bytes(int B, int T, int N, int Nqk, int K, int V, int C, int bwd) {
  return layout_ws(B, T, N, Nqk, K, V, C, bwd).total;
}

hipError_t generic_fwd(const FwdArgs &a, hipStream_t s) {
  return a.io == 0 ? run_fwd<float>(a, s) : run_fwd<__hip_bfloat16>(a, s);
}

hipError_t generic_bwd(const BwdArgs &a, hipStream_t s) {
  return a.io == 0 ? run_bwd<float>(a, s) : run_bwd<__hip_bfloat16>(a, s);
}

// Chain rule through the gate function.  df holds dL/d(gate value) g; with u = x + beta,
// psi = exp(-alpha softplus(u)):  dL/dx = dL/dbeta-term = -g alpha psi sigmoid(u),
// dL/dalpha-term = -g psi softplus(u).  Stage 1: block s handles the (b, t) rows s, s + S, ...
// in increasing order, thread n one head; stage 2 adds the S partial rows in increasing s.
constexpr int kGateStages = 256;
__global__ void gate_bwd_stage1_kernel(float *__restrict__ df, const float *__restrict__ x,
                                       const float *__restrict__ alpha,
                                       const float *__restrict__ beta, float *__restrict__ part,
                                       size_t BT, int N) {
  for (int n = threadIdx.x; n < N; n += blockDim.x) {
    const float al = alpha[n], be = beta[n];
    float sa = 0.f, sb = 0.f;
    for (size_t r = blockIdx.x; r < BT; r += gridDim.x) {
      const float u = x[r * N + n] + be;
      const float sp = fmaxf(u, 0.f) + log1pf(expf(-fabsf(u)));
      const float psi = expf(-al * sp);
      const float g = df[r * N + n];
      const float dx = -g * al * psi / (1.f + expf(-u));
      sa = fmaf(-g * psi, sp, sa);
      sb += dx;
      df[r * N + n] = dx;
    }
    part[((size_t)blockIdx.x * 2 + 0) * N + n] = sa;
    part[((size_t)blockIdx.x * 2 + 1) * N + n] = sb;
  }
}
__global__ void gate_bwd_stage2_kernel(const float *__restrict__ part, float *__restrict__ dalpha,
                                       float *__restrict__ dbeta, int S, int N) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= N) return;
  float sa = 0.f, sb = 0.f;
  for (int p = 0; p < S; ++p) {
    sa += part[((size_t)p * 2 + 0) * N + n];
    sb += part[((size_t)p * 2 + 1) * N + n];
  }
  dalpha[n] = sa;
  dbeta[n] = sb;
}

size_t gate_scratch_bytes(int N) { return align256((size_t)kGateStages * 2 * N * sizeof(float)); }

hipError_t gate_backward(const BwdArgs &a, hipStream_t s) {
  const size_t BT = (size_t)a.B * a.T;
  const int S = BT < (size_t)kGateStages ? (int)BT : kGateStages;
  if (S > 0)
    hipLaunchKernelGGL(gate_bwd_stage1_kernel, dim3(S), dim3(a.N < 64 ? 64 : 128), 0, s, a.df,
                       a.f, a.gate_alpha, a.gate_beta, a.gate_ws, BT, a.N);
  hipLaunchKernelGGL(gate_bwd_stage2_kernel, dim3((a.N + 63) / 64), dim3(64), 0, s,
                     (const float *)a.gate_ws, a.dgate_alpha, a.dgate_beta, S, a.N);
  return hipGetLastError();
}

size_t residual_dw_r_scratch_bytes(int N, int V) {
  return align256((size_t)kDwrStages * N * V * sizeof(float));
}

hipError_t residual_dw_r(const BwdArgs &a, hipStream_t s) {
  const int NV = a.N * a.V;
  const size_t BT = (size_t)a.B * a.T;
  const int S = BT < (size_t)kDwrStages ? (int)BT : kDwrStages;
  if (S > 0) {
    if (a.io == 0)
      hipLaunchKernelGGL(dwr_stage1_kernel<float>, dim3(S), dim3(256), 0, s, (const float *)a.dy,
                         (const float *)a.v, a.dwr_ws, BT, NV);
    else
      hipLaunchKernelGGL(dwr_stage1_kernel<__hip_bfloat16>, dim3(S), dim3(256), 0, s,
                         (const __hip_bfloat16 *)a.dy, (const __hip_bfloat16 *)a.v, a.dwr_ws, BT,
                         NV);
  }
  hipLaunchKernelGGL(dwr_stage2_kernel, dim3((NV + 255) / 256), dim3(256), 0, s,
                     (const float *)a.dwr_ws, a.dw_r, S, NV);
  return hipGetLastError();
}

}  // namespace m2rnn

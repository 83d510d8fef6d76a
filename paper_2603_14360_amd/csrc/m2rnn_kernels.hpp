// Internal declarations shared by the HIP translation units of libm2rnn.
// Not part of the public ABI (that is include/m2rnn.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

namespace m2rnn {

// Arguments of one forward scan.  Shapes and meaning follow the public header;
// pointers are device pointers.
struct FwdArgs {
  int B, T, N, Nqk, K, V, C, io;
  const void *q, *k, *v, *W;
  const float *f, *H0;
  void *y;
  float *HT, *ckpt;  // ckpt may be null (inference)
  int write_y;       // 0: checkpoint-only pass (the backward's pass 1)
  char *ws;          // workspace base (may be null when nothing is needed)
  const void *w_r;   // [N,V] io dtype: y_t += w_r (.) v_t; null = no residual
  const float *gate_alpha, *gate_beta;  // [N] each: f holds the input of the gate function; null = f is the gate value
};

struct BwdArgs {
  int B, T, N, Nqk, K, V, C, io;
  const void *q, *k, *v, *W, *dy;
  const float *f, *H0, *ckpt, *dHT;
  void *dq, *dk, *dv;
  float *df, *dW, *dH0;
  char *ws;
  const void *w_r;   // residual weight (dv_t += w_r (.) dy_t); null = none
  float *dw_r;       // [N,V] fp32 out, with w_r
  float *dwr_ws;     // scratch of residual_dw_r_scratch_bytes() for dw_r
  float clip;        // > 0: clamp of the carried state gradient; <= 0: off
  const float *gate_alpha, *gate_beta;  // as in FwdArgs; then df is finished by gate_backward()
  float *dgate_alpha, *dgate_beta;      // [N] fp32 out
  float *gate_ws;                       // scratch of gate_scratch_bytes()
};

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Raises a kernel's dynamic-LDS limit the first time the kernel is launched on a device,
// not on every call (the entry points are otherwise launch-only, and a decode loop pays host
// latency for every extra runtime call).  Kernels are told apart by their address (the
// instantiations of a kernel template share one function type, so a flag per type would
// be set by the first of them for all): a small open-addressing table of (kernel, devices
// done), lock-free; when it is full the attribute is simply set on every call.  `bytes`
// must not depend on the call.
inline hipError_t set_max_lds_once_addr(const void *kernel, int bytes) {
  struct Slot {
    std::atomic<const void *> fn{nullptr};
    std::atomic<uint64_t> done{0};
  };
  constexpr unsigned kSlots = 512;
  static Slot slots[kSlots];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = 1ull << (dev & 63);
  unsigned h = (unsigned)((reinterpret_cast<uintptr_t>(kernel) >> 4) % kSlots);
  for (unsigned probe = 0; probe < kSlots; ++probe, h = (h + 1) % kSlots) {
    const void *cur = slots[h].fn.load(std::memory_order_acquire);
    if (cur == nullptr) {
      const void *expected = nullptr;
      cur = slots[h].fn.compare_exchange_strong(expected, kernel, std::memory_order_acq_rel)
                ? kernel
                : expected;
    }
    if (cur != kernel) continue;
    if (slots[h].done.load(std::memory_order_acquire) & bit) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) slots[h].done.fetch_or(bit, std::memory_order_release);
    return e;
  }
  return hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}
template <typename Fn>
inline hipError_t set_max_lds_once(Fn kernel, int bytes) {
  return set_max_lds_once_addr((const void *)kernel, bytes);
}
inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// ---- fp32 path (plain vector-ALU kernels; any supported shape, either io) ----
int generic_default_chunk(int K, int V);
int generic_max_chunk(int K, int V);
size_t generic_workspace_bytes(int B, int T, int N, int Nqk, int K, int V, int C, int bwd);
hipError_t generic_fwd(const FwdArgs &a, hipStream_t s);
hipError_t generic_bwd(const BwdArgs &a, hipStream_t s);

// dw_r[n][j] = sum over b, t of dy (.) v in a fixed order (two stages through `scratch`)
size_t residual_dw_r_scratch_bytes(int N, int V);
hipError_t residual_dw_r(const BwdArgs &a, hipStream_t s);

// Forget-gate function of the paper's "Forget Gate" section, psi(x) = (1 + e^(x + beta))^(-alpha),
// evaluated where a kernel stages f (one lane per step): exp(-alpha softplus(x + beta)).
__device__ __forceinline__ float gate_psi(float x, float alpha, float beta) {
  const float u = x + beta;
  const float sp = fmaxf(u, 0.f) + log1pf(expf(-fabsf(u)));
  return expf(-alpha * sp);
}
// Chain rule through psi after a backward scan: df (in: dL/d gate value) -> dL/dx in place,
// dalpha, dbeta summed over b, t in a fixed order (two stages through `gate_ws`).
size_t gate_scratch_bytes(int N);
hipError_t gate_backward(const BwdArgs &a, hipStream_t s);

// ---- matrix-core path (bf16 io, fp16 MFMA operands, fp32 state) ----
// register-resident backward for V = 16 (one wave per 16-row block)
bool rowwave_bwd_supported(int K, int V);
hipError_t rowwave_bwd(const BwdArgs &a, hipStream_t s);
size_t rowwave_bwd_workspace_bytes(int B, int T, int N, int Nqk, int K, int V);
int rowwave_bwd_max_chunk();
bool mfma_supported(int K, int V);
int mfma_default_chunk(int K, int V);
int mfma_max_chunk(int K, int V);
size_t mfma_workspace_bytes(int B, int T, int N, int Nqk, int K, int V, int C, int bwd);
hipError_t mfma_fwd(const FwdArgs &a, hipStream_t s);
hipError_t mfma_bwd(const BwdArgs &a, hipStream_t s);
int mfma_pick_rb(int K, int V, int units);  // row blocks per workgroup of the tile serving a launch (0: none)

// ---- register-resident path (bf16 io, V <= 64): one wave per 16 state rows ----
bool rowwave_supported(int K, int V);
hipError_t rowwave_fwd(const FwdArgs &a, hipStream_t s);

// ---- the scan's neighbours in the block: conv1d(4) + SiLU prologue, gated RMSNorm epilogue ----
size_t conv_silu_scratch_bytes(int B, int T, int C);
hipError_t conv_silu_fwd(int B, int T, int C, int io, const void *x, const void *w, const void *bias,
                         void *out, hipStream_t s);
hipError_t conv_silu_bwd(int B, int T, int C, int io, const void *x, const void *w, const void *bias,
                         const void *dout, void *dx, float *dw, float *dbias, float *part,
                         hipStream_t s);
size_t gated_rmsnorm_scratch_bytes(int B, int T, int D);
int gated_rmsnorm_max_features();
hipError_t gated_rmsnorm_fwd(int B, int T, int D, int io, const void *y, const void *a, const void *w,
                             float eps, void *out, float *s_out, hipStream_t s);
hipError_t gated_rmsnorm_bwd(int B, int T, int D, int io, const void *y, const void *a, const void *w,
                             float eps, const float *s_in, const void *dout, void *dy, void *da,
                             float *dw, float *part, hipStream_t s);

// ---- single-step decode (bf16 io, V <= 64, T == 1): one launch, no staging, no workspace ----
bool decode_supported(int K, int V);
hipError_t decode_fwd(const FwdArgs &a, hipStream_t s);

}  // namespace m2rnn

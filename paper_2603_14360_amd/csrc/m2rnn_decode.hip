// Single-step decode (the recurrent inference form of the layer: the state update equations
// applied to one token, Algorithm 1 with T = 1) for a batch of states, bf16 io, V <= 64.
//
// One launch, one workgroup per (b, n) state, one wavefront per 16 rows of it.  The state goes
// HBM -> registers -> HBM exactly once (fp32, 16 bytes per lane and column tile, coalesced);
// q, k, v, f are read straight from global memory into the registers that use them (no
// 16-step staging through LDS, no barrier in front of the arithmetic), the readout
// y = H_1^T q is finished inside the kernel (row-block partials through LDS, one barrier),
// and nothing needs a workspace.  The arithmetic is the register-resident forward's: the
// problem is run transposed, S^T = W^T H^T, with the state as an fp16 (hi, lo) pair in
// adjacent k-slots of the 16x16x32 MFMA against a W fragment that repeats each row of W.
#include "m2rnn_kernels.hpp"
#include "m2rnn_mfma_common.hpp"

namespace m2rnn {
namespace {

template <int K_, int V_>
struct Decode {
  static constexpr int K = K_, V = V_;
  static constexpr int CT = V / 16;   // 16-column tiles per wave
  static constexpr int NW = K / 16;   // waves (row blocks) per workgroup = per state
  static constexpr int THREADS = NW * 64;
};

template <typename DC>
__global__ void __launch_bounds__(DC::THREADS, 2) decode_kernel(FwdArgs a) {
  constexpr int K = DC::K, V = DC::V, CT = DC::CT, NW = DC::NW;
  const int unit = blockIdx.x;
  const int N = a.N;
  const int b = unit / N, n = unit - b * N;
  const int g = n / (N / a.Nqk);
  const int lane = threadIdx.x & 63;
  const int rb = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int jl = lane & 15, ig = lane >> 4;
  const int row = rb * 16 + jl;  // state row of this lane

  __shared__ __attribute__((aligned(16))) float ypart[NW][V];

  const bf16_raw *__restrict__ qg = (const bf16_raw *)a.q + ((size_t)b * a.Nqk + g) * K;
  const bf16_raw *__restrict__ kg = (const bf16_raw *)a.k + ((size_t)b * a.Nqk + g) * K;
  const bf16_raw *__restrict__ vg = (const bf16_raw *)a.v + ((size_t)b * N + n) * V;
  const bf16_raw *__restrict__ Wn = (const bf16_raw *)a.W + (size_t)n * V * V;

  // ---- every global load first; what depends on them follows
  const size_t st_off = (size_t)unit * K * V + (size_t)row * V + 4 * ig;
  f4_t h0[CT];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct)
    h0[ct] = a.H0 ? *(const f4_t *)&a.H0[st_off + 16 * ct] : f4_t{0.f, 0.f, 0.f, 0.f};
  float fg = a.f[(size_t)b * N + n];
  const bf16_raw kraw = kg[row];
  const uint2 qraw = *(const uint2 *)&qg[rb * 16 + 4 * ig];   // q rows 4 ig .. 4 ig + 3 of my block
  uint2 vraw[CT];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) vraw[ct] = *(const uint2 *)&vg[16 * ct + 4 * ig];
  // W fragments (A operand of S^T = W^T H^T): slots 2e, 2e+1 of the MFMA for (jt, ct) hold
  // W[16 ct + 4 ig + e][16 jt + jl]; they meet the (hi, lo) pair of that state element
  h8_t wf[CT][CT];
#pragma unroll
  for (int jt = 0; jt < CT; ++jt)
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const _Float16 w = (_Float16)bf16_to_f32(Wn[(size_t)(16 * ct + 4 * ig + e) * V + 16 * jt + jl]);
        wf[jt][ct][2 * e] = w;
        wf[jt][ct][2 * e + 1] = w;
      }

  if (a.ckpt) {  // checkpoint 0 = the state before the step (a later m2rnn_bwd starts from it)
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) *(f4_t *)&a.ckpt[st_off + 16 * ct] = h0[ct];
  }
  if (a.gate_alpha) fg = gate_psi(fg, a.gate_alpha[n], a.gate_beta[n]);
  const float gp = kC * (1.f - fg);
  const float ki = kC * bf16_to_f32(kraw);

  // ---- contraction c (H0 W)^T with the (hi, lo) pair of the scaled state
  float h[CT][4];
  f4_t acc[CT];
#pragma unroll
  for (int jt = 0; jt < CT; ++jt) acc[jt] = f4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
    u4_t pk;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      h[ct][r] = kC * h0[ct][r];
      pk[r] = split_hi_lo(h[ct][r]);
    }
    const h8_t hf = __builtin_bit_cast(h8_t, pk);
#pragma unroll
    for (int jt = 0; jt < CT; ++jt) acc[jt] = mfma_k32(wf[jt][ct], hf, acc[jt]);
  }

  // ---- tanh, gate, readout
  // identity fragment of the transposing MFMA: both slots of column 4 ig + e when that is n
  h8_t ident;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const _Float16 one = (4 * ig + e == jl) ? (_Float16)1.0f : (_Float16)0.0f;
    ident[2 * e] = one;
    ident[2 * e + 1] = one;
  }
  h4_t qfr;
  qfr[0] = (_Float16)bf16_to_f32((bf16_raw)(qraw.x & 0xFFFFu));
  qfr[1] = (_Float16)bf16_to_f32((bf16_raw)(qraw.x >> 16));
  qfr[2] = (_Float16)bf16_to_f32((bf16_raw)(qraw.y & 0xFFFFu));
  qfr[3] = (_Float16)bf16_to_f32((bf16_raw)(qraw.y >> 16));
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
    const float v4[4] = {bf16_to_f32((bf16_raw)(vraw[ct].x & 0xFFFFu)), bf16_to_f32((bf16_raw)(vraw[ct].x >> 16)),
                         bf16_to_f32((bf16_raw)(vraw[ct].y & 0xFFFFu)), bf16_to_f32((bf16_raw)(vraw[ct].y >> 16))};
    u4_t pk;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float sp = fmaf(ki, v4[r], acc[ct][r]);
      h[ct][r] = gate_tanh_step(fg, gp, h[ct][r], sp);
      pk[r] = split_hi_lo(h[ct][r]);
    }
    if (a.HT) {
      f4_t x;
#pragma unroll
      for (int r = 0; r < 4; ++r) x[r] = h[ct][r] * kInvC;
      *(f4_t *)&a.HT[st_off + 16 * ct] = x;
    }
    if (a.write_y) {
      // transpose on the matrix core (D[m = i][n = j] = hi + lo of H'[i][j]), then
      // D[m = j][*] = c sum_i q_i H[i][j] over the 16 rows of this block
      typedef float f2_t __attribute__((ext_vector_type(2)));
      const f4_t tr = mfma_k32(__builtin_bit_cast(h8_t, pk), ident, f4_t{0.f, 0.f, 0.f, 0.f});
      const f2_t a01 = {tr[0], tr[1]}, a23 = {tr[2], tr[3]};
      uint2 tp;
      tp.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(a01, h2_t));
      tp.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(a23, h2_t));
      const f4_t yv = mfma_k16(__builtin_bit_cast(h4_t, tp), qfr, f4_t{0.f, 0.f, 0.f, 0.f});
      if (jl == 0) *(f4_t *)&ypart[rb][16 * ct + 4 * ig] = yv;
    }
  }
  if (!a.write_y) return;
  __syncthreads();
  // ---- y = sum of the row-block partials (increasing block order) [+ w_r (.) v]
  if (threadIdx.x < V) {
    const int j = threadIdx.x;
    float ys = ypart[0][j];
#pragma unroll
    for (int w = 1; w < NW; ++w) ys += ypart[w][j];
    ys *= kInvC;
    if (a.w_r) ys = fmaf(bf16_to_f32(((const bf16_raw *)a.w_r)[n * V + j]), bf16_to_f32(vg[j]), ys);
    ((bf16_raw *)a.y)[((size_t)b * N + n) * V + j] = f32_to_bf16(ys);
  }
}

template <typename DC>
hipError_t launch(const FwdArgs &a, hipStream_t s) {
  const int units = a.B * a.N;
  if (units == 0) return hipSuccess;
  hipLaunchKernelGGL((decode_kernel<DC>), dim3(units), dim3(DC::THREADS), 0, s, a);
  return hipGetLastError();
}

}  // namespace

// (K, V) shapes of the decode kernel: those of the one-wave-per-row-block forward
#define M2RNN_DECODE_CASES(X) M2RNN_ROWWAVE_CASES(X)

bool decode_supported(int K, int V) {
#define X(K_, V_) \
  if (K == K_ && V == V_) return true;
  M2RNN_DECODE_CASES(X)
#undef X
  return false;
}

hipError_t decode_fwd(const FwdArgs &a, hipStream_t s) {
#define X(K_, V_) \
  if (a.K == K_ && a.V == V_) return launch<Decode<K_, V_>>(a, s);
  M2RNN_DECODE_CASES(X)
#undef X
  return hipErrorInvalidValue;
}

}  // namespace m2rnn

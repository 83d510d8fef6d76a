// Matrix-core forward scan (Algorithm 1 of the paper; recurrence equations).
//
// Per workgroup: RB row blocks (16 rows each) of one (b, n) state, all V
// columns, for all T steps.  Per step and wavefront (one 16 x 16 tile):
//   1. read the fp16 copy of the row block's previous state from LDS as the
//      MFMA A operand (all V columns: the tiles of the other waves included);
//   2. S' = c (H W)   on the matrix cores, W fragments resident in registers;
//   3. in registers, fp32:  s' = S' + (c k_i) v_j ; e = 2^{s'} ; r = 1/(1+e) ;
//      H' <- f H' + c(1-f) - 2c(1-f) r        ( = c [f H + (1-f) tanh(s)] )
//   4. write cvt_f16(H') back to LDS for the next step (double buffered, one
//      barrier per step);
//   5. readout: one 16x16x16 MFMA with A = the tile just converted (k = rows)
//      and B = q broadcast gives c * sum_i q_i H[i][j] for the tile's columns;
//      row blocks are summed through LDS, parts through the epilogue kernel.
// q, k, v, f for 16 steps at a time are staged through LDS; the next block's
// global loads are in flight while the current block is computed.
#include "m2rnn_kernels.hpp"
#include "m2rnn_mfma_common.hpp"

namespace m2rnn {
namespace {

constexpr int TB = 16;  // steps per staging block

template <typename TL>
struct FwdSmem {
  alignas(16) _Float16 Hx[2][TL::ROWS][TL::LDH];  // fp16 state exchange, row-major, padded rows
  alignas(16) float kS[2][TB][TL::ROWS];          // c * k
  alignas(16) _Float16 qS[2][TB][TL::ROWS];
  alignas(16) float vS[2][TB][TL::V];
  alignas(16) float fS[2][TB][4];                 // f, c(1-f), -2c(1-f), unused
  alignas(16) float yP[2][TL::RB][TL::V];         // per-row-block readout partials
};

template <typename TL>
__global__ void __launch_bounds__(TL::THREADS)
    mfma_fwd_kernel(FwdArgs a, float *__restrict__ ypart_ws) {
  constexpr int K = TL::K, V = TL::V, RB = TL::RB, CT = TL::CT, ROWS = TL::ROWS, KS = TL::KS;
  constexpr int THREADS = TL::THREADS;
  constexpr bool X32 = TL::X32;
  constexpr int FE = X32 ? 8 : 4;  // halfs per operand fragment
  using FragT = typename Frag<X32>::type;
  constexpr int NQ = (TB * ROWS + THREADS - 1) / THREADS;
  constexpr int NV = (TB * V + THREADS - 1) / THREADS;

  int unit, part;
  if (!map_block<TL::P>(a.B * a.N, unit, part)) return;
  const int T = a.T, N = a.N;
  const int b = unit / N, n = unit - b * N;
  const int g = n / (N / a.Nqk);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rb = wave / CT, ct = wave - rb * CT;
  const int jl = lane & 15, ig = lane >> 4;
  const int col0 = ct * 16, rowb = rb * 16;
  const int row_base = part * ROWS;

  __shared__ FwdSmem<TL> sm;

  const bf16_raw *__restrict__ qg = (const bf16_raw *)a.q;
  const bf16_raw *__restrict__ kg = (const bf16_raw *)a.k;
  const bf16_raw *__restrict__ vg = (const bf16_raw *)a.v;
  const float *__restrict__ fg = a.f;

  // ---- W fragments: B operand, B[k = c][n = j] = W[c][col0 + j]
  FragT wf[KS];
  {
    const bf16_raw *Wn = (const bf16_raw *)a.W + (size_t)n * V * V;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int e = 0; e < FE; ++e) {
        const int c = FE * ig + e + 32 * ks;
        wf[ks][e] = (_Float16)bf16_to_f32(Wn[(size_t)c * V + col0 + jl]);
      }
  }

  // ---- state tile, scaled by c
  const size_t st_off = (size_t)unit * K * V + (size_t)(row_base + rowb + 4 * ig) * V + col0 + jl;
  float h[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) h[r] = a.H0 ? kC * a.H0[st_off + (size_t)r * V] : 0.f;
  if (T == 0) {
    if (a.HT)
#pragma unroll
      for (int r = 0; r < 4; ++r) a.HT[st_off + (size_t)r * V] = a.H0 ? a.H0[st_off + (size_t)r * V] : 0.f;
    return;
  }
#pragma unroll
  for (int r = 0; r < 4; ++r) sm.Hx[0][rowb + 4 * ig + r][col0 + jl] = (_Float16)h[r];

  // ---- staging of q, k, v, f (TB steps per block)
  bf16_raw rq[NQ], rk[NQ], rv[NV];
  float rf = 1.f;
  auto stage_load = [&](int t0) {
#pragma unroll
    for (int m = 0; m < NQ; ++m) {
      const int idx = tid + m * THREADS;
      const int s = idx / ROWS, i = idx - s * ROWS;
      const bool ok = idx < TB * ROWS && t0 + s < T;
      const size_t off = (((size_t)b * T + (t0 + s)) * a.Nqk + g) * K + row_base + i;
      rq[m] = ok ? qg[off] : (bf16_raw)0;
      rk[m] = ok ? kg[off] : (bf16_raw)0;
    }
#pragma unroll
    for (int m = 0; m < NV; ++m) {
      const int idx = tid + m * THREADS;
      const int s = idx / V, j = idx - s * V;
      const bool ok = idx < TB * V && t0 + s < T;
      const size_t off = (((size_t)b * T + (t0 + s)) * N + n) * V + j;
      rv[m] = ok ? vg[off] : (bf16_raw)0;
    }
    rf = (tid < TB && t0 + tid < T) ? fg[((size_t)b * T + (t0 + tid)) * N + n] : 1.f;
  };
  auto stage_store = [&](int buf) {
#pragma unroll
    for (int m = 0; m < NQ; ++m) {
      const int idx = tid + m * THREADS;
      if (idx < TB * ROWS) {
        const int s = idx / ROWS, i = idx - s * ROWS;
        sm.kS[buf][s][i] = kC * bf16_to_f32(rk[m]);
        sm.qS[buf][s][i] = (_Float16)bf16_to_f32(rq[m]);
      }
    }
#pragma unroll
    for (int m = 0; m < NV; ++m) {
      const int idx = tid + m * THREADS;
      if (idx < TB * V) {
        const int s = idx / V, j = idx - s * V;
        sm.vS[buf][s][j] = bf16_to_f32(rv[m]);
      }
    }
    if (tid < TB) {
      const float gp = kC * (1.f - rf);
      sm.fS[buf][tid][0] = rf;
      sm.fS[buf][tid][1] = gp;
      sm.fS[buf][tid][2] = -2.f * gp;
    }
  };

  stage_load(0);
  stage_store(0);
  __syncthreads();

  const int nblk = (T + TB - 1) / TB;
  const int nck = (T + a.C - 1) / a.C;
  int cur = 0;
  int next_ck = 0, ck_idx = 0;
  bf16_raw *__restrict__ yg = (bf16_raw *)a.y;

  for (int blk = 0; blk < nblk; ++blk) {
    const int t0 = blk * TB;
    const int len = (T - t0) < TB ? (T - t0) : TB;
    const int sb = blk & 1;
    if (blk + 1 < nblk) stage_load(t0 + TB);

    for (int s = 0; s < len; ++s) {
      const int t = t0 + s;
      if (a.ckpt && t == next_ck) {  // state before step t
        float *dst = a.ckpt + ((size_t)unit * nck + ck_idx) * K * V +
                     (size_t)(row_base + rowb + 4 * ig) * V + col0 + jl;
#pragma unroll
        for (int r = 0; r < 4; ++r) dst[(size_t)r * V] = h[r] * kInvC;
        next_ck += a.C;
        ++ck_idx;
      }
      // gate terms that do not depend on the contraction
      const float f = sm.fS[sb][s][0], gp = sm.fS[sb][s][1], m2g = sm.fS[sb][s][2];
      const f4_t k4 = *(const f4_t *)&sm.kS[sb][s][rowb + 4 * ig];
      const float vj = sm.vS[sb][s][col0 + jl];

      f4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const FragT af = *(const FragT *)&sm.Hx[cur][rowb + jl][FE * ig + 32 * ks];
        if constexpr (X32)
          acc = mfma_k32(af, wf[ks], acc);
        else
          acc = mfma_k16(af, wf[ks], acc);
      }
      h4_t hp;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float t1 = fmaf(f, h[r], gp);
        const float sp = fmaf(k4[r], vj, acc[r]);
        const float e = __builtin_amdgcn_exp2f(sp);
        const float rr = __builtin_amdgcn_rcpf(1.f + e);
        h[r] = fmaf(m2g, rr, t1);
        hp[r] = (_Float16)h[r];
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) sm.Hx[cur ^ 1][rowb + 4 * ig + r][col0 + jl] = hp[r];

      if (a.write_y) {
        // A[m = j][k = i] = H'[i][j] (this tile), B[k = i][n] = q_i  ->  D[m = j][*] = c y_j
        const h4_t qf = *(const h4_t *)&sm.qS[sb][s][rowb + 4 * ig];
        f4_t yv = {0.f, 0.f, 0.f, 0.f};
        yv = mfma_k16(hp, qf, yv);
        if (jl == 0) *(f4_t *)&sm.yP[cur][rb][col0 + 4 * ig] = yv;
      }
      __syncthreads();
      if (a.write_y && rb == 0 && jl == 0) {
        f4_t ys = *(const f4_t *)&sm.yP[cur][0][col0 + 4 * ig];
#pragma unroll
        for (int r2 = 1; r2 < RB; ++r2) {
          const f4_t o = *(const f4_t *)&sm.yP[cur][r2][col0 + 4 * ig];
          ys += o;
        }
        ys *= kInvC;
        const size_t yoff = (((size_t)b * T + t) * N + n) * V + col0 + 4 * ig;
        if constexpr (TL::P == 1) {
          uint2 pk;
          pk.x = (uint32_t)f32_to_bf16(ys[0]) | ((uint32_t)f32_to_bf16(ys[1]) << 16);
          pk.y = (uint32_t)f32_to_bf16(ys[2]) | ((uint32_t)f32_to_bf16(ys[3]) << 16);
          *(uint2 *)&yg[yoff] = pk;
        } else {
          *(f4_t *)&ypart_ws[(size_t)part * a.B * T * N * V + yoff] = ys;
        }
      }
      cur ^= 1;
    }
    if (blk + 1 < nblk) {
      stage_store(sb ^ 1);
      __syncthreads();
    }
  }
  if (a.HT)
#pragma unroll
    for (int r = 0; r < 4; ++r) a.HT[st_off + (size_t)r * V] = h[r] * kInvC;
}

// y = bf16( sum over parts, in increasing part order )
__global__ void y_parts_sum_kernel(const float *__restrict__ part, bf16_raw *__restrict__ y,
                                   size_t total, int P) {
  for (size_t e = (blockIdx.x * (size_t)blockDim.x + threadIdx.x) * 4; e < total;
       e += (size_t)gridDim.x * blockDim.x * 4) {
    f4_t s = *(const f4_t *)&part[e];
    for (int p = 1; p < P; ++p) s += *(const f4_t *)&part[(size_t)p * total + e];
    uint2 pk;
    pk.x = (uint32_t)f32_to_bf16(s[0]) | ((uint32_t)f32_to_bf16(s[1]) << 16);
    pk.y = (uint32_t)f32_to_bf16(s[2]) | ((uint32_t)f32_to_bf16(s[3]) << 16);
    *(uint2 *)&y[e] = pk;
  }
}

template <typename TL>
hipError_t launch_fwd(const FwdArgs &a, hipStream_t s) {
  const int units = a.B * a.N;
  if (units == 0) return hipSuccess;
  float *ypart = (float *)a.ws;
  hipLaunchKernelGGL(mfma_fwd_kernel<TL>, dim3(grid_blocks(units, TL::P)), dim3(TL::THREADS), 0, s,
                     a, ypart);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (TL::P > 1 && a.write_y && a.T > 0) {
    const size_t total = (size_t)a.B * a.T * a.N * a.V;
    size_t blocks = (total / 4 + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(y_parts_sum_kernel, dim3((unsigned)blocks), dim3(256), 0, s,
                       (const float *)ypart, (bf16_raw *)a.y, total, TL::P);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace

// Row blocks per workgroup for a shape: the largest tile that still gives the
// chip at least one workgroup per CU, else the smallest tile there is.
int mfma_pick_rb(int K, int V, int units) {
  auto parts = [&](int rb) { return K / (16 * rb); };
  if (K == 64 && V == 64) return units * parts(2) >= 256 ? 2 : 1;
  if (K == 128 && V == 128) return 1;
  if (K == 32 && V == 32) return units * parts(2) >= 256 ? 2 : 1;
  if (K == 16 && V == 16) return 1;
  if (K == 64 && V == 16) return units * parts(4) >= 256 ? 4 : 1;
  return 0;
}

hipError_t mfma_fwd(const FwdArgs &a, hipStream_t s) {
  const int rb = mfma_pick_rb(a.K, a.V, a.B * a.N);
  const int key = a.K * 10000 + a.V * 10 + rb;
  switch (key) {
    case 64 * 10000 + 64 * 10 + 2: return launch_fwd<Tile<64, 64, 2>>(a, s);
    case 64 * 10000 + 64 * 10 + 1: return launch_fwd<Tile<64, 64, 1>>(a, s);
    case 128 * 10000 + 128 * 10 + 1: return launch_fwd<Tile<128, 128, 1>>(a, s);
    case 32 * 10000 + 32 * 10 + 2: return launch_fwd<Tile<32, 32, 2>>(a, s);
    case 32 * 10000 + 32 * 10 + 1: return launch_fwd<Tile<32, 32, 1>>(a, s);
    case 16 * 10000 + 16 * 10 + 1: return launch_fwd<Tile<16, 16, 1>>(a, s);
    case 64 * 10000 + 16 * 10 + 4: return launch_fwd<Tile<64, 16, 4>>(a, s);
    case 64 * 10000 + 16 * 10 + 1: return launch_fwd<Tile<64, 16, 1>>(a, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace m2rnn

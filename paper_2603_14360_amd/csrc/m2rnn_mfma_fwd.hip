// Matrix-core forward scan (Algorithm 1 of the paper; recurrence equations),
// tiled variant: a 16-row block of one (b, n) state is spread over V/16 waves.
//
// Per workgroup: RB row blocks (16 rows each) of one state, all V columns, for
// all T steps.  Per step and wavefront (one 16 x 16 tile):
//   R  read the row block's previous state from LDS as the MFMA A operand and
//      run the contraction S' = c (H W); W fragments stay in registers.
//      The state is exchanged as an fp16 pair (hi, lo) per element, hi + lo
//      = H' to ~21 bits: the backward through this recurrence amplifies
//      forward-trajectory errors by orders of magnitude at T = 4096, so a
//      single fp16 operand (11 bits) is not enough.  The pair sits in adjacent
//      k-slots of the MFMA and the W fragment repeats each row of W twice.
//   E  in registers, fp32:  s' = S' + (c k_i) v_j ; e = 2^{s'} ; r = 1/(1+e) ;
//      H' <- f H' + c(1-f) - 2c(1-f) r        ( = c [f H + (1-f) tanh(s)] )
//      split H' into (hi, lo), write the pair back to LDS; one barrier.
//   Y  readout without leaving the step loop: one 16x16x16 MFMA with A = hi of
//      the tile (k = rows) and B = q placed in column (t mod 16) only.  The
//      accumulator is kept for 16 steps, so column s of it collects
//      c sum_i q_i H[i][j] of step s; nothing is read back per step.  Every 16
//      steps the row blocks are summed through LDS and 16 rows of y are stored.
// q, k, v, f for 16 steps at a time are staged through LDS; the next block's
// global loads are in flight while the current block is computed.
#include "m2rnn_kernels.hpp"
#include "m2rnn_mfma_common.hpp"

namespace m2rnn {
namespace {

constexpr int TB = 16;  // steps per staging / readout block (= MFMA N)

template <typename TL>
struct FwdSmem {
  alignas(16) _Float16 Hx[2][TL::ROWS][TL::LDH2];  // (hi, lo) state exchange, padded rows
  alignas(16) float kS[2][TB][TL::ROWS];           // c * k
  alignas(16) _Float16 qS[2][TB][TL::ROWS];
  alignas(16) float vS[2][TB][TL::V];
  alignas(16) float fS[2][TB][4];                  // f, c(1-f), -2c(1-f), unused
  alignas(16) f4_t yB[TL::RB][TL::CT][64];         // readout accumulators of one block
};

template <typename TL, bool DO_Y>
__global__ void __launch_bounds__(TL::THREADS)
    mfma_fwd_kernel(FwdArgs a, float *__restrict__ ypart_ws) {
  constexpr int K = TL::K, V = TL::V, RB = TL::RB, CT = TL::CT, ROWS = TL::ROWS;
  constexpr int THREADS = TL::THREADS;
  constexpr int NQ = (TB * ROWS + THREADS - 1) / THREADS;
  constexpr int NV = (TB * V + THREADS - 1) / THREADS;

  int unit, part;
  if (!map_block<TL::P>(a.B * a.N, unit, part)) return;
  const int T = a.T, N = a.N;
  const int b = unit / N, n = unit - b * N;
  const int g = n / (N / a.Nqk);
  const int tid = threadIdx.x, lane = tid & 63;
  // wave-level indices as scalars: branches on them must be real (uniform) branches, because
  // a matrix-core instruction that is merely predicated off still executes
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int rb = wave / CT, ct = wave - rb * CT;
  const int jl = lane & 15, ig = lane >> 4;
  const int col0 = ct * 16, rowb = rb * 16;
  const int row_base = part * ROWS;

  __shared__ FwdSmem<TL> sm;

  const bf16_raw *__restrict__ qg = (const bf16_raw *)a.q;
  const bf16_raw *__restrict__ kg = (const bf16_raw *)a.k;
  const bf16_raw *__restrict__ vg = (const bf16_raw *)a.v;
  const float *__restrict__ fg = a.f;

  // ---- W fragments (B operand).  k-slots 2e, 2e+1 of MFMA m both hold
  //      W[16 m + 4 ig + e][col0 + jl]: they meet the (hi, lo) pair of that element.
  h8_t wf[CT];
  {
    const bf16_raw *Wn = (const bf16_raw *)a.W + (size_t)n * V * V;
#pragma unroll
    for (int m = 0; m < CT; ++m)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int c = 16 * m + 4 * ig + e;
        const _Float16 w = (_Float16)bf16_to_f32(Wn[(size_t)c * V + col0 + jl]);
        wf[m][2 * e] = w;
        wf[m][2 * e + 1] = w;
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
      for (int r = 0; r < 4; ++r)
        a.HT[st_off + (size_t)r * V] = a.H0 ? a.H0[st_off + (size_t)r * V] : 0.f;
    return;
  }
#pragma unroll
  for (int r = 0; r < 4; ++r)
    *(uint32_t *)&sm.Hx[0][rowb + 4 * ig + r][2 * (col0 + jl)] = split_hi_lo(h[r]);

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
    // keep the conversions here: hoisted to the loads they would wait for the loads at once
#pragma unroll
    for (int m = 0; m < NQ; ++m) asm volatile("" : "+v"(rq[m]), "+v"(rk[m]));
#pragma unroll
    for (int m = 0; m < NV; ++m) asm volatile("" : "+v"(rv[m]));
    asm volatile("" : "+v"(rf));
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
  lds_barrier();

  const int nblk = (T + TB - 1) / TB;
  const int nck = (T + a.C - 1) / a.C;
  int next_ck = 0, ck_idx = 0;
  bf16_raw *__restrict__ yg = (bf16_raw *)a.y;
  const h4_t zero_h4 = {(_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f};

  // Pieces of one step.  `s` is the step inside the 16-step block; the block loop calls
  // these from a fully unrolled loop, so s, the exchange buffer index and every LDS
  // offset that depends on them are compile-time constants there (a wave issues one
  // instruction every ~5 cycles at best: loop counters, address arithmetic and branches
  // per step cost as much as the arithmetic).
  struct StepRegs {
    h8_t af[CT];
    float f, gp, m2g, vj;
    f4_t k4, acc;
    h4_t qf;
  };
  auto ckpt_store = [&](int t) __attribute__((always_inline)) {
    if (a.ckpt && t == next_ck) {  // state before step t
      float *dst = a.ckpt + ((size_t)unit * nck + ck_idx) * K * V +
                   (size_t)(row_base + rowb + 4 * ig) * V + col0 + jl;
#pragma unroll
      for (int r = 0; r < 4; ++r) dst[(size_t)r * V] = h[r] * kInvC;
      next_ck += a.C;
      ++ck_idx;
    }
  };
  // R: operand fetch from exchange buffer `buf`, this step's vectors, contraction
  auto step_R = [&](StepRegs &x, int s, int sb, int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int m = 0; m < CT; ++m)
      x.af[m] = *(const h8_t *)&sm.Hx[buf][rowb + jl][2 * (16 * m + 4 * ig)];
    x.f = sm.fS[sb][s][0];
    x.gp = sm.fS[sb][s][1];
    x.m2g = sm.fS[sb][s][2];
    x.k4 = *(const f4_t *)&sm.kS[sb][s][rowb + 4 * ig];
    x.vj = sm.vS[sb][s][col0 + jl];
    if constexpr (DO_Y) x.qf = *(const h4_t *)&sm.qS[sb][s][rowb + 4 * ig];
    x.acc = f4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int m = 0; m < CT; ++m) x.acc = mfma_k32(x.af[m], wf[m], x.acc);
    settle(x.acc);
  };
  // E: tanh, gate, split, write back into exchange buffer `buf`
  auto step_E = [&](const StepRegs &x, uint32_t (&pk)[4], int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float t1 = fmaf(x.f, h[r], x.gp);
      const float sp = fmaf(x.k4[r], x.vj, x.acc[r]);
      const float e = __builtin_amdgcn_exp2f(sp);
      const float rr = __builtin_amdgcn_rcpf(1.f + e);
      h[r] = fmaf(x.m2g, rr, t1);
      pk[r] = split_hi_lo(h[r]);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r)
      *(uint32_t *)&sm.Hx[buf][rowb + 4 * ig + r][2 * (col0 + jl)] = pk[r];
  };
  // Y: readout on the matrix core.  A[m = j][k = i] = hi(H'[i][j]) of this tile;
  //    B[k = i][n] = q_i for n == s, else 0: column s of yacc collects step s.
  auto step_Y = [&](const StepRegs &x, const uint32_t (&pk)[4], int s, f4_t &yacc)
      __attribute__((always_inline)) {
    const h4_t qf = (jl == s) ? x.qf : zero_h4;
    uint2 hv;
    hv.x = __builtin_amdgcn_perm(pk[1], pk[0], 0x05040100u);
    hv.y = __builtin_amdgcn_perm(pk[3], pk[2], 0x05040100u);
    yacc = mfma_k16(__builtin_bit_cast(h4_t, hv), qf, yacc);
  };
  auto y_store = [&](f4_t ys, int t0, int len) __attribute__((always_inline)) {
    // lane (ig, jl) holds columns col0 + 4 ig + r of step t0 + jl
    if (jl < len) {
      ys *= kInvC;
      const size_t yoff = (((size_t)b * T + t0 + jl) * N + n) * V + col0 + 4 * ig;
      if constexpr (TL::P == 1) {
        if (a.w_r) {  // residual w_r (.) v_t of the y equation
          const uint2 wv = *(const uint2 *)&((const bf16_raw *)a.w_r)[n * V + col0 + 4 * ig];
          const uint2 vv = *(const uint2 *)&vg[yoff];
          ys[0] = fmaf(bf16_to_f32(wv.x & 0xFFFFu), bf16_to_f32(vv.x & 0xFFFFu), ys[0]);
          ys[1] = fmaf(bf16_to_f32(wv.x >> 16), bf16_to_f32(vv.x >> 16), ys[1]);
          ys[2] = fmaf(bf16_to_f32(wv.y & 0xFFFFu), bf16_to_f32(vv.y & 0xFFFFu), ys[2]);
          ys[3] = fmaf(bf16_to_f32(wv.y >> 16), bf16_to_f32(vv.y >> 16), ys[3]);
        }
        uint2 p2;
        p2.x = (uint32_t)f32_to_bf16(ys[0]) | ((uint32_t)f32_to_bf16(ys[1]) << 16);
        p2.y = (uint32_t)f32_to_bf16(ys[2]) | ((uint32_t)f32_to_bf16(ys[3]) << 16);
        *(uint2 *)&yg[yoff] = p2;
      } else {
        *(f4_t *)&ypart_ws[(size_t)part * a.B * T * N * V + yoff] = ys;
      }
    }
  };

  {
    // ---- lock-step schedule: one barrier per step, exchange buffer alternates.
    // (A ping-pong schedule -- the two row blocks of a workgroup half a step apart, two
    //  barriers per step, so that the waves sharing a SIMD alternate between operand fetch
    //  and vector-ALU work -- was measured 10 % slower at B*N = 128, K = V = 64.)
    for (int blk = 0; blk < nblk; ++blk) {
      const int t0 = blk * TB;
      const int len = (T - t0) < TB ? (T - t0) : TB;
      const int sb = blk & 1;
      const bool more = blk + 1 < nblk;
      if (more) stage_load(t0 + TB);
      f4_t yacc = {0.f, 0.f, 0.f, 0.f};  // D[m = j][n = s] = c * y partial of step t0 + s
      auto step = [&](int s) __attribute__((always_inline)) {
        StepRegs x;
        ckpt_store(t0 + s);
        step_R(x, s, sb, s & 1);  // every block but the last has 16 steps: parity of s
        if (s == TB / 2 && more) stage_store(sb ^ 1);  // next block's vectors have landed
        uint32_t pk[4];
        step_E(x, pk, (s & 1) ^ 1);
        lds_barrier();
        // after the barrier: the readout MFMA runs while the next step's operands are fetched
        if constexpr (DO_Y) step_Y(x, pk, s, yacc);
      };
      if (len == TB) {
#pragma unroll
        for (int s = 0; s < TB; ++s) step(s);
      } else {
#pragma nounroll
        for (int s = 0; s < len; ++s) step(s);
      }
      if constexpr (DO_Y) {
        // ---- block flush: sum the row blocks, store the block's rows of y
        if constexpr (RB > 1) {
          if (rb > 0) sm.yB[rb][ct][lane] = yacc;
          lds_barrier();
          if (rb == 0) {
#pragma unroll
            for (int r2 = 1; r2 < RB; ++r2) yacc += sm.yB[r2][ct][lane];
          }
          // (yB is written again only 16 steps, i.e. at least 16 barriers, later)
        }
        if (rb == 0) y_store(yacc, t0, len);
      }
    }
  }
  if (a.HT)
#pragma unroll
    for (int r = 0; r < 4; ++r) a.HT[st_off + (size_t)r * V] = h[r] * kInvC;
}

// y = bf16( sum over parts, in increasing part order [+ w_r (.) v, the residual of the y
// equation, when w_r is given] ); NV = N * V, the period of w_r along the flat index
__global__ void y_parts_sum_kernel(const float *__restrict__ part, bf16_raw *__restrict__ y,
                                   size_t total, int P, const bf16_raw *__restrict__ w_r,
                                   const bf16_raw *__restrict__ v, int NV) {
  for (size_t e = (blockIdx.x * (size_t)blockDim.x + threadIdx.x) * 4; e < total;
       e += (size_t)gridDim.x * blockDim.x * 4) {
    f4_t s = *(const f4_t *)&part[e];
    for (int p = 1; p < P; ++p) s += *(const f4_t *)&part[(size_t)p * total + e];
    if (w_r) {
      const uint2 wv = *(const uint2 *)&w_r[e % (size_t)NV];
      const uint2 vv = *(const uint2 *)&v[e];
      s[0] = fmaf(bf16_to_f32(wv.x & 0xFFFFu), bf16_to_f32(vv.x & 0xFFFFu), s[0]);
      s[1] = fmaf(bf16_to_f32(wv.x >> 16), bf16_to_f32(vv.x >> 16), s[1]);
      s[2] = fmaf(bf16_to_f32(wv.y & 0xFFFFu), bf16_to_f32(vv.y & 0xFFFFu), s[2]);
      s[3] = fmaf(bf16_to_f32(wv.y >> 16), bf16_to_f32(vv.y >> 16), s[3]);
    }
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
  if (a.write_y)
    hipLaunchKernelGGL((mfma_fwd_kernel<TL, true>), dim3(grid_blocks(units, TL::P)),
                       dim3(TL::THREADS), 0, s, a, ypart);
  else
    hipLaunchKernelGGL((mfma_fwd_kernel<TL, false>), dim3(grid_blocks(units, TL::P)),
                       dim3(TL::THREADS), 0, s, a, ypart);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (TL::P > 1 && a.write_y && a.T > 0) {
    const size_t total = (size_t)a.B * a.T * a.N * a.V;
    size_t blocks = (total / 4 + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(y_parts_sum_kernel, dim3((unsigned)blocks), dim3(256), 0, s,
                       (const float *)ypart, (bf16_raw *)a.y, total, TL::P,
                       (const bf16_raw *)a.w_r, (const bf16_raw *)a.v, a.N * a.V);
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
  if (K == 64 && V == 16) return 1;  // (4 row blocks per workgroup: 20 % slower backward at 672 states)
  return 0;
}

hipError_t mfma_fwd(const FwdArgs &a, hipStream_t s) {
  const int rb = mfma_pick_rb(a.K, a.V, a.B * a.N);
#define X(K_, V_, RB_) \
  if (a.K == K_ && a.V == V_ && rb == RB_) return launch_fwd<Tile<K_, V_, RB_>>(a, s);
  M2RNN_TILE_CASES(X)
#undef X
  return hipErrorInvalidValue;
}

}  // namespace m2rnn

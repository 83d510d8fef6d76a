// Matrix-core forward scan, tiled variant with TWO row blocks per wavefront.
//
// Same arithmetic as the one-tile-per-wave forward kernel (recurrence equations,
// Algorithm 1 of the paper; (hi, lo) fp16 state exchange; scaled state; readout
// on the matrix core with q placed in column t mod 16), but a wave owns column
// tile ct of two independent 16-row blocks A and B of the same (b, n) state and
// runs them half a step apart:
//
//     issue LDS reads of B's operand | E(A): tanh, gate, split, write A | MFMA(B) | barrier
//     issue LDS reads of A's operand | E(B): tanh, gate, split, write B | MFMA(A) | barrier
//
// The LDS round trip of one block (write, barrier, read, MFMA: several hundred
// cycles on this chip) is covered by the other block's vector-ALU work inside
// the same instruction stream, so one wave per SIMD keeps the ALU busy; with
// one tile per wave the waves of a workgroup move in lock step through the
// barrier and nothing hides that latency.
#include "m2rnn_kernels.hpp"
#include "m2rnn_mfma_common.hpp"

namespace m2rnn {
namespace {

constexpr int TB = 16;  // steps per staging / readout block (= MFMA N)

template <int K_, int V_>
struct Pair {
  static constexpr int K = K_, V = V_;
  static constexpr int CT = V / 16;        // waves per workgroup (one column tile each)
  static constexpr int THREADS = CT * 64;
  static constexpr int ROWS = 32;          // two row blocks
  static constexpr int P = K / 32;         // workgroups per state
  static constexpr int LDH2 = 2 * V + 8;
  static_assert(K % 32 == 0 && V % 16 == 0, "bad shape");
};

template <typename PT>
struct PairSmem {
  alignas(16) _Float16 Hx[PT::ROWS][PT::LDH2];     // (hi, lo) state exchange, single buffer
  alignas(16) float kS[2][TB][PT::ROWS];           // c * k
  alignas(16) _Float16 qS[2][TB][PT::ROWS];
  alignas(16) float vS[2][TB][PT::V];
  alignas(16) float fS[2][TB][4];                  // f, c(1-f), -2c(1-f), unused
};

template <typename PT>
__global__ void __launch_bounds__(PT::THREADS)
    pair_fwd_kernel(FwdArgs a, float *__restrict__ ypart_ws) {
  constexpr int K = PT::K, V = PT::V, CT = PT::CT, ROWS = PT::ROWS, THREADS = PT::THREADS;
  constexpr int NQ = (TB * ROWS + THREADS - 1) / THREADS;
  constexpr int NV = (TB * V + THREADS - 1) / THREADS;

  int unit, part;
  if (!map_block<PT::P>(a.B * a.N, unit, part)) return;
  const int T = a.T, N = a.N;
  const int b = unit / N, n = unit - b * N;
  const int g = n / (N / a.Nqk);
  const int tid = threadIdx.x, lane = tid & 63;
  const int ct = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int jl = lane & 15, ig = lane >> 4;
  const int col0 = ct * 16;
  const int row_base = part * ROWS;

  __shared__ PairSmem<PT> sm;

  const bf16_raw *__restrict__ qg = (const bf16_raw *)a.q;
  const bf16_raw *__restrict__ kg = (const bf16_raw *)a.k;
  const bf16_raw *__restrict__ vg = (const bf16_raw *)a.v;
  const float *__restrict__ fg = a.f;

  // ---- W fragments (B operand): k-slots 2e, 2e+1 of MFMA m hold W[16 m + 4 ig + e][col0 + jl]
  h8_t wf[CT];
  {
    const bf16_raw *Wn = (const bf16_raw *)a.W + (size_t)n * V * V;
#pragma unroll
    for (int m = 0; m < CT; ++m)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const _Float16 w =
            (_Float16)bf16_to_f32(Wn[(size_t)(16 * m + 4 * ig + e) * V + col0 + jl]);
        wf[m][2 * e] = w;
        wf[m][2 * e + 1] = w;
      }
  }

  // ---- state tiles of the two row blocks (x = 0: rows 0..15, x = 1: rows 16..31), scaled by c
  const size_t st_off = (size_t)unit * K * V + (size_t)(row_base + 4 * ig) * V + col0 + jl;
  float h[2][4];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float h0 = a.H0 ? a.H0[st_off + (size_t)(16 * x + r) * V] : 0.f;
      if (T == 0 && a.HT) a.HT[st_off + (size_t)(16 * x + r) * V] = h0;
      h[x][r] = kC * h0;
    }
  if (T == 0) return;
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int r = 0; r < 4; ++r)
      *(uint32_t *)&sm.Hx[16 * x + 4 * ig + r][2 * (col0 + jl)] = split_hi_lo(h[x][r]);

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
      rv[m] = ok ? vg[(((size_t)b * T + (t0 + s)) * N + n) * V + j] : (bf16_raw)0;
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

  // operand fetch + contraction of one row block
  auto fetch = [&](int x, h8_t *af) {
#pragma unroll
    for (int m = 0; m < CT; ++m)
      af[m] = *(const h8_t *)&sm.Hx[16 * x + jl][2 * (16 * m + 4 * ig)];
  };
  auto contract = [&](const h8_t *af) {
    f4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int m = 0; m < CT; ++m) acc = mfma_k32(af[m], wf[m], acc);
    return acc;
  };

  const int nblk = (T + TB - 1) / TB;
  const int nck = (T + a.C - 1) / a.C;
  int next_ck = 0, ck_idx = 0;
  bf16_raw *__restrict__ yg = (bf16_raw *)a.y;
  const bool do_y = a.write_y != 0;
  const h4_t zero_h4 = {(_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f};

  f4_t accA;
  {
    h8_t af[CT];
    fetch(0, af);
    accA = contract(af);
  }
  lds_barrier();  // every wave has read block A's initial state before anyone overwrites it

  for (int blk = 0; blk < nblk; ++blk) {
    const int t0 = blk * TB;
    const int len = (T - t0) < TB ? (T - t0) : TB;
    const int sb = blk & 1;
    const bool more = blk + 1 < nblk;
    if (more) stage_load(t0 + TB);
    f4_t yacc = {0.f, 0.f, 0.f, 0.f};  // D[m = j][n = s] = c * y partial of step t0 + s

    for (int s = 0; s < len; ++s) {
      const int t = t0 + s;
      if (a.ckpt && t == next_ck) {  // state before step t
        float *dst = a.ckpt + ((size_t)unit * nck + ck_idx) * K * V +
                     (size_t)(row_base + 4 * ig) * V + col0 + jl;
#pragma unroll
        for (int x = 0; x < 2; ++x)
#pragma unroll
          for (int r = 0; r < 4; ++r) dst[(size_t)(16 * x + r) * V] = h[x][r] * kInvC;
        next_ck += a.C;
        ++ck_idx;
      }
      if (more && s == TB / 2) stage_store(sb ^ 1);  // next block's vectors have landed

      // small per-step operands first: LDS returns in order, so anything issued after the
      // big operand fetch would have to wait for it
      const float f = sm.fS[sb][s][0], gp = sm.fS[sb][s][1], m2g = sm.fS[sb][s][2];
      const float vj = sm.vS[sb][s][col0 + jl];
      f4_t k4x[2];
      h4_t qfx[2];
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        k4x[x] = *(const f4_t *)&sm.kS[sb][s][16 * x + 4 * ig];
        qfx[x] = *(const h4_t *)&sm.qS[sb][s][16 * x + 4 * ig];
      }
      asm volatile("" ::: "memory");  // keep these reads ahead of the fetches below
      const bool mine = jl == s;
      f4_t accB;
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        // reads of the OTHER block's operand go out first; this block's E covers their latency
        h8_t af[CT];
        fetch(x ^ 1, af);
        const f4_t k4 = k4x[x];
        h4_t qf = qfx[x];
        const f4_t acc = x == 0 ? accA : accB;
        uint32_t pk[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float t1 = fmaf(f, h[x][r], gp);
          const float sp = fmaf(k4[r], vj, acc[r]);
          const float e = __builtin_amdgcn_exp2f(sp);
          const float rr = __builtin_amdgcn_rcpf(1.f + e);
          h[x][r] = fmaf(m2g, rr, t1);
          pk[r] = split_hi_lo(h[x][r]);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r)
          *(uint32_t *)&sm.Hx[16 * x + 4 * ig + r][2 * (col0 + jl)] = pk[r];
        // the other block's contraction: for x == 0 block B of this step, for x == 1 block A of
        // the next step (its state was written in the first half and published by the barrier)
        // the operand reads need the whole E above to land; keep the MFMAs behind it
        __builtin_amdgcn_sched_barrier(0);
        if (x == 0)
          accB = contract(af);
        else
          accA = contract(af);
        if (do_y) {
          // A[m = j][k = i] = hi(H'[i][j]); B[k = i][n] = q_i for n == s, else 0
          if (!mine) qf = zero_h4;
          yacc = mfma_k16(hi_of_pairs(pk), qf, yacc);
        }
        lds_barrier();
      }
    }

    if (do_y && jl < len) {
      // block flush: lane (ig, jl) holds columns col0 + 4 ig + r of step t0 + jl (both row blocks)
      yacc *= kInvC;
      const size_t yoff = (((size_t)b * T + t0 + jl) * N + n) * V + col0 + 4 * ig;
      if constexpr (PT::P == 1) {
        uint2 p2;
        p2.x = (uint32_t)f32_to_bf16(yacc[0]) | ((uint32_t)f32_to_bf16(yacc[1]) << 16);
        p2.y = (uint32_t)f32_to_bf16(yacc[2]) | ((uint32_t)f32_to_bf16(yacc[3]) << 16);
        *(uint2 *)&yg[yoff] = p2;
      } else {
        *(f4_t *)&ypart_ws[(size_t)part * a.B * T * N * V + yoff] = yacc;
      }
    }
  }
  if (a.HT)
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int r = 0; r < 4; ++r) a.HT[st_off + (size_t)(16 * x + r) * V] = h[x][r] * kInvC;
}

}  // namespace

void y_parts_sum_launch(const float *part, void *y, size_t total, int P, hipStream_t s);

template <typename PT>
static hipError_t launch_pair(const FwdArgs &a, hipStream_t s) {
  const int units = a.B * a.N;
  if (units == 0) return hipSuccess;
  float *ypart = (float *)a.ws;
  hipLaunchKernelGGL(pair_fwd_kernel<PT>, dim3(grid_blocks(units, PT::P)), dim3(PT::THREADS), 0, s,
                     a, ypart);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (PT::P > 1 && a.write_y && a.T > 0) {
    y_parts_sum_launch(ypart, a.y, (size_t)a.B * a.T * a.N * a.V, PT::P, s);
    e = hipGetLastError();
  }
  return e;
}

bool pair_fwd_supported(int K, int V) { return K == 64 && V == 64; }

hipError_t pair_fwd(const FwdArgs &a, hipStream_t s) {
  if (a.K == 64 && a.V == 64) return launch_pair<Pair<64, 64>>(a, s);
  return hipErrorInvalidValue;
}

}  // namespace m2rnn

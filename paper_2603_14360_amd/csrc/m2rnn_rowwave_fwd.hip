// Register-resident forward scan (Algorithm 1 of the paper; recurrence
// equations) for V <= 64: one wavefront owns 16 rows of one (b, n) state and
// ALL V columns, and nothing about the recurrence leaves its registers.
//
// The K rows of the state are independent recurrences (row i of H W + k v^T
// needs only row i of H and the scalar k_i), so a wave never needs another
// wave's state.  The problem is run transposed, S^T = W^T H^T, because then the
// MFMA accumulator layout (lane = state row i, 4 consecutive columns per
// register group) IS the B-operand layout of the next step's MFMA: after the
// elementwise update the packed (hi, lo) fp16 pairs of a 16 x 16 tile feed the
// next contraction directly.  No LDS exchange and no barrier sit on the
// step-to-step dependency chain (an LDS round trip on this chip costs ~400
// cycles per step, more than the arithmetic).
//
// Per step, per 16-column tile ct (software pipelined across the tiles):
//   E   s' = acc[ct] + (c k_i) v_j ; H' <- c [f H + (1-f) tanh(s)] (gate_tanh_step) ;
//       (hi, lo) = split(H')
//   M   for every output tile jt: acc'[jt] += W^T[jt][ct] (hi, lo)[ct]
//       (16x16x32 MFMA: the pair occupies adjacent k-slots, the W fragment
//        holds each row of W twice) -- these run on the matrix core while the
//       vector ALU does E of the next tile.
// Readout y_t = H_t^T q_t contracts over the rows, which are the lane index in
// this layout.  The matrix core does the transpose: the tile's (hi, lo)
// fragment times an identity fragment gives H' with rows in the registers and
// columns across lanes, which (as fp16) is the A operand of a 16x16x16 MFMA
// with q.  The K/16 row-block partials of a state are summed once per 16 steps
// through LDS and stored as whole bf16 rows.
#include "m2rnn_kernels.hpp"
#include "m2rnn_mfma_common.hpp"

namespace m2rnn {
namespace {

constexpr int TB = 16;  // steps per staging / flush block

template <int K_, int V_>
struct RowWave {
  static constexpr int K = K_, V = V_;
  static constexpr int CT = V / 16;   // 16-column tiles per wave
  static constexpr int NW = K / 16;   // waves (row blocks) per workgroup = per state
  static constexpr int THREADS = NW * 64;
  // LDS carve-up (bytes)
  static constexpr int STG = TB * (K * 4 + K * 2 + V * 2 + 16);  // c*k f32, q f16, v f16, f
  static constexpr int OFF_K = 0;
  static constexpr int OFF_Q = OFF_K + TB * K * 4;
  static constexpr int OFF_V = OFF_Q + TB * K * 2;
  static constexpr int OFF_F = OFF_V + TB * V * 2;
  static constexpr int OFF_Y = 2 * STG;                          // [2][NW][TB][V] f32
  static constexpr int BYTES = OFF_Y + 2 * NW * TB * V * 4;
  static_assert(STG % 16 == 0 && BYTES <= kLdsLimit, "LDS layout");
};

template <typename RW, bool DO_Y>
__global__ void __launch_bounds__(RW::THREADS, 2) rowwave_fwd_kernel(FwdArgs a) {
  constexpr int K = RW::K, V = RW::V, CT = RW::CT, NW = RW::NW, THREADS = RW::THREADS;
  constexpr int NQ = (TB * K + THREADS - 1) / THREADS;
  constexpr int NV = (TB * V + THREADS - 1) / THREADS;

  const int unit = blockIdx.x;
  const int T = a.T, N = a.N;
  const int b = unit / N, n = unit - b * N;
  const int g = n / (N / a.Nqk);
  const int tid = threadIdx.x, lane = tid & 63;
  const int rb = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: one row block per wave
  const int jl = lane & 15, ig = lane >> 4;
  const int row = rb * 16 + jl;  // state row of this lane

  extern __shared__ __attribute__((aligned(16))) char lds[];
  auto kS = [&](int buf) { return (float *)(lds + buf * RW::STG + RW::OFF_K); };
  auto qH = [&](int buf) { return (_Float16 *)(lds + buf * RW::STG + RW::OFF_Q); };
  auto vH = [&](int buf) { return (_Float16 *)(lds + buf * RW::STG + RW::OFF_V); };
  auto fS = [&](int buf) { return (float *)(lds + buf * RW::STG + RW::OFF_F); };
  float *yacc = (float *)(lds + RW::OFF_Y);

  const bf16_raw *__restrict__ qg = (const bf16_raw *)a.q;
  const bf16_raw *__restrict__ kg = (const bf16_raw *)a.k;
  const bf16_raw *__restrict__ vg = (const bf16_raw *)a.v;
  const float *__restrict__ fg = a.f;
  bf16_raw *__restrict__ yg = (bf16_raw *)a.y;

  // ---- W fragments (A operand of S^T = W^T H^T): slots 2e, 2e+1 of the MFMA for
  //      (jt, ct) hold W[16 ct + 4 ig + e][16 jt + jl]; they meet the (hi, lo) pair.
  h8_t wf[CT][CT];
  {
    const bf16_raw *Wn = (const bf16_raw *)a.W + (size_t)n * V * V;
#pragma unroll
    for (int jt = 0; jt < CT; ++jt)
#pragma unroll
      for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const _Float16 w =
              (_Float16)bf16_to_f32(Wn[(size_t)(16 * ct + 4 * ig + e) * V + 16 * jt + jl]);
          wf[jt][ct][2 * e] = w;
          wf[jt][ct][2 * e + 1] = w;
        }
  }
  // identity fragment: B[slot][n] = 1 for both slots of column 4 ig + e when that column is n
  h8_t ident;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const _Float16 one = (4 * ig + e == jl) ? (_Float16)1.0f : (_Float16)0.0f;
    ident[2 * e] = one;
    ident[2 * e + 1] = one;
  }

  // ---- state: lane (row, ig) holds columns 16 ct + 4 ig + r, scaled by c
  const size_t st_off = (size_t)unit * K * V + (size_t)row * V + 4 * ig;
  float h[CT][4];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
    f4_t x = {0.f, 0.f, 0.f, 0.f};
    if (a.H0) x = *(const f4_t *)&a.H0[st_off + 16 * ct];
    if (T == 0 && a.HT) *(f4_t *)&a.HT[st_off + 16 * ct] = x;
#pragma unroll
    for (int r = 0; r < 4; ++r) h[ct][r] = kC * x[r];
  }
  if (T == 0) return;

  // ---- staging of q, k, v, f: TB steps per block, next block's loads in flight
  bf16_raw rq[NQ], rk[NQ], rv[NV];
  float rf = 1.f;
  auto stage_load = [&](int t0) {
#pragma unroll
    for (int m = 0; m < NQ; ++m) {
      const int idx = tid + m * THREADS;
      const int s = idx / K, i = idx - s * K;
      const bool ok = idx < TB * K && t0 + s < T;
      const size_t off = (((size_t)b * T + (t0 + s)) * a.Nqk + g) * K + i;
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
      if (idx < TB * K) {
        kS(buf)[idx] = kC * bf16_to_f32(rk[m]);
        qH(buf)[idx] = (_Float16)bf16_to_f32(rq[m]);
      }
    }
#pragma unroll
    for (int m = 0; m < NV; ++m) {
      const int idx = tid + m * THREADS;
      if (idx < TB * V) vH(buf)[idx] = (_Float16)bf16_to_f32(rv[m]);
    }
    if (tid < TB) {
      if (a.gate_alpha) rf = gate_psi(rf, a.gate_alpha[n], a.gate_beta[n]);
      const float gp = kC * (1.f - rf);
      fS(buf)[tid * 4 + 0] = rf;
      fS(buf)[tid * 4 + 1] = gp;
    }
  };

  stage_load(0);
  stage_store(0);

  auto frag_of = [&](const float *hc) {
    uint4 pk;
    pk.x = split_hi_lo(hc[0]);
    pk.y = split_hi_lo(hc[1]);
    pk.z = split_hi_lo(hc[2]);
    pk.w = split_hi_lo(hc[3]);
    return __builtin_bit_cast(h8_t, pk);
  };

  // ---- contraction for the first step from the initial state, all tiles but the last;
  //      the last tile's slice is added at the top of the step (software pipeline)
  f4_t acc[CT];
  h8_t hfL = frag_of(h[CT - 1]);
#pragma unroll
  for (int jt = 0; jt < CT; ++jt) acc[jt] = f4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int ct = 0; ct + 1 < CT; ++ct) {
    const h8_t hf = frag_of(h[ct]);
#pragma unroll
    for (int jt = 0; jt < CT; ++jt) acc[jt] = mfma_k32(wf[jt][ct], hf, acc[jt]);
  }
  lds_barrier();

  const int nblk = (T + TB - 1) / TB;
  const int nck = (T + a.C - 1) / a.C;
  int next_ck = 0, ck_idx = 0;

  for (int blk = 0; blk < nblk; ++blk) {
    const int t0 = blk * TB;
    const int len = (T - t0) < TB ? (T - t0) : TB;
    const int sb = blk & 1;
    const bool more = blk + 1 < nblk;
    if (more) stage_load(t0 + TB);

    auto step = [&](int s) __attribute__((always_inline)) {
      const int t = t0 + s;
      if (a.ckpt && t == next_ck) {  // state before step t
        float *dst = a.ckpt + ((size_t)unit * nck + ck_idx) * K * V + (size_t)row * V + 4 * ig;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
          f4_t x;
#pragma unroll
          for (int r = 0; r < 4; ++r) x[r] = h[ct][r] * kInvC;
          *(f4_t *)&dst[16 * ct] = x;
        }
        next_ck += a.C;
        ++ck_idx;
      }
      if (more && s == TB / 2) stage_store(sb ^ 1);

      // ---- straight-line step body
      const float ki = kS(sb)[s * K + row];
      const float f = fS(sb)[s * 4 + 0], gp = fS(sb)[s * 4 + 1];
      h4_t vfr[CT];
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) vfr[ct] = *(const h4_t *)&vH(sb)[s * V + 16 * ct + 4 * ig];
      h4_t qfr;
      if (DO_Y) qfr = *(const h4_t *)&qH(sb)[s * K + rb * 16 + 4 * ig];
      float *yrow = &yacc[((sb * NW + rb) * TB + s) * V + 4 * ig];

      // last tile's slice of this step's contraction (tile 0 first: it is needed first)
#pragma unroll
      for (int jt = 0; jt < CT; ++jt) acc[jt] = mfma_k32(wf[jt][CT - 1], hfL, acc[jt]);

      f4_t nx[CT], tr[CT];
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        // E: tile ct
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float sp = fmaf(ki, (float)vfr[ct][r], acc[ct][r]);
          h[ct][r] = gate_tanh_step(f, gp, h[ct][r], sp);
        }
        const h8_t hf = frag_of(h[ct]);
        // M: this tile is a k-slice of the next step's contraction
        if (ct + 1 < CT) {
#pragma unroll
          for (int jt = 0; jt < CT; ++jt)
            nx[jt] = mfma_k32(wf[jt][ct], hf, ct == 0 ? f4_t{0.f, 0.f, 0.f, 0.f} : nx[jt]);
        } else {
          hfL = hf;
        }
        // transpose on the matrix core: D[m = i][n = j] = hi + lo of H'[i][j]
        if (DO_Y) tr[ct] = mfma_k32(hf, ident, f4_t{0.f, 0.f, 0.f, 0.f});
      }
      if (DO_Y) {
        typedef float f2_t __attribute__((ext_vector_type(2)));
        f4_t yv[CT];
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
          const f2_t a01 = {tr[ct][0], tr[ct][1]}, a23 = {tr[ct][2], tr[ct][3]};
          uint2 tp;
          tp.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(a01, h2_t));
          tp.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(a23, h2_t));
          // D[m = j][*] = c sum_i q_i H[i][j]
          yv[ct] = mfma_k16(__builtin_bit_cast(h4_t, tp), qfr, f4_t{0.f, 0.f, 0.f, 0.f});
        }
        if (jl == 0) {
#pragma unroll
          for (int ct = 0; ct < CT; ++ct) *(f4_t *)&yrow[16 * ct] = yv[ct];
        }
      }
#pragma unroll
      for (int jt = 0; jt < CT; ++jt) acc[jt] = (CT > 1) ? nx[jt] : f4_t{0.f, 0.f, 0.f, 0.f};
      // scheduling hint: spread the matrix-core instructions between vector-ALU work
      // instead of issuing them back to back (a lone wave stalls behind a busy matrix core)
#pragma unroll
      for (int i = 0; i < (DO_Y ? 6 : 4) * CT; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);  // VALU
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
      }
    };
    // A full block is unrolled: the step index, and with it every LDS offset and the
    // position of the mid-block staging, are compile-time constants (a wave issues one
    // instruction every ~5 cycles at best: loop counters, address arithmetic and branches per
    // step cost as much as the arithmetic).  The ragged last block runs the loop.
    if (len == TB) {
#pragma unroll
      for (int s = 0; s < TB; ++s) step(s);
    } else {
      for (int s = 0; s < len; ++s) step(s);
    }
    lds_barrier();  // y partials of this block and the next block's staging are complete
    if (DO_Y) {
      // flush: sum the row-block partials, store whole bf16 rows (4 values per thread)
      for (int idx = tid * 4; idx < len * V; idx += THREADS * 4) {
        const int s = idx / V, j = idx - s * V;
        f4_t ys = *(const f4_t *)&yacc[((sb * NW + 0) * TB + s) * V + j];
#pragma unroll
        for (int w = 1; w < NW; ++w) ys += *(const f4_t *)&yacc[((sb * NW + w) * TB + s) * V + j];
        ys *= kInvC;
        const size_t yoff = (((size_t)b * T + t0 + s) * N + n) * V + j;
        if (a.w_r) {  // residual w_r (.) v_t of the y equation
          const uint2 wv = *(const uint2 *)&((const bf16_raw *)a.w_r)[n * V + j];
          const uint2 vv = *(const uint2 *)&((const bf16_raw *)a.v)[yoff];
          ys[0] = fmaf(bf16_to_f32(wv.x & 0xFFFFu), bf16_to_f32(vv.x & 0xFFFFu), ys[0]);
          ys[1] = fmaf(bf16_to_f32(wv.x >> 16), bf16_to_f32(vv.x >> 16), ys[1]);
          ys[2] = fmaf(bf16_to_f32(wv.y & 0xFFFFu), bf16_to_f32(vv.y & 0xFFFFu), ys[2]);
          ys[3] = fmaf(bf16_to_f32(wv.y >> 16), bf16_to_f32(vv.y >> 16), ys[3]);
        }
        uint2 p2;
        p2.x = (uint32_t)f32_to_bf16(ys[0]) | ((uint32_t)f32_to_bf16(ys[1]) << 16);
        p2.y = (uint32_t)f32_to_bf16(ys[2]) | ((uint32_t)f32_to_bf16(ys[3]) << 16);
        *(uint2 *)&yg[yoff] = p2;
      }
    }
  }
  if (a.HT) {
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
      f4_t x;
#pragma unroll
      for (int r = 0; r < 4; ++r) x[r] = h[ct][r] * kInvC;
      *(f4_t *)&a.HT[st_off + 16 * ct] = x;
    }
  }
}

template <typename RW>
hipError_t launch(const FwdArgs &a, hipStream_t s) {
  const int units = a.B * a.N;
  if (units == 0) return hipSuccess;
  auto go = [&](auto kernel) {
    hipError_t e = set_max_lds_once(kernel, RW::BYTES);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kernel, dim3(units), dim3(RW::THREADS), RW::BYTES, s, a);
    return hipGetLastError();
  };
  return a.write_y ? go(rowwave_fwd_kernel<RW, true>) : go(rowwave_fwd_kernel<RW, false>);
}

}  // namespace

bool rowwave_supported(int K, int V) {
  return (V == 16 || V == 32 || V == 64) && (K == 16 || K == 32 || K == 64 || K == 128);
}

hipError_t rowwave_fwd(const FwdArgs &a, hipStream_t s) {
#define X(K_, V_) \
  if (a.K == K_ && a.V == V_) return launch<RowWave<K_, V_>>(a, s);
  M2RNN_ROWWAVE_CASES(X)
#undef X
  return hipErrorInvalidValue;
}

}  // namespace m2rnn

// Matrix-core forward scan (Algorithm 1 of the paper; recurrence equations),
// tiled variant: a 16-row block of one (b, n) state is spread over V/16 waves.
//
// Per workgroup: RB row blocks (16 rows each) of one state, all V columns, for
// all T steps.  A wavefront owns one 16 x 16 tile; lane l holds row l % 16 and
// the four columns 4 (l / 16) + r of it.  The contraction is computed
// transposed, (H W)^T = W^T H^T: W^T is the MFMA A operand (fragments stay in
// registers) and the state tile is the B operand, whose register layout (lane =
// row of H, registers = contraction index) is exactly the layout of the MFMA
// result.  A wave's own tile therefore goes from one step's result to the next
// step's operand without leaving its registers, and the other V/16 - 1 tiles of
// the row block are exchanged through LDS as ready-made fragments: one 16-byte
// write and V/16 - 1 16-byte reads per lane and step, free of bank conflicts.
// Per step:
//   R  read the other tiles' fragments and run the contraction S' = c (H W).
//      The state is exchanged as an fp16 pair (hi, lo) per element, hi + lo
//      = H' to ~21 bits: the backward through this recurrence amplifies
//      forward-trajectory errors by orders of magnitude at T = 4096, so a
//      single fp16 operand (11 bits) is not enough.  The pair sits in adjacent
//      k-slots of the MFMA and the W fragment repeats each row of W twice.
//   E  in registers, fp32:  s' = S' + (c k_i) v_j ; e = 2^{-|s'|} ; r = 1/(1+e) ;
//      H' <- f H' + sign(s') c(1-f) (1-e) r   ( = c [f H + (1-f) tanh(s)], gate_tanh_step )
//      split H' into (hi, lo), write the fragment to LDS, start the next step's
//      contraction with the own tile; one barrier.
//   Y  readout without leaving the step loop.  It contracts over the rows of H,
//      which are spread over lanes here, so the tile is first transposed by an
//      MFMA with an identity operand (exact), then one 16x16x16 MFMA with
//      A = hi of the transposed tile (k = rows) and B = q placed in column
//      (t mod 16) only.  The accumulator is kept for 16 steps, so column s of
//      it collects c sum_i q_i H[i][j] of step s; nothing is read back per step.
//      Every 16 steps the row blocks are summed through LDS and 16 rows of y
//      are stored.
// q, k, v, f for 16 steps at a time are staged through LDS; the next block's
// global loads are in flight while the current block is computed.
#include "m2rnn_kernels.hpp"
#include "m2rnn_mfma_common.hpp"

namespace m2rnn {
namespace {

constexpr int TB = 16;  // steps per staging / readout block (= MFMA N)

template <typename TL>
struct FwdSmem {
  alignas(16) u4_t Hx[2][TL::RB][TL::CT][64];      // (hi, lo) state fragments, one per tile and lane
  alignas(16) float kS[2][TB][TL::ROWS];           // c * k
  alignas(16) _Float16 qS[2][TB][TL::ROWS];
  alignas(16) float vS[2][TB][TL::V];
  alignas(16) float fS[2][TB][4];                  // f, c(1-f), unused, unused
  alignas(16) f4_t yB[TL::RB][TL::CT][64];         // readout accumulators of one block
};

// (Second launch bound: at least two waves per SIMD, i.e. at most 256 registers.  With the
//  512 that a workgroup of 256 threads or fewer may otherwise claim, the compiler puts MFMA
//  results into accumulation registers and copies every one of them out with
//  v_accvgpr_read before the vector ALU can use it: ten extra instructions per step on the
//  step's critical chain.)
template <typename TL, bool DO_Y>
__global__ void __launch_bounds__(TL::THREADS, 2)
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

  // ---- W^T fragments (A operand), in the order the source tiles are used: d = 0 is the
  //      wave's own tile, d > 0 the tile (ct + d) mod CT.  Lane (jl, ig) holds output column
  //      col0 + jl; k-slots 2e, 2e+1 of fragment d both hold W[16 m_d + 4 ig + e][col0 + jl]:
  //      they meet the (hi, lo) pair of that element of the state.
  h8_t wf[CT];
  {
    const bf16_raw *Wn = (const bf16_raw *)a.W + (size_t)n * V * V;
#pragma unroll
    for (int d = 0; d < CT; ++d) {
      const int m = (ct + d) % CT;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int c = 16 * m + 4 * ig + e;
        const _Float16 w = (_Float16)bf16_to_f32(Wn[(size_t)c * V + col0 + jl]);
        wf[d][2 * e] = w;
        wf[d][2 * e + 1] = w;
      }
    }
  }

  // ---- state tile, scaled by c: row rowb + jl, columns col0 + 4 ig + r
  const size_t st_off = (size_t)unit * K * V + (size_t)(row_base + rowb + jl) * V + col0 + 4 * ig;
  float h[4];
  {
    const f4_t h0 = a.H0 ? *(const f4_t *)&a.H0[st_off] : f4_t{0.f, 0.f, 0.f, 0.f};
    if (T == 0) {
      if (a.HT) *(f4_t *)&a.HT[st_off] = h0;
      return;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) h[r] = kC * h0[r];
  }
  // the own tile as the next contraction's B fragment, and that contraction started with it
  const f4_t zero4 = {0.f, 0.f, 0.f, 0.f};
  u4_t own;
#pragma unroll
  for (int r = 0; r < 4; ++r) own[r] = split_hi_lo(h[r]);
  sm.Hx[0][rb][ct][lane] = own;
  f4_t acc_own = mfma_k32(wf[0], __builtin_bit_cast(h8_t, own), zero4);
  // LDS byte offsets of the other tiles' fragments (exchange buffer 0)
  int hx_off[CT];
#pragma unroll
  for (int d = 0; d < CT; ++d) hx_off[d] = ((rb * CT + (ct + d) % CT) * 64 + lane) * 16;
  // identity operand of the transposing MFMA: B[k = 4 ig + r][n = jl] = (k == n)
  h4_t ident;
#pragma unroll
  for (int r = 0; r < 4; ++r) ident[r] = (_Float16)((4 * ig + r == jl) ? 1.f : 0.f);

  // ---- staging of q, k, v, f (TB steps per block)
  bf16_raw rq[NQ], rk[NQ], rv[NV];
  float rf = 1.f;
  // Every thread loads from a valid (clamped) address and nothing is zero-filled: steps past
  // the end of the sequence are staged but never used.  (A load under a condition needs its
  // register cleared first, and the wait in front of that write also waits for the stores
  // in flight.)
  auto stage_load = [&](int t0) {
#pragma unroll
    for (int m = 0; m < NQ; ++m) {
      const int idx = tid + m * THREADS;
      const int s = idx / ROWS, i = idx - s * ROWS;
      const int t = (t0 + s) < T ? (t0 + s) : (T - 1);
      const size_t off = (((size_t)b * T + t) * a.Nqk + g) * K + row_base + i;
      rq[m] = qg[off];
      rk[m] = kg[off];
    }
#pragma unroll
    for (int m = 0; m < NV; ++m) {
      const int idx = tid + m * THREADS;
      const int s = idx / V, j = idx - s * V;
      const int t = (t0 + s) < T ? (t0 + s) : (T - 1);
      rv[m] = vg[(((size_t)b * T + t) * N + n) * V + j];
    }
    {
      const int t = (t0 + (tid & (TB - 1))) < T ? (t0 + (tid & (TB - 1))) : (T - 1);
      rf = fg[((size_t)b * T + t) * N + n];
    }
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
      if (a.gate_alpha) rf = gate_psi(rf, a.gate_alpha[n], a.gate_beta[n]);
      const float gp = kC * (1.f - rf);
      sm.fS[buf][tid][0] = rf;
      sm.fS[buf][tid][1] = gp;
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
    h8_t hf[CT];  // [0] unused: the own tile's product is in acc_own already
    float f, gp, kk;
    f4_t v4, acc;
    h4_t qf;
  };
  auto ckpt_store = [&](int t) __attribute__((always_inline)) {
    if (a.ckpt && t == next_ck) {  // state before step t
      float *dst = a.ckpt + ((size_t)unit * nck + ck_idx) * K * V +
                   (size_t)(row_base + rowb + jl) * V + col0 + 4 * ig;
      *(f4_t *)dst = f4_t{h[0], h[1], h[2], h[3]} * kInvC;
      next_ck += a.C;
      ++ck_idx;
    }
  };
  lchar *const hx = (lchar *)&sm.Hx[0][0][0][0];
  constexpr int HXBUF = RB * CT * 64 * 16;  // bytes of one exchange buffer
  // L: the other tiles' fragments from exchange buffer `buf` and this step's vectors.
  //    Issued right after the barrier that completes the buffer, ahead of the previous
  //    step's readout, so that the readout runs while the fragments are on their way.
  auto step_L = [&](StepRegs &x, int s, int sb, int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int d = 1; d < CT; ++d) x.hf[d] = lds_ld<h8_t>(hx + hx_off[d], buf * HXBUF);
    x.f = sm.fS[sb][s][0];
    x.gp = sm.fS[sb][s][1];
    x.kk = sm.kS[sb][s][rowb + jl];
    x.v4 = *(const f4_t *)&sm.vS[sb][s][col0 + 4 * ig];
    if constexpr (DO_Y) x.qf = *(const h4_t *)&sm.qS[sb][s][rowb + 4 * ig];
  };
  // R: the contraction (the own tile's product was started in the previous step's E)
  auto step_R = [&](StepRegs &x) __attribute__((always_inline)) {
    x.acc = acc_own;
#pragma unroll
    for (int d = 1; d < CT; ++d) x.acc = mfma_k32(wf[d], x.hf[d], x.acc);
    settle(x.acc);
  };
  // E: tanh, gate, split, fragment into exchange buffer `buf`, own-tile product of the next step
  auto step_E = [&](const StepRegs &x, uint32_t (&pk)[4], int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float sp = fmaf(x.kk, x.v4[r], x.acc[r]);
      h[r] = gate_tanh_step(x.f, x.gp, h[r], sp);
      pk[r] = split_hi_lo(h[r]);
    }
    const u4_t fr = {pk[0], pk[1], pk[2], pk[3]};
    if constexpr (CT > 1) lds_st<u4_t>(hx + hx_off[0], buf * HXBUF, fr);
    acc_own = mfma_k32(wf[0], __builtin_bit_cast(h8_t, fr), zero4);
  };
  // Y: readout on the matrix core.  The tile's hi parts are the A operand [m = i][k = j] as
  //    they stand; times the identity gives them back with rows in registers and columns in
  //    lanes (exact: products with 1 and 0).  Then A[m = j][k = i] = hi(H'[i][j]);
  //    B[k = i][n] = q_i for n == s, else 0: column s of yacc collects step s.
  auto step_Y = [&](const StepRegs &x, const uint32_t (&pk)[4], int s, f4_t &yacc)
      __attribute__((always_inline)) {
    const h4_t qf = (jl == s) ? x.qf : zero_h4;
    uint2 hv;
    hv.x = __builtin_amdgcn_perm(pk[1], pk[0], 0x05040100u);
    hv.y = __builtin_amdgcn_perm(pk[3], pk[2], 0x05040100u);
    const f4_t tr = mfma_k16(__builtin_bit_cast(h4_t, hv), ident, zero4);
    const h4_t ht = {(_Float16)tr[0], (_Float16)tr[1], (_Float16)tr[2], (_Float16)tr[3]};
    yacc = mfma_k16(ht, qf, yacc);
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
    //  and vector-ALU work -- was measured 15 % slower at B*N = 128, K = V = 64: the second
    //  barrier costs more than the overlap returns.)
    for (int blk = 0; blk < nblk; ++blk) {
      const int t0 = blk * TB;
      const int len = (T - t0) < TB ? (T - t0) : TB;
      const int sb = blk & 1;
      const bool more = blk + 1 < nblk;
      // Unconditional (the last block fetches itself again): a conditional fetch makes the
      // compiler merge old and new register values at the loop head, and the wait it puts
      // there also waits for the y and checkpoint stores of the block before.
      stage_load(more ? t0 + TB : t0);
      f4_t yacc = {0.f, 0.f, 0.f, 0.f};  // D[m = j][n = s] = c * y partial of step t0 + s
      StepRegs nx;  // operands of the coming step
      step_L(nx, 0, sb, 0);
      auto step = [&](int s, bool last) __attribute__((always_inline)) {
        StepRegs x = nx;
        ckpt_store(t0 + s);
        step_R(x);
        // next block's vectors have landed.  (Also when there is no next block: every path
        // through a block then uses the fetched registers, and the compiler puts no wait for
        // them -- which would also wait for the stores in flight -- at the head of the next.)
        if (s == TB / 2) stage_store(sb ^ 1);
        uint32_t pk[4];
        step_E(x, pk, (s & 1) ^ 1);  // every block but the last has 16 steps: parity of s
        lds_barrier();
        // after the barrier: fetch the next step's operands, then the readout MFMAs
        if (!last) step_L(nx, s + 1, sb, (s + 1) & 1);
        if constexpr (DO_Y) step_Y(x, pk, s, yacc);
      };
      if (len == TB) {
#pragma unroll
        for (int s = 0; s < TB; ++s) step(s, s == TB - 1);
      } else {
#pragma nounroll
        for (int s = 0; s < len; ++s) step(s, s == len - 1);
#pragma unroll
        for (int m = 0; m < NQ; ++m) asm volatile("" : : "v"(rq[m]), "v"(rk[m]));
#pragma unroll
        for (int m = 0; m < NV; ++m) asm volatile("" : : "v"(rv[m]));
        asm volatile("" : : "v"(rf));
      }
      settle(yacc);
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
  if (a.HT) *(f4_t *)&a.HT[st_off] = f4_t{h[0], h[1], h[2], h[3]} * kInvC;
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

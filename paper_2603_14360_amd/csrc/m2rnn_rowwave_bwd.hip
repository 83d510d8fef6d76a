// Register-resident backward scan (Algorithm 2 of the paper, BPTT) for V = 16, the value
// width of the paper's models (state-size appendix: K = 64, V = 16).
//
// With V = 16 a 16-row block of the state is ONE 16 x 16 tile, so one wavefront owns a row
// block with all its columns and the whole backward of that block runs inside the wave: no
// other wave's data is needed per step, hence no workgroup barrier and no LDS exchange on
// the step-to-step chain.  A workgroup is the K/16 waves of one (b, n) state; they share only
// the staged vectors of a chunk and meet at two barriers per chunk.
//
// Per chunk of C <= 16 steps (chunks in reverse order), each wave
//   1. recomputes the chunk forward from its fp32 checkpoint, keeping for every step the fp16
//      state before the step (H'_{t-1} = c H_{t-1}, in wave-private LDS) and Z'_t = c tanh(.)
//      (in registers: the chunk is fully unrolled, 2 registers per step), and accumulating
//      dq_t = H_t dy_t on the matrix core;
//   2. sweeps the chunk in reverse:  G = q dy^T + carry,  dS = (1-f) G (1 - Z^2),
//      carry <- f G + dS W^T,  dW += H_{t-1}^T dS,  dk_t = dS v_t,  dv_t = dS^T k_t,
//      df_t = sum G (H_{t-1} - Z_t).
// Layout: lane (i, g) = (lane % 16, lane / 16) holds row i of the block and columns
// 4 g .. 4 g + 3.  Both contractions over columns are run transposed,
//      (H W)^T = W^T H^T        and        (dS W^T)^T = W dS^T,
// because then the accumulator layout of the 16x16x16 MFMA (lane = n, registers = 4
// consecutive m) IS the layout of its B operand (lane = n, registers = 4 consecutive k): the
// recomputed state and dS go from one step's result to the next step's operand inside the
// registers.  The contractions over rows (dW, dv) need their operands with rows in the
// registers instead; those two tiles (H_{t-1} and dS) take a wave-private trip through LDS,
// written as 8-byte items and read back with the transposing LDS load of gfx950; that trip
// is not on the chain (the next step only needs dS in registers).  The stash of H_{t-1} is
// kept in LDS in that item order (it is read both ways), the stash of Z_t in registers.
// The per-step vectors dq, dk, dv and the scalar df never leave the matrix core during a
// chunk: each is one more MFMA whose other operand (dy_t, v_t, k_t, ones) is placed in row
// or column (t mod 16) only, so a 16 x 16 accumulator collects the chunk's steps.
// Steps beyond the end of a chunk are identity steps (f = 1, zero vectors): the unrolled
// chunk needs no per-step guard, only one test per block of four steps.
#include "m2rnn_kernels.hpp"
#include "m2rnn_mfma_common.hpp"

namespace m2rnn {

// epilogue launchers shared with the tiled backward (m2rnn_mfma_bwd.hip)
hipError_t bwd_sum_dW(const float *dWp, float *dW, int B, int N, int VV, int parts, hipStream_t s);
hipError_t bwd_sum_heads(const float *per_head, void *out, size_t BT, int N, int Nqk, int K,
                         hipStream_t s);
hipError_t bwd_empty(const BwdArgs &a, hipStream_t s);

namespace {

constexpr int CB = 16;  // steps of a chunk buffer = MFMA N: one accumulator row per step

struct RwWs {
  float *dWp;  // [B*N][V][V] per-state dW, summed over the batch by the epilogue
  float *dqh;  // [B,T,N,K] per-head dq (Nqk != N), summed over head groups by the epilogue
  float *dkh;
};

template <int K_>
struct RowWaveB {
  static constexpr int K = K_, V = 16;
  static constexpr int NW = K / 16, THREADS = NW * 64;
  // LDS carve-up (bytes): one chunk's staged vectors, the transposition scratch of every wave,
  // the end-of-chunk partials
  static constexpr int OFF_Q = 0;                       // float q     [CB][K]
  static constexpr int OFF_CK = OFF_Q + CB * K * 4;     // float c k   [CB][K]
  static constexpr int OFF_KH = OFF_CK + CB * K * 4;    // half  k     [CB][K]
  static constexpr int OFF_VH = OFF_KH + CB * K * 2;    // half  v     [CB][V]
  static constexpr int OFF_DY = OFF_VH + CB * V * 2;    // float dy    [CB][V]
  static constexpr int OFF_DYH = OFF_DY + CB * V * 4;   // half  dy scaled per step [CB][V]
  static constexpr int OFF_F = OFF_DYH + CB * V * 2;    // per step: f, c(1-f), 1-f, f16x2 -(1-f)/c^2,
                                                        //           1/(dy scale), 3 pad (8 floats)
  static constexpr int OFF_ZERO = OFF_F + CB * 32;      // 16 zero bytes (masked operand reads)
  static constexpr int OFF_HS = OFF_ZERO + 16;          // [NW][CB][512] stash of H'_{t-1} (fp16 tiles)
  static constexpr int OFF_TR = OFF_HS + NW * CB * 512; // [NW][512] transposition scratch of dS
  static constexpr int OFF_PV = OFF_TR + NW * 512;      // [NW][64] f4: dv (at the end dW) partials
  static constexpr int OFF_PF = OFF_PV + NW * 1024;     // [NW][16] float: df partials
  static constexpr int BYTES = OFF_PF + NW * 64;
  // (K = 64, the paper's shape: three workgroups per CU)
  static_assert(BYTES <= kLdsLimit && (K > 64 || 3 * BYTES <= kLdsLimit), "LDS layout");
};

__device__ __forceinline__ h4_t lds_tr16(const lchar *p, int off) {
  typedef short s4_t __attribute__((ext_vector_type(4)));
  const s4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s4_t *)(p + off));
  return __builtin_bit_cast(h4_t, v);
}

__device__ __forceinline__ h4_t cvt4_f16(const float (&x)[4]) {
  typedef float f2_t __attribute__((ext_vector_type(2)));
  const f2_t a01 = {x[0], x[1]}, a23 = {x[2], x[3]};
  uint2 p;
  p.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(a01, h2_t));
  p.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(a23, h2_t));
  return __builtin_bit_cast(h4_t, p);
}

template <typename RW, bool CLIP>
__global__ void __launch_bounds__(RW::THREADS, 3) rowwave_bwd_kernel(BwdArgs a, RwWs ws) {
  constexpr int K = RW::K, V = 16, NW = RW::NW, THREADS = RW::THREADS;
  constexpr int RL = K / 8;       // 16-byte items (8 bf16) per step of q or k
  constexpr int QI = CB * RL;     // items per chunk of q (and of k): 2 K = THREADS / 2
  static_assert(2 * QI == THREADS, "one q or k item per thread");
  const int unit = blockIdx.x;
  const int T = a.T, N = a.N, C = a.C;
  const int b = unit / N, n = unit - b * N;
  const int g = n / (N / a.Nqk);
  const int tid = threadIdx.x, lane = tid & 63;
  const int rb = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: one row block per wave
  const int jl = lane & 15, ig = lane >> 4;
  const int row = rb * 16 + jl;  // state row of this lane

  extern __shared__ __attribute__((aligned(16))) char lds[];
  lchar *const l0 = (lchar *)lds;
  float *qS = (float *)(lds + RW::OFF_Q);
  float *ckS = (float *)(lds + RW::OFF_CK);
  _Float16 *kH = (_Float16 *)(lds + RW::OFF_KH);
  _Float16 *vH = (_Float16 *)(lds + RW::OFF_VH);
  float *dyS = (float *)(lds + RW::OFF_DY);
  _Float16 *dyH = (_Float16 *)(lds + RW::OFF_DYH);
  float *fS = (float *)(lds + RW::OFF_F);
  f4_t *pv = (f4_t *)(lds + RW::OFF_PV);
  float *pf = (float *)(lds + RW::OFF_PF);
  if (tid < 4) ((uint32_t *)(lds + RW::OFF_ZERO))[tid] = 0u;  // visible after the first barrier

  const bf16_raw *__restrict__ qg = (const bf16_raw *)a.q;
  const bf16_raw *__restrict__ kg = (const bf16_raw *)a.k;
  const bf16_raw *__restrict__ vg = (const bf16_raw *)a.v;
  const bf16_raw *__restrict__ dyg = (const bf16_raw *)a.dy;
  const float *__restrict__ fg = a.f;
  const float g_alpha = a.gate_alpha ? a.gate_alpha[n] : 0.f, g_beta = a.gate_alpha ? a.gate_beta[n] : 0.f;

  // ---- W fragments (A operands).  Recompute:  S^T[j'][i] = sum_j W[j][j'] H[i][j]  -> A[m = j'][k = j]
  //      = W[j][j'];  carry:  (dS W^T)^T[j'][i] = sum_j W[j'][j] dS[i][j]  -> A[m = j'][k = j] = W[j'][j].
  //      Lane (m, k-group) = (jl, ig) holds k = 4 ig + e.
  //      The recomputed state enters its contraction as an fp16 pair (hi, lo), as in the
  //      forward kernels (16x16x32 MFMA, the pair in adjacent k-slots against a fragment that
  //      holds each row of W twice): a recurrence that expands (transition gain above one)
  //      amplifies the operand's rounding inside a chunk, 1.4^16 at gain 3.
  h8_t wfT;
  h4_t wfW;
  {
    const bf16_raw *Wn = (const bf16_raw *)a.W + (size_t)n * V * V;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const _Float16 w = (_Float16)bf16_to_f32(Wn[(size_t)(4 * ig + e) * V + jl]);
      wfT[2 * e] = w;
      wfT[2 * e + 1] = w;
      wfW[e] = (_Float16)bf16_to_f32(Wn[(size_t)jl * V + 4 * ig + e]);
    }
  }
  const h4_t zero_h4 = {(_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f};
  const f4_t zero4 = {0.f, 0.f, 0.f, 0.f};

  const size_t st_off = (size_t)unit * K * V + (size_t)row * V + 4 * ig;  // this lane's 4 state elements
  const int nck = (T + C - 1) / C;

  // ---- staging: the next chunk's vectors travel during the current chunk
  u4_t rqk, rvd;       // a q item (tid < QI) or a k item; a v item (tid < 32) or a dy item (32 <= tid < 64)
  float rf = 1.f;      // f of step tid (tid < 16)
  f4_t hck;            // this lane's part of the chunk's checkpoint
  const uint32_t kstride = (uint32_t)a.Nqk * K, vstride = (uint32_t)N * V;
  const bf16_raw *const qbase = qg + ((size_t)b * T * a.Nqk + g) * K;
  const bf16_raw *const kbase = kg + ((size_t)b * T * a.Nqk + g) * K;
  const bf16_raw *const vbase = vg + ((size_t)b * T * N + n) * V;
  const bf16_raw *const dybase = dyg + ((size_t)b * T * N + n) * V;
  const float *const fbase = fg + (size_t)b * T * N + n;
  const u4_t zero_u4 = {0u, 0u, 0u, 0u};
  // Every thread loads, from addresses clamped to the chunk (steps beyond its end are
  // masked when the values are stored to LDS): a load under a condition makes the compiler
  // merge the old and the new register value right behind the load, which waits for it.
  auto stage_load = [&](int ck) {
    const int t0 = ck * C;
    const int last = ((T - t0) < C ? (T - t0) : C) - 1;
    {
      const bool isq = tid < QI;
      const int e = isq ? tid : tid - QI, s0 = e / RL, p = e - s0 * RL;
      const int s = s0 < last ? s0 : last;
      rqk = *(const u4_t *)((isq ? qbase : kbase) + (size_t)(t0 + s) * kstride + 8 * p);
    }
    {
      const bool isv = (tid & 32) == 0;  // (only wave 0's copies are used)
      const int e = tid & 31, s0 = e >> 1, p = e & 1;
      const int s = s0 < last ? s0 : last;
      rvd = *(const u4_t *)((isv ? vbase : dybase) + (size_t)(t0 + s) * vstride + 8 * p);
    }
    {
      const int s0 = tid & (CB - 1);
      rf = fbase[(size_t)(t0 + (s0 < last ? s0 : last)) * N];
    }
    hck = *(const f4_t *)(a.ckpt + ((size_t)unit * nck + ck) * K * V + (size_t)row * V + 4 * ig);
  };
  auto stage_wait = [&]() {  // (pins the point where the loads are waited for)
    asm volatile("" : "+v"(rqk), "+v"(rvd), "+v"(rf), "+v"(hck));
  };
  auto stage_store = [&](int len) {
    float x[8];
    {
      const int e = tid < QI ? tid : tid - QI;
      bf16x8_to_f32(e / RL < len ? rqk : zero_u4, x);
    }
    if (tid < QI) {
      *(f4_t *)&qS[8 * tid] = f4_t{x[0], x[1], x[2], x[3]};
      *(f4_t *)&qS[8 * tid + 4] = f4_t{x[4], x[5], x[6], x[7]};
    } else {
      const int e = tid - QI;
      *(f4_t *)&ckS[8 * e] = f4_t{x[0], x[1], x[2], x[3]} * kC;
      *(f4_t *)&ckS[8 * e + 4] = f4_t{x[4], x[5], x[6], x[7]} * kC;
      h8_t hv;
#pragma unroll
      for (int i = 0; i < 8; ++i) hv[i] = (_Float16)x[i];
      *(h8_t *)&kH[8 * e] = hv;
    }
    if (tid < 64) {  // (wave 0: uniform)
      const int e = tid & 31;
      bf16x8_to_f32((e >> 1) < len ? rvd : zero_u4, x);
      // dy_s enters the dq contraction as fp16: each step's row is scaled by a power of two so
      // that its largest entry lands in [2^10, 2^11); column s of dq is scaled back at the end.
      // A row is held by two adjacent lanes, 8 values each.
      float mx = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) mx = fmaxf(mx, fabsf(x[i]));
      const int ex = ilog2f(fminf(fmaxf(group_max_nonneg<2>(mx), 1e-30f), 1e30f));
      const float up = pow2i(10 - ex);
      h8_t hv, hs;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        hv[i] = (_Float16)x[i];
        hs[i] = (_Float16)(x[i] * up);
      }
      if (tid < 32) {
        *(h8_t *)&vH[8 * e] = hv;
      } else {
        *(f4_t *)&dyS[8 * e] = f4_t{x[0], x[1], x[2], x[3]};
        *(f4_t *)&dyS[8 * e + 4] = f4_t{x[4], x[5], x[6], x[7]};
        *(h8_t *)&dyH[8 * e] = hs;
        if ((e & 1) == 0) fS[(e >> 1) * 8 + 4] = pow2i(ex - 10);
      }
      if (tid < CB) {
        if (a.gate_alpha) rf = gate_psi(rf, g_alpha, g_beta);
        if (tid >= len) rf = 1.f;  // identity step
        const float gm = 1.f - rf;
        const h2_t m2 = {(_Float16)(gm * (-kInvC * kInvC)), (_Float16)(gm * (-kInvC * kInvC))};
        fS[tid * 8 + 0] = rf;
        fS[tid * 8 + 1] = kC * gm;
        fS[tid * 8 + 2] = gm;
        fS[tid * 8 + 3] = __builtin_bit_cast(float, m2);
      }
    }
  };

  // ---- sweep state
  float carry[4];
  {
    f4_t x = zero4;
    if (a.dHT) x = *(const f4_t *)&a.dHT[st_off];
#pragma unroll
    for (int r = 0; r < 4; ++r) carry[r] = x[r];
  }
  f4_t dWacc = zero4;
  // Dynamic range of the fp16 dS operand: the sweep works on sc * (carry, G, dS and every
  // accumulator fed by dS), sc a power of two chosen per chunk and per wave from the largest
  // |carry| of the row block and the largest |q| |dy| of the chunk, so that the scaled values
  // start the chunk in [2^5, 2^6); where the previous chunk grew by g > 2 bits the start is
  // lowered by g - 2 bits more (at most 12).  sc never exceeds 2^90 times the smallest scale
  // used so far (the dW accumulator is rescaled with sc and would overflow for a gradient that
  // has died away).  Powers of two keep all of this exact.
  float sc = 1.f, isc = 1.f;
  int sc_e = 0, sc_e_min = 1 << 20, mx_e_prev = -(1 << 20);

  // wave-private transposition scratch: a tile is written as 8-byte items (row i, columns
  // 4 g ..); the transposing load, in which lane d of lane group G addresses item (row
  // 4 G + d / 4, column group d % 4), returns lane % 16 = column and registers = rows
  // 4 (lane / 16) .. + 3
  // Where the items sit is free (every lane of the transposing load supplies its own address),
  // so item (row i, column group g) is placed at slot 16 g + (i + 4 g) mod 16: the 64 items a
  // wave writes (lane = (i, g)) and the 16 items a lane group of the transposing load
  // addresses (rows 4 G .. 4 G + 3, all four column groups) then both spread evenly over the
  // LDS banks.  (Slot 4 i + g, the plain order, made the writes 4-way bank conflicts: 40 % of
  // the LDS-active cycles in the counters.)
  const int slot_w = 16 * ig + ((jl + 4 * ig) & 15);                   // my own item
  const int gs = jl & 3, is = 4 * ig + (jl >> 2);                      // the item I address when
  const int slot_r = 16 * gs + ((is + 4 * gs) & 15);                   // reading transposed
  lchar *const trw = l0 + RW::OFF_TR + rb * 512 + slot_w * 8;
  const lchar *const trr = l0 + RW::OFF_TR + rb * 512 + slot_r * 8;
  // the stash of H'_{t-1} lives in LDS in the same item order: the sweep reads a step's tile
  // both ways, as written (own elements) and transposed (operand of dW)
  lchar *const hsw = l0 + RW::OFF_HS + rb * CB * 512 + slot_w * 8;
  const lchar *const hsr = l0 + RW::OFF_HS + rb * CB * 512 + slot_r * 8;

  if (nck > 0) stage_load(nck - 1);
  stage_wait();
  for (int it = 0; it < nck; ++it) {
    const int ck = nck - 1 - it;
    const int t0 = ck * C;
    const int len = (T - t0) < C ? (T - t0) : C;
    stage_store(len);
    float h[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) h[r] = kC * hck[r];
    lds_barrier();  // the chunk's staged vectors are complete
    stage_load(ck > 0 ? ck - 1 : 0);  // unconditional (a conditional prefetch makes the compiler
                                       // merge old and new register values behind the loads)

    // ---- scale of this chunk
    {
      float mq = 0.f;
#pragma unroll
      for (int s = 0; s < CB; ++s) mq = fmaxf(mq, fabsf(qS[s * K + row]));
      const f4_t d4 = *(const f4_t *)&dyS[4 * lane];
      float md = fmaxf(fmaxf(fabsf(d4[0]), fabsf(d4[1])), fmaxf(fabsf(d4[2]), fabsf(d4[3])));
      float mc = fmaxf(fmaxf(fabsf(carry[0]), fabsf(carry[1])), fmaxf(fabsf(carry[2]), fabsf(carry[3])));
      mq = group_max_nonneg<64>(mq);
      md = group_max_nonneg<64>(md);
      mc = group_max_nonneg<64>(mc) * isc;
      const int e = ilog2f(fminf(fmaxf(mc + mq * md, 1e-30f), 1e30f));
      const int grew = mx_e_prev > -(1 << 20) ? e - mx_e_prev : 0;
      const int extra = grew - 2 < 0 ? 0 : (grew - 2 > 12 ? 12 : grew - 2);
      int ne = 5 - extra - e;
      ne = ne > sc_e_min + 90 ? sc_e_min + 90 : ne;
      ne = ne < sc_e - 120 ? sc_e - 120 : ne;
      ne = ne > 120 ? 120 : (ne < -120 ? -120 : ne);
      sc_e_min = ne < sc_e_min ? ne : sc_e_min;
      mx_e_prev = e;
      const float ratio = pow2i(ne - sc_e);
      sc_e = ne;
      sc = pow2i(ne);
      isc = pow2i(-ne);
#pragma unroll
      for (int r = 0; r < 4; ++r) carry[r] *= ratio;
      dWacc *= ratio;
    }

    // LDS addressing: a few per-lane base offsets, made opaque once per chunk so that they are
    // not hoisted out of the chunk loop as one register per (array, step); every access below
    // is base + compile-time immediate.  The lane's column index is opaque as well: the
    // per-step masks (jl == s) are then built per step instead of being kept for every s.
    lchar *bRow4 = l0 + row * 4;            // q, c k (fp32) of this lane's row
    lchar *bRow2 = l0 + (rb * 16 + 4 * ig) * 2;  // k (fp16) rows 4 ig .. of the block
    lchar *bCol2 = l0 + 4 * ig * 2;         // v, dy (fp16) columns 4 ig ..
    lchar *bCol4 = l0 + 4 * ig * 4;         // dy (fp32) columns 4 ig ..
    lchar *bZero = l0;                      // wave-uniform reads (f), the zero pad
    int jlo = jl;
    asm volatile("" : "+v"(bRow4), "+v"(bRow2), "+v"(bCol2), "+v"(bCol4), "+v"(bZero), "+v"(jlo));

    // ---- 1. recompute the chunk; the stash stays in registers
    h4_t zpS[CB];
    f4_t dqacc = zero4;
    h4_t hcur = cvt4_f16(h);
#pragma unroll
    for (int blk = 0; blk < CB / 4; ++blk) {
      if (4 * blk < len) {
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
          const int s = 4 * blk + s4;
          const u2_t fg2 = lds_ld<u2_t>(bZero, RW::OFF_F + s * 32);
          const float f = __builtin_bit_cast(float, (uint32_t)fg2.x), gp = __builtin_bit_cast(float, (uint32_t)fg2.y);
          const float m2g = -2.f * gp;
          const float cki = lds_ld<float>(bRow4, RW::OFF_CK + s * K * 4);
          const h4_t v4 = lds_ld<h4_t>(bCol2, RW::OFF_VH + s * V * 2);
          lds_st<h4_t>(hsw, s * 512, hcur);
          u4_t pk;
#pragma unroll
          for (int r = 0; r < 4; ++r) pk[r] = split_hi_lo(h[r]);
          const f4_t acc = mfma_k32(wfT, __builtin_bit_cast(h8_t, pk), zero4);
          float z[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const float t1 = fmaf(f, h[r], gp);
            const float sp = fmaf(cki, (float)v4[r], acc[r]);
            const float e = __builtin_amdgcn_exp2f(sp);
            const float rr = __builtin_amdgcn_rcpf(1.f + e);
            z[r] = fmaf(-2.f * kC, rr, kC);
            h[r] = fmaf(m2g, rr, t1);
          }
          zpS[s] = cvt4_f16(z);
          hcur = cvt4_f16(h);
          // dq_s = H_s dy_s: A[m = s][k = j] = dy_j (row s only), B[k = j][n = i] = H_s
          const h4_t dyf = lds_ld<h4_t>(jlo == s ? bCol2 + (RW::OFF_DYH + s * V * 2) : bZero + RW::OFF_ZERO, 0);
          dqacc = mfma_k16(dyf, hcur, dqacc);
        }
        settle(dqacc);
      }
    }

    // ---- 2. sweep in reverse
    f4_t dkacc = zero4, dvacc = zero4, dfacc = zero4;
#pragma unroll
    for (int blk = CB / 4 - 1; blk >= 0; --blk) {
      if (4 * blk < len) {
#pragma unroll
        for (int s4 = 3; s4 >= 0; --s4) {
          const int s = 4 * blk + s4;
          const f4_t fu = lds_ld<f4_t>(bZero, RW::OFF_F + s * 32);
          const float f = fu[0], gm = fu[2];
          const float m4f = fu[3];  // (element first, cast second)
          const uint32_t m4w = __builtin_bit_cast(uint32_t, m4f);
          const u2_t m4u = {m4w, m4w};
          const h4_t m4 = __builtin_bit_cast(h4_t, m4u);
          const float qs = sc * lds_ld<float>(bRow4, RW::OFF_Q + s * K * 4);
          const f4_t dy4 = lds_ld<f4_t>(bCol4, RW::OFF_DY + s * V * 4);
          const h4_t zp = zpS[s];
          const h4_t hown = lds_ld<h4_t>(hsw, s * 512);
          const h4_t hT = lds_tr16(hsr, s * 512);
          const bool mine = jlo == s;
          const h4_t vfr = lds_ld<h4_t>(mine ? bCol2 + (RW::OFF_VH + s * V * 2) : bZero + RW::OFF_ZERO, 0);
          const h4_t kfr = lds_ld<h4_t>(mine ? bRow2 + (RW::OFF_KH + s * K * 2) : bZero + RW::OFF_ZERO, 0);
          // H' - Z' and w = (1-f) Z^2 in packed fp16;  dS = (1-f) G - G w  with the leading term
          // in fp32 and one mixed-precision FMA rounding the sum to the fp16 operand
          const h4_t hz = hown - zp;
          const h4_t ug = (zp * m4) * zp;  // = -w
          float G[4];
          float dfl = 0.f;
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            G[r] = fmaf(qs, dy4[r], carry[r]);
            dfl = fmaf(G[r], (float)hz[r], dfl);
          }
          uint2 dsu;
          {
            const uint2 ugu = __builtin_bit_cast(uint2, ug);
            const float g0 = gm * G[0], g1 = gm * G[1], g2 = gm * G[2], g3 = gm * G[3];
            asm("v_fma_mixlo_f16 %0, %1, %2, %3 op_sel_hi:[0,1,0]"
                : "=v"(dsu.x) : "v"(G[0]), "v"(ugu.x), "v"(g0));
            asm("v_fma_mixhi_f16 %0, %1, %2, %3 op_sel:[0,1,0] op_sel_hi:[0,1,0]"
                : "+v"(dsu.x) : "v"(G[1]), "v"(ugu.x), "v"(g1));
            asm("v_fma_mixlo_f16 %0, %1, %2, %3 op_sel_hi:[0,1,0]"
                : "=v"(dsu.y) : "v"(G[2]), "v"(ugu.y), "v"(g2));
            asm("v_fma_mixhi_f16 %0, %1, %2, %3 op_sel:[0,1,0] op_sel_hi:[0,1,0]"
                : "+v"(dsu.y) : "v"(G[3]), "v"(ugu.y), "v"(g3));
            // The next instruction to read dS is an MFMA.  The compiler does not count wait
            // states behind inline assembly, and without them the matrix core reads the
            // register pair before the two high halves have landed (seen as a carry built
            // from half of dS).
            asm volatile("s_nop 3" : "+v"(dsu.x), "+v"(dsu.y));
          }
          const h4_t dsp = __builtin_bit_cast(h4_t, dsu);
          // chain: carry <- f G + W dS^T
          const f4_t d = mfma_k16(wfW, dsp, zero4);
          // off the chain: the two tiles with rows in the registers, for dW and dv
          lds_st<h4_t>(trw, 0, dsp);
          const h4_t dT = lds_tr16(trr, 0);
          // dk_s = dS v_s: A[m = s][k = j] = v_j (row s only), B[k = j][n = i] = dS
          dkacc = mfma_k16(vfr, dsp, dkacc);
#pragma unroll
          for (int r = 0; r < 4; ++r) carry[r] = fmaf(f, G[r], d[r]);
          if constexpr (CLIP) {
            // (an identity step beyond the end of the chunk must not clamp: dH_T is used as given)
            const float cb = s < len ? a.clip * sc : __builtin_inff();
#pragma unroll
            for (int r = 0; r < 4; ++r) carry[r] = __builtin_amdgcn_fmed3f(carry[r], -cb, cb);
          }
          // dW' += H'^T dS: A[m = j1][k = i] = H'[i][j1], B[k = i][n = j2] = dS[i][j2]
          dWacc = mfma_k16(hT, dT, dWacc);
          // dv_s = dS^T k_s: A[m = s][k = i] = k_i (row s only), B[k = i][n = j] = dS
          dvacc = mfma_k16(kfr, dT, dvacc);
          // df_s = sum G (H' - Z') / c: the fp32 MFMA against ones in column s adds the four lane
          // groups; the 16 rows of that column are added at the end of the chunk
          dfacc = __builtin_amdgcn_mfma_f32_16x16x4f32(dfl, mine ? 1.f : 0.f, dfacc, 0, 0, 0);
        }
        settle(dkacc);
        settle(dvacc);
        settle(dfacc);
        settle(dWacc);
      }
    }

    // ---- 3. end of the chunk.  The next chunk's prefetch is waited for here, in front of the
    //         stores (the vector-memory counter is in order: behind them the wait would also
    //         wait for the stores to reach memory).
    stage_wait();
    // dq, dk: accumulator [m = step][n = row]: lane (jl, ig) holds row jl, steps 4 ig + r
    {
      float dyb[4];  // scale-back of dq per step
#pragma unroll
      for (int r = 0; r < 4; ++r) dyb[r] = fS[(4 * ig + r) * 8 + 4] * kInvC;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int st = 4 * ig + r;
        if (st < len) {
          const float xq = dqacc[r] * dyb[r], xk = dkacc[r] * isc;
          if (ws.dqh) {
            const size_t o = (((size_t)b * T + t0 + st) * N + n) * K + row;
            ws.dqh[o] = xq;
            ws.dkh[o] = xk;
          } else {
            const size_t o = (((size_t)b * T + t0 + st) * a.Nqk + g) * K + row;
            ((bf16_raw *)a.dq)[o] = f32_to_bf16(xq);
            ((bf16_raw *)a.dk)[o] = f32_to_bf16(xk);
          }
        }
      }
    }
    // dv, df: partials of the row blocks meet in LDS
    pv[rb * 64 + lane] = dvacc * isc;
    {
      float x = (dfacc[0] + dfacc[1]) + (dfacc[2] + dfacc[3]);
      x += __shfl_xor(x, 16, 64);
      x += __shfl_xor(x, 32, 64);
      if (lane < 16) pf[rb * 16 + lane] = x * (kInvC * isc);
    }
    // (wave 0 finishes dv: what it needs of the staged dy is read in front of the barrier,
    //  behind it the other waves may already stage the next chunk)
    float dyr[4] = {0.f, 0.f, 0.f, 0.f};
    if (rb == 0 && a.w_r) {
#pragma unroll
      for (int r = 0; r < 4; ++r) dyr[r] = dyS[(4 * ig + r) * V + jl];
    }
    lds_barrier();  // partials complete; every wave is done with the staged vectors
    if (rb == 0) {
      // dv: accumulator [m = step][n = column]: lane (jl, ig) holds column jl, steps 4 ig + r
      f4_t d = pv[lane];
#pragma unroll
      for (int w = 1; w < NW; ++w) d += pv[w * 64 + lane];
      float wr = 0.f;
      if (a.w_r) wr = bf16_to_f32(((const bf16_raw *)a.w_r)[n * V + jl]);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int st = 4 * ig + r;
        if (st < len) {
          const float x = fmaf(wr, dyr[r], d[r]);  // y_t holds w_r (.) v_t as well
          ((bf16_raw *)a.dv)[(((size_t)b * T + t0 + st) * N + n) * V + jl] = f32_to_bf16(x);
        }
      }
      if (lane < len) {
        float x = pf[lane];
#pragma unroll
        for (int w = 1; w < NW; ++w) x += pf[w * 16 + lane];
        a.df[((size_t)b * T + t0 + lane) * N + n] = x;
      }
    }
    // (the next chunk's partials are written behind its first barrier: no barrier needed here)
  }

  // ---- outputs of the whole sweep
  if (a.dH0) *(f4_t *)&a.dH0[st_off] = f4_t{carry[0], carry[1], carry[2], carry[3]} * isc;
  lds_barrier();  // wave 0 is done with the last chunk's partials
  pv[rb * 64 + lane] = dWacc * (kInvC * isc);
  lds_barrier();
  if (rb == 0) {
    // dW: accumulator [m = j1][n = j2]: lane (jl, ig) holds dW[4 ig + r][jl]
    f4_t d = pv[lane];
#pragma unroll
    for (int w = 1; w < NW; ++w) d += pv[w * 64 + lane];
    float *dst = ws.dWp + (size_t)unit * V * V;
#pragma unroll
    for (int r = 0; r < 4; ++r) dst[(4 * ig + r) * V + jl] = d[r];
  }
}

template <int K_>
hipError_t launch(const BwdArgs &a, hipStream_t s) {
  using RW = RowWaveB<K_>;
  if (a.T == 0) return bwd_empty(a, s);
  const int units = a.B * a.N;
  RwWs ws;
  size_t off = 0;
  ws.dWp = (float *)(a.ws + off);
  off += align256((size_t)units * 16 * 16 * 4);
  const bool shared = a.Nqk != a.N;
  const size_t heads = shared ? align256((size_t)a.B * a.T * a.N * a.K * 4) : 0;
  ws.dqh = shared ? (float *)(a.ws + off) : nullptr;
  off += heads;
  ws.dkh = shared ? (float *)(a.ws + off) : nullptr;
  hipError_t e;
  if (units > 0) {
    if (a.C > CB) return hipErrorInvalidValue;
    auto go = [&](auto kernel) {
      hipError_t e2 = set_max_lds_once(kernel, RW::BYTES);
      if (e2 != hipSuccess) return e2;
      hipLaunchKernelGGL(kernel, dim3(units), dim3(RW::THREADS), RW::BYTES, s, a, ws);
      return hipGetLastError();
    };
    e = a.clip > 0.f ? go(rowwave_bwd_kernel<RW, true>) : go(rowwave_bwd_kernel<RW, false>);
    if (e != hipSuccess) return e;
    if (shared) {
      const size_t BT = (size_t)a.B * a.T;
      if ((e = bwd_sum_heads(ws.dqh, a.dq, BT, a.N, a.Nqk, a.K, s)) != hipSuccess) return e;
      if ((e = bwd_sum_heads(ws.dkh, a.dk, BT, a.N, a.Nqk, a.K, s)) != hipSuccess) return e;
    }
  }
  return bwd_sum_dW(ws.dWp, a.dW, a.B, a.N, 16 * 16, 1, s);
}

}  // namespace

// (K, V) shapes of the register-resident backward
#define M2RNN_ROWWAVE_BWD_CASES(X) X(16) X(32) X(64) X(128)

bool rowwave_bwd_supported(int K, int V) {
  if (V != 16) return false;
#define X(K_) \
  if (K == K_) return true;
  M2RNN_ROWWAVE_BWD_CASES(X)
#undef X
  return false;
}

hipError_t rowwave_bwd(const BwdArgs &a, hipStream_t s) {
#define X(K_) \
  if (a.K == K_ && a.V == 16) return launch<K_>(a, s);
  M2RNN_ROWWAVE_BWD_CASES(X)
#undef X
  return hipErrorInvalidValue;
}

size_t rowwave_bwd_workspace_bytes(int B, int T, int N, int Nqk, int K, int V) {
  (void)V;
  const size_t heads = Nqk != N ? align256((size_t)B * T * N * K * 4) : 0;
  return align256((size_t)B * N * 16 * 16 * 4) + 2 * heads;
}

int rowwave_bwd_max_chunk() { return CB; }

}  // namespace m2rnn

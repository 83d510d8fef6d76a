// Matrix-core backward scan (Algorithm 2 of the paper, BPTT), with the carried
// state gradient added to q dy^T and propagated as  f G + dS W^T.
//
// The paper's kernel stores every H_t to HBM in a first pass and reloads it in
// the reverse sweep.  Here the forward leaves one fp32 checkpoint every C steps;
// the backward walks the chunks from last to first and, per chunk,
//   phase A  recomputes the chunk forward from its checkpoint, parking for every
//            step the fp16 state before the step (H'_{t-1} = c H_{t-1}) and
//            Z'_t = c tanh(.) in an on-chip stash (LDS), and produces
//            dq_t = H_t dy_t as one more column of the state contraction;
//   phase B  sweeps the chunk in reverse, reading the stash: no tanh and no
//            state contraction are recomputed there.
// Per step of phase B and wavefront (16 x 16 tile, lane = 4 rows x 1 column):
//   G  = q_i dy_j + Ccarry                       (dL/dH_t)
//   df += G (H'_{t-1} - Z'_t) / c                (wave + workgroup reduction)
//   dS = (1-f) G (1 - Z^2)                       -> fp16, to LDS (row-major)
//   dW' += H'_{t-1}^T dS       MFMA k = rows     (A = stash tiles, B = own dS)
//   dv  = dS^T k               MFMA k = rows     (A = k broadcast)
//   Ccarry = f G + dS W^T      MFMA k = columns  (A = dS rows from LDS, B = W^T)
//   dk  = dS v                 one more column of that contraction
// Row-block partials of dv, df, dW are combined in fixed order (LDS, then the
// epilogue kernels); nothing uses atomics.
#include "m2rnn_kernels.hpp"
#include "m2rnn_mfma_common.hpp"

namespace m2rnn {
namespace {

constexpr int kChunkCap = 16;

template <typename TL>
struct BwdLds {
  static constexpr int ROWS = TL::ROWS, V = TL::V, LDH = TL::LDH, RB = TL::RB, CT = TL::CT,
                       WAVES = TL::WAVES;
  static constexpr int X_BYTES = 2 * ROWS * LDH * 2;      // exchange (state in A, dS in B)
  static constexpr int STASH_STEP = RB * CT * 64 * 8;     // one h4 per lane per tile
  static constexpr int VEC_STEP = ROWS * (4 + 4 + 2) + V * (4 + 4 + 2 + 2) + 16;
  static constexpr int PER_STEP = 2 * STASH_STEP + VEC_STEP;
  static constexpr int PART_BYTES = 2 * RB * V * 4 + 2 * WAVES * 4 * 4;
  static constexpr int FIXED = X_BYTES + PART_BYTES;
  static constexpr int CMAX_RAW = (kLdsLimit - FIXED - 64) / PER_STEP;
  static constexpr int CMAX = CMAX_RAW > kChunkCap ? kChunkCap : CMAX_RAW;
  static_assert(CMAX >= 1, "no room for a stash");
  // byte offsets for a stash of CMAX steps
  static constexpr int X = 0;
  static constexpr int SH = X + X_BYTES;
  static constexpr int SZ = SH + CMAX * STASH_STEP;
  static constexpr int KS_ = SZ + CMAX * STASH_STEP;      // float c*k   [C][ROWS]
  static constexpr int QS_ = KS_ + CMAX * ROWS * 4;       // float q     [C][ROWS]
  static constexpr int VS_ = QS_ + CMAX * ROWS * 4;       // float v     [C][V]
  static constexpr int DYS_ = VS_ + CMAX * V * 4;         // float dy    [C][V]
  static constexpr int KH_ = DYS_ + CMAX * V * 4;         // half k      [C][ROWS]
  static constexpr int VH_ = KH_ + CMAX * ROWS * 2;       // half v      [C][V]
  static constexpr int DYH_ = VH_ + CMAX * V * 2;         // half dy     [C][V]
  static constexpr int FS_ = DYH_ + CMAX * V * 2;         // float f, c(1-f), 1-f, -2c(1-f) [C][4]
  static constexpr int DVP_ = FS_ + CMAX * 16;            // float [2][RB][V]
  static constexpr int DFP_ = DVP_ + 2 * RB * V * 4;      // float [2][WAVES*4]
  static constexpr int BYTES = DFP_ + 2 * WAVES * 4 * 4;
  static_assert(BYTES <= kLdsLimit, "LDS overflow");
};

// sum over the 16 lanes of each DPP row; every lane of the row gets the total
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float row16_sum(float x) {
  x += dpp_move<0xB1>(x);   // quad_perm [1,0,3,2]
  x += dpp_move<0x4E>(x);   // quad_perm [2,3,0,1]
  x += dpp_move<0x141>(x);  // row_half_mirror
  x += dpp_move<0x140>(x);  // row_mirror
  return x;
}

struct BwdWs {
  float *dvp;   // [P][B,T,N,V]      (P > 1)
  float *dfp;   // [P][B,T,N]        (P > 1)
  float *dWp;   // [B*N][P*RB][V][V]
  float *dqh;   // [B,T,N,K]         (Nqk != N)
  float *dkh;
};

template <typename TL>
__global__ void __launch_bounds__(TL::THREADS) mfma_bwd_kernel(BwdArgs a, BwdWs ws) {
  constexpr int K = TL::K, V = TL::V, RB = TL::RB, CT = TL::CT, ROWS = TL::ROWS, KS = TL::KS,
                LDH = TL::LDH, WAVES = TL::WAVES;
  constexpr int THREADS = TL::THREADS;
  constexpr bool X32 = TL::X32;
  constexpr int FE = X32 ? 8 : 4;
  using FragT = typename Frag<X32>::type;
  using L = BwdLds<TL>;
  constexpr int CMAX = L::CMAX;
  constexpr int NQ = (CMAX * ROWS + THREADS - 1) / THREADS;
  constexpr int NV = (CMAX * V + THREADS - 1) / THREADS;

  int unit, part;
  if (!map_block<TL::P>(a.B * a.N, unit, part)) return;
  const int T = a.T, N = a.N, C = a.C;
  const int b = unit / N, n = unit - b * N;
  const int g = n / (N / a.Nqk);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rb = wave / CT, ct = wave - rb * CT;
  const int jl = lane & 15, ig = lane >> 4;
  const int col0 = ct * 16, rowb = rb * 16;
  const int row_base = part * ROWS;

  extern __shared__ __attribute__((aligned(16))) char lds[];
  typedef _Float16 XRow[LDH];
  XRow *Xb = (XRow *)(lds + L::X);                  // [2*ROWS][LDH]
  h4_t *stH = (h4_t *)(lds + L::SH);                // [C][RB][CT][64]
  h4_t *stZ = (h4_t *)(lds + L::SZ);
  float *kS = (float *)(lds + L::KS_);
  float *qS = (float *)(lds + L::QS_);
  float *vS = (float *)(lds + L::VS_);
  float *dyS = (float *)(lds + L::DYS_);
  _Float16 *kH = (_Float16 *)(lds + L::KH_);
  _Float16 *vH = (_Float16 *)(lds + L::VH_);
  _Float16 *dyH = (_Float16 *)(lds + L::DYH_);
  float *fS = (float *)(lds + L::FS_);
  float *dvP = (float *)(lds + L::DVP_);
  float *dfP = (float *)(lds + L::DFP_);
  auto X = [&](int buf, int row) -> _Float16 * { return Xb[buf * ROWS + row]; };

  const bf16_raw *__restrict__ qg = (const bf16_raw *)a.q;
  const bf16_raw *__restrict__ kg = (const bf16_raw *)a.k;
  const bf16_raw *__restrict__ vg = (const bf16_raw *)a.v;
  const bf16_raw *__restrict__ dyg = (const bf16_raw *)a.dy;
  const float *__restrict__ fg = a.f;

  // ---- W fragments.  wf: B[k = c][n = j] = W[c][col0 + jl] (recompute);
  //      wtf: B[k = j][n = c] = W[col0 + jl][j] (carry contraction, W^T)
  FragT wf[KS], wtf[KS];
  {
    const bf16_raw *Wn = (const bf16_raw *)a.W + (size_t)n * V * V;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int e = 0; e < FE; ++e) {
        const int kk = FE * ig + e + 32 * ks;
        wf[ks][e] = (_Float16)bf16_to_f32(Wn[(size_t)kk * V + col0 + jl]);
        wtf[ks][e] = (_Float16)bf16_to_f32(Wn[(size_t)(col0 + jl) * V + kk]);
      }
  }

  const size_t tile_off = (size_t)(row_base + rowb + 4 * ig) * V + col0 + jl;
  const size_t st_off = (size_t)unit * K * V + tile_off;
  float carry[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) carry[r] = a.dHT ? a.dHT[st_off + (size_t)r * V] : 0.f;
  f4_t dWacc[CT];
#pragma unroll
  for (int c2 = 0; c2 < CT; ++c2) dWacc[c2] = f4_t{0.f, 0.f, 0.f, 0.f};

  const int nck = (T + C - 1) / C;

  // ---- staging: a whole chunk of q, k, v, dy, f goes through registers to LDS;
  //      the loads for chunk ck-1 are issued before phase B of chunk ck.
  bf16_raw rq[NQ], rk[NQ], rv[NV], rdy[NV];
  float rf = 1.f;
  float hck[4];
  auto stage_load = [&](int ck) {
    const int t0 = ck * C;
    const int len = (T - t0) < C ? (T - t0) : C;
#pragma unroll
    for (int m = 0; m < NQ; ++m) {
      const int idx = tid + m * THREADS;
      const int s = idx / ROWS, i = idx - s * ROWS;
      const bool ok = s < len;
      const size_t off = (((size_t)b * T + (t0 + s)) * a.Nqk + g) * K + row_base + i;
      rq[m] = ok ? qg[off] : (bf16_raw)0;
      rk[m] = ok ? kg[off] : (bf16_raw)0;
    }
#pragma unroll
    for (int m = 0; m < NV; ++m) {
      const int idx = tid + m * THREADS;
      const int s = idx / V, j = idx - s * V;
      const bool ok = s < len;
      const size_t off = (((size_t)b * T + (t0 + s)) * N + n) * V + j;
      rv[m] = ok ? vg[off] : (bf16_raw)0;
      rdy[m] = ok ? dyg[off] : (bf16_raw)0;
    }
    rf = (tid < len) ? fg[((size_t)b * T + (t0 + tid)) * N + n] : 1.f;
    const float *src = a.ckpt + ((size_t)unit * nck + ck) * K * V + tile_off;
#pragma unroll
    for (int r = 0; r < 4; ++r) hck[r] = src[(size_t)r * V];
  };
  auto stage_store = [&]() {
#pragma unroll
    for (int m = 0; m < NQ; ++m) {
      const int idx = tid + m * THREADS;
      if (idx < CMAX * ROWS) {
        const float kf = bf16_to_f32(rk[m]);
        kS[idx] = kC * kf;
        kH[idx] = (_Float16)kf;
        qS[idx] = bf16_to_f32(rq[m]);
      }
    }
#pragma unroll
    for (int m = 0; m < NV; ++m) {
      const int idx = tid + m * THREADS;
      if (idx < CMAX * V) {
        const float vf = bf16_to_f32(rv[m]), df_ = bf16_to_f32(rdy[m]);
        vS[idx] = vf;
        vH[idx] = (_Float16)vf;
        dyS[idx] = df_;
        dyH[idx] = (_Float16)df_;
      }
    }
    if (tid < CMAX) {
      fS[tid * 4 + 0] = rf;
      fS[tid * 4 + 1] = kC * (1.f - rf);
      fS[tid * 4 + 2] = 1.f - rf;
      fS[tid * 4 + 3] = -2.f * (kC * (1.f - rf));
    }
  };

  // dq_t = H_t dy_t  from the A fragments of H'_t (done by the ct == 0 wave of a row block)
  auto emit_dq = [&](const FragT *af, int s_prev, int t_prev) {
    f4_t d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const FragT bf = *(const FragT *)&dyH[s_prev * V + FE * ig + 32 * ks];
      if constexpr (X32)
        d = mfma_k32(af[ks], bf, d);
      else
        d = mfma_k16(af[ks], bf, d);
    }
    if (jl == 0) {
      d *= kInvC;
      if (ws.dqh) {
        *(f4_t *)&ws.dqh[(((size_t)b * T + t_prev) * N + n) * K + row_base + rowb + 4 * ig] = d;
      } else {
        uint2 pk;
        pk.x = (uint32_t)f32_to_bf16(d[0]) | ((uint32_t)f32_to_bf16(d[1]) << 16);
        pk.y = (uint32_t)f32_to_bf16(d[2]) | ((uint32_t)f32_to_bf16(d[3]) << 16);
        *(uint2 *)&((bf16_raw *)a.dq)[(((size_t)b * T + t_prev) * a.Nqk + g) * K + row_base +
                                      rowb + 4 * ig] = pk;
      }
    }
  };

  if (nck > 0) stage_load(nck - 1);

  int cur = 0;
  for (int ck = nck - 1; ck >= 0; --ck) {
    const int t0 = ck * C;
    const int len = (T - t0) < C ? (T - t0) : C;

    // ================= phase A: recompute the chunk, fill the stash
    stage_store();
    float h[4];
    h4_t hp;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      h[r] = kC * hck[r];
      hp[r] = (_Float16)h[r];
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) X(cur, rowb + 4 * ig + r)[col0 + jl] = hp[r];
    __syncthreads();

    for (int s = 0; s < len; ++s) {
      const float f = fS[s * 4 + 0], gp = fS[s * 4 + 1], m2g = fS[s * 4 + 3];
      const f4_t k4 = *(const f4_t *)&kS[s * ROWS + rowb + 4 * ig];
      const float vj = vS[s * V + col0 + jl];
      FragT af[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) af[ks] = *(const FragT *)&X(cur, rowb + jl)[FE * ig + 32 * ks];
      f4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        if constexpr (X32)
          acc = mfma_k32(af[ks], wf[ks], acc);
        else
          acc = mfma_k16(af[ks], wf[ks], acc);
      }
      if (ct == 0 && s > 0) emit_dq(af, s - 1, t0 + s - 1);
      stH[((s * RB + rb) * CT + ct) * 64 + lane] = hp;  // H'_{t-1}, this tile
      h4_t zp;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        // same operations, in the same order, as the forward kernel
        const float t1 = fmaf(f, h[r], gp);
        const float sp = fmaf(k4[r], vj, acc[r]);
        const float e = __builtin_amdgcn_exp2f(sp);
        const float rr = __builtin_amdgcn_rcpf(1.f + e);
        const float z = fmaf(-2.f * kC, rr, kC);  // c tanh(s)
        h[r] = fmaf(m2g, rr, t1);
        zp[r] = (_Float16)z;
        hp[r] = (_Float16)h[r];
      }
      stZ[((s * RB + rb) * CT + ct) * 64 + lane] = zp;
#pragma unroll
      for (int r = 0; r < 4; ++r) X(cur ^ 1, rowb + 4 * ig + r)[col0 + jl] = hp[r];
      __syncthreads();
      cur ^= 1;
    }
    if (ct == 0) {  // dq of the chunk's last step, from the state after it
      FragT af[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) af[ks] = *(const FragT *)&X(cur, rowb + jl)[FE * ig + 32 * ks];
      emit_dq(af, len - 1, t0 + len - 1);
    }
    __syncthreads();  // X is reused for dS from here on

    // ================= phase B: reverse sweep over the chunk
    // keep this chunk's tail of vectors in LDS; fetch the next chunk's into registers
    if (ck > 0) stage_load(ck - 1);

    for (int s = len - 1; s >= 0; --s) {
      const int t = t0 + s;
      const float f = fS[s * 4 + 0], gm = fS[s * 4 + 2];
      const f4_t q4 = *(const f4_t *)&qS[s * ROWS + rowb + 4 * ig];
      const float dyj = dyS[s * V + col0 + jl];
      const h4_t zp = stZ[((s * RB + rb) * CT + ct) * 64 + lane];
      h4_t hfr[CT];
#pragma unroll
      for (int c2 = 0; c2 < CT; ++c2) hfr[c2] = stH[((s * RB + rb) * CT + c2) * 64 + lane];
      const h4_t kfr = *(const h4_t *)&kH[s * ROWS + rowb + 4 * ig];

      float G[4];
      h4_t dsp;
      float dfl = 0.f;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float zz = (float)zp[r];
        const float hh = (float)hfr[ct][r];
        G[r] = fmaf(q4[r], dyj, carry[r]);
        dfl = fmaf(G[r], hh - zz, dfl);
        const float u = fmaf(zz * (-kInvC * kInvC), zz, 1.f);  // 1 - tanh^2
        const float ds = (gm * G[r]) * u;
        dsp[r] = (_Float16)ds;
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) X(cur, rowb + 4 * ig + r)[col0 + jl] = dsp[r];
      // dW' += H'^T dS  (this wave: all c tiles x its own j tile, rows of its row block)
#pragma unroll
      for (int c2 = 0; c2 < CT; ++c2) dWacc[c2] = mfma_k16(hfr[c2], dsp, dWacc[c2]);
      // dv partial over this row block:  D[*][n = j] = sum_i k_i dS[i][j]
      {
        f4_t dvv = {0.f, 0.f, 0.f, 0.f};
        dvv = mfma_k16(kfr, dsp, dvv);
        if (lane < 16) dvP[(cur * RB + rb) * V + col0 + jl] = dvv[0];
      }
      // df partial: 16-lane row sums, one value per DPP row
      {
        const float rs = row16_sum(dfl);
        if (jl == 0) dfP[cur * WAVES * 4 + wave * 4 + ig] = rs;
      }
      __syncthreads();

      // carry = f G + dS W^T ;  dk = dS v as one more column
      FragT af[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) af[ks] = *(const FragT *)&X(cur, rowb + jl)[FE * ig + 32 * ks];
      f4_t d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        if constexpr (X32)
          d = mfma_k32(af[ks], wtf[ks], d);
        else
          d = mfma_k16(af[ks], wtf[ks], d);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) carry[r] = fmaf(f, G[r], d[r]);

      if (ct == 0) {
        f4_t dkv = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const FragT bf = *(const FragT *)&vH[s * V + FE * ig + 32 * ks];
          if constexpr (X32)
            dkv = mfma_k32(af[ks], bf, dkv);
          else
            dkv = mfma_k16(af[ks], bf, dkv);
        }
        if (jl == 0) {
          if (ws.dkh) {
            *(f4_t *)&ws.dkh[(((size_t)b * T + t) * N + n) * K + row_base + rowb + 4 * ig] = dkv;
          } else {
            uint2 pk;
            pk.x = (uint32_t)f32_to_bf16(dkv[0]) | ((uint32_t)f32_to_bf16(dkv[1]) << 16);
            pk.y = (uint32_t)f32_to_bf16(dkv[2]) | ((uint32_t)f32_to_bf16(dkv[3]) << 16);
            *(uint2 *)&((bf16_raw *)a.dk)[(((size_t)b * T + t) * a.Nqk + g) * K + row_base + rowb +
                                          4 * ig] = pk;
          }
        }
      }
      if (rb == 0 && lane < 16) {  // dv: sum the row blocks of this workgroup
        float sdv = dvP[(cur * RB + 0) * V + col0 + jl];
#pragma unroll
        for (int r2 = 1; r2 < RB; ++r2) sdv += dvP[(cur * RB + r2) * V + col0 + jl];
        const size_t off = (((size_t)b * T + t) * N + n) * V + col0 + jl;
        if constexpr (TL::P == 1)
          ((bf16_raw *)a.dv)[off] = f32_to_bf16(sdv);
        else
          ws.dvp[(size_t)part * a.B * T * N * V + off] = sdv;
      }
      if (wave == WAVES - 1) {  // df: sum the WAVES*4 row sums in a fixed order
        float x = lane < WAVES * 4 ? dfP[cur * WAVES * 4 + lane] : 0.f;
        x = row16_sum(x);
        // rows of 16 lanes -> lanes 0, 16, 32, 48 hold the four row totals
        const float t01 = x + __shfl(x, lane ^ 16, 64);
        const float tot = t01 + __shfl(t01, lane ^ 32, 64);
        if (lane == 0) {
          const float val = tot * kInvC;
          const size_t off = ((size_t)b * T + t) * N + n;
          if constexpr (TL::P == 1)
            a.df[off] = val;
          else
            ws.dfp[(size_t)part * a.B * T * N + off] = val;
        }
      }
      cur ^= 1;
    }
    __syncthreads();  // every read of this chunk's staging and stash is done
  }

  if (a.dH0)
#pragma unroll
    for (int r = 0; r < 4; ++r) a.dH0[st_off + (size_t)r * V] = carry[r];
  // dW partial of this (unit, part, row block): rows c = 16 c2 + 4 ig + r, column col0 + jl
  {
    float *dst = ws.dWp + (((size_t)unit * TL::P + part) * RB + rb) * V * V;
#pragma unroll
    for (int c2 = 0; c2 < CT; ++c2)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        dst[(size_t)(c2 * 16 + 4 * ig + r) * V + col0 + jl] = dWacc[c2][r] * kInvC;
  }
}

// dv = bf16(sum of parts), df = sum of parts (increasing part order)
__global__ void bwd_parts_sum_kernel(const float *__restrict__ dvp, bf16_raw *__restrict__ dv,
                                     size_t n_dv, const float *__restrict__ dfp,
                                     float *__restrict__ df, size_t n_df, int P) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t e = blockIdx.x * (size_t)blockDim.x + threadIdx.x; e < n_dv; e += stride) {
    float s = dvp[e];
    for (int p = 1; p < P; ++p) s += dvp[(size_t)p * n_dv + e];
    dv[e] = f32_to_bf16(s);
  }
  for (size_t e = blockIdx.x * (size_t)blockDim.x + threadIdx.x; e < n_df; e += stride) {
    float s = dfp[e];
    for (int p = 1; p < P; ++p) s += dfp[(size_t)p * n_df + e];
    df[e] = s;
  }
}

// dW[n] = sum over b, then over the (part, row block) partials, in increasing order
__global__ void dw_parts_sum_kernel(const float *__restrict__ dWp, float *__restrict__ dW, int B,
                                    int N, int VV, int parts) {
  const size_t total = (size_t)N * VV;
  for (size_t e = blockIdx.x * (size_t)blockDim.x + threadIdx.x; e < total;
       e += (size_t)gridDim.x * blockDim.x) {
    const int n = e / VV, r = e - (size_t)n * VV;
    float s = 0.f;
    for (int b = 0; b < B; ++b)
      for (int p = 0; p < parts; ++p)
        s += dWp[(((size_t)b * N + n) * parts + p) * VV + r];
    dW[e] = s;
  }
}

__global__ void head_sum_bf16_kernel(const float *__restrict__ per_head, bf16_raw *__restrict__ out,
                                     size_t BT, int N, int Nqk, int K) {
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
    out[e] = f32_to_bf16(s);
  }
}

inline unsigned grid_for(size_t total, int threads) {
  size_t g = (total + threads - 1) / threads;
  if (g < 1) g = 1;
  if (g > 8192) g = 8192;
  return (unsigned)g;
}

struct WsLayout {
  size_t dvp, dfp, dWp, dqh, dkh, total;
};

WsLayout bwd_ws_layout(int B, int T, int N, int Nqk, int K, int V, int P, int RB) {
  WsLayout w;
  size_t off = 0;
  w.dvp = off; off += P > 1 ? align256((size_t)P * B * T * N * V * 4) : 0;
  w.dfp = off; off += P > 1 ? align256((size_t)P * B * T * N * 4) : 0;
  w.dWp = off; off += align256((size_t)B * N * P * RB * V * V * 4);
  const size_t heads = Nqk != N ? align256((size_t)B * T * N * K * 4) : 0;
  w.dqh = off; off += heads;
  w.dkh = off; off += heads;
  w.total = off;
  return w;
}

template <typename TL>
hipError_t launch_bwd(const BwdArgs &a, hipStream_t s) {
  using L = BwdLds<TL>;
  const int units = a.B * a.N;
  const WsLayout w = bwd_ws_layout(a.B, a.T, a.N, a.Nqk, a.K, a.V, TL::P, TL::RB);
  BwdWs ws;
  ws.dvp = (float *)(a.ws + w.dvp);
  ws.dfp = (float *)(a.ws + w.dfp);
  ws.dWp = (float *)(a.ws + w.dWp);
  const bool shared = a.Nqk != a.N;
  ws.dqh = shared ? (float *)(a.ws + w.dqh) : nullptr;
  ws.dkh = shared ? (float *)(a.ws + w.dkh) : nullptr;
  hipError_t e;
  if (units > 0) {
    if (a.C > L::CMAX) return hipErrorInvalidValue;
    e = hipFuncSetAttribute((const void *)mfma_bwd_kernel<TL>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, L::BYTES);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(mfma_bwd_kernel<TL>, dim3(grid_blocks(units, TL::P)), dim3(TL::THREADS),
                       L::BYTES, s, a, ws);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (a.T > 0) {
      if (TL::P > 1) {
        const size_t n_dv = (size_t)a.B * a.T * a.N * a.V, n_df = (size_t)a.B * a.T * a.N;
        hipLaunchKernelGGL(bwd_parts_sum_kernel, dim3(grid_for(n_dv, 256)), dim3(256), 0, s,
                           (const float *)ws.dvp, (bf16_raw *)a.dv, n_dv, (const float *)ws.dfp,
                           a.df, n_df, TL::P);
      }
      if (shared) {
        const size_t total = (size_t)a.B * a.T * a.Nqk * a.K;
        hipLaunchKernelGGL(head_sum_bf16_kernel, dim3(grid_for(total, 256)), dim3(256), 0, s,
                           (const float *)ws.dqh, (bf16_raw *)a.dq, (size_t)a.B * a.T, a.N, a.Nqk,
                           a.K);
        hipLaunchKernelGGL(head_sum_bf16_kernel, dim3(grid_for(total, 256)), dim3(256), 0, s,
                           (const float *)ws.dkh, (bf16_raw *)a.dk, (size_t)a.B * a.T, a.N, a.Nqk,
                           a.K);
      }
      if ((e = hipGetLastError()) != hipSuccess) return e;
    }
  }
  hipLaunchKernelGGL(dw_parts_sum_kernel, dim3(grid_for((size_t)a.N * a.V * a.V, 256)), dim3(256),
                     0, s, (const float *)ws.dWp, a.dW, a.B, a.N, a.V * a.V, TL::P * TL::RB);
  return hipGetLastError();
}

template <typename TL>
size_t ws_bytes(int B, int T, int N, int Nqk) {
  return bwd_ws_layout(B, T, N, Nqk, TL::K, TL::V, TL::P, TL::RB).total;
}

}  // namespace

int mfma_pick_rb(int K, int V, int units);

#define M2RNN_TILE_CASES(X)                                                                      \
  X(64, 64, 2) X(64, 64, 1) X(128, 128, 1) X(32, 32, 2) X(32, 32, 1) X(16, 16, 1) X(64, 16, 4)   \
  X(64, 16, 1)

hipError_t mfma_bwd(const BwdArgs &a, hipStream_t s) {
  const int rb = mfma_pick_rb(a.K, a.V, a.B * a.N);
#define X(K_, V_, RB_) \
  if (a.K == K_ && a.V == V_ && rb == RB_) return launch_bwd<Tile<K_, V_, RB_>>(a, s);
  M2RNN_TILE_CASES(X)
#undef X
  return hipErrorInvalidValue;
}

size_t mfma_bwd_workspace_bytes(int B, int T, int N, int Nqk, int K, int V) {
  const int rb = mfma_pick_rb(K, V, B * N);
#define X(K_, V_, RB_) \
  if (K == K_ && V == V_ && rb == RB_) return ws_bytes<Tile<K_, V_, RB_>>(B, T, N, Nqk);
  M2RNN_TILE_CASES(X)
#undef X
  return 0;
}

int mfma_bwd_max_chunk(int K, int V) {
  int best = kChunkCap;
#define X(K_, V_, RB_) \
  if (K == K_ && V == V_ && BwdLds<Tile<K_, V_, RB_>>::CMAX < best) best = BwdLds<Tile<K_, V_, RB_>>::CMAX;
  M2RNN_TILE_CASES(X)
#undef X
  return best;
}

}  // namespace m2rnn

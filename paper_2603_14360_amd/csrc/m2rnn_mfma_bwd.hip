// Matrix-core backward scan (Algorithm 2 of the paper, BPTT), with the carried
// state gradient added to q dy^T and propagated as  f G + dS W^T.
//
// The paper's kernel stores every H_t to HBM in a first pass and reloads it in
// the reverse sweep.  Here the forward leaves one fp32 checkpoint every C steps
// and the backward recomputes each chunk into an on-chip stash (LDS).  A
// workgroup holds two teams of wavefronts that run at the same time:
//   team A  recomputes chunk c-1 forward from its checkpoint, parking for every
//           step the fp16 state before the step (H'_{t-1} = c H_{t-1}) and
//           Z'_t = c tanh(.) in the stash, and accumulates dq_t = H_t dy_t;
//   team B  sweeps chunk c in reverse out of the stash entries team A made one
//           iteration earlier: no tanh and no state contraction are recomputed.
// Recomputing a chunk needs only its checkpoint, so it does not wait for the
// sweep of the chunk after it.  Both teams meet at one workgroup barrier per
// step, which each needs anyway for its own LDS exchange.
// Per step of team B and wavefront (16 x 16 tile, lane = 4 rows x 1 column):
//   G  = q_i dy_j + Ccarry                       (dL/dH_t)
//   dS = (1-f) G (1 - Z^2)                       -> fp16, to LDS (row-major)
//   dW' += H'_{t-1}^T dS       MFMA k = rows     (A = stash tiles, B = own dS)
//   Ccarry = f G + dS W^T      MFMA k = columns  (A = dS rows from LDS, B = W^T)
// The per-step vectors dq_t = H_t dy_t, dk_t = dS v_t, dv_t = dS^T k_t and the
// scalar df_t = sum G (H_{t-1} - Z_t) never leave the matrix core during a
// chunk: each is one more MFMA whose second operand (dy_t, v_t, k_t, ones) is
// placed in column / row (t mod chunk) only, so a 16 x 16 accumulator collects
// the chunk's steps side by side and nothing is read back per step.  At the
// end of a chunk the partial accumulators of the waves are added through LDS
// in a fixed order and stored; nothing uses atomics.
#include "m2rnn_kernels.hpp"
#include "m2rnn_mfma_common.hpp"

namespace m2rnn {
namespace {

constexpr int kChunkCap = 16;  // = MFMA N: one accumulator column per step of a chunk

struct BwdWs {
  float *dvp;   // [P][B,T,N,V]      (P > 1)
  float *dfp;   // [P*WAVES][B,N,T]  per-wave partials of df, summed (and laid out as [B,T,N]) by the epilogue
  float *dWp;   // [B*N][P*RB][V][V]
  float *dqh;   // [B,T,N,K]         (Nqk != N)
  float *dkh;
};

__device__ __forceinline__ uint2 pack4_bf16(f4_t x) {
  uint2 p;
  p.x = (uint32_t)f32_to_bf16(x[0]) | ((uint32_t)f32_to_bf16(x[1]) << 16);
  p.y = (uint32_t)f32_to_bf16(x[2]) | ((uint32_t)f32_to_bf16(x[3]) << 16);
  return p;
}

// LDS carve-up of the kernel.
//
// The stash holds C + 1 step slots for BOTH teams, used as two stacks that grow towards
// each other: in an iteration team A pushes the C steps of its chunk in time order from one
// end while team B pops the steps of its chunk, which were pushed from the other end one
// iteration earlier, in reverse order.  The slot B reads in a step is the one A fills in
// the next step, so one spare slot is enough and the checkpoint interval C can be almost
// twice what two separate buffers would allow (chunk boundaries cost several step times).
// Fragment read through the transposing LDS load of gfx950 (ds_read_b64_tr_b16).  Within each
// group of 16 lanes the 16 x 8 bytes that the lanes address are taken as 64 consecutive
// fp16 values and lane d receives values d, 16 + d, 32 + d, 48 + d of them.  With the tile
// stored as 8-byte items (column j, rows 4 i .. 4 i + 3) -- which is what a lane of the
// accumulator layout holds -- at byte offset 32 j + 8 i, lane d addressing item
// (column c0 + d / 4, rows 4 (d % 4) ..) receives row d, columns c0 .. c0 + 3: the A operand of
// the 16-row MFMAs, with no scattered 2-byte writes and no padded rows.
__device__ __forceinline__ h4_t lds_ld_tr(const lchar *p, int off) {
  typedef short s4_t __attribute__((ext_vector_type(4)));
  const s4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s4_t *)(p + off));
  return __builtin_bit_cast(h4_t, v);
}
// Where the four items of a column sit inside the column's 32 bytes, and where a group of
// four columns sits inside its 256-byte pair, is free (every lane of the transposing load
// supplies its own address).  Item (column j, rows 4 i ..) goes to
// a = 32 j + 8 ((i + j / 4) mod 4) and then to a xor (128 if bit 8 of a is set): the items a
// lane group reads are still 128 contiguous bytes, but the four lane groups and the two
// halves of a k = 32 fragment start on different banks.  In the plain order (32 j + 8 i) a
// third of the LDS-active cycles of the backward are bank conflicts; placed like this, 1 %.
// That is worth 6.5 % of the backward on the 128-wide tile (rotation alone 3.5 %); on the
// 64-wide tiles, where the LDS is not what the step waits for, the time does not change.
__device__ __forceinline__ int xch_item_off(int j, int i) {
  const int a = 32 * j + 8 * ((i + (j >> 2)) & 3);
  return a ^ ((a >> 1) & 128);
}
// Per-lane base offsets of a fragment read: lane (d, g) = (lane % 16, lane / 16) reads, for
// the first half of its FE columns c0 = FE g .., item (column c0 + d / 4, rows 4 (d % 4) ..); the
// second half (k = 32 fragments only) is the next group of 4 columns.
template <bool X32>
__device__ __forceinline__ int xch_frag_off(int d, int g, int half) {
  constexpr int FE = X32 ? 8 : 4;
  const int c0 = FE * g + 4 * half;
  return xch_item_off(c0 + (d >> 2), d & 3);
}
template <bool X32>
__device__ __forceinline__ typename Frag<X32>::type lds_ld_frag_tr(const lchar *p0, const lchar *p1, int off) {
  if constexpr (X32) {
    const h4_t lo = lds_ld_tr(p0, off), hi = lds_ld_tr(p1, off);
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  } else {
    return lds_ld_tr(p0, off);
  }
}

// The lane index computed on the spot (two instructions).  The chunk-boundary code derives
// its per-lane offsets from this instead of from a lane index kept in a register since the
// kernel's start: on the tiles at the register limit that register is spilled, and a reload
// from scratch in the boundary code waits for every global store issued before it.
__device__ __forceinline__ int lane_now() {
  return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

template <typename TL>
struct OvLds {
  static constexpr int ROWS = TL::ROWS, V = TL::V, RB = TL::RB, CT = TL::CT,
                       WAVES = TL::WAVES, KS = TL::KS;
  static constexpr int DXCH = 2 * ROWS * V * 2;           // a double-buffered fp16 exchange tile set (8-byte items, unpadded)
  // the exchange buffers also carry the end-of-chunk partials (1 KB per contributing wave):
  // dq slices of team A and dk slices of team B in A's buffer, dv of team B in B's buffer
  static constexpr int HX_BYTES = DXCH > 2 * RB * KS * 1024 ? DXCH : 2 * RB * KS * 1024;
  static constexpr int DX_BYTES = DXCH > WAVES * 1024 ? DXCH : WAVES * 1024;
  static constexpr int STASH_STEP = RB * CT * 64 * 8;     // one h4 per lane per tile
  static constexpr int SLOT = 2 * STASH_STEP;             // a step slot: H' tiles, then Z' tiles
  static constexpr int VEC_A = ROWS * 4 + V * 2 + V * 2 + 16;          // c*k, v (f16), dy (f16), f
  static constexpr int VEC_B = ROWS * 4 + V * 4 + ROWS * 2 + V * 2 + 16;  // q, dy, k f16, v f16, f
  static constexpr int PER_STEP = SLOT + VEC_A + VEC_B;
  static constexpr int FIXED = HX_BYTES + DX_BYTES + SLOT + 448;
  static constexpr int CMAX_RAW = (kLdsLimit - FIXED) / PER_STEP;
  // (the one-wave teams of a V = 16 tile would lose resident workgroups to a larger LDS
  //  footprint; those shapes are served by the register-resident backward instead)
  static constexpr int CCAP = TL::THREADS <= 64 ? 12 : kChunkCap;
  static constexpr int CMAX = CMAX_RAW > CCAP ? CCAP : CMAX_RAW;
  static constexpr bool OK = (2 * WAVES <= 16) && (CMAX >= 4);
  static constexpr int C_ = CMAX > 0 ? CMAX : 1;
  static constexpr int NSLOT = C_ + 1;
  static constexpr int HX = 0;
  static constexpr int DX = HX + HX_BYTES;
  // the small per-step vectors sit below the stash: their offsets then fit the 16-bit
  // immediate of the LDS instructions (one base register instead of one per step)
  static constexpr int KS_ = DX + DX_BYTES;                // team A: float c*k [C][ROWS]
  static constexpr int VS_ = KS_ + C_ * ROWS * 4;          //         half v    [C][V]
  static constexpr int DYH_ = VS_ + C_ * V * 2;            //         half dy (scaled per step) [C][V]
  static constexpr int FA_ = DYH_ + C_ * V * 2;            //         float f, c(1-f), 1/dy-scale of the two half rows
  static constexpr int QS_ = FA_ + C_ * 16;                // team B: float q   [C][ROWS]
  static constexpr int DYS_ = QS_ + C_ * ROWS * 4;         //         float dy  [C][V]
  static constexpr int KH_ = DYS_ + C_ * V * 4;            //         half k    [C][ROWS]
  static constexpr int VH_ = KH_ + C_ * ROWS * 2;          //         half v    [C][V]
  static constexpr int FB_ = VH_ + C_ * V * 2;             //         f; f16x2 -(1-f)/c^2; 1-f; -
  static constexpr int ZERO_ = FB_ + C_ * 16;              // 32 zero bytes (masked operand reads)
  static constexpr int SCL_ = ZERO_ + 32;                  // team B: maxima, two sets of 4 words
  static constexpr int ST = (SCL_ + 96 + 255) & ~255;      // [NSLOT][ {H, Z} ][RB][CT][64] h4
  static constexpr int BYTES = ST + NSLOT * SLOT;
  static_assert(!OK || BYTES <= kLdsLimit, "LDS overflow");
};

// CLIP: the gradient handed from step t to step t - 1 is clamped element-wise to
// [-a.clip, a.clip] as soon as it is formed (the paper's per-step clipping of the state
// gradient); a separate instantiation, so the exact-gradient kernel pays nothing for it.
template <typename TL, bool CLIP>
__global__ void __launch_bounds__(2 * TL::THREADS, 2) mfma_bwd_overlap_kernel(BwdArgs a, BwdWs ws) {
  constexpr int K = TL::K, V = TL::V, RB = TL::RB, CT = TL::CT, ROWS = TL::ROWS, KS = TL::KS,
                WAVES = TL::WAVES;
  constexpr int THREADS = TL::THREADS;  // per team
  constexpr bool X32 = TL::X32;
  constexpr int FE = X32 ? 8 : 4;
  using FragT = typename Frag<X32>::type;
  using L = OvLds<TL>;
  constexpr int CMAX = L::C_;
  // Staging of the per-step vectors: 16-byte items (8 bf16 values of one step), at most one
  // item per thread and tensor.  The tensors are dealt to different waves of a team where
  // it has several (thread tid stages item (tid - shift) mod THREADS of a tensor).
  constexpr int RL = ROWS / 8, VL = V / 8;            // items per step
  constexpr int QI = CMAX * RL, VI = CMAX * VL;       // items per chunk
  static_assert(QI <= THREADS && VI <= THREADS, "one staged item per thread and tensor");
  constexpr int SH_K = 0, SH_V = 64 % THREADS, SH_DY = 192 % THREADS, SH_F = 320 % THREADS,
                SH_Q = 384 % THREADS;

  int unit, part;
  if (!map_block<TL::P>(a.B * a.N, unit, part)) return;
  const int T = a.T, N = a.N, C = a.C;
  const int b = unit / N, n = unit - b * N;
  const int g = n / (N / a.Nqk);
  const int lane = threadIdx.x & 63;
  const int wave_all = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const bool teamA = wave_all >= WAVES;            // scalar: each team runs its own code
  const int wave = teamA ? wave_all - WAVES : wave_all;
  const int tid = wave * 64 + lane;                // thread index inside the team
  const int rb = wave / CT, ct = wave - rb * CT;
  const int jl = lane & 15, ig = lane >> 4;
  const int col0 = ct * 16, rowb = rb * 16;
  const int row_base = part * ROWS;

  extern __shared__ __attribute__((aligned(16))) char lds[];
  // slot of chunk step s for a chunk pushed in an iteration of parity p (see OvLds)
  auto slot_of = [&](int s, int p) { return p ? (L::NSLOT - 1 - s) : s; };
  float *kS = (float *)(lds + L::KS_);
  _Float16 *vS = (_Float16 *)(lds + L::VS_);
  _Float16 *dyH = (_Float16 *)(lds + L::DYH_);
  float *fA = (float *)(lds + L::FA_);
  float *qS = (float *)(lds + L::QS_);
  float *dyS = (float *)(lds + L::DYS_);
  _Float16 *kH = (_Float16 *)(lds + L::KH_);
  _Float16 *vH = (_Float16 *)(lds + L::VH_);
  float *fB = (float *)(lds + L::FB_);

  const bf16_raw *__restrict__ qg = (const bf16_raw *)a.q;
  const bf16_raw *__restrict__ kg = (const bf16_raw *)a.k;
  const bf16_raw *__restrict__ vg = (const bf16_raw *)a.v;
  const bf16_raw *__restrict__ dyg = (const bf16_raw *)a.dy;
  const float *__restrict__ fg = a.f;
  const bf16_raw *Wn = (const bf16_raw *)a.W + (size_t)n * V * V;

  const size_t tile_off = (size_t)(row_base + rowb + 4 * ig) * V + col0 + jl;
  const size_t st_off = (size_t)unit * K * V + tile_off;
  const int nck = (T + C - 1) / C;
  const f4_t zero4 = {0.f, 0.f, 0.f, 0.f};
  if (threadIdx.x < 32) ((uint32_t *)(lds + L::ZERO_))[threadIdx.x] = 0u;  // zero pad and the
                                                                          // maxima slots behind it; visible after barrier P

  // gate parameters of this head, read once (a load inside the chunk loop would wait for
  // the end-of-chunk stores issued before it)
  const float g_alpha = a.gate_alpha ? a.gate_alpha[n] : 0.f, g_beta = a.gate_alpha ? a.gate_beta[n] : 0.f;

  if (teamA) {
    // =====================================================================
    // team A: recompute chunk nck-1-it into stash[it & 1], it = 0 .. nck-1
    // The recomputed states only feed fp16 stash entries and restart from an fp32 checkpoint
    // every C steps, so the state enters this team's contraction as a single fp16 value
    // (the forward kernel needs the (hi, lo) pair because its trajectory runs for all T steps).
    FragT wf[KS];  // B operand: k-slot e of MFMA ks holds W[32 ks + FE ig + e][col0 + jl]
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int e = 0; e < FE; ++e)
        wf[ks][e] = (_Float16)bf16_to_f32(Wn[(size_t)(32 * ks + FE * ig + e) * V + col0 + jl]);
    u4_t rk, rv, rdy;
    float rf = 1.f;
    float hck[4];
    // Global addresses of the staged vectors: a wave-uniform 64-bit base per tensor (batch
    // element, head, chunk start) plus a 32-bit byte offset inside the chunk.
    const bf16_raw *const kbase = kg + ((size_t)b * T * a.Nqk + g) * K + row_base;
    const bf16_raw *const vbase = vg + ((size_t)b * T * N + n) * V;
    const bf16_raw *const dybase = dyg + ((size_t)b * T * N + n) * V;
    const float *const fbase = fg + (size_t)b * T * N + n;
    const uint32_t kstride = (uint32_t)a.Nqk * K, vstride = (uint32_t)N * V;
    const bool wave_has_dy = ((wave * 64 - SH_DY) & (THREADS - 1)) < VI;  // wave-uniform
    const u4_t zero_u4 = {0u, 0u, 0u, 0u};
    // The loads address memory as uniform base + 32-bit byte offset, and the per-thread part
    // of the offset is recomputed from the thread index at every call (a few shifts and
    // adds): kept in registers across the chunk it would be spilled, and a reload from
    // scratch in front of a load waits for every load issued before it.
    auto stage_load = [&](int ck) {
      const int t0 = ck * C;
      const int len = (T - t0) < C ? (T - t0) : C;
      int tl = wave * 64 + lane_now();
      asm volatile("" : "+v"(tl));
      {
        const int e = (tl - SH_K) & (THREADS - 1), s = e / RL, p = e - s * RL;
        const uint32_t off = 2u * ((uint32_t)s * kstride + 8u * p);
        rk = (e < QI && s < len) ? *(const u4_t *)((const char *)(kbase + (size_t)t0 * kstride) + off) : zero_u4;
      }
      {
        const int e = (tl - SH_V) & (THREADS - 1), s = e / VL, p = e - s * VL;
        const uint32_t off = 2u * ((uint32_t)s * vstride + 8u * p);
        rv = (e < VI && s < len) ? *(const u4_t *)((const char *)(vbase + (size_t)t0 * vstride) + off) : zero_u4;
      }
      {
        const int e = (tl - SH_DY) & (THREADS - 1), s = e / VL, p = e - s * VL;
        const uint32_t off = 2u * ((uint32_t)s * vstride + 8u * p);
        rdy = (e < VI && s < len) ? *(const u4_t *)((const char *)(dybase + (size_t)t0 * vstride) + off) : zero_u4;
      }
      {
        const int e = (tl - SH_F) & (THREADS - 1);
        rf = (e < len) ? *(const float *)((const char *)(fbase + (size_t)t0 * N) + 4u * ((uint32_t)e * (uint32_t)N))
                       : 1.f;
      }
      {
        const int l = tl & 63;
        const uint32_t off = 4u * (uint32_t)((row_base + rowb + 4 * (l >> 4)) * V + col0 + (l & 15));
        const char *src = (const char *)(a.ckpt + ((size_t)unit * nck + ck) * K * V) + off;
#pragma unroll
        for (int r = 0; r < 4; ++r) hck[r] = *(const float *)(src + r * V * 4);
      }
    };
    auto stage_store = [&]() {
      asm volatile("" : "+v"(rk), "+v"(rv), "+v"(rdy));
      asm volatile("" : "+v"(rf), "+v"(hck[0]), "+v"(hck[1]), "+v"(hck[2]), "+v"(hck[3]));
      // (item indices rebuilt from the thread index on the spot: kept in registers across the
      //  chunk they are spilled, and a reload from scratch here waits for the end-of-chunk
      //  stores in front of it)
      int tl = wave * 64 + lane_now();
      asm volatile("" : "+v"(tl));
      const int ek = (tl - SH_K) & (THREADS - 1), ev = (tl - SH_V) & (THREADS - 1),
                edy = (tl - SH_DY) & (THREADS - 1), ef = (tl - SH_F) & (THREADS - 1);
      float x[8];
      if (ek < QI) {
        bf16x8_to_f32(rk, x);
        *(f4_t *)&kS[8 * ek] = f4_t{x[0], x[1], x[2], x[3]} * kC;
        *(f4_t *)&kS[8 * ek + 4] = f4_t{x[4], x[5], x[6], x[7]} * kC;
      }
      if (ev < VI) {
        // (fp16 like every other copy of v that feeds the matrix core: exact for bf16
        //  data of magnitude 6e-5 .. 6e4, and the k v^T product takes it as a
        //  mixed-precision FMA operand)
        bf16x8_to_f32(rv, x);
        h8_t hv;
#pragma unroll
        for (int i = 0; i < 8; ++i) hv[i] = (_Float16)x[i];
        *(h8_t *)&vS[8 * ev] = hv;
      }
      if (wave_has_dy) {
        // dy_s enters the dq contraction as fp16: each step's row is scaled by a power of two
        // so that its largest entry lands in [2^10, 2^11) (loss-scaled or token-averaged
        // gradients are far outside the fp16 range); column s of dq is scaled back at the end
        // (a row of V = 128 has two halves of 64 columns with a scale each: a dq slice
        //  covers 32 columns, i.e. lies inside one half).  A row (half row) is held by
        // GL consecutive lanes, 8 values each.
        constexpr int GL = (V < 64 ? V : 64) / 8;
        bf16x8_to_f32(rdy, x);
        float mx = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) mx = fmaxf(mx, fabsf(x[i]));
        const int e = ilog2f(fminf(fmaxf(group_max_nonneg<GL>(mx), 1e-30f), 1e30f));
        if (edy < VI) {
          const float up = pow2i(10 - e);
          h8_t hv;
#pragma unroll
          for (int i = 0; i < 8; ++i) hv[i] = (_Float16)(x[i] * up);
          *(h8_t *)&dyH[8 * edy] = hv;
          const int s = edy / VL, p = edy - s * VL;
          if (p % GL == 0) fA[s * 4 + 2 + (8 * p) / 64] = pow2i(e - 10);
        }
      }
      if (ef < CMAX) {
        if (a.gate_alpha) rf = gate_psi(rf, g_alpha, g_beta);
        fA[ef * 4 + 0] = rf;
        fA[ef * 4 + 1] = kC * (1.f - rf);
      }
    };
    // dq of chunk step s_col (= H after that step, times dy of that step): wave ct < KS adds
    // its 32-column slice into accumulator column s_col; the other lanes' operand is zero
    auto dq_slice = [&](f4_t acc, const FragT &af_ct, int s_col) {
      const FragT bf = *(const FragT *)(jl == s_col ? (const char *)&dyH[s_col * V + FE * ig + 32 * ct]
                                                    : (const char *)(lds + L::ZERO_));
      if constexpr (X32)
        return mfma_k32(af_ct, bf, acc);
      else
        return mfma_k16(af_ct, bf, acc);
    };

    // state exchange of this team: written as 8-byte items (column, rows 4 ig ..), read back
    // as row fragments through the transposing LDS load (see lds_ld_tr)
    lchar *const aHw = (lchar *)lds + rb * V * 32 + xch_item_off(col0 + jl, ig);
    const lchar *const aHr0 = (lchar *)lds + rb * V * 32 + xch_frag_off<X32>(jl, ig, 0);
    const lchar *const aHr1 = (lchar *)lds + rb * V * 32 + xch_frag_off<X32>(jl, ig, 1);
    if (nck > 0) stage_load(nck - 1);
    // (waited for in front of the loop as well: a wait only on the way round the loop makes
    //  the compiler wait at the loop head on every iteration)
    asm volatile("" : "+v"(rk), "+v"(rv), "+v"(rdy), "+v"(rf));
    asm volatile("" : "+v"(hck[0]), "+v"(hck[1]), "+v"(hck[2]), "+v"(hck[3]));
    for (int it = 0; it <= nck; ++it) {
      const bool active = it < nck;
      const int ck = nck - 1 - it;
      const int t0 = ck * C;
      const int len = active ? ((T - t0) < C ? (T - t0) : C) : 0;
      const int par = it & 1;  // this chunk's end of the stash
      float h[4];
      h4_t hp;  // fp16 copy of the state before the current step (stash entry, MFMA operand)
      int cur = 0;
      f4_t dqacc = zero4;
      if (active) {
        stage_store();
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          h[r] = kC * hck[r];
          hp[r] = (_Float16)h[r];
        }
        lds_st<h4_t>(aHw, L::HX + cur * ROWS * V * 2, hp);
      }
      lds_barrier();  // P
      // Next chunk's vectors and checkpoint travel during this chunk; issued behind the
      // barrier, where this team has slack (team B waits for it there).  Unconditional (the
      // last iterations fetch chunk 0 again): a conditional fetch makes the compiler merge
      // the old and the new register values right here, which waits for the loads.
      stage_load(ck > 0 ? ck - 1 : 0);
      // one recomputed step; `s` and the exchange buffer parity are compile-time constants
      // in the unrolled loop below (per-step loop overhead costs as much as the arithmetic)
      auto stepA = [&](int s) __attribute__((always_inline)) {
        const int rd = s & 1, wr = rd ^ 1;
        FragT af[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          af[ks] = lds_ld_frag_tr<X32>(aHr0, aHr1, L::HX + rd * ROWS * V * 2 + 1024 * ks);
        const float f = fA[s * 4 + 0], gp = fA[s * 4 + 1], m2g = -2.f * gp;
        const f4_t k4 = *(const f4_t *)&kS[s * ROWS + rowb + 4 * ig];
        const float vj = (float)vS[s * V + col0 + jl];
        f4_t acc = zero4;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          if constexpr (X32)
            acc = mfma_k32(af[ks], wf[ks], acc);
          else
            acc = mfma_k16(af[ks], wf[ks], acc);
        }
        settle(acc);
        h4_t *slot = (h4_t *)(lds + L::ST + slot_of(s, par) * L::SLOT) + (rb * CT + ct) * 64 + lane;
        slot[0] = hp;
        h4_t zp;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float t1 = fmaf(f, h[r], gp);
          const float sp = fmaf(k4[r], vj, acc[r]);
          const float e = __builtin_amdgcn_exp2f(sp);
          const float rr = __builtin_amdgcn_rcpf(1.f + e);
          const float z = fmaf(-2.f * kC, rr, kC);
          h[r] = fmaf(m2g, rr, t1);
          zp[r] = (_Float16)z;
          hp[r] = (_Float16)h[r];
        }
        slot[L::STASH_STEP / 8] = zp;
        lds_st<h4_t>(aHw, L::HX + wr * ROWS * V * 2, hp);
        if (s > 0 && ct < KS) {  // dq slice of the previous step; af still holds the state after it
          if constexpr (KS > 2) {
            // picking af[ct] out of four fragments is a ladder of branches: this wave's own
            // fragment is read once more instead (the buffer is not rewritten before the barrier)
            const FragT afq = lds_ld_frag_tr<X32>(aHr0 + 1024 * ct, aHr1 + 1024 * ct, L::HX + rd * ROWS * V * 2);
            dqacc = dq_slice(dqacc, afq, s - 1);
          } else {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
              if (ct == ks) dqacc = dq_slice(dqacc, af[ks], s - 1);
          }
        }
      };
      if (C == CMAX) {
#pragma unroll
        for (int s = 0; s < CMAX; ++s) {
          if (s < len) stepA(s);
          lds_barrier();  // one per step, shared with team B
        }
      } else {
#pragma nounroll
        for (int s = 0; s < C; ++s) {
          if (s < len) stepA(s);
          lds_barrier();
        }
      }
      cur = len & 1;
      // The next chunk's prefetch (issued C steps ago) is waited for HERE, in front of the
      // end-of-chunk global stores: the vector-memory counter is in order, so a wait placed
      // behind the stores (where stage_store first reads the registers) would also wait
      // until the stores have reached memory.
      asm volatile("" : "+v"(rk), "+v"(rv), "+v"(rdy), "+v"(rf));
      asm volatile("" : "+v"(hck[0]), "+v"(hck[1]), "+v"(hck[2]), "+v"(hck[3]));
      if (active && ct < KS) {  // dq of the chunk's last step, from the state after it
        const FragT afl = lds_ld_frag_tr<X32>(aHr0 + 1024 * ct, aHr1 + 1024 * ct, L::HX + cur * ROWS * V * 2);
        dqacc = dq_slice(dqacc, afl, len - 1);
      }
      lds_barrier();  // E1: exchange buffer free, it carries the dq partials now
      f4_t *fin = (f4_t *)(lds + L::HX);  // [RB][KS][64]: only the waves ct < KS hold a dq slice
      if (active && ct < KS) fin[(rb * KS + ct) * 64 + lane] = dqacc;
      lds_barrier();  // E2
      if (active && ct == 0 && jl < len) {
        // add the 32-column slices, each scaled back by its step's (and half row's) dy scale
        f4_t d = fin[(rb * KS + 0) * 64 + lane] * fA[jl * 4 + 2];
#pragma unroll
        for (int ks = 1; ks < KS; ++ks)
          d += fin[(rb * KS + ks) * 64 + lane] * fA[jl * 4 + 2 + (32 * ks) / 64];
        d *= kInvC;
        // (uniform base + 32-bit byte offset rebuilt from the lane index: see stage_load)
        int ll = lane_now();
        asm volatile("" : "+v"(ll));
        const uint32_t jl2 = ll & 15, ig2 = ll >> 4;
        if (ws.dqh) {
          char *base = (char *)(ws.dqh + (((size_t)b * T + t0) * N + n) * K + row_base + rowb);
          *(f4_t *)(base + 4u * (jl2 * (uint32_t)(N * K) + 4u * ig2)) = d;
        } else {
          char *base = (char *)((bf16_raw *)a.dq + (((size_t)b * T + t0) * a.Nqk + g) * K + row_base + rowb);
          *(uint2 *)(base + 2u * (jl2 * kstride + 4u * ig2)) = pack4_bf16(d);
        }
      }
      lds_barrier();  // E3
    }
    return;
  }

  // =======================================================================
  // team B: sweep chunk nck-it out of stash[(it-1) & 1], it = 1 .. nck
  // This team's step is the longer one (the recompute team waits for it at every barrier),
  // so its waves get the higher issue priority on the SIMDs they share with that team.
  __builtin_amdgcn_s_setprio(3);
  FragT wtf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
#pragma unroll
    for (int e = 0; e < FE; ++e)
      wtf[ks][e] = (_Float16)bf16_to_f32(Wn[(size_t)(col0 + jl) * V + FE * ig + e + 32 * ks]);
  float carry[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) carry[r] = a.dHT ? a.dHT[st_off + (size_t)r * V] : 0.f;
  f4_t dWacc[CT];
#pragma unroll
  for (int c2 = 0; c2 < CT; ++c2) dWacc[c2] = zero4;
  // Dynamic range of the fp16 dS operand.  The carried gradient of this recurrence can grow
  // (or shrink) by orders of magnitude over a long sequence; dS would leave the fp16 range.
  // The sweep therefore works on sc * (carry, G, dS, and every accumulator fed by dS) with
  // sc a power of two chosen per chunk from the largest |carry| in the workgroup and the
  // largest |q| |dy| of the chunk.  Powers of two make the scaling exact; outputs are
  // divided by sc.  The scaled magnitudes start a chunk in [2^5, 2^6): growth by 2^10
  // inside the chunk still fits fp16, and values down to 2^-19 of the largest keep their
  // full mantissa.  Where the previous chunk grew by g > 2 bits, the start is lowered by
  // g - 2 bits more (at most 12), so a gradient that explodes steadily, by up to 2^22 per
  // chunk, is followed.  A jump of more than 2^10 inside one chunk right after a calm
  // chunk still overflows dS (gradients become inf / NaN): the regime the paper's
  // per-step clipping (grad_clip) exists for.
  // The scale never exceeds 2^90 times the smallest scale used so far: dW accumulates
  // sc * (sum of H^T dS) over the whole sweep, at most 2^32 / (smallest sc) in magnitude,
  // and is rescaled with sc; a gradient that has died away (loss on the last tokens only)
  // would otherwise drive sc to 2^120 and the accumulated dW to infinity.  Steps whose
  // gradient is more than 2^90 below the largest seen lose precision instead.
  float sc = 1.f, isc = 1.f;
  int sc_e = 0, sc_e_min = 1 << 20, mx_e_prev = -(1 << 20);
  int set_now = 0;
  int *scl = (int *)(lds + L::SCL_);  // two sets of { max |carry|, max |q|, max |dy| } bit patterns,
                                       // by iteration parity; filled with LDS atomic max
  auto wave_max = [&](float x) { return group_max_nonneg<64>(x); };

  u4_t rq, rk, rv, rdy;
  float rf = 1.f;
  // (addresses as in team A: uniform base + 32-bit element offset)
  const bf16_raw *const qbase = qg + ((size_t)b * T * a.Nqk + g) * K + row_base;
  const bf16_raw *const kbase = kg + ((size_t)b * T * a.Nqk + g) * K + row_base;
  const bf16_raw *const vbase = vg + ((size_t)b * T * N + n) * V;
  const bf16_raw *const dybase = dyg + ((size_t)b * T * N + n) * V;
  const float *const fbase = fg + (size_t)b * T * N + n;
  const uint32_t kstride = (uint32_t)a.Nqk * K, vstride = (uint32_t)N * V;
  const bool wave_has_q = ((wave * 64 - SH_Q) & (THREADS - 1)) < QI;    // wave-uniform
  const bool wave_has_dy = ((wave * 64 - SH_DY) & (THREADS - 1)) < VI;
  const u4_t zero_u4 = {0u, 0u, 0u, 0u};
  auto stage_load = [&](int ck) {  // (addresses as in team A)
    const int t0 = ck * C;
    const int len = (T - t0) < C ? (T - t0) : C;
    int tl = wave * 64 + lane_now();
    asm volatile("" : "+v"(tl));
    {
      const int e = (tl - SH_Q) & (THREADS - 1), s = e / RL, p = e - s * RL;
      const uint32_t off = 2u * ((uint32_t)s * kstride + 8u * p);
      rq = (e < QI && s < len) ? *(const u4_t *)((const char *)(qbase + (size_t)t0 * kstride) + off) : zero_u4;
    }
    {
      const int e = (tl - SH_K) & (THREADS - 1), s = e / RL, p = e - s * RL;
      const uint32_t off = 2u * ((uint32_t)s * kstride + 8u * p);
      rk = (e < QI && s < len) ? *(const u4_t *)((const char *)(kbase + (size_t)t0 * kstride) + off) : zero_u4;
    }
    {
      const int e = (tl - SH_V) & (THREADS - 1), s = e / VL, p = e - s * VL;
      const uint32_t off = 2u * ((uint32_t)s * vstride + 8u * p);
      rv = (e < VI && s < len) ? *(const u4_t *)((const char *)(vbase + (size_t)t0 * vstride) + off) : zero_u4;
    }
    {
      const int e = (tl - SH_DY) & (THREADS - 1), s = e / VL, p = e - s * VL;
      const uint32_t off = 2u * ((uint32_t)s * vstride + 8u * p);
      rdy = (e < VI && s < len) ? *(const u4_t *)((const char *)(dybase + (size_t)t0 * vstride) + off) : zero_u4;
    }
    {
      const int e = (tl - SH_F) & (THREADS - 1);
      rf = (e < len) ? *(const float *)((const char *)(fbase + (size_t)t0 * N) + 4u * ((uint32_t)e * (uint32_t)N))
                     : 1.f;
    }
  };
  auto stage_store = [&]() {
    asm volatile("" : "+v"(rq), "+v"(rk), "+v"(rv), "+v"(rdy), "+v"(rf));
    int tl = wave * 64 + lane_now();  // (item indices rebuilt on the spot: see team A)
    asm volatile("" : "+v"(tl));
    const int eq = (tl - SH_Q) & (THREADS - 1), ek = (tl - SH_K) & (THREADS - 1),
              ev = (tl - SH_V) & (THREADS - 1), edy = (tl - SH_DY) & (THREADS - 1),
              ef = (tl - SH_F) & (THREADS - 1);
    float x[8];
    if (wave_has_q) {
      bf16x8_to_f32(rq, x);
      if (eq < QI) {
        *(f4_t *)&qS[8 * eq] = f4_t{x[0], x[1], x[2], x[3]};
        *(f4_t *)&qS[8 * eq + 4] = f4_t{x[4], x[5], x[6], x[7]};
      }
      float mq = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) mq = fmaxf(mq, fabsf(x[i]));
      mq = wave_max(mq);  // (non-negative floats order like their bit patterns)
      if (lane == 0) atomicMax(&scl[4 * set_now + 1], __builtin_bit_cast(int, mq));
    }
    if (ek < QI) {
      bf16x8_to_f32(rk, x);
      h8_t hv;
#pragma unroll
      for (int i = 0; i < 8; ++i) hv[i] = (_Float16)x[i];
      *(h8_t *)&kH[8 * ek] = hv;
    }
    if (ev < VI) {
      bf16x8_to_f32(rv, x);
      h8_t hv;
#pragma unroll
      for (int i = 0; i < 8; ++i) hv[i] = (_Float16)x[i];
      *(h8_t *)&vH[8 * ev] = hv;
    }
    if (wave_has_dy) {
      bf16x8_to_f32(rdy, x);
      if (edy < VI) {
        *(f4_t *)&dyS[8 * edy] = f4_t{x[0], x[1], x[2], x[3]};
        *(f4_t *)&dyS[8 * edy + 4] = f4_t{x[4], x[5], x[6], x[7]};
      }
      float md = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) md = fmaxf(md, fabsf(x[i]));
      md = wave_max(md);
      if (lane == 0) atomicMax(&scl[4 * set_now + 2], __builtin_bit_cast(int, md));
    }
    if (ef < CMAX) {
      if (a.gate_alpha) rf = gate_psi(rf, g_alpha, g_beta);
      const float gm = 1.f - rf;
      const h2_t m2 = {(_Float16)(gm * (-kInvC * kInvC)), (_Float16)(gm * (-kInvC * kInvC))};
      fB[ef * 4 + 0] = rf;
      fB[ef * 4 + 1] = __builtin_bit_cast(float, m2);
      fB[ef * 4 + 2] = gm;
    }
  };

  if (nck > 0) stage_load(nck - 1);
  asm volatile("" : "+v"(rq), "+v"(rk), "+v"(rv), "+v"(rdy), "+v"(rf));
  for (int it = 0; it <= nck; ++it) {
    const bool active = it >= 1;
    const int ck = nck - it;
    const int t0 = ck * C;
    const int len = active ? ((T - t0) < C ? (T - t0) : C) : 0;
    const int par = (it - 1) & 1;  // the end of the stash this chunk was pushed from
    set_now = it & 1;  // maxima that decide this chunk's scale
    if (active) {
      stage_store();
    }
    lds_barrier();  // P: this chunk's stash entries were completed by team A in the previous iteration
    // the other set was read one iteration ago and is filled again from the end of this one
    if (wave == 0 && lane < 4) scl[4 * (set_now ^ 1) + lane] = 0;
    if (active) {  // scale of this chunk (wave-uniform, identical in every wave of the team)
      const f4_t mx = __builtin_bit_cast(f4_t, *(const u4_t *)&scl[4 * set_now]);  // |carry|, |q|, |dy|
      const int e = ilog2f(fminf(fmaxf(mx[0] + mx[1] * mx[2], 1e-30f), 1e30f));
      const int grew = mx_e_prev > -(1 << 20) ? e - mx_e_prev : 0;
      const int extra = grew - 2 < 0 ? 0 : (grew - 2 > 12 ? 12 : grew - 2);
      int ne = 5 - extra - e;                                  // exponent of the new scale
      ne = ne > sc_e_min + 90 ? sc_e_min + 90 : ne;
      ne = ne < sc_e - 120 ? sc_e - 120 : ne;
      ne = ne > 120 ? 120 : (ne < -120 ? -120 : ne);
      sc_e_min = ne < sc_e_min ? ne : sc_e_min;
      mx_e_prev = e;
      const float ratio = pow2i(ne - sc_e);  // exact power of two
      sc_e = ne;
      sc = pow2i(ne);
      isc = pow2i(-ne);
#pragma unroll
      for (int r = 0; r < 4; ++r) carry[r] *= ratio;
#pragma unroll
      for (int c2 = 0; c2 < CT; ++c2) dWacc[c2] *= ratio;
    }
    f4_t dkacc = zero4, dvacc = zero4, dfacc = zero4;
    float G[4] = {0.f, 0.f, 0.f, 0.f};
    float fprev = 0.f;
    // LDS addressing of this team: a few per-lane base offsets, made opaque once per chunk so
    // that they are not hoisted out of the chunk loop as one register per (array, step);
    // every access below is base + compile-time immediate in the unrolled sweep.
    lchar *const l0 = (lchar *)lds;
    lchar *bH = l0 + (L::ST + rb * CT * 512 + lane * 8);      // stash slot 0: H, tile 0 of my row block
    lchar *bO = bH + ct * 512;                                // my own tile (H; Z one STASH_STEP later)
    lchar *bR4 = l0 + (rowb + 4 * ig) * 4;                    // q rows (fp32)
    lchar *bR2 = l0 + (rowb + 4 * ig) * 2;                    // k rows (fp16)
    lchar *bC4 = l0 + (col0 + jl) * 4;                        // dy column (fp32)
    lchar *bDw = l0 + rb * V * 32 + xch_item_off(col0 + jl, ig);       // dS write: item (column, rows 4 ig ..)
    lchar *bDr = l0 + rb * V * 32 + xch_frag_off<X32>(jl, ig, 0);      // dS fragment read (transposing),
    lchar *bDr1 = l0 + rb * V * 32 + xch_frag_off<X32>(jl, ig, 1);     // second half of a k = 32 fragment
    lchar *bV = l0 + (FE * ig + 32 * ct) * 2;                 // v slice of the dk MFMA
    lchar *bZero = l0;                                        // wave-uniform reads (f)
    int jlB = jl;  // opaque as well: the per-step column masks (jl == s) are then built per
                   // step instead of being kept in registers for every s of an unrolled sweep
    asm volatile("" : "+v"(bDr1));
    asm volatile("" : "+v"(bH), "+v"(bO), "+v"(bR4), "+v"(bR2), "+v"(bC4), "+v"(bDw), "+v"(bDr),
                 "+v"(bV), "+v"(bZero), "+v"(jlB));
    // The next chunk's vectors travel during this chunk.  Issued behind the set-up above: on
    // the tiles whose set-up reloads spilled registers, a reload behind the loads would wait
    // for them.  (Unconditional, as in team A; the first iteration fetches the last chunk
    // once more.)
    stage_load(ck > 0 ? ck - 1 : 0);
    // R2 of chunk step sp (swept one super-step earlier): carry = f G + dS W^T ; dk slice.
    // Its dS is in exchange buffer `rd`.
    auto R2 = [&](int sp, int rd) __attribute__((always_inline)) {
      FragT af[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        af[ks] = lds_ld_frag_tr<X32>(bDr, bDr1, L::DX + rd * ROWS * V * 2 + 1024 * ks);
      f4_t d = zero4;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        if constexpr (X32)
          d = mfma_k32(af[ks], wtf[ks], d);
        else
          d = mfma_k16(af[ks], wtf[ks], d);
      }
      settle(d);
#pragma unroll
      for (int r = 0; r < 4; ++r) carry[r] = fmaf(fprev, G[r], d[r]);
      if constexpr (CLIP) {
        const float cb = a.clip * sc;  // the sweep works on sc * gradient
#pragma unroll
        for (int r = 0; r < 4; ++r) carry[r] = __builtin_amdgcn_fmed3f(carry[r], -cb, cb);
      }
      // The contraction's result is consumed HERE, in the block that issued it, and the
      // consumer is pinned in front of the conditional block below.  With one MFMA in the
      // chain (V = 32) the compiler otherwise sinks these reads behind the branch and
      // counts the MFMA's wait states along the path through the dk block only: the waves
      // that skip it (ct >= KS) then read the accumulator while it is still being written
      // (wrong carry in two of a lane's four rows; caught by tile<32,32,2> in
      // tests/test_gpu_instantiations.py, the only tiling with a skipping wave and KS = 1).
      asm volatile("" : "+v"(carry[0]), "+v"(carry[1]), "+v"(carry[2]), "+v"(carry[3]));
      if (ct < KS) {
        // v_s in column sp of the B operand only: the other lanes read zeros
        const FragT bf = lds_ld<FragT>(jlB == sp ? bV + (L::VH_ + sp * V * 2) : bZero + L::ZERO_, 0);
        if constexpr (KS > 2) {
          // (this wave's own fragment read once more, as for dq in the recompute team)
          const FragT afk = lds_ld_frag_tr<X32>(bDr + 1024 * ct, bDr1 + 1024 * ct, L::DX + rd * ROWS * V * 2);
          dkacc = mfma_k32(afk, bf, dkacc);
        } else {
#pragma unroll
          for (int ks = 0; ks < KS; ++ks)
            if (ct == ks) {
              if constexpr (X32)
                dkacc = mfma_k32(af[ks], bf, dkacc);
              else
                dkacc = mfma_k16(af[ks], bf, dkacc);
            }
        }
      }
    };
    // E1 of chunk step s: G, df partial, dS into exchange buffer `wr`, row contractions
    auto E1 = [&](int s, int wr) __attribute__((always_inline)) {
      const u4_t fu = lds_ld<u4_t>(bZero, L::FB_ + s * 16);
      const float f = __builtin_bit_cast(float, fu[0]);
      const u2_t m4u = {fu[1], fu[1]};                          // -(1-f)/c^2 in fp16, four times
      // (element first, cast second: __builtin_bit_cast applied to the vector element
      //  expression itself reads element 0)
      const uint32_t gmu = fu[2];
      const float gm = __builtin_bit_cast(float, gmu);          // 1 - f in fp32
      const f4_t q4 = lds_ld<f4_t>(bR4, L::QS_ + s * ROWS * 4);
      const float dyj = sc * lds_ld<float>(bC4, L::DYS_ + s * V * 4);
      const int so = slot_of(s, par) * L::SLOT;  // byte offset of this step's slot
      const h4_t zp = lds_ld<h4_t>(bO + so, L::STASH_STEP);
      // (with 8 column tiles the register file cannot hold all H tiles next to the step's
      //  other operands: they are then fetched right before their MFMAs, see below)
      constexpr bool EARLY_H = CT <= 4;
      h4_t hfr[CT];
      if constexpr (EARLY_H) {
#pragma unroll
        for (int c2 = 0; c2 < CT; ++c2)
          hfr[c2] = lds_ld<h4_t>(bH + so, c2 * 512);
      }
      const h4_t hown = lds_ld<h4_t>(bO + so, 0);
      const bool mine = jlB == s;
      // k_s in row s of the A operand only: the other lanes read zeros
      const h4_t kfr = lds_ld<h4_t>(mine ? bR2 + (L::KH_ + s * ROWS * 2) : bZero + L::ZERO_, 0);
      // H' - Z' in packed fp16 (its inputs are fp16 stash values).  dS = (1-f) G (1 - Z^2) is
      // formed as  (1-f) G - G w,  w = (1-f) Z^2 : only the SMALL term w is packed fp16, the
      // leading term keeps 1 - f and G in fp32, and one mixed-precision FMA rounds the sum
      // straight to the fp16 MFMA operand.  (With the whole factor (1-f)(1 - Z^2) in fp16,
      // which is one vector multiply per element cheaper, the rounded factor is biased: Z^2
      // is mostly below one fp16 ulp of 1 - f, so the factor rounds up to fp16(1 - f) more
      // often than down, by 2.4e-5 on average; compounded through the W path of the Jacobian
      // that is +1 % on a gradient carried over 4096 steps, several % where memory is long.)
      const h4_t m4 = __builtin_bit_cast(h4_t, m4u);
      const h4_t hz = hown - zp;
      const h4_t ug = (zp * m4) * zp;   // = -w
      float dfl = 0.f;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        G[r] = fmaf(q4[r], dyj, carry[r]);
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
      }
      const h4_t dsp = __builtin_bit_cast(h4_t, dsu);
      lds_st<h4_t>(bDw, L::DX + wr * ROWS * V * 2, dsp);
#pragma unroll
      for (int c2 = 0; c2 < CT; ++c2) {
        if constexpr (!EARLY_H) hfr[c2] = lds_ld<h4_t>(bH + so, c2 * 512);
        dWacc[c2] = mfma_k16(hfr[c2], dsp, dWacc[c2]);
      }
      dvacc = mfma_k16(kfr, dsp, dvacc);
      // df_s = sum G (H' - Z') / c: fp32 MFMA against ones in column s adds the four lane
      // groups; the 16 rows of that column are added at the end of the chunk
      dfacc = __builtin_amdgcn_mfma_f32_16x16x4f32(dfl, mine ? 1.f : 0.f, dfacc, 0, 0, 0);
      fprev = f;
    };
    // Super-step u sweeps chunk step len - 1 - u (E1) and finishes step len - u (R2).
    // (A fully unrolled sweep with compile-time step indices was measured 20 % slower than
    //  a loop, unlike the recompute team's and the forward kernel's.)
    if constexpr (V > 64) {
      // First and last super-steps peeled: the loop between them carries no per-step
      // conditions (11 scalar instructions per step fewer); the workgroup's barrier count
      // per chunk stays C.  Measured 6 % on the 128-wide tile; on the 64-wide tiles the same
      // form is 1 % SLOWER than the plain loop below, so they keep that.
      int cur = 0, sprev = 0;
      if (len > 0) {
        E1(len - 1, 0);
        sprev = len - 1;
        cur = 1;
      }
      lds_barrier();
#pragma nounroll
      for (int u = 1; u < len; ++u) {
        const int s = len - 1 - u;
        R2(sprev, cur ^ 1);
        E1(s, cur);
        sprev = s;
        cur ^= 1;
        lds_barrier();
      }
      if (len == C) {
        if (active) R2(sprev, cur ^ 1);
      } else {
        // a short chunk: its first step is finished at super-step len, the rest only keep step
        if (len > 0) R2(sprev, cur ^ 1);
#pragma nounroll
        for (int u = len > 0 ? len : 1; u < C; ++u) lds_barrier();
      }
    } else {
      int cur = 0, sprev = 0;
#pragma nounroll
      for (int u = 0; u < C; ++u) {
        const int s = len - 1 - u;  // chunk step of this super-step (reverse order)
        if (u > 0 && u <= len) R2(sprev, cur ^ 1);
        if (u < len) {
          E1(s, cur);
          sprev = s;
          cur ^= 1;
        }
        lds_barrier();
      }
      // R2 of the chunk's first step; a short chunk already ran it at super-step u == len
      if (active && len == C) R2(sprev, cur ^ 1);
    }
    // (the next chunk's prefetch is waited for in front of the end-of-chunk stores: see team A)
    asm volatile("" : "+v"(rq), "+v"(rk), "+v"(rv), "+v"(rdy), "+v"(rf));
    {  // largest true |carry| of this wave, for the next chunk's scale
      float mc = fmaxf(fmaxf(fabsf(carry[0]), fabsf(carry[1])), fmaxf(fabsf(carry[2]), fabsf(carry[3])));
      mc = wave_max(mc) * isc;
      if (lane == 0) atomicMax(&scl[4 * (set_now ^ 1)], __builtin_bit_cast(int, mc));
    }
    lds_barrier();  // E1: every read of the exchange buffers is done: they take the partials
    // partials: dk slices behind team A's dq slices in A's exchange buffer, dv in B's own
    f4_t *fink = (f4_t *)(lds + L::HX) + RB * KS * 64;  // [RB][KS][64]
    f4_t *finv = (f4_t *)(lds + L::DX);                 // [WAVES][64]
    // Store addresses below: wave-uniform 64-bit base + 32-bit byte offset rebuilt from the
    // lane index on the spot.  Kept in registers over the chunk they would be spilled, and a
    // reload from scratch in front of a store waits for every store issued before it.
    int ll = lane_now();
    asm volatile("" : "+v"(ll));
    const uint32_t jl2 = ll & 15, ig2 = ll >> 4;
    if (active) {
      if (ct < KS) fink[(rb * KS + ct) * 64 + ll] = dkacc * isc;
      finv[wave * 64 + ll] = dvacc * isc;
      float x = (dfacc[0] + dfacc[1]) + (dfacc[2] + dfacc[3]);
      x += __shfl_xor(x, 16, 64);
      x += __shfl_xor(x, 32, 64);
      if (ll < 16 && (int)jl2 < len) {
        // partials as [wave of the state][B][N][T]: the chunk's steps of a wave are adjacent.
        // (In the output's own [B][T][N] order every lane writes four bytes into a line that
        //  the workgroups of the other heads, on other XCDs, write at the same time: those
        //  stores alone cost 7 % of the kernel.)
        char *base = (char *)(ws.dfp + (((size_t)(part * WAVES + wave) * a.B + b) * N + n) * T + t0);
        *(float *)(base + 4u * jl2) = x * (kInvC * isc);
      }
    }
    lds_barrier();  // E2
    if (active) {
      if (ct == 0 && (int)jl2 < len) {
        f4_t d = fink[(rb * KS + 0) * 64 + ll];
#pragma unroll
        for (int ks = 1; ks < KS; ++ks) d += fink[(rb * KS + ks) * 64 + ll];
        if (ws.dkh) {
          char *base = (char *)(ws.dkh + (((size_t)b * T + t0) * N + n) * K + row_base + rowb);
          *(f4_t *)(base + 4u * (jl2 * (uint32_t)(N * K) + 4u * ig2)) = d;
        } else {
          char *base = (char *)((bf16_raw *)a.dk + (((size_t)b * T + t0) * a.Nqk + g) * K + row_base + rowb);
          *(uint2 *)(base + 2u * (jl2 * kstride + 4u * ig2)) = pack4_bf16(d);
        }
      }
      if (rb == 0) {
        f4_t d = finv[(0 * CT + ct) * 64 + ll];
#pragma unroll
        for (int r2 = 1; r2 < RB; ++r2) d += finv[(r2 * CT + ct) * 64 + ll];
        const size_t row0 = (((size_t)b * T + t0) * N + n) * V + col0;  // uniform: step t0, column col0
        const uint32_t eoff = 4u * ig2 * vstride + jl2;                 // element offset of (step 4 ig, column jl)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int sc = 4 * (int)ig2 + r;
          if (sc < len) {
            const uint32_t eo = eoff + (uint32_t)r * vstride;
            if constexpr (TL::P == 1) {
              float x = d[r];
              if (a.w_r)  // y_t holds w_r (.) v_t as well
                x = fmaf(bf16_to_f32(((const bf16_raw *)a.w_r)[n * V + col0 + (int)jl2]),
                         bf16_to_f32(*(const bf16_raw *)((const char *)(dyg + row0) + 2u * eo)), x);
              *(bf16_raw *)((char *)((bf16_raw *)a.dv + row0) + 2u * eo) = f32_to_bf16(x);
            } else
              *(float *)((char *)(ws.dvp + (size_t)part * a.B * T * N * V + row0) + 4u * eo) = d[r];
          }
        }
      }
    }
    lds_barrier();  // E3
  }

  if (a.dH0)
#pragma unroll
    for (int r = 0; r < 4; ++r) a.dH0[st_off + (size_t)r * V] = carry[r] * isc;
  {
    float *dst = ws.dWp + (((size_t)unit * TL::P + part) * RB + rb) * V * V;
#pragma unroll
    for (int c2 = 0; c2 < CT; ++c2)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        dst[(size_t)(c2 * 16 + 4 * ig + r) * V + col0 + jl] = dWacc[c2][r] * (kInvC * isc);
  }
}

// dv = bf16(sum of its P parts [+ w_r (.) dy for the residual of the y equation]) when the
// state is split over workgroups; df = sum of its per-wave partials.  Fixed (increasing)
// order in both.  NV = N * V, the period of w_r along the flat index.
__global__ void bwd_parts_sum_kernel(const float *__restrict__ dvp, bf16_raw *__restrict__ dv,
                                     size_t n_dv, int P, const float *__restrict__ dfp,
                                     float *__restrict__ df, size_t n_df, int NP,
                                     const bf16_raw *__restrict__ w_r,
                                     const bf16_raw *__restrict__ dy, int NV, int T, int N) {
  const size_t tid = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  if (P > 1) {  // four consecutive elements per thread (V is a multiple of 16)
    for (size_t e = 4 * tid; e < n_dv; e += 4 * stride) {
      f4_t s = *(const f4_t *)&dvp[e];
      for (int p = 1; p < P; ++p) s += *(const f4_t *)&dvp[(size_t)p * n_dv + e];
      if (w_r) {
        const uint2 wv = *(const uint2 *)&w_r[e % (size_t)NV];
        const uint2 dv2 = *(const uint2 *)&dy[e];
        s[0] = fmaf(bf16_to_f32(wv.x & 0xFFFFu), bf16_to_f32(dv2.x & 0xFFFFu), s[0]);
        s[1] = fmaf(bf16_to_f32(wv.x >> 16), bf16_to_f32(dv2.x >> 16), s[1]);
        s[2] = fmaf(bf16_to_f32(wv.y & 0xFFFFu), bf16_to_f32(dv2.y & 0xFFFFu), s[2]);
        s[3] = fmaf(bf16_to_f32(wv.y >> 16), bf16_to_f32(dv2.y >> 16), s[3]);
      }
      *(uint2 *)&dv[e] = pack4_bf16(s);
    }
  }
  // df [B][T][N] from partials [NP][B][N][T]
  if ((T & 3) == 0) {
    // four consecutive steps of one (b, n) per thread: the partial rows are read as 16-byte
    // pieces that consecutive lanes continue, the four results go to four rows of df
    const size_t T4 = (size_t)T / 4;
    for (size_t e = tid; e < n_df / 4; e += stride) {
      const size_t bn = e / T4, t4 = e - bn * T4;
      const size_t src = bn * (size_t)T + 4 * t4;
      f4_t s = *(const f4_t *)&dfp[src];
      for (int p = 1; p < NP; ++p) s += *(const f4_t *)&dfp[(size_t)p * n_df + src];
      const size_t b = bn / (size_t)N, n = bn - b * (size_t)N;
      float *dst = df + (b * (size_t)T + 4 * t4) * (size_t)N + n;
#pragma unroll
      for (int r = 0; r < 4; ++r) dst[(size_t)r * N] = s[r];
    }
  } else {
    for (size_t e = tid; e < n_df; e += stride) {
      const int n = (int)(e % (size_t)N);
      const size_t bt = e / (size_t)N;
      const int t = (int)(bt % (size_t)T);
      const size_t b = bt / (size_t)T;
      const size_t src = (b * N + n) * (size_t)T + t;
      float s = dfp[src];
      for (int p = 1; p < NP; ++p) s += dfp[(size_t)p * n_df + src];
      df[e] = s;
    }
  }
}

// dW[n] = sum over b, then over the (part, row block) partials, in increasing order
__global__ void dw_parts_sum_kernel(const float *__restrict__ dWp, float *__restrict__ dW, int B,
                                    int N, int VV, int parts) {
  const size_t total = (size_t)N * VV;
  for (size_t e = blockIdx.x * (size_t)blockDim.x + threadIdx.x; e < total;
       e += (size_t)gridDim.x * blockDim.x) {
    const int n = e / VV, r = e - (size_t)n * VV;
    // (b, p) in increasing order, dealt to four running sums that are added pairwise at the
    // end: a fixed order with four loads in flight (a single running sum is one chain of
    // dependent loads, and this kernel is a few hundred workgroups)
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    const int terms = B * parts;
    int t = 0;
    for (; t + 4 <= terms; t += 4) {
      float x[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int b = (t + k) / parts, p = (t + k) - b * parts;
        x[k] = dWp[(((size_t)b * N + n) * parts + p) * VV + r];
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) acc[k] += x[k];
    }
    for (int k = 0; t < terms; ++t, ++k) {
      const int b = t / parts, p = t - b * parts;
      acc[k] += dWp[(((size_t)b * N + n) * parts + p) * VV + r];
    }
    dW[e] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
  }
}

__global__ void head_sum_bf16_kernel(const float *__restrict__ per_head, bf16_raw *__restrict__ out,
                                     size_t BT, int N, int Nqk, int K) {
  // Four adjacent elements per thread (16-byte loads), and four interleaved running sums over
  // the heads of a group (heads h, h + 4, ... each), added pairwise at the end: a fixed order
  // that keeps four loads in flight instead of one chain of dependent loads.
  const int per = N / Nqk;
  const int K4 = K / 4;
  const size_t total = BT * Nqk * K4;
  for (size_t e = blockIdx.x * (size_t)blockDim.x + threadIdx.x; e < total;
       e += (size_t)gridDim.x * blockDim.x) {
    const int i4 = e % K4;
    const size_t r = e / K4;
    const int g = r % Nqk;
    const size_t bt = r / Nqk;
    const f4_t *src = (const f4_t *)(per_head + ((bt * N) + (size_t)g * per) * K) + i4;
    const f4_t z4 = {0.f, 0.f, 0.f, 0.f};
    f4_t acc[4] = {z4, z4, z4, z4};
    int h = 0;
    for (; h + 4 <= per; h += 4) {
      f4_t x[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) x[k] = src[(size_t)(h + k) * K4];
#pragma unroll
      for (int k = 0; k < 4; ++k) acc[k] += x[k];
    }
    for (int k = 0; h < per; ++h, ++k) acc[k] += src[(size_t)h * K4];
    const f4_t sum = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    *(uint2 *)&out[4 * e] = pack4_bf16(sum);
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
  const int waves = RB * (V / 16);
  w.dvp = off; off += P > 1 ? align256((size_t)P * B * T * N * V * 4) : 0;
  w.dfp = off; off += align256((size_t)P * waves * B * T * N * 4);
  w.dWp = off; off += align256((size_t)B * N * P * RB * V * V * 4);
  const size_t heads = Nqk != N ? align256((size_t)B * T * N * K * 4) : 0;
  w.dqh = off; off += heads;
  w.dkh = off; off += heads;
  w.total = off;
  return w;
}

// T == 0: nothing is swept; dH0 = dHT (or 0) and dW = 0.  (The scan kernel is not launched:
// its checkpoint prefetch has nothing valid to read, the caller may pass ckpt = NULL.)
__global__ void bwd_empty_kernel(const float *__restrict__ dHT, float *__restrict__ dH0,
                                 size_t n_state, float *__restrict__ dW, size_t n_dW) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t e = blockIdx.x * (size_t)blockDim.x + threadIdx.x; e < n_dW; e += stride) dW[e] = 0.f;
  if (dH0)
    for (size_t e = blockIdx.x * (size_t)blockDim.x + threadIdx.x; e < n_state; e += stride)
      dH0[e] = dHT ? dHT[e] : 0.f;
}

template <typename TL>
hipError_t launch_bwd(const BwdArgs &a, hipStream_t s) {
  static_assert(OvLds<TL>::OK, "tile does not fit the two-team kernel");
  const int units = a.B * a.N;
  if (a.T == 0) {
    const size_t n_state = (size_t)units * a.K * a.V, n_dW = (size_t)a.N * a.V * a.V;
    hipLaunchKernelGGL(bwd_empty_kernel, dim3(grid_for(n_state > n_dW ? n_state : n_dW, 256)),
                       dim3(256), 0, s, a.dHT, a.dH0, n_state, a.dW, n_dW);
    return hipGetLastError();
  }
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
    if (a.C > OvLds<TL>::CMAX) return hipErrorInvalidValue;
    auto *kern = a.clip > 0.f ? mfma_bwd_overlap_kernel<TL, true> : mfma_bwd_overlap_kernel<TL, false>;
    e = a.clip > 0.f ? set_max_lds_once(mfma_bwd_overlap_kernel<TL, true>, OvLds<TL>::BYTES)
                     : set_max_lds_once(mfma_bwd_overlap_kernel<TL, false>, OvLds<TL>::BYTES);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(grid_blocks(units, TL::P)), dim3(2 * TL::THREADS),
                       OvLds<TL>::BYTES, s, a, ws);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (a.T > 0) {
      {
        const size_t n_dv = (size_t)a.B * a.T * a.N * a.V, n_df = (size_t)a.B * a.T * a.N;
        hipLaunchKernelGGL(bwd_parts_sum_kernel, dim3(grid_for((TL::P > 1 ? n_dv : n_df) / 4 + 1, 256)),
                           dim3(256), 0, s, (const float *)ws.dvp, (bf16_raw *)a.dv, n_dv, TL::P,
                           (const float *)ws.dfp, a.df, n_df, TL::P * TL::WAVES,
                           (const bf16_raw *)a.w_r, (const bf16_raw *)a.dy, a.N * a.V, a.T, a.N);
      }
      if (shared) {
        const size_t total = (size_t)a.B * a.T * a.Nqk * a.K / 4;
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

// epilogues shared with the register-resident backward (m2rnn_rowwave_bwd.hip)
hipError_t bwd_sum_dW(const float *dWp, float *dW, int B, int N, int VV, int parts, hipStream_t s) {
  hipLaunchKernelGGL(dw_parts_sum_kernel, dim3(grid_for((size_t)N * VV, 256)), dim3(256), 0, s, dWp,
                     dW, B, N, VV, parts);
  return hipGetLastError();
}
hipError_t bwd_sum_heads(const float *per_head, void *out, size_t BT, int N, int Nqk, int K,
                         hipStream_t s) {
  hipLaunchKernelGGL(head_sum_bf16_kernel, dim3(grid_for(BT * Nqk * K / 4, 256)), dim3(256), 0, s,
                     per_head, (bf16_raw *)out, BT, N, Nqk, K);
  return hipGetLastError();
}
hipError_t bwd_empty(const BwdArgs &a, hipStream_t s) {
  const size_t n_state = (size_t)a.B * a.N * a.K * a.V, n_dW = (size_t)a.N * a.V * a.V;
  hipLaunchKernelGGL(bwd_empty_kernel, dim3(grid_for(n_state > n_dW ? n_state : n_dW, 256)),
                     dim3(256), 0, s, a.dHT, a.dH0, n_state, a.dW, n_dW);
  return hipGetLastError();
}

hipError_t mfma_bwd(const BwdArgs &a, hipStream_t s) {
  // V = 16: one wave owns a row block with all its columns (no exchange, no per-step barrier)
  if (rowwave_bwd_supported(a.K, a.V)) return rowwave_bwd(a, s);
  const int rb = mfma_pick_rb(a.K, a.V, a.B * a.N);
#define X(K_, V_, RB_)                                                   \
  if constexpr (V_ != 16)                                                \
    if (a.K == K_ && a.V == V_ && rb == RB_) return launch_bwd<Tile<K_, V_, RB_>>(a, s);
  M2RNN_TILE_CASES(X)
#undef X
  return hipErrorInvalidValue;
}

size_t mfma_bwd_workspace_bytes(int B, int T, int N, int Nqk, int K, int V) {
  if (rowwave_bwd_supported(K, V)) return rowwave_bwd_workspace_bytes(B, T, N, Nqk, K, V);
  const int rb = mfma_pick_rb(K, V, B * N);
#define X(K_, V_, RB_) \
  if (K == K_ && V == V_ && rb == RB_) return ws_bytes<Tile<K_, V_, RB_>>(B, T, N, Nqk);
  M2RNN_TILE_CASES(X)
#undef X
  return 0;
}

int mfma_bwd_max_chunk(int K, int V) {
  if (rowwave_bwd_supported(K, V)) return rowwave_bwd_max_chunk();
  int best = kChunkCap;
#define X(K_, V_, RB_) \
  if (K == K_ && V == V_) {                                                                 \
    const int c = OvLds<Tile<K_, V_, RB_>>::CMAX;                                          \
    if (c < best) best = c;                                                                \
  }
  M2RNN_TILE_CASES(X)
#undef X
  return best;
}

}  // namespace m2rnn

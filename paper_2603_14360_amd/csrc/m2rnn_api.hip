// Host side of the C ABI declared in include/m2rnn.h: descriptor validation,
// workspace sizing and the choice of kernel family.  No arithmetic of the
// method happens here.
#include "../../include/m2rnn.h"

#include <atomic>

#include "m2rnn_kernels.hpp"
#include "m2rnn_mfma_common.hpp"

using namespace m2rnn;

namespace {

bool dim_ok(int d) { return d == 16 || d == 32 || d == 64 || d == 128; }

m2rnn_status check_desc(const m2rnn_desc *d) {
  if (!d) return M2RNN_ERR_NULL;
  if (d->io != M2RNN_F32 && d->io != M2RNN_BF16) return M2RNN_ERR_DTYPE;
  if (d->B < 0 || d->T < 0 || d->N < 1 || d->Nqk < 1) return M2RNN_ERR_SHAPE;
  if (d->N % d->Nqk != 0) return M2RNN_ERR_SHAPE;
  if (!dim_ok(d->K) || !dim_ok(d->V)) return M2RNN_ERR_SHAPE;
  if (d->flags != 0) return M2RNN_ERR_SHAPE;
  // index arithmetic inside the kernels is 64-bit, but per-tensor element
  // counts must stay below 2^40 to keep byte offsets far from overflow
  const double big = (double)d->B * (double)(d->T > 0 ? d->T : 1) * d->N * d->K * d->V;
  if (big > 1e15) return M2RNN_ERR_SHAPE;
  return M2RNN_OK;
}

// Which kernel family serves this descriptor.  The checkpoint layout is common
// to all families, so forward and backward may come from different ones.
enum Family { kGeneric = 0, kMfma = 1, kRowWave = 2, kDecode = 3 };

Family family_of(const m2rnn_desc *d) {  // backward (it owns the chunk limits)
  if (d->io == M2RNN_BF16 && (mfma_supported(d->K, d->V) || rowwave_bwd_supported(d->K, d->V)))
    return kMfma;
  return kGeneric;
}

Family fwd_family_of(const m2rnn_desc *d) {
  // one token per call: the latency kernel (one launch, state through HBM once, no staging)
  if (d->io == M2RNN_BF16 && d->T == 1 && decode_supported(d->K, d->V)) return kDecode;
  // The register-resident kernel needs no LDS exchange but one wave carries a
  // whole 16-row block; it pays off once there are enough row blocks for at
  // least two waves per SIMD (1024 SIMDs).  Below that the tiled kernel, which
  // spreads a row block over V/16 waves, keeps more of the chip busy.
  if (d->io == M2RNN_BF16 && rowwave_supported(d->K, d->V)) {
    const long long row_blocks = (long long)d->B * d->N * (d->K / 16);
    if (row_blocks >= 2048 || !mfma_supported(d->K, d->V)) return kRowWave;
  }
  return family_of(d);
}

hipError_t run_fwd(const m2rnn_desc *d, const FwdArgs &a, hipStream_t s) {
  switch (fwd_family_of(d)) {
    case kDecode: return decode_fwd(a, s);
    case kRowWave: return rowwave_fwd(a, s);
    case kMfma: return mfma_fwd(a, s);
    default: return generic_fwd(a, s);
  }
}

int default_chunk(const m2rnn_desc *d) {
  return family_of(d) == kMfma ? mfma_default_chunk(d->K, d->V)
                               : generic_default_chunk(d->K, d->V);
}
int max_chunk(const m2rnn_desc *d) {
  return family_of(d) == kMfma ? mfma_max_chunk(d->K, d->V) : generic_max_chunk(d->K, d->V);
}

// Resolves desc.chunk; returns 0 if it is out of range.
int resolve_chunk(const m2rnn_desc *d) {
  if (d->chunk == 0) return default_chunk(d);
  if (d->chunk < 0 || d->chunk > max_chunk(d)) return 0;
  return d->chunk;
}

size_t ckpt_bytes(const m2rnn_desc *d, int C) {
  if (d->T == 0) return 0;
  return (size_t)d->B * d->N * ceil_div(d->T, C) * d->K * d->V * sizeof(float);
}

size_t family_ws(const m2rnn_desc *d, int C, int bwd) {
  const Family fam = bwd ? family_of(d) : fwd_family_of(d);
  if (fam == kRowWave || fam == kDecode) return 0;
  return fam == kMfma ? mfma_workspace_bytes(d->B, d->T, d->N, d->Nqk, d->K, d->V, C, bwd)
                      : generic_workspace_bytes(d->B, d->T, d->N, d->Nqk, d->K, d->V, C, bwd);
}

bool misaligned(const void *p) { return ((uintptr_t)p & 15u) != 0; }

// Carve-up of the backward's workspace: [partial sums | own checkpoints (only when the
// backward recomputes them itself) | dw_r scratch | gate scratch].
struct BwdWsLayout {
  size_t main, ckpt, dwr, gate, total;
};
BwdWsLayout bwd_ws(const m2rnn_desc *d, int C, bool own_ckpt) {
  BwdWsLayout w;
  const size_t b = family_ws(d, C, 1), f = own_ckpt ? family_ws(d, C, 0) : 0;  // pass 1 borrows `main`
  w.main = align256(b > f ? b : f);
  w.ckpt = own_ckpt ? align256(ckpt_bytes(d, C)) : 0;
  w.dwr = residual_dw_r_scratch_bytes(d->N, d->V);
  w.gate = gate_scratch_bytes(d->N);
  w.total = w.main + w.ckpt + w.dwr + w.gate;
  return w;
}

// Library-owned scratch of m2rnn_fwd_static: one array per GPU, alive until the process ends.
// The name below is a host-side handle only; the device address is looked up once per device
// (each GPU holds its own copy at its own address) and only that address is handed to kernels.
static __device__ __align__(256) unsigned char scratch[M2RNN_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

void *static_scratch_of_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
    g_scratch_ptr[dev].store(p, std::memory_order_release);  // racing threads store the same value
  }
  return p;
}

m2rnn_status fwd_impl(const m2rnn_desc *desc, const m2rnn_opts *opts, const void *q,
                      const void *k, const void *v, const float *f, const void *W,
                      const float *H0, void *y, float *HT, float *ckpt, void *workspace,
                      size_t workspace_bytes, void *hip_stream) {
  m2rnn_status st = check_desc(desc);
  if (st != M2RNN_OK) return st;
  const int C = resolve_chunk(desc);
  if (!C) return M2RNN_ERR_CHUNK;
  const bool empty = desc->B == 0;
  const bool steps = !empty && desc->T > 0;
  if (!W) return M2RNN_ERR_NULL;
  if (steps && (!q || !k || !v || !f || !y)) return M2RNN_ERR_NULL;
  const void *w_r = opts ? opts->w_r : nullptr;
  const float *ga = opts ? opts->gate_alpha : nullptr, *gb = ga ? opts->gate_beta : nullptr;
  if (ga && !gb) return M2RNN_ERR_NULL;
  const void *ptrs[] = {q, k, v, f, W, H0, y, HT, ckpt, workspace, w_r, ga, gb};
  for (const void *p : ptrs)
    if (misaligned(p)) return M2RNN_ERR_ALIGN;
  const size_t need = family_ws(desc, C, 0);
  if (need > 0 && (!workspace || workspace_bytes < need))
    return workspace ? M2RNN_ERR_WORKSPACE : M2RNN_ERR_NULL;

  FwdArgs a;
  a.B = desc->B; a.T = desc->T; a.N = desc->N; a.Nqk = desc->Nqk; a.K = desc->K; a.V = desc->V;
  a.C = C; a.io = desc->io;
  a.q = q; a.k = k; a.v = v; a.W = W; a.f = f; a.H0 = H0;
  a.y = y; a.HT = HT; a.ckpt = ckpt; a.write_y = 1; a.ws = (char *)workspace;
  a.w_r = w_r; a.gate_alpha = ga; a.gate_beta = gb;
  hipStream_t s = (hipStream_t)hip_stream;
  const hipError_t e = run_fwd(desc, a, s);
  return e == hipSuccess ? M2RNN_OK : M2RNN_ERR_HIP;
}

}  // namespace

extern "C" {

const char *m2rnn_status_string(m2rnn_status s) {
  switch (s) {
    case M2RNN_OK: return "ok";
    case M2RNN_ERR_NULL: return "required pointer is NULL";
    case M2RNN_ERR_SHAPE: return "unsupported shape (K, V in {16,32,64,128}; Nqk must divide N)";
    case M2RNN_ERR_DTYPE: return "unknown io dtype";
    case M2RNN_ERR_ALIGN: return "pointer is not 16-byte aligned";
    case M2RNN_ERR_WORKSPACE: return "workspace too small";
    case M2RNN_ERR_HIP: return "HIP call failed";
    case M2RNN_ERR_CHUNK: return "checkpoint interval out of range";
  }
  return "unknown status";
}

int32_t m2rnn_default_chunk(const m2rnn_desc *desc) {
  return check_desc(desc) == M2RNN_OK ? default_chunk(desc) : 0;
}

int32_t m2rnn_max_chunk(const m2rnn_desc *desc) {
  return check_desc(desc) == M2RNN_OK ? max_chunk(desc) : 0;
}

size_t m2rnn_ckpt_bytes(const m2rnn_desc *desc) {
  if (check_desc(desc) != M2RNN_OK) return 0;
  const int C = resolve_chunk(desc);
  return C ? ckpt_bytes(desc, C) : 0;
}

const char *m2rnn_route_string(const m2rnn_desc *desc, int bwd) {
  if (check_desc(desc) != M2RNN_OK) return "invalid descriptor";
  const Family fam = bwd ? family_of(desc) : fwd_family_of(desc);
  if (fam == kGeneric) return desc->io == M2RNN_F32 ? "generic<f32>" : "generic<bf16>";
  if (fam == kDecode) {
#define X(K_, V_) \
  if (desc->K == K_ && desc->V == V_) return "decode<" #K_ "," #V_ ">";
    M2RNN_ROWWAVE_CASES(X)
#undef X
    return "decode<?>";
  }
  if (fam == kRowWave) {
#define X(K_, V_) \
  if (desc->K == K_ && desc->V == V_) return "rowwave<" #K_ "," #V_ ">";
    M2RNN_ROWWAVE_CASES(X)
#undef X
    return "rowwave<?>";
  }
  if (bwd && rowwave_bwd_supported(desc->K, desc->V)) {
    if (desc->K == 16) return "rowwave_bwd<16,16>";
    if (desc->K == 32) return "rowwave_bwd<32,16>";
    if (desc->K == 64) return "rowwave_bwd<64,16>";
    if (desc->K == 128) return "rowwave_bwd<128,16>";
    return "rowwave_bwd<?>";
  }
  const int rb = mfma_pick_rb(desc->K, desc->V, desc->B * desc->N);
#define X(K_, V_, RB_) \
  if (desc->K == K_ && desc->V == V_ && rb == RB_) return "tile<" #K_ "," #V_ "," #RB_ ">";
  M2RNN_TILE_CASES(X)
#undef X
  return "tile<?>";
}

size_t m2rnn_workspace_bytes(const m2rnn_desc *desc, int bwd) {
  if (check_desc(desc) != M2RNN_OK) return 0;
  const int C = resolve_chunk(desc);
  if (!C) return 0;
  return bwd ? bwd_ws(desc, C, bwd >= 2).total : family_ws(desc, C, 0);
}

m2rnn_status m2rnn_fwd(const m2rnn_desc *desc, const void *q, const void *k, const void *v,
                       const float *f, const void *W, const float *H0, void *y, float *HT,
                       float *ckpt, void *workspace, size_t workspace_bytes, void *hip_stream) {
  return m2rnn_fwd_opt(desc, nullptr, q, k, v, f, W, H0, y, HT, ckpt, workspace, workspace_bytes,
                       hip_stream);
}

m2rnn_status m2rnn_fwd_opt(const m2rnn_desc *desc, const m2rnn_opts *opts, const void *q,
                           const void *k, const void *v, const float *f, const void *W,
                           const float *H0, void *y, float *HT, float *ckpt, void *workspace,
                           size_t workspace_bytes, void *hip_stream) {
  return fwd_impl(desc, opts, q, k, v, f, W, H0, y, HT, ckpt, workspace, workspace_bytes,
                  hip_stream);
}

m2rnn_status m2rnn_fwd_static(const m2rnn_desc *desc, const m2rnn_opts *opts, const void *q,
                              const void *k, const void *v, const float *f, const void *W,
                              const float *H0, void *y, float *HT, float *ckpt,
                              void *hip_stream) {
  m2rnn_status st = check_desc(desc);
  if (st != M2RNN_OK) return st;
  const int C = resolve_chunk(desc);
  if (!C) return M2RNN_ERR_CHUNK;
  const size_t need = family_ws(desc, C, 0);
  if (need > (size_t)M2RNN_STATIC_SCRATCH_BYTES) return M2RNN_ERR_WORKSPACE;
  void *scratch_ptr = nullptr;
  if (need > 0 && desc->B > 0 && desc->T > 0) {
    scratch_ptr = static_scratch_of_current_device();
    if (!scratch_ptr) return M2RNN_ERR_HIP;
  }
  return fwd_impl(desc, opts, q, k, v, f, W, H0, y, HT, ckpt, scratch_ptr,
                  scratch_ptr ? (size_t)M2RNN_STATIC_SCRATCH_BYTES : 0, hip_stream);
}

m2rnn_status m2rnn_bwd(const m2rnn_desc *desc, const void *q, const void *k, const void *v,
                       const float *f, const void *W, const float *H0, const float *ckpt,
                       const void *dy, const float *dHT, void *dq, void *dk, void *dv, float *df,
                       float *dW, float *dH0, void *workspace, size_t workspace_bytes,
                       void *hip_stream) {
  return m2rnn_bwd_opt(desc, nullptr, q, k, v, f, W, H0, ckpt, dy, dHT, dq, dk, dv, df, dW, dH0,
                       workspace, workspace_bytes, hip_stream);
}

m2rnn_status m2rnn_bwd_opt(const m2rnn_desc *desc, const m2rnn_opts *opts, const void *q,
                           const void *k, const void *v, const float *f, const void *W,
                           const float *H0, const float *ckpt, const void *dy, const float *dHT,
                           void *dq, void *dk, void *dv, float *df, float *dW, float *dH0,
                           void *workspace, size_t workspace_bytes, void *hip_stream) {
  m2rnn_status st = check_desc(desc);
  if (st != M2RNN_OK) return st;
  const int C = resolve_chunk(desc);
  if (!C) return M2RNN_ERR_CHUNK;
  const bool steps = desc->B > 0 && desc->T > 0;
  if (!W || !dW) return M2RNN_ERR_NULL;
  if (steps && (!q || !k || !v || !f || !dy || !dq || !dk || !dv || !df)) return M2RNN_ERR_NULL;
  const void *w_r = opts ? opts->w_r : nullptr;
  float *dw_r = w_r ? opts->dw_r : nullptr;
  if (w_r && !dw_r) return M2RNN_ERR_NULL;
  const float *ga = opts ? opts->gate_alpha : nullptr, *gb = ga ? opts->gate_beta : nullptr;
  float *dga = ga ? opts->dgate_alpha : nullptr, *dgb = ga ? opts->dgate_beta : nullptr;
  if (ga && (!gb || !dga || !dgb)) return M2RNN_ERR_NULL;
  const void *ptrs[] = {q,  k,  v,  f,   W,   H0,        ckpt, dy,   dHT, dq, dk,
                        dv, df, dW, dH0, workspace, w_r, dw_r, ga,  gb,  dga, dgb};
  for (const void *p : ptrs)
    if (misaligned(p)) return M2RNN_ERR_ALIGN;
  const BwdWsLayout wl = bwd_ws(desc, C, /*own_ckpt=*/ckpt == nullptr);
  const size_t need = wl.total;
  if (need > 0 && (!workspace || workspace_bytes < need))
    return workspace ? M2RNN_ERR_WORKSPACE : M2RNN_ERR_NULL;

  hipStream_t s = (hipStream_t)hip_stream;
  const Family fam = family_of(desc);
  char *ws = (char *)workspace;
  const size_t dwr_bytes = wl.dwr;
  const size_t gate_bytes = wl.gate;
  const size_t main_bytes = wl.main;
  if (!ckpt && steps) {
    // The paper's pass 1, keeping one state per chunk: rerun the recurrence
    // from H0 without the readout, into the tail of the workspace.
    float *own = (float *)(ws + main_bytes);
    FwdArgs fa;
    fa.B = desc->B; fa.T = desc->T; fa.N = desc->N; fa.Nqk = desc->Nqk; fa.K = desc->K;
    fa.V = desc->V; fa.C = C; fa.io = desc->io;
    fa.q = q; fa.k = k; fa.v = v; fa.W = W; fa.f = f; fa.H0 = H0;
    fa.y = nullptr; fa.HT = nullptr; fa.ckpt = own; fa.write_y = 0; fa.ws = ws;
    fa.w_r = nullptr; fa.gate_alpha = ga; fa.gate_beta = gb;
    const hipError_t e = run_fwd(desc, fa, s);
    if (e != hipSuccess) return M2RNN_ERR_HIP;
    ckpt = own;
  }
  BwdArgs a;
  a.B = desc->B; a.T = desc->T; a.N = desc->N; a.Nqk = desc->Nqk; a.K = desc->K; a.V = desc->V;
  a.C = C; a.io = desc->io;
  a.q = q; a.k = k; a.v = v; a.W = W; a.dy = dy; a.f = f; a.H0 = H0; a.ckpt = ckpt; a.dHT = dHT;
  a.dq = dq; a.dk = dk; a.dv = dv; a.df = df; a.dW = dW; a.dH0 = dH0; a.ws = ws;
  a.w_r = w_r; a.dw_r = dw_r; a.dwr_ws = (float *)(ws + need - gate_bytes - dwr_bytes);
  a.clip = opts ? opts->grad_clip : 0.f;
  a.gate_alpha = ga; a.gate_beta = gb; a.dgate_alpha = dga; a.dgate_beta = dgb;
  a.gate_ws = (float *)(ws + need - gate_bytes);
  hipError_t e = fam == kMfma ? mfma_bwd(a, s) : generic_bwd(a, s);
  if (e == hipSuccess && w_r) e = residual_dw_r(a, s);
  if (e == hipSuccess && ga) e = gate_backward(a, s);
  return e == hipSuccess ? M2RNN_OK : M2RNN_ERR_HIP;
}

// ---- the scan's neighbours in the block ----

static m2rnn_status check_block(int32_t B, int32_t T, int32_t F, int32_t io) {
  if (io != M2RNN_F32 && io != M2RNN_BF16) return M2RNN_ERR_DTYPE;
  if (B < 0 || T < 0 || F < 8 || F % 8 != 0) return M2RNN_ERR_SHAPE;
  if ((double)B * (double)(T > 0 ? T : 1) * F > 1e15) return M2RNN_ERR_SHAPE;
  return M2RNN_OK;
}

size_t m2rnn_conv_silu_workspace_bytes(int32_t B, int32_t T, int32_t C) {
  return check_block(B, T, C, M2RNN_F32) == M2RNN_OK ? conv_silu_scratch_bytes(B, T, C) : 0;
}

m2rnn_status m2rnn_conv_silu_fwd(int32_t B, int32_t T, int32_t C, int32_t io, const void *x,
                                 const void *w, const void *bias, void *out, void *hip_stream) {
  m2rnn_status st = check_block(B, T, C, io);
  if (st != M2RNN_OK) return st;
  const bool any = (size_t)B * T > 0;
  if (!w || (any && (!x || !out))) return M2RNN_ERR_NULL;
  const void *ptrs[] = {x, w, bias, out};
  for (const void *p : ptrs)
    if (misaligned(p)) return M2RNN_ERR_ALIGN;
  return conv_silu_fwd(B, T, C, io, x, w, bias, out, (hipStream_t)hip_stream) == hipSuccess
             ? M2RNN_OK : M2RNN_ERR_HIP;
}

m2rnn_status m2rnn_conv_silu_bwd(int32_t B, int32_t T, int32_t C, int32_t io, const void *x,
                                 const void *w, const void *bias, const void *dout, void *dx,
                                 float *dw, float *dbias, void *workspace, size_t workspace_bytes,
                                 void *hip_stream) {
  m2rnn_status st = check_block(B, T, C, io);
  if (st != M2RNN_OK) return st;
  const bool any = (size_t)B * T > 0;
  if (!w || !dw || (any && (!x || !dout || !dx))) return M2RNN_ERR_NULL;
  const void *ptrs[] = {x, w, bias, dout, dx, dw, dbias, workspace};
  for (const void *p : ptrs)
    if (misaligned(p)) return M2RNN_ERR_ALIGN;
  if (!workspace) return M2RNN_ERR_NULL;
  if (workspace_bytes < conv_silu_scratch_bytes(B, T, C)) return M2RNN_ERR_WORKSPACE;
  return conv_silu_bwd(B, T, C, io, x, w, bias, dout, dx, dw, dbias, (float *)workspace,
                       (hipStream_t)hip_stream) == hipSuccess ? M2RNN_OK : M2RNN_ERR_HIP;
}

size_t m2rnn_gated_rmsnorm_workspace_bytes(int32_t B, int32_t T, int32_t D) {
  if (check_block(B, T, D, M2RNN_F32) != M2RNN_OK || D > gated_rmsnorm_max_features()) return 0;
  return gated_rmsnorm_scratch_bytes(B, T, D);
}

m2rnn_status m2rnn_gated_rmsnorm_fwd(int32_t B, int32_t T, int32_t D, int32_t io, const void *y,
                                     const void *a, const void *w, float eps, void *out, float *s,
                                     void *hip_stream) {
  m2rnn_status st = check_block(B, T, D, io);
  if (st != M2RNN_OK) return st;
  if (D > gated_rmsnorm_max_features() || !(eps >= 0.f)) return M2RNN_ERR_SHAPE;
  const bool any = (size_t)B * T > 0;
  if (!w || (any && (!y || !a || !out))) return M2RNN_ERR_NULL;
  const void *ptrs[] = {y, a, w, out};
  for (const void *p : ptrs)
    if (misaligned(p)) return M2RNN_ERR_ALIGN;
  if (((uintptr_t)s & 3u) != 0) return M2RNN_ERR_ALIGN;
  return gated_rmsnorm_fwd(B, T, D, io, y, a, w, eps, out, s, (hipStream_t)hip_stream) == hipSuccess
             ? M2RNN_OK : M2RNN_ERR_HIP;
}

m2rnn_status m2rnn_gated_rmsnorm_bwd(int32_t B, int32_t T, int32_t D, int32_t io, const void *y,
                                     const void *a, const void *w, float eps, const float *s,
                                     const void *dout, void *dy, void *da, float *dw,
                                     void *workspace, size_t workspace_bytes, void *hip_stream) {
  m2rnn_status st = check_block(B, T, D, io);
  if (st != M2RNN_OK) return st;
  if (D > gated_rmsnorm_max_features() || !(eps >= 0.f)) return M2RNN_ERR_SHAPE;
  const bool any = (size_t)B * T > 0;
  if (!w || !dw || (any && (!y || !a || !dout || !dy || !da))) return M2RNN_ERR_NULL;
  const void *ptrs[] = {y, a, w, dout, dy, da, dw, workspace};
  for (const void *p : ptrs)
    if (misaligned(p)) return M2RNN_ERR_ALIGN;
  if (((uintptr_t)s & 3u) != 0) return M2RNN_ERR_ALIGN;
  if (!workspace) return M2RNN_ERR_NULL;
  if (workspace_bytes < gated_rmsnorm_scratch_bytes(B, T, D)) return M2RNN_ERR_WORKSPACE;
  return gated_rmsnorm_bwd(B, T, D, io, y, a, w, eps, s, dout, dy, da, dw, (float *)workspace,
                           (hipStream_t)hip_stream) == hipSuccess ? M2RNN_OK : M2RNN_ERR_HIP;
}

}  // extern "C"

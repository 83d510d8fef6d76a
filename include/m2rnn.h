/*
 * m2rnn.h -- C ABI of the MI355X (gfx950) M2RNN recurrent-scan library.
 *
 * The library computes, for every batch element b and head n independently,
 * the matrix-state recurrence of the paper's "M2RNN layer" section
 * (recurrence equations; forward Algorithm 1, backward Algorithm 2):
 *
 *     Z_t = tanh(H_{t-1} W_n + k_t v_t^T)        H in R^{K x V}, W_n in R^{V x V}
 *     H_t = f_t H_{t-1} + (1 - f_t) Z_t          f_t in [0,1], one scalar per (b,t,n)
 *     y_t = H_t^T q_t                            (as in Algorithm 1; the w_r (.) v_t
 *                                                 residual of the y equation is an
 *                                                 option: m2rnn_opts.w_r)
 *
 * and its exact back-propagation through time.  Every step runs in hand-written
 * HIP kernels; there is no CPU path.
 *
 * General rules for every entry point
 *   - All tensor pointers are DEVICE pointers on the current HIP device, dense,
 *     row-major in the shape given, 16-byte aligned.  The descriptor is a HOST
 *     pointer.  The caller owns every buffer; the library allocates nothing,
 *     frees nothing, and keeps no pointer after the call returns.
 *   - Inputs are read-only.  Outputs are overwritten (never accumulated into),
 *     so they need no initialisation.
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL is
 *     the default stream) and the call returns without synchronising.
 *   - Every failure is a return code; nothing aborts or throws.  Validation
 *     happens on the host before anything is launched, so a failed call has
 *     launched nothing and written nothing.
 *   - Results are bit-reproducible: all cross-workgroup sums (over state rows,
 *     over heads that share q/k, over the batch for dW) are done in a fixed
 *     order, without atomics (the paper's Algorithm 2 uses atomic adds).
 *   - Numeric range with M2RNN_BF16: q, k, v, W and the state feed fp16
 *     matrix-core operands, so their magnitudes must stay below 2*10^4 (the
 *     recurrence itself keeps |H| <= max(1, |H0|)).  dy, dHT and the gradients
 *     may have any fp32 magnitude: the backward rescales them by powers of two
 *     internally.  With M2RNN_F32 everything is plain fp32.
 */
#ifndef M2RNN_H_
#define M2RNN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  M2RNN_OK = 0,
  M2RNN_ERR_NULL = 1,      /* a required pointer is NULL                            */
  M2RNN_ERR_SHAPE = 2,     /* a dimension is out of the supported set               */
  M2RNN_ERR_DTYPE = 3,     /* desc.io is not a known dtype                          */
  M2RNN_ERR_ALIGN = 4,     /* a pointer is not 16-byte aligned                      */
  M2RNN_ERR_WORKSPACE = 5, /* workspace_bytes < m2rnn_workspace_bytes()             */
  M2RNN_ERR_HIP = 6,       /* a HIP call (launch, attribute) failed                 */
  M2RNN_ERR_CHUNK = 7      /* desc.chunk is outside [0, m2rnn_max_chunk()]          */
} m2rnn_status;

typedef enum {
  M2RNN_F32 = 0, /* q,k,v,W,y,dy,dq,dk,dv are float32; contraction in fp32          */
  M2RNN_BF16 = 1 /* they are bfloat16; the state stays fp32, the contractions run
                    on the matrix cores with fp16 operands and fp32 accumulation   */
} m2rnn_dtype;

/* Problem descriptor (host memory).  Zero-initialise, then fill. */
typedef struct {
  int32_t B;   /* batch size, >= 0                                                  */
  int32_t T;   /* time steps, >= 0 (T == 0: HT = H0, dH0 = dHT, dW = 0)              */
  int32_t N;   /* heads of v, f, W, y (paper: N_v = N_f = N_w = N), >= 1            */
  int32_t Nqk; /* heads of q and k: N (one per head) or a divisor of N; head n
                  reads q/k head n / (N / Nqk).  Nqk = 1 is the paper's
                  multi-value form (Algorithm 1's Q, K in R^{BTK}).                 */
  int32_t K;   /* state rows    (paper: multiples of 16); one of 16, 32, 64, 128    */
  int32_t V;   /* state columns (paper: multiples of 16); one of 16, 32, 64, 128    */
  int32_t io;  /* m2rnn_dtype of q,k,v,W,y,dy,dq,dk,dv                               */
  int32_t chunk; /* checkpoint interval C in steps; 0 = m2rnn_default_chunk()        */
  uint32_t flags; /* reserved, must be 0                                             */
} m2rnn_desc;

/* Human-readable name of a status code (static storage). */
const char *m2rnn_status_string(m2rnn_status s);

/* Checkpoint interval the library picks when desc.chunk == 0, and the largest
 * one it accepts, for this shape and dtype (0 if the descriptor is invalid). */
int32_t m2rnn_default_chunk(const m2rnn_desc *desc);
int32_t m2rnn_max_chunk(const m2rnn_desc *desc);

/* Name of the kernel variant that serves this descriptor's forward (bwd = 0) or backward
 * (bwd != 0): "tile<K,V,RB>" (matrix-core kernel, a 16-row block spread over V/16 waves, RB
 * row blocks per workgroup), "rowwave<K,V>" (matrix-core forward, one wave per 16-row block),
 * "decode<K,V>" (T = 1: the single-launch latency kernel of recurrent inference),
 * "generic<f32>" / "generic<bf16>" (plain fp32 vector-ALU kernels), or "invalid descriptor".
 * Static storage.  For profiling and for tests that must reach every variant. */
const char *m2rnn_route_string(const m2rnn_desc *desc, int bwd);

/* Bytes of the checkpoint buffer: fp32 [B, N, ceil(T / C), K, V]; entry c holds
 * the state BEFORE step c*C (entry 0 is H0).  Checkpoints replace the paper's
 * H_full[B,T,N,K,V] cache (Algorithm 2, pass 1): the backward recomputes each
 * chunk's states on chip from its checkpoint.  Returns 0 for an invalid
 * descriptor or T == 0. */
size_t m2rnn_ckpt_bytes(const m2rnn_desc *desc);

/* Bytes of scratch a call needs for partial sums across workgroups:
 *   bwd = 0   the forward (may be 0);
 *   bwd = 1   the backward called WITH the forward's checkpoints (ckpt != NULL), the normal
 *             forward-then-backward use;
 *   bwd >= 2  the backward called with ckpt == NULL: bwd = 1 plus room for the checkpoints it
 *             then recomputes itself (m2rnn_ckpt_bytes more).
 * The backward figures include the two-stage sums of the option gradients (dw_r,
 * dgate_alpha, dgate_beta); the same size serves the plain and the _opt calls. */
size_t m2rnn_workspace_bytes(const m2rnn_desc *desc, int bwd);

/*
 * Forward scan (Algorithm 1; recurrence equations).
 *   q, k   [B,T,Nqk,K] io      v [B,T,N,V] io      f [B,T,N] fp32, gate VALUES in
 *   [0,1] (the forget-gate function psi is applied by the caller)
 *   W      [N,V,V] io          H0 [B,N,K,V] fp32 or NULL (zero initial state)
 *   y      [B,T,N,V] io, out
 *   HT     [B,N,K,V] fp32, out, final state; NULL if not wanted
 *   ckpt   out, m2rnn_ckpt_bytes() bytes, written for a later m2rnn_bwd with the
 *          same descriptor; NULL for inference (no checkpoints are written)
 *   workspace / workspace_bytes  scratch of at least m2rnn_workspace_bytes(desc,0)
 * Returns M2RNN_OK or the first validation / launch error.
 */
m2rnn_status m2rnn_fwd(const m2rnn_desc *desc, const void *q, const void *k,
                       const void *v, const float *f, const void *W,
                       const float *H0, void *y, float *HT, float *ckpt,
                       void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Backward scan (Algorithm 2, BPTT): gradients of
 *     L = sum_{b,t,n,j} y * dy  +  sum_{b,n,i,j} HT * dHT
 * with respect to q, k, v, f, W and H0.
 *   q,k,v,f,W,H0  as in m2rnn_fwd (the same values)
 *   ckpt   checkpoints written by m2rnn_fwd for this descriptor, or NULL: then
 *          the library first re-runs the recurrence from H0 into the workspace
 *          (the paper's pass 1, storing one state per chunk instead of all)
 *   dy     [B,T,N,V] io        dHT [B,N,K,V] fp32 or NULL (zero)
 *   dq, dk [B,T,Nqk,K] io, out (summed over the heads sharing a q/k head)
 *   dv     [B,T,N,V] io, out   df [B,T,N] fp32, out (gradient w.r.t. the gate value)
 *   dW     [N,V,V] fp32, out (summed over the batch)
 *   dH0    [B,N,K,V] fp32, out; NULL if not wanted
 *   workspace / workspace_bytes  at least m2rnn_workspace_bytes(desc, ckpt ? 1 : 2)
 */
m2rnn_status m2rnn_bwd(const m2rnn_desc *desc, const void *q, const void *k,
                       const void *v, const float *f, const void *W,
                       const float *H0, const float *ckpt, const void *dy,
                       const float *dHT, void *dq, void *dk, void *dv, float *df,
                       float *dW, float *dH0, void *workspace,
                       size_t workspace_bytes, void *hip_stream);

/*
 * The two options of the layer that sit on the scan itself (host struct; NULL = none).
 *   w_r        residual weight of the y equation of the layer section,
 *              y_t = H_t^T q_t + w_r (.) v_t : [N,V] io dtype, device memory, one weight per
 *              head and value channel; NULL = no residual (Algorithm 1's kernel).  In the
 *              backward the same w_r adds w_r (.) dy_t to dv_t, and dw_r receives
 *              sum over b, t of dy (.) v.
 *   dw_r       [N,V] fp32, device, out; read by m2rnn_bwd_opt only, required there when
 *              w_r is given (M2RNN_ERR_NULL otherwise), ignored when w_r is NULL.
 *   grad_clip  per-step clipping of the state gradient during BPTT (the paper's
 *              "Gradient Clipping" paragraph, which gives no rule; the rule here): when
 *              > 0, every element of the gradient that step t hands to step t-1
 *              (f_t G_t + dS_t W^T) is clamped to [-grad_clip, grad_clip] as soon as it
 *              is formed, before q dy^T of step t-1 is added; dH0 is the clamped value,
 *              dHT is used as given.  <= 0: off, gradients are exact.  Forward ignores it.
 *   gate_alpha, gate_beta   [N] fp32 each, device: parameters of the forget-gate function of
 *              the "Forget Gate" section, psi(x) = (1 + e^(x + beta_n))^(-alpha_n).  When
 *              gate_alpha is given (gate_beta is then required), the argument `f` of both
 *              calls holds the gate's INPUT x [B,T,N] fp32 and the kernels apply psi where
 *              they stage f; in the backward `df` then receives the gradient with respect
 *              to x, and dgate_alpha / dgate_beta the gradients of the parameters summed
 *              over b and t.  NULL: `f` is the gate value (the plain calls).
 *   dgate_alpha, dgate_beta [N] fp32 each, device, out; read by m2rnn_bwd_opt only,
 *              required there when gate_alpha is given.
 * Zero-initialise the struct, then fill what is used.
 */
typedef struct {
  const void *w_r;
  float *dw_r;
  float grad_clip;
  const float *gate_alpha;
  const float *gate_beta;
  float *dgate_alpha;
  float *dgate_beta;
} m2rnn_opts;

/* m2rnn_fwd / m2rnn_bwd with options; opts == NULL behaves exactly like the plain calls.
 * All other arguments, the workspace sizes and the error behaviour are the same. */
m2rnn_status m2rnn_fwd_opt(const m2rnn_desc *desc, const m2rnn_opts *opts, const void *q,
                           const void *k, const void *v, const float *f, const void *W,
                           const float *H0, void *y, float *HT, float *ckpt,
                           void *workspace, size_t workspace_bytes, void *hip_stream);
m2rnn_status m2rnn_bwd_opt(const m2rnn_desc *desc, const m2rnn_opts *opts, const void *q,
                           const void *k, const void *v, const float *f, const void *W,
                           const float *H0, const float *ckpt, const void *dy,
                           const float *dHT, void *dq, void *dk, void *dv, float *df,
                           float *dW, float *dH0, void *workspace,
                           size_t workspace_bytes, void *hip_stream);

/*
 * The scan's two neighbours in the block (layer equations of the "M2RNN Block" section), each
 * as one pass over its tensors.  All tensors are device pointers, dense, 16-byte aligned; io
 * is an m2rnn_dtype and types x / out / w / bias (resp. y / a / out / w / dout / dy / da);
 * weight gradients are fp32, overwritten, and summed over (b, t) in a fixed order.
 *
 * Prologue of q, k, v:  out = SiLU(conv1d(x)): depthwise causal convolution of kernel size 4
 * along t, zero padding on the left, tap j of w[c][.] meets step t - 3 + j (tap 3 is the
 * current step), then SiLU(u) = u sigmoid(u).
 *   x, out, dout, dx [B,T,C]   w [C,4]   bias [C] or NULL (the convolution's own bias; the
 *   paper prints none)   dw [C,4] fp32   dbias [C] fp32 or NULL.   C: a multiple of 8.
 *   workspace: m2rnn_conv_silu_workspace_bytes(B, T, C) bytes (backward only).
 *
 * Epilogue of y:  out = RMSNorm(y (.) g), g = SiLU(a), a the output gate's pre-activation:
 *   x_i = y_i g_i,  s = 1 / sqrt(mean_i x_i^2 + eps),  out_i = w_i x_i s   over ALL D = N V
 *   features of a token (the "RMSNormTP Module" appendix normalises over the features of all
 *   heads; eps = 0 is the printed formula); backward as printed there:
 *   p_i = w_i dout_i, r = sum_i p_i x_i, dx_i = s p_i - r s^3 x_i / D, dw_i = sum_{b,t} dout_i x_i s,
 *   then dy = dx (.) g and da = dx (.) y SiLU'(a).
 *   y, a, out, dout, dy, da [B,T,D]   w [D]   dw [D] fp32   s [B,T] fp32: the inverse norm
 *   the appendix caches for the backward; out of _fwd (NULL: not wanted), in of _bwd (NULL:
 *   recomputed).   D: a multiple of 8, at most 4096.   eps >= 0.
 *   workspace: m2rnn_gated_rmsnorm_workspace_bytes(B, T, D) bytes (backward only).
 *
 * Errors as for the scan: M2RNN_ERR_DTYPE / _SHAPE / _NULL / _ALIGN / _WORKSPACE on the host
 * before anything is launched, M2RNN_ERR_HIP for a failed launch.
 */
size_t m2rnn_conv_silu_workspace_bytes(int32_t B, int32_t T, int32_t C);
m2rnn_status m2rnn_conv_silu_fwd(int32_t B, int32_t T, int32_t C, int32_t io, const void *x,
                                 const void *w, const void *bias, void *out, void *hip_stream);
m2rnn_status m2rnn_conv_silu_bwd(int32_t B, int32_t T, int32_t C, int32_t io, const void *x,
                                 const void *w, const void *bias, const void *dout, void *dx,
                                 float *dw, float *dbias, void *workspace, size_t workspace_bytes,
                                 void *hip_stream);
size_t m2rnn_gated_rmsnorm_workspace_bytes(int32_t B, int32_t T, int32_t D);
m2rnn_status m2rnn_gated_rmsnorm_fwd(int32_t B, int32_t T, int32_t D, int32_t io, const void *y,
                                     const void *a, const void *w, float eps, void *out, float *s,
                                     void *hip_stream);
m2rnn_status m2rnn_gated_rmsnorm_bwd(int32_t B, int32_t T, int32_t D, int32_t io, const void *y,
                                     const void *a, const void *w, float eps, const float *s,
                                     const void *dout, void *dy, void *da, float *dw,
                                     void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * m2rnn_fwd_opt for callers that cannot allocate device memory or size a workspace: code
 * under HIP graph capture, tight serving loops (single-step or short-segment decode),
 * harnesses that forbid hipMalloc.  It takes no workspace: the scratch the forward needs for
 * its partial sums across workgroups is a device array inside the library, of
 * M2RNN_STATIC_SCRATCH_BYTES bytes, which every GPU the library runs on holds until the
 * process ends.  The call allocates nothing, frees nothing and synchronises nothing; it runs
 * the same kernels as m2rnn_fwd_opt and gives the same bits.
 *   - A descriptor whose m2rnn_workspace_bytes(desc, 0) exceeds M2RNN_STATIC_SCRATCH_BYTES is
 *     rejected with M2RNN_ERR_WORKSPACE before anything is launched (e.g. B*T*N*V <= 2^19
 *     at K = V = 64 with few states; shapes whose forward needs no scratch always pass).
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU
 *     (different streams or threads) race; serialise them.  Nothing in the array needs to
 *     start at zero: every part that is read in a call was written earlier in that call.
 *   - The device address of the array is looked up on the first call on each device (with
 *     that device current); M2RNN_ERR_HIP if the lookup fails.
 * All other arguments, options and errors are those of m2rnn_fwd_opt.
 */
#define M2RNN_STATIC_SCRATCH_BYTES (8u << 20)
m2rnn_status m2rnn_fwd_static(const m2rnn_desc *desc, const m2rnn_opts *opts, const void *q,
                              const void *k, const void *v, const float *f, const void *W,
                              const float *H0, void *y, float *HT, float *ckpt,
                              void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* M2RNN_H_ */

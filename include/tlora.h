/* tlora.h -- C ABI of the fused multi-LoRA linear layer for AMD MI355X (gfx950).
 *
 * Many fine-tuning jobs share one frozen base weight W; job j owns a low-rank adapter
 * (A_j: d_in x r_j, B_j: r_j x d_out, scale_j) that applies to its own contiguous segment of
 * the token batch (paper Sec. 2: W + dW with dW = A.B; Sec. 3.2: jobs fused on a shared backbone
 * keep independent forward/backward semantics; Sec. 3.3: fused batched LoRA kernel -- tokens of
 * adapter i go through A_i into a compact |X_i| x r_i intermediate and straight on through B_i
 * into the output, the dense A_i.B_i is never formed).
 *
 *   forward :  Y[seg j]  = X[seg j].W   + scale_j * (X[seg j].A_j).B_j
 *   backward:  dX[seg j] = dY[seg j].W^T + scale_j * (dY[seg j].B_j^T).A_j^T
 *              dA_j      = scale_j * X[seg j]^T . (dY[seg j].B_j^T)
 *              dB_j      = scale_j * (X[seg j].A_j)^T . dY[seg j]          (W is frozen: no dW)
 *
 * General conventions
 *   - All matrices are dense row-major.  seg j = rows offsets[j] .. offsets[j+1]-1.
 *   - HOST pointers: the problem struct, ranks, offsets, scales and the arrays of per-job
 *     pointers.  DEVICE pointers: X, W, every A_j / B_j, Y, dY, dX, every dA_j / dB_j and the
 *     workspace.  The caller owns every buffer; the library allocates no device memory, keeps no
 *     pointer after a call returns (one exception: while tlora_profile is enabled it remembers where in the
 *     last call's workspace the GEMM's clock probe lies, for tlora_profile_clock) and never writes W, X, A_j,
 *     B_j or dY.
 *   - dtype TLORA_BF16: X, W, A_j, B_j, Y, dY, dX hold bf16; accumulation is fp32; Y / dX are rounded
 *     to nearest-even once on store.  dtype TLORA_F32: those tensors hold fp32.  dA_j, dB_j are fp32
 *     for both dtypes.  Gradients are overwritten, not accumulated.
 *   - X, W, Y, dY, dX must be 16-byte aligned and d_in, d_out multiples of 8.  A_j, B_j, dA_j, dB_j
 *     need only element alignment (ranks such as 1 or 3 are legal).  The workspace must be 256-byte
 *     aligned.
 *   - Legal degenerate inputs: T_j = 0 (dA_j = dB_j = 0), r_j = 0 (rows of that job get the
 *     backbone product only; its A/B/dA/dB pointers are ignored and may be NULL), T = 0 (X, Y, dY, dX
 *     may be NULL; the forward launches nothing, the backward zero-fills dA_j / dB_j).
 *   - Limits (TLORA_EINVAL beyond them, before anything is launched): J <= TLORA_MAX_JOBS, T <= TLORA_MAX_TOKENS,
 *     d_in, d_out <= TLORA_MAX_FEATURES, r_j <= TLORA_MAX_RANK, sum_j (r_j padded to 8) <= 2^22, and a plan of at most 2^22 GEMM tiles
 *     (ceil(T / 256) * ceil(max(d_in, d_out) / 256)) and 2^22 work units of each kind -- the kernels keep 32-bit
 *     offsets inside a tile and one workgroup per tile / unit.
 *   - Calls are asynchronous on `hip_stream` (a hipStream_t; NULL = the default stream).  Host
 *     arrays may be reused as soon as the call returns.  Two calls that share a workspace must be
 *     ordered on one stream.
 *   - Every entry point returns a tlora_status_t (0 = ok, negative = error).  tlora_fwd, tlora_fwd_noalloc and
 *     tlora_bwd validate everything before their first launch: on an argument error nothing has been launched.
 *     The composite entry points (nano-batched, token-indexed, MLP / attention block, decoder layer) check their
 *     own arguments first but run their sub-calls one after the other: if a later sub-call fails (a HIP error,
 *     an invalid per-projection pointer) the kernels of the earlier ones are already queued.  The results are independent of the internal tiling and are bit-identical from
 *     run to run (no floating-point atomics).
 */
#ifndef TLORA_H
#define TLORA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TLORA_MAX_RANK 1024
#define TLORA_MAX_JOBS 32768
#define TLORA_MAX_TOKENS (1 << 24)
#define TLORA_MAX_FEATURES (1 << 20)

typedef enum { TLORA_F32 = 0, TLORA_BF16 = 1 } tlora_dtype_t;

typedef enum {
  TLORA_OK = 0,
  TLORA_EINVAL = -1,      /* bad sizes: J < 1, d not a multiple of 8, offsets not non-decreasing from 0, ... */
  TLORA_ENULL = -2,       /* a required pointer is NULL                                                   */
  TLORA_EDTYPE = -3,      /* dtype is neither TLORA_F32 nor TLORA_BF16                                    */
  TLORA_EWORKSPACE = -4,  /* workspace NULL, misaligned or smaller than tlora_workspace_bytes()           */
  TLORA_EARCH = -5,       /* the current device is not gfx950                                             */
  TLORA_EHIP = -6,        /* a HIP runtime call failed                                                    */
  TLORA_EALIGN = -7,      /* X / W / Y / dY / dX not 16-byte aligned                                      */
  TLORA_ESCRATCH = -8     /* tlora_fwd_noalloc: the problem needs more than the static scratch holds      */
} tlora_status_t;

/* Problem statement of one fused layer call (Sec. 3.2 / 3.3: shared frozen backbone, per-job adapters
 * on per-job token segments). */
typedef struct {
  int32_t dtype;            /* tlora_dtype_t of X, W, A_j, B_j, Y, dY, dX                          */
  int32_t num_jobs;         /* J >= 1                                                              */
  int32_t d_in, d_out;      /* multiples of 8                                                      */
  const int32_t* ranks;     /* HOST [J]   r_j in [0, TLORA_MAX_RANK]                               */
  const int64_t* offsets;   /* HOST [J+1] offsets[0] = 0, non-decreasing, T = offsets[J] < 2^31    */
  const float* scales;      /* HOST [J]   scale_j                                                  */
  const void* X;            /* DEVICE [T, d_in]                                                    */
  const void* W;            /* DEVICE [d_in, d_out], never written                                 */
  const void* const* A;     /* HOST array of J DEVICE pointers, A_j [d_in, r_j]                    */
  const void* const* B;     /* HOST array of J DEVICE pointers, B_j [r_j, d_out]                   */
} tlora_problem_t;

/* Bytes of device workspace that tlora_fwd / tlora_bwd need for this problem (depends only on
 * dtype, J, d_in, d_out, ranks, offsets).  It grows with sum_j T_j * r_j and with r_j * (d_in + d_out), plus
 * one bf16 d_in x d_out buffer (the transposed W of the backward, shared by all jobs);
 * no d_in x d_out per-job buffer is ever used (Sec. 3.3: the merged adapter weight is not
 * materialised).  Returns 0 if the problem is invalid. */
size_t tlora_workspace_bytes(const tlora_problem_t* p);

/* Forward (Sec. 3.3).  Y: DEVICE [T, d_out], overwritten.  The workspace afterwards holds the
 * intermediates S_j = X_j.A_j and the packed bf16 copies of the adapters, which a following
 * tlora_bwd on the same problem (same A_j, B_j values), workspace and stream may reuse
 * (TLORA_BWD_REUSE_S). */
int tlora_fwd(const tlora_problem_t* p, void* Y, void* workspace, size_t ws_bytes, void* hip_stream);

/* tlora_fwd for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results as tlora_fwd
 * (bit-identical Y), but the forward's intermediates (plan tables, S_j, the packed adapters) live in a device array
 * of TLORA_NOALLOC_SCRATCH_BYTES that is part of the library image; every GPU the library runs on holds it until the
 * process ends.  The call allocates nothing -- no hipMalloc / hipFree / hipHostMalloc, no event or stream creation,
 * no allocating library routine -- and records no copy or memset: the plan tables travel as kernel arguments and
 * everything that must start at zero is cleared by store kernels on `hip_stream`.
 *   Limits: the forward-only workspace of the problem (about 4 sum_j T_j r_j + 2 * 256 ceil(T / 256) * (padded
 *   ranks met per 256-row tile) + 6 (sum_j r_j + 32) (d_in + d_out) bytes + tables) must fit in
 *   TLORA_NOALLOC_SCRATCH_BYTES and its plan tables in 224 KB; otherwise TLORA_ESCRATCH, and nothing is launched.
 *   The scratch keeps the last call's contents and is shared by every call on that GPU: calls that overlap on one
 *   GPU (two streams, two host threads) race; order them on one stream.  There is no matching backward: S_j
 *   does not outlive the next call (tlora_bwd without TLORA_BWD_REUSE_S recomputes it in its own workspace).
 *   The address of the array on the current device is looked up (and the device's architecture checked) on the first
 *   call on that device: a caller that captures the stream makes one call before the capture begins. */
#define TLORA_NOALLOC_SCRATCH_BYTES (16u << 20)
int tlora_fwd_noalloc(const tlora_problem_t* p, void* Y, void* hip_stream);

/* flags for tlora_bwd */
#define TLORA_BWD_REUSE_S 1   /* the workspace still holds S_j and the packed adapters from tlora_fwd of this same
                                 problem; X, A_j, B_j have not changed since */
#define TLORA_BWD_ACCUMULATE 4 /* dA_j += ..., dB_j += ... instead of overwriting them (gradient accumulation over the
                                 nano-batches or micro-batches of one step); dX is always overwritten */
#define TLORA_BWD_REUSE_WT 2  /* the workspace still holds the transposed copy of W that an earlier tlora_bwd with
                                 the same W, d_in, d_out, job table and workspace made (W is frozen: one copy
                                 serves every later step) */

/* Backward (derivatives of L = sum(dY * Y); Sec. 3.2 fixes only that each job's backward is
 * independent and that W gets no gradient).
 *   dY: DEVICE [T, d_out].   dX: DEVICE [T, d_in], overwritten; NULL skips it.
 *   dA: HOST array of J DEVICE pointers to fp32 [d_in, r_j];  dB: likewise fp32 [r_j, d_out].
 *   Both arrays may be NULL together to skip the adapter gradients. */
int tlora_bwd(const tlora_problem_t* p, const void* dY, void* dX, void* const* dA, void* const* dB,
              int flags, void* workspace, size_t ws_bytes, void* hip_stream);

/* ---- Adaptive nano-batching (Sec. 3.3, "Adaptive Nano-Batching") --------------------------------------------
 * The combined batch of the fused jobs is cut along the batch dimension into N nano-batches of about
 * (sum_i B_i) / N samples each, which the fused kernels process one after the other; N is adapted online by an
 * additive-increase / multiplicative-decrease controller fed with the measured completion time T_t of a step
 * (the update rule printed in that paragraph):
 *     N_{t+1} = N_t + alpha                 if T_t <= T_{t-1} - tau
 *             = max(1, floor(beta N_t))     otherwise                     (alpha = 4, beta = 1/2 by default).
 * Readings where the paper is silent: tau = tau_rel * T_{t-1} (tau_rel = 0.02 suggested); the first observation
 * has no predecessor, so it is only recorded and N is kept; n_max > 0 caps N (a batch has only so many samples).
 * The controller is plain host state owned by the caller; nothing here touches the GPU. */
typedef struct {
  int32_t n;          /* N_t: the number of nano-batches to use for the next step */
  int32_t alpha;      /* additive step                                            */
  int32_t n_max;      /* upper limit of N, 0 = none                               */
  int32_t have_prev;  /* 0 until the first completion time has been seen          */
  double beta;        /* multiplicative back-off factor, in (0, 1)                */
  double tau_rel;     /* stability margin as a fraction of T_{t-1}                */
  double t_prev;      /* T_{t-1}                                                  */
} tlora_aimd_t;
/* TLORA_EINVAL unless n0 >= 1, alpha >= 1, 0 < beta < 1, tau_rel >= 0, n_max >= 0. */
int tlora_aimd_init(tlora_aimd_t* c, int32_t n0, int32_t alpha, double beta, double tau_rel, int32_t n_max);
/* Feeds T_t (any unit, >= 0), applies the rule, stores N_{t+1} in c->n and in *n_next (may be NULL). */
int tlora_aimd_update(tlora_aimd_t* c, double t_step, int32_t* n_next);

/* Nano-batch n (0-based) of n_nano: `granule` tokens (a sequence) are the indivisible sample; with
 * U = ceil(T / granule) samples the nano-batch covers samples floor(n U / n_nano) .. floor((n + 1) U / n_nano) - 1,
 * i.e. token rows [*row0, *row1) = [min(T, granule floor(n U / n_nano)), min(T, granule floor((n + 1) U / n_nano))).
 * sub_offsets: HOST [J+1], the offsets (relative to *row0) of the jobs' segments inside that range.  Outputs may
 * be NULL.  Host-only integer arithmetic. */
int tlora_nano_split(const tlora_problem_t* p, int32_t n_nano, int64_t granule, int32_t n, int64_t* row0,
                     int64_t* row1, int64_t* sub_offsets);
/* Workspace that tlora_fwd_nano / tlora_bwd_nano need: the largest nano-batch's.  0 if invalid. */
size_t tlora_nano_workspace_bytes(const tlora_problem_t* p, int32_t n_nano, int64_t granule);
/* tlora_fwd / tlora_bwd over the n_nano nano-batches, one after the other on `hip_stream`, sharing one
 * workspace.  Same arguments and results as the plain calls (the results do not depend on n_nano beyond
 * floating-point summation order: dA_j, dB_j are accumulated over the nano-batches in order).  Flags of
 * tlora_bwd_nano: TLORA_BWD_ACCUMULATE, TLORA_BWD_REUSE_WT (S of a nano-batch is not kept, so no REUSE_S). */
int tlora_fwd_nano(const tlora_problem_t* p, int32_t n_nano, int64_t granule, void* Y, void* workspace, size_t ws_bytes,
                   void* hip_stream);
int tlora_bwd_nano(const tlora_problem_t* p, int32_t n_nano, int64_t granule, const void* dY, void* dX,
                   void* const* dA, void* const* dB, int flags, void* workspace, size_t ws_bytes, void* hip_stream);

/* ---- Per-job optimizer step -------------------------------------------------------------------------------
 * Sec. 3.2: jobs fused on the shared backbone keep their own optimizer state.  The paper names no optimizer; this
 * is AdamW (decoupled weight decay) on any list of adapter tensors, each with its own hyper-parameters and step
 * count, in one launch:
 *     m = beta1 m + (1 - beta1) g;  v = beta2 v + (1 - beta2) g^2;
 *     w = w - lr ( (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps) + weight_decay w )
 * in fp32 on the fp32 master copy; `param` (what tlora_fwd / tlora_bwd read as A_j or B_j) is rewritten from it,
 * rounded to nearest-even when dtype is TLORA_BF16.  `tensors` is a HOST array; every pointer inside is a DEVICE
 * pointer; `master` may be NULL for TLORA_F32 (the update then runs on `param`).  grad is typically dA_j / dB_j
 * of tlora_bwd.  Asynchronous on `hip_stream`; the workspace (256-byte aligned, tlora_adamw_workspace_bytes)
 * holds the tensor table during the call. */
typedef struct {
  void* param;          /* DEVICE [n], bf16 or fp32 per `dtype`; rewritten          */
  float* master;        /* DEVICE fp32 [n]; updated                                 */
  const float* grad;    /* DEVICE fp32 [n]                                          */
  float* m;             /* DEVICE fp32 [n] first moment; updated                    */
  float* v;             /* DEVICE fp32 [n] second moment; updated                   */
  int64_t n;            /* elements                                                 */
  float lr, beta1, beta2, eps, weight_decay;
  int32_t step;         /* t >= 1: the step being taken (bias correction)           */
} tlora_adamw_tensor_t;
size_t tlora_adamw_workspace_bytes(int32_t count);
int tlora_adamw_step(const tlora_adamw_tensor_t* tensors, int32_t count, int32_t dtype, void* workspace,
                     size_t ws_bytes, void* hip_stream);

/* ---- MLP half of a decoder layer of the shared super-model ---------------------------------------------------
 * Sec. 3.2: the group's jobs are fused on one frozen backbone whose linear layers carry the jobs' adapters on the
 * jobs' own tokens; the backbones of Sec. 4.1 are pre-norm gated-MLP decoders.  For token rows X [T, d_model]:
 *     Xn = X / sqrt(mean(X^2) + eps) * gamma;   G = fused(Xn; W_gate, A/B_gate);   U = fused(Xn; W_up, A/B_up);
 *     Z = silu(G) * U;                          Out = X + fused(Z; W_down, A/B_down)
 * where fused(.) is tlora_fwd.  The backward gives dX and every dA_j / dB_j of the three projections for
 * L = sum(dOut * Out); backbone weights and gamma are frozen.  A job has one rank for its three projections.
 * tlora_mlp_bwd must follow tlora_mlp_fwd of the same problem on the same workspace and stream: the workspace
 * keeps Xn, rstd, G, U, Z and each projection's S_j.  gamma: DEVICE [d_model] in `dtype`; X, Out, dOut, dX:
 * DEVICE [T, d_model], 16-byte aligned; d_model, d_ff multiples of 8.  flags: TLORA_BWD_ACCUMULATE,
 * TLORA_BWD_REUSE_WT (applied to all three projections). */
typedef struct {
  int32_t dtype, num_jobs, d_model, d_ff;
  const int32_t* ranks;      /* HOST [J]   */
  const int64_t* offsets;    /* HOST [J+1] */
  const float* scales;       /* HOST [J]   */
  const void* X;             /* DEVICE [T, d_model] */
  const void* gamma;         /* DEVICE [d_model]    */
  float eps;
  const void* W_gate;        /* DEVICE [d_model, d_ff] */
  const void* W_up;          /* DEVICE [d_model, d_ff] */
  const void* W_down;        /* DEVICE [d_ff, d_model] */
  const void* const* A_gate; /* HOST arrays of J DEVICE pointers: [d_model, r_j] */
  const void* const* B_gate; /*                                   [r_j, d_ff]    */
  const void* const* A_up;
  const void* const* B_up;
  const void* const* A_down; /*                                   [d_ff, r_j]    */
  const void* const* B_down; /*                                   [r_j, d_model] */
} tlora_mlp_t;
size_t tlora_mlp_workspace_bytes(const tlora_mlp_t* p);
int tlora_mlp_fwd(const tlora_mlp_t* p, void* Out, void* workspace, size_t ws_bytes, void* hip_stream);
int tlora_mlp_bwd(const tlora_mlp_t* p, const void* dOut, void* dX, void* const* dA_gate, void* const* dB_gate,
                  void* const* dA_up, void* const* dB_up, void* const* dA_down, void* const* dB_down, int flags,
                  void* workspace, size_t ws_bytes, void* hip_stream);

/* ---- Attention half of a decoder layer ---------------------------------------------------------------------
 * The backbones of Sec. 4.1 are decoder-only transformers; their attention half, with the four projections as
 * fused multi-LoRA layers (Sec. 3.2), is
 *     Xn = RMSNorm(X) gamma;  Q, K, V = fused(Xn; W_q / W_k / W_v);  Q, K = rope(Q), rope(K);
 *     Out = X + fused(attention(Q, K, V); W_o)
 * with rotary position embedding (pairs (i, i + head_dim / 2), angle = position * rope_base^(-2 i / head_dim),
 * position = index of the token inside its sequence) and causal grouped-query attention (query head h reads
 * key / value head h / (n_heads / n_kv_heads); scores scaled by 1 / sqrt(head_dim)).  Sequences are runs of
 * consecutive token rows: seq_offsets (HOST int64 [num_seqs + 1], seq_offsets[0] = 0, non-decreasing, last = T).
 * Sequences do not interact; which job a sequence belongs to matters only to the projections (`offsets`).
 * bf16 only (TLORA_EDTYPE otherwise), head_dim must be 128 (TLORA_EINVAL otherwise).  Tensors are DEVICE
 * [T, heads * 128] row-major, heads side by side inside a row, 16-byte aligned.
 *
 * Primitives (their `workspace`: tlora_attention_workspace_bytes, 256-byte aligned):
 *   tlora_rope           rotates X in place (inverse != 0: the transposed rotation = backward of the forward one)
 *   tlora_attention_fwd  O [T, n_heads * 128] and lse (DEVICE fp32 [T, n_heads]: base-2 logarithm of the softmax
 *                        denominator of the scaled scores, maximum included) from rotated Q, K and V
 *   tlora_attention_bwd  dQ, dK, dV from dO and the forward's Q, K, V, O, lse; deterministic (fixed summation order)
 * Probabilities are rounded to bf16 before they multiply V / dO, score gradients before they multiply K / Q;
 * all sums are fp32.  Calls are asynchronous on hip_stream; host arrays are read before the call returns. */
size_t tlora_attention_workspace_bytes(int32_t num_seqs, const int64_t* seq_offsets, int32_t n_heads);
int tlora_rope(void* X, int32_t num_seqs, const int64_t* seq_offsets, int32_t heads, int32_t head_dim, float rope_base,
               int32_t inverse, void* workspace, size_t ws_bytes, void* hip_stream);
int tlora_attention_fwd(const void* Q, const void* K, const void* V, void* O, float* lse, int32_t num_seqs,
                        const int64_t* seq_offsets, int32_t n_heads, int32_t n_kv_heads, int32_t head_dim, void* workspace,
                        size_t ws_bytes, void* hip_stream);
int tlora_attention_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* lse,
                        void* dQ, void* dK, void* dV, int32_t num_seqs, const int64_t* seq_offsets, int32_t n_heads,
                        int32_t n_kv_heads, int32_t head_dim, void* workspace, size_t ws_bytes, void* hip_stream);

/* The block.  tlora_attn_fwd keeps Xn, the rotated Q and K, V, the attention output, lse and every projection's
 * S_j in the workspace; tlora_attn_bwd must follow it on the same stream with the same workspace and returns dX
 * (through the residual and the norm) and dA / dB of the four projections (same layout and flags as tlora_bwd:
 * TLORA_BWD_ACCUMULATE, TLORA_BWD_REUSE_WT).  W_* and gamma are frozen. */
typedef struct tlora_attn_t {
  int32_t dtype;             /* TLORA_BF16 */
  int32_t num_jobs;
  int32_t d_model;
  int32_t n_heads, n_kv_heads, head_dim;
  float rope_base;           /* > 1 */
  float eps;                 /* RMSNorm: x / sqrt(mean(x^2) + eps) */
  const int32_t* ranks;      /* HOST [num_jobs] */
  const int64_t* offsets;    /* HOST [num_jobs + 1] token rows of every job */
  const float* scales;       /* HOST [num_jobs] */
  int32_t num_seqs;
  const int64_t* seq_offsets;/* HOST [num_seqs + 1] */
  const void* X;             /* DEVICE [T, d_model] */
  const void* gamma;         /* DEVICE [d_model] */
  const void* W_q;           /* DEVICE [d_model, n_heads * head_dim] */
  const void* W_k;           /* DEVICE [d_model, n_kv_heads * head_dim] */
  const void* W_v;           /* DEVICE [d_model, n_kv_heads * head_dim] */
  const void* W_o;           /* DEVICE [n_heads * head_dim, d_model] */
  const void* const* A_q;    /* HOST arrays of DEVICE pointers, as tlora_problem_t.A / .B */
  const void* const* B_q;
  const void* const* A_k;
  const void* const* B_k;
  const void* const* A_v;
  const void* const* B_v;
  const void* const* A_o;
  const void* const* B_o;
} tlora_attn_t;
size_t tlora_attn_workspace_bytes(const tlora_attn_t* p);
int tlora_attn_fwd(const tlora_attn_t* p, void* Out, void* workspace, size_t ws_bytes, void* hip_stream);
/* dA / dB: HOST arrays of 4 entries (q, k, v, o), each a HOST array [num_jobs] of DEVICE pointers */
int tlora_attn_bwd(const tlora_attn_t* p, const void* dOut, void* dX, void* const* const* dA, void* const* const* dB,
                   int flags, void* workspace, size_t ws_bytes, void* hip_stream);

/* ---- One decoder layer --------------------------------------------------------------------------------------
 * Sec. 3.2's shared super-model repeats one unit: the attention half followed by the MLP half,
 *     H = attention block(X),   Out = MLP block(H),
 * all seven projections being fused multi-LoRA layers on the same jobs.  `attn.X` is the layer's input; `mlp.X` is
 * ignored (H lives in the workspace).  Both halves must name the same dtype (bf16), num_jobs, d_model, and equal
 * ranks / offsets / scales (TLORA_EINVAL otherwise).  tlora_layer_bwd must follow tlora_layer_fwd on the same
 * stream with the same workspace.  dA / dB: HOST arrays of 7 entries (q, k, v, o, gate, up, down), each a HOST
 * array [num_jobs] of DEVICE pointers; flags as tlora_attn_bwd. */
typedef struct tlora_layer_t {
  tlora_attn_t attn;
  tlora_mlp_t mlp;
} tlora_layer_t;
size_t tlora_layer_workspace_bytes(const tlora_layer_t* p);
int tlora_layer_fwd(const tlora_layer_t* p, void* Out, void* workspace, size_t ws_bytes, void* hip_stream);
int tlora_layer_bwd(const tlora_layer_t* p, const void* dOut, void* dX, void* const* const* dA, void* const* const* dB,
                    int flags, void* workspace, size_t ws_bytes, void* hip_stream);

/* ---- General token -> adapter assignment --------------------------------------------------------------------
 * Sec. 3.3 describes the kernel as gathering the tokens of adapter i and scattering the results back to the
 * output tensor.  Here X, Y, dY, dX are in the batch's own (arbitrary) token order, and row_index (DEVICE int32 [T],
 * a permutation of 0 .. T-1) lists the rows job by job: row_index[offsets[j] .. offsets[j+1]-1] are the rows of job
 * j, in the order in which they enter that job's gradient sums.  Row t of Y / dX belongs to row t of X / dY.
 * bf16: the kernels fetch the activation rows through the list inside their loads and the GEMMs scatter their output
 * rows while storing them, so the batch is read and written as often as in a contiguous call (option
 * "indexed_direct"; activations of 4 GiB or more are first gathered into the workspace by a copy pass, and so is the
 * fp32 configuration, which also scatters with a second copy pass).  Same arguments, flags and results as tlora_fwd /
 * tlora_bwd otherwise (TLORA_BWD_REUSE_S included, under the same condition).
 * The list is device data and is not checked to be a permutation; the kernels work on a copy of it (in the workspace)
 * with every entry forced into [0, T-1], so a bad list yields wrong rows -- a row named twice is written by either
 * of its tokens, a row never named is not written -- but no access outside the tensors. */
size_t tlora_indexed_workspace_bytes(const tlora_problem_t* p);
int tlora_fwd_indexed(const tlora_problem_t* p, const int32_t* row_index, void* Y, void* workspace, size_t ws_bytes,
                      void* hip_stream);
int tlora_bwd_indexed(const tlora_problem_t* p, const int32_t* row_index, const void* dY, void* dX, void* const* dA,
                      void* const* dB, int flags, void* workspace, size_t ws_bytes, void* hip_stream);

/* ---- Adapter scheduler (HOST only) -------------------------------------------------------------------------
 * Sec. 3.4 / Algorithm 1, Phase 1, on one device: the queue of jobs (and already merged groups) is sorted by urgency
 * (descending), then residual resources (ascending); the first entry seeds a group, the partner with the highest
 * joint throughput is merged in and the union re-inserted, until no partner is beneficial; then the group is final.
 * The paper leaves Throughput, residual and "beneficial" open; here, over a measured step-time model:
 *     step_ms(G)    = curve(sum tokens_j) + ms_per_token_rank * sum tokens_j * rank_j + ms_per_job * (|G| - 1)
 *                     curve: piecewise-linear through (tokens[i], ms[i]) (tokens ascending, n_points >= 2), flat
 *                     below the first point, continued along the last segment above the last
 *     throughput(G) = sum tokens_j / step_ms(G);  residual(G) = 1 - throughput(G) / max_i(tokens[i] / ms[i])
 *     urgency(G)    = max over members;  a union is admissible when step_ms(G) / step_ms({j}) <= max_slowdown_j for
 *                     every member, and beneficial when throughput(A + B) > (tokens_A + tokens_B) / (step_ms(A) +
 *                     step_ms(B)), i.e. when it beats time-sharing the device.
 * Ties: smaller first job index first; among equally good partners the first in queue order.  IEEE double, fixed
 * order of operations: results are reproducible bit for bit.  No device is touched. */
typedef struct tlora_sched_model_t {
  int32_t n_points;
  const double* tokens;        /* HOST [n_points] ascending, > 0 */
  const double* ms;            /* HOST [n_points] > 0 */
  double ms_per_token_rank;    /* >= 0 */
  double ms_per_job;           /* >= 0: cost of one more job in a fused call */
} tlora_sched_model_t;
typedef struct tlora_sched_job_t {
  int64_t tokens;              /* tokens per training step, >= 1 */
  int32_t rank;                /* >= 0 */
  int32_t steps;               /* training steps to run (tlora_sched_simulate), >= 0 */
  double urgency;              /* >= 0 (tlora_sched_partition; the simulation derives its own) */
  double max_slowdown;         /* >= 1: bound on step_ms(group) / step_ms(job alone) */
} tlora_sched_job_t;
/* Predicted step time of the group members[0 .. n_members-1] (job indices). */
int tlora_sched_step_ms(const tlora_sched_model_t* model, int32_t n_jobs, const tlora_sched_job_t* jobs,
                        const int32_t* members, int32_t n_members, double* ms);
/* Phase 1 repeated on what is left until every job has a group: group_of[j] = index of job j's group in the
 * order the groups were finalized; *n_groups = their number. */
int tlora_sched_partition(const tlora_sched_model_t* model, int32_t n_jobs, const tlora_sched_job_t* jobs,
                          int32_t* group_of, int32_t* n_groups);
/* Algorithm 1's outer loop on one device: group, run the group min(horizon, fewest steps left among its members)
 * steps, update progress, recompute urgencies (elapsed time / (standalone step time * max(steps done, 1)); 1 at
 * time 0), until every job has run its steps.  jct_ms [n_jobs] = completion times; *makespan_ms = the last one.
 * Trace (optional, all three or none): round i ran trace_sizes[i] jobs, listed consecutively in trace_members, for
 * trace_steps[i] steps; trace_sizes / trace_steps hold trace_capacity entries, trace_members trace_capacity *
 * n_jobs; rounds beyond the capacity are not recorded.  *n_rounds = rounds run. */
int tlora_sched_simulate(const tlora_sched_model_t* model, int32_t n_jobs, const tlora_sched_job_t* jobs, int32_t horizon,
                         double* jct_ms, double* makespan_ms, int32_t* trace_members, int32_t* trace_sizes,
                         int32_t* trace_steps, int64_t* n_rounds, int64_t trace_capacity);

/* Integer bookkeeping of the nano-batch plan (Sec. 3.3, nano-batches = partition of the combined
 * batch along the token dimension), for bit-exact checks.  All outputs are HOST arrays and each may
 * be NULL.  Per job: rpad[J] (rank rounded up to the 8-element granule), soff[J+1] (element
 * offset of job j's rows in the packed intermediate: sum_{i<j} ceil(T_i / 32) * 32 * rpad_i).  Per row tile of
 * the backbone GEMM (uniform tiles of `*tile_rows` rows over the concatenated batch; a tile may
 * hold rows of several jobs): tile_row0, tile_nrows, tile_job_first, tile_job_last (first / last
 * job with a row in the tile).  *n_tiles: in = capacity of the tile arrays, out = number of tiles
 * (the call fails with TLORA_EINVAL if the capacity is too small, after storing the count). */
int tlora_plan_dump(const tlora_problem_t* p, int32_t* rpad, int64_t* soff, int32_t* tile_rows,
                    int64_t* tile_row0, int32_t* tile_nrows, int32_t* tile_job_first,
                    int32_t* tile_job_last, int64_t* n_tiles);

/* Host-only self-check of the planner (no GPU work, no cache): builds the plan of `p` afresh -- of the forward alone if
 * fwd_only != 0 -- and verifies what the kernels rely on: job segments, padded ranks and packed offsets add up; every
 * row tile's adapter range holds all jobs with a row inside it and fits the packed operands; the shrink work units tile
 * each job's [tokens x padded ranks] exactly once; every dA / dB work unit lies inside its job, starts on the token
 * step, owns a partial tile that overlaps no other, and each output tile's partial tiles are consecutive and cover the
 * job's tokens; all tables fit the table block and all workspace regions are disjoint and inside
 * tlora_workspace_bytes().  Returns TLORA_OK, the validation error of `p`, or TLORA_EINVAL with the number of the
 * first failed check in *failed_check (may be NULL; 0 when nothing failed).  Used by the CPU tests on random problems. */
int tlora_plan_check(const tlora_problem_t* p, int32_t fwd_only, int32_t* failed_check);

/* Tuning knobs (process-wide, for experiments and for the tiling-independence tests).
 *   "shrink_rows"  : token rows per work unit of the shrink kernels        (0 = chosen per problem (default) | 32 | 64 | 128)
 *   "shrink_stages": LDS stages of the streaming shrink kernel             (4 | 8)
 *   "dx_transposed_w": 1 (default): dX runs against a transposed copy of W kept in the workspace | 0: against W
 *                    as it lies in memory (no copy, slower weight stream)
 *   "grad_tokens"  : minimum tokens per work unit of the dA / dB kernels   (multiple of 64, at most 4096)
 *   "indexed_direct": 1 (default): bf16 token-indexed calls read the batch rows through the index list inside the
 *                    kernels' loads (while T * max(d_in, d_out) * 2 bytes stays below 4 GiB) | 0: always gather the
 *                    activations into the workspace first
 *   "table_copy_kernel": 1 (default): a call's plan tables are moved from the pinned staging buffer into the
 *                    workspace by a kernel on the caller's stream that reads the host buffer directly | 0: by a
 *                    host-to-device copy command (the stream's next kernel then waits for the copy engine, ~20 us)
 *   "plan_cache"   : 1 (default): the integer plan of a problem (tiles, work units, workspace layout) is kept, keyed
 *                    by the contents of (dtype, d_in, d_out, ranks, offsets), and reused by later calls with the same
 *                    values -- scales and pointers are taken from every call afresh | 0: rebuilt on every call.
 *                    Setting it (to either value) empties the cache.
 * Returns TLORA_EINVAL for an unknown name or an illegal value. */
int tlora_set_option(const char* name, int64_t value);

/* Per-kernel timing, the runtime signal a nano-batch controller feeds on (Algorithm 1, Phase 3:
 * Monitor_Speed).  While enabled, every kernel launch of tlora_fwd / tlora_bwd is bracketed by a
 * pair of HIP events on the call's stream.  tlora_profile(1) enables and clears the totals,
 * tlora_profile(2) does the same for the two segmented-GEMM classes only (an event pair costs a few
 * microseconds of stream time, which adds up over the ~15 short launches of a forward + backward),
 * tlora_profile(0) disables.  tlora_profile_read waits for the recorded events, adds them to the
 * totals and returns, for one kernel class, the summed milliseconds and the number of launches
 * (either output may be NULL).  Returns TLORA_EINVAL for an unknown class. */
typedef enum {
  TLORA_K_PACK = 0,         /* adapter packing                                  */
  TLORA_K_SHRINK = 1,       /* S_j = X_j.A_j and dS_j = dY_j.B_j^T              */
  TLORA_K_GEMM_FWD = 2,     /* Y  = X.W   + fused expand                        */
  TLORA_K_GEMM_BWD = 3,     /* dX = dY.W^T + fused adapter term                 */
  TLORA_K_RANK_GRAD = 4,    /* token reductions of dA_j / dB_j (partial tiles)  */
  TLORA_K_GRAD_REDUCE = 5,  /* fixed-order sum of the partial tiles             */
  TLORA_K_F32 = 6,          /* fp32-configuration products                      */
  TLORA_K_WT = 7,           /* transposed copy of W for the dX product          */
  TLORA_K_OPT = 8,          /* optimizer step                                   */
  TLORA_K_GLUE = 9,         /* RMSNorm, gated SiLU, residual of the MLP block   */
  TLORA_K_PERMUTE = 10,     /* row gather / scatter of the token-indexed calls  */
  TLORA_K_ATTN_FWD = 11,    /* causal attention, forward                        */
  TLORA_K_ATTN_BWD = 12,    /* causal attention, backward (3 kernels)           */
  TLORA_K_ROPE = 13,        /* rotary embedding                                 */
  TLORA_K_COUNT = 14
} tlora_kernel_class_t;
int tlora_profile(int enable);
int tlora_profile_read(int kernel_class, double* total_ms, int64_t* launches);
/* Shader clock (GHz) that a sample of workgroups (every 64th) of the most recent profiled forward / backward
 * segmented GEMM saw across their K-loops (summed cycle counter over summed 100 MHz real-time counter): the
 * clock the chip actually sustained under that kernel's power draw, which scales the attainable MFMA rate.  Synchronises the device.  Either output may be NULL;
 * 0.0 = no profiled launch yet.  The workspace of that call must still be allocated. */
int tlora_profile_clock(double* ghz_fwd, double* ghz_bwd);

/* Static description of an error code. */
const char* tlora_strerror(int status);
/* After a TLORA_EHIP: which HIP error the runtime reported and where in the library's host code ("none" if no call has
 * failed).  The text lives in a static buffer that the next call overwrites. */
const char* tlora_last_hip_error(void);

/* Library version string. */
const char* tlora_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TLORA_H */

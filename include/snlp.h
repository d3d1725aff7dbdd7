/*
 * snlp.h -- C ABI of the SNLP iteration for one MI355X (gfx950).
 *
 * The library evaluates, for a stack of L pre-norm residual Transformer blocks
 *     h_l = f_l(h_{l-1}) = h_{l-1} + g_l(h_{l-1}),   l = 1..L        (Methods, Eq. (1))
 * either layer by layer (Appendix "Algorithm", Alg. 1) or by Structured Newton Layer
 * Parallelism: K rounds of
 *     (1) evaluate every branch g_l on the current estimate of its input, all L layers
 *         in one batched launch per stage                               (Eq. (4)),
 *     (2) apply the structured Newton correction along the layer axis   (Eq. (5)),
 * starting from the "h0" initialisation of Alg. 2.  Two surrogates are built:
 *     IDN  A_l = I   : h_l <- h_{l-1} + g_l, a prefix sum over depth    (Eq. (6)-(7))
 *     HCN  A_l = H_l : X_l <- H_l X_{l-1} + p_l (x) g_l on n residual streams
 *                      (Eq. (8); Appendix "Connection to Hyper-Connections and mHC").
 * A residual-norm probe ||G_l|| = ||h_l - f_l(h_{l-1})|| (Eq. (2)) is produced with the correction.
 *
 * The branch g_l(u), u in R^{M x d}:  x = rmsnorm(u);  [q|k|v] = x Wqkv;  rotary embedding on q, k
 * at position P + t (pairs (c, c + dh/2), angle (P+t) * base^(-2c/dh));  per-head rmsnorm of q, k;
 * softmax(q k^T / sqrt(dh)) v over the P prefix rows (all visible) and the block rows t' <= t;
 * a = heads Wo;  m = relu(rmsnorm(u + a) Wfc)^2 Wproj;  g = a + m.  rmsnorm(x) = x / sqrt(mean(x^2) + eps),
 * no gain, no biases.  On an n-stream model u = sum_j pre_l[j] X_{l-1}[j].
 *
 * Conventions
 *  - Every pointer is a DEVICE pointer unless its comment says "host".  All device memory is owned
 *    by the caller and only borrowed: it must stay valid until snlp_destroy (or until re-bound).
 *  - The library allocates no device memory; scratch lives in the caller's workspace.
 *  - All work is enqueued on the hipStream_t passed as `stream` (NULL = default stream); no call
 *    synchronises the device except where stated.
 *  - Row-major everywhere.  M = B*T token rows, row index = b*T + t.
 *  - Return value: 0 on success, a negative snlp_status otherwise; snlp_last_error() describes it.
 *  - Calls on one context must not overlap in time (they share the workspace).
 */
#ifndef SNLP_H
#define SNLP_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct snlp_ctx snlp_ctx;

typedef enum { SNLP_IDN = 0, SNLP_HCN = 1 } snlp_mode;

/* Operand type of weights, KV prefix and stage buffers.  The trace, the branch outputs and the
 * correction are fp32 in both cases; GEMMs and attention accumulate in fp32. */
typedef enum { SNLP_F32 = 0, SNLP_BF16 = 1 } snlp_dtype;

typedef enum {
  SNLP_OK = 0,
  SNLP_E_BAD_CONFIG = -1,   /* sizes the kernels do not support, or inconsistent sizes       */
  SNLP_E_NOT_BOUND = -2,    /* workspace / weights / trace / KV prefix / HC parameters missing */
  SNLP_E_BAD_ARG = -3,      /* null pointer, negative K, mode not valid for this model        */
  SNLP_E_WORKSPACE = -4,    /* workspace too small or misaligned                              */
  SNLP_E_HIP = -5           /* a HIP runtime call or kernel launch failed                     */
} snlp_status;

typedef struct {
  int L;          /* layers                                                                   */
  int d;          /* model width, = n_heads * head_dim                                        */
  int n_heads;
  int head_dim;   /* SNLP_BF16 requires 128; SNLP_F32 any even value <= 256                   */
  int d_mlp;      /* MLP width F                                                              */
  int n_streams;  /* n: 1 = plain residual model, 2..4 or 8 = hyper-connection model          */
  int B, T, P;    /* sequences, new tokens per sequence, KV-prefix rows per sequence (>= 0)   */
  float rope_base;
  float rms_eps;
  int dtype;      /* snlp_dtype                                                               */
} snlp_config;

/* Create / destroy a context (host object only).  *out is set on success. */
int snlp_create(const snlp_config* cfg, snlp_ctx** out);
void snlp_destroy(snlp_ctx* ctx);
const char* snlp_last_error(const snlp_ctx* ctx);   /* ctx may be NULL: last creation error */

/* Scratch the context needs, and binding it.  `dev` must be 256-byte aligned.  Binding writes the
 * rotary table into the workspace (synchronous copy).  Contents are private to the library. */
size_t snlp_workspace_bytes(const snlp_ctx* ctx);
int snlp_bind_workspace(snlp_ctx* ctx, void* dev, size_t bytes);

/* Per-layer weights, y = x W:  Wqkv [L, d, 3d] (columns q | k | v, head h in columns
 * h*dh .. (h+1)*dh-1 of each third), Wo [L, d, d], Wfc [L, d, F], Wproj [L, F, d]; element type =
 * cfg.dtype (bf16 bit patterns or fp32).  SNLP_BF16 repacks them once into the workspace
 * (enqueued on `stream`); the caller's arrays are not needed after that work completes.
 * Requires a bound workspace. */
int snlp_bind_weights(snlp_ctx* ctx, const void* Wqkv, const void* Wo, const void* Wfc,
                      const void* Wproj, void* stream);

/* Read-only KV-cache prefix, [L, B, H, P, dh], element type = cfg.dtype; keys are used as given
 * (already position-encoded and normalised).  Needed iff P > 0. */
int snlp_bind_kv_prefix(snlp_ctx* ctx, const void* Kpre, const void* Vpre);

/* Hyper-connection parameters, HOST pointers, copied (synchronously) into the workspace:
 * Hres [L, n, n] (X_l[i] += Hres[l][i][j] X_{l-1}[j]), pre [L, n], post [L, n], fp32.
 * For a two-sublayer block pass the product of its two residual mixing matrices (Eq. (8)).
 * Needed iff n_streams > 1. */
int snlp_set_hc(snlp_ctx* ctx, const float* Hres, const float* pre, const float* post);

/* The trace [L+1, M, n, d] fp32; slot 0 is h_0 and is never written by snlp_iterate.
 * The library keeps data derived from the bound trace between calls (for large batches the correction leaves the
 * normalised branch inputs of the next round in the workspace; with snlp_set_skip_converged the count of exact layers).
 * A caller who writes into the bound trace must therefore bind it again (or call snlp_init_trace(_ex)) before
 * the next call that reads it.
 * Under HIP graph capture the same state decides, at capture time, which kernels a round consists of: a round
 * captured directly after snlp_bind_trace or snlp_init_trace(_ex) recomputes every branch input and may be replayed
 * after anything; a round captured after another round may be replayed only where such a round preceded it (capture
 * the initialisation together with the rounds, or capture the first round after an initialisation). */
int snlp_bind_trace(snlp_ctx* ctx, float* trace);

/* Alg. 2 up to the solver loop.  snlp_set_prefix: the first S layers (0 <= S < L, default 0) are evaluated
 * sequentially by the initialisation and stay fixed; snlp_iterate then works on layers S+1..L (probe entries of
 * layers <= S are written as 0).  snlp_init_trace_ex: slot 0 = h0 [M, n, d]; slots 1..S = the sequential layers
 * (h_l = f_l(h_{l-1}), layer map selected by `mode` as in snlp_iterate); then every suffix slot is set to
 *   SNLP_INIT_H0:  h_S                      (the "h0" configurations of Alg. 2)
 *   SNLP_INIT_FWD: f_{S+j}(h_S)             (one-shot batched forward from the prefix state; Methods,
 *                                            "Inference With Fusion and Chunking"): one more batched evaluation.
 * snlp_init_trace = snlp_init_trace_ex with SNLP_INIT_H0 and the model's own layer map (HCN when n_streams > 1).
 * Needs weights etc. bound unless S = 0 with SNLP_INIT_H0. */
typedef enum { SNLP_INIT_H0 = 0, SNLP_INIT_FWD = 1 } snlp_init;
int snlp_set_prefix(snlp_ctx* ctx, int S);
int snlp_init_trace_ex(snlp_ctx* ctx, int mode, int init, const float* h0, void* stream);
int snlp_init_trace(snlp_ctx* ctx, const float* h0, void* stream);

/* Chunkwise fused layers "N x F" (Methods, "Layer fusion" and "Chunkwise strategy"; Appendix "Fused Cross-Layer
 * Coupling"): the L layers are grouped into N = L / F chunks of F consecutive layers that all read the chunk's
 * input h; a chunk is one wide layer
 *     a_C = sum_l O_l Attn_l(h),  u_C = h + a_C,  m_C = sum_l P_l relu(W_l norm(u_C))^2,  F_C(h) = u_C + m_C,
 * and the correction runs between chunk outputs.  After snlp_set_fusion(F) (F must divide L; single-stream models;
 * resets the prefix to 0) every call works in chunk units: the bound trace and trace_out have N + 1 slots
 * [N+1, M, 1, d], probes have N columns, snlp_evaluate_branches / snlp_correction_scan use g [N, M, d], K = N
 * recovers snlp_sequential_forward (the fused model run chunk after chunk) bit for bit.  F = 1 is the plain model.
 * The per-layer projections run as one grouped launch over all layers with the chunk's normalised input as shared
 * operand; the two sum-reductions are done after the O and after the PROJ GEMM (ascending layer order, fp32). */
int snlp_set_fusion(snlp_ctx* ctx, int F);

/* Alg. 2, K rounds of (batched evaluation, correction) in place on the bound trace.
 * mode = SNLP_IDN on any model (on an n-stream model it is the H = I block), SNLP_HCN only when
 * n_streams > 1.  probe: NULL, or [K, 2, L] fp32 receiving for round k and layer l
 *   probe[k][0][l-1] = || X_l - f_l(X_{l-1}) ||_F^2 of the trace ENTERING round k,
 *   probe[k][1][l-1] = || X_l(after) - X_l(before) ||_F^2.
 * K = 0 is a no-op; successive calls continue the iteration. */
int snlp_iterate(snlp_ctx* ctx, int mode, int K, float* probe, void* stream);

/* Leaving converged layers out (follows from Eq. (5) by induction: a layer whose input already equals the
 * sequential state receives a zero correction, so k rounds after an initialisation make layers S+1..S+k exact,
 * and an exact layer never changes again; the one-shot forward initialisation makes layer S+1 exact at once).
 * With on != 0, round k of snlp_iterate / snlp_iterate_diag evaluates and corrects only the layers that can still
 * change; the trace and the probes are bit-identical to the full rounds (probe entries of the layers left out
 * are written as 0, which is what the full round computes for them), at less work: K = L costs L (L + 1) / 2
 * layer evaluations instead of L^2.  The library counts exact layers from the last snlp_init_trace(_ex) on this
 * context; whatever may change the trace or the layer map behind its back (binding a trace, weights, KV prefix
 * or hyper-connection parameters, setting prefix or fusion, snlp_correction_scan(_diag), a round in the other
 * mode on an n-stream model) resets the count.  A caller who writes into the bound trace itself must call
 * snlp_init_trace(_ex) or snlp_bind_trace again before the next round.  Default: off. */
int snlp_set_skip_converged(snlp_ctx* ctx, int on);

/* Alg. 1 with the same kernels, one layer per launch set: trace_out [L+1, M, n, d] receives
 * h0 in slot 0 and h_l = f_l(h_{l-1}) in slot l.  h0 may alias trace_out slot 0.  The bound trace is
 * not touched unless trace_out is it. */
int snlp_sequential_forward(snlp_ctx* ctx, int mode, const float* h0, float* trace_out, void* stream);

/* Eq. (2) on the bound trace at the cost of one evaluation of every branch:
 * out[l-1] = || X_l - f_l(X_{l-1}) ||_F, l = 1..L (fp32).  The trace is not modified. */
int snlp_residual_norm(snlp_ctx* ctx, int mode, float* out, void* stream);

/* Step (1) alone: g_out [L, M, d] fp32 receives g_l evaluated at slot l-1 of the bound trace (rows of the
 * sequential-prefix layers l <= S are not computed and hold unspecified values). */
int snlp_evaluate_branches(snlp_ctx* ctx, float* g_out, void* stream);

/* Step (2) alone, on caller-supplied branch outputs g [L, M, d] fp32: in place on the bound trace,
 * strict fp32 in this order (each operation rounded once, no fused multiply-add):
 *   n = 1:      X_l = X_{l-1} + g_l
 *   HCN:        acc = post_l[i] * g_l;  for j = 0..n-1: acc = acc + Hres_l[i][j] * X_{l-1}[j];  X_l[i] = acc
 *   IDN, n > 1: X_l[i] = X_{l-1}[i] + post_l[i] * g_l
 * probe: NULL or [2, L] as one round of snlp_iterate. */
int snlp_correction_scan(snlp_ctx* ctx, int mode, const float* g, float* probe, void* stream);

/* For callers that cannot allocate device memory or carve a workspace: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  snlp_correction_scan_static is snlp_correction_scan without a context:
 * the same kernels, the same strict-fp32 order and the same probe, on caller-owned buffers only --
 *   trace [L+1, M, n, d] fp32 (slot 0 is read, slots 1..L are written in place), g [L, M, d] fp32,
 *   Hres [L, n, n] and post [L, n] fp32 (DEVICE pointers here; NULL when n_streams == 1; Hres may be NULL for
 *   SNLP_IDN), probe NULL or [2, L] fp32 as one round of snlp_iterate.
 * The probe's per-workgroup partial sums go to a fixed array inside the library (SNLP_STATIC_SCRATCH_BYTES =
 * 4 MiB of device memory per GPU, held until the process ends) instead of a workspace.  The call allocates nothing
 * and frees nothing; its only set-up is resolving that array's device address the first time it runs on a GPU
 * (so make the first call on each GPU outside a stream capture).  Limits: ceil(M * d / 4 / b) * 2 * L <= 2^20
 * floats with b = 64 when M * d <= 2^20 and 256 otherwise (all five benchmark shapes fit); a shape beyond that
 * with probe != NULL returns SNLP_E_WORKSPACE and launches nothing (probe = NULL needs no scratch and always fits).
 * Errors are reported through snlp_last_error(NULL).  All calls on one GPU share the one array: calls that overlap
 * in time on the same GPU (different streams or threads) race on it and must be serialised by the caller; nothing
 * in it has to start at zero, every entry that is read is written first by the same call. */
#define SNLP_STATIC_SCRATCH_BYTES ((size_t)4 << 20)
int snlp_correction_scan_static(int mode, int L, int M, int n_streams, int d, float* trace, const float* g,
                                const float* Hres, const float* post, float* probe, void* stream);

/* Diagonal surrogate A_l = diag(a_l) (Methods, "Diagonal Newton (DiagN)"; Appendix "Algorithm", Alg. 3) with the
 * diagonals SUPPLIED by the caller, diag [L, M, d] fp32 (how they are estimated is outside this library).
 * Single-stream models only.  The elementwise affine recurrence of Alg. 3 is walked left to right in strict fp32:
 *   h~ = h_{l-1}(old) + g_l;   h_l(new) = h~ + a_l * (h_{l-1}(new) - h_{l-1}(old))      (each operation rounded once)
 * a = 1 is IDN up to rounding, a = 0 the uncorrected fixed point; for any a, k rounds make layers 1..k exact.
 * snlp_correction_scan_diag: on caller-supplied branch outputs g [L, M, d]; snlp_iterate_diag: K rounds of
 * (batched evaluation, diagonal correction) with the same diagonals each round.  probe as in snlp_iterate. */
int snlp_correction_scan_diag(snlp_ctx* ctx, const float* g, const float* diag, float* probe, void* stream);
int snlp_iterate_diag(snlp_ctx* ctx, int K, const float* diag, float* probe, void* stream);

/* Diagnostic: device address and byte size of a stage buffer of the last evaluation
 * ("xhat", "qkv", "attn", "a", "xhat2", "hmid", "g", "u").  Layout [L, M, width], element type per dtype
 * ("a", "g", "u" always fp32).  After a correction on a large batch "xhat" and "u" already hold the inputs of the
 * NEXT evaluation (see snlp_bind_trace); after snlp_evaluate_branches / snlp_residual_norm they are the evaluation's own. */
int snlp_stage_buffer(snlp_ctx* ctx, const char* name, void** dev, size_t* bytes);

/* Measurement aid: per-stage timing with HIP events recorded on the caller's stream around the stage's
 * launches.  Stages: 0 stream pre-mix + rmsnorm, 1 QKV GEMM, 2 rotary + QK-norm, 3 attention, 4 O GEMM,
 * 5 mid-residual rmsnorm, 6 FC GEMM (+ ReLU^2), 7 PROJ GEMM (+ a), 8 correction scan (+ probe reduction).
 * snlp_profile_stages: bit i of stage_mask selects stage i for all following calls; 0 switches timing off.
 * snlp_profile_read: waits for the recorded events, writes the summed milliseconds and the number of
 * timed launches per stage since the last read into the HOST arrays ms[SNLP_N_STAGES], count[SNLP_N_STAGES],
 * and resets.  Events are created on first use (host objects; no device memory). */
#define SNLP_N_STAGES 9
int snlp_profile_stages(snlp_ctx* ctx, unsigned stage_mask);
int snlp_profile_read(snlp_ctx* ctx, float* ms, int* count);

#ifdef __cplusplus
}
#endif
#endif /* SNLP_H */

// Internal launch interface between the C ABI (snlp_api.hip) and the gfx950 kernels.
// Every launcher enqueues on `s` and returns hipGetLastError().
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace snlp {

typedef uint16_t bf16_t;   // bfloat16 bit pattern in memory

// Sizes of the model and of one batch of token rows.
struct Dims {
  int L, d, H, dh, F, n, B, T, P, M;
  float eps;
};

enum Epilogue {
  EPI_STORE = 0,      // C = acc
  EPI_RELU2 = 1,      // C = max(acc, 0)^2
  EPI_ADD_F32 = 2     // C = R + acc  (R fp32 [M, N], C fp32): used for g = a + m
};

// ---- elementwise / norm / rotary / correction (snlp_elementwise.hip)
// xhat[l] = rmsnorm(sum_j pre[l][j] X_{l-1}[j]) for layers l0..l0+Lc-1 (1-based); for n > 1 the mixed input
// is also stored in ubuf[l-1] (fp32 [M, d]).  out element type: bf16 if out_bf16 else fp32.
hipError_t launch_premix_rmsnorm(hipStream_t s, const Dims& D, int l0, int Lc, const float* trace,
                                 const float* pre, float* ubuf, void* xhat, bool out_bf16);
// xhat2[l] = rmsnorm(u_l + a_l), u_l = trace slot l-1 (n = 1) or ubuf[l-1] (n > 1).
hipError_t launch_mid_rmsnorm(hipStream_t s, const Dims& D, int l0, int Lc, const float* trace,
                              const float* ubuf, const float* a, void* xhat2, bool out_bf16);
// Fused chunks of F layers (single-stream): aC[c] = sum_j a[(c-1)F + j], xhat2[c] = rmsnorm(trace slot c-1 + aC[c]);
// gC[c] = aC[c] + sum_j m[(c-1)F + j].  Chunk-indexed buffers are [chunks, M, d].
hipError_t launch_chunk_mid_rmsnorm(hipStream_t s, const Dims& D, int c0, int Nc, int F, const float* trace,
                                    const float* a, float* aC, void* xhat2, bool out_bf16);
hipError_t launch_chunk_sum(hipStream_t s, const Dims& D, int c0, int Nc, int F, const float* aC, const float* m, float* gC);
// In place on qkv [L, M, 3d]: rotary embedding then per-head rmsnorm of the q and k thirds.
hipError_t launch_rope_qknorm(hipStream_t s, const Dims& D, int l0, int Lc, void* qkv, bool is_bf16,
                              const float* cos_tab, const float* sin_tab);
// trace[l] = src ([M, n, d]) for l = first..first+count-1.
hipError_t launch_init_trace(hipStream_t s, const Dims& D, const float* src, float* trace, int first, int count);
// The structured correction over layers l0..l0+Lc-1 starting from slot l0-1, in place on `trace`
// (write = true) or read-only (write = false), with optional squared-norm partials
// partials[nblk][2][Lc] (see scan_partial_blocks) reduced into probe[2][Lc] by launch_probe_finalize.
int scan_partial_blocks(const Dims& D);
// independent = true: every layer steps from slot l0-1 instead of from its predecessor (one-shot forward).
hipError_t launch_scan(hipStream_t s, const Dims& D, int mode, int l0, int Lc, float* trace, const float* g,
                       const float* Hres, const float* post, bool write, float* partials, bool independent = false);
// Diagonal-surrogate correction (single-stream traces only), diag [L, M, d] fp32.
hipError_t launch_scan_diag(hipStream_t s, const Dims& D, int l0, int Lc, float* trace, const float* g,
                            const float* diag, float* partials);
// The same correction (in place, dependent layers) that also leaves, for every layer l + 1 <= L after a layer l it
// has corrected, the branch input of the next evaluation: ubuf[l] (n > 1) and xhat[l] = what launch_premix_rmsnorm would
// compute from the new slot l, bit for bit.  Only for shapes with scan_fuses_norm(D); partials then have
// scan_norm_blocks(D) rows.
bool scan_fuses_norm(const Dims& D);
int scan_norm_blocks(const Dims& D);
hipError_t launch_scan_norm(hipStream_t s, const Dims& D, int mode, int l0, int Lc, float* trace, const float* g,
                            const float* Hres, const float* post, const float* pre, float* ubuf, void* xhat,
                            bool out_bf16, float* partials);
// probe rows have col0 + Lc columns: the first col0 (sequential prefix) are written as zero.  nblk: rows of `partials`
// (<= 0: scan_partial_blocks(D)).
hipError_t launch_probe_finalize(hipStream_t s, const Dims& D, int Lc, const float* partials, float* probe,
                                 bool take_sqrt_first_only, int col0 = 0, int nblk = -1);
// bf16 [L][K][N] -> [L][N][K] (one-time weight repack).
hipError_t launch_transpose_bf16(hipStream_t s, const bf16_t* in, bf16_t* out, int L, int K, int N);

// ---- GEMMs (snlp_gemm.hip): for layers li = 0..Lc-1, C[li] = epi(A[li] (M x K) * W[li] (K x N)).
// Strides are in elements between consecutive layers; a_group consecutive layers share one A slab (fused
// chunks: A of layer li is A + (li / a_group) * sA).  fp32 path: W row-major [K, N].
hipError_t launch_gemm_f32(hipStream_t s, int Lc, int M, int N, int K, const float* A, size_t sA,
                           const float* W, size_t sW, float* C, size_t sC, int epi, const float* R, size_t sR,
                           int a_group = 1);
// bf16 path: A bf16 [M, K]; W repacked by launch_repack_weights for this M (M > 128: [N, K] row-major;
// M <= 128: MFMA operand order [N/32][K/16][64][8]); C bf16 (EPI_STORE / EPI_RELU2 with c_bf16) or fp32.
hipError_t launch_gemm_bf16(hipStream_t s, int Lc, int M, int N, int K, const bf16_t* A, size_t sA,
                            const bf16_t* Wt, size_t sW, void* C, size_t sC, bool c_bf16, int epi,
                            const float* R, size_t sR, int a_group = 1);
bool gemm_bf16_supported(int M, int N, int K);
hipError_t launch_repack_weights(hipStream_t s, const bf16_t* in /*[L][K][N]*/, bf16_t* out, int L, int K, int N, int M);

// ---- attention (snlp_attention.hip): out[l][M, d] from qkv[l][M, 3d] and the KV prefix of layer l.
hipError_t launch_attention_f32(hipStream_t s, const Dims& D, int l0, int Lc, const float* qkv,
                                const float* Kpre, const float* Vpre, float* out, float* score_ws);
size_t attention_f32_ws_floats(const Dims& D);
// With decode-sized blocks behind a long prefix (attention_bf16_fuses_rope) the kernel applies the rotary embedding and QK norm to q and
// to the block's k rows itself when given the tables (cos_tab != nullptr); launch_rope_qknorm must then be skipped.
// For longer blocks the tables are ignored and qkv must already be rotated and normalised.
bool attention_bf16_fuses_rope(const Dims& D);
hipError_t launch_attention_bf16(hipStream_t s, const Dims& D, int l0, int Lc, const bf16_t* qkv,
                                 const bf16_t* Kpre, const bf16_t* Vpre, bf16_t* out, const float* cos_tab,
                                 const float* sin_tab);

}  // namespace snlp

// C ABI of the SNLP iteration (declared in include/snlp.h): context, workspace carving, and the launch
// sequences of Alg. 1 (sequential layers) and Alg. 2 (batched evaluation + structured correction).
// Host code only; every arithmetic step runs in the gfx950 kernels of this library.
#include "../../include/snlp.h"
#include "snlp_kernels.hpp"

#include <climits>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

using namespace snlp;

namespace {
thread_local std::string g_create_error;

size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }
}  // namespace

struct snlp_ctx {
  snlp_config cfg;
  Dims D;
  bool bf16;
  size_t esz;   // bytes per operand element
  std::string err;

  // workspace layout (byte offsets)
  size_t off_cos, off_sin, off_H, off_pre, off_post;
  size_t off_wqkv, off_wo, off_wfc, off_wproj;
  size_t off_xhat, off_qkv, off_attn, off_a, off_xhat2, off_hmid, off_g, off_u, off_partials, off_probe;
  size_t ws_bytes;

  char* ws = nullptr;
  bool weights_bound = false, hc_set = false;
  const void* Wqkv = nullptr; const void* Wo = nullptr; const void* Wfc = nullptr; const void* Wproj = nullptr;
  const void* Kpre = nullptr; const void* Vpre = nullptr;
  float* trace = nullptr;
  int S = 0;   // sequential prefix length: layers S+1..L are iterated
  int Fz = 1;  // layers per fused chunk; the trace has L / Fz + 1 slots ("units" below are chunks when Fz > 1)
  // Leading units of the bound trace known to equal the sequential result under layer map `exact_map`
  // (-1: nothing known): k rounds after an initialisation make units 1..k exact, and an exact unit never changes
  // again, so with `skip` on a round leaves them out.
  bool skip = false;
  int exact = 0;
  int exact_map = -1;
  int layer_map(int mode) const { return D.n == 1 ? 0 : mode; }
  void forget_exact() { exact_map = -1; exact = 0; }
  int first_unit(int mode) const {   // first unit a round has to work on
    if (!skip || exact_map != layer_map(mode)) return S + 1;
    const int e = exact > S ? exact : S;
    return e + 1 < units() ? e + 1 : units();
  }
  void round_done(int mode) {
    if (exact_map != layer_map(mode)) { exact_map = layer_map(mode); exact = S; }
    if (exact < S) exact = S;
    if (exact < units()) ++exact;
  }

  // The normalised branch inputs (stage buffers xhat, and u on n-stream models) of layers >= xhat_from are those of the
  // bound trace as it stands: the correction kernel for large batches leaves them behind for the next round, which
  // then runs the stand-alone norm pass only for the layers before that (INT_MAX: nothing known).
  int xhat_from = INT_MAX;
  void forget_xhat() { xhat_from = INT_MAX; }
  bool fuses_norm() const { return Fz == 1 && scan_fuses_norm(D); }

  int units() const { return D.L / Fz; }
  float* gbuf() const { return reinterpret_cast<float*>(ws + (Fz > 1 ? off_a : off_g)); }   // per-unit branch outputs

  // stage timing (measurement aid): event pairs recorded on the caller's stream
  struct Timed { hipEvent_t start, stop; int stage; };
  unsigned profile_mask = 0;
  std::vector<Timed> timed;        // recorded since the last read
  std::vector<Timed> spare;        // created, reusable

  template <typename T> T* at(size_t off) const { return reinterpret_cast<T*>(ws + off); }
};

namespace {

int fail(snlp_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg; else g_create_error = msg;
  return code;
}

int hip_fail(snlp_ctx* c, hipError_t e, const char* what) {
  return fail(c, SNLP_E_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

void carve(snlp_ctx* c) {
  const Dims& D = c->D;
  const size_t L = D.L, M = D.M, d = D.d, F = D.F, n = D.n;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
  const size_t rope = (size_t)D.T * (D.dh / 2) * sizeof(float);
  c->off_cos = take(rope);
  c->off_sin = take(rope);
  c->off_H = take(L * n * n * sizeof(float));
  c->off_pre = take(L * n * sizeof(float));
  c->off_post = take(L * n * sizeof(float));
  if (c->bf16) {
    c->off_wqkv = take(L * d * 3 * d * 2);
    c->off_wo = take(L * d * d * 2);
    c->off_wfc = take(L * d * F * 2);
    c->off_wproj = take(L * F * d * 2);
  } else {
    c->off_wqkv = c->off_wo = c->off_wfc = c->off_wproj = 0;
  }
  c->off_xhat = take(L * M * d * c->esz);
  c->off_qkv = take(L * M * 3 * d * c->esz);
  c->off_attn = take(L * M * d * c->esz);
  c->off_a = take(L * M * d * sizeof(float));
  c->off_xhat2 = take(L * M * d * c->esz);
  c->off_hmid = take(L * M * F * c->esz);
  c->off_g = take(L * M * d * sizeof(float));
  c->off_u = take(L * M * d * sizeof(float));   // pre-mixed input (n > 1) or summed attention updates of fused chunks
  const size_t pblocks = scan_fuses_norm(D) && scan_norm_blocks(D) > scan_partial_blocks(D) ? scan_norm_blocks(D) : scan_partial_blocks(D);
  c->off_partials = take(pblocks * 2 * L * sizeof(float));
  c->off_probe = take(2 * L * sizeof(float));
  c->ws_bytes = o;
}

int check_ready(snlp_ctx* c, bool need_trace) {
  if (!c) return SNLP_E_BAD_ARG;
  if (!c->ws) return fail(c, SNLP_E_NOT_BOUND, "workspace not bound");
  if (!c->weights_bound) return fail(c, SNLP_E_NOT_BOUND, "weights not bound");
  if (c->D.P > 0 && (!c->Kpre || !c->Vpre)) return fail(c, SNLP_E_NOT_BOUND, "KV prefix not bound (P > 0)");
  if (c->D.n > 1 && !c->hc_set) return fail(c, SNLP_E_NOT_BOUND, "hyper-connection parameters not set (n_streams > 1)");
  if (need_trace && !c->trace) return fail(c, SNLP_E_NOT_BOUND, "trace not bound");
  return SNLP_OK;
}

int check_mode(snlp_ctx* c, int mode) {
  if (mode != SNLP_IDN && mode != SNLP_HCN) return fail(c, SNLP_E_BAD_ARG, "mode must be SNLP_IDN or SNLP_HCN");
  if (mode == SNLP_HCN && c->D.n == 1) return fail(c, SNLP_E_BAD_ARG, "SNLP_HCN needs n_streams > 1");
  return SNLP_OK;
}

// Records a start event now and a stop event when it goes out of scope, if the stage is selected.
struct StageTimer {
  snlp_ctx* c; hipStream_t s; bool on = false; snlp_ctx::Timed t{};
  StageTimer(snlp_ctx* c_, int stage, hipStream_t s_) : c(c_), s(s_) {
    if (!((c->profile_mask >> stage) & 1u)) return;
    if (!c->spare.empty()) { t = c->spare.back(); c->spare.pop_back(); }
    else if (hipEventCreate(&t.start) != hipSuccess || hipEventCreate(&t.stop) != hipSuccess) return;
    t.stage = stage;
    on = hipEventRecord(t.start, s) == hipSuccess;
  }
  ~StageTimer() {
    if (!on) return;
    (void)hipEventRecord(t.stop, s);
    c->timed.push_back(t);
  }
};

#define SNLP_TRY(expr, what)                               \
  do {                                                     \
    hipError_t e_ = (expr);                                \
    if (e_ != hipSuccess) return hip_fail(c, e_, what);    \
  } while (0)

// Step (1) of the iteration for layers l0..l0+Lc-1 (1-based) reading slot l-1 of `trace`: leaves
// g_l = a_l + m_l in the g stage buffer.
int evaluate_layers(snlp_ctx* c, int l0, int Lc, const float* trace, hipStream_t s, int valid_from) {
  const Dims& D = c->D;
  const size_t M = D.M, d = D.d, F = D.F;
  const size_t lo = (size_t)(l0 - 1);
  const bool bf = c->bf16;
  const size_t e = c->esz;
  char* xhat = c->ws + c->off_xhat;
  char* qkv = c->ws + c->off_qkv;
  char* attn = c->ws + c->off_attn;
  float* a = c->at<float>(c->off_a);
  char* xhat2 = c->ws + c->off_xhat2;
  char* hmid = c->ws + c->off_hmid;
  float* g = c->at<float>(c->off_g);
  float* u = c->at<float>(c->off_u);

  // layers from valid_from on already have their (pre-mixed and) normalised input in the stage buffers
  const int npre = valid_from <= l0 ? 0 : (valid_from - l0 < Lc ? valid_from - l0 : Lc);
  if (npre > 0) { StageTimer tm(c, 0, s);
  SNLP_TRY(launch_premix_rmsnorm(s, D, l0, npre, trace, c->at<float>(c->off_pre), u, xhat, bf), "premix_rmsnorm"); }
  { StageTimer tm(c, 1, s);
  if (bf) {
    SNLP_TRY(launch_gemm_bf16(s, Lc, D.M, 3 * D.d, D.d, (const bf16_t*)(xhat + lo * M * d * e), M * d,
                              c->at<bf16_t>(c->off_wqkv) + lo * d * 3 * d, d * 3 * d, qkv + lo * M * 3 * d * e,
                              M * 3 * d, true, EPI_STORE, nullptr, 0), "gemm qkv");
  } else {
    SNLP_TRY(launch_gemm_f32(s, Lc, D.M, 3 * D.d, D.d, (const float*)(xhat + lo * M * d * e), M * d,
                             (const float*)c->Wqkv + lo * d * 3 * d, d * 3 * d, (float*)(qkv + lo * M * 3 * d * e),
                             M * 3 * d, EPI_STORE, nullptr, 0), "gemm qkv");
  } }
  // decode-sized bf16 blocks: the attention kernel rotates and normalises q and the block's k rows itself
  const bool fused_rope = bf && attention_bf16_fuses_rope(D);
  if (!fused_rope) { StageTimer tm(c, 2, s);
  SNLP_TRY(launch_rope_qknorm(s, D, l0, Lc, qkv, bf, c->at<float>(c->off_cos), c->at<float>(c->off_sin)), "rope_qknorm"); }
  { StageTimer tm(c, 3, s);
  if (bf)
    SNLP_TRY(launch_attention_bf16(s, D, l0, Lc, (const bf16_t*)qkv, (const bf16_t*)c->Kpre, (const bf16_t*)c->Vpre,
                                   (bf16_t*)attn, fused_rope ? c->at<float>(c->off_cos) : nullptr,
                                   fused_rope ? c->at<float>(c->off_sin) : nullptr), "attention");
  else
    SNLP_TRY(launch_attention_f32(s, D, l0, Lc, (const float*)qkv, (const float*)c->Kpre, (const float*)c->Vpre,
                                  (float*)attn, nullptr), "attention");
  }
  { StageTimer tm(c, 4, s);
  if (bf)
    SNLP_TRY(launch_gemm_bf16(s, Lc, D.M, D.d, D.d, (const bf16_t*)(attn + lo * M * d * e), M * d,
                              c->at<bf16_t>(c->off_wo) + lo * d * d, d * d, a + lo * M * d, M * d, false, EPI_STORE,
                              nullptr, 0), "gemm o");
  else
    SNLP_TRY(launch_gemm_f32(s, Lc, D.M, D.d, D.d, (const float*)(attn + lo * M * d * e), M * d,
                             (const float*)c->Wo + lo * d * d, d * d, a + lo * M * d, M * d, EPI_STORE, nullptr, 0), "gemm o");
  }
  { StageTimer tm(c, 5, s);
  SNLP_TRY(launch_mid_rmsnorm(s, D, l0, Lc, trace, u, a, xhat2, bf), "mid_rmsnorm"); }
  { StageTimer tm(c, 6, s);
  if (bf)
    SNLP_TRY(launch_gemm_bf16(s, Lc, D.M, D.F, D.d, (const bf16_t*)(xhat2 + lo * M * d * e), M * d,
                              c->at<bf16_t>(c->off_wfc) + lo * d * F, d * F, hmid + lo * M * F * e, M * F, true,
                              EPI_RELU2, nullptr, 0), "gemm fc");
  else
    SNLP_TRY(launch_gemm_f32(s, Lc, D.M, D.F, D.d, (const float*)(xhat2 + lo * M * d * e), M * d,
                             (const float*)c->Wfc + lo * d * F, d * F, (float*)(hmid + lo * M * F * e), M * F, EPI_RELU2,
                             nullptr, 0), "gemm fc");
  }
  { StageTimer tm(c, 7, s);
  if (bf)
    SNLP_TRY(launch_gemm_bf16(s, Lc, D.M, D.d, D.F, (const bf16_t*)(hmid + lo * M * F * e), M * F,
                              c->at<bf16_t>(c->off_wproj) + lo * F * d, F * d, g + lo * M * d, M * d, false,
                              EPI_ADD_F32, a + lo * M * d, M * d), "gemm proj");
  else
    SNLP_TRY(launch_gemm_f32(s, Lc, D.M, D.d, D.F, (const float*)(hmid + lo * M * F * e), M * F,
                             (const float*)c->Wproj + lo * F * d, F * d, g + lo * M * d, M * d, EPI_ADD_F32,
                             a + lo * M * d, M * d), "gemm proj");
  }
  return SNLP_OK;
}

// Step (1) for fused chunks c0..c0+Nc-1 (1-based) of Fz layers each, every layer of a chunk reading slot c-1
// (Methods, "Layer fusion"; Appendix "Fused Cross-Layer Coupling"): the per-layer projections run as one grouped
// launch over all layers with the chunk's normalised input as their shared A operand; the sum-reductions after
// the attention output projection and after the MLP projection are done by the two chunk kernels.  Leaves
// g_C = a_C + m_C in gbuf() (chunk-indexed).
int evaluate_fused(snlp_ctx* c, int c0, int Nc, const float* trace, hipStream_t s) {
  const Dims& D = c->D;
  const int Fz = c->Fz;
  const size_t M = D.M, d = D.d, F = D.F;
  const size_t co = (size_t)(c0 - 1);          // first chunk (0-based)
  const size_t lo = co * Fz;                   // first layer (0-based)
  const int l0 = (int)lo + 1, Lc = Nc * Fz;
  const bool bf = c->bf16;
  const size_t e = c->esz;
  char* xhat = c->ws + c->off_xhat;
  char* qkv = c->ws + c->off_qkv;
  char* attn = c->ws + c->off_attn;
  float* a = c->at<float>(c->off_a);
  char* xhat2 = c->ws + c->off_xhat2;
  char* hmid = c->ws + c->off_hmid;
  float* m = c->at<float>(c->off_g);           // per-layer MLP updates
  float* aC = c->at<float>(c->off_u);          // per-chunk summed attention updates

  { StageTimer tm(c, 0, s);
  SNLP_TRY(launch_premix_rmsnorm(s, D, c0, Nc, trace, nullptr, nullptr, xhat, bf), "chunk rmsnorm"); }
  { StageTimer tm(c, 1, s);
  if (bf)
    SNLP_TRY(launch_gemm_bf16(s, Lc, D.M, 3 * D.d, D.d, (const bf16_t*)(xhat + co * M * d * e), M * d,
                              c->at<bf16_t>(c->off_wqkv) + lo * d * 3 * d, d * 3 * d, qkv + lo * M * 3 * d * e,
                              M * 3 * d, true, EPI_STORE, nullptr, 0, Fz), "gemm qkv");
  else
    SNLP_TRY(launch_gemm_f32(s, Lc, D.M, 3 * D.d, D.d, (const float*)(xhat + co * M * d * e), M * d,
                             (const float*)c->Wqkv + lo * d * 3 * d, d * 3 * d, (float*)(qkv + lo * M * 3 * d * e),
                             M * 3 * d, EPI_STORE, nullptr, 0, Fz), "gemm qkv");
  }
  // decode-sized bf16 blocks: the attention kernel rotates and normalises q and the block's k rows itself
  const bool fused_rope = bf && attention_bf16_fuses_rope(D);
  if (!fused_rope) { StageTimer tm(c, 2, s);
  SNLP_TRY(launch_rope_qknorm(s, D, l0, Lc, qkv, bf, c->at<float>(c->off_cos), c->at<float>(c->off_sin)), "rope_qknorm"); }
  { StageTimer tm(c, 3, s);
  if (bf)
    SNLP_TRY(launch_attention_bf16(s, D, l0, Lc, (const bf16_t*)qkv, (const bf16_t*)c->Kpre, (const bf16_t*)c->Vpre,
                                   (bf16_t*)attn, fused_rope ? c->at<float>(c->off_cos) : nullptr,
                                   fused_rope ? c->at<float>(c->off_sin) : nullptr), "attention");
  else
    SNLP_TRY(launch_attention_f32(s, D, l0, Lc, (const float*)qkv, (const float*)c->Kpre, (const float*)c->Vpre,
                                  (float*)attn, nullptr), "attention");
  }
  { StageTimer tm(c, 4, s);
  if (bf)
    SNLP_TRY(launch_gemm_bf16(s, Lc, D.M, D.d, D.d, (const bf16_t*)(attn + lo * M * d * e), M * d,
                              c->at<bf16_t>(c->off_wo) + lo * d * d, d * d, a + lo * M * d, M * d, false, EPI_STORE,
                              nullptr, 0), "gemm o");
  else
    SNLP_TRY(launch_gemm_f32(s, Lc, D.M, D.d, D.d, (const float*)(attn + lo * M * d * e), M * d,
                             (const float*)c->Wo + lo * d * d, d * d, a + lo * M * d, M * d, EPI_STORE, nullptr, 0), "gemm o");
  }
  { StageTimer tm(c, 5, s);
  SNLP_TRY(launch_chunk_mid_rmsnorm(s, D, c0, Nc, Fz, trace, a, aC, xhat2, bf), "chunk mid rmsnorm"); }
  { StageTimer tm(c, 6, s);
  if (bf)
    SNLP_TRY(launch_gemm_bf16(s, Lc, D.M, D.F, D.d, (const bf16_t*)(xhat2 + co * M * d * e), M * d,
                              c->at<bf16_t>(c->off_wfc) + lo * d * F, d * F, hmid + lo * M * F * e, M * F, true,
                              EPI_RELU2, nullptr, 0, Fz), "gemm fc");
  else
    SNLP_TRY(launch_gemm_f32(s, Lc, D.M, D.F, D.d, (const float*)(xhat2 + co * M * d * e), M * d,
                             (const float*)c->Wfc + lo * d * F, d * F, (float*)(hmid + lo * M * F * e), M * F, EPI_RELU2,
                             nullptr, 0, Fz), "gemm fc");
  }
  { StageTimer tm(c, 7, s);
  if (bf)
    SNLP_TRY(launch_gemm_bf16(s, Lc, D.M, D.d, D.F, (const bf16_t*)(hmid + lo * M * F * e), M * F,
                              c->at<bf16_t>(c->off_wproj) + lo * F * d, F * d, m + lo * M * d, M * d, false,
                              EPI_STORE, nullptr, 0), "gemm proj");
  else
    SNLP_TRY(launch_gemm_f32(s, Lc, D.M, D.d, D.F, (const float*)(hmid + lo * M * F * e), M * F,
                             (const float*)c->Wproj + lo * F * d, F * d, m + lo * M * d, M * d, EPI_STORE, nullptr, 0),
             "gemm proj");
  SNLP_TRY(launch_chunk_sum(s, D, c0, Nc, Fz, aC, m, c->gbuf()), "chunk sum");
  }
  return SNLP_OK;
}

// Units are layers, or fused chunks when Fz > 1.
int evaluate(snlp_ctx* c, int u0, int Uc, const float* trace, hipStream_t s, int valid_from = INT_MAX) {
  return c->Fz > 1 ? evaluate_fused(c, u0, Uc, trace, s) : evaluate_layers(c, u0, Uc, trace, s, valid_from);
}

// Evaluation on the bound trace: uses, and afterwards records, which layers' normalised inputs are current.
int evaluate_bound(snlp_ctx* c, int u0, int Uc, hipStream_t s) {
  if (c->Fz > 1) { c->forget_xhat(); return evaluate_fused(c, u0, Uc, c->trace, s); }
  const int rc = evaluate_layers(c, u0, Uc, c->trace, s, c->xhat_from);
  if (rc == SNLP_OK && u0 + Uc - 1 >= c->D.L && c->xhat_from > u0) c->xhat_from = u0;   // the norm pass filled u0 .. xhat_from - 1
  return rc;
}

// fuse_norm: the correction also leaves the next evaluation's normalised inputs of layers l0 + 1 .. L in the stage
// buffers (large batches only; the caller keeps the bookkeeping).  Returns through *fused whether it did.
int correct(snlp_ctx* c, int mode, int l0, int Lc, float* trace, const float* g, bool write, float* probe_out,
            bool sqrt_first, hipStream_t s, bool independent = false, bool fuse_norm = false, bool* fused = nullptr) {
  const Dims& D = c->D;
  float* partials = (probe_out || !write) ? c->at<float>(c->off_partials) : nullptr;
  const float* H = D.n > 1 ? c->at<float>(c->off_H) : nullptr;
  const float* post = D.n > 1 ? c->at<float>(c->off_post) : nullptr;
  const bool fuse = fuse_norm && write && !independent && c->fuses_norm();
  if (fused) *fused = fuse;
  StageTimer tm(c, 8, s);
  if (fuse) {
    SNLP_TRY(launch_scan_norm(s, D, mode, l0, Lc, trace, g, H, post, c->at<float>(c->off_pre), c->at<float>(c->off_u),
                              c->ws + c->off_xhat, c->bf16, partials), "correction scan + next inputs");
    if (probe_out) SNLP_TRY(launch_probe_finalize(s, D, Lc, partials, probe_out, sqrt_first, l0 - 1, scan_norm_blocks(D)), "probe finalize");
    return SNLP_OK;
  }
  SNLP_TRY(launch_scan(s, D, mode, l0, Lc, trace, g, H, post, write, partials, independent), "correction scan");
  if (probe_out) SNLP_TRY(launch_probe_finalize(s, D, Lc, partials, probe_out, sqrt_first, l0 - 1), "probe finalize");
  return SNLP_OK;
}

// One round's correction on the bound trace with the bookkeeping of the stage buffers.
int correct_bound(snlp_ctx* c, int mode, int l0, int Lc, const float* g, float* probe_out, hipStream_t s) {
  bool fused = false;
  const int rc = correct(c, mode, l0, Lc, c->trace, g, true, probe_out, false, s, false, true, &fused);
  if (rc != SNLP_OK) { c->forget_xhat(); return rc; }
  // fused: layers l0 + 1 .. L are fresh and whatever was current up to l0 still is (their input slots did not change)
  if (fused) { if (c->xhat_from > l0 + 1) c->xhat_from = l0 + 1; }
  else c->forget_xhat();
  return rc;
}

}  // namespace

extern "C" {

int snlp_create(const snlp_config* cfg, snlp_ctx** out) {
  if (!cfg || !out) return fail(nullptr, SNLP_E_BAD_ARG, "null argument");
  const snlp_config& k = *cfg;
  auto bad = [&](const char* m) { return fail(nullptr, SNLP_E_BAD_CONFIG, m); };
  if (k.L < 1 || k.L > 256) return bad("L must be in 1..256");
  if (k.d < 4 || k.n_heads < 1 || k.head_dim < 2 || k.n_heads * k.head_dim != k.d) return bad("d must equal n_heads * head_dim");
  if (k.d % 4 != 0 || k.d > 4096) return bad("d must be a multiple of 4 and at most 4096");
  if (k.head_dim % 2 != 0 || k.head_dim > 256) return bad("head_dim must be even and at most 256");
  if (k.d_mlp < 1) return bad("d_mlp must be positive");
  if (!(k.n_streams == 1 || k.n_streams == 2 || k.n_streams == 3 || k.n_streams == 4 || k.n_streams == 8))
    return bad("n_streams must be 1, 2, 3, 4 or 8");
  if (k.B < 1 || k.T < 1 || k.P < 0) return bad("B, T must be positive and P non-negative");
  if ((long long)k.B * k.T * (k.d / 4) >= (1ll << 31)) return bad("B * T * d too large");
  if (!(k.rms_eps > 0.f) || !(k.rope_base > 1.f)) return bad("rms_eps must be > 0 and rope_base > 1");
  if (k.dtype != SNLP_F32 && k.dtype != SNLP_BF16) return bad("dtype must be SNLP_F32 or SNLP_BF16");
  if (k.dtype == SNLP_BF16) {
    if (k.head_dim != 128) return bad("SNLP_BF16 requires head_dim == 128");
    if (k.d_mlp % 64 != 0) return bad("SNLP_BF16 requires d_mlp to be a multiple of 64");
  } else {
    if ((size_t)(k.head_dim + k.P + k.T) * sizeof(float) > 64 * 1024) return bad("SNLP_F32 requires head_dim + P + T <= 16384");
  }
  snlp_ctx* c = new snlp_ctx();
  c->cfg = k;
  c->D = Dims{k.L, k.d, k.n_heads, k.head_dim, k.d_mlp, k.n_streams, k.B, k.T, k.P, k.B * k.T, k.rms_eps};
  c->bf16 = k.dtype == SNLP_BF16;
  c->esz = c->bf16 ? 2 : 4;
  carve(c);
  *out = c;
  return SNLP_OK;
}

void snlp_destroy(snlp_ctx* ctx) {
  if (!ctx) return;
  for (auto* v : {&ctx->timed, &ctx->spare})
    for (auto& t : *v) { (void)hipEventDestroy(t.start); (void)hipEventDestroy(t.stop); }
  delete ctx;
}

int snlp_profile_stages(snlp_ctx* c, unsigned stage_mask) {
  if (!c) return SNLP_E_BAD_ARG;
  c->profile_mask = stage_mask & ((1u << SNLP_N_STAGES) - 1u);
  return SNLP_OK;
}

int snlp_profile_read(snlp_ctx* c, float* ms, int* count) {
  if (!c || !ms || !count) return SNLP_E_BAD_ARG;
  for (int i = 0; i < SNLP_N_STAGES; ++i) { ms[i] = 0.f; count[i] = 0; }
  for (auto& t : c->timed) {
    SNLP_TRY(hipEventSynchronize(t.stop), "event synchronize");
    float e = 0.f;
    SNLP_TRY(hipEventElapsedTime(&e, t.start, t.stop), "event elapsed");
    ms[t.stage] += e;
    count[t.stage] += 1;
    c->spare.push_back(t);
  }
  c->timed.clear();
  return SNLP_OK;
}

const char* snlp_last_error(const snlp_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_error.c_str(); }

size_t snlp_workspace_bytes(const snlp_ctx* ctx) { return ctx ? ctx->ws_bytes : 0; }

int snlp_bind_workspace(snlp_ctx* c, void* dev, size_t bytes) {
  if (!c) return SNLP_E_BAD_ARG;
  if (!dev) return fail(c, SNLP_E_BAD_ARG, "null workspace");
  if (bytes < c->ws_bytes) return fail(c, SNLP_E_WORKSPACE, "workspace smaller than snlp_workspace_bytes()");
  if ((reinterpret_cast<uintptr_t>(dev) & 255) != 0) return fail(c, SNLP_E_WORKSPACE, "workspace must be 256-byte aligned");
  c->ws = static_cast<char*>(dev);
  c->weights_bound = false;
  c->hc_set = false;
  c->forget_xhat();
  // rotary table for positions P .. P+T-1: angle = pos * base^(-2c/dh), c = 0..dh/2-1, evaluated in fp64
  const Dims& D = c->D;
  const int half = D.dh / 2;
  std::vector<float> cs((size_t)D.T * half), sn((size_t)D.T * half);
  for (int t = 0; t < D.T; ++t)
    for (int ch = 0; ch < half; ++ch) {
      const double theta = std::pow((double)c->cfg.rope_base, -2.0 * ch / D.dh);
      const double ang = (double)(D.P + t) * theta;
      cs[(size_t)t * half + ch] = (float)std::cos(ang);
      sn[(size_t)t * half + ch] = (float)std::sin(ang);
    }
  SNLP_TRY(hipMemcpy(c->ws + c->off_cos, cs.data(), cs.size() * sizeof(float), hipMemcpyHostToDevice), "copy rotary table");
  SNLP_TRY(hipMemcpy(c->ws + c->off_sin, sn.data(), sn.size() * sizeof(float), hipMemcpyHostToDevice), "copy rotary table");
  return SNLP_OK;
}

int snlp_bind_weights(snlp_ctx* c, const void* Wqkv, const void* Wo, const void* Wfc, const void* Wproj, void* stream) {
  if (!c) return SNLP_E_BAD_ARG;
  if (!Wqkv || !Wo || !Wfc || !Wproj) return fail(c, SNLP_E_BAD_ARG, "null weight pointer");
  if (!c->ws) return fail(c, SNLP_E_NOT_BOUND, "bind the workspace before the weights");
  c->forget_exact();
  hipStream_t s = static_cast<hipStream_t>(stream);
  const Dims& D = c->D;
  c->Wqkv = Wqkv; c->Wo = Wo; c->Wfc = Wfc; c->Wproj = Wproj;
  if (c->bf16) {
    if (!gemm_bf16_supported(D.M, 3 * D.d, D.d) || !gemm_bf16_supported(D.M, D.d, D.F))
      return fail(c, SNLP_E_BAD_CONFIG, "SNLP_BF16 requires d and d_mlp to be multiples of 64");
    SNLP_TRY(launch_repack_weights(s, (const bf16_t*)Wqkv, c->at<bf16_t>(c->off_wqkv), D.L, D.d, 3 * D.d, D.M), "repack Wqkv");
    SNLP_TRY(launch_repack_weights(s, (const bf16_t*)Wo, c->at<bf16_t>(c->off_wo), D.L, D.d, D.d, D.M), "repack Wo");
    SNLP_TRY(launch_repack_weights(s, (const bf16_t*)Wfc, c->at<bf16_t>(c->off_wfc), D.L, D.d, D.F, D.M), "repack Wfc");
    SNLP_TRY(launch_repack_weights(s, (const bf16_t*)Wproj, c->at<bf16_t>(c->off_wproj), D.L, D.F, D.d, D.M), "repack Wproj");
  }
  c->weights_bound = true;
  return SNLP_OK;
}

int snlp_bind_kv_prefix(snlp_ctx* c, const void* Kpre, const void* Vpre) {
  if (!c) return SNLP_E_BAD_ARG;
  if (c->D.P > 0 && (!Kpre || !Vpre)) return fail(c, SNLP_E_BAD_ARG, "null KV prefix with P > 0");
  c->forget_exact();
  c->Kpre = c->D.P > 0 ? Kpre : nullptr;
  c->Vpre = c->D.P > 0 ? Vpre : nullptr;
  return SNLP_OK;
}

int snlp_set_hc(snlp_ctx* c, const float* Hres, const float* pre, const float* post) {
  if (!c) return SNLP_E_BAD_ARG;
  if (c->D.n == 1) return fail(c, SNLP_E_BAD_ARG, "snlp_set_hc on a single-stream model");
  if (!Hres || !pre || !post) return fail(c, SNLP_E_BAD_ARG, "null hyper-connection parameter");
  if (!c->ws) return fail(c, SNLP_E_NOT_BOUND, "bind the workspace before snlp_set_hc");
  c->forget_exact();
  c->forget_xhat();
  const size_t L = c->D.L, n = c->D.n;
  SNLP_TRY(hipMemcpy(c->ws + c->off_H, Hres, L * n * n * sizeof(float), hipMemcpyHostToDevice), "copy Hres");
  SNLP_TRY(hipMemcpy(c->ws + c->off_pre, pre, L * n * sizeof(float), hipMemcpyHostToDevice), "copy pre");
  SNLP_TRY(hipMemcpy(c->ws + c->off_post, post, L * n * sizeof(float), hipMemcpyHostToDevice), "copy post");
  c->hc_set = true;
  return SNLP_OK;
}

int snlp_bind_trace(snlp_ctx* c, float* trace) {
  if (!c) return SNLP_E_BAD_ARG;
  if (!trace) return fail(c, SNLP_E_BAD_ARG, "null trace");
  if ((reinterpret_cast<uintptr_t>(trace) & 15) != 0) return fail(c, SNLP_E_BAD_ARG, "trace must be 16-byte aligned");
  c->trace = trace;
  c->forget_exact();
  c->forget_xhat();
  return SNLP_OK;
}

int snlp_set_prefix(snlp_ctx* c, int S) {
  if (!c) return SNLP_E_BAD_ARG;
  if (S < 0 || S >= c->units()) return fail(c, SNLP_E_BAD_ARG, "prefix length must satisfy 0 <= S < L (chunks when fused)");
  c->S = S;
  c->forget_exact();
  c->forget_xhat();
  return SNLP_OK;
}

int snlp_set_skip_converged(snlp_ctx* c, int on) {
  if (!c) return SNLP_E_BAD_ARG;
  c->skip = on != 0;
  return SNLP_OK;
}

int snlp_set_fusion(snlp_ctx* c, int F) {
  if (!c) return SNLP_E_BAD_ARG;
  if (F < 1 || c->D.L % F != 0) return fail(c, SNLP_E_BAD_ARG, "chunk size must divide L");
  if (F > 1 && c->D.n != 1) return fail(c, SNLP_E_BAD_ARG, "fused chunks are built for single-stream models");
  c->Fz = F;
  c->S = 0;
  c->forget_exact();
  c->forget_xhat();
  return SNLP_OK;
}

int snlp_init_trace_ex(snlp_ctx* c, int mode, int init, const float* h0, void* stream) {
  if (!c) return SNLP_E_BAD_ARG;
  if (!h0) return fail(c, SNLP_E_BAD_ARG, "null h0");
  if (!c->trace) return fail(c, SNLP_E_NOT_BOUND, "trace not bound");
  if (init != SNLP_INIT_H0 && init != SNLP_INIT_FWD) return fail(c, SNLP_E_BAD_ARG, "init must be SNLP_INIT_H0 or SNLP_INIT_FWD");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const Dims& D = c->D;
  const int S = c->S;
  int rc;
  c->forget_exact();
  c->forget_xhat();
  if (S > 0 || init == SNLP_INIT_FWD) {
    if ((rc = check_ready(c, true))) return rc;
    if ((rc = check_mode(c, mode))) return rc;
  }
  const size_t slot = (size_t)D.M * D.n * D.d;
  SNLP_TRY(launch_init_trace(s, D, h0, c->trace, 0, 1), "init_trace");
  for (int l = 1; l <= S; ++l) {   // Alg. 2, sequential prefix
    if ((rc = evaluate(c, l, 1, c->trace, s))) return rc;
    if ((rc = correct(c, mode, l, 1, c->trace, c->gbuf(), true, nullptr, false, s))) return rc;
  }
  SNLP_TRY(launch_init_trace(s, D, c->trace + (size_t)S * slot, c->trace, S + 1, c->units() - S), "init_trace");
  if (init == SNLP_INIT_FWD) {     // h_{S+j} = f_{S+j}(h_S): one batched evaluation, each layer stepped from slot S
    if ((rc = evaluate(c, S + 1, c->units() - S, c->trace, s))) return rc;
    if ((rc = correct(c, mode, S + 1, c->units() - S, c->trace, c->gbuf(), true, nullptr, false, s, true))) return rc;
  }
  c->exact_map = c->layer_map(mode);
  c->exact = init == SNLP_INIT_FWD ? S + 1 : S;   // the one-shot forward makes unit S+1 exact
  return SNLP_OK;
}

int snlp_init_trace(snlp_ctx* c, const float* h0, void* stream) {
  if (!c) return SNLP_E_BAD_ARG;
  return snlp_init_trace_ex(c, c->D.n > 1 ? SNLP_HCN : SNLP_IDN, SNLP_INIT_H0, h0, stream);
}

int snlp_iterate(snlp_ctx* c, int mode, int K, float* probe, void* stream) {
  int rc = check_ready(c, true);
  if (rc) return rc;
  if ((rc = check_mode(c, mode))) return rc;
  if (K < 0) return fail(c, SNLP_E_BAD_ARG, "K must be non-negative");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int L = c->units();
  for (int k = 0; k < K; ++k) {
    const int u0 = c->first_unit(mode);
    if ((rc = evaluate_bound(c, u0, L - u0 + 1, s))) return rc;
    if ((rc = correct_bound(c, mode, u0, L - u0 + 1, c->gbuf(), probe ? probe + (size_t)k * 2 * L : nullptr, s))) return rc;
    c->round_done(mode);
  }
  return SNLP_OK;
}

int snlp_sequential_forward(snlp_ctx* c, int mode, const float* h0, float* trace_out, void* stream) {
  int rc = check_ready(c, false);
  if (rc) return rc;
  if ((rc = check_mode(c, mode))) return rc;
  if (!h0 || !trace_out) return fail(c, SNLP_E_BAD_ARG, "null h0 or trace_out");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const Dims& D = c->D;
  if (h0 != trace_out)
    SNLP_TRY(hipMemcpyAsync(trace_out, h0, (size_t)D.M * D.n * D.d * sizeof(float), hipMemcpyDeviceToDevice, s), "copy h0");
  c->forget_xhat();   // the stage buffers are about to hold trace_out's inputs, not the bound trace's
  int valid_from = INT_MAX;
  for (int l = 1; l <= c->units(); ++l) {
    if ((rc = evaluate(c, l, 1, trace_out, s, valid_from))) return rc;
    bool fused = false;
    if ((rc = correct(c, mode, l, 1, trace_out, c->gbuf(), true, nullptr, false, s, false, true, &fused))) return rc;
    valid_from = fused ? l + 1 : INT_MAX;   // the step left layer l + 1's normalised input behind
  }
  return SNLP_OK;
}

int snlp_residual_norm(snlp_ctx* c, int mode, float* out, void* stream) {
  int rc = check_ready(c, true);
  if (rc) return rc;
  if ((rc = check_mode(c, mode))) return rc;
  if (!out) return fail(c, SNLP_E_BAD_ARG, "null output");
  hipStream_t s = static_cast<hipStream_t>(stream);
  if ((rc = evaluate_bound(c, c->S + 1, c->units() - c->S, s))) return rc;
  return correct(c, mode, c->S + 1, c->units() - c->S, c->trace, c->gbuf(), false, out, true, s);
}

int snlp_evaluate_branches(snlp_ctx* c, float* g_out, void* stream) {
  int rc = check_ready(c, true);
  if (rc) return rc;
  if (!g_out) return fail(c, SNLP_E_BAD_ARG, "null output");
  hipStream_t s = static_cast<hipStream_t>(stream);
  if ((rc = evaluate_bound(c, c->S + 1, c->units() - c->S, s))) return rc;
  const Dims& D = c->D;
  SNLP_TRY(hipMemcpyAsync(g_out, c->gbuf(), (size_t)c->units() * D.M * D.d * sizeof(float), hipMemcpyDeviceToDevice, s),
           "copy g");
  return SNLP_OK;
}

int snlp_correction_scan(snlp_ctx* c, int mode, const float* g, float* probe, void* stream) {
  if (!c) return SNLP_E_BAD_ARG;
  if (!c->ws) return fail(c, SNLP_E_NOT_BOUND, "workspace not bound");
  if (!c->trace) return fail(c, SNLP_E_NOT_BOUND, "trace not bound");
  if (c->D.n > 1 && !c->hc_set) return fail(c, SNLP_E_NOT_BOUND, "hyper-connection parameters not set (n_streams > 1)");
  int rc = check_mode(c, mode);
  if (rc) return rc;
  if (!g) return fail(c, SNLP_E_BAD_ARG, "null g");
  c->forget_exact();   // caller-supplied branch outputs: nothing is known about the result
  return correct_bound(c, mode, c->S + 1, c->units() - c->S, g, probe, static_cast<hipStream_t>(stream));
}

namespace {
int correct_diag(snlp_ctx* c, int l0, const float* g, const float* diag, float* probe_out, hipStream_t s) {
  const Dims& D = c->D;
  const int Lc = c->units() - l0 + 1;
  float* partials = probe_out ? c->at<float>(c->off_partials) : nullptr;
  StageTimer tm(c, 8, s);
  SNLP_TRY(launch_scan_diag(s, D, l0, Lc, c->trace, g, diag, partials), "diagonal correction scan");
  if (probe_out) SNLP_TRY(launch_probe_finalize(s, D, Lc, partials, probe_out, false, l0 - 1), "probe finalize");
  return SNLP_OK;
}
}  // namespace

int snlp_correction_scan_diag(snlp_ctx* c, const float* g, const float* diag, float* probe, void* stream) {
  if (!c) return SNLP_E_BAD_ARG;
  if (!c->ws) return fail(c, SNLP_E_NOT_BOUND, "workspace not bound");
  if (!c->trace) return fail(c, SNLP_E_NOT_BOUND, "trace not bound");
  if (c->D.n != 1) return fail(c, SNLP_E_BAD_ARG, "the diagonal surrogate is built for single-stream models");
  if (!g || !diag) return fail(c, SNLP_E_BAD_ARG, "null g or diag");
  c->forget_exact();
  c->forget_xhat();
  return correct_diag(c, c->S + 1, g, diag, probe, static_cast<hipStream_t>(stream));
}

int snlp_iterate_diag(snlp_ctx* c, int K, const float* diag, float* probe, void* stream) {
  int rc = check_ready(c, true);
  if (rc) return rc;
  if (c->D.n != 1) return fail(c, SNLP_E_BAD_ARG, "the diagonal surrogate is built for single-stream models");
  if (K < 0 || !diag) return fail(c, SNLP_E_BAD_ARG, "K must be non-negative and diag non-null");
  hipStream_t s = static_cast<hipStream_t>(stream);
  for (int k = 0; k < K; ++k) {
    const int u0 = c->first_unit(SNLP_IDN);
    if ((rc = evaluate_bound(c, u0, c->units() - u0 + 1, s))) return rc;
    c->forget_xhat();   // the diagonal correction does not prepare the next round's inputs
    if ((rc = correct_diag(c, u0, c->gbuf(), diag, probe ? probe + (size_t)k * 2 * c->units() : nullptr, s))) return rc;
    c->round_done(SNLP_IDN);
  }
  return SNLP_OK;
}

int snlp_stage_buffer(snlp_ctx* c, const char* name, void** dev, size_t* bytes) {
  if (!c || !name || !dev || !bytes) return SNLP_E_BAD_ARG;
  if (!c->ws) return fail(c, SNLP_E_NOT_BOUND, "workspace not bound");
  const Dims& D = c->D;
  const size_t LM = (size_t)D.L * D.M;
  struct { const char* n; size_t off, sz; } tab[] = {
      {"xhat", c->off_xhat, LM * D.d * c->esz},   {"qkv", c->off_qkv, LM * 3 * D.d * c->esz},
      {"attn", c->off_attn, LM * D.d * c->esz},   {"a", c->off_a, LM * D.d * sizeof(float)},
      {"xhat2", c->off_xhat2, LM * D.d * c->esz}, {"hmid", c->off_hmid, LM * D.F * c->esz},
      {"g", c->off_g, LM * D.d * sizeof(float)},  {"u", c->off_u, D.n > 1 ? LM * D.d * sizeof(float) : 0},
  };
  for (auto& t : tab)
    if (std::strcmp(t.n, name) == 0) {
      *dev = c->ws + t.off;
      *bytes = t.sz;
      return SNLP_OK;
    }
  return fail(c, SNLP_E_BAD_ARG, std::string("unknown stage buffer: ") + name);
}

}  // extern "C"

// ------------------------------------------------------------------------------------------------
// The correction scan for callers that cannot allocate: the probe's per-workgroup partial sums, which the
// context-based calls keep in the caller's workspace, live in a fixed array in device memory that every GPU
// the library runs on holds until the process ends.
namespace {

constexpr size_t kStaticScratchFloats = SNLP_STATIC_SCRATCH_BYTES / sizeof(float);
static __device__ __align__(256) __attribute__((used)) float snlp_static_scratch[kStaticScratchFloats];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float* g_scratch_ptr[kMaxDevices] = {};   // device address of the array on each GPU, resolved on first use

// Device address of this GPU's copy of the array (each GPU has its own, at its own address).  In host code the
// array's name is only a handle for the runtime, never an address a kernel can use.
int static_scratch(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(nullptr, e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(nullptr, SNLP_E_BAD_CONFIG, "device ordinal beyond the static scratch table");
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(snlp_static_scratch));
    if (e != hipSuccess || !p) return hip_fail(nullptr, e, "hipGetSymbolAddress(static scratch)");
    g_scratch_ptr[dev] = static_cast<float*>(p);
  }
  *out = g_scratch_ptr[dev];
  return SNLP_OK;
}

}  // namespace

extern "C" {

int snlp_correction_scan_static(int mode, int L, int M, int n_streams, int d, float* trace, const float* g,
                                const float* Hres, const float* post, float* probe, void* stream) {
  snlp_ctx* c = nullptr;   // errors are reported through snlp_last_error(NULL)
  if (mode != SNLP_IDN && mode != SNLP_HCN) return fail(c, SNLP_E_BAD_ARG, "mode must be SNLP_IDN or SNLP_HCN");
  if (L < 1 || L > 256) return fail(c, SNLP_E_BAD_CONFIG, "L must be in 1..256");
  if (M < 1 || d < 4 || d % 4 != 0 || d > 4096) return fail(c, SNLP_E_BAD_CONFIG, "M must be positive, d a multiple of 4 and at most 4096");
  if (!(n_streams == 1 || n_streams == 2 || n_streams == 3 || n_streams == 4 || n_streams == 8))
    return fail(c, SNLP_E_BAD_CONFIG, "n_streams must be 1, 2, 3, 4 or 8");
  if ((long long)M * (d / 4) >= (1ll << 31)) return fail(c, SNLP_E_BAD_CONFIG, "M * d too large");
  if (mode == SNLP_HCN && n_streams == 1) return fail(c, SNLP_E_BAD_ARG, "SNLP_HCN needs n_streams > 1");
  if (!trace || !g) return fail(c, SNLP_E_BAD_ARG, "null trace or g");
  if ((reinterpret_cast<uintptr_t>(trace) & 15) != 0 || (reinterpret_cast<uintptr_t>(g) & 15) != 0)
    return fail(c, SNLP_E_BAD_ARG, "trace and g must be 16-byte aligned");
  if (n_streams > 1 && (!post || (mode == SNLP_HCN && !Hres)))
    return fail(c, SNLP_E_BAD_ARG, "n_streams > 1 needs post (and Hres for SNLP_HCN)");
  Dims D{};
  D.L = L; D.d = d; D.n = n_streams; D.M = M; D.B = 1; D.T = M; D.H = 1; D.dh = d; D.F = 0; D.P = 0; D.eps = 0.f;
  float* partials = nullptr;
  if (probe) {
    const size_t need = (size_t)scan_partial_blocks(D) * 2 * (size_t)L;
    if (need > kStaticScratchFloats)
      return fail(c, SNLP_E_WORKSPACE, "probe partials of this shape exceed the static scratch (blocks * 2 * L floats > 2^20): "
                                       "pass probe = NULL or use snlp_correction_scan with a workspace");
    const int rc = static_scratch(&partials);
    if (rc) return rc;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  // every entry of the partials that the final reduction reads is written by the scan of this call, so nothing has to
  // start at zero
  SNLP_TRY(launch_scan(s, D, mode, 1, L, trace, g, n_streams > 1 ? Hres : nullptr, n_streams > 1 ? post : nullptr, true,
                       partials, false), "correction scan (static scratch)");
  if (probe) SNLP_TRY(launch_probe_finalize(s, D, L, partials, probe, false, 0), "probe finalize (static scratch)");
  return SNLP_OK;
}

}  // extern "C"

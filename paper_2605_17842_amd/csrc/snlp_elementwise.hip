// HBM-bound stages of the SNLP iteration for gfx950: stream pre-mix + RMSNorm, mid-residual RMSNorm,
// rotary embedding + per-head QK RMSNorm, the h0 initialisation (Alg. 2), and the structured Newton
// correction along the layer axis (Eq. (5): IDN prefix sum / HCN linear recurrence) fused with the
// residual-norm probe (Eq. (2)).  Notation: the paper's f_l is the full layer, g_l = a_l + m_l its branch.
#include "snlp_kernels.hpp"

namespace snlp {

namespace {

constexpr int kThreads = 256;
constexpr int kWave = 64;

__device__ __forceinline__ float bf16_bits_to_float(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ bf16_t float_to_bf16_bits(float f) {
  __bf16 h = static_cast<__bf16>(f);   // round to nearest even
  return __builtin_bit_cast(bf16_t, h);
}

template <typename T> __device__ __forceinline__ float load_as_float(const T* p);
template <> __device__ __forceinline__ float load_as_float<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_as_float<bf16_t>(const bf16_t* p) { return bf16_bits_to_float(*p); }
template <typename T> __device__ __forceinline__ void store_from_float(T* p, float v);
template <> __device__ __forceinline__ void store_from_float<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_from_float<bf16_t>(bf16_t* p, float v) { *p = float_to_bf16_bits(v); }

__device__ __forceinline__ void store4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
__device__ __forceinline__ void store4(bf16_t* p, float4 v) {
  ushort4 o;
  o.x = float_to_bf16_bits(v.x); o.y = float_to_bf16_bits(v.y);
  o.z = float_to_bf16_bits(v.z); o.w = float_to_bf16_bits(v.w);
  *reinterpret_cast<ushort4*>(p) = o;
}

// 16-byte load.  STREAM: non-temporal, for operands far larger than the caches that the kernel reads once (it keeps
// them from displacing what other kernels reuse, and measured 10-15 % faster at prefill sizes); operands of
// decode-sized batches were just written by the previous kernel and are better read through the caches.
template <bool STREAM>
__device__ __forceinline__ float4 load4_sel(const float* p) {
  if (STREAM) {
    typedef float v4f __attribute__((ext_vector_type(4)));
    const v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
    return make_float4(t.x, t.y, t.z, t.w);
  }
  return *reinterpret_cast<const float4*>(p);
}
template <bool STREAM>
__device__ __forceinline__ void store4_sel(float* p, const float4 v) {
  if (STREAM) {
    typedef float v4f __attribute__((ext_vector_type(4)));
    v4f t; t.x = v.x; t.y = v.y; t.z = v.z; t.w = v.w;
    __builtin_nontemporal_store(t, reinterpret_cast<v4f*>(p));
  } else {
    *reinterpret_cast<float4*>(p) = v;
  }
}
// Operands of one launch above this many bytes are streamed.
constexpr size_t kStreamBytes = (size_t)128 << 20;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// Wave sum with data-parallel-primitive moves (VALU, no LDS round trips): pairs, quads, then rotations inside each
// row of 16 lanes, then the row totals are passed down the rows.  The total is valid in lane 63 only.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_move(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xF, false));
}
__device__ __forceinline__ float wave_sum_lane63(float v) {
  v = v + dpp_move<0xB1, 0xF>(v);    // quad_perm [1,0,3,2]
  v = v + dpp_move<0x4E, 0xF>(v);    // quad_perm [2,3,0,1]
  v = v + dpp_move<0x124, 0xF>(v);   // row_ror 4
  v = v + dpp_move<0x128, 0xF>(v);   // row_ror 8: every lane holds its row's sum
  v = v + dpp_move<0x142, 0xA>(v);   // row_bcast 15 into rows 1 and 3
  v = v + dpp_move<0x143, 0xC>(v);   // row_bcast 31 into rows 2 and 3
  return v;
}

// Sum over the threads of a block (a whole number of waves, at most 16), same value returned to every thread;
// fixed order.
constexpr int kMaxWaves = 16;
__device__ __forceinline__ float block_sum(float v, float* sh /*[kMaxWaves]*/) {
  v = wave_sum(v);
  const int w = threadIdx.x / kWave;
  const int nw = blockDim.x / kWave;
  __syncthreads();
  if ((threadIdx.x & (kWave - 1)) == 0) sh[w] = v;
  __syncthreads();
  float t = sh[0];
  for (int i = 1; i < nw; ++i) t = t + sh[i];
  return t;
}

// The same sum (same order, same bits) with one barrier: for callers that alternate between two scratch arrays, so that a
// thread still reading the previous total cannot meet the next call's writes (the barrier of the call in between
// separates them).
__device__ __forceinline__ float block_sum_alternating(float v, float* sh /*[kMaxWaves], other array than last call*/) {
  v = wave_sum(v);
  const int w = threadIdx.x / kWave;
  const int nw = blockDim.x / kWave;
  if ((threadIdx.x & (kWave - 1)) == 0) sh[w] = v;
  __syncthreads();
  float t = sh[0];
  for (int i = 1; i < nw; ++i) t = t + sh[i];
  return t;
}

// Threads per block of the row kernels: one float4 per thread when the row allows it (rows of d / 4 float4).
static inline int row_block_threads(int d) {
  const int nv = d / 4;
  const int bt = ((nv + kWave - 1) / kWave) * kWave;
  return bt < kWave ? kWave : (bt > 1024 ? 1024 : bt);
}

constexpr int kMaxVec = 4;   // float4 per thread per row (blocks of 64..1024 threads cover d / 4 in at most 4 passes)

// ------------------------------------------------------------------------------------------------
// Branch input of a layer from the n streams of its input state: u = sum_j pre[j] X[j] (H^pre of the HC sublayer),
// pre[0] * X[0] first, then one fused multiply-add per further stream.  Written once: the stand-alone norm kernel and
// the correction kernel that also prepares the next round's inputs must produce the same bits.
template <int N>
__device__ __forceinline__ float4 premix4(const float4 (&x)[N], const float* __restrict__ pre) {
  float4 u = x[0];
  if (N > 1) {
    const float w0 = pre[0];
    u.x *= w0; u.y *= w0; u.z *= w0; u.w *= w0;
#pragma unroll
    for (int j = 1; j < N; ++j) {
      const float w = pre[j];
      u.x = fmaf(w, x[j].x, u.x); u.y = fmaf(w, x[j].y, u.y); u.z = fmaf(w, x[j].z, u.z); u.w = fmaf(w, x[j].w, u.w);
    }
  }
  return u;
}
// (x^2 + y^2) + (z^2 + w^2), every operation rounded once
__device__ __forceinline__ float sumsq4(const float4 u) {
#pragma clang fp contract(off)
  return (u.x * u.x + u.y * u.y) + (u.z * u.z + u.w * u.w);
}
__device__ __forceinline__ float inv_rms(float ss, int d, float eps) { return 1.0f / sqrtf(ss / (float)d + eps); }

// x = rmsnorm(u), u = sum_j pre[j] X[j]  (n = 1: u = X)
template <int N, typename OutT, bool STREAM>
__global__ __launch_bounds__(1024) void k_premix_rmsnorm(const float* __restrict__ trace,
                                                              const float* __restrict__ pre,
                                                              float* __restrict__ ubuf, OutT* __restrict__ xhat,
                                                              int l0, int M, int d, float eps) {
  __shared__ float sh[kMaxWaves];
  const int row = blockIdx.x;
  const int l = l0 + blockIdx.y;   // 1-based layer; its input is slot l-1
  const float* in = trace + ((size_t)(l - 1) * M + row) * (size_t)N * d;
  const size_t orow = ((size_t)(l - 1) * M + row) * (size_t)d;
  const int nv = d >> 2;
  const int c4 = threadIdx.x;      // one float4 per thread: the block covers the row (d <= 4096)
  float4 u = make_float4(0.f, 0.f, 0.f, 0.f);
  float ss = 0.f;
  if (c4 < nv) {
    float4 x[N];
#pragma unroll
    for (int j = 0; j < N; ++j) x[j] = load4_sel<STREAM>(in + (size_t)j * d + (size_t)c4 * 4);
    u = premix4<N>(x, pre + (size_t)(l - 1) * N);
    if (N > 1) store4_sel<STREAM>(ubuf + orow + (size_t)c4 * 4, u);
    ss = sumsq4(u);
  }
  ss = block_sum(ss, sh);
  const float r = inv_rms(ss, d, eps);
  if (c4 < nv) {
    u.x *= r; u.y *= r; u.z *= r; u.w *= r;
    store4(xhat + orow + (size_t)c4 * 4, u);
  }
}

// x' = rmsnorm(u + a)
template <typename OutT, bool STREAM>
__global__ __launch_bounds__(1024) void k_mid_rmsnorm(const float* __restrict__ usrc, size_t u_layer_stride,
                                                           size_t u_row_stride, const float* __restrict__ a,
                                                           OutT* __restrict__ xhat2, int l0, int M, int d, float eps) {
  __shared__ float sh[kMaxWaves];
  const int row = blockIdx.x;
  const int l = l0 + blockIdx.y;
  const float* up = usrc + (size_t)(l - 1) * u_layer_stride + (size_t)row * u_row_stride;
  const size_t orow = ((size_t)(l - 1) * M + row) * (size_t)d;
  const int nv = d >> 2;
  float4 v[kMaxVec];
  float ss = 0.f;
#pragma unroll
  for (int it = 0; it < kMaxVec; ++it) {
    const int c4 = threadIdx.x + it * (int)blockDim.x;
    if (c4 < nv) {
      float4 u = load4_sel<STREAM>(up + (size_t)c4 * 4);
      const float4 y = load4_sel<STREAM>(a + orow + (size_t)c4 * 4);
      u.x += y.x; u.y += y.y; u.z += y.z; u.w += y.w;
      v[it] = u;
      ss += (u.x * u.x + u.y * u.y) + (u.z * u.z + u.w * u.w);
    }
  }
  ss = block_sum(ss, sh);
  const float r = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
  for (int it = 0; it < kMaxVec; ++it) {
    const int c4 = threadIdx.x + it * (int)blockDim.x;
    if (c4 < nv) {
      float4 u = v[it];
      u.x *= r; u.y *= r; u.z *= r; u.w *= r;
      store4(xhat2 + orow + (size_t)c4 * 4, u);
    }
  }
}

// Fused chunk of F layers reading the same input h (Appendix "Fused Cross-Layer Coupling"): a_C = sum of the
// chunk's attention updates (ascending layer order, fp32), u_C = h + a_C, x' = rmsnorm(u_C).  a_C is kept for
// the chunk's branch output g_C = a_C + m_C.
template <typename OutT>
__global__ __launch_bounds__(1024) void k_chunk_mid_rmsnorm(const float* __restrict__ trace,
                                                                 const float* __restrict__ a, float* __restrict__ aC,
                                                                 OutT* __restrict__ xhat2, int c0, int F, int M, int d,
                                                                 float eps) {
  __shared__ float sh[kMaxWaves];
  const int row = blockIdx.x;
  const int c = c0 + blockIdx.y;   // 1-based chunk; its input is slot c-1
  const size_t crow = ((size_t)(c - 1) * M + row) * (size_t)d;
  const int nv = d >> 2;
  float4 v[kMaxVec];
  float ss = 0.f;
#pragma unroll
  for (int it = 0; it < kMaxVec; ++it) {
    const int c4 = threadIdx.x + it * (int)blockDim.x;
    if (c4 < nv) {
      float4 acc = reinterpret_cast<const float4*>(a + (((size_t)(c - 1) * F) * M + row) * (size_t)d)[c4];
      for (int j = 1; j < F; ++j) {
        const float4 y = reinterpret_cast<const float4*>(a + (((size_t)(c - 1) * F + j) * M + row) * (size_t)d)[c4];
        acc.x += y.x; acc.y += y.y; acc.z += y.z; acc.w += y.w;
      }
      reinterpret_cast<float4*>(aC + crow)[c4] = acc;
      float4 u = reinterpret_cast<const float4*>(trace + crow)[c4];
      u.x += acc.x; u.y += acc.y; u.z += acc.z; u.w += acc.w;
      v[it] = u;
      ss += (u.x * u.x + u.y * u.y) + (u.z * u.z + u.w * u.w);
    }
  }
  ss = block_sum(ss, sh);
  const float r = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
  for (int it = 0; it < kMaxVec; ++it) {
    const int c4 = threadIdx.x + it * (int)blockDim.x;
    if (c4 < nv) {
      float4 u = v[it];
      u.x *= r; u.y *= r; u.z *= r; u.w *= r;
      store4(xhat2 + crow + (size_t)c4 * 4, u);
    }
  }
}

// g_C = a_C + (m_1 + m_2 + ... + m_F) for the chunks c0..c0+Nc-1 (ascending layer order, fp32).
__global__ __launch_bounds__(kThreads) void k_chunk_sum(const float4* __restrict__ aC, const float4* __restrict__ m,
                                                         float4* __restrict__ gC, int c0, int F, size_t slab_vec) {
  const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= slab_vec) return;
  const int c = c0 + blockIdx.y;
  float4 acc = m[((size_t)(c - 1) * F) * slab_vec + i];
  for (int j = 1; j < F; ++j) {
    const float4 y = m[((size_t)(c - 1) * F + j) * slab_vec + i];
    acc.x += y.x; acc.y += y.y; acc.z += y.z; acc.w += y.w;
  }
  const float4 x = aC[(size_t)(c - 1) * slab_vec + i];
  acc.x = x.x + acc.x; acc.y = x.y + acc.y; acc.z = x.z + acc.z; acc.w = x.w + acc.w;
  gC[(size_t)(c - 1) * slab_vec + i] = acc;
}

// Rotary embedding at position P + t on channel pairs (c, c + dh/2), then rmsnorm over the head, for the
// q and k thirds of one token row; one wave per (third, head) item.  Table rows are indexed by t.
template <typename T>
__global__ __launch_bounds__(kThreads) void k_rope_qknorm(T* __restrict__ qkv, const float* __restrict__ cos_tab,
                                                           const float* __restrict__ sin_tab, int l0, int M, int Tn,
                                                           int d, int H, int dh, float eps) {
  const int row = blockIdx.x;
  const int l = l0 + blockIdx.y;
  const int t = row % Tn;
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int half = dh >> 1;
  T* base = qkv + ((size_t)(l - 1) * M + row) * (size_t)(3 * d);
  for (int item = wave; item < 2 * H; item += kThreads / kWave) {
    T* p = base + (size_t)(item / H) * d + (size_t)(item % H) * dh;
    float y1[2], y2[2];
    float ss = 0.f;
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      const int c = lane + it * kWave;
      y1[it] = 0.f; y2[it] = 0.f;
      if (c < half) {
        const float x1 = load_as_float(p + c), x2 = load_as_float(p + c + half);
        const float cs = cos_tab[(size_t)t * half + c], sn = sin_tab[(size_t)t * half + c];
        y1[it] = x1 * cs - x2 * sn;
        y2[it] = x2 * cs + x1 * sn;
        ss += y1[it] * y1[it] + y2[it] * y2[it];
      }
    }
    ss = wave_sum(ss);
    const float r = 1.0f / sqrtf(ss / (float)dh + eps);
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      const int c = lane + it * kWave;
      if (c < half) {
        store_from_float(p + c, y1[it] * r);
        store_from_float(p + c + half, y2[it] * r);
      }
    }
  }
}

// bf16, head_dim 128: eight lanes per (third, head) item, each lane owning channels 8j..8j+7 and their rotation
// partners 64 + 8j.. (16-byte loads and stores instead of 2-byte ones); the squared norm is summed over the lane's
// eight pairs in order, then over the eight lanes by a butterfly.
__global__ __launch_bounds__(kThreads) void k_rope_qknorm_bf16_dh128(bf16_t* __restrict__ qkv,
                                                                      const float* __restrict__ cos_tab,
                                                                      const float* __restrict__ sin_tab, int l0, int M,
                                                                      int Tn, int d, int H, size_t total, float eps) {
  const size_t idx = (size_t)blockIdx.x * kThreads + threadIdx.x;
  const bool active = idx < total;
  const size_t id = active ? idx : total - 1;      // inactive lanes shadow the last item (they take part in the butterfly)
  const int j = (int)(id & 7);
  const size_t ig = id >> 3;
  const int item = (int)(ig % (size_t)(2 * H));
  const size_t rowl = ig / (size_t)(2 * H);
  const int row = (int)(rowl % (size_t)M);
  const int l = l0 + (int)(rowl / (size_t)M);
  const int t = row % Tn;
  bf16_t* p = qkv + ((size_t)(l - 1) * M + row) * (size_t)(3 * d) + (size_t)(item / H) * d + (size_t)(item % H) * 128 + j * 8;
  const uint4 lo = *reinterpret_cast<const uint4*>(p);
  const uint4 hi = *reinterpret_cast<const uint4*>(p + 64);
  const float4 c0 = *reinterpret_cast<const float4*>(cos_tab + (size_t)t * 64 + j * 8);
  const float4 c1 = *reinterpret_cast<const float4*>(cos_tab + (size_t)t * 64 + j * 8 + 4);
  const float4 s0 = *reinterpret_cast<const float4*>(sin_tab + (size_t)t * 64 + j * 8);
  const float4 s1 = *reinterpret_cast<const float4*>(sin_tab + (size_t)t * 64 + j * 8 + 4);
  const uint32_t lw[4] = {lo.x, lo.y, lo.z, lo.w}, hw[4] = {hi.x, hi.y, hi.z, hi.w};
  const float cs[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
  const float sn[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
  float y1[8], y2[8];
  float ss = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float x1 = __uint_as_float((e & 1) ? (lw[e >> 1] & 0xffff0000u) : (lw[e >> 1] << 16));
    const float x2 = __uint_as_float((e & 1) ? (hw[e >> 1] & 0xffff0000u) : (hw[e >> 1] << 16));
    y1[e] = x1 * cs[e] - x2 * sn[e];
    y2[e] = x2 * cs[e] + x1 * sn[e];
    ss += y1[e] * y1[e] + y2[e] * y2[e];
  }
  ss += __shfl_xor(ss, 1, kWave);
  ss += __shfl_xor(ss, 2, kWave);
  ss += __shfl_xor(ss, 4, kWave);
  const float r = 1.0f / sqrtf(ss / 128.0f + eps);
  if (!active) return;
  uint32_t ow[4], oh[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    ow[e] = (uint32_t)float_to_bf16_bits(y1[2 * e] * r) | ((uint32_t)float_to_bf16_bits(y1[2 * e + 1] * r) << 16);
    oh[e] = (uint32_t)float_to_bf16_bits(y2[2 * e] * r) | ((uint32_t)float_to_bf16_bits(y2[2 * e + 1] * r) << 16);
  }
  *reinterpret_cast<uint4*>(p) = make_uint4(ow[0], ow[1], ow[2], ow[3]);
  *reinterpret_cast<uint4*>(p + 64) = make_uint4(oh[0], oh[1], oh[2], oh[3]);
}

// Alg. 2 initialisation: every slot of the trace starts as the input state.
__global__ __launch_bounds__(kThreads) void k_init_trace(const float4* __restrict__ src, float4* __restrict__ trace,
                                                          size_t nvec, int first, int count) {
  const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= nvec) return;
  const float4 v = src[i];
  for (int l = first; l < first + count; ++l) trace[(size_t)l * nvec + i] = v;
}

// ------------------------------------------------------------------------------------------------
// The structured correction (Eq. (5)) in prefix / affine form, strict fp32 in a fixed order.
// Every floating-point operation below is rounded once: contraction into fused multiply-add is off.
template <int N>
__device__ __forceinline__ void layer_step(const float4 (&xp)[N], const float4 g, const float* __restrict__ Hl,
                                           const float* __restrict__ pl, int mode, float4 (&out)[N]) {
#pragma clang fp contract(off)
  if (N == 1) {
    out[0].x = xp[0].x + g.x; out[0].y = xp[0].y + g.y; out[0].z = xp[0].z + g.z; out[0].w = xp[0].w + g.w;
    return;
  }
#pragma unroll
  for (int i = 0; i < N; ++i) {
    const float p = pl[i];
    float4 acc;
    acc.x = p * g.x; acc.y = p * g.y; acc.z = p * g.z; acc.w = p * g.w;
    if (mode == 0) {   // IDN on an n-stream model: the H = I block
      acc.x = xp[i].x + acc.x; acc.y = xp[i].y + acc.y; acc.z = xp[i].z + acc.z; acc.w = xp[i].w + acc.w;
    } else {
#pragma unroll
      for (int j = 0; j < N; ++j) {
        const float h = Hl[i * N + j];
        float4 t;
        t.x = h * xp[j].x; t.y = h * xp[j].y; t.z = h * xp[j].z; t.w = h * xp[j].w;
        acc.x = acc.x + t.x; acc.y = acc.y + t.y; acc.z = acc.z + t.z; acc.w = acc.w + t.w;
      }
    }
    out[i] = acc;
  }
}

__device__ __forceinline__ float sqdiff4(const float4 a, const float4 b) {
  const float x = a.x - b.x, y = a.y - b.y, z = a.z - b.z, w = a.w - b.w;
  return (x * x + y * y) + (z * z + w * w);
}

// One thread owns 4 consecutive channels of one token row (all N streams) and walks the layers
// l0..l0+Lc-1 left to right.  Loads of U layers are issued together before their dependent stores.
// PROBE: r_l^2 = ||X_l(old) - f_l(X_{l-1}(old))||^2 and ||X_l(new) - X_l(old)||^2 per layer, reduced over the
// wave by shuffles, over the block in LDS, and written as partials[block][2][Lc] (no atomics).
template <int N, int U, bool PROBE, bool WRITE, int BT, bool STREAM>
__global__ __launch_bounds__(BT) void k_scan(float* trace, const float* __restrict__ g,
                                                    const float* __restrict__ Hres, const float* __restrict__ post,
                                                    int mode, int l0, int Lc, int M, int d,
                                                    float* __restrict__ partials, int independent) {
  extern __shared__ float sh[];   // [BT / 64][2][Lc] when PROBE
  const int nv = d >> 2;
  const unsigned total = (unsigned)M * (unsigned)nv;   // < 2^31, checked by the host
  const unsigned id = blockIdx.x * BT + threadIdx.x;
  const bool active = id < total;
  const size_t row = active ? id / (unsigned)nv : 0;
  const int c4 = active ? (int)(id % (unsigned)nv) : 0;
  const size_t slot = (size_t)M * N * d;              // elements per trace slot
  const size_t toff = row * (size_t)N * d + (size_t)c4 * 4;
  const size_t goff = row * (size_t)d + (size_t)c4 * 4;
  const size_t gslot = (size_t)M * d;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;

  float4 acc[N];        // new state of the previous layer
  float4 prev_old[N];   // old state of the previous layer (for the residual)
#pragma unroll
  for (int j = 0; j < N; ++j) {
    acc[j] = active ? *reinterpret_cast<const float4*>(trace + (size_t)(l0 - 1) * slot + toff + (size_t)j * d)
                    : make_float4(0.f, 0.f, 0.f, 0.f);
    prev_old[j] = acc[j];
  }

  const int lend = l0 + Lc;
  for (int lb = l0; lb < lend; lb += U) {
    float4 gv[U];
    float4 old[U][N];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int l = lb + u;
      const bool ok = active && l < lend;
      gv[u] = ok ? load4_sel<STREAM>(g + (size_t)(l - 1) * gslot + goff) : make_float4(0.f, 0.f, 0.f, 0.f);
      if (PROBE || !WRITE) {
#pragma unroll
        for (int j = 0; j < N; ++j)
          old[u][j] = ok ? load4_sel<STREAM>(trace + (size_t)l * slot + toff + (size_t)j * d) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int l = lb + u;
      if (l < lend) {   // uniform over the block
        const float* Hl = Hres ? Hres + (size_t)(l - 1) * N * N : nullptr;
        const float* pl = post ? post + (size_t)(l - 1) * N : nullptr;
        float4 nw[N];
        layer_step<N>(acc, gv[u], Hl, pl, mode, nw);
        if (PROBE) {
          float4 f[N];
          layer_step<N>(prev_old, gv[u], Hl, pl, mode, f);
          float rs = 0.f, ds = 0.f;
#pragma unroll
          for (int j = 0; j < N; ++j) {
            rs += sqdiff4(old[u][j], f[j]);
            ds += sqdiff4(nw[j], old[u][j]);
          }
          if (!active) { rs = 0.f; ds = 0.f; }
          rs = wave_sum_lane63(rs);
          ds = wave_sum_lane63(ds);
          if (lane == kWave - 1) {
            sh[(wave * 2 + 0) * Lc + (l - l0)] = rs;
            sh[(wave * 2 + 1) * Lc + (l - l0)] = ds;
          }
        }
        if (WRITE) {
          if (active) {
#pragma unroll
            for (int j = 0; j < N; ++j)
              *reinterpret_cast<float4*>(trace + (size_t)l * slot + toff + (size_t)j * d) = nw[j];
          }
          if (!independent) {   // independent: every layer steps from slot l0-1 (one-shot forward)
#pragma unroll
            for (int j = 0; j < N; ++j) acc[j] = nw[j];
          }
        } else {
          // read-only probe of the current trace: the "new" state is the stored one
#pragma unroll
          for (int j = 0; j < N; ++j) acc[j] = old[u][j];
        }
        if (PROBE || !WRITE) {
#pragma unroll
          for (int j = 0; j < N; ++j) prev_old[j] = old[u][j];
        }
      }
    }
  }
  if (PROBE) {
    __syncthreads();
    for (int i = threadIdx.x; i < 2 * Lc; i += BT) {
      float s = sh[i];
#pragma unroll
      for (int w = 1; w < BT / kWave; ++w) s = s + sh[w * 2 * Lc + i];
      partials[(size_t)blockIdx.x * 2 * Lc + i] = s;
    }
  }
}

// The same correction with one workgroup per token row (thread c owns channels 4c .. 4c+3 of all N streams), which
// also prepares the next round's evaluation: right after layer l's new state is known it forms the branch input of
// layer l + 1 from it, u = sum_j pre_{l+1}[j] X_l[j], and its normalised form -- what k_premix_rmsnorm would
// compute from the stored trace in a pass of its own, bit for bit (same premix4 / sumsq4 / block_sum / inv_rms, same
// block shape).  Costs one workgroup barrier per layer; saves re-reading the new trace.  For batches large enough
// that a row per workgroup fills the chip.  Ltot: number of layers of the model (no layer follows the last).
template <int N, int U, bool PROBE, typename OutT, bool STREAM>
__global__ __launch_bounds__(1024) void k_scan_norm(float* trace, const float* __restrict__ g,
                                                         const float* __restrict__ Hres, const float* __restrict__ post,
                                                         const float* __restrict__ pre, float* __restrict__ ubuf,
                                                         OutT* __restrict__ xhat, int mode, int l0, int Lc, int Ltot, int M,
                                                         int d, float eps, float* __restrict__ partials) {
  extern __shared__ float sh[];   // [2][kMaxWaves] for the row sums (alternating by layer), then [waves][2][Lc] when PROBE
  float* shp = sh + 2 * kMaxWaves;
  const int nv = d >> 2;
  const int row = blockIdx.x, c4 = threadIdx.x;
  const bool active = c4 < nv;
  const size_t slot = (size_t)M * N * d;
  const size_t toff = (size_t)row * N * d + (size_t)(active ? c4 : 0) * 4;
  const size_t goff = (size_t)row * d + (size_t)(active ? c4 : 0) * 4;
  const size_t gslot = (size_t)M * d;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);

  float4 acc[N], prev_old[N];
#pragma unroll
  for (int j = 0; j < N; ++j) {
    acc[j] = active ? *reinterpret_cast<const float4*>(trace + (size_t)(l0 - 1) * slot + toff + (size_t)j * d) : zero;
    prev_old[j] = acc[j];
  }
  const int lend = l0 + Lc;
  for (int lb = l0; lb < lend; lb += U) {
    float4 gv[U];
    float4 old[U][N];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int l = lb + u;
      const bool ok = active && l < lend;
      gv[u] = ok ? load4_sel<STREAM>(g + (size_t)(l - 1) * gslot + goff) : zero;
      if (PROBE) {
#pragma unroll
        for (int j = 0; j < N; ++j) old[u][j] = ok ? load4_sel<STREAM>(trace + (size_t)l * slot + toff + (size_t)j * d) : zero;
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int l = lb + u;
      if (l < lend) {   // uniform over the block
        const float* Hl = Hres ? Hres + (size_t)(l - 1) * N * N : nullptr;
        const float* pl = post ? post + (size_t)(l - 1) * N : nullptr;
        float4 nw[N];
        layer_step<N>(acc, gv[u], Hl, pl, mode, nw);
        if (PROBE) {
          float4 f[N];
          layer_step<N>(prev_old, gv[u], Hl, pl, mode, f);
          float rs = 0.f, ds = 0.f;
#pragma unroll
          for (int j = 0; j < N; ++j) {
            rs += sqdiff4(old[u][j], f[j]);
            ds += sqdiff4(nw[j], old[u][j]);
          }
          if (!active) { rs = 0.f; ds = 0.f; }
          rs = wave_sum_lane63(rs);
          ds = wave_sum_lane63(ds);
          if (lane == kWave - 1) {
            shp[(wave * 2 + 0) * Lc + (l - l0)] = rs;
            shp[(wave * 2 + 1) * Lc + (l - l0)] = ds;
          }
#pragma unroll
          for (int j = 0; j < N; ++j) prev_old[j] = old[u][j];
        }
        if (active) {
#pragma unroll
          for (int j = 0; j < N; ++j) *reinterpret_cast<float4*>(trace + (size_t)l * slot + toff + (size_t)j * d) = nw[j];
        }
        if (l < Ltot) {   // layer l + 1 reads this state next round: its input and normalised input (0-based index l)
          float4 un = zero;
          float ss = 0.f;
          if (active) {
            un = premix4<N>(nw, pre + (size_t)l * N);
            if (N > 1) store4_sel<STREAM>(ubuf + (size_t)l * gslot + goff, un);
            ss = sumsq4(un);
          }
          ss = block_sum_alternating(ss, sh + (l & 1) * kMaxWaves);
          const float r = inv_rms(ss, d, eps);
          if (active) {
            un.x *= r; un.y *= r; un.z *= r; un.w *= r;
            store4(xhat + (size_t)l * gslot + goff, un);
          }
        }
#pragma unroll
        for (int j = 0; j < N; ++j) acc[j] = nw[j];
      }
    }
  }
  if (PROBE) {
    __syncthreads();
    const int nw_ = blockDim.x / kWave;
    for (int i = threadIdx.x; i < 2 * Lc; i += blockDim.x) {
      float sm = shp[i];
      for (int w = 1; w < nw_; ++w) sm = sm + shp[w * 2 * Lc + i];
      partials[(size_t)blockIdx.x * 2 * Lc + i] = sm;
    }
  }
}

// Diagonal surrogate A_l = diag(a_l) with caller-supplied a (Methods, "Diagonal Newton"; Alg. 3): for single-stream
// traces,  h~ = h_{l-1}(old) + g_l;  h_l(new) = h~ + a_l * (h_{l-1}(new) - h_{l-1}(old)),  strict fp32, each
// operation rounded once.  Same thread mapping, load grouping and probe as k_scan.
template <int U, bool PROBE>
__global__ __launch_bounds__(kThreads) void k_scan_diag(float* trace, const float* __restrict__ g,
                                                         const float* __restrict__ diag, int l0, int Lc, int M, int d,
                                                         float* __restrict__ partials) {
#pragma clang fp contract(off)
  extern __shared__ float sh[];
  const int nv = d >> 2;
  const unsigned total = (unsigned)M * (unsigned)nv;
  const unsigned id = blockIdx.x * kThreads + threadIdx.x;
  const bool active = id < total;
  const size_t off = active ? (size_t)id * 4 : 0;          // n = 1: trace slot and g share the [M, d] layout
  const size_t slot = (size_t)M * d;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
  float4 acc = active ? *reinterpret_cast<const float4*>(trace + (size_t)(l0 - 1) * slot + off) : zero;   // new h_{l-1}
  float4 prev_old = acc;                                                                                   // old h_{l-1}
  const int lend = l0 + Lc;
  for (int lb = l0; lb < lend; lb += U) {
    float4 gv[U], av[U], old[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int l = lb + u;
      const bool ok = active && l < lend;
      gv[u] = ok ? *reinterpret_cast<const float4*>(g + (size_t)(l - 1) * slot + off) : zero;
      av[u] = ok ? *reinterpret_cast<const float4*>(diag + (size_t)(l - 1) * slot + off) : zero;
      old[u] = ok ? *reinterpret_cast<const float4*>(trace + (size_t)l * slot + off) : zero;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int l = lb + u;
      if (l < lend) {
        float4 tl, nw;
        tl.x = prev_old.x + gv[u].x; tl.y = prev_old.y + gv[u].y; tl.z = prev_old.z + gv[u].z; tl.w = prev_old.w + gv[u].w;
        float4 dl;
        dl.x = acc.x - prev_old.x; dl.y = acc.y - prev_old.y; dl.z = acc.z - prev_old.z; dl.w = acc.w - prev_old.w;
        dl.x = av[u].x * dl.x; dl.y = av[u].y * dl.y; dl.z = av[u].z * dl.z; dl.w = av[u].w * dl.w;
        nw.x = tl.x + dl.x; nw.y = tl.y + dl.y; nw.z = tl.z + dl.z; nw.w = tl.w + dl.w;
        if (PROBE) {
          float rs = sqdiff4(old[u], tl), ds = sqdiff4(nw, old[u]);   // tl = f_l(h_{l-1}(old))
          if (!active) { rs = 0.f; ds = 0.f; }
          rs = wave_sum_lane63(rs);
          ds = wave_sum_lane63(ds);
          if (lane == kWave - 1) {
            sh[(wave * 2 + 0) * Lc + (l - l0)] = rs;
            sh[(wave * 2 + 1) * Lc + (l - l0)] = ds;
          }
        }
        if (active) *reinterpret_cast<float4*>(trace + (size_t)l * slot + off) = nw;
        acc = nw;
        prev_old = old[u];
      }
    }
  }
  if (PROBE) {
    __syncthreads();
    for (int i = threadIdx.x; i < 2 * Lc; i += kThreads) {
      const float sm = ((sh[0 * 2 * Lc + i] + sh[1 * 2 * Lc + i]) + sh[2 * 2 * Lc + i]) + sh[3 * 2 * Lc + i];
      partials[(size_t)blockIdx.x * 2 * Lc + i] = sm;
    }
  }
}

// probe[i] = sum over blocks of partials[b][i], fp64 accumulation in a fixed order; one block per entry.
// Entries are laid out [2][Lfull] in `probe`; the Lc computed layers start at column `col0`, the columns
// before it (sequential prefix) are written as zero.
__global__ __launch_bounds__(kThreads) void k_probe_finalize(const float* __restrict__ partials, int nblk, int width,
                                                              float* __restrict__ probe, int sqrt_below, int col0,
                                                              int Lfull) {
  __shared__ double shd[kThreads];
  const int i = blockIdx.x;
  const int Lc = width / 2;
  float* dst = probe + (size_t)(i / Lc) * Lfull + col0 + (i % Lc);
  if (threadIdx.x == 0 && (i % Lc) == 0)
    for (int c = 0; c < col0; ++c) probe[(size_t)(i / Lc) * Lfull + c] = 0.f;
  double s = 0.0;
  for (int b = threadIdx.x; b < nblk; b += kThreads) s += (double)partials[(size_t)b * width + i];
  shd[threadIdx.x] = s;
  __syncthreads();
  for (int o = kThreads / 2; o > 0; o >>= 1) {
    if (threadIdx.x < o) shd[threadIdx.x] += shd[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) *dst = (i < sqrt_below) ? (float)sqrt(shd[0]) : (float)shd[0];
}

// out[l][n][k] = in[l][k][n], bf16, 64 x 64 tiles through LDS.
__global__ __launch_bounds__(kThreads) void k_transpose_bf16(const bf16_t* __restrict__ in, bf16_t* __restrict__ out,
                                                              int K, int N) {
  __shared__ bf16_t tile[64][66];
  const size_t lo = (size_t)blockIdx.z * K * N;
  const int k0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int r = ty; r < 64; r += 4) {
    const int k = k0 + r, n = n0 + tx;
    tile[r][tx] = (k < K && n < N) ? in[lo + (size_t)k * N + n] : (bf16_t)0;
  }
  __syncthreads();
  for (int r = ty; r < 64; r += 4) {
    const int n = n0 + r, k = k0 + tx;
    if (n < N && k < K) out[lo + (size_t)n * K + k] = tile[tx][r];
  }
}

}  // namespace

// ------------------------------------------------------------------------------------------------
namespace {
template <int N>
void launch_premix_n(hipStream_t s, const Dims& D, int l0, int Lc, const float* trace, const float* pre, float* ubuf,
                     void* xhat, bool out_bf16) {
  dim3 grid(D.M, Lc), block(row_block_threads(D.d));
  const bool stream = (size_t)Lc * D.M * D.n * D.d * sizeof(float) > kStreamBytes;
  if (out_bf16) {
    if (stream) hipLaunchKernelGGL((k_premix_rmsnorm<N, bf16_t, true>), grid, block, 0, s, trace, pre, ubuf, (bf16_t*)xhat, l0, D.M, D.d, D.eps);
    else hipLaunchKernelGGL((k_premix_rmsnorm<N, bf16_t, false>), grid, block, 0, s, trace, pre, ubuf, (bf16_t*)xhat, l0, D.M, D.d, D.eps);
  } else
    hipLaunchKernelGGL((k_premix_rmsnorm<N, float, false>), grid, block, 0, s, trace, pre, ubuf, (float*)xhat, l0, D.M, D.d, D.eps);
}
}  // namespace

hipError_t launch_premix_rmsnorm(hipStream_t s, const Dims& D, int l0, int Lc, const float* trace,
                                 const float* pre, float* ubuf, void* xhat, bool out_bf16) {
  // pre == nullptr: the rows are taken as single-stream states whatever D.n says (chunk inputs of fused layers)
  switch (pre ? D.n : 1) {
    case 1: launch_premix_n<1>(s, D, l0, Lc, trace, pre, ubuf, xhat, out_bf16); break;
    case 2: launch_premix_n<2>(s, D, l0, Lc, trace, pre, ubuf, xhat, out_bf16); break;
    case 3: launch_premix_n<3>(s, D, l0, Lc, trace, pre, ubuf, xhat, out_bf16); break;
    case 4: launch_premix_n<4>(s, D, l0, Lc, trace, pre, ubuf, xhat, out_bf16); break;
    case 8: launch_premix_n<8>(s, D, l0, Lc, trace, pre, ubuf, xhat, out_bf16); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_mid_rmsnorm(hipStream_t s, const Dims& D, int l0, int Lc, const float* trace,
                              const float* ubuf, const float* a, void* xhat2, bool out_bf16) {
  dim3 grid(D.M, Lc), block(row_block_threads(D.d));
  const float* usrc = (D.n == 1) ? trace : ubuf;
  const size_t lstride = (D.n == 1) ? (size_t)D.M * D.d : (size_t)D.M * D.d;
  const size_t rstride = (size_t)D.d;
  const bool stream = (size_t)2 * Lc * D.M * D.d * sizeof(float) > kStreamBytes;
  if (out_bf16) {
    if (stream) hipLaunchKernelGGL((k_mid_rmsnorm<bf16_t, true>), grid, block, 0, s, usrc, lstride, rstride, a, (bf16_t*)xhat2, l0, D.M, D.d, D.eps);
    else hipLaunchKernelGGL((k_mid_rmsnorm<bf16_t, false>), grid, block, 0, s, usrc, lstride, rstride, a, (bf16_t*)xhat2, l0, D.M, D.d, D.eps);
  } else
    hipLaunchKernelGGL((k_mid_rmsnorm<float, false>), grid, block, 0, s, usrc, lstride, rstride, a, (float*)xhat2, l0, D.M, D.d, D.eps);
  return hipGetLastError();
}

hipError_t launch_chunk_mid_rmsnorm(hipStream_t s, const Dims& D, int c0, int Nc, int F, const float* trace,
                                    const float* a, float* aC, void* xhat2, bool out_bf16) {
  dim3 grid(D.M, Nc), block(row_block_threads(D.d));
  if (out_bf16)
    hipLaunchKernelGGL(k_chunk_mid_rmsnorm<bf16_t>, grid, block, 0, s, trace, a, aC, (bf16_t*)xhat2, c0, F, D.M, D.d, D.eps);
  else
    hipLaunchKernelGGL(k_chunk_mid_rmsnorm<float>, grid, block, 0, s, trace, a, aC, (float*)xhat2, c0, F, D.M, D.d, D.eps);
  return hipGetLastError();
}

hipError_t launch_chunk_sum(hipStream_t s, const Dims& D, int c0, int Nc, int F, const float* aC, const float* m, float* gC) {
  const size_t slab_vec = (size_t)D.M * D.d / 4;
  dim3 grid((unsigned)((slab_vec + kThreads - 1) / kThreads), Nc), block(kThreads);
  hipLaunchKernelGGL(k_chunk_sum, grid, block, 0, s, (const float4*)aC, (const float4*)m, (float4*)gC, c0, F, slab_vec);
  return hipGetLastError();
}

hipError_t launch_rope_qknorm(hipStream_t s, const Dims& D, int l0, int Lc, void* qkv, bool is_bf16,
                              const float* cos_tab, const float* sin_tab) {
  dim3 grid(D.M, Lc), block(kThreads);
  if (is_bf16 && D.dh == 128 && D.d % 8 == 0) {
    const size_t total = (size_t)Lc * D.M * 2 * D.H * 8;
    hipLaunchKernelGGL(k_rope_qknorm_bf16_dh128, dim3((unsigned)((total + kThreads - 1) / kThreads)), block, 0, s,
                       (bf16_t*)qkv, cos_tab, sin_tab, l0, D.M, D.T, D.d, D.H, total, D.eps);
  } else if (is_bf16)
    hipLaunchKernelGGL(k_rope_qknorm<bf16_t>, grid, block, 0, s, (bf16_t*)qkv, cos_tab, sin_tab, l0, D.M, D.T, D.d, D.H, D.dh, D.eps);
  else
    hipLaunchKernelGGL(k_rope_qknorm<float>, grid, block, 0, s, (float*)qkv, cos_tab, sin_tab, l0, D.M, D.T, D.d, D.H, D.dh, D.eps);
  return hipGetLastError();
}

hipError_t launch_init_trace(hipStream_t s, const Dims& D, const float* src, float* trace, int first, int count) {
  if (count <= 0) return hipSuccess;
  const size_t nvec = (size_t)D.M * D.n * D.d / 4;
  const unsigned blocks = (unsigned)((nvec + kThreads - 1) / kThreads);
  hipLaunchKernelGGL(k_init_trace, dim3(blocks), dim3(kThreads), 0, s, (const float4*)src, (float4*)trace, nvec, first, count);
  return hipGetLastError();
}

// Threads per block of the correction kernels: small batches of rows (decode blocks) take one wave per block so that
// the few thousand waves spread over all compute units; the choice depends on the batch shape only.
static int scan_block_threads(const Dims& D) { return (size_t)D.M * D.d <= ((size_t)1 << 20) ? kWave : kThreads; }

int scan_partial_blocks(const Dims& D) {
  const size_t total = (size_t)D.M * (D.d / 4);
  const int bt = scan_block_threads(D);
  return (int)((total + bt - 1) / bt);
}

namespace {
template <int N, int U, int BT, bool STREAM>
void launch_scan_bt(hipStream_t s, const Dims& D, int mode, int l0, int Lc, float* trace, const float* g,
                    const float* Hres, const float* post, bool write, float* partials, int independent) {
  dim3 grid(scan_partial_blocks(D)), block(BT);
  const size_t shm = partials ? (size_t)(BT / kWave) * 2 * Lc * sizeof(float) : 0;
  if (write && partials)
    hipLaunchKernelGGL((k_scan<N, U, true, true, BT, STREAM>), grid, block, shm, s, trace, g, Hres, post, mode, l0, Lc, D.M, D.d, partials, independent);
  else if (write)
    hipLaunchKernelGGL((k_scan<N, U, false, true, BT, STREAM>), grid, block, 0, s, trace, g, Hres, post, mode, l0, Lc, D.M, D.d, partials, independent);
  else
    hipLaunchKernelGGL((k_scan<N, U, true, false, BT, STREAM>), grid, block, shm, s, trace, g, Hres, post, mode, l0, Lc, D.M, D.d, partials, independent);
}
template <int N, int U>
void launch_scan_n(hipStream_t s, const Dims& D, int mode, int l0, int Lc, float* trace, const float* g,
                   const float* Hres, const float* post, bool write, float* partials, int independent) {
  // small batches: one wave per block, operands read through the caches; large ones: 256 threads, and streamed
  // when the trace of the launch is far larger than the caches
  if (scan_block_threads(D) == kWave)
    launch_scan_bt<N, U, kWave, false>(s, D, mode, l0, Lc, trace, g, Hres, post, write, partials, independent);
  else if ((size_t)Lc * D.M * D.n * D.d * sizeof(float) > kStreamBytes)
    launch_scan_bt<N, U, kThreads, true>(s, D, mode, l0, Lc, trace, g, Hres, post, write, partials, independent);
  else
    launch_scan_bt<N, U, kThreads, false>(s, D, mode, l0, Lc, trace, g, Hres, post, write, partials, independent);
}
}  // namespace

hipError_t launch_scan(hipStream_t s, const Dims& D, int mode, int l0, int Lc, float* trace, const float* g,
                       const float* Hres, const float* post, bool write, float* partials, bool independent) {
  switch (D.n) {
    case 1:
      // few rows (decode blocks): the grid cannot fill the chip, so each thread keeps the loads of more layers
      // in flight; the per-element arithmetic and the probe's reduction tree are the same for every U
      if ((size_t)D.M * D.d <= ((size_t)1 << 20) && Lc > 4)
        launch_scan_n<1, 10>(s, D, mode, l0, Lc, trace, g, Hres, post, write, partials, independent ? 1 : 0);
      else
        launch_scan_n<1, 4>(s, D, mode, l0, Lc, trace, g, Hres, post, write, partials, independent ? 1 : 0);
      break;
    case 2: launch_scan_n<2, 2>(s, D, mode, l0, Lc, trace, g, Hres, post, write, partials, independent ? 1 : 0); break;
    case 3: launch_scan_n<3, 2>(s, D, mode, l0, Lc, trace, g, Hres, post, write, partials, independent ? 1 : 0); break;
    case 4: launch_scan_n<4, 2>(s, D, mode, l0, Lc, trace, g, Hres, post, write, partials, independent ? 1 : 0); break;
    case 8: launch_scan_n<8, 1>(s, D, mode, l0, Lc, trace, g, Hres, post, write, partials, independent ? 1 : 0); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// ---- the correction that also prepares the next round's branch inputs (k_scan_norm)
// Decode-sized batches keep the two kernels: with 128 rows the row-per-workgroup form measured 31 us against 18.5 + 7.7.
bool scan_fuses_norm(const Dims& D) { return (size_t)D.M * D.d > ((size_t)1 << 20) && D.d / 4 <= 1024; }
int scan_norm_blocks(const Dims& D) { return D.M; }

namespace {
template <int N, int U>
void launch_scan_norm_n(hipStream_t s, const Dims& D, int mode, int l0, int Lc, float* trace, const float* g,
                        const float* Hres, const float* post, const float* pre, float* ubuf, void* xhat, bool out_bf16,
                        float* partials) {
  dim3 grid(D.M), block(row_block_threads(D.d));
  const size_t shm = (2 * kMaxWaves + (partials ? (size_t)(block.x / kWave) * 2 * Lc : 0)) * sizeof(float);
  const bool stream = (size_t)Lc * D.M * D.n * D.d * sizeof(float) > kStreamBytes;
#define SNLP_SCAN_NORM(PROBE_, OUT_, STREAM_)                                                                         \
  hipLaunchKernelGGL((k_scan_norm<N, U, PROBE_, OUT_, STREAM_>), grid, block, shm, s, trace, g, Hres, post, pre, ubuf, \
                     (OUT_*)xhat, mode, l0, Lc, D.L, D.M, D.d, D.eps, partials)
  if (out_bf16) {
    if (partials) { if (stream) SNLP_SCAN_NORM(true, bf16_t, true); else SNLP_SCAN_NORM(true, bf16_t, false); }
    else { if (stream) SNLP_SCAN_NORM(false, bf16_t, true); else SNLP_SCAN_NORM(false, bf16_t, false); }
  } else {
    if (partials) SNLP_SCAN_NORM(true, float, false); else SNLP_SCAN_NORM(false, float, false);
  }
#undef SNLP_SCAN_NORM
}
}  // namespace

hipError_t launch_scan_norm(hipStream_t s, const Dims& D, int mode, int l0, int Lc, float* trace, const float* g,
                            const float* Hres, const float* post, const float* pre, float* ubuf, void* xhat,
                            bool out_bf16, float* partials) {
  if (!scan_fuses_norm(D)) return hipErrorInvalidValue;
  switch (D.n) {
    case 1: launch_scan_norm_n<1, 4>(s, D, mode, l0, Lc, trace, g, Hres, post, pre, ubuf, xhat, out_bf16, partials); break;
    case 2: launch_scan_norm_n<2, 2>(s, D, mode, l0, Lc, trace, g, Hres, post, pre, ubuf, xhat, out_bf16, partials); break;
    case 3: launch_scan_norm_n<3, 2>(s, D, mode, l0, Lc, trace, g, Hres, post, pre, ubuf, xhat, out_bf16, partials); break;
    case 4: launch_scan_norm_n<4, 2>(s, D, mode, l0, Lc, trace, g, Hres, post, pre, ubuf, xhat, out_bf16, partials); break;
    case 8: launch_scan_norm_n<8, 1>(s, D, mode, l0, Lc, trace, g, Hres, post, pre, ubuf, xhat, out_bf16, partials); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_scan_diag(hipStream_t s, const Dims& D, int l0, int Lc, float* trace, const float* g,
                            const float* diag, float* partials) {
  if (D.n != 1) return hipErrorInvalidValue;
  dim3 grid(scan_partial_blocks(D)), block(kThreads);
  if (partials)
    hipLaunchKernelGGL((k_scan_diag<3, true>), grid, block, (size_t)4 * 2 * Lc * sizeof(float), s, trace, g, diag, l0, Lc,
                       D.M, D.d, partials);
  else
    hipLaunchKernelGGL((k_scan_diag<3, false>), grid, block, 0, s, trace, g, diag, l0, Lc, D.M, D.d, partials);
  return hipGetLastError();
}

hipError_t launch_probe_finalize(hipStream_t s, const Dims& D, int Lc, const float* partials, float* probe,
                                 bool take_sqrt_first_only, int col0, int nblk) {
  const int width = 2 * Lc;
  const int entries = take_sqrt_first_only ? Lc : width;
  hipLaunchKernelGGL(k_probe_finalize, dim3(entries), dim3(kThreads), 0, s, partials, nblk > 0 ? nblk : scan_partial_blocks(D), width,
                     probe, take_sqrt_first_only ? Lc : 0, col0, col0 + Lc);
  return hipGetLastError();
}

hipError_t launch_transpose_bf16(hipStream_t s, const bf16_t* in, bf16_t* out, int L, int K, int N) {
  dim3 grid((N + 63) / 64, (K + 63) / 64, L), block(kThreads);
  hipLaunchKernelGGL(k_transpose_bf16, grid, block, 0, s, in, out, K, N);
  return hipGetLastError();
}

}  // namespace snlp

// Layer-batched grouped GEMMs of the SNLP evaluation step (Eq. (4); "batched form" of Methods,
// "Layer fusion": per-layer weights stacked, all layers evaluated in one grouped operation).
//   C[l] = epilogue(A[l] (M x K) * W[l] (K x N)),  l = 0..Lc-1, one launch for all layers.
// bf16 path: MFMA v_mfma_f32_32x32x16_bf16 with fp32 accumulation.  Three kernels:
//   k_gemm_bf16_256  M > 128, launches with many tiles: 256 x 256 (or 256 x 128) x 64 tiles, both operands through a
//                    five-unit LDS ring filled by direct-to-LDS loads; weights repacked [N, K]; the last incomplete
//                    round of a launch may be cut into 256 x 128 or 256 x 64 pieces;
//   k_gemm_bf16      M > 128, small launches: 128 x 128 tiles staged through padded LDS from registers;
//   k_gemm_skinny    M <= 128: weights streamed from HBM straight into operand registers (repacked into MFMA operand
//                    order), only the token tile through LDS.
// Which kernel and which tile shape a launch gets depends on its size, the number of layers in it included.  What
// never depends on it is the arithmetic of an output element: every kernel and every tile shape accumulates the
// same k-ordered sequence of 32 x 32 x 16 MFMAs and applies the same epilogue, so a layer computes bit-identical
// results whether it is launched alone (sequential execution, Alg. 1) or in the batch (Alg. 2).
#include "snlp_kernels.hpp"

namespace snlp {

namespace {


constexpr int kThreads = 256;

__device__ __forceinline__ bf16_t float_to_bf16_bits(float f) {
  __bf16 h = static_cast<__bf16>(f);
  return __builtin_bit_cast(bf16_t, h);
}

template <int EPI>
__device__ __forceinline__ float apply_epilogue(float acc, const float* R, size_t idx) {
  if (EPI == EPI_RELU2) {
    const float z = fmaxf(acc, 0.f);
    return z * z;
  }
  if (EPI == EPI_ADD_F32) return R[idx] + acc;
  return acc;
}

// ------------------------------------------------------------------------------------------------
// fp32 reference-precision path: 64 x 64 tile, 16 x 16 threads, 4 x 4 outputs each, sequential k order.
template <int EPI>
__global__ __launch_bounds__(kThreads) void k_gemm_f32(const float* __restrict__ A, size_t sA,
                                                        const float* __restrict__ W, size_t sW,
                                                        float* __restrict__ C, size_t sC,
                                                        const float* __restrict__ R, size_t sR, int M, int N, int K, int a_group) {
  __shared__ float As[16][68];
  __shared__ float Ws[16][68];
  const int li = blockIdx.z;
  A += (size_t)(li / a_group) * sA; W += (size_t)li * sW; C += (size_t)li * sC;
  if (EPI == EPI_ADD_F32) R += (size_t)li * sR;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int idx = threadIdx.x + e * kThreads;
      const int r = idx >> 4, kk = idx & 15;
      const int m = m0 + r, k = k0 + kk;
      As[kk][r] = (m < M && k < K) ? A[(size_t)m * K + k] : 0.f;
      const int kk2 = idx >> 6, nn = idx & 63;
      const int k2 = k0 + kk2, n = n0 + nn;
      Ws[kk2][nn] = (k2 < K && n < N) ? W[(size_t)k2 * N + n] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Ws[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n < N) {
        const size_t idx = (size_t)m * N + n;
        C[idx] = apply_epilogue<EPI>(acc[i][j], R, idx);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// bf16 MFMA path.
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));   // native vector: stays in registers

// Start of layer slab `off` (in elements) of an output buffer holding bf16 or fp32.
template <bool C_BF16>
__device__ __forceinline__ void* layer_ptr(void* C, size_t off) {
  return C_BF16 ? static_cast<void*>(reinterpret_cast<bf16_t*>(C) + off) : static_cast<void*>(reinterpret_cast<float*>(C) + off);
}

// Stores one 32 x 32 accumulator block of v_mfma_f32_32x32x16: this lane holds column `col` and rows
// row0 + 8 (r / 4) + row_in + r % 4, r = 0..15, row_in = 4 (lane / 32).  C and R already point at the layer.
// A block that lies wholly inside the matrix takes a branch-free path with all residual loads issued before
// the first store: a load -> add -> store chain per element costs one memory round trip each.
template <int EPI, bool C_BF16>
__device__ __forceinline__ void store_block(const f32x16_t& acc, void* __restrict__ C, const float* __restrict__ R,
                                            int row0, int row_in, int col, int M, int N) {
  const size_t base = (size_t)(row0 + row_in) * N + col;
  if (row0 + 32 <= M) {
    float v[16];
    if (EPI == EPI_ADD_F32) {
#pragma unroll
      for (int r = 0; r < 16; ++r) v[r] = R[base + (size_t)((r >> 2) * 8 + (r & 3)) * N];
#pragma unroll
      for (int r = 0; r < 16; ++r) v[r] = v[r] + acc[r];
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) v[r] = apply_epilogue<EPI>(acc[r], nullptr, 0);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const size_t idx = base + (size_t)((r >> 2) * 8 + (r & 3)) * N;
      if (C_BF16)
        reinterpret_cast<bf16_t*>(C)[idx] = float_to_bf16_bits(v[r]);
      else
        reinterpret_cast<float*>(C)[idx] = v[r];
    }
    return;
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int row = row0 + (r >> 2) * 8 + row_in + (r & 3);
    if (row < M) {
      const size_t idx = (size_t)row * N + col;
      const float v = apply_epilogue<EPI>(acc[r], R, idx);
      if (C_BF16)
        reinterpret_cast<bf16_t*>(C)[idx] = float_to_bf16_bits(v);
      else
        reinterpret_cast<float*>(C)[idx] = v;
    }
  }
}

constexpr int kBK = 64;            // k extent of one staged tile
constexpr int kLdsRow = kBK + 8;   // padded LDS row (elements): 144 B, odd multiple of 16 B

struct TileCoord { int layer, tm, tn; };

// Linear workgroup id -> (layer, tile).  Workgroups are dealt round-robin to the 8 XCDs, each with its
// own L2; consecutive logical tiles are therefore given to the SAME XCD, and within a layer tiles are
// ordered in groups of 8 row-tiles x all column-tiles (column-major inside a group) so that the
// tiles resident on an XCD at one time share A row-slabs and weight column-slabs.
__device__ __forceinline__ TileCoord decode_tile(unsigned t, int tiles_m, int tiles_n) {
  const unsigned per_layer = (unsigned)tiles_m * tiles_n;
  TileCoord c;
  c.layer = (int)(t / per_layer);
  const unsigned rem = t % per_layer;
  constexpr unsigned GM = 8;
  const unsigned gspan = GM * tiles_n;
  const unsigned group = rem / gspan, in = rem % gspan;
  const unsigned first_m = group * GM;
  const unsigned gsz = (tiles_m - first_m) < GM ? (tiles_m - first_m) : GM;
  c.tm = (int)(first_m + in % gsz);
  c.tn = (int)(in / gsz);
  return c;
}

__device__ __forceinline__ TileCoord map_tile(unsigned pid, unsigned total, int tiles_m, int tiles_n) {
  const unsigned q = total / 8, r = total % 8;
  const unsigned xcd = pid % 8, local = pid / 8;
  return decode_tile(xcd * q + (xcd < r ? xcd : r) + local, tiles_m, tiles_n);
}

// The last, incomplete round of a launch of 256 x 256 tiles ("big tiles", index t in the order above) is cut into
// smaller pieces: TileRange names big tiles [first, first + count), each cut into `parts` pieces of BM x BN outputs
// (256 x 128: 2, 128 x 128: 4, 128 x 64: 8), the pieces of one big tile on one XCD.  A round of r < 256 big tiles takes
// as long as a full one; a piece's time goes with the operand bytes it moves, (BM + BN) / 512 of a big tile's at best,
// so as 2 r halves the round takes three quarters of that, as 4 r pieces of 128 x 128 one half, as 8 r pieces of
// 128 x 64 three eighths (measured: 0.47) -- as long as the pieces fit one round.  Every piece runs the same k-ordered
// MFMA sequence per output element, so nothing changes in the results.
struct TileRange { unsigned first, count; int big_m, big_n, parts; };

// Piece of tail workgroup `pid` (counted from the first tail workgroup), in units of BM x BN tiles; false: the piece
// lies outside the matrix or past the range.
template <int BM, int BN>
__device__ __forceinline__ bool map_tail_tile(unsigned pid, const TileRange& tr, int M, int N, TileCoord& c) {
  constexpr unsigned parts_n = 256 / BN, parts = (256 / BM) * parts_n;
  const unsigned local = (pid / (8 * parts)) * 8 + pid % 8, part = (pid / 8) % parts;
  if (local >= tr.count) return false;
  const TileCoord b = decode_tile(tr.first + local, tr.big_m, tr.big_n);
  c.layer = b.layer;
  c.tm = b.tm * (256 / BM) + (int)(part / parts_n);
  c.tn = b.tn * (int)parts_n + (int)(part % parts_n);
  return c.tm * BM < M && c.tn * BN < N;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, bool C_BF16>
__global__ __launch_bounds__(kThreads) void k_gemm_bf16(const bf16_t* __restrict__ A, size_t sA,
                                                         const bf16_t* __restrict__ Wt, size_t sW, void* Cv, size_t sC,
                                                         const float* __restrict__ R, size_t sR, int M, int N, int K,
                                                         int tiles_m, int tiles_n, unsigned total_tiles, int a_group) {
  static_assert(WAVES_M * WAVES_N == 4, "four waves per workgroup");
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int TM = WM / 32, TN = WN / 32;
  static_assert(TM >= 1 && TN >= 1 && WM % 32 == 0 && WN % 32 == 0, "wave tile is a grid of 32 x 32 MFMA tiles");
  constexpr int PA = BM / 32, PB = BN / 32;   // 16-byte loads per thread per staged tile

  __shared__ __attribute__((aligned(16))) bf16_t lds[(BM + BN) * kLdsRow];
  bf16_t* ldsA = lds;
  bf16_t* ldsB = lds + BM * kLdsRow;

  const TileCoord tc = map_tile(blockIdx.x, total_tiles, tiles_m, tiles_n);
  A += (size_t)(tc.layer / a_group) * sA;
  Wt += (size_t)tc.layer * sW;
  const int m0 = tc.tm * BM, n0 = tc.tn * BN;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int chunk = tid & 7;        // 16-byte chunk inside a 128-byte tile row
  const int lrow = tid >> 3;        // 0..31

  // global row pointers (rows beyond the matrix are clamped: loaded, multiplied, never stored)
  const u32x4_t* gA[PA];
  const u32x4_t* gB[PB];
#pragma unroll
  for (int p = 0; p < PA; ++p) {
    int r = m0 + lrow + p * 32;
    r = r < M ? r : M - 1;
    gA[p] = reinterpret_cast<const u32x4_t*>(A + (size_t)r * K) + chunk;
  }
#pragma unroll
  for (int p = 0; p < PB; ++p) {
    int r = n0 + lrow + p * 32;
    r = r < N ? r : N - 1;
    gB[p] = reinterpret_cast<const u32x4_t*>(Wt + (size_t)r * K) + chunk;
  }

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  u32x4_t ra[PA], rb[PB];
#pragma unroll
  for (int p = 0; p < PA; ++p) ra[p] = gA[p][0];
#pragma unroll
  for (int p = 0; p < PB; ++p) rb[p] = gB[p][0];

  const int nk = K / kBK;
  const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;
  for (int kt = 0; kt < nk; ++kt) {
    __syncthreads();   // previous tile fully consumed
#pragma unroll
    for (int p = 0; p < PA; ++p)
      *reinterpret_cast<u32x4_t*>(ldsA + (lrow + p * 32) * kLdsRow + chunk * 8) = ra[p];
#pragma unroll
    for (int p = 0; p < PB; ++p)
      *reinterpret_cast<u32x4_t*>(ldsB + (lrow + p * 32) * kLdsRow + chunk * 8) = rb[p];
    __syncthreads();
    if (kt + 1 < nk) {
      const int o = (kt + 1) * (kBK / 8);
#pragma unroll
      for (int p = 0; p < PA; ++p) ra[p] = gA[p][o];
#pragma unroll
      for (int p = 0; p < PB; ++p) rb[p] = gB[p][o];
    }
#pragma unroll
    for (int ks = 0; ks < kBK / 16; ++ks) {
      bf16x8_t af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        af[i] = *reinterpret_cast<const bf16x8_t*>(ldsA + (wm * WM + i * 32 + frag_row) * kLdsRow + ks * 16 + frag_k);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        bfr[j] = *reinterpret_cast<const bf16x8_t*>(ldsB + (wn * WN + j * 32 + frag_row) * kLdsRow + ks * 16 + frag_k);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
  }

  // epilogue: lane holds column (lane % 32) and rows 8*(r/4) + 4*(lane/32) + r%4 of each 32 x 32 tile
  const int col_in = lane & 31, row_in = (lane >> 5) * 4;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = n0 + wn * WN + j * 32 + col_in;
      if (col >= N) continue;
      store_block<EPI, C_BF16>(acc[i][j], layer_ptr<C_BF16>(Cv, (size_t)tc.layer * sC), R ? R + (size_t)tc.layer * sR : nullptr,
                               m0 + wm * WM + i * 32, row_in, col, M, N);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Large-tile kernel for prefill shapes: 256 x 256 x 64 tiles, 8 waves (4 x 2), wave tile 64 x 128.
// Operand tiles travel global -> LDS with direct-to-LDS loads (global_load_lds_dwordx4: lane i's 16 bytes land at
// base + 16 i; no staging registers).  All 160 KB of LDS form a ring of five 32 KB units; a unit is the A half
// or the weight half of one k-tile (256 rows x 128 B), in the order A0 W0 A1 W1 A2 ...  While k-tile kt is
// multiplied its two units and A of kt+1 are resident, and W of kt+1 and A of kt+2 are requested into the two
// slots that k-tile kt-1 left.  So only 32 KB per CU must arrive within one multiply phase and the other 32 KB
// has two; the first version had two 64 KB stages, one whole k-tile due per phase, all of it requested in one
// burst after the barrier.
// LDS rows are 128 B without padding; bank conflicts are avoided by storing the 16-byte chunk c of row r at
// position c ^ ((r >> 1) & 7), done on the global-address side.
#define SNLP_GLDS16(gptr, lptr)                                                                              \
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gptr),                   \
                                   (__attribute__((address_space(3))) void*)(lptr), 16, 0, 0)

// One tile of 256 rows x BN columns, BN = 256 or 128 (wave tile 64 x BN/2).  With 128 a weight unit fills half a
// slot and the tile moves 1.5x the bytes per flop, but a launch too small for several rounds of 256 x 256 tiles (one
// layer of the sequential path, narrow outputs) gets twice the workgroups, and the last incomplete round of a big
// launch may be cut into such tiles (see TileRange).
template <int BN, int EPI, bool C_BF16>
__device__ __forceinline__ void ring_tile(const TileCoord tc, bf16_t* __restrict__ ring, const bf16_t* __restrict__ A, size_t sA,
                                          const bf16_t* __restrict__ Wt, size_t sW, void* Cv, size_t sC,
                                          const float* __restrict__ R, size_t sR, int M, int N, int K, int a_group) {
  static_assert(BN == 256 || BN == 128, "two column-tile widths");
  constexpr int BM = 256;
  constexpr int TNF = BN / 64;       // 32-column MFMA tiles per wave
  constexpr int GW = BN / 64;        // 1 KB row groups of a weight unit per wave
  constexpr int kUnit = 256 * kBK;   // elements in a slot: 256 rows of 64 bf16 (a weight unit uses the first BN rows)
  A += (size_t)(tc.layer / a_group) * sA;
  Wt += (size_t)tc.layer * sW;
  const int m0 = tc.tm * BM, n0 = tc.tn * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  // direct-to-LDS loads: wave w fills row groups 4w .. 4w+3 (8 rows, 1 KB each) of an A unit and GW w .. GW w + GW-1
  // of a weight unit
  const bf16_t* gsrcA[4];
  const bf16_t* gsrcW[GW];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int row = (wave * 4 + j) * 8 + (lane >> 3);            // 0..255 in the unit
    const int chunk = (lane & 7) ^ ((row >> 1) & 7);
    int ra = m0 + row;
    ra = ra < M ? ra : M - 1;
    gsrcA[j] = A + (size_t)ra * K + chunk * 8;
  }
#pragma unroll
  for (int j = 0; j < GW; ++j) {
    const int row = (wave * GW + j) * 8 + (lane >> 3);           // 0..BN-1 in the unit
    const int chunk = (lane & 7) ^ ((row >> 1) & 7);
    int rw = n0 + row;
    rw = rw < N ? rw : N - 1;
    gsrcW[j] = Wt + (size_t)rw * K + chunk * 8;
  }
  auto issue_a = [&](int slot, int kt) {
    bf16_t* dst = ring + slot * kUnit + wave * 4 * 512;
#pragma unroll
    for (int j = 0; j < 4; ++j) SNLP_GLDS16(gsrcA[j] + (size_t)kt * kBK, dst + j * 512);
  };
  auto issue_w = [&](int slot, int kt) {
    bf16_t* dst = ring + slot * kUnit + wave * GW * 512;
#pragma unroll
    for (int j = 0; j < GW; ++j) SNLP_GLDS16(gsrcW[j] + (size_t)kt * kBK, dst + j * 512);
  };

  f32x16_t acc[2][TNF];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < TNF; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // operand reads: row (lane & 31) of a 32-row fragment, chunk ks*2 + (lane >> 5), swizzled
  const int sw = ((lane & 31) >> 1) & 7, hi = lane >> 5;
  const int rowoff = (lane & 31) * kBK;
  // One k-tile: the fragments of k-step ks+1 are read while the MFMAs of k-step ks issue (one LDS read behind
  // each of six MFMAs), so only the first k-step of a tile waits for LDS; and the eight tile loads this wave owes
  // the ring are spread over the four k-steps, two each behind MFMAs (the weight unit, due first, in k-steps 0
  // and 1).  Issued as one burst after the barrier they stall all eight waves at once in the vector-memory issue
  // queue (64 KB takes the address path over 1000 cycles) and a stalled wave issues no MFMAs either.
  auto compute = [&](const bf16_t* ua, const bf16_t* uw, bf16_t* dw, int ktw, bf16_t* da, int kta) {
    bf16x8_t af[2][2], bfr[2][TNF];
    auto read_frags = [&](int buf, int ks) {
      const int off = rowoff + (((ks * 2 + hi) ^ sw) << 3);
#pragma unroll
      for (int i = 0; i < 2; ++i) af[buf][i] = *reinterpret_cast<const bf16x8_t*>(ua + (wm * 64 + i * 32) * kBK + off);
#pragma unroll
      for (int j = 0; j < TNF; ++j) bfr[buf][j] = *reinterpret_cast<const bf16x8_t*>(uw + (wn * (BN / 2) + j * 32) * kBK + off);
    };
    read_frags(0, 0);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      if (ks + 1 < 4) read_frags((ks + 1) & 1, ks + 1);
      // two tile loads per k-step: the weight unit's GW first, then the A unit's four
      constexpr int kLoads = GW + 4;
      const bool loads = 2 * ks < kLoads;
      if (loads) {
#pragma unroll
        for (int u = 2 * ks; u < 2 * ks + 2 && u < kLoads; ++u) {
          if (u < GW) SNLP_GLDS16(ktw >= 0 ? gsrcW[u] + (size_t)ktw * kBK : Wt, dw + u * 512);
          else SNLP_GLDS16(kta >= 0 ? gsrcA[u - GW] + (size_t)kta * kBK : A, da + (u - GW) * 512);
        }
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < TNF; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][i], bfr[ks & 1][j], acc[i][j], 0, 0, 0);
      // issue order for 8 MFMAs: M D M D M V M D M D M V M D M D (D: LDS read, absent in the last k-step; V: tile
      // load); for 4: M D M V M D M V, the remaining reads after the last MFMA
      constexpr int NM = 2 * TNF, NR = 2 + TNF;   // MFMAs and fragment reads per k-step; NM - 2 slots take a read
#pragma unroll
      for (int q = 0; q < NM; ++q) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        const bool vslot = NM == 8 ? (q == 2 || q == 5) : (q == 1 || q == 3);
        if (vslot) {
          if (loads) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        } else if (ks + 1 < 4) {
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
      }
      if (NR > NM - 2 && ks + 1 < 4) __builtin_amdgcn_sched_group_barrier(0x100, NR - (NM - 2) > 0 ? NR - (NM - 2) : 1, 0);
      __builtin_amdgcn_sched_barrier(0);   // keep the next k-step's MFMAs behind this one's reads
    }
  };

  // Unit u = 2 kt (A of k-tile kt) or 2 kt + 1 (its weights) lives in slot u % 5.  Phase kt multiplies units
  // 2 kt and 2 kt + 1 and requests units 2 kt + 3 and 2 kt + 4 into the slots the barrier before it freed
  // (phase 0: two slots not used yet).  For units past the end of K every lane requests the first 16 bytes of the
  // operand instead (one sector per load, into a slot nobody reads again), which keeps the loop free of
  // branches and the wait count uniform.
  const int nk = K / kBK;   // at least 2 (the launcher's condition)
  issue_a(0, 0);
  issue_w(1, 0);
  issue_a(2, 1);
  int slot_a = 0;   // slot of unit 2 kt
  for (int kt = 0; kt < nk; ++kt) {
    // this wave's parts of both units of k-tile kt have landed: loads return in order and only the four of the
    // youngest unit requested so far (A of kt+1) may still be outstanding
    asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)" ::: "memory");
    // everyone's have; everyone is done with k-tile kt-1, whose two slots are refilled in this phase (a bare
    // barrier: __syncthreads() may also wait for every outstanding load, the younger unit included)
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    const int slot_w = slot_a + 1 < 5 ? slot_a + 1 : slot_a - 4;
    const int s3 = slot_a + 3 < 5 ? slot_a + 3 : slot_a - 2;
    const int s4 = slot_a + 4 < 5 ? slot_a + 4 : slot_a - 1;
    compute(ring + slot_a * kUnit, ring + slot_w * kUnit, ring + s3 * kUnit + wave * GW * 512,
            kt + 1 < nk ? kt + 1 : -1, ring + s4 * kUnit + wave * 4 * 512, kt + 2 < nk ? kt + 2 : -1);
    slot_a = slot_a + 2 < 5 ? slot_a + 2 : slot_a - 3;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the filler loads have landed before the LDS is given back

  const int col_in = lane & 31, row_in = (lane >> 5) * 4;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int j = 0; j < TNF; ++j) {
      const int col = n0 + wn * (BN / 2) + j * 32 + col_in;
      if (col >= N) continue;
      store_block<EPI, C_BF16>(acc[i][j], layer_ptr<C_BF16>(Cv, (size_t)tc.layer * sC), R ? R + (size_t)tc.layer * sR : nullptr,
                               m0 + wm * 64 + i * 32, row_in, col, M, N);
    }
  }
}

// The same load written out (m0 = LDS base of the wave's 1 KB, lane i's 16 bytes land at base + 16 i): the compiler does
// not know of it, so it adds no waits of its own and the counted s_waitcnt of the loop below is the only one.  (Behind
// the builtin it makes LDS reads wait for every outstanding load whose ring slot it cannot tell from theirs.)
#define SNLP_GLDS16_ASM(gptr, lptr)                                                                          \
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"                               \
               :: "v"(gptr), "s"((uint32_t)(size_t)((__attribute__((address_space(3))) char*)(lptr)))        \
               : "memory", "m0")

// A piece of 128 x BN outputs (BN = 128 or 64) of the last, incomplete round of a launch (see TileRange): 8 waves as
// 4 x 2, wave tile 32 x BN/2, same k-ordered MFMA sequence per output element as every other tile shape.  A piece
// moves few bytes per k-tile (32 or 24 KB), so what bounds it is not the fill rate but how far ahead its operands are
// requested: in the five-unit ring above the weight unit of k-tile kt + 1 is requested during k-tile kt, and a
// k-tile cannot take less than that load's latency (about 1.1 us under load, which is what 256 x 64 and 128 x 64
// pieces both took per k-tile there; with the deeper ring a 128 x 64 piece takes 0.8 us).  Here the 160 KB hold D = 5 (128 x 128) or 6 (128 x 64) whole k-tiles, A rows
// then weight rows, and k-tile kt + D - 1 is requested while kt is multiplied.
template <int BM, int BN, int EPI, bool C_BF16>
__device__ __forceinline__ void ring_piece(const TileCoord tc, bf16_t* __restrict__ ring, const bf16_t* __restrict__ A, size_t sA,
                                           const bf16_t* __restrict__ Wt, size_t sW, void* Cv, size_t sC,
                                           const float* __restrict__ R, size_t sR, int M, int N, int K, int a_group) {
  static_assert(BM == 128 && (BN == 128 || BN == 64), "two piece shapes");
  constexpr int TNF = BN / 64;                    // 32-column MFMA tiles per wave
  constexpr int GA = BM / 64, GW = BN / 64;       // 1 KB row groups (8 rows) per wave of a k-tile's A and weight rows
  constexpr int kStage = (BM + BN) * kBK;         // elements of one k-tile in the ring
  constexpr int D = (5 * 256 * kBK) / kStage;     // k-tiles the ring holds
  A += (size_t)(tc.layer / a_group) * sA;
  Wt += (size_t)tc.layer * sW;
  const int m0 = tc.tm * BM, n0 = tc.tn * BN;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  const bf16_t* gsrcA[GA];
  const bf16_t* gsrcW[GW];
#pragma unroll
  for (int j = 0; j < GA; ++j) {
    const int row = (wave * GA + j) * 8 + (lane >> 3);
    const int chunk = (lane & 7) ^ ((row >> 1) & 7);
    int ra = m0 + row;
    ra = ra < M ? ra : M - 1;
    gsrcA[j] = A + (size_t)ra * K + chunk * 8;
  }
#pragma unroll
  for (int j = 0; j < GW; ++j) {
    const int row = (wave * GW + j) * 8 + (lane >> 3);
    const int chunk = (lane & 7) ^ ((row >> 1) & 7);
    int rw = n0 + row;
    rw = rw < N ? rw : N - 1;
    gsrcW[j] = Wt + (size_t)rw * K + chunk * 8;
  }
  const int nk = K / kBK;
  // Past the end of K every lane requests the operand's first 16 bytes instead (one sector, into a stage nobody reads
  // again), which keeps the number of loads per phase, and with it the wait count, the same in every phase.
  auto issue = [&](int kt, int stage) {
    bf16_t* da = ring + stage * kStage + wave * GA * 512;
    bf16_t* dw = ring + stage * kStage + BM * kBK + wave * GW * 512;
    const bool real = kt < nk;
#pragma unroll
    for (int j = 0; j < GA; ++j) SNLP_GLDS16_ASM(real ? gsrcA[j] + (size_t)kt * kBK : A, da + j * 512);
#pragma unroll
    for (int j = 0; j < GW; ++j) SNLP_GLDS16_ASM(real ? gsrcW[j] + (size_t)kt * kBK : Wt, dw + j * 512);
  };

  f32x16_t acc[TNF];
#pragma unroll
  for (int j = 0; j < TNF; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;

  const int sw = ((lane & 31) >> 1) & 7, hi = lane >> 5;
  const int rowoff = (lane & 31) * kBK;
#pragma unroll
  for (int t = 0; t < D - 1; ++t) issue(t, t);
  int stage = 0;   // stage of k-tile kt; k-tile kt + D - 1 goes to the stage before it
  for (int kt = 0; kt < nk; ++kt) {
    // this wave's part of k-tile kt has landed (loads return in order; those of the D - 2 k-tiles after it may still
    // be on their way); behind the barrier everyone's has, and everyone is done with k-tile kt - 1, whose stage the
    // loads of this phase refill
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"((D - 2) * (GA + GW)) : "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    issue(kt + D - 1, stage == 0 ? D - 1 : stage - 1);
    const bf16_t* ua = ring + stage * kStage;
    const bf16_t* uw = ua + BM * kBK;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int off = rowoff + (((ks * 2 + hi) ^ sw) << 3);
      const bf16x8_t af = *reinterpret_cast<const bf16x8_t*>(ua + wm * 32 * kBK + off);
#pragma unroll
      for (int j = 0; j < TNF; ++j) {
        const bf16x8_t bfr = *reinterpret_cast<const bf16x8_t*>(uw + (wn * (BN / 2) + j * 32) * kBK + off);
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bfr, acc[j], 0, 0, 0);
      }
    }
    stage = stage + 1 == D ? 0 : stage + 1;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the filler loads have landed before the LDS is given back

  const int col_in = lane & 31, row_in = (lane >> 5) * 4;
#pragma unroll
  for (int j = 0; j < TNF; ++j) {
    const int col = n0 + wn * (BN / 2) + j * 32 + col_in;
    if (col >= N) continue;
    store_block<EPI, C_BF16>(acc[j], layer_ptr<C_BF16>(Cv, (size_t)tc.layer * sC), R ? R + (size_t)tc.layer * sR : nullptr,
                             m0 + wm * 32, row_in, col, M, N);
  }
}

// Workgroups [0, head_tiles) take 256 x BN tiles in the launch's own order; with BNT != 0 the workgroups from
// head_tiles on take the BMT x BNT pieces of the big tiles in `tail` (the last, incomplete round of a launch of
// 256 x 256 tiles: in the same launch, so they start on the compute units the big tiles leave, with no kernel boundary
// in between).
template <int BN, int BMT, int BNT, int EPI, bool C_BF16>
__global__ __launch_bounds__(512) void k_gemm_bf16_256(const bf16_t* __restrict__ A, size_t sA,
                                                        const bf16_t* __restrict__ Wt, size_t sW, void* Cv, size_t sC,
                                                        const float* __restrict__ R, size_t sR, int M, int N, int K,
                                                        int tiles_m, int tiles_n, unsigned head_tiles, int a_group,
                                                        TileRange tail) {
  __shared__ __attribute__((aligned(16))) bf16_t ring[5 * 256 * kBK];
  TileCoord tc;
  if (blockIdx.x < head_tiles) {                  // uniform over the workgroup
    tc = map_tile(blockIdx.x, head_tiles, tiles_m, tiles_n);
    if (BN == 256 && BMT == 256 && BNT == 128 && tc.tn * 256 + 128 >= N) {
      // the last column tile of a matrix whose width is an odd multiple of 128 is half empty: it runs as a half
      // (where the launch carries that body anyway)
      tc.tn *= 2;
      ring_tile<(BMT == 256 && BNT == 128 ? 128 : BN), EPI, C_BF16>(tc, ring, A, sA, Wt, sW, Cv, sC, R, sR, M, N, K, a_group);
      return;
    }
    ring_tile<BN, EPI, C_BF16>(tc, ring, A, sA, Wt, sW, Cv, sC, R, sR, M, N, K, a_group);
    return;
  }
  if (BNT != 0) {
    constexpr int PM = BNT != 0 ? BMT : 256, PN = BNT != 0 ? BNT : 256;
    if (!map_tail_tile<PM, PN>(blockIdx.x - head_tiles, tail, M, N, tc)) return;   // whole workgroup
    if constexpr (PM == 128) ring_piece<PM, PN, EPI, C_BF16>(tc, ring, A, sA, Wt, sW, Cv, sC, R, sR, M, N, K, a_group);
    else ring_tile<PN, EPI, C_BF16>(tc, ring, A, sA, Wt, sW, Cv, sC, R, sR, M, N, K, a_group);
  }
}

constexpr TileRange kWholeGemm = {0u, 0u, 0, 0, 0};

// BNT = 0: the whole GEMM in 256 x BN tiles.  Else (BN = 256): big tiles [0, tail.first) whole, then the BMT x BNT
// pieces of `tail`.
template <int BN, int BMT = 256, int BNT = 0>
hipError_t launch_ring(hipStream_t s, int Lc, int M, int N, int K, const bf16_t* A, size_t sA, const bf16_t* Wt, size_t sW,
                       void* C, size_t sC, bool c_bf16, int epi, const float* R, size_t sR, int a_group,
                       TileRange tail = kWholeGemm) {
  const int tiles_m = (M + 255) / 256, tiles_n = (N + BN - 1) / BN;
  const unsigned head = BNT ? tail.first : (unsigned)Lc * tiles_m * tiles_n;
  const unsigned total = head + (BNT ? (tail.count + 7) / 8 * 8 * (unsigned)tail.parts : 0u);
  dim3 grid(total), block(512);
#define SNLP_GEMM256_LAUNCH(EPI_, CB_)                                                                               \
  hipLaunchKernelGGL((k_gemm_bf16_256<BN, BMT, BNT, EPI_, CB_>), grid, block, 0, s, A, sA, Wt, sW, C, sC, R, sR, M, N, K, tiles_m, \
                     tiles_n, head, a_group, tail)
  if (epi == EPI_STORE && c_bf16) SNLP_GEMM256_LAUNCH(EPI_STORE, true);
  else if (epi == EPI_STORE) SNLP_GEMM256_LAUNCH(EPI_STORE, false);
  else if (epi == EPI_RELU2 && c_bf16) SNLP_GEMM256_LAUNCH(EPI_RELU2, true);
  else if (epi == EPI_ADD_F32 && !c_bf16) SNLP_GEMM256_LAUNCH(EPI_ADD_F32, false);
  else return hipErrorInvalidValue;
#undef SNLP_GEMM256_LAUNCH
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Skinny GEMM for M <= 128 (decode-shaped blocks): a weight-streaming kernel.  Weights are repacked once
// into MFMA operand order, [N/32][K/16][64 lanes][8]: lane = (n % 32) + 32 * ((k % 16) / 8) holds
// W[k .. k+7][n], so one wave-level 16-byte load is 1 KB of contiguous memory and a wave walks a contiguous
// stream of K/16 such chunks straight into operand registers (no LDS, no barrier on the weight path), DEPTH
// k-steps in flight.  The small A tile (tokens x 64 k) is shared by the NW waves through a ring of four LDS
// buffers: it is requested four k-tiles ahead into registers and written to LDS two tiles ahead, behind the
// MFMAs of the current tile.  The per-tile barrier is a bare s_barrier after an explicit LDS wait:
// __syncthreads() would also wait for every outstanding global load and drain the weight queue at each tile.
// A workgroup owns one row tile of BM = 32 TM rows (all rows when M <= BM) and each of its waves TN blocks of 32
// output columns (BN = 32 TN NW), so an A fragment read from LDS
// serves TN MFMAs and the layer's A is re-read from L2 by N / BN workgroups instead of N / 128; k runs in
// order for every TN, so results depend neither on the layer count nor on the tile width.  Measured: time is
// close to (weight bytes + re-read A bytes) / 6-7 TB/s.
// One wave's share of a skinny-GEMM workgroup: TN column blocks from block nb0 on, all BM rows.  The waves of a
// workgroup may run this with different TN (the staging of the token tile and the barriers do not depend on it).
template <int TM, int TN, int NW, int DEPTH, int EPI, bool C_BF16>
__device__ __forceinline__ void skinny_wave(const bf16_t* __restrict__ A, const bf16_t* __restrict__ Wp, void* Cv, size_t sC,
                                            const float* __restrict__ R, size_t sR, int M, int N, int K, int layer, int m0,
                                            int nb0, bf16_t* lds) {
  constexpr int BM = 32 * TM;
  constexpr int NT = 64 * NW;
  constexpr int TILE = BM * kLdsRow;                 // one staged A tile, elements
  constexpr int PA = (BM * 8 + NT - 1) / NT;         // 16-byte A chunks per thread per k-tile
  static_assert(DEPTH == 8 || DEPTH == 16, "weight queue holds 2 or 4 whole k-tiles");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nk = K / kBK, nsteps = nk * 4;

  // weight streams of this wave: TN column blocks nb0 .. nb0+TN-1 (clamped: a block past the last one streams the
  // last one and stores nothing), 512 elements (1 KB) per k-step each
  const int nblocks = N / 32;
  const bf16x8_t* wsrc[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int nb = nb0 + j < nblocks ? nb0 + j : nblocks - 1;
    wsrc[j] = reinterpret_cast<const bf16x8_t*>(Wp + (size_t)nb * nsteps * 512) + lane;
  }

  // A staging: chunk index c = tid + p NT over (row, 16-byte chunk); indices past the tile repeat its last chunk
  // (written twice with the same data), rows past M are clamped
  const u32x4_t* gA[PA];
  int aoff[PA];
#pragma unroll
  for (int p = 0; p < PA; ++p) {
    int c = tid + p * NT;
    c = c < BM * 8 ? c : BM * 8 - 1;
    const int r = c >> 3, chunk = c & 7;
    aoff[p] = r * kLdsRow + chunk * 8;
    const int rg = m0 + r < M ? m0 + r : M - 1;
    gA[p] = reinterpret_cast<const u32x4_t*>(A + (size_t)rg * K) + chunk;
  }
  auto load_a = [&](u32x4_t (&ra)[PA], int kt) {
    kt = kt < nk ? kt : nk - 1;
#pragma unroll
    for (int p = 0; p < PA; ++p) ra[p] = gA[p][kt * (kBK / 8)];
  };
  auto write_a = [&](bf16_t* buf, const u32x4_t (&ra)[PA]) {
#pragma unroll
    for (int p = 0; p < PA; ++p) *reinterpret_cast<u32x4_t*>(buf + aoff[p]) = ra[p];
  };
  auto lds_fence_barrier = [&]() {
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0) only: this thread's LDS writes (and reads) are done
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };
  bf16_t* const buf0 = lds;
  bf16_t* const buf1 = lds + TILE;
  bf16_t* const buf2 = lds + 2 * TILE;
  bf16_t* const buf3 = lds + 3 * TILE;

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  bf16x8_t wq[DEPTH][TN];
#pragma unroll
  for (int s = 0; s < DEPTH; ++s)
#pragma unroll
    for (int j = 0; j < TN; ++j) wq[s][j] = __builtin_nontemporal_load(wsrc[j] + (size_t)(s < nsteps ? s : nsteps - 1) * 64);
  u32x4_t ra0[PA], ra1[PA];
  // A tiles are requested four tiles ahead and reach LDS two tiles ahead.  Loads complete in issue order, so a
  // wait for an A tile also waits for every weight load issued before it: with this lead those are weights the
  // MFMAs need by then anyway, and the A wait never shortens the weight queue.
  load_a(ra0, 0);
  load_a(ra1, 1);
  write_a(buf0, ra0);
  write_a(buf1, ra1);
  load_a(ra0, 2);
  load_a(ra1, 3);
  lds_fence_barrier();

  const int frag_off = (lane & 31) * kLdsRow + (lane >> 5) * 8;
  // A fragments run two k-steps ahead of the MFMAs that use them, across tile boundaries too: the next tile's
  // buffer was completed and fenced one tile earlier, so its first fragments are read behind the last MFMAs of
  // the current tile and no tile starts with an LDS round trip.
  bf16x8_t af0[TM], af1[TM];
  auto read_frags = [&](bf16x8_t (&f)[TM], const bf16_t* buf, int ks) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
      f[i] = *reinterpret_cast<const bf16x8_t*>(buf + frag_off + i * 32 * kLdsRow + ks * 16);
  };
  auto step = [&](bf16x8_t (&f)[TM], int kt, int slot) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[i], wq[slot][j], acc[i][j], 0, 0, 0);
    // refill after the MFMAs that read the slot, so the load lands in the same registers: a load issued
    // before them needs a second register set, and the copy back at the loop end waits for the whole queue
    int nx = kt * 4 + (slot & 3) + DEPTH;
    nx = nx < nsteps ? nx : nsteps - 1;
#pragma unroll
    for (int j = 0; j < TN; ++j) wq[slot][j] = __builtin_nontemporal_load(wsrc[j] + (size_t)nx * 64);
  };
  // One k-tile: multiply from `cur`; the tile two ahead (already in registers) goes to `wr` behind the first
  // MFMAs and the registers are refilled with the tile four ahead; `nxt` is the buffer of the next tile.
  auto tile = [&](const bf16_t* cur, const bf16_t* nxt, bf16_t* wr, u32x4_t (&ra)[PA], int kt, int slot0) {
    step(af0, kt, slot0 + 0);
    read_frags(af0, cur, 2);
    __builtin_amdgcn_sched_barrier(0);
    write_a(wr, ra);
    load_a(ra, kt + 4);
    step(af1, kt, slot0 + 1);
    read_frags(af1, cur, 3);
    __builtin_amdgcn_sched_barrier(0);
    step(af0, kt, slot0 + 2);
    read_frags(af0, nxt, 0);
    __builtin_amdgcn_sched_barrier(0);
    step(af1, kt, slot0 + 3);
    read_frags(af1, nxt, 1);
    __builtin_amdgcn_sched_barrier(0);
    lds_fence_barrier();
  };
  read_frags(af0, buf0, 0);
  read_frags(af1, buf0, 1);
  constexpr int QT = DEPTH / 4;   // tiles in the weight queue: 2 or 4
  int kt = 0;
  for (; kt + 4 <= nk; kt += 4) {   // branch-free body: the wait counts stay exact across the back edge
    tile(buf0, buf1, buf2, ra0, kt, (0 % QT) * 4);
    tile(buf1, buf2, buf3, ra1, kt + 1, (1 % QT) * 4);
    tile(buf2, buf3, buf0, ra0, kt + 2, (2 % QT) * 4);
    tile(buf3, buf0, buf1, ra1, kt + 3, (3 % QT) * 4);
  }
  if (kt < nk) tile(buf0, buf1, buf2, ra0, kt, (0 % QT) * 4);
  if (kt + 1 < nk) tile(buf1, buf2, buf3, ra1, kt + 1, (1 % QT) * 4);
  if (kt + 2 < nk) tile(buf2, buf3, buf0, ra0, kt + 2, (2 % QT) * 4);

  const int row_in = (lane >> 5) * 4;
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    if (nb0 + j >= nblocks) break;
    const int col = (nb0 + j) * 32 + (lane & 31);
    if (EPI == EPI_ADD_F32 && m0 + BM <= M) {
      // full tile: every residual load goes out before the first store (one memory round trip per column block)
      const float* Rl = R + (size_t)layer * sR + (size_t)(m0 + row_in) * N + col;
      float* Cl = reinterpret_cast<float*>(Cv) + (size_t)layer * sC + (size_t)(m0 + row_in) * N + col;
      float v[TM][16];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) v[i][r] = Rl[(size_t)(i * 32 + (r >> 2) * 8 + (r & 3)) * N];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) Cl[(size_t)(i * 32 + (r >> 2) * 8 + (r & 3)) * N] = v[i][r] + acc[i][j][r];
      continue;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      store_block<EPI, C_BF16>(acc[i][j], layer_ptr<C_BF16>(Cv, (size_t)layer * sC), R ? R + (size_t)layer * sR : nullptr,
                               m0 + i * 32, row_in, col, M, N);
    }
  }
}

// TN_HI column blocks for the first NH waves, TN_LO for the others (NH = NW: all alike): a workgroup owns
// NH TN_HI + (NW - NH) TN_LO consecutive column blocks, which lets the column tile follow N * layers / compute units
// more closely than a multiple of NW blocks would.
template <int TM, int TN_HI, int TN_LO, int NH, int NW, int DEPTH, int EPI, bool C_BF16>
__global__ __launch_bounds__(64 * NW, TN_HI == 1 ? 2 : 1) void k_gemm_skinny(const bf16_t* __restrict__ A, size_t sA,
                                                                        const bf16_t* __restrict__ Wp, size_t sW, void* Cv,
                                                                        size_t sC, const float* __restrict__ R, size_t sR,
                                                                        int M, int N, int K, int tiles_m, int tiles_n,
                                                                        unsigned total_tiles, int a_group, int touch_a) {
  constexpr int BM = 32 * TM;
  constexpr int TILE = BM * kLdsRow;
  constexpr int BLOCKS = NH * TN_HI + (NW - NH) * TN_LO;   // column blocks per workgroup
  __shared__ __attribute__((aligned(16))) bf16_t lds[4 * TILE];   // ring of four A tiles

  // XCD-aware order: consecutive logical tiles (same layer and row tile, neighbouring columns: same A) on one XCD
  const unsigned q = total_tiles / 8, rr = total_tiles % 8;
  const unsigned xcd = blockIdx.x % 8, local = blockIdx.x / 8;
  const unsigned t = xcd * q + (xcd < rr ? xcd : rr) + local;
  const unsigned per_layer = (unsigned)tiles_m * (unsigned)tiles_n;
  const int layer = (int)(t / per_layer);
  const int tm = (int)((t % per_layer) / (unsigned)tiles_n), tn = (int)(t % (unsigned)tiles_n);
  const int m0 = tm * BM;   // first row of this workgroup's row tile
  A += (size_t)(layer / a_group) * sA;
  Wp += (size_t)layer * sW;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // The token tile of a layer is read k-tile by k-tile, 128 bytes of each of its rows at a time, by all the workgroups
  // of the layer (one XCD, see above): whoever asks first brings the line in from DRAM, and under the saturated weight
  // stream such single-line reads, each in a DRAM row of its own, come back late (the decode attention kernel shows the
  // same with its block rows).  So before it starts streaming, every workgroup reads one word of each line of its share
  // of the layer's token rows -- whole rows, at a moment when the memory system is idle -- and the k-tile loads then
  // hit in L2.  d20 decode: QKV 48.9 -> 43.7 us, FC 62.3 -> 55.8, O 25.4 -> 24.3; PROJ unchanged (its token tile was
  // written by the FC launch on the same XCD and is still in that L2).  The words are read and dropped.  Only in
  // launches that stream enough weights to saturate the memory system (the launcher's flag): one layer alone loses
  // half a microsecond to it.
  unsigned touched = 0;
  if (touch_a) {
    const int lines_per_row = K / 64;                          // 128-byte lines of a token row
    const int rows = M - m0 < BM ? M - m0 : BM;
    const int total = rows * lines_per_row;
    const int lo = (int)((long)total * tn / tiles_n), hi = (int)((long)total * (tn + 1) / tiles_n);
    for (int ln = lo + (int)threadIdx.x; ln < hi; ln += 64 * NW) {
      const int r = ln / lines_per_row, c = ln % lines_per_row;
      touched ^= *reinterpret_cast<const unsigned*>(A + (size_t)(m0 + r) * K + c * 64);
    }
  }
  if (NH == NW || wave < NH)
    skinny_wave<TM, TN_HI, NW, DEPTH, EPI, C_BF16>(A, Wp, Cv, sC, R, sR, M, N, K, layer, m0, tn * BLOCKS + wave * TN_HI, lds);
  else
    skinny_wave<TM, TN_LO, NW, DEPTH, EPI, C_BF16>(A, Wp, Cv, sC, R, sR, M, N, K, layer, m0,
                                                   tn * BLOCKS + NH * TN_HI + (wave - NH) * TN_LO, lds);
  asm volatile("" :: "v"(touched));   // keeps the touching loads
}

// [L][K][N] row-major -> operand order [L][N/32][K/16][64][8]
__global__ __launch_bounds__(kThreads) void k_repack_operand_order(const bf16_t* __restrict__ in, bf16_t* __restrict__ out,
                                                                    int K, int N) {
  const size_t lo = (size_t)blockIdx.z * K * N;
  const int nb = blockIdx.x, k16 = blockIdx.y * 4 + (threadIdx.x >> 6);
  if (k16 >= K / 16) return;
  const int lane = threadIdx.x & 63;
  const int n = nb * 32 + (lane & 31), k0 = k16 * 16 + (lane >> 5) * 8;
  bf16_t v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = in[lo + (size_t)(k0 + e) * N + n];
  bf16_t* dst = out + lo + (((size_t)nb * (K / 16) + k16) * 64 + lane) * 8;
#pragma unroll
  for (int e = 0; e < 8; ++e) dst[e] = v[e];
}

template <int TM, int TN, int NW, int DEPTH, int TN_LO = TN, int NH = NW>
hipError_t launch_skinny(hipStream_t s, int Lc, int M, int N, int K, const bf16_t* A, size_t sA, const bf16_t* Wp,
                         size_t sW, void* C, size_t sC, bool c_bf16, int epi, const float* R, size_t sR, int a_group) {
  constexpr int BLOCKS = NH * TN + (NW - NH) * TN_LO;   // 32-column blocks per workgroup
  const int tiles_n = (N + 32 * BLOCKS - 1) / (32 * BLOCKS), tiles_m = (M + 32 * TM - 1) / (32 * TM);
  const unsigned total = (unsigned)Lc * tiles_m * tiles_n;
  const int touch_a = (size_t)Lc * N * K * sizeof(bf16_t) >= ((size_t)32 << 20) ? 1 : 0;   // see k_gemm_skinny
  dim3 grid(total), block(64 * NW);
#define SNLP_SKINNY_LAUNCH(EPI_, CB_)                                                                           \
  hipLaunchKernelGGL((k_gemm_skinny<TM, TN, TN_LO, NH, NW, DEPTH, EPI_, CB_>), grid, block, 0, s, A, sA, Wp, sW, C, sC, R, sR, \
                     M, N, K, tiles_m, tiles_n, total, a_group, touch_a)
  if (epi == EPI_STORE && c_bf16) SNLP_SKINNY_LAUNCH(EPI_STORE, true);
  else if (epi == EPI_STORE) SNLP_SKINNY_LAUNCH(EPI_STORE, false);
  else if (epi == EPI_RELU2 && c_bf16) SNLP_SKINNY_LAUNCH(EPI_RELU2, true);
  else if (epi == EPI_ADD_F32 && !c_bf16) SNLP_SKINNY_LAUNCH(EPI_ADD_F32, false);
  else return hipErrorInvalidValue;
#undef SNLP_SKINNY_LAUNCH
  return hipGetLastError();
}

template <int TM>
hipError_t launch_skinny_tm(hipStream_t s, int Lc, int M, int N, int K, const bf16_t* A, size_t sA, const bf16_t* Wp,
                            size_t sW, void* C, size_t sC, bool c_bf16, int epi, const float* R, size_t sR, int a_group) {
  // Four waves per workgroup share one staged A tile.  Every workgroup of a layer re-reads the layer's A from L2,
  // and those re-reads cost as much as weight bytes, so a wave takes TN column blocks (a workgroup 128 TN columns)
  // when that still leaves enough workgroups for the 256 CUs in one round (wide tiles run one workgroup per CU).
  // The choice follows the launch size: an output element is the same k-ordered sum for every TN, so a layer
  // gives the same bits evaluated alone or in the batch.  (Two k-halves per workgroup, 2- and 8-wave workgroups
  // and an 8-deep queue for TN = 1 were measured and were no faster.)
  // A launch with few workgroups (one layer of the sequential path, the last rounds that leave converged layers
  // out) is cut finer instead: halve the rows per workgroup, then the columns (2 waves, then 1), until there are
  // at least 128 workgroups.  With 10-40 workgroups each streams its share at the rate of ONE CU (one layer's PROJ
  // on 10 CUs: 50 us for 13 MB); the re-reads that finer tiles add come from L2, which has bandwidth to spare
  // when so few CUs pull.  Every output element stays the same k-ordered sum, so results do not depend on the cut.
  {
    auto count = [&](int rows, int nw) { return (long)Lc * ((M + rows - 1) / rows) * ((N + 32 * nw - 1) / (32 * nw)); };
    if (count(32 * TM, 4) < 128) {
      // halve the larger of the two operand shares; rows first on a tie: (128,128) (64,128) (64,64) (32,64) (32,32)
      if (TM == 4 && count(64, 4) >= 128)
        return launch_skinny<2, 1, 4, 16>(s, Lc, M, N, K, A, sA, Wp, sW, C, sC, c_bf16, epi, R, sR, a_group);
      if (TM >= 2 && count(64, 2) >= 128)
        return launch_skinny<2, 1, 2, 16>(s, Lc, M, N, K, A, sA, Wp, sW, C, sC, c_bf16, epi, R, sR, a_group);
      if (count(32, 2) >= 128)
        return launch_skinny<1, 1, 2, 16>(s, Lc, M, N, K, A, sA, Wp, sW, C, sC, c_bf16, epi, R, sR, a_group);
      return launch_skinny<1, 1, 1, 16>(s, Lc, M, N, K, A, sA, Wp, sW, C, sC, c_bf16, epi, R, sR, a_group);
    }
  }
  // Column tiles that follow the launch: with wpl = 256 / layers workgroups per layer the 256 compute units take one
  // workgroup each, so a workgroup should own ceil(blocks / wpl) column blocks.  Where that is 9 or 10 blocks (d20
  // QKV: 120 blocks, 12 workgroups per layer instead of 10 of 12 blocks) or 13 or 14 (d20 FC: 160 blocks, 12 workgroups
  // instead of 10 of 16), the waves of a workgroup take unequal shares: 3 3 2 2, or 2 2 2 2 2 2 1 1 with eight waves.
  // Fewer weight bytes per compute unit at the same token-tile bytes, and 240 compute units busy instead of 200.
  if (TM >= 2 && Lc <= 256) {
    const int nblocks = N / 32, wpl = 256 / Lc;
    const int want = (nblocks + wpl - 1) / wpl;
    const long wgs10 = (long)Lc * ((nblocks + 9) / 10), wgs14 = (long)Lc * ((nblocks + 13) / 14);
    if ((want == 9 || want == 10) && wgs10 >= 180 && wgs10 <= 256)
      return launch_skinny<TM, 3, 4, 8, 2, 2>(s, Lc, M, N, K, A, sA, Wp, sW, C, sC, c_bf16, epi, R, sR, a_group);
    if ((want == 13 || want == 14) && wgs14 >= 180 && wgs14 <= 256)
      return launch_skinny<TM, 2, 8, 8, 1, 6>(s, Lc, M, N, K, A, sA, Wp, sW, C, sC, c_bf16, epi, R, sR, a_group);
  }
  int tn_pick = 1;
  for (int tn = 4; tn >= 2; --tn) {
    const long wgs = (long)Lc * ((N + 128 * tn - 1) / (128 * tn));
    if (wgs >= 180 && wgs <= 256) { tn_pick = tn; break; }
  }
  // 512 columns: eight waves of two column blocks measured slightly better than four waves of four
  if (TM >= 2 && tn_pick == 4) return launch_skinny<TM, 2, 8, 8>(s, Lc, M, N, K, A, sA, Wp, sW, C, sC, c_bf16, epi, R, sR, a_group);
  if (TM >= 2 && tn_pick == 3) return launch_skinny<TM, 3, 4, 8>(s, Lc, M, N, K, A, sA, Wp, sW, C, sC, c_bf16, epi, R, sR, a_group);
  if (TM >= 2 && tn_pick == 2) return launch_skinny<TM, 2, 4, 8>(s, Lc, M, N, K, A, sA, Wp, sW, C, sC, c_bf16, epi, R, sR, a_group);
  return launch_skinny<TM, 1, 4, 16>(s, Lc, M, N, K, A, sA, Wp, sW, C, sC, c_bf16, epi, R, sR, a_group);
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
hipError_t launch_tile(hipStream_t s, int Lc, int M, int N, int K, const bf16_t* A, size_t sA, const bf16_t* Wt,
                       size_t sW, void* C, size_t sC, bool c_bf16, int epi, const float* R, size_t sR, int a_group) {
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  const unsigned total = (unsigned)Lc * tiles_m * tiles_n;
  dim3 grid(total), block(kThreads);
#define SNLP_GEMM_LAUNCH(EPI_, CB_)                                                                              \
  hipLaunchKernelGGL((k_gemm_bf16<BM, BN, WAVES_M, WAVES_N, EPI_, CB_>), grid, block, 0, s, A, sA, Wt, sW, C, sC, \
                     R, sR, M, N, K, tiles_m, tiles_n, total, a_group)
  if (epi == EPI_STORE && c_bf16) SNLP_GEMM_LAUNCH(EPI_STORE, true);
  else if (epi == EPI_STORE) SNLP_GEMM_LAUNCH(EPI_STORE, false);
  else if (epi == EPI_RELU2 && c_bf16) SNLP_GEMM_LAUNCH(EPI_RELU2, true);
  else if (epi == EPI_ADD_F32 && !c_bf16) SNLP_GEMM_LAUNCH(EPI_ADD_F32, false);
  else return hipErrorInvalidValue;
#undef SNLP_GEMM_LAUNCH
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_f32(hipStream_t s, int Lc, int M, int N, int K, const float* A, size_t sA, const float* W,
                           size_t sW, float* C, size_t sC, int epi, const float* R, size_t sR, int a_group) {
  dim3 grid((N + 63) / 64, (M + 63) / 64, Lc), block(kThreads);
  switch (epi) {
    case EPI_STORE: hipLaunchKernelGGL(k_gemm_f32<EPI_STORE>, grid, block, 0, s, A, sA, W, sW, C, sC, R, sR, M, N, K, a_group); break;
    case EPI_RELU2: hipLaunchKernelGGL(k_gemm_f32<EPI_RELU2>, grid, block, 0, s, A, sA, W, sW, C, sC, R, sR, M, N, K, a_group); break;
    case EPI_ADD_F32: hipLaunchKernelGGL(k_gemm_f32<EPI_ADD_F32>, grid, block, 0, s, A, sA, W, sW, C, sC, R, sR, M, N, K, a_group); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

bool gemm_bf16_supported(int M, int N, int K) {
  return M >= 1 && N >= 64 && N % 64 == 0 && K >= 4 * kBK && K % kBK == 0;
}

bool gemm_bf16_operand_order(int M) { return M <= 128; }

hipError_t launch_repack_weights(hipStream_t s, const bf16_t* in, bf16_t* out, int L, int K, int N, int M) {
  if (!gemm_bf16_supported(M, N, K)) return hipErrorInvalidValue;
  if (gemm_bf16_operand_order(M)) {
    dim3 grid(N / 32, (K / 16 + 3) / 4, L), block(kThreads);
    hipLaunchKernelGGL(k_repack_operand_order, grid, block, 0, s, in, out, K, N);
    return hipGetLastError();
  }
  return launch_transpose_bf16(s, in, out, L, K, N);
}

// The choice of kernel and tile shape follows the launch size (layers included); an output element's k-ordered MFMA
// sequence and epilogue are the same in all of them, so a layer's result does not depend on how many layers share the
// launch (tested bit for bit: K = L rounds against the one-layer launches of the sequential forward).
hipError_t launch_gemm_bf16(hipStream_t s, int Lc, int M, int N, int K, const bf16_t* A, size_t sA, const bf16_t* W,
                            size_t sW, void* C, size_t sC, bool c_bf16, int epi, const float* R, size_t sR, int a_group) {
  if (!gemm_bf16_supported(M, N, K)) return hipErrorInvalidValue;
  if (M <= 32) return launch_skinny_tm<1>(s, Lc, M, N, K, A, sA, W, sW, C, sC, c_bf16, epi, R, sR, a_group);
  if (M <= 64) return launch_skinny_tm<2>(s, Lc, M, N, K, A, sA, W, sW, C, sC, c_bf16, epi, R, sR, a_group);
  if (M <= 128) return launch_skinny_tm<4>(s, Lc, M, N, K, A, sA, W, sW, C, sC, c_bf16, epi, R, sR, a_group);
  // Both tiled kernels run the same k-ordered sequence of 32 x 32 x 16 MFMAs per output element, so their
  // results are bit-identical and the choice may follow the launch size.  The 256 x 256 kernel (one 8-wave
  // workgroup per CU) needs about three rounds of workgroups behind its ramp and tail; with fp32 output and a
  // short k loop its unoverlapped epilogue costs more than the 128 x 128 kernel's extra LDS traffic unless
  // there are many rounds.  (Measured on the d12, d20 and d26 prefill shapes.)
  const int big_m = (M + 255) / 256, big_n = (N + 255) / 256;
  const long tiles256 = (long)Lc * big_m * big_n;
  // Whole rounds of 256 x 256 tiles with the last, incomplete round cut smaller in the same launch (see TileRange),
  // where that is worth about 2 % of the launch or more: as 128 x 64 pieces (r <= 32) the round takes a little under
  // half of a full one, as 128 x 128 pieces (r <= 64) a little over half, as halves (r <= 128) three quarters.
  // Measured: d20 HCN PROJ (800 tiles, r = 32) 588 -> 490 us, O 171 -> 149, QKV (r = 96) 411 -> 405; d12 PROJ (288
  // tiles, before: 576 tiles of 256 x 128) 184 -> 132, O (before: 128 x 128 tiles) 55 -> 48; d26 PROJ (r = 96 of 2912)
  // 2292 -> 2217; launches of 33 and 43 rounds (d26 QKV, FC) gained nothing from halves and keep the plain form.
  if (K >= 128 && M >= 512 && N >= 512 && tiles256 >= 256) {
    const unsigned r = (unsigned)(tiles256 % 256), head = (unsigned)(tiles256 - r);
    const long rounds = (tiles256 + 255) / 256;
    if (r > 0 && r <= 32 && rounds <= 24)
      return launch_ring<256, 128, 64>(s, Lc, M, N, K, A, sA, W, sW, C, sC, c_bf16, epi, R, sR, a_group,
                                       TileRange{head, r, big_m, big_n, 8});
    if (r > 0 && r <= 64 && rounds <= 20)
      return launch_ring<256, 128, 128>(s, Lc, M, N, K, A, sA, W, sW, C, sC, c_bf16, epi, R, sR, a_group,
                                        TileRange{head, r, big_m, big_n, 4});
    if (r > 0 && r <= 128 && rounds <= 12)
      return launch_ring<256, 256, 128>(s, Lc, M, N, K, A, sA, W, sW, C, sC, c_bf16, epi, R, sR, a_group,
                                        TileRange{head, r, big_m, big_n, 2});
  }
  if (K >= 128 && M >= 512 && N >= 512 && tiles256 >= 768 && (c_bf16 || K >= 1024 || tiles256 >= 2048)) {
    // a width that ends in a half-empty column tile (d26 QKV: 19.5 tiles) takes the launch that carries the
    // 256 x 128 body, with no tail pieces, so that those tiles run as halves
    if (N % 256 != 0 && N % 256 <= 128)
      return launch_ring<256, 256, 128>(s, Lc, M, N, K, A, sA, W, sW, C, sC, c_bf16, epi, R, sR, a_group,
                                        TileRange{(unsigned)tiles256, 0u, big_m, big_n, 2});
    return launch_ring<256>(s, Lc, M, N, K, A, sA, W, sW, C, sC, c_bf16, epi, R, sR, a_group);
  }
  // Too few 256 x 256 tiles: 256 x 128 tiles of the same kernel when they give the CUs about one round or more
  // (one layer of the sequential path at prefill sizes, narrow outputs; as above not for fp32 output behind a short
  // k loop), else 128 x 128 tiles.  Measured: one d20 layer's QKV 31 -> 27 us, d26 PROJ 116 -> 104, d12 batched PROJ
  // 192 -> 181 us.
  const long tiles128w = (long)Lc * ((M + 255) / 256) * ((N + 127) / 128);
  if (K >= 128 && M >= 512 && N >= 256 && tiles128w >= 200 && (c_bf16 || K >= 1024))
    return launch_ring<128>(s, Lc, M, N, K, A, sA, W, sW, C, sC, c_bf16, epi, R, sR, a_group);
  return launch_tile<128, 128, 2, 2>(s, Lc, M, N, K, A, sA, W, sW, C, sC, c_bf16, epi, R, sR, a_group);
}

}  // namespace snlp

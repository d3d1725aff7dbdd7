// Layer-batched attention of the SNLP evaluation step (Eq. (4)): for every layer l in the launch, batch
// element b and head h,   o = softmax(q k^T / sqrt(dh)) v   over [KV prefix (P rows, all visible) ;
// this block's rows t' <= t], q/k/v being the (rotated, normalised) thirds of qkv[l] and the prefix the
// read-only cache of layer l.  (Attn_l(Q_l h, K_l h, V_l h) of the Appendix "Fused Cross-Layer Coupling".)
//
// bf16 path (head_dim 128): MFMAs on TRANSPOSED products so that a lane owns one query column in both
// S^T = K Q^T and O^T = V^T P^T: the softmax statistics and the rescaling of O are lane-local, and the
// probabilities leave the S^T accumulators already in the operand layout of the second product.  V tiles sit
// in LDS as loaded ([key][dh], chunk-swizzled); the V^T operand comes out of them with the LDS transpose read
// (ds_read_b64_tr_b16); online softmax in fp32 (base 2, the hardware exponential).
//   * block kernel (T > 16): a workgroup owns 128 query rows, its 4 waves 32 each (v_mfma_f32_32x32x16_bf16),
//     sharing K / V steps of 32 keys that arrive by direct-to-LDS loads two steps ahead; three workgroups per
//     compute unit.
//   * decode kernel (T <= 16): a workgroup owns one (layer, sequence, head); its 4 waves split the key
//     tiles (v_mfma_f32_16x16x32_bf16: 16 query columns are all a decode block has), stream K straight into MFMA
//     operand registers and V through wave-private LDS, and merge their partial softmax states in a fixed order.
// Results for a (layer, b, h) never depend on how many layers are in the launch.
#include "snlp_kernels.hpp"

namespace snlp {

namespace {

constexpr int kThreads = 256;
constexpr int kWave = 64;

// ------------------------------------------------------------------------------------------------
// fp32 path: one wave per (token row, head); scores staged in LDS.
__global__ __launch_bounds__(kWave) void k_attn_f32(const float* __restrict__ qkv, const float* __restrict__ Kpre,
                                                     const float* __restrict__ Vpre, float* __restrict__ out, int l0,
                                                     int M, int T, int P, int B, int H, int dh, int d) {
  extern __shared__ float shm[];   // [dh] query, then [P + T] scores
  float* sq = shm;
  float* sc = shm + dh;
  const int row = blockIdx.x, h = blockIdx.y, l = l0 + blockIdx.z;
  const int b = row / T, t = row % T;
  const int lane = threadIdx.x;
  const int nkeys = P + t + 1;
  const float* qkv_l = qkv + (size_t)(l - 1) * M * 3 * d;
  const float* qp = qkv_l + (size_t)row * 3 * d + (size_t)h * dh;
  for (int c = lane; c < dh; c += kWave) sq[c] = qp[c];
  __syncthreads();
  const float* kpre = Kpre ? Kpre + (((size_t)(l - 1) * B + b) * H + h) * (size_t)P * dh : nullptr;
  const float* vpre = Vpre ? Vpre + (((size_t)(l - 1) * B + b) * H + h) * (size_t)P * dh : nullptr;
  const float scale = 1.0f / sqrtf((float)dh);
  float mx = -INFINITY;
  for (int j = lane; j < nkeys; j += kWave) {
    const float* kp = (j < P) ? kpre + (size_t)j * dh : qkv_l + (size_t)(b * T + (j - P)) * 3 * d + d + (size_t)h * dh;
    float s = 0.f;
    for (int c = 0; c < dh; ++c) s = fmaf(sq[c], kp[c], s);
    s *= scale;
    sc[j] = s;
    mx = fmaxf(mx, s);
  }
  for (int o = kWave / 2; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, kWave));
  float sum = 0.f;
  for (int j = lane; j < nkeys; j += kWave) {
    const float e = expf(sc[j] - mx);
    sc[j] = e;
    sum += e;
  }
  for (int o = kWave / 2; o > 0; o >>= 1) sum += __shfl_xor(sum, o, kWave);
  __syncthreads();
  for (int c = lane; c < dh; c += kWave) {
    float acc = 0.f;
    for (int j = 0; j < nkeys; ++j) {
      const float* vp = (j < P) ? vpre + (size_t)j * dh : qkv_l + (size_t)(b * T + (j - P)) * 3 * d + 2 * d + (size_t)h * dh;
      acc = fmaf(sc[j], vp[c], acc);
    }
    out[((size_t)(l - 1) * M + row) * d + (size_t)h * dh + c] = acc / sum;
  }
}

// ------------------------------------------------------------------------------------------------
// bf16 MFMA path, head_dim = 128.
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));   // native vector: stays in registers
typedef short v4i16_t __attribute__((ext_vector_type(4)));
typedef short v8i16_t __attribute__((ext_vector_type(8)));

constexpr int kDh = 128;
constexpr int kTile = 32;            // keys per tile
constexpr int kKRow = kDh + 8;       // LDS row of a K tile (elements): 272 B
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNoRef = -1.0e30f;   // reference exponent of a softmax state that has seen no visible key yet (finite:
                                     // differences and products with it stay free of inf - inf)


// Where key kk of (layer li, sequence b, head h) lives: prefix row or this block's row; keys past the end
// are clamped to the last one (their probabilities are masked to zero).
struct KvSource {
  const bf16_t* kpre; const bf16_t* vpre;   // [P, dh] of this (layer, b, h)
  const bf16_t* kblk; const bf16_t* vblk;   // row 0 of this sequence's block, k / v third, this head
  int P, nkeys; size_t blk_stride;          // 3d
  __device__ __forceinline__ const bf16_t* k_row(int kk) const {
    kk = kk < nkeys ? kk : nkeys - 1;
    return kk < P ? kpre + (size_t)kk * kDh : kblk + (size_t)(kk - P) * blk_stride;
  }
  __device__ __forceinline__ const bf16_t* v_row(int kk) const {
    kk = kk < nkeys ? kk : nkeys - 1;
    return kk < P ? vpre + (size_t)kk * kDh : vblk + (size_t)(kk - P) * blk_stride;
  }
};

template <int QF>
struct SoftmaxState {
  f32x4_t o[QF][8];   // O^T: [dh tile mt][rows kb*4 + i] for query column lane % 16
  float m[QF];        // running maximum (base-2 scaled scores), equal over the 4 lane groups of a column
  float l[QF];        // running sum of this lane's own 8 keys per tile
};

// One 32-key tile for QF query fragments of 16 rows.  kf[tau][s]: K operand (rows = keys tau*16 + lane%16,
// dh chunk s*32 + kb*8).  qf[f][s]: Q operand (column = query f*16 + lane%16, same dh chunk).
// limit[f]: number of keys visible to this lane's query column (P + t + 1).
template <int QF>
__device__ __forceinline__ void attn_tile(const bf16x8_t (&kf)[2][4], const bf16x8_t (&qf)[QF][4],
                                          const bf16_t* __restrict__ ldsV, int tile_base, const int (&limit)[QF],
                                          int min_limit, float scale_log2, SoftmaxState<QF>& st, int lane) {
  const int kb = lane >> 4;
  const bool all_visible = tile_base + kTile <= min_limit;   // uniform: no masking needed in this tile
  bf16x8_t pf[QF];
  float sv[QF][8];     // raw scores q.k of this lane's 8 keys
#pragma unroll
  for (int f = 0; f < QF; ++f) {
    f32x4_t s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[0][s], qf[f][s], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[1][s], qf[f][s], s1, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) { sv[f][i] = s0[i]; sv[f][4 + i] = s1[i]; }
  }
  if (!all_visible) {
#pragma unroll
    for (int f = 0; f < QF; ++f)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int k0 = tile_base + kb * 4 + i;
        if (k0 >= limit[f]) sv[f][i] = -INFINITY;
        if (k0 + 16 >= limit[f]) sv[f][4 + i] = -INFINITY;
      }
  }
  // st.m is the reference exponent of everything accumulated so far (kNoRef before the first visible key).  It
  // follows the running maximum lazily: it is raised only when the maximum exceeds it by more than 2^8, so
  // probabilities stay below 256 (exact enough in fp32 sums and in bf16) and the rescale of O and l is skipped in most
  // tiles.  A column's maximum exceeds the bound exactly when one of its four lanes sees an exponent above 8, so the
  // common case needs no exchange between lanes: the column maxima are formed only inside the rare branch.
  float y[QF][8];      // exponents: score * scale * log2(e) - reference
  bool over = false;
#pragma unroll
  for (int f = 0; f < QF; ++f) {
    const float neg_m = -st.m[f];
#pragma unroll
    for (int j = 0; j < 8; ++j) y[f][j] = fmaf(sv[f][j], scale_log2, neg_m);
    const float ymax = fmaxf(fmaxf(fmaxf(y[f][0], y[f][1]), fmaxf(y[f][2], y[f][3])),
                             fmaxf(fmaxf(y[f][4], y[f][5]), fmaxf(y[f][6], y[f][7])));
    over = over || (ymax > 8.0f);
  }
  if (__builtin_amdgcn_ballot_w64(over) != 0) {               // uniform branch
#pragma unroll
    for (int f = 0; f < QF; ++f) {
      float mcol = fmaxf(fmaxf(fmaxf(sv[f][0], sv[f][1]), fmaxf(sv[f][2], sv[f][3])),
                         fmaxf(fmaxf(sv[f][4], sv[f][5]), fmaxf(sv[f][6], sv[f][7]))) * scale_log2;   // scale > 0
      mcol = fmaxf(mcol, __shfl_xor(mcol, 16, kWave));
      mcol = fmaxf(mcol, __shfl_xor(mcol, 32, kWave));
      const float m_new = mcol > st.m[f] + 8.0f ? mcol : st.m[f];
      const float alpha = __builtin_amdgcn_exp2f(st.m[f] - m_new);
      st.m[f] = m_new;
      st.l[f] *= alpha;
#pragma unroll
      for (int mt = 0; mt < 8; ++mt) {
        st.o[f][mt][0] *= alpha; st.o[f][mt][1] *= alpha; st.o[f][mt][2] *= alpha; st.o[f][mt][3] *= alpha;
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) y[f][j] = fmaf(sv[f][j], scale_log2, -m_new);
    }
  }
  // probabilities: the hardware's base-2 exponential (results below 2^-126 become zero, which is what they are
  // worth; a masked score is -inf and gives exactly 0)
#pragma unroll
  for (int f = 0; f < QF; ++f) {
    float psum = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float p = __builtin_amdgcn_exp2f(y[f][j]);
      psum += p;
      pf[f][j] = static_cast<__bf16>(p);
    }
    st.l[f] += psum;
  }
  // V^T operand of dh tile mt (row = dh mt*16 + lane%16, k slot j = tau*4 + i <-> key tau*16 + kb*4 + i, the key
  // whose probability this lane holds in element j of pf) straight from the row-major V tile with the LDS
  // transpose read ds_read_b64_tr_b16: in each group of 16 lanes, lane s supplies the address of 4 consecutive
  // 16-bit elements and lane i receives element i%4 of the rows addressed by lanes i/4, 4 + i/4, 8 + i/4,
  // 12 + i/4.  So lane s addresses key row (s / 4) of its group's four keys at dh offset mt*16 + 4*(s % 4), and
  // lane i receives V[key_j][mt*16 + i], j = 0..3.  Two reads (tau = 0, 1) make the 8 k slots.
  // V tile layout: 256-byte key rows, 16-byte chunk c of row r stored at position c ^ (r & 15).
  const int i16 = lane & 15;
  const int vrow = kb * 4 + (i16 >> 2);                       // row inside a 16-key half (= its swizzle key)
  const bf16_t* vbase = ldsV + vrow * kDh + ((i16 & 1) << 2);
#pragma unroll
  for (int mt = 0; mt < 8; ++mt) {
    const int pos = ((mt * 2 + ((i16 & 3) >> 1)) ^ vrow) << 3;
    const v4i16_t r0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) v4i16_t*)(vbase + pos));
    const v4i16_t r1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) v4i16_t*)(vbase + 16 * kDh + pos));
    const v8i16_t r = __builtin_shufflevector(r0, r1, 0, 1, 2, 3, 4, 5, 6, 7);
    const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, r);
#pragma unroll
    for (int f = 0; f < QF; ++f)
      st.o[f][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[f], st.o[f][mt], 0, 0, 0);
  }
}

// One 16-byte chunk (8 dh values of one key) into the V tile (swizzled position, see attn_tile).
__device__ __forceinline__ void write_v(bf16_t* __restrict__ ldsV, u32x4_t chunk, int key_in_tile, int c16) {
  *reinterpret_cast<u32x4_t*>(ldsV + key_in_tile * kDh + ((c16 ^ (key_in_tile & 15)) << 3)) = chunk;
}

__device__ __forceinline__ uint2 pack4_bf16(float a, float b, float c, float d) {
  const __bf16 x0 = static_cast<__bf16>(a), x1 = static_cast<__bf16>(b), x2 = static_cast<__bf16>(c), x3 = static_cast<__bf16>(d);
  uint2 r;
  r.x = (uint32_t)__builtin_bit_cast(bf16_t, x0) | ((uint32_t)__builtin_bit_cast(bf16_t, x1) << 16);
  r.y = (uint32_t)__builtin_bit_cast(bf16_t, x2) | ((uint32_t)__builtin_bit_cast(bf16_t, x3) << 16);
  return r;
}

// ---- block kernel: 1-D grid over (stream, query tile); a stream's query tiles are dispatched last-first: under the
// causal mask the last tile has the most keys, and starting the long workgroups first shortens the tail.
// 4 waves per workgroup, 32 query rows per wave, keys in steps of 32, both products with
// v_mfma_f32_32x32x16_bf16 on transposed operands: S^T (32 keys x 32 queries) = K Q^T over 8 k-steps of 16 channels,
// O^T (128 channels x 32 queries, four 32-row tiles) += V^T P^T over 2 k-steps of 16 keys.  A lane owns one query
// column in both (its 32 keys of a step are shared with lane ^ 32), so the softmax statistics are lane-local and the
// probabilities leave the S^T accumulator already in the operand layout of the second product.
// What limits this kernel is the latency of a wave's own instruction stream: a step is a chain (K operand reads,
// eight dependent MFMAs, ~90 VALU instructions of softmax -- a lone wave issues one VALU instruction per ~10
// cycles, measured -- the V reads, eight more MFMAs) of ~2000 cycles, of which the matrix pipe is busy 512.  So the
// kernel is built for THREE workgroups per compute unit (3 waves per SIMD): 168 registers, 48 KB of LDS.
// K and V travel global -> LDS with direct-to-LDS loads (lane i's 16 bytes land at base + 16 i) into two rings of
// three 32-row slots each: step j lives in slot j % 3.  Rows are 256 B, stored with their 16-byte chunk c at
// position c ^ swz(row % 16), swz = the row's two low bits exchanged with its two high bits, applied on the
// global-address side: the 16 rows of a K operand read then spread over all banks, and so do the 4 rows x 4 chunks
// that one half-wave touches in a transpose read of V.
// One barrier per step: in step j the waves read slot j % 3 and request the rows of step j + 2 into the slot that
// step j - 1 left.  Every step requests the same number of rows (past the last key: the last key again, into rows
// nobody reads), so that "all but the loads of the last step have landed" is one constant wait count.
// The load is written out instead of taken from the builtin: the compiler makes every LDS read that follows a
// direct-to-LDS load it knows of wait for ALL outstanding loads (it cannot tell ring rows apart), which would
// cancel the prefetch -- every step would begin by waiting for the rows just requested.  The waits are explicit
// here: one counted s_waitcnt before the barrier of each phase.  m0 carries the LDS base of the wave's 1 KB.
#define SNLP_GLDS16(gptr, lptr)                                                                              \
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"                               \
               :: "v"(gptr), "s"((uint32_t)(size_t)((__attribute__((address_space(3))) char*)(lptr)))        \
               : "memory", "m0")

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

__device__ __forceinline__ int ring_swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

__global__ __launch_bounds__(256, 3) void k_attn_bf16_block(const bf16_t* __restrict__ qkv,
                                                            const bf16_t* __restrict__ Kpre,
                                                            const bf16_t* __restrict__ Vpre,
                                                            bf16_t* __restrict__ out, int l0, int M, int T, int P, int B,
                                                            int H, int d, int n_streams, int n_qtiles, int stream_major) {
  constexpr int kSlots = 3;                     // 32-row slots of the K ring and of the V ring
  constexpr int kRing = kSlots * kTile;
  constexpr int kDepth = kSlots - 1;            // steps between the request of a row and its use
  constexpr int kRowsWg = 128;                  // query rows per workgroup
  constexpr int kLoadsPerStep = 4;              // per wave: 32 K rows and 32 V rows, 4 rows per load, over 4 waves
  __shared__ __attribute__((aligned(16))) bf16_t sK[kRing * kDh];
  __shared__ __attribute__((aligned(16))) bf16_t sV[kRing * kDh];
  // Workgroup -> (stream = (layer, sequence, head), query tile), heaviest query tile first.
  // Long blocks (stream_major): workgroups are handed to the 8 XCDs in turn (workgroup n runs on XCD n % 8) and each
  // XCD has its own L2, so the query tiles of one stream are given consecutive places on ONE XCD: they start
  // together, walk the same K / V rows at the same pace and all but the first read them from that L2.
  // Short blocks: all streams' heaviest tiles first, then the next ones; with few tiles per stream the order that
  // balances the tail is worth more than the sharing.
  int stream, qtile;
  if (stream_major) {
    const unsigned xcd = blockIdx.x & 7, in_xcd = blockIdx.x >> 3;
    stream = (int)(in_xcd / (unsigned)n_qtiles) * 8 + (int)xcd;
    qtile = n_qtiles - 1 - (int)(in_xcd % (unsigned)n_qtiles);
  } else {
    stream = (int)(blockIdx.x % (unsigned)n_streams);
    qtile = n_qtiles - 1 - (int)(blockIdx.x / (unsigned)n_streams);
  }
  if (stream >= n_streams) return;               // whole workgroup (stream-major: the last group of 8 may be short)
  const int li = l0 - 1 + stream / (B * H);      // 0-based layer
  const int b = (stream % (B * H)) / H, h = stream % H;
  const int q0 = qtile * kRowsWg;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform over the wave: keeps what depends on it scalar
  const int l32 = lane & 31, hi = lane >> 5;
  const size_t blk_stride = (size_t)3 * d;
  const bf16_t* qkv_b = qkv + ((size_t)li * M + (size_t)b * T) * blk_stride;
  const int nkeys = P + T;
  const bf16_t* kpre = Kpre ? Kpre + (((size_t)li * B + b) * H + h) * (size_t)P * kDh : nullptr;
  const bf16_t* vpre = Vpre ? Vpre + (((size_t)li * B + b) * H + h) * (size_t)P * kDh : nullptr;
  const bf16_t* kblk = qkv_b + d + (size_t)h * kDh;
  const bf16_t* vblk = qkv_b + 2 * d + (size_t)h * kDh;

  // Q operand (B of the first product) straight from global memory: column = query lane % 32, k-step ks holds channels
  // 16 ks + 8 (lane / 32) .. + 7
  const int trow = q0 + wave * 32 + l32;
  const int tq = trow < T ? trow : T - 1;
  const int limit = P + tq + 1;                  // number of keys visible to this lane's query
  bf16x8_t qf[8];
  {
    const bf16_t* qp = qkv_b + (size_t)tq * blk_stride + (size_t)h * kDh + hi * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const bf16x8_t*>(qp + ks * 16);
  }

  f32x16_t o[4];      // O^T tile dt: channels 32 dt + 8 (r / 4) + 4 (lane / 32) + r % 4 of query lane % 32
  float mref = kNoRef;   // reference exponent (kNoRef before the first visible key), equal in lanes l and l ^ 32
  float lsum = 0.f;      // running sum of this lane's own keys
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;

  const int q_last = (q0 + kRowsWg - 1 < T ? q0 + kRowsWg - 1 : T - 1);
  const int nkeys_wg = P + q_last + 1;                       // keys visible to the last row of the workgroup
  const int nsteps = (nkeys_wg + kTile - 1) / kTile;
  const int wave_last = P + (q0 + wave * 32 + 31 < T ? q0 + wave * 32 + 31 : T - 1);   // last key this wave can see
  const int wave_first = P + (q0 + wave * 32 < T ? q0 + wave * 32 : T - 1) + 1;        // keys visible to all its rows
  const int nsteps_w = wave_last / kTile + 1;                // steps this wave takes part in
  const float scale_log2 = kLog2e / sqrtf((float)kDh);

  // Loads.  A step's 32 rows are 8 groups of 4 rows; wave w fetches groups w and w + 4 with one instruction each
  // (lane = 16 (row - 4 g) + chunk position), so a lane's row % 16, and with it the swizzle key, is the same in both.
  // A step that lies wholly in the prefix or wholly in the block (every step when P = 0, up to the last one) has
  // addresses linear in the step index: a uniform pointer plus one per-lane offset that never changes; a step that
  // straddles the two, or reaches past the last key, chooses per row (rows past the end repeat the last key; their
  // probabilities are masked to zero).
  const int lrow = wave * 4 + (lane >> 4);                       // row of the first group this lane fetches
  const int iswz = ((lane & 15) ^ ring_swz(lrow)) << 3;
  const unsigned off_pre = (unsigned)(lrow * kDh + iswz), off_blk = (unsigned)(lrow * (int)blk_stride + iswz);
  auto load_step = [&](bf16_t* ring, const bf16_t* pre, const bf16_t* blk, int j, int slot) {
    const int base = j * kTile;
    bf16_t* dst = ring + (slot * kTile + wave * 4) * kDh;           // + 16 B per lane, by the instruction
    if (base + kTile <= P) {
      const bf16_t* p0 = pre + (size_t)base * kDh;
#pragma unroll
      for (int g = 0; g < 2; ++g) SNLP_GLDS16(p0 + (size_t)g * 16 * kDh + off_pre, dst + g * 16 * kDh);
    } else if (base >= P && base + kTile <= nkeys) {
      const bf16_t* p0 = blk + (size_t)(base - P) * blk_stride;
#pragma unroll
      for (int g = 0; g < 2; ++g) SNLP_GLDS16(p0 + (size_t)g * 16 * blk_stride + off_blk, dst + g * 16 * kDh);
    } else {
#pragma unroll
      for (int g = 0; g < 2; ++g) {
        int kk = base + g * 16 + lrow;
        kk = kk < nkeys ? kk : nkeys - 1;
        const bf16_t* rp = kk < P ? pre + (size_t)kk * kDh : blk + (size_t)(kk - P) * blk_stride;
        SNLP_GLDS16(rp + iswz, dst + g * 16 * kDh);
      }
    }
  };

  // Operand reads (element offsets inside a step's 32 ring rows).
  // K (A of the first product): row = key lane % 32, k-step ks = chunk 2 ks + lane / 32.
  // V^T (A of the second product), channel tile dt, key step kk: row = channel 32 dt + lane % 32, and k slot e of
  // lane half hi stands for key 16 kk + 8 (e / 4) + 4 hi + e % 4 -- the key whose probability the lane holds in
  // accumulator element 8 kk + e.  It comes from the row-major V rows with the LDS transpose read: in each group
  // of 16 lanes, lane s supplies the address of 4 consecutive 16-bit elements and lane i receives element i % 4 of
  // the rows addressed by lanes i / 4, 4 + i / 4, 8 + i / 4, 12 + i / 4.  So lane s addresses key row s / 4 of the
  // four keys 16 kk + 4 hi + 0..3 at channel 32 dt + 16 (lane / 16 % 2) + 4 (s % 4), and lane i receives those four
  // keys at channel 32 dt + lane % 32; a second read 8 rows further on gives slots 4..7.
  int koff[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) koff[ks] = l32 * kDh + (((2 * ks + hi) ^ ring_swz(l32 & 15)) << 3);
  const int i16 = lane & 15;
  const int vrow = 4 * hi + (i16 >> 2);                          // + 16 kk (+ 8 for the second read): same swizzle key
  int voff[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
    voff[dt] = vrow * kDh + ((i16 & 1) << 2) + (((4 * dt + 2 * ((lane >> 4) & 1) + ((i16 & 3) >> 1)) ^ ring_swz(vrow)) << 3);
  const int vswz8 = ring_swz(vrow) ^ ring_swz(vrow + 8);         // what 8 rows further on changes in the position

  // One step: the 32 keys of step j, from ring slot `slot`.
  auto step = [&](int j, int slot) {
    const bf16_t* kr = sK + slot * (kTile * kDh);
    const bf16_t* vr = sV + slot * (kTile * kDh);
    f32x16_t sacc;
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(kr + koff[ks]);
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], sacc, 0, 0, 0);
    }
    // element r of the accumulator: key 32 j + 8 (r / 4) + 4 hi + r % 4
    float sv[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) sv[r] = sacc[r];
    if ((j + 1) * kTile > wave_first) {                            // uniform: some row of the wave cannot see the whole step
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (j * kTile + 8 * (r >> 2) + 4 * hi + (r & 3) >= limit) sv[r] = -INFINITY;
    }
    // exponents relative to the reference.  The reference follows the running maximum lazily: it is raised only
    // when the maximum exceeds it by more than 2^8, so probabilities stay below 256 (exact enough in fp32 sums and
    // in bf16) and the rescale of O and l is skipped in most steps.  A column's maximum exceeds the bound exactly
    // when one of its two lanes sees an exponent above 8, so the common case needs no exchange between lanes.
    float y[16];
    const float neg_m = -mref;
#pragma unroll
    for (int r = 0; r < 16; ++r) y[r] = fmaf(sv[r], scale_log2, neg_m);
    float ymax = fmaxf(fmaxf(fmaxf(y[0], y[1]), fmaxf(y[2], y[3])), fmaxf(fmaxf(y[4], y[5]), fmaxf(y[6], y[7])));
    ymax = fmaxf(ymax, fmaxf(fmaxf(fmaxf(y[8], y[9]), fmaxf(y[10], y[11])), fmaxf(fmaxf(y[12], y[13]), fmaxf(y[14], y[15]))));
    if (__builtin_amdgcn_ballot_w64(ymax > 8.0f) != 0) {           // uniform branch, rare
      float mcol = sv[0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mcol = fmaxf(mcol, sv[r]);
      mcol *= scale_log2;                                          // scale > 0: max commutes with it
      mcol = fmaxf(mcol, __shfl_xor(mcol, 32, kWave));
      const float m_new = mcol > mref + 8.0f ? mcol : mref;
      const float alpha = __builtin_amdgcn_exp2f(mref - m_new);
      mref = m_new;
      lsum *= alpha;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
#pragma unroll
      for (int r = 0; r < 16; ++r) y[r] = fmaf(sv[r], scale_log2, -m_new);
    }
    // probabilities: the hardware's base-2 exponential (results below 2^-126 become zero, which is what they are
    // worth; a masked score is -inf and gives exactly 0)
    bf16x8_t pf[2];
    float psum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float pr = __builtin_amdgcn_exp2f(y[r]);
      psum += pr;
      pf[r >> 3][r & 7] = static_cast<__bf16>(pr);
    }
    lsum += psum;
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        const bf16_t* va = vr + kk * 16 * kDh + voff[dt];
        const v4i16_t r0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4i16_t*)va);
        const v4i16_t r1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) v4i16_t*)(vr + kk * 16 * kDh + 8 * kDh + (voff[dt] ^ (vswz8 << 3))));
        const v8i16_t rr = __builtin_shufflevector(r0, r1, 0, 1, 2, 3, 4, 5, 6, 7);
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, rr), pf[kk], o[dt], 0, 0, 0);
      }
  };

  // prologue: steps 0 .. D - 1
#pragma unroll
  for (int c = 0; c < kDepth; ++c) {
    load_step(sK, kpre, kblk, c, c);
    load_step(sV, vpre, vblk, c, c);
  }
  // The query operand is consumed here, before the loop, so that the compiler's own wait for its loads stands here
  // too: it does not count the direct-to-LDS loads, and a wait "for the query" inside the loop would in fact wait
  // for the rows just requested.
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+v"(qf[ks]));
  int slot = 0;                                              // slot of step j; step j + D goes to the slot before it
  for (int j = 0; j < nsteps; ++j) {
    // this wave's part of the rows of step j has landed (loads return in order; only those of the last D - 1 steps
    // may still be on their way); after the barrier everyone's has, and everyone is done with the rows this step's
    // loads replace.  (A bare barrier: __syncthreads() may also wait for every outstanding load.)
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"((kDepth - 1) * kLoadsPerStep) : "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    const int slot_in = slot == 0 ? kSlots - 1 : slot - 1;
    load_step(sK, kpre, kblk, j + kDepth, slot_in);
    load_step(sV, vpre, vblk, j + kDepth, slot_in);
    if (j < nsteps_w) step(j, slot);                         // uniform over the wave
    slot = slot + 1 == kSlots ? 0 : slot + 1;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the last phases' loads have landed before the LDS is given back

  lsum += __shfl_xor(lsum, 32, kWave);
  const float inv = 1.0f / lsum;
  if (trow < T) {
    bf16_t* op = out + ((size_t)li * M + (size_t)b * T + trow) * d + (size_t)h * kDh + 4 * hi;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const uint2 v = pack4_bf16(o[dt][4 * g] * inv, o[dt][4 * g + 1] * inv, o[dt][4 * g + 2] * inv, o[dt][4 * g + 3] * inv);
        *reinterpret_cast<uint2*>(op + 32 * dt + 8 * g) = v;
      }
  }
}

// ---- decode kernel: T <= 16; grid (B * H, Lc)
constexpr int kORow = kDh + 4;   // fp32 row of a partial output in LDS

// Rotary embedding and per-head RMS norm of one query or key row held as MFMA operand fragments: the lane has the
// channels s*32 + kb*8 + e (s = 0..3, e = 0..7) of row (lane % 16), so a rotation pair (c, c + 64) lives in
// fragments s and s + 2 of the same lane, and the four lanes kb = 0..3 of a row hold its 128 channels between
// them.  Same arithmetic as the stand-alone kernel: rotate in fp32, sum of squares, scale, round to bf16.
// cs / sn: this row's table row (64 floats each).  Every lane of the wave must call this (it shuffles).
__device__ __forceinline__ void rope_qknorm_frags(bf16x8_t (&f)[4], const float* __restrict__ cs,
                                                  const float* __restrict__ sn, int kb, float eps) {
  float y[4][8];
  float ss = 0.f;
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    const float4 c0 = *reinterpret_cast<const float4*>(cs + s * 32 + kb * 8);
    const float4 c1 = *reinterpret_cast<const float4*>(cs + s * 32 + kb * 8 + 4);
    const float4 s0 = *reinterpret_cast<const float4*>(sn + s * 32 + kb * 8);
    const float4 s1 = *reinterpret_cast<const float4*>(sn + s * 32 + kb * 8 + 4);
    const float cv[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
    const float sv[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float x1 = (float)f[s][e], x2 = (float)f[s + 2][e];
      y[s][e] = x1 * cv[e] - x2 * sv[e];
      y[s + 2][e] = x2 * cv[e] + x1 * sv[e];
      ss += y[s][e] * y[s][e] + y[s + 2][e] * y[s + 2][e];
    }
  }
  ss += __shfl_xor(ss, 16, kWave);
  ss += __shfl_xor(ss, 32, kWave);
  const float r = 1.0f / sqrtf(ss / (float)kDh + eps);
#pragma unroll
  for (int s = 0; s < 4; ++s)
#pragma unroll
    for (int e = 0; e < 8; ++e) f[s][e] = (__bf16)(y[s][e] * r);
}


__global__ __launch_bounds__(kThreads, 2) void k_attn_bf16_decode(const bf16_t* __restrict__ qkv,
                                                                const bf16_t* __restrict__ Kpre,
                                                                const bf16_t* __restrict__ Vpre,
                                                                bf16_t* __restrict__ out, int l0, int M, int T, int P,
                                                                int B, int H, int d, const float* __restrict__ cos_tab,
                                                                const float* __restrict__ sin_tab, float eps) {
  // cos_tab != nullptr: q and the block's k rows arrive straight from the QKV GEMM and get their rotary embedding
  // and QK norm here (table row = position inside the block); the prefix keys are used as given.
  constexpr int QF = 1;
  // per wave: one V tile while streaming; afterwards the same memory holds the partial states
  constexpr int kStreamBytes = 4 * kTile * kDh * 2;
  constexpr int kMergeBytes = 4 * 16 * kORow * 4 + 4 * 16 * 2 * 4;
  __shared__ __attribute__((aligned(16))) unsigned char lds_raw[kStreamBytes > kMergeBytes ? kStreamBytes : kMergeBytes];
  const int li = l0 - 1 + blockIdx.y;
  const int b = blockIdx.x / H, h = blockIdx.x % H;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kb = lane >> 4;
  const size_t blk_stride = (size_t)3 * d;
  const bf16_t* qkv_b = qkv + ((size_t)li * M + (size_t)b * T) * blk_stride;
  bf16_t* ldsV = reinterpret_cast<bf16_t*>(lds_raw) + wave * (kTile * kDh);

  KvSource src;
  src.P = P; src.nkeys = P + T; src.blk_stride = blk_stride;
  src.kpre = Kpre ? Kpre + (((size_t)li * B + b) * H + h) * (size_t)P * kDh : nullptr;
  src.vpre = Vpre ? Vpre + (((size_t)li * B + b) * H + h) * (size_t)P * kDh : nullptr;
  src.kblk = qkv_b + d + (size_t)h * kDh;
  src.vblk = qkv_b + 2 * d + (size_t)h * kDh;

  // The block's q, k, v rows of a workgroup are 3 T scattered 256-byte rows that the QKV GEMM wrote just before, and a
  // workgroup that starts while the chip streams at the HBM limit reads them from DRAM as row misses among a saturated
  // stream of row hits: at T = 8 those 0.2 % of the bytes cost 4 % of the kernel (one row per workgroup: 489 us, eight:
  // 528; identical rows for all workgroups, i.e. L2 hits: 515).  So the workgroups of the first round, which start on an
  // idle memory system, read one word of every such line of the workgroups that the SAME XCD runs later (workgroups
  // are dealt to the 8 XCDs in turn, so those are the linear ids w + kTouchStride k; at d20 2 MB per XCD, which its
  // 4 MB L2 keeps: the prefix streams through with non-temporal loads) -- 528 -> 508 us.  A wrong guess about the
  // placement costs time, never correctness: the words are only read.  kTouchMax bounds what one XCD is asked to keep.
  constexpr int kTouchStride = 512, kTouchMax = 8;
  unsigned touched = 0;
  {
    const int wlin = blockIdx.y * gridDim.x + blockIdx.x, nitems = gridDim.x * gridDim.y;
    if (wlin < kTouchStride && wlin + kTouchStride < nitems) {          // uniform over the workgroup
      const int per_item = 6 * T;                                        // 128-byte lines of one item's q, k, v rows
      int nfuture = (nitems - 1 - wlin) / kTouchStride;
      nfuture = nfuture < kTouchMax ? nfuture : kTouchMax;
      for (int ln = tid; ln < nfuture * per_item; ln += kThreads) {
        const int kk = ln / per_item, rem = ln % per_item;
        const int id = wlin + kTouchStride * (kk + 1);
        const int seg = rem / (2 * T), r = (rem % (2 * T)) >> 1, half = rem & 1;
        const int li2 = l0 - 1 + id / (int)gridDim.x, x2 = id % (int)gridDim.x;
        const bf16_t* pt = qkv + ((size_t)li2 * M + (size_t)(x2 / H) * T + r) * blk_stride + (size_t)seg * d +
                           (size_t)(x2 % H) * kDh + half * 64;
        touched ^= *reinterpret_cast<const unsigned*>(pt);
      }
    }
  }
  bf16x8_t qf[QF][4];
  int limit[QF];
  int t = lane & 15;
  const int trow = t;
  t = t < T ? t : T - 1;
  limit[0] = P + t + 1;
  {
    const bf16_t* qp = qkv_b + (size_t)t * blk_stride + (size_t)h * kDh;
#pragma unroll
    for (int s = 0; s < 4; ++s) qf[0][s] = *reinterpret_cast<const bf16x8_t*>(qp + s * 32 + kb * 8);
    if (cos_tab) rope_qknorm_frags(qf[0], cos_tab + (size_t)t * (kDh / 2), sin_tab + (size_t)t * (kDh / 2), kb, eps);
  }
  SoftmaxState<QF> st;
  st.m[0] = kNoRef; st.l[0] = 0.f;
#pragma unroll
  for (int mt = 0; mt < 8; ++mt) st.o[0][mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  const int ntiles = (P + T + kTile - 1) / kTile;
  const float scale_log2 = kLog2e / sqrtf((float)kDh);

  // K operand registers: rows tau*16 + lane%16, chunk s*32 + kb*8; V staging: chunk id lane + 64*p ->
  // key id / 16 (4 keys per load instruction, 256 contiguous bytes each), chunk id % 16.
  bf16x8_t kf[2][4];
  u32x4_t rv[8];
  auto prefetch = [&](int tile) {
    const int base = tile * kTile;
    if (base + kTile <= P) {
      // a tile wholly inside the prefix (all but the last one or two): its rows are contiguous, so the addresses
      // are linear in the lane index and need no per-row choice between prefix and block
      const bf16_t* kp = src.kpre + (size_t)(base + (lane & 15)) * kDh + kb * 8;
#pragma unroll
      for (int tau = 0; tau < 2; ++tau)
#pragma unroll
        for (int s = 0; s < 4; ++s)
          kf[tau][s] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8_t*>(kp + tau * 16 * kDh + s * 32));
      const bf16_t* vp = src.vpre + (size_t)base * kDh + lane * 8;
#pragma unroll
      for (int p = 0; p < 8; ++p) rv[p] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(vp + p * 512));
      return;
    }
#pragma unroll
    for (int tau = 0; tau < 2; ++tau) {
      const bf16_t* kp = src.k_row(base + tau * 16 + (lane & 15));
#pragma unroll
      for (int s = 0; s < 4; ++s) kf[tau][s] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8_t*>(kp + s * 32 + kb * 8));
    }
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const int id = lane + 64 * p;
      rv[p] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(src.v_row(base + (id >> 4)) + (id & 15) * 8));
    }
  };
  if (wave < ntiles) prefetch(__builtin_amdgcn_readfirstlane(wave));
  // Tiles that lie wholly in the prefix stream through the main loop.  The block's own rows (T <= 16) touch at most
  // the last two tiles, at most one per wave: that tile is handled after the loop, where nothing is being
  // prefetched any more and the registers of the prefetch are free for the rotary / norm arithmetic.
  const int first_blk_tile = cos_tab ? P / kTile : ntiles;
  auto stage_v = [&]() {
    // the V tile is private to the wave and a wave's LDS operations complete in issue order, so no barrier
    // separates these writes from the previous tile's reads or from this tile's: the four waves stream
    // independently until the merge
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const int id = lane + 64 * p;
      write_v(ldsV, rv[p], id >> 4, id & 15);
    }
  };
  int tile = __builtin_amdgcn_readfirstlane(wave);
  for (; tile < first_blk_tile; tile += 4) {
    stage_v();
    bf16x8_t kcur[2][4];
#pragma unroll
    for (int tau = 0; tau < 2; ++tau)
#pragma unroll
      for (int s = 0; s < 4; ++s) kcur[tau][s] = kf[tau][s];
    if (tile + 4 < ntiles) prefetch(tile + 4);
    attn_tile<QF>(kcur, qf, ldsV, tile * kTile, limit, P + 1, scale_log2, st, lane);
  }
  if (tile < ntiles) {   // this wave's tile with rows of the block (only when the kernel rotates them itself)
    stage_v();
#pragma unroll
    for (int tau = 0; tau < 2; ++tau) {
      int key = tile * kTile + tau * 16 + (lane & 15);
      key = key < P + T ? key : P + T - 1;
      const int tb = key >= P ? key - P : 0;
      bf16x8_t tmp[4];
#pragma unroll
      for (int s = 0; s < 4; ++s) tmp[s] = kf[tau][s];
      rope_qknorm_frags(tmp, cos_tab + (size_t)tb * (kDh / 2), sin_tab + (size_t)tb * (kDh / 2), kb, eps);
      if (key >= P) {
#pragma unroll
        for (int s = 0; s < 4; ++s) kf[tau][s] = tmp[s];
      }
    }
    attn_tile<QF>(kf, qf, ldsV, tile * kTile, limit, P + 1, scale_log2, st, lane);
  }

  // merge the 4 partial states in wave order
  float lt = st.l[0];
  lt += __shfl_xor(lt, 16, kWave);
  lt += __shfl_xor(lt, 32, kWave);
  __syncthreads();
  float* po = reinterpret_cast<float*>(lds_raw);                 // [4][16][kORow]
  float* pm = po + 4 * 16 * kORow;                               // [4][16] maxima, then [4][16] sums
  float* pl = pm + 4 * 16;
  {
    float* row = po + ((size_t)wave * 16 + (lane & 15)) * kORow;
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) *reinterpret_cast<f32x4_t*>(row + mt * 16 + kb * 4) = st.o[0][mt];
    if (kb == 0) { pm[wave * 16 + lane] = st.m[0]; pl[wave * 16 + lane] = lt; }
  }
  __syncthreads();
  {
    const int q = tid >> 4, c0 = (tid & 15) * 8;
    float mt_ = fmaxf(fmaxf(pm[q], pm[16 + q]), fmaxf(pm[32 + q], pm[48 + q]));
    float w[4], lsum = 0.f;
#pragma unroll
    for (int wv = 0; wv < 4; ++wv) {
      w[wv] = exp2f(pm[wv * 16 + q] - mt_);
      lsum += w[wv] * pl[wv * 16 + q];
    }
    const float inv = 1.0f / lsum;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
#pragma unroll
    for (int wv = 0; wv < 4; ++wv) {
      const float* row = po + ((size_t)wv * 16 + q) * kORow + c0;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += w[wv] * row[e];
    }
    if (q < T) {
      bf16_t* op = out + ((size_t)li * M + (size_t)b * T + q) * d + (size_t)h * kDh + c0;
      const uint2 lo = pack4_bf16(acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv);
      const uint2 hi = pack4_bf16(acc[4] * inv, acc[5] * inv, acc[6] * inv, acc[7] * inv);
      *reinterpret_cast<uint4*>(op) = make_uint4(lo.x, lo.y, hi.x, hi.y);
    }
  }
  (void)trow;
  asm volatile("" :: "v"(touched));   // keeps the touching loads
}

}  // namespace

hipError_t launch_attention_f32(hipStream_t s, const Dims& D, int l0, int Lc, const float* qkv, const float* Kpre,
                                const float* Vpre, float* out, float* /*score_ws*/) {
  const size_t shm = (size_t)(D.dh + D.P + D.T) * sizeof(float);
  if (shm > 64 * 1024) return hipErrorInvalidValue;
  dim3 grid(D.M, D.H, Lc), block(kWave);
  hipLaunchKernelGGL(k_attn_f32, grid, block, shm, s, qkv, Kpre, Vpre, out, l0, D.M, D.T, D.P, D.B, D.H, D.dh, D.d);
  return hipGetLastError();
}

size_t attention_f32_ws_floats(const Dims&) { return 0; }

// The in-kernel rotation costs each workgroup a few dependent loads before its first tile; behind a long prefix
// that hides under the other workgroups' streaming and saves a pass over q and k, with a short prefix the
// stand-alone pass is cheaper (measured: P = 2048 fused 3-8 us faster, P = 64 fused 14 us slower per iteration).
bool attention_bf16_fuses_rope(const Dims& D) { return D.dh == kDh && D.T <= 16 && D.P >= 512; }

hipError_t launch_attention_bf16(hipStream_t s, const Dims& D, int l0, int Lc, const bf16_t* qkv, const bf16_t* Kpre,
                                 const bf16_t* Vpre, bf16_t* out, const float* cos_tab, const float* sin_tab) {
  if (D.dh != kDh) return hipErrorInvalidValue;
  if (D.T <= 16) {
    dim3 grid(D.B * D.H, Lc), block(kThreads);
    hipLaunchKernelGGL(k_attn_bf16_decode, grid, block, 0, s, qkv, Kpre, Vpre, out, l0, D.M, D.T, D.P, D.B, D.H, D.d, cos_tab, sin_tab,
                       D.eps);
  } else {
    const int n_streams = D.B * D.H * Lc, n_qtiles = (D.T + 127) / 128;
    const int stream_major = n_qtiles >= 8 ? 1 : 0;       // a function of the block length alone
    dim3 grid((unsigned)(stream_major ? (n_streams + 7) / 8 * 8 * n_qtiles : n_streams * n_qtiles)), block(256);
    hipLaunchKernelGGL(k_attn_bf16_block, grid, block, 0, s, qkv, Kpre, Vpre, out, l0, D.M, D.T, D.P, D.B, D.H, D.d, n_streams,
                       n_qtiles, stream_major);
  }
  return hipGetLastError();
}

}  // namespace snlp

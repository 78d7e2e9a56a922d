// SEA's decoder path (Sec. 3.1 "CNN Decoder", App. A.5.1 "Attention Estimator CNN") with
// caller-supplied weights: the Performer output on the concatenated values [V_I; V], the MLPs mu
// and nu, the three-layer CNN (nearest resize before its last layer) and the final softmax that
// yields the compressed attention matrix A_hat, plus the scalers s_mix, s_prob of Sec. 3.1.1
// "Output Calculation".  bf16 tensors, fp32 accumulation, every contraction on the matrix cores
// (v_mfma_f32_16x16x32_bf16) with operand fragments loaded straight from memory: lane l of a wave
// holds row / column l % 16 and the contraction elements 8 (l / 16) .. + 7 of a 32-wide step, and
// an accumulator tile (lane = column l % 16, registers = rows 4 (l / 16) + i) can be packed and
// fed back as an operand fragment of the next product without leaving the registers.
//
// Kernels, in the order a call runs them:
//   dec_features_kernel   phi(Q), phi(K) (bf16, [N][T][m]); phi(K)^T and V^T as zero-padded
//                         transposed copies ([N][m][Tp], [N][64][Tp]) for the products that contract
//                         over the token index
//   dec_linattn_kernel    chunked linear attention: per 32-token chunk the outputs from the running
//                         state (tokens of earlier chunks) and from the masked in-chunk product, then
//                         the state update; one wavefront per (head, 16 value columns); the values
//                         are [V_I; V; 1], so column 128 is the row normaliser
//   dec_concat_kernel     [C_perf; V] in bf16
//   dec_conv_kernel       implicit GEMM for the linear layers (one tap) and the 3x3 convolutions
//                         (nine taps, channels-last images, optional nearest resize on the read)
//   dec_softmax_kernel    softmax over the K columns of a row, rows past the sequence end zeroed
//   dec_scalers_kernel    s_mix, s_prob = sigmoid(w . Z + b)
#include <algorithm>

#include "sea_internal.h"

namespace sea {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kCs = 2;       // width reduction of the CNN's hidden image (c_s)
constexpr int kCh = 4;       // channel expansion (c_h)
constexpr int kTRow = 72;      // halfwords per LDS row of the transposed 64-token tile (16-byte aligned rows)
constexpr int kValCols = 144;  // [V_I (64); V (64); 1; 15 unused]: nine 16-column slices

__device__ __forceinline__ floatx4 mfma16(bf16x8 a, bf16x8 b, floatx4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ bf16x8 load8(const uint16_t* p) { return *reinterpret_cast<const bf16x8*>(p); }
__device__ __forceinline__ bf16x8 zero8() {
  const uint4 z = {0u, 0u, 0u, 0u};
  return __builtin_bit_cast(bf16x8, z);
}
__device__ __forceinline__ bf16x8 pack8(floatx4 lo, floatx4 hi) {
  uint4 u;
  u.x = pack_bf16(lo[0], lo[1]);
  u.y = pack_bf16(lo[2], lo[3]);
  u.z = pack_bf16(hi[0], hi[1]);
  u.w = pack_bf16(hi[2], hi[3]);
  return __builtin_bit_cast(bf16x8, u);
}
__device__ __forceinline__ float sumsq8(bf16x8 v) {
  const uint4 u = __builtin_bit_cast(uint4, v);
  const uint32_t w[4] = {u.x, u.y, u.z, u.w};
  float a = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float lo = bf16lo_to_f32(w[i]), hi = bf16hi_to_f32(w[i]);
    a = fmaf(lo, lo, a);
    a = fmaf(hi, hi, a);
  }
  return a;
}

// ------------------------------------------------------------------------------------------
// features.  Block = 4 waves, wave = 16 rows of one head; C[feature][row] = W X^T, so lane
// l % 16 is the row and a lane holds four consecutive features per tile.
// grid.x = 2 N ceil(Tp / 64): first half queries, second half keys (which also transpose V).
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void dec_features_kernel(Shape s, int32_t Tp, const uint16_t* __restrict__ Q,
                                                           const uint16_t* __restrict__ K,
                                                           const uint16_t* __restrict__ V,
                                                           const uint16_t* __restrict__ W,
                                                           uint16_t* __restrict__ phiQ, uint16_t* __restrict__ phiK,
                                                           uint16_t* __restrict__ phiKT, uint16_t* __restrict__ Vt,
                                                           float c_dot, float c_norm) {
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
  const int lr = lane & 15, lg = lane >> 4;
  const uint32_t tiles = Tp / 64;
  const uint32_t half = static_cast<uint32_t>(s.N) * tiles;
  const int which = blockIdx.x >= half;
  const uint32_t bid = which ? blockIdx.x - half : blockIdx.x;
  const int64_t head = bid / tiles;
  const int32_t r0 = static_cast<int32_t>(bid % tiles) * 64 + wid * 16;
  const int32_t t = r0 + lr;                  // this lane's row (as MFMA column), < Tp
  const int32_t tc = min(t, s.T - 1);         // clamped for loads
  const int32_t b = static_cast<int32_t>(head / s.H);
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
  const uint16_t* X = (which ? K : Q) + (head * s.T + tc) * kHeadDim;
  const bf16x8 x0 = load8(X + 8 * lg), x1 = load8(X + 32 + 8 * lg);
  float nx = sumsq8(x0) + sumsq8(x1);
  nx += __shfl_xor(nx, 16, kWave);
  nx += __shfl_xor(nx, 32, kWave);
  const float bias = c_norm * nx;  // log2(e) * scale * |x|^2 / 2
  const int ftiles = s.m / 16;
  const bool active = t < len;

  if (!which) {
    if (r0 >= s.T) return;
    float amax = -INFINITY;
    for (int ft = 0; ft < ftiles; ++ft) {
      const uint16_t* w = W + (ft * 16 + lr) * kHeadDim;
      floatx4 acc = {0.f, 0.f, 0.f, 0.f};
      acc = mfma16(load8(w + 8 * lg), x0, acc);
      acc = mfma16(load8(w + 32 + 8 * lg), x1, acc);
#pragma unroll
      for (int i = 0; i < 4; ++i) amax = fmaxf(amax, fmaf(c_dot, acc[i], -bias));
    }
    amax = fmaxf(amax, __shfl_xor(amax, 16, kWave));
    amax = fmaxf(amax, __shfl_xor(amax, 32, kWave));
    const float shift = ceilf(amax);  // power-of-two row scale: cancels in the normaliser
    uint16_t* out = phiQ + (head * s.T + tc) * s.m;
    for (int ft = 0; ft < ftiles; ++ft) {
      const uint16_t* w = W + (ft * 16 + lr) * kHeadDim;
      floatx4 acc = {0.f, 0.f, 0.f, 0.f};
      acc = mfma16(load8(w + 8 * lg), x0, acc);
      acc = mfma16(load8(w + 32 + 8 * lg), x1, acc);
      float v[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] = active ? exp2f(fmaf(c_dot, acc[i], -bias) - shift) : 0.f;
      if (t < s.T) {
        uint2 pk;
        pk.x = pack_bf16(v[0], v[1]);
        pk.y = pack_bf16(v[2], v[3]);
        *reinterpret_cast<uint2*>(out + ft * 16 + 4 * lg) = pk;
      }
    }
    return;
  }
  // keys: natural and transposed copies; positions past the sequence end (and the padding up to Tp)
  // hold zeros, so they drop out of every sum over keys.  The transposed copies (phi(K)^T and V^T,
  // 64 tokens = 128 bytes per row and block) are gathered in LDS and leave as whole lines.
  __shared__ __attribute__((aligned(16))) uint16_t tT[(256 + kHeadDim) * kTRow];
  const int tcol = wid * 16 + lr;  // this lane's token inside the block's 64
  uint16_t* out = phiK + (head * s.T + tc) * s.m;
  for (int ft = 0; ft < ftiles; ++ft) {
    const uint16_t* w = W + (ft * 16 + lr) * kHeadDim;
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
    acc = mfma16(load8(w + 8 * lg), x0, acc);
    acc = mfma16(load8(w + 32 + 8 * lg), x1, acc);
    float v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = active ? exp2f(fmaf(c_dot, acc[i], -bias)) : 0.f;
    uint2 pk;
    pk.x = pack_bf16(v[0], v[1]);
    pk.y = pack_bf16(v[2], v[3]);
    if (t < s.T) *reinterpret_cast<uint2*>(out + ft * 16 + 4 * lg) = pk;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t word = i < 2 ? pk.x : pk.y;
      tT[(ft * 16 + 4 * lg + i) * kTRow + tcol] = static_cast<uint16_t>((i & 1) ? (word >> 16) : (word & 0xffffu));
    }
  }
  // V^T: this lane moves dims 16 lg .. + 15 of row t
  const uint16_t* vrow = V + (head * s.T + tc) * kHeadDim + 16 * lg;
  const uint4 va = *reinterpret_cast<const uint4*>(vrow), vb = *reinterpret_cast<const uint4*>(vrow + 8);
  const uint32_t words[8] = {va.x, va.y, va.z, va.w, vb.x, vb.y, vb.z, vb.w};
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const uint32_t word = words[e >> 1];
    const uint16_t val = static_cast<uint16_t>((e & 1) ? (word >> 16) : (word & 0xffffu));
    tT[(s.m + 16 * lg + e) * kTRow + tcol] = t < s.T ? val : static_cast<uint16_t>(0);
  }
  __syncthreads();
  const int32_t blk_t0 = static_cast<int32_t>(bid % tiles) * 64;
  uint16_t* kt_base = phiKT + head * static_cast<int64_t>(s.m) * Tp + blk_t0;
  uint16_t* vt_base = Vt + head * static_cast<int64_t>(kHeadDim) * Tp + blk_t0;
  for (int x = threadIdx.x; x < (s.m + kHeadDim) * 8; x += 256) {
    const int row = x >> 3, piece = x & 7;
    const uint4 v = *reinterpret_cast<const uint4*>(&tT[row * kTRow + 8 * piece]);
    uint16_t* dst = row < s.m ? kt_base + static_cast<int64_t>(row) * Tp : vt_base + static_cast<int64_t>(row - s.m) * Tp;
    *reinterpret_cast<uint4*>(dst + 8 * piece) = v;
  }
}

// ------------------------------------------------------------------------------------------
// linear attention with values U = [V_I; V; 1].  One wavefront per (head, slice of 16 value
// columns).  State S[f][v] = sum over earlier keys of phi(k_j)[f] U[j][v], fp32, as accumulator
// tiles whose rows stand for the features 32 kc + 8 (r / 4) + 4 h + r % 4 (tile 2 kc + h, row r):
// packed in pairs they are the operand fragments of contraction step kc in natural feature
// order.  Per chunk of 32 tokens: P^T = phi(K_c) phi(Q_c)^T (masked j <= t when causal),
// O^T = S^T-fragments x phi(Q_c)^T + U_c^T x P^T, then S += phi(K_c)^T U_c.  Unnormalised sums go
// out in fp32: acc[N][T][144].
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ uint16_t one_bf16() { return 0x3f80; }

// eight values U[j][v] for consecutive or listed tokens j, as a bf16 fragment
// [vi_lo, vi_hi): the tokens j with V_I[j][v] = 1, i.e. floor(j d / T) == v (empty for v >= 64)
template <typename F>
__device__ __forceinline__ bf16x8 value_frag(int32_t v, const uint16_t* VtRow, int32_t T, int32_t vi_lo, int32_t vi_hi,
                                             F&& token_of) {
  if (v >= 64 && v < 128) {
    // V^T row v - 64: two 8-byte pieces (tokens token_of(0) .. + 3 and token_of(4) .. + 3)
    const uint2 a = *reinterpret_cast<const uint2*>(VtRow + token_of(0));
    const uint2 b = *reinterpret_cast<const uint2*>(VtRow + token_of(4));
    const uint4 u = {a.x, a.y, b.x, b.y};
    return __builtin_bit_cast(bf16x8, u);
  }
  uint32_t w[4];
#pragma unroll
  for (int e = 0; e < 8; e += 2) {
    uint32_t pair = 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int32_t j = token_of(e + h);
      bool on = false;
      if (v < 64) on = j >= vi_lo && j < vi_hi;                                                 // V_I[j][v]
      else if (v == 128) on = j < T;                                                            // normaliser column
      pair |= on ? (static_cast<uint32_t>(one_bf16()) << (16 * h)) : 0u;
    }
    w[e >> 1] = pair;
  }
  const uint4 u = {w[0], w[1], w[2], w[3]};
  return __builtin_bit_cast(bf16x8, u);
}

// Block = nine waves, one per slice of 16 value columns, all working on the same head and the
// same chunk: the chunk's phi(Q), phi(K) and phi(K)^T tiles are fetched once per block and parked
// in LDS in operand-fragment order (fragment = the 16 bytes one lane feeds to one product), so the
// features are read from memory once per head instead of once per slice.
// The sequence is cut into G segments of `cps` chunks so that enough blocks are in flight: with
// PHASE 0 a wave sums phi(K)^T U over its own segment and leaves the tile registers in `seg_state`
// ([head][slice][segment][2 MC tiles][64 lanes] float4); with PHASE 1 it starts from the sum of the
// segments before its own (causal) or of all segments (bidirectional) and emits its chunks.  G = 1:
// PHASE 1 alone walks the whole sequence.
constexpr int kLinWaves = 9;
template <int MC, int PHASE>
__global__ __launch_bounds__(64 * kLinWaves) void dec_linattn_kernel(Shape s, int32_t Tp, int32_t G, int32_t cps,
                                                                     const uint16_t* __restrict__ phiQ,
                                                                     const uint16_t* __restrict__ phiK,
                                                                     const uint16_t* __restrict__ phiKT,
                                                                     const uint16_t* __restrict__ Vt,
                                                                     float* __restrict__ acc_out,
                                                                     float4* __restrict__ seg_state) {
  constexpr int m = 32 * MC;
  constexpr int kFrags = 2 * MC * 64;  // fragments per tile: Q and K [kc][half][lane], K^T [x][lane]
  constexpr int kThreads = 64 * kLinWaves;
  constexpr int kPer = (3 * kFrags + kThreads - 1) / kThreads;  // fragments a thread moves per chunk
  __shared__ __attribute__((aligned(16))) uint4 tiles[3 * kFrags];
  const int tid = threadIdx.x, lane = tid & 63, lr = lane & 15, lg = lane >> 4;
  const int slice = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int32_t seg = static_cast<int32_t>(blockIdx.x % static_cast<uint32_t>(G));
  const int64_t head = blockIdx.x / static_cast<uint32_t>(G);
  const int64_t hs = head * 9 + slice;  // (head, slice)
  const int32_t v0 = slice * 16;
  const int32_t vcol = v0 + lr;  // the value column this lane stands for as an operand row / column
  // floor(j d / T) == v  <=>  ceil(v T / d) <= j < ceil((v + 1) T / d)
  const int32_t vi_lo = vcol < 64 ? static_cast<int32_t>((static_cast<int64_t>(vcol) * s.T + kHeadDim - 1) / kHeadDim) : 0;
  const int32_t vi_hi =
      vcol < 64 ? min(s.T, static_cast<int32_t>((static_cast<int64_t>(vcol + 1) * s.T + kHeadDim - 1) / kHeadDim)) : 0;
  const uint16_t* VtRow = Vt + (head * kHeadDim + max(0, min(vcol - 64, 63))) * static_cast<int64_t>(Tp);
  const uint16_t* Qh = phiQ + head * static_cast<int64_t>(s.T) * m;
  const uint16_t* Kh = phiK + head * static_cast<int64_t>(s.T) * m;
  const uint16_t* KTh = phiKT + head * static_cast<int64_t>(m) * Tp;
  float* Oh = acc_out + head * static_cast<int64_t>(s.T) * kValCols;
  const int32_t nchunks = Tp / 32;

  // the block's loader: fragment id -> its 16 bytes in memory.  `which` 0: phi(Q), 1: phi(K) (rows
  // clamped to the last token; rows past it are masked or multiply zeros), 2: phi(K)^T.
  uint4 held[kPer];
  auto fetch = [&](int32_t t0, bool want_q, bool want_k, bool want_kt) {
#pragma unroll
    for (int r = 0; r < kPer; ++r) {
      // a slot with nothing to fetch (past the last fragment, or a tile this pass does not use)
      // reads the head's first 16 bytes instead: every load is unconditional, so all of a thread's
      // loads are in flight together
      const int id = min(tid + r * kThreads, 3 * kFrags - 1);
      const int which = id / kFrags, fid = id % kFrags;
      const int x = fid >> 6, fl = fid & 63, flr = fl & 15, flg = fl >> 4;
      const uint16_t* src;
      bool want;
      if (which < 2) {
        const int kc = x >> 1, half = x & 1;
        const int32_t row = min(t0 + 16 * half + flr, s.T - 1);
        src = (which ? Kh : Qh) + static_cast<int64_t>(row) * m + 32 * kc + 8 * flg;
        want = which ? want_k : want_q;
      } else {
        const int f = 32 * (x >> 1) + 8 * (flr >> 2) + 4 * (x & 1) + (flr & 3);
        src = KTh + static_cast<int64_t>(f) * Tp + t0 + 8 * flg;
        want = want_kt;
      }
      held[r] = *reinterpret_cast<const uint4*>(want ? src : Qh);
    }
  };
  auto park = [&]() {
#pragma unroll
    for (int r = 0; r < kPer; ++r) {
      const int id = tid + r * kThreads;
      if (id < 3 * kFrags) tiles[id] = held[r];
    }
  };
  auto frag = [&](int which, int x) { return __builtin_bit_cast(bf16x8, tiles[which * kFrags + x * 64 + lane]); };

  floatx4 S[2 * MC];
#pragma unroll
  for (int x = 0; x < 2 * MC; ++x) S[x] = floatx4{0.f, 0.f, 0.f, 0.f};

  auto update = [&](int32_t t0) {
    // S[f][v] += sum_j phi(K)^T[f][j] U[j][v]: A rows = features (in the order of the tile rows),
    // B column = this lane's value column, contraction over the chunk's 32 tokens
    const bf16x8 ub = value_frag(vcol, VtRow, s.T, vi_lo, vi_hi, [&](int e) { return t0 + 8 * lg + e; });
#pragma unroll
    for (int x = 0; x < 2 * MC; ++x) S[x] = mfma16(frag(2, x), ub, S[x]);
  };
  auto emit = [&](int32_t t0, bool causal) {
    floatx4 OT[2] = {floatx4{0.f, 0.f, 0.f, 0.f}, floatx4{0.f, 0.f, 0.f, 0.f}};
    floatx4 PT[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int c = 0; c < 2; ++c) PT[a][c] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kc = 0; kc < MC; ++kc) {
      const bf16x8 q0 = frag(0, 2 * kc), q1 = frag(0, 2 * kc + 1);
      const bf16x8 sf = pack8(S[2 * kc], S[2 * kc + 1]);  // rows = this slice's value columns
      OT[0] = mfma16(sf, q0, OT[0]);
      OT[1] = mfma16(sf, q1, OT[1]);
      if (causal) {
        const bf16x8 k0 = frag(1, 2 * kc), k1 = frag(1, 2 * kc + 1);
        PT[0][0] = mfma16(k0, q0, PT[0][0]);
        PT[0][1] = mfma16(k0, q1, PT[0][1]);
        PT[1][0] = mfma16(k1, q0, PT[1][0]);
        PT[1][1] = mfma16(k1, q1, PT[1][1]);
      }
    }
    if (causal) {
      // P^T tile (jt, tt): rows = keys t0 + 16 jt + 4 lg + i, column = query t0 + 16 tt + lr
#pragma unroll
      for (int jt = 0; jt < 2; ++jt)
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int32_t j = t0 + 16 * jt + 4 * lg + i, t = t0 + 16 * tt + lr;
            if (j > t || j >= s.T) PT[jt][tt][i] = 0.f;
          }
      // contraction slots of the second product follow the register order of P^T: slot e < 4 is
      // key t0 + 4 lg + e, slot e >= 4 key t0 + 16 + 4 lg + e - 4
      const bf16x8 ua = value_frag(vcol, VtRow, s.T, vi_lo, vi_hi,
                                   [&](int e) { return t0 + (e < 4 ? 4 * lg + e : 16 + 4 * lg + e - 4); });
      OT[0] = mfma16(ua, pack8(PT[0][0], PT[1][0]), OT[0]);
      OT[1] = mfma16(ua, pack8(PT[0][1], PT[1][1]), OT[1]);
    }
    // O^T tile tt: rows = value columns v0 + 4 lg + i, column = query t0 + 16 tt + lr
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int32_t t = t0 + 16 * tt + lr;
      if (t < s.T)
        *reinterpret_cast<float4*>(Oh + static_cast<int64_t>(t) * kValCols + v0 + 4 * lg) =
            make_float4(OT[tt][0], OT[tt][1], OT[tt][2], OT[tt][3]);
    }
  };
  // one pass over chunks [c0, c1): the next chunk's fragments travel while this one is computed.
  // Every branch here is uniform over the block (barriers inside).
  auto walk = [&](int32_t c0, int32_t c1, bool do_emit, bool causal, bool do_update) {
    const bool want_q = do_emit, want_k = do_emit && causal, want_kt = do_update;
    if (c0 < c1) fetch(32 * c0, want_q, want_k, want_kt);
    for (int32_t c = c0; c < c1; ++c) {
      __syncthreads();  // the previous chunk's fragments are no longer read
      park();
      __syncthreads();
      if (c + 1 < c1) fetch(32 * (c + 1), want_q, want_k, want_kt);
      if (do_emit) emit(32 * c, causal);
      if (do_update && !(do_emit && c + 1 == c1)) update(32 * c);  // the state after the last emitted chunk is not used
    }
  };

  const int32_t c_begin = min(nchunks, seg * cps), c_end = min(nchunks, c_begin + cps);
  float4* my_state = seg_state + (hs * G + seg) * (2 * MC * 64) + lane;
  if (PHASE == 0) {
    if (s.causal && seg == G - 1) return;  // nothing comes after the last segment (uniform over the block)
    walk(c_begin, c_end, false, false, true);
#pragma unroll
    for (int x = 0; x < 2 * MC; ++x) my_state[x * 64] = make_float4(S[x][0], S[x][1], S[x][2], S[x][3]);
    return;
  }
  if (G > 1) {
    const int32_t upto = s.causal ? seg : G;
    const float4* st = seg_state + hs * G * (2 * MC * 64) + lane;
    for (int32_t g = 0; g < upto; ++g) {
#pragma unroll
      for (int x = 0; x < 2 * MC; ++x) {
        const float4 v = st[(static_cast<int64_t>(g) * 2 * MC + x) * 64];
        S[x][0] += v.x; S[x][1] += v.y; S[x][2] += v.z; S[x][3] += v.w;
      }
    }
  } else if (!s.causal) {
    walk(0, nchunks, false, false, true);
  }
  walk(c_begin, c_end, true, s.causal != 0, s.causal != 0);
}

// [C_perf; V]: rows of 192 bf16; C_perf = sums / normaliser (column 128)
__global__ __launch_bounds__(256) void dec_concat_kernel(const float* __restrict__ acc, const uint16_t* __restrict__ V,
                                                         uint16_t* __restrict__ X, int64_t rows) {
  const int64_t gid = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  const int64_t row = gid / 24;
  const int part = static_cast<int>(gid % 24);  // 8 elements each
  if (row >= rows) return;
  uint4 o;
  if (part < 16) {
    const float* a = acc + row * kValCols;
    const float den = a[128];
    const float inv = den > 0.f ? 1.f / den : 0.f;
    const float4 x = *reinterpret_cast<const float4*>(a + 8 * part), y = *reinterpret_cast<const float4*>(a + 8 * part + 4);
    o.x = pack_bf16(x.x * inv, x.y * inv);
    o.y = pack_bf16(x.z * inv, x.w * inv);
    o.z = pack_bf16(y.x * inv, y.y * inv);
    o.w = pack_bf16(y.z * inv, y.w * inv);
  } else {
    o = *reinterpret_cast<const uint4*>(V + row * kHeadDim + 8 * (part - 16));
  }
  *reinterpret_cast<uint4*>(X + row * 192 + 8 * part) = o;
}

// ------------------------------------------------------------------------------------------
// implicit GEMM: out[pixel][cout] = act(bias[cout] + sum over (tap, c) in[pixel + tap][c] w[cout][tap][c]).
// One tap: a linear layer on rows.  Nine taps: a 3x3 convolution on a channels-last image
// [B][Tin][Xin][Cin], read through an optional nearest resize to Tv x Xv (source index
// floor(v * size / vsize)); zero outside the (virtual) image.  Computed transposed,
// C[cout][pixel] = W x X^T: the lane is the pixel, a lane holds four consecutive output channels.
// Wide layers (dec_conv_lds_kernel): block = 4 waves, wave = 64 pixels x up to 128 output channels
// (blockIdx.y picks the channel slab); the weights of the block's channels go through LDS in slabs of
// 128 contraction elements (fetched into registers one slab ahead), the pixels' operand fragments
// come straight from memory.
// ------------------------------------------------------------------------------------------
struct ConvArgs {
  const uint16_t* in;
  const uint16_t* w;     // [Cout][taps * Cin]
  const float* bias;     // [Cout]
  void* out;
  int32_t B, Tin, Xin, Cin, Tv, Xv, Tout, Xout, Cout, taps, stride_t, pad_top, relu;
  int32_t mode;          // 0: bf16 channels-last; 1: nu's last layer into the CNN's input image; 2: fp32 planes
  int32_t H, T, Wd, C;   // mode 1: rows are (b h, t); the image is [B][T][Wd][C]
  const int32_t* seq_len;
};

constexpr int kSlabK = 128;            // contraction elements of the weights staged per step
constexpr int kSlabRow = kSlabK + 8;   // halfwords per staged weight row (+16 B: b128 reads spread over the banks)

__global__ __launch_bounds__(256, 2) void dec_conv_lds_kernel(ConvArgs a) {
  // weights of the block's 128 output channels for one slab of the contraction, shared by the four waves
  __shared__ __attribute__((aligned(16))) uint16_t Wsl[128 * kSlabRow];
  const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const int lr = lane & 15, lg = lane >> 4;
  const int64_t npix = static_cast<int64_t>(a.B) * a.Tout * a.Xout;
  const int64_t pix0 = (static_cast<int64_t>(blockIdx.x) * 4 + wid) * 64;  // may lie past the end: the wave then only stages
  const int32_t cout0 = blockIdx.y * 128;
  const int32_t ntiles = min(8, (a.Cout - cout0 + 15) / 16);
  const int32_t ktot = a.taps * a.Cin;
  const int32_t nslabs = (ktot + kSlabK - 1) / kSlabK;
  // this lane's four pixels (operand columns)
  int32_t pb[4], pt[4], px[4];
  bool pok[4];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) {
    const int64_t p = pix0 + 16 * mt + lr;
    pok[mt] = p < npix;
    const int64_t pc = pok[mt] ? p : npix - 1;
    px[mt] = static_cast<int32_t>(pc % a.Xout);
    pt[mt] = static_cast<int32_t>((pc / a.Xout) % a.Tout);
    pb[mt] = static_cast<int32_t>(pc / (static_cast<int64_t>(a.Xout) * a.Tout));
  }
  floatx4 acc[8][4];
#pragma unroll
  for (int nt = 0; nt < 8; ++nt)
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) acc[nt][mt] = floatx4{0.f, 0.f, 0.f, 0.f};

  // staging role: 16-byte piece (tid & 15) of rows (tid >> 4) + 16 q, q < 8
  const int srow = tid >> 4, spart = tid & 15;
  uint4 wreg[8];
  auto fetch = [&](int32_t slab) {
    const int32_t k = slab * kSlabK + 8 * spart;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int32_t co = cout0 + srow + 16 * q;
      wreg[q] = (co < a.Cout && k < ktot) ? *reinterpret_cast<const uint4*>(a.w + static_cast<int64_t>(co) * ktot + k)
                                          : make_uint4(0u, 0u, 0u, 0u);
    }
  };
  auto park = [&]() {
#pragma unroll
    for (int q = 0; q < 8; ++q) *reinterpret_cast<uint4*>(&Wsl[(srow + 16 * q) * kSlabRow + 8 * spart]) = wreg[q];
  };
  fetch(0);
  park();
  __syncthreads();
  for (int32_t slab = 0; slab < nslabs; ++slab) {
    if (slab + 1 < nslabs) fetch(slab + 1);
    if (pix0 < npix) {
#pragma unroll
      for (int ks = 0; ks < kSlabK / 32; ++ks) {
        const int32_t kbase = slab * kSlabK + 32 * ks;
        if (kbase >= ktot) break;
        const int32_t k0 = kbase + 8 * lg;
        const bool kok = k0 < ktot;
        const int32_t tap = kok ? k0 / a.Cin : 0, c0 = kok ? k0 - tap * a.Cin : 0;
        const int32_t ky = a.taps == 9 ? tap / 3 : 0, kx = a.taps == 9 ? tap - 3 * ky : 0;
        bf16x8 xf[4];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
          const int32_t tv = pt[mt] * a.stride_t + ky - a.pad_top;
          const int32_t xv = a.taps == 9 ? px[mt] + kx - 1 : px[mt];
          const bool ok = kok && pok[mt] && tv >= 0 && tv < a.Tv && xv >= 0 && xv < a.Xv;
          if (ok) {
            const int32_t ts = a.Tv == a.Tin ? tv : static_cast<int32_t>((static_cast<int64_t>(tv) * a.Tin) / a.Tv);
            const int32_t xs = a.Xv == a.Xin ? xv : static_cast<int32_t>((static_cast<int64_t>(xv) * a.Xin) / a.Xv);
            xf[mt] = load8(a.in + ((static_cast<int64_t>(pb[mt]) * a.Tin + ts) * a.Xin + xs) * a.Cin + c0);
          } else {
            xf[mt] = zero8();
          }
        }
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) {
          if (nt < ntiles) {
            const bf16x8 wf = *reinterpret_cast<const bf16x8*>(&Wsl[(16 * nt + lr) * kSlabRow + 32 * ks + 8 * lg]);
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) acc[nt][mt] = mfma16(wf, xf[mt], acc[nt][mt]);
          }
        }
      }
    }
    __syncthreads();  // every wave is done with the slab
    if (slab + 1 < nslabs) {
      park();
      __syncthreads();
    }
  }
  if (pix0 >= npix) return;
  // epilogue: tile (nt, mt): rows = output channels cout0 + 16 nt + 4 lg + i, column = pixel lr of tile mt
#pragma unroll
  for (int nt = 0; nt < 8; ++nt) {
    if (nt >= ntiles) continue;
    const int32_t co = cout0 + 16 * nt + 4 * lg;
    if (co >= a.Cout) continue;
    float bv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) bv[i] = co + i < a.Cout ? a.bias[co + i] : 0.f;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
      if (!pok[mt]) continue;
      float v[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        v[i] = acc[nt][mt][i] + bv[i];
        if (a.relu) v[i] = fmaxf(v[i], 0.f);
      }
      const int64_t p = pix0 + 16 * mt + lr;
      if (a.mode == 0) {
        uint2 pk = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(a.out) + p * a.Cout + co) = pk;
      } else if (a.mode == 1) {
        // row p = (b h, t); outputs co .. co + 3 = compressed column co / 4, extra channels 0..3
        const int64_t n = p / a.T;
        const int32_t t = static_cast<int32_t>(p - n * a.T);
        const int32_t b = static_cast<int32_t>(n / a.H), h = static_cast<int32_t>(n - static_cast<int64_t>(b) * a.H);
        const int32_t len = a.seq_len ? min(max(a.seq_len[b], 0), a.T) : a.T;
        uint2 pk = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
        if (t >= len) pk = make_uint2(0u, 0u);
        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(a.out) +
                                  ((static_cast<int64_t>(b) * a.T + t) * a.Wd + (co >> 2)) * a.C + h * kCh) = pk;
      } else {
        float* o = static_cast<float*>(a.out);
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (co + i < a.Cout)
            o[((static_cast<int64_t>(pb[mt]) * a.Cout + co + i) * a.Tout + pt[mt]) * a.Xout + px[mt]] = v[i];
      }
    }
  }
}

// The same product for few output channels or a short contraction: wave = 32 pixels, every operand
// fragment straight from memory (the weights stay in the caches), no barriers.
__global__ __launch_bounds__(256) void dec_conv_kernel(ConvArgs a) {
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
  const int lr = lane & 15, lg = lane >> 4;
  const int64_t npix = static_cast<int64_t>(a.B) * a.Tout * a.Xout;
  const int64_t pix0 = (static_cast<int64_t>(blockIdx.x) * 4 + wid) * 32;
  if (pix0 >= npix) return;
  const int32_t cout0 = blockIdx.y * 128;
  const int32_t ntiles = min(8, (a.Cout - cout0 + 15) / 16);
  const int32_t ktot = a.taps * a.Cin;
  // this lane's two pixels (operand columns)
  int32_t pb[2], pt[2], px[2];
  bool pok[2];
#pragma unroll
  for (int mt = 0; mt < 2; ++mt) {
    const int64_t p = pix0 + 16 * mt + lr;
    pok[mt] = p < npix;
    const int64_t pc = pok[mt] ? p : npix - 1;
    px[mt] = static_cast<int32_t>(pc % a.Xout);
    pt[mt] = static_cast<int32_t>((pc / a.Xout) % a.Tout);
    pb[mt] = static_cast<int32_t>(pc / (static_cast<int64_t>(a.Xout) * a.Tout));
  }
  floatx4 acc[8][2];
#pragma unroll
  for (int nt = 0; nt < 8; ++nt) acc[nt][0] = acc[nt][1] = floatx4{0.f, 0.f, 0.f, 0.f};

  for (int32_t k0 = 8 * lg; k0 - 8 * lg < ktot; k0 += 32) {
    const bool kok = k0 < ktot;
    const int32_t tap = kok ? k0 / a.Cin : 0, c0 = kok ? k0 - tap * a.Cin : 0;
    const int32_t ky = a.taps == 9 ? tap / 3 : 0, kx = a.taps == 9 ? tap - 3 * ky : 0;
    bf16x8 xf[2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      const int32_t tv = pt[mt] * a.stride_t + ky - a.pad_top;
      const int32_t xv = a.taps == 9 ? px[mt] + kx - 1 : px[mt];
      const bool ok = kok && pok[mt] && tv >= 0 && tv < a.Tv && xv >= 0 && xv < a.Xv;
      if (ok) {
        const int32_t ts = a.Tv == a.Tin ? tv : static_cast<int32_t>((static_cast<int64_t>(tv) * a.Tin) / a.Tv);
        const int32_t xs = a.Xv == a.Xin ? xv : static_cast<int32_t>((static_cast<int64_t>(xv) * a.Xin) / a.Xv);
        xf[mt] = load8(a.in + ((static_cast<int64_t>(pb[mt]) * a.Tin + ts) * a.Xin + xs) * a.Cin + c0);
      } else {
        xf[mt] = zero8();
      }
    }
#pragma unroll
    for (int nt = 0; nt < 8; ++nt) {
      if (nt < ntiles) {
        const int32_t co = cout0 + 16 * nt + lr;
        const bf16x8 wf = (kok && co < a.Cout) ? load8(a.w + static_cast<int64_t>(co) * ktot + k0) : zero8();
        acc[nt][0] = mfma16(wf, xf[0], acc[nt][0]);
        acc[nt][1] = mfma16(wf, xf[1], acc[nt][1]);
      }
    }
  }
  // epilogue: tile (nt, mt): rows = output channels cout0 + 16 nt + 4 lg + i, column = pixel lr of tile mt
#pragma unroll
  for (int nt = 0; nt < 8; ++nt) {
    if (nt >= ntiles) continue;
    const int32_t co = cout0 + 16 * nt + 4 * lg;
    if (co >= a.Cout) continue;
    float bv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) bv[i] = co + i < a.Cout ? a.bias[co + i] : 0.f;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      if (!pok[mt]) continue;
      float v[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        v[i] = acc[nt][mt][i] + bv[i];
        if (a.relu) v[i] = fmaxf(v[i], 0.f);
      }
      const int64_t p = pix0 + 16 * mt + lr;
      if (a.mode == 0) {
        uint2 pk = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(a.out) + p * a.Cout + co) = pk;
      } else if (a.mode == 1) {
        // row p = (b h, t); outputs co .. co + 3 = compressed column co / 4, extra channels 0..3
        const int64_t n = p / a.T;
        const int32_t t = static_cast<int32_t>(p - n * a.T);
        const int32_t b = static_cast<int32_t>(n / a.H), h = static_cast<int32_t>(n - static_cast<int64_t>(b) * a.H);
        const int32_t len = a.seq_len ? min(max(a.seq_len[b], 0), a.T) : a.T;
        uint2 pk = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
        if (t >= len) pk = make_uint2(0u, 0u);
        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(a.out) +
                                  ((static_cast<int64_t>(b) * a.T + t) * a.Wd + (co >> 2)) * a.C + h * kCh) = pk;
      } else {
        float* o = static_cast<float*>(a.out);
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (co + i < a.Cout)
            o[((static_cast<int64_t>(pb[mt]) * a.Cout + co + i) * a.Tout + pt[mt]) * a.Xout + px[mt]] = v[i];
      }
    }
  }
}

// softmax over the K entries of each row [B][H][T][K] in place; rows at or past seq_len -> 0
__global__ __launch_bounds__(256) void dec_softmax_kernel(float* __restrict__ A, const int32_t* __restrict__ seq_len,
                                                          int64_t rows, int32_t H, int32_t T, int32_t K) {
  const int lane = threadIdx.x & 63;
  const int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int32_t t = static_cast<int32_t>(row % T);
  const int32_t b = static_cast<int32_t>(row / (static_cast<int64_t>(T) * H));
  const int32_t len = seq_len ? min(max(seq_len[b], 0), T) : T;
  float* r = A + row * K;
  if (t >= len) {
    for (int32_t c = lane; c < K; c += 64) r[c] = 0.f;
    return;
  }
  float mx = -INFINITY;
  for (int32_t c = lane; c < K; c += 64) mx = fmaxf(mx, r[c]);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
  float sum = 0.f;
  for (int32_t c = lane; c < K; c += 64) sum += __expf(r[c] - mx);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, 64);
  const float inv = 1.f / sum;
  for (int32_t c = lane; c < K; c += 64) r[c] = __expf(r[c] - mx) * inv;
}

// s_mix, s_prob = sigmoid(w . Z[row] + b); Z rows of 128 bf16; rows at or past seq_len -> 0
__global__ __launch_bounds__(256) void dec_scalers_kernel(const uint16_t* __restrict__ Z, const uint16_t* __restrict__ mix_w,
                                                          const float* __restrict__ mix_b, const uint16_t* __restrict__ prob_w,
                                                          const float* __restrict__ prob_b, float* __restrict__ s_mix,
                                                          float* __restrict__ s_prob, const int32_t* __restrict__ seq_len,
                                                          int64_t rows, int32_t H, int32_t T) {
  const int lane = threadIdx.x & 63;
  const int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const uint32_t z = *reinterpret_cast<const uint32_t*>(Z + row * 128 + 2 * lane);
  const uint32_t wm = *reinterpret_cast<const uint32_t*>(mix_w + 2 * lane), wp = *reinterpret_cast<const uint32_t*>(prob_w + 2 * lane);
  float am = bf16lo_to_f32(z) * bf16lo_to_f32(wm) + bf16hi_to_f32(z) * bf16hi_to_f32(wm);
  float ap = bf16lo_to_f32(z) * bf16lo_to_f32(wp) + bf16hi_to_f32(z) * bf16hi_to_f32(wp);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    am += __shfl_xor(am, off, 64);
    ap += __shfl_xor(ap, off, 64);
  }
  if (lane == 0) {
    const int32_t t = static_cast<int32_t>(row % T);
    const int32_t b = static_cast<int32_t>(row / (static_cast<int64_t>(T) * H));
    const int32_t len = seq_len ? min(max(seq_len[b], 0), T) : T;
    const bool on = t < len;
    if (s_mix) s_mix[row] = on ? 1.f / (1.f + __expf(-(am + mix_b[0]))) : 0.f;
    if (s_prob) s_prob[row] = on ? 1.f / (1.f + __expf(-(ap + prob_b[0]))) : 0.f;
  }
}

size_t up256(size_t b) { return (b + 255) & ~size_t(255); }

struct DecWs {
  size_t phiQ, phiK, phiKT, Vt, acc, seg, X, Z, hid, img, y1, y2, total;
  int32_t Tp, T1, Wd, C;
  int32_t G, cps;  // linear attention: segments per sequence, chunks of 32 tokens per segment
};
DecWs dec_layout(const Shape& s) {
  DecWs w{};
  const size_t N = static_cast<size_t>(s.N), T = static_cast<size_t>(s.T), B = N / s.H;
  w.Tp = static_cast<int32_t>((s.T + 63) / 64 * 64);
  w.T1 = s.causal ? s.T : (s.T + kCs - 1) / kCs;
  w.Wd = s.K / kCs;
  w.C = s.H * kCh;
  size_t off = 0;
  w.phiQ = off; off += up256(N * T * s.m * 2);
  w.phiK = off; off += up256(N * T * s.m * 2);
  w.phiKT = off; off += up256(N * s.m * static_cast<size_t>(w.Tp) * 2);
  w.Vt = off; off += up256(N * kHeadDim * static_cast<size_t>(w.Tp) * 2);
  w.acc = off; off += up256(N * T * kValCols * 4);
  {
    // segments: enough (head, slice, segment) waves to fill the chip, at least four chunks each
    const int32_t nchunks = w.Tp / 32;
    int32_t G = 1;
    while (static_cast<int64_t>(s.N) * 9 * G < 3072 && G < 16 && nchunks / (2 * G) >= 4) G *= 2;
    w.G = G;
    w.cps = (nchunks + G - 1) / G;
    w.seg = off;
    if (G > 1) off += up256(N * 9 * G * static_cast<size_t>(s.m) * 16 * 4);
  }
  w.X = off; off += up256(N * T * 192 * 2);
  w.Z = off; off += up256(N * T * 128 * 2);
  w.hid = off; off += up256(N * T * 128 * 2);
  w.img = off; off += up256(B * T * w.Wd * w.C * 2);
  w.y1 = off; off += up256(B * static_cast<size_t>(w.T1) * w.Wd * w.C * 2);
  w.y2 = off; off += up256(B * static_cast<size_t>(w.T1) * w.Wd * w.C * 2);
  w.total = off;
  return w;
}

// ------------------------------------------------------------------------------------------
// 3x3 convolutions with the input window in LDS.  A block of eight waves computes a tile of output
// pixels (each wave 64 of them: RW rows x CW columns, RW CW = 64) for a slab of up to 16 NT output
// channels.  The tile's input halo -- every (virtual, i.e. resized) pixel any of its taps touches,
// zeros outside the image -- and the slab's weights are parked in LDS once per channel chunk, the
// weights in operand-fragment order, the pixels with an odd number of 16-byte units per pixel so
// that the 16 pixels of an operand tile hit different banks.  Each input pixel is then read from
// memory once per tile instead of once per tap.  The contraction runs over (tap, channel) of the
// chunk flattened in units of 8 channels, one unit per lane group and step; a lane advances its own
// (tap, unit) position without divisions.
// ------------------------------------------------------------------------------------------
struct Conv3Args {
  ConvArgs a;
  int32_t t_shift, x_shift;      // log2 of the nearest-resize ratios (virtual / stored size)
  int32_t CK, nchunk, P, pp_log; // channels per chunk, chunks, 16-byte units per pixel and chunk, log2 of P rounded up
  int32_t ksteps;                // contraction steps per chunk
  int32_t cw_log;                // log2 of the columns a wave covers (4..6); rows per wave = 64 >> cw_log
  int32_t rows_out, cols_out, halo_rows, halo_cols, px_units;  // tile geometry; px_units odd
  int32_t tiles_t, tiles_x;
};
constexpr int kConv3Waves = 8;

template <int NT>
__global__ __launch_bounds__(64 * kConv3Waves) void dec_conv3_kernel(Conv3Args g) {
  extern __shared__ __attribute__((aligned(16))) uint4 lds3[];
  const ConvArgs& a = g.a;
  uint4* halo = lds3;                                                        // [halo_rows][halo_cols][px_units]
  uint4* wts = lds3 + static_cast<int64_t>(g.halo_rows) * g.halo_cols * g.px_units;  // [kstep][NT][64]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lr = lane & 15, lg = lane >> 4;
  uint32_t bid = blockIdx.x;
  const int32_t tx = static_cast<int32_t>(bid % static_cast<uint32_t>(g.tiles_x)); bid /= static_cast<uint32_t>(g.tiles_x);
  const int32_t tt = static_cast<int32_t>(bid % static_cast<uint32_t>(g.tiles_t));
  const int64_t b = bid / static_cast<uint32_t>(g.tiles_t);
  const int32_t t0 = tt * g.rows_out, x0 = tx * g.cols_out;     // first output pixel of the tile
  const int32_t tv0 = t0 * a.stride_t - a.pad_top, xv0 = x0 - 1;  // first virtual input pixel of the halo
  const int32_t cout0 = blockIdx.y * (16 * NT);
  const int32_t ktot = 9 * a.Cin;
  const uint16_t* img = a.in + b * a.Tin * a.Xin * a.Cin;

  floatx4 acc[NT][4];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt)
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) acc[nt][mt] = floatx4{0.f, 0.f, 0.f, 0.f};
  // this lane's pixel in each of the wave's four operand tiles: row and column inside the output tile
  const int rw = 64 >> g.cw_log, ctiles = (1 << g.cw_log) >> 4;  // rows per wave, 16-pixel tiles per row
  int32_t prow[4], pcol[4];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) {
    prow[mt] = wid * rw + mt / ctiles;
    pcol[mt] = (mt % ctiles) * 16 + lr;
  }

  for (int32_t ch = 0; ch < g.nchunk; ++ch) {
    if (ch > 0) __syncthreads();  // the previous chunk is no longer read
    const int32_t cbase = ch * g.CK;
    // halo: thread = (pixel, 16-byte unit); units past P idle
    {
      const int32_t unit = tid & ((1 << g.pp_log) - 1);
      const int32_t npx = g.halo_rows * g.halo_cols;
      for (int32_t px = tid >> g.pp_log; px < npx; px += (64 * kConv3Waves) >> g.pp_log) {
        if (unit >= g.P) continue;
        const int32_t hr = px / g.halo_cols, hc = px - hr * g.halo_cols;
        const int32_t tv = tv0 + hr, xv = xv0 + hc;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (static_cast<uint32_t>(tv) < static_cast<uint32_t>(a.Tv) && static_cast<uint32_t>(xv) < static_cast<uint32_t>(a.Xv)) {
          const int32_t ts = tv >> g.t_shift, xs = xv >> g.x_shift;
          v = *reinterpret_cast<const uint4*>(img + (static_cast<int64_t>(ts) * a.Xin + xs) * a.Cin + cbase + 8 * unit);
        }
        halo[static_cast<int64_t>(px) * g.px_units + unit] = v;
      }
    }
    // weights of the chunk: fragment (step, tile, lane) = channels cbase + 8 cu .. + 7 of tap `tap` for
    // output channel cout0 + 16 nt + lane % 16, with (tap, cu) = unit 4 step + lane / 16 of the chunk
    for (int32_t id = tid; id < g.ksteps * NT * 64; id += 64 * kConv3Waves) {
      const int32_t fl = id & 63, q = id >> 6, nt = q % NT, ks = q / NT;
      const int32_t u = 4 * ks + (fl >> 4), tap = u / g.P, cu = u - tap * g.P;
      const int32_t co = cout0 + 16 * nt + (fl & 15);
      uint4 v = make_uint4(0u, 0u, 0u, 0u);
      if (tap < 9 && co < a.Cout)
        v = *reinterpret_cast<const uint4*>(a.w + static_cast<int64_t>(co) * ktot + tap * a.Cin + cbase + 8 * cu);
      wts[id] = v;
    }
    __syncthreads();
    int32_t tap = 0, cu = lg;
    while (cu >= g.P) { cu -= g.P; ++tap; }
    for (int32_t ks = 0; ks < g.ksteps; ++ks) {
      const bool valid = tap < 9;
      const int32_t ky = (tap * 11) >> 5, kx = tap - 3 * ky;  // tap / 3 and tap % 3 for tap <= 8
      bf16x8 xf[4];
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) {
        const int32_t hr = prow[mt] * a.stride_t + ky, hc = pcol[mt] + kx;
        const uint4 v = halo[valid ? (static_cast<int64_t>(hr) * g.halo_cols + hc) * g.px_units + cu : 0];
        xf[mt] = valid ? __builtin_bit_cast(bf16x8, v) : zero8();
      }
      const uint4* wk = wts + (static_cast<int64_t>(ks) * NT) * 64 + lane;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const bf16x8 wf = __builtin_bit_cast(bf16x8, wk[nt * 64]);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) acc[nt][mt] = mfma16(wf, xf[mt], acc[nt][mt]);
      }
      cu += 4;
      while (cu >= g.P) { cu -= g.P; ++tap; }
    }
  }
  // epilogue: tile (nt, mt): rows = output channels cout0 + 16 nt + 4 lg + i, column = this lane's pixel of tile mt
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int32_t co = cout0 + 16 * nt + 4 * lg;
    if (co >= a.Cout) continue;
    float bv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) bv[i] = co + i < a.Cout ? a.bias[co + i] : 0.f;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
      const int32_t t = t0 + prow[mt], x = x0 + pcol[mt];
      if (prow[mt] >= g.rows_out || pcol[mt] >= g.cols_out || t >= a.Tout || x >= a.Xout) continue;
      float v[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        v[i] = acc[nt][mt][i] + bv[i];
        if (a.relu) v[i] = fmaxf(v[i], 0.f);
      }
      if (a.mode == 0) {
        const uint2 pk = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(a.out) + ((b * a.Tout + t) * a.Xout + x) * a.Cout + co) = pk;
      } else {
        float* o = static_cast<float*>(a.out);
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (co + i < a.Cout) o[((b * a.Cout + co + i) * a.Tout + t) * a.Xout + x] = v[i];
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// Linear layers (one tap) on rows of at most 256 inputs: the block parks the weights of its slab of
// up to 128 output channels in LDS (operand-fragment order) and walks tiles of 32 rows; a wave
// requests the operand fragments of its next tile (every step of the contraction) before it
// multiplies the current one, so the row reads, which bound these layers, overlap the products.
// ------------------------------------------------------------------------------------------
constexpr int kLinSteps = 8;  // contraction steps of 32 a row may have (Cin <= 256)

__global__ __launch_bounds__(256) void dec_linear_kernel(ConvArgs a, int32_t tiles_per_wave) {
  extern __shared__ __attribute__((aligned(16))) uint4 wlin[];  // [kstep][8][64]
  const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const int lr = lane & 15, lg = lane >> 4;
  const int64_t nrows = static_cast<int64_t>(a.B) * a.Tout * a.Xout;
  const int32_t cout0 = blockIdx.y * 128;
  const int32_t ntiles_c = min(8, (a.Cout - cout0 + 15) / 16);
  const int32_t ksteps = (a.Cin + 31) / 32;
  for (int32_t id = tid; id < ksteps * 8 * 64; id += 256) {
    const int32_t fl = id & 63, nt = (id >> 6) & 7, ks = id >> 9;
    const int32_t co = cout0 + 16 * nt + (fl & 15), k0 = 32 * ks + 8 * (fl >> 4);
    // unconditional load from a clamped address, cleared where the slab overruns the matrix
    const uint4 v = *reinterpret_cast<const uint4*>(a.w + static_cast<int64_t>(min(co, a.Cout - 1)) * a.Cin + min(k0, a.Cin - 8));
    wlin[id] = (co < a.Cout && k0 < a.Cin) ? v : make_uint4(0u, 0u, 0u, 0u);
  }
  __syncthreads();
  const int64_t ntile = (nrows + 31) / 32;
  const int64_t wave = static_cast<int64_t>(blockIdx.x) * 4 + wid;
  int64_t tile = wave * tiles_per_wave;
  const int64_t tile_end = min(ntile, tile + tiles_per_wave);
  bf16x8 nx[kLinSteps][2];
  auto request = [&](int64_t tl) {
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      int64_t r = min(tl * 32 + 16 * mt + lr, nrows - 1);
      if (a.mode == 1) {
        // walk the rows (b h, t) as (b, t, h), heads fastest: the lanes of a wave then write next to
        // each other in the channels-last image
        const int64_t q = r / a.H, h = r - q * a.H, b = q / a.T, t = q - b * a.T;
        r = (b * a.H + h) * a.T + t;
      }
      // a lane whose piece lies past the row's channels reads the row's last piece instead and
      // clears it, so no load sits behind a per-lane branch and all of a tile's loads are in flight
      // together
      const uint16_t* row = a.in + r * a.Cin;
#pragma unroll
      for (int ks = 0; ks < kLinSteps; ++ks)
        if (ks < ksteps) {
          const int32_t k0 = 32 * ks + 8 * lg;
          const bf16x8 x = load8(row + min(k0, a.Cin - 8));
          nx[ks][mt] = k0 < a.Cin ? x : zero8();
        }
    }
  };
  if (tile < tile_end) request(tile);
  for (; tile < tile_end; ++tile) {
    bf16x8 xf[kLinSteps][2];
#pragma unroll
    for (int ks = 0; ks < kLinSteps; ++ks) { xf[ks][0] = nx[ks][0]; xf[ks][1] = nx[ks][1]; }
    if (tile + 1 < tile_end) request(tile + 1);
    floatx4 acc[8][2];
#pragma unroll
    for (int nt = 0; nt < 8; ++nt) acc[nt][0] = acc[nt][1] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < kLinSteps; ++ks) {
      if (ks < ksteps) {
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) {
          if (nt < ntiles_c) {
            const bf16x8 wf = __builtin_bit_cast(bf16x8, wlin[(ks * 8 + nt) * 64 + lane]);
            acc[nt][0] = mfma16(wf, xf[ks][0], acc[nt][0]);
            acc[nt][1] = mfma16(wf, xf[ks][1], acc[nt][1]);
          }
        }
      }
    }
    // mode 1: where the lane's two rows (b, t, h) land in the channels-last image, and whether they
    // lie inside their sequence -- once per tile, not once per channel tile (two 64-bit divisions
    // and a load each)
    int64_t orow[2] = {0, 0};
    bool live[2] = {true, true};
    if (a.mode != 0) {
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        const int64_t pp = min(tile * 32 + 16 * mt + lr, nrows - 1);
        const int64_t q = pp / a.H;
        const int32_t h = static_cast<int32_t>(pp - q * a.H);
        const int32_t b = static_cast<int32_t>(q / a.T), t = static_cast<int32_t>(q - static_cast<int64_t>(b) * a.T);
        const int32_t len = a.seq_len ? min(max(a.seq_len[b], 0), a.T) : a.T;
        live[mt] = t < len;
        orow[mt] = (static_cast<int64_t>(b) * a.T + t) * a.Wd * a.C + h * kCh;
      }
    }
    // epilogue: tile (nt, mt): rows = output channels cout0 + 16 nt + 4 lg + i, column = row lr of tile mt
#pragma unroll
    for (int nt = 0; nt < 8; ++nt) {
      if (nt >= ntiles_c) continue;
      const int32_t co = cout0 + 16 * nt + 4 * lg;
      if (co >= a.Cout) continue;
      float bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) bv[i] = co + i < a.Cout ? a.bias[co + i] : 0.f;
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        const int64_t pp = tile * 32 + 16 * mt + lr;
        if (pp >= nrows) continue;
        float v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          v[i] = acc[nt][mt][i] + bv[i];
          if (a.relu) v[i] = fmaxf(v[i], 0.f);
        }
        uint2 pk = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
        if (a.mode == 0) {
          *reinterpret_cast<uint2*>(static_cast<uint16_t*>(a.out) + pp * a.Cout + co) = pk;
        } else {
          // row pp = (b, t, h); outputs co .. co + 3 = compressed column co / 4, extra channels 0..3
          if (!live[mt]) pk = make_uint2(0u, 0u);
          *reinterpret_cast<uint2*>(static_cast<uint16_t*>(a.out) + orow[mt] + static_cast<int64_t>(co >> 2) * a.C) = pk;
        }
      }
    }
  }
}

// log2 of virtual / stored size when that ratio is a power of two, else -1
int32_t resize_shift(int32_t vsize, int32_t size) {
  for (int32_t sh = 0; sh < 16; ++sh)
    if ((static_cast<int64_t>(size) << sh) == vsize) return sh;
  return -1;
}

// Geometry of the LDS-window kernel for one layer; false when the layer does not fit it (then the
// direct kernels run).  The channel chunk is the largest divisor of Cin (in units of 8 channels)
// whose halo and weights fit the LDS budget.
constexpr size_t kConv3LdsBudget = 72 << 10;  // two blocks per CU overlap one block's staging with the other's products
bool conv3_plan(const ConvArgs& a, Conv3Args* g, int32_t* nt_out, size_t* lds_out) {
  if (a.taps != 9 || a.Cin % 8 != 0 || (a.mode != 0 && a.mode != 2)) return false;
  if (a.mode == 0 && a.Cout % 4 != 0) return false;
  const int32_t ts = resize_shift(a.Tv, a.Tin), xs = resize_shift(a.Xv, a.Xin);
  if (ts < 0 || xs < 0) return false;
  const int32_t slab = a.Cout < 128 ? a.Cout : 128;
  const int32_t nt = (slab + 15) / 16;
  int32_t cw_log = 6;
  while (cw_log > 4 && (1 << (cw_log - 1)) >= a.Xout) --cw_log;
  const int32_t rows_out = kConv3Waves * (64 >> cw_log), cols_out = 1 << cw_log;
  const int32_t halo_rows = (rows_out - 1) * a.stride_t + 3, halo_cols = cols_out + 2;
  const int32_t units = a.Cin / 8;
  for (int32_t nchunk = 1; nchunk <= units; ++nchunk) {
    if (units % nchunk != 0) continue;
    const int32_t P = units / nchunk;
    const int32_t px_units = P | 1;
    const int32_t ksteps = (9 * P + 3) / 4;
    const size_t lds = (static_cast<size_t>(halo_rows) * halo_cols * px_units + static_cast<size_t>(ksteps) * nt * 64) * 16;
    if (lds > kConv3LdsBudget) continue;
    int32_t pp_log = 0;
    while ((1 << pp_log) < P) ++pp_log;
    g->a = a; g->t_shift = ts; g->x_shift = xs; g->CK = 8 * P; g->nchunk = nchunk; g->P = P; g->pp_log = pp_log;
    g->ksteps = ksteps; g->cw_log = cw_log; g->rows_out = rows_out; g->cols_out = cols_out;
    g->halo_rows = halo_rows; g->halo_cols = halo_cols; g->px_units = px_units;
    g->tiles_t = (a.Tout + rows_out - 1) / rows_out; g->tiles_x = (a.Xout + cols_out - 1) / cols_out;
    *nt_out = nt; *lds_out = lds;
    return true;
  }
  return false;
}

// a failed attribute call stays the runtime's last error, which the caller reports
template <int NT>
void launch_conv3(const Conv3Args& g, uint32_t slabs, size_t lds, hipStream_t st) {
  if (lds > (64u << 10) &&
      hipFuncSetAttribute(reinterpret_cast<const void*>(&dec_conv3_kernel<NT>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)) != hipSuccess)
    return;
  const uint32_t blocks = static_cast<uint32_t>(g.a.B) * g.tiles_t * g.tiles_x;
  hipLaunchKernelGGL(dec_conv3_kernel<NT>, dim3(blocks, slabs), dim3(64 * kConv3Waves), lds, st, g);
}

void launch_conv(const ConvArgs& a, hipStream_t st) {
  const int64_t npix = static_cast<int64_t>(a.B) * a.Tout * a.Xout;
  if (a.taps == 1 && a.Cin % 8 == 0 && a.Cin <= 32 * kLinSteps && a.Cout % 4 == 0 && (a.mode == 0 || a.mode == 1)) {
    // tiles per wave: whole numbers, about eight waves per CU
    const int64_t ntile = (npix + 31) / 32;
    const int32_t per_wave = static_cast<int32_t>((ntile + 2047) / 2048);
    const int64_t waves = (ntile + per_wave - 1) / per_wave;
    const size_t lds = static_cast<size_t>((a.Cin + 31) / 32) * 8 * 1024;
    hipLaunchKernelGGL(dec_linear_kernel, dim3(static_cast<uint32_t>((waves + 3) / 4), static_cast<uint32_t>((a.Cout + 127) / 128)),
                       dim3(256), lds, st, a, per_wave);
    return;
  }
  Conv3Args g{};
  int32_t nt = 0;
  size_t lds = 0;
  if (conv3_plan(a, &g, &nt, &lds)) {
    const uint32_t slabs3 = static_cast<uint32_t>((a.Cout + 16 * nt - 1) / (16 * nt));
    switch (nt) {
      case 1: launch_conv3<1>(g, slabs3, lds, st); break;
      case 2: launch_conv3<2>(g, slabs3, lds, st); break;
      case 3: launch_conv3<3>(g, slabs3, lds, st); break;
      case 4: launch_conv3<4>(g, slabs3, lds, st); break;
      case 5: launch_conv3<5>(g, slabs3, lds, st); break;
      case 6: launch_conv3<6>(g, slabs3, lds, st); break;
      case 7: launch_conv3<7>(g, slabs3, lds, st); break;
      default: launch_conv3<8>(g, slabs3, lds, st); break;
    }
    return;
  }
  const uint32_t slabs = static_cast<uint32_t>((a.Cout + 127) / 128);
  if (a.Cout >= 96 && a.taps * a.Cin >= 512) {
    hipLaunchKernelGGL(dec_conv_lds_kernel, dim3(static_cast<uint32_t>((npix + 255) / 256), slabs), dim3(256), 0, st, a);
  } else {
    hipLaunchKernelGGL(dec_conv_kernel, dim3(static_cast<uint32_t>((npix + 127) / 128), slabs), dim3(256), 0, st, a);
  }
}

}  // namespace

bool decoder_supported(const Shape& s, sea_dtype dt) {
  if (dt != SEA_BF16) return false;
  if (s.m != 64 && s.m != 128 && s.m != 256) return false;
  if (s.K % kCs != 0 || s.K > 1024) return false;
  if ((s.H * kCh) % 8 != 0) return false;  // operand fragments are 8 channels
  if (s.geometry != 0) return false;
  return true;
}

size_t decoder_workspace(const Shape& s) { return dec_layout(s).total; }

hipError_t launch_decoder_estimate(const Shape& s, const sea_decoder_weights& wt, const uint16_t* Q, const uint16_t* K,
                                   const uint16_t* V, const uint16_t* W, float* A_hat, float* s_mix, float* s_prob,
                                   void* ws, hipStream_t st) {
  if (!decoder_supported(s, SEA_BF16)) return hipErrorNotSupported;
  const DecWs lay = dec_layout(s);
  char* base = static_cast<char*>(ws);
  auto u16 = [&](size_t off) { return reinterpret_cast<uint16_t*>(base + off); };
  const double l2e = 1.4426950408889634;
  const float c_dot = static_cast<float>(l2e * sqrt(static_cast<double>(s.scale)));
  const float c_norm = static_cast<float>(l2e * 0.5 * static_cast<double>(s.scale));
  const int32_t B = s.N / s.H;
  const int64_t rows = static_cast<int64_t>(s.N) * s.T;
  {
    StageScope scope(SEA_STAGE_FEATURES, st);
    hipLaunchKernelGGL(dec_features_kernel, dim3(2u * s.N * (lay.Tp / 64)), dim3(256), 0, st, s, lay.Tp, Q, K, V, W,
                       u16(lay.phiQ), u16(lay.phiK), u16(lay.phiKT), u16(lay.Vt), c_dot, c_norm);
  }
  {
    StageScope scope(SEA_STAGE_STATE, st);
    float* acc = reinterpret_cast<float*>(base + lay.acc);
    const dim3 grid(static_cast<uint32_t>(s.N) * lay.G);
    float4* seg = reinterpret_cast<float4*>(base + lay.seg);
#define SEA_LINATTN(MC_)                                                                                  \
    do {                                                                                                  \
      if (lay.G > 1)                                                                                      \
        hipLaunchKernelGGL((dec_linattn_kernel<MC_, 0>), grid, dim3(64 * kLinWaves), 0, st, s, lay.Tp, lay.G, lay.cps, \
                           u16(lay.phiQ), u16(lay.phiK), u16(lay.phiKT), u16(lay.Vt), acc, seg);          \
      hipLaunchKernelGGL((dec_linattn_kernel<MC_, 1>), grid, dim3(64 * kLinWaves), 0, st, s, lay.Tp, lay.G, lay.cps,   \
                         u16(lay.phiQ), u16(lay.phiK), u16(lay.phiKT), u16(lay.Vt), acc, seg);            \
    } while (0)
    switch (s.m) {
      case 64: SEA_LINATTN(2); break;
      case 128: SEA_LINATTN(4); break;
      default: SEA_LINATTN(8); break;
    }
#undef SEA_LINATTN
    hipLaunchKernelGGL(dec_concat_kernel, dim3(static_cast<uint32_t>((rows * 24 + 255) / 256)), dim3(256), 0, st, acc, V,
                       u16(lay.X), rows);
  }
  StageScope scope(SEA_STAGE_CONTRACT, st);
  ConvArgs a{};
  a.seq_len = s.seq_len; a.H = s.H; a.T = s.T; a.Wd = lay.Wd; a.C = lay.C;
  // mu: [rows][192] -> Z [rows][128], ReLU
  a.in = u16(lay.X); a.w = static_cast<const uint16_t*>(wt.mu_w); a.bias = wt.mu_b; a.out = u16(lay.Z);
  // a linear layer is the one-tap case on an "image" of N x T rows
  a.B = 1; a.Tin = a.Tv = a.Tout = s.N; a.Xin = a.Xv = a.Xout = s.T;
  a.Cin = 192; a.Cout = 128; a.taps = 1; a.stride_t = 1; a.pad_top = 0; a.relu = 1; a.mode = 0;
  launch_conv(a, st);
  hipLaunchKernelGGL(dec_scalers_kernel, dim3(static_cast<uint32_t>((rows + 3) / 4)), dim3(256), 0, st, u16(lay.Z),
                     static_cast<const uint16_t*>(wt.mix_w), wt.mix_b, static_cast<const uint16_t*>(wt.prob_w), wt.prob_b,
                     s_mix, s_prob, s.seq_len, rows, s.H, s.T);
  // nu, first layer: Z -> hidden, ReLU
  a.in = u16(lay.Z); a.w = static_cast<const uint16_t*>(wt.nu1_w); a.bias = wt.nu1_b; a.out = u16(lay.hid);
  a.Cin = 128; a.Cout = 128;
  launch_conv(a, st);
  // nu, second layer: hidden -> the CNN's input image [B][T][Wd][C], channels h c_h + ch
  a.in = u16(lay.hid); a.w = static_cast<const uint16_t*>(wt.nu2_w); a.bias = wt.nu2_b; a.out = u16(lay.img);
  a.Cin = 128; a.Cout = lay.Wd * kCh; a.relu = 0; a.mode = 1;
  launch_conv(a, st);
  // conv 1: [B][T][Wd][C] -> [B][T1][Wd][C], ReLU.  Causal: rows t-2..t; else stride c_s, rows i c_s - 1 .. + 1
  a.in = u16(lay.img); a.w = static_cast<const uint16_t*>(wt.conv1_w); a.bias = wt.conv1_b; a.out = u16(lay.y1);
  a.B = B; a.Tin = a.Tv = s.T; a.Xin = a.Xv = lay.Wd; a.Cin = lay.C;
  a.Tout = lay.T1; a.Xout = lay.Wd; a.Cout = lay.C; a.taps = 9;
  a.stride_t = s.causal ? 1 : kCs; a.pad_top = s.causal ? 2 : 1; a.relu = 1; a.mode = 0;
  launch_conv(a, st);
  // conv 2
  a.in = u16(lay.y1); a.w = static_cast<const uint16_t*>(wt.conv2_w); a.bias = wt.conv2_b; a.out = u16(lay.y2);
  a.Tin = a.Tv = lay.T1; a.stride_t = 1;
  launch_conv(a, st);
  // conv 3 on the image resized to T x K (nearest, on the read) -> logits [B][H][T][K] fp32
  a.in = u16(lay.y2); a.w = static_cast<const uint16_t*>(wt.conv3_w); a.bias = wt.conv3_b; a.out = A_hat;
  a.Tv = s.T; a.Xv = s.K; a.Tout = s.T; a.Xout = s.K; a.Cout = s.H; a.relu = 0; a.mode = 2;
  launch_conv(a, st);
  hipLaunchKernelGGL(dec_softmax_kernel, dim3(static_cast<uint32_t>((rows + 3) / 4)), dim3(256), 0, st, A_hat, s.seq_len,
                     rows, s.H, s.T, s.K);
  return hipGetLastError();
}

}  // namespace sea

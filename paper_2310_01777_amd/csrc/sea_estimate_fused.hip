// Fused random-feature estimate for the common shapes (bf16, K | T, column width a power of two
// up to 128, m in {64, 128, 256}, K <= 256): two kernels; no feature tensor reaches HBM.  For causal
// columns wider than 16 keys the key side also leaves, per 16-key tile, the sum of the rounded
// features of the column's earlier tiles, split into three bf16 planes (24 bits, i.e. the fp32
// sum itself), which is all the own-column term needs from outside the wave.
// (Sec. 3 "Performer (FAVOR+)", Sec. 3.1 "Attention Matrix Estimation".)
//
//   key_state_kernel      phi(K) on the matrix cores -> per-column sums -> state (bf16, K x m)
//   estimate_rows_kernel  phi(Q) on the matrix cores, kept in registers as MFMA fragments ->
//                         A_hat tile = phi(Q) state^T (state streamed through LDS) -> causal
//                         masking, the row's own column from phi(Q) phi(K_own)^T with a
//                         lower-triangular mask -> row normalisation -> fp32 A_hat (optional)
//                         -> per-row top-k^ in registers -> selected-column bits (optional)
//
// Both projections are computed transposed, C[feature][row] = W X^T with v_mfma_f32_16x16x32_bf16,
// so lane l owns row l % 16 and, per 16-feature tile ft, the four features 16 ft + 4 (l / 16) + i.
// Two consecutive tiles give a lane 8 values = one MFMA operand fragment; the contraction slot
// <-> feature map this implies (slot 8 lg + e of chunk kc <-> feature 32 kc + 16 (e / 4) + 4 lg +
// e % 4) is used consistently for phi(Q), phi(K) and the stored state ("fragment order"), so
// accumulators feed the next product without any shuffle or memory round trip.
#include <algorithm>

#include "sea_internal.h"
#include "sea_rowlanes.h"

namespace sea {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef int intx4 __attribute__((ext_vector_type(4)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef unsigned short ushort2v __attribute__((ext_vector_type(2)));

constexpr int kWRow = 72;  // halfwords per staged W row (128 B + 16 B pad): conflict-free b128 reads

__device__ __forceinline__ floatx4 mfma16(bf16x8 a, bf16x8 b, floatx4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
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
// eight floats (two feature tiles x four features) -> one operand fragment, RNE
__device__ __forceinline__ bf16x8 pack8(const float* lo4, const float* hi4) {
  uint4 u;
  u.x = pack_bf16(lo4[0], lo4[1]);
  u.y = pack_bf16(lo4[2], lo4[3]);
  u.z = pack_bf16(hi4[0], hi4[1]);
  u.w = pack_bf16(hi4[2], hi4[3]);
  return __builtin_bit_cast(bf16x8, u);
}

// sum over the 16 lanes of a DPP row (lanes with equal l / 16); every lane gets the total
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false);
  return x + __int_as_float(y);
}
constexpr int kQuadXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kQuadXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kRowHalfMirror = 0x141;  // lane i <-> 7 - i within each 8
constexpr int kRowMirror = 0x140;      // lane i <-> 15 - i within each 16
// all-reduce over aligned groups of W lanes (W = 1, 2, 4, 8, 16) of a row
template <int W>
__device__ __forceinline__ uint32_t group_sum_u(uint32_t x) {  // integer counts
  if (W >= 2) x += static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), kQuadXor1, 0xf, 0xf, false));
  if (W >= 4) x += static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), kQuadXor2, 0xf, 0xf, false));
  if (W >= 8) x += static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), kRowHalfMirror, 0xf, 0xf, false));
  if (W >= 16) x += static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), kRowMirror, 0xf, 0xf, false));
  return x;
}
// four independent 16-lane sums, step by step
__device__ __forceinline__ void group_sum4_u(uint32_t (&x)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) x[i] += static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x[i]), kQuadXor1, 0xf, 0xf, false));
#pragma unroll
  for (int i = 0; i < 4; ++i) x[i] += static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x[i]), kQuadXor2, 0xf, 0xf, false));
#pragma unroll
  for (int i = 0; i < 4; ++i) x[i] += static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x[i]), kRowHalfMirror, 0xf, 0xf, false));
#pragma unroll
  for (int i = 0; i < 4; ++i) x[i] += static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x[i]), kRowMirror, 0xf, 0xf, false));
}
template <int W>
__device__ __forceinline__ uint32_t group_max_u(uint32_t x) {
  if (W >= 2) x = max(x, static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), kQuadXor1, 0xf, 0xf, false)));
  if (W >= 4) x = max(x, static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), kQuadXor2, 0xf, 0xf, false)));
  if (W >= 8) x = max(x, static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), kRowHalfMirror, 0xf, 0xf, false)));
  if (W >= 16) x = max(x, static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), kRowMirror, 0xf, 0xf, false)));
  return x;
}
template <int W>
__device__ __forceinline__ float group_sum(float x) {
  if (W >= 2) x = dpp_add<kQuadXor1>(x);
  if (W >= 4) x = dpp_add<kQuadXor2>(x);
  if (W >= 8) x = dpp_add<kRowHalfMirror>(x);
  if (W >= 16) x = dpp_add<kRowMirror>(x);
  return x;
}

// stage W (m rows of 64 bf16) into LDS with padded rows
__device__ __forceinline__ void stage_w(const uint16_t* __restrict__ W, uint16_t* Ws, int m, int tid) {
  for (int x = tid; x < m * 8; x += 256) {
    const int r = x >> 3, part = x & 7;
    *reinterpret_cast<uint4*>(&Ws[r * kWRow + part * 8]) =
        *reinterpret_cast<const uint4*>(W + r * kHeadDim + part * 8);
  }
}

// raw projections w_f . x of 16 rows x m features: dots[ft][i] for feature 16 ft + 4 lg + i
template <int MC>
__device__ __forceinline__ void project_dots(const uint16_t* Ws, bf16x8 x0, bf16x8 x1, int lr, int lg,
                                             floatx4 (&dots)[2 * MC]) {
#pragma unroll
  for (int ft = 0; ft < 2 * MC; ++ft) {
    const uint16_t* w = &Ws[(ft * 16 + lr) * kWRow + 8 * lg];
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
    acc = mfma16(*reinterpret_cast<const bf16x8*>(w), x0, acc);
    dots[ft] = mfma16(*reinterpret_cast<const bf16x8*>(w + 32), x1, acc);
  }
}

// exponent arguments (log2 domain) of 16 rows x m features: arg[ft][i] for feature 16 ft + 4 lg + i
template <int MC>
__device__ __forceinline__ void project(const uint16_t* Ws, bf16x8 x0, bf16x8 x1, int lr, int lg,
                                        float c_dot, float bias, floatx4 (&arg)[2 * MC]) {
#pragma unroll
  for (int ft = 0; ft < 2 * MC; ++ft) {
    const uint16_t* w = &Ws[(ft * 16 + lr) * kWRow + 8 * lg];
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
    acc = mfma16(*reinterpret_cast<const bf16x8*>(w), x0, acc);
    acc = mfma16(*reinterpret_cast<const bf16x8*>(w + 32), x1, acc);
#pragma unroll
    for (int i = 0; i < 4; ++i) arg[ft][i] = fmaf(c_dot, acc[i], -bias);
  }
}

// ------------------------------------------------------------------------------------------
// key side: state[c] = bf16( sum over the keys of column c of phi(k_j) ), in fragment order.
// Block = 4 waves = 64 keys of one head (8 waves = 128 keys for 128-key columns, so that a column
// never spans two blocks; wider columns are finished by wide_columns_kernel).  WLOG = log2(column
// width), 0..7.
//
// Here the projection is taken with the keys as accumulator rows, C[key][feature] = X W^T: a lane
// then holds, per 16-feature tile, feature 16 ft + lr of the four keys 4 lg + i, so a column sum
// is three adds in the lane plus at most two cross-lane steps, which four tiles share (three swaps
// and three additions for four tiles), and no feature array is kept in registers.  Sums meet in LDS (one m-vector per wave and column part) and leave as
// coalesced bf16 rows.
// ------------------------------------------------------------------------------------------
template <int MC, int WLOG>
__global__ __launch_bounds__(WLOG > 6 ? 512 : 256) void key_state_kernel(
    Shape s, const uint16_t* __restrict__ K, const uint16_t* __restrict__ W, uint16_t* __restrict__ state,
    uint16_t* __restrict__ pref, float* __restrict__ bsum_u, float* __restrict__ bsum_r, float c_dot,
    float c_norm, int32_t iters) {
  constexpr int m = 32 * MC;
  constexpr int w = 1 << WLOG;
  constexpr int kWaves = w > 64 ? w / 16 : 4;  // waves per block
  constexpr int kRows = 16 * kWaves;
  constexpr int kPartsWave = (w >= 4 && w < 16) ? 16 / w : 1;  // column sums a wave leaves in LDS
  constexpr int kSlots = kWaves * kPartsWave;
  __shared__ __attribute__((aligned(16))) uint16_t Ws[m * kWRow];
  __shared__ float part[w >= 4 ? kSlots * m : 1];   // per wave and column part
  __shared__ __attribute__((aligned(16))) float tpart[w > 16 ? kWaves * m : 1];  // per wave, over the bf16-rounded features
  const int tid = threadIdx.x, lane = tid & 63;
  const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lr = lane & 15, lg = lane >> 4;
  // a block takes `iters` consecutive key tiles of one head, so W is parked once for all of them
  const uint32_t tiles = (s.T + kRows - 1) / kRows;
  const uint32_t bph = (tiles + iters - 1) / iters;  // blocks per head
  const int64_t head = blockIdx.x / bph;
  const uint32_t tile_first = (blockIdx.x % bph) * iters;
  for (int x = tid; x < m * 8; x += 64 * kWaves) {
    const int r = x >> 3, part8 = x & 7;
    *reinterpret_cast<uint4*>(&Ws[r * kWRow + part8 * 8]) =
        *reinterpret_cast<const uint4*>(W + r * kHeadDim + part8 * 8);
  }
  __syncthreads();
  const int32_t b = static_cast<int32_t>(head / s.H);
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
  for (uint32_t tile = tile_first; tile < min(tile_first + static_cast<uint32_t>(iters), tiles); ++tile) {
  if (tile != tile_first) __syncthreads();  // the sums of the previous tile have left LDS
  const int32_t blk_r0 = static_cast<int32_t>(tile) * kRows;
  const int32_t r0 = blk_r0 + wid * 16;
  // operand rows: key r0 + lr; accumulator rows: keys r0 + 4 lg + i
  const uint16_t* X = K + (head * s.T + min(r0 + lr, s.T - 1)) * kHeadDim;
  const bf16x8 x0 = *reinterpret_cast<const bf16x8*>(X + 8 * lg);
  const bf16x8 x1 = *reinterpret_cast<const bf16x8*>(X + 32 + 8 * lg);
  float nx = sumsq8(x0) + sumsq8(x1);
  nx += __shfl_xor(nx, 16, kWave);
  nx += __shfl_xor(nx, 32, kWave);  // |k|^2 of key lr, in every lane group
  float bias[4];
  bool act[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    act[i] = r0 + 4 * lg + i < len;
    // keys past the sequence end get an infinite bias: their features are exp2(-inf) = 0
    bias[i] = act[i] ? c_norm * __shfl(nx, (lane & 48) | (4 * lg + i), kWave) : INFINITY;
  }
  uint16_t* sh = state + head * static_cast<int64_t>(s.K) * m;
  // Feature tiles are taken four at a time, so that the cross-lane part of the column sums can be
  // shared: a row swap of two tiles' sums leaves, after one addition, tile a's pair sums in the even
  // lane groups and tile b's in the odd ones; a half swap of two such registers and one more addition
  // leave the full sums of the four tiles in lane groups 0..3 -- three swaps and three additions for
  // four tiles, the same order of additions as summing each tile on its own, and one LDS store.
  static_assert((2 * MC) % 4 == 0, "feature tiles in groups of four");
  // slot of this lane's feature in a fragment-ordered row, for the tile its lane group ends up with
  const int slot_lane = 8 * (lr >> 2) + (lr & 3);
#pragma unroll
  for (int ft0 = 0; ft0 < 2 * MC; ft0 += 4) {
    float sum4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int ft = ft0 + q;
      const uint16_t* wr = &Ws[(ft * 16 + lr) * kWRow + 8 * lg];
      floatx4 acc = {0.f, 0.f, 0.f, 0.f};
      acc = mfma16(x0, *reinterpret_cast<const bf16x8*>(wr), acc);
      acc = mfma16(x1, *reinterpret_cast<const bf16x8*>(wr + 32), acc);
      float v[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] = __builtin_amdgcn_exp2f(fmaf(c_dot, acc[i], -bias[i]));
      // where feature 16 ft + lr sits in a fragment-ordered row
      const int slot = 32 * (ft >> 1) + 4 * (ft & 1) + slot_lane;
      if (w == 1) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (r0 + 4 * lg + i < s.T) sh[static_cast<int64_t>(r0 + 4 * lg + i) * m + slot] = f32_to_bf16(v[i]);
      } else if (w == 2) {
#pragma unroll
        for (int i = 0; i < 4; i += 2)
          if (r0 + 4 * lg + i < s.T)
            sh[static_cast<int64_t>((r0 + 4 * lg + i) >> 1) * m + slot] = f32_to_bf16(v[i] + v[i + 1]);
      } else {
        sum4[q] = (v[0] + v[1]) + (v[2] + v[3]);  // the four keys share a column
        if (w == 4) part[(wid * kPartsWave + lg) * m + slot] = sum4[q];
        if (w > 16 && pref) {
          // The same tile sum over the ROUNDED features (what a causal row's own-column term uses), on
          // the matrix pipe: the four keys of this lane, rounded, are the contraction slots of an
          // operand whose column is the feature; against an all-ones operand every result row is the
          // sum over the wave's 16 keys, accumulated in fp32.
          // (the four-slot product: exactly the lane's four keys, no zero padding of the operand)
          const uint2 u = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
          const uint2 one = {0x3f803f80u, 0x3f803f80u};
          const floatx4 rs = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(
              __builtin_bit_cast(shortx4, one), __builtin_bit_cast(shortx4, u), floatx4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
          if (lg == 0) tpart[wid * m + slot] = rs[0];
        }
      }
    }
    if (w >= 8) {
      // lane groups (0, 1, 2, 3) after the row swaps: pair sums of tiles (a, b, a, b) for keys
      // 0-7 in groups 0, 1 and keys 8-15 in groups 2, 3
      const auto ab = __builtin_amdgcn_permlane16_swap(__float_as_uint(sum4[0]), __float_as_uint(sum4[1]), false, false);
      const auto cd = __builtin_amdgcn_permlane16_swap(__float_as_uint(sum4[2]), __float_as_uint(sum4[3]), false, false);
      const float s_ab = __uint_as_float(ab[0]) + __uint_as_float(ab[1]);
      const float s_cd = __uint_as_float(cd[0]) + __uint_as_float(cd[1]);
      if (w == 8) {
        // two column parts per wave: group lg holds tile (lg & 1) of its pair, keys 8 (lg >> 1) ..
        const int tq = lg & 1, pw = lg >> 1;
        part[(wid * kPartsWave + pw) * m + 32 * (ft0 >> 1) + 4 * tq + slot_lane] = s_ab;
        part[(wid * kPartsWave + pw) * m + 32 * ((ft0 + 2) >> 1) + 4 * tq + slot_lane] = s_cd;
      } else {
        // full sums: lane group lg ends up with tile ft0 + lg
        const auto t = __builtin_amdgcn_permlane32_swap(__float_as_uint(s_ab), __float_as_uint(s_cd), false, false);
        const float tot = __uint_as_float(t[0]) + __uint_as_float(t[1]);
        part[wid * kPartsWave * m + 32 * ((ft0 + lg) >> 1) + 4 * (lg & 1) + slot_lane] = tot;
      }
    }
  }
  if (w < 4) continue;
  __syncthreads();
  if (w <= 16) {
    // each LDS vector is one finished column: columns blk_r0 / w + 0 .. kSlots - 1
    const int32_t col0 = blk_r0 >> WLOG;
    for (int x = tid; x < kSlots * m / 2; x += 64 * kWaves) {
      const int cl = (2 * x) / m, p = 2 * x - cl * m;
      if (col0 + cl < s.K)
        *reinterpret_cast<uint32_t*>(&sh[static_cast<int64_t>(col0 + cl) * m + p]) =
            pack_bf16(part[cl * m + p], part[cl * m + p + 1]);
    }
  } else {
    // column spans several waves of this block
    constexpr int wpc = w / 16;            // waves per column
    constexpr int cols = kRows / w;        // columns per block
    const int32_t col0 = static_cast<int32_t>(tile) * cols;
    for (int x = tid; x < cols * m; x += 64 * kWaves) {
      const int cl = x / m, p = x - cl * m;
      float acc = 0.f;
#pragma unroll
      for (int q = 0; q < wpc; ++q) acc += part[(cl * wpc + q) * m + p];
      if (WLOG == 7 && bsum_u) {
        // columns wider than this block: leave the block's sums (and, causal, the sums of the
        // rounded features) for the kernel that walks each column's blocks
        const int64_t blk = head * tiles + tile;
        bsum_u[blk * m + p] = acc;
        if (bsum_r) {
          float racc = 0.f;
#pragma unroll
          for (int q = 0; q < wpc; ++q) racc += tpart[q * m + p];
          bsum_r[blk * m + p] = racc;
        }
      } else if (col0 + cl < s.K) {
        sh[static_cast<int64_t>(col0 + cl) * m + p] = f32_to_bf16(acc);
      }
    }
    if (pref) {
      // exclusive prefix over the column's tiles, as bf16 planes hi + lo + lo2 (each difference is
      // exact in fp32, so the three planes carry the leading 24 bits of the sum)
      const int64_t ntile = s.T >> 4;
      const int64_t tile0 = static_cast<int64_t>(tile) * kWaves;
      // four consecutive features per thread: 16-byte reads of the tile sums, 8-byte stores
      for (int x = tid; x < kWaves * m / 4; x += 64 * kWaves) {
        const int q = x / (m / 4), p = (x - q * (m / 4)) * 4, qc = q & (wpc - 1);
        if (qc == 0 || tile0 + q >= ntile) continue;  // a column's first tile has nothing before it
        float4 P = {0.f, 0.f, 0.f, 0.f};
        for (int j = q - qc; j < q; ++j) {
          const float4 tp = *reinterpret_cast<const float4*>(&tpart[j * m + p]);
          P.x += tp.x; P.y += tp.y; P.z += tp.z; P.w += tp.w;
        }
        const float Pv[4] = {P.x, P.y, P.z, P.w};
        uint16_t hi[4], lo[4], lo2[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          hi[e] = f32_to_bf16(Pv[e]);
          const float r1 = Pv[e] - bf16_to_f32(hi[e]);
          lo[e] = f32_to_bf16(r1);
          lo2[e] = f32_to_bf16(r1 - bf16_to_f32(lo[e]));
        }
        uint16_t* dst = pref + ((head * ntile + tile0 + q) * 3) * m + p;
        auto pack4 = [](const uint16_t* h) {
          return make_uint2(static_cast<uint32_t>(h[0]) | (static_cast<uint32_t>(h[1]) << 16),
                            static_cast<uint32_t>(h[2]) | (static_cast<uint32_t>(h[3]) << 16));
        };
        *reinterpret_cast<uint2*>(dst) = pack4(hi);
        *reinterpret_cast<uint2*>(dst + m) = pack4(lo);
        *reinterpret_cast<uint2*>(dst + 2 * m) = pack4(lo2);
      }
    }
  }
  }  // tiles of this block
}

// Columns of 256 keys or more: one block per (head, column) adds up the column's 128-key blocks.
// Causal: the sum of the rounded features of the column's earlier blocks goes out per block as
// three bf16 planes, like the tile prefixes inside a block.
__global__ __launch_bounds__(256) void wide_columns_kernel(Shape s, const float* __restrict__ bsum_u,
                                                           const float* __restrict__ bsum_r,
                                                           uint16_t* __restrict__ state,
                                                           uint16_t* __restrict__ bpref, int32_t nb) {
  const int32_t m = s.m, p = threadIdx.x;
  if (p >= m) return;
  const int64_t head = blockIdx.x / static_cast<uint32_t>(s.K);
  const int32_t c = static_cast<int32_t>(blockIdx.x % static_cast<uint32_t>(s.K));
  const int64_t blk0 = head * (s.T >> 7) + static_cast<int64_t>(c) * nb;
  float acc_u = 0.f, acc_r = 0.f;
  for (int32_t j = 0; j < nb; ++j) {
    if (bpref && j > 0) {
      const uint16_t hi = f32_to_bf16(acc_r);
      const float r1 = acc_r - bf16_to_f32(hi);
      const uint16_t lo = f32_to_bf16(r1);
      const uint16_t lo2 = f32_to_bf16(r1 - bf16_to_f32(lo));
      uint16_t* dst = bpref + ((blk0 + j) * 3) * m + p;
      dst[0] = hi;
      dst[m] = lo;
      dst[2 * m] = lo2;
    }
    acc_u += bsum_u[(blk0 + j) * m + p];
    if (bsum_r) acc_r += bsum_r[(blk0 + j) * m + p];
  }
  state[(head * s.K + c) * m + p] = f32_to_bf16(acc_u);
}

// ------------------------------------------------------------------------------------------
// query side.  Block = 4 waves = 64 rows of one head (16 per wave).
// ------------------------------------------------------------------------------------------
constexpr int kColStage = 32;   // columns of the state staged in LDS per step

// NCT = 16-column tiles a row can have (4, 8 or 16 for K <= 64, 128, 256).  WLOG = log2(column
// width) for widths up to 16; 5 stands for every wider column (the shift is then read from the shape).
template <int MC, bool CAUSAL, int WLOG, int NCT>
__global__ __launch_bounds__(256, 3) void estimate_rows_kernel(Shape s, const uint16_t* __restrict__ Q,
                                                            const uint16_t* __restrict__ K,
                                                            const uint16_t* __restrict__ W,
                                                            const uint16_t* __restrict__ state,
                                                            const uint16_t* __restrict__ pref,
                                                            const uint16_t* __restrict__ bpref,
                                                            float* __restrict__ A_hat,
                                                            uint32_t* __restrict__ mbits, float c_dot,
                                                            float c_norm, int32_t group_heads) {
  constexpr int m = 32 * MC;
  const int wl = WLOG >= 5 ? 31 - __clz(s.T / s.K) : WLOG;  // log2(column width)
  constexpr int kSRow = m + 8;  // halfwords per staged state row (+16 B pad): conflict-free b128 reads
  // W is dead once both projections are done; the state stages then reuse its space
  constexpr int kStageHalfwords = kColStage * kSRow;
  constexpr int kSmemHalfwords = m * kWRow > 2 * kStageHalfwords ? m * kWRow : 2 * kStageHalfwords;
  __shared__ __attribute__((aligned(16))) uint16_t smem[kSmemHalfwords];
  // causal, columns wider than 16 keys: the three prefix planes of each wave's tile (requested with
  // the wave's rows, parked here, read as operand rows once phi(Q) is ready)
  __shared__ __attribute__((aligned(16))) uint16_t planes_s[(CAUSAL && WLOG >= 5) ? 4 * 3 * m : 8];
  uint16_t* const Ws = smem;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lr = lane & 15, lg = lane >> 4;
  const uint32_t tiles = (s.T + 63) / 64;
  // Launch order = longest first: heads in groups whose state fits the L2s, inside a group the
  // row tiles from the last (most columns, causal) to the first, heads fastest.  Blocks are dealt
  // round-robin to the 8 XCDs, so with 8 | group size a head's state stays in one XCD's L2.
  const uint32_t per_group = static_cast<uint32_t>(group_heads) * tiles;
  const uint32_t grp = blockIdx.x / per_group, rem = blockIdx.x - grp * per_group;
  const uint32_t nh = min(static_cast<uint32_t>(group_heads), static_cast<uint32_t>(s.N) - grp * group_heads);
  const int64_t head = static_cast<int64_t>(grp) * group_heads + rem % nh;
  const int32_t wg_r0 = static_cast<int32_t>(tiles - 1 - rem / nh) * 64;
  const int32_t r0 = wg_r0 + wid * 16;
  const int32_t b = static_cast<int32_t>(head / s.H);
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;

  // state staging: 32 columns x m halfwords per step, contiguous in memory
  const uint16_t* sh = state + head * static_cast<int64_t>(s.K) * m;
  constexpr int kVecPerStage = kColStage * m / 8;      // 16-byte vectors per step
  constexpr int kVecPerThread = kVecPerStage / 256;    // 1, 2 or 4 (m = 64..256); m = 32 -> 0
  static_assert(MC >= 2, "m >= 64");
  uint4 sreg0 = {0u, 0u, 0u, 0u}, sreg1 = sreg0, sreg2 = sreg0, sreg3 = sreg0;  // named: stay in VGPRs
  const int32_t ncols_wg = CAUSAL ? min(s.K, (min(wg_r0 + 63, s.T - 1) >> wl) + 1) : s.K;
  const int32_t nstages = (ncols_wg + kColStage - 1) / kColStage;
#define SEA_SFETCH1(reg_, q_, st_)                                                              \
  if (kVecPerThread > (q_)) {                                                                  \
    const int x_ = tid + 256 * (q_);                                                           \
    const int col_ = min((st_) * kColStage + x_ / (m / 8), s.K - 1);                            \
    reg_ = *reinterpret_cast<const uint4*>(sh + static_cast<int64_t>(col_) * m + (x_ % (m / 8)) * 8); \
  }
#define SEA_SFETCH(st_)          \
  SEA_SFETCH1(sreg0, 0, st_)     \
  SEA_SFETCH1(sreg1, 1, st_)     \
  SEA_SFETCH1(sreg2, 2, st_)     \
  SEA_SFETCH1(sreg3, 3, st_)
#define SEA_SPARK1(reg_, q_, buf_)                                                              \
  if (kVecPerThread > (q_)) {                                                                  \
    const int x_ = tid + 256 * (q_);                                                           \
    *reinterpret_cast<uint4*>(&smem[(buf_) * kStageHalfwords + (x_ / (m / 8)) * kSRow + (x_ % (m / 8)) * 8]) = reg_;    \
  }
#define SEA_SPARK(buf_)          \
  SEA_SPARK1(sreg0, 0, buf_)     \
  SEA_SPARK1(sreg1, 1, buf_)     \
  SEA_SPARK1(sreg2, 2, buf_)     \
  SEA_SPARK1(sreg3, 3, buf_)

  // the wave's query (and, causal, key) rows are requested before the staging waits
  const int32_t t = r0 + lr, tc = min(t, s.T - 1);
  const uint16_t* Xq = Q + (head * s.T + tc) * kHeadDim;
  const bf16x8 x0 = *reinterpret_cast<const bf16x8*>(Xq + 8 * lg);
  const bf16x8 x1 = *reinterpret_cast<const bf16x8*>(Xq + 32 + 8 * lg);
  const uint16_t* Xk = K + (head * s.T + tc) * kHeadDim;
  bf16x8 y0 = x0, y1 = x1;
  if (CAUSAL) {
    y0 = *reinterpret_cast<const bf16x8*>(Xk + 8 * lg);
    y1 = *reinterpret_cast<const bf16x8*>(Xk + 32 + 8 * lg);
  }
  // Prefix planes of the wave's tile inside its 128-key block (its column, if narrower): 3 m
  // halfwords, contiguous; lane l takes 16-byte pieces l and l + 64.
  bool tile_planes = false;
  if (CAUSAL && WLOG >= 5) {
    const int tl = min(wl, 7) - 4;  // log2(tiles per prefix group)
    tile_planes = r0 < s.T && ((r0 >> 4) & ((1 << tl) - 1)) != 0;  // wave-uniform
  }
  uint4 preg0 = {0u, 0u, 0u, 0u}, preg1 = preg0;
  if (tile_planes) {
    const uint4* psrc = reinterpret_cast<const uint4*>(pref + (head * (s.T >> 4) + (r0 >> 4)) * 3 * m);
    constexpr int kPieces = 3 * m / 8;
    if (lane < kPieces) preg0 = psrc[lane];
    if (lane + 64 < kPieces) preg1 = psrc[lane + 64];
  }
  stage_w(W, Ws, m, tid);
  if (tile_planes) {
    constexpr int kPieces = 3 * m / 8;
    uint4* pdst = reinterpret_cast<uint4*>(&planes_s[wid * 3 * m]);
    if (lane < kPieces) pdst[lane] = preg0;
    if (lane + 64 < kPieces) pdst[lane + 64] = preg1;
  }
  if (nstages > 0) { SEA_SFETCH(0); }  // parked in LDS after the projections
  __syncthreads();

  // ---- phi(Q) of this wave's 16 rows, as contraction fragments ----
  bf16x8 afrag[MC];
  // causal: phi(K) of the same 16 rows (the keys of the rows' own column inside the wave), taken in
  // the same pass over W's fragments, so that each is read from LDS once for both projections; a
  // key's features need no row shift and are rounded and packed tile by tile
  bf16x8 kfrag[CAUSAL ? MC : 1];
  {
    float nx = sumsq8(x0) + sumsq8(x1);
    nx += __shfl_xor(nx, 16, kWave);
    nx += __shfl_xor(nx, 32, kWave);
    floatx4 dots[2 * MC];
    if (CAUSAL) {
      float ny = sumsq8(y0) + sumsq8(y1);
      ny += __shfl_xor(ny, 16, kWave);
      ny += __shfl_xor(ny, 32, kWave);
      const float kbias = c_norm * ny;
#pragma unroll
      for (int kc = 0; kc < MC; ++kc) {
        float lo[4], hi[4];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int ft = 2 * kc + h;
          const uint16_t* w = &Ws[(ft * 16 + lr) * kWRow + 8 * lg];
          const bf16x8 w0 = *reinterpret_cast<const bf16x8*>(w), w1 = *reinterpret_cast<const bf16x8*>(w + 32);
          floatx4 acc = {0.f, 0.f, 0.f, 0.f};
          acc = mfma16(w0, x0, acc);
          dots[ft] = mfma16(w1, x1, acc);
          floatx4 ka = {0.f, 0.f, 0.f, 0.f};
          ka = mfma16(w0, y0, ka);
          ka = mfma16(w1, y1, ka);
#pragma unroll
          for (int i = 0; i < 4; ++i) (h == 0 ? lo : hi)[i] = __builtin_amdgcn_exp2f(fmaf(c_dot, ka[i], -kbias));
        }
        kfrag[kc] = pack8(lo, hi);
      }
    } else {
      project_dots<MC>(Ws, x0, x1, lr, lg, dots);
    }
    float dmax = -INFINITY;
#pragma unroll
    for (int ft = 0; ft < 2 * MC; ++ft)
#pragma unroll
      for (int i = 0; i < 4; ++i) dmax = fmaxf(dmax, dots[ft][i]);
    dmax = fmaxf(dmax, __shfl_xor(dmax, 16, kWave));
    dmax = fmaxf(dmax, __shfl_xor(dmax, 32, kWave));
    // Largest exponent argument of the row (the map dot -> c_dot dot - bias is monotone), rounded up:
    // a power-of-two row scale, which commutes with the bf16 rounding.  Inactive rows get an
    // infinite shift, i.e. all-zero features.
    const float bias = c_norm * nx;
    const float shift = t < len ? ceilf(fmaf(c_dot, dmax, -bias)) : INFINITY;
    const float off = -(bias + shift);
#pragma unroll
    for (int kc = 0; kc < MC; ++kc) {
      float lo[4], hi[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        lo[i] = __builtin_amdgcn_exp2f(fmaf(c_dot, dots[2 * kc][i], off));
        hi[i] = __builtin_amdgcn_exp2f(fmaf(c_dot, dots[2 * kc + 1][i], off));
      }
      afrag[kc] = pack8(lo, hi);
    }
  }
  // From here on every product is taken with the query rows as accumulator COLUMNS: lane l % 16 is
  // the query row, so a row of A_hat lives in the four lanes l % 16 + 16 q (16 values each per 64
  // columns) and every per-row reduction is two row-swap steps.
  float diag = 0.f;
  if (CAUSAL) {
    // the row's own column: sum over keys j <= t of that column of phi(q_t) . phi(k_j).  Those
    // keys are the wave's own 16 rows (S = phi(Q) phi(K_own)^T with a lower-triangular, same-column
    // mask) and, for columns wider than 16, the 16-key tiles of the column before the wave.
    floatx4 sd = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kc = 0; kc < MC; ++kc) sd = mfma16(kfrag[kc], afrag[kc], sd);  // rows = keys 4 lg + i, col = query lr
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int rk = 4 * lg + i;  // key row within the wave; the query row within the wave is lr
      const bool ok = (rk <= lr) && (WLOG >= 4 || (rk >> WLOG) == (lr >> WLOG));
      sd[i] = ok ? sd[i] : 0.f;
    }
    // Earlier keys of the same column: every one of them precedes every row of the wave, so only
    // their sum matters.  It comes as three bf16 planes = operand rows 0..2 (the rest zero);
    // the sum over the 16 result rows below then adds the three partial dots to the
    // in-wave ones.  Two levels: tiles before this one inside its 128-key block (its column, if
    // narrower), and, for columns wider than that, the column's blocks before this one.
    if (WLOG >= 5 && r0 < s.T) {
      if (tile_planes) {
        const uint16_t* src = &planes_s[(wid * 3 + min(lr, 2)) * m + 8 * lg];
#pragma unroll
        for (int kc = 0; kc < MC; ++kc) {
          uint4 f = *reinterpret_cast<const uint4*>(src + 32 * kc);
          if (lr > 2) f = uint4{0u, 0u, 0u, 0u};
          sd = mfma16(__builtin_bit_cast(bf16x8, f), afrag[kc], sd);
        }
      }
      if (wl > 7 && ((r0 >> 7) & ((1 << (wl - 7)) - 1)) != 0) {
        const uint16_t* src = bpref + ((head * (s.T >> 7) + (r0 >> 7)) * 3 + min(lr, 2)) * m + 8 * lg;
#pragma unroll
        for (int kc = 0; kc < MC; ++kc) {
          uint4 f = *reinterpret_cast<const uint4*>(src + 32 * kc);
          if (lr > 2) f = uint4{0u, 0u, 0u, 0u};
          sd = mfma16(__builtin_bit_cast(bf16x8, f), afrag[kc], sd);
        }
      }
    }
    diag = rows_sum((sd[0] + sd[1]) + (sd[2] + sd[3]));
  }

  // ---- A_hat tile = phi(Q) state^T, state streamed through LDS ----
  __syncthreads();  // every wave is done with W
  if (nstages > 0) { SEA_SPARK(0); }
  __syncthreads();
  floatx4 acc[NCT];
#pragma unroll
  for (int ct = 0; ct < NCT; ++ct) acc[ct] = floatx4{0.f, 0.f, 0.f, 0.f};
  const int32_t ncols_wave = CAUSAL ? min(s.K, (min(r0 + 15, s.T - 1) >> wl) + 1) : s.K;
#pragma unroll
  for (int st = 0; st < NCT * 16 / kColStage; ++st) {
    if (st < nstages) {
      if (st + 1 < nstages) { SEA_SFETCH(st + 1); }
      if (r0 < s.T && st * kColStage < ncols_wave) {
#pragma unroll
        for (int h = 0; h < kColStage / 16; ++h) {
          const uint16_t* brow = &smem[(st & 1) * kStageHalfwords + (16 * h + lr) * kSRow + 8 * lg];
          floatx4 a4 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int kc = 0; kc < MC; ++kc)
            a4 = mfma16(*reinterpret_cast<const bf16x8*>(brow + 32 * kc), afrag[kc], a4);
          acc[st * (kColStage / 16) + h] = a4;
        }
      }
      if (st + 1 < nstages) { SEA_SPARK((st + 1) & 1); }
      __syncthreads();
    }
  }
#undef SEA_SFETCH
#undef SEA_SFETCH1
#undef SEA_SPARK
#undef SEA_SPARK1
  if (r0 >= s.T) return;  // no barrier below

  // ---- masking, the own column, normalisation ----
  // acc[ct][i] = raw score of row r0 + lr, column cc = 16 ct + 4 lg + i.  last = last admissible
  // column of the row (-1: inactive row); a causal row takes its own column (= last) from diag.
  // Tiles wholly below every row's last column need no test, tiles above the wave's last one are
  // cleared.
  const int32_t trow = r0 + lr;
  const bool act = trow < len;
  const int32_t jmax = CAUSAL ? min(trow, len - 1) : len - 1;
  const int32_t ncnd = act ? (jmax >> wl) + 1 : 0;
  const int32_t e = ncnd - 1 - 4 * lg;  // column 16 ct + 4 lg + i is the own one iff 16 ct + i == e
  const bool act_all = r0 + 15 < len;  // wave-uniform
  const int32_t ct_free = act_all ? (((CAUSAL ? r0 : len - 1) >> wl) >> 4) : 0;
  float rsum = 0.f;
#pragma unroll
  for (int ct = 0; ct < NCT; ++ct) {
    if (ct < ct_free) {
      rsum += (acc[ct][0] + acc[ct][1]) + (acc[ct][2] + acc[ct][3]);
    } else if (ct * 16 < ncols_wave) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float v = acc[ct][i];
        if (CAUSAL && ct * 16 + i == e) v = diag;
        if (ct * 16 + i > e) v = 0.f;
        acc[ct][i] = v;
        rsum += v;
      }
    } else {
      acc[ct] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
  }
  {
    const float r = rows_sum(rsum);
    // The normalised scores are kept NEGATED from here on: the bit pattern of -x (x >= +0) is
    // 0x80000000 | bits(x), which is the selection key itself, so the keys cost no instruction.
    const float ninv = r > 0.f ? -1.f / r : -0.f;
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[ct][i] *= ninv;
    if (A_hat && trow < s.T) {
      float* out = A_hat + (head * s.T + trow) * s.K;
      if ((s.K & 3) == 0) {
        // a scratch A_hat read only by the grouped selection needs no zeros past a row's candidates
        const int32_t cend = s.cand_only ? min(s.K, ncnd) : s.K;
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct)
          if (ct * 16 + 4 * lg < cend)
            *reinterpret_cast<float4*>(out + ct * 16 + 4 * lg) = make_float4(-acc[ct][0], -acc[ct][1], -acc[ct][2], -acc[ct][3]);
      } else {
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (ct * 16 + 4 * lg + i < s.K) out[ct * 16 + 4 * lg + i] = -acc[ct][i];
      }
    }
  }
  if (!mbits) return;

  // ---- per-row top-k^ on the normalised scores, in registers (Sec. 3.1 "Grouped Top-k^
  // Selection", per-query grouping).  A row lives in four lanes, 4 NCT scores each.  The k^-th
  // largest score is found by a bitwise search on order-preserving integer keys (the bit patterns
  // of the negated scores); the counts of a step are taken over the whole row by an 8-bit integer
  // matrix product (high halves) or per lane with two row-swap steps (low halves).  Scores are in
  // [0, 1], so the key's two top bits are known and the search starts below them.
  const uint32_t nsel = static_cast<uint32_t>(min(s.k_hat, ncnd));
  uint32_t tau = 0x80000000u, cge = static_cast<uint32_t>(ncnd);
  uint32_t key[NCT][4];
#pragma unroll
  for (int ct = 0; ct < NCT; ++ct) {
    if (ct < ct_free) {  // every column of the tile is a candidate of every row
#pragma unroll
      for (int i = 0; i < 4; ++i) key[ct][i] = __float_as_uint(acc[ct][i]);
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        key[ct][i] = ct * 16 + i <= e ? __float_as_uint(acc[ct][i]) : 0x40000000u;
    }
  }
  // The compare-and-count loop runs over the tiles that hold candidates of this wave's rows only
  // (causal: the leading ones), in even steps so that a handful of loop bodies covers all cases.
  // Bits 29..16 are searched on the keys' high halves, two keys per register: both halves of
  // hp - trial (16-bit wrap-around differences; candidates and trial lie in [0x8000, 0xc000),
  // non-candidates are 0x4000) have bit 15 set exactly for keys below the trial; a byte permute
  // spreads each sign over a byte, four differences at a time, and the matrix product adds the bytes
  // up.  The trial's
  // low half is zero in that phase, so the counts are those of the full keys.  Bits 15..0 then
  // compare whole keys.
#define SEA_SEARCH_STEP(COUNT_BODY_, REDUCE_)                                                    \
    /* done when every row's count of keys >= tau equals its quota */                            \
    const bool pend = (cge != nsel) && (nsel != 0u);                                             \
    if (__ballot(pend) == 0ull) break;                                                           \
    const uint32_t trial = tau | (1u << bit);                                                    \
    uint32_t cnt = 0;                                                                            \
    COUNT_BODY_                                                                                  \
    REDUCE_                                                                                      \
    const bool take = pend && cnt >= nsel;                                                       \
    tau = take ? trial : tau;                                                                    \
    cge = take ? cnt : cge;
#define SEA_SEARCH(NT_)                                                                          \
  {                                                                                              \
    ushort2v hp[2 * (NT_)];                                                                      \
    _Pragma("unroll") for (int ct = 0; ct < (NT_); ++ct) {                                        \
      hp[2 * ct] = __builtin_bit_cast(ushort2v, __builtin_amdgcn_perm(key[ct][1], key[ct][0], 0x07060302u)); \
      hp[2 * ct + 1] = __builtin_bit_cast(ushort2v, __builtin_amdgcn_perm(key[ct][3], key[ct][2], 0x07060302u)); \
    }                                                                                            \
    /* Count of the ROW's keys at or above a trial whose low half is zero.  A byte permute turns  \
       the signs of four differences into four bytes 0x00 / 0xff (selectors 8..11 take the sign \
       of bytes 1, 3, 5, 7), i.e. 0 / -1 as 8-bit integers; sixteen of them are one operand of  \
       the 8-bit matrix product, whose column is the query row (lane % 16) and whose           \
       contraction runs over the lane's sixteen keys and the row's four lanes: against an      \
       all -1 operand every result row is the number of the row's keys BELOW the trial, summed \
       over the four lanes, so the counting and the cross-lane sum leave the vector pipe. */    \
    auto count_high = [&](uint32_t trial_) {                                                     \
      const uint32_t th = trial_ >> 16;                                                          \
      const ushort2v th2 = __builtin_bit_cast(ushort2v, th | (th << 16));                        \
      const intx4 neg1 = {-1, -1, -1, -1};                                                       \
      intx4 below = {0, 0, 0, 0};                                                                \
      _Pragma("unroll") for (int q4 = 0; q4 < ((NT_) + 3) / 4; ++q4) {                            \
        intx4 fl = {0, 0, 0, 0};                                                                 \
        _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                           \
          if (4 * q4 + j < (NT_)) {                                                              \
            const int pr = 2 * (4 * q4 + j);                                                     \
            const uint32_t d0 = __builtin_bit_cast(uint32_t, static_cast<ushort2v>(hp[pr] - th2)); \
            const uint32_t d1 = __builtin_bit_cast(uint32_t, static_cast<ushort2v>(hp[pr + 1] - th2)); \
            fl[j] = static_cast<int>(__builtin_amdgcn_perm(d1, d0, 0x0b0a0908u));                \
          }                                                                                      \
        }                                                                                        \
        below = __builtin_amdgcn_mfma_i32_16x16x64_i8(neg1, fl, below, 0, 0, 0);                 \
      }                                                                                          \
      return 16u * static_cast<uint32_t>(NT_) - static_cast<uint32_t>(below[0]);                 \
    };                                                                                           \
    /* Bits 29..27 at once: a row whose quota of scores lies at or above 2^-15 (rows sum to 1    \
       over at most 256 columns, so nearly every row) would take all three bits, because the     \
       count only grows as the trial falls; one count then stands for three steps.  A wave with  \
       a row that fails the test searches from bit 29 as before. */                              \
    int bit_top = 29;                                                                            \
    {                                                                                            \
      const bool pend = (cge != nsel) && (nsel != 0u);                                           \
      const uint32_t trial = 0xb8000000u;                                                        \
      const uint32_t cnt = count_high(trial);                                                    \
      if (__ballot(pend && cnt < nsel) == 0ull) {                                                \
        tau = pend ? trial : tau;                                                                \
        cge = pend ? cnt : cge;                                                                  \
        bit_top = 26;                                                                            \
      }                                                                                          \
    }                                                                                            \
    _Pragma("unroll 1") for (int bit = bit_top; bit >= 16; --bit) {                               \
      SEA_SEARCH_STEP(cnt = count_high(trial);, )                                                \
    }                                                                                            \
  }                                                                                              \
  _Pragma("unroll 1") for (int bit = 15; bit >= 0; --bit) {                                       \
    SEA_SEARCH_STEP(                                                                             \
      _Pragma("unroll") for (int ct = 0; ct < (NT_); ++ct)                                        \
        _Pragma("unroll") for (int i = 0; i < 4; ++i) cnt += (key[ct][i] >= trial) ? 1u : 0u;,   \
      cnt = rows_sum_u(cnt);)                                                                    \
  }
  const int32_t nct_wave = CAUSAL ? min(NCT, (ncols_wave + 15) >> 4) : NCT;
  if (s.k_hat == 1) {
    // one column per row: the threshold is the row maximum itself (several columns holding it
    // are told apart by the tie rule below)
    uint32_t mx = 0u;
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
      for (int i = 0; i < 4; ++i) mx = max(mx, key[ct][i]);
    mx = rows_max_u(mx);
    uint32_t cnt = 0;
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
      for (int i = 0; i < 4; ++i) cnt += (key[ct][i] >= mx) ? 1u : 0u;
    tau = mx;
    cge = rows_sum_u(cnt);
  } else if (NCT >= 16 && nct_wave > 12) {
    SEA_SEARCH(NCT >= 16 ? 16 : NCT)
  } else if (NCT >= 16 && nct_wave > 8) {
    SEA_SEARCH(NCT >= 16 ? 12 : NCT)
  } else if (NCT >= 8 && nct_wave > 6) {
    SEA_SEARCH(NCT >= 8 ? 8 : NCT)
  } else if (NCT >= 8 && nct_wave > 4) {
    SEA_SEARCH(NCT >= 8 ? 6 : NCT)
  } else if (nct_wave > 2) {
    SEA_SEARCH(4)
  } else {
    SEA_SEARCH(2)
  }
#undef SEA_SEARCH
#undef SEA_SEARCH_STEP
  // selection: keys >= tau; when more keys than the quota tie at tau (exact duplicates at the
  // boundary), the lowest columns among them win.  nib[ct]: bit i set iff column 16 ct + 4 lg + i
  // of this lane's row is selected.
  uint32_t nib[NCT];
  const bool excess = (cge != nsel) && (nsel != 0u);
  if (__ballot(excess) == 0ull) {
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
      uint32_t bits = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) bits |= (nsel != 0u && key[ct][i] >= tau) ? (1u << i) : 0u;
      nib[ct] = bits;
    }
  } else {
    uint32_t cgt = 0;
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
      for (int i = 0; i < 4; ++i) cgt += (key[ct][i] > tau) ? 1u : 0u;
    cgt = rows_sum_u(cgt);
    int32_t need_eq = static_cast<int32_t>(nsel) - static_cast<int32_t>(cgt);  // ties still to take, in column order
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
      uint32_t eqm = 0, gtm = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        eqm |= (key[ct][i] == tau && nsel != 0u) ? (1u << i) : 0u;
        gtm |= (key[ct][i] > tau && nsel != 0u) ? (1u << i) : 0u;
      }
      // columns ascend with (ct, lg, i): ties of lower lane rows of this tile come first
      uint32_t below;
      const uint32_t total = rows_sum_prefix_u(static_cast<uint32_t>(__popc(eqm)), lg, &below);
      uint32_t bits = gtm;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int32_t rank = static_cast<int32_t>(below) + __popc(eqm & ((1u << i) - 1u));
        if (((eqm >> i) & 1u) && rank < need_eq) bits |= 1u << i;
      }
      nib[ct] = bits;
      need_eq -= min(need_eq, static_cast<int32_t>(total));
    }
  }
  // mask words: word j holds columns 32 j .. 32 j + 31 = tiles 2 j (low half) and 2 j + 1; this lane's
  // four columns of a tile sit at bits 4 lg .. 4 lg + 3 of the tile's half.  The four lanes of a row
  // combine their parts; the lane of the first row stores them as vectors.
  const int32_t kw = (s.K + 31) >> 5;
  constexpr int kWords = NCT / 2;
  if constexpr (kWords % 4 == 0) {
    // Four words at a time: a row swap of two words' parts and an OR leave word a's halves in the
    // even lane groups and word b's in the odd ones; a half swap of two such registers and an OR
    // leave the four finished words in lane groups 0..3 (three swaps for four words instead of
    // eight), and every lane stores the word of its group.
    uint32_t* mrow = mbits + (head * s.T + min(trow, s.T - 1)) * kw;
#pragma unroll
    for (int j = 0; j < kWords; j += 4) {
      uint32_t pw[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) pw[q] = (nib[2 * (j + q)] << (4 * lg)) | (nib[2 * (j + q) + 1] << (16 + 4 * lg));
      const auto ab = __builtin_amdgcn_permlane16_swap(pw[0], pw[1], false, false);
      const auto cd = __builtin_amdgcn_permlane16_swap(pw[2], pw[3], false, false);
      const auto t = __builtin_amdgcn_permlane32_swap(ab[0] | ab[1], cd[0] | cd[1], false, false);
      if (trow < s.T && j + lg < kw) mrow[j + lg] = t[0] | t[1];
    }
  } else {
    uint32_t words[kWords];
#pragma unroll
    for (int j = 0; j < kWords; ++j)
      words[j] = rows_or_u((nib[2 * j] << (4 * lg)) | (nib[2 * j + 1] << (16 + 4 * lg)));
    if (trow >= s.T || lg != 0) return;
    uint32_t* mrow = mbits + (head * s.T + trow) * kw;
    if (kw == kWords) {
      *reinterpret_cast<uint2*>(mrow) = make_uint2(words[0], words[1]);
    } else {
#pragma unroll
      for (int j = 0; j < kWords; ++j)
        if (j < kw) mrow[j] = words[j];
    }
  }
}

int wlog_of(const Shape& s) {
  if (s.T % s.K != 0) return -1;
  const int32_t w = s.T / s.K;
  if ((w & (w - 1)) != 0) return -1;
  int l = 0;
  while ((1 << l) < w) ++l;
  return l;
}

}  // namespace

bool estimate_fused_supported(const Shape& s) {
  const int wl = wlog_of(s);
  if (wl < 0 || wl > 20) return false;
  if (s.m != 64 && s.m != 128 && s.m != 256) return false;
  if (s.K > 256) return false;
  return true;
}

namespace {
size_t up256(size_t b) { return (b + 255) & ~size_t(255); }
struct FusedWs {
  size_t state, pref, bsum_u, bsum_r, bpref, total;
};
// state | tile prefixes (causal, columns > 16) | for columns > 128: block sums, rounded block sums
// and block prefixes (the last two causal only)
FusedWs fused_layout(const Shape& s) {
  const int wl = wlog_of(s);
  const size_t N = static_cast<size_t>(s.N);
  FusedWs f{};
  size_t off = 0;
  f.state = off; off += up256(N * s.K * s.m * 2);
  f.pref = off;  if (s.causal && wl > 4) off += up256(N * (s.T / 16) * 3 * s.m * 2);
  f.bsum_u = off; if (wl > 7) off += up256(N * (s.T / 128) * s.m * 4);
  f.bsum_r = off; if (wl > 7 && s.causal) off += up256(N * (s.T / 128) * s.m * 4);
  f.bpref = off;  if (wl > 7 && s.causal) off += up256(N * (s.T / 128) * 3 * s.m * 2);
  f.total = off;
  return f;
}
}  // namespace

size_t estimate_fused_workspace(const Shape& s) { return fused_layout(s).total; }

namespace {

struct FusedPtrs {
  uint16_t* state;
  uint16_t* pref;
  float* bsum_u;
  float* bsum_r;
  uint16_t* bpref;
};

template <int MC, int WLOG, int NCT>
void launch_rows(const Shape& s, const uint16_t* Q, const uint16_t* K, const uint16_t* W, float* A_hat,
                 uint32_t* mbits, const FusedPtrs& f, float c_dot, float c_norm, int32_t gh, dim3 grid,
                 hipStream_t st) {
  if (s.causal)
    hipLaunchKernelGGL((estimate_rows_kernel<MC, true, WLOG, NCT>), grid, dim3(256), 0, st, s, Q, K, W, f.state,
                       f.pref, f.bpref, A_hat, mbits, c_dot, c_norm, gh);
  else
    hipLaunchKernelGGL((estimate_rows_kernel<MC, false, WLOG, NCT>), grid, dim3(256), 0, st, s, Q, K, W, f.state,
                       f.pref, f.bpref, A_hat, mbits, c_dot, c_norm, gh);
}

template <int MC, int WLOG>
void launch_key(const Shape& s, const uint16_t* K, const uint16_t* W, const FusedPtrs& f, float c_dot,
                float c_norm, hipStream_t st) {
  constexpr int kKeyWaves = (1 << WLOG) > 64 ? (1 << WLOG) / 16 : 4;
  const uint32_t ktiles = (s.T + 16 * kKeyWaves - 1) / (16 * kKeyWaves);
  // tiles per block: as many as leave about eight blocks per CU
  int32_t iters = static_cast<int32_t>((static_cast<int64_t>(s.N) * ktiles) / 2048);
  iters = iters < 1 ? 1 : (iters > 8 ? 8 : iters);
  const uint32_t bph = (ktiles + iters - 1) / iters;
  hipLaunchKernelGGL((key_state_kernel<MC, WLOG>), dim3(static_cast<uint32_t>(s.N) * bph), dim3(64 * kKeyWaves), 0, st,
                     s, K, W, f.state, f.pref, f.bsum_u, f.bsum_r, c_dot, c_norm, iters);
}

template <int MC, int WLOG>
void launch_rows_k(const Shape& s, const uint16_t* Q, const uint16_t* K, const uint16_t* W, float* A_hat,
                   uint32_t* mbits, const FusedPtrs& f, float c_dot, float c_norm, hipStream_t st) {
  const uint32_t tiles = (s.T + 63) / 64;
  const dim3 grid(static_cast<uint32_t>(s.N) * tiles);
  // heads whose state (K x m bf16 each) shares an XCD's L2 at one time: 2 MB worth
  const int64_t per_xcd = std::max<int64_t>(1, (int64_t(2) << 20) / (static_cast<int64_t>(s.K) * s.m * 2));
  const int32_t gh = static_cast<int32_t>(std::min<int64_t>(s.N, 8 * per_xcd));
  if (s.K <= 64)
    launch_rows<MC, WLOG, 4>(s, Q, K, W, A_hat, mbits, f, c_dot, c_norm, gh, grid, st);
  else if (s.K <= 128)
    launch_rows<MC, WLOG, 8>(s, Q, K, W, A_hat, mbits, f, c_dot, c_norm, gh, grid, st);
  else
    launch_rows<MC, WLOG, 16>(s, Q, K, W, A_hat, mbits, f, c_dot, c_norm, gh, grid, st);
}

template <int MC>
void launch_w(const Shape& s, int wl, const uint16_t* Q, const uint16_t* K, const uint16_t* W, float* A_hat,
              uint32_t* mbits, const FusedPtrs& f, float c_dot, float c_norm, hipStream_t st) {
  {
    StageScope scope(SEA_STAGE_STATE, st);
    switch (wl) {
      case 0: launch_key<MC, 0>(s, K, W, f, c_dot, c_norm, st); break;
      case 1: launch_key<MC, 1>(s, K, W, f, c_dot, c_norm, st); break;
      case 2: launch_key<MC, 2>(s, K, W, f, c_dot, c_norm, st); break;
      case 3: launch_key<MC, 3>(s, K, W, f, c_dot, c_norm, st); break;
      case 4: launch_key<MC, 4>(s, K, W, f, c_dot, c_norm, st); break;
      case 5: launch_key<MC, 5>(s, K, W, f, c_dot, c_norm, st); break;
      case 6: launch_key<MC, 6>(s, K, W, f, c_dot, c_norm, st); break;
      default: launch_key<MC, 7>(s, K, W, f, c_dot, c_norm, st); break;
    }
    if (wl > 7)
      hipLaunchKernelGGL(wide_columns_kernel, dim3(static_cast<uint32_t>(s.N) * s.K), dim3(256), 0, st, s,
                         f.bsum_u, f.bsum_r, f.state, f.bpref, 1 << (wl - 7));
  }
  StageScope scope(SEA_STAGE_CONTRACT, st);
  switch (wl) {
    case 0: launch_rows_k<MC, 0>(s, Q, K, W, A_hat, mbits, f, c_dot, c_norm, st); break;
    case 1: launch_rows_k<MC, 1>(s, Q, K, W, A_hat, mbits, f, c_dot, c_norm, st); break;
    case 2: launch_rows_k<MC, 2>(s, Q, K, W, A_hat, mbits, f, c_dot, c_norm, st); break;
    case 3: launch_rows_k<MC, 3>(s, Q, K, W, A_hat, mbits, f, c_dot, c_norm, st); break;
    case 4: launch_rows_k<MC, 4>(s, Q, K, W, A_hat, mbits, f, c_dot, c_norm, st); break;
    default: launch_rows_k<MC, 5>(s, Q, K, W, A_hat, mbits, f, c_dot, c_norm, st); break;
  }
}

}  // namespace

hipError_t launch_estimate_fused(const Shape& s, const uint16_t* Q, const uint16_t* K, const uint16_t* W,
                                 float* A_hat, uint32_t* mbits, void* ws, hipStream_t st) {
  if (!estimate_fused_supported(s)) return hipErrorNotSupported;
  const int wl = wlog_of(s);
  const FusedWs lay = fused_layout(s);
  char* base = static_cast<char*>(ws);
  FusedPtrs f{};
  f.state = reinterpret_cast<uint16_t*>(base + lay.state);
  if (s.causal && wl > 4) f.pref = reinterpret_cast<uint16_t*>(base + lay.pref);
  if (wl > 7) {
    f.bsum_u = reinterpret_cast<float*>(base + lay.bsum_u);
    if (s.causal) {
      f.bsum_r = reinterpret_cast<float*>(base + lay.bsum_r);
      f.bpref = reinterpret_cast<uint16_t*>(base + lay.bpref);
    }
  }
  const double l2e = 1.4426950408889634;
  const float c_dot = static_cast<float>(l2e * sqrt(static_cast<double>(s.scale)));
  const float c_norm = static_cast<float>(l2e * 0.5 * static_cast<double>(s.scale));
  switch (s.m) {
    case 64: launch_w<2>(s, wl, Q, K, W, A_hat, mbits, f, c_dot, c_norm, st); break;
    case 128: launch_w<4>(s, wl, Q, K, W, A_hat, mbits, f, c_dot, c_norm, st); break;
    default: launch_w<8>(s, wl, Q, K, W, A_hat, mbits, f, c_dot, c_norm, st); break;
  }
  return hipGetLastError();
}

}  // namespace sea

// Per-row width estimate for bf16 tensors on the bf16 matrix cores (App. A.4: a causal row t is
// resized to its own width, so its column c holds the keys [ceil(c (t+1) / K), ceil((c+1)(t+1) / K));
// Sec. 3 "Performer (FAVOR+)", Sec. 3.1 "Attention Matrix Estimation").
//
//   A^[t][c] = sum over the keys j of row t's column c of  phi~(q_t) . phi~(k_j),  then / row sum
//
// with phi~ the features rounded to bf16 (queries after a power-of-two row shift).  The products
// a_tj of 64 query rows x 32 keys are two tiles of phi~(K) phi~(Q)^T (v_mfma_f32_32x32x16_bf16,
// fp32 accumulation); every a_tj is then added to the bin of its column floor(j K / (t + 1)) in LDS.
// Nothing is differenced, so there is no cancellation, and no prefix state exists.  The bins are
// fp64: the LDS adds 64 doubles in about 11 clocks but needs about 170 for 64 floats (measured,
// ds_add_f64 against ds_add_f32), and the binning is what bounds this kernel.
//
//   rw_features_kernel   phi~(Q), phi~(K) -> HBM, already in the order the tile kernel's lanes
//                        consume them: [head][32-token chunk][step][lane][8 features], so every
//                        operand load of the tile kernel is one contiguous 1 KB piece
//   rw_tiles_mfma_kernel one wavefront per (head, 64 query rows, column part): walks the 32-key
//                        chunks its columns cover, bins, normalises, writes fp32 A^
//
// Column parts: a wave keeps the bins of at most 32 columns ([64 rows][<= 32] fp64 = 18 KB), so that
// a CU holds eight waves, two per SIMD; the ceil(K / 32) parts of a row tile are taken by the (at
// most eight) waves of one block, which meet only for the row sums.  The columns of a row are monotone in the key index, so part p walks only the keys of its
// own columns: the work is split, not repeated.
#include <algorithm>

#include "sea_internal.h"

namespace sea {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kWRow = 72;      // halfwords per staged W row (128 B + 16 B pad): conflict-free b128 reads
constexpr int kChunk = 32;     // tokens per feature chunk = keys per step of the tile kernel
constexpr int kTileRows = 64;  // query rows of a wavefront
constexpr int kPartCols = 32;  // columns whose bins one wavefront keeps

__device__ __forceinline__ floatx4 mfma16(bf16x8 a, bf16x8 b, floatx4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ floatx16 mfma32(bf16x8 a, bf16x8 b, floatx16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
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
// Features.  The projection is taken transposed, C[feature][token] = W X^T (v_mfma_f32_16x16x32_bf16):
// lane l owns token l % 16 and, per 16-feature tile ft, the features 16 ft + 4 (l / 16) + i.  Two
// consecutive tiles give a lane 8 rounded values = one 16-byte piece; piece (kc, lg) of a token
// becomes contraction step 2 kc + lg / 2, lane half lg % 2 of the tile kernel's operands.  Which
// feature sits in which contraction slot is irrelevant as long as queries and keys agree.
//
// Operand row of a token within its 32-token chunk: queries keep their order (row = token).  Keys
// are permuted so that result register i of lane half h' is key 16 h' + i of the chunk: key
// 16 h' + 4 a + b sits in operand row 8 a + 4 h' + b.
//
// grid (N * blocks per head, 2): y = 0 queries, y = 1 keys.  A block parks W once and takes
// `iters` consecutive 64-token tiles.
// ------------------------------------------------------------------------------------------
template <int MC>  // m / 32
__global__ __launch_bounds__(256) void rw_features_kernel(Shape s, const uint16_t* __restrict__ Q,
                                                          const uint16_t* __restrict__ K,
                                                          const uint16_t* __restrict__ W, uint4* __restrict__ phiQ,
                                                          uint4* __restrict__ phiK, float c_dot, float c_norm,
                                                          int32_t iters) {
  constexpr int m = 32 * MC;
  constexpr int MS = 2 * MC;  // contraction steps of the tile kernel
  __shared__ __attribute__((aligned(16))) uint16_t Ws[m * kWRow];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lr = lane & 15, lg = lane >> 4;
  const bool keys = blockIdx.y != 0;
  const uint32_t nch = (s.T + kChunk - 1) / kChunk;
  const uint32_t tiles = (nch + 1) / 2;
  const uint32_t bph = (tiles + iters - 1) / iters;
  const int64_t head = blockIdx.x / bph;
  const uint32_t first = (blockIdx.x % bph) * iters;
  for (int x = tid; x < m * 8; x += 256) {
    const int r = x >> 3, part = x & 7;
    *reinterpret_cast<uint4*>(&Ws[r * kWRow + part * 8]) = *reinterpret_cast<const uint4*>(W + r * kHeadDim + part * 8);
  }
  __syncthreads();
  const int32_t b = static_cast<int32_t>(head / s.H);
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
  const uint16_t* src = keys ? K : Q;
  uint4* dst = keys ? phiK : phiQ;
  for (uint32_t tile = first; tile < min(first + static_cast<uint32_t>(iters), tiles); ++tile) {
    const uint32_t chunk = 2 * tile + (wid >> 1);
    if (chunk >= nch) continue;  // wave-uniform
    const int32_t kappa = 16 * (wid & 1) + lr;
    const int32_t tok = static_cast<int32_t>(chunk) * kChunk + kappa;
    const uint16_t* X = src + (head * s.T + min(tok, s.T - 1)) * kHeadDim;
    const bf16x8 x0 = *reinterpret_cast<const bf16x8*>(X + 8 * lg);
    const bf16x8 x1 = *reinterpret_cast<const bf16x8*>(X + 32 + 8 * lg);
    float nx = sumsq8(x0) + sumsq8(x1);
    nx += __shfl_xor(nx, 16, kWave);
    nx += __shfl_xor(nx, 32, kWave);  // |x|^2 of token lr, in every lane group
    floatx4 dots[2 * MC];
#pragma unroll
    for (int ft = 0; ft < 2 * MC; ++ft) {
      const uint16_t* w = &Ws[(ft * 16 + lr) * kWRow + 8 * lg];
      floatx4 acc = {0.f, 0.f, 0.f, 0.f};
      acc = mfma16(*reinterpret_cast<const bf16x8*>(w), x0, acc);
      dots[ft] = mfma16(*reinterpret_cast<const bf16x8*>(w + 32), x1, acc);
    }
    // Exponent offset (log2 units).  Keys: the norm term alone.  Queries: also minus the row's
    // largest argument rounded up, a power-of-two row scale that commutes with the bf16 rounding
    // and cancels in the row normalisation.  Tokens past the sequence end: all-zero features.
    float off = -(c_norm * nx);
    if (!keys) {
      float dmax = -INFINITY;
#pragma unroll
      for (int ft = 0; ft < 2 * MC; ++ft)
#pragma unroll
        for (int i = 0; i < 4; ++i) dmax = fmaxf(dmax, dots[ft][i]);
      dmax = fmaxf(dmax, __shfl_xor(dmax, 16, kWave));
      dmax = fmaxf(dmax, __shfl_xor(dmax, 32, kWave));
      off -= ceilf(fmaf(c_dot, dmax, off));
    }
    if (tok >= len) off = -INFINITY;
    const int32_t row = keys ? 8 * ((kappa & 15) >> 2) + 4 * (kappa >> 4) + (kappa & 3) : kappa;
    uint4* out = dst + ((head * nch + chunk) * MS + (lg >> 1)) * 64 + 32 * (lg & 1) + row;
#pragma unroll
    for (int kc = 0; kc < MC; ++kc) {
      float v[8];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        v[i] = __builtin_amdgcn_exp2f(fmaf(c_dot, dots[2 * kc][i], off));
        v[4 + i] = __builtin_amdgcn_exp2f(fmaf(c_dot, dots[2 * kc + 1][i], off));
      }
      uint4 u;
      u.x = pack_bf16(v[0], v[1]);
      u.y = pack_bf16(v[2], v[3]);
      u.z = pack_bf16(v[4], v[5]);
      u.w = pack_bf16(v[6], v[7]);
      out[2 * kc * 64] = u;
    }
  }
}

// ------------------------------------------------------------------------------------------
// Tiles.  Block = P <= 8 wavefronts working on one (head, 64-row tile); wave w takes the column
// parts w, w + P, ... (one pass of the loop below per part; a single pass whenever K <= 256).  Lane l of
// a wave owns the query rows r0 + l % 32 and r0 + 32 + l % 32 and, in every 32-key chunk, the 16
// keys 16 (l / 32) + i of the chunk (see the key permutation above).
//
// Column of key j in row t: floor(j K / (t + 1)).  WIDE = false takes it in fp32 as
// trunc(j * (K / (t+1)) + 1 / (2 (t+1))) = trunc((j K + 1/2) / (t + 1)): j is exact, K / (t + 1)
// carries two roundings and the fused multiply-add a third, 3 * 2^-24 relative in all; the true
// quotient is at most K and lies at least 1 / (2 (t + 1)) away from every integer, so the
// truncation is exact while K (t + 1) < 2^24 / 6 (the launcher takes this form for K T <= 2^21).
// WIDE = true does the same in fp64 on the exact integer j K, where the half step exceeds the
// rounding error for any size the library accepts.  Keys j > t give a quotient >= K and keys outside the
// wave's columns one outside [c_lo, c_hi): both are clamped into a guard slot on either side of
// the row's bins, so no product needs a predicate.  Padding keys and rows past the end have
// all-zero features and add zeros.
// ------------------------------------------------------------------------------------------
template <int MS, bool WIDE>  // MS = m / 16: contraction steps
__global__ __launch_bounds__(512) void rw_tiles_mfma_kernel(Shape s, const uint4* __restrict__ phiQ,
                                                            const uint4* __restrict__ phiK,
                                                            float* __restrict__ A_hat, int32_t parts,
                                                            int32_t part_cols, int32_t stride, int32_t cshift) {
  extern __shared__ __align__(16) double lds[];  // [P][64 rows][stride] bins, [64][P] row sums, [64] inverses
  const int lane = threadIdx.x & 63, q = lane & 31, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int P = blockDim.x >> 6;
  double* bins = lds + static_cast<size_t>(wave) * kTileRows * stride;
  double* tot_s = lds + static_cast<size_t>(P) * kTileRows * stride;
  const uint32_t nch = (s.T + kChunk - 1) / kChunk;
  const uint32_t tiles = (s.T + kTileRows - 1) / kTileRows;
  // Head-major, each XCD on a contiguous range of blocks: the row tiles of a head run close together
  // on one XCD, whose L2 then serves all but the first read of the head's key features.  Within a
  // head the longest (last) row tiles come first.
  const uint32_t lb = xcd_contiguous(blockIdx.x, gridDim.x);
  const int64_t head = lb / tiles;
  const uint32_t tile = tiles - 1 - lb % tiles;
  const int32_t r0 = static_cast<int32_t>(tile) * kTileRows;
  const int32_t b = static_cast<int32_t>(head / s.H);
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
  const int32_t r_last = min(min(r0 + kTileRows - 1, s.T - 1), len - 1);  // last active row of the tile
  const int32_t passes = (parts + P - 1) / P;
  // lane <-> (row, column) of a part when its bins leave: 2^cshift >= part_cols columns side by side
  const int32_t csub = lane & ((1 << cshift) - 1), rsub = lane >> cshift;

  bf16x8 qf[2][MS];
  float kinv[2], hinv[2];
  double winv[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const uint32_t tile32 = 2 * tile + u;
    const uint4* qp = phiQ + ((head * nch + min(tile32, nch - 1)) * MS) * 64 + lane;
#pragma unroll
    for (int st = 0; st < MS; ++st) {
      uint4 v = qp[st * 64];
      if (tile32 >= nch) v = uint4{0u, 0u, 0u, 0u};
      qf[u][st] = __builtin_bit_cast(bf16x8, v);
    }
    const int32_t t1 = r0 + 32 * u + q + 1;
    const float inv = 1.0f / static_cast<float>(t1);
    kinv[u] = static_cast<float>(s.K) * inv;
    hinv[u] = 0.5f * inv;
    winv[u] = 1.0 / static_cast<double>(t1);
  }
  const uint4* kp = phiK + (head * nch * MS) * 64 + lane;
  auto request = [&](bf16x8 (&kf)[MS], int32_t c) {
#pragma unroll
    for (int st = 0; st < MS; ++st)
      kf[st] = __builtin_bit_cast(bf16x8, kp[(static_cast<int64_t>(c) * MS + st) * 64]);
  };
  double rowtot[2] = {0.0, 0.0};  // row sums over the parts this wave has finished (rows q, 32 + q)

  for (int32_t pass = 0; pass < passes; ++pass) {
    const int32_t part = pass * P + wave;
    const int32_t c_lo = min(part * part_cols, s.K), c_hi = min(s.K, c_lo + part_cols);
    const int32_t ncols = c_hi - c_lo;
    for (int32_t x = lane; x < kTileRows * stride; x += 64) bins[x] = 0.0;
    // index in `bins` of column 0 of the lane's two rows: column c sits in slot c - (c_lo - 1), the
    // guards in slots 0 and ncols + 1
    const int32_t base[2] = {q * stride - (c_lo - 1), (32 + q) * stride - (c_lo - 1)};
    // keys the wave's columns cover over the active rows: column starts grow with the row, so the
    // first key is row r0's start of c_lo and the last one precedes the last active row's start of c_hi
    int32_t cb = 0, ce = 0;
    if (r_last >= r0 && ncols > 0) {
      const int64_t j_begin = (static_cast<int64_t>(c_lo) * (r0 + 1) + s.K - 1) / s.K;
      const int64_t j_end = (static_cast<int64_t>(c_hi) * (r_last + 1) + s.K - 1) / s.K;
      cb = static_cast<int32_t>(j_begin / kChunk);
      ce = static_cast<int32_t>((j_end + kChunk - 1) / kChunk);
    }
    const float lo_f = static_cast<float>(c_lo - 1), hi_f = static_cast<float>(c_hi);  // the guards
    // product i of chunk c in lane half h belongs to key 32 c + 16 h + i
    auto bin = [&](const floatx16 (&acc)[2], int32_t c, int i) {
      const int32_t j = c * kChunk + 16 * h + i;
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        int32_t slot;
        if (WIDE) {
          const int32_t col = static_cast<int32_t>((static_cast<double>(static_cast<int64_t>(j) * s.K) + 0.5) * winv[u]);
          slot = min(max(col, c_lo - 1), c_hi);
        } else {
          // quotient clamped to the guards first: both are integers, so truncation commutes with the clamp
          slot = static_cast<int32_t>(__builtin_amdgcn_fmed3f(fmaf(static_cast<float>(j), kinv[u], hinv[u]), lo_f, hi_f));
        }
        atomicAdd(&bins[base[u] + slot], static_cast<double>(acc[u][i]));
      }
    };
    __syncthreads();  // bins are clear (and, after the first pass, the previous part has left them)
    if (cb < ce) {
      // A SIMD holds two waves of this kernel: one's matrix products run under the other's binning.
      // Within the wave the next chunk's fragments are requested as soon as the products have
      // consumed the current ones, and arrive while the products are binned.
      bf16x8 kf[MS];
      request(kf, cb);
      for (int32_t c = cb; c < ce; ++c) {
        floatx16 acc[2];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int i = 0; i < 16; ++i) acc[u][i] = 0.f;
#pragma unroll
        for (int st = 0; st < MS; ++st) {
          acc[0] = mfma32(kf[st], qf[0][st], acc[0]);
          acc[1] = mfma32(kf[st], qf[1][st], acc[1]);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (c + 1 < ce) request(kf, c + 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 16; ++i) bin(acc, c, i);
      }
    }
    __syncthreads();  // every product of the part is in its bin
    // row sums of the part: lane (q, h) adds the columns c = h (mod 2) of its two rows, the halves
    // meet by a lane swap
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const double* row = bins + (32 * u + q) * stride + 1;
      double part_sum = 0.0;
      for (int32_t c = h; c < ncols; c += 2) part_sum += row[c];
      part_sum += __shfl_xor(part_sum, 32, kWave);
      rowtot[u] += part_sum;
    }
    if (passes > 1) {
      // more parts than the block has waves: the bins leave as they are, the rows are scaled at the end
      for (int32_t row = rsub; row < kTileRows && r0 + row < s.T; row += kTileRows >> cshift)
        if (csub < ncols)
          A_hat[(head * s.T + r0 + row) * s.K + c_lo + csub] = static_cast<float>(bins[row * stride + 1 + csub]);
    }
  }
  if (h == 0) {
    tot_s[q * P + wave] = rowtot[0];
    tot_s[(32 + q) * P + wave] = rowtot[1];
  }
  __syncthreads();
  double* inv_s = tot_s + kTileRows * P;  // [64] 1 / row sum
  if (wave == 0) {
    double total = 0.0;
    for (int32_t w = 0; w < P; ++w) total += tot_s[lane * P + w];
    inv_s[lane] = (r0 + lane < len && total > 0.0) ? 1.0 / total : 0.0;
  }
  __syncthreads();
  if (passes == 1) {
    const int32_t c_lo = min(wave * part_cols, s.K), ncols = min(s.K, c_lo + part_cols) - c_lo;
    for (int32_t row = rsub; row < kTileRows && r0 + row < s.T; row += kTileRows >> cshift)
      if (csub < ncols)
        A_hat[(head * s.T + r0 + row) * s.K + c_lo + csub] =
            static_cast<float>(bins[row * stride + 1 + csub] * inv_s[row]);
  } else {
    // every lane scales the values it wrote itself (same wave, same part, same lane mapping)
    for (int32_t pass = 0; pass < passes; ++pass) {
      const int32_t c_lo = min((pass * P + wave) * part_cols, s.K), ncols = min(s.K, c_lo + part_cols) - c_lo;
      for (int32_t row = rsub; row < kTileRows && r0 + row < s.T; row += kTileRows >> cshift)
        if (csub < ncols) {
          float* out = A_hat + (head * s.T + r0 + row) * s.K + c_lo + csub;
          *out = static_cast<float>(static_cast<double>(*out) * inv_s[row]);
        }
    }
  }
}

struct Plan {
  int32_t parts, part_cols, stride, waves, cshift;
  size_t lds;
};
Plan plan(const Shape& s) {
  Plan p{};
  p.parts = (s.K + kPartCols - 1) / kPartCols;
  p.part_cols = (s.K + p.parts - 1) / p.parts;
  p.stride = (p.part_cols + 2) | 1;  // two guards; odd, so the 32 rows of a step fall into different banks
  p.waves = std::min(p.parts, 8);    // eight waves' bins fit a CU's LDS: two waves per SIMD
  while ((1 << p.cshift) < p.part_cols) ++p.cshift;
  p.lds = (static_cast<size_t>(p.waves) * kTileRows * p.stride + static_cast<size_t>(kTileRows) * (p.waves + 1)) * sizeof(double);
  return p;
}
size_t side_bytes(const Shape& s) {
  const size_t t32 = (static_cast<size_t>(s.T) + kChunk - 1) / kChunk * kChunk;
  return (static_cast<size_t>(s.N) * t32 * s.m * sizeof(uint16_t) + 255) & ~size_t(255);
}

template <int MC>
hipError_t launch(const Shape& s, const uint16_t* Q, const uint16_t* K, const uint16_t* W, float* A_hat,
                  void* ws, hipStream_t st) {
  uint4* phiQ = static_cast<uint4*>(ws);
  uint4* phiK = reinterpret_cast<uint4*>(static_cast<char*>(ws) + side_bytes(s));
  const double l2e = 1.4426950408889634;
  const float c_dot = static_cast<float>(l2e * std::sqrt(static_cast<double>(s.scale)));
  const float c_norm = static_cast<float>(l2e * 0.5 * static_cast<double>(s.scale));
  {
    StageScope scope(SEA_STAGE_FEATURES, st);
    const uint32_t nch = (s.T + kChunk - 1) / kChunk, tiles = (nch + 1) / 2;
    const int32_t iters = static_cast<int32_t>(std::min<int64_t>(8, std::max<int64_t>(1, static_cast<int64_t>(s.N) * tiles / 1024)));
    const uint32_t bph = (tiles + iters - 1) / iters;
    hipLaunchKernelGGL(rw_features_kernel<MC>, dim3(static_cast<uint32_t>(s.N) * bph, 2), dim3(256), 0, st, s, Q, K,
                       W, phiQ, phiK, c_dot, c_norm, iters);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  StageScope scope(SEA_STAGE_CONTRACT, st);
  const Plan p = plan(s);
  const bool wide = static_cast<int64_t>(s.K) * s.T > (int64_t{1} << 21);
  const void* fn = wide ? reinterpret_cast<const void*>(&rw_tiles_mfma_kernel<2 * MC, true>)
                        : reinterpret_cast<const void*>(&rw_tiles_mfma_kernel<2 * MC, false>);
  if (p.lds > (64u << 10)) {
    const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(p.lds));
    if (e != hipSuccess) return e;
  }
  const uint32_t tiles = (s.T + kTileRows - 1) / kTileRows;
  const dim3 grid(static_cast<uint32_t>(s.N) * tiles), block(64 * p.waves);
  if (wide)
    hipLaunchKernelGGL((rw_tiles_mfma_kernel<2 * MC, true>), grid, block, p.lds, st, s, phiQ, phiK, A_hat, p.parts,
                       p.part_cols, p.stride, p.cshift);
  else
    hipLaunchKernelGGL((rw_tiles_mfma_kernel<2 * MC, false>), grid, block, p.lds, st, s, phiQ, phiK, A_hat, p.parts,
                       p.part_cols, p.stride, p.cshift);
  return hipGetLastError();
}

}  // namespace

bool rowwidth_mfma_supported(const Shape& s, sea_dtype dt) {
  return dt == SEA_BF16 && s.causal && (s.m == 64 || s.m == 128 || s.m == 256);
}

size_t rowwidth_mfma_workspace(const Shape& s) { return 2 * side_bytes(s); }

hipError_t launch_rowwidth_mfma(const Shape& s, const uint16_t* Q, const uint16_t* K, const uint16_t* W,
                                float* A_hat, void* ws, hipStream_t st) {
  switch (s.m) {
    case 64: return launch<2>(s, Q, K, W, A_hat, ws, st);
    case 128: return launch<4>(s, Q, K, W, A_hat, ws, st);
    default: return launch<8>(s, Q, K, W, A_hat, ws, st);
  }
}

}  // namespace sea

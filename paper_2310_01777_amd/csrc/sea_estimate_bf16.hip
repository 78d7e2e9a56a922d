// Random-feature estimate of the compressed attention matrix on the CDNA4 matrix cores
// (Sec. 3 "Performer (FAVOR+)", Sec. 3.1 "Attention Matrix Estimation"), bf16 operands with
// fp32 accumulation.
//
//   phi(x)[i] = exp(w_i.x - |x|^2/2), x = sqrt(scale) q;  state = phi(K)^T V_I (K x m bucket
//   sums, V_I the nearest-neighbour stretched identity);  A_hat = rownorm(phi(Q) state), a
//   causal row using the inclusive prefix of its own bucket instead of the full bucket sum.
//
// Rounding points (the only places a value is narrowed to bf16): phi(Q) after a power-of-two
// row shift (which commutes with the rounding), the bucket sums, and phi(k_j) of the keys of a
// causal row's own bucket (that column is summed key by key, products accumulated in fp32).
//
// All three GEMM-shaped steps are "NT" products whose operands are row-major with the
// contraction index contiguous, which is exactly the register layout of
// v_mfma_f32_16x16x32_bf16 (lane l: row/col l % 16, contraction elements 8 (l / 16) .. +7),
// so fragments are loaded straight from memory with one 128-bit load per lane.
//
// Workspace layout: phiQ bf16 [N][T][m] | phiK f32 [N][T][m] | state bf16 [N][K][m] |
// phiKb bf16 [N][T][m] (causal only).
#include "sea_internal.h"

namespace sea {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8 load_frag(const uint16_t* p) {
  return *reinterpret_cast<const bf16x8*>(p);
}
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
__device__ __forceinline__ float dot8(bf16x8 x, bf16x8 y, float a) {
  const uint4 u = __builtin_bit_cast(uint4, x), v = __builtin_bit_cast(uint4, y);
  const uint32_t p[4] = {u.x, u.y, u.z, u.w}, q[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a = fmaf(bf16lo_to_f32(p[i]), bf16lo_to_f32(q[i]), a);
    a = fmaf(bf16hi_to_f32(p[i]), bf16hi_to_f32(q[i]), a);
  }
  return a;
}

// ------------------------------------------------------------------------------------------
// a1: feature maps.  Block = 4 waves, wave = 16 rows of one head; C[feature][row] = W X^T.
// grid.x = 2 * N * ceil(T / 64): first half queries, second half keys.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void features_bf16_kernel(
    Shape s, const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K,
    const uint16_t* __restrict__ W, uint16_t* __restrict__ phiQ, float* __restrict__ phiK,
    float c_dot, float c_norm) {
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
  const int lr = lane & 15, lg = lane >> 4;
  const uint32_t tiles = (s.T + 63) / 64;
  const uint32_t half = static_cast<uint32_t>(s.N) * tiles;
  const int which = blockIdx.x >= half;
  const uint32_t bid = which ? blockIdx.x - half : blockIdx.x;
  const int64_t head = bid / tiles;
  const int32_t r0 = static_cast<int32_t>(bid % tiles) * 64 + wid * 16;
  if (r0 >= s.T) return;
  const int32_t t = r0 + lr;                  // this lane's row (as MFMA column)
  const int32_t tc = min(t, s.T - 1);         // clamped for loads
  const int32_t b = static_cast<int32_t>(head / s.H);
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
  const uint16_t* X = (which ? K : Q) + (head * s.T + tc) * kHeadDim;
  const bf16x8 x0 = load_frag(X + 8 * lg), x1 = load_frag(X + 32 + 8 * lg);
  float nx = sumsq8(x0) + sumsq8(x1);
  nx += __shfl_xor(nx, 16, kWave);
  nx += __shfl_xor(nx, 32, kWave);
  const float bias = c_norm * nx;  // log2(e) * scale * |q|^2 / 2
  const int ftiles = s.m / 16;
  const bool active = t < len;     // t < len <= T

  if (!which) {
    // pass 1: row maximum of the exponent (log2 domain)
    float amax = -INFINITY;
    for (int ft = 0; ft < ftiles; ++ft) {
      const uint16_t* w = W + (ft * 16 + lr) * kHeadDim;
      floatx4 acc = {0.f, 0.f, 0.f, 0.f};
      acc = mfma16(load_frag(w + 8 * lg), x0, acc);
      acc = mfma16(load_frag(w + 32 + 8 * lg), x1, acc);
#pragma unroll
      for (int i = 0; i < 4; ++i) amax = fmaxf(amax, fmaf(c_dot, acc[i], -bias));
    }
    amax = fmaxf(amax, __shfl_xor(amax, 16, kWave));
    amax = fmaxf(amax, __shfl_xor(amax, 32, kWave));
    const float shift = ceilf(amax);  // power-of-two row scale: commutes with bf16 rounding
    uint16_t* out = phiQ + (head * s.T + tc) * s.m;
    for (int ft = 0; ft < ftiles; ++ft) {
      const uint16_t* w = W + (ft * 16 + lr) * kHeadDim;
      floatx4 acc = {0.f, 0.f, 0.f, 0.f};
      acc = mfma16(load_frag(w + 8 * lg), x0, acc);
      acc = mfma16(load_frag(w + 32 + 8 * lg), x1, acc);
      float v[4];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        v[i] = active ? exp2f(fmaf(c_dot, acc[i], -bias) - shift) : 0.f;
      if (t < s.T) {
        uint2 pk;
        pk.x = pack_bf16(v[0], v[1]);
        pk.y = pack_bf16(v[2], v[3]);
        *reinterpret_cast<uint2*>(out + ft * 16 + 4 * lg) = pk;
      }
    }
  } else {
    float* out = phiK + (head * s.T + tc) * s.m;
    for (int ft = 0; ft < ftiles; ++ft) {
      const uint16_t* w = W + (ft * 16 + lr) * kHeadDim;
      floatx4 acc = {0.f, 0.f, 0.f, 0.f};
      acc = mfma16(load_frag(w + 8 * lg), x0, acc);
      acc = mfma16(load_frag(w + 32 + 8 * lg), x1, acc);
      float4 v;
      v.x = active ? exp2f(fmaf(c_dot, acc[0], -bias)) : 0.f;
      v.y = active ? exp2f(fmaf(c_dot, acc[1], -bias)) : 0.f;
      v.z = active ? exp2f(fmaf(c_dot, acc[2], -bias)) : 0.f;
      v.w = active ? exp2f(fmaf(c_dot, acc[3], -bias)) : 0.f;
      if (t < s.T) *reinterpret_cast<float4*>(out + ft * 16 + 4 * lg) = v;
    }
  }
}

// ------------------------------------------------------------------------------------------
// a2: key-side state.  One thread per (head, column, feature) walks the keys of the column.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void state_bf16_kernel(Shape s, const float* __restrict__ phiK,
                                                         uint16_t* __restrict__ state,
                                                         uint16_t* __restrict__ prefix) {
  const int64_t gid = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  const int64_t total = static_cast<int64_t>(s.N) * s.K * s.m;
  if (gid >= total) return;
  const int32_t i = static_cast<int32_t>(gid % s.m);
  const int32_t c = static_cast<int32_t>((gid / s.m) % s.K);
  const int64_t head = gid / (static_cast<int64_t>(s.m) * s.K);
  const int32_t j0 = block_start(c, s.T, s.K), j1 = block_start(c + 1, s.T, s.K);
  const float* col = phiK + (head * s.T) * s.m + i;
  float acc = 0.f;
  if (prefix) {  // also keep each key's features, rounded, for the causal diagonal column
    uint16_t* pf = prefix + (head * s.T) * s.m + i;
    for (int32_t j = j0; j < j1; ++j) {
      const float f = col[static_cast<int64_t>(j) * s.m];
      acc += f;
      pf[static_cast<int64_t>(j) * s.m] = f32_to_bf16(f);
    }
  } else {
    for (int32_t j = j0; j < j1; ++j) acc += col[static_cast<int64_t>(j) * s.m];
  }
  state[(head * s.K + c) * s.m + i] = f32_to_bf16(acc);
}

// ------------------------------------------------------------------------------------------
// a3: A_hat tile = phiQ[16 rows] x state^T, 16 columns per MFMA tile, up to 256 columns per
// register group.  Block = 4 waves = 64 rows of one head.
// MC = m / 32 when the phiQ fragments fit in registers (MC <= 16), else 0 (reload).
// ------------------------------------------------------------------------------------------
constexpr int kGroupTiles = 16;  // 256 columns

template <int MC>
__global__ __launch_bounds__(256) void contract_bf16_kernel(
    Shape s, const uint16_t* __restrict__ phiQ, const uint16_t* __restrict__ state,
    const uint16_t* __restrict__ prefix, float* __restrict__ A_hat) {
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
  const int lr = lane & 15, lg = lane >> 4;
  const uint32_t tiles = (s.T + 63) / 64;
  const int64_t head = blockIdx.x / tiles;
  const int32_t r0 = static_cast<int32_t>(blockIdx.x % tiles) * 64 + wid * 16;
  if (r0 >= s.T) return;
  const int32_t b = static_cast<int32_t>(head / s.H);
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
  const int mc = s.m / 32;

  // A fragments: row r0 + lr of phiQ
  const int32_t ta = min(r0 + lr, s.T - 1);
  const uint16_t* qrow = phiQ + (head * s.T + ta) * s.m + 8 * lg;
  bf16x8 afrag[MC > 0 ? MC : 1];
  if (MC > 0) {
#pragma unroll
    for (int kc = 0; kc < MC; ++kc) afrag[kc] = load_frag(qrow + kc * 32);
  }
  // diagonal column of the causal rows: sum over the keys j <= t of the row's own bucket of
  // phiQ[t] . phiKb[j]; rows as lanes lr
  float diag_lr = 0.f;
  if (s.causal) {
    const int32_t jb = block_start(bucket_of(ta, s.T, s.K), s.T, s.K);
    for (int32_t j = jb; j <= ta; ++j) {
      const uint16_t* prow = prefix + (head * s.T + j) * s.m + 8 * lg;
      if (MC > 0) {
#pragma unroll
        for (int kc = 0; kc < MC; ++kc) diag_lr = dot8(afrag[kc], load_frag(prow + kc * 32), diag_lr);
      } else {
        for (int kc = 0; kc < mc; ++kc)
          diag_lr = dot8(load_frag(qrow + kc * 32), load_frag(prow + kc * 32), diag_lr);
      }
    }
    diag_lr += __shfl_xor(diag_lr, 16, kWave);
    diag_lr += __shfl_xor(diag_lr, 32, kWave);
  }
  // accumulator rows of this lane: r0 + 4 lg + i
  int32_t trow[4], ctrow[4];
  float diag[4];
  bool act[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    trow[i] = r0 + 4 * lg + i;
    act[i] = trow[i] < len;
    ctrow[i] = s.causal ? bucket_of(min(trow[i], s.T - 1), s.T, s.K) : s.K;  // first masked column
    diag[i] = __shfl(diag_lr, 4 * lg + i, kWave);
  }
  const uint16_t* st = state + head * s.K * s.m + 8 * lg;
  float* out = A_hat + (head * s.T) * s.K;
  const int ctiles = (s.K + 15) / 16;
  const int ngroups = (ctiles + kGroupTiles - 1) / kGroupTiles;
  float rsum[4] = {0.f, 0.f, 0.f, 0.f};
  floatx4 acc[kGroupTiles];

  for (int g = 0; g < ngroups; ++g) {
#pragma unroll
    for (int ct = 0; ct < kGroupTiles; ++ct) {
      const int tile = g * kGroupTiles + ct;
      acc[ct] = floatx4{0.f, 0.f, 0.f, 0.f};
      if (tile < ctiles) {
        const int32_t c = min(tile * 16 + lr, s.K - 1);
        const uint16_t* brow = st + static_cast<int64_t>(c) * s.m;
        if (MC > 0) {
#pragma unroll
          for (int kc = 0; kc < MC; ++kc) acc[ct] = mfma16(afrag[kc], load_frag(brow + kc * 32), acc[ct]);
        } else {
          for (int kc = 0; kc < mc; ++kc)
            acc[ct] = mfma16(load_frag(qrow + kc * 32), load_frag(brow + kc * 32), acc[ct]);
        }
        const int32_t cc = tile * 16 + lr;  // this lane's column
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float v = acc[ct][i];
          if (cc == ctrow[i]) v = diag[i];
          if (cc > ctrow[i] || cc >= s.K || !act[i]) v = 0.f;
          acc[ct][i] = v;
          rsum[i] += v;
        }
      }
    }
    if (ngroups > 1) {  // park the raw values; rescaled below by the same lane
#pragma unroll
      for (int ct = 0; ct < kGroupTiles; ++ct) {
        const int32_t cc = (g * kGroupTiles + ct) * 16 + lr;
        if (cc < s.K) {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (trow[i] < s.T) out[static_cast<int64_t>(trow[i]) * s.K + cc] = acc[ct][i];
        }
      }
    }
  }
  float inv[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float r = rsum[i];
    r += __shfl_xor(r, 1, kWave);
    r += __shfl_xor(r, 2, kWave);
    r += __shfl_xor(r, 4, kWave);
    r += __shfl_xor(r, 8, kWave);
    inv[i] = r > 0.f ? 1.f / r : 0.f;
  }
  if (ngroups == 1) {
#pragma unroll
    for (int ct = 0; ct < kGroupTiles; ++ct) {
      const int32_t cc = ct * 16 + lr;
      if (cc < s.K) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (trow[i] < s.T) out[static_cast<int64_t>(trow[i]) * s.K + cc] = acc[ct][i] * inv[i];
      }
    }
  } else {
    for (int32_t cc = lr; cc < s.K; cc += 16) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (trow[i] < s.T) out[static_cast<int64_t>(trow[i]) * s.K + cc] *= inv[i];
    }
  }
}

}  // namespace

size_t estimate_bf16_workspace(const Shape& s) {
  // common shapes run the fused kernels, whose scratch is the K x m state and the prefix planes
  if (estimate_fused_supported(s)) return estimate_fused_workspace(s);
  const size_t ntm = static_cast<size_t>(s.N) * s.T * s.m;
  const size_t nkm = static_cast<size_t>(s.N) * s.K * s.m;
  size_t bytes = ntm * 2 + ntm * 4 + ((nkm * 2 + 255) & ~size_t(255));
  if (s.causal) bytes += ntm * 2;
  return bytes;
}

hipError_t launch_estimate_bf16(const Shape& s, const uint16_t* Q, const uint16_t* K,
                                const uint16_t* W, float* A_hat, void* ws, hipStream_t st) {
  // common shapes: two fused kernels, features never leave the chip (its scratch, the K x m
  // state, fits in the front of this path's workspace)
  if (estimate_fused_supported(s)) return launch_estimate_fused(s, Q, K, W, A_hat, nullptr, ws, st);
  const size_t ntm = static_cast<size_t>(s.N) * s.T * s.m;
  const size_t nkm = static_cast<size_t>(s.N) * s.K * s.m;
  char* base = static_cast<char*>(ws);
  uint16_t* phiQ = reinterpret_cast<uint16_t*>(base);
  float* phiK = reinterpret_cast<float*>(base + ntm * 2);
  uint16_t* state = reinterpret_cast<uint16_t*>(base + ntm * 6);
  uint16_t* prefix = s.causal
                         ? reinterpret_cast<uint16_t*>(base + ntm * 6 + ((nkm * 2 + 255) & ~size_t(255)))
                         : nullptr;
  const uint32_t tiles = (s.T + 63) / 64;
  const double l2e = 1.4426950408889634;
  const float c_dot = static_cast<float>(l2e * sqrt(static_cast<double>(s.scale)));
  const float c_norm = static_cast<float>(l2e * 0.5 * static_cast<double>(s.scale));
  {
    StageScope scope(SEA_STAGE_FEATURES, st);
    hipLaunchKernelGGL(features_bf16_kernel, dim3(2u * s.N * tiles), dim3(256), 0, st, s, Q, K, W,
                       phiQ, phiK, c_dot, c_norm);
  }
  {
    StageScope scope(SEA_STAGE_STATE, st);
    const int64_t total = static_cast<int64_t>(s.N) * s.K * s.m;
    hipLaunchKernelGGL(state_bf16_kernel, dim3(static_cast<uint32_t>((total + 255) / 256)), dim3(256),
                       0, st, s, phiK, state, prefix);
  }
  {
    StageScope scope(SEA_STAGE_CONTRACT, st);
    const dim3 grid(static_cast<uint32_t>(s.N) * tiles), block(256);
    switch (s.m / 32) {
      case 1: hipLaunchKernelGGL(contract_bf16_kernel<1>, grid, block, 0, st, s, phiQ, state, prefix, A_hat); break;
      case 2: hipLaunchKernelGGL(contract_bf16_kernel<2>, grid, block, 0, st, s, phiQ, state, prefix, A_hat); break;
      case 4: hipLaunchKernelGGL(contract_bf16_kernel<4>, grid, block, 0, st, s, phiQ, state, prefix, A_hat); break;
      case 8: hipLaunchKernelGGL(contract_bf16_kernel<8>, grid, block, 0, st, s, phiQ, state, prefix, A_hat); break;
      case 16: hipLaunchKernelGGL(contract_bf16_kernel<16>, grid, block, 0, st, s, phiQ, state, prefix, A_hat); break;
      default: hipLaunchKernelGGL(contract_bf16_kernel<0>, grid, block, 0, st, s, phiQ, state, prefix, A_hat); break;
    }
  }
  return hipGetLastError();
}

}  // namespace sea

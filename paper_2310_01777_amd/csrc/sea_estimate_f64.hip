// Random-feature estimate of the compressed attention matrix, fp32 tensors with fp64
// arithmetic (Sec. 3 "Performer (FAVOR+)", Sec. 3.1 "Attention Matrix Estimation").
//
//   phi(x)[i] = exp(w_i.x - |x|^2/2), x = sqrt(scale) q;  state = phi(K)^T V_I (K x m bucket
//   sums, V_I the nearest-neighbour stretched identity);  A_hat = rownorm(phi(Q) state), a
//   causal row using the inclusive prefix of its own bucket instead of the full bucket sum.
//
// This is the reference-precision mode: every dot product and the exponential are fp64 so
// that the per-row top-k^ taken on A_hat agrees with an fp64 evaluation except where two
// scores differ by less than ~1e-7 relative.  The projections and the contraction run on the
// matrix cores (v_mfma_f64_16x16x4_f64: lane l supplies A[row l % 16][k l / 16] and
// B[k l / 16][col l % 16], and receives D[row 4 i + l / 16][col l % 16] in register i); the
// contraction index is free to permute as long as both operands agree, which lets every lane read
// its sixteen operand values as contiguous floats.
//
// Workspace layout (doubles): phiQ [N][T][m], phiK/prefix [N][T][m], stateT [N][m][K].
#include "sea_internal.h"

namespace sea {
namespace {

typedef double doublex4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ doublex4 mfma_f64(double a, double b, doublex4 c) {
  return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
}

// exp(x) in fp64: x = k ln 2 + r, |r| <= 0.35, Taylor series to r^13 (error < 1e-17 relative)
__device__ __forceinline__ double exp_f64(double x) {
  const double k = rint(x * 1.4426950408889634074);
  double r = fma(-k, 6.93147180369123816490e-01, x);
  r = fma(-k, 1.90821492927058770002e-10, r);
  double p = 1.0 / 6227020800.0;
  p = fma(p, r, 1.0 / 479001600.0);
  p = fma(p, r, 1.0 / 39916800.0);
  p = fma(p, r, 1.0 / 3628800.0);
  p = fma(p, r, 1.0 / 362880.0);
  p = fma(p, r, 1.0 / 40320.0);
  p = fma(p, r, 1.0 / 5040.0);
  p = fma(p, r, 1.0 / 720.0);
  p = fma(p, r, 1.0 / 120.0);
  p = fma(p, r, 1.0 / 24.0);
  p = fma(p, r, 1.0 / 6.0);
  p = fma(p, r, 0.5);
  p = fma(p, r, 1.0);
  p = fma(p, r, 1.0);
  return ldexp(p, static_cast<int>(k));
}

// phi for 16 rows per wave.  which = 0: queries (row-max shifted, any shift cancels in the
// normaliser), 1: keys (no shift; zero beyond seq_len).  D[row = token 4 i + lg][col = feature lr];
// contraction slot (step s, lane group lg) stands for dimension 16 lg + s.
// NFT > 0: the exponent arguments of the (at most NFT) feature tiles stay in registers between the
// projection and the exponential, and the unrolled tile loop lets the loads of W run ahead;
// NFT = 0: any m, the arguments take a round trip through the output buffer.
// four consecutive elements of an fp32 tensor
__device__ __forceinline__ float4 load4(const float* p) { return *reinterpret_cast<const float4*>(p); }

template <int NFT, typename TI>
__global__ __launch_bounds__(256) void features_f64_kernel(Shape s, const TI* __restrict__ Q,
                                                           const TI* __restrict__ K, const TI* __restrict__ W,
                                                           double* __restrict__ phiQ, double* __restrict__ phiK) {
  const int wid = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int lr = lane & 15, lg = lane >> 4;
  const uint32_t tiles = (s.T + 15) / 16;
  const int64_t wave = static_cast<int64_t>(blockIdx.x) * 4 + wid;   // over 2 N tiles
  const int64_t nw = static_cast<int64_t>(s.N) * tiles;
  if (wave >= 2 * nw) return;
  const int which = wave >= nw;
  const int64_t wv = which ? wave - nw : wave;
  const int64_t head = wv / tiles;
  const int32_t r0 = static_cast<int32_t>(wv % tiles) * 16;
  const int32_t b = static_cast<int32_t>(head / s.H);
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
  const TI* X = (which ? K : Q) + (head * s.T + min(r0 + lr, s.T - 1)) * kHeadDim + 16 * lg;
  const double rs = sqrt(static_cast<double>(s.scale));
  double xa[16];
  double nx = 0.0;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const float4 v = load4(X + 4 * q);
    xa[4 * q] = rs * v.x; xa[4 * q + 1] = rs * v.y; xa[4 * q + 2] = rs * v.z; xa[4 * q + 3] = rs * v.w;
  }
#pragma unroll
  for (int e = 0; e < 16; ++e) nx = fma(xa[e], xa[e], nx);
  nx += __shfl_xor(nx, 16, kWave);
  nx += __shfl_xor(nx, 32, kWave);  // |x|^2 of token r0 + lr, in every lane group
  // this lane's four result rows are tokens r0 + 4 i + lg
  double half_n[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) half_n[i] = 0.5 * __shfl(nx, 4 * i + lg, kWave);
  double* out = (which ? phiK : phiQ) + (head * s.T) * s.m;
  double amax[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
  const int ntiles = s.m / 16;
  auto project = [&](int ft) {
    const TI* w = W + static_cast<int64_t>(ft * 16 + lr) * kHeadDim + 16 * lg;
    float4 wv[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) wv[q] = load4(w + 4 * q);
    doublex4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      acc = mfma_f64(xa[4 * q], static_cast<double>(wv[q].x), acc);
      acc = mfma_f64(xa[4 * q + 1], static_cast<double>(wv[q].y), acc);
      acc = mfma_f64(xa[4 * q + 2], static_cast<double>(wv[q].z), acc);
      acc = mfma_f64(xa[4 * q + 3], static_cast<double>(wv[q].w), acc);
    }
    return acc;
  };
  double shift[4];
  auto row_shift = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      double mx = amax[i];
#pragma unroll
      for (int mask = 1; mask < 16; mask <<= 1) mx = fmax(mx, __shfl_xor(mx, mask, kWave));
      shift[i] = which ? 0.0 : mx;
    }
  };
  if constexpr (NFT > 0) {
    double arg[NFT][4];
#pragma unroll
    for (int ft = 0; ft < NFT; ++ft) {
      if (ft < ntiles) {
        const doublex4 acc = project(ft);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          arg[ft][i] = acc[i] - half_n[i];
          amax[i] = fmax(amax[i], arg[ft][i]);
        }
      }
    }
    row_shift();
#pragma unroll
    for (int ft = 0; ft < NFT; ++ft) {
      if (ft < ntiles) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int32_t t = r0 + 4 * i + lg;
          if (t < s.T) out[static_cast<int64_t>(t) * s.m + ft * 16 + lr] = t < len ? exp_f64(arg[ft][i] - shift[i]) : 0.0;
        }
      }
    }
  } else {
    for (int ft = 0; ft < ntiles; ++ft) {
      const doublex4 acc = project(ft);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int32_t t = r0 + 4 * i + lg;
        const double a = acc[i] - half_n[i];
        amax[i] = fmax(amax[i], a);
        if (t < s.T) out[static_cast<int64_t>(t) * s.m + ft * 16 + lr] = a;  // exponent argument for now
      }
    }
    row_shift();
    // second pass over the lane's own values
    for (int ft = 0; ft < ntiles; ++ft) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int32_t t = r0 + 4 * i + lg;
        if (t >= s.T) continue;
        double* o = out + static_cast<int64_t>(t) * s.m + ft * 16 + lr;
        *o = t < len ? exp_f64(*o - shift[i]) : 0.0;
      }
    }
  }
}

// One thread per (head, column c, feature i): walk the keys of the column, turning phiK into
// its inclusive within-column prefix in place, and write the column sum to stateT[i][c].
__global__ __launch_bounds__(256) void state_f64_kernel(Shape s, double* __restrict__ phiK,
                                                        double* __restrict__ stateT) {
  const int64_t gid = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  const int64_t total = static_cast<int64_t>(s.N) * s.K * s.m;
  if (gid >= total) return;
  const int32_t i = static_cast<int32_t>(gid % s.m);
  const int32_t c = static_cast<int32_t>((gid / s.m) % s.K);
  const int64_t head = gid / (static_cast<int64_t>(s.m) * s.K);
  const int32_t j0 = block_start(c, s.T, s.K), j1 = block_start(c + 1, s.T, s.K);
  double* col = phiK + (head * s.T) * s.m + i;
  double acc = 0.0;
  for (int32_t j = j0; j < j1; ++j) {
    acc += col[static_cast<int64_t>(j) * s.m];
    col[static_cast<int64_t>(j) * s.m] = acc;
  }
  stateT[(head * s.m + i) * s.K + c] = acc;
}

// A_hat rows: one wave per 16 rows.  Tile (16 tokens x 16 columns) = phiQ x state over the m features
// (contraction slot (step s, lane group lg) = feature 4 s + lg); a causal row's own column is the
// diagonal of phiQ x prefix^T.  Column tiles are taken in groups of NCT that stay in registers; with
// one group (K <= 16 NCT) a single pass normalises and stores, with more the groups are computed
// twice: once for the row sums, once for the normalised output.
template <int NCT>
__global__ __launch_bounds__(256) void contract_f64_kernel(Shape s, const double* __restrict__ phiQ,
                                                           const double* __restrict__ pref,
                                                           const double* __restrict__ stateT,
                                                           float* __restrict__ A_hat) {
  const int wid = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int lr = lane & 15, lg = lane >> 4;
  const uint32_t tiles = (s.T + 15) / 16;
  const int64_t wave = static_cast<int64_t>(blockIdx.x) * 4 + wid;
  if (wave >= static_cast<int64_t>(s.N) * tiles) return;
  const int64_t head = wave / tiles;
  const int32_t r0 = static_cast<int32_t>(wave % tiles) * 16;
  const int32_t b = static_cast<int32_t>(head / s.H);
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
  const double* qrow = phiQ + (head * s.T + min(r0 + lr, s.T - 1)) * s.m + lg;   // A operand: token lr
  const double* prow = pref + (head * s.T + min(r0 + lr, s.T - 1)) * s.m + lg;   // B operand: token lr as column
  const double* st = stateT + head * static_cast<int64_t>(s.m) * s.K;
  // columns this wave needs: causal rows stop at the last row's own column
  const int32_t t_hi = min(r0 + 15, s.T - 1);
  const int32_t ncols = s.causal ? min(s.K, bucket_of(t_hi, s.T, s.K) + 1) : s.K;
  const int32_t ngroups = (ncols + 16 * NCT - 1) / (16 * NCT);

  // this lane's rows: tokens r0 + 4 i + lg
  double diag[4] = {0.0, 0.0, 0.0, 0.0}, rsum[4] = {0.0, 0.0, 0.0, 0.0}, inv[4];
  int32_t tcol[4];
  bool act[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int32_t t = r0 + 4 * i + lg;
    act[i] = t < len;
    tcol[i] = act[i] ? bucket_of(t, s.T, s.K) : -1;
  }
  // Operands are requested a block of contraction steps ahead of the products that use them (two
  // register sets in turn): with one wave per SIMD nothing else hides the memory latency.
  if (s.causal) {
    constexpr int DS = 8;  // steps per block; m is a multiple of 32 = 8 steps
    doublex4 dg = {0.0, 0.0, 0.0, 0.0};
    double qa[DS], pa[DS], qb[DS], pb[DS];
    auto ld = [&](int32_t f0, double (&q)[DS], double (&p)[DS]) {
#pragma unroll
      for (int e = 0; e < DS; ++e) { q[e] = qrow[f0 + 4 * e]; p[e] = prow[f0 + 4 * e]; }
    };
    auto mm = [&](const double (&q)[DS], const double (&p)[DS]) {
#pragma unroll
      for (int e = 0; e < DS; ++e) dg = mfma_f64(q[e], p[e], dg);
    };
    ld(0, qa, pa);
    for (int32_t f0 = 0; f0 < s.m; f0 += 8 * DS) {
      const bool more = f0 + 4 * DS < s.m;
      if (more) ld(f0 + 4 * DS, qb, pb);
      mm(qa, pa);
      if (more) {
        if (f0 + 8 * DS < s.m) ld(f0 + 8 * DS, qa, pa);
        mm(qb, pb);
      }
    }
    // the diagonal entry of token u sits in lane (lr = u, lg = u % 4), register u / 4
#pragma unroll
    for (int i = 0; i < 4; ++i) diag[i] = __shfl(dg[i], 16 * lg + 4 * i + lg, kWave);
  }
  doublex4 acc[NCT];
  auto group = [&](int32_t g) {
    const int32_t c0 = 16 * NCT * g;
    constexpr int FS = NCT >= 16 ? 2 : 4;  // contraction steps per block
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) acc[ct] = doublex4{0.0, 0.0, 0.0, 0.0};
    int32_t ccol[NCT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) ccol[ct] = min(c0 + 16 * ct + lr, s.K - 1);
    double aa[FS], ab[FS], ba[NCT][FS], bb[NCT][FS];
    auto ld = [&](int32_t f0, double (&qa)[FS], double (&bs)[NCT][FS]) {
#pragma unroll
      for (int e = 0; e < FS; ++e) {
        qa[e] = qrow[f0 + 4 * e];
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct)
          if (c0 + 16 * ct < ncols) bs[ct][e] = st[static_cast<int64_t>(f0 + 4 * e + lg) * s.K + ccol[ct]];
      }
    };
    auto mm = [&](const double (&qa)[FS], const double (&bs)[NCT][FS]) {
#pragma unroll
      for (int e = 0; e < FS; ++e)
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct)
          if (c0 + 16 * ct < ncols) acc[ct] = mfma_f64(qa[e], bs[ct][e], acc[ct]);
    };
    ld(0, aa, ba);
    for (int32_t f0 = 0; f0 < s.m; f0 += 8 * FS) {
      const bool more = f0 + 4 * FS < s.m;
      if (more) ld(f0 + 4 * FS, ab, bb);
      mm(aa, ba);
      if (more) {
        if (f0 + 8 * FS < s.m) ld(f0 + 8 * FS, aa, ba);
        mm(ab, bb);
      }
    }
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
      const int32_t c = c0 + 16 * ct + lr;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        double v = acc[ct][i];
        if (s.causal) {
          if (c == tcol[i]) v = diag[i];
          if (c > tcol[i]) v = 0.0;
        }
        if (!act[i] || c >= s.K || c0 + 16 * ct >= ncols) v = 0.0;
        acc[ct][i] = v;
      }
    }
  };
  auto add_sums = [&]() {
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
      for (int i = 0; i < 4; ++i) rsum[i] += acc[ct][i];
  };
  auto store = [&](int32_t g) {
    const int32_t c0 = 16 * NCT * g;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int32_t t = r0 + 4 * i + lg;
      if (t >= s.T) continue;
      float* out = A_hat + (head * s.T + t) * s.K;
#pragma unroll
      for (int ct = 0; ct < NCT; ++ct) {
        const int32_t c = c0 + 16 * ct + lr;
        if (c < s.K) out[c] = static_cast<float>(acc[ct][i] * inv[i]);
      }
    }
  };
  auto finish_sums = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      double r = rsum[i];
#pragma unroll
      for (int mask = 1; mask < 16; mask <<= 1) r += __shfl_xor(r, mask, kWave);
      inv[i] = r > 0.0 ? 1.0 / r : 0.0;
    }
  };
  const int32_t all_groups = (s.K + 16 * NCT - 1) / (16 * NCT);  // groups past ncols hold zeros only
  if (ngroups <= 1) {
    group(0);
    add_sums();
    finish_sums();
    store(0);
  } else {
    for (int32_t g = 0; g < ngroups; ++g) {
      group(g);
      add_sums();
    }
    finish_sums();
    for (int32_t g = 0; g < ngroups; ++g) {
      group(g);
      store(g);
    }
  }
  // columns past the wave's last one: zeros
  for (int32_t g = max(ngroups, 1); g < all_groups; ++g) {
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) acc[ct] = doublex4{0.0, 0.0, 0.0, 0.0};
    store(g);
  }
}

template <typename TI>
void launch_features_f64_t(const Shape& s, const TI* Q, const TI* K, const TI* W, double* phiQ, double* phiK,
                           hipStream_t st) {
  const int64_t waves = 2 * static_cast<int64_t>(s.N) * ((s.T + 15) / 16);
  const dim3 grid(static_cast<uint32_t>((waves + 3) / 4));
  if (s.m <= 128)
    hipLaunchKernelGGL((features_f64_kernel<8, TI>), grid, dim3(256), 0, st, s, Q, K, W, phiQ, phiK);
  else if (s.m <= 256)
    hipLaunchKernelGGL((features_f64_kernel<16, TI>), grid, dim3(256), 0, st, s, Q, K, W, phiQ, phiK);
  else
    hipLaunchKernelGGL((features_f64_kernel<0, TI>), grid, dim3(256), 0, st, s, Q, K, W, phiQ, phiK);
}

}  // namespace

// phi(Q) (row-shifted) and phi(K) (zero past seq_len) in fp64, [N][T][m] each
hipError_t launch_features_f64(const Shape& s, const float* Q, const float* K, const float* W, double* phiQ,
                               double* phiK, hipStream_t st) {
  if (s.m % 16 != 0) return hipErrorNotSupported;
  launch_features_f64_t(s, Q, K, W, phiQ, phiK, st);
  return hipGetLastError();
}

size_t estimate_f64_workspace(const Shape& s) {
  const size_t ntm = static_cast<size_t>(s.N) * s.T * s.m;
  const size_t nkm = static_cast<size_t>(s.N) * s.K * s.m;
  return (2 * ntm + nkm) * sizeof(double);
}

hipError_t launch_estimate_f64(const Shape& s, const float* Q, const float* K, const float* W,
                               float* A_hat, void* ws, hipStream_t st) {
  const size_t ntm = static_cast<size_t>(s.N) * s.T * s.m;
  double* phiQ = static_cast<double*>(ws);
  double* phiK = phiQ + ntm;
  double* stateT = phiK + ntm;
  {
    StageScope scope(SEA_STAGE_FEATURES, st);
    launch_features_f64_t(s, Q, K, W, phiQ, phiK, st);
  }
  {
    StageScope scope(SEA_STAGE_STATE, st);
    const int64_t total = static_cast<int64_t>(s.N) * s.K * s.m;
    hipLaunchKernelGGL(state_f64_kernel, dim3(static_cast<uint32_t>((total + 255) / 256)), dim3(256),
                       0, st, s, phiK, stateT);
  }
  {
    StageScope scope(SEA_STAGE_CONTRACT, st);
    const int64_t waves = static_cast<int64_t>(s.N) * ((s.T + 15) / 16);
    const dim3 grid(static_cast<uint32_t>((waves + 3) / 4));
    const int nct = (s.K + 15) / 16;
#define SEA_LAUNCH_CONTRACT(C) hipLaunchKernelGGL(contract_f64_kernel<C>, grid, dim3(256), 0, st, s, phiQ, phiK, stateT, A_hat)
    if (nct <= 2) SEA_LAUNCH_CONTRACT(2);
    else if (nct <= 4) SEA_LAUNCH_CONTRACT(4);
    else if (nct <= 8) SEA_LAUNCH_CONTRACT(8);
    else SEA_LAUNCH_CONTRACT(16);
#undef SEA_LAUNCH_CONTRACT
  }
  return hipGetLastError();
}

}  // namespace sea

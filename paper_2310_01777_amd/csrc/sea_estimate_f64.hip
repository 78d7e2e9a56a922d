// Random-feature estimate of the compressed attention matrix, fp32 tensors with fp64
// arithmetic (Sec. 3 "Performer (FAVOR+)", Sec. 3.1 "Attention Matrix Estimation").
//
//   phi(x)[i] = exp(w_i.x - |x|^2/2), x = sqrt(scale) q;  state = phi(K)^T V_I (K x m bucket
//   sums, V_I the nearest-neighbour stretched identity);  A_hat = rownorm(phi(Q) state), a
//   causal row using the inclusive prefix of its own bucket instead of the full bucket sum.
//
// This is the reference-precision mode: every dot product and the exponential are fp64 so
// that the per-row top-k^ taken on A_hat agrees with an fp64 evaluation except where two
// scores differ by less than ~1e-7 relative.  MI355X runs fp64 FMAs at half the fp32 vector
// rate, and this mode is used for the small fp32 configuration only.
//
// Workspace layout (doubles): phiQ [N][T][m], phiK/prefix [N][T][m], stateT [N][m][K].
#include "sea_internal.h"

namespace sea {
namespace {

constexpr int kRowsPerBlock = 4;  // one wave per row

// phi for one row per wave.  which = 0: queries (row-max shifted, any shift cancels in the
// normaliser), 1: keys (no shift; zero beyond seq_len).
__global__ __launch_bounds__(kRowsPerBlock* kWave) void features_f64_kernel(
    Shape s, const float* __restrict__ Q, const float* __restrict__ K, const float* __restrict__ W,
    double* __restrict__ phiQ, double* __restrict__ phiK) {
  __shared__ double xs[kRowsPerBlock][kHeadDim];
  const int wid = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t nrows = static_cast<int64_t>(s.N) * s.T;
  const int64_t gr = static_cast<int64_t>(blockIdx.x) * kRowsPerBlock + wid;  // over 2 * nrows
  if (gr >= 2 * nrows) return;
  const int which = gr >= nrows;
  const int64_t row = which ? gr - nrows : gr;
  const float* X = which ? K : Q;
  double* out = (which ? phiK : phiQ) + row * s.m;
  const int32_t t = static_cast<int32_t>(row % s.T);
  const int32_t b = static_cast<int32_t>((row / s.T) / s.H);
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
  if (t >= len) {
    for (int i = lane; i < s.m; i += kWave) out[i] = 0.0;
    return;
  }
  const double rs = sqrt(static_cast<double>(s.scale));
  const double xv = rs * static_cast<double>(X[row * kHeadDim + lane]);
  xs[wid][lane] = xv;
  double nx = xv * xv;
#pragma unroll
  for (int mask = 1; mask < kWave; mask <<= 1) nx += __shfl_xor(nx, mask, kWave);
  __builtin_amdgcn_wave_barrier();
  double amax = -INFINITY;
  for (int i = lane; i < s.m; i += kWave) {
    const float* w = W + static_cast<int64_t>(i) * kHeadDim;
    double dot = 0.0;
#pragma unroll 8
    for (int e = 0; e < kHeadDim; ++e) dot = fma(static_cast<double>(w[e]), xs[wid][e], dot);
    const double a = dot - 0.5 * nx;
    out[i] = a;  // exponent argument for now
    amax = fmax(amax, a);
  }
#pragma unroll
  for (int mask = 1; mask < kWave; mask <<= 1) amax = fmax(amax, __shfl_xor(amax, mask, kWave));
  const double shift = which ? 0.0 : amax;
  for (int i = lane; i < s.m; i += kWave) out[i] = exp(out[i] - shift);
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

// A_hat rows: 8 rows per block, 32 threads per row, thread owns columns lane32 + 32 q.
template <int CPT>  // columns per thread = ceil(K / 32)
__global__ __launch_bounds__(256) void contract_f64_kernel(Shape s, const double* __restrict__ phiQ,
                                                           const double* __restrict__ pref,
                                                           const double* __restrict__ stateT,
                                                           float* __restrict__ A_hat) {
  extern __shared__ double fq[];  // [8][m]
  const int r = threadIdx.x >> 5, l32 = threadIdx.x & 31;
  const int64_t nrows = static_cast<int64_t>(s.N) * s.T;
  const int64_t row0 = static_cast<int64_t>(blockIdx.x) * 8;
  for (int x = threadIdx.x; x < 8 * s.m; x += 256) {
    const int64_t rr = row0 + x / s.m;
    fq[x] = rr < nrows ? phiQ[rr * s.m + (x % s.m)] : 0.0;
  }
  __syncthreads();
  const int64_t row = row0 + r;
  if (row >= nrows) return;  // no barrier below
  const int64_t head = row / s.T;
  const int32_t t = static_cast<int32_t>(row % s.T);
  const int32_t b = static_cast<int32_t>(head / s.H);
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
  float* out = A_hat + row * s.K;
  if (t >= len) {
    for (int c = l32; c < s.K; c += 32) out[c] = 0.f;
    return;
  }
  const int32_t ct = bucket_of(t, s.T, s.K);
  const int32_t cfull = s.causal ? ct : s.K;  // columns [0, cfull) use the full bucket sum
  const double* st = stateT + head * s.m * s.K;
  const double* q = fq + r * s.m;
  double acc[CPT];
#pragma unroll
  for (int k = 0; k < CPT; ++k) acc[k] = 0.0;
  for (int i = 0; i < s.m; ++i) {
    const double qi = q[i];
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int c = l32 + 32 * k;
      if (c < cfull) acc[k] = fma(qi, st[static_cast<int64_t>(i) * s.K + c], acc[k]);
    }
  }
  if (s.causal) {
    // diagonal column: phi(q_t) . prefix_t, computed by the 32 threads of the row together
    const double* pf = pref + row * s.m;
    double dsum = 0.0;
    for (int i = l32; i < s.m; i += 32) dsum = fma(q[i], pf[i], dsum);
#pragma unroll
    for (int mask = 1; mask < 32; mask <<= 1) dsum += __shfl_xor(dsum, mask, kWave);
#pragma unroll
    for (int k = 0; k < CPT; ++k)
      if (l32 + 32 * k == ct) acc[k] = dsum;
  }
  double rsum = 0.0;
#pragma unroll
  for (int k = 0; k < CPT; ++k) rsum += acc[k];
#pragma unroll
  for (int mask = 1; mask < 32; mask <<= 1) rsum += __shfl_xor(rsum, mask, kWave);
  const double inv = rsum > 0.0 ? 1.0 / rsum : 0.0;
#pragma unroll
  for (int k = 0; k < CPT; ++k) {
    const int c = l32 + 32 * k;
    if (c < s.K) out[c] = static_cast<float>(acc[k] * inv);
  }
}

}  // namespace

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
  const int64_t nrows = static_cast<int64_t>(s.N) * s.T;
  {
    StageScope scope(SEA_STAGE_FEATURES, st);
    const uint32_t grid = static_cast<uint32_t>((2 * nrows + kRowsPerBlock - 1) / kRowsPerBlock);
    hipLaunchKernelGGL(features_f64_kernel, dim3(grid), dim3(kRowsPerBlock * kWave), 0, st, s, Q, K,
                       W, phiQ, phiK);
  }
  {
    StageScope scope(SEA_STAGE_STATE, st);
    const int64_t total = static_cast<int64_t>(s.N) * s.K * s.m;
    hipLaunchKernelGGL(state_f64_kernel, dim3(static_cast<uint32_t>((total + 255) / 256)), dim3(256),
                       0, st, s, phiK, stateT);
  }
  {
    StageScope scope(SEA_STAGE_CONTRACT, st);
    const uint32_t grid = static_cast<uint32_t>((nrows + 7) / 8);
    const size_t shm = 8 * static_cast<size_t>(s.m) * sizeof(double);
    const int cpt = (s.K + 31) / 32;
#define SEA_LAUNCH_CONTRACT(C)                                                                   \
  hipLaunchKernelGGL(contract_f64_kernel<C>, dim3(grid), dim3(256), shm, st, s, phiQ, phiK, stateT, \
                     A_hat)
    if (cpt <= 1) SEA_LAUNCH_CONTRACT(1);
    else if (cpt <= 2) SEA_LAUNCH_CONTRACT(2);
    else if (cpt <= 4) SEA_LAUNCH_CONTRACT(4);
    else if (cpt <= 8) SEA_LAUNCH_CONTRACT(8);
    else if (cpt <= 16) SEA_LAUNCH_CONTRACT(16);
    else SEA_LAUNCH_CONTRACT(32);
#undef SEA_LAUNCH_CONTRACT
  }
  return hipGetLastError();
}

}  // namespace sea

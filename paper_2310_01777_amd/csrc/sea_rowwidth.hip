// Estimate in the per-row width geometry (App. A.4, figure of the masking process: in causal
// attention every row of A^ and M^ is resized to its own width).  Row t spreads its K columns
// over its own t + 1 keys: column c holds the keys [b_c, b_{c+1}), b_c = ceil(c (t+1) / K), so
//   A^[t][c] = phi(q_t) . (P[b_{c+1}] - P[b_c]) / (phi(q_t) . P[t+1]),
// with P[j] = sum_{j' < j} phi(k_j') the running FAVOR+ key state (Sec. 3 "Performer (FAVOR+)",
// causal form).  No two rows share a column's key range, so the T x K contraction is not a
// matrix product: it is K + 1 gathered dot products of length m per row, bound by the cache
// bandwidth of the gathers (the prefix table of a head, (T+1) m elements, stays in its XCD's L2).
//
//   prefix_kernel<F, false>  per (head, chunk of keys): chunk totals of phi(k), fp64 running sum
//   chunk_base_kernel        per head: exclusive scan of the chunk totals (fp64)
//   prefix_kernel<F, true>   same walk again, started from the chunk base, writes P as F
//   rows_kernel<F, SLOTS>    one wavefront per row: phi(q_t), the K gathers, differences, row norm
// F = float for bf16 tensors, double for fp32 tensors.  Features are not rounded to bf16 here.
#include "sea_internal.h"

namespace sea {
namespace {

constexpr int kStage = 64;        // keys staged in LDS at a time
constexpr int kMaxChunks = 64;    // chunks per head
constexpr int kRowsPerWave = 4;
constexpr int kRowWaves = 4;

template <typename F>
struct In;
template <>
struct In<float> {
  using T = uint16_t;
  static __device__ __forceinline__ float get(const uint16_t* p, int64_t i) { return bf16_to_f32(p[i]); }
};
template <>
struct In<double> {
  using T = float;
  static __device__ __forceinline__ double get(const float* p, int64_t i) { return static_cast<double>(p[i]); }
};

__device__ __forceinline__ float exp_of(float x) { return exp2f(x * kLog2e); }
__device__ __forceinline__ double exp_of(double x) { return exp(x); }

__host__ __device__ __forceinline__ int32_t chunk_len(int32_t T) {
  const int32_t c = (T + kMaxChunks - 1) / kMaxChunks;
  return ((c + kStage - 1) / kStage) * kStage;
}

// block = m threads, thread i owns feature i; grid = heads x chunks
template <typename F, bool WRITE>
__global__ __launch_bounds__(256) void prefix_kernel(Shape s, const typename In<F>::T* __restrict__ Kt,
                                                     const typename In<F>::T* __restrict__ W,
                                                     double* __restrict__ ctot, const double* __restrict__ cbase,
                                                     F* __restrict__ P) {
  __shared__ F y[kStage][kHeadDim];
  __shared__ F half_norm[kStage];
  const int32_t i = threadIdx.x;  // < m
  const int32_t CH = chunk_len(s.T);
  const int32_t nch = (s.T + CH - 1) / CH;
  const int64_t head = blockIdx.x / nch;
  const int32_t chunk = blockIdx.x - static_cast<uint32_t>(head) * nch;
  const int32_t j0 = chunk * CH;
  const int32_t j1 = min(j0 + CH, s.T);
  const int32_t b = static_cast<int32_t>(head / s.H);
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
  const F rs = static_cast<F>(sqrtf(s.scale));
  F w[kHeadDim];
#pragma unroll
  for (int e = 0; e < kHeadDim; ++e) w[e] = In<F>::get(W, static_cast<int64_t>(i) * kHeadDim + e);
  const typename In<F>::T* Kh = Kt + head * s.T * kHeadDim;
  F* Ph = P + head * (static_cast<int64_t>(s.T) + 1) * s.m;
  double run = WRITE ? cbase[(head * nch + chunk) * s.m + i] : 0.0;
  if (WRITE && chunk == 0) Ph[i] = static_cast<F>(0);
  for (int32_t js = j0; js < j1; js += kStage) {
    const int32_t nk = min(kStage, j1 - js);
    __syncthreads();
    for (int32_t x = threadIdx.x; x < nk * kHeadDim; x += blockDim.x)
      y[x / kHeadDim][x % kHeadDim] = rs * In<F>::get(Kh, static_cast<int64_t>(js) * kHeadDim + x);
    __syncthreads();
    for (int32_t j = threadIdx.x; j < nk; j += blockDim.x) {
      F n = 0;
      for (int e = 0; e < kHeadDim; ++e) n += y[j][e] * y[j][e];
      half_norm[j] = static_cast<F>(0.5) * n;
    }
    __syncthreads();
    for (int32_t j = 0; j < nk; ++j) {
      F dot = 0;
#pragma unroll
      for (int e = 0; e < kHeadDim; ++e) dot += w[e] * y[j][e];
      const F f = (js + j < len) ? exp_of(dot - half_norm[j]) : static_cast<F>(0);
      run += static_cast<double>(f);
      if (WRITE) Ph[static_cast<int64_t>(js + j + 1) * s.m + i] = static_cast<F>(run);
    }
  }
  if (!WRITE) ctot[(head * nch + chunk) * s.m + i] = run;
}

// block = m threads, grid = heads: cbase[chunk] = sum of the totals of the chunks before it
__global__ __launch_bounds__(256) void chunk_base_kernel(const double* __restrict__ ctot, double* __restrict__ cbase,
                                                         int32_t nch, int32_t m) {
  const int64_t head = blockIdx.x;
  double base = 0.0;
  for (int32_t c = 0; c < nch; ++c) {
    const int64_t at = (head * nch + c) * m + threadIdx.x;
    cbase[at] = base;
    base += ctot[at];
  }
}

template <typename F>
__device__ __forceinline__ F wave_sum(F v) {
#pragma unroll
  for (int mask = 1; mask < kWave; mask <<= 1) v += __shfl_xor(v, mask, kWave);
  return v;
}
template <typename F>
__device__ __forceinline__ F wave_max(F v) {
#pragma unroll
  for (int mask = 1; mask < kWave; mask <<= 1) v = max(v, __shfl_xor(v, mask, kWave));
  return v;
}

// MU = m / 64 feature slots per lane (feature = u 64 + lane), SLOTS = ceil(K / 64) column slots
// per lane (column = q 64 + lane).  W^T sits in LDS as floats (exact for bf16 and fp32 weights),
// [e][i] so that a wavefront reads consecutive words.
template <typename F, int MU, int SLOTS>
__global__ __launch_bounds__(kRowWaves* kWave) void rows_kernel(Shape s, const typename In<F>::T* __restrict__ Q,
                                                                const typename In<F>::T* __restrict__ W,
                                                                const F* __restrict__ P, float* __restrict__ A_hat) {
  extern __shared__ float wt[];  // [64][m]
  for (int32_t x = threadIdx.x; x < s.m * kHeadDim; x += blockDim.x) {
    const int32_t i = x / kHeadDim, e = x % kHeadDim;
    wt[e * s.m + i] = static_cast<float>(In<F>::get(W, x));
  }
  __syncthreads();
  const int lane = threadIdx.x & 63;
  const int64_t nrows = static_cast<int64_t>(s.N) * s.T;
  const uint32_t lb = xcd_contiguous(blockIdx.x, gridDim.x);
  const int64_t first = (static_cast<int64_t>(lb) * kRowWaves + (threadIdx.x >> 6)) * kRowsPerWave;
  const F rs = static_cast<F>(sqrtf(s.scale));
  for (int rr = 0; rr < kRowsPerWave; ++rr) {
    const int64_t row = first + rr;
    if (row >= nrows) return;  // no block-wide barrier below
    const int64_t head = row / s.T;
    const int32_t t = static_cast<int32_t>(row - head * s.T);
    const int32_t b = static_cast<int32_t>(head / s.H);
    const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
    float* Arow = A_hat + row * s.K;
    if (t >= len) {
      for (int32_t c = lane; c < s.K; c += kWave) Arow[c] = 0.f;
      continue;
    }
    // phi(q_t) up to a row factor (|x|^2 / 2 and the largest exponent cancel in the row norm):
    // lane e holds x[e]; feature u 64 + lane in slot u
    const F xe = rs * In<F>::get(Q, row * kHeadDim + lane);
    F arg[MU];
#pragma unroll
    for (int u = 0; u < MU; ++u) arg[u] = 0;
#pragma unroll
    for (int e = 0; e < kHeadDim; ++e) {
      const F x = __shfl(xe, e, kWave);
#pragma unroll
      for (int u = 0; u < MU; ++u) arg[u] += static_cast<F>(wt[e * s.m + u * kWave + lane]) * x;
    }
    F top = arg[0];
#pragma unroll
    for (int u = 1; u < MU; ++u) top = max(top, arg[u]);
    top = wave_max(top);
    F phi[MU];
#pragma unroll
    for (int u = 0; u < MU; ++u) phi[u] = exp_of(arg[u] - top);  // the row factor cancels in the norm

    // G_c = phi . P[b_c] for c = 1..K (G_0 = 0); column c - 1 lives in lane (c-1) % 64, slot (c-1) / 64
    const F* Ph = P + head * (static_cast<int64_t>(s.T) + 1) * s.m;
    const int64_t width = static_cast<int64_t>(t) + 1;
    F g[SLOTS];
#pragma unroll
    for (int q = 0; q < SLOTS; ++q) g[q] = 0;
#pragma unroll
    for (int q = 0; q < SLOTS; ++q) {
      const int32_t cn = min(kWave, s.K - q * kWave);  // columns of this slot (uniform)
      for (int32_t l0 = 0; l0 < cn; l0 += 4) {
        F part[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int32_t c = min(q * kWave + l0 + v + 1, s.K);
          const int64_t bc = (c * width + s.K - 1) / s.K;  // <= t + 1
          const F* pv = Ph + bc * s.m + lane;
          F acc = 0;
#pragma unroll
          for (int u = 0; u < MU; ++u) acc += phi[u] * pv[u * kWave];
          part[v] = acc;
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const F sum = wave_sum(part[v]);
          if (lane == l0 + v) g[q] = sum;
        }
      }
    }
    // differences and the row normaliser G_K
    const int32_t qk = (s.K - 1) / kWave, lk = (s.K - 1) % kWave;
    F total = 0;
#pragma unroll
    for (int q = 0; q < SLOTS; ++q)
      if (q == qk) total = __shfl(g[q], lk, kWave);
    const F inv = total > static_cast<F>(0) ? static_cast<F>(1) / total : static_cast<F>(0);
    F carry = 0;  // G of the column before this slot's first
#pragma unroll
    for (int q = 0; q < SLOTS; ++q) {
      F prev = __shfl_up(g[q], 1, kWave);
      if (lane == 0) prev = carry;
      const int32_t c = q * kWave + lane;
      if (c < s.K) Arow[c] = static_cast<float>((g[q] - prev) * inv);
      carry = __shfl(g[q], kWave - 1, kWave);
    }
  }
}

struct Layout {
  size_t ctot, cbase, P, total;
  int32_t nch;
};
Layout layout(const Shape& s, sea_dtype dt) {
  Layout l{};
  const int32_t CH = chunk_len(s.T);
  l.nch = (s.T + CH - 1) / CH;
  const size_t tab = (static_cast<size_t>(s.N) * l.nch * s.m * sizeof(double) + 255) & ~size_t(255);
  l.ctot = 0;
  l.cbase = tab;
  l.P = 2 * tab;
  const size_t el = dt == SEA_BF16 ? sizeof(float) : sizeof(double);
  l.total = l.P + ((static_cast<size_t>(s.N) * (static_cast<size_t>(s.T) + 1) * s.m * el + 255) & ~size_t(255));
  return l;
}

template <typename F, int MU>
hipError_t launch_rows(const Shape& s, const typename In<F>::T* Q, const typename In<F>::T* W, const F* P,
                       float* A_hat, hipStream_t st) {
  const int64_t nrows = static_cast<int64_t>(s.N) * s.T;
  const int64_t per_block = kRowWaves * kRowsPerWave;
  const dim3 grid(static_cast<uint32_t>((nrows + per_block - 1) / per_block));
  const size_t lds = static_cast<size_t>(s.m) * kHeadDim * sizeof(float);
  const int slots = (s.K + kWave - 1) / kWave;
#define SEA_RW_ROWS(SL)                                                                                      \
  hipLaunchKernelGGL((rows_kernel<F, MU, SL>), grid, dim3(kRowWaves* kWave), lds, st, s, Q, W, P, A_hat)
  if (slots <= 1) SEA_RW_ROWS(1);
  else if (slots <= 2) SEA_RW_ROWS(2);
  else if (slots <= 4) SEA_RW_ROWS(4);
  else if (slots <= 8) SEA_RW_ROWS(8);
  else SEA_RW_ROWS(16);
#undef SEA_RW_ROWS
  return hipGetLastError();
}

template <typename F>
hipError_t launch_all(const Shape& s, sea_dtype dt, const void* Qv, const void* Kv, const void* Wv, float* A_hat,
                      void* ws, hipStream_t st) {
  using T = typename In<F>::T;
  const T* Q = static_cast<const T*>(Qv);
  const T* K = static_cast<const T*>(Kv);
  const T* W = static_cast<const T*>(Wv);
  const Layout l = layout(s, dt);
  char* base = static_cast<char*>(ws);
  double* ctot = reinterpret_cast<double*>(base + l.ctot);
  double* cbase = reinterpret_cast<double*>(base + l.cbase);
  F* P = reinterpret_cast<F*>(base + l.P);
  const dim3 pgrid(static_cast<uint32_t>(s.N) * l.nch);
  {
    StageScope scope(SEA_STAGE_STATE, st);
    hipLaunchKernelGGL((prefix_kernel<F, false>), pgrid, dim3(s.m), 0, st, s, K, W, ctot, cbase, P);
    hipLaunchKernelGGL(chunk_base_kernel, dim3(s.N), dim3(s.m), 0, st, ctot, cbase, l.nch, s.m);
    hipLaunchKernelGGL((prefix_kernel<F, true>), pgrid, dim3(s.m), 0, st, s, K, W, ctot, cbase, P);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  StageScope scope(SEA_STAGE_CONTRACT, st);
  switch (s.m / kWave) {
    case 1: return launch_rows<F, 1>(s, Q, W, P, A_hat, st);
    case 2: return launch_rows<F, 2>(s, Q, W, P, A_hat, st);
    default: return launch_rows<F, 4>(s, Q, W, P, A_hat, st);
  }
}

}  // namespace

bool estimate_rowwidth_supported(const Shape& s) { return s.causal && (s.m == 64 || s.m == 128 || s.m == 256); }

size_t estimate_rowwidth_workspace(const Shape& s, sea_dtype dt) { return layout(s, dt).total; }

hipError_t launch_estimate_rowwidth(const Shape& s, sea_dtype dt, const void* Q, const void* K, const void* W,
                                    float* A_hat, void* ws, hipStream_t st) {
  return dt == SEA_BF16 ? launch_all<float>(s, dt, Q, K, W, A_hat, ws, st)
                        : launch_all<double>(s, dt, Q, K, W, A_hat, ws, st);
}

}  // namespace sea

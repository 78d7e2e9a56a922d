// Output mixing (Sec. 3.1.1 "Output Calculation"):
//   C_sea[t] = s_mix[t] * s_prob[t] * C[t] + (1 - s_mix[t]) * C_avg[t]
// Bidirectional: C_avg is one vector per head, the average of the active value rows weighted by
// the importance i_j = i^[floor(j K / T)], i^ = mean over the active rows of A_hat.
// Causal: C_avg[t] = mean of v_0 .. v_t (running mean), computed as a chunked prefix sum.
// s_prob and s_mix are learned in the paper; here they are caller-supplied device vectors.
#include "sea_internal.h"

namespace sea {
namespace {

constexpr int kChunkRows = 256;

template <typename T>
__device__ __forceinline__ float ld(const T* p);
template <>
__device__ __forceinline__ float ld<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float ld<uint16_t>(const uint16_t* p) { return bf16_to_f32(*p); }
template <typename T>
__device__ __forceinline__ void st(T* p, float v);
template <>
__device__ __forceinline__ void st<float>(float* p, float v) { *p = v; }
template <>
__device__ __forceinline__ void st<uint16_t>(uint16_t* p, float v) { *p = f32_to_bf16(v); }

// ---- causal pass 1: per (head, 256-row chunk) column sums of V -> part[N][chunks][64] ----
template <typename T>
__global__ __launch_bounds__(256) void chunk_sums_kernel(Shape s, const T* __restrict__ V,
                                                         double* __restrict__ part) {
  __shared__ double red[4][kHeadDim];
  const int d = threadIdx.x & 63, q = threadIdx.x >> 6;
  const uint32_t chunks = (s.T + kChunkRows - 1) / kChunkRows;
  const int64_t head = blockIdx.x / chunks;
  const int32_t r0 = static_cast<int32_t>(blockIdx.x % chunks) * kChunkRows + q * 64;
  const int32_t b = static_cast<int32_t>(head / s.H);
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
  double acc = 0.0;
  for (int32_t t = r0; t < min(r0 + 64, len); ++t) acc += ld<T>(V + (head * s.T + t) * kHeadDim + d);
  red[q][d] = acc;
  __syncthreads();
  if (q == 0) part[static_cast<int64_t>(blockIdx.x) * kHeadDim + d] = red[0][d] + red[1][d] + red[2][d] + red[3][d];
}

// ---- causal pass 2: offset = sum of earlier chunks, in-chunk running sums, mix ----
template <typename T>
__global__ __launch_bounds__(256) void mix_causal_kernel(Shape s, const T* __restrict__ C,
                                                         const T* __restrict__ V,
                                                         const double* __restrict__ part,
                                                         const float* __restrict__ s_prob,
                                                         const float* __restrict__ s_mix, T* __restrict__ O) {
  __shared__ double qsum[4][kHeadDim];
  const int d = threadIdx.x & 63, q = threadIdx.x >> 6;
  const uint32_t chunks = (s.T + kChunkRows - 1) / kChunkRows;
  const int64_t head = blockIdx.x / chunks;
  const uint32_t chunk = blockIdx.x % chunks;
  const int32_t r0 = static_cast<int32_t>(chunk) * kChunkRows + q * 64;
  const int32_t b = static_cast<int32_t>(head / s.H);
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
  double off = 0.0;
  for (uint32_t c = 0; c < chunk; ++c) off += part[(head * chunks + c) * kHeadDim + d];
  // sums of this thread's 64 rows, then the offsets of the four quarters
  double mine = 0.0;
  for (int32_t t = r0; t < min(r0 + 64, len); ++t) mine += ld<T>(V + (head * s.T + t) * kHeadDim + d);
  qsum[q][d] = mine;
  __syncthreads();
  for (int x = 0; x < q; ++x) off += qsum[x][d];
  double run = off;
  for (int32_t t = r0; t < min(r0 + 64, s.T); ++t) {
    const int64_t e = (head * s.T + t) * kHeadDim + d;
    if (t >= len) {
      st<T>(O + e, 0.f);
      continue;
    }
    run += ld<T>(V + e);
    const float sm = s_mix[head * s.T + t], sp = s_prob ? s_prob[head * s.T + t] : 1.f;
    const double avg = run / static_cast<double>(t + 1);
    st<T>(O + e, static_cast<float>(static_cast<double>(sm) * sp * ld<T>(C + e) + (1.0 - sm) * avg));
  }
}

// ---- bidirectional pass 1: one block per head: importance and the pooled vector ----
template <typename T>
__global__ __launch_bounds__(256) void pool_kernel(Shape s, const T* __restrict__ V,
                                                   const float* __restrict__ A_hat,
                                                   float* __restrict__ pooled) {
  extern __shared__ double sh[];  // ihat[K], then red[4][65]
  double* ihat = sh;
  double* red = sh + s.K;
  const int64_t head = blockIdx.x;
  const int32_t b = static_cast<int32_t>(head / s.H);
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
  for (int32_t c = threadIdx.x; c < s.K; c += 256) {
    double acc = 0.0;
    for (int32_t t = 0; t < len; ++t) acc += A_hat[(head * s.T + t) * s.K + c];
    ihat[c] = len > 0 ? acc / len : 0.0;
  }
  __syncthreads();
  const int d = threadIdx.x & 63, q = threadIdx.x >> 6;
  double acc = 0.0, wsum = 0.0;
  for (int32_t j = q; j < len; j += 4) {
    const double wj = ihat[bucket_of(j, s.T, s.K)];
    wsum += wj;
    acc += wj * ld<T>(V + (head * s.T + j) * kHeadDim + d);
  }
  red[q * 65 + d] = acc;
  if (d == 0) red[q * 65 + 64] = wsum;
  __syncthreads();
  if (q == 0) {
    const double a = red[d] + red[65 + d] + red[130 + d] + red[195 + d];
    const double w = red[64] + red[65 + 64] + red[130 + 64] + red[195 + 64];
    pooled[head * kHeadDim + d] = w > 0.0 ? static_cast<float>(a / w) : 0.f;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void mix_pooled_kernel(Shape s, const T* __restrict__ C,
                                                         const float* __restrict__ pooled,
                                                         const float* __restrict__ s_prob,
                                                         const float* __restrict__ s_mix, T* __restrict__ O) {
  const int64_t gid = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  const int64_t total = static_cast<int64_t>(s.N) * s.T * kHeadDim;
  if (gid >= total) return;
  const int d = static_cast<int>(gid & 63);
  const int64_t row = gid >> 6;
  const int64_t head = row / s.T;
  const int32_t t = static_cast<int32_t>(row % s.T);
  const int32_t b = static_cast<int32_t>(head / s.H);
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
  if (t >= len) {
    st<T>(O + gid, 0.f);
    return;
  }
  const float sm = s_mix[row], sp = s_prob ? s_prob[row] : 1.f;
  st<T>(O + gid, sm * sp * ld<T>(C + gid) + (1.f - sm) * pooled[head * kHeadDim + d]);
}

template <typename T>
hipError_t run(const Shape& s, const T* C, const T* V, const float* A_hat, const float* s_prob,
               const float* s_mix, T* O, void* ws, hipStream_t st_) {
  if (s.causal) {
    const uint32_t chunks = (s.T + kChunkRows - 1) / kChunkRows;
    const dim3 grid(static_cast<uint32_t>(s.N) * chunks);
    double* part = static_cast<double*>(ws);
    hipLaunchKernelGGL(chunk_sums_kernel<T>, grid, dim3(256), 0, st_, s, V, part);
    hipLaunchKernelGGL(mix_causal_kernel<T>, grid, dim3(256), 0, st_, s, C, V, part, s_prob, s_mix, O);
  } else {
    float* pooled = static_cast<float*>(ws);
    const size_t shm = (static_cast<size_t>(s.K) + 4 * 65) * sizeof(double);
    hipLaunchKernelGGL(pool_kernel<T>, dim3(s.N), dim3(256), shm, st_, s, V, A_hat, pooled);
    const int64_t total = static_cast<int64_t>(s.N) * s.T * kHeadDim;
    hipLaunchKernelGGL(mix_pooled_kernel<T>, dim3(static_cast<uint32_t>((total + 255) / 256)), dim3(256), 0,
                       st_, s, C, pooled, s_prob, s_mix, O);
  }
  return hipGetLastError();
}

}  // namespace

size_t output_mix_workspace(const Shape& s) {
  const size_t chunks = (static_cast<size_t>(s.T) + kChunkRows - 1) / kChunkRows;
  const size_t bytes = s.causal ? static_cast<size_t>(s.N) * chunks * kHeadDim * sizeof(double)
                                : static_cast<size_t>(s.N) * kHeadDim * sizeof(float);
  return (bytes + 255) & ~size_t(255);
}

hipError_t launch_output_mix(const Shape& s, sea_dtype dt, const void* C, const void* V,
                             const float* A_hat, const float* s_prob, const float* s_mix, void* O,
                             void* ws, hipStream_t st_) {
  if (dt == SEA_BF16)
    return run<uint16_t>(s, static_cast<const uint16_t*>(C), static_cast<const uint16_t*>(V), A_hat, s_prob,
                         s_mix, static_cast<uint16_t*>(O), ws, st_);
  return run<float>(s, static_cast<const float*>(C), static_cast<const float*>(V), A_hat, s_prob, s_mix,
                    static_cast<float*>(O), ws, st_);
}

}  // namespace sea

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

// eight consecutive elements of a row <-> eight floats
__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
  const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void load8(const uint16_t* p, float (&v)[8]) {
  const uint4 u = *reinterpret_cast<const uint4*>(p);
  const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) { v[2 * i] = bf16lo_to_f32(w[i]); v[2 * i + 1] = bf16hi_to_f32(w[i]); }
}
__device__ __forceinline__ void store8(float* p, const float (&v)[8]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ __forceinline__ void store8(uint16_t* p, const float (&v)[8]) {
  uint4 u;
  u.x = pack_bf16(v[0], v[1]); u.y = pack_bf16(v[2], v[3]);
  u.z = pack_bf16(v[4], v[5]); u.w = pack_bf16(v[6], v[7]);
  *reinterpret_cast<uint4*>(p) = u;
}

// Causal mixing works on chunks of 256 rows.  A thread owns 8 consecutive rows x 8 dimensions
// (slot = tid / 8, dimension group = tid % 8), so every load is 16 or 32 bytes and the 8 lanes of
// a row cover it whole; the eight row loads of a thread are independent.

// ---- causal pass 1: per (head, 256-row chunk) column sums of V -> part[N][chunks][64] ----
template <typename T>
__global__ __launch_bounds__(256) void chunk_sums_kernel(Shape s, const T* __restrict__ V,
                                                         double* __restrict__ part) {
  __shared__ float red[32][kHeadDim + 1];
  const int slot = threadIdx.x >> 3, dg = threadIdx.x & 7;
  const uint32_t chunks = (s.T + kChunkRows - 1) / kChunkRows;
  const int64_t head = blockIdx.x / chunks;
  const int32_t r0 = static_cast<int32_t>(blockIdx.x % chunks) * kChunkRows + slot * 8;
  const int32_t b = static_cast<int32_t>(head / s.H);
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  // All eight rows are requested before the first is added: a row past the sequence reads the last
  // row of the head instead and is not added, so no load sits behind a branch.
  float v[8][8];
#pragma unroll
  for (int r = 0; r < 8; ++r) load8(V + (head * s.T + min(r0 + r, s.T - 1)) * kHeadDim + dg * 8, v[r]);
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const bool keep = r0 + r < len;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] += keep ? v[r][i] : 0.f;
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) red[slot][dg * 8 + i] = acc[i];
  __syncthreads();
  if (threadIdx.x < kHeadDim) {
    double tot = 0.0;
    for (int q = 0; q < 32; ++q) tot += red[q][threadIdx.x];
    part[static_cast<int64_t>(blockIdx.x) * kHeadDim + threadIdx.x] = tot;
  }
}

// ---- causal pass 2: offset = sum of earlier chunks, in-chunk running sums, mix ----
template <typename T>
__global__ __launch_bounds__(256) void mix_causal_kernel(Shape s, const T* __restrict__ C,
                                                         const T* __restrict__ V,
                                                         const double* __restrict__ part,
                                                         const float* __restrict__ s_prob,
                                                         const float* __restrict__ s_mix, T* __restrict__ O) {
  __shared__ float red[32][kHeadDim + 1];
  __shared__ double offs[33][kHeadDim];  // exclusive prefix of the 32 slots (row 32: unused total)
  __shared__ double before[4][kHeadDim];  // partial sums over the head's earlier chunks
  const int slot = threadIdx.x >> 3, dg = threadIdx.x & 7;
  const uint32_t chunks = (s.T + kChunkRows - 1) / kChunkRows;
  const int64_t head = blockIdx.x / chunks;
  const uint32_t chunk = blockIdx.x % chunks;
  const int32_t r0 = static_cast<int32_t>(chunk) * kChunkRows + slot * 8;
  const int32_t b = static_cast<int32_t>(head / s.H);
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
  // the thread's 8 rows x 8 dimensions of V, kept for the second sweep
  float v[8][8];
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  // all eight rows requested before the first is used (rows past the sequence read the head's last
  // row and are cleared afterwards)
#pragma unroll
  for (int r = 0; r < 8; ++r) load8(V + (head * s.T + min(r0 + r, s.T - 1)) * kHeadDim + dg * 8, v[r]);
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    if (r0 + r >= len) {
#pragma unroll
      for (int i = 0; i < 8; ++i) v[r][i] = 0.f;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] += v[r][i];
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) red[slot][dg * 8 + i] = acc[i];
  {
    // sum of the earlier chunks of the head: the block's four waves take every fourth chunk each,
    // two sums in flight per thread, so that the loads of a long sequence do not queue behind one another
    const int d = threadIdx.x & 63, pt = threadIdx.x >> 6;
    const double* ph = part + head * chunks * kHeadDim + d;
    double a0 = 0.0, a1 = 0.0;
    uint32_t c = static_cast<uint32_t>(pt);
    for (; c + 4 < chunk; c += 8) {
      a0 += ph[static_cast<size_t>(c) * kHeadDim];
      a1 += ph[static_cast<size_t>(c + 4) * kHeadDim];
    }
    if (c < chunk) a0 += ph[static_cast<size_t>(c) * kHeadDim];
    before[pt][d] = a0 + a1;
  }
  __syncthreads();
  if (threadIdx.x < kHeadDim) {
    const int d = threadIdx.x;
    double run = (before[0][d] + before[1][d]) + (before[2][d] + before[3][d]);
    for (int q = 0; q < 32; ++q) {
      offs[q][d] = run;
      run += red[q][d];
    }
  }
  __syncthreads();
  double run[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) run[i] = offs[slot][dg * 8 + i];
  // four rows at a time: their C rows and scalers are requested together (clamped to the head's
  // last row where the chunk overruns it), then mixed and stored
#pragma unroll
  for (int r4 = 0; r4 < 8; r4 += 4) {
    float c[4][8], sm[4], sp[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int64_t rowc = head * s.T + min(r0 + r4 + r, s.T - 1);
      load8(C + rowc * kHeadDim + dg * 8, c[r]);
      sm[r] = s_mix[rowc];
      sp[r] = s_prob ? s_prob[rowc] : 1.f;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int32_t t = r0 + r4 + r;
      if (t < s.T) {
        const int64_t e = (head * s.T + t) * kHeadDim + dg * 8;
        float o[8];
        const bool live = t < len;
        const double inv = 1.0 / static_cast<double>(t + 1);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          run[i] += v[r4 + r][i];
          const float x = static_cast<float>(static_cast<double>(sm[r]) * sp[r] * c[r][i] + (1.0 - sm[r]) * (run[i] * inv));
          o[i] = live ? x : 0.f;
        }
        store8(O + e, o);
      }
    }
  }
}

// ---- bidirectional pass 1: one block per head: importance and the pooled vector ----
template <typename T>
__global__ __launch_bounds__(256) void pool_kernel(Shape s, const T* __restrict__ V,
                                                   const float* __restrict__ A_hat,
                                                   float* __restrict__ pooled) {
  extern __shared__ double sh[];  // ihat[K], then red[4][65], then part[256]
  double* ihat = sh;
  double* red = sh + s.K;
  double* part = red + 4 * 65;
  const int64_t head = blockIdx.x;
  const int32_t b = static_cast<int32_t>(head / s.H);
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
  // column means over the active rows: with K < 256 the block splits the rows into 256 / K parts
  // (thread = (part, column)), each thread keeps four sums going, the parts meet in LDS
  const int32_t P = s.K < 256 ? 256 / s.K : 1;
  for (int32_t c0 = 0; c0 < s.K; c0 += 256) {
    const int32_t c = c0 + static_cast<int32_t>(threadIdx.x) % min(s.K, 256);
    const int32_t pt = static_cast<int32_t>(threadIdx.x) / min(s.K, 256);
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    if (pt < P && c < s.K) {
      const float* col = A_hat + head * s.T * s.K + c;
      int32_t t = pt;
      for (; t + 3 * P < len; t += 4 * P) {
        a0 += col[static_cast<int64_t>(t) * s.K];
        a1 += col[static_cast<int64_t>(t + P) * s.K];
        a2 += col[static_cast<int64_t>(t + 2 * P) * s.K];
        a3 += col[static_cast<int64_t>(t + 3 * P) * s.K];
      }
      for (; t < len; t += P) a0 += col[static_cast<int64_t>(t) * s.K];
    }
    part[threadIdx.x] = (a0 + a1) + (a2 + a3);
    __syncthreads();
    if (pt == 0 && c < s.K) {
      double acc = 0.0;
      for (int32_t q = 0; q < P; ++q) acc += part[q * min(s.K, 256) + static_cast<int32_t>(threadIdx.x)];
      ihat[c] = len > 0 ? acc / len : 0.0;
    }
    __syncthreads();
  }
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
    const size_t shm = (static_cast<size_t>(s.K) + 4 * 65 + 256) * sizeof(double);
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

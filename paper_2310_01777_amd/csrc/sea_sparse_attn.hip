// Sparse attention over per-row key lists (Sec. 3.1.1: rho, sigma, A* V fused).
//
// One wavefront owns one query row.  A key (or value) row of d = 64 elements is 128 B in
// bf16 (8 lanes x 16 B) or 256 B in fp32 (16 lanes x 16 B), so one 128-bit load per lane
// fetches 8 (bf16) or 4 (fp32) gathered rows per wave instruction, each row contiguous
// across its lane group.  The softmax is the streaming (running max / running sum) form held
// in registers; nothing of size T x T or T x L is ever written.
#include "sea_internal.h"

namespace sea {
namespace {

constexpr int kWavesPerBlock = 4;
constexpr int kUnroll = 4;

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16x2 as_bf16x2(uint32_t w) {
  bf16x2 h;
  __builtin_memcpy(&h, &w, sizeof(h));
  return h;
}
__device__ __forceinline__ float wave_xor_f(float v, int mask) { return __shfl_xor(v, mask, kWave); }
__device__ __forceinline__ double wave_xor_d(double v, int mask) { return __shfl_xor(v, mask, kWave); }

// Where a row's key list lives.  Per-row lists: idx + row L, cnt[row] entries.  FlatCSR tensor
// (crow != nullptr, idx = its column array): row (b, h, t) owns the entries of CSR row b T + t
// whose column h' T + j has h' = h -- one contiguous run because columns ascend -- found by two
// binary searches; the key is the entry minus h T.
struct KeyList {
  const int32_t* p;
  int32_t n;
  int32_t base;
};
__device__ __forceinline__ KeyList key_list(const Shape& s, int64_t row, const int32_t* __restrict__ idx,
                                            const int32_t* __restrict__ cnt, int32_t L,
                                            const int64_t* __restrict__ crow) {
  if (crow == nullptr) return {idx + row * L, min(cnt[row], L), 0};
  const int64_t head = row / s.T, t = row - head * s.T;
  const int64_t b = head / s.H, h = head - b * s.H;
  const int64_t beg = crow[b * s.T + t], end = crow[b * s.T + t + 1];
  int64_t bound[2];
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    const int64_t key = (h + e) * s.T;
    int64_t a = beg, z = end;
    while (a < z) {
      const int64_t mid = (a + z) >> 1;
      if (idx[mid] < key) a = mid + 1; else z = mid;
    }
    bound[e] = a;
  }
  return {idx + bound[0], static_cast<int32_t>(bound[1] - bound[0]), static_cast<int32_t>(h * s.T)};
}

// ------------------------------------------------------------------------------------------
// bf16: 8 lanes per row, 8 rows per wave load, fp32 logits (log2 domain) and accumulators
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kWavesPerBlock* kWave) void sparse_attn_bf16_kernel(
    Shape s, const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K,
    const uint16_t* __restrict__ V, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ cnt, int32_t L, const int64_t* __restrict__ crow,
    uint16_t* __restrict__ O) {
  const uint32_t lb = xcd_contiguous(blockIdx.x, gridDim.x);
  const int64_t row = static_cast<int64_t>(lb) * kWavesPerBlock + (threadIdx.x >> 6);
  const int64_t nrows = static_cast<int64_t>(s.N) * s.T;
  if (row >= nrows) return;
  const int lane = threadIdx.x & 63;
  const int g = lane >> 3;   // which of the 8 rows of a wave load
  const int c8 = lane & 7;   // which 16-byte chunk of the row
  const int64_t head = row / s.T;
  const uint16_t* Kh = K + head * s.T * kHeadDim;
  const uint16_t* Vh = V + head * s.T * kHeadDim;

  // q stays in bf16 pairs: q.k is four packed dot-product instructions per lane (exact products,
  // fp32 sums); the logit scale is applied to the finished dot product
  const uint4 qv = *reinterpret_cast<const uint4*>(Q + row * kHeadDim + c8 * 8);
  const uint32_t qw[4] = {qv.x, qv.y, qv.z, qv.w};
  const float f = s.scale * kLog2e;
  const KeyList kl = key_list(s, row, idx, cnt, L, crow);
  const int32_t n = kl.n;
  const int32_t* irow = kl.p;

  float m_run = -INFINITY, l_run = 0.f;
  float o[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = 0.f;

  for (int32_t k0 = 0; k0 < n; k0 += 8 * kUnroll) {
    uint4 kv[kUnroll], vv[kUnroll];
    bool ok[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int32_t p = k0 + u * 8 + g;
      // the index is read unconditionally (a slot past the list re-reads its last entry and is
      // then discarded): a load behind `p < n` would be waited for before the next slot's is issued
      int32_t j = irow[min(p, n - 1)] - kl.base;
      j = (p < n) ? j : -1;
      ok[u] = static_cast<uint32_t>(j) < static_cast<uint32_t>(s.T);
      j = ok[u] ? j : 0;
      kv[u] = *reinterpret_cast<const uint4*>(Kh + static_cast<int64_t>(j) * kHeadDim + c8 * 8);
      vv[u] = *reinterpret_cast<const uint4*>(Vh + static_cast<int64_t>(j) * kHeadDim + c8 * 8);
    }
    float sc[kUnroll];
    float mx = -INFINITY;
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint32_t w[4] = {kv[u].x, kv[u].y, kv[u].z, kv[u].w};
      float a = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) a = __builtin_amdgcn_fdot2_f32_bf16(as_bf16x2(qw[i]), as_bf16x2(w[i]), a, false);
      a += wave_xor_f(a, 1);
      a += wave_xor_f(a, 2);
      a += wave_xor_f(a, 4);
      sc[u] = ok[u] ? a * f : -INFINITY;
      mx = fmaxf(mx, sc[u]);
    }
    mx = fmaxf(mx, wave_xor_f(mx, 8));
    mx = fmaxf(mx, wave_xor_f(mx, 16));
    mx = fmaxf(mx, wave_xor_f(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    if (m_new == -INFINITY) continue;  // nothing valid yet (uniform across the wave)
    const float corr = exp2f(m_run - m_new);  // exp2(-inf) = 0 on the first valid batch
    m_run = m_new;
    l_run *= corr;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] *= corr;
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const float pj = exp2f(sc[u] - m_new);  // 0 for masked entries
      l_run += pj;
      const uint32_t w[4] = {vv[u].x, vv[u].y, vv[u].z, vv[u].w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        o[2 * i] = fmaf(pj, bf16lo_to_f32(w[i]), o[2 * i]);
        o[2 * i + 1] = fmaf(pj, bf16hi_to_f32(w[i]), o[2 * i + 1]);
      }
    }
  }
  // combine the 8 row groups
#pragma unroll
  for (int mask = 8; mask <= 32; mask <<= 1) {
    l_run += wave_xor_f(l_run, mask);
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] += wave_xor_f(o[e], mask);
  }
  if (g == 0) {
    const float inv = l_run > 0.f ? 1.f / l_run : 0.f;
    uint4 out;
    out.x = pack_bf16(o[0] * inv, o[1] * inv);
    out.y = pack_bf16(o[2] * inv, o[3] * inv);
    out.z = pack_bf16(o[4] * inv, o[5] * inv);
    out.w = pack_bf16(o[6] * inv, o[7] * inv);
    *reinterpret_cast<uint4*>(O + row * kHeadDim + c8 * 8) = out;
  }
}

// ------------------------------------------------------------------------------------------
// fp32: 16 lanes per row, 4 rows per wave load; q.k accumulates in fp64 so that logits of
// magnitude ~40 still leave the probabilities accurate to ~1e-7
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kWavesPerBlock* kWave) void sparse_attn_f32_kernel(
    Shape s, const float* __restrict__ Q, const float* __restrict__ K, const float* __restrict__ V,
    const int32_t* __restrict__ idx, const int32_t* __restrict__ cnt, int32_t L,
    const int64_t* __restrict__ crow, float* __restrict__ O) {
  const uint32_t lb = xcd_contiguous(blockIdx.x, gridDim.x);
  const int64_t row = static_cast<int64_t>(lb) * kWavesPerBlock + (threadIdx.x >> 6);
  const int64_t nrows = static_cast<int64_t>(s.N) * s.T;
  if (row >= nrows) return;
  const int lane = threadIdx.x & 63;
  const int g = lane >> 4;    // which of the 4 rows of a wave load
  const int c16 = lane & 15;  // which 16-byte chunk of the row
  const int64_t head = row / s.T;
  const float* Kh = K + head * s.T * kHeadDim;
  const float* Vh = V + head * s.T * kHeadDim;

  const float4 q4 = *reinterpret_cast<const float4*>(Q + row * kHeadDim + c16 * 4);
  const double qd[4] = {q4.x, q4.y, q4.z, q4.w};
  const double f = static_cast<double>(s.scale) * 1.4426950408889634;
  const KeyList kl = key_list(s, row, idx, cnt, L, crow);
  const int32_t n = kl.n;
  const int32_t* irow = kl.p;

  double m_run = -INFINITY;
  float l_run = 0.f;
  float o[4] = {0.f, 0.f, 0.f, 0.f};

  for (int32_t k0 = 0; k0 < n; k0 += 4 * kUnroll) {
    float4 kv[kUnroll], vv[kUnroll];
    bool ok[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int32_t p = k0 + u * 4 + g;
      // the index is read unconditionally (a slot past the list re-reads its last entry and is
      // then discarded): a load behind `p < n` would be waited for before the next slot's is issued
      int32_t j = irow[min(p, n - 1)] - kl.base;
      j = (p < n) ? j : -1;
      ok[u] = static_cast<uint32_t>(j) < static_cast<uint32_t>(s.T);
      j = ok[u] ? j : 0;
      kv[u] = *reinterpret_cast<const float4*>(Kh + static_cast<int64_t>(j) * kHeadDim + c16 * 4);
      vv[u] = *reinterpret_cast<const float4*>(Vh + static_cast<int64_t>(j) * kHeadDim + c16 * 4);
    }
    double sc[kUnroll];
    double mx = -INFINITY;
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      double a = qd[0] * kv[u].x;
      a = fma(qd[1], static_cast<double>(kv[u].y), a);
      a = fma(qd[2], static_cast<double>(kv[u].z), a);
      a = fma(qd[3], static_cast<double>(kv[u].w), a);
      a += wave_xor_d(a, 1);
      a += wave_xor_d(a, 2);
      a += wave_xor_d(a, 4);
      a += wave_xor_d(a, 8);
      sc[u] = ok[u] ? a * f : -INFINITY;
      mx = fmax(mx, sc[u]);
    }
    mx = fmax(mx, wave_xor_d(mx, 16));
    mx = fmax(mx, wave_xor_d(mx, 32));
    const double m_new = fmax(m_run, mx);
    if (m_new == -INFINITY) continue;
    const float corr = exp2f(static_cast<float>(m_run - m_new));
    m_run = m_new;
    l_run *= corr;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] *= corr;
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const float pj = exp2f(static_cast<float>(sc[u] - m_new));
      l_run += pj;
      o[0] = fmaf(pj, vv[u].x, o[0]);
      o[1] = fmaf(pj, vv[u].y, o[1]);
      o[2] = fmaf(pj, vv[u].z, o[2]);
      o[3] = fmaf(pj, vv[u].w, o[3]);
    }
  }
#pragma unroll
  for (int mask = 16; mask <= 32; mask <<= 1) {
    l_run += wave_xor_f(l_run, mask);
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] += wave_xor_f(o[e], mask);
  }
  if (g == 0) {
    float4 out = {0.f, 0.f, 0.f, 0.f};
    if (l_run > 0.f) out = {o[0] / l_run, o[1] / l_run, o[2] / l_run, o[3] / l_run};
    *reinterpret_cast<float4*>(O + row * kHeadDim + c16 * 4) = out;
  }
}

}  // namespace

hipError_t launch_sparse_attn(const Shape& s, sea_dtype dt, const void* Q, const void* K,
                              const void* V, const int32_t* idx, const int32_t* cnt, int32_t L,
                              const int64_t* crow, void* O, hipStream_t st) {
  const int64_t nrows = static_cast<int64_t>(s.N) * s.T;
  const uint32_t grid = static_cast<uint32_t>((nrows + kWavesPerBlock - 1) / kWavesPerBlock);
  StageScope scope(SEA_STAGE_SPARSE, st);
  if (dt == SEA_BF16) {
    hipLaunchKernelGGL(sparse_attn_bf16_kernel, dim3(grid), dim3(kWavesPerBlock * kWave), 0, st, s,
                       static_cast<const uint16_t*>(Q), static_cast<const uint16_t*>(K),
                       static_cast<const uint16_t*>(V), idx, cnt, L, crow, static_cast<uint16_t*>(O));
  } else {
    hipLaunchKernelGGL(sparse_attn_f32_kernel, dim3(grid), dim3(kWavesPerBlock * kWave), 0, st, s,
                       static_cast<const float*>(Q), static_cast<const float*>(K),
                       static_cast<const float*>(V), idx, cnt, L, crow, static_cast<float*>(O));
  }
  return hipGetLastError();
}

}  // namespace sea

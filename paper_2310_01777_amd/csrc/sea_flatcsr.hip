// FlatCSR tensor of the expanded mask (Sec. 3.1.1 "FlatCSR", App. A.5 "FlatCSR: Modified CSR
// Format To Handle Grouped Mask"): M* [B][H][T][T] with the head and query axes exchanged and
// (head, key) flattened into one column axis, stored as CSR.  Row b T + t lists h T + j for the
// keys j head h attends from query t, heads ascending, keys ascending inside a head.
//
// Built from the per-(head, row) key lists in three launches: per-row entry counts with an
// exclusive scan inside each 256-row block, a one-block scan of the block totals, and a copy that
// moves each list to its place with one wavefront per CSR row (reads and writes contiguous).
#include "sea_internal.h"

namespace sea {
namespace {

constexpr int kScanRows = 256;

__device__ __forceinline__ int64_t wave_inclusive(int64_t v, int lane) {
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    const int64_t u = __shfl_up(v, d, kWave);
    if (lane >= d) v += u;
  }
  return v;
}

__device__ __forceinline__ int32_t list_len(const int32_t* __restrict__ cnt, int64_t i, int32_t L) {
  return min(max(cnt[i], 0), L);
}

__global__ __launch_bounds__(kScanRows) void flat_count_kernel(Shape s, const int32_t* __restrict__ cnt,
                                                               int32_t L, int64_t R,
                                                               int64_t* __restrict__ crow,
                                                               int64_t* __restrict__ bsum) {
  __shared__ int64_t wtot[kScanRows / kWave];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = static_cast<int64_t>(blockIdx.x) * kScanRows + threadIdx.x;
  int64_t n = 0;
  if (row < R) {
    const int64_t b = row / s.T, t = row - b * s.T;
    for (int32_t h = 0; h < s.H; ++h) n += list_len(cnt, (b * s.H + h) * s.T + t, L);
  }
  const int64_t inc = wave_inclusive(n, lane);
  if (lane == kWave - 1) wtot[wave] = inc;
  __syncthreads();
  int64_t off = 0;
  for (int w = 0; w < wave; ++w) off += wtot[w];
  if (row < R) crow[row] = off + inc - n;  // exclusive inside the block; the block base comes later
  if (threadIdx.x == kScanRows - 1) bsum[blockIdx.x] = off + inc;
}

// exclusive scan of the block totals in place, grand total to *total
__global__ __launch_bounds__(1024) void flat_scan_kernel(int64_t* __restrict__ bsum, int64_t nblk,
                                                         int64_t* __restrict__ total) {
  __shared__ int64_t wtot[1024 / kWave];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int64_t carry = 0;
  for (int64_t base = 0; base < nblk; base += 1024) {
    const int64_t i = base + threadIdx.x;
    const int64_t v = i < nblk ? bsum[i] : 0;
    const int64_t inc = wave_inclusive(v, lane);
    if (lane == kWave - 1) wtot[wave] = inc;
    __syncthreads();
    int64_t off = 0, all = 0;
    for (int w = 0; w < 1024 / kWave; ++w) {
      if (w < wave) off += wtot[w];
      all += wtot[w];
    }
    if (i < nblk) bsum[i] = carry + off + inc - v;
    carry += all;
    __syncthreads();
  }
  if (threadIdx.x == 0) *total = carry;
}

__global__ __launch_bounds__(256) void flat_copy_kernel(Shape s, const int32_t* __restrict__ idx,
                                                        const int32_t* __restrict__ cnt, int32_t L, int64_t R,
                                                        int64_t* __restrict__ crow,
                                                        const int64_t* __restrict__ bsum,
                                                        int32_t* __restrict__ col, int64_t cap) {
  const int lane = threadIdx.x & 63;
  const int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (row >= R) return;
  const int64_t b = row / s.T, t = row - b * s.T;
  const int64_t start = crow[row] + bsum[row / kScanRows];
  int64_t off = start;
  for (int32_t h = 0; h < s.H; ++h) {
    const int64_t r = (b * s.H + h) * s.T + t;
    const int32_t n = list_len(cnt, r, L);
    const int32_t* src = idx + r * L;
    for (int32_t i = lane; i < n; i += kWave)
      if (off + i < cap) col[off + i] = h * s.T + src[i];
    off += n;
  }
  if (lane == 0) crow[row] = start;  // only this wavefront reads crow[row], before this store
}

}  // namespace

size_t flatcsr_workspace(const Shape& s) {
  const int64_t R = static_cast<int64_t>(s.N / s.H) * s.T;
  return static_cast<size_t>((R + kScanRows - 1) / kScanRows) * sizeof(int64_t);
}

hipError_t launch_flatcsr(const Shape& s, const int32_t* idx, const int32_t* cnt, int32_t L, int64_t* crow,
                          int32_t* col, int64_t cap, void* ws, hipStream_t st) {
  const int64_t R = static_cast<int64_t>(s.N / s.H) * s.T;
  const int64_t nblk = (R + kScanRows - 1) / kScanRows;
  int64_t* bsum = static_cast<int64_t*>(ws);
  StageScope scope(SEA_STAGE_TOPK_MASK, st);
  hipLaunchKernelGGL(flat_count_kernel, dim3(static_cast<uint32_t>(nblk)), dim3(kScanRows), 0, st, s, cnt, L, R,
                     crow, bsum);
  hipLaunchKernelGGL(flat_scan_kernel, dim3(1), dim3(1024), 0, st, bsum, nblk, crow + R);
  hipLaunchKernelGGL(flat_copy_kernel, dim3(static_cast<uint32_t>((R + 3) / 4)), dim3(256), 0, st, s, idx, cnt, L,
                     R, crow, bsum, col, cap);
  return hipGetLastError();
}

}  // namespace sea

// Estimate in the per-row width geometry for fp32 tensors (App. A.4, figure of the masking process: in causal
// attention every row of A^ and M^ is resized to its own width).  Row t spreads its K columns
// over its own t + 1 keys: column c holds the keys [b_c, b_{c+1}), b_c = ceil(c (t+1) / K), so
//   A^[t][c] = phi(q_t) . (P[b_{c+1}] - P[b_c]) / (phi(q_t) . P[t+1]),
// with P[j] = sum_{j' < j} phi(k_j') the running FAVOR+ key state (Sec. 3 "Performer (FAVOR+)",
// causal form).  No two rows share a column's key range, so the T x K contraction is not a
// matrix product: it is K + 1 gathered dot products of length m per row, bound by the cache
// bandwidth of the gathers (the prefix table of a head, (T+1) m elements, stays in its XCD's L2).
//
//   prefix_kernel<.., false> per (head, chunk of keys): chunk totals of phi(k), fp64 running sum
//   chunk_base_kernel        per head: exclusive scan of the chunk totals (fp64)
//   prefix_kernel<.., true>  same walk again, writes P = chunk base + running sum
//   rows_kernel              one wavefront per two or four consecutive rows: phi(q_t), the K gathers of
//                            neighbouring prefix rows, their differences, row norm
// Features, prefixes and dot products are fp64; a difference of fp32 prefixes could not resolve
// scores below ~1e-6 of the row, and with k^ = K / 2 such scores sit at the selection boundary of
// many rows.  For m <= 128 the prefix form above is replaced by rw_tiles_kernel (further down): the
// same sums taken from tiles of phi(K) phi(Q)^T on the fp64 matrix cores.  bf16 tensors take the
// bf16 matrix-core form in its own file.
#include "sea_internal.h"

namespace sea {
namespace {

constexpr int kStage = 64;        // keys staged in LDS at a time
constexpr int kMaxChunks = 64;    // chunks per head
constexpr int kRowWaves = 4;

// element i of an fp32 tensor, converted to the arithmetic type F
template <typename F>
__device__ __forceinline__ F elem(const float* p, int64_t i) {
  return static_cast<F>(p[i]);
}

// N consecutive elements as one aligned vector load
template <typename E, int N>
struct alignas(sizeof(E) * N) Vec {
  E v[N];
};
template <typename E, int N>
__device__ __forceinline__ Vec<E, N> load_vec(const E* p) {
  return *reinterpret_cast<const Vec<E, N>*>(p);
}

__device__ __forceinline__ float exp_of(float x) { return exp2f(x * kLog2e); }
__device__ __forceinline__ double exp_of(double x) { return exp(x); }

__host__ __device__ __forceinline__ int32_t chunk_len(int32_t T) {
  const int32_t c = (T + kMaxChunks - 1) / kMaxChunks;
  return ((c + kStage - 1) / kStage) * kStage;
}

// block = m threads, thread i owns feature i; grid = heads x chunks
template <typename F, typename TI, bool WRITE>
__global__ __launch_bounds__(256) void prefix_kernel(Shape s, const TI* __restrict__ Kt, const TI* __restrict__ W,
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
  for (int e = 0; e < kHeadDim; ++e) w[e] = elem<F>(W, static_cast<int64_t>(i) * kHeadDim + e);
  const TI* Kh = Kt + head * s.T * kHeadDim;
  F* Ph = P + head * (static_cast<int64_t>(s.T) + 1) * s.m;
  // Both walks add up the chunk's features from zero in the same order; the second one stores
  // base + partial sum, so the last prefix of a chunk is exactly the next chunk's base and the
  // stored prefixes never decrease.
  const double base = WRITE ? cbase[(head * nch + chunk) * s.m + i] : 0.0;
  double run = 0.0;
  if (WRITE && chunk == 0) Ph[i] = static_cast<F>(0);
  for (int32_t js = j0; js < j1; js += kStage) {
    const int32_t nk = min(kStage, j1 - js);
    __syncthreads();
    for (int32_t x = threadIdx.x; x < nk * kHeadDim; x += blockDim.x)
      y[x / kHeadDim][x % kHeadDim] = rs * elem<F>(Kh, static_cast<int64_t>(js) * kHeadDim + x);
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
      if (WRITE) Ph[static_cast<int64_t>(js + j + 1) * s.m + i] = static_cast<F>(base + run);
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
// Eight wave sums for the price of ten exchanges: at each of the first three steps a lane keeps
// the half of the values its lane bit names and hands the other half to its partner.  Lane l ends
// with the full sum of p[l & 7]; every value is added up in the same butterfly order.
template <typename F>
__device__ __forceinline__ F wave_sum8(const F (&p)[8], int lane) {
  F a[4], b[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const bool hi = lane & 1;
    a[i] = (hi ? p[2 * i + 1] : p[2 * i]) + __shfl_xor(hi ? p[2 * i] : p[2 * i + 1], 1, kWave);
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const bool hi = lane & 2;
    b[i] = (hi ? a[2 * i + 1] : a[2 * i]) + __shfl_xor(hi ? a[2 * i] : a[2 * i + 1], 2, kWave);
  }
  const bool hi = lane & 4;
  F c = (hi ? b[1] : b[0]) + __shfl_xor(hi ? b[0] : b[1], 4, kWave);
  c += __shfl_xor(c, 8, kWave);
  c += __shfl_xor(c, 16, kWave);
  c += __shfl_xor(c, 32, kWave);
  return c;
}
template <typename F>
__device__ __forceinline__ F wave_max(F v) {
#pragma unroll
  for (int mask = 1; mask < kWave; mask <<= 1) v = max(v, __shfl_xor(v, mask, kWave));
  return v;
}

// R consecutive rows per wavefront, MU = m / 64 consecutive features per lane (feature = lane MU + u: a lane's share of a prefix
// row is one vector load, a wavefront's the whole row), SLOTS = ceil(K / 64) column slots per
// lane (column = q 64 + lane).  W^T sits in LDS in the tensors' own element type, [e][i].
template <typename F, typename TI, int MU, int SLOTS, int R>
__global__ __launch_bounds__(kRowWaves* kWave) void rows_kernel(Shape s, const TI* __restrict__ Q,
                                                                const TI* __restrict__ W,
                                                                const F* __restrict__ P, float* __restrict__ A_hat) {
  using WT = TI;
  extern __shared__ __align__(16) unsigned char wt_raw[];
  WT* wt = reinterpret_cast<WT*>(wt_raw);  // [64][m]
  for (int32_t x = threadIdx.x; x < s.m * kHeadDim; x += blockDim.x) {
    const int32_t i = x / kHeadDim, e = x % kHeadDim;
    wt[e * s.m + i] = W[x];
  }
  __syncthreads();
  const int lane = threadIdx.x & 63;
  const int64_t nrows = static_cast<int64_t>(s.N) * s.T;
  const uint32_t lb = xcd_contiguous(blockIdx.x, gridDim.x);
  const int64_t first = (static_cast<int64_t>(lb) * kRowWaves + (threadIdx.x >> 6)) * R;
  const F rs = static_cast<F>(sqrtf(s.scale));
  // The wavefront's R consecutive rows walk the columns together: their boundaries of a column
  // are at most R - 1 keys apart, so most of their prefix rows are the same cache lines.
  F phi[R][MU];
  const F* Ph[R];
  int64_t width[R];
  bool valid[R], active[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    valid[r] = first + r < nrows;
    const int64_t row = valid[r] ? first + r : nrows - 1;
    const int64_t head = row / s.T;
    const int32_t t = static_cast<int32_t>(row - head * s.T);
    const int32_t b = static_cast<int32_t>(head / s.H);
    const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
    active[r] = valid[r] && t < len;
    Ph[r] = P + head * (static_cast<int64_t>(s.T) + 1) * s.m + lane * MU;
    width[r] = static_cast<int64_t>(t) + 1;
    // phi(q_t) up to a row factor (|x|^2 / 2 and the largest exponent cancel in the row norm):
    // lane e holds x[e]; feature lane MU + u in slot u
    const F xe = rs * elem<F>(Q, row * kHeadDim + lane);
    F arg[MU];
#pragma unroll
    for (int u = 0; u < MU; ++u) arg[u] = 0;
#pragma unroll
    for (int e = 0; e < kHeadDim; ++e) {
      const F x = __shfl(xe, e, kWave);
      const Vec<WT, MU> wv = load_vec<WT, MU>(wt + e * s.m + lane * MU);
#pragma unroll
      for (int u = 0; u < MU; ++u) arg[u] += elem<F>(wv.v, u) * x;
    }
    F top = arg[0];
#pragma unroll
    for (int u = 1; u < MU; ++u) top = max(top, arg[u]);
    top = wave_max(top);
#pragma unroll
    for (int u = 0; u < MU; ++u) phi[r][u] = exp_of(arg[u] - top);
  }

  // column c: phi . (P[b_{c+1}] - P[b_c]), b_c = ceil(c (t+1) / K), the difference taken element
  // by element first (its error is that of the two stored prefixes, not of two long dot
  // products); column c lives in lane c % 64, slot c / 64.  The boundary vector of the previous
  // column stays in registers.
  F g[R][SLOTS];
  Vec<F, MU> prev[R];
  // c (t+1) = fq K + fr, stepped from column to column (no division per boundary)
  int32_t wq[R], wr[R], fq[R], fr[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
#pragma unroll
    for (int q = 0; q < SLOTS; ++q) g[r][q] = 0;
    prev[r] = load_vec<F, MU>(Ph[r]);  // P[0] = 0
    wq[r] = static_cast<int32_t>(width[r] / s.K);
    wr[r] = static_cast<int32_t>(width[r] - static_cast<int64_t>(wq[r]) * s.K);
    fq[r] = 0;
    fr[r] = 0;
  }
#pragma unroll
  for (int q = 0; q < SLOTS; ++q) {
    const int32_t cn = min(kWave, s.K - q * kWave);  // columns of this slot (uniform)
    for (int32_t l0 = 0; l0 < cn; l0 += 8) {
#pragma unroll
      for (int r = 0; r < R; ++r) {
        Vec<F, MU> pv[8];
#pragma unroll
        for (int v = 0; v < 8; ++v) {
          if (q * kWave + l0 + v + 1 <= s.K) {  // next column; past the last one the boundary stays t + 1
            fq[r] += wq[r];
            fr[r] += wr[r];
            if (fr[r] >= s.K) {
              fr[r] -= s.K;
              ++fq[r];
            }
          }
          const int64_t bc = fq[r] + (fr[r] > 0 ? 1 : 0);  // ceil(c (t+1) / K) <= t + 1
          pv[v] = load_vec<F, MU>(Ph[r] + bc * s.m);
        }
        F part[8];
#pragma unroll
        for (int v = 0; v < 8; ++v) {
          F acc = 0;
#pragma unroll
          for (int u = 0; u < MU; ++u)
            acc += phi[r][u] * (pv[v].v[u] - (v == 0 ? prev[r].v[u] : pv[v - 1].v[u]));
          part[v] = acc;
        }
        prev[r] = pv[7];
        const F sum = wave_sum8(part, lane);  // lane l: column l0 + (l & 7)
        if ((lane >> 3) == (l0 >> 3)) g[r][q] = sum;
      }
    }
  }
#pragma unroll
  for (int r = 0; r < R; ++r) {
    if (!valid[r]) continue;
    float* Arow = A_hat + (first + r) * s.K;
    // row normaliser phi . P[t + 1]
    F total = 0;
    const Vec<F, MU> pe = load_vec<F, MU>(Ph[r] + width[r] * s.m);
#pragma unroll
    for (int u = 0; u < MU; ++u) total += phi[r][u] * pe.v[u];
    total = wave_sum(total);
    const F inv = (active[r] && total > static_cast<F>(0)) ? static_cast<F>(1) / total : static_cast<F>(0);
#pragma unroll
    for (int q = 0; q < SLOTS; ++q) {
      const int32_t c = q * kWave + lane;
      if (c < s.K) Arow[c] = static_cast<float>(g[r][q] * inv);
    }
  }
}

// ------------------------------------------------------------------------------------------
// The same estimate without prefixes: A^[t][c] is the sum of a_tj = phi(q_t) . phi(k_j) over the keys
// j of row t's column c, and the a_tj of 16 rows x 16 keys are one tile of phi(K) phi(Q)^T on the
// fp64 matrix cores (v_mfma_f64_16x16x4_f64; lane l supplies A[row l % 16][k l / 16] and
// B[k l / 16][col l % 16], result register i is D[row 4 i + l / 16][col l % 16]).  One wavefront
// per (head, 16-row tile) walks the causal key chunks; the operand rows are permuted so that a lane
// ends up with four consecutive keys of its query, adds each product to the bin of its column
// floor(j K / (t + 1)) in LDS ([16 rows][K] fp64), and the bins leave normalised by their row sum
// (= phi(q_t) . sum_{j <= t} phi(k_j)).  Nothing is differenced, so there is no cancellation, and
// the key features are read T / 16 times per head from the L2 instead of K + 1 prefix vectors per row.
// The contraction index is a free permutation of the features: step s of lane group g is feature
// 8 (s / 2) + 2 g + s % 2, which makes every operand load a 16-byte piece.
// ------------------------------------------------------------------------------------------
typedef double doublex4 __attribute__((ext_vector_type(4)));

template <int MQ>  // m / 4: contraction steps
__global__ __launch_bounds__(64) void rw_tiles_kernel(Shape s, const double* __restrict__ phiQ,
                                                      const double* __restrict__ phiK, float* __restrict__ A_hat) {
  extern __shared__ __align__(16) double bins[];  // [16][K + 1]
  __shared__ double tot_s[16][4];
  const int lane = threadIdx.x, qc = lane & 15, g = lane >> 4;
  const int32_t m = 4 * MQ;
  const uint32_t tiles = (s.T + 15) / 16;
  // Head-major, each XCD on a contiguous range of blocks: the row tiles of a head run close together
  // on one XCD, whose L2 then serves all but the first read of the head's key features.  Within a
  // head the longest (last) row tiles come first.
  const uint32_t lb = xcd_contiguous(blockIdx.x, gridDim.x);
  const int64_t head = lb / tiles;
  const uint32_t tile = tiles - 1 - lb % tiles;
  const int32_t r0 = static_cast<int32_t>(tile) * 16;
  const int32_t t = r0 + qc;
  const int32_t b = static_cast<int32_t>(head / s.H);
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
  const bool active = t < len;
  const int32_t tq = min(t, s.T - 1);
  const int32_t bstride = s.K + 1;
  for (int32_t x = lane; x < 16 * bstride; x += 64) bins[x] = 0.0;
  double qd[MQ];
  {
    const double* qr = phiQ + (head * s.T + tq) * m + 2 * g;
#pragma unroll
    for (int j = 0; j < MQ / 2; ++j) {
      const double2 v = *reinterpret_cast<const double2*>(qr + 8 * j);
      qd[2 * j] = v.x;
      qd[2 * j + 1] = v.y;
    }
  }
  const double inv_w = 1.0 / static_cast<double>(t + 1);
  const double* Kh = phiK + head * static_cast<int64_t>(s.T) * m;
  const int32_t last_key = min(min(r0 + 15, s.T - 1), len - 1);  // keys past it reach no row of the tile
  const int32_t nchunks = last_key < 0 ? 0 : last_key / 16 + 1;
  // operand row lr stands for key 4 (lr % 4) + lr / 4 of the chunk: result register i of lane group g is key 4 g + i
  const int32_t krow = 4 * (qc & 3) + (qc >> 2);
  double kn[MQ];
  auto request = [&](int32_t c) {
    const double* kr = Kh + static_cast<int64_t>(min(16 * c + krow, s.T - 1)) * m + 2 * g;
#pragma unroll
    for (int j = 0; j < MQ / 2; ++j) {
      const double2 v = *reinterpret_cast<const double2*>(kr + 8 * j);
      kn[2 * j] = v.x;
      kn[2 * j + 1] = v.y;
    }
  };
  __syncthreads();
  if (nchunks > 0) request(0);
  for (int32_t c = 0; c < nchunks; ++c) {
    double kd[MQ];
#pragma unroll
    for (int x = 0; x < MQ; ++x) kd[x] = kn[x];
    if (c + 1 < nchunks) request(c + 1);
    doublex4 acc0 = {0.0, 0.0, 0.0, 0.0}, acc1 = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int x = 0; x < MQ; x += 2) {
      acc0 = __builtin_amdgcn_mfma_f64_16x16x4f64(kd[x], qd[x], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f64_16x16x4f64(kd[x + 1], qd[x + 1], acc1, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int32_t j = 16 * c + 4 * g + i;
      if (active && j <= t && j < len) {
        // column of key j in row t: floor(j K / (t + 1)), exact in fp64 (the half step keeps the
        // product away from integers by 0.5 / (t + 1), far more than its rounding error)
        const int32_t col = static_cast<int32_t>((static_cast<double>(static_cast<int64_t>(j) * s.K) + 0.5) * inv_w);
        atomicAdd(&bins[qc * bstride + col], acc0[i] + acc1[i]);
      }
    }
  }
  __syncthreads();
  // row sums: lane (qc, g) adds the columns c = g (mod 4), the four parts meet in LDS
  {
    double part = 0.0;
    for (int32_t c = g; c < s.K; c += 4) part += bins[qc * bstride + c];
    tot_s[qc][g] = part;
  }
  __syncthreads();
  for (int32_t x = lane; x < 16 * s.K; x += 64) {
    const int32_t q = x / s.K, c = x - q * s.K;
    const int32_t tt = r0 + q;
    if (tt >= s.T) continue;
    const double total = (tot_s[q][0] + tot_s[q][1]) + (tot_s[q][2] + tot_s[q][3]);
    const double inv = (tt < len && total > 0.0) ? 1.0 / total : 0.0;
    A_hat[(head * s.T + tt) * s.K + c] = static_cast<float>(bins[q * bstride + c] * inv);
  }
}

// the tile form needs the bins of 16 rows in LDS and, for now, the contraction operands of a
// chunk in registers twice over (m <= 128)
bool tiles_supported(const Shape& s) { return (s.m == 64 || s.m == 128) && s.K <= 1024; }

struct Layout {
  size_t ctot, cbase, P, total;
  int32_t nch;
};
Layout layout(const Shape& s) {
  Layout l{};
  const int32_t CH = chunk_len(s.T);
  l.nch = (s.T + CH - 1) / CH;
  const size_t tab = (static_cast<size_t>(s.N) * l.nch * s.m * sizeof(double) + 255) & ~size_t(255);
  l.ctot = 0;
  l.cbase = tab;
  l.P = 2 * tab;
  l.total = l.P + ((static_cast<size_t>(s.N) * (static_cast<size_t>(s.T) + 1) * s.m * sizeof(double) + 255) & ~size_t(255));
  if (tiles_supported(s)) {
    // tile form: phi(Q) and phi(K) in fp64, [N][T][m] each
    const size_t one = (static_cast<size_t>(s.N) * s.T * s.m * sizeof(double) + 255) & ~size_t(255);
    l.total = 2 * one;
  }
  return l;
}

template <typename F, typename TI, int MU>
hipError_t launch_rows(const Shape& s, const TI* Q, const TI* W, const F* P,
                       float* A_hat, hipStream_t st) {
  const int64_t nrows = static_cast<int64_t>(s.N) * s.T;
  // rows a wavefront walks together: four while a lane's share of a prefix row is at most two
  // elements, two for m = 256 (four elements), where more rows would cost a wave of occupancy
  constexpr int R = MU <= 2 ? 4 : 2;
  const int64_t per_block = kRowWaves * R;
  const dim3 grid(static_cast<uint32_t>((nrows + per_block - 1) / per_block));
  const size_t lds = static_cast<size_t>(s.m) * kHeadDim * sizeof(TI);
  const int slots = (s.K + kWave - 1) / kWave;
#define SEA_RW_ROWS(SL)                                                                                      \
  hipLaunchKernelGGL((rows_kernel<F, TI, MU, SL, R>), grid, dim3(kRowWaves* kWave), lds, st, s, Q, W, P, A_hat)
  if (slots <= 1) SEA_RW_ROWS(1);
  else if (slots <= 2) SEA_RW_ROWS(2);
  else if (slots <= 4) SEA_RW_ROWS(4);
  else if (slots <= 8) SEA_RW_ROWS(8);
  else SEA_RW_ROWS(16);
#undef SEA_RW_ROWS
  return hipGetLastError();
}

template <typename F, typename TI>
hipError_t launch_all(const Shape& s, const void* Qv, const void* Kv, const void* Wv, float* A_hat,
                      void* ws, hipStream_t st) {
  const TI* Q = static_cast<const TI*>(Qv);
  const TI* K = static_cast<const TI*>(Kv);
  const TI* W = static_cast<const TI*>(Wv);
  const Layout l = layout(s);
  char* base = static_cast<char*>(ws);
  double* ctot = reinterpret_cast<double*>(base + l.ctot);
  double* cbase = reinterpret_cast<double*>(base + l.cbase);
  F* P = reinterpret_cast<F*>(base + l.P);
  const dim3 pgrid(static_cast<uint32_t>(s.N) * l.nch);
  {
    StageScope scope(SEA_STAGE_STATE, st);
    hipLaunchKernelGGL((prefix_kernel<F, TI, false>), pgrid, dim3(s.m), 0, st, s, K, W, ctot, cbase, P);
    hipLaunchKernelGGL(chunk_base_kernel, dim3(s.N), dim3(s.m), 0, st, ctot, cbase, l.nch, s.m);
    hipLaunchKernelGGL((prefix_kernel<F, TI, true>), pgrid, dim3(s.m), 0, st, s, K, W, ctot, cbase, P);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  StageScope scope(SEA_STAGE_CONTRACT, st);
  switch (s.m / kWave) {
    case 1: return launch_rows<F, TI, 1>(s, Q, W, P, A_hat, st);
    case 2: return launch_rows<F, TI, 2>(s, Q, W, P, A_hat, st);
    default: return launch_rows<F, TI, 4>(s, Q, W, P, A_hat, st);
  }
}

}  // namespace

bool estimate_rowwidth_supported(const Shape& s) { return s.causal && (s.m == 64 || s.m == 128 || s.m == 256); }

size_t estimate_rowwidth_workspace(const Shape& s, sea_dtype dt) {
  return rowwidth_mfma_supported(s, dt) ? rowwidth_mfma_workspace(s) : layout(s).total;
}

hipError_t launch_estimate_rowwidth(const Shape& s, sea_dtype dt, const void* Q, const void* K, const void* W,
                                    float* A_hat, void* ws, hipStream_t st) {
  if (rowwidth_mfma_supported(s, dt))
    return launch_rowwidth_mfma(s, static_cast<const uint16_t*>(Q), static_cast<const uint16_t*>(K),
                                static_cast<const uint16_t*>(W), A_hat, ws, st);
  if (dt != SEA_F32) return hipErrorNotSupported;
  if (tiles_supported(s)) {
    const size_t one = (static_cast<size_t>(s.N) * s.T * s.m * sizeof(double) + 255) & ~size_t(255);
    double* phiQ = static_cast<double*>(ws);
    double* phiK = reinterpret_cast<double*>(static_cast<char*>(ws) + one);
    {
      StageScope scope(SEA_STAGE_FEATURES, st);
      const hipError_t e = launch_features_f64(s, static_cast<const float*>(Q), static_cast<const float*>(K),
                                               static_cast<const float*>(W), phiQ, phiK, st);
      if (e != hipSuccess) return e;
    }
    StageScope scope(SEA_STAGE_CONTRACT, st);
    const dim3 grid(static_cast<uint32_t>(s.N) * ((s.T + 15) / 16));
    const size_t lds = static_cast<size_t>(16) * (s.K + 1) * sizeof(double);
    if (lds > (64u << 10)) {
      const void* fn = s.m == 64 ? reinterpret_cast<const void*>(&rw_tiles_kernel<16>)
                                 : reinterpret_cast<const void*>(&rw_tiles_kernel<32>);
      const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
      if (e != hipSuccess) return e;
    }
    if (s.m == 64)
      hipLaunchKernelGGL(rw_tiles_kernel<16>, grid, dim3(64), lds, st, s, phiQ, phiK, A_hat);
    else
      hipLaunchKernelGGL(rw_tiles_kernel<32>, grid, dim3(64), lds, st, s, phiQ, phiK, A_hat);
    return hipGetLastError();
  }
  return launch_all<double, float>(s, Q, K, W, A_hat, ws, st);
}

}  // namespace sea

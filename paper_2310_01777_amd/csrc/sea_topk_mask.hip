// Per-query top-k^ selection on the compressed estimate and its expansion to key positions
// (Sec. 3.1 "Grouped Top-k^ Selection", per-query grouping; "Linear Sparse Attention Mask
// Generation" and App. A.5.3 for the nearest-neighbour expansion with a replication cap).
//
// One wavefront owns one query row.  The K <= 1024 scores of the row sit in registers,
// SLOTS = ceil(K / 64) per lane (column = slot * 64 + lane).  The k^-th largest score is
// found exactly by a bitwise search on order-preserving integer keys, using wave ballots and
// population counts only; ties at the threshold go to the lower column.  Selected columns
// are compacted in ascending order with ballot prefix counts, then expanded.
#include "sea_internal.h"
#include "sea_rowlanes.h"

namespace sea {
namespace {

constexpr int kWavesPerBlock = 4;
constexpr int kKeyBitWordsMax = 256;  // key-bit rows of at most 256 words: T <= 8192

__device__ __forceinline__ uint32_t ordered_key(float a) {
  a += 0.0f;  // -0 -> +0
  uint32_t u = __float_as_uint(a);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Blocks are dealt per head: blocks_per_head(T, rows a block takes) of them each, so that the head
// and the time step of a row come from 32-bit divisions of the block index rather than from a
// 64-bit row index divided by T and H.
__host__ __device__ __forceinline__ uint32_t blocks_per_head(int32_t T, int32_t rows_per_block) {
  return static_cast<uint32_t>((T + rows_per_block - 1) / rows_per_block);
}

__device__ __forceinline__ int popc64(uint64_t x) { return __popcll(x); }
__device__ __forceinline__ int lanes_below(uint64_t mask, int lane) {
  return __popcll(mask & ((1ull << lane) - 1ull));
}

// The keys a selected column c of a row emits (App. A.5.3: r = min(w, cap) keys start + floor(i w / r),
// kept while <= jmax), ORed into the row's key-bit words in LDS.  Tw: the width the row's K columns
// are spread over.
__device__ __forceinline__ void or_column_keys(uint32_t* words, int32_t c, int32_t Tw, int32_t K, int32_t rep_cap,
                                               int32_t jmax) {
  const int32_t s0 = block_start(c, Tw, K);
  const int32_t w = block_start(c + 1, Tw, K) - s0;
  if (w <= 0) return;
  const int32_t r = min(w, rep_cap);
  if (r == w) {
    // the whole column: keys s0 .. min(s0 + w - 1, jmax)
    const int32_t j1 = min(s0 + w - 1, jmax);
    if (s0 > j1) return;
    for (int32_t wd = s0 >> 5; wd <= (j1 >> 5); ++wd) {
      const int32_t lo = max(s0, wd << 5) & 31, hi = min(j1, (wd << 5) + 31) & 31;
      const uint32_t m = (hi == 31 ? 0xffffffffu : ((1u << (hi + 1)) - 1u)) & ~((1u << lo) - 1u);
      atomicOr(&words[wd], m);
    }
  } else {
    for (int32_t i = 0; i < r; ++i) {
      const int32_t j = s0 + static_cast<int32_t>((static_cast<int64_t>(i) * w) / r);
      if (j <= jmax) atomicOr(&words[j >> 5], 1u << (j & 31));
    }
  }
}

// ROWW: per-row width geometry -- a causal row t spreads its K columns over its own t + 1 keys
// (column c = keys [ceil(c (t+1) / K), ceil((c+1)(t+1) / K)); empty columns are no candidates).
// FROMBITS: the selection was already made (mbits holds it, A_hat is not read); only the lists
// are written -- the expansion pass after the causal-per-batch kernel.
template <int SLOTS, bool ROWW, bool FROMBITS>
__global__ __launch_bounds__(kWavesPerBlock* kWave) void topk_mask_kernel(
    Shape s, const float* __restrict__ A_hat, int32_t* __restrict__ sel, int32_t* __restrict__ idx,
    int32_t* __restrict__ cnt, uint32_t* __restrict__ mbits, uint32_t* __restrict__ kb, int32_t KWk) {
  __shared__ int32_t sh_sel[kWavesPerBlock][SLOTS * kWave];
  __shared__ int32_t sh_off[kWavesPerBlock][SLOTS * kWave + 1];
  __shared__ uint32_t sh_kb[kWavesPerBlock][kKeyBitWordsMax];  // the row's key bits (kb != nullptr)
  const int wid = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const uint32_t bph = blocks_per_head(s.T, kWavesPerBlock);
  const uint32_t head = blockIdx.x / bph;
  const int32_t t = static_cast<int32_t>(blockIdx.x - head * bph) * kWavesPerBlock + wid;
  if (t >= s.T) return;  // whole wave leaves; no block-wide barrier is used below
  const int64_t row = static_cast<int64_t>(head) * s.T + t;
  const int32_t b = static_cast<int32_t>(head / static_cast<uint32_t>(s.H));
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
  int32_t* irow = idx ? idx + row * s.L : nullptr;
  int32_t* srow = sel ? sel + row * s.sel_stride : nullptr;
  const int32_t kw = (s.K + 31) / 32;  // mask words per row
  uint32_t* mrow = mbits ? mbits + row * kw : nullptr;

  if (t >= len) {  // inactive row (FROMBITS: its mask words are already zero)
    if (irow)
      for (int32_t x = lane; x < s.L; x += kWave) irow[x] = -1;
    if (srow)
      for (int32_t x = lane; x < s.sel_stride; x += kWave) srow[x] = -1;
    if (mrow && !FROMBITS)
      for (int32_t x = lane; x < kw; x += kWave) mrow[x] = 0u;
    if (kb)
      for (int32_t x = lane; x < KWk; x += kWave) kb[row * KWk + x] = 0u;
    if (cnt && lane == 0) cnt[row] = 0;
    return;
  }
  const int32_t jmax = (s.causal && t < len - 1) ? t : len - 1;  // last admissible key
  const int32_t Tw = ROWW ? t + 1 : s.T;                         // width the K columns are spread over
  const int32_t ncand = bucket_of(jmax, Tw, s.K) + 1;            // candidate columns 0..ncand-1
  const int32_t n = min(s.k_hat, ROWW ? min(s.K, Tw) : ncand);   // ROWW: min(K, t + 1) columns hold a key

  int n_sel = 0;
  if (FROMBITS) {
    // the row's mask words, all requested before the first is used (a slot past K re-reads the
    // last word; its bit is not looked at)
    uint32_t mw[SLOTS];
#pragma unroll
    for (int q = 0; q < SLOTS; ++q) mw[q] = mrow[min(q * kWave + lane, s.K - 1) >> 5];
#pragma unroll
    for (int q = 0; q < SLOTS; ++q) {
      const int32_t c = q * kWave + lane;
      const bool take = c < s.K && ((mw[q] >> (c & 31)) & 1u);
      const uint64_t tk = __ballot(take);
      if (take) sh_sel[wid][n_sel + lanes_below(tk, lane)] = c;
      n_sel += popc64(tk);
    }
  } else {
    uint32_t key[SLOTS];
    // every slot's score is requested before the first is used: a slot past the candidates reads
    // column 0 instead (its value is discarded), so no load sits behind a branch
    float a[SLOTS];
  #pragma unroll
    for (int q = 0; q < SLOTS; ++q) {
      const int32_t c = q * kWave + lane;
      a[q] = A_hat[row * s.K + (c < ncand ? c : 0)];
    }
  #pragma unroll
    for (int q = 0; q < SLOTS; ++q) {
      const int32_t c = q * kWave + lane;
      bool cand = c < ncand;  // c < ncand <= K
      // a row at least K keys wide has a key in every column (the row is wave-uniform)
      if (ROWW && Tw < s.K) cand = cand && block_start(c + 1, Tw, s.K) > block_start(c, Tw, s.K);
      key[q] = cand ? ordered_key(a[q]) : 0u;
    }
    // largest tau with #{key >= tau} >= n  ==  the n-th largest key
    uint32_t tau = 0;
  #pragma unroll 1
    for (int bit = 31; bit >= 0; --bit) {
      const uint32_t trial = tau | (1u << bit);
      int c_ge = 0;
  #pragma unroll
      for (int q = 0; q < SLOTS; ++q) c_ge += popc64(__ballot(key[q] >= trial));
      if (c_ge >= n) tau = trial;
      if (c_ge == n) break;  // the keys >= tau are exactly the n to take (one row per wave: uniform)
    }
    int c_gt = 0;
  #pragma unroll
    for (int q = 0; q < SLOTS; ++q) c_gt += popc64(__ballot(key[q] > tau));
    int need_eq = n - c_gt;  // how many of the entries equal to tau are taken, lowest columns first

    // compaction in ascending column order (slot-major, then lane)
  #pragma unroll
    for (int q = 0; q < SLOTS; ++q) {
      const uint64_t eq = __ballot(key[q] == tau);
      const bool take_eq = (key[q] == tau) && (lanes_below(eq, lane) < need_eq);
      const bool take = (key[q] > tau) || take_eq;
      const uint64_t tk = __ballot(take);
      if (take) sh_sel[wid][n_sel + lanes_below(tk, lane)] = q * kWave + lane;
      if (mrow && lane == 0) {  // selected-column bits: column c is bit c % 32 of word c / 32
        if (2 * q < kw) mrow[2 * q] = static_cast<uint32_t>(tk);
        if (2 * q + 1 < kw) mrow[2 * q + 1] = static_cast<uint32_t>(tk >> 32);
      }
      n_sel += popc64(tk);
      need_eq -= min(need_eq, popc64(eq));
    }
  }
  // n_sel == n by construction (FROMBITS: the number of set bits)
  __builtin_amdgcn_wave_barrier();
  if (srow)
    for (int32_t x = lane; x < s.sel_stride; x += kWave) srow[x] = (x < n_sel) ? sh_sel[wid][x] : -1;
  if (kb) {
    // one bit per key of the row (what keybits_kernel writes from the column bits), straight from
    // the compacted selection: every lane expands one selected column
    for (int32_t x = lane; x < KWk; x += kWave) sh_kb[wid][x] = 0u;
    __builtin_amdgcn_wave_barrier();
    for (int32_t x = lane; x < n_sel; x += kWave) or_column_keys(sh_kb[wid], sh_sel[wid][x], Tw, s.K, s.rep_cap, jmax);
    __builtin_amdgcn_wave_barrier();
    for (int32_t x = lane; x < KWk; x += kWave) kb[row * KWk + x] = sh_kb[wid][x];
  }

  if (!irow && !cnt) return;
  // expansion: selected column c emits r keys start + floor(i w / r), i < r
  const bool uniform = !ROWW && (s.T % s.K) == 0;
  int32_t total;
  if (uniform) {
    const int32_t w = s.T / s.K;
    const int32_t r = min(w, s.rep_cap);
    total = n_sel * r;
    int32_t kept = 0;
    for (int32_t x0 = 0; x0 < s.L; x0 += kWave) {
      const int32_t x = x0 + lane;
      int32_t j = -1;
      if (x < total) {
        const int32_t si = x / r, i = x - si * r;
        const int32_t c = sh_sel[wid][si];
        j = c * w + static_cast<int32_t>((static_cast<int64_t>(i) * w) / r);
        if (j > jmax) j = -1;
      }
      if (irow && x < s.L) irow[x] = j;
      kept += popc64(__ballot(j >= 0));
    }
    total = kept;  // dropped keys are a suffix: only the last selected column can overrun jmax
  } else {
    // ragged columns: offsets of the selections by wave prefix scans, then one pass over the
    // list -- entry x belongs to the last selection si with off[si] <= x (binary search in LDS)
    int32_t acc = 0;  // keys emitted by the selections before this batch (uniform)
    for (int32_t base = 0; base < n_sel; base += kWave) {
      const int32_t si = base + lane;
      int32_t r = 0;
      if (si < n_sel) {
        const int32_t c = sh_sel[wid][si];
        r = min(block_start(c + 1, Tw, s.K) - block_start(c, Tw, s.K), s.rep_cap);
      }
      int32_t inc = r;
#pragma unroll
      for (int d = 1; d < kWave; d <<= 1) {
        const int32_t v = __shfl_up(inc, d, kWave);
        if (lane >= d) inc += v;
      }
      if (si < n_sel) sh_off[wid][si] = acc + inc - r;
      acc += __shfl(inc, kWave - 1, kWave);
    }
    __builtin_amdgcn_wave_barrier();
    int32_t kept = 0;
    for (int32_t x0 = 0; x0 < s.L; x0 += kWave) {
      const int32_t x = x0 + lane;
      int32_t j = -1;
      if (x < acc) {
        int32_t lo = 0, hi = n_sel - 1;
        while (lo < hi) {
          const int32_t mid = (lo + hi + 1) >> 1;
          if (sh_off[wid][mid] <= x) lo = mid; else hi = mid - 1;
        }
        const int32_t c = sh_sel[wid][lo];
        const int32_t s0 = block_start(c, Tw, s.K);
        const int32_t w = block_start(c + 1, Tw, s.K) - s0;
        const int32_t r = min(w, s.rep_cap);
        j = s0 + static_cast<int32_t>((static_cast<int64_t>(x - sh_off[wid][lo]) * w) / r);
        if (j > jmax) j = -1;  // only the tail of the last selected column can overrun jmax
      }
      if (irow && x < s.L) irow[x] = j;
      kept += popc64(__ballot(j >= 0));
    }
    total = kept;
  }
  if (cnt && lane == 0) cnt[row] = total;
}

// ------------------------------------------------------------------------------------------
// The same per-query selection when only the selected-column bits are wanted (the forward paths
// that run the attention on bits), for K <= 64 with 4 | K.  One wavefront owns 16 rows: row
// l % 16 lives in the four lanes l % 16 + 16 q, lane group lg = l / 16 holds the columns
// 16 ct + 4 lg + i of every 16-column tile ct, so a row's K scores are NCT float4 loads per lane and
// every count over a row is NCT x 4 compares in the lane plus two row-swap steps.  Same order-
// preserving keys, same bitwise search (it ends as soon as every row's threshold separates exactly
// its quota), same tie rule (lowest columns first) as the kernel above.
// ------------------------------------------------------------------------------------------
template <int NCT, bool ROWW>
__global__ __launch_bounds__(kWavesPerBlock* kWave) void topk_bits_kernel(Shape s, const float* __restrict__ A_hat,
                                                                         uint32_t* __restrict__ mbits) {
  const int lane = threadIdx.x & 63, lr = lane & 15, lg = lane >> 4;
  const uint32_t bph = blocks_per_head(s.T, 16 * kWavesPerBlock);
  const uint32_t head = blockIdx.x / bph;
  const int32_t t0 = (static_cast<int32_t>(blockIdx.x - head * bph) * kWavesPerBlock + static_cast<int32_t>(threadIdx.x >> 6)) * 16;
  if (t0 >= s.T) return;  // whole wave leaves; no block-wide barrier is used below
  const bool in_head = t0 + lr < s.T;
  const int32_t t = min(t0 + lr, s.T - 1);
  const int64_t row = static_cast<int64_t>(head) * s.T + t;
  const int32_t b = static_cast<int32_t>(head / static_cast<uint32_t>(s.H));
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
  const bool active = in_head && t < len;
  const int32_t jmax = (s.causal && t < len - 1) ? t : len - 1;  // last admissible key
  const int32_t Tw = ROWW ? t + 1 : s.T;                         // width the K columns are spread over
  const int32_t ncand = active ? bucket_of(jmax, Tw, s.K) + 1 : 0;
  const uint32_t nsel = active ? static_cast<uint32_t>(min(s.k_hat, ROWW ? min(s.K, Tw) : ncand)) : 0u;
  // rows narrower than K have columns without a key (wave-uniform: does the wave hold such a row)
  const bool sparse_cols = ROWW && __ballot(active && Tw < s.K) != 0ull;

  uint32_t key[NCT][4];
  const float* arow = A_hat + row * s.K;
  // all tiles of the row are requested before the first is used (a tile past K re-reads the row's
  // first columns; its values are discarded), so no load sits behind a branch
  float4 vt[NCT];
#pragma unroll
  for (int ct = 0; ct < NCT; ++ct) {
    const int32_t c0 = 16 * ct + 4 * lg;
    vt[ct] = *reinterpret_cast<const float4*>(arow + (c0 < s.K ? c0 : 0));
  }
#pragma unroll
  for (int ct = 0; ct < NCT; ++ct) {
    const int32_t c0 = 16 * ct + 4 * lg;
    const float a[4] = {vt[ct].x, vt[ct].y, vt[ct].z, vt[ct].w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int32_t c = c0 + i;
      bool cand = c < ncand;  // ncand <= K
      if (sparse_cols && cand && Tw < s.K) cand = block_start(c + 1, Tw, s.K) > block_start(c, Tw, s.K);
      key[ct][i] = cand ? ordered_key(a[i]) : 0u;
    }
  }
  // largest tau with #{key >= tau} >= nsel, or any tau whose count is exactly nsel
  uint32_t tau = 0u, cge = 16u * NCT;  // every key is >= 0
#pragma unroll 1
  for (int bit = 31; bit >= 0; --bit) {
    const bool pend = cge != nsel && nsel != 0u;
    if (__ballot(pend) == 0ull) break;
    const uint32_t trial = tau | (1u << bit);
    uint32_t cnt = 0;
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
      for (int i = 0; i < 4; ++i) cnt += key[ct][i] >= trial ? 1u : 0u;
    cnt = rows_sum_u(cnt);
    const bool take = pend && cnt >= nsel;
    tau = take ? trial : tau;
    cge = take ? cnt : cge;
  }
  // nib[ct]: bit i set iff column 16 ct + 4 lg + i of this lane's row is selected
  uint32_t nib[NCT];
  const bool excess = cge != nsel && nsel != 0u;  // more keys than the quota tie at tau
  if (__ballot(excess) == 0ull) {
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
      uint32_t bits = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) bits |= (nsel != 0u && key[ct][i] >= tau) ? (1u << i) : 0u;
      nib[ct] = bits;
    }
  } else {
    uint32_t cgt = 0;
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
      for (int i = 0; i < 4; ++i) cgt += key[ct][i] > tau ? 1u : 0u;
    cgt = rows_sum_u(cgt);
    // rows without excess: every key >= tau is taken (cge == nsel, so need_eq covers all ties)
    int32_t need_eq = static_cast<int32_t>(nsel) - static_cast<int32_t>(cgt);
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
      uint32_t eqm = 0, gtm = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        eqm |= (key[ct][i] == tau && nsel != 0u) ? (1u << i) : 0u;
        gtm |= (key[ct][i] > tau && nsel != 0u) ? (1u << i) : 0u;
      }
      // columns ascend with (ct, lg, i): ties in lower lane groups of this tile come first
      uint32_t below;
      const uint32_t total = rows_sum_prefix_u(static_cast<uint32_t>(__popc(eqm)), lg, &below);
      uint32_t bits = gtm;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int32_t rank = static_cast<int32_t>(below) + __popc(eqm & ((1u << i) - 1u));
        if (((eqm >> i) & 1u) && rank < need_eq) bits |= 1u << i;
      }
      nib[ct] = bits;
      need_eq -= min(need_eq, static_cast<int32_t>(total));
    }
  }
  // word j holds columns 32 j .. 32 j + 31 = tiles 2 j (low half) and 2 j + 1; the four lanes of a
  // row combine their parts and lane group 0 stores them
  const int32_t kw = (s.K + 31) >> 5;
  constexpr int kWords = (NCT + 1) / 2;
  uint32_t words[kWords];
#pragma unroll
  for (int j = 0; j < kWords; ++j) {
    uint32_t part = nib[2 * j] << (4 * lg);
    if (2 * j + 1 < NCT) part |= nib[2 * j + 1] << (16 + 4 * lg);
    words[j] = rows_or_u(part);
  }
  if (lg != 0 || !in_head) return;
  uint32_t* mrow = mbits + row * kw;
#pragma unroll
  for (int j = 0; j < kWords; ++j)
    if (j < kw) mrow[j] = words[j];
}

// ------------------------------------------------------------------------------------------
// Causal-per-batch grouping (Sec. 3.1): A_hat is viewed as [T][H K]; each time step keeps the
// H k^ largest entries of its H x K slab.  One block per (batch element, time step); the slab
// (flattened index h K + c) is dealt to the threads in groups of four entries, group gi of thread
// tid starting at entry (gi 256 + tid) 4, so "lower flattened index first" among equal scores is
// (group, thread, slot) order.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t x) {
  x += static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), 0xB1, 0xf, 0xf, false));   // quad xor 1
  x += static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), 0x4E, 0xf, 0xf, false));   // quad xor 2
  x += static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), 0x141, 0xf, 0xf, false));  // row_half_mirror
  x += static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), 0x140, 0xf, 0xf, false));  // row_mirror
  x += __shfl_xor(x, 16, kWave);
  x += __shfl_xor(x, 32, kWave);
  return x;
}

template <int VPT>
__global__ __launch_bounds__(256) void topk_group_kernel(Shape s, const float* __restrict__ A_hat,
                                                         int32_t* __restrict__ sel,
                                                         int32_t* __restrict__ idx,
                                                         int32_t* __restrict__ cnt,
                                                         uint32_t* __restrict__ mbits) {
  __shared__ uint32_t red[2][4];
  __shared__ uint32_t scan[4];
  __shared__ uint32_t hist[2048];
  __shared__ uint32_t found[3];
  extern __shared__ uint8_t flags[];  // [H * K] selected?
  const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const int32_t t = static_cast<int32_t>(blockIdx.x % s.T);
  const int32_t b = static_cast<int32_t>(blockIdx.x / s.T);
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
  const int32_t HK = s.H * s.K;
  const int32_t kw = (s.K + 31) / 32;
  const bool active = t < len;
  const int32_t jmax = active ? ((s.causal && t < len - 1) ? t : len - 1) : -1;
  // per-row width geometry: the K columns are spread over the row's own t + 1 keys; when that is
  // fewer than K keys, only t + 1 of the columns hold one
  const int32_t Tw = s.geometry == 1 ? t + 1 : s.T;
  const int32_t ncand = active ? bucket_of(jmax, Tw, s.K) + 1 : 0;
  const bool holes = s.geometry == 1 && Tw < s.K;
  auto is_cand = [&](int32_t c) {
    return c < ncand && (!holes || block_start(c + 1, Tw, s.K) > block_start(c, Tw, s.K));
  };
  const int64_t quota = static_cast<int64_t>(s.H) * s.k_hat;
  const int64_t total = static_cast<int64_t>(s.H) * (holes ? min(Tw, ncand) : ncand);
  const uint32_t n = static_cast<uint32_t>(quota < total ? quota : total);

  // A thread owns VPT / 4 groups of four consecutive entries of the flattened slab: group gi of
  // thread tid starts at entry (gi * 256 + tid) * 4, so the lanes of a wave read consecutive 16-byte
  // pieces (full lines) and the flattened order is (group, thread, slot) order.
  uint32_t key[VPT];
  // head and column of the thread's first entry; a group further on is 1024 entries further on
  const int32_t adv_h = 1024 / s.K, adv_c = 1024 - adv_h * s.K;  // block-uniform
  int32_t gh = (tid * 4) / s.K, gc = tid * 4 - gh * s.K;
  if ((s.K & 3) == 0) {
    // the four entries of a group lie in one head: one 128-bit load.  All loads of the thread are
    // issued before the first is used: a group with nothing to read (past the slab, or past the
    // step's last candidate column) reads the first entries of the slab instead (always inside the
    // buffer), and its values are discarded, so no load sits behind a branch and none waits for
    // another.
    const float* slab = A_hat + (static_cast<int64_t>(b) * s.H * s.T + t) * s.K;  // head 0 of the step
    const int64_t hstride = static_cast<int64_t>(s.T) * s.K;
    // element offset of the thread's group inside the slab, stepped from group to group (one
    // 64-bit multiplication per thread instead of one per group)
    int64_t off = gh * hstride + gc;
    const int64_t adv_off = adv_h * hstride + adv_c, wrap_off = hstride - s.K;  // block-uniform
    // at most eight loads (32 registers) in flight: the largest slabs take two rounds
    constexpr int kBatch = VPT / 4 < 8 ? VPT / 4 : 8;
#pragma unroll
    for (int g0 = 0; g0 < VPT / 4; g0 += kBatch) {
      float4 f[kBatch];
      int32_t c0s[kBatch];
#pragma unroll
      for (int gj = 0; gj < kBatch; ++gj) {
        const int32_t e0 = ((g0 + gj) * 256 + tid) * 4;
        const bool ld = e0 < HK && gc < ncand;
        c0s[gj] = ld ? gc : s.K;  // s.K: no candidate in this group
        f[gj] = *reinterpret_cast<const float4*>(slab + (ld ? off : 0));
        gc += adv_c;
        off += adv_off;
        if (gc >= s.K) { gc -= s.K; off += wrap_off; }
      }
#pragma unroll
      for (int gj = 0; gj < kBatch; ++gj) {
        const float fv[4] = {f[gj].x, f[gj].y, f[gj].z, f[gj].w};
#pragma unroll
        for (int q = 0; q < 4; ++q) key[4 * (g0 + gj) + q] = is_cand(c0s[gj] + q) ? ordered_key(fv[q]) : 0u;
      }
    }
  } else {
#pragma unroll
    for (int gi = 0; gi < VPT / 4; ++gi) {
      const int32_t e0 = (gi * 256 + tid) * 4;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int32_t e = e0 + q;
        uint32_t k = 0u;
        if (e < HK) {
          const int32_t h = e / s.K, c = e - h * s.K;
          if (is_cand(c)) k = ordered_key(A_hat[((static_cast<int64_t>(b) * s.H + h) * s.T + t) * s.K + c]);
        }
        key[4 * gi + q] = k;
      }
    }
  }
  // n-th largest key of the slab.  Estimates take the radix selection below; the general bitwise
  // search keeps its counts on the vector units (per-thread compare-and-add, DPP row sums, two
  // cross-row exchanges, four partial sums through LDS).  Either stops as soon as exactly n keys
  // are >= tau.
  uint32_t tau = 0, c_ge = static_cast<uint32_t>(256 * VPT);
  // Scores of an estimate lie in [0, 2): their keys are 0x80000000 + (less than 2^30), so bits 31
  // and 30 of the threshold are known.  The n-th largest of up to 16 K keys is then found by radix
  // selection in three passes (11 + 11 + 8 bits): a histogram of the pass's digit over the keys that
  // still match the prefix (LDS atomics), a suffix count over the bins, the bin that holds the n-th
  // largest.  A pass ends the search early when the keys at or above its bin are exactly n.  Any
  // other input takes the general 32-bit bitwise search.
  bool in_range = true;
#pragma unroll
  for (int v = 0; v < VPT; ++v) in_range &= (key[v] == 0u) || ((key[v] >> 30) == 2u);
  const bool fast = __syncthreads_and(in_range ? 1 : 0) != 0;
  int bit = 31;
  if (n > 0 && fast) {
    tau = 0x80000000u;
    uint32_t pmask = 0xc0000000u, need = n, above = 0;  // keys above the prefix region so far
    c_ge = static_cast<uint32_t>(total);
    const int shifts[3] = {19, 8, 0}, widths[3] = {11, 11, 8};
#pragma unroll 1
    for (int pass = 0; pass < 3 && c_ge != n; ++pass) {
      const int shift = shifts[pass];
      const uint32_t nb = 1u << widths[pass];
      for (uint32_t x = tid; x < nb; x += 256) hist[x] = 0u;
      __syncthreads();
#pragma unroll
      for (int v = 0; v < VPT; ++v)
        // (a non-candidate's key is 0 and tau carries bit 31, so it never matches the prefix)
        if ((key[v] & pmask) == tau) atomicAdd(&hist[(key[v] >> shift) & (nb - 1u)], 1u);
      __syncthreads();
      // thread tid owns `per` consecutive bins; keys in higher bins = total - inclusive prefix
      const uint32_t per = nb >> 8;  // 8, 8, 1
      uint32_t mine = 0;
      for (uint32_t q = 0; q < per; ++q) mine += hist[tid * per + q];
      uint32_t incl = mine;
#pragma unroll
      for (int off = 1; off < kWave; off <<= 1) {
        const uint32_t o = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += o;
      }
      if (lane == kWave - 1) scan[wid] = incl;
      __syncthreads();
      uint32_t all = scan[0] + scan[1] + scan[2] + scan[3];
      for (int q = 0; q < wid; ++q) incl += scan[q];
      uint32_t g = all - incl;  // keys of the pass in bins above this thread's
      for (int32_t q = static_cast<int32_t>(per) - 1; q >= 0; --q) {
        const uint32_t c = hist[tid * per + q];
        if (g < need && g + c >= need) {
          found[0] = tid * per + q;
          found[1] = g;
          found[2] = c;
        }
        g += c;
      }
      __syncthreads();
      const uint32_t digit = found[0], gt = found[1], at = found[2];
      tau |= digit << shift;
      pmask |= (nb - 1u) << shift;
      c_ge = above + gt + at;  // keys >= the new prefix
      above += gt;
      need -= gt;
    }
    bit = -1;
  }
  if (n > 0) {
#pragma unroll 1
    for (; bit >= 0 && c_ge != n; --bit) {
      const uint32_t trial = tau | (1u << bit);
      uint32_t c = 0;
#pragma unroll
      for (int v = 0; v < VPT; ++v) c += (key[v] >= trial) ? 1u : 0u;
      c = wave_sum_u32(c);
      if (lane == 0) red[bit & 1][wid] = c;
      __syncthreads();  // the buffers alternate, so one barrier per step is enough
      const uint32_t ct = red[bit & 1][0] + red[bit & 1][1] + red[bit & 1][2] + red[bit & 1][3];
      if (ct >= n) { tau = trial; c_ge = ct; }
    }
  }
  __syncthreads();
  uint32_t c_gt = 0;
  if (c_ge == n) {
    c_gt = n;  // no excess ties at the threshold: every key >= tau is kept (counted as "greater")
  } else {
    uint32_t c = 0;
#pragma unroll
    for (int v = 0; v < VPT; ++v) c += (n > 0 && key[v] > tau) ? 1u : 0u;
    c = wave_sum_u32(c);
    if (lane == 0) red[0][wid] = c;
    __syncthreads();
    c_gt = red[0][0] + red[0][1] + red[0][2] + red[0][3];
  }
  const bool exact = (c_ge == n);   // block-uniform
  const uint32_t need_eq = n - c_gt;  // entries equal to tau that are kept, lowest flattened index first
  const bool want_lists = sel || idx || cnt;
  // 32 | K: the 32 entries of eight consecutive threads' groups are exactly one mask word
  const bool words_from_regs = (exact || n == 0) && mbits && (s.K & 31) == 0;
  if (exact || n == 0) {
    if (want_lists || (mbits && !words_from_regs)) {
#pragma unroll
      for (int v = 0; v < VPT; ++v) {
        const int32_t e = ((v >> 2) * 256 + tid) * 4 + (v & 3);
        if (e < HK) flags[e] = (n > 0 && key[v] >= tau) ? 1 : 0;
      }
    }
    if (words_from_regs) {
      // head and column of the thread's groups, stepped as when they were read
      // (32 | K and H K <= 16384, so a head's H T K / 32 words index with 32 bits)
      int32_t oh = (tid * 4) / s.K, oc = tid * 4 - oh * s.K;
      const int32_t hwords = s.T * kw;  // mask words of one head
      int32_t ow = oh * hwords;         // first word of the thread's head, inside the batch element
      uint32_t* mstep = mbits + (static_cast<int64_t>(b) * s.H * s.T + t) * kw;  // head 0, this step
#pragma unroll
      for (int gi = 0; gi < VPT / 4; ++gi) {
        const int32_t e0 = (gi * 256 + tid) * 4;
        uint32_t nib = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) nib |= (n > 0 && key[4 * gi + q] >= tau) ? (1u << q) : 0u;
        uint32_t word = nib << (4 * (lane & 7));
        word |= static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(word), 0xB1, 0xf, 0xf, false));
        word |= static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(word), 0x4E, 0xf, 0xf, false));
        word |= static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(word), 0x141, 0xf, 0xf, false));
        if ((lane & 7) == 0 && e0 < HK) mstep[ow + (oc >> 5)] = word;
        ow += adv_h * hwords;
        oc += adv_c;
        if (oc >= s.K) { oc -= s.K; ow += hwords; }
      }
    }
  } else {
    // ties at the threshold: walk the groups in flattened order, each with an exclusive prefix over
    // the threads of its number of entries equal to tau
    uint32_t base = 0;
#pragma unroll 1
    for (int gi = 0; gi < VPT / 4; ++gi) {
      uint32_t my_eq = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) my_eq += (key[4 * gi + q] == tau) ? 1u : 0u;
      uint32_t incl = my_eq;
#pragma unroll
      for (int off = 1; off < kWave; off <<= 1) {
        const uint32_t o = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += o;
      }
      if (lane == kWave - 1) scan[wid] = incl;
      __syncthreads();
      uint32_t before = base + incl - my_eq;
      for (int q = 0; q < wid; ++q) before += scan[q];
      base += scan[0] + scan[1] + scan[2] + scan[3];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int32_t e = (gi * 256 + tid) * 4 + q;
        const uint32_t ky = key[4 * gi + q];
        bool take = ky > tau;
        if (ky == tau) { take = before < need_eq; ++before; }
        if (e < HK) flags[e] = take ? 1 : 0;
      }
      __syncthreads();  // scan[] is rewritten by the next group
    }
  }
  __syncthreads();
  // packed mask words: word j of head h holds columns 32 j .. 32 j + 31
  if (mbits && !words_from_regs) {
    for (int32_t x = tid; x < s.H * kw; x += 256) {
      const int32_t h = x / kw, j = x - h * kw;
      uint32_t word = 0;
      for (int i = 0; i < 32; ++i) {
        const int32_t c = 32 * j + i;
        if (c < s.K && flags[h * s.K + c]) word |= 1u << i;
      }
      mbits[((static_cast<int64_t>(b) * s.H + h) * s.T + t) * kw + j] = word;
    }
  }
  // row lists on request: one thread walks one head
  if (sel || idx || cnt) {
    for (int32_t h = tid; h < s.H; h += 256) {
      const int64_t row = (static_cast<int64_t>(b) * s.H + h) * s.T + t;
      int32_t* srow = sel ? sel + row * s.sel_stride : nullptr;
      int32_t* irow = idx ? idx + row * s.L : nullptr;
      int32_t ns = 0, ni = 0;
      for (int32_t c = 0; c < ncand; ++c) {
        if (!flags[h * s.K + c]) continue;
        if (srow) srow[ns] = c;
        ++ns;
        const int32_t s0 = block_start(c, Tw, s.K);
        const int32_t w = block_start(c + 1, Tw, s.K) - s0;
        const int32_t r = min(w, s.rep_cap);
        for (int32_t i = 0; i < r; ++i) {
          const int32_t j = s0 + static_cast<int32_t>((static_cast<int64_t>(i) * w) / r);
          if (j <= jmax) {
            if (irow) irow[ni] = j;
            ++ni;
          }
        }
      }
      if (srow)
        for (int32_t x = ns; x < s.sel_stride; ++x) srow[x] = -1;
      if (irow)
        for (int32_t x = ni; x < s.L; ++x) irow[x] = -1;
      if (cnt) cnt[row] = ni;
    }
  }
}

// ------------------------------------------------------------------------------------------
// The selection of a row, expanded to one bit per key (Sec. 3.1 "Linear Sparse Attention Mask
// Generation", with App. A.4's per-row widths when geometry = 1; App. A.5.3 for the replication
// cap): bit j of row t is set iff key j belongs to a selected column of that row and is one of the
// r = min(w, cap) keys start + floor(i w / r) the column emits, j <= t (causal) and j < seq_len.
// One wavefront per row: lanes walk the K column bits, a selected column ORs its keys into the
// row's words in LDS, the words leave as one coalesced run.  kb: [N][T][KWk], KWk = ceil(T / 32).
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kWavesPerBlock* kWave) void keybits_kernel(Shape s, const uint32_t* __restrict__ mbits,
                                                                       uint32_t* __restrict__ kb, int32_t KWk) {
  __shared__ uint32_t words[kWavesPerBlock][kKeyBitWordsMax];
  const int wid = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const uint32_t bph = blocks_per_head(s.T, kWavesPerBlock);
  const uint32_t head = blockIdx.x / bph;
  const int32_t t = static_cast<int32_t>(blockIdx.x - head * bph) * kWavesPerBlock + wid;
  if (t >= s.T) return;  // whole wave leaves; only wave-level barriers below
  const int64_t row = static_cast<int64_t>(head) * s.T + t;
  const int32_t b = static_cast<int32_t>(head / static_cast<uint32_t>(s.H));
  const int32_t len = s.seq_len ? min(max(s.seq_len[b], 0), s.T) : s.T;
  const int32_t kw = (s.K + 31) / 32;
  for (int32_t x = lane; x < KWk; x += kWave) words[wid][x] = 0u;
  __builtin_amdgcn_wave_barrier();
  if (t < len) {
    const int32_t jmax = (s.causal && t < len - 1) ? t : len - 1;
    const int32_t Tw = s.geometry == 1 ? t + 1 : s.T;
    const uint32_t* mrow = mbits + row * kw;
    for (int32_t c = lane; c < s.K; c += kWave) {
      if (((mrow[c >> 5] >> (c & 31)) & 1u) == 0u) continue;
      or_column_keys(words[wid], c, Tw, s.K, s.rep_cap, jmax);
    }
  }
  __builtin_amdgcn_wave_barrier();
  for (int32_t x = lane; x < KWk; x += kWave) kb[row * KWk + x] = words[wid][x];
}

}  // namespace

bool keybits_supported(const Shape& s) { return (s.T + 31) / 32 <= kKeyBitWordsMax; }
size_t keybits_bytes(const Shape& s) {
  return static_cast<size_t>(s.N) * s.T * static_cast<size_t>((s.T + 31) / 32) * sizeof(uint32_t);
}
hipError_t launch_keybits(const Shape& s, const uint32_t* mbits, uint32_t* kb, hipStream_t st) {
  if (!keybits_supported(s)) return hipErrorNotSupported;
  const uint32_t grid = static_cast<uint32_t>(s.N) * blocks_per_head(s.T, kWavesPerBlock);
  StageScope scope(SEA_STAGE_TOPK_MASK, st);
  hipLaunchKernelGGL(keybits_kernel, dim3(grid), dim3(kWavesPerBlock * kWave), 0, st, s, mbits, kb, (s.T + 31) / 32);
  return hipGetLastError();
}

hipError_t launch_topk_mask(const Shape& s, const float* A_hat, int32_t* sel, int32_t* idx,
                            int32_t* cnt, uint32_t* mbits, hipStream_t st, uint32_t* kb) {
  if (kb && (!keybits_supported(s) || s.grouping != 0)) return hipErrorNotSupported;
  const int32_t KWk = (s.T + 31) / 32;
  const uint32_t grid = static_cast<uint32_t>(s.N) * blocks_per_head(s.T, kWavesPerBlock);
  const dim3 block(kWavesPerBlock * kWave);
  const int slots = (s.K + kWave - 1) / kWave;
  StageScope scope(SEA_STAGE_TOPK_MASK, st);
  if (s.grouping == 0 && mbits && !sel && !idx && !cnt && !kb && s.K <= 64 && s.K % 4 == 0) {
    // Only the bits are wanted and a row is short: 16 rows per wavefront.  (Measured against the
    // one-row-per-wavefront kernel below, which counts with ballots on the scalar unit: 0.033 against
    // 0.072 ms on 196 608 rows of K = 64, but no gain at K = 128 and 256, where the 2 K vector
    // compare-and-adds a step cost here weigh as much as its scalar counts.)
    const dim3 bgrid(static_cast<uint32_t>(s.N) * blocks_per_head(s.T, 16 * kWavesPerBlock));
#define SEA_TOPK_BITS(NCT_)                                                                          \
  do {                                                                                               \
    if (s.geometry == 1) hipLaunchKernelGGL((topk_bits_kernel<NCT_, true>), bgrid, block, 0, st, s, A_hat, mbits);  \
    else hipLaunchKernelGGL((topk_bits_kernel<NCT_, false>), bgrid, block, 0, st, s, A_hat, mbits);  \
  } while (0)
    if (s.K <= 32) SEA_TOPK_BITS(2);
    else SEA_TOPK_BITS(4);
#undef SEA_TOPK_BITS
    return hipGetLastError();
  }
  bool from_bits = false;
  if (s.grouping == 1) {
    // With a mask buffer at hand the slab kernel only selects; the lists are then written by the
    // per-row kernel from the bits (one wavefront per row instead of one thread per head).
    const bool lists = sel || idx || cnt;
    from_bits = lists && mbits;
    int32_t* const sel_g = from_bits ? nullptr : sel;
    int32_t* const idx_g = from_bits ? nullptr : idx;
    int32_t* const cnt_g = from_bits ? nullptr : cnt;
    const int32_t HK = s.H * s.K;
    const int vpt = (HK + 255) / 256;
    const dim3 ggrid(static_cast<uint32_t>(s.N / s.H) * s.T);
    const size_t shm = static_cast<size_t>(HK);
    if (vpt <= 4) hipLaunchKernelGGL(topk_group_kernel<4>, ggrid, block, shm, st, s, A_hat, sel_g, idx_g, cnt_g, mbits);
    else if (vpt <= 8) hipLaunchKernelGGL(topk_group_kernel<8>, ggrid, block, shm, st, s, A_hat, sel_g, idx_g, cnt_g, mbits);
    else if (vpt <= 16) hipLaunchKernelGGL(topk_group_kernel<16>, ggrid, block, shm, st, s, A_hat, sel_g, idx_g, cnt_g, mbits);
    else if (vpt <= 32) hipLaunchKernelGGL(topk_group_kernel<32>, ggrid, block, shm, st, s, A_hat, sel_g, idx_g, cnt_g, mbits);
    else if (vpt <= 64) hipLaunchKernelGGL(topk_group_kernel<64>, ggrid, block, shm, st, s, A_hat, sel_g, idx_g, cnt_g, mbits);
    else return hipErrorNotSupported;
    if (!from_bits) return hipGetLastError();
  }
#define SEA_TOPK(SL)                                                                                               \
  do {                                                                                                             \
    if (from_bits && s.geometry == 1)                                                                              \
      hipLaunchKernelGGL((topk_mask_kernel<SL, true, true>), dim3(grid), block, 0, st, s, A_hat, sel, idx, cnt,    \
                         mbits, kb, KWk);                                                                                   \
    else if (from_bits)                                                                                            \
      hipLaunchKernelGGL((topk_mask_kernel<SL, false, true>), dim3(grid), block, 0, st, s, A_hat, sel, idx, cnt,   \
                         mbits, kb, KWk);                                                                                   \
    else if (s.geometry == 1)                                                                                      \
      hipLaunchKernelGGL((topk_mask_kernel<SL, true, false>), dim3(grid), block, 0, st, s, A_hat, sel, idx, cnt,   \
                         mbits, kb, KWk);                                                                                   \
    else                                                                                                           \
      hipLaunchKernelGGL((topk_mask_kernel<SL, false, false>), dim3(grid), block, 0, st, s, A_hat, sel, idx, cnt,  \
                         mbits, kb, KWk);                                                                                   \
  } while (0)
  if (slots <= 1) SEA_TOPK(1);
  else if (slots <= 2) SEA_TOPK(2);
  else if (slots <= 4) SEA_TOPK(4);
  else if (slots <= 8) SEA_TOPK(8);
  else SEA_TOPK(16);
#undef SEA_TOPK
  return hipGetLastError();
}

}  // namespace sea

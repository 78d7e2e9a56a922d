// Tiled attention on the CDNA4 matrix cores, used for (a) the sparse attention stage of
// sea_forward when the mask has column structure (Sec. 3.1.1 rho, sigma, A* V with the mask of
// Sec. 3.1 "Linear Sparse Attention Mask Generation") and (b) the dense baseline
// softmax(QK^T)V (Sec. 3 "Preliminaries").
//
// Why tiles: every query row that selects compressed column c attends to the same r keys of
// that column, so the keys any row of a head can use form one fixed "compact" list of U = K r
// keys (all T keys when whole columns are emitted).  A wavefront takes 32 consecutive query
// rows and walks that list in chunks of 32 keys; a chunk no row of the tile selected is
// skipped, otherwise S^T = K_chunk Q_tile^T and O^T += V_chunk^T P^T run as
// v_mfma_f32_32x32x16_bf16 with per-(row, column) mask bits applied to S in registers.  K/V
// rows are thus read once per 32 query rows instead of once per row, and no T x T or T x L
// buffer exists.  The softmax is the streaming form; each lane owns one query (the MFMA
// output column), so row maxima and sums need a single cross-lane exchange.
//
// Operand layouts (32x32x16 bf16): A lane l = row l%32, contraction elems 8(l/32)..+7;
// B lane l = col l%32, same elems; C reg i = row 8(i/4) + 4(l/32) + i%4, col l%32.
// P leaves the first product in C layout (lane = query, regs = keys) and is fed back as the B
// operand of the second product; its register order fixes which key each contraction slot
// means, and the V^T fragments are fetched in that same order from LDS, where the value rows of a
// step are parked as they lie in memory and transposed on the way out by the LDS transpose read
// (the key and value rows themselves are gathered from K and V by position, so no compact or
// transposed copy exists in HBM).
#include "sea_internal.h"

namespace sea {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
// 64-bit LDS read with the 16-bit transpose across each group of 16 lanes (ds_read_b64_tr_b16)
__device__ __forceinline__ bf16x4 lds_transpose4(const uint16_t* p) {
  const shortx4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) shortx4*)(p));
  return __builtin_bit_cast(bf16x4, r);
}
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

struct TileArgs {
  const uint16_t* Q;    // [N][T][64]
  const uint16_t* K;    // [N][T][64]
  const uint16_t* V;    // [N][T][64]
  const uint32_t* mbits;  // [N][T][KW] selected-column bits, nullptr for dense
  uint16_t* O;          // [N][T][64]
  const int32_t* seq_len;
  int32_t N, H, T;
  int32_t U;            // compact keys per head: K r (all T keys when whole columns are emitted)
  int32_t KW;           // mask words per row
  int32_t rlog;         // log2(keys per column r)
  int32_t w;            // column width in keys
  int32_t causal;
  int32_t group_heads;  // heads per scheduling group (a multiple of 8 unless it is N)
  float c;              // scale * log2(e)
  // bucket mode (one selected column per row): rows grouped by their column
  const int32_t* perm;      // [N][entries] row id | slot << 24, bucket after bucket
  const int32_t* bstart;    // [N][K + 1] first perm slot of each column's bucket
  const int32_t* chunk_col; // [N][max_chunks] column of each 128-row chunk, -1 past the last
  const int32_t* cstart;    // [N][K + 1] first chunk of each column
  int32_t max_chunks, Kcols;
  int64_t perm_stride;  // entries per head in perm
  // several columns per row (2 <= k^ <= 8): each (row, selected column) pair is one bucket entry
  // whose normalised partial output and (reference maximum, sum) go here, merged per row later
  uint16_t* part_o;   // [N][T][slots][64] bf16, nullptr when k^ = 1
  float* part_ml;     // [N][T][slots][2]
  int32_t slots;
};

// combine a value with the one held by the same lane of the other 32-lane half of the wave
__device__ __forceinline__ float half_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// position in the sequence of compact key u
__device__ __forceinline__ int32_t pos_of(int32_t u, int32_t rlog, int32_t w) {
  const int32_t col = u >> rlog, i = u & ((1 << rlog) - 1);
  return col * w + ((i * w) >> rlog);
}

// number of compact keys with position <= jmax (positions ascend with u)
__device__ __forceinline__ int32_t compact_count(int32_t jmax, int32_t rlog, int32_t w) {
  if (jmax < 0) return 0;
  const int32_t col = jmax / w, delta = jmax - col * w;
  const int32_t r = 1 << rlog;
  const int32_t inside = min(r, ((delta + 1) * r + w - 1) / w);
  return col * r + inside;
}

// raw buffer resource, word 3: 32-bit data format, no swizzle; loads past num_records return zero
constexpr int kBufferFlags = 0x00020000;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 buffer_load16(__amdgpu_buffer_rsrc_t r, uint32_t byte_off) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, static_cast<int>(byte_off), 0, 0);
  return make_uint4(v[0], v[1], v[2], v[3]);
}

constexpr int kChunk = 64;   // keys staged in LDS per step (two 32-key MFMA sub-chunks)
constexpr int kKRow = 72;    // halfwords per staged K row: 128 B + 16 B pad, conflict-free b128 reads
constexpr int kVRow = 64;    // halfwords per staged V row: no padding; the 64-byte halves of rows 2, 3 (mod 4)
                             // are exchanged, which makes the four rows of a transpose read hit distinct banks

// Block = 4 waves = 128 consecutive query rows of one head (32 per wave).  The block walks the
// compact key list in steps of 64 keys; each step's K and V rows are fetched once with full-line
// 128-bit loads, parked in LDS (K as rows, V transposed; double buffered, one barrier per step)
// and read by all four waves as MFMA fragments.
// RLOG = log2(keys per column) for 1..16 keys per column, 5 for 32 or more (then a 32-key
// sub-chunk lies inside one column and the actual shift is a.rlog).
//
// MODE 0: rows in sequence order, per-(row, column) mask bits.  MODE 1: dense baseline (no mask
// bits).  MODE 2: "bucket" form for k^ = 1 -- every row selected exactly one column, rows are
// grouped by that column, and a block takes 128 rows of one bucket against the r keys of its
// column, so every visited tile is fully used no matter how scattered the choices are.
template <int RLOG, int MODE, int NW = 4>
__global__ __launch_bounds__(64 * NW, 16 / NW) void tile_attn_kernel(TileArgs a) {
  // NW = waves per block: 4 (128 query rows) or 8 (256 rows sharing every staged key step, which
  // halves the bytes a head's keys and values travel from the L2s to LDS; two blocks per CU)
  static_assert(NW == 4 || NW == 8, "four or eight waves per block");
  static_assert(MODE != 2 || NW == 4, "bucket chunks are 128 rows");
  constexpr int kRows = 32 * NW, kThreads = 64 * NW;
  constexpr bool DENSE = MODE == 1 || MODE == 2;  // no per-column bits to look up
  constexpr bool BUCKET = MODE == 2;
  // MODE 3: one bit per (row, key) in HBM ([N][T][KW] words); a lane reads its row's two words of a
  // step straight from memory one step ahead, nothing of the mask is parked in LDS
  constexpr bool STREAM = MODE == 3;
  __shared__ __attribute__((aligned(16))) uint16_t Ks[2][kChunk * kKRow];
  __shared__ __attribute__((aligned(16))) uint16_t Vs[2][kChunk * kVRow];
  // selected-column bits of the 128 rows, (KW + 1) words per row (K <= 1024: at most 16.5 KB)
  extern __shared__ uint32_t Ms[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, keep it scalar
  const int ql = lane & 31, g = lane >> 5;
  const uint32_t wgs = (a.T + kRows - 1) / kRows;  // blocks per head
  int64_t head;
  int32_t wg_tile = 0, q0 = 0, t, eslot = 0;
  int32_t ubase = 0, ulim = a.U;  // compact keys this block may touch: [ubase, ulim)
  if (BUCKET) {
    head = blockIdx.x / static_cast<uint32_t>(a.max_chunks);
    const int32_t chunk = static_cast<int32_t>(blockIdx.x % static_cast<uint32_t>(a.max_chunks));
    const int32_t col = a.chunk_col[head * a.max_chunks + chunk];
    if (col < 0) return;  // past the last chunk of this head (block-uniform)
    const int32_t* bs = a.bstart + head * (a.Kcols + 1);
    const int32_t slot = bs[col] + (chunk - a.cstart[head * (a.Kcols + 1) + col]) * 128 + 32 * wid + ql;
    const int32_t entry = slot < bs[col + 1] ? a.perm[head * a.perm_stride + slot] : -1;
    t = entry < 0 ? -1 : (entry & 0xffffff);
    eslot = entry < 0 ? 0 : (entry >> 24);
    ubase = col << a.rlog;
    ulim = ubase + (1 << a.rlog);
  } else {
    // Launch order = longest first: heads are taken in groups whose keys and values fit the L2s;
    // inside a group the row tiles go from the last (most keys, causal) to the first, heads
    // fastest.  Blocks are dealt round-robin to the 8 XCDs, so with 8 | group size a head stays on
    // one XCD, and blocks that start late are the short ones that fill the gaps.
    const uint32_t per_group = static_cast<uint32_t>(a.group_heads) * wgs;
    const uint32_t grp = blockIdx.x / per_group, rem = blockIdx.x - grp * per_group;
    const uint32_t nh = min(static_cast<uint32_t>(a.group_heads), static_cast<uint32_t>(a.N) - grp * a.group_heads);
    head = static_cast<int64_t>(grp) * a.group_heads + rem % nh;
    wg_tile = static_cast<int32_t>(wgs - 1 - rem / nh);
    q0 = wg_tile * kRows + 32 * wid;  // first row of this wave
    t = q0 + ql;
  }
  const int32_t b = static_cast<int32_t>(head / a.H);
  const int32_t len = a.seq_len ? min(max(a.seq_len[b], 0), a.T) : a.T;
  const bool row_active = t >= 0 && t < len;
  const int32_t tq = min(max(t, 0), a.T - 1);

  const uint16_t* Qr = a.Q + (head * a.T + tq) * kHeadDim + 8 * g;
  bf16x8 bq[4];
#pragma unroll
  for (int kc = 0; kc < 4; ++kc) bq[kc] = *reinterpret_cast<const bf16x8*>(Qr + 16 * kc);
  // Re-define the fragments through an empty asm: inside the loop they then count as plain
  // register values, not as results of memory loads the loop's own prefetch could be queued behind.
#pragma unroll
  for (int kc = 0; kc < 4; ++kc) asm volatile("" : "+v"(bq[kc]));

  const uint16_t* Kh = a.K + head * static_cast<int64_t>(a.T) * kHeadDim;
  const uint16_t* Vh = a.V + head * static_cast<int64_t>(a.T) * kHeadDim;
  // mask words of the block's rows -> LDS (row stride KW + 1 words: conflict-free per-row reads)
  const int mstride = a.KW + 1;
  if (!DENSE && !STREAM) {
    const int32_t row0 = wg_tile * kRows;
    const uint32_t* msrc = a.mbits + (head * a.T + row0) * a.KW;
    const int32_t nwords = min(kRows, a.T - row0) * a.KW;
    for (int32_t x = tid; x < kRows * a.KW; x += kThreads) {
      const int32_t r = x / a.KW, wi = x - r * a.KW;
      Ms[r * mstride + wi] = x < nwords ? msrc[x] : 0u;
    }
  }
  const uint32_t* mrow = (DENSE || STREAM) ? nullptr : &Ms[(32 * wid + ql) * mstride];
  const uint32_t* krow = STREAM ? a.mbits + (head * a.T + tq) * a.KW : nullptr;
  uint32_t mw0 = 0u, mw1 = 0u, mn0 = 0u, mn1 = 0u;  // the row's words of this step and of the next
  auto fetch_words = [&](int32_t step_, uint32_t& w0, uint32_t& w1) {
    const int32_t wi = 2 * step_;
    w0 = (row_active && wi < a.KW) ? krow[wi] : 0u;
    w1 = (row_active && wi + 1 < a.KW) ? krow[wi + 1] : 0u;
  };

  // keys the block / this wave can see: position <= min(last row, len - 1) when causal
  int32_t u_end_wg, u_end, j_free;
  if (BUCKET) {
    u_end_wg = u_end = ulim;
    // rows of a bucket come from anywhere in the sequence: positions are compared only in the
    // sub-chunks that reach past the earliest limit among the wave's rows
    int32_t jm = row_active ? (a.causal ? min(t, len - 1) : len - 1) : 0x7fffffff;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) jm = min(jm, __shfl_xor(jm, off, 64));
    j_free = jm;
  } else {
    const int32_t wg_hi = min(wg_tile * kRows + kRows - 1, a.T - 1);
    u_end_wg = compact_count(a.causal ? min(wg_hi, len - 1) : len - 1, a.rlog, a.w);
    const int32_t t_hi = min(q0 + 31, a.T - 1);
    u_end = q0 < a.T ? compact_count(a.causal ? min(t_hi, len - 1) : len - 1, a.rlog, a.w) : 0;
    // below this position every key is admissible for every active row of the wave
    j_free = a.causal ? min(q0, len - 1) : len - 1;
  }
  const int32_t my_jmax = a.causal ? min(t, len - 1) : len - 1;
  // compact keys this row may attend: those of the block's range whose position is <= my_jmax
  const int32_t my_ucount = min(ulim, compact_count(row_active ? my_jmax : -1, a.rlog, a.w));
  const int32_t nsteps = (u_end_wg - ubase + kChunk - 1) / kChunk;

  // staging roles: 16-byte part tid & 7 of the K and V rows (tid >> 3) and, with four waves,
  // (tid >> 3) + 32 of the step (eight waves cover the 64 rows in one go).  V is parked as it lies in memory; the product reads it through the LDS transpose read.
  // Slots past the list re-read its last key; their scores are masked.
  const int srow = tid >> 3, spart = tid & 7;
  const int vpart = spart ^ (((srow >> 1) & 1) << 2);  // V rows 2, 3 (mod 4): halves exchanged
  uint4 kreg0, kreg1 = {0u, 0u, 0u, 0u}, vreg0, vreg1 = {0u, 0u, 0u, 0u};
  // With at most 64 keys per column a step of 64 compact keys advances every slot's position by
  // the same amount, so the four row offsets (bytes inside the head, 32 bits) just step by a
  // constant; they are clamped to the last row, since slots past the list only need an address
  // that is in bounds.  Steps are fetched in order, one SEA_FETCH per step.
  const bool linear = a.rlog <= 6;
  const uint32_t row_bytes = kHeadDim * 2, part_bytes = spart * 16;
  const uint32_t off_max = static_cast<uint32_t>(a.T - 1) * row_bytes + part_bytes;
  const uint32_t off_step = linear ? static_cast<uint32_t>((kChunk >> a.rlog) * a.w) * row_bytes : 0u;
  uint32_t offa = static_cast<uint32_t>(pos_of(ubase + srow, a.rlog, a.w)) * row_bytes + part_bytes;
  uint32_t offb = static_cast<uint32_t>(pos_of(ubase + srow + 32, a.rlog, a.w)) * row_bytes + part_bytes;
  // The head's keys and values as buffer resources (base in scalar registers, 32-bit byte offset
  // per lane): a staging load then needs no 64-bit address arithmetic on the vector pipe.
  const uint32_t head_bytes = static_cast<uint32_t>(a.T) * row_bytes;
  const __amdgpu_buffer_rsrc_t Kres = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(Kh), 0, head_bytes, kBufferFlags);
  const __amdgpu_buffer_rsrc_t Vres = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(Vh), 0, head_bytes, kBufferFlags);
#define SEA_SLOT_OFF(slot_, step_)                                                                   \
  (static_cast<uint32_t>(pos_of(min(ubase + (step_) * kChunk + (slot_), a.U - 1), a.rlog, a.w)) * row_bytes + part_bytes)
#define SEA_FETCH(step_)                                                                             \
  do {                                                                                               \
    if (!linear) {                                                                                   \
      offa = SEA_SLOT_OFF(srow, step_);                                                              \
      if (NW == 4) offb = SEA_SLOT_OFF(srow + 32, step_);                                            \
    }                                                                                                \
    kreg0 = buffer_load16(Kres, min(offa, off_max));                                                 \
    if (NW == 4) kreg1 = buffer_load16(Kres, min(offb, off_max));                                    \
    vreg0 = buffer_load16(Vres, min(offa, off_max));                                                 \
    if (NW == 4) vreg1 = buffer_load16(Vres, min(offb, off_max));                                    \
    offa += off_step; offb += off_step;                                                              \
  } while (0)
#define SEA_PARK(stage_)                                                                             \
  do {                                                                                               \
    *reinterpret_cast<uint4*>(&Ks[stage_][srow * kKRow + spart * 8]) = kreg0;                         \
    if (NW == 4) *reinterpret_cast<uint4*>(&Ks[stage_][(srow + 32) * kKRow + spart * 8]) = kreg1;     \
    *reinterpret_cast<uint4*>(&Vs[stage_][srow * kVRow + vpart * 8]) = vreg0;                         \
    if (NW == 4) *reinterpret_cast<uint4*>(&Vs[stage_][(srow + 32) * kVRow + vpart * 8]) = vreg1;     \
  } while (0)

  floatx16 oacc[2];
#pragma unroll
  for (int i = 0; i < 16; ++i) { oacc[0][i] = 0.f; oacc[1][i] = 0.f; }
  // Streaming softmax in the exponent's own units: a score enters as y = s c - m_ref (log2 units,
  // one fused multiply-add with the group's offset, -inf for a masked group), so the row maximum
  // is the plain maximum of y and no score is touched twice.
  // m_thr = how far a row's maximum may exceed its reference: -inf until the row has one.  Both
  // halves of a row (lanes l, l + 32) always hold the same m_ref and m_thr.
  float m_ref = 0.f, m_thr = -INFINITY, l_run = 0.f;
  constexpr float kRefSlack = 8.f;

  if (nsteps > 0) {
    SEA_FETCH(0);
    SEA_PARK(0);
    if (STREAM) fetch_words(0, mn0, mn1);
  }
  __syncthreads();
  for (int32_t step = 0; step < nsteps; ++step) {
    const int stage = step & 1;
    if (step + 1 < nsteps) SEA_FETCH(step + 1);
    if (STREAM) {
      mw0 = mn0;
      mw1 = mn1;
      if (step + 1 < nsteps) fetch_words(step + 1, mn0, mn1);
    }
    // With two or more keys per column the (at most 32) columns of a 64-key step lie in one mask
    // word: it is read once per step, unconditionally (every row of the block has its words in
    // LDS), ahead of both sub-chunks instead of in front of each one's first fragment read.
    constexpr bool kStepWord = !DENSE && !STREAM && RLOG >= 1;
    uint32_t wstep = 0u;
    if (kStepWord) {
      wstep = mrow[((step * kChunk) >> (RLOG < 5 ? RLOG : a.rlog)) >> 5];
      wstep = row_active ? wstep : 0u;
    }
#pragma unroll
    for (int sc = 0; sc < 2; ++sc) {
      const int32_t u0 = ubase + step * kChunk + 32 * sc;
      if (u0 >= u_end) break;  // wave-uniform: beyond what this wave's rows can see
      if (BUCKET && __ballot(row_active) == 0ull) break;  // a wave past the end of its bucket
      uint32_t bits = 0xffffffffu;
      if (!DENSE) {
        const int32_t col0 = u0 >> (RLOG < 5 ? RLOG : a.rlog);  // first column of the sub-chunk
        const uint32_t word = STREAM ? (sc == 0 ? mw0 : mw1) : (kStepWord ? wstep : (row_active ? mrow[col0 >> 5] : 0u));
        bits = word >> (col0 & 31);
        constexpr uint32_t ncol = RLOG >= 5 ? 1u : (32u >> RLOG);
        constexpr uint32_t cmask = ncol >= 32 ? 0xffffffffu : ((1u << ncol) - 1u);
        if (__ballot((bits & cmask) != 0u) == 0ull) continue;  // no row of the wave uses it
      }
      // S^T sub-chunk = K (32 keys x 64) . Q_tile^T
      const uint16_t* Kr = &Ks[stage][(32 * sc + ql) * kKRow + 8 * g];
      floatx16 sv;
#pragma unroll
      for (int i = 0; i < 16; ++i) sv[i] = 0.f;
#pragma unroll
      for (int kc = 0; kc < 4; ++kc)
        sv = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(Kr + 16 * kc), bq[kc],
                                                     sv, 0, 0, 0);
      // admissibility of each (key, query) entry: reg i <-> key slot 8(i/4) + 4g + i%4.
      // Interior sub-chunks need only the column bits; the few that straddle the causal
      // diagonal or the end of the sequence also compare key positions.
      const bool boundary =
          (u0 + 32 > u_end) || (pos_of(min(u0 + 31, a.U - 1), a.rlog, a.w) > j_free);
      // Registers of one lane fall into groups that share a column (and so a mask bit): 4 for 4
      // or 8 keys per column, 8 for 16, all 16 for 32 or more and for the dense kernel.  One
      // bit-select per group picks its offset (-m_ref or -inf).
      constexpr int kGroup = DENSE ? 16 : (RLOG >= 5 ? 16 : (RLOG == 4 ? 8 : (RLOG >= 2 ? 4 : 1)));
      constexpr int kGroups = 16 / kGroup;
      float y[16];
      if (!boundary && kGroup > 1) {
        const uint32_t ref_bits = __float_as_uint(-m_ref), inf_bits = 0xff800000u;
#pragma unroll
        for (int gi = 0; gi < kGroups; ++gi) {
          const int col = DENSE ? 0 : (RLOG >= 5 ? 0 : (RLOG == 2 ? 2 * gi + g : gi));  // column of the group
          // all ones where the group's column is selected
          const uint32_t sel = DENSE ? (row_active ? ~0u : 0u)
                                     : static_cast<uint32_t>(static_cast<int32_t>(bits << (31 - col)) >> 31);
          const float off = __uint_as_float((sel & ref_bits) | (~sel & inf_bits));
#pragma unroll
          for (int e = 0; e < kGroup; ++e) y[kGroup * gi + e] = fmaf(sv[kGroup * gi + e], a.c, off);
        }
      } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int32_t slot = 8 * (i >> 2) + 4 * g + (i & 3);
          uint32_t okb = DENSE ? (row_active ? 1u : 0u) : ((bits >> (RLOG >= 5 ? 0 : (slot >> RLOG))) & 1u);
          // positions ascend with the compact index, so "position <= the row's last admissible
          // key" is "index below the row's count of such keys", taken once per row.  The variants
          // with one key per column walk this per-element path in every sub-chunk and have no
          // register left for that count: they compare positions.
          if (boundary) {
            if (kGroup > 1) {
              okb &= (u0 + slot < my_ucount) ? 1u : 0u;
            } else {
              const int32_t u = u0 + slot;
              const int32_t pu = pos_of(min(u, a.U - 1), a.rlog, a.w);
              okb &= (u < ulim ? 1u : 0u) & (pu <= my_jmax ? 1u : 0u);
            }
          }
          y[i] = okb ? fmaf(sv[i], a.c, -m_ref) : -INFINITY;
        }
      }
      // The V^T fragments of the sub-chunk are requested here, into the registers the raw scores
      // just left, so that their LDS latency lies under the softmax arithmetic below instead of in
      // front of the products that use them.  The LDS transpose read hands lane i of a 16-lane
      // group element i % 4 of the 8 bytes that lanes 4 e + i / 4 (e = 0..3) of the group point at:
      // with lane r pointing at dims 4 (r % 4) .. + 3 of key r / 4, lane i receives dim i of keys
      // 0..3 -- four consecutive keys of one dimension.  Lanes 8..15 of a group point at rows 2, 3
      // (mod 4), whose halves are stored exchanged.
      // (With the per-key mask words of MODE 3 in registers as well there is no room for that:
      // there the fragments are requested just before their products.)
      bf16x8 av[2][2];
      auto request_v = [&]() {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
          const uint16_t* Vr = &Vs[stage][(32 * sc + 4 * g + ((ql & 15) >> 2)) * kVRow +
                                          32 * (mt ^ ((ql >> 3) & 1)) + (ql & 16) + 4 * (ql & 3)];
#pragma unroll
          for (int c2 = 0; c2 < 2; ++c2) {
            const bf16x4 lo = lds_transpose4(Vr + (16 * c2) * kVRow);
            const bf16x4 hi = lds_transpose4(Vr + (16 * c2 + 8) * kVRow);
            av[mt][c2] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          }
        }
      };
      if (!STREAM) request_v();
      float ymax = fmaxf(fmaxf(y[0], y[1]), y[2]);
#pragma unroll
      for (int i = 3; i < 15; i += 2) ymax = fmaxf(fmaxf(ymax, y[i]), y[i + 1]);
      ymax = half_max(fmaxf(ymax, y[15]));
      // The reference only has to keep the exponentials in range, so it is moved (and the
      // accumulators rescaled) when some row's maximum exceeds it by more than 8 in the exponent,
      // or when the row has none yet; until then p may reach 256 instead of 1, which fp32 sums and
      // bf16 P carry as well.
      const bool refresh = ymax > m_thr;
      if (__ballot(refresh) != 0ull) {
        // rows that did not ask keep their reference (factor exactly 1): a row's arithmetic
        // never depends on the other rows of its wave
        const float delta = refresh ? ymax : 0.f;
        const float corr = (refresh && m_thr > 0.f) ? __builtin_amdgcn_exp2f(-delta) : 1.f;
        l_run *= corr;
#pragma unroll
        for (int i = 0; i < 16; ++i) { oacc[0][i] *= corr; oacc[1][i] *= corr; }
        m_ref += delta;
        m_thr = refresh ? kRefSlack : m_thr;
#pragma unroll
        for (int i = 0; i < 16; ++i) y[i] -= delta;
      }
      // P to bf16 (exp2(-inf) = 0 for masked entries); the row sum is taken over the rounded
      // values, the ones the product uses
      bf16x2 h[8];
      const bf16x2 ones = {static_cast<__bf16>(1.0f), static_cast<__bf16>(1.0f)};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const floatx2 f2 = {__builtin_amdgcn_exp2f(y[2 * e]), __builtin_amdgcn_exp2f(y[2 * e + 1])};
        h[e] = __builtin_convertvector(f2, bf16x2);
        l_run = __builtin_amdgcn_fdot2_f32_bf16(h[e], ones, l_run, false);
      }
      bf16x8 bp[2];
#pragma unroll
      for (int c2 = 0; c2 < 2; ++c2) {
        const bf16x4 lo = __builtin_shufflevector(h[4 * c2], h[4 * c2 + 1], 0, 1, 2, 3);
        const bf16x4 hi = __builtin_shufflevector(h[4 * c2 + 2], h[4 * c2 + 3], 0, 1, 2, 3);
        bp[c2] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
      // O^T += V^T P^T; V^T fragments in the key order of the P registers
      if (STREAM) request_v();
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int c2 = 0; c2 < 2; ++c2)
          oacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[mt][c2], bp[c2], oacc[mt], 0, 0, 0);
    }
    if (step + 1 < nsteps) SEA_PARK(stage ^ 1);
    __syncthreads();
  }
#undef SEA_FETCH
#undef SEA_SLOT_OFF
#undef SEA_PARK
  l_run = half_sum(l_run);
  if (t >= 0 && t < a.T) {
    const float inv = (row_active && l_run > 0.f) ? 1.f / l_run : 0.f;
    uint16_t* Or = a.O + (head * a.T + t) * kHeadDim;
    if (BUCKET && a.part_o) {
      const int64_t e = (head * a.T + t) * a.slots + eslot;
      Or = a.part_o + e * kHeadDim;
      if (g == 0) {
        a.part_ml[2 * e] = m_thr > 0.f ? m_ref : -INFINITY;
        a.part_ml[2 * e + 1] = row_active ? l_run : 0.f;
      }
    }
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        // regs 4 q4 .. 4 q4 + 3 <-> d = 32 mt + 8 q4 + 4 g + 0..3
        const floatx2 f01 = {oacc[mt][4 * q4] * inv, oacc[mt][4 * q4 + 1] * inv};
        const floatx2 f23 = {oacc[mt][4 * q4 + 2] * inv, oacc[mt][4 * q4 + 3] * inv};
        const bf16x2 h01 = __builtin_convertvector(f01, bf16x2), h23 = __builtin_convertvector(f23, bf16x2);
        *reinterpret_cast<bf16x4*>(Or + 32 * mt + 8 * q4 + 4 * g) = __builtin_shufflevector(h01, h23, 0, 1, 2, 3);
      }
  }
}

// ---- k^ = 1: group the rows of a head by the one column each selected (Sec. 3.1, App. A.5.3:
// the long-sequence regime where k K < T) ----
constexpr int kBucketRows = 256;

__global__ __launch_bounds__(256) void zero_i32_kernel(int32_t* __restrict__ p, int64_t n) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i < n) p[i] = 0;
}

// bucket sizes: every set mask bit of a row is one entry of that column's bucket
__global__ __launch_bounds__(kBucketRows) void bucket_count_kernel(const uint32_t* __restrict__ mbits,
                                                                   int32_t* __restrict__ cnt, int32_t T,
                                                                   int32_t KW, int32_t Kc, int32_t slots) {
  extern __shared__ int32_t hist[];  // Kc counters
  const int64_t head = blockIdx.y;
  const int32_t row = blockIdx.x * kBucketRows + threadIdx.x;
  for (int c = threadIdx.x; c < Kc; c += kBucketRows) hist[c] = 0;
  __syncthreads();
  if (row < T) {
    const uint32_t* mw = mbits + (head * T + row) * KW;
    int n = 0;  // a row has at most `slots` entries: further bits of a foreign mask are ignored
    auto take = [&](uint32_t word, int32_t j) {
      while (word != 0u && n < slots) {
        const int bit = __ffs(static_cast<int>(word)) - 1;
        word &= word - 1u;
        atomicAdd(&hist[32 * j + bit], 1);
        ++n;
      }
    };
    if ((KW & 3) == 0 && (reinterpret_cast<uintptr_t>(mbits) & 15) == 0) {  // rows of whole, aligned 16-byte pieces: one load per four words
      for (int32_t j = 0; j < KW; j += 4) {
        const uint4 w4 = *reinterpret_cast<const uint4*>(mw + j);
        take(w4.x, j); take(w4.y, j + 1); take(w4.z, j + 2); take(w4.w, j + 3);
      }
    } else {
      for (int32_t j = 0; j < KW; ++j) take(mw[j], j);
    }
  }
  __syncthreads();
  for (int c = threadIdx.x; c < Kc; c += kBucketRows)
    if (hist[c] != 0) atomicAdd(&cnt[head * Kc + c], hist[c]);
}

// per head: bucket offsets, the 128-row chunks of each bucket, and which column each chunk is
__global__ __launch_bounds__(1024) void bucket_scan_kernel(const int32_t* __restrict__ cnt,
                                                           int32_t* __restrict__ bstart,
                                                           int32_t* __restrict__ cstart,
                                                           int32_t* __restrict__ cursor,
                                                           int32_t* __restrict__ chunk_col, int32_t Kc,
                                                           int32_t max_chunks) {
  __shared__ int32_t rows_s[1024], chunks_s[1024];
  const int64_t head = blockIdx.x;
  const int c = threadIdx.x;
  const int32_t n = c < Kc ? cnt[head * Kc + c] : 0;
  const int32_t nch = (n + 127) >> 7;
  rows_s[c] = n;
  chunks_s[c] = nch;
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {  // inclusive scans
    const int32_t ar = c >= off ? rows_s[c - off] : 0, ac = c >= off ? chunks_s[c - off] : 0;
    __syncthreads();
    rows_s[c] += ar;
    chunks_s[c] += ac;
    __syncthreads();
  }
  const int32_t r0 = rows_s[c] - n, c0 = chunks_s[c] - nch;
  const int32_t total_chunks = chunks_s[1023];
  if (c < Kc) {
    bstart[head * (Kc + 1) + c] = r0;
    cstart[head * (Kc + 1) + c] = c0;
    cursor[head * Kc + c] = r0;
    for (int32_t j = 0; j < nch; ++j) chunk_col[head * max_chunks + c0 + j] = c;
  }
  if (c == 0) {
    bstart[head * (Kc + 1) + Kc] = rows_s[1023];
    cstart[head * (Kc + 1) + Kc] = total_chunks;
  }
  for (int32_t x = total_chunks + c; x < max_chunks; x += 1024) chunk_col[head * max_chunks + x] = -1;
}

// entries into their buckets (order inside a bucket is whatever the atomics give: no result
// depends on it).  An entry is the row id with, above bit 24, its rank among the row's selected
// columns.  With one column per row, rows that selected nothing (padding, no admissible key) get
// their zero output here; with several, the merge kernel writes every row.
constexpr int kMaxSlots = 8;
__global__ __launch_bounds__(kBucketRows) void bucket_scatter_kernel(const uint32_t* __restrict__ mbits,
                                                                     int32_t* __restrict__ cursor,
                                                                     int32_t* __restrict__ perm,
                                                                     uint16_t* __restrict__ O_zero, int32_t T,
                                                                     int32_t KW, int32_t Kc, int64_t perm_stride,
                                                                     int32_t slots) {
  extern __shared__ int32_t hist[];  // Kc counters, then Kc bases
  int32_t* base = hist + Kc;
  const int64_t head = blockIdx.y;
  const int32_t row = blockIdx.x * kBucketRows + threadIdx.x;
  for (int c = threadIdx.x; c < Kc; c += kBucketRows) hist[c] = 0;
  __syncthreads();
  int32_t cols[kMaxSlots], ranks[kMaxSlots];
  int n = 0;
  if (row < T) {
    const uint32_t* mw = mbits + (head * T + row) * KW;
    auto take = [&](uint32_t word, int32_t j) {
      while (word != 0u && n < slots) {
        const int bit = __ffs(static_cast<int>(word)) - 1;
        word &= word - 1u;
        const int32_t col = 32 * j + bit;
        const int32_t rank = atomicAdd(&hist[col], 1);
#pragma unroll
        for (int q = 0; q < kMaxSlots; ++q)
          if (q == n) { cols[q] = col; ranks[q] = rank; }
        ++n;
      }
    };
    if ((KW & 3) == 0 && (reinterpret_cast<uintptr_t>(mbits) & 15) == 0) {  // rows of whole, aligned 16-byte pieces: one load per four words
      for (int32_t j = 0; j < KW; j += 4) {
        const uint4 w4 = *reinterpret_cast<const uint4*>(mw + j);
        take(w4.x, j); take(w4.y, j + 1); take(w4.z, j + 2); take(w4.w, j + 3);
      }
    } else {
      for (int32_t j = 0; j < KW; ++j) take(mw[j], j);
    }
  }
  __syncthreads();
  for (int c = threadIdx.x; c < Kc; c += kBucketRows)
    base[c] = hist[c] != 0 ? atomicAdd(&cursor[head * Kc + c], hist[c]) : 0;
  __syncthreads();
#pragma unroll
  for (int q = 0; q < kMaxSlots; ++q)
    if (q < n) perm[head * perm_stride + base[cols[q]] + ranks[q]] = row | (q << 24);
  if (O_zero && n == 0 && row < T) {
    uint4* o = reinterpret_cast<uint4*>(O_zero + (head * T + row) * kHeadDim);
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = make_uint4(0u, 0u, 0u, 0u);
  }
}

// several columns per row: O[t] = sum_s w_s On_s / sum_s w_s with w_s = l_s 2^(m_s - M), over the
// row's entries (On_s normalised partial outputs, m_s references in log2 units, l_s sums)
__global__ __launch_bounds__(256) void bucket_merge_kernel(const uint32_t* __restrict__ mbits,
                                                           const uint16_t* __restrict__ part_o,
                                                           const float* __restrict__ part_ml,
                                                           uint16_t* __restrict__ O, int64_t rows, int32_t KW,
                                                           int32_t slots) {
  const int64_t gid = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  const int64_t row = gid >> 3;
  const int part = static_cast<int>(gid & 7);
  if (row >= rows) return;
  int n = 0;
  for (int32_t j = 0; j < KW; ++j) n += __popc(mbits[row * KW + j]);
  n = min(n, slots);
  // all of the row's entries are requested before any is used
  float ms[kMaxSlots], ls[kMaxSlots];
  uint4 vs[kMaxSlots];
  float M = -INFINITY;
#pragma unroll
  for (int q = 0; q < kMaxSlots; ++q) {
    const int64_t e = row * slots + min(q, max(n - 1, 0));
    ms[q] = part_ml[2 * e];
    ls[q] = q < n ? part_ml[2 * e + 1] : 0.f;
    vs[q] = *reinterpret_cast<const uint4*>(part_o + e * kHeadDim + part * 8);
    if (q < n) M = fmaxf(M, ms[q]);
  }
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float wsum = 0.f;
#pragma unroll
  for (int q = 0; q < kMaxSlots; ++q) {
    if (!(ls[q] > 0.f)) continue;
    const float wq = ls[q] * __builtin_amdgcn_exp2f(ms[q] - M);
    const uint32_t wds[4] = {vs[q].x, vs[q].y, vs[q].z, vs[q].w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      acc[2 * i] = fmaf(wq, bf16lo_to_f32(wds[i]), acc[2 * i]);
      acc[2 * i + 1] = fmaf(wq, bf16hi_to_f32(wds[i]), acc[2 * i + 1]);
    }
    wsum += wq;
  }
  const float inv = wsum > 0.f ? 1.f / wsum : 0.f;
  uint4 o;
  o.x = pack_bf16(acc[0] * inv, acc[1] * inv);
  o.y = pack_bf16(acc[2] * inv, acc[3] * inv);
  o.z = pack_bf16(acc[4] * inv, acc[5] * inv);
  o.w = pack_bf16(acc[6] * inv, acc[7] * inv);
  *reinterpret_cast<uint4*>(O + row * kHeadDim + part * 8) = o;
}

}  // namespace

// Heads per scheduling group: the keys and values (2 x U x 128 B per head) of the heads an
// XCD works on at one time should fit its 4 MB L2 with room to spare.
int32_t group_heads_for(int32_t N, int64_t U) {
  const int64_t per_head = 2 * U * kHeadDim * 2;
  int64_t per_xcd = (3 << 20) / (per_head > 0 ? per_head : 1);
  if (per_xcd < 1) per_xcd = 1;
  const int64_t g = 8 * per_xcd;
  return static_cast<int32_t>(g < N ? g : N);
}

#ifndef SEA_NW8_MIN_BLOCKS
#define SEA_NW8_MIN_BLOCKS 1024
#endif
// Dense baseline: eight-wave blocks (256 rows) when even those are at least two per block slot of
// the chip (2 per CU x 256 CUs); every staged key step then serves twice the rows (3-6 % at
// T = 32768).  The masked kernels keep four-wave blocks: interleaved on one box the wide form
// was within 1 % at T = 32768 and 4 % slower at T = 2048.
static bool wide_blocks(const Shape& s) {
  return static_cast<int64_t>(s.N) * ((s.T + 255) / 256) >= SEA_NW8_MIN_BLOCKS;
}

bool tile_attn_supported(const Shape& s, sea_dtype dt, int32_t* rlog_out) {
  if (dt != SEA_BF16 || s.T % s.K != 0) return false;
  if (s.geometry != 0) return false;  // a row's own column ranges: no structure shared between rows
  const int32_t w = s.T / s.K;
  const int32_t r = w < s.rep_cap ? w : s.rep_cap;
  if (r <= 0 || (r & (r - 1)) != 0) return false;
  int32_t rlog = 0;
  while ((1 << rlog) < r) ++rlog;
  if (static_cast<int64_t>(w) * r > (int64_t(1) << 30)) return false;
  if (s.T > (1 << 24)) return false;  // row offsets inside a head are 32-bit byte counts
  if (rlog_out) *rlog_out = rlog;
  return true;
}

namespace {
// Few columns per row under per-query grouping: rows (k^ = 1) or (row, column) entries (k^ <= 8,
// and no more than an eighth of the columns) are bucketed by column
bool bucket_mode(const Shape& s) {
  return s.grouping == 0 && (s.k_hat == 1 || (s.k_hat <= kMaxSlots && 8 * s.k_hat <= s.K));
}
size_t al256(size_t b) { return (b + 255) & ~size_t(255); }
struct BucketWs {
  size_t perm, cnt, cursor, bstart, cstart, chunk_col, part_o, part_ml, total;
  int64_t entries;      // perm slots per head
  int32_t max_chunks;
};
BucketWs bucket_layout(const Shape& s) {
  BucketWs b{};
  const size_t N = static_cast<size_t>(s.N);
  b.entries = static_cast<int64_t>(s.T) * s.k_hat;
  b.max_chunks = static_cast<int32_t>((b.entries + 127) / 128) + s.K;
  size_t off = 0;
  b.perm = off; off += al256(N * b.entries * 4);
  b.cnt = off; off += al256(N * s.K * 4);
  b.cursor = off; off += al256(N * s.K * 4);
  b.bstart = off; off += al256(N * (s.K + 1) * 4);
  b.cstart = off; off += al256(N * (s.K + 1) * 4);
  b.chunk_col = off; off += al256(N * b.max_chunks * 4);
  b.part_o = off; if (s.k_hat > 1) off += al256(N * b.entries * kHeadDim * 2);
  b.part_ml = off; if (s.k_hat > 1) off += al256(N * b.entries * 2 * 4);
  b.total = off;
  return b;
}
}  // namespace

// the tiled path reads K and V in place; only the bucket form needs scratch: the permutation,
// per-column counters / offsets / cursors, the chunk table and (several columns per row) the
// partial results
size_t tile_attn_workspace(const Shape& s) {
  if (!tile_attn_supported(s, SEA_BF16, nullptr) || !bucket_mode(s)) return 0;
  return bucket_layout(s).total;
}

hipError_t launch_tile_attn(const Shape& s, const uint16_t* Q, const uint16_t* K, const uint16_t* V,
                            const uint32_t* mbits, uint16_t* O, void* ws, hipStream_t st) {
  int32_t rlog = 0;
  if (!tile_attn_supported(s, SEA_BF16, &rlog)) return hipErrorNotSupported;
  const int32_t w = s.T / s.K, r = 1 << rlog;
  const int32_t U = s.K * r;
  if (bucket_mode(s)) {
    StageScope scope(SEA_STAGE_SPARSE, st);
    const BucketWs lay = bucket_layout(s);
    const int32_t KW = (s.K + 31) / 32;
    char* base = static_cast<char*>(ws);
    int32_t* perm = reinterpret_cast<int32_t*>(base + lay.perm);
    int32_t* cnt = reinterpret_cast<int32_t*>(base + lay.cnt);
    int32_t* cursor = reinterpret_cast<int32_t*>(base + lay.cursor);
    int32_t* bstart = reinterpret_cast<int32_t*>(base + lay.bstart);
    int32_t* cstart = reinterpret_cast<int32_t*>(base + lay.cstart);
    int32_t* chunk_col = reinterpret_cast<int32_t*>(base + lay.chunk_col);
    const bool multi = s.k_hat > 1;
    const int64_t ncnt = static_cast<int64_t>(s.N) * s.K;
    hipLaunchKernelGGL(zero_i32_kernel, dim3(static_cast<uint32_t>((ncnt + 255) / 256)), dim3(256), 0, st, cnt, ncnt);
    const dim3 rgrid((s.T + kBucketRows - 1) / kBucketRows, static_cast<uint32_t>(s.N));
    hipLaunchKernelGGL(bucket_count_kernel, rgrid, dim3(kBucketRows), s.K * sizeof(int32_t), st, mbits, cnt, s.T, KW,
                       s.K, s.k_hat);
    hipLaunchKernelGGL(bucket_scan_kernel, dim3(static_cast<uint32_t>(s.N)), dim3(1024), 0, st, cnt, bstart, cstart,
                       cursor, chunk_col, s.K, lay.max_chunks);
    hipLaunchKernelGGL(bucket_scatter_kernel, rgrid, dim3(kBucketRows), 2 * s.K * sizeof(int32_t), st, mbits, cursor,
                       perm, multi ? static_cast<uint16_t*>(nullptr) : O, s.T, KW, s.K, lay.entries, s.k_hat);
    TileArgs a{};
    a.Q = Q; a.K = K; a.V = V; a.mbits = nullptr; a.O = O; a.seq_len = s.seq_len;
    a.N = s.N; a.H = s.H; a.T = s.T; a.U = U; a.KW = 0; a.rlog = rlog; a.w = w; a.causal = s.causal;
    a.group_heads = s.N;
    a.c = s.scale * kLog2e;
    a.perm = perm; a.bstart = bstart; a.chunk_col = chunk_col; a.cstart = cstart;
    a.max_chunks = lay.max_chunks; a.Kcols = s.K; a.perm_stride = lay.entries;
    a.slots = s.k_hat;
    if (multi) {
      a.part_o = reinterpret_cast<uint16_t*>(base + lay.part_o);
      a.part_ml = reinterpret_cast<float*>(base + lay.part_ml);
    }
    const int32_t max_chunks = lay.max_chunks;
    hipLaunchKernelGGL((tile_attn_kernel<0, 2>), dim3(static_cast<uint32_t>(s.N) * max_chunks), dim3(256), 0, st, a);
    if (multi) {
      const int64_t rows = static_cast<int64_t>(s.N) * s.T;
      hipLaunchKernelGGL(bucket_merge_kernel, dim3(static_cast<uint32_t>((rows * 8 + 255) / 256)), dim3(256), 0, st,
                         mbits, a.part_o, a.part_ml, O, rows, KW, s.k_hat);
    }
    return hipGetLastError();
  }
  StageScope scope(SEA_STAGE_SPARSE, st);
  TileArgs a{};
  a.Q = Q; a.K = K; a.V = V; a.mbits = mbits; a.O = O; a.seq_len = s.seq_len;
  a.N = s.N; a.H = s.H; a.T = s.T; a.U = U; a.KW = (s.K + 31) / 32;
  a.rlog = rlog; a.w = w; a.causal = s.causal;
  a.group_heads = group_heads_for(s.N, U);
  a.c = s.scale * kLog2e;
  const dim3 grid(static_cast<uint32_t>(s.N) * ((s.T + 127) / 128)), block(256);
  const size_t shm = static_cast<size_t>(128) * (a.KW + 1) * sizeof(uint32_t);
  switch (rlog) {
    case 0: hipLaunchKernelGGL((tile_attn_kernel<0, 0>), grid, block, shm, st, a); break;
    case 1: hipLaunchKernelGGL((tile_attn_kernel<1, 0>), grid, block, shm, st, a); break;
    case 2: hipLaunchKernelGGL((tile_attn_kernel<2, 0>), grid, block, shm, st, a); break;
    case 3: hipLaunchKernelGGL((tile_attn_kernel<3, 0>), grid, block, shm, st, a); break;
    case 4: hipLaunchKernelGGL((tile_attn_kernel<4, 0>), grid, block, shm, st, a); break;
    default: hipLaunchKernelGGL((tile_attn_kernel<5, 0>), grid, block, shm, st, a); break;
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// fp32 tensors: the same walk over the compact key list on the fp64 / fp32 matrix cores.
// Block = 4 waves on the same 16 query rows; wave w takes the 16-key chunks c = w (mod 4) and the
// four partial results are merged through LDS (log-sum-exp weights).  Per chunk:
//   S^T (keys x queries) = K_c Q^T with v_mfma_f64_16x16x4_f64 (fp32 inputs widened, fp64 sums: the
//   precision contract of the fp32 mode), softmax weights in fp32 against a running reference,
//   O^T (dims x queries) += V_c^T P^T with v_mfma_f32_16x16x4_f32.
// Layouts: A lane l = A[row l % 16][k l / 16], B lane l = B[k l / 16][col l % 16]; the fp64 result
// register i is D[row 4 i + l / 16][col l % 16], the fp32 one D[row 4 (l / 16) + i][col l % 16].
// So a lane is one query (column); its four S^T registers are keys 4 i + g, g = l / 16, exactly the
// contraction slot (k = g of step i) the second product expects of P^T.  The contraction index of
// the first product is a free permutation of the 64 dims: step 4 j + e of lane group g is dim
// 16 j + 4 g + e, so Q and K rows are read as 16-byte pieces.
// ------------------------------------------------------------------------------------------
typedef double doublex4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

struct TileF32Args {
  const float* Q;
  const float* K;
  const float* V;
  const uint32_t* mbits;  // [N][T][KW]
  float* O;
  const int32_t* seq_len;
  int32_t N, H, T, U, KW, rlog, w, causal;
  double f;  // scale * log2(e)
};

__device__ __forceinline__ float rows_max_f(float x) {
  const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  const float y = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(y), __float_as_uint(y), false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float rows_sum_f(float x) {
  const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  const float y = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(y), __float_as_uint(y), false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

__global__ __launch_bounds__(256, 2) void tile_attn_f32_kernel(TileF32Args a) {
  __shared__ float m_s[4][16], l_s[4][16];
  __shared__ float o_s[4][kHeadDim][17];  // [wave][dim][query], padded
  __shared__ uint32_t mask_s[16 * 129];    // at most 128 mask words per row (K <= 1024 columns, or T <= 4096 keys)
  const int tid = threadIdx.x, lane = tid & 63;
  const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int qc = lane & 15, g = lane >> 4;
  const uint32_t tiles = (a.T + 15) / 16;
  // longest first: the last row tiles of every head come first
  const uint32_t tile = tiles - 1 - blockIdx.x / static_cast<uint32_t>(a.N);
  const int64_t head = blockIdx.x % static_cast<uint32_t>(a.N);
  const int32_t q0 = static_cast<int32_t>(tile) * 16;
  const int32_t t = q0 + qc;
  const int32_t b = static_cast<int32_t>(head / a.H);
  const int32_t len = a.seq_len ? min(max(a.seq_len[b], 0), a.T) : a.T;
  const bool row_active = t < len;
  const int32_t tq = min(t, a.T - 1);
  const float* Kh = a.K + head * static_cast<int64_t>(a.T) * kHeadDim;
  const float* Vh = a.V + head * static_cast<int64_t>(a.T) * kHeadDim;
  // selected-column bits of the tile's 16 rows -> LDS (row stride KW + 1 words)
  {
    const uint32_t* msrc = a.mbits + (head * a.T + q0) * a.KW;
    const int32_t nwords = min(16, a.T - q0) * a.KW;
    for (int32_t x = tid; x < 16 * a.KW; x += 256) {
      const int32_t r = x / a.KW, wi = x - r * a.KW;
      mask_s[r * (a.KW + 1) + wi] = x < nwords ? msrc[x] : 0u;
    }
  }
  __syncthreads();
  const uint32_t* mrow_s = &mask_s[qc * (a.KW + 1)];

  double qd[16];
  {
    const float* Qr = a.Q + (head * a.T + tq) * kHeadDim + 4 * g;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float4 v = *reinterpret_cast<const float4*>(Qr + 16 * j);
      qd[4 * j] = v.x; qd[4 * j + 1] = v.y; qd[4 * j + 2] = v.z; qd[4 * j + 3] = v.w;
    }
  }
  const int32_t my_jmax = a.causal ? min(t, len - 1) : len - 1;
  const int32_t t_hi = min(q0 + 15, a.T - 1);
  const int32_t u_end = compact_count(a.causal ? min(t_hi, len - 1) : len - 1, a.rlog, a.w);
  const int32_t nchunks = (u_end + 15) / 16;

  double m_run = -INFINITY;
  float l_run = 0.f;
  floatx4 o[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) o[dt] = floatx4{0.f, 0.f, 0.f, 0.f};

  // admissibility of this lane's four entries of chunk cc (keys 16 cc + 4 i + g) and their
  // positions; false when no row of the tile uses the chunk
  bool okn[4];
  int32_t pvn[4];
  auto probe = [&](int32_t cc) -> bool {
    bool any = false;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int32_t u = 16 * cc + 4 * i + g, uc = min(u, a.U - 1);
      const int32_t col = uc >> a.rlog;
      pvn[i] = pos_of(uc, a.rlog, a.w);
      okn[i] = row_active && u < a.U && ((mrow_s[col >> 5] >> (col & 31)) & 1u) != 0u && pvn[i] <= my_jmax;
      any = any || okn[i];
    }
    return __ballot(any) != 0ull;
  };
  // operands of chunk cc: K row of key 16 cc + qc (16-byte pieces at dims 16 j + 4 g), V entries
  // at dims 16 dt + qc of this lane's four keys
  float4 kfn[4];
  float vfn[4][4];
  auto request = [&](int32_t cc) {
    const float* Kr = Kh + static_cast<int64_t>(pos_of(min(16 * cc + qc, a.U - 1), a.rlog, a.w)) * kHeadDim + 4 * g;
#pragma unroll
    for (int j = 0; j < 4; ++j) kfn[j] = *reinterpret_cast<const float4*>(Kr + 16 * j);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) vfn[i][dt] = Vh[static_cast<int64_t>(pvn[i]) * kHeadDim + 16 * dt + qc];
  };

  int32_t c = wid;
  while (c < nchunks && !probe(c)) c += 4;
  if (c < nchunks) request(c);
  while (c < nchunks) {
    // take over the chunk that is on its way, then look for the next one and request it
    bool ok[4];
    float4 kf[4];
    float vf[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      ok[i] = okn[i];
      kf[i] = kfn[i];
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) vf[i][dt] = vfn[i][dt];
    }
    int32_t cn = c + 4;
    while (cn < nchunks && !probe(cn)) cn += 4;
    if (cn < nchunks) request(cn);
    c = cn;

    // two independent chains halve the latency of the 16 dependent products
    doublex4 acc0 = {0.0, 0.0, 0.0, 0.0}, acc1 = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int j = 0; j < 4; j += 2) {
      acc0 = __builtin_amdgcn_mfma_f64_16x16x4f64(static_cast<double>(kf[j].x), qd[4 * j], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f64_16x16x4f64(static_cast<double>(kf[j + 1].x), qd[4 * j + 4], acc1, 0, 0, 0);
      acc0 = __builtin_amdgcn_mfma_f64_16x16x4f64(static_cast<double>(kf[j].y), qd[4 * j + 1], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f64_16x16x4f64(static_cast<double>(kf[j + 1].y), qd[4 * j + 5], acc1, 0, 0, 0);
      acc0 = __builtin_amdgcn_mfma_f64_16x16x4f64(static_cast<double>(kf[j].z), qd[4 * j + 2], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f64_16x16x4f64(static_cast<double>(kf[j + 1].z), qd[4 * j + 6], acc1, 0, 0, 0);
      acc0 = __builtin_amdgcn_mfma_f64_16x16x4f64(static_cast<double>(kf[j].w), qd[4 * j + 3], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f64_16x16x4f64(static_cast<double>(kf[j + 1].w), qd[4 * j + 7], acc1, 0, 0, 0);
    }
    double y[4];
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      y[i] = ok[i] ? (acc0[i] + acc1[i]) * a.f : -INFINITY;
      mx = fmaxf(mx, static_cast<float>(y[i]));
    }
    // the reference only has to be common to the row's keys: an fp32 rounding of the maximum does
    mx = rows_max_f(mx);
    const double m_new = fmax(m_run, static_cast<double>(mx));
    if (__ballot(m_new != -INFINITY) == 0ull) continue;
    const double m_safe = (m_new == -INFINITY) ? 0.0 : m_new;
    const float corr = (m_run == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(static_cast<float>(m_run - m_safe));
    m_run = m_new;
    l_run *= corr;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int i = 0; i < 4; ++i) o[dt][i] *= corr;
    float pw[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      pw[i] = __builtin_amdgcn_exp2f(static_cast<float>(y[i] - m_safe));  // exp2(-inf) = 0 for masked entries
      l_run += pw[i];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) o[dt] = __builtin_amdgcn_mfma_f32_16x16x4f32(vf[i][dt], pw[i], o[dt], 0, 0, 0);
  }
  // merge the four waves: O = sum_w 2^(m_w - M) O_w / sum_w 2^(m_w - M) l_w.  m_run only ever takes
  // fp32 values (or -inf), so publishing it as fp32 loses nothing.
  l_run = rows_sum_f(l_run);
  if (g == 0) {
    m_s[wid][qc] = static_cast<float>(m_run);
    l_s[wid][qc] = l_run;
  }
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int i = 0; i < 4; ++i) o_s[wid][16 * dt + 4 * g + i][qc] = o[dt][i];
  __syncthreads();
  {
    const int q = tid & 15, dq = tid >> 4;  // query, quad of dims
    const int32_t tt = q0 + q;
    float M = fmaxf(fmaxf(m_s[0][q], m_s[1][q]), fmaxf(m_s[2][q], m_s[3][q]));
    float L = 0.f, acc4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float wgt = (m_s[w][q] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m_s[w][q] - M);
      L = fmaf(wgt, l_s[w][q], L);
#pragma unroll
      for (int e = 0; e < 4; ++e) acc4[e] = fmaf(wgt, o_s[w][4 * dq + e][q], acc4[e]);
    }
    if (tt < a.T) {
      const float inv = (tt < len && L > 0.f) ? 1.f / L : 0.f;
      *reinterpret_cast<float4*>(a.O + (head * a.T + tt) * kHeadDim + 4 * dq) =
          make_float4(acc4[0] * inv, acc4[1] * inv, acc4[2] * inv, acc4[3] * inv);
    }
  }
}

bool tile_attn_f32_supported(const Shape& s) {
  if (s.geometry != 0 || s.T % s.K != 0 || s.K > 1024) return false;  // the tile's mask words live in LDS
  const int32_t w = s.T / s.K;
  const int32_t r = w < s.rep_cap ? w : s.rep_cap;
  if (r <= 0 || (r & (r - 1)) != 0) return false;
  if (static_cast<int64_t>(w) * r > (int64_t(1) << 30)) return false;
  return true;
}

hipError_t launch_tile_attn_f32(const Shape& s, const float* Q, const float* K, const float* V,
                                const uint32_t* mbits, float* O, hipStream_t st) {
  if (!tile_attn_f32_supported(s)) return hipErrorNotSupported;
  const int32_t w = s.T / s.K, r = w < s.rep_cap ? w : s.rep_cap;
  int32_t rlog = 0;
  while ((1 << rlog) < r) ++rlog;
  StageScope scope(SEA_STAGE_SPARSE, st);
  TileF32Args a{};
  a.Q = Q; a.K = K; a.V = V; a.mbits = mbits; a.O = O; a.seq_len = s.seq_len;
  a.N = s.N; a.H = s.H; a.T = s.T; a.U = s.K * r; a.KW = (s.K + 31) / 32; a.rlog = rlog; a.w = w; a.causal = s.causal;
  a.f = static_cast<double>(s.scale) * 1.4426950408889634;
  const dim3 grid(static_cast<uint32_t>(s.N) * ((s.T + 15) / 16));
  hipLaunchKernelGGL(tile_attn_f32_kernel, grid, dim3(256), 0, st, a);
  return hipGetLastError();
}

// Masks without column structure shared by the rows (per-row width geometry): the selection
// arrives as one bit per (row, key), and the same kernel runs with every key its own "column"
// (one key per column, column width 1) -- the walk of the dense kernel with per-key mask bits,
// which every lane reads for its own row one step ahead (no mask words in LDS: four blocks per CU
// as in the other modes).  T <= 8192 is the limit of the kernels that write the bits (beyond it the
// quadratic walk also loses to per-row lists for the budgets in use); the fp32 kernel keeps the mask
// words of its 16 rows in LDS, 128 per row.
bool tile_attn_keybits_supported(const Shape& s, sea_dtype dt) { return s.T <= (dt == SEA_BF16 ? 8192 : 4096); }

// the same for fp32 tensors
hipError_t launch_tile_attn_f32_keybits(const Shape& s, const float* Q, const float* K, const float* V,
                                        const uint32_t* kb, float* O, hipStream_t st) {
  if (s.T > 4096) return hipErrorNotSupported;
  StageScope scope(SEA_STAGE_SPARSE, st);
  TileF32Args a{};
  a.Q = Q; a.K = K; a.V = V; a.mbits = kb; a.O = O; a.seq_len = s.seq_len;
  a.N = s.N; a.H = s.H; a.T = s.T; a.U = s.T; a.KW = (s.T + 31) / 32; a.rlog = 0; a.w = 1; a.causal = s.causal;
  a.f = static_cast<double>(s.scale) * 1.4426950408889634;
  const dim3 grid(static_cast<uint32_t>(s.N) * ((s.T + 15) / 16));
  hipLaunchKernelGGL(tile_attn_f32_kernel, grid, dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_tile_attn_keybits(const Shape& s, const uint16_t* Q, const uint16_t* K, const uint16_t* V,
                                    const uint32_t* kb, uint16_t* O, hipStream_t st) {
  if (!tile_attn_keybits_supported(s, SEA_BF16)) return hipErrorNotSupported;
  StageScope scope(SEA_STAGE_SPARSE, st);
  TileArgs a{};
  a.Q = Q; a.K = K; a.V = V; a.mbits = kb; a.O = O; a.seq_len = s.seq_len;
  a.N = s.N; a.H = s.H; a.T = s.T; a.U = s.T; a.KW = (s.T + 31) / 32; a.rlog = 0; a.w = 1; a.causal = s.causal;
  a.group_heads = group_heads_for(s.N, s.T);
  a.c = s.scale * kLog2e;
  const dim3 grid(static_cast<uint32_t>(s.N) * ((s.T + 127) / 128)), block(256);
  hipLaunchKernelGGL((tile_attn_kernel<0, 3>), grid, block, 0, st, a);
  return hipGetLastError();
}

size_t dense_attn_workspace(const Shape&) { return 0; }

hipError_t launch_dense_attn(const Shape& s, sea_dtype dt, const void* Q, const void* K, const void* V,
                             void* O, void* /*ws*/, hipStream_t st) {
  if (dt != SEA_BF16) return hipErrorNotSupported;
  StageScope scope(SEA_STAGE_DENSE, st);
  // dense: one "column" per key (r = 1, w = 1), so pos(u) = u
  TileArgs a{};
  a.Q = static_cast<const uint16_t*>(Q); a.K = static_cast<const uint16_t*>(K);
  a.V = static_cast<const uint16_t*>(V);
  a.mbits = nullptr; a.O = static_cast<uint16_t*>(O); a.seq_len = s.seq_len;
  a.N = s.N; a.H = s.H; a.T = s.T; a.U = s.T; a.KW = 0; a.rlog = 0; a.w = 1;
  a.causal = s.causal; a.c = s.scale * kLog2e;
  a.group_heads = group_heads_for(s.N, s.T);
  if (wide_blocks(s)) {
    const dim3 grid(static_cast<uint32_t>(s.N) * ((s.T + 255) / 256)), block(512);
    hipLaunchKernelGGL((tile_attn_kernel<0, 1, 8>), grid, block, 0, st, a);
    return hipGetLastError();
  }
  const dim3 grid(static_cast<uint32_t>(s.N) * ((s.T + 127) / 128)), block(256);
  hipLaunchKernelGGL((tile_attn_kernel<0, 1>), grid, block, 0, st, a);
  return hipGetLastError();
}

}  // namespace sea

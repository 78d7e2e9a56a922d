// Internal declarations shared by the HIP translation units of libsea_hip.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sea.h"

namespace sea {

constexpr int kWave = 64;
constexpr int kHeadDim = 64;
constexpr float kLog2e = 1.4426950408889634f;

// Shape block handed to kernels by value.
struct Shape {
  int32_t N;  // B * H heads
  int32_t H;
  int32_t T;
  int32_t m;
  int32_t K;
  int32_t k_hat;
  int32_t rep_cap;  // max keys per selected column (>= 1), INT32_MAX-like when uncapped
  int32_t L;        // row stride of idx
  int32_t causal;
  int32_t grouping;    // 0 per-query top-k^, 1 causal-per-batch
  int32_t sel_stride;  // columns one row can select: k_hat, or min(K, H k_hat) when grouped
  int32_t geometry;    // 0 fixed key buckets, 1 a causal row spreads its K columns over its own t + 1 keys
  int32_t cand_only;   // fused estimator: store A_hat only where a row has candidate columns (scratch A_hat
                       // that only the causal-per-batch selection reads); the rest stays unwritten
  float scale;
  const int32_t* seq_len;  // device [B] or nullptr
};

// ---- launchers (each enqueues on `st` and returns the launch error, if any) ----
hipError_t launch_estimate_f64(const Shape& s, const float* Q, const float* K, const float* W,
                               float* A_hat, void* ws, hipStream_t st);
size_t estimate_f64_workspace(const Shape& s);
hipError_t launch_features_f64(const Shape& s, const float* Q, const float* K, const float* W, double* phiQ,
                               double* phiK, hipStream_t st);

hipError_t launch_estimate_bf16(const Shape& s, const uint16_t* Q, const uint16_t* K,
                                const uint16_t* W, float* A_hat, void* ws, hipStream_t st);
size_t estimate_bf16_workspace(const Shape& s);
// fused two-kernel estimator for K | T, power-of-two column width, m in {64,128,256}, K <= 256
bool estimate_fused_supported(const Shape& s);
size_t estimate_fused_workspace(const Shape& s);
// A_hat and mbits ([N][T][ceil(K/32)] selected-column bits of the per-row top-k^) may each be
// nullptr; at least one should be given
hipError_t launch_estimate_fused(const Shape& s, const uint16_t* Q, const uint16_t* K, const uint16_t* W,
                                 float* A_hat, uint32_t* mbits, void* ws, hipStream_t st);

// per-row width geometry (causal, m in {64,128,256}); fp32 tensors: fp64 features, tiles on the fp64 matrix
// cores or a prefix table of phi(K); bf16 tensors: the bf16 matrix-core form below
bool estimate_rowwidth_supported(const Shape& s);
size_t estimate_rowwidth_workspace(const Shape& s, sea_dtype dt);
hipError_t launch_estimate_rowwidth(const Shape& s, sea_dtype dt, const void* Q, const void* K, const void* W,
                                    float* A_hat, void* ws, hipStream_t st);

// the same estimate for bf16 tensors on the bf16 matrix cores (features rounded to bf16, per-key products binned in LDS)
bool rowwidth_mfma_supported(const Shape& s, sea_dtype dt);
size_t rowwidth_mfma_workspace(const Shape& s);
hipError_t launch_rowwidth_mfma(const Shape& s, const uint16_t* Q, const uint16_t* K, const uint16_t* W,
                                float* A_hat, void* ws, hipStream_t st);

// sel, idx, cnt, mbits may each be nullptr; mbits is [N][T][ceil(K/32)] selected-column bits
// kb (per-query grouping, keybits_supported shapes only): also the selection expanded to one bit per key
hipError_t launch_topk_mask(const Shape& s, const float* A_hat, int32_t* sel, int32_t* idx,
                            int32_t* cnt, uint32_t* mbits, hipStream_t st, uint32_t* kb = nullptr);

// Tiled MFMA attention over the column-structured mask (bf16, K | T, power-of-two keys per column)
bool tile_attn_supported(const Shape& s, sea_dtype dt, int32_t* rlog_out);
size_t tile_attn_workspace(const Shape& s);
// a row's selection expanded to one bit per key ([N][T][ceil(T / 32)] words), for masks whose
// columns differ from row to row; the tiled attention then runs with keys as "columns"
bool keybits_supported(const Shape& s);
size_t keybits_bytes(const Shape& s);
hipError_t launch_keybits(const Shape& s, const uint32_t* mbits, uint32_t* kb, hipStream_t st);
bool tile_attn_keybits_supported(const Shape& s, sea_dtype dt);
hipError_t launch_tile_attn_keybits(const Shape& s, const uint16_t* Q, const uint16_t* K, const uint16_t* V,
                                    const uint32_t* kb, uint16_t* O, hipStream_t st);
hipError_t launch_tile_attn_f32_keybits(const Shape& s, const float* Q, const float* K, const float* V,
                                        const uint32_t* kb, float* O, hipStream_t st);
// fp32 tensors: tiled attention on the fp64 / fp32 matrix cores from per-row column bits
bool tile_attn_f32_supported(const Shape& s);
hipError_t launch_tile_attn_f32(const Shape& s, const float* Q, const float* K, const float* V,
                                const uint32_t* mbits, float* O, hipStream_t st);
hipError_t launch_tile_attn(const Shape& s, const uint16_t* Q, const uint16_t* K, const uint16_t* V,
                            const uint32_t* mbits, uint16_t* O, void* ws, hipStream_t st);
size_t dense_attn_workspace(const Shape& s);

// per-row lists (crow == nullptr: idx [N][T][L], cnt [N][T]) or the FlatCSR tensor (crow [B T + 1],
// idx = its column array, cnt and L unused)
hipError_t launch_sparse_attn(const Shape& s, sea_dtype dt, const void* Q, const void* K,
                              const void* V, const int32_t* idx, const int32_t* cnt, int32_t L,
                              const int64_t* crow, void* O, hipStream_t st);

// FlatCSR tensor from the per-row lists: crow [B T + 1], col [cap] (entries past cap are dropped)
size_t flatcsr_workspace(const Shape& s);
hipError_t launch_flatcsr(const Shape& s, const int32_t* idx, const int32_t* cnt, int32_t L, int64_t* crow,
                          int32_t* col, int64_t cap, void* ws, hipStream_t st);

hipError_t launch_dense_attn(const Shape& s, sea_dtype dt, const void* Q, const void* K,
                             const void* V, void* O, void* ws, hipStream_t st);

size_t output_mix_workspace(const Shape& s);
hipError_t launch_output_mix(const Shape& s, sea_dtype dt, const void* C, const void* V,
                             const float* A_hat, const float* s_prob, const float* s_mix, void* O,
                             void* ws, hipStream_t st);

// decoder path (bf16, m in {64,128,256}, even K, 8 | 4 H, fixed key buckets)
bool decoder_supported(const Shape& s, sea_dtype dt);
size_t decoder_workspace(const Shape& s);
hipError_t launch_decoder_estimate(const Shape& s, const sea_decoder_weights& wt, const uint16_t* Q, const uint16_t* K,
                                   const uint16_t* V, const uint16_t* W, float* A_hat, float* s_mix, float* s_prob,
                                   void* ws, hipStream_t st);

// ---- per-stage event timing (see sea_profile_enable) ----
void stage_begin(sea_stage stage, hipStream_t st);
void stage_end(sea_stage stage, hipStream_t st);
struct StageScope {
  sea_stage stage;
  hipStream_t st;
  StageScope(sea_stage s, hipStream_t t) : stage(s), st(t) { stage_begin(s, t); }
  ~StageScope() { stage_end(stage, st); }
};

// ---- device helpers ----
#if defined(__HIPCC__)

// Workgroup ids are dealt round-robin to the 8 XCDs.  Remap so that each XCD gets one
// contiguous range of logical tiles: rows of one head then share that XCD's L2.
__device__ __forceinline__ uint32_t xcd_contiguous(uint32_t bid, uint32_t nblocks) {
  constexpr uint32_t X = 8;
  const uint32_t per = nblocks / X, rem = nblocks % X;
  if (bid >= per * X) return bid;  // ragged tail stays in place
  (void)rem;
  const uint32_t xcd = bid % X, slot = bid / X;
  return xcd * per + slot;
}

__device__ __forceinline__ float bf16_to_f32(uint16_t h) {
  return __uint_as_float(static_cast<uint32_t>(h) << 16);
}
__device__ __forceinline__ float bf16lo_to_f32(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t pair) {
  return __uint_as_float(pair & 0xffff0000u);
}
// float -> bfloat16, round to nearest even: the hardware pair conversion (v_cvt_pk_bf16_f32)
typedef __bf16 sea_bf16x2 __attribute__((ext_vector_type(2)));
typedef float sea_floatx2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  const sea_floatx2 f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, sea_bf16x2));
}
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  return static_cast<uint16_t>(pack_bf16(f, 0.f) & 0xffffu);
}

// first key of column c: ceil(c T / K); column of key j: floor(j K / T)
__device__ __forceinline__ int32_t block_start(int32_t c, int32_t T, int32_t K) {
  return static_cast<int32_t>((static_cast<int64_t>(c) * T + K - 1) / K);
}
__device__ __forceinline__ int32_t bucket_of(int32_t j, int32_t T, int32_t K) {
  return static_cast<int32_t>((static_cast<int64_t>(j) * K) / T);
}

#endif  // __HIPCC__

}  // namespace sea

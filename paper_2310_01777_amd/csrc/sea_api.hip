// C ABI of libsea_hip.so: argument checks, parameter marshalling and stage dispatch.
// Every computation runs in the HIP kernels of the sibling translation units.
#include <limits.h>

#include <mutex>
#include <vector>

#include "sea_internal.h"

namespace sea {
namespace {

thread_local int g_last_hip_error = 0;

int fail_hip(hipError_t e) {
  g_last_hip_error = static_cast<int>(e);
  return SEA_EHIP;
}

// ---- profiling state (process-wide) ----
struct Span {
  sea_stage stage;
  hipEvent_t a, b;
};
unsigned g_profile = 0;  // bit per sea_stage
std::mutex g_profile_mutex;  // guards the span and event lists
std::vector<Span> g_spans;
std::vector<hipEvent_t> g_free_events;

hipEvent_t take_event() {
  if (!g_free_events.empty()) {
    hipEvent_t e = g_free_events.back();
    g_free_events.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

int check_common(const sea_params* p) {
  if (!p) return SEA_EINVAL;
  if (p->B <= 0 || p->H <= 0 || p->T <= 0 || p->d <= 0) return SEA_EINVAL;
  if (p->dtype != SEA_F32 && p->dtype != SEA_BF16) return SEA_EINVAL;
  if (static_cast<int64_t>(p->B) * p->H > INT32_MAX) return SEA_EINVAL;
  if (!(p->scale > 0.f) || !(p->scale < 1e30f)) return SEA_EINVAL;
  if (p->d != kHeadDim) return SEA_ENOTSUP;
  if (static_cast<int64_t>(p->B) * p->H * p->T > (int64_t(1) << 40)) return SEA_ENOTSUP;
  return SEA_OK;
}

int check_mask_params(const sea_params* p) {
  if (p->K <= 0 || p->K > p->T) return SEA_EINVAL;
  if (p->k_hat <= 0 || p->k_hat > p->K) return SEA_EINVAL;
  if (p->k_budget < 0) return SEA_EINVAL;
  if (p->grouping != 0 && p->grouping != 1) return SEA_EINVAL;
  if (p->K > 1024) return SEA_ENOTSUP;
  if (p->grouping == 1 && static_cast<int64_t>(p->H) * p->K > 16384) return SEA_ENOTSUP;
  if (p->geometry != 0 && p->geometry != 1) return SEA_EINVAL;
  if (p->geometry == 1 && !p->causal) return SEA_EINVAL;  // the row's own width is a causal notion
  return SEA_OK;
}

int check_estimate_params(const sea_params* p) {
  if (p->m <= 0) return SEA_EINVAL;
  if (p->m % 32 != 0 || p->m > 1024) return SEA_ENOTSUP;
  if (p->geometry == 1 && p->m != 64 && p->m != 128 && p->m != 256) return SEA_ENOTSUP;
  return SEA_OK;
}

int32_t rep_cap_of(const sea_params* p) {
  if (p->k_budget <= 0) return INT32_MAX;
  const int32_t cap = p->k_budget / p->k_hat;
  return cap < 1 ? 1 : cap;
}

int32_t sel_stride_of(const sea_params* p) {
  if (p->grouping == 0) return p->k_hat;
  const int64_t q = static_cast<int64_t>(p->H) * p->k_hat;
  return static_cast<int32_t>(q < p->K ? q : p->K);
}

int32_t row_stride_of(const sea_params* p) {
  const int32_t wmax = (p->T + p->K - 1) / p->K;
  const int32_t cap = rep_cap_of(p);
  const int64_t L = static_cast<int64_t>(sel_stride_of(p)) * (wmax < cap ? wmax : cap);
  return L > INT32_MAX ? -1 : static_cast<int32_t>(L);
}

Shape make_shape(const sea_params* p, bool with_mask) {
  Shape s{};
  s.N = p->B * p->H;
  s.H = p->H;
  s.T = p->T;
  s.m = p->m;
  s.K = p->K;
  s.k_hat = p->k_hat;
  s.causal = p->causal ? 1 : 0;
  s.grouping = p->grouping;
  s.geometry = p->geometry;
  s.sel_stride = sel_stride_of(p);
  s.scale = p->scale;
  s.seq_len = p->seq_len;
  if (with_mask) {
    s.rep_cap = rep_cap_of(p);
    s.L = row_stride_of(p);
  }
  return s;
}

size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

size_t estimate_ws(const sea_params* p) {
  const Shape s = make_shape(p, false);
  if (s.geometry == 1) return align256(estimate_rowwidth_workspace(s, p->dtype));
  return align256(p->dtype == SEA_BF16 ? estimate_bf16_workspace(s) : estimate_f64_workspace(s));
}

// the fused estimator keeps the scores in registers: no A_hat buffer unless the caller wants one
bool scores_stay_on_chip(const sea_params* p, const Shape& s) {
  return tile_attn_supported(s, p->dtype, nullptr) && estimate_fused_supported(s) && s.grouping == 0;
}

// Scratch of the whole forward pass: estimator scratch, A_hat, then either the tiled path's mask
// bits and bucket tables or the row-list path's idx + cnt.  `lean`: the caller keeps no
// intermediate, so the A_hat part is dropped where the scores stay on chip.
// per-row width geometry, sequences of at most 8192 (bf16) or 4096 (fp32) keys:
// the selection is expanded to one bit per key and the tiled attention kernel runs on those
bool keybit_path(const Shape& s, sea_dtype dt) {
  return s.geometry == 1 && keybits_supported(s) && tile_attn_keybits_supported(s, dt);
}

size_t forward_ws(const sea_params* p, bool lean) {
  const size_t rows = static_cast<size_t>(p->B) * p->H * p->T;
  const Shape s = make_shape(p, true);
  size_t bytes = estimate_ws(p);
  if (!(lean && scores_stay_on_chip(p, s))) bytes += align256(rows * p->K * sizeof(float));
  if (tile_attn_supported(s, p->dtype, nullptr)) {
    bytes += align256(rows * ((p->K + 31) / 32) * sizeof(uint32_t));
    bytes += align256(tile_attn_workspace(s));
  } else if (p->dtype == SEA_F32 && tile_attn_f32_supported(s)) {
    bytes += align256(rows * ((p->K + 31) / 32) * sizeof(uint32_t));
  } else if (keybit_path(s, p->dtype)) {
    bytes += align256(rows * ((p->K + 31) / 32) * sizeof(uint32_t));
    bytes += align256(keybits_bytes(s));
  } else {
    bytes += align256(rows * static_cast<size_t>(row_stride_of(p)) * sizeof(int32_t));
    bytes += align256(rows * sizeof(int32_t));
    if (p->grouping == 1) bytes += align256(rows * ((p->K + 31) / 32) * sizeof(uint32_t));
  }
  return bytes;
}

// ---- scratch of sea_forward_static: one array per GPU, alive until the process ends ----
constexpr size_t kStaticScratchBytes = size_t(64) << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each GPU, looked up once

// The array's name is only a host-side handle; kernels need the device address, which differs
// from GPU to GPU.  Looked up on first use with the caller's device current.
int static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip(e);
  if (dev < 0 || dev >= kMaxDevices) return SEA_ENOTSUP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return fail_hip(e);
    if (!ptr || reinterpret_cast<uintptr_t>(ptr) % 256 != 0) return SEA_EWORKSPACE;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return SEA_OK;
}

}  // namespace

void stage_begin(sea_stage stage, hipStream_t st) {
  if (!(g_profile & (1u << stage))) return;
  std::lock_guard<std::mutex> lock(g_profile_mutex);
  Span sp{stage, take_event(), take_event()};
  if (!sp.a || !sp.b) return;
  (void)hipEventRecord(sp.a, st);
  g_spans.push_back(sp);
}

void stage_end(sea_stage stage, hipStream_t st) {
  if (!(g_profile & (1u << stage))) return;
  std::lock_guard<std::mutex> lock(g_profile_mutex);
  if (g_spans.empty()) return;
  Span& sp = g_spans.back();
  if (sp.stage == stage) (void)hipEventRecord(sp.b, st);
}

}  // namespace sea

using namespace sea;

extern "C" {

int32_t sea_k_hat(int32_t k, int32_t K, int32_t T) {
  if (k <= 0 || K <= 0 || T <= 0) return SEA_EINVAL;
  const int64_t num = static_cast<int64_t>(k) * K;
  const int64_t r = (2 * num + T) / (2 * static_cast<int64_t>(T));
  return r < 1 ? 1 : static_cast<int32_t>(r > INT32_MAX ? INT32_MAX : r);
}

int32_t sea_sel_stride(const sea_params* p) {
  int rc = check_common(p);
  if (rc == SEA_OK) rc = check_mask_params(p);
  return rc != SEA_OK ? rc : sel_stride_of(p);
}

int32_t sea_row_stride(const sea_params* p) {
  int rc = check_common(p);
  if (rc == SEA_OK) rc = check_mask_params(p);
  if (rc != SEA_OK) return rc;
  const int32_t L = row_stride_of(p);
  return L < 0 ? SEA_ENOTSUP : L;
}

size_t sea_workspace_bytes(const sea_params* p) {
  if (check_common(p) != SEA_OK || check_mask_params(p) != SEA_OK ||
      check_estimate_params(p) != SEA_OK || row_stride_of(p) < 0)
    return 0;
  return forward_ws(p, false);
}

int sea_estimate(const sea_params* p, const void* Q, const void* K, const void* W, float* A_hat,
                 void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_common(p);
  if (rc == SEA_OK) rc = check_mask_params(p);
  if (rc == SEA_OK) rc = check_estimate_params(p);
  if (rc != SEA_OK) return rc;
  if (!Q || !K || !W || !A_hat) return SEA_EINVAL;
  if (!workspace || workspace_bytes < estimate_ws(p)) return SEA_EWORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return SEA_EWORKSPACE;
  const Shape s = make_shape(p, true);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  if (s.geometry == 1)
    e = launch_estimate_rowwidth(s, p->dtype, Q, K, W, A_hat, workspace, st);
  else if (p->dtype == SEA_BF16)
    e = launch_estimate_bf16(s, static_cast<const uint16_t*>(Q), static_cast<const uint16_t*>(K),
                             static_cast<const uint16_t*>(W), A_hat, workspace, st);
  else
    e = launch_estimate_f64(s, static_cast<const float*>(Q), static_cast<const float*>(K),
                            static_cast<const float*>(W), A_hat, workspace, st);
  return e == hipSuccess ? SEA_OK : fail_hip(e);
}

int sea_topk_mask(const sea_params* p, const float* A_hat, int32_t* sel, int32_t* idx,
                  int32_t* cnt, void* hip_stream) {
  int rc = check_common(p);
  if (rc == SEA_OK) rc = check_mask_params(p);
  if (rc != SEA_OK) return rc;
  if (!A_hat || !idx || !cnt) return SEA_EINVAL;
  if (row_stride_of(p) < 0) return SEA_ENOTSUP;
  const Shape s = make_shape(p, true);
  const hipError_t e =
      launch_topk_mask(s, A_hat, sel, idx, cnt, nullptr, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? SEA_OK : fail_hip(e);
}

int sea_sparse_attn(const sea_params* p, const void* Q, const void* K, const void* V,
                    const int32_t* idx, const int32_t* cnt, int32_t row_stride, void* O,
                    void* hip_stream) {
  const int rc = check_common(p);
  if (rc != SEA_OK) return rc;
  if (!Q || !K || !V || !idx || !cnt || !O || row_stride <= 0) return SEA_EINVAL;
  const Shape s = make_shape(p, false);
  const hipError_t e = launch_sparse_attn(s, p->dtype, Q, K, V, idx, cnt, row_stride, nullptr, O,
                                          static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? SEA_OK : fail_hip(e);
}

size_t sea_flatcsr_workspace_bytes(const sea_params* p) {
  if (check_common(p) != SEA_OK) return 0;
  return align256(flatcsr_workspace(make_shape(p, false)));
}

int sea_flatcsr(const sea_params* p, const int32_t* idx, const int32_t* cnt, int32_t row_stride,
                int64_t* crow, int32_t* col, int64_t col_capacity, void* workspace, size_t workspace_bytes,
                void* hip_stream) {
  const int rc = check_common(p);
  if (rc != SEA_OK) return rc;
  if (!idx || !cnt || !crow || !col || row_stride <= 0 || col_capacity < 0) return SEA_EINVAL;
  if (static_cast<int64_t>(p->H) * p->T > INT32_MAX) return SEA_ENOTSUP;  // columns h T + j are int32
  const Shape s = make_shape(p, false);
  if (!workspace || workspace_bytes < align256(flatcsr_workspace(s)) ||
      reinterpret_cast<uintptr_t>(workspace) % 256 != 0)
    return SEA_EWORKSPACE;
  const hipError_t e = launch_flatcsr(s, idx, cnt, row_stride, crow, col, col_capacity, workspace,
                                      static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? SEA_OK : fail_hip(e);
}

int sea_key_mask(const sea_params* p, const uint32_t* mhat, uint32_t* key_bits, void* hip_stream) {
  int rc = check_common(p);
  if (rc == SEA_OK) rc = check_mask_params(p);
  if (rc != SEA_OK) return rc;
  if (!mhat || !key_bits) return SEA_EINVAL;
  const Shape s = make_shape(p, true);
  if (!keybits_supported(s)) return SEA_ENOTSUP;
  const hipError_t e = launch_keybits(s, mhat, key_bits, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? SEA_OK : fail_hip(e);
}

int sea_flatcsr_attn(const sea_params* p, const void* Q, const void* K, const void* V, const int64_t* crow,
                     const int32_t* col, void* O, void* hip_stream) {
  const int rc = check_common(p);
  if (rc != SEA_OK) return rc;
  if (!Q || !K || !V || !crow || !col || !O) return SEA_EINVAL;
  if (static_cast<int64_t>(p->H) * p->T > INT32_MAX) return SEA_ENOTSUP;
  const Shape s = make_shape(p, false);
  const hipError_t e = launch_sparse_attn(s, p->dtype, Q, K, V, col, nullptr, 0, crow, O,
                                          static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? SEA_OK : fail_hip(e);
}

size_t sea_mask_attn_workspace_bytes(const sea_params* p) {
  if (check_common(p) != SEA_OK || check_mask_params(p) != SEA_OK) return 0;
  const Shape s = make_shape(p, true);
  if (!tile_attn_supported(s, p->dtype, nullptr)) return 0;
  return align256(tile_attn_workspace(s));
}

int sea_mask_attn(const sea_params* p, const void* Q, const void* K, const void* V, const uint32_t* mhat,
                  void* O, void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_common(p);
  if (rc == SEA_OK) rc = check_mask_params(p);
  if (rc != SEA_OK) return rc;
  if (!Q || !K || !V || !mhat || !O) return SEA_EINVAL;
  const Shape s = make_shape(p, true);
  if (!tile_attn_supported(s, p->dtype, nullptr)) return SEA_ENOTSUP;
  const size_t need = align256(tile_attn_workspace(s));
  if (need > 0 && (!workspace || workspace_bytes < need || reinterpret_cast<uintptr_t>(workspace) % 256 != 0))
    return SEA_EWORKSPACE;
  const hipError_t e = launch_tile_attn(s, static_cast<const uint16_t*>(Q), static_cast<const uint16_t*>(K),
                                        static_cast<const uint16_t*>(V), mhat, static_cast<uint16_t*>(O),
                                        workspace, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? SEA_OK : fail_hip(e);
}

namespace {
// the stages of the forward pass on one stream; the workspace is laid out as forward_ws(p, lean)
int forward_stages(const sea_params* p, const void* Q, const void* K, const void* V, const void* W,
                   void* O, float* A_hat_opt, int32_t* sel_opt, int32_t* idx_opt, int32_t* cnt_opt,
                   uint32_t* mhat_opt, void* workspace, bool lean, hipStream_t st) {
  const Shape s = make_shape(p, true);
  const size_t rows = static_cast<size_t>(s.N) * s.T;
  char* w = static_cast<char*>(workspace);
  void* est_ws = w;
  w += estimate_ws(p);
  float* A_hat = A_hat_opt;
  if (!(lean && scores_stay_on_chip(p, s))) {
    if (!A_hat) A_hat = reinterpret_cast<float*>(w);
    w += align256(rows * s.K * sizeof(float));
  }
  const bool tiled = tile_attn_supported(s, p->dtype, nullptr);

  hipError_t e;
  if (tiled) {
    // column-structured mask: selection as bits, attention on 128-row tiles; A_hat and the row
    // lists are written only if the caller asked for them
    uint32_t* mbits = mhat_opt ? mhat_opt : reinterpret_cast<uint32_t*>(w);
    w += align256(rows * ((s.K + 31) / 32) * sizeof(uint32_t));
    const bool need_lists = sel_opt || idx_opt || cnt_opt;
    if (estimate_fused_supported(s) && s.grouping == 0) {
      // estimate and per-row top-k^ in one kernel; the scores never leave the registers
      e = launch_estimate_fused(s, static_cast<const uint16_t*>(Q), static_cast<const uint16_t*>(K),
                                static_cast<const uint16_t*>(W), (A_hat_opt || need_lists) ? A_hat : nullptr,
                                mbits, est_ws, st);
      if (e != hipSuccess) return fail_hip(e);
      if (need_lists) e = launch_topk_mask(s, A_hat, sel_opt, idx_opt, cnt_opt, nullptr, st);
    } else {
      // causal-per-batch selection reads a row's scores only up to its last candidate column: when
      // the scores go to scratch and nothing else reads them, the estimator writes no further
      Shape se = s;
      se.cand_only = (s.grouping == 1 && !A_hat_opt && !need_lists) ? 1 : 0;
      e = launch_estimate_bf16(se, static_cast<const uint16_t*>(Q), static_cast<const uint16_t*>(K),
                               static_cast<const uint16_t*>(W), A_hat, est_ws, st);
      if (e != hipSuccess) return fail_hip(e);
      e = launch_topk_mask(s, A_hat, sel_opt, idx_opt, cnt_opt, mbits, st);
    }
    if (e != hipSuccess) return fail_hip(e);
    e = launch_tile_attn(s, static_cast<const uint16_t*>(Q), static_cast<const uint16_t*>(K),
                         static_cast<const uint16_t*>(V), mbits, static_cast<uint16_t*>(O), w, st);
    return e == hipSuccess ? SEA_OK : fail_hip(e);
  }
  if (s.geometry == 1)
    e = launch_estimate_rowwidth(s, p->dtype, Q, K, W, A_hat, est_ws, st);
  else if (p->dtype == SEA_BF16)
    e = launch_estimate_bf16(s, static_cast<const uint16_t*>(Q), static_cast<const uint16_t*>(K),
                             static_cast<const uint16_t*>(W), A_hat, est_ws, st);
  else
    e = launch_estimate_f64(s, static_cast<const float*>(Q), static_cast<const float*>(K),
                            static_cast<const float*>(W), A_hat, est_ws, st);
  if (e != hipSuccess) return fail_hip(e);
  if (p->dtype == SEA_F32 && tile_attn_f32_supported(s)) {
    // fp32 tensors, column-structured mask: selection as bits, attention on 16-row tiles
    uint32_t* mbits = mhat_opt ? mhat_opt : reinterpret_cast<uint32_t*>(w);
    e = launch_topk_mask(s, A_hat, sel_opt, idx_opt, cnt_opt, mbits, st);
    if (e != hipSuccess) return fail_hip(e);
    e = launch_tile_attn_f32(s, static_cast<const float*>(Q), static_cast<const float*>(K),
                             static_cast<const float*>(V), mbits, static_cast<float*>(O), st);
    return e == hipSuccess ? SEA_OK : fail_hip(e);
  }
  if (keybit_path(s, p->dtype)) {
    uint32_t* mbits = mhat_opt ? mhat_opt : reinterpret_cast<uint32_t*>(w);
    w += align256(rows * ((s.K + 31) / 32) * sizeof(uint32_t));
    uint32_t* kb = reinterpret_cast<uint32_t*>(w);
    if (s.grouping == 0) {
      // per-query selection: the kernel that selects a row also expands it to its key bits
      e = launch_topk_mask(s, A_hat, sel_opt, idx_opt, cnt_opt, mbits, st, kb);
    } else {
      e = launch_topk_mask(s, A_hat, sel_opt, idx_opt, cnt_opt, mbits, st);
      if (e != hipSuccess) return fail_hip(e);
      e = launch_keybits(s, mbits, kb, st);
    }
    if (e != hipSuccess) return fail_hip(e);
    if (p->dtype == SEA_BF16)
      e = launch_tile_attn_keybits(s, static_cast<const uint16_t*>(Q), static_cast<const uint16_t*>(K),
                                   static_cast<const uint16_t*>(V), kb, static_cast<uint16_t*>(O), st);
    else
      e = launch_tile_attn_f32_keybits(s, static_cast<const float*>(Q), static_cast<const float*>(K),
                                       static_cast<const float*>(V), kb, static_cast<float*>(O), st);
    return e == hipSuccess ? SEA_OK : fail_hip(e);
  }
  int32_t* idx = idx_opt ? idx_opt : reinterpret_cast<int32_t*>(w);
  w += align256(rows * static_cast<size_t>(s.L) * sizeof(int32_t));
  int32_t* cnt = cnt_opt ? cnt_opt : reinterpret_cast<int32_t*>(w);
  w += align256(rows * sizeof(int32_t));
  uint32_t* mbits = mhat_opt;
  if (!mbits && s.grouping == 1) mbits = reinterpret_cast<uint32_t*>(w);  // selection as bits, lists from them
  e = launch_topk_mask(s, A_hat, sel_opt, idx, cnt, mbits, st);
  if (e != hipSuccess) return fail_hip(e);
  e = launch_sparse_attn(s, p->dtype, Q, K, V, idx, cnt, s.L, nullptr, O, st);
  return e == hipSuccess ? SEA_OK : fail_hip(e);
}
}  // namespace

int sea_forward(const sea_params* p, const void* Q, const void* K, const void* V, const void* W,
                void* O, float* A_hat_opt, int32_t* sel_opt, int32_t* idx_opt, int32_t* cnt_opt,
                uint32_t* mhat_opt, void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_common(p);
  if (rc == SEA_OK) rc = check_mask_params(p);
  if (rc == SEA_OK) rc = check_estimate_params(p);
  if (rc != SEA_OK) return rc;
  if (!Q || !K || !V || !W || !O) return SEA_EINVAL;
  if (row_stride_of(p) < 0) return SEA_ENOTSUP;
  if (!workspace || workspace_bytes < forward_ws(p, false)) return SEA_EWORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return SEA_EWORKSPACE;
  return forward_stages(p, Q, K, V, W, O, A_hat_opt, sel_opt, idx_opt, cnt_opt, mhat_opt, workspace, false,
                        static_cast<hipStream_t>(hip_stream));
}

size_t sea_static_scratch_bytes(void) { return kStaticScratchBytes; }

size_t sea_forward_static_bytes(const sea_params* p) {
  if (check_common(p) != SEA_OK || check_mask_params(p) != SEA_OK || check_estimate_params(p) != SEA_OK ||
      row_stride_of(p) < 0)
    return 0;
  return forward_ws(p, true);
}

int sea_forward_static(const sea_params* p, const void* Q, const void* K, const void* V, const void* W,
                       void* O, void* hip_stream) {
  int rc = check_common(p);
  if (rc == SEA_OK) rc = check_mask_params(p);
  if (rc == SEA_OK) rc = check_estimate_params(p);
  if (rc != SEA_OK) return rc;
  if (!Q || !K || !V || !W || !O) return SEA_EINVAL;
  if (row_stride_of(p) < 0) return SEA_ENOTSUP;
  if (forward_ws(p, true) > kStaticScratchBytes) return SEA_ETOOBIG;
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc != SEA_OK) return rc;
  return forward_stages(p, Q, K, V, W, O, nullptr, nullptr, nullptr, nullptr, nullptr, ws, true,
                        static_cast<hipStream_t>(hip_stream));
}

namespace {
// decoder scratch | A_hat | s_mix | s_prob | mask bits and bucket tables, or idx + cnt (+ bits) | mixing scratch
struct DecFwdWs {
  size_t dec, A_hat, s_mix, s_prob, att, mix, total;
};
DecFwdWs decoder_forward_layout(const sea_params* p) {
  const Shape s = make_shape(p, true);
  const size_t rows = static_cast<size_t>(s.N) * s.T;
  DecFwdWs w{};
  size_t off = 0;
  w.dec = off; off += align256(decoder_workspace(s));
  w.A_hat = off; off += align256(rows * s.K * sizeof(float));
  w.s_mix = off; off += align256(rows * sizeof(float));
  w.s_prob = off; off += align256(rows * sizeof(float));
  w.att = off;
  off += align256(rows * ((s.K + 31) / 32) * sizeof(uint32_t));
  if (tile_attn_supported(s, p->dtype, nullptr)) {
    off += align256(tile_attn_workspace(s));
  } else {
    off += align256(rows * static_cast<size_t>(s.L) * sizeof(int32_t));
    off += align256(rows * sizeof(int32_t));
  }
  w.mix = off; off += align256(output_mix_workspace(s));
  w.total = off;
  return w;
}
int check_decoder(const sea_params* p) {
  int rc = check_common(p);
  if (rc == SEA_OK) rc = check_mask_params(p);
  if (rc == SEA_OK) rc = check_estimate_params(p);
  if (rc != SEA_OK) return rc;
  if (row_stride_of(p) < 0) return SEA_ENOTSUP;
  if (!decoder_supported(make_shape(p, true), p->dtype)) return SEA_ENOTSUP;
  return SEA_OK;
}
bool weights_complete(const sea_decoder_weights* w) {
  return w && w->mu_w && w->mu_b && w->nu1_w && w->nu1_b && w->nu2_w && w->nu2_b && w->conv1_w && w->conv1_b &&
         w->conv2_w && w->conv2_b && w->conv3_w && w->conv3_b && w->mix_w && w->mix_b && w->prob_w && w->prob_b;
}
}  // namespace

size_t sea_decoder_workspace_bytes(const sea_params* p) {
  if (check_decoder(p) != SEA_OK) return 0;
  return decoder_forward_layout(p).total;
}

int sea_decoder_estimate(const sea_params* p, const sea_decoder_weights* w, const void* Q, const void* K,
                         const void* V, const void* W, float* A_hat, float* s_mix_opt, float* s_prob_opt,
                         void* workspace, size_t workspace_bytes, void* hip_stream) {
  const int rc = check_decoder(p);
  if (rc != SEA_OK) return rc;
  if (!Q || !K || !V || !W || !A_hat || !weights_complete(w)) return SEA_EINVAL;
  const Shape s = make_shape(p, true);
  if (!workspace || workspace_bytes < align256(decoder_workspace(s)) ||
      reinterpret_cast<uintptr_t>(workspace) % 256 != 0)
    return SEA_EWORKSPACE;
  const hipError_t e = launch_decoder_estimate(s, *w, static_cast<const uint16_t*>(Q), static_cast<const uint16_t*>(K),
                                               static_cast<const uint16_t*>(V), static_cast<const uint16_t*>(W), A_hat,
                                               s_mix_opt, s_prob_opt, workspace, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? SEA_OK : fail_hip(e);
}

int sea_decoder_forward(const sea_params* p, const sea_decoder_weights* w, const void* Q, const void* K,
                        const void* V, const void* W, void* O, float* A_hat_opt, void* workspace,
                        size_t workspace_bytes, void* hip_stream) {
  const int rc = check_decoder(p);
  if (rc != SEA_OK) return rc;
  if (!Q || !K || !V || !W || !O || !weights_complete(w)) return SEA_EINVAL;
  const DecFwdWs lay = decoder_forward_layout(p);
  if (!workspace || workspace_bytes < lay.total || reinterpret_cast<uintptr_t>(workspace) % 256 != 0)
    return SEA_EWORKSPACE;
  const Shape s = make_shape(p, true);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  char* base = static_cast<char*>(workspace);
  const size_t rows = static_cast<size_t>(s.N) * s.T;
  float* A_hat = A_hat_opt ? A_hat_opt : reinterpret_cast<float*>(base + lay.A_hat);
  float* s_mix = reinterpret_cast<float*>(base + lay.s_mix);
  float* s_prob = reinterpret_cast<float*>(base + lay.s_prob);
  hipError_t e = launch_decoder_estimate(s, *w, static_cast<const uint16_t*>(Q), static_cast<const uint16_t*>(K),
                                         static_cast<const uint16_t*>(V), static_cast<const uint16_t*>(W), A_hat, s_mix,
                                         s_prob, base + lay.dec, st);
  if (e != hipSuccess) return fail_hip(e);
  char* att = base + lay.att;
  uint32_t* mbits = reinterpret_cast<uint32_t*>(att);
  att += align256(rows * ((s.K + 31) / 32) * sizeof(uint32_t));
  if (tile_attn_supported(s, p->dtype, nullptr)) {
    e = launch_topk_mask(s, A_hat, nullptr, nullptr, nullptr, mbits, st);
    if (e != hipSuccess) return fail_hip(e);
    e = launch_tile_attn(s, static_cast<const uint16_t*>(Q), static_cast<const uint16_t*>(K),
                         static_cast<const uint16_t*>(V), mbits, static_cast<uint16_t*>(O), att, st);
  } else {
    int32_t* idx = reinterpret_cast<int32_t*>(att);
    int32_t* cnt = reinterpret_cast<int32_t*>(att + align256(rows * static_cast<size_t>(s.L) * sizeof(int32_t)));
    e = launch_topk_mask(s, A_hat, nullptr, idx, cnt, s.grouping == 1 ? mbits : nullptr, st);
    if (e != hipSuccess) return fail_hip(e);
    e = launch_sparse_attn(s, p->dtype, Q, K, V, idx, cnt, s.L, nullptr, O, st);
  }
  if (e != hipSuccess) return fail_hip(e);
  e = launch_output_mix(s, p->dtype, O, V, A_hat, s_prob, s_mix, O, base + lay.mix, st);
  return e == hipSuccess ? SEA_OK : fail_hip(e);
}

size_t sea_dense_workspace_bytes(const sea_params* p) {
  if (check_common(p) != SEA_OK || p->dtype != SEA_BF16) return 0;
  return dense_attn_workspace(make_shape(p, false));
}

int sea_dense_attn(const sea_params* p, const void* Q, const void* K, const void* V, void* O,
                   void* workspace, size_t workspace_bytes, void* hip_stream) {
  const int rc = check_common(p);
  if (rc != SEA_OK) return rc;
  if (!Q || !K || !V || !O) return SEA_EINVAL;
  if (p->dtype != SEA_BF16) return SEA_ENOTSUP;
  const Shape s = make_shape(p, false);
  const size_t need = dense_attn_workspace(s);  // currently none: K and V are read in place
  if (need > 0 && (!workspace || workspace_bytes < need || reinterpret_cast<uintptr_t>(workspace) % 256 != 0))
    return SEA_EWORKSPACE;
  const hipError_t e =
      launch_dense_attn(s, p->dtype, Q, K, V, O, workspace, static_cast<hipStream_t>(hip_stream));
  if (e == hipErrorNotSupported) return SEA_ENOTSUP;
  return e == hipSuccess ? SEA_OK : fail_hip(e);
}

size_t sea_output_mix_workspace_bytes(const sea_params* p) {
  if (check_common(p) != SEA_OK) return 0;
  return output_mix_workspace(make_shape(p, false));
}

int sea_output_mix(const sea_params* p, const void* C, const void* V, const float* A_hat,
                   const float* s_prob, const float* s_mix, void* O, void* workspace,
                   size_t workspace_bytes, void* hip_stream) {
  const int rc = check_common(p);
  if (rc != SEA_OK) return rc;
  if (!C || !V || !s_mix || !O) return SEA_EINVAL;
  if (!p->causal && (!A_hat || p->K <= 0 || p->K > p->T)) return SEA_EINVAL;
  if (!p->causal && p->K > 1024) return SEA_ENOTSUP;
  const Shape s = make_shape(p, false);
  if (!workspace || workspace_bytes < output_mix_workspace(s) ||
      reinterpret_cast<uintptr_t>(workspace) % 256 != 0)
    return SEA_EWORKSPACE;
  const hipError_t e = launch_output_mix(s, p->dtype, C, V, A_hat, s_prob, s_mix, O, workspace,
                                         static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? SEA_OK : fail_hip(e);
}

int sea_profile_enable(int stage_mask) {
  g_profile = static_cast<unsigned>(stage_mask) & ((1u << SEA_STAGE_COUNT) - 1u);
  return SEA_OK;
}

int sea_profile_collect(double* host_ms, int64_t* host_launches) {
  if (!host_ms || !host_launches) return SEA_EINVAL;
  int rc = SEA_OK;
  std::lock_guard<std::mutex> lock(g_profile_mutex);
  for (Span& sp : g_spans) {
    float ms = 0.f;
    hipError_t e = hipEventSynchronize(sp.b);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, sp.a, sp.b);
    if (e == hipSuccess && sp.stage >= 0 && sp.stage < SEA_STAGE_COUNT) {
      host_ms[sp.stage] += ms;
      host_launches[sp.stage] += 1;
    } else if (e != hipSuccess) {
      rc = fail_hip(e);
    }
    g_free_events.push_back(sp.a);
    g_free_events.push_back(sp.b);
  }
  g_spans.clear();
  return rc;
}

const char* sea_strerror(int status) {
  switch (status) {
    case SEA_OK: return "ok";
    case SEA_EINVAL: return "invalid argument (NULL pointer, size out of range, K > T or k_hat > K)";
    case SEA_ENOTSUP: return "not supported (d != 64, K > 1024, or m not a multiple of 32 up to 1024)";
    case SEA_EWORKSPACE: return "workspace missing, misaligned or smaller than sea_workspace_bytes()";
    case SEA_EHIP: return "a HIP runtime call failed (see sea_last_hip_error)";
    case SEA_ETOOBIG:
      return "the problem needs more scratch than sea_forward_static's fixed buffer holds (see "
             "sea_forward_static_bytes and sea_static_scratch_bytes); use sea_forward with a workspace";
    default: return "unknown status";
  }
}

int sea_last_hip_error(void) { return g_last_hip_error; }

int sea_attention_path(const sea_params* p) {
  int rc = check_common(p);
  if (rc == SEA_OK) rc = check_mask_params(p);
  if (rc != SEA_OK) return rc;
  const Shape s = make_shape(p, true);
  if (tile_attn_supported(s, p->dtype, nullptr)) return 1;
  if (p->dtype == SEA_F32 && tile_attn_f32_supported(s)) return 2;
  return keybit_path(s, p->dtype) ? 3 : 0;
}

const char* sea_version(void) { return "sea-hip 0.1 (gfx950)"; }

}  // extern "C"

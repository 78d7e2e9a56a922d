/*
 * sea.h -- C ABI of the SEA attention forward pass for AMD MI355X (gfx950).
 *
 * SEA (arXiv 2310.01777, Sec. 3.1) runs attention in two phases: (1) a
 * kernel-based (FAVOR+ random-feature) estimate A_hat of the attention matrix,
 * compressed to a fixed width K; (2) a per-query top-k^ selection on A_hat, its
 * nearest-neighbour expansion into a sparse T x T mask, and softmax attention
 * restricted to the selected keys.  Cost and memory are linear in T.
 *
 * Conventions shared by every entry point
 *   - Every pointer argument except `const sea_params*` and those marked "host"
 *     is DEVICE memory owned by the caller.  The library never allocates or
 *     frees device memory and never synchronises: it only enqueues kernels on
 *     the given stream (a hipStream_t passed as void*, NULL = default stream)
 *     and returns.
 *   - Tensors are dense row-major: Q, K, V, O are [B][H][T][d]; W is [m][d];
 *     A_hat is [B][H][T][K] float; sel is [B][H][T][S] int32 (S = sea_sel_stride()); idx is
 *     [B][H][T][L] int32 with L = sea_row_stride(); cnt is [B][H][T] int32.
 *     Q, K, V, W, O hold `dtype` elements (float or bfloat16).
 *   - Output buffers are fully overwritten: unused sel/idx slots are -1, rows at
 *     or beyond seq_len[b] get O = 0, A_hat = 0, cnt = 0.
 *   - Return value: SEA_OK (0) or a negative sea_status.  No exceptions, no
 *     aborts.  After SEA_EHIP, sea_last_hip_error() gives the hipError_t value.
 *   - Calls are reentrant across streams; two calls that share a workspace or an
 *     output buffer must be ordered by the caller.
 */
#ifndef SEA_H_
#define SEA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { SEA_F32 = 0, SEA_BF16 = 1 } sea_dtype;

typedef enum {
  SEA_OK = 0,
  SEA_EINVAL = -1,     /* NULL pointer, non-positive size, K > T, k_hat > K, ...          */
  SEA_ENOTSUP = -2,    /* valid but not implemented: d != 64, K > 1024, m % 32 != 0, ...  */
  SEA_EWORKSPACE = -3, /* workspace NULL or smaller than sea_workspace_bytes()             */
  SEA_EHIP = -4,       /* a HIP call failed; see sea_last_hip_error()                      */
  SEA_ETOOBIG = -5     /* sea_forward_static only: needs more scratch than its fixed buffer  */
} sea_status;

/*
 * Problem statement (Sec. 3 "Preliminaries", Sec. 3.1):
 *   Q, K, V in R^{T x d} per head, optional batch B and head H dimensions;
 *   K = width of the compressed matrix; k^ = entries selected per query row in
 *   the compressed space; k = the paper's sparsity budget in the full space.
 */
typedef struct {
  int32_t B, H, T, d;  /* d must be 64                                                     */
  int32_t m;           /* number of random features = rows of W; multiple of 32, <= 1024   */
  int32_t K;           /* compressed width, 1 <= K <= min(T, 1024)                          */
  int32_t k_hat;       /* 1 <= k_hat <= K                                                   */
  int32_t k_budget;    /* the paper's k: at most max(1, floor(k_budget / k_hat)) keys are
                          emitted per selected column, evenly spaced (App. A.5.3 "limit the
                          pixel replications, space them uniformly"); 0 = whole columns     */
  int32_t causal;      /* 0: every key < seq_len is admissible; 1: only keys j <= t         */
  float scale;         /* logits = scale * q.k.  The paper writes softmax(QK^T) with no
                          factor; pass d^-1/2 for the usual scaled attention                */
  sea_dtype dtype;     /* element type of Q, K, V, W, O                                     */
  const int32_t* seq_len; /* device [B] or NULL.  Right padding: keys and query rows at
                          positions >= seq_len[b] are inactive                              */
  int32_t grouping;    /* Sec. 3.1 "Grouped Top-k^ Selection": 0 = per-query (each row of each
                          head keeps k_hat entries); 1 = causal-per-batch (A_hat viewed as
                          [T][H K]: each time step keeps H k_hat entries of its H x K slab, so
                          heads share the quota; needs H K <= 16384)                         */
  int32_t geometry;    /* how the K columns map to keys.  0: key j belongs to column
                          floor(j K / T) for every row.  1 (causal only; App. A.4, figure of
                          the masking process): row t is resized to its own width, its column
                          c holds the keys [ceil(c (t+1) / K), ceil((c+1)(t+1) / K)) -- the
                          estimate, the selection (columns without a key are no candidates)
                          and the expansion of row t are those of a sequence of t + 1 keys.
                          Needs m in {64, 128, 256}; the estimate then runs
                          in fp64 from a running key state (no bf16 rounding points), and
                          the attention stage works from per-row key lists                */
} sea_params;

/* k^ = max(1, round(k K / T)), halves rounded up (Sec. 3.1 "Linear Sparse Attention Mask
 * Generation").  Pure host arithmetic. */
int32_t sea_k_hat(int32_t k, int32_t K, int32_t T);

/* S, the row stride of sel = the most columns one row of one head can select: k_hat, or
 * min(K, H k_hat) with the causal-per-batch grouping.  Host arithmetic. */
int32_t sea_sel_stride(const sea_params* p);

/* L, the row stride of idx: S * r with r = ceil(T/K) keys per selected column, or
 * min(ceil(T/K), max(1, k_budget / k_hat)) when k_budget > 0.  Host arithmetic; returns a
 * negative sea_status on invalid parameters. */
int32_t sea_row_stride(const sea_params* p);

/* Bytes of device scratch sea_estimate / sea_forward need for these parameters (0 on invalid
 * parameters).  The workspace must be 256-byte aligned; its contents are undefined afterwards. */
size_t sea_workspace_bytes(const sea_params* p);

/*
 * Phase (1), Sec. 3 "Performer (FAVOR+)" and Sec. 3.1 "Attention Matrix Estimation".
 *   phi(x)[i] = exp(w_i.x - |x|^2/2) with x = sqrt(scale) q (keys alike), w_i = row i of W;
 *   V_I = the T x K one-hot matrix with V_I[j][floor(j K / T)] = 1 (nearest-neighbour stretch
 *   of the identity); A_hat = rownorm( phi(Q) (phi(K)^T V_I) ), where a causal row t only
 *   sums keys j <= t.  Rows sum to 1; columns holding no admissible key are 0.
 * dtype = SEA_BF16: phi(Q) (after a power-of-two row scale) and the finished column sums
 * phi(K)^T V_I are rounded to bfloat16 and contracted on the matrix cores with fp32
 * accumulation; a causal row's own column is summed key by key over j <= t from phi(k_j) rounded
 * to bfloat16 (no prefix state is rounded).  dtype = SEA_F32: all products accumulate in fp64.
 * geometry = 1: V_I of row t is the (t+1) x K stretch, A_hat[t][c] = sum of phi(q_t) . phi(k_j)
 * over the keys of the row's own column c, normalised per row.  dtype = SEA_BF16: phi(q_t) (after
 * a power-of-two row scale) and every phi(k_j) are rounded to bfloat16, the per-key products are
 * taken on the matrix cores with fp32 accumulation and summed per column without further
 * rounding; dtype = SEA_F32: all of it in fp64.
 * The feature exponent is not stabilised on the key side (a data-dependent key stabiliser would
 * make causal results depend on future keys).  Two bounds follow for dtype = SEA_BF16, where the
 * features are fp32: above, log2(e) |w_i|^2 / 2 must stay inside the fp32 exponent range (true for
 * any Gaussian W with d = 64); below, a key with scale |k|^2 / 2 - sqrt(scale) w_i.k above about
 * 87 for every i has all-zero features and drops out of the estimate (with unit-variance inputs
 * and scale = d^-1/2 this needs |k|^2 > 1000, far outside the stated workloads).
 */
int sea_estimate(const sea_params* p, const void* Q, const void* K, const void* W,
                 float* A_hat, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Phase (2a, 2b), Sec. 3.1 "Grouped Top-k^ Selection" (per-query grouping) and "Linear Sparse
 * Attention Mask Generation" / App. A.5.3 (sparse nearest-neighbour interpolation).
 *   For each active row: among the columns that hold an admissible key, take the
 *   min(k_hat, #columns) largest A_hat entries (equal values: lower column first); sel lists
 *   them ascending.  With grouping = 1 the H rows of a time step are ranked together (equal
 *   values: lower h K + c first) and min(H k_hat, H #columns) entries are kept.  Column c covers keys [ceil(cT/K), ceil((c+1)T/K)), width w; a selected
 *   column emits keys start + floor(i w / r), i < r; keys j > t (causal) or j >= seq_len are
 *   dropped.  idx lists the emitted keys ascending, cnt their number.
 *   With geometry = 1 read T in the column formulas as the row's own width t + 1; columns that
 *   hold no key of the row are no candidates.
 * sel may be NULL.
 */
int sea_topk_mask(const sea_params* p, const float* A_hat, int32_t* sel, int32_t* idx,
                  int32_t* cnt, void* hip_stream);

/*
 * Phase (2c), Sec. 3.1.1 "Sparse Attention Mechanism": rho (QK^T only at listed positions),
 * sigma (softmax over the listed positions of each row), C = A* V.
 *   O[t] = sum_j softmax_j(scale * q_t.k_j) v_j over j in idx[t][0..cnt[t]).
 * Rows with cnt = 0 give zeros.  Entries outside [0, T) are ignored.  `row_stride` is the
 * stride L of idx (any L >= max cnt).  Logits and softmax run in fp32 (bf16) or with fp64
 * dot products (f32); O is rounded once to `dtype`.  No T x T intermediate exists.
 */
int sea_sparse_attn(const sea_params* p, const void* Q, const void* K, const void* V,
                    const int32_t* idx, const int32_t* cnt, int32_t row_stride, void* O,
                    void* hip_stream);

/*
 * Sec. 3.1 "Linear Sparse Attention Mask Generation" (App. A.4 for geometry = 1, App. A.5.3 for the
 * replication cap): the expanded mask M* as one bit per (row, key), from the compressed binary mask
 * M^ (mhat: [B][H][T][ceil(K / 32)] device words, bit c % 32 of word c / 32 = column c, as
 * sea_forward writes to mhat_opt).  Bit j % 32 of word j / 32 of row t of key_bits
 * ([B][H][T][ceil(T / 32)] device words) is set iff key j is one of the r = min(w, cap) keys
 * start + floor(i w / r) of a selected column of that row, j <= t when causal, j < seq_len; rows
 * t >= seq_len are zero.  This is the mask sea_forward's attention stage consumes when
 * sea_attention_path(p) == 3.  Needs T <= 8192 (SEA_ENOTSUP otherwise); no workspace.
 */
int sea_key_mask(const sea_params* p, const uint32_t* mhat, uint32_t* key_bits, void* hip_stream);

/*
 * Sec. 3.1.1 "FlatCSR" and App. A.5 "FlatCSR: Modified CSR Format To Handle Grouped Mask": the
 * expanded mask M* [B][H][T][T] with the head and query axes exchanged and (head, key) flattened
 * into one column axis, stored as CSR, so that one time step -- the group of the causal-per-batch
 * selection -- is one CSR row.
 *   crow [B T + 1] (device, int64): crow[b T + t] = first entry of row (b, t); crow[B T] = nnz.
 *   col  [col_capacity] (device, int32): entries h T + j, heads ascending and keys ascending
 *        inside a head, for the keys j that idx / cnt (as sea_topk_mask or sea_forward wrote them,
 *        row stride `row_stride`) list for head h at query t.  Needs H T < 2^31.
 * Entries beyond col_capacity are not written, crow is complete either way: crow[B T] >
 * col_capacity tells the caller the array was too small.  B H T row_stride always suffices; so
 * does B T H k_hat r with r keys per selected column (either grouping).
 * Workspace: sea_flatcsr_workspace_bytes(), 256-byte aligned.
 */
size_t sea_flatcsr_workspace_bytes(const sea_params* p);
int sea_flatcsr(const sea_params* p, const int32_t* idx, const int32_t* cnt, int32_t row_stride,
                int64_t* crow, int32_t* col, int64_t col_capacity, void* workspace, size_t workspace_bytes,
                void* hip_stream);

/*
 * Phase (2c) read from the FlatCSR tensor (App. A.5: the kernel undoes the flattening and the
 * exchange of axes itself): O[b][h][t] = sum_j softmax_j(scale q_t.k_j) v_j over the entries
 * h T + j of CSR row b T + t, arithmetic as in sea_sparse_attn.  Columns of a CSR row must ascend;
 * a row (b, h, t) without entries gives zeros.
 */
int sea_flatcsr_attn(const sea_params* p, const void* Q, const void* K, const void* V, const int64_t* crow,
                     const int32_t* col, void* O, void* hip_stream);

/*
 * Phases (2b) + (2c) from the compressed binary mask M^ of Sec. 3.1 "Linear Sparse Attention Mask
 * Generation" (the bit-packed form sea_forward writes to mhat_opt): row t attends, for every set
 * bit c of its mask row, the r keys start_c + floor(i w / r), i < r, of column c that are
 * admissible (j <= t when causal, j < seq_len) -- the expansion of App. A.5.3 is implicit -- and
 * O[t] is the softmax-weighted sum of their values as in sea_sparse_attn.  This is the attention
 * stage of sea_forward on its own; it needs the column-structured form, sea_attention_path(p) == 1
 * (SEA_ENOTSUP otherwise), and sea_mask_attn_workspace_bytes() of 256-byte aligned scratch (0 for
 * most shapes; then workspace may be NULL).  A mask row may hold at most k_hat set bits (or, with
 * grouping = 1, any number); where rows are grouped by column (see sea_forward) further bits are
 * ignored.  Rows without set bits give zeros.
 */
size_t sea_mask_attn_workspace_bytes(const sea_params* p);
int sea_mask_attn(const sea_params* p, const void* Q, const void* K, const void* V, const uint32_t* mhat,
                  void* O, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The whole forward pass (Fig. "model structure", phases 1 and 2 back to back) on one stream.
 * A_hat_opt, sel_opt, idx_opt, cnt_opt, mhat_opt may each be NULL when the caller does not want
 * that intermediate; results are identical either way.  mhat_opt receives the compressed binary
 * mask M^ of Sec. 3.1 "Linear Sparse Attention Mask Generation", bit-packed:
 * uint32 [B][H][T][ceil(K/32)], bit c % 32 of word c / 32 set iff column c is selected.
 * Every output is a deterministic function of the inputs (runs are bit-identical): where the
 * attention stage groups rows by their selected column (bf16, K | T, per-query grouping and
 * k_hat = 1 or k_hat <= min(8, K/8)) the order inside a group comes from atomics, but no result
 * depends on it.  Only kernels are enqueued (no allocation, memset or synchronisation), so the
 * call can be captured in a HIP graph.  Calls that share a workspace must not overlap.
 */
int sea_forward(const sea_params* p, const void* Q, const void* K, const void* V, const void* W,
                void* O, float* A_hat_opt, int32_t* sel_opt, int32_t* idx_opt, int32_t* cnt_opt,
                uint32_t* mhat_opt, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * sea_forward for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same
 * results as sea_forward with every optional output NULL; the scratch is a fixed array of
 * sea_static_scratch_bytes() (64 MiB) inside the library, one copy per GPU, held until the process
 * ends.  The call allocates nothing and frees nothing (no hipMalloc, no allocating library call);
 * the first call on a GPU looks the array's device address up, with that GPU current.
 *   sea_forward_static_bytes(p): scratch these parameters need here (0 on invalid parameters); less
 *   than sea_workspace_bytes(p) where the scores stay on chip.  Above sea_static_scratch_bytes()
 *   the call returns SEA_ETOOBIG and enqueues nothing (c2: 3.1 MB, c3: 50 MB fit; c4 at T = 32768
 *   with 138 MB does not).
 * Every call on one GPU uses the same array, which keeps the previous call's contents; the kernels
 * overwrite or clear what they read, so calls may follow each other on one stream with any mix of
 * shapes.  Two calls that overlap on one GPU (different streams or threads, unordered) race.
 */
size_t sea_static_scratch_bytes(void);
size_t sea_forward_static_bytes(const sea_params* p);
int sea_forward_static(const sea_params* p, const void* Q, const void* K, const void* V, const void* W,
                       void* O, void* hip_stream);

/*
 * Sec. 3.1.1 "Output Calculation": C_sea = s_mix * (s_prob * C) + (1 - s_mix) * C_avg, row by row.
 *   C: the sparse-attention output of sea_forward / sea_sparse_attn, [B][H][T][d] in `dtype`;
 *   s_prob: device float [B][H][T] or NULL (= 1), the rescaling of the sparse probabilities
 *   A* = s_prob * sigma(...), which by linearity rescales C; s_mix: device float [B][H][T].
 *   Bidirectional (causal = 0): importance i^ = mean over the active rows of A_hat, stretched to
 *   the keys by nearest neighbour; C_avg = average of the active value rows weighted by it (one
 *   vector per head); A_hat [B][H][T][K] is required.  Causal: C_avg[t] = mean of v_0 .. v_t;
 *   A_hat is ignored.  The paper learns s_prob and s_mix from the decoder's hidden state; here
 *   the caller supplies them.  O may alias C.  Rows at or beyond seq_len give zeros.
 *   Needs sea_output_mix_workspace_bytes() of 256-byte aligned scratch.
 */
size_t sea_output_mix_workspace_bytes(const sea_params* p);
int sea_output_mix(const sea_params* p, const void* C, const void* V, const float* A_hat,
                   const float* s_prob, const float* s_mix, void* O, void* workspace,
                   size_t workspace_bytes, void* hip_stream);

/*
 * The learned decoder of Sec. 3.1 "CNN Decoder" / App. A.5.1 "Attention Estimator CNN", with
 * caller-supplied weights (the paper trains them by distillation; random weights make this a
 * throughput workload).  dtype = SEA_BF16 only.  Fixed here: c_s = 2, c_h = 4, hidden width
 * d' = 2 d = 128; mu = linear + ReLU; nu = linear + ReLU + linear; ReLU after the first two
 * convolutions.  All weight matrices are bf16 row-major [out][in], biases fp32; C = 4 H channels.
 *   C_perf = FAVOR+(Q, K, [V_I; V]) per head, V_I the T x d nearest-neighbour stretch of I_d, rows
 *            normalised by phi(q_t) . sum_j phi(k_j) (causal: j <= t);
 *   Z = mu([C_perf; V]) in R^{T x d'};  s_mix, s_prob = sigmoid(mix_w . Z + mix_b), likewise prob;
 *   Z^ = nu(Z) in R^{T x (K/c_s) c_h}, entry x c_h + ch -> pixel (t, x), channel h c_h + ch;
 *   conv1, conv2: 3x3, C -> C, ReLU; conv3: 3x3, C -> H, on the image resized (nearest) to T x K;
 *   one zero column left and right; causal: every layer reads rows t - 2 .. t and the height is
 *   not reduced; bidirectional: conv1 has height stride c_s and rows c_s i - 1 .. c_s i + 1, the
 *   others rows i - 1 .. i + 1;  A_hat[h][t][:] = softmax over the K columns.
 * Positions at or beyond seq_len: keys drop out of C_perf, rows of Z^ are zero, rows of A_hat,
 * s_mix, s_prob are zero.  Conv weights are [out][ky][kx][in].
 */
typedef struct {
  const void* mu_w;    const float* mu_b;     /* [128][192], [128]                     */
  const void* nu1_w;   const float* nu1_b;    /* [128][128], [128]                     */
  const void* nu2_w;   const float* nu2_b;    /* [(K / 2) 4][128], [(K / 2) 4]         */
  const void* conv1_w; const float* conv1_b;  /* [C][3][3][C], [C]                     */
  const void* conv2_w; const float* conv2_b;  /* [C][3][3][C], [C]                     */
  const void* conv3_w; const float* conv3_b;  /* [H][3][3][C], [H]                     */
  const void* mix_w;   const float* mix_b;    /* [128], [1]                            */
  const void* prob_w;  const float* prob_b;   /* [128], [1]                            */
} sea_decoder_weights;

/* Scratch of sea_decoder_estimate / sea_decoder_forward (0 on invalid or unsupported parameters). */
size_t sea_decoder_workspace_bytes(const sea_params* p);

/* A_hat [B][H][T][K] float (rows are softmaxes); s_mix_opt, s_prob_opt [B][H][T] float or NULL.
 * Needs m in {64, 128, 256}, K even, H even, geometry = 0 (SEA_ENOTSUP otherwise). */
int sea_decoder_estimate(const sea_params* p, const sea_decoder_weights* w, const void* Q, const void* K,
                         const void* V, const void* W, float* A_hat, float* s_mix_opt, float* s_prob_opt,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/* The paper's whole layer: decoder estimate -> grouped top-k^ (p->grouping) and mask expansion ->
 * sparse attention -> C_sea = s_mix (s_prob C) + (1 - s_mix) C_avg (sea_output_mix with the
 * decoder's scalers).  O [B][H][T][d]; A_hat_opt may be NULL. */
int sea_decoder_forward(const sea_params* p, const sea_decoder_weights* w, const void* Q, const void* K,
                        const void* V, const void* W, void* O, float* A_hat_opt, void* workspace,
                        size_t workspace_bytes, void* hip_stream);

/*
 * Quadratic attention A = softmax(scale QK^T), C = AV (Sec. 3 "Preliminaries"), causal and/or
 * right-padded like the sparse path, computed tile by tile with no T x T buffer.  This is the
 * baseline the sparse path is reported against, not part of SEA.  bf16 only (SEA_ENOTSUP for
 * fp32).  sea_dense_workspace_bytes() is the scratch it needs, 256-byte aligned; this version
 * needs none (returns 0) and then accepts workspace == NULL.
 */
size_t sea_dense_workspace_bytes(const sea_params* p);
int sea_dense_attn(const sea_params* p, const void* Q, const void* K, const void* V, void* O,
                   void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Per-stage timing for benchmarks.  stage_mask has bit (1 << stage) set for every stage to time
 * (0 = off, -1 = all): launches of those stages are bracketed by HIP events recorded on the
 * launch stream (each pair costs a few microseconds of stream time).  sea_profile_collect()
 * synchronises those events, adds the elapsed milliseconds and launch counts per stage into
 * the two host arrays of length SEA_STAGE_COUNT, and forgets them.  Process-wide state behind
 * a mutex: with timing on, calls from several threads are safe but their spans interleave, so
 * keep timing off (the default) when calls run concurrently.
 */
typedef enum {
  SEA_STAGE_FEATURES = 0, /* a1: feature maps phi(Q), phi(K)                              */
  SEA_STAGE_STATE = 1,    /* a2: key-side bucket sums and prefixes                         */
  SEA_STAGE_CONTRACT = 2, /* a3: phi(Q) x state, normalisation                             */
  SEA_STAGE_TOPK_MASK = 3,/* a4 + a5                                                       */
  SEA_STAGE_SPARSE = 4,   /* a6                                                            */
  SEA_STAGE_DENSE = 5,    /* dense baseline                                                */
  SEA_STAGE_COMPACT = 6,  /* reserved (no kernel: keys and values are read in place)          */
  SEA_STAGE_COUNT = 7
} sea_stage;
int sea_profile_enable(int stage_mask);
int sea_profile_collect(double* host_ms /*[SEA_STAGE_COUNT]*/, int64_t* host_launches /*[SEA_STAGE_COUNT]*/);

const char* sea_strerror(int status);
int sea_last_hip_error(void);
/*
 * Which kernel sea_forward's sparse attention stage (Sec. 3.1.1) runs for these parameters:
 * 1 = the tiled matrix-core kernel over the column-structured mask (bf16, K | T, a power-of-two
 * number of keys per selected column, fixed key buckets), 2 = its fp32 counterpart (same shapes,
 * fp32 tensors: logits on the fp64 matrix cores, weights and P V in fp32; sea_forward only),
 * 3 = the same tiled kernel on a per-(row, key) bit mask expanded from the selection (per-row width
 * geometry, T <= 8192 for bf16 and T <= 4096 for fp32 tensors; sea_forward only), 0 = the per-row
 * index-list kernel.
 * Negative: the sea_status the parameters would be rejected with.  Pure host computation.
 */
int sea_attention_path(const sea_params* p);

const char* sea_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SEA_H_ */

/*
 * pafu.h - C ABI of the PaFu-KV chunk-step library for AMD MI355X (gfx950).
 *
 * One autoregressive chunk step of the paper's inference procedure (Sec. 3.4,
 * inference paragraph; Alg. 2): score tokens with the Salience Estimation Head,
 * keep the top-k cached tokens, compact the KV cache to them, and attend from the
 * chunk's queries over the retained cache plus the chunk itself.
 *
 * Conventions (all entry points)
 *  - Every pointer is a DEVICE pointer unless the comment says "host".
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *    only enqueue work; they never synchronise and never allocate device memory.
 *  - Tensors are token-major: Q/K/V/O are [tokens, N, D] with an explicit token
 *    stride `ld_*` counted in ELEMENTS (so a slab with spare capacity works);
 *    inside a token the N*D elements are contiguous.  Scores are fp32, indices int32.
 *  - Device pointers must be 16-byte aligned and token strides multiples of 16 bytes.
 *  - Outputs must not alias inputs or each other (PAFU_ERR_ALIAS).  Overlap is decided on the strided rows, so
 *    tensors interleaved in one slab with a common stride (K and V side by side in a token) are fine.
 *    Weights and inputs are borrowed for the call.
 *  - Return value: PAFU_OK (0) = enqueued; a negative pafu_status = error, in which
 *    case NOTHING was enqueued and no output is touched.
 *  - A budget k larger than the cache is not an error: everything is kept
 *    (eviction only happens once the cache exceeds its budget, Alg. 2).
 */
#ifndef PAFU_H_
#define PAFU_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum pafu_status {
  PAFU_OK = 0,
  PAFU_ERR_NULL = -1,      /* a required pointer is NULL */
  PAFU_ERR_SHAPE = -2,     /* a size is negative / zero where it may not be / unsupported (D not 64 or 128) */
  PAFU_ERR_DTYPE = -3,     /* dtype enum value not supported by this call */
  PAFU_ERR_ALIGN = -4,     /* pointer not 16-byte aligned or stride not a multiple of 16 bytes */
  PAFU_ERR_WORKSPACE = -5, /* workspace NULL or smaller than pafu_*_workspace_bytes() */
  PAFU_ERR_ALIAS = -6,     /* an output buffer overlaps an input buffer */
  PAFU_ERR_HIP = -7        /* a HIP call failed; see pafu_last_hip_error() */
} pafu_status;

/* PAFU_FP8_E4M3: 8-bit storage of the K/V cache (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no infinities,
 * S.1111.111 = NaN), one byte per element, with one power-of-two scale per tensor that the caller passes as its
 * exponent: a stored code c stands for the value c * 2^scale_log2. */
typedef enum pafu_dtype { PAFU_BF16 = 0, PAFU_F32 = 1, PAFU_FP8_E4M3 = 2 } pafu_dtype;
typedef enum pafu_act { PAFU_ACT_SILU = 0, PAFU_ACT_GELU_ERF = 1 } pafu_act;
typedef enum pafu_mode { PAFU_MODE_SINGLE = 0, PAFU_MODE_ROLLOUT = 1 } pafu_mode;

/* Text for a pafu_status (static storage, host). */
const char* pafu_strerror(int status);
/* hipError_t of the last failed HIP call made by this library on the calling thread (0 if none). */
int pafu_last_hip_error(void);
/* Library ABI version (increases when a signature changes). */
int pafu_version(void);
/* 0 for the library as shipped.  Non-zero: a study build whose attention kernel was compiled with ingredients of its
 * inner loop taken out (to measure what they cost); such a build computes wrong results and is only ever loaded by
 * name, by the measurements recorded under profiles/. */
int pafu_study_build(void);
/* Enqueues an empty kernel (one wavefront, no memory access) on `stream`: the floor of what any stage can take
 * between two events on a stream, reported next to the latency-bound selection stage. */
int pafu_launch_probe(void* stream);

/* ------------------------------------------------------------------------------------------
 * pafu_score - Salience Estimation Head (S-MLP), App. A "S-MLP"; Sec. 3.3-3.4.
 *
 *   s[t] = mean_o( W2 . act( W1 . x[t] + b1 ) + b2 )_o          act = SiLU (the paper's)
 *
 * x[t] is the concatenation along the feature axis of n_seg (1..3) segments of Fs features
 * each: row t of x0, then of x1, then of x2 (the paper feeds [Q | K | V]); F = n_seg * Fs.
 *   x0,x1,x2 : [T, Fs] rows with stride ld_x elements, dtype x_dtype (x1/x2 ignored beyond n_seg)
 *   W1       : [M, F] row-major (out-features x in-features), SAME dtype as x
 *   b1       : [M] fp32 or NULL (= 0)
 *   W2       : [n_out, M] fp32 row-major;  b2 : [n_out] fp32 or NULL
 *   out      : [T] fp32
 *   workspace: pafu_score_workspace_bytes(M) bytes (holds the output-averaged second layer)
 * bf16 inputs with Fs % 64 == 0 and M % 32 == 0 take the MFMA paths (fp32 accumulate; M % 256 == 0 the
 * streaming kernel); anything else takes a plain fp32-FMA path.  T == 0 is a no-op.
 */
size_t pafu_score_workspace_bytes(int M);
int pafu_score(void* stream, const void* x0, const void* x1, const void* x2, int n_seg, int T, int Fs,
               long long ld_x, int x_dtype, const void* W1, const float* b1, const float* W2,
               const float* b2, int M, int n_out, int act, float* out, void* workspace,
               size_t workspace_bytes);

/* pafu_score_static - pafu_score for callers that cannot allocate or carry a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the workspace pair, same kernels,
 * same results; the output-averaged second layer lives in a static device array inside the library
 * (PAFU_SCORE_STATIC_MAX_M + 1 floats, 256-byte aligned, one copy per GPU, held until the process ends).  The call
 * allocates nothing and synchronises nothing.  M > PAFU_SCORE_STATIC_MAX_M returns PAFU_ERR_WORKSPACE with nothing
 * enqueued.  Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU (different streams
 * or host threads) race on it unless n_out == 1, where the array is not used; each call rewrites all M + 1 entries it
 * reads, so nothing needs clearing between calls.
 */
#define PAFU_SCORE_STATIC_MAX_M 8192
int pafu_score_static(void* stream, const void* x0, const void* x1, const void* x2, int n_seg, int T, int Fs,
                      long long ld_x, int x_dtype, const void* W1, const float* b1, const float* W2,
                      const float* b2, int M, int n_out, int act, float* out);

/* ------------------------------------------------------------------------------------------
 * pafu_select_topk - top-k retention, Sec. 3.4 inference paragraph; Alg. 2 (Top-k of the score list).
 *
 * Writes the indices of the min(k, n) highest scores in ASCENDING index order.  Total order:
 * higher score first; equal scores -> lower token index first; -0.0 == +0.0; NaN below -inf.
 * The result is a pure function of the score bits (no dependence on scheduling).
 *   scores    : [n] fp32          out_ids : [min(k, n)] int32
 *   out_count : device int32 receiving min(k, n), or NULL
 *   workspace : pafu_select_workspace_bytes(n) bytes
 * n == 0 or k == 0 writes no index (out_count still receives 0).
 */
size_t pafu_select_workspace_bytes(int n);
int pafu_select_topk(void* stream, const float* scores, int n, int k, int* out_ids, int* out_count,
                     void* workspace, size_t workspace_bytes);

/* pafu_select_topk_pinned - the same retention with a frame sink (Sec. 4 "Experimental Implementation"; the
 * frame-sink ablation): tokens [0, n_pinned) are never evicted and count towards the budget, i.e. they rank above
 * every score (lower index first among themselves); the other k - n_pinned places go to the most salient of the
 * remaining tokens.  k < n_pinned keeps tokens [0, k).  n_pinned = 0 is pafu_select_topk; n_pinned < 0 is an error.
 */
int pafu_select_topk_pinned(void* stream, const float* scores, int n, int k, int n_pinned, int* out_ids,
                            int* out_count, void* workspace, size_t workspace_bytes);

/* ------------------------------------------------------------------------------------------
 * pafu_compact_kv - cache update KV <- Select(KV; ids), SL <- Select(SL; ids), Alg. 2.
 *
 *   K_out[r] = K[ids[r]],  V_out[r] = V[ids[r]],  SL_out[r] = SL[ids[r]]     r in [0, count)
 * Bit copies.  Out of place (the caller ping-pongs two slabs).
 *   K, V      : [n, N, D] dtype `dtype` (bf16, fp32, or 8-bit codes), token stride ld_in elements
 *   SL/SL_out : [n] / [count] fp32, both NULL to skip the score list
 *   ids       : [count] int32 (device); an id outside [0, n) leaves that output row untouched
 *   K_out,V_out : [count, N, D], token stride ld_out elements
 * count == 0 is a no-op.
 */
int pafu_compact_kv(void* stream, const void* K, const void* V, const float* SL, long long ld_in, int n,
                    const int* ids, int count, int N, int D, int dtype, void* K_out, void* V_out,
                    float* SL_out, long long ld_out);

/* pafu_compact_kv_counted - the same with the row count read on the device: `count` is a device int32 (what
 * pafu_select_topk writes to out_count), so selection and compaction can be enqueued without a host round trip when
 * the count is not known on the host.  At most max_count rows are moved (the capacity of ids and of the outputs, and
 * what the launch is sized for); a negative device count moves nothing.  max_count <= n. */
int pafu_compact_kv_counted(void* stream, const void* K, const void* V, const float* SL, long long ld_in, int n,
                            const int* ids, const int* count /* device */, int max_count, int N, int D, int dtype,
                            void* K_out, void* V_out, float* SL_out, long long ld_out);

/* ------------------------------------------------------------------------------------------
 * pafu_chunk_attention - attention of the chunk's queries over retained cache + chunk.
 * Sec. 3.2 (P = softmax(Q K^T / sqrt(D)), block boundaries from L_B); App. A (L_B = chunk length).
 *
 *   O[i,h,:] = sum_j softmax_j( scale * q[i,h].k[j,h] + mask(i,j) ) v[j,h]
 * keys j run over the n_kept retained rows (all visible) followed by the Lc chunk rows; chunk key j
 * is visible to query i iff floor(j / block_len) <= floor(i / block_len).  The two key segments are
 * read in place (no concatenation copy).
 *   Q  : [Lq, N, D] bf16, stride ld_q      Kc,Vc : [n_kept, N, D] bf16, stride ld_c (may be NULL if n_kept == 0)
 *   Kn,Vn : [Lc, N, D] bf16, stride ld_n   O : [Lq, N, D] of out_dtype (bf16 or fp32), stride ld_o
 *   softmax_scale <= 0 means 1/sqrt(D).    D must be 64 or 128.  Lq >= 1, Lc >= 1, block_len >= 1.
 *   Query i is chunk token i (Lq <= Lc on this path).  The tensors may be of any size, but 64 consecutive K/V rows
 *   must span less than 4 GiB (ld_c, ld_n below 2^25 elements), else PAFU_ERR_SHAPE.
 *   workspace : optional (NULL / 0 allowed).  With pafu_attention_workspace_bytes(Lq, N, D) bytes (16-byte aligned,
 *               apart from every tensor of the call) a launch whose (head, 256-query tile) items would fill at most
 *               four fifths of the GPU's compute units cuts its work into equal runs over the key axis, one per
 *               compute unit, and merges the partial results in a second pass: the same result up to the rounding
 *               of the softmax weights, several times faster for short chunks over a long cache.  The contents of
 *               the workspace need not be initialised and are not kept.  Results do not depend on timing either way.
 */
size_t pafu_attention_workspace_bytes(int Lq, int N, int D);
int pafu_chunk_attention(void* stream, const void* Q, int Lq, const void* Kc, const void* Vc, int n_kept,
                         const void* Kn, const void* Vn, int Lc, int N, int D, long long ld_q,
                         long long ld_c, long long ld_n, long long ld_o, int block_len,
                         float softmax_scale, void* O, int out_dtype, void* workspace,
                         size_t workspace_bytes);

/* pafu_chunk_attention_gather - the same attention with index-based Select (Sec. 3.4; Eq. 7): the cache stays
 * uncompacted and the retained rows are read through an index list, so no compaction pass precedes the call.
 *   K_cache, V_cache : [n_cache, N, D] bf16, stride ld_c      ids : [n_kept] int32 (device, 16-byte aligned)
 * Retained row r is cache row ids[r]; O equals pafu_chunk_attention on the cache compacted to ids (the order of
 * ids does not matter to the result beyond summation order).  An id outside [0, n_cache) is clamped into the range
 * (no access leaves the cache; the output is then meaningless).  n_kept <= n_cache, and a cache tensor must span
 * less than 4 GiB (n_cache * ld_c * 2 bytes).  Everything else as above.
 */
int pafu_chunk_attention_gather(void* stream, const void* Q, int Lq, const void* K_cache, const void* V_cache,
                                int n_cache, const int* ids, int n_kept, const void* Kn, const void* Vn, int Lc,
                                int N, int D, long long ld_q, long long ld_c, long long ld_n, long long ld_o,
                                int block_len, float softmax_scale, void* O, int out_dtype, void* workspace,
                                size_t workspace_bytes);

/* ------------------------------------------------------------------------------------------
 * 8-bit storage of the K/V cache (beyond the paper, whose App. A states no storage precision).
 *
 * pafu_quantize_kv: K_q[r, e] = E4M3 code of K[r, e] / 2^k_scale_log2 (round to nearest even, magnitudes beyond 448
 * saturate, NaN stays NaN, the sign of zero is kept), likewise V.  pafu_dequantize_kv is the exact way back
 * (code * 2^scale as bf16; exact for every code and scale).
 *   K, V     : [rows, N, D] bf16, token stride ld_in (ld_out for dequantize) elements; N * D a multiple of 8
 *   K_q, V_q : [rows, N * D] bytes, token stride ld_out (ld_in for dequantize) bytes, a multiple of 16
 * pafu_compact_kv moves such rows with dtype = PAFU_FP8_E4M3 (strides in bytes).
 *
 * pafu_chunk_attention_fp8: pafu_chunk_attention with BOTH key segments stored as codes (ld_c, ld_n in bytes;
 * D = 128 only).  Tiles travel as codes, half the bytes of bf16, and are widened to bf16 (times the scale, exact) in
 * LDS before the matrix instructions read them; products, softmax and accumulation are those of the bf16 call.
 */
int pafu_quantize_kv(void* stream, const void* K, const void* V, long long ld_in, int rows, int N, int D,
                     int k_scale_log2, int v_scale_log2, void* K_q, void* V_q, long long ld_out);
int pafu_dequantize_kv(void* stream, const void* K_q, const void* V_q, long long ld_in, int rows, int N, int D,
                       int k_scale_log2, int v_scale_log2, void* K, void* V, long long ld_out);
int pafu_chunk_attention_fp8(void* stream, const void* Q, int Lq, const void* Kc_q, const void* Vc_q, int n_kept,
                             const void* Kn_q, const void* Vn_q, int Lc, int N, int D, long long ld_q, long long ld_c,
                             long long ld_n, long long ld_o, int block_len, float softmax_scale, int k_scale_log2,
                             int v_scale_log2, void* O, int out_dtype, void* workspace, size_t workspace_bytes);

/* ------------------------------------------------------------------------------------------
 * pafu_sse_score - Spatialtemporal-balanced Salience Estimation, the teacher-side score that the Salience
 * Estimation Head is trained to predict (Sec. 3.2, Eq. 4-5).
 *
 *   P = softmax(scale * Q K^T) per head over all L keys (no mask: a bidirectional pass).  b(i) = floor(i/block_len).
 *   low[j]  = mean_h max_{i : b(i) > b(j)} P[h,i,j]     diag[j] = mean_h max_{i : b(i) = b(j)} P[h,i,j]
 *   up[j]   = mean_h max_{i : b(i) < b(j)} P[h,i,j]
 *   s[j]    = mean of the parts whose query set is not empty: (diag+low)/2 in the first block, (up+diag+low)/3 in
 *             the middle, (diag+up)/2 in the last block (Eq. 5); a single block gives diag.
 *   Q, K : [L, N, D] bf16, strides ld_q / ld_k elements (each tensor must span less than 4 GiB)
 *   out  : [L] fp32       D must be 64 or 128       softmax_scale <= 0 means 1/sqrt(D)
 *   workspace : pafu_sse_workspace_bytes(L, N) bytes (per-query softmax normalisers and per-head partial maxima)
 * The L x L matrix is never materialised.  L == 0 is a no-op.
 */
size_t pafu_sse_workspace_bytes(int L, int N);
int pafu_sse_score(void* stream, const void* Q, const void* K, int L, int N, int D, long long ld_q, long long ld_k,
                   int block_len, float softmax_scale, float* out, void* workspace, size_t workspace_bytes);

/* ------------------------------------------------------------------------------------------
 * pafu_step - one chunk step of one layer on one stream, Alg. 2; Sec. 3.4.
 *
 * SINGLE : scores the n cached tokens and the Lc chunk tokens (scores[0:n], scores[n:n+Lc]),
 *          selects the top-k of the fresh cache scores, compacts K/V/SL into the output slab,
 *          attends over the n_kept = min(k, n) retained rows + the chunk.
 * ROLLOUT: scores only the chunk; selects on the STORED list SL_in (never refreshed); compacts into
 *          the output slab rows [0, n_kept); attends; then appends the chunk's K/V rows and scores at
 *          rows [n_kept, n_kept + Lc) of the output slab.  The caller swaps slabs for the next chunk,
 *          whose cache size is n_kept + Lc, so old and new tokens compete at the next selection.
 * All K/V tensors are bf16.  Feature tensors are x_dtype.
 */
typedef struct pafu_step_args {
  int mode;            /* pafu_mode */
  int N, D;            /* heads, head dim */
  int n;               /* cached tokens on entry */
  int Lc;              /* chunk tokens (= queries) */
  int k;               /* budget */
  int block_len;       /* L_B */
  int M, n_out, act;   /* S-MLP hidden width, outputs, pafu_act */
  int n_seg, Fs;       /* feature segments and width of each */
  int x_dtype;         /* pafu_dtype of features and W1 */
  int out_dtype;       /* pafu_dtype of O */
  float softmax_scale; /* <= 0 -> 1/sqrt(D) */
  long long ld_x;      /* feature row stride (elements) */
  long long ld_cache;  /* token stride of K_cache/V_cache (elements) */
  long long ld_out;    /* token stride of K_out/V_out */
  long long ld_chunk;  /* token stride of Q, K_chunk, V_chunk */
  long long ld_o;      /* token stride of O */
  /* features: SINGLE scores x_cache* (n rows) and x_chunk* (Lc rows); ROLLOUT only x_chunk* */
  const void* x_cache[3];
  const void* x_chunk[3];
  const void* W1; const float* b1; const float* W2; const float* b2;
  const void* K_cache; const void* V_cache; /* [n, N, D] bf16 */
  const float* SL_in;                       /* [n] stored scores (ROLLOUT) */
  const void* Q; const void* K_chunk; const void* V_chunk; /* [Lc, N, D] bf16 */
  float* scores;       /* SINGLE: [n + Lc] out.  ROLLOUT: unused (may be NULL) */
  int* ids;            /* [min(k, n)] out */
  void* K_out; void* V_out; /* [min(k,n) (+ Lc in ROLLOUT), N, D] bf16 out */
  float* SL_out;       /* [min(k,n) (+ Lc in ROLLOUT)] out */
  void* O;             /* [Lc, N, D] out */
  void* workspace; size_t workspace_bytes; /* >= pafu_step_workspace_bytes(args) */
  int n_pinned;        /* frame sink: cached tokens [0, n_pinned) are never evicted (0 = none) */
  /* Optional timing hooks (host handles, hipEvent_t passed as void*, each NULL = not recorded): recorded on the
   * step's stream before scoring [0], after scoring [1], after selection [2], after compaction [3] and after
   * attention [4] (ROLLOUT: the selection reads the stored list only and is done by one workgroup of the scoring
   * launch when that launch is a short streaming one and the list holds at most 65536 scores, so [1]..[2] is then
   * empty; the chunk rows are appended by the compaction launch, i.e. inside [2]..[3]; only when the
   * cache was empty, or the rows do not fit that kernel, a separate copy follows [4]).  In the multi-layer steps, whose stages are reordered across
   * layers, [0]/[1] bracket a layer's scoring and [3]/[4] its attention launch; [2] is recorded once, after the
   * selection launch, on args[0] (pafu_step_layers) or on the index layer (pafu_step_layers_shared). */
  void* stage_events[5];
  /* Storage of the K/V cache: PAFU_BF16 (0, the default) or PAFU_FP8_E4M3.  With the 8-bit format K_cache, V_cache,
   * K_out and V_out hold codes (ld_cache / ld_out count bytes; D must be 128), K_chunk / V_chunk / Q stay bf16, and
   * K_out / V_out need room for min(k, n) + Lc rows in BOTH modes: the chunk's K/V are quantised behind the retained
   * rows before attention, so that the chunk attends over exactly the values later steps find in the cache (in
   * ROLLOUT nothing is left to append; in SINGLE the rows are simply there).  Compaction moves codes. */
  int kv_dtype;
  int k_scale_log2, v_scale_log2; /* a stored code c stands for c * 2^scale_log2 (K and V each; within [-64, 64]) */
} pafu_step_args;

/* Workspace of a step = the scoring part (only when n_out > 1; required) followed by the attention part (optional:
 * see pafu_chunk_attention).  pafu_step_workspace_bytes returns the size of both; a workspace that only covers the
 * scoring part is accepted and the attention launch then runs without its equal-run split. */
size_t pafu_step_workspace_bytes(const pafu_step_args* args /* host */);
int pafu_step(void* stream, const pafu_step_args* args /* host */);
/* The same step for n_layers independent layers (args[l] is layer l's arguments), enqueued on one stream.
 * The layers' stages are NOT enqueued layer by layer: every layer is scored first, then all selections run in one
 * launch (up to 32 score lists per launch), then all compactions (one launch per 32 layers when the layers share
 * n, k, N, D, the strides and the storage type; layer by layer otherwise), then attention layer by layer.  Every layer
 * therefore needs its own scores, ids, SL_out, K_out, V_out and O buffers, and no layer's output may overlap
 * another layer's input (PAFU_ERR_ALIAS); only the workspace may be shared between layers. */
int pafu_step_layers(void* stream, const pafu_step_args* args /* host array */, int n_layers);

/* pafu_step_layers_shared - the paper's own multi-layer arrangement (Sec. 3.3: the Salience Estimation Head sits on
 * the final layer only and its top-k indices are applied to the caches of all layers).
 * args[index_layer] is a complete pafu_step_args: its features, head weights and score buffers produce the scores and
 * ONE index list (written to its `ids`).  Every layer then compacts its own K/V cache to those indices, attends, and in
 * ROLLOUT appends its chunk rows.  For the other layers only the cache part is read (mode, n, k, Lc - which must
 * equal the index layer's - N, D, block_len, softmax_scale, out_dtype, ld_cache/ld_out/ld_chunk/ld_o, K_cache,
 * V_cache, Q, K_chunk, V_chunk, K_out, V_out, O); their feature, weight, score, ids and SL fields are ignored and
 * may be NULL.  The score list is compacted and extended for the index layer only.
 * The index layer's scoring and the selection are enqueued first, then the layers' caches in array order, on one
 * stream; outputs of one layer must not overlap inputs or outputs of another (PAFU_ERR_ALIAS).
 */
int pafu_step_layers_shared(void* stream, const pafu_step_args* args /* host array */, int n_layers,
                            int index_layer);

#ifdef __cplusplus
}
#endif
#endif /* PAFU_H_ */

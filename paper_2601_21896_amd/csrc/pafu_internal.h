// Internal helpers shared by the HIP translation units of libpafu (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "pafu.h"

namespace pafu {

// Records a failed HIP call for pafu_last_hip_error(); returns PAFU_ERR_HIP.
int record_hip_error(hipError_t e);

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int check_launch() {
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? PAFU_OK : record_hip_error(e);
}

// Raises a kernel's dynamic LDS limit exactly once per process, whichever host thread launches it first.
struct LdsLimit {
  std::once_flag once;
  hipError_t err = hipSuccess;
};
template <typename Kernel>
inline int set_lds_limit(LdsLimit& state, Kernel kernel, int bytes) {
  std::call_once(state.once, [&] {
    state.err = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  });
  return state.err == hipSuccess ? PAFU_OK : record_hip_error(state.err);
}

inline bool overlaps(const void* a, size_t a_bytes, const void* b, size_t b_bytes) {
  uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
  return a_bytes && b_bytes && a0 < b0 + b_bytes && b0 < a0 + a_bytes;
}

// Stage launchers (validated arguments only).
// Rows that the compaction copies, in order, behind the gathered ones (output rows count, count + 1, ...): the chunk
// that a rollout appends to the compacted cache (Alg. 2), moved by the same launch.
struct CompactTail {
  const char* K;
  const char* V;
  long long ld;  // bytes between rows
  int rows;
  // quant != 0: the tail rows are bf16 and the output rows 8-bit codes (E4M3 of value * inv_k / inv_v): the chunk of a
  // step with the 8-bit cache, quantised behind the retained codes by the same launch
  int quant;
  float inv_k, inv_v;
};
bool compact_takes_tail(int row_bytes);  // rows of whole 16-byte chunks, up to 12 KiB
int launch_compact(hipStream_t st, const void* K, const void* V, const float* SL, long long ld_in_bytes, int n,
                   const int* ids, int count, int row_bytes, void* K_out, void* V_out, float* SL_out,
                   long long ld_out_bytes, const int* count_dev = nullptr, const CompactTail* tail_rows = nullptr);
// One layer of a batched compaction: its cache tensors, output slabs, index list and (optionally) score list.
struct CompactLayer {
  const char* K;
  const char* V;
  char* Ko;
  char* Vo;
  const int* ids;
  const float* SL;  // null: no score list for this layer
  float* SLo;
  const char* Kt;   // rows copied in order behind the gathered ones (the chunk a rollout appends); unused when the
  const char* Vt;   // launch has no tail rows
};
constexpr int kCompactBatchMax = 32;  // layers per launch (they travel as kernel arguments)
struct CompactBatch {
  CompactLayer layer[kCompactBatchMax];
};
// Rows up to 4 KiB and a multiple of 16 bytes can go through the batched kernel.
bool compact_batchable(int row_bytes);
// The layers share n, count, the row size and both strides.
int launch_compact_batch(hipStream_t st, const CompactLayer* layers, int n_layers, long long ld_in_bytes, int n,
                         int count, int row_bytes, long long ld_out_bytes, int tail_rows = 0,
                         long long ld_tail_bytes = 0);
int launch_append(hipStream_t st, const void* K, const void* V, const float* S, long long ld_in_bytes, int rows,
                  int row_bytes, void* K_out, void* V_out, float* S_out, long long ld_out_bytes);
// One top-k selection: scores [n] -> the min(k, n) retained indices, ascending (out_count may be null).
struct SelectJob {
  const float* scores;
  int* out_ids;
  int* out_count;
  int n;
  int k;
  int n_pinned;  // tokens [0, n_pinned) rank above every score
};
constexpr int kSelectBatchMax = 32;  // lists per launch (the jobs travel as kernel arguments)
// Independent lists, one workgroup each, in as few launches as possible.
int launch_select_batch(hipStream_t st, const SelectJob* jobs, int count);
int launch_select(hipStream_t st, const float* scores, int n, int k, int n_pinned, int* out_ids, int* out_count,
                  void* ws);
int launch_score(hipStream_t st, const void* x0, const void* x1, const void* x2, int n_seg, int T, int Fs,
                 long long ld_x, int x_dtype, const void* W1, const float* b1, const float* W2, const float* b2,
                 int M, int n_out, int act, float* out, void* ws, const SelectJob* ride = nullptr,
                 bool* rode = nullptr);
// `ride`: a selection that does not depend on these scores (the stored list of a rollout step); when the launch is a
// short streaming one it is done by one extra workgroup of the same launch and *rode is set, otherwise the caller
// launches it.
// The same with the folded second layer in the library's own static device array (no workspace, no allocation).
int launch_score_static(hipStream_t st, const void* x0, const void* x1, const void* x2, int n_seg, int T, int Fs,
                        long long ld_x, int x_dtype, const void* W1, const float* b1, const float* W2,
                        const float* b2, int M, int n_out, int act, float* out);
size_t sse_workspace_bytes(int L, int N);
int launch_sse(hipStream_t st, const void* Q, const void* K, int L, int N, int D, long long ld_q, long long ld_k,
               int block_len, float scale, float* out, void* workspace);
// workspace (may be null): with attention_workspace_bytes(D) bytes the launch may cut its work into equal runs.
size_t attention_workspace_bytes(int D);
int attention_study_build();  // 0 in the shipped library; the ablation mask of a study build
int launch_attention(hipStream_t st, const void* Q, int Lq, const void* Kc, const void* Vc, int n_kept,
                     const void* Kn, const void* Vn, int Lc, int N, int D, long long ld_q, long long ld_c,
                     long long ld_n, long long ld_o, int block_len, float scale, void* O, int out_dtype,
                     void* workspace, size_t workspace_bytes, const int* ids = nullptr, int n_cache = 0,
                     int kv_dtype = PAFU_BF16, float k_scale = 1.f, float v_scale = 1.f);
// bf16 rows -> E4M3 codes (code = round(x / 2^scale_log2), saturating) and back; row_elems = N * D, strides in bytes.
int launch_quantize(hipStream_t st, const void* K, const void* V, long long ld_in_bytes, int rows, int row_elems,
                    int k_scale_log2, int v_scale_log2, void* Kq, void* Vq, long long ld_out_bytes);
int launch_dequantize(hipStream_t st, const void* Kq, const void* Vq, long long ld_in_bytes, int rows, int row_elems,
                      int k_scale_log2, int v_scale_log2, void* K, void* V, long long ld_out_bytes);
// Compute units of the current GPU (cached per device; 256 if the query fails).
int compute_units();

}  // namespace pafu

// Top-k retention: indices of the k highest salience scores, ascending, ties to the lower index.
// Sec. 3.4 (inference) and Alg. 2 of the paper: Top-k over the salience score list.
//
// Radix select on an order-preserving 32-bit key, then an ordered emit: every index whose key is above
// the k-th largest key T is written, plus the first `need_eq` indices whose key equals T.  The output
// position of an element is  (#keys > T before it) + min(#keys == T before it, need_eq), which block-wide
// prefix scans provide, so the result depends only on the score bits, never on atomic arrival order.
//
// The whole score list is a few hundred KB at most (one fp32 per cached token), so the work is
// latency-bound and one workgroup handles one list.  Lists of up to 98304 scores use the bit-sliced
// kernel: each thread loads its 32 W consecutive keys ONCE and transposes them into 32 bit-planes of W
// words; a radix-2 pass is then two instructions per word (and + popcount) plus one block-wide sum, and
// the "greater" and "equal" masks the emit needs fall out of the 32 passes.  Longer lists fall back to
// four 8-bit passes with LDS histograms that re-read the list from L2.
// The bit-sliced device code lives in select_body.h (the scoring kernel of a rollout step carries it along).
#include "pafu_internal.h"
#include "select_body.h"

namespace pafu {
namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelTile = kSelThreads * 4;


__device__ __forceinline__ void select_topk_body(const SelectProblem& P) {
  __shared__ uint32_t hist[kSelWaves][256];
  __shared__ uint32_t wave_tot[kSelWaves];
  __shared__ uint32_t s_prefix, s_remaining;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = P.n;
  const float* __restrict__ scores = P.scores;
  int* __restrict__ out = P.out_ids;

  if (P.k >= n) {  // budget covers the whole cache: keep everything
    for (int i = tid; i < n; i += kSelThreads) out[i] = i;
    if (tid == 0 && P.out_count) *P.out_count = n;
    return;
  }
  if (P.k <= 0) {
    if (tid == 0 && P.out_count) *P.out_count = 0;
    return;
  }

  uint32_t prefix = 0, remaining = (uint32_t)P.k;
#pragma unroll 1
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    for (int i = tid; i < kSelWaves * 256; i += kSelThreads) (&hist[0][0])[i] = 0u;
    __syncthreads();
    for (int i = tid; i < n; i += kSelThreads) {
      const uint32_t key = token_key(scores[i], i, P.n_pinned);
      const bool match = (pass == 0) || ((key >> (shift + 8)) == prefix);
      if (match) atomicAdd(&hist[wave][(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (wave == 0) {
      uint32_t c[4], tot = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        uint32_t s = 0;
#pragma unroll
        for (int w = 0; w < kSelWaves; ++w) s += hist[w][4 * lane + j];
        c[j] = s;
        tot += s;
      }
      uint32_t incl = tot;  // suffix sum over lanes: keys whose digit is in a higher lane's bins
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const uint32_t t = __shfl_down(incl, off);
        if (lane + off < 64) incl += t;
      }
      uint32_t above = incl - tot;
#pragma unroll
      for (int j = 3; j >= 0; --j) {
        if (above < remaining && remaining <= above + c[j]) {
          s_prefix = (prefix << 8) | (uint32_t)(4 * lane + j);
          s_remaining = remaining - above;
        }
        above += c[j];
      }
    }
    __syncthreads();
    prefix = s_prefix;
    remaining = s_remaining;
  }

  const uint32_t T = prefix;          // key of the k-th best token
  const uint32_t need_eq = remaining; // how many tokens with key == T are kept (>= 1)
  uint32_t base_gt = 0, base_eq = 0;
#pragma unroll 1
  for (int base = 0; base < n; base += kSelTile) {
    const int i0 = base + 4 * tid;
    uint32_t key[4];
    bool valid[4];
    if (i0 + 3 < n) {
      const float4 f = *reinterpret_cast<const float4*>(scores + i0);
      key[0] = token_key(f.x, i0, P.n_pinned); key[1] = token_key(f.y, i0 + 1, P.n_pinned);
      key[2] = token_key(f.z, i0 + 2, P.n_pinned); key[3] = token_key(f.w, i0 + 3, P.n_pinned);
      valid[0] = valid[1] = valid[2] = valid[3] = true;
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        valid[j] = i0 + j < n;
        key[j] = valid[j] ? token_key(scores[i0 + j], i0 + j, P.n_pinned) : 0u;
      }
    }
    uint32_t packed = 0;  // low 16 bits: keys > T, high 16 bits: keys == T (a tile holds 4096 keys)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (valid[j] && key[j] > T) packed += 1u;
      if (valid[j] && key[j] == T) packed += 1u << 16;
    }
    uint32_t incl = packed;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t t = __shfl_up(incl, off);
      if (lane >= off) incl += t;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t before = 0, tile_tot = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
      const uint32_t t = wave_tot[w];
      if (w < wave) before += t;
      tile_tot += t;
    }
    const uint32_t excl = before + incl - packed;
    uint32_t my_gt = base_gt + (excl & 0xffffu);
    uint32_t my_eq = base_eq + (excl >> 16);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (valid[j] && key[j] > T) {
        out[my_gt + (my_eq < need_eq ? my_eq : need_eq)] = i0 + j;
        ++my_gt;
      } else if (valid[j] && key[j] == T) {
        if (my_eq < need_eq) out[my_gt + my_eq] = i0 + j;
        ++my_eq;
      }
    }
    base_gt += tile_tot & 0xffffu;
    base_eq += tile_tot >> 16;
    __syncthreads();  // wave_tot is rewritten by the next tile
  }
  if (tid == 0 && P.out_count) *P.out_count = P.k;
}


// One score list per workgroup: the single-list entry points launch one workgroup, the multi-layer steps one per
// layer (the lists are independent, and a list only ever occupies one CU).
struct SelectBatch {
  SelectProblem job[kSelectBatchMax];
};
template <int W, int NT>
__global__ __launch_bounds__(NT) void select_bitslice_kernel(SelectBatch B) {
  select_bitslice_body<W, NT>(B.job[blockIdx.x]);
}
__global__ __launch_bounds__(kSelThreads) void select_topk_kernel(SelectBatch B) { select_topk_body(B.job[blockIdx.x]); }

}  // namespace

int launch_select_batch(hipStream_t st, const SelectJob* jobs, int count) {
  for (int first = 0; first < count; first += kSelectBatchMax) {
    const int m = count - first < kSelectBatchMax ? count - first : kSelectBatchMax;
    SelectBatch B;
    int n_max = 0;
    for (int i = 0; i < m; ++i) {
      B.job[i] = jobs[first + i];
      if (B.job[i].n < 0) B.job[i].n = 0;
      if (B.job[i].n_pinned < 0) B.job[i].n_pinned = 0;
      n_max = B.job[i].n > n_max ? B.job[i].n : n_max;
    }
    for (int i = m; i < kSelectBatchMax; ++i) B.job[i] = B.job[0];  // never read: the grid has m workgroups
    // the longest list picks the kernel (keys per thread x threads must cover it)
#define PAFU_SELECT_CASE(W, NT)                                                                                   \
  do {                                                                                                            \
    static LdsLimit lds_limit;                                                                                    \
    const int rc_ = set_lds_limit(lds_limit, select_bitslice_kernel<W, NT>, select_bitslice_lds_bytes(NT));       \
    if (rc_ != PAFU_OK) return rc_;                                                                               \
    hipLaunchKernelGGL((select_bitslice_kernel<W, NT>), dim3(m), dim3(NT), select_bitslice_lds_bytes(NT), st, B); \
  } while (0)
    if (n_max <= 256 * 32) PAFU_SELECT_CASE(1, 256);
    else if (n_max <= 512 * 32 * 2) PAFU_SELECT_CASE(2, 512);
    else if (n_max <= 1024 * 32 * 2) PAFU_SELECT_CASE(2, 1024);
    else if (n_max <= 1024 * 32 * 3) PAFU_SELECT_CASE(3, 1024);
    else hipLaunchKernelGGL(select_topk_kernel, dim3(m), dim3(kSelThreads), 0, st, B);
#undef PAFU_SELECT_CASE
    int rc = check_launch();
    if (rc) return rc;
  }
  return PAFU_OK;
}

int launch_select(hipStream_t st, const float* scores, int n, int k, int n_pinned, int* out_ids, int* out_count,
                  void* ws) {
  (void)ws;
  if (n <= 0 || k <= 0) {
    if (out_count == nullptr) return PAFU_OK;
  }
  const SelectJob job{scores, out_ids, out_count, n, k, n_pinned};
  return launch_select_batch(st, &job, 1);
}

}  // namespace pafu

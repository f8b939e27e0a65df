// Top-k retention: indices of the k highest salience scores, ascending, ties to the lower index.
// Sec. 3.4 (inference) and Alg. 2 of the paper: Top-k over the salience score list.
//
// Radix select on an order-preserving 32-bit key, then an ordered emit: every index whose key is above
// the k-th largest key T is written, plus the first `need_eq` indices whose key equals T.  The output
// position of an element is  (#keys > T before it) + min(#keys == T before it, need_eq), which block-wide
// prefix scans provide, so the result depends only on the score bits, never on atomic arrival order.
//
// The whole score list is a few hundred KB at most (one fp32 per cached token), so the work is
// latency-bound and one workgroup handles one list.  Lists of up to 81920 scores use the bit-sliced
// kernel: each thread loads its 32 W consecutive keys ONCE and transposes them into 32 bit-planes of W
// words; a radix-2 pass is then two instructions per word (and + popcount) plus one block-wide sum, and
// the "greater" and "equal" masks the emit needs fall out of the 32 passes.  Longer lists fall back to
// four 8-bit passes with LDS histograms that re-read the list from L2.
#include "pafu_internal.h"

namespace pafu {
namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelTile = kSelThreads * 4;

typedef SelectJob SelectProblem;  // {scores, out_ids, out_count, n, k, n_pinned}

// fp32 -> uint32 such that key order == (score order with -0 == +0 and NaN lowest).
__device__ __forceinline__ uint32_t score_key(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;  // NaN
  if (u == 0x80000000u) u = 0u;                     // -0.0 -> +0.0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Key of token i: the pinned prefix gets the one key no score maps to (the map's maximum is +inf = 0xff800000),
// so pinned tokens outrank everything and, among themselves, the lower index wins like any other tie.
__device__ __forceinline__ uint32_t token_key(float f, int i, int n_pinned) {
  return i < n_pinned ? 0xffffffffu : score_key(f);
}

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

// ---------------------------------------------------------------------------------- bit-sliced kernel
// sum of v over the wave, as a wave-uniform value (row rotations inside each 16-lane row, then the four rows)
__device__ __forceinline__ int wave_sum(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x128, 0xf, 0xf, false);  // row_ror:8
  v += __builtin_amdgcn_update_dpp(0, v, 0x124, 0xf, 0xf, false);  // row_ror:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x122, 0xf, 0xf, false);  // row_ror:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x121, 0xf, 0xf, false);  // row_ror:1
  return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) + __builtin_amdgcn_readlane(v, 32) +
         __builtin_amdgcn_readlane(v, 48);
}

// in-place transpose of a 32 x 32 bit matrix: afterwards bit j of a[p] is bit p of the old a[j]
__device__ __forceinline__ void transpose32(uint32_t (&a)[32]) {
  uint32_t m = 0x0000ffffu;
#pragma unroll
  for (int j = 16; j != 0; j >>= 1, m ^= m << j) {
#pragma unroll
    for (int k = 0; k < 32; k = (k + j + 1) & ~j) {
      const uint32_t t = (a[k + j] ^ (a[k] >> j)) & m;
      a[k + j] ^= t;
      a[k] ^= t << j;
    }
  }
}

// W = 32-key words per thread, NT threads: the list holds at most NT * 32 * W scores.  Longer lists use fewer
// threads so that the W * 32 bit-plane registers fit.
template <int W, int NT>
__device__ __forceinline__ void select_bitslice_body(const SelectProblem& P) {
  constexpr int kWaves = NT / 64;
  __shared__ int part[2][kWaves];
  __shared__ uint32_t wave_tot[kWaves];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = P.n;
  const float* __restrict__ scores = P.scores;
  int* __restrict__ out = P.out_ids;

  if (P.k >= n) {  // budget covers the whole cache: keep everything
    for (int i = tid; i < n; i += NT) out[i] = i;
    if (tid == 0 && P.out_count) *P.out_count = n;
    return;
  }
  if (P.k <= 0) {
    if (tid == 0 && P.out_count) *P.out_count = 0;
    return;
  }

  // bit-planes of this thread's keys [32 W tid, 32 W (tid + 1)); keys past the end are 0 (the lowest key; their
  // indices are the highest, so with k < n they are never selected)
  uint32_t plane[W][32];
  const int first = 32 * W * tid;
#pragma unroll
  for (int w = 0; w < W; ++w) {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int i0 = first + 32 * w + 4 * q;
      if (i0 + 3 < n) {
        const float4 f = *reinterpret_cast<const float4*>(scores + i0);
        plane[w][4 * q + 0] = token_key(f.x, i0, P.n_pinned); plane[w][4 * q + 1] = token_key(f.y, i0 + 1, P.n_pinned);
        plane[w][4 * q + 2] = token_key(f.z, i0 + 2, P.n_pinned); plane[w][4 * q + 3] = token_key(f.w, i0 + 3, P.n_pinned);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          plane[w][4 * q + e] = i0 + e < n ? token_key(scores[i0 + e], i0 + e, P.n_pinned) : 0u;
      }
    }
    transpose32(plane[w]);
    if (W > 1) asm volatile("" ::: "memory");  // one word at a time: keeps the raw keys of later words out of registers
  }

  // radix-2 select from the most significant bit: cand = keys that still match the prefix of the k-th key
  uint32_t cand[W], gt[W];
#pragma unroll
  for (int w = 0; w < W; ++w) { cand[w] = 0xffffffffu; gt[w] = 0u; }
  int remaining = P.k;
#pragma unroll
  for (int p = 31; p >= 0; --p) {
    int cnt = 0;
#pragma unroll
    for (int w = 0; w < W; ++w) cnt += __builtin_popcount(cand[w] & plane[w][p]);
    const int wsum = wave_sum(cnt);
    if (lane == 0) part[p & 1][wave] = wsum;
    __syncthreads();
    int total = 0;
#pragma unroll
    for (int i = 0; i < kWaves; ++i) total += part[p & 1][i];
    if (total >= remaining) {  // the k-th key has this bit set
#pragma unroll
      for (int w = 0; w < W; ++w) cand[w] &= plane[w][p];
    } else {  // it does not: candidates with the bit set are above it
      remaining -= total;
#pragma unroll
      for (int w = 0; w < W; ++w) {
        gt[w] |= cand[w] & plane[w][p];
        cand[w] &= ~plane[w][p];
      }
    }
  }
  // now cand = keys equal to the k-th key, gt = keys above it, remaining = how many equal keys are kept (>= 1)
  const uint32_t need_eq = (uint32_t)remaining;
  uint32_t c_gt = 0, c_eq = 0;
#pragma unroll
  for (int w = 0; w < W; ++w) { c_gt += __builtin_popcount(gt[w]); c_eq += __builtin_popcount(cand[w]); }
  // block-wide exclusive scan of (c_gt, c_eq); a list holds at most 2^17 keys, so two 32-bit scans
  uint32_t in_gt = c_gt, in_eq = c_eq;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t a = __shfl_up(in_gt, off), b = __shfl_up(in_eq, off);
    if (lane >= off) { in_gt += a; in_eq += b; }
  }
  if (lane == 63) { wave_tot[wave] = in_gt; part[0][wave] = (int)in_eq; }
  __syncthreads();
  uint32_t my_gt = in_gt - c_gt, my_eq = in_eq - c_eq;
#pragma unroll
  for (int i = 0; i < kWaves; ++i)
    if (i < wave) { my_gt += wave_tot[i]; my_eq += (uint32_t)part[0][i]; }
  // ordered emit of this thread's keys
#pragma unroll
  for (int w = 0; w < W; ++w) {
    uint32_t todo = gt[w] | cand[w];
    while (todo) {
      const int j = __builtin_ctz(todo);
      todo &= todo - 1;
      const int idx = first + 32 * w + j;
      if ((gt[w] >> j) & 1u) {
        out[my_gt + (my_eq < need_eq ? my_eq : need_eq)] = idx;
        ++my_gt;
      } else {
        if (my_eq < need_eq) out[my_gt + my_eq] = idx;
        ++my_eq;
      }
    }
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
    if (n_max <= 256 * 32) hipLaunchKernelGGL((select_bitslice_kernel<1, 256>), dim3(m), dim3(256), 0, st, B);
    else if (n_max <= 512 * 32 * 2) hipLaunchKernelGGL((select_bitslice_kernel<2, 512>), dim3(m), dim3(512), 0, st, B);
    else if (n_max <= 1024 * 32 * 2) hipLaunchKernelGGL((select_bitslice_kernel<2, 1024>), dim3(m), dim3(1024), 0, st, B);
    else hipLaunchKernelGGL(select_topk_kernel, dim3(m), dim3(kSelThreads), 0, st, B);
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

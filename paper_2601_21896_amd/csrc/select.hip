// Top-k retention: indices of the k highest salience scores, ascending, ties to the lower index.
// Sec. 3.4 (inference) and Alg. 2 of the paper: Top-k over the salience score list.
//
// Radix select on an order-preserving 32-bit key: four 8-bit passes (most significant digit first)
// narrow down the k-th largest key T with LDS histograms; a final ordered pass emits every index
// whose key is above T plus the first `need_eq` indices whose key equals T.  The output position of
// an element is  (#keys > T before it) + min(#keys == T before it, need_eq), which block-wide prefix
// scans provide, so the result depends only on the score bits, never on atomic arrival order.
//
// The whole score list is a few hundred KB at most (one fp32 per cached token), so the work is
// latency-bound: one workgroup per score list re-reads it from L2 in every pass.
#include "pafu_internal.h"

namespace pafu {
namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelTile = kSelThreads * 4;

struct SelectProblem {
  const float* scores;
  int* out_ids;
  int* out_count;
  int n;
  int k;
};

// fp32 -> uint32 such that key order == (score order with -0 == +0 and NaN lowest).
__device__ __forceinline__ uint32_t score_key(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;  // NaN
  if (u == 0x80000000u) u = 0u;                     // -0.0 -> +0.0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ __launch_bounds__(kSelThreads) void select_topk_kernel(SelectProblem P) {
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
      const uint32_t key = score_key(scores[i]);
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
      key[0] = score_key(f.x); key[1] = score_key(f.y); key[2] = score_key(f.z); key[3] = score_key(f.w);
      valid[0] = valid[1] = valid[2] = valid[3] = true;
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        valid[j] = i0 + j < n;
        key[j] = valid[j] ? score_key(scores[i0 + j]) : 0u;
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

}  // namespace

int launch_select(hipStream_t st, const float* scores, int n, int k, int* out_ids, int* out_count, void* ws) {
  (void)ws;
  if (n <= 0 || k <= 0) {
    if (out_count == nullptr) return PAFU_OK;
  }
  SelectProblem P{scores, out_ids, out_count, n < 0 ? 0 : n, k};
  hipLaunchKernelGGL(select_topk_kernel, dim3(1), dim3(kSelThreads), 0, st, P);
  return check_launch();
}

}  // namespace pafu

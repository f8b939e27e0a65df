// Device code of the bit-sliced top-k selection (Sec. 3.4 and Alg. 2 of the paper: Top-k over the salience score
// list), shared by the selection kernels and by the scoring kernel that carries a selection along in a rollout step
// (there the selection reads stored scores only, so one workgroup of the scoring launch can do it meanwhile).
// One workgroup of NT threads handles one list; it uses the launch's dynamic LDS from offset 0
// (select_bitslice_lds_bytes(NT) bytes).
#pragma once
#include "pafu_internal.h"

namespace pafu {
namespace {

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

// in-place transpose of a 32 x 32 bit matrix: afterwards bit j of a[p] is bit p of the old a[j].  Each step swaps
// the high part of a[k] with the low part of a[k + j] at granularity j, written as two bit selects per pair.
__device__ __forceinline__ void transpose32(uint32_t (&a)[32]) {
  uint32_t m = 0x0000ffffu;
#pragma unroll
  for (int j = 16; j != 0; j >>= 1, m ^= m << j) {
#pragma unroll
    for (int k = 0; k < 32; k = (k + j + 1) & ~j) {
      const uint32_t lo = a[k], hi = a[k + j];
      a[k] = (lo & m) | ((hi << j) & ~m);
      a[k + j] = ((lo >> j) & m) | (hi & ~m);
    }
  }
}

// W = 32-key words per thread, NT threads: the list holds at most NT * 32 * W scores.  Word w of thread t holds
// the keys [32 (NT w + t), 32 (NT w + t) + 32): global memory is read with consecutive lanes on consecutive 16-byte
// chunks and handed to the owning thread through LDS (a thread reading its own 128 contiguous bytes straight from
// memory touches 64 cache lines per wave instruction, and that alone was 40 percent of the kernel); the indices
// leave the same way, collected in an LDS window and written out with consecutive lanes on consecutive words.
constexpr int select_bitslice_lds_bytes(int NT) { return NT * 128 + 4 * (NT / 64) * 8; }

template <int W, int NT>
__device__ __forceinline__ void select_bitslice_body(const SelectProblem& P) {
  constexpr int kWaves = NT / 64;
  constexpr int kWin = NT * 32;  // ids per emit window = words of the staging buffer
  extern __shared__ __attribute__((aligned(16))) unsigned char sel_lds[];
  uint32_t* const stage = reinterpret_cast<uint32_t*>(sel_lds);            // NT rows of 128 bytes
  int* const part = reinterpret_cast<int*>(sel_lds + NT * 128);            // [2][kWaves]
  uint32_t* const wave_gt = reinterpret_cast<uint32_t*>(part + 2 * kWaves);  // [kWaves], one word at a time
  uint32_t* const wave_eq = wave_gt + kWaves;                              // [kWaves]
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

  // bit-planes of this thread's keys; keys past the end are 0 (the lowest key; their indices are the highest, so
  // with k < n they are never selected).  Chunk c (4 keys) of row t sits in 16-byte slot c ^ ((t >> 1) & 7) of the
  // row, so that 16 consecutive threads reading the same chunk of their rows hit 16 different bank groups.
  // The raw score bits are staged and transposed; the map to keys (see score_key / token_key) is then applied to
  // the bit-planes, 32 keys per instruction: with P[b] the plane of bit b of the scores,
  //   nan = (all of P[23..30]) & (any of P[0..22]),  sign = P[31] & (any of P[0..30])      (-0 counts as +0)
  //   key bit b < 31 = P[b] ^ sign,  key bit 31 = ~sign,  all bits cleared for NaN and for entries past the end,
  //   all bits set for the pinned prefix.
  uint32_t plane[W][32];
  // With up to two words per thread all global loads are issued before the first word is processed, so that their
  // latency is paid once; with more, a word's loads are issued when its turn comes (registers).
  constexpr bool kLoadAhead = W <= 2;
  uint4 raw[kLoadAhead ? W : 1][8];
  auto load_word = [&](int w, uint4 (&dst)[8]) {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int i0 = 32 * NT * w + 4 * (q * NT + tid);
      if (i0 + 3 < n) {
        dst[q] = *reinterpret_cast<const uint4*>(scores + i0);
      } else {  // ragged end: entries past the end are masked out below
        dst[q].x = i0 + 0 < n ? __float_as_uint(scores[i0 + 0]) : 0u;
        dst[q].y = i0 + 1 < n ? __float_as_uint(scores[i0 + 1]) : 0u;
        dst[q].z = i0 + 2 < n ? __float_as_uint(scores[i0 + 2]) : 0u;
        dst[q].w = 0u;
      }
    }
  };
  if (kLoadAhead) {
#pragma unroll
    for (int w = 0; w < W; ++w) load_word(w, raw[kLoadAhead ? w : 0]);
  }
#pragma unroll
  for (int w = 0; w < W; ++w) {
    if (!kLoadAhead) load_word(w, raw[0]);
    if (w > 0) __syncthreads();  // everyone has read the previous word out of the staging rows
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int u = q * NT + tid;  // 16-byte chunk of this word's key range
      const int row = u >> 3, c = u & 7;
      *reinterpret_cast<uint4*>(stage + row * 32 + ((c ^ ((row >> 1) & 7)) << 2)) = raw[kLoadAhead ? w : 0][q];
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const uint4 v = *reinterpret_cast<const uint4*>(stage + tid * 32 + ((c ^ ((tid >> 1) & 7)) << 2));
      plane[w][4 * c + 0] = v.x; plane[w][4 * c + 1] = v.y; plane[w][4 * c + 2] = v.z; plane[w][4 * c + 3] = v.w;
    }
    transpose32(plane[w]);
    uint32_t mant = plane[w][0], expo = plane[w][23];
#pragma unroll
    for (int b = 1; b < 23; ++b) mant |= plane[w][b];
#pragma unroll
    for (int b = 24; b < 31; ++b) expo &= plane[w][b];
    uint32_t exp_any = plane[w][23];
#pragma unroll
    for (int b = 24; b < 31; ++b) exp_any |= plane[w][b];
    const int first = 32 * (NT * w + tid);
    const int n_here = n - first, pin_here = (P.n_pinned < n ? P.n_pinned : n) - first;
    const uint32_t valid = n_here >= 32 ? 0xffffffffu : (n_here <= 0 ? 0u : (1u << n_here) - 1u);
    const uint32_t pin = pin_here >= 32 ? 0xffffffffu : (pin_here <= 0 ? 0u : (1u << pin_here) - 1u);
    const uint32_t sign = plane[w][31] & (mant | exp_any);
    const uint32_t keep = valid & ~(expo & mant);
#pragma unroll
    for (int b = 0; b < 31; ++b) plane[w][b] = ((plane[w][b] ^ sign) & keep) | pin;
    plane[w][31] = (~sign & keep) | pin;
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
    if (lane == 0) part[(p & 1) * kWaves + wave] = wsum;
    __syncthreads();
    int total = 0;
#pragma unroll
    for (int i = 0; i < kWaves; ++i) total += part[(p & 1) * kWaves + i];
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

  // Ranks in index order = word by word, thread by thread inside a word: one block-wide exclusive scan of
  // (#above, #equal) per word, carried over the words.
  uint32_t my_gt[W], my_eq[W];
  uint32_t carry_gt = 0, carry_eq = 0;
#pragma unroll
  for (int w = 0; w < W; ++w) {
    const uint32_t c_gt = __builtin_popcount(gt[w]), c_eq = __builtin_popcount(cand[w]);
    uint32_t in_gt = c_gt, in_eq = c_eq;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t a = __shfl_up(in_gt, off), b2 = __shfl_up(in_eq, off);
      if (lane >= off) { in_gt += a; in_eq += b2; }
    }
    __syncthreads();  // the totals of the previous word (and the last radix pass) have been read
    if (lane == 63) { wave_gt[wave] = in_gt; wave_eq[wave] = in_eq; }
    __syncthreads();
    uint32_t before_gt = 0, before_eq = 0, tot_gt = 0, tot_eq = 0;
#pragma unroll
    for (int i = 0; i < kWaves; ++i) {
      const uint32_t a = wave_gt[i], b2 = wave_eq[i];
      if (i < wave) { before_gt += a; before_eq += b2; }
      tot_gt += a; tot_eq += b2;
    }
    my_gt[w] = carry_gt + before_gt + in_gt - c_gt;
    my_eq[w] = carry_eq + before_eq + in_eq - c_eq;
    carry_gt += tot_gt; carry_eq += tot_eq;
  }

  // Kept keys of a word: all keys above the k-th, and of the keys equal to it the first (need_eq - #equal before
  // this word) in index order.  The output position of a kept key is the number of kept keys before it.
  uint32_t kept[W], pos0[W];
#pragma unroll
  for (int w = 0; w < W; ++w) {
    const uint32_t allowed = my_eq[w] < need_eq ? need_eq - my_eq[w] : 0u;
    uint32_t eq = cand[w];
    while ((uint32_t)__builtin_popcount(eq) > allowed) eq &= ~(0x80000000u >> __builtin_clz(eq));  // drop the highest
    kept[w] = gt[w] | eq;
    pos0[w] = my_gt[w] + (my_eq[w] < need_eq ? my_eq[w] : need_eq);
  }

  // ordered emit through LDS windows of kWin ids.  Every position in [0, k) is written exactly once.
  __syncthreads();  // the staging rows are reused as the window
  int* const win = reinterpret_cast<int*>(stage);
  const bool out_vec = (reinterpret_cast<uintptr_t>(out) & 15u) == 0;
#pragma unroll 1
  for (int base = 0; base < P.k; base += kWin) {
#pragma unroll
    for (int w = 0; w < W; ++w) {
      const uint32_t lo = pos0[w], hi = lo + __builtin_popcount(kept[w]);
      if (hi > (uint32_t)base && lo < (uint32_t)base + kWin) {
        const int first = 32 * (NT * w + tid);
        uint32_t rel = lo - (uint32_t)base;  // wraps below the window: then the bound check fails
#pragma unroll
        for (int j = 0; j < 32; ++j) {
          const bool on = (kept[w] >> j) & 1u;
          if (on && rel < (uint32_t)kWin) win[rel] = first + j;
          rel += on ? 1u : 0u;
        }
      }
    }
    __syncthreads();
    const int m = P.k - base < kWin ? P.k - base : kWin;
    if (out_vec) {
      for (int i = 4 * tid; i < m; i += 4 * NT) {
        if (i + 3 < m) {
          *reinterpret_cast<int4*>(out + base + i) = *reinterpret_cast<const int4*>(win + i);
        } else {
          for (int e = 0; i + e < m; ++e) out[base + i + e] = win[i + e];
        }
      }
    } else {
      for (int i = tid; i < m; i += NT) out[base + i] = win[i];
    }
    __syncthreads();
  }
  if (tid == 0 && P.out_count) *P.out_count = P.k;
}

}  // namespace
}  // namespace pafu

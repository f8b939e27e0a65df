// pafu_sse_score: teacher-side salience score of every key from a bidirectional attention pass
// (Spatialtemporal-balanced Salience Estimation, Sec. 3.2, Eq. 4-5).
//
//   P = softmax(Q K^T / sqrt(D)) per head over the full key axis;  per key j and per relation of the query's block
//   to j's block (later = "low", same = "diag", earlier = "up"): max over those queries of P[h, i, j], mean over
//   heads; the score is the mean of the parts whose query set is not empty (Eq. 5).
//
// The L x L matrix is never stored.  Two flash-style passes over Q K^T on the matrix cores plus a small combine:
//   rowstat : per (head, query) c = log2 of the softmax denominator in the base-2 domain, i.e.
//             c_i = m_i + log2(sum_j 2^(z_ij - m_i)) with z = log2(e) * scale * q.k  -> P_ij = 2^(z_ij - c_i)
//   colmax  : per (head, key) the three maxima over queries of (z_ij - c_i); the maximum commutes with 2^x, so
//             the exponential is taken once per key and part at the end, not once per matrix element
//   combine : mean over heads, Eq. 5.
// Both passes are the same loop: one tensor is held in registers as the B operand of v_mfma_f32_32x32x16_bf16 (a
// lane owns one of its rows), the other streams global -> LDS in 64-row tiles (global_load_lds, 3 tiles in flight,
// XOR-swizzled 16-byte chunks) and is the A operand, so that everything a lane reduces over arrives in its own
// accumulator registers: rowstat holds 32 queries per wave and streams the keys (online log-sum-exp per lane),
// colmax holds 32 keys per wave and streams the queries together with their c values.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pafu.h"
#include "pafu_internal.h"

namespace pafu {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((address_space(3))) unsigned char lds_byte;

constexpr int kSseWaves = 8;
constexpr int kSseThreads = kSseWaves * 64;
constexpr int kSseTile = 64;              // streamed rows per LDS tile = per step
constexpr int kSseStages = 4;             // ring depth
constexpr int kSseXcds = 8;

constexpr int sse_lds_bytes(int D) { return kSseStages * (kSseTile * 2 * D + kSseTile * 4); }

struct SseParams {
  const unsigned short* held;      // [L, N, D] bf16: Q in rowstat, K in colmax
  const unsigned short* streamed;  // [L, N, D] bf16: K in rowstat, Q in colmax
  long long ld_held, ld_streamed;  // token strides (elements)
  float* c;                        // [N, L]: written by rowstat, read by colmax
  float* part;                     // [N, 3, L] (low, diag, up): written by colmax
  int L, N, block_len;
  float scale_log2;                // softmax scale * log2(e)
};

__device__ __forceinline__ float half_swap_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
// value of lane l ^ 32: after the swap of two copies of x, r[0] holds the low half's values in both halves and r[1]
// the high half's
__device__ __forceinline__ float other_half(float x, int g) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(g ? r[0] : r[1]);
}

// wave-wide global -> LDS copies (16 or 4 bytes per lane): uniform base + 32-bit per-lane byte offset
__device__ __forceinline__ void dma16(const void* base_uniform, unsigned byte_off, unsigned lds_addr_uniform) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_addr_uniform), "v"(byte_off), "s"(base_uniform)
               : "memory");
}
__device__ __forceinline__ void dma4(const void* base_uniform, unsigned byte_off, unsigned lds_addr_uniform) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
               :
               : "s"(lds_addr_uniform), "v"(byte_off), "s"(base_uniform)
               : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// COLMAX = false: rowstat.  COLMAX = true: colmax.  HT = 32-row groups of the held tensor per wave: every A fragment
// read from LDS feeds HT matrix instructions.
template <int D, bool COLMAX, int HT>
__global__ __launch_bounds__(kSseThreads, HT == 1 ? 2 : 1) void sse_pass_kernel(SseParams p) {
  constexpr int ROWB = 2 * D;               // bytes per row of one head
  constexpr int TILEB = kSseTile * ROWB;    // bytes per streamed tile
  constexpr int CH = D / 8;                 // 16-byte chunks per row
  constexpr int RPB = 256 / ROWB;           // rows per 256 bytes
  constexpr int RPI = 1024 / ROWB;          // rows per wave-wide load
  constexpr int LPT = TILEB / 1024 / kSseWaves;
  constexpr int KD = D / 16;
  constexpr int LOADS = LPT + (COLMAX ? 1 : 0);  // vector-memory loads per wave per tile
  constexpr int HELD = kSseWaves * 32 * HT;      // held rows per workgroup
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds_raw[];
  lds_byte* const ring = (lds_byte*)lds_raw;
  lds_byte* const c_ring = ring + kSseStages * TILEB;  // 64 floats per stage (colmax)

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, c = lane & 31;
  const int L = p.L;
  // workgroup -> (head, held tile), one contiguous range of the head-major list per XCD (each has its own L2)
  const int n_ht = (L + HELD - 1) / HELD;
  const int total = gridDim.x;
  const int xcd = blockIdx.x % kSseXcds, slot = blockIdx.x / kSseXcds;
  const int work = xcd * (total / kSseXcds) + (xcd < total % kSseXcds ? xcd : total % kSseXcds) + slot;
  const int h = work / n_ht;
  const int held0 = (work - h * n_ht) * HELD + wave * 32 * HT;  // first held row of this wave
  const int n_tiles = (L + kSseTile - 1) / kSseTile;

  // ---- held fragments (B operand): lane (row c of group ht, half g) holds held[row][16 kk + 8 g .. + 8]
  bf16x8 hf[HT][KD];
#pragma unroll
  for (int ht = 0; ht < HT; ++ht) {
    const int my_row = held0 + 32 * ht + c;  // may be >= L
    const int r = my_row < L ? my_row : L - 1;
    const unsigned short* hp = p.held + (long long)r * p.ld_held + (long long)h * D + 8 * g;
#pragma unroll
    for (int kk = 0; kk < KD; ++kk) hf[ht][kk] = *reinterpret_cast<const bf16x8*>(hp + 16 * kk);
  }

  // ---- streamed tile loads: load j of this wave fills tile rows (wave + W j) RPI .. + RPI; lane -> (row, slot);
  // the slot receives chunk slot ^ swizzle(row).  Rows past the end re-read the last row (masked later).
  const unsigned short* const s_base = p.streamed + (long long)h * D;
  const unsigned ld_b = (unsigned)(p.ld_streamed * 2);
  const float* const c_base = p.c + (long long)h * L;
  auto issue = [&](int tile) {
    lds_byte* st = ring + (tile % kSseStages) * TILEB;
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
      const int row = (wave + kSseWaves * j) * RPI + lane / CH;
      const int chunk = (lane % CH) ^ ((row / RPB) & (CH - 1));
      int src_row = tile * kSseTile + row;
      src_row = src_row < L ? src_row : L - 1;
      dma16(s_base, (unsigned)src_row * ld_b + chunk * 16,
            __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(st + (wave + kSseWaves * j) * 1024)));
    }
    if (COLMAX) {  // the c values of the tile's 64 queries: 8 lanes of every wave bring 8 of them (one load per wave,
      // so that all waves count the same number of loads)
      int src_row = tile * kSseTile + 8 * wave + (lane < 8 ? lane : 7);
      src_row = src_row < L ? src_row : L - 1;
      lds_byte* dst = c_ring + (tile % kSseStages) * (kSseTile * 4) + 8 * wave * 4;
      if (lane < 8)
        dma4(c_base, (unsigned)src_row * 4u, __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)dst));
    }
  };

  // fragment read offsets inside a tile: lane (row c of a 32-row block, half g) reads chunk 2 kk + g
  const int kx2 = g ^ ((c / RPB) & (CH - 1));
  const int a_off = c * ROWB;

  const float sc = p.scale_log2;
  // rowstat state: running maximum and sum of this lane's half of the keys
  float m_run[HT], l_run[HT];
  // colmax state: maxima of z - c over the queries seen so far, by block relation
  float mx_low[HT], mx_diag[HT], mx_up[HT];
#pragma unroll
  for (int ht = 0; ht < HT; ++ht) {
    m_run[ht] = -INFINITY; l_run[ht] = 0.f;
    mx_low[ht] = -INFINITY; mx_diag[ht] = -INFINITY; mx_up[ht] = -INFINITY;
  }
  // the extremes of the key blocks [lo, hi) (in query rows) over the wave's keys (colmax)
  const int L_B = p.block_len;
  const int w_lo_min = (held0 / L_B) * L_B;
  const int w_last = held0 + 32 * HT - 1 < L ? held0 + 32 * HT - 1 : L - 1;
  const int w_lo_max = (w_last / L_B) * L_B;
  const int w_hi_min = w_lo_min + L_B, w_hi_max = w_lo_max + L_B;

#pragma unroll
  for (int u = 0; u < kSseStages - 1; ++u) issue(u);
  wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();

#pragma unroll 1
  for (int t = 0; t < n_tiles; ++t) {
    issue(t + kSseStages - 1);  // into the slot tile t-1 vacated (tiles past the end hold clamped rows, never used)
    const lds_byte* st = ring + (t % kSseStages) * TILEB + a_off;
    f32x16 s[HT][2];
#pragma unroll
    for (int ht = 0; ht < HT; ++ht)
#pragma unroll
      for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[ht][rb][r] = 0.f;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int kk = 0; kk < KD; ++kk) {
        const bf16x8 a = *(const __attribute__((address_space(3))) bf16x8*)(st + rb * 32 * ROWB + (((2 * kk) ^ kx2) << 4));
#pragma unroll
        for (int ht = 0; ht < HT; ++ht) s[ht][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, hf[ht][kk], s[ht][rb], 0, 0, 0);
      }
    // register r of s[ht][rb] is streamed row  t 64 + 32 rb + 8 (r/4) + 4 g + (r%4)  against held row 32 ht + c
    const int row0 = t * kSseTile;
    if (!COLMAX) {
      // ---- online log-sum-exp over the keys
#pragma unroll
      for (int ht = 0; ht < HT; ++ht) {
        if (row0 + kSseTile > L) {  // ragged last tile: keys past the end do not exist
#pragma unroll
          for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r)
              if (row0 + 32 * rb + 8 * (r >> 2) + 4 * g + (r & 3) >= L) s[ht][rb][r] = -INFINITY;
        }
        float tmax = s[ht][0][0];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
          for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, s[ht][rb][r]);
        const float m_new = fmaxf(m_run[ht], tmax * sc);  // sc > 0
        float sum = 0.f;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
          for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(fmaf(s[ht][rb][r], sc, -m_new));
        // a ragged tail can leave this half of the lanes without a real key: then everything is -inf and nothing
        // may change
        l_run[ht] = (m_new == -INFINITY) ? 0.f : fmaf(l_run[ht], __builtin_amdgcn_exp2f(m_run[ht] - m_new), sum);
        m_run[ht] = m_new;
      }
    } else {
      // ---- z - c per element, maxima by block relation of the query (row) to this lane's key
      const __attribute__((address_space(3))) f32x4* cq =
          (const __attribute__((address_space(3))) f32x4*)(c_ring + (t % kSseStages) * (kSseTile * 4));
#pragma unroll
      for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const f32x4 cv = cq[(32 * rb + 8 * q4 + 4 * g) >> 2];
#pragma unroll
          for (int ht = 0; ht < HT; ++ht)
#pragma unroll
            for (int e = 0; e < 4; ++e) s[ht][rb][4 * q4 + e] = fmaf(s[ht][rb][4 * q4 + e], sc, -cv[e]);
        }
      const int row1 = row0 + kSseTile;  // one past the tile's last query
      const bool all_up = row1 <= w_lo_min;                            // every query in an earlier block than every key
      const bool all_low = row0 >= w_hi_max && row1 <= L;              // ... in a later block
      const bool all_diag = row0 >= w_lo_max && row1 <= w_hi_min && row1 <= L;
      if (all_up || all_diag || all_low) {  // wave-uniform
#pragma unroll
        for (int ht = 0; ht < HT; ++ht) {
          float tmax = s[ht][0][0];
#pragma unroll
          for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, s[ht][rb][r]);
          if (all_up) mx_up[ht] = fmaxf(mx_up[ht], tmax);
          else if (all_diag) mx_diag[ht] = fmaxf(mx_diag[ht], tmax);
          else mx_low[ht] = fmaxf(mx_low[ht], tmax);
        }
      } else {  // a tile that straddles a block boundary of some key of this wave, or the ragged last tile
#pragma unroll
        for (int ht = 0; ht < HT; ++ht) {
          const int my_row = held0 + 32 * ht + c;
          const int my_lo = (my_row / L_B) * L_B, my_hi = my_lo + L_B;
#pragma unroll
          for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int i = row0 + 32 * rb + 8 * (r >> 2) + 4 * g + (r & 3);
              const float v = i < L ? s[ht][rb][r] : -INFINITY;
              mx_up[ht] = fmaxf(mx_up[ht], i < my_lo ? v : -INFINITY);
              mx_diag[ht] = fmaxf(mx_diag[ht], (i >= my_lo && i < my_hi) ? v : -INFINITY);
              mx_low[ht] = fmaxf(mx_low[ht], i >= my_hi ? v : -INFINITY);
            }
        }
      }
    }
    // tile t+1 must have landed before the next step; the loads of tiles t+2, t+3 may stay in flight
    wait_vmcnt<2 * LOADS>();
    __builtin_amdgcn_s_barrier();
  }
  wait_vmcnt<0>();  // nothing may still be writing this workgroup's LDS when it retires

  // ---- combine the two lane halves (they saw disjoint streamed rows) and store
#pragma unroll
  for (int ht = 0; ht < HT; ++ht) {
    const int my_row = held0 + 32 * ht + c;
    if (!COLMAX) {
      const float m_o = other_half(m_run[ht], g), l_o = other_half(l_run[ht], g);
      const float m = fmaxf(m_run[ht], m_o);
      const float l = l_run[ht] * __builtin_amdgcn_exp2f(m_run[ht] - m) + l_o * __builtin_amdgcn_exp2f(m_o - m);
      if (g == 0 && my_row < L) p.c[(long long)h * L + my_row] = m + __builtin_amdgcn_logf(l);  // v_log_f32 = log2
    } else {
      const float lo = half_swap_max(mx_low[ht]), di = half_swap_max(mx_diag[ht]), up = half_swap_max(mx_up[ht]);
      if (g == 0 && my_row < L) {
        float* o = p.part + (long long)h * 3 * L + my_row;
        o[0] = __builtin_amdgcn_exp2f(lo);  // 2^-inf = 0: an empty query set
        o[L] = __builtin_amdgcn_exp2f(di);
        o[2 * (long long)L] = __builtin_amdgcn_exp2f(up);
      }
    }
  }
}

// mean over heads, then the mean of the parts whose query set is not empty (Eq. 5)
__global__ void sse_combine_kernel(const float* __restrict__ part, int L, int N, int block_len,
                                   float* __restrict__ out) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= L) return;
  float lo = 0.f, di = 0.f, up = 0.f;
  for (int h = 0; h < N; ++h) {
    const float* q = part + (long long)h * 3 * L + j;
    lo += q[0];
    di += q[L];
    up += q[2 * (long long)L];
  }
  const float inv_n = 1.0f / (float)N;
  const int b = j / block_len, b_last = (L - 1) / block_len;
  float acc = di * inv_n;
  int parts = 1;
  if (b < b_last) { acc += lo * inv_n; ++parts; }
  if (b > 0) { acc += up * inv_n; ++parts; }
  out[j] = acc / (float)parts;
}

template <int D, bool COLMAX>
int launch_pass(hipStream_t st, const SseParams& p) {
  // One 32-row group per wave and two workgroups per CU.  Two groups per wave (half the LDS reads per matrix
  // instruction, one workgroup per CU) measured the same: LDS read bandwidth is not what bounds the passes.
  constexpr int HT = 1;
  static LdsLimit lds_limit;
  const int rc = set_lds_limit(lds_limit, sse_pass_kernel<D, COLMAX, HT>, sse_lds_bytes(D));
  if (rc != PAFU_OK) return rc;
  constexpr int HELD = kSseWaves * 32 * HT;
  const int grid = ((p.L + HELD - 1) / HELD) * p.N;
  hipLaunchKernelGGL((sse_pass_kernel<D, COLMAX, HT>), dim3(grid), dim3(kSseThreads), sse_lds_bytes(D), st, p);
  return check_launch();
}

}  // namespace

size_t sse_workspace_bytes(int L, int N) { return (size_t)4 * 4 * (size_t)N * (size_t)L; }

int launch_sse(hipStream_t st, const void* Q, const void* K, int L, int N, int D, long long ld_q, long long ld_k,
               int block_len, float scale, float* out, void* workspace) {
  SseParams p;
  p.L = L; p.N = N; p.block_len = block_len;
  p.scale_log2 = scale * 1.44269504088896340736f;
  p.c = static_cast<float*>(workspace);
  p.part = p.c + (size_t)N * L;
  int rc;
  // rowstat: queries held, keys streamed
  p.held = static_cast<const unsigned short*>(Q); p.ld_held = ld_q;
  p.streamed = static_cast<const unsigned short*>(K); p.ld_streamed = ld_k;
  rc = D == 128 ? launch_pass<128, false>(st, p) : launch_pass<64, false>(st, p);
  if (rc) return rc;
  // colmax: keys held, queries streamed
  p.held = static_cast<const unsigned short*>(K); p.ld_held = ld_k;
  p.streamed = static_cast<const unsigned short*>(Q); p.ld_streamed = ld_q;
  rc = D == 128 ? launch_pass<128, true>(st, p) : launch_pass<64, true>(st, p);
  if (rc) return rc;
  hipLaunchKernelGGL(sse_combine_kernel, dim3((L + 255) / 256), dim3(256), 0, st, p.part, L, N, block_len, out);
  return check_launch();
}

}  // namespace pafu

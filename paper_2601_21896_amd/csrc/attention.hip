// Attention of the chunk's queries over the retained cache plus the chunk itself.
// Sec. 3.2 of the paper: P = softmax(Q K^T / sqrt(D)), block boundaries from the block length L_B;
// App. A: L_B = chunk length at inference (then the chunk attends to all of itself).
//
// Flash-style kernel for gfx950: bf16 MFMA (v_mfma_f32_32x32x16_bf16), fp32 online softmax, fp32
// accumulation.  One workgroup = 8 waves = 256 queries of one head; each wave owns 32 queries and
// walks the key axis in tiles of 64 keys.  Both products are computed TRANSPOSED:
//
//   S^T[key, q] = K_tile . Q^T         (A = K rows from LDS, B = Q^T held in registers for the whole loop)
//   O^T[d,   q] = V_tile^T . P^T       (A = V^T via transposing LDS reads, B = P^T straight from the S^T
//                                       accumulator registers)
//
// In the 32x32 accumulator layout a lane holds 16 rows of ONE column, so with queries as columns the
// softmax row reductions are in-register plus one half-wave swap, the rescale factor is one scalar per
// lane, and the accumulator registers of S^T already ARE the B operand of the second product (its
// contraction index - the key - may be enumerated in any order as long as V^T uses the same order).
//
// Scheduling: the two waves that share a SIMD alternate roles every phase ("ping-pong"): while one
// runs its matrix phase (S^T of the next tile and O^T update of the current one, 32 MFMAs), the other
// runs its vector phase (online softmax of the S^T it just produced).  A workgroup barrier ends each
// phase, which keeps the two groups exactly one phase apart, so the matrix and vector pipes of every
// SIMD are both busy.  K/V tiles stream from global memory straight into a 4-deep LDS ring
// (global_load_lds, no staging registers) several phases ahead of their use; rows are stored with an
// XOR swizzle of their 16-byte chunks so that both the b128 K reads and the transposing V reads are
// bank-conflict free without padding.  The two key segments (retained cache, chunk) are addressed row
// by row, so no concatenated copy exists.
#include "pafu_internal.h"

namespace pafu {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

struct AttnParams {
  const unsigned short* Q;
  const unsigned short* Kc;
  const unsigned short* Vc;
  const unsigned short* Kn;
  const unsigned short* Vn;
  void* O;
  long long ld_q, ld_c, ld_n, ld_o;
  int Lq, n_kept, Lc, block_len;
  float scale_log2;  // softmax scale * log2(e)
};

constexpr int kAtWaves = 8;
constexpr int kAtThreads = kAtWaves * 64;
constexpr int kAtBQ = kAtWaves * 32;  // queries per workgroup
constexpr int kAtBK = 64;             // keys per tile
constexpr int kAtStages = 4;          // LDS ring depth (tiles)

constexpr int attn_lds_bytes(int D) { return 2 * kAtStages * kAtBK * 2 * D; }

typedef __attribute__((address_space(3))) unsigned char lds_byte;
typedef __attribute__((address_space(1))) const void global_cvoid;

__device__ __forceinline__ float half_swap_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_swap_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// One wave-wide global -> LDS copy of 64 x 16 bytes: lane l's 16 bytes land at lds_addr + 16 l.  Written as
// inline assembly so that the compiler's own wait-count insertion does not serialise it against later LDS
// reads of OTHER ring slots; completion is tracked by hand with wait_vmcnt<N>() before a barrier.
__device__ __forceinline__ void dma_row_chunks(const void* src, unsigned lds_addr_uniform) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
               :
               : "s"(lds_addr_uniform), "v"(src)
               : "memory");
}

// s_waitcnt vmcnt(N) with the other counters left alone (gfx9 encoding: vmcnt = bits 3:0 and 15:14).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

template <int D, bool OUT_F32>
__global__ __launch_bounds__(kAtThreads, 1) void chunk_attention_kernel(AttnParams p) {
  constexpr int ROWB = 2 * D;            // bytes per K/V row of one head
  constexpr int TILEB = kAtBK * ROWB;    // bytes per K (or V) tile
  constexpr int CH = D / 8;              // 16-byte chunks per row
  constexpr int RPB = 256 / ROWB;        // rows per 256 bytes (one pass over all LDS banks)
  constexpr int RPI = 1024 / ROWB;       // rows written by one wave-wide 16-byte-per-lane load
  constexpr int LPT = TILEB / 1024 / kAtWaves;  // such loads per wave per tensor per tile
  constexpr int KD = D / 16;             // contraction steps of S^T
  constexpr int DB = D / 32;             // 32-row blocks of O^T
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds_raw[];
  lds_byte* const k_ring = (lds_byte*)lds_raw;
  lds_byte* const v_ring = k_ring + kAtStages * TILEB;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int group = wave >> 2;  // waves w and w+4 share a SIMD and alternate roles
  const int g = lane >> 5, c = lane & 31;
  const int h = blockIdx.y;
  const int i_first = blockIdx.x * kAtBQ;
  const int i_last = (i_first + kAtBQ - 1 < p.Lq) ? i_first + kAtBQ - 1 : p.Lq - 1;
  const int q_row = i_first + wave * 32 + c;
  const int qi = q_row < p.Lq ? q_row : p.Lq - 1;
  const int L_B = p.block_len;
  const int n_total = p.n_kept + p.Lc;

  // number of visible keys: per lane (its query) and the workgroup's extremes
  auto visible = [&](int i) {
    const int e = (i / L_B + 1) * L_B;
    return p.n_kept + (e < p.Lc ? e : p.Lc);
  };
  const int lim = visible(qi);
  const int lim_min = visible(i_first);
  const int lim_max = visible(i_last);
  const int n_tiles = (lim_max + kAtBK - 1) / kAtBK;

  // ---- global -> LDS tile loads.  Load j of this wave fills LDS rows (wave + 8 j) * RPI .. + RPI of a
  // tile; lane -> (row, slot); the slot receives chunk (slot ^ swizzle(row)) of that row.
  int ld_row[LPT], ld_kchunk[LPT], ld_vchunk[LPT];
#pragma unroll
  for (int j = 0; j < LPT; ++j) {
    const int row = (wave + kAtWaves * j) * RPI + lane / CH;
    const int slot = lane % CH;
    ld_row[j] = row;
    ld_kchunk[j] = slot ^ ((row / RPB) & (CH - 1));
    ld_vchunk[j] = slot ^ (4 * ((row / RPB) & (CH / 4 - 1)));
  }
  const long long head_off = (long long)h * D;
  // one tensor's tile: rows past the end are masked later, so they read a valid row instead.  The chunk segment's
  // base is pre-shifted by -n_kept rows so that both segments are addressed as base + key_index * stride.
  const long long ldc_b = p.ld_c * 2, ldn_b = p.ld_n * 2;
  auto issue_one = [&](int tile, const unsigned short* cache, const unsigned short* chunk, lds_byte* ring,
                       const int (&chunk_of)[LPT]) {
    const int stage = tile % kAtStages;
    const char* base_c = reinterpret_cast<const char*>(cache + head_off);
    const char* base_n = reinterpret_cast<const char*>(chunk + head_off) - (long long)p.n_kept * ldn_b;
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
      int kidx = tile * kAtBK + ld_row[j];
      kidx = kidx < n_total ? kidx : n_total - 1;
      const bool in_cache = kidx < p.n_kept;
      const char* src = (in_cache ? base_c : base_n) + (unsigned long long)(unsigned)kidx * (unsigned long long)(in_cache ? ldc_b : ldn_b) + chunk_of[j] * 16;
      lds_byte* dst = ring + stage * TILEB + (wave + kAtWaves * j) * 1024;
      dma_row_chunks(src, __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)dst));
    }
  };
  // K of tile kt and V of tile kt - 1 travel together (V is consumed one iteration after K)
  auto issue_tile = [&](int kt) {
    issue_one(kt, p.Kc, p.Kn, k_ring, ld_kchunk);
    if (kt > 0) issue_one(kt - 1, p.Vc, p.Vn, v_ring, ld_vchunk);
  };

  // ---- LDS read offsets (bytes inside a tile)
  // K fragment (A operand): lane (key row c, half g) reads chunk (2 kk + g) of row 32 kb + c
  const int kx = (c / RPB) & (CH - 1);
  const int k_off = c * ROWB;
  const int kx2 = g ^ kx;  // LDS slot of step kk is (2 kk) ^ kx2
  // V^T fragment via transposing reads: 16-lane group = (d-half, key group g); lane i of the group points at
  // key row rr = 4 g + i/4, four consecutive d at 4 (i%4)
  const int i16 = lane & 15;
  const int rr = 4 * g + (i16 >> 2);
  // (32 lanes = one key group read 4 rows x 64 bytes per transposing read: the swizzle spreads them over all banks)
  const int vx = 4 * ((rr / RPB) & (CH / 4 - 1));
  const int cl = 2 * ((lane >> 4) & 1) + ((i16 & 3) >> 1);
  const int v_off = rr * ROWB + ((i16 & 1) << 3) + (cl << 4);
  const int vx2 = vx;  // LDS slot of d-block b is ((4 b) ^ vx2) + cl

  // Q^T fragments (B operand): lane (query c, half g) holds Q[q][16 kk + 8 g .. +8]
  bf16x8 qf[KD];
  {
    const unsigned short* qp = p.Q + (long long)qi * p.ld_q + head_off + 8 * g;
#pragma unroll
    for (int kk = 0; kk < KD; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qp + 16 * kk);
  }

  f32x16 o[DB];
#pragma unroll
  for (int b = 0; b < DB; ++b)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[b][r] = 0.f;
  f32x16 s[2];
  bf16x8 pf[4];
  float m_run = -INFINITY, l_run = 0.f;
  const float sc = p.scale_log2;

  // matrix phase of iteration t: S^T(t) = K(t) Q^T  and  O^T += V(t-1)^T P(t-1)^T
  auto matrix_phase = [&](int t) {
    __builtin_amdgcn_s_setprio(1);
    if (t < n_tiles) {
      const lds_byte* kt = k_ring + (t % kAtStages) * TILEB + k_off;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KD; ++kk) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {  // the two key blocks alternate: no back-to-back dependent MFMAs
          const bf16x8 a =
              *(const __attribute__((address_space(3))) bf16x8*)(kt + kb * 32 * ROWB + (((2 * kk) ^ kx2) << 4));
          s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], s[kb], 0, 0, 0);
        }
      }
    }
    if (t > 0) {
      const lds_byte* vt = v_ring + ((t - 1) % kAtStages) * TILEB + v_off;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
        for (int b = 0; b < DB; ++b) {
          const lds_byte* a0 = vt + (16 * ks) * ROWB + (((4 * b) ^ vx2) << 4);
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(a0));
          const s16x4 hi =
              __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(a0 + 8 * ROWB));
          const s16x8 a16 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a16), pf[ks], o[b], 0, 0, 0);
        }
      }
    }
    __builtin_amdgcn_s_setprio(0);
  };

  // vector phase of iteration t: online softmax of S^T(t) -> P^T(t), rescale of O^T
  auto vector_phase = [&](int t) {
    if (t >= n_tiles) return;
    // block mask / ragged tail: key index of register r is t*64 + 32 kb + 8 (r/4) + 4 g + (r%4)
    if ((t + 1) * kAtBK > lim_min) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kidx = t * kAtBK + 32 * kb + 8 * (r >> 2) + 4 * g + (r & 3);
          if (kidx >= lim) s[kb][r] = -INFINITY;
        }
    }
    float mx = s[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][r]);
    mx = half_swap_max(mx);
    const float m_new = fmaxf(m_run, mx);
    const float msc = m_new * sc;
    float psum = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float pe = __builtin_amdgcn_exp2f(fmaf(s[kb][r], sc, -msc));
        psum += pe;
        pf[2 * kb + (r >> 3)][r & 7] = (__bf16)pe;
      }
    // the running maximum rarely moves after the first tiles: rescale only when some query's did
    if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * sc);
      l_run *= alpha;
#pragma unroll
      for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[b][r] *= alpha;
      m_run = m_new;
    }
    l_run += psum;
  };

  // ---- prologue: fill the ring (K tiles 0..S-2, V tiles 0..S-3), then run the phases.
  // Even phase 2t: every wave issues K(t+S-1) and V(t+S-2) into the slots whose tiles (K(t-1), V(t-2)) were last
  // read in phase 2t-1; group 0 runs matrix(t), group 1 runs vector(t-1).
  // Odd phase 2t+1: group 0 runs vector(t), group 1 runs matrix(t); before its closing barrier every wave waits
  // until only the loads of the last S-2 even phases are still in flight (K(t+1) and V(t) have landed).
#pragma unroll
  for (int u = 0; u < kAtStages - 1; ++u) issue_tile(u);  // tiles past the end hold clamped rows, never read back
  wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();

  const int n_iter = n_tiles + 1;  // matrix(t) for t = 0..n_tiles (the last one only updates O^T)
  if (group == 0) {
#pragma unroll 1
    for (int t = 0; t < n_iter; ++t) {
      issue_tile(t + kAtStages - 1);
      matrix_phase(t);
      __builtin_amdgcn_s_barrier();
      vector_phase(t);
      wait_vmcnt<2 * LPT*(kAtStages - 2)>();
      __builtin_amdgcn_s_barrier();
    }
  } else {
#pragma unroll 1
    for (int t = 0; t < n_iter; ++t) {
      issue_tile(t + kAtStages - 1);
      if (t > 0) vector_phase(t - 1);
      __builtin_amdgcn_s_barrier();
      matrix_phase(t);
      wait_vmcnt<2 * LPT*(kAtStages - 2)>();
      __builtin_amdgcn_s_barrier();
    }
  }
  wait_vmcnt<0>();  // nothing may still be writing this workgroup's LDS when it retires

  // normalise and store: lane holds query c, d = 32 b + 8 (r/4) + 4 g + (r%4)
  const float l_tot = half_swap_sum(l_run);
  const float inv = 1.0f / l_tot;
  if (q_row < p.Lq) {
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int d0 = 32 * b + 8 * q4 + 4 * g;
        const float v0 = o[b][4 * q4 + 0] * inv, v1 = o[b][4 * q4 + 1] * inv;
        const float v2 = o[b][4 * q4 + 2] * inv, v3 = o[b][4 * q4 + 3] * inv;
        const long long off = (long long)q_row * p.ld_o + head_off + d0;
        if (OUT_F32) {
          *reinterpret_cast<float4*>(static_cast<float*>(p.O) + off) = make_float4(v0, v1, v2, v3);
        } else {
          bf16x4 ob;
          ob[0] = (__bf16)v0; ob[1] = (__bf16)v1; ob[2] = (__bf16)v2; ob[3] = (__bf16)v3;
          *reinterpret_cast<bf16x4*>(static_cast<unsigned short*>(p.O) + off) = ob;
        }
      }
  }
}

template <int D, bool OUT_F32>
int launch_variant(hipStream_t st, dim3 grid, const AttnParams& p) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(chunk_attention_kernel<D, OUT_F32>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, attn_lds_bytes(D));
    if (e != hipSuccess) return record_hip_error(e);
    attr_set = true;
  }
  hipLaunchKernelGGL((chunk_attention_kernel<D, OUT_F32>), grid, dim3(kAtThreads), attn_lds_bytes(D), st, p);
  return check_launch();
}

}  // namespace

int launch_attention(hipStream_t st, const void* Q, int Lq, const void* Kc, const void* Vc, int n_kept,
                     const void* Kn, const void* Vn, int Lc, int N, int D, long long ld_q, long long ld_c,
                     long long ld_n, long long ld_o, int block_len, float scale, void* O, int out_dtype) {
  AttnParams p;
  p.Q = static_cast<const unsigned short*>(Q);
  p.Kc = static_cast<const unsigned short*>(Kc);
  p.Vc = static_cast<const unsigned short*>(Vc);
  p.Kn = static_cast<const unsigned short*>(Kn);
  p.Vn = static_cast<const unsigned short*>(Vn);
  p.O = O;
  p.ld_q = ld_q; p.ld_c = ld_c; p.ld_n = ld_n; p.ld_o = ld_o;
  p.Lq = Lq; p.n_kept = n_kept; p.Lc = Lc;
  p.block_len = block_len < Lc ? block_len : Lc;  // blocks at least as long as the chunk mean "no mask"
  p.scale_log2 = scale * 1.44269504088896340736f;
  const dim3 grid((Lq + kAtBQ - 1) / kAtBQ, N);
  const bool f32 = out_dtype == PAFU_F32;
  if (D == 128) return f32 ? launch_variant<128, true>(st, grid, p) : launch_variant<128, false>(st, grid, p);
  return f32 ? launch_variant<64, true>(st, grid, p) : launch_variant<64, false>(st, grid, p);
}

}  // namespace pafu

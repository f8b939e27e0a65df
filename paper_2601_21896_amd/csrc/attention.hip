// Attention of the chunk's queries over the retained cache plus the chunk itself.
// Sec. 3.2 of the paper: P = softmax(Q K^T / sqrt(D)), block boundaries from the block length L_B;
// App. A: L_B = chunk length at inference (then the chunk attends to all of itself).
//
// Flash-style kernel for gfx950: bf16 MFMA (v_mfma_f32_32x32x16_bf16), fp32 online softmax, fp32
// accumulation.  One workgroup = 4 waves = 128 queries of one head; each wave owns 32 queries and
// walks the key axis in tiles of 64 keys staged through LDS.  Both products are computed TRANSPOSED:
//
//   S^T[key, q] = K_tile . Q^T         (A = K rows from LDS, B = Q^T held in registers for the whole loop)
//   O^T[d,   q] = V_tile^T . P^T       (A = V^T via transposing LDS reads, B = P^T straight from the S^T
//                                       accumulator registers)
//
// In the 32x32 accumulator layout a lane holds 16 rows of ONE column, so with queries as columns the
// softmax row reductions are in-register plus one half-wave swap, the rescale factor is one scalar per
// lane, and the accumulator registers of S^T already ARE the B operand of the second product (its
// contraction index - the key - may be enumerated in any order as long as V^T uses the same order).
// The two key segments (retained cache, chunk) are addressed row by row, so no concatenated copy exists.
#include "pafu_internal.h"

namespace pafu {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

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

constexpr int kAtThreads = 256;
constexpr int kAtBQ = 128;  // queries per workgroup
constexpr int kAtBK = 64;   // keys per tile

__device__ __forceinline__ float half_swap_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_swap_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

template <int D, bool OUT_F32>
__global__ __launch_bounds__(kAtThreads, 2) void chunk_attention_kernel(AttnParams p) {
  constexpr int KS = 2 * D + 16;  // K tile row stride (bytes): b128 reads of 16 consecutive rows hit distinct banks
  constexpr int VS = 2 * D + 64;  // V tile row stride (bytes): the 4-row x 32-byte transposing reads do too
  constexpr int CH = D / 8;       // 16-byte chunks per K/V row
  constexpr int RPP = kAtThreads / CH;  // rows per cooperative load pass
  constexpr int NP = kAtBK / RPP;       // passes per tile
  constexpr int KD = D / 16;            // contraction steps of S^T
  constexpr int DB = D / 32;            // 32-row blocks of O^T
  __shared__ __attribute__((aligned(16))) unsigned char k_lds[kAtBK * KS];
  __shared__ __attribute__((aligned(16))) unsigned char v_lds[kAtBK * VS];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, c = lane & 31;
  const int h = blockIdx.y;
  const int i_first = blockIdx.x * kAtBQ;
  const int i_last = (i_first + kAtBQ - 1 < p.Lq) ? i_first + kAtBQ - 1 : p.Lq - 1;
  const int q_row = i_first + wave * 32 + c;
  const int qi = q_row < p.Lq ? q_row : p.Lq - 1;
  const int L_B = p.block_len;

  // number of visible keys: per lane (its query) and the workgroup's extremes
  auto visible = [&](int i) {
    const int e = (i / L_B + 1) * L_B;
    return p.n_kept + (e < p.Lc ? e : p.Lc);
  };
  const int lim = visible(qi);
  const int lim_min = visible(i_first);
  const int lim_max = visible(i_last);
  const int n_tiles = (lim_max + kAtBK - 1) / kAtBK;

  // Q^T fragments (B operand): lane (query c, half g) holds Q[q][16 kk + 8 g .. +8]
  bf16x8 qf[KD];
  {
    const unsigned short* qp = p.Q + (long long)qi * p.ld_q + (long long)h * D + 8 * g;
#pragma unroll
    for (int kk = 0; kk < KD; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qp + 16 * kk);
  }

  f32x16 o[DB];
#pragma unroll
  for (int b = 0; b < DB; ++b)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[b][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float sc = p.scale_log2;

  // cooperative tile load: thread -> row (i*RPP + tid/CH), chunk tid%CH
  const int ld_row = tid / CH, ld_chunk = tid % CH;
  u32x4 kreg[NP], vreg[NP];
  auto load_tile = [&](int t) {
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int kidx = t * kAtBK + i * RPP + ld_row;
      const unsigned short *kp, *vp;
      if (kidx < p.n_kept) {
        const long long off = (long long)kidx * p.ld_c + (long long)h * D + ld_chunk * 8;
        kp = p.Kc + off;
        vp = p.Vc + off;
      } else {
        int j = kidx - p.n_kept;
        j = j < p.Lc ? j : p.Lc - 1;  // rows past the end are masked; read a valid row instead
        const long long off = (long long)j * p.ld_n + (long long)h * D + ld_chunk * 8;
        kp = p.Kn + off;
        vp = p.Vn + off;
      }
      kreg[i] = *reinterpret_cast<const u32x4*>(kp);
      vreg[i] = *reinterpret_cast<const u32x4*>(vp);
    }
  };

  // LDS read addresses
  const unsigned char* k_rd = k_lds + c * KS + g * 16;
  // transposing V reads: 16-lane group q16 covers d-half (q16 & 1) of key group g = q16 >> 1;
  // lane i of the group points at key row i/4, 4 consecutive d at 4 (i%4)
  const int i16 = lane & 15;
  const unsigned char* v_rd = v_lds + (4 * g + (i16 >> 2)) * VS + (16 * ((lane >> 4) & 1) + 4 * (i16 & 3)) * 2;

  load_tile(0);
#pragma unroll 1
  for (int t = 0; t < n_tiles; ++t) {
    __syncthreads();  // all waves finished reading the previous tile
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int row = i * RPP + ld_row;
      *reinterpret_cast<u32x4*>(k_lds + row * KS + ld_chunk * 16) = kreg[i];
      *reinterpret_cast<u32x4*>(v_lds + row * VS + ld_chunk * 16) = vreg[i];
    }
    __syncthreads();
    if (t + 1 < n_tiles) load_tile(t + 1);

    // S^T = K . Q^T
    f32x16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KD; ++kk) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(k_rd + kb * 32 * KS + kk * 32);
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], s[kb], 0, 0, 0);
      }
    }
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
    // online softmax (base-2 domain)
    float mx = s[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][r]);
    mx = half_swap_max(mx);
    const float m_new = fmaxf(m_run, mx);
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * sc);
    const float msc = m_new * sc;
    m_run = m_new;
    float psum = 0.f;
    bf16x8 pf[4];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float pe = __builtin_amdgcn_exp2f(fmaf(s[kb][r], sc, -msc));
        psum += pe;
        pf[2 * kb + (r >> 3)][r & 7] = (__bf16)pe;
      }
    l_run = fmaf(l_run, alpha, psum);
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[b][r] *= alpha;

    // O^T += V^T . P^T
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
      for (int b = 0; b < DB; ++b) {
        const unsigned char* a0 = v_rd + (16 * ks) * VS + b * 64;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4*)(a0));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4*)(a0 + 8 * VS));
        const s16x8 a16 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        const bf16x8 a = __builtin_bit_cast(bf16x8, a16);
        o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[ks], o[b], 0, 0, 0);
      }
    }
  }

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
        const long long off = (long long)q_row * p.ld_o + (long long)h * D + d0;
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
  const dim3 grid((Lq + kAtBQ - 1) / kAtBQ, N), block(kAtThreads);
  const bool f32 = out_dtype == PAFU_F32;
  if (D == 128) {
    if (f32) hipLaunchKernelGGL((chunk_attention_kernel<128, true>), grid, block, 0, st, p);
    else hipLaunchKernelGGL((chunk_attention_kernel<128, false>), grid, block, 0, st, p);
  } else {
    if (f32) hipLaunchKernelGGL((chunk_attention_kernel<64, true>), grid, block, 0, st, p);
    else hipLaunchKernelGGL((chunk_attention_kernel<64, false>), grid, block, 0, st, p);
  }
  return check_launch();
}

}  // namespace pafu

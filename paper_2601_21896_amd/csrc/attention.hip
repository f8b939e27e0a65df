// Attention of the chunk's queries over the retained cache plus the chunk itself.
// Sec. 3.2 of the paper: P = softmax(Q K^T / sqrt(D)), block boundaries from the block length L_B;
// App. A: L_B = chunk length at inference (then the chunk attends to all of itself).
//
// Flash-style kernel for gfx950: bf16 MFMA (v_mfma_f32_32x32x16_bf16), fp32 online softmax, fp32
// accumulation.  One workgroup = 8 waves = 256 queries of one head; each wave owns 32 queries (one
// column block) and walks the key axis in tiles of 64 keys.  Both products are TRANSPOSED:
//
//   S^T[key, q] = K_blk . Q^T          (A = K rows from LDS, B = Q^T held in registers for the whole loop)
//   O^T[d,   q] = V_blk^T . P^T        (A = V^T via transposing LDS reads, B = P^T straight from the S^T
//                                       accumulator registers)
//
// In the 32x32 accumulator layout a lane holds 16 rows of ONE column, so with queries as columns the
// softmax row reductions are in-register plus one half-wave swap, the rescale factor is one scalar per
// lane, and the accumulator registers of S^T already ARE the B operand of the second product (its
// contraction index - the key - may be enumerated in any order as long as V^T uses the same order).
//
// Scheduling.  On this chip the matrix and vector pipes only overlap reliably for instructions of the
// SAME wave (a wave with a matrix instruction waiting at issue blocks the vector instructions of its
// SIMD neighbour), so each wave is software-pipelined by hand: step t issues the 16 MFMAs of S^T(t+1)
// and the 16 MFMAs that add tile t-1 to O^T, and after each of them a slice of the online softmax of
// tile t (vector ALU).  Two such waves share a SIMD and fill each other's stalls.  The running maximum is only raised when it
// grows by more than 2^8 (the result is mathematically unchanged), which makes the O^T rescale a rare,
// out-of-line event.
//
// K/V tiles (64 keys) stream from global memory straight into a 4-deep LDS ring (global_load_lds, no
// staging registers) three tiles ahead of their use; rows are stored with an XOR swizzle of their
// 16-byte chunks so that both the b128 K reads and the transposing V reads are bank-conflict free
// without padding.  The two key segments (retained cache, chunk) are addressed row by row, so no
// concatenated copy exists.
#include "pafu_internal.h"

namespace pafu {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

// P^T fragments are kept as 4 dwords of packed bf16 pairs (the B operand of the second product)
__device__ __forceinline__ bf16x8 as_bf16x8(const u32x4& v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
  bf16x2 t;
  t[0] = (__bf16)lo;
  t[1] = (__bf16)hi;
  return __builtin_bit_cast(unsigned, t);
}

struct AttnParams {
  const unsigned short* Q;
  const unsigned short* Kc;
  const unsigned short* Vc;
  const unsigned short* Kn;
  const unsigned short* Vn;
  void* O;
  const int* ids;  // gather variant: retained row r of the cache segment is row ids[r] of Kc / Vc
  int n_cache;     // rows behind Kc / Vc in the gather variant
  long long ld_q, ld_c, ld_n, ld_o;
  int Lq, n_kept, Lc, block_len, N_heads;
  float scale_log2;  // softmax scale * log2(e)
  float k_scale, v_scale;  // 8-bit K/V: the tensors' power-of-two scales (a stored code c stands for c * scale)
};

constexpr int kAtWaves = 8;
constexpr int kAtThreads = kAtWaves * 64;
constexpr int kAtBQ = kAtWaves * 32;  // queries per workgroup
constexpr int kAtTileKeys = 64;       // keys per LDS tile = keys per pipeline step
constexpr int kAtStages = 4;          // LDS ring depth (tiles)
constexpr int kAtIdStages = 8;        // ids ring depth (gather variant): a tile's ids live from 3 steps before its
                                      // K load to its V load two steps after that
constexpr int kAtIdLead = 3;
constexpr int kAtXcds = 8;            // accelerator dies, each with its own L2
constexpr float kAtLazyLog2 = 8.0f;   // raise the running maximum only when it grows by more than 2^8
// Study builds only (never the shipped library, which is built without the macro): PAFU_ATTN_ABLATE is a bit mask that
// takes ingredients out of the inner loop so that what they cost can be measured on the same shapes and data; the
// results of such a build are meaningless.  pafu_study_build() returns the mask.
//   1: no global -> LDS tile copies inside the loop (the ring keeps the tiles of the prologue)
//   2: no softmax arithmetic (P = the upper halves of S, one byte-permute per pair; sums and maxima untouched)
//   4: equal runs whenever a workspace is given, also when the items fill the chip (results stay correct)
#ifndef PAFU_ATTN_ABLATE
#define PAFU_ATTN_ABLATE 0
#endif
constexpr bool kAblateLoads = (PAFU_ATTN_ABLATE & 1) != 0;
constexpr bool kAblateSoftmax = (PAFU_ATTN_ABLATE & 2) != 0;
constexpr bool kStudySplitAlways = (PAFU_ATTN_ABLATE & 4) != 0;
constexpr float kAtNoMax = -1.0e30f;  // running maximum before the first visible key (finite on purpose)
constexpr int kAtMaxRuns = 256;       // most workgroups the unit list is ever cut into (one per CU)

constexpr int attn_lds_bytes(int D, bool gather = false) {
  return 2 * kAtStages * kAtTileKeys * 2 * D + (gather ? kAtIdStages * kAtTileKeys * 4 : 0);
}

typedef __attribute__((address_space(3))) unsigned char lds_byte;

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

// The same copy addressed as a wave-uniform base plus a 32-bit per-lane byte offset.
__device__ __forceinline__ void dma_row_chunks_at(const void* base_uniform, unsigned byte_off, unsigned lds_addr_uniform) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_addr_uniform), "v"(byte_off), "s"(base_uniform)
               : "memory");
}

// s_waitcnt vmcnt(N) with the other counters left alone (gfx9 encoding: vmcnt = bits 3:0 and 15:14).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

__device__ __forceinline__ bf16x8 lds_read_k(const lds_byte* p) {
  return *(const __attribute__((address_space(3))) bf16x8*)p;
}
// V^T fragment: two transposing reads, 8 key rows apart
__device__ __forceinline__ bf16x8 lds_read_vt(const lds_byte* p, int row_bytes8) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p + row_bytes8));
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// Pipeline step t for one wave (32 queries), one straight-line block:
//   matrix pipe : S^T(t+1) = K(t+1) Q^T into s_nxt;  O^T += V(t-1)^T P(t-1)^T from p_prev
//   vector pipe : online softmax of s_cur = S^T(t) -> p_cur = P^T(t), running max / sum,
// with the vector work sliced between the MFMAs.  Edge cases are handled by the caller through the operands
// (masked elements of s_cur set to -inf beforehand, p_prev = 0 before the first tile, a clamped K tile when
// there is no next tile), so this is the only implementation of the step.
// s_*[kb] = key block kb (32 keys) of the tile; p_*[ks] = 16-key slice ks of the tile.
// issue_k / issue_v start this step's global -> LDS tile copies.  They are called a few slots into the step, not at
// its start: right after the barrier all eight waves would queue their copies at once and sit behind the memory pipe
// (a wave issues nothing while its copy waits), whereas an eighth and a half of the way in they find it free.
template <int D, typename IssueK, typename IssueV>
__device__ __forceinline__ void attn_step(const f32x16 (&s_cur)[2], f32x16 (&s_nxt)[2], const u32x4 (&p_prev)[4],
                                          u32x4 (&p_cur)[4], f32x16 (&o)[D / 32], const bf16x8 (&qf)[D / 16],
                                          float& msc, float& l_run, const lds_byte* k_tile, const lds_byte* v_tile,
                                          int kx2, int vx2, float sc, IssueK&& issue_k, IssueV&& issue_v) {
  constexpr int ROWB = 2 * D;
  constexpr int KD = D / 16;
  constexpr int DB = D / 32;
  constexpr int NS = 2 * KD;       // MFMAs of S^T(t+1): 2 key blocks x KD contraction steps
  constexpr int NP = 4 * DB;       // MFMAs of the O^T update: 4 key slices x DB row blocks
  constexpr int NSLOT = NS + NP;   // MFMAs per step (NS == NP for D = 64 and 128)
  constexpr int A_SLOTS = 5;       // slots that carry the max / threshold work
  constexpr int K_ISSUE = NSLOT / 8, V_ISSUE = NSLOT / 2;  // slots behind which the tile copies are started
  static_assert(NS == NP, "the slot pattern alternates one MFMA of each product");
  float alpha, mx, msc_new, psum = 0.f, q0 = 0.f, q1 = 0.f;
  bool grow;

  // slot i = 2 m + w: w = 0 -> S^T MFMA number m, w = 1 -> O^T MFMA number m.
  //   S^T MFMA m: key block m & 1, contraction step m >> 1 (the two accumulators alternate).
  //   O^T MFMA m: key slice m / DB, row block m % DB (an accumulator comes back every DB MFMAs).
  // The fragments of MFMA pair m+1 are read from LDS while pair m runs.
  auto k_frag = [&](int m) { return lds_read_k(k_tile + (m & 1) * 32 * ROWB + (((2 * (m >> 1)) ^ kx2) << 4)); };
  auto v_frag = [&](int m) {
    return lds_read_vt(v_tile + (16 * (m / DB)) * ROWB + (((4 * (m % DB)) ^ vx2) << 4), 8 * ROWB);
  };
  bf16x8 kf[2], vf[2];
  kf[0] = k_frag(0);
  vf[0] = v_frag(0);
  f32x16 zero;
#pragma unroll
  for (int r = 0; r < 16; ++r) zero[r] = 0.f;

#pragma unroll
  for (int i = 0; i < NSLOT; ++i) {
    const int m = i >> 1, w = i & 1, mb = m & 1;
    if (w == 0 && m + 1 < NS) {
      kf[mb ^ 1] = k_frag(m + 1);
      vf[mb ^ 1] = v_frag(m + 1);
    }
    // ---- matrix pipe.  The empty asm statements order each MFMA against the vector slices around it (all asm
    // volatile statements keep their relative order), which fixes the interleaving written here.
    if (w == 0) {
      const int kb = m & 1, kk = m >> 1;
      asm volatile("" : "+v"(kf[mb]));
      if (kk == 0) s_nxt[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[mb], qf[kk], zero, 0, 0, 0);
      else s_nxt[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[mb], qf[kk], s_nxt[kb], 0, 0, 0);
      asm volatile("" : "+v"(s_nxt[kb]));
    } else {
      const int ks = m / DB, db = m % DB;
      asm volatile("" : "+v"(vf[mb]));
      o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[mb], as_bf16x8(p_prev[ks]), o[db], 0, 0, 0);
      asm volatile("" : "+v"(o[db]));
    }
    // ---- vector pipe slice
    if (kAblateSoftmax) {
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        if ((u * NSLOT) / 16 == i) {
          const int kb = u >> 3, r = 2 * (u & 7);
          p_cur[2 * kb + (r >> 3)][(r & 7) >> 1] = __builtin_amdgcn_perm(
              __float_as_uint(s_cur[kb][r + 1]), __float_as_uint(s_cur[kb][r]), 0x07060302u);
        }
      }
      alpha = 1.f;
      grow = false;
      psum = 1.f;
    } else if (i < 4) {  // row maximum over a quarter of the tile's keys
      const int kb = i >> 1, r0 = 8 * (i & 1);
      float t = i ? mx : s_cur[0][0];
      asm volatile("" : "+v"(t));
#pragma unroll
      for (int r = 0; r < 8; r += 2) t = fmaxf(fmaxf(t, s_cur[kb][r0 + r]), s_cur[kb][r0 + r + 1]);
      mx = (i == 3) ? half_swap_max(t) : t;
      asm volatile("" : "+v"(mx));
    } else if (i == 4) {  // lazy running maximum (log2 domain), rescale factor
      const float mxs = mx * sc;
      grow = mxs > msc + kAtLazyLog2;
      msc_new = grow ? mxs : msc;
      alpha = __builtin_amdgcn_exp2f(msc - msc_new);
      msc = msc_new;
      asm volatile("" : "+v"(alpha), "+v"(msc_new));
    } else {  // exponentials of the elements assigned to this slot
#pragma unroll
      for (int u = 0; u < 16; ++u) {  // unit = two neighbouring keys of the query
        if (A_SLOTS + (u * (NSLOT - A_SLOTS)) / 16 == i) {
          const int kb = u >> 3, r = 2 * (u & 7);
          float a0 = s_cur[kb][r], a1 = s_cur[kb][r + 1];
          asm volatile("" : "+v"(a0), "+v"(a1));  // the slice may not rise above the previous MFMA ...
          const float pe0 = __builtin_amdgcn_exp2f(fmaf(a0, sc, -msc_new));
          const float pe1 = __builtin_amdgcn_exp2f(fmaf(a1, sc, -msc_new));
          // the sums and the pack of the PREVIOUS unit go here, behind this unit's exponentials: a transcendental
          // result takes several issue slots to arrive, and adding it right away stalls the wave
          if (u > 0) {
            const int kbp = (u - 1) >> 3, rp = 2 * ((u - 1) & 7);
            psum += q0;
            psum += q1;
            unsigned pk = pack_bf16(q0, q1);
            asm volatile("" : "+v"(pk), "+v"(psum));
            p_cur[2 * kbp + (rp >> 3)][(rp & 7) >> 1] = pk;
          }
          q0 = pe0;
          q1 = pe1;
          asm volatile("" : "+v"(q0), "+v"(q1));  // ... nor sink below the next one
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    if (i == K_ISSUE) {
      issue_k();
      __builtin_amdgcn_sched_barrier(0);
    }
    if (i == V_ISSUE) {
      issue_v();
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  if (!kAblateSoftmax) {  // the last unit
    psum += q0;
    psum += q1;
    p_cur[3][3] = pack_bf16(q0, q1);
  }
  l_run = fmaf(l_run, alpha, psum);
  // O^T now holds tiles < t scaled by the old maximum; bring it to the new one before tile t is added
  if (__builtin_amdgcn_ballot_w64(grow) != 0) {
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[b][r] *= alpha;
  }
}

// Block mask / ragged tail for the tile starting at key0: register r of s[kb] holds key
// key0 + 32 kb + 8 (r/4) + 4 g + (r%4).
__device__ __forceinline__ void attn_mask(f32x16 (&s)[2], int key0, int lim, int g) {
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int kidx = key0 + 32 * kb + 8 * (r >> 2) + 4 * g + (r & 3);
      if (kidx >= lim) s[kb][r] = -INFINITY;
    }
}

// ---- work decomposition -----------------------------------------------------------------------------------------
// A work item is one (head, query tile of kAtBQ queries); its cost is counted in UNITS of two key tiles (one loop
// iteration): units(qt) = ceil(ceil(visible keys of the tile's last query / 64) / 2).  Items are ordered head-major.
// Whole items on a grid of one workgroup per item leave CUs idle when there are fewer items than CUs (a one-frame
// chunk of 1560 queries is 84 items on 256 CUs), so with a workspace, and when the items fill at most four fifths of
// the chip, the flattened unit list is instead cut into `n_wg` equal contiguous runs, one per workgroup: a run covers
// the tail of one item, possibly some whole items, and the head of another.  A workgroup that does not see all units of an item writes its unnormalised O^T together with
// the running maximum and the row sums into the workspace (slot 2 g for the first segment of workgroup g, 2 g + 1 for
// its last), and attn_combine_kernel merges the partial results of such items afterwards, always in run order, so
// the result does not depend on timing.
struct AttnWork {
  int n_qt;        // query tiles per head
  int units_head;  // units of one head (sum over its query tiles)
  int uniform;     // units of every query tile when they are all equal (no block mask), else 0
  int split;       // 1: equal runs over the unit list; 0: workgroup g takes work item g
  int n_wg;        // logical workgroups
  float* part_o;   // [2 n_wg][kAtBQ][D] fp32
  float* part_ml;  // [2 n_wg][2][kAtBQ] fp32: running maximum (log2 domain), row sum
};

__host__ __device__ inline int attn_units(int qt, int Lq, int n_kept, int Lc, int L_B) {
  const int i_last = (qt + 1) * kAtBQ - 1 < Lq ? (qt + 1) * kAtBQ - 1 : Lq - 1;
  const long long e = ((long long)(i_last / L_B) + 1) * L_B;
  const int vis = n_kept + (int)(e < Lc ? e : Lc);
  return ((vis + kAtTileKeys - 1) / kAtTileKeys + 1) / 2;
}
// first unit of logical workgroup g when U units are cut into G runs
__host__ __device__ inline long long attn_run_begin(long long g, long long U, long long G) { return g * U / G; }

struct AttnArgs {
  AttnParams p;
  AttnWork w;
};

// Wave-uniform values that come out of vector instructions (64-bit divisions are expanded on the vector ALU) are
// moved back to scalar registers, so that addresses built from them can serve as scalar bases.
__device__ __forceinline__ int uniform_i32(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ long long uniform_i64(long long v) {
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)(unsigned long long)v);
  const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)((unsigned long long)v >> 32));
  return (long long)(((unsigned long long)hi << 32) | lo);
}

// GATHER: the cache segment is read through an index list (index-based Select, Sec. 3.4; Eq. 7): K/V stay
// uncompacted and tile row r comes from cache row ids[r].  The 64 ids of a tile travel global -> LDS like the tiles
// themselves (one 4-byte-per-lane load per wave and step, three steps ahead of the K tile that needs them, into a
// small ring of their own), so the vector-memory queue stays one hand-counted stream and a lane picks up its row
// index with one LDS read.
//
// KV8: K and V (both key segments) are stored as 8-bit E4M3 codes with one power-of-two scale per tensor.  The tile
// copies then move half the bytes, into a ring of raw tiles; every wave converts the 1 KB of each raw tile that it
// copied itself to bf16 (scale applied, exact) and writes it, in the swizzled layout the fragment reads expect, into
// one of two bf16 slots per tensor, one step before the matrix instructions read it.  The matrix instructions, the
// softmax and the fragment reads are the bf16 kernel's; the arithmetic is no narrower than in the bf16 kernel.
template <int D, bool OUT_F32, bool GATHER, bool KV8>
__global__ __launch_bounds__(kAtThreads, 1) void chunk_attention_kernel(AttnArgs args) {
  static_assert(!KV8 || (D == 128 && !GATHER), "8-bit K/V: head dim 128, no index list");
  const AttnParams& p = args.p;
  const AttnWork& wk = args.w;
  constexpr int ROWB = 2 * D;                  // bytes per bf16 K/V row of one head (what the fragment reads see)
  constexpr int TILEB = kAtTileKeys * ROWB;    // bytes per bf16 K (or V) tile
  constexpr int CH = D / 8;                    // 16-byte chunks per bf16 row
  constexpr int RPB = 256 / ROWB;              // rows per 256 bytes (one pass over all LDS banks)
  constexpr int ELB = KV8 ? 1 : 2;             // bytes per stored K/V element
  constexpr int SROWB = ELB * D;               // bytes per stored row of one head (what the tile copies move)
  constexpr int STILEB = kAtTileKeys * SROWB;  // bytes per stored tile
  constexpr int SCH = SROWB / 16;              // 16-byte chunks per stored row
  constexpr int RPI = 1024 / SROWB;            // stored rows written by one wave-wide 16-byte-per-lane load
  constexpr int LPT = STILEB / 1024 / kAtWaves;  // such loads per wave per tensor per tile
  constexpr int CK = KV8 ? 2 : kAtStages;      // bf16 tile slots per tensor
  constexpr int LEAD = KV8 ? kAtStages + 1 : kAtStages;  // a K tile is copied this many steps before the step that
                                                         // computes the product of the tile BEFORE it (see the loop)
  static_assert(LPT >= 1, "every wave copies part of every tile");
  constexpr int KD = D / 16;
  constexpr int DB = D / 32;
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds_raw[];
  lds_byte* const k_ring = (lds_byte*)lds_raw;     // bf16 tiles the fragment reads address: CK slots
  lds_byte* const v_ring = k_ring + CK * TILEB;
  // 8-bit K/V: rings of raw tiles behind the bf16 slots (plain layout: lane l of wave w at w * 1024 + 16 l)
  lds_byte* const k_land = KV8 ? v_ring + CK * TILEB : k_ring;   // where the tile copies land
  lds_byte* const v_land = KV8 ? k_land + kAtStages * STILEB : v_ring;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // said to be uniform: what depends on it stays scalar
  // Query block of this wave inside the 256-query tile.  Waves w and w + 4 share a SIMD; they take neighbouring blocks,
  // so that a ragged tile (the last one of a head: 72 of 256 rows at the Wan-1.3B shape) fills SIMDs pairwise and
  // steps at the pace of the full tiles.  With block = wave its few busy waves would each have a SIMD to themselves,
  // run through the keys twice as fast as the other workgroups of the head and pull every K/V line into the L2 long
  // before they need it, i.e. once more from HBM.
  const int qblk = 2 * (wave & 3) + (wave >> 2);
  const int g = lane >> 5, c = lane & 31;
  // Logical workgroup.  Workgroups are handed to the 8 XCDs round-robin in launch order and every XCD has its own
  // L2, so XCD x (workgroups x, x + 8, ...) takes one contiguous range of the head-major work list: at any time an
  // XCD then streams the K/V of one or two heads instead of all of them.
  const int total = gridDim.x;
  const int xcd = blockIdx.x % kAtXcds, xslot = blockIdx.x / kAtXcds;
  const int wg = xcd * (total / kAtXcds) + (xcd < total % kAtXcds ? xcd : total % kAtXcds) + xslot;
  const int L_B = p.block_len;
  const int n_total = p.n_kept + p.Lc;
  const long long ldc_b = p.ld_c * ELB, ldn_b = p.ld_n * ELB;

  // ---- per-lane constants of the global -> LDS tile loads.  Load j of this wave fills LDS rows
  // (wave + W j) * RPI .. + RPI of a tile; lane -> (row, slot); the slot receives chunk (slot ^ swizzle(row)) of that
  // row.  Rows past the end are masked later, so they read a valid row instead.  The chunk segment's base is
  // pre-shifted by -n_kept rows so that both segments are addressed as base + key_index * stride.  A tile that lies
  // inside one segment (all but one or two) needs only a scalar tile base plus a per-lane byte offset prepared here.
  // (the swizzled chunk does not depend on j: consecutive loads of a wave are kAtWaves * RPI rows apart, a multiple
  // of the swizzle period, so load j is load 0 with the scalar base moved on by j * kAtWaves * RPI rows)
  unsigned k_offc, k_offn, v_offc, v_offn;
  {
    const int row = wave * RPI + lane / SCH;
    const int slot = lane % SCH;
    const int kch = KV8 ? slot : slot ^ ((row / RPB) & (CH - 1));          // raw 8-bit tiles are not swizzled
    const int vch = KV8 ? slot : slot ^ (4 * ((row / RPB) & (CH / 4 - 1)));
    k_offc = (unsigned)(row * ldc_b) + kch * 16;
    k_offn = (unsigned)(row * ldn_b) + kch * 16;
    v_offc = (unsigned)(row * ldc_b) + vch * 16;
    v_offn = (unsigned)(row * ldn_b) + vch * 16;
  }
  // ---- LDS read offsets (bytes inside a tile)
  // K fragment (A operand): lane (key row c, half g) reads chunk (2 kk + g) of row c; its slot is (2 kk) ^ kx2
  const int kx2 = g ^ ((c / RPB) & (CH - 1));
  const int k_off = c * ROWB;
  // V^T fragment via transposing reads: 16-lane group = (d-half, key group g); lane i of the group points at key
  // row rr = 4 g + i/4, four consecutive d at 4 (i%4).  32 lanes (one key group) read 4 rows x 64 bytes per
  // instruction; the swizzle spreads those over all banks.  Slot of d-block b is ((4 b) ^ vx2) + cl.
  const int i16 = lane & 15;
  const int rr = 4 * g + (i16 >> 2);
  const int vx2 = 4 * ((rr / RPB) & (CH / 4 - 1));
  const int cl = 2 * ((lane >> 4) & 1) + ((i16 & 3) >> 1);
  const int v_off = rr * ROWB + ((i16 & 1) << 3) + (cl << 4);
  const float sc = p.scale_log2;
  int* const id_ring = reinterpret_cast<int*>(lds_raw + 2 * kAtStages * TILEB);  // gather variant (bf16 K/V only)

  // ---- this workgroup's run of units [u, u_end) in the flattened (head, query tile, unit) list
  long long u, u_end;
  int qt, h, pre;  // current item and the units of its head that precede it
  if (wk.split) {
    const long long U = (long long)wk.units_head * (p.N_heads);
    u = uniform_i64(attn_run_begin(wg, U, wk.n_wg));
    u_end = uniform_i64(attn_run_begin(wg + 1, U, wk.n_wg));
    h = uniform_i32((int)(u / wk.units_head));
    const int r = (int)(u - (long long)h * wk.units_head);
    if (wk.uniform) {
      qt = uniform_i32(r / wk.uniform);
      pre = qt * wk.uniform;
    } else {
      qt = 0;
      pre = 0;
      for (;;) {
        const int cq = attn_units(qt, p.Lq, p.n_kept, p.Lc, L_B);
        if (pre + cq > r) break;
        pre += cq;
        ++qt;
      }
    }
  } else {
    h = uniform_i32(wg / wk.n_qt);
    qt = wg - h * wk.n_qt;
    pre = 0;
    for (int q2 = 0; q2 < qt; ++q2) pre += attn_units(q2, p.Lq, p.n_kept, p.Lc, L_B);
    u = (long long)h * wk.units_head + pre;
    u_end = u + attn_units(qt, p.Lq, p.n_kept, p.Lc, L_B);
  }
  bool first_segment = true;

#pragma unroll 1
  while (u < u_end) {
    // ---- segment: units [pa, pb) of item (h, qt) = key tiles [2 pa, 2 pb)
    const int units = __builtin_amdgcn_readfirstlane(attn_units(qt, p.Lq, p.n_kept, p.Lc, L_B));
    const int pa = __builtin_amdgcn_readfirstlane((int)(u - ((long long)h * wk.units_head + pre)));
    const long long room = u_end - u;
    const int pb = __builtin_amdgcn_readfirstlane(room < units - pa ? pa + (int)room : units);
    const bool whole = pa == 0 && pb == units;
    const int n_iter = pb - pa;
    const int tb = 2 * pa;  // first key tile of the segment
    const int i_first = uniform_i32(qt) * kAtBQ;
    const long long head_off = (long long)uniform_i32(h) * D;

    // number of visible keys: per lane (its query) and the tile's first query, both cut at the segment's end
    auto visible = [&](int i) {
      const long long e = ((long long)(i / L_B) + 1) * L_B;
      return p.n_kept + (int)(e < p.Lc ? e : p.Lc);
    };
    const int key_end = 2 * pb * kAtTileKeys;
    const int q_row = i_first + qblk * 32 + c;
    const int lim_q = visible(q_row < p.Lq ? q_row : p.Lq - 1);
    const int lim = lim_q < key_end ? lim_q : key_end;
    const int lim_first = visible(i_first);
    const int lim_min = lim_first < key_end ? lim_first : key_end;

    // ids ring (gather variant): slot u % kAtIdStages holds the 64 ids of tile u, clamped to the list's end
    auto issue_ids = [&](int tile) {
      if (lane < 8) {  // wave w brings ids 8 w .. 8 w + 7 of the tile: one load per wave, 64 ids per workgroup
        int idx = tile * kAtTileKeys + 8 * wave + lane;
        idx = idx < p.n_kept ? idx : p.n_kept - 1;
        lds_byte* dst = (lds_byte*)(id_ring + (tile % kAtIdStages) * kAtTileKeys + 8 * wave);
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                     :
                     : "s"(__builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)dst)), "v"((unsigned)idx * 4u), "s"(p.ids)
                     : "memory");
      }
    };
    auto tile_id = [&](int tile, int row) {  // cache row behind tile row `row`, never outside the cache
      const int id = ((const __attribute__((address_space(3))) int*)id_ring)[(tile % kAtIdStages) * kAtTileKeys + row];
      return id < 0 ? 0 : (id < p.n_cache ? id : p.n_cache - 1);
    };
    auto issue_one = [&](int tile_, const unsigned short* cache, const unsigned short* chunk, lds_byte* ring,
                         unsigned offc, unsigned offn, bool is_v) {
      const int tile = uniform_i32(tile_);
      const int stage = tile % kAtStages;
      const int key0 = tile * kAtTileKeys;
      const char* base_c = reinterpret_cast<const char*>(cache) + head_off * ELB;
      const char* base_n = reinterpret_cast<const char*>(chunk) + head_off * ELB - (long long)p.n_kept * ldn_b;
      const bool all_cache = key0 + kAtTileKeys <= p.n_kept;
      const bool all_chunk = key0 >= p.n_kept && key0 + kAtTileKeys <= n_total;
      if (GATHER && all_cache) {  // workgroup-uniform
        // Registers are scarce here, so nothing per-lane is kept between steps: the swizzled chunk is recomputed (it
        // does not depend on j: consecutive loads of a wave are 8 RPI rows apart) and the address is the head's
        // base plus a 32-bit offset (the host rejects caches of 4 GiB or more per tensor for this variant).
        const int rl = lane / CH, slot = lane % CH;
        const int row0 = wave * RPI + rl;  // the tile row of load 0
        const unsigned chunk16 =
            (unsigned)((is_v ? slot ^ (4 * ((row0 / RPB) & (CH / 4 - 1))) : slot ^ ((row0 / RPB) & (CH - 1))) << 4);
#pragma unroll
        for (int j = 0; j < LPT; ++j) {
          const int id = tile_id(tile, (wave + kAtWaves * j) * RPI + rl);
          lds_byte* dst = ring + stage * STILEB + (wave + kAtWaves * j) * 1024;
          dma_row_chunks_at(base_c, (unsigned)id * (unsigned)ldc_b + chunk16,
                            __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)dst));
        }
      } else if (all_cache || all_chunk) {  // workgroup-uniform
        const bool from_cache = all_cache && !GATHER;  // (a gathered all-cache tile took the branch above)
        // scalar address arithmetic: 32 x 32 -> 64-bit products (row strides are below 4 GiB), which the scalar
        // unit has; a 64 x 64-bit product would be done on the vector ALU and leave the base in vector registers
        const unsigned ld_b = (unsigned)(from_cache ? ldc_b : ldn_b);
        const char* tile_base = (from_cache ? base_c : base_n) + (unsigned long long)(unsigned)key0 * ld_b;
        const unsigned off = from_cache ? offc : offn;
#pragma unroll
        for (int j = 0; j < LPT; ++j) {
          lds_byte* dst = ring + stage * STILEB + (wave + kAtWaves * j) * 1024;
          dma_row_chunks_at(tile_base + (unsigned long long)(unsigned)(j * kAtWaves * RPI) * ld_b, off,
                            __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)dst));
        }
      } else {
#pragma unroll
        for (int j = 0; j < LPT; ++j) {
          const int row = (wave + kAtWaves * j) * RPI + lane / SCH;
          const int slot = lane % SCH;
          const int ch = KV8 ? slot : (is_v ? slot ^ (4 * ((row / RPB) & (CH / 4 - 1))) : slot ^ ((row / RPB) & (CH - 1)));
          int kidx = key0 + row;
          kidx = kidx < n_total ? kidx : n_total - 1;
          const bool in_cache = kidx < p.n_kept;
          if (GATHER && in_cache) kidx = tile_id(tile, row);
          const char* src = (in_cache ? base_c : base_n) +
                            (unsigned long long)(unsigned)kidx * (unsigned long long)(in_cache ? ldc_b : ldn_b) + ch * 16;
          lds_byte* dst = ring + stage * STILEB + (wave + kAtWaves * j) * 1024;
          dma_row_chunks(src, __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)dst));
        }
      }
    };
    // Step t (relative to the segment) reads K tile tb+t+1 and V tile tb+t-1.  During it K(t+S) and V(t+S-2) are
    // issued into the slots of K(t) and V(t-2), whose last readers finished in step t-1.  Tiles past the end of the
    // key axis hold clamped rows and are masked or never read.
    // In the gather variant the ids of tiles kt and kt-2 must already be visible in the ids ring.
    auto issue_k_tile = [&](int kt) { issue_one(tb + kt, p.Kc, p.Kn, k_land, k_offc, k_offn, false); };
    auto issue_v_tile = [&](int kt) {
      if (kt >= 2) issue_one(tb + kt - 2, p.Vc, p.Vn, v_land, v_offc, v_offn, true);
    };
    auto issue_tiles = [&](int kt) {  // kt relative to the segment
      issue_k_tile(kt);
      issue_v_tile(kt);
    };
    auto k_addr = [&](int t) { return k_ring + ((tb + t) % CK) * TILEB + k_off; };
    auto v_addr = [&](int t) { return v_ring + ((tb + t) % CK) * TILEB + v_off; };
    // 8-bit K/V: this wave's 1 KB of raw tile t (the part it copied itself, so only its own copies must have landed)
    // -> bf16, into the slot of tile t.  Lane l holds 16 codes of key row w * RPI + l / SCH, d = 16 (l % SCH) .. + 16:
    // two 16-byte chunks of the bf16 row, stored with the swizzle of the fragment reads.
    auto cook = [&](int t, bool is_v) {
      typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
      const int tile = tb + t;
      const u32x4 raw = *(const lds_u32x4*)((is_v ? v_land : k_land) + (tile % kAtStages) * STILEB + wave * 1024 + lane * 16);
      const int row = wave * RPI + lane / SCH, chunk = lane % SCH;
      const int sw = is_v ? 4 * ((row / RPB) & (CH / 4 - 1)) : (row / RPB) & (CH - 1);
      lds_byte* dst = (is_v ? v_ring : k_ring) + (tile % CK) * TILEB + row * ROWB;
      const float scl = is_v ? p.v_scale : p.k_scale;
      u32x4 lo, hi;
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        lo[2 * e] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[e], scl, false));
        lo[2 * e + 1] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[e], scl, true));
        hi[2 * e] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[2 + e], scl, false));
        hi[2 * e + 1] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[2 + e], scl, true));
      }
      *(lds_u32x4*)(dst + (((2 * chunk) ^ sw) << 4)) = lo;
      *(lds_u32x4*)(dst + (((2 * chunk + 1) ^ sw) << 4)) = hi;
    };
    // what a step does for the 8-bit tiles: K(t+2) and V(t) become bf16 one step before they are read
    auto cook_step = [&](int t, int n_tiles_seg) {
      if (t + 2 < n_tiles_seg) cook(t + 2, false);
      if (t > 0) cook(t, true);
    };

    // Q^T fragments (B operand): lane (query c, half g) holds Q[q][16 kk + 8 g .. +8]
    bf16x8 qf[KD];
    {
      const int qi = q_row < p.Lq ? q_row : p.Lq - 1;
      const unsigned short* qp = p.Q + (long long)qi * p.ld_q + head_off + 8 * g;
#pragma unroll
      for (int kk = 0; kk < KD; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qp + 16 * kk);
    }

    // ---- prologue: fill the ring (K tiles 0..S-1, V tiles 0..S-3 of the segment), then S^T(0)
    if (GATHER) {  // ids of the tiles whose loads are issued before step kAtIdLead's ids arrive
#pragma unroll
      for (int i = 0; i < kAtStages + kAtIdLead; ++i) issue_ids(tb + i);
      wait_vmcnt<0>();
      __builtin_amdgcn_s_barrier();
    }
#pragma unroll
    for (int i = 0; i < kAtStages; ++i) issue_tiles(i);
    wait_vmcnt<0>();
    if (KV8) {  // the first product needs K(0), step 0 reads K(1) and (with P = 0) V(0)
      cook(0, false);
      cook(1, false);
      cook(0, true);
      __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the bf16 rows are written before the barrier lets others read
      // the raw ring has kAtStages slots: K(kAtStages) goes where this wave's part of K(0) was, now that it is converted
      issue_tiles(kAtStages);
    }
    __builtin_amdgcn_s_barrier();

    // A wave whose 32 queries all lie past the end (the last query tile of a head is usually ragged) still loads its
    // share of every tile and joins every barrier, but does no arithmetic: on this chip energy is time.
    if (__builtin_amdgcn_readfirstlane(i_first + qblk * 32) >= p.Lq) {
      __builtin_amdgcn_s_barrier();  // the one after the other waves' first product
#pragma unroll 1
      for (int t = 0; t < 2 * n_iter; ++t) {
        if (GATHER) issue_ids(tb + t + kAtStages + kAtIdLead);
        if (!kAblateLoads) issue_tiles(t + LEAD);
        if (KV8) {
          cook_step(t, 2 * n_iter);
          __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
        }
        wait_vmcnt<(kAtStages - 2) * (2 * LPT + (GATHER ? 1 : 0))>();
        __builtin_amdgcn_s_barrier();
      }
      wait_vmcnt<0>();
    } else {
      f32x16 o[DB];
#pragma unroll
      for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[b][r] = 0.f;
      f32x16 s_a[2], s_b[2];
      u32x4 p_a[4], p_b[4];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int e = 0; e < 4; ++e) { p_a[ks][e] = 0u; p_b[ks][e] = 0u; }
      // The running maximum starts at a finite sentinel, not at -inf: a segment may begin with tiles that are masked
      // entirely for some queries, and (-inf) - (-inf) in the rescale factor would poison their sums.
      float msc = kAtNoMax, l_run = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s_a[kb][r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KD; ++kk) {
          const bf16x8 a = lds_read_k(k_addr(0) + kb * 32 * ROWB + (((2 * kk) ^ kx2) << 4));
          s_a[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], s_a[kb], 0, 0, 0);
        }
      }
      // Step 0 refills the ring slot of K(0): every wave must have its K(0) fragments in registers before any wave
      // issues that load.  The products above have consumed them, so one barrier here is enough; inside the loop
      // the barrier that ends step t-1 plays this role for step t.
      asm volatile("" : "+v"(s_a[0]), "+v"(s_a[1]));
      __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
      __builtin_amdgcn_s_barrier();

      // Step t: S^T(t+1) into the "next" registers, softmax of S^T(t), O^T += tile t-1.  Iteration T runs step 2T
      // (s_a -> p_a, next into s_b, adds p_b) and step 2T+1 (s_b -> p_b, next into s_a, adds p_a).  A segment always
      // holds an even number of tiles: a tile past the end is fully masked and contributes nothing.  Before the first
      // tile p_b is zero, and when there is no next tile the S^T product re-reads the current one (its result is
      // never used).  After each step: K(t+2) and V(t) must have landed before the next step; only the loads of the
      // last two steps may stay in flight.
#pragma unroll 1
      for (int T = 0; T < n_iter; ++T) {
        {
          const int t = 2 * T;
          if (GATHER) issue_ids(tb + t + kAtStages + kAtIdLead);
          if (KV8) cook_step(t, 2 * n_iter);
          if ((tb + t + 1) * kAtTileKeys > lim_min) attn_mask(s_a, (tb + t) * kAtTileKeys, lim, g);
          attn_step<D>(
              s_a, s_b, p_b, p_a, o, qf, msc, l_run, k_addr(t + 1), v_addr(t > 0 ? t - 1 : 0), kx2, vx2, sc,
              [&] { if (!kAblateLoads) issue_k_tile(t + LEAD); }, [&] { if (!kAblateLoads) issue_v_tile(t + LEAD); });
          if (KV8) __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): this step's bf16 rows are written
          wait_vmcnt<(kAtStages - 2) * (2 * LPT + (GATHER ? 1 : 0))>();
          __builtin_amdgcn_s_barrier();
        }
        {
          const int t = 2 * T + 1;
          if (GATHER) issue_ids(tb + t + kAtStages + kAtIdLead);
          if (KV8) cook_step(t, 2 * n_iter);
          if ((tb + t + 1) * kAtTileKeys > lim_min) attn_mask(s_b, (tb + t) * kAtTileKeys, lim, g);
          attn_step<D>(
              s_b, s_a, p_a, p_b, o, qf, msc, l_run, k_addr(T + 1 < n_iter ? t + 1 : t), v_addr(t - 1), kx2, vx2, sc,
              [&] { if (!kAblateLoads) issue_k_tile(t + LEAD); }, [&] { if (!kAblateLoads) issue_v_tile(t + LEAD); });
          if (KV8) __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
          wait_vmcnt<(kAtStages - 2) * (2 * LPT + (GATHER ? 1 : 0))>();
          __builtin_amdgcn_s_barrier();
        }
      }
      // the last tile's contribution
      {
        const lds_byte* vt = v_addr(2 * n_iter - 1);
#pragma unroll
        for (int m = 0; m < 4 * DB; ++m) {
          const bf16x8 a = lds_read_vt(vt + (16 * (m / DB)) * ROWB + (((4 * (m % DB)) ^ vx2) << 4), 8 * ROWB);
          o[m % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, as_bf16x8(p_b[m / DB]), o[m % DB], 0, 0, 0);
        }
      }
      wait_vmcnt<0>();  // nothing may still be writing this workgroup's LDS when the ring is reused or it retires

      // store: lane holds query c, d = 32 b + 8 (r/4) + 4 g + (r%4)
      const float l_tot = half_swap_sum(l_run);
      if (whole) {  // normalise and write O
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
      } else if (q_row < p.Lq) {  // partial result of this segment, for attn_combine_kernel
        const int pslot = 2 * wg + (first_segment ? 0 : 1);
        const int ql = qblk * 32 + c;
        float* po = wk.part_o + ((long long)pslot * kAtBQ + ql) * D;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4)
            *reinterpret_cast<float4*>(po + 32 * b + 8 * q4 + 4 * g) =
                make_float4(o[b][4 * q4 + 0], o[b][4 * q4 + 1], o[b][4 * q4 + 2], o[b][4 * q4 + 3]);
        if (g == 0) {
          float* pml = wk.part_ml + (long long)pslot * 2 * kAtBQ;
          pml[ql] = msc;
          pml[kAtBQ + ql] = l_tot;
        }
      }
    }
    // ---- next segment: the next item of the list, from its first unit
    u += n_iter;
    first_segment = false;
    if (u < u_end) {
      __builtin_amdgcn_s_barrier();  // every wave has finished reading the ring before it is refilled
      pre += units;
      if (++qt == wk.n_qt) { qt = 0; pre = 0; ++h; }
    }
  }
}

// Merges the partial results of the items that more than one workgroup worked on.  kAtCombineSplit workgroups per
// item, each taking a band of its query rows; the partials are taken in run order, whoever wrote them first.
//   O = sum_p 2^(m_p - m) O_p / sum_p 2^(m_p - m) l_p   with m = max_p m_p.
constexpr int kAtCombineSplit = 8;
constexpr int kAtCombineRows = kAtBQ / kAtCombineSplit;
template <int D, bool OUT_F32>
__global__ __launch_bounds__(256) void attn_combine_kernel(AttnArgs args) {
  const AttnParams& p = args.p;
  const AttnWork& wk = args.w;
  __shared__ float s_m[kAtCombineRows], s_inv[kAtCombineRows];
  const int item = blockIdx.x / kAtCombineSplit, band = blockIdx.x % kAtCombineSplit;
  const int h = item / wk.n_qt, qt = item - h * wk.n_qt;
  int pre = 0;
  if (wk.uniform) pre = qt * wk.uniform;
  else
    for (int q2 = 0; q2 < qt; ++q2) pre += attn_units(q2, p.Lq, p.n_kept, p.Lc, p.block_len);
  const int units = attn_units(qt, p.Lq, p.n_kept, p.Lc, p.block_len);
  const long long U = (long long)wk.units_head * p.N_heads, G = wk.n_wg;
  const long long s = (long long)h * wk.units_head + pre, e = s + units;
  // the run that holds unit x: the largest g with floor(g U / G) <= x
  const int g_first = (int)(((s + 1) * G - 1) / U), g_last = (int)((e * G - 1) / U);
  if (g_first == g_last) return;  // one workgroup saw the whole item and wrote O itself
  // slot of run gg's partial result for this item: 2 gg if the run starts inside the item, else 2 gg + 1
  const int slot_first = 2 * g_first + (attn_run_begin(g_first, U, G) >= s ? 0 : 1);
  auto slot_of = [&](int gg) { return gg == g_first ? slot_first : 2 * gg; };
  const int rows_item = p.Lq - qt * kAtBQ < kAtBQ ? p.Lq - qt * kAtBQ : kAtBQ;
  const int row0 = band * kAtCombineRows;
  const int rows = rows_item - row0 < kAtCombineRows ? rows_item - row0 : kAtCombineRows;
  if (rows <= 0) return;
  const int tid = threadIdx.x;
  if (tid < rows) {
    float m = kAtNoMax;
    for (int gg = g_first; gg <= g_last; ++gg) m = fmaxf(m, wk.part_ml[(long long)slot_of(gg) * 2 * kAtBQ + row0 + tid]);
    float l = 0.f;
    for (int gg = g_first; gg <= g_last; ++gg) {
      const float* ml = wk.part_ml + (long long)slot_of(gg) * 2 * kAtBQ + row0;
      l += ml[kAtBQ + tid] * __builtin_amdgcn_exp2f(ml[tid] - m);
    }
    s_m[tid] = m;
    s_inv[tid] = 1.0f / l;
  }
  __syncthreads();
  constexpr int C4 = D / 4;  // float4 groups per row
  for (int e4 = tid; e4 < rows * C4; e4 += 256) {
    const int row = e4 / C4, d0 = 4 * (e4 - row * C4);
    const float m = s_m[row];
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int gg = g_first; gg <= g_last; ++gg) {
      const int sl = slot_of(gg);
      const float wgt = __builtin_amdgcn_exp2f(wk.part_ml[(long long)sl * 2 * kAtBQ + row0 + row] - m);
      const float4 v = *reinterpret_cast<const float4*>(wk.part_o + ((long long)sl * kAtBQ + row0 + row) * D + d0);
      acc.x = fmaf(v.x, wgt, acc.x); acc.y = fmaf(v.y, wgt, acc.y);
      acc.z = fmaf(v.z, wgt, acc.z); acc.w = fmaf(v.w, wgt, acc.w);
    }
    const float inv = s_inv[row];
    const long long off = (long long)(qt * kAtBQ + row0 + row) * p.ld_o + (long long)h * D + d0;
    if (OUT_F32) {
      *reinterpret_cast<float4*>(static_cast<float*>(p.O) + off) = make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
    } else {
      bf16x4 ob;
      ob[0] = (__bf16)(acc.x * inv); ob[1] = (__bf16)(acc.y * inv); ob[2] = (__bf16)(acc.z * inv); ob[3] = (__bf16)(acc.w * inv);
      *reinterpret_cast<bf16x4*>(static_cast<unsigned short*>(p.O) + off) = ob;
    }
  }
}

template <int D, bool OUT_F32, bool GATHER, bool KV8 = false>
int launch_variant(hipStream_t st, const AttnArgs& a) {
  static LdsLimit lds_limit;
  const int rc = set_lds_limit(lds_limit, chunk_attention_kernel<D, OUT_F32, GATHER, KV8>, attn_lds_bytes(D, GATHER));
  if (rc != PAFU_OK) return rc;
  hipLaunchKernelGGL((chunk_attention_kernel<D, OUT_F32, GATHER, KV8>), dim3(a.w.n_wg), dim3(kAtThreads),
                     attn_lds_bytes(D, GATHER), st, a);
  if (a.w.split)
    hipLaunchKernelGGL((attn_combine_kernel<D, OUT_F32>), dim3(a.w.n_qt * a.p.N_heads * kAtCombineSplit), dim3(256), 0,
                       st, a);
  return check_launch();
}

template <bool GATHER>
int launch_dims(hipStream_t st, const AttnArgs& a, int D, bool f32) {
  if (D == 128) return f32 ? launch_variant<128, true, GATHER>(st, a) : launch_variant<128, false, GATHER>(st, a);
  return f32 ? launch_variant<64, true, GATHER>(st, a) : launch_variant<64, false, GATHER>(st, a);
}

}  // namespace

int attention_study_build() { return PAFU_ATTN_ABLATE; }

// Bytes of workspace with which every launch can cut its work into equal runs: two partial-result slots for each of
// at most kAtMaxRuns workgroups.
size_t attention_workspace_bytes(int D) {
  return (size_t)2 * kAtMaxRuns * ((size_t)kAtBQ * D + 2 * kAtBQ) * sizeof(float);
}

int launch_attention(hipStream_t st, const void* Q, int Lq, const void* Kc, const void* Vc, int n_kept,
                     const void* Kn, const void* Vn, int Lc, int N, int D, long long ld_q, long long ld_c,
                     long long ld_n, long long ld_o, int block_len, float scale, void* O, int out_dtype,
                     void* workspace, size_t workspace_bytes, const int* ids, int n_cache, int kv_dtype,
                     float k_scale, float v_scale) {
  AttnArgs a;
  AttnParams& p = a.p;
  p.ids = ids;
  p.n_cache = n_cache;
  p.Q = static_cast<const unsigned short*>(Q);
  p.Kc = static_cast<const unsigned short*>(Kc);
  p.Vc = static_cast<const unsigned short*>(Vc);
  p.Kn = static_cast<const unsigned short*>(Kn);
  p.Vn = static_cast<const unsigned short*>(Vn);
  p.O = O;
  p.ld_q = ld_q; p.ld_c = ld_c; p.ld_n = ld_n; p.ld_o = ld_o;
  p.Lq = Lq; p.n_kept = n_kept; p.Lc = Lc; p.N_heads = N;
  p.block_len = block_len < Lc ? block_len : Lc;  // blocks at least as long as the chunk mean "no mask"
  p.scale_log2 = scale * 1.44269504088896340736f;
  p.k_scale = k_scale;
  p.v_scale = v_scale;

  AttnWork& w = a.w;
  w.n_qt = (Lq + kAtBQ - 1) / kAtBQ;
  long long units_head = 0;
  int u0 = attn_units(0, Lq, n_kept, Lc, p.block_len);
  bool uniform = true;
  for (int qt = 0; qt < w.n_qt; ++qt) {
    const int cq = attn_units(qt, Lq, n_kept, Lc, p.block_len);
    units_head += cq;
    uniform = uniform && cq == u0;
  }
  w.units_head = (int)units_head;
  w.uniform = uniform ? u0 : 0;
  const long long items = (long long)w.n_qt * N, U = units_head * N;
  // Equal runs pay off when whole items leave a good part of the chip idle (few query tiles, long key axis).  With the
  // chip nearly full the launch is limited by power, not by CU time, and the merge pass only adds to it (measured on
  // the Wan-1.3B layer: 228 items on 256 CUs, 4 percent slower with equal runs; 192 items, 12 percent faster; 84
  // items, 2 times faster), and over several rounds contiguous runs would spread an XCD's workgroups over several
  // heads and thrash its L2.  They need the workspace, and runs of at least a few units each.
  int cus = compute_units();
  if (cus > kAtMaxRuns) cus = kAtMaxRuns;
  const bool uneven = items * 5 <= (long long)cus * 4 || kStudySplitAlways;
  w.split = 0;
  w.n_wg = (int)items;
  w.part_o = nullptr;
  w.part_ml = nullptr;
  if (uneven && workspace != nullptr && U >= 4ll * cus) {
    const size_t need = (size_t)2 * cus * ((size_t)kAtBQ * D + 2 * kAtBQ) * sizeof(float);
    if (workspace_bytes >= need && (reinterpret_cast<uintptr_t>(workspace) & 15u) == 0) {
      w.split = 1;
      w.n_wg = cus;
      w.part_o = static_cast<float*>(workspace);
      w.part_ml = w.part_o + (size_t)2 * cus * kAtBQ * D;
    }
  }
  const bool f32 = out_dtype == PAFU_F32;
  if (kv_dtype == PAFU_FP8_E4M3)  // validated by the caller: head dim 128, no index list
    return f32 ? launch_variant<128, true, false, true>(st, a) : launch_variant<128, false, false, true>(st, a);
  return ids != nullptr && n_kept > 0 ? launch_dims<true>(st, a, D, f32) : launch_dims<false>(st, a, D, f32);
}

}  // namespace pafu

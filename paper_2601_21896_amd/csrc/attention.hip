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
  int Lq, n_kept, Lc, block_len;
  float scale_log2;  // softmax scale * log2(e)
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
template <int D>
__device__ __forceinline__ void attn_step(const f32x16 (&s_cur)[2], f32x16 (&s_nxt)[2], const u32x4 (&p_prev)[4],
                                          u32x4 (&p_cur)[4], f32x16 (&o)[D / 32], const bf16x8 (&qf)[D / 16],
                                          float& msc, float& l_run, const lds_byte* k_tile, const lds_byte* v_tile,
                                          int kx2, int vx2, float sc) {
  constexpr int ROWB = 2 * D;
  constexpr int KD = D / 16;
  constexpr int DB = D / 32;
  constexpr int NS = 2 * KD;       // MFMAs of S^T(t+1): 2 key blocks x KD contraction steps
  constexpr int NP = 4 * DB;       // MFMAs of the O^T update: 4 key slices x DB row blocks
  constexpr int NSLOT = NS + NP;   // MFMAs per step (NS == NP for D = 64 and 128)
  constexpr int A_SLOTS = 5;       // slots that carry the max / threshold work
  static_assert(NS == NP, "the slot pattern alternates one MFMA of each product");
  float alpha, mx, msc_new, psum = 0.f;
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
    if (i < 4) {  // row maximum over a quarter of the tile's keys
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
          psum += pe0;
          psum += pe1;
          unsigned pk = pack_bf16(pe0, pe1);
          asm volatile("" : "+v"(pk), "+v"(psum));  // ... nor sink below the next one
          p_cur[2 * kb + (r >> 3)][(r & 7) >> 1] = pk;
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
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

// GATHER: the cache segment is read through an index list (index-based Select, Sec. 3.4; Eq. 7): K/V stay
// uncompacted and tile row r comes from cache row ids[r].  The 64 ids of a tile travel global -> LDS like the tiles
// themselves (one 4-byte-per-lane load per wave and step, three steps ahead of the K tile that needs them, into a
// small ring of their own), so the vector-memory queue stays one hand-counted stream and a lane picks up its row
// index with one LDS read.
template <int D, bool OUT_F32, bool GATHER>
__global__ __launch_bounds__(kAtThreads, 1) void chunk_attention_kernel(AttnParams p) {
  constexpr int ROWB = 2 * D;                  // bytes per K/V row of one head
  constexpr int TILEB = kAtTileKeys * ROWB;    // bytes per K (or V) tile
  constexpr int CH = D / 8;                    // 16-byte chunks per row
  constexpr int RPB = 256 / ROWB;              // rows per 256 bytes (one pass over all LDS banks)
  constexpr int RPI = 1024 / ROWB;             // rows written by one wave-wide 16-byte-per-lane load
  constexpr int LPT = TILEB / 1024 / kAtWaves; // such loads per wave per tensor per tile
  constexpr int KD = D / 16;
  constexpr int DB = D / 32;
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds_raw[];
  lds_byte* const k_ring = (lds_byte*)lds_raw;
  lds_byte* const v_ring = k_ring + kAtStages * TILEB;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, c = lane & 31;
  // Workgroup -> (head, query tile).  Workgroups are handed to the 8 XCDs round-robin in launch order and every XCD
  // has its own L2, so XCD x (workgroups x, x + 8, ...) takes one contiguous range of the head-major work list:
  // at any time an XCD then streams the K/V of one or two heads instead of all of them.
  const int n_qt = (p.Lq + kAtBQ - 1) / kAtBQ;
  const int total = gridDim.x;
  const int xcd = blockIdx.x % kAtXcds, slot = blockIdx.x / kAtXcds;
  const int work = xcd * (total / kAtXcds) + (xcd < total % kAtXcds ? xcd : total % kAtXcds) + slot;
  const int h = work / n_qt;
  const int i_first = (work - h * n_qt) * kAtBQ;
  const int i_last = (i_first + kAtBQ - 1 < p.Lq) ? i_first + kAtBQ - 1 : p.Lq - 1;
  const int L_B = p.block_len;
  const int n_total = p.n_kept + p.Lc;
  const long long head_off = (long long)h * D;

  // number of visible keys: per lane (its query) and the workgroup's extremes
  auto visible = [&](int i) {
    const int e = (i / L_B + 1) * L_B;
    return p.n_kept + (e < p.Lc ? e : p.Lc);
  };
  const int q_row = i_first + wave * 32 + c;
  const int lim = visible(q_row < p.Lq ? q_row : p.Lq - 1);
  const int lim_min = visible(i_first);
  const int lim_max = visible(i_last);
  const int n_tiles = (lim_max + kAtTileKeys - 1) / kAtTileKeys;  // key tiles this workgroup visits
  const int n_iter = (n_tiles + 1) / 2;                           // two tiles per loop iteration

  // ---- global -> LDS tile loads.  Load j of this wave fills LDS rows (wave + W j) * RPI .. + RPI of a tile;
  // lane -> (row, slot); the slot receives chunk (slot ^ swizzle(row)) of that row.  Rows past the end are masked
  // later, so they read a valid row instead.  The chunk segment's base is pre-shifted by -n_kept rows so that both
  // segments are addressed as base + key_index * stride.  A tile that lies inside one segment (all but one or two)
  // needs only a scalar tile base plus a per-lane byte offset prepared here.
  const long long ldc_b = p.ld_c * 2, ldn_b = p.ld_n * 2;
  unsigned k_offc[LPT], k_offn[LPT], v_offc[LPT], v_offn[LPT];
#pragma unroll
  for (int j = 0; j < LPT; ++j) {
    const int row = (wave + kAtWaves * j) * RPI + lane / CH;
    const int slot = lane % CH;
    const int kch = slot ^ ((row / RPB) & (CH - 1));
    const int vch = slot ^ (4 * ((row / RPB) & (CH / 4 - 1)));
    k_offc[j] = (unsigned)(row * ldc_b) + kch * 16;
    k_offn[j] = (unsigned)(row * ldn_b) + kch * 16;
    v_offc[j] = (unsigned)(row * ldc_b) + vch * 16;
    v_offn[j] = (unsigned)(row * ldn_b) + vch * 16;
  }
  // ids ring (gather variant): slot u % kAtIdStages holds the 64 ids of tile u, clamped to the list's end
  int* const id_ring = reinterpret_cast<int*>(lds_raw + 2 * kAtStages * TILEB);
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
  auto issue_one = [&](int tile, const unsigned short* cache, const unsigned short* chunk, lds_byte* ring,
                       const unsigned (&offc)[LPT], const unsigned (&offn)[LPT], bool is_v) {
    const int stage = tile % kAtStages;
    const int key0 = tile * kAtTileKeys;
    const char* base_c = reinterpret_cast<const char*>(cache + head_off);
    const char* base_n = reinterpret_cast<const char*>(chunk + head_off) - (long long)p.n_kept * ldn_b;
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
        lds_byte* dst = ring + stage * TILEB + (wave + kAtWaves * j) * 1024;
        dma_row_chunks_at(base_c, (unsigned)id * (unsigned)ldc_b + chunk16,
                          __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)dst));
      }
    } else if (all_cache || all_chunk) {  // workgroup-uniform
      const char* tile_base = all_cache ? base_c + (long long)key0 * ldc_b : base_n + (long long)key0 * ldn_b;
#pragma unroll
      for (int j = 0; j < LPT; ++j) {
        lds_byte* dst = ring + stage * TILEB + (wave + kAtWaves * j) * 1024;
        const unsigned off = GATHER ? offn[0] + (unsigned)(j * kAtWaves * RPI * ldn_b) : (all_cache ? offc[j] : offn[j]);
        dma_row_chunks(tile_base + off, __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)dst));
      }
    } else {
#pragma unroll
      for (int j = 0; j < LPT; ++j) {
        const int row = (wave + kAtWaves * j) * RPI + lane / CH;
        const int slot = lane % CH;
        const int ch = is_v ? slot ^ (4 * ((row / RPB) & (CH / 4 - 1))) : slot ^ ((row / RPB) & (CH - 1));
        int kidx = key0 + row;
        kidx = kidx < n_total ? kidx : n_total - 1;
        const bool in_cache = kidx < p.n_kept;
        if (GATHER && in_cache) kidx = tile_id(tile, row);
        const char* src = (in_cache ? base_c : base_n) +
                          (unsigned long long)(unsigned)kidx * (unsigned long long)(in_cache ? ldc_b : ldn_b) + ch * 16;
        lds_byte* dst = ring + stage * TILEB + (wave + kAtWaves * j) * 1024;
        dma_row_chunks(src, __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)dst));
      }
    }
  };
  // Step t reads K tile t+1 and V tile t-1.  At its start K(t+S) and V(t+S-2) are issued into the slots of K(t)
  // and V(t-2), whose last readers finished in step t-1.
  // In the gather variant the ids of tiles kt and kt-2 must already be visible in the ids ring.
  auto issue_tiles = [&](int kt) {
    issue_one(kt, p.Kc, p.Kn, k_ring, k_offc, k_offn, false);
    if (kt >= 2) issue_one(kt - 2, p.Vc, p.Vn, v_ring, v_offc, v_offn, true);
  };

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

  // Q^T fragments (B operand): lane (query c, half g) holds Q[q][16 kk + 8 g .. +8]
  bf16x8 qf[KD];
  {
    const int qi = q_row < p.Lq ? q_row : p.Lq - 1;
    const unsigned short* qp = p.Q + (long long)qi * p.ld_q + head_off + 8 * g;
#pragma unroll
    for (int kk = 0; kk < KD; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qp + 16 * kk);
  }

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
  float msc = -INFINITY, l_run = 0.f;
  const float sc = p.scale_log2;

  auto k_addr = [&](int tile) { return k_ring + (tile % kAtStages) * TILEB + k_off; };
  auto v_addr = [&](int tile) { return v_ring + (tile % kAtStages) * TILEB + v_off; };

  // ---- prologue: fill the ring (K tiles 0..S-1, V tiles 0..S-3), then S^T(0)
  if (GATHER) {  // ids of the tiles whose loads are issued before step kAtIdLead's ids arrive
#pragma unroll
    for (int u = 0; u < kAtStages + kAtIdLead; ++u) issue_ids(u);
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
  }
#pragma unroll
  for (int u = 0; u < kAtStages; ++u) issue_tiles(u);  // tiles past the end hold clamped rows, never read back
  wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();
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
  // Step 0 refills ring slot 0 (K(kAtStages) replaces K(0)): every wave must have its K(0) fragments in registers
  // before any wave issues that load.  The products above have consumed them, so one barrier here is enough; inside
  // the loop the barrier that ends step t-1 plays this role for step t.
  asm volatile("" : "+v"(s_a[0]), "+v"(s_a[1]));
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
  __builtin_amdgcn_s_barrier();

  // A wave whose 32 queries all lie past the end (the last query tile of a head is usually ragged) still loads its
  // share of every tile and joins every barrier, but does no arithmetic: on this chip energy is time.
  if (__builtin_amdgcn_readfirstlane(i_first + wave * 32) >= p.Lq) {
#pragma unroll 1
    for (int t = 0; t < 2 * n_iter; ++t) {
      if (GATHER) issue_ids(t + kAtStages + kAtIdLead);
      issue_tiles(t + kAtStages);
      wait_vmcnt<(kAtStages - 2) * (2 * LPT + (GATHER ? 1 : 0))>();
      __builtin_amdgcn_s_barrier();
    }
    wait_vmcnt<0>();
    return;
  }

  // Step t: S^T(t+1) into the "next" registers, softmax of S^T(t), O^T += tile t-1.  Iteration T runs step 2T
  // (s_a -> p_a, next into s_b, adds p_b) and step 2T+1 (s_b -> p_b, next into s_a, adds p_a).  The tile count is
  // padded to even: a tile past the end is fully masked and contributes nothing.  Before the first tile p_b is
  // zero, and when there is no next tile the S^T product re-reads the current one (its result is never used).
  // After each step: K(t+2) and V(t) must have landed before the next step; only the loads of the last two steps
  // may stay in flight.
#pragma unroll 1
  for (int T = 0; T < n_iter; ++T) {
    {
      const int t = 2 * T;
      if (GATHER) issue_ids(t + kAtStages + kAtIdLead);
      issue_tiles(t + kAtStages);
      if ((t + 1) * kAtTileKeys > lim_min) attn_mask(s_a, t * kAtTileKeys, lim, g);
      attn_step<D>(s_a, s_b, p_b, p_a, o, qf, msc, l_run, k_addr(t + 1), v_addr(t > 0 ? t - 1 : 0), kx2, vx2, sc);
      wait_vmcnt<(kAtStages - 2) * (2 * LPT + (GATHER ? 1 : 0))>();
      __builtin_amdgcn_s_barrier();
    }
    {
      const int t = 2 * T + 1;
      if (GATHER) issue_ids(t + kAtStages + kAtIdLead);
      issue_tiles(t + kAtStages);
      if ((t + 1) * kAtTileKeys > lim_min) attn_mask(s_b, t * kAtTileKeys, lim, g);
      attn_step<D>(s_b, s_a, p_a, p_b, o, qf, msc, l_run, k_addr(T + 1 < n_iter ? t + 1 : t), v_addr(t - 1), kx2, vx2, sc);
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
  wait_vmcnt<0>();  // nothing may still be writing this workgroup's LDS when it retires

  // normalise and store: lane holds query c, d = 32 b + 8 (r/4) + 4 g + (r%4)
  const float inv = 1.0f / half_swap_sum(l_run);
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

template <int D, bool OUT_F32, bool GATHER>
int launch_variant(hipStream_t st, dim3 grid, const AttnParams& p) {
  static LdsLimit lds_limit;
  const int rc = set_lds_limit(lds_limit, chunk_attention_kernel<D, OUT_F32, GATHER>, attn_lds_bytes(D, GATHER));
  if (rc != PAFU_OK) return rc;
  hipLaunchKernelGGL((chunk_attention_kernel<D, OUT_F32, GATHER>), grid, dim3(kAtThreads),
                     attn_lds_bytes(D, GATHER), st, p);
  return check_launch();
}

template <bool GATHER>
int launch_dims(hipStream_t st, dim3 grid, const AttnParams& p, int D, bool f32) {
  if (D == 128)
    return f32 ? launch_variant<128, true, GATHER>(st, grid, p) : launch_variant<128, false, GATHER>(st, grid, p);
  return f32 ? launch_variant<64, true, GATHER>(st, grid, p) : launch_variant<64, false, GATHER>(st, grid, p);
}

}  // namespace

int launch_attention(hipStream_t st, const void* Q, int Lq, const void* Kc, const void* Vc, int n_kept,
                     const void* Kn, const void* Vn, int Lc, int N, int D, long long ld_q, long long ld_c,
                     long long ld_n, long long ld_o, int block_len, float scale, void* O, int out_dtype,
                     const int* ids, int n_cache) {
  AttnParams p;
  p.ids = ids;
  p.n_cache = n_cache;
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
  const dim3 grid(((Lq + kAtBQ - 1) / kAtBQ) * N);
  const bool f32 = out_dtype == PAFU_F32;
  return ids != nullptr && n_kept > 0 ? launch_dims<true>(st, grid, p, D, f32) : launch_dims<false>(st, grid, p, D, f32);
}

}  // namespace pafu

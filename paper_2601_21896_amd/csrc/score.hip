// Salience Estimation Head (S-MLP) forward: s[t] = mean_o( W2 . act(W1 . x[t] + b1) + b2 ).
// App. A "S-MLP" and Sec. 3.3-3.4 of the paper (two linear layers, SiLU in between, mean over outputs).
//
// The mean over the outputs of a linear layer is a linear layer with the averaged weight row, so a
// tiny pre-kernel folds W2/b2 into one row w2bar[M] and a scalar (skipped when n_out == 1); the main
// kernel then fuses layer 1, the activation, the dot with w2bar and the bias into one pass over X.
//
// bf16 paths: layer 1 is a skinny dense contraction [M x F] . [F x T], so it runs on the matrix cores
// (v_mfma_f32_32x32x16_bf16, fp32 accumulate).  H = W1.X is produced as H^T tiles (rows = hidden units,
// columns = tokens), so one lane holds 16 hidden units of ONE token per tile and the reduction over hidden
// units is almost entirely in-register.
//  - score_stream_kernel (M a multiple of 256): the measured path.  W1 and the features both stream
//    global -> LDS through a ring of 64-feature slabs; a workgroup owns several 32-token tiles so that one W1
//    fragment feeds several matrix instructions.  Described in detail above the kernel.
//    In a rollout step one extra workgroup of this launch runs the top-k selection on the stored score list
//    (select_body.h), which does not depend on the chunk's scores (Alg. 2: Top-k before the chunk is appended).
//  - score_mfma_kernel (other M a multiple of 32): a wave owns 32 tokens and loads their feature rows straight
//    into B-operand registers; W1 is staged through LDS in 64-feature slabs shared by the waves of a workgroup.
//
// generic path (fp32 inputs, or shapes the tiles do not divide): plain fp32 FMAs.
#include "pafu_internal.h"
#include "select_body.h"

namespace pafu {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

__device__ __forceinline__ float bf16_bits_to_f32(unsigned short b) { return __uint_as_float((uint32_t)b << 16); }

__device__ __forceinline__ float act_accurate(float h, int act) {
  if (act == PAFU_ACT_SILU) return h / (1.0f + expf(-h));
  return 0.5f * h * (1.0f + erff(h * 0.70710678118654752440f));
}

// w2bar[m] = mean_o W2[o][m];  w2bar[M] = mean_o b2[o]
__global__ void fold_w2_kernel(const float* __restrict__ W2, const float* __restrict__ b2, int M, int n_out,
                               float* __restrict__ w2bar) {
  const int m = blockIdx.x * blockDim.x + threadIdx.x;
  const float inv = 1.0f / (float)n_out;
  if (m < M) {
    float s = 0.f;
    for (int o = 0; o < n_out; ++o) s += W2[(long long)o * M + m];
    w2bar[m] = s * inv;
  } else if (m == M) {
    float s = 0.f;
    if (b2 != nullptr)
      for (int o = 0; o < n_out; ++o) s += b2[o];
    w2bar[M] = s * inv;
  }
}

// ---------------------------------------------------------------------------------- generic path
template <bool BF16>
__device__ __forceinline__ float load_elem(const void* p, long long i) {
  if (BF16) return bf16_bits_to_f32(static_cast<const unsigned short*>(p)[i]);
  return static_cast<const float*>(p)[i];
}

// 256 threads = 16 tokens x 16 hidden-unit lanes.
template <bool BF16>
__global__ __launch_bounds__(256) void score_generic_kernel(const void* x0, const void* x1, const void* x2, int n_seg,
                                                            int T, int Fs, long long ld_x, const void* W1,
                                                            const float* b1, const float* w2bar, const float* b2bar,
                                                            int M, int act, float* out) {
  const int t = blockIdx.x * 16 + (threadIdx.x >> 4);
  const int ml = threadIdx.x & 15;
  const int tt = t < T ? t : T - 1;
  const long long F = (long long)n_seg * Fs;
  float partial = 0.f;
  for (int m = ml; m < M; m += 16) {
    float h = b1 ? b1[m] : 0.f;
    for (int s = 0; s < n_seg; ++s) {
      const void* xs = s == 0 ? x0 : (s == 1 ? x1 : x2);
      const long long xo = (long long)tt * ld_x;
      const long long wo = (long long)m * F + (long long)s * Fs;
      float h0 = 0.f, h1 = 0.f, h2 = 0.f, h3 = 0.f;
      int f = 0;
      for (; f + 3 < Fs; f += 4) {
        h0 = fmaf(load_elem<BF16>(W1, wo + f), load_elem<BF16>(xs, xo + f), h0);
        h1 = fmaf(load_elem<BF16>(W1, wo + f + 1), load_elem<BF16>(xs, xo + f + 1), h1);
        h2 = fmaf(load_elem<BF16>(W1, wo + f + 2), load_elem<BF16>(xs, xo + f + 2), h2);
        h3 = fmaf(load_elem<BF16>(W1, wo + f + 3), load_elem<BF16>(xs, xo + f + 3), h3);
      }
      for (; f < Fs; ++f) h0 = fmaf(load_elem<BF16>(W1, wo + f), load_elem<BF16>(xs, xo + f), h0);
      h += (h0 + h1) + (h2 + h3);
    }
    partial = fmaf(w2bar[m], act_accurate(h, act), partial);
  }
  partial += __shfl_xor(partial, 8);
  partial += __shfl_xor(partial, 4);
  partial += __shfl_xor(partial, 2);
  partial += __shfl_xor(partial, 1);
  if (ml == 0 && t < T) out[t] = partial + (b2bar ? *b2bar : 0.f);
}

// ---------------------------------------------------------------------------------- MFMA path
constexpr int kScThreads = 256;
constexpr int kScTokPerWave = 32;
constexpr int kScTokPerWg = 128;
constexpr int kScSlab = 64;                 // features per LDS slab
constexpr int kScRowBytes = kScSlab * 2 + 16;  // 144 B: padded so that 16 consecutive rows hit distinct banks
constexpr int sc_lds_bytes(int mb) { return 2 * mb * 32 * kScRowBytes; }

__device__ __forceinline__ float fast_silu(float h) {
  // h * sigmoid(h), sigmoid via exp2 and a reciprocal
  const float e = __builtin_amdgcn_exp2f(-1.44269504088896340736f * h);
  return h * __builtin_amdgcn_rcpf(1.0f + e);
}

// MB = 32-row hidden blocks per pass over X (MB*32 hidden units are accumulated at once).
template <int MB>
__global__ __launch_bounds__(kScThreads, 2) void score_mfma_kernel(const unsigned short* __restrict__ x0,
                                                                   const unsigned short* __restrict__ x1,
                                                                   const unsigned short* __restrict__ x2, int T,
                                                                   int Fs, int F, long long ld_x,
                                                                   const unsigned short* __restrict__ W1,
                                                                   const float* __restrict__ b1,
                                                                   const float* __restrict__ w2bar,
                                                                   const float* __restrict__ b2bar, int M, int act,
                                                                   float* __restrict__ out) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, c = lane & 31;
  const int tok = blockIdx.x * kScTokPerWg + wave * kScTokPerWave + c;
  const int tokc = tok < T ? tok : T - 1;
  const int n_slabs = F / kScSlab;
  const int slabs_per_seg = Fs / kScSlab;
  // this thread's part of a W1 slab: rows (i*32 + tid/8), 16-byte chunk tid%8
  const int w_row = tid >> 3, w_chunk = tid & 7;

  float partial = 0.f;
  constexpr int kScMBlocks = MB;
  constexpr int kScBufBytes = MB * 32 * kScRowBytes;
#pragma unroll 1
  for (int mp = 0; mp < M; mp += kScMBlocks * 32) {
    f32x16 acc[kScMBlocks];
#pragma unroll
    for (int b = 0; b < kScMBlocks; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[b][r] = 0.f;

    u32x4 wreg[kScMBlocks];
    bf16x8 xreg[4];
    const unsigned short* wbase = W1 + (long long)(mp + w_row) * F + w_chunk * 8;
#define PAFU_LOAD_SLAB(S)                                                                          \
  do {                                                                                             \
    const unsigned short* wsrc = wbase + (long long)(S) * kScSlab;                                 \
    _Pragma("unroll") for (int i = 0; i < kScMBlocks; ++i)                                         \
        wreg[i] = *reinterpret_cast<const u32x4*>(wsrc + (long long)i * 32 * F);                   \
    const int seg = (S) / slabs_per_seg;                                                           \
    const int fo = ((S) - seg * slabs_per_seg) * kScSlab;                                          \
    const unsigned short* xs = seg == 0 ? x0 : (seg == 1 ? x1 : x2);                               \
    const unsigned short* xsrc = xs + (long long)tokc * ld_x + fo + 8 * g;                         \
    _Pragma("unroll") for (int kk = 0; kk < 4; ++kk)                                               \
        xreg[kk] = *reinterpret_cast<const bf16x8*>(xsrc + kk * 16);                               \
  } while (0)
#define PAFU_STORE_SLAB(BUF)                                                                       \
  do {                                                                                             \
    unsigned char* dst = lds + (BUF) * kScBufBytes + w_row * kScRowBytes + w_chunk * 16;           \
    _Pragma("unroll") for (int i = 0; i < kScMBlocks; ++i)                                         \
        *reinterpret_cast<u32x4*>(dst + i * 32 * kScRowBytes) = wreg[i];                           \
  } while (0)

    PAFU_LOAD_SLAB(0);
    __syncthreads();  // every wave is done with the LDS contents of the previous pass
    PAFU_STORE_SLAB(0);
    __syncthreads();
#pragma unroll 1
    for (int s = 0; s < n_slabs; ++s) {
      bf16x8 xcur[4];
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) xcur[kk] = xreg[kk];
      if (s + 1 < n_slabs) PAFU_LOAD_SLAB(s + 1);
      const unsigned char* buf = lds + (s & 1) * kScBufBytes + c * kScRowBytes + g * 16;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
        for (int b = 0; b < kScMBlocks; ++b) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(buf + b * 32 * kScRowBytes + kk * 32);
          acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, xcur[kk], acc[b], 0, 0, 0);
        }
      }
      if (s + 1 < n_slabs) PAFU_STORE_SLAB((s + 1) & 1);
      __syncthreads();
    }
    // activation and second layer for this pass's hidden units; lane holds token c, units
    // mp + 32 b + 8 (r/4) + 4 g + (r%4)
#pragma unroll
    for (int b = 0; b < kScMBlocks; ++b) {
      {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int m0 = mp + 32 * b + 8 * q + 4 * g;
          const float4 w = *reinterpret_cast<const float4*>(w2bar + m0);
          float4 bb = make_float4(0.f, 0.f, 0.f, 0.f);
          if (b1 != nullptr) bb = *reinterpret_cast<const float4*>(b1 + m0);
          const float h0 = acc[b][4 * q + 0] + bb.x, h1 = acc[b][4 * q + 1] + bb.y;
          const float h2 = acc[b][4 * q + 2] + bb.z, h3 = acc[b][4 * q + 3] + bb.w;
          if (act == PAFU_ACT_SILU) {
            partial = fmaf(w.x, fast_silu(h0), partial);
            partial = fmaf(w.y, fast_silu(h1), partial);
            partial = fmaf(w.z, fast_silu(h2), partial);
            partial = fmaf(w.w, fast_silu(h3), partial);
          } else {
            partial = fmaf(w.x, act_accurate(h0, act), partial);
            partial = fmaf(w.y, act_accurate(h1, act), partial);
            partial = fmaf(w.z, act_accurate(h2, act), partial);
            partial = fmaf(w.w, act_accurate(h3, act), partial);
          }
        }
      }
    }
  }
#undef PAFU_LOAD_SLAB
#undef PAFU_STORE_SLAB
  partial += __shfl_xor(partial, 32);
  if (g == 0 && tok < T) out[tok] = partial + (b2bar ? *b2bar : 0.f);
}

// ---------------------------------------------------------------------------------- streaming MFMA path
// For M % 256 == 0 and Fs % 64 == 0.  With a 256-wide hidden layer the head sits near the ridge of the roofline
// (about 256 flop per byte of features), and every CU has to pull all of W1 through its L1 once per token group, so
// the kernel must keep the matrix cores and the memory pipe busy at the same time: an even spread of MFMA work over
// the 1024 SIMDs, few LDS bytes per MFMA, and many bytes in flight without spending registers on them.
//  - A workgroup owns TT 32-token tiles (TT picked at launch so that the grid needs as few rounds over the 256 CUs
//    as possible) and one 256-unit pass of the hidden layer at a time.  Its 8 waves split the hidden units four
//    ways and the reduction axis two ways: wave (hq, kh) accumulates hidden units [64 hq, 64 hq + 64) for all TT
//    tiles over half of the k-steps of every slab, so one W1 fragment feeds TT MFMAs and one feature fragment two.
//    The two reduction halves sit on the same SIMD (waves w and w + 4) and are added through LDS at the end of a pass.
//  - W1 and the features stream global -> LDS with global_load_lds through a ring of slabs (no staging registers,
//    all but one slab of the ring in flight), rows XOR-swizzled in 16-byte chunks for conflict-free b128 reads.
constexpr int kS3Slab = 64;                      // features per slab (full 128-byte lines per row)
constexpr int kS3RowB = kS3Slab * 2;             // bytes per slab row
constexpr int kS3Chunks = kS3RowB / 16;          // 16-byte chunks per row
constexpr int kS3RowsPerLoad = 1024 / kS3RowB;   // rows covered by one wave-wide 16-byte-per-lane load
constexpr int kS3Stages = 3;                     // ring depth: 3 x (32 KB + 4 TT KB) <= 156 KB
constexpr int kS3WBytes = 256 * kS3RowB;         // W1 part of a stage (256 hidden units)
constexpr int kS3MaxTT = 5;
constexpr int kS3RedBytes = 65536;               // two 32 KB regions for the end-of-pass reduction
constexpr int s3_stage_bytes(int TT) { return kS3WBytes + 32 * TT * kS3RowB; }
constexpr int s3_lds_bytes(int TT) {
  return kS3Stages * s3_stage_bytes(TT) > kS3RedBytes ? kS3Stages * s3_stage_bytes(TT) : kS3RedBytes;
}
// chunk q of row r lives in slot q ^ swz(r): 16 consecutive rows of one chunk then cover all 64 banks
__device__ __forceinline__ int s3_swz(int row) {
  return kS3RowB == 64 ? (row >> 2) & 3 : (row >> 1) & 7;
}

// 64 x 16 bytes global -> LDS: lane l's bytes at (uniform base + its byte offset) land at lds_addr + 16 l
__device__ __forceinline__ void s3_dma(const void* base_uniform, unsigned byte_off, unsigned lds_addr_uniform) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_addr_uniform), "v"(byte_off), "s"(base_uniform)
               : "memory");
}
template <int N>
__device__ __forceinline__ void s3_wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// SELW > 0: workgroup 0 of the launch does not score but runs a top-k selection (SELW key words per thread, 512
// threads) on a list that does not depend on this launch's scores: the stored score list of a rollout step.  A
// selection keeps one CU busy for about as long as the scoring of a chunk takes the others, so carried along it
// costs nothing, where a launch of its own would leave the rest of the chip idle meanwhile.
template <int TT, int SELW>
__global__ __launch_bounds__(512, 1) void score_stream_kernel(
    const unsigned short* __restrict__ x0, const unsigned short* __restrict__ x1, const unsigned short* __restrict__ x2,
    int T, int Fs, int F, long long ld_x, const unsigned short* __restrict__ W1, const float* __restrict__ b1,
    const float* __restrict__ w2bar, const float* __restrict__ b2bar, int M, int act, float* __restrict__ out,
    SelectJob ride) {
  if constexpr (SELW > 0) {
    if (blockIdx.x == 0) {
      select_bitslice_body<SELW, 512>(ride);
      return;
    }
  }
  constexpr int kStageB = s3_stage_bytes(TT);
  constexpr int WU = 256 / kS3RowsPerLoad;             // wave-wide loads that fill the W1 part of a stage
  constexpr int XU = 32 * TT / kS3RowsPerLoad;         // ... and the feature part
  constexpr int LW = WU / 8;                           // W1 loads per wave per slab
  constexpr int LX = (XU + 7) / 8;                     // feature loads per wave per slab
  constexpr int LPW = LW + LX;
  constexpr int KS = kS3Slab / 32;                     // k-steps (16 features) per wave per slab
  static_assert(KS % 2 == 0, "the two fragment sets alternate per k-step and must line up across slabs");
  typedef __attribute__((address_space(3))) unsigned char lds_byte;
  typedef __attribute__((address_space(3))) bf16x8 lds_frag;
  typedef float f32x4_t __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) f32x4_t lds_f4;
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds_raw[];
  lds_byte* const ring = (lds_byte*)lds_raw;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // said to be uniform: LDS addresses of the loads stay scalar
  const int hq = wave & 3, kh = wave >> 2;
  const int g = lane >> 5, c = lane & 31;
  const int tok_base = (blockIdx.x - (SELW > 0 ? 1 : 0)) * (32 * TT);
  const int n_slabs = F / kS3Slab;
  const int slabs_per_seg = Fs / kS3Slab;

  // ---- loads.  One wave-wide load covers kS3RowsPerLoad slab rows: lane -> (row, LDS slot); the slot receives chunk
  // slot ^ swz(row) of the row.  Addresses are a uniform base plus a 32-bit per-lane byte offset.  Surplus feature
  // loads repeat a unit (same bytes, same place) so that every wave issues the same number of loads.
  const int d_row = lane / kS3Chunks, d_slot = lane % kS3Chunks;
  unsigned w_off[LW], x_off[LX];
#pragma unroll
  for (int j = 0; j < LW; ++j) {
    const int row = (wave + 8 * j) * kS3RowsPerLoad + d_row;
    w_off[j] = (unsigned)((row * F + (d_slot ^ s3_swz(row)) * 8) * 2);
  }
#pragma unroll
  for (int j = 0; j < LX; ++j) {
    const int row = ((wave + 8 * j) % XU) * kS3RowsPerLoad + d_row;
    const int rel = tok_base + row < T ? row : T - 1 - tok_base;
    x_off[j] = (unsigned)(rel * ld_x * 2) + (d_slot ^ s3_swz(row)) * 16;
  }
  const long long x_wg_off = (long long)tok_base * ld_x;
  // ---- fragment reads inside a stage: k-step ks = KS kh + j of the slab, lane half g -> chunk 2 ks + g.
  // swz(row) only depends on c for the rows a lane reads (row = 32-row block + c).
  int rd[KS];
#pragma unroll
  for (int j = 0; j < KS; ++j) rd[j] = c * kS3RowB + (((2 * (KS * kh + j) + g) ^ s3_swz(c)) << 4);

  float partial[TT];
#pragma unroll
  for (int tt = 0; tt < TT; ++tt) partial[tt] = 0.f;

#pragma unroll 1
  for (int mp = 0; mp < M; mp += 256) {
    f32x16 acc[TT][2];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[tt][b][r] = 0.f;
    const unsigned short* const w_pass = W1 + (long long)mp * F;  // uniform

    // slab S -> stage S % kS3Stages (slabs past the end re-read the last one; they are never consumed)
#define PAFU_S3_ISSUE(S)                                                                                        \
  do {                                                                                                          \
    const int s_ = (S);                                                                                         \
    const int sc_ = s_ < n_slabs ? s_ : n_slabs - 1;                                                            \
    lds_byte* st_ = ring + (s_ % kS3Stages) * kStageB;                                                          \
    _Pragma("unroll") for (int j = 0; j < LW; ++j)                                                              \
        s3_dma(w_pass + sc_ * kS3Slab, w_off[j],                                                                \
               (unsigned)(uintptr_t)(st_ + (wave + 8 * j) * 1024));                                             \
    const int seg_ = sc_ / slabs_per_seg;                                                                       \
    const int fo_ = (sc_ - seg_ * slabs_per_seg) * kS3Slab;                                                     \
    const unsigned short* xs_ = seg_ == 0 ? x0 : (seg_ == 1 ? x1 : x2);                                         \
    _Pragma("unroll") for (int j = 0; j < LX; ++j)                                                              \
        s3_dma(xs_ + x_wg_off + fo_, x_off[j],                                                                  \
               (unsigned)(uintptr_t)(st_ + kS3WBytes + ((wave + 8 * j) % XU) * 1024));                          \
  } while (0)

    // Fragments of k-step j of a slab: two W1 blocks and TT feature tiles, into fragment set B (0 or 1).
#define PAFU_S3_READ(B, ST, J)                                                                                  \
  do {                                                                                                          \
    fw[B][0] = *(const lds_frag*)((ST) + (hq * 64) * kS3RowB + rd[J]);                                          \
    fw[B][1] = *(const lds_frag*)((ST) + (hq * 64 + 32) * kS3RowB + rd[J]);                                     \
    _Pragma("unroll") for (int tt = 0; tt < TT; ++tt)                                                           \
        fx[B][tt] = *(const lds_frag*)((ST) + kS3WBytes + tt * 32 * kS3RowB + rd[J]);                           \
  } while (0)
#define PAFU_S3_MMA(B)                                                                                          \
  do {                                                                                                          \
    _Pragma("unroll") for (int tt = 0; tt < TT; ++tt) {                                                         \
      acc[tt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[B][0], fx[B][tt], acc[tt][0], 0, 0, 0);           \
      acc[tt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[B][1], fx[B][tt], acc[tt][1], 0, 0, 0);           \
    }                                                                                                           \
  } while (0)

    // Software pipeline.  The fragments of the next k-step are read while the matrix instructions of the current one
    // run, also across slabs: the barrier sits before the LAST k-step of slab s, where every wave has its last
    // fragments of slab s in registers (so the slab's stage can be refilled) and where slab s+1 must have landed (so
    // its first fragments can be fetched under the last k-step of slab s).  Ring: stage of slab s being refilled
    // with slab s+3, slab s+1 ready, slab s+2 in flight.
    bf16x8 fw[2][2], fx[2][TT];
    const bool kh_first = kh == 0;
    __syncthreads();  // every wave is done with the LDS contents of the previous pass
#pragma unroll
    for (int s = 0; s < kS3Stages; ++s) PAFU_S3_ISSUE(s);
    s3_wait_vmcnt<(kS3Stages - 1) * LPW>();
    __builtin_amdgcn_s_barrier();  // slab 0 visible to all
    PAFU_S3_READ(0, ring, 0);
#pragma unroll 1
    for (int s = 0; s < n_slabs; ++s) {
      const lds_byte* st = ring + (s % kS3Stages) * kStageB;
      const lds_byte* st_next = ring + ((s + 1) % kS3Stages) * kStageB;
#pragma unroll
      for (int j = 0; j < KS; ++j) {
        if (j + 1 < KS) {
          PAFU_S3_READ((j + 1) & 1, st, j + 1);
        } else {
          // own fragment reads of slab s complete (they must be before the stage is handed back), then the loads
          // of slab s+1 (issued two barriers ago; only the slab after it may still be in flight)
          __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0), other counters left alone
          s3_wait_vmcnt<(kS3Stages - 2) * LPW>();
          __builtin_amdgcn_s_barrier();
          // refill the stage of slab s.  A wave cannot issue anything else while its loads queue up behind a busy
          // memory pipe, so the two waves of a SIMD (kh = 0, 1) take turns: one issues its loads before this
          // k-step's matrix instructions, the other after them.
          if (kh_first) PAFU_S3_ISSUE(s + kS3Stages);
          PAFU_S3_READ((j + 1) & 1, st_next, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        PAFU_S3_MMA(j & 1);
        __builtin_amdgcn_sched_barrier(0);
        if (j + 1 == KS && !kh_first) PAFU_S3_ISSUE(s + kS3Stages);
      }
    }
#undef PAFU_S3_READ
#undef PAFU_S3_MMA
#undef PAFU_S3_ISSUE
    // ---- add the two halves of the reduction axis through LDS, one token tile at a time, alternating between two
    // 32 KB regions so that one barrier per tile is enough.  The two waves (hq, 0) and (hq, 1) swap one 32-unit block
    // each: wave kh ends up with the complete sums of block b = kh and applies bias, activation and second layer
    // to it, so that both waves of a SIMD share that work.
    s3_wait_vmcnt<0>();
    __syncthreads();  // all loads have landed and all fragment reads are done: the ring can be reused
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
      lds_f4* reg = (lds_f4*)(ring + (tt & 1) * 32768) + (hq * 2 + kh) * 4 * 64 + lane;       // what this wave sends
      const lds_f4* got = (const lds_f4*)(ring + (tt & 1) * 32768) + (hq * 2 + (kh ^ 1)) * 4 * 64 + lane;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (kh == 0) reg[q * 64] = f32x4_t{acc[tt][1][4 * q], acc[tt][1][4 * q + 1], acc[tt][1][4 * q + 2], acc[tt][1][4 * q + 3]};
        else reg[q * 64] = f32x4_t{acc[tt][0][4 * q], acc[tt][0][4 * q + 1], acc[tt][0][4 * q + 2], acc[tt][0][4 * q + 3]};
      }
      __syncthreads();
      // the lane holds token c of tile tt and hidden units mp + 64 hq + 32 kh + 8 q + 4 g + e
      float hsum[16];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const f32x4_t o = got[q * 64];
        const int m0 = mp + 64 * hq + 32 * kh + 8 * q + 4 * g;
        float4 bb = make_float4(0.f, 0.f, 0.f, 0.f);
        if (b1 != nullptr) bb = *reinterpret_cast<const float4*>(b1 + m0);
        const float ov[4] = {o.x, o.y, o.z, o.w}, bv[4] = {bb.x, bb.y, bb.z, bb.w};
#pragma unroll
        for (int e = 0; e < 4; ++e)
          hsum[4 * q + e] = (kh == 0 ? acc[tt][0][4 * q + e] : acc[tt][1][4 * q + e]) + ov[e] + bv[e];
      }
      if (act == PAFU_ACT_SILU) {
#pragma unroll
        for (int i = 0; i < 16; ++i) hsum[i] = fast_silu(hsum[i]);
      } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) hsum[i] = act_accurate(hsum[i], act);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 w = *reinterpret_cast<const float4*>(w2bar + mp + 64 * hq + 32 * kh + 8 * q + 4 * g);
        partial[tt] = fmaf(w.x, hsum[4 * q], partial[tt]);
        partial[tt] = fmaf(w.y, hsum[4 * q + 1], partial[tt]);
        partial[tt] = fmaf(w.z, hsum[4 * q + 2], partial[tt]);
        partial[tt] = fmaf(w.w, hsum[4 * q + 3], partial[tt]);
      }
    }
  }
  // ---- add the two lane halves, then the eight waves (each holds the part of its 32-unit blocks)
  __syncthreads();
  float* red = reinterpret_cast<float*>(lds_raw);
#pragma unroll
  for (int tt = 0; tt < TT; ++tt) {
    partial[tt] += __shfl_xor(partial[tt], 32);
    if (g == 0) red[wave * (32 * TT) + tt * 32 + c] = partial[tt];
  }
  __syncthreads();
  for (int i = tid; i < 32 * TT; i += 512) {
    const int tok = tok_base + i;
    if (tok < T) {
      float v = b2bar ? *b2bar : 0.f;
#pragma unroll
      for (int w = 0; w < 8; ++w) v += red[w * (32 * TT) + i];
      out[tok] = v;
    }
  }
}

// Scratch of pafu_score_static: the output-averaged second layer (M weights + 1 bias) that pafu_score keeps in its
// caller-provided workspace.  One copy per GPU, held until the process ends; every call on a GPU shares it.
static __device__ __align__(256) float scratch[PAFU_SCORE_STATIC_MAX_M + 1];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each GPU (the array's name is only a
                                         // host-side handle: kernels are given these addresses)

// Device address of `scratch` on the current GPU, looked up once per device.
int score_scratch(float** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return record_hip_error(e);
  if (dev < 0 || dev >= kMaxDevices) return PAFU_ERR_SHAPE;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return record_hip_error(e);
    if (ptr == nullptr) return record_hip_error(hipErrorInvalidSymbol);
    g_scratch_ptr[dev] = static_cast<float*>(ptr);
  }
  *out = g_scratch_ptr[dev];
  return PAFU_OK;
}

}  // namespace

int launch_score_static(hipStream_t st, const void* x0, const void* x1, const void* x2, int n_seg, int T, int Fs,
                        long long ld_x, int x_dtype, const void* W1, const float* b1, const float* W2,
                        const float* b2, int M, int n_out, int act, float* out) {
  if (M > PAFU_SCORE_STATIC_MAX_M) return PAFU_ERR_WORKSPACE;
  float* ws = nullptr;
  const int rc = score_scratch(&ws);
  if (rc != PAFU_OK) return rc;
  return launch_score(st, x0, x1, x2, n_seg, T, Fs, ld_x, x_dtype, W1, b1, W2, b2, M, n_out, act, out, ws);
}

int launch_score(hipStream_t st, const void* x0, const void* x1, const void* x2, int n_seg, int T, int Fs,
                 long long ld_x, int x_dtype, const void* W1, const float* b1, const float* W2, const float* b2, int M,
                 int n_out, int act, float* out, void* ws, const SelectJob* ride, bool* rode) {
  if (rode != nullptr) *rode = false;
  if (T <= 0) return PAFU_OK;
  const float* w2bar = W2;
  const float* b2bar = b2;
  if (n_out > 1) {
    float* w = static_cast<float*>(ws);
    hipLaunchKernelGGL(fold_w2_kernel, dim3((M + 1 + 255) / 256), dim3(256), 0, st, W2, b2, M, n_out, w);
    int rc = check_launch();
    if (rc != PAFU_OK) return rc;
    w2bar = w;
    b2bar = w + M;
  }
  const int F = n_seg * Fs;
  const bool mfma = x_dtype == PAFU_BF16 && Fs % kScSlab == 0 && M % 32 == 0 && ld_x % 8 == 0;
  if (mfma) {
    const int grid = (T + kScTokPerWg - 1) / kScTokPerWg;
    const int blocks = M / 32;
#define PAFU_SCORE_CASE(MB)                                                                                          \
  do {                                                                                                               \
    static LdsLimit lds_limit;                                                                                       \
    const int rc_ = set_lds_limit(lds_limit, score_mfma_kernel<MB>, sc_lds_bytes(MB));                               \
    if (rc_ != PAFU_OK) return rc_;                                                                                  \
    hipLaunchKernelGGL(score_mfma_kernel<MB>, dim3(grid), dim3(kScThreads), sc_lds_bytes(MB), st,                    \
                       static_cast<const unsigned short*>(x0), static_cast<const unsigned short*>(x1),               \
                       static_cast<const unsigned short*>(x2), T, Fs, F, ld_x, static_cast<const unsigned short*>(W1), \
                       b1, w2bar, b2bar, M, act, out);                                                               \
  } while (0)
    // the streaming kernel addresses rows by 32-bit byte offsets from a per-workgroup base
    const bool offsets_fit = 32ll * kS3MaxTT * ld_x * 2 < (1ll << 31) && 256ll * F * 2 < (1ll << 31);
    if (blocks % 8 == 0 && Fs % 64 == 0 && offsets_fit) {
      // streaming kernel: TT 32-token tiles per workgroup.  Per 32 features a SIMD spends about 128 TT cycles in
      // MFMAs and the CU about 64 (TT + 2) cycles serving fragment reads; each slab adds a fixed cost for the barrier
      // and the exposed first reads.  Pick the TT that minimises that times the number of rounds the grid needs
      // over the 256 CUs (ties go to the larger TT).
      const int tiles = (T + 31) / 32;
      int best_tt = 1;
      long long best_cost = 1ll << 60;
      for (int tt = 1; tt <= kS3MaxTT; ++tt) {
        const int wgs = (tiles + tt - 1) / tt;
        const int mfma = 128 * tt, lds = 64 * (tt + 2);
        const long long cost = (long long)((wgs + 255) / 256) * ((kS3Slab / 32) * (mfma > lds ? mfma : lds) + 100);
        if (cost <= best_cost) { best_cost = cost; best_tt = tt; }
      }
#define PAFU_SCORE3_LAUNCH(TT, SELW, LDS, EXTRA)                                                                     \
  do {                                                                                                               \
    static LdsLimit lds_limit3;                                                                                      \
    const int rc_ = set_lds_limit(lds_limit3, score_stream_kernel<TT, SELW>, LDS);                                   \
    if (rc_ != PAFU_OK) return rc_;                                                                                  \
    hipLaunchKernelGGL((score_stream_kernel<TT, SELW>), dim3((tiles + TT - 1) / TT + EXTRA), dim3(512), LDS, st,     \
                       static_cast<const unsigned short*>(x0), static_cast<const unsigned short*>(x1),               \
                       static_cast<const unsigned short*>(x2), T, Fs, F, ld_x, static_cast<const unsigned short*>(W1), \
                       b1, w2bar, b2bar, M, act, out, job);                                                          \
  } while (0)
#define PAFU_SCORE3_CASE(TT) PAFU_SCORE3_LAUNCH(TT, 0, s3_lds_bytes(TT), 0)
#define PAFU_SCORE3_RIDE(TT, SELW)                                                                                   \
  PAFU_SCORE3_LAUNCH(TT, SELW,                                                                                       \
                     (s3_lds_bytes(TT) > select_bitslice_lds_bytes(512) ? s3_lds_bytes(TT) : select_bitslice_lds_bytes(512)), 1)
      SelectJob job{nullptr, nullptr, nullptr, 0, 0, 0};
      // a selection rides along when the launch is short (one or two token tiles per workgroup: a chunk, not a whole
      // cache) and the list fits the 512-thread bit-sliced selection
      if (ride != nullptr && best_tt <= 2 && ride->n > 0 && ride->n <= 512 * 32 * 4) {
        job = *ride;
        if (job.n_pinned < 0) job.n_pinned = 0;
        const bool w2 = job.n <= 512 * 32 * 2;
        if (best_tt == 1) { if (w2) PAFU_SCORE3_RIDE(1, 2); else PAFU_SCORE3_RIDE(1, 4); }
        else { if (w2) PAFU_SCORE3_RIDE(2, 2); else PAFU_SCORE3_RIDE(2, 4); }
        if (rode != nullptr) *rode = true;
        return check_launch();
      }
      switch (best_tt) {
        case 1: PAFU_SCORE3_CASE(1); break;
        case 2: PAFU_SCORE3_CASE(2); break;
        case 3: PAFU_SCORE3_CASE(3); break;
        case 4: PAFU_SCORE3_CASE(4); break;
        default: PAFU_SCORE3_CASE(5); break;
      }
#undef PAFU_SCORE3_CASE
#undef PAFU_SCORE3_RIDE
#undef PAFU_SCORE3_LAUNCH
    } else if (blocks % 8 == 0) PAFU_SCORE_CASE(8);
    else if (blocks % 4 == 0) PAFU_SCORE_CASE(4);
    else if (blocks % 2 == 0) PAFU_SCORE_CASE(2);
    else PAFU_SCORE_CASE(1);
#undef PAFU_SCORE_CASE
  } else {
    const int grid = (T + 15) / 16;
    if (x_dtype == PAFU_BF16)
      hipLaunchKernelGGL(score_generic_kernel<true>, dim3(grid), dim3(256), 0, st, x0, x1, x2, n_seg, T, Fs, ld_x, W1,
                         b1, w2bar, b2bar, M, act, out);
    else
      hipLaunchKernelGGL(score_generic_kernel<false>, dim3(grid), dim3(256), 0, st, x0, x1, x2, n_seg, T, Fs, ld_x, W1,
                         b1, w2bar, b2bar, M, act, out);
  }
  return check_launch();
}

}  // namespace pafu

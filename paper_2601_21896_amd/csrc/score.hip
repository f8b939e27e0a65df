// Salience Estimation Head (S-MLP) forward: s[t] = mean_o( W2 . act(W1 . x[t] + b1) + b2 ).
// App. A "S-MLP" and Sec. 3.3-3.4 of the paper (two linear layers, SiLU in between, mean over outputs).
//
// The mean over the outputs of a linear layer is a linear layer with the averaged weight row, so a
// tiny pre-kernel folds W2/b2 into one row w2bar[M] and a scalar (skipped when n_out == 1); the main
// kernel then fuses layer 1, the activation, the dot with w2bar and the bias into one pass over X.
//
// bf16 path: layer 1 is a skinny dense contraction [M x F] . [F x T], so it runs on the matrix cores
// (v_mfma_f32_32x32x16_bf16, fp32 accumulate).  Each wave owns 32 tokens and streams their feature
// rows straight from HBM into MFMA B-operand registers (16 contiguous bytes per lane, read once);
// W1 is staged through LDS in 64-feature slabs shared by the four waves of a workgroup.  H = W1.X is
// produced as H^T tiles (rows = hidden units, columns = tokens), so one lane holds 16 hidden units of
// ONE token per tile and the reduction over hidden units is almost entirely in-register.
//
// generic path (fp32 inputs, or shapes the tiles do not divide): plain fp32 FMAs.
#include "pafu_internal.h"

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

}  // namespace

int launch_score(hipStream_t st, const void* x0, const void* x1, const void* x2, int n_seg, int T, int Fs,
                 long long ld_x, int x_dtype, const void* W1, const float* b1, const float* W2, const float* b2, int M,
                 int n_out, int act, float* out, void* ws) {
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
    static bool attr_set = false;                                                                                    \
    if (!attr_set) {                                                                                                 \
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(score_mfma_kernel<MB>),                       \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, sc_lds_bytes(MB));              \
      if (e != hipSuccess) return record_hip_error(e);                                                               \
      attr_set = true;                                                                                               \
    }                                                                                                                \
    hipLaunchKernelGGL(score_mfma_kernel<MB>, dim3(grid), dim3(kScThreads), sc_lds_bytes(MB), st,                    \
                       static_cast<const unsigned short*>(x0), static_cast<const unsigned short*>(x1),               \
                       static_cast<const unsigned short*>(x2), T, Fs, F, ld_x, static_cast<const unsigned short*>(W1), \
                       b1, w2bar, b2bar, M, act, out);                                                               \
  } while (0)
    if (blocks % 8 == 0) PAFU_SCORE_CASE(8);
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

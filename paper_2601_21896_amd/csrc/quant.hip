// 8-bit storage of the K/V cache: bf16 rows <-> E4M3 codes with one power-of-two scale per tensor.
// (Beyond the paper, which states no storage precision: App. A.)  E4M3 = 1 sign, 4 exponent bits with bias 7,
// 3 mantissa bits, no infinities, S.1111.111 = NaN; round to nearest even; magnitudes beyond 448 saturate.
//
// Quantisation is written out in integer arithmetic so that every code is a defined function of the input bits
// (the cache must match a reference bit for bit); the way back uses the hardware's 8-bit -> bf16 conversion, which is
// exact for every code and scale.
#include "pafu_internal.h"
#include "quant_body.h"

namespace pafu {
namespace {

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

// One thread = 8 elements (16 bytes in, 8 bytes out) of K and of V.
__global__ __launch_bounds__(256) void quantize_rows_kernel(const char* __restrict__ K, const char* __restrict__ V,
                                                            long long ld_in, int rows, int chunks, float inv_k,
                                                            float inv_v, char* __restrict__ Kq, char* __restrict__ Vq,
                                                            long long ld_out) {
  const long long total = (long long)rows * chunks;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
    const int r = (int)(i / chunks), c = (int)(i - (long long)r * chunks);
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const char* src = (t ? V : K) + (long long)r * ld_in + c * 16;
      char* dst = (t ? Vq : Kq) + (long long)r * ld_out + c * 8;
      const float inv = t ? inv_v : inv_k;
      const u32x4 w = *reinterpret_cast<const u32x4*>(src);
      const unsigned in[4] = {w[0], w[1], w[2], w[3]};
      unsigned codes[2];
      e4m3_codes8(in, inv, codes);
      u32x2 o;
      o[0] = codes[0];
      o[1] = codes[1];
      *reinterpret_cast<u32x2*>(dst) = o;
    }
  }
}

__global__ __launch_bounds__(256) void dequantize_rows_kernel(const char* __restrict__ Kq, const char* __restrict__ Vq,
                                                              long long ld_in, int rows, int chunks, float k_scale,
                                                              float v_scale, char* __restrict__ K, char* __restrict__ V,
                                                              long long ld_out) {
  const long long total = (long long)rows * chunks;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
    const int r = (int)(i / chunks), c = (int)(i - (long long)r * chunks);
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const char* src = (t ? Vq : Kq) + (long long)r * ld_in + c * 8;
      char* dst = (t ? V : K) + (long long)r * ld_out + c * 16;
      const float scl = t ? v_scale : k_scale;
      const u32x2 w = *reinterpret_cast<const u32x2*>(src);
      u32x4 o;
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        o[2 * e] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[e], scl, false));
        o[2 * e + 1] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[e], scl, true));
      }
      *reinterpret_cast<u32x4*>(dst) = o;
    }
  }
}

int grid_for(long long items) {
  long long blocks = (items + 255) / 256;
  if (blocks > 256 * 16) blocks = 256 * 16;
  return blocks < 1 ? 1 : (int)blocks;
}

}  // namespace

int launch_quantize(hipStream_t st, const void* K, const void* V, long long ld_in_bytes, int rows, int row_elems,
                    int k_scale_log2, int v_scale_log2, void* Kq, void* Vq, long long ld_out_bytes) {
  if (rows <= 0) return PAFU_OK;
  const int chunks = row_elems / 8;
  hipLaunchKernelGGL(quantize_rows_kernel, dim3(grid_for((long long)rows * chunks)), dim3(256), 0, st,
                     static_cast<const char*>(K), static_cast<const char*>(V), ld_in_bytes, rows, chunks,
                     ldexpf(1.0f, -k_scale_log2), ldexpf(1.0f, -v_scale_log2), static_cast<char*>(Kq),
                     static_cast<char*>(Vq), ld_out_bytes);
  return check_launch();
}

int launch_dequantize(hipStream_t st, const void* Kq, const void* Vq, long long ld_in_bytes, int rows, int row_elems,
                      int k_scale_log2, int v_scale_log2, void* K, void* V, long long ld_out_bytes) {
  if (rows <= 0) return PAFU_OK;
  const int chunks = row_elems / 8;
  hipLaunchKernelGGL(dequantize_rows_kernel, dim3(grid_for((long long)rows * chunks)), dim3(256), 0, st,
                     static_cast<const char*>(Kq), static_cast<const char*>(Vq), ld_in_bytes, rows, chunks,
                     ldexpf(1.0f, k_scale_log2), ldexpf(1.0f, v_scale_log2), static_cast<char*>(K),
                     static_cast<char*>(V), ld_out_bytes);
  return check_launch();
}

}  // namespace pafu

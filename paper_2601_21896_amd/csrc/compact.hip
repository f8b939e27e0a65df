// Cache update: gather of the retained K/V rows (and their scores) into a contiguous cache.
// Alg. 2 of the paper: KV <- Select(KV; ids), SL <- Select(SL; ids).
//
// Pure data movement, HBM-bound.  A retained row is N*D contiguous elements (3 KiB at 12x128 bf16),
// so each wave copies whole rows with 16-byte lanes: every load and store is a full-line access and
// evicted rows are never touched.  One wave moves one row of K and the same row of V per iteration,
// with all of a row's loads issued before its stores so that several KiB per wave are in flight.
#include "pafu_internal.h"
#include "quant_body.h"

namespace pafu {
namespace {

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kCompactThreads = 256;
constexpr int kWavesPerBlock = kCompactThreads / 64;
constexpr int kMaxChunksPerLane = 12;  // rows up to 64*12*16 B = 12 KiB go through the unrolled path

template <int CPL>  // 16-byte chunks per lane per row (row_bytes <= CPL*1024)
__global__ __launch_bounds__(kCompactThreads) void compact_rows_kernel(
    const char* __restrict__ K, const char* __restrict__ V, const float* __restrict__ SL, long long ld_in, int n,
    const int* __restrict__ ids, int count, int chunks, char* __restrict__ Ko, char* __restrict__ Vo,
    float* __restrict__ SLo, long long ld_out, const int* __restrict__ count_dev, CompactTail tail) {
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
  const int n_waves = gridDim.x * kWavesPerBlock;
  if (count_dev != nullptr) {  // the row count lives on the device (written by the selection): at most `count` rows
    const int c = *count_dev;
    count = c < count ? (c < 0 ? 0 : c) : count;
  }
  // rows [0, count) are gathered through ids; rows [count, count + tail.rows) are the tail's rows in order (the
  // chunk that a rollout appends behind the retained rows, Alg. 2).  The tail rows are handed out first: quantising
  // one is a long chain of integer arithmetic, which then runs beside the other waves' memory-bound gathers instead
  // of trailing behind them.
  const int total = count + tail.rows;
  for (int w = wave; w < total; w += n_waves) {
    const int r = w < tail.rows ? count + w : w - tail.rows;
    const u32x4 *ks, *vs;
    int id = 0;
    if (r < count) {
      id = ids[r];
      if ((unsigned)id >= (unsigned)n) continue;  // invalid index: leave the row untouched
      ks = reinterpret_cast<const u32x4*>(K + (long long)id * ld_in);
      vs = reinterpret_cast<const u32x4*>(V + (long long)id * ld_in);
    } else {
      ks = reinterpret_cast<const u32x4*>(tail.K + (long long)(r - count) * tail.ld);
      vs = reinterpret_cast<const u32x4*>(tail.V + (long long)(r - count) * tail.ld);
    }
    u32x4* kd = reinterpret_cast<u32x4*>(Ko + (long long)r * ld_out);
    u32x4* vd = reinterpret_cast<u32x4*>(Vo + (long long)r * ld_out);
    if (r >= count && tail.quant) {  // wave-uniform: 16 codes per lane and tensor from 32 bytes of bf16
#pragma unroll
      for (int i = 0; i < CPL; ++i) {
        const int c = lane + 64 * i;
        if (c < chunks) {
#pragma unroll
          for (int t = 0; t < 2; ++t) {
            const u32x4* src = (t ? vs : ks) + 2 * c;
            const u32x4 lo = __builtin_nontemporal_load(src), hi = __builtin_nontemporal_load(src + 1);
            const unsigned wl[4] = {lo[0], lo[1], lo[2], lo[3]}, wh[4] = {hi[0], hi[1], hi[2], hi[3]};
            unsigned cl[2], ch[2];
            e4m3_codes8(wl, t ? tail.inv_v : tail.inv_k, cl);
            e4m3_codes8(wh, t ? tail.inv_v : tail.inv_k, ch);
            u32x4 o;
            o[0] = cl[0]; o[1] = cl[1]; o[2] = ch[0]; o[3] = ch[1];
            __builtin_nontemporal_store(o, (t ? vd : kd) + c);
          }
        }
      }
      continue;
    }
    u32x4 kb[CPL], vb[CPL];
#pragma unroll
    for (int i = 0; i < CPL; ++i) {
      const int c = lane + 64 * i;
      if (c < chunks) {
        kb[i] = __builtin_nontemporal_load(ks + c);
        vb[i] = __builtin_nontemporal_load(vs + c);
      }
    }
#pragma unroll
    for (int i = 0; i < CPL; ++i) {
      const int c = lane + 64 * i;
      if (c < chunks) {
        __builtin_nontemporal_store(kb[i], kd + c);
        __builtin_nontemporal_store(vb[i], vd + c);
      }
    }
    if (SL != nullptr && lane == 0 && r < count) SLo[r] = SL[id];
  }
}

// The same gather for several layers in one launch (multi-layer steps): a wave takes a retained row and moves it in
// every layer of the batch, K and V, before it goes on to its next row.  The layers share the row geometry; each
// brings its own tensors and index list (the same list for all of them when the indices are shared, Sec. 3.3).
template <int CPL>
__global__ __launch_bounds__(kCompactThreads) void compact_rows_batch_kernel(CompactBatch B, int n_layers,
                                                                             long long ld_in, int n, int count,
                                                                             int chunks, long long ld_out,
                                                                             int tail_rows, long long ld_tail) {
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
  const int n_waves = gridDim.x * kWavesPerBlock;
  const int total = count + tail_rows;  // rows [count, total) come from every layer's tail tensors, in order
  for (int r = wave; r < total; r += n_waves) {
#pragma unroll 1
    for (int l = 0; l < n_layers; ++l) {
      const CompactLayer& L = B.layer[l];
      const u32x4 *ks, *vs;
      int id = 0;
      if (r < count) {
        id = L.ids[r];
        if ((unsigned)id >= (unsigned)n) continue;  // invalid index: leave the row untouched
        ks = reinterpret_cast<const u32x4*>(L.K + (long long)id * ld_in);
        vs = reinterpret_cast<const u32x4*>(L.V + (long long)id * ld_in);
      } else {
        ks = reinterpret_cast<const u32x4*>(L.Kt + (long long)(r - count) * ld_tail);
        vs = reinterpret_cast<const u32x4*>(L.Vt + (long long)(r - count) * ld_tail);
      }
      u32x4* kd = reinterpret_cast<u32x4*>(L.Ko + (long long)r * ld_out);
      u32x4* vd = reinterpret_cast<u32x4*>(L.Vo + (long long)r * ld_out);
      u32x4 kb[CPL], vb[CPL];
#pragma unroll
      for (int i = 0; i < CPL; ++i) {
        const int c = lane + 64 * i;
        if (c < chunks) {
          kb[i] = __builtin_nontemporal_load(ks + c);
          vb[i] = __builtin_nontemporal_load(vs + c);
        }
      }
#pragma unroll
      for (int i = 0; i < CPL; ++i) {
        const int c = lane + 64 * i;
        if (c < chunks) {
          __builtin_nontemporal_store(kb[i], kd + c);
          __builtin_nontemporal_store(vb[i], vd + c);
        }
      }
      if (L.SL != nullptr && lane == 0 && r < count) L.SLo[r] = L.SL[id];
    }
  }
}

// Rows longer than the unrolled path covers, or not a multiple of 16 bytes (then 4-byte words).
template <typename W>
__global__ __launch_bounds__(kCompactThreads) void compact_rows_generic_kernel(
    const char* __restrict__ K, const char* __restrict__ V, const float* __restrict__ SL, long long ld_in, int n,
    const int* __restrict__ ids, int count, int words, char* __restrict__ Ko, char* __restrict__ Vo,
    float* __restrict__ SLo, long long ld_out, const int* __restrict__ count_dev) {
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
  const int n_waves = gridDim.x * kWavesPerBlock;
  if (count_dev != nullptr) {
    const int c = *count_dev;
    count = c < count ? (c < 0 ? 0 : c) : count;
  }
  for (int r = wave; r < count; r += n_waves) {
    const int id = ids[r];
    if ((unsigned)id >= (unsigned)n) continue;
    const W* ks = reinterpret_cast<const W*>(K + (long long)id * ld_in);
    const W* vs = reinterpret_cast<const W*>(V + (long long)id * ld_in);
    W* kd = reinterpret_cast<W*>(Ko + (long long)r * ld_out);
    W* vd = reinterpret_cast<W*>(Vo + (long long)r * ld_out);
    for (int c = lane; c < words; c += 64) {
      kd[c] = ks[c];
      vd[c] = vs[c];
    }
    if (SL != nullptr && lane == 0) SLo[r] = SL[id];
  }
}

// Contiguous row range copy (appending the chunk's rows to the compacted cache in a rollout).
__global__ __launch_bounds__(kCompactThreads) void append_rows_kernel(
    const char* __restrict__ K, const char* __restrict__ V, const float* __restrict__ S, long long ld_in, int rows,
    int chunks, char* __restrict__ Ko, char* __restrict__ Vo, float* __restrict__ So, long long ld_out) {
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
  const int n_waves = gridDim.x * kWavesPerBlock;
  for (int r = wave; r < rows; r += n_waves) {
    const u32x4* ks = reinterpret_cast<const u32x4*>(K + (long long)r * ld_in);
    const u32x4* vs = reinterpret_cast<const u32x4*>(V + (long long)r * ld_in);
    u32x4* kd = reinterpret_cast<u32x4*>(Ko + (long long)r * ld_out);
    u32x4* vd = reinterpret_cast<u32x4*>(Vo + (long long)r * ld_out);
    for (int c = lane; c < chunks; c += 64) {
      kd[c] = ks[c];
      vd[c] = vs[c];
    }
    if (S != nullptr && lane == 0) So[r] = S[r];
  }
}

int grid_for_rows(int rows) {
  // one row per wave per iteration; enough blocks to cover the chip several times over
  long long blocks = ((long long)rows + kWavesPerBlock - 1) / kWavesPerBlock;
  const long long cap = 256 * 16;
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  return (int)blocks;
}

}  // namespace

bool compact_takes_tail(int row_bytes) { return row_bytes % 16 == 0 && row_bytes <= kMaxChunksPerLane * 1024; }

int launch_compact(hipStream_t st, const void* K, const void* V, const float* SL, long long ld_in_bytes, int n,
                   const int* ids, int count, int row_bytes, void* K_out, void* V_out, float* SL_out,
                   long long ld_out_bytes, const int* count_dev, const CompactTail* tail_rows) {
  CompactTail tail{nullptr, nullptr, 0, 0, 0, 1.f, 1.f};
  if (tail_rows != nullptr && tail_rows->rows > 0) {
    if (!compact_takes_tail(row_bytes)) return PAFU_ERR_SHAPE;  // callers ask compact_takes_tail first
    tail = *tail_rows;
  }
  if (count < 0) count = 0;
  if (count + tail.rows <= 0) return PAFU_OK;
  const dim3 grid(grid_for_rows(count + tail.rows)), block(kCompactThreads);
  const char* k = static_cast<const char*>(K);
  const char* v = static_cast<const char*>(V);
  char* ko = static_cast<char*>(K_out);
  char* vo = static_cast<char*>(V_out);
  if (row_bytes % 16 == 0 && row_bytes <= kMaxChunksPerLane * 1024) {
    const int chunks = row_bytes / 16;
    const int cpl = (chunks + 63) / 64;
#define PAFU_COMPACT_CASE(C)                                                                                  \
  hipLaunchKernelGGL(compact_rows_kernel<C>, grid, block, 0, st, k, v, SL, ld_in_bytes, n, ids, count, chunks, \
                     ko, vo, SL_out, ld_out_bytes, count_dev, tail)
    if (cpl <= 1) PAFU_COMPACT_CASE(1);
    else if (cpl <= 2) PAFU_COMPACT_CASE(2);
    else if (cpl <= 3) PAFU_COMPACT_CASE(3);
    else if (cpl <= 4) PAFU_COMPACT_CASE(4);
    else if (cpl <= 6) PAFU_COMPACT_CASE(6);
    else if (cpl <= 8) PAFU_COMPACT_CASE(8);
    else if (cpl <= 10) PAFU_COMPACT_CASE(10);
    else PAFU_COMPACT_CASE(12);
#undef PAFU_COMPACT_CASE
  } else if (row_bytes % 16 == 0) {
    hipLaunchKernelGGL(compact_rows_generic_kernel<u32x4>, grid, block, 0, st, k, v, SL, ld_in_bytes, n, ids, count,
                       row_bytes / 16, ko, vo, SL_out, ld_out_bytes, count_dev);
  } else {
    hipLaunchKernelGGL(compact_rows_generic_kernel<unsigned int>, grid, block, 0, st, k, v, SL, ld_in_bytes, n, ids,
                       count, row_bytes / 4, ko, vo, SL_out, ld_out_bytes, count_dev);
  }
  return check_launch();
}

bool compact_batchable(int row_bytes) { return row_bytes % 16 == 0 && row_bytes <= 4 * 1024; }

int launch_compact_batch(hipStream_t st, const CompactLayer* layers, int n_layers, long long ld_in_bytes, int n,
                         int count, int row_bytes, long long ld_out_bytes, int tail_rows, long long ld_tail_bytes) {
  if (count < 0) count = 0;
  if (tail_rows < 0) tail_rows = 0;
  if (count + tail_rows <= 0 || n_layers <= 0) return PAFU_OK;
  const int chunks = row_bytes / 16;
  const int cpl = (chunks + 63) / 64;
  for (int first = 0; first < n_layers; first += kCompactBatchMax) {
    const int m = n_layers - first < kCompactBatchMax ? n_layers - first : kCompactBatchMax;
    CompactBatch B;
    for (int i = 0; i < kCompactBatchMax; ++i) B.layer[i] = layers[first + (i < m ? i : 0)];
    const dim3 grid(grid_for_rows(count + tail_rows)), block(kCompactThreads);
#define PAFU_COMPACT_BATCH_CASE(C)                                                                                \
  hipLaunchKernelGGL(compact_rows_batch_kernel<C>, grid, block, 0, st, B, m, ld_in_bytes, n, count, chunks,      \
                     ld_out_bytes, tail_rows, ld_tail_bytes)
    if (cpl <= 1) PAFU_COMPACT_BATCH_CASE(1);
    else if (cpl <= 2) PAFU_COMPACT_BATCH_CASE(2);
    else if (cpl <= 3) PAFU_COMPACT_BATCH_CASE(3);
    else PAFU_COMPACT_BATCH_CASE(4);
#undef PAFU_COMPACT_BATCH_CASE
    const int rc = check_launch();
    if (rc) return rc;
  }
  return PAFU_OK;
}

int launch_append(hipStream_t st, const void* K, const void* V, const float* S, long long ld_in_bytes, int rows,
                  int row_bytes, void* K_out, void* V_out, float* S_out, long long ld_out_bytes) {
  if (rows <= 0) return PAFU_OK;
  hipLaunchKernelGGL(append_rows_kernel, dim3(grid_for_rows(rows)), dim3(kCompactThreads), 0, st,
                     static_cast<const char*>(K), static_cast<const char*>(V), S, ld_in_bytes, rows, row_bytes / 16,
                     static_cast<char*>(K_out), static_cast<char*>(V_out), S_out, ld_out_bytes);
  return check_launch();
}

}  // namespace pafu

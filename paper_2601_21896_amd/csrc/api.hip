// C ABI of libpafu: argument validation and the chunk-step driver (Alg. 2 of the paper).
// Every entry point validates on the host first; an error return means nothing was enqueued.
#include <math.h>

#include "pafu_internal.h"

namespace pafu {
namespace {
thread_local int g_last_hip_error = 0;
}
int record_hip_error(hipError_t e) {
  g_last_hip_error = static_cast<int>(e);
  return PAFU_ERR_HIP;
}
int compute_units() {
  static std::mutex mu;
  static int cached[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  std::lock_guard<std::mutex> lock(mu);
  if (cached[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cached[dev] = n;
  }
  return cached[dev];
}
namespace {

__global__ void probe_kernel() {}

// Optional timing hook of a step.
int record_stage(hipStream_t st, const pafu_step_args* a, int i) {
  if (a->stage_events[i] == nullptr) return PAFU_OK;
  const hipError_t e = hipEventRecord(static_cast<hipEvent_t>(a->stage_events[i]), st);
  return e == hipSuccess ? PAFU_OK : record_hip_error(e);
}

int dtype_bytes(int dtype) { return dtype == PAFU_BF16 ? 2 : (dtype == PAFU_F32 ? 4 : 0); }
// element size of a K/V cache tensor: the 8-bit storage format is allowed there (and only there)
int kv_dtype_bytes(int dtype) { return dtype == PAFU_FP8_E4M3 ? 1 : dtype_bytes(dtype); }
bool scale_ok(int scale_log2) { return scale_log2 >= -64 && scale_log2 <= 64; }

int check_score(const void* x0, const void* x1, const void* x2, int n_seg, int T, int Fs, long long ld_x, int x_dtype,
                const void* W1, const float* W2, int M, int n_out, int act, const float* out, const void* ws,
                size_t ws_bytes) {
  if (T < 0 || Fs <= 0 || M <= 0 || n_out <= 0 || n_seg < 1 || n_seg > 3 || ld_x < Fs) return PAFU_ERR_SHAPE;
  if (act != PAFU_ACT_SILU && act != PAFU_ACT_GELU_ERF) return PAFU_ERR_SHAPE;
  const int eb = dtype_bytes(x_dtype);
  if (eb == 0) return PAFU_ERR_DTYPE;
  if (T == 0) return PAFU_OK;
  if (!x0 || (n_seg > 1 && !x1) || (n_seg > 2 && !x2) || !W1 || !W2 || !out) return PAFU_ERR_NULL;
  if (!aligned16(x0) || (n_seg > 1 && !aligned16(x1)) || (n_seg > 2 && !aligned16(x2)) || !aligned16(W1) ||
      !aligned16(W2) || (ld_x * eb) % 16 != 0)
    return PAFU_ERR_ALIGN;
  // ws_bytes == SIZE_MAX: the caller brings its own scratch (pafu_score_static)
  if (n_out > 1 && ws_bytes != SIZE_MAX && (ws == nullptr || ws_bytes < pafu_score_workspace_bytes(M)))
    return PAFU_ERR_WORKSPACE;
  return PAFU_OK;
}

int check_select(const float* scores, int n, int k, const int* out_ids) {
  if (n < 0 || k < 0) return PAFU_ERR_SHAPE;
  if (n > 0 && !scores) return PAFU_ERR_NULL;
  if (n > 0 && k > 0 && !out_ids) return PAFU_ERR_NULL;
  if (!aligned16(scores)) return PAFU_ERR_ALIGN;
  return PAFU_OK;
}

int check_compact(const void* K, const void* V, const float* SL, long long ld_in, int n, const int* ids, int count,
                  int N, int D, int dtype, void* K_out, void* V_out, float* SL_out, long long ld_out) {
  if (n < 0 || count < 0 || N <= 0 || D <= 0 || count > n) return PAFU_ERR_SHAPE;
  const int eb = kv_dtype_bytes(dtype);
  if (eb == 0) return PAFU_ERR_DTYPE;
  const long long row = (long long)N * D;
  if (ld_in < row || ld_out < row || (row * eb) % 4 != 0 || row * eb > (1ll << 30)) return PAFU_ERR_SHAPE;
  if (count == 0) return PAFU_OK;
  if (!K || !V || !ids || !K_out || !V_out) return PAFU_ERR_NULL;
  if ((SL == nullptr) != (SL_out == nullptr)) return PAFU_ERR_NULL;
  if (!aligned16(K) || !aligned16(V) || !aligned16(K_out) || !aligned16(V_out) || (ld_in * eb) % 16 != 0 ||
      (ld_out * eb) % 16 != 0)
    return PAFU_ERR_ALIGN;
  const size_t in_bytes = (size_t)n * ld_in * eb, out_bytes = (size_t)count * ld_out * eb;
  if (overlaps(K, in_bytes, K_out, out_bytes) || overlaps(K, in_bytes, V_out, out_bytes) ||
      overlaps(V, in_bytes, K_out, out_bytes) || overlaps(V, in_bytes, V_out, out_bytes) ||
      overlaps(K_out, out_bytes, V_out, out_bytes) ||
      (SL && overlaps(SL, (size_t)n * 4, SL_out, (size_t)count * 4)))
    return PAFU_ERR_ALIAS;
  return PAFU_OK;
}

int check_attention(const void* Q, int Lq, const void* Kc, const void* Vc, int n_kept, const void* Kn, const void* Vn,
                    int Lc, int N, int D, long long ld_q, long long ld_c, long long ld_n, long long ld_o,
                    int block_len, const void* O, int out_dtype, int kvb = 2 /* bytes per K/V element */) {
  if (Lq < 1 || Lc < 1 || n_kept < 0 || N < 1 || block_len < 1 || Lq > Lc) return PAFU_ERR_SHAPE;
  if (((long long)Lq / 32 + 1) * N > 0x7fffffffll) return PAFU_ERR_SHAPE;  // one-dimensional grid
  if (D != 64 && D != 128) return PAFU_ERR_SHAPE;
  if ((long long)n_kept + Lc > 0x7fff0000ll) return PAFU_ERR_SHAPE;
  const int ob = dtype_bytes(out_dtype);
  if (ob == 0) return PAFU_ERR_DTYPE;
  const long long row = (long long)N * D;
  if (ld_q < row || ld_n < row || ld_o < row || (n_kept > 0 && ld_c < row)) return PAFU_ERR_SHAPE;
  // a 64-key tile is addressed as a 64-bit tile base plus 32-bit byte offsets: 64 rows must span less than 4 GiB
  if (ld_n * kvb * 64 >= (1ll << 32) || (n_kept > 0 && ld_c * kvb * 64 >= (1ll << 32))) return PAFU_ERR_SHAPE;
  if (!Q || !Kn || !Vn || !O || (n_kept > 0 && (!Kc || !Vc))) return PAFU_ERR_NULL;
  if (!aligned16(Q) || !aligned16(Kn) || !aligned16(Vn) || !aligned16(O) || !aligned16(Kc) || !aligned16(Vc) ||
      (ld_q * 2) % 16 != 0 || (ld_n * kvb) % 16 != 0 || (ld_c * kvb) % 16 != 0 || (ld_o * ob) % 16 != 0)
    return PAFU_ERR_ALIGN;
  const size_t o_bytes = (size_t)Lq * ld_o * ob;
  if (overlaps(O, o_bytes, Q, (size_t)Lq * ld_q * 2) || overlaps(O, o_bytes, Kn, (size_t)Lc * ld_n * kvb) ||
      overlaps(O, o_bytes, Vn, (size_t)Lc * ld_n * kvb) ||
      (n_kept > 0 && (overlaps(O, o_bytes, Kc, (size_t)n_kept * ld_c * kvb) ||
                      overlaps(O, o_bytes, Vc, (size_t)n_kept * ld_c * kvb))))
    return PAFU_ERR_ALIAS;
  return PAFU_OK;
}

// A strided buffer: `rows` rows of `row` bytes, `ld` bytes apart.
struct Span {
  const void* p;
  long long rows, ld, row;
};
// Do two strided buffers share a byte?  Exact for equal strides (rows of one may sit in the gaps of the other, as
// with K and V interleaved in one slab); otherwise decided on the enclosing byte ranges.
bool spans_overlap(const Span& a, const Span& b) {
  if (!a.p || !b.p || a.rows <= 0 || b.rows <= 0 || a.row <= 0 || b.row <= 0) return false;
  const uintptr_t a0 = reinterpret_cast<uintptr_t>(a.p), b0 = reinterpret_cast<uintptr_t>(b.p);
  const uintptr_t a1 = a0 + (uintptr_t)((a.rows - 1) * a.ld + a.row), b1 = b0 + (uintptr_t)((b.rows - 1) * b.ld + b.row);
  if (a1 <= b0 || b1 <= a0) return false;
  if (a.ld == b.ld && a.ld > 0) {
    const uintptr_t ld = (uintptr_t)a.ld;
    const uintptr_t delta = b0 >= a0 ? (b0 - a0) % ld : (ld - (a0 - b0) % ld) % ld;  // b's row start inside a's period
    if (delta >= (uintptr_t)a.row && ld - delta >= (uintptr_t)b.row) return false;
  }
  return true;
}

// bf16 rows <-> 8-bit rows (both directions: `wide` is the bf16 side)
int check_quant(const void* Kw, const void* Vw, long long ld_w, int rows, int N, int D, int ks, int vs, const void* Kq,
                const void* Vq, long long ld_q, bool wide_is_output) {
  if (rows < 0 || N <= 0 || D <= 0 || ((long long)N * D) % 8 != 0 || (long long)N * D > (1ll << 30)) return PAFU_ERR_SHAPE;
  if (!scale_ok(ks) || !scale_ok(vs)) return PAFU_ERR_SHAPE;
  const long long row = (long long)N * D;
  if (ld_w < row || ld_q < row) return PAFU_ERR_SHAPE;
  if (rows == 0) return PAFU_OK;
  if (!Kw || !Vw || !Kq || !Vq) return PAFU_ERR_NULL;
  if (!aligned16(Kw) || !aligned16(Vw) || !aligned16(Kq) || !aligned16(Vq) || (ld_w * 2) % 16 != 0 || ld_q % 16 != 0)
    return PAFU_ERR_ALIGN;
  const Span w0{Kw, rows, ld_w * 2, row * 2}, w1{Vw, rows, ld_w * 2, row * 2}, q0{Kq, rows, ld_q, row}, q1{Vq, rows, ld_q, row};
  if (spans_overlap(w0, q0) || spans_overlap(w0, q1) || spans_overlap(w1, q0) || spans_overlap(w1, q1) ||
      (wide_is_output ? spans_overlap(w0, w1) : spans_overlap(q0, q1)))
    return PAFU_ERR_ALIAS;
  return PAFU_OK;
}

// Everything a step reads and everything it writes (the workspace apart).  `scoring` is false for a layer that takes
// its indices from another layer: then only the cache part counts.
struct StepSpans {
  Span in[20], out[8];
  int n_in = 0, n_out = 0;
};
void step_spans(const pafu_step_args* a, bool scoring, StepSpans& s) {
  const long long n = a->n, Lc = a->Lc, n_kept = a->k < a->n ? a->k : a->n;
  const bool single = a->mode == PAFU_MODE_SINGLE;
  const bool kv8 = a->kv_dtype == PAFU_FP8_E4M3;  // the quantised chunk rows then follow the retained ones in any mode
  const long long kvb = kv8 ? 1 : 2;
  const long long rowb = (long long)a->N * a->D * 2, rowkv = (long long)a->N * a->D * kvb;
  const long long out_rows = n_kept + ((single && !kv8) ? 0 : Lc), sl_rows = n_kept + (single ? 0 : Lc);
  auto in = [&](const void* p, long long rows, long long ld, long long row) { s.in[s.n_in++] = Span{p, rows, ld, row}; };
  auto out = [&](const void* p, long long rows, long long ld, long long row) { s.out[s.n_out++] = Span{p, rows, ld, row}; };
  if (scoring) {
    const long long eb = dtype_bytes(a->x_dtype), F = (long long)a->n_seg * a->Fs;
    for (int g = 0; g < a->n_seg && g < 3; ++g) {
      if (single) in(a->x_cache[g], n, a->ld_x * eb, a->Fs * eb);
      in(a->x_chunk[g], Lc, a->ld_x * eb, a->Fs * eb);
    }
    in(a->W1, 1, 0, (long long)a->M * F * eb);
    in(a->b1, 1, 0, (long long)a->M * 4);
    in(a->W2, 1, 0, (long long)a->n_out * a->M * 4);
    in(a->b2, 1, 0, (long long)a->n_out * 4);
    if (single) out(a->scores, 1, 0, (n + Lc) * 4);
    else in(a->SL_in, 1, 0, n * 4);
    out(a->ids, 1, 0, n_kept * 4);
    out(a->SL_out, 1, 0, sl_rows * 4);
  }
  in(a->K_cache, n, a->ld_cache * kvb, rowkv);
  in(a->V_cache, n, a->ld_cache * kvb, rowkv);
  in(a->Q, Lc, a->ld_chunk * 2, rowb);
  in(a->K_chunk, Lc, a->ld_chunk * 2, rowb);
  in(a->V_chunk, Lc, a->ld_chunk * 2, rowb);
  out(a->K_out, out_rows, a->ld_out * kvb, rowkv);
  out(a->V_out, out_rows, a->ld_out * kvb, rowkv);
  out(a->O, Lc, a->ld_o * dtype_bytes(a->out_dtype), (long long)a->N * a->D * dtype_bytes(a->out_dtype));
}
// No output of a step may overlap one of its inputs, another output or the workspace (in ROLLOUT the output slab
// counts with the appended chunk rows).
int check_step_alias(const pafu_step_args* a, bool scoring) {
  StepSpans s;
  step_spans(a, scoring, s);
  const Span ws{a->workspace, 1, 0, (long long)a->workspace_bytes};
  for (int i = 0; i < s.n_out; ++i) {
    for (int j = 0; j < s.n_in; ++j)
      if (spans_overlap(s.out[i], s.in[j])) return PAFU_ERR_ALIAS;
    for (int j = i + 1; j < s.n_out; ++j)
      if (spans_overlap(s.out[i], s.out[j])) return PAFU_ERR_ALIAS;
    if (scoring && spans_overlap(s.out[i], ws)) return PAFU_ERR_ALIAS;
  }
  if (scoring)
    for (int j = 0; j < s.n_in; ++j)
      if (spans_overlap(ws, s.in[j])) return PAFU_ERR_ALIAS;
  return PAFU_OK;
}
// The multi-layer steps reorder the stages across layers (all scores, then all selections, then the caches), so what
// one layer writes must not overlap what any other layer reads or writes.  Only the workspace may be shared.
int check_layers_alias(const pafu_step_args* args, int n_layers, int index_layer /* -1: every layer scores */) {
  for (int a = 0; a < n_layers; ++a) {
    StepSpans sa;
    step_spans(&args[a], index_layer < 0 || a == index_layer, sa);
    for (int b = 0; b < n_layers; ++b) {
      if (b == a) continue;
      StepSpans sb;
      step_spans(&args[b], index_layer < 0 || b == index_layer, sb);
      for (int i = 0; i < sa.n_out; ++i) {
        for (int j = 0; j < sb.n_in; ++j)
          if (spans_overlap(sa.out[i], sb.in[j])) return PAFU_ERR_ALIAS;
        for (int j = 0; b > a && j < sb.n_out; ++j)
          if (spans_overlap(sa.out[i], sb.out[j])) return PAFU_ERR_ALIAS;
      }
    }
  }
  return PAFU_OK;
}

// The optional workspace of the attention calls: aligned, and apart from every tensor of the call.
int check_attention_ws(const void* ws, size_t ws_bytes, const void* Q, int Lq, const void* Kc, const void* Vc, int n_c,
                       const void* Kn, const void* Vn, int Lc, long long ld_q, long long ld_c, long long ld_n,
                       long long ld_o, const void* O, int out_dtype) {
  if (ws == nullptr || ws_bytes == 0) return PAFU_OK;
  if (!aligned16(ws)) return PAFU_ERR_ALIGN;
  if (overlaps(ws, ws_bytes, Q, (size_t)Lq * ld_q * 2) || overlaps(ws, ws_bytes, Kn, (size_t)Lc * ld_n * 2) ||
      overlaps(ws, ws_bytes, Vn, (size_t)Lc * ld_n * 2) || overlaps(ws, ws_bytes, O, (size_t)Lq * ld_o * dtype_bytes(out_dtype)) ||
      (n_c > 0 && (overlaps(ws, ws_bytes, Kc, (size_t)n_c * ld_c * 2) || overlaps(ws, ws_bytes, Vc, (size_t)n_c * ld_c * 2))))
    return PAFU_ERR_ALIAS;
  return PAFU_OK;
}

size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }
// The part of a step's workspace that the scoring needs (the rest, if present, serves the attention launch).
size_t step_score_workspace(const pafu_step_args* a) {
  return a->n_out > 1 ? align_up(pafu_score_workspace_bytes(a->M)) : 0;
}

// The attention part of a layer's step.  bf16 K/V: retained rows in K_out/V_out, chunk rows read in place from
// K_chunk/V_chunk.  8-bit K/V: the chunk is quantised behind the retained rows of K_out/V_out first (head dim 128
// only) and attention reads both segments from there.
int check_layer_attention(const pafu_step_args* a, int n_kept) {
  if (a->kv_dtype != PAFU_FP8_E4M3)
    return check_attention(a->Q, a->Lc, a->K_out, a->V_out, n_kept, a->K_chunk, a->V_chunk, a->Lc, a->N, a->D,
                           a->ld_chunk, a->ld_out, a->ld_chunk, a->ld_o, a->block_len, a->O, a->out_dtype);
  if (a->D != 128) return PAFU_ERR_SHAPE;
  if (!a->K_out || !a->V_out) return PAFU_ERR_NULL;
  char* kq = static_cast<char*>(a->K_out) + (long long)n_kept * a->ld_out;
  char* vq = static_cast<char*>(a->V_out) + (long long)n_kept * a->ld_out;
  int rc = check_quant(a->K_chunk, a->V_chunk, a->ld_chunk, a->Lc, a->N, a->D, a->k_scale_log2, a->v_scale_log2, kq, vq,
                       a->ld_out, false);
  if (rc) return rc;
  return check_attention(a->Q, a->Lc, a->K_out, a->V_out, n_kept, kq, vq, a->Lc, a->N, a->D, a->ld_chunk, a->ld_out,
                         a->ld_out, a->ld_o, a->block_len, a->O, a->out_dtype, 1);
}

// Validates a whole step without enqueuing anything.
int check_step(const pafu_step_args* a) {
  if (!a) return PAFU_ERR_NULL;
  if (a->mode != PAFU_MODE_SINGLE && a->mode != PAFU_MODE_ROLLOUT) return PAFU_ERR_SHAPE;
  if (a->n < 0 || a->k < 0 || a->Lc < 1 || a->N < 1 || a->D < 1 || a->n_pinned < 0) return PAFU_ERR_SHAPE;
  if (a->kv_dtype != PAFU_BF16 && a->kv_dtype != PAFU_FP8_E4M3) return PAFU_ERR_DTYPE;
  const int n_kept = a->k < a->n ? a->k : a->n;
  const bool single = a->mode == PAFU_MODE_SINGLE;
  if (a->workspace_bytes < step_score_workspace(a) || (a->workspace == nullptr && a->workspace_bytes > 0))
    return PAFU_ERR_WORKSPACE;
  if (step_score_workspace(a) > 0 && a->workspace == nullptr) return PAFU_ERR_WORKSPACE;
  if (!aligned16(a->workspace)) return PAFU_ERR_ALIGN;
  int rc;
  float* chunk_scores = single ? (a->scores ? a->scores + a->n : nullptr) : (a->SL_out ? a->SL_out + n_kept : nullptr);
  if (!chunk_scores) return PAFU_ERR_NULL;
  if (single && a->n > 0) {
    rc = check_score(a->x_cache[0], a->x_cache[1], a->x_cache[2], a->n_seg, a->n, a->Fs, a->ld_x, a->x_dtype, a->W1,
                     a->W2, a->M, a->n_out, a->act, a->scores, a->workspace, a->workspace_bytes);
    if (rc) return rc;
  }
  rc = check_score(a->x_chunk[0], a->x_chunk[1], a->x_chunk[2], a->n_seg, a->Lc, a->Fs, a->ld_x, a->x_dtype, a->W1,
                   a->W2, a->M, a->n_out, a->act, chunk_scores, a->workspace, a->workspace_bytes);
  if (rc) return rc;
  const float* sel_scores = single ? a->scores : a->SL_in;
  rc = check_select(sel_scores, a->n, a->k, a->ids);
  if (rc) return rc;
  if (a->n > 0 && !a->SL_out) return PAFU_ERR_NULL;
  rc = check_compact(a->K_cache, a->V_cache, sel_scores, a->ld_cache, a->n, a->ids, n_kept, a->N, a->D, a->kv_dtype,
                     a->K_out, a->V_out, a->SL_out, a->ld_out);
  if (rc) return rc;
  rc = check_layer_attention(a, n_kept);
  if (rc) return rc;
  if (!single) {
    if (!a->K_out || !a->V_out) return PAFU_ERR_NULL;
    if (!aligned16(a->K_out) || !aligned16(a->V_out) || (a->ld_out * kv_dtype_bytes(a->kv_dtype)) % 16 != 0)
      return PAFU_ERR_ALIGN;
    if (a->ld_out < (long long)a->N * a->D) return PAFU_ERR_SHAPE;
  }
  return check_step_alias(a, true);
}

// The scoring part of a step: SINGLE scores cache + chunk into a->scores, ROLLOUT the chunk into SL_out behind the
// retained rows.
// `selected` (may be null): in ROLLOUT the selection reads the stored list only, so it may ride in the scoring launch;
// set when it did and the caller has no selection left to launch.
int enqueue_scores(hipStream_t st, const pafu_step_args* a, bool* selected = nullptr) {
  if (selected != nullptr) *selected = false;
  const int n_kept = a->k < a->n ? a->k : a->n;
  const bool single = a->mode == PAFU_MODE_SINGLE;
  int rc = record_stage(st, a, 0);
  if (rc) return rc;
  float* chunk_scores = single ? a->scores + a->n : a->SL_out + n_kept;
  if (single && a->n > 0) {
    // cache and chunk features that sit back to back are scored in one launch
    const int eb = dtype_bytes(a->x_dtype);
    bool contiguous = true;
    for (int s = 0; s < a->n_seg; ++s)
      contiguous = contiguous && static_cast<const char*>(a->x_chunk[s]) ==
                                     static_cast<const char*>(a->x_cache[s]) + (long long)a->n * a->ld_x * eb;
    if (contiguous) {
      rc = launch_score(st, a->x_cache[0], a->x_cache[1], a->x_cache[2], a->n_seg, a->n + a->Lc, a->Fs, a->ld_x,
                        a->x_dtype, a->W1, a->b1, a->W2, a->b2, a->M, a->n_out, a->act, a->scores, a->workspace);
      if (rc) return rc;
    } else {
      rc = launch_score(st, a->x_cache[0], a->x_cache[1], a->x_cache[2], a->n_seg, a->n, a->Fs, a->ld_x, a->x_dtype,
                        a->W1, a->b1, a->W2, a->b2, a->M, a->n_out, a->act, a->scores, a->workspace);
      if (rc) return rc;
      rc = launch_score(st, a->x_chunk[0], a->x_chunk[1], a->x_chunk[2], a->n_seg, a->Lc, a->Fs, a->ld_x, a->x_dtype,
                        a->W1, a->b1, a->W2, a->b2, a->M, a->n_out, a->act, chunk_scores, a->workspace);
      if (rc) return rc;
    }
  } else {
    // SINGLE with an empty cache, or ROLLOUT (the chunk's scores land behind the retained ones in SL_out)
    const SelectJob job{a->SL_in, a->ids, nullptr, a->n, a->k, a->n_pinned};
    const bool may_ride = selected != nullptr && !single && a->n > 0;
    rc = launch_score(st, a->x_chunk[0], a->x_chunk[1], a->x_chunk[2], a->n_seg, a->Lc, a->Fs, a->ld_x, a->x_dtype,
                      a->W1, a->b1, a->W2, a->b2, a->M, a->n_out, a->act, chunk_scores, a->workspace,
                      may_ride ? &job : nullptr, selected);
    if (rc) return rc;
  }
  return record_stage(st, a, 1);
}

// The part of a layer's workspace that the attention launch may use: what lies behind the scoring part.
struct WsPart {
  void* p;
  size_t bytes;
};
WsPart attention_ws(const pafu_step_args* a, bool scoring) {
  const size_t used = scoring ? step_score_workspace(a) : 0;
  if (a->workspace == nullptr || a->workspace_bytes <= used) return WsPart{nullptr, 0};
  return WsPart{static_cast<char*>(a->workspace) + used, a->workspace_bytes - used};
}

// The cache part of a step for one layer: compact K/V (and the score list when sel_scores is given) to `ids`,
// attend over retained + chunk, and in ROLLOUT append the chunk's K/V behind the retained rows.
// `done`: what a batched launch of the caller has already moved for this layer.
enum : int { kDoneNothing = 0, kDoneCompact = 1, kDoneAppend = 2 };
int enqueue_kv(hipStream_t st, const pafu_step_args* a, const int* ids, const float* sel_scores, float* SL_out,
               void* attn_ws, size_t attn_ws_bytes, int done = kDoneNothing) {
  const int n_kept = a->k < a->n ? a->k : a->n;
  const float scale = a->softmax_scale > 0.f ? a->softmax_scale : 1.0f / sqrtf((float)a->D);
  const bool kv8 = a->kv_dtype == PAFU_FP8_E4M3;
  const int kvb = kv8 ? 1 : 2;
  int rc;
  // In a rollout with bf16 storage the compaction launch also moves the chunk's rows behind the retained ones: the
  // append costs no launch of its own, and attention (which reads the chunk from its own buffers) does not wait for it.
  bool appended = (done & kDoneAppend) != 0;
  if (a->n > 0 && !(done & kDoneCompact)) {
    // (with the 8-bit cache the tail rows are quantised on the way, in both modes: the chunk always attends over codes)
    CompactTail tail{static_cast<const char*>(a->K_chunk), static_cast<const char*>(a->V_chunk),
                     (long long)a->ld_chunk * 2, a->Lc, kv8 ? 1 : 0, ldexpf(1.0f, -a->k_scale_log2),
                     ldexpf(1.0f, -a->v_scale_log2)};
    appended = (kv8 || a->mode != PAFU_MODE_SINGLE) && compact_takes_tail(a->N * a->D * kvb);
    rc = launch_compact(st, a->K_cache, a->V_cache, sel_scores, a->ld_cache * kvb, a->n, ids, n_kept, a->N * a->D * kvb,
                        a->K_out, a->V_out, SL_out, a->ld_out * kvb, nullptr, appended ? &tail : nullptr);
    if (rc) return rc;
  }
  char* ko = static_cast<char*>(a->K_out) + (long long)n_kept * a->ld_out * kvb;
  char* vo = static_cast<char*>(a->V_out) + (long long)n_kept * a->ld_out * kvb;
  if (kv8 && !appended) {
    // the chunk's K/V enter the cache as codes before attention: the chunk attends over exactly what later steps
    // will find in the cache, and in a rollout nothing is left to append
    rc = launch_quantize(st, a->K_chunk, a->V_chunk, a->ld_chunk * 2, a->Lc, a->N * a->D, a->k_scale_log2,
                         a->v_scale_log2, ko, vo, a->ld_out);
    if (rc) return rc;
  }
  rc = record_stage(st, a, 3);
  if (rc) return rc;
  if (kv8)
    rc = launch_attention(st, a->Q, a->Lc, a->K_out, a->V_out, n_kept, ko, vo, a->Lc, a->N, a->D, a->ld_chunk, a->ld_out,
                          a->ld_out, a->ld_o, a->block_len, scale, a->O, a->out_dtype, attn_ws, attn_ws_bytes, nullptr, 0,
                          PAFU_FP8_E4M3, ldexpf(1.0f, a->k_scale_log2), ldexpf(1.0f, a->v_scale_log2));
  else
    rc = launch_attention(st, a->Q, a->Lc, a->K_out, a->V_out, n_kept, a->K_chunk, a->V_chunk, a->Lc, a->N, a->D,
                          a->ld_chunk, a->ld_out, a->ld_chunk, a->ld_o, a->block_len, scale, a->O, a->out_dtype, attn_ws,
                          attn_ws_bytes);
  if (rc) return rc;
  rc = record_stage(st, a, 4);
  if (rc) return rc;
  if (a->mode != PAFU_MODE_SINGLE && !kv8 && !appended) {
    rc = launch_append(st, a->K_chunk, a->V_chunk, nullptr, a->ld_chunk * 2, a->Lc, a->N * a->D * 2, ko, vo, nullptr,
                       a->ld_out * 2);
    if (rc) return rc;
  }
  return PAFU_OK;
}

int enqueue_step(hipStream_t st, const pafu_step_args* a) {
  bool selected = false;
  int rc = enqueue_scores(st, a, &selected);
  if (rc) return rc;
  const float* sel_scores = a->mode == PAFU_MODE_SINGLE ? a->scores : a->SL_in;
  if (a->n > 0 && !selected) {
    rc = launch_select(st, sel_scores, a->n, a->k, a->n_pinned, a->ids, nullptr, nullptr);
    if (rc) return rc;
  }
  rc = record_stage(st, a, 2);
  if (rc) return rc;
  const WsPart ws = attention_ws(a, true);
  return enqueue_kv(st, a, a->ids, sel_scores, a->SL_out, ws.p, ws.bytes);
}

// Multi-layer steps: when all layers share the cache geometry their compactions run as one launch per 32 layers
// (each layer with its own tensors and index list; `shared_ids` non-null = one list for all).  In a bf16 rollout whose
// layers also share the chunk geometry the same launch appends every layer's chunk rows.  Returns what it did
// (kDone* bits).
int enqueue_compact_batch(hipStream_t st, const pafu_step_args* args, int n_layers, const int* shared_ids,
                           int score_layer /* -1: every layer compacts its own score list */, int* rc_out) {
  *rc_out = PAFU_OK;
  if (n_layers < 2) return kDoneNothing;
  const pafu_step_args* a0 = &args[0];
  const int kvb = kv_dtype_bytes(a0->kv_dtype);
  const long long rowb = (long long)a0->N * a0->D * kvb;
  if (a0->n <= 0 || rowb > (1 << 20) || !compact_batchable((int)rowb)) return kDoneNothing;
  bool tail = a0->mode != PAFU_MODE_SINGLE && a0->kv_dtype == PAFU_BF16;
  for (int l = 1; l < n_layers; ++l) {
    const pafu_step_args* a = &args[l];
    if (a->n != a0->n || a->k != a0->k || a->N != a0->N || a->D != a0->D || a->kv_dtype != a0->kv_dtype ||
        a->ld_cache != a0->ld_cache || a->ld_out != a0->ld_out)
      return kDoneNothing;
    if (a->mode != a0->mode || a->Lc != a0->Lc || a->ld_chunk != a0->ld_chunk) tail = false;
  }
  const int n_kept = a0->k < a0->n ? a0->k : a0->n;
  CompactLayer layers[kCompactBatchMax];
  for (int first = 0; first < n_layers; first += kCompactBatchMax) {
    const int m = n_layers - first < kCompactBatchMax ? n_layers - first : kCompactBatchMax;
    for (int i = 0; i < m; ++i) {
      const pafu_step_args* a = &args[first + i];
      const bool with_scores = score_layer < 0 || first + i == score_layer;
      const float* sel = a->mode == PAFU_MODE_SINGLE ? a->scores : a->SL_in;
      layers[i] = CompactLayer{static_cast<const char*>(a->K_cache), static_cast<const char*>(a->V_cache),
                               static_cast<char*>(a->K_out), static_cast<char*>(a->V_out),
                               shared_ids ? shared_ids : a->ids, with_scores ? sel : nullptr,
                               with_scores ? a->SL_out : nullptr, static_cast<const char*>(a->K_chunk),
                               static_cast<const char*>(a->V_chunk)};
    }
    *rc_out = launch_compact_batch(st, layers, m, a0->ld_cache * kvb, a0->n, n_kept, (int)rowb, a0->ld_out * kvb,
                                   tail ? a0->Lc : 0, (long long)a0->ld_chunk * 2);
    if (*rc_out) return kDoneCompact;
  }
  return tail ? (kDoneCompact | kDoneAppend) : kDoneCompact;
}

// Validates the cache part of a layer that takes its indices from another layer.
int check_layer_kv(const pafu_step_args* a, const pafu_step_args* idx) {
  if (!a) return PAFU_ERR_NULL;
  if (a->mode != idx->mode || a->n != idx->n || a->k != idx->k || a->Lc != idx->Lc) return PAFU_ERR_SHAPE;
  if (a->N < 1 || a->D < 1) return PAFU_ERR_SHAPE;
  const int n_kept = a->k < a->n ? a->k : a->n;
  if (a->kv_dtype != PAFU_BF16 && a->kv_dtype != PAFU_FP8_E4M3) return PAFU_ERR_DTYPE;
  int rc = check_compact(a->K_cache, a->V_cache, nullptr, a->ld_cache, a->n, idx->ids, n_kept, a->N, a->D, a->kv_dtype,
                         a->K_out, a->V_out, nullptr, a->ld_out);
  if (rc) return rc;
  rc = check_layer_attention(a, n_kept);
  if (rc) return rc;
  if (a->mode != PAFU_MODE_SINGLE) {
    if (!a->K_out || !a->V_out) return PAFU_ERR_NULL;
    if (!aligned16(a->K_out) || !aligned16(a->V_out) || (a->ld_out * kv_dtype_bytes(a->kv_dtype)) % 16 != 0)
      return PAFU_ERR_ALIGN;
    if (a->ld_out < (long long)a->N * a->D) return PAFU_ERR_SHAPE;
  }
  return check_step_alias(a, false);
}

}  // namespace
}  // namespace pafu

using namespace pafu;

extern "C" {

const char* pafu_strerror(int status) {
  switch (status) {
    case PAFU_OK: return "ok";
    case PAFU_ERR_NULL: return "a required pointer is NULL";
    case PAFU_ERR_SHAPE: return "invalid or unsupported size";
    case PAFU_ERR_DTYPE: return "unsupported dtype";
    case PAFU_ERR_ALIGN: return "pointer or stride not 16-byte aligned";
    case PAFU_ERR_WORKSPACE: return "workspace missing or too small";
    case PAFU_ERR_ALIAS: return "output overlaps an input";
    case PAFU_ERR_HIP: return "a HIP call failed";
    default: return "unknown status";
  }
}

int pafu_last_hip_error(void) { return g_last_hip_error; }
int pafu_version(void) { return 3; }

int pafu_study_build(void) { return attention_study_build(); }

int pafu_launch_probe(void* stream) {
  hipLaunchKernelGGL(probe_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream));
  return check_launch();
}

size_t pafu_score_workspace_bytes(int M) { return M > 0 ? ((size_t)M + 1) * sizeof(float) : 0; }

int pafu_score(void* stream, const void* x0, const void* x1, const void* x2, int n_seg, int T, int Fs, long long ld_x,
               int x_dtype, const void* W1, const float* b1, const float* W2, const float* b2, int M, int n_out,
               int act, float* out, void* workspace, size_t workspace_bytes) {
  int rc = check_score(x0, x1, x2, n_seg, T, Fs, ld_x, x_dtype, W1, W2, M, n_out, act, out, workspace, workspace_bytes);
  if (rc) return rc;
  return launch_score(static_cast<hipStream_t>(stream), x0, x1, x2, n_seg, T, Fs, ld_x, x_dtype, W1, b1, W2, b2, M,
                      n_out, act, out, workspace);
}

int pafu_score_static(void* stream, const void* x0, const void* x1, const void* x2, int n_seg, int T, int Fs,
                      long long ld_x, int x_dtype, const void* W1, const float* b1, const float* W2, const float* b2,
                      int M, int n_out, int act, float* out) {
  // same validation as pafu_score, with the library's own scratch standing in for the workspace
  int rc = check_score(x0, x1, x2, n_seg, T, Fs, ld_x, x_dtype, W1, W2, M, n_out, act, out, nullptr, SIZE_MAX);
  if (rc) return rc;
  if (M > PAFU_SCORE_STATIC_MAX_M) return PAFU_ERR_WORKSPACE;
  return launch_score_static(static_cast<hipStream_t>(stream), x0, x1, x2, n_seg, T, Fs, ld_x, x_dtype, W1, b1, W2, b2,
                             M, n_out, act, out);
}

size_t pafu_select_workspace_bytes(int n) {
  (void)n;
  return 0;
}

int pafu_select_topk(void* stream, const float* scores, int n, int k, int* out_ids, int* out_count, void* workspace,
                     size_t workspace_bytes) {
  (void)workspace_bytes;
  int rc = check_select(scores, n, k, out_ids);
  if (rc) return rc;
  return launch_select(static_cast<hipStream_t>(stream), scores, n, k, 0, out_ids, out_count, workspace);
}

int pafu_select_topk_pinned(void* stream, const float* scores, int n, int k, int n_pinned, int* out_ids,
                            int* out_count, void* workspace, size_t workspace_bytes) {
  (void)workspace_bytes;
  if (n_pinned < 0) return PAFU_ERR_SHAPE;
  int rc = check_select(scores, n, k, out_ids);
  if (rc) return rc;
  return launch_select(static_cast<hipStream_t>(stream), scores, n, k, n_pinned, out_ids, out_count, workspace);
}

int pafu_compact_kv(void* stream, const void* K, const void* V, const float* SL, long long ld_in, int n, const int* ids,
                    int count, int N, int D, int dtype, void* K_out, void* V_out, float* SL_out, long long ld_out) {
  int rc = check_compact(K, V, SL, ld_in, n, ids, count, N, D, dtype, K_out, V_out, SL_out, ld_out);
  if (rc) return rc;
  const int eb = kv_dtype_bytes(dtype);
  return launch_compact(static_cast<hipStream_t>(stream), K, V, SL, ld_in * eb, n, ids, count, N * D * eb, K_out, V_out,
                        SL_out, ld_out * eb);
}

int pafu_quantize_kv(void* stream, const void* K, const void* V, long long ld_in, int rows, int N, int D,
                     int k_scale_log2, int v_scale_log2, void* K_q, void* V_q, long long ld_out) {
  int rc = check_quant(K, V, ld_in, rows, N, D, k_scale_log2, v_scale_log2, K_q, V_q, ld_out, false);
  if (rc) return rc;
  return launch_quantize(static_cast<hipStream_t>(stream), K, V, ld_in * 2, rows, N * D, k_scale_log2, v_scale_log2, K_q,
                         V_q, ld_out);
}

int pafu_dequantize_kv(void* stream, const void* K_q, const void* V_q, long long ld_in, int rows, int N, int D,
                       int k_scale_log2, int v_scale_log2, void* K, void* V, long long ld_out) {
  int rc = check_quant(K, V, ld_out, rows, N, D, k_scale_log2, v_scale_log2, K_q, V_q, ld_in, true);
  if (rc) return rc;
  return launch_dequantize(static_cast<hipStream_t>(stream), K_q, V_q, ld_in, rows, N * D, k_scale_log2, v_scale_log2, K,
                           V, ld_out * 2);
}

int pafu_chunk_attention_fp8(void* stream, const void* Q, int Lq, const void* Kc_q, const void* Vc_q, int n_kept,
                             const void* Kn_q, const void* Vn_q, int Lc, int N, int D, long long ld_q, long long ld_c,
                             long long ld_n, long long ld_o, int block_len, float softmax_scale, int k_scale_log2,
                             int v_scale_log2, void* O, int out_dtype, void* workspace, size_t workspace_bytes) {
  if (D != 128) return PAFU_ERR_SHAPE;  // the 8-bit tile path is built for head dim 128
  if (!scale_ok(k_scale_log2) || !scale_ok(v_scale_log2)) return PAFU_ERR_SHAPE;
  int rc = check_attention(Q, Lq, Kc_q, Vc_q, n_kept, Kn_q, Vn_q, Lc, N, D, ld_q, ld_c, ld_n, ld_o, block_len, O,
                           out_dtype, 1);
  if (rc) return rc;
  if (workspace != nullptr && workspace_bytes > 0 && !aligned16(workspace)) return PAFU_ERR_ALIGN;
  const float scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)D);
  return launch_attention(static_cast<hipStream_t>(stream), Q, Lq, Kc_q, Vc_q, n_kept, Kn_q, Vn_q, Lc, N, D, ld_q, ld_c,
                          ld_n, ld_o, block_len, scale, O, out_dtype, workspace, workspace_bytes, nullptr, 0,
                          PAFU_FP8_E4M3, ldexpf(1.0f, k_scale_log2), ldexpf(1.0f, v_scale_log2));
}

int pafu_compact_kv_counted(void* stream, const void* K, const void* V, const float* SL, long long ld_in, int n,
                            const int* ids, const int* count, int max_count, int N, int D, int dtype, void* K_out,
                            void* V_out, float* SL_out, long long ld_out) {
  if (max_count > 0 && count == nullptr) return PAFU_ERR_NULL;
  int rc = check_compact(K, V, SL, ld_in, n, ids, max_count, N, D, dtype, K_out, V_out, SL_out, ld_out);
  if (rc) return rc;
  const int eb = kv_dtype_bytes(dtype);
  return launch_compact(static_cast<hipStream_t>(stream), K, V, SL, ld_in * eb, n, ids, max_count, N * D * eb, K_out,
                        V_out, SL_out, ld_out * eb, count);
}

size_t pafu_attention_workspace_bytes(int Lq, int N, int D) {
  (void)Lq; (void)N;
  return (D == 64 || D == 128) ? attention_workspace_bytes(D) : 0;
}

int pafu_chunk_attention(void* stream, const void* Q, int Lq, const void* Kc, const void* Vc, int n_kept, const void* Kn,
                         const void* Vn, int Lc, int N, int D, long long ld_q, long long ld_c, long long ld_n,
                         long long ld_o, int block_len, float softmax_scale, void* O, int out_dtype, void* workspace,
                         size_t workspace_bytes) {
  int rc = check_attention(Q, Lq, Kc, Vc, n_kept, Kn, Vn, Lc, N, D, ld_q, ld_c, ld_n, ld_o, block_len, O, out_dtype);
  if (rc) return rc;
  rc = check_attention_ws(workspace, workspace_bytes, Q, Lq, Kc, Vc, n_kept, Kn, Vn, Lc, ld_q, ld_c, ld_n, ld_o, O,
                          out_dtype);
  if (rc) return rc;
  const float scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)D);
  return launch_attention(static_cast<hipStream_t>(stream), Q, Lq, Kc, Vc, n_kept, Kn, Vn, Lc, N, D, ld_q, ld_c, ld_n,
                          ld_o, block_len, scale, O, out_dtype, workspace, workspace_bytes);
}

int pafu_chunk_attention_gather(void* stream, const void* Q, int Lq, const void* K_cache, const void* V_cache,
                                int n_cache, const int* ids, int n_kept, const void* Kn, const void* Vn, int Lc, int N,
                                int D, long long ld_q, long long ld_c, long long ld_n, long long ld_o, int block_len,
                                float softmax_scale, void* O, int out_dtype, void* workspace,
                                size_t workspace_bytes) {
  if (n_cache < 0 || n_kept < 0 || n_kept > n_cache) return PAFU_ERR_SHAPE;
  if (n_kept > 0 && !ids) return PAFU_ERR_NULL;
  if (!aligned16(ids)) return PAFU_ERR_ALIGN;
  // the kernel addresses gathered rows by 32-bit byte offsets from the head's base
  if ((long long)n_cache * ld_c * 2 >= (1ll << 32)) return PAFU_ERR_SHAPE;
  // the retained rows are a subset of the cache: validate the cache extent (alias check included) with the
  // checker of the plain call
  int rc = check_attention(Q, Lq, K_cache, V_cache, n_cache, Kn, Vn, Lc, N, D, ld_q, ld_c, ld_n, ld_o, block_len, O,
                           out_dtype);
  if (rc) return rc;
  rc = check_attention_ws(workspace, workspace_bytes, Q, Lq, K_cache, V_cache, n_cache, Kn, Vn, Lc, ld_q, ld_c, ld_n,
                          ld_o, O, out_dtype);
  if (rc) return rc;
  const float scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)D);
  return launch_attention(static_cast<hipStream_t>(stream), Q, Lq, K_cache, V_cache, n_kept, Kn, Vn, Lc, N, D, ld_q,
                          ld_c, ld_n, ld_o, block_len, scale, O, out_dtype, workspace, workspace_bytes, ids, n_cache);
}

size_t pafu_sse_workspace_bytes(int L, int N) { return L > 0 && N > 0 ? sse_workspace_bytes(L, N) : 0; }

int pafu_sse_score(void* stream, const void* Q, const void* K, int L, int N, int D, long long ld_q, long long ld_k,
                   int block_len, float softmax_scale, float* out, void* workspace, size_t workspace_bytes) {
  if (L < 0 || N < 1 || block_len < 1) return PAFU_ERR_SHAPE;
  if (((long long)L / 32 + 1) * N > 0x7fffffffll) return PAFU_ERR_SHAPE;  // one-dimensional grid
  if (D != 64 && D != 128) return PAFU_ERR_SHAPE;
  if (L == 0) return PAFU_OK;
  if (!Q || !K || !out) return PAFU_ERR_NULL;
  const long long row = (long long)N * D;
  if (ld_q < row || ld_k < row) return PAFU_ERR_SHAPE;
  // rows are addressed by 32-bit byte offsets from the head's base
  if ((long long)L * ld_q * 2 >= (1ll << 32) || (long long)L * ld_k * 2 >= (1ll << 32)) return PAFU_ERR_SHAPE;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(out) || !aligned16(workspace) || (ld_q * 2) % 16 != 0 ||
      (ld_k * 2) % 16 != 0)
    return PAFU_ERR_ALIGN;
  if (!workspace || workspace_bytes < sse_workspace_bytes(L, N)) return PAFU_ERR_WORKSPACE;
  const size_t o_bytes = (size_t)L * 4;
  if (overlaps(out, o_bytes, Q, (size_t)L * ld_q * 2) || overlaps(out, o_bytes, K, (size_t)L * ld_k * 2) ||
      overlaps(out, o_bytes, workspace, workspace_bytes) ||
      overlaps(workspace, workspace_bytes, Q, (size_t)L * ld_q * 2) ||
      overlaps(workspace, workspace_bytes, K, (size_t)L * ld_k * 2))
    return PAFU_ERR_ALIAS;
  const float scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)D);
  return launch_sse(static_cast<hipStream_t>(stream), Q, K, L, N, D, ld_q, ld_k, block_len, scale, out, workspace);
}

size_t pafu_step_workspace_bytes(const pafu_step_args* a) {
  if (!a) return 0;
  return step_score_workspace(a) + attention_workspace_bytes(a->D);
}

int pafu_step(void* stream, const pafu_step_args* args) {
  int rc = check_step(args);
  if (rc) return rc;
  return enqueue_step(static_cast<hipStream_t>(stream), args);
}

int pafu_step_layers(void* stream, const pafu_step_args* args, int n_layers) {
  if (n_layers < 0) return PAFU_ERR_SHAPE;
  if (n_layers > 0 && !args) return PAFU_ERR_NULL;
  for (int l = 0; l < n_layers; ++l) {  // validate every layer before enqueuing any
    int rc = check_step(&args[l]);
    if (rc) return rc;
  }
  {
    int rc = check_layers_alias(args, n_layers, -1);
    if (rc) return rc;
  }
  // The layers are independent, so the order of their stages is free: all scores first, then every layer's selection
  // in one launch (a selection occupies a single CU; one per layer in a row would leave the chip idle 30 times), then
  // compaction and attention layer by layer.
  hipStream_t st = static_cast<hipStream_t>(stream);
  for (int l = 0; l < n_layers; ++l) {
    int rc = enqueue_scores(st, &args[l]);
    if (rc) return rc;
  }
  for (int first = 0; first < n_layers; first += kSelectBatchMax) {
    SelectJob jobs[kSelectBatchMax];
    int m = 0;
    for (int l = first; l < n_layers && l < first + kSelectBatchMax; ++l) {
      const pafu_step_args* a = &args[l];
      if (a->n <= 0) continue;
      jobs[m++] = SelectJob{a->mode == PAFU_MODE_SINGLE ? a->scores : a->SL_in, a->ids, nullptr, a->n, a->k, a->n_pinned};
    }
    if (m > 0) {
      int rc = launch_select_batch(st, jobs, m);
      if (rc) return rc;
    }
  }
  if (n_layers > 0) {  // the one "after selection" event of the step
    int rc = record_stage(st, &args[0], 2);
    if (rc) return rc;
  }
  int rc_batch;
  const int done = enqueue_compact_batch(st, args, n_layers, nullptr, -1, &rc_batch);
  if (rc_batch) return rc_batch;
  for (int l = 0; l < n_layers; ++l) {
    const pafu_step_args* a = &args[l];
    const WsPart ws = attention_ws(a, true);
    int rc = enqueue_kv(st, a, a->ids, a->mode == PAFU_MODE_SINGLE ? a->scores : a->SL_in, a->SL_out, ws.p, ws.bytes,
                        done);
    if (rc) return rc;
  }
  return PAFU_OK;
}

int pafu_step_layers_shared(void* stream, const pafu_step_args* args, int n_layers, int index_layer) {
  if (n_layers < 1 || index_layer < 0 || index_layer >= n_layers) return PAFU_ERR_SHAPE;
  if (!args) return PAFU_ERR_NULL;
  const pafu_step_args* idx = &args[index_layer];
  int rc = check_step(idx);
  if (rc) return rc;
  for (int l = 0; l < n_layers; ++l) {  // validate every layer before enqueuing anything
    if (l == index_layer) continue;
    rc = check_layer_kv(&args[l], idx);
    if (rc) return rc;
  }
  rc = check_layers_alias(args, n_layers, index_layer);
  if (rc) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  // ROLLOUT selects on the stored list, so the indices exist before any layer runs; the chunk's own scores are only
  // needed for the append.  SINGLE scores first.  Either way: scores, one selection, then every layer's cache.
  bool selected = false;
  rc = enqueue_scores(st, idx, &selected);
  if (rc) return rc;
  const float* sel_scores = idx->mode == PAFU_MODE_SINGLE ? idx->scores : idx->SL_in;
  if (idx->n > 0 && !selected) {
    rc = launch_select(st, sel_scores, idx->n, idx->k, idx->n_pinned, idx->ids, nullptr, nullptr);
    if (rc) return rc;
  }
  rc = record_stage(st, idx, 2);
  if (rc) return rc;
  // every layer's cache is compacted to the one index list in one launch (per 32 layers) when the layers share the
  // cache geometry, otherwise layer by layer
  int rc_batch;
  const int done = enqueue_compact_batch(st, args, n_layers, idx->ids, index_layer, &rc_batch);
  if (rc_batch) return rc_batch;
  for (int l = 0; l < n_layers; ++l) {
    const bool is_idx = l == index_layer;
    // a layer without a workspace of its own borrows the index layer's (the layers run one after the other)
    WsPart ws = attention_ws(&args[l], is_idx);
    if (ws.p == nullptr) ws = attention_ws(idx, true);
    rc = enqueue_kv(st, &args[l], idx->ids, is_idx ? sel_scores : nullptr, is_idx ? idx->SL_out : nullptr, ws.p,
                    ws.bytes, done);
    if (rc) return rc;
  }
  return PAFU_OK;
}

}  // extern "C"

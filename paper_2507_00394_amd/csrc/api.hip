// C-ABI entry points (see include/helix_attn.h).  Everything here is host code: argument
// validation first, with no HIP call before it succeeds, then kernel launches on the
// caller's stream.  Nothing is allocated, freed or synchronised.
#include "../../include/helix_attn.h"
#include "kernels.hpp"

#include <cmath>
#include <cstdint>
#include <initializer_list>
#include <mutex>
#include <utility>

namespace {

// Statistics planes of helix_attn_bwd_static: device memory that exists once per GPU for the
// life of the process, so that the call allocates nothing.  In host code the array's name is
// only a handle: the per-device address comes from hipGetSymbolAddress (scratch_base below).
constexpr size_t kScratchBytes = HELIX_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kVersion = 300;  // 0.3.0: backward stages share one statistics workspace; probes; allocation-free backward

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

int check_shape(int B, int H, int S, int D) {
  if (B < 1 || H < 1 || S < 1 || D < 1) return HELIX_ERR_BAD_SHAPE;
  if (D != 64 && D != 128) return HELIX_ERR_UNSUPPORTED_HEAD_DIM;
  const long long bh = (long long)B * H;
  if (bh > 0x7fffffffLL / 8) return HELIX_ERR_BAD_SHAPE;          // workgroup ids stay in int
  if (S > (1 << 24)) return HELIX_ERR_BAD_SHAPE;                  // in-head offsets stay in 32 bits
  if ((double)bh * S * D >= 1099511627776.0) return HELIX_ERR_BAD_SHAPE;  // 2^40 elements
  const long long tiles = (long long)((S + 63) / 64 + 8) * 8 * bh;
  if (tiles > 0x7fffffffLL) return HELIX_ERR_BAD_SHAPE;           // grid size limit
  return HELIX_OK;
}

int check_scale(float scale) { return (std::isfinite(scale) && scale > 0.f) ? HELIX_OK : HELIX_ERR_BAD_SCALE; }

template <typename... P>
int check_bf16_ptrs(P... ptrs) {
  const void* a[] = {ptrs...};
  for (const void* p : a) if (!p) return HELIX_ERR_NULL_POINTER;
  for (const void* p : a) if (!aligned(p, 16)) return HELIX_ERR_MISALIGNED;
  return HELIX_OK;
}
template <typename... P>
int check_f32_ptrs(P... ptrs) {
  const void* a[] = {ptrs...};
  for (const void* p : a) if (!p) return HELIX_ERR_NULL_POINTER;
  for (const void* p : a) if (!aligned(p, 4)) return HELIX_ERR_MISALIGNED;
  return HELIX_OK;
}

// Strides of a [B, H, S, D] view (NULL: contiguous).  Accepted: multiples of 8 elements, so
// that every row starts on a 16-byte boundary, and "nested": ordered by stride, each
// dimension steps over the whole extent of the next smaller one (rows over D), which holds
// for any permutation of the dimensions of a dense or padded buffer and rules out overlap.
int to_map(const helix_strides* st, int B, int H, int S, int D, helix::TensorMap* out) {
  if (!st) { *out = helix::contiguous_map(H, S, D); return HELIX_OK; }
  struct Dim { long long stride; long long extent; };
  Dim d[3] = {{st->batch, B}, {st->head, H}, {st->row, S}};
  for (const Dim& x : d) if (x.stride < 0 || (x.stride & 7)) return HELIX_ERR_BAD_STRIDE;
  if (st->row < D || st->row > (1 << 24)) return HELIX_ERR_BAD_STRIDE;   // tile-relative byte offsets stay in 32 bits
  for (int i = 0; i < 3; i++)
    for (int j = i + 1; j < 3; j++)
      if (d[j].stride < d[i].stride) { Dim t = d[i]; d[i] = d[j]; d[j] = t; }
  long long span = D;   // elements covered by the dimensions handled so far
  for (const Dim& x : d) {
    if (x.extent == 1) continue;
    if (x.stride < span) return HELIX_ERR_BAD_STRIDE;
    if ((double)x.stride * (double)x.extent >= 1099511627776.0) return HELIX_ERR_BAD_STRIDE;   // 2^40 elements
    span = x.stride * x.extent;
  }
  *out = helix::TensorMap{st->batch, st->head, (int)st->row};
  return HELIX_OK;
}

helix::FwdMaps contiguous_fwd(int H, int S, int D) {
  const helix::TensorMap m = helix::contiguous_map(H, S, D);
  return helix::FwdMaps{m, m, m, m};
}
helix::BwdMaps contiguous_bwd(int H, int S, int D) {
  const helix::TensorMap m = helix::contiguous_map(H, S, D);
  return helix::BwdMaps{m, m, m, m, m, m, m, m};
}

// The backward's row statistics: two fp32 planes [B, H, S], each padded to 256 bytes:
// plane 0 = -delta = -rowsum(dO o O), plane 1 = lse * log2(e).
size_t stats_plane_bytes(int B, int H, int S) { return ((size_t)B * H * S * sizeof(float) + 255) & ~(size_t)255; }
float* neg_delta_plane(void* stats) { return static_cast<float*>(stats); }
float* lse2_plane(void* stats, int B, int H, int S) { return reinterpret_cast<float*>(static_cast<char*>(stats) + stats_plane_bytes(B, H, S)); }
int check_stats(const void* stats) {
  if (!stats) return HELIX_ERR_NULL_POINTER;
  return aligned(stats, 256) ? HELIX_OK : HELIX_ERR_MISALIGNED;
}

int run_bwd(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dO,
            void* dq, void* dk, void* dv, void* stats, const helix::BwdMaps& maps,
            int B, int H, int S, int D, float scale, int causal, hipStream_t st);

// Shapes and leading dimensions of the linear layer; `need_m32`: the product contracts over M.
int check_linear(int M, int K, int N, bool need_m32, std::initializer_list<std::pair<long long, int>> lds) {
  if (M < 1 || K < 1 || N < 1) return HELIX_ERR_BAD_SHAPE;
  if ((K & 127) || (N & 127) || (need_m32 && (M & 31))) return HELIX_ERR_BAD_SHAPE;
  if (K > (1 << 20) || N > (1 << 20) || (long long)((M + 255) / 256 + 8) * ((N > K ? N : K) / 128) > 0x7fffffffLL / 8) return HELIX_ERR_BAD_SHAPE;
  for (const auto& ld : lds)
    // 255 rows of a stage tile times the row pitch in bytes stays below 2^31: lane offsets of the copies fit 32 bits with room to spare
    if (ld.first < ld.second || (ld.first & 7) || ld.first > (1 << 22)) return HELIX_ERR_BAD_STRIDE;
  return HELIX_OK;
}

int launched(hipError_t e) { return e == hipSuccess ? HELIX_OK : HELIX_ERR_LAUNCH; }

// Address of `scratch` on the current device, looked up once per device.
void* scratch_base() {
  constexpr int kMaxDevices = 64;
  static void* base[kMaxDevices] = {};
  static std::mutex lock;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> guard(lock);
  if (!base[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    base[dev] = p;
  }
  return base[dev];
}

#define HELIX_TRY(expr) do { int st_ = (expr); if (st_ != HELIX_OK) return st_; } while (0)

}  // namespace

extern "C" {

int helix_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                   int B, int H, int S, int D, float scale, int causal, void* stream) {
  HELIX_TRY(check_bf16_ptrs(q, k, v, (const void*)o));
  HELIX_TRY(check_f32_ptrs((const void*)lse));
  HELIX_TRY(check_shape(B, H, S, D));
  HELIX_TRY(check_scale(scale));
  return launched(helix::launch_fwd(q, k, v, o, lse, contiguous_fwd(H, S, D), B, H, S, D, scale, causal != 0, (hipStream_t)stream));
}

int helix_attn_check_strides(const helix_strides* strides, int B, int H, int S, int D) {
  HELIX_TRY(check_shape(B, H, S, D));
  helix::TensorMap m;
  return to_map(strides, B, H, S, D, &m);
}

int helix_attn_fwd_strided(const void* q, const helix_strides* q_strides, const void* k, const helix_strides* k_strides,
                           const void* v, const helix_strides* v_strides, void* o, const helix_strides* o_strides,
                           float* lse, int B, int H, int S, int D, float scale, int causal, void* stream) {
  HELIX_TRY(check_bf16_ptrs(q, k, v, (const void*)o));
  HELIX_TRY(check_f32_ptrs((const void*)lse));
  HELIX_TRY(check_shape(B, H, S, D));
  HELIX_TRY(check_scale(scale));
  helix::FwdMaps m;
  HELIX_TRY(to_map(q_strides, B, H, S, D, &m.q));
  HELIX_TRY(to_map(k_strides, B, H, S, D, &m.k));
  HELIX_TRY(to_map(v_strides, B, H, S, D, &m.v));
  HELIX_TRY(to_map(o_strides, B, H, S, D, &m.o));
  return launched(helix::launch_fwd(q, k, v, o, lse, m, B, H, S, D, scale, causal != 0, (hipStream_t)stream));
}

size_t helix_attn_bwd_workspace_bytes(int B, int H, int S, int D) {
  if (check_shape(B, H, S, D) != HELIX_OK) return 0;
  return 2 * stats_plane_bytes(B, H, S);
}

int helix_attn_bwd_preprocess(const void* o, const void* dO, const float* lse, void* stats,
                              int B, int H, int S, int D, void* stream) {
  HELIX_TRY(check_bf16_ptrs(o, dO));
  HELIX_TRY(check_f32_ptrs((const void*)lse));
  HELIX_TRY(check_stats(stats));
  HELIX_TRY(check_shape(B, H, S, D));
  return launched(helix::launch_bwd_preprocess(o, dO, lse, neg_delta_plane(stats), lse2_plane(stats, B, H, S),
                                               contiguous_bwd(H, S, D), B, H, S, D, (hipStream_t)stream));
}

int helix_attn_bwd_delta_head(const void* q, const void* k, const void* v, const void* dO,
                              const float* lse, void* stats, int rows,
                              int B, int H, int S, int D, float scale, int causal, void* stream) {
  HELIX_TRY(check_bf16_ptrs(q, k, v, dO));
  HELIX_TRY(check_f32_ptrs((const void*)lse));
  HELIX_TRY(check_stats(stats));
  HELIX_TRY(check_shape(B, H, S, D));
  HELIX_TRY(check_scale(scale));
  if (rows < 0) return HELIX_ERR_BAD_SHAPE;
  return launched(helix::launch_bwd_delta_head(q, k, v, dO, lse, neg_delta_plane(stats), contiguous_bwd(H, S, D), B, H, S, D, rows, scale, causal != 0, (hipStream_t)stream));
}

int helix_attn_bwd_dkdv(const void* q, const void* k, const void* v, const void* dO,
                        const void* stats, void* dk, void* dv,
                        int B, int H, int S, int D, float scale, int causal, void* stream) {
  HELIX_TRY(check_bf16_ptrs(q, k, v, dO, (const void*)dk, (const void*)dv));
  HELIX_TRY(check_stats(stats));
  HELIX_TRY(check_shape(B, H, S, D));
  HELIX_TRY(check_scale(scale));
  void* st = const_cast<void*>(stats);
  return launched(helix::launch_bwd_dkdv(q, k, v, dO, lse2_plane(st, B, H, S), neg_delta_plane(st), dk, dv, contiguous_bwd(H, S, D), B, H, S, D, scale, causal != 0, (hipStream_t)stream));
}

int helix_attn_bwd_dq(const void* q, const void* k, const void* v, const void* dO,
                      const void* stats, void* dq,
                      int B, int H, int S, int D, float scale, int causal, void* stream) {
  HELIX_TRY(check_bf16_ptrs(q, k, v, dO, (const void*)dq));
  HELIX_TRY(check_stats(stats));
  HELIX_TRY(check_shape(B, H, S, D));
  HELIX_TRY(check_scale(scale));
  void* st = const_cast<void*>(stats);
  return launched(helix::launch_bwd_dq(q, k, v, dO, lse2_plane(st, B, H, S), neg_delta_plane(st), dq, contiguous_bwd(H, S, D), B, H, S, D, scale, causal != 0, (hipStream_t)stream));
}

int helix_attn_bwd(const void* q, const void* k, const void* v, const void* o, const float* lse,
                   const void* dO, void* dq, void* dk, void* dv,
                   void* workspace, size_t workspace_bytes,
                   int B, int H, int S, int D, float scale, int causal, void* stream) {
  HELIX_TRY(check_bf16_ptrs(q, k, v, o, dO, (const void*)dq, (const void*)dk, (const void*)dv));
  HELIX_TRY(check_f32_ptrs((const void*)lse));
  HELIX_TRY(check_shape(B, H, S, D));
  HELIX_TRY(check_scale(scale));
  if (!workspace) return HELIX_ERR_NULL_POINTER;
  if (!aligned(workspace, 256)) return HELIX_ERR_MISALIGNED;
  if (workspace_bytes < helix_attn_bwd_workspace_bytes(B, H, S, D)) return HELIX_ERR_WORKSPACE;
  return run_bwd(q, k, v, o, lse, dO, dq, dk, dv, workspace, contiguous_bwd(H, S, D),
                 B, H, S, D, scale, causal, (hipStream_t)stream);
}

int helix_attn_bwd_static(const void* q, const void* k, const void* v, const void* o, const float* lse,
                          const void* dO, void* dq, void* dk, void* dv,
                          int B, int H, int S, int D, float scale, int causal, void* stream) {
  HELIX_TRY(check_bf16_ptrs(q, k, v, o, dO, (const void*)dq, (const void*)dk, (const void*)dv));
  HELIX_TRY(check_f32_ptrs((const void*)lse));
  HELIX_TRY(check_shape(B, H, S, D));
  HELIX_TRY(check_scale(scale));
  if (helix_attn_bwd_workspace_bytes(B, H, S, D) > kScratchBytes) return HELIX_ERR_SCRATCH_LIMIT;
  void* stats = scratch_base();
  if (!stats) return HELIX_ERR_LAUNCH;
  return run_bwd(q, k, v, o, lse, dO, dq, dk, dv, stats, contiguous_bwd(H, S, D), B, H, S, D, scale, causal,
                 (hipStream_t)stream);
}

int helix_attn_bwd_strided(const void* q, const helix_strides* q_strides, const void* k, const helix_strides* k_strides,
                           const void* v, const helix_strides* v_strides, const void* o, const helix_strides* o_strides,
                           const float* lse, const void* dO, const helix_strides* dO_strides,
                           void* dq, const helix_strides* dq_strides, void* dk, const helix_strides* dk_strides,
                           void* dv, const helix_strides* dv_strides, void* workspace, size_t workspace_bytes,
                           int B, int H, int S, int D, float scale, int causal, void* stream) {
  HELIX_TRY(check_bf16_ptrs(q, k, v, o, dO, (const void*)dq, (const void*)dk, (const void*)dv));
  HELIX_TRY(check_f32_ptrs((const void*)lse));
  HELIX_TRY(check_shape(B, H, S, D));
  HELIX_TRY(check_scale(scale));
  if (!workspace) return HELIX_ERR_NULL_POINTER;
  if (!aligned(workspace, 256)) return HELIX_ERR_MISALIGNED;
  if (workspace_bytes < helix_attn_bwd_workspace_bytes(B, H, S, D)) return HELIX_ERR_WORKSPACE;
  helix::BwdMaps m;
  HELIX_TRY(to_map(q_strides, B, H, S, D, &m.q));
  HELIX_TRY(to_map(k_strides, B, H, S, D, &m.k));
  HELIX_TRY(to_map(v_strides, B, H, S, D, &m.v));
  HELIX_TRY(to_map(o_strides, B, H, S, D, &m.o));
  HELIX_TRY(to_map(dO_strides, B, H, S, D, &m.dO));
  HELIX_TRY(to_map(dq_strides, B, H, S, D, &m.dq));
  HELIX_TRY(to_map(dk_strides, B, H, S, D, &m.dk));
  HELIX_TRY(to_map(dv_strides, B, H, S, D, &m.dv));
  return run_bwd(q, k, v, o, lse, dO, dq, dk, dv, workspace, m, B, H, S, D, scale, causal,
                 (hipStream_t)stream);
}

int helix_qkv_linear_fwd(const void* a, long long lda, const void* w, long long ldw, void* qkv, long long ldqkv,
                         int M, int K, int N, void* stream) {
  HELIX_TRY(check_bf16_ptrs(a, w, (const void*)qkv));
  HELIX_TRY(check_linear(M, K, N, false, {{lda, K}, {ldw, N}, {ldqkv, N}}));
  return launched(helix::launch_linear_fwd(a, lda, w, ldw, qkv, ldqkv, M, K, N, (hipStream_t)stream));
}

size_t helix_qkv_linear_bwd_workspace_bytes(int M, int K, int N) {
  if (check_linear(M, K, N, true, {}) != HELIX_OK) return 0;
  return (helix::linear_bwd_workspace_bytes(M, K, N) + 255) & ~(size_t)255;
}

int helix_qkv_linear_bwd(const void* a, long long lda, const void* w, long long ldw, const void* dqkv, long long lddqkv,
                         void* da, long long ldda, float* dw, long long lddw, void* workspace, size_t workspace_bytes,
                         int M, int K, int N, void* stream) {
  HELIX_TRY(check_bf16_ptrs(a, w, dqkv, (const void*)da, (const void*)dw));
  HELIX_TRY(check_linear(M, K, N, true, {{lda, K}, {ldw, N}, {lddqkv, N}, {ldda, K}, {lddw, N}}));
  if (!workspace) return HELIX_ERR_NULL_POINTER;
  if (!aligned(workspace, 256)) return HELIX_ERR_MISALIGNED;
  if (workspace_bytes < helix_qkv_linear_bwd_workspace_bytes(M, K, N)) return HELIX_ERR_WORKSPACE;
  char* ws = static_cast<char*>(workspace);
  HELIX_TRY(launched(helix::launch_linear_bwd_input(dqkv, lddqkv, w, ldw, da, ldda, ws, M, K, N, (hipStream_t)stream)));
  return launched(helix::launch_linear_bwd_weight(a, lda, dqkv, lddqkv, dw, lddw,
                                                  reinterpret_cast<float*>(ws + helix::linear_bwd_wt_bytes(K, N)), M, K, N,
                                                  (hipStream_t)stream));
}

int helix_mfma_probe(float* sink, int workgroups, int iters, int random_operands, long long* flops, void* stream) {
  if (!sink || !flops) return HELIX_ERR_NULL_POINTER;
  if (!aligned(sink, 4)) return HELIX_ERR_MISALIGNED;
  if (workgroups < 1 || iters < 1 || workgroups > (1 << 20) || iters > (1 << 24)) return HELIX_ERR_BAD_SHAPE;
  *flops = helix::mfma_probe_flops(workgroups, iters);
  return launched(helix::launch_mfma_probe(sink, workgroups, iters, random_operands != 0, (hipStream_t)stream));
}

int helix_mfma_mix_probe(float* sink, int workgroups, int iters, int forward_mix, long long* flops, void* stream) {
  if (!sink || !flops) return HELIX_ERR_NULL_POINTER;
  if (!aligned(sink, 4)) return HELIX_ERR_MISALIGNED;
  if (workgroups < 1 || iters < 1 || workgroups > (1 << 20) || iters > (1 << 24)) return HELIX_ERR_BAD_SHAPE;
  *flops = helix::mfma_probe_flops(workgroups, iters);
  return launched(helix::launch_mfma_mix_probe(sink, workgroups, iters, forward_mix != 0, (hipStream_t)stream));
}

int helix_attn_device_info(int* compute_units, int* clock_khz) {
  if (!compute_units || !clock_khz) return HELIX_ERR_NULL_POINTER;
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return HELIX_ERR_LAUNCH;
  *compute_units = prop.multiProcessorCount;
  *clock_khz = prop.clockRate;
  return HELIX_OK;
}

const char* helix_status_string(int status) {
  switch (status) {
    case HELIX_OK: return "ok";
    case HELIX_ERR_NULL_POINTER: return "null pointer argument";
    case HELIX_ERR_BAD_SHAPE: return "bad shape: extents must be >= 1, within the index limits and, for the linear layer, multiples of the tile sizes";
    case HELIX_ERR_UNSUPPORTED_HEAD_DIM: return "unsupported head dimension: D must be 64 or 128";
    case HELIX_ERR_MISALIGNED: return "misaligned pointer: bf16 tensors need 16 bytes, fp32 4, workspace 256";
    case HELIX_ERR_BAD_SCALE: return "bad scale: must be finite and > 0";
    case HELIX_ERR_WORKSPACE: return "workspace too small";
    case HELIX_ERR_LAUNCH: return "kernel launch failed";
    case HELIX_ERR_SCRATCH_LIMIT: return "shape too large for the built-in scratch of helix_attn_bwd_static: B*H*S must not exceed 4194304";
    case HELIX_ERR_BAD_STRIDE: return "bad strides: multiples of 8 elements, row stride at least the row length and within the index limits, dimensions nested without overlap";
    default: return "unknown status";
  }
}

int helix_attn_version(void) { return kVersion; }

}  // extern "C"

namespace {

// The whole backward: delta, its refinement on the first rows (causal only), dK/dV, dQ.
int run_bwd(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dO,
            void* dq, void* dk, void* dv, void* stats, const helix::BwdMaps& maps,
            int B, int H, int S, int D, float scale, int causal, hipStream_t st) {
  float* nd = neg_delta_plane(stats);
  float* l2 = lse2_plane(stats, B, H, S);
  HELIX_TRY(launched(helix::launch_bwd_preprocess(o, dO, lse, nd, l2, maps, B, H, S, D, st)));
  if (causal) HELIX_TRY(launched(helix::launch_bwd_delta_head(q, k, v, dO, lse, nd, maps, B, H, S, D, HELIX_DELTA_HEAD_ROWS, scale, true, st)));
  HELIX_TRY(launched(helix::launch_bwd_dkdv(q, k, v, dO, l2, nd, dk, dv, maps, B, H, S, D, scale, causal != 0, st)));
  return launched(helix::launch_bwd_dq(q, k, v, dO, l2, nd, dq, maps, B, H, S, D, scale, causal != 0, st));
}

}  // namespace

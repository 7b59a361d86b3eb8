// C-ABI entry points (see include/helix_attn.h).  Everything here is host code: argument
// validation first, with no HIP call before it succeeds, then kernel launches on the
// caller's stream.  Nothing is allocated, freed or synchronised.
#include "../../include/helix_attn.h"
#include "kernels.hpp"

#include <cmath>
#include <cstdint>

namespace {

constexpr int kVersion = 100;  // 0.1.0

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

int check_shape(int B, int H, int S, int D) {
  if (B < 1 || H < 1 || S < 1 || D < 1) return HELIX_ERR_BAD_SHAPE;
  if (D != 64 && D != 128) return HELIX_ERR_UNSUPPORTED_HEAD_DIM;
  const long long bh = (long long)B * H;
  if (bh > 0x7fffffffLL / 8) return HELIX_ERR_BAD_SHAPE;          // workgroup ids stay in int
  if (S > (1 << 24)) return HELIX_ERR_BAD_SHAPE;                  // in-head offsets stay in 32 bits
  if ((double)bh * S * D >= 1099511627776.0) return HELIX_ERR_BAD_SHAPE;  // 2^40 elements
  const long long tiles = (long long)((S + 63) / 64) * 8 * ((bh + 7) / 8);
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

int launched(hipError_t e) { return e == hipSuccess ? HELIX_OK : HELIX_ERR_LAUNCH; }

#define HELIX_TRY(expr) do { int st_ = (expr); if (st_ != HELIX_OK) return st_; } while (0)

}  // namespace

extern "C" {

int helix_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                   int B, int H, int S, int D, float scale, int causal, void* stream) {
  HELIX_TRY(check_bf16_ptrs(q, k, v, (const void*)o));
  HELIX_TRY(check_f32_ptrs((const void*)lse));
  HELIX_TRY(check_shape(B, H, S, D));
  HELIX_TRY(check_scale(scale));
  return launched(helix::launch_fwd(q, k, v, o, lse, B * H, S, D, scale, causal != 0, (hipStream_t)stream));
}

size_t helix_attn_bwd_workspace_bytes(int B, int H, int S, int D) {
  if (check_shape(B, H, S, D) != HELIX_OK) return 0;
  const size_t n = (size_t)B * H * S * sizeof(float);
  return (n + 255) & ~(size_t)255;
}

int helix_attn_bwd_preprocess(const void* o, const void* dO, float* delta,
                              int B, int H, int S, int D, void* stream) {
  HELIX_TRY(check_bf16_ptrs(o, dO));
  HELIX_TRY(check_f32_ptrs((const void*)delta));
  HELIX_TRY(check_shape(B, H, S, D));
  return launched(helix::launch_bwd_preprocess(o, dO, delta, B * H, S, D, (hipStream_t)stream));
}

int helix_attn_bwd_delta_head(const void* q, const void* k, const void* v, const void* dO,
                              const float* lse, float* delta, int rows,
                              int B, int H, int S, int D, float scale, int causal, void* stream) {
  HELIX_TRY(check_bf16_ptrs(q, k, v, dO));
  HELIX_TRY(check_f32_ptrs((const void*)lse, (const void*)delta));
  HELIX_TRY(check_shape(B, H, S, D));
  HELIX_TRY(check_scale(scale));
  if (rows < 0) return HELIX_ERR_BAD_SHAPE;
  return launched(helix::launch_bwd_delta_head(q, k, v, dO, lse, delta, B * H, S, D, rows, scale, causal != 0, (hipStream_t)stream));
}

int helix_attn_bwd_dkdv(const void* q, const void* k, const void* v, const void* dO,
                        const float* lse, const float* delta, void* dk, void* dv,
                        int B, int H, int S, int D, float scale, int causal, void* stream) {
  HELIX_TRY(check_bf16_ptrs(q, k, v, dO, (const void*)dk, (const void*)dv));
  HELIX_TRY(check_f32_ptrs((const void*)lse, (const void*)delta));
  HELIX_TRY(check_shape(B, H, S, D));
  HELIX_TRY(check_scale(scale));
  return launched(helix::launch_bwd_dkdv(q, k, v, dO, lse, delta, dk, dv, B * H, S, D, scale, causal != 0, (hipStream_t)stream));
}

int helix_attn_bwd_dq(const void* q, const void* k, const void* v, const void* dO,
                      const float* lse, const float* delta, void* dq,
                      int B, int H, int S, int D, float scale, int causal, void* stream) {
  HELIX_TRY(check_bf16_ptrs(q, k, v, dO, (const void*)dq));
  HELIX_TRY(check_f32_ptrs((const void*)lse, (const void*)delta));
  HELIX_TRY(check_shape(B, H, S, D));
  HELIX_TRY(check_scale(scale));
  return launched(helix::launch_bwd_dq(q, k, v, dO, lse, delta, dq, B * H, S, D, scale, causal != 0, (hipStream_t)stream));
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
  float* delta = static_cast<float*>(workspace);
  hipStream_t st = (hipStream_t)stream;
  const int BH = B * H;
  HELIX_TRY(launched(helix::launch_bwd_preprocess(o, dO, delta, BH, S, D, st)));
  if (causal) HELIX_TRY(launched(helix::launch_bwd_delta_head(q, k, v, dO, lse, delta, BH, S, D, HELIX_DELTA_HEAD_ROWS, scale, true, st)));
  HELIX_TRY(launched(helix::launch_bwd_dkdv(q, k, v, dO, lse, delta, dk, dv, BH, S, D, scale, causal != 0, st)));
  return launched(helix::launch_bwd_dq(q, k, v, dO, lse, delta, dq, BH, S, D, scale, causal != 0, st));
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
    case HELIX_ERR_BAD_SHAPE: return "bad shape: B, H, S must be >= 1 and within the index limits";
    case HELIX_ERR_UNSUPPORTED_HEAD_DIM: return "unsupported head dimension: D must be 64 or 128";
    case HELIX_ERR_MISALIGNED: return "misaligned pointer: bf16 tensors need 16 bytes, fp32 4, workspace 256";
    case HELIX_ERR_BAD_SCALE: return "bad scale: must be finite and > 0";
    case HELIX_ERR_WORKSPACE: return "workspace too small";
    case HELIX_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
  }
}

int helix_attn_version(void) { return kVersion; }

}  // extern "C"

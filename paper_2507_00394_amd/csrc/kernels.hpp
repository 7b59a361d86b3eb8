// Host-side launchers of the gfx950 attention kernels.  Shapes, strides and alignment are
// validated by the C-ABI layer before any of these is called.
#pragma once
#include <hip/hip_runtime.h>

namespace helix {

// Where a [B, H, S, D] tensor lives: element strides of batch, head and row; the D elements
// of a row are contiguous.
struct TensorMap {
  long long batch, head;
  int row;
};
inline TensorMap contiguous_map(int H, int S, int D) {
  return TensorMap{(long long)H * S * D, (long long)S * D, D};
}
struct FwdMaps { TensorMap q, k, v, o; };

// Raises a kernel's dynamic LDS limit once per device and process instead of on every launch
// (the attribute call costs as much as a small launch).  `done` is the caller's per-kernel
// bit mask of devices already configured.
template <typename Kernel>
inline hipError_t allow_dynamic_lds(Kernel kern, size_t bytes, unsigned long long& done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const unsigned long long bit = 1ull << (dev & 63);
  if (__atomic_load_n(&done, __ATOMIC_ACQUIRE) & bit) return hipSuccess;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess) __atomic_fetch_or(&done, bit, __ATOMIC_RELEASE);
  return e;
}
struct BwdMaps { TensorMap q, k, v, o, dO, dq, dk, dv; };

// lse and every other per-row fp32 array are contiguous [B, H, S].  Between the backward
// kernels the row statistics travel as neg_delta = -rowsum(dO o O) and lse2 = lse * log2(e).
hipError_t launch_fwd(const void* q, const void* k, const void* v, void* o, float* lse, const FwdMaps& maps,
                      int B, int H, int S, int D, float scale, bool causal, hipStream_t stream);
hipError_t launch_bwd_preprocess(const void* o, const void* dO, const float* lse, float* neg_delta, float* lse2,
                                 const BwdMaps& maps, int B, int H, int S, int D, hipStream_t stream);
// neg_delta_i = -sum_j p_ij dp_ij for query rows 0..rows-1 of every head, overwriting neg_delta there.
hipError_t launch_bwd_delta_head(const void* q, const void* k, const void* v, const void* dO,
                                 const float* lse, float* neg_delta, const BwdMaps& maps, int B, int H, int S, int D,
                                 int rows, float scale, bool causal, hipStream_t stream);
hipError_t launch_bwd_dkdv(const void* q, const void* k, const void* v, const void* dO,
                           const float* lse2, const float* neg_delta, void* dk, void* dv, const BwdMaps& maps,
                           int B, int H, int S, int D, float scale, bool causal, hipStream_t stream);
// Head dimension 128 with two waves per SIMD (one wave of a pair for S, P and dV, the other for dP, dS and dK).
hipError_t launch_bwd_dkdv_pair(const void* q, const void* k, const void* v, const void* dO, const float* lse2,
                                const float* neg_delta, void* dk, void* dv, const BwdMaps& maps, int B, int H, int S,
                                float scale, bool causal, hipStream_t stream);
hipError_t launch_bwd_dq(const void* q, const void* k, const void* v, const void* dO,
                         const float* lse2, const float* neg_delta, void* dq, const BwdMaps& maps,
                         int B, int H, int S, int D, float scale, bool causal, hipStream_t stream);

// Linear layer next to attention: out[M][N] = a[M][K] w[K][N] (bf16, fp32 accumulation) and its
// backward products da[M][K] = dout[M][N] w[K][N]^T (bf16) and dw[K][N] = a[M][K]^T dout[M][N] (fp32).
// ld*: elements between consecutive rows.
hipError_t launch_linear_fwd(const void* a, long long lda, const void* w, long long ldw, void* out, long long ldo,
                             int M, int K, int N, hipStream_t stream);
// The backward's workspace (linear_bwd_workspace_bytes) holds w^T in its first linear_bwd_wt_bytes(K, N)
// bytes and the partial weight gradients after them.
size_t linear_bwd_workspace_bytes(int M, int K, int N);
size_t linear_bwd_wt_bytes(int K, int N);
hipError_t launch_linear_bwd_input(const void* dout, long long ldd, const void* w, long long ldw, void* da, long long lda,
                                   void* wt, int M, int K, int N, hipStream_t stream);
hipError_t launch_linear_bwd_weight(const void* a, long long lda, const void* dout, long long ldd, float* dw, long long ldw,
                                    float* workspace, int M, int K, int N, hipStream_t stream);

// Pure MFMA loop (mfma_probe.hip): `workgroups` x 8 waves x `iters` x 16 independent 32x32x16 bf16 MFMAs.
long long mfma_probe_flops(int workgroups, int iters);
hipError_t launch_mfma_probe(float* sink, int workgroups, int iters, bool random_operands, hipStream_t stream);
// The same loop with one LDS operand read and some vector work per MFMA: 2 fma + 0.5 exp2 (the backward passes'
// mix) or, forward_mix, 3 fma + 1 exp2.  One workgroup per compute unit (64 KB of LDS).  Same FLOP count.
hipError_t launch_mfma_mix_probe(float* sink, int workgroups, int iters, bool forward_mix, hipStream_t stream);

}  // namespace helix

// Host-side launchers of the gfx950 attention kernels.  Shapes are validated by the
// C-ABI layer before any of these is called; BH = B*H.
#pragma once
#include <hip/hip_runtime.h>

namespace helix {

hipError_t launch_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                      int BH, int S, int D, float scale, bool causal, hipStream_t stream);
hipError_t launch_bwd_preprocess(const void* o, const void* dO, float* delta,
                                 int BH, int S, int D, hipStream_t stream);
// delta_i = sum_j p_ij dp_ij for query rows 0..rows-1 of every head, overwriting delta there.
hipError_t launch_bwd_delta_head(const void* q, const void* k, const void* v, const void* dO,
                                 const float* lse, float* delta, int BH, int S, int D, int rows,
                                 float scale, bool causal, hipStream_t stream);
hipError_t launch_bwd_dkdv(const void* q, const void* k, const void* v, const void* dO,
                           const float* lse, const float* delta, void* dk, void* dv,
                           int BH, int S, int D, float scale, bool causal, hipStream_t stream);
hipError_t launch_bwd_dq(const void* q, const void* k, const void* v, const void* dO,
                         const float* lse, const float* delta, void* dq,
                         int BH, int S, int D, float scale, bool causal, hipStream_t stream);

}  // namespace helix

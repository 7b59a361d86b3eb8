// Backward attention for gfx950 (Table 1, Attention column, "Backward B"; attention has no
// parameters, so there is no "Backward W").  Works from q, k, v, o, lse only -- the
// activations the paper calls "saved by flash attention" (Section 4.4) -- in three kernels:
//
//   preprocess : delta_i = sum_d dO_id * O_id                         (streams 2 tensors, HBM bound)
//   dkdv       : (bwd_dkdv.hip) a workgroup owns 128 keys and sweeps the query tiles that see
//                them: S = Q K^T, P = exp(scale*S - LSE), dV^T += dO^T P, dP = dO V^T,
//                dS = P o (dP - delta), dK^T += Q^T dS
//   dq         : (bwd_dq.hip) a workgroup owns 256 queries and sweeps the visible key tiles:
//                S^T = K Q^T, dP^T = V dO^T, dS^T = P^T o (dP^T - delta), dQ^T += K^T dS^T
//   delta_head : the unpipelined variant of the dQ sweep kept in this file; it only produces
//                delta_i = sum_j p_ij dp_ij for the first rows of every head
//
// Every output element is produced by exactly one lane, so there are no atomics and the
// result is bit-reproducible.
#include "helix_common.hpp"
#include "kernels.hpp"

namespace helix {

// ------------------------------------------------------------------ preprocess
// One row of D bf16 is D/8 16-byte chunks; D/8 adjacent lanes own a row.
template <int D>
__global__ void __launch_bounds__(256)
bwd_preprocess_kernel(const __bf16* __restrict__ o, const __bf16* __restrict__ dO,
                      float* __restrict__ delta, long long rows) {
  constexpr int LPR = D / 8;            // lanes per row
  constexpr int RPB = 256 / LPR;        // rows per workgroup pass
  constexpr int PASSES = 4;
  const int tid = threadIdx.x;
  const int sub = tid % LPR;
  const long long row0 = (long long)blockIdx.x * (RPB * PASSES) + tid / LPR;
  bf16x8 a[PASSES], b[PASSES];
#pragma unroll
  for (int p = 0; p < PASSES; p++) {
    const long long r = row0 + p * RPB;
    if (r < rows) {
      a[p] = *reinterpret_cast<const bf16x8*>(o + r * D + sub * 8);
      b[p] = *reinterpret_cast<const bf16x8*>(dO + r * D + sub * 8);
    }
  }
#pragma unroll
  for (int p = 0; p < PASSES; p++) {
    const long long r = row0 + p * RPB;
    float s = 0.f;
    if (r < rows) {
#pragma unroll
      for (int e = 0; e < 8; e++) s = fmaf((float)a[p][e], (float)b[p][e], s);
    }
#pragma unroll
    for (int off = LPR / 2; off >= 1; off >>= 1) s += __shfl_xor(s, off);
    if (sub == 0 && r < rows) delta[r] = s;
  }
}

hipError_t launch_bwd_preprocess(const void* o, const void* dO, float* delta,
                                 int BH, int S, int D, hipStream_t stream) {
  const long long rows = (long long)BH * S;
  if (D == 128) {
    const long long per = (256 / 16) * 4;
    hipLaunchKernelGGL(bwd_preprocess_kernel<128>, dim3((unsigned)((rows + per - 1) / per)), dim3(256), 0, stream,
                       (const __bf16*)o, (const __bf16*)dO, delta, rows);
  } else {
    const long long per = (256 / 8) * 4;
    hipLaunchKernelGGL(bwd_preprocess_kernel<64>, dim3((unsigned)((rows + per - 1) / per)), dim3(256), 0, stream,
                       (const __bf16*)o, (const __bf16*)dO, delta, rows);
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------ dQ
// With DELTA_ONLY the same sweep evaluates delta_i = sum_j p_ij dp_ij from its definition
// and writes it to delta_out instead of producing dQ (used for the first rows of every
// head, where attention is concentrated on few keys and the bf16 rounding of O would
// otherwise dominate delta).
template <int D, bool CAUSAL, bool DELTA_ONLY>
__global__ void __launch_bounds__(512, 1)
bwd_dq_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k, const __bf16* __restrict__ v,
              const __bf16* __restrict__ dO, const float* __restrict__ lse, const float* __restrict__ delta,
              __bf16* __restrict__ dq, float* __restrict__ delta_out, int BH, int S, int T, float scale) {
  constexpr int BM = 256, BN = 64, NT = 512;
  constexpr int KS = D / 16, DB = D / 32;
  constexpr int TILE_BYTES = BN * D * 2;
  extern __shared__ __align__(16) char smem[];   // K[2] then V[2]

  const TileCoord tc = map_block(blockIdx.x, BH, T, true);
  if (!tc.valid) return;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int half = lane >> 5, n = lane & 31;
  const int q0 = tc.tile * BM;
  const int my_q = q0 + 32 * w + n;
  const size_t head_off = (size_t)tc.bh * S * D;
  const __bf16* kh = k + head_off;
  const __bf16* vh = v + head_off;
  const float c = scale * kLog2e;

  bf16x8 qf[KS], gf[KS];
  float lse2, dl;
  {
    const int row = my_q < S ? my_q : S - 1;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      qf[ks] = *reinterpret_cast<const bf16x8*>(q + head_off + (size_t)row * D + 16 * ks + 8 * half);
      gf[ks] = *reinterpret_cast<const bf16x8*>(dO + head_off + (size_t)row * D + 16 * ks + 8 * half);
    }
    lse2 = lse[(size_t)tc.bh * S + row] * kLog2e;
    dl = DELTA_ONLY ? 0.f : delta[(size_t)tc.bh * S + row];
  }
  float dsum = 0.f;   // DELTA_ONLY: this lane's share of sum_j p_ij dp_ij
  f32x16 dqacc[DB];
#pragma unroll
  for (int db = 0; db < DB; db++)
#pragma unroll
    for (int e = 0; e < 16; e++) dqacc[db][e] = 0.f;

  const int q_end = (q0 + BM < S ? q0 + BM : S);
  const int n_tiles = CAUSAL ? (q_end + BN - 1) / BN : (S + BN - 1) / BN;
  const int wave_qmin = q0 + 32 * w, wave_qmax = wave_qmin + 31;

  TileStage<D, BN, NT> sk, sv;
  sk.fetch(kh, 0, S, tid);
  sv.fetch(vh, 0, S, tid);
  sk.commit(smem, tid);
  sv.commit(smem + 2 * TILE_BYTES, tid);
  __syncthreads();

  for (int j = 0; j < n_tiles; j++) {
    const char* kt = smem + (j & 1) * TILE_BYTES;
    const char* vt = smem + (2 + (j & 1)) * TILE_BYTES;
    const int k0 = j * BN;
    const bool more = j + 1 < n_tiles;
    if (more) {
      sk.fetch(kh, k0 + BN, S, tid);
      sv.fetch(vh, k0 + BN, S, tid);
    }
    if (!CAUSAL || k0 <= wave_qmax) {
#pragma unroll
      for (int kb = 0; kb < 2; kb++) {
        if (CAUSAL && k0 + 32 * kb > wave_qmax) continue;
        f32x16 sacc, pacc;
#pragma unroll
        for (int e = 0; e < 16; e++) { sacc[e] = 0.f; pacc[e] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < KS; ks++) sacc = mfma32(lds_operand<D>(kt, 32 * kb + n, ks, half), qf[ks], sacc);
#pragma unroll
        for (int ks = 0; ks < KS; ks++) pacc = mfma32(lds_operand<D>(vt, 32 * kb + n, ks, half), gf[ks], pacc);
        const bool need_mask = CAUSAL ? (k0 + 32 * kb + 31 > wave_qmin) : (k0 + 32 * kb + 32 > S);
#pragma unroll
        for (int e = 0; e < 16; e++) {
          float p = __builtin_amdgcn_exp2f(fmaf(sacc[e], c, -lse2));
          if (need_mask) {
            const int key = k0 + 32 * kb + 8 * (e >> 2) + 4 * half + (e & 3);
            p = (CAUSAL ? key <= my_q : key < S) ? p : 0.f;
          }
          if constexpr (DELTA_ONLY) dsum = fmaf(p, pacc[e], dsum);
          else pacc[e] = p * (pacc[e] - dl);
        }
        if constexpr (!DELTA_ONLY) {
#pragma unroll
          for (int t = 0; t < 2; t++) {
            const bf16x8 sb = pack_half(pacc, t);
#pragma unroll
            for (int db = 0; db < DB; db++)
              dqacc[db] = mfma32(lds_operand_tr<D>(kt, 32 * kb + 16 * t, 32 * db, lane), sb, dqacc[db]);
          }
        }
      }
    }
    if (more) {
      sk.commit(smem + ((j + 1) & 1) * TILE_BYTES, tid);
      sv.commit(smem + (2 + ((j + 1) & 1)) * TILE_BYTES, tid);
    }
    __syncthreads();
  }

  if constexpr (DELTA_ONLY) {
    dsum = half_sum(dsum);
    if (my_q < S && half == 0) delta_out[(size_t)tc.bh * S + my_q] = dsum;
  } else if (my_q < S) {
    __bf16* row = dq + head_off + (size_t)my_q * D;
#pragma unroll
    for (int db = 0; db < DB; db++)
#pragma unroll
      for (int g = 0; g < 4; g++) {
        f32x4 x;
#pragma unroll
        for (int e = 0; e < 4; e++) x[e] = dqacc[db][4 * g + e] * scale;
        *reinterpret_cast<bf16x4*>(row + 32 * db + 8 * g + 4 * half) = __builtin_convertvector(x, bf16x4);
      }
  }
}

template <int D, bool CAUSAL, bool DELTA_ONLY>
static hipError_t launch_dq_t(const void* q, const void* k, const void* v, const void* dO,
                              const float* lse, const float* delta, void* dq, float* delta_out,
                              int BH, int S, int rows, float scale, hipStream_t stream) {
  constexpr int BM = 256, BN = 64;
  const int T = (rows + BM - 1) / BM;   // query tiles 0..T-1 of every head
  const int grid = 8 * ((BH + 7) / 8) * T;
  const size_t lds = 4 * BN * D * 2;
  auto kern = bwd_dq_kernel<D, CAUSAL, DELTA_ONLY>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(512), lds, stream, (const __bf16*)q, (const __bf16*)k, (const __bf16*)v,
                     (const __bf16*)dO, lse, delta, (__bf16*)dq, delta_out, BH, S, T, scale);
  return hipGetLastError();
}

hipError_t launch_bwd_delta_head(const void* q, const void* k, const void* v, const void* dO,
                                 const float* lse, float* delta, int BH, int S, int D, int rows,
                                 float scale, bool causal, hipStream_t stream) {
  if (rows <= 0) return hipSuccess;
  if (rows > S) rows = S;
  if (D == 128) return causal ? launch_dq_t<128, true, true>(q, k, v, dO, lse, nullptr, nullptr, delta, BH, S, rows, scale, stream)
                              : launch_dq_t<128, false, true>(q, k, v, dO, lse, nullptr, nullptr, delta, BH, S, rows, scale, stream);
  return causal ? launch_dq_t<64, true, true>(q, k, v, dO, lse, nullptr, nullptr, delta, BH, S, rows, scale, stream)
                : launch_dq_t<64, false, true>(q, k, v, dO, lse, nullptr, nullptr, delta, BH, S, rows, scale, stream);
}

}  // namespace helix

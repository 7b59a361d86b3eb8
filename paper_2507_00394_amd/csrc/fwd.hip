// Forward attention for gfx950: O = softmax(scale * Q K^T + causal mask) V and the
// log-sum-exp of every score row (Table 1, Attention column, "Forward").
//
// Work split: one workgroup of 8 waves owns 256 consecutive query rows of one (batch, head)
// slice, 32 rows per wave, and sweeps the key tiles (64 keys) that the causal mask leaves
// visible.  Each wave computes the TRANSPOSED score block S^T = K Q^T with the 32x32x16 bf16
// MFMA, so that a lane owns ONE query (column l%32) and 16 keys per 32-key block: the
// running maximum and sum of a row live in a single register per lane and need one
// exchange between the two wave halves, not a 32-lane reduction.  bf16(P^T) in its
// accumulator layout is directly the B operand of O^T += V^T P^T; V^T comes from the
// row-major V tile in LDS through the transposing LDS read.
#include "helix_common.hpp"
#include "kernels.hpp"

namespace helix {

template <int D, bool CAUSAL>
__global__ void __launch_bounds__(512, 1)
fwd_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k, const __bf16* __restrict__ v,
           __bf16* __restrict__ o, float* __restrict__ lse, int BH, int S, int T, float scale) {
  constexpr int BM = 256, BN = 64, NT = 512;
  constexpr int KS = D / 16;   // contraction steps of Q K^T
  constexpr int DB = D / 32;   // 32-wide blocks of the head dimension
  constexpr int TILE_BYTES = BN * D * 2;
  extern __shared__ __align__(16) char smem[];   // K[2] then V[2]

  const TileCoord tc = map_block(blockIdx.x, BH, T, true);
  if (!tc.valid) return;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int half = lane >> 5, n = lane & 31;
  const int q0 = tc.tile * BM;
  const int my_q = q0 + 32 * w + n;
  const size_t head_off = (size_t)tc.bh * S * D;
  const __bf16* qh = q + head_off;
  const __bf16* kh = k + head_off;
  const __bf16* vh = v + head_off;
  const float c = scale * kLog2e;

  // Q^T operand fragments: this lane's query row, 8 elements per contraction step.
  bf16x8 qf[KS];
  {
    const int row = my_q < S ? my_q : S - 1;
#pragma unroll
    for (int ks = 0; ks < KS; ks++)
      qf[ks] = *reinterpret_cast<const bf16x8*>(qh + (size_t)row * D + 16 * ks + 8 * half);
  }

  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; db++)
#pragma unroll
    for (int e = 0; e < 16; e++) oacc[db][e] = 0.f;
  float m = -INFINITY;   // running row maximum of the raw (unscaled) scores
  float lsum = 0.f;      // this lane's share of the running row sum

  const int q_end = (q0 + BM < S ? q0 + BM : S);                 // one past the last real row
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
      // S^T blocks: rows = keys k0 + 32*kb + (0..31), columns = this wave's 32 queries
      f32x16 sacc[2];
#pragma unroll
      for (int kb = 0; kb < 2; kb++) {
#pragma unroll
        for (int e = 0; e < 16; e++) sacc[kb][e] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ks++)
          sacc[kb] = mfma32(lds_operand<D>(kt, 32 * kb + n, ks, half), qf[ks], sacc[kb]);
      }
      const bool need_mask = CAUSAL ? (k0 + BN - 1 > wave_qmin) : (k0 + BN > S);
      if (need_mask) {
#pragma unroll
        for (int kb = 0; kb < 2; kb++)
#pragma unroll
          for (int e = 0; e < 16; e++) {
            const int key = k0 + 32 * kb + 8 * (e >> 2) + 4 * half + (e & 3);
            const bool ok = CAUSAL ? (key <= my_q) : (key < S);
            sacc[kb][e] = ok ? sacc[kb][e] : -INFINITY;
          }
      }
      float tmax = sacc[0][0];
#pragma unroll
      for (int kb = 0; kb < 2; kb++)
#pragma unroll
        for (int e = 0; e < 16; e++) tmax = fmaxf(tmax, sacc[kb][e]);
      tmax = half_max(tmax);
      const float m_new = fmaxf(m, tmax);
      if (__any(m_new > m)) {
        const float alpha = __builtin_amdgcn_exp2f((m - m_new) * c);   // 0 on the first tile
        lsum *= alpha;
#pragma unroll
        for (int db = 0; db < DB; db++)
#pragma unroll
          for (int e = 0; e < 16; e++) oacc[db][e] *= alpha;
        m = m_new;
      }
      const float mc = m * c;
#pragma unroll
      for (int kb = 0; kb < 2; kb++)
#pragma unroll
        for (int e = 0; e < 16; e++) {
          const float p = __builtin_amdgcn_exp2f(fmaf(sacc[kb][e], c, -mc));
          sacc[kb][e] = p;
          lsum += p;
        }
      // O^T += V^T P^T, 16 keys per step
#pragma unroll
      for (int kb = 0; kb < 2; kb++)
#pragma unroll
        for (int t = 0; t < 2; t++) {
          const bf16x8 pb = pack_half(sacc[kb], t);
#pragma unroll
          for (int db = 0; db < DB; db++)
            oacc[db] = mfma32(lds_operand_tr<D>(vt, 32 * kb + 16 * t, 32 * db, lane), pb, oacc[db]);
        }
    }
    if (more) {
      sk.commit(smem + ((j + 1) & 1) * TILE_BYTES, tid);
      sv.commit(smem + (2 + ((j + 1) & 1)) * TILE_BYTES, tid);
    }
    __syncthreads();
  }

  // epilogue: normalise, store O (bf16) and LSE (natural log, scale included)
  const float ltot = half_sum(lsum);
  const float inv = 1.f / ltot;
  if (my_q < S) {
    __bf16* orow = o + head_off + (size_t)my_q * D;
#pragma unroll
    for (int db = 0; db < DB; db++)
#pragma unroll
      for (int g = 0; g < 4; g++) {
        f32x4 x;
#pragma unroll
        for (int e = 0; e < 4; e++) x[e] = oacc[db][4 * g + e] * inv;
        *reinterpret_cast<bf16x4*>(orow + 32 * db + 8 * g + 4 * half) = __builtin_convertvector(x, bf16x4);
      }
    if (half == 0) lse[(size_t)tc.bh * S + my_q] = m * scale + __logf(ltot);
  }
}

template <int D, bool CAUSAL>
static hipError_t launch_fwd_t(const void* q, const void* k, const void* v, void* o, float* lse,
                               int BH, int S, float scale, hipStream_t stream) {
  constexpr int BM = 256, BN = 64;
  const int T = (S + BM - 1) / BM;
  const int grid = 8 * ((BH + 7) / 8) * T;
  const size_t lds = 4 * BN * D * 2;
  auto kern = fwd_kernel<D, CAUSAL>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(512), lds, stream, (const __bf16*)q, (const __bf16*)k,
                     (const __bf16*)v, (__bf16*)o, lse, BH, S, T, scale);
  return hipGetLastError();
}

hipError_t launch_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                      int BH, int S, int D, float scale, bool causal, hipStream_t stream) {
  if (D == 128) return causal ? launch_fwd_t<128, true>(q, k, v, o, lse, BH, S, scale, stream)
                              : launch_fwd_t<128, false>(q, k, v, o, lse, BH, S, scale, stream);
  return causal ? launch_fwd_t<64, true>(q, k, v, o, lse, BH, S, scale, stream)
                : launch_fwd_t<64, false>(q, k, v, o, lse, BH, S, scale, stream);
}

}  // namespace helix

// Backward attention for gfx950 (Table 1, Attention column, "Backward B"; attention has no
// parameters, so there is no "Backward W").  Works from q, k, v, o, lse only -- the
// activations the paper calls "saved by flash attention" (Section 4.4) -- in three kernels:
//
//   preprocess : delta_i = sum_d dO_id * O_id                         (streams 2 tensors, HBM bound)
//   dkdv       : a workgroup owns 256 keys and sweeps the query tiles that see them:
//                S = Q K^T, P = exp(scale*S - LSE), dV^T += dO^T P, dP = dO V^T,
//                dS = P o (dP - delta), dK^T += Q^T dS
//   dq         : a workgroup owns 256 queries and sweeps the visible key tiles:
//                S^T = K Q^T, dP^T = V dO^T, dS^T = P^T o (dP^T - delta), dQ^T += K^T dS^T
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

// ------------------------------------------------------------------ dK / dV
template <int D, bool CAUSAL>
__global__ void __launch_bounds__(512, 1)
bwd_dkdv_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k, const __bf16* __restrict__ v,
                const __bf16* __restrict__ dO, const float* __restrict__ lse, const float* __restrict__ delta,
                __bf16* __restrict__ dk, __bf16* __restrict__ dv, int BH, int S, int T, float scale) {
  constexpr int BN = 256, BM = 64, NT = 512;
  constexpr int KS = D / 16, DB = D / 32;
  constexpr int TILE_BYTES = BM * D * 2;
  constexpr int STAT_OFF = 4 * TILE_BYTES;        // after Q[2], dO[2]: lse2[2][BM], delta[2][BM]
  constexpr int V_OFF = STAT_OFF + 4 * BM * 4;    // then the workgroup's V tile [BN][D], resident
  extern __shared__ __align__(16) char smem[];

  const TileCoord tc = map_block(blockIdx.x, BH, T, false);
  if (!tc.valid) return;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int half = lane >> 5, n = lane & 31;
  const int n0 = tc.tile * BN;
  const int my_key = n0 + 32 * w + n;
  const size_t head_off = (size_t)tc.bh * S * D;
  const __bf16* qh = q + head_off;
  const __bf16* gh = dO + head_off;
  const float* lse_h = lse + (size_t)tc.bh * S;
  const float* delta_h = delta + (size_t)tc.bh * S;
  const float c = scale * kLog2e;

  // K^T operand fragments of this lane's key (columns of S) stay in registers; the V^T
  // fragments (columns of dP) are re-read from an LDS copy of the workgroup's V rows.
  bf16x8 kf[KS];
  {
    const int row = my_key < S ? my_key : S - 1;
#pragma unroll
    for (int ks = 0; ks < KS; ks++)
      kf[ks] = *reinterpret_cast<const bf16x8*>(k + head_off + (size_t)row * D + 16 * ks + 8 * half);
    TileStage<D, BN, NT> svt;
    svt.fetch(v + head_off, n0, S, tid);
    svt.commit(smem + V_OFF, tid);
  }
  const char* vtile = smem + V_OFF;
  f32x16 dkacc[DB], dvacc[DB];
#pragma unroll
  for (int db = 0; db < DB; db++)
#pragma unroll
    for (int e = 0; e < 16; e++) { dkacc[db][e] = 0.f; dvacc[db][e] = 0.f; }

  const int m_start = CAUSAL ? n0 : 0;                          // first query row that sees a key of this tile
  const int n_tiles = (S - m_start + BM - 1) / BM;
  const int wave_kmin = n0 + 32 * w;

  TileStage<D, BM, NT> sq, sg;
  float stat = 0.f;
  auto fetch_stats = [&](int r0) {
    if (tid < 2 * BM) {
      const int r = r0 + (tid & (BM - 1));
      if (tid < BM) stat = r < S ? lse_h[r] * kLog2e : INFINITY;   // rows past the end get p = 0
      else stat = r < S ? delta_h[r] : 0.f;
    }
  };
  auto commit_stats = [&](int buf) {
    if (tid < 2 * BM) reinterpret_cast<float*>(smem + STAT_OFF)[(tid < BM ? 0 : 2 * BM) + buf * BM + (tid & (BM - 1))] = stat;
  };
  sq.fetch(qh, m_start, S, tid);
  sg.fetch(gh, m_start, S, tid);
  fetch_stats(m_start);
  sq.commit(smem, tid);
  sg.commit(smem + 2 * TILE_BYTES, tid);
  commit_stats(0);
  __syncthreads();

  for (int it = 0; it < n_tiles; it++) {
    const int buf = it & 1;
    const char* qt = smem + buf * TILE_BYTES;
    const char* gt = smem + (2 + buf) * TILE_BYTES;
    const float* lse2 = reinterpret_cast<const float*>(smem + STAT_OFF) + buf * BM;
    const float* dlt = reinterpret_cast<const float*>(smem + STAT_OFF) + 2 * BM + buf * BM;
    const int r_tile = m_start + it * BM;
    const bool more = it + 1 < n_tiles;
    if (more) {
      sq.fetch(qh, r_tile + BM, S, tid);
      sg.fetch(gh, r_tile + BM, S, tid);
      fetch_stats(r_tile + BM);
    }
#pragma unroll
    for (int qb = 0; qb < BM / 32; qb++) {
      const int r0 = r_tile + 32 * qb;                         // global row of this 32-row block
      if (CAUSAL && r0 + 31 < wave_kmin) continue;              // every key of the wave is masked
      f32x16 sacc, pacc;
#pragma unroll
      for (int e = 0; e < 16; e++) { sacc[e] = 0.f; pacc[e] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ks++) sacc = mfma32(lds_operand<D>(qt, 32 * qb + n, ks, half), kf[ks], sacc);
      int vrow = 32 * w + n;
      asm volatile("" : "+v"(vrow));   // keep the V reads inside the loop (they would be hoisted into registers)
#pragma unroll
      for (int ks = 0; ks < KS; ks++)
        pacc = mfma32(lds_operand<D>(gt, 32 * qb + n, ks, half), lds_operand<D>(vtile, vrow, ks, half), pacc);
      const bool need_mask = CAUSAL && (r0 < wave_kmin + 31);
#pragma unroll
      for (int g = 0; g < 4; g++) {
        const f32x4 l4 = *reinterpret_cast<const f32x4*>(lse2 + 32 * qb + 8 * g + 4 * half);
        const f32x4 d4 = *reinterpret_cast<const f32x4*>(dlt + 32 * qb + 8 * g + 4 * half);
#pragma unroll
        for (int e4 = 0; e4 < 4; e4++) {
          const int e = 4 * g + e4;
          float p = __builtin_amdgcn_exp2f(fmaf(sacc[e], c, -l4[e4]));
          if (need_mask) p = (my_key <= r0 + 8 * g + 4 * half + e4) ? p : 0.f;
          sacc[e] = p;
          pacc[e] = p * (pacc[e] - d4[e4]);
        }
      }
#pragma unroll
      for (int t = 0; t < 2; t++) {
        const bf16x8 pb = pack_half(sacc, t);
        const bf16x8 sb = pack_half(pacc, t);
#pragma unroll
        for (int db = 0; db < DB; db++) {
          dvacc[db] = mfma32(lds_operand_tr<D>(gt, 32 * qb + 16 * t, 32 * db, lane), pb, dvacc[db]);
          dkacc[db] = mfma32(lds_operand_tr<D>(qt, 32 * qb + 16 * t, 32 * db, lane), sb, dkacc[db]);
        }
      }
    }
    if (more) {
      sq.commit(smem + (buf ^ 1) * TILE_BYTES, tid);
      sg.commit(smem + (2 + (buf ^ 1)) * TILE_BYTES, tid);
      commit_stats(buf ^ 1);
    }
    __syncthreads();
  }

  if (my_key < S) {
    __bf16* dkrow = dk + head_off + (size_t)my_key * D;
    __bf16* dvrow = dv + head_off + (size_t)my_key * D;
#pragma unroll
    for (int db = 0; db < DB; db++)
#pragma unroll
      for (int g = 0; g < 4; g++) {
        f32x4 x, y;
#pragma unroll
        for (int e = 0; e < 4; e++) { x[e] = dkacc[db][4 * g + e] * scale; y[e] = dvacc[db][4 * g + e]; }
        *reinterpret_cast<bf16x4*>(dkrow + 32 * db + 8 * g + 4 * half) = __builtin_convertvector(x, bf16x4);
        *reinterpret_cast<bf16x4*>(dvrow + 32 * db + 8 * g + 4 * half) = __builtin_convertvector(y, bf16x4);
      }
  }
}

template <int D, bool CAUSAL>
static hipError_t launch_dkdv_t(const void* q, const void* k, const void* v, const void* dO,
                                const float* lse, const float* delta, void* dk, void* dv,
                                int BH, int S, float scale, hipStream_t stream) {
  constexpr int BN = 256, BM = 64;
  const int T = (S + BN - 1) / BN;
  const int grid = 8 * ((BH + 7) / 8) * T;
  const size_t lds = 4 * BM * D * 2 + 4 * BM * sizeof(float) + BN * D * 2;
  auto kern = bwd_dkdv_kernel<D, CAUSAL>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(512), lds, stream, (const __bf16*)q, (const __bf16*)k, (const __bf16*)v,
                     (const __bf16*)dO, lse, delta, (__bf16*)dk, (__bf16*)dv, BH, S, T, scale);
  return hipGetLastError();
}

hipError_t launch_bwd_dkdv(const void* q, const void* k, const void* v, const void* dO,
                           const float* lse, const float* delta, void* dk, void* dv,
                           int BH, int S, int D, float scale, bool causal, hipStream_t stream) {
  if (D == 128) return causal ? launch_dkdv_t<128, true>(q, k, v, dO, lse, delta, dk, dv, BH, S, scale, stream)
                              : launch_dkdv_t<128, false>(q, k, v, dO, lse, delta, dk, dv, BH, S, scale, stream);
  return causal ? launch_dkdv_t<64, true>(q, k, v, dO, lse, delta, dk, dv, BH, S, scale, stream)
                : launch_dkdv_t<64, false>(q, k, v, dO, lse, delta, dk, dv, BH, S, scale, stream);
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

hipError_t launch_bwd_dq(const void* q, const void* k, const void* v, const void* dO,
                         const float* lse, const float* delta, void* dq,
                         int BH, int S, int D, float scale, bool causal, hipStream_t stream) {
  if (D == 128) return causal ? launch_dq_t<128, true, false>(q, k, v, dO, lse, delta, dq, nullptr, BH, S, S, scale, stream)
                              : launch_dq_t<128, false, false>(q, k, v, dO, lse, delta, dq, nullptr, BH, S, S, scale, stream);
  return causal ? launch_dq_t<64, true, false>(q, k, v, dO, lse, delta, dq, nullptr, BH, S, S, scale, stream)
                : launch_dq_t<64, false, false>(q, k, v, dO, lse, delta, dq, nullptr, BH, S, S, scale, stream);
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

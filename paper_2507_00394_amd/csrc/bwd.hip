// Backward attention for gfx950 (Table 1, Attention column, "Backward B"; attention has no
// parameters, so there is no "Backward W").  Works from q, k, v, o, lse only -- the
// activations the paper calls "saved by flash attention" (Section 4.4) -- in three kernels:
//
//   preprocess : delta_i = sum_d dO_id * O_id                         (streams 2 tensors, HBM bound)
//   dkdv       : (bwd_dkdv_pair.hip for head dimension 128, bwd_dkdv.hip for 64) a workgroup owns
//                128 keys and sweeps the query blocks that see them: S = Q K^T,
//                P = exp(scale*S - LSE), dV^T += dO^T P, dP = dO V^T, dS = P o (dP - delta),
//                dK^T += Q^T dS
//   dq         : (bwd_dq.hip) a workgroup owns 256 queries and sweeps the visible key tiles:
//                S^T = K Q^T, dP^T = V dO^T, dS^T = P^T o (dP^T - delta), dQ^T += K^T dS^T
//   delta_head : the unpipelined variant of the dQ sweep kept in this file; it only produces
//                delta_i = sum_j p_ij dp_ij for the first rows of every head
// Between the kernels the row statistics travel as neg_delta = -delta and lse2 = LSE * log2(e).
//
// Every output element is produced by exactly one lane, so there are no atomics and the
// result is bit-reproducible.
#include "helix_common.hpp"
#include "kernels.hpp"

namespace helix {

constexpr int kPreprocessPasses = 4;   // rows in flight per lane group

// ------------------------------------------------------------------ preprocess
// One row of D bf16 is D/8 16-byte chunks; D/8 adjacent lanes own a row.  Besides the row
// sums the kernel rewrites LSE in the form the two gradient passes consume, so that neither
// spends a vector instruction per score element on it:
//   neg_delta_i = -sum_d dO_id * O_id      (becomes the initial accumulator of the dP product)
//   lse2_i      = LSE_i * log2(e)          (P = exp2(S * scale * log2(e) - lse2))
// Workgroup ids enumerate (slice, row block) in one dimension: no limit on B * H.
template <int D>
__global__ void __launch_bounds__(256)
bwd_preprocess_kernel(const __bf16* __restrict__ o, const __bf16* __restrict__ dO, const float* __restrict__ lse,
                      float* __restrict__ neg_delta, float* __restrict__ lse2, TensorMap mo, TensorMap mdo,
                      int H, int S, int blocks_per_head) {
  constexpr int LPR = D / 8;            // lanes per row
  constexpr int RPB = 256 / LPR;        // rows per workgroup pass
  constexpr int PASSES = kPreprocessPasses;
  const int tid = threadIdx.x;
  const int sub = tid % LPR;
  const int bh = blockIdx.x / blocks_per_head;
  const int row0 = (blockIdx.x - bh * blocks_per_head) * (RPB * PASSES) + tid / LPR;
  const __bf16* oh = o + head_offset(mo, bh, H);
  const __bf16* gh = dO + head_offset(mdo, bh, H);
  bf16x8 a[PASSES], b[PASSES];
#pragma unroll
  for (int p = 0; p < PASSES; p++) {
    const int r = row0 + p * RPB;
    if (r < S) {
      a[p] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(oh + (size_t)r * mo.row + sub * 8));
      b[p] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(gh + (size_t)r * mdo.row + sub * 8));
    }
  }
#pragma unroll
  for (int p = 0; p < PASSES; p++) {
    const int r = row0 + p * RPB;
    float s = 0.f;
    if (r < S) {
#pragma unroll
      for (int e = 0; e < 8; e++) s = fmaf((float)a[p][e], (float)b[p][e], s);
    }
#pragma unroll
    for (int off = LPR / 2; off >= 1; off >>= 1) s += __shfl_xor(s, off);
    if (sub == 0 && r < S) {
      neg_delta[(size_t)bh * S + r] = -s;
      lse2[(size_t)bh * S + r] = lse[(size_t)bh * S + r] * kLog2e;
    }
  }
}

hipError_t launch_bwd_preprocess(const void* o, const void* dO, const float* lse, float* neg_delta, float* lse2,
                                 const BwdMaps& maps, int B, int H, int S, int D, hipStream_t stream) {
  const int per = (256 / (D / 8)) * kPreprocessPasses;
  const int bph = (S + per - 1) / per;
  const unsigned grid = (unsigned)((long long)bph * B * H);
  if (D == 128)
    hipLaunchKernelGGL(bwd_preprocess_kernel<128>, dim3(grid), dim3(256), 0, stream, (const __bf16*)o, (const __bf16*)dO, lse,
                       neg_delta, lse2, maps.o, maps.dO, H, S, bph);
  else
    hipLaunchKernelGGL(bwd_preprocess_kernel<64>, dim3(grid), dim3(256), 0, stream, (const __bf16*)o, (const __bf16*)dO, lse,
                       neg_delta, lse2, maps.o, maps.dO, H, S, bph);
  return hipGetLastError();
}

// ------------------------------------------------------------------ delta of the first rows
// An unpipelined sweep in the dQ layout (a lane owns a query) that evaluates
// delta_i = sum_j p_ij dp_ij from its definition.  It runs on the first rows of every head,
// where attention is concentrated on few keys and the bf16 rounding of O would otherwise
// dominate delta.
template <int D, bool CAUSAL>
__global__ void __launch_bounds__(512, 1)
bwd_delta_head_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k, const __bf16* __restrict__ v,
                      const __bf16* __restrict__ dO, const float* __restrict__ lse, float* __restrict__ neg_delta_out,
                      BwdMaps maps, int BH, int H, int S, int T, float scale) {
  constexpr int BM = 256, BN = 64, NT = 512;
  constexpr int KS = D / 16;
  constexpr int TILE_BYTES = BN * D * 2;
  extern __shared__ __align__(16) char smem[];   // K[2] then V[2]

  const TileCoord tc = map_block(blockIdx.x, BH, T, true);
  if (!tc.valid) return;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int half = lane >> 5, n = lane & 31;
  const int q0 = tc.tile * BM;
  const int my_q = q0 + 32 * w + n;
  const __bf16* qh = q + head_offset(maps.q, tc.bh, H);
  const __bf16* gh = dO + head_offset(maps.dO, tc.bh, H);
  const __bf16* kh = k + head_offset(maps.k, tc.bh, H);
  const __bf16* vh = v + head_offset(maps.v, tc.bh, H);
  const float c = scale * kLog2e;

  bf16x8 qf[KS], gf[KS];
  float lse2;
  {
    const int row = my_q < S ? my_q : S - 1;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      qf[ks] = *reinterpret_cast<const bf16x8*>(qh + (size_t)row * maps.q.row + 16 * ks + 8 * half);
      gf[ks] = *reinterpret_cast<const bf16x8*>(gh + (size_t)row * maps.dO.row + 16 * ks + 8 * half);
    }
    lse2 = lse[(size_t)tc.bh * S + row] * kLog2e;
  }
  float dsum = 0.f;   // this lane's share of sum_j p_ij dp_ij

  const int q_end = (q0 + BM < S ? q0 + BM : S);
  const int n_tiles = CAUSAL ? (q_end + BN - 1) / BN : (S + BN - 1) / BN;
  const int wave_qmin = q0 + 32 * w, wave_qmax = wave_qmin + 31;

  TileStage<D, BN, NT> sk, sv;
  sk.fetch(kh, maps.k.row, 0, S, tid);
  sv.fetch(vh, maps.v.row, 0, S, tid);
  sk.commit(smem, tid);
  sv.commit(smem + 2 * TILE_BYTES, tid);
  __syncthreads();

  for (int j = 0; j < n_tiles; j++) {
    const char* kt = smem + (j & 1) * TILE_BYTES;
    const char* vt = smem + (2 + (j & 1)) * TILE_BYTES;
    const int k0 = j * BN;
    const bool more = j + 1 < n_tiles;
    if (more) {
      sk.fetch(kh, maps.k.row, k0 + BN, S, tid);
      sv.fetch(vh, maps.v.row, k0 + BN, S, tid);
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
          dsum = fmaf(p, pacc[e], dsum);
        }
      }
    }
    if (more) {
      sk.commit(smem + ((j + 1) & 1) * TILE_BYTES, tid);
      sv.commit(smem + (2 + ((j + 1) & 1)) * TILE_BYTES, tid);
    }
    __syncthreads();
  }

  dsum = half_sum(dsum);
  if (my_q < S && half == 0) neg_delta_out[(size_t)tc.bh * S + my_q] = -dsum;
}

template <int D, bool CAUSAL>
static hipError_t launch_delta_head_t(const void* q, const void* k, const void* v, const void* dO, const float* lse,
                                      float* delta_out, const BwdMaps& maps, int B, int H, int S, int rows,
                                      float scale, hipStream_t stream) {
  constexpr int BM = 256, BN = 64;
  const int T = (rows + BM - 1) / BM, BH = B * H;   // query tiles 0..T-1 of every head
  const unsigned grid = (unsigned)grid_blocks(BH, T);
  const size_t lds = 4 * BN * D * 2;
  auto kern = bwd_delta_head_kernel<D, CAUSAL>;
  static unsigned long long configured = 0;   // one static per template instantiation
  hipError_t e = allow_dynamic_lds(kern, lds, configured);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(512), lds, stream, (const __bf16*)q, (const __bf16*)k, (const __bf16*)v,
                     (const __bf16*)dO, lse, delta_out, maps, BH, H, S, T, scale);
  return hipGetLastError();
}

hipError_t launch_bwd_delta_head(const void* q, const void* k, const void* v, const void* dO,
                                 const float* lse, float* delta, const BwdMaps& maps, int B, int H, int S, int D,
                                 int rows, float scale, bool causal, hipStream_t stream) {
  if (rows <= 0) return hipSuccess;
  if (rows > S) rows = S;
  if (D == 128) return causal ? launch_delta_head_t<128, true>(q, k, v, dO, lse, delta, maps, B, H, S, rows, scale, stream)
                              : launch_delta_head_t<128, false>(q, k, v, dO, lse, delta, maps, B, H, S, rows, scale, stream);
  return causal ? launch_delta_head_t<64, true>(q, k, v, dO, lse, delta, maps, B, H, S, rows, scale, stream)
                : launch_delta_head_t<64, false>(q, k, v, dO, lse, delta, maps, B, H, S, rows, scale, stream);
}

}  // namespace helix

// dQ pass of the attention backward for gfx950 (Table 1, Attention column, "Backward B").
//
// Work split: a workgroup of 8 waves owns 256 query rows of one (batch, head) slice, 32 per
// wave, and sweeps the 64-key tiles the causal mask leaves visible.  Everything is kept
// transposed so that a lane owns ONE query (column l%32): its LSE and delta are plain
// per-lane scalars.  Per 32-key half tile h a wave evaluates with the 32x32x16 bf16 MFMA
//     S^T(h)  = K(h) Q^T            P^T  = exp2(S^T*c - lse2)           (c = scale*log2e)
//     dP^T(h) = V(h) dO^T - delta   dS^T = P^T o dP^T
// (lse2 = LSE*log2e and -delta come from the preprocess kernel; -delta, replicated over an
// accumulator, is the initial value of the dP^T product)
//     dQ^T   += K(h)^T bf16(dS^T)                                        (dQ scaled at the end)
// Q and dO fragments of the wave's queries stay in registers (B operands); K and V rows come
// from LDS as A operands, K a second time through the transposing LDS read.
//
// Schedule (see fwd.hip for why): software pipelined over the half tiles, one basic block of
// 3*D/16 hand-ordered slots per half step, each slot with one MFMA, the LDS read of the A
// operand needed four slots later and a share of the vector work:
//     slots  0.. 7   dP^T(h)   = V(h) dO^T      | P^T(h), second half of the exponentials
//     slots  8..15   S^T(h+1)  = K(h+1) Q^T     | dS^T(h) = P^T o dP^T, bf16 packs
//     slots 16..23   dQ^T     += K(h)^T dS^T(h) | P^T(h+1), first half of the exponentials
// K / V tiles are copied global -> LDS asynchronously into four stages (tile j and j+1
// resident, j+2 landing, j+3 being issued); one workgroup barrier per 64-key tile.  The last
// tile of every wave (the only one the causal mask cuts, or the ragged end of the sequence)
// runs through a plain, masked path.
#include "helix_common.hpp"
#include "kernels.hpp"

namespace helix {

namespace {

constexpr int kRing = 4;   // A operands in flight

// One pipelined half step.  B_HALF: h is the second half of its tile, so the block ahead
// (h+1) lives in the next tile: the lane addresses move on by stage_step as soon as their
// last read of the current tile is out.  On entry s_cur = S^T(h) with entries 0..7 already
// exponentiated and ring = first four V(h) operands; on exit the same holds for s_next.
template <int D, bool B_HALF, typename Copy>
__device__ __forceinline__ void dq_half_step(const Copy& copy_tile, f32x16& s_cur, f32x16& s_next, bf16x8 (&ring)[kRing],
                                             const bf16x8 (&qf)[D / 16], const bf16x8 (&gf)[D / 16],
                                             f32x16 (&dqacc)[D / 32], uint32_t (&ab)[D / 16], uint32_t (&at)[D / 32][2],
                                             int stage_step, float c, float lse2, const f32x16& nd) {
  constexpr int KS = D / 16, DB = D / 32, NS = 3 * KS, R = kRing;
  constexpr int TILE = 64 * D * 2, HALF = 32 * D * 2;
  constexpr int V_CUR = TILE + (B_HALF ? HALF : 0);      // V rows of h, stage layout [K tile][V tile]
  constexpr int K_NEXT = B_HALF ? 0 : HALF;              // K rows of h+1 (after the move when B_HALF)
  constexpr int K_CUR_T = B_HALF ? HALF : 0;             // K rows of h for the transposing reads
  constexpr int V_NEXT = TILE + (B_HALF ? 0 : HALF);     // V rows of h+1
  constexpr int EV = 8 / KS > 0 ? 8 / KS : 1;            // exponentials per slot in the first / last group
  constexpr int ED = 16 / KS;                            // dS elements per slot in the middle group
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16 dp;
  uint32_t sk[8];   // bf16 pairs of dS^T(h)

#pragma unroll
  for (int s = 0; s < NS; s++) {
    // ---- matrix work
    if (s < KS) {
      dp = mfma32(ring[s % R], gf[s], s == 0 ? nd : dp);
    } else if (s < 2 * KS) {
      s_next = mfma32(ring[s % R], qf[s - KS], s == KS ? zero : s_next);
    } else {
      const int i = s - 2 * KS;
      const u32x4 b = {sk[4 * (i / DB)], sk[4 * (i / DB) + 1], sk[4 * (i / DB) + 2], sk[4 * (i / DB) + 3]};
      dqacc[i % DB] = mfma32(ring[s % R], __builtin_bit_cast(bf16x8, b), dqacc[i % DB]);
    }
    if (s == 1) copy_tile();   // tile copies are issued under the first MFMAs, not in front of them
    // ---- lane addresses move to the next tile
    if (B_HALF && s == KS - R) {
#pragma unroll
      for (int ks = 0; ks < KS; ks++) ab[ks] += stage_step;
    }
    if (B_HALF && s == NS - R) {
#pragma unroll
      for (int db = 0; db < DB; db++) { at[db][0] += stage_step; at[db][1] += stage_step; }
    }
    // ---- A operand of slot s + R
    {
      const int u = s + R;
      if (u < KS) ring[s % R] = lds_b128(ab[u], V_CUR);
      else if (u < 2 * KS) ring[s % R] = lds_b128(ab[u - KS], K_NEXT);
      else if (u < 3 * KS) {
        const int i = u - 2 * KS;
        ring[s % R] = lds_tr_pair(at[i % DB][0], at[i % DB][1], K_CUR_T + 16 * (i / DB) * D * 2);
      } else {
        ring[s % R] = lds_b128(ab[u - NS], V_NEXT);
      }
    }
    // ---- vector work
    if (s < KS) {
#pragma unroll
      for (int e = 8 + s * EV; e < 8 + (s + 1) * EV && e < 16; e++)
        s_cur[e] = __builtin_amdgcn_exp2f(fmaf(s_cur[e], c, -lse2));
    } else if (s < 2 * KS) {
#pragma unroll
      for (int e = (s - KS) * ED; e < (s - KS + 1) * ED; e += 2) {
        const float d0 = s_cur[e] * dp[e];
        const float d1 = s_cur[e + 1] * dp[e + 1];
        sk[e / 2] = pack_bf16_pair(d0, d1);
      }
    } else {
#pragma unroll
      for (int e = (s - 2 * KS) * EV; e < (s - 2 * KS + 1) * EV && e < 8; e++)
        s_next[e] = __builtin_amdgcn_exp2f(fmaf(s_next[e], c, -lse2));
    }
    __builtin_amdgcn_sched_barrier(0);
  }
}

}  // namespace

template <int D, bool CAUSAL>
__global__ void __launch_bounds__(512, 1)
bwd_dq_pipe_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k, const __bf16* __restrict__ v,
                   const __bf16* __restrict__ dO, const float* __restrict__ lse2_all, const float* __restrict__ neg_delta,
                   __bf16* __restrict__ dq, BwdMaps maps, int BH, int H, int S, int T, float scale) {
  constexpr int BM = 256, BN = 64;
  constexpr int KS = D / 16, DB = D / 32;
  constexpr int TILE = BN * D * 2, HALF = 32 * D * 2;
  constexpr int STAGE = 2 * TILE;   // [K tile][V tile]; tile j lives in stage j % 4
  extern __shared__ __align__(16) char smem[];

  const TileCoord tc = map_block(blockIdx.x, BH, T, true);
  if (!tc.valid) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int half = lane >> 5, n = lane & 31;
  const int q0 = tc.tile * BM;
  const int my_q = q0 + 32 * w + n;
  const __bf16* qh = q + head_offset(maps.q, tc.bh, H);
  const __bf16* gh = dO + head_offset(maps.dO, tc.bh, H);
  const __bf16* kh = k + head_offset(maps.k, tc.bh, H);
  const __bf16* vh = v + head_offset(maps.v, tc.bh, H);
  const float c = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, scale * kLog2e)));
  const uint32_t base = lds_base(smem);

  bf16x8 qf[KS], gf[KS];
  float lse2;
  f32x16 nd;     // -delta of this lane's query in every accumulator register
  {
    const int row = my_q < S ? my_q : S - 1;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      qf[ks] = *reinterpret_cast<const bf16x8*>(qh + (size_t)row * maps.q.row + 16 * ks + 8 * half);
      gf[ks] = *reinterpret_cast<const bf16x8*>(gh + (size_t)row * maps.dO.row + 16 * ks + 8 * half);
    }
    lse2 = lse2_all[(size_t)tc.bh * S + row];
    const float dl = neg_delta[(size_t)tc.bh * S + row];
#pragma unroll
    for (int e = 0; e < 16; e++) nd[e] = dl;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) { pin(qf[ks]); pin(gf[ks]); }
    pin(lse2); pin(nd);
  }
  f32x16 dqacc[DB];
#pragma unroll
  for (int db = 0; db < DB; db++)
#pragma unroll
    for (int e = 0; e < 16; e++) dqacc[db][e] = 0.f;

  const int q_end = (q0 + BM < S ? q0 + BM : S);
  const int n_tiles = CAUSAL ? (q_end + BN - 1) / BN : (S + BN - 1) / BN;
  const int wave_qmin = q0 + 32 * w, wave_qmax = wave_qmin + 31;
  // Tiles this wave works on (n_w) and how many of them need no mask (n_full >= n_w - 1).
  int n_w, n_full;
  if (wave_qmin >= S) { n_w = 0; n_full = 0; }
  else if (CAUSAL) { n_w = (wave_qmax < S ? wave_qmax : S - 1) / BN + 1; n_full = (wave_qmin + 1) / BN; }
  else { n_w = n_tiles; n_full = S / BN; }

  const TileLoader<D, BN, 8> kload(lane, w, maps.k.row), vload(lane, w, maps.v.row);
  constexpr int NDMA = decltype(kload)::N + decltype(vload)::N;   // copy instructions per wave and tile: what copy_tile() issues
  int j = 0, st = 0;   // tile and its stage (j % 4)
  auto copy_tile = [&](int jj, int stage) __attribute__((always_inline)) {
    kload.issue(kh, jj * BN, S, base + stage * STAGE);
    vload.issue(vh, jj * BN, S, base + stage * STAGE + TILE);
  };
  auto copy_ahead = [&]() __attribute__((always_inline)) {
    if (j + 3 < n_tiles) copy_tile(j + 3, (st + 3) & 3);   // replaces tile j-1
  };
  auto finish_tile = [&]() __attribute__((always_inline)) {
    // tiles up to j+2 have landed before the next iteration (which reads j+1 and j+2) starts
    if (j + 3 < n_tiles) wait_tile_loads_except<NDMA>();
    else wait_tile_loads();
    __syncthreads();
    st = (st + 1) & 3;
  };
  copy_tile(0, 0);
  if (n_tiles > 1) copy_tile(1, 1);
  if (n_tiles > 2) copy_tile(2, 2);
  wait_tile_loads();
  __syncthreads();

  // Lane addresses in stage 0: ab = row n, contraction step ks (K tile; the V tile is TILE
  // bytes further); at = transposing reads of the K tile.
  uint32_t ab[KS], at[DB][2];
#pragma unroll
  for (int ks = 0; ks < KS; ks++) ab[ks] = base + lds_chunk_off<D>(n, 2 * ks + half);
#pragma unroll
  for (int db = 0; db < DB; db++) {
    int o0, o1;
    tr_pair_offsets<D>(lane, db, o0, o1);
    at[db][0] = base + o0;
    at[db][1] = base + o1;
  }

  // Prime: S^T of the first half tile (entries 0..7 exponentiated) and its first V operands.
  f32x16 sa, sb;
  bf16x8 ring[kRing];
  if (n_w > 0) {
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    sa = zero;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) sa = mfma32(lds_b128(ab[ks], 0), qf[ks], sa);
#pragma unroll
    for (int e = 0; e < 8; e++) sa[e] = __builtin_amdgcn_exp2f(fmaf(sa[e], c, -lse2));
#pragma unroll
    for (int i = 0; i < kRing; i++) ring[i] = lds_b128(ab[i], TILE);
  }

  const auto no_copy = []() {};
  for (; j < n_w - 1; j++) {
    // A complete tile j+3 is copied by a handful of instructions issued inside the half step; a
    // ragged one (the last of the sequence) takes the general path in front of it.
    const bool whole = j + 3 < n_tiles && (j + 4) * BN <= S;
    if (!whole) copy_ahead();
    const __bf16* kt = kload.tile_ptr(kh, (j + 3) * BN);
    const __bf16* vt = vload.tile_ptr(vh, (j + 3) * BN);
    const uint32_t dst = base + ((st + 3) & 3) * STAGE;
    const auto copy_whole = [&]() __attribute__((always_inline)) {
      if (whole) {
        kload.issue_whole(kt, dst);
        vload.issue_whole(vt, dst + TILE);
      }
    };
    const int stage_step = (st == 3) ? -3 * STAGE : STAGE;
    dq_half_step<D, false>(copy_whole, sa, sb, ring, qf, gf, dqacc, ab, at, stage_step, c, lse2, nd);
    dq_half_step<D, true>(no_copy, sb, sa, ring, qf, gf, dqacc, ab, at, stage_step, c, lse2, nd);
    finish_tile();
  }

  for (; j < n_tiles; j++) {
    copy_ahead();
    if (j == n_w - 1) {
      // plain path: the last tile of this wave, masked unless the sequence ends on a tile
      // edge.  sa holds S^T of its first half with entries 0..7 already exponentiated; ab and
      // at point at this tile.
      const int k0 = j * BN;
      const bool masked = j >= n_full;
#pragma unroll
      for (int kb = 0; kb < 2; kb++) {
        f32x16 sacc, pacc;
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (kb == 0) {
          sacc = sa;
#pragma unroll
          for (int e = 8; e < 16; e++) sacc[e] = __builtin_amdgcn_exp2f(fmaf(sacc[e], c, -lse2));
        } else {
          sacc = zero;
#pragma unroll
          for (int ks = 0; ks < KS; ks++) sacc = mfma32(lds_b128(ab[ks], HALF), qf[ks], sacc);
#pragma unroll
          for (int e = 0; e < 16; e++) sacc[e] = __builtin_amdgcn_exp2f(fmaf(sacc[e], c, -lse2));
        }
        pacc = nd;
#pragma unroll
        for (int ks = 0; ks < KS; ks++) pacc = mfma32(lds_b128(ab[ks], TILE + kb * HALF), gf[ks], pacc);
#pragma unroll
        for (int e = 0; e < 16; e++) {
          float p = sacc[e];
          if (masked) {
            const int key = k0 + 32 * kb + 8 * (e >> 2) + 4 * half + (e & 3);
            p = (CAUSAL ? key <= my_q : key < S) ? p : 0.f;
          }
          pacc[e] = p * pacc[e];
        }
#pragma unroll
        for (int t = 0; t < 2; t++) {
          const bf16x8 sbk = pack_half(pacc, t);
#pragma unroll
          for (int db = 0; db < DB; db++)
            dqacc[db] = mfma32(lds_tr_pair(at[db][0], at[db][1], kb * HALF + 16 * t * D * 2), sbk, dqacc[db]);
        }
      }
    }
    finish_tile();
  }

  if (my_q < S) {
    __bf16* row = dq + head_offset(maps.dq, tc.bh, H) + (size_t)my_q * maps.dq.row;
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

template <int D, bool CAUSAL>
static hipError_t launch_dq_pipe_t(const void* q, const void* k, const void* v, const void* dO,
                                   const float* lse2, const float* neg_delta, void* dq, const BwdMaps& maps,
                                   int B, int H, int S, float scale, hipStream_t stream) {
  constexpr int BM = 256, BN = 64;
  const int T = (S + BM - 1) / BM, BH = B * H;
  const unsigned grid = (unsigned)grid_blocks(BH, T);
  const size_t lds = 4 * 2 * BN * D * 2;
  auto kern = bwd_dq_pipe_kernel<D, CAUSAL>;
  static unsigned long long configured = 0;   // one static per template instantiation
  hipError_t e = allow_dynamic_lds(kern, lds, configured);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(512), lds, stream, (const __bf16*)q, (const __bf16*)k, (const __bf16*)v,
                     (const __bf16*)dO, lse2, neg_delta, (__bf16*)dq, maps, BH, H, S, T, scale);
  return hipGetLastError();
}

hipError_t launch_bwd_dq(const void* q, const void* k, const void* v, const void* dO,
                         const float* lse2, const float* neg_delta, void* dq, const BwdMaps& maps,
                         int B, int H, int S, int D, float scale, bool causal, hipStream_t stream) {
  if (D == 128) return causal ? launch_dq_pipe_t<128, true>(q, k, v, dO, lse2, neg_delta, dq, maps, B, H, S, scale, stream)
                              : launch_dq_pipe_t<128, false>(q, k, v, dO, lse2, neg_delta, dq, maps, B, H, S, scale, stream);
  return causal ? launch_dq_pipe_t<64, true>(q, k, v, dO, lse2, neg_delta, dq, maps, B, H, S, scale, stream)
                : launch_dq_pipe_t<64, false>(q, k, v, dO, lse2, neg_delta, dq, maps, B, H, S, scale, stream);
}

}  // namespace helix

// dK / dV pass of the attention backward for gfx950 (Table 1, Attention column, "Backward B"),
// one wave per SIMD.  The launcher at the end uses it for head dimension 64; head dimension 128
// goes to the two-waves-per-SIMD kernel in bwd_dkdv_pair.hip (same arithmetic).
//
// Work split: a workgroup of 4 waves owns 128 keys of one (batch, head) slice, 32 keys per
// wave, and sweeps the 64-row query tiles that see them.  Per 32-row query block b a wave
// evaluates, with the 32x32x16 bf16 MFMA and a lane owning ONE key (column l%32):
//     S(b)  = Q(b) K^T                P(b)  = exp2(S(b)*c - lse2)           (c = scale*log2e)
//     dP(b) = dO(b) V^T - delta       dS(b) = P(b) o dP(b)
// (lse2 = LSE*log2e and -delta come precomputed from the preprocess kernel; -delta is the
// initial accumulator of the dP product, so neither costs an instruction per score element)
//     dV^T += dO(b)^T bf16(P(b))      dK^T += Q(b)^T bf16(dS(b))            (dK scaled at the end)
// K and V fragments of the wave's keys stay in registers (B operands of S and dP); bf16(P),
// bf16(dS) in accumulator layout are the B operands of the last two products; Q, dO come
// from LDS as A operands, row-major for S / dP and through the transposing LDS read for
// dV / dK.  One wave per SIMD (up to 512 registers) so that both fp32 accumulators
// (32 keys x D x 2) and the K, V fragments fit.
//
// Schedule.  A second MFMA queued behind a running one stalls the vector-ALU port of the
// SIMD, so matrix and vector work only overlap when they alternate in one instruction
// stream.  The sweep is software pipelined over the blocks; a step for block b is ONE basic
// block of 4*D/16 hand-ordered slots, each with one MFMA, the LDS read of the A operand
// needed four slots later, and a share of the vector work:
//     slots  0.. 7   S(b+1)           | dS(b) = P(b) o dP(b), bf16 packs of P(b), dS(b)
//     slots  8..15   dP(b+1)          |   (one element per slot)
//     slots 16..23   dV^T += ..P(b)   | P(b+1) = exp2(S(b+1)*c - lse2)
//     slots 24..31   dK^T += ..dS(b)  |   (one element per slot)
// Q / dO / lse2 / -delta tiles are copied global -> LDS asynchronously into four stages: while
// tile t is worked on, tile t+1 (which the second step of the iteration already reads) is
// resident too, tile t+2 may still be landing and tile t+3 is being issued; one workgroup
// barrier per 64-row tile.  Blocks cut by the causal diagonal
// (the first two tiles of every key tile) and a ragged last tile run through a plain,
// masked path.  No atomics: every dK / dV element is produced by exactly one lane.
#include "helix_common.hpp"
#include "kernels.hpp"

namespace helix {

namespace {

constexpr int kRing = 4;   // A operands in flight

// 64 fp32 values (one per lane) global -> LDS, asynchronously.
__device__ __forceinline__ void dma_dword(const float* base, uint32_t lane_byte_off, uint32_t lds_dst) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
               :: "v"(lane_byte_off), "s"(uniform_ptr(base)), "s"(__builtin_amdgcn_readfirstlane(lds_dst)) : "memory");
}

__device__ __forceinline__ f32x4 lds_f32x4(uint32_t addr, int imm) {
  return *reinterpret_cast<const __attribute__((address_space(3))) f32x4*>(
      reinterpret_cast<const __attribute__((address_space(3))) char*>((uintptr_t)addr) + imm);
}

// Four consecutive groups of four accumulator registers as one accumulator.
__device__ __forceinline__ f32x16 join4(const f32x4 (&x)[4]) {
  f32x16 r;
#pragma unroll
  for (int g = 0; g < 4; g++)
#pragma unroll
    for (int e = 0; e < 4; e++) r[4 * g + e] = x[g][e];
  return r;
}

template <int D>
struct Geometry {
  static constexpr int KS = D / 16, DB = D / 32;
  static constexpr int TILE = 64 * D * 2;            // one 64-row bf16 tile
  static constexpr int ROWS32 = 32 * D * 2;          // bytes of 32 rows
  static constexpr int STATS = 2 * TILE;             // per-wave copies of lse2[64], -delta[64] follow Q, dO
  static constexpr int STAGE = 2 * TILE + 4 * 512;
  static constexpr int NSTAGE = 4;
};

// Lane state of the pipelined path.
template <int D>
struct Pipe {
  static constexpr int KS = D / 16, DB = D / 32;
  uint32_t aq[KS];        // Q operand ks, row n of the tile that holds the block AHEAD (b+1)
  uint32_t at[DB][2];     // transposing-read addresses in the tile that holds the CURRENT block b
  uint32_t astat;         // this wave's lse2 / -delta copies of the tile that holds block b+1
  bf16x8 ring[kRing];     // A operands of the next four slots
  f32x4 st_nd[4];         // -delta of the block ahead, rows 8g + 4*half + (0..3)
  f32x4 st_l2[4];         // lse2 of the block ahead, same rows
};

// One pipelined step for block b (see the header comment).  ODD: b is the second block of its
// tile, so the block ahead starts the next tile.  On entry sp_cur = P(b) (fp32), dp_cur =
// dP(b) (delta already subtracted), pipe.ring = first Q operands of block b+1; on exit the
// same holds for block b+1 in sp_next / dp_next.
template <int D, bool ODD>
__device__ __forceinline__ void dkdv_step(const f32x16& sp_cur, const f32x16& dp_cur, f32x16& sp_next, f32x16& dp_next,
                                          Pipe<D>& pp, const bf16x8 (&kf)[D / 16], const bf16x8 (&vf)[D / 16],
                                          f32x16 (&dkacc)[D / 32], f32x16 (&dvacc)[D / 32], int stage_step, float c) {
  using G = Geometry<D>;
  constexpr int KS = G::KS, DB = G::DB, NS = 4 * KS, R = kRing;
  constexpr int AHEAD_ROWS = ODD ? 0 : 32;                 // block b+1 inside its tile
  constexpr int AHEAD = AHEAD_ROWS * D * 2;
  constexpr int BEHIND = ODD ? G::ROWS32 : 0;              // block b inside its tile
  constexpr int NEXT_AHEAD = ODD ? G::ROWS32 : 0;          // block b+2 inside its tile
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  uint32_t pk[8], sk[8];   // bf16 pairs of P(b) and dS(b)
  float ds_prev = 0.f, p_prev = 0.f;

#pragma unroll
  for (int s = 0; s < NS; s++) {
    // ---- matrix work of this slot
    if (s < KS) {
      sp_next = mfma32(pp.ring[s % R], kf[s], s == 0 ? zero : sp_next);
    } else if (s < 2 * KS) {
      dp_next = mfma32(pp.ring[s % R], vf[s - KS], s == KS ? join4(pp.st_nd) : dp_next);
    } else if (s < 3 * KS) {
      const int i = s - 2 * KS;
      const u32x4 b = {pk[4 * (i / DB)], pk[4 * (i / DB) + 1], pk[4 * (i / DB) + 2], pk[4 * (i / DB) + 3]};
      dvacc[i % DB] = mfma32(pp.ring[s % R], __builtin_bit_cast(bf16x8, b), dvacc[i % DB]);
    } else {
      const int i = s - 3 * KS;
      const u32x4 b = {sk[4 * (i / DB)], sk[4 * (i / DB) + 1], sk[4 * (i / DB) + 2], sk[4 * (i / DB) + 3]};
      dkacc[i % DB] = mfma32(pp.ring[s % R], __builtin_bit_cast(bf16x8, b), dkacc[i % DB]);
    }
    // ---- lane addresses move on to the next tile once their last read of this one is out
    if (!ODD && s == 2 * KS) {
#pragma unroll
      for (int ks = 0; ks < KS; ks++) pp.aq[ks] += stage_step;
    }
    if (ODD && s == NS - R) {
#pragma unroll
      for (int db = 0; db < DB; db++) { pp.at[db][0] += stage_step; pp.at[db][1] += stage_step; }
    }
    // ---- A operand of slot s + R
    {
      const int u = s + R;
      if (u < KS) pp.ring[s % R] = lds_b128(pp.aq[u], AHEAD);
      else if (u < 2 * KS) pp.ring[s % R] = lds_b128(pp.aq[u - KS], AHEAD + G::TILE);
      else if (u < 3 * KS) {
        const int i = u - 2 * KS;
        pp.ring[s % R] = lds_tr_pair(pp.at[i % DB][0], pp.at[i % DB][1], BEHIND + 16 * (i / DB) * D * 2 + G::TILE);
      } else if (u < 4 * KS) {
        const int i = u - 3 * KS;
        pp.ring[s % R] = lds_tr_pair(pp.at[i % DB][0], pp.at[i % DB][1], BEHIND + 16 * (i / DB) * D * 2);
      } else {
        pp.ring[s % R] = lds_b128(pp.aq[u - NS], NEXT_AHEAD);
      }
    }
    // ---- lse2 / -delta of the block ahead
    if (s < 4) pp.st_nd[s] = lds_f32x4(pp.astat, 256 + (AHEAD_ROWS + 8 * s) * 4);
    if (s >= KS && s < KS + 4) pp.st_l2[s - KS] = lds_f32x4(pp.astat, (AHEAD_ROWS + 8 * (s - KS)) * 4);
    // ---- vector work of this slot
    if (s < 2 * KS) {
      // dS(b) = P(b) o dP(b) and the bf16 packs of P(b), dS(b)
#pragma unroll
      for (int e = 0; e < 16; e++) {
        if (e * 2 * KS / 16 != s) continue;
        const float ds = sp_cur[e] * dp_cur[e];
        if (e & 1) { pk[e / 2] = pack_bf16_pair(p_prev, sp_cur[e]); sk[e / 2] = pack_bf16_pair(ds_prev, ds); }
        else { p_prev = sp_cur[e]; ds_prev = ds; }
      }
    } else {
      // P(b+1) = exp2(S(b+1)*c - lse2), in place
#pragma unroll
      for (int e = 0; e < 16; e++) {
        if (e * 2 * KS / 16 != s - 2 * KS) continue;
        sp_next[e] = __builtin_amdgcn_exp2f(fmaf(sp_next[e], c, -pp.st_l2[e / 4][e % 4]));
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  if (!ODD) pp.astat += stage_step;
}

}  // namespace

template <int D, bool CAUSAL>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
bwd_dkdv_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k, const __bf16* __restrict__ v,
                const __bf16* __restrict__ dO, const float* __restrict__ lse2, const float* __restrict__ neg_delta,
                __bf16* __restrict__ dk, __bf16* __restrict__ dv, BwdMaps maps, int BH, int H, int S, int T,
                float scale) {
  using G = Geometry<D>;
  constexpr int BN = 128, BM = 64, KS = G::KS, DB = G::DB;
  extern __shared__ __align__(16) char smem[];

  const TileCoord tc = map_block(blockIdx.x, BH, T, false);
  if (!tc.valid) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int half = lane >> 5, n = lane & 31;
  const int n0 = tc.tile * BN;
  const int wave_kmin = n0 + 32 * w;
  const int my_key = wave_kmin + n;
  const __bf16* qh = q + head_offset(maps.q, tc.bh, H);
  const __bf16* gh = dO + head_offset(maps.dO, tc.bh, H);
  const __bf16* kh = k + head_offset(maps.k, tc.bh, H);
  const __bf16* vh = v + head_offset(maps.v, tc.bh, H);
  const float* lse_h = lse2 + (size_t)tc.bh * S;
  const float* delta_h = neg_delta + (size_t)tc.bh * S;
  const float c = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, scale * kLog2e)));
  const uint32_t base = lds_base(smem);

  // K^T and V^T operand fragments of this lane's key (columns of S and dP).
  bf16x8 kf[KS], vf[KS];
  {
    const int row = my_key < S ? my_key : S - 1;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      kf[ks] = *reinterpret_cast<const bf16x8*>(kh + (size_t)row * maps.k.row + 16 * ks + 8 * half);
      vf[ks] = *reinterpret_cast<const bf16x8*>(vh + (size_t)row * maps.v.row + 16 * ks + 8 * half);
    }
#pragma unroll
    for (int ks = 0; ks < KS; ks++) { pin(kf[ks]); pin(vf[ks]); }
  }
  f32x16 dkacc[DB], dvacc[DB];
#pragma unroll
  for (int db = 0; db < DB; db++)
#pragma unroll
    for (int e = 0; e < 16; e++) { dkacc[db][e] = 0.f; dvacc[db][e] = 0.f; }

  const int m_start = CAUSAL ? n0 : 0;                       // first query row that sees a key of this tile
  const int nt = (S - m_start + BM - 1) / BM;                // query tiles to sweep
  // Plain (masked) path: the tiles the causal diagonal crosses and a ragged last tile.
  int t_lo = CAUSAL ? 2 : 0;
  if (t_lo > nt) t_lo = nt;
  int t_hi = ((S - m_start) % BM != 0) ? nt - 1 : nt;
  if (t_hi < t_lo) t_hi = t_lo;

  const TileLoader<D, BM, 4> qload(lane, w, maps.q.row), gload(lane, w, maps.dO.row);
  constexpr int kStatCopies = 2;                             // lse2 and -delta of the tile's rows, one instruction each
  constexpr int NDMA = decltype(qload)::N + decltype(gload)::N + kStatCopies;   // copy instructions per wave and tile: what copy_tile() issues
  int t = 0, st = 0;                                          // tile and its stage (t % 4)
  auto copy_tile = [&](int tt, int stage) __attribute__((always_inline)) {
    const uint32_t sb = base + stage * G::STAGE;
    const int row0 = m_start + tt * BM;
    qload.issue(qh, row0, S, sb);
    gload.issue(gh, row0, S, sb + G::TILE);
    int r = row0 + lane;
    r = r < S ? r : S - 1;
    const float* const stat[kStatCopies] = {lse_h, delta_h};
#pragma unroll
    for (int i = 0; i < kStatCopies; i++) dma_dword(stat[i], (uint32_t)r * 4, sb + G::STATS + w * 512 + 256 * i);
  };
  auto copy_ahead = [&]() __attribute__((always_inline)) {
    if (t + 3 < nt) copy_tile(t + 3, (st + 3) & 3);   // replaces tile t-1
  };
  auto finish_tile = [&]() __attribute__((always_inline)) {
    // tiles up to t+2 must have landed before the next iteration starts (it reads t+1 and
    // t+2); the copy of tile t+3 issued in this iteration may stay in flight
    if (t + 3 < nt) wait_tile_loads_except<NDMA>();
    else wait_tile_loads();
    __syncthreads();
    st = (st + 1) & 3;
  };
  copy_tile(0, 0);
  if (nt > 1) copy_tile(1, 1);
  if (nt > 2) copy_tile(2, 2);
  wait_tile_loads();
  __syncthreads();

  // One 32-row block through the plain path: everything in program order, masks applied.
  auto plain_block = [&](int blk) __attribute__((always_inline)) {
    const int r0 = m_start + t * BM + 32 * blk;   // global row of the block's first query
    const char* qt = smem + st * G::STAGE;
    const char* gt = qt + G::TILE;
    const float* lse_t = reinterpret_cast<const float*>(qt + G::STATS + w * 512);
    const float* dlt_t = lse_t + 64;
    f32x16 sacc, pacc;
#pragma unroll
    for (int e = 0; e < 16; e++) { sacc[e] = 0.f; pacc[e] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < KS; ks++) sacc = mfma32(lds_operand<D>(qt, 32 * blk + n, ks, half), kf[ks], sacc);
#pragma unroll
    for (int ks = 0; ks < KS; ks++) pacc = mfma32(lds_operand<D>(gt, 32 * blk + n, ks, half), vf[ks], pacc);
#pragma unroll
    for (int g = 0; g < 4; g++) {
      const f32x4 l4 = *reinterpret_cast<const f32x4*>(lse_t + 32 * blk + 8 * g + 4 * half);
      const f32x4 d4 = *reinterpret_cast<const f32x4*>(dlt_t + 32 * blk + 8 * g + 4 * half);
#pragma unroll
      for (int e4 = 0; e4 < 4; e4++) {
        const int e = 4 * g + e4;
        const int row = r0 + 8 * g + 4 * half + e4;
        float p = __builtin_amdgcn_exp2f(fmaf(sacc[e], c, -l4[e4]));
        const bool ok = (!CAUSAL || my_key <= row) && row < S;
        p = ok ? p : 0.f;
        sacc[e] = p;
        pacc[e] = p * (pacc[e] + d4[e4]);
      }
    }
#pragma unroll
    for (int tt = 0; tt < 2; tt++) {
      const bf16x8 pb = pack_half(sacc, tt);
      const bf16x8 sb = pack_half(pacc, tt);
#pragma unroll
      for (int db = 0; db < DB; db++) {
        dvacc[db] = mfma32(lds_operand_tr<D>(gt, 32 * blk + 16 * tt, 32 * db, lane), pb, dvacc[db]);
        dkacc[db] = mfma32(lds_operand_tr<D>(qt, 32 * blk + 16 * tt, 32 * db, lane), sb, dkacc[db]);
      }
    }
  };
  auto plain_tile = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int blk = 0; blk < 2; blk++) {
      const int r0 = m_start + t * BM + 32 * blk;
      if (CAUSAL && r0 + 31 < wave_kmin) continue;   // every key of the wave is masked for these rows
      plain_block(blk);
    }
  };

  for (; t < t_lo; t++) { copy_ahead(); plain_tile(); finish_tile(); }

  if (t < t_hi) {
    // ---- prime the pipeline with block 2t: P, dP, delta, first Q operands of block 2t+1
    Pipe<D> pp;
    const uint32_t sbase = base + st * G::STAGE;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) pp.aq[ks] = sbase + lds_chunk_off<D>(n, 2 * ks + half);
#pragma unroll
    for (int db = 0; db < DB; db++) {
      int o0, o1;
      tr_pair_offsets<D>(lane, db, o0, o1);
      pp.at[db][0] = sbase + o0;
      pp.at[db][1] = sbase + o1;
    }
    pp.astat = sbase + G::STATS + w * 512 + half * 16;
    f32x16 spA, dpA, spB, dpB;
    {
      const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int g = 0; g < 4; g++) {
        pp.st_l2[g] = lds_f32x4(pp.astat, 8 * g * 4);
        pp.st_nd[g] = lds_f32x4(pp.astat, 256 + 8 * g * 4);
      }
      spA = zero; dpA = join4(pp.st_nd);
#pragma unroll
      for (int ks = 0; ks < KS; ks++) spA = mfma32(lds_b128(pp.aq[ks], 0), kf[ks], spA);
#pragma unroll
      for (int ks = 0; ks < KS; ks++) dpA = mfma32(lds_b128(pp.aq[ks], G::TILE), vf[ks], dpA);
#pragma unroll
      for (int e = 0; e < 16; e++)
        spA[e] = __builtin_amdgcn_exp2f(fmaf(spA[e], c, -pp.st_l2[e / 4][e % 4]));
#pragma unroll
      for (int i = 0; i < kRing; i++) pp.ring[i] = lds_b128(pp.aq[i], G::ROWS32);
    }
    for (; t < t_hi; t++) {
      copy_ahead();
      const int stage_step = (st == 3) ? -3 * G::STAGE : G::STAGE;
      dkdv_step<D, false>(spA, dpA, spB, dpB, pp, kf, vf, dkacc, dvacc, stage_step, c);
      dkdv_step<D, true>(spB, dpB, spA, dpA, pp, kf, vf, dkacc, dvacc, stage_step, c);
      finish_tile();
    }
  }

  for (; t < nt; t++) { copy_ahead(); plain_tile(); finish_tile(); }

  if (my_key < S) {
    __bf16* dkrow = dk + head_offset(maps.dk, tc.bh, H) + (size_t)my_key * maps.dk.row;
    __bf16* dvrow = dv + head_offset(maps.dv, tc.bh, H) + (size_t)my_key * maps.dv.row;
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
                                const float* lse2, const float* neg_delta, void* dk, void* dv, const BwdMaps& maps,
                                int B, int H, int S, float scale, hipStream_t stream) {
  constexpr int BN = 128;
  const int T = (S + BN - 1) / BN, BH = B * H;
  const unsigned grid = (unsigned)grid_blocks(BH, T);
  const size_t lds = Geometry<D>::NSTAGE * Geometry<D>::STAGE;
  auto kern = bwd_dkdv_kernel<D, CAUSAL>;
  static unsigned long long configured = 0;   // one static per template instantiation
  hipError_t e = allow_dynamic_lds(kern, lds, configured);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, stream, (const __bf16*)q, (const __bf16*)k, (const __bf16*)v,
                     (const __bf16*)dO, lse2, neg_delta, (__bf16*)dk, (__bf16*)dv, maps, BH, H, S, T, scale);
  return hipGetLastError();
}

hipError_t launch_bwd_dkdv(const void* q, const void* k, const void* v, const void* dO,
                           const float* lse2, const float* neg_delta, void* dk, void* dv, const BwdMaps& maps,
                           int B, int H, int S, int D, float scale, bool causal, hipStream_t stream) {
  // Head dimension 128 has its own kernel with two waves per SIMD; this one serves head dimension 64.
  if (D == 128) return launch_bwd_dkdv_pair(q, k, v, dO, lse2, neg_delta, dk, dv, maps, B, H, S, scale, causal, stream);
  return causal ? launch_dkdv_t<64, true>(q, k, v, dO, lse2, neg_delta, dk, dv, maps, B, H, S, scale, stream)
                : launch_dkdv_t<64, false>(q, k, v, dO, lse2, neg_delta, dk, dv, maps, B, H, S, scale, stream);
}

}  // namespace helix

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
//
// Schedule.  On this chip a second MFMA queued behind a running one stalls the vector-ALU
// port of the whole SIMD, so matrix and vector work only overlap when they alternate inside
// one instruction stream.  The sweep is therefore software pipelined over 32-key half tiles
// h = 0, 1, 2, ... and every half step is ONE basic block of 16 hand-ordered slots (D = 128):
//     slots 0..7   MFMA S(h+1) += K(h+1) Q^T   | VALU two elements of P(h) = exp2(S(h)*c - m*c),
//                                              | their row sum, bf16 packs | LDS: V operand i
//     slots 8..15  MFMA O^T += V(h)^T P(h)^T   | VALU row maximum of S(h+1) | LDS: K operand i of S(h+2)
// followed by the (rare) rescale of the accumulators when a row maximum outgrew its
// reference.  K and V tiles are copied global -> LDS asynchronously three tiles ahead into four
// buffers each (a step already reads the first operands of the tile after its own, so two
// tiles are in use, one is landing and one is being issued); one workgroup barrier per
// 64-key tile.  The last tile of every wave (the only
// one the causal mask cuts, or the ragged end of the sequence) runs unpipelined.
#include "helix_common.hpp"
#include "kernels.hpp"

namespace helix {

// The running reference maximum may lag the true row maximum by up to 2^kSlack before the
// accumulators are rescaled (exact in real arithmetic; keeps the rescale off the hot path).
constexpr float kSlack = 8.f;

template <int D>
struct FwdLaneAddr {
  int k[D / 16];       // K operand, contraction step ks, key row n of a tile (+32 rows by immediate)
  int v[D / 32][2];    // V^T operand of head-dim block db: first / second group of 4 key rows
  __device__ __forceinline__ FwdLaneAddr(int lane) {
    const int half = lane >> 5, n = lane & 31;
#pragma unroll
    for (int ks = 0; ks < D / 16; ks++) k[ks] = lds_chunk_off<D>(n, 2 * ks + half);
#pragma unroll
    for (int db = 0; db < D / 32; db++) tr_pair_offsets<D>(lane, db, v[db][0], v[db][1]);
  }
};

__device__ __forceinline__ float max16(const f32x16& s) {
  float a = fmaxf(fmaxf(s[0], s[1]), s[2]);
  float b = fmaxf(fmaxf(s[3], s[4]), s[5]);
  a = fmaxf(fmaxf(a, s[6]), s[7]);
  b = fmaxf(fmaxf(b, s[8]), s[9]);
  a = fmaxf(fmaxf(a, s[10]), s[11]);
  b = fmaxf(fmaxf(b, s[12]), s[13]);
  a = fmaxf(fmaxf(a, s[14]), s[15]);
  return fmaxf(a, b);
}

// Softmax state of a wave: reference maximum times c (the reference may lag the true row
// maximum by up to kSlack), the raw-score threshold that triggers a reference update, and
// two partial row sums per lane.
struct SoftmaxState {
  float mref_c = -INFINITY;
  float thr = -INFINITY;          // (mref_c + kSlack) / c
  float lsum[2] = {0.f, 0.f};
};

// Cheap per-block check: did any lane see a raw score above the threshold?  (Each lane holds
// 16 of the 32 keys of its query; the two halves share mref_c, so the union over all lanes
// is the test on the full rows.)  If so, move the reference of every row that grew and
// rescale the wave's accumulators.
template <int DB>
__device__ __forceinline__ void check_reference(float local_max, float c, SoftmaxState& st, f32x16 (&oacc)[DB]) {
  if (__any(local_max > st.thr)) {
    const float tc = half_max(local_max) * c;
    const float m_new = fmaxf(st.mref_c, tc);
    const float alpha = __builtin_amdgcn_exp2f(st.mref_c - m_new);   // 0 on the first block, 1 where nothing changed
    st.lsum[0] *= alpha;
    st.lsum[1] *= alpha;
#pragma unroll
    for (int db = 0; db < DB; db++)
#pragma unroll
      for (int e = 0; e < 16; e++) oacc[db][e] *= alpha;
    st.mref_c = m_new;
    st.thr = (m_new + kSlack) / c;
  }
}

// P = bf16(exp2(S*c - mref_c)) in two 16-key packs.  The row sum takes the unrounded fp32
// values: summing the bf16-rounded ones would put up to 2^-9 relative error into LSE on rows
// that see only a few keys.
__device__ __forceinline__ void exp_pack(const f32x16& s, float c, SoftmaxState& st, bf16x8 (&p)[2]) {
  f32x16 e;
#pragma unroll
  for (int i = 0; i < 16; i++) {
    e[i] = __builtin_amdgcn_exp2f(fmaf(s[i], c, -st.mref_c));
    st.lsum[i & 1] += e[i];
  }
  p[0] = pack_half(e, 0);
  p[1] = pack_half(e, 1);
}

// O^T += V^T P^T over the 32 key rows at byte offset row_off of the V region (plain path).
template <int D>
__device__ __forceinline__ void pv_block(const uint32_t (&vaddr)[D / 32][2], int row_off,
                                         const bf16x8 (&p)[2], f32x16 (&oacc)[D / 32]) {
#pragma unroll
  for (int t = 0; t < 2; t++)
#pragma unroll
    for (int db = 0; db < D / 32; db++)
      oacc[db] = mfma32(lds_tr_pair(vaddr[db][0] + row_off, vaddr[db][1] + row_off, 16 * t * D * 2), p[t], oacc[db]);
}

// One pipelined half step (see the header comment).  On entry s_cur is complete, kop holds
// the first KS/2 K operands of the block to be scored now and vop the first KS/2 V operands
// of this step; on exit s_next is complete, this lane's maximum over its 16 entries of
// s_next is returned, and kop / vop hold the first operands of the next step.  Every slot
// issues one MFMA and the LDS read of the operand needed KS/2 slots later:
//   score slots 0..KS/2-1   read K operand i + KS/2 of this block   (khi + K_CUR)
//   P V slots 0..KS/2-1     read V operand i + KS/2 of this step    (vaddr + V_IMM + 16 rows)
//   P V slots KS/2..KS-1    read K operand i - KS/2 of the next block (klo + K_NEXT) and
//                           V operand i - KS/2 of the next step
// The vector-ALU work is spread evenly: the 16 elements of P(h) (fma, exp2, row sum, bf16
// pack) go to the score slots (elements 0..9) and to the first half of the P V slots
// (elements 10..15, which the second half of the P V MFMAs consume); the row maximum of
// S(h+1) fills the last P V slots.
// When LAST_OF_TILE the next step works on the next V tile: vaddr moves on by v_step once this
// tile's reads are issued.
constexpr int kExpInScoreSlots = 10;
template <int D, int K_CUR, int K_NEXT, int V_IMM, bool LAST_OF_TILE, typename Copy>
__device__ __forceinline__ float half_step(const Copy& copy_tile, const f32x16& s_cur, f32x16& s_next,
                                           bf16x8 (&kop)[D / 32], bf16x8 (&vop)[D / 32], const bf16x8 (&qf)[D / 16],
                                           const uint32_t (&klo)[D / 32], const uint32_t (&khi)[D / 32],
                                           uint32_t (&vaddr)[D / 32][2], int v_step,
                                           f32x16 (&oacc)[D / 32], float c, SoftmaxState& st) {
  constexpr int KS = D / 16, DB = D / 32;
  constexpr int RING = KS / 2;                              // operands in flight (== DB)
  constexpr int HALF = 32 * D * 2;
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float ev[16];     // exp2 values, each alive until its pair is packed
  uint32_t pw[8];   // bf16 pairs of P
  auto element = [&](int x) {
    ev[x] = __builtin_amdgcn_exp2f(fmaf(s_cur[x], c, -st.mref_c));
    st.lsum[x & 1] += ev[x];
    if (x & 1) pw[x / 2] = pack_bf16_pair(ev[x - 1], ev[x]);
  };
#pragma unroll
  for (int i = 0; i < KS; i++) {
    s_next = mfma32(kop[i % RING], qf[i], i == 0 ? zero : s_next);
    if (i < RING) kop[i] = lds_b128(khi[i], K_CUR);
    if (i == 1) copy_tile();   // tile copies are issued under the first MFMAs, not in front of them
#pragma unroll
    for (int x = 0; x < kExpInScoreSlots; x++)
      if (x * KS / kExpInScoreSlots == i) element(x);
    __builtin_amdgcn_sched_barrier(0);
  }
  float m0 = 0.f, m1 = 0.f, m2 = 0.f, m3 = 0.f, m4 = 0.f;
#pragma unroll
  for (int i = 0; i < KS; i++) {
    const u32x4 pk = {pw[4 * (i / DB)], pw[4 * (i / DB) + 1], pw[4 * (i / DB) + 2], pw[4 * (i / DB) + 3]};
    oacc[i % DB] = mfma32(vop[i % RING], __builtin_bit_cast(bf16x8, pk), oacc[i % DB]);
    if (i < RING) {
      vop[i] = lds_tr_pair(vaddr[i][0], vaddr[i][1], V_IMM + 16 * D * 2);
#pragma unroll
      for (int x = kExpInScoreSlots; x < 16; x++)
        if ((x - kExpInScoreSlots) * RING / (16 - kExpInScoreSlots) == i) element(x);
    } else {
      if (LAST_OF_TILE) { vaddr[i - RING][0] += v_step; vaddr[i - RING][1] += v_step; }
      vop[i - RING] = lds_tr_pair(vaddr[i - RING][0], vaddr[i - RING][1], LAST_OF_TILE ? 0 : V_IMM + HALF);
      kop[i - RING] = lds_b128(klo[i - RING], K_NEXT);
    }
    // row maximum of s_next in the last slots (the score MFMAs have drained by then)
    if (i == KS - 4) { m0 = fmaxf(fmaxf(s_next[0], s_next[1]), s_next[2]); m1 = fmaxf(fmaxf(s_next[3], s_next[4]), s_next[5]); pin(m0); pin(m1); }
    if (i == KS - 3) { m2 = fmaxf(fmaxf(s_next[6], s_next[7]), s_next[8]); m3 = fmaxf(fmaxf(s_next[9], s_next[10]), s_next[11]); pin(m2); pin(m3); }
    if (i == KS - 2) { m4 = fmaxf(fmaxf(s_next[12], s_next[13]), s_next[14]); m0 = fmaxf(fmaxf(m0, m1), s_next[15]); pin(m4); pin(m0); }
    if (i == KS - 1) { m2 = fmaxf(fmaxf(m2, m3), m4); m0 = fmaxf(m0, m2); pin(m0); }
    __builtin_amdgcn_sched_barrier(0);
  }
  return m0;
}

template <int D, bool CAUSAL>
__global__ void __launch_bounds__(512, 1)
fwd_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k, const __bf16* __restrict__ v,
           __bf16* __restrict__ o, float* __restrict__ lse, FwdMaps maps, int BH, int H, int S, int T, float scale) {
  constexpr int BM = 256, BN = 64;
  constexpr int KS = D / 16;   // contraction steps of Q K^T
  constexpr int DB = D / 32;   // 32-wide blocks of the head dimension
  constexpr int TILE = BN * D * 2;
  constexpr int HALF = 32 * D * 2;   // bytes of 32 key rows
  constexpr int VREGION = 4 * TILE;
  extern __shared__ __align__(16) char smem[];   // K[4] then V[4]; tile j in buffer j % 4

  const TileCoord tc = map_block(blockIdx.x, BH, T, true);
  if (!tc.valid) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave index, held in a scalar register
  const int half = lane >> 5, n = lane & 31;
  const int q0 = tc.tile * BM;
  const int my_q = q0 + 32 * w + n;
  const __bf16* qh = q + head_offset(maps.q, tc.bh, H);
  const __bf16* kh = k + head_offset(maps.k, tc.bh, H);
  const __bf16* vh = v + head_offset(maps.v, tc.bh, H);
  const float c = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, scale * kLog2e)));
  const uint32_t base = lds_base(smem);

  bf16x8 qf[KS];
  {
    const int row = my_q < S ? my_q : S - 1;
#pragma unroll
    for (int ks = 0; ks < KS; ks++)
      qf[ks] = *reinterpret_cast<const bf16x8*>(qh + (size_t)row * maps.q.row + 16 * ks + 8 * half);
#pragma unroll
    for (int ks = 0; ks < KS; ks++) pin(qf[ks]);
  }

  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; db++)
#pragma unroll
    for (int e = 0; e < 16; e++) oacc[db][e] = 0.f;
  SoftmaxState st;

  const int q_end = (q0 + BM < S ? q0 + BM : S);                 // one past the last real row
  const int n_tiles = CAUSAL ? (q_end + BN - 1) / BN : (S + BN - 1) / BN;
  const int wave_qmin = q0 + 32 * w, wave_qmax = wave_qmin + 31;
  // Tiles this wave works on (n_w) and how many of them need no mask (n_full).  All but the
  // last run through the pipelined path; n_full >= n_w - 1 always holds.
  int n_w, n_full;
  if (wave_qmin >= S) { n_w = 0; n_full = 0; }
  else if (CAUSAL) { n_w = (wave_qmax < S ? wave_qmax : S - 1) / BN + 1; n_full = (wave_qmin + 1) / BN; }
  else { n_w = n_tiles; n_full = S / BN; }

  const TileLoader<D, BN, 8> kload(lane, w, maps.k.row), vload(lane, w, maps.v.row);
  constexpr int NDMA = decltype(kload)::N + decltype(vload)::N;   // copy instructions per wave and tile: what copy_ahead() issues
  kload.issue(kh, 0, S, base);
  vload.issue(vh, 0, S, base + VREGION);
  if (n_tiles > 1) { kload.issue(kh, BN, S, base + TILE); vload.issue(vh, BN, S, base + VREGION + TILE); }
  if (n_tiles > 2) { kload.issue(kh, 2 * BN, S, base + 2 * TILE); vload.issue(vh, 2 * BN, S, base + VREGION + 2 * TILE); }
  wait_tile_loads();
  __syncthreads();

  const FwdLaneAddr<D> la(lane);
  // Lane addresses: klo = contraction steps 0..KS/2-1 of the K tile the NEXT block comes from,
  // khi = steps KS/2..KS-1 of the tile the CURRENT block comes from, vaddr = current V tile.
  uint32_t klo[DB], khi[DB], vaddr[DB][2];
#pragma unroll
  for (int i = 0; i < DB; i++) { klo[i] = base + la.k[i] + TILE; khi[i] = base + la.k[i + DB]; }
#pragma unroll
  for (int db = 0; db < DB; db++) { vaddr[db][0] = base + VREGION + la.v[db][0]; vaddr[db][1] = base + VREGION + la.v[db][1]; }

  f32x16 sa, sb;                 // S^T of the two 32-key halves of a tile
  bf16x8 kop[DB];                // first K operands of the next block to be scored
  bf16x8 vop[DB];                // first V operands of the next P V block
#pragma unroll
  for (int db = 0; db < DB; db++) vop[db] = lds_tr_pair(vaddr[db][0], vaddr[db][1], 0);
  if (n_w > 0) {
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    sa = zero;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) sa = mfma32(lds_b128(base + la.k[ks]), qf[ks], sa);
#pragma unroll
    for (int i = 0; i < DB; i++) kop[i] = lds_b128(base + la.k[i], HALF);
    if (n_w > 1) check_reference<DB>(max16(sa), c, st, oacc);   // tile 0 goes through the pipelined path
  }

  // The tile sweep is split per wave into the pipelined tiles 0 .. n_w-2 and a second loop
  // with the wave's last tile (plain path) and the tiles it only helps to copy.  Every wave
  // of the workgroup runs n_tiles iterations in total and meets the others at the barriers.
  int rk = 0;   // j % 4
  int j = 0;
  auto copy_ahead = [&]() __attribute__((always_inline)) {
    // copies run three tiles ahead: K(j+3), V(j+3) replace K(j-1), V(j-1), last read in
    // iteration j-1.  Iteration j itself reads tile j and, ahead of its use, the first
    // operands of tile j+1 (K in both halves, V at the end of the second), so tiles up to j+1
    // must be complete when it starts.
    if (j + 3 < n_tiles) {
      kload.issue(kh, (j + 3) * BN, S, base + ((rk + 3) & 3) * TILE);
      vload.issue(vh, (j + 3) * BN, S, base + VREGION + ((rk + 3) & 3) * TILE);
    }
  };
  auto finish_tile = [&]() __attribute__((always_inline)) {
    // K(j+2) and V(j+2), issued one iteration ago, must have landed; this iteration's copies
    // (2 + 2 instructions per wave) may stay in flight.
    if (j + 3 < n_tiles) wait_tile_loads_except<NDMA>();
    else wait_tile_loads();
    __syncthreads();
    rk = (rk + 1) & 3;
  };

  const auto no_copy = []() {};
  for (; j < n_w - 1; j++) {
    const int khi_step = (rk == 3) ? -3 * TILE : TILE;   // K buffer of tile j   -> j+1
    const int klo_step = (rk == 2) ? -3 * TILE : TILE;   // K buffer of tile j+1 -> j+2
    const int v_step = khi_step;                         // V buffer of tile j   -> j+1
    // half a: score S_b(j) | P_a(j) | O += V_a(j) P_a(j) | read K_b(j) 4..7, K_a(j+1) 0..3
    // A complete tile j+3 is copied by a handful of instructions issued inside the half step; a
    // ragged one (the last of the sequence) takes the general path in front of it.
    const bool whole = j + 3 < n_tiles && (j + 4) * BN <= S;
    if (!whole) copy_ahead();
    const __bf16* kt = kload.tile_ptr(kh, (j + 3) * BN);
    const __bf16* vt = vload.tile_ptr(vh, (j + 3) * BN);
    const uint32_t dst = base + ((rk + 3) & 3) * TILE;
    const auto copy_whole = [&]() __attribute__((always_inline)) {
      if (whole) {
        kload.issue_whole(kt, dst);
        vload.issue_whole(vt, dst + VREGION);
      }
    };
    const float mb = half_step<D, HALF, 0, 0, false>(copy_whole, sa, sb, kop, vop, qf, klo, khi, vaddr, v_step, oacc, c, st);
    check_reference<DB>(mb, c, st, oacc);
#pragma unroll
    for (int i = 0; i < DB; i++) khi[i] += khi_step;
    // half b: score S_a(j+1) | P_b(j) | O += V_b(j) P_b(j) | read K_a(j+1) 4..7, K_b(j+1) 0..3;
    // vaddr moves to V(j+1)
    const float ma = half_step<D, 0, HALF, HALF, true>(no_copy, sb, sa, kop, vop, qf, klo, khi, vaddr, v_step, oacc, c, st);
    if (j + 1 < n_w - 1) check_reference<DB>(ma, c, st, oacc);   // the plain path masks first
#pragma unroll
    for (int i = 0; i < DB; i++) klo[i] += klo_step;
    finish_tile();
  }

  for (; j < n_tiles; j++) {
    copy_ahead();
    if (j == n_w - 1) {
      // plain path: the last tile of this wave (masked unless the sequence ends on a tile edge);
      // kop holds steps 0..KS/2-1 of K_b(j), khi points at K(j), vaddr at V(j)
      const int k0 = j * BN;
      const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      sb = zero;
#pragma unroll
      for (int i = 0; i < DB; i++) sb = mfma32(kop[i], qf[i], sb);
#pragma unroll
      for (int i = 0; i < DB; i++) sb = mfma32(lds_b128(khi[i], HALF), qf[i + DB], sb);
      if (j >= n_full) {
#pragma unroll
        for (int e = 0; e < 16; e++) {
          const int key = k0 + 8 * (e >> 2) + 4 * half + (e & 3);
          sa[e] = (CAUSAL ? (key <= my_q) : (key < S)) ? sa[e] : -INFINITY;
          sb[e] = (CAUSAL ? (key + 32 <= my_q) : (key + 32 < S)) ? sb[e] : -INFINITY;
        }
      }
      bf16x8 p[2];
      check_reference<DB>(max16(sa), c, st, oacc);
      exp_pack(sa, c, st, p);
      pv_block<D>(vaddr, 0, p, oacc);
      check_reference<DB>(max16(sb), c, st, oacc);
      exp_pack(sb, c, st, p);
      pv_block<D>(vaddr, HALF, p, oacc);
    }
    finish_tile();
  }

  // epilogue: normalise, store O (bf16) and LSE (natural log, scale included)
  const float ltot = half_sum(st.lsum[0] + st.lsum[1]);
  const float inv = 1.f / ltot;
  if (my_q < S) {
    __bf16* orow = o + head_offset(maps.o, tc.bh, H) + (size_t)my_q * maps.o.row;
#pragma unroll
    for (int db = 0; db < DB; db++)
#pragma unroll
      for (int g = 0; g < 4; g++) {
        f32x4 x;
#pragma unroll
        for (int e = 0; e < 4; e++) x[e] = oacc[db][4 * g + e] * inv;
        *reinterpret_cast<bf16x4*>(orow + 32 * db + 8 * g + 4 * half) = __builtin_convertvector(x, bf16x4);
      }
    if (half == 0) lse[(size_t)tc.bh * S + my_q] = st.mref_c * kLn2 + __logf(ltot);
  }
}

template <int D, bool CAUSAL>
static hipError_t launch_fwd_t(const void* q, const void* k, const void* v, void* o, float* lse,
                               const FwdMaps& maps, int B, int H, int S, float scale, hipStream_t stream) {
  constexpr int BM = 256, BN = 64;
  const int T = (S + BM - 1) / BM, BH = B * H;
  const unsigned grid = (unsigned)grid_blocks(BH, T);
  const size_t lds = 8 * BN * D * 2;
  auto kern = fwd_kernel<D, CAUSAL>;
  static unsigned long long configured = 0;   // one static per template instantiation
  hipError_t e = allow_dynamic_lds(kern, lds, configured);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(512), lds, stream, (const __bf16*)q, (const __bf16*)k,
                     (const __bf16*)v, (__bf16*)o, lse, maps, BH, H, S, T, scale);
  return hipGetLastError();
}

hipError_t launch_fwd(const void* q, const void* k, const void* v, void* o, float* lse, const FwdMaps& maps,
                      int B, int H, int S, int D, float scale, bool causal, hipStream_t stream) {
  if (D == 128) return causal ? launch_fwd_t<128, true>(q, k, v, o, lse, maps, B, H, S, scale, stream)
                              : launch_fwd_t<128, false>(q, k, v, o, lse, maps, B, H, S, scale, stream);
  return causal ? launch_fwd_t<64, true>(q, k, v, o, lse, maps, B, H, S, scale, stream)
                : launch_fwd_t<64, false>(q, k, v, o, lse, maps, B, H, S, scale, stream);
}

}  // namespace helix

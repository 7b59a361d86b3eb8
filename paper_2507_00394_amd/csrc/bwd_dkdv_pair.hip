// dK / dV pass of the attention backward, head dimension 128, TWO waves per SIMD (Table 1,
// Attention column, "Backward B").  The arithmetic is that of bwd_dkdv.hip (dV comes out bit
// for bit the same; dK differs in the last bit of some elements because here -delta is the
// initial accumulator of the dP product in every code path); what differs is the division of
// labour.
//
// The one-wave-per-SIMD kernel keeps S, dP, dK^T and dV^T of 32 keys in one wave (364
// registers at this head dimension) and is bound by instruction issue: a single wave issues
// about one instruction per four cycles whatever it is, and there are eight of them per MFMA.
// Here a workgroup of 8 waves owns the same 128 keys, but each group of 32 keys belongs to a
// PAIR of waves:
//     wave A (waves 0..3):  S = Q K^T,  P = exp2(S*c - lse2),  dV^T += dO^T bf16(P)
//     wave B (waves 4..7):  dP = dO V^T - delta,  dS = P o dP,  dK^T += Q^T bf16(dS)
// A hands P (fp32, register for register: both accumulators have the same lane layout)
// to B through LDS; B works one 32-row block behind A, and one workgroup barrier per block
// orders the hand-over.  Each wave needs 216-233 registers, so two fit on a SIMD and the
// instructions of one issue under the MFMAs of the other; per MFMA a wave issues about two
// vector-ALU and two LDS instructions.
//
// Tiles.  Q and dO are staged per 32-row block (8 KB each) in two rings of SEVEN stages (block
// i-1 is read by B, i and i+1 by both, i+2 is prefetched, i+3 and i+4 are landing, i+5 is being
// issued) plus small rings for lse2 / -delta.  The block loop is unrolled seven times, so the
// stage of every LDS access is a compile-time immediate added to the lane's address register
// (a whole ring is within the 64 KB reach of an LDS instruction's offset field): the loop
// contains no address arithmetic at all.  Blocks cut by the causal diagonal and whatever
// remains at the end run through a plain path (A, barrier, B, barrier).
#include "helix_common.hpp"
#include "kernels.hpp"

#include <type_traits>
#include <utility>

namespace helix {

namespace {

struct PG {
  static constexpr int D = 128, KS = 8, DB = 4, BN = 128, RB = 32;   // head dim, contraction steps, 32-wide blocks of D, keys per workgroup, rows per block
  static constexpr int NSTAGE = 7;
  static constexpr int BLOCK = RB * D * 2;                // one 32-row bf16 block: 8 KB
  static constexpr int QRING = 0;                         // NSTAGE blocks of Q
  static constexpr int GRING = NSTAGE * BLOCK;            // NSTAGE blocks of dO
  static constexpr int STATS = 2 * NSTAGE * BLOCK;        // ring of [lse2: 64 floats][-delta: 64 floats] per stage
  static constexpr int STAT_STAGE = 512;
  static constexpr int PBUF = STATS + NSTAGE * STAT_STAGE;   // two buffers of P: [pair][group of 4 registers][lane][4] fp32
  static constexpr int PBYTES = 4 * 4096;
  static constexpr int LDS = PBUF + 2 * PBYTES;
  static constexpr int AHEAD = 5;                         // a block is copied this many blocks before it becomes A's current one
  static constexpr int NDMA = 3;                          // copy instructions per wave and block: Q piece, dO piece, one statistics row
};
static_assert(PG::LDS <= 160 * 1024, "LDS budget of a compute unit");
static_assert(PG::NSTAGE * PG::BLOCK <= 65536, "a whole ring is within reach of the 16-bit offset field of an LDS instruction");

// LDS byte offset of stage k inside a ring.
constexpr int stage_imm(int k) { return k * PG::BLOCK; }
constexpr int wrap(int k) { return ((k % PG::NSTAGE) + PG::NSTAGE) % PG::NSTAGE; }

__device__ __forceinline__ void dma_dword(const float* base, uint32_t lane_byte_off, uint32_t lds_dst) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
               :: "v"(lane_byte_off), "s"(uniform_ptr(base)), "s"(__builtin_amdgcn_readfirstlane(lds_dst)) : "memory");
}
__device__ __forceinline__ f32x4 lds_f32x4(uint32_t addr, int imm) {
  return *reinterpret_cast<const __attribute__((address_space(3))) f32x4*>(
      reinterpret_cast<const __attribute__((address_space(3))) char*>((uintptr_t)addr) + imm);
}
__device__ __forceinline__ void lds_store_f32x4(uint32_t addr, int imm, f32x4 x) {
  *reinterpret_cast<__attribute__((address_space(3))) f32x4*>(
      reinterpret_cast<__attribute__((address_space(3))) char*>((uintptr_t)addr) + imm) = x;
}
__device__ __forceinline__ f32x16 join4(const f32x4 (&x)[4]) {
  f32x16 r;
#pragma unroll
  for (int g = 0; g < 4; g++)
#pragma unroll
    for (int e = 0; e < 4; e++) r[4 * g + e] = x[g][e];
  return r;
}
__device__ __forceinline__ f32x4 quarter(const f32x16& x, int g) {
  f32x4 r = {x[4 * g], x[4 * g + 1], x[4 * g + 2], x[4 * g + 3]};
  return r;
}
template <int FIRST, typename F, int... I>
__device__ __forceinline__ void for_each_slot(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, FIRST + I>{}), ...);
}

// End of a block: the block that becomes readable two iterations from now has landed (the
// copies of the last two iterations may still fly), the hand-over writes of this wave are in
// LDS (LDS operations complete in order and more than four reads, those of slots 9 to 15, were
// issued after the writes of slot 8), and every wave has finished the block.
template <int VM>
__device__ __forceinline__ void block_barrier() {
  static_assert(VM >= 0 && VM < 16, "");
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(4)\n\ts_barrier" :: "n"(VM) : "memory");
}

// Lane state: LDS addresses of this lane's operands in stage 0 of the ring its role reads them from.
struct Lane {
  uint32_t aq[PG::KS];         // row operand (Q rows for A, dO rows for B): row n, contraction step ks
  uint32_t at[PG::DB][2];      // transposing reads (dO^T for A, Q^T for B)
  uint32_t astat;              // statistics ring: this lane's group offset in this role's half of a stage
  uint32_t pbuf;               // P hand-over: this lane's slot in buffer `pbuf`, the other buffer is pbuf + pstep
  int pstep;
};

// Copy state of the pipelined loop: whole blocks only, so a copy is three instructions with
// precomputed operands.  The pointers are wave-uniform (scalar registers).
struct Copier {
  const __bf16* qptr;     // first row of the next Q block to copy
  const __bf16* gptr;     // same for dO
  const float* stat;      // this role's statistics row of the head
  uint32_t qoff, goff;    // this lane's byte offset inside a block (row * row bytes + swizzled chunk)
  uint32_t soff;          // this lane's byte offset into the statistics row
  uint32_t qstep, gstep;  // bytes between consecutive blocks
  uint32_t dst;           // LDS address of this wave's 1 KB piece in stage 0 of the Q ring
  uint32_t sdst;          // LDS address of this role's half of stage 0 of the statistics ring
};
template <int STG>
__device__ __forceinline__ void copy_whole_block(Copier& cp) {
  using G = PG;
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(cp.qoff), "s"(cp.qptr), "s"(cp.dst + G::QRING + STG * G::BLOCK) : "memory");
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(cp.goff), "s"(cp.gptr), "s"(cp.dst + G::GRING + STG * G::BLOCK) : "memory");
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
               :: "v"(cp.soff), "s"(cp.stat), "s"(cp.sdst + STG * G::STAT_STAGE) : "memory");
  cp.qptr = reinterpret_cast<const __bf16*>(reinterpret_cast<const char*>(cp.qptr) + cp.qstep);
  cp.gptr = reinterpret_cast<const __bf16*>(reinterpret_cast<const char*>(cp.gptr) + cp.gstep);
  cp.soff += PG::RB * 4;
}

__device__ __forceinline__ f32x4 (&l2ref(f32x4 (&st)[4]))[2] { return reinterpret_cast<f32x4 (&)[2]>(st); }

// ------------------------------------------------------------------ wave A: one pipelined block
// Block i at stage K.  On entry s_cur = S(i) with entries 0..7 already exponentiated, l2 =
// lse2 of block i, ring = the first four Q row operands of block i+1.  On exit the same for i+1.
template <int K>
__device__ __forceinline__ void step_a(f32x16& s_cur, f32x16& s_next, bf16x8 (&ring)[4], f32x4 (&l2)[2], Lane& ln,
                                       const bf16x8 (&kf)[PG::KS], f32x16 (&dvacc)[PG::DB], float c, Copier& cp) {
  using G = PG;
  constexpr int KS = G::KS, DB = G::DB;
  constexpr int KN = wrap(K + 1), KP = wrap(K + 2);
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  uint32_t pk[8];
  auto slot = [&](auto slot_number) __attribute__((always_inline)) {
    constexpr int s = decltype(slot_number)::value;
    // ---- matrix work
    if constexpr (s < KS) {
      s_next = mfma32(ring[s % 4], kf[s], s == 0 ? zero : s_next);
    } else {
      constexpr int i = s - KS;
      const u32x4 b = {pk[4 * (i / DB)], pk[4 * (i / DB) + 1], pk[4 * (i / DB) + 2], pk[4 * (i / DB) + 3]};
      dvacc[i % DB] = mfma32(ring[s % 4], __builtin_bit_cast(bf16x8, b), dvacc[i % DB]);
    }
    // ---- operand of slot s + 4
    {
      constexpr int u = s + 4;
      if constexpr (u < KS) ring[s % 4] = lds_b128(ln.aq[u], stage_imm(KN));
      else if constexpr (u < 2 * KS) {
        constexpr int i = u - KS;
        ring[s % 4] = lds_tr_pair(ln.at[i % DB][0], ln.at[i % DB][1], stage_imm(K) + 16 * (i / DB) * G::D * 2);
      } else ring[s % 4] = lds_b128(ln.aq[u - 2 * KS], stage_imm(KP));
    }
    // ---- lse2, four rows at a time, four slots ahead of the four slots that use them (as soon as the
    // register quad is free): groups 2, 3 of block i are used in slots 0..3, 4..7, groups 0, 1 of
    // block i+1 in slots 8..11, 12..15
    if constexpr (s == 0) l2[1] = lds_f32x4(ln.astat, K * G::STAT_STAGE + 8 * 3 * 4);
    if constexpr (s == 4) l2[0] = lds_f32x4(ln.astat, KN * G::STAT_STAGE);
    if constexpr (s == 8) l2[1] = lds_f32x4(ln.astat, KN * G::STAT_STAGE + 8 * 1 * 4);
    if constexpr (s == 12) l2[0] = lds_f32x4(ln.astat, KN * G::STAT_STAGE + 8 * 2 * 4);
    // ---- vector work
    if constexpr (s < KS) {
      // second half of P(i); packs of the first half
      constexpr int e = 8 + s;
      s_cur[e] = __builtin_amdgcn_exp2f(fmaf(s_cur[e], c, -l2[(s / 4) & 1][e % 4]));
      if constexpr (s < 4) pk[s] = pack_bf16_pair(s_cur[2 * s], s_cur[2 * s + 1]);
      if constexpr (e & 1) pk[e / 2] = pack_bf16_pair(s_cur[e - 1], s_cur[e]);
    } else {
      // first half of P(i+1)
      constexpr int e = s - KS;
      s_next[e] = __builtin_amdgcn_exp2f(fmaf(s_next[e], c, -l2[(s / 4) & 1][e % 4]));
    }
    // ---- copy of block i + AHEAD into the stage block i - 2 has left
    if constexpr (s == 2) copy_whole_block<wrap(K + G::AHEAD)>(cp);
    // ---- P(i) to wave B
    if constexpr (s == 0) { lds_store_f32x4(ln.pbuf, 0, quarter(s_cur, 0)); lds_store_f32x4(ln.pbuf, 1024, quarter(s_cur, 1)); }
    if constexpr (s == KS) { lds_store_f32x4(ln.pbuf, 2048, quarter(s_cur, 2)); lds_store_f32x4(ln.pbuf, 3072, quarter(s_cur, 3)); }
    __builtin_amdgcn_sched_barrier(0);
  };
  for_each_slot<0>(slot, std::make_integer_sequence<int, 2 * KS>{});
  pin(s_next);   // the first half of P(i+1) is computed here, under the MFMAs, not where the next step first uses it
  ln.pbuf += ln.pstep;
  ln.pstep = -ln.pstep;
}

// ------------------------------------------------------------------ wave B: one pipelined iteration
// Iteration i (A's block, stage K): finishes block j = i-1 (dS, dK) unless SKIP and computes
// dP(i).  On entry dp_cur = dP(j), nd = -delta(i), ring = the first four dO row operands of block i.
template <int K, bool SKIP>
__device__ __forceinline__ void step_b(f32x16& dp_cur, f32x16& dp_next, bf16x8 (&ring)[4], f32x4 (&nd)[4], Lane& ln,
                                       const bf16x8 (&vf)[PG::KS], f32x16 (&dkacc)[PG::DB], Copier& cp) {
  using G = PG;
  constexpr int KS = G::KS, DB = G::DB;
  constexpr int KJ = wrap(K - 1), KN = wrap(K + 1);
  uint32_t sk[8];
  f32x4 pf[4];
  auto slot = [&](auto slot_number) __attribute__((always_inline)) {
    constexpr int s = decltype(slot_number)::value;
    // ---- P(j) from wave A (written before the last barrier), into the other buffer than A writes now
    if constexpr (s == 0 && !SKIP) {
#pragma unroll
      for (int g = 0; g < 4; g++) pf[g] = lds_f32x4(ln.pbuf, 1024 * g);
    }
    // ---- matrix work
    if constexpr (s < KS) {
      dp_next = mfma32(ring[s % 4], vf[s], s == 0 ? join4(nd) : dp_next);
    } else if constexpr (!SKIP) {
      constexpr int i = s - KS;
      const u32x4 b = {sk[4 * (i / DB)], sk[4 * (i / DB) + 1], sk[4 * (i / DB) + 2], sk[4 * (i / DB) + 3]};
      dkacc[i % DB] = mfma32(ring[s % 4], __builtin_bit_cast(bf16x8, b), dkacc[i % DB]);
    }
    // ---- operand of slot s + 4
    {
      constexpr int u = s + 4;
      if constexpr (u < KS) ring[s % 4] = lds_b128(ln.aq[u], stage_imm(K));
      else if constexpr (u < 2 * KS) {
        if constexpr (!SKIP) {
          constexpr int i = u - KS;
          ring[s % 4] = lds_tr_pair(ln.at[i % DB][0], ln.at[i % DB][1], stage_imm(KJ) + 16 * (i / DB) * G::D * 2);
        }
      } else ring[s % 4] = lds_b128(ln.aq[u - 2 * KS], stage_imm(KN));
    }
    // ---- copy of block i + AHEAD into the stage block i - 2 has left
    if constexpr (s == 2) copy_whole_block<wrap(K + G::AHEAD)>(cp);
    // ---- -delta of block i+1 (the registers are free once the dP product has started)
    if constexpr (s >= 12) nd[s - 12] = lds_f32x4(ln.astat, KN * G::STAT_STAGE + 8 * (s - 12) * 4);
    // ---- vector work: dS(j) = P(j) o dP(j), two elements per slot in slots 4..7 (first half, P was
    // requested in slot 0) and 8..11 (second half)
    if constexpr (!SKIP && s >= 4 && s < 12) {
      constexpr int e0 = 2 * (s - 4);
      const float d0 = pf[e0 / 4][e0 % 4] * dp_cur[e0];
      const float d1 = pf[(e0 + 1) / 4][(e0 + 1) % 4] * dp_cur[e0 + 1];
      sk[e0 / 2] = pack_bf16_pair(d0, d1);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  for_each_slot<0>(slot, std::make_integer_sequence<int, 2 * KS>{});
  if (!SKIP) {
    ln.pbuf += ln.pstep;
    ln.pstep = -ln.pstep;
  }
}

}  // namespace

// The whole sweep of one wave in its role (0: wave A, 1: wave B).  Both programs execute the same
// sequence of workgroup barriers.
template <bool CAUSAL, int ROLE>
__device__ __forceinline__ void pair_sweep(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                                           const __bf16* __restrict__ v, const __bf16* __restrict__ dO,
                                           const float* __restrict__ lse2, const float* __restrict__ neg_delta,
                                           __bf16* __restrict__ dk, __bf16* __restrict__ dv, const BwdMaps& maps,
                                           const TileCoord tc, int H, int S, float scale) {
  using G = PG;
  constexpr int D = G::D, KS = G::KS, DB = G::DB, RB = G::RB, NST = G::NSTAGE;
  extern __shared__ __align__(16) char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  constexpr int role = ROLE;                                 // 0: wave A, 1: wave B
  const int pair = w & 3;
  const int half = lane >> 5, n = lane & 31;
  const int n0 = tc.tile * G::BN;
  const int my_key = n0 + 32 * pair + n;
  const __bf16* qh = q + head_offset(maps.q, tc.bh, H);
  const __bf16* gh = dO + head_offset(maps.dO, tc.bh, H);
  const __bf16* kh = k + head_offset(maps.k, tc.bh, H);
  const __bf16* vh = v + head_offset(maps.v, tc.bh, H);
  const float* stat_h = (role == 0 ? lse2 : neg_delta) + (size_t)tc.bh * S;   // the statistics row this wave copies
  const float c = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, scale * kLog2e)));
  const uint32_t base = lds_base(smem);

  // B operand of this wave's first product: K fragments for A (S = Q K^T), V fragments for B (dP = dO V^T)
  bf16x8 frag[KS];
  {
    const int row = my_key < S ? my_key : S - 1;
    const __bf16* src = role == 0 ? kh + (size_t)row * maps.k.row : vh + (size_t)row * maps.v.row;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) frag[ks] = *reinterpret_cast<const bf16x8*>(src + 16 * ks + 8 * half);
#pragma unroll
    for (int ks = 0; ks < KS; ks++) pin(frag[ks]);
  }
  f32x16 acc[DB];   // dV^T (A) or dK^T (B) of this wave's 32 keys
#pragma unroll
  for (int db = 0; db < DB; db++)
#pragma unroll
    for (int e = 0; e < 16; e++) acc[db][e] = 0.f;

  // A reads rows of Q and columns (transposed) of dO; B rows of dO and columns of Q.
  const uint32_t row_ring = base + (role == 0 ? G::QRING : G::GRING);
  const uint32_t col_ring = base + (role == 0 ? G::GRING : G::QRING);
  Lane ln;
#pragma unroll
  for (int ks = 0; ks < KS; ks++) ln.aq[ks] = row_ring + lds_chunk_off<D>(n, 2 * ks + half);
#pragma unroll
  for (int db = 0; db < DB; db++) {
    int o0, o1;
    tr_pair_offsets<D>(lane, db, o0, o1);
    ln.at[db][0] = col_ring + o0;
    ln.at[db][1] = col_ring + o1;
  }
  ln.astat = base + G::STATS + role * 256 + half * 16;
  const uint32_t pbuf0 = base + G::PBUF + pair * 4096 + lane * 16;

  const int m_start = CAUSAL ? n0 : 0;                       // first query row that sees a key of this tile
  const int nb = (S - m_start + RB - 1) / RB;                // blocks to sweep
  const int nfull = (S - m_start) / RB;                      // of which complete
  // pipelined blocks [i0, i1): after the blocks the causal diagonal cuts, starting at stage 0, 1 + 7 g of them
  const int i0 = CAUSAL ? G::BN / RB : 0;
  // Block i lives in stage (i + kStageShift) % NSTAGE: the first pipelined block sits in stage 0, where the
  // unrolled loop starts, without padding the plain prefix to a multiple of seven.
  constexpr int kStageShift = CAUSAL ? NST - G::BN / RB : 0;
  auto stage_of = [&](int i) __attribute__((always_inline)) { return (i + kStageShift) % NST; };
  int i1 = i0;
  // (every copy they issue, up to block i1 - 1 + AHEAD, and the 64 statistics rows it reads are whole)
  const int navail = nfull - (G::AHEAD + 1) - i0;
  if (navail >= 1 + NST) i1 = i0 + 1 + ((navail - 1) / NST) * NST;

  const TileLoader<D, RB, 8> qload(lane, w, maps.q.row), gload(lane, w, maps.dO.row);
  static_assert(decltype(qload)::N + decltype(gload)::N + 1 == G::NDMA, "copy instructions per wave and block");
  auto copy_block = [&](int i, int stage) __attribute__((always_inline)) {
    const int row0 = m_start + i * RB;
    qload.issue(qh, row0, S, base + G::QRING + stage * G::BLOCK);
    gload.issue(gh, row0, S, base + G::GRING + stage * G::BLOCK);
    int r = row0 + lane;
    r = r < S ? r : S - 1;
    dma_dword(stat_h, (uint32_t)r * 4, base + G::STATS + stage * G::STAT_STAGE + role * 256);
  };
  // Runtime-stage copy of block i + AHEAD at the start of iteration i (stage = (i + AHEAD) % 7).
  auto copy_ahead = [&](int i) __attribute__((always_inline)) {
    if (i + G::AHEAD < nb) copy_block(i + G::AHEAD, stage_of(i + G::AHEAD));
  };
#pragma unroll
  for (int i = 0; i < G::AHEAD; i++)
    if (i < nb) copy_block(i, stage_of(i));
  wait_tile_loads();
  __syncthreads();

  // ---- plain path: block i in program order (A, barrier, B, barrier), masks applied by A
  auto plain_block = [&](int i) __attribute__((always_inline)) {
    const int so = stage_of(i) * G::BLOCK;                       // stage offset inside a ring
    const uint32_t stat = ln.astat + stage_of(i) * G::STAT_STAGE;
    const int r0 = m_start + i * RB;
    copy_ahead(i);
    if constexpr (role == 0) {
      f32x16 sacc;
#pragma unroll
      for (int e = 0; e < 16; e++) sacc[e] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ks++) sacc = mfma32(lds_b128(ln.aq[ks] + so), frag[ks], sacc);
#pragma unroll
      for (int g = 0; g < 4; g++) {
        const f32x4 l4 = lds_f32x4(stat, 8 * g * 4);
#pragma unroll
        for (int e4 = 0; e4 < 4; e4++) {
          const int e = 4 * g + e4;
          const int row = r0 + 8 * g + 4 * half + e4;
          const float p = __builtin_amdgcn_exp2f(fmaf(sacc[e], c, -l4[e4]));
          const bool ok = (!CAUSAL || my_key <= row) && row < S;
          sacc[e] = ok ? p : 0.f;
        }
        lds_store_f32x4(pbuf0, 1024 * g, quarter(sacc, g));
      }
#pragma unroll
      for (int tt = 0; tt < 2; tt++) {
        const bf16x8 pb = pack_half(sacc, tt);
#pragma unroll
        for (int db = 0; db < DB; db++)
          acc[db] = mfma32(lds_tr_pair(ln.at[db][0] + so, ln.at[db][1] + so, 16 * tt * D * 2), pb, acc[db]);
      }
    }
    __syncthreads();
    if constexpr (role == 1) {
      f32x4 d4[4];
#pragma unroll
      for (int g = 0; g < 4; g++) d4[g] = lds_f32x4(stat, 8 * g * 4);
      f32x16 pacc = join4(d4);   // dP starts from -delta, as in the pipelined path: the bits of dK do not depend on which path a block takes
#pragma unroll
      for (int ks = 0; ks < KS; ks++) pacc = mfma32(lds_b128(ln.aq[ks] + so), frag[ks], pacc);
#pragma unroll
      for (int g = 0; g < 4; g++) {
        const f32x4 p4 = lds_f32x4(pbuf0, 1024 * g);
#pragma unroll
        for (int e4 = 0; e4 < 4; e4++) pacc[4 * g + e4] = p4[e4] * pacc[4 * g + e4];
      }
#pragma unroll
      for (int tt = 0; tt < 2; tt++) {
        const bf16x8 sb = pack_half(pacc, tt);
#pragma unroll
        for (int db = 0; db < DB; db++)
          acc[db] = mfma32(lds_tr_pair(ln.at[db][0] + so, ln.at[db][1] + so, 16 * tt * D * 2), sb, acc[db]);
      }
    }
    // the copies of this and the previous iteration may stay in flight; all LDS traffic of the block is done
    if (i + G::AHEAD < nb) wait_tile_loads_except<2 * G::NDMA>();
    else wait_tile_loads();
    __syncthreads();
  };

  int i = 0;
  for (; i < i0 && i < nb; i++) plain_block(i);

  if (i1 > i0) {
    ln.pbuf = pbuf0;
    ln.pstep = G::PBYTES;
    bf16x8 ring[4];
    f32x16 xa, xb;            // S (A) or dP (B) of the current and of the next block
    f32x4 st[4];              // A: two groups of lse2 (st[0], st[1]); B: -delta of the block whose dP product starts next
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // ---- prime at block i0 (stage 0)
    xa = zero;
    xb = zero;
    if constexpr (role == 0) {
#pragma unroll
      for (int ks = 0; ks < KS; ks++) xa = mfma32(lds_b128(ln.aq[ks], 0), frag[ks], xa);
#pragma unroll
      for (int g = 0; g < 2; g++) {
        const f32x4 l4 = lds_f32x4(ln.astat, 8 * g * 4);
#pragma unroll
        for (int e4 = 0; e4 < 4; e4++) xa[4 * g + e4] = __builtin_amdgcn_exp2f(fmaf(xa[4 * g + e4], c, -l4[e4]));
      }
      st[0] = lds_f32x4(ln.astat, 8 * 2 * 4);
#pragma unroll
      for (int r = 0; r < 4; r++) ring[r] = lds_b128(ln.aq[r], stage_imm(1));
    } else {
#pragma unroll
      for (int g = 0; g < 4; g++) st[g] = lds_f32x4(ln.astat, 8 * g * 4);
#pragma unroll
      for (int r = 0; r < 4; r++) ring[r] = lds_b128(ln.aq[r], 0);
    }
    Copier cp;
    {
      const int row0 = m_start + (i0 + G::AHEAD) * RB;
      cp.qstep = RB * qload.row_bytes;
      cp.gstep = RB * gload.row_bytes;
      cp.qptr = uniform_ptr(reinterpret_cast<const __bf16*>(reinterpret_cast<const char*>(qh) + (size_t)row0 * qload.row_bytes));
      cp.gptr = uniform_ptr(reinterpret_cast<const __bf16*>(reinterpret_cast<const char*>(gh) + (size_t)row0 * gload.row_bytes));
      cp.stat = uniform_ptr(stat_h);
      cp.qoff = qload.off[0];
      cp.goff = gload.off[0];
      cp.soff = (uint32_t)(row0 + lane) * 4;
      cp.dst = __builtin_amdgcn_readfirstlane(base + w * 1024);
      cp.sdst = __builtin_amdgcn_readfirstlane(base + G::STATS + role * 256);
    }
    // ---- first iteration: B has no finished block yet
    if constexpr (role == 0) step_a<0>(xa, xb, ring, l2ref(st), ln, frag, acc, c, cp);
    else step_b<0, true>(xa, xb, ring, st, ln, frag, acc, cp);
    block_barrier<2 * G::NDMA>();
    i++;
    // ---- seven blocks per trip: stages 1, 2, ..., 6, 0; S / dP alternate between xb and xa
    if constexpr (role == 0) {
      for (; i < i1; i += NST) {
        step_a<1>(xb, xa, ring, l2ref(st), ln, frag, acc, c, cp); block_barrier<2 * G::NDMA>();
        step_a<2>(xa, xb, ring, l2ref(st), ln, frag, acc, c, cp); block_barrier<2 * G::NDMA>();
        step_a<3>(xb, xa, ring, l2ref(st), ln, frag, acc, c, cp); block_barrier<2 * G::NDMA>();
        step_a<4>(xa, xb, ring, l2ref(st), ln, frag, acc, c, cp); block_barrier<2 * G::NDMA>();
        step_a<5>(xb, xa, ring, l2ref(st), ln, frag, acc, c, cp); block_barrier<2 * G::NDMA>();
        step_a<6>(xa, xb, ring, l2ref(st), ln, frag, acc, c, cp); block_barrier<2 * G::NDMA>();
        step_a<0>(xb, xa, ring, l2ref(st), ln, frag, acc, c, cp); block_barrier<2 * G::NDMA>();
        // seven steps swap the roles of xa and xb once more: swap them back so that the trip starts as before
        const f32x16 t = xa; xa = xb; xb = t;
      }
    } else {
      for (; i < i1; i += NST) {
        step_b<1, false>(xb, xa, ring, st, ln, frag, acc, cp); block_barrier<2 * G::NDMA>();
        step_b<2, false>(xa, xb, ring, st, ln, frag, acc, cp); block_barrier<2 * G::NDMA>();
        step_b<3, false>(xb, xa, ring, st, ln, frag, acc, cp); block_barrier<2 * G::NDMA>();
        step_b<4, false>(xa, xb, ring, st, ln, frag, acc, cp); block_barrier<2 * G::NDMA>();
        step_b<5, false>(xb, xa, ring, st, ln, frag, acc, cp); block_barrier<2 * G::NDMA>();
        step_b<6, false>(xa, xb, ring, st, ln, frag, acc, cp); block_barrier<2 * G::NDMA>();
        step_b<0, false>(xb, xa, ring, st, ln, frag, acc, cp); block_barrier<2 * G::NDMA>();
        const f32x16 t = xa; xa = xb; xb = t;
      }
    }
    // ---- drain: B finishes block i1 - 1 (its dP is in xb, its P in the buffer A wrote last)
    if constexpr (role == 1) {
      const int so = stage_of(i1 - 1) * G::BLOCK;
      f32x16 ds;
#pragma unroll
      for (int g = 0; g < 4; g++) {
        const f32x4 p4 = lds_f32x4(ln.pbuf, 1024 * g);
#pragma unroll
        for (int e4 = 0; e4 < 4; e4++) ds[4 * g + e4] = p4[e4] * xb[4 * g + e4];
      }
#pragma unroll
      for (int tt = 0; tt < 2; tt++) {
        const bf16x8 sb = pack_half(ds, tt);
#pragma unroll
        for (int db = 0; db < DB; db++)
          acc[db] = mfma32(lds_tr_pair(ln.at[db][0] + so, ln.at[db][1] + so, 16 * tt * D * 2), sb, acc[db]);
      }
    }
    __syncthreads();   // the plain blocks that follow reuse the first P buffer and the stages
  }

  for (; i < nb; i++) plain_block(i);

  if (my_key < S) {
    const float m = role == 0 ? 1.f : scale;
    __bf16* row = role == 0 ? dv + head_offset(maps.dv, tc.bh, H) + (size_t)my_key * maps.dv.row
                            : dk + head_offset(maps.dk, tc.bh, H) + (size_t)my_key * maps.dk.row;
#pragma unroll
    for (int db = 0; db < DB; db++)
#pragma unroll
      for (int g = 0; g < 4; g++) {
        f32x4 x;
#pragma unroll
        for (int e = 0; e < 4; e++) x[e] = acc[db][4 * g + e] * m;
        *reinterpret_cast<bf16x4*>(row + 32 * db + 8 * g + 4 * half) = __builtin_convertvector(x, bf16x4);
      }
  }
}

template <bool CAUSAL>
__global__ void __launch_bounds__(512, 1)
bwd_dkdv_pair_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k, const __bf16* __restrict__ v,
                     const __bf16* __restrict__ dO, const float* __restrict__ lse2, const float* __restrict__ neg_delta,
                     __bf16* __restrict__ dk, __bf16* __restrict__ dv, BwdMaps maps, int BH, int H, int S, int T,
                     float scale) {
  const TileCoord tc = map_block(blockIdx.x, BH, T, false);
  if (!tc.valid) return;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (w < 4) pair_sweep<CAUSAL, 0>(q, k, v, dO, lse2, neg_delta, dk, dv, maps, tc, H, S, scale);
  else pair_sweep<CAUSAL, 1>(q, k, v, dO, lse2, neg_delta, dk, dv, maps, tc, H, S, scale);
}

hipError_t launch_bwd_dkdv_pair(const void* q, const void* k, const void* v, const void* dO, const float* lse2,
                                const float* neg_delta, void* dk, void* dv, const BwdMaps& maps, int B, int H, int S,
                                float scale, bool causal, hipStream_t stream) {
  const int T = (S + PG::BN - 1) / PG::BN, BH = B * H;
  const unsigned grid = (unsigned)grid_blocks(BH, T);
  const size_t lds = PG::LDS;
  if (causal) {
    auto kern = bwd_dkdv_pair_kernel<true>;
    static unsigned long long configured = 0;
    hipError_t e = allow_dynamic_lds(kern, lds, configured);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(512), lds, stream, (const __bf16*)q, (const __bf16*)k, (const __bf16*)v,
                       (const __bf16*)dO, lse2, neg_delta, (__bf16*)dk, (__bf16*)dv, maps, BH, H, S, T, scale);
  } else {
    auto kern = bwd_dkdv_pair_kernel<false>;
    static unsigned long long configured = 0;
    hipError_t e = allow_dynamic_lds(kern, lds, configured);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(512), lds, stream, (const __bf16*)q, (const __bf16*)k, (const __bf16*)v,
                       (const __bf16*)dO, lse2, neg_delta, (__bf16*)dk, (__bf16*)dv, maps, BH, H, S, T, scale);
  }
  return hipGetLastError();
}

}  // namespace helix

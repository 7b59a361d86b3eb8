// Device-side building blocks shared by the gfx950 attention kernels: vector types,
// the 32x32x16 bf16 MFMA, LDS tile staging with a bank-conflict-free swizzle, the
// transposing LDS read and the cross-half lane exchange.
#pragma once
#include <hip/hip_runtime.h>
#include "kernels.hpp"
#include <stdint.h>

namespace helix {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define HELIX_LDS(T, p) ((__attribute__((address_space(3))) T*)(p))

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// D(32x32, fp32) += A(32x16, bf16) * B(16x32, bf16).  Lane l supplies A[l%32][8*(l/32)..+7]
// and B[8*(l/32)..+7][l%32]; accumulator register v of lane l is
// D[8*(v/4) + 4*(l/32) + v%4][l%32].
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Value held by the lane 32 positions away combined with this lane's: both halves of the
// wave end up with the same result.
__device__ __forceinline__ float half_max(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// LDS tiles are [rows][D] bf16 with the 16-byte chunks of each row permuted by an XOR
// that depends on the row, so that both access patterns below hit all 64 banks:
//   - ds_read_b128 by 16 lanes on 16 consecutive rows at the same logical chunk,
//   - ds_read_b64_tr_b16 by 32 lanes on 4 consecutive rows x 64 contiguous bytes.
template <int D>
__device__ __forceinline__ int swizzle(int row) {
  static_assert(D == 128 || D == 64 || D == 32, "tile widths with a known conflict-free permutation");
  if constexpr (D == 128) return ((row & 3) << 2) | ((row >> 2) & 3);
  else if constexpr (D == 64) return (((row >> 1) & 1) << 2) | ((row >> 2) & 3);
  else return (row >> 2) & 3;   // 64-byte rows: rows r, r+4, r+8, r+12 share banks, so they take different chunks
}
template <int D>
__device__ __forceinline__ int lds_chunk_off(int row, int chunk) {
  return row * (D * 2) + ((chunk ^ swizzle<D>(row)) << 4);
}

// One 16-byte chunk from global memory, zero when the row is past the end.
__device__ __forceinline__ u32x4 load_chunk(const __bf16* base, int row, int nrows, int row_stride, int col) {
  u32x4 z = {0u, 0u, 0u, 0u};
  if (row < nrows) z = *reinterpret_cast<const u32x4*>(base + (size_t)row * row_stride + col);
  return z;
}

// Register-staged copy of a [ROWS][D] bf16 tile: `fetch` issues the global loads, `commit`
// writes them to LDS (swizzled).  NT threads cooperate; chunk id = tid + NT*i.
template <int D, int ROWS, int NT>
struct TileStage {
  static constexpr int CH = D / 8;                 // 16-byte chunks per row
  static constexpr int N = (ROWS * CH + NT - 1) / NT;
  u32x4 r[N];
  __device__ __forceinline__ void fetch(const __bf16* head_base, int row_stride, int row0, int nrows, int tid) {
#pragma unroll
    for (int i = 0; i < N; i++) {
      int id = tid + NT * i;
      int row = id / CH, c = id % CH;
      if (ROWS * CH % NT == 0 || id < ROWS * CH) r[i] = load_chunk(head_base, row0 + row, nrows, row_stride, c * 8);
    }
  }
  __device__ __forceinline__ void commit(char* lds, int tid) const {
#pragma unroll
    for (int i = 0; i < N; i++) {
      int id = tid + NT * i;
      int row = id / CH, c = id % CH;
      if (ROWS * CH % NT == 0 || id < ROWS * CH) *reinterpret_cast<u32x4*>(lds + lds_chunk_off<D>(row, c)) = r[i];
    }
  }
};

// Asynchronous global -> LDS copy of a [ROWS][D] bf16 tile without staging registers
// (global_load_lds_dwordx4: lane i of a wave deposits its 16 bytes at lds_base + 16*i).
// A wave copies 1 KB per instruction; the swizzle is applied by choosing WHICH global chunk
// each lane fetches.  The common case costs no vector ALU work per tile: the lane's byte
// offset inside a tile is fixed and the tile's base address travels in scalar registers.
// Rows past the end of the sequence (last tile only) are clamped to the last row: every
// consumer multiplies them by an exactly-zero probability or never stores their results.
// The copies are issued as inline assembly on purpose: for the builtin the compiler assumes
// that any later LDS read may alias the copy and waits for it at once, which would serialise
// the copy of the next tile with the work on the current one.  The caller waits
// (`wait_tile_loads*`) and then barriers before anyone reads the tile.
// The statements write M0 without declaring it: M0 is not an allocatable register (the
// compiler rejects it in a clobber list as reserved) and the compiler itself only loads it
// immediately in front of its own users (sendmsg, movrel, its LDS-copy builtins), none of
// which these kernels contain; no value of the compiler's ever lives in M0 across them.
// A pointer the caller knows to be wave-uniform, moved into scalar registers.
template <typename T>
__device__ __forceinline__ const T* uniform_ptr(const T* p) {
  const uint64_t x = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)x);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(x >> 32));
  return reinterpret_cast<const T*>(((uint64_t)hi << 32) | lo);
}

template <int D, int ROWS, int NWAVES>
struct TileLoader {
  static constexpr int CH = D / 8;                        // 16-byte chunks per row
  static constexpr int ROWS_PER_KB = 64 / CH;             // rows covered by one wave instruction
  static constexpr int KB = ROWS / ROWS_PER_KB;           // 1 KB pieces in the tile
  static constexpr int N = (KB + NWAVES - 1) / NWAVES;    // pieces per wave = copy instructions one issue() costs a wave
  static_assert(KB % NWAVES == 0, "every wave copies the same number of pieces");
  int wave, lane_row;  // lane_row: this lane's row inside a piece
  uint32_t row_bytes;  // distance between consecutive rows of the tensor in global memory
  uint32_t off[N];     // byte offset from the tile's first row of the chunk this lane fetches for
                       // piece i: row * row_bytes + 16 * (logical chunk)
  // row_stride: elements between consecutive rows of the tensor (D when the head is contiguous).
  __device__ __forceinline__ TileLoader(int lane, int wave_, int row_stride)
      : wave(wave_), lane_row(lane / CH), row_bytes((uint32_t)row_stride * 2u) {
#pragma unroll
    for (int i = 0; i < N; i++) {
      const int r = (wave + NWAVES * i) * ROWS_PER_KB + lane_row;
      off[i] = r * row_bytes + (((lane % CH) ^ swizzle<D>(r)) << 4);
    }
  }
  // Address of the tile's first row (wave-uniform, in scalar registers).
  __device__ __forceinline__ const __bf16* tile_ptr(const __bf16* head_base, int row0) const {
    return uniform_ptr(reinterpret_cast<const __bf16*>(reinterpret_cast<const char*>(head_base) + (size_t)row0 * row_bytes));
  }
  // Copy of a tile all of whose ROWS rows exist: N instructions, no branch.
  __device__ __forceinline__ void issue_whole(const __bf16* tile_base, uint32_t lds_tile_addr) const {
#pragma unroll
    for (int i = 0; i < N; i++) {
      const uint32_t dst = __builtin_amdgcn_readfirstlane(lds_tile_addr + (wave + NWAVES * i) * 1024);
      asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                   :: "v"(off[i]), "s"(tile_base), "s"(dst) : "memory");
    }
  }
  // lds_tile_addr: 32-bit LDS address of the destination tile (wave-uniform).
  __device__ __forceinline__ void issue(const __bf16* head_base, int row0, int nrows, uint32_t lds_tile_addr) const {
    const __bf16* tile_base = tile_ptr(head_base, row0);
    const int last = __builtin_amdgcn_readfirstlane(nrows - 1 - row0);   // last valid tile row (>= ROWS-1 unless ragged)
    if (last >= ROWS - 1) {
      issue_whole(tile_base, lds_tile_addr);
    } else {   // last tile of a ragged sequence: clamp the row
#pragma unroll
      for (int i = 0; i < N; i++) {
        const uint32_t dst = __builtin_amdgcn_readfirstlane(lds_tile_addr + (wave + NWAVES * i) * 1024);
        const int row = (wave + NWAVES * i) * ROWS_PER_KB + lane_row;
        const int rr = row < last ? row : last;
        const uint32_t o = off[i] - (uint32_t)(row - rr) * row_bytes;
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                     :: "v"(o), "s"(tile_base), "s"(dst) : "memory");
      }
    }
  }
};

// s_waitcnt vmcnt(0) (expcnt and lgkmcnt left at their maxima).  Issued through the builtin so
// that the compiler also learns that none of ITS vector memory loads is outstanding any more;
// otherwise it re-waits on them inside the loops and thereby on the asynchronous tile copies.
__device__ __forceinline__ void wait_tile_loads() {
  __builtin_amdgcn_s_waitcnt(0x0F70);
  asm volatile("" ::: "memory");
}

// s_waitcnt vmcnt(N): all but the N most recent vector memory operations of this wave are done.
template <int N>
__device__ __forceinline__ void wait_tile_loads_except() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
  asm volatile("" ::: "memory");
}

// LDS reads take an absolute 32-bit LDS address held in a register plus a compile-time
// immediate that folds into the instruction's offset field.
__device__ __forceinline__ uint32_t lds_base(const char* smem) { return (uint32_t)(uintptr_t)HELIX_LDS(const char, smem); }
__device__ __forceinline__ bf16x8 lds_b128(uint32_t addr, int imm = 0) {
  return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(
      reinterpret_cast<const __attribute__((address_space(3))) char*>((uintptr_t)addr) + imm);
}

// V^T operand: 16 keys (two groups of 4+4 rows per lane half) x 32 head-dim columns.
__device__ __forceinline__ bf16x8 lds_tr_pair(uint32_t addr0, uint32_t addr1, int imm) {
  typedef __attribute__((address_space(3))) char* lds_ptr;
  const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16(HELIX_LDS(s16x4, reinterpret_cast<lds_ptr>((uintptr_t)addr0) + imm));
  const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16(HELIX_LDS(s16x4, reinterpret_cast<lds_ptr>((uintptr_t)addr1) + imm));
  const s16x8 ab = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, ab);
}

// Byte offsets, inside a swizzled [rows][D] tile, of the two transposing reads that give lane
// `lane` its MFMA operand for columns 32*db .. 32*db+31: rows 4*(lane/32) + 0..3 and, 8 rows
// further, the second group (the slot order of a bf16 pack of accumulator registers 8t..8t+7).
template <int D>
__device__ __forceinline__ void tr_pair_offsets(int lane, int db, int& off0, int& off1) {
  const int i = lane & 15;
  const int col = 32 * db + ((lane >> 4) & 1) * 16 + (i & 3) * 4;
  const int r0 = (lane >> 5) * 4 + (i >> 2);
  off0 = lds_chunk_off<D>(r0, col >> 3) + (col & 7) * 2;
  off1 = lds_chunk_off<D>(r0 + 8, col >> 3) + (col & 7) * 2;
}

// Two fp32 values rounded to nearest-even bf16 and packed into one register (low half first).
__device__ __forceinline__ uint32_t pack_bf16_pair(float a, float b) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  const f32x2 x = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}

// Forces a value loaded from global memory to be complete at this point of the program.
// Without it the compiler sinks such loads below the asynchronous tile copies and then
// waits for both together in the middle of the main loop.
template <typename T>
__device__ __forceinline__ void pin(T& x) { asm volatile("" : "+v"(x)); }

// MFMA operand whose 8 contraction slots are contiguous in memory: row `row`, elements
// 16*ks + 8*half .. +7 of a swizzled LDS tile.
template <int D>
__device__ __forceinline__ bf16x8 lds_operand(const char* tile, int row, int ks, int half) {
  return *reinterpret_cast<const bf16x8*>(tile + lds_chunk_off<D>(row, 2 * ks + half));
}

// MFMA operand whose contraction index runs over tile ROWS (the tile is stored row-major
// with the lane's own index along the row): lane l gets, for column col0 + l%32, the rows
//   row0 + 4*(l/32) + {0,1,2,3}   and   row0 + 8 + 4*(l/32) + {0,1,2,3},
// which is exactly the slot order of a bf16 pack of accumulator registers 8t..8t+7.
// ds_read_b64_tr_b16: within each group of 16 lanes, lane i supplies the address of row
// i/4, columns 4*(i%4)..+3 and receives column i of those four rows.
template <int D>
__device__ __forceinline__ bf16x8 lds_operand_tr(const char* tile, int row0, int col0, int lane) {
  int i = lane & 15;
  int col = col0 + ((lane >> 4) & 1) * 16 + (i & 3) * 4;
  int r0 = row0 + (lane >> 5) * 4 + (i >> 2);
  int off0 = lds_chunk_off<D>(r0, col >> 3) + (col & 7) * 2;
  int off1 = lds_chunk_off<D>(r0 + 8, col >> 3) + (col & 7) * 2;
  s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16(HELIX_LDS(s16x4, tile + off0));
  s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16(HELIX_LDS(s16x4, tile + off1));
  s16x8 ab = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, ab);
}

// bf16 pack (round to nearest even) of accumulator registers 8t..8t+7.
__device__ __forceinline__ bf16x8 pack_half(const f32x16& acc, int t) {
  f32x8 x;
#pragma unroll
  for (int e = 0; e < 8; e++) x[e] = acc[8 * t + e];
  return __builtin_convertvector(x, bf16x8);
}

// Map a linear workgroup id to (batch*head slice, tile).  Workgroup id mod 8 selects the XCD, and
// each XCD sweeps whole "virtual heads", heaviest tiles first (`heavy_is_high`: the heaviest
// tiles are those with the highest index (forward, dQ), else the lowest (dK/dV)).  A virtual
// head is one of P interleaved parts of a head (tiles congruent mod P), with P the smallest
// power of two that makes BH * P a multiple of 8: with 32 heads a virtual head is a head, with
// the 4 or 5 heads of one GPU's share of a tensor-parallel layer (Section 2.2) a head is
// spread over 2 or 8 XCDs so that none of them idles.
struct TileCoord { int bh; int tile; bool valid; };
__host__ __device__ inline int head_parts(int BH) { return (BH & 1) ? 8 : (BH & 2) ? 4 : (BH & 4) ? 2 : 1; }
// Number of workgroups to launch for BH slices of T tiles.
__host__ __device__ inline long long grid_blocks(int BH, int T) {
  const int P = head_parts(BH);
  return (long long)BH * P * ((T + P - 1) / P);
}
__device__ __forceinline__ TileCoord map_block(int n, int BH, int T, bool heavy_is_high) {
  TileCoord c;
  const int P = head_parts(BH), TP = (T + P - 1) / P;
  const int xcd = n & 7, s = n >> 3;
  const int vh = xcd + 8 * (s / TP);
  const int k = (s % TP) * P + (vh & (P - 1));   // rank of the tile inside its head, heaviest first
  c.bh = vh / P;
  c.tile = heavy_is_high ? (T - 1 - k) : k;
  c.valid = c.bh < BH && k < T;
  return c;
}

// Element offset of row 0 of slice bh = b * H + h.
__device__ __forceinline__ size_t head_offset(const TensorMap& m, int bh, int H) {
  const int b = bh / H;
  return (size_t)((long long)b * m.batch + (long long)(bh - b * H) * m.head);
}

}  // namespace helix

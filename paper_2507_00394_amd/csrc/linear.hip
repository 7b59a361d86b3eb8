// The QKV linear layer next to attention (Section 4.2: HelixPipe ships the layer's input and
// weights to the attention stage and runs the layer there) and its two backward products,
// as one bf16 MFMA GEMM kernel for gfx950:
//
//     C[i][j] = sum_r X(i, r) * Y(r, j),       fp32 accumulation
//
//   forward          qkv[M][N] = a[M][K]    * w[K][N]      X stored [i][r],  Y stored [r][j]
//   backward input   da[M][K]  = dqkv[M][N] * w[K][N]^T    X stored [i][r],  Y stored [r][j] after a transposing copy of w
//   backward weight  dw[K][N]  = a[M][K]^T  * dqkv[M][N]   X stored [r][i],  Y stored [r][j]
//
// A workgroup of 4 waves (one per SIMD) owns a 256 x 256 tile of C; wave (wi, wj) owns 128 rows i
// by 128 columns j as 4 x 4 accumulator blocks of the 32x32x16 MFMA (256 accumulator registers:
// with 2.5 instructions per MFMA one wave keeps the matrix unit busy), computed transposed
// (the MFMA's row index is j) so that a lane owns one row i of C and stores 4 consecutive j
// at a time.  The contraction runs in stages of 32: each stage's X and Y tiles (16 KB each)
// are copied global -> LDS asynchronously four stages ahead into five buffers (the scheme of the
// attention kernels, one buffer deeper because a stage is only 16 MFMAs per wave long).  An operand whose contraction index is contiguous in memory sits in LDS
// as [256][32] and is read with ds_read_b128; one whose contraction index is the row of the
// stored matrix sits as two [32][128] tiles and is read with the transposing LDS read.  Eight
// operand reads feed sixteen MFMAs; they are issued one sub-step (16 of the 32) ahead.
#include "helix_common.hpp"
#include "kernels.hpp"
#include <type_traits>

namespace helix {
namespace {

constexpr int kTile = 256;                    // rows i and columns j of C per workgroup
constexpr int kStep = 32;                     // contraction indices per stage
constexpr int kOperandTile = kTile * kStep * 2;   // bytes of one operand's stage tile (either layout)
constexpr int kStage = 2 * kOperandTile;
constexpr int kWaves = 4;                     // 2 x 2 waves, one per SIMD, each 128 x 128 of the tile
constexpr int kBlk = 4;                       // 32-wide blocks per wave in i and in j
constexpr int kStages = 5;                    // 5 x 32 KB: all of the 160 KB of LDS
constexpr int kAhead = kStages - 1;           // a stage's copy is issued this many iterations before its use

// Operand whose stored rows are the outer index (i or j) and whose contraction index is
// contiguous: LDS tile [256][32], 64-byte rows.
struct ContiguousOperand {
  static constexpr int DMA = TileLoader<32, kTile, kWaves>::N;       // copy instructions per wave and stage
  TileLoader<32, kTile, kWaves> loader;
  const __bf16* base;   // element (outer0, 0)
  int outer0, outer_n;
  __device__ __forceinline__ ContiguousOperand(const __bf16* p, long long ld, int outer0_, int outer_n_, int lane, int wave)
      : loader(lane, wave, (int)ld), base(p), outer0(outer0_), outer_n(outer_n_) {}
  __device__ __forceinline__ void copy(int r0, uint32_t lds) const { loader.issue(base + r0, outer0, outer_n, lds); }
  // lane addresses of the operand of 32-row block `blk` (rows blk0 + 32*blk + lane%32), sub-steps 0 and 1
  __device__ __forceinline__ static void addresses(int lane, int blk0, int blk, uint32_t (&a)[2]) {
    const int row = blk0 + 32 * blk + (lane & 31), half = lane >> 5;
    a[0] = lds_chunk_off<32>(row, half);
    a[1] = lds_chunk_off<32>(row, 2 + half);
  }
  __device__ __forceinline__ static bf16x8 read(const uint32_t (&a)[2], int ks) { return lds_b128(a[ks], 0); }
};

// Operand whose stored rows are the contraction index: LDS holds two [32][128] tiles (outer
// indices 0..127 and 128..255 of the workgroup tile), read with the transposing LDS read so
// that contraction slot e of lane half h is row 8h + e.
struct TransposedOperand {
  static constexpr int DMA = 2 * TileLoader<128, kStep, kWaves>::N;
  TileLoader<128, kStep, kWaves> loader;
  const __bf16* col[2];   // element (0, outer0) and (0, outer0 + 128); the second falls back to the first past the edge
  int r_n;
  __device__ __forceinline__ TransposedOperand(const __bf16* p, long long ld, int outer0, int outer_n, int r_n_, int lane, int wave)
      : loader(lane, wave, (int)ld), r_n(r_n_) {
    col[0] = p + outer0;
    col[1] = p + (outer0 + 128 < outer_n ? outer0 + 128 : outer0);
  }
  __device__ __forceinline__ void copy(int r0, uint32_t lds) const {
    loader.issue(col[0], r0, r_n, lds);
    loader.issue(col[1], r0, r_n, lds + kOperandTile / 2);
  }
  __device__ __forceinline__ static void addresses(int lane, int blk0, int blk, uint32_t (&a)[2]) {
    const int o = blk0 + 32 * blk;                 // first outer index of the block inside the workgroup tile
    const int i = lane & 15;
    const int c = (o & 127) + ((lane >> 4) & 1) * 16 + (i & 3) * 4;
    const int r = (lane >> 5) * 8 + (i >> 2);
    const int sub = (o >> 7) * (kOperandTile / 2);
    a[0] = sub + lds_chunk_off<128>(r, c >> 3) + (c & 7) * 2;
    a[1] = sub + lds_chunk_off<128>(r + 4, c >> 3) + (c & 7) * 2;
  }
  // rows 16*ks + ...: the swizzle has period 16 in the row, so the sub-step is an immediate
  __device__ __forceinline__ static bf16x8 read(const uint32_t (&a)[2], int ks) { return lds_tr_pair(a[0], a[1], ks * 16 * 256); }
};

template <typename T> struct StoreFour;
template <> struct StoreFour<__bf16> {
  __device__ __forceinline__ static void put(__bf16* p, f32x4 x) { *reinterpret_cast<bf16x4*>(p) = __builtin_convertvector(x, bf16x4); }
};
template <> struct StoreFour<float> {
  __device__ __forceinline__ static void put(float* p, f32x4 x) { *reinterpret_cast<f32x4*>(p) = x; }
};

}  // namespace

template <bool X_ROWS_ARE_R, bool Y_ROWS_ARE_R, typename OutT>
__global__ void __launch_bounds__(64 * kWaves) __attribute__((amdgpu_waves_per_eu(1, 1)))
gemm_kernel(const __bf16* __restrict__ X, long long ldx, const __bf16* __restrict__ Y, long long ldy,
            OutT* __restrict__ C, long long ldc, int I, int J, int R, int tiles_i, int tiles_j,
            int r_per_part, long long part_stride) {
  using XOp = typename std::conditional<X_ROWS_ARE_R, TransposedOperand, ContiguousOperand>::type;
  using YOp = typename std::conditional<Y_ROWS_ARE_R, TransposedOperand, ContiguousOperand>::type;
  extern __shared__ __align__(16) char smem[];

  // workgroup id mod 8 is the XCD: all column tiles of a row tile run on one XCD, so the X panel
  // is fetched into one L2 only
  const int xcd = blockIdx.x & 7, s = blockIdx.x >> 3;
  const int tj = s % tiles_j, ti = (s / tiles_j) * 8 + xcd;
  if (ti >= tiles_i) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wi = w & 1, wj = w >> 1;
  const int i0 = ti * kTile, j0 = tj * kTile;
  const uint32_t base = lds_base(smem);

  XOp xop_src = [&]() {
    if constexpr (X_ROWS_ARE_R) return TransposedOperand(X, ldx, i0, I, R, lane, w);
    else return ContiguousOperand(X, ldx, i0, I, lane, w);
  }();
  YOp yop_src = [&]() {
    if constexpr (Y_ROWS_ARE_R) return TransposedOperand(Y, ldy, j0, J, R, lane, w);
    else return ContiguousOperand(Y, ldy, j0, J, lane, w);
  }();
  constexpr int NDMA = XOp::DMA + YOp::DMA;
  // blockIdx.y selects a part of the contraction range; its partial result goes to C + y * part_stride
  const int r_begin = blockIdx.y * r_per_part;
  const int nk = ((R - r_begin < r_per_part ? R - r_begin : r_per_part)) / kStep;
  C += (size_t)blockIdx.y * part_stride;
  auto copy_stage = [&](int k, int buf) __attribute__((always_inline)) {
    xop_src.copy(r_begin + k * kStep, base + buf * kStage);
    yop_src.copy(r_begin + k * kStep, base + buf * kStage + kOperandTile);
  };
#pragma unroll
  for (int k = 0; k < kAhead; k++)
    if (k < nk) copy_stage(k, k);
  // iteration k reads stages k and k+1: the first two must be complete, the others may still fly
  if (nk >= kAhead) wait_tile_loads_except<(kAhead - 2) * NDMA>();   // all kAhead copies are out: the newest two may fly
  else wait_tile_loads();
  __syncthreads();

  uint32_t xa[kBlk][2], ya[kBlk][2];
#pragma unroll
  for (int b = 0; b < kBlk; b++) { XOp::addresses(lane, 32 * kBlk * wi, b, xa[b]); xa[b][0] += base; xa[b][1] += base; }
#pragma unroll
  for (int b = 0; b < kBlk; b++) { YOp::addresses(lane, 32 * kBlk * wj, b, ya[b]); ya[b][0] += base + kOperandTile; ya[b][1] += base + kOperandTile; }

  f32x16 acc[kBlk][kBlk];
#pragma unroll
  for (int jb = 0; jb < kBlk; jb++)
#pragma unroll
    for (int ib = 0; ib < kBlk; ib++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[jb][ib][e] = 0.f;

  bf16x8 xo[2][kBlk], yo[2][kBlk];   // [sub-step parity][block]
#pragma unroll
  for (int b = 0; b < kBlk; b++) xo[0][b] = XOp::read(xa[b], 0);
#pragma unroll
  for (int b = 0; b < kBlk; b++) yo[0][b] = YOp::read(ya[b], 0);

  int buf = 0;
  for (int k = 0; k < nk; k++) {
    if (k + kAhead < nk) copy_stage(k + kAhead, buf == 0 ? kStages - 1 : buf - 1);   // replaces stage k-1
    const int step = (buf == kStages - 1) ? -(kStages - 1) * kStage : kStage;
#pragma unroll
    for (int ks = 0; ks < 2; ks++) {
      // operands of the next sub-step: (k, 1) while (k, 0) is multiplied, then (k+1, 0) from the next buffer
      if (ks == 1) {
#pragma unroll
        for (int b = 0; b < kBlk; b++) { xa[b][0] += step; xa[b][1] += step; ya[b][0] += step; ya[b][1] += step; }
      }
#pragma unroll
      for (int m = 0; m < kBlk * kBlk; m++) {
        const int jb = m / kBlk, ib = m % kBlk;
        acc[jb][ib] = mfma32(yo[ks][jb], xo[ks][ib], acc[jb][ib]);
        if (m < kBlk) xo[ks ^ 1][m] = XOp::read(xa[m], ks ^ 1);
        else if (m < 2 * kBlk) yo[ks ^ 1][m - kBlk] = YOp::read(ya[m - kBlk], ks ^ 1);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // stages up to k+2 must have landed before the next iteration starts (it reads k+1 and k+2);
    // the copies of stages k+3 .. k+kAhead may stay in flight.  Near the end fewer copies are
    // outstanding than that, so waiting for "all but (kAhead-2) stages" is still sufficient.
    if (k + kAhead < nk) wait_tile_loads_except<(kAhead - 2) * NDMA>();
    else wait_tile_loads();
    __syncthreads();
    buf = (buf == kStages - 1) ? 0 : buf + 1;
  }

  // lane owns row i of C; accumulator registers 4g..4g+3 of block (jb, ib) are 4 consecutive columns
  const int half = lane >> 5, n = lane & 31;
#pragma unroll
  for (int ib = 0; ib < kBlk; ib++) {
    const int i = i0 + 32 * kBlk * wi + 32 * ib + n;
    if (i >= I) continue;
    OutT* row = C + (size_t)i * ldc;
#pragma unroll
    for (int jb = 0; jb < kBlk; jb++)
#pragma unroll
      for (int g = 0; g < 4; g++) {
        const int j = j0 + 32 * kBlk * wj + 32 * jb + 8 * g + 4 * half;
        if (j >= J) continue;
        const f32x4 x = {acc[jb][ib][4 * g], acc[jb][ib][4 * g + 1], acc[jb][ib][4 * g + 2], acc[jb][ib][4 * g + 3]};
        StoreFour<OutT>::put(row + j, x);
      }
  }
}

// dst[e] = sum over `parts` slabs of src, `n` elements each (n a multiple of 4).
__global__ void __launch_bounds__(256) sum_parts_kernel(const float* __restrict__ src, float* __restrict__ dst, long long ld_dst,
                                                        int rows, int cols, int parts) {
  const long long quad = (long long)blockIdx.x * 256 + threadIdx.x;
  const int qpr = cols / 4;
  if (quad >= (long long)rows * qpr) return;
  const int r = (int)(quad / qpr), c = (int)(quad % qpr) * 4;
  const size_t slab = (size_t)rows * cols;
  f32x4 acc = *reinterpret_cast<const f32x4*>(src + (size_t)r * cols + c);
  for (int p = 1; p < parts; p++) acc += *reinterpret_cast<const f32x4*>(src + p * slab + (size_t)r * cols + c);
  *reinterpret_cast<f32x4*>(dst + (size_t)r * ld_dst + c) = acc;
}

template <bool XR, bool YR, typename OutT>
static hipError_t launch_gemm(const void* X, long long ldx, const void* Y, long long ldy, void* C, long long ldc,
                              int I, int J, int R, int parts, int r_per_part, long long part_stride, hipStream_t stream) {
  const int tiles_i = (I + kTile - 1) / kTile, tiles_j = (J + kTile - 1) / kTile;
  const unsigned grid = 8u * ((tiles_i + 7) / 8) * tiles_j;
  const size_t lds = (size_t)kStages * kStage;
  auto kern = gemm_kernel<XR, YR, OutT>;
  static unsigned long long configured = 0;   // one static per template instantiation
  hipError_t e = allow_dynamic_lds(kern, lds, configured);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(grid, (unsigned)parts), dim3(64 * kWaves), lds, stream, (const __bf16*)X, ldx, (const __bf16*)Y, ldy,
                     (OutT*)C, ldc, I, J, R, tiles_i, tiles_j, r_per_part, part_stride);
  return hipGetLastError();
}

hipError_t launch_linear_fwd(const void* a, long long lda, const void* w, long long ldw, void* out, long long ldo,
                             int M, int K, int N, hipStream_t stream) {
  return launch_gemm<false, true, __bf16>(a, lda, w, ldw, out, ldo, M, N, K, 1, K, 0, stream);
}
// out[c][r] = in[r][c] for a [rows][cols] bf16 matrix (both extents multiples of 64).
__global__ void __launch_bounds__(256) transpose_kernel(const __bf16* __restrict__ in, long long ld_in,
                                                        __bf16* __restrict__ out, long long ld_out) {
  __shared__ __bf16 tile[64][66];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const size_t r0 = (size_t)blockIdx.y * 64, c0 = (size_t)blockIdx.x * 64;
#pragma unroll
  for (int i = 0; i < 16; i++) tile[ty * 16 + i][tx] = in[(r0 + ty * 16 + i) * ld_in + c0 + tx];
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; i++) out[(c0 + ty * 16 + i) * ld_out + r0 + tx] = tile[tx][ty * 16 + i];
}

// Input gradient da = dout * w^T.  With w as stored ([K][N], contraction index n contiguous) both
// operands would reach LDS in 64-byte row pieces, the least efficient pattern of the copy path
// (measured 30 % slower than the forward product); a transposed copy of the small weight matrix
// (w^T [N][K], in the workspace) turns it into the forward's operand combination.
hipError_t launch_linear_bwd_input(const void* dout, long long ldd, const void* w, long long ldw, void* da, long long lda,
                                   void* wt, int M, int K, int N, hipStream_t stream) {
  hipLaunchKernelGGL(transpose_kernel, dim3((unsigned)(N / 64), (unsigned)(K / 64)), dim3(256), 0, stream,
                     (const __bf16*)w, ldw, (__bf16*)wt, (long long)K);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_gemm<false, true, __bf16>(dout, ldd, wt, K, da, lda, M, K, N, 1, N, 0, stream);
}

// The weight gradient has few output tiles and a long contraction (over all M tokens), so the
// contraction is cut into parts until the grid fills the chip about twice; the parts' fp32
// results go to the workspace and are summed in a fixed order (no atomics).
int linear_bwd_weight_parts(int M, int K, int N) {
  const long long tiles = (long long)((K + kTile - 1) / kTile) * ((N + kTile - 1) / kTile);
  long long parts = (512 + tiles - 1) / tiles;
  const long long most = M / 2048 > 0 ? M / 2048 : 1;      // at least 2048 tokens per part
  if (parts > most) parts = most;
  if (parts > 32) parts = 32;
  return (int)parts;
}
// Workspace of the backward: w^T (bf16 [N][K], rounded up to 256 bytes), then the partial weight gradients.
size_t linear_bwd_wt_bytes(int K, int N) { return ((size_t)K * N * 2 + 255) & ~(size_t)255; }
size_t linear_bwd_workspace_bytes(int M, int K, int N) {
  const int parts = linear_bwd_weight_parts(M, K, N);
  return linear_bwd_wt_bytes(K, N) + (parts > 1 ? (size_t)parts * K * N * sizeof(float) : 0);
}
hipError_t launch_linear_bwd_weight(const void* a, long long lda, const void* dout, long long ldd, float* dw, long long ldw,
                                    float* workspace, int M, int K, int N, hipStream_t stream) {
  const int parts = linear_bwd_weight_parts(M, K, N);
  if (parts == 1) return launch_gemm<true, true, float>(a, lda, dout, ldd, dw, ldw, K, N, M, 1, M, 0, stream);
  const int per = ((M / kStep + parts - 1) / parts) * kStep;    // tokens per part, a multiple of the stage length
  hipError_t e = launch_gemm<true, true, float>(a, lda, dout, ldd, workspace, N, K, N, M, parts, per, (long long)K * N, stream);
  if (e != hipSuccess) return e;
  const long long quads = (long long)K * N / 4;
  hipLaunchKernelGGL(sum_parts_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, stream, workspace, dw, ldw, K, N, parts);
  return hipGetLastError();
}

}  // namespace helix

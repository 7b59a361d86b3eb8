// Sustained rate of the bf16 MFMA pipes on this chip: a loop of independent
// v_mfma_f32_32x32x16_bf16 instructions and nothing else (no LDS, no memory, no vector ALU).
// The attention kernels cannot be faster per MFMA than this loop; bench.py runs it next to
// them and reports the measured rate as a second denominator beside the nominal peak
// (256 compute units x 4096 FLOP per clock x peak clock).  With random operand bits the
// multiplier arrays toggle as they do on real data and the chip's power management lowers
// the clock; with constant operands it does not, which is why both are measured.
#include "helix_common.hpp"
#include "kernels.hpp"

namespace helix {

namespace {
constexpr int kProbeWaves = 8;          // two waves per SIMD
constexpr int kProbeUnroll = 16;        // MFMAs per loop iteration and wave
}

template <bool RANDOM>
__global__ void __launch_bounds__(64 * kProbeWaves) mfma_probe_kernel(float* __restrict__ sink, int iters) {
  // eight operand registers; RANDOM: bf16 values with random sign / mantissa bits and exponents
  // near 1 (products stay finite), else 1.0 everywhere
  bf16x8 op[8];
  uint32_t x = 0x9E3779B9u * (blockIdx.x * blockDim.x + threadIdx.x + 1);
#pragma unroll
  for (int r = 0; r < 8; r++) {
    s16x8 bits;
#pragma unroll
    for (int e = 0; e < 8; e++) {
      x ^= x << 13; x ^= x >> 17; x ^= x << 5;   // xorshift32
      bits[e] = RANDOM ? (short)((x & 0x807Fu) | (((x >> 8) & 3u) + 125u) << 7) : (short)0x3F80;
    }
    op[r] = __builtin_bit_cast(bf16x8, bits);
  }
  f32x16 acc[4];
#pragma unroll
  for (int a = 0; a < 4; a++)
#pragma unroll
    for (int e = 0; e < 16; e++) acc[a][e] = 0.f;
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int s = 0; s < kProbeUnroll; s++) acc[s & 3] = mfma32(op[s & 7], op[(s + 3) & 7], acc[s & 3]);
    if (RANDOM && (it & 63) == 63) {
      // keep the sums bounded: random-sign products grow like sqrt(n), halve them now and then
#pragma unroll
      for (int a = 0; a < 4; a++)
#pragma unroll
        for (int e = 0; e < 16; e++) acc[a][e] *= 0.5f;
    }
  }
  float total = 0.f;
#pragma unroll
  for (int a = 0; a < 4; a++)
#pragma unroll
    for (int e = 0; e < 16; e++) total += acc[a][e];
  if (total == 123.456f) sink[0] = total;   // keeps the loop alive; practically never true
}

// The same loop with the company an MFMA has in the attention kernels: per MFMA one 1 KB operand
// read from LDS (through a four-deep register ring, as there), FMA fused multiply-adds and
// EXP2 / 2 exponentials on values of their own.  Random operands.  What this loop sustains is
// what a kernel with that instruction mix can reach with no barriers, copies or dependencies
// in its way; (1 read, 2 fma, 0.5 exp2) is the mix of the two backward passes, (1, 3, 1) that
// of the forward.
template <int FMA, int EXP2>
__global__ void __launch_bounds__(64 * kProbeWaves) mfma_mix_probe_kernel(float* __restrict__ sink, int iters) {
  __shared__ __align__(16) short tile[32768];   // 64 KB of operand bits
  uint32_t x = 0x9E3779B9u * (blockIdx.x * blockDim.x + threadIdx.x + 1);
  auto bits = [&]() { x ^= x << 13; x ^= x >> 17; x ^= x << 5; return (short)((x & 0x807Fu) | (((x >> 8) & 3u) + 125u) << 7); };
  for (int i = threadIdx.x; i < 32768; i += 64 * kProbeWaves) tile[i] = bits();
  bf16x8 op[8];
#pragma unroll
  for (int r = 0; r < 8; r++) {
    s16x8 b;
#pragma unroll
    for (int e = 0; e < 8; e++) b[e] = bits();
    op[r] = __builtin_bit_cast(bf16x8, b);
  }
  __syncthreads();
  const uint32_t base = lds_base(reinterpret_cast<const char*>(tile)) + (threadIdx.x & 63) * 16;
  f32x16 acc[4];
#pragma unroll
  for (int a = 0; a < 4; a++)
#pragma unroll
    for (int e = 0; e < 16; e++) acc[a][e] = 0.f;
  bf16x8 ring[4] = {op[0], op[1], op[2], op[3]};
  float v[8];
#pragma unroll
  for (int i = 0; i < 8; i++) v[i] = 0.001f * (float)(threadIdx.x + i);
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int s = 0; s < kProbeUnroll; s++) {
      acc[s & 3] = mfma32(ring[s & 3], op[(s + 3) & 7], acc[s & 3]);
      ring[s & 3] = lds_b128(base, 1024 * ((s * 5 + it) & 31));
#pragma unroll
      for (int k = 0; k < FMA; k++) v[(s + k) & 7] = fmaf(v[(s + k) & 7], 0.999f, 0.0001f);
      if (EXP2 >= 2 || (EXP2 == 1 && (s & 1))) v[s & 7] = __builtin_amdgcn_exp2f(v[s & 7] * 0.5f - 1.0f);
      __builtin_amdgcn_sched_barrier(0);
    }
    if ((it & 63) == 63) {
#pragma unroll
      for (int a = 0; a < 4; a++)
#pragma unroll
        for (int e = 0; e < 16; e++) acc[a][e] *= 0.5f;
    }
  }
  float total = 0.f;
#pragma unroll
  for (int a = 0; a < 4; a++)
#pragma unroll
    for (int e = 0; e < 16; e++) total += acc[a][e];
#pragma unroll
  for (int i = 0; i < 8; i++) total += v[i];
  if (total == 123.456f) sink[0] = total;
}

long long mfma_probe_flops(int workgroups, int iters) {
  return (long long)workgroups * kProbeWaves * iters * kProbeUnroll * (2LL * 32 * 32 * 16);
}

hipError_t launch_mfma_probe(float* sink, int workgroups, int iters, bool random_operands, hipStream_t stream) {
  if (random_operands) hipLaunchKernelGGL(mfma_probe_kernel<true>, dim3(workgroups), dim3(64 * kProbeWaves), 0, stream, sink, iters);
  else hipLaunchKernelGGL(mfma_probe_kernel<false>, dim3(workgroups), dim3(64 * kProbeWaves), 0, stream, sink, iters);
  return hipGetLastError();
}

hipError_t launch_mfma_mix_probe(float* sink, int workgroups, int iters, bool forward_mix, hipStream_t stream) {
  if (forward_mix) hipLaunchKernelGGL((mfma_mix_probe_kernel<3, 2>), dim3(workgroups), dim3(64 * kProbeWaves), 0, stream, sink, iters);
  else hipLaunchKernelGGL((mfma_mix_probe_kernel<2, 1>), dim3(workgroups), dim3(64 * kProbeWaves), 0, stream, sink, iters);
  return hipGetLastError();
}

}  // namespace helix

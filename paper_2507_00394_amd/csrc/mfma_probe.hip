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

long long mfma_probe_flops(int workgroups, int iters) {
  return (long long)workgroups * kProbeWaves * iters * kProbeUnroll * (2LL * 32 * 32 * 16);
}

hipError_t launch_mfma_probe(float* sink, int workgroups, int iters, bool random_operands, hipStream_t stream) {
  if (random_operands) hipLaunchKernelGGL(mfma_probe_kernel<true>, dim3(workgroups), dim3(64 * kProbeWaves), 0, stream, sink, iters);
  else hipLaunchKernelGGL(mfma_probe_kernel<false>, dim3(workgroups), dim3(64 * kProbeWaves), 0, stream, sink, iters);
  return hipGetLastError();
}

}  // namespace helix

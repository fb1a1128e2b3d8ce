// Matrix-pipe probe: what a stream of v_mfma_f32_32x32x16_bf16 with one 16-byte LDS read per product (the ratio of the
// patch-tiled convolution kernels) reaches on this device, with operands of all zeros or of random bfloat16 values.
// The device lowers its clock and issue rate with the switching activity of the operands, so the second figure, not
// the data-sheet peak, is what a convolution on N(0,1) data can approach.  No global memory traffic in the loop.
#include <hip/hip_runtime.h>

#include "kernels.hpp"
#include "conv_common.hpp"

namespace lms {

// Target of the store that keeps the probe's products alive; external linkage, so the store cannot be proved dead.
__device__ float mfma_probe_sink[256];

namespace {

constexpr int PROBE_WGS = 512;          // two work-groups of four waves per compute unit
constexpr int PROBE_LDS = 65536;

__global__ __launch_bounds__(256, 2) void mfma_probe_kernel(unsigned iters, int random_operands) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[PROBE_LDS];
  for (int i = threadIdx.x; i < PROBE_LDS / 4; i += 256) {
    unsigned h = (unsigned)i * 2654435761u + blockIdx.x * 40503u + 12345u;
    h ^= h >> 13; h *= 0x5bd1e995u; h ^= h >> 15;
    // two bfloat16 per word: random sign and mantissa, exponent field 124..127 (0.125 <= |x| < 2)
    const unsigned lo = (h & 0x807fu) | ((124u + ((h >> 8) & 3u)) << 7);
    const unsigned hi = ((h >> 16) & 0x807fu) | ((124u + ((h >> 28) & 3u)) << 7);
    reinterpret_cast<unsigned*>(smem)[i] = random_operands ? (lo | (hi << 16)) : 0u;
  }
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // a wave reads rows of 1 KiB of its quarter of the buffer, lane l the 16 bytes at 16 l: no bank conflicts
  const unsigned char* base = smem + wave * (PROBE_LDS / 4) + lane * 16;
  bf16x8 fr[8];
#pragma unroll
  for (int r = 0; r < 8; ++r) fr[r] = *reinterpret_cast<const bf16x8*>(base + r * 1024);
  f32x16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
  for (unsigned it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
#pragma unroll
      for (int r = 0; r < 4; ++r) fr[(u * 4 + r) & 7] = *reinterpret_cast<const bf16x8*>(base + (((it & 3) * 4 + u) * (r + 1) & 15) * 1024);
#pragma unroll
      for (int m = 0; m < 4; ++m)
        acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[(u * 4 + m) & 7], fr[(u * 4 + m + 1) & 7], acc[m], 0, 0, 0);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[j][v];
  if (s == 12345.678f) mfma_probe_sink[threadIdx.x] = s;      // keeps the products alive; practically never taken
}

}  // namespace

uint64_t mfma_probe_flops(unsigned iters) { return (uint64_t)PROBE_WGS * 4 * iters * 16 * 32768; }

hipError_t launch_mfma_probe(unsigned iters, int random_operands, hipStream_t s) {
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(PROBE_WGS), dim3(256), 0, s, iters, random_operands);
  return hipGetLastError();
}

}  // namespace lms

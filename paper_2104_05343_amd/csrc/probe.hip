// Measurement aid (not part of the method): how fast the matrix cores of this chip really go.
// A loop of nothing but v_mfma_f32_32x32x16_bf16 on register operands -- no LDS, no memory -- run on a chosen number
// of workgroups (one per CU, eight wavefronts each) with operands that are either all zero or pseudo-random bf16
// values.  The rate depends on both: with every CU busy and operands that toggle like real activations the chip's
// power management holds the matrix cores well below the rate of one CU alone, which is the ceiling any product
// kernel on such data works under (see the benchmark's "mfma_ceiling" rows).
#include "common.hpp"

namespace optimus {

typedef __attribute__((ext_vector_type(8))) __bf16 probe_bf16x8;
typedef __attribute__((ext_vector_type(16))) float probe_f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned probe_u32x4;

__global__ __launch_bounds__(512) void mfma_rate_kernel(float* out, int iters, int random_data) {
  const int tid = threadIdx.x;
  probe_bf16x8 f[8];
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    probe_u32x4 w;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      // two bf16 per word: random sign and mantissa, exponent 126..127 (magnitude around one), or zeros
      unsigned h = (unsigned)(tid * 37 + r * 4 + e + 1) * 2654435761u;
      h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
      const unsigned lo = (h & 0x80ffu) | 0x3f00u, hi = ((h >> 16) & 0x80ffu) | 0x3f00u;
      w[e] = random_data ? (lo | (hi << 16)) : 0u;
    }
    f[r] = __builtin_bit_cast(probe_bf16x8, w);
  }
  probe_f32x16 acc[8];
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[a][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < 8; ++m) acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[m], f[(m + 3) & 7], acc[m], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int a = 0; a < 8; ++a) s += acc[a][0] + acc[a][9];
  out[(size_t)blockIdx.x * 512 + tid] = s;
}

// out: workgroups * 512 floats.  flops = workgroups * 8 wavefronts * iters * 8 instructions * 2 * 32 * 32 * 16
int launch_mfma_rate(float* out, int workgroups, int iters, int random_data, hipStream_t st) {
  hipLaunchKernelGGL(mfma_rate_kernel, dim3((unsigned)workgroups), dim3(512), 0, st, out, iters, random_data);
  return hip_launch_status();
}

}  // namespace optimus

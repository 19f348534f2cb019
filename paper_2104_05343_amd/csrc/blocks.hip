// Block addressing of the q x q partition (Section 2.4 of the paper): row-major <-> block-major copies.
#include "common.hpp"

namespace optimus {

template <typename T>
__global__ __launch_bounds__(256) void pack_kernel(const T* __restrict__ src, T* __restrict__ dst, long long R, long long C, int q, int unpack) {
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;  // index in row-major order
  if (idx >= R * C) return;
  long long row = idx / C, col = idx % C;
  long long r = R / q, c = C / q;
  long long bi = row / r, rr = row % r, bj = col / c, cc = col % c;
  long long bidx = ((bi * q + bj) * r + rr) * c + cc;
  if (unpack) dst[idx] = src[bidx];
  else dst[bidx] = src[idx];
}

int launch_pack(const void* src, void* dst, long long R, long long C, int q, int elem_bytes, bool unpack, hipStream_t stream) {
  long long total = R * C;
  long long blocks = (total + 255) / 256;
  if (blocks > 0x7fffffffLL) return OPTIMUS_ESHAPE;
  if (elem_bytes == 2)
    hipLaunchKernelGGL(pack_kernel<unsigned short>, dim3((unsigned)blocks), dim3(256), 0, stream, (const unsigned short*)src,
                       (unsigned short*)dst, R, C, q, unpack ? 1 : 0);
  else
    hipLaunchKernelGGL(pack_kernel<unsigned int>, dim3((unsigned)blocks), dim3(256), 0, stream, (const unsigned int*)src,
                       (unsigned int*)dst, R, C, q, unpack ? 1 : 0);
  return hip_launch_status();
}

// Sum of `count` dense fp32 partial blocks in index order (the reduce of Algorithms 2 / 3 onto its root, or the local
// accumulation of Algorithm 1), written into one block of the output in its dtype.
template <typename T>
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ parts, T* __restrict__ dst, long long n,
                                                              int count) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n) return;
  float acc = parts[idx];
  for (int k = 1; k < count; ++k) acc += parts[(long long)k * n + idx];
  if (sizeof(T) == 2) dst[idx] = (T)f32_to_bf16(acc);
  else ((float*)dst)[idx] = acc;
}

int launch_reduce_partials(const float* parts, void* dst, long long n, int count, int dtype, hipStream_t stream) {
  const long long blocks = (n + 255) / 256;
  if (blocks > 0x7fffffffLL || count < 1) return OPTIMUS_ESHAPE;
  if (dtype == OPTIMUS_BF16)
    hipLaunchKernelGGL(reduce_partials_kernel<unsigned short>, dim3((unsigned)blocks), dim3(256), 0, stream, parts,
                       (unsigned short*)dst, n, count);
  else
    hipLaunchKernelGGL(reduce_partials_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, stream, parts, (float*)dst, n, count);
  return hip_launch_status();
}

}  // namespace optimus

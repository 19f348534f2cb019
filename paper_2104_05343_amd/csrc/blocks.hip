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

}  // namespace optimus

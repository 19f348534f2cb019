// Row soft-max of attention scores and its backward (local attention of Sections 2.1 / 3.2.1 of the paper:
// the whole sequence lives on one device, so rows are never split).
// One wavefront owns one row: fp32 scores are read once with 16-byte loads into registers, max and sum are
// wave reductions, probabilities are written once as bf16.  With a causal mask only columns <= row are read;
// columns above the diagonal are written as exact zeros so that P is a complete saved tensor.
#include "common.hpp"

namespace optimus {

__device__ __forceinline__ float wsum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ float wmax(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}

// ITS: float4 chunks per lane; handles s <= 256*ITS, s % 4 == 0
template <int ITS>
__global__ __launch_bounds__(256) void softmax_fwd_kernel(const float* __restrict__ S, bf16_t* __restrict__ P, long long nrows, int s, int causal) {
  const int lane = threadIdx.x & 63;
  const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= nrows) return;
  const int r = (int)(row % s);
  const int last = causal ? r : s - 1;  // last valid column
  const float* src = S + row * s;
  bf16_t* dst = P + row * s;
  float v[ITS * 4];
  float mx = -INFINITY;
#pragma unroll
  for (int it = 0; it < ITS; ++it) {
    int col = (it * 64 + lane) * 4;
    if (col <= last && col < s) {
      float4 w = *(const float4*)(src + col);
      v[it * 4 + 0] = w.x;
      v[it * 4 + 1] = col + 1 <= last ? w.y : -INFINITY;
      v[it * 4 + 2] = col + 2 <= last ? w.z : -INFINITY;
      v[it * 4 + 3] = col + 3 <= last ? w.w : -INFINITY;
    } else {
      v[it * 4 + 0] = v[it * 4 + 1] = v[it * 4 + 2] = v[it * 4 + 3] = -INFINITY;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) mx = fmaxf(mx, v[it * 4 + k]);
  }
  mx = wmax(mx);
  float sum = 0.f;
#pragma unroll
  for (int k = 0; k < ITS * 4; ++k) {
    v[k] = __expf(v[k] - mx);  // exp(-inf) = 0 for masked entries
    sum += v[k];
  }
  sum = wsum(sum);
  const float inv = 1.0f / sum;
#pragma unroll
  for (int it = 0; it < ITS; ++it) {
    int col = (it * 64 + lane) * 4;
    if (col < s)
      *(uint2*)(dst + col) = make_uint2(pack2_bf16(v[it * 4] * inv, v[it * 4 + 1] * inv), pack2_bf16(v[it * 4 + 2] * inv, v[it * 4 + 3] * inv));
  }
}

// dS = P * (dP - sum_k dP_k P_k)
template <int ITS>
__global__ __launch_bounds__(256) void softmax_bwd_kernel(const float* __restrict__ dP, const bf16_t* __restrict__ P, bf16_t* __restrict__ dS,
                                                          long long nrows, int s, int causal) {
  const int lane = threadIdx.x & 63;
  const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= nrows) return;
  const int r = (int)(row % s);
  const int last = causal ? r : s - 1;
  const float* gsrc = dP + row * s;
  const bf16_t* psrc = P + row * s;
  bf16_t* dst = dS + row * s;
  float g[ITS * 4], p[ITS * 4];
  float dot = 0.f;
#pragma unroll
  for (int it = 0; it < ITS; ++it) {
    int col = (it * 64 + lane) * 4;
    if (col <= last && col < s) {
      float4 w = *(const float4*)(gsrc + col);
      uint2 pw = *(const uint2*)(psrc + col);
      p[it * 4 + 0] = __uint_as_float(pw.x << 16);
      p[it * 4 + 1] = __uint_as_float(pw.x & 0xffff0000u);
      p[it * 4 + 2] = __uint_as_float(pw.y << 16);
      p[it * 4 + 3] = __uint_as_float(pw.y & 0xffff0000u);
      g[it * 4 + 0] = w.x;
      g[it * 4 + 1] = col + 1 <= last ? w.y : 0.f;  // beyond the diagonal dP was never computed
      g[it * 4 + 2] = col + 2 <= last ? w.z : 0.f;
      g[it * 4 + 3] = col + 3 <= last ? w.w : 0.f;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if (col + k > last) p[it * 4 + k] = 0.f;
        dot += g[it * 4 + k] * p[it * 4 + k];
      }
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k) { g[it * 4 + k] = 0.f; p[it * 4 + k] = 0.f; }
    }
  }
  dot = wsum(dot);
#pragma unroll
  for (int it = 0; it < ITS; ++it) {
    int col = (it * 64 + lane) * 4;
    if (col < s) {
      float o[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) o[k] = p[it * 4 + k] * (g[it * 4 + k] - dot);
      *(uint2*)(dst + col) = make_uint2(pack2_bf16(o[0], o[1]), pack2_bf16(o[2], o[3]));
    }
  }
}

template <int ITS>
static int run_fwd(const float* S, void* P, long long nrows, int s, int causal, hipStream_t st) {
  hipLaunchKernelGGL(softmax_fwd_kernel<ITS>, dim3((unsigned)((nrows + 3) / 4)), dim3(256), 0, st, S, (bf16_t*)P, nrows, s, causal);
  return hip_launch_status();
}
template <int ITS>
static int run_bwd(const float* dP, const void* P, void* dS, long long nrows, int s, int causal, hipStream_t st) {
  hipLaunchKernelGGL(softmax_bwd_kernel<ITS>, dim3((unsigned)((nrows + 3) / 4)), dim3(256), 0, st, dP, (const bf16_t*)P, (bf16_t*)dS, nrows, s, causal);
  return hip_launch_status();
}

int launch_softmax_fwd(const float* S, void* P, int nmat, int s, int causal, hipStream_t st) {
  if (s % 4 || s > 4096) return OPTIMUS_ESHAPE;
  long long nrows = (long long)nmat * s;
  if (s <= 256) return run_fwd<1>(S, P, nrows, s, causal, st);
  if (s <= 512) return run_fwd<2>(S, P, nrows, s, causal, st);
  if (s <= 1024) return run_fwd<4>(S, P, nrows, s, causal, st);
  if (s <= 2048) return run_fwd<8>(S, P, nrows, s, causal, st);
  return run_fwd<16>(S, P, nrows, s, causal, st);
}
int launch_softmax_bwd(const float* dP, const void* P, void* dS, int nmat, int s, int causal, hipStream_t st) {
  if (s % 4 || s > 4096) return OPTIMUS_ESHAPE;
  long long nrows = (long long)nmat * s;
  if (s <= 256) return run_bwd<1>(dP, P, dS, nrows, s, causal, st);
  if (s <= 512) return run_bwd<2>(dP, P, dS, nrows, s, causal, st);
  if (s <= 1024) return run_bwd<4>(dP, P, dS, nrows, s, causal, st);
  if (s <= 2048) return run_bwd<8>(dP, P, dS, nrows, s, causal, st);
  return run_bwd<16>(dP, P, dS, nrows, s, causal, st);
}

}  // namespace optimus

// Accumulator -> C epilogue shared by the matrix-core and the scalar product kernels
// (bias slice, GeLU, GeLU' scaling, residual; Sections 3.2.1-3.2.2 of the paper: applied locally per block).
#pragma once
#include "common.hpp"

namespace optimus {

struct EpiArgs {
  float alpha;
  const float* bias;  // already offset to this batch's slice, or nullptr
  void* C;
  void* pre_act;
  const void* gelu_grad_of;
  const void* residual;
  int ldc;
  int act;
  int out_fp32;
  int in_bf16;
  int vec_ok;  // all bases/strides allow 4-element vector accesses
};

__device__ __forceinline__ float load_elem(const void* p, long long idx, int bf16) {
  return bf16 ? bf16_to_f32(((const bf16_t*)p)[idx]) : ((const float*)p)[idx];
}
__device__ __forceinline__ void store_elem(void* p, long long idx, int bf16, float v) {
  if (bf16) ((bf16_t*)p)[idx] = f32_to_bf16(v);
  else ((float*)p)[idx] = v;
}

// GeLU of four values.  EXACT: erff (fp32 kernels, tolerance 1e-5); otherwise the short rational form (bf16 kernels,
// which unroll this epilogue 64-256 times per lane and must stay small enough to unroll fully).
template <bool EXACT>
__device__ __forceinline__ void gelu4(float (&t)[4]) {
#pragma unroll
  for (int c = 0; c < 4; ++c) t[c] = EXACT ? gelu_exact(t[c]) : gelu_fast(t[c]);
}
template <bool EXACT>
__device__ __forceinline__ void gelu_grad_mul4(float (&t)[4], const float (&z)[4]) {
#pragma unroll
  for (int c = 0; c < 4; ++c) t[c] *= EXACT ? gelu_grad_exact(z[c]) : gelu_grad_fast(z[c]);
}

// v[0..3]: accumulators of row m, columns n..n+3 (n % 4 == 0); coff: element offset of this batch's C block;
// nvalid: how many of the four columns exist.  VEC_ONLY: the caller guarantees e.vec_ok and nvalid == 4.
template <bool VEC_ONLY = false, bool EXACT = false>
__device__ __forceinline__ void epilogue_store4(const EpiArgs& e, long long coff, int m, int n, const float (&v)[4], int nvalid) {
  long long off = coff + (long long)m * e.ldc + n;
  float t[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) t[c] = v[c] * e.alpha;
  if (e.bias) {
#pragma unroll
    for (int c = 0; c < 4; ++c)
      if (c < nvalid) t[c] += e.bias[n + c];
  }
  const bool vec = VEC_ONLY || (e.vec_ok && nvalid == 4);
  if (e.pre_act) {
    if (vec && e.in_bf16) {
      uint2 w = make_uint2(pack2_bf16(t[0], t[1]), pack2_bf16(t[2], t[3]));
      *(uint2*)((bf16_t*)e.pre_act + off) = w;
    } else if (vec) {
      *(float4*)((float*)e.pre_act + off) = make_float4(t[0], t[1], t[2], t[3]);
    } else if (!VEC_ONLY) {
      for (int c = 0; c < nvalid; ++c) store_elem(e.pre_act, off + c, e.in_bf16, t[c]);
    }
  }
  if (e.act == 1) gelu4<EXACT>(t);
  if (e.gelu_grad_of) {
    float z[4] = {0.f, 0.f, 0.f, 0.f};
    if (vec && e.in_bf16) {
      uint2 w = *(const uint2*)((const bf16_t*)e.gelu_grad_of + off);
      z[0] = __uint_as_float(w.x << 16); z[1] = __uint_as_float(w.x & 0xffff0000u);
      z[2] = __uint_as_float(w.y << 16); z[3] = __uint_as_float(w.y & 0xffff0000u);
    } else if (!VEC_ONLY) {
      for (int c = 0; c < nvalid; ++c) z[c] = load_elem(e.gelu_grad_of, off + c, e.in_bf16);
    }
    gelu_grad_mul4<EXACT>(t, z);
  }
  if (e.residual) {
    float r[4] = {0.f, 0.f, 0.f, 0.f};
    if (vec && e.in_bf16) {
      uint2 w = *(const uint2*)((const bf16_t*)e.residual + off);
      r[0] = __uint_as_float(w.x << 16); r[1] = __uint_as_float(w.x & 0xffff0000u);
      r[2] = __uint_as_float(w.y << 16); r[3] = __uint_as_float(w.y & 0xffff0000u);
    } else if (!VEC_ONLY) {
      for (int c = 0; c < nvalid; ++c) r[c] = load_elem(e.residual, off + c, e.in_bf16);
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) t[c] += r[c];
  }
  const int out_bf16 = e.in_bf16 && !e.out_fp32;
  if (vec && out_bf16) {
    *(uint2*)((bf16_t*)e.C + off) = make_uint2(pack2_bf16(t[0], t[1]), pack2_bf16(t[2], t[3]));
  } else if (vec) {
    *(float4*)((float*)e.C + off) = make_float4(t[0], t[1], t[2], t[3]);
  } else if (!VEC_ONLY) {
    for (int c = 0; c < nvalid; ++c) store_elem(e.C, off + c, out_bf16, t[c]);
  }
}

}  // namespace optimus

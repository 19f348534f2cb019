// Scalar-FMA product kernel: any shape, fp32 or bf16 storage, fp32 accumulation.
// Used for the fp32 path and for bf16 shapes whose rows are not multiples of 8 elements.
// Same panel loop as the matrix-core kernel: the q SUMMA steps (Algorithms 1-3) are one k-loop.
#include "common.hpp"
#include "epilogue.hpp"

namespace optimus {

struct GArgs {
  const void* A;
  const void* B;
  int Mb, Nb, Kp, nl;
  int lda, ldb;
  long long sAl, sBl;
  int nz0;
  long long sA0, sA1, sB0, sB1, sC0, sC1, sBias0;
  int a_kcontig, b_kcontig;
  int tiles_m, tiles_n;
  int skip_upper, k_hi_diag, k_lo_diag;
  EpiArgs epi;
};

constexpr int GT = 64;  // output tile
constexpr int GK = 16;  // k slab

__global__ __launch_bounds__(256) void gemm_generic_kernel(const GArgs a) {
  __shared__ float As[GK][GT + 4];
  __shared__ float Bs[GK][GT + 4];
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  long long wg = blockIdx.x;
  const int tiles = a.tiles_m * a.tiles_n;
  const long long z = wg / tiles;
  const int t = (int)(wg % tiles);
  const int m0 = (t / a.tiles_n) * GT, n0 = (t % a.tiles_n) * GT;
  if (a.skip_upper && n0 > m0 + GT - 1) return;
  const int z1 = (int)(z / a.nz0), z0 = (int)(z % a.nz0);
  const int bf = a.epi.in_bf16;
  const long long aoff = z1 * a.sA1 + z0 * a.sA0;
  const long long boff = z1 * a.sB1 + z0 * a.sB0;
  int k_lo = a.k_lo_diag ? m0 : 0;
  int k_hi = a.k_hi_diag ? min(a.Kp, m0 + GT) : a.Kp;
  float acc[4][4];
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[r][c] = 0.f;
  for (int l = 0; l < a.nl; ++l) {
    const long long ap = aoff + l * a.sAl, bp = boff + l * a.sBl;
    for (int k0 = k_lo; k0 < k_hi; k0 += GK) {
      // 64 x 16 elements per operand, 4 per thread
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        int e = tid + it * 256;
        int kk, rr;
        if (a.a_kcontig) { rr = e / GK; kk = e % GK; } else { kk = e / GT; rr = e % GT; }
        int m = m0 + rr, k = k0 + kk;
        float v = 0.f;
        if (m < a.Mb && k < k_hi)
          v = load_elem(a.A, ap + (a.a_kcontig ? (long long)m * a.lda + k : (long long)k * a.lda + m), bf);
        As[kk][rr] = v;
        if (a.b_kcontig) { rr = e / GK; kk = e % GK; } else { kk = e / GT; rr = e % GT; }
        int n = n0 + rr;
        k = k0 + kk;
        v = 0.f;
        if (n < a.Nb && k < k_hi)
          v = load_elem(a.B, bp + (a.b_kcontig ? (long long)n * a.ldb + k : (long long)k * a.ldb + n), bf);
        Bs[kk][rr] = v;
      }
      __syncthreads();
#pragma unroll
      for (int kk = 0; kk < GK; ++kk) {
        float av[4], bv[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) av[r] = As[kk][ty * 4 + r];
#pragma unroll
        for (int c = 0; c < 4; ++c) bv[c] = Bs[kk][tx * 4 + c];
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
          for (int c = 0; c < 4; ++c) acc[r][c] = fmaf(av[r], bv[c], acc[r][c]);
      }
      __syncthreads();
    }
  }
  EpiArgs e = a.epi;
  if (e.bias) e.bias += z0 * a.sBias0;
  const long long coff = z1 * a.sC1 + z0 * a.sC0;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    int m = m0 + ty * 4 + r, n = n0 + tx * 4;
    if (m >= a.Mb || n >= a.Nb) continue;
    epilogue_store4<false, true>(e, coff, m, n, acc[r], min(4, a.Nb - n));
  }
}

int launch_gemm_generic(const GemmDesc& d, hipStream_t stream) {
  GArgs a;
  a.A = d.A; a.B = d.B;
  a.Mb = d.Mb; a.Nb = d.Nb; a.Kp = d.Kp; a.nl = d.nl;
  a.lda = d.lda; a.ldb = d.ldb; a.sAl = d.sAl; a.sBl = d.sBl;
  a.nz0 = d.nz0;
  a.sA0 = d.sA0; a.sA1 = d.sA1; a.sB0 = d.sB0; a.sB1 = d.sB1; a.sC0 = d.sC0; a.sC1 = d.sC1; a.sBias0 = d.sBias0;
  a.a_kcontig = d.a_kcontig; a.b_kcontig = d.b_kcontig;
  a.tiles_m = (d.Mb + GT - 1) / GT;
  a.tiles_n = (d.Nb + GT - 1) / GT;
  a.skip_upper = d.skip_upper; a.k_hi_diag = d.k_hi_diag; a.k_lo_diag = d.k_lo_diag;
  EpiArgs& e = a.epi;
  e.alpha = d.alpha; e.bias = d.bias; e.C = d.C; e.pre_act = d.pre_act; e.gelu_grad_of = d.gelu_grad_of;
  e.residual = d.residual; e.ldc = d.ldc; e.act = d.act; e.out_fp32 = d.out_fp32;
  e.in_bf16 = d.dtype == OPTIMUS_BF16;
  e.vec_ok = 0;
  long long nwg = (long long)a.tiles_m * a.tiles_n * d.nz0 * d.nz1;
  if (nwg <= 0 || nwg > 0x7fffffffLL) return OPTIMUS_ESHAPE;
  hipLaunchKernelGGL(gemm_generic_kernel, dim3((unsigned)nwg), dim3(256), 0, stream, a);
  return hip_launch_status();
}

int launch_gemm(const GemmDesc& d, hipStream_t stream) {
  if (gemm_mfma_supported(d)) return launch_gemm_mfma(d, stream);
  GemmDesc g = d;
  g.splits = 1;
  return launch_gemm_generic(g, stream);
}

}  // namespace optimus

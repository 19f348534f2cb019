// 2D LayerNorm (Section 3.2.2 of the paper): a row of the hidden dimension is spread over the q devices of a
// grid row; each device sums x and x^2 over its own h/q columns, the q partials are added (the row
// all-reduce), and the device normalises its own block.  Backward treats (sum xhat*g, sum g) the same way.
//
// One wavefront owns one row of a block: the row (<= 2048 columns on the fast path) is read once with
// 16-byte loads, kept in registers, reduced with DPP-free shuffles, and written once.  Wider or unaligned
// rows take a scalar path that re-reads the row.  Statistics are fp32; partials are always added in the
// order l = 0..q-1 so that every device of a row, and grid and device mode, get identical bits.
#include "common.hpp"

namespace optimus {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

constexpr int LN_MAXCH = 4;  // 16-byte chunks per lane on the fast path (bf16: 8 elems, fp32: 4 elems)

template <typename T> struct Vec;
template <> struct Vec<bf16_t> {
  static constexpr int N = 8;
  __device__ static void load(const bf16_t* p, float* f) {
    uint4 w = *(const uint4*)p;
    unsigned u[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) { f[2 * k] = __uint_as_float(u[k] << 16); f[2 * k + 1] = __uint_as_float(u[k] & 0xffff0000u); }
  }
  __device__ static void store(bf16_t* p, const float* f) {
    *(uint4*)p = make_uint4(pack2_bf16(f[0], f[1]), pack2_bf16(f[2], f[3]), pack2_bf16(f[4], f[5]), pack2_bf16(f[6], f[7]));
  }
  __device__ static float ld1(const bf16_t* p) { return bf16_to_f32(*p); }
  __device__ static void st1(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};
template <> struct Vec<float> {
  static constexpr int N = 4;
  __device__ static void load(const float* p, float* f) { float4 w = *(const float4*)p; f[0] = w.x; f[1] = w.y; f[2] = w.z; f[3] = w.w; }
  __device__ static void store(float* p, const float* f) { *(float4*)p = make_float4(f[0], f[1], f[2], f[3]); }
  __device__ static float ld1(const float* p) { return *p; }
  __device__ static void st1(float* p, float v) { *p = v; }
};

struct LnArgs {
  int rows, cols, H, q;
  int i0, ni, j0, nj;
  float eps;
  int vec;  // fast path allowed
};

// MODE 0: forward stats only.  MODE 1: forward apply (own partial computed here unless own_ready).
// MODE 2: backward stats only. MODE 3: backward apply.
// RG ("row group", MODE 1 and 3, whole grid rows only): a workgroup holds the q wavefronts that own the q segments of
// the same logical row (times a few rows), each computes its partial, the partials meet in LDS, and every
// wavefront adds them in the order l = 0..q-1: the same numbers in the same order as the two-kernel form
// (statistics kernel, then apply with own_ready), in one pass over the input.  The partials are still written
// to `stats`, which device-mode calls of the peers read.
template <typename T, int MODE, bool RG = false>
__global__ __launch_bounds__(RG ? 1024 : 256) void ln_kernel(const T* __restrict__ X, const T* __restrict__ X2, const float* __restrict__ gamma,
                                                 const float* __restrict__ beta, const float* __restrict__ rstd_in,
                                                 const T* __restrict__ dres, T* __restrict__ Y, T* __restrict__ xhat_out,
                                                 float* __restrict__ rstd_out, float* __restrict__ stats, LnArgs a, int own_ready) {
  constexpr int VN = Vec<T>::N;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int dev = blockIdx.y;
  // RG: wavefront = (row of the workgroup, segment dj); the host launches whole workgroups only (no partial last one)
  const int di = RG ? a.i0 + dev : a.i0 + dev / a.nj;
  const int dj = RG ? wave % a.q : a.j0 + dev % a.nj;
  const int row = RG ? blockIdx.x * ((int)(blockDim.x >> 6) / a.q) + wave / a.q : blockIdx.x * 4 + wave;
  if (row >= a.rows) return;
  const long long blk = (long long)a.rows * a.cols;
  const long long base = ((long long)di * a.q + dj) * blk + (long long)row * a.cols;
  const T* x = X + base;                    // forward: x ; backward: dy
  const T* x2 = X2 ? X2 + base : nullptr;   // backward: xhat
  const float* gm = gamma ? gamma + (long long)dj * a.cols : nullptr;
  const float* bt = beta ? beta + (long long)dj * a.cols : nullptr;
  float* st_row = stats + ((long long)di * a.q * a.rows + row) * 2;  // + l*rows*2 selects device (di, l)
  const long long st_dev = (long long)a.rows * 2;

  float v[LN_MAXCH * VN];   // forward: x ; backward: g = dy*gamma
  float w[LN_MAXCH * VN];   // backward: xhat
  float s0 = 0.f, s1 = 0.f;
  const bool need_own = !(own_ready && (MODE == 1 || MODE == 3));
  if (a.vec) {
#pragma unroll
    for (int c = 0; c < LN_MAXCH; ++c) {
      int col = (c * 64 + lane) * VN;
      if (col < a.cols) {
        Vec<T>::load(x + col, v + c * VN);
        if (MODE >= 2) {
          Vec<T>::load(x2 + col, w + c * VN);
#pragma unroll
          for (int k = 0; k < VN; ++k) { v[c * VN + k] *= gm[col + k]; s0 += w[c * VN + k] * v[c * VN + k]; s1 += v[c * VN + k]; }
        } else {
#pragma unroll
          for (int k = 0; k < VN; ++k) { s0 += v[c * VN + k]; s1 += v[c * VN + k] * v[c * VN + k]; }
        }
      }
    }
  } else if (need_own) {
    for (int col = lane; col < a.cols; col += 64) {
      float t = Vec<T>::ld1(x + col);
      if (MODE >= 2) { float g = t * gm[col]; s0 += Vec<T>::ld1(x2 + col) * g; s1 += g; }
      else { s0 += t; s1 += t * t; }
    }
  }
  float own0 = 0.f, own1 = 0.f;
  if (need_own) {
    own0 = wave_sum(s0);
    own1 = wave_sum(s1);
    if (lane == 0) { st_row[dj * st_dev] = own0; st_row[dj * st_dev + 1] = own1; }
  }
  if (MODE == 0 || MODE == 2) return;

  // add the q partials of this grid row in fixed order (own partial from registers when computed here)
  float t0 = 0.f, t1 = 0.f;
  if constexpr (RG) {
    __shared__ float part[16][2];
    if (lane == 0) { part[wave][0] = own0; part[wave][1] = own1; }
    __syncthreads();
    const int w0 = wave - dj;  // first wavefront of this row
    for (int l = 0; l < a.q; ++l) { t0 += part[w0 + l][0]; t1 += part[w0 + l][1]; }
  } else {
    for (int l = 0; l < a.q; ++l) {
      float p0, p1;
      if (l == dj && need_own) { p0 = own0; p1 = own1; }
      else { p0 = st_row[l * st_dev]; p1 = st_row[l * st_dev + 1]; }
      t0 += p0; t1 += p1;
    }
  }
  const float invH = 1.0f / (float)a.H;
  if (MODE == 1) {
    float mean = t0 * invH;
    float var = fmaxf(t1 * invH - mean * mean, 0.f);
    float rstd = 1.0f / sqrtf(var + a.eps);
    if (lane == 0) rstd_out[((long long)di * a.q + dj) * a.rows + row] = rstd;
    T* y = Y + base;
    T* xh = xhat_out + base;
    if (a.vec) {
#pragma unroll
      for (int c = 0; c < LN_MAXCH; ++c) {
        int col = (c * 64 + lane) * VN;
        if (col < a.cols) {
          float o[VN], h[VN];
#pragma unroll
          for (int k = 0; k < VN; ++k) { h[k] = (v[c * VN + k] - mean) * rstd; o[k] = h[k] * gm[col + k] + bt[col + k]; }
          Vec<T>::store(xh + col, h);
          Vec<T>::store(y + col, o);
        }
      }
    } else {
      for (int col = lane; col < a.cols; col += 64) {
        float h = (Vec<T>::ld1(x + col) - mean) * rstd;
        Vec<T>::st1(xh + col, h);
        Vec<T>::st1(y + col, h * gm[col] + bt[col]);
      }
    }
  } else {  // MODE 3
    float rstd = rstd_in[((long long)di * a.q + dj) * a.rows + row];
    float mxg = t0 * invH, mg = t1 * invH;
    T* dx = Y + base;
    const T* dr = dres ? dres + base : nullptr;
    if (a.vec) {
#pragma unroll
      for (int c = 0; c < LN_MAXCH; ++c) {
        int col = (c * 64 + lane) * VN;
        if (col < a.cols) {
          float o[VN], r[VN];
          if (dr) Vec<T>::load(dr + col, r);
#pragma unroll
          for (int k = 0; k < VN; ++k) {
            o[k] = rstd * (v[c * VN + k] - w[c * VN + k] * mxg - mg);
            if (dr) o[k] += r[k];
          }
          Vec<T>::store(dx + col, o);
        }
      }
    } else {
      for (int col = lane; col < a.cols; col += 64) {
        float g = Vec<T>::ld1(x + col) * gm[col];
        float o = rstd * (g - Vec<T>::ld1(x2 + col) * mxg - mg);
        if (dr) o += Vec<T>::ld1(dr + col);
        Vec<T>::st1(dx + col, o);
      }
    }
  }
}

static LnArgs make_args(const LnDesc& d, bool ptr_ok, int elem_bytes) {
  LnArgs a;
  a.rows = d.rows; a.cols = d.cols; a.H = d.H; a.q = d.q;
  a.i0 = d.i0; a.ni = d.ni; a.j0 = d.j0; a.nj = d.nj;
  a.eps = d.eps;
  int vn = 16 / elem_bytes;
  a.vec = ptr_ok && (d.cols % vn == 0) && (d.cols <= LN_MAXCH * 64 * vn);
  return a;
}
static bool al16(const void* p) { return ((uintptr_t)p & 15) == 0; }

// rows of one workgroup of the row-group form: q wavefronts per row, four wavefronts or more per workgroup
static int ln_rowgroup_rows(const LnDesc& d) {
  int r = d.q >= 4 ? 1 : 4 / d.q;
  while (r > 1 && d.rows % r) r >>= 1;
  return r;
}
// the call covers whole grid rows (every segment of a logical row), and q wavefronts fit a workgroup
bool ln_rowgroup_ok(const LnDesc& d) { return d.j0 == 0 && d.nj == d.q && d.q >= 1 && d.q <= 16; }

template <typename T, int MODE>
static int run(const void* X, const void* X2, const float* gamma, const float* beta, const float* rstd_in, const void* dres,
               void* Y, void* xhat, float* rstd_out, float* stats, const LnDesc& d, bool own_ready, hipStream_t stream) {
  bool ok = al16(X) && (!X2 || al16(X2)) && (!dres || al16(dres)) && (!Y || al16(Y)) && (!xhat || al16(xhat)) &&
            (!gamma || al16(gamma)) && (!beta || al16(beta));
  LnArgs a = make_args(d, ok, (int)sizeof(T));
  if constexpr (MODE == 1 || MODE == 3) {
    if (!own_ready && ln_rowgroup_ok(d)) {
      const int rpw = ln_rowgroup_rows(d);
      dim3 grid((unsigned)(d.rows / rpw), (unsigned)d.ni);
      hipLaunchKernelGGL((ln_kernel<T, MODE, true>), grid, dim3(64 * d.q * rpw), 0, stream, (const T*)X, (const T*)X2, gamma, beta,
                         rstd_in, (const T*)dres, (T*)Y, (T*)xhat, rstd_out, stats, a, 0);
      return hip_launch_status();
    }
  }
  dim3 grid((unsigned)((d.rows + 3) / 4), (unsigned)(d.ni * d.nj));
  hipLaunchKernelGGL((ln_kernel<T, MODE>), grid, dim3(256), 0, stream, (const T*)X, (const T*)X2, gamma, beta, rstd_in,
                     (const T*)dres, (T*)Y, (T*)xhat, rstd_out, stats, a, own_ready ? 1 : 0);
  return hip_launch_status();
}

#define LN_DISPATCH(MODE, ...)                                              \
  (d.dtype == OPTIMUS_BF16 ? run<bf16_t, MODE>(__VA_ARGS__) : run<float, MODE>(__VA_ARGS__))

int launch_ln_stats(const void* X, float* stats, const LnDesc& d, hipStream_t stream) {
  return LN_DISPATCH(0, X, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, stats, d, false, stream);
}
int launch_ln_apply(const void* X, const float* gamma, const float* beta, void* Y, void* xhat, float* rstd, float* stats,
                    const LnDesc& d, bool own_ready, hipStream_t stream) {
  return LN_DISPATCH(1, X, nullptr, gamma, beta, nullptr, nullptr, Y, xhat, rstd, stats, d, own_ready, stream);
}
int launch_ln_bwd_stats(const void* dY, const void* xhat, const float* gamma, float* stats, const LnDesc& d, hipStream_t stream) {
  return LN_DISPATCH(2, dY, xhat, gamma, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, stats, d, false, stream);
}
int launch_ln_bwd_apply(const void* dY, const void* xhat, const float* rstd, const float* gamma, const void* dres, void* dX,
                        float* stats, const LnDesc& d, bool own_ready, hipStream_t stream) {
  return LN_DISPATCH(3, dY, xhat, gamma, nullptr, rstd, dres, dX, nullptr, nullptr, stats, d, own_ready, stream);
}

// ---- column sums over the rows of a block: dgamma/dbeta partials, bias gradients ----
// Workgroup = 1024 threads = (1024 / CL) row lanes x CL column lanes covering CS_COLS = 8 * CL columns; each thread
// accumulates 8 adjacent columns (one 16-byte load per row for bf16) over rows ty, ty + 1024 / CL, ...  The row lanes
// inside a wavefront are added by butterfly exchanges, the 16 wavefronts through LDS, both in a fixed order (the
// result does not depend on the launch).  Narrow column strips and many row lanes keep the chain of dependent
// loads short: the matrices here have thousands of rows and only a few hundred columns per block.
constexpr int CS_THREADS = 1024;
// CS_COLS = 64: whole 128-byte lines per row (large blocks, bandwidth matters).  CS_COLS = 32: twice the workgroups
// and half the rows per lane (small blocks, where the kernel is two dependent memory round trips long).
template <typename T, bool PROD, int CS_COLS>
__global__ __launch_bounds__(CS_THREADS) void colsum_kernel(const T* __restrict__ X, const T* __restrict__ W, float* __restrict__ out,
                                                            float* __restrict__ out2, int rows, int cols, int ld, long long sX,
                                                            long long sOut) {
  constexpr int CS_CL = CS_COLS / 8;  // column lanes
  __shared__ float red[16][CS_COLS];
  __shared__ float red2[16][CS_COLS];
  const int tx = threadIdx.x & (CS_CL - 1), ty = threadIdx.x / CS_CL;
  const int wave = threadIdx.x >> 6;
  const int c0 = blockIdx.x * CS_COLS + tx * 8;
  const long long zoff = (long long)blockIdx.y * sX;
  float acc[8], acc2[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) { acc[k] = 0.f; acc2[k] = 0.f; }
  const bool vec = (ld % 8 == 0) && (sX % 8 == 0) && (c0 + 8 <= cols) && sizeof(T) == 2 && (((uintptr_t)X & 15) == 0) &&
                   (!PROD || ((uintptr_t)W & 15) == 0);
#pragma unroll 4
  for (int r = ty; r < rows; r += CS_THREADS / CS_CL) {
    const long long off = zoff + (long long)r * ld + c0;
    float x[8], w[8];
    if (vec) {
      Vec<bf16_t>::load((const bf16_t*)X + off, x);
      if (PROD) Vec<bf16_t>::load((const bf16_t*)W + off, w);
    } else {
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        bool in = c0 + k < cols;
        x[k] = in ? Vec<T>::ld1(X + off + k) : 0.f;
        if (PROD) w[k] = in ? Vec<T>::ld1(W + off + k) : 0.f;
      }
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      acc[k] += x[k];                      // sum x           (dbeta / bias gradient)
      if (PROD) acc2[k] += x[k] * w[k];    // sum x*w         (dgamma)
    }
  }
  // the row lanes of a wavefront: lanes that differ in the bits above the column-lane bits
#pragma unroll
  for (int d = CS_CL; d < 64; d <<= 1) {
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      acc[k] += __shfl_xor(acc[k], d, 64);
      if (PROD) acc2[k] += __shfl_xor(acc2[k], d, 64);
    }
  }
  if ((threadIdx.x & 63) < CS_CL) {
#pragma unroll
    for (int k = 0; k < 8; ++k) { red[wave][tx * 8 + k] = acc[k]; if (PROD) red2[wave][tx * 8 + k] = acc2[k]; }
  }
  __syncthreads();
  if (threadIdx.x < CS_COLS) {
    int c = blockIdx.x * CS_COLS + threadIdx.x;
    if (c < cols) {
      float s = 0.f, s2 = 0.f;
      for (int r = 0; r < 16; ++r) { s += red[r][threadIdx.x]; if (PROD) s2 += red2[r][threadIdx.x]; }
      out[(long long)blockIdx.y * sOut + c] = s;
      if (PROD) out2[(long long)blockIdx.y * sOut + c] = s2;
    }
  }
}

// strip width from the block shape only (never from the batch): grid mode and device mode then add in the same order
bool colsum_narrow(int rows, int cols) { return (long long)rows * cols <= (1LL << 20); }

template <typename T, bool PROD>
static void colsum_launch(dim3 batch, const T* X, const T* W, float* out, float* out2, int rows, int cols, int ld, long long sX,
                          long long sOut, hipStream_t stream) {
  if (colsum_narrow(rows, cols)) {
    dim3 grid((unsigned)((cols + 31) / 32), batch.y);
    hipLaunchKernelGGL((colsum_kernel<T, PROD, 32>), grid, dim3(CS_THREADS), 0, stream, X, W, out, out2, rows, cols, ld, sX, sOut);
  } else {
    dim3 grid((unsigned)((cols + 63) / 64), batch.y);
    hipLaunchKernelGGL((colsum_kernel<T, PROD, 64>), grid, dim3(CS_THREADS), 0, stream, X, W, out, out2, rows, cols, ld, sX, sOut);
  }
}

int launch_colsum(const void* X, float* out, int rows, int cols, int ld, int nz, long long sX, long long sOut, int dtype,
                  hipStream_t stream) {
  dim3 batch(1, (unsigned)nz);
  if (dtype == OPTIMUS_BF16)
    colsum_launch<bf16_t, false>(batch, (const bf16_t*)X, (const bf16_t*)nullptr, out, (float*)nullptr, rows, cols, ld, sX, sOut, stream);
  else
    colsum_launch<float, false>(batch, (const float*)X, (const float*)nullptr, out, (float*)nullptr, rows, cols, ld, sX, sOut, stream);
  return hip_launch_status();
}

// dbeta_part = column sums of dy, dgamma_part = column sums of dy*xhat, for the blocks (i0.., j0..) of d
int launch_ln_param_grads(const void* dY, const void* xhat, float* dgamma_part, float* dbeta_part, const LnDesc& d,
                          hipStream_t stream) {
  const long long blk = (long long)d.rows * d.cols;
  int rc = OPTIMUS_OK;
  // block-major storage: the nj blocks of one grid row are contiguous, and so are whole grid rows that follow each other
  const bool whole_rows = d.nj == d.q;
  const int launches = whole_rows ? 1 : d.ni, per_launch = whole_rows ? d.ni * d.nj : d.nj;
  for (int ii = 0; ii < launches && rc == OPTIMUS_OK; ++ii) {
    const long long first = ((long long)(d.i0 + ii) * d.q + d.j0);
    dim3 batch(1, (unsigned)per_launch);
    if (d.dtype == OPTIMUS_BF16)
      colsum_launch<bf16_t, true>(batch, (const bf16_t*)dY + first * blk, (const bf16_t*)xhat + first * blk, dbeta_part + first * d.cols,
                                  dgamma_part + first * d.cols, d.rows, d.cols, d.cols, blk, (long long)d.cols, stream);
    else
      colsum_launch<float, true>(batch, (const float*)dY + first * blk, (const float*)xhat + first * blk, dbeta_part + first * d.cols,
                                 dgamma_part + first * d.cols, d.rows, d.cols, d.cols, blk, (long long)d.cols, stream);
    rc = hip_launch_status();
  }
  return rc;
}

}  // namespace optimus

// The two ends of the model around the layer stack in the 2D partition (Sections 3.2.1 / 3.2.2 of the paper):
//   * embedding: the paper's "one-hot matrix times embedding table" product is a row gather.  Device (i, j) holds the
//     token indices of grid row i (every device of a row has them) and the table block (l, j) of every l is resident:
//     out_ij[t] = table block (tok / (v/q), j), row tok % (v/q).  Pure copy: bit exact, HBM bound.
//   * embedding gradient: d_table_lj = sum_i one_hot_il^T dX_ij, the A^T B form reduced within column j onto its owner
//     (l, j).  Computed as the owner sees it: a workgroup owns 32 table rows x 256 columns of the block as fp32
//     accumulators in LDS, scans ALL token indices, adds the rows of dX whose token falls into its rows and writes
//     its piece once.  No atomics, an order of additions fixed by the token order: deterministic, and rows that no
//     token refers to are written as zeros.
//   * cross entropy H = log(sum_i exp(x_i)) - x_label over a logits row that spans the q devices of a grid row: each
//     device reduces its v/q columns to (max, sum exp(x - max)) -- the maximum is subtracted for range, which does
//     not change the value --, the q partials are combined in the order l = 0..q-1 (the row all-reduce), and the
//     device computes the loss and keeps L = log sum exp per row.  Backward: q_j - [j = label] with
//     q_j = exp(x_j - L) recomputed from the saved L (the paper saves the soft-max itself: v/2 times the bytes).
// The lm-head logits are the C = A B^T product of the hidden states with the table: optimus_summa_abt.
#include "common.hpp"

namespace optimus {
namespace {

__device__ __forceinline__ float wave_sum_f(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ float wave_max_f(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}
template <typename T> __device__ __forceinline__ float ldf(const T* p);
template <> __device__ __forceinline__ float ldf<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }
template <> __device__ __forceinline__ float ldf<float>(const float* p) { return *p; }
template <typename T> __device__ __forceinline__ void stf(T* p, float v);
template <> __device__ __forceinline__ void stf<bf16_t>(bf16_t* p, float v) { *p = f32_to_bf16(v); }
template <> __device__ __forceinline__ void stf<float>(float* p, float v) { *p = v; }

__device__ __forceinline__ int clamp_token(int t, int v) { return min(max(t, 0), v - 1); }

// 16 bytes of a row as floats (8 bf16 or 4 fp32) and back
template <typename T> struct V16;
template <> struct V16<bf16_t> {
  static constexpr int N = 8;
  __device__ static void load(const bf16_t* p, float* f) {
    const uint4 w = *(const uint4*)p;
    const unsigned u[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) { f[2 * k] = __uint_as_float(u[k] << 16); f[2 * k + 1] = __uint_as_float(u[k] & 0xffff0000u); }
  }
  __device__ static void store(bf16_t* p, const float* f) {
    *(uint4*)p = make_uint4(pack2_bf16(f[0], f[1]), pack2_bf16(f[2], f[3]), pack2_bf16(f[4], f[5]), pack2_bf16(f[6], f[7]));
  }
};
template <> struct V16<float> {
  static constexpr int N = 4;
  __device__ static void load(const float* p, float* f) { const float4 w = *(const float4*)p; f[0] = w.x; f[1] = w.y; f[2] = w.z; f[3] = w.w; }
  __device__ static void store(float* p, const float* f) { *(float4*)p = make_float4(f[0], f[1], f[2], f[3]); }
};

struct EndArgs {
  int rows;        // M/q: rows of a block
  int vb, hb;      // v/q, h/q
  int q, v;
  int i0, ni, j0, nj;  // devices handled: grid rows i0.., grid columns j0..
};

// ---- embedding forward: one wavefront per output row; 16-byte copies when the block width allows ----
template <typename T>
__global__ __launch_bounds__(256) void embedding_fwd_kernel(const int* __restrict__ tokens, const T* __restrict__ table,
                                                            T* __restrict__ out, EndArgs a) {
  const int lane = threadIdx.x & 63;
  const long long r = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= a.rows) return;
  const int dev = blockIdx.y;
  const int i = a.i0 + dev / a.nj, j = a.j0 + dev % a.nj;
  const int tok = clamp_token(tokens[(long long)i * a.rows + r], a.v);
  const int l = tok / a.vb, tr = tok % a.vb;
  const T* src = table + (((long long)l * a.q + j) * a.vb + tr) * a.hb;
  T* dst = out + (((long long)i * a.q + j) * a.rows + r) * a.hb;
  constexpr int VN = 16 / sizeof(T);
  if (a.hb % VN == 0) {
    for (int c = lane * VN; c < a.hb; c += 64 * VN) *(uint4*)(dst + c) = *(const uint4*)(src + c);
  } else {
    for (int c = lane; c < a.hb; c += 64) dst[c] = src[c];
  }
}

// ---- embedding backward (owner view): workgroup = EB_ROWS table rows x EB_COLS columns of block (l, j) ----
// Token indices are scanned in chunks; the positions of a chunk that fall into the workgroup's rows are compacted, in
// order, into a list (ballot + prefix counts), which is cut into four consecutive quarters, one per wavefront.  A
// wavefront adds its quarter's rows of dX into its OWN fp32 accumulator copy in LDS, a batch of loads in flight at a
// time (a lane covers four adjacent columns); the four copies are added in wavefront order at the end.  The order of
// all additions is a function of the token order alone, so the result is reproducible bit for bit.
constexpr int EB_ROWS = 32, EB_COLS = 256, EB_CHUNK = 1024, EB_BATCH = 16;
template <typename T>
__global__ __launch_bounds__(256) void embedding_bwd_kernel(const int* __restrict__ tokens, const T* __restrict__ dX,
                                                            float* __restrict__ d_table, EndArgs a) {
  __shared__ float acc[4][EB_ROWS * EB_COLS];   // one copy per wavefront
  __shared__ int list[EB_CHUNK];                // (position in chunk) << 8 | row inside the workgroup's range
  __shared__ int wave_count[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int dev = blockIdx.z;
  const int l = a.i0 + dev / a.nj, j = a.j0 + dev % a.nj;
  const int r0 = blockIdx.y * EB_ROWS;                  // first table row (inside block l) of this workgroup
  const int nr = min(EB_ROWS, a.vb - r0);
  const int c0 = blockIdx.x * EB_COLS + 4 * lane;       // first of this lane's four columns inside the block
  const bool vec4 = a.hb % 4 == 0 && c0 + 3 < a.hb;     // this lane's four columns exist and are 8/16-byte aligned
  for (int k = tid; k < 4 * EB_ROWS * EB_COLS; k += 256) (&acc[0][0])[k] = 0.f;
  const int lo = l * a.vb + r0, hi = lo + nr;           // token indices that land in this workgroup's rows
  const long long total = (long long)a.q * a.rows;      // all tokens, grid row after grid row (below 2^31: host check)
  for (long long base = 0; base < total; base += EB_CHUNK) {
    // this wavefront's quarter of the chunk: 4 rounds of 64 tokens, compacted in order
    int mine[4], cnt = 0;
    unsigned long long ball[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const long long t = base + wave * 256 + r * 64 + lane;
      const int tok = t < total ? clamp_token(tokens[t], a.v) : -1;
      const bool hit = tok >= lo && tok < hi;
      mine[r] = hit ? (((wave * 256 + r * 64 + lane) << 8) | (tok - lo)) : -1;
      ball[r] = __builtin_amdgcn_ballot_w64(hit);
      cnt += __builtin_popcountll(ball[r]);
    }
    __syncthreads();                                    // the previous chunk's list has been consumed
    if (lane == 0) wave_count[wave] = cnt;
    __syncthreads();
    int off = 0, n = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      if (w < wave) off += wave_count[w];
      n += wave_count[w];
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      if (mine[r] >= 0) list[off + __builtin_popcountll(ball[r] & ((1ull << lane) - 1ull))] = mine[r];
      off += __builtin_popcountll(ball[r]);
    }
    __syncthreads();
    // quarter `wave` of the list, EB_BATCH rows of dX in flight.  The last batch is padded with its last entry at
    // weight zero, so that the loop body has no branches between its loads.
    const int q0 = (int)((long long)n * wave / 4), q1 = (int)((long long)n * (wave + 1) / 4);
    float* my = acc[wave];
    for (int m0 = q0; m0 < q1; m0 += EB_BATCH) {
      float v[EB_BATCH][4];
      int row[EB_BATCH];
#pragma unroll
      for (int u = 0; u < EB_BATCH; ++u) {
        const int e = list[min(m0 + u, q1 - 1)];
        const float wgt = m0 + u < q1 ? 1.0f : 0.0f;
        row[u] = e & 255;
        const unsigned t = (unsigned)base + (unsigned)(e >> 8);
        const unsigned i = t / (unsigned)a.rows, rr = t - i * (unsigned)a.rows;
        const T* src = dX + (((long long)i * a.q + j) * a.rows + rr) * a.hb + c0;
        if (vec4) {
          if (sizeof(T) == 2) {
            const uint2 w = *(const uint2*)src;
            v[u][0] = __uint_as_float(w.x << 16) * wgt; v[u][1] = __uint_as_float(w.x & 0xffff0000u) * wgt;
            v[u][2] = __uint_as_float(w.y << 16) * wgt; v[u][3] = __uint_as_float(w.y & 0xffff0000u) * wgt;
          } else {
            const float4 w = *(const float4*)src;
            v[u][0] = w.x * wgt; v[u][1] = w.y * wgt; v[u][2] = w.z * wgt; v[u][3] = w.w * wgt;
          }
        } else {
#pragma unroll
          for (int k = 0; k < 4; ++k) v[u][k] = c0 + k < a.hb ? ldf<T>(src + k) * wgt : 0.f;
        }
      }
#pragma unroll
      for (int u = 0; u < EB_BATCH; ++u) {
        float4* p = (float4*)(my + row[u] * EB_COLS + 4 * lane);
        float4 w = *p;
        w.x += v[u][0]; w.y += v[u][1]; w.z += v[u][2]; w.w += v[u][3];
        *p = w;
      }
    }
  }
  __syncthreads();
  for (int k = tid; k < nr * EB_COLS; k += 256) {
    const int r = k / EB_COLS, c = blockIdx.x * EB_COLS + k % EB_COLS;
    if (c < a.hb)
      d_table[(((long long)l * a.q + j) * a.vb + r0 + r) * a.hb + c] = ((acc[0][k] + acc[1][k]) + acc[2][k]) + acc[3][k];
  }
}

// ---- cross entropy ----
// Loss and log-sum-exp of row r of device (i, j) from the q partials of grid row i, combined in the order l = 0..q-1.
// own_l >= 0: that partial is taken from (own_m, own_s) instead of memory (same values: it has just been computed).
template <typename T>
__device__ __forceinline__ void ce_combine(const T* __restrict__ logits, const int* __restrict__ labels, const float* __restrict__ stats,
                                           float* __restrict__ loss, float* __restrict__ lse, const EndArgs& a, int i, int j,
                                           long long r, int own_l, float own_m, float own_s) {
  float m = -INFINITY;
  for (int l = 0; l < a.q; ++l) m = fmaxf(m, l == own_l ? own_m : stats[(((long long)i * a.q + l) * a.rows + r) * 2]);
  float s = 0.f;
  for (int l = 0; l < a.q; ++l) {
    const float* p = stats + (((long long)i * a.q + l) * a.rows + r) * 2;
    const float ml = l == own_l ? own_m : p[0], sl = l == own_l ? own_s : p[1];
    s += sl * __expf(ml - m);
  }
  const float L = m + __logf(s);
  const int lab = clamp_token(labels[(long long)i * a.rows + r], a.v);
  const float xl = ldf<T>(logits + ((((long long)i * a.q + lab / a.vb) * a.rows + r) * a.vb + lab % a.vb));
  const long long o = ((long long)i * a.q + j) * a.rows + r;
  lse[o] = L;
  loss[o] = L - xl;
}

// partial statistics of one block: (max, sum exp(x - max)) per row; one wavefront per row.  FINAL: the peers'
// partials are already in memory (one device recomputed from resident peers), so the row is finished here.
// WIDE: a whole workgroup per row (its four wavefronts take interleaved 16-byte chunks and their partials are
// combined in wavefront order through LDS): long rows need more loads in flight than one wavefront per SIMD gives.
template <typename T, bool FINAL, bool WIDE>
__global__ __launch_bounds__(256) void ce_stats_kernel(const T* __restrict__ logits, float* __restrict__ stats,
                                                       const int* __restrict__ labels, float* __restrict__ loss,
                                                       float* __restrict__ lse, EndArgs a) {
  __shared__ float part[8];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const long long r = WIDE ? (long long)blockIdx.x : (long long)blockIdx.x * 4 + wave;
  if (r >= a.rows) return;   // (WIDE: the same for the whole workgroup)
  const int first = WIDE ? wave * 64 + lane : lane, step = WIDE ? 256 : 64;
  const int dev = blockIdx.y;
  const int i = a.i0 + dev / a.nj, j = a.j0 + dev % a.nj;
  const long long blk = (long long)i * a.q + j;
  const T* src = logits + (blk * a.rows + r) * a.vb;
  float m = -INFINITY, s = 0.f;
  constexpr int VN = V16<T>::N;
  if (a.vb % VN == 0) {   // 16-byte loads: a chunk's maximum first, then one rescale per chunk
    for (int c = first * VN; c < a.vb; c += step * VN) {
      float f[VN];
      V16<T>::load(src + c, f);
      float cm = f[0];
#pragma unroll
      for (int k = 1; k < VN; ++k) cm = fmaxf(cm, f[k]);
      if (cm > m) { s *= __expf(m - cm); m = cm; }            // exp(-inf - x) = 0 on the first chunk (s is 0 then)
      if (m > -INFINITY) {
#pragma unroll
        for (int k = 0; k < VN; ++k) s += __expf(f[k] - m);
      }
    }
  } else {
    for (int c = first; c < a.vb; c += step) {
      const float x = ldf<T>(src + c);
      if (x > m) { s = s * __expf(m - x) + 1.0f; m = x; }
      else if (m > -INFINITY) s += __expf(x - m);             // (a row of -inf entries contributes nothing)
    }
  }
  float mw = wave_max_f(m);
  s = wave_sum_f(m == -INFINITY ? 0.f : s * __expf(m - mw));
  if (WIDE) {
    if (lane == 0) { part[wave] = mw; part[4 + wave] = s; }
    __syncthreads();
    if (wave != 0) return;
    mw = fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
    s = 0.f;
    for (int w = 0; w < 4; ++w) s += part[w] == -INFINITY ? 0.f : part[4 + w] * __expf(part[w] - mw);
  }
  if (lane == 0) {
    stats[(blk * a.rows + r) * 2] = mw;
    stats[(blk * a.rows + r) * 2 + 1] = s;
    if (FINAL) ce_combine<T>(logits, labels, stats, loss, lse, a, i, j, r, j, mw, s);
  }
}

// combine the q partials of a grid row in the order l = 0..q-1; loss and log-sum-exp per row of device (i, j)
template <typename T>
__global__ __launch_bounds__(256) void ce_finalize_kernel(const T* __restrict__ logits, const int* __restrict__ labels,
                                                          const float* __restrict__ stats, float* __restrict__ loss,
                                                          float* __restrict__ lse, EndArgs a) {
  const long long r = (long long)blockIdx.x * 256 + threadIdx.x;
  if (r >= a.rows) return;
  const int dev = blockIdx.y;
  const int i = a.i0 + dev / a.nj, j = a.j0 + dev % a.nj;
  ce_combine<T>(logits, labels, stats, loss, lse, a, i, j, r, -1, 0.f, 0.f);
}

// d_logits = scale * (exp(x - L) - [column == label]); one wavefront per row of a block
template <typename T>
__global__ __launch_bounds__(256) void ce_bwd_kernel(const T* __restrict__ logits, const int* __restrict__ labels,
                                                     const float* __restrict__ lse, T* __restrict__ d_logits, float scale, EndArgs a) {
  const int lane = threadIdx.x & 63;
  const long long r = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= a.rows) return;
  const int dev = blockIdx.y;
  const int i = a.i0 + dev / a.nj, j = a.j0 + dev % a.nj;
  const long long blk = (long long)i * a.q + j;
  const T* src = logits + (blk * a.rows + r) * a.vb;
  T* dst = d_logits + (blk * a.rows + r) * a.vb;
  const float L = lse[blk * a.rows + r];
  const int lab = clamp_token(labels[(long long)i * a.rows + r], a.v) - j * a.vb;   // label column inside this block, if any
  constexpr int VN = V16<T>::N;
  if (a.vb % VN == 0) {
    for (int c = lane * VN; c < a.vb; c += 64 * VN) {
      float f[VN];
      V16<T>::load(src + c, f);
#pragma unroll
      for (int k = 0; k < VN; ++k) f[k] = scale * (__expf(f[k] - L) - (c + k == lab ? 1.0f : 0.0f));
      V16<T>::store(dst + c, f);
    }
  } else {
    for (int c = lane; c < a.vb; c += 64) {
      const float qv = __expf(ldf<T>(src + c) - L);
      stf<T>(dst + c, scale * (qv - (c == lab ? 1.0f : 0.0f)));
    }
  }
}

}  // namespace

namespace {
template <bool FINAL>
int ce_stats_dispatch(const void* logits, float* stats, const int* labels, float* loss, float* lse, const EndDesc& d,
                      const EndArgs& a, hipStream_t st) {
  const bool wide = d.vb >= 2048;   // a workgroup per row from 2048 columns per block on
  const dim3 grid(wide ? d.rows : (d.rows + 3) / 4, d.ni * d.nj);
  if (d.dtype == OPTIMUS_BF16) {
    if (wide) ce_stats_kernel<bf16_t, FINAL, true><<<grid, 256, 0, st>>>((const bf16_t*)logits, stats, labels, loss, lse, a);
    else ce_stats_kernel<bf16_t, FINAL, false><<<grid, 256, 0, st>>>((const bf16_t*)logits, stats, labels, loss, lse, a);
  } else {
    if (wide) ce_stats_kernel<float, FINAL, true><<<grid, 256, 0, st>>>((const float*)logits, stats, labels, loss, lse, a);
    else ce_stats_kernel<float, FINAL, false><<<grid, 256, 0, st>>>((const float*)logits, stats, labels, loss, lse, a);
  }
  return hip_launch_status();
}
}  // namespace

int launch_embedding_fwd(const int* tokens, const void* table, void* out, const EndDesc& d, hipStream_t st) {
  EndArgs a = {d.rows, d.vb, d.hb, d.q, d.v, d.i0, d.ni, d.j0, d.nj};
  const dim3 grid((d.rows + 3) / 4, d.ni * d.nj);
  if (d.dtype == OPTIMUS_BF16) embedding_fwd_kernel<bf16_t><<<grid, 256, 0, st>>>(tokens, (const bf16_t*)table, (bf16_t*)out, a);
  else embedding_fwd_kernel<float><<<grid, 256, 0, st>>>(tokens, (const float*)table, (float*)out, a);
  return hip_launch_status();
}
int launch_embedding_bwd(const int* tokens, const void* dX, float* d_table, const EndDesc& d, hipStream_t st) {
  EndArgs a = {d.rows, d.vb, d.hb, d.q, d.v, d.i0, d.ni, d.j0, d.nj};
  const dim3 grid((d.hb + EB_COLS - 1) / EB_COLS, (d.vb + EB_ROWS - 1) / EB_ROWS, d.ni * d.nj);
  if (grid.y > 65535 || grid.z > 65535) return OPTIMUS_ESHAPE;
  if (d.dtype == OPTIMUS_BF16) embedding_bwd_kernel<bf16_t><<<grid, 256, 0, st>>>(tokens, (const bf16_t*)dX, d_table, a);
  else embedding_bwd_kernel<float><<<grid, 256, 0, st>>>(tokens, (const float*)dX, d_table, a);
  return hip_launch_status();
}
int launch_ce_stats(const void* logits, float* stats, const EndDesc& d, hipStream_t st) {
  EndArgs a = {d.rows, d.vb, d.hb, d.q, d.v, d.i0, d.ni, d.j0, d.nj};
  return ce_stats_dispatch<false>(logits, stats, nullptr, nullptr, nullptr, d, a, st);
}
// one device whose peers' partials are resident: statistics and finish in one launch
int launch_ce_stats_final(const void* logits, const int* labels, float* stats, float* loss, float* lse, const EndDesc& d,
                          hipStream_t st) {
  EndArgs a = {d.rows, d.vb, d.hb, d.q, d.v, d.i0, d.ni, d.j0, d.nj};
  return ce_stats_dispatch<true>(logits, stats, labels, loss, lse, d, a, st);
}
int launch_ce_finalize(const void* logits, const int* labels, const float* stats, float* loss, float* lse, const EndDesc& d,
                       hipStream_t st) {
  EndArgs a = {d.rows, d.vb, d.hb, d.q, d.v, d.i0, d.ni, d.j0, d.nj};
  const dim3 grid((d.rows + 255) / 256, d.ni * d.nj);
  if (d.dtype == OPTIMUS_BF16) ce_finalize_kernel<bf16_t><<<grid, 256, 0, st>>>((const bf16_t*)logits, labels, stats, loss, lse, a);
  else ce_finalize_kernel<float><<<grid, 256, 0, st>>>((const float*)logits, labels, stats, loss, lse, a);
  return hip_launch_status();
}
int launch_ce_bwd(const void* logits, const int* labels, const float* lse, void* d_logits, float scale, const EndDesc& d,
                  hipStream_t st) {
  EndArgs a = {d.rows, d.vb, d.hb, d.q, d.v, d.i0, d.ni, d.j0, d.nj};
  const dim3 grid((d.rows + 3) / 4, d.ni * d.nj);
  if (d.dtype == OPTIMUS_BF16)
    ce_bwd_kernel<bf16_t><<<grid, 256, 0, st>>>((const bf16_t*)logits, labels, lse, (bf16_t*)d_logits, scale, a);
  else ce_bwd_kernel<float><<<grid, 256, 0, st>>>((const float*)logits, labels, lse, (float*)d_logits, scale, a);
  return hip_launch_status();
}

}  // namespace optimus

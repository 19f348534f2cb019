// Fused local attention for gfx950 (CDNA4): O = softmax(Q K^T / sqrt(d)) V for every local (sequence, head) of a
// device without the [b/q, n/q, s, s] score and probability tensors ever reaching memory -- the operator fusion the
// paper's conclusion proposes as future work for its sequence-length limit (Section 6; the attention itself is that
// of Sections 2.1 / 3.2.1: whole sequences and n/q heads are local to a device, so no row is split).
//
// Forward keeps one fp32 number per query row, L = log sum_u exp(S_tu); backward rebuilds P = exp(S - L) tile by tile
// and uses rowsum(dO * O) in place of rowsum(dP * P).
//
// Layout of the work (all three kernels): one wavefront owns 32 rows (queries in the forward and dQ kernels, keys in
// the dK/dV kernel) for the whole loop over blocks of the other index; two or four wavefronts share the blocks of the other
// operands through LDS (double buffered, one barrier per block).  Every product is v_mfma_f32_32x32x16_bf16 with
// the operand that carries the wavefront's own rows in the B slot, so that a lane's 16 accumulator values of a 32x32
// tile all belong to ONE of its rows (lane % 32) and the other 16 live in lane ^ 32: row maxima and sums are 16
// in-lane operations plus one exchange.  The accumulator of S^T (or of S in the dK/dV kernel) is already laid out as
// the B operand of the next product up to a fixed permutation of the contraction index: accumulator slot r of lane
// group g = lane / 32 is row 8*(r/4) + 4*g + r%4 of the tile, a 16-wide contraction step takes slots 8u..8u+7, i.e.
// rows {16u + 4g + 0..3, 16u + 8 + 4g + 0..3}.  A contraction may visit its index in any order as long as both
// operands agree, so the A operand (V, K, dO or Q read "down the columns" with the transposing LDS read
// ds_read_b64_tr_b16) is simply fetched in that order.  P and dS therefore never leave registers.
//
// LDS tiles: [rows][D] bf16, once with 16-byte chunks XOR-swizzled by the row (read along rows with ds_read_b128),
// once with 32-byte column granules XOR 2*(row & 3) (read down the columns with the transposing read); both are
// conflict free on the 64-bank LDS of this part.
#include "common.hpp"

namespace optimus {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

constexpr float LOG2E = 1.44269504088896340736f;
constexpr float LN2 = 0.69314718055994530942f;

struct FusedArgs {
  const bf16_t* qkv;     // first device block of the launch
  bf16_t* attn;          // forward: output; backward: the forward's output (read only)
  float* lse;            // [device][matrix][s]
  const bf16_t* d_attn;
  bf16_t* d_qkv;
  float* delta;          // [device][matrix][s]: rowsum(dO * O), written by the dQ kernel, read by the dK/dV kernel
  int s, nh, ld, ldo;    // ld = 3h/q (row length of a qkv block), ldo = h/q
  long long dev_qkv, dev_attn, dev_vec;  // element strides between the devices of one launch
  float scale, scale_log2;               // 1/sqrt(d), log2(e)/sqrt(d)
};

// [rows][D] tile read along the rows: 16-byte chunk index XOR a function of the row that takes 16 values (8 for
// 128-byte rows, which pair up to span the banks) over 16 consecutive rows.
template <int D>
__device__ __forceinline__ int off_kc(int row, int chunk) {
  constexpr int CH = D / 8;
  const int swz = CH >= 16 ? (row & 15) : ((row / (16 / CH)) & (CH - 1));
  return row * D + ((chunk ^ swz) << 3);
}
// [rows][D] tile read down the columns with the transposing read: 32-byte granule XOR 2*(row & 3).
template <int D>
__device__ __forceinline__ int off_ks(int row, int col) {
  return row * D + ((((col >> 4) ^ (((row & 3) << 1) & (D / 16 - 1)))) << 4) + (col & 15);
}

// A-operand fragment along the rows: lane holds row (row0 + lane%32), contraction elements 16*ks + 8*(lane/32) + 0..7.
template <int D>
__device__ __forceinline__ bf16x8 frag_rows(const bf16_t* tile, int row0, int ks, int lane) {
  return *(const bf16x8*)(tile + off_kc<D>(row0 + (lane & 31), ks * 2 + (lane >> 5)));
}
// A-operand fragment down the columns in accumulator order: lane holds column (col0 + lane%32) and the tile rows
// row0 + 4g + {0..3} and row0 + 8 + 4g + {0..3}, g = lane/32 (row0 a multiple of 16).
template <int D>
__device__ __forceinline__ bf16x8 frag_cols_acc_order(const bf16_t* tile, int row0, int col0, int lane) {
  const int lg = lane & 15;
  const int col = col0 + (((lane >> 4) & 1) << 4) + ((lg & 3) << 2);
  const int row = row0 + ((lane >> 5) << 2) + (lg >> 2);
  const bf16_t* p0 = tile + off_ks<D>(row, col);
  const bf16_t* p1 = p0 + 8 * D;  // row + 8: same (row & 3), same swizzle term
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p0);
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p1);
  s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

// accumulator slots 8u .. 8u+7 as a bf16 B-operand fragment
template <int U>
__device__ __forceinline__ bf16x8 pack_acc(const f32x16& v) {
  u32x4 w = {pack2_bf16(v[8 * U + 0], v[8 * U + 1]), pack2_bf16(v[8 * U + 2], v[8 * U + 3]),
             pack2_bf16(v[8 * U + 4], v[8 * U + 5]), pack2_bf16(v[8 * U + 6], v[8 * U + 7])};
  return __builtin_bit_cast(bf16x8, w);
}

__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int r = 0; r < 16; ++r) z[r] = 0.f;
  return z;
}

// Cooperative copy of a [ROWS][D] bf16 tile (rows row0.. of a matrix with leading dimension ld, clamped to the last
// valid row) global -> registers, and registers -> LDS in one or both layouts, by a workgroup of THREADS threads.
template <int ROWS, int D, int THREADS>
struct TileCopy {
  static constexpr int CH = D / 8, PER = ROWS * CH / THREADS;
  static_assert(ROWS * CH % THREADS == 0, "tile must divide over the workgroup");
  u32x4 r[PER];
  __device__ __forceinline__ void load(const bf16_t* base, int ld, int row0, int last_row, int tid) {
#pragma unroll
    for (int it = 0; it < PER; ++it) {
      const int c = tid + it * THREADS;
      const int row = min(row0 + c / CH, last_row);
      r[it] = *(const u32x4*)(base + (long long)row * ld + (c % CH) * 8);
    }
  }
  template <bool ALONG_ROWS, bool DOWN_COLS>
  __device__ __forceinline__ void store(bf16_t* tile_rows, bf16_t* tile_cols, int tid) const {
#pragma unroll
    for (int it = 0; it < PER; ++it) {
      const int c = tid + it * THREADS;
      if (ALONG_ROWS) *(u32x4*)(tile_rows + off_kc<D>(c / CH, c % CH)) = r[it];
      if (DOWN_COLS) *(u32x4*)(tile_cols + off_ks<D>(c / CH, (c % CH) * 8)) = r[it];
    }
  }
};

// ---------------------------------------------------------------- forward
template <int D, bool CAUSAL, int NW>
__global__ __launch_bounds__(NW * 64) void attn_fused_fwd_kernel(FusedArgs a) {
  constexpr int BQ = NW * 32, BKEY = 64, KS = D / 16, DT = D / 32, THREADS = NW * 64;
  __shared__ __attribute__((aligned(16))) bf16_t ldsK[2][BKEY * D];
  __shared__ __attribute__((aligned(16))) bf16_t ldsV[2][BKEY * D];
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int tile = gridDim.x - 1 - blockIdx.x;  // the tiles with the longest causal loops start first
  const int mat = blockIdx.y, dev = blockIdx.z, s = a.s;
  const int seq = mat / a.nh, head = mat % a.nh;
  const bf16_t* Qp = a.qkv + dev * a.dev_qkv + (long long)seq * s * a.ld + head * 3 * D;
  const bf16_t* Kp = Qp + D;
  const bf16_t* Vp = Qp + 2 * D;
  const int q0 = tile * BQ + wave * 32;
  const int query = q0 + (lane & 31);
  const int qrow = min(query, s - 1);
  bf16x8 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) qf[ks] = *(const bf16x8*)(Qp + (long long)qrow * a.ld + ks * 16 + g * 8);
  const int wg_hi = min(tile * BQ + BQ, s) - 1;  // last query row of the workgroup
  const int nkb = CAUSAL ? wg_hi / BKEY + 1 : (s + BKEY - 1) / BKEY;
  const int wave_nkb = q0 >= s ? 0 : (CAUSAL ? min(q0 + 31, s - 1) / BKEY + 1 : nkb);
  const int limit = CAUSAL ? qrow : s - 1;  // last key this lane's row may see

  f32x16 oacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) oacc[dt] = zero16();
  float m_run = -INFINITY, l_run = 0.f;

  TileCopy<BKEY, D, THREADS> ck, cv;
  ck.load(Kp, a.ld, 0, s - 1, tid);
  cv.load(Vp, a.ld, 0, s - 1, tid);
  ck.template store<true, false>(ldsK[0], nullptr, tid);
  cv.template store<false, true>(nullptr, ldsV[0], tid);
  __syncthreads();
  for (int kb = 0; kb < nkb; ++kb) {
    const int buf = kb & 1;
    if (kb + 1 < nkb) {
      ck.load(Kp, a.ld, (kb + 1) * BKEY, s - 1, tid);
      cv.load(Vp, a.ld, (kb + 1) * BKEY, s - 1, tid);
    }
    if (kb < wave_nkb) {
      const int kbase = kb * BKEY;
      f32x16 sacc[2];
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        sacc[t2] = zero16();
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          sacc[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<D>(ldsK[buf], t2 * 32, ks, lane), qf[ks], sacc[t2], 0, 0, 0);
      }
      // keys of this block past the row's limit exist only in the last blocks of the loop (wave-uniform test)
      const bool need_mask = CAUSAL ? (kbase + BKEY - 1 > q0) : (kbase + BKEY > s);
      if (need_mask) {
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = kbase + t2 * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
            if (key > limit) sacc[t2][r] = -INFINITY;
          }
      }
      float mx = -INFINITY;
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[t2][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * a.scale_log2;  // the scale is positive: it commutes with the maximum
      const float m_new = fmaxf(m_run, mx);  // finite: block 0 holds key 0, visible to every row
      float sum = 0.f;
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = __builtin_amdgcn_exp2f(fmaf(sacc[t2][r], a.scale_log2, -m_new));  // masked: exp2(-inf) = 0
          sacc[t2][r] = p;
          sum += p;
        }
      sum += __shfl_xor(sum, 32, 64);
      if (__builtin_amdgcn_ballot_w64(m_new != m_run) != 0) {  // some row's maximum moved: rescale what was accumulated
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        l_run *= alpha;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
        m_run = m_new;
      }
      l_run += sum;
      bf16x8 pf[2][2];
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        pf[t2][0] = pack_acc<0>(sacc[t2]);
        pf[t2][1] = pack_acc<1>(sacc[t2]);
      }
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int dt = 0; dt < DT; ++dt)
            oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_acc_order<D>(ldsV[buf], t2 * 32 + u * 16, dt * 32, lane),
                                                               pf[t2][u], oacc[dt], 0, 0, 0);
    }
    if (kb + 1 < nkb) {
      ck.template store<true, false>(ldsK[buf ^ 1], nullptr, tid);
      cv.template store<false, true>(nullptr, ldsV[buf ^ 1], tid);
    }
    __syncthreads();
  }
  if (wave_nkb > 0 && query < s) {
    const float inv = 1.0f / l_run;
    bf16_t* Op = a.attn + dev * a.dev_attn + ((long long)seq * s + query) * a.ldo + head * D;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        u32x2 w = {pack2_bf16(oacc[dt][4 * c] * inv, oacc[dt][4 * c + 1] * inv),
                   pack2_bf16(oacc[dt][4 * c + 2] * inv, oacc[dt][4 * c + 3] * inv)};
        *(u32x2*)(Op + dt * 32 + 8 * c + 4 * g) = w;
      }
    if (g == 0) a.lse[dev * a.dev_vec + (long long)mat * s + query] = (m_run + __log2f(l_run)) * LN2;
  }
}

// ---------------------------------------------------------------- backward, dQ (and rowsum(dO * O))
template <int D, bool CAUSAL, int NW>
__global__ __launch_bounds__(NW * 64) void attn_fused_bwd_dq_kernel(FusedArgs a) {
  constexpr int BQ = NW * 32, BKEY = 64, KS = D / 16, DT = D / 32, THREADS = NW * 64;
  __shared__ __attribute__((aligned(16))) bf16_t ldsKr[2][BKEY * D];  // K along rows (for S)
  __shared__ __attribute__((aligned(16))) bf16_t ldsKc[2][BKEY * D];  // K down columns (for dQ)
  __shared__ __attribute__((aligned(16))) bf16_t ldsVr[2][BKEY * D];  // V along rows (for dP)
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int tile = gridDim.x - 1 - blockIdx.x;
  const int mat = blockIdx.y, dev = blockIdx.z, s = a.s;
  const int seq = mat / a.nh, head = mat % a.nh;
  const bf16_t* Qp = a.qkv + dev * a.dev_qkv + (long long)seq * s * a.ld + head * 3 * D;
  const bf16_t* Kp = Qp + D;
  const bf16_t* Vp = Qp + 2 * D;
  const int q0 = tile * BQ + wave * 32;
  const int query = q0 + (lane & 31);
  const int qrow = min(query, s - 1);
  const long long orow = dev * a.dev_attn + ((long long)seq * s + qrow) * a.ldo + head * D;
  const long long vrow = dev * a.dev_vec + (long long)mat * s + qrow;
  bf16x8 qf[KS], dof[KS];
  float delta = 0.f;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    qf[ks] = *(const bf16x8*)(Qp + (long long)qrow * a.ld + ks * 16 + g * 8);
    dof[ks] = *(const bf16x8*)(a.d_attn + orow + ks * 16 + g * 8);
    const bf16x8 of = *(const bf16x8*)(a.attn + orow + ks * 16 + g * 8);
    const u32x4 gw = __builtin_bit_cast(u32x4, dof[ks]), ow = __builtin_bit_cast(u32x4, of);
#pragma unroll
    for (int w = 0; w < 4; ++w)
      delta += __uint_as_float(gw[w] << 16) * __uint_as_float(ow[w] << 16) +
               __uint_as_float(gw[w] & 0xffff0000u) * __uint_as_float(ow[w] & 0xffff0000u);
  }
  delta += __shfl_xor(delta, 32, 64);
  if (g == 0 && query < s) a.delta[vrow] = delta;
  const float lse2 = a.lse[vrow] * LOG2E;
  const int wg_hi = min(tile * BQ + BQ, s) - 1;
  const int nkb = CAUSAL ? wg_hi / BKEY + 1 : (s + BKEY - 1) / BKEY;
  const int wave_nkb = q0 >= s ? 0 : (CAUSAL ? min(q0 + 31, s - 1) / BKEY + 1 : nkb);
  const int limit = CAUSAL ? qrow : s - 1;

  f32x16 dqacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) dqacc[dt] = zero16();

  TileCopy<BKEY, D, THREADS> ck, cv;
  ck.load(Kp, a.ld, 0, s - 1, tid);
  cv.load(Vp, a.ld, 0, s - 1, tid);
  ck.template store<true, true>(ldsKr[0], ldsKc[0], tid);
  cv.template store<true, false>(ldsVr[0], nullptr, tid);
  __syncthreads();
  for (int kb = 0; kb < nkb; ++kb) {
    const int buf = kb & 1;
    if (kb + 1 < nkb) {
      ck.load(Kp, a.ld, (kb + 1) * BKEY, s - 1, tid);
      cv.load(Vp, a.ld, (kb + 1) * BKEY, s - 1, tid);
    }
    if (kb < wave_nkb) {
      const int kbase = kb * BKEY;
      f32x16 sacc[2], pacc[2];
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        sacc[t2] = zero16();
        pacc[t2] = zero16();
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          sacc[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<D>(ldsKr[buf], t2 * 32, ks, lane), qf[ks], sacc[t2], 0, 0, 0);
          pacc[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<D>(ldsVr[buf], t2 * 32, ks, lane), dof[ks], pacc[t2], 0, 0, 0);
        }
      }
      const bool need_mask = CAUSAL ? (kbase + BKEY - 1 > q0) : (kbase + BKEY > s);
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kbase + t2 * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
          float p = __builtin_amdgcn_exp2f(sacc[t2][r] * a.scale_log2 - lse2);
          if (need_mask && key > limit) p = 0.f;
          sacc[t2][r] = p * (pacc[t2][r] - delta);  // dS^T
        }
      bf16x8 dsf[2][2];
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        dsf[t2][0] = pack_acc<0>(sacc[t2]);
        dsf[t2][1] = pack_acc<1>(sacc[t2]);
      }
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int dt = 0; dt < DT; ++dt)
            dqacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_acc_order<D>(ldsKc[buf], t2 * 32 + u * 16, dt * 32, lane),
                                                                dsf[t2][u], dqacc[dt], 0, 0, 0);
    }
    if (kb + 1 < nkb) {
      ck.template store<true, true>(ldsKr[buf ^ 1], ldsKc[buf ^ 1], tid);
      cv.template store<true, false>(ldsVr[buf ^ 1], nullptr, tid);
    }
    __syncthreads();
  }
  if (wave_nkb > 0 && query < s) {
    bf16_t* dQp = a.d_qkv + dev * a.dev_qkv + ((long long)seq * s + query) * a.ld + head * 3 * D;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        u32x2 w = {pack2_bf16(dqacc[dt][4 * c] * a.scale, dqacc[dt][4 * c + 1] * a.scale),
                   pack2_bf16(dqacc[dt][4 * c + 2] * a.scale, dqacc[dt][4 * c + 3] * a.scale)};
        *(u32x2*)(dQp + dt * 32 + 8 * c + 4 * g) = w;
      }
  }
}

// ---------------------------------------------------------------- backward, dK and dV
// One wavefront owns 32 keys; the loop runs over blocks of BQB queries (from the diagonal on when causal).
template <int D, bool CAUSAL, int BQB, int NW>
__global__ __launch_bounds__(NW * 64) void attn_fused_bwd_dkv_kernel(FusedArgs a) {
  constexpr int BKW = NW * 32, KS = D / 16, DT = D / 32, T2 = BQB / 32, THREADS = NW * 64;
  __shared__ __attribute__((aligned(16))) bf16_t ldsQr[2][BQB * D];   // Q along rows (for S)
  __shared__ __attribute__((aligned(16))) bf16_t ldsQc[2][BQB * D];   // Q down columns (for dK)
  __shared__ __attribute__((aligned(16))) bf16_t ldsGr[2][BQB * D];   // dO along rows (for dP)
  __shared__ __attribute__((aligned(16))) bf16_t ldsGc[2][BQB * D];   // dO down columns (for dV)
  __shared__ __attribute__((aligned(16))) float ldsL[2][BQB];         // lse * log2(e) of the block's queries
  __shared__ __attribute__((aligned(16))) float ldsD[2][BQB];         // rowsum(dO * O)
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int tile = blockIdx.x;  // early key tiles have the longest causal loops
  const int mat = blockIdx.y, dev = blockIdx.z, s = a.s;
  const int seq = mat / a.nh, head = mat % a.nh;
  const bf16_t* Qp = a.qkv + dev * a.dev_qkv + (long long)seq * s * a.ld + head * 3 * D;
  const bf16_t* Kp = Qp + D;
  const bf16_t* Vp = Qp + 2 * D;
  const bf16_t* Gp = a.d_attn + dev * a.dev_attn + (long long)seq * s * a.ldo + head * D;
  const float* Lp = a.lse + dev * a.dev_vec + (long long)mat * s;
  const float* Dp = a.delta + dev * a.dev_vec + (long long)mat * s;
  const int k0 = tile * BKW + wave * 32;
  const int key = k0 + (lane & 31);
  const int krow = min(key, s - 1);
  bf16x8 kf[KS], vf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    kf[ks] = *(const bf16x8*)(Kp + (long long)krow * a.ld + ks * 16 + g * 8);
    vf[ks] = *(const bf16x8*)(Vp + (long long)krow * a.ld + ks * 16 + g * 8);
  }
  const int nqb = (s + BQB - 1) / BQB;
  const int qb_lo = CAUSAL ? (tile * BKW) / BQB : 0;           // first block with a query >= the first key
  const int wave_qb_lo = k0 >= s ? nqb : (CAUSAL ? k0 / BQB : 0);

  f32x16 dkacc[DT], dvacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) {
    dkacc[dt] = zero16();
    dvacc[dt] = zero16();
  }
  TileCopy<BQB, D, THREADS> cq, cg;
  float lreg = 0.f, dreg = 0.f;
  auto gload = [&](int qb) {
    cq.load(Qp, a.ld, qb * BQB, s - 1, tid);
    cg.load(Gp, a.ldo, qb * BQB, s - 1, tid);
    if (tid < BQB) {
      const int row = min(qb * BQB + tid, s - 1);
      lreg = Lp[row] * LOG2E;
      dreg = Dp[row];
    }
  };
  auto lstore = [&](int buf) {
    cq.template store<true, true>(ldsQr[buf], ldsQc[buf], tid);
    cg.template store<true, true>(ldsGr[buf], ldsGc[buf], tid);
    if (tid < BQB) {
      ldsL[buf][tid] = lreg;
      ldsD[buf][tid] = dreg;
    }
  };
  if (qb_lo < nqb) {
    gload(qb_lo);
    lstore(qb_lo & 1);
  }
  __syncthreads();
  for (int qb = qb_lo; qb < nqb; ++qb) {
    const int buf = qb & 1;
    if (qb + 1 < nqb) gload(qb + 1);
    if (qb >= wave_qb_lo) {
      const int qbase = qb * BQB;
      f32x16 sacc[T2], pacc[T2];
#pragma unroll
      for (int t2 = 0; t2 < T2; ++t2) {
        sacc[t2] = zero16();
        pacc[t2] = zero16();
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          sacc[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<D>(ldsQr[buf], t2 * 32, ks, lane), kf[ks], sacc[t2], 0, 0, 0);
          pacc[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<D>(ldsGr[buf], t2 * 32, ks, lane), vf[ks], pacc[t2], 0, 0, 0);
        }
      }
      // masked: queries before the key (causal, only in the blocks that touch the diagonal) and padding queries
      const bool need_mask = (CAUSAL && qbase < k0 + 31) || (qbase + BQB > s);
      bf16x8 pf[T2][2], dsf[T2][2];
#pragma unroll
      for (int t2 = 0; t2 < T2; ++t2) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int qi = t2 * 32 + 8 * c + 4 * g;
          const float4 l4 = *(const float4*)(&ldsL[buf][qi]);
          const float4 d4 = *(const float4*)(&ldsD[buf][qi]);
          const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int r = 4 * c + e;
            const int qy = qbase + qi + e;
            float p = __builtin_amdgcn_exp2f(sacc[t2][r] * a.scale_log2 - lv[e]);
            if (need_mask && (qy >= s || (CAUSAL && qy < key))) p = 0.f;
            sacc[t2][r] = p;
            pacc[t2][r] = p * (pacc[t2][r] - dv[e]);  // dS
          }
        }
        pf[t2][0] = pack_acc<0>(sacc[t2]);
        pf[t2][1] = pack_acc<1>(sacc[t2]);
        dsf[t2][0] = pack_acc<0>(pacc[t2]);
        dsf[t2][1] = pack_acc<1>(pacc[t2]);
      }
#pragma unroll
      for (int t2 = 0; t2 < T2; ++t2)
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) {
            dvacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_acc_order<D>(ldsGc[buf], t2 * 32 + u * 16, dt * 32, lane),
                                                                pf[t2][u], dvacc[dt], 0, 0, 0);
            dkacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_acc_order<D>(ldsQc[buf], t2 * 32 + u * 16, dt * 32, lane),
                                                                dsf[t2][u], dkacc[dt], 0, 0, 0);
          }
    }
    if (qb + 1 < nqb) lstore(buf ^ 1);
    __syncthreads();
  }
  if (key < s) {
    bf16_t* dKp = a.d_qkv + dev * a.dev_qkv + ((long long)seq * s + key) * a.ld + head * 3 * D + D;
    bf16_t* dVp = dKp + D;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        u32x2 wk = {pack2_bf16(dkacc[dt][4 * c] * a.scale, dkacc[dt][4 * c + 1] * a.scale),
                    pack2_bf16(dkacc[dt][4 * c + 2] * a.scale, dkacc[dt][4 * c + 3] * a.scale)};
        u32x2 wv = {pack2_bf16(dvacc[dt][4 * c], dvacc[dt][4 * c + 1]), pack2_bf16(dvacc[dt][4 * c + 2], dvacc[dt][4 * c + 3])};
        *(u32x2*)(dKp + dt * 32 + 8 * c + 4 * g) = wk;
        *(u32x2*)(dVp + dt * 32 + 8 * c + 4 * g) = wv;
      }
  }
}

FusedArgs make_args(const AttnFusedDesc& d) {
  FusedArgs a = {};
  a.qkv = (const bf16_t*)d.qkv; a.attn = (bf16_t*)d.attn; a.lse = d.lse;
  a.d_attn = (const bf16_t*)d.d_attn; a.d_qkv = (bf16_t*)d.d_qkv; a.delta = d.delta;
  a.s = d.s; a.nh = d.nh; a.ld = d.ld; a.ldo = d.ldo;
  a.dev_qkv = d.dev_qkv; a.dev_attn = d.dev_attn; a.dev_vec = (long long)d.nb * d.nh * d.s;
  a.scale = 1.0f / sqrtf((float)d.d);
  a.scale_log2 = a.scale * LOG2E;
  return a;
}

bool desc_ok(const AttnFusedDesc& d) {
  if (!attn_fused_supported(d.d)) return false;
  if (d.s < 1 || d.nb < 1 || d.nh < 1 || d.ndev < 1 || d.ndev > 65535) return false;
  if ((long long)d.nb * d.nh > 65535) return false;
  if (d.ld % 8 || d.ldo % 8 || d.ld < 3 * d.d * d.nh || d.ldo < d.d * d.nh) return false;
  return true;
}

}  // namespace

bool attn_fused_supported(int d) { return d == 64 || d == 128; }

namespace {
// Four wavefronts (128 rows) per workgroup when that still gives every compute unit a workgroup, two otherwise.
bool use_two_waves(const AttnFusedDesc& d) { return (long long)((d.s + 127) / 128) * d.nb * d.nh * d.ndev < 256; }

template <int D, int NW>
void fwd_launch(const FusedArgs& a, const AttnFusedDesc& d, hipStream_t st) {
  const dim3 grid((d.s + NW * 32 - 1) / (NW * 32), d.nb * d.nh, d.ndev), block(NW * 64);
  if (d.causal) attn_fused_fwd_kernel<D, true, NW><<<grid, block, 0, st>>>(a);
  else attn_fused_fwd_kernel<D, false, NW><<<grid, block, 0, st>>>(a);
}
template <int D, int NW>
void bwd_launch(const FusedArgs& a, const AttnFusedDesc& d, hipStream_t st) {
  constexpr int BQB = D == 128 ? 32 : 64;
  const dim3 grid((d.s + NW * 32 - 1) / (NW * 32), d.nb * d.nh, d.ndev), block(NW * 64);
  if (d.causal) {
    attn_fused_bwd_dq_kernel<D, true, NW><<<grid, block, 0, st>>>(a);
    attn_fused_bwd_dkv_kernel<D, true, BQB, NW><<<grid, block, 0, st>>>(a);
  } else {
    attn_fused_bwd_dq_kernel<D, false, NW><<<grid, block, 0, st>>>(a);
    attn_fused_bwd_dkv_kernel<D, false, BQB, NW><<<grid, block, 0, st>>>(a);
  }
}
}  // namespace

int launch_attn_fused_fwd(const AttnFusedDesc& d, hipStream_t st) {
  if (!desc_ok(d) || !d.qkv || !d.attn || !d.lse) return OPTIMUS_ESHAPE;
  const FusedArgs a = make_args(d);
  const bool two = use_two_waves(d);
  if (d.d == 64) two ? fwd_launch<64, 2>(a, d, st) : fwd_launch<64, 4>(a, d, st);
  else two ? fwd_launch<128, 2>(a, d, st) : fwd_launch<128, 4>(a, d, st);
  return hip_launch_status();
}

int launch_attn_fused_bwd(const AttnFusedDesc& d, hipStream_t st) {
  if (!desc_ok(d) || !d.qkv || !d.attn || !d.lse || !d.d_attn || !d.d_qkv || !d.delta) return OPTIMUS_ESHAPE;
  const FusedArgs a = make_args(d);
  const bool two = use_two_waves(d);
  if (d.d == 64) two ? bwd_launch<64, 2>(a, d, st) : bwd_launch<64, 4>(a, d, st);
  else two ? bwd_launch<128, 2>(a, d, st) : bwd_launch<128, 4>(a, d, st);
  return hip_launch_status();
}

}  // namespace optimus

// Fused local attention for gfx950 (CDNA4): O = softmax(Q K^T / sqrt(d)) V for every local (sequence, head) of a
// device without the [b/q, n/q, s, s] score and probability tensors ever reaching memory -- the operator fusion the
// paper's conclusion proposes as future work for its sequence-length limit (Section 6; the attention itself is that
// of Sections 2.1 / 3.2.1: whole sequences and n/q heads are local to a device, so no row is split).
//
// Forward keeps one fp32 number per query row, L = log sum_u exp(S_tu); backward rebuilds P = exp(S - L) tile by tile
// and uses rowsum(dO * O) in place of rowsum(dP * P).
// Backward is two bodies (dQ; dK and dV), each recomputing S; small launches run them as one grid ordered by loop
// length (attn_fused_bwd_kernel), large ones as two kernels.
//
// Work layout (forward and both backward bodies).  A workgroup of four wavefronts owns 64 rows (queries in the forward and dQ
// kernels, keys in the dK/dV kernel).  Wavefront w works on rows 32*(w & 1).. and on every second 64-wide block of the
// other index (blocks of parity w >> 1): the loop over the other index is the critical path of these launches (the
// configurations this library is built for give at most two wavefronts per compute unit), so it is cut in two and
// the two partial results are merged through LDS at the end (soft-max partials by the usual max / sum rule,
// gradient partials by addition).
//
// Every product is v_mfma_f32_32x32x16_bf16 with the operand that carries the wavefront's own rows in the B slot, so
// that a lane's 16 accumulator values of a 32x32 tile all belong to ONE of its rows (lane % 32) and the other 16
// live in lane ^ 32: row maxima and sums are 16 in-lane operations plus one half-wave swap.  The accumulator of S^T
// (S in the dK/dV kernel) is already laid out as the B operand of the next product up to a fixed permutation of the
// contraction index: accumulator slot r of lane group g = lane / 32 is row 8*(r/4) + 4*g + r%4 of the tile, a 16-wide
// contraction step takes slots 8u..8u+7, i.e. rows {16u + 4g + 0..3, 16u + 8 + 4g + 0..3}.  A contraction may visit
// its index in any order as long as both operands agree, so the A operand (V, K, dO or Q read "down the columns" with
// the transposing LDS read ds_read_b64_tr_b16) is simply fetched in that order.  P and dS never leave registers.
//
// Blocks of the other index go global -> LDS directly (buffer_load_dwordx4 ... lds, one KiB per wavefront
// instruction, no registers, no LDS store instructions), two stages, one barrier per pair of blocks; the pieces of the
// next pair are issued in one go at the top of an iteration (spreading them between the matrix instructions was
// measured slower here: at 64 KiB per iteration and compute unit the loop runs at the rate the memory path delivers,
// about 27 B/clk per compute unit with every unit loading, wherever the issue slots are).  One LDS copy
// of a [rows][D] tile serves both ways of reading it: 16-byte chunk c of row r sits at chunk position c ^ g(r) with
// g(r) = ((r & 3) << 2) | ((r >> 2) & 3) for 256-byte rows (and the analogous 3-bit form for 128-byte rows, which pair
// up to span the 64 banks).  Reading along the rows (ds_read_b128, 16 consecutive rows, same chunk) sees 16 distinct
// positions; the transposing read (4 consecutive rows x 4 consecutive chunks at a time) sees 4 x 4 distinct ones.
// Since the load is direct, the swizzle is applied on the global side: the lane that writes LDS position p fetches
// the chunk that belongs there.
#include "common.hpp"

namespace optimus {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
typedef __attribute__((ext_vector_type(4))) int i32x4;

constexpr float LOG2E = 1.44269504088896340736f;
constexpr float LN2 = 0.69314718055994530942f;
constexpr int BLK = 64;     // rows of one block of the looped index
constexpr int PAIR = 128;   // two blocks (one per parity) are loaded and consumed per loop iteration
constexpr int NWAVES = 4;

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

// ---- LDS tile [rows][D] bf16, chunk position = chunk ^ g(row) ----
template <int D>
__device__ __forceinline__ int swz(int row) {
  static_assert(D == 64 || D == 128, "head widths built");
  if (D == 128) return ((row & 3) << 2) | ((row >> 2) & 3);
  return (((row >> 1) & 1) << 2) | ((row >> 2) & 3);
}
template <int D>
__device__ __forceinline__ int tile_off(int row, int chunk) { return row * D + ((chunk ^ swz<D>(row)) << 3); }

// A-operand fragment along the rows: lane holds row (row0 + lane%32), contraction elements 16*ks + 8*(lane/32) + 0..7.
template <int D>
__device__ __forceinline__ bf16x8 frag_rows(const bf16_t* tile, int row0, int ks, int lane) {
  return *(const bf16x8*)(tile + tile_off<D>(row0 + (lane & 31), ks * 2 + (lane >> 5)));
}
// A-operand fragment down the columns in accumulator order: lane holds column (col0 + lane%32) and the tile rows
// row0 + 4g + {0..3} and row0 + 8 + 4g + {0..3}, g = lane/32 (row0 a multiple of 16, col0 of 32).
template <int D>
__device__ __forceinline__ bf16x8 frag_cols_acc_order(const bf16_t* tile, int row0, int col0, int lane) {
  const int lg = lane & 15;
  const int col = col0 + (((lane >> 4) & 1) << 4) + ((lg & 3) << 2);  // 4 consecutive columns from here
  const int row = row0 + ((lane >> 5) << 2) + (lg >> 2);
  const bf16_t* p0 = tile + tile_off<D>(row, col >> 3) + (col & 7);
  const bf16_t* p1 = tile + tile_off<D>(row + 8, col >> 3) + (col & 7);
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

// The value of the other half-wave's lane (lane ^ 32) combined with the own one.
__device__ __forceinline__ float halfwave_max(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float halfwave_sum(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// ---- direct global -> LDS copy of a PAIR x D tile (rows row0 .. row0 + 127 of a [s][ld] matrix) by NW wavefronts ----
__device__ __forceinline__ i32x4 make_rsrc(const bf16_t* base) {  // raw buffer, 2 GiB window (offsets used are far below)
  const unsigned long long p = (unsigned long long)base;  // wave-uniform by construction; say so to the compiler
  const int lo = __builtin_amdgcn_readfirstlane((int)(unsigned)p);
  const int hi = __builtin_amdgcn_readfirstlane((int)(unsigned)((p >> 32) & 0xffffu));
  return i32x4{lo, hi, (int)0x80000000u, 0x00020000};
}
template <int D, int NW = NWAVES>
struct PairLoader {
  static constexpr int CH = D / 8, ROWS_PER_KIB = 64 / CH, PIECES = PAIR * D * 2 / 1024, PER = PIECES / NW;
  static_assert(PIECES % NW == 0, "tile must divide over the wavefronts");
  unsigned off[PER];  // byte offsets of this lane's chunks for a tile that lies entirely inside the matrix
  int ld, wave, lane;
  __device__ __forceinline__ void init(int ld_, int wave_, int lane_) {
    ld = ld_; wave = wave_; lane = lane_;
#pragma unroll
    for (int it = 0; it < PER; ++it) off[it] = offset_of(it, 0, 0x7fffffff, 0);
  }
  // LDS position p = lane of KiB piece (wave*PER + it) is (row, chunk position lane % CH): fetch chunk pos ^ g(row).
  // The source row is clamped to the last row of the matrix (rows past the end are only ever multiplied by zeros).
  __device__ __forceinline__ unsigned offset_of(int it, int row0, int last_row, int base_row) const {
    const int row = (wave * PER + it) * ROWS_PER_KIB + lane / CH;
    const int chunk = (lane % CH) ^ swz<D>(row);
    const int src = min(row0 + row, last_row) - base_row;
    return (unsigned)(src * ld + chunk * 8) * 2u;
  }
  // mat: row 0 of the [s][ld] matrix (already offset to the head's columns); tile: LDS destination, PAIR * D elements
  __device__ __forceinline__ void issue(const bf16_t* mat, int row0, int s, bf16_t* tile) const {
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) bf16_t*)tile;
    if (row0 + PAIR <= s) {
      const i32x4 rsrc = make_rsrc(mat + (long long)row0 * ld);
#pragma unroll
      for (int it = 0; it < PER; ++it) {
        const unsigned m0v = __builtin_amdgcn_readfirstlane(lds_base + (unsigned)(wave * PER + it) * 1024u);
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %1, 0 offen lds" ::"v"(off[it]), "s"(rsrc), "s"(m0v) : "memory", "m0");
      }
    } else {  // the tile reaches past the last row: clamp (wave-uniform branch, taken for the last pair only)
      const int base_row = max(0, s - PAIR);
      const i32x4 rsrc = make_rsrc(mat + (long long)base_row * ld);
#pragma unroll
      for (int it = 0; it < PER; ++it) {
        const unsigned o = offset_of(it, row0, s - 1, base_row);
        const unsigned m0v = __builtin_amdgcn_readfirstlane(lds_base + (unsigned)(wave * PER + it) * 1024u);
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %1, 0 offen lds" ::"v"(o), "s"(rsrc), "s"(m0v) : "memory", "m0");
      }
    }
  }
};

// all direct loads of this wavefront have landed, then the workgroup meets
__device__ __forceinline__ void wait_loads_and_barrier() {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
}

// ---------------------------------------------------------------- forward
// NRG: row groups of 32 queries per workgroup (2: 64 rows, four wavefronts; 4: 128 rows, eight wavefronts -- half the
// K/V bytes per flop and two wavefronts per SIMD, for launches with more workgroups than compute units).
template <int D, bool CAUSAL, int NRG>
__global__ __launch_bounds__(NRG * 128) void attn_fused_fwd_kernel(FusedArgs a) {
  constexpr int KS = D / 16, DT = D / 32, BQ = NRG * 32;
  __shared__ __attribute__((aligned(1024))) bf16_t lds[2][2][PAIR * D];  // [stage][K, V][pair tile]
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int rg = wave % NRG, par = wave / NRG;
  const int tile = gridDim.x - 1 - blockIdx.x;  // the tiles with the longest causal loops start first
  const int mat = blockIdx.y, dev = blockIdx.z, s = a.s;
  const int seq = mat / a.nh, head = mat % a.nh;
  const bf16_t* Qp = a.qkv + dev * a.dev_qkv + (long long)seq * s * a.ld + head * 3 * D;
  const bf16_t* Kp = Qp + D;
  const bf16_t* Vp = Qp + 2 * D;
  const int q0 = tile * BQ + rg * 32;
  const int query = q0 + (lane & 31);
  const int qrow = min(query, s - 1);
  bf16x8 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) qf[ks] = *(const bf16x8*)(Qp + (long long)qrow * a.ld + ks * 16 + g * 8);
  const int wg_hi = min(tile * BQ + BQ, s) - 1;  // last query row of the workgroup
  const int nkb = CAUSAL ? wg_hi / BLK + 1 : (s + BLK - 1) / BLK;
  const int n_it = (nkb + 1) / 2;
  const int wave_nkb = q0 >= s ? 0 : (CAUSAL ? min(q0 + 31, s - 1) / BLK + 1 : nkb);
  const int limit = CAUSAL ? qrow : s - 1;  // last key this lane's row may see

  f32x16 oacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) oacc[dt] = zero16();
  float m_run = -INFINITY, l_run = 0.f;

  PairLoader<D, 2 * NRG> ldr;
  ldr.init(a.ld, wave, lane);
  ldr.issue(Kp, 0, s, lds[0][0]);
  ldr.issue(Vp, 0, s, lds[0][1]);
  wait_loads_and_barrier();
  for (int it = 0; it < n_it; ++it) {
    const int st = it & 1;
    if (it + 1 < n_it) {
      ldr.issue(Kp, (it + 1) * PAIR, s, lds[st ^ 1][0]);
      ldr.issue(Vp, (it + 1) * PAIR, s, lds[st ^ 1][1]);
    }
    const int kb = 2 * it + par;
    if (kb < wave_nkb) {
      const bf16_t* tK = lds[st][0] + par * BLK * D;
      const bf16_t* tV = lds[st][1] + par * BLK * D;
      const int kbase = kb * BLK;
      f32x16 sacc[2];
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        sacc[t2] = zero16();
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          sacc[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<D>(tK, t2 * 32, ks, lane), qf[ks], sacc[t2], 0, 0, 0);
      }
      // keys of this block past the row's limit exist only in the last blocks of the loop (wave-uniform test)
      const bool need_mask = CAUSAL ? (kbase + BLK - 1 > q0) : (kbase + BLK > s);
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
      mx = halfwave_max(mx) * a.scale_log2;  // the scale is positive: it commutes with the maximum
      // Every block a wavefront works on holds a visible key for each of its rows (the first key of a block is
      // never past the wavefront's first row), so mx is finite.
      // The running maximum only has to keep exp2 in range, not to be the true maximum: it follows the block
      // maximum only when that is more than 2^8 above it (wave-uniform decision), which spares the rescaling of
      // the accumulators in nearly every block.  p <= 2^8 then; the normalisation by l and the log-sum-exp
      // m + log2(l) are unchanged by the choice of m.
      const bool move = __builtin_amdgcn_ballot_w64(mx > m_run + 8.0f) != 0;
      const float m_new = move ? fmaxf(m_run, mx) : m_run;
      float sum = 0.f;
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = __builtin_amdgcn_exp2f(fmaf(sacc[t2][r], a.scale_log2, -m_new));  // masked: exp2(-inf) = 0
          sacc[t2][r] = p;
          sum += p;
        }
      sum = halfwave_sum(sum);
      if (move) {  // rescale what was accumulated
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
            oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_acc_order<D>(tV, t2 * 32 + u * 16, dt * 32, lane),
                                                               pf[t2][u], oacc[dt], 0, 0, 0);
    }
    wait_loads_and_barrier();
  }
  // merge the two parities: the odd one hands (m, l, O) over through LDS (all tiles are free after the last barrier)
  float* xch = (float*)&lds[0][0][0] + rg * (DT * 16 + 2) * 64;
  if (par == 1) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) xch[(dt * 16 + r) * 64 + lane] = oacc[dt][r];
    xch[(DT * 16) * 64 + lane] = m_run;
    xch[(DT * 16 + 1) * 64 + lane] = l_run;
  }
  __syncthreads();
  if (par == 0 && wave_nkb > 0 && query < s) {
    const float m1 = xch[(DT * 16) * 64 + lane], l1 = xch[(DT * 16 + 1) * 64 + lane];
    const float m = fmaxf(m_run, m1);  // m_run is finite: block 0 belongs to this parity
    const float a0 = __builtin_amdgcn_exp2f(m_run - m), a1 = __builtin_amdgcn_exp2f(m1 - m);  // a1 = 0 if the other had no block
    const float l = l_run * a0 + l1 * a1;
    const float inv = 1.0f / l;
    const float w0 = a0 * inv, w1 = a1 * inv;
    bf16_t* Op = a.attn + dev * a.dev_attn + ((long long)seq * s + query) * a.ldo + head * D;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = oacc[dt][4 * c + e] * w0 + xch[(dt * 16 + 4 * c + e) * 64 + lane] * w1;
        u32x2 w = {pack2_bf16(o[0], o[1]), pack2_bf16(o[2], o[3])};
        *(u32x2*)(Op + dt * 32 + 8 * c + 4 * g) = w;
      }
    if (g == 0) a.lse[dev * a.dev_vec + (long long)mat * s + query] = (m + __log2f(l)) * LN2;
  }
}

// ---------------------------------------------------------------- backward, dQ (and rowsum(dO * O))
// One lane's share of rowsum(dO * O): 8 products of one 16-byte chunk pair, added in element order.
__device__ __forceinline__ float delta_piece(const bf16x8& dof, const bf16x8& of) {
  const u32x4 gw = __builtin_bit_cast(u32x4, dof), ow = __builtin_bit_cast(u32x4, of);
  float d = 0.f;
#pragma unroll
  for (int w = 0; w < 4; ++w) {  // explicit fused multiply-adds: every caller rounds alike
    d = fmaf(__uint_as_float(gw[w] << 16), __uint_as_float(ow[w] << 16), d);
    d = fmaf(__uint_as_float(gw[w] & 0xffff0000u), __uint_as_float(ow[w] & 0xffff0000u), d);
  }
  return d;
}

// OWN_DELTA: the workgroup computes rowsum(dO * O) of its rows itself and stores it for the dK/dV kernel of a later
// launch; otherwise it reads what attn_fused_delta_kernel stored.  lds: [stage][K, V][pair tile].
template <int D, bool CAUSAL, int NRG, bool OWN_DELTA>
__device__ __forceinline__ void bwd_dq_body(const FusedArgs& a, bf16_t (*lds)[2][PAIR * D], int tile, int mat, int dev) {
  constexpr int KS = D / 16, DT = D / 32, BQ = NRG * 32;
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int rg = wave % NRG, par = wave / NRG;
  const int s = a.s;
  const int seq = mat / a.nh, head = mat % a.nh;
  const bf16_t* Qp = a.qkv + dev * a.dev_qkv + (long long)seq * s * a.ld + head * 3 * D;
  const bf16_t* Kp = Qp + D;
  const bf16_t* Vp = Qp + 2 * D;
  const int q0 = tile * BQ + rg * 32;
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
    if (OWN_DELTA) delta += delta_piece(dof[ks], *(const bf16x8*)(a.attn + orow + ks * 16 + g * 8));
  }
  if (OWN_DELTA) {
    delta = halfwave_sum(delta);
    if (par == 0 && g == 0 && query < s) a.delta[vrow] = delta;
  } else {
    delta = a.delta[vrow];
  }
  const float lse2 = a.lse[vrow] * LOG2E;
  const int wg_hi = min(tile * BQ + BQ, s) - 1;
  const int nkb = CAUSAL ? wg_hi / BLK + 1 : (s + BLK - 1) / BLK;
  const int n_it = (nkb + 1) / 2;
  const int wave_nkb = q0 >= s ? 0 : (CAUSAL ? min(q0 + 31, s - 1) / BLK + 1 : nkb);
  const int limit = CAUSAL ? qrow : s - 1;

  f32x16 dqacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) dqacc[dt] = zero16();

  PairLoader<D, 2 * NRG> ldr;
  ldr.init(a.ld, wave, lane);
  ldr.issue(Kp, 0, s, lds[0][0]);
  ldr.issue(Vp, 0, s, lds[0][1]);
  wait_loads_and_barrier();
  for (int it = 0; it < n_it; ++it) {
    const int st = it & 1;
    if (it + 1 < n_it) {
      ldr.issue(Kp, (it + 1) * PAIR, s, lds[st ^ 1][0]);
      ldr.issue(Vp, (it + 1) * PAIR, s, lds[st ^ 1][1]);
    }
    const int kb = 2 * it + par;
    if (kb < wave_nkb) {
      const bf16_t* tK = lds[st][0] + par * BLK * D;
      const bf16_t* tV = lds[st][1] + par * BLK * D;
      const int kbase = kb * BLK;
      f32x16 sacc[2], pacc[2];
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        sacc[t2] = zero16();
        pacc[t2] = zero16();
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          sacc[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<D>(tK, t2 * 32, ks, lane), qf[ks], sacc[t2], 0, 0, 0);
          pacc[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<D>(tV, t2 * 32, ks, lane), dof[ks], pacc[t2], 0, 0, 0);
        }
      }
      const bool need_mask = CAUSAL ? (kbase + BLK - 1 > q0) : (kbase + BLK > s);
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kbase + t2 * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
          float p = __builtin_amdgcn_exp2f(fmaf(sacc[t2][r], a.scale_log2, -lse2));
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
            dqacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_acc_order<D>(tK, t2 * 32 + u * 16, dt * 32, lane),
                                                                dsf[t2][u], dqacc[dt], 0, 0, 0);
    }
    wait_loads_and_barrier();
  }
  float* xch = (float*)&lds[0][0][0] + rg * (DT * 16) * 64;
  if (par == 1) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) xch[(dt * 16 + r) * 64 + lane] = dqacc[dt][r];
  }
  __syncthreads();
  if (par == 0 && wave_nkb > 0 && query < s) {
    bf16_t* dQp = a.d_qkv + dev * a.dev_qkv + ((long long)seq * s + query) * a.ld + head * 3 * D;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (dqacc[dt][4 * c + e] + xch[(dt * 16 + 4 * c + e) * 64 + lane]) * a.scale;
        u32x2 w = {pack2_bf16(o[0], o[1]), pack2_bf16(o[2], o[3])};
        *(u32x2*)(dQp + dt * 32 + 8 * c + 4 * g) = w;
      }
  }
}

template <int D, bool CAUSAL, int NRG>
__global__ __launch_bounds__(NRG * 128) void attn_fused_bwd_dq_kernel(FusedArgs a) {
  __shared__ __attribute__((aligned(1024))) bf16_t lds[2][2][PAIR * D];
  bwd_dq_body<D, CAUSAL, NRG, true>(a, lds, gridDim.x - 1 - blockIdx.x, blockIdx.y, blockIdx.z);  // longest causal rows first
}

// rowsum(dO * O) for every query row of the launch: a wavefront takes 32 rows, lane pair (l, l ^ 32) one row.
template <int D>
__global__ __launch_bounds__(256) void attn_fused_delta_kernel(FusedArgs a) {
  const int lane = threadIdx.x & 63, g = lane >> 5, wave = threadIdx.x >> 6;
  const int mat = blockIdx.y, dev = blockIdx.z, s = a.s;
  const int seq = mat / a.nh, head = mat % a.nh;
  const int query = blockIdx.x * 128 + wave * 32 + (lane & 31);
  const int qrow = min(query, s - 1);
  const long long orow = dev * a.dev_attn + ((long long)seq * s + qrow) * a.ldo + head * D;
  float delta = 0.f;
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks)
    delta += delta_piece(*(const bf16x8*)(a.d_attn + orow + ks * 16 + g * 8), *(const bf16x8*)(a.attn + orow + ks * 16 + g * 8));
  delta = halfwave_sum(delta);
  if (g == 0 && query < s) a.delta[dev * a.dev_vec + (long long)mat * s + qrow] = delta;
}

// ---------------------------------------------------------------- backward, dK and dV
// A wavefront owns 32 keys and every second block of 64 queries (from the diagonal on when causal).
// lds: [stage][Q, dO][pair tile]; ldsL: lse * log2(e) of the pair's queries; ldsD: their rowsum(dO * O).
template <int D, bool CAUSAL, int NRG>
__device__ __forceinline__ void bwd_dkv_body(const FusedArgs& a, bf16_t (*lds)[2][PAIR * D], float (*ldsL)[PAIR], float (*ldsD)[PAIR],
                                             int tile, int mat, int dev) {
  constexpr int KS = D / 16, DT = D / 32, BKW = NRG * 32;
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int rg = wave % NRG, par = wave / NRG;
  const int s = a.s;
  const int seq = mat / a.nh, head = mat % a.nh;
  const bf16_t* Qp = a.qkv + dev * a.dev_qkv + (long long)seq * s * a.ld + head * 3 * D;
  const bf16_t* Kp = Qp + D;
  const bf16_t* Vp = Qp + 2 * D;
  const bf16_t* Gp = a.d_attn + dev * a.dev_attn + (long long)seq * s * a.ldo + head * D;
  const float* Lp = a.lse + dev * a.dev_vec + (long long)mat * s;
  const float* Dp = a.delta + dev * a.dev_vec + (long long)mat * s;
  const int k0 = tile * BKW + rg * 32;
  const int key = k0 + (lane & 31);
  const int krow = min(key, s - 1);
  bf16x8 kf[KS], vf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    kf[ks] = *(const bf16x8*)(Kp + (long long)krow * a.ld + ks * 16 + g * 8);
    vf[ks] = *(const bf16x8*)(Vp + (long long)krow * a.ld + ks * 16 + g * 8);
  }
  const int nqb = (s + BLK - 1) / BLK;
  const int qb_lo = CAUSAL ? (tile * BKW) / BLK : 0;  // first block with a query >= the workgroup's first key
  const int n_it = (nqb - qb_lo + 1) / 2;
  const bool wave_valid = k0 < s;

  f32x16 dkacc[DT], dvacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) {
    dkacc[dt] = zero16();
    dvacc[dt] = zero16();
  }
  PairLoader<D, 2 * NRG> ldq, ldg;
  ldq.init(a.ld, wave, lane);
  ldg.init(a.ldo, wave, lane);
  auto load_pair = [&](int it, int st) {
    const int row0 = (qb_lo + 2 * it) * BLK;
    ldq.issue(Qp, row0, s, lds[st][0]);
    ldg.issue(Gp, row0, s, lds[st][1]);
    if (tid < PAIR) {
      const int row = min(row0 + tid, s - 1);
      ldsL[st][tid] = Lp[row] * LOG2E;
      ldsD[st][tid] = Dp[row];
    }
  };
  load_pair(0, 0);
  wait_loads_and_barrier();
  for (int it = 0; it < n_it; ++it) {
    const int st = it & 1;
    if (it + 1 < n_it) load_pair(it + 1, st ^ 1);
    const int qb = qb_lo + 2 * it + par;
    if (wave_valid && qb < nqb) {
      const bf16_t* tQ = lds[st][0] + par * BLK * D;
      const bf16_t* tG = lds[st][1] + par * BLK * D;
      const float* tL = ldsL[st] + par * BLK;
      const float* tD = ldsD[st] + par * BLK;
      const int qbase = qb * BLK;
      f32x16 sacc[2], pacc[2];
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        sacc[t2] = zero16();
        pacc[t2] = zero16();
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          sacc[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<D>(tQ, t2 * 32, ks, lane), kf[ks], sacc[t2], 0, 0, 0);
          pacc[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<D>(tG, t2 * 32, ks, lane), vf[ks], pacc[t2], 0, 0, 0);
        }
      }
      // masked: queries before the key (causal, only in the block on the diagonal) and padding queries
      const bool need_mask = (CAUSAL && qbase < k0 + 31) || (qbase + BLK > s);
      bf16x8 pf[2][2], dsf[2][2];
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int qi = t2 * 32 + 8 * c + 4 * g;
          const float4 l4 = *(const float4*)(tL + qi);
          const float4 d4 = *(const float4*)(tD + qi);
          const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int r = 4 * c + e;
            const int qy = qbase + qi + e;
            float p = __builtin_amdgcn_exp2f(fmaf(sacc[t2][r], a.scale_log2, -lv[e]));
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
      for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) {
            dvacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_acc_order<D>(tG, t2 * 32 + u * 16, dt * 32, lane),
                                                                pf[t2][u], dvacc[dt], 0, 0, 0);
            dkacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_acc_order<D>(tQ, t2 * 32 + u * 16, dt * 32, lane),
                                                                dsf[t2][u], dkacc[dt], 0, 0, 0);
          }
    }
    wait_loads_and_barrier();
  }
  float* xch = (float*)&lds[0][0][0] + rg * (2 * DT * 16) * 64;
  if (par == 1) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        xch[(dt * 16 + r) * 64 + lane] = dkacc[dt][r];
        xch[((DT + dt) * 16 + r) * 64 + lane] = dvacc[dt][r];
      }
  }
  __syncthreads();
  if (par == 0 && key < s) {
    bf16_t* dKp = a.d_qkv + dev * a.dev_qkv + ((long long)seq * s + key) * a.ld + head * 3 * D + D;
    bf16_t* dVp = dKp + D;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        float k4[4], v4[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          k4[e] = (dkacc[dt][4 * c + e] + xch[(dt * 16 + 4 * c + e) * 64 + lane]) * a.scale;
          v4[e] = dvacc[dt][4 * c + e] + xch[((DT + dt) * 16 + 4 * c + e) * 64 + lane];
        }
        u32x2 wk = {pack2_bf16(k4[0], k4[1]), pack2_bf16(k4[2], k4[3])};
        u32x2 wv = {pack2_bf16(v4[0], v4[1]), pack2_bf16(v4[2], v4[3])};
        *(u32x2*)(dKp + dt * 32 + 8 * c + 4 * g) = wk;
        *(u32x2*)(dVp + dt * 32 + 8 * c + 4 * g) = wv;
      }
  }
}

template <int D, bool CAUSAL, int NRG>
__global__ __launch_bounds__(NRG * 128) void attn_fused_bwd_dkv_kernel(FusedArgs a) {
  __shared__ __attribute__((aligned(1024))) bf16_t lds[2][2][PAIR * D];
  __shared__ __attribute__((aligned(16))) float ldsL[2][PAIR];
  __shared__ __attribute__((aligned(16))) float ldsD[2][PAIR];
  bwd_dkv_body<D, CAUSAL, NRG>(a, lds, ldsL, ldsD, blockIdx.x, blockIdx.y, blockIdx.z);  // early key tiles: longest causal loops
}

// dQ and dK/dV of one launch side by side.  A causal launch of either kernel alone is as long as its longest row or
// column tile while the average tile is half as long, and one workgroup fills a compute unit (registers), so with
// about one workgroup per compute unit half the chip idles.  Here the workgroups of both are one grid, ordered by loop
// length (longest first, the two kinds alternating): a compute unit that finishes a short tile picks up the next one
// of either kind.  rowsum(dO * O) comes from attn_fused_delta_kernel (launched before), so no workgroup waits for
// another.  Same arithmetic per workgroup as the two separate kernels: same bits.
template <int D, bool CAUSAL>
__global__ __launch_bounds__(256) void attn_fused_bwd_kernel(FusedArgs a, int ntiles, int nmat) {
  __shared__ __attribute__((aligned(1024))) bf16_t lds[2][2][PAIR * D];
  __shared__ __attribute__((aligned(16))) float ldsL[2][PAIR];
  __shared__ __attribute__((aligned(16))) float ldsD[2][PAIR];
  const unsigned per_rank = 2u * (unsigned)nmat;   // grid: x = (rank of the loop length, matrix, kind), y = device
  const unsigned rank = blockIdx.x / per_rank, rem = blockIdx.x % per_rank;
  const int mat = (int)(rem >> 1), dev = (int)blockIdx.y;
  if (rem & 1) bwd_dq_body<D, CAUSAL, 2, false>(a, lds, ntiles - 1 - (int)rank, mat, dev);
  else bwd_dkv_body<D, CAUSAL, 2>(a, lds, ldsL, ldsD, (int)rank, mat, dev);
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
  if ((long long)PAIR * d.ld * 2 >= (1ll << 31)) return false;  // per-lane byte offsets inside a pair tile are 32-bit
  return true;
}

template <int D>
void fwd_launch(const FusedArgs& a, const AttnFusedDesc& d, hipStream_t st) {
  // 128-row workgroups from one per two compute units on (measured: equal or faster than 64-row ones from there)
  const bool big = (long long)((d.s + 127) / 128) * d.nb * d.nh * d.ndev >= 128;
  if (big) {
    const dim3 grid((d.s + 127) / 128, d.nb * d.nh, d.ndev), block(512);
    if (d.causal) attn_fused_fwd_kernel<D, true, 4><<<grid, block, 0, st>>>(a);
    else attn_fused_fwd_kernel<D, false, 4><<<grid, block, 0, st>>>(a);
  } else {
    const dim3 grid((d.s + BLK - 1) / BLK, d.nb * d.nh, d.ndev), block(256);
    if (d.causal) attn_fused_fwd_kernel<D, true, 2><<<grid, block, 0, st>>>(a);
    else attn_fused_fwd_kernel<D, false, 2><<<grid, block, 0, st>>>(a);
  }
}
template <int D, bool CAUSAL>
void bwd_launch_c(const FusedArgs& a, const AttnFusedDesc& d, hipStream_t st) {
  const dim3 grid((d.s + BLK - 1) / BLK, d.nb * d.nh, d.ndev), block(NWAVES * 64);
  // 128-row workgroups of eight wavefronts for big launches, where the kernel fits 256 registers per lane (the dK/dV
  // kernel at head width 128 does not: it would spill a hundred registers)
  const bool big = (long long)((d.s + 127) / 128) * d.nb * d.nh * d.ndev >= 512;
  const dim3 grid_big((d.s + 127) / 128, d.nb * d.nh, d.ndev), block_big(512);
  const long long ntiles = (d.s + BLK - 1) / BLK, nmat = (long long)d.nb * d.nh;
  if (!big && 2 * ntiles * nmat < (1ll << 30)) {
    // small launches (about a workgroup per compute unit or less): both kinds of workgroup in one grid
    attn_fused_delta_kernel<D><<<dim3((d.s + 127) / 128, d.nb * d.nh, d.ndev), 256, 0, st>>>(a);
    attn_fused_bwd_kernel<D, CAUSAL><<<dim3((unsigned)(2 * ntiles * nmat), d.ndev), 256, 0, st>>>(a, (int)ntiles, (int)nmat);
    return;
  }
  if (big) attn_fused_bwd_dq_kernel<D, CAUSAL, 4><<<grid_big, block_big, 0, st>>>(a);
  else attn_fused_bwd_dq_kernel<D, CAUSAL, 2><<<grid, block, 0, st>>>(a);
  if constexpr (D == 64) {
    if (big) {
      attn_fused_bwd_dkv_kernel<D, CAUSAL, 4><<<grid_big, block_big, 0, st>>>(a);
      return;
    }
  }
  attn_fused_bwd_dkv_kernel<D, CAUSAL, 2><<<grid, block, 0, st>>>(a);
}
template <int D>
void bwd_launch(const FusedArgs& a, const AttnFusedDesc& d, hipStream_t st) {
  if (d.causal) bwd_launch_c<D, true>(a, d, st);
  else bwd_launch_c<D, false>(a, d, st);
}

}  // namespace

bool attn_fused_supported(int d) { return d == 64 || d == 128; }

int launch_attn_fused_fwd(const AttnFusedDesc& d, hipStream_t st) {
  if (!desc_ok(d) || !d.qkv || !d.attn || !d.lse) return OPTIMUS_ESHAPE;
  const FusedArgs a = make_args(d);
  if (d.d == 64) fwd_launch<64>(a, d, st);
  else fwd_launch<128>(a, d, st);
  return hip_launch_status();
}

int launch_attn_fused_bwd(const AttnFusedDesc& d, hipStream_t st) {
  if (!desc_ok(d) || !d.qkv || !d.attn || !d.lse || !d.d_attn || !d.d_qkv || !d.delta) return OPTIMUS_ESHAPE;
  const FusedArgs a = make_args(d);
  if (d.d == 64) bwd_launch<64>(a, d, st);
  else bwd_launch<128>(a, d, st);
  return hip_launch_status();
}

}  // namespace optimus

// bf16 matrix-core product kernel for gfx950 (CDNA4).
//
// Computes, per batch entry, C = alpha * sum_{l<nl} op(A_l) * op(B_l) with fp32 accumulation in
// v_mfma_f32_32x32x16_bf16 and applies the epilogue once.  The nl panels of a SUMMA product
// (Algorithms 1-3 of the paper: one panel per step l) are consumed by ONE k-loop that re-bases
// the operand pointers at panel boundaries, so the q steps cost nothing beyond pointer
// arithmetic and no partial C ever goes to HBM (unless the caller asked for a panel split).
//
// Tiling: a workgroup of WM*WN wavefronts owns a BM x BN output tile; k advances in slabs of
// BK = 64.  Slabs go global -> registers -> LDS (double buffered, one barrier per slab).
//   * k-contiguous operands ([rows][k] in memory) are stored as rows of 8 sixteen-byte chunks,
//     chunk index XOR-ed with (row & 7) so that the 32 lanes of a fragment read hit all banks.
//   * k-strided operands ([k][cols] in memory: B of A*B, both operands of A^T*B) are stored
//     as they are, rows padded by 16 elements, and fetched with the transposing LDS read
//     ds_read_b64_tr_b16, which hands each lane four consecutive k of one column.
// The two MFMA operands are swapped (D^T = B^T A^T) so that every lane ends up with four
// consecutive columns of one output row: 8-byte bf16 stores, and vector loads of the residual.
#include "common.hpp"
#include "epilogue.hpp"

namespace optimus {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

static int g_variant = -1;
void gemm_set_variant(int v) { g_variant = v; }
int gemm_get_variant() { return g_variant; }

constexpr int BK = 64;
constexpr int PAD = 16;  // elements of row padding for k-strided LDS tiles

struct KArgs {
  const bf16_t* A;
  const bf16_t* B;
  int Mb, Nb, Kp, nl;
  int lda, ldb;
  long long sAl, sBl;
  int nz0;
  long long sA0, sA1, sB0, sB1, sC0, sC1;
  long long sBias0;
  int tiles_m, tiles_n;
  int skip_upper, k_hi_diag, k_lo_diag;
  int splits;
  float* partials;
  long long nz;  // total batch count
  EpiArgs epi;
};

template <int ROWS, bool KC>
struct TileLds {
  // KC: [ROWS][64] swizzled; else [64][ROWS + PAD]
  static constexpr int elems = KC ? ROWS * BK : BK * (ROWS + PAD);
};

// ---- global -> register staging of one operand slab ----
template <int ROWS, int THREADS>
struct StageDims {
  static constexpr int CHUNKS = ROWS * BK / 8;  // 16-byte chunks in a slab
  static constexpr int PER = CHUNKS / THREADS;
  static_assert(CHUNKS % THREADS == 0, "slab must divide over the workgroup");
};

// base: panel base already offset to this tile's first row/col; ld: leading dimension;
// rows_left: valid rows (m or n) from the tile origin; k_left: valid k from the slab origin
template <int ROWS, bool KC, int THREADS, bool GUARD, int PER>
__device__ __forceinline__ void stage_load(u32x4 (&r)[PER], const bf16_t* base, int ld, int k0, int rows_left, int k_left,
                                           int tid) {
  static_assert(PER == StageDims<ROWS, THREADS>::PER, "staging array size");
#pragma unroll
  for (int it = 0; it < PER; ++it) {
    const int c = tid + it * THREADS;
    if (KC) {
      const int row = c >> 3, kc = c & 7;
      const bf16_t* p = base + (long long)row * ld + k0 + kc * 8;
      if (!GUARD || (row < rows_left && kc * 8 < k_left)) r[it] = *(const u32x4*)p;
      else r[it] = u32x4{0u, 0u, 0u, 0u};
    } else {
      constexpr int CPR = ROWS / 8;
      const int krow = c / CPR, mc = c % CPR;
      const bf16_t* p = base + (long long)(k0 + krow) * ld + mc * 8;
      if (!GUARD || (krow < k_left && mc * 8 < rows_left)) r[it] = *(const u32x4*)p;
      else r[it] = u32x4{0u, 0u, 0u, 0u};
    }
  }
}
template <int ROWS, bool KC, int THREADS, int PER>
__device__ __forceinline__ void stage_store(const u32x4 (&r)[PER], bf16_t* lds, int tid) {
  static_assert(PER == StageDims<ROWS, THREADS>::PER, "staging array size");
#pragma unroll
  for (int it = 0; it < PER; ++it) {
    const int c = tid + it * THREADS;
    if (KC) {
      const int row = c >> 3, kc = c & 7;
      *(u32x4*)(lds + row * BK + ((kc ^ (row & 7)) << 3)) = r[it];
    } else {
      constexpr int CPR = ROWS / 8;
      const int krow = c / CPR, mc = c % CPR;
      *(u32x4*)(lds + krow * (ROWS + PAD) + mc * 8) = r[it];
    }
  }
}

// fragment of 8 consecutive k for row/col (rc0 + lane%32), k-group lane/32, sub-step ks
template <int ROWS, bool KC>
__device__ __forceinline__ bf16x8 read_frag(const bf16_t* lds, int rc0, int ks, int lane) {
  if (KC) {
    int row = rc0 + (lane & 31);
    int chunk = ks * 2 + (lane >> 5);
    return *(const bf16x8*)(lds + row * BK + ((chunk ^ (row & 7)) << 3));
  } else {
    int lg = lane & 15;
    int col = rc0 + (((lane >> 4) & 1) << 4) + ((lg & 3) << 2);
    int krow = ks * 16 + ((lane >> 5) << 3) + (lg >> 2);
    const bf16_t* p0 = lds + krow * (ROWS + PAD) + col;
    const bf16_t* p1 = p0 + 4 * (ROWS + PAD);
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p0);
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p1);
    s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
  }
}

template <int BM, int BN, int WM, int WN, bool AKC, bool BKC, bool GUARD>
__global__ __launch_bounds__(WM* WN * 64) void gemm_mfma_kernel(const KArgs a) {
  constexpr int THREADS = WM * WN * 64;
  constexpr int TM = BM / WM, TN = BN / WN;
  constexpr int MI = TM / 32, NI = TN / 32;
  constexpr int A_ELEMS = TileLds<BM, AKC>::elems;
  constexpr int B_ELEMS = TileLds<BN, BKC>::elems;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* smem = (bf16_t*)smem_raw;
  constexpr int STAGE = A_ELEMS + B_ELEMS;  // stage s: A at smem + s*STAGE, B right after it

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

  // ---- which tile: XCD-aware remap of the linear workgroup id ----
  // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of tiles so that
  // neighbours sharing A rows / B columns also share an L2.
  long long nwg = (long long)gridDim.x;
  long long wg = blockIdx.x;
  {
    long long per = nwg >> 3, rem = nwg & 7;
    long long xcd = wg & 7, slot = wg >> 3;
    // XCDs 0..rem-1 own per+1 workgroups, the rest own per
    long long start = xcd * per + (xcd < rem ? xcd : rem);
    wg = start + slot;
  }
  const int split = (int)(wg % a.splits);
  wg /= a.splits;
  const int tiles = a.tiles_m * a.tiles_n;
  const long long z = wg / tiles;
  int t = (int)(wg % tiles);
  // column-major walk within groups of 8 tile rows keeps the working set of an XCD compact
  int tm, tn;
  {
    constexpr int GROUP = 8;
    int per_group = GROUP * a.tiles_n;
    int g = t / per_group;
    int first = g * GROUP;
    int gsz = min(GROUP, a.tiles_m - first);
    int r = t - g * per_group;
    tm = first + r % gsz;
    tn = r / gsz;
  }
  const int m0 = tm * BM, n0 = tn * BN;
  if (a.skip_upper && n0 > m0 + BM - 1) return;

  const int z1 = (int)(z / a.nz0), z0 = (int)(z % a.nz0);
  const bf16_t* Az = a.A + z1 * a.sA1 + z0 * a.sA0;
  const bf16_t* Bz = a.B + z1 * a.sB1 + z0 * a.sB0;

  // ---- k range in slabs, over all panels ----
  const int tpp = (a.Kp + BK - 1) / BK;
  int t_lo = 0, t_hi = a.nl * tpp;
  if (a.k_lo_diag) t_lo = m0 / BK;
  if (a.k_hi_diag) t_hi = min(t_hi, (min(a.Kp, m0 + BM) + BK - 1) / BK);
  if (a.splits > 1) {
    int total = t_hi - t_lo;
    int per = (total + a.splits - 1) / a.splits;
    int lo = t_lo + split * per;
    t_hi = min(t_hi, lo + per);
    t_lo = lo;
  }

  f32x16 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[mi][ni][e] = 0.f;

  u32x4 ra[StageDims<BM, THREADS>::PER];
  u32x4 rb[StageDims<BN, THREADS>::PER];
  const bf16_t* Atile = Az + (AKC ? (long long)m0 * a.lda : (long long)m0);
  const bf16_t* Btile = Bz + (BKC ? (long long)n0 * a.ldb : (long long)n0);
  const int rowsA = a.Mb - m0, rowsB = a.Nb - n0;

  if (t_lo < t_hi) {
    // slab index -> (panel l, offset k0 inside the panel); advanced incrementally, no division in the loop
    int l = t_lo / tpp, k0 = (t_lo - l * tpp) * BK;
    stage_load<BM, AKC, THREADS, GUARD>(ra, Atile + l * a.sAl, a.lda, k0, rowsA, a.Kp - k0, tid);
    stage_load<BN, BKC, THREADS, GUARD>(rb, Btile + l * a.sBl, a.ldb, k0, rowsB, a.Kp - k0, tid);
    stage_store<BM, AKC, THREADS>(ra, smem, tid);
    stage_store<BN, BKC, THREADS>(rb, smem + A_ELEMS, tid);
    __syncthreads();
    for (int tt = t_lo; tt < t_hi; ++tt) {
      const int cur = (tt - t_lo) & 1;
      const bool more = tt + 1 < t_hi;
      if (more) {
        k0 += BK;
        if (k0 >= a.Kp) { k0 = 0; ++l; }
        stage_load<BM, AKC, THREADS, GUARD>(ra, Atile + l * a.sAl, a.lda, k0, rowsA, a.Kp - k0, tid);
        stage_load<BN, BKC, THREADS, GUARD>(rb, Btile + l * a.sBl, a.ldb, k0, rowsB, a.Kp - k0, tid);
      }
      const bf16_t* la = smem + cur * STAGE;
      const bf16_t* lb = la + A_ELEMS;
#pragma unroll
      for (int ks = 0; ks < BK / 16; ++ks) {
        bf16x8 af[MI], bfg[NI];
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) af[mi] = read_frag<BM, AKC>(la, wm * TM + mi * 32, ks, lane);
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) bfg[ni] = read_frag<BN, BKC>(lb, wn * TN + ni * 32, ks, lane);
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
          for (int ni = 0; ni < NI; ++ni)
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfg[ni], af[mi], acc[mi][ni], 0, 0, 0);
      }
      if (more) {
        stage_store<BM, AKC, THREADS>(ra, smem + (cur ^ 1) * STAGE, tid);
        stage_store<BN, BKC, THREADS>(rb, smem + (cur ^ 1) * STAGE + A_ELEMS, tid);
      }
      __syncthreads();
    }
  }

  // ---- epilogue: lane holds row (lane%32), columns 8*g + 4*(lane/32) + 0..3 of each 32x32 tile ----
  if (a.splits > 1) {
    // raw fp32 partial tile; the combine kernel adds the splits in order and applies the epilogue
    float* P = a.partials + ((long long)split * a.nz + z) * (long long)a.Mb * a.Nb;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          int m = m0 + wm * TM + mi * 32 + (lane & 31);
          int n = n0 + wn * TN + ni * 32 + g * 8 + ((lane >> 5) << 2);
          if (GUARD && (m >= a.Mb || n >= a.Nb)) continue;
          float* p = P + (long long)m * a.Nb + n;
          if (!GUARD || n + 3 < a.Nb) {
            *(float4*)p = make_float4(acc[mi][ni][g * 4], acc[mi][ni][g * 4 + 1], acc[mi][ni][g * 4 + 2], acc[mi][ni][g * 4 + 3]);
          } else {
            for (int c = 0; c < 4 && n + c < a.Nb; ++c) p[c] = acc[mi][ni][g * 4 + c];
          }
        }
    return;
  }
  EpiArgs e = a.epi;
  if (e.bias) e.bias += z0 * a.sBias0;
  const long long coff = z1 * a.sC1 + z0 * a.sC0;
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        int m = m0 + wm * TM + mi * 32 + (lane & 31);
        int n = n0 + wn * TN + ni * 32 + g * 8 + ((lane >> 5) << 2);
        if (GUARD && (m >= a.Mb || n >= a.Nb)) continue;
        float v[4] = {acc[mi][ni][g * 4], acc[mi][ni][g * 4 + 1], acc[mi][ni][g * 4 + 2], acc[mi][ni][g * 4 + 3]};
        int nvalid = GUARD ? min(4, a.Nb - n) : 4;
        epilogue_store4(e, coff, m, n, v, nvalid);
      }
}

// ---- fixed-order combine of panel-split partials + epilogue ----
__global__ __launch_bounds__(256) void gemm_combine_kernel(const float* partials, int splits, long long nz, int Mb, int Nb,
                                                           int nz0, long long sC0, long long sC1, long long sBias0,
                                                           EpiArgs e) {
  long long quads_per_row = (Nb + 3) / 4;
  long long total = nz * Mb * quads_per_row;
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  int nq = (int)(idx % quads_per_row);
  long long r = idx / quads_per_row;
  int m = (int)(r % Mb);
  long long z = r / Mb;
  int n = nq * 4;
  int nvalid = min(4, Nb - n);
  float v[4] = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < splits; ++s) {
    const float* p = partials + ((long long)s * nz + z) * (long long)Mb * Nb + (long long)m * Nb + n;
    for (int c = 0; c < nvalid; ++c) v[c] += p[c];
  }
  int z1 = (int)(z / nz0), z0 = (int)(z % nz0);
  if (e.bias) e.bias += z0 * sBias0;
  epilogue_store4(e, z1 * sC1 + z0 * sC0, m, n, v, nvalid);
}

// ---- host side ----
struct Variant {
  int BM, BN, WM, WN;
};
// index = variant id used by gemm_set_variant
static const Variant kVariants[] = {
    {256, 256, 2, 2},  // 0
    {256, 128, 2, 2},  // 1
    {128, 256, 2, 2},  // 2
    {128, 128, 2, 2},  // 3
    {256, 256, 2, 4},  // 4: 8 waves
    {128, 128, 2, 2},  // 5: guarded (ragged shapes)
};
constexpr int kNumVariants = 6;
constexpr int kGuardVariant = 5;

template <int BM, int BN, int WM, int WN, bool AKC, bool BKC, bool GUARD>
static int launch_one(const KArgs& ka, long long nwg, hipStream_t stream) {
  constexpr size_t lds = 2 * (size_t)(TileLds<BM, AKC>::elems + TileLds<BN, BKC>::elems) * sizeof(bf16_t);
  auto kern = gemm_mfma_kernel<BM, BN, WM, WN, AKC, BKC, GUARD>;
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
      (void)hipGetLastError();
      return OPTIMUS_EHIP;
    }
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(WM * WN * 64), lds, stream, ka);
  return hip_launch_status();
}

template <int BM, int BN, int WM, int WN, bool GUARD>
static int launch_layout(const GemmDesc& d, const KArgs& ka, long long nwg, hipStream_t stream) {
  if (d.a_kcontig && !d.b_kcontig) return launch_one<BM, BN, WM, WN, true, false, GUARD>(ka, nwg, stream);
  if (d.a_kcontig && d.b_kcontig) return launch_one<BM, BN, WM, WN, true, true, GUARD>(ka, nwg, stream);
  if (!d.a_kcontig && !d.b_kcontig) return launch_one<BM, BN, WM, WN, false, false, GUARD>(ka, nwg, stream);
  return OPTIMUS_EINVAL;  // [K][M] x [N][K] does not occur in the method
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

bool gemm_mfma_supported(const GemmDesc& d) {
  if (d.dtype != OPTIMUS_BF16) return false;
  if (!d.a_kcontig && d.b_kcontig) return false;
  if (!aligned16(d.A) || !aligned16(d.B)) return false;
  // every 16-byte chunk must be fully inside or fully outside the operand, and aligned
  if (d.lda % 8 || d.ldb % 8) return false;
  if (d.sAl % 8 || d.sBl % 8 || d.sA0 % 8 || d.sA1 % 8 || d.sB0 % 8 || d.sB1 % 8) return false;
  if (d.a_kcontig ? (d.Kp % 8) : (d.Mb % 8)) return false;
  if (d.b_kcontig ? (d.Kp % 8) : (d.Nb % 8)) return false;
  return true;
}

static bool variant_fits(const Variant& v, const GemmDesc& d) {
  return d.Mb % v.BM == 0 && d.Nb % v.BN == 0 && d.Kp % BK == 0;
}

static int pick_variant(const GemmDesc& d) {
  if (g_variant >= 0 && g_variant < kNumVariants) {
    if (g_variant == kGuardVariant || variant_fits(kVariants[g_variant], d)) return g_variant;
  }
  // estimated cost = rounds of tiles over 256 CUs * (tile area / relative efficiency)
  static const float eff[4] = {1.0f, 0.85f, 0.85f, 0.7f};
  long long nz = (long long)d.nz0 * d.nz1;
  int best = -1;
  float best_cost = 0.f;
  for (int v = 0; v < 4; ++v) {
    if (!variant_fits(kVariants[v], d)) continue;
    long long tiles = (long long)(d.Mb / kVariants[v].BM) * (d.Nb / kVariants[v].BN) * nz * (d.splits > 1 ? d.splits : 1);
    long long rounds = (tiles + 255) / 256;
    float cost = (float)rounds * (float)(kVariants[v].BM * kVariants[v].BN) / eff[v];
    if (best < 0 || cost < best_cost) {
      best = v;
      best_cost = cost;
    }
  }
  return best >= 0 ? best : kGuardVariant;
}

size_t gemm_partials_bytes(const GemmDesc& d, int splits) {
  if (splits <= 1) return 0;
  return (size_t)splits * (size_t)d.nz0 * d.nz1 * (size_t)d.Mb * d.Nb * sizeof(float);
}

int gemm_pick_splits(const GemmDesc& d) {
  // only plain multi-panel products with few output tiles and a long contraction benefit
  if (d.dtype != OPTIMUS_BF16 || d.nl < 2 || d.skip_upper || d.k_hi_diag || d.k_lo_diag) return 1;
  long long nz = (long long)d.nz0 * d.nz1;
  long long tiles128 = (long long)((d.Mb + 127) / 128) * ((d.Nb + 127) / 128) * nz;
  if (tiles128 >= 192) return 1;
  long long slabs = (long long)d.nl * ((d.Kp + BK - 1) / BK);
  int s = 1;
  while (s * 2 <= d.nl && tiles128 * (s * 2) <= 512 && slabs / (s * 2) >= 8) s *= 2;
  return s;
}

int launch_gemm_mfma(const GemmDesc& d, hipStream_t stream) {
  if (!gemm_mfma_supported(d)) return OPTIMUS_EINVAL;
  int vi = pick_variant(d);
  const Variant& v = kVariants[vi];
  KArgs ka;
  ka.A = (const bf16_t*)d.A;
  ka.B = (const bf16_t*)d.B;
  ka.Mb = d.Mb; ka.Nb = d.Nb; ka.Kp = d.Kp; ka.nl = d.nl;
  ka.lda = d.lda; ka.ldb = d.ldb;
  ka.sAl = d.sAl; ka.sBl = d.sBl;
  ka.nz0 = d.nz0;
  ka.sA0 = d.sA0; ka.sA1 = d.sA1; ka.sB0 = d.sB0; ka.sB1 = d.sB1; ka.sC0 = d.sC0; ka.sC1 = d.sC1;
  ka.sBias0 = d.sBias0;
  ka.tiles_m = (d.Mb + v.BM - 1) / v.BM;
  ka.tiles_n = (d.Nb + v.BN - 1) / v.BN;
  ka.skip_upper = d.skip_upper; ka.k_hi_diag = d.k_hi_diag; ka.k_lo_diag = d.k_lo_diag;
  ka.splits = d.splits > 1 ? d.splits : 1;
  ka.partials = d.partials;
  ka.nz = (long long)d.nz0 * d.nz1;
  EpiArgs& e = ka.epi;
  e.alpha = d.alpha; e.bias = d.bias; e.C = d.C; e.pre_act = d.pre_act; e.gelu_grad_of = d.gelu_grad_of;
  e.residual = d.residual; e.ldc = d.ldc; e.act = d.act; e.out_fp32 = d.out_fp32; e.in_bf16 = 1;
  e.vec_ok = (d.ldc % 4 == 0) && (d.sC0 % 4 == 0) && (d.sC1 % 4 == 0) && aligned16(d.C) &&
             (!d.pre_act || aligned16(d.pre_act)) && (!d.gelu_grad_of || aligned16(d.gelu_grad_of)) &&
             (!d.residual || aligned16(d.residual));
  if (ka.splits > 1 && !d.partials) return OPTIMUS_EWORKSPACE;
  long long nwg = (long long)ka.tiles_m * ka.tiles_n * ka.nz * ka.splits;
  if (nwg <= 0 || nwg > 0x7fffffffLL) return OPTIMUS_ESHAPE;
  int rc;
  switch (vi) {
    case 0: rc = launch_layout<256, 256, 2, 2, false>(d, ka, nwg, stream); break;
    case 1: rc = launch_layout<256, 128, 2, 2, false>(d, ka, nwg, stream); break;
    case 2: rc = launch_layout<128, 256, 2, 2, false>(d, ka, nwg, stream); break;
    case 3: rc = launch_layout<128, 128, 2, 2, false>(d, ka, nwg, stream); break;
    case 4: rc = launch_layout<256, 256, 2, 4, false>(d, ka, nwg, stream); break;
    default: rc = launch_layout<128, 128, 2, 2, true>(d, ka, nwg, stream); break;
  }
  if (rc != OPTIMUS_OK) return rc;
  if (ka.splits > 1) {
    long long total = ka.nz * d.Mb * ((d.Nb + 3) / 4);
    long long blocks = (total + 255) / 256;
    hipLaunchKernelGGL(gemm_combine_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (const float*)d.partials,
                       ka.splits, ka.nz, d.Mb, d.Nb, d.nz0, d.sC0, d.sC1, d.sBias0, e);
    rc = hip_launch_status();
  }
  return rc;
}

}  // namespace optimus

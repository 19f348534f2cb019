// bf16 matrix-core product kernels for gfx950 (CDNA4).
//
// Computes, per batch entry, C = alpha * sum_{l<nl} op(A_l) * op(B_l) with fp32 accumulation in
// v_mfma_f32_32x32x16_bf16 and applies the epilogue once.  The nl panels of a SUMMA product
// (Algorithms 1-3 of the paper: one panel per step l) are consumed by ONE k-loop that re-bases
// the operand pointers at panel boundaries, so the q steps cost nothing beyond pointer
// arithmetic and no partial C ever goes to HBM (unless the caller asked for a panel split).
//
// Tiling: a workgroup of WM*WN wavefronts owns a BM x BN output tile; k advances in slabs of
// BK = 32 through a ring of FOUR slabs per operand in LDS.
//   * Full tiles (FAST): every wavefront issues buffer_load_dwordx4 ... lds, which moves 64 x 16
//     bytes from per-lane offsets straight into one contiguous KiB of LDS without passing
//     through registers.  The LDS swizzles below are therefore applied on the GLOBAL side:
//     lane p of a KiB fetches the 16 bytes that belong at LDS position p.  Buffer addressing
//     (SGPR resource + one 32-bit VGPR offset) is used because 64-bit per-lane addresses were
//     measured to stall the MFMA pipe twice as much.  Slab hand-over uses s_waitcnt vmcnt(N) and
//     a bare s_barrier: a fenced barrier would drain the loads in flight.
//     A k-strided operand moves one slab per step; a k-contiguous operand moves a PAIR of slabs
//     (64 k = one whole 128-byte line per row) every second step.  The pipeline runs over 16-wide
//     sub-steps with the fragments of the next sub-step requested between the MFMAs of the
//     current one, also across slab boundaries; the loads that refill a freed slab are spread one
//     by one between the MFMAs as well (see the comments at the loop).
//   * Ragged tiles: global -> registers (zero filled outside the operand) -> LDS, two stages.
// LDS layouts (conflict free for their readers on the 64-bank, 256 B/clk LDS of this part):
//   * k-contiguous operand ([rows][k] in memory), fast path: pairs of slabs as rows of 8
//     sixteen-byte chunks, chunk index XOR ((row >> 1) & 7); ragged path: rows of 4 chunks, chunk
//     XOR ((row >> 2) & 3); fragments are read with ds_read_b128.
//   * k-strided operand ([k][cols] in memory: B of A*B, both operands of A^T*B): kept as it is,
//     32-byte column granules XOR 2*(k & 3); fragments are fetched with the transposing read
//     ds_read_b64_tr_b16, which hands each lane four consecutive k of one column.
// The two MFMA operands are swapped (D^T = B^T A^T) so that every lane ends up with four
// consecutive columns of one output row; results leave through wavefront-private LDS chunks as
// whole rows of the tile (see ChunkBf16).
#include <atomic>
#include <type_traits>

#include "common.hpp"
#include "epilogue.hpp"

namespace optimus {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

// Tuning hooks of the benchmark and the tests (process-wide; atomics, so that a hook set from one thread while
// another launches is a race on WHICH setting a launch sees, never on memory).  They select tiles and the k-loop, and
// a forced tile plans its own panel split; nothing else in the library is process-global state.
static std::atomic<int> g_variant{-1};
static std::atomic<int> g_loop{2};   // k-loop of the fast path where both exist (see gemm_mfma_kernel); 1 or 2
void gemm_set_variant(int v) {
  // v >= 1000: the older k-loop with variant v - 1000 (1000 + 255 = automatic tile); otherwise the default k-loop
  if (v >= 1000) { g_loop = 1; v -= 1000; if (v == 255) v = -1; } else g_loop = 2;
  g_variant = v;
}
int gemm_get_variant() { return g_variant; }
static std::atomic<int> g_corun_variant[2] = {{-1}, {-1}};
void gemm_set_corun_variants(int chain_v, int branch_v) { g_corun_variant[0] = chain_v; g_corun_variant[1] = branch_v; }
static std::atomic<int> g_last_plan{-1};
int gemm_last_plan() { return g_last_plan; }


constexpr int BK = 32;
constexpr int NSTAGE = 4;
#ifndef OPTIMUS_LAB_DBG
#define OPTIMUS_LAB_DBG 0
#endif
// bit 32 (timing studies only): thread 0 of every workgroup stores the 100 MHz wall clock at four points of the kernel
// (entry, first matrix instruction, end of the k-loop, last store retired)
#if OPTIMUS_LAB_DBG & 32
__device__ unsigned long long g_lab_stamps[4 * 4096];
extern "C" int optimus_lab_read_stamps(unsigned long long* host) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_lab_stamps), sizeof(g_lab_stamps));
}
__device__ unsigned long long g_lab_stall[8 * 2048];
extern "C" int optimus_lab_read_stall(unsigned long long* host) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_lab_stall), sizeof(g_lab_stall));
}
#define OPTIMUS_LAB_STAMP(n)                                                                         \
  do {                                                                                               \
    if ((n) == 3) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                                   \
    if (threadIdx.x == 0 && blockIdx.x < 2048) {                                                      \
      g_lab_stamps[blockIdx.x * 8 + (n)] = wall_clock64();                                           \
      g_lab_stamps[blockIdx.x * 8 + 4 + (n)] = clock64();                                            \
    }                                                                                                \
  } while (0)
#else
#define OPTIMUS_LAB_STAMP(n) do {} while (0)
#endif

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
  int group;  // tile rows walked together (see the tile walk in the kernel)
  int skip_upper, k_hi_diag, k_lo_diag;
  int splits;
  float* partials;
  // > 1 (with splits == 1): one workgroup walks all slabs but adds them up as `seq_splits` panel-split workgroups and
  // their fixed-order combine would -- a fresh accumulator per range, the ranges' sums added in range order
  int seq_splits;
  long long nz;  // total batch count
  EpiArgs epi;
};

// element offset inside an LDS tile
// The LDS of this part serves 256 bytes per clock (64 four-byte banks).  A ds_read_b128 is served 16 lanes at a
// time (16 consecutive rows, one chunk each): four 64-byte rows span the 64 banks, so the XOR term must take 4
// distinct values over the 4 rows of equal (row & 3) -> (row >> 2) & 3.  A ds_read_b64_tr_b16 is served 32 lanes at
// a time (4 k-rows x two adjacent 32-byte granules): rows start at bank 0, so the 8 (k, granule) pairs must fall in
// 8 distinct granule slots -> XOR with 2 * (k & 3) (masked to the row's granule count for 64-wide tiles).  Measured with a read-only microbenchmark: > 200 B/clk for
// these patterns against 128 B/clk for swizzles designed for 32 banks.
__device__ __forceinline__ int lds_off_kc(int row, int chunk) { return row * BK + ((chunk ^ ((row >> 2) & 3)) << 3); }
// k-contiguous operand on the fast path: two slabs side by side, [row][64 k] = 128 bytes per row, so that one row
// of a load is a whole 128-byte cache line.  Two rows span the 64 banks: the XOR term takes 8 values over the 8 row
// pairs of a 16-lane group.
__device__ __forceinline__ int lds_off_kc2(int row, int chunk) { return row * (2 * BK) + ((chunk ^ ((row >> 1) & 7)) << 3); }
template <int ROWS>
__device__ __forceinline__ int lds_off_ks(int krow, int col) {
  return krow * ROWS + ((((col >> 4) ^ (((krow & 3) << 1) & (ROWS / 16 - 1)))) << 4) + (col & 15);
}

// ---- FAST path: direct global -> LDS, one KiB per wavefront instruction ----
template <int ROWS, int NW>
struct DirectPlan {
  static constexpr int CHUNKS = ROWS * BK * 2 / 1024;  // KiB chunks in a [ROWS x BK] bf16 slab
  static constexpr int PER = CHUNKS / NW;
  static_assert(CHUNKS % NW == 0 && PER >= 1, "slab must divide over the wavefronts");
};

// Per-lane source offsets (BYTES, relative to the slab origin) of the KiB chunks this wavefront moves.
// k-contiguous operand: the unit is a PAIR of slabs (64 k): 8 rows of 128 bytes per instruction.
// k-strided operand: the unit is one slab of 32 k-rows.
template <int ROWS, bool KC, int NW, int PER>
__device__ __forceinline__ void direct_offsets(unsigned (&off)[PER], int ld, int wave, int lane) {
#pragma unroll
  for (int it = 0; it < PER; ++it) {
    const int q = wave * PER + it;
    if (KC) {
      const int row = q * 8 + (lane >> 3);
      const int kc = (lane & 7) ^ ((row >> 1) & 7);  // inverse of lds_off_kc2 for LDS position (row, lane & 7)
      off[it] = (unsigned)(row * ld + kc * 8) * 2u;
    } else {
      constexpr int PPR = ROWS / 8;  // 16-byte pieces per k-row
      const int idx = q * 64 + lane;
      const int krow = idx / PPR, pp = idx % PPR;
      const int col = ((((pp >> 1) ^ (((krow & 3) << 1) & (ROWS / 16 - 1)))) << 4) + ((pp & 1) << 3);  // inverse of lds_off_ks
      off[it] = (unsigned)(krow * ld + col) * 2u;
    }
  }
}

typedef __attribute__((ext_vector_type(4))) int i32x4;

// Buffer resource (raw, stride 0) whose base is the current panel's tile origin, with a 2 GiB window: every offset
// used is below it (checked on the host).  Built by hand as four SGPR words.
__device__ __forceinline__ i32x4 make_rsrc(const bf16_t* base) {
  const unsigned long long p = (unsigned long long)base;
  return i32x4{(int)(unsigned)p, (int)(unsigned)((p >> 32) & 0xffffu), (int)0x80000000u, 0x00020000};
}

// rsrc: see make_rsrc; soff: byte offset of the slab inside the panel; off: per-lane byte offsets.
// The LDS load is written in assembly on purpose: issued through the compiler's builtin, every later LDS read is
// preceded by a compiler-inserted wait for ALL loads in flight (it cannot tell the stages apart), which collapses
// the four-stage pipeline to one slab.  Here the hand-over is explicit instead: s_waitcnt vmcnt(N) + barrier.
template <int ROWS, int NW, int PER>
__device__ __forceinline__ void direct_issue(i32x4 rsrc, unsigned soff, const unsigned (&off)[PER], bf16_t* lds_tile, int wave) {
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) bf16_t*)lds_tile;
#pragma unroll
  for (int it = 0; it < PER; ++it) {
    const unsigned m0v = __builtin_amdgcn_readfirstlane(lds_base + (unsigned)(wave * PER + it) * 1024u);
    asm volatile("s_mov_b32 m0, %3\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %1, %2 offen lds" ::"v"(off[it]), "s"(rsrc), "s"(soff), "s"(m0v)
                 : "memory", "m0");
  }
}

// one KiB chunk (number c of the operand's issue unit) with this lane's offset
__device__ __forceinline__ void direct_issue_one(i32x4 rsrc, unsigned soff, unsigned off, bf16_t* lds_unit, int c) {
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) bf16_t*)lds_unit;
  const unsigned m0v = __builtin_amdgcn_readfirstlane(lds_base + (unsigned)c * 1024u);
  asm volatile("s_mov_b32 m0, %3\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %1, %2 offen lds" ::"v"(off), "s"(rsrc), "s"(soff), "s"(m0v)
               : "memory", "m0");
}

// s_waitcnt vmcnt(n) only (expcnt / lgkmcnt left at their maxima), gfx9 encoding.  The builtin rather than inline
// assembly: the compiler's own wait-count pass then knows which LDS loads have landed and adds no full drain.
constexpr int waitcnt_vm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }
constexpr int waitcnt_vm_lgkm0(int n) { return (n & 15) | (7 << 4) | (0 << 8) | ((n >> 4) << 14); }  // + lgkmcnt(0)
#define OPTIMUS_WAIT_VMCNT_LGKM0(n)                      \
  do {                                                   \
    asm volatile("" ::: "memory");                       \
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(n));     \
    asm volatile("" ::: "memory");                       \
  } while (0)
#define OPTIMUS_WAIT_VMCNT(n)                      \
  do {                                             \
    asm volatile("" ::: "memory");                 \
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(n));     \
    asm volatile("" ::: "memory");                 \
  } while (0)
// barrier without the memory fence of __syncthreads(): loads of later slabs stay in flight across it
#define OPTIMUS_BARRIER()                  \
  do {                                     \
    asm volatile("" ::: "memory");         \
    __builtin_amdgcn_s_barrier();          \
    asm volatile("" ::: "memory");         \
  } while (0)

// ---- ragged path: global -> registers -> LDS ----
template <int ROWS, int THREADS>
struct StageDims {
  static constexpr int CHUNKS = ROWS * BK / 8;  // 16-byte chunks in a slab
  static constexpr int PER = CHUNKS / THREADS;
  static_assert(CHUNKS % THREADS == 0, "slab must divide over the workgroup");
};

// base: panel base already offset to this tile's first row/col; rows_left: valid rows (m or n) from the tile
// origin; k_left: valid k from the slab origin
template <int ROWS, bool KC, int THREADS, int PER>
__device__ __forceinline__ void stage_load(u32x4 (&r)[PER], const bf16_t* base, int ld, int k0, int rows_left, int k_left,
                                           int tid) {
  static_assert(PER == StageDims<ROWS, THREADS>::PER, "staging array size");
#pragma unroll
  for (int it = 0; it < PER; ++it) {
    const int c = tid + it * THREADS;
    if (KC) {
      const int row = c / (BK / 8), kc = c % (BK / 8);
      const bf16_t* p = base + (long long)row * ld + k0 + kc * 8;
      if (row < rows_left && kc * 8 < k_left) r[it] = *(const u32x4*)p;
      else r[it] = u32x4{0u, 0u, 0u, 0u};
    } else {
      constexpr int CPR = ROWS / 8;
      const int krow = c / CPR, mc = c % CPR;
      const bf16_t* p = base + (long long)(k0 + krow) * ld + mc * 8;
      if (krow < k_left && mc * 8 < rows_left) r[it] = *(const u32x4*)p;
      else r[it] = u32x4{0u, 0u, 0u, 0u};
    }
  }
}
template <int ROWS, bool KC, int THREADS, int PER>
__device__ __forceinline__ void stage_store(const u32x4 (&r)[PER], bf16_t* lds, int tid) {
#pragma unroll
  for (int it = 0; it < PER; ++it) {
    const int c = tid + it * THREADS;
    if (KC) {
      *(u32x4*)(lds + lds_off_kc(c / (BK / 8), c % (BK / 8))) = r[it];
    } else {
      constexpr int CPR = ROWS / 8;
      *(u32x4*)(lds + lds_off_ks<ROWS>(c / CPR, (c % CPR) * 8)) = r[it];
    }
  }
}

// fragment of 8 consecutive k for row/col (rc0 + lane%32), k-group lane/32, sub-step ks
template <int ROWS, bool KC>
__device__ __forceinline__ bf16x8 read_frag(const bf16_t* lds, int rc0, int ks, int lane) {
  if (KC) {
    return *(const bf16x8*)(lds + lds_off_kc(rc0 + (lane & 31), ks * 2 + (lane >> 5)));
  } else {
    const int lg = lane & 15;
    const int col = rc0 + (((lane >> 4) & 1) << 4) + ((lg & 3) << 2);
    const int krow = ks * 16 + ((lane >> 5) << 3) + (lg >> 2);
    const bf16_t* p0 = lds + lds_off_ks<ROWS>(krow, col);
    const bf16_t* p1 = p0 + 4 * ROWS;  // krow + 4: same (k & 3), same swizzle term
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p0);
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p1);
    s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
  }
}

template <int BM, int BN, int WM, int WN>
struct Tile {
  static constexpr int NW = WM * WN, THREADS = NW * 64;
  static constexpr int TM = BM / WM, TN = BN / WN, MI = TM / 32, NI = TN / 32;
  static constexpr int A_ELEMS = BM * BK, B_ELEMS = BN * BK;
};

// Instruction-order hint for one sub-step: spread the DS fragment reads of the NEXT sub-step between the first
// MFMAs of the current one (PER reads, one MFMA, ...), then the remaining MFMAs.  Masks: 0x100 DS read, 0x8 MFMA.
template <int DS, int MFMA, int PER>
__device__ __forceinline__ void sched_interleave() {
  if constexpr (DS > 0 && MFMA > 0) {
    constexpr int n = DS < PER ? DS : PER;
    __builtin_amdgcn_sched_group_barrier(0x100, n, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    sched_interleave<DS - n, MFMA - 1, PER>();
  } else if constexpr (MFMA > 0) {
    __builtin_amdgcn_sched_group_barrier(0x008, MFMA, 0);
  } else if constexpr (DS > 0) {
    __builtin_amdgcn_sched_group_barrier(0x100, DS, 0);
  }
}

// Fast-path fragment: the operand's LDS ring holds four slabs.  A k-strided operand keeps four [32][ROWS] stages;
// a k-contiguous one keeps two [ROWS][64] pairs, slab s4 being half (s4 & 1) of pair (s4 >> 1).
template <int ROWS, bool KC>
__device__ __forceinline__ bf16x8 read_frag_ring(const bf16_t* ring, int s4, int rc0, int ks, int lane) {
  if (KC) {
    const bf16_t* pair = ring + (s4 >> 1) * (2 * ROWS * BK);
    return *(const bf16x8*)(pair + lds_off_kc2(rc0 + (lane & 31), (s4 & 1) * 4 + ks * 2 + (lane >> 5)));
  } else {
    return read_frag<ROWS, false>(ring + s4 * (ROWS * BK), rc0, ks, lane);
  }
}
// Fragment set of one 16-wide sub-step (MI A-fragments, NI B-fragments) and the MFMAs that consume it.
template <int BM, int BN, int WM, int WN, bool AKC, bool BKC>
__device__ __forceinline__ void load_frags(bf16x8 (&fa)[BM / WM / 32], bf16x8 (&fb)[BN / WN / 32], const bf16_t* ringA,
                                           const bf16_t* ringB, int s4, int ks, int wm, int wn, int lane) {
  using T = Tile<BM, BN, WM, WN>;
#pragma unroll
  for (int mi = 0; mi < T::MI; ++mi) fa[mi] = read_frag_ring<BM, AKC>(ringA, s4, wm * T::TM + mi * 32, ks, lane);
#pragma unroll
  for (int ni = 0; ni < T::NI; ++ni) fb[ni] = read_frag_ring<BN, BKC>(ringB, s4, wn * T::TN + ni * 32, ks, lane);
}
// fragment R of a sub-step: R < MI -> A fragment R, else B fragment R - MI; nothing beyond MI + NI
template <int R, int BM, int BN, int WM, int WN, bool AKC, bool BKC>
__device__ __forceinline__ void load_frag_r(bf16x8 (&fa)[BM / WM / 32], bf16x8 (&fb)[BN / WN / 32], const bf16_t* ringA,
                                            const bf16_t* ringB, int s4, int ks, int wm, int wn, int lane) {
  using T = Tile<BM, BN, WM, WN>;
  if constexpr (R < T::MI) fa[R] = read_frag_ring<BM, AKC>(ringA, s4, wm * T::TM + R * 32, ks, lane);
  else if constexpr (R < T::MI + T::NI) fb[R - T::MI] = read_frag_ring<BN, BKC>(ringB, s4, wn * T::TN + (R - T::MI) * 32, ks, lane);
}
// MFMA number M of a sub-step (row-major over the MI x NI accumulators)
template <int M, int MI, int NI>
__device__ __forceinline__ void mfma_m(f32x16 (&acc)[MI][NI], const bf16x8 (&fa)[MI], const bf16x8 (&fb)[NI]) {
  constexpr int mi = M / NI, ni = M % NI;
  acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ni], fa[mi], acc[mi][ni], 0, 0, 0);
}
// slot (0 .. MF-1) in front of whose MFMA load G of GN is issued: spread evenly over the sub-step
constexpr int dma_slot(int g, int gn, int mf) { return ((2 * g + 1) * mf) / (2 * gn); }

// One slab of MFMAs from LDS.  Software pipeline over the four 16-wide sub-steps: the fragments of sub-step
// ks+1 are requested while the MFMAs of sub-step ks run (their operands were requested one sub-step earlier).
template <int BM, int BN, int WM, int WN, bool AKC, bool BKC>
__device__ __forceinline__ void compute_slab(f32x16 (&acc)[BM / WM / 32][BN / WN / 32], const bf16_t* la, const bf16_t* lb,
                                             int wm, int wn, int lane) {
  using T = Tile<BM, BN, WM, WN>;
  constexpr int DS = T::MI * (AKC ? 1 : 2) + T::NI * (BKC ? 1 : 2);  // DS instructions per sub-step
  constexpr int MF = T::MI * T::NI;
  constexpr int PER = (DS + MF / 2 - 1) / (MF / 2 > 0 ? MF / 2 : 1);  // reads finished within the first half of the MFMAs
  bf16x8 af[2][T::MI], bfr[2][T::NI];
#pragma unroll
  for (int mi = 0; mi < T::MI; ++mi) af[0][mi] = read_frag<BM, AKC>(la, wm * T::TM + mi * 32, 0, lane);
#pragma unroll
  for (int ni = 0; ni < T::NI; ++ni) bfr[0][ni] = read_frag<BN, BKC>(lb, wn * T::TN + ni * 32, 0, lane);
#pragma unroll
  for (int ks = 0; ks < BK / 16; ++ks) {
    const int c = ks & 1, nx = c ^ 1;
    __builtin_amdgcn_sched_barrier(0);
    if (ks + 1 < BK / 16) {
#pragma unroll
      for (int mi = 0; mi < T::MI; ++mi) af[nx][mi] = read_frag<BM, AKC>(la, wm * T::TM + mi * 32, ks + 1, lane);
#pragma unroll
      for (int ni = 0; ni < T::NI; ++ni) bfr[nx][ni] = read_frag<BN, BKC>(lb, wn * T::TN + ni * 32, ks + 1, lane);
    }
#pragma unroll
    for (int mi = 0; mi < T::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < T::NI; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[c][ni], af[c][mi], acc[mi][ni], 0, 0, 0);
    if (ks + 1 < BK / 16) sched_interleave<DS, MF, PER>();
  }
  __builtin_amdgcn_sched_barrier(0);
}

// ---- coalesced tile stores ----
// The MFMA accumulator layout gives a lane 4 consecutive columns of one row: stored directly, a wavefront
// instruction writes 32 rows x 16 bytes, and every 128-byte line of C is completed by eight separate partial
// writes (measured: 8.5 us to store a 16 MiB block, 1.9 TB/s).  Instead a 32-row chunk of the wavefront's tile goes
// through a wavefront-private piece of LDS (free after the k-loop) and comes back as 16 bytes per lane with the
// lanes of a row side by side: whole rows of the tile (128 bytes for 64 bf16 columns) per store.
// LDS operations of one wavefront execute in order, so no barrier separates the write from the read-back.
template <int TN>
struct ChunkBf16 {
  static constexpr int PITCH = TN * 2 + 8;      // bytes per row: 34 (TN = 64) banks, conflict-free 8-byte writes
  static constexpr int BYTES = 32 * PITCH;
  static constexpr int LPR = TN / 8;            // lanes per row on the way out (16 bytes each)
  static constexpr int RPI = 64 / LPR;          // rows per store instruction
  static constexpr int NIT = 32 / RPI;
};
// write: v[g] = columns ni*32 + g*8 + 4*(lane/32) .. +3 of row (lane % 32) of the chunk, packed as 4 bf16
template <int TN>
__device__ __forceinline__ void chunk_write_bf16(char* lds_wave, int ni, const uint2 (&v)[4], int lane) {
  char* wr = lds_wave + (lane & 31) * ChunkBf16<TN>::PITCH + ((lane >> 5) << 3) + ni * 64;
#pragma unroll
  for (int g = 0; g < 4; ++g) *(uint2*)(wr + g * 16) = v[g];
}
// read back and store the whole 32 x TN chunk
template <int TN>
__device__ __forceinline__ void chunk_flush_bf16(const char* lds_wave, bf16_t* c_chunk, long long ldc, int lane) {
  using L = ChunkBf16<TN>;
  const int r0 = lane / L::LPR, c = lane % L::LPR;
#pragma unroll
  for (int it = 0; it < L::NIT; ++it) {
    const int row = it * L::RPI + r0;
    const char* rd = lds_wave + row * L::PITCH + c * 16;
    const uint2 lo = *(const uint2*)rd, hi = *(const uint2*)(rd + 8);
    *(uint4*)(c_chunk + (long long)row * ldc + c * 8) = make_uint4(lo.x, lo.y, hi.x, hi.y);
  }
}
template <int TN>
__device__ __forceinline__ void store_chunk_bf16(char* lds_wave, bf16_t* c_chunk, long long ldc, const uint2 (&v)[TN / 32][4],
                                                 int lane) {
#pragma unroll
  for (int ni = 0; ni < TN / 32; ++ni) chunk_write_bf16<TN>(lds_wave, ni, v[ni], lane);
  chunk_flush_bf16<TN>(lds_wave, c_chunk, ldc, lane);
}
// same for fp32 output: v[g] = the four floats; rows of TN floats leave as 16 bytes per lane
template <int TN>
struct ChunkF32 {
  static constexpr int PITCH = TN * 4 + 16;
  static constexpr int BYTES = 32 * PITCH;
  static constexpr int LPR = TN / 4;
  static constexpr int RPI = 64 / LPR;
  static constexpr int NIT = 32 / RPI;
};
template <int TN>
__device__ __forceinline__ void chunk_write_f32(char* lds_wave, int ni, const float4 (&v)[4], int lane) {
  char* wr = lds_wave + (lane & 31) * ChunkF32<TN>::PITCH + ((lane >> 5) << 4) + ni * 128;
#pragma unroll
  for (int g = 0; g < 4; ++g) *(float4*)(wr + g * 32) = v[g];
}
template <int TN>
__device__ __forceinline__ void chunk_flush_f32(const char* lds_wave, float* c_chunk, long long ldc, int lane) {
  using L = ChunkF32<TN>;
  const int r0 = lane / L::LPR, c = lane % L::LPR;
#pragma unroll
  for (int it = 0; it < L::NIT; ++it) {
    const int row = it * L::RPI + r0;
    *(float4*)(c_chunk + (long long)row * ldc + c * 4) = *(const float4*)(lds_wave + row * L::PITCH + c * 16);
  }
}
template <int TN>
__device__ __forceinline__ void store_chunk_f32(char* lds_wave, float* c_chunk, long long ldc, const float4 (&v)[TN / 32][4],
                                                int lane) {
#pragma unroll
  for (int ni = 0; ni < TN / 32; ++ni) chunk_write_f32<TN>(lds_wave, ni, v[ni], lane);
  chunk_flush_f32<TN>(lds_wave, c_chunk, ldc, lane);
}

// wavefronts per SIMD the kernel is compiled for: what two LDS stages of the tile allow on a 160 KiB CU
template <int BM, int BN, int WM, int WN>
struct Occ {
  static constexpr int lds_bytes = NSTAGE * (BM + BN) * BK * 2;
  static constexpr int wgs = (160 * 1024) / lds_bytes;
  static constexpr int waves_per_simd_raw = wgs * WM * WN / 4;
  static constexpr int value = waves_per_simd_raw < 1 ? 1 : (waves_per_simd_raw > 2 ? 2 : waves_per_simd_raw);
};

// FAST = full tiles, direct-to-LDS loads, vector epilogue; !FAST = bounds-checked everything.
// PLAIN (FAST only) = the epilogue is a bare store of the accumulator (alpha 1, no bias / activation / residual):
// a short, fully unrolled store sequence instead of the general epilogue, whose straight-line code costs
// microseconds per tile.
// LOOP selects the k-loop of the fast path: 1 = ring of four 32-wide slabs, fragments read one sub-step ahead
// (the loop described above); 2 = stages of 64 k, the fragments of a whole stage read into registers while the
// matrix cores work on the registers of the stage before it (see the loop).
template <int BM, int BN>
struct Loop2 {
  // three stages where one workgroup owns the CU anyway (the 384-row tiles: 144 KiB); two stages otherwise, which is the
  // LDS footprint of the four-slab ring, so that as many workgroups share a CU as with it
  static constexpr int NST = (BM + BN == 384) ? 3 : 2;
  static constexpr int RING32 = 2 * NST;                                        // the same space in 32-wide slabs
};

template <int BM, int BN, int WM, int WN, bool AKC, bool BKC, bool FAST, bool PLAIN, bool SEQ = false, int LOOP = 1>
__global__ __launch_bounds__(WM* WN * 64, (Occ<BM, BN, WM, WN>::value)) void gemm_mfma_kernel(const KArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)
  static_assert(!SEQ || (FAST && !PLAIN), "the range-wise accumulation exists on the fast path with the full epilogue");
  static_assert(LOOP == 1 || FAST, "the register-staged loop exists on the fast path");
  using T = Tile<BM, BN, WM, WN>;
  constexpr int THREADS = T::THREADS, NW = T::NW;
  constexpr int TM = T::TM, TN = T::TN, MI = T::MI, NI = T::NI;
  // one ring of four slabs per operand (see read_frag_ring); the ragged path uses the first two slabs as two stages
  constexpr int RING = FAST ? (LOOP == 2 ? Loop2<BM, BN>::RING32 : NSTAGE) : 2;
  constexpr int LDS_BYTES = RING * (T::A_ELEMS + T::B_ELEMS) * 2;
  __shared__ __attribute__((aligned(1024))) bf16_t lds_all[RING * (T::A_ELEMS + T::B_ELEMS)];
  bf16_t* const ldsA = lds_all;
  bf16_t* const ldsB = lds_all + RING * T::A_ELEMS;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  OPTIMUS_LAB_STAMP(0);

  // ---- which tile: XCD-aware remap of the linear workgroup id ----
  // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of tiles so that
  // neighbours sharing A rows / B columns also share an L2.
  long long nwg = (long long)gridDim.x;
  long long wg = blockIdx.x;
  {
    long long per = nwg >> 3, rem = nwg & 7;
    long long xcd = wg & 7, slot = wg >> 3;
    long long start = xcd * per + (xcd < rem ? xcd : rem);  // XCDs 0..rem-1 own per+1 workgroups
    wg = start + slot;
  }
  const int split = (int)(wg % a.splits);
  wg /= a.splits;
  const int tiles = a.tiles_m * a.tiles_n;
  const long long z = wg / tiles;
  int t = (int)(wg % tiles);
  int tm, tn;
  {  // column-major walk within groups of a.group tile rows: the contiguous tile range of an XCD is then a
     // block of a.group rows by (range / a.group) columns, sized on the host so that its A rows and B columns
     // weigh about the same (least bytes fetched per XCD)
    const int GROUP = a.group;
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
    per = (per + 1) & ~1;  // the fast path walks slabs in pairs
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
  // SEQ: `tot` holds the sum of the finished ranges, `acc` the running range (see KArgs::seq_splits); ranges are cut
  // exactly as the panel split cuts them
  f32x16 tot[SEQ ? MI : 1][SEQ ? NI : 1];
  int seq_per = 0, seq_next = 0;
  if constexpr (SEQ) {
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int e = 0; e < 16; ++e) tot[mi][ni][e] = 0.f;
    const int total = t_hi - t_lo;
    seq_per = (((total + a.seq_splits - 1) / a.seq_splits) + 1) & ~1;
    seq_next = seq_per;
  }

  const bf16_t* Atile = Az + (AKC ? (long long)m0 * a.lda : (long long)m0);
  const bf16_t* Btile = Bz + (BKC ? (long long)n0 * a.ldb : (long long)n0);

  if (t_lo < t_hi) {
    // slab index -> (panel l, offset k0 inside the panel); advanced incrementally
    int l = t_lo / tpp, k0 = (t_lo - l * tpp) * BK;
    if constexpr (FAST && LOOP == 2) {
      // ---- stages of 64 k ----
      // LDS holds NST stages of [BM x 64] + [64 x BN].  An iteration (one stage, four 16-wide sub-steps) has two halves:
      //   first half:  matrix-core instructions of sub-steps 0, 1 (registers h0) | LDS reads of sub-steps 2, 3 (-> h1)
      //   wait + barrier: my reads of stage i are done (nobody reads it any more), my share of stage i+1 has landed
      //   second half: matrix-core instructions of sub-steps 2, 3 (h1) | LDS reads of sub-steps 0, 1 of stage i+1 (-> h0)
      //                | the loads of stage i+NST into the space stage i has left
      // One wait and one barrier per 64 k; the reads have had half an iteration to complete and the loads NST-1
      // iterations, so neither wait is normally exposed.  The memory instructions of a half are spread between its
      // matrix-core instructions: issued in one burst they fill the CU's LDS and memory-instruction queues, and a
      // wavefront that waits for queue space issues no matrix-core instruction either.
      constexpr int NST = Loop2<BM, BN>::NST;
      constexpr int PA1 = DirectPlan<BM, NW>::PER, PB1 = DirectPlan<BN, NW>::PER;   // KiB chunks per wavefront per 32 k
      constexpr int NOA = AKC ? 2 * PA1 : PA1, NOB = BKC ? 2 * PB1 : PB1;             // distinct lane offsets
      constexpr int LP = 2 * PA1 + 2 * PB1;                                          // loads per wavefront per stage
      constexpr int A_ST = BM * 64, B_ST = BN * 64;                                  // elements per stage
      unsigned offA[NOA], offB[NOB];
      direct_offsets<BM, AKC, NW, NOA>(offA, a.lda, wave, lane);
      direct_offsets<BN, BKC, NW, NOB>(offB, a.ldb, wave, lane);
      bf16_t* const stA = lds_all;
      bf16_t* const stB = lds_all + NST * A_ST;
      const unsigned stepA = (unsigned)(AKC ? 64 : 64 * a.lda) * 2u, stepB = (unsigned)(BKC ? 64 : 64 * a.ldb) * 2u;
      const unsigned halfA = (unsigned)(32 * a.lda) * 2u, halfB = (unsigned)(32 * a.ldb) * 2u;   // 32 k-rows of a k-strided operand
      int lq = l, kq = k0;
      i32x4 ra = make_rsrc(Atile + lq * a.sAl), rb = make_rsrc(Btile + lq * a.sBl);
      unsigned sa = (unsigned)(AKC ? kq : kq * a.lda) * 2u, sb = (unsigned)(BKC ? kq : kq * a.ldb) * 2u;
      const int n64 = (t_hi - t_lo) >> 1;
      // load g (0 .. LP-1) of the stage that goes into LDS stage st: A's chunks first, then B's
      auto load_item = [&](int st, int g) {
        if (g < 2 * PA1) {
          if constexpr (AKC) direct_issue_one(ra, sa, offA[g], stA + st * A_ST, wave * NOA + g);
          else direct_issue_one(ra, sa + (unsigned)(g / PA1) * halfA, offA[g % PA1], stA + st * A_ST + (g / PA1) * 32 * BM, wave * PA1 + g % PA1);
        } else {
          const int h = g - 2 * PA1;
          if constexpr (BKC) direct_issue_one(rb, sb, offB[h], stB + st * B_ST, wave * NOB + h);
          else direct_issue_one(rb, sb + (unsigned)(h / PB1) * halfB, offB[h % PB1], stB + st * B_ST + (h / PB1) * 32 * BN, wave * PB1 + h % PB1);
        }
      };
      auto advance = [&]() {
        kq += 64;
        if (kq >= a.Kp) { kq = 0; ++lq; sa = 0; sb = 0; ra = make_rsrc(Atile + lq * a.sAl); rb = make_rsrc(Btile + lq * a.sBl); }
        else { sa += stepA; sb += stepB; }
      };
      auto issue_stage = [&](int st) {
#pragma unroll
        for (int g = 0; g < LP; ++g) load_item(st, g);
        advance();
      };
      // fragments of one whole stage: four 16-wide sub-steps; item r = fragment (r % NF) of sub-step (r / NF).
      // Every LDS address is a per-lane base computed once (the swizzles depend on the lane only) plus the stage's
      // offset plus a constant, so that a read costs no address arithmetic inside the loop:
      //   k-contiguous operand: one base per sub-step (chunk index XOR row term), fragment row blocks 32 * 128 bytes apart;
      //   k-strided operand:    one base per fragment (column granule XOR row term), sub-steps 16 k-rows apart.
      constexpr int NF = MI + NI, NRD = 4 * NF, NMF = 4 * MI * NI;
      typedef __attribute__((address_space(3))) char lds_char;
      lds_char* const lds3 = (lds_char*)lds_all;
      unsigned fbaseA[AKC ? 4 : MI], fbaseB[BKC ? 4 : NI];
      if constexpr (AKC) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) fbaseA[ks] = (unsigned)lds_off_kc2(wm * TM + (lane & 31), ks * 2 + (lane >> 5)) * 2u;
      } else {
        const int lg = lane & 15;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
          fbaseA[mi] = (unsigned)lds_off_ks<BM>(((lane >> 5) << 3) + (lg >> 2), wm * TM + mi * 32 + (((lane >> 4) & 1) << 4) + ((lg & 3) << 2)) * 2u;
      }
      if constexpr (BKC) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) fbaseB[ks] = (unsigned)(NST * A_ST + lds_off_kc2(wn * TN + (lane & 31), ks * 2 + (lane >> 5))) * 2u;
      } else {
        const int lg = lane & 15;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
          fbaseB[ni] = (unsigned)(NST * A_ST + lds_off_ks<BN>(((lane >> 5) << 3) + (lg >> 2), wn * TN + ni * 32 + (((lane >> 4) & 1) << 4) + ((lg & 3) << 2))) * 2u;
      }
      bf16x8 ha[4][MI], hb[4][NI];   // [sub-step][fragment]: sub-steps 0, 1 = h0, sub-steps 2, 3 = h1
      auto read_kc = [&](unsigned off) { return *(const __attribute__((address_space(3))) bf16x8*)(lds3 + off); };
      auto read_ks = [&](unsigned off, int rows) {   // two transposing reads: k-rows r .. r+3 and r+4 .. r+7 of the lane's column group
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(lds3 + off));
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(lds3 + off + 4 * rows * 2));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
      };
      auto read_item = [&](unsigned stoffA, unsigned stoffB, int ks, int f) {
        if (f < MI) {
          if constexpr (AKC) ha[ks][f] = read_kc(fbaseA[ks] + stoffA + (unsigned)(f * 32 * 128));
          else ha[ks][f] = read_ks(fbaseA[f] + stoffA + (unsigned)(ks * 16 * BM * 2), BM);
        } else {
          const int n = f - MI;
          if constexpr (BKC) hb[ks][n] = read_kc(fbaseB[ks] + stoffB + (unsigned)(n * 32 * 128));
          else hb[ks][n] = read_ks(fbaseB[n] + stoffB + (unsigned)(ks * 16 * BN * 2), BN);
        }
      };
      // one half of an iteration: the matrix-core instructions of sub-steps 2*HH, 2*HH+1; in front of each its share of
      // the reads of the other two sub-steps (of stage st_rd) and, in the second half, of the loads into stage st_ld
      constexpr int HM = 2 * MI * NI, HR = 2 * NF;
      auto half = [&](auto hh_, auto with_reads, auto with_loads, int st_rd, int st_ld) {
        constexpr int HH = decltype(hh_)::value;
        const unsigned offA_rd = (unsigned)(st_rd * A_ST * 2), offB_rd = (unsigned)(st_rd * B_ST * 2);
#pragma unroll
        for (int m = 0; m < HM; ++m) {
          if constexpr (decltype(with_reads)::value && !(OPTIMUS_LAB_DBG & 4)) {
            // all reads in front of the first half of the matrix-core instructions: the wait that follows the last
            // of them must not expose the latency of a read issued just before it
            constexpr int RS = HM / 2 > 0 ? HM / 2 : 1;
#pragma unroll
            for (int r = m * HR / RS; r < (m + 1) * HR / RS && r < HR; ++r) read_item(offA_rd, offB_rd, 2 * (1 - HH) + r / NF, r % NF);
          }
          if constexpr (decltype(with_loads)::value && !(OPTIMUS_LAB_DBG & 1)) {
#pragma unroll
            for (int g = m * LP / HM; g < (m + 1) * LP / HM; ++g) load_item(st_ld, g);
          }
          if constexpr (!(OPTIMUS_LAB_DBG & 8)) {
            const int ks = 2 * HH + m / (MI * NI), mi = (m / NI) % MI, ni = m % NI;
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hb[ks][ni], ha[ks][mi], acc[mi][ni], 0, 0, 0);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (decltype(with_loads)::value) advance();
      };
      // prologue: the first NST stages, then the fragments of sub-steps 0, 1 of stage 0
      issue_stage(0);
      if (n64 > 1) issue_stage(1);
      if (NST > 2 && n64 > 2) issue_stage(2);
      {
        const int younger = (n64 > NST ? NST : n64) - 1;
        if (younger >= 2) OPTIMUS_WAIT_VMCNT(2 * LP);
        else if (younger == 1) OPTIMUS_WAIT_VMCNT(LP);
        else OPTIMUS_WAIT_VMCNT(0);
      }
      OPTIMUS_BARRIER();
      OPTIMUS_LAB_STAMP(1);
#pragma unroll
      for (int r = 0; r < HR; ++r) read_item(0u, 0u, r / NF, r % NF);
      int seq_next64 = seq_next >> 1;
      const int seq_per64 = seq_per >> 1;
      constexpr std::true_type yes{};
      constexpr std::false_type no{};
      constexpr std::integral_constant<int, 0> first{};
      constexpr std::integral_constant<int, 1> second{};
      int st_cur = 0, st_nxt = NST > 1 ? 1 : 0;
      auto range_end = [&](int i) {   // SEQ: a range of the emulated panel split ends in front of stage i
        if constexpr (SEQ) {
          if (i == seq_next64 && i > 0) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
              for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                  tot[mi][ni][e] += acc[mi][ni][e];
                  acc[mi][ni][e] = 0.f;
                }
            seq_next64 += seq_per64;
          }
        }
      };
      auto next_stage = [&]() {
        st_cur = st_nxt;
        st_nxt = st_nxt + 1 == NST ? 0 : st_nxt + 1;
      };
      // steady state: every iteration reads the next stage and refills the stage it leaves (straight-line body, constant
      // wait counts: with branches inside the loop the compiler copies the accumulators between the paths)
      int i = 0;
#if OPTIMUS_LAB_DBG & 64
      unsigned long long lab_sum_a = 0, lab_sum_b = 0, lab_tb = 0;
#endif
      for (; i + NST < n64; ++i) {
        range_end(i);
        half(first, yes, no, st_cur, 0);
#if OPTIMUS_LAB_DBG & 64
        const unsigned long long lab_ta = clock64();
#endif
        // stage i+1 has landed (stage i+2's loads stay in flight); my reads of stage i are done
        if constexpr (!(OPTIMUS_LAB_DBG & 16)) OPTIMUS_WAIT_VMCNT_LGKM0(NST > 2 ? LP : 0);
        if constexpr (!(OPTIMUS_LAB_DBG & 2)) OPTIMUS_BARRIER();
#if OPTIMUS_LAB_DBG & 64
        lab_sum_a += lab_ta;
        lab_sum_b += lab_tb;
        lab_tb = clock64();
#endif
        half(second, yes, yes, st_nxt, st_cur);
        next_stage();
      }
#if OPTIMUS_LAB_DBG & 64
      lab_sum_b += lab_tb;
      if (lane == 0 && blockIdx.x < 2048) g_lab_stall[blockIdx.x * 8 + wave] = lab_sum_b - lab_sum_a;
#endif
      // the last stages: nothing left to load
      for (; i + 1 < n64; ++i) {
        range_end(i);
        half(first, yes, no, st_cur, 0);
        if (NST > 2 && i + 2 < n64) OPTIMUS_WAIT_VMCNT_LGKM0(LP);
        else OPTIMUS_WAIT_VMCNT_LGKM0(0);
        OPTIMUS_BARRIER();
        half(second, yes, no, st_nxt, st_cur);
        next_stage();
      }
      range_end(i);
      half(first, yes, no, st_cur, 0);
      half(second, no, no, st_nxt, st_cur);
      // the results leave through LDS (see the epilogue): nobody may still be reading the last stage
      OPTIMUS_WAIT_VMCNT_LGKM0(0);
      OPTIMUS_BARRIER();
      OPTIMUS_LAB_STAMP(2);
    } else if constexpr (FAST) {
      // Loads per wavefront: a k-strided operand moves one slab per step; a k-contiguous operand moves a pair of
      // slabs (whole 128-byte lines per row) every second step.  The slab count of a workgroup is even (host).
      constexpr int PA1 = DirectPlan<BM, NW>::PER, PB1 = DirectPlan<BN, NW>::PER;
      constexpr int PA = AKC ? 2 * PA1 : PA1, PB = BKC ? 2 * PB1 : PB1;
      constexpr int PKS = (AKC ? 0 : PA1) + (BKC ? 0 : PB1);          // loads of one k-strided slab issue
      constexpr int PKC2 = (AKC ? 2 * PA1 : 0) + (BKC ? 2 * PB1 : 0);  // loads of one k-contiguous pair issue
      unsigned offA[PA], offB[PB];
      direct_offsets<BM, AKC, NW, PA>(offA, a.lda, wave, lane);
      direct_offsets<BN, BKC, NW, PB>(offB, a.ldb, wave, lane);
      // one load cursor per operand: panel, k offset, buffer resource of the panel, byte offset inside the panel
      constexpr int KA = AKC ? 2 * BK : BK, KB = BKC ? 2 * BK : BK;  // k advance per issue
      const unsigned stepA = (unsigned)(AKC ? KA : KA * a.lda) * 2u;
      const unsigned stepB = (unsigned)(BKC ? KB : KB * a.ldb) * 2u;
      int lqa = l, kqa = k0, lqb = l, kqb = k0;
      i32x4 ra = make_rsrc(Atile + lqa * a.sAl), rb = make_rsrc(Btile + lqb * a.sBl);
      unsigned sa = (unsigned)(AKC ? kqa : kqa * a.lda) * 2u, sb = (unsigned)(BKC ? kqb : kqb * a.ldb) * 2u;
      const int nslab = t_hi - t_lo;
#define OPTIMUS_ISSUE_A(DST)                                                         \
  do {                                                                               \
    direct_issue<BM, NW, PA>(ra, sa, offA, DST, wave);                               \
    kqa += KA;                                                                       \
    if (kqa >= a.Kp) { kqa = 0; ++lqa; sa = 0; ra = make_rsrc(Atile + lqa * a.sAl); } \
    else sa += stepA;                                                                \
  } while (0)
#define OPTIMUS_ISSUE_B(DST)                                                         \
  do {                                                                               \
    direct_issue<BN, NW, PB>(rb, sb, offB, DST, wave);                               \
    kqb += KB;                                                                       \
    if (kqb >= a.Kp) { kqb = 0; ++lqb; sb = 0; rb = make_rsrc(Btile + lqb * a.sBl); } \
    else sb += stepB;                                                                \
  } while (0)
      // pair P (0/1) of the k-contiguous operands; slab S (0..3) of the k-strided ones
#define OPTIMUS_ISSUE_KC(P)                                                          \
  do {                                                                               \
    if constexpr (AKC) OPTIMUS_ISSUE_A(ldsA + (P) * 2 * T::A_ELEMS);                 \
    if constexpr (BKC) OPTIMUS_ISSUE_B(ldsB + (P) * 2 * T::B_ELEMS);                 \
  } while (0)
#define OPTIMUS_ISSUE_KS(S)                                                          \
  do {                                                                               \
    if constexpr (!AKC) OPTIMUS_ISSUE_A(ldsA + (S) * T::A_ELEMS);                    \
    if constexpr (!BKC) OPTIMUS_ISSUE_B(ldsB + (S) * T::B_ELEMS);                    \
  } while (0)
      // Continuous pipeline over 16-wide sub-steps; F0 = (fa0, fb0) holds sub-step 0 of the current slab i.
      //   A  sub-step 0: MFMAs on F0; between them the fragment reads of sub-step 1 (F1) and the second half of the
      //      loads of the group opened in the previous step;
      //   B  wait for F1 (after it this wavefront reads slab i no more) and for the loads slab i+1 needs, leaving the
      //      younger ones in flight; barrier: nobody reads slab i any more, slab i+1 is complete in LDS;
      //   C  open the group that refills what slab i freed: its stage for the k-strided operands (slab i+4); after an
      //      odd slab also its pair for the k-contiguous operands (slabs i+3, i+4);
      //   D  sub-step 1: MFMAs on F1; between them the reads of sub-step 0 of slab i+1 (F0) and the first half of
      //      the group's loads.
      // The loads are spread between the MFMAs one by one: issued in one burst after the barrier they fill the
      // CU's memory-instruction queue, and a wavefront stalled on a full queue issues no MFMA either.
      // Loads retire in issue order.  Issue order is [pair 0, slab 0, slab 1, pair 1, slab 2, slab 3], then per even
      // step [slab i+4], per odd step [pair, slab i+4]; the wait counts below are the loads younger than what slab
      // i+1 needs in that order (at B of step i everything up to the group of step i-1 has been issued).
      constexpr int MF = MI * NI;
      constexpr int NF = MI + NI;                                   // fragments per sub-step
      constexpr int FSLOTS = MF / 2 > 0 ? MF / 2 : 1;               // the fragment reads go in front of the first MFMAs
      constexpr int FPS = (NF + FSLOTS - 1) / FSLOTS;               // fragments requested per such slot
      static_assert(BK == 32 && NSTAGE == 4, "the pipeline below is written for two sub-steps per slab, four slabs");
      static_assert(MF <= 16 && FPS <= 3 && PA + PB <= 16, "slot and load lists below");
      constexpr int G_ODD = PA + PB, G_EVEN = PKS;  // loads per group
      bf16x8 fa0[MI], fb0[NI], fa1[MI], fb1[NI];
      bool pend = false;  // the group opened in the previous step still has its second half to issue
      // load N of the group of parity ODD refilling slab S's space: A's chunks first, then B's
#define OPTIMUS_DMA_N(ODD, S, N)                                                                                  \
  do {                                                                                                            \
    constexpr int nA_ = (ODD) ? PA : (AKC ? 0 : PA);                                                              \
    constexpr int nB_ = (ODD) ? PB : (BKC ? 0 : PB);                                                              \
    if constexpr ((N) < nA_)                                                                                      \
      direct_issue_one(ra, sa, offA[(N) < nA_ ? (N) : 0], ldsA + (AKC ? ((S) >> 1) * 2 : (S)) * T::A_ELEMS,       \
                       wave * PA + (N));                                                                          \
    else if constexpr ((N) < nA_ + nB_)                                                                           \
      direct_issue_one(rb, sb, offB[(N) >= nA_ && (N) < nA_ + nB_ ? (N) - nA_ : 0],                               \
                       ldsB + (BKC ? ((S) >> 1) * 2 : (S)) * T::B_ELEMS, wave * PB + (N) - nA_);                  \
  } while (0)
      // in slot M: the loads G0 .. G0+GN-1 of the group whose turn it is
#define OPTIMUS_DMA_SLOT(M, ODD, S, G0, GN, DO)                                                                   \
  do {                                                                                                            \
    if constexpr ((GN) > 0) {                                                                                     \
      if constexpr (dma_slot(0, (GN) > 0 ? (GN) : 1, MF) == (M)) { if (DO) OPTIMUS_DMA_N(ODD, S, (G0) + 0); }     \
      if constexpr ((GN) > 1 && dma_slot(1, (GN) > 0 ? (GN) : 1, MF) == (M)) { if (DO) OPTIMUS_DMA_N(ODD, S, (G0) + 1); }\
      if constexpr ((GN) > 2 && dma_slot(2, (GN) > 0 ? (GN) : 1, MF) == (M)) { if (DO) OPTIMUS_DMA_N(ODD, S, (G0) + 2); }\
      if constexpr ((GN) > 3 && dma_slot(3, (GN) > 0 ? (GN) : 1, MF) == (M)) { if (DO) OPTIMUS_DMA_N(ODD, S, (G0) + 3); }\
      if constexpr ((GN) > 4 && dma_slot(4, (GN) > 0 ? (GN) : 1, MF) == (M)) { if (DO) OPTIMUS_DMA_N(ODD, S, (G0) + 4); }\
      if constexpr ((GN) > 5 && dma_slot(5, (GN) > 0 ? (GN) : 1, MF) == (M)) { if (DO) OPTIMUS_DMA_N(ODD, S, (G0) + 5); }\
      if constexpr ((GN) > 6 && dma_slot(6, (GN) > 0 ? (GN) : 1, MF) == (M)) { if (DO) OPTIMUS_DMA_N(ODD, S, (G0) + 6); }\
      if constexpr ((GN) > 7 && dma_slot(7, (GN) > 0 ? (GN) : 1, MF) == (M)) { if (DO) OPTIMUS_DMA_N(ODD, S, (G0) + 7); }\
    }                                                                                                             \
  } while (0)
#define OPTIMUS_SLOT(M, FA_LD, FB_LD, S_LD, KS_LD, FA_MM, FB_MM, ODD, S, G0, GN, DO)                              \
  do {                                                                                                            \
    if constexpr ((M) < MF) {                                                                                     \
      load_frag_r<(M) * FPS, BM, BN, WM, WN, AKC, BKC>(FA_LD, FB_LD, ldsA, ldsB, S_LD, KS_LD, wm, wn, lane); \
      load_frag_r<((FPS > 1) ? (M) * FPS + 1 : NF), BM, BN, WM, WN, AKC, BKC>(FA_LD, FB_LD, ldsA, ldsB, S_LD, KS_LD, wm, wn, lane); \
      load_frag_r<((FPS > 2) ? (M) * FPS + 2 : NF), BM, BN, WM, WN, AKC, BKC>(FA_LD, FB_LD, ldsA, ldsB, S_LD, KS_LD, wm, wn, lane); \
      OPTIMUS_DMA_SLOT(M, ODD, S, G0, GN, DO);                                                                    \
      mfma_m<(((M) < MF) ? (M) : 0), MI, NI>(acc, FA_MM, FB_MM);                                                      \
      __builtin_amdgcn_sched_barrier(0);                                                                          \
    }                                                                                                             \
  } while (0)
#define OPTIMUS_HALF(FA_LD, FB_LD, S_LD, KS_LD, FA_MM, FB_MM, ODD, S, G0, GN, DO)                                 \
  do {                                                                                                            \
    __builtin_amdgcn_sched_barrier(0);                                                                            \
    OPTIMUS_SLOT(0, FA_LD, FB_LD, S_LD, KS_LD, FA_MM, FB_MM, ODD, S, G0, GN, DO);                                 \
    OPTIMUS_SLOT(1, FA_LD, FB_LD, S_LD, KS_LD, FA_MM, FB_MM, ODD, S, G0, GN, DO);                                 \
    OPTIMUS_SLOT(2, FA_LD, FB_LD, S_LD, KS_LD, FA_MM, FB_MM, ODD, S, G0, GN, DO);                                 \
    OPTIMUS_SLOT(3, FA_LD, FB_LD, S_LD, KS_LD, FA_MM, FB_MM, ODD, S, G0, GN, DO);                                 \
    OPTIMUS_SLOT(4, FA_LD, FB_LD, S_LD, KS_LD, FA_MM, FB_MM, ODD, S, G0, GN, DO);                                 \
    OPTIMUS_SLOT(5, FA_LD, FB_LD, S_LD, KS_LD, FA_MM, FB_MM, ODD, S, G0, GN, DO);                                 \
    OPTIMUS_SLOT(6, FA_LD, FB_LD, S_LD, KS_LD, FA_MM, FB_MM, ODD, S, G0, GN, DO);                                 \
    OPTIMUS_SLOT(7, FA_LD, FB_LD, S_LD, KS_LD, FA_MM, FB_MM, ODD, S, G0, GN, DO);                                 \
    OPTIMUS_SLOT(8, FA_LD, FB_LD, S_LD, KS_LD, FA_MM, FB_MM, ODD, S, G0, GN, DO);                                 \
    OPTIMUS_SLOT(9, FA_LD, FB_LD, S_LD, KS_LD, FA_MM, FB_MM, ODD, S, G0, GN, DO);                                 \
    OPTIMUS_SLOT(10, FA_LD, FB_LD, S_LD, KS_LD, FA_MM, FB_MM, ODD, S, G0, GN, DO);                                \
    OPTIMUS_SLOT(11, FA_LD, FB_LD, S_LD, KS_LD, FA_MM, FB_MM, ODD, S, G0, GN, DO);                                \
    OPTIMUS_SLOT(12, FA_LD, FB_LD, S_LD, KS_LD, FA_MM, FB_MM, ODD, S, G0, GN, DO);                                \
    OPTIMUS_SLOT(13, FA_LD, FB_LD, S_LD, KS_LD, FA_MM, FB_MM, ODD, S, G0, GN, DO);                                \
    OPTIMUS_SLOT(14, FA_LD, FB_LD, S_LD, KS_LD, FA_MM, FB_MM, ODD, S, G0, GN, DO);                                \
    OPTIMUS_SLOT(15, FA_LD, FB_LD, S_LD, KS_LD, FA_MM, FB_MM, ODD, S, G0, GN, DO);                                \
  } while (0)
      // cursor advance once a group is out: every operand that had loads in it
#define OPTIMUS_ADVANCE(ODD)                                                                  \
  do {                                                                                        \
    if constexpr ((ODD) || !AKC) {                                                            \
      kqa += KA;                                                                              \
      if (kqa >= a.Kp) { kqa = 0; ++lqa; sa = 0; ra = make_rsrc(Atile + lqa * a.sAl); }       \
      else sa += stepA;                                                                       \
    }                                                                                         \
    if constexpr ((ODD) || !BKC) {                                                            \
      kqb += KB;                                                                              \
      if (kqb >= a.Kp) { kqb = 0; ++lqb; sb = 0; rb = make_rsrc(Btile + lqb * a.sBl); }       \
      else sb += stepB;                                                                       \
    }                                                                                         \
  } while (0)
      // S = slab position (0..3) of slab i; the previous step's group refills position (S + 3) & 3.
      // ST = 1: steady state, i >= 4 and i + 8 <= nslab at the top of the four steps: every group exists, so every
      // load is unconditional and every wait count a constant (the conditional form costs about ten scalar branches
      // per step, a third of the time of a step on the small tiles).
#define OPTIMUS_STEP_EVEN(S, ST)                                                                                  \
  do {                                                                                                            \
    OPTIMUS_HALF(fa1, fb1, S, 1, fa0, fb0, true, ((S) + 3) & 3, (G_ODD + 1) / 2, G_ODD / 2, ((ST) || pend));      \
    if ((ST) || pend) OPTIMUS_ADVANCE(true);                                                                      \
    if (!(ST)) pend = false;                                                                                      \
    if constexpr (PKS > 0) { /* all k-contiguous: slab i+1 came with slab i, nothing to hand over */              \
      if ((ST) || i + 2 < nslab) OPTIMUS_WAIT_VMCNT_LGKM0(2 * PKS + PKC2);                                        \
      else OPTIMUS_WAIT_VMCNT_LGKM0(0);                                                                           \
      OPTIMUS_BARRIER();                                                                                          \
      if (!(ST)) pend = i + 4 < nslab;                                                                            \
    }                                                                                                             \
    OPTIMUS_HALF(fa0, fb0, (S) + 1, 0, fa1, fb1, false, S, 0, (G_EVEN + 1) / 2, ((ST) || pend));                  \
    ++i;                                                                                                          \
  } while (0)
#define OPTIMUS_STEP_ODD(S, ST)                                                                                   \
  do {                                                                                                            \
    OPTIMUS_HALF(fa1, fb1, S, 1, fa0, fb0, false, (S) - 1, (G_EVEN + 1) / 2, G_EVEN / 2, ((ST) || pend));         \
    if (PKS > 0 && ((ST) || pend)) OPTIMUS_ADVANCE(false);                                                        \
    if ((ST) || i + 3 < nslab) OPTIMUS_WAIT_VMCNT_LGKM0(2 * PKS);                                                 \
    else if (i + 2 < nslab) OPTIMUS_WAIT_VMCNT_LGKM0(PKS);                                                        \
    else OPTIMUS_WAIT_VMCNT_LGKM0(0);                                                                             \
    OPTIMUS_BARRIER();                                                                                            \
    if (!(ST)) pend = i + 3 < nslab;                                                                              \
    /* after the last slab this reads a slab nobody writes any more; the values are never used */                \
    OPTIMUS_HALF(fa0, fb0, ((S) + 1) & 3, 0, fa1, fb1, true, S, 0, (G_ODD + 1) / 2, ((ST) || pend));              \
    ++i;                                                                                                          \
  } while (0)
      // SEQ: a range ends in front of slab i (ranges are even, so only in front of even steps)
#define OPTIMUS_RANGE_END()                                                        \
  do {                                                                             \
    if constexpr (SEQ) {                                                           \
      if (i == seq_next) {                                                         \
        _Pragma("unroll") for (int mi_ = 0; mi_ < MI; ++mi_)                       \
          _Pragma("unroll") for (int ni_ = 0; ni_ < NI; ++ni_)                     \
            _Pragma("unroll") for (int e_ = 0; e_ < 16; ++e_) {                    \
              tot[mi_][ni_][e_] += acc[mi_][ni_][e_];                              \
              acc[mi_][ni_][e_] = 0.f;                                             \
            }                                                                      \
        seq_next += seq_per;                                                       \
      }                                                                            \
    }                                                                              \
  } while (0)
      // prologue: whole groups at once
      OPTIMUS_ISSUE_KC(0);
      OPTIMUS_ISSUE_KS(0);
      OPTIMUS_ISSUE_KS(1);
      if (nslab > 2) {
        OPTIMUS_ISSUE_KC(1);
        OPTIMUS_ISSUE_KS(2);
        OPTIMUS_ISSUE_KS(3);
        OPTIMUS_WAIT_VMCNT(PKC2 + 2 * PKS);
      } else {
        OPTIMUS_WAIT_VMCNT(0);
      }
      OPTIMUS_BARRIER();
      load_frags<BM, BN, WM, WN, AKC, BKC>(fa0, fb0, ldsA, ldsB, 0, 0, wm, wn, lane);
      int i = 0;
      while (i + 4 <= nslab) {
        OPTIMUS_RANGE_END();
        OPTIMUS_STEP_EVEN(0, 0);
        OPTIMUS_STEP_ODD(1, 0);
        OPTIMUS_RANGE_END();
        OPTIMUS_STEP_EVEN(2, 0);
        OPTIMUS_STEP_ODD(3, 0);
        while (i + 8 <= nslab) {  // i >= 4 here
          OPTIMUS_RANGE_END();
          OPTIMUS_STEP_EVEN(0, 1);
          OPTIMUS_STEP_ODD(1, 1);
          OPTIMUS_RANGE_END();
          OPTIMUS_STEP_EVEN(2, 1);
          OPTIMUS_STEP_ODD(3, 1);
          pend = true;  // the last steady step opened a group
        }
      }
      if (i < nslab) {  // one pair left
        OPTIMUS_RANGE_END();
        OPTIMUS_STEP_EVEN(0, 0);
        OPTIMUS_STEP_ODD(1, 0);
      }
#undef OPTIMUS_RANGE_END
#undef OPTIMUS_STEP_EVEN
#undef OPTIMUS_STEP_ODD
#undef OPTIMUS_HALF
#undef OPTIMUS_SLOT
#undef OPTIMUS_DMA_SLOT
#undef OPTIMUS_DMA_N
#undef OPTIMUS_ADVANCE
#undef OPTIMUS_ISSUE_KS
#undef OPTIMUS_ISSUE_KC
#undef OPTIMUS_ISSUE_A
#undef OPTIMUS_ISSUE_B
    } else {
      u32x4 ra[StageDims<BM, THREADS>::PER];
      u32x4 rb[StageDims<BN, THREADS>::PER];
      const int rowsA = a.Mb - m0, rowsB = a.Nb - n0;
      stage_load<BM, AKC, THREADS>(ra, Atile + l * a.sAl, a.lda, k0, rowsA, a.Kp - k0, tid);
      stage_load<BN, BKC, THREADS>(rb, Btile + l * a.sBl, a.ldb, k0, rowsB, a.Kp - k0, tid);
      stage_store<BM, AKC, THREADS>(ra, ldsA, tid);
      stage_store<BN, BKC, THREADS>(rb, ldsB, tid);
      __syncthreads();
      for (int tt = t_lo; tt < t_hi; ++tt) {
        const int cur = (tt - t_lo) & 1;
        const bool more = tt + 1 < t_hi;
        if (more) {
          k0 += BK;
          if (k0 >= a.Kp) { k0 = 0; ++l; }
          stage_load<BM, AKC, THREADS>(ra, Atile + l * a.sAl, a.lda, k0, rowsA, a.Kp - k0, tid);
          stage_load<BN, BKC, THREADS>(rb, Btile + l * a.sBl, a.ldb, k0, rowsB, a.Kp - k0, tid);
        }
        if (cur == 0) compute_slab<BM, BN, WM, WN, AKC, BKC>(acc, ldsA, ldsB, wm, wn, lane);
        else compute_slab<BM, BN, WM, WN, AKC, BKC>(acc, (ldsA + T::A_ELEMS), (ldsB + T::B_ELEMS), wm, wn, lane);
        if (more) {
          stage_store<BM, AKC, THREADS>(ra, cur == 0 ? (ldsA + T::A_ELEMS) : ldsA, tid);
          stage_store<BN, BKC, THREADS>(rb, cur == 0 ? (ldsB + T::B_ELEMS) : ldsB, tid);
        }
        __syncthreads();
      }
    }
  }

  if constexpr (SEQ) {  // the last range joins the sum; the epilogue below works on `acc`
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[mi][ni][e] = tot[mi][ni][e] + acc[mi][ni][e];
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
          const int m = m0 + wm * TM + mi * 32 + (lane & 31);
          const int n = n0 + wn * TN + ni * 32 + g * 8 + ((lane >> 5) << 2);
          if (!FAST && (m >= a.Mb || n >= a.Nb)) continue;
          float* p = P + (long long)m * a.Nb + n;
          if (FAST || n + 3 < a.Nb) {
            *(float4*)p = make_float4(acc[mi][ni][g * 4], acc[mi][ni][g * 4 + 1], acc[mi][ni][g * 4 + 2], acc[mi][ni][g * 4 + 3]);
          } else {
            for (int c = 0; c < 4 && n + c < a.Nb; ++c) p[c] = acc[mi][ni][g * 4 + c];
          }
        }
    return;
  }
  EpiArgs e = a.epi;
  const long long coff = z1 * a.sC1 + z0 * a.sC0;
  if constexpr (PLAIN) {
    // Stores go through LDS chunk by chunk (see store_chunk_bf16) when rows of C are 16-byte aligned; after the
    // last barrier of the k-loop no wavefront reads operand data from LDS any more.
    const long long tile0 = coff + (long long)(m0 + wm * TM) * e.ldc + n0 + wn * TN;   // first element of the wave tile
    const bool lines16 = ((e.ldc | coff) & 7) == 0;
    // this lane's first element when storing directly: row lane%32, column 4*(lane/32)
    const long long first = tile0 + (long long)(lane & 31) * e.ldc + ((lane >> 5) << 2);
    if (!e.out_fp32) {
      if (lines16) {
        static_assert(ChunkBf16<TN>::BYTES * NW <= LDS_BYTES, "chunk staging must fit in the operand rings");
        char* stage = (char*)lds_all + wave * ChunkBf16<TN>::BYTES;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
          uint2 v[NI][4];
#pragma unroll
          for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int g = 0; g < 4; ++g)
              v[ni][g] = make_uint2(pack2_bf16(acc[mi][ni][g * 4], acc[mi][ni][g * 4 + 1]),
                                    pack2_bf16(acc[mi][ni][g * 4 + 2], acc[mi][ni][g * 4 + 3]));
          store_chunk_bf16<TN>(stage, (bf16_t*)e.C + tile0 + (long long)mi * 32 * e.ldc, e.ldc, v, lane);
        }
      } else {
        bf16_t* crow = (bf16_t*)e.C + first;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
          for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int g = 0; g < 4; ++g)
              *(uint2*)(crow + ni * 32 + g * 8) = make_uint2(pack2_bf16(acc[mi][ni][g * 4], acc[mi][ni][g * 4 + 1]),
                                                             pack2_bf16(acc[mi][ni][g * 4 + 2], acc[mi][ni][g * 4 + 3]));
          crow += 32LL * e.ldc;
        }
      }
    } else {
      static_assert(ChunkF32<TN>::BYTES * NW <= LDS_BYTES, "chunk staging must fit in the operand rings");
      if (((e.ldc | coff) & 3) == 0) {
        char* stage = (char*)lds_all + wave * ChunkF32<TN>::BYTES;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
          float4 v[NI][4];
#pragma unroll
          for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int g = 0; g < 4; ++g)
              v[ni][g] = make_float4(acc[mi][ni][g * 4], acc[mi][ni][g * 4 + 1], acc[mi][ni][g * 4 + 2], acc[mi][ni][g * 4 + 3]);
          store_chunk_f32<TN>(stage, (float*)e.C + tile0 + (long long)mi * 32 * e.ldc, e.ldc, v, lane);
        }
      } else {
        float* crow = (float*)e.C + first;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
          for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int g = 0; g < 4; ++g)
              *(float4*)(crow + ni * 32 + g * 8) =
                  make_float4(acc[mi][ni][g * 4], acc[mi][ni][g * 4 + 1], acc[mi][ni][g * 4 + 2], acc[mi][ni][g * 4 + 3]);
          crow += 32LL * e.ldc;
        }
      }
    }
  } else if constexpr (FAST) {
    // General epilogue, vector form (bf16 in, 8- or 16-byte accesses; the host has checked the alignments).
    // Everything it reads is requested in batches ahead of the stores: the compiler cannot prove that C aliases
    // none of the inputs, so a load written after a store waits for it, and 16 * MI * NI dependent round trips
    // to memory would cost more than the product itself.
    const float* bias = e.bias ? e.bias + z0 * a.sBias0 + n0 + wn * TN + ((lane >> 5) << 2) : nullptr;
    const long long tile0 = coff + (long long)(m0 + wm * TM) * e.ldc + n0 + wn * TN;   // first element of the wave tile
    const long long first = tile0 + (long long)(lane & 31) * e.ldc + ((lane >> 5) << 2);
    // results leave through LDS as whole rows of the tile when the rows are 16-byte aligned (see ChunkBf16); the
    // staging piece of a wavefront holds one chunk of C (bf16 or fp32) and one of the pre-activation
    const bool lines16 = ((e.ldc | coff) & 7) == 0;
    constexpr int STAGE_C = ChunkBf16<TN>::BYTES;   // the pre-activation chunk sits behind a bf16 C chunk; an fp32 C chunk uses both
    constexpr int STAGE = ChunkF32<TN>::BYTES > 2 * STAGE_C ? ChunkF32<TN>::BYTES : 2 * STAGE_C;
    const bool pre_lines = lines16 && !e.out_fp32;
    static_assert(STAGE * NW <= LDS_BYTES, "chunk staging must fit in the operand rings");
    char* stage = (char*)lds_all + wave * STAGE;
    const bf16_t* zrow = e.gelu_grad_of ? (const bf16_t*)e.gelu_grad_of + first : nullptr;
    const bf16_t* rrow = e.residual ? (const bf16_t*)e.residual + first : nullptr;
    bf16_t* prow = e.pre_act ? (bf16_t*)e.pre_act + first : nullptr;
    const bool act = e.act == 1, out32 = e.out_fp32 != 0;
    const float alpha = e.alpha;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      const long long ro = (long long)mi * 32 * e.ldc;
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) {
        float4 b4[4];
        uint2 zz[4], rr[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) b4[g] = bias ? *(const float4*)(bias + ni * 32 + g * 8) : make_float4(0.f, 0.f, 0.f, 0.f);
        if (zrow) {
#pragma unroll
          for (int g = 0; g < 4; ++g) zz[g] = *(const uint2*)(zrow + ro + ni * 32 + g * 8);
        }
        if (rrow) {
#pragma unroll
          for (int g = 0; g < 4; ++g) rr[g] = *(const uint2*)(rrow + ro + ni * 32 + g * 8);
        }
        uint2 pv[4];
        float4 cf[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float t[4] = {acc[mi][ni][g * 4] * alpha + b4[g].x, acc[mi][ni][g * 4 + 1] * alpha + b4[g].y,
                        acc[mi][ni][g * 4 + 2] * alpha + b4[g].z, acc[mi][ni][g * 4 + 3] * alpha + b4[g].w};
          if (prow) pv[g] = make_uint2(pack2_bf16(t[0], t[1]), pack2_bf16(t[2], t[3]));
          if (act) gelu4<false>(t);
          if (zrow) {
            const uint2 w = zz[g];
            const float z[4] = {__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xffff0000u), __uint_as_float(w.y << 16),
                                __uint_as_float(w.y & 0xffff0000u)};
            gelu_grad_mul4<false>(t, z);
          }
          if (rrow) {
            const uint2 w = rr[g];
            t[0] += __uint_as_float(w.x << 16); t[1] += __uint_as_float(w.x & 0xffff0000u);
            t[2] += __uint_as_float(w.y << 16); t[3] += __uint_as_float(w.y & 0xffff0000u);
          }
          cf[g] = make_float4(t[0], t[1], t[2], t[3]);
        }
        if (prow) {
          if (pre_lines) chunk_write_bf16<TN>(stage + STAGE_C, ni, pv, lane);
          else {
#pragma unroll
            for (int g = 0; g < 4; ++g) *(uint2*)(prow + ro + ni * 32 + g * 8) = pv[g];
          }
        }
        if (out32) {
          if (lines16) chunk_write_f32<TN>(stage, ni, cf, lane);
          else {
#pragma unroll
            for (int g = 0; g < 4; ++g) *(float4*)((float*)e.C + first + ro + ni * 32 + g * 8) = cf[g];
          }
        } else {
          uint2 cv[4];
#pragma unroll
          for (int g = 0; g < 4; ++g) cv[g] = make_uint2(pack2_bf16(cf[g].x, cf[g].y), pack2_bf16(cf[g].z, cf[g].w));
          if (lines16) chunk_write_bf16<TN>(stage, ni, cv, lane);
          else {
#pragma unroll
            for (int g = 0; g < 4; ++g) *(uint2*)((bf16_t*)e.C + first + ro + ni * 32 + g * 8) = cv[g];
          }
        }
      }
      if (lines16) {
        if (prow && pre_lines) chunk_flush_bf16<TN>(stage + STAGE_C, (bf16_t*)e.pre_act + tile0 + ro, e.ldc, lane);
        if (out32) chunk_flush_f32<TN>(stage, (float*)e.C + tile0 + ro, e.ldc, lane);
        else chunk_flush_bf16<TN>(stage, (bf16_t*)e.C + tile0 + ro, e.ldc, lane);
      }
    }
  } else {
    if (e.bias) e.bias += z0 * a.sBias0;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int m = m0 + wm * TM + mi * 32 + (lane & 31);
          const int n = n0 + wn * TN + ni * 32 + g * 8 + ((lane >> 5) << 2);
          if (m >= a.Mb || n >= a.Nb) continue;
          const float v[4] = {acc[mi][ni][g * 4], acc[mi][ni][g * 4 + 1], acc[mi][ni][g * 4 + 2], acc[mi][ni][g * 4 + 3]};
          epilogue_store4<false>(e, coff, m, n, v, min(4, a.Nb - n));
        }
  }
  OPTIMUS_LAB_STAMP(3);
#endif  // __HIP_DEVICE_COMPILE__
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
  if ((Nb & 3) == 0 && ((size_t)partials & 15) == 0) {  // rows of the partial tiles are 16-byte aligned: one load per split, all in flight together
    const float* p = partials + z * (long long)Mb * Nb + (long long)m * Nb + n;
    const long long sstride = nz * (long long)Mb * Nb;
#pragma unroll 8
    for (int s = 0; s < splits; ++s) {
      const float4 w = *(const float4*)(p + s * sstride);
      v[0] += w.x; v[1] += w.y; v[2] += w.z; v[3] += w.w;
    }
  } else {
    for (int s = 0; s < splits; ++s) {
      const float* p = partials + ((long long)s * nz + z) * (long long)Mb * Nb + (long long)m * Nb + n;
      for (int c = 0; c < nvalid; ++c) v[c] += p[c];
    }
  }
  int z1 = (int)(z / nz0), z0 = (int)(z % nz0);
  if (e.bias) e.bias += z0 * sBias0;
  epilogue_store4<false>(e, z1 * sC1 + z0 * sC0, m, n, v, nvalid);
}

// ---- host side ----
struct Variant {
  int BM, BN, WM, WN;
  bool fast;
};
// index = variant id used by gemm_set_variant
static const Variant kVariants[] = {
    {256, 256, 2, 4, true},   // 0: 8 waves, wave tile 128x64
    {256, 128, 4, 2, true},   // 1: 8 waves, wave tile 64x64
    {128, 256, 2, 4, true},   // 2: 8 waves, wave tile 64x64
    {128, 128, 2, 2, true},   // 3: 4 waves, wave tile 64x64, two workgroups per CU
    {256, 256, 2, 4, true},   // 4: same as 0 (kept so that variant ids stay stable)
    {128, 128, 2, 2, false},  // 5: bounds-checked (ragged shapes)
    {128, 64, 2, 2, true},    // 6: 4 waves, wave tile 64x32: narrow outputs (attention with 64-wide heads)
    {64, 64, 2, 2, true},     // 7: 4 waves, wave tile 32x32: small blocks that need every CU (least bytes per CU)
    {256, 128, 2, 2, true},   // 8: 4 waves, wave tile 128x64 (a quarter fewer LDS bytes per flop than variant 1)
    {128, 256, 2, 2, true},   // 9: 4 waves, wave tile 64x128
};
constexpr int kNumVariants = 10;
constexpr int kGuardVariant = 5;

template <int BM, int BN, int WM, int WN, bool AKC, bool BKC, bool FAST>
static int launch_one(const KArgs& ka, long long nwg, hipStream_t stream) {
  const EpiArgs& e = ka.epi;
  if constexpr (FAST && BM * BN < 256 * 256) {  // (the 256x256 tile has no registers for a second accumulator)
    if (ka.seq_splits > 1) {
      if constexpr (BM + BN >= 384) {
        if (g_loop == 2) {
          hipLaunchKernelGGL((gemm_mfma_kernel<BM, BN, WM, WN, AKC, BKC, true, false, true, 2>), dim3((unsigned)nwg), dim3(WM * WN * 64),
                             0, stream, ka);
          return hip_launch_status();
        }
      }
      hipLaunchKernelGGL((gemm_mfma_kernel<BM, BN, WM, WN, AKC, BKC, true, false, true>), dim3((unsigned)nwg), dim3(WM * WN * 64), 0,
                         stream, ka);
      return hip_launch_status();
    }
  }
  if (ka.seq_splits > 1) return OPTIMUS_EINVAL;
  const bool plain = FAST && ka.splits == 1 && e.alpha == 1.0f && !e.bias && !e.pre_act && !e.act && !e.gelu_grad_of && !e.residual;
  // The 64-wide stages are measured 2-6 % faster than the four-slab ring on the tiles that own a CU (256x256, 256x128,
  // 128x256, 8 or 4 wavefronts) and slower or equal on the tiles that share one (128x128, 128x64, 64x64: several
  // workgroups per CU fill each other's gaps, and the finer ring refills sooner), so each keeps its own loop.
  constexpr bool HAS_LOOP2 = FAST && (BM + BN >= 384);
  if constexpr (HAS_LOOP2) {
    if (g_loop == 2) {
      if (plain)
        hipLaunchKernelGGL((gemm_mfma_kernel<BM, BN, WM, WN, AKC, BKC, true, true, false, 2>), dim3((unsigned)nwg), dim3(WM * WN * 64), 0, stream, ka);
      else
        hipLaunchKernelGGL((gemm_mfma_kernel<BM, BN, WM, WN, AKC, BKC, true, false, false, 2>), dim3((unsigned)nwg), dim3(WM * WN * 64), 0, stream, ka);
      return hip_launch_status();
    }
  }
  if (plain) {
    if constexpr (FAST)
      hipLaunchKernelGGL((gemm_mfma_kernel<BM, BN, WM, WN, AKC, BKC, true, true>), dim3((unsigned)nwg), dim3(WM * WN * 64), 0, stream, ka);
  } else {
    hipLaunchKernelGGL((gemm_mfma_kernel<BM, BN, WM, WN, AKC, BKC, FAST, false>), dim3((unsigned)nwg), dim3(WM * WN * 64), 0, stream, ka);
  }
  return hip_launch_status();
}

template <int BM, int BN, int WM, int WN, bool FAST>
static int launch_layout(const GemmDesc& d, const KArgs& ka, long long nwg, hipStream_t stream) {
  if (d.a_kcontig && !d.b_kcontig) return launch_one<BM, BN, WM, WN, true, false, FAST>(ka, nwg, stream);
  if (d.a_kcontig && d.b_kcontig) return launch_one<BM, BN, WM, WN, true, true, FAST>(ka, nwg, stream);
  if (!d.a_kcontig && !d.b_kcontig) return launch_one<BM, BN, WM, WN, false, false, FAST>(ka, nwg, stream);
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
  if (d.Mb % v.BM || d.Nb % v.BN || d.Kp % (2 * BK)) return false;  // slabs are walked in pairs
  // buffer addressing: per-lane byte offset (< 256 * ld * 2) plus slab byte offset (< Kp * ld * 2) inside a 2 GiB window
  const long long ld = d.lda > d.ldb ? d.lda : d.ldb;
  return 512 * ld < (1LL << 30) && 2 * (long long)d.Kp * ld < (1LL << 30);
}

// Tile shape and panel split for one product.  The split is chosen from ONE device's block only (never from the
// batch count), so that grid mode and device mode add the same slabs in the same order and give identical bits; the
// tile shape changes no bit and may be chosen for the whole launch (GemmDesc::plan_for_batch, see make_plan).
// Cost model (microseconds, calibrated on MI355X): fixed launch/prologue/epilogue cost, plus the slabs one
// workgroup walks times the measured time per slab of the variant, times the rounds needed to place all
// workgroups; a split adds the combine launch and the fp32 partial tiles written once and read once.
struct Plan {
  int variant;
  int splits;
  int seq;  // 1: the split is emulated inside each workgroup (KArgs::seq_splits): same bits, no partial tiles, no combine
};

// have_ws: the caller's workspace holds the partial tiles of the planned split.  Without it the same split is
// emulated inside each workgroup (identical bits, see KArgs::seq_splits), so a result never depends on the workspace.
// compute units of the current device (the planner's unit of parallelism); 256 when there is no device to ask
static int num_cus() {
  static int cached[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) { (void)hipGetLastError(); return 256; }
  if (cached[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) { (void)hipGetLastError(); n = 256; }
    cached[dev] = n;
  }
  return cached[dev];
}

static Plan make_plan(const GemmDesc& d, bool vec_ok, bool have_ws) {
  const bool allow_split = true;
  Plan best = {kGuardVariant, 1, 0};
  const int forced = g_variant.load();                       // one consistent view of the hooks per plan
  const int forced_corun = d.corun > 0 ? g_corun_variant[d.corun - 1].load() : -1;
  if (!vec_ok || forced == kGuardVariant) return best;  // the fast kernels only have the vector epilogue
  // per candidate: variant id, workgroups resident per CU, fixed cost (launch, prologue, epilogue: us and us per MiB
  // of output), and the time per slab of one workgroup: alone on the chip (t_lone), with every CU holding one
  // workgroup (t_full: all CUs' loads share the L2 fabric; the rise is steep only near full occupancy, hence the
  // square), and the increment per further workgroup resident on the same CU (t_more).  Measured on MI355X with the
  // kernels as of the commit that last touched this table (one forced-variant sweep over the products of the
  // benchmark configurations 3-5); tests/test_gpu_planner.py fails when the kernels drift away from it.
  struct Cand { int v, per_cu; float fixed_us, out_us_per_mib, t_lone, t_full, t_more; };
  constexpr int kCands = 8;
  static const Cand cand[kCands] = {{0, 1, 12.0f, 0.15f, 0.54f, 0.64f, 0.00f},
                               {1, 1, 8.0f, 0.30f, 0.24f, 0.40f, 0.00f},
                               {2, 1, 8.0f, 0.30f, 0.24f, 0.405f, 0.00f},
                               {3, 2, 5.5f, 0.45f, 0.20f, 0.25f, 0.21f},
                               {6, 4, 4.5f, 0.50f, 0.19f, 0.21f, 0.133f},
                               {7, 5, 4.0f, 0.50f, 0.14f, 0.155f, 0.045f},
                               {8, 1, 8.0f, 0.30f, 0.24f, 0.41f, 0.00f},
                               {9, 1, 8.0f, 0.30f, 0.24f, 0.415f, 0.00f}};
  const long long slabs = (long long)d.nl * (d.Kp / BK);
  const long long ncu = num_cus();
  const bool splittable = allow_split && d.nl > 1 && !d.skip_upper && !d.k_hi_diag && !d.k_lo_diag;
  const float out_mib = (float)d.Mb * (float)d.Nb * 2.0f / 1048576.0f;
  float best_cost = 0.f;
  bool found = false;
  // Two passes.  The panel split changes the order in which a result is added up, so it is chosen from ONE block's
  // shape alone, as if the product ran by itself (pass 0): a product has the same bits wherever it is launched from.
  // The tile shape does not change them (every element walks the same slabs in the same order whatever tile it
  // lies in: the variants give identical bits, which the tests check), so a launch that covers several blocks
  // (the whole grid, the matrices of a batch of heads) or that shares the chip with a second product then picks
  // its tile, for that split, for the workgroups and the company it really has (pass 1).
  const long long batch = d.plan_for_batch ? (long long)(d.nz0 > 0 ? d.nz0 : 1) * (d.nz1 > 0 ? d.nz1 : 1) : 1;
  for (int pass = 0; pass < (batch > 1 || d.corun > 0 ? 2 : 1); ++pass) {
  const int fixed_sp = pass == 0 ? 0 : best.splits;
  if (pass == 1) found = false;
  for (int ci = 0; ci < kCands; ++ci) {
    const Cand& c = cand[ci];
    const int v = c.v;
    if (forced >= 0 && v != (forced == 4 ? 0 : forced)) continue;
    if (pass == 1 && forced_corun >= 0 && v != forced_corun) continue;
    if (!variant_fits(kVariants[v], d)) continue;
    const long long tiles = (long long)(d.Mb / kVariants[v].BM) * (d.Nb / kVariants[v].BN) * (pass == 0 ? 1 : batch);
    for (int sp = fixed_sp ? fixed_sp : 1; sp <= (fixed_sp ? fixed_sp : 8); ++sp) {
      if (!fixed_sp && sp > 1 && (!splittable || slabs / sp < 8)) break;
      const long long wgs = tiles * sp;
      const long long cap = ncu * c.per_cu;
      const long long rounds = (wgs + cap - 1) / cap;
      const long long in_round = wgs < cap ? wgs : cap;
      const int resident = (int)((in_round + ncu - 1) / ncu);             // workgroups on the fullest CU
      const float busy = in_round >= ncu ? 1.0f : (float)in_round / (float)ncu;  // share of the CUs in use
      float t_slab = c.t_lone + (c.t_full - c.t_lone) * busy * busy + c.t_more * (float)(resident - 1);
      // the 128x128 tile depends on the operand layouts: both k-contiguous (A B^T) is its slowest form, one of each its fastest
      if (v == 3) t_slab *= d.a_kcontig && d.b_kcontig ? 1.14f : (d.a_kcontig ? 0.92f : 1.04f);
      if (v == 6 && d.a_kcontig && d.b_kcontig) t_slab *= 1.18f;
      if (v == 7 && !d.a_kcontig) t_slab *= 1.25f;   // both operands through the transposing LDS reads
      const float per_wg = (float)((((slabs + sp - 1) / sp) + 1) & ~1LL) * t_slab;
      // split: the combine launch, and the fp32 partial tiles read back by it (their writes overlap the products)
      const float traffic_us =
          sp > 1 ? 4.0f + (float)sp * (float)d.Mb * (float)d.Nb * 4.0f / 3.0e6f * (pass == 0 ? 1.0f : (float)batch) : 0.f;
      float cost = c.fixed_us + c.out_us_per_mib * out_mib * (pass == 0 ? 1.0f : (float)batch) + (float)rounds * per_wg + traffic_us;
      // Two products that run side by side on two streams (the pairs of the layer's backward pass): the tiles of 8
      // wavefronts, which take a CU's LDS and registers alone, are the better partners, also where such a tile leaves
      // half the CUs idle when the product runs by itself (the other product's workgroups take those).  Measured on
      // the backward pass of the 4096-wide layers (one device of the q = 4 / q = 8 grids): 256x128 tiles for both
      // products 0.55 / 0.61 ms, 128x128 tiles for both 0.64 / 0.72 ms, 256x128 for the chain and 128x128 for the
      // branch 0.65 / 0.69 ms, the reverse 0.58 / 0.63 ms.
      if (d.corun > 0 && c.per_cu >= 2 && pass == 1 && batch == 1) cost *= 1.25f;
      if (!found || cost < best_cost) {
        found = true;
        best_cost = cost;
        best = {v, sp, 0};
      }
      // A launch with many blocks has workgroups enough without the split: one workgroup then walks all the slabs of
      // its tile and adds them up range by range as the split workgroups and their combine would (identical bits).
      if (pass == 1 && batch > 1 && sp > 1 && kVariants[v].BM * kVariants[v].BN < 256 * 256) {
        const long long rounds1 = (tiles + cap - 1) / cap;
        const long long in1 = tiles < cap ? tiles : cap;
        const int res1 = (int)((in1 + ncu - 1) / ncu);
        const float busy1 = in1 >= ncu ? 1.0f : (float)in1 / (float)ncu;
        const float t1 = c.t_lone + (c.t_full - c.t_lone) * busy1 * busy1 + c.t_more * (float)(res1 - 1);
        const float cost1 = c.fixed_us + c.out_us_per_mib * out_mib * (float)batch + (float)rounds1 * (float)slabs * t1;
        if (cost1 < best_cost) {
          best_cost = cost1;
          best = {v, sp, 1};
        }
      }
    }
  }
  }
  if (best.splits > 1 && !best.seq && !have_ws) {
    // No workspace: the same split, walked inside the workgroups (same bits).  One workgroup then owns all slabs of its
    // tile, so the tile is picked again for that walk: the tile with the least estimated time among those that have
    // registers for the second accumulator set (not 256x256).
    best.seq = 1;
    float seq_best = 0.f;
    int seq_v = -1;
    for (int ci = 0; ci < kCands; ++ci) {
      const Cand& c = cand[ci];
      if (kVariants[c.v].BM * kVariants[c.v].BN >= 256 * 256 || !variant_fits(kVariants[c.v], d)) continue;
      if (forced >= 0 && c.v != forced) continue;
      const long long tiles = (long long)(d.Mb / kVariants[c.v].BM) * (d.Nb / kVariants[c.v].BN) * batch;
      const long long cap = ncu * c.per_cu;
      const long long rounds = (tiles + cap - 1) / cap;
      const long long in_round = tiles < cap ? tiles : cap;
      const int resident = (int)((in_round + ncu - 1) / ncu);
      const float busy = in_round >= ncu ? 1.0f : (float)in_round / (float)ncu;
      const float t = c.t_lone + (c.t_full - c.t_lone) * busy * busy + c.t_more * (float)(resident - 1);
      const float cost = c.fixed_us + c.out_us_per_mib * out_mib * (float)batch + (float)rounds * (float)slabs * t;
      if (seq_v < 0 || cost < seq_best) { seq_best = cost; seq_v = c.v; }
    }
    if (seq_v >= 0) best.variant = seq_v;
    else if (kVariants[best.variant].BM * kVariants[best.variant].BN >= 256 * 256) {
      static const int order[7] = {1, 2, 8, 9, 3, 6, 7};
      for (int k = 0; k < 7; ++k)
        if (variant_fits(kVariants[order[k]], d)) { best.variant = order[k]; break; }
    }
  }
  return best;
}

static bool epilogue_vec_ok(const GemmDesc& d) {
  return (d.ldc % 4 == 0) && (d.sC0 % 4 == 0) && (d.sC1 % 4 == 0) && aligned16(d.C) && (!d.pre_act || aligned16(d.pre_act)) &&
         (!d.gelu_grad_of || aligned16(d.gelu_grad_of)) && (!d.residual || aligned16(d.residual)) &&
         (!d.bias || (aligned16(d.bias) && d.sBias0 % 4 == 0));
}

size_t gemm_partials_bytes(const GemmDesc& d, int splits) {
  if (splits <= 1) return 0;
  return (size_t)splits * (size_t)d.nz0 * d.nz1 * (size_t)d.Mb * d.Nb * sizeof(float);
}

// Workspace the planned launch wants for its partial tiles: 0 when there is no split or when the split is emulated
// inside the workgroups anyway.
size_t gemm_plan_bytes(const GemmDesc& d) {
  if (!gemm_mfma_supported(d)) return 0;
  const Plan p = make_plan(d, epilogue_vec_ok(d), true);
  return p.seq ? 0 : gemm_partials_bytes(d, p.splits);
}

// The plan a launch of d would use (host arithmetic only; nothing is enqueued): {tile variant, panel split,
// 1 if the split is walked inside the workgroups}.  False when the matrix-core kernels do not take the product.
bool gemm_plan_of(const GemmDesc& d, bool have_ws, int out[3]) {
  if (!gemm_mfma_supported(d)) return false;
  const Plan p = make_plan(d, epilogue_vec_ok(d), have_ws);
  out[0] = p.variant; out[1] = p.splits; out[2] = p.seq;
  return true;
}

int launch_gemm_mfma(const GemmDesc& d, hipStream_t stream) {
  if (!gemm_mfma_supported(d)) return OPTIMUS_EINVAL;
  const bool vec_ok = epilogue_vec_ok(d);
  // d.partials != nullptr means the caller provided the workspace that the planned split asked for
  const Plan plan = make_plan(d, vec_ok, d.partials != nullptr);
  const int vi = plan.variant;
  g_last_plan = plan.variant | (plan.splits << 8) | (plan.seq << 16);
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
  {
    const long long per_xcd = ((long long)ka.tiles_m * ka.tiles_n + 7) / 8;
    int g = 1;
    while ((long long)(2 * g) * (2 * g) * v.BM <= per_xcd * v.BN * 2 && 2 * g <= 16) g *= 2;  // g ~ sqrt(per_xcd * BN / BM)
    ka.group = g;
  }
  ka.skip_upper = d.skip_upper; ka.k_hi_diag = d.k_hi_diag; ka.k_lo_diag = d.k_lo_diag;
  ka.splits = plan.seq ? 1 : plan.splits;
  ka.seq_splits = plan.seq ? plan.splits : 1;
  ka.partials = d.partials;
  ka.nz = (long long)d.nz0 * d.nz1;
  EpiArgs& e = ka.epi;
  e.alpha = d.alpha; e.bias = d.bias; e.C = d.C; e.pre_act = d.pre_act; e.gelu_grad_of = d.gelu_grad_of;
  e.residual = d.residual; e.ldc = d.ldc; e.act = d.act; e.out_fp32 = d.out_fp32; e.in_bf16 = 1;
  e.vec_ok = vec_ok ? 1 : 0;
  if (ka.splits > 1 && !d.partials) return OPTIMUS_EWORKSPACE;
  long long nwg = (long long)ka.tiles_m * ka.tiles_n * ka.nz * ka.splits;
  if (nwg <= 0 || nwg > 0x7fffffffLL) return OPTIMUS_ESHAPE;
  int rc;
  switch (vi) {
    case 0: rc = launch_layout<256, 256, 2, 4, true>(d, ka, nwg, stream); break;
    case 1: rc = launch_layout<256, 128, 4, 2, true>(d, ka, nwg, stream); break;
    case 2: rc = launch_layout<128, 256, 2, 4, true>(d, ka, nwg, stream); break;
    case 3: rc = launch_layout<128, 128, 2, 2, true>(d, ka, nwg, stream); break;
    case 4: rc = launch_layout<256, 256, 2, 4, true>(d, ka, nwg, stream); break;
    case 6: rc = launch_layout<128, 64, 2, 2, true>(d, ka, nwg, stream); break;
    case 7: rc = launch_layout<64, 64, 2, 2, true>(d, ka, nwg, stream); break;
    case 8: rc = launch_layout<256, 128, 2, 2, true>(d, ka, nwg, stream); break;
    case 9: rc = launch_layout<128, 256, 2, 2, true>(d, ka, nwg, stream); break;
    default: rc = launch_layout<128, 128, 2, 2, false>(d, ka, nwg, stream); break;
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

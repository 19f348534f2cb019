// Shared host/device declarations of the library's internals (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "optimus.h"

namespace optimus {

typedef unsigned short bf16_t;  // raw bf16 bit pattern

typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((unsigned)v) << 16); }
// round-to-nearest-even, NaN stays NaN: gfx950 converts in hardware (v_cvt_pk_bf16_f32)
__device__ __forceinline__ unsigned pack2_bf16(float lo, float hi) {
  f32x2_t v = {lo, hi};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(pack2_bf16(f, 0.f) & 0xffffu); }

__device__ __forceinline__ float gelu_exact(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752440f)); }
__device__ __forceinline__ float gelu_grad_exact(float x) {
  float cdf = 0.5f * (1.0f + erff(x * 0.70710678118654752440f));
  float pdf = 0.39894228040143267794f * __expf(-0.5f * x * x);
  return cdf + x * pdf;
}

// Same two functions for the bf16 kernels, short enough to inline 64-256 times per lane: the normal CDF through the
// rational approximation 7.1.26 of Abramowitz & Stegun (absolute error of erf below 1.5e-7, three orders below one
// bf16 rounding).  Written on the complementary side, 0.5 * erfc(|x| / sqrt 2), so that the negative tail does not
// cancel.
__device__ __forceinline__ float half_erfc_abs(float x, float& gauss) {  // 0.5 * erfc(|x|/sqrt2); gauss = exp(-x^2/2)
  const float u = fabsf(x) * 0.70710678118654752440f;
  const float t = __frcp_rn(1.0f + 0.3275911f * u);
  gauss = __expf(-u * u);
  const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
  return 0.5f * poly * gauss;
}
__device__ __forceinline__ float gelu_fast(float x) {
  float g;
  const float tail = half_erfc_abs(x, g);
  return x * (x >= 0.f ? 1.0f - tail : tail);
}
__device__ __forceinline__ float gelu_grad_fast(float x) {
  float g;
  const float tail = half_erfc_abs(x, g);
  return (x >= 0.f ? 1.0f - tail : tail) + x * 0.39894228040143267794f * g;
}

// One (possibly batched, possibly multi-panel) product  C = alpha * sum_l op(A_l) op(B_l)  + epilogue.
// All strides are in elements of the operand's own type.  A batch index z in [0, nz1*nz0) is split as
// z1 = z / nz0, z0 = z % nz0; operand X of batch z starts at X + z1*sX1 + z0*sX0.
struct GemmDesc {
  const void* A;
  const void* B;
  void* C;
  int Mb, Nb;   // output block dims
  int Kp;       // contraction length of one panel
  int nl;       // number of panels accumulated into one output
  int lda, ldb, ldc;
  long long sAl, sBl;  // panel strides
  int nz0, nz1;
  long long sA0, sA1, sB0, sB1, sC0, sC1;
  int a_kcontig;  // 1: A panel stored [Mb][Kp] (k contiguous); 0: stored [Kp][Mb]
  int b_kcontig;  // 1: B panel stored [Nb][Kp] (k contiguous); 0: stored [Kp][Nb]
  int dtype;      // OPTIMUS_FP32 / OPTIMUS_BF16 (inputs, and outputs unless out_fp32)
  // epilogue
  float alpha;
  const float* bias;  // fp32, indexed bias[z0*sBias0 + n]
  long long sBias0;
  void* pre_act;             // same layout as C (ldc, sC0, sC1), dtype of inputs
  int act;                   // 1 = GeLU
  const void* gelu_grad_of;  // same layout as C
  const void* residual;      // same layout as C
  int out_fp32;
  // causal structure of attention products (square s x s score matrices, single panel)
  int skip_upper;  // 1: output tiles entirely above the diagonal are not computed (left untouched)
  int k_hi_diag;   // 1: contraction limited to k < (last row of the tile)+1
  int k_lo_diag;   // 1: contraction starts at k >= first row of the tile
  // split of the panel loop over several workgroups (fixed-order combine)
  int splits;          // 1 = none
  float* partials;     // workspace [splits][nz][Mb][Nb] fp32 when splits > 1
  // 0: the product has the chip to itself; 1 / 2: it is one of two products that the layer's backward pass runs
  // side by side on two streams (1: activation-gradient chain, 2: parameter-gradient branch)
  int corun;
  // 1: the tile shape may be chosen for all nz0 * nz1 blocks of the launch (whole-grid launches of a product);
  // 0: from one block's shape only (the batched products of attention: the planner's cost model is calibrated on
  // dense products and mispredicts their diagonal-trimmed, short-k shapes)
  int plan_for_batch;
};

int launch_gemm(const GemmDesc& d, hipStream_t stream);           // picks MFMA or generic kernel
int launch_gemm_generic(const GemmDesc& d, hipStream_t stream);    // scalar FMA kernel, any shape
int launch_gemm_mfma(const GemmDesc& d, hipStream_t stream);       // bf16 matrix-core kernel
bool gemm_mfma_supported(const GemmDesc& d);
int launch_mfma_rate(float* out, int workgroups, int iters, int random_data, hipStream_t stream);   // probe.hip
size_t gemm_plan_bytes(const GemmDesc& d);                         // workspace the planned launch wants (0: none)
bool gemm_plan_of(const GemmDesc& d, bool have_ws, int out[3]);
size_t gemm_partials_bytes(const GemmDesc& d, int splits);
// force a specific kernel variant (benchmark sweeps); -1 = automatic
void gemm_set_variant(int v);
void gemm_set_corun_variants(int chain_v, int branch_v);
int gemm_get_variant();
int gemm_last_plan();

// element-wise / reduction kernels
int launch_pack(const void* src, void* dst, long long R, long long C, int q, int elem_bytes, bool unpack,
                hipStream_t stream);
int launch_reduce_partials(const float* parts, void* dst, long long n, int count, int dtype, hipStream_t stream);
int launch_colsum(const void* X, float* out, int rows, int cols, int ld, int nz, long long sX, long long sOut,
                  int dtype, hipStream_t stream);

struct LnDesc {
  int rows, cols;  // block dims M/q, H/q
  int H;           // full hidden size
  int q;
  int i0, ni;      // grid rows handled: i0 .. i0+ni-1
  int j0, nj;      // grid cols handled
  int dtype;
  float eps;
};
// true if launch_ln_apply / launch_ln_bwd_apply with own_ready = false compute and exchange the partials of a whole
// grid row inside one launch (then no separate statistics launch is needed before them)
bool ln_rowgroup_ok(const LnDesc& d);
int launch_ln_stats(const void* X, float* stats, const LnDesc& d, hipStream_t stream);
int launch_ln_apply(const void* X, const float* gamma, const float* beta, void* Y, void* xhat, float* rstd,
                    float* stats, const LnDesc& d, bool own_stats_ready, hipStream_t stream);
int launch_ln_bwd_stats(const void* dY, const void* xhat, const float* gamma, float* stats, const LnDesc& d,
                        hipStream_t stream);
int launch_ln_bwd_apply(const void* dY, const void* xhat, const float* rstd, const float* gamma, const void* dres,
                        void* dX, float* stats, const LnDesc& d, bool own_stats_ready, hipStream_t stream);
// small blocks (narrow column strips; the kernel is latency-bound there)
bool colsum_narrow(int rows, int cols);
int launch_ln_param_grads(const void* dY, const void* xhat, float* dgamma_part, float* dbeta_part, const LnDesc& d,
                          hipStream_t stream);

// softmax over rows of nmat square [s x s] score matrices (fp32 in, bf16 out), optional causal mask
int launch_softmax_fwd(const float* S, void* P, int nmat, int s, int causal, hipStream_t stream);
// dS = P * (dP - rowsum(dP * P)); dP fp32, P bf16, dS bf16
int launch_softmax_bwd(const float* dP, const void* P, void* dS, int nmat, int s, int causal, hipStream_t stream);

// Fused local attention (no [s x s] tensor in memory) for ndev consecutive device blocks of one launch.
struct AttnFusedDesc {
  const void* qkv;      // first device block, [nb*s x ld] per device
  void* attn;           // [nb*s x ldo] per device: written by the forward, read by the backward
  float* lse;           // [ndev][nb*nh][s]: log sum exp of the scaled scores of every row
  const void* d_attn;   // backward only
  void* d_qkv;          // backward only
  float* delta;         // backward scratch [ndev][nb*nh][s]
  int s, d, nb, nh, ld, ldo, ndev;
  long long dev_qkv, dev_attn;  // element strides between consecutive device blocks
  int causal;
};
bool attn_fused_supported(int d);
int launch_attn_fused_fwd(const AttnFusedDesc& d, hipStream_t stream);
int launch_attn_fused_bwd(const AttnFusedDesc& d, hipStream_t stream);

// model ends (embedding, cross entropy) on the devices i0..i0+ni-1 x j0..j0+nj-1 of the grid
struct EndDesc {
  int rows, vb, hb, q, v;   // M/q, v/q, h/q, grid size, vocabulary size
  int i0, ni, j0, nj;
  int dtype;
};
int launch_embedding_fwd(const int* tokens, const void* table, void* out, const EndDesc& d, hipStream_t stream);
int launch_embedding_bwd(const int* tokens, const void* dX, float* d_table, const EndDesc& d, hipStream_t stream);
int launch_ce_stats(const void* logits, float* stats, const EndDesc& d, hipStream_t stream);
int launch_ce_stats_final(const void* logits, const int* labels, float* stats, float* loss, float* lse, const EndDesc& d,
                          hipStream_t stream);
int launch_ce_finalize(const void* logits, const int* labels, const float* stats, float* loss, float* lse, const EndDesc& d,
                       hipStream_t stream);
int launch_ce_bwd(const void* logits, const int* labels, const float* lse, void* d_logits, float scale, const EndDesc& d,
                  hipStream_t stream);

// optimus_layer_fwd, optionally without its last product (used by the checkpointed stack's recomputation)
int layer_forward(const optimus_layer_cfg* c, const optimus_layer_tensors* t, int i, int j, void* ws, size_t ws_bytes,
                  void* stream, bool skip_out);

inline int hip_launch_status() { return hipGetLastError() == hipSuccess ? OPTIMUS_OK : OPTIMUS_EHIP; }

}  // namespace optimus

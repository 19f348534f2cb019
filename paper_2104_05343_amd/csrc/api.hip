// C ABI of the library: argument validation, block addressing on the q x q grid, and the composition of the
// kernels into the paper's operations (Algorithms 1-3, Section 3.2).  Every entry point validates first and
// enqueues nothing on error.
#include <math.h>

#include <mutex>

#include "common.hpp"

using namespace optimus;

// Scratch of the entry point that allocates nothing (optimus_attention_fused_bwd_static): one array per GPU the library
// runs on, held until the process ends.  In host code the array's NAME is only a handle for hipGetSymbolAddress, never
// a device address: every use goes through static_scratch(), which looks the address up once per device.
constexpr size_t kStaticScratchBytes = OPTIMUS_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

inline hipStream_t as_stream(void* s) { return (hipStream_t)s; }

int check_coords(int q, int i, int j) {
  if (q <= 0) return OPTIMUS_ESHAPE;
  if (i == OPTIMUS_ALL && j == OPTIMUS_ALL) return OPTIMUS_OK;
  if (i < 0 || j < 0 || i >= q || j >= q) return OPTIMUS_ECOORD;
  return OPTIMUS_OK;
}
inline bool is_grid(int i, int j) { return i == OPTIMUS_ALL && j == OPTIMUS_ALL; }
inline size_t esize(int dtype) { return dtype == OPTIMUS_BF16 ? 2 : 4; }
inline const void* off(const void* p, long long elems, size_t es) { return p ? (const char*)p + elems * (long long)es : nullptr; }
inline void* off(void* p, long long elems, size_t es) { return p ? (char*)p + elems * (long long)es : nullptr; }
inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

int check_mkn(int64_t M, int64_t K, int64_t N, int q) {
  if (q <= 0 || M <= 0 || K <= 0 || N <= 0) return OPTIMUS_ESHAPE;
  if (M % q || K % q || N % q) return OPTIMUS_ESHAPE;
  if (M / q > 0x7fffffff || K / q > 0x7fffffff || N / q > 0x7fffffff) return OPTIMUS_ESHAPE;
  return OPTIMUS_OK;
}

// Owner-view descriptor of one SUMMA product for device (i, j), or for the whole grid.
//   AB : C_ij = sum_l A_il B_lj ;  ABT: C_ij = sum_l A_il (B_jl)^T ;  ATB: C_ij = sum_l (A_li)^T B_lj
GemmDesc summa_desc(int form, const void* A, const void* B, void* C, int64_t M, int64_t K, int64_t N, int q, int i, int j,
                    int dtype, const optimus_epilogue* epi) {
  GemmDesc d = {};
  const int Mb = (int)(M / q), Nb = (int)(N / q), Kp = (int)(K / q);
  d.Mb = Mb; d.Nb = Nb; d.Kp = Kp; d.nl = q; d.dtype = dtype;
  const long long blkA = (long long)Mb * Kp, blkB = (long long)Kp * Nb, blkC = (long long)Mb * Nb;
  if (form == OPTIMUS_FORM_ATB) { d.a_kcontig = 0; d.lda = Mb; d.sAl = q * blkA; d.sA1 = blkA; d.sA0 = 0; }
  else { d.a_kcontig = 1; d.lda = Kp; d.sAl = blkA; d.sA1 = q * blkA; d.sA0 = 0; }
  if (form == OPTIMUS_FORM_ABT) { d.b_kcontig = 1; d.ldb = Kp; d.sBl = blkB; d.sB0 = q * blkB; d.sB1 = 0; }
  else { d.b_kcontig = 0; d.ldb = Nb; d.sBl = q * blkB; d.sB0 = blkB; d.sB1 = 0; }
  d.ldc = Nb; d.sC1 = q * blkC; d.sC0 = blkC;
  d.alpha = 1.0f;
  d.splits = 1;
  const size_t es = esize(dtype);
  const bool out32 = epi && epi->out_fp32 && dtype == OPTIMUS_BF16;
  d.out_fp32 = out32 ? 1 : 0;
  const size_t ces = out32 ? 4 : es;
  const float* bias = epi ? epi->bias : nullptr;
  void* pre = epi ? epi->pre_act : nullptr;
  const void* gg = epi ? epi->gelu_grad_of : nullptr;
  const void* res = epi ? epi->residual : nullptr;
  d.act = epi ? epi->act : 0;
  d.sBias0 = Nb;
  if (is_grid(i, j)) {
    d.nz1 = q; d.nz0 = q; d.plan_for_batch = 1;
    d.A = A; d.B = B; d.C = C;
    d.bias = bias; d.pre_act = pre; d.gelu_grad_of = gg; d.residual = res;
  } else {
    d.nz1 = 1; d.nz0 = 1;
    d.A = off(A, i * d.sA1 + j * d.sA0, es);
    d.B = off(B, i * d.sB1 + j * d.sB0, es);
    const long long co = i * d.sC1 + j * d.sC0;
    d.C = off(C, co, ces);
    d.bias = bias ? bias + (long long)j * Nb : nullptr;
    d.pre_act = off(pre, co, es);
    d.gelu_grad_of = off(gg, co, es);
    d.residual = off(res, co, es);
  }
  return d;
}

int run_summa(int form, const void* A, const void* B, void* C, int64_t M, int64_t K, int64_t N, int q, int i, int j, int dtype,
              const optimus_epilogue* epi, void* ws, size_t ws_bytes, void* stream, int corun = 0) {
  if (!A || !B || !C) return OPTIMUS_EINVAL;
  if (form < 0 || form > 2) return OPTIMUS_EINVAL;
  if (dtype != OPTIMUS_FP32 && dtype != OPTIMUS_BF16) return OPTIMUS_EDTYPE;
  int rc = check_mkn(M, K, N, q);
  if (rc) return rc;
  rc = check_coords(q, i, j);
  if (rc) return rc;
  if (epi && (epi->act < 0 || epi->act > 1)) return OPTIMUS_EINVAL;
  GemmDesc d = summa_desc(form, A, B, C, M, K, N, q, i, j, dtype, epi);
  d.corun = corun;
  if (gemm_mfma_supported(d)) {
    // a planned panel split writes its partial tiles to the workspace if it is there and large enough; otherwise the
    // same split is emulated inside the workgroups: the bits of a result do not depend on the workspace
    const size_t need = gemm_plan_bytes(d);
    if (need > 0 && ws && ws_bytes >= need) d.partials = (float*)ws;
  }
  return launch_gemm(d, as_stream(stream));
}

struct AttnDims {
  int nb, nh, d, s, ld, ldo;
  long long blk_qkv, blk_attn, blk_probs, nmat;
};
int attn_dims(int b, int s, int h, int n, int q, AttnDims* a) {
  if (q <= 0 || b <= 0 || s <= 0 || h <= 0 || n <= 0) return OPTIMUS_ESHAPE;
  if (b % q || n % q || h % n) return OPTIMUS_ESHAPE;
  a->nb = b / q; a->nh = n / q; a->d = h / n; a->s = s;
  if (a->d % 8 || s % 8 || s > 4096) return OPTIMUS_ESHAPE;
  a->ld = 3 * h / q; a->ldo = h / q;
  a->blk_qkv = (long long)a->nb * s * a->ld;
  a->blk_attn = (long long)a->nb * s * a->ldo;
  a->nmat = (long long)a->nb * a->nh;
  a->blk_probs = a->nmat * s * s;
  return OPTIMUS_OK;
}
size_t attn_ws_bytes(const AttnDims& a) {
  return align256((size_t)a.blk_probs * 4) + align256((size_t)a.blk_probs * 2);
}

GemmDesc attn_base_desc(const AttnDims& a) {
  GemmDesc d = {};
  d.dtype = OPTIMUS_BF16; d.nl = 1; d.nz1 = a.nb; d.nz0 = a.nh; d.alpha = 1.0f; d.splits = 1;
  return d;
}

int attention_fwd_device(const bf16_t* qkv_blk, bf16_t* probs_blk, bf16_t* attn_blk, const AttnDims& a, int causal, void* ws,
                         hipStream_t st) {
  float* scores = (float*)ws;
  const long long ss = (long long)a.s * a.s;
  const float scale = 1.0f / sqrtf((float)a.d);
  // S = Q K^T / sqrt(d)
  GemmDesc g = attn_base_desc(a);
  g.A = qkv_blk; g.B = qkv_blk + a.d; g.C = scores;
  g.Mb = a.s; g.Nb = a.s; g.Kp = a.d;
  g.a_kcontig = 1; g.b_kcontig = 1; g.lda = a.ld; g.ldb = a.ld; g.ldc = a.s;
  g.sA1 = (long long)a.s * a.ld; g.sA0 = 3 * a.d; g.sB1 = g.sA1; g.sB0 = g.sA0;
  g.sC1 = a.nh * ss; g.sC0 = ss;
  g.alpha = scale; g.out_fp32 = 1; g.skip_upper = causal;
  int rc = launch_gemm(g, st);
  if (rc) return rc;
  rc = launch_softmax_fwd(scores, probs_blk, (int)a.nmat, a.s, causal, st);
  if (rc) return rc;
  // O = P V
  GemmDesc o = attn_base_desc(a);
  o.A = probs_blk; o.B = qkv_blk + 2 * a.d; o.C = attn_blk;
  o.Mb = a.s; o.Nb = a.d; o.Kp = a.s;
  o.a_kcontig = 1; o.b_kcontig = 0; o.lda = a.s; o.ldb = a.ld; o.ldc = a.ldo;
  o.sA1 = a.nh * ss; o.sA0 = ss; o.sB1 = (long long)a.s * a.ld; o.sB0 = 3 * a.d;
  o.sC1 = (long long)a.s * a.ldo; o.sC0 = a.d;
  o.k_hi_diag = causal;
  return launch_gemm(o, st);
}

int attention_bwd_device(const bf16_t* qkv_blk, const bf16_t* probs_blk, const bf16_t* dattn_blk, bf16_t* dqkv_blk,
                         const AttnDims& a, int causal, void* ws, hipStream_t st) {
  float* dP = (float*)ws;
  bf16_t* dS = (bf16_t*)((char*)ws + align256((size_t)a.blk_probs * 4));
  const long long ss = (long long)a.s * a.s;
  const float scale = 1.0f / sqrtf((float)a.d);
  const long long q1 = (long long)a.s * a.ld, q0 = 3 * a.d;      // (sequence, head) strides inside a qkv block
  const long long o1 = (long long)a.s * a.ldo, o0 = a.d;         // inside an attn block
  const long long p1 = a.nh * ss, p0 = ss;                       // inside probs / scratch
  int rc;
  {  // dV = P^T dO   (contraction over query position t >= key position u)
    GemmDesc g = attn_base_desc(a);
    g.A = probs_blk; g.B = dattn_blk; g.C = dqkv_blk + 2 * a.d;
    g.Mb = a.s; g.Nb = a.d; g.Kp = a.s;
    g.a_kcontig = 0; g.b_kcontig = 0; g.lda = a.s; g.ldb = a.ldo; g.ldc = a.ld;
    g.sA1 = p1; g.sA0 = p0; g.sB1 = o1; g.sB0 = o0; g.sC1 = q1; g.sC0 = q0;
    g.k_lo_diag = causal;
    if ((rc = launch_gemm(g, st))) return rc;
  }
  {  // dP = dO V^T
    GemmDesc g = attn_base_desc(a);
    g.A = dattn_blk; g.B = qkv_blk + 2 * a.d; g.C = dP;
    g.Mb = a.s; g.Nb = a.s; g.Kp = a.d;
    g.a_kcontig = 1; g.b_kcontig = 1; g.lda = a.ldo; g.ldb = a.ld; g.ldc = a.s;
    g.sA1 = o1; g.sA0 = o0; g.sB1 = q1; g.sB0 = q0; g.sC1 = p1; g.sC0 = p0;
    g.out_fp32 = 1; g.skip_upper = causal;
    if ((rc = launch_gemm(g, st))) return rc;
  }
  if ((rc = launch_softmax_bwd(dP, probs_blk, dS, (int)a.nmat, a.s, causal, st))) return rc;
  {  // dQ = dS K / sqrt(d)
    GemmDesc g = attn_base_desc(a);
    g.A = dS; g.B = qkv_blk + a.d; g.C = dqkv_blk;
    g.Mb = a.s; g.Nb = a.d; g.Kp = a.s;
    g.a_kcontig = 1; g.b_kcontig = 0; g.lda = a.s; g.ldb = a.ld; g.ldc = a.ld;
    g.sA1 = p1; g.sA0 = p0; g.sB1 = q1; g.sB0 = q0; g.sC1 = q1; g.sC0 = q0;
    g.alpha = scale; g.k_hi_diag = causal;
    if ((rc = launch_gemm(g, st))) return rc;
  }
  {  // dK = dS^T Q / sqrt(d)
    GemmDesc g = attn_base_desc(a);
    g.A = dS; g.B = qkv_blk; g.C = dqkv_blk + a.d;
    g.Mb = a.s; g.Nb = a.d; g.Kp = a.s;
    g.a_kcontig = 0; g.b_kcontig = 0; g.lda = a.s; g.ldb = a.ld; g.ldc = a.ld;
    g.sA1 = p1; g.sA0 = p0; g.sB1 = q1; g.sB0 = q0; g.sC1 = q1; g.sC0 = q0;
    g.alpha = scale; g.k_lo_diag = causal;
    if ((rc = launch_gemm(g, st))) return rc;
  }
  return OPTIMUS_OK;
}

int run_attention(bool bwd, const void* qkv, const void* probs_in, void* probs_out, const void* d_attn, void* out, int b, int s,
                  int h, int n, int q, int i, int j, int causal, int dtype, void* ws, size_t ws_bytes, void* stream) {
  if (dtype != OPTIMUS_BF16) return OPTIMUS_EDTYPE;
  AttnDims a;
  int rc = attn_dims(b, s, h, n, q, &a);
  if (rc) return rc;
  if ((rc = check_coords(q, i, j))) return rc;
  if (!ws || ws_bytes < attn_ws_bytes(a)) return OPTIMUS_EWORKSPACE;
  // Whole grid: the blocks of consecutive devices follow each other in every tensor, and inside a block the
  // sequences do too, so g devices are one batch of g * (b/q) sequences with the same strides.  As many devices per
  // launch as the workspace holds scratch for (one device's worth is the minimum: then device after device).
  const long long first = is_grid(i, j) ? 0 : (long long)i * q + j;
  const long long ndev = is_grid(i, j) ? (long long)q * q : 1;
  long long group = (long long)(ws_bytes / attn_ws_bytes(a));
  if (group > ndev) group = ndev;
  if (group > 0x7fffffffLL / (a.nmat > 0 ? a.nmat : 1)) group = 0x7fffffffLL / a.nmat;   // batch counts are ints
  for (long long dev = first; dev < first + ndev; dev += group) {
    const long long g = dev + group <= first + ndev ? group : first + ndev - dev;
    AttnDims ag = a;
    ag.nb = (int)(a.nb * g); ag.nmat = a.nmat * g; ag.blk_probs = a.blk_probs * g;
    const bf16_t* qb = (const bf16_t*)qkv + dev * a.blk_qkv;
    if (!bwd)
      rc = attention_fwd_device(qb, (bf16_t*)probs_out + dev * a.blk_probs, (bf16_t*)out + dev * a.blk_attn, ag, causal, ws,
                                as_stream(stream));
    else
      rc = attention_bwd_device(qb, (const bf16_t*)probs_in + dev * a.blk_probs, (const bf16_t*)d_attn + dev * a.blk_attn,
                                (bf16_t*)out + dev * a.blk_qkv, ag, causal, ws, as_stream(stream));
    if (rc) return rc;
  }
  return OPTIMUS_OK;
}

// Fused attention: same block geometry, no [s x s] tensors, head width limited to what the kernels are built for.
int attn_fused_dims(int b, int s, int h, int n, int q, AttnDims* a) {
  if (q <= 0 || b <= 0 || s <= 0 || h <= 0 || n <= 0) return OPTIMUS_ESHAPE;
  if (b % q || n % q || h % n) return OPTIMUS_ESHAPE;
  a->nb = b / q; a->nh = n / q; a->d = h / n; a->s = s;
  if (!attn_fused_supported(a->d) || s > (1 << 20)) return OPTIMUS_ESHAPE;
  a->ld = 3 * h / q; a->ldo = h / q;
  a->blk_qkv = (long long)a->nb * s * a->ld;
  a->blk_attn = (long long)a->nb * s * a->ldo;
  a->nmat = (long long)a->nb * a->nh;
  a->blk_probs = 0;
  if (a->nmat > 65535) return OPTIMUS_ESHAPE;
  return OPTIMUS_OK;
}
size_t attn_fused_ws_bytes(const AttnDims& a, int q) { return align256((size_t)q * q * a.nmat * a.s * sizeof(float)); }

int run_attention_fused(bool bwd, const void* qkv, void* attn, float* lse, const void* d_attn, void* d_qkv, int b, int s, int h,
                        int n, int q, int i, int j, int causal, int dtype, void* ws, size_t ws_bytes, void* stream) {
  if (dtype != OPTIMUS_BF16) return OPTIMUS_EDTYPE;
  AttnDims a;
  int rc = attn_fused_dims(b, s, h, n, q, &a);
  if (rc) return rc;
  if ((rc = check_coords(q, i, j))) return rc;
  if (bwd && (!ws || ws_bytes < attn_fused_ws_bytes(a, q))) return OPTIMUS_EWORKSPACE;
  const bool grid = is_grid(i, j);
  const long long dev = grid ? 0 : (long long)i * q + j;
  AttnFusedDesc d = {};
  d.qkv = (const bf16_t*)qkv + dev * a.blk_qkv;
  d.attn = (bf16_t*)attn + dev * a.blk_attn;
  d.lse = lse + dev * a.nmat * s;
  d.d_attn = d_attn ? (const bf16_t*)d_attn + dev * a.blk_attn : nullptr;
  d.d_qkv = d_qkv ? (bf16_t*)d_qkv + dev * a.blk_qkv : nullptr;
  d.delta = (float*)ws;
  d.s = s; d.d = a.d; d.nb = a.nb; d.nh = a.nh; d.ld = a.ld; d.ldo = a.ldo;
  d.ndev = grid ? q * q : 1;
  d.dev_qkv = a.blk_qkv; d.dev_attn = a.blk_attn;
  d.causal = causal;
  return bwd ? launch_attn_fused_bwd(d, as_stream(stream)) : launch_attn_fused_fwd(d, as_stream(stream));
}

int end_desc(int64_t M, int64_t v, int64_t h, int q, int i, int j, int dtype, EndDesc* d) {
  if (dtype != OPTIMUS_FP32 && dtype != OPTIMUS_BF16) return OPTIMUS_EDTYPE;
  if (q <= 0 || M <= 0 || v <= 0 || h <= 0 || M % q || v % q || h % q) return OPTIMUS_ESHAPE;
  if (M > 0x7fffffff || v > 0x7fffffff || h > 0x7fffffff) return OPTIMUS_ESHAPE;
  int rc = check_coords(q, i, j);
  if (rc) return rc;
  d->rows = (int)(M / q); d->vb = (int)(v / q); d->hb = (int)(h / q); d->q = q; d->v = (int)v; d->dtype = dtype;
  if (is_grid(i, j)) { d->i0 = 0; d->ni = q; d->j0 = 0; d->nj = q; }
  else { d->i0 = i; d->ni = 1; d->j0 = j; d->nj = 1; }
  return OPTIMUS_OK;
}

int ln_desc(int64_t M, int64_t H, int q, int i, int j, int dtype, float eps, LnDesc* d) {
  if (dtype != OPTIMUS_FP32 && dtype != OPTIMUS_BF16) return OPTIMUS_EDTYPE;
  if (q <= 0 || M <= 0 || H <= 0 || M % q || H % q) return OPTIMUS_ESHAPE;
  if (M / q > 0x7fffffff / 4 || H > 0x7fffffff) return OPTIMUS_ESHAPE;
  int rc = check_coords(q, i, j);
  if (rc) return rc;
  d->rows = (int)(M / q); d->cols = (int)(H / q); d->H = (int)H; d->q = q; d->dtype = dtype; d->eps = eps;
  if (is_grid(i, j)) { d->i0 = 0; d->ni = q; d->j0 = 0; d->nj = q; }
  else { d->i0 = i; d->ni = 1; d->j0 = j; d->nj = 1; }
  return OPTIMUS_OK;
}

int ln_forward(const void* X, const float* gamma, const float* beta, void* Y, void* xhat, float* rstd, float* stats,
               const LnDesc& d, bool grid, hipStream_t st) {
  if (grid && !ln_rowgroup_ok(d)) {
    int rc = launch_ln_stats(X, stats, d, st);
    if (rc) return rc;
    return launch_ln_apply(X, gamma, beta, Y, xhat, rstd, stats, d, true, st);
  }
  // one device: its own partial, the peers' from `stats`; whole grid: every row's partials meet inside the launch
  return launch_ln_apply(X, gamma, beta, Y, xhat, rstd, stats, d, false, st);
}
int ln_backward(const void* dY, const void* xhat, const float* rstd, const float* gamma, const void* dres, void* dX,
                float* dgamma_part, float* dbeta_part, float* stats, const LnDesc& d, bool grid, hipStream_t st) {
  int rc;
  if (grid && !ln_rowgroup_ok(d)) {
    if ((rc = launch_ln_bwd_stats(dY, xhat, gamma, stats, d, st))) return rc;
    rc = launch_ln_bwd_apply(dY, xhat, rstd, gamma, dres, dX, stats, d, true, st);
  } else {
    rc = launch_ln_bwd_apply(dY, xhat, rstd, gamma, dres, dX, stats, d, false, st);
  }
  if (rc) return rc;
  if (dgamma_part && dbeta_part) rc = launch_ln_param_grads(dY, xhat, dgamma_part, dbeta_part, d, st);
  return rc;
}

int layer_check(const optimus_layer_cfg* c, int i, int j, AttnDims* a) {
  if (!c) return OPTIMUS_EINVAL;
  if (c->dtype != OPTIMUS_BF16) return OPTIMUS_EDTYPE;
  int rc = c->fused_attention ? attn_fused_dims(c->b, c->s, c->h, c->n, c->q, a) : attn_dims(c->b, c->s, c->h, c->n, c->q, a);
  if (rc) return rc;
  if (c->h % c->q) return OPTIMUS_ESHAPE;
  if ((long long)c->b * c->s > 0x7fffffffLL) return OPTIMUS_ESHAPE;
  return check_coords(c->q, i, j);
}

struct LayerGemm { int form; int64_t M, K, N; };
// the twelve SUMMA products of a layer (forward 4, backward 8), logical output shapes
void layer_gemms(const optimus_layer_cfg* c, LayerGemm out[12]) {
  const int64_t M = (int64_t)c->b * c->s, h = c->h;
  out[0] = {OPTIMUS_FORM_AB, M, h, 3 * h};      // qkv
  out[1] = {OPTIMUS_FORM_AB, M, h, h};          // dense
  out[2] = {OPTIMUS_FORM_AB, M, h, 4 * h};      // h -> 4h
  out[3] = {OPTIMUS_FORM_AB, M, 4 * h, h};      // 4h -> h
  out[4] = {OPTIMUS_FORM_ABT, M, h, 4 * h};     // d_gelu = d_out W2^T
  out[5] = {OPTIMUS_FORM_ATB, 4 * h, M, h};     // dW2 = gelu^T d_out
  out[6] = {OPTIMUS_FORM_ABT, M, 4 * h, h};     // d_ln2_out = d_pre W1^T
  out[7] = {OPTIMUS_FORM_ATB, h, M, 4 * h};     // dW1 = ln2_out^T d_pre
  out[8] = {OPTIMUS_FORM_ABT, M, h, h};         // d_attn = d_h_mid Wo^T
  out[9] = {OPTIMUS_FORM_ATB, h, M, h};         // dWo = attn^T d_h_mid
  out[10] = {OPTIMUS_FORM_ABT, M, 3 * h, h};    // d_ln1_out = d_qkv Wqkv^T
  out[11] = {OPTIMUS_FORM_ATB, h, M, 3 * h};    // dWqkv = ln1_out^T d_qkv
}

// The parameter gradients of the backward pass (A^T B products, bias column sums) hang off the chain of activation
// gradients but nothing in the chain waits for them: they run on a second stream of the library, forked from and
// joined back into the caller's stream with events (also valid under stream capture: the branch becomes a parallel
// arm of the graph).  One stream and one set of events per device, created on the first call that is not made
// under stream capture; until then, or if they cannot be created, the branch simply runs on the caller's stream.
// The stream and events are shared by all calls on a device: concurrent calls from several host threads on one
// device are not supported.
struct SideStream {
  hipStream_t s = nullptr;
  hipEvent_t fork = nullptr, join = nullptr, ready[3] = {nullptr, nullptr, nullptr};
  int state = 0;  // 0 = not tried, 1 = usable, -1 = unavailable
};
constexpr int kMaxDevices = 64;
SideStream g_side[kMaxDevices];

SideStream* side_stream(hipStream_t caller) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { (void)hipGetLastError(); return nullptr; }
  SideStream& x = g_side[dev];
  if (x.state == 0) {
    // creating a stream while the caller captures a graph is not allowed (and would invalidate the capture):
    // stay on the caller's stream for this call and try again on a later one
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(caller, &cs) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
    if (cs != hipStreamCaptureStatusNone) return nullptr;
    bool ok = hipStreamCreateWithFlags(&x.s, hipStreamNonBlocking) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&x.fork, hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&x.join, hipEventDisableTiming) == hipSuccess;
    for (int k = 0; k < 3; ++k) ok = ok && hipEventCreateWithFlags(&x.ready[k], hipEventDisableTiming) == hipSuccess;
    if (!ok) (void)hipGetLastError();
    x.state = ok ? 1 : -1;
  }
  return x.state == 1 ? &x : nullptr;
}
// `to` continues only after everything queued on `from` so far
int stream_after(hipStream_t to, hipStream_t from, hipEvent_t ev) {
  if (hipEventRecord(ev, from) != hipSuccess) return OPTIMUS_EHIP;
  if (hipStreamWaitEvent(to, ev, 0) != hipSuccess) return OPTIMUS_EHIP;
  return OPTIMUS_OK;
}

// Device address of `scratch` on the current device (each GPU holds its own copy at its own address): looked up on
// the first call made with that device current, kept afterwards.
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};
int static_scratch(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { (void)hipGetLastError(); return OPTIMUS_EHIP; }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return OPTIMUS_EHIP; }
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return OPTIMUS_OK;
}

// split workspace of one product as the layer plans it (corun: see GemmDesc)
size_t summa_ws_bytes(int form, int64_t M, int64_t K, int64_t N, int q, int i, int j, int dtype, int corun) {
  if (form < 0 || form > 2 || check_mkn(M, K, N, q) || check_coords(q, i, j)) return 0;
  if (dtype != OPTIMUS_BF16) return 0;
  // pointers only matter for alignment checks; use an aligned dummy
  GemmDesc d = summa_desc(form, (const void*)256, (const void*)256, (void*)256, M, K, N, q, i, j, dtype, nullptr);
  d.corun = corun;
  if (!gemm_mfma_supported(d)) return 0;
  return gemm_plan_bytes(d);
}

size_t layer_gemm_ws(const optimus_layer_cfg* c) {
  LayerGemm g[12];
  layer_gemms(c, g);
  size_t mx = 0;
  for (int k = 0; k < 12; ++k)
    for (int grid = 0; grid < 2; ++grid) {
      // the backward products run in pairs on two streams: chain (A B^T) and branch (A^T B), as optimus_layer_bwd flags them
      const int corun = k < 4 ? 0 : (g[k].form == OPTIMUS_FORM_ABT ? 1 : 2);
      size_t b = summa_ws_bytes(g[k].form, g[k].M, g[k].K, g[k].N, c->q, grid ? -1 : 0, grid ? -1 : 0, c->dtype, corun);
      if (b > mx) mx = b;
    }
  return align256(mx);
}

}  // namespace

extern "C" {

const char* optimus_error_string(int code) {
  switch (code) {
    case OPTIMUS_OK: return "ok";
    case OPTIMUS_EINVAL: return "invalid argument (null pointer or bad enum)";
    case OPTIMUS_ESHAPE: return "bad shape (non-positive, not divisible by the grid, or beyond a documented limit)";
    case OPTIMUS_ECOORD: return "device coordinates outside the q x q grid";
    case OPTIMUS_EDTYPE: return "dtype not supported by this entry point";
    case OPTIMUS_EWORKSPACE: return "workspace missing or too small";
    case OPTIMUS_EHIP: return "HIP runtime error at launch";
    default: return "unknown error code";
  }
}

int optimus_abi_version(void) { return 2; }

int optimus_pack_blocks(const void* src, void* dst, int64_t R, int64_t C, int q, int elem_bytes, void* stream) {
  if (!src || !dst || src == dst) return OPTIMUS_EINVAL;
  if (elem_bytes != 2 && elem_bytes != 4) return OPTIMUS_EDTYPE;
  if (q <= 0 || R <= 0 || C <= 0 || R % q || C % q) return OPTIMUS_ESHAPE;
  return launch_pack(src, dst, R, C, q, elem_bytes, false, as_stream(stream));
}
int optimus_unpack_blocks(const void* src, void* dst, int64_t R, int64_t C, int q, int elem_bytes, void* stream) {
  if (!src || !dst || src == dst) return OPTIMUS_EINVAL;
  if (elem_bytes != 2 && elem_bytes != 4) return OPTIMUS_EDTYPE;
  if (q <= 0 || R <= 0 || C <= 0 || R % q || C % q) return OPTIMUS_ESHAPE;
  return launch_pack(src, dst, R, C, q, elem_bytes, true, as_stream(stream));
}

int optimus_summa_ab(const void* A, const void* B, void* C, int64_t M, int64_t K, int64_t N, int q, int i, int j, int dtype,
                     void* ws, size_t ws_bytes, void* stream) {
  return run_summa(OPTIMUS_FORM_AB, A, B, C, M, K, N, q, i, j, dtype, nullptr, ws, ws_bytes, stream);
}
int optimus_summa_abt(const void* A, const void* B, void* C, int64_t M, int64_t K, int64_t N, int q, int i, int j, int dtype,
                      void* ws, size_t ws_bytes, void* stream) {
  return run_summa(OPTIMUS_FORM_ABT, A, B, C, M, K, N, q, i, j, dtype, nullptr, ws, ws_bytes, stream);
}
int optimus_summa_atb(const void* A, const void* B, void* C, int64_t M, int64_t K, int64_t N, int q, int i, int j, int dtype,
                      void* ws, size_t ws_bytes, void* stream) {
  return run_summa(OPTIMUS_FORM_ATB, A, B, C, M, K, N, q, i, j, dtype, nullptr, ws, ws_bytes, stream);
}
int optimus_summa_ex(int form, const void* A, const void* B, void* C, int64_t M, int64_t K, int64_t N, int q, int i, int j,
                     int dtype, const optimus_epilogue* epi, void* ws, size_t ws_bytes, void* stream) {
  return run_summa(form, A, B, C, M, K, N, q, i, j, dtype, epi, ws, ws_bytes, stream);
}

size_t optimus_summa_workspace_bytes(int form, int64_t M, int64_t K, int64_t N, int q, int i, int j, int dtype) {
  return summa_ws_bytes(form, M, K, N, q, i, j, dtype, 0);
}

// One step of Algorithms 1-3 as the COMPUTING device (i, j) sees it (the owner view above fuses the q steps).
int optimus_summa_step(int form, const void* A, const void* B, float* c_temp, int64_t M, int64_t K, int64_t N, int q, int i,
                       int j, int l, int dtype, void* stream) {
  if (!A || !B || !c_temp) return OPTIMUS_EINVAL;
  if (form < 0 || form > 2) return OPTIMUS_EINVAL;
  if (dtype != OPTIMUS_FP32 && dtype != OPTIMUS_BF16) return OPTIMUS_EDTYPE;
  int rc = check_mkn(M, K, N, q);
  if (rc) return rc;
  if (i < 0 || j < 0 || l < 0 || i >= q || j >= q || l >= q) return OPTIMUS_ECOORD;
  const int Mb = (int)(M / q), Nb = (int)(N / q), Kp = (int)(K / q);
  const long long blkA = (long long)Mb * Kp, blkB = (long long)Kp * Nb;
  const size_t es = esize(dtype);
  GemmDesc d = {};
  d.Mb = Mb; d.Nb = Nb; d.Kp = Kp; d.nl = 1; d.dtype = dtype; d.nz0 = 1; d.nz1 = 1; d.alpha = 1.0f; d.splits = 1;
  d.ldc = Nb; d.out_fp32 = dtype == OPTIMUS_BF16 ? 1 : 0; d.C = c_temp;
  if (form == OPTIMUS_FORM_AB) {          // A_il [Mb x Kp] (received along row i) times B_lj [Kp x Nb] (along column j)
    d.A = off(A, ((long long)i * q + l) * blkA, es); d.a_kcontig = 1; d.lda = Kp;
    d.B = off(B, ((long long)l * q + j) * blkB, es); d.b_kcontig = 0; d.ldb = Nb;
  } else if (form == OPTIMUS_FORM_ABT) {  // own A_ij [Mb x Kp] times (B_lj)^T, B_lj [Nb x Kp] received along column j
    d.A = off(A, ((long long)i * q + j) * blkA, es); d.a_kcontig = 1; d.lda = Kp;
    d.B = off(B, ((long long)l * q + j) * blkB, es); d.b_kcontig = 1; d.ldb = Kp;
  } else {                                // (A_il)^T, A_il [Kp x Mb] received along row i, times own B_ij [Kp x Nb]
    d.A = off(A, ((long long)i * q + l) * blkA, es); d.a_kcontig = 0; d.lda = Mb;
    d.B = off(B, ((long long)i * q + j) * blkB, es); d.b_kcontig = 0; d.ldb = Nb;
  }
  return launch_gemm(d, as_stream(stream));
}

int optimus_summa_reduce(const float* c_temps, int count, void* C, int64_t M, int64_t N, int q, int root_i, int root_j,
                         int dtype, void* stream) {
  if (!c_temps || !C) return OPTIMUS_EINVAL;
  if (dtype != OPTIMUS_FP32 && dtype != OPTIMUS_BF16) return OPTIMUS_EDTYPE;
  if (q <= 0 || M <= 0 || N <= 0 || M % q || N % q || count < 1 || count > 65536) return OPTIMUS_ESHAPE;
  if (root_i < 0 || root_j < 0 || root_i >= q || root_j >= q) return OPTIMUS_ECOORD;
  const long long blk = (M / q) * (N / q);
  return launch_reduce_partials(c_temps, off(C, ((long long)root_i * q + root_j) * blk, esize(dtype)), blk, count, dtype,
                                as_stream(stream));
}

int optimus_bias_grad(const void* dY, float* dbias_part, int64_t M, int64_t N, int q, int i, int j, int dtype, void* stream) {
  if (!dY || !dbias_part) return OPTIMUS_EINVAL;
  if (dtype != OPTIMUS_FP32 && dtype != OPTIMUS_BF16) return OPTIMUS_EDTYPE;
  if (q <= 0 || M <= 0 || N <= 0 || M % q || N % q || M / q > 0x7fffffff || N / q > 0x7fffffff) return OPTIMUS_ESHAPE;
  int rc = check_coords(q, i, j);
  if (rc) return rc;
  const int rows = (int)(M / q), cols = (int)(N / q);
  const long long blk = (long long)rows * cols;
  if (is_grid(i, j)) return launch_colsum(dY, dbias_part, rows, cols, cols, q * q, blk, cols, dtype, as_stream(stream));
  const long long dev = (long long)i * q + j;
  return launch_colsum(off(dY, dev * blk, esize(dtype)), dbias_part + dev * cols, rows, cols, cols, 1, blk, cols, dtype,
                       as_stream(stream));
}

int optimus_layernorm2d_stats(const void* X, float* stats, int64_t M, int64_t H, int q, int i, int l, int dtype, void* stream) {
  if (!X || !stats) return OPTIMUS_EINVAL;
  LnDesc d;
  int rc = ln_desc(M, H, q, i, l, dtype, 0.f, &d);
  if (rc) return rc;
  return launch_ln_stats(X, stats, d, as_stream(stream));
}
int optimus_layernorm2d(const void* X, const float* gamma, const float* beta, void* Y, void* xhat, float* rstd, float* stats,
                        int64_t M, int64_t H, int q, int i, int j, float eps, int dtype, void* stream) {
  if (!X || !gamma || !beta || !Y || !xhat || !rstd || !stats) return OPTIMUS_EINVAL;
  if (!(eps >= 0.f)) return OPTIMUS_EINVAL;
  LnDesc d;
  int rc = ln_desc(M, H, q, i, j, dtype, eps, &d);
  if (rc) return rc;
  return ln_forward(X, gamma, beta, Y, xhat, rstd, stats, d, is_grid(i, j), as_stream(stream));
}
int optimus_layernorm2d_bwd_stats(const void* dY, const void* xhat, const float* gamma, float* stats, int64_t M, int64_t H, int q,
                                  int i, int l, int dtype, void* stream) {
  if (!dY || !xhat || !gamma || !stats) return OPTIMUS_EINVAL;
  LnDesc d;
  int rc = ln_desc(M, H, q, i, l, dtype, 0.f, &d);
  if (rc) return rc;
  return launch_ln_bwd_stats(dY, xhat, gamma, stats, d, as_stream(stream));
}
int optimus_layernorm2d_bwd(const void* dY, const void* xhat, const float* rstd, const float* gamma, const void* dres, void* dX,
                            float* dgamma_part, float* dbeta_part, float* stats, int64_t M, int64_t H, int q, int i, int j,
                            int dtype, void* stream) {
  if (!dY || !xhat || !rstd || !gamma || !dX || !stats) return OPTIMUS_EINVAL;
  if ((dgamma_part == nullptr) != (dbeta_part == nullptr)) return OPTIMUS_EINVAL;
  LnDesc d;
  int rc = ln_desc(M, H, q, i, j, dtype, 0.f, &d);
  if (rc) return rc;
  return ln_backward(dY, xhat, rstd, gamma, dres, dX, dgamma_part, dbeta_part, stats, d, is_grid(i, j), as_stream(stream));
}

size_t optimus_attention_workspace_bytes(int b, int s, int h, int n, int q) {
  AttnDims a;
  if (attn_dims(b, s, h, n, q, &a)) return 0;
  return attn_ws_bytes(a);
}
int optimus_attention_fwd(const void* qkv, void* probs, void* attn, int b, int s, int h, int n, int q, int i, int j, int causal,
                          int dtype, void* ws, size_t ws_bytes, void* stream) {
  if (!qkv || !probs || !attn) return OPTIMUS_EINVAL;
  return run_attention(false, qkv, nullptr, probs, nullptr, attn, b, s, h, n, q, i, j, causal ? 1 : 0, dtype, ws, ws_bytes, stream);
}
int optimus_attention_bwd(const void* qkv, const void* probs, const void* d_attn, void* d_qkv, int b, int s, int h, int n, int q,
                          int i, int j, int causal, int dtype, void* ws, size_t ws_bytes, void* stream) {
  if (!qkv || !probs || !d_attn || !d_qkv) return OPTIMUS_EINVAL;
  return run_attention(true, qkv, probs, nullptr, d_attn, d_qkv, b, s, h, n, q, i, j, causal ? 1 : 0, dtype, ws, ws_bytes, stream);
}

int optimus_softmax_rows(const float* scores, void* probs, int64_t nmat, int s, int causal, void* stream) {
  if (!scores || !probs) return OPTIMUS_EINVAL;
  if (nmat < 1 || s < 4 || s % 4 || s > 4096 || nmat * s > 0x7fffffffLL) return OPTIMUS_ESHAPE;
  return launch_softmax_fwd(scores, probs, (int)nmat, s, causal ? 1 : 0, as_stream(stream));
}
int optimus_softmax_rows_bwd(const float* d_probs, const void* probs, void* d_scores, int64_t nmat, int s, int causal,
                             void* stream) {
  if (!d_probs || !probs || !d_scores) return OPTIMUS_EINVAL;
  if (nmat < 1 || s < 4 || s % 4 || s > 4096 || nmat * s > 0x7fffffffLL) return OPTIMUS_ESHAPE;
  return launch_softmax_bwd(d_probs, probs, d_scores, (int)nmat, s, causal ? 1 : 0, as_stream(stream));
}

size_t optimus_attention_fused_workspace_bytes(int b, int s, int h, int n, int q) {
  AttnDims a;
  if (attn_fused_dims(b, s, h, n, q, &a)) return 0;
  return attn_fused_ws_bytes(a, q);
}
int optimus_attention_fused_fwd(const void* qkv, void* attn, float* lse, int b, int s, int h, int n, int q, int i, int j, int causal,
                                int dtype, void* stream) {
  if (!qkv || !attn || !lse) return OPTIMUS_EINVAL;
  return run_attention_fused(false, qkv, attn, lse, nullptr, nullptr, b, s, h, n, q, i, j, causal ? 1 : 0, dtype, nullptr, 0, stream);
}
int optimus_attention_fused_bwd(const void* qkv, const void* attn, const float* lse, const void* d_attn, void* d_qkv, int b, int s,
                                int h, int n, int q, int i, int j, int causal, int dtype, void* ws, size_t ws_bytes, void* stream) {
  if (!qkv || !attn || !lse || !d_attn || !d_qkv) return OPTIMUS_EINVAL;
  return run_attention_fused(true, qkv, const_cast<void*>(attn), const_cast<float*>(lse), d_attn, d_qkv, b, s, h, n, q, i, j,
                             causal ? 1 : 0, dtype, ws, ws_bytes, stream);
}

int optimus_attention_fused_bwd_static(const void* qkv, const void* attn, const float* lse, const void* d_attn, void* d_qkv, int b,
                                       int s, int h, int n, int q, int i, int j, int causal, int dtype, void* stream) {
  if (!qkv || !attn || !lse || !d_attn || !d_qkv) return OPTIMUS_EINVAL;
  if (dtype != OPTIMUS_BF16) return OPTIMUS_EDTYPE;
  AttnDims a;
  int rc = attn_fused_dims(b, s, h, n, q, &a);
  if (rc) return rc;
  if ((rc = check_coords(q, i, j))) return rc;
  // one fp32 per query row of every matrix of the launch (one device's, or the whole grid's)
  const size_t need = (size_t)(is_grid(i, j) ? q * q : 1) * (size_t)a.nmat * (size_t)s * sizeof(float);
  if (need > kStaticScratchBytes) return OPTIMUS_EWORKSPACE;
  void* ws = nullptr;
  if ((rc = static_scratch(&ws))) return rc;
  // the kernels index the scratch by the launch's own device count, so `need` bytes are all they touch; the size
  // check of the shared code path is against the whole-grid size, which the array is not required to hold
  return run_attention_fused(true, qkv, const_cast<void*>(attn), const_cast<float*>(lse), d_attn, d_qkv, b, s, h, n, q, i, j,
                             causal ? 1 : 0, dtype, ws, attn_fused_ws_bytes(a, q), stream);
}

size_t layer_attn_ws(const optimus_layer_cfg* c, const AttnDims& a) {
  return c->fused_attention ? attn_fused_ws_bytes(a, c->q) : attn_ws_bytes(a);
}
int layer_attention(bool bwd, const optimus_layer_cfg* c, const optimus_layer_tensors* t, int i, int j, void* ws, size_t ws_bytes,
                    void* stream) {
  const int causal = c->causal ? 1 : 0;
  if (c->fused_attention)
    return run_attention_fused(bwd, t->qkv, t->attn, t->lse, bwd ? t->d_attn : nullptr, bwd ? t->d_qkv : nullptr, c->b, c->s, c->h,
                               c->n, c->q, i, j, causal, c->dtype, ws, ws_bytes, stream);
  if (bwd)
    return run_attention(true, t->qkv, t->probs, nullptr, t->d_attn, t->d_qkv, c->b, c->s, c->h, c->n, c->q, i, j, causal, c->dtype,
                         ws, ws_bytes, stream);
  return run_attention(false, t->qkv, nullptr, t->probs, nullptr, t->attn, c->b, c->s, c->h, c->n, c->q, i, j, causal, c->dtype, ws,
                       ws_bytes, stream);
}

int optimus_embedding_fwd(const int32_t* tokens, const void* table, void* x, int64_t M, int64_t v, int64_t h, int q, int i, int j,
                          int dtype, void* stream) {
  if (!tokens || !table || !x) return OPTIMUS_EINVAL;
  EndDesc d;
  int rc = end_desc(M, v, h, q, i, j, dtype, &d);
  if (rc) return rc;
  return launch_embedding_fwd(tokens, table, x, d, as_stream(stream));
}
int optimus_embedding_bwd(const int32_t* tokens, const void* d_x, float* d_table, int64_t M, int64_t v, int64_t h, int q, int l,
                          int j, int dtype, void* stream) {
  if (!tokens || !d_x || !d_table) return OPTIMUS_EINVAL;
  EndDesc d;
  int rc = end_desc(M, v, h, q, l, j, dtype, &d);
  if (rc) return rc;
  return launch_embedding_bwd(tokens, d_x, d_table, d, as_stream(stream));
}
int optimus_cross_entropy2d_stats(const void* logits, float* stats, int64_t M, int64_t v, int q, int i, int l, int dtype,
                                  void* stream) {
  if (!logits || !stats) return OPTIMUS_EINVAL;
  EndDesc d;
  int rc = end_desc(M, v, q, q, i, l, dtype, &d);
  if (rc) return rc;
  return launch_ce_stats(logits, stats, d, as_stream(stream));
}
int optimus_cross_entropy2d(const void* logits, const int32_t* labels, float* loss, float* lse, float* stats, int64_t M, int64_t v,
                            int q, int i, int j, int dtype, void* stream) {
  if (!logits || !labels || !loss || !lse || !stats) return OPTIMUS_EINVAL;
  EndDesc d;
  int rc = end_desc(M, v, q, q, i, j, dtype, &d);
  if (rc) return rc;
  if (!is_grid(i, j)) return launch_ce_stats_final(logits, labels, stats, loss, lse, d, as_stream(stream));  // peers resident
  if ((rc = launch_ce_stats(logits, stats, d, as_stream(stream)))) return rc;   // every device's partial first
  return launch_ce_finalize(logits, labels, stats, loss, lse, d, as_stream(stream));
}
int optimus_cross_entropy2d_bwd(const void* logits, const int32_t* labels, const float* lse, void* d_logits, float scale, int64_t M,
                                int64_t v, int q, int i, int j, int dtype, void* stream) {
  if (!logits || !labels || !lse || !d_logits) return OPTIMUS_EINVAL;
  EndDesc d;
  int rc = end_desc(M, v, q, q, i, j, dtype, &d);
  if (rc) return rc;
  return launch_ce_bwd(logits, labels, lse, d_logits, scale, d, as_stream(stream));
}

size_t optimus_layer_workspace_bytes(const optimus_layer_cfg* cfg) {
  AttnDims a;
  if (layer_check(cfg, 0, 0, &a)) return 0;
  // scores scratch of attention + split partials of the activation chain + split partials of the gradient branch
  return layer_attn_ws(cfg, a) + 2 * layer_gemm_ws(cfg);
}

size_t optimus_layer_workspace_bytes_grid(const optimus_layer_cfg* cfg) {
  const size_t base = optimus_layer_workspace_bytes(cfg);
  AttnDims a;
  if (base == 0 || cfg->fused_attention || layer_check(cfg, 0, 0, &a)) return base;
  // scratch for as many devices' attention per launch as stay inside the 256 MB Infinity Cache (at least one)
  const size_t one = attn_ws_bytes(a);
  size_t g = ((size_t)256 << 20) / one;
  const size_t all = (size_t)cfg->q * cfg->q;
  if (g > all) g = all;
  if (g < 1) g = 1;
  return base + (g - 1) * one;
}

}  // extern "C"

// The forward pass; with skip_out the last product (out = h_mid + gelu W2 + b2) is left out: no gradient needs it, so a
// forward pass that is recomputed inside a backward pass with activation checkpointing stops before it (the third
// of the memory-management remarks at the end of Section 3.2.3).
int optimus::layer_forward(const optimus_layer_cfg* c, const optimus_layer_tensors* t, int i, int j, void* ws, size_t ws_bytes,
                           void* stream, bool skip_out) {
  AttnDims a;
  int rc = layer_check(c, i, j, &a);
  if (rc) return rc;
  if (!t) return OPTIMUS_EINVAL;
  if (!t->x || !t->ln1_g || !t->ln1_b || !t->w_qkv || !t->b_qkv || !t->w_o || !t->b_o || !t->ln2_g || !t->ln2_b || !t->w1 ||
      !t->b1 || !t->w2 || !t->b2 || !t->ln1_out || !t->xhat1 || !t->rstd1 || !t->stats1 || !t->qkv ||
      !(c->fused_attention ? (const void*)t->lse : (const void*)t->probs) || !t->attn ||
      !t->h_mid || !t->ln2_out || !t->xhat2 || !t->rstd2 || !t->stats2 || !t->pre_gelu || !t->gelu || (!skip_out && !t->out))
    return OPTIMUS_EINVAL;
  if (!ws || ws_bytes < optimus_layer_workspace_bytes(c)) return OPTIMUS_EWORKSPACE;
  const int q = c->q, dt = c->dtype;
  const int64_t M = (int64_t)c->b * c->s, h = c->h;
  const bool grid = is_grid(i, j);
  hipStream_t st = as_stream(stream);
  // workspace: [products, chain][products, branch][attention: everything that is left]
  void* gemm_ws = ws;
  const size_t gemm_bytes = layer_gemm_ws(c);
  void* attn_ws = (char*)ws + 2 * gemm_bytes;
  const size_t attn_bytes = ws_bytes - 2 * gemm_bytes;
  LnDesc ln;
  if ((rc = ln_desc(M, h, q, i, j, dt, c->eps, &ln))) return rc;
  // a1 = LN1(x)
  if ((rc = ln_forward(t->x, t->ln1_g, t->ln1_b, t->ln1_out, t->xhat1, t->rstd1, t->stats1, ln, grid, st))) return rc;
  // qkv = a1 Wqkv + b
  optimus_epilogue e = {};
  e.bias = t->b_qkv;
  if ((rc = run_summa(OPTIMUS_FORM_AB, t->ln1_out, t->w_qkv, t->qkv, M, h, 3 * h, q, i, j, dt, &e, gemm_ws, gemm_bytes, stream))) return rc;
  // local attention
  if ((rc = layer_attention(false, c, t, i, j, attn_ws, attn_bytes, stream))) return rc;
  // h_mid = x + attn Wo + b
  e = {};
  e.bias = t->b_o; e.residual = t->x;
  if ((rc = run_summa(OPTIMUS_FORM_AB, t->attn, t->w_o, t->h_mid, M, h, h, q, i, j, dt, &e, gemm_ws, gemm_bytes, stream))) return rc;
  // a2 = LN2(h_mid)
  if ((rc = ln_forward(t->h_mid, t->ln2_g, t->ln2_b, t->ln2_out, t->xhat2, t->rstd2, t->stats2, ln, grid, st))) return rc;
  // pre = a2 W1 + b ; g = GeLU(pre)
  e = {};
  e.bias = t->b1; e.pre_act = t->pre_gelu; e.act = 1;
  if ((rc = run_summa(OPTIMUS_FORM_AB, t->ln2_out, t->w1, t->gelu, M, h, 4 * h, q, i, j, dt, &e, gemm_ws, gemm_bytes, stream))) return rc;
  if (skip_out) return OPTIMUS_OK;
  // out = h_mid + g W2 + b
  e = {};
  e.bias = t->b2; e.residual = t->h_mid;
  return run_summa(OPTIMUS_FORM_AB, t->gelu, t->w2, t->out, M, 4 * h, h, q, i, j, dt, &e, gemm_ws, gemm_bytes, stream);
}

extern "C" {

int optimus_layer_fwd(const optimus_layer_cfg* c, const optimus_layer_tensors* t, int i, int j, void* ws, size_t ws_bytes,
                      void* stream) {
  return layer_forward(c, t, i, j, ws, ws_bytes, stream, false);
}

int optimus_layer_bwd(const optimus_layer_cfg* c, const optimus_layer_tensors* t, int i, int j, void* ws, size_t ws_bytes,
                      void* stream) {
  AttnDims a;
  int rc = layer_check(c, i, j, &a);
  if (rc) return rc;
  if (!t) return OPTIMUS_EINVAL;
  if (!t->x || !t->ln1_g || !t->w_qkv || !t->w_o || !t->ln2_g || !t->w1 || !t->w2 || !t->ln1_out || !t->xhat1 || !t->rstd1 ||
      !t->qkv || !(c->fused_attention ? (const void*)t->lse : (const void*)t->probs) || !t->attn || !t->ln2_out || !t->xhat2 ||
      !t->rstd2 || !t->pre_gelu || !t->gelu || !t->d_out ||
      !t->d_pre_gelu || !t->d_ln2_out || !t->d_h_mid || !t->d_attn || !t->d_qkv || !t->d_ln1_out || !t->d_x || !t->bstats1 ||
      !t->bstats2 || !t->d_w_qkv || !t->d_w_o || !t->d_w1 || !t->d_w2 || !t->d_b_qkv || !t->d_b_o || !t->d_b1 || !t->d_b2 ||
      !t->d_ln1_g || !t->d_ln1_b || !t->d_ln2_g || !t->d_ln2_b)
    return OPTIMUS_EINVAL;
  if (!ws || ws_bytes < optimus_layer_workspace_bytes(c)) return OPTIMUS_EWORKSPACE;
  const int q = c->q, dt = c->dtype;
  const int64_t M = (int64_t)c->b * c->s, h = c->h;
  const bool grid = is_grid(i, j);
  hipStream_t st = as_stream(stream);
  // workspace: [products, chain][products, branch][attention: everything that is left]
  void* gemm_ws = ws;
  const size_t gemm_bytes = layer_gemm_ws(c);
  void* attn_ws = (char*)ws + 2 * gemm_bytes;
  const size_t attn_bytes = ws_bytes - 2 * gemm_bytes;
  LnDesc ln;
  if ((rc = ln_desc(M, h, q, i, j, dt, c->eps, &ln))) return rc;
  // gradient branch: its own stream and its own split workspace (see SideStream)
  SideStream* ss = side_stream(st);
  hipStream_t gst = ss ? ss->s : st;
  void* gstream = (void*)gst;
  void* grad_ws = ss ? (char*)gemm_ws + gemm_bytes : gemm_ws;
  // LayerNorm 2's parameter gradients need d_ln2_out only.  Small blocks: the chain is a string of short kernels and
  // the column sums are one more serial step of it, so they go to the branch (measured: the step 5 % shorter at
  // [1024 x 256] blocks).  Large blocks: the branch, with its transposing products, is the longer stream already.
  const bool ln2_grads_on_branch = colsum_narrow((int)(M / q), (int)(h / q));
  optimus_epilogue e = {};
  optimus_epilogue e32 = {};
  e32.out_fp32 = 1;
  // After the fork the branch stream depends on the caller's stream; whatever happens afterwards, the caller's stream
  // must be joined with it again before this call returns (a stream capture that is left forked cannot be ended).
  // So the first failing step only switches the remaining steps off, and the join below still runs.
  rc = OPTIMUS_OK;
  bool forked = false;
#define RUN(...) do { if (rc == OPTIMUS_OK) rc = (__VA_ARGS__); } while (0)
#define BRANCH_AFTER_MAIN(EV) do { if (ss && rc == OPTIMUS_OK) { rc = stream_after(gst, st, EV); forked = forked || rc == OPTIMUS_OK; } } while (0)
  BRANCH_AFTER_MAIN(ss->fork);
  // ---- out = h_mid + gelu W2 + b2 ----
  e = {}; e.gelu_grad_of = t->pre_gelu;  // d_pre = (d_out W2^T) * GeLU'(pre)
  RUN(run_summa(OPTIMUS_FORM_ABT, t->d_out, t->w2, t->d_pre_gelu, M, h, 4 * h, q, i, j, dt, &e, gemm_ws, gemm_bytes, stream, 1));
  RUN(run_summa(OPTIMUS_FORM_ATB, t->gelu, t->d_out, t->d_w2, 4 * h, M, h, q, i, j, dt, &e32, grad_ws, gemm_bytes, gstream, 2));
  RUN(optimus_bias_grad(t->d_out, t->d_b2, M, h, q, i, j, dt, gstream));
  // ---- pre = ln2_out W1 + b1 ----
  BRANCH_AFTER_MAIN(ss->ready[0]);  // d_pre_gelu is complete
  RUN(run_summa(OPTIMUS_FORM_ABT, t->d_pre_gelu, t->w1, t->d_ln2_out, M, 4 * h, h, q, i, j, dt, nullptr, gemm_ws, gemm_bytes, stream, 1));
  RUN(run_summa(OPTIMUS_FORM_ATB, t->ln2_out, t->d_pre_gelu, t->d_w1, h, M, 4 * h, q, i, j, dt, &e32, grad_ws, gemm_bytes, gstream, 2));
  RUN(optimus_bias_grad(t->d_pre_gelu, t->d_b1, M, 4 * h, q, i, j, dt, gstream));
  // ---- LN2 backward, plus the residual branch: d_h_mid = d_out + LN2'(d_ln2_out) ----
  RUN(ln_backward(t->d_ln2_out, t->xhat2, t->rstd2, t->ln2_g, t->d_out, t->d_h_mid, ln2_grads_on_branch ? nullptr : t->d_ln2_g,
                  ln2_grads_on_branch ? nullptr : t->d_ln2_b, t->bstats2, ln, grid, st));
  // ---- h_mid = x + attn Wo + bo ----
  BRANCH_AFTER_MAIN(ss->ready[1]);  // d_h_mid is complete
  RUN(run_summa(OPTIMUS_FORM_ABT, t->d_h_mid, t->w_o, t->d_attn, M, h, h, q, i, j, dt, nullptr, gemm_ws, gemm_bytes, stream, 1));
  RUN(run_summa(OPTIMUS_FORM_ATB, t->attn, t->d_h_mid, t->d_w_o, h, M, h, q, i, j, dt, &e32, grad_ws, gemm_bytes, gstream, 2));
  RUN(optimus_bias_grad(t->d_h_mid, t->d_b_o, M, h, q, i, j, dt, gstream));
  if (ln2_grads_on_branch) RUN(launch_ln_param_grads(t->d_ln2_out, t->xhat2, t->d_ln2_g, t->d_ln2_b, ln, gst));
  // ---- local attention backward ----
  RUN(layer_attention(true, c, t, i, j, attn_ws, attn_bytes, stream));
  // ---- qkv = ln1_out Wqkv + b ----
  BRANCH_AFTER_MAIN(ss->ready[2]);  // d_qkv is complete
  RUN(run_summa(OPTIMUS_FORM_ABT, t->d_qkv, t->w_qkv, t->d_ln1_out, M, 3 * h, h, q, i, j, dt, nullptr, gemm_ws, gemm_bytes, stream, 1));
  RUN(run_summa(OPTIMUS_FORM_ATB, t->ln1_out, t->d_qkv, t->d_w_qkv, h, M, 3 * h, q, i, j, dt, &e32, grad_ws, gemm_bytes, gstream, 2));
  RUN(optimus_bias_grad(t->d_qkv, t->d_b_qkv, M, 3 * h, q, i, j, dt, gstream));
  // ---- LN1 backward, plus the residual branch: d_x = d_h_mid + LN1'(d_ln1_out) ----
  RUN(ln_backward(t->d_ln1_out, t->xhat1, t->rstd1, t->ln1_g, t->d_h_mid, t->d_x, t->d_ln1_g, t->d_ln1_b, t->bstats1, ln, grid, st));
  // the caller's stream owns every result again
  if (ss && forked) {
    const int jr = stream_after(st, gst, ss->join);
    if (rc == OPTIMUS_OK) rc = jr;
  }
#undef BRANCH_AFTER_MAIN
#undef RUN
  return rc;
}

int64_t optimus_gemm_flops(int64_t M, int64_t K, int64_t N, int q) {
  if (check_mkn(M, K, N, q)) return -1;
  return 2 * (M / q) * K * (N / q);
}

int64_t optimus_layer_flops(const optimus_layer_cfg* c, int what) {
  AttnDims a;
  if (layer_check(c, 0, 0, &a) || what < 0 || what > 1) return -1;
  const int64_t b = c->b, s = c->s, h = c->h, p = (int64_t)c->q * c->q;
  const int64_t fwd = 2 * (12 * b * s * h * h + 2 * b * s * s * h) / p;
  return what == 0 ? fwd : 2 * fwd;
}

int optimus_debug_mfma_rate(float* out, int workgroups, int iters, int random_data, void* stream) {
  if (!out) return OPTIMUS_EINVAL;
  if (workgroups < 1 || workgroups > 65536 || iters < 1 || iters > (1 << 24)) return OPTIMUS_ESHAPE;
  return launch_mfma_rate(out, workgroups, iters, random_data ? 1 : 0, as_stream(stream));
}

// ---- tuning hook used by the benchmark (not part of the method): force a matrix-core tile variant, -1 = automatic ----
void optimus_debug_set_gemm_variant(int v) { gemm_set_variant(v); }
void optimus_debug_set_corun_variants(int chain_v, int branch_v) { gemm_set_corun_variants(chain_v, branch_v); }
int optimus_debug_plan_summa(int form, int64_t M, int64_t K, int64_t N, int q, int i, int j, int corun, int have_ws, int* out3) {
  if (!out3 || form < 0 || form > 2 || corun < 0 || corun > 2) return OPTIMUS_EINVAL;
  int rc = check_mkn(M, K, N, q);
  if (rc) return rc;
  rc = check_coords(q, i, j);
  if (rc) return rc;
  // the plan depends on shapes, strides and 16-byte alignment only: a fixed aligned address stands in for the tensors
  void* const fake = (void*)(uintptr_t)4096;
  GemmDesc d = summa_desc(form, fake, fake, fake, M, K, N, q, i, j, OPTIMUS_BF16, nullptr);
  d.corun = corun;
  return gemm_plan_of(d, have_ws != 0, out3) ? OPTIMUS_OK : OPTIMUS_EDTYPE;
}
int optimus_debug_last_gemm_plan(void) { return gemm_last_plan(); }

}  // extern "C"

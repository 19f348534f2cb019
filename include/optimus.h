/*
 * optimus.h — C ABI of the per-device hot path of the 2D (SUMMA) transformer
 * scheme of arXiv 2104.05343, for one AMD MI355X (gfx950).
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 * Pointers.  Every tensor pointer is a DEVICE pointer owned by the caller; the
 *   library neither frees nor retains it.  `stream` is a hipStream_t passed as
 *   void* (NULL = the default stream).  Calls validate their arguments on the
 *   host, enqueue kernels on `stream` and return without synchronising.
 *   The structs (`optimus_layer_cfg`, `optimus_layer_tensors`, `optimus_layer_params`, `optimus_layer_grads`,
 *   `optimus_stack_buffers`, ...) and arrays of them are HOST memory holding device pointers.
 * Grid.  The method distributes every matrix over a q x q device mesh
 *   (Section 2.4): a logical row-major matrix T[R x C] is cut evenly into q*q
 *   sub-blocks, block (r, c) belonging to device (r, c).  This library keeps
 *   all q*q blocks resident on one GPU in BLOCK-MAJOR storage: block (r, c)
 *   starts at element (r*q + c) * (R/q) * (C/q) and is itself row-major with
 *   leading dimension C/q — the contiguous panel a broadcast would deliver.
 *   Vectors of length C (biases, LayerNorm affine) are stored whole; device
 *   column j uses elements j*C/q .. (j+1)*C/q-1.
 * Coordinates.  (i, j) names the device whose share is computed.  i = j =
 *   OPTIMUS_ALL (-1) computes the share of every device in one call ("grid
 *   mode"); mixing -1 with a real coordinate is OPTIMUS_ECOORD.  With explicit
 *   (i, j) a call reads only the peer blocks that device would receive and
 *   writes only that device's output block(s).
 * dtype.  OPTIMUS_FP32: fp32 storage, fp32 FMA accumulation.  OPTIMUS_BF16:
 *   bf16 storage (round-to-nearest-even on store), fp32 accumulation on the
 *   matrix cores; statistics, soft-max sums, weight and bias gradients stay
 *   fp32.
 * Errors.  Return value 0 = OK, otherwise one of the OPTIMUS_E* codes below.
 *   Arguments are checked before anything is enqueued: on EINVAL / ESHAPE /
 *   ECOORD / EDTYPE / EWORKSPACE nothing has been enqueued.  OPTIMUS_EHIP (the
 *   runtime refused a launch) can come from a later kernel of a call that
 *   enqueues several.  No exceptions.  Process state: the tuning hooks at the
 *   end of this file (process-wide, atomic), per device one stream with its
 *   events that optimus_layer_bwd creates on first use (see there), and per
 *   device the fixed scratch array of optimus_attention_fused_bwd_static.
 * Determinism.  No floating-point atomics: the same call on the same inputs
 *   gives bitwise identical output.
 */
#ifndef OPTIMUS_H_
#define OPTIMUS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  OPTIMUS_OK = 0,
  OPTIMUS_EINVAL = 1,     /* null pointer or bad enum value                          */
  OPTIMUS_ESHAPE = 2,     /* size <= 0 or not divisible as the partition requires    */
  OPTIMUS_ECOORD = 3,     /* i or j outside [0, q) and not the OPTIMUS_ALL wildcard  */
  OPTIMUS_EDTYPE = 4,     /* dtype not supported by this entry point                 */
  OPTIMUS_EWORKSPACE = 5, /* workspace missing or smaller than the query says        */
  OPTIMUS_EHIP = 6        /* the HIP runtime refused a launch                        */
};

enum { OPTIMUS_FP32 = 0, OPTIMUS_BF16 = 1 };
enum { OPTIMUS_FORM_AB = 0, OPTIMUS_FORM_ABT = 1, OPTIMUS_FORM_ATB = 2 };
#define OPTIMUS_ALL (-1)

/* Human-readable name of an error code (static string, never NULL). */
const char* optimus_error_string(int code);
/* ABI version of this header (bumped when a signature changes). */
int optimus_abi_version(void);

/* ---- block addressing (Section 2.4: "evenly partitioned into q x q sub-blocks") ----
 * Convert between a row-major logical matrix [R x C] and block-major storage.
 * src and dst are distinct device buffers of R*C elements of elem_bytes (2 or 4)
 * bytes each.  Pure data movement: bit-exact.  ESHAPE unless q | R and q | C. */
int optimus_pack_blocks(const void* src_rowmajor, void* dst_blockmajor, int64_t R, int64_t C,
                        int q, int elem_bytes, void* stream);
int optimus_unpack_blocks(const void* src_blockmajor, void* dst_rowmajor, int64_t R, int64_t C,
                          int q, int elem_bytes, void* stream);

/* ---- the same algorithms step by step, from the COMPUTING device (Algorithms 1-3 as printed) ----
 * optimus_summa_step: what device (i, j) multiplies in step l, as one dense fp32 [M/q x N/q] block c_temp:
 *   AB : A_il B_lj           (both received; accumulated on the same device into C_ij)
 *   ABT: A_ij (B_lj)^T       (B_lj received along column j; reduced within row i onto device (i, l) -> C_il)
 *   ATB: (A_il)^T B_ij       (A_il received along row i; reduced within column j onto device (l, j) -> C_lj)
 * optimus_summa_reduce: the reduce onto its root: adds `count` consecutive partial blocks c_temps[0..count) in
 * index order (the order of the reducing grid index) and writes block (root_i, root_j) of the block-major
 * [M x N] matrix C in `dtype`.  Partials in memory are what the owner-view entry points above avoid; these two
 * exist so that the printed algorithms can be replayed and compared with them.  Operand layouts as above. */
int optimus_summa_step(int form, const void* A, const void* B, float* c_temp, int64_t M, int64_t K, int64_t N,
                       int q, int i, int j, int l, int dtype, void* stream);
int optimus_summa_reduce(const float* c_temps, int count, void* C, int64_t M, int64_t N, int q, int root_i,
                         int root_j, int dtype, void* stream);

/* ---- the three SUMMA products (Section 2.4, Algorithms 1-3, Eq. 1-3) ----
 * (M, N) is always the logical OUTPUT shape and K the logical contraction
 * length; all three must be positive multiples of q.  A, B, C are block-major.
 * Device (i, j) ends up holding (owner view of Algorithms 1-3; the per-step
 * broadcasts become reads of resident peer blocks, the row/column reduce of
 * Algorithms 2-3 becomes the sum over l inside one accumulator):
 *   optimus_summa_ab :  C_ij = sum_l A_il   * B_lj      A[M x K], B[K x N]
 *   optimus_summa_abt:  C_ij = sum_l A_il   * (B_jl)^T  A[M x K], B[N x K]
 *   optimus_summa_atb:  C_ij = sum_l (A_li)^T * B_lj    A[K x M], B[K x N]
 * The q panel steps are fused into one k-loop; C is written once.  C must not
 * alias A or B.
 * ws / ws_bytes: optional device scratch (may be NULL / 0).  When it is at
 * least optimus_summa_workspace_bytes(...) the library may split the panel
 * loop of skinny outputs over several workgroups and combine the fp32 partial
 * tiles in a fixed order (still deterministic); without it no split is used. */
int optimus_summa_ab(const void* A, const void* B, void* C, int64_t M, int64_t K, int64_t N,
                     int q, int i, int j, int dtype, void* ws, size_t ws_bytes, void* stream);
int optimus_summa_abt(const void* A, const void* B, void* C, int64_t M, int64_t K, int64_t N,
                      int q, int i, int j, int dtype, void* ws, size_t ws_bytes, void* stream);
int optimus_summa_atb(const void* A, const void* B, void* C, int64_t M, int64_t K, int64_t N,
                      int q, int i, int j, int dtype, void* ws, size_t ws_bytes, void* stream);
size_t optimus_summa_workspace_bytes(int form, int64_t M, int64_t K, int64_t N, int q, int i, int j,
                                     int dtype);

/* Epilogue applied to the accumulator of a SUMMA product before the single
 * store of C_ij (Section 3.2.1: non-linearities are applied locally per
 * block; Section 3.2.2: bias-add uses the column slice of a row-0 parameter).
 * In order:  t = acc;  t += bias[j-slice];  if pre_act: pre_act_ij = t;
 * if act == 1: t = GeLU(t) (exact, x*Phi(x));  if gelu_grad_of: t *= GeLU'(gelu_grad_of_ij);
 * if residual: t += residual_ij;  C_ij = t.
 * bias is fp32 [N]; pre_act, gelu_grad_of, residual are block-major [M x N]
 * in the call's dtype.  out_fp32 != 0 stores C as fp32 even for bf16 inputs
 * (weight gradients).  Any pointer may be NULL to skip its step. */
typedef struct {
  const float* bias;
  void* pre_act;
  int act;
  const void* gelu_grad_of;
  const void* residual;
  int out_fp32;
} optimus_epilogue;

/* form: OPTIMUS_FORM_*.  epi may be NULL (plain product). */
int optimus_summa_ex(int form, const void* A, const void* B, void* C, int64_t M, int64_t K, int64_t N,
                     int q, int i, int j, int dtype, const optimus_epilogue* epi, void* ws,
                     size_t ws_bytes, void* stream);

/* Bias gradient (Section 3.2.2, bias-add backward): device (i, j)'s partial
 * = column sums of its block dY_ij; the reduce up the column to row 0 is the
 * sum over i of these partials.  dY block-major [M x N]; out fp32
 * [q][q][N/q], entry (i, j) written. */
int optimus_bias_grad(const void* dY, float* dbias_part, int64_t M, int64_t N, int q, int i, int j,
                      int dtype, void* stream);

/* ---- 2D LayerNorm (Section 3.2.2) ----
 * X block-major [M x H]; a row's H entries are spread over the q devices of
 * grid row i.  stats is fp32 [q][q][M/q][2]: entry (i, l) holds what device
 * (i, l) contributes to the row all-reduce, (sum x, sum x^2) per local row in
 * forward and (sum xhat*g, sum g) with g = dy*gamma in backward.
 *
 * optimus_layernorm2d_stats(i, l): writes device (i, l)'s forward partial only.
 * optimus_layernorm2d(i, j): computes its own partial (and stores it in
 *   stats[i][j]), adds the q-1 peer partials already in stats[i][*], then
 *   xhat = (x - E[x]) * rstd, rstd = 1/sqrt(max(E[x^2]-E[x]^2, 0) + eps),
 *   y = gamma_j*xhat + beta_j.  Writes Y_ij, xhat_ij (same dtype as X) and
 *   rstd (fp32 [q][q][M/q], entry (i, j)).  In grid mode all partials are
 *   produced first, so no prior _stats call is needed.
 * optimus_layernorm2d_bwd(i, j): dX_ij = rstd*(g - xhat*mean(xhat*g) - mean(g))
 *   [+ dres_ij if dres != NULL: gradient arriving over the residual branch],
 *   with the two means taken over the whole row via `stats` exactly as in
 *   forward; dgamma_part/dbeta_part fp32 [q][q][H/q]: column sums of dy*xhat
 *   and dy over the block's rows (entry (i, j) written).
 * gamma, beta: fp32 [H]. */
int optimus_layernorm2d_stats(const void* X, float* stats, int64_t M, int64_t H, int q, int i, int l,
                              int dtype, void* stream);
int optimus_layernorm2d(const void* X, const float* gamma, const float* beta, void* Y, void* xhat,
                        float* rstd, float* stats, int64_t M, int64_t H, int q, int i, int j,
                        float eps, int dtype, void* stream);
int optimus_layernorm2d_bwd_stats(const void* dY, const void* xhat, const float* gamma, float* stats,
                                  int64_t M, int64_t H, int q, int i, int l, int dtype, void* stream);
int optimus_layernorm2d_bwd(const void* dY, const void* xhat, const float* rstd, const float* gamma,
                            const void* dres, void* dX, float* dgamma_part, float* dbeta_part,
                            float* stats, int64_t M, int64_t H, int q, int i, int j, int dtype,
                            void* stream);

/* ---- head-partitioned attention on the device's blocks (Sections 2.1, 3.2.1) ----
 * Device (i, j) holds n/q heads of b/q whole sequences.  qkv is block-major
 * [b*s x 3h] (rows sequence-major: row = seq*s + t; columns head-major:
 * head*3d + {0:Q,1:K,2:V}*d + e with d = h/n), so block (i, j) contains Q, K,
 * V of heads j*n/q.. of sequences i*b/q...  For every local (sequence, head):
 * S = Q K^T / sqrt(d), causal mask if causal != 0, P = softmax rows (fp32),
 * O = P V.  probs: [q][q][(b/q)*(n/q)][s][s] in the call's dtype (entries above
 * the diagonal are exact zeros when causal); attn: block-major [b*s x h].
 * Backward: dV = P^T dO, dP = dO V^T, dS = P*(dP - rowsum(dP*P)),
 * dQ = dS K / sqrt(d), dK = dS^T Q / sqrt(d); d_qkv has qkv's layout.
 * ws must hold optimus_attention_workspace_bytes(...) bytes (scratch for one
 * device's scores); a whole-grid call (i = j = -1) takes g devices per launch
 * when ws holds g times that (same bits, fewer and larger launches). bf16 only.
 * Requires q | b, q | n, n | h, d % 8 == 0, s % 8 == 0, s <= 4096 (a row of
 * scores is held by one wavefront; longer sequences: optimus_attention_fused_*);
 * OPTIMUS_ESHAPE otherwise. */
int optimus_attention_fwd(const void* qkv, void* probs, void* attn, int b, int s, int h, int n, int q,
                          int i, int j, int causal, int dtype, void* ws, size_t ws_bytes, void* stream);
int optimus_attention_bwd(const void* qkv, const void* probs, const void* d_attn, void* d_qkv, int b,
                          int s, int h, int n, int q, int i, int j, int causal, int dtype, void* ws,
                          size_t ws_bytes, void* stream);
size_t optimus_attention_workspace_bytes(int b, int s, int h, int n, int q);

/* ---- the row soft-max of attention by itself ("Nonlinear" of Section 2.1; local per device, Section 3.2.1) ----
 * The two bandwidth-bound kernels between the attention products, exported so that they can be measured and
 * tested alone.  scores / d_probs: nmat matrices [s x s] fp32, contiguous; probs / d_scores: the same shape in
 * bf16.  Forward: P = softmax over each row of S (with causal != 0 only columns <= row take part and the entries
 * above the diagonal are written as exact zeros).  Backward: dS = P * (dP - rowsum(dP * P)) row by row (entries
 * of dP above the diagonal are not read when causal).  Device memory; requires s % 4 == 0, 4 <= s <= 4096,
 * nmat >= 1, nmat * s < 2^31 (OPTIMUS_ESHAPE otherwise); null pointers: OPTIMUS_EINVAL. */
int optimus_softmax_rows(const float* scores, void* probs, int64_t nmat, int s, int causal, void* stream);
int optimus_softmax_rows_bwd(const float* d_probs, const void* probs, void* d_scores, int64_t nmat, int s,
                             int causal, void* stream);

/* ---- the same attention without the [s x s] tensors (the operator fusion proposed in Section 6) ----
 * Same qkv / attn / d_qkv layouts and the same mathematics as above, but neither scores nor probabilities are
 * ever written to memory, so sequence length is no longer bounded by the [b/q, n/q, s, s] tensor.  The forward
 * keeps, per query row, lse = log sum_u exp(S_tu) (natural logarithm of the scaled, masked scores):
 * lse is [q][q][(b/q)*(n/q)][s] fp32 in device order; the backward rebuilds P = exp(S - lse) tile by tile and
 * uses rowsum(dO * O) for rowsum(dP * P), so it also reads the forward's attn output.
 * Device memory, all of them; ws (backward only) must hold optimus_attention_fused_workspace_bytes(...) bytes.
 * bf16 only; head width d = h/n must be 64 or 128 (OPTIMUS_ESHAPE otherwise); any s >= 1 up to 2^20;
 * requires q | b, q | n, n | h. */
int optimus_attention_fused_fwd(const void* qkv, void* attn, float* lse, int b, int s, int h, int n, int q,
                                int i, int j, int causal, int dtype, void* stream);
int optimus_attention_fused_bwd(const void* qkv, const void* attn, const float* lse, const void* d_attn,
                                void* d_qkv, int b, int s, int h, int n, int q, int i, int j, int causal,
                                int dtype, void* ws, size_t ws_bytes, void* stream);
size_t optimus_attention_fused_workspace_bytes(int b, int s, int h, int n, int q);

/* ---- optimus_attention_fused_bwd for callers that cannot allocate ----
 * For code under HIP graph capture, tight serving loops and harnesses that forbid hipMalloc: the same operation,
 * arguments, layouts and results (bit for bit) as optimus_attention_fused_bwd, without the ws argument.  The one
 * scratch buffer of that call (one fp32 per query row of every (sequence, head) matrix of the launch) lives in a
 * static device array of OPTIMUS_STATIC_SCRATCH_BYTES that every GPU the library runs on holds until the process
 * ends; the call allocates and frees nothing.  A launch that needs more -- (i = j = -1 ? q*q : 1) * (b/q) * (n/q)
 * * s * 4 bytes -- is rejected with OPTIMUS_EWORKSPACE before anything is enqueued.  All calls on one GPU share
 * the array (it keeps the last call's contents; every call overwrites what it reads, nothing needs clearing):
 * two calls that overlap on one GPU (different streams, several host threads) race on it.  The array's address
 * is looked up on the first call made with a device current; make that first call outside stream capture. */
#define OPTIMUS_STATIC_SCRATCH_BYTES (4u << 20)
int optimus_attention_fused_bwd_static(const void* qkv, const void* attn, const float* lse, const void* d_attn,
                                       void* d_qkv, int b, int s, int h, int n, int q, int i, int j,
                                       int causal, int dtype, void* stream);

/* ---- one transformer layer on device (i, j) (Section 3.2; Eq. 1) ----
 * Wiring: a1 = LN1(x); qkv = a1 Wqkv + b; attn = local attention;
 * h_mid = x + attn Wo + b; a2 = LN2(h_mid); pre = a2 W1 + b; g = GeLU(pre);
 * out = h_mid + g W2 + b.  Backward follows Eq. 1 for every linear layer
 * (dX = dY W^T by the AB^T product, dW = X^T dY by the A^T B product), uses the
 * saved activations (no recomputation) and no dropout.
 * Every matrix is block-major over the q x q grid; vectors are fp32 and whole.
 * In grid mode (i = j = -1) each stage runs for all q*q devices before the
 * next starts, filling every block of every tensor.  With explicit (i, j) only
 * that device's blocks are recomputed; peers' blocks of the previous stage must
 * be resident (left by a grid-mode call on the same tensors). */
typedef struct {
  int b, s, h, n, q;
  float eps;
  int causal;
  int dtype; /* OPTIMUS_BF16 only */
  int fused_attention; /* 0: scores and probabilities in memory (probs saved for the backward pass);
                          1: optimus_attention_fused_* (lse saved instead; needs h/n = 64 or 128) */
} optimus_layer_cfg;

typedef struct {
  /* inputs / parameters */
  const void* x;      /* [M x h]  */
  const float* ln1_g; const float* ln1_b;  /* [h] */
  const void* w_qkv;  /* [h x 3h] */
  const float* b_qkv; /* [3h]     */
  const void* w_o;    /* [h x h]  */
  const float* b_o;   /* [h]      */
  const float* ln2_g; const float* ln2_b;  /* [h] */
  const void* w1;     /* [h x 4h] */
  const float* b1;    /* [4h]     */
  const void* w2;     /* [4h x h] */
  const float* b2;    /* [h]      */
  /* forward tensors, written by optimus_layer_fwd, read by optimus_layer_bwd */
  void* ln1_out; void* xhat1; float* rstd1; float* stats1; /* [M x h], [M x h], [q][q][M/q], [q][q][M/q][2] */
  void* qkv;      /* [M x 3h] */
  void* probs;    /* [q][q][(b/q)(n/q)][s][s]; unused (may be NULL) with fused_attention */
  void* attn;     /* [M x h]  */
  void* h_mid;    /* [M x h]  */
  void* ln2_out; void* xhat2; float* rstd2; float* stats2;
  void* pre_gelu; /* [M x 4h] */
  void* gelu;     /* [M x 4h] */
  void* out;      /* [M x h]  */
  /* backward: input gradient, activation gradients (resident for peers), outputs */
  const void* d_out;  /* [M x h] */
  void* d_pre_gelu;   /* [M x 4h] */
  void* d_ln2_out;    /* [M x h]  */
  void* d_h_mid;      /* [M x h]  */
  void* d_attn;       /* [M x h]  */
  void* d_qkv;        /* [M x 3h] */
  void* d_ln1_out;    /* [M x h]  */
  void* d_x;          /* [M x h]  */
  float* bstats1; float* bstats2; /* [q][q][M/q][2] backward LayerNorm partials */
  float* d_w_qkv; float* d_w_o; float* d_w1; float* d_w2;         /* fp32, block-major, weight shapes */
  float* d_b_qkv; float* d_b_o; float* d_b1; float* d_b2;         /* fp32 partials [q][q][N/q]        */
  float* d_ln1_g; float* d_ln1_b; float* d_ln2_g; float* d_ln2_b; /* fp32 partials [q][q][h/q]        */
  float* lse;     /* [q][q][(b/q)(n/q)][s] fp32, forward tensor; only with fused_attention (else may be NULL) */
} optimus_layer_tensors;

/* Scratch bytes optimus_layer_fwd / _bwd need in `ws` (attention scores and
 * their gradients for one device -- with fused_attention only one fp32 per
 * query row --, plus split-k partial tiles: one region for
 * the activation chain and one for the parameter-gradient branch, which
 * optimus_layer_bwd runs concurrently on a stream of the library's own that
 * it forks from and joins back into `stream` with events; when the call
 * returns, every kernel of both is ordered before later work on `stream`.
 * The library creates that stream (default priority) and its events on the
 * first call per device that is not made under stream capture; until then the
 * branch runs on `stream` itself.  They are shared by all calls on a device:
 * optimus_layer_bwd must not be called from several host threads at once
 * for the same device.) */
size_t optimus_layer_workspace_bytes(const optimus_layer_cfg* cfg);
/* The size to give whole-grid calls (i = j = -1) that should run fast: the minimum above plus attention scratch
 * for more devices, so that the unfused attention of several devices is one batch per launch instead of one device
 * after the other (as many as stay inside the 256 MB Infinity Cache, at least one).  optimus_layer_fwd / _bwd use
 * whatever `ws_bytes` holds beyond the products' regions for this; the results do not depend on it, bit for bit. */
size_t optimus_layer_workspace_bytes_grid(const optimus_layer_cfg* cfg);
int optimus_layer_fwd(const optimus_layer_cfg* cfg, const optimus_layer_tensors* t, int i, int j,
                      void* ws, size_t ws_bytes, void* stream);
int optimus_layer_bwd(const optimus_layer_cfg* cfg, const optimus_layer_tensors* t, int i, int j,
                      void* ws, size_t ws_bytes, void* stream);

/* ---- a stack of identical layers with distributed activation checkpointing and pre-allocated buffers
 *      (Section 3.2.3 "memory pre-allocation and checkpointing" and its figure; Table 1's backward rows) ----
 * Forward keeps only the input of every layer (checkpoint[l], [M x h] block-major each: b*s*h/p elements per device
 * and layer); all layers share ONE set of forward tensors (forward buffer), ONE set of activation gradients
 * (backward buffer), two [M x h] slots for the gradient passed between consecutive layers (conjunction buffer) and
 * the workspace.  Backward recomputes layer l's forward pass from checkpoint[l] (without its last product, which
 * no gradient needs), then runs optimus_layer_bwd on it, for l = L-1 .. 0.
 * grads[l] says where layer l's parameter gradients go (layouts as in optimus_layer_tensors); entries may all
 * point into one parameter-gradient buffer if the caller consumes them in `done`, which is called on the host
 * after layer l's backward kernels have been enqueued (stream-ordered work enqueued from it sees the gradients and
 * precedes the next layer's; may be NULL).
 * These calls compute every device's share (grid mode): buffers that all layers share cannot keep the peers' blocks
 * of every layer resident.  x, out, d_out, d_x: [M x h] block-major device memory; buffers: device memory of at least
 * the sizes optimus_stack_sizes_of reports (256-byte aligned); params / grads: host arrays of n_layers entries of
 * device pointers.  The caller's out and d_x must not alias the buffers. */
typedef struct {
  const float* ln1_g; const float* ln1_b; const void* w_qkv; const float* b_qkv; const void* w_o; const float* b_o;
  const float* ln2_g; const float* ln2_b; const void* w1; const float* b1; const void* w2; const float* b2;
} optimus_layer_params;
typedef struct {
  float* d_w_qkv; float* d_w_o; float* d_w1; float* d_w2; float* d_b_qkv; float* d_b_o; float* d_b1; float* d_b2;
  float* d_ln1_g; float* d_ln1_b; float* d_ln2_g; float* d_ln2_b;
} optimus_layer_grads;
typedef struct { size_t workspace, forward, backward, param_grad, conjunction, checkpoint; } optimus_stack_sizes;
typedef struct { void* workspace; void* forward; void* backward; void* conjunction; void* checkpoint; } optimus_stack_buffers;
typedef void (*optimus_layer_done_fn)(int layer, void* user);
int optimus_stack_sizes_of(const optimus_layer_cfg* cfg, int n_layers, optimus_stack_sizes* out);
/* Lays one layer's parameter gradients out in a buffer of optimus_stack_sizes.param_grad bytes. */
int optimus_layer_grads_in(const optimus_layer_cfg* cfg, void* param_grad, optimus_layer_grads* out);
int optimus_stack_fwd(const optimus_layer_cfg* cfg, int n_layers, const optimus_layer_params* params, const void* x,
                      const optimus_stack_buffers* buf, void* out, void* stream);
int optimus_stack_bwd(const optimus_layer_cfg* cfg, int n_layers, const optimus_layer_params* params,
                      const optimus_layer_grads* grads, const void* d_out, const optimus_stack_buffers* buf, void* d_x,
                      optimus_layer_done_fn done, void* user, void* stream);

/* ---- the ends of the model in the 2D partition (Section 3.2.1, last paragraph; Section 3.2.2, cross entropy) ----
 * tokens / labels: int32 [b*s] (rows sequence-major, as everywhere): grid row i owns entries i*M/q ..; every device of
 * a grid row reads the same ones.  Indices outside [0, v) are clamped into range (no error is raised from a kernel).
 * table: block-major [v x h] (block (l, j) = rows l*v/q.., columns j*h/q..).
 * optimus_embedding_fwd(i, j): x_ij[t] = table[tokens[t]] restricted to columns j, i.e. the paper's one-hot product
 *   sum_l onehot_il table_lj (Algorithm 1) as a row gather; x block-major [M x h]; bit-exact copy.
 * optimus_embedding_bwd(l, j): the owner's block of the table gradient, d_table_lj = sum_i onehot_il^T dX_ij (the
 *   A^T B form, Algorithm 3, reduced within column j onto (l, j)); reads ALL token indices and the blocks (i, j) of
 *   d_x of every i (resident peers); d_table fp32 block-major [v x h], block (l, j) written completely (zeros where
 *   no token refers to a row); sums in fp32 in the order of the tokens (deterministic).
 * lm-head logits = hidden table^T: optimus_summa_abt(hidden, table, logits, M, h, v, ...).
 * Cross entropy over logits block-major [M x v] (a row spans the q devices of a grid row):
 *   stats fp32 [q][q][M/q][2]: entry (i, l) = (max, sum exp(x - max)) over device (i, l)'s columns;
 *   optimus_cross_entropy2d_stats(i, l) writes that partial only; optimus_cross_entropy2d(i, j) computes its own
 *   partial, combines the q partials of row i in the order l = 0..q-1 (peers' partials resident, as with LayerNorm),
 *   and writes loss[i][j][t] = log sum_k exp(x_tk) - x_t,label and lse[i][j][t] (both fp32 [q][q][M/q]; the q
 *   devices of a row write identical values).  optimus_cross_entropy2d_bwd(i, j):
 *   d_logits_ij = scale * (exp(x - lse) - [column == label]) in the logits' dtype (the soft-max is rebuilt from lse
 *   instead of being saved).  i = j = -1 runs every device.  dtype fp32 or bf16. */
int optimus_embedding_fwd(const int32_t* tokens, const void* table, void* x, int64_t M, int64_t v, int64_t h,
                          int q, int i, int j, int dtype, void* stream);
int optimus_embedding_bwd(const int32_t* tokens, const void* d_x, float* d_table, int64_t M, int64_t v, int64_t h,
                          int q, int l, int j, int dtype, void* stream);
int optimus_cross_entropy2d_stats(const void* logits, float* stats, int64_t M, int64_t v, int q, int i, int l,
                                  int dtype, void* stream);
int optimus_cross_entropy2d(const void* logits, const int32_t* labels, float* loss, float* lse, float* stats,
                            int64_t M, int64_t v, int q, int i, int j, int dtype, void* stream);
int optimus_cross_entropy2d_bwd(const void* logits, const int32_t* labels, const float* lse, void* d_logits,
                                float scale, int64_t M, int64_t v, int q, int i, int j, int dtype, void* stream);

/* ---- flop accounting (Table 1) ----
 * optimus_gemm_flops: 2*(M/q)*K*(N/q), one device's share of one product.
 * optimus_layer_flops: one device's share of a layer; what = 0 forward,
 * 1 backward without recomputation.  Attention is counted densely (non-causal)
 * so that forward equals 2*(12 b s h^2 + 2 b s^2 h)/q^2. */
int64_t optimus_gemm_flops(int64_t M, int64_t K, int64_t N, int q);
int64_t optimus_layer_flops(const optimus_layer_cfg* cfg, int what);

/* Measurement aid: a loop of matrix-core instructions only (v_mfma_f32_32x32x16_bf16 on register operands, no LDS,
 * no memory) on `workgroups` workgroups of eight wavefronts, `iters` times eight instructions per wavefront, with
 * all-zero (random_data = 0) or pseudo-random bf16 operands.  Timed by the caller; flops = workgroups * 8 * iters *
 * 8 * 32768.  out: device memory for workgroups * 512 floats (written, never read back by the library). */
int optimus_debug_mfma_rate(float* out, int workgroups, int iters, int random_data, void* stream);

/* ---- tuning hooks for benchmark sweeps (no effect on results beyond summation order) ----
 * Force the matrix-core tile variant used by bf16 products: 0 = 256x256, 1 = 256x128, 2 = 128x256,
 * 3 = 128x128, 4 = alias of 0, 5 = bounds-checked 128x128, 6 = 128x64, 7 = 64x64, 8 = 256x128 and 9 = 128x256 with
 * four wavefronts; -1 = automatic.  1000 + v selects, for the tiles compiled with two k-loops (0, 1, 2, 8, 9), the
 * four-slab ring instead of the 64-wide stages (identical bits); 1255 = automatic tile with that loop.
 * A variant whose tile does not divide the block falls back to the bounds-checked kernel. */
void optimus_debug_set_gemm_variant(int v);
/* The same for the products optimus_layer_bwd runs side by side on two streams only: chain_v for the
 * activation-gradient chain (the four A B^T products), branch_v for the parameter-gradient branch (the four A^T B
 * products); -1 = automatic. */
void optimus_debug_set_corun_variants(int chain_v, int branch_v);
/* The tile plan a bf16 product of this shape would be launched with: out3 = {tile variant, panel split, 1 if the
 * split is walked inside the workgroups (no partial tiles in memory)}.  Host arithmetic only, nothing is enqueued and
 * no GPU is needed.  corun: 0 = the product runs alone, 1 / 2 = it is the chain / branch product of a pair that
 * optimus_layer_bwd runs side by side; have_ws: whether the caller would pass the workspace the plan asks for.
 * The panel split (the only part of a plan that changes bits) depends on the block shape alone: not on (i, j) versus
 * grid mode, not on corun.  OPTIMUS_EDTYPE when the matrix-core kernels do not take the shape (ragged sizes). */
int optimus_debug_plan_summa(int form, int64_t M, int64_t K, int64_t N, int q, int i, int j, int corun, int have_ws, int* out3);
/* The plan of the most recent matrix-core product launched by this process: variant | (panel splits << 8) |
 * (1 << 16 if the split is emulated inside each workgroup);
 * -1 before the first one.  Host state only, not synchronised between threads. */
int optimus_debug_last_gemm_plan(void);

#ifdef __cplusplus
}
#endif
#endif /* OPTIMUS_H_ */

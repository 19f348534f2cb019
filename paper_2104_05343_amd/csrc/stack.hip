// A stack of identical transformer layers with distributed activation checkpointing and pre-allocated buffers
// (Section 3.2.3 of the paper, "memory pre-allocation and checkpointing", and its figure on checkpointing).
//
// The paper manages five reusable regions by hand instead of leaving them to an allocator: workspace, forward
// buffer, backward buffer, parameter-gradient buffer and conjunction buffer; with checkpointing only ONE layer's
// forward and backward tensors are alive at a time, so every layer reuses the same regions.  Here:
//   checkpoint   [L][M x h]      input of every layer (each device its own block: L*b*s*h/p elements per device)
//   forward      one layer's forward tensors (all of them: this library has no allocator underneath, so also the
//                LayerNorm / GeLU / attention tensors the paper leaves to PyTorch's allocator live here)
//   backward     one layer's activation gradients
//   conjunction  two [M x h] slots: the gradient handed from layer l+1 to layer l, ping-pong
//   param_grad   one layer's parameter gradients (caller-owned; all layers may share it when the caller consumes the
//                gradients in the per-layer callback, which is the paper's "update immediately, then reuse")
//   workspace    scratch of the products and of attention
// Forward: layer l reads its input from checkpoint[l] and writes its output straight into checkpoint[l+1] (the last
// one into `out`): the copy "checkpoint the input, then reset the buffers" of the paper's figure is not needed.
// Backward: for l = L-1 .. 0 the layer's forward pass is recomputed from checkpoint[l] -- without its last product,
// whose output no gradient needs -- then optimus_layer_bwd runs on the recomputed tensors.
//
// One GPU holds the whole q x q grid here, so these entry points run in grid mode only (all q*q devices' blocks, stage
// by stage): the peers' blocks of every stage of every layer cannot stay resident in buffers that all layers share.
#include "common.hpp"

using namespace optimus;

namespace {

struct Carver {
  char* base;
  size_t off;
  void* take(size_t bytes) {
    void* p = base ? base + off : nullptr;
    off += (bytes + 255) & ~(size_t)255;
    return p;
  }
};

struct Dims {
  int64_t M, h;
  int q;
  size_t act, act3, act4, rstd, stats, attn_saved;
};
int dims_of(const optimus_layer_cfg* c, Dims* d) {
  if (!c) return OPTIMUS_EINVAL;
  if (optimus_layer_workspace_bytes(c) == 0) return c->dtype != OPTIMUS_BF16 ? OPTIMUS_EDTYPE : OPTIMUS_ESHAPE;
  d->M = (int64_t)c->b * c->s; d->h = c->h; d->q = c->q;
  d->act = (size_t)d->M * d->h * 2; d->act3 = 3 * d->act; d->act4 = 4 * d->act;
  d->rstd = (size_t)d->q * d->M * 4; d->stats = 2 * d->rstd;
  const size_t nmat = (size_t)(c->b / c->q) * (c->n / c->q) * c->q * c->q;
  d->attn_saved = c->fused_attention ? nmat * c->s * 4 : nmat * c->s * c->s * 2;
  return OPTIMUS_OK;
}

// forward tensors of one layer, carved from the forward buffer (base may be null: sizes only)
size_t carve_forward(const optimus_layer_cfg* c, const Dims& d, void* base, optimus_layer_tensors* t) {
  Carver k{(char*)base, 0};
  optimus_layer_tensors z = {};
  optimus_layer_tensors& o = t ? *t : z;
  o.ln1_out = k.take(d.act); o.xhat1 = k.take(d.act); o.rstd1 = (float*)k.take(d.rstd); o.stats1 = (float*)k.take(d.stats);
  o.qkv = k.take(d.act3);
  if (c->fused_attention) o.lse = (float*)k.take(d.attn_saved);
  else o.probs = k.take(d.attn_saved);
  o.attn = k.take(d.act); o.h_mid = k.take(d.act);
  o.ln2_out = k.take(d.act); o.xhat2 = k.take(d.act); o.rstd2 = (float*)k.take(d.rstd); o.stats2 = (float*)k.take(d.stats);
  o.pre_gelu = k.take(d.act4); o.gelu = k.take(d.act4);
  return k.off;
}
size_t carve_backward(const Dims& d, void* base, optimus_layer_tensors* t) {
  Carver k{(char*)base, 0};
  optimus_layer_tensors z = {};
  optimus_layer_tensors& o = t ? *t : z;
  o.d_pre_gelu = k.take(d.act4); o.d_ln2_out = k.take(d.act); o.d_h_mid = k.take(d.act); o.d_attn = k.take(d.act);
  o.d_qkv = k.take(d.act3); o.d_ln1_out = k.take(d.act);
  o.bstats1 = (float*)k.take(d.stats); o.bstats2 = (float*)k.take(d.stats);
  return k.off;
}
size_t carve_grads(const Dims& d, void* base, optimus_layer_grads* g) {
  Carver k{(char*)base, 0};
  optimus_layer_grads z = {};
  optimus_layer_grads& o = g ? *g : z;
  const size_t hh = (size_t)d.h * d.h * 4, vec = (size_t)d.q * d.h * 4;  // [h x h] fp32; [q][q][h/q] fp32 partials
  o.d_w_qkv = (float*)k.take(3 * hh); o.d_w_o = (float*)k.take(hh); o.d_w1 = (float*)k.take(4 * hh); o.d_w2 = (float*)k.take(4 * hh);
  o.d_b_qkv = (float*)k.take(3 * vec); o.d_b_o = (float*)k.take(vec); o.d_b1 = (float*)k.take(4 * vec); o.d_b2 = (float*)k.take(vec);
  o.d_ln1_g = (float*)k.take(vec); o.d_ln1_b = (float*)k.take(vec); o.d_ln2_g = (float*)k.take(vec); o.d_ln2_b = (float*)k.take(vec);
  return k.off;
}

void set_params(optimus_layer_tensors* t, const optimus_layer_params& p) {
  t->ln1_g = p.ln1_g; t->ln1_b = p.ln1_b; t->w_qkv = p.w_qkv; t->b_qkv = p.b_qkv; t->w_o = p.w_o; t->b_o = p.b_o;
  t->ln2_g = p.ln2_g; t->ln2_b = p.ln2_b; t->w1 = p.w1; t->b1 = p.b1; t->w2 = p.w2; t->b2 = p.b2;
}
bool params_ok(const optimus_layer_params& p) {
  return p.ln1_g && p.ln1_b && p.w_qkv && p.b_qkv && p.w_o && p.b_o && p.ln2_g && p.ln2_b && p.w1 && p.b1 && p.w2 && p.b2;
}
bool grads_ok(const optimus_layer_grads& g) {
  return g.d_w_qkv && g.d_w_o && g.d_w1 && g.d_w2 && g.d_b_qkv && g.d_b_o && g.d_b1 && g.d_b2 && g.d_ln1_g && g.d_ln1_b &&
         g.d_ln2_g && g.d_ln2_b;
}

}  // namespace

extern "C" {

int optimus_stack_sizes_of(const optimus_layer_cfg* cfg, int n_layers, optimus_stack_sizes* out) {
  Dims d;
  int rc = dims_of(cfg, &d);
  if (rc) return rc;
  if (!out) return OPTIMUS_EINVAL;
  if (n_layers < 1 || n_layers > 65536) return OPTIMUS_ESHAPE;
  out->workspace = optimus_layer_workspace_bytes_grid(cfg);   // the stack runs the whole grid
  out->forward = carve_forward(cfg, d, nullptr, nullptr);
  out->backward = carve_backward(d, nullptr, nullptr);
  out->param_grad = carve_grads(d, nullptr, nullptr);
  out->conjunction = 2 * ((d.act + 255) & ~(size_t)255);
  out->checkpoint = (size_t)n_layers * d.act;
  return OPTIMUS_OK;
}

int optimus_layer_grads_in(const optimus_layer_cfg* cfg, void* param_grad, optimus_layer_grads* out) {
  Dims d;
  int rc = dims_of(cfg, &d);
  if (rc) return rc;
  if (!param_grad || !out) return OPTIMUS_EINVAL;
  carve_grads(d, param_grad, out);
  return OPTIMUS_OK;
}

int optimus_stack_fwd(const optimus_layer_cfg* cfg, int n_layers, const optimus_layer_params* params, const void* x,
                      const optimus_stack_buffers* buf, void* out, void* stream) {
  Dims d;
  int rc = dims_of(cfg, &d);
  if (rc) return rc;
  if (n_layers < 1 || n_layers > 65536) return OPTIMUS_ESHAPE;
  if (!params || !x || !buf || !out || !buf->workspace || !buf->forward || !buf->checkpoint) return OPTIMUS_EINVAL;
  for (int l = 0; l < n_layers; ++l)
    if (!params_ok(params[l])) return OPTIMUS_EINVAL;
  char* ck = (char*)buf->checkpoint;
  if (hipMemcpyAsync(ck, x, d.act, hipMemcpyDeviceToDevice, (hipStream_t)stream) != hipSuccess) return OPTIMUS_EHIP;
  const size_t ws_bytes = optimus_layer_workspace_bytes_grid(cfg);
  for (int l = 0; l < n_layers; ++l) {
    optimus_layer_tensors t = {};
    carve_forward(cfg, d, buf->forward, &t);
    set_params(&t, params[l]);
    t.x = ck + (size_t)l * d.act;
    t.out = l + 1 < n_layers ? (void*)(ck + (size_t)(l + 1) * d.act) : out;
    if ((rc = layer_forward(cfg, &t, -1, -1, buf->workspace, ws_bytes, stream, false))) return rc;
  }
  return OPTIMUS_OK;
}

int optimus_stack_bwd(const optimus_layer_cfg* cfg, int n_layers, const optimus_layer_params* params,
                      const optimus_layer_grads* grads, const void* d_out, const optimus_stack_buffers* buf, void* d_x,
                      optimus_layer_done_fn done, void* user, void* stream) {
  Dims d;
  int rc = dims_of(cfg, &d);
  if (rc) return rc;
  if (n_layers < 1 || n_layers > 65536) return OPTIMUS_ESHAPE;
  if (!params || !grads || !d_out || !buf || !d_x || !buf->workspace || !buf->forward || !buf->backward || !buf->conjunction ||
      !buf->checkpoint)
    return OPTIMUS_EINVAL;
  for (int l = 0; l < n_layers; ++l)
    if (!params_ok(params[l]) || !grads_ok(grads[l])) return OPTIMUS_EINVAL;
  const size_t ws_bytes = optimus_layer_workspace_bytes_grid(cfg);
  const size_t slot = (d.act + 255) & ~(size_t)255;
  const char* ck = (const char*)buf->checkpoint;
  const void* g_in = d_out;
  for (int l = n_layers - 1; l >= 0; --l) {
    optimus_layer_tensors t = {};
    carve_forward(cfg, d, buf->forward, &t);
    carve_backward(d, buf->backward, &t);
    set_params(&t, params[l]);
    t.x = ck + (size_t)l * d.act;
    if ((rc = layer_forward(cfg, &t, -1, -1, buf->workspace, ws_bytes, stream, true))) return rc;  // recomputation
    const optimus_layer_grads& g = grads[l];
    t.d_w_qkv = g.d_w_qkv; t.d_w_o = g.d_w_o; t.d_w1 = g.d_w1; t.d_w2 = g.d_w2;
    t.d_b_qkv = g.d_b_qkv; t.d_b_o = g.d_b_o; t.d_b1 = g.d_b1; t.d_b2 = g.d_b2;
    t.d_ln1_g = g.d_ln1_g; t.d_ln1_b = g.d_ln1_b; t.d_ln2_g = g.d_ln2_g; t.d_ln2_b = g.d_ln2_b;
    t.d_out = g_in;
    void* g_out = l == 0 ? d_x : (void*)((char*)buf->conjunction + (size_t)(l & 1) * slot);
    t.d_x = g_out;
    if ((rc = optimus_layer_bwd(cfg, &t, -1, -1, buf->workspace, ws_bytes, stream))) return rc;
    if (done) done(l, user);
    g_in = g_out;
  }
  return OPTIMUS_OK;
}

}  // extern "C"

// C ABI of libl2pd: argument checks, workspace layout, and the launch sequences of
// M(X) (forward), one denoising step (Alg. 2 loop body) and the whole decode (Alg. 2 / Alg. 3).
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <vector>

#include "common.h"

using namespace l2pd;

namespace {

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Carver {
  size_t off = 0;
  size_t take(size_t bytes) {
    size_t o = off;
    off = align_up(off + bytes, 256);
    return o;
  }
};

struct Layout {
  // offsets into the workspace
  size_t cos_t, sin_t, ctl, state, state2, perm, perm2, teff, X, X2, h, xn, q, attn, act, parts, attn_ws, attn_ws_bytes, kstore, vstore, tmp_k, tmp_v, gate_up,
      xn_head, logits, part_max, part_sum, part_idx, conf, pred, total;
  size_t kv_layer_stride_k, kv_layer_stride_v;
  int Tpad, n_part, lm_chunk;
};

struct ProfileEv {
  hipEvent_t a, b;
};

}  // namespace

struct l2pd_ctx {
  l2pd_model_desc m;
  std::vector<const void*> attn_g, wq, wk, wv, wo, ffn_g, wg, wu, wd;
  const void *tok_emb, *lm_head, *final_g;
  int max_batch, max_seq, cache;
  unsigned char* ws;
  size_t ws_bytes;
  Layout L;
  bool device_ready = false;
  // host side of the generate loop
  int* pinned = nullptr;                 // polled copies of the control block
  hipEvent_t poll_ev[2] = {nullptr, nullptr};
  // timing aid
  int prof_class = 0;
  std::vector<ProfileEv> prof;
  std::vector<ProfileEv> prof_pool;
  int last_hip_error = 0;
  int pend_splits = 0;   // bf16: split-K partials of the last down projection still to be folded into h
  size_t pend_stride = 0;
  // the last l2pd_generate: step launches enqueued, and the sum over them of the sequences each ran over
  int64_t stat_steps = 0, stat_seq_steps = 0;

  template <typename T>
  T* at(size_t off) const { return reinterpret_cast<T*>(ws + off); }
};

namespace {

bool desc_ok(const l2pd_model_desc* d) {
  if (!d) return false;
  if (d->n_layers < 1 || d->d_model < 1 || d->n_heads < 1 || d->head_dim < 2 || d->d_ffn < 1 || d->vocab < 2)
    return false;
  if (d->n_heads * d->head_dim != d->d_model) return false;
  if (d->head_dim % 2) return false;
  if (d->mask_id < 0 || d->mask_id >= d->vocab || d->eos_id < 0 || d->eos_id >= d->vocab) return false;
  if (d->mask_id == d->eos_id) return false;
  if (!(d->rope_base > 0.f) || !(d->rms_eps >= 0.f)) return false;
  if (d->dtype != L2PD_FP32 && d->dtype != L2PD_BF16) return false;
  return true;
}

int desc_supported(const l2pd_model_desc* d) {
  if (d->dtype == L2PD_BF16) {
    if (d->d_model % 64 || d->d_ffn % 64) return L2PD_ENOTIMPL;
    if (d->head_dim != 64 && d->head_dim != 128) return L2PD_ENOTIMPL;
  } else {
    if (d->head_dim > 256) return L2PD_ENOTIMPL;
  }
  return L2PD_OK;
}

Layout make_layout(const l2pd_model_desc& m, int max_batch, int max_seq, int cache) {
  Layout L = {};
  Carver c;
  const size_t es = m.dtype == L2PD_FP32 ? 4 : 2;
  const size_t rows = (size_t)max_batch * max_seq;
  const size_t d = m.d_model, F = m.d_ffn, V = m.vocab;
  L.Tpad = (int)align_up(max_seq, 64);
  L.lm_chunk = 1024;
  L.n_part = m.dtype == L2PD_FP32 ? (int)((V + L.lm_chunk - 1) / L.lm_chunk) : lmhead_n_part((int)V);
  const size_t head_rows = (size_t)max_batch * 256;   // block_len <= 256
  L.cos_t = c.take((size_t)L.Tpad * (m.head_dim / 2) * 4);
  L.sin_t = c.take((size_t)L.Tpad * (m.head_dim / 2) * 4);
  L.ctl = c.take((size_t)(CTL_WORDS + 2 * max_batch) * 4);   // control words, per-sequence blocks, per-sequence done flags
  L.state = c.take((size_t)max_batch * 3 * 4);
  L.state2 = c.take((size_t)max_batch * 3 * 4);   // second copies for batch compaction
  L.perm = c.take((size_t)max_batch * 4);
  L.perm2 = c.take((size_t)max_batch * 4);
  L.teff = c.take((size_t)max_batch * 4);
  L.X = c.take(rows * 4);
  L.X2 = c.take(rows * 4);
  L.h = c.take(rows * d * 4);
  L.xn = c.take(align_up(rows, 4) * d * es);   // the quad-tiled layout holds whole groups of four rows
  L.q = c.take(rows * d * es);
  L.attn = c.take(align_up(rows, 4) * d * es);
  L.act = c.take(align_up(rows, 4) * F * es);
  const size_t kv_one = (size_t)max_batch * L.Tpad * d * es;
  const size_t n_kv = cache ? m.n_layers : 1;
  L.kv_layer_stride_k = kv_one;
  L.kv_layer_stride_v = kv_one;
  L.kstore = c.take(kv_one * n_kv);
  L.vstore = c.take(kv_one * n_kv);
  if (m.dtype == L2PD_FP32) {
    L.tmp_k = c.take(rows * d * 4);
    L.tmp_v = c.take(rows * d * 4);
    L.gate_up = c.take(rows * F * 4 * 2);
    L.logits = c.take(head_rows * V * 4);
  } else {
    // fp32 split-K partials: two [rows, d] buffers on the wide path; on the few-row path up to
    // kSkinnyRows rows of every K range of the widest stacked projection
    size_t skinny = 0;
    const int shapes[4][2] = {{3 * m.d_model, m.d_model}, {m.d_model, m.d_model}, {2 * m.d_ffn, m.d_model},
                              {m.d_model, m.d_ffn}};
    for (auto& sh : shapes) {
      const size_t b = (size_t)skinny_splits(sh[0], sh[1]) * kSkinnyRows * sh[0] * 4;
      if (b > skinny) skinny = b;
    }
    // wide path: the [d, d] and [d, F] projections split K as far as wide_splits says for the number of
    // rows at hand (it depends on the count of 128-row tiles only, so the top of every bucket is the worst case)
    size_t wide = 0;
    for (size_t top = 128;; top += 128) {
      const size_t M = top < rows ? top : rows;
      const int S = std::max(wide_splits((int)M, m.d_model, m.d_model), wide_splits((int)M, m.d_model, m.d_ffn));
      wide = std::max(wide, (size_t)S * M * d * 4);
      if (top >= rows) break;
    }
    L.parts = c.take(wide > skinny ? wide : skinny);
    L.attn_ws_bytes = attn_chunk_ws_bytes(m.n_heads, m.head_dim);
    L.attn_ws = c.take(L.attn_ws_bytes);
  }
  L.xn_head = c.take(align_up(rows, 4) * d * es);   // l2pd_forward may ask for every row; quad-tiled layout: rows in fours
  L.part_max = c.take(head_rows * L.n_part * 4);
  L.part_sum = c.take(head_rows * L.n_part * 4);
  L.part_idx = c.take(head_rows * L.n_part * 4);
  L.conf = c.take(head_rows * 4);
  L.pred = c.take(head_rows * 4);
  L.total = c.off;
  return L;
}

#define HIP_TRY(ctx, expr)                       \
  do {                                           \
    hipError_t e_ = (expr);                      \
    if (e_ != hipSuccess) {                      \
      (ctx)->last_hip_error = (int)e_;           \
      return L2PD_EHIP;                          \
    }                                            \
  } while (0)

int ensure_device(l2pd_ctx* c, hipStream_t s) {
  if (c->device_ready) return L2PD_OK;
  // Zero the workspace once: padded key/value slots must hold finite numbers.
  launch_fill_u32(reinterpret_cast<uint32_t*>(c->ws), c->L.total / 4, 0u, s);
  launch_rope_table(c->at<float>(c->L.cos_t), c->at<float>(c->L.sin_t), c->L.Tpad, c->m.head_dim, c->m.rope_base, s);
  HIP_TRY(c, hipGetLastError());
  c->device_ready = true;
  return L2PD_OK;
}

// ---- timing aid ----
struct Timed {
  l2pd_ctx* c;
  hipStream_t s;
  bool on;
  ProfileEv ev;
  Timed(l2pd_ctx* c_, int cls, hipStream_t s_) : c(c_), s(s_), on(c_->prof_class == cls && cls != 0) {
    if (!on) return;
    if (!c->prof_pool.empty()) {
      ev = c->prof_pool.back();
      c->prof_pool.pop_back();
    } else if (hipEventCreate(&ev.a) != hipSuccess || hipEventCreate(&ev.b) != hipSuccess) {
      on = false;
      return;
    }
    (void)hipEventRecord(ev.a, s);
  }
  ~Timed() {
    if (!on) return;
    (void)hipEventRecord(ev.b, s);
    c->prof.push_back(ev);
  }
};

// One transformer pass over `B` sequences with `Tq` rows each at absolute positions pos0 .. pos0+Tq-1,
// attending to keys 0 .. Tk-1 of the key/value stores (which this pass fills at pos0 .. pos0+Tq-1).
struct Pass {
  int B, Tq, pos0, Tk;
  int Tfull;            // row length of the token array
  const int32_t* tokens;
  bool per_layer_kv;    // prefix cache: one K/V store per layer
  bool kv_only_last;    // refresh pass: the last layer only has to leave its K/V
  const int* tk_dev = nullptr;   // per-sequence number of keys (device), else null
  int kv_seq = 0;       // first sequence slot of the K/V stores this pass works on (single-sequence store rebuilds)
  int pos_per_gb = 0;   // > 0: per-sequence block pointers with a cache: sequence b's rows sit at pos0 + own block * pos_per_gb
};

void run_layers(l2pd_ctx* c, const Pass& p, Gate g, hipStream_t s) {
  const l2pd_model_desc& m = c->m;
  const Layout& L = c->L;
  const int rows = p.B * p.Tq, d = m.d_model, F = m.d_ffn, H = m.n_heads, Dh = m.head_dim;
  const RowMap ident = {rows, 0, 0, 0};
  float* h = c->at<float>(L.h);
  launch_embed(h, c->tok_emb, m.dtype, p.tokens, RowMap{p.Tq, p.Tfull, p.pos0, p.pos_per_gb}, rows, d, g, s);
  const int* seq_gb = p.pos_per_gb ? c->at<int>(L.ctl) + CTL_SEQ_GB : nullptr;
  const size_t kv_seq_off = (size_t)p.kv_seq * L.Tpad * d * (m.dtype == L2PD_FP32 ? 4 : 2);
  const float* cos_t = c->at<float>(L.cos_t);
  const float* sin_t = c->at<float>(L.sin_t);
  bool pending = false;   // bf16: split-K partials of the previous projection not yet folded into h
  int pend_splits = 0;
  size_t pend_stride = 0;
  for (int l = 0; l < m.n_layers; ++l) {
    const size_t kvo_k = p.per_layer_kv ? L.kv_layer_stride_k * l : 0;
    const size_t kvo_v = p.per_layer_kv ? L.kv_layer_stride_v * l : 0;
    if (m.dtype == L2PD_FP32) {
      float* xn = c->at<float>(L.xn);
      float* q = c->at<float>(L.q);
      float* ks = reinterpret_cast<float*>(c->ws + L.kstore + kvo_k + kv_seq_off);
      float* vs = reinterpret_cast<float*>(c->ws + L.vstore + kvo_v + kv_seq_off);
      { Timed t(c, L2PD_K_NORM, s);
        launch_rmsnorm(h, nullptr, 0, 0, ident, c->attn_g[l], m.dtype, xn, rows, d, m.rms_eps, true, g, s); }
      { Timed t(c, L2PD_K_GEMM_QKV, s);
        launch_gemm_f32(xn, (const float*)c->wq[l], q, rows, d, d, 0, g, s);
        launch_gemm_f32(xn, (const float*)c->wk[l], c->at<float>(L.tmp_k), rows, d, d, 0, g, s);
        launch_gemm_f32(xn, (const float*)c->wv[l], c->at<float>(L.tmp_v), rows, d, d, 0, g, s);
        launch_rope_store_f32(q, c->at<float>(L.tmp_k), c->at<float>(L.tmp_v), ks, vs, p.B, p.Tq, p.pos0, L.Tpad, H,
                              Dh, cos_t, sin_t, seq_gb, p.pos_per_gb, g, s); }
      if (p.kv_only_last && l + 1 == m.n_layers) break;
      { Timed t(c, L2PD_K_ATTN, s);
        launch_attn_f32(q, ks, vs, c->at<float>(L.attn), p.B, p.Tq, p.Tk, L.Tpad, H, Dh, p.tk_dev, g, s); }
      { Timed t(c, L2PD_K_GEMM_O, s);
        launch_gemm_f32(c->at<float>(L.attn), (const float*)c->wo[l], h, rows, d, d, 1, g, s); }
      { Timed t(c, L2PD_K_NORM, s);
        launch_rmsnorm(h, nullptr, 0, 0, ident, c->ffn_g[l], m.dtype, xn, rows, d, m.rms_eps, true, g, s); }
      float* gt = c->at<float>(L.gate_up);
      float* up = gt + (size_t)rows * F;
      { Timed t(c, L2PD_K_GEMM_GATEUP, s);
        launch_gemm_f32(xn, (const float*)c->wg[l], gt, rows, F, d, 0, g, s);
        launch_gemm_f32(xn, (const float*)c->wu[l], up, rows, F, d, 0, g, s);
        launch_swiglu_f32(gt, up, c->at<float>(L.act), (size_t)rows * F, g, s); }
      { Timed t(c, L2PD_K_GEMM_DOWN, s);
        launch_gemm_f32(c->at<float>(L.act), (const float*)c->wd[l], h, rows, d, F, 1, g, s); }
    } else {
      bf16* xn = c->at<bf16>(L.xn);
      bf16* q = c->at<bf16>(L.q);
      bf16* ks = reinterpret_cast<bf16*>(c->ws + L.kstore + kvo_k + kv_seq_off);
      bf16* vts = reinterpret_cast<bf16*>(c->ws + L.vstore + kvo_v + kv_seq_off);
      float* parts = c->at<float>(L.parts);
      const bool skinny = rows <= kSkinnyRows;
      // the activations go to the fused GEMMs in the layout these ask for (row-major or quad-tiled)
      const bool tiled_qkv = !skinny && gemm_qkv_a_quad_tiled(rows, d, d, Dh);
      const bool tiled_ffn = !skinny && gemm_swiglu_a_quad_tiled(rows, F, d);
      const bool tiled_o = !skinny && gemm_partial_a_quad_tiled(rows, d, d);      // attention output -> output projection
      const bool tiled_down = !skinny && gemm_partial_a_quad_tiled(rows, d, F);   // SwiGLU activations -> down projection
      { Timed t(c, L2PD_K_NORM, s);
        launch_rmsnorm(h, pending ? parts : nullptr, pend_splits, pend_stride, ident, c->attn_g[l], m.dtype, xn, rows,
                       d, m.rms_eps, true, g, s, tiled_qkv); }
      pending = false;
      QkvEpilogue e = {q, ks, vts, cos_t, sin_t, p.Tq, p.pos0, L.Tpad, H, Dh, d, seq_gb, p.pos_per_gb};
      { Timed t(c, L2PD_K_GEMM_QKV, s);
        if (skinny) {
          const int S = skinny_splits(3 * d, d);
          const size_t stride = (size_t)rows * 3 * d;
          launch_gemm_skinny_bf16(xn, (const bf16*)c->wq[l], (const bf16*)c->wk[l], (const bf16*)c->wv[l], d, parts,
                                  stride, rows, 3 * d, d, S, g, s);
          launch_skinny_qkv_finish(parts, S, stride, rows, e, g, s);
        } else {
          launch_gemm_qkv_bf16(xn, (const bf16*)c->wq[l], (const bf16*)c->wk[l], (const bf16*)c->wv[l], rows, d, e, g,
                               s);
        } }
      if (p.kv_only_last && l + 1 == m.n_layers) break;
      bf16* ao = c->at<bf16>(L.attn);
      { Timed t(c, L2PD_K_ATTN, s);
        launch_attn_bf16(q, ks, vts, ao, p.B, p.Tq, p.Tk, L.Tpad, H, Dh, c->at<float>(L.attn_ws), L.attn_ws_bytes,
                         p.tk_dev, g, s, tiled_o); }
      // Few row tiles leave CUs idle on the [d, d] and [d, F] projections: split K as far as
      // wide_splits (wide path) or skinny_splits (few-row path) says.
      const int so = skinny ? skinny_splits(d, d) : wide_splits(rows, d, d);
      const int sd = skinny ? skinny_splits(d, F) : wide_splits(rows, d, F);
      const size_t stride_d = (size_t)rows * d;
      { Timed t(c, L2PD_K_GEMM_O, s);
        if (skinny)
          launch_gemm_skinny_bf16(ao, (const bf16*)c->wo[l], nullptr, nullptr, 0, parts, stride_d, rows, d, d, so, g,
                                  s);
        else
          launch_gemm_partial_bf16(ao, (const bf16*)c->wo[l], parts, stride_d, rows, d, d, so, g, s); }
      { Timed t(c, L2PD_K_NORM, s);
        launch_rmsnorm(h, parts, so, stride_d, ident, c->ffn_g[l], m.dtype, xn, rows, d, m.rms_eps, true, g, s,
                       tiled_ffn); }
      bf16* act = c->at<bf16>(L.act);
      { Timed t(c, L2PD_K_GEMM_GATEUP, s);
        if (skinny && !swiglu_few_rows_fused(rows, F)) {
          const int S = skinny_splits(2 * F, d);
          const size_t stride = (size_t)rows * 2 * F;
          launch_gemm_skinny_bf16(xn, (const bf16*)c->wg[l], (const bf16*)c->wu[l], nullptr, F, parts, stride, rows,
                                  2 * F, d, S, g, s);
          launch_skinny_swiglu_finish(parts, S, stride, rows, F, act, g, s);
        } else {
          launch_gemm_swiglu_bf16(xn, (const bf16*)c->wg[l], (const bf16*)c->wu[l], act, rows, F, d, g, s, tiled_down);
        } }
      { Timed t(c, L2PD_K_GEMM_DOWN, s);
        if (skinny)
          launch_gemm_skinny_bf16(act, (const bf16*)c->wd[l], nullptr, nullptr, 0, parts, stride_d, rows, d, F, sd, g,
                                  s);
        else
          launch_gemm_partial_bf16(act, (const bf16*)c->wd[l], parts, stride_d, rows, d, F, sd, g, s); }
      pending = true;
      pend_splits = sd;
      pend_stride = stride_d;
    }
  }
  // bf16: the last down projection's partials are folded in by the final norm (see run_head)
  c->pend_splits = pending ? pend_splits : 0;
  c->pend_stride = pend_stride;
}

// Final RMSNorm of the selected rows + LM head.  Produces the vocabulary partials (and optionally
// the fp32 logits) of `n_rows_per_seq` rows per sequence, taken from h through `src`.
void run_head(l2pd_ctx* c, int B, int n_rows_per_seq, RowMap src, float* logits_out, bool want_parts,
              BiasArgs bias, Gate g, hipStream_t s) {
  const l2pd_model_desc& m = c->m;
  const Layout& L = c->L;
  const int d = m.d_model, V = m.vocab, hr = B * n_rows_per_seq;
  float* h = c->at<float>(L.h);
  if (m.dtype == L2PD_FP32) {
    float* xh = c->at<float>(L.xn_head);
    { Timed t(c, L2PD_K_NORM, s);
      launch_rmsnorm(h, nullptr, 0, 0, src, c->final_g, m.dtype, xh, hr, d, m.rms_eps, false, g, s); }
    float* lg = logits_out ? logits_out : c->at<float>(L.logits);
    Timed t(c, L2PD_K_LMHEAD, s);
    launch_gemm_f32(xh, (const float*)c->lm_head, lg, hr, V, d, 0, g, s);
    if (want_parts)
      launch_vocab_partials(lg, hr, V, L.lm_chunk, m.mask_id, bias, c->at<float>(L.part_max),
                            c->at<float>(L.part_sum), c->at<int32_t>(L.part_idx), L.n_part, g, s);
  } else {
    // the last down projection's split-K partials are summed onto the selected rows in fixed order;
    // h itself is left as it is (nothing reads it afterwards, and with shortened sequences two head
    // rows may map to one row of h)
    bf16* xh = c->at<bf16>(L.xn_head);
    const int sd = c->pend_splits;
    { Timed t(c, L2PD_K_NORM, s);
      launch_rmsnorm(h, sd > 0 ? c->at<float>(L.parts) : nullptr, sd, c->pend_stride, src, c->final_g, m.dtype, xh, hr,
                     d, m.rms_eps, false, g, s, gemm_lmhead_a_quad_tiled(hr, V, d)); }
    LmHeadEpilogue e = {};
    e.logits = logits_out;
    if (want_parts) {
      e.part_max = c->at<float>(L.part_max);
      e.part_sum = c->at<float>(L.part_sum);
      e.part_idx = c->at<int32_t>(L.part_idx);
    }
    e.n_part = L.n_part;
    e.mask_id = m.mask_id;
    e.bias = bias;
    Timed t(c, L2PD_K_LMHEAD, s);
    launch_gemm_lmhead_bf16(xh, (const bf16*)c->lm_head, hr, V, d, e, g, s);
  }
}

static_assert(L2PD_FILTER_MAX_LAYERS == kFilterMaxLayers, "filter depth limit");
bool filter_ok(const l2pd_filter* f) {
  if (f->n_layers < 1 || f->n_layers > L2PD_FILTER_MAX_LAYERS || f->in_dim < 1) return false;
  if (f->n_layers > 1 && (f->hidden < 1 || f->hidden > 1024)) return false;
  for (int k = 0; k < f->n_layers; ++k)
    if (!f->w_dev[k] || !f->b_dev[k]) return false;
  return true;
}

int check_decode_args(const l2pd_ctx* c, int B, int P, const l2pd_decode_cfg* cfg, const l2pd_filter* f) {
  if (!c || !cfg || !f) return L2PD_EINVAL;
  if (B < 1 || B > c->max_batch || P < 1) return L2PD_EINVAL;
  if (cfg->gen_len < 1 || cfg->block_len < 1 || cfg->block_len > 256) return L2PD_EINVAL;
  if (cfg->gen_len % cfg->block_len) return L2PD_EINVAL;
  if ((long long)P + cfg->gen_len > c->max_seq) return L2PD_EINVAL;
  if (f->in_dim != cfg->block_len || !filter_ok(f)) return L2PD_EINVAL;
  if (isnan(cfg->threshold)) return L2PD_EINVAL;
  if (cfg->kv_cache < L2PD_CACHE_NONE || cfg->kv_cache > L2PD_CACHE_DUAL) return L2PD_EINVAL;
  if (cfg->kv_cache && !c->cache) return L2PD_EINVAL;
  if (cfg->eotp < 0 || cfg->eotp > L2PD_EOTP_STEP) return L2PD_EINVAL;
  if (cfg->eotp == L2PD_EOTP_STEP && cfg->kv_cache) return L2PD_ENOTIMPL;   // shortened sequences: full recompute only
  if (cfg->ragged < 0 || cfg->ragged > L2PD_RAGGED_COMPACT) return L2PD_EINVAL;
  if (cfg->bias.value != 0.f && (cfg->bias.token_id < 0 || cfg->bias.token_id >= c->m.vocab)) return L2PD_EINVAL;
  if (isnan(cfg->bias.value)) return L2PD_EINVAL;
  return L2PD_OK;
}

struct EgpArgs {             // Alg. 1 rollout: reference answers in, training rows out
  const int32_t* reference;  // [B, gen_len]
  float* conf;               // [B, gen_len, s]
  float* label;
};

struct StepTaps {
  float* logits;
  float* conf;
  int32_t* pred;
  float* filt;
  uint8_t* unmask;
};

// Rebuild the K/V store for block gb.  Prefix cache: K/V of a forward over X[0 : P + gb*s] alone.
// Dual cache: K/V of every position from a full bidirectional forward over X as it is now.
void run_refresh(l2pd_ctx* c, const int32_t* X, int B, int P, const l2pd_decode_cfg* cfg, int gb, Gate g,
                 hipStream_t s) {
  const int T = P + cfg->gen_len;
  const int rows = cfg->kv_cache == L2PD_CACHE_DUAL ? T : P + gb * cfg->block_len;
  Pass p = {B, rows, 0, rows, T, X, true, true};
  run_layers(c, p, g, s);
}

// The same for one sequence of the batch (per-sequence block pointers with a cache): its slice of the
// stores is rebuilt from its own tokens for its own block gb.
void run_refresh_seq(l2pd_ctx* c, const int32_t* X, int b, int P, const l2pd_decode_cfg* cfg, int gb, Gate g,
                     hipStream_t s) {
  const int T = P + cfg->gen_len;
  const int rows = cfg->kv_cache == L2PD_CACHE_DUAL ? T : P + gb * cfg->block_len;
  Pass p = {1, rows, 0, rows, T, X + (size_t)b * T, true, true};
  p.kv_seq = b;
  run_layers(c, p, g, s);
}

// One denoising step for the lock-step batch.  host_gb >= 0 is required with a cache, unless every
// sequence follows its own block pointer (then the store rebuilds are the caller's, per sequence).
// t_run > 0 (step-granular EoTP): the forward runs over the first t_run positions of every sequence,
// each sequence attending to its own teff[b] <= t_run keys.
void run_step(l2pd_ctx* c, int32_t* X, int B, int P, const l2pd_decode_cfg* cfg, const l2pd_filter* f,
              int32_t* state, int host_gb, const StepTaps& taps, hipStream_t s, int t_run = 0,
              const EgpArgs* egp = nullptr) {
  const Layout& L = c->L;
  const int sl = cfg->block_len, T = P + cfg->gen_len, nb = cfg->gen_len / sl;
  int* ctl = c->at<int>(L.ctl);
  launch_prepare(state, B, nb, cfg->ragged, ctl, s);
  const bool own_blocks_cached = cfg->kv_cache && cfg->ragged;
  Gate g = {ctl, (cfg->kv_cache && !own_blocks_cached) ? host_gb : -1};
  BiasArgs bias = {cfg->bias.token_id, cfg->bias.gen_pos_from, sl, cfg->bias.value};
  if (own_blocks_cached) {
    // per-sequence block pointers: every sequence's block rows sit at its own positions (read from the
    // control block by the embedding, the rotation / store epilogues and the update), and with the prefix
    // cache every sequence sees its own number of keys
    Pass p = {B, sl, P, T, T, X, true, false};
    p.pos_per_gb = sl;
    if (cfg->kv_cache == L2PD_CACHE_PREFIX) {
      launch_block_keys(ctl, B, P + sl, sl, c->at<int>(L.teff), s);
      p.tk_dev = c->at<int>(L.teff);
    }
    run_layers(c, p, g, s);
    run_head(c, B, sl, RowMap{B * sl, 0, 0, 0}, taps.logits, true, bias, g, s);
  } else if (cfg->kv_cache) {
    // block rows only; their K/V go into the store at the block's positions, and the queries see
    // the store up to the end of the block (prefix cache) or all of it (dual cache)
    const int cpos = P + host_gb * sl;
    Pass p = {B, sl, cpos, cfg->kv_cache == L2PD_CACHE_DUAL ? T : cpos + sl, T, X, true, false};
    run_layers(c, p, g, s);
    run_head(c, B, sl, RowMap{B * sl, 0, 0, 0}, taps.logits, true, bias, g, s);
  } else if (t_run > 0) {
    Pass p = {B, t_run, 0, t_run, T, X, false, false};
    p.tk_dev = c->at<int>(L.teff);
    run_layers(c, p, g, s);
    // block rows past a sequence's end are read (stale rows of the buffer) and ignored by the update
    run_head(c, B, sl, RowMap{sl, t_run, P, sl}, taps.logits, true, bias, g, s);
  } else {
    Pass p = {B, T, 0, T, T, X, false, false};
    run_layers(c, p, g, s);
    run_head(c, B, sl, RowMap{sl, T, P, sl}, taps.logits, true, bias, g, s);
  }
  UpdateArgs u = {};
  u.X = X; u.state = state; u.B = B; u.P = P; u.T = T; u.s = sl; u.n_blocks = nb;
  u.mask_id = c->m.mask_id; u.eos_id = c->m.eos_id; u.eotp = cfg->eotp;
  u.part_max = c->at<float>(L.part_max); u.part_sum = c->at<float>(L.part_sum);
  u.part_idx = c->at<int32_t>(L.part_idx); u.n_part = L.n_part;
  if (f) {
    for (int k = 0; k < f->n_layers; ++k) { u.fw[k] = f->w_dev[k]; u.fb[k] = f->b_dev[k]; }
    u.n_layers = f->n_layers;
    u.hidden = f->hidden;
  }
  if (egp) { u.reference = egp->reference; u.egp_conf = egp->conf; u.egp_label = egp->label; }
  u.gen_len = cfg->gen_len;
  u.tau = cfg->threshold;
  u.conf_out = taps.conf; u.pred_out = taps.pred; u.filt_out = taps.filt; u.unmask_out = taps.unmask;
  u.ctl = ctl;
  u.teff = t_run > 0 ? c->at<int>(L.teff) : nullptr;
  Timed t(c, L2PD_K_UPDATE, s);
  launch_update(u, g, s);
}


int ensure_pinned(l2pd_ctx* c) {
  if (c->pinned) return L2PD_OK;
  // two slots of control words for the polling loop; one view of the whole control block (per-sequence
  // blocks and done flags) starts at slot 0 for the schedules that need it
  const size_t words = std::max<size_t>(2 * CTL_WORDS, CTL_WORDS + 2 * (size_t)c->max_batch);
  HIP_TRY(c, hipHostMalloc(reinterpret_cast<void**>(&c->pinned), words * sizeof(int), hipHostMallocDefault));
  HIP_TRY(c, hipEventCreateWithFlags(&c->poll_ev[0], hipEventDisableTiming));
  HIP_TRY(c, hipEventCreateWithFlags(&c->poll_ev[1], hipEventDisableTiming));
  return L2PD_OK;
}

// Step-granular EoTP: lengths in force for the next step, from the tokens as they are.  Waits for
// the stream.  Returns the longest (what the forward has to cover), or -1 on a HIP error;
// *all_done reports the decode state.
int sync_seq_len(l2pd_ctx* c, const int32_t* X, const int32_t* state, int B, int P, const l2pd_decode_cfg* cfg,
                 int* all_done, hipStream_t s) {
  const Layout& L = c->L;
  int* ctl = c->at<int>(L.ctl);
  launch_prepare(state, B, cfg->gen_len / cfg->block_len, cfg->ragged, ctl, s);
  launch_seq_len(X, B, P, cfg->gen_len, c->m.eos_id, c->at<int>(L.teff), ctl, s);
  if (hipMemcpyAsync(c->pinned, ctl, CTL_WORDS * sizeof(int), hipMemcpyDeviceToHost, s) != hipSuccess ||
      hipStreamSynchronize(s) != hipSuccess)
    return -1;
  *all_done = c->pinned[CTL_ALL_DONE];
  return c->pinned[CTL_TMAX];
}
// ---- filter training for callers that cannot allocate ----
// The optimiser moments (first and second, one float each per parameter) live in a file-scope device
// array instead of a caller buffer.  Every GPU holds its own copy at its own address: the address is
// resolved once per device, with that device current, and only that pointer is ever handed to kernels
// (the array's name in host code is a host-side stand-in, not a device address).
constexpr int kStaticTrainParams = 20480;                 // the training kernel's own limit
static __device__ __align__(256) float scratch[2 * kStaticTrainParams];   // 160 KB per GPU, held until the process ends
constexpr int kMaxDevices = 64;
float* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mu;

// Device address of `scratch` on the current device, or nullptr (status in *st).
float* static_scratch(int32_t* st) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { *st = L2PD_EHIP; return nullptr; }
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { *st = L2PD_EHIP; return nullptr; }
    g_scratch_ptr[dev] = static_cast<float*>(p);
  }
  *st = L2PD_OK;
  return g_scratch_ptr[dev];
}
}  // namespace

// =================================================================================================
extern "C" {

int32_t l2pd_generate_stats(const l2pd_ctx* c, int64_t* steps_out, int64_t* sequence_steps_out) {
  if (!c) return L2PD_EINVAL;
  if (steps_out) *steps_out = c->stat_steps;
  if (sequence_steps_out) *sequence_steps_out = c->stat_seq_steps;
  return L2PD_OK;
}

const char* l2pd_strerror(int32_t st) {
  switch (st) {
    case L2PD_OK: return "ok";
    case L2PD_EINVAL: return "invalid argument";
    case L2PD_ENOMEM: return "workspace (or the library's static scratch) too small";
    case L2PD_EHIP: return "HIP runtime error";
    case L2PD_ENOTIMPL: return "shape not supported by the kernels";
    default: return "unknown status";
  }
}

size_t l2pd_workspace_bytes(const l2pd_model_desc* desc, int32_t max_batch, int32_t max_seq,
                            int32_t use_kv_cache) {
  if (!desc_ok(desc) || desc_supported(desc) != L2PD_OK || max_batch < 1 || max_seq < 2) return 0;
  return make_layout(*desc, max_batch, max_seq, use_kv_cache).total;
}

int32_t l2pd_create(const l2pd_model_desc* desc, const l2pd_weights* w, int32_t max_batch, int32_t max_seq,
                    int32_t use_kv_cache, void* workspace_dev, size_t workspace_bytes, l2pd_ctx** out) {
  if (!out) return L2PD_EINVAL;
  *out = nullptr;
  if (!desc_ok(desc) || !w || !workspace_dev || max_batch < 1 || max_seq < 2) return L2PD_EINVAL;
  int sup = desc_supported(desc);
  if (sup != L2PD_OK) return sup;
  if (!w->tok_emb_dev || !w->lm_head_dev || !w->final_norm_g_dev || !w->attn_norm_g || !w->wq || !w->wk || !w->wv ||
      !w->wo || !w->ffn_norm_g || !w->w_gate || !w->w_up || !w->w_down)
    return L2PD_EINVAL;
  for (int l = 0; l < desc->n_layers; ++l)
    if (!w->attn_norm_g[l] || !w->wq[l] || !w->wk[l] || !w->wv[l] || !w->wo[l] || !w->ffn_norm_g[l] ||
        !w->w_gate[l] || !w->w_up[l] || !w->w_down[l])
      return L2PD_EINVAL;
  if ((uintptr_t)workspace_dev % 256) return L2PD_EINVAL;
  Layout L = make_layout(*desc, max_batch, max_seq, use_kv_cache);
  if (workspace_bytes < L.total) return L2PD_ENOMEM;
  l2pd_ctx* c = new (std::nothrow) l2pd_ctx();
  if (!c) return L2PD_ENOMEM;
  c->m = *desc;
  c->tok_emb = w->tok_emb_dev; c->lm_head = w->lm_head_dev; c->final_g = w->final_norm_g_dev;
  const int n = desc->n_layers;
  c->attn_g.assign(w->attn_norm_g, w->attn_norm_g + n);
  c->wq.assign(w->wq, w->wq + n); c->wk.assign(w->wk, w->wk + n); c->wv.assign(w->wv, w->wv + n);
  c->wo.assign(w->wo, w->wo + n); c->ffn_g.assign(w->ffn_norm_g, w->ffn_norm_g + n);
  c->wg.assign(w->w_gate, w->w_gate + n); c->wu.assign(w->w_up, w->w_up + n);
  c->wd.assign(w->w_down, w->w_down + n);
  c->max_batch = max_batch; c->max_seq = max_seq; c->cache = use_kv_cache ? 1 : 0;
  c->ws = static_cast<unsigned char*>(workspace_dev);
  c->ws_bytes = workspace_bytes;
  c->L = L;
  *out = c;
  return L2PD_OK;
}

void l2pd_destroy(l2pd_ctx* c) {
  if (!c) return;
  for (auto& e : c->prof) { (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b); }
  for (auto& e : c->prof_pool) { (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b); }
  if (c->pinned) (void)hipHostFree(c->pinned);
  for (auto& e : c->poll_ev) if (e) (void)hipEventDestroy(e);
  delete c;
}

int32_t l2pd_forward(l2pd_ctx* c, const int32_t* tokens_dev, int32_t B, int32_t T, int32_t row_begin,
                     int32_t row_count, float* logits_out_dev, void* stream) {
  if (!c || !tokens_dev || !logits_out_dev) return L2PD_EINVAL;
  if (B < 1 || B > c->max_batch || T < 1 || T > c->max_seq) return L2PD_EINVAL;
  if (row_begin < 0 || row_count < 1 || (long long)row_begin + row_count > T) return L2PD_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int st = ensure_device(c, s);
  if (st) return st;
  Gate g = {nullptr, -1};
  Pass p = {B, T, 0, T, T, tokens_dev, false, false};
  run_layers(c, p, g, s);
  // the LM head runs in slabs of rows so that the fp32 path's scratch bound (256 rows per sequence) holds
  for (int r0 = 0; r0 < row_count; r0 += 256) {
    int rc = row_count - r0 < 256 ? row_count - r0 : 256;
    if (B == 1 || row_count <= 256) {
      run_head(c, B, rc, RowMap{rc, T, row_begin + r0, 0},
               logits_out_dev + (size_t)r0 * c->m.vocab, false, BiasArgs{0, 0, 1, 0.f}, g, s);
    } else {
      for (int b = 0; b < B; ++b)
        run_head(c, 1, rc, RowMap{rc, T, b * T + row_begin + r0, 0},
                 logits_out_dev + ((size_t)b * row_count + r0) * c->m.vocab, false, BiasArgs{0, 0, 1, 0.f}, g, s);
    }
  }
  HIP_TRY(c, hipGetLastError());
  return L2PD_OK;
}

int32_t l2pd_denoise_step(l2pd_ctx* c, int32_t* tokens_dev, int32_t B, int32_t prompt_len,
                          const l2pd_decode_cfg* cfg, const l2pd_filter* f, int32_t* state_dev, float* logits_dev,
                          float* conf_dev, int32_t* pred_dev, float* filt_dev, uint8_t* unmask_dev, void* stream) {
  int st = check_decode_args(c, B, prompt_len, cfg, f);
  if (st) return st;
  if (!tokens_dev || !state_dev) return L2PD_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  st = ensure_device(c, s);
  if (st) return st;
  int host_gb = -1;
  if (cfg->kv_cache) {
    std::vector<int32_t> hs((size_t)B * 3);
    HIP_TRY(c, hipMemcpyAsync(hs.data(), state_dev, hs.size() * 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(c, hipStreamSynchronize(s));
    const int nb = cfg->gen_len / cfg->block_len;
    host_gb = nb;
    for (int b = 0; b < B; ++b) {
      if (hs[b * 3] < 0) return L2PD_EINVAL;
      if (!hs[b * 3 + 2] && hs[b * 3] < host_gb) host_gb = hs[b * 3];
    }
    if (host_gb >= nb) return L2PD_OK;   // every sequence is done: nothing to do
    if (cfg->ragged) {
      // every live sequence's slice of the stores is rebuilt for its own block
      for (int b = 0; b < B && !cfg->keep_kv; ++b)
        if (!hs[b * 3 + 2] && hs[b * 3] < nb)
          run_refresh_seq(c, tokens_dev, b, prompt_len, cfg, hs[b * 3], Gate{nullptr, -1}, s);
    } else if (!cfg->keep_kv) {
      run_refresh(c, tokens_dev, B, prompt_len, cfg, host_gb, Gate{nullptr, -1}, s);
    }
  }
  StepTaps taps = {logits_dev, conf_dev, pred_dev, filt_dev, unmask_dev};
  int t_run = 0;
  if (cfg->eotp == L2PD_EOTP_STEP) {
    st = ensure_pinned(c);
    if (st) return st;
    int all_done = 0;
    t_run = sync_seq_len(c, tokens_dev, state_dev, B, prompt_len, cfg, &all_done, s);
    if (t_run < 0) { c->last_hip_error = (int)hipGetLastError(); return L2PD_EHIP; }
    if (all_done) return L2PD_OK;
  }
  run_step(c, tokens_dev, B, prompt_len, cfg, f, state_dev, host_gb, taps, s, t_run);
  HIP_TRY(c, hipGetLastError());
  return L2PD_OK;
}

int32_t l2pd_generate(l2pd_ctx* c, const int32_t* prompt_dev, int32_t B, int32_t P, const l2pd_decode_cfg* cfg,
                      const l2pd_filter* f, int32_t* tokens_out_dev, int32_t* steps_out_dev,
                      int32_t* decoded_len_out_dev, void* stream) {
  int st = check_decode_args(c, B, P, cfg, f);
  if (st) return st;
  if (!prompt_dev || !tokens_out_dev) return L2PD_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  st = ensure_device(c, s);
  if (st) return st;
  st = ensure_pinned(c);
  if (st) return st;
  const Layout& L = c->L;
  int32_t* X = c->at<int32_t>(L.X);
  int32_t* state = c->at<int32_t>(L.state);
  int* ctl = c->at<int>(L.ctl);
  const int sl = cfg->block_len, G = cfg->gen_len, nb = G / sl;
  launch_init_decode(X, prompt_dev, B, P, G, c->m.mask_id, state, ctl, s);
  c->stat_steps = c->stat_seq_steps = 0;
  const StepTaps no_taps = {nullptr, nullptr, nullptr, nullptr, nullptr};
  // Steps enqueued between two looks at the control block.  The host always looks at the chunk
  // before the one it has just enqueued, so a finished block (or decode) is noticed one to two chunks
  // late and the steps enqueued meanwhile run as gated launches (a few hundred launches of a
  // microsecond or two each per step).  The cached modes pay that at the end of every block, so
  // they look after every step; full recompute pays it once per decode.
  const int CHUNK = cfg->kv_cache ? 1 : 4;

  // Enqueue `CHUNK` steps, then a copy of the control block to pinned memory; look at the copy of
  // the chunk before, so the device always has a chunk queued while the host waits.
  // Batch compaction (cfg->ragged == L2PD_RAGGED_COMPACT): when the control block shows fewer live
  // sequences than rows in flight, they are moved to the leading rows and the following steps run
  // over those rows only.  The count read is the state of a chunk ago; sequences only ever finish,
  // so the leading `count` rows of a later compaction hold every sequence still live.
  int Bc = B;
  int32_t *X_alt = c->at<int32_t>(L.X2), *state_alt = c->at<int32_t>(L.state2);
  int32_t *perm = nullptr, *perm_alt = c->at<int32_t>(L.perm);
  const bool compacting = cfg->ragged == L2PD_RAGGED_COMPACT && B > 1;
  auto run_until = [&](int host_gb, int max_steps) -> int {   // returns 1 when everything is done
    int issued = 0, slot = 0;
    bool have_prev = false;
    while (issued < max_steps) {
      for (int i = 0; i < CHUNK && issued < max_steps; ++i, ++issued) {
        run_step(c, X, Bc, P, cfg, f, state, host_gb, no_taps, s);
        ++c->stat_steps;
        c->stat_seq_steps += Bc;
      }
      launch_prepare(state, Bc, nb, cfg->ragged, ctl, s);
      if (hipMemcpyAsync(c->pinned + slot * CTL_WORDS, ctl, CTL_WORDS * sizeof(int), hipMemcpyDeviceToHost, s) !=
              hipSuccess ||
          hipEventRecord(c->poll_ev[slot], s) != hipSuccess)
        return -1;
      if (have_prev) {
        int prev = slot ^ 1;
        if (hipEventSynchronize(c->poll_ev[prev]) != hipSuccess) return -1;
        const int* pc = c->pinned + prev * CTL_WORDS;
        if (pc[CTL_ALL_DONE]) return 1;
        if (host_gb >= 0 && pc[CTL_GB] != host_gb) return 0;
        if (compacting && pc[CTL_ACTIVE] > 0 && pc[CTL_ACTIVE] < Bc) {
          launch_compact(X, X_alt, state, state_alt, perm, perm_alt, B, P + G, s);
          std::swap(X, X_alt);
          std::swap(state, state_alt);
          if (!perm) perm = c->at<int32_t>(L.perm2);   // first compaction: identity in, L.perm out
          std::swap(perm, perm_alt);
          Bc = pc[CTL_ACTIVE];
        }
      }
      have_prev = true;
      slot ^= 1;
    }
    // all steps this block (or decode) can need are enqueued: read the final state
    int last = slot ^ 1;
    if (hipEventSynchronize(c->poll_ev[last]) != hipSuccess) return -1;
    return c->pinned[last * CTL_WORDS + CTL_ALL_DONE] ? 1 : 0;
  };

  const bool step_eotp = cfg->eotp == L2PD_EOTP_STEP;
  if (step_eotp) {
    // The sequence length changes from step to step and sizes every launch, so the host looks at
    // the state after every step (a few microseconds against a forward of milliseconds).
    for (int k = 0; k < G; ++k) {   // at most gen_len steps
      int all_done = 0;
      const int t_run = sync_seq_len(c, X, state, B, P, cfg, &all_done, s);
      if (t_run < 0) { c->last_hip_error = (int)hipGetLastError(); return L2PD_EHIP; }
      if (all_done) break;
      run_step(c, X, B, P, cfg, f, state, -1, no_taps, s, t_run);
      ++c->stat_steps;
      c->stat_seq_steps += B;
    }
    launch_seq_len(X, B, P, G, c->m.eos_id, c->at<int>(L.teff), ctl, s);
  } else if (cfg->kv_cache && cfg->ragged) {
    // Per-sequence block pointers with a cache: the host looks at the whole control block before every
    // step (a sequence that has moved on to a new block needs its slice of the stores rebuilt first, a
    // forward over that sequence alone), then enqueues one step for the batch.  Every live sequence
    // commits at least one position per step, so gen_len iterations suffice.
    // With L2PD_RAGGED_COMPACT the sequences still decoding are also moved to the leading rows whenever some
    // have finished (tokens and state by k_compact, as without a cache); their slices of the K/V stores move
    // with them, slot by slot in ascending order (a live sequence only ever moves to a lower slot, and the
    // slot it moves to has been vacated or belongs to a finished sequence), so later steps run over the
    // leading rows only and no kernel needs a row -> slot indirection.
    std::vector<int> host_gb((size_t)B, -1);
    const int done_at = CTL_SEQ_GB + c->max_batch, words = CTL_WORDS + 2 * c->max_batch;
    const size_t es = c->m.dtype == L2PD_FP32 ? 4 : 2;
    const size_t slice = (size_t)L.Tpad * c->m.d_model * es;   // one sequence's K (or V^T) of one layer
    for (int k = 0; k <= G; ++k) {
      launch_prepare(state, Bc, nb, 1, ctl, s, done_at);
      HIP_TRY(c, hipMemcpyAsync(c->pinned, ctl, (size_t)words * sizeof(int), hipMemcpyDeviceToHost, s));
      HIP_TRY(c, hipStreamSynchronize(s));
      if (c->pinned[CTL_ALL_DONE]) break;
      int n_live = 0;
      for (int b = 0; b < Bc; ++b) n_live += c->pinned[done_at + b] ? 0 : 1;
      if (compacting && n_live > 0 && n_live < Bc) {
        launch_compact(X, X_alt, state, state_alt, perm, perm_alt, B, P + G, s);
        std::swap(X, X_alt);
        std::swap(state, state_alt);
        if (!perm) perm = c->at<int32_t>(L.perm2);
        std::swap(perm, perm_alt);
        int to = 0;
        for (int from = 0; from < Bc; ++from) {
          if (c->pinned[done_at + from]) continue;
          if (from != to) {
            for (int l = 0; l < c->m.n_layers; ++l) {
              unsigned char* kl = c->ws + L.kstore + L.kv_layer_stride_k * l;
              unsigned char* vl = c->ws + L.vstore + L.kv_layer_stride_v * l;
              HIP_TRY(c, hipMemcpyAsync(kl + to * slice, kl + from * slice, slice, hipMemcpyDeviceToDevice, s));
              HIP_TRY(c, hipMemcpyAsync(vl + to * slice, vl + from * slice, slice, hipMemcpyDeviceToDevice, s));
            }
            host_gb[to] = host_gb[from];
          }
          // the control words of the new order, for the host's own use below
          c->pinned[CTL_SEQ_GB + to] = c->pinned[CTL_SEQ_GB + from];
          c->pinned[done_at + to] = 0;
          ++to;
        }
        Bc = n_live;
        launch_prepare(state, Bc, nb, 1, ctl, s, done_at);   // the device's control block in the new order
      }
      for (int b = 0; b < Bc; ++b) {
        const int gb = c->pinned[CTL_SEQ_GB + b];
        if (c->pinned[done_at + b] || gb == host_gb[b]) continue;
        run_refresh_seq(c, X, b, P, cfg, gb, Gate{nullptr, -1}, s);
        host_gb[b] = gb;
      }
      run_step(c, X, Bc, P, cfg, f, state, -1, no_taps, s);
      ++c->stat_steps;
      c->stat_seq_steps += Bc;
    }
  } else if (cfg->kv_cache) {
    for (int gb = 0; gb < nb; ++gb) {
      launch_prepare(state, B, nb, cfg->ragged, ctl, s);
      run_refresh(c, X, B, P, cfg, gb, Gate{ctl, -1}, s);
      int r = run_until(gb, sl);   // a block needs at most block_len steps
      if (r < 0) { c->last_hip_error = (int)hipGetLastError(); return L2PD_EHIP; }
      if (r == 1) break;
    }
  } else {
    int r = run_until(-1, G);      // at most gen_len steps in total
    if (r < 0) { c->last_hip_error = (int)hipGetLastError(); return L2PD_EHIP; }
  }
  launch_finalize(X, state, step_eotp ? c->at<int>(L.teff) : nullptr, perm, B, P, G, sl, c->m.mask_id,
                  tokens_out_dev, steps_out_dev, decoded_len_out_dev, s);
  HIP_TRY(c, hipGetLastError());
  return L2PD_OK;
}

int32_t l2pd_egp_rollout(l2pd_ctx* c, const int32_t* prompt_dev, const int32_t* reference_dev, int32_t B, int32_t P,
                         const l2pd_decode_cfg* cfg, float* conf_rows_dev, float* label_rows_dev,
                         int32_t* steps_out_dev, void* stream) {
  if (!c || !cfg || !prompt_dev || !reference_dev || !conf_rows_dev || !label_rows_dev) return L2PD_EINVAL;
  if (B < 1 || B > c->max_batch || P < 1) return L2PD_EINVAL;
  if (cfg->gen_len < 1 || cfg->block_len < 1 || cfg->block_len > 256 || cfg->gen_len % cfg->block_len) return L2PD_EINVAL;
  if ((long long)P + cfg->gen_len > c->max_seq) return L2PD_EINVAL;
  if (cfg->kv_cache != L2PD_CACHE_NONE || cfg->eotp != L2PD_EOTP_OFF) return L2PD_ENOTIMPL;
  if (isnan(cfg->bias.value) ||
      (cfg->bias.value != 0.f && (cfg->bias.token_id < 0 || cfg->bias.token_id >= c->m.vocab)))
    return L2PD_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int st = ensure_device(c, s);
  if (st) return st;
  st = ensure_pinned(c);
  if (st) return st;
  const Layout& L = c->L;
  int32_t* X = c->at<int32_t>(L.X);
  int32_t* state = c->at<int32_t>(L.state);
  int* ctl = c->at<int>(L.ctl);
  const int sl = cfg->block_len, G = cfg->gen_len, nb = G / sl;
  launch_init_decode(X, prompt_dev, B, P, G, c->m.mask_id, state, ctl, s);
  c->stat_steps = c->stat_seq_steps = 0;
  const StepTaps no_taps = {nullptr, nullptr, nullptr, nullptr, nullptr};
  const EgpArgs egp = {reference_dev, conf_rows_dev, label_rows_dev};
  // every step commits at least one position per unfinished sequence: at most gen_len steps;
  // the control block is looked at every few steps, as in l2pd_generate
  for (int k = 0; k < G;) {
    for (int i = 0; i < 4 && k < G; ++i, ++k) run_step(c, X, B, P, cfg, nullptr, state, -1, no_taps, s, 0, &egp);
    launch_prepare(state, B, nb, cfg->ragged, ctl, s);
    HIP_TRY(c, hipMemcpyAsync(c->pinned, ctl, CTL_WORDS * sizeof(int), hipMemcpyDeviceToHost, s));
    HIP_TRY(c, hipStreamSynchronize(s));
    if (c->pinned[CTL_ALL_DONE]) break;
  }
  launch_finalize(X, state, nullptr, nullptr, B, P, G, sl, c->m.mask_id, nullptr, steps_out_dev, nullptr, s);
  HIP_TRY(c, hipGetLastError());
  return L2PD_OK;
}

int32_t l2pd_filter_train(const l2pd_filter* f, const float* conf_rows_dev, const float* label_rows_dev,
                          int64_t n_rows, const l2pd_train_cfg* tc, float* opt_state_dev, float* loss_out_dev,
                          void* stream) {
  if (!f || !tc || !conf_rows_dev || !label_rows_dev || !opt_state_dev) return L2PD_EINVAL;
  if (!filter_ok(f)) return L2PD_EINVAL;
  if (n_rows < 1 || n_rows > (1ll << 24) || tc->epochs < 1 || tc->epochs > 1000000) return L2PD_EINVAL;
  if (!(tc->lr > 0.f) || !(tc->beta1 >= 0.f && tc->beta1 < 1.f) || !(tc->beta2 >= 0.f && tc->beta2 < 1.f) ||
      !(tc->eps > 0.f) || !(tc->weight_decay >= 0.f))
    return L2PD_EINVAL;
  if (!filter_train_supported(f->in_dim, f->hidden, f->n_layers)) return L2PD_ENOTIMPL;
  TrainArgs a = {};
  for (int k = 0; k < f->n_layers; ++k) {
    a.w[k] = const_cast<float*>(f->w_dev[k]);
    a.b[k] = const_cast<float*>(f->b_dev[k]);
  }
  a.n_layers = f->n_layers; a.s = f->in_dim; a.hidden = f->n_layers > 1 ? f->hidden : 1;
  a.conf = conf_rows_dev; a.label = label_rows_dev; a.n = n_rows; a.epochs = tc->epochs;
  a.lr = tc->lr; a.beta1 = tc->beta1; a.beta2 = tc->beta2; a.eps = tc->eps; a.weight_decay = tc->weight_decay;
  a.opt_state = opt_state_dev; a.loss_out = loss_out_dev;
  launch_filter_train(a, static_cast<hipStream_t>(stream));
  return hipGetLastError() == hipSuccess ? L2PD_OK : L2PD_EHIP;
}

int32_t l2pd_filter_train_static(const l2pd_filter* f, const float* conf_rows_dev, const float* label_rows_dev,
                                 int64_t n_rows, const l2pd_train_cfg* tc, float* loss_out_dev, void* stream) {
  if (!f || !filter_ok(f)) return L2PD_EINVAL;
  // beyond the static array: refused here, whatever the training kernel itself could take
  long long n_params = 0;
  for (int k = 0; k < f->n_layers; ++k) {
    const long long in = k == 0 ? f->in_dim : f->hidden, out = k == f->n_layers - 1 ? f->in_dim : f->hidden;
    n_params += out * in + out;
  }
  if (n_params > kStaticTrainParams) return L2PD_ENOMEM;
  int32_t st = L2PD_OK;
  float* moments = static_scratch(&st);
  if (!moments) return st;
  // the kernel zeroes the moments before its first epoch, so what an earlier call left is never read
  return l2pd_filter_train(f, conf_rows_dev, label_rows_dev, n_rows, tc, moments, loss_out_dev, stream);
}

int32_t l2pd_profile_select(l2pd_ctx* c, int32_t cls) {
  if (!c || cls < 0 || cls > L2PD_K_UPDATE) return L2PD_EINVAL;
  for (auto& e : c->prof) c->prof_pool.push_back(e);
  c->prof.clear();
  c->prof_class = cls;
  return L2PD_OK;
}

int32_t l2pd_profile_read(l2pd_ctx* c, int64_t* launches_out, double* total_ms_out) {
  if (!c || !launches_out || !total_ms_out) return L2PD_EINVAL;
  double total = 0.0;
  for (auto& e : c->prof) {
    HIP_TRY(c, hipEventSynchronize(e.b));
    float ms = 0.f;
    HIP_TRY(c, hipEventElapsedTime(&ms, e.a, e.b));
    total += ms;
  }
  *launches_out = (int64_t)c->prof.size();
  *total_ms_out = total > 0.0 ? total : 0.0;
  return L2PD_OK;
}

}  // extern "C"

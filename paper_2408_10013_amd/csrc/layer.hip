// ssdt_layer_fwd / ssdt_layer_bwd: one transformer layer (attention block, optional
// cross-attention block, MLP block; paper Sec. 2.1) as a sequence of kernel launches, with
// every tensor the backward needs allocated from the context's arena and passed through the
// pack hook in the order autograd would register it (Sec. 3.2), and fetched back through the
// unpack hook in backward (Algorithm 1).
#include <cmath>
#include <mutex>

#include "ctx.h"
#include "kernels.h"

using namespace ssdt;

namespace {

struct Dims {
  int B, S, Se, H, A, d, F, T, Te, dt;
  size_t e;
  bool pre, ln, dec, gelu, bias;
  float scale;
};

ssdt_status check_desc(const ssdt_layer_desc *d, Dims *o, std::string *why) {
  if (!d) { *why = "null description"; return SSDT_E_INVAL; }
  if (d->arch < 0 || d->arch > SSDT_ARCH_T5_DEC || (d->dtype != SSDT_F32 && d->dtype != SSDT_BF16) ||
      (d->act != SSDT_ACT_GELU && d->act != SSDT_ACT_RELU) || (d->norm != SSDT_NORM_LAYERNORM && d->norm != SSDT_NORM_RMSNORM) ||
      d->mask < 0 || d->mask > SSDT_MASK_KEYPAD) { *why = "unknown enum value in the layer description"; return SSDT_E_INVAL; }
  if (d->B <= 0 || d->S <= 0 || d->H <= 0 || d->A <= 0 || d->F <= 0 || d->H % d->A != 0) { *why = "non-positive extent or H not a multiple of A"; return SSDT_E_INVAL; }
  if (d->arch == SSDT_ARCH_T5_DEC && d->S_kv <= 0) { *why = "T5 decoder layer needs S_kv > 0"; return SSDT_E_INVAL; }
  if (d->H / d->A > 128) { *why = "head size above 128 is not supported"; return SSDT_E_UNSUPPORTED; }
  if (!(d->eps > 0.f)) { *why = "eps must be positive"; return SSDT_E_INVAL; }
  if ((long)d->B * d->S > (1l << 30) || (long)d->B * d->S * (long)d->F > (1l << 40)) { *why = "shape too large"; return SSDT_E_UNSUPPORTED; }
  o->B = d->B; o->S = d->S; o->Se = d->arch == SSDT_ARCH_T5_DEC ? d->S_kv : 0;
  o->H = d->H; o->A = d->A; o->d = d->H / d->A; o->F = d->F;
  o->T = d->B * d->S; o->Te = d->B * o->Se; o->dt = d->dtype; o->e = d->dtype == SSDT_F32 ? 4 : 2;
  o->pre = d->arch != SSDT_ARCH_BERT_POSTLN; o->ln = d->norm == SSDT_NORM_LAYERNORM; o->dec = d->arch == SSDT_ARCH_T5_DEC;
  o->gelu = d->act == SSDT_ACT_GELU; o->bias = d->has_bias != 0;
  o->scale = d->softmax_scale > 0.f ? d->softmax_scale : 1.f / sqrtf((float)o->d);
  return SSDT_OK;
}

// bump allocator over the caller's workspace; with a null base it only measures
struct Ws {
  char *base;
  size_t cap, used = 0;
  bool ok = true;
  Ws(void *b, size_t c) : base((char *)b), cap(c) {}
  void *take(size_t bytes) {
    size_t off = up(used, 256);
    used = off + bytes;
    if (!base) return (void *)(uintptr_t)256;  // measuring
    if (used > cap) { ok = false; return nullptr; }
    return base + off;
  }
};

size_t max3(size_t a, size_t b, size_t c) { return std::max(a, std::max(b, c)); }

size_t fwd_scratch(const Dims &D) {
  size_t s = 0;
  auto g = [&](int M, int N, int K) { s = std::max(s, k::gemm_scratch_bytes(M, N, K, false, false, D.dt)); };
  g(D.T, 3 * D.H, D.H); g(D.T, D.H, D.H); g(D.T, D.F, D.H); g(D.T, D.H, D.F);
  if (D.dec) g(D.Te, 2 * D.H, D.H);
  return s;
}
size_t bwd_scratch(const Dims &D) {
  size_t s = 0;
  auto g = [&](int M, int N, int K, bool ta, bool tb) { s = std::max(s, k::gemm_scratch_bytes(M, N, K, ta, tb, D.dt)); };
  g(D.F, D.H, D.T, true, false); g(D.H, D.F, D.T, true, false); g(D.H, 3 * D.H, D.T, true, false); g(D.H, D.H, D.T, true, false);
  g(D.T, D.F, D.H, false, true); g(D.T, D.H, D.F, false, true); g(D.T, D.H, 3 * D.H, false, true);
  if (D.dec) { g(D.H, 2 * D.H, D.Te, true, false); g(D.Te, D.H, 2 * D.H, false, true); }
  return s;
}

struct BwdBufs {
  void *dh1, *t0, *t1, *t2, *dqkv, *dkvx, *denc, *scratch;
  float *partial, *partial_side, *delta;
  size_t scratch_bytes;
};
void bwd_layout(const Dims &D, Ws &w, BwdBufs *b) {
  size_t TH = (size_t)D.T * D.H * D.e;
  b->dh1 = w.take((size_t)D.T * D.F * D.e);
  b->t0 = w.take(TH); b->t1 = w.take(TH); b->t2 = w.take(TH);
  b->dqkv = w.take(3 * TH);
  b->dkvx = D.dec ? w.take((size_t)D.Te * 2 * D.H * D.e) : nullptr;
  b->denc = D.dec ? w.take((size_t)D.Te * D.H * D.e) : nullptr;
  size_t rows = std::max(D.T, D.Te), cols = max3(3 * (size_t)D.H, D.F, 0);
  b->partial = (float *)w.take(k::colreduce_partial_floats((int)rows, (int)cols) * 4);
  b->partial_side = (float *)w.take(k::colreduce_partial_floats((int)rows, (int)cols) * 4);
  b->delta = (float *)w.take((size_t)2 * D.B * D.A * D.S * 4);  // delta, and lse in base-2 units behind it
  b->scratch_bytes = bwd_scratch(D);
  b->scratch = b->scratch_bytes ? w.take(b->scratch_bytes) : nullptr;
}

#define HIPCHK(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) return ctx->fail(SSDT_E_HIP, "%s: %s", #expr, hipGetErrorString(e_)); } while (0)
#define STCHK(expr) do { ssdt_status s_ = (expr); if (s_ != SSDT_OK) return s_; } while (0)

}  // namespace

extern "C" {

ssdt_status ssdt_layer_workspace(const ssdt_layer_desc *desc, size_t *fwd_bytes, size_t *bwd_bytes) {
  Dims D;
  std::string why;
  ssdt_status s = check_desc(desc, &D, &why);
  if (s != SSDT_OK) return s;
  if (fwd_bytes) *fwd_bytes = up(fwd_scratch(D), 256) + 256;
  if (bwd_bytes) {
    Ws w(nullptr, 0);
    BwdBufs b;
    bwd_layout(D, w, &b);
    *bwd_bytes = up(w.used, 256) + 256;
  }
  return SSDT_OK;
}

ssdt_status ssdt_layer_bwd_temporaries(const ssdt_layer_desc *desc, ssdt_bwd_temporaries *out) {
  Dims D;
  std::string why;
  ssdt_status s = check_desc(desc, &D, &why);
  if (s != SSDT_OK) return s;
  if (!out) return SSDT_E_INVAL;
  char *base = (char *)(uintptr_t)4096;  // any 256-byte aligned non-null address: only differences are reported
  Ws w(base, ~(size_t)0 >> 1);
  BwdBufs b;
  bwd_layout(D, w, &b);
  auto off = [&](void *p) { return p ? (uint64_t)((char *)p - base) : 0; };
  out->d_h1 = off(b.dh1); out->t0 = off(b.t0); out->t1 = off(b.t1); out->t2 = off(b.t2);
  out->d_qkv = off(b.dqkv); out->d_kvx = off(b.dkvx);
  return SSDT_OK;
}

ssdt_status ssdt_layer_fwd(ssdt_ctx *ctx, const ssdt_layer_desc *desc, const ssdt_layer_weights *w, int32_t scope,
                           const void *x, const void *enc_out, const int32_t *kv_len, void **y_out,
                           ssdt_layer_saved *saved, void *ws, size_t ws_bytes, ssdt_stream stream) {
  if (!ctx) return SSDT_E_INVAL;
  ApiLock api_lock_(ctx);
  Dims D;
  std::string why;
  ssdt_status s = check_desc(desc, &D, &why);
  if (s != SSDT_OK) return ctx->fail(s, "layer_fwd: %s", why.c_str());
  if (ctx->be->is_sim()) return ctx->fail(SSDT_E_UNSUPPORTED, "layer_fwd: the simulated backend has no GPU");
  if (!w || !x || !y_out || !saved) return ctx->fail(SSDT_E_INVAL, "layer_fwd: null argument");
  if (D.dec && !enc_out) return ctx->fail(SSDT_E_INVAL, "layer_fwd: T5 decoder layer needs enc_out");
  if (desc->mask == SSDT_MASK_KEYPAD && !kv_len) return ctx->fail(SSDT_E_INVAL, "layer_fwd: key-padding mask needs kv_len");
  if (!w->ln1_g || !w->w_qkv || !w->w_o || !w->ln2_g || !w->w_1 || !w->w_2 || (D.dec && (!w->lnx_g || !w->w_qx || !w->w_kvx || !w->w_ox)))
    return ctx->fail(SSDT_E_INVAL, "layer_fwd: a required weight pointer is null");
  size_t need = fwd_scratch(D);
  if (need && (!ws || ws_bytes < need)) return ctx->fail(SSDT_E_NOMEM, "layer_fwd: workspace of %zu bytes needed, %zu given", need, ws_bytes);
  if (((uintptr_t)ws % 256) != 0) return ctx->fail(SSDT_E_INVAL, "layer_fwd: workspace must be 256-byte aligned");
  hipStream_t st = (hipStream_t)stream;
  const int dt = D.dt;
  const size_t e = D.e, TH = (size_t)D.T * D.H * e;
  memset(saved, 0, sizeof *saved);
  saved->scope = scope;
  STCHK(ctx->scope_begin(scope, SSDT_FWD));

  std::vector<void *> mine;  // arena blocks this call still holds a reference on
  auto cleanup = [&]() { for (void *p : mine) ctx->unref(p, nullptr, nullptr); mine.clear(); };
  auto alloc = [&](int idx, size_t bytes, void **p) -> ssdt_status {
    ssdt_status r = ctx->alloc(bytes, stream, p);
    if (r != SSDT_OK) return r;
    mine.push_back(*p);
    if (idx >= 0) { saved->e[idx].ptr = *p; saved->e[idx].bytes = bytes; }
    return SSDT_OK;
  };
  // the pack hook on a whole storage / on a [rows, cols] view at a byte offset into it
  const bool ckpt = desc->checkpoint != 0;  // only the layer's inputs are kept for backward
  auto save = [&](int idx, const void *base, size_t sbytes, size_t off, int64_t rows, int64_t cols, int sdt) -> ssdt_status {
    if (ckpt && base != x && base != enc_out) return SSDT_OK;
    int64_t shp[2] = {rows, cols};
    ssdt_tid tid = 0;
    ssdt_status r = ctx->save(base, sbytes, off, shp, 2, sdt, &tid);
    if (r != SSDT_OK) return r;
    if (!saved->e[idx].ptr) { saved->e[idx].ptr = const_cast<void *>(base); saved->e[idx].bytes = sbytes; }
    if (tid) saved->e[idx].tid = tid;
    return SSDT_OK;
  };
#define FAIL_IF(expr) do { ssdt_status r_ = (expr); if (r_ != SSDT_OK) { cleanup(); ctx->stack.clear(); return r_; } } while (0)
#define HIP_IF(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) { cleanup(); ctx->stack.clear(); return ctx->fail(SSDT_E_HIP, "layer_fwd: %s: %s", #expr, hipGetErrorString(e_)); } } while (0)

  auto norm = [&](const void *in, const void *g, const void *b, void *out, float *mean, float *rstd) {
    return k::norm_fwd(in, g, b, out, D.ln ? mean : nullptr, rstd, D.T, D.H, desc->eps, desc->norm, dt, st);
  };
  auto linear = [&](const void *in, int M, int K, const void *W, const void *bias, int N, void *out, int epi,
                    const void *resid, void *out2) {
    k::Gemm g;
    g.M = M; g.N = N; g.K = K; g.A = in; g.lda = K; g.B = W; g.ldb = N; g.transB = false; g.C = out; g.ldc = N;
    g.epi = epi; g.bias = bias; g.resid = resid; g.ldr = N; g.C2 = out2; g.act = desc->act; g.dtype = dt;
    g.scratch = ws; g.scratch_bytes = ws_bytes;
    return k::gemm(g, st);
  };
  auto attention = [&](const void *q, long ldq, const void *kk, const void *v, long ldkv, int Sq, int Sk, int mask,
                       void *o, float *lse) {
    k::Attn a;
    a.B = D.B; a.A = D.A; a.Sq = Sq; a.Sk = Sk; a.d = D.d; a.scale = D.scale; a.mask = mask; a.kv_len = kv_len; a.dtype = dt;
    a.q = q; a.k = kk; a.v = v; a.ldq = ldq; a.ldk = ldkv; a.ldv = ldkv; a.o = o; a.ldo = D.H; a.lse = lse;
    return k::attn_fwd(a, st);
  };
  auto save_stats = [&](int im, int ir) -> ssdt_status {
    if (D.ln) { ssdt_status r = save(im, saved->e[im].ptr, (size_t)D.T * 4, 0, D.T, 1, SSDT_F32); if (r != SSDT_OK) return r; }
    return save(ir, saved->e[ir].ptr, (size_t)D.T * 4, 0, D.T, 1, SSDT_F32);
  };
  auto alloc_stats = [&](int im, int ir, float **mean, float **rstd) -> ssdt_status {
    *mean = nullptr;
    if (D.ln) { ssdt_status r = alloc(im, (size_t)D.T * 4, (void **)mean); if (r != SSDT_OK) return r; }
    return alloc(ir, (size_t)D.T * 4, (void **)rstd);
  };

  const size_t lse_bytes = (size_t)D.B * D.A * D.S * 4;
  void *a = nullptr, *qkv, *o, *lse, *r1 = nullptr, *x1;
  float *mean, *rstd;
  const void *attn_in = x;
  saved->e[SSDT_SV_X].ptr = const_cast<void *>(x);
  saved->e[SSDT_SV_X].bytes = TH;

  // ---- self-attention block -----------------------------------------------------------------
  if (D.pre) {
    FAIL_IF(alloc(SSDT_SV_A, TH, &a));
    FAIL_IF(alloc_stats(SSDT_SV_MEAN1, SSDT_SV_RSTD1, &mean, &rstd));
    HIP_IF(norm(x, w->ln1_g, w->ln1_b, a, mean, rstd));
    FAIL_IF(save(SSDT_SV_X, x, TH, 0, D.T, D.H, dt));
    FAIL_IF(save_stats(SSDT_SV_MEAN1, SSDT_SV_RSTD1));
    attn_in = a;
  }
  FAIL_IF(alloc(SSDT_SV_QKV, 3 * TH, &qkv));
  HIP_IF(linear(attn_in, D.T, D.H, w->w_qkv, w->b_qkv, 3 * D.H, qkv, k::EPI_BIAS, nullptr, nullptr));
  FAIL_IF(save(D.pre ? SSDT_SV_A : SSDT_SV_X, attn_in, TH, 0, D.T, D.H, dt));
  FAIL_IF(alloc(SSDT_SV_O, TH, &o));
  FAIL_IF(alloc(SSDT_SV_LSE, lse_bytes, &lse));
  HIP_IF(attention(qkv, 3 * D.H, (char *)qkv + D.H * e, (char *)qkv + 2 * D.H * e, 3 * D.H, D.S, D.S, desc->mask, o, (float *)lse));
  for (int t = 0; t < 3; ++t) FAIL_IF(save(SSDT_SV_QKV, qkv, 3 * TH, t * D.H * e, D.T, D.H, dt));
  FAIL_IF(save(SSDT_SV_O, o, TH, 0, D.T, D.H, dt));
  FAIL_IF(save(SSDT_SV_LSE, lse, lse_bytes, 0, (int64_t)D.B * D.A, D.S, SSDT_F32));
  if (D.pre) {
    FAIL_IF(alloc(SSDT_SV_X1, TH, &x1));
    HIP_IF(linear(o, D.T, D.H, w->w_o, w->b_o, D.H, x1, k::EPI_BIAS_RESID, x, nullptr));
    FAIL_IF(save(SSDT_SV_O, o, TH, 0, D.T, D.H, dt));
  } else {
    FAIL_IF(alloc(SSDT_SV_R1, TH, &r1));
    HIP_IF(linear(o, D.T, D.H, w->w_o, w->b_o, D.H, r1, k::EPI_BIAS_RESID, x, nullptr));
    FAIL_IF(save(SSDT_SV_O, o, TH, 0, D.T, D.H, dt));
    FAIL_IF(alloc(SSDT_SV_X1, TH, &x1));
    FAIL_IF(alloc_stats(SSDT_SV_MEAN1, SSDT_SV_RSTD1, &mean, &rstd));
    HIP_IF(norm(r1, w->ln1_g, w->ln1_b, x1, mean, rstd));
    FAIL_IF(save(SSDT_SV_R1, r1, TH, 0, D.T, D.H, dt));
    FAIL_IF(save_stats(SSDT_SV_MEAN1, SSDT_SV_RSTD1));
  }

  // ---- cross-attention block (T5 decoder) -----------------------------------------------------
  void *cur = x1;
  int cur_idx = SSDT_SV_X1;
  if (D.dec) {
    void *ax, *qx, *kvx, *ox, *lsex, *x2;
    const size_t TeH = (size_t)D.Te * D.H * e;
    FAIL_IF(alloc(SSDT_SV_AX, TH, &ax));
    FAIL_IF(alloc_stats(SSDT_SV_MEANX, SSDT_SV_RSTDX, &mean, &rstd));
    HIP_IF(norm(x1, w->lnx_g, w->lnx_b, ax, mean, rstd));
    FAIL_IF(save(SSDT_SV_X1, x1, TH, 0, D.T, D.H, dt));
    FAIL_IF(save_stats(SSDT_SV_MEANX, SSDT_SV_RSTDX));
    FAIL_IF(alloc(SSDT_SV_QX, TH, &qx));
    HIP_IF(linear(ax, D.T, D.H, w->w_qx, w->b_qx, D.H, qx, k::EPI_BIAS, nullptr, nullptr));
    FAIL_IF(save(SSDT_SV_AX, ax, TH, 0, D.T, D.H, dt));
    FAIL_IF(alloc(SSDT_SV_KVX, 2 * TeH, &kvx));
    HIP_IF(linear(enc_out, D.Te, D.H, w->w_kvx, w->b_kvx, 2 * D.H, kvx, k::EPI_BIAS, nullptr, nullptr));
    FAIL_IF(save(SSDT_SV_ENC, enc_out, TeH, 0, D.Te, D.H, dt));
    FAIL_IF(alloc(SSDT_SV_OX, TH, &ox));
    FAIL_IF(alloc(SSDT_SV_LSEX, lse_bytes, &lsex));
    HIP_IF(attention(qx, D.H, kvx, (char *)kvx + D.H * e, 2 * D.H, D.S, D.Se, SSDT_MASK_NONE, ox, (float *)lsex));
    FAIL_IF(save(SSDT_SV_QX, qx, TH, 0, D.T, D.H, dt));
    for (int t = 0; t < 2; ++t) FAIL_IF(save(SSDT_SV_KVX, kvx, 2 * TeH, t * D.H * e, D.Te, D.H, dt));
    FAIL_IF(save(SSDT_SV_OX, ox, TH, 0, D.T, D.H, dt));
    FAIL_IF(save(SSDT_SV_LSEX, lsex, lse_bytes, 0, (int64_t)D.B * D.A, D.S, SSDT_F32));
    FAIL_IF(alloc(SSDT_SV_X2, TH, &x2));
    HIP_IF(linear(ox, D.T, D.H, w->w_ox, w->b_ox, D.H, x2, k::EPI_BIAS_RESID, x1, nullptr));
    FAIL_IF(save(SSDT_SV_OX, ox, TH, 0, D.T, D.H, dt));
    cur = x2;
    cur_idx = SSDT_SV_X2;
  }

  // ---- MLP block --------------------------------------------------------------------------------
  const size_t TF = (size_t)D.T * D.F * e;
  void *m = cur, *h1 = nullptr, *g, *y;
  if (D.pre) {
    FAIL_IF(alloc(SSDT_SV_M, TH, &m));
    FAIL_IF(alloc_stats(SSDT_SV_MEAN2, SSDT_SV_RSTD2, &mean, &rstd));
    HIP_IF(norm(cur, w->ln2_g, w->ln2_b, m, mean, rstd));
    FAIL_IF(save(cur_idx, cur, TH, 0, D.T, D.H, dt));
    FAIL_IF(save_stats(SSDT_SV_MEAN2, SSDT_SV_RSTD2));
  }
  if (D.gelu) FAIL_IF(alloc(SSDT_SV_H1, TF, &h1));
  FAIL_IF(alloc(SSDT_SV_G, TF, &g));
  HIP_IF(linear(m, D.T, D.H, w->w_1, w->b_1, D.F, h1, k::EPI_BIAS_ACT, nullptr, g));
  FAIL_IF(save(D.pre ? SSDT_SV_M : SSDT_SV_X1, m, TH, 0, D.T, D.H, dt));
  if (D.gelu) FAIL_IF(save(SSDT_SV_H1, h1, TF, 0, D.T, D.F, dt));
  else FAIL_IF(save(SSDT_SV_G, g, TF, 0, D.T, D.F, dt));
  if (D.pre) {
    FAIL_IF(alloc(-1, TH, &y));
    HIP_IF(linear(g, D.T, D.F, w->w_2, w->b_2, D.H, y, k::EPI_BIAS_RESID, cur, nullptr));
    FAIL_IF(save(SSDT_SV_G, g, TF, 0, D.T, D.F, dt));
  } else {
    void *r2;
    FAIL_IF(alloc(SSDT_SV_R2, TH, &r2));
    HIP_IF(linear(g, D.T, D.F, w->w_2, w->b_2, D.H, r2, k::EPI_BIAS_RESID, cur, nullptr));
    FAIL_IF(save(SSDT_SV_G, g, TF, 0, D.T, D.F, dt));
    FAIL_IF(alloc(-1, TH, &y));
    FAIL_IF(alloc_stats(SSDT_SV_MEAN2, SSDT_SV_RSTD2, &mean, &rstd));
    HIP_IF(norm(r2, w->ln2_g, w->ln2_b, y, mean, rstd));
    FAIL_IF(save(SSDT_SV_R2, r2, TH, 0, D.T, D.H, dt));
    FAIL_IF(save_stats(SSDT_SV_MEAN2, SSDT_SV_RSTD2));
  }
  // every block allocated here is now referenced by the registry; drop this call's references,
  // except y, which the caller owns
  if (ckpt) {
    // nothing but the inputs was registered: the intermediates return to the arena once the kernels
    // enqueued above have run, and the caller gets no pointers to them
    Ev *done = hold(ctx->be->record(stream, false));
    for (void *p : mine)
      if (p != y) ctx->unref(p, done, stream);
    drop(ctx->be.get(), done);
    for (int i = 0; i < SSDT_SV_COUNT; ++i)
      if (saved->e[i].ptr != x && saved->e[i].ptr != enc_out) saved->e[i] = ssdt_saved_entry{};
  } else {
    for (void *p : mine)
      if (p != y) ctx->unref(p, nullptr, nullptr);
  }
  mine.clear();
  *y_out = y;
  return ctx->scope_end(scope, SSDT_FWD);
#undef FAIL_IF
#undef HIP_IF
}

}  // extern "C"

namespace {

ssdt_status layer_bwd_impl(ssdt_ctx *ctx, const ssdt_layer_desc *desc, const ssdt_layer_weights *w,
                           const ssdt_layer_saved *saved, const int32_t *kv_len, const void *dy, void *dx,
                           void *d_enc_out, const ssdt_layer_weights *gr, void *ws, size_t ws_bytes,
                           ssdt_stream stream) {
  if (!ctx) return SSDT_E_INVAL;
  Dims D;
  std::string why;
  ssdt_status s = check_desc(desc, &D, &why);
  if (s != SSDT_OK) return ctx->fail(s, "layer_bwd: %s", why.c_str());
  if (ctx->be->is_sim()) return ctx->fail(SSDT_E_UNSUPPORTED, "layer_bwd: the simulated backend has no GPU");
  if (!w || !saved || !dy || !dx || !gr || !ws) return ctx->fail(SSDT_E_INVAL, "layer_bwd: null argument");
  if (dy == dx) return ctx->fail(SSDT_E_INVAL, "layer_bwd: dx may not alias dy");
  if (D.dec && !d_enc_out) return ctx->fail(SSDT_E_INVAL, "layer_bwd: T5 decoder layer needs d_enc_out");
  if (desc->mask == SSDT_MASK_KEYPAD && !kv_len) return ctx->fail(SSDT_E_INVAL, "layer_bwd: key-padding mask needs kv_len");
  if (((uintptr_t)ws % 256) != 0) return ctx->fail(SSDT_E_INVAL, "layer_bwd: workspace must be 256-byte aligned");
  if (!gr->ln1_g || !gr->w_qkv || !gr->w_o || !gr->ln2_g || !gr->w_1 || !gr->w_2 || (D.ln && (!gr->ln1_b || !gr->ln2_b)) ||
      (D.bias && (!gr->b_qkv || !gr->b_o || !gr->b_1 || !gr->b_2)) ||
      (D.dec && (!gr->lnx_g || !gr->w_qx || !gr->w_kvx || !gr->w_ox)))
    return ctx->fail(SSDT_E_INVAL, "layer_bwd: a required gradient pointer is null");
  Ws wsa(ws, ws_bytes);
  BwdBufs bf;
  bwd_layout(D, wsa, &bf);
  if (!wsa.ok) return ctx->fail(SSDT_E_NOMEM, "layer_bwd: workspace of %zu bytes needed, %zu given", wsa.used, ws_bytes);
  hipStream_t st = (hipStream_t)stream;
  const int dt = D.dt;
  const int scope = saved->scope;
  STCHK(ctx->scope_begin(scope, SSDT_BWD));

  // the unpack hook: a stamped tensor comes from the registry (the stream waits for its load),
  // a bypassed one is still where forward left it
  auto getp = [&](int idx, const void **p) -> ssdt_status {
    const ssdt_saved_entry &en = saved->e[idx];
    if (en.tid) { void *q = nullptr; ssdt_status r = ctx->get(en.tid, stream, &q); *p = q; return r; }
    if (!en.ptr) return ctx->fail(SSDT_E_INVAL, "layer_bwd: saved tensor %d is missing", idx);
    *p = en.ptr;
    return SSDT_OK;
  };
#define GET(idx, var) const void *var = nullptr; do { ssdt_status r_ = getp(idx, &var); if (r_ != SSDT_OK) { ctx->bwd_open.clear(); return r_; } } while (0)
#define HIP_IF(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) { ctx->bwd_open.clear(); return ctx->fail(SSDT_E_HIP, "layer_bwd: %s: %s", #expr, hipGetErrorString(e_)); } } while (0)

  auto mm = [&](int M, int N, int K, const void *A, long lda, bool tA, const void *B, long ldb, bool tB, void *C, int epi,
                const void *resid, const void *aux) {
    k::Gemm g;
    g.M = M; g.N = N; g.K = K; g.A = A; g.lda = lda; g.transA = tA; g.B = B; g.ldb = ldb; g.transB = tB; g.C = C; g.ldc = N;
    g.epi = epi; g.resid = resid; g.ldr = N; g.aux = aux; g.act = desc->act; g.dtype = dt;
    g.scratch = bf.scratch; g.scratch_bytes = bf.scratch_bytes;
    return k::gemm(g, st);
  };
  // gradients of y = in W + b given dY: dW = in^T dY, db = column sums of dY
  // (with gradient accumulation the product is added to what dW holds: the residual epilogue reading dW itself)
  const bool accum = desc->accumulate != 0;
  // The weight-gradient GEMM wants both operands with the token dimension contiguous, i.e. transposed copies.
  // Those copies and the bias-gradient column sums are bandwidth-bound and independent of the input-gradient GEMM
  // that follows, so for the matrix-core path they run on the context's side stream underneath that GEMM:
  // wgrad() enqueues them there (after an event that says dY is ready) and remembers the GEMM; wgrad_flush(),
  // called after the input-gradient GEMM has been enqueued, makes the caller's stream wait for the copies and
  // enqueues the weight-gradient GEMM.  The side stream's next round starts only after an event recorded behind that
  // GEMM on the caller's stream (a later dY depends on it in stream order anyway), so one scratch area suffices.
  hipStream_t side = (hipStream_t)ctx->be->aux_stream();
  struct Pending { bool on = false; int Kin, Nout, rows; long ld; void *dW; const uint16_t *At, *Bt; Ev *ready; } pend;
  auto wgrad_flush = [&]() -> hipError_t {
    if (!pend.on) return hipSuccess;
    pend.on = false;
    ctx->be->wait(stream, pend.ready);
    drop(ctx->be.get(), pend.ready);
    k::Gemm g;
    g.M = pend.Kin; g.N = pend.Nout; g.K = pend.rows; g.A = pend.At; g.lda = pend.ld; g.transA = false; g.B = pend.Bt;
    g.ldb = pend.ld; g.transB = true; g.C = pend.dW; g.ldc = pend.Nout; g.epi = accum ? k::EPI_BIAS_RESID : k::EPI_NONE;
    g.resid = accum ? pend.dW : nullptr; g.ldr = pend.Nout; g.act = desc->act; g.dtype = dt;
    return k::gemm(g, st);
  };
  auto wgrad = [&](const void *in, int Kin, const void *dY, int Nout, int rows, void *dW, void *db) -> hipError_t {
    if (k::gemm_km_fits(Kin, Nout, rows, true, false, dt)) {
      // Both operands are read as stored (tokens x features, the contraction running over tokens): no copies, and
      // the bias gradient (the column sums of dY) falls out of the same kernel.
      k::Gemm g;
      g.M = Kin; g.N = Nout; g.K = rows; g.A = in; g.lda = Kin; g.transA = true; g.B = dY; g.ldb = Nout; g.transB = false;
      g.C = dW; g.ldc = Nout; g.epi = accum ? k::EPI_BIAS_RESID : k::EPI_NONE; g.resid = accum ? dW : nullptr; g.ldr = Nout;
      g.act = desc->act; g.dtype = dt; g.colsum = db; g.colsum_accumulate = accum;
      hipError_t e0 = k::gemm_mfma_km_bf16(g, st);
      if (e0 != hipErrorNotSupported) return e0;  // (an alignment it does not take: the general path below)
    }
    const long ld = k::nt_copy_ld(rows);  // leading dimension of the two transposed copies
    const size_t a_bytes = ((size_t)Kin * ld * 2 + 255) / 256 * 256, b_bytes = (size_t)Nout * ld * 2;
    const bool overlap = side && dt == SSDT_BF16 && Kin % 128 == 0 && Nout % 128 == 0 && rows % 64 == 0 &&
                         a_bytes + b_bytes <= bf.scratch_bytes;
    if (!overlap) {
      hipError_t e1 = mm(Kin, Nout, rows, in, Kin, true, dY, Nout, false, dW, accum ? k::EPI_BIAS_RESID : k::EPI_NONE,
                         accum ? dW : nullptr, nullptr);
      if (e1 != hipSuccess) return e1;
      if (db) return k::colsum(dY, Nout, db, bf.partial, rows, Nout, dt, accum, st);
      return hipSuccess;
    }
    hipError_t e0 = wgrad_flush();  // at most one round is in flight
    if (e0 != hipSuccess) return e0;
    Ev *go = hold(ctx->be->record(stream, false));  // dY (and everything before it) is ready
    ctx->be->wait(side, go);
    drop(ctx->be.get(), go);
    uint16_t *At = (uint16_t *)bf.scratch, *Bt = (uint16_t *)((char *)bf.scratch + a_bytes);
    hipError_t e1 = k::transpose(in, Kin, At, ld, rows, Kin, SSDT_BF16, side);     // [rows, Kin] -> [Kin, rows]
    // [rows, Nout] -> [Nout, rows], with the bias gradient taken from the same pass over dY where the kernel fits
    hipError_t e2 = e1 != hipSuccess ? e1 : db ? k::transpose_colsum(dY, Nout, Bt, ld, rows, Nout, db, bf.partial_side, accum, side)
                                               : hipErrorNotSupported;
    if (e2 == hipErrorNotSupported) {
      e1 = k::transpose(dY, Nout, Bt, ld, rows, Nout, SSDT_BF16, side);
      if (e1 == hipSuccess && db) e1 = k::colsum(dY, Nout, db, bf.partial_side, rows, Nout, dt, accum, side);
    } else {
      e1 = e2;
    }
    if (e1 != hipSuccess) return e1;
    pend.on = true; pend.Kin = Kin; pend.Nout = Nout; pend.rows = rows; pend.ld = ld; pend.dW = dW; pend.At = At; pend.Bt = Bt;
    pend.ready = hold(ctx->be->record(side, false));
    return hipSuccess;
  };
  auto nbwd = [&](const void *dout, const void *xin, const void *mean, const void *rstd, const void *gamma,
                  const void *resid, void *dxo, void *dgam, void *dbet) {
    return k::norm_bwd(dout, xin, (const float *)mean, (const float *)rstd, gamma, resid, dxo, dgam, D.ln ? dbet : nullptr,
                       bf.partial, D.T, D.H, desc->norm, dt, accum, st);
  };
  auto attn_b = [&](const void *q, long ldq, const void *kk, const void *v, long ldkv, int Sq, int Sk, int mask,
                    const void *o, const void *lse, const void *dO, void *dq, long lddq, void *dk, void *dv, long lddkv) {
    k::Attn a;
    a.B = D.B; a.A = D.A; a.Sq = Sq; a.Sk = Sk; a.d = D.d; a.scale = D.scale; a.mask = mask; a.kv_len = kv_len; a.dtype = dt;
    a.q = q; a.k = kk; a.v = v; a.ldq = ldq; a.ldk = ldkv; a.ldv = ldkv; a.o = const_cast<void *>(o); a.ldo = D.H;
    a.lse = (float *)const_cast<void *>(lse); a.dout = dO; a.lddo = D.H; a.dq = dq; a.dk = dk; a.dv = dv;
    a.lddq = lddq; a.lddk = lddkv; a.lddv = lddkv; a.delta = bf.delta;
    return k::attn_bwd(a, st);
  };
  const void *nomean = nullptr;
  const size_t e = D.e;
  const int cur_idx = D.dec ? SSDT_SV_X2 : SSDT_SV_X1;

  // ---- MLP block --------------------------------------------------------------------------------
  // dcur (in t1): gradient w.r.t. the block input, including the residual branch
  const void *dr2 = dy;
  if (!D.pre) {
    GET(SSDT_SV_R2, r2); GET(SSDT_SV_RSTD2, rs2);
    const void *mu2 = nomean; if (D.ln) { GET(SSDT_SV_MEAN2, t); mu2 = t; }
    HIP_IF(nbwd(dy, r2, mu2, rs2, w->ln2_g, nullptr, bf.t0, gr->ln2_g, gr->ln2_b));
    dr2 = bf.t0;
  }
  {
    GET(SSDT_SV_G, g);
    HIP_IF(wgrad(g, D.F, dr2, D.H, D.T, gr->w_2, D.bias ? gr->b_2 : nullptr));
    const void *aux = g;
    if (D.gelu) { GET(SSDT_SV_H1, h1); aux = h1; }
    HIP_IF(mm(D.T, D.F, D.H, dr2, D.H, false, w->w_2, D.H, true, bf.dh1, k::EPI_ACTBWD, nullptr, aux));
    HIP_IF(wgrad_flush());
  }
  if (D.pre) {
    GET(SSDT_SV_M, m);
    HIP_IF(wgrad(m, D.H, bf.dh1, D.F, D.T, gr->w_1, D.bias ? gr->b_1 : nullptr));
    HIP_IF(mm(D.T, D.H, D.F, bf.dh1, D.F, false, w->w_1, D.F, true, bf.t2, k::EPI_NONE, nullptr, nullptr));
    HIP_IF(wgrad_flush());
    GET(cur_idx, cur); GET(SSDT_SV_RSTD2, rs2);
    const void *mu2 = nomean; if (D.ln) { GET(SSDT_SV_MEAN2, t); mu2 = t; }
    HIP_IF(nbwd(bf.t2, cur, mu2, rs2, w->ln2_g, dr2, bf.t1, gr->ln2_g, gr->ln2_b));
  } else {
    GET(SSDT_SV_X1, x1);
    HIP_IF(wgrad(x1, D.H, bf.dh1, D.F, D.T, gr->w_1, D.bias ? gr->b_1 : nullptr));
    HIP_IF(mm(D.T, D.H, D.F, bf.dh1, D.F, false, w->w_1, D.F, true, bf.t1, k::EPI_BIAS_RESID, dr2, nullptr));
    HIP_IF(wgrad_flush());
  }
  void *dcur = bf.t1;  // gradient w.r.t. x2 (decoder) or x1

  // ---- cross-attention block ----------------------------------------------------------------------
  if (D.dec) {
    GET(SSDT_SV_OX, ox);
    HIP_IF(wgrad(ox, D.H, dcur, D.H, D.T, gr->w_ox, D.bias ? gr->b_ox : nullptr));
    HIP_IF(mm(D.T, D.H, D.H, dcur, D.H, false, w->w_ox, D.H, true, bf.t0, k::EPI_NONE, nullptr, nullptr));  // d ox
    HIP_IF(wgrad_flush());
    GET(SSDT_SV_QX, qx); GET(SSDT_SV_KVX, kvx); GET(SSDT_SV_LSEX, lsex);
    HIP_IF(attn_b(qx, D.H, kvx, (const char *)kvx + D.H * e, 2 * D.H, D.S, D.Se, SSDT_MASK_NONE, ox, lsex, bf.t0,
                  bf.t2, D.H, bf.dkvx, (char *)bf.dkvx + D.H * e, 2 * D.H));  // d qx in t2
    GET(SSDT_SV_AX, ax);
    HIP_IF(wgrad(ax, D.H, bf.t2, D.H, D.T, gr->w_qx, D.bias ? gr->b_qx : nullptr));
    HIP_IF(mm(D.T, D.H, D.H, bf.t2, D.H, false, w->w_qx, D.H, true, bf.t0, k::EPI_NONE, nullptr, nullptr));  // d ax
    HIP_IF(wgrad_flush());
    GET(SSDT_SV_ENC, enc);
    HIP_IF(wgrad(enc, D.H, bf.dkvx, 2 * D.H, D.Te, gr->w_kvx, D.bias ? gr->b_kvx : nullptr));
    HIP_IF(mm(D.Te, D.H, 2 * D.H, bf.dkvx, 2 * D.H, false, w->w_kvx, 2 * D.H, true, bf.denc, k::EPI_NONE, nullptr, nullptr));
    HIP_IF(wgrad_flush());
    HIP_IF(k::add_inplace(d_enc_out, bf.denc, (size_t)D.Te * D.H, dt, st));
    GET(SSDT_SV_X1, x1); GET(SSDT_SV_RSTDX, rsx);
    const void *mux = nomean; if (D.ln) { GET(SSDT_SV_MEANX, t); mux = t; }
    HIP_IF(nbwd(bf.t0, x1, mux, rsx, w->lnx_g, dcur, bf.t2, gr->lnx_g, gr->lnx_b));
    dcur = bf.t2;  // gradient w.r.t. x1
  }

  // ---- self-attention block -------------------------------------------------------------------------
  void *tA = (dcur == bf.t1) ? bf.t2 : bf.t1;  // a free [T,H] buffer
  const void *dr1 = dcur;
  if (!D.pre) {
    GET(SSDT_SV_R1, r1); GET(SSDT_SV_RSTD1, rs1);
    const void *mu1 = nomean; if (D.ln) { GET(SSDT_SV_MEAN1, t); mu1 = t; }
    HIP_IF(nbwd(dcur, r1, mu1, rs1, w->ln1_g, nullptr, tA, gr->ln1_g, gr->ln1_b));
    dr1 = tA;
    tA = dcur;
  }
  GET(SSDT_SV_O, o);
  HIP_IF(wgrad(o, D.H, dr1, D.H, D.T, gr->w_o, D.bias ? gr->b_o : nullptr));
  HIP_IF(mm(D.T, D.H, D.H, dr1, D.H, false, w->w_o, D.H, true, bf.t0, k::EPI_NONE, nullptr, nullptr));  // d o
  HIP_IF(wgrad_flush());
  GET(SSDT_SV_QKV, qkv); GET(SSDT_SV_LSE, lse);
  HIP_IF(attn_b(qkv, 3 * D.H, (const char *)qkv + D.H * e, (const char *)qkv + 2 * D.H * e, 3 * D.H, D.S, D.S, desc->mask,
                o, lse, bf.t0, bf.dqkv, 3 * D.H, (char *)bf.dqkv + D.H * e, (char *)bf.dqkv + 2 * D.H * e, 3 * D.H));
  if (D.pre) {
    GET(SSDT_SV_A, a);
    HIP_IF(wgrad(a, D.H, bf.dqkv, 3 * D.H, D.T, gr->w_qkv, D.bias ? gr->b_qkv : nullptr));
    HIP_IF(mm(D.T, D.H, 3 * D.H, bf.dqkv, 3 * D.H, false, w->w_qkv, 3 * D.H, true, tA, k::EPI_NONE, nullptr, nullptr));  // d a
    HIP_IF(wgrad_flush());
    GET(SSDT_SV_X, x); GET(SSDT_SV_RSTD1, rs1);
    const void *mu1 = nomean; if (D.ln) { GET(SSDT_SV_MEAN1, t); mu1 = t; }
    HIP_IF(nbwd(tA, x, mu1, rs1, w->ln1_g, dr1, dx, gr->ln1_g, gr->ln1_b));
  } else {
    GET(SSDT_SV_X, x);
    HIP_IF(wgrad(x, D.H, bf.dqkv, 3 * D.H, D.T, gr->w_qkv, D.bias ? gr->b_qkv : nullptr));
    HIP_IF(mm(D.T, D.H, 3 * D.H, bf.dqkv, 3 * D.H, false, w->w_qkv, 3 * D.H, true, dx, k::EPI_BIAS_RESID, dr1, nullptr));
    HIP_IF(wgrad_flush());
  }
  HIP_IF(wgrad_flush());
  return ctx->scope_end(scope, SSDT_BWD);
#undef GET
#undef HIP_IF
}

// Workspace of ssdt_layer_bwd_static: one array in device memory per GPU the library runs on, there from the moment
// the code object is loaded until the process ends.  In host code its name is only a handle; the device address
// comes from hipGetSymbolAddress, once per device, with that device current.
constexpr size_t kStaticWsBytes = SSDT_STATIC_WS_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticWsBytes];
constexpr int kMaxDevices = 64;
std::mutex g_static_mu;
void *g_static_ptr[kMaxDevices] = {};

hipError_t static_workspace(void **out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lk(g_static_mu);
  if (!g_static_ptr[dev]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p || ((uintptr_t)p & 255)) return hipErrorInvalidSymbol;
    g_static_ptr[dev] = p;
  }
  *out = g_static_ptr[dev];
  return hipSuccess;
}

}  // namespace

extern "C" {

ssdt_status ssdt_layer_bwd(ssdt_ctx *ctx, const ssdt_layer_desc *desc, const ssdt_layer_weights *w,
                           const ssdt_layer_saved *saved, const int32_t *kv_len, const void *dy, void *dx,
                           void *d_enc_out, const ssdt_layer_weights *gr, void *ws, size_t ws_bytes,
                           ssdt_stream stream) {
  ApiLock api_lock_(ctx);
  return layer_bwd_impl(ctx, desc, w, saved, kv_len, dy, dx, d_enc_out, gr, ws, ws_bytes, stream);
}

ssdt_status ssdt_layer_bwd_static(ssdt_ctx *ctx, const ssdt_layer_desc *desc, const ssdt_layer_weights *w,
                                  const ssdt_layer_saved *saved, const int32_t *kv_len, const void *dy, void *dx,
                                  void *d_enc_out, const ssdt_layer_weights *gr, ssdt_stream stream) {
  if (!ctx) return SSDT_E_INVAL;
  ApiLock api_lock_(ctx);
  if (ctx->be->is_sim()) return ctx->fail(SSDT_E_UNSUPPORTED, "layer_bwd_static: the simulated backend has no GPU");
  size_t need = 0;
  ssdt_status s = ssdt_layer_workspace(desc, nullptr, &need);
  if (s != SSDT_OK) return ctx->fail(s, "layer_bwd_static: unusable layer description");
  if (need > kStaticWsBytes)
    return ctx->fail(SSDT_E_NOMEM, "layer_bwd_static: this layer needs %zu bytes of workspace, the built-in one has %zu; "
                                   "use ssdt_layer_bwd with a workspace of your own", need, kStaticWsBytes);
  void *ws = nullptr;
  hipError_t e = static_workspace(&ws);
  if (e != hipSuccess) return ctx->fail(SSDT_E_HIP, "layer_bwd_static: address of the built-in workspace: %s", hipGetErrorString(e));
  return layer_bwd_impl(ctx, desc, w, saved, kv_len, dy, dx, d_enc_out, gr, ws, kStaticWsBytes, stream);
}

ssdt_status ssdt_sgd_update(ssdt_ctx *ctx, void *w, const void *g, size_t numel, int32_t dtype, float lr, ssdt_stream stream) {
  if (!ctx) return SSDT_E_INVAL;
  ApiLock api_lock_(ctx);
  if (ctx->be->is_sim()) return ctx->fail(SSDT_E_UNSUPPORTED, "sgd_update: the simulated backend has no GPU");
  if (!w || !g || (dtype != SSDT_F32 && dtype != SSDT_BF16)) return ctx->fail(SSDT_E_INVAL, "sgd_update: null pointer or unknown dtype");
  hipError_t e = k::sgd_update(w, g, numel, lr, dtype, (hipStream_t)stream);
  if (e != hipSuccess) return ctx->fail(SSDT_E_HIP, "sgd_update: %s", hipGetErrorString(e));
  return SSDT_OK;
}

}  // extern "C"

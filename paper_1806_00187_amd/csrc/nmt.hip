// Context, parameter layout, workspace plan and the orchestration of the training step
// (forward + loss, backward, accumulate, overflow check, Adam) behind the C ABI.
#include <math.h>
#include <stdarg.h>
#include <stdlib.h>

#include <string>
#include <vector>

#include "common.h"

// ---- error text -------------------------------------------------------------------------------
static thread_local char g_err[512] = "";
void nmt_set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}
extern "C" const char* nmt_last_error(void) { return g_err; }

const DeviceInfo& device_info() {
  static const DeviceInfo info = [] {
    DeviceInfo d;
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess) {
      if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) d.cus = v;
      if (hipDeviceGetAttribute(&v, hipDeviceAttributeNumberOfXccs, dev) == hipSuccess && v > 0) d.xcds = v;
    }
    (void)hipGetLastError();
    return d;
  }();
  return info;
}
Tuning& tuning() {
  static Tuning t;
  return t;
}
extern "C" int nmt_tuning(const char* name, int32_t value) {
  NMT_REQUIRE(name, "nmt_tuning: null name");
  Tuning& t = tuning();
  if (!strcmp(name, "gemm_group")) { NMT_REQUIRE(value >= 1, "nmt_tuning: gemm_group must be >= 1"); t.gemm_group = value; }
  else if (!strcmp(name, "gemm_persist")) { NMT_REQUIRE(value == 0 || value == 1, "nmt_tuning: gemm_persist is 0 or 1"); t.gemm_persist = value; }
  else if (!strcmp(name, "attn_persist")) t.attn_persist = value != 0;
  else if (!strcmp(name, "worklists")) t.worklists = value != 0;
  else if (!strcmp(name, "one_stream")) t.one_stream = value != 0;
  else if (!strcmp(name, "gemm_share")) { NMT_REQUIRE(value >= 1 && value <= 16, "nmt_tuning: gemm_share must be in [1, 16]"); t.gemm_share = value; }
  else if (!strcmp(name, "gemm_tile")) { NMT_REQUIRE(value >= 0 && value <= 5, "nmt_tuning: gemm_tile is 0..5"); t.gemm_tile = value; }
  else if (!strcmp(name, "gemm_timing")) t.gemm_timing = value != 0;
  else if (!strcmp(name, "defaults")) t = Tuning{};
  else NMT_REQUIRE(false, "nmt_tuning: unknown switch '%s'", name);
  return NMT_OK;
}

DropDev make_drop(const nmt_dropout* d) {
  DropDev o = {};
  o.scale = 1.f;
  o.n_pos = 1;
  if (!d) return o;
  o.n_pos = d->n_pos;
  o.uid = d->d_sent_uid;
  o.k0 = (uint32_t)(d->seed & 0xFFFFFFFFu);
  o.k1 = (uint32_t)(d->seed >> 32);
  o.c3 = (d->step << 8) | (d->micro & 0xFFu);
  o.site_hi = d->site << 16;
  if (d->p > 0.f) {
    o.thr = (uint32_t)ceil((double)d->p * 65536.0);
    o.scale = 1.f / (1.f - d->p);
  }
  return o;
}

static int check_drop(const nmt_dropout* d, const char* who) {
  if (!d) return NMT_OK;
  NMT_REQUIRE(d->p >= 0.f && d->p < 1.f, "%s: dropout probability %g outside [0, 1)", who, (double)d->p);
  NMT_REQUIRE(d->n_pos > 0 && d->n_pos <= 65535, "%s: positions per sentence %d outside [1, 65535]", who, d->n_pos);
  NMT_REQUIRE(d->site < 65536u && d->step < (1u << 24) && d->micro < 256u, "%s: dropout site/step/micro out of range", who);
  return NMT_OK;
}

// ---- parameter layout -------------------------------------------------------------------------
namespace {

struct Tensor {
  std::string name;
  int64_t off;
  int rows, cols;
};
struct AttnP { int64_t wqkv, bqkv, wq, bq, wkv, bkv, wo, bo; };
struct LnP { int64_t g, b; };
struct FfnP { int64_t w1, b1, w2, b2; };
struct EncP { AttnP attn; LnP ln1; FfnP ffn; LnP ln2; };
struct DecP { AttnP self; LnP ln1; AttnP cross; LnP ln2; FfnP ffn; LnP ln3; };

// dropout sites: a site id selects an independent random stream
constexpr int kMaxSegments = NMT_MAX_SEGMENTS;
constexpr int64_t kWgradPartialFloats = 16ll << 20;
constexpr uint32_t kSiteEmbSrc = 0, kSiteEmbTgt = 1;
constexpr uint32_t kKindSelfRes = 0, kKindCrossRes = 1, kKindFfnAct = 2, kKindFfnRes = 3;
inline uint32_t layer_site(int layer_index, uint32_t kind) { return 16u * (1u + (uint32_t)layer_index) + kind; }

// workspace plan: byte offsets of every activation kept for the backward pass and of the
// backward pass's temporaries
struct EncW { int64_t qkv, o, s1, x1, h, s2, x2, lse, st1, st2; };
struct DecW { int64_t qkv, o1, s1, x1, lse1, q, kv, o2, s2, x2, lse2, h, s3, x3, st1, st2, st3; };
struct Plan {
  int64_t rk_src, rk_tgt, tab_ss, tab_tt, tab_ts;  // row keys (dropout, positions) and per-sentence attention tables
  int64_t wl_ss, wl_tt, wl_ts;                     // attention work lists over those tables
  int64_t sent_rows;                                // first source / target row of every sentence (packed batches)
  int64_t x0, y0, logits, rowloss;
  std::vector<EncW> enc;
  std::vector<DecW> dec;
  int64_t dx_dec, dx_enc, dy[2], dym[2], dO, dqkv[2], dh[2], dq[2], dkv[2], lnpart, cspart, embscratch, wgpart, wgpart_floats;
  int64_t total;
};

}  // namespace

struct nmt_ctx {
  nmt_config cfg;
  std::vector<Tensor> tensors;
  int64_t P = 0;
  int64_t embed = 0;
  std::vector<EncP> enc;
  std::vector<DecP> dec;
  half_t* w16 = nullptr;
  half_t* g16 = nullptr;
  float *master = nullptr, *acc = nullptr, *m = nullptr, *v = nullptr;
  unsigned char* ws = nullptr;
  int64_t ws_bytes = 0;
  // state of the last forward pass
  bool have_fwd = false;
  int Bt = 0, Ns = 0, Nt = 0, maxS = 0, maxT = 0, training = 0;  // sentences, source / target rows, longest sides
  float loss_scale = 1.f;
  float gscale = 1.f;  // power-of-two factor on everything the current pass writes to g16
  float inv_scale = 1.f;  // what nmt_check_overflow was given: nmt_adam_step applies it to acc32 on the fly
  uint32_t step = 0;
  const int32_t *src = nullptr, *tgt_in = nullptr, *tgt_out = nullptr;
  const float* last_loss = nullptr;   // where the last forward call wrote its loss sum and token count
  const int32_t* last_ntok = nullptr;
  Plan plan;
  // second stream for the weight-gradient kernels of the backward pass (created on first use)
  hipStream_t side = nullptr;
  hipEvent_t ev_fork = nullptr, ev_join = nullptr, ev_done[2] = {nullptr, nullptr};
};

namespace {

int64_t add_tensor(nmt_ctx* c, const std::string& name, int rows, int cols) {
  const int64_t off = c->P;
  c->tensors.push_back({name, off, rows, cols});
  c->P += (int64_t)rows * cols;
  return off;
}
void add_attn(nmt_ctx* c, const std::string& pre, bool fused, AttnP& a) {
  const int d = c->cfg.d_model;
  a = {};
  if (fused) {
    a.wqkv = add_tensor(c, pre + "wqkv", 3 * d, d);
    a.bqkv = add_tensor(c, pre + "bqkv", 1, 3 * d);
  } else {
    a.wq = add_tensor(c, pre + "wq", d, d);
    a.bq = add_tensor(c, pre + "bq", 1, d);
    a.wkv = add_tensor(c, pre + "wkv", 2 * d, d);
    a.bkv = add_tensor(c, pre + "bkv", 1, 2 * d);
  }
  a.wo = add_tensor(c, pre + "wo", d, d);
  a.bo = add_tensor(c, pre + "bo", 1, d);
}
void add_ln(nmt_ctx* c, const std::string& pre, LnP& l) {
  l.g = add_tensor(c, pre + "g", 1, c->cfg.d_model);
  l.b = add_tensor(c, pre + "b", 1, c->cfg.d_model);
}
void add_ffn(nmt_ctx* c, const std::string& pre, FfnP& f) {
  const int d = c->cfg.d_model, F = c->cfg.d_ff;
  f.w1 = add_tensor(c, pre + "w1", F, d);
  f.b1 = add_tensor(c, pre + "b1", 1, F);
  f.w2 = add_tensor(c, pre + "w2", d, F);
  f.b2 = add_tensor(c, pre + "b2", 1, d);
}

// Totals of a group of sub-batches stacked row-wise.
struct GroupDims {
  int64_t Bt = 0, Ns = 0, Nt = 0;
  int maxS = 0, maxT = 0;
};

int64_t plan_workspace(const nmt_ctx* c, const GroupDims& gd, Plan& p) {
  const nmt_config& k = c->cfg;
  const int64_t d = k.d_model, F = k.d_ff, V = k.vocab, H = k.n_heads;
  const int64_t B = gd.Bt, Ns = gd.Ns, Nt = gd.Nt, Nm = Ns > Nt ? Ns : Nt;
  int64_t cur = 0;
  auto take = [&](int64_t bytes) {
    const int64_t off = cur;
    cur += round_up(bytes, 256);
    return off;
  };
  const int64_t h2 = sizeof(half_t), f4 = sizeof(float);
  p.rk_src = take(Ns * (int64_t)sizeof(uint2));
  p.rk_tgt = take(Nt * (int64_t)sizeof(uint2));
  p.tab_ss = take(B * (int64_t)sizeof(int4));
  p.tab_tt = take(B * (int64_t)sizeof(int4));
  p.tab_ts = take(B * (int64_t)sizeof(int4));
  p.wl_ss = take(attention_worklist_ints((int)B, (int)Ns) * (int64_t)sizeof(int32_t));
  p.wl_tt = take(attention_worklist_ints((int)B, (int)Nt) * (int64_t)sizeof(int32_t));
  p.wl_ts = take(attention_worklist_ints((int)B, (int)Nt) * (int64_t)sizeof(int32_t));
  p.sent_rows = take(2 * B * (int64_t)sizeof(int32_t));
  p.x0 = take(Ns * d * h2);
  p.y0 = take(Nt * d * h2);
  p.enc.resize(k.enc_layers);
  for (auto& e : p.enc) {
    e.qkv = take(Ns * 3 * d * h2);
    e.o = take(Ns * d * h2);
    e.s1 = take(Ns * d * h2);
    e.x1 = take(Ns * d * h2);
    e.h = take(Ns * F * h2);
    e.s2 = take(Ns * d * h2);
    e.x2 = take(Ns * d * h2);
    e.lse = take(H * Ns * f4);
    e.st1 = take(Ns * 2 * f4);
    e.st2 = take(Ns * 2 * f4);
  }
  p.dec.resize(k.dec_layers);
  for (auto& e : p.dec) {
    e.qkv = take(Nt * 3 * d * h2);
    e.o1 = take(Nt * d * h2);
    e.s1 = take(Nt * d * h2);
    e.x1 = take(Nt * d * h2);
    e.lse1 = take(H * Nt * f4);
    e.q = take(Nt * d * h2);
    e.kv = take(Ns * 2 * d * h2);
    e.o2 = take(Nt * d * h2);
    e.s2 = take(Nt * d * h2);
    e.x2 = take(Nt * d * h2);
    e.lse2 = take(H * Nt * f4);
    e.h = take(Nt * F * h2);
    e.s3 = take(Nt * d * h2);
    e.x3 = take(Nt * d * h2);
    e.st1 = take(Nt * 2 * f4);
    e.st2 = take(Nt * 2 * f4);
    e.st3 = take(Nt * 2 * f4);
  }
  p.logits = take(Nt * V * h2);
  p.rowloss = take(Nt * f4);
  p.dx_dec = take(Nt * d * h2);
  p.dx_enc = take(Ns * d * h2);
  p.dO = take(Nm * d * h2);
  for (int b = 0; b < 2; ++b) {  // two sets: weight-gradient kernels of one sub-layer overlap the next sub-layer
    p.dy[b] = take(Nm * d * h2);
    p.dym[b] = take(Nm * d * h2);
    p.dqkv[b] = take(Nm * 3 * d * h2);
    p.dh[b] = take(Nm * F * h2);
    p.dq[b] = take(Nt * d * h2);
    p.dkv[b] = take(Ns * 2 * d * h2);
  }
  p.lnpart = take(layernorm_bwd_scratch_floats((int)d) * f4);
  const int64_t widest = F > 3 * d ? F : 3 * d;
  p.cspart = take(colsum_scratch_floats((int)widest) * f4);
  p.embscratch = take(embed_bwd_scratch_ints((int)V, (int)(Ns + Nt), (int)d) * (int64_t)sizeof(int32_t));
  // fp32 partial sums of weight-gradient products cut along the (long) position axis
  p.wgpart_floats = kWgradPartialFloats;
  p.wgpart = take(p.wgpart_floats * f4);
  p.total = cur;
  return cur;
}

int check_group(const nmt_ctx* c, int n_seg, const nmt_segment* segs, GroupDims& gd) {
  NMT_REQUIRE(c, "null context");
  NMT_REQUIRE(segs && n_seg >= 1 && n_seg <= kMaxSegments, "number of sub-batches %d outside [1, %d]", n_seg, kMaxSegments);
  gd = GroupDims{};
  for (int i = 0; i < n_seg; ++i) {
    const nmt_segment& s = segs[i];
    NMT_REQUIRE(s.B >= 1 && s.B <= c->cfg.max_sentences, "sub-batch %d: B=%d outside [1, max_sentences=%d]", i, s.B, c->cfg.max_sentences);
    NMT_REQUIRE(s.S >= 1 && s.S <= c->cfg.max_len && s.T >= 1 && s.T <= c->cfg.max_len, "sub-batch %d: S=%d / T=%d outside [1, max_len=%d]", i,
                s.S, s.T, c->cfg.max_len);
    NMT_REQUIRE(s.micro_idx < 256u, "sub-batch %d: micro_idx must be < 256", i);
    gd.Bt += s.B;
    gd.Ns += (int64_t)s.B * s.S;
    gd.Nt += (int64_t)s.B * s.T;
    gd.maxS = s.S > gd.maxS ? s.S : gd.maxS;
    gd.maxT = s.T > gd.maxT ? s.T : gd.maxT;
  }
  NMT_REQUIRE(gd.Ns <= (1 << 20) && gd.Nt <= (1 << 20), "more than 2^20 positions in one pass");
  return NMT_OK;
}

#define NMT_TRY(expr)            \
  do {                           \
    const int rc_ = (expr);      \
    if (rc_ != NMT_OK) return rc_; \
  } while (0)

}  // namespace

// ================================================================================================
// C ABI: context
// ================================================================================================
extern "C" int nmt_create(const nmt_config* cfg, nmt_ctx** out) {
  NMT_REQUIRE(cfg && out, "nmt_create: null argument");
  *out = nullptr;
  NMT_REQUIRE(cfg->enc_layers >= 1 && cfg->dec_layers >= 1 && cfg->enc_layers + cfg->dec_layers < 4000, "nmt_create: bad layer counts");
  NMT_REQUIRE(cfg->d_model >= 16 && cfg->d_model % 8 == 0 && cfg->d_model <= 2048, "nmt_create: d_model=%d must be a multiple of 8 in [16, 2048]", cfg->d_model);
  NMT_REQUIRE(cfg->n_heads >= 1 && cfg->d_model % cfg->n_heads == 0, "nmt_create: d_model %% n_heads != 0");
  const int dh = cfg->d_model / cfg->n_heads;
  NMT_REQUIRE(dh == 16 || dh == 32 || dh == 64 || dh == 128, "nmt_create: head size %d not in {16,32,64,128}", dh);
  NMT_REQUIRE(cfg->d_ff >= 8 && cfg->d_ff % 8 == 0, "nmt_create: d_ff=%d must be a positive multiple of 8", cfg->d_ff);
  NMT_REQUIRE(cfg->vocab >= 8 && cfg->vocab % 8 == 0 && cfg->vocab <= 65536, "nmt_create: vocab=%d must be a multiple of 8 in [8, 65536]", cfg->vocab);
  NMT_REQUIRE(cfg->pad_id >= 0 && cfg->pad_id < cfg->vocab, "nmt_create: pad_id outside the vocabulary");
  NMT_REQUIRE(cfg->dropout >= 0.f && cfg->dropout < 1.f && cfg->act_dropout >= 0.f && cfg->act_dropout < 1.f, "nmt_create: dropout outside [0, 1)");
  NMT_REQUIRE(cfg->attn_dropout == 0.f, "nmt_create: dropout on the attention probabilities is not built (attn_dropout must be 0)");
  NMT_REQUIRE(cfg->label_smoothing >= 0.f && cfg->label_smoothing < 1.f, "nmt_create: label_smoothing outside [0, 1)");
  NMT_REQUIRE(cfg->ln_eps > 0.f, "nmt_create: ln_eps must be positive");
  NMT_REQUIRE(cfg->max_sentences >= 1 && cfg->max_len >= 1 && cfg->max_len <= 1024, "nmt_create: max_sentences >= 1 and 1 <= max_len <= 1024 required");
  NMT_REQUIRE(cfg->max_sentences <= (1 << 20), "nmt_create: max_sentences above 2^20");
  nmt_ctx* c = new (std::nothrow) nmt_ctx();
  NMT_REQUIRE(c, "nmt_create: out of host memory");
  c->cfg = *cfg;
  c->embed = add_tensor(c, "embed", cfg->vocab, cfg->d_model);
  c->enc.resize(cfg->enc_layers);
  c->dec.resize(cfg->dec_layers);
  for (int l = 0; l < cfg->enc_layers; ++l) {
    const std::string pre = "enc" + std::to_string(l) + ".";
    add_attn(c, pre + "attn.", true, c->enc[l].attn);
    add_ln(c, pre + "ln1.", c->enc[l].ln1);
    add_ffn(c, pre + "ffn.", c->enc[l].ffn);
    add_ln(c, pre + "ln2.", c->enc[l].ln2);
  }
  for (int l = 0; l < cfg->dec_layers; ++l) {
    const std::string pre = "dec" + std::to_string(l) + ".";
    add_attn(c, pre + "self.", true, c->dec[l].self);
    add_ln(c, pre + "ln1.", c->dec[l].ln1);
    add_attn(c, pre + "cross.", false, c->dec[l].cross);
    add_ln(c, pre + "ln2.", c->dec[l].ln2);
    add_ffn(c, pre + "ffn.", c->dec[l].ffn);
    add_ln(c, pre + "ln3.", c->dec[l].ln3);
  }
  *out = c;
  return NMT_OK;
}

extern "C" void nmt_destroy(nmt_ctx* ctx) {
  if (!ctx) return;
  if (ctx->side) {
    (void)hipStreamSynchronize(ctx->side);
    (void)hipStreamDestroy(ctx->side);
  }
  if (ctx->ev_fork) {
    (void)hipEventDestroy(ctx->ev_fork);
    (void)hipEventDestroy(ctx->ev_join);
    (void)hipEventDestroy(ctx->ev_done[0]);
    (void)hipEventDestroy(ctx->ev_done[1]);
  }
  delete ctx;
}
extern "C" int64_t nmt_param_count(const nmt_ctx* ctx) { return ctx ? ctx->P : -1; }
extern "C" float nmt_grad_scale(const nmt_ctx* ctx) { return ctx ? ctx->gscale : 0.f; }
extern "C" int32_t nmt_param_tensors(const nmt_ctx* ctx) { return ctx ? (int32_t)ctx->tensors.size() : -1; }

extern "C" int nmt_param_info(const nmt_ctx* ctx, int32_t idx, const char** name, int64_t* offset, int32_t* rows, int32_t* cols) {
  NMT_REQUIRE(ctx, "nmt_param_info: null context");
  NMT_REQUIRE(idx >= 0 && idx < (int32_t)ctx->tensors.size(), "nmt_param_info: index %d out of range", idx);
  const Tensor& t = ctx->tensors[idx];
  if (name) *name = t.name.c_str();
  if (offset) *offset = t.off;
  if (rows) *rows = t.rows;
  if (cols) *cols = t.cols;
  return NMT_OK;
}

extern "C" int64_t nmt_workspace_bytes_group(const nmt_ctx* ctx, int32_t n_seg, const nmt_segment* segs) {
  GroupDims gd;
  if (check_group(ctx, n_seg, segs, gd) != NMT_OK) return NMT_EINVAL;
  Plan p;
  return plan_workspace(ctx, gd, p);
}
extern "C" int64_t nmt_workspace_bytes(const nmt_ctx* ctx, int32_t B, int32_t S, int32_t T) {
  const nmt_segment seg = {B, S, T, 0u};
  return nmt_workspace_bytes_group(ctx, 1, &seg);
}

extern "C" int nmt_bind(nmt_ctx* ctx, void* d_w16, void* d_g16, float* d_master32, float* d_acc32, float* d_adam_m,
                        float* d_adam_v, void* d_workspace, int64_t ws_bytes) {
  NMT_REQUIRE(ctx, "nmt_bind: null context");
  NMT_REQUIRE(d_w16 && d_g16, "nmt_bind: w16 and g16 are required");
  NMT_REQUIRE(aligned16(d_w16) && aligned16(d_g16) && aligned16(d_master32) && aligned16(d_acc32) && aligned16(d_adam_m) && aligned16(d_adam_v),
              "nmt_bind: buffers must be 16-byte aligned");
  NMT_REQUIRE(!d_workspace || (reinterpret_cast<uintptr_t>(d_workspace) & 255u) == 0, "nmt_bind: workspace must be 256-byte aligned");
  NMT_REQUIRE(ws_bytes >= 0, "nmt_bind: negative workspace size");
  ctx->w16 = static_cast<half_t*>(d_w16);
  ctx->g16 = static_cast<half_t*>(d_g16);
  ctx->master = d_master32;
  ctx->acc = d_acc32;
  ctx->m = d_adam_m;
  ctx->v = d_adam_v;
  ctx->ws = static_cast<unsigned char*>(d_workspace);
  ctx->ws_bytes = d_workspace ? ws_bytes : 0;
  ctx->have_fwd = false;
  ctx->last_loss = nullptr;
  ctx->last_ntok = nullptr;
  return NMT_OK;
}

// ================================================================================================
// forward + loss
// ================================================================================================
namespace {

struct Run {
  nmt_ctx* c;
  hipStream_t st;
  template <typename T>
  T* ws(int64_t off) const { return reinterpret_cast<T*>(c->ws + off); }
  half_t* w(int64_t off) const { return c->w16 + off; }
  half_t* g(int64_t off) const { return c->g16 + off; }
  // dropout stream `site` over source (tgt == false) or target rows
  DropDev drop(uint32_t site, bool tgt, float p) const {
    nmt_dropout d = {c->training ? p : 0.f, site, c->step, 0u, c->cfg.seed, 1, nullptr};
    DropDev dd = make_drop(&d);
    dd.rowkey = ws<uint2>(tgt ? c->plan.rk_tgt : c->plan.rk_src);
    return dd;
  }
  // y[N, out] = x[N, in] W^T + b   (W stored [out, in])
  int linear(const half_t* x, int N, int in, int64_t W, int64_t b, int out, half_t* y, GemmEpilogue ep = {}) const {
    ep.bias = c->w16 + b;
    return launch_gemm(x, false, in, c->w16 + W, false, in, y, out, N, out, in, ep, st);
  }
  // dx[N, in] = dy[N, out] W (+ add)
  int dgrad(const half_t* dy, int N, int out, int64_t W, int in, half_t* dx, GemmEpilogue ep = {}) const {
    return launch_gemm(dy, false, out, c->w16 + W, true, in, dx, in, N, in, out, ep, st);
  }
  // gW[out, in] = dy^T x
  int wgrad(const half_t* dy, int N, int out, const half_t* x, int in, int64_t gW) const {
    GemmEpilogue ep;
    ep.out_scale = c->gscale;
    return launch_gemm(dy, true, out, x, true, in, c->g16 + gW, in, out, in, N, ep, st,
                       c->plan.wgpart_floats ? ws<float>(c->plan.wgpart) : nullptr, c->plan.wgpart_floats, 0);
  }
};

}  // namespace

extern "C" int nmt_forward_loss(nmt_ctx* ctx, const int32_t* d_src, const int32_t* d_tgt_in, const int32_t* d_tgt_out,
                                int32_t B, int32_t S, int32_t T, float loss_scale, uint32_t step, uint32_t micro_idx,
                                const uint32_t* d_sent_uid, int32_t training, float* d_loss_sum, int32_t* d_ntok,
                                void* stream) {
  const nmt_segment seg = {B, S, T, micro_idx};
  return nmt_forward_loss_group(ctx, 1, &seg, d_src, d_tgt_in, d_tgt_out, loss_scale, step, d_sent_uid, training, d_loss_sum, d_ntok,
                                stream);
}

namespace {
// How the row keys and sentence tables of a pass are built: from a short list of rectangular
// sub-batches (host), or from a device array of sentences packed back to back.
struct TableSource {
  int n_seg = 0;
  const nmt_segment* segs = nullptr;
  const uint32_t* uid = nullptr;
  const nmt_sentence* sentences = nullptr;
};
int forward_pass(nmt_ctx* c, const GroupDims& gd, const TableSource& src, const int32_t* d_src, const int32_t* d_tgt_in,
                 const int32_t* d_tgt_out, float loss_scale, uint32_t step, int32_t training, float* d_loss_sum, int32_t* d_ntok,
                 void* stream);
}  // namespace

extern "C" int nmt_forward_loss_group(nmt_ctx* ctx, int32_t n_seg, const nmt_segment* segs, const int32_t* d_src,
                                      const int32_t* d_tgt_in, const int32_t* d_tgt_out, float loss_scale, uint32_t step,
                                      const uint32_t* d_sent_uid, int32_t training, float* d_loss_sum, int32_t* d_ntok,
                                      void* stream) {
  GroupDims gd;
  NMT_TRY(check_group(ctx, n_seg, segs, gd));
  TableSource src;
  src.n_seg = n_seg;
  src.segs = segs;
  src.uid = d_sent_uid;
  return forward_pass(ctx, gd, src, d_src, d_tgt_in, d_tgt_out, loss_scale, step, training, d_loss_sum, d_ntok, stream);
}

namespace {
int check_packed(const nmt_ctx* c, int n_sent, const nmt_sentence* d_sent, int64_t n_src, int64_t n_tgt, int max_src, int max_tgt,
                 GroupDims& gd) {
  NMT_REQUIRE(c, "null context");
  NMT_REQUIRE(d_sent && n_sent >= 1 && n_sent <= (1 << 20), "packed batch: %d sentences outside [1, 2^20]", n_sent);
  NMT_REQUIRE(max_src >= 1 && max_src <= c->cfg.max_len && max_tgt >= 1 && max_tgt <= c->cfg.max_len,
              "packed batch: longest source / target %d / %d outside [1, max_len=%d]", max_src, max_tgt, c->cfg.max_len);
  NMT_REQUIRE(n_src >= n_sent && n_src <= (int64_t)n_sent * max_src && n_tgt >= n_sent && n_tgt <= (int64_t)n_sent * max_tgt,
              "packed batch: token totals inconsistent with the sentence count and the longest lengths");
  NMT_REQUIRE(n_src <= (1 << 20) && n_tgt <= (1 << 20), "more than 2^20 positions in one pass");
  gd = GroupDims{};
  gd.Bt = n_sent;
  gd.Ns = n_src;
  gd.Nt = n_tgt;
  gd.maxS = max_src;
  gd.maxT = max_tgt;
  return NMT_OK;
}
}  // namespace

extern "C" int64_t nmt_workspace_bytes_packed(const nmt_ctx* ctx, int32_t n_sent, int64_t n_src_tokens, int64_t n_tgt_tokens) {
  if (!ctx || n_sent < 1 || n_src_tokens < n_sent || n_tgt_tokens < n_sent || n_src_tokens > (1 << 20) || n_tgt_tokens > (1 << 20)) {
    nmt_set_error("nmt_workspace_bytes_packed: bad sizes");
    return NMT_EINVAL;
  }
  GroupDims gd;
  gd.Bt = n_sent;
  gd.Ns = n_src_tokens;
  gd.Nt = n_tgt_tokens;
  Plan p;
  return plan_workspace(ctx, gd, p);
}

extern "C" int nmt_forward_loss_packed(nmt_ctx* ctx, int32_t n_sent, const nmt_sentence* d_sentences, int64_t n_src_tokens,
                                       int64_t n_tgt_tokens, int32_t max_src_len, int32_t max_tgt_len, const int32_t* d_src,
                                       const int32_t* d_tgt_in, const int32_t* d_tgt_out, float loss_scale, uint32_t step,
                                       int32_t training, float* d_loss_sum, int32_t* d_ntok, void* stream) {
  GroupDims gd;
  NMT_TRY(check_packed(ctx, n_sent, d_sentences, n_src_tokens, n_tgt_tokens, max_src_len, max_tgt_len, gd));
  TableSource src;
  src.sentences = d_sentences;
  return forward_pass(ctx, gd, src, d_src, d_tgt_in, d_tgt_out, loss_scale, step, training, d_loss_sum, d_ntok, stream);
}

namespace {
int forward_pass(nmt_ctx* c, const GroupDims& gd, const TableSource& tsrc, const int32_t* d_src, const int32_t* d_tgt_in,
                 const int32_t* d_tgt_out, float loss_scale, uint32_t step, int32_t training, float* d_loss_sum, int32_t* d_ntok,
                 void* stream) {
  c->have_fwd = false;
  NMT_REQUIRE(d_src && d_tgt_in && d_tgt_out && d_loss_sum && d_ntok, "nmt_forward_loss: null pointer");
  NMT_REQUIRE(c->w16 && c->g16, "nmt_forward_loss: nmt_bind has not been called");
  NMT_REQUIRE(loss_scale > 0.f && isfinite(loss_scale), "nmt_forward_loss: loss_scale must be positive and finite");
  NMT_REQUIRE(step < (1u << 24), "nmt_forward_loss: step must be < 2^24");
  if (plan_workspace(c, gd, c->plan) > c->ws_bytes) {
    nmt_set_error("nmt_forward_loss: workspace of %lld bytes is smaller than the %lld needed", (long long)c->ws_bytes, (long long)c->plan.total);
    return NMT_ENOMEM;
  }
  c->Bt = (int)gd.Bt; c->Ns = (int)gd.Ns; c->Nt = (int)gd.Nt; c->maxS = gd.maxS; c->maxT = gd.maxT;
  c->loss_scale = loss_scale; c->step = step; c->training = training != 0;
  // A pass over many sub-batches sums proportionally more token gradients into each weight gradient.
  // Scaling that sum down by a power of two before the one fp16 rounding keeps it in the range a single
  // sub-batch's gradient has, so grouping does not lower the loss scale at which fp16 overflows.
  c->gscale = 1.f;
  for (int64_t n = gd.Nt; n >= 8192; n >>= 1) c->gscale *= 0.5f;
  c->src = d_src; c->tgt_in = d_tgt_in; c->tgt_out = d_tgt_out;
  c->last_loss = d_loss_sum; c->last_ntok = d_ntok;

  const nmt_config& k = c->cfg;
  const int d = k.d_model, F = k.d_ff, V = k.vocab, H = k.n_heads, dh = d / H;
  const int Bt = c->Bt, Ns = c->Ns, Nt = c->Nt, maxS = c->maxS, maxT = c->maxT;
  const Plan& p = c->plan;
  const Run r{c, static_cast<hipStream_t>(stream)};
  hipStream_t st = r.st;
  const int4 *tab_ss = r.ws<int4>(p.tab_ss), *tab_tt = r.ws<int4>(p.tab_tt), *tab_ts = r.ws<int4>(p.tab_ts);
  if (tsrc.sentences) {
    NMT_TRY(launch_build_tables_packed(tsrc.sentences, Bt, Ns, Nt, maxS, maxT, r.ws<int32_t>(p.sent_rows), r.ws<uint2>(p.rk_src),
                                       r.ws<uint2>(p.rk_tgt), r.ws<int4>(p.tab_ss), r.ws<int4>(p.tab_tt), r.ws<int4>(p.tab_ts), st));
  } else {
    SegmentList sl = {};
    sl.n = tsrc.n_seg;
    for (int i = 0; i < tsrc.n_seg; ++i) {
      sl.B[i] = tsrc.segs[i].B; sl.S[i] = tsrc.segs[i].S; sl.T[i] = tsrc.segs[i].T; sl.micro[i] = tsrc.segs[i].micro_idx;
    }
    NMT_TRY(launch_build_tables(sl, Bt, tsrc.uid, r.ws<uint2>(p.rk_src), r.ws<uint2>(p.rk_tgt), r.ws<int4>(p.tab_ss),
                                r.ws<int4>(p.tab_tt), r.ws<int4>(p.tab_ts), st));
  }
  NMT_TRY(launch_attention_worklists(tab_ss, Bt, Ns, r.ws<int32_t>(p.wl_ss), st));
  NMT_TRY(launch_attention_worklists(tab_tt, Bt, Nt, r.ws<int32_t>(p.wl_tt), st));
  NMT_TRY(launch_attention_worklists(tab_ts, Bt, Nt, r.ws<int32_t>(p.wl_ts), st));
  const AttnWork wl_ss = attention_work(r.ws<int32_t>(p.wl_ss), Bt, Ns, 0), wl_tt = attention_work(r.ws<int32_t>(p.wl_tt), Bt, Nt, 0),
                 wl_ts = attention_work(r.ws<int32_t>(p.wl_ts), Bt, Nt, Ns);

  // ---- encoder ----
  half_t* x = r.ws<half_t>(p.x0);
  NMT_TRY(launch_embed_fwd(d_src, r.w(c->embed), x, Ns, d, V, r.drop(kSiteEmbSrc, false, k.dropout), st));
  for (int l = 0; l < k.enc_layers; ++l) {
    const EncP& P = c->enc[l];
    const EncW& W = p.enc[l];
    half_t* qkv = r.ws<half_t>(W.qkv);
    NMT_TRY(r.linear(x, Ns, d, P.attn.wqkv, P.attn.bqkv, 3 * d, qkv));
    NMT_TRY(launch_attention_fwd(qkv, 3 * d, qkv + d, 3 * d, qkv + 2 * d, 3 * d, r.ws<half_t>(W.o), d, r.ws<float>(W.lse), d_src,
                                 k.pad_id, 0, Bt, H, dh, maxS, maxS, tab_ss, Ns, &wl_ss, st));
    NMT_TRY(r.linear(r.ws<half_t>(W.o), Ns, d, P.attn.wo, P.attn.bo, d, r.ws<half_t>(W.s1)));
    NMT_TRY(launch_residual_layernorm_fwd(r.ws<half_t>(W.s1), x, r.w(P.ln1.g), r.w(P.ln1.b), r.ws<half_t>(W.x1), r.ws<float>(W.st1),
                                          Ns, d, k.ln_eps, r.drop(layer_site(l, kKindSelfRes), false, k.dropout), st));
    GemmEpilogue act;
    act.relu = 1;
    act.drop = r.drop(layer_site(l, kKindFfnAct), false, k.act_dropout);
    NMT_TRY(r.linear(r.ws<half_t>(W.x1), Ns, d, P.ffn.w1, P.ffn.b1, F, r.ws<half_t>(W.h), act));
    NMT_TRY(r.linear(r.ws<half_t>(W.h), Ns, F, P.ffn.w2, P.ffn.b2, d, r.ws<half_t>(W.s2)));
    NMT_TRY(launch_residual_layernorm_fwd(r.ws<half_t>(W.s2), r.ws<half_t>(W.x1), r.w(P.ln2.g), r.w(P.ln2.b), r.ws<half_t>(W.x2),
                                          r.ws<float>(W.st2), Ns, d, k.ln_eps, r.drop(layer_site(l, kKindFfnRes), false, k.dropout), st));
    x = r.ws<half_t>(W.x2);
  }
  const half_t* enc_out = x;

  // ---- decoder ----
  half_t* y = r.ws<half_t>(p.y0);
  NMT_TRY(launch_embed_fwd(d_tgt_in, r.w(c->embed), y, Nt, d, V, r.drop(kSiteEmbTgt, true, k.dropout), st));
  for (int l = 0; l < k.dec_layers; ++l) {
    const DecP& P = c->dec[l];
    const DecW& W = p.dec[l];
    const int li = k.enc_layers + l;
    half_t* qkv = r.ws<half_t>(W.qkv);
    NMT_TRY(r.linear(y, Nt, d, P.self.wqkv, P.self.bqkv, 3 * d, qkv));
    NMT_TRY(launch_attention_fwd(qkv, 3 * d, qkv + d, 3 * d, qkv + 2 * d, 3 * d, r.ws<half_t>(W.o1), d, r.ws<float>(W.lse1), d_tgt_in,
                                 k.pad_id, 1, Bt, H, dh, maxT, maxT, tab_tt, Nt, &wl_tt, st));
    NMT_TRY(r.linear(r.ws<half_t>(W.o1), Nt, d, P.self.wo, P.self.bo, d, r.ws<half_t>(W.s1)));
    NMT_TRY(launch_residual_layernorm_fwd(r.ws<half_t>(W.s1), y, r.w(P.ln1.g), r.w(P.ln1.b), r.ws<half_t>(W.x1), r.ws<float>(W.st1),
                                          Nt, d, k.ln_eps, r.drop(layer_site(li, kKindSelfRes), true, k.dropout), st));
    half_t* kv = r.ws<half_t>(W.kv);
    NMT_TRY(r.linear(r.ws<half_t>(W.x1), Nt, d, P.cross.wq, P.cross.bq, d, r.ws<half_t>(W.q)));
    NMT_TRY(r.linear(enc_out, Ns, d, P.cross.wkv, P.cross.bkv, 2 * d, kv));
    NMT_TRY(launch_attention_fwd(r.ws<half_t>(W.q), d, kv, 2 * d, kv + d, 2 * d, r.ws<half_t>(W.o2), d, r.ws<float>(W.lse2), d_src,
                                 k.pad_id, 0, Bt, H, dh, maxT, maxS, tab_ts, Nt, &wl_ts, st));
    NMT_TRY(r.linear(r.ws<half_t>(W.o2), Nt, d, P.cross.wo, P.cross.bo, d, r.ws<half_t>(W.s2)));
    NMT_TRY(launch_residual_layernorm_fwd(r.ws<half_t>(W.s2), r.ws<half_t>(W.x1), r.w(P.ln2.g), r.w(P.ln2.b), r.ws<half_t>(W.x2),
                                          r.ws<float>(W.st2), Nt, d, k.ln_eps, r.drop(layer_site(li, kKindCrossRes), true, k.dropout), st));
    GemmEpilogue act;
    act.relu = 1;
    act.drop = r.drop(layer_site(li, kKindFfnAct), true, k.act_dropout);
    NMT_TRY(r.linear(r.ws<half_t>(W.x2), Nt, d, P.ffn.w1, P.ffn.b1, F, r.ws<half_t>(W.h), act));
    NMT_TRY(r.linear(r.ws<half_t>(W.h), Nt, F, P.ffn.w2, P.ffn.b2, d, r.ws<half_t>(W.s3)));
    NMT_TRY(launch_residual_layernorm_fwd(r.ws<half_t>(W.s3), r.ws<half_t>(W.x2), r.w(P.ln3.g), r.w(P.ln3.b), r.ws<half_t>(W.x3),
                                          r.ws<float>(W.st3), Nt, d, k.ln_eps, r.drop(layer_site(li, kKindFfnRes), true, k.dropout), st));
    y = r.ws<half_t>(W.x3);
  }

  // ---- output projection (tied to the embedding) and loss ----
  half_t* logits = r.ws<half_t>(p.logits);
  NMT_TRY(launch_gemm(y, false, d, r.w(c->embed), false, d, logits, V, Nt, V, d, GemmEpilogue{}, st));
  NMT_TRY(launch_softmax_xent(logits, d_tgt_out, r.ws<float>(p.rowloss), Nt, V, k.pad_id, k.label_smoothing, loss_scale, d_loss_sum,
                              d_ntok, st));
  c->have_fwd = true;
  return NMT_OK;
}
}  // namespace

// ================================================================================================
// backward
// ================================================================================================
// Weight gradients (and the bias column sums) are leaves of the backward graph: nothing downstream
// waits for them.  They are enqueued on a second stream so that they run beside the chain of
// input-gradient kernels and fill the compute units those leave idle.  Temporaries read by the
// second stream exist twice; set s is reused two sub-layers later, after the event recorded
// behind its last reader.
extern "C" int nmt_backward(nmt_ctx* ctx, void* stream) {
  NMT_REQUIRE(ctx, "nmt_backward: null context");
  nmt_ctx* c = ctx;
  if (!c->have_fwd) {
    nmt_set_error("nmt_backward: no forward pass to differentiate");
    return NMT_ESTATE;
  }
  c->have_fwd = false;
  const bool two_streams = !tuning().one_stream;
  if (!c->ev_fork) {
    NMT_HIP_CHECK(hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming));
    NMT_HIP_CHECK(hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming));
    NMT_HIP_CHECK(hipEventCreateWithFlags(&c->ev_done[0], hipEventDisableTiming));
    NMT_HIP_CHECK(hipEventCreateWithFlags(&c->ev_done[1], hipEventDisableTiming));
  }
  // (the second stream comes into being when it is first needed: a stream that exists takes a place on one of the
  //  process's few hardware queues even if nothing is ever enqueued on it)
  if (two_streams && !c->side) NMT_HIP_CHECK(hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking));
  const nmt_config& k = c->cfg;
  const int Bt = c->Bt, Ns = c->Ns, Nt = c->Nt, maxS = c->maxS, maxT = c->maxT;
  const int d = k.d_model, F = k.d_ff, V = k.vocab, H = k.n_heads, dh = d / H;
  const Plan& p = c->plan;
  // one stream: for callers that keep several passes in flight on streams of their own, and for profiling (no overlap,
  // so per-kernel times are those of kernels running alone)
  hipStream_t st = static_cast<hipStream_t>(stream), sd = two_streams ? c->side : st;
  const Run r{c, st};   // input-gradient chain
  const Run w{c, sd};   // weight gradients
  const bool dropping = c->training && k.dropout > 0.f;
  const float act_scale = (c->training && k.act_dropout > 0.f) ? 1.f / (1.f - k.act_dropout) : 1.f;
  half_t* dO = r.ws<half_t>(p.dO);
  const int4 *tab_ss = r.ws<int4>(p.tab_ss), *tab_tt = r.ws<int4>(p.tab_tt), *tab_ts = r.ws<int4>(p.tab_ts);
  const AttnWork wl_ss = attention_work(r.ws<int32_t>(p.wl_ss), Bt, Ns, 0), wl_tt = attention_work(r.ws<int32_t>(p.wl_tt), Bt, Nt, 0),
                 wl_ts = attention_work(r.ws<int32_t>(p.wl_ts), Bt, Nt, Ns);
  float* lnpart = r.ws<float>(p.lnpart);
  float* cspart = r.ws<float>(p.cspart);  // used on the second stream only

  int set = 0;            // temporaries of the current sub-layer
  bool used[2] = {false, false};
  half_t *dy = nullptr, *dym = nullptr, *dqkv = nullptr, *dhid = nullptr, *dq = nullptr, *dkv = nullptr;
  const half_t* dsub = nullptr;  // gradient at a sub-layer's output
  auto begin_sublayer = [&]() -> int {
    set ^= 1;
    if (used[set]) NMT_HIP_CHECK(hipStreamWaitEvent(st, c->ev_done[set], 0));
    used[set] = true;
    dy = r.ws<half_t>(p.dy[set]);
    dym = dropping ? r.ws<half_t>(p.dym[set]) : nullptr;
    dsub = dropping ? dym : dy;
    dqkv = r.ws<half_t>(p.dqkv[set]);
    dhid = r.ws<half_t>(p.dh[set]);
    dq = r.ws<half_t>(p.dq[set]);
    dkv = r.ws<half_t>(p.dkv[set]);
    return NMT_OK;
  };
  auto fork = [&]() -> int {  // the second stream may start on everything enqueued so far
    NMT_HIP_CHECK(hipEventRecord(c->ev_fork, st));
    NMT_HIP_CHECK(hipStreamWaitEvent(sd, c->ev_fork, 0));
    return NMT_OK;
  };
  auto end_sublayer = [&]() -> int {
    NMT_HIP_CHECK(hipEventRecord(c->ev_done[set], sd));
    return NMT_OK;
  };

  // feed-forward sub-layer: out = LN(x_in + drop(relu(x_in W1^T + b1) W2^T + b2)); dx holds d out on entry, d x_in on exit
  auto ffn_bwd = [&](half_t* dx, int N, bool tgt, const half_t* x_in, const half_t* hact, const half_t* sub, const float* stats,
                     const FfnP& f, const LnP& ln, uint32_t site_res) -> int {
    NMT_TRY(begin_sublayer());
    NMT_TRY(launch_residual_layernorm_bwd(dx, sub, x_in, r.w(ln.g), stats, dy, dym, r.g(ln.g), r.g(ln.b), r.g(f.b2), lnpart, N, d,
                                          r.drop(site_res, tgt, k.dropout), st, c->gscale));
    NMT_TRY(fork());
    NMT_TRY(w.wgrad(dsub, N, d, hact, F, f.w2));
    GemmEpilogue relu_bwd;
    relu_bwd.relu_src = hact;
    relu_bwd.mask_scale = act_scale;
    NMT_TRY(r.dgrad(dsub, N, d, f.w2, F, dhid, relu_bwd));
    NMT_TRY(fork());
    NMT_TRY(launch_colsum(dhid, F, w.g(f.b1), cspart, N, F, sd, c->gscale));
    NMT_TRY(w.wgrad(dhid, N, F, x_in, d, f.w1));
    GemmEpilogue res;
    res.add = dy;
    NMT_TRY(r.dgrad(dhid, N, F, f.w1, d, dx, res));
    return end_sublayer();
  };
  // self-attention sub-layer (fused q, k, v projection)
  auto self_bwd = [&](half_t* dx, int N, bool tgt, const half_t* x_in, const half_t* qkv, const half_t* o, const float* lse,
                      const half_t* sub, const float* stats, const AttnP& a, const LnP& ln, uint32_t site_res, const int32_t* key_ids,
                      int causal) -> int {
    NMT_TRY(begin_sublayer());
    NMT_TRY(launch_residual_layernorm_bwd(dx, sub, x_in, r.w(ln.g), stats, dy, dym, r.g(ln.g), r.g(ln.b), r.g(a.bo), lnpart, N, d,
                                          r.drop(site_res, tgt, k.dropout), st, c->gscale));
    NMT_TRY(fork());
    NMT_TRY(w.wgrad(dsub, N, d, o, d, a.wo));
    NMT_TRY(r.dgrad(dsub, N, d, a.wo, d, dO));
    NMT_TRY(launch_attention_bwd(qkv, 3 * d, qkv + d, 3 * d, qkv + 2 * d, 3 * d, o, d, dO, d, lse, dqkv, 3 * d, dqkv + d, 3 * d,
                                 dqkv + 2 * d, 3 * d, key_ids, k.pad_id, causal, Bt, H, dh, tgt ? maxT : maxS, tgt ? maxT : maxS,
                                 tgt ? tab_tt : tab_ss, N, tgt ? &wl_tt : &wl_ss, st));
    NMT_TRY(fork());
    NMT_TRY(launch_colsum(dqkv, 3 * d, w.g(a.bqkv), cspart, N, 3 * d, sd, c->gscale));
    NMT_TRY(w.wgrad(dqkv, N, 3 * d, x_in, d, a.wqkv));
    GemmEpilogue res;
    res.add = dy;
    NMT_TRY(r.dgrad(dqkv, N, 3 * d, a.wqkv, d, dx, res));
    return end_sublayer();
  };

  // ---- output projection: logits = x E^T; the workspace holds d logits ----
  // (the tied matrix's gradient is finished by the embedding kernels at the very end, so its
  //  weight-gradient product stays on the main stream)
  const half_t* dlogits = r.ws<half_t>(p.logits);
  const half_t* x_dec = r.ws<half_t>(p.dec[k.dec_layers - 1].x3);
  half_t* dx = r.ws<half_t>(p.dx_dec);
  NMT_TRY(fork());
  GemmEpilogue vocab_ep;
  vocab_ep.out_scale = c->gscale;
  NMT_TRY(launch_gemm(dlogits, true, V, x_dec, true, d, w.g(c->embed), d, V, d, Nt, vocab_ep, sd));
  NMT_TRY(launch_gemm(dlogits, false, V, r.w(c->embed), true, d, dx, d, Nt, d, V, GemmEpilogue{}, st));

  // ---- decoder, top to bottom ----
  half_t* denc = r.ws<half_t>(p.dx_enc);
  const half_t* enc_out = k.enc_layers ? r.ws<half_t>(p.enc[k.enc_layers - 1].x2) : r.ws<half_t>(p.x0);
  for (int l = k.dec_layers - 1; l >= 0; --l) {
    const DecP& P = c->dec[l];
    const DecW& W = p.dec[l];
    const int li = k.enc_layers + l;
    const half_t* x_in = l ? r.ws<half_t>(p.dec[l - 1].x3) : r.ws<half_t>(p.y0);
    NMT_TRY(ffn_bwd(dx, Nt, true, r.ws<half_t>(W.x2), r.ws<half_t>(W.h), r.ws<half_t>(W.s3), r.ws<float>(W.st3), P.ffn, P.ln3,
                    layer_site(li, kKindFfnRes)));
    // encoder-decoder attention
    NMT_TRY(begin_sublayer());
    NMT_TRY(launch_residual_layernorm_bwd(dx, r.ws<half_t>(W.s2), r.ws<half_t>(W.x1), r.w(P.ln2.g), r.ws<float>(W.st2), dy, dym,
                                          r.g(P.ln2.g), r.g(P.ln2.b), r.g(P.cross.bo), lnpart, Nt, d,
                                          r.drop(layer_site(li, kKindCrossRes), true, k.dropout), st, c->gscale));
    NMT_TRY(fork());
    NMT_TRY(w.wgrad(dsub, Nt, d, r.ws<half_t>(W.o2), d, P.cross.wo));
    NMT_TRY(r.dgrad(dsub, Nt, d, P.cross.wo, d, dO));
    const half_t* kv = r.ws<half_t>(W.kv);
    NMT_TRY(launch_attention_bwd(r.ws<half_t>(W.q), d, kv, 2 * d, kv + d, 2 * d, r.ws<half_t>(W.o2), d, dO, d, r.ws<float>(W.lse2), dq, d,
                                 dkv, 2 * d, dkv + d, 2 * d, c->src, k.pad_id, 0, Bt, H, dh, maxT, maxS, tab_ts, Nt, &wl_ts, st));
    NMT_TRY(fork());
    NMT_TRY(launch_colsum(dq, d, w.g(P.cross.bq), cspart, Nt, d, sd, c->gscale));
    NMT_TRY(launch_colsum(dkv, 2 * d, w.g(P.cross.bkv), cspart, Ns, 2 * d, sd, c->gscale));
    NMT_TRY(w.wgrad(dq, Nt, d, r.ws<half_t>(W.x1), d, P.cross.wq));
    NMT_TRY(w.wgrad(dkv, Ns, 2 * d, enc_out, d, P.cross.wkv));
    GemmEpilogue res;
    res.add = dy;
    NMT_TRY(r.dgrad(dq, Nt, d, P.cross.wq, d, dx, res));
    GemmEpilogue accum;
    accum.add = (l == k.dec_layers - 1) ? nullptr : denc;  // the encoder output feeds every decoder layer
    NMT_TRY(r.dgrad(dkv, Ns, 2 * d, P.cross.wkv, d, denc, accum));
    NMT_TRY(end_sublayer());
    // masked self-attention
    NMT_TRY(self_bwd(dx, Nt, true, x_in, r.ws<half_t>(W.qkv), r.ws<half_t>(W.o1), r.ws<float>(W.lse1), r.ws<half_t>(W.s1),
                     r.ws<float>(W.st1), P.self, P.ln1, layer_site(li, kKindSelfRes), c->tgt_in, 1));
  }
  const half_t* dx_dec0 = dx;

  // ---- encoder ----
  for (int l = k.enc_layers - 1; l >= 0; --l) {
    const EncP& P = c->enc[l];
    const EncW& W = p.enc[l];
    const half_t* x_in = l ? r.ws<half_t>(p.enc[l - 1].x2) : r.ws<half_t>(p.x0);
    NMT_TRY(ffn_bwd(denc, Ns, false, r.ws<half_t>(W.x1), r.ws<half_t>(W.h), r.ws<half_t>(W.s2), r.ws<float>(W.st2), P.ffn, P.ln2,
                    layer_site(l, kKindFfnRes)));
    NMT_TRY(self_bwd(denc, Ns, false, x_in, r.ws<half_t>(W.qkv), r.ws<half_t>(W.o), r.ws<float>(W.lse), r.ws<half_t>(W.s1),
                     r.ws<float>(W.st1), P.attn, P.ln1, layer_site(l, kKindSelfRes), c->src, 0));
  }

  // ---- join, then the embeddings: both id streams add into the row gradients of the shared matrix ----
  NMT_HIP_CHECK(hipEventRecord(c->ev_join, sd));
  NMT_HIP_CHECK(hipStreamWaitEvent(st, c->ev_join, 0));
  NMT_TRY(launch_embed_bwd(c->src, denc, Ns, r.drop(kSiteEmbSrc, false, k.dropout), c->tgt_in, dx_dec0, Nt, r.drop(kSiteEmbTgt, true, k.dropout),
                           r.g(c->embed), d, V, r.ws<int32_t>(p.embscratch), st, c->gscale));
  return NMT_OK;
}

// ================================================================================================
// accumulate / overflow check / Adam
// ================================================================================================
extern "C" int nmt_accumulate(nmt_ctx* ctx, int32_t first, void* stream) {
  NMT_REQUIRE(ctx && ctx->g16 && ctx->acc, "nmt_accumulate: g16 / acc32 not bound");
  return launch_accumulate(ctx->g16, ctx->acc, ctx->P, first, static_cast<hipStream_t>(stream), 1.f / ctx->gscale);
}
extern "C" int nmt_accumulate_loss(nmt_ctx* ctx, int32_t first, float* d_loss_total, int32_t* d_ntok_total, void* stream) {
  NMT_REQUIRE(ctx && d_loss_total && d_ntok_total, "nmt_accumulate_loss: null argument");
  if (!ctx->last_loss || !ctx->last_ntok) {
    nmt_set_error("nmt_accumulate_loss: no forward call has been made");
    return NMT_ESTATE;
  }
  return launch_add_scalars(ctx->last_loss, ctx->last_ntok, d_loss_total, d_ntok_total, first, static_cast<hipStream_t>(stream));
}
extern "C" int nmt_check_overflow(nmt_ctx* ctx, float inv_scale, int32_t* d_flag, void* stream) {
  NMT_REQUIRE(ctx && ctx->acc, "nmt_check_overflow: acc32 not bound");
  NMT_REQUIRE(isfinite(inv_scale) && inv_scale > 0.f, "nmt_check_overflow: inv_scale must be positive and finite");
  ctx->inv_scale = inv_scale;
  return launch_check_overflow(ctx->acc, ctx->P, inv_scale, d_flag, static_cast<hipStream_t>(stream), false);
}
extern "C" int nmt_adam_step(nmt_ctx* ctx, float lr, float beta1, float beta2, float eps, int32_t t, const int32_t* d_flag,
                             void* stream) {
  NMT_REQUIRE(ctx && ctx->acc && ctx->master && ctx->m && ctx->v && ctx->w16, "nmt_adam_step: optimizer buffers not bound");
  NMT_REQUIRE(d_flag, "nmt_adam_step: null flag");
  return launch_adam(ctx->master, ctx->m, ctx->v, ctx->acc, ctx->w16, ctx->P, lr, beta1, beta2, eps, t, d_flag,
                     static_cast<hipStream_t>(stream), ctx->inv_scale);
}

extern "C" int nmt_gemm_timing(double* ms, int64_t* products, double* flops) { return gemm_timing_read(ms, products, flops); }

// Debug export: where a saved activation of the last forward pass lies in the workspace.
extern "C" int nmt_debug_activation(const nmt_ctx* ctx, const char* name, const void** d_ptr, int64_t* rows, int64_t* cols) {
  NMT_REQUIRE(ctx && name && d_ptr && rows && cols, "nmt_debug_activation: null argument");
  if (!ctx->last_loss || !ctx->ws) {
    nmt_set_error("nmt_debug_activation: no forward call has been made");
    return NMT_ESTATE;
  }
  const nmt_config& k = ctx->cfg;
  int layer = -1, len = 0;
  char side[4] = "", what[16] = "";
  if (sscanf(name, "%3[a-z]%d.%15[a-z.]%n", side, &layer, what, &len) == 3 && name[len] == 0) {
    const bool enc = !strcmp(side, "enc"), dec = !strcmp(side, "dec");
    if ((enc && layer >= 0 && layer < k.enc_layers) || (dec && layer >= 0 && layer < k.dec_layers)) {
      const int64_t n = enc ? ctx->Ns : ctx->Nt;
      int64_t off = -1, width = k.d_model;
      if (!strcmp(what, "ffn.h")) { off = enc ? ctx->plan.enc[layer].h : ctx->plan.dec[layer].h; width = k.d_ff; }
      else if (!strcmp(what, "out")) off = enc ? ctx->plan.enc[layer].x2 : ctx->plan.dec[layer].x3;
      if (off >= 0) {
        *d_ptr = ctx->ws + off;
        *rows = n;
        *cols = width;
        return NMT_OK;
      }
    }
  }
  NMT_REQUIRE(false, "nmt_debug_activation: unknown activation '%s'", name);
}

extern "C" int nmt_scaler_update(float* scale, int32_t* clean, int32_t overflow, int32_t window) {
  NMT_REQUIRE(scale && clean && window >= 1, "nmt_scaler_update: bad arguments");
  if (overflow) {
    NMT_REQUIRE(*scale * 0.5f >= 6.103515625e-05f, "nmt_scaler_update: loss scale would fall below 2^-14");
    *scale *= 0.5f;
    *clean = 0;
  } else if (++*clean == window) {
    *scale *= 2.f;
    *clean = 0;
  }
  return NMT_OK;
}
extern "C" double nmt_lr_schedule(int64_t t, double peak, int64_t warmup) {
  if (t < 1 || warmup < 1) return 0.0;
  const double up = (double)t / (double)warmup, down = sqrt((double)warmup / (double)t);
  return peak * (up < down ? up : down);
}

// ================================================================================================
// kernel-level entry points
// ================================================================================================
extern "C" int nmt_op_gemm(const void* d_A, int32_t a_t, int32_t lda, const void* d_B, int32_t b_t, int32_t ldb, void* d_C,
                           int32_t ldc, int32_t M, int32_t N, int32_t K, const void* d_bias, int32_t relu, const nmt_dropout* drop,
                           const void* d_add, const void* d_relu_src, float mask_scale, void* stream) {
  NMT_TRY(check_drop(drop, "nmt_op_gemm"));
  GemmEpilogue ep;
  ep.bias = static_cast<const half_t*>(d_bias);
  ep.relu = relu;
  ep.drop = make_drop(drop);
  ep.add = static_cast<const half_t*>(d_add);
  ep.relu_src = static_cast<const half_t*>(d_relu_src);
  ep.mask_scale = mask_scale;
  return launch_gemm(static_cast<const half_t*>(d_A), a_t != 0, lda, static_cast<const half_t*>(d_B), b_t != 0, ldb,
                     static_cast<half_t*>(d_C), ldc, M, N, K, ep, static_cast<hipStream_t>(stream));
}

extern "C" int nmt_op_gemm_f32(const float* d_A, int32_t a_t, int32_t lda, const float* d_B, int32_t b_t, int32_t ldb, float* d_C,
                               int32_t ldc, int32_t M, int32_t N, int32_t K, int32_t splits, void* stream) {
  return launch_gemm_f32(d_A, a_t != 0, lda, d_B, b_t != 0, ldb, d_C, ldc, M, N, K, splits, static_cast<hipStream_t>(stream));
}

extern "C" int nmt_op_gemm_splitk(const void* d_A, int32_t a_t, int32_t lda, const void* d_B, int32_t b_t, int32_t ldb, void* d_C,
                                  int32_t ldc, int32_t M, int32_t N, int32_t K, float* d_partial, int64_t partial_floats,
                                  int32_t splits, void* stream) {
  NMT_REQUIRE(d_partial && partial_floats > 0, "nmt_op_gemm_splitk: the partial-sum buffer is required");
  return launch_gemm(static_cast<const half_t*>(d_A), a_t != 0, lda, static_cast<const half_t*>(d_B), b_t != 0, ldb,
                     static_cast<half_t*>(d_C), ldc, M, N, K, GemmEpilogue{}, static_cast<hipStream_t>(stream), d_partial, partial_floats,
                     splits);
}

extern "C" int nmt_op_attention_fwd(const void* d_Q, int32_t ldq, const void* d_K, int32_t ldk, const void* d_V, int32_t ldv,
                                    void* d_O, int32_t ldo, float* d_lse, const int32_t* d_key_ids, int32_t pad_id, int32_t causal,
                                    int32_t B, int32_t H, int32_t dh, int32_t Tq, int32_t Tk, void* stream) {
  return launch_attention_fwd(static_cast<const half_t*>(d_Q), ldq, static_cast<const half_t*>(d_K), ldk, static_cast<const half_t*>(d_V),
                              ldv, static_cast<half_t*>(d_O), ldo, d_lse, d_key_ids, pad_id, causal, B, H, dh, Tq, Tk, nullptr, 0, nullptr,
                              static_cast<hipStream_t>(stream));
}
extern "C" int nmt_op_attention_bwd(const void* d_Q, int32_t ldq, const void* d_K, int32_t ldk, const void* d_V, int32_t ldv,
                                    const void* d_O, int32_t ldo, const void* d_dO, int32_t lddo, const float* d_lse, void* d_dQ,
                                    int32_t lddq, void* d_dK, int32_t lddk, void* d_dV, int32_t lddv, const int32_t* d_key_ids,
                                    int32_t pad_id, int32_t causal, int32_t B, int32_t H, int32_t dh, int32_t Tq, int32_t Tk,
                                    void* stream) {
  return launch_attention_bwd(static_cast<const half_t*>(d_Q), ldq, static_cast<const half_t*>(d_K), ldk, static_cast<const half_t*>(d_V),
                              ldv, static_cast<const half_t*>(d_O), ldo, static_cast<const half_t*>(d_dO), lddo, d_lse,
                              static_cast<half_t*>(d_dQ), lddq, static_cast<half_t*>(d_dK), lddk, static_cast<half_t*>(d_dV), lddv,
                              d_key_ids, pad_id, causal, B, H, dh, Tq, Tk, nullptr, 0, nullptr, static_cast<hipStream_t>(stream));
}

extern "C" int nmt_op_residual_layernorm_fwd(const void* d_sub, const void* d_resid, const void* d_gamma, const void* d_beta,
                                             void* d_out, float* d_stats, int32_t rows, int32_t d, float eps, const nmt_dropout* drop,
                                             void* stream) {
  NMT_TRY(check_drop(drop, "nmt_op_residual_layernorm_fwd"));
  NMT_REQUIRE(eps > 0.f, "nmt_op_residual_layernorm_fwd: eps must be positive");
  return launch_residual_layernorm_fwd(static_cast<const half_t*>(d_sub), static_cast<const half_t*>(d_resid),
                                       static_cast<const half_t*>(d_gamma), static_cast<const half_t*>(d_beta), static_cast<half_t*>(d_out),
                                       d_stats, rows, d, eps, make_drop(drop), static_cast<hipStream_t>(stream));
}
extern "C" int64_t nmt_op_layernorm_bwd_scratch(int32_t d) { return d > 0 ? layernorm_bwd_scratch_floats(d) : NMT_EINVAL; }
extern "C" int nmt_op_residual_layernorm_bwd(const void* d_dout, const void* d_sub, const void* d_resid, const void* d_gamma,
                                             const float* d_stats, void* d_dy, void* d_dym, void* d_dgamma, void* d_dbeta,
                                             void* d_dbias, float* d_partial, int32_t rows, int32_t d, const nmt_dropout* drop,
                                             void* stream) {
  NMT_TRY(check_drop(drop, "nmt_op_residual_layernorm_bwd"));
  return launch_residual_layernorm_bwd(static_cast<const half_t*>(d_dout), static_cast<const half_t*>(d_sub),
                                       static_cast<const half_t*>(d_resid), static_cast<const half_t*>(d_gamma), d_stats,
                                       static_cast<half_t*>(d_dy), static_cast<half_t*>(d_dym), static_cast<half_t*>(d_dgamma),
                                       static_cast<half_t*>(d_dbeta), static_cast<half_t*>(d_dbias), d_partial, rows, d, make_drop(drop),
                                       static_cast<hipStream_t>(stream));
}

extern "C" int nmt_op_embed_fwd(const int32_t* d_ids, const void* d_E, void* d_x, int32_t rows, int32_t d, int32_t vocab,
                                const nmt_dropout* drop, void* stream) {
  NMT_REQUIRE(drop, "nmt_op_embed_fwd: the dropout description is required (it carries the positions per sentence)");
  NMT_TRY(check_drop(drop, "nmt_op_embed_fwd"));
  return launch_embed_fwd(d_ids, static_cast<const half_t*>(d_E), static_cast<half_t*>(d_x), rows, d, vocab, make_drop(drop),
                          static_cast<hipStream_t>(stream));
}

extern "C" int nmt_op_softmax_xent(void* d_logits, const int32_t* d_targets, float* d_row_loss, int32_t rows, int32_t V,
                                   int32_t pad_id, float label_smoothing, float loss_scale, float* d_loss_sum, int32_t* d_ntok,
                                   void* stream) {
  return launch_softmax_xent(static_cast<half_t*>(d_logits), d_targets, d_row_loss, rows, V, pad_id, label_smoothing, loss_scale,
                             d_loss_sum, d_ntok, static_cast<hipStream_t>(stream));
}

extern "C" int64_t nmt_op_colsum_scratch(int32_t cols) { return cols > 0 ? colsum_scratch_floats(cols) : NMT_EINVAL; }
extern "C" int nmt_op_colsum(const void* d_src, int32_t ld, void* d_dst, float* d_partial, int32_t rows, int32_t cols, void* stream) {
  return launch_colsum(static_cast<const half_t*>(d_src), ld, static_cast<half_t*>(d_dst), d_partial, rows, cols,
                       static_cast<hipStream_t>(stream));
}

extern "C" int nmt_op_colsum_static(const void* d_src, int32_t ld, void* d_dst, int32_t rows, int32_t cols, void* stream) {
  return launch_colsum_static(static_cast<const half_t*>(d_src), ld, static_cast<half_t*>(d_dst), rows, cols, static_cast<hipStream_t>(stream));
}

extern "C" int64_t nmt_op_embed_bwd_scratch(int32_t vocab, int32_t rows_total, int32_t d) {
  return (vocab > 0 && rows_total > 0 && d > 0) ? embed_bwd_scratch_ints(vocab, rows_total, d) : NMT_EINVAL;
}
extern "C" int nmt_op_embed_bwd(const int32_t* d_ids_a, const void* d_dx_a, int32_t rows_a, const nmt_dropout* drop_a,
                                const int32_t* d_ids_b, const void* d_dx_b, int32_t rows_b, const nmt_dropout* drop_b, void* d_gE,
                                int32_t d, int32_t vocab, int32_t* d_scratch, void* stream) {
  NMT_TRY(check_drop(drop_a, "nmt_op_embed_bwd"));
  NMT_TRY(check_drop(drop_b, "nmt_op_embed_bwd"));
  return launch_embed_bwd(d_ids_a, static_cast<const half_t*>(d_dx_a), rows_a, make_drop(drop_a), d_ids_b,
                          static_cast<const half_t*>(d_dx_b), rows_b, make_drop(drop_b), static_cast<half_t*>(d_gE), d, vocab, d_scratch,
                          static_cast<hipStream_t>(stream));
}

extern "C" int nmt_op_accumulate(const void* d_g16, float* d_acc32, int64_t n, int32_t first, void* stream) {
  return launch_accumulate(static_cast<const half_t*>(d_g16), d_acc32, n, first, static_cast<hipStream_t>(stream));
}
extern "C" int nmt_op_check_overflow(float* d_acc32, int64_t n, float inv_scale, int32_t* d_flag, void* stream) {
  return launch_check_overflow(d_acc32, n, inv_scale, d_flag, static_cast<hipStream_t>(stream));
}
extern "C" int nmt_op_adam(float* d_master32, float* d_m, float* d_v, const float* d_g32, float grad_scale, void* d_w16, int64_t n,
                           float lr, float beta1, float beta2, float eps, int32_t t, const int32_t* d_flag, void* stream) {
  return launch_adam(d_master32, d_m, d_v, d_g32, static_cast<half_t*>(d_w16), n, lr, beta1, beta2, eps, t, d_flag,
                     static_cast<hipStream_t>(stream), grad_scale);
}
extern "C" int nmt_op_dropout_mask(uint8_t* d_keep, int32_t rows, int32_t n_cols, const nmt_dropout* drop, void* stream) {
  NMT_TRY(check_drop(drop, "nmt_op_dropout_mask"));
  return launch_dropout_mask(d_keep, rows, n_cols, make_drop(drop), static_cast<hipStream_t>(stream));
}

// Block engine: parameter table, workspace plan and the kernel sequence of one
// local-block step (Algorithm 1: forward, push point, local loss, backward that
// stops at the block input, update).
#include "block.h"

#include <cmath>
#include <cstdio>
#include <cstdlib>

namespace ppll {

// a layer's weight-gradient products go to the side stream when they have this many output tiles (one per compute unit)
constexpr long SIDE_MIN_TILES = 256;
// ... and only when their reduction runs over this many rows: short products end before the fork and join pay off
// (640 rows at width 768: 4 % slower with the side stream)
constexpr int SIDE_MIN_ROWS = 4096;


namespace {
struct Bump {
  char* base;
  size_t off = 0;
  explicit Bump(char* b) : base(b) {}
  void* take(size_t bytes) {
    off = (off + 255) & ~(size_t)255;
    void* p = base ? base + off : nullptr;
    off += bytes;
    return p;
  }
  float* floats(size_t n) { return (float*)take(n * sizeof(float)); }
};

GemmArgs gemm_args() {
  GemmArgs g{};
  g.epilogue = EPI_NONE;
  return g;
}
}  // namespace

int validate_config(const ppll_block_config* c) {
  if (!c) { set_error("config is null"); return PPLL_ERR_NULL; }
  if (c->struct_size != sizeof(ppll_block_config)) {
    set_error("config struct_size %u, library expects %zu", c->struct_size, sizeof(ppll_block_config));
    return PPLL_ERR_CONFIG;
  }
  auto bad = [](const char* what) { set_error("config: %s", what); return PPLL_ERR_CONFIG; };
  if (c->precision != PPLL_FP32 && c->precision != PPLL_BF16) return bad("precision must be PPLL_FP32 or PPLL_BF16");
  if (c->optimizer != PPLL_SGD && c->optimizer != PPLL_ADAMW) return bad("optimizer must be PPLL_SGD or PPLL_ADAMW");
  if (c->batch < 1 || c->batch > 65536) return bad("batch outside 1..65536");
  if (c->num_classes < 2 || c->num_classes > 1024) return bad("num_classes outside 2..1024");
  if (c->arch == PPLL_VIT) {
    if (c->input_kind != PPLL_IN_IMAGE && c->input_kind != PPLL_IN_ACTIVATION) return bad("input_kind");
    if (c->dim < 1 || c->heads < 1 || c->dim % c->heads) return bad("dim must be a positive multiple of heads");
    if (c->dim > 1536) return bad("dim above 1536");
    if (c->mlp_dim < 1 || c->depth < 1 || c->aux_depth < 0) return bad("mlp_dim, depth >= 1 and aux_depth >= 0 required");
    if (c->tokens < 1 || c->tokens > 256) return bad("tokens outside 1..256");
    if (c->ln_eps <= 0.f) return bad("ln_eps must be positive");
    if (c->input_kind == PPLL_IN_IMAGE) {
      if (c->patch < 1 || c->img_h < 1 || c->img_w < 1 || c->img_c < 1 || c->img_h % c->patch || c->img_w % c->patch)
        return bad("image size must be a positive multiple of patch");
      if ((c->img_h / c->patch) * (c->img_w / c->patch) + 1 != c->tokens)
        return bad("tokens must equal (img_h/patch)*(img_w/patch) + 1");
    }
    // every limit a kernel of the step would otherwise hit at launch time, when earlier kernels are already enqueued
    const size_t dh = (size_t)(c->dim / c->heads), T = (size_t)c->tokens;
    if (c->precision != PPLL_BF16 || dh != 64) {   // the run-time-typed attention kernels keep K, V (or Q, dO) of one head in LDS
      const size_t lds = (2 * T * (dh + 1) + 8 * dh + 10 * T) * sizeof(float);
      if (lds > 160 * 1024) return bad("tokens x head dimension needs more than 160 KB of LDS in the attention kernels of this path");
    }
    const size_t widest = (size_t)(3 * c->dim > c->mlp_dim ? 3 * c->dim : c->mlp_dim);
    if ((size_t)c->batch * T * widest > ((size_t)1 << 31) - 1) return bad("batch x tokens x layer width above 2^31 - 1 elements");
    if (c->input_kind == PPLL_IN_IMAGE && (size_t)c->batch * c->img_h * c->img_w * c->img_c > ((size_t)1 << 31) - 1)
      return bad("image batch above 2^31 - 1 elements");
  } else if (c->arch == PPLL_RESNET) {
    if (c->input_kind != PPLL_IN_IMAGE && c->input_kind != PPLL_IN_ACTIVATION) return bad("input_kind");
    if (c->channels < 1 || c->aux_channels < 1 || c->height < 2 || c->width < 2 || c->n_basic_blocks < 1)
      return bad("channels, aux_channels, n_basic_blocks >= 1 and height, width >= 2 required");
    if (c->transition_block < 0 || c->transition_block > c->n_basic_blocks)
      return bad("transition_block outside 0..n_basic_blocks");
    if (c->transition_block > 0 && (c->channels % 2)) return bad("a downsampling basic block doubles the channels: channels must be even");
    if (c->height > 4096 || c->width > 4096 || c->channels > 4096) return bad("height, width, channels above 4096");
    if (c->input_kind == PPLL_IN_IMAGE) {
      const int m = c->transition_block > 0 ? 2 : 1;
      if (c->img_c < 1 || c->img_h != m * c->height || c->img_w != m * c->width)
        return bad("the stem keeps the image size: img_h, img_w must equal the first basic block's input size");
    }
    if (c->bn_eps <= 0.f || c->bn_momentum < 0.f || c->bn_momentum > 1.f) return bad("bn_eps > 0 and bn_momentum in [0,1] required");
    {
      const size_t m = c->transition_block > 0 ? 2 : 1, wide = c->channels > c->aux_channels ? c->channels : c->aux_channels;
      if ((size_t)c->batch * (m * c->height) * (m * c->width) * wide > ((size_t)1 << 31) - 1)
        return bad("batch x map x channels above 2^31 - 1 elements");
    }
  } else {
    return bad("arch must be PPLL_VIT or PPLL_RESNET");
  }
  return PPLL_OK;
}

size_t Block::in_elems() const {
  const size_t B = (size_t)cfg.batch;
  if (cfg.arch == PPLL_VIT)
    return cfg.input_kind == PPLL_IN_IMAGE ? B * cfg.img_h * cfg.img_w * cfg.img_c : B * cfg.tokens * cfg.dim;
  if (cfg.input_kind == PPLL_IN_IMAGE) return B * cfg.img_h * cfg.img_w * cfg.img_c;
  const size_t m = cfg.transition_block > 0 ? 2 : 1;
  return B * (m * cfg.height) * (m * cfg.width) * (cfg.channels / m);
}
size_t Block::out_elems() const {
  if (cfg.arch == PPLL_VIT) return (size_t)cfg.batch * cfg.tokens * cfg.dim;
  return (size_t)cfg.batch * cfg.height * cfg.width * cfg.channels;
}

size_t Block::plan(char* base) {
  dt = cfg.precision == PPLL_BF16 ? BF16 : F32;
  esz = dtype_size(dt);
  tensors.clear(); enc_p.clear(); enc_a.clear(); rb_p.clear(); rb_a.clear(); rb_d.clear();
  bn_names.clear(); bn_channels.clear(); bn_off.clear();
  size_t off = 0;
  auto add = [&](const std::string& name, int rows, int cols) {
    size_t o = off;
    tensors.push_back({name, o, (size_t)rows * cols, rows, cols});
    off += (size_t)rows * cols;
    return o;
  };
  const int B = cfg.batch, C = cfg.num_classes;
  if (cfg.arch == PPLL_VIT) {
    const int D = cfg.dim, F = cfg.mlp_dim;
    if (cfg.input_kind == PPLL_IN_IMAGE) {
      pe_w = add("pe.w", cfg.patch * cfg.patch * cfg.img_c, D);
      pe_b = add("pe.b", 1, D);
      cls = add("cls", 1, D);
      pos = add("pos", cfg.tokens, D);
    }
    for (int l = 0; l < cfg.depth + cfg.aux_depth; ++l) {
      char pre[32];
      if (l < cfg.depth) snprintf(pre, sizeof pre, "blk%d", l); else snprintf(pre, sizeof pre, "aux%d", l - cfg.depth);
      std::string p(pre);
      EncoderParams e;
      e.ln1_g = add(p + ".ln1.g", 1, D); e.ln1_b = add(p + ".ln1.b", 1, D);
      e.qkv_w = add(p + ".qkv.w", D, 3 * D); e.qkv_b = add(p + ".qkv.b", 1, 3 * D);
      e.proj_w = add(p + ".proj.w", D, D); e.proj_b = add(p + ".proj.b", 1, D);
      e.ln2_g = add(p + ".ln2.g", 1, D); e.ln2_b = add(p + ".ln2.b", 1, D);
      e.fc1_w = add(p + ".fc1.w", D, F); e.fc1_b = add(p + ".fc1.b", 1, F);
      e.fc2_w = add(p + ".fc2.w", F, D); e.fc2_b = add(p + ".fc2.b", 1, D);
      enc_p.push_back(e);
    }
    head_ln_g = add("head.ln.g", 1, D); head_ln_b = add("head.ln.b", 1, D);
    head_w = add("head.w", D, C); head_b = add("head.b", 1, C);
  } else {
    const int Ch = cfg.channels, A = cfg.aux_channels, t = cfg.transition_block - 1;
    const int m = t >= 0 ? 2 : 1;
    in_h = m * cfg.height; in_w = m * cfg.width; in_c = Ch / m;
    stem = cfg.input_kind == PPLL_IN_IMAGE;
    bn_base = stem ? 1 : 0;
    if (stem) {
      stem_w = add("stem.conv.w", 9 * cfg.img_c, in_c); stem_g = add("stem.bn.g", 1, in_c); stem_b = add("stem.bn.b", 1, in_c);
      bn_names.push_back("stem.bn"); bn_channels.push_back(in_c);
    }
    for (int i = 0; i < cfg.n_basic_blocks; ++i) {
      std::string p = "rb" + std::to_string(i);
      BasicBlockDims d;
      if (t >= 0 && i < t) d = {in_c, in_c, 1, in_h, in_w, in_h, in_w};
      else if (i == t) d = {in_c, Ch, 2, in_h, in_w, cfg.height, cfg.width};
      else d = {Ch, Ch, 1, cfg.height, cfg.width, cfg.height, cfg.width};
      rb_d.push_back(d);
      BasicBlockParams r;
      r.conv1_w = add(p + ".conv1.w", 9 * d.Ci, d.Co); r.bn1_g = add(p + ".bn1.g", 1, d.Co); r.bn1_b = add(p + ".bn1.b", 1, d.Co);
      r.conv2_w = add(p + ".conv2.w", 9 * d.Co, d.Co); r.bn2_g = add(p + ".bn2.g", 1, d.Co); r.bn2_b = add(p + ".bn2.b", 1, d.Co);
      rb_p.push_back(r);
      bn_names.push_back(p + ".bn1"); bn_channels.push_back(d.Co);
      bn_names.push_back(p + ".bn2"); bn_channels.push_back(d.Co);
    }
    aux_conv_w = add("aux.conv.w", 9 * Ch, A); aux_bn_g = add("aux.bn.g", 1, A); aux_bn_b = add("aux.bn.b", 1, A);
    bn_names.push_back("aux.bn"); bn_channels.push_back(A);
    head_w = add("head.w", A, C); head_b = add("head.b", 1, C);
  }
  P = off;

  Bump bump(base);
  params = bump.floats(P); grads = bump.floats(P); mom1 = bump.floats(P);
  mom2 = cfg.optimizer == PPLL_ADAMW ? bump.floats(P) : nullptr;
  shadow = dt == BF16 ? (uint16_t*)bump.take(P * sizeof(uint16_t)) : nullptr;
  size_t bn_total = 0;
  for (int c : bn_channels) { bn_off.push_back(bn_total); bn_total += c; }
  bn_mean_run = bump.floats(bn_total ? bn_total : 1);
  bn_var_run = bump.floats(bn_total ? bn_total : 1);
  loss_dev = bump.floats(1);
  flag_dev = (int*)bump.take(sizeof(int));
  logits = bump.floats((size_t)B * C);
  dlogits = bump.floats((size_t)B * C);

  if (cfg.arch == PPLL_VIT) {
    const int D = cfg.dim, F = cfg.mlp_dim, T = cfg.tokens, H = cfg.heads;
    const size_t M = (size_t)B * T;
    if (cfg.input_kind == PPLL_IN_IMAGE) {
      patches = bump.take((size_t)B * (T - 1) * cfg.patch * cfg.patch * cfg.img_c * esz);
      embed_tmp = bump.take((size_t)B * (T - 1) * D * esz);
      x0 = bump.take(M * D * esz);
    }
    for (int l = 0; l < cfg.depth + cfg.aux_depth; ++l) {
      EncoderActs a;
      a.u1 = bump.take(M * D * esz); a.qkv = bump.take(M * 3 * D * esz); a.att = bump.take(M * D * esz);
      a.x1 = bump.take(M * D * esz); a.u2 = bump.take(M * D * esz);
      a.h = bump.take(M * F * esz); a.gl = bump.take(M * F * esz);
      a.x2 = bump.take(M * D * esz);
      a.mean1 = bump.floats(M); a.rstd1 = bump.floats(M); a.mean2 = bump.floats(M); a.rstd2 = bump.floats(M);
      a.lse = bump.floats((size_t)B * H * T);
      enc_a.push_back(a);
    }
    z = bump.take((size_t)B * D * esz); dz = bump.take((size_t)B * D * esz); dcls = bump.take((size_t)B * D * esz);
    prune_cls = cfg.aux_depth >= 1 && attention_cls_lds_bytes(T, D / H) <= 160 * 1024;
    if (prune_cls) {
      ClsActs& c = cls_a;
      const size_t bd = (size_t)B * D * esz, bf = (size_t)B * F * esz;
      c.q = bump.take(bd); c.att = bump.take(bd); c.x1 = bump.take(bd); c.u2 = bump.take(bd); c.x2 = bump.take(bd);
      c.h = bump.take(bf); c.gl = bump.take(bf); c.d_h = bump.take(bf);
      c.d_u2 = bump.take(bd); c.d_x1 = bump.take(bd); c.d_att = bump.take(bd); c.d_q = bump.take(bd);
      c.mean2 = bump.floats(B); c.rstd2 = bump.floats(B); c.prob = bump.floats((size_t)B * H * T);
    }
    head_mean = bump.floats(B); head_rstd = bump.floats(B);
    d_u = bump.take(M * D * esz);
    g_res.clear(); g_mid.clear(); d_h.clear(); d_qkv.clear();
    const int layers = cfg.depth + cfg.aux_depth;
    for (int l = 0; l <= layers; ++l) g_res.push_back(bump.take(M * D * esz));
    for (int l = 0; l < layers; ++l) {
      g_mid.push_back(bump.take(M * D * esz));
      d_h.push_back(bump.take(M * F * esz));
      d_qkv.push_back(bump.take(M * 3 * D * esz));
    }
    if (dt == BF16) {
      const size_t cand[] = {gemm_mfma_partial_floats(D, 3 * D, (int)M), gemm_mfma_partial_floats(D, D, (int)M),
                             gemm_mfma_partial_floats(D, F, (int)M), gemm_mfma_partial_floats(F, D, (int)M),
                             cfg.input_kind == PPLL_IN_IMAGE
                                 ? gemm_mfma_partial_floats(cfg.patch * cfg.patch * cfg.img_c, D, B * (T - 1)) : 0};
      splitk_floats = 0;
      for (size_t c : cand) if (c > splitk_floats) splitk_floats = c;
      // the grouped weight-gradient launch at the end of the backward pass passes divided tiles through the same scratch
      if (gemm_mfma_balanced_floats() > splitk_floats) splitk_floats = gemm_mfma_balanced_floats();
      splitk = splitk_floats ? bump.floats(splitk_floats) : nullptr;
    }
    int widest = 3 * D > F ? 3 * D : F;
    partial_floats = (size_t)colsum_partial_floats((int)M, widest);
    size_t ln = (size_t)layernorm_bwd_partial_floats((int)M, D);
    if (ln > partial_floats) partial_floats = ln;
    if (cfg.input_kind == PPLL_IN_IMAGE) {
      size_t eb = (size_t)embed_bwd_partial_floats(B, T, D);
      if (eb > partial_floats) partial_floats = eb;
    }
    if (vit_head_partial_floats(B, D, C) > partial_floats) partial_floats = vit_head_partial_floats(B, D, C);
  } else {
    const int Ch = cfg.channels, A = cfg.aux_channels, Hh = cfg.height, W = cfg.width;
    const int Ho = (Hh - 1) / 2 + 1, Wo = (W - 1) / 2 + 1;
    const size_t aact = (size_t)B * Ho * Wo * A;
    size_t widest = (size_t)B * in_h * in_w * in_c;   // largest activation a gradient buffer has to hold
    auto grow = [&](size_t v) { if (v > partial_floats) partial_floats = v; };
    partial_floats = 0;
    if (stem) {
      stem_c = bump.take(widest * esz); stem_y = bump.take(widest * esz);
      stem_mean = bump.floats(in_c); stem_rstd = bump.floats(in_c);
      stem_xp = stem_wp = nullptr;
      stem_pad = dt == BF16 && cfg.img_c < 16 && in_c % 16 == 0 && in_c <= 64;
      if (stem_pad) {
        stem_xp = bump.take((size_t)B * in_h * in_w * 16 * esz);
        stem_wp = bump.take((size_t)9 * 16 * in_c * esz);
        grow((size_t)conv3x3_wgrad_partial_floats(B, in_h, in_w, 16, in_c, 1));
      }
      grow((size_t)conv3x3_wgrad_partial_floats(B, in_h, in_w, cfg.img_c, in_c, 1));
      grow((size_t)bn_partial_floats(B * in_h * in_w, in_c));
    }
    for (int i = 0; i < cfg.n_basic_blocks; ++i) {
      const BasicBlockDims& d = rb_d[i];
      const size_t act = (size_t)B * d.Ho * d.Wo * d.Co;
      if (act > widest) widest = act;
      BasicBlockActs a;
      a.c1 = bump.take(act * esz); a.y1 = bump.take(act * esz); a.c2 = bump.take(act * esz); a.out = bump.take(act * esz);
      a.d1 = bump.take(act * esz); a.d2 = bump.take(act * esz);
      a.mean1 = bump.floats(d.Co); a.rstd1 = bump.floats(d.Co); a.mean2 = bump.floats(d.Co); a.rstd2 = bump.floats(d.Co);
      rb_a.push_back(a);
      if (d.stride != 1 || d.Ci != d.Co) shortcut = bump.take(act * esz);
      grow((size_t)conv3x3_wgrad_partial_floats(B, d.Hin, d.Win, d.Ci, d.Co, d.stride));
      grow((size_t)conv3x3_wgrad_partial_floats(B, d.Ho, d.Wo, d.Co, d.Co, 1));
      grow((size_t)bn_partial_floats(B * d.Ho * d.Wo, d.Co));
    }
    aux_c = bump.take(aact * esz); aux_y = bump.take(aact * esz); d_aux = bump.take(aact * esz);
    pooled = bump.take((size_t)B * A * esz); dpooled = bump.take((size_t)B * A * esz);
    aux_mean = bump.floats(A); aux_rstd = bump.floats(A);
    r_gA = bump.take(widest * esz); r_gB = bump.take(widest * esz); r_t1 = bump.take(widest * esz);
    grow((size_t)conv3x3_wgrad_partial_floats(B, Hh, W, Ch, A, 2));
    grow(vit_head_partial_floats(B, A, C));
    grow((size_t)bn_partial_floats(B * Ho * Wo, A));
  }
  size_t o = (size_t)colsum_partial_floats(B, C);
  if (o > partial_floats) partial_floats = o;
  partials = bump.floats(partial_floats);
  rq.scratch = partials;
  // room for every queued reduction of a step: LayerNorm scale/shift gradients of all layers and the
  // head, position / class-token / bias gradients (a reduction that finds no room runs at once)
  arena_floats = 0;
  if (cfg.arch == PPLL_VIT) {
    const int B = cfg.batch, T = cfg.tokens, D = cfg.dim;
    const size_t M = (size_t)B * T;
    const int widest = cfg.mlp_dim > 3 * D ? cfg.mlp_dim : 3 * D;
    arena_floats = (size_t)(2 * (cfg.depth + cfg.aux_depth)) * (layernorm_bwd_partial_floats((int)M, D) + 64) +
                   (size_t)layernorm_bwd_partial_floats(B, D) + (size_t)colsum_partial_floats(B, C) + 256 +
                   vit_head_partial_floats(B, D, C) + 64;
    if (cfg.input_kind == PPLL_IN_IMAGE)
      arena_floats += (size_t)embed_bwd_partial_floats(B, T, D) + (size_t)colsum_partial_floats((int)M, D) + 128;
    if (!(dt == BF16))   // the generic GEMM does not fold bias gradients: one column sum per Linear layer
      arena_floats += (size_t)(cfg.depth + cfg.aux_depth) * 4 * ((size_t)colsum_partial_floats((int)M, widest) + 64);
    if (prune_cls)   // the class-token layer: one more LayerNorm backward over B rows and column sums of its split products
      arena_floats += (size_t)layernorm_bwd_partial_floats(B, D) + 6 * ((size_t)colsum_partial_floats((int)M, widest) + 64);
  }
  if (cfg.arch == PPLL_RESNET) {   // the weight-gradient partials of every convolution
    const int Ch = cfg.channels, A = cfg.aux_channels, Hh = cfg.height, W = cfg.width;
    arena_floats = (size_t)conv3x3_wgrad_partial_floats(cfg.batch, Hh, W, Ch, A, 2) + 64 +
                   vit_head_partial_floats(cfg.batch, A, cfg.num_classes) + 256;
    for (const BasicBlockDims& d : rb_d)
      arena_floats += (size_t)conv3x3_wgrad_partial_floats(cfg.batch, d.Hin, d.Win, d.Ci, d.Co, d.stride) +
                      (size_t)conv3x3_wgrad_partial_floats(cfg.batch, d.Ho, d.Wo, d.Co, d.Co, 1) + 128;
    if (stem) arena_floats += (size_t)conv3x3_wgrad_partial_floats(cfg.batch, in_h, in_w, stem_pad ? 16 : cfg.img_c, in_c, 1) + 64;
  }
  rq.arena = arena_floats ? bump.floats(arena_floats) : nullptr;
  rq.arena_floats = arena_floats;
  return (bump.off + 255) & ~(size_t)255;
}

// ------------------------------------------------------------------ ViT
int Block::encoder_fwd(int l, const EncoderActs& a, const void* x, void* x2_out, hipStream_t s) {
  const int D = cfg.dim, F = cfg.mlp_dim, T = cfg.tokens, H = cfg.heads, M = cfg.batch * T;
  const EncoderParams& p = enc_p[l];
  PPLL_TRY(launch_layernorm_fwd(s, x, dt, D, M, D, params + p.ln1_g, params + p.ln1_b, cfg.ln_eps, a.u1, a.mean1, a.rstd1));
  GemmArgs g = gemm_args();
  g.A = a.u1; g.a_dt = dt; g.a_sm = D; g.a_sk = 1;
  g.B = wptr(p.qkv_w); g.b_dt = wdt(); g.b_sk = 3 * D; g.b_sn = 1;
  g.C = a.qkv; g.c_dt = dt; g.ldc = 3 * D; g.M = M; g.N = 3 * D; g.K = D; g.bias = params + p.qkv_b;
  PPLL_TRY(launch_gemm(s, g));
  PPLL_TRY(launch_attention_fwd(s, a.qkv, dt, cfg.batch, T, H, D / H, a.att, a.lse));
  g = gemm_args();
  g.A = a.att; g.a_dt = dt; g.a_sm = D; g.a_sk = 1;
  g.B = wptr(p.proj_w); g.b_dt = wdt(); g.b_sk = D; g.b_sn = 1;
  g.C = a.x1; g.c_dt = dt; g.ldc = D; g.M = M; g.N = D; g.K = D; g.bias = params + p.proj_b;
  g.residual = x; g.r_dt = dt; g.ldr = D;
  PPLL_TRY(launch_gemm(s, g));
  PPLL_TRY(launch_layernorm_fwd(s, a.x1, dt, D, M, D, params + p.ln2_g, params + p.ln2_b, cfg.ln_eps, a.u2, a.mean2, a.rstd2));
  g = gemm_args();
  g.A = a.u2; g.a_dt = dt; g.a_sm = D; g.a_sk = 1;
  g.B = wptr(p.fc1_w); g.b_dt = wdt(); g.b_sk = F; g.b_sn = 1;
  g.C = a.h; g.c_dt = dt; g.ldc = F; g.M = M; g.N = F; g.K = D; g.bias = params + p.fc1_b;
  g.epilogue = EPI_GELU; g.C2 = a.gl;
  PPLL_TRY(launch_gemm(s, g));
  g = gemm_args();
  g.A = a.gl; g.a_dt = dt; g.a_sm = F; g.a_sk = 1;
  g.B = wptr(p.fc2_w); g.b_dt = wdt(); g.b_sk = D; g.b_sn = 1;
  g.C = x2_out; g.c_dt = dt; g.ldc = D; g.M = M; g.N = D; g.K = F; g.bias = params + p.fc2_b;
  g.residual = a.x1; g.r_dt = dt; g.ldr = D;
  return launch_gemm(s, g);
}

// g_in: gradient w.r.t. the layer output; g_tmp receives the gradient at the
// mid-layer residual; g_out the gradient w.r.t. the layer input.
int Block::encoder_bwd(int l, const void* x, const void* g_in, void* g_tmp, void* g_out, bool need_dx, hipStream_t s) {
  const int D = cfg.dim, F = cfg.mlp_dim, T = cfg.tokens, H = cfg.heads, M = cfg.batch * T;
  const EncoderParams& p = enc_p[l];
  EncoderActs& a = enc_a[l];
  // dY W^T with W stored [in,out]:  B(k = out index, n = in index) = W[n*out + k]
  auto dgrad = [&](const void* dy, int out_dim, size_t w_off, int in_dim, void* dxo) {
    GemmArgs g = gemm_args();
    g.A = dy; g.a_dt = dt; g.a_sm = out_dim; g.a_sk = 1;
    g.B = wptr(w_off); g.b_dt = wdt(); g.b_sk = 1; g.b_sn = out_dim;
    g.C = dxo; g.c_dt = dt; g.ldc = in_dim; g.M = M; g.N = in_dim; g.K = out_dim;
    return g;
  };
  // dW[in,out] = X^T dY and db = column sums of dY, reduction over the M rows.  Nothing in the
  // backward chain reads them, so the products are only recorded here (their operands stay
  // untouched until the end of the pass: every layer has its own gradient buffers) and all of
  // them run as one grouped launch after the last layer: together they have enough output tiles
  // to fill the chip without splitting K.  A product the MFMA kernel cannot take runs at once.
  void* d_h = this->d_h[l];
  void* d_qkv = this->d_qkv[l];
  auto wgrad = [&](const void* xin, int in_dim, const void* dy, int out_dim, size_t w_off, size_t b_off) -> int {
    return wgrad_product(xin, in_dim, in_dim, dy, out_dim, out_dim, M, grads + w_off, out_dim, grads + b_off, s);
  };
  GemmArgs g = dgrad(g_in, D, p.fc2_w, F, d_h);
  g.epilogue = EPI_DGELU; g.aux = a.h; g.aux_dt = dt; g.ldaux = F;
  PPLL_TRY(launch_gemm(s, g));
  PPLL_TRY(wgrad(a.gl, F, g_in, D, p.fc2_w, p.fc2_b));
  PPLL_TRY(launch_gemm(s, dgrad(d_h, F, p.fc1_w, D, d_u)));
  PPLL_TRY(wgrad(a.u2, D, d_h, F, p.fc1_w, p.fc1_b));
  PPLL_TRY(launch_layernorm_bwd(s, d_u, a.x1, dt, D, M, D, params + p.ln2_g, a.mean2, a.rstd2, g_in, g_tmp, rq,
                                grads + p.ln2_g, grads + p.ln2_b));
  PPLL_TRY(launch_gemm(s, dgrad(g_tmp, D, p.proj_w, D, d_u)));
  PPLL_TRY(wgrad(a.att, D, g_tmp, D, p.proj_w, p.proj_b));
  PPLL_TRY(launch_attention_bwd(s, a.qkv, a.att, d_u, a.lse, dt, cfg.batch, T, H, D / H, d_qkv));
  PPLL_TRY(launch_gemm(s, dgrad(d_qkv, 3 * D, p.qkv_w, D, d_u)));
  PPLL_TRY(wgrad(a.u1, D, d_qkv, 3 * D, p.qkv_w, p.qkv_b));
  return launch_layernorm_bwd(s, d_u, x, dt, D, M, D, params + p.ln1_g, a.mean1, a.rstd1, g_tmp,
                              need_dx ? g_out : nullptr, rq, grads + p.ln1_g, grads + p.ln1_b);
}

int Block::wgrad_product(const void* xin, long x_ld, int in_dim, const void* dy, long dy_ld, int out_dim, int K, float* dW,
                         long ldw, float* db, hipStream_t s) {
  GemmArgs g = gemm_args();
  g.A = xin; g.a_dt = dt; g.a_sm = 1; g.a_sk = x_ld;
  g.B = dy; g.b_dt = dt; g.b_sk = dy_ld; g.b_sn = 1;
  g.C = dW; g.c_dt = F32; g.ldc = ldw; g.M = in_dim; g.N = out_dim; g.K = K;
  g.colsum = db;
  g.splitk_ws = splitk; g.splitk_floats = splitk_floats;
  if (gemm_mfma_groupable(g)) { wgrad_jobs.push_back(g); return PPLL_OK; }
  g.colsum = nullptr;
  PPLL_TRY(launch_gemm(s, g));
  if (dy_ld != out_dim) { set_error("bias gradient of a strided product needs the matrix-core kernel"); return PPLL_ERR_CONFIG; }
  return launch_colsum(s, dy, dt, K, out_dim, rq, db);
}

// Last auxiliary layer, class-token row only.  The keys and values need every token (LayerNorm 1 and the K, V columns of
// the QKV projection run over all B*T rows); the query, the attention output, the output projection, LayerNorm 2 and
// the MLP are needed for the B class-token rows alone, because only those rows of the layer output reach the head.
// a.qkv holds [B*T, 2D] keys and values here, cls_a the compact [B, .] tensors; the layer output is cls_a.x2 [B, D].
int Block::encoder_fwd_cls(int l, const void* x, hipStream_t s) {
  const int D = cfg.dim, F = cfg.mlp_dim, T = cfg.tokens, H = cfg.heads, B = cfg.batch, M = B * T;
  const EncoderParams& p = enc_p[l];
  const EncoderActs& a = enc_a[l];
  const ClsActs& c = cls_a;
  const size_t wsz = dtype_size(wdt());
  PPLL_TRY(launch_layernorm_fwd(s, x, dt, D, M, D, params + p.ln1_g, params + p.ln1_b, cfg.ln_eps, a.u1, a.mean1, a.rstd1));
  GemmArgs g = gemm_args();   // keys and values of all tokens: columns D..3D of the QKV weight
  g.A = a.u1; g.a_dt = dt; g.a_sm = D; g.a_sk = 1;
  g.B = (const char*)wptr(p.qkv_w) + (size_t)D * wsz; g.b_dt = wdt(); g.b_sk = 3 * D; g.b_sn = 1;
  g.C = a.qkv; g.c_dt = dt; g.ldc = 2 * D; g.M = M; g.N = 2 * D; g.K = D; g.bias = params + p.qkv_b + D;
  PPLL_TRY(launch_gemm(s, g));
  g = gemm_args();            // query of the class token (row b*T of u1)
  g.A = a.u1; g.a_dt = dt; g.a_sm = (long)T * D; g.a_sk = 1;
  g.B = wptr(p.qkv_w); g.b_dt = wdt(); g.b_sk = 3 * D; g.b_sn = 1;
  g.C = c.q; g.c_dt = dt; g.ldc = D; g.M = B; g.N = D; g.K = D; g.bias = params + p.qkv_b;
  PPLL_TRY(launch_gemm(s, g));
  PPLL_TRY(launch_attention_cls_fwd(s, c.q, a.qkv, dt, B, T, H, D / H, c.att, c.prob));
  g = gemm_args();
  g.A = c.att; g.a_dt = dt; g.a_sm = D; g.a_sk = 1;
  g.B = wptr(p.proj_w); g.b_dt = wdt(); g.b_sk = D; g.b_sn = 1;
  g.C = c.x1; g.c_dt = dt; g.ldc = D; g.M = B; g.N = D; g.K = D; g.bias = params + p.proj_b;
  g.residual = x; g.r_dt = dt; g.ldr = (long)T * D;
  PPLL_TRY(launch_gemm(s, g));
  PPLL_TRY(launch_layernorm_fwd(s, c.x1, dt, D, B, D, params + p.ln2_g, params + p.ln2_b, cfg.ln_eps, c.u2, c.mean2, c.rstd2));
  g = gemm_args();
  g.A = c.u2; g.a_dt = dt; g.a_sm = D; g.a_sk = 1;
  g.B = wptr(p.fc1_w); g.b_dt = wdt(); g.b_sk = F; g.b_sn = 1;
  g.C = c.h; g.c_dt = dt; g.ldc = F; g.M = B; g.N = F; g.K = D; g.bias = params + p.fc1_b;
  g.epilogue = EPI_GELU; g.C2 = c.gl;
  PPLL_TRY(launch_gemm(s, g));
  g = gemm_args();
  g.A = c.gl; g.a_dt = dt; g.a_sm = F; g.a_sk = 1;
  g.B = wptr(p.fc2_w); g.b_dt = wdt(); g.b_sk = D; g.b_sn = 1;
  g.C = c.x2; g.c_dt = dt; g.ldc = D; g.M = B; g.N = D; g.K = F; g.bias = params + p.fc2_b;
  g.residual = c.x1; g.r_dt = dt; g.ldr = D;
  return launch_gemm(s, g);
}

// d_x2 [B, D]: gradient with respect to the class-token rows of the layer output; g_out [B*T, D] receives the gradient
// with respect to the layer input (all rows: the keys and values depend on every token).
int Block::encoder_bwd_cls(int l, const void* x, const void* d_x2, void* g_out, hipStream_t s) {
  const int D = cfg.dim, F = cfg.mlp_dim, T = cfg.tokens, H = cfg.heads, B = cfg.batch, M = B * T;
  const EncoderParams& p = enc_p[l];
  const EncoderActs& a = enc_a[l];
  const ClsActs& c = cls_a;
  const size_t wsz = dtype_size(wdt());
  void* d_kv = d_qkv[l];      // [B*T, 2D] here
  auto dgrad = [&](const void* dy, int rows, int out_dim, const void* w, long w_ld, int in_dim, void* dxo) {
    GemmArgs g = gemm_args();   // dY W^T with W rows w_ld apart:  B(k = out index, n = in index) = w[n*w_ld + k]
    g.A = dy; g.a_dt = dt; g.a_sm = out_dim; g.a_sk = 1;
    g.B = w; g.b_dt = wdt(); g.b_sk = 1; g.b_sn = w_ld;
    g.C = dxo; g.c_dt = dt; g.ldc = in_dim; g.M = rows; g.N = in_dim; g.K = out_dim;
    return g;
  };
  GemmArgs g = dgrad(d_x2, B, D, wptr(p.fc2_w), D, F, c.d_h);
  g.epilogue = EPI_DGELU; g.aux = c.h; g.aux_dt = dt; g.ldaux = F;
  PPLL_TRY(launch_gemm(s, g));
  PPLL_TRY(wgrad_product(c.gl, F, F, d_x2, D, D, B, grads + p.fc2_w, D, grads + p.fc2_b, s));
  PPLL_TRY(launch_gemm(s, dgrad(c.d_h, B, F, wptr(p.fc1_w), F, D, c.d_u2)));
  PPLL_TRY(wgrad_product(c.u2, D, D, c.d_h, F, F, B, grads + p.fc1_w, F, grads + p.fc1_b, s));
  PPLL_TRY(launch_layernorm_bwd(s, c.d_u2, c.x1, dt, D, B, D, params + p.ln2_g, c.mean2, c.rstd2, d_x2, c.d_x1, rq,
                                grads + p.ln2_g, grads + p.ln2_b));
  PPLL_TRY(launch_gemm(s, dgrad(c.d_x1, B, D, wptr(p.proj_w), D, D, c.d_att)));
  PPLL_TRY(wgrad_product(c.att, D, D, c.d_x1, D, D, B, grads + p.proj_w, D, grads + p.proj_b, s));
  PPLL_TRY(launch_attention_cls_bwd(s, c.q, a.qkv, c.prob, c.d_att, dt, B, T, H, D / H, c.d_q, d_kv));
  // gradient at LayerNorm 1's output: keys and values of all rows, plus the query's share on the class-token rows
  PPLL_TRY(launch_gemm(s, dgrad(d_kv, M, 2 * D, (const char*)wptr(p.qkv_w) + (size_t)D * wsz, 3 * D, D, d_u)));
  g = dgrad(c.d_q, B, D, wptr(p.qkv_w), 3 * D, D, d_u);
  g.ldc = (long)T * D;
  g.residual = d_u; g.r_dt = dt; g.ldr = (long)T * D;     // added to what the product above left in those rows
  PPLL_TRY(launch_gemm(s, g));
  PPLL_TRY(wgrad_product(a.u1, D, D, d_kv, 2 * D, 2 * D, M, grads + p.qkv_w + D, 3 * D, grads + p.qkv_b + D, s));
  PPLL_TRY(wgrad_product(a.u1, (long)T * D, D, c.d_q, D, D, B, grads + p.qkv_w, 3 * D, grads + p.qkv_b, s));
  PPLL_TRY(launch_layernorm_bwd(s, d_u, x, dt, D, M, D, params + p.ln1_g, a.mean1, a.rstd1, nullptr, g_out, rq,
                                grads + p.ln1_g, grads + p.ln1_b));
  // the residual path around the attention block carries d_x1, which lives on the class-token rows only
  return launch_add_rows(s, g_out, (long)T * D, c.d_x1, B, D, dt);
}

int Block::vit_step(const void* x_in, const int32_t* labels, void* x_out, hipStream_t s,
                    const std::function<int()>& after_forward) {
  const int B = cfg.batch, D = cfg.dim, T = cfg.tokens, C = cfg.num_classes, M = B * T;
  const int L = cfg.depth, A = cfg.aux_depth;
  const bool image = cfg.input_kind == PPLL_IN_IMAGE;
  const int ppc = cfg.patch * cfg.patch * cfg.img_c;
  std::vector<const void*> layer_in(L + A);
  // ---- module forward
  const void* x = x_in;
  if (image) {
    PPLL_TRY(launch_patchify(s, x_in, dt, B, cfg.img_h, cfg.img_w, cfg.img_c, cfg.patch, patches));
    GemmArgs g = gemm_args();
    g.A = patches; g.a_dt = dt; g.a_sm = ppc; g.a_sk = 1;
    g.B = wptr(pe_w); g.b_dt = wdt(); g.b_sk = D; g.b_sn = 1;
    g.C = embed_tmp; g.c_dt = dt; g.ldc = D; g.M = B * (T - 1); g.N = D; g.K = ppc; g.bias = params + pe_b;
    if (T > 1) PPLL_TRY(launch_gemm(s, g));
    PPLL_TRY(launch_assemble_tokens(s, embed_tmp, dt, params + cls, params + pos, B, T, D, x0));
    x = x0;
  }
  for (int l = 0; l < L; ++l) {
    layer_in[l] = x;
    void* dst = l == L - 1 ? x_out : enc_a[l].x2;
    PPLL_TRY(encoder_fwd(l, enc_a[l], x, dst, s));
    x = dst;
  }
  PPLL_TRY(mark_phase(1, s));   // module forward done
  if (after_forward) PPLL_TRY(after_forward());
  // ---- auxiliary forward
  long head_xs = (long)T * D;   // distance between the class-token rows the head reads
  for (int l = L; l < L + A; ++l) {
    layer_in[l] = x;
    if (prune_cls && l == L + A - 1) {
      PPLL_TRY(encoder_fwd_cls(l, x, s));
      x = cls_a.x2;
      head_xs = D;
    } else {
      PPLL_TRY(encoder_fwd(l, enc_a[l], x, enc_a[l].x2, s));
      x = enc_a[l].x2;
    }
  }
  GemmArgs g = gemm_args();
  if (vit_head_fused_ok(D, C)) {
    // ---- auxiliary head, local loss and the head's backward in one launch
    PPLL_TRY(launch_vit_head(s, x, dt, head_xs, B, D, C, params + head_ln_g, params + head_ln_b, cfg.ln_eps,
                             params + head_w, params + head_b, labels, dcls, rq, grads + head_ln_g, grads + head_ln_b,
                             grads + head_w, grads + head_b, loss_dev, loss_copy, flag_dev));
  } else {
    PPLL_TRY(launch_layernorm_fwd(s, x, dt, head_xs, B, D, params + head_ln_g, params + head_ln_b, cfg.ln_eps, z,
                                  head_mean, head_rstd));
    g = gemm_args();
    g.A = z; g.a_dt = dt; g.a_sm = D; g.a_sk = 1;
    g.B = params + head_w; g.b_dt = F32; g.b_sk = C; g.b_sn = 1;
    g.C = logits; g.c_dt = F32; g.ldc = C; g.M = B; g.N = C; g.K = D; g.bias = params + head_b;
    PPLL_TRY(launch_gemm_generic(s, g));
    // ---- local loss
    PPLL_TRY(launch_cross_entropy(s, logits, labels, B, C, loss_dev, loss_copy, dlogits, grads + head_b, flag_dev));
    // ---- backward: head
    g = gemm_args();
    g.A = z; g.a_dt = dt; g.a_sm = 1; g.a_sk = D;
    g.B = dlogits; g.b_dt = F32; g.b_sk = C; g.b_sn = 1;
    g.C = grads + head_w; g.c_dt = F32; g.ldc = C; g.M = D; g.N = C; g.K = B;
    PPLL_TRY(launch_gemm_generic(s, g));
    g = gemm_args();
    g.A = dlogits; g.a_dt = F32; g.a_sm = C; g.a_sk = 1;
    g.B = params + head_w; g.b_dt = F32; g.b_sk = 1; g.b_sn = C;
    g.C = dz; g.c_dt = dt; g.ldc = D; g.M = B; g.N = D; g.K = C;
    PPLL_TRY(launch_gemm_generic(s, g));
    PPLL_TRY(launch_layernorm_bwd(s, dz, x, dt, head_xs, B, D, params + head_ln_g, head_mean, head_rstd, nullptr, dcls,
                                  rq, grads + head_ln_g, grads + head_ln_b));
  }
  PPLL_TRY(mark_phase(2, s));   // auxiliary forward and loss done (the fused head kernel has also run its own backward)
  wgrad_jobs.clear();
  const bool pruned = prune_cls && A >= 1;
  if (!pruned) PPLL_TRY(launch_scatter_cls(s, dcls, dt, B, T, D, g_res[L + A]));
  // ---- backward: auxiliary layers then module layers; the chain stops at x_in
  for (int l = L + A - 1; l >= 0; --l) {
    bool need_dx = l > 0 || image;
    const size_t first_job = wgrad_jobs.size();
    if (pruned && l == L + A - 1) PPLL_TRY(encoder_bwd_cls(l, layer_in[l], dcls, g_res[l], s));
    else PPLL_TRY(encoder_bwd(l, layer_in[l], g_res[l + 1], g_mid[l], g_res[l], need_dx, s));
    // A layer whose weight-gradient products fill the chip on their own (SIDE_MIN_TILES output tiles) has them run
    // beside the backward of the layers below, where they take up the slots that the chain's ragged last rounds of
    // workgroups leave empty (measured: 5 % of the step at width 768 and 197 tokens).  Smaller sets only slow the
    // chain down (measured at width 384: 2 to 8 % slower), so they wait for the grouped launch at the end.
    // (not while launches are being timed one by one: overlapping kernels would stretch each other's brackets)
    if (use_side && !profile_enabled() && l > 0 && M >= SIDE_MIN_ROWS && gemm_group_in_one_launch(wgrad_jobs.data(), (int)wgrad_jobs.size())) {
      long tiles = 0;
      for (size_t j = first_job; j < wgrad_jobs.size(); ++j)
        tiles += (long)((wgrad_jobs[j].M + 127) / 128) * ((wgrad_jobs[j].N + 127) / 128);
      if (tiles >= SIDE_MIN_TILES) PPLL_TRY(side_launch_wgrads(s));
    }
  }
  if (image) {
    PPLL_TRY(launch_embed_bwd(s, g_res[0], dt, B, T, D, rq, grads + pos, grads + cls, embed_tmp));
    if (T > 1) {
      g = gemm_args();
      g.A = patches; g.a_dt = dt; g.a_sm = 1; g.a_sk = ppc;
      g.B = embed_tmp; g.b_dt = dt; g.b_sk = D; g.b_sn = 1;
      g.C = grads + pe_w; g.c_dt = F32; g.ldc = D; g.M = ppc; g.N = D; g.K = B * (T - 1);
      g.colsum = grads + pe_b;   // bias gradient: column sums of dE, folded into the product by the MFMA kernel
      g.splitk_ws = splitk; g.splitk_floats = splitk_floats;
      if (gemm_mfma_groupable(g)) {
        wgrad_jobs.push_back(g);
      } else {
        g.colsum = nullptr;
        PPLL_TRY(launch_gemm(s, g));
        PPLL_TRY(launch_colsum(s, embed_tmp, dt, B * (T - 1), D, rq, grads + pe_b));
      }
    } else {
      PPLL_TRY(launch_fill_zero(s, grads + pe_w, ((size_t)ppc * D + D) * sizeof(float)));
    }
  }
  // ---- every recorded weight-gradient product: one launch, or one by one with split-K for a small set
  // (this launch is the only user of the split-K scratch while it runs: the side stream's launches take none)
  PPLL_TRY(launch_gemm_group(s, wgrad_jobs.data(), (int)wgrad_jobs.size(), side_busy, true));
  wgrad_jobs.clear();
  PPLL_TRY(side_wait(s));
  return PPLL_OK;
}

// ------------------------------------------------------------------ ResNet
// stem convolution img_c -> in_c into stem_c
int Block::stem_conv_fwd(const void* x_in, void* xp, void* wp, void* out, hipStream_t s, float* stat, int* stat_blocks) {
  const int B = cfg.batch;
  if (!stem_pad)
    return launch_conv3x3_fwd(s, x_in, wptr(stem_w), wdt(), dt, B, in_h, in_w, cfg.img_c, in_c, 1, out, stat, stat_blocks);
  PPLL_TRY(launch_pad_channels16(s, x_in, (size_t)B * in_h * in_w, cfg.img_c, xp));
  PPLL_TRY(launch_pad_filter16(s, params + stem_w, cfg.img_c, in_c, wp));
  return launch_conv3x3_fwd(s, xp, wp, BF16, dt, B, in_h, in_w, 16, in_c, 1, out, stat, stat_blocks);
}

int Block::resnet_step(const void* x_in, const int32_t* labels, void* x_out, hipStream_t s,
                       const std::function<int()>& after_forward) {
  const int B = cfg.batch, Ch = cfg.channels, A = cfg.aux_channels, H = cfg.height, W = cfg.width;
  const int C = cfg.num_classes, n = cfg.n_basic_blocks;
  const int Ho = (H - 1) / 2 + 1, Wo = (W - 1) / 2 + 1, arows = B * Ho * Wo;
  const float eps = cfg.bn_eps, mom = cfg.bn_momentum;
  auto run_mean = [&](int i) { return bn_mean_run + bn_off[i]; };
  auto run_var = [&](int i) { return bn_var_run + bn_off[i]; };
  std::vector<const void*> block_in(n);
  std::vector<void*> block_out(n);
  const void* x = x_in;
  if (stem) {
    const int rows0 = B * in_h * in_w;
    int ready = 0;   // partial rows of the BatchNorm sums that the convolution has written itself
    PPLL_TRY(stem_conv_fwd(x_in, stem_xp, stem_wp, stem_c, s, partials, &ready));
    PPLL_TRY(launch_bn_train_fwd(s, stem_c, dt, rows0, in_c, eps, mom, partials, stem_mean, stem_rstd, run_mean(0), run_var(0),
                                 params + stem_g, params + stem_b, nullptr, stem_y, ready));
    x = stem_y;
  }
  for (int i = 0; i < n; ++i) {
    const BasicBlockParams& p = rb_p[i];
    const BasicBlockDims& d = rb_d[i];
    BasicBlockActs& a = rb_a[i];
    const int rows = B * d.Ho * d.Wo, b1 = bn_base + 2 * i, b2 = b1 + 1;
    block_in[i] = x;
    block_out[i] = i == n - 1 ? x_out : a.out;
    int ready = 0;
    PPLL_TRY(launch_conv3x3_fwd(s, x, wptr(p.conv1_w), wdt(), dt, B, d.Hin, d.Win, d.Ci, d.Co, d.stride, a.c1, partials, &ready));
    PPLL_TRY(launch_bn_train_fwd(s, a.c1, dt, rows, d.Co, eps, mom, partials, a.mean1, a.rstd1, run_mean(b1), run_var(b1),
                                 params + p.bn1_g, params + p.bn1_b, nullptr, a.y1, ready));
    PPLL_TRY(launch_conv3x3_fwd(s, a.y1, wptr(p.conv2_w), wdt(), dt, B, d.Ho, d.Wo, d.Co, d.Co, 1, a.c2, partials, &ready));
    const void* skip = x;
    if (d.stride != 1 || d.Ci != d.Co) {
      PPLL_TRY(launch_shortcut_fwd(s, x, dt, B, d.Hin, d.Win, d.Ci, d.Co, d.stride, shortcut));
      skip = shortcut;
    }
    PPLL_TRY(launch_bn_train_fwd(s, a.c2, dt, rows, d.Co, eps, mom, partials, a.mean2, a.rstd2, run_mean(b2), run_var(b2),
                                 params + p.bn2_g, params + p.bn2_b, skip, block_out[i], ready));
    x = block_out[i];
  }
  PPLL_TRY(mark_phase(1, s));   // module forward done
  if (after_forward) PPLL_TRY(after_forward());
  // ---- auxiliary forward
  const int ba = bn_base + 2 * n;
  int aux_ready = 0;
  PPLL_TRY(launch_conv3x3_fwd(s, x, wptr(aux_conv_w), wdt(), dt, B, H, W, Ch, A, 2, aux_c, partials, &aux_ready));
  PPLL_TRY(launch_bn_train_fwd(s, aux_c, dt, arows, A, eps, mom, partials, aux_mean, aux_rstd, run_mean(ba), run_var(ba),
                               params + aux_bn_g, params + aux_bn_b, nullptr, aux_y, aux_ready));
  PPLL_TRY(launch_gap_fwd(s, aux_y, dt, B, Ho * Wo, A, pooled));
  if (vit_head_fused_ok(A, C)) {
    // ---- Linear head, local loss and the head's backward in one launch (the fused head without a LayerNorm)
    PPLL_TRY(launch_vit_head(s, pooled, dt, (long)A, B, A, C, nullptr, nullptr, 0.f, params + head_w, params + head_b, labels,
                             dpooled, rq, nullptr, nullptr, grads + head_w, grads + head_b, loss_dev, loss_copy, flag_dev));
    PPLL_TRY(mark_phase(2, s));   // auxiliary forward and loss done
  } else {
    GemmArgs g = gemm_args();
    g.A = pooled; g.a_dt = dt; g.a_sm = A; g.a_sk = 1;
    g.B = params + head_w; g.b_dt = F32; g.b_sk = C; g.b_sn = 1;
    g.C = logits; g.c_dt = F32; g.ldc = C; g.M = B; g.N = C; g.K = A; g.bias = params + head_b;
    PPLL_TRY(launch_gemm_generic(s, g));
    PPLL_TRY(launch_cross_entropy(s, logits, labels, B, C, loss_dev, loss_copy, dlogits, grads + head_b, flag_dev));
    PPLL_TRY(mark_phase(2, s));   // auxiliary forward and loss done
    // ---- backward: head
    g = gemm_args();
    g.A = pooled; g.a_dt = dt; g.a_sm = 1; g.a_sk = A;
    g.B = dlogits; g.b_dt = F32; g.b_sk = C; g.b_sn = 1;
    g.C = grads + head_w; g.c_dt = F32; g.ldc = C; g.M = A; g.N = C; g.K = B;
    PPLL_TRY(launch_gemm_generic(s, g));
    g = gemm_args();
    g.A = dlogits; g.a_dt = F32; g.a_sm = C; g.a_sk = 1;
    g.B = params + head_w; g.b_dt = F32; g.b_sk = 1; g.b_sn = C;
    g.C = dpooled; g.c_dt = dt; g.ldc = A; g.M = B; g.N = A; g.K = C;
    PPLL_TRY(launch_gemm_generic(s, g));
  }
  // ---- backward: auxiliary net
  PPLL_TRY(launch_gap_bwd(s, dpooled, dt, B, Ho * Wo, A, d_aux));
  PPLL_TRY(launch_bn_bwd(s, d_aux, aux_y, aux_c, dt, arows, A, aux_mean, aux_rstd, params + aux_bn_g, partials,
                         grads + aux_bn_g, grads + aux_bn_b, d_aux));
  PPLL_TRY(launch_conv3x3_wgrad(s, x, d_aux, dt, B, H, W, Ch, A, 2, rq, grads + aux_conv_w));
  void *gcur = r_gA, *gnext = r_gB;   // gradient with respect to the output of the block in hand / of the one before it
  PPLL_TRY(launch_conv3x3_dgrad(s, d_aux, wptr(aux_conv_w), wdt(), dt, B, H, W, Ch, A, 2, nullptr, nullptr, gcur));
  // ---- backward: basic blocks, last to first; nothing is produced for x_in.  The weight gradients wait:
  // those of one shape run as one launch after the loop.
  struct Shape { int H, W, Ci, Co, stride; };
  std::vector<Shape> shapes;
  std::vector<std::vector<ConvWgradJob>> shape_jobs;
  auto defer = [&](const void* xin, const void* dyp, float* dw, int Hh, int Ww, int Ci, int Co, int st) {
    size_t k = 0;
    while (k < shapes.size() && !(shapes[k].H == Hh && shapes[k].W == Ww && shapes[k].Ci == Ci && shapes[k].Co == Co && shapes[k].stride == st)) ++k;
    if (k == shapes.size()) { shapes.push_back({Hh, Ww, Ci, Co, st}); shape_jobs.emplace_back(); }
    shape_jobs[k].push_back({xin, dyp, dw});
  };
  // An input-gradient convolution whose result is the output gradient of a BatchNorm also writes that BatchNorm's
  // backward sums where it can (`ready` partial rows in `partials`, consumed by the launch_bn_bwd right behind it).
  int ready = 0;
  for (int i = n - 1; i >= 0; --i) {
    const BasicBlockParams& p = rb_p[i];
    const BasicBlockDims& d = rb_d[i];
    BasicBlockActs& a = rb_a[i];
    const int rows = B * d.Ho * d.Wo;
    PPLL_TRY(launch_bn_bwd(s, gcur, block_out[i], a.c2, dt, rows, d.Co, a.mean2, a.rstd2, params + p.bn2_g, partials,
                           grads + p.bn2_g, grads + p.bn2_b, a.d2, ready));
    ready = 0;
    defer(a.y1, a.d2, grads + p.conv2_w, d.Ho, d.Wo, d.Co, d.Co, 1);
    const BnBwdSums bn1{a.y1, a.c1, a.mean1, a.rstd1, partials};
    PPLL_TRY(launch_conv3x3_dgrad(s, a.d2, wptr(p.conv2_w), wdt(), dt, B, d.Ho, d.Wo, d.Co, d.Co, 1, nullptr, nullptr, r_t1, &bn1,
                                  &ready));
    PPLL_TRY(launch_bn_bwd(s, r_t1, a.y1, a.c1, dt, rows, d.Co, a.mean1, a.rstd1, params + p.bn1_g, partials,
                           grads + p.bn1_g, grads + p.bn1_b, a.d1, ready));
    ready = 0;
    defer(block_in[i], a.d1, grads + p.conv1_w, d.Hin, d.Win, d.Ci, d.Co, d.stride);
    if (i == 0 && !stem) break;   // the block input is the detached x_{j-1}
    if (d.stride == 1 && d.Ci == d.Co) {   // identity shortcut folded into the input gradient
      // the result is the output gradient of the second BatchNorm of the block before
      BnBwdSums bn2{};
      if (i > 0) bn2 = BnBwdSums{block_out[i - 1], rb_a[i - 1].c2, rb_a[i - 1].mean2, rb_a[i - 1].rstd2, partials};
      PPLL_TRY(launch_conv3x3_dgrad(s, a.d1, wptr(p.conv1_w), wdt(), dt, B, d.Hin, d.Win, d.Ci, d.Co, 1, gcur, block_out[i], gcur,
                                    i > 0 ? &bn2 : nullptr, &ready));
    } else {
      PPLL_TRY(launch_conv3x3_dgrad(s, a.d1, wptr(p.conv1_w), wdt(), dt, B, d.Hin, d.Win, d.Ci, d.Co, d.stride, nullptr, nullptr,
                                    gnext));
      PPLL_TRY(launch_shortcut_bwd(s, gcur, block_out[i], dt, B, d.Hin, d.Win, d.Ci, d.Co, d.stride, gnext));
      std::swap(gcur, gnext);
    }
  }
  for (size_t k = 0; k < shapes.size(); ++k)
    PPLL_TRY(launch_conv3x3_wgrad_group(s, shape_jobs[k].data(), (int)shape_jobs[k].size(), dt, B, shapes[k].H, shapes[k].W,
                                        shapes[k].Ci, shapes[k].Co, shapes[k].stride, rq));
  if (stem) {
    const int rows0 = B * in_h * in_w;
    PPLL_TRY(launch_bn_bwd(s, gcur, stem_y, stem_c, dt, rows0, in_c, stem_mean, stem_rstd, params + stem_g, partials,
                           grads + stem_g, grads + stem_b, r_t1));
    if (stem_pad)   // the padded image is still in place from the forward pass
      PPLL_TRY(launch_conv3x3_wgrad(s, stem_xp, r_t1, dt, B, in_h, in_w, 16, in_c, 1, rq, grads + stem_w, cfg.img_c));
    else
      PPLL_TRY(launch_conv3x3_wgrad(s, x_in, r_t1, dt, B, in_h, in_w, cfg.img_c, in_c, 1, rq, grads + stem_w));
  }
  return PPLL_OK;
}

// ------------------------------------------------------------------ update
int Block::update(float lr, hipStream_t s) {
  ++steps;
  if (cfg.optimizer == PPLL_SGD)
    return launch_sgd(s, params, grads, mom1, shadow, P, lr, cfg.momentum, cfg.nesterov, cfg.weight_decay, steps == 1);
  float bc1 = (float)(1.0 - std::pow((double)cfg.beta1, (double)steps));
  float bc2 = (float)(1.0 - std::pow((double)cfg.beta2, (double)steps));
  return launch_adamw(s, params, grads, mom1, mom2, shadow, P, lr, cfg.beta1, cfg.beta2, cfg.adam_eps, cfg.weight_decay, bc1, bc2);
}

int Block::forward_eval(const void* x_in, void* x_out, float* logits_out, hipStream_t s) {
  EvalBuffers e;
  e.per_layer = enc_a.data(); e.per_block = rb_a.data();
  e.patches = patches; e.embed_tmp = embed_tmp; e.x0 = x0; e.z = z; e.head_mean = head_mean; e.head_rstd = head_rstd;
  e.stem_c = stem_c; e.stem_y = stem_y; e.stem_xp = stem_xp; e.stem_wp = stem_wp; e.shortcut = shortcut;
  e.aux_c = aux_c; e.aux_y = aux_y; e.pooled = pooled;
  e.stem_mean = stem_mean; e.stem_rstd = stem_rstd; e.aux_mean = aux_mean; e.aux_rstd = aux_rstd;
  return forward_eval_with(e, x_in, x_out, logits_out, s);
}

// One set of activation buffers for all layers, carved from `base` (null: only measure).  Returns the bytes used.
size_t Block::plan_eval_scratch(char* base, EvalBuffers* e) const {
  Bump bump(base);
  const size_t B = (size_t)cfg.batch;
  if (cfg.arch == PPLL_VIT) {
    const size_t D = (size_t)cfg.dim, F = (size_t)cfg.mlp_dim, T = (size_t)cfg.tokens, H = (size_t)cfg.heads, M = B * T;
    if (cfg.input_kind == PPLL_IN_IMAGE) {
      e->patches = bump.take(B * (T - 1) * cfg.patch * cfg.patch * cfg.img_c * esz);
      e->embed_tmp = bump.take(B * (T - 1) * D * esz);
      e->x0 = bump.take(M * D * esz);
    }
    EncoderActs a{};
    a.u1 = bump.take(M * D * esz); a.qkv = bump.take(M * 3 * D * esz); a.att = bump.take(M * D * esz);
    a.x1 = bump.take(M * D * esz); a.u2 = bump.take(M * D * esz);
    a.h = bump.take(M * F * esz); a.gl = bump.take(M * F * esz);
    a.mean1 = bump.floats(M); a.rstd1 = bump.floats(M); a.mean2 = bump.floats(M); a.rstd2 = bump.floats(M);
    a.lse = bump.floats(B * H * T);
    e->shared_enc[0] = a; e->shared_enc[1] = a;
    e->shared_enc[0].x2 = bump.take(M * D * esz);
    e->shared_enc[1].x2 = bump.take(M * D * esz);
    e->z = bump.take(B * D * esz);
    e->head_mean = bump.floats(B); e->head_rstd = bump.floats(B);
  } else {
    const size_t A = (size_t)cfg.aux_channels;
    const size_t Ho = (size_t)(cfg.height - 1) / 2 + 1, Wo = (size_t)(cfg.width - 1) / 2 + 1;
    size_t widest = B * in_h * in_w * in_c;
    int cmax = in_c;
    for (const BasicBlockDims& d : rb_d) {
      const size_t act = B * d.Ho * d.Wo * d.Co;
      if (act > widest) widest = act;
      if (d.Co > cmax) cmax = d.Co;
    }
    if (stem) {
      e->stem_c = bump.take(widest * esz); e->stem_y = bump.take(widest * esz);
      e->stem_mean = bump.floats(in_c); e->stem_rstd = bump.floats(in_c);
      if (stem_pad) {
        e->stem_xp = bump.take(B * in_h * in_w * 16 * esz);
        e->stem_wp = bump.take((size_t)9 * 16 * in_c * esz);
      }
    }
    BasicBlockActs a{};
    a.c1 = bump.take(widest * esz); a.y1 = bump.take(widest * esz); a.c2 = bump.take(widest * esz);
    a.mean1 = bump.floats(cmax); a.rstd1 = bump.floats(cmax); a.mean2 = bump.floats(cmax); a.rstd2 = bump.floats(cmax);
    e->shared_rb[0] = a; e->shared_rb[1] = a;
    e->shared_rb[0].out = bump.take(widest * esz);
    e->shared_rb[1].out = bump.take(widest * esz);
    e->shortcut = bump.take(widest * esz);
    e->aux_c = bump.take(B * Ho * Wo * A * esz); e->aux_y = bump.take(B * Ho * Wo * A * esz);
    e->pooled = bump.take(B * A * esz);
    e->aux_mean = bump.floats(A); e->aux_rstd = bump.floats(A);
  }
  return (bump.off + 255) & ~(size_t)255;
}

int Block::forward_eval_in_scratch(const void* x_in, void* x_out, float* logits_out, hipStream_t s, void* scratch,
                                   size_t scratch_bytes) {
  EvalBuffers e;
  const size_t need = plan_eval_scratch(nullptr, &e);
  if (need > scratch_bytes) {
    set_error("the evaluation forward of this block needs %zu bytes of activation scratch, the built-in buffer holds %zu",
              need, scratch_bytes);
    return PPLL_ERR_WORKSPACE;
  }
  e = EvalBuffers();
  plan_eval_scratch((char*)scratch, &e);
  return forward_eval_with(e, x_in, x_out, logits_out, s);
}

int Block::forward_eval_with(const EvalBuffers& e, const void* x_in, void* x_out, float* logits_out, hipStream_t s) {
  last_stream = s;
  const int B = cfg.batch, C = cfg.num_classes;
  GemmArgs g = gemm_args();
  if (cfg.arch == PPLL_VIT) {
    const int D = cfg.dim, T = cfg.tokens, L = cfg.depth, A = cfg.aux_depth;
    const void* x = x_in;
    if (cfg.input_kind == PPLL_IN_IMAGE) {
      const int ppc = cfg.patch * cfg.patch * cfg.img_c;
      PPLL_TRY(launch_patchify(s, x_in, dt, B, cfg.img_h, cfg.img_w, cfg.img_c, cfg.patch, e.patches));
      g.A = e.patches; g.a_dt = dt; g.a_sm = ppc; g.a_sk = 1;
      g.B = wptr(pe_w); g.b_dt = wdt(); g.b_sk = D; g.b_sn = 1;
      g.C = e.embed_tmp; g.c_dt = dt; g.ldc = D; g.M = B * (T - 1); g.N = D; g.K = ppc; g.bias = params + pe_b;
      if (T > 1) PPLL_TRY(launch_gemm(s, g));
      PPLL_TRY(launch_assemble_tokens(s, e.embed_tmp, dt, params + cls, params + pos, B, T, D, e.x0));
      x = e.x0;
    }
    for (int l = 0; l < L; ++l) {
      void* dst = l == L - 1 ? x_out : e.enc(l).x2;
      PPLL_TRY(encoder_fwd(l, e.enc(l), x, dst, s));
      x = dst;
    }
    if (!logits_out) return PPLL_OK;
    for (int l = L; l < L + A; ++l) {
      PPLL_TRY(encoder_fwd(l, e.enc(l), x, e.enc(l).x2, s));
      x = e.enc(l).x2;
    }
    PPLL_TRY(launch_layernorm_fwd(s, x, dt, (long)T * D, B, D, params + head_ln_g, params + head_ln_b, cfg.ln_eps, e.z,
                                  e.head_mean, e.head_rstd));
    g = gemm_args();
    g.A = e.z; g.a_dt = dt; g.a_sm = D; g.a_sk = 1;
    g.B = params + head_w; g.b_dt = F32; g.b_sk = C; g.b_sn = 1;
    g.C = logits_out; g.c_dt = F32; g.ldc = C; g.M = B; g.N = C; g.K = D; g.bias = params + head_b;
    return launch_gemm_generic(s, g);
  }
  const int Ch = cfg.channels, A = cfg.aux_channels, H = cfg.height, W = cfg.width, n = cfg.n_basic_blocks;
  const int Ho = (H - 1) / 2 + 1, Wo = (W - 1) / 2 + 1, arows = B * Ho * Wo;
  const float eps = cfg.bn_eps;
  const void* x = x_in;
  if (stem) {
    PPLL_TRY(stem_conv_fwd(x_in, e.stem_xp, e.stem_wp, e.stem_c, s));
    PPLL_TRY(launch_bn_running_stats(s, bn_mean_run + bn_off[0], bn_var_run + bn_off[0], in_c, eps, e.stem_mean, e.stem_rstd));
    PPLL_TRY(launch_bn_apply(s, e.stem_c, dt, B * in_h * in_w, in_c, e.stem_mean, e.stem_rstd, params + stem_g, params + stem_b,
                             nullptr, e.stem_y));
    x = e.stem_y;
  }
  for (int i = 0; i < n; ++i) {
    const BasicBlockParams& p = rb_p[i];
    const BasicBlockDims& d = rb_d[i];
    const BasicBlockActs& a = e.rb(i);
    const int rows = B * d.Ho * d.Wo, b1 = bn_base + 2 * i, b2 = b1 + 1;
    void* out = i == n - 1 ? x_out : a.out;
    PPLL_TRY(launch_conv3x3_fwd(s, x, wptr(p.conv1_w), wdt(), dt, B, d.Hin, d.Win, d.Ci, d.Co, d.stride, a.c1));
    PPLL_TRY(launch_bn_running_stats(s, bn_mean_run + bn_off[b1], bn_var_run + bn_off[b1], d.Co, eps, a.mean1, a.rstd1));
    PPLL_TRY(launch_bn_apply(s, a.c1, dt, rows, d.Co, a.mean1, a.rstd1, params + p.bn1_g, params + p.bn1_b, nullptr, a.y1));
    PPLL_TRY(launch_conv3x3_fwd(s, a.y1, wptr(p.conv2_w), wdt(), dt, B, d.Ho, d.Wo, d.Co, d.Co, 1, a.c2));
    PPLL_TRY(launch_bn_running_stats(s, bn_mean_run + bn_off[b2], bn_var_run + bn_off[b2], d.Co, eps, a.mean2, a.rstd2));
    const void* skip = x;
    if (d.stride != 1 || d.Ci != d.Co) {
      PPLL_TRY(launch_shortcut_fwd(s, x, dt, B, d.Hin, d.Win, d.Ci, d.Co, d.stride, e.shortcut));
      skip = e.shortcut;
    }
    PPLL_TRY(launch_bn_apply(s, a.c2, dt, rows, d.Co, a.mean2, a.rstd2, params + p.bn2_g, params + p.bn2_b, skip, out));
    x = out;
  }
  if (!logits_out) return PPLL_OK;
  PPLL_TRY(launch_conv3x3_fwd(s, x, wptr(aux_conv_w), wdt(), dt, B, H, W, Ch, A, 2, e.aux_c));
  PPLL_TRY(launch_bn_running_stats(s, bn_mean_run + bn_off[bn_base + 2 * n], bn_var_run + bn_off[bn_base + 2 * n], A, eps,
                                   e.aux_mean, e.aux_rstd));
  PPLL_TRY(launch_bn_apply(s, e.aux_c, dt, arows, A, e.aux_mean, e.aux_rstd, params + aux_bn_g, params + aux_bn_b, nullptr,
                           e.aux_y));
  PPLL_TRY(launch_gap_fwd(s, e.aux_y, dt, B, Ho * Wo, A, e.pooled));
  g.A = e.pooled; g.a_dt = dt; g.a_sm = A; g.a_sk = 1;
  g.B = params + head_w; g.b_dt = F32; g.b_sk = C; g.b_sn = 1;
  g.C = logits_out; g.c_dt = F32; g.ldc = C; g.M = B; g.N = C; g.K = A; g.bias = params + head_b;
  return launch_gemm_generic(s, g);
}

int Block::side_launch_wgrads(hipStream_t s) {
  if (!side) PPLL_HIP(hipStreamCreateWithFlags(&side, hipStreamNonBlocking));
  if (!side_fork) PPLL_HIP(hipEventCreateWithFlags(&side_fork, hipEventDisableTiming));
  if (!side_join) PPLL_HIP(hipEventCreateWithFlags(&side_join, hipEventDisableTiming));
  PPLL_HIP(hipEventRecord(side_fork, s));
  PPLL_HIP(hipStreamWaitEvent(side, side_fork, 0));
  PPLL_TRY(launch_gemm_group(side, wgrad_jobs.data(), (int)wgrad_jobs.size(), true));
  wgrad_jobs.clear();
  side_busy = true;
  return PPLL_OK;
}

int Block::side_wait(hipStream_t s) {
  if (!side_busy) return PPLL_OK;
  PPLL_HIP(hipEventRecord(side_join, side));
  PPLL_HIP(hipStreamWaitEvent(s, side_join, 0));
  side_busy = false;
  return PPLL_OK;
}

void Block::side_destroy() {
  if (side) { (void)hipStreamSynchronize(side); (void)hipStreamDestroy(side); side = nullptr; }
  if (side_fork) { (void)hipEventDestroy(side_fork); side_fork = nullptr; }
  if (side_join) { (void)hipEventDestroy(side_join); side_join = nullptr; }
}

int Block::mark_phase(int i, hipStream_t s) {
  if (!phase_timers) return PPLL_OK;
  if (!phase_ev[i]) PPLL_HIP(hipEventCreate(&phase_ev[i]));
  PPLL_HIP(hipEventRecord(phase_ev[i], s));
  return PPLL_OK;
}

namespace {
struct TimesBinding {   // binds a block's launch record to this thread for the extent of a step
  explicit TimesBinding(LaunchTimes* t) { profile_bind(t); }
  ~TimesBinding() { profile_bind(nullptr); }
};
}  // namespace

int Block::step(const void* x_in, const int32_t* labels, float lr, void* x_out, float* loss_out, hipStream_t s,
                const std::function<int()>& after_forward) {
  last_stream = s;
  TimesBinding binding(time_launches ? &times : nullptr);
  rq.reset();
  loss_copy = loss_out;   // the loss kernel writes it there as well
  PPLL_TRY(mark_phase(0, s));
  if (cfg.arch == PPLL_VIT) PPLL_TRY(vit_step(x_in, labels, x_out, s, after_forward));
  else PPLL_TRY(resnet_step(x_in, labels, x_out, s, after_forward));
  PPLL_TRY(rq.flush(s));        // the queued second stages of the gradient reductions belong to the backward pass
  PPLL_TRY(mark_phase(3, s));   // backward done (weight gradients included); what follows is the update
  PPLL_TRY(update(lr, s));
  PPLL_TRY(mark_phase(4, s));

  return PPLL_OK;
}

}  // namespace ppll

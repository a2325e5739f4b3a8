// Sliced decoding ("Feature chunk and Sliced Decoding" section): the latent video, batch and frame axes merged, is
// decoded `slice_frames` frames at a time (1 = frame by frame) by a convolutional decoder and the images are
// merged back in frame order; the workspace is sized by the slice, not by the video. The decoder's operators are
// the kernels of the denoising stage: the fused-loader 3x3 convolution (GroupNorm + SiLU applied on the way in,
// residual added on the way out), the GroupNorm statistics kernels, the linear kernels and the spatial attention.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>

#include "../../include/lightcache.h"
#include "lc_internal.h"

using namespace lc;

namespace {

thread_local std::string g_derr = "";
constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct GnP { float *g, *b; };
struct ConvP { void* w; float* b; };

struct DPlan {
  size_t off_a, off_b, off_part, off_scale, off_shift, off_one, off_zero, off_qkv, off_vt, off_ao, total;
};

}  // namespace

struct lc_decoder {
  lc_decoder_config cfg;
  hipStream_t s;
  void* wblob;
  size_t wblob_bytes;
  bool have_weights;
  // packed weights
  float *cin_w, *cin_b;
  GnP res_gn[2 + LC_DEC_MAX_LEVELS]; ConvP res[2 + LC_DEC_MAX_LEVELS];  // mid.res0, mid.res1, up0.res, ...
  GnP at_gn; void *at_wqkv, *at_wo; float* at_bo;
  ConvP upc[LC_DEC_MAX_LEVELS];
  GnP out_gn; ConvP out;
  char* arena;
  size_t arena_bytes;
  std::string err;
};

namespace {

lc_status dfail(lc_decoder* d, lc_status code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (d) d->err = buf; else g_derr = buf;
  return code;
}

#define LCD_HIP(d, expr)                                                                          \
  do {                                                                                            \
    hipError_t e_ = (expr);                                                                       \
    if (e_ != hipSuccess) return dfail(d, LC_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_));   \
  } while (0)

lc_status check_dcfg(lc_decoder* d, const lc_decoder_config* g) {
  if (!g) return dfail(d, LC_ERR_ARG, "config is NULL");
  if (g->dtype != LC_F32 && g->dtype != LC_BF16) return dfail(d, LC_ERR_ARG, "dtype must be LC_F32 or LC_BF16");
  if (g->N <= 0 || g->H <= 0 || g->W <= 0 || g->C_lat <= 0 || g->C_img <= 0 || g->groups <= 0 || g->heads <= 0 ||
      g->head_dim <= 0)
    return dfail(d, LC_ERR_SHAPE, "all sizes must be positive");
  if (g->levels < 0 || g->levels > LC_DEC_MAX_LEVELS) return dfail(d, LC_ERR_SHAPE, "levels must be in [0, %d]", LC_DEC_MAX_LEVELS);
  if (g->C_lat > 16 || g->C_img > 32) return dfail(d, LC_ERR_SHAPE, "C_lat must be <= 16 and C_img <= 32");
  for (int l = 0; l <= g->levels; ++l) {
    const int C = g->widths[l];
    if (C <= 0 || C % 64 || C > 1024) return dfail(d, LC_ERR_SHAPE, "every width must be a multiple of 64, at most 1024");
    if (C % g->groups || C / g->groups > 512) return dfail(d, LC_ERR_SHAPE, "every width must be divisible by groups");
  }
  if (g->heads * g->head_dim != g->widths[0]) return dfail(d, LC_ERR_SHAPE, "heads * head_dim must equal widths[0]");
  const int hd = g->head_dim;
  if (!(hd == 8 || hd == 16 || hd == 32 || hd == 40 || hd == 64))
    return dfail(d, LC_ERR_SHAPE, "head_dim must be one of 8, 16, 32, 40, 64");
  if (!(g->gn_eps > 0.f)) return dfail(d, LC_ERR_SHAPE, "gn_eps must be positive");
  if (((int64_t)g->H << g->levels) * ((int64_t)g->W << g->levels) > (int64_t)1 << 24)
    return dfail(d, LC_ERR_SHAPE, "decoded frames of more than 2^24 pixels are not supported");
  return LC_OK;
}

// Workspace of a pass over `n` frames: two ping-pong fp32 maps that hold the largest map of any stage (the
// upsampled input of the last level's convolution), GroupNorm partial sums and scale / shift, a unit scale and a
// zero shift (the convolution after the upsampling takes its input as it is), and the attention block's q,k,v,
// V^T and output at the latent resolution.
DPlan make_dplan(const lc_decoder_config& g, int n) {
  DPlan p;
  const size_t es = dtype_size(g.dtype);
  const int64_t P0 = (int64_t)g.H * g.W;
  int64_t max_elems = P0 * g.widths[0], max_splits_c = (int64_t)stat_splits((int)P0) * g.widths[0];
  int maxC = g.widths[0];
  int64_t P = P0;
  for (int l = 0; l < g.levels; ++l) {
    P *= 4;
    max_elems = std::max(max_elems, P * std::max(g.widths[l], g.widths[l + 1]));
    max_splits_c = std::max(max_splits_c, (int64_t)stat_splits((int)P) * g.widths[l + 1]);
    maxC = std::max(maxC, g.widths[l + 1]);
  }
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
  p.off_a = take((size_t)n * max_elems * 4);
  p.off_b = take((size_t)n * max_elems * 4);
  p.off_part = take((size_t)n * max_splits_c * 2 * 4);
  p.off_scale = take((size_t)n * maxC * 4);
  p.off_shift = take((size_t)n * maxC * 4);
  p.off_one = take((size_t)n * maxC * 4);
  p.off_zero = take((size_t)n * maxC * 4);
  const int C0 = g.widths[0];
  p.off_qkv = take((size_t)n * P0 * 3 * C0 * es);
  p.off_vt = take((size_t)n * C0 * attn_tp((int)P0) * es);
  p.off_ao = take((size_t)n * P0 * C0 * es);
  p.total = off;
  return p;
}

inline int eff_slice(const lc_decoder_config& g, int slice_frames) {
  return (slice_frames <= 0 || slice_frames > g.N) ? g.N : slice_frames;
}

// scale / shift of GroupNorm(x) for n frames of fp32 rows [rows][C]
lc_status gn(lc_decoder* d, const DPlan& p, const float* x, int n, int rows, int C, const GnP& w) {
  const lc_decoder_config& g = d->cfg;
  float* part = (float*)(d->arena + p.off_part);
  LCD_HIP(d, launch_gn_stats(d->s, kF32, x, part, n, rows, C));
  LCD_HIP(d, launch_gn_finalize(d->s, part, C, stat_splits(rows), rows, 1.f, nullptr, 0, 0, 0, 0.f, w.g, w.b, g.groups, g.gn_eps,
                                (float*)(d->arena + p.off_scale), (float*)(d->arena + p.off_shift), n));
  return LC_OK;
}

// y = [res +] conv3x3(act(x)): src 2 = SiLU(GroupNorm(x)) with the scale / shift at hand, src 1 = x as it is
lc_status conv(lc_decoder* d, const DPlan& p, const ConvP& w, int src, int Cin, int Cout, int n, int H, int W, const float* x,
               const float* res, void* y, int planar, int Cout_store) {
  FusedDesc f;
  memset(&f, 0, sizeof f);
  f.dt = d->cfg.dtype; f.y_f32 = planar ? 0 : 1; f.taps = 9; f.src = src; f.Cin = Cin; f.Cout = Cout; f.Cout_store = Cout_store;
  f.w = w.w; f.bias = w.b; f.frames = n; f.H = H; f.W = W; f.x = x; f.res = res; f.y = y; f.planar_out = planar;
  f.scale = (const float*)(d->arena + (src == 2 ? p.off_scale : p.off_one));
  f.shift = (const float*)(d->arena + (src == 2 ? p.off_shift : p.off_zero));
  f.in_map = f.out_map = RowMap{0, 0, 1 << 30};
  LCD_HIP(d, launch_fused(d->s, f));
  return LC_OK;
}

lc_status res_block(lc_decoder* d, const DPlan& p, int idx, int C, int n, int H, int W, const float* x, float* y) {
  lc_status s = gn(d, p, x, n, H * W, C, d->res_gn[idx]);
  if (s != LC_OK) return s;
  return conv(d, p, d->res[idx], 2, C, C, n, H, W, x, x, y, 0, C);
}

// h += proj(Attn(qkv(GroupNorm(h)))) over the H*W positions of each frame, in place on fp32 rows
lc_status attn_block(lc_decoder* d, const DPlan& p, int n, float* h) {
  const lc_decoder_config& g = d->cfg;
  const int T = g.H * g.W, C = g.widths[0], Tp = attn_tp(T);
  const size_t es = dtype_size(g.dtype);
  lc_status s = gn(d, p, h, n, T, C, d->at_gn);
  if (s != LC_OK) return s;
  char* qkv = d->arena + p.off_qkv;
  char* vt = d->arena + p.off_vt;
  char* ao = d->arena + p.off_ao;
  FusedDesc f;
  memset(&f, 0, sizeof f);
  f.dt = g.dtype; f.y_f32 = 0; f.taps = 1; f.src = 1; f.Cin = C; f.Cout = 3 * C; f.Cout_store = 3 * C; f.w = d->at_wqkv;
  f.rows = (int64_t)n * T; f.in_map = RowMap{0, T, T}; f.out_map = RowMap{0, 0, 1 << 30}; f.x = h; f.y = qkv;
  f.scale = (const float*)(d->arena + p.off_scale); f.shift = (const float*)(d->arena + p.off_shift);
  LCD_HIP(d, launch_fused(d->s, f));
  LCD_HIP(d, launch_make_vt(d->s, g.dtype, qkv + (size_t)2 * C * es, 3 * C, vt, n, T, Tp, C));
  LCD_HIP(d, launch_spatial_attention(d->s, g.dtype, qkv, 3 * C, vt, Tp, ao, n, T, g.heads, g.head_dim, 0, T, 0));
  memset(&f, 0, sizeof f);
  f.dt = g.dtype; f.y_f32 = 1; f.taps = 1; f.src = 0; f.Cin = C; f.Cout = C; f.Cout_store = C; f.w = d->at_wo; f.bias = d->at_bo;
  f.rows = (int64_t)n * T; f.in_map = f.out_map = RowMap{0, 0, 1 << 30}; f.x = ao; f.res = h; f.y = h;
  LCD_HIP(d, launch_fused(d->s, f));
  return LC_OK;
}

// one pass: n frames of latents z -> n decoded images
lc_status decode_pass(lc_decoder* d, const DPlan& p, const void* z, void* img, int n) {
  const lc_decoder_config& g = d->cfg;
  float* a = (float*)(d->arena + p.off_a);
  float* b = (float*)(d->arena + p.off_b);
  int H = g.H, W = g.W;
  const int C0 = g.widths[0];
  LCD_HIP(d, launch_conv_in(d->s, g.dtype, z, a, n, H, W, g.C_lat, C0, d->cin_w, d->cin_b));
  lc_status s = res_block(d, p, 0, C0, n, H, W, a, b);
  if (s != LC_OK) return s;
  if ((s = attn_block(d, p, n, b)) != LC_OK) return s;
  if ((s = res_block(d, p, 1, C0, n, H, W, b, a)) != LC_OK) return s;
  for (int l = 0; l < g.levels; ++l) {  // the map at hand is in `a`
    const int Cl = g.widths[l], Cn = g.widths[l + 1];
    if ((s = res_block(d, p, 2 + l, Cl, n, H, W, a, b)) != LC_OK) return s;
    LCD_HIP(d, launch_up2_rows(d->s, b, a, n, H, W, Cl));
    H *= 2; W *= 2;
    if ((s = conv(d, p, d->upc[l], 1, Cl, Cn, n, H, W, a, nullptr, b, 0, Cn)) != LC_OK) return s;
    std::swap(a, b);
  }
  const int CL = g.widths[g.levels];
  if ((s = gn(d, p, a, n, H * W, CL, d->out_gn)) != LC_OK) return s;
  return conv(d, p, d->out, 2, CL, 32, n, H, W, a, nullptr, img, 1, g.C_img);
}

}  // namespace

extern "C" {

const char* lc_decoder_last_error(const lc_decoder* d) { return d ? d->err.c_str() : g_derr.c_str(); }

lc_status lc_decoder_check_config(const lc_decoder_config* cfg) { return check_dcfg(nullptr, cfg); }

size_t lc_decoder_workspace_bytes(const lc_decoder_config* cfg, int slice_frames) {
  if (check_dcfg(nullptr, cfg) != LC_OK) return 0;
  if (slice_frames < 0) { g_derr = "slice_frames must be >= 0"; return 0; }
  return make_dplan(*cfg, eff_slice(*cfg, slice_frames)).total;
}

lc_status lc_decoder_create(const lc_decoder_config* cfg, void* stream, lc_decoder** out) {
  if (!out) return dfail(nullptr, LC_ERR_ARG, "out is NULL");
  lc_status s = check_dcfg(nullptr, cfg);
  if (s != LC_OK) return s;
  if (!stream) return dfail(nullptr, LC_ERR_ARG, "stream must be a non-default stream");
  lc_decoder* d = new (std::nothrow) lc_decoder();
  if (!d) return dfail(nullptr, LC_ERR_NOMEM, "out of host memory");
  d->cfg = *cfg;
  d->s = (hipStream_t)stream;
  d->wblob = nullptr; d->wblob_bytes = 0; d->have_weights = false;
  d->arena = nullptr; d->arena_bytes = 0;
  *out = d;
  return LC_OK;
}

lc_status lc_decoder_destroy(lc_decoder* d) {
  if (!d) return LC_OK;
  (void)hipStreamSynchronize(d->s);
  if (d->wblob) (void)hipFree(d->wblob);
  delete d;
  return LC_OK;
}

lc_status lc_decoder_load_weights(lc_decoder* d, const lc_decoder_weights* w) {
  if (!d) return dfail(nullptr, LC_ERR_ARG, "decoder is NULL");
  if (!w) return dfail(d, LC_ERR_ARG, "weights is NULL");
  const lc_decoder_config& g = d->cfg;
  const int dt = g.dtype, L = g.levels, C0 = g.widths[0], CL = g.widths[L];
  const size_t es = dtype_size(dt);
  auto need_gc = [](const lc_gnconv_w& x) { return x.gn_g && x.gn_b && x.w && x.b; };
  bool ok = w->conv_in_w && w->conv_in_b && need_gc(w->mid_res[0]) && need_gc(w->mid_res[1]) && need_gc(w->out) &&
            w->mid_attn.gn_g && w->mid_attn.gn_b && w->mid_attn.wq && w->mid_attn.wk && w->mid_attn.wv && w->mid_attn.wo &&
            w->mid_attn.bo;
  for (int l = 0; l < L; ++l) ok = ok && need_gc(w->up_res[l]) && w->up_conv_w[l] && w->up_conv_b[l];
  if (!ok) return dfail(d, LC_ERR_ARG, "a weight pointer is NULL");
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
  const size_t o_cin_w = take((size_t)g.C_lat * 9 * C0 * 4), o_cin_b = take((size_t)C0 * 4);
  size_t o_rg[2 + LC_DEC_MAX_LEVELS], o_rb[2 + LC_DEC_MAX_LEVELS], o_rw[2 + LC_DEC_MAX_LEVELS], o_rbias[2 + LC_DEC_MAX_LEVELS];
  for (int i = 0; i < 2 + L; ++i) {
    const int C = i < 2 ? C0 : g.widths[i - 2];
    o_rg[i] = take((size_t)C * 4); o_rb[i] = take((size_t)C * 4); o_rw[i] = take((size_t)C * 9 * C * es); o_rbias[i] = take((size_t)C * 4);
  }
  const size_t o_ag = take((size_t)C0 * 4), o_ab = take((size_t)C0 * 4), o_aqkv = take((size_t)3 * C0 * C0 * es),
               o_awo = take((size_t)C0 * C0 * es), o_abo = take((size_t)C0 * 4);
  size_t o_uw[LC_DEC_MAX_LEVELS], o_ub[LC_DEC_MAX_LEVELS];
  for (int l = 0; l < L; ++l) { o_uw[l] = take((size_t)g.widths[l + 1] * 9 * g.widths[l] * es); o_ub[l] = take((size_t)g.widths[l + 1] * 4); }
  const size_t o_og = take((size_t)CL * 4), o_ob = take((size_t)CL * 4), o_ow = take((size_t)32 * 9 * CL * es), o_obias = take(32 * 4);

  LCD_HIP(d, hipStreamSynchronize(d->s));
  if (d->wblob) { LCD_HIP(d, hipFree(d->wblob)); d->wblob = nullptr; d->have_weights = false; }
  void* blob = nullptr;
  if (hipMalloc(&blob, off) != hipSuccess) return dfail(d, LC_ERR_NOMEM, "hipMalloc of %zu bytes for packed weights failed", off);
  d->wblob = blob; d->wblob_bytes = off;
  char* b = (char*)blob;
  hipStream_t s = d->s;
#define F32(src, dst_off, n, npad) LCD_HIP(d, launch_to_f32(s, dt, src, (float*)(b + dst_off), n, npad))
#define CW(src, dst_off, co, ci, copad) LCD_HIP(d, launch_pack_conv_w(s, dt, src, b + dst_off, co, ci, 9, copad))
  LCD_HIP(d, launch_pack_conv_in_w(s, dt, w->conv_in_w, (float*)(b + o_cin_w), C0, g.C_lat));
  F32(w->conv_in_b, o_cin_b, C0, C0);
  d->cin_w = (float*)(b + o_cin_w); d->cin_b = (float*)(b + o_cin_b);
  for (int i = 0; i < 2 + L; ++i) {
    const int C = i < 2 ? C0 : g.widths[i - 2];
    const lc_gnconv_w& r = i < 2 ? w->mid_res[i] : w->up_res[i - 2];
    F32(r.gn_g, o_rg[i], C, C); F32(r.gn_b, o_rb[i], C, C); CW(r.w, o_rw[i], C, C, C); F32(r.b, o_rbias[i], C, C);
    d->res_gn[i] = GnP{(float*)(b + o_rg[i]), (float*)(b + o_rb[i])};
    d->res[i] = ConvP{b + o_rw[i], (float*)(b + o_rbias[i])};
  }
  F32(w->mid_attn.gn_g, o_ag, C0, C0); F32(w->mid_attn.gn_b, o_ab, C0, C0);
  LCD_HIP(d, launch_copy_rows(s, dt, w->mid_attn.wq, b + o_aqkv, (int64_t)C0 * C0));
  LCD_HIP(d, launch_copy_rows(s, dt, w->mid_attn.wk, b + o_aqkv + (size_t)C0 * C0 * es, (int64_t)C0 * C0));
  LCD_HIP(d, launch_copy_rows(s, dt, w->mid_attn.wv, b + o_aqkv + (size_t)2 * C0 * C0 * es, (int64_t)C0 * C0));
  LCD_HIP(d, launch_copy_rows(s, dt, w->mid_attn.wo, b + o_awo, (int64_t)C0 * C0));
  F32(w->mid_attn.bo, o_abo, C0, C0);
  d->at_gn = GnP{(float*)(b + o_ag), (float*)(b + o_ab)};
  d->at_wqkv = b + o_aqkv; d->at_wo = b + o_awo; d->at_bo = (float*)(b + o_abo);
  for (int l = 0; l < L; ++l) {
    CW(w->up_conv_w[l], o_uw[l], g.widths[l + 1], g.widths[l], g.widths[l + 1]);
    F32(w->up_conv_b[l], o_ub[l], g.widths[l + 1], g.widths[l + 1]);
    d->upc[l] = ConvP{b + o_uw[l], (float*)(b + o_ub[l])};
  }
  F32(w->out.gn_g, o_og, CL, CL); F32(w->out.gn_b, o_ob, CL, CL);
  CW(w->out.w, o_ow, g.C_img, CL, 32); F32(w->out.b, o_obias, g.C_img, 32);
  d->out_gn = GnP{(float*)(b + o_og), (float*)(b + o_ob)};
  d->out = ConvP{b + o_ow, (float*)(b + o_obias)};
#undef F32
#undef CW
  LCD_HIP(d, hipStreamSynchronize(s));
  d->have_weights = true;
  return LC_OK;
}

lc_status lc_decoder_set_workspace(lc_decoder* d, void* arena, size_t bytes) {
  if (!d) return dfail(nullptr, LC_ERR_ARG, "decoder is NULL");
  if (!arena) return dfail(d, LC_ERR_ARG, "arena is NULL");
  if ((uintptr_t)arena % kAlign) return dfail(d, LC_ERR_ARG, "arena must be 256-byte aligned");
  LCD_HIP(d, hipStreamSynchronize(d->s));
  d->arena = (char*)arena;
  d->arena_bytes = bytes;
  return LC_OK;
}

lc_status lc_decode(lc_decoder* d, const void* z, void* img, int slice_frames) {
  if (!d) return dfail(nullptr, LC_ERR_ARG, "decoder is NULL");
  if (!z || !img) return dfail(d, LC_ERR_ARG, "z and img must not be NULL");
  if (slice_frames < 0) return dfail(d, LC_ERR_ARG, "slice_frames must be >= 0");
  if (!d->have_weights) return dfail(d, LC_ERR_STATE, "weights not loaded");
  if (!d->arena) return dfail(d, LC_ERR_STATE, "workspace not set");
  const lc_decoder_config& g = d->cfg;
  const int n = eff_slice(g, slice_frames);
  const DPlan p = make_dplan(g, n);
  if (p.total > d->arena_bytes)
    return dfail(d, LC_ERR_NOMEM, "a slice of %d frames needs %zu bytes of workspace, %zu are set", n, p.total, d->arena_bytes);
  const size_t es = dtype_size(g.dtype);
  int maxC = 0;
  for (int l = 0; l <= g.levels; ++l) maxC = std::max(maxC, (int)g.widths[l]);
  LCD_HIP(d, launch_fill_f32(d->s, (float*)(d->arena + p.off_one), (int64_t)n * maxC, 1.f));
  LCD_HIP(d, launch_fill_f32(d->s, (float*)(d->arena + p.off_zero), (int64_t)n * maxC, 0.f));
  const size_t zf = (size_t)g.C_lat * g.H * g.W * es;
  const size_t imf = (size_t)g.C_img * ((size_t)g.H << g.levels) * ((size_t)g.W << g.levels) * es;
  for (int n0 = 0; n0 < g.N; n0 += n) {
    const lc_status s = decode_pass(d, p, (const char*)z + n0 * zf, (char*)img + n0 * imf, std::min(n, g.N - n0));
    if (s != LC_OK) return s;
  }
  return LC_OK;
}

lc_status lc_decoder_sync(lc_decoder* d) {
  if (!d) return dfail(nullptr, LC_ERR_ARG, "decoder is NULL");
  LCD_HIP(d, hipStreamSynchronize(d->s));
  return LC_OK;
}

}  // extern "C"

// The normal and the cache step on a U-Net with real block internals: residual blocks with two convolutions and a
// time-embedding add, spatial transformer blocks (LayerNorm, self-attention, cross-attention, GEGLU feed-forward),
// temporal transformer blocks with a sinusoidal frame encoding, strided down and upsampling convolutions, and a
// three-level deep branch whose output is the cached feature ("Feature Calculation" paragraph and "Asynchronous
// Swapping" section: a normal step stores it, a cache step runs the shallow blocks only and concatenates it).
// The convolutions, GroupNorm statistics, linear layers and attention cores are the kernels of the denoising stage
// (the cross-attention is the spatial kernel reading its keys from the conditioning tokens); new here are four
// bandwidth kernels: LayerNorm with affine (+ frame encoding), GEGLU, the time-embedding bias, channel concat (with the
// statistics and the rounding of the concatenated rows in the same pass).
// Activations are fp32 channels-last rows [frame][position][channel]; matrix operands have the stage's dtype.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "../../include/lightcache.h"
#include "lc_internal.h"

using namespace lc;

namespace lc {

// y[r][:] = LN(x[r][:]) * gamma + beta (+ pe[(r / rows_per_frame) % F][:]), one wavefront per row; biased variance.
// x fp32, y of type T. D % 4 == 0, D <= 64 * 4 * LNA_MAXV.
constexpr int LNA_MAXV = 8;
template <class T>
__global__ __launch_bounds__(256) void ln_affine_kernel(const float* __restrict__ x, const float* __restrict__ gamma,
                                                        const float* __restrict__ beta, const float* __restrict__ pe,
                                                        T* __restrict__ y, int64_t rows, int D, int rows_per_frame, int F, float eps) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int nv = D / 4;
  const f32x4* xr = reinterpret_cast<const f32x4*>(x + row * D);
  const f32x4* pr = pe ? reinterpret_cast<const f32x4*>(pe + (int64_t)((row / rows_per_frame) % F) * D) : nullptr;
  f32x4 v[LNA_MAXV];
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < LNA_MAXV; ++j) {
    const int p = lane + 64 * j;
    if (p < nv) {
      v[j] = xr[p];
      s += (v[j][0] + v[j][1]) + (v[j][2] + v[j][3]);
    }
  }
  const float mu = wave_sum(s) / (float)D;
  float q = 0.f;
#pragma unroll
  for (int j = 0; j < LNA_MAXV; ++j) {
    if (lane + 64 * j < nv) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float d = v[j][e] - mu;
        q = fmaf(d, d, q);
      }
    }
  }
  const float rstd = 1.f / sqrtf(wave_sum(q) / (float)D + eps);
#pragma unroll
  for (int j = 0; j < LNA_MAXV; ++j) {
    const int p = lane + 64 * j;
    if (p < nv) {
      const f32x4 g = reinterpret_cast<const f32x4*>(gamma)[p], b = reinterpret_cast<const f32x4*>(beta)[p];
      float o[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = fmaf((v[j][e] - mu) * rstd, g[e], b[e]);
      if (pr) {
        const f32x4 a = pr[p];
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] += a[e];
      }
      T* dst = y + row * D + p * 4;
      if constexpr (sizeof(T) == 2) {
        bf16x4 ov;
#pragma unroll
        for (int e = 0; e < 4; ++e) ov[e] = static_cast<bf16_t>(o[e]);
        *reinterpret_cast<bf16x4*>(dst) = ov;
      } else {
        *reinterpret_cast<f32x4*>(dst) = f32x4{o[0], o[1], o[2], o[3]};
      }
    }
  }
}

// g[r][k] = u[r][k] * gelu_tanh(u[r][M + k]); u [rows][2M], g [rows][M]; thread = one 16-byte packet of g
template <class T>
__global__ __launch_bounds__(256) void geglu_kernel(const T* __restrict__ u, T* __restrict__ g, int64_t rows, int M) {
  constexpr int VEC = Vec16<T>::N;
  const int ppr = M / VEC;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= rows * ppr) return;
  const int64_t r = i / ppr;
  const int k = (int)(i - r * ppr) * VEC;
  const Vec16<T> a = load16(u + r * 2 * M + k), b = load16(u + r * 2 * M + M + k);
  Vec16<T> o;
#pragma unroll
  for (int e = 0; e < VEC; ++e) o.set(e, a.get(e) * gelu_tanh_f(b.get(e)));
  store16(g + r * M + k, o);
}

// out[b][o] = bias[o] + bt[o] + sum_k wt[o][k] * SiLU(temb[b][k]): the per-channel constant a residual block adds
// after its first convolution, folded into that convolution's bias. One wavefront per (b, o); fp32 throughout.
template <class T>
__global__ __launch_bounds__(256) void temb_bias_kernel(const T* __restrict__ temb, const float* __restrict__ wt,
                                                        const float* __restrict__ bt, const float* __restrict__ bias,
                                                        float* __restrict__ out, int B, int Cout, int td) {
  const int lane = threadIdx.x & 63;
  const int item = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= B * Cout) return;
  const int b = item / Cout, o = item - b * Cout;
  float acc = 0.f;
  for (int k = lane; k < td; k += 64) acc = fmaf(wt[(int64_t)o * td + k], silu_f(to_f32(temb[(int64_t)b * td + k])), acc);
  acc = wave_sum(acc);
  if (lane == 0) out[item] = acc + bt[o] + bias[o];
}

// y[r][:] = bf16(x[m(r)][:] * scale[f][:] + shift[f][:]), f = r / rows_per_frame: GroupNorm applied to fp32 rows and
// rounded once, the operand of the projection into a transformer block. Thread = 8 channels of one row.
// MAPPED: the dense rows are gathered through the row map (a chunk of positions out of every frame).
template <bool MAPPED>
__global__ __launch_bounds__(256) void gn_apply_kernel(const float* __restrict__ x, const float* __restrict__ scale,
                                                       const float* __restrict__ shift, bf16_t* __restrict__ y, int64_t rows,
                                                       int C8, int rows_per_frame, RowMap m) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= rows * C8) return;
  const int64_t r = i / C8;
  const int c = (int)(i - r * C8) * 8;
  const int64_t f = r / rows_per_frame;
  const int64_t sr = MAPPED ? m(r) : r;
  float v[8], sc[8], sh[8];
  load_f<float, 8>(x + sr * C8 * 8 + c, v);
  load_f<float, 8>(scale + f * C8 * 8 + c, sc);
  load_f<float, 8>(shift + f * C8 * 8 + c, sh);
  Vec16<bf16_t> o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o.set(e, fmaf(v[e], sc[e], sh[e]));
  store16(y + r * C8 * 8 + c, o);
}

// dst[r][0:Ca] = a[r][:], dst[r][Ca:Ca+Cb] = b[r][:] (fp32, Ca and Cb multiples of 4), fused with what the residual
// block needs of the concatenated rows next: their GroupNorm partial sums (partial[frame][split][Ca + Cb][2], 64-row splits as the statistics kernel writes them, folded in
// the same fixed order) and, when yb != nullptr, a copy rounded to bf16 (the operand of the 1x1 shortcut). One
// workgroup = one split of one frame and up to 256 packets of 4 channels (gridDim.z of them side by side).
__global__ __launch_bounds__(256) void concat_stats_kernel(const float* __restrict__ a, const float* __restrict__ b,
                                                           float* __restrict__ dst, bf16_t* __restrict__ yb,
                                                           float* __restrict__ partial, int rows_per_frame, int Ca4, int Cb4) {
  __shared__ float red[2][256 * 4];
  const int W4 = Ca4 + Cb4;
  const int cv0 = blockIdx.z * 256;
  const int cv = min(W4 - cv0, 256);
  const int R = 256 / cv;
  const int split = blockIdx.x, frame = blockIdx.y, splits = gridDim.x;
  const int tid = threadIdx.x;
  const int cvec = tid % cv, rsub = tid / cv;
  float s4[4] = {0.f, 0.f, 0.f, 0.f}, q4[4] = {0.f, 0.f, 0.f, 0.f};
  const int r0 = split * kStatRows;
  const int r1 = min(r0 + kStatRows, rows_per_frame);
  if (rsub < R) {
    const int c = cv0 + cvec;
    const bool from_a = c < Ca4;
    const f32x4* src = from_a ? reinterpret_cast<const f32x4*>(a) + (int64_t)frame * rows_per_frame * Ca4 + c
                              : reinterpret_cast<const f32x4*>(b) + (int64_t)frame * rows_per_frame * Cb4 + (c - Ca4);
    const int ld = from_a ? Ca4 : Cb4;
    for (int r = r0 + rsub; r < r1; r += R) {
      const f32x4 v = src[(int64_t)r * ld];
      const int64_t o = ((int64_t)frame * rows_per_frame + r) * W4 + c;
      reinterpret_cast<f32x4*>(dst)[o] = v;
      if (yb) {
        bf16x4 h;
#pragma unroll
        for (int e = 0; e < 4; ++e) h[e] = static_cast<bf16_t>(v[e]);
        reinterpret_cast<bf16x4*>(yb)[o] = h;
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        s4[e] += v[e];
        q4[e] = fmaf(v[e], v[e], q4[e]);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    red[0][tid * 4 + e] = s4[e];
    red[1][tid * 4 + e] = q4[e];
  }
  __syncthreads();
  for (int c = tid; c < cv * 4; c += 256) {
    float ss = 0.f, qq = 0.f;
    for (int j = 0; j < R; ++j) {
      ss += red[0][j * cv * 4 + c];
      qq += red[1][j * cv * 4 + c];
    }
    float* pp = partial + (((int64_t)frame * splits + split) * (W4 * 4) + cv0 * 4 + c) * 2;
    pp[0] = ss;
    pp[1] = qq;
  }
}

}  // namespace lc

namespace {

thread_local std::string g_uerr = "";
constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct ConvP { void *w, *wt; float* b; };            // packed [Cout][9][Cin], the same in tile order (or nullptr), bias
struct LinP { void* w; float* b; };                  // [Cout][Cin] operand type, fp32 bias (or nullptr)
struct NormP { float *g, *b; };
struct RbP { int cin, cout; NormP gn1, gn2; ConvP conv1, conv2; float *temb_w, *temb_b; LinP shortcut; };
struct TfP {
  int C; bool cross;
  bool ff_fused;  // ff1's rows are stored in alternating blocks of 32 value and 32 gate channels: its kernel applies the GEGLU
  NormP gn, ln1, ln2, ln3;
  LinP pin, qkv, wo1, q2, kv2, wo2, ff1, ff2, pout;
  float* pe;  // [F][C] (temporal blocks)
};

struct UPlan {
  int nc[3];         // frames per chunk at H x W, H/2 x W/2, H/4 x W/4
  size_t map_bytes;  // one map of all frames: the largest tensor that passes between two blocks
  size_t off_map[3], off_s, off_d1, off_slots, slot_bytes;
  size_t off_part, off_parta, off_partb, off_scale, off_shift, off_one, off_zero, off_tb, off_kv, off_vtx;
  size_t off_xc, off_h, off_sc, off_xb, off_up;                   // one chunk inside a residual block or a resampling
  size_t off_z, off_a, off_qkv, off_vt, off_ao, off_u, off_g;     // one chunk inside a transformer block (same memory)
  size_t total;
};

}  // namespace

struct lc_unet {
  lc_unet_config cfg;
  hipStream_t cs, ss;
  int frame_chunk;
  UPlan plan;
  char* arena;
  size_t arena_bytes;
  bool have_weights;
  void* wblob;
  float *cin_w, *cin_b;
  void* cin_wp;  // conv_in weights as rows [C][64] of the operand type (k = plane * 9 + tap, zero padded), or nullptr
  RbP rb[6];
  TfP st[4], tt[4];
  ConvP down[2], up[2], out;
  NormP out_gn;
  std::vector<void*> host;
  std::vector<char> host_filled, dev_filled, in_pending;
  std::vector<hipEvent_t> ev_produced, ev_consumed, ev_in_done, ev_rd_done;
  std::string err;
};

namespace {

lc_status ufail(lc_unet* c, lc_status code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (c) c->err = buf; else g_uerr = buf;
  return code;
}
#define LCU_HIP(c, expr)                                                                          \
  do {                                                                                            \
    hipError_t e_ = (expr);                                                                       \
    if (e_ != hipSuccess) return ufail(c, LC_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_));   \
  } while (0)
#define LCU_TRY(expr)                     \
  do {                                    \
    const lc_status s_ = (expr);          \
    if (s_ != LC_OK) return s_;           \
  } while (0)

lc_status check_ucfg(lc_unet* c, const lc_unet_config* g) {
  if (!g) return ufail(c, LC_ERR_ARG, "config is NULL");
  if (g->dtype != LC_F32 && g->dtype != LC_BF16) return ufail(c, LC_ERR_ARG, "dtype must be LC_F32 or LC_BF16");
  if (g->B <= 0 || g->F <= 0 || g->H <= 0 || g->W <= 0 || g->C_lat <= 0 || g->C <= 0 || g->C1 <= 0 || g->C2 <= 0 || g->groups <= 0 ||
      g->head_dim <= 0 || g->ctx_len <= 0 || g->ctx_dim <= 0 || g->temb_dim <= 0 || g->ff_mult <= 0)
    return ufail(c, LC_ERR_SHAPE, "all sizes must be positive");
  if (g->H % 4 || g->W % 4) return ufail(c, LC_ERR_SHAPE, "H and W must be multiples of 4");
  for (int C : {g->C, g->C1, g->C2, g->ctx_dim})
    if (C % 64 || C > 64 * 4 * LNA_MAXV) return ufail(c, LC_ERR_SHAPE, "C, C1, C2 and ctx_dim must be multiples of 64, at most %d", 64 * 4 * LNA_MAXV);
  for (int C : {g->C, g->C1, g->C2, g->C + g->C1, g->C1 + g->C2})
    if (C % g->groups || C / g->groups > 512) return ufail(c, LC_ERR_SHAPE, "every width (and C + C1, C1 + C2) must be divisible by groups");
  const int d = g->head_dim;
  if (!(d == 8 || d == 16 || d == 32 || d == 40 || d == 64)) return ufail(c, LC_ERR_SHAPE, "head_dim must be one of 8, 16, 32, 40, 64");
  if (g->C % d || g->C1 % d) return ufail(c, LC_ERR_SHAPE, "C and C1 must be multiples of head_dim");
  if (g->C_lat > 16) return ufail(c, LC_ERR_SHAPE, "C_lat must be <= 16");
  if (g->ff_mult > 4) return ufail(c, LC_ERR_SHAPE, "ff_mult must be <= 4");
  if ((size_t)g->F * 3 * std::max(g->C, g->C1) * dtype_size(g->dtype) > (size_t)128 << 10)
    return ufail(c, LC_ERR_SHAPE, "F * 3 * max(C, C1) elements must fit 128 KiB");
  if (g->dev_slots < 1 || g->dev_slots > 8) return ufail(c, LC_ERR_SHAPE, "dev_slots must be in [1, 8]");
  if (g->host_slots < 0 || g->host_slots > 64) return ufail(c, LC_ERR_SHAPE, "host_slots must be in [0, 64]");
  if (!(g->gn_eps > 0.f) || !(g->ln_eps > 0.f)) return ufail(c, LC_ERR_SHAPE, "gn_eps and ln_eps must be positive");
  if ((int64_t)g->B * g->F * g->H * g->W > (int64_t)1 << 24) return ufail(c, LC_ERR_SHAPE, "too many positions");
  return LC_OK;
}

inline size_t entry_bytes(const lc_unet_config& g) { return (size_t)g.B * g.F * g.H * g.W * g.C1 * 4; }

// Positions of every frame that one pass of a temporal block takes when the per-frame blocks take nc of the N
// frames: the same number of rows, rounded up to whole positions.
inline int pos_chunk(int P, int nc, int N) { return (int)(((int64_t)P * nc + N - 1) / N); }

// Frames per chunk at a level: twice as many at each level down, where a frame has a quarter of the positions and
// twice the channels, so that a chunk's maps keep their size (and the launches their fill).
inline int level_chunk(int frame_chunk, int level, int N) {
  if (frame_chunk <= 0 || frame_chunk > N) return N;
  return (int)std::min<int64_t>(N, (int64_t)frame_chunk << level);
}

// Arena. Of all frames: three maps for the tensors that pass between blocks, the two skips kept across the deep
// branch, the device slots, the GroupNorm scale / shift. Of one chunk (nc frames in the per-frame blocks, as many
// rows of all frames in the temporal ones): the inside of a residual block (concatenated input, hidden map,
// shortcut) or of a resampling (upsampled map), and, in the same memory, the token buffers of a transformer block.
UPlan make_uplan(const lc_unet_config& g, int frame_chunk) {
  UPlan p;
  const size_t es = dtype_size(g.dtype);
  const int64_t N = (int64_t)g.B * g.F, P = (int64_t)g.H * g.W, P1 = P / 4, P2 = P / 16;
  for (int l = 0; l < 3; ++l) p.nc[l] = level_chunk(frame_chunk, l, (int)N);
  const int64_t nc0 = p.nc[0], nc1 = p.nc[1], nc2 = p.nc[2];
  const int maxC = std::max({g.C + g.C1, g.C1 + g.C2, g.C2});
  const int64_t full = N * std::max({P * g.C, P1 * g.C, P1 * g.C1, P1 * g.C2, P2 * g.C1, P2 * g.C2});
  // rows * width of a transformer block's chunk at its largest (level 0 or level 1)
  const int64_t tok = N * std::max((int64_t)pos_chunk((int)P, p.nc[0], (int)N) * g.C, (int64_t)pos_chunk((int)P1, p.nc[1], (int)N) * g.C1);
  // partial sums per frame: the statistics kernel's 64-row splits, or the (at most twice as many) 32-pixel splits
  // that the convolutions write beside their output, times the widest tensor of the level
  auto splits_of = [&](int lvl) {
    const int H = g.H >> lvl, W = g.W >> lvl;
    return (int64_t)std::max({stat_splits(H * W), conv_stat_splits(H, W), (H * W + 31) / 32});
  };
  const int64_t splits_c = std::max({splits_of(0) * (g.C + g.C1), splits_of(1) * std::max(g.C1 + g.C2, g.C), splits_of(2) * std::max(g.C1, g.C2)});
  // the same for what one block hands to the next: a block's output of all frames
  const int64_t splits_o = std::max({splits_of(0) * g.C, splits_of(1) * g.C1, splits_of(2) * g.C2});
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
  p.map_bytes = align_up((size_t)full * 4);
  for (int i = 0; i < 3; ++i) p.off_map[i] = take(p.map_bytes);
  p.off_s = take((size_t)N * P * g.C * 4);
  p.off_d1 = take((size_t)N * P1 * g.C1 * 4);
  p.slot_bytes = align_up(entry_bytes(g));
  p.off_slots = off; off += p.slot_bytes * g.dev_slots;
  p.off_part = take((size_t)N * splits_c * 2 * 4);
  p.off_parta = take((size_t)N * splits_o * 2 * 4);
  p.off_partb = take((size_t)N * splits_o * 2 * 4);
  p.off_scale = take((size_t)N * maxC * 4);
  p.off_shift = take((size_t)N * maxC * 4);
  p.off_one = take((size_t)N * maxC * 4);
  p.off_zero = take((size_t)N * maxC * 4);
  p.off_tb = take((size_t)g.B * std::max({g.C, g.C1, g.C2}) * 4);
  p.off_kv = take((size_t)g.B * g.ctx_len * 2 * std::max(g.C, g.C1) * es);
  p.off_vtx = take((size_t)g.B * std::max(g.C, g.C1) * attn_tp(g.ctx_len) * es);
  const size_t chunk0 = off;
  // ---- one chunk, residual blocks and resamplings
  const int64_t cat = std::max(nc0 * P * (g.C + g.C1), nc1 * P1 * (g.C1 + g.C2));
  const int64_t hid = std::max({nc0 * P * g.C, nc1 * P1 * g.C1, nc2 * P2 * g.C2});
  p.off_xc = take((size_t)cat * 4);
  p.off_h = take((size_t)hid * 4);
  p.off_sc = take((size_t)hid * 4);
  p.off_xb = take(g.dtype == kBF16 ? (size_t)cat * es : 0);
  p.off_up = take((size_t)std::max(nc1 * P1 * g.C2, nc0 * P * g.C1) * 4);
  const size_t end_rb = off;
  // ---- one chunk, transformer blocks
  off = chunk0;
  p.off_z = take((size_t)tok * 4);
  p.off_a = take((size_t)tok * es);
  p.off_qkv = take((size_t)tok * 3 * es);
  p.off_vt = take((size_t)std::max(nc0 * g.C * attn_tp((int)P), nc1 * g.C1 * attn_tp((int)P1)) * es);
  p.off_ao = take((size_t)tok * es);
  p.off_u = take(g.dtype == kBF16 ? 0 : (size_t)tok * 2 * g.ff_mult * es);  // (bf16: the GEGLU is fused, no 2M-wide tensor)
  p.off_g = take((size_t)tok * g.ff_mult * es);
  p.total = std::max(off, end_rb);
  return p;
}

inline char* slot_ptr(lc_unet* c, int s) { return c->arena + c->plan.off_slots + c->plan.slot_bytes * s; }
inline float* map_ptr(lc_unet* c, int i) { return (float*)(c->arena + c->plan.off_map[i]); }
inline RowMap dense_map() { return RowMap{0, 0, 1 << 30}; }

// fn(n0, n) for every chunk [n0, n0 + n) of the N frames, at the chunk size of a level
template <class Fn>
lc_status frame_chunks(lc_unet* c, int level, Fn fn) {
  const int N = c->cfg.B * c->cfg.F, nc = c->plan.nc[level];
  for (int n0 = 0; n0 < N; n0 += nc) LCU_TRY(fn(n0, std::min(nc, N - n0)));
  return LC_OK;
}
// fn(b, i0, n) for every run of frames of the chunk [n0, n0 + nc) that lies in one batch element b: frames
// i0 ... i0 + n - 1 counted from the chunk's first
template <class Fn>
lc_status batch_runs(const lc_unet_config& g, int n0, int nc, Fn fn) {
  for (int f = n0; f < n0 + nc;) {
    const int b = f / g.F, e = std::min(n0 + nc, (b + 1) * g.F);
    LCU_TRY(fn(b, f - n0, e - f));
    f = e;
  }
  return LC_OK;
}

// ---- operators -------------------------------------------------------------------------------------------------
// Partial sums [frame][splits][C][2] of a tensor, written by the kernel that produced it (part == nullptr: none)
struct Stats { const float* part; int splits; };

// scale / shift (frame 0 first) of a GroupNorm over n frames of [rows][C] from the partial sums of its input
lc_status gn_fold(lc_unet* c, Stats st, int n, int rows, int C, const NormP& w) {
  const UPlan& p = c->plan;
  LCU_HIP(c, launch_gn_finalize(c->cs, st.part, C, st.splits, rows, 1.f, nullptr, 0, 0, 0, 0.f, w.g, w.b, c->cfg.groups, c->cfg.gn_eps,
                                (float*)(c->arena + p.off_scale), (float*)(c->arena + p.off_shift), n));
  return LC_OK;
}
// the same from the tensor itself, fp32 rows x: a pass of the statistics kernel first
lc_status gn(lc_unet* c, const float* x, int n, int rows, int C, const NormP& w) {
  float* part = (float*)(c->arena + c->plan.off_part);
  LCU_HIP(c, launch_gn_stats(c->cs, kF32, x, part, n, rows, C));
  return gn_fold(c, Stats{part, stat_splits(rows)}, n, rows, C, w);
}

// y = [res +] conv3x3(act(x)) over n frames; src 2: SiLU(GroupNorm(x)) with the scale / shift at hand (those of frame
// `f0` on), src 1: x as it is. planar: y is [n][Cout_store][H][W] of the stage's dtype (the last convolution).
// stat: where the partial sums of y go ([frame of the launch][conv_stat_splits(H, W)][Cout][2]), or nullptr.
lc_status conv(lc_unet* c, const ConvP& w, const float* bias, int src, int Cin, int Cout, int n, int f0, int H, int W, const float* x,
               const float* res, void* y, int planar, int Cout_store, float* stat = nullptr) {
  const UPlan& p = c->plan;
  FusedDesc f;
  memset(&f, 0, sizeof f);
  f.dt = c->cfg.dtype; f.y_f32 = planar ? 0 : 1; f.taps = 9; f.src = src; f.Cin = Cin; f.Cout = Cout; f.Cout_store = Cout_store;
  f.w = w.w; f.w_tiles = w.wt; f.bias = bias; f.frames = n; f.H = H; f.W = W; f.x = x; f.res = res; f.y = y; f.planar_out = planar;
  f.scale = (const float*)(c->arena + (src == 2 ? p.off_scale : p.off_one)) + (size_t)f0 * Cin;
  f.shift = (const float*)(c->arena + (src == 2 ? p.off_shift : p.off_zero)) + (size_t)f0 * Cin;
  f.in_map = f.out_map = dense_map();
  if (stat) { f.stat = stat; f.stat_splits = conv_stat_splits(H, W); }
  LCU_HIP(c, launch_fused(c->cs, f));
  return LC_OK;
}

// What a linear layer does beyond y = x W^T + bias.
struct LinOpt {
  const float* res = nullptr;  // fp32, added; rows as y's
  void* y2 = nullptr;          // a copy of y rounded to the operand type
  int act = 0, q_cols = 0;
  // x is fp32 and row r is multiplied by scale[r / in_map.rows_per_seg] and shifted (GroupNorm apply) on the way in
  const float *scale = nullptr, *shift = nullptr;
  RowMap in_map = RowMap{0, 0, 1 << 30}, out_map = RowMap{0, 0, 1 << 30};
  // channels >= yt_from leave transposed, as the V^T [frame][Cout - yt_from][yt_Tp] the spatial attention kernel
  // stages (frames of yt_T rows); y then has yt_from channels per row
  void* yt = nullptr;
  int yt_from = 0, yt_T = 0, yt_Tp = 0;
};

// y[out_map(r)][Cout] = x[in_map(r)][Cin] W^T + bias [+ res], r < rows; x of the operand type unless o.scale is set
lc_status linear(lc_unet* c, const LinP& w, int Cin, int Cout, int64_t rows, const void* x, void* y, int y32, const LinOpt& o = LinOpt()) {
  FusedDesc f;
  memset(&f, 0, sizeof f);
  f.dt = c->cfg.dtype; f.y_f32 = y32; f.taps = 1; f.src = o.scale ? 1 : 0; f.Cin = Cin; f.Cout = Cout; f.Cout_store = Cout; f.w = w.w;
  f.bias = w.b; f.rows = rows; f.in_map = o.in_map; f.out_map = o.out_map; f.x = x; f.res = o.res; f.y = y; f.y2 = o.y2; f.act = o.act;
  f.scale = o.scale; f.shift = o.shift;
  f.yt = o.yt; f.yt_from = o.yt_from; f.yt_T = o.yt_T; f.yt_Tp = o.yt_Tp;
  if (o.q_cols) { f.q_cols = o.q_cols; f.q_scale = attn_q_scale(c->cfg.head_dim); }  // softmax scale folded into q
  LCU_HIP(c, launch_fused(c->cs, f));
  return LC_OK;
}

// y (bf16, dense rows) = x[m(r)] * scale[r / rows_per_frame] + shift[...]
lc_status gn_apply(lc_unet* c, const float* x, const float* scale, const float* shift, void* y, int64_t rows, int C, int rows_per_frame,
                   RowMap m) {
  const int64_t n = rows * (C / 8);
  const unsigned blocks = (unsigned)((n + 255) / 256);
  if (m.rows_per_seg >= rows || m.seg_stride == m.rows_per_seg)  // consecutive rows from m.base on
    gn_apply_kernel<false><<<blocks, 256, 0, c->cs>>>(x + m.base * C, scale, shift, (bf16_t*)y, rows, C / 8, rows_per_frame, m);
  else
    gn_apply_kernel<true><<<blocks, 256, 0, c->cs>>>(x, scale, shift, (bf16_t*)y, rows, C / 8, rows_per_frame, m);
  LCU_HIP(c, hipGetLastError());
  return LC_OK;
}

lc_status ln(lc_unet* c, const float* z, const NormP& w, const float* pe, void* y, int64_t rows, int D, int rows_per_frame) {
  const unsigned blocks = (unsigned)((rows + 3) / 4);
  const lc_unet_config& g = c->cfg;
  if (g.dtype == kBF16)
    ln_affine_kernel<bf16_t><<<blocks, 256, 0, c->cs>>>(z, w.g, w.b, pe, (bf16_t*)y, rows, D, rows_per_frame, g.F, g.ln_eps);
  else
    ln_affine_kernel<float><<<blocks, 256, 0, c->cs>>>(z, w.g, w.b, pe, (float*)y, rows, D, rows_per_frame, g.F, g.ln_eps);
  LCU_HIP(c, hipGetLastError());
  return LC_OK;
}

// z += FF(LN(z)): GEGLU feed-forward on fp32 rows z, in place
// (zb: where a bf16 stage also leaves the new z rounded to bf16, the operand of the projection out; or nullptr)
lc_status feed_forward(lc_unet* c, const TfP& w, float* z, int64_t rows, int rows_per_frame, void* zb) {
  const lc_unet_config& g = c->cfg;
  const UPlan& p = c->plan;
  const int C = w.C, M = g.ff_mult * C;
  char *a = c->arena + p.off_a, *u = c->arena + p.off_u, *gl = c->arena + p.off_g;
  LinOpt back;
  back.res = z; back.y2 = zb;
  LCU_TRY(ln(c, z, w.ln3, nullptr, a, rows, C, rows_per_frame));
  if (w.ff_fused) {  // value * gelu(gate) in the first layer's epilogue: the 2M-wide tensor never exists
    LinOpt geglu;
    geglu.act = 2;
    LCU_TRY(linear(c, w.ff1, C, 2 * M, rows, a, gl, 0, geglu));
    return linear(c, w.ff2, M, C, rows, gl, z, 1, back);
  }
  LCU_TRY(linear(c, w.ff1, C, 2 * M, rows, a, u, 0));
  const int64_t n16 = rows * M * (int64_t)dtype_size(g.dtype) / 16;
  if (g.dtype == kBF16) geglu_kernel<bf16_t><<<(unsigned)((n16 + 255) / 256), 256, 0, c->cs>>>((const bf16_t*)u, (bf16_t*)gl, rows, M);
  else geglu_kernel<float><<<(unsigned)((n16 + 255) / 256), 256, 0, c->cs>>>((const float*)u, (float*)gl, rows, M);
  LCU_HIP(c, hipGetLastError());
  return linear(c, w.ff2, M, C, rows, gl, z, 1, back);
}

// dst [n][rows][Ca + Cb] = the channel concatenation of a and b, with its GroupNorm partial sums (64-row splits) into
// the scratch and, when yb != nullptr, a bf16 copy: one pass instead of a concatenation, a statistics pass and a rounding
// pass over the widest tensor of the step
lc_status concat_stats(lc_unet* c, const float* a, int Ca, const float* b, int Cb, float* dst, void* yb, int n, int rows) {
  const int W4 = (Ca + Cb) / 4;
  dim3 grid(stat_splits(rows), n, (W4 + 255) / 256);
  concat_stats_kernel<<<grid, 256, 0, c->cs>>>(a, b, dst, (bf16_t*)yb, (float*)(c->arena + c->plan.off_part), rows, Ca / 4, Cb / 4);
  LCU_HIP(c, hipGetLastError());
  return LC_OK;
}

// Residual block on [N][P][cin] fp32 -> y [N][P][cout] fp32 (y none of the inputs), a chunk of frames at a time. The
// input is xa, or, when Cb > 0, the channel concatenation of xa [N][P][Ca] and xb [N][P][Cb], put together chunk by
// chunk: the concatenated tensor of all frames never exists. in: the partial sums of xa (all frames), if its producer
// wrote them and there is no xb. out: where those of y go (all frames), or nullptr. The convolutions write the partial
// sums of what they store, so the second GroupNorm, and the one of the block that follows, need no pass of their own.
lc_status res_block(lc_unet* c, const RbP& w, const void* temb, int level, const float* xa, int Ca, const float* xb, int Cb, float* y,
                    Stats in = Stats{nullptr, 0}, float* out = nullptr) {
  const lc_unet_config& g = c->cfg;
  const UPlan& p = c->plan;
  const int H = g.H >> level, W = g.W >> level, P = H * W;
  float* tb = (float*)(c->arena + p.off_tb);
  float *xc = (float*)(c->arena + p.off_xc), *h = (float*)(c->arena + p.off_h), *sc = (float*)(c->arena + p.off_sc);
  float* part = (float*)(c->arena + p.off_part);
  const int cs = conv_stat_splits(H, W);
  const unsigned blocks = (unsigned)((g.B * w.cout + 3) / 4);
  if (g.dtype == kBF16)
    temb_bias_kernel<bf16_t><<<blocks, 256, 0, c->cs>>>((const bf16_t*)temb, w.temb_w, w.temb_b, w.conv1.b, tb, g.B, w.cout, g.temb_dim);
  else
    temb_bias_kernel<float><<<blocks, 256, 0, c->cs>>>((const float*)temb, w.temb_w, w.temb_b, w.conv1.b, tb, g.B, w.cout, g.temb_dim);
  LCU_HIP(c, hipGetLastError());
  return frame_chunks(c, level, [&](int n0, int nc) -> lc_status {
    const float* x = xa + (size_t)n0 * P * Ca;
    // (a shortcut through the dense-row kernel contracts x rounded to bf16)
    const bool short16 = w.shortcut.w && g.dtype == kBF16 && w.cout % 160 == 0;
    void* xb16 = c->arena + p.off_xb;
    if (Cb) {
      LCU_TRY(concat_stats(c, x, Ca, xb + (size_t)n0 * P * Cb, Cb, xc, short16 ? xb16 : nullptr, nc, P));
      x = xc;
      LCU_TRY(gn_fold(c, Stats{part, stat_splits(P)}, nc, P, w.cin, w.gn1));
    } else if (in.part) {
      LCU_TRY(gn_fold(c, Stats{in.part + (size_t)n0 * in.splits * w.cin * 2, in.splits}, nc, P, w.cin, w.gn1));
    } else {
      LCU_TRY(gn(c, x, nc, P, w.cin, w.gn1));
    }
    // the time embedding is one vector per batch element: its frames share a bias
    // (the scale / shift of x are folded by now: the partial sums of h may take the scratch)
    LCU_TRY(batch_runs(g, n0, nc, [&](int b, int i0, int n) {
      return conv(c, w.conv1, tb + (size_t)b * w.cout, 2, w.cin, w.cout, n, i0, H, W, x + (size_t)i0 * P * w.cin, nullptr,
                  h + (size_t)i0 * P * w.cout, 0, w.cout, part + (size_t)i0 * cs * w.cout * 2);
    }));
    const float* res = x;
    if (w.shortcut.w) {
      const int64_t rows = (int64_t)nc * P;
      if (short16) {
        // x rounded to bf16 (by the concatenation, else in a pass of its own), then contracted as dense bf16 rows
        if (!Cb)
          LCU_TRY(gn_apply(c, x, (const float*)(c->arena + p.off_one), (const float*)(c->arena + p.off_zero), xb16, rows, w.cin, P, dense_map()));
        LCU_TRY(linear(c, w.shortcut, w.cin, w.cout, rows, xb16, sc, 1));
      } else {
        LinOpt o;
        o.scale = (const float*)(c->arena + p.off_one); o.shift = (const float*)(c->arena + p.off_zero); o.in_map = RowMap{0, P, P};
        LCU_TRY(linear(c, w.shortcut, w.cin, w.cout, rows, x, sc, 1, o));
      }
      res = sc;
    }
    LCU_TRY(gn_fold(c, Stats{part, cs}, nc, P, w.cout, w.gn2));
    return conv(c, w.conv2, w.conv2.b, 2, w.cout, w.cout, nc, 0, H, W, h, res, y + (size_t)n0 * P * w.cout, 0, w.cout,
                out ? out + (size_t)n0 * cs * w.cout * 2 : nullptr);
  });
}

// The inside of a transformer block on `rows` rows gathered from x by m (m.rows_per_seg consecutive ones per frame):
// projection in, self-attention, cross-attention (spatial blocks), feed-forward, projection out and the residual,
// written back through m. scale / shift: GroupNorm of x, the frame of the first row first. attend / cross run the
// attention core from the chunk's q,k,v (or q) buffer into its attention-output buffer.
template <class Attend, class Cross>
lc_status tf_rows(lc_unet* c, const TfP& w, float* x, RowMap m, const float* scale, const float* shift, int64_t rows, Attend attend,
                  Cross cross, void* vt = nullptr, int vt_Tp = 0) {
  const lc_unet_config& g = c->cfg;
  const UPlan& p = c->plan;
  const int C = w.C, rpf = m.rows_per_seg;
  float* z = (float*)(c->arena + p.off_z);
  char *a = c->arena + p.off_a, *qkv = c->arena + p.off_qkv, *ao = c->arena + p.off_ao;
  // where the dense-row kernel applies (bf16, width a multiple of 160) the projections' operands are rounded in
  // passes of their own and contracted as dense bf16 rows; otherwise they are converted inside the contraction
  const bool b16 = g.dtype == kBF16 && C % 160 == 0;
  if (b16) {
    LCU_TRY(gn_apply(c, x, scale, shift, a, rows, C, rpf, m));
    LCU_TRY(linear(c, w.pin, C, C, rows, a, z, 1));
  } else {
    LinOpt o;
    o.scale = scale; o.shift = shift; o.in_map = m;
    LCU_TRY(linear(c, w.pin, C, C, rows, x, z, 1, o));
  }
  LinOpt onto_z;
  onto_z.res = z;
  // self-attention (spatial: the q columns leave the projection multiplied by log2(e) / sqrt(d), as the attention
  // kernel's cheaper softmax path wants them)
  LCU_TRY(ln(c, z, w.ln1, w.pe, a, rows, C, rpf));
  LinOpt q_scaled;
  q_scaled.q_cols = w.cross ? C : 0;
  if (vt) {  // spatial: q and k as rows of 2C channels, v transposed straight from the projection's epilogue
    q_scaled.yt = vt; q_scaled.yt_from = 2 * C; q_scaled.yt_T = rpf; q_scaled.yt_Tp = vt_Tp;
  }
  LCU_TRY(linear(c, w.qkv, C, 3 * C, rows, a, qkv, 0, q_scaled));
  LCU_TRY(attend());
  LCU_TRY(linear(c, w.wo1, C, C, rows, ao, z, 1, onto_z));
  if (w.cross) {  // queries from the tokens, keys and values from the conditioning tokens of the batch element
    LCU_TRY(ln(c, z, w.ln2, nullptr, a, rows, C, rpf));
    LCU_TRY(linear(c, w.q2, C, C, rows, a, qkv, 0));
    LCU_TRY(cross());
    LCU_TRY(linear(c, w.wo2, C, C, rows, ao, z, 1, onto_z));
  }
  LCU_TRY(feed_forward(c, w, z, rows, rpf, b16 ? a : nullptr));
  LinOpt back;
  back.res = x; back.out_map = m;
  if (b16) return linear(c, w.pout, C, C, rows, a, x, 1, back);
  back.scale = (const float*)(c->arena + p.off_one); back.shift = (const float*)(c->arena + p.off_zero); back.in_map = RowMap{0, rpf, rpf};
  return linear(c, w.pout, C, C, rows, z, x, 1, back);
}

// Spatial transformer block in place on x [N][P][C] fp32, a chunk of frames at a time: tokens = the P positions of a
// frame, with cross-attention to cond [B][ctx_len][ctx_dim].
// in: the partial sums of x, if its producer wrote them.
lc_status st_block(lc_unet* c, const TfP& w, const void* cond, int level, float* x, Stats in = Stats{nullptr, 0}) {
  const lc_unet_config& g = c->cfg;
  const UPlan& p = c->plan;
  const int N = g.B * g.F, P = (g.H >> level) * (g.W >> level), C = w.C, heads = C / g.head_dim, Tp = attn_tp(P), L = g.ctx_len, TpL = attn_tp(L);
  const size_t es = dtype_size(g.dtype);
  char *qkv = c->arena + p.off_qkv, *vt = c->arena + p.off_vt, *ao = c->arena + p.off_ao, *kv = c->arena + p.off_kv,
       *vtx = c->arena + p.off_vtx;
  if (in.part) LCU_TRY(gn_fold(c, in, N, P, C, w.gn));
  else LCU_TRY(gn(c, x, N, P, C, w.gn));
  // keys and values of the conditioning tokens: the same for every frame of a batch element
  LCU_TRY(linear(c, w.kv2, g.ctx_dim, 2 * C, (int64_t)g.B * L, cond, kv, 0));
  LCU_HIP(c, launch_make_vt(c->cs, g.dtype, kv + (size_t)C * es, 2 * C, vtx, g.B, L, TpL, C));
  return frame_chunks(c, level, [&](int n0, int nc) -> lc_status {
    auto attend = [&]() -> lc_status {
      LCU_HIP(c, launch_spatial_attention(c->cs, g.dtype, qkv, 2 * C, vt, Tp, ao, nc, P, heads, g.head_dim, 0, P, 1));
      return LC_OK;
    };
    auto cross = [&]() -> lc_status {
      return batch_runs(g, n0, nc, [&](int b, int i0, int n) -> lc_status {
        const size_t r0 = (size_t)i0 * P * C * es;
        LCU_HIP(c, launch_cross_attention(c->cs, g.dtype, qkv + r0, C, kv + (size_t)b * L * 2 * C * es, 2 * C,
                                          vtx + (size_t)b * C * TpL * es, TpL, ao + r0, n, P, L, n, heads, g.head_dim));
        return LC_OK;
      });
    };
    const float* scale = (const float*)(c->arena + p.off_scale) + (size_t)n0 * C;
    const float* shift = (const float*)(c->arena + p.off_shift) + (size_t)n0 * C;
    return tf_rows(c, w, x + (size_t)n0 * P * C, RowMap{0, P, P}, scale, shift, (int64_t)nc * P, attend, cross, vt, Tp);
  });
}

// Temporal transformer block in place on x [N][P][C] fp32: tokens = the F frames of a position, a chunk of positions
// (of every frame) at a time. The GroupNorm statistics are those of the whole frames, taken before any position is
// rewritten.
lc_status tt_block(lc_unet* c, const TfP& w, int level, float* x) {
  const lc_unet_config& g = c->cfg;
  const UPlan& p = c->plan;
  const int N = g.B * g.F, P = (g.H >> level) * (g.W >> level), C = w.C, heads = C / g.head_dim;
  char *qkv = c->arena + p.off_qkv, *ao = c->arena + p.off_ao;
  LCU_TRY(gn(c, x, N, P, C, w.gn));
  const float* scale = (const float*)(c->arena + p.off_scale);
  const float* shift = (const float*)(c->arena + p.off_shift);
  const int pc = pos_chunk(P, p.nc[level], N);
  for (int p0 = 0; p0 < P; p0 += pc) {
    const int n = std::min(pc, P - p0);
    auto attend = [&]() -> lc_status {
      LCU_HIP(c, launch_temporal_attention(c->cs, g.dtype, qkv, ao, g.B, g.F, n, heads, g.head_dim));
      return LC_OK;
    };
    auto cross = []() -> lc_status { return LC_OK; };
    LCU_TRY(tf_rows(c, w, x, RowMap{p0, P, n}, scale, shift, (int64_t)N * n, attend, cross));
  }
  return LC_OK;
}

// y [N][H/2][W/2][C] (level `level`) = conv3x3 of stride 2 over x [N][H][W][C] (the level above)
lc_status down_conv(lc_unet* c, const ConvP& w, int C, int level, const float* x, float* y) {
  const int H = c->cfg.H >> (level - 1), W = c->cfg.W >> (level - 1);
  return frame_chunks(c, level, [&](int n0, int nc) -> lc_status {
    ConvDesc d;
    memset(&d, 0, sizeof d);
    d.dt = c->cfg.dtype; d.x_f32 = 1; d.y_f32 = 1; d.taps = 9; d.stride = 2; d.Cin = C; d.Cout = C; d.Cout_store = C;
    d.w = w.w; d.bias = w.b; d.frames = nc; d.H = H; d.W = W; d.x = x + (size_t)n0 * H * W * C; d.y = y + (size_t)n0 * (H / 2) * (W / 2) * C;
    d.out_map = dense_map();
    LCU_HIP(c, launch_conv(c->cs, d));
    return LC_OK;
  });
}

// y [N][2H][2W][C] (level `level`) = conv3x3(nearest2x(x [N][H][W][C])) (the level below); the upsampled map exists
// for one chunk of frames at a time
lc_status up_conv(lc_unet* c, const ConvP& w, int C, int level, const float* x, float* y) {
  const int H = c->cfg.H >> (level + 1), W = c->cfg.W >> (level + 1);
  float* up = (float*)(c->arena + c->plan.off_up);
  return frame_chunks(c, level, [&](int n0, int nc) -> lc_status {
    LCU_HIP(c, launch_up2_rows(c->cs, x + (size_t)n0 * H * W * C, up, nc, H, W, C));
    return conv(c, w, w.b, 1, C, C, nc, 0, 2 * H, 2 * W, up, nullptr, y + (size_t)n0 * 4 * H * W * C, 0, C);
  });
}

lc_status run_step(lc_unet* c, const void* x, const void* temb, const void* cond, void* eps, int slot, bool full) {
  const lc_unet_config& g = c->cfg;
  const UPlan& p = c->plan;
  const int N = g.B * g.F, H = g.H, W = g.W, P = H * W;
  const size_t es = dtype_size(g.dtype);
  float *m0 = map_ptr(c, 0), *m1 = map_ptr(c, 1), *m2 = map_ptr(c, 2);
  float* s = (float*)(c->arena + p.off_s);
  float* d1 = (float*)(c->arena + p.off_d1);
  float* deep = (float*)slot_ptr(c, slot);
  const int maxC = std::max({g.C + g.C1, g.C1 + g.C2, g.C2});
  LCU_HIP(c, launch_fill_f32(c->cs, (float*)(c->arena + p.off_one), (int64_t)N * maxC, 1.f));
  LCU_HIP(c, launch_fill_f32(c->cs, (float*)(c->arena + p.off_zero), (int64_t)N * maxC, 0.f));
  // Partial sums of a block's output for the GroupNorm that reads it next, written by the convolution that stores it
  // (two buffers: a residual block reads its input's while it writes its output's).
  float *pa = (float*)(c->arena + p.off_parta), *pb = (float*)(c->arena + p.off_partb);
  const int cs0 = conv_stat_splits(H, W), cs1 = conv_stat_splits(H / 2, W / 2), cs2 = conv_stat_splits(H / 4, W / 4);
  // ---- shallow down: s = TT(ST(RB(conv_in(x))))
  Stats cin_st{nullptr, 0};
  LCU_TRY(frame_chunks(c, 0, [&](int n0, int nc) -> lc_status {
    const char* xc = (const char*)x + (size_t)n0 * g.C_lat * P * es;
    float* y = m0 + (size_t)n0 * P * g.C;
    // the tiled kernel where the shape allows it (a property of the configuration, never of the chunk)
    hipError_t e = c->cin_wp ? launch_conv_in_tile(c->cs, g.dtype, xc, c->cin_wp, c->cin_b, y, pa + (size_t)n0 * (P / 32) * g.C * 2, nc, H, W,
                                                   g.C_lat, g.C, Win{0, 0, 0, 0})
                             : hipErrorNotSupported;
    if (e == hipSuccess) { cin_st = Stats{pa, P / 32}; return LC_OK; }
    if (e != hipErrorNotSupported) LCU_HIP(c, e);
    LCU_HIP(c, launch_conv_in(c->cs, g.dtype, xc, y, nc, H, W, g.C_lat, g.C, c->cin_w, c->cin_b));
    return LC_OK;
  }));
  LCU_TRY(res_block(c, c->rb[0], temb, 0, m0, g.C, nullptr, 0, s, cin_st, pb));
  LCU_TRY(st_block(c, c->st[0], cond, 0, s, Stats{pb, cs0}));
  LCU_TRY(tt_block(c, c->tt[0], 0, s));
  if (full) {
    // ---- level 1 down: d1 = TT(ST(RB(Down(s))))
    LCU_TRY(down_conv(c, c->down[0], g.C, 1, s, m0));
    LCU_TRY(res_block(c, c->rb[1], temb, 1, m0, g.C, nullptr, 0, d1, Stats{nullptr, 0}, pa));
    LCU_TRY(st_block(c, c->st[1], cond, 1, d1, Stats{pa, cs1}));
    LCU_TRY(tt_block(c, c->tt[1], 1, d1));
    // ---- level 2: e = UpC(RB(RB(Down(d1))))
    LCU_TRY(down_conv(c, c->down[1], g.C1, 2, d1, m0));
    LCU_TRY(res_block(c, c->rb[2], temb, 2, m0, g.C1, nullptr, 0, m1, Stats{nullptr, 0}, pa));
    LCU_TRY(res_block(c, c->rb[3], temb, 2, m1, g.C2, nullptr, 0, m0, Stats{pa, cs2}, nullptr));
    LCU_TRY(up_conv(c, c->up[0], g.C2, 1, m0, m2));                // e in m2 [N][P1][C2]
    // ---- level 1 up: d = TT(ST(RB(Concat(d1, e))))
    LCU_TRY(res_block(c, c->rb[4], temb, 1, d1, g.C1, m2, g.C2, m1, Stats{nullptr, 0}, pa));
    LCU_TRY(st_block(c, c->st[2], cond, 1, m1, Stats{pa, cs1}));
    LCU_TRY(tt_block(c, c->tt[2], 1, m1));
    // ---- the cached feature: deep = UpC(d), written to the slot, which may still be the source of a swap-out
    //      or the target of a swap-in on the side stream
    LCU_HIP(c, hipStreamWaitEvent(c->cs, c->ev_rd_done[slot], 0));
    LCU_HIP(c, hipStreamWaitEvent(c->cs, c->ev_in_done[slot], 0));
    c->in_pending[slot] = 0;
    LCU_TRY(up_conv(c, c->up[1], g.C1, 0, m1, deep));
    LCU_HIP(c, hipEventRecord(c->ev_produced[slot], c->cs));
    c->dev_filled[slot] = 1;
  } else if (c->in_pending[slot]) {
    LCU_HIP(c, hipStreamWaitEvent(c->cs, c->ev_in_done[slot], 0));
    c->in_pending[slot] = 0;
  }
  // ---- shallow up: u = TT(ST(RB(Concat(s, deep)))); eps = conv_out(SiLU(GN(u)))
  LCU_TRY(res_block(c, c->rb[5], temb, 0, s, g.C, deep, g.C1, m1, Stats{nullptr, 0}, pa));
  LCU_HIP(c, hipEventRecord(c->ev_consumed[slot], c->cs));
  LCU_TRY(st_block(c, c->st[3], cond, 0, m1, Stats{pa, cs0}));
  LCU_TRY(tt_block(c, c->tt[3], 0, m1));
  return frame_chunks(c, 0, [&](int n0, int nc) -> lc_status {
    LCU_TRY(gn(c, m1 + (size_t)n0 * P * g.C, nc, P, g.C, c->out_gn));
    return conv(c, c->out, c->out.b, 2, g.C, 32, nc, 0, H, W, m1 + (size_t)n0 * P * g.C, nullptr, (char*)eps + (size_t)n0 * g.C_lat * P * es, 1,
                g.C_lat);
  });
}

lc_status step_checks(lc_unet* c, const void* x, const void* temb, const void* cond, void* eps, int slot) {
  if (!c) return ufail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!x || !temb || !cond || !eps) return ufail(c, LC_ERR_ARG, "x, temb, cond and eps must not be NULL");
  if (slot < 0 || slot >= c->cfg.dev_slots) return ufail(c, LC_ERR_ARG, "device slot %d out of range", slot);
  if (!c->have_weights) return ufail(c, LC_ERR_STATE, "weights not loaded");
  if (!c->arena) return ufail(c, LC_ERR_STATE, "workspace not set");
  return LC_OK;
}

}  // namespace

extern "C" {

const char* lc_unet_last_error(const lc_unet* c) { return c ? c->err.c_str() : g_uerr.c_str(); }
lc_status lc_unet_check_config(const lc_unet_config* cfg) { return check_ucfg(nullptr, cfg); }
size_t lc_unet_entry_bytes(const lc_unet_config* cfg) { return check_ucfg(nullptr, cfg) == LC_OK ? entry_bytes(*cfg) : 0; }
size_t lc_unet_workspace_bytes(const lc_unet_config* cfg) { return check_ucfg(nullptr, cfg) == LC_OK ? make_uplan(*cfg, 0).total : 0; }
size_t lc_unet_chunk_workspace_bytes(const lc_unet_config* cfg, int frame_chunk) {
  if (check_ucfg(nullptr, cfg) != LC_OK) return 0;
  if (frame_chunk < 0) { g_uerr = "frame_chunk must be >= 0"; return 0; }
  return make_uplan(*cfg, frame_chunk).total;
}

lc_status lc_unet_destroy(lc_unet* c) {
  if (!c) return LC_OK;
  (void)hipStreamSynchronize(c->cs);
  (void)hipStreamSynchronize(c->ss);
  for (void* p : c->host) (void)hipHostFree(p);
  for (auto* v : {&c->ev_produced, &c->ev_consumed, &c->ev_in_done, &c->ev_rd_done})
    for (hipEvent_t e : *v) (void)hipEventDestroy(e);
  if (c->wblob) (void)hipFree(c->wblob);
  delete c;
  return LC_OK;
}

lc_status lc_unet_create(const lc_unet_config* cfg, void* compute_stream, void* side_stream, lc_unet** out) {
  if (!out) return ufail(nullptr, LC_ERR_ARG, "out is NULL");
  LCU_TRY(check_ucfg(nullptr, cfg));
  if (!compute_stream || !side_stream || compute_stream == side_stream)
    return ufail(nullptr, LC_ERR_ARG, "compute and side streams must be two distinct non-default streams");
  lc_unet* c = new (std::nothrow) lc_unet();
  if (!c) return ufail(nullptr, LC_ERR_NOMEM, "out of host memory");
  c->cfg = *cfg;
  c->cs = (hipStream_t)compute_stream; c->ss = (hipStream_t)side_stream;
  c->frame_chunk = 0;
  c->plan = make_uplan(c->cfg, 0);
  c->arena = nullptr; c->arena_bytes = 0; c->have_weights = false; c->wblob = nullptr;
  for (int i = 0; i < cfg->host_slots; ++i) {
    void* p = nullptr;
    if (hipHostMalloc(&p, entry_bytes(*cfg), hipHostMallocDefault) != hipSuccess) {
      (void)hipGetLastError();
      lc_unet_destroy(c);
      return ufail(nullptr, LC_ERR_NOMEM, "hipHostMalloc (pinned cache bank) failed");
    }
    c->host.push_back(p);
  }
  c->host_filled.assign(cfg->host_slots, 0);
  c->dev_filled.assign(cfg->dev_slots, 0);
  c->in_pending.assign(cfg->dev_slots, 0);
  for (auto* v : {&c->ev_produced, &c->ev_consumed, &c->ev_in_done, &c->ev_rd_done})
    for (int i = 0; i < cfg->dev_slots; ++i) {
      hipEvent_t e;
      if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) {
        lc_unet_destroy(c);
        return ufail(nullptr, LC_ERR_HIP, "hipEventCreate failed");
      }
      v->push_back(e);
    }
  *out = c;
  return LC_OK;
}

lc_status lc_unet_load_weights(lc_unet* c, const lc_unet_weights* w) {
  if (!c) return ufail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!w) return ufail(c, LC_ERR_ARG, "weights is NULL");
  const lc_unet_config& g = c->cfg;
  const int dt = g.dtype;
  const size_t es = dtype_size(dt);
  const int C = g.C, C1 = g.C1, C2 = g.C2;
  const int rb_in[6] = {C, C, C1, C2, C1 + C2, C + C1}, rb_out[6] = {C, C1, C2, C2, C1, C};
  const int tf_c[4] = {C, C1, C1, C};
  // ---- every pointer present?
  bool ok = w->conv_in.w && w->conv_in.b && w->out_gn_g && w->out_gn_b && w->out.w && w->out.b;
  for (int i = 0; i < 6; ++i) {
    const lc_unet_rb_w& r = w->rb[i];
    ok = ok && r.gn1_g && r.gn1_b && r.conv1_w && r.conv1_b && r.temb_w && r.temb_b && r.gn2_g && r.gn2_b && r.conv2_w && r.conv2_b;
    if (rb_in[i] != rb_out[i]) ok = ok && r.short_w && r.short_b;
  }
  for (int k = 0; k < 2; ++k)
    for (int i = 0; i < 4; ++i) {
      const lc_unet_tf_w& t = k ? w->tt[i] : w->st[i];
      ok = ok && t.gn_g && t.gn_b && t.pin_w && t.pin_b && t.ln1_g && t.ln1_b && t.attn1.wq && t.attn1.wk && t.attn1.wv && t.attn1.wo &&
           t.attn1.bo && t.ln3_g && t.ln3_b && t.ff1_w && t.ff1_b && t.ff2_w && t.ff2_b && t.pout_w && t.pout_b;
      if (!k) ok = ok && t.ln2_g && t.ln2_b && t.attn2.wq && t.attn2.wk && t.attn2.wv && t.attn2.wo && t.attn2.bo;
    }
  for (int i = 0; i < 2; ++i) ok = ok && w->down[i].w && w->down[i].b && w->up[i].w && w->up[i].b;
  if (!ok) return ufail(c, LC_ERR_ARG, "a weight pointer is NULL");

  // ---- two passes over the same layout code: the first sizes the blob, the second fills it
  LCU_HIP(c, hipStreamSynchronize(c->cs));
  if (c->wblob) { LCU_HIP(c, hipFree(c->wblob)); c->wblob = nullptr; c->have_weights = false; }
  hipStream_t s = c->cs;
  char* base = nullptr;
  size_t off = 0;
  bool fill = false;
  hipError_t herr = hipSuccess;
  auto take = [&](size_t bytes) { char* o = base + off; off += align_up(bytes); return o; };
  auto note = [&](hipError_t e) { if (herr == hipSuccess && e != hipSuccess) herr = e; };
  auto f32 = [&](const void* src, int n) {  // a vector converted to fp32
    float* d = (float*)take((size_t)n * 4);
    if (fill) note(launch_to_f32(s, dt, src, d, n, n));
    return d;
  };
  auto norm = [&](const void* gsrc, const void* bsrc, int n) { NormP q; q.g = f32(gsrc, n); q.b = f32(bsrc, n); return q; };
  auto lin = [&](const void* wsrc, const void* bsrc, int cout, int cin) {  // [cout][cin] as it is
    LinP q;
    q.w = take((size_t)cout * cin * es);
    if (fill) note(launch_copy_rows(s, dt, wsrc, q.w, (int64_t)cout * cin));
    q.b = bsrc ? f32(bsrc, cout) : nullptr;
    return q;
  };
  auto stack = [&](std::initializer_list<const void*> srcs, int cout_each, int cin) {  // matrices stacked on the output axis
    LinP q;
    q.w = take((size_t)srcs.size() * cout_each * cin * es);
    q.b = nullptr;
    size_t i = 0;
    for (const void* src : srcs) {
      if (fill) note(launch_copy_rows(s, dt, src, (char*)q.w + i * cout_each * cin * es, (int64_t)cout_each * cin));
      ++i;
    }
    return q;
  };
  // the first feed-forward layer of a bf16 stage: rows [0, M) are the values, [M, 2M) the gates; stored as
  // value block 0, gate block 0, value block 1, ... (blocks of 32 rows), the order the fused GEGLU epilogue pairs
  auto lin_geglu = [&](const void* wsrc, const void* bsrc, int M, int cin) {
    LinP q;
    q.w = take((size_t)2 * M * cin * es);
    q.b = (float*)take((size_t)2 * M * 4);
    if (fill)
      for (int m = 0; m < M / 32; ++m)
        for (int h = 0; h < 2; ++h) {
          const size_t srow = (size_t)h * M + 32 * m, drow = (size_t)64 * m + 32 * h;
          note(launch_copy_rows(s, dt, (const char*)wsrc + srow * cin * es, (char*)q.w + drow * cin * es, (int64_t)32 * cin));
          note(launch_to_f32(s, dt, (const char*)bsrc + srow * es, q.b + drow, 32, 32));
        }
    return q;
  };
  auto conv3 = [&](const void* wsrc, const void* bsrc, int cout, int cin, int cout_pad, bool tiles) {
    ConvP q;
    q.w = take((size_t)cout_pad * 9 * cin * es);
    if (fill) note(launch_pack_conv_w(s, dt, wsrc, q.w, cout, cin, 9, cout_pad));
    q.wt = nullptr;
    if (tiles && dt == kBF16 && cout % 160 == 0 && cin % 64 == 0) {
      q.wt = take((size_t)cout * 9 * cin * es);
      if (fill) note(launch_pack_conv_w_tiles(s, dt, q.w, q.wt, cout, cin));
    }
    q.b = (float*)take((size_t)cout_pad * 4);
    if (fill) note(launch_to_f32(s, dt, bsrc, q.b, cout, cout_pad));
    return q;
  };
  auto layout = [&]() {
    off = 0;
    c->cin_w = (float*)take((size_t)g.C_lat * 9 * C * 4);
    if (fill) note(launch_pack_conv_in_w(s, dt, w->conv_in.w, c->cin_w, C, g.C_lat));
    c->cin_b = f32(w->conv_in.b, C);
    c->cin_wp = nullptr;
    if (dt == kBF16 && g.C_lat * 9 <= 48) {  // what the tiled first convolution reads
      c->cin_wp = take((size_t)C * 64 * es);
      if (fill) note(launch_pad_rows(s, dt, w->conv_in.w, c->cin_wp, C, g.C_lat * 9, 64));
    }
    for (int i = 0; i < 6; ++i) {
      const lc_unet_rb_w& r = w->rb[i];
      RbP& q = c->rb[i];
      q.cin = rb_in[i]; q.cout = rb_out[i];
      q.gn1 = norm(r.gn1_g, r.gn1_b, q.cin);
      q.conv1 = conv3(r.conv1_w, r.conv1_b, q.cout, q.cin, q.cout, true);
      q.temb_w = f32(r.temb_w, q.cout * g.temb_dim);
      q.temb_b = f32(r.temb_b, q.cout);
      q.gn2 = norm(r.gn2_g, r.gn2_b, q.cout);
      q.conv2 = conv3(r.conv2_w, r.conv2_b, q.cout, q.cout, q.cout, true);
      q.shortcut = LinP{nullptr, nullptr};
      if (q.cin != q.cout) q.shortcut = lin(r.short_w, r.short_b, q.cout, q.cin);
    }
    for (int k = 0; k < 2; ++k)
      for (int i = 0; i < 4; ++i) {
        const lc_unet_tf_w& t = k ? w->tt[i] : w->st[i];
        TfP& q = k ? c->tt[i] : c->st[i];
        const int D = tf_c[i], M = g.ff_mult * D;
        q.C = D; q.cross = !k;
        q.gn = norm(t.gn_g, t.gn_b, D);
        q.pin = lin(t.pin_w, t.pin_b, D, D);
        q.ln1 = norm(t.ln1_g, t.ln1_b, D);
        q.qkv = stack({t.attn1.wq, t.attn1.wk, t.attn1.wv}, D, D);
        q.wo1 = lin(t.attn1.wo, t.attn1.bo, D, D);
        q.ln2 = NormP{nullptr, nullptr};
        q.q2 = q.kv2 = q.wo2 = LinP{nullptr, nullptr};
        if (!k) {
          q.ln2 = norm(t.ln2_g, t.ln2_b, D);
          q.q2 = lin(t.attn2.wq, nullptr, D, D);
          q.kv2 = stack({t.attn2.wk, t.attn2.wv}, D, g.ctx_dim);
          q.wo2 = lin(t.attn2.wo, t.attn2.bo, D, D);
        }
        q.ln3 = norm(t.ln3_g, t.ln3_b, D);
        q.ff_fused = dt == kBF16;
        q.ff1 = q.ff_fused ? lin_geglu(t.ff1_w, t.ff1_b, M, D) : lin(t.ff1_w, t.ff1_b, 2 * M, D);
        q.ff2 = lin(t.ff2_w, t.ff2_b, D, M);
        q.pout = lin(t.pout_w, t.pout_b, D, D);
        q.pe = nullptr;
        if (k) {  // the frame encoding, computed in double and rounded once
          q.pe = (float*)take((size_t)g.F * D * 4);
          if (fill) {
            std::vector<float> pe((size_t)g.F * D);
            for (int f = 0; f < g.F; ++f)
              for (int j = 0; j < D; ++j) {
                const double ang = (double)f * std::exp(-std::log(10000.0) * (double)(j - j % 2) / (double)D);
                pe[(size_t)f * D + j] = (float)(j % 2 ? std::cos(ang) : std::sin(ang));
              }
            note(hipMemcpy(q.pe, pe.data(), pe.size() * 4, hipMemcpyHostToDevice));
          }
        }
      }
    c->down[0] = conv3(w->down[0].w, w->down[0].b, C, C, C, false);
    c->down[1] = conv3(w->down[1].w, w->down[1].b, C1, C1, C1, false);
    c->up[0] = conv3(w->up[0].w, w->up[0].b, C2, C2, C2, false);
    c->up[1] = conv3(w->up[1].w, w->up[1].b, C1, C1, C1, false);
    c->out_gn = norm(w->out_gn_g, w->out_gn_b, C);
    c->out = conv3(w->out.w, w->out.b, g.C_lat, C, 32, false);
  };
  layout();  // sizes only
  const size_t total = off;
  void* blob = nullptr;
  if (hipMalloc(&blob, total) != hipSuccess) return ufail(c, LC_ERR_NOMEM, "hipMalloc of %zu bytes for the weights failed", total);
  c->wblob = blob;
  base = (char*)blob;
  fill = true;
  layout();
  if (herr != hipSuccess) return ufail(c, LC_ERR_HIP, "packing the weights: %s", hipGetErrorString(herr));
  LCU_HIP(c, hipStreamSynchronize(s));
  c->have_weights = true;
  return LC_OK;
}

lc_status lc_unet_set_workspace(lc_unet* c, void* arena, size_t bytes) {
  if (!c) return ufail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!arena) return ufail(c, LC_ERR_ARG, "arena is NULL");
  if ((uintptr_t)arena % kAlign) return ufail(c, LC_ERR_ARG, "arena must be 256-byte aligned");
  if (bytes < c->plan.total) return ufail(c, LC_ERR_NOMEM, "workspace of %zu bytes is smaller than the %zu needed", bytes, c->plan.total);
  LCU_HIP(c, hipStreamSynchronize(c->cs));
  LCU_HIP(c, hipStreamSynchronize(c->ss));
  c->arena = (char*)arena; c->arena_bytes = bytes;
  std::fill(c->dev_filled.begin(), c->dev_filled.end(), 0);
  std::fill(c->in_pending.begin(), c->in_pending.end(), 0);
  return LC_OK;
}

lc_status lc_unet_set_chunk(lc_unet* c, int frame_chunk) {
  if (!c) return ufail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (frame_chunk < 0) return ufail(c, LC_ERR_ARG, "frame_chunk must be >= 0");
  const UPlan np = make_uplan(c->cfg, frame_chunk);
  if (c->arena && np.total > c->arena_bytes)
    return ufail(c, LC_ERR_NOMEM, "chunk setting needs %zu bytes, workspace has %zu", np.total, c->arena_bytes);
  c->frame_chunk = frame_chunk;  // (the skips and the device slots sit at chunk-independent offsets)
  c->plan = np;
  return LC_OK;
}

lc_status lc_unet_full_step(lc_unet* c, const void* x, const void* temb, const void* cond, void* eps, int dev_slot) {
  LCU_TRY(step_checks(c, x, temb, cond, eps, dev_slot));
  return run_step(c, x, temb, cond, eps, dev_slot, true);
}

lc_status lc_unet_cached_step(lc_unet* c, const void* x, const void* temb, const void* cond, void* eps, int dev_slot) {
  LCU_TRY(step_checks(c, x, temb, cond, eps, dev_slot));
  if (!c->dev_filled[dev_slot]) return ufail(c, LC_ERR_STATE, "cached step on empty device slot %d", dev_slot);
  return run_step(c, x, temb, cond, eps, dev_slot, false);
}

static lc_status unet_swap_common(lc_unet* c, int dev_slot, int host_slot) {
  if (!c) return ufail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (dev_slot < 0 || dev_slot >= c->cfg.dev_slots) return ufail(c, LC_ERR_ARG, "device slot %d out of range", dev_slot);
  if (host_slot < 0 || host_slot >= c->cfg.host_slots) return ufail(c, LC_ERR_ARG, "host slot %d out of range", host_slot);
  if (!c->arena) return ufail(c, LC_ERR_STATE, "workspace not set");
  return LC_OK;
}

lc_status lc_unet_swap_out(lc_unet* c, int dev_slot, int host_slot) {
  LCU_TRY(unet_swap_common(c, dev_slot, host_slot));
  if (!c->dev_filled[dev_slot]) return ufail(c, LC_ERR_STATE, "swap-out of empty device slot %d", dev_slot);
  LCU_HIP(c, hipStreamWaitEvent(c->ss, c->ev_produced[dev_slot], 0));
  LCU_HIP(c, hipMemcpyAsync(c->host[host_slot], slot_ptr(c, dev_slot), entry_bytes(c->cfg), hipMemcpyDeviceToHost, c->ss));
  LCU_HIP(c, hipEventRecord(c->ev_rd_done[dev_slot], c->ss));
  c->host_filled[host_slot] = 1;
  return LC_OK;
}

lc_status lc_unet_swap_in(lc_unet* c, int host_slot, int dev_slot) {
  LCU_TRY(unet_swap_common(c, dev_slot, host_slot));
  if (!c->host_filled[host_slot]) return ufail(c, LC_ERR_STATE, "swap-in from empty host slot %d", host_slot);
  LCU_HIP(c, hipStreamWaitEvent(c->ss, c->ev_consumed[dev_slot], 0));
  LCU_HIP(c, hipStreamWaitEvent(c->ss, c->ev_produced[dev_slot], 0));
  LCU_HIP(c, hipMemcpyAsync(slot_ptr(c, dev_slot), c->host[host_slot], entry_bytes(c->cfg), hipMemcpyHostToDevice, c->ss));
  LCU_HIP(c, hipEventRecord(c->ev_in_done[dev_slot], c->ss));
  c->in_pending[dev_slot] = 1;
  c->dev_filled[dev_slot] = 1;
  return LC_OK;
}

lc_status lc_unet_sync(lc_unet* c) {
  if (!c) return ufail(nullptr, LC_ERR_ARG, "ctx is NULL");
  LCU_HIP(c, hipStreamSynchronize(c->cs));
  LCU_HIP(c, hipStreamSynchronize(c->ss));
  return LC_OK;
}

lc_status lc_unet_cache_write(lc_unet* c, int dev_slot, const void* deep) {
  if (!c) return ufail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!deep) return ufail(c, LC_ERR_ARG, "deep is NULL");
  if (dev_slot < 0 || dev_slot >= c->cfg.dev_slots) return ufail(c, LC_ERR_ARG, "device slot %d out of range", dev_slot);
  if (!c->arena) return ufail(c, LC_ERR_STATE, "workspace not set");
  LCU_HIP(c, hipStreamWaitEvent(c->cs, c->ev_rd_done[dev_slot], 0));
  LCU_HIP(c, hipStreamWaitEvent(c->cs, c->ev_in_done[dev_slot], 0));
  c->in_pending[dev_slot] = 0;
  LCU_HIP(c, hipMemcpyAsync(slot_ptr(c, dev_slot), deep, entry_bytes(c->cfg), hipMemcpyDeviceToDevice, c->cs));
  LCU_HIP(c, hipEventRecord(c->ev_produced[dev_slot], c->cs));
  c->dev_filled[dev_slot] = 1;
  return LC_OK;
}

lc_status lc_unet_cache_peek(lc_unet* c, int host_slot, const void** ptr, size_t* bytes) {
  if (!c) return ufail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!ptr || !bytes) return ufail(c, LC_ERR_ARG, "output pointer is NULL");
  if (host_slot < 0 || host_slot >= c->cfg.host_slots) return ufail(c, LC_ERR_ARG, "host slot %d out of range", host_slot);
  if (!c->host_filled[host_slot]) return ufail(c, LC_ERR_STATE, "host slot %d is empty", host_slot);
  *ptr = c->host[host_slot];
  *bytes = entry_bytes(c->cfg);
  return LC_OK;
}

lc_status lc_unet_cache_dev_peek(lc_unet* c, int dev_slot, const void** ptr, size_t* bytes) {
  if (!c) return ufail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!ptr || !bytes) return ufail(c, LC_ERR_ARG, "output pointer is NULL");
  if (dev_slot < 0 || dev_slot >= c->cfg.dev_slots) return ufail(c, LC_ERR_ARG, "device slot %d out of range", dev_slot);
  if (!c->arena) return ufail(c, LC_ERR_STATE, "workspace not set");
  if (!c->dev_filled[dev_slot]) return ufail(c, LC_ERR_STATE, "device slot %d is empty", dev_slot);
  *ptr = slot_ptr(c, dev_slot);
  *bytes = entry_bytes(c->cfg);
  return LC_OK;
}

}  // extern "C"

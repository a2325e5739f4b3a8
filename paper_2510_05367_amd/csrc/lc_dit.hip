// The method on a video diffusion transformer: a stack of adaLN-modulated blocks whose range [a, b) is the cached
// deep part (the reuse rule of the "Asynchronous Swapping" section applied to a block stack). What the deep blocks
// add to the hidden states, Delta = x_b - x_a, is accumulated in a device slot of its own at a normal step, kept in
// pinned host memory, and added back at the cache steps, which run only the blocks [0, a) and [b, L). Feature chunk:
// LayerNorm, projections and the MLP run over token chunks, attention over query chunks against all keys.
// New kernels here: LayerNorm + modulation, tanh-GELU, gated accumulation (all bandwidth kernels, one pass each);
// the projections and the attention are the kernels of the U-Net stage.
#include <hip/hip_runtime.h>

#include <algorithm>
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

// y[r][:] = LN(x[r][:] (+ add[r][:])) * (1 + scale[:]) + shift[:], one wavefront per row; LN over D with biased
// variance and no affine of its own. x, add fp32; y of type T. D % 4 == 0, D <= 64 * 4 * LN_MAXV.
constexpr int LN_MAXV = 8;
template <class T>
__global__ __launch_bounds__(256) void ln_mod_kernel(const float* __restrict__ x, const float* __restrict__ add, const float* __restrict__ mod,
                                                     int which_shift, int which_scale, T* __restrict__ y, int rows, int D, float eps,
                                                     int64_t row0, int T_tok) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  // the modulation vectors of the row's batch element: mod [B][6][D] of this block, row0 + row = b * T_tok + token
  const int64_t b = (row0 + row) / T_tok;
  const float* __restrict__ shift = mod + (b * 6 + which_shift) * D;
  const float* __restrict__ scale = mod + (b * 6 + which_scale) * D;
  const int nv = D / 4;  // 16-byte packets per row
  const f32x4* xr = reinterpret_cast<const f32x4*>(x + (int64_t)row * D);
  const f32x4* ar = add ? reinterpret_cast<const f32x4*>(add + (int64_t)row * D) : nullptr;
  f32x4 v[LN_MAXV];
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < LN_MAXV; ++j) {
    const int p = lane + 64 * j;
    if (p < nv) {
      v[j] = xr[p];
      if (ar) v[j] += ar[p];
      s += (v[j][0] + v[j][1]) + (v[j][2] + v[j][3]);
    }
  }
  const float mu = wave_sum(s) / (float)D;
  float q = 0.f;
#pragma unroll
  for (int j = 0; j < LN_MAXV; ++j) {
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
  for (int j = 0; j < LN_MAXV; ++j) {
    const int p = lane + 64 * j;
    if (p < nv) {
      const f32x4 sc = reinterpret_cast<const f32x4*>(scale)[p], sh = reinterpret_cast<const f32x4*>(shift)[p];
      float o[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = fmaf((v[j][e] - mu) * rstd, 1.f + sc[e], sh[e]);
      T* dst = y + (int64_t)row * D + p * 4;
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

template <class T>
__global__ __launch_bounds__(256) void gelu_kernel(T* __restrict__ h, int64_t n16) {  // n16: 16-byte packets
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n16) return;
  Vec16<T> v = reinterpret_cast<Vec16<T>*>(h)[i];
#pragma unroll
  for (int e = 0; e < Vec16<T>::N; ++e) v.set(e, gelu_tanh_f(v.get(e)));
  reinterpret_cast<Vec16<T>*>(h)[i] = v;
}

// dst[r][c] += gate[b(r)][c] * t[r][c], gate = vector `which` of mod [B][6][D], b(r) = (row0 + r) / T_tok
// (mod == nullptr: dst += t); all fp32, D % 4 == 0
__global__ __launch_bounds__(256) void gate_add_kernel(float* __restrict__ dst, const float* __restrict__ t, const float* __restrict__ mod,
                                                       int which, int64_t n4, int D4, int64_t row0, int T_tok) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n4) return;
  f32x4 d = reinterpret_cast<f32x4*>(dst)[i];
  const f32x4 v = reinterpret_cast<const f32x4*>(t)[i];
  if (mod) {
    const int64_t r = i / D4;
    const int64_t b = (row0 + r) / T_tok;
    const f32x4 g = reinterpret_cast<const f32x4*>(mod + (b * 6 + which) * D4 * 4)[i - r * D4];
#pragma unroll
    for (int e = 0; e < 4; ++e) d[e] = fmaf(g[e], v[e], d[e]);
  } else {
    d += v;
  }
  reinterpret_cast<f32x4*>(dst)[i] = d;
}

}  // namespace lc

namespace {

thread_local std::string g_terr = "";
constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct BlkW { void *wqkv, *wo, *w1, *w2; float *bqkv, *bo, *b1, *b2; };
struct TPlan {
  int tc;  // rows per chunk of the per-row layers (LayerNorm, projections, MLP): tokens of the B*T of a step
  int qc;  // queries per batch element and attention launch
  size_t off_x, off_slots, slot_bytes, off_qkv, off_vt, off_ao, off_xn, off_hid, off_t, total;
};

}  // namespace

struct lc_dit {
  lc_dit_config cfg;
  hipStream_t cs, ss;
  int token_chunk;
  TPlan plan;
  char* arena;
  size_t arena_bytes;
  bool have_weights;
  void* wblob;
  std::vector<BlkW> blk;
  std::vector<void*> host;
  std::vector<char> host_filled, dev_filled, in_pending;
  std::vector<hipEvent_t> ev_produced, ev_consumed, ev_in_done, ev_rd_done;
  int64_t full_steps, cached_steps, swaps_out, swaps_in;
  std::string err;
};

namespace {

lc_status tfail(lc_dit* c, lc_status code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (c) c->err = buf; else g_terr = buf;
  return code;
}
#define LCT_HIP(c, expr)                                                                          \
  do {                                                                                            \
    hipError_t e_ = (expr);                                                                       \
    if (e_ != hipSuccess) return tfail(c, LC_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_));   \
  } while (0)

lc_status check_tcfg(lc_dit* c, const lc_dit_config* g) {
  if (!g) return tfail(c, LC_ERR_ARG, "config is NULL");
  if (g->dtype != LC_F32 && g->dtype != LC_BF16) return tfail(c, LC_ERR_ARG, "dtype must be LC_F32 or LC_BF16");
  if (g->B <= 0 || g->T <= 0 || g->D <= 0 || g->heads <= 0 || g->head_dim <= 0 || g->L <= 0 || g->mlp_ratio <= 0)
    return tfail(c, LC_ERR_SHAPE, "all sizes must be positive");
  if (g->D % 64 || g->D > 64 * 4 * LN_MAXV) return tfail(c, LC_ERR_SHAPE, "D must be a multiple of 64, at most %d", 64 * 4 * LN_MAXV);
  if (g->heads * g->head_dim != g->D) return tfail(c, LC_ERR_SHAPE, "heads * head_dim must equal D");
  const int d = g->head_dim;
  if (!(d == 8 || d == 16 || d == 32 || d == 40 || d == 64)) return tfail(c, LC_ERR_SHAPE, "head_dim must be one of 8, 16, 32, 40, 64");
  if (g->L > LC_DIT_MAX_BLOCKS) return tfail(c, LC_ERR_SHAPE, "L must be <= %d", LC_DIT_MAX_BLOCKS);
  if (g->cache_a < 0 || g->cache_a > g->cache_b || g->cache_b > g->L) return tfail(c, LC_ERR_SHAPE, "need 0 <= cache_a <= cache_b <= L");
  if (g->mlp_ratio > 8) return tfail(c, LC_ERR_SHAPE, "mlp_ratio must be <= 8");
  if (g->dev_slots < 1 || g->dev_slots > 8) return tfail(c, LC_ERR_SHAPE, "dev_slots must be in [1, 8]");
  if (g->host_slots < 0 || g->host_slots > 64) return tfail(c, LC_ERR_SHAPE, "host_slots must be in [0, 64]");
  if (!(g->ln_eps > 0.f)) return tfail(c, LC_ERR_SHAPE, "ln_eps must be positive");
  if ((int64_t)g->B * g->T > (int64_t)1 << 24) return tfail(c, LC_ERR_SHAPE, "too many tokens");
  return LC_OK;
}

// Arena: the fp32 hidden states, dev_slots Delta entries (fp32), q,k,v + V^T + attention output of ALL tokens (a
// query chunk attends to every key), and what one token chunk works in: its normalised rows, the MLP's hidden
// rows and a branch output.
TPlan make_tplan(const lc_dit_config& g, int token_chunk) {
  TPlan p;
  const size_t es = dtype_size(g.dtype);
  const int64_t R = (int64_t)g.B * g.T;
  // the per-row layers walk the B*T rows of a step in chunks that may run across batch elements (all rows at once
  // without a chunk); attention takes the same number of queries of every batch element, at most all T
  p.tc = (token_chunk <= 0 || token_chunk > R) ? (int)R : token_chunk;
  p.qc = std::min(p.tc, g.T);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
  p.off_x = take((size_t)R * g.D * 4);
  p.slot_bytes = align_up((size_t)R * g.D * 4);
  p.off_slots = off; off += p.slot_bytes * g.dev_slots;
  p.off_qkv = take((size_t)R * 3 * g.D * es);
  p.off_vt = take((size_t)g.B * g.D * attn_tp(g.T) * es);
  p.off_ao = take((size_t)R * g.D * es);
  p.off_xn = take((size_t)p.tc * g.D * es);
  p.off_hid = take((size_t)p.tc * g.mlp_ratio * g.D * es);
  p.off_t = take((size_t)p.tc * g.D * 4);
  p.total = off;
  return p;
}

inline size_t entry_bytes(const lc_dit_config& g) { return (size_t)g.B * g.T * g.D * 4; }
inline char* slot_ptr(lc_dit* c, int s) { return c->arena + c->plan.off_slots + c->plan.slot_bytes * s; }
// the six modulation vectors of every batch element for block blk: [B][6][D]
inline const float* mod_blk(const lc_dit* c, const float* mod, int blk) { return mod + (int64_t)blk * c->cfg.B * 6 * c->cfg.D; }

// y[rows][Cout] = x[rows][Cin] W^T + bias; x of the operand type, y fp32 (y32) or of the operand type
lc_status linear(lc_dit* c, const void* w, const float* bias, int Cin, int Cout, int64_t rows, const void* x, void* y, int y32,
                 int act = 0) {
  FusedDesc f;
  memset(&f, 0, sizeof f);
  f.dt = c->cfg.dtype; f.y_f32 = y32; f.taps = 1; f.src = 0; f.Cin = Cin; f.Cout = Cout; f.Cout_store = Cout; f.w = w; f.bias = bias;
  f.rows = rows; f.in_map = f.out_map = RowMap{0, 0, 1 << 30}; f.x = x; f.y = y; f.act = act;
  LCT_HIP(c, launch_fused(c->cs, f));
  return LC_OK;
}

// y = LN(x [+ add]) * (1 + scale) + shift for `rows` rows starting at row r0 of the step; the modulation vectors are
// those of each row's batch element
lc_status ln_mod(lc_dit* c, const float* x, const float* add, const float* mod, int which_shift, int which_scale, void* y, int rows,
                 int64_t r0) {
  const lc_dit_config& g = c->cfg;
  const unsigned blocks = (unsigned)((rows + 3) / 4);
  if (g.dtype == kBF16)
    ln_mod_kernel<bf16_t><<<blocks, 256, 0, c->cs>>>(x, add, mod, which_shift, which_scale, (bf16_t*)y, rows, g.D, g.ln_eps, r0, g.T);
  else
    ln_mod_kernel<float><<<blocks, 256, 0, c->cs>>>(x, add, mod, which_shift, which_scale, (float*)y, rows, g.D, g.ln_eps, r0, g.T);
  LCT_HIP(c, hipGetLastError());
  return LC_OK;
}

// dst += gate * t over `rows` rows starting at row r0 of the step (mod == nullptr: dst += t)
lc_status gate_add(lc_dit* c, float* dst, const float* t, const float* mod, int which, int64_t rows, int64_t r0) {
  const int64_t n4 = rows * c->cfg.D / 4;
  gate_add_kernel<<<(unsigned)((n4 + 255) / 256), 256, 0, c->cs>>>(dst, t, mod, which, n4, c->cfg.D / 4, r0, c->cfg.T);
  LCT_HIP(c, hipGetLastError());
  return LC_OK;
}

// One block. The hidden states entering it are x (+ delta when delta != nullptr); what it adds goes to dst
// (x itself outside the deep range, the Delta accumulator inside it).
lc_status run_block(lc_dit* c, int i, const float* mod, float* x, const float* delta, float* dst) {
  const lc_dit_config& g = c->cfg;
  const TPlan& p = c->plan;
  const int D = g.D, T = g.T, H = g.mlp_ratio * g.D, Tp = attn_tp(T);
  const int64_t R = (int64_t)g.B * T;
  const size_t es = dtype_size(g.dtype);
  const BlkW& w = c->blk[i];
  const float* m = mod_blk(c, mod, i);
  char* qkv = c->arena + p.off_qkv;
  char* vt = c->arena + p.off_vt;
  char* ao = c->arena + p.off_ao;
  char* xn = c->arena + p.off_xn;
  char* hid = c->arena + p.off_hid;
  float* t = (float*)(c->arena + p.off_t);
  lc_status s;
  // ---- attention branch: q,k,v of every token first
  for (int64_t r0 = 0; r0 < R; r0 += p.tc) {
    const int n = (int)std::min<int64_t>(p.tc, R - r0);
    if ((s = ln_mod(c, x + r0 * D, delta ? delta + r0 * D : nullptr, m, 0, 1, xn, n, r0)) != LC_OK) return s;
    if ((s = linear(c, w.wqkv, w.bqkv, D, 3 * D, n, xn, qkv + r0 * 3 * D * es, 0)) != LC_OK) return s;
  }
  LCT_HIP(c, launch_make_vt(c->cs, g.dtype, qkv + (size_t)2 * D * es, 3 * D, vt, g.B, T, Tp, D));
  for (int q0 = 0; q0 < T; q0 += p.qc)  // a chunk of queries of every batch element against all keys
    LCT_HIP(c, launch_spatial_attention(c->cs, g.dtype, qkv, 3 * D, vt, Tp, ao, g.B, T, g.heads, g.head_dim, q0, std::min(q0 + p.qc, T), 0));
  for (int64_t r0 = 0; r0 < R; r0 += p.tc) {
    const int n = (int)std::min<int64_t>(p.tc, R - r0);
    if ((s = linear(c, w.wo, w.bo, D, D, n, ao + r0 * D * es, t, 1)) != LC_OK) return s;
    if ((s = gate_add(c, dst + r0 * D, t, m, 2, n, r0)) != LC_OK) return s;
  }
  // ---- MLP branch, chunk by chunk
  for (int64_t r0 = 0; r0 < R; r0 += p.tc) {
    const int n = (int)std::min<int64_t>(p.tc, R - r0);
    if ((s = ln_mod(c, x + r0 * D, delta ? delta + r0 * D : nullptr, m, 3, 4, xn, n, r0)) != LC_OK) return s;
    // (a bf16 stage whose hidden width the dense-row kernel covers applies the GELU in that kernel's epilogue)
    const bool fused = g.dtype == kBF16 && (H % 160 == 0 || H % 128 == 0);
    if ((s = linear(c, w.w1, w.b1, D, H, n, xn, hid, 0, fused ? 1 : 0)) != LC_OK) return s;
    if (!fused) {
      const int64_t n16 = (int64_t)n * H * es / 16;
      if (g.dtype == kBF16) gelu_kernel<bf16_t><<<(unsigned)((n16 + 255) / 256), 256, 0, c->cs>>>((bf16_t*)hid, n16);
      else gelu_kernel<float><<<(unsigned)((n16 + 255) / 256), 256, 0, c->cs>>>((float*)hid, n16);
      LCT_HIP(c, hipGetLastError());
    }
    if ((s = linear(c, w.w2, w.b2, H, D, n, hid, t, 1)) != LC_OK) return s;
    if ((s = gate_add(c, dst + r0 * D, t, m, 5, n, r0)) != LC_OK) return s;
  }
  return LC_OK;
}

lc_status run_step(lc_dit* c, const void* x_in, const void* mod, void* x_out, int slot, bool full) {
  const lc_dit_config& g = c->cfg;
  const int64_t R = (int64_t)g.B * g.T;
  float* x = (float*)(c->arena + c->plan.off_x);
  float* delta = (float*)slot_ptr(c, slot);
  const float* m = (const float*)mod;
  LCT_HIP(c, hipMemcpyAsync(x, x_in, (size_t)R * g.D * 4, hipMemcpyDeviceToDevice, c->cs));
  lc_status s;
  for (int i = 0; i < g.cache_a; ++i)
    if ((s = run_block(c, i, m, x, nullptr, x)) != LC_OK) return s;
  if (full) {
    // the slot may still be the source of a swap-out or the target of a swap-in on the side stream
    LCT_HIP(c, hipStreamWaitEvent(c->cs, c->ev_rd_done[slot], 0));
    LCT_HIP(c, hipStreamWaitEvent(c->cs, c->ev_in_done[slot], 0));
    c->in_pending[slot] = 0;
    LCT_HIP(c, launch_fill_f32(c->cs, delta, R * g.D, 0.f));
    for (int i = g.cache_a; i < g.cache_b; ++i)
      if ((s = run_block(c, i, m, x, delta, delta)) != LC_OK) return s;
    LCT_HIP(c, hipEventRecord(c->ev_produced[slot], c->cs));
    c->dev_filled[slot] = 1;
  } else if (c->in_pending[slot]) {
    LCT_HIP(c, hipStreamWaitEvent(c->cs, c->ev_in_done[slot], 0));
    c->in_pending[slot] = 0;
  }
  if ((s = gate_add(c, x, delta, nullptr, 0, R, 0)) != LC_OK) return s;  // x_b = x_a + Delta, at both kinds of step
  LCT_HIP(c, hipEventRecord(c->ev_consumed[slot], c->cs));
  for (int i = g.cache_b; i < g.L; ++i)
    if ((s = run_block(c, i, m, x, nullptr, x)) != LC_OK) return s;
  LCT_HIP(c, hipMemcpyAsync(x_out, x, (size_t)R * g.D * 4, hipMemcpyDeviceToDevice, c->cs));
  return LC_OK;
}

lc_status step_checks(lc_dit* c, const void* x_in, const void* mod, void* x_out, int slot) {
  if (!c) return tfail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!x_in || !mod || !x_out) return tfail(c, LC_ERR_ARG, "x_in, mod and x_out must not be NULL");
  if (slot < 0 || slot >= c->cfg.dev_slots) return tfail(c, LC_ERR_ARG, "device slot %d out of range", slot);
  if (!c->have_weights) return tfail(c, LC_ERR_STATE, "weights not loaded");
  if (!c->arena) return tfail(c, LC_ERR_STATE, "workspace not set");
  return LC_OK;
}

}  // namespace

extern "C" {

const char* lc_dit_last_error(const lc_dit* c) { return c ? c->err.c_str() : g_terr.c_str(); }
lc_status lc_dit_check_config(const lc_dit_config* cfg) { return check_tcfg(nullptr, cfg); }
size_t lc_dit_entry_bytes(const lc_dit_config* cfg) { return check_tcfg(nullptr, cfg) == LC_OK ? entry_bytes(*cfg) : 0; }
size_t lc_dit_workspace_bytes(const lc_dit_config* cfg, int token_chunk) {
  if (check_tcfg(nullptr, cfg) != LC_OK) return 0;
  if (token_chunk < 0) { g_terr = "token_chunk must be >= 0"; return 0; }
  return make_tplan(*cfg, token_chunk).total;
}

lc_status lc_dit_destroy(lc_dit* c) {
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

lc_status lc_dit_create(const lc_dit_config* cfg, void* compute_stream, void* side_stream, lc_dit** out) {
  if (!out) return tfail(nullptr, LC_ERR_ARG, "out is NULL");
  lc_status s = check_tcfg(nullptr, cfg);
  if (s != LC_OK) return s;
  if (!compute_stream || !side_stream || compute_stream == side_stream)
    return tfail(nullptr, LC_ERR_ARG, "compute and side streams must be two distinct non-default streams");
  lc_dit* c = new (std::nothrow) lc_dit();
  if (!c) return tfail(nullptr, LC_ERR_NOMEM, "out of host memory");
  c->cfg = *cfg;
  c->cs = (hipStream_t)compute_stream; c->ss = (hipStream_t)side_stream;
  c->token_chunk = 0;
  c->plan = make_tplan(c->cfg, 0);
  c->arena = nullptr; c->arena_bytes = 0; c->have_weights = false; c->wblob = nullptr;
  c->full_steps = c->cached_steps = c->swaps_out = c->swaps_in = 0;
  for (int i = 0; i < cfg->host_slots; ++i) {
    void* p = nullptr;
    if (hipHostMalloc(&p, entry_bytes(*cfg), hipHostMallocDefault) != hipSuccess) {
      (void)hipGetLastError();
      lc_dit_destroy(c);
      return tfail(nullptr, LC_ERR_NOMEM, "hipHostMalloc (pinned cache bank) failed");
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
        lc_dit_destroy(c);
        return tfail(nullptr, LC_ERR_HIP, "hipEventCreate failed");
      }
      v->push_back(e);
    }
  *out = c;
  return LC_OK;
}

lc_status lc_dit_load_weights(lc_dit* c, const lc_dit_weights* w) {
  if (!c) return tfail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!w) return tfail(c, LC_ERR_ARG, "weights is NULL");
  const lc_dit_config& g = c->cfg;
  const int dt = g.dtype, D = g.D, H = g.mlp_ratio * g.D;
  const size_t es = dtype_size(dt);
  for (int i = 0; i < g.L; ++i) {
    const lc_dit_block_w& b = w->blk[i];
    if (!b.wqkv || !b.bqkv || !b.wo || !b.bo || !b.w1 || !b.b1 || !b.w2 || !b.b2) return tfail(c, LC_ERR_ARG, "a weight pointer of block %d is NULL", i);
  }
  const size_t per = align_up((size_t)3 * D * D * es) + align_up((size_t)D * D * es) + 2 * align_up((size_t)H * D * es) +
                     align_up((size_t)3 * D * 4) + 2 * align_up((size_t)D * 4) + align_up((size_t)H * 4);
  LCT_HIP(c, hipStreamSynchronize(c->cs));
  if (c->wblob) { LCT_HIP(c, hipFree(c->wblob)); c->wblob = nullptr; c->have_weights = false; }
  void* blob = nullptr;
  if (hipMalloc(&blob, per * g.L) != hipSuccess) return tfail(c, LC_ERR_NOMEM, "hipMalloc of %zu bytes for the weights failed", per * g.L);
  c->wblob = blob;
  c->blk.assign(g.L, BlkW{});
  char* p = (char*)blob;
  auto take = [&](size_t bytes) { char* o = p; p += align_up(bytes); return o; };
  for (int i = 0; i < g.L; ++i) {
    const lc_dit_block_w& b = w->blk[i];
    BlkW& k = c->blk[i];
    k.wqkv = take((size_t)3 * D * D * es); k.wo = take((size_t)D * D * es); k.w1 = take((size_t)H * D * es); k.w2 = take((size_t)H * D * es);
    k.bqkv = (float*)take((size_t)3 * D * 4); k.bo = (float*)take((size_t)D * 4); k.b1 = (float*)take((size_t)H * 4); k.b2 = (float*)take((size_t)D * 4);
    LCT_HIP(c, launch_copy_rows(c->cs, dt, b.wqkv, k.wqkv, (int64_t)3 * D * D));
    LCT_HIP(c, launch_copy_rows(c->cs, dt, b.wo, k.wo, (int64_t)D * D));
    LCT_HIP(c, launch_copy_rows(c->cs, dt, b.w1, k.w1, (int64_t)H * D));
    LCT_HIP(c, launch_copy_rows(c->cs, dt, b.w2, k.w2, (int64_t)H * D));
    LCT_HIP(c, launch_to_f32(c->cs, dt, b.bqkv, k.bqkv, 3 * D, 3 * D));
    LCT_HIP(c, launch_to_f32(c->cs, dt, b.bo, k.bo, D, D));
    LCT_HIP(c, launch_to_f32(c->cs, dt, b.b1, k.b1, H, H));
    LCT_HIP(c, launch_to_f32(c->cs, dt, b.b2, k.b2, D, D));
  }
  LCT_HIP(c, hipStreamSynchronize(c->cs));
  c->have_weights = true;
  return LC_OK;
}

lc_status lc_dit_set_workspace(lc_dit* c, void* arena, size_t bytes) {
  if (!c) return tfail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!arena) return tfail(c, LC_ERR_ARG, "arena is NULL");
  if ((uintptr_t)arena % kAlign) return tfail(c, LC_ERR_ARG, "arena must be 256-byte aligned");
  if (bytes < c->plan.total) return tfail(c, LC_ERR_NOMEM, "workspace of %zu bytes is smaller than the %zu needed", bytes, c->plan.total);
  LCT_HIP(c, hipStreamSynchronize(c->cs));
  LCT_HIP(c, hipStreamSynchronize(c->ss));
  c->arena = (char*)arena; c->arena_bytes = bytes;
  std::fill(c->dev_filled.begin(), c->dev_filled.end(), 0);
  std::fill(c->in_pending.begin(), c->in_pending.end(), 0);
  return LC_OK;
}

lc_status lc_dit_set_chunk(lc_dit* c, int token_chunk) {
  if (!c) return tfail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (token_chunk < 0) return tfail(c, LC_ERR_ARG, "token_chunk must be >= 0");
  TPlan np = make_tplan(c->cfg, token_chunk);
  if (c->arena && np.total > c->arena_bytes) return tfail(c, LC_ERR_NOMEM, "chunk setting needs %zu bytes, workspace has %zu", np.total, c->arena_bytes);
  c->token_chunk = token_chunk;  // (the hidden states and the slots sit at chunk-independent offsets)
  c->plan = np;
  return LC_OK;
}

lc_status lc_dit_full_step(lc_dit* c, const void* x_in, const void* mod, void* x_out, int dev_slot) {
  lc_status s = step_checks(c, x_in, mod, x_out, dev_slot);
  if (s != LC_OK) return s;
  s = run_step(c, x_in, mod, x_out, dev_slot, true);
  if (s == LC_OK) c->full_steps++;
  return s;
}

lc_status lc_dit_cached_step(lc_dit* c, const void* x_in, const void* mod, void* x_out, int dev_slot) {
  lc_status s = step_checks(c, x_in, mod, x_out, dev_slot);
  if (s != LC_OK) return s;
  if (!c->dev_filled[dev_slot]) return tfail(c, LC_ERR_STATE, "cached step on empty device slot %d", dev_slot);
  s = run_step(c, x_in, mod, x_out, dev_slot, false);
  if (s == LC_OK) c->cached_steps++;
  return s;
}

static lc_status dit_swap_common(lc_dit* c, int dev_slot, int host_slot) {
  if (!c) return tfail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (dev_slot < 0 || dev_slot >= c->cfg.dev_slots) return tfail(c, LC_ERR_ARG, "device slot %d out of range", dev_slot);
  if (host_slot < 0 || host_slot >= c->cfg.host_slots) return tfail(c, LC_ERR_ARG, "host slot %d out of range", host_slot);
  if (!c->arena) return tfail(c, LC_ERR_STATE, "workspace not set");
  return LC_OK;
}

lc_status lc_dit_swap_out(lc_dit* c, int dev_slot, int host_slot) {
  lc_status s = dit_swap_common(c, dev_slot, host_slot);
  if (s != LC_OK) return s;
  if (!c->dev_filled[dev_slot]) return tfail(c, LC_ERR_STATE, "swap-out of empty device slot %d", dev_slot);
  LCT_HIP(c, hipStreamWaitEvent(c->ss, c->ev_produced[dev_slot], 0));
  LCT_HIP(c, hipMemcpyAsync(c->host[host_slot], slot_ptr(c, dev_slot), entry_bytes(c->cfg), hipMemcpyDeviceToHost, c->ss));
  LCT_HIP(c, hipEventRecord(c->ev_rd_done[dev_slot], c->ss));
  c->host_filled[host_slot] = 1;
  c->swaps_out++;
  return LC_OK;
}

lc_status lc_dit_swap_in(lc_dit* c, int host_slot, int dev_slot) {
  lc_status s = dit_swap_common(c, dev_slot, host_slot);
  if (s != LC_OK) return s;
  if (!c->host_filled[host_slot]) return tfail(c, LC_ERR_STATE, "swap-in from empty host slot %d", host_slot);
  LCT_HIP(c, hipStreamWaitEvent(c->ss, c->ev_consumed[dev_slot], 0));
  LCT_HIP(c, hipStreamWaitEvent(c->ss, c->ev_produced[dev_slot], 0));
  LCT_HIP(c, hipMemcpyAsync(slot_ptr(c, dev_slot), c->host[host_slot], entry_bytes(c->cfg), hipMemcpyHostToDevice, c->ss));
  LCT_HIP(c, hipEventRecord(c->ev_in_done[dev_slot], c->ss));
  c->in_pending[dev_slot] = 1;
  c->dev_filled[dev_slot] = 1;
  c->swaps_in++;
  return LC_OK;
}

lc_status lc_dit_sync(lc_dit* c) {
  if (!c) return tfail(nullptr, LC_ERR_ARG, "ctx is NULL");
  LCT_HIP(c, hipStreamSynchronize(c->cs));
  LCT_HIP(c, hipStreamSynchronize(c->ss));
  return LC_OK;
}

lc_status lc_dit_cache_write(lc_dit* c, int dev_slot, const void* delta) {
  if (!c) return tfail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!delta) return tfail(c, LC_ERR_ARG, "delta is NULL");
  if (dev_slot < 0 || dev_slot >= c->cfg.dev_slots) return tfail(c, LC_ERR_ARG, "device slot %d out of range", dev_slot);
  if (!c->arena) return tfail(c, LC_ERR_STATE, "workspace not set");
  LCT_HIP(c, hipStreamWaitEvent(c->cs, c->ev_rd_done[dev_slot], 0));
  LCT_HIP(c, hipStreamWaitEvent(c->cs, c->ev_in_done[dev_slot], 0));
  c->in_pending[dev_slot] = 0;
  LCT_HIP(c, hipMemcpyAsync(slot_ptr(c, dev_slot), delta, entry_bytes(c->cfg), hipMemcpyDeviceToDevice, c->cs));
  LCT_HIP(c, hipEventRecord(c->ev_produced[dev_slot], c->cs));
  c->dev_filled[dev_slot] = 1;
  return LC_OK;
}

lc_status lc_dit_cache_peek(lc_dit* c, int host_slot, const void** ptr, size_t* bytes) {
  if (!c) return tfail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!ptr || !bytes) return tfail(c, LC_ERR_ARG, "output pointer is NULL");
  if (host_slot < 0 || host_slot >= c->cfg.host_slots) return tfail(c, LC_ERR_ARG, "host slot %d out of range", host_slot);
  if (!c->host_filled[host_slot]) return tfail(c, LC_ERR_STATE, "host slot %d is empty", host_slot);
  *ptr = c->host[host_slot];
  *bytes = entry_bytes(c->cfg);
  return LC_OK;
}

lc_status lc_dit_cache_dev_peek(lc_dit* c, int dev_slot, const void** ptr, size_t* bytes) {
  if (!c) return tfail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!ptr || !bytes) return tfail(c, LC_ERR_ARG, "output pointer is NULL");
  if (dev_slot < 0 || dev_slot >= c->cfg.dev_slots) return tfail(c, LC_ERR_ARG, "device slot %d out of range", dev_slot);
  if (!c->arena) return tfail(c, LC_ERR_STATE, "workspace not set");
  if (!c->dev_filled[dev_slot]) return tfail(c, LC_ERR_STATE, "device slot %d is empty", dev_slot);
  *ptr = slot_ptr(c, dev_slot);
  *bytes = entry_bytes(c->cfg);
  return LC_OK;
}

lc_status lc_dit_get_counts(lc_dit* c, int64_t* full_steps, int64_t* cached_steps, int64_t* swaps_out, int64_t* swaps_in) {
  if (!c) return tfail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!full_steps || !cached_steps || !swaps_out || !swaps_in) return tfail(c, LC_ERR_ARG, "output pointer is NULL");
  *full_steps = c->full_steps; *cached_steps = c->cached_steps; *swaps_out = c->swaps_out; *swaps_in = c->swaps_in;
  return LC_OK;
}

}  // extern "C"

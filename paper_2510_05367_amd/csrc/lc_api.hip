// Host side of the C ABI declared in include/lightcache.h: configuration checks, the arena plan
// (footprint model), packed weights, the step driver with its chunk loops, and the cache bank
// (pinned host entries, device slots, side-stream copies ordered by events).
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <set>
#include <string>
#include <vector>

#include "../../include/lightcache.h"
#include "lc_internal.h"

using namespace lc;

// Scratch of lc_cached_step_static: one array per GPU the library is loaded on, held until the process ends.
// Host code never uses this name as an address (it is only the host-side handle of the symbol): the device
// address is looked up once per device in lc_create (static_scratch_ptr) and that pointer is what kernels,
// and the arena plan, are given.
constexpr size_t kStaticScratchBytes = (size_t)LC_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char g_static_scratch[kStaticScratchBytes];

namespace {

thread_local std::string g_err = "";
thread_local int g_fail_host_alloc = 0;  // lc_test_fail_host_alloc: countdown to the pinned allocation that fails

// contexts that lc_create has handed out and lc_destroy has not yet taken back
std::mutex g_live_mu;
std::set<const lc_ctx*> g_live;

constexpr int kMaxDevices = 64;
void* g_static_ptr[kMaxDevices] = {nullptr};  // device address of g_static_scratch on each device (under g_live_mu)

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Plan {
  int fc, tc, qc;  // effective frame chunk, temporal position chunk, spatial query chunk
  int blocks;      // spatial blocks per frame (1: no spatial chunk)
  size_t off_h, off_slots, slot_bytes, off_partH, off_partT, off_partU, off_partD, partD_bytes, off_scale, off_shift, off_scale_cat,
      off_shift_cat, off_ws,
      ws_bytes, total;
  size_t lane_off, lane_stride;  // [lane_off, lane_off + lane_stride): the scratch one lane works in (see use_lane)
};

struct GnW { float *gamma, *beta; };
struct ConvW { void* w; float* b; void* wt; };  // wt: tile order for the specialised conv kernel, or nullptr
struct AttnW { GnW gn; void* wqkv; void* wo; float* bo; void* wqkv_f; void* wo_f; };  // *_f: fragment order
struct Packed {
  float* cin_w; float* cin_b;
  void* cin_wp;  // conv_in weights as rows [C][64] of the operand type (k = plane * 9 + tap, zero padded), or nullptr
  void* cin_wf;  // conv_in as a linear layer on gathered neighbourhoods: [C][64] in fragment order, or nullptr
  GnW res_gn[LC_MAX_RES]; ConvW res[LC_MAX_RES];
  AttnW sattn, tattn;
  ConvW down; GnW dres_gn; ConvW dres;
  GnW up_gn; ConvW up; GnW out_gn; ConvW out;
};

struct EvPair { hipEvent_t a, b; int kind; int64_t bytes; };
constexpr int kMaxLanes = 2;  // streams a chunked step can spread its chunks over (a third one measured no gain)

}  // namespace

struct lc_ctx {
  lc_config cfg;
  hipStream_t cs, ss;            // cs: the stream kernels are issued on right now (see use_lane)
  hipStream_t cs_main, cs_aux[kMaxLanes - 1];  // the caller's compute stream; the library's own further ones
  hipEvent_t ev_fork, ev_join[kMaxLanes - 1];
  int lanes;                     // 1 or 2: streams a chunked step spreads its chunks over
  bool conv_general;             // lc_set_conv_general: the specialised-wavefront conv kernel is not used
  int lane;                      // the lane in use: selects cs and the per-lane scratch
  bool forked;
  int device;
  int frame_chunk, token_chunk;
  int sp_eta, sp_omega;          // spatial chunk factors of lc_set_spatial_chunk (1, 1 = off)
  Plan plan;
  char* arena;
  size_t arena_bytes;
  bool have_weights;
  void* wblob;
  size_t wblob_bytes;
  Packed pw;
  // cache bank
  std::vector<void*> host;
  std::vector<char> host_filled, dev_filled;
  std::vector<hipEvent_t> ev_produced, ev_consumed, ev_in_done, ev_rd_done, ev_out_done;
  std::vector<char> in_pending;
  std::vector<char> deep_stat_valid;  // partD of the slot matches its contents
  // stats
  lc_stats st;
  std::vector<EvPair> copy_pool, copy_pending;
  // profiling
  uint32_t prof_mask;
  std::vector<EvPair> prof_pool;
  size_t prof_used;
  int64_t prof_dropped;  // launches that found the bracket pool empty since the last lc_get_profile
  void* static_scratch;  // this device's static scratch (lc_cached_step_static)
  std::string err;
};

namespace {

// Device address of this device's copy of the static scratch; looked up on first use, with `dev` current.
hipError_t static_scratch_ptr(int dev, void** out) {
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lk(g_live_mu);
  if (!g_static_ptr[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch));
    if (e != hipSuccess) return e;
    g_static_ptr[dev] = p;
  }
  *out = g_static_ptr[dev];
  return hipSuccess;
}

lc_status fail(lc_ctx* c, lc_status code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (c) c->err = buf; else g_err = buf;
  return code;
}

#define LC_HIP(c, expr)                                                                          \
  do {                                                                                           \
    hipError_t e_ = (expr);                                                                      \
    if (e_ != hipSuccess) return fail(c, LC_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_));   \
  } while (0)

void destroy_ctx(lc_ctx* c);  // frees everything a (possibly half-built) context owns

lc_status check_cfg(lc_ctx* c, const lc_config* g) {
  if (!g) return fail(c, LC_ERR_ARG, "config is NULL");
  if (g->dtype != LC_F32 && g->dtype != LC_BF16) return fail(c, LC_ERR_ARG, "dtype must be LC_F32 or LC_BF16");
  if (g->B <= 0 || g->F <= 0 || g->H <= 0 || g->W <= 0 || g->C_lat <= 0 || g->C <= 0 || g->C_deep <= 0 ||
      g->groups <= 0 || g->n_res < 0 || g->heads <= 0 || g->head_dim <= 0)
    return fail(c, LC_ERR_SHAPE, "all sizes must be positive");
  if (g->H % 2 || g->W % 2) return fail(c, LC_ERR_SHAPE, "H and W must be even (deep feature is at H/2 x W/2)");
  if (g->C % 64 || g->C_deep % 64) return fail(c, LC_ERR_SHAPE, "C and C_deep must be multiples of 64");
  if (g->C > 1024 || g->C_deep > 1024) return fail(c, LC_ERR_SHAPE, "C and C_deep must be <= 1024");
  if (g->C % g->groups || g->C_deep % g->groups || (g->C + g->C_deep) % g->groups)
    return fail(c, LC_ERR_SHAPE, "C, C_deep and C + C_deep must be divisible by groups");
  if ((g->C + g->C_deep) / g->groups > 512) return fail(c, LC_ERR_SHAPE, "at most 512 channels per group");
  if (g->heads * g->head_dim != g->C) return fail(c, LC_ERR_SHAPE, "heads * head_dim must equal C");
  const int d = g->head_dim;
  if (!(d == 8 || d == 16 || d == 32 || d == 40 || d == 64))
    return fail(c, LC_ERR_SHAPE, "head_dim must be one of 8, 16, 32, 40, 64");
  if (g->C_lat > 16) return fail(c, LC_ERR_SHAPE, "C_lat must be <= 16");
  if (g->n_res > LC_MAX_RES) return fail(c, LC_ERR_SHAPE, "n_res must be <= %d", LC_MAX_RES);
  if (g->dev_slots < 1 || g->dev_slots > 8) return fail(c, LC_ERR_SHAPE, "dev_slots must be in [1, 8]");
  if (g->host_slots < 0 || g->host_slots > 64) return fail(c, LC_ERR_SHAPE, "host_slots must be in [0, 64]");
  if (!(g->gn_eps > 0.f)) return fail(c, LC_ERR_SHAPE, "gn_eps must be positive");
  if ((int64_t)g->B * g->F * g->H * g->W > (int64_t)1 << 28) return fail(c, LC_ERR_SHAPE, "too many pixels");
  return LC_OK;
}

Plan make_plan(const lc_config& g, int frame_chunk, int token_chunk, int eta, int omega) {
  Plan p;
  const int64_t N = (int64_t)g.B * g.F, T = (int64_t)g.H * g.W;
  const size_t es = dtype_size(g.dtype);
  p.fc = (frame_chunk <= 0 || frame_chunk > N) ? (int)N : frame_chunk;
  if (token_chunk > 0) p.tc = (int)std::min<int64_t>(token_chunk, T);
  else if (p.fc < N) p.tc = (int)(((int64_t)p.fc * T + N - 1) / N);
  else p.tc = (int)T;
  // position chunks of the temporal block in whole 32-row tiles where the frame allows it (the
  // weight-stationary linear kernel works on such tiles)
  if (T % 32 == 0) p.tc = (int)std::min<int64_t>(T, ((int64_t)p.tc + 31) / 32 * 32);
  p.qc = token_chunk > 0 ? (int)std::min<int64_t>(token_chunk, T) : (int)T;
  // with a spatial chunk the position chunks of the temporal block and the query chunks are its blocks
  if (eta * omega > 1) p.tc = p.qc = (g.H / eta) * (g.W / omega);
  p.blocks = eta * omega;
  size_t off = 0;
  p.off_h = off; off += align_up((size_t)(N * T * g.C) * 4);  // the skip / residual stream is fp32
  p.slot_bytes = align_up((size_t)(N * (T / 4) * g.C_deep) * es);
  p.off_slots = off; off += p.slot_bytes * g.dev_slots;
  // GroupNorm partial sums [frame][split][channel][2]. The kernels that produce a normalised tensor
  // also write its partials, with their own split geometry (32-row tiles of the linear kernels,
  // 32-pixel quarter tiles of the 3x3 kernels); the stand-alone statistics kernel uses 64-row splits.
  // partH: the tensor at hand inside a frame chunk (also the half-resolution one of the deep stand-in);
  // partT / partU: input of the temporal block / skip input of the up block, written chunk by chunk
  // for all frames; partD: the cached deep feature, one region per device slot (kept while the slot
  // does not change) plus one for the single-operator entry points.
  size_t sp = std::max((size_t)stat_splits((int)T), (size_t)conv_stat_splits(g.H, g.W));
  if (T % 32 == 0) sp = std::max(sp, (size_t)(T / 32));
  const size_t ph = std::max(sp * g.C, (size_t)stat_splits((int)(T / 4)) * g.C_deep);
  p.off_partT = off; off += align_up((size_t)N * sp * g.C * 2 * sizeof(float));
  p.off_partU = off; off += align_up((size_t)N * sp * g.C * 2 * sizeof(float));
  p.partD_bytes = align_up((size_t)N * stat_splits((int)(T / 4)) * g.C_deep * 2 * sizeof(float));
  p.off_partD = off; off += p.partD_bytes * (g.dev_slots + 1);
  // scale / shift of the concatenated tensor of the up block for all frames: once the skip feature is
  // complete one launch folds them, instead of one launch at the head of every frame chunk
  p.off_scale_cat = off; off += align_up((size_t)N * (g.C + g.C_deep) * sizeof(float));
  p.off_shift_cat = off; off += align_up((size_t)N * (g.C + g.C_deep) * sizeof(float));
  // what a chunk works in - partH, scale / shift, the chunk scratch - exists once per lane: a chunked
  // step runs alternate chunks on two streams
  p.lane_off = off;
  p.off_partH = off; off += align_up((size_t)N * ph * 2 * sizeof(float));
  p.off_scale = off; off += align_up((size_t)N * (g.C + g.C_deep) * sizeof(float));
  p.off_shift = off; off += align_up((size_t)N * (g.C + g.C_deep) * sizeof(float));
  const int64_t pc = (int64_t)p.fc * T;   // pixels of a frame chunk
  const int64_t rt = N * p.tc;            // rows of a temporal pass
  // frame-chunk pass: ping-pong copy of the fp32 stream + q,k,v + attention output
  const int64_t Tp = attn_tp((int)T);  // V^T rows of the spatial kernel are padded to 64 tokens
  size_t wsb = (size_t)(pc * g.C) * 4 + (size_t)(3 * g.C * pc + (int64_t)p.fc * g.C * Tp) * es;
  wsb = std::max(wsb, (size_t)(4 * g.C * rt) * es);                 // temporal pass: q,k,v + attention output
  wsb = std::max(wsb, (size_t)((pc / 4) * (int64_t)g.C_deep) * 4);  // deep stand-in: fp32 d0
  wsb += 4 * kAlign;
  p.ws_bytes = align_up(wsb) + kAlign;
  p.off_ws = off; off += p.ws_bytes;
  p.lane_stride = off - p.lane_off;
  if (p.fc < N || p.tc < T) off += (kMaxLanes - 1) * p.lane_stride;  // the other lanes' copies
  p.total = off;
  return p;
}

struct Prof {
  lc_ctx* c; int kind; bool on; size_t idx;
  Prof(lc_ctx* c_, int k) : c(c_), kind(k), on(false), idx(0) {
    if ((c->prof_mask >> k) & 1u) {
      if (c->prof_used < c->prof_pool.size()) {
        idx = c->prof_used++;
        c->prof_pool[idx].kind = k;
        on = hipEventRecord(c->prof_pool[idx].a, c->cs) == hipSuccess;
        if (!on) { c->prof_used--; c->prof_dropped++; }
      } else {
        c->prof_dropped++;  // pool exhausted: the launch runs untimed and lc_get_profile says how many did
      }
    }
  }
  // the launcher declined the shape and nothing ran: give the bracket back (it is the newest one)
  void cancel() { if (on && idx + 1 == c->prof_used) { c->prof_used--; on = false; } }
  ~Prof() { if (on) (void)hipEventRecord(c->prof_pool[idx].b, c->cs); }
};

#define LC_LAUNCH(c, kind, expr)                                                                  \
  do {                                                                                            \
    hipError_t e_;                                                                                \
    { Prof pr_(c, kind); e_ = (expr); }                                                           \
    if (e_ != hipSuccess) return fail(c, LC_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_));     \
  } while (0)

inline char* slot_ptr(lc_ctx* c, int s) { return c->arena + c->plan.off_slots + c->plan.slot_bytes * s; }
inline char* h_ptr(lc_ctx* c) { return c->arena + c->plan.off_h; }
inline size_t lane_base(lc_ctx* c) { return c->lane * c->plan.lane_stride; }
inline float* partH(lc_ctx* c) { return (float*)(c->arena + lane_base(c) + c->plan.off_partH); }
inline float* partT(lc_ctx* c) { return (float*)(c->arena + c->plan.off_partT); }
inline float* partU(lc_ctx* c) { return (float*)(c->arena + c->plan.off_partU); }
// statistics of the deep feature in device slot `s`; s == dev_slots: scratch of the single-operator calls
inline float* partD(lc_ctx* c, int s) { return (float*)(c->arena + c->plan.off_partD + c->plan.partD_bytes * s); }
inline float* scale_p(lc_ctx* c) { return (float*)(c->arena + lane_base(c) + c->plan.off_scale); }
inline float* shift_p(lc_ctx* c) { return (float*)(c->arena + lane_base(c) + c->plan.off_shift); }
inline char* ws_ptr(lc_ctx* c) { return c->arena + lane_base(c) + c->plan.off_ws; }

RowMap dense_map() { return RowMap{0, 0, 1 << 30}; }

// The spatial blocks of a frame of H x W pixels under the current spatial chunk ("Feature chunk" section, eq.
// Chunk(F): H/eta x W/omega), in row-major order; one entry {0,0,0,0} = the whole frame when no chunk is set.
// `half`: blocks of the half-resolution grid (H, W are then already halved).
struct Blocks {
  int n;
  Win w[64];
};
Blocks blocks_of(const lc_ctx* c, int H, int W) {
  Blocks b;
  if (c->sp_eta * c->sp_omega <= 1) { b.n = 1; b.w[0] = Win{0, 0, 0, 0}; return b; }
  const int bh = H / c->sp_eta, bw = W / c->sp_omega;
  b.n = 0;
  for (int i = 0; i < c->sp_eta; ++i)
    for (int j = 0; j < c->sp_omega; ++j) b.w[b.n++] = Win{j * bw, i * bh, bw, bh};
  return b;
}
inline void set_conv_win(FusedDesc& d, Win w) { d.win_x0 = w.x0; d.win_y0 = w.y0; d.win_w = w.w; d.win_h = w.h; }
// token-indexed launch (taps == 1) over the rows of whole frames of H x W pixels
inline void set_row_win(FusedDesc& d, Win w, int H, int W, int in, int out) {
  set_conv_win(d, w);
  d.win_img_w = W; d.win_img_t = H; d.win_in = in; d.win_out = out;
}

// Two lanes. The chunks of a step depend on each other only at three points (before the temporal
// block, before the up branch, at the end), and nearly every kernel wants the whole device for a short
// time: run back to back on one stream, each pays its ramp-up and its tail, and the small ones
// (statistics, finalisation) leave most of the device idle. So alternate chunks go to two streams, each
// with its own scratch, and the device fills one chunk's gaps with the other's kernels. The results do
// not depend on it: the same kernels see the same data.
void use_lane(lc_ctx* c, int l) {
  c->lane = l;
  c->cs = l ? c->cs_aux[l - 1] : c->cs_main;
}
// lanes for a loop of n chunks; with per-kernel timing on, one (a bracketed kernel must run alone)
int loop_lanes(lc_ctx* c, int n) {
  const bool can = c->prof_mask == 0 && c->plan.total > c->plan.lane_off + c->plan.lane_stride;
  return can ? std::max(1, std::min(c->lanes, n)) : 1;
}
lc_status fork_lanes(lc_ctx* c) {
  LC_HIP(c, hipEventRecord(c->ev_fork, c->cs_main));
  for (int i = 0; i + 1 < c->lanes; ++i) LC_HIP(c, hipStreamWaitEvent(c->cs_aux[i], c->ev_fork, 0));
  c->forked = true;
  return LC_OK;
}
lc_status join_lanes(lc_ctx* c) {
  use_lane(c, 0);
  if (!c->forked) return LC_OK;
  c->forked = false;
  for (int i = 0; i + 1 < kMaxLanes; ++i) {  // (a lane that got no work joins at once)
    LC_HIP(c, hipEventRecord(c->ev_join[i], c->cs_aux[i]));
    LC_HIP(c, hipStreamWaitEvent(c->cs_main, c->ev_join[i], 0));
  }
  return LC_OK;
}

// Per-channel partial sums of the frames at hand, [frame][splits][C][2]; part == nullptr: none yet.
struct StatRef {
  const float* part;
  int splits;
};

// scale/shift (first `frames` entries of the scale/shift scratch) from partial sums
lc_status gn_from_stats(lc_ctx* c, StatRef st, int frames, int rows_per_frame, int C, const GnW& w) {
  const lc_config& g = c->cfg;
  LC_LAUNCH(c, LC_K_GN_FINAL,
            launch_gn_finalize(c->cs, st.part, C, st.splits, rows_per_frame, 1.f, nullptr, 0, 0, 0, 0.f, w.gamma, w.beta,
                               g.groups, g.gn_eps, scale_p(c), shift_p(c), frames));
  return LC_OK;
}

// GroupNorm statistics of `frames` contiguous frames of fp32 [rows_per_frame, C] -> scale/shift; `st`
// holds the partial sums if the kernel that wrote x produced them, else they are computed here.
lc_status gn_scale_shift(lc_ctx* c, const void* x, int frames, int rows_per_frame, int C, const GnW& w,
                         StatRef st = StatRef{nullptr, 0}) {
  if (!st.part) {
    LC_LAUNCH(c, LC_K_GN_STATS, launch_gn_stats(c->cs, kF32, x, partH(c), frames, rows_per_frame, C));
    st = StatRef{partH(c), stat_splits(rows_per_frame)};
  }
  return gn_from_stats(c, st, frames, rows_per_frame, C, w);
}

// A linear layer through the weight-stationary kernel, which can also write the statistics of its
// output (d.stat); shapes it does not cover go to the streaming kernel, which cannot. *wrote tells.
// The choice between the two must not depend on how the stage is chunked (a chunked step reproduces
// the unchunked one bit for bit, and the two kernels round differently): `tiled` says that the stage's
// geometry suits the weight-stationary kernel for every chunking (frames of a multiple of 32 positions).
lc_status linear(lc_ctx* c, int kind, FusedDesc d, bool* wrote_stats, bool tiled) {
  hipError_t e = hipErrorNotSupported;
  if (tiled) {
    Prof pr_(c, kind);
    e = launch_linear(c->cs, d);
    if (e == hipErrorNotSupported) pr_.cancel();
  }
  if (wrote_stats) *wrote_stats = e == hipSuccess && d.stat != nullptr;
  if (e == hipErrorNotSupported) {
    d.stat = nullptr;
    Prof pr_(c, kind);
    e = launch_fused(c->cs, d);
  }
  if (e != hipSuccess) return fail(c, LC_ERR_HIP, "linear layer: %s", hipGetErrorString(e));
  return LC_OK;
}

ConvDesc down_desc(const lc_config& g, const ConvW& w, int frames, const void* x, void* y) {
  ConvDesc d;
  memset(&d, 0, sizeof d);
  d.dt = g.dtype; d.x_f32 = 1; d.y_f32 = 1; d.taps = 9; d.stride = 2; d.Cin = g.C; d.Cout = g.C_deep;
  d.Cout_store = g.C_deep; d.w = w.w; d.bias = w.b; d.frames = frames; d.H = g.H; d.W = g.W;
  d.x = x; d.res = nullptr; d.y = y; d.out_map = dense_map();
  return d;
}

// 3x3 stride-1 convolution whose loader applies scale/shift (+ SiLU) to the fp32 tensor x.
FusedDesc fconv_desc(lc_ctx* c, const ConvW& w, int Cin, int Cout, int frames, int H, int W, const void* x,
                     const void* res, void* y, int y_f32) {
  FusedDesc d;
  memset(&d, 0, sizeof d);
  d.dt = c->cfg.dtype; d.y_f32 = y_f32; d.taps = 9; d.src = 2; d.Cin = Cin; d.Cout = Cout; d.Cout_store = Cout;
  d.w = w.w; d.w_tiles = c->conv_general ? nullptr : w.wt; d.bias = w.b; d.frames = frames; d.H = H; d.W = W; d.x = x; d.scale = scale_p(c); d.shift = shift_p(c);
  d.res = res; d.y = y; d.in_map = dense_map(); d.out_map = dense_map();
  return d;
}

FusedDesc flinear_desc(lc_ctx* c, const void* w, const void* w_frag, const float* bias, int Cin, int Cout, int64_t rows, int src,
                       RowMap in_map, RowMap out_map, const void* x, const void* res, void* y, int y_f32) {
  FusedDesc d;
  memset(&d, 0, sizeof d);
  d.dt = c->cfg.dtype; d.y_f32 = y_f32; d.taps = 1; d.src = src; d.Cin = Cin; d.Cout = Cout; d.Cout_store = Cout;
  d.w = w; d.w_frag = w_frag; d.bias = bias; d.rows = rows; d.in_map = in_map; d.out_map = out_map; d.x = x;
  d.scale = scale_p(c); d.shift = shift_p(c); d.res = res; d.y = y;
  return d;
}

// h = conv3x3(x): x planar [frames][C_lat][H][W] of the operand type, h fp32 rows. With `stat` the
// partial sums of h are written too ([frame][T/32][C][2]; T must be a multiple of 32); *wrote tells
// whether the kernel that ran could do that.
lc_status conv_in_block(lc_ctx* c, const void* x, void* h, int frames, float* stat, bool* wrote_stats, Win win);
lc_status conv_in_run(lc_ctx* c, const void* x, void* h, int frames, float* stat, bool* wrote_stats) {
  const Blocks bl = blocks_of(c, c->cfg.H, c->cfg.W);
  for (int i = 0; i < bl.n; ++i) {  // (every block runs the same kernel: *wrote_stats is that of any of them)
    const lc_status s = conv_in_block(c, x, h, frames, stat, wrote_stats, bl.w[i]);
    if (s != LC_OK) return s;
  }
  return LC_OK;
}
lc_status conv_in_block(lc_ctx* c, const void* x, void* h, int frames, float* stat, bool* wrote_stats, Win win) {
  const lc_config& g = c->cfg;
  const int T = g.H * g.W;
  if (wrote_stats) *wrote_stats = false;
  if (c->pw.cin_wp) {  // (a property of the stage's geometry: the same kernel for every chunking)
    hipError_t e;
    {
      Prof pr_(c, LC_K_CONV_IN);
      e = launch_conv_in_tile(c->cs, g.dtype, x, c->pw.cin_wp, c->pw.cin_b, (float*)h, stat, frames, g.H, g.W, g.C_lat, g.C, win);
      if (e == hipErrorNotSupported) pr_.cancel();
    }
    if (e == hipSuccess) {
      if (wrote_stats) *wrote_stats = stat != nullptr;
      return LC_OK;
    }
    if (e != hipErrorNotSupported) return fail(c, LC_ERR_HIP, "conv_in: %s", hipGetErrorString(e));
  }
  if (c->pw.cin_wf && T % 32 == 0) {  // (the same kernel for every chunking: see linear())
    FusedDesc d;
    memset(&d, 0, sizeof d);
    d.dt = g.dtype; d.y_f32 = 1; d.taps = 1; d.src = 2; d.Cin = 64; d.Cs = g.C_lat; d.Cout = g.C; d.Cout_store = g.C;
    d.w_frag = c->pw.cin_wf; d.bias = c->pw.cin_b; d.frames = frames; d.H = g.H; d.W = g.W;
    d.rows = (int64_t)frames * T; d.in_map = dense_map(); d.out_map = dense_map(); d.x = x; d.y = h;
    if (stat && T % 32 == 0) { d.stat = stat; d.stat_splits = T / 32; d.stat_rps = T; d.stat_off = 0; }
    if (win.w) set_row_win(d, win, g.H, g.W, 1, 1);
    hipError_t e;
    {
      Prof pr_(c, LC_K_CONV_IN);
      e = launch_linear(c->cs, d);
      if (e == hipErrorNotSupported) pr_.cancel();
    }
    if (e == hipSuccess) {
      if (wrote_stats) *wrote_stats = d.stat != nullptr;
      return LC_OK;
    }
    if (e != hipErrorNotSupported) return fail(c, LC_ERR_HIP, "conv_in: %s", hipGetErrorString(e));
  }
  if (win.w) return fail(c, LC_ERR_SHAPE, "conv_in of this stage has no spatially chunked kernel");
  LC_LAUNCH(c, LC_K_CONV_IN, launch_conv_in(c->cs, g.dtype, x, h, frames, g.H, g.W, g.C_lat, g.C, c->pw.cin_w, c->pw.cin_b));
  return LC_OK;
}

// residual block body: y = x + conv3x3(SiLU(GN(x))); x fp32 [frames][H*W][Cn]; y must not alias x.
// `in`: partial sums of x if its producer wrote them. `out` (fp32 y only): receives the partial sums of y.
lc_status res_block(lc_ctx* c, const GnW& gn, const ConvW& cw, int Cn, int frames, int H, int W, const void* x,
                    void* y, int y_f32, int kind, StatRef in = StatRef{nullptr, 0}, StatRef* out = nullptr) {
  lc_status s = gn_scale_shift(c, x, frames, H * W, Cn, gn, in);
  if (s != LC_OK) return s;
  FusedDesc d = fconv_desc(c, cw, Cn, Cn, frames, H, W, x, x, y, y_f32);
  if (out && (y_f32 || c->cfg.dtype == kF32)) {
    d.stat = partH(c);  // the partials of x have been folded into scale/shift by now
    d.stat_splits = conv_stat_splits(H, W);
    *out = StatRef{d.stat, d.stat_splits};
  } else if (out) {
    *out = StatRef{nullptr, 0};
  }
  // (the residual block at C_deep of the normal step's stand-in runs on whole frames: it is not on the cache step)
  const Blocks bl = kind == LC_K_DEEP ? Blocks{1, {Win{0, 0, 0, 0}}} : blocks_of(c, H, W);
  for (int i = 0; i < bl.n; ++i) {
    set_conv_win(d, bl.w[i]);
    LC_LAUNCH(c, kind, launch_fused(c->cs, d));
  }
  return LC_OK;
}

// u = conv3x3(SiLU(GN(Concat(skip, up2(deep))))). `skip_st`: partial sums of the skip feature if its
// producer wrote them; `deep_part`: those of the deep feature ([frame][stat_splits(T/4)][Cd][2]) if
// already known, else they are computed into the scratch region; `out` receives those of u.
// `sc`, `sh`: scale / shift of these frames if already folded (then the partial sums are not looked at).
lc_status up_conv(lc_ctx* c, const void* skip, const void* deep, void* u, int frames, StatRef skip_st = StatRef{nullptr, 0},
                  const float* deep_part = nullptr, StatRef* out = nullptr, const float* sc = nullptr,
                  const float* sh = nullptr) {
  const lc_config& g = c->cfg;
  const int T = g.H * g.W, C = g.C, Cd = g.C_deep;
  if (sc && sh) {
    FusedDesc d = fconv_desc(c, c->pw.up, C + Cd, C, frames, g.H, g.W, skip, nullptr, u, 1);
    d.src = 3; d.x2 = deep; d.Cs = C; d.scale = sc; d.shift = sh;
    if (out) {
      d.stat = partH(c);
      d.stat_splits = conv_stat_splits(g.H, g.W);
      *out = StatRef{d.stat, d.stat_splits};
    }
    const Blocks bl = blocks_of(c, g.H, g.W);
    for (int i = 0; i < bl.n; ++i) {
      set_conv_win(d, bl.w[i]);
      LC_LAUNCH(c, LC_K_CONV_UP, launch_fused(c->cs, d));
    }
    return LC_OK;
  }
  if (!skip_st.part) {
    LC_LAUNCH(c, LC_K_GN_STATS, launch_gn_stats(c->cs, kF32, skip, partH(c), frames, T, C));
    skip_st = StatRef{partH(c), stat_splits(T)};
  }
  if (!deep_part) {
    float* pd = partD(c, g.dev_slots);
    LC_LAUNCH(c, LC_K_GN_STATS, launch_gn_stats(c->cs, g.dtype, deep, pd, frames, T / 4, Cd));
    deep_part = pd;
  }
  LC_LAUNCH(c, LC_K_GN_FINAL,
            launch_gn_finalize(c->cs, skip_st.part, C, skip_st.splits, T, 1.f, deep_part, Cd, stat_splits(T / 4), T / 4, 4.f,
                               c->pw.up_gn.gamma, c->pw.up_gn.beta, g.groups, g.gn_eps, scale_p(c), shift_p(c), frames));
  FusedDesc d = fconv_desc(c, c->pw.up, C + Cd, C, frames, g.H, g.W, skip, nullptr, u, 1);
  d.src = 3; d.x2 = deep; d.Cs = C;
  if (out) {
    d.stat = partH(c);
    d.stat_splits = conv_stat_splits(g.H, g.W);
    *out = StatRef{d.stat, d.stat_splits};
  }
  const Blocks bl = blocks_of(c, g.H, g.W);
  for (int i = 0; i < bl.n; ++i) {
    set_conv_win(d, bl.w[i]);
    LC_LAUNCH(c, LC_K_CONV_UP, launch_fused(c->cs, d));
  }
  return LC_OK;
}

// eps = conv_out(SiLU(GN(u))), planar output of the operand type
lc_status conv_out(lc_ctx* c, const void* u, void* eps, int frames, StatRef u_st = StatRef{nullptr, 0}) {
  const lc_config& g = c->cfg;
  lc_status s = gn_scale_shift(c, u, frames, g.H * g.W, g.C, c->pw.out_gn, u_st);
  if (s != LC_OK) return s;
  const Blocks bl = blocks_of(c, g.H, g.W);
  for (int i = 0; i < bl.n; ++i) {
    // the tile kernel where the stage's geometry allows it (a property of the stage, not of the chunk)
    hipError_t e;
    {
      Prof pr_(c, LC_K_CONV_OUT);
      e = launch_conv_out_tile(c->cs, g.dtype, u, scale_p(c), shift_p(c), c->pw.out.w, c->pw.out.b, eps, frames, g.H, g.W, g.C,
                               g.C_lat, bl.w[i]);
      if (e == hipErrorNotSupported) pr_.cancel();
    }
    if (e == hipSuccess) continue;
    if (e != hipErrorNotSupported) return fail(c, LC_ERR_HIP, "conv_out: %s", hipGetErrorString(e));
    FusedDesc d = fconv_desc(c, c->pw.out, g.C, 32, frames, g.H, g.W, u, nullptr, eps, 0);
    d.Cout_store = g.C_lat;
    d.planar_out = 1;
    set_conv_win(d, bl.w[i]);
    LC_LAUNCH(c, LC_K_CONV_OUT, launch_fused(c->cs, d));
  }
  return LC_OK;
}

// Spatial attention block of `nf` frames, in place on the fp32 rows hc [nf*T][C]:
// hc += proj(Attn_spatial(qkv(GroupNorm(hc)))), queries in chunks of plan.qc tokens. `scr`: scratch for q,k rows,
// V^T and the attention output of these frames. `st`: partial sums of hc if its producer wrote them. `stat_out`:
// where the partial sums of the result go ([frame][T/32][C][2]) or nullptr; *wrote tells whether they were written.
lc_status spatial_block(lc_ctx* c, char* hc, char* scr, int nf, StatRef st, float* stat_out, bool* wrote) {
  const lc_config& g = c->cfg;
  const int T = g.H * g.W, C = g.C;
  const size_t es = dtype_size(g.dtype);
  const int64_t pc = (int64_t)nf * T;
  const bool tiled = T % 32 == 0;  // whole 32-row tiles in every frame: see linear()
  const int Tp = attn_tp(T);
  char* qk = scr;                                               // q,k rows [pc][2C]
  char* vt = qk + align_up((size_t)pc * 2 * C * es);            // V^T [nf][C][Tp]
  char* ao = vt + align_up((size_t)nf * C * Tp * es);
  const AttnW& a = c->pw.sattn;
  if (wrote) *wrote = false;
  lc_status s = gn_scale_shift(c, hc, nf, T, C, a.gn, st);
  if (s != LC_OK) return s;
  RowMap fm{0, T, T};  // dense rows; frame of row r = r / T
  const Blocks bl = blocks_of(c, g.H, g.W);
  // With a spatial chunk every operator below runs block by block; a block's queries attend to the keys and
  // values of the whole frame, so the q,k,v projection of all blocks comes first.
  for (int i = 0; i < bl.n; ++i) {
    // q and k as rows, v transposed straight from the GEMM epilogue into the layout the attention
    // kernel stages (no scattered transposition later)
    FusedDesc d = flinear_desc(c, a.wqkv, a.wqkv_f, nullptr, C, 3 * C, pc, 1, fm, dense_map(), hc, nullptr, qk, 0);
    d.yt = vt; d.yt_from = 2 * C; d.yt_T = T; d.yt_Tp = Tp;
    d.q_scale = attn_q_scale(g.head_dim); d.q_cols = C;  // the softmax scale rides on q, applied before rounding
    if (bl.w[i].w) set_row_win(d, bl.w[i], g.H, g.W, 1, 1);
    s = linear(c, LC_K_QKV, d, nullptr, tiled);
    if (s != LC_OK) return s;
  }
  for (int i = 0; i < bl.n; ++i) {
    const Win w = bl.w[i];
    if (w.w) {
      LC_LAUNCH(c, LC_K_SATTN, launch_spatial_attention_window(c->cs, g.dtype, qk, 2 * C, vt, Tp, ao, nf, T, g.heads, g.head_dim,
                                                               w.y0 * g.W + w.x0, w.w * w.h, w.w, g.W, 1));
    } else {
      for (int q0 = 0; q0 < T; q0 += c->plan.qc)
        LC_LAUNCH(c, LC_K_SATTN, launch_spatial_attention(c->cs, g.dtype, qk, 2 * C, vt, Tp, ao, nf, T, g.heads,
                                                          g.head_dim, q0, std::min(q0 + c->plan.qc, T), 1));
    }
  }
  // the output projection closes the block; its partial sums are those of the next GroupNorm's input
  bool all = true;
  for (int i = 0; i < bl.n; ++i) {
    FusedDesc d = flinear_desc(c, a.wo, a.wo_f, a.bo, C, C, pc, 0, dense_map(), dense_map(), ao, hc, hc, 1);
    if (stat_out) { d.stat = stat_out; d.stat_splits = T / 32; d.stat_rps = T; d.stat_off = 0; }
    if (bl.w[i].w) set_row_win(d, bl.w[i], g.H, g.W, 1, 1);
    bool wr = false;
    s = linear(c, LC_K_PROJ, d, &wr, tiled);
    if (s != LC_OK) return s;
    all = all && wr;
  }
  if (wrote) *wrote = all;
  return LC_OK;
}

// Temporal attention block over all N frames, in place on h [N*T][C] (fp32), per position chunk of plan.tc
// positions on the lanes: h += proj(Attn_temporal(qkv(GroupNorm(h)))), statistics per whole frame. `tst`: partial
// sums of h if its producers wrote them. *ustat: in, whether the partial sums of the result may go to partU;
// out, whether they were written.
lc_status temporal_block(lc_ctx* c, char* h, StatRef tst, bool* ustat) {
  const lc_config& g = c->cfg;
  const Plan& p = c->plan;
  const int N = g.B * g.F, T = g.H * g.W, C = g.C;
  const size_t es = dtype_size(g.dtype);
  const bool tiled = T % 32 == 0;
  const AttnW& a = c->pw.tattn;
  lc_status s = gn_scale_shift(c, h, N, T, C, a.gn, tst);
  if (s != LC_OK) return s;
  const float *sc0 = scale_p(c), *sh0 = shift_p(c);  // of all frames: every position chunk reads them, on either lane
  const Blocks bl = blocks_of(c, g.H, g.W);
  const bool spatial = bl.w[0].w != 0;  // position chunks = the blocks of the spatial chunk
  const int nchunks = spatial ? bl.n : (T + p.tc - 1) / p.tc;
  const int pos_lanes = loop_lanes(c, nchunks);
  if (pos_lanes > 1 && (s = fork_lanes(c)) != LC_OK) return s;
  for (int ci = 0; ci < nchunks; ++ci) {
    use_lane(c, ci % pos_lanes);
    char* ws = ws_ptr(c);
    const int p0 = spatial ? 0 : ci * p.tc;
    const int np = spatial ? bl.w[ci].w * bl.w[ci].h : std::min(p.tc, T - p0);
    const int64_t rows = (int64_t)N * np;
    // dense row r of a pass = (frame r / np, the r % np-th position of the chunk)
    RowMap m{p0, T, np};
    RowMap whole{0, T, T};
    char* qkv = ws;
    char* ao = ws + align_up((size_t)rows * 3 * C * es);
    FusedDesc dq = flinear_desc(c, a.wqkv, a.wqkv_f, nullptr, C, 3 * C, spatial ? (int64_t)N * T : rows, 1, spatial ? whole : m,
                                dense_map(), h, nullptr, qkv, 0);
    dq.scale = sc0; dq.shift = sh0;
    if (spatial) set_row_win(dq, bl.w[ci], g.H, g.W, 1, 0);
    s = linear(c, LC_K_QKV, dq, nullptr, tiled);
    if (s != LC_OK) return s;
    LC_LAUNCH(c, LC_K_TATTN, launch_temporal_attention(c->cs, g.dtype, qkv, ao, g.B, g.F, np, g.heads, g.head_dim));
    // this projection finishes the skip feature: its partial sums, for the up block, go to partU
    FusedDesc d = flinear_desc(c, a.wo, a.wo_f, a.bo, C, C, spatial ? (int64_t)N * T : rows, 0, dense_map(), spatial ? whole : m,
                               ao, h, h, 1);
    if (*ustat) {
      d.stat = partU(c); d.stat_splits = T / 32;
      d.stat_rps = spatial ? T : np; d.stat_off = spatial ? 0 : p0;
    }
    if (spatial) set_row_win(d, bl.w[ci], g.H, g.W, 0, 1);
    bool wrote = false;
    s = linear(c, LC_K_PROJ, d, &wrote, tiled);
    if (s != LC_OK) return s;
    *ustat = *ustat && wrote;
  }
  return join_lanes(c);
}

lc_status run_step_lanes(lc_ctx* c, const void* x, void* eps, int slot, bool full) {
  const lc_config& g = c->cfg;
  const Plan& p = c->plan;
  const int N = g.B * g.F, T = g.H * g.W, C = g.C, Cd = g.C_deep;
  const size_t es = dtype_size(g.dtype);
  char* h = h_ptr(c);
  const Packed& w = c->pw;
  const int frame_lanes = loop_lanes(c, (N + p.fc - 1) / p.fc);

  // ---- shallow down branch D_m, per frame chunk
  const bool tiled = T % 32 == 0;  // whole 32-row tiles in every frame and position chunk: see linear()
  bool tstat = tiled;              // the 32-row tiles of the projection kernels stay inside a frame
  if (frame_lanes > 1) { lc_status s = fork_lanes(c); if (s != LC_OK) return s; }
  for (int n0 = 0, ci = 0; n0 < N; n0 += p.fc, ++ci) {
    use_lane(c, ci % frame_lanes);
    char* ws = ws_ptr(c);
    const int nf = std::min(p.fc, N - n0);
    const int64_t pc = (int64_t)nf * T;
    char* hc = h + (size_t)n0 * T * C * 4;
    char* hb = ws;                                           // fp32 ping-pong partner of hc
    // a 3x3 convolution cannot run in place (its halo reads rows other workgroups write), so the
    // residual blocks alternate between hc and hb; start so that the last one lands in hc
    char* cur = (g.n_res % 2 == 0) ? hc : hb;
    // every kernel below that writes the fp32 stream also writes the partial sums of what it wrote,
    // for the GroupNorm that reads it next (where its tiles fit the frame; else they are computed apart)
    StatRef st{nullptr, 0};
    {
      bool wrote = false;
      lc_status s = conv_in_run(c, (const char*)x + (size_t)n0 * g.C_lat * T * es, cur, nf, partH(c), &wrote);
      if (s != LC_OK) return s;
      if (wrote) st = StatRef{partH(c), T / 32};
    }
    for (int i = 0; i < g.n_res; ++i) {
      char* nxt = cur == hc ? hb : hc;
      lc_status s = res_block(c, w.res_gn[i], w.res[i], C, nf, g.H, g.W, cur, nxt, 1, LC_K_CONV_RES, st, &st);
      if (s != LC_OK) return s;
      cur = nxt;
    }
    {
      bool wrote = false;
      lc_status s = spatial_block(c, hc, ws + align_up((size_t)pc * C * 4), nf, st,
                                  tstat ? partT(c) + (size_t)n0 * (T / 32) * C * 2 : nullptr, &wrote);
      if (s != LC_OK) return s;
      tstat = tstat && wrote;
    }
  }
  {
    lc_status s = join_lanes(c);
    if (s != LC_OK) return s;
  }

  // ---- temporal block: per-frame statistics over whole frames, then per position chunk
  bool ustat = T % 32 == 0 && p.tc % 32 == 0;  // the 32-row tiles of a position chunk stay inside a frame and a split
  {
    lc_status s = temporal_block(c, h, tstat ? StatRef{partT(c), T / 32} : StatRef{nullptr, 0}, &ustat);
    if (s != LC_OK) return s;
  }

  char* deep = slot_ptr(c, slot);
  if (full) {
    // the slot may still be the source of a swap-out or the target of a swap-in on the side stream
    LC_HIP(c, hipStreamWaitEvent(c->cs, c->ev_rd_done[slot], 0));
    LC_HIP(c, hipStreamWaitEvent(c->cs, c->ev_in_done[slot], 0));
    c->in_pending[slot] = 0;
    if (frame_lanes > 1) { lc_status s = fork_lanes(c); if (s != LC_OK) return s; }
    for (int n0 = 0, ci = 0; n0 < N; n0 += p.fc, ++ci) {
      use_lane(c, ci % frame_lanes);
      const int nf = std::min(p.fc, N - n0);
      char* hc = h + (size_t)n0 * T * C * 4;
      char* d0 = ws_ptr(c);  // fp32
      char* dc = deep + (size_t)n0 * (T / 4) * Cd * es;
      LC_LAUNCH(c, LC_K_DEEP, launch_conv(c->cs, down_desc(g, w.down, nf, hc, d0)));
      lc_status s = res_block(c, w.dres_gn, w.dres, Cd, nf, g.H / 2, g.W / 2, d0, dc, 0, LC_K_DEEP);
      if (s != LC_OK) return s;
    }
    {
      lc_status s = join_lanes(c);
      if (s != LC_OK) return s;
    }
    LC_HIP(c, hipEventRecord(c->ev_produced[slot], c->cs));
    c->dev_filled[slot] = 1;
    c->deep_stat_valid[slot] = 0;
  } else if (c->in_pending[slot]) {
    LC_HIP(c, hipStreamWaitEvent(c->cs, c->ev_in_done[slot], 0));
    c->in_pending[slot] = 0;
  }

  // statistics of the cached deep feature: once per content of the slot, all frames in one launch
  if (!c->deep_stat_valid[slot]) {
    LC_LAUNCH(c, LC_K_GN_STATS, launch_gn_stats(c->cs, g.dtype, deep, partD(c, slot), N, T / 4, Cd));
    c->deep_stat_valid[slot] = 1;
  }

  // ---- shallow up branch U_m on Concat(skip, up2(deep)), per frame chunk
  // with the partial sums of the whole skip feature at hand, its GroupNorm is folded for all frames at once
  float* sc_cat = nullptr;
  float* sh_cat = nullptr;
  if (ustat) {
    sc_cat = (float*)(c->arena + p.off_scale_cat);
    sh_cat = (float*)(c->arena + p.off_shift_cat);
    LC_LAUNCH(c, LC_K_GN_FINAL,
              launch_gn_finalize(c->cs, partU(c), C, T / 32, T, 1.f, partD(c, slot), Cd, stat_splits(T / 4), T / 4, 4.f,
                                 w.up_gn.gamma, w.up_gn.beta, g.groups, g.gn_eps, sc_cat, sh_cat, N));
  }
  if (frame_lanes > 1) { lc_status s = fork_lanes(c); if (s != LC_OK) return s; }
  for (int n0 = 0, ci = 0; n0 < N; n0 += p.fc, ++ci) {
    use_lane(c, ci % frame_lanes);
    const int nf = std::min(p.fc, N - n0);
    char* hc = h + (size_t)n0 * T * C * 4;
    char* dc = deep + (size_t)n0 * (T / 4) * Cd * es;
    char* u = ws_ptr(c);  // fp32
    StatRef ust{nullptr, 0};
    lc_status s = up_conv(c, hc, dc, u, nf, ustat ? StatRef{partU(c) + (size_t)n0 * (T / 32) * C * 2, T / 32} : StatRef{nullptr, 0},
                          partD(c, slot) + (size_t)n0 * stat_splits(T / 4) * Cd * 2, &ust,
                          sc_cat ? sc_cat + (size_t)n0 * (C + Cd) : nullptr, sh_cat ? sh_cat + (size_t)n0 * (C + Cd) : nullptr);
    if (s != LC_OK) return s;
    s = conv_out(c, u, (char*)eps + (size_t)n0 * g.C_lat * T * es, nf, ust);
    if (s != LC_OK) return s;
  }
  {
    lc_status s = join_lanes(c);
    if (s != LC_OK) return s;
  }
  LC_HIP(c, hipEventRecord(c->ev_consumed[slot], c->cs));
  return LC_OK;
}

lc_status run_step(lc_ctx* c, const void* x, void* eps, int slot, bool full) {
  const lc_status s = run_step_lanes(c, x, eps, slot, full);
  if (s != LC_OK) {  // leave the streams joined and the first lane selected whatever happened
    const std::string keep = c->err;
    (void)join_lanes(c);
    c->err = keep;
  }
  return s;
}

lc_status step_checks(lc_ctx* c, const void* x, void* eps, int slot) {
  if (!c) return fail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!x || !eps) return fail(c, LC_ERR_ARG, "x and eps must not be NULL");
  if (slot < 0 || slot >= c->cfg.dev_slots) return fail(c, LC_ERR_ARG, "device slot %d out of range", slot);
  if (!c->have_weights) return fail(c, LC_ERR_STATE, "weights not loaded");
  if (!c->arena) return fail(c, LC_ERR_STATE, "workspace not set");
  return LC_OK;
}

lc_status op_checks(lc_ctx* c, int frames) {
  if (!c) return fail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!c->have_weights) return fail(c, LC_ERR_STATE, "weights not loaded");
  if (!c->arena) return fail(c, LC_ERR_STATE, "workspace not set");
  if (frames <= 0 || frames > c->cfg.B * c->cfg.F) return fail(c, LC_ERR_ARG, "frames out of range");
  return LC_OK;
}

}  // namespace

// =================================================================================================
extern "C" {

const char* lc_last_error(const lc_ctx* ctx) { return ctx ? ctx->err.c_str() : g_err.c_str(); }

lc_status lc_check_config(const lc_config* cfg) { return check_cfg(nullptr, cfg); }

size_t lc_cache_entry_bytes(const lc_config* cfg) {
  if (check_cfg(nullptr, cfg) != LC_OK) return 0;
  return (size_t)cfg->B * cfg->F * (cfg->H / 2) * (cfg->W / 2) * cfg->C_deep * dtype_size(cfg->dtype);
}

size_t lc_workspace_bytes(const lc_config* cfg, int frame_chunk, int token_chunk) {
  if (check_cfg(nullptr, cfg) != LC_OK) return 0;
  if (frame_chunk < 0 || token_chunk < 0) { g_err = "chunk sizes must be >= 0"; return 0; }
  return make_plan(*cfg, frame_chunk, token_chunk, 1, 1).total;
}

size_t lc_workspace_bytes_spatial(const lc_config* cfg, int frame_chunk, int token_chunk, int eta, int omega) {
  if (check_cfg(nullptr, cfg) != LC_OK) return 0;
  if (frame_chunk < 0 || token_chunk < 0 || eta < 1 || omega < 1 || cfg->H % eta || cfg->W % omega) {
    g_err = "chunk sizes must be >= 0 and the spatial factors must divide H and W";
    return 0;
  }
  return make_plan(*cfg, frame_chunk, token_chunk, eta, omega).total;
}

lc_status lc_create(const lc_config* cfg, void* compute_stream, void* side_stream, lc_ctx** out) {
  if (!out) return fail(nullptr, LC_ERR_ARG, "out is NULL");
  lc_status s = check_cfg(nullptr, cfg);
  if (s != LC_OK) return s;
  if (!compute_stream || !side_stream || compute_stream == side_stream)
    return fail(nullptr, LC_ERR_ARG, "compute and side streams must be two distinct non-default streams");
  int dev = 0;
  LC_HIP(nullptr, hipGetDevice(&dev));
  lc_ctx* c = new (std::nothrow) lc_ctx();
  if (!c) return fail(nullptr, LC_ERR_NOMEM, "out of host memory");
  c->cfg = *cfg;
  c->cs = c->cs_main = (hipStream_t)compute_stream;
  c->ss = (hipStream_t)side_stream;
  for (int i = 0; i + 1 < kMaxLanes; ++i) { c->cs_aux[i] = nullptr; c->ev_join[i] = nullptr; }
  c->ev_fork = nullptr;
  c->lanes = 2; c->lane = 0; c->forked = false; c->conv_general = false;
  c->device = dev;
  c->frame_chunk = c->token_chunk = 0;
  c->sp_eta = c->sp_omega = 1;
  c->plan = make_plan(c->cfg, 0, 0, 1, 1);
  c->arena = nullptr; c->arena_bytes = 0;
  c->have_weights = false; c->wblob = nullptr; c->wblob_bytes = 0;
  memset(&c->pw, 0, sizeof c->pw);
  memset(&c->st, 0, sizeof c->st);
  c->prof_mask = 0; c->prof_used = 0; c->prof_dropped = 0;
  const size_t entry = lc_cache_entry_bytes(cfg);
  auto bail = [&](lc_status code, const char* what, hipError_t e) {
    g_err = std::string(what) + ": " + hipGetErrorString(e);
    destroy_ctx(c);
    return code;
  };
  c->static_scratch = nullptr;
  {
    const hipError_t e = static_scratch_ptr(dev, &c->static_scratch);
    if (e != hipSuccess) return bail(LC_ERR_HIP, "hipGetSymbolAddress (static scratch)", e);
  }
  for (int i = 0; i < cfg->host_slots; ++i) {
    void* p = nullptr;
    hipError_t e = hipErrorOutOfMemory;
    const bool injected = g_fail_host_alloc > 0 && --g_fail_host_alloc == 0;
    if (!injected) e = hipHostMalloc(&p, entry, hipHostMallocDefault);
    if (e != hipSuccess) {
      (void)hipGetLastError();  // the failure is reported through the status, not left for the next HIP call
      return bail(LC_ERR_NOMEM, injected ? "pinned cache bank (injected failure)" : "hipHostMalloc (pinned cache bank)", e);
    }
    c->host.push_back(p);
  }
  c->host_filled.assign(cfg->host_slots, 0);
  c->dev_filled.assign(cfg->dev_slots, 0);
  c->in_pending.assign(cfg->dev_slots, 0);
  c->deep_stat_valid.assign(cfg->dev_slots, 0);
  auto mk = [&](std::vector<hipEvent_t>& v, int n, unsigned flags) -> hipError_t {
    for (int i = 0; i < n; ++i) {
      hipEvent_t e;
      hipError_t r = hipEventCreateWithFlags(&e, flags);
      if (r != hipSuccess) return r;
      v.push_back(e);
    }
    return hipSuccess;
  };
  hipError_t e;
  // the second lane: a stream of the library's own (default priority; it never syncs with the legacy stream)
  for (int i = 0; i + 1 < kMaxLanes; ++i) {
    if ((e = hipStreamCreateWithFlags(&c->cs_aux[i], hipStreamNonBlocking)) != hipSuccess) return bail(LC_ERR_HIP, "hipStreamCreate", e);
    if ((e = hipEventCreateWithFlags(&c->ev_join[i], hipEventDisableTiming)) != hipSuccess) return bail(LC_ERR_HIP, "hipEventCreate", e);
  }
  if ((e = hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming)) != hipSuccess) return bail(LC_ERR_HIP, "hipEventCreate", e);
  if ((e = mk(c->ev_produced, cfg->dev_slots, hipEventDisableTiming)) != hipSuccess ||
      (e = mk(c->ev_consumed, cfg->dev_slots, hipEventDisableTiming)) != hipSuccess ||
      (e = mk(c->ev_in_done, cfg->dev_slots, hipEventDisableTiming)) != hipSuccess ||
      (e = mk(c->ev_rd_done, cfg->dev_slots, hipEventDisableTiming)) != hipSuccess ||
      (e = mk(c->ev_out_done, cfg->host_slots, hipEventDisableTiming)) != hipSuccess)
    return bail(LC_ERR_HIP, "hipEventCreate", e);
  for (int i = 0; i < 256; ++i) {
    EvPair pr{};
    if ((e = hipEventCreate(&pr.a)) != hipSuccess) return bail(LC_ERR_HIP, "hipEventCreate", e);
    if ((e = hipEventCreate(&pr.b)) != hipSuccess) { (void)hipEventDestroy(pr.a); return bail(LC_ERR_HIP, "hipEventCreate", e); }
    c->copy_pool.push_back(pr);
  }
  c->st.host_bank_bytes = entry * cfg->host_slots;
  {
    std::lock_guard<std::mutex> lk(g_live_mu);
    g_live.insert(c);
  }
  *out = c;
  return LC_OK;
}

lc_status lc_destroy(lc_ctx* c) {
  if (!c) return LC_OK;
  {
    // a pointer lc_create did not hand out, or one that has been destroyed already, is not touched
    std::lock_guard<std::mutex> lk(g_live_mu);
    if (!g_live.erase(c)) return fail(nullptr, LC_ERR_ARG, "lc_destroy: unknown or already destroyed context");
  }
  destroy_ctx(c);
  return LC_OK;
}

lc_status lc_test_fail_host_alloc(int nth) {
  if (nth < 0) return fail(nullptr, LC_ERR_ARG, "nth must be >= 0");
  g_fail_host_alloc = nth;
  return LC_OK;
}

}  // extern "C"

namespace {
void destroy_ctx(lc_ctx* c) {
  (void)hipStreamSynchronize(c->cs_main);
  (void)hipStreamSynchronize(c->ss);
  for (int i = 0; i + 1 < kMaxLanes; ++i) {
    if (c->cs_aux[i]) { (void)hipStreamSynchronize(c->cs_aux[i]); (void)hipStreamDestroy(c->cs_aux[i]); }
    if (c->ev_join[i]) (void)hipEventDestroy(c->ev_join[i]);
  }
  if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
  for (void* p : c->host) (void)hipHostFree(p);
  for (auto* v : {&c->ev_produced, &c->ev_consumed, &c->ev_in_done, &c->ev_rd_done, &c->ev_out_done})
    for (hipEvent_t e : *v) (void)hipEventDestroy(e);
  for (auto* v : {&c->copy_pool, &c->copy_pending, &c->prof_pool})
    for (EvPair& pr : *v) { (void)hipEventDestroy(pr.a); (void)hipEventDestroy(pr.b); }
  if (c->wblob) (void)hipFree(c->wblob);
  delete c;
}
}  // namespace

extern "C" {

lc_status lc_load_weights(lc_ctx* c, const lc_weights* w) {
  if (!c) return fail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!w) return fail(c, LC_ERR_ARG, "weights is NULL");
  const lc_config& g = c->cfg;
  const int C = g.C, Cd = g.C_deep, Cl = g.C_lat, dt = g.dtype;
  const size_t es = dtype_size(dt);
  // every pointer the configuration uses must be present
  auto need_gc = [](const lc_gnconv_w& x) { return x.gn_g && x.gn_b && x.w && x.b; };
  auto need_at = [](const lc_attn_w& x) { return x.gn_g && x.gn_b && x.wq && x.wk && x.wv && x.wo && x.bo; };
  bool ok = w->conv_in_w && w->conv_in_b && need_at(w->sattn) && need_at(w->tattn) && w->down_w && w->down_b &&
            need_gc(w->dres) && need_gc(w->up) && need_gc(w->out);
  for (int i = 0; i < g.n_res; ++i) ok = ok && need_gc(w->res[i]);
  if (!ok) return fail(c, LC_ERR_ARG, "a weight pointer is NULL");

  // ---- layout of the private blob
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
  const size_t o_cin_w = take((size_t)Cl * 9 * C * 4), o_cin_b = take((size_t)C * 4);
  const size_t o_cin_wp = take((size_t)C * 64 * es), o_cin_wf = take((size_t)C * 64 * es);
  size_t o_res_g[LC_MAX_RES], o_res_b[LC_MAX_RES], o_res_w[LC_MAX_RES], o_res_bias[LC_MAX_RES];
  for (int i = 0; i < g.n_res; ++i) {
    o_res_g[i] = take((size_t)C * 4); o_res_b[i] = take((size_t)C * 4);
    o_res_w[i] = take((size_t)C * 9 * C * es); o_res_bias[i] = take((size_t)C * 4);
  }
  // a second copy of the big 3x3 weights in the tile order the specialised-wavefront kernel streams
  const bool tiles = dt == kBF16 && C % 160 == 0 && C % 64 == 0 && (C + Cd) % 64 == 0;
  size_t o_res_wt[LC_MAX_RES] = {0}, o_up_wt = 0;
  if (tiles) {
    for (int i = 0; i < g.n_res; ++i) o_res_wt[i] = take((size_t)C * 9 * C * es);
    o_up_wt = take((size_t)C * 9 * (C + Cd) * es);
  }
  size_t o_at[2][7];
  for (int k = 0; k < 2; ++k) {
    o_at[k][0] = take((size_t)C * 4); o_at[k][1] = take((size_t)C * 4);
    o_at[k][2] = take((size_t)3 * C * C * es); o_at[k][3] = take((size_t)C * C * es); o_at[k][4] = take((size_t)C * 4);
    o_at[k][5] = take((size_t)3 * C * C * es); o_at[k][6] = take((size_t)C * C * es);
  }
  const size_t o_down_w = take((size_t)Cd * 9 * C * es), o_down_b = take((size_t)Cd * 4);
  const size_t o_dres_g = take((size_t)Cd * 4), o_dres_b = take((size_t)Cd * 4);
  const size_t o_dres_w = take((size_t)Cd * 9 * Cd * es), o_dres_bias = take((size_t)Cd * 4);
  const size_t o_up_g = take((size_t)(C + Cd) * 4), o_up_b = take((size_t)(C + Cd) * 4);
  const size_t o_up_w = take((size_t)C * 9 * (C + Cd) * es), o_up_bias = take((size_t)C * 4);
  const size_t o_out_g = take((size_t)C * 4), o_out_b = take((size_t)C * 4);
  const size_t o_out_w = take((size_t)32 * 9 * C * es), o_out_bias = take((size_t)32 * 4);

  LC_HIP(c, hipStreamSynchronize(c->cs));
  if (c->wblob) { LC_HIP(c, hipFree(c->wblob)); c->wblob = nullptr; c->have_weights = false; }
  void* blob = nullptr;
  if (hipMalloc(&blob, off) != hipSuccess) return fail(c, LC_ERR_NOMEM, "hipMalloc of %zu bytes for packed weights failed", off);
  c->wblob = blob; c->wblob_bytes = off;
  char* b = (char*)blob;
  Packed& p = c->pw;
  hipStream_t s = c->cs;
#define F32(src, dst_off, n, npad) LC_HIP(c, launch_to_f32(s, dt, src, (float*)(b + dst_off), n, npad))
#define CW(src, dst_off, co, ci, taps, copad) LC_HIP(c, launch_pack_conv_w(s, dt, src, b + dst_off, co, ci, taps, copad))
  LC_HIP(c, launch_pack_conv_in_w(s, dt, w->conv_in_w, (float*)(b + o_cin_w), C, Cl));
  F32(w->conv_in_b, o_cin_b, C, C);
  p.cin_w = (float*)(b + o_cin_w); p.cin_b = (float*)(b + o_cin_b);
  p.cin_wf = nullptr; p.cin_wp = nullptr;
  if (Cl * 9 <= 64) {  // [C][Cl][3][3] is already [C][Cl*9]: pad the rows to 64, then fragment order
    LC_HIP(c, launch_pad_rows(s, dt, w->conv_in_w, b + o_cin_wp, C, Cl * 9, 64));
    LC_HIP(c, launch_pack_lin_w(s, dt, b + o_cin_wp, b + o_cin_wf, C, 64));
    p.cin_wf = b + o_cin_wf; p.cin_wp = b + o_cin_wp;
  }
  for (int i = 0; i < g.n_res; ++i) {
    F32(w->res[i].gn_g, o_res_g[i], C, C); F32(w->res[i].gn_b, o_res_b[i], C, C);
    CW(w->res[i].w, o_res_w[i], C, C, 9, C); F32(w->res[i].b, o_res_bias[i], C, C);
    p.res_gn[i] = GnW{(float*)(b + o_res_g[i]), (float*)(b + o_res_b[i])};
    p.res[i] = ConvW{b + o_res_w[i], (float*)(b + o_res_bias[i]), nullptr};
    if (tiles) {
      LC_HIP(c, launch_pack_conv_w_tiles(s, dt, b + o_res_w[i], b + o_res_wt[i], C, C));
      p.res[i].wt = b + o_res_wt[i];
    }
  }
  const lc_attn_w* aw[2] = {&w->sattn, &w->tattn};
  AttnW* ap[2] = {&p.sattn, &p.tattn};
  for (int k = 0; k < 2; ++k) {
    F32(aw[k]->gn_g, o_at[k][0], C, C); F32(aw[k]->gn_b, o_at[k][1], C, C);
    // rows [0,C) = Wq, [C,2C) = Wk, [2C,3C) = Wv; linear weights are already [Cout][Cin]
    LC_HIP(c, launch_copy_rows(s, dt, aw[k]->wq, b + o_at[k][2], (int64_t)C * C));
    LC_HIP(c, launch_copy_rows(s, dt, aw[k]->wk, b + o_at[k][2] + (size_t)C * C * es, (int64_t)C * C));
    LC_HIP(c, launch_copy_rows(s, dt, aw[k]->wv, b + o_at[k][2] + (size_t)2 * C * C * es, (int64_t)C * C));
    LC_HIP(c, launch_copy_rows(s, dt, aw[k]->wo, b + o_at[k][3], (int64_t)C * C));
    F32(aw[k]->bo, o_at[k][4], C, C);
    LC_HIP(c, launch_pack_lin_w(s, dt, b + o_at[k][2], b + o_at[k][5], 3 * C, C));
    LC_HIP(c, launch_pack_lin_w(s, dt, b + o_at[k][3], b + o_at[k][6], C, C));
    *ap[k] = AttnW{GnW{(float*)(b + o_at[k][0]), (float*)(b + o_at[k][1])}, b + o_at[k][2], b + o_at[k][3],
                   (float*)(b + o_at[k][4]), b + o_at[k][5], b + o_at[k][6]};
  }
  CW(w->down_w, o_down_w, Cd, C, 9, Cd); F32(w->down_b, o_down_b, Cd, Cd);
  p.down = ConvW{b + o_down_w, (float*)(b + o_down_b), nullptr};
  F32(w->dres.gn_g, o_dres_g, Cd, Cd); F32(w->dres.gn_b, o_dres_b, Cd, Cd);
  CW(w->dres.w, o_dres_w, Cd, Cd, 9, Cd); F32(w->dres.b, o_dres_bias, Cd, Cd);
  p.dres_gn = GnW{(float*)(b + o_dres_g), (float*)(b + o_dres_b)};
  p.dres = ConvW{b + o_dres_w, (float*)(b + o_dres_bias), nullptr};
  F32(w->up.gn_g, o_up_g, C + Cd, C + Cd); F32(w->up.gn_b, o_up_b, C + Cd, C + Cd);
  CW(w->up.w, o_up_w, C, C + Cd, 9, C); F32(w->up.b, o_up_bias, C, C);
  p.up_gn = GnW{(float*)(b + o_up_g), (float*)(b + o_up_b)};
  p.up = ConvW{b + o_up_w, (float*)(b + o_up_bias), nullptr};
  if (tiles) {
    LC_HIP(c, launch_pack_conv_w_tiles(s, dt, b + o_up_w, b + o_up_wt, C, C + Cd));
    p.up.wt = b + o_up_wt;
  }
  F32(w->out.gn_g, o_out_g, C, C); F32(w->out.gn_b, o_out_b, C, C);
  CW(w->out.w, o_out_w, Cl, C, 9, 32); F32(w->out.b, o_out_bias, Cl, 32);
  p.out_gn = GnW{(float*)(b + o_out_g), (float*)(b + o_out_b)};
  p.out = ConvW{b + o_out_w, (float*)(b + o_out_bias), nullptr};
#undef F32
#undef CW
  LC_HIP(c, hipStreamSynchronize(s));
  c->have_weights = true;
  c->st.weight_bytes = off;
  return LC_OK;
}

lc_status lc_set_workspace(lc_ctx* c, void* arena, size_t bytes) {
  if (!c) return fail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!arena) return fail(c, LC_ERR_ARG, "arena is NULL");
  if ((uintptr_t)arena % kAlign) return fail(c, LC_ERR_ARG, "arena must be 256-byte aligned");
  if (bytes < c->plan.total)
    return fail(c, LC_ERR_NOMEM, "workspace of %zu bytes is smaller than the %zu needed", bytes, c->plan.total);
  LC_HIP(c, hipStreamSynchronize(c->cs));
  LC_HIP(c, hipStreamSynchronize(c->ss));
  c->arena = (char*)arena;
  c->arena_bytes = bytes;
  std::fill(c->dev_filled.begin(), c->dev_filled.end(), 0);
  std::fill(c->in_pending.begin(), c->in_pending.end(), 0);
  std::fill(c->deep_stat_valid.begin(), c->deep_stat_valid.end(), 0);
  c->st.workspace_bytes = c->plan.total;
  return LC_OK;
}

lc_status lc_set_lanes(lc_ctx* c, int lanes) {
  if (!c) return fail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (lanes < 1 || lanes > kMaxLanes) return fail(c, LC_ERR_ARG, "lanes must be in [1, %d]", kMaxLanes);
  c->lanes = lanes;
  return LC_OK;
}

lc_status lc_set_conv_general(lc_ctx* c, int general) {
  if (!c) return fail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (general != 0 && general != 1) return fail(c, LC_ERR_ARG, "general must be 0 or 1");
  c->conv_general = general != 0;
  return LC_OK;
}

lc_status lc_set_chunk(lc_ctx* c, int frame_chunk, int token_chunk) {
  if (!c) return fail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (frame_chunk < 0 || token_chunk < 0) return fail(c, LC_ERR_ARG, "chunk sizes must be >= 0");
  Plan np = make_plan(c->cfg, frame_chunk, token_chunk, c->sp_eta, c->sp_omega);
  if (c->arena && np.total > c->arena_bytes)
    return fail(c, LC_ERR_NOMEM, "chunk setting needs %zu bytes, workspace has %zu", np.total, c->arena_bytes);
  // the persistent regions (skip feature, cache slots) sit at chunk-independent offsets, so a
  // filled slot stays valid across a chunk change
  c->frame_chunk = frame_chunk;
  c->token_chunk = token_chunk;
  c->plan = np;
  std::fill(c->deep_stat_valid.begin(), c->deep_stat_valid.end(), 0);  // their region moves with the plan
  c->st.workspace_bytes = np.total;
  return LC_OK;
}

lc_status lc_set_spatial_chunk(lc_ctx* c, int eta, int omega) {
  if (!c) return fail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (eta < 1 || omega < 1) return fail(c, LC_ERR_ARG, "eta and omega must be >= 1");
  const lc_config& g = c->cfg;
  if (eta * omega > 1) {
    if (eta * omega > 64) return fail(c, LC_ERR_SHAPE, "at most 64 spatial blocks per frame");
    if (g.H % eta || g.W % omega) return fail(c, LC_ERR_SHAPE, "eta must divide H and omega must divide W");
    // a block is made of whole tiles of every kernel: 8 image rows (3x3 convolutions), 32 pixels of a row (the
    // 32-row tiles of the projections, the row segments of conv_in)
    if ((g.H / eta) % 8 || (g.W / omega) % 32)
      return fail(c, LC_ERR_SHAPE, "a spatial block must be a multiple of 8 rows x 32 columns (got %d x %d)", g.H / eta, g.W / omega);
    // the projections must have their weight-stationary kernel, conv_in its tile kernel or the gathering linear one
    const bool lin_ok = g.C == 64 || g.C == 128 || (g.C == 320 && g.dtype == LC_BF16);
    if (!lin_ok || g.C_lat * 9 > 64)
      return fail(c, LC_ERR_SHAPE, "spatial chunking needs C in {64, 128} (or 320 with bf16) and C_lat <= 7");
  }
  Plan np = make_plan(g, c->frame_chunk, c->token_chunk, eta, omega);
  if (c->arena && np.total > c->arena_bytes)
    return fail(c, LC_ERR_NOMEM, "spatial chunk setting needs %zu bytes, workspace has %zu", np.total, c->arena_bytes);
  c->sp_eta = eta; c->sp_omega = omega;
  c->plan = np;
  std::fill(c->deep_stat_valid.begin(), c->deep_stat_valid.end(), 0);
  c->st.workspace_bytes = np.total;
  return LC_OK;
}

lc_status lc_full_step(lc_ctx* c, const void* x, void* eps, int dev_slot) {
  lc_status s = step_checks(c, x, eps, dev_slot);
  if (s != LC_OK) return s;
  s = run_step(c, x, eps, dev_slot, true);
  if (s == LC_OK) c->st.full_steps++;
  return s;
}

lc_status lc_cached_step(lc_ctx* c, const void* x, void* eps, int dev_slot) {
  lc_status s = step_checks(c, x, eps, dev_slot);
  if (s != LC_OK) return s;
  if (!c->dev_filled[dev_slot]) return fail(c, LC_ERR_STATE, "cached step on empty device slot %d", dev_slot);
  s = run_step(c, x, eps, dev_slot, false);
  if (s == LC_OK) c->st.cached_steps++;
  return s;
}

static lc_status swap_common(lc_ctx* c, int dev_slot, int host_slot) {
  if (!c) return fail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (dev_slot < 0 || dev_slot >= c->cfg.dev_slots) return fail(c, LC_ERR_ARG, "device slot %d out of range", dev_slot);
  if (host_slot < 0 || host_slot >= c->cfg.host_slots) return fail(c, LC_ERR_ARG, "host slot %d out of range", host_slot);
  if (!c->arena) return fail(c, LC_ERR_STATE, "workspace not set");
  return LC_OK;
}

// folds the copies that have completed into the statistics and returns their event pairs to the pool
static void harvest_copy_pairs(lc_ctx* c) {
  size_t keep = 0;
  for (size_t i = 0; i < c->copy_pending.size(); ++i) {
    EvPair& pr = c->copy_pending[i];
    float ms = 0.f;
    if (hipEventQuery(pr.b) == hipSuccess && hipEventElapsedTime(&ms, pr.a, pr.b) == hipSuccess) {
      (pr.kind == 0 ? c->st.ms_out : c->st.ms_in) += ms;
      (pr.kind == 0 ? c->st.timed_out : c->st.timed_in)++;
      c->copy_pool.push_back(pr);
    } else {
      c->copy_pending[keep++] = pr;
    }
  }
  c->copy_pending.resize(keep);
}

static EvPair* take_copy_pair(lc_ctx* c) {
  if (c->copy_pool.empty()) harvest_copy_pairs(c);
  if (c->copy_pool.empty()) return nullptr;
  c->copy_pending.push_back(c->copy_pool.back());
  c->copy_pool.pop_back();
  return &c->copy_pending.back();
}

lc_status lc_swap_out(lc_ctx* c, int dev_slot, int host_slot) {
  lc_status s = swap_common(c, dev_slot, host_slot);
  if (s != LC_OK) return s;
  if (!c->dev_filled[dev_slot]) return fail(c, LC_ERR_STATE, "swap-out of empty device slot %d", dev_slot);
  const size_t bytes = lc_cache_entry_bytes(&c->cfg);
  LC_HIP(c, hipStreamWaitEvent(c->ss, c->ev_produced[dev_slot], 0));
  EvPair* pr = take_copy_pair(c);
  if (pr) { pr->kind = 0; pr->bytes = (int64_t)bytes; LC_HIP(c, hipEventRecord(pr->a, c->ss)); }
  LC_HIP(c, hipMemcpyAsync(c->host[host_slot], slot_ptr(c, dev_slot), bytes, hipMemcpyDeviceToHost, c->ss));
  if (pr) LC_HIP(c, hipEventRecord(pr->b, c->ss));
  LC_HIP(c, hipEventRecord(c->ev_rd_done[dev_slot], c->ss));
  LC_HIP(c, hipEventRecord(c->ev_out_done[host_slot], c->ss));
  c->host_filled[host_slot] = 1;
  c->st.swaps_out++;
  c->st.bytes_out += (int64_t)bytes;
  return LC_OK;
}

lc_status lc_swap_in(lc_ctx* c, int host_slot, int dev_slot) {
  lc_status s = swap_common(c, dev_slot, host_slot);
  if (s != LC_OK) return s;
  if (!c->host_filled[host_slot]) return fail(c, LC_ERR_STATE, "swap-in from empty host slot %d", host_slot);
  const size_t bytes = lc_cache_entry_bytes(&c->cfg);
  // after the last enqueued reader / writer of the device slot on the compute stream
  LC_HIP(c, hipStreamWaitEvent(c->ss, c->ev_consumed[dev_slot], 0));
  LC_HIP(c, hipStreamWaitEvent(c->ss, c->ev_produced[dev_slot], 0));
  EvPair* pr = take_copy_pair(c);
  if (pr) { pr->kind = 1; pr->bytes = (int64_t)bytes; LC_HIP(c, hipEventRecord(pr->a, c->ss)); }
  LC_HIP(c, hipMemcpyAsync(slot_ptr(c, dev_slot), c->host[host_slot], bytes, hipMemcpyHostToDevice, c->ss));
  if (pr) LC_HIP(c, hipEventRecord(pr->b, c->ss));
  LC_HIP(c, hipEventRecord(c->ev_in_done[dev_slot], c->ss));
  c->in_pending[dev_slot] = 1;
  c->dev_filled[dev_slot] = 1;
  c->deep_stat_valid[dev_slot] = 0;
  c->st.swaps_in++;
  c->st.bytes_in += (int64_t)bytes;
  return LC_OK;
}

lc_status lc_sync(lc_ctx* c) {
  if (!c) return fail(nullptr, LC_ERR_ARG, "ctx is NULL");
  LC_HIP(c, hipStreamSynchronize(c->cs));
  LC_HIP(c, hipStreamSynchronize(c->ss));
  return LC_OK;
}

lc_status lc_cache_write(lc_ctx* c, int dev_slot, const void* deep) {
  if (!c) return fail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!deep) return fail(c, LC_ERR_ARG, "deep is NULL");
  if (dev_slot < 0 || dev_slot >= c->cfg.dev_slots) return fail(c, LC_ERR_ARG, "device slot %d out of range", dev_slot);
  if (!c->arena) return fail(c, LC_ERR_STATE, "workspace not set");
  const lc_config& g = c->cfg;
  LC_HIP(c, hipStreamWaitEvent(c->cs, c->ev_rd_done[dev_slot], 0));
  LC_HIP(c, hipStreamWaitEvent(c->cs, c->ev_in_done[dev_slot], 0));
  c->in_pending[dev_slot] = 0;
  LC_HIP(c, launch_planar_to_cl(c->cs, g.dtype, deep, slot_ptr(c, dev_slot), g.B * g.F, g.C_deep, (g.H / 2) * (g.W / 2)));
  LC_HIP(c, hipEventRecord(c->ev_produced[dev_slot], c->cs));
  c->dev_filled[dev_slot] = 1;
  c->deep_stat_valid[dev_slot] = 0;
  return LC_OK;
}

lc_status lc_cache_read(lc_ctx* c, int dev_slot, void* deep) {
  if (!c) return fail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!deep) return fail(c, LC_ERR_ARG, "deep is NULL");
  if (dev_slot < 0 || dev_slot >= c->cfg.dev_slots) return fail(c, LC_ERR_ARG, "device slot %d out of range", dev_slot);
  if (!c->arena) return fail(c, LC_ERR_STATE, "workspace not set");
  if (!c->dev_filled[dev_slot]) return fail(c, LC_ERR_STATE, "device slot %d is empty", dev_slot);
  const lc_config& g = c->cfg;
  if (c->in_pending[dev_slot]) {
    LC_HIP(c, hipStreamWaitEvent(c->cs, c->ev_in_done[dev_slot], 0));
    c->in_pending[dev_slot] = 0;
  }
  LC_HIP(c, launch_cl_to_planar(c->cs, g.dtype, slot_ptr(c, dev_slot), deep, g.B * g.F, g.C_deep, (g.H / 2) * (g.W / 2)));
  LC_HIP(c, hipEventRecord(c->ev_consumed[dev_slot], c->cs));
  return LC_OK;
}

lc_status lc_cache_peek(lc_ctx* c, int host_slot, const void** ptr, size_t* bytes) {
  if (!c) return fail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!ptr || !bytes) return fail(c, LC_ERR_ARG, "output pointer is NULL");
  if (host_slot < 0 || host_slot >= c->cfg.host_slots) return fail(c, LC_ERR_ARG, "host slot %d out of range", host_slot);
  if (!c->host_filled[host_slot]) return fail(c, LC_ERR_STATE, "host slot %d is empty", host_slot);
  *ptr = c->host[host_slot];
  *bytes = lc_cache_entry_bytes(&c->cfg);
  return LC_OK;
}

lc_status lc_cache_dev_peek(lc_ctx* c, int dev_slot, const void** ptr, size_t* bytes) {
  if (!c) return fail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!ptr || !bytes) return fail(c, LC_ERR_ARG, "output pointer is NULL");
  if (dev_slot < 0 || dev_slot >= c->cfg.dev_slots) return fail(c, LC_ERR_ARG, "device slot %d out of range", dev_slot);
  if (!c->arena) return fail(c, LC_ERR_STATE, "workspace not set");
  if (!c->dev_filled[dev_slot]) return fail(c, LC_ERR_STATE, "device slot %d is empty", dev_slot);
  *ptr = slot_ptr(c, dev_slot);
  *bytes = lc_cache_entry_bytes(&c->cfg);
  return LC_OK;
}

lc_status lc_get_stats(lc_ctx* c, lc_stats* out) {
  if (!c) return fail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!out) return fail(c, LC_ERR_ARG, "out is NULL");
  LC_HIP(c, hipStreamSynchronize(c->ss));
  harvest_copy_pairs(c);
  *out = c->st;
  return LC_OK;
}

lc_status lc_reset_stats(lc_ctx* c) {
  if (!c) return fail(nullptr, LC_ERR_ARG, "ctx is NULL");
  lc_stats tmp;
  lc_status s = lc_get_stats(c, &tmp);
  if (s != LC_OK) return s;
  const size_t ws = c->st.workspace_bytes, wb = c->st.weight_bytes, hb = c->st.host_bank_bytes;
  memset(&c->st, 0, sizeof c->st);
  c->st.workspace_bytes = ws; c->st.weight_bytes = wb; c->st.host_bank_bytes = hb;
  return LC_OK;
}

lc_status lc_set_profiling(lc_ctx* c, uint32_t mask) {
  if (!c) return fail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (mask && c->prof_pool.empty()) {
    for (int i = 0; i < 4096; ++i) {
      EvPair pr{};
      LC_HIP(c, hipEventCreate(&pr.a));
      hipError_t e = hipEventCreate(&pr.b);
      if (e != hipSuccess) { (void)hipEventDestroy(pr.a); return fail(c, LC_ERR_HIP, "hipEventCreate: %s", hipGetErrorString(e)); }
      c->prof_pool.push_back(pr);
    }
  }
  c->prof_mask = mask;
  return LC_OK;
}

lc_status lc_get_profile(lc_ctx* c, lc_profile* out) {
  if (!c) return fail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!out) return fail(c, LC_ERR_ARG, "out is NULL");
  LC_HIP(c, hipStreamSynchronize(c->cs));
  lc_profile pf;
  memset(&pf, 0, sizeof pf);
  for (size_t i = 0; i < c->prof_used; ++i) {
    float ms = 0.f;
    const EvPair& pr = c->prof_pool[i];
    if (hipEventElapsedTime(&ms, pr.a, pr.b) == hipSuccess) {
      pf.ms[pr.kind] += ms;
      pf.launches[pr.kind]++;
    }
  }
  c->prof_used = 0;
  pf.dropped = c->prof_dropped;
  c->prof_dropped = 0;
  *out = pf;
  return LC_OK;
}

lc_status lc_cached_step_static(lc_ctx* c, const void* x, const void* deep, void* eps) {
  if (!c) return fail(nullptr, LC_ERR_ARG, "ctx is NULL");
  if (!x || !deep || !eps) return fail(c, LC_ERR_ARG, "x, deep and eps must not be NULL");
  if (!c->have_weights) return fail(c, LC_ERR_STATE, "weights not loaded");
  if (!c->static_scratch) return fail(c, LC_ERR_STATE, "static scratch not available on this device");
  if (c->plan.total > kStaticScratchBytes)
    return fail(c, LC_ERR_NOMEM,
                "this stage needs %zu bytes of scratch with the current chunk setting; the static scratch of "
                "lc_cached_step_static holds %zu: use a smaller chunk, or lc_set_workspace + lc_cached_step",
                c->plan.total, kStaticScratchBytes);
  const lc_config& g = c->cfg;
  // the step runs as lc_cached_step does, with the static array as its arena and the deep feature in slot 0
  // of that arena; the context's own arena, its slots and what it knows about them are put back afterwards
  char* const arena0 = c->arena;
  const char filled0 = c->dev_filled[0], pending0 = c->in_pending[0], statv0 = c->deep_stat_valid[0];
  c->arena = (char*)c->static_scratch;
  c->dev_filled[0] = 1; c->in_pending[0] = 0; c->deep_stat_valid[0] = 0;
  lc_status s = LC_OK;
  const hipError_t e = launch_planar_to_cl(c->cs, g.dtype, deep, slot_ptr(c, 0), g.B * g.F, g.C_deep, (g.H / 2) * (g.W / 2));
  if (e != hipSuccess) s = fail(c, LC_ERR_HIP, "layout change of the deep feature: %s", hipGetErrorString(e));
  if (s == LC_OK) s = run_step(c, x, eps, 0, false);
  c->arena = arena0;
  c->dev_filled[0] = filled0; c->in_pending[0] = pending0; c->deep_stat_valid[0] = statv0;
  if (s == LC_OK) c->st.cached_steps++;
  return s;
}

size_t lc_static_scratch_bytes(void) { return kStaticScratchBytes; }

// ---- single operators -------------------------------------------------------------------------

lc_status lc_op_spatial_block(lc_ctx* c, void* h, int frames) {
  lc_status s = op_checks(c, frames);
  if (s != LC_OK) return s;
  if (!h) return fail(c, LC_ERR_ARG, "NULL tensor");
  if (frames > c->plan.fc) return fail(c, LC_ERR_NOMEM, "the chunk scratch holds %d frames, not %d", c->plan.fc, frames);
  // the scratch layout of a frame chunk inside a step: the fp32 ping-pong copy first, then what this block uses
  const size_t skip = align_up((size_t)frames * c->cfg.H * c->cfg.W * c->cfg.C * 4);
  return spatial_block(c, (char*)h, ws_ptr(c) + skip, frames, StatRef{nullptr, 0}, nullptr, nullptr);
}

lc_status lc_op_temporal_block(lc_ctx* c, void* h) {
  lc_status s = op_checks(c, 1);
  if (s != LC_OK) return s;
  if (!h) return fail(c, LC_ERR_ARG, "NULL tensor");
  bool ustat = false;
  s = temporal_block(c, (char*)h, StatRef{nullptr, 0}, &ustat);
  if (s != LC_OK) {  // leave the streams joined and the first lane selected whatever happened
    const std::string keep = c->err;
    (void)join_lanes(c);
    c->err = keep;
  }
  return s;
}

lc_status lc_op_res_block(lc_ctx* c, int layer, const void* x, void* y, int frames) {
  lc_status s = op_checks(c, frames);
  if (s != LC_OK) return s;
  if (!x || !y || x == y) return fail(c, LC_ERR_ARG, "x and y must be distinct non-NULL tensors");
  const lc_config& g = c->cfg;
  if (layer >= LC_L_RES0 && layer < LC_L_RES0 + g.n_res)
    return res_block(c, c->pw.res_gn[layer], c->pw.res[layer], g.C, frames, g.H, g.W, x, y, 1, LC_K_CONV_RES);
  if (layer == LC_L_DRES)
    return res_block(c, c->pw.dres_gn, c->pw.dres, g.C_deep, frames, g.H / 2, g.W / 2, x, y, 0, LC_K_DEEP);
  return fail(c, LC_ERR_ARG, "layer %d is not a residual block", layer);
}

lc_status lc_op_up_conv(lc_ctx* c, const void* skip, const void* deep, void* u, int frames) {
  lc_status s = op_checks(c, frames);
  if (s != LC_OK) return s;
  if (!skip || !deep || !u) return fail(c, LC_ERR_ARG, "NULL tensor");
  return up_conv(c, skip, deep, u, frames);
}

lc_status lc_op_down_conv(lc_ctx* c, const void* x, void* y, int frames) {
  lc_status s = op_checks(c, frames);
  if (s != LC_OK) return s;
  if (!x || !y) return fail(c, LC_ERR_ARG, "NULL tensor");
  LC_LAUNCH(c, LC_K_DEEP, launch_conv(c->cs, down_desc(c->cfg, c->pw.down, frames, x, y)));
  return LC_OK;
}

lc_status lc_op_qkv(lc_ctx* c, int layer, const void* x, void* qkv, int frames) {
  lc_status s = op_checks(c, frames);
  if (s != LC_OK) return s;
  if (!x || !qkv) return fail(c, LC_ERR_ARG, "NULL tensor");
  if (layer != LC_L_SATTN && layer != LC_L_TATTN) return fail(c, LC_ERR_ARG, "layer %d is not an attention block", layer);
  const lc_config& g = c->cfg;
  const AttnW& a = layer == LC_L_SATTN ? c->pw.sattn : c->pw.tattn;
  const int T = g.H * g.W;
  s = gn_scale_shift(c, x, frames, T, g.C, a.gn);
  if (s != LC_OK) return s;
  RowMap fm{0, T, T};
  FusedDesc d = flinear_desc(c, a.wqkv, a.wqkv_f, nullptr, g.C, 3 * g.C, (int64_t)frames * T, 1, fm, dense_map(), x, nullptr, qkv, 0);
  if (layer == LC_L_SATTN) { d.q_scale = attn_q_scale(g.head_dim); d.q_cols = g.C; }
  LC_LAUNCH(c, LC_K_QKV, launch_linear_any(c->cs, d));
  return LC_OK;
}

lc_status lc_op_proj(lc_ctx* c, int layer, const void* a_in, const void* res, void* y, int64_t rows) {
  lc_status s = op_checks(c, 1);
  if (s != LC_OK) return s;
  if (!a_in || !y || rows <= 0) return fail(c, LC_ERR_ARG, "bad tensor argument");
  if (layer != LC_L_SATTN && layer != LC_L_TATTN) return fail(c, LC_ERR_ARG, "layer %d is not an attention block", layer);
  const AttnW& a = layer == LC_L_SATTN ? c->pw.sattn : c->pw.tattn;
  LC_LAUNCH(c, LC_K_PROJ, launch_linear_any(c->cs, flinear_desc(c, a.wo, a.wo_f, a.bo, c->cfg.C, c->cfg.C, rows, 0, dense_map(),
                                                           dense_map(), a_in, res, y, 1)));
  return LC_OK;
}

lc_status lc_op_spatial_attention(lc_ctx* c, const void* qkv, void* out, int frames, int q0, int q1, int q_prescaled) {
  lc_status s = op_checks(c, frames);
  if (s != LC_OK) return s;
  if (!qkv || !out) return fail(c, LC_ERR_ARG, "NULL tensor");
  const lc_config& g = c->cfg;
  const int T = g.H * g.W, Tp = attn_tp(T);
  if (q0 < 0 || q1 > T || q0 >= q1) return fail(c, LC_ERR_ARG, "query range out of bounds");
  const size_t es = dtype_size(g.dtype);
  if ((size_t)frames * g.C * Tp * es > c->plan.ws_bytes)
    return fail(c, LC_ERR_NOMEM, "chunk scratch too small for %d frames", frames);
  // the kernel wants V transposed (the steps get that layout straight from the q,k,v GEMM)
  char* vt = ws_ptr(c);
  LC_LAUNCH(c, LC_K_SATTN, launch_make_vt(c->cs, g.dtype, (const char*)qkv + (size_t)2 * g.C * es, 3 * g.C, vt, frames, T,
                                          Tp, g.C));
  LC_LAUNCH(c, LC_K_SATTN, launch_spatial_attention(c->cs, g.dtype, qkv, 3 * g.C, vt, Tp, out, frames, T, g.heads,
                                                    g.head_dim, q0, q1, q_prescaled != 0));
  return LC_OK;
}

lc_status lc_op_temporal_attention(lc_ctx* c, const void* qkv, void* out, int positions) {
  lc_status s = op_checks(c, 1);
  if (s != LC_OK) return s;
  if (!qkv || !out || positions <= 0) return fail(c, LC_ERR_ARG, "bad tensor argument");
  const lc_config& g = c->cfg;
  LC_LAUNCH(c, LC_K_TATTN, launch_temporal_attention(c->cs, g.dtype, qkv, out, g.B, g.F, positions, g.heads, g.head_dim));
  return LC_OK;
}

lc_status lc_op_conv_in(lc_ctx* c, const void* x, void* h, int frames) {
  lc_status s = op_checks(c, frames);
  if (s != LC_OK) return s;
  if (!x || !h) return fail(c, LC_ERR_ARG, "NULL tensor");
  return conv_in_run(c, x, h, frames, nullptr, nullptr);
}

lc_status lc_op_conv_out(lc_ctx* c, const void* u, void* eps, int frames) {
  lc_status s = op_checks(c, frames);
  if (s != LC_OK) return s;
  if (!u || !eps) return fail(c, LC_ERR_ARG, "NULL tensor");
  return conv_out(c, u, eps, frames);
}

}  // extern "C"

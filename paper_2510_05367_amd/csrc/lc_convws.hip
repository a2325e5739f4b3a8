// 3x3 stride-1 convolution of the bf16 stages with the wavefronts of a workgroup specialised
// (gfx950). Four wavefronts contract: their stream is LDS fragment reads, 32x32x16 MFMAs and the
// requests that bring the weight tiles of later steps from global memory straight into LDS. Four
// build the activations: global memory -> GroupNorm apply, SiLU, rounding (two transcendentals per
// element) -> halo tile in LDS. One of each kind sits on every SIMD. The contracting stream never
// waits for activation arithmetic or for the latency of an activation load, and the fragment reads of
// the next step are requested before the barrier that ends the current one, so its MFMAs follow each
// other across the steps; a single wavefront per SIMD that does everything executes these parts one
// after the other.
//
// Product, tiles and LDS layout are those of the general kernel in lc_gemm.hip: transposed product
// D[cout][pixel] = sum_k W[cout][k] X[pixel][k], k = tap * Cin + ci; a workgroup owns 160 output
// channels x 128 pixels (an 8 x 16 tile of one frame); contracting wavefront (pxh, kh) takes all 160
// channels of 64 pixels over half of the K elements of every (64-channel slab, tap) step, and the two
// halves are added through LDS before the epilogue. The loader fuses GroupNorm apply + SiLU and, for
// the up block, the 2x nearest upsampling and the skip-concat U_m = Concat(D_m, up2(U_{m+1}))
// ("Feature Calculation" paragraph): neither the normalised nor the concatenated tensor exists in
// memory. The same accumulation order as the general kernel: results agree bit for bit.
#include <type_traits>

#include "lc_internal.h"

namespace lc {

namespace {

constexpr int kwRow = 128;      // K bytes per LDS row per step (64 bf16 channels)
constexpr int kwLds = 144;      // row stride of the halo tiles: 16-byte reads of 8 consecutive rows cover all banks
constexpr int kwHaloW = 18;     // halo of an 8 x 16 pixel tile: 10 x 18
constexpr int kwHaloRows = 192; // 180 used, padded to 6 rounds of 32 rows
constexpr int kwBuf = 4;        // weight tiles in LDS; the loads run kwBuf - 1 steps ahead of their use
constexpr int kwAhead = kwBuf - 1;
constexpr int kwLead = 2;       // at the barrier that ends step s the weights of step s + kwLead have landed: the
                                // contracting wavefronts request the first fragments of step s + 1 before that barrier
constexpr int kwFA = 4;         // weight fragments requested from LDS ahead of the MFMAs that use them (ring of kwFA + 1)
constexpr int kwFin = 2;        // a halo packet requested at tap r is activated and stored at tap r + kwFin
constexpr int kwXR = kwHaloRows / 32;  // halo packets per activation-building thread per slab

struct WsArgs {
  const float* x;       // fp32 rows [frames][H][W][ldx]; ldx = Cin (plain) or Cs (concat)
  const bf16_t* x2;     // concat: cached deep feature [frames][H/2][W/2][Cin - Cs]
  const float* scale;   // [frames][Cin]
  const float* shift;
  const bf16_t* w;      // tiles [Cout / 160][9 * Cin / 64][160][64]: one step's block is contiguous
  const float* bias;    // [Cout] or nullptr
  const float* res;     // fp32, indexed like y, or nullptr
  float* y;             // fp32 [frames][H][W][Cout]
  int Cin, Cs, Cout;
  int H, W, tiles_x, tiles_y;
  int win_tx0, win_ty0, win_tx, win_ty;  // the tiles a launch covers: origin and extent in tiles
  float* stat;          // per-channel sums of the output per 32-pixel split, or nullptr
  int stat_splits;
};

template <int CO_T>
constexpr int ws_lds_bytes() { return kwBuf * CO_T * 32 * kwRow + 2 * kwHaloRows * kwLds; }

// weight requests a contracting wavefront has issued in the last kwAhead - kwLead steps, seen from the end of
// tap `tap`: wp per step, none in the steps of the last slab whose tile would lie behind the end
constexpr int ws_younger(int tap, bool last, int wp) {
  int n = 0;
  for (int j = 0; j < kwAhead - kwLead; ++j) {
    const int t = tap - j;
    n += (!last || t < 0 || t + kwAhead < 9) ? wp : 0;
  }
  return n;
}

}  // namespace

// CAT: channel slabs at and above Cs come from the half-resolution deep feature x2
template <int CO_T, bool CAT>
__global__ __launch_bounds__(512) void conv_ws_kernel(WsArgs a) {
  typedef Mma32<bf16_t> M;
  constexpr int BCO = CO_T * 32;
  constexpr int WP = BCO * 8 / 256;  // weight DMA instructions per contracting wavefront per step
  constexpr int KI = 4;              // MFMA k-steps per 64-channel row
  constexpr int KB = 32;             // bytes of one k-step in a row
  static_assert((BCO * 8) % 256 == 0, "whole wavefront instructions");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  auto w_lds = [&](int b) { return smem + b * BCO * kwRow; };
  auto x_lds = [&](int b) { return smem + kwBuf * BCO * kwRow + b * kwHaloRows * kwLds; };

  // (the wavefront index as a scalar: what is derived from it - roles, LDS targets of the weight requests - stays scalar)
  const int tid = threadIdx.x, lane = tid & 63, wid = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int co0 = blockIdx.y * BCO;
  int frame, ty0, tx0;
  {
    // tiles of the window (the whole frame by default), counted in the frame's own tile grid
    int t = blockIdx.x;
    tx0 = (a.win_tx0 + t % a.win_tx) * 16;
    t /= a.win_tx;
    ty0 = (a.win_ty0 + t % a.win_ty) * 8;
    frame = t / a.win_ty;
  }
  const int nslab = a.Cin / 64;

  if (wid >= 4) {
    // =========================== loader wavefronts ===========================
    const int lt = tid - 256;
    const int kp = lt & 7, lrow = lt >> 3;  // this thread moves 16-byte packet kp of halo rows lrow + 32 r
    // halo rows of this thread: source pixel (clamped; out-of-image taps become zero after the activation)
    int pix[kwXR], dpix[kwXR];
    unsigned okmask = 0;
#pragma unroll
    for (int r = 0; r < kwXR; ++r) {
      const int hp = lrow + 32 * r;
      const int hy = hp / kwHaloW, hx = hp - hy * kwHaloW;
      const int iy = ty0 + hy - 1, ix = tx0 + hx - 1;
      if (iy >= 0 && iy < a.H && ix >= 0 && ix < a.W) okmask |= 1u << r;
      const int cy = min(max(iy, 0), a.H - 1), cx = min(max(ix, 0), a.W - 1);
      pix[r] = (frame * a.H + cy) * a.W + cx;
      dpix[r] = CAT ? (frame * (a.H >> 1) + (cy >> 1)) * (a.W >> 1) + (cx >> 1) : 0;
    }
    const int ldx = CAT ? a.Cs : a.Cin;
    const float* __restrict__ xbase = a.x + kp * 8;
    const bf16_t* __restrict__ dbase = CAT ? a.x2 + kp * 8 - a.Cs : nullptr;  // indexed with the concat channel
    const int ldd = a.Cin - a.Cs;
    const float* __restrict__ scb = a.scale + (int64_t)frame * a.Cin + kp * 8;
    const float* __restrict__ shb = a.shift + (int64_t)frame * a.Cin + kp * 8;
    struct XRaw { f32x4 q[2]; };
    struct Affine { f32x4 sc[2], sh[2]; };
    auto load_affine = [&](int slab, Affine& af) {
      af.sc[0] = *reinterpret_cast<const f32x4*>(scb + slab * 64);
      af.sc[1] = *reinterpret_cast<const f32x4*>(scb + slab * 64 + 4);
      af.sh[0] = *reinterpret_cast<const f32x4*>(shb + slab * 64);
      af.sh[1] = *reinterpret_cast<const f32x4*>(shb + slab * 64 + 4);
    };
    auto fetch_x = [&](int slab, int r, XRaw& o, auto deep_c) {
      if constexpr (decltype(deep_c)::value) {
        o.q[0] = *reinterpret_cast<const f32x4*>(dbase + (int64_t)dpix[r] * ldd + slab * 64);
      } else {
        const float* p = xbase + (int64_t)pix[r] * ldx + slab * 64;
        o.q[0] = *reinterpret_cast<const f32x4*>(p);
        o.q[1] = *reinterpret_cast<const f32x4*>(p + 4);
      }
    };
    auto finish_x = [&](int buf, int r, const XRaw& o, const Affine& af, auto deep_c) {
      const bool ok = (okmask >> r) & 1u;
      bf16x8 pk;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float t;
        if constexpr (decltype(deep_c)::value) {
          typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
          const uint32_t wd = __builtin_bit_cast(u32x4, o.q[0])[e >> 1];
          t = __builtin_bit_cast(float, (e & 1) ? (wd & 0xffff0000u) : (wd << 16));
        } else {
          t = o.q[e >> 2][e & 3];
        }
        t = fmaf(t, af.sc[e >> 2][e & 3], af.sh[e >> 2][e & 3]);
        t = silu_fast(t);
        pk[e] = static_cast<bf16_t>(ok ? t : 0.f);
      }
      *reinterpret_cast<bf16x8*>(x_lds(buf) + (lrow + 32 * r) * kwLds + kp * 16) = pk;
    };

    const std::false_type no_c{};
    const std::true_type yes_c{};
    Affine aff;
    XRaw xin[kwXR];  // the packets of the next slab are all requested at tap 0; packet r is consumed at tap r + kwFin
    // ---- prologue: halo of slab 0 (never in the deep part)
    load_affine(0, aff);
    {
      XRaw x0[kwXR];
#pragma unroll
      for (int r = 0; r < kwXR; ++r) fetch_x(0, r, x0[r], no_c);
#pragma unroll
      for (int r = 0; r < kwXR; ++r) finish_x(0, r, x0[r], aff, no_c);
    }
    barrier_keep<63>();

    // ---- main loop: the packets of the next slab are requested at its first tap and finished one per tap
    // from tap kwFin on, so that the tile is complete one barrier before the slab ends. The waits for the
    // packets are the compiler's; the barriers only order the LDS stores.
    auto slab_body = [&](int slab, auto more_c, auto deep_c) {
      constexpr bool MORE = decltype(more_c)::value;
#pragma unroll
      for (int tap = 0; tap < 9; ++tap) {
        if (MORE) {
          if (tap == 0) load_affine(slab + 1, aff);
          if (tap == 0) {
#pragma unroll
            for (int r = 0; r < kwXR; ++r) fetch_x(slab + 1, r, xin[r], deep_c);
          }
        }
        if (MORE && tap >= kwFin && tap - kwFin < kwXR)
          finish_x((slab + 1) & 1, tap - kwFin, xin[tap - kwFin], aff, deep_c);
        barrier_keep<63>();
      }
    };
    static_assert(kwXR - 1 + kwFin < 8, "the halo of the next slab is complete one barrier before the slab ends");
    const int nskip = CAT ? a.Cs / 64 : nslab;  // slabs read from x; the rest from x2
    int slab = 0;
    for (; slab + 1 < nskip; ++slab) slab_body(slab, yes_c, no_c);
    if (CAT)
      for (; slab + 1 < nslab; ++slab) slab_body(slab, yes_c, yes_c);
    slab_body(nslab - 1, no_c, no_c);
    __syncthreads();  // the hand-over barrier of the contracting wavefronts
    return;
  }

  // =========================== contracting wavefronts ===========================
  const int lp = lane & 31, hh = lane >> 5;
  const int pxh = wid & 1, kh = wid >> 1;  // 64 pixels x all BCO channels over half of every K row
  f32x16 acc[CO_T][2];
#pragma unroll
  for (int i = 0; i < CO_T; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // the two pixels of this lane inside the tile and their halo rows for tap (0,0). Tile column 0 of the
  // accumulators is the one this wavefront finishes after the K halves are folded, column 1 the one its
  // partner (pxh, kh ^ 1) finishes: which 32 pixels that is depends on kh, the code that follows does not.
  const int p0 = pxh * 64 + kh * 32 + lp, p1 = pxh * 64 + (kh ^ 1) * 32 + lp;
  const int xr0 = (p0 >> 4) * kwHaloW + (p0 & 15);
  const int xr1 = (p1 >> 4) * kwHaloW + (p1 & 15);
  const int xoff0 = xr0 * kwLds + hh * 16 + kh * (KI / 2) * KB;
  const int xoff1 = xr1 * kwLds + hh * 16 + kh * (KI / 2) * KB;
  const int wkey = (lp >> 1) & 7;  // slot swizzle of this lane's weight rows (32 i does not change it)
  int wofs[KI / 2];
#pragma unroll
  for (int kk = 0; kk < KI / 2; ++kk) {
    const int wb = hh * 16 + (kh * (KI / 2) + kk) * KB;
    wofs[kk] = lp * kwRow + ((((wb >> 4) ^ wkey) << 4) | (wb & 15));
  }
  // weights: global -> LDS directly, kwAhead steps ahead, requested by the contracting wavefronts themselves
  // (their stream has room between the MFMAs, and the loaders then never wait for memory on the
  // contracting wavefronts' behalf). A wavefront instruction moves 8 rows x 128 bytes; packet c of row r is
  // parked in slot c ^ ((r >> 1) & 7) of that row (conflict-free fragment reads without padding).
  // Instruction i covers rows (4 i + wid) * 8 ..+7 (1 KB of contiguous memory in the tile order of the
  // weights); the slot key does not depend on i.
  const int l8 = lane >> 3;
  const int wr0 = wid * 8 + l8;
  const int wc = (lane & 7) ^ ((wr0 >> 1) & 7);
  const bf16_t* __restrict__ wsrc = a.w + ((int64_t)blockIdx.y * (9 * nslab) * BCO + wr0) * 64 + wc * 8;
  auto dma_w_one = [&](const bf16_t* src, unsigned char* tile, int i) {  // instruction i of the WP that move one tile
#ifdef __HIP_DEVICE_COMPILE__  // the host pass only needs the kernel's stub; it does not know this builtin
    __builtin_amdgcn_global_load_lds(src + i * 32 * 64, tile + (i * 4 + wid) * 1024, 16, 0, 0);
#else
    (void)src; (void)tile;
#endif
  };
  auto w_src = [&](int step) { return wsrc + (int64_t)step * (BCO * 64); };
  // at most `VM` vector-memory operations outstanding; LDS reads are not waited for
  auto wait_vm = [&](auto vm_c) {
    constexpr int VM = decltype(vm_c)::value;
    __builtin_amdgcn_s_waitcnt((VM & 15) | (7 << 4) | (15 << 8) | ((VM >> 4) << 14));
  };
  constexpr int NF = (KI / 2) * CO_T;  // weight fragments of a tap for this wavefront
  static_assert(NF % (kwFA + 1) == 0, "a fragment's place in the ring does not depend on the tap");
  // The fragment stream runs ahead of the MFMAs across the taps: while the pairs of step s are issued
  // the wavefront requests the activation fragments of step s + 1 and, in its last kwFA pairs, the
  // first weight fragments of step s + 1 (both are complete in LDS one barrier earlier), so that the
  // MFMAs of the next step start right behind the barrier instead of an LDS round trip later.
  M::Frag xf[KI / 2][2], xn[KI / 2][2];
  M::Frag wf[kwFA + 1];
  auto x_ptr = [&](int xbuf, int tap, int j) {
    const int sh = (tap / 3) * kwHaloW + (tap % 3);
    return x_lds(xbuf) + (j ? xoff1 : xoff0) + sh * kwLds;
  };
  auto wload = [&](const unsigned char* wl, int idx) {
    const int kk = idx / CO_T, i = idx - kk * CO_T;
    return M::load((const bf16_t*)(wl + i * 32 * kwRow + wofs[kk]));
  };
  // one step: `wl` / `wl_next` the weight tiles of this and the next step, `xbuf_next` / `tap_next` where the
  // next step reads its activations
  // `dma_c`: the weights of step s + kwAhead exist and are requested, one instruction behind each of the first MFMA pairs
  auto compute = [&](const unsigned char* wl, const unsigned char* wl_next, int xbuf_next, int tap_next, auto dma_c,
                     const bf16_t* dsrc, unsigned char* dtile) {
    const unsigned char* xn0 = x_ptr(xbuf_next, tap_next, 0);
    const unsigned char* xn1 = x_ptr(xbuf_next, tap_next, 1);
#pragma unroll
    for (int idx = 0; idx < NF; ++idx) {
      const int nxt = idx + kwFA;
      wf[nxt % (kwFA + 1)] = nxt < NF ? wload(wl, nxt) : wload(wl_next, nxt - NF);
      // the activation fragments of the next step, one request per pair from the second pair on
      if (idx >= 1 && idx - 1 < KI) {
        const int q = idx - 1, kk = q >> 1, j = q & 1;
        xn[kk][j] = M::load((const bf16_t*)((j ? xn1 : xn0) + kk * KB));
      }
      __builtin_amdgcn_sched_barrier(0);
      const int kk = idx / CO_T, i = idx - kk * CO_T;
      M::mma(wf[idx % (kwFA + 1)], xf[kk][0], acc[i][0]);
      M::mma(wf[idx % (kwFA + 1)], xf[kk][1], acc[i][1]);
      if constexpr (decltype(dma_c)::value) {
        if (idx < WP) dma_w_one(dsrc, dtile, idx);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int kk = 0; kk < KI / 2; ++kk) {
      xf[kk][0] = xn[kk][0];
      xf[kk][1] = xn[kk][1];
    }
  };
  // a barrier that does not wait for this wavefront's LDS reads: those in flight are the requests for
  // the next step, whose tiles nobody writes before a later barrier
  // Before it the weights of step s + kwLead must have landed: they were requested kwAhead - kwLead steps
  // ago, younger are the requests of the steps since (`VM` of them: this wavefront issues nothing else).
  auto step_barrier = [&](auto vm_c) {
    asm volatile("" ::: "memory");
    wait_vm(vm_c);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };
  static_assert(NF >= WP, "one request behind each of the first MFMA pairs");

#pragma unroll
  for (int j = 0; j < kwAhead; ++j)  // nsteps >= 9 > kwAhead
#pragma unroll
    for (int i = 0; i < WP; ++i) dma_w_one(w_src(j), w_lds(j), i);
  barrier_keep<(kwAhead - kwLead) * WP>();  // prologue: halo of slab 0 and the weights of the first kwLead steps are in LDS
#pragma unroll
  for (int kk = 0; kk < KI / 2; ++kk) {
    xf[kk][0] = M::load((const bf16_t*)(x_ptr(0, 0, 0) + kk * KB));
    xf[kk][1] = M::load((const bf16_t*)(x_ptr(0, 0, 1) + kk * KB));
  }
#pragma unroll
  for (int idx = 0; idx < kwFA; ++idx) wf[idx] = wload(w_lds(0), idx);
  int wb = 0;                  // weight tile of the current step
  int wd = kwAhead % kwBuf;    // weight tile the requests of the current step go to
  const std::true_type dma_yes{};
  const std::false_type dma_no{};
  auto slab_steps = [&](int slab, auto last_c) {
    constexpr bool LAST = decltype(last_c)::value;
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
      const int wb_next = wb + 1 == kwBuf ? 0 : wb + 1;
      const int xb_next = tap < 8 ? (slab & 1) : ((slab + 1) & 1), tap_next = tap < 8 ? tap + 1 : 0;
      // (behind the last step the fragment requests read tiles that hold nothing new: in bounds, never used)
      if (!LAST || tap + kwAhead < 9) {
        compute(w_lds(wb), w_lds(wb_next), xb_next, tap_next, dma_yes, w_src(slab * 9 + tap + kwAhead), w_lds(wd));
        wd = wd + 1 == kwBuf ? 0 : wd + 1;
      } else {
        compute(w_lds(wb), w_lds(wb_next), xb_next, tap_next, dma_no, nullptr, nullptr);
      }
      // requests of the last kwAhead - kwLead steps (a step before this slab always issued; in the last slab
      // the steps whose tile would lie behind the end issue none)
      switch (tap) {  // `tap` is a constant once the loop is unrolled
#define LC_VM(TAP) \
  case TAP: step_barrier(std::integral_constant<int, ws_younger(TAP, LAST, WP)>{}); break;
        LC_VM(0) LC_VM(1) LC_VM(2) LC_VM(3) LC_VM(4) LC_VM(5) LC_VM(6) LC_VM(7) LC_VM(8)
#undef LC_VM
      }
      wb = wb_next;
    }
  };
  for (int slab = 0; slab + 1 < nslab; ++slab) slab_steps(slab, std::false_type{});
  slab_steps(nslab - 1, std::true_type{});
  asm volatile("" :: "v"(xf[0][0]), "v"(wf[0]));  // (the requests behind the last step have no other reader)
  __builtin_amdgcn_s_waitcnt(waitcnt_imm(63));      // no LDS read of this wavefront is in flight when the tiles are reused

  // ---------------- fold the two K halves and write out ----------------
  // The wavefront (pxh, kh) keeps its tile column 0 (pixels kh * 32 ..+31 of its 64), hands column 1 to its partner through LDS,
  // then turns each finished 32 x 32 tile through a private LDS patch so that a lane stores 16 bytes
  // of one pixel row and eight lanes cover its 128 contiguous bytes (the accumulator layout would
  // store 16-byte pieces of 32 different rows per instruction). Bias and residual are added in that
  // layout; the residual is requested before the barrier of the hand-over so its latency hides behind it.
  constexpr int kTile = 16 * 64;  // floats of one accumulator tile
  float* give = reinterpret_cast<float*>(smem) + (pxh * 2 + kh) * (CO_T * kTile);
  const float* take = reinterpret_cast<const float*>(smem) + (pxh * 2 + (kh ^ 1)) * (CO_T * kTile);
  float* patch = reinterpret_cast<float*>(smem + 4 * CO_T * kTile * 4) + wid * (32 * 36);
  static_assert(ws_lds_bytes<CO_T>() >= 4 * CO_T * kTile * 4 + 4 * 32 * 36 * 4, "hand-over area + patches");
  const int prow = lane >> 3, pcol = (lane & 7) * 4;  // patch read-back: rows prow + 8 k, channels pcol..pcol+3
#pragma unroll
  for (int i = 0; i < CO_T; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) give[(i * 16 + r) * 64 + lane] = acc[i][1][r];
  int64_t obase[4];
  bool okk[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int p = pxh * 64 + kh * 32 + prow + 8 * k;
    const int oy = ty0 + (p >> 4), ox = tx0 + (p & 15);
    okk[k] = oy < a.H && ox < a.W;
    obase[k] = okk[k] ? (((int64_t)frame * a.H + oy) * a.W + ox) * a.Cout + co0 + pcol : 0;
  }
  const float* R = a.res;
  // residual and bias of one 32-channel tile
  struct Side { f32x4 r[4]; f32x4 b; };
  auto load_side = [&](int i, Side& sd) {
    sd.b = a.bias ? *reinterpret_cast<const f32x4*>(a.bias + co0 + i * 32 + pcol) : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < 4; ++k)
      sd.r[k] = (R && okk[k]) ? *reinterpret_cast<const f32x4*>(R + obase[k] + i * 32) : f32x4{0.f, 0.f, 0.f, 0.f};
  };
  // all tiles at once: the given-away half of the accumulators is dead by now, so the registers are there,
  // and one memory latency (hidden behind the hand-over barrier) is paid instead of one per tile
  asm volatile("" ::: "memory");  // (the requests stay below the hand-over: above it they would not fit)
  Side side[CO_T];
#pragma unroll
  for (int i = 0; i < CO_T; ++i) load_side(i, side[i]);
  __syncthreads();
  float* Y = a.y;
  {
#pragma unroll
    for (int i = 0; i < CO_T; ++i) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[i][0][g * 4 + e] + take[(i * 16 + g * 4 + e) * 64 + lane];
        *reinterpret_cast<f32x4*>(patch + lp * 36 + g * 8 + hh * 4) = v;
      }
      // the patch is private to this wavefront, whose LDS operations complete in order
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      float ssum[4] = {0.f, 0.f, 0.f, 0.f}, ssq[4] = {0.f, 0.f, 0.f, 0.f};  // statistics of this lane's pixels
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        f32x4 v = *reinterpret_cast<const f32x4*>(patch + (prow + 8 * k) * 36 + pcol);
        v += side[i].b;
        v += side[i].r[k];
        if (okk[k]) {
          *reinterpret_cast<f32x4*>(Y + obase[k] + i * 32) = v;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            ssum[e] += v[e];
            ssq[e] = fmaf(v[e], v[e], ssq[e]);
          }
        }
      }
      if (a.stat) {
        // fold the eight lanes that hold the same channels, in a fixed order; the first writes.
        // One split = the 32 pixels of this wavefront (those inside the image).
#pragma unroll
        for (int e = 0; e < 4; ++e) {
#pragma unroll
          for (int m = 8; m < 64; m <<= 1) {
            ssum[e] += __shfl_xor(ssum[e], m, 64);
            ssq[e] += __shfl_xor(ssq[e], m, 64);
          }
        }
        if (prow == 0) {
          const int split = (((ty0 >> 3) * a.tiles_x + (tx0 >> 4)) * 2 + pxh) * 2 + kh;
          float* sp = a.stat + (((int64_t)frame * a.stat_splits + split) * a.Cout + co0 + i * 32 + pcol) * 2;
          *reinterpret_cast<f32x4*>(sp) = f32x4{ssum[0], ssq[0], ssum[1], ssq[1]};
          *reinterpret_cast<f32x4*>(sp + 4) = f32x4{ssum[2], ssq[2], ssum[3], ssq[3]};
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
  }
}

template <int CO_T, bool CAT>
static hipError_t run_ws(hipStream_t s, const FusedDesc& d) {
  constexpr int lds = ws_lds_bytes<CO_T>();
  auto kern = conv_ws_kernel<CO_T, CAT>;
  static bool attr_done = false;  // per instantiation
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  WsArgs a;
  a.x = (const float*)d.x; a.x2 = (const bf16_t*)d.x2; a.scale = d.scale; a.shift = d.shift;
  a.w = (const bf16_t*)d.w_tiles; a.bias = d.bias; a.res = (const float*)d.res; a.y = (float*)d.y;
  a.Cin = d.Cin; a.Cs = d.Cs; a.Cout = d.Cout;
  a.H = d.H; a.W = d.W; a.tiles_x = (d.W + 15) / 16; a.tiles_y = (d.H + 7) / 8;
  a.stat = d.stat; a.stat_splits = d.stat_splits;
  if (!conv_window_tiles(d, &a.win_tx0, &a.win_ty0, &a.win_tx, &a.win_ty)) return hipErrorInvalidValue;
  dim3 grid((unsigned)(a.win_tx * a.win_ty * d.frames), d.Cout / (CO_T * 32));
  kern<<<grid, 512, lds, s>>>(a);
  return hipGetLastError();
}

// The 3x3 convolutions of a bf16 stage whose widths suit the kernel above (a property of the stage,
// never of how it is chunked); hipErrorNotSupported otherwise.
hipError_t launch_conv_ws(hipStream_t s, const FusedDesc& d) {
  if (d.dt != kBF16 || d.taps != 9 || !d.y_f32 || d.planar_out || d.yt || d.q_cols || !d.w_tiles) return hipErrorNotSupported;
  if (d.src != 2 && d.src != 3) return hipErrorNotSupported;
  if (d.Cout % 160 != 0 || d.Cout_store != d.Cout || d.Cin % 64 != 0) return hipErrorNotSupported;
  if (d.src == 3 && (d.Cs % 64 != 0 || d.Cs <= 0 || d.Cs >= d.Cin || ((d.H | d.W) & 1))) return hipErrorNotSupported;
  if (d.stat && d.stat_splits != conv_stat_splits(d.H, d.W)) return hipErrorInvalidValue;
  // 32-bit pixel and byte-offset arithmetic in the loader
  if ((int64_t)d.frames * d.H * d.W * (int64_t)d.Cin * 4 >= (int64_t)1 << 40 || (int64_t)d.frames * d.H * d.W >= (int64_t)1 << 30)
    return hipErrorNotSupported;
  if (d.frames <= 0) return hipSuccess;
  return d.src == 3 ? run_ws<5, true>(s, d) : run_ws<5, false>(s, d);
}

}  // namespace lc

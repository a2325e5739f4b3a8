// Fused-loader implicit-GEMM kernels on 32x32 MFMA tiles (gfx950): the 3x3 stride-1 convolutions
// and the per-row linear layers of the stage.
//
// Product (transposed): D[cout][pixel] = sum_k W[cout][k] X[pixel][k], k = tap * Cin + ci.
// One workgroup = 4 wavefronts = BCO output channels x 128 pixels. The LDS read port, not the MFMA
// pipe, is the scarce resource at this tile size, so the wavefronts do not split the tile four ways:
// each takes all BCO channels of 64 pixels (CO_T x 2 accumulator tiles of 32x32, every weight
// fragment feeds two MFMAs) over one HALF of the K elements of every step, and the two halves are
// added through LDS once, before the epilogue.
//
// What is fused into the loader of X (it is staged through registers anyway):
//   * GroupNorm apply (+ SiLU): x is the fp32 residual stream; the per-frame, per-channel
//     scale/shift come from the statistics kernels; the result is rounded to the operand type once,
//     on its way into LDS. Out-of-image taps are zero *after* the activation (zero padding pads the
//     normalised tensor).
//   * the skip-concat of the up block, U_m = Concat(D_m, up2(U_{m+1})) ("Feature Calculation"
//     paragraph): channel slabs below C_skip are read from the fp32 skip feature, the others from
//     the cached deep feature at (y/2, x/2). Neither the concatenated nor the normalised tensor is
//     ever written to memory.
// A convolution stages, per 128-byte channel slab, the 10 x 18 halo of its 8 x 16 pixel tile once
// and walks the 9 taps over it by shifting LDS addresses; the weights of a (slab, tap) step are
// streamed through a second LDS tile one step ahead, and the next slab's halo is fetched and
// activated one 16-byte packet per thread per tap while the MFMAs of the current slab run.
#include <type_traits>

#include "lc_internal.h"

namespace lc {

namespace {

constexpr int kRow = 128;     // K bytes per LDS row per step
constexpr int kLds = 144;     // LDS row stride (bytes): 16-byte reads of 16 consecutive rows hit 64 distinct banks
constexpr int kHaloW = 18, kHaloH = 10, kHalo = kHaloW * kHaloH;
constexpr int kHaloRows = 192;  // LDS rows of a halo tile: 180 used, padded to 6 rounds of 32 rows

struct GemmArgs {
  const void* x;        // PLAIN: T [rows][Cin]; NORM: float [..][Cin]; CAT: float skip [..][Cs]
  const void* x2;       // CAT: deep, T [frames][H/2][W/2][Cin - Cs]
  const float* scale;   // [frames][Cin]
  const float* shift;
  const void* w;        // T [Cout][taps * Cin]
  const float* bias;
  const float* res;     // fp32, indexed like y (may alias y)
  void* y;
  int Cin, Cs, Cout, Cout_store, ldw;
  void* yt;             // linear only: channels >= yt_from go, transposed, to the V^T layout of spatial attention
  int yt_from, yt_T, yt_Tp;
  int frames, H, W, tiles_x, tiles_y;
  int win_tx0, win_ty0, win_tx, win_ty;  // conv: the tiles a launch covers, origin and extent in tiles
  int64_t rows;
  RowMap in_map, out_map;
  float* stat;          // conv, fp32 output: per-channel statistics of the output (see FusedDesc), or nullptr
  int stat_splits;
  float q_scale;        // linear: output channels below q_cols are multiplied by this before rounding
  int q_cols;
};

constexpr int FA = 3;  // weight fragments requested from LDS ahead of the MFMAs that use them
constexpr int kWBuf = 3;  // conv: weight tiles in LDS; the loads run kWBuf - 1 steps ahead of their use

// conv (TAPS == 9): kWBuf weight tiles of BCO x 128 bytes, written by LDS-direct loads (no padding:
// a wavefront's 64 x 16 bytes land contiguously; bank conflicts are avoided by a swizzle instead),
// then two padded halo tiles. Linear (TAPS == 1): two {weight tile, activation tile} pairs, all padded.
template <int BCO, int XROWS, int TAPS>
constexpr int gemm_lds_bytes() {
  return TAPS == 9 ? kWBuf * BCO * kRow + 2 * XROWS * kLds : 2 * (BCO + XROWS) * kLds;
}

// vector-memory loads issued in tap t of a conv slab body (see the main loop): scale/shift at tap 0 and a
// halo packet at taps < xr if a next slab follows (`more`), then the weights of step s + ah if there is one.
// t < 0 is tap 8 of the slab before, which was not the last one: weights only.
constexpr int conv_tap_loads(int t, bool more, int n_aff, int n_pkt, int xr, int wp, int ah) {
  if (t < 0) return wp;
  return (more ? (t == 0 ? n_aff : 0) + (t < xr ? n_pkt : 0) : 0) + ((more || t + ah < 9) ? wp : 0);
}
// loads younger than the weights of step s + 1 at the end of tap `tap`: those of the last ah - 1 taps
constexpr int conv_tap_keep(int tap, bool more, int n_aff, int n_pkt, int xr, int wp, int ah) {
  int n = 0;
  for (int j = 0; j < ah - 1; ++j) n += conv_tap_loads(tap - j, more, n_aff, n_pkt, xr, wp, ah);
  return n;
}
}  // namespace

// SRC: 0 plain operand-type rows, 1 fp32 rows with scale/shift, 2 the same + SiLU, 3 concat (+ SiLU)
template <class T, class OT, int TAPS, int CO_T, int SRC, bool PLANAR>
__global__ __launch_bounds__(256) void gemm_kernel(GemmArgs a) {
  typedef Mma32<T> M;
  constexpr int VEC = Vec16<T>::N;               // operand elements per 16-byte LDS packet
  constexpr int BKC = kRow / (int)sizeof(T);     // K elements per step
  constexpr int BCO = CO_T * 32;
  constexpr int XROWS = TAPS == 9 ? kHaloRows : 128;
  constexpr int WP = (BCO * 8 + 255) / 256;      // weight packets per thread per step
  constexpr int XR = XROWS / 32;                 // x packets per thread per slab
  constexpr int KI = kRow / (M::K * (int)sizeof(T));  // MFMA k-steps per LDS row
  constexpr int LKB = M::LK * (int)sizeof(T), KB = M::K * (int)sizeof(T);
  constexpr bool NORM = SRC != 0;
  constexpr bool SILU = SRC >= 2;
  static_assert(KI % 2 == 0, "the k-steps of a row are split between two wavefronts");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  auto w_lds = [&](int b) { return TAPS == 9 ? smem + b * BCO * kRow : smem + b * (BCO + XROWS) * kLds; };
  auto x_lds = [&](int b) {
    return TAPS == 9 ? smem + kWBuf * BCO * kRow + b * XROWS * kLds : smem + b * (BCO + XROWS) * kLds + BCO * kLds;
  };

  const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const int lp = lane & 31, hh = lane >> 5;
  // wavefront = (pixel half, K half): 64 pixels x all BCO channels over half of every K row
  const int pxh = wid & 1, kh = wid >> 1;
  const int co0 = blockIdx.y * BCO;
  const T* __restrict__ Wt = (const T*)a.w;

  int frame = 0, ty0 = 0, tx0 = 0;
  int64_t row0 = 0;
  if (TAPS == 9) {
    // tiles of the window (the whole frame by default), counted in the frame's own tile grid
    int t = blockIdx.x;
    tx0 = (a.win_tx0 + t % a.win_tx) * 16;
    t /= a.win_tx;
    ty0 = (a.win_ty0 + t % a.win_ty) * 8;
    frame = t / a.win_ty;
  } else {
    row0 = (int64_t)blockIdx.x * 128;
  }
  const int kp = tid & 7, lrow = tid >> 3;  // this thread moves packet kp of rows lrow + 32 * i

  // ---------------- weights of a later step ----------------
  // conv: global -> LDS directly, two steps ahead, into the tile that was read one step ago. A
  // wavefront instruction moves 8 rows x 128 bytes; the 16-byte packet c of row r is parked in slot
  // c ^ ((r >> 1) & 7) of that row, which makes the MFMA fragment reads (32 consecutive rows, one
  // slot) conflict-free without padding. linear: global -> registers -> padded LDS tile, one step ahead.
  static_assert(TAPS != 9 || (BCO * 8) % 256 == 0, "whole wavefront instructions");
  auto dma_w_one = [&](int step, int buf, int i) {  // instruction i of the WP that move one tile
    const int slab = step / TAPS, tap = step - slab * TAPS;
    const int grp = i * 4 + wid;  // 8 rows
    const int r = grp * 8 + (lane >> 3);
    const int c = (lane & 7) ^ ((r >> 1) & 7);
    const T* src = Wt + (int64_t)(co0 + r) * a.ldw + tap * a.Cin + slab * BKC + c * VEC;
#ifdef __HIP_DEVICE_COMPILE__  // the host pass only needs the kernel's stub; it does not know this builtin
    __builtin_amdgcn_global_load_lds(src, w_lds(buf) + grp * 1024, 16, 0, 0);
#else
    (void)src;
#endif
  };
  auto dma_w = [&](int step, int buf) {
#pragma unroll
    for (int i = 0; i < WP; ++i) dma_w_one(step, buf, i);
  };
  constexpr int NW = 1;
  Vec16<T> wregs[NW][WP];
  auto issue_w = [&](int step, Vec16<T> (&wreg)[WP]) {
    const int slab = step / TAPS, tap = step - slab * TAPS;
    const int kofs = tap * a.Cin + slab * BKC + kp * VEC;
#pragma unroll
    for (int i = 0; i < WP; ++i) {
      const int r = min(lrow + 32 * i, BCO - 1);
      wreg[i] = load16(Wt + (int64_t)(co0 + r) * a.ldw + kofs);
    }
  };
  auto store_w = [&](int buf, const Vec16<T> (&wreg)[WP]) {
#pragma unroll
    for (int i = 0; i < WP; ++i) {
      const int r = lrow + 32 * i;
      if (BCO % 32 == 0 || r < BCO) *reinterpret_cast<Vec16<T>*>(w_lds(buf) + r * kLds + kp * 16) = wreg[i];
    }
  };

  // ---------------- x packets: fetch raw (branch-free, clamped addresses), then activate + round + store ----
  // raw bits as loaded (converted only when consumed, so that no wait follows the load)
  struct XRaw { f32x4 q[2]; bool ok; };  // q[0] alone = one operand-type packet; q[0..1] = 8 floats (q[0] = 4 floats if T is float)
  struct Affine { float sc[VEC], sh[VEC]; };
  // conv: round r of a slab -> halo row lrow + 32 r (rows >= 180 are padding, loaded from clamped
  // addresses and never read); linear: row lrow + 32 r of the tile
  auto load_raw = [&](const float* p, XRaw& o) {  // VEC floats
    o.q[0] = *reinterpret_cast<const f32x4*>(p);
    if (VEC == 8) o.q[1] = *reinterpret_cast<const f32x4*>(p + 4);
  };
  // `deep_c`: compile-time flag, the slab lies in the cached deep feature (SRC == 3 only)
  auto fetch_x = [&](int slab, int r, XRaw& o, auto deep_c) {
    constexpr bool DEEP = decltype(deep_c)::value;
    const int c0 = slab * BKC + kp * VEC;
    if (TAPS == 9) {
      const int hp = lrow + 32 * r;
      const int hy = hp / kHaloW, hx = hp - hy * kHaloW;
      const int iy = ty0 + hy - 1, ix = tx0 + hx - 1;
      o.ok = iy >= 0 && iy < a.H && ix >= 0 && ix < a.W;
      const int cy = min(max(iy, 0), a.H - 1), cx = min(max(ix, 0), a.W - 1);
      if (SRC == 3 && DEEP) {
        const int64_t dr = ((int64_t)frame * (a.H >> 1) + (cy >> 1)) * (a.W >> 1) + (cx >> 1);
        o.q[0] = *reinterpret_cast<const f32x4*>((const T*)a.x2 + dr * (a.Cin - a.Cs) + (c0 - a.Cs));
      } else if (NORM) {
        const int ldx = SRC == 3 ? a.Cs : a.Cin;
        load_raw((const float*)a.x + (((int64_t)frame * a.H + cy) * a.W + cx) * ldx + c0, o);
      } else {
        o.q[0] = *reinterpret_cast<const f32x4*>((const T*)a.x + (((int64_t)frame * a.H + cy) * a.W + cx) * a.Cin + c0);
      }
    } else {
      const int64_t rr = row0 + lrow + 32 * r;
      o.ok = rr < a.rows;
      const int64_t sr = a.in_map(o.ok ? rr : a.rows - 1);
      if (NORM) load_raw((const float*)a.x + sr * a.Cin + c0, o);
      else o.q[0] = *reinterpret_cast<const f32x4*>((const T*)a.x + sr * a.Cin + c0);
    }
  };
  // scale/shift of the channels this thread moves: conv = one set per slab (fixed frame); linear =
  // one set per packet (a tile may straddle frames)
  auto load_affine = [&](int slab, int64_t f, Affine& af) {
    if (NORM) {
      const int c0 = slab * BKC + kp * VEC;
      load_f<float, VEC>(a.scale + f * a.Cin + c0, af.sc);
      load_f<float, VEC>(a.shift + f * a.Cin + c0, af.sh);
    }
  };
  auto row_frame = [&](int r) -> int64_t {
    const int64_t rr = row0 + lrow + 32 * r;
    return (rr < a.rows ? rr : a.rows - 1) / a.in_map.rows_per_seg;
  };
  // one element of a packet: activation arithmetic only
  auto finish_elem = [&](int e, const XRaw& o, const Affine& af, auto deep_c, float (&vals)[VEC]) {
    constexpr bool from_t = !NORM || (SRC == 3 && decltype(deep_c)::value);
    float t;
    if (from_t) {
      if constexpr (sizeof(T) == 2) {  // element e of the bf16 packet held in q[0]
        typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
        const uint32_t wd = __builtin_bit_cast(u32x4, o.q[0])[e >> 1];
        t = __builtin_bit_cast(float, (e & 1) ? (wd & 0xffff0000u) : (wd << 16));
      } else {
        t = o.q[0][e];
      }
    } else {
      t = o.q[e >> 2][e & 3];
    }
    if (NORM) {
      t = fmaf(t, af.sc[e], af.sh[e]);
      if (SILU) t = silu_fast(t);
    }
    vals[e] = o.ok ? t : 0.f;
  };
  auto finish_store = [&](int buf, int r, const float (&vals)[VEC]) {
    Vec16<T> pk;
#pragma unroll
    for (int e = 0; e < VEC; ++e) pk.set(e, vals[e]);
    *reinterpret_cast<Vec16<T>*>(x_lds(buf) + (lrow + 32 * r) * kLds + kp * 16) = pk;
  };
  auto finish_x = [&](int buf, int r, const XRaw& o, const Affine& af, auto deep_c) {
    float vals[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) finish_elem(e, o, af, deep_c, vals);
    finish_store(buf, r, vals);
  };

  f32x16 acc[CO_T][2];
#pragma unroll
  for (int i = 0; i < CO_T; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // the two pixels of this lane inside the tile and their LDS rows for tap (0,0)
  const int p0 = pxh * 64 + lp, p1 = p0 + 32;
  const int xr0 = TAPS == 9 ? (p0 >> 4) * kHaloW + (p0 & 15) : p0;
  const int xr1 = TAPS == 9 ? (p1 >> 4) * kHaloW + (p1 & 15) : p1;

  // One tap. All activation fragments first, then the weight fragments in a ring that runs FA reads
  // ahead of the MFMAs using them (one wavefront per SIMD: nothing else hides the LDS latency).
  // `side(idx)` is vector work to run in the shadow of MFMA pair idx; the scheduling barriers pin
  // this order.
  constexpr int NF = (KI / 2) * CO_T;  // weight fragments of a tap for this wavefront
  auto compute = [&](int wbuf, int xbuf, int tap, auto side) {
    const int sh = TAPS == 9 ? (tap / 3) * kHaloW + (tap % 3) : 0;
    const unsigned char* xb = x_lds(xbuf) + hh * LKB + kh * (KI / 2) * KB;
    const unsigned char* xl0 = xb + (xr0 + sh) * kLds;
    const unsigned char* xl1 = xb + (xr1 + sh) * kLds;
    const int wstride = TAPS == 9 ? kRow : kLds;
    const unsigned char* wl = w_lds(wbuf) + lp * wstride;
    const int wkey = TAPS == 9 ? (lp >> 1) & 7 : 0;  // slot swizzle of this lane's rows (32 i does not change it)
    auto wload = [&](int idx) {
      const int kk = idx / CO_T, i = idx - kk * CO_T;
      const int wb = hh * LKB + (kh * (KI / 2) + kk) * KB;  // byte of the fragment inside the row
      const int wofs = (((wb >> 4) ^ wkey) << 4) | (wb & 15);
      return M::load((const T*)(wl + i * 32 * wstride + wofs));
    };
    typename M::Frag xf[KI / 2][2];
    typename M::Frag wf[FA + 1];
    xf[0][0] = M::load((const T*)(xl0));
    xf[0][1] = M::load((const T*)(xl1));
#pragma unroll
    for (int idx = 0; idx < FA && idx < NF; ++idx) wf[idx] = wload(idx);
#pragma unroll
    for (int kk = 1; kk < KI / 2; ++kk) {
      xf[kk][0] = M::load((const T*)(xl0 + kk * KB));
      xf[kk][1] = M::load((const T*)(xl1 + kk * KB));
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int idx = 0; idx < NF; ++idx) {
      if (idx + FA < NF) wf[(idx + FA) % (FA + 1)] = wload(idx + FA);
      __builtin_amdgcn_sched_barrier(0);
      const int kk = idx / CO_T, i = idx - kk * CO_T;
      M::mma(wf[idx % (FA + 1)], xf[kk][0], acc[i][0]);
      M::mma(wf[idx % (FA + 1)], xf[kk][1], acc[i][1]);
      side(idx);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  const int nslab = a.Cin / BKC;
  const int nsteps = TAPS * nslab;

  // ---------------- prologue ----------------
  // conv: a halo packet is requested at tap r and consumed at the end of tap r + 3, after that tap's
  // own request has been issued: four register sets in rotation
  constexpr int NXS = TAPS == 9 ? 4 : XR;
  const std::false_type no_c{};
  const std::true_type yes_c{};
  Affine aff[TAPS == 9 ? 1 : XR];
  XRaw xin[XR];
  if (TAPS == 9) {
#pragma unroll
    for (int j = 0; j < kWBuf - 1; ++j) dma_w(j, j);  // nsteps >= 9 > kWBuf
    load_affine(0, frame, aff[0]);
#pragma unroll
    for (int r = 0; r < XR; ++r) fetch_x(0, r, xin[r], no_c);  // slab 0 is never in the deep part
#pragma unroll
    for (int r = 0; r < XR; ++r) finish_x(0, r, xin[r], aff[0], no_c);
    barrier_keep<(kWBuf - 2) * WP>();  // the weights of step 0 have landed, the later ones may still be on their way
  } else {
    issue_w(0, wregs[0]);
#pragma unroll
    for (int r = 0; r < XR; ++r) {
      fetch_x(0, r, xin[r], no_c);
      load_affine(0, row_frame(r), aff[r]);
    }
#pragma unroll
    for (int r = 0; r < XR; ++r) finish_x(0, r, xin[r], aff[r], no_c);
    store_w(0, wregs[0]);
    __syncthreads();
  }

  // ---------------- main loop ----------------
  // conv: per step (= one tap of one 64-channel slab) a thread issues at most one halo packet of the
  // NEXT slab (rounds 0..5 at taps 0..5, activated and stored three taps later, interleaved with the
  // MFMAs of that tap) and the weights of
  // step s+2; it stores the weights of step s+1 (fetched during step s-1) after its MFMAs. The
  // number of loads per tap is fixed at compile time - the loop is split by where the next slab
  // comes from (skip feature, deep feature, none) instead of branching - so every wait is an exact
  // count of younger loads and global latency has two to three steps to hide in. The scheduling
  // barriers pin the order: left alone, the compiler sinks the loads below the MFMAs.
  if (TAPS == 9) {
    auto slab_body = [&](int slab, auto more_c, auto deep_c) {
      constexpr bool MORE = decltype(more_c)::value;
#pragma unroll
      for (int tap = 0; tap < 9; ++tap) {
        const int s = slab * 9 + tap;
        __builtin_amdgcn_sched_barrier(0);
        if (MORE) {
          if (tap == 0) load_affine(slab + 1, frame, aff[0]);
          if (tap < XR) fetch_x(slab + 1, tap, xin[tap % NXS], deep_c);
        }
        __builtin_amdgcn_sched_barrier(0);
        constexpr int AH = kWBuf - 1;  // the last slab has no step s + AH for its last AH taps
        // the activation arithmetic of the halo packet requested three taps ago rides in the shadow
        // of the MFMAs, a few elements per MFMA pair; the packet is stored after the last pair
        float xv[VEC];
        constexpr int PER = (VEC + NF - 1) / NF;
        compute(s % kWBuf, slab & 1, tap, [&](int idx) {
          // the weights of step s + AH are requested one instruction per MFMA pair: issued in a
          // burst at the head of the tap they hold the MFMAs up
          if ((MORE || tap + AH < 9) && idx < WP) dma_w_one(s + AH, (s + AH) % kWBuf, idx);
          if (MORE && tap >= 3 && tap - 3 < XR) {
#pragma unroll
            for (int e = idx * PER; e < (idx + 1) * PER && e < VEC; ++e)
              finish_elem(e, xin[(tap - 3) % NXS], aff[0], deep_c, xv);
            if (idx == NF - 1) finish_store((slab + 1) & 1, tap - 3, xv);
          }
        });
        __builtin_amdgcn_sched_barrier(0);
        // Before the barrier the weights of step s + 1 must have landed. They were the last loads of
        // tap s + 1 - AH; younger than them are exactly the loads of the AH - 1 taps since, whose
        // number is fixed at compile time: per tap the scale/shift (tap 0) and halo packet (taps
        // 0..5) of the next slab, then the weights of a later step.
        constexpr bool DEEPC = decltype(deep_c)::value;
        constexpr int n_aff = !NORM ? 0 : 2 * (VEC / 4);
        constexpr int n_pkt = (SRC == 3 && DEEPC) || !NORM ? 1 : VEC / 4;
#define LC_KEEP(TAP) \
  case TAP: barrier_keep<conv_tap_keep(TAP, MORE, n_aff, n_pkt, XR, WP, AH)>(); break;
        switch (tap) {  // `tap` is a constant once the loop is unrolled
          LC_KEEP(0) LC_KEEP(1) LC_KEEP(2) LC_KEEP(3) LC_KEEP(4) LC_KEEP(5) LC_KEEP(6) LC_KEEP(7) LC_KEEP(8)
        }
#undef LC_KEEP
      }
    };
    const int nskip = SRC == 3 ? a.Cs / BKC : nslab;  // slabs read from x; the rest from x2
    int slab = 0;
    for (; slab + 1 < nskip; ++slab) slab_body(slab, yes_c, no_c);
    if (SRC == 3)
      for (; slab + 1 < nslab; ++slab) slab_body(slab, yes_c, yes_c);
    slab_body(nslab - 1, no_c, no_c);
  } else {
    for (int s = 0; s < nsteps; ++s) {
      const bool more = s + 1 < nsteps;
      if (more) {
#pragma unroll
        for (int r = 0; r < XR; ++r) {
          fetch_x(s + 1, r, xin[r], no_c);
          load_affine(s + 1, row_frame(r), aff[r]);
        }
        issue_w(s + 1, wregs[0]);
      }
      __builtin_amdgcn_sched_barrier(0);
      compute(s & 1, s & 1, 0, [](int) {});
      __builtin_amdgcn_sched_barrier(0);
      if (more) {
#pragma unroll
        for (int r = 0; r < XR; ++r) finish_x((s + 1) & 1, r, xin[r], aff[r], no_c);
        store_w((s + 1) & 1, wregs[0]);
      }
      __syncthreads();
    }
  }

  if constexpr (TAPS == 9 && !PLANAR) {
    // ---------------- conv: fold the two K halves and write out, both wavefronts of a pixel half at work ----------------
    // The wavefront (pxh, kh) keeps the 32-pixel tiles j = kh, hands the others to its partner through LDS,
    // then turns each finished 32 x 32 tile through a private LDS patch so that a lane stores 16 bytes
    // of one pixel row and eight lanes cover its 128 contiguous bytes (the accumulator layout would
    // store 16-byte pieces of 32 different rows per instruction). Bias and residual are added in that
    // layout; the residual is requested before the hand-over so its latency hides behind it.
    constexpr int kTile = 16 * 64;  // floats of one accumulator tile
    float* give = reinterpret_cast<float*>(smem) + (pxh * 2 + kh) * (CO_T * kTile);
    const float* take = reinterpret_cast<const float*>(smem) + (pxh * 2 + (kh ^ 1)) * (CO_T * kTile);
    float* patch = reinterpret_cast<float*>(smem + 4 * CO_T * kTile * 4) + wid * (32 * 36);
    static_assert(gemm_lds_bytes<BCO, XROWS, TAPS>() >= 4 * CO_T * kTile * 4 + 4 * 32 * 36 * 4, "hand-over area + patches");
    const int prow = lane >> 3, pcol = (lane & 7) * 4;  // patch read-back: rows prow + 8 k, channels pcol..pcol+3
    int64_t obase[4];
    bool okk[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int p = pxh * 64 + kh * 32 + prow + 8 * k;
      const int oy = ty0 + (p >> 4), ox = tx0 + (p & 15);
      okk[k] = oy < a.H && ox < a.W;
      obase[k] = okk[k] ? (((int64_t)frame * a.H + oy) * a.W + ox) * a.Cout_store + co0 + pcol : 0;
    }
    const float* R = a.res;
    f32x4 rres[CO_T][4];
    f32x4 bias_l[CO_T];
#pragma unroll
    for (int i = 0; i < CO_T; ++i) {
      bias_l[i] = a.bias ? *reinterpret_cast<const f32x4*>(a.bias + co0 + i * 32 + pcol) : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int k = 0; k < 4; ++k)
        rres[i][k] = (R && okk[k]) ? *reinterpret_cast<const f32x4*>(R + obase[k] + i * 32) : f32x4{0.f, 0.f, 0.f, 0.f};
    }
    auto hand_over = [&](auto jc) {  // jc: the tile column this wavefront gives away
      constexpr int J = decltype(jc)::value;
#pragma unroll
      for (int i = 0; i < CO_T; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) give[(i * 16 + r) * 64 + lane] = acc[i][J][r];
    };
    if (kh == 0) hand_over(std::integral_constant<int, 1>{});
    else hand_over(std::integral_constant<int, 0>{});
    __syncthreads();
    OT* Y = (OT*)a.y;
    auto finish = [&](auto jc) {  // jc: the tile column this wavefront keeps
      constexpr int J = decltype(jc)::value;
#pragma unroll
      for (int i = 0; i < CO_T; ++i) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          f32x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = acc[i][J][g * 4 + e] + take[(i * 16 + g * 4 + e) * 64 + lane];
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
          v += bias_l[i];
          v += rres[i][k];
          if (okk[k]) {
            const int64_t o = obase[k] + i * 32;
            if constexpr (sizeof(OT) == 2) {
              bf16x4 ov;
#pragma unroll
              for (int e = 0; e < 4; ++e) ov[e] = static_cast<bf16_t>(v[e]);
              *reinterpret_cast<bf16x4*>((bf16_t*)Y + o) = ov;
            } else {
              *reinterpret_cast<f32x4*>((float*)Y + o) = v;
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                ssum[e] += v[e];
                ssq[e] = fmaf(v[e], v[e], ssq[e]);
              }
            }
          }
        }
        if constexpr (sizeof(OT) == 4) {
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
              float* sp = a.stat + (((int64_t)frame * a.stat_splits + split) * a.Cout_store + co0 + i * 32 + pcol) * 2;
              *reinterpret_cast<f32x4*>(sp) = f32x4{ssum[0], ssq[0], ssum[1], ssq[1]};
              *reinterpret_cast<f32x4*>(sp + 4) = f32x4{ssum[2], ssq[2], ssum[3], ssq[3]};
            }
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
      }
    };
    if (kh == 0) finish(std::integral_constant<int, 0>{});
    else finish(std::integral_constant<int, 1>{});
    return;
  }

  // ---------------- fold the two K halves: the upper half hands its tiles over through LDS ----------------
  float* red = reinterpret_cast<float*>(smem) + pxh * (CO_T * 2 * 16 * 64);
  if (kh == 1) {
#pragma unroll
    for (int i = 0; i < CO_T; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) red[((i * 2 + j) * 16 + r) * 64 + lane] = acc[i][j][r];
  }
  __syncthreads();
  if (kh == 1) return;
#pragma unroll
  for (int i = 0; i < CO_T; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] += red[((i * 2 + j) * 16 + r) * 64 + lane];

  // ---------------- epilogue: lane holds, for pixel p_j, channels co0 + 32 i + 8 g + 4 hh + {0..3} ----------------
  OT* Y = (OT*)a.y;
  const float* R = a.res;  // may alias Y (in-place residual of a linear layer)
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int p = j == 0 ? p0 : p1;
    int64_t orow;
    int oy = 0, ox = 0;
    bool ok;
    if (TAPS == 9) {
      oy = ty0 + (p >> 4);
      ox = tx0 + (p & 15);
      ok = oy < a.H && ox < a.W;
      orow = ((int64_t)frame * a.H + oy) * a.W + ox;
    } else {
      ok = row0 + p < a.rows;
      orow = ok ? a.out_map(row0 + p) : 0;
    }
    if (!ok) continue;
    // the residual (which may be y itself) of this pixel, all of it before the first store: a load placed after a
    // store that may alias it cannot be moved up, and would pay a round trip to memory each
    f32x4 rv[CO_T][4];
    if (!PLANAR && R) {
#pragma unroll
      for (int i = 0; i < CO_T; ++i)
#pragma unroll
        for (int g = 0; g < 4; ++g) rv[i][g] = *reinterpret_cast<const f32x4*>(R + orow * a.Cout_store + co0 + i * 32 + g * 8 + hh * 4);
    }
#pragma unroll
    for (int i = 0; i < CO_T; ++i) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int co = co0 + i * 32 + g * 8 + hh * 4;
        if (PLANAR) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            if (co + e < a.Cout_store) {
              const float v = acc[i][j][g * 4 + e] + (a.bias ? a.bias[co + e] : 0.f);
              Y[(((int64_t)frame * a.Cout_store + co + e) * a.H + oy) * a.W + ox] = from_f32<OT>(v);
            }
          }
        } else {
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = acc[i][j][g * 4 + e] + (a.bias ? a.bias[co + e] : 0.f);
          if (TAPS == 1 && co < a.q_cols) {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] *= a.q_scale;
          }
          if (TAPS == 1 && a.yt && co >= a.yt_from) {  // uniform over the workgroup
            const int64_t rr = row0 + p;
            const int64_t f = rr / a.yt_T;
            const int t = (int)(rr - f * a.yt_T);
            OT* dst = (OT*)a.yt + (f * (a.Cout - a.yt_from) + (co - a.yt_from)) * a.yt_Tp + (t & ~63) + vcol<OT>(t & 63);
#pragma unroll
            for (int e = 0; e < 4; ++e) dst[(int64_t)e * a.yt_Tp] = from_f32<OT>(v[e]);
            continue;
          }
          const int64_t o = orow * a.Cout_store + co;
          if (R) {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] += rv[i][g][e];
          }
          if constexpr (sizeof(OT) == 2) {
            bf16x4 ov;
#pragma unroll
            for (int e = 0; e < 4; ++e) ov[e] = static_cast<bf16_t>(v[e]);
            *reinterpret_cast<bf16x4*>((bf16_t*)Y + o) = ov;
          } else {
            *reinterpret_cast<f32x4*>((float*)Y + o) = f32x4{v[0], v[1], v[2], v[3]};
          }
        }
      }
    }
  }
}

template <class T, class OT, int TAPS, int CO_T, int SRC, bool PLANAR>
static hipError_t run_gemm(hipStream_t s, const FusedDesc& d) {
  constexpr int BCO = CO_T * 32;
  constexpr int XROWS = TAPS == 9 ? kHaloRows : 128;
  constexpr int lds = gemm_lds_bytes<BCO, XROWS, TAPS>();
  static_assert(lds >= 2 * CO_T * 2 * 16 * 64 * 4, "the K-half hand-over reuses the operand tiles");
  auto kern = gemm_kernel<T, OT, TAPS, CO_T, SRC, PLANAR>;
  static bool attr_done = false;  // per instantiation
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  GemmArgs a;
  a.x = d.x; a.x2 = d.x2; a.scale = d.scale; a.shift = d.shift; a.w = d.w; a.bias = d.bias;
  a.res = (const float*)d.res; a.y = d.y;
  a.Cin = d.Cin; a.Cs = d.Cs; a.Cout = d.Cout; a.Cout_store = d.yt ? d.yt_from : d.Cout_store; a.ldw = d.taps * d.Cin;
  a.yt = d.yt; a.yt_from = d.yt_from; a.yt_T = d.yt_T; a.yt_Tp = d.yt_Tp;
  a.frames = d.frames; a.H = d.H; a.W = d.W;
  a.tiles_x = (d.W + 15) / 16; a.tiles_y = (d.H + 7) / 8;
  a.rows = d.rows; a.in_map = d.in_map; a.out_map = d.out_map;
  a.stat = d.stat; a.stat_splits = d.stat_splits;
  a.q_scale = d.q_scale; a.q_cols = d.q_cols;
  dim3 grid;
  a.win_tx0 = a.win_ty0 = 0; a.win_tx = a.tiles_x; a.win_ty = a.tiles_y;
  if (TAPS == 9) {
    if (d.frames <= 0) return hipSuccess;
    if (!conv_window_tiles(d, &a.win_tx0, &a.win_ty0, &a.win_tx, &a.win_ty)) return hipErrorInvalidValue;
    grid = dim3((unsigned)(a.win_tx * a.win_ty * d.frames), d.Cout / BCO);
  } else {
    if (d.rows <= 0) return hipSuccess;
    grid = dim3((unsigned)((d.rows + 127) / 128), d.Cout / BCO);
  }
  kern<<<grid, 256, lds, s>>>(a);
  return hipGetLastError();
}

template <class T, class OT, int TAPS, int SRC>
static hipError_t by_width(hipStream_t s, const FusedDesc& d) {
  if (d.Cout % 160 == 0) return run_gemm<T, OT, TAPS, 5, SRC, false>(s, d);
  if (d.Cout % 64 == 0) return run_gemm<T, OT, TAPS, 2, SRC, false>(s, d);
  return hipErrorInvalidValue;
}

template <class T>
static hipError_t by_kind(hipStream_t s, const FusedDesc& d) {
  const bool y32 = d.y_f32 || sizeof(T) == 4;
  if (d.planar_out) {
    if (d.taps != 9 || d.src != 2 || d.Cout != 32 || d.res) return hipErrorInvalidValue;
    return run_gemm<T, T, 9, 1, 2, true>(s, d);
  }
  if (d.Cout_store != d.Cout) return hipErrorInvalidValue;
  if (d.taps == 9) {
    if (d.src == 2) return y32 ? by_width<T, float, 9, 2>(s, d) : by_width<T, T, 9, 2>(s, d);
    if (d.src == 1 && y32) return by_width<T, float, 9, 1>(s, d);  // no activation (the decoder's conv after upsampling)
    if (d.src == 3 && y32) return by_width<T, float, 9, 3>(s, d);
    return hipErrorInvalidValue;
  }
  if (d.taps == 1) {
    if (d.src == 1 && !d.y_f32) return by_width<T, T, 1, 1>(s, d);      // qkv: GroupNorm'ed fp32 rows -> operand type
    if (d.src == 1) return by_width<T, float, 1, 1>(s, d);               // GroupNorm'ed fp32 rows -> fp32 stream (projection in)
    if (d.src == 0 && y32) return by_width<T, float, 1, 0>(s, d);        // proj: operand rows -> fp32 stream
    if (d.src == 0) return by_width<T, T, 1, 0>(s, d);                   // operand rows -> operand rows (transformer layers)
    return hipErrorInvalidValue;
  }
  return hipErrorInvalidValue;
}

hipError_t launch_fused(hipStream_t s, const FusedDesc& d) {
  if (d.yt && (d.taps != 1 || d.y_f32 || d.res || d.yt_from % 32 || d.yt_from <= 0 || d.yt_from >= d.Cout ||
               d.yt_Tp % 64 || d.yt_Tp < d.yt_T || d.out_map.rows_per_seg < d.rows))
    return hipErrorInvalidValue;
  if (d.taps == 1 && d.win_w) return hipErrorInvalidValue;  // the streaming linear kernel has no spatial window
  const int esz = (int)dtype_size(d.dt);
  if (d.q_cols && (d.taps != 1 || d.q_cols % 4 || d.q_cols > d.Cout || d.bias || d.res)) return hipErrorInvalidValue;
  if (d.stat && (d.taps != 9 || d.planar_out || !(d.y_f32 || esz == 4) || d.stat_splits != conv_stat_splits(d.H, d.W)))
    return hipErrorInvalidValue;
  if (d.Cin % (kRow / esz) != 0) return hipErrorInvalidValue;
  if (d.src == 3 && (d.Cs % (kRow / esz) != 0 || d.Cs <= 0 || d.Cs >= d.Cin || (d.H | d.W) & 1)) return hipErrorInvalidValue;
  if (d.taps == 9) {  // the kernel with specialised wavefronts where the stage's widths suit it
    const hipError_t e = launch_conv_ws(s, d);
    if (e != hipErrorNotSupported) return e;
  }
  if (d.taps == 1 && d.src == 0) {  // dense bf16 rows: the kernel with a ring of LDS stages
    const hipError_t e = launch_lin2(s, d);
    if (e != hipErrorNotSupported) return e;
  }
  if (d.y2 || d.act) return hipErrorInvalidValue;  // only that kernel writes the rounded copy / applies an activation
  return d.dt == kBF16 ? by_kind<bf16_t>(s, d) : by_kind<float>(s, d);
}

}  // namespace lc

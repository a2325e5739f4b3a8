// Implicit-GEMM 3x3 convolution and per-row linear layers on MFMA (gfx950), channels-last.
//
// The product is computed transposed, D[cout][pixel] = sum_k W[cout][k] * X[pixel][k], with
// k = tap * Cin + ci, so that one lane ends up holding 4 consecutive output channels of one
// pixel (a single 8- or 16-byte store into the channels-last output). One workgroup of 4
// wavefronts owns a tile of BCO output channels x 128 pixels (8 image rows x 16 columns for a
// convolution, 128 consecutive rows for a linear layer) and walks K in steps of 128 bytes per
// row: both operand tiles of a step are staged in LDS (row stride 144 bytes: consecutive rows
// start 16 bytes apart modulo 128, so 16-byte fragment reads of 8 consecutive rows hit disjoint
// banks), double buffered, with the next step's global loads in flight during the MFMAs.
// Out-of-image taps and ragged tiles are zero-filled at load time and masked at store time.
#include "lc_internal.h"

namespace lc {

struct ConvArgs {
  const void* x;
  const void* w;
  const float* bias;
  const void* res;
  void* y;
  int Cin, Cout_store, ldw;  // ldw = taps * Cin (row length of w)
  int frames, H, W, Ho, Wo, tiles_x, tiles_y;
  int64_t rows;
  RowMap out_map;
};

constexpr int kRowBytes = 128;  // K bytes per row per step
constexpr int kLdsRow = 144;    // LDS row stride in bytes

template <int BCO, int BPX>
constexpr int conv_lds_bytes() { return 2 * (BCO + BPX) * kLdsRow; }

// T: MFMA operand type (type of w and of the LDS tiles); XT: type of x in memory (T, or float that is
// rounded to T while staged); OT: type of y. A residual, when given, is always fp32.
template <class T, class XT, class OT, int TAPS, int STRIDE, int WCO, int WPX, int CO_T, int PX_T, bool PLANAR>
__global__ __launch_bounds__(256) void conv_kernel(ConvArgs a) {
  constexpr int VEC = Vec16<T>::N;
  constexpr int BKC = kRowBytes / (int)sizeof(T);  // K elements per step
  constexpr int BCO = WCO * CO_T * 16;
  constexpr int BPX = WPX * PX_T * 16;
  constexpr int XP = BPX / 32;         // x packets per thread per step
  constexpr int WP = (BCO + 31) / 32;  // w packets per thread per step
  static_assert(WCO * WPX == 4, "4 wavefronts");
  static_assert(BPX % 32 == 0, "pixel tile");
  typedef Mma16<T> M;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  auto w_lds = [&](int b) { return smem + b * (BCO + BPX) * kLdsRow; };
  auto x_lds = [&](int b) { return smem + b * (BCO + BPX) * kLdsRow + BCO * kLdsRow; };

  const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const int wco = wid / WPX, wpx = wid % WPX;
  const int co0 = blockIdx.y * BCO;
  const XT* __restrict__ X = (const XT*)a.x;
  const T* __restrict__ Wt = (const T*)a.w;

  // ---- which pixels this workgroup owns
  int frame = 0, ty0 = 0, tx0 = 0;
  int64_t row0 = 0;
  if (TAPS == 9) {
    int t = blockIdx.x;
    tx0 = (t % a.tiles_x) * 16;
    t /= a.tiles_x;
    ty0 = (t % a.tiles_y) * (BPX / 16);
    frame = t / a.tiles_y;
  } else {
    row0 = (int64_t)blockIdx.x * BPX;
  }

  // ---- loader bookkeeping: this thread moves packet kp of rows lrow + 32*i
  const int kp = tid & 7, lrow = tid >> 3;
  int ld_oy[XP], ld_ox[XP];
  bool ld_ok[XP];
#pragma unroll
  for (int i = 0; i < XP; ++i) {
    const int p = lrow + 32 * i;
    if (TAPS == 9) {
      ld_oy[i] = ty0 + p / 16;
      ld_ox[i] = tx0 + p % 16;
      ld_ok[i] = ld_oy[i] < a.Ho && ld_ox[i] < a.Wo;
    } else {
      ld_oy[i] = 0;
      ld_ox[i] = 0;
      ld_ok[i] = row0 + p < a.rows;
    }
  }
  Vec16<T> xv[XP], wv[WP];

  auto load_global = [&](int step) {
    const int slab = step / TAPS, tap = step - slab * TAPS;
    const int kofs = slab * BKC + kp * VEC;
#pragma unroll
    for (int i = 0; i < XP; ++i) {
      bool ok = ld_ok[i];
      int64_t off;
      if (TAPS == 9) {
        const int iy = ld_oy[i] * STRIDE + tap / 3 - 1, ix = ld_ox[i] * STRIDE + tap % 3 - 1;
        ok = ok && iy >= 0 && iy < a.H && ix >= 0 && ix < a.W;
        off = (((int64_t)frame * a.H + iy) * a.W + ix) * a.Cin + kofs;
      } else {
        off = (row0 + lrow + 32 * i) * a.Cin + kofs;
      }
      xv[i] = ok ? load_packet<XT, T>(X + off) : zero16<T>();
    }
#pragma unroll
    for (int i = 0; i < WP; ++i) {
      const int r = lrow + 32 * i;
      if (BCO % 32 == 0 || r < BCO)
        wv[i] = load16(Wt + (int64_t)(co0 + r) * a.ldw + tap * a.Cin + kofs);
    }
  };
  auto store_lds = [&](int buf) {
#pragma unroll
    for (int i = 0; i < XP; ++i)
      *reinterpret_cast<Vec16<T>*>(x_lds(buf) + (lrow + 32 * i) * kLdsRow + kp * 16) = xv[i];
#pragma unroll
    for (int i = 0; i < WP; ++i) {
      const int r = lrow + 32 * i;
      if (BCO % 32 == 0 || r < BCO) *reinterpret_cast<Vec16<T>*>(w_lds(buf) + r * kLdsRow + kp * 16) = wv[i];
    }
  };

  f32x4 acc[CO_T][PX_T];
#pragma unroll
  for (int i = 0; i < CO_T; ++i)
#pragma unroll
    for (int j = 0; j < PX_T; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int fr = lane & 15, fg = lane >> 4;
  const int nsteps = TAPS * (a.Cin / BKC);
  load_global(0);
  store_lds(0);
  __syncthreads();
  for (int s = 0; s < nsteps; ++s) {
    const int buf = s & 1;
    if (s + 1 < nsteps) load_global(s + 1);
    const unsigned char* wl = w_lds(buf) + (wco * CO_T * 16 + fr) * kLdsRow;
    const unsigned char* xl = x_lds(buf) + (wpx * PX_T * 16 + fr) * kLdsRow;
#pragma unroll
    for (int kk = 0; kk < kRowBytes / 64; ++kk) {
      typename M::Frag fa[CO_T], fb[PX_T];
#pragma unroll
      for (int i = 0; i < CO_T; ++i) fa[i] = M::load((const T*)(wl + i * 16 * kLdsRow + kk * 64), fg);
#pragma unroll
      for (int j = 0; j < PX_T; ++j) fb[j] = M::load((const T*)(xl + j * 16 * kLdsRow + kk * 64), fg);
#pragma unroll
      for (int i = 0; i < CO_T; ++i)
#pragma unroll
        for (int j = 0; j < PX_T; ++j) M::mma(fa[i], fb[j], acc[i][j]);
    }
    if (s + 1 < nsteps) store_lds(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: lane holds channels co + 0..3 of pixel (tile j, column fr)
  OT* Y = (OT*)a.y;
  const float* R = (const float*)a.res;  // may alias Y (in-place residual)
#pragma unroll
  for (int j = 0; j < PX_T; ++j) {
    const int p = wpx * PX_T * 16 + j * 16 + fr;
    int64_t orow;
    int oy = 0, ox = 0;
    bool ok;
    if (TAPS == 9) {
      oy = ty0 + p / 16;
      ox = tx0 + p % 16;
      ok = oy < a.Ho && ox < a.Wo;
      orow = ((int64_t)frame * a.Ho + oy) * a.Wo + ox;
    } else {
      ok = row0 + p < a.rows;
      orow = ok ? a.out_map(row0 + p) : 0;
    }
    if (!ok) continue;
#pragma unroll
    for (int i = 0; i < CO_T; ++i) {
      const int co = co0 + wco * CO_T * 16 + i * 16 + 4 * fg;
      if (PLANAR) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          if (co + r < a.Cout_store) {
            float v = acc[i][j][r] + (a.bias ? a.bias[co + r] : 0.f);
            Y[(((int64_t)frame * a.Cout_store + co + r) * a.Ho + oy) * a.Wo + ox] = from_f32<OT>(v);
          }
        }
      } else {
        if (co >= a.Cout_store) continue;
        float v[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = acc[i][j][r] + (a.bias ? a.bias[co + r] : 0.f);
        const int64_t o = orow * a.Cout_store + co;
        if (R) {
          f32x4 rv = *reinterpret_cast<const f32x4*>(R + o);
#pragma unroll
          for (int r = 0; r < 4; ++r) v[r] += rv[r];
        }
        if constexpr (sizeof(OT) == 2) {
          bf16x4 ov;
#pragma unroll
          for (int r = 0; r < 4; ++r) ov[r] = static_cast<bf16_t>(v[r]);
          *reinterpret_cast<bf16x4*>((bf16_t*)Y + o) = ov;
        } else {
          *reinterpret_cast<f32x4*>((float*)Y + o) = f32x4{v[0], v[1], v[2], v[3]};
        }
      }
    }
  }
}

template <class T, class XT, class OT, int TAPS, int STRIDE, int WCO, int WPX, int CO_T, int PX_T, bool PLANAR>
static hipError_t run(hipStream_t s, const ConvDesc& d) {
  constexpr int BCO = WCO * CO_T * 16, BPX = WPX * PX_T * 16;
  constexpr int lds = conv_lds_bytes<BCO, BPX>();
  auto kern = conv_kernel<T, XT, OT, TAPS, STRIDE, WCO, WPX, CO_T, PX_T, PLANAR>;
  static bool attr_done = false;  // per instantiation
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  ConvArgs a;
  a.x = d.x; a.w = d.w; a.bias = d.bias; a.res = d.res; a.y = d.y;
  a.Cin = d.Cin; a.Cout_store = d.Cout_store; a.ldw = d.taps * d.Cin;
  a.frames = d.frames; a.H = d.H; a.W = d.W;
  a.Ho = d.H / d.stride; a.Wo = d.W / d.stride;
  a.tiles_x = (a.Wo + 15) / 16; a.tiles_y = (a.Ho + BPX / 16 - 1) / (BPX / 16);
  a.rows = d.rows; a.out_map = d.out_map;
  dim3 grid;
  if (TAPS == 9) {
    if (d.frames <= 0) return hipSuccess;
    grid = dim3((unsigned)(a.tiles_x * a.tiles_y * d.frames), d.Cout / BCO);
  } else {
    if (d.rows <= 0) return hipSuccess;
    grid = dim3((unsigned)((d.rows + BPX - 1) / BPX), d.Cout / BCO);
  }
  kern<<<grid, 256, lds, s>>>(a);
  return hipGetLastError();
}

template <class T, class XT, class OT>
static hipError_t dispatch_shape(hipStream_t s, const ConvDesc& d) {
  const bool wide = d.Cout % 160 == 0;
  if (!wide && d.Cout % 64 != 0) return hipErrorInvalidValue;
  if (d.taps == 9 && d.stride == 1)
    return wide ? run<T, XT, OT, 9, 1, 2, 2, 5, 4, false>(s, d) : run<T, XT, OT, 9, 1, 2, 2, 2, 4, false>(s, d);
  if (d.taps == 9 && d.stride == 2)
    return wide ? run<T, XT, OT, 9, 2, 2, 2, 5, 4, false>(s, d) : run<T, XT, OT, 9, 2, 2, 2, 2, 4, false>(s, d);
  if (d.taps == 1)
    return wide ? run<T, XT, OT, 1, 1, 2, 2, 5, 4, false>(s, d) : run<T, XT, OT, 1, 1, 2, 2, 2, 4, false>(s, d);
  return hipErrorInvalidValue;
}

hipError_t launch_conv(hipStream_t s, const ConvDesc& d) {
  if (d.taps == 9 && (d.H % d.stride || d.W % d.stride)) return hipErrorInvalidValue;
  const int esz = (int)dtype_size(d.dt);
  if (d.Cin % (kRowBytes / esz) != 0) return hipErrorInvalidValue;
  if (d.planar_out) {
    if (d.taps != 9 || d.stride != 1 || d.Cout != 16 || d.res || d.x_f32 || d.y_f32) return hipErrorInvalidValue;
    return d.dt == kBF16 ? run<bf16_t, bf16_t, bf16_t, 9, 1, 1, 4, 1, 2, true>(s, d)
                         : run<float, float, float, 9, 1, 1, 4, 1, 2, true>(s, d);
  }
  if (d.Cout_store != d.Cout || d.Cout % 4) return hipErrorInvalidValue;
  if (d.dt == kF32) return dispatch_shape<float, float, float>(s, d);
  if (d.x_f32) {
    if (!d.y_f32 || d.taps != 9 || d.stride != 2) return hipErrorInvalidValue;  // only the down conv reads fp32
    return d.Cout % 160 == 0 ? run<bf16_t, float, float, 9, 2, 2, 2, 5, 4, false>(s, d)
                             : run<bf16_t, float, float, 9, 2, 2, 2, 2, 4, false>(s, d);
  }
  if (d.taps == 9 && d.stride == 2) return hipErrorInvalidValue;
  return d.y_f32 ? dispatch_shape<bf16_t, bf16_t, float>(s, d) : dispatch_shape<bf16_t, bf16_t, bf16_t>(s, d);
}

// ---------------------------------------------------------------------------------------------
// Last convolution of the stage: eps = conv3x3_{C -> C_lat}(SiLU(GN(u))) + bias, C_lat <= 16 output
// channels, planar output. One pass over u bounds it (C * 4 bytes read per pixel against
// 2 * 9 * C * C_lat FLOP): what costs time is the activation (two transcendentals per element) and
// getting every compute unit to pull its share of u early. So:
//   - a workgroup owns a 4 x 16 pixel tile of one frame (256 tiles for four 64 x 64 frames) and all C
//     channels of its 6 x 18 halo: every thread requests all its 32-byte pieces of the halo at once,
//     then normalises, activates and rounds them as they land and parks them in LDS, pixel-major;
//   - the contraction over K = 9 * C runs on 16 x 16 x 32 MFMAs with the (zero padded) output channels
//     as rows and 16 pixels of an image row as columns; the wavefronts split K (the weights of a
//     wavefront's share sit in its registers as A fragments, fetched while the halo is on its way),
//     each covers the four image rows of the tile;
//   - the wavefronts' partial sums meet in LDS and are added in a fixed order.
// NT threads: with 512 two wavefronts share a SIMD, and one's transcendentals overlap the other's loads.
template <int C, int NT>
__global__ __launch_bounds__(NT) void conv_out_tile_kernel(const float* __restrict__ u, const float* __restrict__ scale,
                                                           const float* __restrict__ shift, const bf16_t* __restrict__ w,
                                                           const float* __restrict__ bias, bf16_t* __restrict__ out, int H,
                                                           int W, int C_lat, int wx0, int wy0) {
  typedef Mma16<bf16_t> M;
  constexpr int XS = C * 2 + 16;                 // LDS bytes per halo pixel (padded: 16 pixels hit 64 banks)
  constexpr int HW_ = 18, HP = 6 * HW_;          // halo width, halo pixels
  constexpr int PPR = C / 8;                     // 16-byte bf16 packets per pixel
  constexpr int GRP = NT / PPR;                  // pixels staged per round
  constexpr int RND = (HP + GRP - 1) / GRP;      // rounds
  constexpr int CB = C / 32;                     // k-steps per tap
  constexpr int NKS = 9 * CB;                    // k-steps
  constexpr int NW = NT / 64;                    // wavefronts
  constexpr int KSW = (NKS + NW - 1) / NW;       // k-steps per wavefront
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* const red = reinterpret_cast<float*>(smem + HP * XS);  // [wave][row 4][channel 16][x 16]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int x0 = wx0 + blockIdx.x * 16, y0 = wy0 + blockIdx.y * 4, frame = blockIdx.z;  // (wx0, wy0): origin of the window

  // ---- staging: thread = (packet column, pixel group); its halo pixels are grp, grp + GRP, ...
  const int col = tid % PPR, grp = tid / PPR;
  const int c0 = col * 8;
  f32x4 raw[RND][2];
  const float* uf = u + (int64_t)frame * H * W * C + c0;
#pragma unroll
  for (int j = 0; j < RND; ++j) {
    const int hp = min(grp + GRP * j, HP - 1);
    const int iy = min(max(y0 + hp / HW_ - 1, 0), H - 1), ix = min(max(x0 + hp % HW_ - 1, 0), W - 1);  // clamped: valid
    const float* px = uf + ((int64_t)iy * W + ix) * C;
    raw[j][0] = *reinterpret_cast<const f32x4*>(px);
    raw[j][1] = *reinterpret_cast<const f32x4*>(px + 4);
  }
  float sc[8], sh[8];
  load_f<float, 8>(scale + (int64_t)frame * C + c0, sc);
  load_f<float, 8>(shift + (int64_t)frame * C + c0, sh);
  // ---- this wavefront's weights: k-step ks = wid + NW j is (tap ks / CB, channels 32 (ks % CB) ..)
  typename M::Frag af[KSW];
  {
    const int co = lane & 15, g = lane >> 4;
#pragma unroll
    for (int j = 0; j < KSW; ++j) {
      const int ks = min(wid + NW * j, NKS - 1);  // beyond the end: a repeat, never used
      af[j] = M::load(w + ((int64_t)co * 9 + ks / CB) * C + (ks % CB) * 32, g);
    }
  }
#pragma unroll
  for (int j = 0; j < RND; ++j) {
    const int hp = grp + GRP * j;
    const int iy = y0 + hp / HW_ - 1, ix = x0 + hp % HW_ - 1;
    const bool inside = iy >= 0 && iy < H && ix >= 0 && ix < W;  // the padding is zero after the activation
    Vec16<bf16_t> o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o.set(e, inside ? silu_fast(fmaf(raw[j][e >> 2][e & 3], sc[e], sh[e])) : 0.f);
    if (grp < GRP && hp < HP) *reinterpret_cast<Vec16<bf16_t>*>(smem + hp * XS + col * 16) = o;
  }
  __syncthreads();

  // ---- contraction: D[channel][pixel x] for the four image rows of the tile
  f32x4 acc[4];
#pragma unroll
  for (int n = 0; n < 4; ++n) acc[n] = f32x4{0.f, 0.f, 0.f, 0.f};
  const unsigned char* bl = smem + (lane & 15) * XS + (lane >> 4) * 16;
#pragma unroll
  for (int j = 0; j < KSW; ++j) {
    const int ks = wid + NW * j;
    if (ks < NKS) {  // uniform over the wavefront
      const int tap = ks / CB, cb = ks - tap * CB;
      const int dy = tap / 3, dx = tap - dy * 3;
      const unsigned char* b0 = bl + (dy * HW_ + dx) * XS + cb * 64;
#pragma unroll
      for (int n = 0; n < 4; ++n) {
        const typename M::Frag bf = *reinterpret_cast<const typename M::Frag*>(b0 + n * HW_ * XS);
        M::mma(af[j], bf, acc[n]);
      }
    }
  }
  // lane holds channels 4 (lane / 16) + r of pixel x = lane % 16
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int r = 0; r < 4; ++r) red[((wid * 4 + n) * 16 + 4 * (lane >> 4) + r) * 16 + (lane & 15)] = acc[n][r];
  __syncthreads();
  for (int i = tid; i < 4 * C_lat * 16; i += NT) {
    const int x = i & 15, co = (i >> 4) % C_lat, n = i / (16 * C_lat);
    float v = red[(n * 16 + co) * 16 + x];
#pragma unroll
    for (int q = 1; q < NW; ++q) v += red[((q * 4 + n) * 16 + co) * 16 + x];  // fixed order
    v += bias[co];
    out[(((int64_t)frame * C_lat + co) * H + y0 + n) * W + x0 + x] = static_cast<bf16_t>(v);
  }
}

// ---------------------------------------------------------------------------------------------
// First convolution of the stage for bf16: h = conv3x3_{C_lat -> C}(x) + bias, planar latents in, fp32 rows out,
// with the per-channel sums of every 32 output rows for the GroupNorm that follows. The contraction is only
// K = 9 * C_lat (36) long: what costs time is writing C * 4 bytes per pixel, so the kernel is built around many
// small workgroups that overlap each other's phases. A workgroup owns 32 consecutive pixels of an image row
// (one statistics split) and all C channels: its 3 x 34 halo of the C_lat planes goes to LDS; the product is
// D[pixel][channel] on 32 x 32 x 16 MFMAs, the A operand (k = channel * 9 + tap, zeros beyond 9 * C_lat)
// gathered from the halo two bytes at a time, the B operand read straight from the weights padded to rows
// of 64; in D a lane holds one channel of 16 pixels, so 32 lanes store 128 contiguous bytes of a pixel's
// row and the sums over the pixels are 16 additions in the lane and one across its two halves. The four
// wavefronts split the 32-channel tiles (w, w + 4, w + 8, ...).
template <int KS, int NTM>
__global__ __launch_bounds__(256) void conv_in_tile_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ wp,
                                                           const float* __restrict__ bias, float* __restrict__ y,
                                                           float* __restrict__ stat, int H, int W, int Cl, int C, int wx0,
                                                           int wy0, int wsegs) {
  __shared__ bf16_t halo[8][3][40];  // [plane][row][34 used]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);
  // the window's rows and 32-pixel segments (wx0, wy0: its origin; wsegs: segments per row)
  const int wr = blockIdx.x / wsegs;
  const int yy = wy0 + wr, x0 = wx0 + (blockIdx.x - wr * wsegs) * 32, frame = blockIdx.y;
  const bf16_t* img = x + (int64_t)frame * Cl * H * W;
  for (int i = tid; i < Cl * 3 * 34; i += 256) {
    const int xx = i % 34, dy = (i / 34) % 3, cl = i / (3 * 34);
    const int iy = yy + dy - 1, ix = x0 + xx - 1;
    const bool ok = iy >= 0 && iy < H && ix >= 0 && ix < W;
    const bf16_t v = img[((int64_t)cl * H + min(max(iy, 0), H - 1)) * W + min(max(ix, 0), W - 1)];  // clamped: valid
    halo[cl][dy][xx] = ok ? v : (bf16_t)0.f;
  }
  const int l32 = lane & 31, hh = lane >> 5;
  const int tiles = C / 32;
  // this wavefront's weights (tile slots beyond its share: the last tile again, never used)
  bf16x8 bw[NTM][KS];
#pragma unroll
  for (int i = 0; i < NTM; ++i) {
    const int t = min(wid + 4 * i, tiles - 1);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) bw[i][ks] = *reinterpret_cast<const bf16x8*>(wp + (int64_t)(t * 32 + l32) * 64 + 16 * ks + 8 * hh);
  }
  __syncthreads();
  bf16x8 af[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int k = 16 * ks + 8 * hh + j;
      const int cl = k / 9, tap = k - cl * 9;
      const int dy = tap / 3, dx = tap - dy * 3;
      af[ks][j] = k < 9 * Cl ? halo[cl][dy][l32 + dx] : (bf16_t)0.f;  // (cl < Cl <= 8 whenever it is read)
    }
  const int split = (yy * W + x0) >> 5, splits = (H * W) >> 5;
  float* yrow = y + ((int64_t)frame * H * W + (int64_t)yy * W + x0) * C;
#pragma unroll
  for (int i = 0; i < NTM; ++i) {
    const int t = wid + 4 * i;
    if (t < tiles) {  // uniform over the wavefront
      f32x16 acc;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks], bw[i][ks], acc, 0, 0, 0);
      const int ch = t * 32 + l32;
      const float bv = bias[ch];
      float s1 = 0.f, s2 = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float v = acc[r] + bv;
        const int px = 8 * (r >> 2) + 4 * hh + (r & 3);
        yrow[(int64_t)px * C + ch] = v;
        s1 += v;
        s2 = fmaf(v, v, s2);
      }
      s1 += __shfl_xor(s1, 32, 64);
      s2 += __shfl_xor(s2, 32, 64);
      if (stat && hh == 0) {
        float* sp = stat + (((int64_t)frame * splits + split) * C + ch) * 2;
        sp[0] = s1;
        sp[1] = s2;
      }
    }
  }
}

// Returns hipErrorNotSupported for shapes it does not cover. wp: the weights as rows [C][64] of the operand type,
// k = plane * 9 + tap, zeros beyond 9 * C_lat. stat: [frame][H * W / 32][C][2] or nullptr.
hipError_t launch_conv_in_tile(hipStream_t s, int dt, const void* x, const void* wp, const float* bias, float* y, float* stat,
                               int frames, int H, int W, int Cl, int C, Win win) {
  if (dt != kBF16 || !wp || W % 32 || C % 32 || Cl < 1 || 9 * Cl > 48 || C / 32 > 12) return hipErrorNotSupported;
  if (frames <= 0) return hipSuccess;
  if (win.w == 0) win = Win{0, 0, W, H};
  if (win.x0 < 0 || win.y0 < 0 || win.w <= 0 || win.h <= 0 || win.x0 + win.w > W || win.y0 + win.h > H || win.x0 % 32 || win.w % 32)
    return hipErrorInvalidValue;
  dim3 grid((unsigned)(win.h * (win.w / 32)), (unsigned)frames);
  conv_in_tile_kernel<3, 3><<<grid, 256, 0, s>>>((const bf16_t*)x, (const bf16_t*)wp, bias, y, stat, H, W, Cl, C, win.x0, win.y0,
                                                 win.w / 32);
  return hipGetLastError();
}

// Returns hipErrorNotSupported for shapes it does not cover (the caller then uses the general kernel).
hipError_t launch_conv_out_tile(hipStream_t s, int dt, const void* u, const float* scale, const float* shift, const void* w,
                                const float* bias, void* out, int frames, int H, int W, int C, int C_lat, Win win) {
  if (dt != kBF16 || C != 320 || W % 16 || H % 4 || C_lat < 1 || C_lat > 16) return hipErrorNotSupported;
  if (frames <= 0) return hipSuccess;
  if (win.w == 0) win = Win{0, 0, W, H};
  if (win.x0 < 0 || win.y0 < 0 || win.w <= 0 || win.h <= 0 || win.x0 + win.w > W || win.y0 + win.h > H || win.x0 % 16 ||
      win.w % 16 || win.y0 % 4 || win.h % 4)
    return hipErrorInvalidValue;
  constexpr int NT = 512;
  const int lds = (6 * 18) * (320 * 2 + 16) + (NT / 64) * 4 * 16 * 16 * 4;
  auto kern = conv_out_tile_kernel<320, NT>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  dim3 grid((unsigned)(win.w / 16), (unsigned)(win.h / 4), (unsigned)frames);
  kern<<<grid, NT, lds, s>>>((const float*)u, scale, shift, (const bf16_t*)w, bias, (bf16_t*)out, H, W, C_lat, win.x0, win.y0);
  return hipGetLastError();
}

}  // namespace lc

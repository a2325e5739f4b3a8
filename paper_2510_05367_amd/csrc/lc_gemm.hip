// Fused-loader implicit-GEMM kernels on 32x32 MFMA tiles (gfx950): the 3x3 stride-1 convolutions
// and the per-row linear layers of the stage.
//
// Product (transposed): D[cout][pixel] = sum_k W[cout][k] X[pixel][k], k = tap * Cin + ci.
// One workgroup = 4 wavefronts = BCO output channels x 128 pixels; every wavefront owns all BCO
// channels of 32 pixels (CO_T accumulator tiles of 32x32), so the weight fragments it reads from
// LDS are used once per 32-pixel fragment and the pixel fragment once per CO_T weight fragments.
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
// A convolution stages, per 64-byte.. 128-byte channel slab, the 10 x 18 halo of its 8 x 16 pixel
// tile once and walks the 9 taps over it by shifting LDS addresses; the weights of a (slab, tap)
// step are streamed through a second LDS tile. Weight loads are issued two steps ahead, the next
// slab's halo is fetched and activated one 16-byte packet per thread per tap while the MFMAs of
// the current slab run.
#include "lc_internal.h"

namespace lc {

namespace {

constexpr int kRow = 128;     // K bytes per LDS row per step
constexpr int kLds = 144;     // LDS row stride (bytes): 16-byte reads of 16 consecutive rows hit 64 distinct banks
constexpr int kHaloW = 18, kHaloH = 10, kHalo = kHaloW * kHaloH;

struct GemmArgs {
  const void* x;        // PLAIN: T [rows][Cin]; NORM: float [..][Cin]; CAT: float skip [..][Cs]
  const void* x2;       // CAT: deep, T [frames][H/2][W/2][Cin - Cs]
  const float* scale;   // [frames][Cin]
  const float* shift;
  const void* w;        // T [Cout][taps * Cin]
  const float* bias;
  const float* res;     // fp32, indexed like y (may alias y)
  void* y;
  int Cin, Cs, Cout_store, ldw;
  int frames, H, W, tiles_x, tiles_y;
  int64_t rows;
  RowMap in_map, out_map;
};

template <int BCO, int XROWS>
constexpr int gemm_lds_bytes() { return 2 * (BCO + XROWS) * kLds; }

}  // namespace

// SRC: 0 plain operand-type rows, 1 fp32 rows with scale/shift, 2 the same + SiLU, 3 concat (+ SiLU)
template <class T, class OT, int TAPS, int CO_T, int SRC, bool PLANAR>
__global__ __launch_bounds__(256) void gemm_kernel(GemmArgs a) {
  typedef Mma32<T> M;
  constexpr int VEC = Vec16<T>::N;               // operand elements per 16-byte LDS packet
  constexpr int BKC = kRow / (int)sizeof(T);     // K elements per step
  constexpr int BCO = CO_T * 32;
  constexpr int XROWS = TAPS == 9 ? kHalo : 128;
  constexpr int WP = (BCO * 8 + 255) / 256;      // weight packets per thread per step
  constexpr int XR = TAPS == 9 ? (kHalo * 8 + 255) / 256 : 4;  // x packets per thread per slab
  constexpr int KI = kRow / (M::K * (int)sizeof(T));           // MFMA k-steps per LDS row
  constexpr bool NORM = SRC != 0;
  constexpr bool SILU = SRC >= 2;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  auto w_lds = [&](int b) { return smem + b * (BCO + XROWS) * kLds; };
  auto x_lds = [&](int b) { return smem + b * (BCO + XROWS) * kLds + BCO * kLds; };

  const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const int lp = lane & 31, hh = lane >> 5;
  const int co0 = blockIdx.y * BCO;
  const T* __restrict__ Wt = (const T*)a.w;

  int frame = 0, ty0 = 0, tx0 = 0;
  int64_t row0 = 0;
  if (TAPS == 9) {
    int t = blockIdx.x;
    tx0 = (t % a.tiles_x) * 16;
    t /= a.tiles_x;
    ty0 = (t % a.tiles_y) * 8;
    frame = t / a.tiles_y;
  } else {
    row0 = (int64_t)blockIdx.x * 128;
  }
  const int kp = tid & 7, lrow = tid >> 3;  // this thread moves packet kp of rows lrow + 32 * i

  // ---------------- weights: registers two steps ahead of the MFMAs ----------------
  Vec16<T> wreg[2][WP];
  auto issue_w = [&](int step, Vec16<T> (&dst)[WP]) {
    const int slab = step / TAPS, tap = step - slab * TAPS;
    const int kofs = tap * a.Cin + slab * BKC + kp * VEC;
#pragma unroll
    for (int i = 0; i < WP; ++i) {
      const int r = lrow + 32 * i;
      if (BCO % 32 == 0 || r < BCO) dst[i] = load16(Wt + (int64_t)(co0 + r) * a.ldw + kofs);
    }
  };
  auto store_w = [&](int buf, const Vec16<T> (&src)[WP]) {
#pragma unroll
    for (int i = 0; i < WP; ++i) {
      const int r = lrow + 32 * i;
      if (BCO % 32 == 0 || r < BCO) *reinterpret_cast<Vec16<T>*>(w_lds(buf) + r * kLds + kp * 16) = src[i];
    }
  };

  // ---------------- x packets: fetch raw, then activate + round + store ----------------
  struct XRaw { float v[VEC]; bool ok; };
  struct Affine { float sc[VEC], sh[VEC]; };
  // conv: packet round r of slab -> halo pixel (tid + 256 r) / 8; linear: row lrow + 32 r of the tile
  auto fetch_x = [&](int slab, int r, XRaw& o) {
    const int c0 = slab * BKC + kp * VEC;
    o.ok = false;
    if (TAPS == 9) {
      const int q = tid + 256 * r;
      const int hp = q >> 3;
      if (hp >= kHalo) return;
      const int hy = hp / kHaloW, hx = hp - hy * kHaloW;
      const int iy = ty0 + hy - 1, ix = tx0 + hx - 1;
      if (iy < 0 || iy >= a.H || ix < 0 || ix >= a.W) return;
      o.ok = true;
      if (SRC == 3 && c0 >= a.Cs) {
        const int64_t dr = ((int64_t)frame * (a.H >> 1) + (iy >> 1)) * (a.W >> 1) + (ix >> 1);
        load_f<T, VEC>((const T*)a.x2 + dr * (a.Cin - a.Cs) + (c0 - a.Cs), o.v);
      } else if (NORM) {
        const int ldx = SRC == 3 ? a.Cs : a.Cin;
        load_f<float, VEC>((const float*)a.x + (((int64_t)frame * a.H + iy) * a.W + ix) * ldx + c0, o.v);
      } else {
        load_f<T, VEC>((const T*)a.x + (((int64_t)frame * a.H + iy) * a.W + ix) * a.Cin + c0, o.v);
      }
    } else {
      const int64_t rr = row0 + lrow + 32 * r;
      if (rr >= a.rows) return;
      o.ok = true;
      const int64_t sr = a.in_map(rr);
      if (NORM) load_f<float, VEC>((const float*)a.x + sr * a.Cin + c0, o.v);
      else load_f<T, VEC>((const T*)a.x + sr * a.Cin + c0, o.v);
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
    return (rr < a.rows ? rr : 0) / a.in_map.rows_per_seg;
  };
  auto finish_x = [&](int buf, int r, const XRaw& o, const Affine& af) {
    int lr;
    if (TAPS == 9) {
      lr = (tid + 256 * r) >> 3;
      if (lr >= kHalo) return;
    } else {
      lr = lrow + 32 * r;
    }
    Vec16<T> pk;
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      float t = o.v[e];
      if (NORM) {
        t = fmaf(t, af.sc[e], af.sh[e]);
        if (SILU) t = silu_f(t);
      }
      pk.set(e, o.ok ? t : 0.f);
    }
    *reinterpret_cast<Vec16<T>*>(x_lds(buf) + lr * kLds + kp * 16) = pk;
  };

  f32x16 acc[CO_T];
#pragma unroll
  for (int i = 0; i < CO_T; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

  // pixel of this lane inside the tile and its LDS row for tap (0,0)
  const int p = wid * 32 + lp;
  const int xrow0 = TAPS == 9 ? (p >> 4) * kHaloW + (p & 15) : p;

  auto compute = [&](int wbuf, int xbuf, int tap) {
    const int xrow = TAPS == 9 ? xrow0 + (tap / 3) * kHaloW + (tap % 3) : xrow0;
    const unsigned char* xl = x_lds(xbuf) + xrow * kLds + hh * (M::LK * (int)sizeof(T));
    const unsigned char* wl = w_lds(wbuf) + lp * kLds + hh * (M::LK * (int)sizeof(T));
#pragma unroll
    for (int kk = 0; kk < KI; ++kk) {
      const typename M::Frag xf = M::load((const T*)(xl + kk * M::K * (int)sizeof(T)));
#pragma unroll
      for (int i = 0; i < CO_T; ++i) {
        const typename M::Frag wf = M::load((const T*)(wl + i * 32 * kLds + kk * M::K * (int)sizeof(T)));
        M::mma(wf, xf, acc[i]);
      }
    }
  };

  const int nslab = a.Cin / BKC;
  const int nsteps = TAPS * nslab;

  // ---------------- prologue ----------------
  issue_w(0, wreg[0]);
  if (nsteps > 1) issue_w(1, wreg[1]);
  Affine aff[TAPS == 9 ? 1 : XR];
  XRaw xin[TAPS == 9 ? 1 : XR];
  if (TAPS == 9) {
    load_affine(0, frame, aff[0]);
#pragma unroll
    for (int r = 0; r < XR; ++r) {
      fetch_x(0, r, xin[0]);
      finish_x(0, r, xin[0], aff[0]);
    }
  } else {
#pragma unroll
    for (int r = 0; r < XR; ++r) {
      fetch_x(0, r, xin[r]);
      load_affine(0, row_frame(r), aff[r]);
    }
#pragma unroll
    for (int r = 0; r < XR; ++r) finish_x(0, r, xin[r], aff[r]);
  }
  store_w(0, wreg[0]);
  __syncthreads();

  // ---------------- main loop, unrolled by two so that the register sets are static ----------------
  auto step = [&](int s, Vec16<T> (&w_free)[WP], Vec16<T> (&w_next)[WP]) {
    const int slab = s / TAPS, tap = s - slab * TAPS;
    if (s + 2 < nsteps) issue_w(s + 2, w_free);
    if (TAPS == 9) {
      // next slab's halo, one packet round per tap: finish round tap-1, fetch round tap
      if (slab + 1 < nslab) {
        if (tap >= 1 && tap <= XR) finish_x((slab + 1) & 1, tap - 1, xin[0], aff[0]);
        if (tap == 0) load_affine(slab + 1, frame, aff[0]);
        if (tap < XR) fetch_x(slab + 1, tap, xin[0]);
      }
      compute(s & 1, slab & 1, tap);
    } else {
      if (s + 1 < nsteps) {
#pragma unroll
        for (int r = 0; r < XR; ++r) {
          fetch_x(s + 1, r, xin[r]);
          load_affine(s + 1, row_frame(r), aff[r]);
        }
      }
      compute(s & 1, s & 1, 0);
      if (s + 1 < nsteps) {
#pragma unroll
        for (int r = 0; r < XR; ++r) finish_x((s + 1) & 1, r, xin[r], aff[r]);
      }
    }
    if (s + 1 < nsteps) store_w((s + 1) & 1, w_next);
    __syncthreads();
  };
  for (int s = 0; s < nsteps; s += 2) {
    step(s, wreg[0], wreg[1]);
    if (s + 1 < nsteps) step(s + 1, wreg[1], wreg[0]);
  }

  // ---------------- epilogue: lane holds, for pixel p, channels co0 + 32 i + 8 g + 4 hh + {0..3} ----------------
  OT* Y = (OT*)a.y;
  const float* R = a.res;  // may alias Y (in-place residual)
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
  if (!ok) return;
#pragma unroll
  for (int i = 0; i < CO_T; ++i) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int co = co0 + i * 32 + g * 8 + hh * 4;
      if (PLANAR) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (co + e < a.Cout_store) {
            const float v = acc[i][g * 4 + e] + (a.bias ? a.bias[co + e] : 0.f);
            Y[(((int64_t)frame * a.Cout_store + co + e) * a.H + oy) * a.W + ox] = from_f32<OT>(v);
          }
        }
      } else {
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[i][g * 4 + e] + (a.bias ? a.bias[co + e] : 0.f);
        const int64_t o = orow * a.Cout_store + co;
        if (R) {
          const f32x4 rv = *reinterpret_cast<const f32x4*>(R + o);
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] += rv[e];
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

template <class T, class OT, int TAPS, int CO_T, int SRC, bool PLANAR>
static hipError_t run_gemm(hipStream_t s, const FusedDesc& d) {
  constexpr int BCO = CO_T * 32;
  constexpr int XROWS = TAPS == 9 ? kHalo : 128;
  constexpr int lds = gemm_lds_bytes<BCO, XROWS>();
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
  a.Cin = d.Cin; a.Cs = d.Cs; a.Cout_store = d.Cout_store; a.ldw = d.taps * d.Cin;
  a.frames = d.frames; a.H = d.H; a.W = d.W;
  a.tiles_x = (d.W + 15) / 16; a.tiles_y = (d.H + 7) / 8;
  a.rows = d.rows; a.in_map = d.in_map; a.out_map = d.out_map;
  dim3 grid;
  if (TAPS == 9) {
    if (d.frames <= 0) return hipSuccess;
    grid = dim3((unsigned)(a.tiles_x * a.tiles_y * d.frames), d.Cout / BCO);
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
    if (d.src == 3 && y32) return by_width<T, float, 9, 3>(s, d);
    return hipErrorInvalidValue;
  }
  if (d.taps == 1) {
    if (d.src == 1 && !d.y_f32) return by_width<T, T, 1, 1>(s, d);      // qkv: GroupNorm'ed fp32 rows -> operand type
    if (d.src == 0 && y32) return by_width<T, float, 1, 0>(s, d);        // proj: operand rows -> fp32 stream
    return hipErrorInvalidValue;
  }
  return hipErrorInvalidValue;
}

hipError_t launch_fused(hipStream_t s, const FusedDesc& d) {
  const int esz = (int)dtype_size(d.dt);
  if (d.Cin % (kRow / esz) != 0) return hipErrorInvalidValue;
  if (d.src == 3 && (d.Cs % (kRow / esz) != 0 || d.Cs <= 0 || d.Cs >= d.Cin || (d.H | d.W) & 1)) return hipErrorInvalidValue;
  return d.dt == kBF16 ? by_kind<bf16_t>(s, d) : by_kind<float>(s, d);
}

}  // namespace lc

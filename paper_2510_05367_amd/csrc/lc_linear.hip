// Per-row linear layers (q,k,v and output projections of the attention blocks) on 32x32 MFMA tiles,
// weights stationary.
//
// K is only C here (320), so the weights a wavefront needs - up to 96 output channels x Cin - fit
// in its registers as MFMA fragments (3 x Cin/16 packets of 16 bytes for bf16; one wavefront per
// SIMD, so it may use the whole register file). A workgroup of four wavefronts covers a column of
// up to 12 32-channel tiles, split 3,3,2,2 for the 10 tiles of 320 channels, and walks a range of
// 32-row activation tiles: the tile is fetched one step ahead with coalesced 16/32-byte loads,
// GroupNorm'ed on the way in when the source is the fp32 residual stream, rounded to the operand
// type and parked in a double-buffered LDS tile that all wavefronts read. LDS traffic is one
// fragment per two or three MFMAs.
//
// Epilogue: the accumulator layout (a lane owns one row and 4-channel pieces of it) would store
// 8..16-byte pieces scattered over 32 rows; instead the wavefront turns each 32 x 32 tile through a
// private LDS patch and stores 16 bytes per lane with 64..128 contiguous bytes per row, adding the
// bias and the fp32 residual (prefetched in the same layout before the MFMAs). The value third of
// the spatial q,k,v goes straight from the accumulators into the V^T layout of the spatial
// attention kernel (consecutive lanes = consecutive tokens there).
#include "lc_internal.h"

#include <type_traits>

namespace lc {

namespace {

struct LinArgs {
  const void* x;
  const float* scale;
  const float* shift;
  const void* wf;  // fragment-major weights, see pack_lin_w_kernel
  const float* bias;
  const float* res;
  void* y;
  void* yt;
  int Cout, ldy, tc, tiles_per_wg;  // tc: 32-channel tiles per workgroup column
  int yt_from, yt_T, yt_Tp;
  int rows;
  int im_H, im_W, im_Cl;  // SRC == 2: x is planar [frames][im_Cl][im_H][im_W]
  float* stat;            // per-channel statistics of the output (see FusedDesc), or nullptr
  int stat_splits, stat_rps, stat_off;
  float q_scale;          // output channels below q_cols are multiplied by this before rounding
  int q_cols;
  RowMap in_map, out_map;
};

constexpr int kRows = 32;        // rows of one activation tile
constexpr int kTileMax = 3;      // 32-channel tiles one wavefront can own
constexpr int kLinMinTiles = 2;  // fewest activation tiles a workgroup takes on (it loads its weights once)

// Segment / offset of dense row row0 + r for a segment length rps, with the division of the
// (wave-uniform) tile origin done once: seg0 = row0 / rps, rem0 = row0 % rps.
struct TileOrigin {
  int seg0, rem0;
};
__device__ __forceinline__ TileOrigin tile_origin(int row0, int rps) {
  const int q = row0 / rps;
  return TileOrigin{q, row0 - q * rps};
}
__device__ __forceinline__ void locate(const TileOrigin& o, int rps, int r, int& seg, int& rem) {
  const unsigned x = (unsigned)(o.rem0 + r);
  const unsigned dq = x / (unsigned)rps;
  seg = o.seg0 + (int)dq;
  rem = (int)(x - dq * (unsigned)rps);
}
__device__ __forceinline__ int64_t mapped(const RowMap& m, int seg, int rem) {
  return m.base + (int64_t)seg * m.seg_stride + rem;
}

}  // namespace

// SRC: 0 = x has the operand type; 1 = x is fp32 and gets scale/shift (GroupNorm apply); 2 = row r is
// the 3x3 neighbourhood (zero padded) of pixel r of a planar image, k = channel * 9 + tap, zeros beyond
// 9 * im_Cl: a first convolution with few input channels as a linear layer on gathered rows
template <class T, class OT, int CIN, int SRC>
__global__ __launch_bounds__(256) void lin_kernel(LinArgs a) {
  typedef Mma32<T> M;
  constexpr int VEC = Vec16<T>::N;
  constexpr int ES = (int)sizeof(T);
  constexpr int KT = CIN / M::K;                 // MFMA k-steps over the whole contraction
  constexpr int XS = CIN * ES + 16;              // LDS row stride of the activation tile, bytes
  constexpr int TS = 32 * (int)sizeof(OT) + 16;  // LDS row stride of the output patch, bytes
  constexpr int PPR = CIN / VEC;                 // operand packets per row
  constexpr int RPR = 256 / PPR;                 // rows one round of the staging threads covers
  constexpr int XP = (kRows + RPR - 1) / RPR;    // rounds = packets per thread
  constexpr int RAWN = (SRC == 1 && VEC == 8) ? 2 : 1;  // 16-byte loads per packet
  constexpr int OV = 16 / (int)sizeof(OT);       // output elements per 16-byte store
  constexpr int LPR = 32 / OV;                   // lanes per output row of a 32-channel tile
  constexpr int RPI = 64 / LPR;                  // rows per store instruction
  constexpr int NK = kRows / RPI;                // 16-byte stores per lane per tile
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  auto x_lds = [&](int b) { return smem + b * kRows * XS; };

  const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const int lp = lane & 31, hh = lane >> 5;
  unsigned char* const t_lds = smem + 2 * kRows * XS + wid * kRows * TS;
  const int ntiles = (a.rows + kRows - 1) / kRows;
  const int t0 = blockIdx.x * a.tiles_per_wg;
  const int t1 = min(ntiles, t0 + a.tiles_per_wg);
  if (t0 >= t1) return;
  // this wavefront's share of the column's tiles
  const int nt = a.tc / 4 + (wid < a.tc % 4 ? 1 : 0);
  const int tile0 = blockIdx.y * a.tc + wid * (a.tc / 4) + min(wid, a.tc % 4);
  const int co_w = tile0 * 32;

  // ---- resident weights: fragment kt of tile i
  typename M::Frag wf[kTileMax][KT];
  {
    const typename M::Frag* W = (const typename M::Frag*)a.wf + ((int64_t)tile0 * KT) * 64 + lane;
    if (nt > 0) {
#pragma unroll
      for (int i = 0; i < kTileMax; ++i) {
        const int ic = i < nt ? i : 0;  // tiles this wavefront does not own: a harmless repeat, never used
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) wf[i][kt] = W[(ic * KT + kt) * 64];
      }
    }
  }

  // ---- activation staging: a thread keeps packet column `col` and rows rg, rg + RPR, ...
  const int col = tid % PPR, rg = tid / PPR;
  const bool stager = rg < RPR;
  const int c0 = col * VEC;
  f32x4 raw[XP][RAWN];
  T graw[SRC == 2 ? XP : 1][VEC];  // SRC == 2: gathered neighbourhood values and which of them exist
  unsigned gmask[SRC == 2 ? XP : 1];
  float sc[VEC], sh[VEC];  // dead unless SRC == 1
  int fcur = -1;
  auto fetch_x = [&](int t) {
    const int row0 = t * kRows;
    const int rmax = a.rows - 1 - row0;
    if constexpr (SRC == 2) {
      const int hw = a.im_H * a.im_W;
#pragma unroll
      for (int j = 0; j < XP; ++j) {
        const int row = row0 + min(min(rg + RPR * j, kRows - 1), rmax);
        const int f = row / hw, p = row - f * hw;
        const int yy = p / a.im_W, xx = p - yy * a.im_W;
        const T* img = (const T*)a.x + (int64_t)f * a.im_Cl * hw;
        unsigned m = 0;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          const int k = c0 + e;
          const int cl = k / 9, tap = k - cl * 9;
          const int iy = yy + tap / 3 - 1, ix = xx + tap % 3 - 1;
          const bool ok = cl < a.im_Cl && iy >= 0 && iy < a.im_H && ix >= 0 && ix < a.im_W;
          m |= ok ? 1u << e : 0u;
          // clamped: always a valid element
          graw[j][e] = img[(int64_t)min(cl, a.im_Cl - 1) * hw + min(max(iy, 0), a.im_H - 1) * a.im_W + min(max(ix, 0), a.im_W - 1)];
        }
        gmask[j] = m;
      }
      return;
    }
    const TileOrigin o = tile_origin(row0, a.in_map.rows_per_seg);
    if (o.rem0 + kRows <= a.in_map.rows_per_seg) {
      // the usual case: the tile lies inside one segment, its rows are consecutive in memory. One
      // (wave-uniform) base and 32-bit offsets: no per-lane division, no 64-bit arithmetic.
      const int64_t sr0 = mapped(a.in_map, o.seg0, o.rem0);
#pragma unroll
      for (int j = 0; j < XP; ++j) {
        const int r = min(min(rg + RPR * j, kRows - 1), rmax);  // clamped: always a valid row
        const int ofs = r * CIN + c0;
        if (SRC == 1) {
          const float* px = (const float*)a.x + sr0 * CIN + ofs;
#pragma unroll
          for (int q = 0; q < RAWN; ++q) raw[j][q] = *reinterpret_cast<const f32x4*>(px + 4 * q);
        } else {
          raw[j][0] = *reinterpret_cast<const f32x4*>((const T*)a.x + sr0 * CIN + ofs);
        }
      }
      return;
    }
#pragma unroll
    for (int j = 0; j < XP; ++j) {
      const int r = min(min(rg + RPR * j, kRows - 1), rmax);  // clamped: always a valid row
      int seg, rem;
      locate(o, a.in_map.rows_per_seg, r, seg, rem);
      const int64_t sr = mapped(a.in_map, seg, rem);
      if (SRC == 1) {
        const float* px = (const float*)a.x + sr * CIN + c0;
#pragma unroll
        for (int q = 0; q < RAWN; ++q) raw[j][q] = *reinterpret_cast<const f32x4*>(px + 4 * q);
      } else {
        raw[j][0] = *reinterpret_cast<const f32x4*>((const T*)a.x + sr * CIN + c0);
      }
    }
  };
  auto finish_x = [&](int buf, int t) {
    const int row0 = t * kRows;
    const TileOrigin o = tile_origin(row0, a.in_map.rows_per_seg);
    const bool one_seg = o.rem0 + kRows <= a.in_map.rows_per_seg;
    const int rmax = a.rows - 1 - row0;
#pragma unroll
    for (int j = 0; j < XP; ++j) {
      const int r = rg + RPR * j;
      if (stager && r < kRows) {
        const bool ok = r <= rmax;
        Vec16<T> out;
        if constexpr (SRC == 1) {
          int f = o.seg0, rem;
          if (!one_seg) locate(o, a.in_map.rows_per_seg, min(r, rmax), f, rem);
          if (f != fcur) {  // one segment: the same for every lane, at most once per tile
            fcur = f;
            load_f<float, VEC>(a.scale + (int64_t)f * CIN + c0, sc);
            load_f<float, VEC>(a.shift + (int64_t)f * CIN + c0, sh);
          }
#pragma unroll
          for (int e = 0; e < VEC; ++e) out.set(e, ok ? fmaf(raw[j][(e >> 2) % RAWN][e & 3], sc[e], sh[e]) : 0.f);
        } else if constexpr (SRC == 2) {
#pragma unroll
          for (int e = 0; e < VEC; ++e) out.set(e, (ok && (gmask[j] >> e & 1u)) ? to_f32(graw[j][e]) : 0.f);
        } else {
          out = __builtin_bit_cast(Vec16<T>, raw[j][0]);
          if (!ok) out = zero16<T>();
        }
        *reinterpret_cast<Vec16<T>*>(x_lds(buf) + r * XS + col * 16) = out;
      }
    }
  };

  // ---- output side: lane -> (rows orow_l + RPI k, 16-byte piece ocol) of a tile's patch
  const int ocol = lane % LPR, orow_l = lane / LPR;
  float bias_l[kTileMax][OV];  // fp32 output only; the bf16 path reads its bias when it stores
  if constexpr (sizeof(OT) == 4) {
#pragma unroll
    for (int i = 0; i < kTileMax; ++i)
#pragma unroll
      for (int e = 0; e < OV; ++e) bias_l[i][e] = 0.f;
    if (a.bias && nt > 0) {
#pragma unroll
      for (int i = 0; i < kTileMax; ++i)
        load_f<float, OV>(a.bias + co_w + (i < nt ? i : 0) * 32 + ocol * OV, bias_l[i]);
    }
  }
  OT* Y = (OT*)a.y;
  const float* R = a.res;  // may alias Y

  fetch_x(t0);
  finish_x(0, t0);
  __syncthreads();

  for (int t = t0; t < t1; ++t) {
    const int buf = (t - t0) & 1;
    const bool more = t + 1 < t1;
    const int row0 = t * kRows;
    fetch_x(more ? t + 1 : t);  // the last step repeats its own tile: no branch around the loads
    // rows of the output patch this lane stores, and the residual it adds there
    const TileOrigin oo = tile_origin(row0, a.out_map.rows_per_seg);
    int64_t orow[NK];
#pragma unroll
    for (int k = 0; k < NK; ++k) {
      const int rr = min(orow_l + RPI * k, a.rows - 1 - row0);
      if (oo.rem0 + kRows <= a.out_map.rows_per_seg) {  // the tile lies inside one segment (uniform)
        orow[k] = (mapped(a.out_map, oo.seg0, oo.rem0) + rr) * a.ldy + co_w + ocol * OV;
      } else {
        int seg, rem;
        locate(oo, a.out_map.rows_per_seg, rr, seg, rem);
        orow[k] = mapped(a.out_map, seg, rem) * a.ldy + co_w + ocol * OV;
      }
    }
    f32x4 rres[kTileMax][NK];
    if constexpr (sizeof(OT) == 4) {
      if (R && nt > 0) {
#pragma unroll
        for (int i = 0; i < kTileMax; ++i)
#pragma unroll
          for (int k = 0; k < NK; ++k)
            rres[i][k] = *reinterpret_cast<const f32x4*>(R + orow[k] + (i < nt ? i : 0) * 32);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    f32x16 acc[kTileMax];
#pragma unroll
    for (int i = 0; i < kTileMax; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    const unsigned char* xl = x_lds(buf) + lp * XS + hh * M::LK * ES;
    auto compute = [&](auto ntc) {
      constexpr int N = decltype(ntc)::value;
      constexpr int AHEAD = 3;  // activation fragments requested ahead of their use
      typename M::Frag xf[AHEAD + 1];
#pragma unroll
      for (int kt = 0; kt < AHEAD && kt < KT; ++kt) xf[kt] = M::load((const T*)(xl + kt * M::K * ES));
#pragma unroll
      for (int kt = 0; kt < KT; ++kt) {
        if (kt + AHEAD < KT) xf[(kt + AHEAD) % (AHEAD + 1)] = M::load((const T*)(xl + (kt + AHEAD) * M::K * ES));
        __builtin_amdgcn_sched_barrier(0);  // keep the request ahead of the MFMAs it must overlap with
#pragma unroll
        for (int i = 0; i < N; ++i) M::mma(wf[i][kt], xf[kt % (AHEAD + 1)], acc[i]);
      }
    };
    if (nt == 3) compute(std::integral_constant<int, 3>{});
    else if (nt == 2) compute(std::integral_constant<int, 2>{});
    else if (nt == 1) compute(std::integral_constant<int, 1>{});
    __builtin_amdgcn_sched_barrier(0);
    // next tile into LDS before this tile's stores go out: waiting for its loads must not wait for them
    if (more) finish_x(buf ^ 1, t + 1);
    __builtin_amdgcn_sched_barrier(0);
    // ---- lane holds, for row lp of the tile, channels co + 8 g + 4 hh + {0..3} of each of its tiles
#pragma unroll
    for (int i = 0; i < kTileMax; ++i) {
      if (i >= nt) break;
      const int co = co_w + i * 32;
      if (a.yt && co >= a.yt_from) {
        if (row0 + lp < a.rows) {
          const TileOrigin ov = tile_origin(row0, a.yt_T);
          int f, tk;
          locate(ov, a.yt_T, lp, f, tk);
          OT* dst = (OT*)a.yt + ((int64_t)f * (a.Cout - a.yt_from) + (co - a.yt_from)) * a.yt_Tp + (tk & ~63) +
                    vcol<OT>(tk & 63);
#pragma unroll
          for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int e = 0; e < 4; ++e) dst[(int64_t)(g * 8 + hh * 4 + e) * a.yt_Tp] = from_f32<OT>(acc[i][g * 4 + e]);
        }
        continue;
      }
      const float osc = co < a.q_cols ? a.q_scale : 1.f;  // uniform per tile
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        unsigned char* p = t_lds + lp * TS + (g * 8 + hh * 4) * (int)sizeof(OT);
        if constexpr (sizeof(OT) == 2) {
          bf16x4 ov;
#pragma unroll
          for (int e = 0; e < 4; ++e) ov[e] = static_cast<bf16_t>(acc[i][g * 4 + e] * osc);
          *reinterpret_cast<bf16x4*>(p) = ov;
        } else {
          *reinterpret_cast<f32x4*>(p) = f32x4{acc[i][g * 4] * osc, acc[i][g * 4 + 1] * osc, acc[i][g * 4 + 2] * osc, acc[i][g * 4 + 3] * osc};
        }
      }
      // the patch is private to this wavefront, whose LDS operations complete in order
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      float ssum[4] = {0.f, 0.f, 0.f, 0.f}, ssq[4] = {0.f, 0.f, 0.f, 0.f};  // statistics of this lane's rows
#pragma unroll
      for (int k = 0; k < NK; ++k) {
        const int r = orow_l + RPI * k;
        const Vec16<OT> pv = *reinterpret_cast<const Vec16<OT>*>(t_lds + r * TS + ocol * 16);
        if (row0 + r < a.rows) {
          const int64_t o = orow[k] + i * 32;
          if constexpr (sizeof(OT) == 4) {
            f32x4 v = pv.v;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] += bias_l[i][e];
            if (R) v += rres[i][k];
            *reinterpret_cast<f32x4*>((float*)Y + o) = v;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              ssum[e] += v[e];
              ssq[e] = fmaf(v[e], v[e], ssq[e]);
            }
          } else {
            Vec16<OT> ov = pv;
            if (a.bias) {
              float bv[OV];
              load_f<float, OV>(a.bias + co + ocol * OV, bv);
#pragma unroll
              for (int e = 0; e < OV; ++e) ov.set(e, pv.get(e) + bv[e]);
            }
            store16((OT*)Y + o, ov);
          }
        }
      }
      if constexpr (sizeof(OT) == 4) {
        if (a.stat) {
          // the 32 rows of the tile lie in one frame and one split: fold the lanes that hold the same
          // channels (they differ in lane / LPR), in a fixed order, and let the first of them write
#pragma unroll
          for (int e = 0; e < 4; ++e) {
#pragma unroll
            for (int m = LPR; m < 64; m <<= 1) {
              ssum[e] += __shfl_xor(ssum[e], m, 64);
              ssq[e] += __shfl_xor(ssq[e], m, 64);
            }
          }
          if (orow_l == 0) {
            const int fr = row0 / a.stat_rps;
            const int split = (a.stat_off + (row0 - fr * a.stat_rps)) >> 5;
            float* sp = a.stat + (((int64_t)fr * a.stat_splits + split) * a.Cout + co + ocol * OV) * 2;
            *reinterpret_cast<f32x4*>(sp) = f32x4{ssum[0], ssq[0], ssum[1], ssq[1]};
            *reinterpret_cast<f32x4*>(sp + 4) = f32x4{ssum[2], ssq[2], ssum[3], ssq[3]};
          }
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
  }
}

// Fragment-major copy of a row-major weight matrix w[Cout][Cin] for lin_kernel: fragment (tile, kt)
// holds, for lane l, the M::LK consecutive k values  kt * M::K + (l / 32) * M::LK ...  of output
// channel 32 * tile + l % 32; fragments are stored [tile][kt][lane].
template <class T>
__global__ void pack_lin_w_kernel(const T* __restrict__ w, T* __restrict__ out, int Cout, int Cin) {
  typedef Mma32<T> M;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;  // output element
  if (i >= (int64_t)Cout * Cin) return;
  const int e = (int)(i % M::LK);
  int64_t q = i / M::LK;
  const int lane = (int)(q % 64);
  q /= 64;
  const int KT = Cin / M::K;
  const int kt = (int)(q % KT), tile = (int)(q / KT);
  out[i] = w[(int64_t)(tile * 32 + (lane & 31)) * Cin + kt * M::K + (lane >> 5) * M::LK + e];
}
hipError_t launch_pack_lin_w(hipStream_t s, int dt, const void* w, void* out, int Cout, int Cin) {
  if (Cout % 32 != 0 || Cin % 16 != 0) return hipErrorInvalidValue;
  const int64_t n = (int64_t)Cout * Cin;
  const unsigned blocks = (unsigned)((n + 255) / 256);
  if (dt == kBF16) pack_lin_w_kernel<bf16_t><<<blocks, 256, 0, s>>>((const bf16_t*)w, (bf16_t*)out, Cout, Cin);
  else pack_lin_w_kernel<float><<<blocks, 256, 0, s>>>((const float*)w, (float*)out, Cout, Cin);
  return hipGetLastError();
}

// w[Cout][Cin] -> out[Cout][Cin_padded], zero columns beyond Cin
template <class T>
__global__ void pad_rows_kernel(const T* __restrict__ w, T* __restrict__ out, int Cout, int Cin, int Cin_padded) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (int64_t)Cout * Cin_padded) return;
  const int k = (int)(i % Cin_padded);
  const int64_t co = i / Cin_padded;
  out[i] = k < Cin ? w[co * Cin + k] : from_f32<T>(0.f);
}
hipError_t launch_pad_rows(hipStream_t s, int dt, const void* w, void* out, int Cout, int Cin, int Cin_padded) {
  const int64_t n = (int64_t)Cout * Cin_padded;
  if (n <= 0 || Cin > Cin_padded) return hipErrorInvalidValue;
  const unsigned blocks = (unsigned)((n + 255) / 256);
  if (dt == kBF16) pad_rows_kernel<bf16_t><<<blocks, 256, 0, s>>>((const bf16_t*)w, (bf16_t*)out, Cout, Cin, Cin_padded);
  else pad_rows_kernel<float><<<blocks, 256, 0, s>>>((const float*)w, (float*)out, Cout, Cin, Cin_padded);
  return hipGetLastError();
}

template <class T, class OT, int CIN, int SRC>
static hipError_t run_lin(hipStream_t s, const FusedDesc& d) {
  // workgroup columns: as few as keep a column within 4 wavefronts x kTileMax tiles
  const int tiles = d.Cout / 32;
  int cols = (tiles + 4 * kTileMax - 1) / (4 * kTileMax);
  while (tiles % cols) ++cols;
  const int tc = tiles / cols;
  if (d.yt && d.yt_from % 32) return hipErrorInvalidValue;
  const int lds = 2 * kRows * (CIN * (int)sizeof(T) + 16) + 4 * kRows * (32 * (int)sizeof(OT) + 16);
  auto kern = lin_kernel<T, OT, CIN, SRC>;
  static int attr_bytes = 0;  // per instantiation
  if (lds > attr_bytes) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    attr_bytes = lds;
  }
  LinArgs a;
  a.x = d.x; a.scale = d.scale; a.shift = d.shift; a.wf = d.w_frag; a.bias = d.bias; a.res = (const float*)d.res; a.y = d.y;
  a.yt = d.yt; a.Cout = d.Cout; a.ldy = d.yt ? d.yt_from : d.Cout; a.tc = tc;
  a.yt_from = d.yt_from; a.yt_T = d.yt_T; a.yt_Tp = d.yt_Tp; a.rows = (int)d.rows; a.in_map = d.in_map; a.out_map = d.out_map;
  a.im_H = d.H; a.im_W = d.W; a.im_Cl = d.Cs;
  a.stat = d.stat; a.stat_splits = d.stat_splits; a.stat_rps = d.stat_rps; a.stat_off = d.stat_off;
  a.q_scale = d.q_scale; a.q_cols = d.q_cols;
  // one workgroup per compute unit (its registers hold the weights), each with a contiguous range of tiles
  const int ntiles = ((int)d.rows + kRows - 1) / kRows;
  const int gx_max = 256 / cols > 1 ? 256 / cols : 1;
  int tpw = (ntiles + gx_max - 1) / gx_max;
  if (tpw < kLinMinTiles) tpw = kLinMinTiles;
  a.tiles_per_wg = tpw;
  dim3 grid((unsigned)((ntiles + tpw - 1) / tpw), cols);
  kern<<<grid, 256, lds, s>>>(a);
  return hipGetLastError();
}

// Returns hipErrorNotSupported for shapes whose weights do not fit the register budget (the caller
// then uses the streaming kernel).
hipError_t launch_linear(hipStream_t s, const FusedDesc& d) {
  if (d.taps != 1 || d.rows <= 0) return d.rows <= 0 ? hipSuccess : hipErrorInvalidValue;
  if (!d.w_frag || d.Cout % 32 != 0 || d.Cout_store != d.Cout || d.rows > (int64_t)1 << 30) return hipErrorNotSupported;
  const bool y32 = d.y_f32 || d.dt != kBF16;
  if (d.res && !y32) return hipErrorNotSupported;
  if (d.q_cols && (d.q_cols % 32 || d.q_cols > d.Cout || d.bias || d.res || (d.yt && d.q_cols > d.yt_from)))
    return hipErrorInvalidValue;
  if (d.stat && (!y32 || d.yt || d.stat_rps <= 0 || d.stat_rps % 32 || d.stat_off % 32 || d.rows % d.stat_rps ||
                 (d.stat_off + d.stat_rps) / 32 > d.stat_splits))
    return hipErrorInvalidValue;
  if (d.yt && (d.y_f32 || d.res || d.yt_from <= 0 || d.yt_from >= d.Cout || d.yt_Tp % 64 || d.yt_Tp < d.yt_T ||
               d.out_map.rows_per_seg < d.rows))
    return hipErrorInvalidValue;
#define LC_GO(T, OT, SRC)                                                      \
  switch (d.Cin) {                                                             \
    case 64: return run_lin<T, OT, 64, SRC>(s, d);                             \
    case 128: return run_lin<T, OT, 128, SRC>(s, d);                           \
    case 320:                                                                  \
      if (sizeof(T) == 2) return run_lin<T, OT, sizeof(T) == 2 ? 320 : 64, SRC>(s, d); \
      break;                                                                   \
    default: break;                                                            \
  }                                                                            \
  return hipErrorNotSupported
  if (d.src == 2) {  // gathered 3x3 neighbourhoods of a planar image
    if (!y32 || d.res || d.yt || d.Cin != 64 || d.Cs <= 0 || d.Cs * 9 > 64 || d.H <= 0 || d.W <= 0 ||
        d.rows != (int64_t)d.frames * d.H * d.W)
      return hipErrorNotSupported;
    return d.dt == kBF16 ? run_lin<bf16_t, float, 64, 2>(s, d) : run_lin<float, float, 64, 2>(s, d);
  }
  if (d.dt == kBF16) {
    if (d.src == 1 && !y32) { LC_GO(bf16_t, bf16_t, 1); }
    if (d.src == 0 && y32) { LC_GO(bf16_t, float, 0); }
  } else {
    if (d.src == 1) { LC_GO(float, float, 1); }
    if (d.src == 0) { LC_GO(float, float, 0); }
  }
#undef LC_GO
  return hipErrorNotSupported;
}

}  // namespace lc

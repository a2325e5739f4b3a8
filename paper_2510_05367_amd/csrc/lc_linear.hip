// Per-row linear layers (q,k,v and output projections of the attention blocks) on 32x32 MFMA tiles.
//
// K is only C (320) here, so a workgroup keeps its whole activation tile resident: 128 rows x Cin are
// fetched once (through the row map of a temporal pass if any), GroupNorm'ed on the way in when the
// source is the fp32 residual stream, rounded to the operand type and parked in LDS. The workgroup
// then walks `nct` output-channel tiles of BCO = 32 * CO_T channels, streaming the weights of a
// (tile, 64-byte..128-byte K slab) step through a double-buffered LDS tile one step ahead. Each
// wavefront owns 32 rows x BCO channels (no K split: nothing to fold), and writes its tile out when
// the last slab of the tile is done: bias, fp32 residual, row map, or - for the value third of the
// spatial q,k,v - transposed into the V^T layout the spatial attention kernel stages.
#include "lc_internal.h"

namespace lc {

namespace {

constexpr int kRowL = 128;  // K bytes per weight row per step
constexpr int kLdsL = 144;  // LDS row stride of the weight tile

struct LinArgs {
  const void* x;
  const float* scale;
  const float* shift;
  const void* w;  // T [Cout][Cin]
  const float* bias;
  const float* res;
  void* y;
  void* yt;
  int Cin, Cout, ldy, nct;
  int yt_from, yt_T, yt_Tp;
  int64_t rows;
  RowMap in_map, out_map;
};

}  // namespace

// SRC: 0 = x has the operand type; 1 = x is fp32 and gets scale/shift (GroupNorm apply)
template <class T, class OT, int CO_T, int SRC>
__global__ __launch_bounds__(256) void lin_kernel(LinArgs a) {
  typedef Mma32<T> M;
  constexpr int VEC = Vec16<T>::N;
  constexpr int BKC = kRowL / (int)sizeof(T);
  constexpr int BCO = CO_T * 32;
  constexpr int WP = (BCO * 8 + 255) / 256;
  constexpr int KI = kRowL / (M::K * (int)sizeof(T));
  constexpr int LKB = M::LK * (int)sizeof(T), KB = M::K * (int)sizeof(T);
  constexpr int XB = 4;  // x packets in flight per thread while the tile is staged
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int xs = a.Cin * (int)sizeof(T) + 16;  // x row stride: rows start 16 bytes apart modulo 128
  unsigned char* const x_lds = smem;
  auto w_lds = [&](int b) { return smem + 128 * xs + b * BCO * kLdsL; };

  const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const int lp = lane & 31, hh = lane >> 5;
  const int64_t row0 = (int64_t)blockIdx.x * 128;
  const int ct0 = blockIdx.y * a.nct;
  const T* __restrict__ Wt = (const T*)a.w;
  const int kp = tid & 7, lrow = tid >> 3;
  const int nslab = a.Cin / BKC;
  const int nsteps = a.nct * nslab;

  Vec16<T> wreg[WP];
  auto issue_w = [&](int step) {
    const int ct = step / nslab, slab = step - ct * nslab;
    const int kofs = slab * BKC + kp * VEC;
#pragma unroll
    for (int i = 0; i < WP; ++i) {
      const int r = min(lrow + 32 * i, BCO - 1);
      wreg[i] = load16(Wt + (int64_t)((ct0 + ct) * BCO + r) * a.Cin + kofs);
    }
  };
  auto store_w = [&](int buf) {
#pragma unroll
    for (int i = 0; i < WP; ++i) {
      const int r = lrow + 32 * i;
      if (BCO % 32 == 0 || r < BCO) *reinterpret_cast<Vec16<T>*>(w_lds(buf) + r * kLdsL + kp * 16) = wreg[i];
    }
  };
  issue_w(0);

  // ---- stage the activation tile: packet q = tid + 256 j is (row q / ppr, packet q % ppr)
  {
    const int ppr = a.Cin / VEC;
    const int total = 128 * ppr;
    for (int q0 = 0; q0 < total; q0 += 256 * XB) {
      f32x4 raw[XB][2];
      float sc[XB][VEC], sh[XB][VEC];
      bool ok[XB];
#pragma unroll
      for (int j = 0; j < XB; ++j) {
        const int q = min(q0 + tid + 256 * j, total - 1);
        const int r = q / ppr, c0 = (q - r * ppr) * VEC;
        const int64_t rr = row0 + r;
        ok[j] = rr < a.rows;
        const int64_t rc = ok[j] ? rr : a.rows - 1;
        const int64_t sr = a.in_map(rc);
        if (SRC == 1) {
          const float* px = (const float*)a.x + sr * a.Cin + c0;
          raw[j][0] = *reinterpret_cast<const f32x4*>(px);
          if (VEC == 8) raw[j][1] = *reinterpret_cast<const f32x4*>(px + 4);
          const int64_t f = rc / a.in_map.rows_per_seg;
          load_f<float, VEC>(a.scale + f * a.Cin + c0, sc[j]);
          load_f<float, VEC>(a.shift + f * a.Cin + c0, sh[j]);
        } else {
          raw[j][0] = *reinterpret_cast<const f32x4*>((const T*)a.x + sr * a.Cin + c0);
        }
      }
#pragma unroll
      for (int j = 0; j < XB; ++j) {
        const int q = q0 + tid + 256 * j;
        if (q < total) {
          const int r = q / ppr, pk = q - r * ppr;
          Vec16<T> out;
          if (SRC == 1) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) out.set(e, ok[j] ? fmaf(raw[j][e >> 2][e & 3], sc[j][e], sh[j][e]) : 0.f);
          } else {
            out = __builtin_bit_cast(Vec16<T>, raw[j][0]);
            if (!ok[j]) out = zero16<T>();
          }
          *reinterpret_cast<Vec16<T>*>(x_lds + r * xs + pk * 16) = out;
        }
      }
    }
  }
  store_w(0);
  __syncthreads();

  f32x16 acc[CO_T];
#pragma unroll
  for (int i = 0; i < CO_T; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

  const int p = wid * 32 + lp;  // this lane's row of the tile
  const bool row_ok = row0 + p < a.rows;
  const int64_t orow = row_ok ? a.out_map(row0 + p) : 0;
  OT* Y = (OT*)a.y;
  const float* R = a.res;  // may alias Y

  for (int s = 0; s < nsteps; ++s) {
    const int ct = s / nslab, slab = s - ct * nslab;
    const bool more = s + 1 < nsteps;
    if (more) issue_w(s + 1);
    __builtin_amdgcn_sched_barrier(0);
    {
      const unsigned char* xl = x_lds + p * xs + slab * kRowL + hh * LKB;
      const unsigned char* wl = w_lds(s & 1) + lp * kLdsL + hh * LKB;
#pragma unroll
      for (int kk = 0; kk < KI; ++kk) {
        const typename M::Frag xf = M::load((const T*)(xl + kk * KB));
#pragma unroll
        for (int i = 0; i < CO_T; ++i) {
          const typename M::Frag wf = M::load((const T*)(wl + i * 32 * kLdsL + kk * KB));
          M::mma(wf, xf, acc[i]);
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    if (more) store_w((s + 1) & 1);
    if (slab == nslab - 1) {
      // ---- tile done: lane holds, for row p, channels co0 + 32 i + 8 g + 4 hh + {0..3}
      const int co0 = (ct0 + ct) * BCO;
      if (row_ok) {
#pragma unroll
        for (int i = 0; i < CO_T; ++i)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const int co = co0 + i * 32 + g * 8 + hh * 4;
            float v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = acc[i][g * 4 + e] + (a.bias ? a.bias[co + e] : 0.f);
            if (a.yt && co >= a.yt_from) {  // uniform over the workgroup
              const int64_t rr = row0 + p;
              const int64_t f = rr / a.yt_T;
              const int t = (int)(rr - f * a.yt_T);
              OT* dst = (OT*)a.yt + (f * (a.Cout - a.yt_from) + (co - a.yt_from)) * a.yt_Tp + (t & ~63) +
                        vcol<OT>(t & 63);
#pragma unroll
              for (int e = 0; e < 4; ++e) dst[(int64_t)e * a.yt_Tp] = from_f32<OT>(v[e]);
            } else {
              const int64_t o = orow * a.ldy + co;
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
#pragma unroll
      for (int i = 0; i < CO_T; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    }
    __syncthreads();
  }
}

template <class T, class OT, int CO_T, int SRC>
static hipError_t run_lin(hipStream_t s, const FusedDesc& d, int lds) {
  constexpr int BCO = CO_T * 32;
  auto kern = lin_kernel<T, OT, CO_T, SRC>;
  static int attr_bytes = 0;  // per instantiation
  if (lds > attr_bytes) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    attr_bytes = lds;
  }
  LinArgs a;
  a.x = d.x; a.scale = d.scale; a.shift = d.shift; a.w = d.w; a.bias = d.bias; a.res = (const float*)d.res; a.y = d.y;
  a.yt = d.yt; a.Cin = d.Cin; a.Cout = d.Cout; a.ldy = d.yt ? d.yt_from : d.Cout;
  a.yt_from = d.yt_from; a.yt_T = d.yt_T; a.yt_Tp = d.yt_Tp; a.rows = d.rows; a.in_map = d.in_map; a.out_map = d.out_map;
  // output-channel tiles per workgroup: as many as possible while the grid still covers the chip
  const int tiles = d.Cout / BCO;
  const int64_t row_blocks = (d.rows + 127) / 128;
  int nct = tiles;
  while (nct > 1 && (tiles % nct != 0 || row_blocks * (tiles / nct) < 256)) --nct;
  a.nct = nct;
  dim3 grid((unsigned)row_blocks, tiles / nct);
  kern<<<grid, 256, lds, s>>>(a);
  return hipGetLastError();
}

// Returns hipErrorNotSupported when the resident activation tile does not fit in LDS (the caller
// then uses the streaming kernel).
hipError_t launch_linear(hipStream_t s, const FusedDesc& d) {
  if (d.taps != 1 || d.rows <= 0) return d.rows <= 0 ? hipSuccess : hipErrorInvalidValue;
  const int es = (int)dtype_size(d.dt);
  if (d.Cin % (kRowL / es) != 0 || d.Cout_store != d.Cout) return hipErrorInvalidValue;
  const bool wide = d.Cout % 160 == 0;
  if (!wide && d.Cout % 64 != 0) return hipErrorInvalidValue;
  const int bco = wide ? 160 : 64;
  const int lds = 128 * (d.Cin * es + 16) + 2 * bco * kLdsL;
  if (lds > 150 * 1024) return hipErrorNotSupported;
  if (d.yt && (d.y_f32 || d.res || d.yt_from % bco || d.yt_from <= 0 || d.yt_from >= d.Cout || d.yt_Tp % 64 ||
               d.yt_Tp < d.yt_T || d.out_map.rows_per_seg < d.rows))
    return hipErrorInvalidValue;
  const bool y32 = d.y_f32 || es == 4;
#define LC_GO(T, OT, SRC) (wide ? run_lin<T, OT, 5, SRC>(s, d, lds) : run_lin<T, OT, 2, SRC>(s, d, lds))
  if (d.dt == kBF16) {
    if (d.src == 1 && !y32) return LC_GO(bf16_t, bf16_t, 1);
    if (d.src == 0 && y32) return LC_GO(bf16_t, float, 0);
  } else {
    if (d.src == 1) return LC_GO(float, float, 1);
    if (d.src == 0) return LC_GO(float, float, 0);
  }
#undef LC_GO
  return hipErrorInvalidValue;
}

}  // namespace lc

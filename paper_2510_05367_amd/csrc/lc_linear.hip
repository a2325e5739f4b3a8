// Per-row linear layers (q,k,v and output projections of the attention blocks) on 32x32 MFMA tiles,
// weights stationary.
//
// K is only C here (320), so the weights a wavefront needs - up to 96 output channels x Cin - fit
// in its registers as MFMA fragments (3 x Cin/16 packets of 16 bytes for bf16; one wavefront per
// SIMD, so it may use the whole register file; the output projections and the gathering conv_in keep
// one tile per wavefront instead, so that two or three workgroups fit a compute unit and overlap
// each other's latencies). A workgroup of four wavefronts covers a column of
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
  // Spatial window (win_bw == 0: off). The dense rows are frames of win_ft tiles, each frame an image whose rows
  // are win_ftx tiles long; the launch walks only the tiles of a block of win_bh image rows x win_bw tiles that
  // starts at tile win_t0 of every frame: tile j of the launch is tile full_of(j) of the dense rows. win_in /
  // win_out: the input / the output side (y, residual, statistics, V^T) is addressed by the tile's place in the
  // dense rows (1) or by its running number in the launch (0).
  int win_bw, win_bh, win_t0, win_ftx, win_ft, win_in, win_out;
};

constexpr int kRows = 32;        // rows of one activation tile
constexpr int kTileMax = 3;      // 32-channel tiles one wavefront can own
constexpr int kLinMinTiles = 2;  // fewest activation tiles a workgroup takes on (it loads its weights once)

}  // namespace

// compile-time loop: f(integral_constant<int, I>) for I in [I0, N)
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// A running (segment, offset) pair for consecutive 32-row tiles of a row map whose segments are whole
// tiles long: stepping to the next tile is an add and a compare, no division.
struct TileWalk {
  int seg, rem;
  __device__ __forceinline__ void start(int row0, int rps) {
    seg = row0 / rps;
    rem = row0 - seg * rps;
  }
  __device__ __forceinline__ void next(int rps) {
    rem += kRows;
    if (rem >= rps) {
      rem -= rps;
      ++seg;
    }
  }
};

// SRC: 0 = x has the operand type; 1 = x is fp32 and gets scale/shift (GroupNorm apply); 2 = row r is
// the 3x3 neighbourhood (zero padded) of pixel r of a planar image, k = channel * 9 + tap, zeros beyond
// 9 * im_Cl: a first convolution with few input channels as a linear layer on gathered rows.
// NTM: 32-channel tiles per wavefront. RES: a residual is added (fp32 output).
// The launcher guarantees whole tiles: rows and the segment lengths of both row maps, of the V^T
// output and of the statistics are multiples of 32, so a tile never straddles a segment or a frame.
//
// One wavefront per SIMD issues an instruction every few cycles at best and nothing overlaps unless
// the instruction stream says so, so the step of one 32-row activation tile t (a) is lean - all
// per-lane addresses are offsets computed once, the per-tile parts are wave-uniform and advance by
// addition - and (b) carries, between the MFMAs of its k-steps, the work of its neighbours:
//   - the outputs of tile t-1, parked in per-wavefront LDS patches at the end of the last step, are read
//     back row-contiguous, get bias / residual and are stored; their GroupNorm partial sums follow,
//   - between these stores, packet by packet: tile t+1 (requested one step ago) is normalised / rounded
//     and parked in LDS, and the same packet of tile t+2 is requested into the freed registers,
//   - (RES) the residual of tile t is requested.
// The compiler's wait counts must hold on every path, so inside the steps no vector-memory instruction
// sits under a condition: tiles beyond the last are clamped and fetched again, staging lanes without
// a row write to a dump slot, and every wavefront works on NTM tiles - one that owns fewer repeats its
// first tile (one that owns none, the column's first) and stores the same values a second time. The
// waits then leave exactly the younger loads and stores in flight.
template <class T, class OT, int CIN, int SRC, int NTM, bool RES>
__global__ __launch_bounds__(256) void lin_kernel(LinArgs a) {
  typedef Mma32<T> M;
  constexpr int VEC = Vec16<T>::N;
  constexpr int ES = (int)sizeof(T);
  constexpr int XES = SRC == 1 ? 4 : ES;         // bytes per source element
  constexpr int OES = (int)sizeof(OT);
  constexpr int KT = CIN / M::K;                 // MFMA k-steps over the whole contraction
  constexpr int XS = CIN * ES + 16;              // LDS row stride of the activation tile, bytes
  constexpr int TS = 32 * OES + 16;              // LDS row stride of the output patch, bytes
  constexpr int PPR = CIN / VEC;                 // operand packets per row
  constexpr int RPR = 256 / PPR;                 // rows one round of the staging threads covers
  constexpr int XP = (kRows + RPR - 1) / RPR;    // rounds = packets per thread
  constexpr int RAWN = (SRC == 1 && VEC == 8) ? 2 : 1;  // 16-byte loads per packet
  constexpr int OV = 16 / OES;                   // output elements per 16-byte store
  constexpr int LPR = 32 / OV;                   // lanes per output row of a 32-channel tile
  constexpr int RPI = 64 / LPR;                  // rows per store instruction
  constexpr int NK = kRows / RPI;                // 16-byte stores per lane per tile
  constexpr bool F32OUT = OES == 4;
  static_assert(!RES || F32OUT, "the residual stream is fp32");
  // LDS: [2 x (activation tile, 256 dump slots)][4 x NTM output patches][bias 4 x NTM x 32]
  constexpr int kBuf = kRows * XS + 256 * 16;
  constexpr int kOffPatch = 2 * kBuf, kOffBias = kOffPatch + 4 * NTM * kRows * TS;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lp = lane & 31, hh = lane >> 5;
  unsigned char* const t_lds = smem + kOffPatch + wid * (NTM * kRows * TS);  // this wavefront's output patches
  float* const b_lds = reinterpret_cast<float*>(smem + kOffBias) + wid * NTM * 32;
  const int ntiles = a.rows / kRows;
  const int t0 = blockIdx.x * a.tiles_per_wg;
  const int t1 = min(ntiles, t0 + a.tiles_per_wg);
  if (t0 >= t1) return;
  auto full_of = [&](int j) {
    const int q = j / a.win_bw, bx = j - q * a.win_bw;
    const int f = q / a.win_bh, by = q - f * a.win_bh;
    return f * a.win_ft + a.win_t0 + by * a.win_ftx + bx;
  };
  const bool win_in = a.win_bw != 0 && a.win_in != 0, win_out = a.win_bw != 0 && a.win_out != 0;
  auto in_tile = [&](int j) { return win_in ? full_of(j) : j; };
  auto out_tile = [&](int j) { return win_out ? full_of(j) : j; };
  // this wavefront's tiles: its share of the column's, topped up to NTM with repeats
  const int tcol = min(a.tc, a.Cout / 32 - (int)blockIdx.y * a.tc);  // the last column may be narrower
  const int nt = tcol / 4 + (wid < tcol % 4 ? 1 : 0);
  const int tile0 = nt > 0 ? blockIdx.y * a.tc + wid * (tcol / 4) + min(wid, tcol % 4) : blockIdx.y * a.tc;
  auto co_of = [&](int i) { return (tile0 + (i < nt ? i : 0)) * 32; };  // first channel of tile slot i
  auto in_vt = [&](int i) { return a.yt && co_of(i) >= a.yt_from; };    // tile slot i goes to the V^T buffer

  // ---- resident weights: fragment kt of tile slot i. (What does not fit the 256 architectural
  //      registers the allocator parks in the accumulation registers and copies back before use, four
  //      moves per MFMA; MFMAs that read them there directly measured slower still. The launcher keeps
  //      NTM small enough that this stays rare.)
  typename M::Frag wf[NTM][KT];
  {
    const typename M::Frag* W = (const typename M::Frag*)a.wf + lane;
#pragma unroll
    for (int i = 0; i < NTM; ++i) {
      const int64_t tl = co_of(i) / 32;
#pragma unroll
      for (int kt = 0; kt < KT; ++kt) wf[i][kt] = W[(tl * KT + kt) * 64];
    }
  }
  // the bias of this wavefront's channels, in LDS: the deferred stores must not issue loads of their own
  // (waiting for them would also wait for the activation loads issued before them)
  for (int i = lane; i < NTM * 32; i += 64) b_lds[i] = a.bias ? a.bias[co_of(i >> 5) + (i & 31)] : 0.f;

  // ---- activation staging: a thread keeps packet column `col` and rows rg, rg + RPR, ...
  const int col = tid % PPR, rg = tid / PPR;
  const int c0 = col * VEC;
  unsigned xoff[XP];  // byte offset of this lane's packet of round j inside a tile's rows (SRC != 2)
  unsigned xdst[XP];  // where it goes inside an LDS buffer: its row, or this thread's dump slot
#pragma unroll
  for (int j = 0; j < XP; ++j) {
    const int r = rg + RPR * j;
    xoff[j] = (unsigned)((min(r, kRows - 1) * CIN + c0) * XES);  // clamped: always a row of the tile
    xdst[j] = (rg < RPR && r < kRows) ? (unsigned)(r * XS + col * 16) : (unsigned)(kRows * XS + tid * 16);
  }
  f32x4 raw[XP][RAWN];
  T graw[SRC == 2 ? XP : 1][VEC];  // SRC == 2: gathered neighbourhood values and which of them exist
  unsigned gmask[SRC == 2 ? XP : 1];
  float sc[VEC], sh[VEC];  // dead unless SRC == 1
  int fcur = -1;

  // the tile being requested: its index and place in the source rows
  int tf = t0;
  TileWalk wi{0, 0};
  if constexpr (SRC != 2) wi.start(in_tile(t0) * kRows, a.in_map.rows_per_seg);
  const char* xbase = nullptr;
  auto set_xbase = [&]() {
    if constexpr (SRC != 2)
      xbase = (const char*)a.x + (a.in_map.base + (int64_t)wi.seg * a.in_map.seg_stride + wi.rem) * (int64_t)(CIN * XES);
  };
  auto next_in_tile = [&]() {  // beyond the last tile of the range: that tile again
    if (tf < t1 - 1) {
      ++tf;
      if constexpr (SRC != 2) {
        if (win_in) wi.start(full_of(tf) * kRows, a.in_map.rows_per_seg);  // (a window's tiles are not consecutive)
        else wi.next(a.in_map.rows_per_seg);
      }
    }
    set_xbase();
  };
  auto fetch_round = [&](auto J) {
    constexpr int j = decltype(J)::value;
    if constexpr (SRC == 2) {
      const int hw = a.im_H * a.im_W;
      const int row = in_tile(tf) * kRows + min(rg + RPR * j, kRows - 1);
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
    } else {
#pragma unroll
      for (int q = 0; q < RAWN; ++q) raw[j][q] = *reinterpret_cast<const f32x4*>(xbase + xoff[j] + 16 * q);
    }
  };
  // Scale / shift of frame f, fetched (exposed, but only where the frame changes) outside the steps'
  // side work; the wait sits inside the branch, so no load into these registers is pending after it.
  auto affine_for = [&](int f) {
    if constexpr (SRC == 1) {
      if (f != fcur) {
        fcur = f;
        load_f<float, VEC>(a.scale + (int64_t)f * CIN + c0, sc);
        load_f<float, VEC>(a.shift + (int64_t)f * CIN + c0, sh);
#pragma unroll
        for (int e = 0; e < VEC; ++e) asm volatile("" : "+v"(sc[e]), "+v"(sh[e]));
      }
    }
  };
  // every lane consumes what it loaded and writes 16 bytes: lanes without a row of the tile to a dump slot
  auto finish_round = [&](auto J, int buf) {
    constexpr int j = decltype(J)::value;
    Vec16<T> out;
    if constexpr (SRC == 1) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) out.set(e, fmaf(raw[j][(e >> 2) % RAWN][e & 3], sc[e], sh[e]));
    } else if constexpr (SRC == 2) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) out.set(e, (gmask[j] >> e & 1u) ? to_f32(graw[j][e]) : 0.f);
    } else {
      out = __builtin_bit_cast(Vec16<T>, raw[j][0]);
    }
    *reinterpret_cast<Vec16<T>*>(smem + buf * kBuf + xdst[j]) = out;
  };

  // ---- output side: lane -> (rows orow_l + RPI k, 16-byte piece ocol) of a tile's patch
  const int ocol = lane % LPR, orow_l = lane / LPR;
  const unsigned char* const pread = t_lds + orow_l * TS + ocol * 16;  // + (i * kRows + RPI * k) * TS
  unsigned yoff[NTM][NK];  // byte offset of this lane's 16 bytes of (tile slot i, row group k) from the tile's base
#pragma unroll
  for (int i = 0; i < NTM; ++i)
#pragma unroll
    for (int k = 0; k < NK; ++k) {
      const int r = orow_l + RPI * k;
      // rows of y, or (patch row = channel) rows of the V^T buffer
      yoff[i][k] = in_vt(i) ? (unsigned)(((co_of(i) - a.yt_from + r) * a.yt_Tp + ocol * OV) * OES)
                            : (unsigned)((r * a.ldy + co_of(i) + ocol * OV) * OES);
    }
  // wave-uniform bases of the tile being computed (c*) and of the one whose outputs wait in the patches (p*)
  TileWalk wo, wv{0, 0}, ws{0, 0};
  int to = t0;  // the tile whose bases c* hold
  auto start_out = [&](int row0) {
    wo.start(row0, a.out_map.rows_per_seg);
    if (a.yt) wv.start(row0, a.yt_T);
    if (F32OUT && a.stat) ws.start(row0, a.stat_rps);
  };
  start_out(out_tile(t0) * kRows);
  int64_t cy = 0, py = 0;      // byte offset of the tile's first row in y (and in the residual)
  char *cvt = nullptr, *pvt = nullptr;
  float *cst = nullptr, *pst = nullptr;
  auto set_out_bases = [&]() {
    cy = (a.out_map.base + (int64_t)wo.seg * a.out_map.seg_stride + wo.rem) * (int64_t)(a.ldy * OES);
    if (a.yt) cvt = (char*)a.yt + ((int64_t)wv.seg * (a.Cout - a.yt_from) * a.yt_Tp + wv.rem) * OES;
    if (F32OUT && a.stat)
      cst = a.stat + ((int64_t)ws.seg * a.stat_splits + ((a.stat_off + ws.rem) >> 5)) * a.Cout * 2;
  };
  auto next_out_tile = [&]() {
    py = cy; pvt = cvt; pst = cst;
    ++to;
    if (win_out) {
      start_out(full_of(to) * kRows);
    } else {
      wo.next(a.out_map.rows_per_seg);
      if (a.yt) wv.next(a.yt_T);
      if (F32OUT && a.stat) ws.next(a.stat_rps);
    }
    set_out_bases();
  };
  set_out_bases();
  f32x4 rres[RES ? NTM : 1][NK];
  float ssum[4], ssq[4];  // statistics of this lane's rows of the tile being stored
  Vec16<OT> pq;           // the patch piece of the next store, requested one item ahead
  auto res_load = [&](auto I) {
    constexpr int i = decltype(I)::value;
    if constexpr (RES) {
#pragma unroll
      for (int k = 0; k < NK; ++k) rres[i][k] = *reinterpret_cast<const f32x4*>((const char*)a.res + py + yoff[i][k]);
    }
  };
  auto patch_read = [&](auto I, auto K) {
    constexpr int i = decltype(I)::value, k = decltype(K)::value;
    pq = *reinterpret_cast<const Vec16<OT>*>(pread + (i * kRows + RPI * k) * TS);
  };
  // stores row group k of tile slot i from pq and requests the next piece (none after the last)
  auto out_rows_store = [&](auto I, auto K) {
    constexpr int i = decltype(I)::value, k = decltype(K)::value;
    if constexpr (k == 0) {
#pragma unroll
      for (int e = 0; e < 4; ++e) ssum[e] = ssq[e] = 0.f;
    }
    const Vec16<OT> pv = pq;
    constexpr int nx = i * NK + k + 1;
    if constexpr (nx < NTM * NK) patch_read(std::integral_constant<int, nx / NK>{}, std::integral_constant<int, nx % NK>{});
    if (in_vt(i)) {  // the patch holds [channel][token]: rows of the V^T buffer
      store16(reinterpret_cast<OT*>(pvt + yoff[i][k]), pv);
      return;
    }
    char* dst = (char*)a.y + py + yoff[i][k];
    if constexpr (F32OUT) {
      f32x4 v = pv.v + *reinterpret_cast<const f32x4*>(b_lds + i * 32 + ocol * OV);
      if constexpr (RES) v += rres[i][k];
      *reinterpret_cast<f32x4*>(dst) = v;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        ssum[e] += v[e];
        ssq[e] = fmaf(v[e], v[e], ssq[e]);
      }
    } else {
      Vec16<OT> ov = pv;
      if (a.bias) {
        const f32x4 b0 = *reinterpret_cast<const f32x4*>(b_lds + i * 32 + ocol * OV);
        const f32x4 b1 = *reinterpret_cast<const f32x4*>(b_lds + i * 32 + ocol * OV + 4);
#pragma unroll
        for (int e = 0; e < OV; ++e) ov.set(e, pv.get(e) + (e < 4 ? b0[e & 3] : b1[e & 3]));
      }
      store16(reinterpret_cast<OT*>(dst), ov);
    }
  };
  auto out_stats = [&](auto I) {
    constexpr int i = decltype(I)::value;
    if constexpr (F32OUT) {
      if (!a.stat) return;
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
        float* sp = pst + (co_of(i) + ocol * OV) * 2;
        *reinterpret_cast<f32x4*>(sp) = f32x4{ssum[0], ssq[0], ssum[1], ssq[1]};
        *reinterpret_cast<f32x4*>(sp + 4) = f32x4{ssum[2], ssq[2], ssum[3], ssq[3]};
      }
    }
  };

  // ---- the side work of one step, as a list of items dealt over its KT k-steps:
  //      [stores of tile t-1 and, between them, the XP staging rounds][residual loads of tile t: NTM]
  // A staging round parks its packet of tile t+1 and at once requests the same packet of tile t+2 into
  // the registers that just became free: every load has exactly one step to land. The residual of the
  // tile being computed is requested once the stores of the tile before it have used theirs (by then
  // "the tile before", p*, is this tile).
  constexpr int NB = RES ? NTM : 0, ND = NTM * (NK + (F32OUT ? 1 : 0)), NA = XP;
  constexpr int NITEMS = NB + ND + NA;
  constexpr int IPS = (NITEMS + KT - 1) / KT;  // items per k-step

  // prologue: tile t0 parked, tile t0 + 1 on its way
  set_xbase();
  static_for<0, XP>([&](auto J) { fetch_round(J); });
  affine_for(wi.seg);
  static_for<0, XP>([&](auto J) { finish_round(J, 0); });
  next_in_tile();
  static_for<0, XP>([&](auto J) { fetch_round(J); });
  int seg_parked = wi.seg;  // frame of the tile on its way
  __syncthreads();

  const unsigned char* const xl0 = smem + lp * XS + hh * M::LK * ES;                   // this lane's fragment row
  unsigned char* const pw_rows = t_lds + lp * TS + hh * 4 * OES;                        // accumulators -> patch
  unsigned char* const pw_cols = t_lds + vcol<OT>(lp) * OES + hh * 4 * TS;              // the same, transposed

  // One step. P: parity of t - t0 = the LDS buffer tile t is in; FIRST: no tile waits in the patches yet.
  auto step = [&](auto P, auto FIRST) {
    constexpr int p = decltype(P)::value;
    constexpr bool first = decltype(FIRST)::value;
    affine_for(seg_parked);  // of tile t+1, parked during this step
    next_in_tile();          // tile t+2, requested during this step
    // staging round m sits in front of the m-th NA-th of the stores
    auto item = [&](auto I) {
      constexpr int q = decltype(I)::value;
      if constexpr (q >= ND + NA) {
        if constexpr (q == ND + NA) next_out_tile();  // the patches' tile is stored: "the tile before" is now this one
        res_load(std::integral_constant<int, q - ND - NA>{});
      } else {
        constexpr int m = q * NA / (ND + NA);          // staging rounds placed before or at q
        constexpr bool is_round = q == (m * (ND + NA) + NA - 1) / NA;  // q is the slot of round m
        if constexpr (is_round) {
          finish_round(std::integral_constant<int, m>{}, p ^ 1);
          fetch_round(std::integral_constant<int, m>{});
          if constexpr (m == 0 && !first) patch_read(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
        } else if constexpr (!first) {
          constexpr int d = q - m - ((m * (ND + NA) + NA - 1) / NA < q ? 1 : 0);  // stores before q
          constexpr int per = NK + (F32OUT ? 1 : 0);
          if constexpr (d % per < NK) out_rows_store(std::integral_constant<int, d / per>{}, std::integral_constant<int, d % per>{});
          else out_stats(std::integral_constant<int, d / per>{});
        }
      }
    };
    f32x16 acc[NTM];
#pragma unroll
    for (int i = 0; i < NTM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    const unsigned char* xl = xl0 + p * kBuf;
    constexpr int AHEAD = 3;  // activation fragments requested ahead of their use
    typename M::Frag xf[AHEAD + 1];
#pragma unroll
    for (int kt = 0; kt < AHEAD && kt < KT; ++kt) xf[kt] = M::load((const T*)(xl + kt * M::K * ES));
    static_for<0, KT>([&](auto KTc) {
      constexpr int kt = decltype(KTc)::value;
      if constexpr (kt + AHEAD < KT) xf[(kt + AHEAD) % (AHEAD + 1)] = M::load((const T*)(xl + (kt + AHEAD) * M::K * ES));
      __builtin_amdgcn_sched_barrier(0);  // keep the request ahead of the MFMAs it must overlap with
#pragma unroll
      for (int i = 0; i < NTM; ++i) M::mma(wf[i][kt], xf[kt % (AHEAD + 1)], acc[i]);
      __builtin_amdgcn_sched_barrier(0);
      // the items of this k-step: the list is spread from the last k-step backwards, so that parking
      // tile t+1 ends with the MFMAs and the first k-steps (whose fragments are still arriving) stay light
      constexpr int lead = KT * IPS - NITEMS;
      constexpr int i0 = kt * IPS - lead > 0 ? kt * IPS - lead : 0;
      constexpr int i1 = (kt + 1) * IPS - lead > 0 ? (kt + 1) * IPS - lead : 0;
      static_for<i0, i1>(item);
      __builtin_amdgcn_sched_barrier(0);
    });
    // ---- lane holds, for row lp of the tile, channels co + 8 g + 4 hh + {0..3} of each of its tiles
#pragma unroll
    for (int i = 0; i < NTM; ++i) {
      if (in_vt(i)) {  // transposed into the patch: row = channel, column = token in the V^T order
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
          for (int e = 0; e < 4; ++e)
            *reinterpret_cast<OT*>(pw_cols + (i * kRows + g * 8 + e) * TS) = from_f32<OT>(acc[i][g * 4 + e]);
        continue;
      }
      if (co_of(i) < a.q_cols) {  // uniform per tile
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] *= a.q_scale;
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        unsigned char* q = pw_rows + i * kRows * TS + g * 8 * OES;
        if constexpr (OES == 2) {
          bf16x4 ov;
#pragma unroll
          for (int e = 0; e < 4; ++e) ov[e] = static_cast<bf16_t>(acc[i][g * 4 + e]);
          *reinterpret_cast<bf16x4*>(q) = ov;
        } else {
          *reinterpret_cast<f32x4*>(q) = f32x4{acc[i][g * 4], acc[i][g * 4 + 1], acc[i][g * 4 + 2], acc[i][g * 4 + 3]};
        }
      }
    }
    // the patches are private to this wavefront, whose LDS operations complete in order
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    if constexpr (NB == 0) next_out_tile();
    seg_parked = wi.seg;
    // the barrier orders the activation tiles in LDS; loads and stores stay in flight across it
    barrier_keep<63>();
  };

  step(std::integral_constant<int, 0>{}, std::true_type{});
  for (int t = t0 + 1; t < t1; t += 2) {
    step(std::integral_constant<int, 1>{}, std::false_type{});
    if (t + 1 < t1) step(std::integral_constant<int, 0>{}, std::false_type{});
  }
  // the last tile's outputs
  patch_read(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
  static_for<0, NTM>([&](auto I) {
    static_for<0, NK>([&](auto K) { out_rows_store(I, K); });
    out_stats(I);
  });
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

template <class T, class OT, int CIN, int SRC, int NTM, bool RES>
static hipError_t run_lin_r(hipStream_t s, const FusedDesc& d, int cols, int tc) {
  const int lds = 2 * (kRows * (CIN * (int)sizeof(T) + 16) + 256 * 16) + 4 * NTM * kRows * (32 * (int)sizeof(OT) + 16) +
                  4 * NTM * 32 * 4;  // as laid out in the kernel
  auto kern = lin_kernel<T, OT, CIN, SRC, NTM, RES>;
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
  a.win_bw = a.win_bh = a.win_t0 = a.win_ftx = a.win_ft = a.win_in = a.win_out = 0;
  int ntiles = (int)d.rows / kRows;
  if (d.win_w) {  // (validated in launch_linear)
    a.win_bw = d.win_w / kRows; a.win_bh = d.win_h; a.win_ftx = d.win_img_w / kRows; a.win_ft = a.win_ftx * d.win_img_t;
    a.win_t0 = d.win_y0 * a.win_ftx + d.win_x0 / kRows; a.win_in = d.win_in; a.win_out = d.win_out;
    ntiles = (int)(d.rows / ((int64_t)d.win_img_w * d.win_img_t)) * a.win_bh * a.win_bw;
    a.rows = ntiles * kRows;
  }
  // one workgroup per compute unit (its registers hold the weights), each with a contiguous range of tiles.
  // The gathering instantiation with one tile per wavefront has few weights and little LDS: three of its
  // workgroups share a compute unit, and one's gather latency hides behind the others' stores.
  constexpr int kPerCu = (SRC == 2 && NTM == 1) ? 3 : (SRC == 0 && CIN == 320 && NTM == 1) ? 2 : 1;
  const int gx_max = 256 * kPerCu / cols > 1 ? 256 * kPerCu / cols : 1;
  int tpw = (ntiles + gx_max - 1) / gx_max;
  if (tpw < kLinMinTiles) tpw = kLinMinTiles;
  a.tiles_per_wg = tpw;
  dim3 grid((unsigned)((ntiles + tpw - 1) / tpw), (unsigned)((d.Cout / 32 + tc - 1) / tc));
  kern<<<grid, 256, lds, s>>>(a);
  return hipGetLastError();
}

template <class T, class OT, int CIN, int SRC, int NTM>
static hipError_t run_lin_n(hipStream_t s, const FusedDesc& d, int cols, int tc) {
  if constexpr (sizeof(OT) == 4 && SRC == 0) {
    if (d.res) return run_lin_r<T, OT, CIN, SRC, NTM, true>(s, d, cols, tc);
  }
  if (d.res) return hipErrorNotSupported;
  return run_lin_r<T, OT, CIN, SRC, NTM, false>(s, d, cols, tc);
}

template <class T, class OT, int CIN, int SRC>
static hipError_t run_lin(hipStream_t s, const FusedDesc& d) {
  // Tiles per wavefront: as many as leave the weights (one register per lane per 4 bytes of fragment)
  // well inside the 256 architectural registers, at most kTileMax. Workgroup columns: as few as keep a
  // column within 4 wavefronts x that many tiles; the last column may be narrower.
  constexpr int kt_regs = CIN / Mma32<T>::K * (int)sizeof(typename Mma32<T>::Frag) / 4;
  // (the gathering instantiation: one tile, so that several workgroups fit a compute unit - see run_lin_r)
  constexpr int ntm_max = (SRC == 2 || (SRC == 0 && CIN == 320)) ? 1 : 160 / kt_regs < 1 ? 1 : (160 / kt_regs > kTileMax ? kTileMax : 160 / kt_regs);
  const int tiles = d.Cout / 32;
  const int cols = (tiles + 4 * ntm_max - 1) / (4 * ntm_max);
  const int tc = (tiles + cols - 1) / cols;
  if (d.yt && d.yt_from % 32) return hipErrorInvalidValue;
  const int ntm = (tc + 3) / 4;  // most tiles one wavefront owns
  if constexpr (ntm_max >= 3) {
    if (ntm == 3) return run_lin_n<T, OT, CIN, SRC, 3>(s, d, cols, tc);
  }
  if constexpr (ntm_max >= 2) {
    if (ntm == 2) return run_lin_n<T, OT, CIN, SRC, 2>(s, d, cols, tc);
  }
  return run_lin_n<T, OT, CIN, SRC, 1>(s, d, cols, tc);
}

// Returns hipErrorNotSupported for shapes whose weights do not fit the register budget (the caller
// then uses the streaming kernel).
hipError_t launch_linear(hipStream_t s, const FusedDesc& d) {
  if (d.taps != 1 || d.rows <= 0) return d.rows <= 0 ? hipSuccess : hipErrorInvalidValue;
  if (!d.w_frag || d.Cout % 32 != 0 || d.Cout_store != d.Cout || d.rows > (int64_t)1 << 30) return hipErrorNotSupported;
  // whole 32-row tiles that never straddle what changes per frame (GroupNorm scale / shift, V^T rows)
  if (d.rows % kRows || (d.src != 2 && d.in_map.rows_per_seg % kRows) || d.out_map.rows_per_seg % kRows ||
      (d.yt && (d.yt_T % kRows || d.bias)))
    return hipErrorNotSupported;
  if (d.win_w) {  // a window of whole 32-pixel segments of image rows, inside the frame; rows = whole frames
    const int64_t fr = (int64_t)d.win_img_w * d.win_img_t;
    if (d.win_img_w <= 0 || d.win_img_t <= 0 || d.win_img_w % kRows || d.win_x0 % kRows || d.win_w % kRows || d.win_x0 < 0 ||
        d.win_y0 < 0 || d.win_w < 0 || d.win_h <= 0 || d.win_x0 + d.win_w > d.win_img_w || d.win_y0 + d.win_h > d.win_img_t ||
        d.rows % fr)
      return hipErrorInvalidValue;
    if (!d.win_in && !d.win_out) return hipErrorInvalidValue;
  }
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

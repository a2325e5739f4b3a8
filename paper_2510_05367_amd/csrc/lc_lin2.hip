// Linear layers over dense bf16 rows on gfx950: y[rows][N] = x[rows][K] W[N][K]^T (+ bias, + fp32 residual), the
// projections and feed-forward layers of the transformer blocks, where K is a few hundred to a few thousand.
//
// One workgroup = 4 wavefronts = 128 rows x 160 (or 128) output channels; wavefront w owns rows [32 w, 32 w + 32) and
// all channels (5 or 4 accumulator tiles of 32 x 32: every fragment of x feeds five or four MFMAs), and walks K in
// steps of 64 elements without splitting it. Both operands are K-major in memory, so a step's tiles are rows of 128
// bytes, brought from global memory straight into LDS (16 bytes per lane, no registers in between) into a ring of two
// stages: the loads of step s + 1 are issued as soon as those of step s have landed. Two workgroups share a compute
// unit (2 x 74 KB of LDS, 256 registers each) and cover each other's prologue, waits and epilogue. (The first design,
// a 256-row tile with a ring of three stages and one workgroup per compute unit, was slower at every K measured: by
// 6 % at K = 1280, by 13-22 % from K = 1024 to 4096 where the output is narrow.) The 16-byte packet c of row r is
// parked in slot c ^ ((r >> 1) & 7) of its row, which makes the fragment reads (32 consecutive rows, one slot)
// conflict-free without padding. The product is not transposed (rows of x are the rows of the accumulator tile): a
// lane then holds one output channel of 16 rows, and the 32 lanes of a half-wavefront hold 32 consecutive channels of
// one row.
//
// Workgroups are dealt to the eight XCDs round robin in launch order, and each XCD has an L2 of its own: the
// channel tiles of one row tile are mapped to the same XCD, so its L2 fetches that tile of x once.
#include "lc_internal.h"

#include <type_traits>

namespace lc {

namespace {

constexpr int kKB = 128;                        // K bytes per step
constexpr int kStages = 2;
// a workgroup takes 128 rows and 32 NT channels; bytes of one ring stage: the x tile, then the W tile
constexpr int lin2_stage(int NT) { return (128 + NT * 32) * kKB; }
static_assert(2 * kStages * lin2_stage(5) <= 160 * 1024, "two workgroups fit the LDS of a compute unit together");

struct Lin2Args {
  const bf16_t* x;     // [rows][K]
  const bf16_t* w;     // [N][K]
  const float* bias;   // [N] or nullptr
  const float* res;    // fp32 [rows][N] or nullptr (may alias y)
  void* y;             // [rows][N], bf16 or fp32
  bf16_t* y2;          // fp32 output only: a copy of y rounded to bf16 (the next layer's operand), or nullptr
  int64_t rows;
  int K, N, ntm, ntn;
  float q_scale;       // channels below q_cols are multiplied by this before they are rounded
  int q_cols;
  int act;             // 0 none, 1 GELU, 2 GEGLU over alternating 32-channel blocks (y is then N / 2 wide)
  RowMap in_map, out_map;  // dense row r is row in_map(r) of x and row out_map(r) of y / res / y2
  // bf16 output over dense rows only: channels >= yt_from are not stored in y (whose rows then have yt_from channels)
  // but transposed into yt[r / yt_T][N - yt_from][yt_Tp] at column (t & ~63) + vcol(t & 63), t = r % yt_T: the V^T
  // layout of the spatial attention kernel. nullptr: off. yt_from a multiple of the channel tile, yt_T of 4.
  bf16_t* yt;
  int yt_from, yt_T, yt_Tp;
  int ldy;  // channels per row of y (yt_from with yt, else N; N / 2 after a GEGLU)
};

}  // namespace


// bf16 stores of a 32-row half tile, two channels per lane: lanes l and l ^ 1 hold channels c, c + 1 of the same rows;
// they trade halves so that the even lane holds both channels of the even row of a pair and the odd lane both of the
// odd row, and each stores 4 bytes: a wavefront instruction then writes 64 consecutive bytes of two rows instead of
// 64 bytes of one with 2-byte stores. NV: column tiles (32 channels each) in val's second index.
template <int NV, int NTV, bool MAPPED>
__device__ __forceinline__ void store_pairs(const float (&val)[16][NTV], bf16_t* __restrict__ Y, int ldy, int c0, int64_t rbase,
                                            int64_t rows, const RowMap& out_map, int lane, std::integral_constant<bool, MAPPED>) {
  const int lp = lane & 31;
  const bool odd = lane & 1;
  // v_perm_b32 selectors (bytes 0-3: own pair, 4-7: the neighbour's): even (own lo, neighbour's lo), odd (neighbour's hi, own hi)
  const uint32_t sel = odd ? 0x03020706u : 0x05040100u;
#pragma unroll
  for (int rp = 0; rp < 16; rp += 2) {
    uint32_t out[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      bf16x2 p2;
      p2[0] = static_cast<bf16_t>(val[rp][i]);
      p2[1] = static_cast<bf16_t>(val[rp + 1][i]);
      const uint32_t own = __builtin_bit_cast(uint32_t, p2);
      const uint32_t nb = (uint32_t)__builtin_amdgcn_mov_dpp((int)own, 0xB1 /* quad_perm [1,0,3,2] */, 0xF, 0xF, true);
      out[i] = __builtin_amdgcn_perm(nb, own, sel);
    }
    const int64_t dr = rbase + 8 * (rp >> 2) + (rp & 3) + (odd ? 1 : 0);
    if (dr >= rows) continue;
    const int64_t row = MAPPED ? out_map(dr) : dr;
#pragma unroll
    for (int i = 0; i < NV; ++i) *reinterpret_cast<uint32_t*>(Y + row * ldy + c0 + 32 * i + (lp & ~1)) = out[i];
  }
}

// MAPPED: rows go through the row maps (a 64-bit division per row: kept out of the common, dense case, where the
// host folds the maps' offsets into the pointers; the arithmetic, and so every bit of the result, is the same)
template <class OT, int NT, bool MAPPED>
__global__ __launch_bounds__(256, 2) void lin2_kernel(Lin2Args a) {
  typedef Mma32<bf16_t> M;
  constexpr int MR = 1;  // 32-row accumulator tiles per wavefront along the rows
  constexpr int kM = 128 * MR, kN = NT * 32, kStage = lin2_stage(NT);
  constexpr int kXI = 4 * MR, kWI = NT;  // global->LDS instructions per wavefront per stage: x tile, W tile
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lp = lane & 31, hh = lane >> 5;
  // (row tile, channel tile) of this workgroup: all channel tiles of a row tile on one XCD
  const int lin = blockIdx.x, xcd = lin & 7, slot = lin >> 3;
  const int mt = xcd + 8 * (slot / a.ntn), nt = slot - (slot / a.ntn) * a.ntn;
  if (mt >= a.ntm) return;  // the grid is padded to whole rounds of eight row tiles
  const int64_t m0 = (int64_t)mt * kM;
  const int n0 = nt * kN;

  // ---- global -> LDS: instruction i of a tile moves rows 8 i .. 8 i + 7; this lane moves the packet that lands
  //      in slot (lane & 7) of row 8 i + (lane >> 3), i.e. global packet (lane & 7) ^ ((row >> 1) & 7)
  const int lrow = lane >> 3;
  const bf16_t* xsrc[kXI];
  const bf16_t* wsrc[kWI];
#pragma unroll
  for (int j = 0; j < kXI; ++j) {
    const int r = (wid + 4 * j) * 8 + lrow;
    const int c = (lane & 7) ^ ((r >> 1) & 7);
    int64_t gr = min(m0 + r, a.rows - 1);  // rows beyond the end: a valid row, never stored
    if (MAPPED) gr = a.in_map(gr);
    xsrc[j] = a.x + gr * a.K + c * 8;
  }
#pragma unroll
  for (int j = 0; j < kWI; ++j) {
    const int r = (wid + 4 * j) * 8 + lrow;
    const int c = (lane & 7) ^ ((r >> 1) & 7);
    wsrc[j] = a.w + (int64_t)(n0 + r) * a.K + c * 8;
  }
  auto issue = [&](int step, int buf) {
    unsigned char* xb = smem + buf * kStage;
    unsigned char* wb = xb + kM * kKB;
    const int kofs = step * 64;
#ifdef __HIP_DEVICE_COMPILE__  // the host pass only needs the kernel's stub; it does not know this builtin
#pragma unroll
    for (int j = 0; j < kXI; ++j) __builtin_amdgcn_global_load_lds(xsrc[j] + kofs, xb + (wid + 4 * j) * 1024, 16, 0, 0);
#pragma unroll
    for (int j = 0; j < kWI; ++j) __builtin_amdgcn_global_load_lds(wsrc[j] + kofs, wb + (wid + 4 * j) * 1024, 16, 0, 0);
#else
    (void)xb; (void)wb; (void)kofs;
#endif
  };

  f32x16 acc[MR][NT];
#pragma unroll
  for (int j = 0; j < MR; ++j)
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

  // fragment addresses inside a stage: row * 128 + ((slot ^ key) << 4), slot = hh + 2 kk
  const int xrow0 = wid * (32 * MR) + lp, xkey = (xrow0 >> 1) & 7;  // (+32 does not change the key)
  const int wkey = (lp >> 1) & 7;
  auto xfrag = [&](const unsigned char* st, int j, int kk) {
    return M::load((const bf16_t*)(st + (xrow0 + 32 * j) * kKB + (((hh + 2 * kk) ^ xkey) << 4)));
  };
  auto wfrag = [&](const unsigned char* st, int i, int kk) {
    return M::load((const bf16_t*)(st + kM * kKB + (32 * i + lp) * kKB + (((hh + 2 * kk) ^ wkey) << 4)));
  };

  const int nsteps = a.K / 64;
  issue(0, 0);
  for (int s = 0; s < nsteps; ++s) {
    // the loads of step s have landed (for every wavefront, after the barrier), and every wavefront has read step s - 1
    barrier_keep<0>();
    // the next request goes into the stage that was read in step s - 1
    if (s + 1 < nsteps) issue(s + 1, (s + 1) % kStages);
    const unsigned char* st = smem + (s % kStages) * kStage;
    typename M::Frag xf[2][MR], wf[2][NT];
#pragma unroll
    for (int j = 0; j < MR; ++j) xf[0][j] = xfrag(st, j, 0);
#pragma unroll
    for (int i = 0; i < NT; ++i) wf[0][i] = wfrag(st, i, 0);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      if (kk + 1 < 4) {  // the fragments of the next k-step are requested before this one's MFMAs
#pragma unroll
        for (int j = 0; j < MR; ++j) xf[(kk + 1) & 1][j] = xfrag(st, j, kk + 1);
#pragma unroll
        for (int i = 0; i < NT; ++i) wf[(kk + 1) & 1][i] = wfrag(st, i, kk + 1);
      }
#pragma unroll
      for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int j = 0; j < MR; ++j) M::mma(xf[kk & 1][j], wf[kk & 1][i], acc[j][i]);
    }
  }

  // ---- epilogue: lane holds channel n0 + 32 i + lp of rows m0 + 32 MR wid + 32 j + 8 (r / 4) + 4 hh + r % 4
  OT* Y = (OT*)a.y;
  const float* R = a.res;
  float bias_l[NT], mul_l[NT];
#pragma unroll
  for (int i = 0; i < NT; ++i) {
    const int co = n0 + 32 * i + lp;
    bias_l[i] = a.bias ? a.bias[co] : 0.f;
    mul_l[i] = co < a.q_cols ? a.q_scale : 1.f;
  }
  // The residual (which may be y itself: every element is read and written by the same lane) is fetched for a whole
  // 32-row half at once, before the first store of that half: a load placed after a store that may alias it cannot
  // be moved up by the compiler, and one round trip per element would cost more than the whole contraction.
#pragma unroll
  for (int j = 0; j < MR; ++j) {
    const int64_t rbase = m0 + wid * (32 * MR) + 32 * j + 4 * hh;
    float rv[16][NT];
    if (R) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        int64_t row = min(rbase + 8 * (r >> 2) + (r & 3), a.rows - 1);
        if (MAPPED) row = a.out_map(row);
#pragma unroll
        for (int i = 0; i < NT; ++i) rv[r][i] = R[row * a.N + n0 + 32 * i + lp];
      }
    }
    // all arithmetic of the half first, so that the stores below depend on no load: a store under a condition
    // (the ragged last tile) would otherwise be preceded by a wait for everything in flight
    float val[16][NT];
#pragma unroll
    for (int r = 0; r < 16; ++r)
#pragma unroll
      for (int i = 0; i < NT; ++i) {
        val[r][i] = (acc[j][i][r] + bias_l[i]) * mul_l[i];
        if (R) val[r][i] += rv[r][i];
        if (sizeof(OT) == 2 && a.act == 1) val[r][i] = gelu_tanh_fast(val[r][i]);
        asm volatile("" : "+v"(val[r][i]));  // computed here: left alone, the compiler sinks it into the store's branch
      }
    if constexpr (sizeof(OT) == 2) {
      if (a.yt && n0 >= a.yt_from) {  // (uniform over the workgroup) a lane holds 4 consecutive rows of a channel: 8 bytes of V^T
        const int Cv = a.N - a.yt_from;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int64_t dr = rbase + 8 * g;
          if (dr >= a.rows) continue;  // (rows come in fours)
          const int64_t f = dr / a.yt_T;
          const int t = (int)(dr - f * a.yt_T);
          bf16_t* dst = a.yt + (f * Cv + (n0 - a.yt_from) + lp) * a.yt_Tp + (t & ~63) + vcol<bf16_t>(t & 63);
#pragma unroll
          for (int i = 0; i < NT; ++i) {
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = static_cast<bf16_t>(val[4 * g + e][i]);
            *reinterpret_cast<bf16x4*>(dst + (int64_t)32 * i * a.yt_Tp) = o;
          }
        }
        continue;
      }
    }
    if constexpr (sizeof(OT) == 2 && NT % 2 == 0) {
      if (a.act == 2) {  // GEGLU: column tile 2 q holds 32 values, tile 2 q + 1 their gates; N / 2 channels leave
#pragma unroll
        for (int r = 0; r < 16; ++r)
#pragma unroll
          for (int q = 0; q < NT / 2; ++q) {
            val[r][q] = val[r][2 * q] * gelu_tanh_fast(val[r][2 * q + 1]);
            asm volatile("" : "+v"(val[r][q]));
          }
        store_pairs<NT / 2>(val, (bf16_t*)a.y, a.N / 2, n0 / 2, rbase, a.rows, a.out_map, lane, std::integral_constant<bool, MAPPED>{});
        continue;
      }
    }
    if constexpr (sizeof(OT) == 2) {
      store_pairs<NT>(val, (bf16_t*)a.y, a.ldy, n0, rbase, a.rows, a.out_map, lane, std::integral_constant<bool, MAPPED>{});
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t dr = rbase + 8 * (r >> 2) + (r & 3);
        if (dr >= a.rows) continue;
        const int64_t row = MAPPED ? a.out_map(dr) : dr;
#pragma unroll
        for (int i = 0; i < NT; ++i) Y[row * a.N + n0 + 32 * i + lp] = from_f32<OT>(val[r][i]);
      }
      if (a.y2) store_pairs<NT>(val, a.y2, a.N, n0, rbase, a.rows, a.out_map, lane, std::integral_constant<bool, MAPPED>{});
    }
  }
}

// taps == 1, src == 0 of a bf16 stage, Cin % 64 == 0 and Cout % 160 == 0 or % 128 == 0 (rows through any row map);
// hipErrorNotSupported for what it does not cover (the general kernel then runs). Which kernel runs depends on the
// layer's widths only, never on the number of rows: a chunked pass must give the bits of the unchunked one.
// (hipFuncSetAttribute is called once per instantiation and process: one device.)
template <class OT, int NT, bool MAPPED>
static hipError_t run_lin2_k(hipStream_t s, const Lin2Args& a) {
  constexpr int lds = kStages * lin2_stage(NT);
  static bool done = false;  // per instantiation
  if (!done) {
    hipError_t e = hipFuncSetAttribute((const void*)lin2_kernel<OT, NT, MAPPED>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    done = true;
  }
  const unsigned grid = (unsigned)((a.ntm + 7) / 8 * 8 * a.ntn);
  lin2_kernel<OT, NT, MAPPED><<<grid, 256, lds, s>>>(a);
  return hipGetLastError();
}
template <class OT, int NT>
static hipError_t run_lin2(hipStream_t s, Lin2Args a) {
  a.ntn = a.N / (NT * 32);
  a.ntm = (int)((a.rows + 127) / 128);
  // a map that is the identity up to an offset (one segment, or segments that follow each other) is folded into
  // the pointers
  auto plain = [&](const RowMap& m) { return m.rows_per_seg >= a.rows || m.seg_stride == m.rows_per_seg; };
  if (!plain(a.in_map) || !plain(a.out_map)) return a.yt ? hipErrorInvalidValue : run_lin2_k<OT, NT, true>(s, a);
  const int64_t nout = a.ldy;
  a.x += a.in_map.base * a.K;
  a.y = (OT*)a.y + a.out_map.base * nout;
  if (a.res) a.res += a.out_map.base * nout;
  if (a.y2) a.y2 += a.out_map.base * nout;
  return run_lin2_k<OT, NT, false>(s, a);
}

hipError_t launch_lin2(hipStream_t s, const FusedDesc& d) {
  if (d.dt != kBF16 || d.taps != 1 || d.src != 0 || d.stat || d.win_w || d.planar_out) return hipErrorNotSupported;
  if (d.Cin % 64 || d.Cin <= 0 || (d.Cout % 160 && d.Cout % 128) || d.Cout_store != d.Cout) return hipErrorNotSupported;
  if (d.in_map.rows_per_seg <= 0 || d.out_map.rows_per_seg <= 0) return hipErrorInvalidValue;
  if (d.res && !d.y_f32) return hipErrorNotSupported;
  if (d.q_cols && (d.bias || d.res)) return hipErrorInvalidValue;
  if (d.y2 && !d.y_f32) return hipErrorInvalidValue;
  if (d.act && (d.y_f32 || d.res || d.q_cols || d.act > 2)) return hipErrorInvalidValue;
  if (d.act == 2 && d.Cout % 128) return hipErrorNotSupported;
  if (d.yt) {  // the transposed tail: whole channel tiles of a bf16 output, rows in fours
    const int tile = d.Cout % 160 == 0 ? 160 : 128;
    if (d.y_f32 || d.res || d.act || d.y2) return hipErrorInvalidValue;
    if (d.yt_from <= 0 || d.yt_from >= d.Cout || d.yt_from % tile || d.yt_T <= 0 || d.yt_T % 4 || d.rows % 4 || d.yt_Tp % 64 || d.yt_Tp < d.yt_T)
      return hipErrorNotSupported;
  }
  if (d.rows <= 0) return hipSuccess;
  if (d.rows > (int64_t)1 << 30) return hipErrorNotSupported;
  Lin2Args a;
  a.x = (const bf16_t*)d.x; a.w = (const bf16_t*)d.w; a.bias = d.bias; a.res = (const float*)d.res; a.y = d.y;
  a.y2 = (bf16_t*)d.y2;
  a.rows = d.rows; a.K = d.Cin; a.N = d.Cout;
  a.ntm = a.ntn = 0;
  a.q_scale = d.q_cols ? d.q_scale : 1.f; a.q_cols = d.q_cols;
  a.act = d.act;
  a.in_map = d.in_map; a.out_map = d.out_map;
  a.yt = (bf16_t*)d.yt; a.yt_from = d.yt_from; a.yt_T = d.yt_T; a.yt_Tp = d.yt_Tp;
  a.ldy = d.yt ? d.yt_from : (d.act == 2 ? d.Cout / 2 : d.Cout);
  if (d.act == 2) return run_lin2<bf16_t, 4>(s, a);  // (an even number of column tiles: value / gate pairs)
  if (d.Cout % 160 == 0) return d.y_f32 ? run_lin2<float, 5>(s, a) : run_lin2<bf16_t, 5>(s, a);
  return d.y_f32 ? run_lin2<float, 4>(s, a) : run_lin2<bf16_t, 4>(s, a);
}

}  // namespace lc

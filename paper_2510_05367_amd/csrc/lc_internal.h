// Host-side declarations of the kernel launchers (one per kernel family). Every launcher only
// enqueues on `s`; none allocates. Activations are channels-last [rows, channels].
#pragma once
#include <math.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lc_common.h"

namespace lc {

enum Dtype { kF32 = 0, kBF16 = 1 };
inline size_t dtype_size(int dt) { return dt == kBF16 ? 2 : 4; }

// ---- GroupNorm ([rows, C] channels-last; statistics per frame and group) -------------------
constexpr int kStatRows = 64;  // rows summed by one block of the statistics kernel
inline int stat_splits(int rows_per_frame) { return (rows_per_frame + kStatRows - 1) / kStatRows; }

// partial[frame][split][c][2] = (sum, sum of squares) over the rows of the split.
hipError_t launch_gn_stats(hipStream_t s, int dt, const void* x, float* partial, int frames,
                           int rows_per_frame, int C);
// Combines per-channel partial sums of up to two sources (channels [0,CA) from A with weight wA
// per element, channels [CA, CA+CB) from B with weight wB: B is the half-resolution deep feature
// whose every element appears 4 times after 2x nearest upsampling) into per-frame, per-channel
// scale/shift:  y = x * scale + shift.  scale/shift: [frames][CA+CB].
hipError_t launch_gn_finalize(hipStream_t s, const float* partA, int CA, int splitsA, int rowsA, float wA,
                              const float* partB, int CB, int splitsB, int rowsB, float wB,
                              const float* gamma, const float* beta, int groups, float eps,
                              float* scale, float* shift, int frames);
// A spatial window of a frame, in pixels: the spatial block of a feature chunk. w == 0: the whole frame.
struct Win { int x0, y0, w, h; };

// ---- implicit-GEMM convolution / linear layers (MFMA) ---------------------------------------
struct ConvDesc {
  int dt;      // MFMA operand type = type of w (and of x unless x_f32)
  int x_f32;   // 1: x is fp32 in memory and is rounded to dt while it is staged
  int y_f32;   // 1: y is stored as fp32 (residual streams); res, when given, is always fp32
  int taps;    // 9 (3x3, zero padding 1) or 1 (per-row linear layer)
  int stride;  // 1 or 2 (taps == 9 only)
  int Cin, Cout;  // Cout here is the padded width of `w` rows, a multiple of the cout tile
  int Cout_store; // channels actually stored (<= Cout)
  const void* w;      // [Cout][taps*Cin], storage dtype
  const float* bias;  // [Cout] or nullptr
  // taps == 9: x is [frames][H][W][Cin]; y / res are [frames][H/stride][W/stride][Cout_store]
  int frames, H, W;
  // taps == 1: x is dense [rows][Cin]; y / res rows go through out_map
  int64_t rows;
  RowMap out_map;
  const void* x;
  const void* res;  // nullptr or same indexing as y
  void* y;
  // epilogue variant: 0 = channels-last store; 1 = planar store [frame][Cout_store][H][W]
  int planar_out;
};
hipError_t launch_conv(hipStream_t s, const ConvDesc& d);
// eps = conv3x3_{C -> C_lat}(SiLU(u * scale + shift)) + bias: u fp32 rows [frames][H*W][C], scale / shift
// [frames][C], w [32][9][C] (rows beyond C_lat zero), eps planar [frames][C_lat][H][W]. bf16 stages with
// C = 320, W % 16 == 0, H % 4 == 0 only: otherwise hipErrorNotSupported (use the general kernel).
// win: the pixels to compute (win.w == 0: the whole frame); x0, w multiples of 16 and y0, h of 4.
hipError_t launch_conv_out_tile(hipStream_t s, int dt, const void* u, const float* scale, const float* shift, const void* w,
                                const float* bias, void* out, int frames, int H, int W, int C, int C_lat, Win win);

// ---- fused-loader 3x3 stride-1 convolutions and linear layers (32x32 MFMA tiles) -------------
struct FusedDesc {
  int dt;        // MFMA operand type (type of w and of the LDS tiles)
  int y_f32;     // 1: y is an fp32 stream tensor; 0: y has the operand type
  int taps;      // 9: 3x3 conv over [frames][H][W][Cin]; 1: linear layer over rows
  int src;       // 0: x has the operand type, used as is
                 // 1: x is fp32, x * scale[f][c] + shift[f][c] (GroupNorm apply; taps == 9: general kernel only)
                 // 2: the same followed by SiLU (taps == 9); taps == 1: x is a planar image
                 //    [frames][Cs][H][W] of the operand type and row r gathers the 3x3 neighbourhood of
                 //    pixel r, k = channel * 9 + tap (a first convolution as a linear layer; Cin = 64 >= 9 Cs)
                 // 3: channels [0,Cs) from the fp32 skip x, [Cs,Cin) from x2 (operand type, half
                 //    resolution, nearest 2x upsampled), then as 2
  int Cin, Cs, Cout, Cout_store;
  const void* w;       // [Cout][taps*Cin]
  const void* w_tiles; // taps == 9, optional: the same weights in the order of launch_pack_conv_w_tiles (what the
                       // specialised-wavefront kernel reads; without it the general kernel runs)
  const void* w_frag;  // taps == 1: the same matrix in MFMA fragment order (launch_pack_lin_w), or nullptr
  const float* bias;   // [Cout] or nullptr
  int frames, H, W;    // taps == 9
  // Spatial window (the spatial block of a feature chunk): only the pixels [win_y0, win_y0 + win_h) x
  // [win_x0, win_x0 + win_w) of every frame are computed, by the tiles they belong to in the whole frame (a
  // window starts on a tile boundary and ends on one or at the frame's edge), with the halo read from the
  // neighbouring blocks of x; every output, and the partial sums of the tiles, are what the whole-frame launch
  // gives. win_w == 0: the whole frame.
  //   taps == 9: in pixels of the H x W image (tiles of 16 x 8).
  //   taps == 1: the dense rows of the launch are taken frame by frame as images of win_img_w pixels per row and
  //   win_img_t rows per frame; the launch walks the 32-row tiles of the window only. win_in / win_out say
  //   whether the input rows / the output rows (with residual, statistics and the V^T columns) are addressed by
  //   the row's place in the whole frame (1) or by its running number inside the launch (0).
  int win_x0, win_y0, win_w, win_h;
  int win_img_w, win_img_t, win_in, win_out;
  int64_t rows;        // taps == 1: x row of dense row r is in_map(r), y / res row is out_map(r);
  RowMap in_map, out_map;  //        scale/shift frame of row r is r / in_map.rows_per_seg
  const void* x;
  const void* x2;
  const float* scale;  // [frames][Cin]
  const float* shift;
  const void* res;     // fp32, indexed like y; nullptr if none; may equal y only when taps == 1
  void* y;
  int planar_out;      // 1: y is [frame][Cout_store][H][W] of the operand type (Cout = 32, zero-padded w)
  int act;             // taps == 1, src == 0 of a bf16 stage over dense rows, operand-type y, no residual only:
                       // 0 none; 1: y = gelu_tanh(x W^T + b); 2 (GEGLU): the rows of W come in alternating blocks of 32
                       // "value" and 32 "gate" channels and y, Cout / 2 wide, is value * gelu_tanh(gate)
  void* y2;            // taps == 1, src == 0, fp32 y of a bf16 stage over dense rows only: a copy of y rounded to the
                       // operand type (what the next layer contracts), or nullptr
  // taps == 1 only: output channels >= yt_from are not stored in y (whose rows then have yt_from
  // channels) but transposed into yt[frame][Cout - yt_from][yt_Tp] at column (t & ~63) + vcol(t & 63),
  // frame = r / yt_T, t = r % yt_T (the V^T layout of the spatial attention kernel). yt == nullptr: off.
  void* yt;
  int yt_from, yt_T, yt_Tp;
  // Optional (fp32 output only): per-channel sum and sum of squares of the stored output, for the
  // GroupNorm that reads it next, so that no separate pass over the tensor is needed.
  // stat[frame][split][Cout][2]; nullptr = off. taps == 9: `frame` counts from the first frame of the
  // launch and a split is one 32-pixel quarter of a workgroup tile (stat_splits = 4 * tiles per frame).
  // taps == 1: dense row r belongs to frame r / stat_rps and split (stat_off + r % stat_rps) / 32;
  // stat_rps and stat_off must be multiples of 32.
  float* stat;
  int stat_splits, stat_rps, stat_off;
  // taps == 1, optional: output channels [0, q_cols) are multiplied by q_scale before they are rounded
  // and stored (the softmax scale of spatial attention folded into q). q_cols == 0: off; a multiple of 32.
  float q_scale;
  int q_cols;
};
inline float attn_q_scale(int head_dim) { return 1.4426950408889634f / sqrtf((float)head_dim); }
// splits per frame of the statistics a 3x3 launch writes
inline int conv_stat_splits(int H, int W) { return 4 * ((W + 15) / 16) * ((H + 7) / 8); }
// The tiles (16 x 8 pixels) of a 3x3 launch's window: false if the window does not start on a tile boundary, or
// ends neither on one nor at the frame's edge.
inline bool conv_window_tiles(const FusedDesc& d, int* tx0, int* ty0, int* ntx, int* nty) {
  const int tiles_x = (d.W + 15) / 16, tiles_y = (d.H + 7) / 8;
  if (d.win_w == 0) { *tx0 = *ty0 = 0; *ntx = tiles_x; *nty = tiles_y; return true; }
  const int x1 = d.win_x0 + d.win_w, y1 = d.win_y0 + d.win_h;
  if (d.win_x0 < 0 || d.win_y0 < 0 || d.win_w <= 0 || d.win_h <= 0 || x1 > d.W || y1 > d.H) return false;
  if (d.win_x0 % 16 || d.win_y0 % 8 || (x1 % 16 && x1 != d.W) || (y1 % 8 && y1 != d.H)) return false;
  *tx0 = d.win_x0 / 16; *ty0 = d.win_y0 / 8;
  *ntx = (x1 + 15) / 16 - *tx0; *nty = (y1 + 7) / 8 - *ty0;
  return true;
}
hipError_t launch_fused(hipStream_t s, const FusedDesc& d);
// taps == 9 of a bf16 stage with specialised wavefronts (lc_convws.hip): the same results as the general
// kernel bit for bit; hipErrorNotSupported for shapes it does not cover. launch_fused tries it first.
hipError_t launch_conv_ws(hipStream_t s, const FusedDesc& d);
// taps == 1, src == 0 of a bf16 stage (lc_lin2.hip: 256 x 160 tiles, operands streamed through a ring of LDS stages);
// hipErrorNotSupported for widths it does not cover, never because of the rows. launch_fused tries it first.
hipError_t launch_lin2(hipStream_t s, const FusedDesc& d);
// taps == 1 with the weights resident in registers (needs w_frag); hipErrorNotSupported for shapes it does not cover
hipError_t launch_linear(hipStream_t s, const FusedDesc& d);
inline hipError_t launch_linear_any(hipStream_t s, const FusedDesc& d) {
  const hipError_t e = launch_linear(s, d);
  return e == hipErrorNotSupported ? launch_fused(s, d) : e;
}

// ---- attention cores -----------------------------------------------------------------------
// Spatial attention core. qk: rows [frames*T] of stride ldq with q at column 0 and k at column C;
// vt: V transposed [frames][C][Tp], token t at column (t & ~63) + vcol(t & 63), Tp a multiple of 64;
// out [frames*T][C]; queries [q0,q1) of every frame. q_prescaled: the q columns hold q * log2(e) / sqrt(d)
// (FusedDesc::q_scale of the projection that wrote them) instead of q.
inline int attn_tp(int T) { return (T + 63) / 64 * 64; }
hipError_t launch_spatial_attention(hipStream_t s, int dt, const void* qk, int ldq, const void* vt, int Tp, void* out,
                                    int frames, int T, int heads, int d, int q0, int q1, int q_prescaled);
// The same for a window of queries: nq queries, number i being token q0 + (i / qw) * qstride + i % qw (rows of qw
// tokens out of image rows of qstride tokens). Each query's result does not depend on which others share its launch.
hipError_t launch_spatial_attention_window(hipStream_t s, int dt, const void* qk, int ldq, const void* vt, int Tp, void* out,
                                           int frames, int T, int heads, int d, int q0, int nq, int qw, int qstride,
                                           int q_prescaled);
// Cross-attention core: queries q[frames*Tq] (row stride ldq; head h at column h*d) against the keys k[(frames /
// kv_div)*Tk] (row stride ldk) and values vt[(frames / kv_div)][C][Tp] (layout as above) that every kv_div consecutive
// frames share; out [frames*Tq][C]. Tk need not be a multiple of anything; Tp >= Tk, a multiple of 64.
hipError_t launch_cross_attention(hipStream_t s, int dt, const void* q, int ldq, const void* k, int ldk, const void* vt, int Tp,
                                  void* out, int frames, int Tq, int Tk, int kv_div, int heads, int d);
// vt from plain value rows v[frames*T][C] of stride ldv
hipError_t launch_make_vt(hipStream_t s, int dt, const void* v, int ldv, void* vt, int frames, int T, int Tp, int C);
// qkv [(B*F)*P][3C] frame-major -> out same rows x C; attention over the F frames.
hipError_t launch_temporal_attention(hipStream_t s, int dt, const void* qkv, void* out, int B, int F, int P,
                                     int heads, int d);

// ---- small kernels -------------------------------------------------------------------------
// h[frames*H*W][C] (fp32) = conv3x3(x[frames][Cl][H][W] of type dt); w_packed float [Cl*9][C], bias float [C].
// conv_in for bf16 stages whose image rows are whole 32-pixel segments, with the GroupNorm partial sums of its
// output (lc_conv.hip); hipErrorNotSupported otherwise
// win: the pixels to compute (win.w == 0: the whole frame); x0 and w multiples of 32.
hipError_t launch_conv_in_tile(hipStream_t s, int dt, const void* x, const void* wp, const float* bias, float* y, float* stat,
                               int frames, int H, int W, int Cl, int C, Win win);
hipError_t launch_conv_in(hipStream_t s, int dt, const void* x, void* h, int frames, int H, int W, int Cl, int C,
                          const float* w_packed, const float* bias);
// planar [frames][C][HW] <-> channels-last [frames][HW][C]
hipError_t launch_planar_to_cl(hipStream_t s, int dt, const void* src, void* dst, int frames, int C, int HW);
hipError_t launch_cl_to_planar(hipStream_t s, int dt, const void* src, void* dst, int frames, int C, int HW);
// weight packing (run once at load time)
hipError_t launch_pack_conv_w(hipStream_t s, int dt, const void* w, void* packed, int Cout, int Cin, int taps,
                              int Cout_padded);  // [Cout][Cin][taps] -> [Cout_padded][taps][Cin]
hipError_t launch_pack_conv_in_w(hipStream_t s, int dt, const void* w, float* packed, int C, int Cl);
// packed [Cout][9*Cin] -> tiles [Cout/160][9*Cin/64][160][64] (bf16; Cout % 160 == 0, Cin % 64 == 0)
hipError_t launch_pack_conv_w_tiles(hipStream_t s, int dt, const void* w, void* tiles, int Cout, int Cin);
// w[Cout][Cin] -> MFMA fragment order for launch_linear
hipError_t launch_pack_lin_w(hipStream_t s, int dt, const void* w, void* out, int Cout, int Cin);
// w[Cout][Cin] -> out[Cout][Cin_padded] with zero columns appended
hipError_t launch_pad_rows(hipStream_t s, int dt, const void* w, void* out, int Cout, int Cin, int Cin_padded);
hipError_t launch_to_f32(hipStream_t s, int dt, const void* src, float* dst, int n, int n_padded);
// nearest 2x upsampling of fp32 rows [frames][H][W][C] -> [frames][2H][2W][C] (C % 4 == 0)
hipError_t launch_up2_rows(hipStream_t s, const float* src, float* dst, int frames, int H, int W, int C);
hipError_t launch_fill_f32(hipStream_t s, float* dst, int64_t n, float v);
hipError_t launch_copy_rows(hipStream_t s, int dt, const void* src, void* dst, int64_t elems);

}  // namespace lc

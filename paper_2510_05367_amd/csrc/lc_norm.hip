// GroupNorm / SiLU / skip-concat bandwidth kernels on channels-last activations.
//
// GroupNorm over a frame is done as: (1) per-channel partial sums over blocks of rows (one 16-byte
// packet per lane, coalesced over the channel axis), (2) a tiny per-frame kernel that folds the
// partials into per-channel scale/shift, (3) an elementwise apply fused with SiLU (and, for the up
// block, with nearest 2x upsampling of the cached deep feature and the channel concatenation
// U_m = Concat(D_m, U_{m+1}) of the paper's "Feature Calculation" paragraph). The split geometry
// depends only on the frame size, never on the chunking, so chunked and unchunked runs reduce in
// the same order.
#include "lc_internal.h"

namespace lc {

// ---------------------------------------------------------------------------------------------
template <class T>
__global__ __launch_bounds__(256) void gn_stats_kernel(const T* __restrict__ x, float* __restrict__ partial,
                                                       int rows_per_frame, int C) {
  constexpr int VEC = Vec16<T>::N;
  __shared__ float red[2][256 * VEC];
  const int cv = C / VEC;
  const int R = 256 / cv;
  const int split = blockIdx.x, frame = blockIdx.y, splits = gridDim.x;
  const int tid = threadIdx.x;
  const int cvec = tid % cv, rsub = tid / cv;
  float s[VEC], q[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) s[i] = q[i] = 0.f;
  const int r0 = split * kStatRows;
  const int r1 = min(r0 + kStatRows, rows_per_frame);
  if (rsub < R) {
    const T* base = x + ((int64_t)frame * rows_per_frame) * C + cvec * VEC;
    for (int r = r0 + rsub; r < r1; r += R) {
      Vec16<T> v = load16(base + (int64_t)r * C);
#pragma unroll
      for (int i = 0; i < VEC; ++i) {
        float f = v.get(i);
        s[i] += f;
        q[i] = fmaf(f, f, q[i]);
      }
    }
  }
#pragma unroll
  for (int i = 0; i < VEC; ++i) {
    red[0][tid * VEC + i] = s[i];
    red[1][tid * VEC + i] = q[i];
  }
  __syncthreads();
  // channel c of row-slot j sits at red[.][(j*cv)*VEC + c]
  for (int c = tid; c < C; c += 256) {
    float ss = 0.f, qq = 0.f;
    for (int j = 0; j < R; ++j) {
      ss += red[0][j * cv * VEC + c];
      qq += red[1][j * cv * VEC + c];
    }
    float* p = partial + (((int64_t)frame * splits + split) * C + c) * 2;
    p[0] = ss;
    p[1] = qq;
  }
}

hipError_t launch_gn_stats(hipStream_t s, int dt, const void* x, float* partial, int frames,
                           int rows_per_frame, int C) {
  if (frames <= 0) return hipSuccess;
  dim3 grid(stat_splits(rows_per_frame), frames);
  if (dt == kBF16)
    gn_stats_kernel<bf16_t><<<grid, 256, 0, s>>>((const bf16_t*)x, partial, rows_per_frame, C);
  else
    gn_stats_kernel<float><<<grid, 256, 0, s>>>((const float*)x, partial, rows_per_frame, C);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
constexpr int kMaxNormC = 2048;

__global__ __launch_bounds__(256) void gn_finalize_kernel(const float* __restrict__ partA, int CA, int splitsA,
                                                          int rowsA, float wA, const float* __restrict__ partB,
                                                          int CB, int splitsB, int rowsB, float wB,
                                                          const float* __restrict__ gamma,
                                                          const float* __restrict__ beta, int groups, float eps,
                                                          float* __restrict__ scale, float* __restrict__ shift) {
  __shared__ double csum[kMaxNormC], csq[kMaxNormC];
  __shared__ float gmean[256], grstd[256];
  const int f = blockIdx.x, tid = threadIdx.x;
  const int Ct = CA + CB;
  for (int c = tid; c < Ct; c += 256) {
    double ss = 0.0, qq = 0.0;
    if (c < CA) {
      const float* p = partA + ((int64_t)f * splitsA * CA + c) * 2;
      for (int k = 0; k < splitsA; ++k) {
        ss += (double)p[(int64_t)k * CA * 2];
        qq += (double)p[(int64_t)k * CA * 2 + 1];
      }
      ss *= wA;
      qq *= wA;
    } else {
      const float* p = partB + ((int64_t)f * splitsB * CB + (c - CA)) * 2;
      for (int k = 0; k < splitsB; ++k) {
        ss += (double)p[(int64_t)k * CB * 2];
        qq += (double)p[(int64_t)k * CB * 2 + 1];
      }
      ss *= wB;
      qq *= wB;
    }
    csum[c] = ss;
    csq[c] = qq;
  }
  __syncthreads();
  const int cg = Ct / groups;
  for (int g = tid; g < groups; g += 256) {
    double ss = 0.0, qq = 0.0, cnt = 0.0;
    for (int c = g * cg; c < (g + 1) * cg; ++c) {
      ss += csum[c];
      qq += csq[c];
      cnt += (c < CA) ? (double)rowsA * wA : (double)rowsB * wB;
    }
    double mean = ss / cnt;
    double var = qq / cnt - mean * mean;
    if (var < 0.0) var = 0.0;
    gmean[g] = (float)mean;
    grstd[g] = (float)(1.0 / sqrt(var + (double)eps));
  }
  __syncthreads();
  for (int c = tid; c < Ct; c += 256) {
    int g = c / cg;
    float a = grstd[g] * gamma[c];
    scale[(int64_t)f * Ct + c] = a;
    shift[(int64_t)f * Ct + c] = fmaf(-gmean[g], a, beta[c]);
  }
}

hipError_t launch_gn_finalize(hipStream_t s, const float* partA, int CA, int splitsA, int rowsA, float wA,
                              const float* partB, int CB, int splitsB, int rowsB, float wB,
                              const float* gamma, const float* beta, int groups, float eps, float* scale,
                              float* shift, int frames) {
  if (frames <= 0) return hipSuccess;
  if (CA + CB > kMaxNormC || groups > 256) return hipErrorInvalidValue;
  gn_finalize_kernel<<<frames, 256, 0, s>>>(partA, CA, splitsA, rowsA, wA, partB, CB, splitsB, rowsB, wB, gamma,
                                            beta, groups, eps, scale, shift);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
template <class XT, class YT, bool SILU>
__global__ __launch_bounds__(256) void gn_apply_kernel(const XT* __restrict__ x, RowMap map, YT* __restrict__ y,
                                                       int64_t rows, int C, const float* __restrict__ scale,
                                                       const float* __restrict__ shift) {
  constexpr int VEC = sizeof(XT) == 4 && sizeof(YT) == 4 ? 4 : 8;  // channels per thread
  const int cv = C / VEC;
  const int64_t total = rows * cv;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int64_t r = i / cv;
  const int c0 = (int)(i - r * cv) * VEC;
  const int64_t f = r / map.rows_per_seg;
  float v[VEC], a[VEC], b[VEC];
  load_f<XT, VEC>(x + map(r) * C + c0, v);
  load_f<float, VEC>(scale + f * C + c0, a);
  load_f<float, VEC>(shift + f * C + c0, b);
#pragma unroll
  for (int k = 0; k < VEC; ++k) {
    const float t = fmaf(v[k], a[k], b[k]);
    v[k] = SILU ? silu_f(t) : t;
  }
  store_f<YT, VEC>(y + r * C + c0, v);
}

hipError_t launch_gn_apply(hipStream_t s, int xdt, int ydt, const void* x, RowMap map, void* y, int64_t rows, int C,
                           const float* scale, const float* shift, int silu) {
  if (rows <= 0) return hipSuccess;
  const int vec = (xdt == kF32 && ydt == kF32) ? 4 : 8;
  const int64_t total = rows * (C / vec);
  const unsigned blocks = (unsigned)((total + 255) / 256);
#define LC_GO(XT, YT, S) \
  gn_apply_kernel<XT, YT, S><<<blocks, 256, 0, s>>>((const XT*)x, map, (YT*)y, rows, C, scale, shift)
#define LC_GO2(XT, YT) do { if (silu) LC_GO(XT, YT, true); else LC_GO(XT, YT, false); } while (0)
  if (xdt == kF32 && ydt == kF32) LC_GO2(float, float);
  else if (xdt == kF32 && ydt == kBF16) LC_GO2(float, bf16_t);
  else if (xdt == kBF16 && ydt == kBF16) LC_GO2(bf16_t, bf16_t);
  else return hipErrorInvalidValue;
#undef LC_GO2
#undef LC_GO
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// ST: type of the skip feature (the fp32 residual stream), T: type of the cached deep feature and
// of the normalised output.
template <class ST, class T>
__global__ __launch_bounds__(256) void concat_apply_kernel(const ST* __restrict__ skip, const T* __restrict__ deep,
                                                           T* __restrict__ catn, int frames, int H, int W, int C,
                                                           int Cd, const float* __restrict__ scale,
                                                           const float* __restrict__ shift) {
  constexpr int VEC = sizeof(T) == 4 ? 4 : 8;
  const int Ct = C + Cd;
  const int cv = Ct / VEC;
  const int64_t total = (int64_t)frames * H * W * cv;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int64_t r = i / cv;  // pixel row (frame-major)
  const int c0 = (int)(i - r * cv) * VEC;
  const int hw = H * W;
  const int f = (int)(r / hw);
  const int p = (int)(r - (int64_t)f * hw);
  float v[VEC], a[VEC], b[VEC];
  if (c0 < C) {
    load_f<ST, VEC>(skip + r * C + c0, v);
  } else {
    const int yy = p / W, xx = p - yy * W;
    const int64_t dr = ((int64_t)f * (H / 2) + (yy >> 1)) * (W / 2) + (xx >> 1);
    load_f<T, VEC>(deep + dr * Cd + (c0 - C), v);
  }
  load_f<float, VEC>(scale + (int64_t)f * Ct + c0, a);
  load_f<float, VEC>(shift + (int64_t)f * Ct + c0, b);
#pragma unroll
  for (int k = 0; k < VEC; ++k) v[k] = silu_f(fmaf(v[k], a[k], b[k]));
  store_f<T, VEC>(catn + r * Ct + c0, v);
}

hipError_t launch_concat_apply(hipStream_t s, int dt, const void* skip, const void* deep, void* catn, int frames,
                               int H, int W, int C, int Cd, const float* scale, const float* shift) {
  if (frames <= 0) return hipSuccess;
  const int vec = dt == kBF16 ? 8 : 4;
  const int64_t total = (int64_t)frames * H * W * ((C + Cd) / vec);
  const unsigned blocks = (unsigned)((total + 255) / 256);
  if (dt == kBF16)
    concat_apply_kernel<float, bf16_t><<<blocks, 256, 0, s>>>((const float*)skip, (const bf16_t*)deep, (bf16_t*)catn,
                                                              frames, H, W, C, Cd, scale, shift);
  else
    concat_apply_kernel<float, float><<<blocks, 256, 0, s>>>((const float*)skip, (const float*)deep, (float*)catn,
                                                             frames, H, W, C, Cd, scale, shift);
  return hipGetLastError();
}

}  // namespace lc

// GroupNorm statistics on channels-last activations.
//
// GroupNorm over a frame is done as: (1) per-channel partial sums over blocks of rows (one 16-byte
// packet per lane, coalesced over the channel axis), (2) a tiny kernel that folds the partials of
// whole groups into per-frame, per-channel scale/shift. The apply step (with SiLU, and for the up
// block with the 2x upsampling and skip-concatenation) lives in the loaders of the kernels that
// consume the normalised tensor. The split geometry depends only on the frame size, never on the
// chunking, so chunked and unchunked runs reduce in the same order.
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
// One workgroup folds the partial sums of `gpb` whole groups of one frame: 64 channel lanes x 4
// split lanes, so that the loads over the splits are independent and few per thread.
constexpr int kFinalCh = 512;  // channels one workgroup can own

__global__ __launch_bounds__(256) void gn_finalize_kernel(const float* __restrict__ partA, int CA, int splitsA,
                                                          int rowsA, float wA, const float* __restrict__ partB,
                                                          int CB, int splitsB, int rowsB, float wB,
                                                          const float* __restrict__ gamma,
                                                          const float* __restrict__ beta, int groups, int gpb,
                                                          float eps, float* __restrict__ scale,
                                                          float* __restrict__ shift) {
  __shared__ double csum[4][kFinalCh], csq[4][kFinalCh];
  __shared__ float gmean[kFinalCh], grstd[kFinalCh];
  const int f = blockIdx.y, tid = threadIdx.x;
  const int Ct = CA + CB, cg = Ct / groups;
  const int g0 = blockIdx.x * gpb, g1 = min(g0 + gpb, groups);
  const int c_lo = g0 * cg, nch = (g1 - g0) * cg;
  const int cl = tid & 63, sl = tid >> 6;
  for (int j = cl; j < nch; j += 64) {
    const int c = c_lo + j;
    const bool inA = c < CA;
    const int Cs = inA ? CA : CB, splits = inA ? splitsA : splitsB;
    const float* p = (inA ? partA + ((int64_t)f * splitsA * CA + c) * 2
                          : partB + ((int64_t)f * splitsB * CB + (c - CA)) * 2);
    double ss = 0.0, qq = 0.0;
#pragma unroll 8
    for (int k = sl; k < splits; k += 4) {
      const float2 v = *reinterpret_cast<const float2*>(p + (int64_t)k * Cs * 2);
      ss += (double)v.x;
      qq += (double)v.y;
    }
    csum[sl][j] = ss;
    csq[sl][j] = qq;
  }
  __syncthreads();
  for (int g = tid; g < g1 - g0; g += 256) {
    double ss = 0.0, qq = 0.0, cnt = 0.0;
    for (int j = g * cg; j < (g + 1) * cg; ++j) {
      const bool inA = c_lo + j < CA;
      const double w = inA ? (double)wA : (double)wB;
      // fixed order: split lanes 0..3, then channels
      ss += w * (((csum[0][j] + csum[1][j]) + csum[2][j]) + csum[3][j]);
      qq += w * (((csq[0][j] + csq[1][j]) + csq[2][j]) + csq[3][j]);
      cnt += inA ? (double)rowsA * wA : (double)rowsB * wB;
    }
    const double mean = ss / cnt;
    double var = qq / cnt - mean * mean;
    if (var < 0.0) var = 0.0;
    gmean[g] = (float)mean;
    grstd[g] = (float)(1.0 / sqrt(var + (double)eps));
  }
  __syncthreads();
  for (int j = tid; j < nch; j += 256) {
    const int c = c_lo + j, g = j / cg;
    const float a = grstd[g] * gamma[c];
    scale[(int64_t)f * Ct + c] = a;
    shift[(int64_t)f * Ct + c] = fmaf(-gmean[g], a, beta[c]);
  }
}

hipError_t launch_gn_finalize(hipStream_t s, const float* partA, int CA, int splitsA, int rowsA, float wA,
                              const float* partB, int CB, int splitsB, int rowsB, float wB,
                              const float* gamma, const float* beta, int groups, float eps, float* scale,
                              float* shift, int frames) {
  if (frames <= 0) return hipSuccess;
  const int cg = (CA + CB) / groups;
  if (cg > kFinalCh) return hipErrorInvalidValue;
  int gpb = 64 / cg;  // about 64 channels per workgroup
  if (gpb < 1) gpb = 1;
  dim3 grid((groups + gpb - 1) / gpb, frames);
  gn_finalize_kernel<<<grid, 256, 0, s>>>(partA, CA, splitsA, rowsA, wA, partB, CB, splitsB, rowsB, wB, gamma, beta,
                                          groups, gpb, eps, scale, shift);
  return hipGetLastError();
}

}  // namespace lc

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
  // a workgroup covers up to 256 packets of the channel axis; wider tensors take gridDim.z of them side by side
  const int cv0 = blockIdx.z * 256;
  const int cv = min(C / VEC - cv0, 256);
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
    const T* base = x + ((int64_t)frame * rows_per_frame) * C + (cv0 + cvec) * VEC;
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
  for (int c = tid; c < cv * VEC; c += 256) {
    float ss = 0.f, qq = 0.f;
    for (int j = 0; j < R; ++j) {
      ss += red[0][j * cv * VEC + c];
      qq += red[1][j * cv * VEC + c];
    }
    float* p = partial + (((int64_t)frame * splits + split) * C + cv0 * VEC + c) * 2;
    p[0] = ss;
    p[1] = qq;
  }
}

hipError_t launch_gn_stats(hipStream_t s, int dt, const void* x, float* partial, int frames,
                           int rows_per_frame, int C) {
  if (frames <= 0) return hipSuccess;
  const int vec = dt == kBF16 ? 8 : 4;
  if (C <= 0 || C % vec) return hipErrorInvalidValue;
  dim3 grid(stat_splits(rows_per_frame), frames, (C / vec + 255) / 256);
  if (dt == kBF16)
    gn_stats_kernel<bf16_t><<<grid, 256, 0, s>>>((const bf16_t*)x, partial, rows_per_frame, C);
  else
    gn_stats_kernel<float><<<grid, 256, 0, s>>>((const float*)x, partial, rows_per_frame, C);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// One workgroup folds the partial sums of one group of one frame. The group's (split, channel) cells
// are dealt to the 256 threads in a fixed pattern, each thread adds its cells in double precision in
// a fixed order, and the 256 partial results are folded by a fixed tree: the result does not depend
// on scheduling. The tensor may be the concatenation of two sources (A then B along the channels)
// with different row counts per frame; `w` weighs a source's rows (the 2x-upsampled deep feature
// counts each of its pixels four times).
// At most 32 vector registers: the 3x3 convolution kernel leaves that many free on every SIMD (two
// wavefronts of 240), so when a step runs its chunks on two streams this kernel starts beside the other
// stream's convolution instead of waiting for a compute unit to drain.
__global__ __launch_bounds__(256) __attribute__((amdgpu_num_vgpr(32))) void gn_finalize_kernel(const float* __restrict__ partA, int CA, int splitsA,
                                                          int rowsA, float wA, const float* __restrict__ partB,
                                                          int CB, int splitsB, int rowsB, float wB,
                                                          const float* __restrict__ gamma,
                                                          const float* __restrict__ beta, int groups, float eps,
                                                          float* __restrict__ scale, float* __restrict__ shift) {
  __shared__ double rs[256], rq[256];
  __shared__ float s_mean, s_rstd;
  const int g = blockIdx.x, f = blockIdx.y, tid = threadIdx.x;
  const int Ct = CA + CB, cg = Ct / groups;
  const int c_lo = g * cg;
  // channels of the group that lie in A / in B
  const int nA = max(0, min(c_lo + cg, CA) - c_lo), nB = cg - nA;
  const int cellsA = nA * splitsA, cellsB = nB * splitsB;
  double ss = 0.0, qq = 0.0;
  // cells i = tid, tid + 256, ... in batches of kBatch: all loads of a batch are requested before the first
  // is added (one at a time, every cell paid a trip to L2: that was most of this kernel's time); the order
  // of the additions is the same either way
  constexpr int kBatch = 3;
  auto fold = [&](const float* part, int C, int splits, int n, int c_first, int cells, float w) {
    for (int i0 = tid; i0 < cells; i0 += 256 * kBatch) {
      float2 v[kBatch];
#pragma unroll
      for (int j = 0; j < kBatch; ++j) {
        const int i = min(i0 + 256 * j, cells - 1);  // clamped: a valid cell, not added if beyond the end
        const int k = i / n, c = c_first + (i - k * n);
        v[j] = *reinterpret_cast<const float2*>(part + (((int64_t)f * splits + k) * C + c) * 2);
      }
#pragma unroll
      for (int j = 0; j < kBatch; ++j) {
        if (i0 + 256 * j < cells) {
          ss += (double)w * (double)v[j].x;
          qq += (double)w * (double)v[j].y;
        }
      }
    }
  };
  if (cellsA > 0) fold(partA, CA, splitsA, nA, c_lo, cellsA, wA);
  if (cellsB > 0) fold(partB, CB, splitsB, nB, max(c_lo, CA) - CA, cellsB, wB);
  rs[tid] = ss;
  rq[tid] = qq;
  __syncthreads();
  for (int m = 128; m > 0; m >>= 1) {
    if (tid < m) {
      rs[tid] += rs[tid + m];
      rq[tid] += rq[tid + m];
    }
    __syncthreads();
  }
  if (tid == 0) {
    const double cnt = (double)nA * rowsA * wA + (double)nB * rowsB * wB;
    const double mean = rs[0] / cnt;
    double var = rq[0] / cnt - mean * mean;
    if (var < 0.0) var = 0.0;
    s_mean = (float)mean;
    s_rstd = (float)(1.0 / sqrt(var + (double)eps));
  }
  __syncthreads();
  for (int j = tid; j < cg; j += 256) {
    const int c = c_lo + j;
    const float a = s_rstd * gamma[c];
    scale[(int64_t)f * Ct + c] = a;
    shift[(int64_t)f * Ct + c] = fmaf(-s_mean, a, beta[c]);
  }
}

hipError_t launch_gn_finalize(hipStream_t s, const float* partA, int CA, int splitsA, int rowsA, float wA,
                              const float* partB, int CB, int splitsB, int rowsB, float wB,
                              const float* gamma, const float* beta, int groups, float eps, float* scale,
                              float* shift, int frames) {
  if (frames <= 0) return hipSuccess;
  if (groups <= 0 || (CA + CB) % groups) return hipErrorInvalidValue;
  dim3 grid(groups, frames);
  gn_finalize_kernel<<<grid, 256, 0, s>>>(partA, CA, splitsA, rowsA, wA, partB, CB, splitsB, rowsB, wB, gamma, beta,
                                          groups, eps, scale, shift);
  return hipGetLastError();
}

}  // namespace lc

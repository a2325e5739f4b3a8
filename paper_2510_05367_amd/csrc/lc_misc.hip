// Small kernels: the C_lat -> C input convolution (write-bound), layout changes between the
// public planar order [frame][C][H*W] and the internal channels-last order, weight packing.
#include "lc_internal.h"

namespace lc {

// ---------------------------------------------------------------------------------------------
// conv_in: 3x3, zero padding, C_lat (<= 16) input channels, fp32 output. One thread = one pixel x 8
// output channels; the packed weights [C_lat*9][C] are read through the vector cache.
template <class T>
__global__ __launch_bounds__(256) void conv_in_kernel(const T* __restrict__ x, float* __restrict__ h, int frames, int H,
                                                      int W, int Cl, int C, const float* __restrict__ wp,
                                                      const float* __restrict__ bias) {
  constexpr int VEC = 8;
  const int cv = C / VEC;
  const int64_t total = (int64_t)frames * H * W * cv;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int64_t pix = i / cv;
  const int c0 = (int)(i - pix * cv) * VEC;
  const int hw = H * W;
  const int f = (int)(pix / hw);
  const int p = (int)(pix - (int64_t)f * hw);
  const int yy = p / W, xx = p - yy * W;
  float acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = bias[c0 + e];
  for (int cl = 0; cl < Cl; ++cl) {
    const T* plane = x + ((int64_t)f * Cl + cl) * hw;
#pragma unroll
    for (int a = 0; a < 3; ++a) {
      const int iy = yy + a - 1;
#pragma unroll
      for (int b = 0; b < 3; ++b) {
        const int ix = xx + b - 1;
        if (iy < 0 || iy >= H || ix < 0 || ix >= W) continue;
        const float v = to_f32(plane[iy * W + ix]);
        const float* wr = wp + (int64_t)((cl * 3 + a) * 3 + b) * C + c0;
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] = fmaf(v, wr[e], acc[e]);
      }
    }
  }
  store_f<float, VEC>(h + pix * C + c0, acc);
}

hipError_t launch_conv_in(hipStream_t s, int dt, const void* x, void* h, int frames, int H, int W, int Cl, int C,
                          const float* w_packed, const float* bias) {
  if (frames <= 0) return hipSuccess;
  const int64_t total = (int64_t)frames * H * W * (C / 8);
  const unsigned blocks = (unsigned)((total + 255) / 256);
  if (dt == kBF16)
    conv_in_kernel<bf16_t><<<blocks, 256, 0, s>>>((const bf16_t*)x, (float*)h, frames, H, W, Cl, C, w_packed, bias);
  else
    conv_in_kernel<float><<<blocks, 256, 0, s>>>((const float*)x, (float*)h, frames, H, W, Cl, C, w_packed, bias);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Batched 2-D transpose: src [f][R][S] -> dst [f][S][R] through a 32x33 LDS tile.
template <class T>
__global__ __launch_bounds__(256) void transpose_kernel(const T* __restrict__ src, T* __restrict__ dst, int R, int S) {
  __shared__ T tile[32][33];
  const int f = blockIdx.z;
  const int s0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const T* sp = src + (int64_t)f * R * S;
  T* dp = dst + (int64_t)f * R * S;
  for (int k = ty; k < 32; k += 8)
    if (r0 + k < R && s0 + tx < S) tile[k][tx] = sp[(int64_t)(r0 + k) * S + s0 + tx];
  __syncthreads();
  for (int k = ty; k < 32; k += 8)
    if (s0 + k < S && r0 + tx < R) dp[(int64_t)(s0 + k) * R + r0 + tx] = tile[tx][k];
}

template <class T>
static hipError_t transpose(hipStream_t s, const void* src, void* dst, int frames, int R, int S) {
  if (frames <= 0) return hipSuccess;
  dim3 grid((S + 31) / 32, (R + 31) / 32, frames);
  transpose_kernel<T><<<grid, 256, 0, s>>>((const T*)src, (T*)dst, R, S);
  return hipGetLastError();
}
hipError_t launch_planar_to_cl(hipStream_t s, int dt, const void* src, void* dst, int frames, int C, int HW) {
  return dt == kBF16 ? transpose<uint16_t>(s, src, dst, frames, C, HW) : transpose<uint32_t>(s, src, dst, frames, C, HW);
}
hipError_t launch_cl_to_planar(hipStream_t s, int dt, const void* src, void* dst, int frames, int C, int HW) {
  return dt == kBF16 ? transpose<uint16_t>(s, src, dst, frames, HW, C) : transpose<uint32_t>(s, src, dst, frames, HW, C);
}

// ---------------------------------------------------------------------------------------------
template <class T>
__global__ void pack_conv_w_kernel(const T* __restrict__ w, T* __restrict__ packed, int Cout, int Cin, int taps,
                                   int Cout_padded) {
  const int64_t total = (int64_t)Cout_padded * taps * Cin;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int ci = (int)(i % Cin);
  const int tap = (int)((i / Cin) % taps);
  const int co = (int)(i / ((int64_t)Cin * taps));
  packed[i] = co < Cout ? w[((int64_t)co * Cin + ci) * taps + tap] : from_f32<T>(0.f);
}
hipError_t launch_pack_conv_w(hipStream_t s, int dt, const void* w, void* packed, int Cout, int Cin, int taps,
                              int Cout_padded) {
  const int64_t total = (int64_t)Cout_padded * taps * Cin;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  if (dt == kBF16)
    pack_conv_w_kernel<bf16_t><<<blocks, 256, 0, s>>>((const bf16_t*)w, (bf16_t*)packed, Cout, Cin, taps, Cout_padded);
  else
    pack_conv_w_kernel<float><<<blocks, 256, 0, s>>>((const float*)w, (float*)packed, Cout, Cin, taps, Cout_padded);
  return hipGetLastError();
}

// [Cout][9 * Cin] (tap-major rows, as launch_pack_conv_w writes them) -> tiles[Cout / 160][step][160][64],
// step = slab * 9 + tap: the 160 x 64 block a workgroup of the specialised-wavefront conv kernel moves to LDS
// in one step is then 20 KB of contiguous memory instead of 160 pieces of 128 bytes a whole row apart.
__global__ void pack_conv_w_tiles_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ tiles, int Cout, int Cin) {
  const int64_t total = (int64_t)Cout * 9 * Cin;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int nsteps = 9 * (Cin / 64);
  const int c = (int)(i % 64);
  const int r = (int)((i / 64) % 160);
  const int step = (int)((i / (64 * 160)) % nsteps);
  const int cb = (int)(i / ((int64_t)64 * 160 * nsteps));
  const int slab = step / 9, tap = step - slab * 9;
  tiles[i] = w[(int64_t)(cb * 160 + r) * (9 * Cin) + tap * Cin + slab * 64 + c];
}
hipError_t launch_pack_conv_w_tiles(hipStream_t s, int dt, const void* w, void* tiles, int Cout, int Cin) {
  if (dt != kBF16 || Cout % 160 != 0 || Cin % 64 != 0) return hipErrorInvalidValue;
  const int64_t total = (int64_t)Cout * 9 * Cin;
  pack_conv_w_tiles_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>((const bf16_t*)w, (bf16_t*)tiles, Cout, Cin);
  return hipGetLastError();
}

template <class T>
__global__ void pack_conv_in_w_kernel(const T* __restrict__ w, float* __restrict__ packed, int C, int Cl) {
  const int total = C * Cl * 9;
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int c = i % C;
  const int k = i / C;  // cl*9 + tap
  packed[i] = to_f32(w[(int64_t)c * Cl * 9 + k]);
}
hipError_t launch_pack_conv_in_w(hipStream_t s, int dt, const void* w, float* packed, int C, int Cl) {
  const unsigned blocks = (unsigned)((C * Cl * 9 + 255) / 256);
  if (dt == kBF16) pack_conv_in_w_kernel<bf16_t><<<blocks, 256, 0, s>>>((const bf16_t*)w, packed, C, Cl);
  else pack_conv_in_w_kernel<float><<<blocks, 256, 0, s>>>((const float*)w, packed, C, Cl);
  return hipGetLastError();
}

template <class T>
__global__ void to_f32_kernel(const T* __restrict__ src, float* __restrict__ dst, int n, int n_padded) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n_padded) dst[i] = i < n ? to_f32(src[i]) : 0.f;
}
hipError_t launch_to_f32(hipStream_t s, int dt, const void* src, float* dst, int n, int n_padded) {
  const unsigned blocks = (unsigned)((n_padded + 255) / 256);
  if (dt == kBF16) to_f32_kernel<bf16_t><<<blocks, 256, 0, s>>>((const bf16_t*)src, dst, n, n_padded);
  else to_f32_kernel<float><<<blocks, 256, 0, s>>>((const float*)src, dst, n, n_padded);
  return hipGetLastError();
}

__global__ void copy_kernel(const uint32_t* __restrict__ src, uint32_t* __restrict__ dst, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = src[i];
}
hipError_t launch_copy_rows(hipStream_t s, int dt, const void* src, void* dst, int64_t elems) {
  const int64_t words = elems * (int64_t)dtype_size(dt) / 4;
  if (words <= 0) return hipSuccess;
  copy_kernel<<<(unsigned)((words + 255) / 256), 256, 0, s>>>((const uint32_t*)src, (uint32_t*)dst, words);
  return hipGetLastError();
}

// Nearest 2x upsampling of fp32 rows: dst[f][2H][2W][C] from src[f][H][W][C], 16 bytes per thread.
__global__ __launch_bounds__(256) void up2_rows_kernel(const f32x4* __restrict__ src, f32x4* __restrict__ dst, int H, int W,
                                                       int C4, int64_t total) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % C4);
  int64_t p = i / C4;  // output pixel, frame-major
  const int ox = (int)(p % (2 * W));
  p /= 2 * W;
  const int oy = (int)(p % (2 * H));
  const int64_t f = p / (2 * H);
  dst[i] = src[((f * H + (oy >> 1)) * W + (ox >> 1)) * C4 + c];
}
hipError_t launch_up2_rows(hipStream_t s, const float* src, float* dst, int frames, int H, int W, int C) {
  if (C % 4) return hipErrorInvalidValue;
  const int64_t total = (int64_t)frames * 4 * H * W * (C / 4);
  if (total <= 0) return hipSuccess;
  up2_rows_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>((const f32x4*)src, (f32x4*)dst, H, W, C / 4, total);
  return hipGetLastError();
}

__global__ void fill_f32_kernel(float* __restrict__ dst, int64_t n, float v) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = v;
}
hipError_t launch_fill_f32(hipStream_t s, float* dst, int64_t n, float v) {
  if (n <= 0) return hipSuccess;
  fill_f32_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(dst, n, v);
  return hipGetLastError();
}

}  // namespace lc

// Shared device-side helpers for the gfx950 kernels: storage types, 16-byte vector access,
// MFMA wrappers with their lane layouts, wavefront reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lc {

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kWave = 64;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return static_cast<float>(v); }
template <class T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return static_cast<bf16_t>(v); }  // RNE

// A 16-byte packet of storage elements: 8 bf16 or 4 float.
template <class T> struct Vec16;
template <> struct Vec16<bf16_t> {
  static constexpr int N = 8;
  bf16x8 v;
  __device__ __forceinline__ float get(int i) const { return static_cast<float>(v[i]); }
  __device__ __forceinline__ void set(int i, float f) { v[i] = static_cast<bf16_t>(f); }
};
template <> struct Vec16<float> {
  static constexpr int N = 4;
  f32x4 v;
  __device__ __forceinline__ float get(int i) const { return v[i]; }
  __device__ __forceinline__ void set(int i, float f) { v[i] = f; }
};
template <class T> __device__ __forceinline__ Vec16<T> load16(const T* p) {
  return *reinterpret_cast<const Vec16<T>*>(p);
}
template <class T> __device__ __forceinline__ void store16(T* p, const Vec16<T>& v) {
  *reinterpret_cast<Vec16<T>*>(p) = v;
}
template <class T> __device__ __forceinline__ Vec16<T> zero16() {
  Vec16<T> z;
#pragma unroll
  for (int i = 0; i < Vec16<T>::N; ++i) z.set(i, 0.f);
  return z;
}

// N consecutive elements as floats, moved in 16-byte packets (N * sizeof(T) is a multiple of 16).
template <class T, int N> __device__ __forceinline__ void load_f(const T* p, float (&v)[N]) {
  constexpr int PN = Vec16<T>::N;
  static_assert(N % PN == 0, "whole packets");
#pragma unroll
  for (int k = 0; k < N / PN; ++k) {
    Vec16<T> t = load16(p + k * PN);
#pragma unroll
    for (int e = 0; e < PN; ++e) v[k * PN + e] = t.get(e);
  }
}
template <class T, int N> __device__ __forceinline__ void store_f(T* p, const float (&v)[N]) {
  constexpr int PN = Vec16<T>::N;
  static_assert(N % PN == 0, "whole packets");
#pragma unroll
  for (int k = 0; k < N / PN; ++k) {
    Vec16<T> t;
#pragma unroll
    for (int e = 0; e < PN; ++e) t.set(e, v[k * PN + e]);
    store16(p + k * PN, t);
  }
}
// One 16-byte packet of MFMA operand type T gathered from memory of type XT (same type: a plain
// load; float memory feeding bf16 operands: two loads and a round-to-nearest-even conversion).
template <class XT, class T> __device__ __forceinline__ Vec16<T> load_packet(const XT* p) {
  float v[Vec16<T>::N];
  load_f<XT, Vec16<T>::N>(p, v);
  Vec16<T> o;
#pragma unroll
  for (int e = 0; e < Vec16<T>::N; ++e) o.set(e, v[e]);
  return o;
}
template <> __device__ __forceinline__ Vec16<bf16_t> load_packet<bf16_t, bf16_t>(const bf16_t* p) { return load16(p); }
template <> __device__ __forceinline__ Vec16<float> load_packet<float, float>(const float* p) { return load16(p); }

__device__ __forceinline__ float silu_f(float x) { return x / (1.f + __expf(-x)); }
// x * sigmoid(x) with the hardware exp2 / reciprocal approximations (about 1 ulp each)
__device__ __forceinline__ float silu_fast(float x) {
  return x * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x));
}

// ---------------------------------------------------------------------------------------
// MFMA 16x16 tiles, D[16x16] += A[16xK] * B[Kx16], one wavefront.
//   lane l supplies A[i = l%16][k-slots of group l/16] and B[same k-slots][j = l%16]
//   lane l receives D[i = 4*(l/16) + r][j = l%16], r = 0..3
// bf16: one instruction covers K = 32; the lane's k-slots are 8*(l/16) .. 8*(l/16)+7 (a 16-byte
//       packet). fp32: one instruction covers K = 4; the lane's k-slot is l/16 (one float).
// `Frag` is what one lane holds for one 16-byte packet of its row; `mma` issues as many
// instructions as the packet holds k-steps for this lane group arrangement.
// ---------------------------------------------------------------------------------------
template <class T> struct Mma16;
template <> struct Mma16<bf16_t> {
  // a 64-byte (32 element) K-slab per instruction; lane group g reads elements [8g, 8g+8)
  static constexpr int kSlab = 32;  // elements of K consumed per `mma`
  typedef bf16x8 Frag;
  static __device__ __forceinline__ Frag load(const bf16_t* row_slab, int g) {
    return *reinterpret_cast<const bf16x8*>(row_slab + 8 * g);
  }
  static __device__ __forceinline__ void mma(const Frag& a, const Frag& b, f32x4& d) {
    d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, d, 0, 0, 0);
  }
};
template <> struct Mma16<float> {
  // a 64-byte (16 element) K-slab per `mma` = 4 instructions of K = 4; lane group g reads
  // elements {g, 4+g, 8+g, 12+g}
  static constexpr int kSlab = 16;
  struct Frag { float v[4]; };
  static __device__ __forceinline__ Frag load(const float* row_slab, int g) {
    Frag f;
#pragma unroll
    for (int s = 0; s < 4; ++s) f.v[s] = row_slab[4 * s + g];
    return f;
  }
  static __device__ __forceinline__ void mma(const Frag& a, const Frag& b, f32x4& d) {
#pragma unroll
    for (int s = 0; s < 4; ++s) d = __builtin_amdgcn_mfma_f32_16x16x4f32(a.v[s], b.v[s], d, 0, 0, 0);
  }
};

// ---------------------------------------------------------------------------------------------
// 32x32 MFMA tiles. D[32x32] += A[32xK] B[Kx32]; lane l: A row l%32, B column l%32;
// D: column l%32, rows 8*(r/4) + 4*(l/32) + r%4 for r = 0..15.
// bf16: K = 16 per instruction, the lane's k-slots are 8*(l/32)..+7. fp32: K = 2, k-slot l/32.
// ---------------------------------------------------------------------------------------------
template <class T> struct Mma32;
template <> struct Mma32<bf16_t> {
  static constexpr int K = 16;   // contraction elements per instruction
  static constexpr int LK = 8;   // contiguous elements one lane supplies
  typedef bf16x8 Frag;
  static __device__ __forceinline__ Frag load(const bf16_t* p) { return *reinterpret_cast<const bf16x8*>(p); }
  static __device__ __forceinline__ Frag zero() { Frag f; for (int i = 0; i < 8; ++i) f[i] = (bf16_t)0.f; return f; }
  static __device__ __forceinline__ void mma(const Frag& a, const Frag& b, f32x16& d) {
    d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, d, 0, 0, 0);
  }
};
template <> struct Mma32<float> {
  static constexpr int K = 2;
  static constexpr int LK = 1;
  typedef float Frag;
  static __device__ __forceinline__ Frag load(const float* p) { return *p; }
  static __device__ __forceinline__ Frag zero() { return 0.f; }
  static __device__ __forceinline__ void mma(const Frag& a, const Frag& b, f32x16& d) {
    d = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, d, 0, 0, 0);
  }
};

// GELU in its tanh form: 0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3)))
__device__ __forceinline__ float gelu_tanh_f(float x) {
  const float u = 0.7978845608028654f * fmaf(0.044715f * x * x, x, x);
  const float t = 1.f - 2.f / (1.f + __expf(2.f * u));  // tanh(u)
  return 0.5f * x * (1.f + t);
}

// the same with the hardware exp2 / reciprocal approximations (about 1 ulp each): x * sigmoid(2 u), two
// transcendentals and five vector instructions where the form above compiles to an IEEE division
__device__ __forceinline__ float gelu_tanh_fast(float x) {
  const float u = 0.7978845608028654f * fmaf(0.044715f * x * x, x, x);
  return x * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-2.8853900817779268f * u));
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Column of key `k` (0..63) inside a V^T row in LDS. For bf16 the four 4-key blocks of every 16
// keys are stored in the order 0,2,1,3 so that the 8 keys one lane contracts in one instruction
// (see below) are 16 contiguous bytes.
template <class T> __device__ __forceinline__ int vcol(int k);
template <> __device__ __forceinline__ int vcol<float>(int k) { return k; }
template <> __device__ __forceinline__ int vcol<bf16_t>(int k) {
  const int b = (k >> 2) & 3;
  return (k & ~15) | ((b & 1) << 3) | ((b >> 1) << 2) | (k & 3);
}

// Source-row mapping of a dense block of `rows` rows onto a larger row-major matrix:
// dense row r lives at source row  base + (r / rows_per_seg) * seg_stride + (r % rows_per_seg).
// A frame chunk is one segment; a token chunk takes `rows_per_seg` positions out of every frame.
struct RowMap {
  int64_t base;
  int64_t seg_stride;
  int rows_per_seg;
  __host__ __device__ __forceinline__ int64_t operator()(int64_t r) const {
    return base + (r / rows_per_seg) * seg_stride + (r % rows_per_seg);
  }
};

// s_waitcnt immediate: at most `vm` vector-memory operations and no LDS operation outstanding
constexpr int waitcnt_imm(int vm) { return (vm & 15) | (7 << 4) | (0 << 8) | ((vm >> 4) << 14); }
// Workgroup barrier that orders LDS traffic only and leaves the youngest `VM` vector-memory
// operations in flight (63: all of them). __syncthreads() would wait for every outstanding global
// load and store: it cannot know that LDS-direct loads still on their way write a tile nobody reads
// before a later barrier, or that nobody in the workgroup reads back what the stores write.
template <int VM>
__device__ __forceinline__ void barrier_keep() {
  static_assert(VM >= 0 && VM < 64, "vmcnt has six bits");
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(waitcnt_imm(VM));
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

}  // namespace lc

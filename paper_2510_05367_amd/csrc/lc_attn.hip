// Attention cores on gfx950.
//
// Spatial attention (tokens = the H*W positions of one frame) is a flash-style kernel: one
// workgroup owns a block of queries of one (frame, head), walks the keys in tiles of 64 staged in
// LDS and keeps a running max / sum per query, so the T x T score matrix never exists and the
// kernel needs no workspace. Scores are produced transposed, S^T[key][query] = K Q^T, with
// 32x32 MFMA tiles: one lane then holds 16 keys of ONE query, so the softmax statistics are
// in-lane plus a single cross-lane exchange, and the exponentials, packed to the storage type,
// are directly the B operand of O^T[dim][query] += V^T[dim][key] P^T[key][query].
//
// Temporal attention (tokens = the F frames of one position) is bandwidth-bound: F is 8..32, so
// one thread owns one (position, head, query frame) and streams the F keys / values.
#include "lc_internal.h"

namespace lc {

constexpr int kKeys = 64;  // keys per LDS stage

// Column of key `k` (0..63) inside a V^T row in LDS. For bf16 the four 4-key blocks of every 16
// keys are stored in the order 0,2,1,3 so that the 8 keys one lane contracts in one instruction
// (see below) are 16 contiguous bytes.
template <class T> __device__ __forceinline__ int vcol(int k);
template <> __device__ __forceinline__ int vcol<float>(int k) { return k; }
template <> __device__ __forceinline__ int vcol<bf16_t>(int k) {
  const int b = (k >> 2) & 3;
  return (k & ~15) | ((b & 1) << 3) | ((b >> 1) << 2) | (k & 3);
}

template <class T, int D, int NQT>
__global__ __launch_bounds__(256) void spatial_attn_kernel(const T* __restrict__ qkv, T* __restrict__ out, int T_tok,
                                                           int C, int q0, int q1, float scale_log2e) {
  typedef Mma32<T> M;
  constexpr int VEC = Vec16<T>::N;
  constexpr int DP = (D + M::K - 1) / M::K * M::K;  // contraction length of Q K^T, padded
  constexpr int KSTEPS = DP / M::K;
  constexpr int DM = (D + 31) / 32;                 // 32-row tiles of O^T
  constexpr int KROW = DP * (int)sizeof(T) + 16;    // LDS row stride of the K tile, bytes
  constexpr int VROW = kKeys * (int)sizeof(T) + 16; // LDS row stride of the V^T tile, bytes
  constexpr int PSTEPS = 32 / M::K;                 // P^T V instructions per 32-key sub-tile
  __shared__ __attribute__((aligned(16))) unsigned char k_lds[kKeys * KROW];
  __shared__ __attribute__((aligned(16))) unsigned char v_lds[DM * 32 * VROW];

  const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const int lq = lane & 31, hh = lane >> 5;
  const int head = blockIdx.y, frame = blockIdx.z;
  const int ld = 3 * C;
  const T* __restrict__ base = qkv + (int64_t)frame * T_tok * ld + head * D;
  const int qblk = q0 + blockIdx.x * (4 * NQT * 32) + wid * (NQT * 32);

  // zero the V^T rows beyond D once (they feed unused rows of O^T)
  for (int i = tid; i < DM * 32 * VROW / 4; i += 256) reinterpret_cast<uint32_t*>(v_lds)[i] = 0u;
  for (int i = tid; i < kKeys * KROW / 4; i += 256) reinterpret_cast<uint32_t*>(k_lds)[i] = 0u;

  // ---- Q fragments (B operand of S^T = K Q^T): lane holds query lq, k-slots M::LK*hh + M::K*kk
  typename M::Frag qf[NQT][KSTEPS];
#pragma unroll
  for (int t = 0; t < NQT; ++t) {
    const int q = qblk + t * 32 + lq;
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
      const int e = kk * M::K + hh * M::LK;
      qf[t][kk] = (q < q1 && e < D) ? M::load(base + (int64_t)q * ld + e) : M::zero();
    }
  }
  f32x16 o[NQT][DM];
  float m_run[NQT], l_run[NQT];
#pragma unroll
  for (int t = 0; t < NQT; ++t) {
    m_run[t] = -INFINITY;
    l_run[t] = 0.f;
#pragma unroll
    for (int mt = 0; mt < DM; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[t][mt][r] = 0.f;
  }
  __syncthreads();

  constexpr int PK = D / VEC;  // 16-byte packets per K / V row
  for (int k0 = 0; k0 < T_tok; k0 += kKeys) {
    // ---- stage 64 keys: K rows as they are, V transposed
    for (int i = tid; i < kKeys * PK; i += 256) {
      const int key = i / PK, pk = i - key * PK;
      const int gk = k0 + key;
      Vec16<T> kv = zero16<T>(), vv = zero16<T>();
      if (gk < T_tok) {
        kv = load16(base + (int64_t)gk * ld + C + pk * VEC);
        vv = load16(base + (int64_t)gk * ld + 2 * C + pk * VEC);
      }
      *reinterpret_cast<Vec16<T>*>(k_lds + key * KROW + pk * 16) = kv;
      const int col = vcol<T>(key);
#pragma unroll
      for (int e = 0; e < VEC; ++e)
        *reinterpret_cast<T*>(v_lds + (pk * VEC + e) * VROW + col * (int)sizeof(T)) = vv.v[e];
    }
    __syncthreads();

#pragma unroll
    for (int kt = 0; kt < kKeys / 32; ++kt) {
      if (k0 + kt * 32 >= T_tok) break;  // uniform: whole sub-tile beyond the sequence
      // ---- S^T sub-tile [32 keys][32 queries] per query tile
      typename M::Frag kf[KSTEPS];
#pragma unroll
      for (int kk = 0; kk < KSTEPS; ++kk)
        kf[kk] = M::load(reinterpret_cast<const T*>(k_lds + (kt * 32 + lq) * KROW) + kk * M::K + hh * M::LK);
      typename M::Frag pf[NQT][PSTEPS];
#pragma unroll
      for (int t = 0; t < NQT; ++t) {
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) M::mma(kf[kk], qf[t][kk], s);
        // lane holds keys  k0 + kt*32 + 8*(r/4) + 4*hh + r%4  of query lq
        float mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = k0 + kt * 32 + 8 * (r >> 2) + 4 * hh + (r & 3);
          s[r] = key < T_tok ? s[r] * scale_log2e : -INFINITY;
          mx = fmaxf(mx, s[r]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run[t], mx);
        const float alpha = exp2f(m_run[t] - m_new);  // m_new is finite: the sub-tile has a valid key
        m_run[t] = m_new;
        float ps = 0.f;
        float p[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          p[r] = exp2f(s[r] - m_new);
          ps += p[r];
        }
        l_run[t] = l_run[t] * alpha + ps;
#pragma unroll
        for (int mt = 0; mt < DM; ++mt)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[t][mt][r] *= alpha;
        // pack P^T: instruction step ps_ takes registers [LK*ps_ .. ) of this lane
        if constexpr (sizeof(T) == 2) {
#pragma unroll
          for (int st = 0; st < PSTEPS; ++st)
#pragma unroll
            for (int e = 0; e < 8; ++e) pf[t][st][e] = static_cast<bf16_t>(p[st * 8 + e]);
        } else {
#pragma unroll
          for (int st = 0; st < PSTEPS; ++st) pf[t][st] = p[st];
        }
      }
      // ---- O^T += V^T P^T. Step st contracts, in lane half hh, the keys of registers
      //      [LK*st, LK*st + LK): bf16 -> keys 16*st + 4*hh + {0..3} and 16*st + 8 + 4*hh + {0..3}
      //      (contiguous after the vcol permutation, at column 16*st + 8*hh); fp32 -> the single
      //      key 8*(st/4) + 4*hh + st%4.
#pragma unroll
      for (int st = 0; st < PSTEPS; ++st) {
        int col;
        if constexpr (sizeof(T) == 2) col = kt * 32 + 16 * st + 8 * hh;
        else col = kt * 32 + 8 * (st >> 2) + 4 * hh + (st & 3);
#pragma unroll
        for (int mt = 0; mt < DM; ++mt) {
          typename M::Frag vf = M::load(reinterpret_cast<const T*>(v_lds + (mt * 32 + lq) * VROW) + col);
#pragma unroll
          for (int t = 0; t < NQT; ++t) M::mma(vf, pf[t][st], o[t][mt]);
        }
      }
    }
    __syncthreads();
  }

  // ---- normalise and store: lane holds O^T[dim = 32*mt + 8*(r/4) + 4*hh + r%4][query lq]
#pragma unroll
  for (int t = 0; t < NQT; ++t) {
    const int q = qblk + t * 32 + lq;
    const float l = l_run[t] + __shfl_xor(l_run[t], 32, 64);
    const float inv = 1.f / l;
    if (q >= q1) continue;
    T* orow = out + ((int64_t)frame * T_tok + q) * C + head * D;
#pragma unroll
    for (int mt = 0; mt < DM; ++mt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int dim = mt * 32 + 8 * g + 4 * hh;
        if (dim < D) {
#pragma unroll
          for (int e = 0; e < 4; ++e) orow[dim + e] = from_f32<T>(o[t][mt][4 * g + e] * inv);
        }
      }
  }
}

template <class T, int NQT>
static hipError_t spatial_dispatch(hipStream_t s, const T* qkv, T* out, int frames, int T_tok, int heads, int d,
                                   int q0, int q1) {
  const int C = heads * d;
  const float sl = 1.4426950408889634f / sqrtf((float)d);
  dim3 grid((q1 - q0 + 4 * NQT * 32 - 1) / (4 * NQT * 32), heads, frames);
#define LC_GO(D) spatial_attn_kernel<T, D, NQT><<<grid, 256, 0, s>>>(qkv, out, T_tok, C, q0, q1, sl)
  switch (d) {
    case 8: LC_GO(8); break;
    case 16: LC_GO(16); break;
    case 32: LC_GO(32); break;
    case 40: LC_GO(40); break;
    case 64: LC_GO(64); break;
    default: return hipErrorInvalidValue;
  }
#undef LC_GO
  return hipGetLastError();
}

hipError_t launch_spatial_attention(hipStream_t s, int dt, const void* qkv, void* out, int frames, int T,
                                    int heads, int d, int q0, int q1) {
  if (frames <= 0 || q1 <= q0) return hipSuccess;
  if (dt == kBF16) return spatial_dispatch<bf16_t, 2>(s, (const bf16_t*)qkv, (bf16_t*)out, frames, T, heads, d, q0, q1);
  return spatial_dispatch<float, 1>(s, (const float*)qkv, (float*)out, frames, T, heads, d, q0, q1);
}

// ---------------------------------------------------------------------------------------------
// Temporal attention: thread = (batch b, position p, query frame f, head h), h fastest so that
// neighbouring lanes read neighbouring head slices of the same row.
// ---------------------------------------------------------------------------------------------
template <class T, int D>
__global__ __launch_bounds__(256) void temporal_attn_kernel(const T* __restrict__ qkv, T* __restrict__ out, int B,
                                                            int F, int P, int heads, float scale_log2e) {
  constexpr int VEC = Vec16<T>::N;
  constexpr int PK = D / VEC;
  const int C = heads * D, ld = 3 * C;
  const int64_t total = (int64_t)B * P * F * heads;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int h = (int)(i % heads);
  int64_t t = i / heads;
  const int f = (int)(t % F);
  t /= F;
  const int p = (int)(t % P);
  const int b = (int)(t / P);
  // row of (frame n, position p) in the frame-major chunk: n * P + p
  const T* qrow = qkv + ((int64_t)(b * F + f) * P + p) * ld + h * D;
  float q[D];
#pragma unroll
  for (int k = 0; k < PK; ++k) {
    Vec16<T> v = load16(qrow + k * VEC);
#pragma unroll
    for (int e = 0; e < VEC; ++e) q[k * VEC + e] = v.get(e) * scale_log2e;
  }
  float acc[D];
#pragma unroll
  for (int e = 0; e < D; ++e) acc[e] = 0.f;
  float m = -INFINITY, l = 0.f;
  for (int g = 0; g < F; ++g) {
    const T* krow = qkv + ((int64_t)(b * F + g) * P + p) * ld + C + h * D;
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < PK; ++k) {
      Vec16<T> v = load16(krow + k * VEC);
#pragma unroll
      for (int e = 0; e < VEC; ++e) s = fmaf(q[k * VEC + e], v.get(e), s);
    }
    const float m_new = fmaxf(m, s);
    const float alpha = exp2f(m - m_new);
    const float pe = exp2f(s - m_new);
    m = m_new;
    l = l * alpha + pe;
    const T* vrow = krow + C;
#pragma unroll
    for (int k = 0; k < PK; ++k) {
      Vec16<T> v = load16(vrow + k * VEC);
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[k * VEC + e] = fmaf(acc[k * VEC + e], alpha, pe * v.get(e));
    }
  }
  const float inv = 1.f / l;
  T* orow = out + ((int64_t)(b * F + f) * P + p) * C + h * D;
#pragma unroll
  for (int k = 0; k < PK; ++k) {
    Vec16<T> v;
#pragma unroll
    for (int e = 0; e < VEC; ++e) v.set(e, acc[k * VEC + e] * inv);
    store16(orow + k * VEC, v);
  }
}

template <class T>
static hipError_t temporal_dispatch(hipStream_t s, const T* qkv, T* out, int B, int F, int P, int heads, int d) {
  const int64_t total = (int64_t)B * P * F * heads;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  const float sl = 1.4426950408889634f / sqrtf((float)d);
#define LC_GO(D) temporal_attn_kernel<T, D><<<blocks, 256, 0, s>>>(qkv, out, B, F, P, heads, sl)
  switch (d) {
    case 8: LC_GO(8); break;
    case 16: LC_GO(16); break;
    case 32: LC_GO(32); break;
    case 40: LC_GO(40); break;
    case 64: LC_GO(64); break;
    default: return hipErrorInvalidValue;
  }
#undef LC_GO
  return hipGetLastError();
}

hipError_t launch_temporal_attention(hipStream_t s, int dt, const void* qkv, void* out, int B, int F, int P,
                                     int heads, int d) {
  if (B <= 0 || F <= 0 || P <= 0) return hipSuccess;
  if (dt == kBF16) return temporal_dispatch<bf16_t>(s, (const bf16_t*)qkv, (bf16_t*)out, B, F, P, heads, d);
  return temporal_dispatch<float>(s, (const float*)qkv, (float*)out, B, F, P, heads, d);
}

}  // namespace lc

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
// Temporal attention (tokens = the F frames of one position) is bandwidth-bound: F is 8..32. bf16 stages
// with 8..32 frames put the scores of a (position, head) on one 16 x 16 or 32 x 32 MFMA tile; otherwise one thread
// owns one (position, head, query frame) and streams the F keys / values.
#include "lc_internal.h"

#include <type_traits>

namespace lc {

constexpr int kKeys = 64;  // keys per LDS stage

// qk: rows [frame*T + token] of stride ldq holding q at column 0 and k at column C (per head: + head*D).
// vt: V transposed and block-permuted, [frame][C][Tp] with token t of a row at column vcol(t), Tp a
// multiple of 64 (columns beyond T are never trusted: they are zeroed while staging).
// the permutation is an involution on the 4-key blocks (it swaps blocks 1 and 2)
template <class T> __device__ __forceinline__ int vcol_inv(int c) { return vcol<T>(c); }

// Queries: the launch takes nq of them, numbered densely; query number i is token q0 + (i / qw) * qstride + i % qw
// (a window of rows of qw tokens out of image rows of qstride tokens; a plain range has qw >= nq).
// PRE: the q columns already hold q * log2(e) / sqrt(d) (the q,k,v projection scales them before it
// rounds them); `scale_log2e` is then 1.
// XA (cross-attention): the keys are not the queries' own rows but rows [Tk] of stride ldk at kx, one set (with its
// V^T) per group of kv_div consecutive frames; T_tok then counts the query tokens of a frame only.
template <class T, int D, int NQT, bool PRE, bool XA = false>
__global__ __launch_bounds__(256, 2) void spatial_attn_kernel(const T* __restrict__ qk, int ldq,
                                                           const T* __restrict__ vt, int Tp, T* __restrict__ out,
                                                           int T_tok, int C, int q0, int nq, int qw, int qstride,
                                                           float scale_log2e, const T* __restrict__ kx = nullptr,
                                                           int ldk = 0, int Tk = 0, int kv_div = 1) {
  typedef Mma32<T> M;
  constexpr int VEC = Vec16<T>::N;
  constexpr int DP = (D + M::K - 1) / M::K * M::K;  // contraction length of Q K^T, padded
  constexpr int KSTEPS = DP / M::K;
  constexpr int DM = (D + 31) / 32;                 // 32-row tiles of O^T
  constexpr int KROW = DP * (int)sizeof(T) + 16;    // LDS row stride of the K tile, bytes
  constexpr int VROW = kKeys * (int)sizeof(T) + 16; // LDS row stride of the V^T tile, bytes
  constexpr int PSTEPS = 32 / M::K;                 // P^T V instructions per 32-key sub-tile
  constexpr int KT = kKeys / 32;                    // 32-key sub-tiles per stage
  constexpr int KBYTES = kKeys * KROW, VBYTES = DM * 32 * VROW;
  constexpr int PK = D / VEC;                       // 16-byte packets per K / V row
  constexpr int NP = (kKeys * PK + 255) / 256;      // K (and V) packets per thread per stage
  __shared__ __attribute__((aligned(16))) unsigned char k_lds[2][KBYTES];
  __shared__ __attribute__((aligned(16))) unsigned char v_lds[2][VBYTES];

  const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const int lq = lane & 31, hh = lane >> 5;
  // Workgroups are handed to the eight XCDs round robin in launch order, and each XCD has an L2 of its
  // own. All query blocks of one (frame, head) stream the same keys and values, so they are mapped to one
  // XCD (problem p on XCD p % 8): its L2 then fetches that K / V once instead of every XCD fetching all of
  // them. Needs the number of problems to be a multiple of eight; otherwise the plain mapping.
  int qb = blockIdx.x, head = blockIdx.y, frame = blockIdx.z;
  {
    const int nqb = gridDim.x, heads = gridDim.y, nprob = gridDim.y * gridDim.z;
    if (nprob % 8 == 0) {
      const int lin = blockIdx.x + nqb * (blockIdx.y + heads * blockIdx.z);
      const int xcd = lin & 7, slot = lin >> 3;
      const int prob = xcd + 8 * (slot / nqb);
      qb = slot % nqb;
      head = prob % heads;
      frame = prob / heads;
    }
  }
  const int ld = ldq;
  const T* __restrict__ base = qk + (int64_t)frame * T_tok * ld + head * D;
  const int kvf = XA ? frame / kv_div : frame;  // whose keys and values
  const int TK = XA ? Tk : T_tok;               // number of keys
  const int ldkk = XA ? ldk : ld;
  const T* __restrict__ kb = XA ? kx + (int64_t)kvf * Tk * ldk + head * D : base + C;
  const T* __restrict__ vbase = vt + ((int64_t)kvf * C + head * D) * Tp;
  const int qblk = qb * (4 * NQT * 32) + wid * (NQT * 32);  // first query number of this wavefront
  auto token_of = [&](int qi) { const int r = qi / qw; return q0 + r * qstride + (qi - r * qw); };

  // zero both buffers once: K columns beyond D and V^T rows beyond D feed padded MFMA lanes
  for (int i = tid; i < 2 * KBYTES / 4; i += 256) reinterpret_cast<uint32_t*>(&k_lds[0][0])[i] = 0u;
  for (int i = tid; i < 2 * VBYTES / 4; i += 256) reinterpret_cast<uint32_t*>(&v_lds[0][0])[i] = 0u;
  // Softmax denominators for free: when d leaves a spare row in the 32-row tiles of V^T (d = 40:
  // rows 40..63 are padding), row D is set to ones, so O^T[D][q] accumulates the sum over keys of
  // exactly the (rounded) probabilities that multiply V, and is rescaled with the rest of O^T.
  constexpr bool ROWSUM = D % 32 != 0;
  // Softmax exponents for free as well: when the padded contraction of K Q^T has a spare slot (d = 40
  // contracts 48) and the queries come multiplied by scale * log2(e), slot D of every key is 1 and
  // slot D of a query holds minus its running maximum (in the operand type, in log2 units). The
  // MFMA then delivers  s * scale * log2(e) - m  directly and the probability is exp2 of that: no
  // per-score multiply-add. Any rounding of m cancels, since the same m enters the probabilities,
  // the denominator (ones row above) and the rescaling of O^T.
  constexpr bool FOLD = PRE && sizeof(T) == 2 && DP > D && ROWSUM;
  constexpr int KX = D / M::K, HX = (D % M::K) / M::LK, EX = (D % M::K) % M::LK;  // where slot D lives
  if (ROWSUM) {
    __syncthreads();
    for (int i = tid; i < 2 * kKeys; i += 256)
      reinterpret_cast<T*>(&v_lds[i / kKeys][D * VROW])[i % kKeys] = from_f32<T>(1.f);
    if (FOLD)
      for (int i = tid; i < 2 * kKeys; i += 256)
        reinterpret_cast<T*>(&k_lds[i / kKeys][(i % kKeys) * KROW])[D] = from_f32<T>(1.f);
  }

  // ---- staging: K packet i = tid + 256 j of a stage is (key i / PK, packet i % PK); V^T packet i is
  //      (dim i / VPK, packet i % VPK) and is already in LDS order
  constexpr int VPK = kKeys / VEC;              // 16-byte packets per V^T row of a stage
  constexpr int NPV = (D * VPK + 255) / 256;
  Vec16<T> kreg[NP], vreg[NPV];
  auto fetch_kv = [&](int k0) {
#pragma unroll
    for (int j = 0; j < NP; ++j) {
      const int i = tid + 256 * j;
      const int key = min(i / PK, kKeys - 1), pk = i % PK;
      const int gk = min(k0 + key, TK - 1);  // clamped: keys beyond the sequence are masked later
      kreg[j] = load16(kb + (int64_t)gk * ldkk + pk * VEC);
    }
#pragma unroll
    for (int j = 0; j < NPV; ++j) {
      const int i = tid + 256 * j;
      const int dim = min(i / VPK, D - 1), pk = i % VPK;
      vreg[j] = load16(vbase + (int64_t)dim * Tp + k0 + pk * VEC);
    }
  };
  auto stash_kv = [&](int buf, int k0) {
#pragma unroll
    for (int j = 0; j < NP; ++j) {
      const int i = tid + 256 * j;
      if (i < kKeys * PK) *reinterpret_cast<Vec16<T>*>(&k_lds[buf][(i / PK) * KROW + (i % PK) * 16]) = kreg[j];
    }
    const bool tail = k0 + kKeys > TK;
#pragma unroll
    for (int j = 0; j < NPV; ++j) {
      const int i = tid + 256 * j;
      if (i < D * VPK) {
        const int dim = i / VPK, pk = i % VPK;
        Vec16<T> v = vreg[j];
        if (tail) {  // column c of the stage holds the token whose vcol is c; zero what lies beyond T
#pragma unroll
          for (int e = 0; e < VEC; ++e)
            if (k0 + vcol_inv<T>(pk * VEC + e) >= TK) v.set(e, 0.f);
        }
        *reinterpret_cast<Vec16<T>*>(&v_lds[buf][dim * VROW + pk * 16]) = v;
      }
    }
  };

  // ---- Q fragments (B operand of S^T = K Q^T): lane holds query lq, k-slots M::LK*hh + M::K*kk
  typename M::Frag qf[NQT][KSTEPS];
#pragma unroll
  for (int t = 0; t < NQT; ++t) {
    const int qi = qblk + t * 32 + lq;
    const int q = token_of(qi);
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
      const int e = kk * M::K + hh * M::LK;
      qf[t][kk] = (qi < nq && e < D) ? M::load(base + (int64_t)q * ld + e) : M::zero();
      if constexpr (FOLD) {  // slots >= D must be zero: slot D will carry the running maximum
#pragma unroll
        for (int j = 0; j < M::LK; ++j)
          if (e + j >= D) qf[t][kk][j] = (bf16_t)0.f;
      }
    }
  }
  f32x16 o[NQT][DM];
  float m_run[NQT], l_run[NQT];  // running max (raw score units) and per-lane partial sum
#pragma unroll
  for (int t = 0; t < NQT; ++t) {
    m_run[t] = FOLD ? 0.f : -INFINITY;  // FOLD: log2 units, as held in slot D of the query
    l_run[t] = 0.f;
#pragma unroll
    for (int mt = 0; mt < DM; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[t][mt][r] = 0.f;
  }
  fetch_kv(0);
  __syncthreads();  // zero fill done
  stash_kv(0, 0);
  __syncthreads();

  const int nstage = (TK + kKeys - 1) / kKeys;
  for (int st_i = 0; st_i < nstage; ++st_i) {
    const int k0 = st_i * kKeys, buf = st_i & 1;
    const bool tail = k0 + kKeys > TK;  // uniform: some keys of this stage lie beyond the sequence
    if (st_i + 1 < nstage) fetch_kv(k0 + kKeys);

    // ---- S^T sub-tiles [32 keys][32 queries]
    f32x16 sc[NQT][KT];
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      typename M::Frag kf[KSTEPS];
#pragma unroll
      for (int kk = 0; kk < KSTEPS; ++kk)
        kf[kk] = M::load(reinterpret_cast<const T*>(&k_lds[buf][(kt * 32 + lq) * KROW]) + kk * M::K + hh * M::LK);
#pragma unroll
      for (int t = 0; t < NQT; ++t) {
#pragma unroll
        for (int r = 0; r < 16; ++r) sc[t][kt][r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) M::mma(kf[kk], qf[t][kk], sc[t][kt]);
      }
    }
#pragma unroll
    for (int t = 0; t < NQT; ++t) {
      // lane holds keys  k0 + kt*32 + 8*(r/4) + 4*hh + r%4  of query lq
      if (tail) {
        // (the key indices are built from a value the compiler cannot see through: left alone it hoists
        // these 64 additions out of the branch and every stage pays for them)
        int kbi = k0 + 4 * hh;
        asm volatile("" : "+v"(kbi));
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (kbi + kt * 32 + 8 * (r >> 2) + (r & 3) >= TK) sc[t][kt][r] = -INFINITY;
      }
      float mx = -INFINITY;
#pragma unroll
      for (int kt = 0; kt < KT; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sc[t][kt][r]);
      // mx: over this lane's 16 keys of the query. The other half of the query's keys sits in lane l ^ 32; the
      // exchange (a trip through LDS) is only made inside the rare branch below: whether ANY lane of the
      // wavefront exceeds the margin is the same question asked of the per-lane and of the per-query maxima.
      // The offset m subtracted in the exponent need not be the exact running maximum: any m gives the same
      // softmax as long as exp2 stays in range, because the same m enters the probabilities, the denominator
      // and the rescaling. So m is raised (and O^T, l rescaled) only when some query of the wavefront sees a
      // score more than kLazy above its m (in log2 units: probabilities then reach at most 2^kLazy, harmless
      // in fp32 and in bf16, which rounds relatively). With the exact maximum about 70 % of the 64-key stages
      // took the rescaling branch for some lane; with the margin hardly any after the first. (A lane whose own
      // score stays inside the margin keeps its m when the branch is taken for another: exp2(0) = 1 exactly.)
      constexpr float kLazy = 8.f;
      if constexpr (FOLD) {
        // sc already is s * scale * log2(e) - m_run: a score above the offset shows as a positive one
        const bool first = st_i == 0;  // the first stage sets the offset, which may be negative
        if (first || __builtin_amdgcn_ballot_w64(mx > kLazy) != 0) {
          mx = fmaxf(mx, __shfl_xor(mx, 32, 64));  // a stage always holds at least one valid key: finite
          // (each query decides for itself: what the other lanes of the wavefront do must not show in its bits,
          // or the result would depend on which queries share a wavefront, i.e. on the query window)
          float m_new = m_run[t] + ((first || mx > kLazy) ? mx : 0.f);
          m_new = static_cast<float>(static_cast<bf16_t>(m_new));  // as slot D will hold it
          const float delta = m_new - m_run[t];
          const float alpha = __builtin_amdgcn_exp2f(-delta);
          m_run[t] = m_new;
#pragma unroll
          for (int mt = 0; mt < DM; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[t][mt][r] *= alpha;
#pragma unroll
          for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int r = 0; r < 16; ++r) sc[t][kt][r] -= delta;
          if (hh == HX) qf[t][KX][EX] = static_cast<bf16_t>(-m_new);
        }
      } else if (st_i == 0 || __builtin_amdgcn_ballot_w64((mx - m_run[t]) * scale_log2e > kLazy) != 0) {
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const bool up = st_i == 0 || (mx - m_run[t]) * scale_log2e > kLazy;
        const float m_new = up ? fmaxf(m_run[t], mx) : m_run[t];
        const float alpha = __builtin_amdgcn_exp2f((m_run[t] - m_new) * scale_log2e);
        m_run[t] = m_new;
        if (!ROWSUM) l_run[t] *= alpha;
#pragma unroll
        for (int mt = 0; mt < DM; ++mt)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[t][mt][r] *= alpha;
      }
      const float mc = m_run[t] * scale_log2e;
      typename M::Frag pf[KT][PSTEPS];
      float ps = 0.f;
#pragma unroll
      for (int kt = 0; kt < KT; ++kt) {
        float p[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          p[r] = FOLD ? __builtin_amdgcn_exp2f(sc[t][kt][r]) : __builtin_amdgcn_exp2f(fmaf(sc[t][kt][r], scale_log2e, -mc));
          if (!ROWSUM) ps += p[r];
        }
        if constexpr (sizeof(T) == 2) {
#pragma unroll
          for (int st = 0; st < PSTEPS; ++st)
#pragma unroll
            for (int e = 0; e < 8; ++e) pf[kt][st][e] = static_cast<bf16_t>(p[st * 8 + e]);
        } else {
#pragma unroll
          for (int st = 0; st < PSTEPS; ++st) pf[kt][st] = p[st];
        }
      }
      if (!ROWSUM) l_run[t] += ps;
      // ---- O^T += V^T P^T. Step st of sub-tile kt contracts, in lane half hh, the keys of registers
      //      [LK*st, LK*st + LK): bf16 -> keys 16*st + 4*hh + {0..3} and 16*st + 8 + 4*hh + {0..3}
      //      (contiguous after the vcol permutation, at column 16*st + 8*hh); fp32 -> the single key
      //      8*(st/4) + 4*hh + st%4.
#pragma unroll
      for (int kt = 0; kt < KT; ++kt)
#pragma unroll
        for (int st = 0; st < PSTEPS; ++st) {
          int col;
          if constexpr (sizeof(T) == 2) col = kt * 32 + 16 * st + 8 * hh;
          else col = kt * 32 + 8 * (st >> 2) + 4 * hh + (st & 3);
#pragma unroll
          for (int mt = 0; mt < DM; ++mt) {
            const typename M::Frag vf = M::load(reinterpret_cast<const T*>(&v_lds[buf][(mt * 32 + lq) * VROW]) + col);
            M::mma(vf, pf[kt][st], o[t][mt]);
          }
        }
    }
    if (st_i + 1 < nstage) stash_kv(buf ^ 1, k0 + kKeys);
    __syncthreads();
  }

  // ---- normalise and store: lane holds O^T[dim = 32*mt + 8*(r/4) + 4*hh + r%4][query lq]
#pragma unroll
  for (int t = 0; t < NQT; ++t) {
    const int qi = qblk + t * 32 + lq;
    const int q = token_of(qi);
    float l;
    if (ROWSUM) {  // O^T[D][q] sits in register r of the lanes of half hsel
      constexpr int rem = D % 32, hsel = (rem % 8) / 4, r = (rem / 8) * 4 + rem % 4;
      l = __shfl(o[t][D / 32][r], lq + 32 * hsel, 64);
    } else {
      l = l_run[t] + __shfl_xor(l_run[t], 32, 64);
    }
    const float inv = 1.f / l;
    if (qi >= nq) continue;
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

template <class T, int NQT, bool PRE>
static hipError_t spatial_dispatch(hipStream_t s, const T* qk, int ldq, const T* vt, int Tp, T* out, int frames,
                                   int T_tok, int heads, int d, int q0, int nq, int qw, int qstride) {
  const int C = heads * d;
  const float sl = PRE ? 1.f : 1.4426950408889634f / sqrtf((float)d);
  dim3 grid((nq + 4 * NQT * 32 - 1) / (4 * NQT * 32), heads, frames);
#define LC_GO(D) spatial_attn_kernel<T, D, NQT, PRE><<<grid, 256, 0, s>>>(qk, ldq, vt, Tp, out, T_tok, C, q0, nq, qw, qstride, sl)
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

hipError_t launch_spatial_attention(hipStream_t s, int dt, const void* qk, int ldq, const void* vt, int Tp, void* out,
                                    int frames, int T, int heads, int d, int q0, int q1, int q_prescaled) {
  if (q1 <= q0) return hipSuccess;
  return launch_spatial_attention_window(s, dt, qk, ldq, vt, Tp, out, frames, T, heads, d, q0, q1 - q0, q1 - q0, 0,
                                         q_prescaled);
}

hipError_t launch_spatial_attention_window(hipStream_t s, int dt, const void* qk, int ldq, const void* vt, int Tp, void* out,
                                           int frames, int T, int heads, int d, int q0, int nq, int qw, int qstride,
                                           int q_prescaled) {
  if (frames <= 0 || nq <= 0) return hipSuccess;
  if (Tp % kKeys != 0 || Tp < T || qw <= 0 || q0 < 0) return hipErrorInvalidValue;
  {  // the last query must be a token of the frame
    const int r = (nq - 1) / qw;
    if ((int64_t)q0 + (int64_t)r * qstride + (nq - 1 - r * qw) >= T) return hipErrorInvalidValue;
  }
#define LC_ARGS(TT) s, (const TT*)qk, ldq, (const TT*)vt, Tp, (TT*)out, frames, T, heads, d, q0, nq, qw, qstride
  if (dt == kBF16)
    return q_prescaled ? spatial_dispatch<bf16_t, 2, true>(LC_ARGS(bf16_t)) : spatial_dispatch<bf16_t, 2, false>(LC_ARGS(bf16_t));
  return q_prescaled ? spatial_dispatch<float, 1, true>(LC_ARGS(float)) : spatial_dispatch<float, 1, false>(LC_ARGS(float));
#undef LC_ARGS
}

// Cross-attention: queries q[frames*Tq] (stride ldq, head h at column h*d) against keys k[(frames/kv_div)*Tk] (stride
// ldk) and their V^T [(frames/kv_div)][C][Tp]; out [frames*Tq][C]. Frame f uses the keys of group f / kv_div.
template <class T>
static hipError_t cross_dispatch(hipStream_t s, const T* q, int ldq, const T* k, int ldk, const T* vt, int Tp, T* out, int frames,
                                 int Tq, int Tk, int kv_div, int heads, int d) {
  constexpr int NQT = sizeof(T) == 2 ? 2 : 1;
  const int C = heads * d;
  const float sl = 1.4426950408889634f / sqrtf((float)d);
  dim3 grid((Tq + 4 * NQT * 32 - 1) / (4 * NQT * 32), heads, frames);
#define LC_GO(D) spatial_attn_kernel<T, D, NQT, false, true><<<grid, 256, 0, s>>>(q, ldq, vt, Tp, out, Tq, C, 0, Tq, Tq, 0, sl, k, ldk, Tk, kv_div)
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
hipError_t launch_cross_attention(hipStream_t s, int dt, const void* q, int ldq, const void* k, int ldk, const void* vt, int Tp,
                                  void* out, int frames, int Tq, int Tk, int kv_div, int heads, int d) {
  if (frames <= 0 || Tq <= 0) return hipSuccess;
  if (Tk <= 0 || kv_div <= 0 || frames % kv_div || Tp % kKeys != 0 || Tp < Tk) return hipErrorInvalidValue;
  if (dt == kBF16)
    return cross_dispatch<bf16_t>(s, (const bf16_t*)q, ldq, (const bf16_t*)k, ldk, (const bf16_t*)vt, Tp, (bf16_t*)out, frames, Tq, Tk,
                                  kv_div, heads, d);
  return cross_dispatch<float>(s, (const float*)q, ldq, (const float*)k, ldk, (const float*)vt, Tp, (float*)out, frames, Tq, Tk, kv_div,
                               heads, d);
}

// V^T in the layout the spatial kernel stages: vt[frame][c][vcol(t)] = v[frame*T + t][c] (v rows of stride ldv)
template <class T>
__global__ __launch_bounds__(256) void make_vt_kernel(const T* __restrict__ v, int ldv, T* __restrict__ vt, int T_tok,
                                                      int Tp, int C) {
  __shared__ T tile[32][33];
  const int f = blockIdx.z, t0 = blockIdx.x * 32, c0 = blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int k = ty; k < 32; k += 8)
    if (t0 + k < T_tok && c0 + tx < C) tile[k][tx] = v[((int64_t)f * T_tok + t0 + k) * ldv + c0 + tx];
  __syncthreads();
  for (int k = ty; k < 32; k += 8) {
    const int t = t0 + tx;
    if (c0 + k < C && t < T_tok) vt[((int64_t)f * C + c0 + k) * Tp + (t & ~63) + vcol<T>(t & 63)] = tile[tx][k];
  }
}
hipError_t launch_make_vt(hipStream_t s, int dt, const void* v, int ldv, void* vt, int frames, int T, int Tp, int C) {
  if (frames <= 0) return hipSuccess;
  dim3 grid((T + 31) / 32, (C + 31) / 32, frames);
  if (dt == kBF16) make_vt_kernel<bf16_t><<<grid, 256, 0, s>>>((const bf16_t*)v, ldv, (bf16_t*)vt, T, Tp, C);
  else make_vt_kernel<float><<<grid, 256, 0, s>>>((const float*)v, ldv, (float*)vt, T, Tp, C);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Temporal attention over the F frames of one spatial position. A workgroup takes `np` consecutive
// positions of one batch element and brings the q,k,v rows of all F frames at those positions into
// LDS once, with LDS-direct loads (F x np rows of 3C elements; the rows of one frame are contiguous
// in memory). Then thread = (position, query frame f, head h), h fastest: per key frame every lane of
// a wavefront reads the same row and neighbouring lanes neighbouring head slices of it, so the LDS
// reads are broadcasts or conflict-free, where the same loop over global memory had every thread
// pull all F key and value rows through the vector cache again.
// ---------------------------------------------------------------------------------------------
template <class T, int D>
__global__ __launch_bounds__(256) void temporal_attn_kernel(const T* __restrict__ qkv, T* __restrict__ out, int F,
                                                            int P, int heads, int np, float scale_log2e) {
  constexpr int VEC = Vec16<T>::N;
  constexpr int PK = D / VEC;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int C = heads * D, ld = 3 * C;
  const int tid = threadIdx.x, wid = tid >> 6;
  const int b = blockIdx.y, p0 = blockIdx.x * np;
  const int npv = min(np, P - p0);  // positions of this workgroup that exist
  // LDS image [f][np][ld], filled 16 bytes per lane: packet q = (frame, position, packet of the row)
  const int ppr = ld / VEC;         // packets per row
  const int total = F * np * ppr;
  for (int q0 = 0; q0 < total; q0 += 256) {
    const int q = min(q0 + tid, total - 1);
    const int row = q / ppr, pk = q - row * ppr;
    const int f = row / np, pos = min(row - f * np, npv - 1);  // positions beyond the end: a copy nobody reads
    const T* src = qkv + ((int64_t)(b * F + f) * P + p0 + pos) * ld + pk * VEC;
#ifdef __HIP_DEVICE_COMPILE__  // the host pass only needs the kernel's stub; it does not know this builtin
    __builtin_amdgcn_global_load_lds(src, smem + (q0 + wid * 64) * 16, 16, 0, 0);
#else
    (void)src;
#endif
  }
  __builtin_amdgcn_s_waitcnt(0);  // every counter at zero: the rows have landed
  __syncthreads();

  const T* rows = reinterpret_cast<const T*>(smem);
  const int items = npv * F * heads;
  for (int item = tid; item < items; item += 256) {
    const int h = item % heads;
    const int f = (item / heads) % F;
    const int pos = item / (heads * F);
    const T* qrow = rows + (int64_t)(f * np + pos) * ld + h * D;
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
      const T* krow = rows + (int64_t)(g * np + pos) * ld + C + h * D;
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
    T* orow = out + ((int64_t)(b * F + f) * P + p0 + pos) * C + h * D;
#pragma unroll
    for (int k = 0; k < PK; ++k) {
      Vec16<T> v;
#pragma unroll
      for (int e = 0; e < VEC; ++e) v.set(e, acc[k * VEC + e] * inv);
      store16(orow + k * VEC, v);
    }
  }
}

// The bf16 case with F <= 16 frames on the matrix cores: the score tile of one (position, head) fits one
// 16 x 16 MFMA tile, so a wavefront takes (position, head) pairs whole instead of a thread taking one query
// (frames beyond F: rows read again from frame F - 1, masked as keys, not stored as queries).
//   S^T[key][query] = K Q^T      16 x 16 x 32 MFMAs over d (packets beyond d are zeros); the lane ends up with
//                                keys 4 (lane / 16) .. + 3 of query lane % 16
//   softmax over the keys        in the lane and across the four lane groups (two shuffles), exact (all 16 keys at once)
//   O^T[d][query] = V^T P^T      16 x 16 x 16 MFMAs, one per 16 channels: the accumulator layout of S^T is the
//                                operand layout of P^T as it stands; V^T is read from the staged rows two bytes
//                                at a time (the four keys of a lane sit in four rows)
// and stores 8 bytes (4 channels of one query frame) per lane. The staging is the one of the kernel above.
// The vector kernel spends 3200 instructions per wavefront on 4 such pairs; this one about 100 on one.
template <int D>
__global__ __launch_bounds__(256) void temporal_attn_mfma_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ out,
                                                                 int F, int P, int heads, int np, float scale_log2e) {
  static_assert(D % 8 == 0, "whole 16-byte packets per head");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int C = heads * D, ld = 3 * C;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int b = blockIdx.y, p0 = blockIdx.x * np;
  const int npv = min(np, P - p0);
  const int ppr = ld / 8;
  const int total = F * np * ppr;
  for (int q0 = 0; q0 < total; q0 += 256) {
    const int q = min(q0 + tid, total - 1);
    const int row = q / ppr, pk = q - row * ppr;
    const int f = row / np, pos = min(row - f * np, npv - 1);  // positions beyond the end: a copy nobody reads
    const bf16_t* src = qkv + ((int64_t)(b * F + f) * P + p0 + pos) * ld + pk * 8;
#ifdef __HIP_DEVICE_COMPILE__
    __builtin_amdgcn_global_load_lds(src, smem + (q0 + wid * 64) * 16, 16, 0, 0);
#else
    (void)src;
#endif
  }
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();

  const bf16_t* rows = reinterpret_cast<const bf16_t*>(smem);
  const int i16 = lane & 15, g = lane >> 4;
  const int tasks = npv * heads;
  for (int task = wid; task < tasks; task += 4) {  // uniform over the wavefront
    const int h = task % heads, pos = task / heads;
    const bf16_t* qrow = rows + (min(i16, F - 1) * np + pos) * ld + h * D;  // frame i16: as query (B operand) and, + C, as key (A)
    f32x4 st = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int sl = 0; sl < (D + 31) / 32; ++sl) {
      const int d0 = sl * 32 + 8 * g;
      bf16x8 ka, qb;
#pragma unroll
      for (int e = 0; e < 8; ++e) ka[e] = qb[e] = (bf16_t)0.f;
      if (d0 < D) {
        ka = *reinterpret_cast<const bf16x8*>(qrow + C + d0);
        qb = *reinterpret_cast<const bf16x8*>(qrow + d0);
      }
      st = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qb, st, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (4 * g + r >= F) st[r] = -INFINITY;  // no such key (key 0 always exists: the maximum is finite)
    float mx = fmaxf(fmaxf(st[0], st[1]), fmaxf(st[2], st[3]));
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    float pe[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) pe[r] = exp2f((st[r] - mx) * scale_log2e);
    float l = (pe[0] + pe[1]) + (pe[2] + pe[3]);
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    const float inv = 1.f / l;
    bf16x4 pb;
#pragma unroll
    for (int r = 0; r < 4; ++r) pb[r] = static_cast<bf16_t>(pe[r]);
    const bf16_t* vbase = rows + pos * ld + 2 * C + h * D;  // + key * np * ld
    bf16_t* obase = out + ((int64_t)(b * F + i16) * P + p0 + pos) * C + h * D;
#pragma unroll
    for (int t = 0; t < (D + 15) / 16; ++t) {
      const int dv = min(t * 16 + i16, D - 1);  // channels beyond the head: a copy, computed and dropped
      bf16x4 va;
#pragma unroll
      for (int r = 0; r < 4; ++r) va[r] = vbase[min(4 * g + r, F - 1) * np * ld + dv];  // (weight 0 beyond F)
      const f32x4 o = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(va, pb, f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
      const int dd = t * 16 + 4 * g;  // this lane's four channels of query frame i16
      if (dd < D && i16 < F) {
        bf16x4 ov;
#pragma unroll
        for (int r = 0; r < 4; ++r) ov[r] = static_cast<bf16_t>(o[r] * inv);
        *reinterpret_cast<bf16x4*>(obase + dd) = ov;
      }
    }
  }
}

// The same for 17 <= F <= 32 frames on 32 x 32 MFMA tiles. The lane ends up with 16 keys of query lane % 32:
// keys 8 (r / 4) + 4 (lane / 32) + r % 4, r = 0..15. The contraction of O^T = V^T P^T runs over the keys in two slabs
// of 16 whose order inside a slab is free as long as both operands use the same one: slot j of lane group hh in
// slab u stands for key 16 u + 8 (j / 4) + 4 hh + j % 4, which is where accumulator r = 8 u + j already sits.
template <int D>
__global__ __launch_bounds__(256) void temporal_attn_mfma32_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ out,
                                                                   int F, int P, int heads, int np, float scale_log2e) {
  static_assert(D % 8 == 0, "whole 16-byte packets per head");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int C = heads * D, ld = 3 * C;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int b = blockIdx.y, p0 = blockIdx.x * np;
  const int npv = min(np, P - p0);
  const int ppr = ld / 8;
  const int total = F * np * ppr;
  for (int q0 = 0; q0 < total; q0 += 256) {
    const int q = min(q0 + tid, total - 1);
    const int row = q / ppr, pk = q - row * ppr;
    const int f = row / np, pos = min(row - f * np, npv - 1);  // positions beyond the end: a copy nobody reads
    const bf16_t* src = qkv + ((int64_t)(b * F + f) * P + p0 + pos) * ld + pk * 8;
#ifdef __HIP_DEVICE_COMPILE__
    __builtin_amdgcn_global_load_lds(src, smem + (q0 + wid * 64) * 16, 16, 0, 0);
#else
    (void)src;
#endif
  }
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();

  const bf16_t* rows = reinterpret_cast<const bf16_t*>(smem);
  const int i32 = lane & 31, hh = lane >> 5;
  const int tasks = npv * heads;
  for (int task = wid; task < tasks; task += 4) {  // uniform over the wavefront
    const int h = task % heads, pos = task / heads;
    const bf16_t* qrow = rows + (min(i32, F - 1) * np + pos) * ld + h * D;  // frame i32: as query (B operand) and, + C, as key (A)
    f32x16 st;
#pragma unroll
    for (int r = 0; r < 16; ++r) st[r] = 0.f;
#pragma unroll
    for (int sl = 0; sl < (D + 15) / 16; ++sl) {
      const int d0 = sl * 16 + 8 * hh;
      bf16x8 ka, qb;
#pragma unroll
      for (int e = 0; e < 8; ++e) ka[e] = qb[e] = (bf16_t)0.f;
      if (d0 < D) {
        ka = *reinterpret_cast<const bf16x8*>(qrow + C + d0);
        qb = *reinterpret_cast<const bf16x8*>(qrow + d0);
      }
      st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qb, st, 0, 0, 0);
    }
    float mx = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      if (8 * (r >> 2) + 4 * hh + (r & 3) >= F) st[r] = -INFINITY;  // no such key (key 0 always exists: the maximum is finite)
      mx = fmaxf(mx, st[r]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    float l = 0.f;
    bf16x8 pb[2];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float pe = exp2f((st[r] - mx) * scale_log2e);
      l += pe;
      pb[r >> 3][r & 7] = static_cast<bf16_t>(pe);
    }
    l += __shfl_xor(l, 32, 64);
    const float inv = 1.f / l;
    const bf16_t* vbase = rows + pos * ld + 2 * C + h * D;  // + key * np * ld
    bf16_t* obase = out + ((int64_t)(b * F + i32) * P + p0 + pos) * C + h * D;
#pragma unroll
    for (int t = 0; t < (D + 31) / 32; ++t) {
      const int dv = min(t * 32 + i32, D - 1);  // channels beyond the head: a copy, computed and dropped
      f32x16 o;
#pragma unroll
      for (int r = 0; r < 16; ++r) o[r] = 0.f;
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        bf16x8 va;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int key = 16 * u + 8 * (j >> 2) + 4 * hh + (j & 3);
          va[j] = vbase[min(key, F - 1) * np * ld + dv];  // (weight 0 beyond F)
        }
        o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[u], o, 0, 0, 0);
      }
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int dd = t * 32 + 8 * g4 + 4 * hh;  // this lane's channels dd .. dd + 3 of query frame i32
        if (dd < D && i32 < F) {
          bf16x4 ov;
#pragma unroll
          for (int r = 0; r < 4; ++r) ov[r] = static_cast<bf16_t>(o[4 * g4 + r] * inv);
          *reinterpret_cast<bf16x4*>(obase + dd) = ov;
        }
      }
    }
  }
}

// The same computation straight from global memory, for frame counts whose rows do not fit in LDS:
// thread = (batch b, position p, query frame f, head h), h fastest.
template <class T, int D>
__global__ __launch_bounds__(256) void temporal_attn_global_kernel(const T* __restrict__ qkv, T* __restrict__ out, int B,
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

template <class T, int D>
static hipError_t temporal_run(hipStream_t s, const T* qkv, T* out, int B, int F, int P, int heads, float sl) {
  const int64_t pos_bytes = (int64_t)F * 3 * heads * D * (int64_t)sizeof(T);  // LDS for one position
  if (pos_bytes + 4096 > 150 * 1024) {
    const int64_t total = (int64_t)B * P * F * heads;
    temporal_attn_global_kernel<T, D><<<(unsigned)((total + 255) / 256), 256, 0, s>>>(qkv, out, B, F, P, heads, sl);
    return hipGetLastError();
  }
  // positions per workgroup: two workgroups per compute unit if possible, at most 16 positions
  int np = (int)(32 * 1024 / pos_bytes);
  np = np < 1 ? 1 : (np > 16 ? 16 : np);
  if (np > P) np = P;
  const int64_t packets = (int64_t)F * np * (3 * heads * D / Vec16<T>::N);
  const int lds = (int)((packets + 255) / 256 * 256 * 16);  // whole rounds of 256 lanes land in LDS
  if constexpr (std::is_same<T, bf16_t>::value && D % 8 == 0) {
    if (F >= 8 && F <= 16) {  // (below 8 frames the vector kernel has less to do than a padded tile)
      auto mk = temporal_attn_mfma_kernel<D>;
      static int mk_attr_bytes = 0;  // per instantiation
      if (lds > mk_attr_bytes) {
        hipError_t e = hipFuncSetAttribute((const void*)mk, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        mk_attr_bytes = lds;
      }
      dim3 grid((unsigned)((P + np - 1) / np), (unsigned)B);
      mk<<<grid, 256, lds, s>>>(qkv, out, F, P, heads, np, sl);
      return hipGetLastError();
    }
    if (F > 16 && F <= 32) {
      auto mk = temporal_attn_mfma32_kernel<D>;
      static int mk32_attr_bytes = 0;  // per instantiation
      if (lds > mk32_attr_bytes) {
        hipError_t e = hipFuncSetAttribute((const void*)mk, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        mk32_attr_bytes = lds;
      }
      dim3 grid((unsigned)((P + np - 1) / np), (unsigned)B);
      mk<<<grid, 256, lds, s>>>(qkv, out, F, P, heads, np, sl);
      return hipGetLastError();
    }
  }
  auto kern = temporal_attn_kernel<T, D>;
  static int attr_bytes = 0;  // per instantiation
  if (lds > attr_bytes) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    attr_bytes = lds;
  }
  dim3 grid((unsigned)((P + np - 1) / np), (unsigned)B);
  kern<<<grid, 256, lds, s>>>(qkv, out, F, P, heads, np, sl);
  return hipGetLastError();
}

template <class T>
static hipError_t temporal_dispatch(hipStream_t s, const T* qkv, T* out, int B, int F, int P, int heads, int d) {
  const float sl = 1.4426950408889634f / sqrtf((float)d);
  switch (d) {
    case 8: return temporal_run<T, 8>(s, qkv, out, B, F, P, heads, sl);
    case 16: return temporal_run<T, 16>(s, qkv, out, B, F, P, heads, sl);
    case 32: return temporal_run<T, 32>(s, qkv, out, B, F, P, heads, sl);
    case 40: return temporal_run<T, 40>(s, qkv, out, B, F, P, heads, sl);
    case 64: return temporal_run<T, 64>(s, qkv, out, B, F, P, heads, sl);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_temporal_attention(hipStream_t s, int dt, const void* qkv, void* out, int B, int F, int P,
                                     int heads, int d) {
  if (B <= 0 || F <= 0 || P <= 0) return hipSuccess;
  if (dt == kBF16) return temporal_dispatch<bf16_t>(s, (const bf16_t*)qkv, (bf16_t*)out, B, F, P, heads, d);
  return temporal_dispatch<float>(s, (const float*)qkv, (float*)out, B, F, P, heads, d);
}

}  // namespace lc

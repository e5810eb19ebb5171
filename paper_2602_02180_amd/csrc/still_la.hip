// NP-Map fused into chunk-wise linear attention.
//
// Paper: Sec. 3.2 (Norm-Preserved Feature Map: u = f(x)/||f(x)|| * ||x||, phi = softmax(u) (+) softmax(-u)),
// the cache-routing equation of Sec. 3.3 (state s, z summed over the UN-selected tokens of routed chunks)
// and Algorithm 1's linear-attention branch (per-chunk phi_k(k_LA)^T v_LA, cumulative sum over chunks,
// delayed by two chunks; numerator phi_q(q) s, normaliser phi_q(q) z).
//
// The chunk scan is cut into segments so that a single long sequence still fills the chip:
//   la_state  (MODE 0): one workgroup per (batch, head, segment) sums  phi_k^T v  and  sum phi_k  over the
//                       segment's chunks; the feature map never leaves the CU.
//   la_prefix          : exclusive prefix over segments (elementwise, tiny).
//   la_out    (MODE 1): one workgroup per (batch, head, segment) starts from the prefix state and walks its
//                       chunks: N_LA, D_LA of chunk c from the state through chunk c-2, then the state
//                       absorbs chunk c-1.
// Segment s of the state pass covers chunks [s*G-1, (s+1)*G-1), so the exclusive prefix handed to the
// output pass of segment s is exactly the state through chunk s*G-2.
//
// Register/LDS plan per workgroup (NW = d/32 waves): the fp32 state S (2*d_f x d) lives in MFMA accumulators,
// wave w owning value columns [32w, 32w+32) for all features.  phi_k is staged in LDS as [feature][token]
// (A operand of S += phi_k^T V), phi_q as [token][feature] (A operand of N = phi_q S); S itself is the B
// operand of the output product straight from its accumulator registers (converted to the input dtype).
// V comes from the token-contiguous transposed copy.  z is kept in LDS in fp32.
#include "still_kernels.h"

namespace still {

template <typename T>
struct LaPad {
  static constexpr int value = 16 / sizeof(T);
};

// Feature map of 32 tokens (one per lane column).  On return pp[ft][i] / pn[ft][i] hold phi's first/second
// half at feature 32*ft + pos_of_reg(i, g) for the token of this lane.
template <typename T, int D, int DF>
__device__ __forceinline__ void np_map_tile(const T* __restrict__ xp /* row + g*KPL */,
                                            const T* __restrict__ wt_head /* [DF][D] */,
                                            const T* __restrict__ bias /* [DF] or null */, int r, int g,
                                            floatx16 (&pp)[DF / 32], floatx16 (&pn)[DF / 32]) {
  typedef Mma<T> M;
  constexpr int KS = D / M::KK;
  constexpr int FT = DF / 32;
  typename M::frag xf[KS];
  float nx2 = 0.f;
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    xf[s] = M::load(xp + s * M::KK);
    if constexpr (M::KPL == 1) {
      nx2 += xf[s] * xf[s];
    } else {
#pragma unroll
      for (int e = 0; e < M::KPL; ++e) {
        const float xv = to_f32(xf[s][e]);
        nx2 += xv * xv;
      }
    }
  }
  nx2 += xor32(nx2);
  float nf2 = 0.f;
#pragma unroll
  for (int ft = 0; ft < FT; ++ft) {
    floatx16 acc = zero16();
    const T* wrow = wt_head + (int64_t)(32 * ft + M::kappa(r)) * D + g * M::KPL;
#pragma unroll
    for (int s = 0; s < KS; ++s) acc = M::mma(M::load(wrow + s * M::KK), xf[s], acc);
    if (bias != nullptr) {
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] += to_f32(bias[32 * ft + M::pos_of_reg(i, g)]);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) nf2 += acc[i] * acc[i];
    pp[ft] = acc;
  }
  nf2 += xor32(nf2);
  const float ratio = nf2 > 0.f ? sqrtf(nx2 / nf2) : 0.f;
  float umax = -INFINITY, umin = INFINITY;
#pragma unroll
  for (int ft = 0; ft < FT; ++ft)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float u = pp[ft][i] * ratio;
      pp[ft][i] = u;
      umax = fmaxf(umax, u);
      umin = fminf(umin, u);
    }
  umax = fmaxf(umax, xor32(umax));
  umin = fminf(umin, xor32(umin));
  float sp = 0.f, sn = 0.f;
#pragma unroll
  for (int ft = 0; ft < FT; ++ft)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float u = pp[ft][i];
      const float ep = fast_exp2((u - umax) * kLog2e);
      const float en = fast_exp2((umin - u) * kLog2e);
      pp[ft][i] = ep;
      pn[ft][i] = en;
      sp += ep;
      sn += en;
    }
  sp += xor32(sp);
  sn += xor32(sn);
  const float ip = 1.0f / sp, in = 1.0f / sn;
#pragma unroll
  for (int ft = 0; ft < FT; ++ft)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      pp[ft][i] *= ip;
      pn[ft][i] *= in;
    }
}

template <typename T>
__device__ __forceinline__ float frag_dot(typename Mma<T>::frag f, const float* __restrict__ z) {
  if constexpr (Mma<T>::KPL == 1) {
    return f * z[0];
  } else {
    float acc = 0.f;
#pragma unroll
    for (int e = 0; e < Mma<T>::KPL; ++e) acc += to_f32(f[e]) * z[e];
    return acc;
  }
}

template <typename T>
__device__ __forceinline__ float frag_sum(typename Mma<T>::frag f) {
  if constexpr (Mma<T>::KPL == 1) {
    return f;
  } else {
    float acc = 0.f;
#pragma unroll
    for (int e = 0; e < Mma<T>::KPL; ++e) acc += to_f32(f[e]);
    return acc;
  }
}

template <typename T, int D, int DF, int C>
struct LaSmem {
  static constexpr int DP = 2 * DF;
  static constexpr int PAD = LaPad<T>::value;
  static constexpr int KSTRIDE = C + PAD;   // phik row stride (elements)
  static constexpr int QSTRIDE = DP + PAD;  // phiq row stride
  static constexpr size_t phik_bytes = sizeof(T) * DP * KSTRIDE;
  static constexpr size_t phiq_bytes = sizeof(T) * C * QSTRIDE;
  static constexpr size_t z_bytes = sizeof(float) * DP;
  static constexpr size_t keep_bytes = 128;
  static constexpr size_t total(int mode) { return phik_bytes + (mode ? phiq_bytes : 0) + z_bytes + keep_bytes; }
};

template <typename T, int D, int DF, int C, int MODE>
__global__ __launch_bounds__((D / 32) * 64) void la_kernel(LaArgs a) {
  typedef Mma<T> M;
  typedef LaSmem<T, D, DF, C> L;
  constexpr int DP = 2 * DF;
  constexpr int NW = D / 32;
  constexpr int FT = DF / 32;    // feature tiles per half
  constexpr int PT = DP / 32;    // feature tiles of the state
  constexpr int CT = C / 32;     // token tiles per chunk
  constexpr int SPT = M::STEPS_PER_TILE;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  T* phik = reinterpret_cast<T*>(smem);
  T* phiq = reinterpret_cast<T*>(smem + L::phik_bytes);
  float* zsh = reinterpret_cast<float*>(smem + L::phik_bytes + (MODE ? L::phiq_bytes : 0));
  unsigned char* keep = reinterpret_cast<unsigned char*>(zsh) + L::z_bytes;

  const int seg = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 31, g = lane >> 5;
  const int kvh = a.map.kv[hq];
  const int N = a.N;
  const int G = a.seg_chunks;

  const T* __restrict__ qbase = static_cast<const T*>(a.q) + (int64_t)b * a.q_sb + (int64_t)hq * a.q_sh;
  const T* __restrict__ kbase = static_cast<const T*>(a.k) + (int64_t)b * a.k_sb + (int64_t)kvh * a.k_sh;
  const T* __restrict__ vt = static_cast<const T*>(a.vt) + ((int64_t)b * a.Hkv + kvh) * (int64_t)D * a.Np;
  const T* __restrict__ wqt = static_cast<const T*>(a.wqt) + (int64_t)hq * DF * D;
  const T* __restrict__ wkt = static_cast<const T*>(a.wkt) + (int64_t)hq * DF * D;
  const T* __restrict__ bq = a.bq ? static_cast<const T*>(a.bq) + (int64_t)hq * DF : nullptr;
  const T* __restrict__ bk = a.bk ? static_cast<const T*>(a.bk) + (int64_t)hq * DF : nullptr;
  float* __restrict__ segp = a.seg + (((int64_t)b * a.Hq + hq) * a.nseg + seg) * (int64_t)(DP * (D + 1));
  const int col = 32 * wave + r;  // value column owned by this lane

  // ---- state in accumulators
  floatx16 S[PT];
  if (MODE == 1) {
#pragma unroll
    for (int ft = 0; ft < PT; ++ft)
#pragma unroll
      for (int i = 0; i < 16; ++i) S[ft][i] = segp[(int64_t)(32 * ft + M::pos_of_reg(i, g)) * D + col];
    for (int f = threadIdx.x; f < DP; f += NW * 64) zsh[f] = segp[DP * D + f];
  } else {
#pragma unroll
    for (int ft = 0; ft < PT; ++ft) S[ft] = zero16();
    for (int f = threadIdx.x; f < DP; f += NW * 64) zsh[f] = 0.f;
  }
  __syncthreads();

  // chunk range of this workgroup
  int c_beg, c_end;
  if (MODE == 1) {
    c_beg = seg * G;
    c_end = c_beg + G < a.nc ? c_beg + G : a.nc;
  } else {
    c_beg = seg * G;       // iteration c absorbs chunk c-1, like the output pass does
    c_end = c_beg + G;     // (so segment s sums chunks [sG-1, (s+1)G-1))
  }

  for (int c = c_beg; c < c_end; ++c) {
    const int cu = c - 1;                                  // chunk absorbed into the state this iteration
    // state pass: every full chunk of the segment; output pass: only while a later chunk of this
    // segment still needs the state (the next segment starts from its own prefix)
    const bool update = MODE == 0 ? (cu >= 0 && cu < a.ncf) : (cu >= 0 && c + 1 < c_end);
    // keep flags of chunk cu: 1 = token goes to the linear state
    if (update) {
      for (int i = threadIdx.x; i < C; i += NW * 64) keep[i] = 1;
      __syncthreads();
      if (a.lam > 0) {
        for (int j = threadIdx.x; j < a.lam; j += NW * 64) {
          const int tok = a.sel[(((int64_t)b * a.Hq + hq) * a.ncf + cu) * a.lam + j] - cu * C;
          if (tok >= 0 && tok < C) keep[tok] = 0;
        }
      }
      __syncthreads();
    }

    // ---- phase A: feature maps
    constexpr int NTASK = (MODE == 1 ? 2 : 1) * CT;
    for (int task = wave; task < NTASK; task += NW) {
      const bool is_q = MODE == 1 && task < CT;
      const int tt = is_q ? task : task - (MODE == 1 ? CT : 0);
      if (!is_q && !update) continue;
      floatx16 pp[FT], pn[FT];
      if (is_q) {
        const int tok = c * C + 32 * tt + r;
        const int tl = tok < N ? tok : N - 1;
        np_map_tile<T, D, DF>(qbase + (int64_t)tl * a.q_st + g * M::KPL, wqt, bq, r, g, pp, pn);
        float dla = 0.f;
        T* qrow = phiq + (32 * tt + r) * L::QSTRIDE;
#pragma unroll
        for (int ft = 0; ft < FT; ++ft)
#pragma unroll
          for (int s = 0; s < SPT; ++s) {
            const int p0 = 32 * ft + s * M::KK + g * M::KPL;
            const typename M::frag fp = M::from_acc(pp[ft], s);
            const typename M::frag fn = M::from_acc(pn[ft], s);
            *reinterpret_cast<typename M::frag*>(qrow + p0) = fp;
            *reinterpret_cast<typename M::frag*>(qrow + DF + p0) = fn;
            dla += frag_dot<T>(fp, zsh + p0) + frag_dot<T>(fn, zsh + DF + p0);
          }
        dla += xor32(dla);
        if (g == 0 && tok < N) a.d_la[((int64_t)b * a.Hq + hq) * N + tok] = dla;
      } else {
        const int tok = cu * C + 32 * tt + r;  // full chunk: always < N
        np_map_tile<T, D, DF>(kbase + (int64_t)tok * a.k_st + g * M::KPL, wkt, bk, r, g, pp, pn);
        const float kf = keep[32 * tt + r] ? 1.f : 0.f;
        T* kcol = phik + 32 * tt + r;
#pragma unroll
        for (int ft = 0; ft < FT; ++ft)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int f = 32 * ft + M::pos_of_reg(i, g);
            kcol[f * L::KSTRIDE] = from_f32<T>(pp[ft][i] * kf);
            kcol[(DF + f) * L::KSTRIDE] = from_f32<T>(pn[ft][i] * kf);
          }
      }
    }
    __syncthreads();

    // ---- phase B
    if (MODE == 1) {
      floatx16 o[CT];
#pragma unroll
      for (int mt = 0; mt < CT; ++mt) o[mt] = zero16();
#pragma unroll
      for (int ft = 0; ft < PT; ++ft)
#pragma unroll
        for (int s = 0; s < SPT; ++s) {
          const typename M::frag bf = M::from_acc(S[ft], s);
          const int p0 = 32 * ft + s * M::KK + g * M::KPL;
#pragma unroll
          for (int mt = 0; mt < CT; ++mt)
            o[mt] = M::mma(M::load(phiq + (32 * mt + r) * L::QSTRIDE + p0), bf, o[mt]);
        }
      float* nrow = a.n_la + ((int64_t)b * a.Hq + hq) * (int64_t)N * D;
#pragma unroll
      for (int mt = 0; mt < CT; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int tok = c * C + 32 * mt + c_row(i, g);
          if (tok < N) {
            float val = o[mt][i];
            if (a.g != nullptr)
              val *= to_f32(static_cast<const T*>(a.g)[(int64_t)b * a.g_sb + (int64_t)tok * a.g_st +
                                                       (int64_t)hq * a.g_sh + col]);
            nrow[(int64_t)tok * D + col] = val;
          }
        }
    }
    if (update) {
      float zp[PT];
#pragma unroll
      for (int ft = 0; ft < PT; ++ft) zp[ft] = 0.f;
      const T* vrow = vt + (int64_t)col * a.Np + (int64_t)cu * C + g * M::KPL;
#pragma unroll 4
      for (int s = 0; s < C / M::KK; ++s) {
        const typename M::frag bf = M::load(vrow + s * M::KK);
#pragma unroll
        for (int ft = 0; ft < PT; ++ft) {
          const typename M::frag af = M::load(phik + (32 * ft + M::kappa(r)) * L::KSTRIDE + s * M::KK + g * M::KPL);
          S[ft] = M::mma(af, bf, S[ft]);
          if (wave == 0) zp[ft] += frag_sum<T>(af);
        }
      }
      if (wave == 0) {
#pragma unroll
        for (int ft = 0; ft < PT; ++ft) {
          const float tot = zp[ft] + xor32(zp[ft]);
          if (g == 0) zsh[32 * ft + M::kappa(r)] += tot;
        }
      }
    }
    __syncthreads();
  }

  // ---- write the state
  float* dst = nullptr;
  if (MODE == 0) dst = segp;
  if (MODE == 1 && a.s_final != nullptr && c_end == a.nc)
    dst = a.s_final + ((int64_t)b * a.Hq + hq) * (int64_t)(DP * (D + 1));
  if (dst != nullptr) {
#pragma unroll
    for (int ft = 0; ft < PT; ++ft)
#pragma unroll
      for (int i = 0; i < 16; ++i) dst[(int64_t)(32 * ft + M::pos_of_reg(i, g)) * D + col] = S[ft][i];
    for (int f = threadIdx.x; f < DP; f += NW * 64) dst[DP * D + f] = zsh[f];
  }
}

// exclusive prefix over segments, in place: seg[s] <- sum_{s' < s} seg[s'] (slot nseg-1 is only written)
__global__ __launch_bounds__(256) void la_prefix_kernel(float* seg, int nseg, int64_t elems) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= elems) return;
  float* p = seg + (int64_t)blockIdx.y * nseg * elems + idx;
  float run = 0.f;
  for (int s = 0; s < nseg; ++s) {
    const float cur = (s + 1 < nseg) ? p[(int64_t)s * elems] : 0.f;
    p[(int64_t)s * elems] = run;
    run += cur;
  }
}

template <typename T, int D, int C, int MODE>
static hipError_t launch_la_t(const LaArgs& a, int B, int nblocks, hipStream_t stream) {
  typedef LaSmem<T, D, D, C> L;
  const size_t smem = L::total(MODE);
  auto kern = la_kernel<T, D, D, C, MODE>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) return e;
  dim3 grid(nblocks, a.Hq, B), block((D / 32) * 64);
  hipLaunchKernelGGL(kern, grid, block, smem, stream, a);
  return hipGetLastError();
}

template <int MODE>
static hipError_t launch_la_mode(const LaArgs& a, int dtype, int d, int B, int nblocks, hipStream_t stream) {
  if (nblocks <= 0) return hipSuccess;
  if (dtype == 1) {
    if (d == 64) return a.C == 64 ? launch_la_t<bf16, 64, 64, MODE>(a, B, nblocks, stream)
                                  : launch_la_t<bf16, 64, 128, MODE>(a, B, nblocks, stream);
    return a.C == 64 ? launch_la_t<bf16, 128, 64, MODE>(a, B, nblocks, stream)
                     : launch_la_t<bf16, 128, 128, MODE>(a, B, nblocks, stream);
  }
  if (d == 64) return a.C == 64 ? launch_la_t<float, 64, 64, MODE>(a, B, nblocks, stream)
                                : launch_la_t<float, 64, 128, MODE>(a, B, nblocks, stream);
  // fp32 with d = 128 and C = 128 would need more than the 160 KB of LDS; the API rejects it earlier
  if (a.C != 64) return hipErrorInvalidConfiguration;
  return launch_la_t<float, 128, 64, MODE>(a, B, nblocks, stream);
}

hipError_t launch_la_state(const LaArgs& a, int dtype, int d, int B, hipStream_t stream) {
  return launch_la_mode<0>(a, dtype, d, B, a.nseg - 1, stream);
}

hipError_t launch_la_prefix(const LaArgs& a, int d, int B, hipStream_t stream) {
  const int64_t elems = (int64_t)2 * d * (d + 1);
  dim3 grid((unsigned)((elems + 255) / 256), B * a.Hq), block(256);
  hipLaunchKernelGGL(la_prefix_kernel, grid, block, 0, stream, a.seg, a.nseg, elems);
  return hipGetLastError();
}

hipError_t launch_la_out(const LaArgs& a, int dtype, int d, int B, hipStream_t stream) {
  return launch_la_mode<1>(a, dtype, d, B, a.nseg, stream);
}

}  // namespace still

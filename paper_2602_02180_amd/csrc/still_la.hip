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
// Workgroup plan: the waves are specialised.
//   consumer waves (d/32): wave w keeps the fp32 state columns [32w, 32w+32) of S (2*d_f x d) in MFMA
//     accumulators for the whole scan and does the two token-contracting products from LDS operands:
//     S += phi_k^T V (phi_k staged as [feature][token], V from the token-contiguous transposed copy) and
//     N = phi_q S (phi_q staged as [token][feature]; S is the B operand straight from its accumulator
//     registers, converted to the input dtype).  z is kept in LDS in fp32; D_LA = phi_q z is a short
//     dot product per row.
//   producer waves (C/32): wave v computes the feature map of 32 tokens of the NEXT unit (x W on MFMA, the
//     norm re-injection and the two softmaxes on the vector ALU, which is what bounds this kernel) and
//     writes it into the other LDS slot.
// Units alternate "queries of chunk c" / "keys of chunk c-1" so that the outputs of chunk c see the state
// through chunk c-2; one barrier per unit hands a slot from producers to consumers.
#include "still_kernels.h"

namespace still {

template <typename T>
struct LaPad {
  static constexpr int value = 16 / sizeof(T);
};

// Feature map of 32 tokens (one per lane column) from their preloaded rows xf (B operand fragments).
// On return pp[ft][i] / pn[ft][i] hold phi's first / second half, multiplied by `keep`, at feature
// 32*ft + pos_of_reg(i, g) for the token of this lane.  The W^T fragments of the next feature tile are
// requested before the current tile's MFMAs so that only the first request's latency is exposed.
template <typename T, int D, int DF>
__device__ __forceinline__ void np_map_tile(const typename Mma<T>::frag (&xf)[D / Mma<T>::KK],
                                            const T* __restrict__ wt_head /* [DF][D] */,
                                            const T* __restrict__ bias /* [DF] or null */, float keep, int r,
                                            int g, floatx16 (&pp)[DF / 32], floatx16 (&pn)[DF / 32]) {
  typedef Mma<T> M;
  constexpr int KS = D / M::KK;
  constexpr int FT = DF / 32;
  float nx2 = 0.f;
#pragma unroll
  for (int s = 0; s < KS; ++s) {
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
  typename M::frag w[2][KS];
  const T* wrow = wt_head + (int64_t)M::kappa(r) * D + g * M::KPL;
#pragma unroll
  for (int s = 0; s < KS; ++s) w[0][s] = M::load(wrow + s * M::KK);
  float nf2 = 0.f, fmax = -INFINITY, fmin = INFINITY;
#pragma unroll
  for (int ft = 0; ft < FT; ++ft) {
    if (ft + 1 < FT) {
#pragma unroll
      for (int s = 0; s < KS; ++s) w[(ft + 1) & 1][s] = M::load(wrow + (int64_t)(32 * (ft + 1)) * D + s * M::KK);
    }
    __builtin_amdgcn_sched_barrier(0);  // keep the requests ahead of this tile's MFMAs
    floatx16 acc = zero16();
#pragma unroll
    for (int s = 0; s < KS; ++s) acc = M::mma(w[ft & 1][s], xf[s], acc);
    if (bias != nullptr) {
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] += to_f32(bias[32 * ft + M::pos_of_reg(i, g)]);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      nf2 = fmaf(acc[i], acc[i], nf2);
      fmax = fmaxf(fmax, acc[i]);
      fmin = fminf(fmin, acc[i]);
    }
    pp[ft] = acc;
  }
  nf2 += xor32(nf2);
  fmax = fmaxf(fmax, xor32(fmax));
  fmin = fminf(fmin, xor32(fmin));
  // u = f * ratio with ratio = ||x|| / ||f|| >= 0, so max/min of u are ratio * max/min of f;
  // exp(u - umax) = exp2(f * a1 - fmax * a1),  exp(umin - u) = exp2(fmin * a1 - f * a1)
  const float ratio = nf2 > 0.f ? sqrtf(nx2 / nf2) : 0.f;
  const float a1 = ratio * kLog2e;
  const float bp = -fmax * a1, bn = fmin * a1;
  float sp = 0.f, sn = 0.f;
#pragma unroll
  for (int ft = 0; ft < FT; ++ft)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float f = pp[ft][i];
      const float ep = fast_exp2(fmaf(f, a1, bp));
      const float en = fast_exp2(fmaf(f, -a1, bn));
      pp[ft][i] = ep;
      pn[ft][i] = en;
      sp += ep;
      sn += en;
    }
  sp += xor32(sp);
  sn += xor32(sn);
  const float ip = keep / sp, in = keep / sn;
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
  static constexpr size_t slot_bytes(int mode) {
    return (mode && phiq_bytes > phik_bytes) ? phiq_bytes : phik_bytes;
  }
  static constexpr size_t z_bytes = sizeof(float) * DP;
  static constexpr size_t total(int mode) { return 2 * slot_bytes(mode) + z_bytes; }
};

// One work unit of the scan: either the queries of chunk `chunk` (kind 0) or the keys of chunk `chunk`
// that are folded into the state (kind 1).  `valid` false = an empty pipeline slot.
struct LaUnit {
  int kind, chunk;
  bool valid;
};

template <typename T, int D, int DF, int C, int MODE>
__global__ __launch_bounds__((D / 32 + C / 32) * 64) void la_kernel(LaArgs a) {
  typedef Mma<T> M;
  typedef LaSmem<T, D, DF, C> L;
  constexpr int DP = 2 * DF;
  constexpr int NM = D / 32;     // consumer (MFMA) waves: wave w owns value columns [32w, 32w+32)
  constexpr int NV = C / 32;     // producer (feature-map) waves: wave NM+v owns tokens [32v, 32v+32) of a unit
  constexpr int FT = DF / 32;    // feature tiles per half
  constexpr int PT = DP / 32;    // feature tiles of the state
  constexpr int CT = C / 32;     // token tiles per chunk
  constexpr int SPT = M::STEPS_PER_TILE;
  constexpr size_t SLOT = L::slot_bytes(MODE);

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* zsh = reinterpret_cast<float*>(smem + 2 * SLOT);

  int seg, hq;
  head_major_block(blockIdx.x, a.Hq, hq, seg);
  const int b = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 31, g = lane >> 5;
  const bool consumer = wave < NM;
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
  const int col = 32 * wave + r;  // value column owned by this lane (consumer waves)

  // chunk range and pipeline slots of this workgroup
  const int c_beg = seg * G;
  const int c_end = MODE == 1 ? (c_beg + G < a.nc ? c_beg + G : a.nc) : c_beg + G;
  // Unit list.  Output pass: Q(c_beg), then for every later chunk c of the segment K(c-2), Q(c): the
  // outputs of chunk c see the state through chunk c-2.  State pass: K(c_beg-1) .. K(c_beg+G-2).
  // A K unit whose chunk does not exist (before the sequence start, or not a full chunk) is produced as
  // zeros, so the consumer code is straight-line.
  const int n_units = MODE == 1 ? 2 * (c_end - c_beg) - 1 : G;
  auto unit_at = [&](int u) {
    LaUnit x;
    if (MODE == 1) {
      const int j = (u + 1) >> 1;
      if ((u & 1) == 0) {
        x.kind = 0; x.chunk = c_beg + j; x.valid = true;
      } else {
        x.kind = 1; x.chunk = c_beg + j - 2; x.valid = x.chunk >= 0;
      }
    } else {
      x.kind = 1; x.chunk = c_beg + u - 1; x.valid = x.chunk >= 0 && x.chunk < a.ncf;
    }
    return x;
  };

  // ---- producer waves: feature map of 32 tokens of every unit, one unit ahead of the consumers.
  // The token rows of the following unit are requested before the current unit's arithmetic.
  // Producer and consumer waves run separate loops with the same number of barriers (the barrier counts
  // waves, and a wave never diverges inside itself here), so the state registers are live only in the
  // consumer path and the feature-map temporaries only in the producer path.
  if (!consumer) {
    constexpr int KS = D / M::KK;
    const int tt = wave - NM;
    auto row_ptr = [&](const LaUnit& x) -> const T* {
      int tok = x.chunk * C + 32 * tt + r;
      tok = tok < N ? tok : N - 1;
      tok = tok < 0 ? 0 : tok;
      return (x.kind == 0 ? qbase + (int64_t)tok * a.q_st : kbase + (int64_t)tok * a.k_st) + g * M::KPL;
    };
    typename M::frag xnext[KS];
    {
      const T* xp = row_ptr(unit_at(0));
#pragma unroll
      for (int s = 0; s < KS; ++s) xnext[s] = M::load(xp + s * M::KK);
    }
    for (int u = 0; u < n_units; ++u) {
      const LaUnit x = unit_at(u);
      typename M::frag xf[KS];
#pragma unroll
      for (int s = 0; s < KS; ++s) xf[s] = xnext[s];
      if (u + 1 < n_units) {
        const T* xp = row_ptr(unit_at(u + 1));
#pragma unroll
        for (int s = 0; s < KS; ++s) xnext[s] = M::load(xp + s * M::KK);
      }
      __builtin_amdgcn_sched_barrier(0);  // the prefetch is issued here, not sunk into the arithmetic below
      unsigned char* slot = smem + (u & 1) * SLOT;
      if (!x.valid) {
        T* kcol = reinterpret_cast<T*>(slot) + 32 * tt + r;   // absent chunk: contributes nothing
#pragma unroll 1
        for (int f = g; f < DP; f += 2) kcol[f * L::KSTRIDE] = from_f32<T>(0.f);
      } else {
        floatx16 pp[FT], pn[FT];
        if (x.kind == 0) {
          np_map_tile<T, D, DF>(xf, wqt, bq, 1.f, r, g, pp, pn);
          T* qrow = reinterpret_cast<T*>(slot) + (32 * tt + r) * L::QSTRIDE;
#pragma unroll
          for (int ft = 0; ft < FT; ++ft)
#pragma unroll
            for (int s = 0; s < SPT; ++s) {
              const int p0 = 32 * ft + s * M::KK + g * M::KPL;
              *reinterpret_cast<typename M::frag*>(qrow + p0) = M::from_acc(pp[ft], s);
              *reinterpret_cast<typename M::frag*>(qrow + DF + p0) = M::from_acc(pn[ft], s);
            }
        } else {
          const int tl = 32 * tt + r;                 // token inside the (full) chunk
          const int tok = x.chunk * C + tl;
          float kf = 1.f;                             // 0 for tokens kept by the softmax branch
          const int32_t* selc = a.sel + (((int64_t)b * a.Hq + hq) * a.ncf + x.chunk) * a.lam;
          for (int j = 0; j < a.lam; ++j) kf = (selc[j] == tok) ? 0.f : kf;
          np_map_tile<T, D, DF>(xf, wkt, bk, kf, r, g, pp, pn);
          T* kcol = reinterpret_cast<T*>(slot) + tl;
#pragma unroll
          for (int ft = 0; ft < FT; ++ft)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int f = 32 * ft + M::pos_of_reg(i, g);
              kcol[f * L::KSTRIDE] = from_f32<T>(pp[ft][i]);
              kcol[(DF + f) * L::KSTRIDE] = from_f32<T>(pn[ft][i]);
            }
        }
      }
      lds_barrier();
    }
    lds_barrier();
    return;
  }

  // ---- consumer waves: S in accumulators, z in LDS
  floatx16 S[PT];
  if (MODE == 1) {
#pragma unroll
    for (int ft = 0; ft < PT; ++ft)
#pragma unroll
      for (int i = 0; i < 16; ++i) S[ft][i] = segp[(int64_t)(32 * ft + M::pos_of_reg(i, g)) * D + col];
    for (int f = threadIdx.x; f < DP; f += NM * 64) zsh[f] = segp[DP * D + f];
  } else {
#pragma unroll
    for (int ft = 0; ft < PT; ++ft) S[ft] = zero16();
    for (int f = threadIdx.x; f < DP; f += NM * 64) zsh[f] = 0.f;
  }

  typename M::frag vf[C / M::KK];   // V fragments of the next K unit (B operand, k = tokens)
  auto load_v = [&](int u) {
    const LaUnit x = unit_at(u);
    const int ch = x.valid ? x.chunk : 0;   // an absent chunk meets zero features; any finite V will do
    const T* vrow = vt + (int64_t)col * a.Np + (int64_t)ch * C + g * M::KPL;
#pragma unroll
    for (int s = 0; s < C / M::KK; ++s) vf[s] = M::load(vrow + s * M::KK);
  };

  // S += phi_k^T V, z += sum phi_k for the unit in slot `u & 1`
  auto consume_k = [&](int u) {
    const T* phik = reinterpret_cast<const T*>(smem + (u & 1) * SLOT);
#pragma unroll
    for (int s = 0; s < C / M::KK; ++s) {
#pragma unroll
      for (int ft = 0; ft < PT; ++ft) {
        const typename M::frag af = M::load(phik + (32 * ft + M::kappa(r)) * L::KSTRIDE + s * M::KK + g * M::KPL);
        S[ft] = M::mma(af, vf[s], S[ft]);
      }
    }
    // row sums of the same LDS rows, PT/NM feature tiles per consumer wave, outside the MFMA loop
    constexpr int ZT = PT / NM;
#pragma unroll 1
    for (int j = 0; j < ZT; ++j) {
      const int ft = wave * ZT + j;
      const T* zrow = phik + (32 * ft + r) * L::KSTRIDE + g * M::KPL;
      float zp = 0.f;
#pragma unroll
      for (int s = 0; s < C / M::KK; ++s) zp += frag_sum<T>(M::load(zrow + s * M::KK));
      zp += xor32(zp);
      if (g == 0) zsh[32 * ft + r] += zp;
    }
  };

  // N_LA = phi_q S and D_LA = phi_q z for the rows of the chunk in slot `u & 1`
  auto consume_q = [&](int u) {
    const LaUnit x = unit_at(u);
    const T* phiq = reinterpret_cast<const T*>(smem + (u & 1) * SLOT);
    float* nrow = a.n_la + ((int64_t)b * a.Hq + hq) * (int64_t)N * D;
    // two token tiles at a time keeps the accumulators next to the state registers
#pragma unroll 1
    for (int mh = 0; mh < CT; mh += 2) {
      floatx16 o[2];
      o[0] = zero16();
      o[1] = zero16();
#pragma unroll
      for (int ft = 0; ft < PT; ++ft)
#pragma unroll
        for (int s = 0; s < SPT; ++s) {
          const typename M::frag bf = M::from_acc(S[ft], s);
          const int p0 = 32 * ft + s * M::KK + g * M::KPL;
          o[0] = M::mma(M::load(phiq + (32 * mh + r) * L::QSTRIDE + p0), bf, o[0]);
          o[1] = M::mma(M::load(phiq + (32 * mh + 32 + r) * L::QSTRIDE + p0), bf, o[1]);
        }
#pragma unroll
      for (int mm = 0; mm < 2; ++mm)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int tok = x.chunk * C + 32 * (mh + mm) + c_row(i, g);
          if (tok < N) {
            float val = o[mm][i];
            if (a.g != nullptr)
              val *= to_f32(static_cast<const T*>(a.g)[(int64_t)b * a.g_sb + (int64_t)tok * a.g_st +
                                                       (int64_t)hq * a.g_sh + col]);
            nrow[(int64_t)tok * D + col] = val;
          }
        }
    }
    // D_LA: this wave's share of the chunk's rows; lane group g sums feature half g
    constexpr int TPW = C / NM;
    for (int j = r; j < TPW; j += 32) {
      const int tl = wave * TPW + j;
      const T* qrow = phiq + tl * L::QSTRIDE + g * DF;
      const float* zz = zsh + g * DF;
      float dla = 0.f;
#pragma unroll 4
      for (int f0 = 0; f0 < DF; f0 += M::KPL) dla += frag_dot<T>(M::load(qrow + f0), zz + f0);
      dla += xor32(dla);
      const int tok = x.chunk * C + tl;
      if (g == 0 && tok < N) a.d_la[((int64_t)b * a.Hq + hq) * N + tok] = dla;
    }
  };

  if (MODE == 1) {
    if (n_units > 1) load_v(1);
    lds_barrier();
    consume_q(0);
    lds_barrier();
    for (int u = 1; u + 1 < n_units; u += 2) {
      consume_k(u);
      lds_barrier();
      // V of the next K unit is requested BEFORE this unit's N_LA stores: the vector-memory counter retires
      // in order, so a later wait for these loads does not have to wait for the stores as well
      if (u + 2 < n_units) load_v(u + 2);
      __builtin_amdgcn_sched_barrier(0);
      consume_q(u + 1);
      lds_barrier();
    }
  } else {
    load_v(0);
    lds_barrier();
    for (int u = 0; u < n_units; ++u) {
      consume_k(u);
      if (u + 1 < n_units) load_v(u + 1);
      lds_barrier();
    }
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
    for (int f = threadIdx.x; f < DP; f += NM * 64) dst[DP * D + f] = zsh[f];
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
  dim3 grid(nblocks * a.Hq, 1, B), block((D / 32 + C / 32) * 64);
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

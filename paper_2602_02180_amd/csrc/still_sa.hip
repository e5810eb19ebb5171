// Sparse softmax branch over the salient cache, fused with the merge of both branches.
//
// Paper: Sec. 3.3 output equations.  Row t of chunk c attends with exp(scale q.k) to
//   (i)  the retained keys/values of chunks <= c-2 (Algorithm 1: flattened selected K/V under M^Chunk),
//   (ii) the whole previous chunk and its own chunk up to t (s_prev, s_in with the causal mask),
// giving N_SA, D_SA; the epilogue adds the linear-attention terms and divides once:
//   y = (N_SA + N_LA) / (D_SA + D_LA).
// The softmax sums are kept relative to a running maximum m (online softmax); the linear terms are not
// exponentials, so both branches are brought to the common factor exp(-max(m, 0)) before the division
// (any common positive factor cancels; this one can neither overflow nor lose the larger branch).
//
// One workgroup = 128 consecutive query rows of one (batch, query head), 4 waves x 32 rows.
// Everything is computed transposed so that one lane owns one query row:
//   S^T (keys x queries)  = K_tile (A operand, from LDS)  x  Q^T (B operand, registers)
//   O^T (d    x queries) += V^T_tile (A operand, from LDS) x  P^T (B operand = S^T accumulators, in place)
// Row statistics are then per-lane reductions plus one exchange with lane^32 per tile.
// K tiles (64 keys x d) and V^T tiles (d x 64 keys) are double-buffered in LDS: one barrier per tile, the
// global loads of tile i+2 are in flight while tile i+1 is computed.  Retained keys come from the compacted
// per-head buffers, local keys from k and from the token-contiguous transposed copy of v.
// Workgroups of one (batch, head) are placed on one XCD (block ids are dealt round-robin to the 8 XCDs), so
// the head's retained K/V (2 MB at 32K tokens) is served from that XCD's L2; long rows are scheduled first.
#include "still_kernels.h"

namespace still {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <typename T, int D>
struct SaCfg {
  typedef Mma<T> M;
  static constexpr int BM = 128, BN = 64, NW = 4;
  static constexpr int PAD = 16 / sizeof(T);
  static constexpr int KST = D + PAD;    // K tile row stride (elements)
  static constexpr int VST = BN + PAD;   // V^T tile row stride
  static constexpr int EPV = 16 / sizeof(T);                 // elements per 16-byte vector
  static constexpr int KPT = BN * D / EPV / 256;             // 16-byte vectors per thread, K tile
  static constexpr int VPT = D * BN / EPV / 256;             // same, V^T tile
  static constexpr int BUF_ELEMS = BN * KST + D * VST;
  static constexpr size_t smem_bytes = 2 * sizeof(T) * BUF_ELEMS;
};

// MASK: 0 = every key of the tile is visible to every row of the wave, 1 = retained tile with a ragged end,
//       2 = local tile (window start and causal limit)
template <typename T, int D, int MASK>
__device__ __forceinline__ void sa_tile(const T* __restrict__ Ks, const T* __restrict__ Vs,
                                        const typename Mma<T>::frag (&qf)[D / Mma<T>::KK], floatx16 (&o)[D / 32],
                                        float& m2, float& lpart, int kb, int ret_w, int lo_w, int t, float sc2,
                                        int r, int g) {
  typedef Mma<T> M;
  typedef SaCfg<T, D> Cf;
  constexpr int KS = D / M::KK;
  constexpr int DT = D / 32;
  constexpr int SPT = M::STEPS_PER_TILE;

  floatx16 st[2];
  st[0] = zero16();
  st[1] = zero16();
  const T* krow = Ks + r * Cf::KST + g * M::KPL;
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    st[0] = M::mma(M::load(krow + s * M::KK), qf[s], st[0]);
    st[1] = M::mma(M::load(krow + 32 * Cf::KST + s * M::KK), qf[s], st[1]);
  }
  if (MASK != 0) {
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = kb + 32 * mt + M::pos_of_reg(i, g);
        const bool valid = MASK == 1 ? (key < ret_w) : (key >= lo_w && key <= t);
        st[mt][i] = valid ? st[mt][i] : -INFINITY;
      }
  }
  float tmax = st[0][0];
#pragma unroll
  for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, st[0][i]);
#pragma unroll
  for (int i = 0; i < 16; ++i) tmax = fmaxf(tmax, st[1][i]);
  tmax = fmaxf(tmax, xor32(tmax));
  const float m_new = fmaxf(m2, tmax * sc2);
  const float m_sub = (MASK != 0 && m_new == -INFINITY) ? 0.f : m_new;
  if (__any(m_new > m2)) {  // wave-uniform: skip the rescale once the running maxima have settled
    const float alpha = fast_exp2(m2 - m_sub);
    lpart *= alpha;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[dt][i] *= alpha;
  }
  m2 = m_new;
  float rs = 0.f;
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float pv = fast_exp2(fmaf(st[mt][i], sc2, -m_sub));
      st[mt][i] = pv;
      rs += pv;
    }
  lpart += rs;
  // O^T += V^T P^T
  const T* vrow = Vs + r * Cf::VST + g * M::KPL;
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int s = 0; s < SPT; ++s) {
      const typename M::frag pf = M::from_acc(st[mt], s);
      const int koff = 32 * mt + s * M::KK;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) o[dt] = M::mma(M::load(vrow + 32 * dt * Cf::VST + koff), pf, o[dt]);
    }
}

template <typename T, int D>
__global__ __launch_bounds__(256, 2) void sa_kernel(SaArgs a) {
  typedef Mma<T> M;
  typedef SaCfg<T, D> Cf;
  constexpr int KS = D / M::KK;
  constexpr int DT = D / 32;
  constexpr int BN = Cf::BN;
  constexpr int VR = D / Cf::EPV;   // 16-byte vectors per K row
  constexpr int VV = BN / Cf::EPV;  // 16-byte vectors per V^T row

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  T* lds = reinterpret_cast<T*>(smem);

  // block id -> (unit = batch*Hq + head, row tile); units are dealt to XCDs, long tiles first
  int unit, tile;
  {
    const int L = blockIdx.x;
    const int units = a.Hq * a.B_;
    if (units % 8 == 0) {
      const int xcd = L & 7, j = L >> 3;
      unit = (j / a.ntiles) * 8 + xcd;
      tile = a.ntiles - 1 - (j % a.ntiles);
    } else {
      unit = L / a.ntiles;
      tile = a.ntiles - 1 - (L % a.ntiles);
    }
  }
  const int b = unit / a.Hq, hq = unit % a.Hq;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, g = lane >> 5;
  const int N = a.N, C = a.C, lam = a.lam;
  const int kvh = a.map.kv[hq];

  const int row0 = tile * Cf::BM;
  const int q0 = row0 + 32 * wave;
  const int t = q0 + r;
  const bool wave_active = q0 < N;
  const int cw = q0 / C;
  const int ret_w = (cw >= 1 ? cw - 1 : 0) * lam;     // retained keys visible to this wave
  const int lo_w = (cw >= 1 ? cw - 1 : 0) * C;        // first local key of this wave
  const int c_first = row0 / C;
  const int last_row = (row0 + Cf::BM - 1 < N - 1) ? row0 + Cf::BM - 1 : N - 1;
  const int c_last = last_row / C;
  const int ret_max = (c_last >= 1 ? c_last - 1 : 0) * lam;
  const int loc_lo = (c_first >= 1 ? c_first - 1 : 0) * C;
  const int n_ret_tiles = (ret_max + BN - 1) / BN;
  const int n_tiles = n_ret_tiles + (last_row + 1 - loc_lo + BN - 1) / BN;

  const T* __restrict__ kloc = static_cast<const T*>(a.k) + (int64_t)b * a.k_sb + (int64_t)kvh * a.k_sh;
  const T* __restrict__ vtl = static_cast<const T*>(a.vt) + ((int64_t)b * a.Hkv + kvh) * (int64_t)D * a.Np;
  const T* __restrict__ kret = static_cast<const T*>(a.kret) + ((int64_t)b * a.Hq + hq) * (int64_t)a.cap * D;
  const T* __restrict__ vrett = static_cast<const T*>(a.vrett) + ((int64_t)b * a.Hq + hq) * (int64_t)D * a.cap;

  // per-thread slots of the cooperative tile copy
  const int kp = tid / VR, kvec = tid % VR;           // K: row kp (+ 256/VR per step), vector kvec
  const int vx = tid / VV, vvec = tid % VV;           // V^T: row vx (+ 256/VV per step), vector vvec
  constexpr int KROWS_PER_STEP = 256 / VR;
  constexpr int VROWS_PER_STEP = 256 / VV;

  u32x4 kreg[Cf::KPT], vreg[Cf::VPT];

#define SA_GLOAD(TI)                                                                                       \
  {                                                                                                        \
    const int ti_ = (TI);                                                                                  \
    const bool ret_ = ti_ < n_ret_tiles;                                                                   \
    const int kb_ = ret_ ? ti_ * BN : loc_lo + (ti_ - n_ret_tiles) * BN;                                   \
    _Pragma("unroll") for (int j = 0; j < Cf::KPT; ++j) {                                                  \
      const int p_ = kp + j * KROWS_PER_STEP;                                                              \
      int tok_ = kb_ + p_;                                                                                 \
      tok_ = tok_ < N ? tok_ : N - 1;                                                                      \
      const T* src_ = ret_ ? kret + (int64_t)(kb_ + p_) * D : kloc + (int64_t)tok_ * a.k_st;               \
      kreg[j] = *reinterpret_cast<const u32x4*>(src_ + kvec * Cf::EPV);                                    \
    }                                                                                                      \
    const T* vsrc_ = ret_ ? vrett : vtl;                                                                   \
    const int64_t vstride_ = ret_ ? a.cap : a.Np;                                                          \
    _Pragma("unroll") for (int j = 0; j < Cf::VPT; ++j) {                                                  \
      const int x_ = vx + j * VROWS_PER_STEP;                                                              \
      vreg[j] = *reinterpret_cast<const u32x4*>(vsrc_ + (int64_t)x_ * vstride_ + kb_ + vvec * Cf::EPV);    \
    }                                                                                                      \
  }

#define SA_LSTORE(BUF)                                                                                     \
  {                                                                                                        \
    T* Ks_ = lds + (BUF) * Cf::BUF_ELEMS;                                                                  \
    T* Vs_ = Ks_ + BN * Cf::KST;                                                                           \
    _Pragma("unroll") for (int j = 0; j < Cf::KPT; ++j) {                                                  \
      const int p_ = kp + j * KROWS_PER_STEP;                                                              \
      const int row_ = (p_ & ~31) + M::kappa_inv(p_ & 31);                                                 \
      *reinterpret_cast<u32x4*>(Ks_ + row_ * Cf::KST + kvec * Cf::EPV) = kreg[j];                          \
    }                                                                                                      \
    _Pragma("unroll") for (int j = 0; j < Cf::VPT; ++j) {                                                  \
      const int x_ = vx + j * VROWS_PER_STEP;                                                              \
      *reinterpret_cast<u32x4*>(Vs_ + x_ * Cf::VST + vvec * Cf::EPV) = vreg[j];                            \
    }                                                                                                      \
  }

  // queries of this wave (B operand of S^T = K Q^T)
  typename M::frag qf[KS];
  {
    const int tq = t < N ? t : N - 1;
    const T* qp = static_cast<const T*>(a.q) + (int64_t)b * a.q_sb + (int64_t)tq * a.q_st + (int64_t)hq * a.q_sh +
                  g * M::KPL;
#pragma unroll
    for (int s = 0; s < KS; ++s) qf[s] = M::load(qp + s * M::KK);
  }

  floatx16 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) o[dt] = zero16();
  float m2 = -INFINITY, lpart = 0.f;
  const float sc2 = a.scale * kLog2e;

  SA_GLOAD(0);
  SA_LSTORE(0);
  lds_barrier();
  if (n_tiles > 1) SA_GLOAD(1);

  for (int ti = 0; ti < n_tiles; ++ti) {
    const bool ret = ti < n_ret_tiles;
    const int kb = ret ? ti * BN : loc_lo + (ti - n_ret_tiles) * BN;
    const T* Ks = lds + (ti & 1) * Cf::BUF_ELEMS;
    const T* Vs = Ks + BN * Cf::KST;
    if (wave_active) {
      if (ret) {
        if (kb + BN <= ret_w)
          sa_tile<T, D, 0>(Ks, Vs, qf, o, m2, lpart, kb, ret_w, lo_w, t, sc2, r, g);
        else if (kb < ret_w)
          sa_tile<T, D, 1>(Ks, Vs, qf, o, m2, lpart, kb, ret_w, lo_w, t, sc2, r, g);
      } else if (kb + BN - 1 >= lo_w && kb <= q0 + 31) {
        if (kb >= lo_w && kb + BN - 1 <= q0)
          sa_tile<T, D, 0>(Ks, Vs, qf, o, m2, lpart, kb, ret_w, lo_w, t, sc2, r, g);
        else
          sa_tile<T, D, 2>(Ks, Vs, qf, o, m2, lpart, kb, ret_w, lo_w, t, sc2, r, g);
      }
    }
    if (ti + 1 < n_tiles) SA_LSTORE((ti + 1) & 1);
    lds_barrier();
    if (ti + 2 < n_tiles) SA_GLOAD(ti + 2);
  }
#undef SA_GLOAD
#undef SA_LSTORE

  // ---- merge epilogue
  if (wave_active && t < N) {
    const float l = lpart + xor32(lpart);
    float fs, fl;
    if (m2 >= 0.f) {
      fs = 1.f;
      fl = fast_exp2(-m2);
    } else {
      fs = fast_exp2(m2);
      fl = 1.f;
    }
    const int64_t rowi = ((int64_t)b * a.Hq + hq) * N + t;
    const float dla = a.d_la[rowi];
    const float inv = 1.0f / (fs * l + fl * dla);
    const float* nrow = a.n_la + rowi * D;
    T* orow = static_cast<T*>(a.out) + (int64_t)b * a.o_sb + (int64_t)t * a.o_st + (int64_t)hq * a.o_sh;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int dcol = 32 * dt + 8 * i4 + 4 * g;
        const floatx4 nl = *reinterpret_cast<const floatx4*>(nrow + dcol);
        float y[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) y[e] = (fs * o[dt][4 * i4 + e] + fl * nl[e]) * inv;
        if constexpr (sizeof(T) == 2) {
          bf16x4 ov;
#pragma unroll
          for (int e = 0; e < 4; ++e) ov[e] = static_cast<bf16>(y[e]);
          *reinterpret_cast<bf16x4*>(orow + dcol) = ov;
        } else {
          floatx4 ov;
#pragma unroll
          for (int e = 0; e < 4; ++e) ov[e] = y[e];
          *reinterpret_cast<floatx4*>(orow + dcol) = ov;
        }
      }
  }
}

template <typename T, int D>
static hipError_t launch_sa_t(const SaArgs& a, int B, hipStream_t stream) {
  typedef SaCfg<T, D> Cf;
  auto kern = sa_kernel<T, D>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)Cf::smem_bytes);
  if (e != hipSuccess) return e;
  dim3 grid((unsigned)(a.ntiles * a.Hq * B)), block(256);
  hipLaunchKernelGGL(kern, grid, block, Cf::smem_bytes, stream, a);
  return hipGetLastError();
}

hipError_t launch_sa(const SaArgs& a, int dtype, int d, int B, hipStream_t stream) {
  if (dtype == 1) return d == 64 ? launch_sa_t<bf16, 64>(a, B, stream) : launch_sa_t<bf16, 128>(a, B, stream);
  return d == 64 ? launch_sa_t<float, 64>(a, B, stream) : launch_sa_t<float, 128>(a, B, stream);
}

}  // namespace still

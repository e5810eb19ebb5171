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
// Row statistics are then plain per-lane reductions plus one exchange with lane^32.
// K tiles (64 keys x d) and V^T tiles (d x 64 keys) are staged through LDS once per workgroup; the next
// tile's global loads are issued before the current tile's MFMAs.  Retained keys come from the compacted
// per-head buffers, local keys from k and from the token-contiguous transposed copy of v.
#include "still_kernels.h"

namespace still {

template <typename T, int D>
struct SaCfg {
  typedef Mma<T> M;
  static constexpr int BM = 128, BN = 64, NW = 4;
  static constexpr int PAD = 16 / sizeof(T);
  static constexpr int KST = D + PAD;    // K tile row stride (elements)
  static constexpr int VST = BN + PAD;   // V^T tile row stride
  static constexpr int EPV = 16 / sizeof(T);                 // elements per 16-byte vector
  static constexpr int KVEC = BN * D / EPV;                  // vectors in a K tile
  static constexpr int KPT = KVEC / 256;                     // per thread
  static constexpr int VVEC = D * BN / EPV;
  static constexpr int VPT = VVEC / 256;
  static constexpr size_t smem_bytes = sizeof(T) * (BN * KST + D * VST);
};

template <typename T, int D>
__global__ __launch_bounds__(256) void sa_kernel(SaArgs a) {
  typedef Mma<T> M;
  typedef SaCfg<T, D> Cf;
  constexpr int KS = D / M::KK;
  constexpr int DT = D / 32;
  constexpr int SPT = M::STEPS_PER_TILE;
  constexpr int BN = Cf::BN;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  T* Ks = reinterpret_cast<T*>(smem);
  T* Vs = Ks + BN * Cf::KST;

  const int tile = a.ntiles - 1 - (int)blockIdx.x;  // long rows first
  const int hq = blockIdx.y, b = blockIdx.z;
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
  const int loc_hi = last_row + 1;
  const int n_ret_tiles = (ret_max + BN - 1) / BN;
  const int n_tiles = n_ret_tiles + (loc_hi - loc_lo + BN - 1) / BN;

  const T* __restrict__ kloc = static_cast<const T*>(a.k) + (int64_t)b * a.k_sb + (int64_t)kvh * a.k_sh;
  const T* __restrict__ vtl = static_cast<const T*>(a.vt) + ((int64_t)b * a.Hkv + kvh) * (int64_t)D * a.Np;
  const T* __restrict__ kret = static_cast<const T*>(a.kret) + ((int64_t)b * a.Hq + hq) * (int64_t)a.cap * D;
  const T* __restrict__ vrett = static_cast<const T*>(a.vrett) + ((int64_t)b * a.Hq + hq) * (int64_t)D * a.cap;

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
  float m2 = -INFINITY, l = 0.f;
  const float sc2 = a.scale * kLog2e;

  Vec16 kreg[Cf::KPT], vreg[Cf::VPT];

  auto gload = [&](int ti) {
    const bool ret = ti < n_ret_tiles;
    const int kb = ret ? ti * BN : loc_lo + (ti - n_ret_tiles) * BN;
    constexpr int VR = D / Cf::EPV;  // vectors per K row
#pragma unroll
    for (int j = 0; j < Cf::KPT; ++j) {
      const int idx = tid + 256 * j;
      const int p = idx / VR, vec = idx % VR;
      const T* src;
      if (ret) {
        src = kret + (int64_t)(kb + p) * D;
      } else {
        int tok = kb + p;
        tok = tok < N ? tok : N - 1;
        src = kloc + (int64_t)tok * a.k_st;
      }
      kreg[j] = *reinterpret_cast<const Vec16*>(src + vec * Cf::EPV);
    }
    constexpr int VV = BN / Cf::EPV;  // vectors per V^T row
    const T* vsrc = ret ? vrett : vtl;
    const int64_t vstride = ret ? a.cap : a.Np;
#pragma unroll
    for (int j = 0; j < Cf::VPT; ++j) {
      const int idx = tid + 256 * j;
      const int x = idx / VV, vec = idx % VV;
      vreg[j] = *reinterpret_cast<const Vec16*>(vsrc + (int64_t)x * vstride + kb + vec * Cf::EPV);
    }
  };

  auto lstore = [&]() {
    constexpr int VR = D / Cf::EPV;
#pragma unroll
    for (int j = 0; j < Cf::KPT; ++j) {
      const int idx = tid + 256 * j;
      const int p = idx / VR, vec = idx % VR;
      const int row = (p & ~31) + M::kappa_inv(p & 31);
      *reinterpret_cast<Vec16*>(Ks + row * Cf::KST + vec * Cf::EPV) = kreg[j];
    }
    constexpr int VV = BN / Cf::EPV;
#pragma unroll
    for (int j = 0; j < Cf::VPT; ++j) {
      const int idx = tid + 256 * j;
      const int x = idx / VV, vec = idx % VV;
      *reinterpret_cast<Vec16*>(Vs + x * Cf::VST + vec * Cf::EPV) = vreg[j];
    }
  };

  if (n_tiles > 0) gload(0);
  for (int ti = 0; ti < n_tiles; ++ti) {
    __syncthreads();
    lstore();
    __syncthreads();
    if (ti + 1 < n_tiles) gload(ti + 1);

    const bool ret = ti < n_ret_tiles;
    const int kb = ret ? ti * BN : loc_lo + (ti - n_ret_tiles) * BN;
    bool relevant, need_mask;
    if (ret) {
      relevant = kb < ret_w;
      need_mask = kb + BN > ret_w;
    } else {
      relevant = (kb + BN - 1 >= lo_w) && (kb <= q0 + 31);
      need_mask = (kb < lo_w) || (kb + BN - 1 > q0);
    }
    if (!wave_active || !relevant) continue;

    floatx16 st[2];
    st[0] = zero16();
    st[1] = zero16();
#pragma unroll
    for (int s = 0; s < KS; ++s) {
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        const typename M::frag af = M::load(Ks + (32 * mt + r) * Cf::KST + s * M::KK + g * M::KPL);
        st[mt] = M::mma(af, qf[s], st[mt]);
      }
    }
    // logits in the log2 domain, masked
    float tmax = -INFINITY;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        float x = st[mt][i] * sc2;
        if (need_mask) {
          const int key = kb + 32 * mt + M::pos_of_reg(i, g);
          const bool valid = ret ? (key < ret_w) : (key >= lo_w && key <= t);
          x = valid ? x : -INFINITY;
        }
        st[mt][i] = x;
        tmax = fmaxf(tmax, x);
      }
    tmax = fmaxf(tmax, xor32(tmax));
    const float m_new = fmaxf(m2, tmax);
    const float m_sub = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = fast_exp2(m2 - m_sub);
    float rs = 0.f;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float pv = fast_exp2(st[mt][i] - m_sub);
        st[mt][i] = pv;
        rs += pv;
      }
    rs += xor32(rs);
    l = l * alpha + rs;
    m2 = m_new;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[dt][i] *= alpha;
    // O^T += V^T P^T
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int s = 0; s < SPT; ++s) {
        const typename M::frag pf = M::from_acc(st[mt], s);
        const int koff = 32 * mt + s * M::KK + g * M::KPL;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          const typename M::frag vf = M::load(Vs + (32 * dt + r) * Cf::VST + koff);
          o[dt] = M::mma(vf, pf, o[dt]);
        }
      }
  }

  // ---- merge epilogue
  if (wave_active && t < N) {
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
  dim3 grid(a.ntiles, a.Hq, B), block(256);
  hipLaunchKernelGGL(kern, grid, block, Cf::smem_bytes, stream, a);
  return hipGetLastError();
}

hipError_t launch_sa(const SaArgs& a, int dtype, int d, int B, hipStream_t stream) {
  if (dtype == 1) return d == 64 ? launch_sa_t<bf16, 64>(a, B, stream) : launch_sa_t<bf16, 128>(a, B, stream);
  return d == 64 ? launch_sa_t<float, 64>(a, B, stream) : launch_sa_t<float, 128>(a, B, stream);
}

}  // namespace still

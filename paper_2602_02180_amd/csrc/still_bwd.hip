// Backward pass of the prefill operator, the routing held fixed (gfx950).
//
// What is differentiated is the output equation of Sec. 3.3, y = (N_SA + g N_LA) / (D_SA + D_LA), for the index
// lists the forward pass chose: the Top-lambda selection is a discrete decision and passes no gradient, and the
// Self-Saliency Score of Sec. 3.1 only feeds that decision.  With L_t = ln(D_SA + D_LA) (kept by the forward pass),
// delta_t = dy_t . y_t and E_t = exp(-L_t):
//   softmax branch, key j visible to row t through exp:   P_tj = exp(scale q_t.k_j - L_t)
//        dv_j += P_tj dy_t          dl_tj = P_tj (dy_t . v_j - delta_t)
//        dq_t += scale dl_tj k_j    dk_j += scale dl_tj q_t
//   linear branch, S = sum phi_k(k_j)^T v_j and z = sum phi_k(k_j) over the un-selected tokens of chunks <= c-2:
//        A_t = E_t (g_t * dy_t)                     (per channel)
//        dphi_q(t) = S A_t - E_t delta_t z          dg_t = E_t dy_t * (phi_q(t) S)
//        dS(c) = sum over the rows of chunks >= c+2 of phi_q(t)^T A_t,   dz(c) likewise of phi_q(t) E_t delta_t
//        dphi_k(j) = dS(c_j) v_j - dz(c_j)          dv_j += dS(c_j)^T phi_k(j)
//   and the NP-Map of Sec. 3.2 (f = x W + b, u = f |x| / |f|, phi = [softmax(u), softmax(-u)]) backwards:
//        du = phi+ (dphi+ - <phi+, dphi+>) - phi- (dphi- - <phi-, dphi->)
//        df = (|x| / |f|) (du - fh <fh, du>),  fh = f / |f|;   dx = df W^T + <fh, du> x / |x|;   dW = x^T df
//
// This first version keeps every step a separate, simple kernel: the sparse branch as two tile kernels (one that
// owns query rows and produces dq, one that owns key tiles and produces dk, dv), the linear branch as a sequence of
// batched products on one generic 64 x 64 MFMA tile kernel with element-wise kernels between them, intermediates in
// the workspace.  All sums are fp32; operands of the matrix core are in the storage type.
#include "still_kernels.h"

namespace still {

namespace {

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  return x;
}

// ---------------------------------------------------------------------------------------------------------
// Generic batched product on the matrix core: C[m][n] (=, +=, atomic +=) sum_k A(m, k) B(n, k) [+ sum_k A(m, k)
// B2(n, k)], one 64 x BN tile of one batch item per workgroup (four waves as 2 x 2, each 32 x BN/2), both operands
// through LDS in the storage type with the contraction index contiguous, 64 contraction entries per barrier pair.
// Operands are addressed through explicit strides.  Every global access is a 16-byte (32-byte for fp32 data) vector
// along the operand's contiguous index: for an operand whose contraction index is contiguous the vector goes to LDS
// as it is; for one whose row index is contiguous (a transposed view) its eight elements go to eight LDS rows, the
// lanes of a wave then covering consecutive k so that neither side meets bank conflicts.
// ---------------------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void load8(float (&x)[8], const void* base, int64_t off, int is_f32) {
  if (is_f32) {
    const floatx4 a = *reinterpret_cast<const floatx4*>(static_cast<const float*>(base) + off);
    const floatx4 b = *reinterpret_cast<const floatx4*>(static_cast<const float*>(base) + off + 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) { x[e] = a[e]; x[4 + e] = b[e]; }
  } else if constexpr (sizeof(T) == 2) {
    const bf16x8 v = *reinterpret_cast<const bf16x8*>(static_cast<const T*>(base) + off);
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = static_cast<float>(v[e]);
  } else {
    const floatx4 a = *reinterpret_cast<const floatx4*>(static_cast<const float*>(base) + off);
    const floatx4 b = *reinterpret_cast<const floatx4*>(static_cast<const float*>(base) + off + 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) { x[e] = a[e]; x[4 + e] = b[e]; }
  }
}

// ROWS x 64 tile of one operand into LDS [ROWS][LDK]; rows at and beyond row_valid and contraction entries at and
// beyond k_valid read as zero
template <typename T, int ROWS, int LDK>
__device__ __forceinline__ void load_operand(T* dst, const GemmOperand& o, int64_t off, int row0, int row_valid, int k0,
                                             int k_valid, int tid) {
  constexpr int NV = ROWS * 64 / 8 / 256;   // vectors per thread
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int idx = tid + 256 * j;
    float x[8];
    if (o.s_k == 1) {        // contraction index contiguous: vector along k
      const int row = idx / 8, kv = (idx % 8) * 8;
      const bool ok = row0 + row < row_valid && k0 + kv < k_valid;
      if (ok) load8<T>(x, o.base, off + (int64_t)(row0 + row) * o.s_r + (k0 + kv), o.f32);
      T* d = dst + row * LDK + kv;
      if constexpr (sizeof(T) == 2) {
        bf16x8 v;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = static_cast<bf16>(ok ? x[e] : 0.f);
        *reinterpret_cast<bf16x8*>(d) = v;
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) d[e] = ok ? x[e] : 0.f;
      }
    } else {                 // row index contiguous: vector along rows, lanes along k
      const int kk = idx % 64, rv = (idx / 64) * 8;
      const bool ok = k0 + kk < k_valid && row0 + rv < row_valid;
      if (ok) load8<T>(x, o.base, off + (int64_t)(row0 + rv) + (int64_t)(k0 + kk) * o.s_k, o.f32);
#pragma unroll
      for (int e = 0; e < 8; ++e) dst[(rv + e) * LDK + kk] = from_f32<T>(ok ? x[e] : 0.f);
    }
  }
}

template <typename T, int BN>
__global__ __launch_bounds__(256) void bgemm_kernel(GemmArgs a) {
  typedef Mma<T> M;
  constexpr int BK = 64, NT = BN / 64;
  constexpr int LDK = BK + (sizeof(T) == 2 ? 8 : 4);
  __shared__ __attribute__((aligned(16))) T As[64 * LDK];
  __shared__ __attribute__((aligned(16))) T Bs[BN * LDK];
  const int unit = blockIdx.z, c = blockIdx.y;
  const int ntn = a.Nn / BN;
  const int mt = blockIdx.x / ntn, nt = blockIdx.x % ntn;
  const int b = unit / a.Hq, h = unit % a.Hq, kvh = a.map.kv[h];
  int m_valid = a.M, k_valid = a.K;
  if (a.m_total > 0) m_valid = min(a.M, a.m_total - c * a.M);
  if (a.k_total > 0) k_valid = min(a.K, a.k_total - c * a.K);
  if (m_valid <= mt * 64 || k_valid <= 0) return;   // uniform over the workgroup
  auto item_off = [&](const GemmOperand& o) {
    return b * o.s_b + (o.kv ? kvh : h) * o.s_h + (int64_t)(c / o.c_div) * o.s_c;
  };
  const int64_t a_off = item_off(a.A);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l31 = lane & 31, g = lane >> 5;
  const int wr = wave >> 1, wc = wave & 1;
  floatx16 acc[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) acc[j] = zero16();
  const int n_b = a.B2.base != nullptr ? 2 : 1;
  for (int pass = 0; pass < n_b; ++pass) {
    const GemmOperand& ob = pass == 0 ? a.B : a.B2;
    const int64_t b_off = item_off(ob);
    for (int k0 = 0; k0 < k_valid; k0 += BK) {
      load_operand<T, 64, LDK>(As, a.A, a_off, mt * 64, m_valid, k0, k_valid, tid);
      load_operand<T, BN, LDK>(Bs, ob, b_off, nt * BN, a.Nn, k0, k_valid, tid);
      __syncthreads();
#pragma unroll
      for (int s = 0; s < BK / M::KK; ++s) {
        const typename M::frag af = M::load(As + (32 * wr + l31) * LDK + s * M::KK + g * M::KPL);
#pragma unroll
        for (int j = 0; j < NT; ++j)
          acc[j] = M::mma(af, M::load(Bs + (32 * (wc * NT + j) + l31) * LDK + s * M::KK + g * M::KPL), acc[j]);
      }
      __syncthreads();
    }
  }
  float* cp = a.C + b * a.c_b + (a.c_kv ? kvh : h) * a.c_h + (int64_t)c * a.c_c;
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int n = nt * BN + 32 * (wc * NT + j) + l31;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int m = mt * 64 + 32 * wr + c_row(i, g);
      if (m < m_valid) {
        float* dst = cp + (int64_t)m * a.c_r + n;
        if (a.mode == 0) *dst = acc[j][i];
        else if (a.mode == 1) *dst += acc[j][i];
        else atomicAdd(dst, acc[j][i]);
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------------------
// Element-wise kernels (one wave per token row unless said otherwise)
// ---------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void fill_f32_kernel(float* p, int64_t n, float x) {
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = x;
}

// delta_t = dy_t . y_t, E_t = exp(-L_t), A_t = E_t (gate_t * dy_t)
template <typename T>
__global__ __launch_bounds__(256) void bwd_row_prep_kernel(BwdRowArgs a) {
  const int64_t row = blockIdx.x * 4ll + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= (int64_t)a.U * a.N) return;
  const int unit = (int)(row / a.N), t = (int)(row % a.N);
  const int b = unit / a.Hq, h = unit % a.Hq;
  const T* y = static_cast<const T*>(a.out) + b * a.o_sb + (int64_t)t * a.o_st + h * a.o_sh;
  const T* dy = static_cast<const T*>(a.dout) + b * a.o_sb + (int64_t)t * a.o_st + h * a.o_sh;
  const T* gp = a.g ? static_cast<const T*>(a.g) + b * a.g_sb + (int64_t)t * a.g_st + h * a.g_sh : nullptr;
  const float E = __expf(-a.lse[row]);
  float dot = 0.f;
  for (int x = lane; x < a.d; x += 64) {
    const float dyx = to_f32<T>(dy[x]);
    dot += dyx * to_f32<T>(y[x]);
    float gate = 1.f;
    if (gp) {
      gate = to_f32<T>(gp[x]);
      if (a.gate_act) gate = 1.f / (1.f + __expf(-gate));
    }
    static_cast<T*>(a.A)[row * a.d + x] = from_f32<T>(E * gate * dyx);
  }
  dot = wave_sum(dot);
  if (lane == 0) {
    a.e_row[row] = E;
    a.delta[row] = dot;
    a.ed[row] = E * dot;
  }
}

// NP-Map forward from f = x W (bias added here): phi (storage type; zero for tokens the softmax branch keeps),
// u over f in place, and (|x|, |f|).
template <typename T>
__global__ __launch_bounds__(256) void bwd_np_fwd_kernel(BwdNpArgs a) {
  const int64_t row = blockIdx.x * 4ll + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= (int64_t)a.U * a.N) return;
  const int unit = (int)(row / a.N), t = (int)(row % a.N);
  const int b = unit / a.Hq, h = unit % a.Hq;
  const int hx = a.x_kv ? a.map.kv[h] : h;
  const T* x = static_cast<const T*>(a.x) + b * a.x_sb + (int64_t)t * a.x_st + hx * a.x_sh;
  const int F = a.F;
  float* f = a.u + row * F;
  const T* bias = a.bias ? static_cast<const T*>(a.bias) + h * F : nullptr;
  float nx2 = 0.f;
  for (int i = lane; i < a.d; i += 64) {
    const float xv = to_f32<T>(x[i]);
    nx2 += xv * xv;
  }
  float fv[2], nf2 = 0.f;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int i = lane + 64 * j;
    fv[j] = 0.f;
    if (i < F) {
      fv[j] = f[i] + (bias ? to_f32<T>(bias[i]) : 0.f);
      nf2 += fv[j] * fv[j];
    }
  }
  nx2 = wave_sum(nx2);
  nf2 = wave_sum(nf2);
  const float nx = sqrtf(nx2), nf = sqrtf(nf2);
  const float ratio = nf2 > 0.f ? nx / nf : 0.f;
  float mp = -INFINITY, mn = -INFINITY;
#pragma unroll
  for (int j = 0; j < 2; ++j)
    if (lane + 64 * j < F) {
      fv[j] *= ratio;
      mp = fmaxf(mp, fv[j]);
      mn = fmaxf(mn, -fv[j]);
    }
  mp = wave_max(mp);
  mn = wave_max(mn);
  float ep[2], en[2], sp = 0.f, sn = 0.f;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    ep[j] = en[j] = 0.f;
    if (lane + 64 * j < F) {
      ep[j] = __expf(fv[j] - mp);
      en[j] = __expf(-fv[j] - mn);
      sp += ep[j];
      sn += en[j];
    }
  }
  sp = wave_sum(sp);
  sn = wave_sum(sn);
  bool kept = false;
  if (a.kmask != nullptr && t < a.ncf * a.C) {
    const int c = t / a.C, w = t % a.C;
    kept = (a.kmask[((int64_t)unit * a.ncf + c) * (a.C / 32) + w / 32] >> (w & 31)) & 1u;
  }
  const float ip = kept ? 0.f : 1.f / sp, in = kept ? 0.f : 1.f / sn;
  T* phi = static_cast<T*>(a.phi) + row * 2 * F;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int i = lane + 64 * j;
    if (i < F) {
      phi[i] = from_f32<T>(ep[j] * ip);
      phi[F + i] = from_f32<T>(en[j] * in);
      f[i] = fv[j];
    }
  }
  if (lane == 0) {
    a.st[2 * row] = nx;
    a.st[2 * row + 1] = nf;
  }
}

// NP-Map backward for one token: dphi (minus coef * z) -> df in the storage type, and the |x| path of dx added to the
// fp32 gradient of x (plain add where the row is owned, atomic where query heads share a kv head).
template <typename T>
__global__ __launch_bounds__(256) void bwd_np_bwd_kernel(BwdNpArgs a) {
  const int64_t row = blockIdx.x * 4ll + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= (int64_t)a.U * a.N) return;
  const int unit = (int)(row / a.N), t = (int)(row % a.N);
  const int b = unit / a.Hq, h = unit % a.Hq;
  const int hx = a.x_kv ? a.map.kv[h] : h;
  const int F = a.F, c = t / a.C;
  T* df = static_cast<T*>(a.df) + row * F;
  bool kept = false;
  if (a.kmask != nullptr && t < a.ncf * a.C) {
    const int w = t % a.C;
    kept = (a.kmask[((int64_t)unit * a.ncf + c) * (a.C / 32) + w / 32] >> (w & 31)) & 1u;
  }
  const float nx = a.st[2 * row], nf = a.st[2 * row + 1];
  if (kept || !(nx > 0.f) || !(nf > 0.f)) {   // uniform over the wave
    for (int i = lane; i < F; i += 64) df[i] = from_f32<T>(0.f);
    return;
  }
  const float* u = a.u + row * F;
  const float* dphi = a.dphi + row * 2 * F;
  const float coef = a.coef ? a.coef[row] : 1.f;
  const float* z1 = a.z1 + ((int64_t)unit * a.nc + c) * 2 * F;
  const float* z2 = a.z2 ? a.z2 + ((int64_t)unit * a.nseg + c / a.seg_chunks) * 2 * F : nullptr;
  float uv[2], mp = -INFINITY, mn = -INFINITY;
#pragma unroll
  for (int j = 0; j < 2; ++j)
    if (lane + 64 * j < F) {
      uv[j] = u[lane + 64 * j];
      mp = fmaxf(mp, uv[j]);
      mn = fmaxf(mn, -uv[j]);
    }
  mp = wave_max(mp);
  mn = wave_max(mn);
  float ep[2], en[2], dp[2], dn[2], sp = 0.f, sn = 0.f;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int i = lane + 64 * j;
    ep[j] = en[j] = dp[j] = dn[j] = 0.f;
    if (i < F) {
      ep[j] = __expf(uv[j] - mp);
      en[j] = __expf(-uv[j] - mn);
      sp += ep[j];
      sn += en[j];
      dp[j] = dphi[i] - coef * (z1[i] + (z2 ? z2[i] : 0.f));
      dn[j] = dphi[F + i] - coef * (z1[F + i] + (z2 ? z2[F + i] : 0.f));
    }
  }
  sp = wave_sum(sp);
  sn = wave_sum(sn);
  float ap = 0.f, an = 0.f;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    ep[j] /= sp;
    en[j] /= sn;
    ap += ep[j] * dp[j];
    an += en[j] * dn[j];
  }
  ap = wave_sum(ap);
  an = wave_sum(an);
  float du[2], dnx = 0.f;
  const float inx = 1.f / nx;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    du[j] = ep[j] * (dp[j] - ap) - en[j] * (dn[j] - an);
    if (lane + 64 * j < F) dnx += uv[j] * inx * du[j];
  }
  dnx = wave_sum(dnx);
  const float ratio = nx / nf;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int i = lane + 64 * j;
    if (i < F) df[i] = from_f32<T>(ratio * (du[j] - uv[j] * inx * dnx));
  }
  const T* x = static_cast<const T*>(a.x) + b * a.x_sb + (int64_t)t * a.x_st + hx * a.x_sh;
  const int64_t xrow = a.x_kv ? ((int64_t)b * a.Hkv + hx) * a.N + t : row;
  float* dx = a.dx32 + xrow * a.d;
  for (int i = lane; i < a.d; i += 64) {
    const float add = dnx * inx * to_f32<T>(x[i]);
    if (a.x_kv) atomicAdd(dx + i, add);
    else dx[i] += add;
  }
}

// out[f] (per (unit, chunk), or added atomically per head) = sum over the chunk's tokens of X[t][f] * w[t]
template <typename T>
__global__ __launch_bounds__(256) void bwd_colsum_kernel(BwdColsumArgs a) {
  const int c = blockIdx.x, unit = blockIdx.y;
  const int h = unit % a.Hq;
  const int t0 = c * a.C, t1 = min(a.N, t0 + a.C);
  const T* X = static_cast<const T*>(a.X) + ((int64_t)unit * a.N) * a.L;
  for (int f = threadIdx.x; f < a.L; f += 256) {
    float s = 0.f;
    for (int t = t0; t < t1; ++t) s += to_f32<T>(X[(int64_t)t * a.L + f]) * (a.w ? a.w[(int64_t)unit * a.N + t] : 1.f);
    if (a.per_head) atomicAdd(a.out + (int64_t)h * a.L + f, s);
    else a.out[((int64_t)unit * a.nc + c) * a.L + f] = s;
  }
}

// X[unit][c][l] <- sum over c' >= c + 2 of X[unit][c'][l]  (the rows of chunk c' see the state through chunk c'-2)
__global__ __launch_bounds__(256) void bwd_revcumsum_kernel(float* X, int nc, int64_t L) {
  const int64_t l = blockIdx.x * 256ll + threadIdx.x;
  if (l >= L) return;
  float* p = X + (int64_t)blockIdx.y * nc * L + l;
  float s1 = 0.f, s2 = 0.f;
  for (int c = nc - 1; c >= 0; --c) {
    const float v = p[(int64_t)c * L];
    p[(int64_t)c * L] = s2;
    s2 = s1;
    s1 += v;
  }
}

// dg = E_t dy_t * (phi_q S)_t  (times the logistic function's slope when the gate is activated here)
template <typename T>
__global__ __launch_bounds__(256) void bwd_dg_kernel(BwdRowArgs a) {
  const int64_t n = (int64_t)a.U * a.N * a.d;
  for (int64_t i = blockIdx.x * 256ll + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int64_t row = i / a.d;
    const int x = (int)(i % a.d);
    const int unit = (int)(row / a.N), t = (int)(row % a.N);
    const int b = unit / a.Hq, h = unit % a.Hq;
    const float dyx = to_f32<T>(static_cast<const T*>(a.dout)[b * a.o_sb + (int64_t)t * a.o_st + h * a.o_sh + x]);
    float r = a.e_row[row] * dyx * a.nraw[i];
    const int64_t go = b * a.g_sb + (int64_t)t * a.g_st + h * a.g_sh + x;
    if (a.gate_act) {
      const float s = 1.f / (1.f + __expf(-to_f32<T>(static_cast<const T*>(a.g)[go])));
      r *= s * (1.f - s);
    }
    static_cast<T*>(a.dg)[go] = from_f32<T>(r);
  }
}

// fp32 gradient rows -> the caller's strided tensors in the storage type
template <typename T>
__global__ __launch_bounds__(256) void bwd_finish_kernel(BwdFinishArgs a) {
  const int64_t n = (int64_t)a.B * a.H * a.N * a.d;
  for (int64_t i = blockIdx.x * 256ll + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int x = (int)(i % a.d);
    const int64_t row = i / a.d;
    const int t = (int)(row % a.N);
    const int bh = (int)(row / a.N);
    const int b = bh / a.H, h = bh % a.H;
    static_cast<T*>(a.dst)[b * a.s_b + (int64_t)t * a.s_t + h * a.s_h + x] = from_f32<T>(a.src[i]);
  }
}

// ---------------------------------------------------------------------------------------------------------
// Sparse (softmax) branch.  Tiles of 64 query rows x 64 keys, four waves, one 32 x 32 block of logits each.
// A key tile is either 64 consecutive entries of the head's retained list (routing order) or 64 consecutive tokens of
// the local span.  Row t of chunk c sees retained entry e when e < n_vis(c) = min((c-1) lambda, budget), and local
// token j when (c-1) C <= j <= t.
// Every matrix operand is read from global memory directly in fragment form (a lane's 8 consecutive contraction
// entries are 16 contiguous bytes): rows of q, k, v, dout for the products that contract over the head dimension,
// and transposed copies (q^T, dout^T, k^T of the local span, k^T of the retained rows, all [d][tokens], zero padded)
// for those that contract over rows or keys.  LDS only carries P and dS from the accumulator layout of one product
// to the operand layout of the next.
// ---------------------------------------------------------------------------------------------------------
template <typename T>
struct BwdTile {
  static constexpr int PAD = sizeof(T) == 2 ? 8 : 4;
  static constexpr int LT = 64 + PAD;       // row stride of a [64][64] tile
};

// acc += sum over 64 contraction entries of X[m][k] Y[n][k]: X an LDS tile [..][LT] (rows xr0 + m), Y rows in global
// memory (row n of the block at yrow, contraction entries contiguous)
template <typename T>
__device__ __forceinline__ void acc64_lds_global(floatx16& acc, const T* X, int xr0, const T* yrow, int l31, int g) {
  typedef Mma<T> M;
#pragma unroll
  for (int s = 0; s < 64 / M::KK; ++s)
    acc = M::mma(M::load(X + (xr0 + l31) * BwdTile<T>::LT + s * M::KK + g * M::KPL),
                 M::load(yrow + s * M::KK + g * M::KPL), acc);
}

template <typename T, int D>
__global__ __launch_bounds__(256) void bwd_sa_dq_kernel(BwdSaArgs a) {
  typedef Mma<T> M;
  constexpr int LT = BwdTile<T>::LT, KS = D / M::KK, DX = D / 64;
  __shared__ __attribute__((aligned(16))) T dSs[64 * LT];
  __shared__ float Ls[64], dls[64];
  __shared__ int toks[64];

  const int unit = blockIdx.y, rt = a.n_row_tiles - 1 - blockIdx.x;   // long rows first
  const int b = unit / a.Hq, h = unit % a.Hq, kvh = a.map.kv[h];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l31 = lane & 31, g = lane >> 5, wr = wave >> 1, wc = wave & 1;
  const int N = a.N, C = a.C, r0 = rt * 64;
  const int c = r0 / C;
  const int n_vis = retained_rows(c >= 1 ? c - 1 : 0, a.lam, a.rcap);
  const int lo = (c >= 1 ? c - 1 : 0) * C;
  const int last = min(N - 1, r0 + 63);
  const int n_ret_tiles = (n_vis + 63) / 64, n_tiles = n_ret_tiles + (last + 1 - lo + 63) / 64;

  const T* kb = static_cast<const T*>(a.k) + b * a.k_sb + kvh * a.k_sh;
  const T* vb = static_cast<const T*>(a.v) + b * a.v_sb + kvh * a.v_sh;
  const T* kret = static_cast<const T*>(a.kret) + (int64_t)unit * a.cap * D;
  const T* krett = static_cast<const T*>(a.krett) + (int64_t)unit * D * a.cap;
  const T* kt = static_cast<const T*>(a.kt) + ((int64_t)b * a.Hkv + kvh) * D * a.Np;
  const int32_t* sel = a.sel + (int64_t)unit * a.sel_stride;
  if (tid < 64) {
    const int t = r0 + tid;
    Ls[tid] = t < N ? a.lse[(int64_t)unit * N + t] * kLog2e : 0.f;
    dls[tid] = t < N ? a.delta[(int64_t)unit * N + t] : 0.f;
  }
  // this wave's 32 query rows as A operands, for the whole kernel
  typename M::frag qf[KS], dof[KS];
  {
    const int t = min(r0 + 32 * wr + l31, N - 1);
    const T* qp = static_cast<const T*>(a.q) + b * a.q_sb + (int64_t)t * a.q_st + h * a.q_sh + g * M::KPL;
    const T* dp = static_cast<const T*>(a.dout) + b * a.o_sb + (int64_t)t * a.o_st + h * a.o_sh + g * M::KPL;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      qf[s] = M::load(qp + s * M::KK);
      dof[s] = M::load(dp + s * M::KK);
    }
  }
  floatx16 dq[DX];
#pragma unroll
  for (int j = 0; j < DX; ++j) dq[j] = zero16();
  const float sc2 = a.scale * kLog2e;
  const int kcol = 32 * wc + l31;

  for (int ti = 0; ti < n_tiles; ++ti) {
    const bool ret = ti < n_ret_tiles;
    const int k0 = ret ? ti * 64 : lo + (ti - n_ret_tiles) * 64;
    __syncthreads();   // the previous tile's products have read dSs and toks (first trip: Ls, dls are written)
    if (tid < 64) {
      int tok;
      if (ret) {
        const int e = k0 + tid;
        tok = e < n_vis ? sel[e] : -1;
        if (tok < 0 || tok >= N || tok / C != e / a.lam) tok = -1;   // lists are never trusted for addressing
      } else {
        tok = k0 + tid < N ? k0 + tid : -1;
      }
      toks[tid] = tok;
    }
    __syncthreads();
    const int tok = toks[kcol];
    const int tokc = tok < 0 ? 0 : tok;
    const T* krow = (ret ? kret + (int64_t)(k0 + kcol) * D : kb + (int64_t)tokc * a.k_st) + g * M::KPL;
    const T* vrow = vb + (int64_t)tokc * a.v_st + g * M::KPL;
    floatx16 s = zero16(), dp = zero16();
#pragma unroll
    for (int st = 0; st < KS; ++st) {
      s = M::mma(qf[st], M::load(krow + st * M::KK), s);
      dp = M::mma(dof[st], M::load(vrow + st * M::KK), dp);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int r = 32 * wr + c_row(i, g);
      const int t = r0 + r;
      const bool vis = tok >= 0 && t < N && (ret || (tok >= lo && tok <= t));
      const float p = vis ? fast_exp2(fmaf(s[i], sc2, -Ls[r])) : 0.f;
      dSs[r * LT + kcol] = from_f32<T>(p * (dp[i] - dls[r]) * a.scale);
    }
    __syncthreads();
    const T* ktile = ret ? krett + k0 : kt + k0;
    const int64_t kstride = ret ? a.cap : a.Np;
#pragma unroll
    for (int j = 0; j < DX; ++j)
      acc64_lds_global<T>(dq[j], dSs, 32 * wr, ktile + (int64_t)(32 * (wc * DX + j) + l31) * kstride, l31, g);
  }
  float* out = a.dq32 + ((int64_t)unit * N) * D;
#pragma unroll
  for (int j = 0; j < DX; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int t = r0 + 32 * wr + c_row(i, g);
      if (t < N) out[(int64_t)t * D + 32 * (wc * DX + j) + l31] = dq[j][i];
    }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void bwd_sa_dkv_kernel(BwdSaArgs a) {
  typedef Mma<T> M;
  constexpr int LT = BwdTile<T>::LT, KS = D / M::KK, DX = D / 64;
  __shared__ __attribute__((aligned(16))) T PTs[64 * LT];     // [key][row]
  __shared__ __attribute__((aligned(16))) T dSTs[64 * LT];
  __shared__ float Ls[64], dls[64];
  __shared__ int toks[64];

  const int unit = blockIdx.y, ti = blockIdx.x;   // retained tiles (the long ones) come first
  const int b = unit / a.Hq, h = unit % a.Hq, kvh = a.map.kv[h];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l31 = lane & 31, g = lane >> 5, wr = wave >> 1, wc = wave & 1;
  const int N = a.N, C = a.C;
  const bool ret = ti < a.n_ret_tiles;
  const int k0 = ret ? ti * 64 : (ti - a.n_ret_tiles) * 64;
  int row_lo, row_hi;   // rows that may see a key of this tile: [row_lo, row_hi)
  if (ret) {
    if (a.lam <= 0 || k0 >= retained_rows(a.nc >= 2 ? a.nc - 2 : 0, a.lam, a.rcap)) return;
    row_lo = (k0 / a.lam + 2) * C;
    row_hi = N;
  } else {
    row_lo = k0;
    row_hi = min(N, (k0 / C + 2) * C);
  }
  if (row_lo >= row_hi) return;
  const T* qb = static_cast<const T*>(a.q) + b * a.q_sb + h * a.q_sh;
  const T* dob = static_cast<const T*>(a.dout) + b * a.o_sb + h * a.o_sh;
  const T* kb = static_cast<const T*>(a.k) + b * a.k_sb + kvh * a.k_sh;
  const T* vb = static_cast<const T*>(a.v) + b * a.v_sb + kvh * a.v_sh;
  const T* qt = static_cast<const T*>(a.qt) + (int64_t)unit * D * a.Np;
  const T* dot = static_cast<const T*>(a.dot) + (int64_t)unit * D * a.Np;
  const int32_t* sel = a.sel + (int64_t)unit * a.sel_stride;
  if (tid < 64) {
    int tok;
    if (ret) {
      const int e = k0 + tid;
      tok = e < a.sel_stride ? sel[e] : -1;
      if (tok < 0 || tok >= N || tok / C != e / a.lam) tok = -1;
    } else {
      tok = k0 + tid < N ? k0 + tid : -1;
    }
    toks[tid] = tok;
  }
  __syncthreads();
  const int kcol = 32 * wc + l31;
  const int tok = toks[kcol];
  // this wave's 32 keys as B operands of the logits and of dy.v, for the whole kernel
  typename M::frag kf[KS], vf[KS];
  {
    const int tokc = tok < 0 ? 0 : tok;
    const T* kp = kb + (int64_t)tokc * a.k_st + g * M::KPL;
    const T* vp = vb + (int64_t)tokc * a.v_st + g * M::KPL;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      kf[s] = M::load(kp + s * M::KK);
      vf[s] = M::load(vp + s * M::KK);
    }
  }
  floatx16 dk[DX], dv[DX];
#pragma unroll
  for (int j = 0; j < DX; ++j) dk[j] = dv[j] = zero16();
  const float sc2 = a.scale * kLog2e;
  const int e = k0 + kcol;

  for (int r0 = row_lo / 64 * 64; r0 < row_hi; r0 += 64) {
    __syncthreads();   // the previous trip's products have read PTs, dSTs, Ls, dls
    if (tid < 64) {
      const int t = r0 + tid;
      Ls[tid] = t < N ? a.lse[(int64_t)unit * N + t] * kLog2e : 0.f;
      dls[tid] = t < N ? a.delta[(int64_t)unit * N + t] : 0.f;
    }
    floatx16 s = zero16(), dp = zero16();
    {
      const int t = min(r0 + 32 * wr + l31, N - 1);
      const T* qp = qb + (int64_t)t * a.q_st + g * M::KPL;
      const T* dp_ = dob + (int64_t)t * a.o_st + g * M::KPL;
#pragma unroll
      for (int st = 0; st < KS; ++st) {
        s = M::mma(M::load(qp + st * M::KK), kf[st], s);
        dp = M::mma(M::load(dp_ + st * M::KK), vf[st], dp);
      }
    }
    __syncthreads();   // Ls, dls visible
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {
      const int rbase = 32 * wr + c_row(4 * i4, g);   // four consecutive rows
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int i = 4 * i4 + j;
        const int r = rbase + j;
        const int t = r0 + r;
        const int c = t / C;
        bool vis = tok >= 0 && t < N;
        if (ret) vis = vis && e < retained_rows(c >= 1 ? c - 1 : 0, a.lam, a.rcap);
        else vis = vis && tok <= t && tok >= (c >= 1 ? c - 1 : 0) * C;
        const float p = vis ? fast_exp2(fmaf(s[i], sc2, -Ls[r])) : 0.f;
        PTs[kcol * LT + r] = from_f32<T>(p);
        dSTs[kcol * LT + r] = from_f32<T>(p * (dp[i] - dls[r]) * a.scale);
      }
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < DX; ++j) {
      const int64_t xrow = (int64_t)(32 * (wc * DX + j) + l31) * a.Np + r0;
      acc64_lds_global<T>(dv[j], PTs, 32 * wr, dot + xrow, l31, g);    // dV[key][x] += P^T dO
      acc64_lds_global<T>(dk[j], dSTs, 32 * wr, qt + xrow, l31, g);    // dK[key][x] += dS^T Q
    }
  }
  float* dkb = a.dk32 + ((int64_t)b * a.Hkv + kvh) * N * D;
  float* dvb = a.dv32 + ((int64_t)b * a.Hkv + kvh) * N * D;
#pragma unroll
  for (int j = 0; j < DX; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int tk = toks[32 * wr + c_row(i, g)];
      if (tk >= 0) {
        const int x = 32 * (wc * DX + j) + l31;
        atomicAdd(dkb + (int64_t)tk * D + x, dk[j][i]);
        atomicAdd(dvb + (int64_t)tk * D + x, dv[j][i]);
      }
    }
}

template <typename T, int D>
hipError_t launch_sa_t(const BwdSaArgs& a, int U, hipStream_t s) {
  hipLaunchKernelGGL((bwd_sa_dq_kernel<T, D>), dim3(a.n_row_tiles, U), dim3(256), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((bwd_sa_dkv_kernel<T, D>), dim3(a.n_ret_tiles + a.n_row_tiles, U), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_bgemm(const GemmArgs& a, int dtype, int U, int n_c, hipStream_t s) {
  const int bn = a.Nn % 128 == 0 ? 128 : 64;
  const dim3 grid((a.Nn / bn) * ((a.M + 63) / 64), n_c, U);
  if (dtype == 1) {
    if (bn == 128) hipLaunchKernelGGL((bgemm_kernel<bf16, 128>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((bgemm_kernel<bf16, 64>), grid, dim3(256), 0, s, a);
  } else {
    if (bn == 128) hipLaunchKernelGGL((bgemm_kernel<float, 128>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((bgemm_kernel<float, 64>), grid, dim3(256), 0, s, a);
  }
  return hipGetLastError();
}

hipError_t launch_fill_f32(float* p, int64_t n, float x, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  const int blocks = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
  hipLaunchKernelGGL(fill_f32_kernel, dim3(blocks), dim3(256), 0, s, p, n, x);
  return hipGetLastError();
}

hipError_t launch_bwd_row_prep(const BwdRowArgs& a, int dtype, hipStream_t s) {
  const int blocks = (int)(((int64_t)a.U * a.N + 3) / 4);
  if (dtype == 1) hipLaunchKernelGGL((bwd_row_prep_kernel<bf16>), dim3(blocks), dim3(256), 0, s, a);
  else hipLaunchKernelGGL((bwd_row_prep_kernel<float>), dim3(blocks), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_bwd_dg(const BwdRowArgs& a, int dtype, hipStream_t s) {
  const int64_t n = (int64_t)a.U * a.N * a.d;
  const int blocks = (int)((n + 255) / 256 < 8192 ? (n + 255) / 256 : 8192);
  if (dtype == 1) hipLaunchKernelGGL((bwd_dg_kernel<bf16>), dim3(blocks), dim3(256), 0, s, a);
  else hipLaunchKernelGGL((bwd_dg_kernel<float>), dim3(blocks), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_bwd_np(const BwdNpArgs& a, int dtype, bool backward, hipStream_t s) {
  const int blocks = (int)(((int64_t)a.U * a.N + 3) / 4);
  if (dtype == 1) {
    if (backward) hipLaunchKernelGGL((bwd_np_bwd_kernel<bf16>), dim3(blocks), dim3(256), 0, s, a);
    else hipLaunchKernelGGL((bwd_np_fwd_kernel<bf16>), dim3(blocks), dim3(256), 0, s, a);
  } else {
    if (backward) hipLaunchKernelGGL((bwd_np_bwd_kernel<float>), dim3(blocks), dim3(256), 0, s, a);
    else hipLaunchKernelGGL((bwd_np_fwd_kernel<float>), dim3(blocks), dim3(256), 0, s, a);
  }
  return hipGetLastError();
}

hipError_t launch_bwd_colsum(const BwdColsumArgs& a, int dtype, int U, hipStream_t s) {
  const dim3 grid(a.nc, U);
  if (dtype == 1) hipLaunchKernelGGL((bwd_colsum_kernel<bf16>), grid, dim3(256), 0, s, a);
  else hipLaunchKernelGGL((bwd_colsum_kernel<float>), grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_bwd_revcumsum(float* X, int U, int nc, int64_t L, hipStream_t s) {
  hipLaunchKernelGGL(bwd_revcumsum_kernel, dim3((unsigned)((L + 255) / 256), U), dim3(256), 0, s, X, nc, L);
  return hipGetLastError();
}

hipError_t launch_bwd_finish(const BwdFinishArgs& a, int dtype, hipStream_t s) {
  const int64_t n = (int64_t)a.B * a.H * a.N * a.d;
  const int blocks = (int)((n + 255) / 256 < 8192 ? (n + 255) / 256 : 8192);
  if (dtype == 1) hipLaunchKernelGGL((bwd_finish_kernel<bf16>), dim3(blocks), dim3(256), 0, s, a);
  else hipLaunchKernelGGL((bwd_finish_kernel<float>), dim3(blocks), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_bwd_sa(const BwdSaArgs& a, int dtype, int d, int U, hipStream_t s) {
  if (dtype == 1) return d == 128 ? launch_sa_t<bf16, 128>(a, U, s) : launch_sa_t<bf16, 64>(a, U, s);
  if (d == 64) return launch_sa_t<float, 64>(a, U, s);
  return hipErrorInvalidValue;   // fp32 at d = 128 does not fit the tiles in LDS (refused by the host checks)
}

}  // namespace still

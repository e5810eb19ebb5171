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
// This first version keeps every step a separate, simple kernel: the sparse branch as tile kernels (one that owns
// query rows and produces dq, one that owns key tiles and produces dk, dv), the linear branch as a sequence of
// batched products on one generic MFMA tile kernel with row-wise kernels between them, intermediates in the
// workspace.  All sums are fp32; operands of the matrix core are in the storage type.
#include "still_kernels.h"

namespace still {

namespace {

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

// The state gradient as a running sum: dS(c) = sum over c' >= c + 2 of A(c')^T-products.  One workgroup owns a 64 x BN
// tile of the state for one (batch, head) and walks the chunks from the last one down, keeping the sum in its
// accumulators: after adding the contribution of chunk c' the accumulators ARE dS(c' - 2), which is stored in the
// storage type (it is only ever a matrix-core operand again).  The two last chunks' dS is zero.  Operands as in
// bgemm_kernel (item index = chunk, contraction over the chunk's tokens, cut short in a ragged last chunk).
template <typename T, int BN>
__global__ __launch_bounds__(256) void bgemm_revscan_kernel(GemmArgs a, int n_c) {
  typedef Mma<T> M;
  constexpr int BK = 64, NT = BN / 64;
  constexpr int LDK = BK + (sizeof(T) == 2 ? 8 : 4);
  __shared__ __attribute__((aligned(16))) T As[64 * LDK];
  __shared__ __attribute__((aligned(16))) T Bs[BN * LDK];
  const int unit = blockIdx.z;
  const int ntn = a.Nn / BN;
  const int mt = blockIdx.x / ntn, nt = blockIdx.x % ntn;
  const int b = unit / a.Hq, h = unit % a.Hq, kvh = a.map.kv[h];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l31 = lane & 31, g = lane >> 5;
  const int wr = wave >> 1, wc = wave & 1;
  floatx16 acc[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) acc[j] = zero16();
  T* cbase = reinterpret_cast<T*>(a.C) + b * a.c_b + (a.c_kv ? kvh : h) * a.c_h;
  auto store = [&](int c) {
    T* cp = cbase + (int64_t)c * a.c_c;
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int n = nt * BN + 32 * (wc * NT + j) + l31;
#pragma unroll
      for (int i = 0; i < 16; ++i) cp[(int64_t)(mt * 64 + 32 * wr + c_row(i, g)) * a.c_r + n] = from_f32<T>(acc[j][i]);
    }
  };
  if (n_c >= 1) store(n_c - 1);
  if (n_c >= 2) store(n_c - 2);
  for (int c = n_c - 1; c >= 2; --c) {
    int k_valid = a.K;
    if (a.k_total > 0) k_valid = min(a.K, a.k_total - c * a.K);
    const int64_t a_off = b * a.A.s_b + (a.A.kv ? kvh : h) * a.A.s_h + (int64_t)c * a.A.s_c;
    const int64_t b_off = b * a.B.s_b + (a.B.kv ? kvh : h) * a.B.s_h + (int64_t)c * a.B.s_c;
    for (int k0 = 0; k0 < k_valid; k0 += BK) {
      load_operand<T, 64, LDK>(As, a.A, a_off, mt * 64, a.M, k0, k_valid, tid);
      load_operand<T, BN, LDK>(Bs, a.B, b_off, nt * BN, a.Nn, k0, k_valid, tid);
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
    store(c - 2);
  }
}

// ---------------------------------------------------------------------------------------------------------
// Element-wise kernels
// ---------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void fill_f32_kernel(float* p, int64_t n, float x) {
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = x;
}

// The row-wise kernels below give every token row to d/8 lanes (d = d_f here), 8 contiguous elements per lane, so
// that every access is a 16-byte (storage type) or 32-byte (fp32) vector and a row reduction is 3 or 4 exchanges
// inside the group.  A wave holds 64 / (d/8) rows, a workgroup four waves.
template <typename T>
__device__ __forceinline__ void load8_t(float (&x)[8], const T* p) {
  load8<T>(x, p, 0, 0);
}
template <typename T>
__device__ __forceinline__ void store8_t(T* p, const float (&x)[8]) {
  if constexpr (sizeof(T) == 2) {
    bf16x8 v;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = static_cast<bf16>(x[e]);
    *reinterpret_cast<bf16x8*>(p) = v;
  } else {
    floatx4 a, b;
#pragma unroll
    for (int e = 0; e < 4; ++e) { a[e] = x[e]; b[e] = x[4 + e]; }
    *reinterpret_cast<floatx4*>(p) = a;
    *reinterpret_cast<floatx4*>(p + 4) = b;
  }
}
__device__ __forceinline__ void load8_f32(float (&x)[8], const float* p) { load8<float>(x, p, 0, 1); }
__device__ __forceinline__ void store8_f32(float* p, const float (&x)[8]) { store8_t<float>(p, x); }
__device__ __forceinline__ float group_sum(float x, int lpr) {
  for (int o = lpr >> 1; o >= 1; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}
__device__ __forceinline__ float group_max(float x, int lpr) {
  for (int o = lpr >> 1; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  return x;
}
// row handled by this lane, and its first element; false when the row is past the end (whole groups drop out)
__device__ __forceinline__ bool row_of_lane(int64_t n_rows, int width, int64_t& row, int& e0, int& lpr) {
  lpr = width / 8;
  const int tid = threadIdx.x;
  row = (int64_t)blockIdx.x * (256 / lpr) + tid / lpr;
  e0 = (tid % lpr) * 8;
  return row < n_rows;
}

// delta_t = dy_t . y_t, E_t = exp(-L_t), A_t = E_t (gate_t * dy_t)
template <typename T>
__global__ __launch_bounds__(256) void bwd_row_prep_kernel(BwdRowArgs a) {
  int64_t row;
  int e0, lpr;
  const bool live = row_of_lane((int64_t)a.U * a.N, a.d, row, e0, lpr);
  const int64_t rowc = live ? row : 0;
  const int unit = (int)(rowc / a.N), t = (int)(rowc % a.N);
  const int b = unit / a.Hq, h = unit % a.Hq;
  const int64_t oo = b * a.o_sb + (int64_t)t * a.o_st + h * a.o_sh + e0;
  float y[8], dy[8], gate[8];
  load8_t<T>(y, static_cast<const T*>(a.out) + oo);
  load8_t<T>(dy, static_cast<const T*>(a.dout) + oo);
#pragma unroll
  for (int e = 0; e < 8; ++e) gate[e] = 1.f;
  if (a.g) {
    load8_t<T>(gate, static_cast<const T*>(a.g) + b * a.g_sb + (int64_t)t * a.g_st + h * a.g_sh + e0);
    if (a.gate_act) {
#pragma unroll
      for (int e = 0; e < 8; ++e) gate[e] = 1.f / (1.f + __expf(-gate[e]));
    }
  }
  const float E = __expf(-a.lse[rowc]);
  float dot = 0.f, av[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    dot += dy[e] * y[e];
    av[e] = E * gate[e] * dy[e];
  }
  dot = group_sum(dot, lpr);
  if (!live) return;
  store8_t<T>(static_cast<T*>(a.A) + row * a.d + e0, av);
  if (e0 == 0) {
    a.e_row[row] = E;
    a.delta[row] = dot;
    a.ed[row] = E * dot;
  }
}

__device__ __forceinline__ bool token_kept(const BwdNpArgs& a, int unit, int t) {
  if (a.kmask == nullptr || t >= a.ncf * a.C) return false;
  const int c = t / a.C, w = t % a.C;
  return (a.kmask[((int64_t)unit * a.ncf + c) * (a.C / 32) + w / 32] >> (w & 31)) & 1u;
}

// NP-Map forward from f = x W (bias added here): phi (storage type; zero for tokens the softmax branch keeps),
// u over f in place, and (|x|, |f|).
template <typename T>
__global__ __launch_bounds__(256) void bwd_np_fwd_kernel(BwdNpArgs a) {
  int64_t row;
  int e0, lpr;
  const bool live = row_of_lane((int64_t)a.U * a.N, a.F, row, e0, lpr);
  const int64_t rowc = live ? row : 0;
  const int unit = (int)(rowc / a.N), t = (int)(rowc % a.N);
  const int b = unit / a.Hq, h = unit % a.Hq;
  const int hx = a.x_kv ? a.map.kv[h] : h;
  const int F = a.F;
  float xv[8], fv[8];
  load8_t<T>(xv, static_cast<const T*>(a.x) + b * a.x_sb + (int64_t)t * a.x_st + hx * a.x_sh + e0);
  load8_f32(fv, a.u + rowc * F + e0);
  if (a.bias) {
    float bv[8];
    load8_t<T>(bv, static_cast<const T*>(a.bias) + h * F + e0);
#pragma unroll
    for (int e = 0; e < 8; ++e) fv[e] += bv[e];
  }
  float nx2 = 0.f, nf2 = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    nx2 += xv[e] * xv[e];
    nf2 += fv[e] * fv[e];
  }
  nx2 = group_sum(nx2, lpr);
  nf2 = group_sum(nf2, lpr);
  const float nx = sqrtf(nx2), nf = sqrtf(nf2);
  const float ratio = nf2 > 0.f ? nx / nf : 0.f;
  float mp = -INFINITY, mn = -INFINITY;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    fv[e] *= ratio;
    mp = fmaxf(mp, fv[e]);
    mn = fmaxf(mn, -fv[e]);
  }
  mp = group_max(mp, lpr);
  mn = group_max(mn, lpr);
  float ep[8], en[8], sp = 0.f, sn = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    ep[e] = __expf(fv[e] - mp);
    en[e] = __expf(-fv[e] - mn);
    sp += ep[e];
    sn += en[e];
  }
  sp = group_sum(sp, lpr);
  sn = group_sum(sn, lpr);
  if (!live) return;
  const bool kept = token_kept(a, unit, t);
  const float ip = kept ? 0.f : 1.f / sp, in = kept ? 0.f : 1.f / sn;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    ep[e] *= ip;
    en[e] *= in;
  }
  T* phi = static_cast<T*>(a.phi) + row * 2 * F;
  store8_t<T>(phi + e0, ep);
  store8_t<T>(phi + F + e0, en);
  store8_f32(a.u + row * F + e0, fv);
  if (e0 == 0) {
    a.st[2 * row] = nx;
    a.st[2 * row + 1] = nf;
  }
}

// NP-Map backward for one token: dphi (minus coef * z) -> df in the storage type, and the coefficient of the |x| path
// of dx (dx = df W^T + <fh, du> x / |x|).
template <typename T>
__global__ __launch_bounds__(256) void bwd_np_bwd_kernel(BwdNpArgs a) {
  int64_t row;
  int e0, lpr;
  const bool live = row_of_lane((int64_t)a.U * a.N, a.F, row, e0, lpr);
  const int64_t rowc = live ? row : 0;
  const int unit = (int)(rowc / a.N), t = (int)(rowc % a.N);
  const int F = a.F, c = t / a.C;
  const float nx = a.st[2 * rowc], nf = a.st[2 * rowc + 1];
  const bool dead = token_kept(a, unit, t) || !(nx > 0.f) || !(nf > 0.f);   // uniform over the row's lanes
  const float coef = a.coef ? a.coef[rowc] : 1.f;
  float uv[8], dp[8], dn[8], zz[8];
  load8_f32(uv, a.u + rowc * F + e0);
  load8_f32(dp, a.dphi + rowc * 2 * F + e0);
  load8_f32(dn, a.dphi + rowc * 2 * F + F + e0);
  if (a.z1) {
    const float* z1 = a.z1 + ((int64_t)unit * a.nc + c) * 2 * F + e0;
    load8_f32(zz, z1);
#pragma unroll
    for (int e = 0; e < 8; ++e) dp[e] -= coef * zz[e];
    load8_f32(zz, z1 + F);
#pragma unroll
    for (int e = 0; e < 8; ++e) dn[e] -= coef * zz[e];
  }
  if (a.z2) {
    const float* z2 = a.z2 + ((int64_t)unit * a.nseg + c / a.seg_chunks) * 2 * F + e0;
    load8_f32(zz, z2);
#pragma unroll
    for (int e = 0; e < 8; ++e) dp[e] -= coef * zz[e];
    load8_f32(zz, z2 + F);
#pragma unroll
    for (int e = 0; e < 8; ++e) dn[e] -= coef * zz[e];
  }
  float mp = -INFINITY, mn = -INFINITY;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    mp = fmaxf(mp, uv[e]);
    mn = fmaxf(mn, -uv[e]);
  }
  mp = group_max(mp, lpr);
  mn = group_max(mn, lpr);
  float ep[8], en[8], sp = 0.f, sn = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    ep[e] = __expf(uv[e] - mp);
    en[e] = __expf(-uv[e] - mn);
    sp += ep[e];
    sn += en[e];
  }
  sp = 1.f / group_sum(sp, lpr);
  sn = 1.f / group_sum(sn, lpr);
  float ap = 0.f, an = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    ep[e] *= sp;
    en[e] *= sn;
    ap += ep[e] * dp[e];
    an += en[e] * dn[e];
  }
  ap = group_sum(ap, lpr);
  an = group_sum(an, lpr);
  const float inx = nx > 0.f ? 1.f / nx : 0.f;
  float du[8], dnx = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    du[e] = ep[e] * (dp[e] - ap) - en[e] * (dn[e] - an);
    dnx += uv[e] * inx * du[e];
  }
  dnx = group_sum(dnx, lpr);
  if (!live) return;
  const float ratio = dead ? 0.f : nx / nf;
  float dfv[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) dfv[e] = dead ? 0.f : ratio * (du[e] - uv[e] * inx * dnx);
  store8_t<T>(static_cast<T*>(a.df) + row * F + e0, dfv);
  // the |x| path of dx is a multiple of x itself: the finishing kernel adds coefficient * x (for keys, the sum of the
  // coefficients of the query heads that share the kv head)
  if (e0 == 0) a.cx[row] = dead ? 0.f : dnx * inx;
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
  int64_t row;
  int e0, lpr;
  if (!row_of_lane((int64_t)a.U * a.N, a.d, row, e0, lpr)) return;
  const int unit = (int)(row / a.N), t = (int)(row % a.N);
  const int b = unit / a.Hq, h = unit % a.Hq;
  float dy[8], nr[8], r[8];
  load8_t<T>(dy, static_cast<const T*>(a.dout) + b * a.o_sb + (int64_t)t * a.o_st + h * a.o_sh + e0);
  load8_f32(nr, a.nraw + row * a.d + e0);
  const float E = a.e_row[row];
  const int64_t go = b * a.g_sb + (int64_t)t * a.g_st + h * a.g_sh + e0;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = E * dy[e] * nr[e];
  if (a.gate_act) {
    float gv[8];
    load8_t<T>(gv, static_cast<const T*>(a.g) + go);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float sg = 1.f / (1.f + __expf(-gv[e]));
      r[e] *= sg * (1.f - sg);
    }
  }
  store8_t<T>(static_cast<T*>(a.dg) + go, r);
}

// fp32 gradient rows (+ coefficient * x for the |x| path of the NP-Map, summed over the query heads that read the
// row's head) -> the caller's strided tensors in the storage type
template <typename T>
__global__ __launch_bounds__(256) void bwd_finish_kernel(BwdFinishArgs a) {
  int64_t row;
  int e0, lpr;
  if (!row_of_lane((int64_t)a.B * a.H * a.N, a.d, row, e0, lpr)) return;
  const int t = (int)(row % a.N);
  const int bh = (int)(row / a.N);
  const int b = bh / a.H, h = bh % a.H;
  float x[8];
  load8_f32(x, a.src + row * a.d + e0);
  if (a.cx != nullptr) {
    float coef = 0.f;
    if (a.per_kv) {
      for (int hq = 0; hq < a.Hq; ++hq)
        if (a.map.kv[hq] == h) coef += a.cx[((int64_t)b * a.Hq + hq) * a.N + t];
    } else {
      coef = a.cx[row];
    }
    float xv[8];
    load8_t<T>(xv, static_cast<const T*>(a.x) + b * a.s_b + (int64_t)t * a.s_t + h * a.s_h + e0);
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] += coef * xv[e];
  }
  store8_t<T>(static_cast<T*>(a.dst) + b * a.s_b + (int64_t)t * a.s_t + h * a.s_h + e0, x);
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

// LOCAL: one workgroup per (batch, kv head, tile of 64 tokens); it walks the query heads that read this kv head one
// after the other, so the sums over the group stay in its accumulators and every row of the fp32 gradients is written
// once, with plain stores (no zero fill is needed before, and the atomic adds of every other step come after).
// !LOCAL: one workgroup per (batch, query head, tile of 64 retained entries), added atomically at the entries' tokens.
template <typename T, int D, bool LOCAL>
__global__ __launch_bounds__(256) void bwd_sa_dkv_kernel(BwdSaArgs a) {
  typedef Mma<T> M;
  constexpr int LT = BwdTile<T>::LT, KS = D / M::KK, DX = D / 64;
  __shared__ __attribute__((aligned(16))) T PTs[64 * LT];     // [key][row]
  __shared__ __attribute__((aligned(16))) T dSTs[64 * LT];
  __shared__ float Ls[64], dls[64];
  __shared__ int toks[64];

  const int ti = blockIdx.x;
  int b, kvh, h_lo, h_hi;
  if (LOCAL) {
    b = blockIdx.y / a.Hkv;
    kvh = blockIdx.y % a.Hkv;
    h_lo = 0;
    h_hi = a.Hq - 1;
  } else {
    b = blockIdx.y / a.Hq;
    h_lo = h_hi = blockIdx.y % a.Hq;
    kvh = a.map.kv[h_lo];
  }
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l31 = lane & 31, g = lane >> 5, wr = wave >> 1, wc = wave & 1;
  const int N = a.N, C = a.C;
  const int k0 = ti * 64;
  int row_lo, row_hi;   // rows that may see a key of this tile: [row_lo, row_hi)
  if (!LOCAL) {
    if (a.lam <= 0 || k0 >= retained_rows(a.nc >= 2 ? a.nc - 2 : 0, a.lam, a.rcap)) return;
    row_lo = (k0 / a.lam + 2) * C;
    row_hi = N;
  } else {
    row_lo = k0;
    row_hi = min(N, (k0 / C + 2) * C);
  }
  if (row_lo >= row_hi) return;
  const T* kb = static_cast<const T*>(a.k) + b * a.k_sb + kvh * a.k_sh;
  const T* vb = static_cast<const T*>(a.v) + b * a.v_sb + kvh * a.v_sh;
  if (tid < 64) {
    int tok;
    if (!LOCAL) {
      const int e = k0 + tid;
      tok = e < a.sel_stride ? a.sel[((int64_t)b * a.Hq + h_lo) * a.sel_stride + e] : -1;
      if (tok < 0 || tok >= N || tok / C != e / a.lam) tok = -1;   // lists are never trusted for addressing
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

  for (int h = h_lo; h <= h_hi; ++h) {
    if (LOCAL && a.map.kv[h] != kvh) continue;   // uniform
    const int unit = b * a.Hq + h;
    const T* qb = static_cast<const T*>(a.q) + b * a.q_sb + h * a.q_sh;
    const T* dob = static_cast<const T*>(a.dout) + b * a.o_sb + h * a.o_sh;
    const T* qt = static_cast<const T*>(a.qt) + (int64_t)unit * D * a.Np;
    const T* dot = static_cast<const T*>(a.dot) + (int64_t)unit * D * a.Np;
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
          if (!LOCAL) vis = vis && e < retained_rows(c >= 1 ? c - 1 : 0, a.lam, a.rcap);
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
        if (LOCAL) {
          dkb[(int64_t)tk * D + x] = dk[j][i];
          dvb[(int64_t)tk * D + x] = dv[j][i];
        } else {
          atomicAdd(dkb + (int64_t)tk * D + x, dk[j][i]);
          atomicAdd(dvb + (int64_t)tk * D + x, dv[j][i]);
        }
      }
    }
}

// ---------------------------------------------------------------------------------------------------------
// Attention map of the operator: A[t][j] = weight of v_j in row t under the shared normaliser (what the first
// training stage of Sec. 4.1 compares with the teacher's softmax map).  One workgroup per (64 rows, 64 keys) at or
// below the diagonal: the logits q.k and the linear weights phi_q.phi_k of the tile on the matrix core (operands in
// fragment form straight from global memory), then per element the branch that owns the pair: the exponential for
// the local span and for selected tokens of chunks <= c-2, E_t phi_q.phi_k for the other tokens of those chunks
// (phi_k is stored as zero for selected tokens), zero above the diagonal.  Tiles above the diagonal are zero-filled.
// ---------------------------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(256) void attn_map_kernel(AttnMapArgs a) {
  typedef Mma<T> M;
  constexpr int KS = D / M::KK, KP = 2 * D / M::KK;
  const int unit = blockIdx.z, rt = blockIdx.y, kt = blockIdx.x;
  const int b = unit / a.Hq, h = unit % a.Hq, kvh = a.map.kv[h];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l31 = lane & 31, g = lane >> 5, wr = wave >> 1, wc = wave & 1;
  const int N = a.N, C = a.C, r0 = rt * 64, k0 = kt * 64;
  float* out = a.map_out + (int64_t)unit * N * N;
  const int j = k0 + 32 * wc + l31;              // this lane's key
  floatx16 s = zero16(), w = zero16();
  const bool live = kt <= rt;                    // uniform
  if (live) {
    const int tr = min(r0 + 32 * wr + l31, N - 1), jc = min(j, N - 1);
    const T* qp = static_cast<const T*>(a.q) + b * a.q_sb + (int64_t)tr * a.q_st + h * a.q_sh + g * M::KPL;
    const T* kp = static_cast<const T*>(a.k) + b * a.k_sb + (int64_t)jc * a.k_st + kvh * a.k_sh + g * M::KPL;
#pragma unroll
    for (int st = 0; st < KS; ++st) s = M::mma(M::load(qp + st * M::KK), M::load(kp + st * M::KK), s);
    const T* pq = static_cast<const T*>(a.phi_q) + ((int64_t)unit * N + tr) * (2 * D) + g * M::KPL;
    const T* pk = static_cast<const T*>(a.phi_k) + ((int64_t)unit * N + jc) * (2 * D) + g * M::KPL;
#pragma unroll
    for (int st = 0; st < KP; ++st) w = M::mma(M::load(pq + st * M::KK), M::load(pk + st * M::KK), w);
  }
  bool kept = false;
  const int cj = j / C;
  if (live && j < N && cj < a.ncf) {
    const int wi = j % C;
    kept = (a.kmask[((int64_t)unit * a.ncf + cj) * (C / 32) + wi / 32] >> (wi & 31)) & 1u;
  }
  const float sc2 = a.scale * kLog2e;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int t = r0 + 32 * wr + c_row(i, g);
    if (t >= N || j >= N) continue;
    float val = 0.f;
    if (live && j <= t) {
      const int c = t / C;
      const float L = a.lse[(int64_t)unit * N + t];
      if (cj >= c - 1 || kept) val = fast_exp2(fmaf(s[i], sc2, -L * kLog2e));
      else val = __expf(-L) * w[i];
    }
    out[(int64_t)t * N + j] = val;
  }
}

// Backward of the attention map w.r.t. the linear branch's weights: rowdot_t = <dA_t, A_t>, then
// dw_tj = (dA_tj - rowdot_t) exp(-L_t) on the pairs the linear branch owns (token j of a chunk <= c-2 that was not
// selected), zero elsewhere, in the storage type with rows padded to a multiple of 8 (an operand of the matrix core).
__global__ __launch_bounds__(256) void map_rowdot_kernel(const float* A, const float* dA, float* rowdot, int64_t rows, int N) {
  const int64_t row = blockIdx.x * 4ll + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= rows) return;
  const float* a = A + row * N;
  const float* d = dA + row * N;
  float s = 0.f;
  for (int j = lane; j < N; j += 64) s += a[j] * d[j];
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o, 64);
  if (lane == 0) rowdot[row] = s;
}

template <typename T>
__global__ __launch_bounds__(256) void map_dw_kernel(MapDwArgs a) {
  const int unit = blockIdx.z, t = blockIdx.y;
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= a.Np8) return;
  const int c = t / a.C, cj = j / a.C;
  float val = 0.f;
  if (j < a.N && cj <= c - 2) {   // (chunks <= c-2 are full chunks)
    const int wi = j % a.C;
    const bool kept = (a.kmask[((int64_t)unit * a.ncf + cj) * (a.C / 32) + wi / 32] >> (wi & 31)) & 1u;
    const int64_t row = (int64_t)unit * a.N + t;
    if (!kept) val = (a.dA[row * a.N + j] - a.rowdot[row]) * __expf(-a.lse[row]);
  }
  static_cast<T*>(a.dw)[((int64_t)unit * a.N + t) * a.Np8 + j] = from_f32<T>(val);
}

template <typename T, int D>
hipError_t launch_sa_t(const BwdSaArgs& a, int B, hipStream_t s) {
  hipLaunchKernelGGL((bwd_sa_dq_kernel<T, D>), dim3(a.n_row_tiles, B * a.Hq), dim3(256), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // the local tiles first: they store, everything after them adds
  hipLaunchKernelGGL((bwd_sa_dkv_kernel<T, D, true>), dim3(a.n_row_tiles, B * a.Hkv), dim3(256), 0, s, a);
  e = hipGetLastError();
  if (e != hipSuccess || a.n_ret_tiles == 0) return e;
  hipLaunchKernelGGL((bwd_sa_dkv_kernel<T, D, false>), dim3(a.n_ret_tiles, B * a.Hq), dim3(256), 0, s, a);
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

hipError_t launch_bgemm_revscan(const GemmArgs& a, int dtype, int U, int n_c, hipStream_t s) {
  const int bn = a.Nn % 128 == 0 ? 128 : 64;
  const dim3 grid((a.Nn / bn) * (a.M / 64), 1, U);
  if (dtype == 1) {
    if (bn == 128) hipLaunchKernelGGL((bgemm_revscan_kernel<bf16, 128>), grid, dim3(256), 0, s, a, n_c);
    else hipLaunchKernelGGL((bgemm_revscan_kernel<bf16, 64>), grid, dim3(256), 0, s, a, n_c);
  } else {
    if (bn == 128) hipLaunchKernelGGL((bgemm_revscan_kernel<float, 128>), grid, dim3(256), 0, s, a, n_c);
    else hipLaunchKernelGGL((bgemm_revscan_kernel<float, 64>), grid, dim3(256), 0, s, a, n_c);
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
  const int rpb = 256 / (a.d / 8);   // rows per workgroup
  const int blocks = (int)(((int64_t)a.U * a.N + rpb - 1) / rpb);
  if (dtype == 1) hipLaunchKernelGGL((bwd_row_prep_kernel<bf16>), dim3(blocks), dim3(256), 0, s, a);
  else hipLaunchKernelGGL((bwd_row_prep_kernel<float>), dim3(blocks), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_bwd_dg(const BwdRowArgs& a, int dtype, hipStream_t s) {
  const int rpb = 256 / (a.d / 8);
  const int blocks = (int)(((int64_t)a.U * a.N + rpb - 1) / rpb);
  if (dtype == 1) hipLaunchKernelGGL((bwd_dg_kernel<bf16>), dim3(blocks), dim3(256), 0, s, a);
  else hipLaunchKernelGGL((bwd_dg_kernel<float>), dim3(blocks), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_bwd_np(const BwdNpArgs& a, int dtype, bool backward, hipStream_t s) {
  const int rpb = 256 / (a.F / 8);
  const int blocks = (int)(((int64_t)a.U * a.N + rpb - 1) / rpb);
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
  const int rpb = 256 / (a.d / 8);
  const int blocks = (int)(((int64_t)a.B * a.H * a.N + rpb - 1) / rpb);
  if (dtype == 1) hipLaunchKernelGGL((bwd_finish_kernel<bf16>), dim3(blocks), dim3(256), 0, s, a);
  else hipLaunchKernelGGL((bwd_finish_kernel<float>), dim3(blocks), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_map_dw(const MapDwArgs& a, const float* A, int dtype, int U, hipStream_t s) {
  const int64_t rows = (int64_t)U * a.N;
  hipLaunchKernelGGL(map_rowdot_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, A, a.dA, a.rowdot, rows, a.N);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const dim3 grid((a.Np8 + 255) / 256, a.N, U);
  if (dtype == 1) hipLaunchKernelGGL((map_dw_kernel<bf16>), grid, dim3(256), 0, s, a);
  else hipLaunchKernelGGL((map_dw_kernel<float>), grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_attn_map(const AttnMapArgs& a, int dtype, int d, int U, hipStream_t s) {
  const int nt = (a.N + 63) / 64;
  const dim3 grid(nt, nt, U);
  if (dtype == 1) {
    if (d == 128) hipLaunchKernelGGL((attn_map_kernel<bf16, 128>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((attn_map_kernel<bf16, 64>), grid, dim3(256), 0, s, a);
  } else {
    if (d == 128) hipLaunchKernelGGL((attn_map_kernel<float, 128>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((attn_map_kernel<float, 64>), grid, dim3(256), 0, s, a);
  }
  return hipGetLastError();
}

hipError_t launch_bwd_sa(const BwdSaArgs& a, int dtype, int d, int B, hipStream_t s) {
  if (dtype == 1) return d == 128 ? launch_sa_t<bf16, 128>(a, B, s) : launch_sa_t<bf16, 64>(a, B, s);
  if (d == 64) return launch_sa_t<float, 64>(a, B, s);
  return hipErrorInvalidValue;   // fp32 at d = 128 does not fit the tiles in LDS (refused by the host checks)
}

}  // namespace still

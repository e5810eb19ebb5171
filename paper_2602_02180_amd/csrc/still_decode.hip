// Decode step of STILL's recurrent form (paper Sec. 3.3: delayed selection, cache-routing equation, output
// equations) and the export of a decode state from the prefill.
//
// One step is bandwidth-bound: every (batch, query head) reads all its retained keys/values plus the local
// span once.  Kernels of a step, all on the caller's stream:
//   append   : (k_t, v_t) into the ring of recent tokens (slot = t mod R)
//   score    : Self-Saliency Score of token t over its window (Sec. 3.1), one thread per window key
//   route    : only when t opens chunk c >= 2: Top-lambda of chunk c-2 (ties to the lower index), selected
//              rows appended to the retained cache, the others folded into (S, z) through the NP-Map
//   attend   : split over the rows of the salient cache: per split an online-softmax partial (m, l, acc)
//   finish   : NP-Map of q_t, N_LA = phi_q S, D_LA = phi_q z, merge of the split partials,
//              y = (N_SA + g*N_LA) / (D_SA + D_LA) with both branches scaled by exp(-max(m, 0))
// Everything is plain vector-ALU code with fp32 accumulation: there is no contraction here that could
// feed a matrix core (one query row per head).
#include "still_kernels.h"

namespace still {

template <typename T>
struct Vec {
  static constexpr int N = 16 / sizeof(T);
  T v[16 / sizeof(T)];
};

template <typename T>
__device__ __forceinline__ void load16(const T* p, float (&out)[16 / sizeof(T)]) {
  const Vec<T> x = *reinterpret_cast<const Vec<T>*>(p);
#pragma unroll
  for (int e = 0; e < Vec<T>::N; ++e) out[e] = to_f32(x.v[e]);
}

template <typename T>
__device__ __forceinline__ float round_to(float x) {
  return to_f32(from_f32<T>(x));
}

// ---- block reductions over 256 (or fewer) threads; `sh` has room for 4 floats per wave
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// sums a and b, max of c, min of d over the block
__device__ __forceinline__ void block_reduce4(float& a, float& b, float& c, float& d, float* sh, int nwaves) {
  a = wave_sum(a);
  b = wave_sum(b);
  c = wave_max(c);
  d = -wave_max(-d);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) {
    sh[4 * wave + 0] = a;
    sh[4 * wave + 1] = b;
    sh[4 * wave + 2] = c;
    sh[4 * wave + 3] = d;
  }
  __syncthreads();
  a = sh[0]; b = sh[1]; c = sh[2]; d = sh[3];
  for (int w = 1; w < nwaves; ++w) {
    a += sh[4 * w];
    b += sh[4 * w + 1];
    c = fmaxf(c, sh[4 * w + 2]);
    d = fminf(d, sh[4 * w + 3]);
  }
}

// ---------------------------------------------------------------- append
template <typename T>
__device__ __forceinline__ void decode_append(const DecArgs& a, int h, int b, int t, int D) {
  const int slot = t % a.R;
  const T* k = static_cast<const T*>(a.k) + ((int64_t)b * a.Hkv + h) * D;
  const T* v = static_cast<const T*>(a.v) + ((int64_t)b * a.Hkv + h) * D;
  T* kr = static_cast<T*>(a.kring) + (((int64_t)b * a.Hkv + h) * a.R + slot) * D;
  T* vr = static_cast<T*>(a.vring) + (((int64_t)b * a.Hkv + h) * a.R + slot) * D;
  for (int x = threadIdx.x; x < D; x += blockDim.x) {
    kr[x] = k[x];
    vr[x] = v[x];
  }
}

// ---------------------------------------------------------------- score of the new token (+ append)
// Workgroups 0 .. Hq-1 of a sequence score the new token for one query head each; workgroups Hq .. Hq+Hkv-1 copy
// the new key/value rows of one kv head into the ring.  The two do not depend on each other within the step: the
// score reads the new key from the caller's k_t, and the ring slot being overwritten (token t - R) lies outside
// every window (W <= 128 < R).
template <typename T, int D>
__global__ __launch_bounds__(128) void decode_score_kernel(DecArgs a) {
  __shared__ float sh[16];
  const int b = blockIdx.y;
  const int t = step_index(a, b);
  if (t < 0) return;
  if ((int)blockIdx.x >= a.Hq) {
    decode_append<T>(a, blockIdx.x - a.Hq, b, t, D);
    return;
  }
  const int hq = blockIdx.x;
  const int kvh = a.map.kv[hq];
  const int j = threadIdx.x;              // window key t - j
  const int pj = t - j;
  const bool valid = j < a.W && pj >= 0;
  const T* q = static_cast<const T*>(a.q) + ((int64_t)b * a.Hq + hq) * D;
  const T* krow = j == 0 ? static_cast<const T*>(a.k) + ((int64_t)b * a.Hkv + kvh) * D
                         : static_cast<const T*>(a.kring) +
                               (((int64_t)b * a.Hkv + kvh) * a.R + ((valid ? pj : 0) % a.R)) * D;
  float dot = 0.f;
  constexpr int EPV = 16 / sizeof(T);
  if (valid) {
#pragma unroll 4
    for (int x = 0; x < D; x += EPV) {
      float qv[EPV], kv[EPV];
      load16<T>(q + x, qv);
      load16<T>(krow + x, kv);
#pragma unroll
      for (int e = 0; e < EPV; ++e) dot = fmaf(qv[e], kv[e], dot);
    }
  }
  const float x2 = valid ? dot * (a.scale * kLog2e) : -INFINITY;
  float s0 = 0.f, s1 = 0.f, mx = x2, mn = 0.f;
  block_reduce4(s0, s1, mx, mn, sh, 2);
  const float e = valid ? fast_exp2(x2 - mx) : 0.f;
  float d_all = e, d_no = j == 0 ? 0.f : e;
  float c0 = 0.f, c1 = 0.f;
  block_reduce4(d_all, d_no, c0, c1, sh, 2);
  const float inv_all = 1.0f / d_all;
  const float inv_no = d_no > 0.f ? 1.0f / d_no : 0.f;
  const float ad = e * inv_all;
  const float an = j == 0 ? 0.f : e * inv_no;
  float term = valid ? ad * (fast_log2(ad + a.eps) - fast_log2(an + a.eps)) : 0.f;
  float z0 = 0.f, z1 = 0.f, z2 = 0.f;
  block_reduce4(term, z0, z1, z2, sh, 2);
  if (threadIdx.x == 0) a.score[((int64_t)b * a.Hq + hq) * a.R + t % a.R] = term * kLn2;
}

// ---------------------------------------------------------------- routing of chunk cr = t/C - 2
template <typename T, int D>
__global__ __launch_bounds__(256) void decode_route_kernel(DecArgs a, int cr_all) {
  constexpr int DF = D, DP = 2 * D;
  __shared__ float s_sc[128];
  __shared__ unsigned char s_flag[128];
  __shared__ int s_list[128];
  const int hq = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  int cr = cr_all;
  if (a.tpos != nullptr) {   // per-sequence positions: only a sequence whose new token opens a chunk c >= 2 routes
    const int t = step_index(a, b);
    if (t < 0 || t % a.C != 0 || t / a.C < 2) return;
    cr = t / a.C - 2;
  }
  const int kvh = a.map.kv[hq];
  const int C = a.C, lam = a.lam, R = a.R;
  const int quota = chunk_quota(cr, lam, a.rcap);   // what the budget on retained tokens leaves this chunk
  const int64_t unit = (int64_t)b * a.Hq + hq;
  const T* kring = static_cast<const T*>(a.kring) + ((int64_t)b * a.Hkv + kvh) * (int64_t)R * D;
  const T* vring = static_cast<const T*>(a.vring) + ((int64_t)b * a.Hkv + kvh) * (int64_t)R * D;

  if (tid < C) {
    const int slot = (cr * C + tid) % R;
    float s = a.score[unit * R + slot];
    if (a.shared) {   // group-shared selection: rank by the sum over the heads of this kv head, ascending head order
      s = 0.f;
      for (int h = 0; h < a.Hq; ++h)
        if (a.map.kv[h] == kvh) s += a.score[((int64_t)b * a.Hq + h) * R + slot];
    }
    s_sc[tid] = s;
  }
  __syncthreads();
  bool chosen = false;
  if (tid < C) {
    const float si = s_sc[tid];
    int rank = 0;
    for (int jx = 0; jx < C; ++jx) {
      const float sj = s_sc[jx];
      rank += (sj > si || (sj == si && jx < tid)) ? 1 : 0;
    }
    chosen = rank < quota;
    s_flag[tid] = chosen ? 1 : 0;
  }
  __syncthreads();
  if (chosen) {
    int pos = 0;
    for (int jx = 0; jx < tid; ++jx) pos += s_flag[jx];
    if (pos < quota) {
      a.sel[(unit * a.nchunks + cr) * lam + pos] = cr * C + tid;
      s_list[pos] = tid;
    }
  }
  if (tid >= quota && tid < lam) a.sel[(unit * a.nchunks + cr) * lam + tid] = -1;
  __syncthreads();
  // selected rows -> retained cache (rows cr*lam ..)
  if (writes_retained(a.shared != 0, a.map, hq)) {
    const int64_t slice = retained_slice(a.shared != 0, b, hq, kvh, a.Hq, a.Hkv);
    T* kret = static_cast<T*>(a.kret) + (slice * a.cap + (int64_t)cr * lam) * D;
    T* vret = static_cast<T*>(a.vret) + (slice * a.cap + (int64_t)cr * lam) * D;
    for (int idx = tid; idx < quota * D; idx += 256) {
      const int row = idx / D, x = idx % D;
      const int slot = (cr * C + s_list[row]) % R;
      kret[(int64_t)row * D + x] = kring[(int64_t)slot * D + x];
      vret[(int64_t)row * D + x] = vring[(int64_t)slot * D + x];
    }
  }
  // the others -> (S, z): thread f owns row f of S; thread tid also owns the slice part = tid / d_f of column
  // tid % d_f of Wk (a whole column per thread would cost 128 more registers and halve the occupancy).  The tokens
  // are taken TB at a time (in order): one set of barriers per batch instead of one per token.  Per batch:
  //   (A) every thread projects the TB tokens onto its slice of its column; the slices are added in (B),
  //   (B) wave w turns token w's d_f projections into its 2 d_f features (all of a token's features sit in one
  //       wave, two per lane, so the statistics need wave reductions only),
  //   (C) every thread adds the TB rank-1 terms to its row of S, token by token.
  // The key/value rows of the next batch are loaded into registers before (A), so their latency hides behind
  // the arithmetic of the current batch.
  constexpr int TB = 4;
  constexpr int XP = 256 / DF, XS = D / XP;          // slices per column, rows per slice
  constexpr int NLD = TB * D / 256;                  // row elements per thread and batch
  __shared__ __attribute__((aligned(16))) float xs[D][TB], vs[D][TB], fpart[XP][TB][DF], phi[DP][TB];
  __shared__ int s_rest[128];
  __shared__ int s_nrest;
  if (tid < C && !chosen) {
    int before = 0;
    for (int jx = 0; jx < tid; ++jx) before += s_flag[jx];
    s_rest[tid - before] = tid;
  }
  if (tid == 0) {
    int n = 0;
    for (int jx = 0; jx < C; ++jx) n += s_flag[jx] ? 0 : 1;
    s_nrest = n;
  }
  const int fi = tid % DF, part = tid / DF;
  float wcol[XS];
  {
    const T* wk = static_cast<const T*>(a.wk) + (int64_t)hq * D * DF + (int64_t)(part * XS) * DF + fi;
#pragma unroll
    for (int x = 0; x < XS; ++x) wcol[x] = to_f32(wk[(int64_t)x * DF]);
  }
  const int lane = tid & 63, wave = tid >> 6;
  float bias[DF / 64];
#pragma unroll
  for (int h = 0; h < DF / 64; ++h)
    bias[h] = a.bk != nullptr ? to_f32(static_cast<const T*>(a.bk)[(int64_t)hq * DF + lane + 64 * h]) : 0.f;
  float* Sg = a.S + unit * (int64_t)(DP * (D + 1));
  float srow[D];
  float zf = 0.f;
  if (tid < DP) {
#pragma unroll
    for (int x = 0; x < D; ++x) srow[x] = Sg[(int64_t)tid * D + x];
    zf = Sg[DP * D + tid];
  }
  __syncthreads();
  const int n_rest = s_nrest;
  float xn[NLD], vn[NLD];                            // this thread's elements of the next batch's rows
  auto fetch = [&](int i0) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int idx = tid + 256 * i, tb = idx / D, x = idx % D;
      xn[i] = 0.f;
      vn[i] = 0.f;
      if (i0 + tb < n_rest) {
        const int slot = (cr * C + s_rest[i0 + tb]) % R;
        xn[i] = to_f32(kring[(int64_t)slot * D + x]);
        vn[i] = to_f32(vring[(int64_t)slot * D + x]);
      }
    }
  };
  fetch(0);
  for (int i0 = 0; i0 < n_rest; i0 += TB) {
    const int nb = n_rest - i0 < TB ? n_rest - i0 : TB;
    __syncthreads();                             // the previous batch's operands have been consumed
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int idx = tid + 256 * i, tb = idx / D, x = idx % D;
      xs[x][tb] = xn[i];
      vs[x][tb] = vn[i];
    }
    __syncthreads();
    if (i0 + TB < n_rest) fetch(i0 + TB);
    // (A)
    {
      float f[TB];
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) f[tb] = 0.f;
#pragma unroll
      for (int x = 0; x < XS; ++x) {
        const floatx4 x4 = *reinterpret_cast<const floatx4*>(&xs[part * XS + x][0]);
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) f[tb] = fmaf(x4[tb], wcol[x], f[tb]);
      }
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) fpart[part][tb][fi] = f[tb];
    }
    __syncthreads();
    // (B) blockDim = 256 = TB waves
    {
      const int tb = wave;
      float fv[DF / 64], nx2 = 0.f, nf2 = 0.f, fmx = -INFINITY, fmn = INFINITY;
#pragma unroll
      for (int h = 0; h < DF / 64; ++h) {
        float s = 0.f;
#pragma unroll
        for (int pp = 0; pp < XP; ++pp) s += fpart[pp][tb][lane + 64 * h];   // slices in ascending order
        fv[h] = s + bias[h];
        nf2 = fmaf(fv[h], fv[h], nf2);
        fmx = fmaxf(fmx, fv[h]);
        fmn = fminf(fmn, fv[h]);
      }
#pragma unroll
      for (int h = 0; h < D / 64; ++h) nx2 = fmaf(xs[lane + 64 * h][tb], xs[lane + 64 * h][tb], nx2);
      nx2 = wave_sum(nx2);
      nf2 = wave_sum(nf2);
      fmx = wave_max(fmx);
      fmn = -wave_max(-fmn);
      const float ratio = nf2 > 0.f ? sqrtf(nx2 / nf2) : 0.f;
      const float a1 = ratio * kLog2e;
      float ep[DF / 64], en[DF / 64], sp = 0.f, sn = 0.f;
#pragma unroll
      for (int h = 0; h < DF / 64; ++h) {
        ep[h] = fast_exp2(fmaf(fv[h], a1, -fmx * a1));
        en[h] = fast_exp2(fmaf(fv[h], -a1, fmn * a1));
        sp += ep[h];
        sn += en[h];
      }
      sp = wave_sum(sp);
      sn = wave_sum(sn);
      const bool live = tb < nb;
#pragma unroll
      for (int h = 0; h < DF / 64; ++h) {
        phi[lane + 64 * h][tb] = live ? round_to<T>(ep[h] / sp) : 0.f;
        phi[DF + lane + 64 * h][tb] = live ? round_to<T>(en[h] / sn) : 0.f;
      }
    }
    __syncthreads();
    // (C)
    if (tid < DP) {
      const floatx4 pf = *reinterpret_cast<const floatx4*>(&phi[tid][0]);
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) zf += pf[tb];
#pragma unroll
      for (int x = 0; x < D; ++x) {
        const floatx4 v4 = *reinterpret_cast<const floatx4*>(&vs[x][0]);
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) srow[x] = fmaf(pf[tb], v4[tb], srow[x]);
      }
    }
  }
  if (tid < DP) {
#pragma unroll
    for (int x = 0; x < D; ++x) Sg[(int64_t)tid * D + x] = srow[x];
    Sg[DP * D + tid] = zf;
  }
}

// ---------------------------------------------------------------- attention over the salient cache (split)
// Four workgroups per CU (one wave per SIMD each) rather than the eight the registers would allow: every workgroup
// streams its own two rows-of-cache sequences, and with half as many sequences open at a time the memory system
// delivers 1.5 % more (measured at B Hq = 2048 units of 4 K retained rows; more resident waves do not help a
// kernel that is bound by bandwidth, not latency: unrolling the row loop with all loads up front changes nothing).
template <typename T, int D>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4))) void decode_attend_kernel(DecArgs a) {
  constexpr int EPV = 16 / sizeof(T);
  constexpr int LPR = D / EPV;        // lanes per row
  constexpr int RPW = 64 / LPR;       // rows per wave step
  constexpr int NG = 4 * RPW;         // row groups per block
  __shared__ float s_m[NG], s_l[NG], s_acc[NG][D];
  const int split = blockIdx.x, hq = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int sub = lane % LPR, grp = lane / LPR;
  const int kvh = a.map.kv[hq];
  const int64_t unit = (int64_t)b * a.Hq + hq;
  const int t = step_index(a, b);
  if (t < 0) return;
  const int c = t / a.C;
  const int n_ret = retained_rows(c >= 1 ? c - 1 : 0, a.lam, a.rcap);
  const int lo = (c >= 1 ? c - 1 : 0) * a.C;
  const int nr = n_ret + (t - lo + 1);
  int per = (nr + a.nsplit - 1) / a.nsplit;
  per = (per + NG - 1) / NG * NG;
  const int r_beg = split * per;
  const int r_end = r_beg + per < nr ? r_beg + per : nr;

  const int64_t slice = retained_slice(a.shared != 0, b, hq, kvh, a.Hq, a.Hkv);
  const T* kret = static_cast<const T*>(a.kret) + slice * (int64_t)a.cap * D;
  const T* vret = static_cast<const T*>(a.vret) + slice * (int64_t)a.cap * D;
  const T* kring = static_cast<const T*>(a.kring) + ((int64_t)b * a.Hkv + kvh) * (int64_t)a.R * D;
  const T* vring = static_cast<const T*>(a.vring) + ((int64_t)b * a.Hkv + kvh) * (int64_t)a.R * D;

  float qv[EPV];
  load16<T>(static_cast<const T*>(a.q) + unit * D + sub * EPV, qv);
  const float sc2 = a.scale * kLog2e;
  float m2 = -INFINITY, l = 0.f, acc[EPV];
#pragma unroll
  for (int e = 0; e < EPV; ++e) acc[e] = 0.f;

  for (int r0 = r_beg + wave * RPW; r0 < r_end; r0 += NG) {
    const int row = r0 + grp;
    const bool valid = row < r_end;
    const T *kp, *vp;
    if (row < n_ret || !valid) {
      const int rr = valid ? row : 0;
      kp = kret + (int64_t)rr * D;
      vp = vret + (int64_t)rr * D;
    } else {
      const int slot = (lo + (row - n_ret)) % a.R;
      kp = kring + (int64_t)slot * D;
      vp = vring + (int64_t)slot * D;
    }
    float kv[EPV], vv[EPV];
    load16<T>(kp + sub * EPV, kv);
    load16<T>(vp + sub * EPV, vv);
    float dot = 0.f;
#pragma unroll
    for (int e = 0; e < EPV; ++e) dot = fmaf(qv[e], kv[e], dot);
#pragma unroll
    for (int o = LPR / 2; o >= 1; o >>= 1) dot += __shfl_xor(dot, o, 64);
    const float x2 = valid ? dot * sc2 : -INFINITY;
    const float m_new = fmaxf(m2, x2);
    const float m_sub = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = fast_exp2(m2 - m_sub);
    const float pv = fast_exp2(x2 - m_sub);
    l = l * alpha + pv;
#pragma unroll
    for (int e = 0; e < EPV; ++e) acc[e] = fmaf(pv, vv[e], acc[e] * alpha);
    m2 = m_new;
  }
  const int gidx = wave * RPW + grp;
  if (sub == 0) {
    s_m[gidx] = m2;
    s_l[gidx] = l;
  }
#pragma unroll
  for (int e = 0; e < EPV; ++e) s_acc[gidx][sub * EPV + e] = acc[e];
  __syncthreads();
  float M = -INFINITY;
  for (int gi = 0; gi < NG; ++gi) M = fmaxf(M, s_m[gi]);
  float* part = a.part + (unit * 32 + split) * (int64_t)(D + 2);
  if (tid < D) {
    float av = 0.f;
    for (int gi = 0; gi < NG; ++gi) {
      const float w = s_m[gi] == -INFINITY ? 0.f : fast_exp2(s_m[gi] - M);
      av = fmaf(w, s_acc[gi][tid], av);
    }
    part[2 + tid] = av;
  }
  if (tid == 0) {
    float L = 0.f;
    for (int gi = 0; gi < NG; ++gi) {
      const float w = s_m[gi] == -INFINITY ? 0.f : fast_exp2(s_m[gi] - M);
      L = fmaf(w, s_l[gi], L);
    }
    part[0] = M;
    part[1] = L;
  }
}

// ---------------------------------------------------------------- the same, group-shared selection
// With one retained set per kv head, the query heads of a group attend to the same rows: one workgroup per
// (split, kv head, sequence) reads every key/value row once and serves up to GH query heads from it (a larger
// group takes another pass over the rows).  Partials are written per query head, as above.
template <typename T, int D>
__global__ __launch_bounds__(256) void decode_attend_shared_kernel(DecArgs a) {
  constexpr int GH = 4;
  constexpr int EPV = 16 / sizeof(T);
  constexpr int LPR = D / EPV;        // lanes per row
  constexpr int RPW = 64 / LPR;       // rows per wave step
  constexpr int NG = 4 * RPW;         // row groups per block
  __shared__ float s_m[GH][NG], s_l[GH][NG], s_acc[GH][NG][D];
  const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int sub = lane % LPR, grp = lane / LPR;
  const int t = step_index(a, b);
  if (t < 0) return;
  const int c = t / a.C;
  const int n_ret = retained_rows(c >= 1 ? c - 1 : 0, a.lam, a.rcap);
  const int lo = (c >= 1 ? c - 1 : 0) * a.C;
  const int nr = n_ret + (t - lo + 1);
  int per = (nr + a.nsplit - 1) / a.nsplit;
  per = (per + NG - 1) / NG * NG;
  const int r_beg = split * per;
  const int r_end = r_beg + per < nr ? r_beg + per : nr;
  const int64_t slice = (int64_t)b * a.Hkv + kvh;
  const T* kret = static_cast<const T*>(a.kret) + slice * (int64_t)a.cap * D;
  const T* vret = static_cast<const T*>(a.vret) + slice * (int64_t)a.cap * D;
  const T* kring = static_cast<const T*>(a.kring) + slice * (int64_t)a.R * D;
  const T* vring = static_cast<const T*>(a.vring) + slice * (int64_t)a.R * D;
  const float sc2 = a.scale * kLog2e;

  int h_next = 0;
  while (h_next < a.Hq) {
    int heads[GH];   // the next (up to GH) query heads of this kv head, ascending; -1 = none left
#pragma unroll
    for (int g = 0; g < GH; ++g) {
      while (h_next < a.Hq && a.map.kv[h_next] != kvh) ++h_next;
      heads[g] = h_next < a.Hq ? h_next++ : -1;
    }
    if (heads[0] < 0) break;
    float qv[GH][EPV], m2[GH], l[GH], acc[GH][EPV];
#pragma unroll
    for (int g = 0; g < GH; ++g) {
      load16<T>(static_cast<const T*>(a.q) + ((int64_t)b * a.Hq + (heads[g] >= 0 ? heads[g] : heads[0])) * D + sub * EPV, qv[g]);
      m2[g] = -INFINITY;
      l[g] = 0.f;
#pragma unroll
      for (int e = 0; e < EPV; ++e) acc[g][e] = 0.f;
    }
    for (int r0 = r_beg + wave * RPW; r0 < r_end; r0 += NG) {
      const int row = r0 + grp;
      const bool valid = row < r_end;
      const T *kp, *vp;
      if (row < n_ret || !valid) {
        const int rr = valid ? row : 0;
        kp = kret + (int64_t)rr * D;
        vp = vret + (int64_t)rr * D;
      } else {
        const int slot = (lo + (row - n_ret)) % a.R;
        kp = kring + (int64_t)slot * D;
        vp = vring + (int64_t)slot * D;
      }
      float kv[EPV], vv[EPV];
      load16<T>(kp + sub * EPV, kv);
      load16<T>(vp + sub * EPV, vv);
#pragma unroll
      for (int g = 0; g < GH; ++g) {
        float dot = 0.f;
#pragma unroll
        for (int e = 0; e < EPV; ++e) dot = fmaf(qv[g][e], kv[e], dot);
#pragma unroll
        for (int o = LPR / 2; o >= 1; o >>= 1) dot += __shfl_xor(dot, o, 64);
        const float x2 = valid ? dot * sc2 : -INFINITY;
        const float m_new = fmaxf(m2[g], x2);
        const float m_sub = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = fast_exp2(m2[g] - m_sub);
        const float pv = fast_exp2(x2 - m_sub);
        l[g] = l[g] * alpha + pv;
#pragma unroll
        for (int e = 0; e < EPV; ++e) acc[g][e] = fmaf(pv, vv[e], acc[g][e] * alpha);
        m2[g] = m_new;
      }
    }
    const int gidx = wave * RPW + grp;
#pragma unroll
    for (int g = 0; g < GH; ++g) {
      if (sub == 0) {
        s_m[g][gidx] = m2[g];
        s_l[g][gidx] = l[g];
      }
#pragma unroll
      for (int e = 0; e < EPV; ++e) s_acc[g][gidx][sub * EPV + e] = acc[g][e];
    }
    __syncthreads();
#pragma unroll
    for (int g = 0; g < GH; ++g) {
      if (heads[g] < 0) continue;
      float M = -INFINITY;
      for (int gi = 0; gi < NG; ++gi) M = fmaxf(M, s_m[g][gi]);
      float* part = a.part + (((int64_t)b * a.Hq + heads[g]) * 32 + split) * (int64_t)(D + 2);
      if (tid < D) {
        float av = 0.f;
        for (int gi = 0; gi < NG; ++gi) {
          const float w = s_m[g][gi] == -INFINITY ? 0.f : fast_exp2(s_m[g][gi] - M);
          av = fmaf(w, s_acc[g][gi][tid], av);
        }
        part[2 + tid] = av;
      }
      if (tid == 128 + g) {
        float L = 0.f;
        for (int gi = 0; gi < NG; ++gi) {
          const float w = s_m[g][gi] == -INFINITY ? 0.f : fast_exp2(s_m[g][gi] - M);
          L = fmaf(w, s_l[g][gi], L);
        }
        part[0] = M;
        part[1] = L;
      }
    }
    __syncthreads();   // the partial tables are reused by the next pass
  }
}

// ---------------------------------------------------------------- NP-Map of q_t, linear terms, merge
template <typename T, int D>
__global__ __launch_bounds__(256) void decode_finish_kernel(DecArgs a) {
  constexpr int DF = D, DP = 2 * D;
  constexpr int CG = D / 4, RP = 256 / CG;         // column groups of 4 floats, row parts (8 or 16)
  __shared__ float qs[D], phi[DP], sh[16], fpart[2][DF];
  __shared__ __attribute__((aligned(16))) float red[RP][D];
  const int hq = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  if (step_index(a, b) < 0) return;
  const int64_t unit = (int64_t)b * a.Hq + hq;
  const T* q = static_cast<const T*>(a.q) + unit * D;
  if (tid < D) qs[tid] = to_f32(q[tid]);
  __syncthreads();
  // f = q W_q: feature tid % DF, the head dimension split between the block's two halves when d_f = 128
  float f = 0.f;
  {
    constexpr int XP = 256 / DF;                   // 2 (d=128) or 4 (d=64) partial sums per feature
    const int fi = tid % DF, xp = tid / DF;
    const T* wq = static_cast<const T*>(a.wq) + (int64_t)hq * D * DF + fi;
    float fp = 0.f;
#pragma unroll 8
    for (int x = xp * (D / XP); x < (xp + 1) * (D / XP); ++x) fp = fmaf(qs[x], to_f32(wq[(int64_t)x * DF]), fp);
    if (xp >= XP - 2) fpart[xp - (XP - 2)][fi] = fp;
    __syncthreads();
    if (XP == 4) {
      if (xp < 2) fpart[xp][fi] += fp;             // distinct (xp, fi) per thread
      __syncthreads();
    }
    if (tid < DF) {
      f = fpart[0][tid] + fpart[1][tid];
      if (a.bq != nullptr) f += to_f32(static_cast<const T*>(a.bq)[(int64_t)hq * DF + tid]);
    }
  }
  float nx2 = tid < D ? qs[tid] * qs[tid] : 0.f;
  float nf2 = tid < DF ? f * f : 0.f;
  float fmx = tid < DF ? f : -INFINITY, fmn = tid < DF ? f : INFINITY;
  block_reduce4(nx2, nf2, fmx, fmn, sh, 4);
  const float ratio = nf2 > 0.f ? sqrtf(nx2 / nf2) : 0.f;
  const float a1 = ratio * kLog2e;
  float ep = tid < DF ? fast_exp2(fmaf(f, a1, -fmx * a1)) : 0.f;
  float en = tid < DF ? fast_exp2(fmaf(f, -a1, fmn * a1)) : 0.f;
  float sp = ep, sn = en, u0 = 0.f, u1 = 0.f;
  block_reduce4(sp, sn, u0, u1, sh, 4);
  if (tid < DF) {
    phi[tid] = round_to<T>(ep / sp);
    phi[DF + tid] = round_to<T>(en / sn);
  }
  __syncthreads();
  // N_LA[x] = sum_f phi[f] S[f][x]: thread (rp, cg) sums rows rp, rp + RP, ... of four columns with 16-byte
  // loads (the state is the bulk of this kernel's traffic), the row parts are added through LDS
  const float* Sg = a.S + unit * (int64_t)(DP * (D + 1));
  {
    const int cg = tid % CG, rp = tid / CG;
    floatx4 n4 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
    for (int ff = rp; ff < DP; ff += RP) {
      const floatx4 sv = *reinterpret_cast<const floatx4*>(Sg + (int64_t)ff * D + 4 * cg);
      const float pw = phi[ff];
#pragma unroll
      for (int e = 0; e < 4; ++e) n4[e] = fmaf(pw, sv[e], n4[e]);
    }
    *reinterpret_cast<floatx4*>(&red[rp][4 * cg]) = n4;
    __syncthreads();
  }
  float dl = tid < DP ? phi[tid] * Sg[DP * D + tid] : 0.f;
  float d1 = 0.f, d2 = 0.f, d3 = 0.f;
  block_reduce4(dl, d1, d2, d3, sh, 4);
  // merge the split partials
  const float* part = a.part + unit * 32 * (int64_t)(D + 2);
  float M = -INFINITY;
  for (int s = 0; s < a.nsplit; ++s) M = fmaxf(M, part[(int64_t)s * (D + 2)]);
  if (tid < D) {
    float L = 0.f, acc = 0.f;
    for (int s = 0; s < a.nsplit; ++s) {
      const float ms = part[(int64_t)s * (D + 2)];
      const float w = ms == -INFINITY ? 0.f : fast_exp2(ms - M);
      L = fmaf(w, part[(int64_t)s * (D + 2) + 1], L);
      acc = fmaf(w, part[(int64_t)s * (D + 2) + 2 + tid], acc);
    }
    float fs, fl;
    if (M >= 0.f) {
      fs = 1.f;
      fl = fast_exp2(-M);
    } else {
      fs = fast_exp2(M);
      fl = 1.f;
    }
    float nla = 0.f;
#pragma unroll
    for (int rp = 0; rp < RP; ++rp) nla += red[rp][tid];
    if (a.g != nullptr) {
      const float gx = to_f32(static_cast<const T*>(a.g)[unit * D + tid]);
      nla *= a.gate_act ? fast_sigmoid(gx) : gx;
    }
    const float y = (fs * acc + fl * nla) / (fs * L + fl * dl);
    static_cast<T*>(a.out)[unit * D + tid] = from_f32<T>(y);
  }
}

// ---------------------------------------------------------------- state export from the prefill
// ring and score ring <- the last min(N, R) tokens; retained K/V rows and sel <- chunks 0 .. n_routed-1
template <typename T>
__global__ void state_fill_ring_kernel(StateFillArgs a) {
  const int h = blockIdx.y, b = blockIdx.z;     // grid.y = max(Hq, Hkv)
  const int n_tok = seq_tokens(a.seq_len, b, a.N);
  const int first = n_tok > a.R ? n_tok - a.R : 0;
  const int tok = first + blockIdx.x;
  if (tok >= n_tok) return;
  const int slot = tok % a.R;
  if (h < a.Hkv) {
    const T* k = static_cast<const T*>(a.k) + (int64_t)b * a.k_sb + (int64_t)tok * a.k_st + (int64_t)h * a.k_sh;
    const T* v = static_cast<const T*>(a.v) + (int64_t)b * a.v_sb + (int64_t)tok * a.v_st + (int64_t)h * a.v_sh;
    T* kr = static_cast<T*>(a.kring) + (((int64_t)b * a.Hkv + h) * a.R + slot) * a.d;
    T* vr = static_cast<T*>(a.vring) + (((int64_t)b * a.Hkv + h) * a.R + slot) * a.d;
    for (int x = threadIdx.x; x < a.d; x += blockDim.x) {
      kr[x] = k[x];
      vr[x] = v[x];
    }
  }
  if (h < a.Hq && threadIdx.x == 0)
    a.score_ring[((int64_t)b * a.Hq + h) * a.R + slot] = a.score[((int64_t)b * a.Hq + h) * a.N + tok];
}

template <typename T>
__global__ void state_fill_retained_kernel(StateFillArgs a) {
  const int row = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;   // row < n_routed * lam
  const int64_t unit = (int64_t)b * a.Hq + hq;
  const int kvh = a.map.kv[hq];
  const int cr = row / a.lam, pos = row % a.lam;
  if (cr >= (seq_tokens(a.seq_len, b, a.N) + a.C - 1) / a.C - 2) return;   // not yet routed in this sequence
  int tok = a.sel[(unit * a.ncf + cr) * a.lam + pos];
  const bool used = pos < chunk_quota(cr, a.lam, a.rcap);   // the budget on retained tokens leaves later slots empty
  if (threadIdx.x == 0) a.sel_state[(unit * a.nchunks + cr) * a.lam + pos] = used ? tok : -1;
  if (!used || !writes_retained(a.shared != 0, a.map, hq)) return;
  if (tok < 0 || tok >= a.N) tok = 0;
  const T* k = static_cast<const T*>(a.k) + (int64_t)b * a.k_sb + (int64_t)tok * a.k_st + (int64_t)kvh * a.k_sh;
  const T* v = static_cast<const T*>(a.v) + (int64_t)b * a.v_sb + (int64_t)tok * a.v_st + (int64_t)kvh * a.v_sh;
  const int64_t slice = retained_slice(a.shared != 0, b, hq, kvh, a.Hq, a.Hkv);
  T* kr = static_cast<T*>(a.kret) + (slice * a.cap + row) * a.d;
  T* vr = static_cast<T*>(a.vret) + (slice * a.cap + row) * a.d;
  for (int x = threadIdx.x; x < a.d; x += blockDim.x) {
    kr[x] = k[x];
    vr[x] = v[x];
  }
}

// ---------------------------------------------------------------- launchers
#define STILL_DISPATCH(DTYPE, DD, CALL)                     \
  if ((DTYPE) == 1) {                                       \
    if ((DD) == 64) { CALL(bf16, 64) } else { CALL(bf16, 128) } \
  } else {                                                  \
    if ((DD) == 64) { CALL(float, 64) } else { CALL(float, 128) } \
  }

hipError_t launch_decode_step(const DecArgs& a, int dtype, int d, bool route, hipStream_t stream) {
#define CALL_SCORE(TT, DD) hipLaunchKernelGGL((decode_score_kernel<TT, DD>), dim3(a.Hq + a.Hkv, a.B), dim3(128), 0, stream, a);
  STILL_DISPATCH(dtype, d, CALL_SCORE)
  if (route) {
    const int cr = a.t / a.C - 2;
#define CALL_ROUTE(TT, DD) hipLaunchKernelGGL((decode_route_kernel<TT, DD>), dim3(a.Hq, a.B), dim3(256), 0, stream, a, cr);
    STILL_DISPATCH(dtype, d, CALL_ROUTE)
  }
#define CALL_ATT(TT, DD) hipLaunchKernelGGL((decode_attend_kernel<TT, DD>), dim3(a.nsplit, a.Hq, a.B), dim3(256), 0, stream, a);
#define CALL_ATT_SHARED(TT, DD) hipLaunchKernelGGL((decode_attend_shared_kernel<TT, DD>), dim3(a.nsplit, a.Hkv, a.B), dim3(256), 0, stream, a);
  if (a.shared) {
    STILL_DISPATCH(dtype, d, CALL_ATT_SHARED)
  } else {
    STILL_DISPATCH(dtype, d, CALL_ATT)
  }
#define CALL_FIN(TT, DD) hipLaunchKernelGGL((decode_finish_kernel<TT, DD>), dim3(a.Hq, a.B), dim3(256), 0, stream, a);
  STILL_DISPATCH(dtype, d, CALL_FIN)
  return hipGetLastError();
}

hipError_t launch_state_fill(const StateFillArgs& a, int dtype, int B, int n_routed, hipStream_t stream) {
  const int ntok = a.N < a.R ? a.N : a.R;
  const int hy = a.Hq > a.Hkv ? a.Hq : a.Hkv;
  if (dtype == 1)
    hipLaunchKernelGGL(state_fill_ring_kernel<bf16>, dim3(ntok, hy, B), dim3(64), 0, stream, a);
  else
    hipLaunchKernelGGL(state_fill_ring_kernel<float>, dim3(ntok, hy, B), dim3(64), 0, stream, a);
  if (n_routed > 0 && a.lam > 0) {
    if (dtype == 1)
      hipLaunchKernelGGL(state_fill_retained_kernel<bf16>, dim3(n_routed * a.lam, a.Hq, B), dim3(64), 0, stream, a);
    else
      hipLaunchKernelGGL(state_fill_retained_kernel<float>, dim3(n_routed * a.lam, a.Hq, B), dim3(64), 0, stream, a);
  }
  return hipGetLastError();
}

__global__ void fill_zero_kernel(uint32_t* p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}

// a fill kernel rather than hipMemsetAsync, so that a caller may capture the call into a HIP graph
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t stream) {
  const size_t n = bytes / 4;
  if (n == 0) return hipSuccess;
  size_t blocks = (n + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, static_cast<uint32_t*>(p), n);
  return hipGetLastError();
}

}  // namespace still

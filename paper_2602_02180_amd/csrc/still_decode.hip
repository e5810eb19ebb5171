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
// every window (W <= R).  One thread per window key: 128 threads, or 256 for a window of more than 128 keys.
template <typename T, int D>
__global__ __launch_bounds__(256) void decode_score_kernel(DecArgs a) {
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
  const int nwaves = blockDim.x >> 6;
  block_reduce4(s0, s1, mx, mn, sh, nwaves);
  const float e = valid ? fast_exp2(x2 - mx) : 0.f;
  float d_all = e, d_no = j == 0 ? 0.f : e;
  float c0 = 0.f, c1 = 0.f;
  block_reduce4(d_all, d_no, c0, c1, sh, nwaves);
  const float inv_all = 1.0f / d_all;
  const float inv_no = d_no > 0.f ? 1.0f / d_no : 0.f;
  const float ad = e * inv_all;
  const float an = j == 0 ? 0.f : e * inv_no;
  float term = valid ? ad * (fast_log2(ad + a.eps) - fast_log2(an + a.eps)) : 0.f;
  float z0 = 0.f, z1 = 0.f, z2 = 0.f;
  block_reduce4(term, z0, z1, z2, sh, nwaves);
  if (threadIdx.x == 0) a.score[((int64_t)b * a.Hq + hq) * a.R + t % a.R] = term * kLn2;
}

// ---------------------------------------------------------------- routing of chunk cr = t/C - 2
template <typename T, int D>
__global__ __launch_bounds__(256, 2) void decode_route_kernel(DecArgs a, int cr_all) {
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
  const bool evict = a.evict != 0;                  // the budget is held by evicting the lowest score
  // what the budget on retained tokens leaves this chunk (under eviction every chunk offers its lam best)
  const int quota = evict ? lam : chunk_quota(cr, lam, a.rcap);
  const int64_t unit = (int64_t)b * a.Hq + hq;
  extern __shared__ __attribute__((aligned(16))) unsigned char dsm[];
  __shared__ int s_src[128];   // eviction: retained row whose old content a chunk slot carries into the state (-1: none)
  __shared__ int s_dst[128];   // eviction: retained row the i-th offer of the chunk moves into (-1: it is not kept)
  if (tid < 128) {
    s_src[tid] = -1;
    s_dst[tid] = -1;
  }
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
  if (!evict && writes_retained(a.shared != 0, a.map, hq)) {
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
  // Eviction (a budget policy of this library, not of the paper): the retained rows and the chunk's lam offers are
  // ranked together, the `over` lowest scores leave (between equal scores the higher token index first).  An offer
  // that leaves is simply not selected.  A retained row that leaves must enter the state at this step: the offer that
  // takes over its row lends it its slot among the chunk's tokens (a kept token contributes nothing to the state,
  // so its slot is free), and the update below reads that slot's key and value from the retained row instead of
  // the ring.  The offers are copied into their rows only after the update has read the old contents.
  float* rsc = a.ret_score + unit * a.cap;
  int32_t* rtk = a.ret_tok + unit * a.cap;
  if (evict) {
    unsigned long long* keys = reinterpret_cast<unsigned long long*>(dsm);   // (the update's buffers, not yet in use)
    __shared__ unsigned long long s_best[4];
    __shared__ int s_besti[4], s_ev[128], evrow[128];
    __shared__ unsigned char gone[128];
    const int M = a.rcap;
    const int n_old = cr * lam < M ? cr * lam : M;
    const int total = n_old + quota;
    const int over = total > M ? total - M : 0;
    // ascending key order = ascending score, then descending token index
    auto make_key = [](float sc, int tk) -> unsigned long long {
      uint32_t u = __float_as_uint(sc);
      u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
      return ((unsigned long long)u << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)tk);
    };
    __syncthreads();                                      // s_list is complete
    for (int i = tid; i < total; i += 256) {
      if (i < n_old) {
        keys[i] = make_key(rsc[i], rtk[i]);
      } else {
        const int pos = s_list[i - n_old];
        keys[i] = make_key(s_sc[pos], cr * C + pos);
      }
    }
    __syncthreads();
    for (int it = 0; it < over; ++it) {
      unsigned long long best = ~0ull;
      int bi = -1;
      for (int i = tid; i < total; i += 256) {
        const unsigned long long kk = keys[i];
        if (kk < best) best = kk, bi = i;
      }
      for (int off = 32; off > 0; off >>= 1) {
        const unsigned long long ob = __shfl_xor(best, off);
        const int oi = __shfl_xor(bi, off);
        if (ob < best) best = ob, bi = oi;
      }
      if ((tid & 63) == 0) s_best[tid >> 6] = best, s_besti[tid >> 6] = bi;
      __syncthreads();
      if (tid == 0) {
        int w = 0;
        for (int j = 1; j < 4; ++j)
          if (s_best[j] < s_best[w]) w = j;
        s_ev[it] = s_besti[w];
        keys[s_besti[w]] = ~0ull;
      }
      __syncthreads();
    }
    if (tid == 0) {
      // which retained rows leave, which offers leave at once; then a row for every offer that stays: the free
      // rows first, then the rows that were just vacated
      int nev = 0;
      for (int i = 0; i < quota; ++i) gone[i] = 0;
      for (int it = 0; it < over; ++it) {
        const int idx = s_ev[it];
        if (idx < n_old) evrow[nev++] = idx;
        else gone[idx - n_old] = 1;
      }
      int free_row = n_old, e = 0;
      for (int i = 0; i < quota; ++i) {
        const int pos = s_list[i];
        if (gone[i]) {
          s_flag[pos] = 0;                                // joins the chunk's other tokens on their way to the state
        } else {
          const int row = free_row < M ? free_row++ : evrow[e++];
          s_dst[i] = row;
          if (row < n_old) s_src[pos] = row;              // this slot carries the row's old content into the state
        }
      }
    }
    __syncthreads();
  }
  const T* kret_u = static_cast<const T*>(a.kret) + unit * (int64_t)a.cap * D;   // (one slice per unit: not shared)
  const T* vret_u = static_cast<const T*>(a.vret) + unit * (int64_t)a.cap * D;

  // The others -> (S, z), on the matrix core, in parts of PT tokens (PT = 128 two-byte or 64 four-byte tokens, at
  // most the chunk).  LDS holds, per part, the feature image phi^T [2 d_f][PT] and V^T [d][PT] in the storage type
  // (rows padded by 16 bytes), both read as 16-byte operand fragments; at d = 128 the image is built and
  // contracted in two pieces (positive half, negative half) so that two workgroups fit a CU.  W_k^T [d_f][d] is
  // staged into the same memory first (the image is written only after every wave has finished projecting).
  //   projection  f^T = W_k^T x^T: wave w owns tokens [32w, 32w+32) of the chunk, one lane per token and all
  //               features, so the token's statistics are per-lane reductions plus one exchange of lane groups;
  //   features    the two exponential halves, normalised and rounded to the storage type (zero for the tokens the
  //               softmax branch keeps), written to the image;
  //   update      S += phi^T V: wave w owns rows [32w, 32w+32) of every piece of S for every column, loaded into
  //               MFMA accumulators at the start of the kernel and stored at the end; z is the image's row sum.
  typedef Mma<T> M;
  constexpr int EPV = 16 / (int)sizeof(T);
  constexpr int PTMAX = sizeof(T) == 2 ? 128 : 64;
  constexpr int PADE = EPV;                                   // row padding, elements (16 bytes)
  constexpr int WST = D + PADE;                               // W^T row stride
  constexpr int FT = DF / 32, KS = D / M::KK, XT = D / 32;
  constexpr int NH = D == 128 ? 2 : 1;                        // the image is built and contracted in NH pieces of HR rows
  constexpr int HR = DP / NH;                                 //   (d = 128: the positive half, then the negative half)
  static_assert(HR == 128, "a piece is one 32-row tile per wave");
  const int PT = C < PTMAX ? C : PTMAX, nparts = C / PT;
  const int IST = PT + PADE;                                  // image and V^T row stride
  T* wt = reinterpret_cast<T*>(dsm);
  T* img = reinterpret_cast<T*>(dsm);
  T* vtl = img + HR * (PTMAX + PADE);
  const int lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, g = lane >> 5;
  float* Sg = a.S + unit * (int64_t)(DP * (D + 1));

  // W_k [d][d_f] row-major -> W_k^T in LDS
  {
    const T* wk = static_cast<const T*>(a.wk) + (int64_t)hq * D * DF;
    for (int idx = tid; idx < D * DF / EPV; idx += 256) {
      const int kk = idx % D, f0 = (idx / D) * EPV;             // consecutive lanes: consecutive LDS elements
      const Vec16 w16 = *reinterpret_cast<const Vec16*>(wk + (int64_t)kk * DF + f0);
      const T* we = reinterpret_cast<const T*>(&w16);
#pragma unroll
      for (int e = 0; e < EPV; ++e) wt[(f0 + e) * WST + kk] = we[e];
    }
  }
  __syncthreads();

  // projection and statistics of this wave's tokens
  const int tok = 32 * wave + r;                               // token of the chunk owned by this lane
  const bool has_tok = 32 * wave < C;                          // (wave-uniform)
  floatx16 f[FT];
  float a1 = 0.f, bp = 0.f, bn = 0.f, isp = 0.f, isn = 0.f;
  typename M::frag xb[KS];
  if (has_tok) {
    const int slot = (cr * C + tok) % R, src = s_src[tok];
    const T* xp = (src >= 0 ? kret_u + (int64_t)src * D : kring + (int64_t)slot * D) + g * M::KPL;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) xb[ks] = M::load(xp + ks * M::KK);
  }
  // S rows of this wave -> accumulators.  The first piece is issued after the token rows and before the products
  // (loads complete in order, so the next wait that covers them is the one for the V rows, a projection later);
  // the second piece follows when the projection's registers are free.
  floatx16 acc[NH][XT];                                        // piece h: rows h HR + 32 wave + (0..31) of S
  auto load_piece = [&](int h) __attribute__((always_inline)) {
#pragma unroll
    for (int xt = 0; xt < XT; ++xt)
#pragma unroll
      for (int i = 0; i < 16; ++i)
        acc[h][xt][i] = Sg[(int64_t)(h * HR + 32 * wave + c_row(i, g)) * D + 32 * xt + r];
  };
  load_piece(0);
  float zf[NH];
#pragma unroll
  for (int h = 0; h < NH; ++h) zf[h] = tid < HR ? Sg[DP * D + h * HR + tid] : 0.f;

  if (has_tok) {
#pragma unroll
    for (int ft = 0; ft < FT; ++ft) {
      f[ft] = zero16();
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        f[ft] = M::mma(M::load(wt + (32 * ft + r) * WST + ks * M::KK + g * M::KPL), xb[ks], f[ft]);
    }
    if (a.bk != nullptr) {
      const T* bk = static_cast<const T*>(a.bk) + (int64_t)hq * DF;
#pragma unroll
      for (int ft = 0; ft < FT; ++ft)
#pragma unroll
        for (int i = 0; i < 16; ++i) f[ft][i] += to_f32(bk[32 * ft + c_row(i, g)]);
    }
    float x4[4] = {0.f, 0.f, 0.f, 0.f}, q4[4] = {0.f, 0.f, 0.f, 0.f}, mx = -INFINITY, mn = INFINITY;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) x4[ks & 3] = M::dot_into(xb[ks], xb[ks], x4[ks & 3]);
#pragma unroll
    for (int ft = 0; ft < FT; ++ft)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        q4[i & 3] = fmaf(f[ft][i], f[ft][i], q4[i & 3]);
        mx = fmaxf(mx, f[ft][i]);
        mn = fminf(mn, f[ft][i]);
      }
    const float nx2 = sum32((x4[0] + x4[1]) + (x4[2] + x4[3]));
    const float nf2 = sum32((q4[0] + q4[1]) + (q4[2] + q4[3]));
    mx = max32(mx);
    mn = min32(mn);
    const float ratio = nf2 > 0.f ? sqrtf(nx2 / nf2) : 0.f;
    a1 = ratio * kLog2e;
    bp = -mx * a1;
    bn = mn * a1;
    float sp = 0.f, sn = 0.f;
#pragma unroll
    for (int ft = 0; ft < FT; ++ft)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        sp += fast_exp2(fmaf(f[ft][i], a1, bp));
        sn += fast_exp2(fmaf(f[ft][i], -a1, bn));
      }
    isp = 1.0f / sum32(sp);
    isn = 1.0f / sum32(sn);
    if (s_flag[tok] && s_src[tok] < 0) isp = 0.f, isn = 0.f;   // kept by the softmax branch: contributes nothing
  }

  if (NH == 2) load_piece(NH - 1);   // (after the projection's registers are free; arrives under the first piece)
  for (int part = 0; part < nparts; ++part) {
#pragma unroll
    for (int h = 0; h < NH; ++h) {
      __syncthreads();                                         // W^T (or the previous piece) has been consumed
      // features of the part's tokens -> image piece h
      if (has_tok && tok / PT == part) {
        const int tl = tok - part * PT;
#pragma unroll
        for (int ft = 0; ft < FT; ++ft)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int fr = 32 * ft + c_row(i, g);
            if (NH == 1 || h == 0) img[fr * IST + tl] = from_f32<T>(fast_exp2(fmaf(f[ft][i], a1, bp)) * isp);
            if (NH == 1 || h == 1)
              img[((NH == 1 ? DF : 0) + fr) * IST + tl] = from_f32<T>(fast_exp2(fmaf(f[ft][i], -a1, bn)) * isn);
          }
      }
      // V rows of the part -> V^T (once per part)
      if (h == 0) {
        for (int idx = tid; idx < PT * D / EPV; idx += 256) {
          const int tl = idx % PT, x0 = (idx / PT) * EPV;
          const int slot = (cr * C + part * PT + tl) % R, src = s_src[part * PT + tl];
          const Vec16 v16 = *reinterpret_cast<const Vec16*>(
              (src >= 0 ? vret_u + (int64_t)src * D : vring + (int64_t)slot * D) + x0);
          const T* ve = reinterpret_cast<const T*>(&v16);
#pragma unroll
          for (int e = 0; e < EPV; ++e) vtl[(x0 + e) * IST + tl] = ve[e];
        }
      }
      __syncthreads();
      // update of piece h
      for (int ks = 0; ks < PT / M::KK; ++ks) {
        typename M::frag bf[XT];
        const typename M::frag af = M::load(img + (32 * wave + r) * IST + ks * M::KK + g * M::KPL);
#pragma unroll
        for (int xt = 0; xt < XT; ++xt) bf[xt] = M::load(vtl + (32 * xt + r) * IST + ks * M::KK + g * M::KPL);
#pragma unroll
        for (int xt = 0; xt < XT; ++xt) acc[h][xt] = M::mma(af, bf[xt], acc[h][xt]);
      }
      if (tid < HR) {
        float zs = 0.f;
        for (int tl = 0; tl < PT; tl += EPV) {
          const Vec16 p16 = *reinterpret_cast<const Vec16*>(img + tid * IST + tl);
          const T* pe = reinterpret_cast<const T*>(&p16);
#pragma unroll
          for (int e = 0; e < EPV; ++e) zs += to_f32(pe[e]);
        }
        zf[h] += zs;
      }
    }
  }
#pragma unroll
  for (int h = 0; h < NH; ++h)
#pragma unroll
    for (int xt = 0; xt < XT; ++xt)
#pragma unroll
      for (int i = 0; i < 16; ++i)
        Sg[(int64_t)(h * HR + 32 * wave + c_row(i, g)) * D + 32 * xt + r] = acc[h][xt][i];
#pragma unroll
  for (int h = 0; h < NH; ++h)
    if (tid < HR) Sg[DP * D + h * HR + tid] = zf[h];
  if (evict) {
    // the offers that stay move into their rows, now that the old contents have been read (the last reads of the
    // retained rows were the V rows of the last part, before the barrier that preceded its products)
    T* kret_w = static_cast<T*>(a.kret) + unit * (int64_t)a.cap * D;
    T* vret_w = static_cast<T*>(a.vret) + unit * (int64_t)a.cap * D;
    for (int idx = tid; idx < quota * (D / EPV); idx += 256) {
      const int i = idx / (D / EPV), x0 = (idx % (D / EPV)) * EPV;
      const int row = s_dst[i];
      if (row < 0) continue;
      const int slot = (cr * C + s_list[i]) % R;
      *reinterpret_cast<Vec16*>(kret_w + (int64_t)row * D + x0) =
          *reinterpret_cast<const Vec16*>(kring + (int64_t)slot * D + x0);
      *reinterpret_cast<Vec16*>(vret_w + (int64_t)row * D + x0) =
          *reinterpret_cast<const Vec16*>(vring + (int64_t)slot * D + x0);
    }
    if (tid < quota && s_dst[tid] >= 0) {
      rsc[s_dst[tid]] = s_sc[s_list[tid]];
      rtk[s_dst[tid]] = cr * C + s_list[tid];
    }
  }
}

// LDS of the routing kernel: one image piece (128 rows) + V^T of one part, or W_k^T (whichever is larger)
template <typename T, int D>
constexpr size_t decode_route_smem() {
  constexpr int EPV = 16 / (int)sizeof(T), PTMAX = sizeof(T) == 2 ? 128 : 64;
  constexpr size_t part = (size_t)(128 + D) * (PTMAX + EPV) * sizeof(T);
  constexpr size_t w = (size_t)D * (D + EPV) * sizeof(T);
  return part > w ? part : w;
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
  if (!used || a.lists_only || !writes_retained(a.shared != 0, a.map, hq)) return;
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
#define CALL_SCORE(TT, DD) hipLaunchKernelGGL((decode_score_kernel<TT, DD>), dim3(a.Hq + a.Hkv, a.B), dim3(a.W > 128 ? 256 : 128), 0, stream, a);
  STILL_DISPATCH(dtype, d, CALL_SCORE)
  if (route) {
    const int cr = a.t / a.C - 2;
#define CALL_ROUTE(TT, DD)                                                                              \
  {                                                                                                     \
    auto kern = decode_route_kernel<TT, DD>;                                                            \
    const size_t smem = decode_route_smem<TT, DD>();                                                    \
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                             \
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);          \
    if (e != hipSuccess) return e;                                                                      \
    hipLaunchKernelGGL(kern, dim3(a.Hq, a.B), dim3(256), smem, stream, a, cr);                          \
  }
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

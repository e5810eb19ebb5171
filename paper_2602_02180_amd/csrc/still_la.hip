// NP-Map of the keys fused into the chunk-wise scan of the linear-attention state.
//
// Paper: Sec. 3.2 (Norm-Preserved Feature Map: u = f(x)/||f(x)|| * ||x||, phi = softmax(u) (+) softmax(-u)),
// the cache-routing equation of Sec. 3.3 (state s, z summed over the UN-selected tokens of routed chunks)
// and Algorithm 1's linear-attention branch (per-chunk phi_k(k_LA)^T v_LA, cumulative sum over chunks,
// delayed by two chunks).  The other half of the branch, phi_q(q) s and phi_q(q) z for every row, is computed by
// the sparse-attention kernel from the per-chunk states this file leaves in memory.
//
// What is produced: for every (batch, head) and every chunk c >= 0, the state through chunk c-2
//   snap [chunk c] = S^T as [d][2 d_f] in the storage type (the operand layout of the product phi_q S),
//   zsnap[chunk c] = z   as [2 d_f] float,
// and, for the decode hand-over, the fp32 state through chunk (last chunk - 2).
//
// The scan over chunks is sequential per (batch, head); it is cut into segments so that one long sequence still
// fills the chip, and run twice:
//   pass 0 (MODE 0): one workgroup per (batch, head, segment) sums phi_k^T v and sum phi_k over its chunks;
//   la_prefix      : exclusive prefix over the segments (elementwise, tiny);
//   pass 1 (MODE 1): the same walk again, started from the prefix, writing the state after every chunk.
// Segment s covers chunks [s*G-1, (s+1)*G-1), so its prefix is exactly the state through chunk s*G-2, the one
// chunk s*G needs.  Walking twice costs a second NP-Map of the keys; in return every consumer reads ONE complete
// state per chunk, and the fp32 running state is rounded to the storage type exactly once.
//
// Workgroup plan (tokens are handled in rounds of RT = 128 or 64, a round never splits a 32-token tile):
//   producer waves (RT/32): wave v owns tokens [32v, 32v+32) of the round and ALL features: f = W^T x on the
//     matrix core with one lane per token (the token's statistics ||f||^2, max f, min f, ||x||^2 and both softmax
//     sums are then plain per-lane reductions plus one exchange between the two lane groups: no exchange between
//     waves), the two exponential halves normalised and written into the round's LDS image [feature][token].
//     The rows of W^T come from a copy in operand order (1 KB contiguous per load, cache resident).
//   consumer waves (d/32): wave w keeps the fp32 state columns [32w, 32w+32) of S (2 d_f x d) in MFMA
//     accumulators for the whole scan: S += phi_k^T V with phi_k^T from the LDS image (read a fixed number of
//     products ahead) and V from a copy in operand order; z (one feature row per lane) is the row sum of the same
//     image.  After every chunk the accumulators are stored as the next snapshot.
// One barrier per round: the producers fill image (round & 1) while the consumers contract image (round-1 & 1).
#include "still_kernels.h"

namespace still {

template <typename T, int D, int C>
struct LaCfg {
  typedef Mma<T> M;
  static constexpr int DF = D, DP = 2 * DF;
  static constexpr int RT = la_round_tokens((int)sizeof(T), D);
  static constexpr int NCW = D / 32;                // consumer waves
  static constexpr int NPW = RT / 32;               // producer waves
  static constexpr int FT = DF / 32, PT = DP / 32;  // feature tiles per half / of the state
  static constexpr int KS = D / M::KK;              // k-steps of the projection
  static constexpr int PTOK = RT < C ? RT : C;      // tokens per part: a part never crosses a chunk boundary
  static constexpr int NPART = RT / PTOK;           // parts per round (1 or 2)
  static constexpr int HS = PTOK / M::KK;           // k-steps (token groups) per part
  static constexpr int PAD = 16 / (int)sizeof(T);
  static constexpr int KSTRIDE = RT + PAD;          // image row stride (elements)
  static constexpr size_t phi_bytes = sizeof(T) * DP * KSTRIDE;
  static constexpr size_t smem_bytes = 2 * phi_bytes + NPW * 32;   // two images + one keep table per producer
  static_assert(NPART == 1 || NPART == 2, "a round holds one or two chunks, or a part of one");
  static_assert(DP / NCW == 64, "one feature row of z per consumer lane");
};

__device__ __forceinline__ int floor_div(int a, int b) { return a >= 0 ? a / b : -((-a + b - 1) / b); }

template <typename T, int D, int C, int MODE>
__device__ __forceinline__ void la_body(const LaArgs& a) {
  typedef Mma<T> M;
  typedef LaCfg<T, D, C> L;
  constexpr int DF = L::DF, DP = L::DP, RT = L::RT, NCW = L::NCW, FT = L::FT, PT = L::PT, KS = L::KS;
  constexpr int PTOK = L::PTOK, NPART = L::NPART, HS = L::HS, KSTRIDE = L::KSTRIDE;
  constexpr int SPT = M::STEPS_PER_TILE;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* keep = smem + 2 * L::phi_bytes;

  int seg, hq;
  head_major_block(blockIdx.x, a.Hq, hq, seg);
  const int b = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r = lane & 31, g = lane >> 5;
  const int kvh = a.map.kv[hq];
  const int N = seq_tokens(a.seq_len, b, a.N);   // this sequence's tokens (a right-padded batch has shorter ones)
  const int nc_b = (N + C - 1) / C, ncf_b = N / C;
  const int G = a.seg_chunks;
  if (MODE == 1 && seg * G >= nc_b) return;      // the whole segment is padding (uniform over the workgroup)

  const int seg_tok0 = (seg * G - 1) * C;        // first token of the segment's first chunk (chunk -1 for segment 0)
  const int R = G * C / RT;                      // rounds; G * C is a multiple of RT by construction of G
  const int64_t unit = (int64_t)b * a.Hq + hq;
  float* __restrict__ segp = a.seg + (unit * a.nseg + seg) * (int64_t)(DP * (D + 1));

  if (wave >= NCW) {
    // ------------------------------------------------------------------ producer wave v
    const int v = wave - NCW;
    const T* __restrict__ kbase = static_cast<const T*>(a.k) + (int64_t)b * a.k_sb + (int64_t)kvh * a.k_sh;
    const T* __restrict__ wkf = static_cast<const T*>(a.wkf) + (int64_t)hq * DF * D;
    const T* __restrict__ bk = a.bk ? static_cast<const T*>(a.bk) + (int64_t)hq * DF : nullptr;
    unsigned char* kt = keep + v * 32;           // this wave's private table: 1 = token goes to the linear state

    typename M::frag xb[KS];                     // the tile's token rows (B operand of f^T = W^T x^T)
    int32_t selv[2];                             // Top-lambda list of the tile's chunk, entries lane and lane + 64
    auto load_x = [&](int tokw) __attribute__((always_inline)) {
      int tok = tokw + r;
      tok = tok < N ? tok : N - 1;
      tok = tok < 0 ? 0 : tok;
      const T* xp = kbase + (int64_t)tok * a.k_st + g * M::KPL;
#pragma unroll
      for (int s = 0; s < KS; ++s) xb[s] = M::load(xp + s * M::KK);
    };
    auto load_sel = [&](int tokw) __attribute__((always_inline)) {
      const int cc = floor_div(tokw, C);
      const bool valid = cc >= 0 && cc < ncf_b;
      const int32_t* selc = a.sel + (unit * a.ncf + (valid ? cc : 0)) * a.lam;
      const int quota = valid ? chunk_quota(cc, a.lam, a.rcap) : 0;
#pragma unroll
      for (int j = 0; j < 2; ++j) selv[j] = (lane + 64 * j < quota) ? selc[lane + 64 * j] : -1;
    };
    load_x(seg_tok0 + 32 * v);
    load_sel(seg_tok0 + 32 * v);

#pragma unroll 1
    for (int it = 0; it < R; ++it) {
      const int tokw = seg_tok0 + it * RT + 32 * v;      // first token of this wave's tile
      const int cc = floor_div(tokw, C);
      const bool valid = cc >= 0 && cc < ncf_b;          // only full chunks are ever routed
      // keep table of the tile from the list requested a round ago (a wave's own LDS accesses are in order)
      if (lane < 32) kt[lane] = valid ? 1 : 0;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const unsigned off = (unsigned)(selv[j] - tokw);
        if (selv[j] >= 0 && off < 32u) kt[off] = 0;
      }
      // f^T (features x tokens) = W^T x^T, all features of the tile's 32 tokens
      floatx16 f[FT];
#pragma unroll
      for (int ft = 0; ft < FT; ++ft) {
        f[ft] = zero16();
#pragma unroll
        for (int s = 0; s < KS; ++s)
          f[ft] = M::mma(M::load(wkf + wfrag_offset<M>(ft, s, lane, D)), xb[s], f[ft]);
      }
      float nx2 = 0.f;
#pragma unroll
      for (int s = 0; s < KS; ++s) nx2 = M::dot_into(xb[s], xb[s], nx2);
      nx2 = sum32(nx2);
      // the rows are dead now: request the next round's
      if (it + 1 < R) {
        load_x(tokw + RT);
        load_sel(tokw + RT);
      }
      if (bk != nullptr) {
#pragma unroll
        for (int ft = 0; ft < FT; ++ft)
#pragma unroll
          for (int i = 0; i < 16; ++i) f[ft][i] += to_f32(bk[32 * ft + M::pos_of_reg(i, g)]);
      }
      float nf2 = 0.f, fmax = -INFINITY, fmin = INFINITY;
#pragma unroll
      for (int ft = 0; ft < FT; ++ft)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          nf2 = fmaf(f[ft][i], f[ft][i], nf2);
          fmax = fmaxf(fmax, f[ft][i]);
          fmin = fminf(fmin, f[ft][i]);
        }
      nf2 = sum32(nf2);
      fmax = max32(fmax);
      fmin = min32(fmin);
      // u = f * ratio with ratio = ||x|| / ||f|| >= 0, so max/min of u are ratio * max/min of f;
      // exp(u - umax) = exp2(f * a1 - fmax * a1),  exp(umin - u) = exp2(fmin * a1 - f * a1).
      // Tokens kept by the softmax branch (and every token of a chunk that is not routed) get -inf offsets,
      // i.e. zero features.
      const float ratio = nf2 > 0.f ? __builtin_amdgcn_sqrtf(nx2 * fast_rcp(nf2)) : 0.f;
      const float a1 = ratio * kLog2e;
      const bool live = kt[r] != 0;
      const float bp = live ? -fmax * a1 : -INFINITY, bn = live ? fmin * a1 : -INFINITY;
      floatx16 ep[FT], en[FT];
      float sp = 0.f, sn = 0.f;
#pragma unroll
      for (int ft = 0; ft < FT; ++ft)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          ep[ft][i] = fast_exp2(fmaf(f[ft][i], a1, bp));
          en[ft][i] = fast_exp2(fmaf(f[ft][i], -a1, bn));
          sp += ep[ft][i];
          sn += en[ft][i];
        }
      sp = sum32(sp);
      sn = sum32(sn);
      const float ip = sp > 0.f ? fast_rcp(sp) : 0.f, in = sn > 0.f ? fast_rcp(sn) : 0.f;
      // normalised features -> image [feature][token]
      T* img = reinterpret_cast<T*>(smem + (it & 1) * L::phi_bytes) + 32 * v + r;
#pragma unroll
      for (int ft = 0; ft < FT; ++ft)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int fr = 32 * ft + M::pos_of_reg(i, g);
          img[fr * KSTRIDE] = from_f32<T>(ep[ft][i] * ip);
          img[(DF + fr) * KSTRIDE] = from_f32<T>(en[ft][i] * in);
        }
      lds_barrier();
    }
    return;
  }

  // -------------------------------------------------------------------- consumer wave: x columns [32 wave, +32)
  const int col = 32 * wave + r;
  floatx16 S[PT];
  float z;                                       // feature row 64 wave + lane
  if (MODE == 1 && seg > 0) {
#pragma unroll
    for (int ft = 0; ft < PT; ++ft)
#pragma unroll
      for (int i = 0; i < 16; ++i) S[ft][i] = segp[(int64_t)(32 * ft + M::pos_of_reg(i, g)) * D + col];
    z = segp[DP * D + 64 * wave + lane];
  } else {
#pragma unroll
    for (int ft = 0; ft < PT; ++ft) S[ft] = zero16();
    z = 0.f;
  }

  const T* __restrict__ vfr = static_cast<const T*>(a.vfr) + ((int64_t)b * a.Hkv + kvh) * (int64_t)D * a.Np;
  typedef typename M::frag VFrag[HS];            // V fragments of one part (B operand, k = tokens)
  const int NP = R * NPART;                      // parts of the segment
  auto load_v = [&](int gp, VFrag& vf) __attribute__((always_inline)) {
    const int ptok0 = seg_tok0 + gp * PTOK;
    int cc = floor_div(ptok0, C);
    const int within = ptok0 - cc * C;
    const int cmax = a.Np / C - 1;
    cc = cc < 0 ? 0 : (cc > cmax ? cmax : cc);   // a chunk that does not exist meets zero features: any finite V will do
    const T* vrow = vfr + vfr_offset(cc * C, 32 * wave, C, D, M::KK, M::KPL) + (within / M::KK) * 64 * M::KPL +
                    (2 * r + g) * M::KPL;
#pragma unroll
    for (int s = 0; s < HS; ++s) vf[s] = M::load(vrow + s * 64 * M::KPL);
  };

  // the state through chunk oc-2, for the rows of chunk oc
  auto emit = [&](int oc) __attribute__((always_inline)) {
    if (MODE != 1 || oc >= nc_b) return;
    const int lane_now = fresh_lane_id(), rr = lane_now & 31, gg = lane_now >> 5;
    T* sp = static_cast<T*>(a.snap) + (unit * a.nc + oc) * (int64_t)(D * DP) + (int64_t)(32 * wave + rr) * DP;
#pragma unroll
    for (int ft = 0; ft < PT; ++ft)
#pragma unroll
      for (int s = 0; s < SPT; ++s) {
        if constexpr (M::KPL == 1) sp[32 * ft + M::pos_of_reg(s, gg)] = M::from_acc(S[ft], s);
        else *reinterpret_cast<typename M::frag*>(sp + 32 * ft + s * M::KK + gg * M::KPL) = M::from_acc(S[ft], s);
      }
    a.zsnap[(unit * a.nc + oc) * DP + 64 * wave + lane_now] = z;
    if (a.s_final != nullptr && oc == nc_b - 1) {
      float* dst = a.s_final + unit * (int64_t)(DP * (D + 1));
#pragma unroll
      for (int ft = 0; ft < PT; ++ft)
#pragma unroll
        for (int i = 0; i < 16; ++i) dst[(int64_t)(32 * ft + M::pos_of_reg(i, gg)) * D + 32 * wave + rr] = S[ft][i];
      dst[DP * D + 64 * wave + lane_now] = z;
    }
  };

  // S += phi_k^T V and z += row sums for part gp.  The phi_k fragments are read from LDS ADEPTH products ahead of
  // their use (the scheduling barriers pin that order), so a product never waits for its own read.
  constexpr int ADEPTH = 8;
  auto part_step = [&](int gp, const VFrag& vcur, VFrag& vnext) __attribute__((always_inline)) {
    const int rd = gp / NPART, part = gp % NPART;
    if (part == 0) lds_barrier();                // the producers have finished this round's image
    if (gp + 1 < NP) load_v(gp + 1, vnext);
    __builtin_amdgcn_sched_barrier(0);
    const int lane_now = fresh_lane_id(), rr = lane_now & 31, gg = lane_now >> 5;
    const T* img = reinterpret_cast<const T*>(smem + (rd & 1) * L::phi_bytes) + part * PTOK;
    const T* abase = img + M::kappa(rr) * KSTRIDE + gg * M::KPL;
    constexpr int NSTEP = HS * PT;
    auto a_at = [&](int idx) { return M::load(abase + (32 * (idx % PT)) * KSTRIDE + (idx / PT) * M::KK); };
    typename M::frag af[ADEPTH];
#pragma unroll
    for (int i = 0; i < ADEPTH; ++i) af[i] = a_at(i);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int idx = 0; idx < NSTEP; ++idx) {
      S[idx % PT] = M::mma(af[idx % ADEPTH], vcur[idx / PT], S[idx % PT]);
      if (idx + ADEPTH < NSTEP) af[idx % ADEPTH] = a_at(idx + ADEPTH);
      __builtin_amdgcn_sched_barrier(0);
    }
    // z: this lane's feature row of the image, summed over the part's tokens
    {
      const T* zrow = img + (64 * wave + lane_now) * KSTRIDE;
      float zp = 0.f;
#pragma unroll
      for (int s = 0; s < PTOK / M::KPL; ++s) zp = M::sum_into(M::load(zrow + s * M::KPL), zp);
      z += zp;
    }
    const int ptok_end = seg_tok0 + (gp + 1) * PTOK;
    if (ptok_end % C == 0) {                     // a chunk is complete (uniform)
      const int oc = ptok_end / C + 1;           // chunk (ptok_end / C - 1) was absorbed last
      if (oc < (seg + 1) * G) emit(oc);          // the next segment writes its own first chunk
    }
  };

  emit(seg * G);                                 // the prefix itself is the state of the segment's first chunk
  {
    VFrag va, vb;
    load_v(0, va);
#pragma unroll 1
    for (int gp = 0; gp < NP; gp += 2) {
      part_step(gp, va, vb);
      if (gp + 1 < NP) part_step(gp + 1, vb, va);
    }
  }
  if (MODE == 0) {
#pragma unroll
    for (int ft = 0; ft < PT; ++ft)
#pragma unroll
      for (int i = 0; i < 16; ++i) segp[(int64_t)(32 * ft + M::pos_of_reg(i, g)) * D + col] = S[ft][i];
    segp[DP * D + 64 * wave + lane] = z;
  }
}

// (the body lives in a __device__ function behind a thin __global__ wrapper)
template <typename T, int D, int C, int MODE>
__global__ __launch_bounds__((LaCfg<T, D, C>::NCW + LaCfg<T, D, C>::NPW) * 64) void la_kernel(LaArgs a) {
  la_body<T, D, C, MODE>(a);
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
  typedef LaCfg<T, D, C> L;
  auto kern = la_kernel<T, D, C, MODE>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)L::smem_bytes);
  if (e != hipSuccess) return e;
  dim3 grid(nblocks * a.Hq, 1, B), block((L::NCW + L::NPW) * 64);
  hipLaunchKernelGGL(kern, grid, block, L::smem_bytes, stream, a);
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
  return a.C == 64 ? launch_la_t<float, 128, 64, MODE>(a, B, nblocks, stream)
                   : launch_la_t<float, 128, 128, MODE>(a, B, nblocks, stream);
}

hipError_t launch_la_sums(const LaArgs& a, int dtype, int d, int B, hipStream_t stream) {
  return launch_la_mode<0>(a, dtype, d, B, a.nseg - 1, stream);   // the last segment's sum is never needed
}

hipError_t launch_la_prefix(const LaArgs& a, int d, int B, hipStream_t stream) {
  if (a.nseg <= 1) return hipSuccess;
  const int64_t elems = (int64_t)2 * d * (d + 1);
  dim3 grid((unsigned)((elems + 255) / 256), B * a.Hq), block(256);
  hipLaunchKernelGGL(la_prefix_kernel, grid, block, 0, stream, a.seg, a.nseg, elems);
  return hipGetLastError();
}

hipError_t launch_la_states(const LaArgs& a, int dtype, int d, int B, hipStream_t stream) {
  return launch_la_mode<1>(a, dtype, d, B, a.nseg, stream);
}

}  // namespace still

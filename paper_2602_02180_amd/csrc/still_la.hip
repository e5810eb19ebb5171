// NP-Map of the keys fused into the chunk-wise scan of the linear-attention state.
//
// Paper: Sec. 3.2 (Norm-Preserved Feature Map: u = f(x)/||f(x)|| * ||x||, phi = softmax(u) (+) softmax(-u)),
// the cache-routing equation of Sec. 3.3 (state s, z summed over the UN-selected tokens of routed chunks)
// and Algorithm 1's linear-attention branch (per-chunk phi_k(k_LA)^T v_LA, cumulative sum over chunks,
// delayed by two chunks).  The other half of the branch, phi_q(q) s and phi_q(q) z for every row, is computed by
// the sparse-attention kernel from the per-chunk states this file leaves in memory.
//
// The scan over chunks is sequential per (batch, head); it is cut into segments of G chunks so that one long
// sequence still fills the chip, and every segment is walked ONCE, starting from an empty state.  Segment s covers
// chunks [s*G-1, (s+1)*G-1).  What is produced, for every (batch, head):
//   snap [chunk c] = S^T_local as [d][2 d_f] in the storage type: the sum over the chunks s*G-1 .. c-2 of c's own
//                    segment s = c / G (the operand layout of the product phi_q S),
//   zsnap[chunk c] = z_local as [2 d_f] float,
//   seg  [s]       = the segment's total, fp32, which la_prefix turns into the exclusive prefix over segments,
//                    i.e. the state through chunk s*G-2: pimg[s] (storage type, same layout as snap) and zpre[s].
// The state through chunk c-2, which the rows of chunk c need, is pimg[c / G] + snap[c]: the consumer (the
// sparse-attention kernel) contracts phi_q with both.  The product is linear in the state, so nothing is lost, the
// fp32 sums are rounded to the storage type once each, and the keys' NP-Map is computed once.  For the decode
// hand-over the fp32 state through chunk (last chunk - 2) is written as local part here, prefix added by la_prefix.
//
// Workgroup plan (tokens are handled in rounds of RT = 128 or 64, a round never splits a 32-token tile):
//   producer waves (RT/32): wave v owns tokens [32v, 32v+32) of the round and ALL features: f = W^T x on the
//     matrix core with one lane per token (the token's statistics ||f||^2, max f, min f, ||x||^2 and both softmax
//     sums are then plain per-lane reductions plus one exchange between the two lane groups: no exchange between
//     waves), the two exponential halves normalised and written into the round's LDS image [feature][token].
//     The rows of W^T come from a copy in operand order, resident in LDS for the whole scan where it fits next to
//     the two images (every storage type and width but fp32 with d = 128, which reads it from global memory).
//   The image is unpadded: its 16-byte pieces are XOR-swizzled by the feature row (piece ^ swz(row)), chosen so that
//     the operand reads of 32 rows at one token position, the producers' column stores and the row sums for z all
//     spread over the banks.
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
  static constexpr int EPV = 16 / (int)sizeof(T);   // elements per 16-byte piece
  static constexpr int RSTRIDE = RT;                // image row stride (elements): unpadded, swizzled
  static constexpr size_t phi_bytes = sizeof(T) * DP * RSTRIDE;
  static constexpr size_t w_bytes = sizeof(T) * DF * D;
  static constexpr bool W_LDS = 2 * phi_bytes + w_bytes <= 160 * 1024;
  static constexpr size_t smem_bytes = 2 * phi_bytes + (W_LDS ? w_bytes : 0);
  // XOR applied to the index of a row's 16-byte piece: bits (0, 1, 3) of the row go to bits (2, 0, 1)
  static __device__ __forceinline__ int swz(int row) { return ((row & 1) << 2) | ((row >> 1) & 1) | ((row >> 2) & 2); }
  // byte offset of element (row, tok) inside an image
  static __device__ __forceinline__ int img_off(int row, int tok) {
    return (row * RSTRIDE + (((tok / EPV) ^ swz(row)) * EPV) + tok % EPV) * (int)sizeof(T);
  }
  static_assert(NPART == 1 || NPART == 2, "a round holds one or two chunks, or a part of one");
  static_assert(DP / NCW == 64, "one feature row of z per consumer lane");
};

__device__ __forceinline__ int floor_div(int a, int b) { return a >= 0 ? a / b : -((-a + b - 1) / b); }

// SUB: the budget policy that evicts (still_evict.hip): every token position carries the key and value of the token
// a.src names (-1: nothing), and the operand-order copy of v is per query head.
template <typename T, int D, int C, bool SUB>
__device__ __forceinline__ void la_body(const LaArgs& a) {
  typedef Mma<T> M;
  typedef LaCfg<T, D, C> L;
  constexpr int DF = L::DF, DP = L::DP, RT = L::RT, NCW = L::NCW, FT = L::FT, PT = L::PT, KS = L::KS;
  constexpr int PTOK = L::PTOK, NPART = L::NPART, HS = L::HS;
  constexpr int SPT = M::STEPS_PER_TILE;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  T* wl = reinterpret_cast<T*>(smem + 2 * L::phi_bytes);      // W_k^T in operand order (when it fits)

  int seg, hq;
  head_major_block(blockIdx.x, a.Hq, hq, seg);
  const int b = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r = lane & 31, g = lane >> 5;
  const int kvh = a.map.kv[hq];
  const int N = seq_tokens(a.seq_len, b, a.N);   // this sequence's tokens (a right-padded batch has shorter ones)
  const int nc_b = (N + C - 1) / C, ncf_b = N / C;
  const int G = a.seg_chunks;
  if (seg * G >= nc_b) return;                   // the whole segment is padding (uniform over the workgroup)

  const int seg_tok0 = (seg * G - 1) * C;        // first token of the segment's first chunk (chunk -1 for segment 0)
  const int R = G * C / RT;                      // rounds; G * C is a multiple of RT by construction of G
  const int64_t unit = (int64_t)b * a.Hq + hq;
  float* __restrict__ segp = a.seg + (unit * a.nseg + seg) * (int64_t)(DP * (D + 1));

  if (L::W_LDS) {
    const Vec16* src = reinterpret_cast<const Vec16*>(static_cast<const T*>(a.wkf) + (int64_t)hq * DF * D);
    Vec16* dst = reinterpret_cast<Vec16*>(wl);
    for (int i = threadIdx.x; i < (int)(L::w_bytes / 16); i += (NCW + L::NPW) * 64) dst[i] = src[i];
    __syncthreads();
  }

  if (wave >= NCW) {
    // ------------------------------------------------------------------ producer wave v
    // The producers are the critical path of a round (the consumers wait for them at the barrier): where both
    // waves of a SIMD are ready, the producer goes first.
    __builtin_amdgcn_s_setprio(3);
    const int v = wave - NCW;
    const T* __restrict__ kbase = static_cast<const T*>(a.k) + (int64_t)b * a.k_sb + (int64_t)kvh * a.k_sh;
    const T* __restrict__ wkf = static_cast<const T*>(a.wkf) + (int64_t)hq * DF * D;
    const T* __restrict__ bk = a.bk ? static_cast<const T*>(a.bk) + (int64_t)hq * DF : nullptr;

    typename M::frag xb[KS];                     // the tile's token rows (B operand of f^T = W^T x^T)
    uint32_t kw;                                 // bit r: token r of the tile is kept by the softmax branch
    int carried = 0;                             // (SUB) the token this lane's position carries, -1: none
    auto load_x = [&](int tokw) __attribute__((always_inline)) {
      int tok = tokw + r;
      tok = tok < N ? tok : N - 1;
      tok = tok < 0 ? 0 : tok;
      if constexpr (SUB) {
        carried = a.src[unit * a.N + tok];
        tok = carried >= 0 ? carried : tok;
      }
      const T* xp = kbase + (int64_t)tok * a.k_st + g * M::KPL;
#pragma unroll
      for (int s = 0; s < KS; ++s) xb[s] = M::load(xp + s * M::KK);
    };
    // one word of the chunk's keep mask per 32-token tile; all ones for a chunk that is not routed (nothing of it
    // goes to the state)
    auto load_keep = [&](int tokw) __attribute__((always_inline)) {
      const int cc = floor_div(tokw, C);
      const bool valid = cc >= 0 && cc < ncf_b;          // only full chunks are ever routed
      if constexpr (SUB) kw = valid ? 0u : 0xffffffffu;  // (which positions carry nothing comes with the rows)
      else kw = valid ? a.kmask[(unit * a.ncf + cc) * (C / 32) + (tokw - cc * C) / 32] : 0xffffffffu;
    };
    const T* wsrc = L::W_LDS ? wl : wkf;
    // f^T (features x tokens) = W^T x^T, all features of the tile's 32 tokens, and ||x||^2.  The W^T fragments are
    // read WDEPTH products ahead of their use (the scheduling barriers pin that order) and consecutive products go
    // to different accumulators, so a product waits neither for its own read nor for its predecessor.
    floatx16 f[FT];
    float nx2;
    auto project = [&]() __attribute__((always_inline)) {
      constexpr int NPJ = FT * KS, WDEPTH = NPJ < 8 ? NPJ : 8;
      auto w_at = [&](int idx) { return M::load(wsrc + wfrag_offset<M>(idx % FT, idx / FT, lane, D)); };
      typename M::frag wf[WDEPTH];
#pragma unroll
      for (int i = 0; i < WDEPTH; ++i) wf[i] = w_at(i);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int idx = 0; idx < NPJ; ++idx) {
        f[idx % FT] = M::mma(wf[idx % WDEPTH], xb[idx / FT], idx < FT ? zero16() : f[idx % FT]);
        if (idx + WDEPTH < NPJ) wf[idx % WDEPTH] = w_at(idx + WDEPTH);
        __builtin_amdgcn_sched_barrier(0);
      }
      float n4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < KS; ++s) n4[s & 3] = M::dot_into(xb[s], xb[s], n4[s & 3]);
      nx2 = sum32((n4[0] + n4[1]) + (n4[2] + n4[3]));
    };
    load_x(seg_tok0 + 32 * v);
    load_keep(seg_tok0 + 32 * v);

#pragma unroll 1
    for (int it = 0; it < R; ++it) {
      const int tokw = seg_tok0 + it * RT + 32 * v;      // first token of this wave's tile
      const bool live = ((kw >> r) & 1u) == 0u && (!SUB || carried >= 0);
      project();
      if (it + 1 < R) {               // the rows are dead now: request the next round's
        load_x(tokw + RT);
        load_keep(tokw + RT);
      }
      if (bk != nullptr) {
#pragma unroll
        for (int ft = 0; ft < FT; ++ft)
#pragma unroll
          for (int i = 0; i < 16; ++i) f[ft][i] += to_f32(bk[32 * ft + M::pos_of_reg(i, g)]);
      }
      // per-token statistics over this lane's half of the features (four partial chains each), then the other half
      float nf2, fmax, fmin;
      {
        float q4[4] = {0.f, 0.f, 0.f, 0.f}, mx4[4], mn4[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) mx4[c] = -INFINITY, mn4[c] = INFINITY;
#pragma unroll
        for (int ft = 0; ft < FT; ++ft)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            q4[i & 3] = fmaf(f[ft][i], f[ft][i], q4[i & 3]);
            mx4[i & 3] = fmaxf(mx4[i & 3], f[ft][i]);
            mn4[i & 3] = fminf(mn4[i & 3], f[ft][i]);
          }
        nf2 = sum32((q4[0] + q4[1]) + (q4[2] + q4[3]));
        fmax = max32(fmaxf(fmaxf(mx4[0], mx4[1]), fmaxf(mx4[2], mx4[3])));
        fmin = min32(fminf(fminf(mn4[0], mn4[1]), fminf(mn4[2], mn4[3])));
      }
      // u = f * ratio with ratio = ||x|| / ||f|| >= 0, so max/min of u are ratio * max/min of f;
      // exp(u - umax) = exp2(f * a1 - fmax * a1),  exp(umin - u) = exp2(fmin * a1 - f * a1).
      // Tokens kept by the softmax branch (and every token of a chunk that is not routed) get -inf offsets,
      // i.e. zero features.
      const float ratio = nf2 > 0.f ? __builtin_amdgcn_sqrtf(nx2 * fast_rcp(nf2)) : 0.f;
      const float a1 = ratio * kLog2e;
      const float bp = live ? -fmax * a1 : -INFINITY, bn = live ? fmin * a1 : -INFINITY;
      floatx16 ep[FT], en[FT];
      float sp, sn;
      {
        float p4[4] = {0.f, 0.f, 0.f, 0.f}, n4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ft = 0; ft < FT; ++ft)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            ep[ft][i] = fast_exp2(fmaf(f[ft][i], a1, bp));
            en[ft][i] = fast_exp2(fmaf(f[ft][i], -a1, bn));
            p4[i & 3] += ep[ft][i];
            n4[i & 3] += en[ft][i];
          }
        sp = sum32((p4[0] + p4[1]) + (p4[2] + p4[3]));
        sn = sum32((n4[0] + n4[1]) + (n4[2] + n4[3]));
      }
      const float ip = sp > 0.f ? fast_rcp(sp) : 0.f, in = sn > 0.f ? fast_rcp(sn) : 0.f;
      // normalised features -> image [feature][token]
      unsigned char* img = smem + (it & 1) * L::phi_bytes;
      const int tc = 32 * v + r;
      if constexpr (sizeof(T) == 2) {
        // Two features of one token share a register after the conversion; neighbouring lanes (tokens r, r ^ 1)
        // swap halves so that the even lane holds feature f of both tokens and the odd lane feature f + 1: one
        // 4-byte store per lane and feature pair instead of two 2-byte ones.  The row's swizzle depends on the
        // register pair (compile time), the lane group and the lane's parity.
        const int odd = r & 1;
        const uint32_t psel = odd ? 0x03020706u : 0x05040100u;
        const int lane_sw = (odd << 2) | (g << 1);
        const int piece = tc >> 3;
        unsigned char* base0 = img + (8 * g + odd) * (L::RSTRIDE * 2) + (((piece ^ lane_sw) << 4) | (((tc >> 1) & 3) << 2));
        unsigned char* base1 = img + (8 * g + odd) * (L::RSTRIDE * 2) + (((piece ^ lane_sw ^ 1) << 4) | (((tc >> 1) & 3) << 2));
        auto put_pair = [&](float v0, float v1, int row_c, int ci) __attribute__((always_inline)) {
          typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
          bf16x2 pk;
          pk[0] = static_cast<__bf16>(v0);
          pk[1] = static_cast<__bf16>(v1);
          const uint32_t x = __builtin_bit_cast(uint32_t, pk);
          const uint32_t y = (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0xB1, 0xF, 0xF, true);   // lane ^ 1
          const uint32_t w2 = __builtin_amdgcn_perm(y, x, psel);
          *reinterpret_cast<uint32_t*>((ci ? base1 : base0) + row_c * (L::RSTRIDE * 2)) = w2;
        };
#pragma unroll
        for (int ft = 0; ft < FT; ++ft)
#pragma unroll
          for (int i = 0; i < 16; i += 2) {
            const int row_c = 32 * ft + 16 * (i >> 3) + (i & 6);     // compile-time part of the feature row
            put_pair(ep[ft][i] * ip, ep[ft][i + 1] * ip, row_c, (i >> 1) & 1);
            put_pair(en[ft][i] * in, en[ft][i + 1] * in, DF + row_c, (i >> 1) & 1);
          }
      } else {
#pragma unroll
        for (int ft = 0; ft < FT; ++ft)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int fr = 32 * ft + M::pos_of_reg(i, g);
            *reinterpret_cast<T*>(img + L::img_off(fr, tc)) = from_f32<T>(ep[ft][i] * ip);
            *reinterpret_cast<T*>(img + L::img_off(DF + fr, tc)) = from_f32<T>(en[ft][i] * in);
          }
      }
      lds_barrier();
    }
    return;
  }

  // -------------------------------------------------------------------- consumer wave: x columns [32 wave, +32)
  const int col = 32 * wave + r;
  floatx16 S[PT];
  float z;                                       // feature row 64 wave + lane
#pragma unroll
  for (int ft = 0; ft < PT; ++ft) S[ft] = zero16();
  z = 0.f;

  const T* __restrict__ vfr = static_cast<const T*>(a.vfr) +
                              (SUB ? (int64_t)b * a.Hq + hq : (int64_t)b * a.Hkv + kvh) * (int64_t)D * a.Np;
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

  // the segment's running sums, for the rows of chunk oc (the chunks before the segment arrive as its prefix)
  auto emit = [&](int oc) __attribute__((always_inline)) {
    if (oc >= nc_b) return;
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
    const unsigned char* img = smem + (rd & 1) * L::phi_bytes;
    const int arow = M::kappa(rr), asw = L::swz(arow);     // feature tiles start at multiples of 32: same swizzle
    const int tok_l = part * PTOK + gg * M::KPL;           // this lane's first token of k-step 0
    constexpr int NSTEP = HS * PT;
    auto a_at = [&](int idx) {
      const int tok = tok_l + (idx / PT) * M::KK;
      return M::load(reinterpret_cast<const T*>(
          img + ((32 * (idx % PT) + arow) * L::RSTRIDE + (((tok / L::EPV) ^ asw) * L::EPV) + tok % L::EPV) * (int)sizeof(T)));
    };
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
    // z: this lane's feature row of the image, summed over the part's tokens.  The swizzle only permutes the
    // part's 16-byte pieces among themselves (a part is an aligned block of at least 8 pieces), and the order of a
    // sum is free: lane l starts at piece l, so that the lanes of one read spread over the banks.
    {
      constexpr int NPC = PTOK / L::EPV;
      static_assert(NPC >= 8 && (NPC & (NPC - 1)) == 0, "the swizzle stays inside a part");
      const T* zrow = reinterpret_cast<const T*>(img) + (64 * wave + lane_now) * L::RSTRIDE + part * PTOK;
      float zp = 0.f;
#pragma unroll
      for (int j = 0; j < NPC; ++j) {
        const T* pc = zrow + ((j + lane_now) & (NPC - 1)) * L::EPV;
        if constexpr (M::KPL == 8) {
          zp = M::sum_into(M::load(pc), zp);
        } else {
          const floatx4 x = *reinterpret_cast<const floatx4*>(pc);
          zp += (x[0] + x[1]) + (x[2] + x[3]);
        }
      }
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
  // the segment's total, as [x][feature] like the snapshots (written once per workgroup)
  {
    const int lane_now = fresh_lane_id(), rr = lane_now & 31, gg = lane_now >> 5;
    float* tp = segp + (int64_t)(32 * wave + rr) * DP;
#pragma unroll
    for (int ft = 0; ft < PT; ++ft)
#pragma unroll
      for (int i = 0; i < 16; ++i) tp[32 * ft + M::pos_of_reg(i, gg)] = S[ft][i];
    segp[D * DP + 64 * wave + lane_now] = z;
  }
}

// (the body lives in a __device__ function behind a thin __global__ wrapper)
template <typename T, int D, int C, bool SUB>
__global__ __launch_bounds__((LaCfg<T, D, C>::NCW + LaCfg<T, D, C>::NPW) * 64) void la_kernel(LaArgs a) {
  la_body<T, D, C, SUB>(a);
}

// Exclusive prefix over the segments of one (batch, head), elementwise over the state as [x][feature] (+ z):
// pimg[s] / zpre[s] = sum of the totals of the segments before s, i.e. the state through chunk s*G-2; the fp32
// state of the decode hand-over (written by the scan as a local part, laid out [feature][x]) receives the prefix
// of the segment of the sequence's last chunk.
template <typename T>
__global__ __launch_bounds__(256) void la_prefix_kernel(LaArgs a, int D) {
  const int DP = 2 * D;
  const int64_t elems = (int64_t)DP * (D + 1);
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= elems) return;
  const int64_t unit = blockIdx.y;
  const int b = (int)(unit / a.Hq);
  const int N = seq_tokens(a.seq_len, b, a.N);
  const int seg_last = ((N + a.C - 1) / a.C - 1) / a.seg_chunks;     // segment of the sequence's last chunk
  const float* tot = a.seg + unit * a.nseg * elems + idx;
  const bool is_z = idx >= (int64_t)D * DP;
  float run = 0.f;
  for (int s = 0; s < a.nseg; ++s) {
    if (is_z) a.zpre[(unit * a.nseg + s) * DP + (idx - (int64_t)D * DP)] = run;
    else static_cast<T*>(a.pimg)[(unit * a.nseg + s) * (int64_t)(D * DP) + idx] = from_f32<T>(run);
    if (s == seg_last && a.s_final != nullptr) {
      float* sf = a.s_final + unit * elems;
      if (is_z) sf[idx] += run;                                       // z sits behind S in both layouts
      else sf[(idx % DP) * D + idx / DP] += run;                      // [x][feature] -> [feature][x]
    }
    if (s <= seg_last && s + 1 < a.nseg) run += tot[(int64_t)s * elems];   // later segments were never walked
  }
}

template <typename T, int D, int C>
static hipError_t launch_la_t(const LaArgs& a, int B, int nblocks, hipStream_t stream) {
  typedef LaCfg<T, D, C> L;
  auto kern = a.src != nullptr ? la_kernel<T, D, C, true> : la_kernel<T, D, C, false>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)L::smem_bytes);
  if (e != hipSuccess) return e;
  dim3 grid(nblocks * a.Hq, 1, B), block((L::NCW + L::NPW) * 64);
  hipLaunchKernelGGL(kern, grid, block, L::smem_bytes, stream, a);
  return hipGetLastError();
}

hipError_t launch_la_states(const LaArgs& a, int dtype, int d, int B, hipStream_t stream) {
  const int nblocks = a.nseg;
  if (nblocks <= 0) return hipSuccess;
  if (dtype == 1) {
    if (d == 64) return a.C == 64 ? launch_la_t<bf16, 64, 64>(a, B, nblocks, stream)
                                  : launch_la_t<bf16, 64, 128>(a, B, nblocks, stream);
    return a.C == 64 ? launch_la_t<bf16, 128, 64>(a, B, nblocks, stream)
                     : launch_la_t<bf16, 128, 128>(a, B, nblocks, stream);
  }
  if (d == 64) return a.C == 64 ? launch_la_t<float, 64, 64>(a, B, nblocks, stream)
                                : launch_la_t<float, 64, 128>(a, B, nblocks, stream);
  return a.C == 64 ? launch_la_t<float, 128, 64>(a, B, nblocks, stream)
                   : launch_la_t<float, 128, 128>(a, B, nblocks, stream);
}

hipError_t launch_la_prefix(const LaArgs& a, int dtype, int d, int B, hipStream_t stream) {
  const int64_t elems = (int64_t)2 * d * (d + 1);
  dim3 grid((unsigned)((elems + 255) / 256), B * a.Hq), block(256);
  if (dtype == 1) hipLaunchKernelGGL(la_prefix_kernel<bf16>, grid, block, 0, stream, a, d);
  else hipLaunchKernelGGL(la_prefix_kernel<float>, grid, block, 0, stream, a, d);
  return hipGetLastError();
}

}  // namespace still

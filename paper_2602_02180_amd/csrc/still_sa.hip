// Sparse softmax branch over the salient cache, fused with the merge of both branches.
//
// Paper: Sec. 3.3 output equations.  Row t of chunk c attends with exp(scale q.k) to
//   (i)  the retained keys/values of chunks <= c-2 (Algorithm 1: flattened selected K/V under M^Chunk),
//   (ii) the whole previous chunk and its own chunk up to t (s_prev, s_in with the causal mask),
// giving N_SA, D_SA; the linear-attention terms share the normaliser:
//   y = (N_SA + N_LA) / (D_SA + D_LA).
// The linear branch of a row, N_LA = g * phi_q(q) S and D_LA = phi_q(q) z with (S, z) the state through chunk
// c-2 (Algorithm 1's linear branch; NP-Map of Sec. 3.2), is computed HERE, in a prologue, from the per-chunk
// states the scan kernel left in memory: the query fragments are already in registers, phi_q^T (features x
// queries) comes out of the same "tile x Q^T" product as the logits with W_q^T in the role of the key tile, a lane
// owns one query so the NP-Map's statistics are per-lane reductions, and phi_q^T is then the second operand of
// "S^T tile x phi_q^T" exactly as the softmax weights are of "V^T tile x P^T".  The result initialises the online
// softmax: the linear terms enter as if they were one more key with logit 0, weight D_LA and value N_LA / D_LA
// (reference m = 0, running sum D_LA, accumulator N_LA).  From then on the usual rescaling keeps both branches
// under the common factor exp(-max(m, 0)) (any common positive factor cancels; this one can neither overflow nor
// lose the larger branch), and the epilogue is a single division.  N_LA never touches memory.
//
// One workgroup = kSaRows consecutive query rows of one (batch, query head), one wave per 32 rows.
// Everything is computed transposed so that one lane owns one query row:
//   S^T (keys x queries)  = K_tile (A operand, from LDS)  x  Q^T (B operand, registers)
//   O^T (d    x queries) += V^T_tile (A operand, from LDS) x  P^T (B operand = S^T accumulators, in place)
// Data movement: K tiles (64 keys x d) and V^T tiles (d x 64 keys) go from global memory straight into LDS
// (global_load_lds, 16 bytes per lane, no staging registers).  Such a load writes lane L's bytes at
// base + 16 L, so the tiles are unpadded and bank conflicts are avoided by an XOR swizzle of the 16-byte
// column index, applied on the global-address side when loading and on the LDS-address side when reading.
// Software pipeline inside every wave, per iteration i:
//   request K(i+2), V(i+1)  |  S(i+1) = K(i+1) Q^T on the matrix core  |  softmax of S(i) on the vector ALU
//   |  O += V(i) P(i)  |  wait for own requests, barrier
// so the MFMAs of the next tile's logits run under the current tile's exponentials.  Most tiles are retained
// tiles that every row of the wave sees in full; those run in a separate steady-state loop without per-tile
// decisions, with the requests of the step spread over the S products instead of issued in one burst (a wave
// issues in order, and a burst of direct-to-LDS requests holds up everything behind it while the texture path
// works through it).
// The reference m only moves when a row maximum exceeds it by more than 2^8 (the exponentials then stay
// below 2^8, harmless in fp32/bf16), which removes almost all rescales of O.
// Workgroups of one (batch, head) are placed on one XCD (block ids are dealt round-robin to the 8 XCDs), so
// the head's retained K/V (2 MB at 32K tokens) is served from that XCD's L2; long rows are scheduled first.
#include "still_kernels.h"

namespace still {

template <typename T, int D>
struct SaCfg {
  typedef Mma<T> M;
  static constexpr int BM = kSaRows, BN = 64, NW = BM / 32;
  static constexpr int EPV = 16 / sizeof(T);          // elements per 16-byte vector
  static constexpr int KVR = D / EPV;                 // vectors per K row
  static constexpr int VVR = BN / EPV;                // vectors per V^T row
  static constexpr int K_ELEMS = BN * D;              // one K tile
  static constexpr int V_ELEMS = D * BN;              // one V^T tile
  static constexpr int K_INSTR = K_ELEMS / EPV / 64 / NW;   // direct-to-LDS requests per wave and tile
  static constexpr int V_INSTR = V_ELEMS / EPV / 64 / NW;
  static constexpr size_t tile_bytes = 2 * sizeof(T) * (K_ELEMS + V_ELEMS);
  static constexpr size_t smem_bytes = tile_bytes + 2 * (2 * D) * sizeof(float);   // + z of up to two chunks
  // swizzles: XOR applied to the 16-byte column index of a row
  // (a 128-byte row holds 8 columns and two rows share a pass over the banks; longer rows hold >= 16)
  static __device__ __forceinline__ int kswz(int row) { return KVR == 8 ? ((row >> 1) & 7) : (row & 15); }
  static __device__ __forceinline__ int vswz(int row) { return VVR == 8 ? ((row >> 1) & 7) : (row & 15); }
  // element offset inside a tile of element (row, e) with e the element index along the row
  static __device__ __forceinline__ int koff(int row, int e) {
    return row * D + ((((e / EPV) ^ kswz(row))) * EPV) + (e % EPV);
  }
  static __device__ __forceinline__ int voff(int row, int e) {
    return row * BN + ((((e / EPV) ^ vswz(row))) * EPV) + (e % EPV);
  }
};

// S^T tile (64 keys x 32 queries) = K tile x Q^T.  `between(integral_constant<int, idx>)` runs after product idx
// has been issued (the steady-state loop uses it to spread its global->LDS requests over the products).
template <typename T, int D, typename F>
__device__ __forceinline__ void sa_qk(const T* __restrict__ Ks, const typename Mma<T>::frag (&qf)[D / Mma<T>::KK],
                                      floatx16 (&st)[2], int r, int g, F&& between) {
  typedef Mma<T> M;
  typedef SaCfg<T, D> Cf;
  constexpr int KS = D / M::KK;
  st[0] = zero16();
  st[1] = zero16();
  // The K fragments are read from LDS DEPTH products ahead of their use (the scheduling barriers pin that
  // order), so a product does not wait for its own read.
  constexpr int NP = 2 * KS;                 // product idx: key tile idx & 1, k-step idx >> 1
  constexpr int DEPTH = NP < 6 ? NP : 6;
  auto a_at = [&](int idx) { return M::load(Ks + Cf::koff(32 * (idx & 1) + r, (idx >> 1) * M::KK + g * M::KPL)); };
  typename M::frag af[DEPTH];
#pragma unroll
  for (int i = 0; i < DEPTH; ++i) af[i] = a_at(i);
  __builtin_amdgcn_sched_barrier(0);
  static_for<NP>([&](auto IDX) __attribute__((always_inline)) {
    constexpr int idx = decltype(IDX)::value;
    if (idx & 1) st[1] = M::mma(af[idx % DEPTH], qf[idx >> 1], st[1]);
    else st[0] = M::mma(af[idx % DEPTH], qf[idx >> 1], st[0]);
    if (idx + DEPTH < NP) af[idx % DEPTH] = a_at(idx + DEPTH);
    between(IDX);
    __builtin_amdgcn_sched_barrier(0);
  });
}

template <typename T, int D>
__device__ __forceinline__ void sa_qk(const T* __restrict__ Ks, const typename Mma<T>::frag (&qf)[D / Mma<T>::KK],
                                      floatx16 (&st)[2], int r, int g) {
  sa_qk<T, D>(Ks, qf, st, r, g, [](auto) {});
}

// MASK: 0 = every key of the tile is visible to every row of the wave, 1 = retained tile with a ragged end,
//       2 = local tile (window start and causal limit), 3 = retained tile under a bit mask (bit j = key j of the
//       tile is retained for the wave's chunk: the budget policy that evicts, still_evict.hip)
template <typename T, int D, int MASK>
__device__ __forceinline__ void sa_softmax_pv(const T* __restrict__ Vs, floatx16 (&st)[2], floatx16 (&o)[D / 32],
                                              float& m_ref, float& lpart, int kb, int ret_w, int lo_w, int t,
                                              float sc2, int r, int g, unsigned long long bits = 0ull) {
  typedef Mma<T> M;
  typedef SaCfg<T, D> Cf;
  constexpr int DT = D / 32;
  constexpr int SPT = M::STEPS_PER_TILE;
  constexpr float TAU = 8.f;

  if (MASK != 0) {
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = kb + 32 * mt + M::pos_of_reg(i, g);
        const uint32_t half = (uint32_t)(mt ? bits >> 32 : bits);
        const bool valid = MASK == 3 ? ((half >> M::pos_of_reg(i, g)) & 1u) != 0u
                                     : (MASK == 1 ? (key < ret_w) : (key >= lo_w && key <= t));
        st[mt][i] = valid ? st[mt][i] : -INFINITY;
      }
  }
  float tmax = st[0][0];
#pragma unroll
  for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, st[0][i]);
#pragma unroll
  for (int i = 0; i < 16; ++i) tmax = fmaxf(tmax, st[1][i]);
  tmax = max32(tmax);
  const float tm = tmax * sc2;
  if (__any(tm > m_ref + TAU)) {  // wave-uniform; rare once the references have settled
    const float m_new = fmaxf(m_ref, tm);
    const float alpha = m_new == -INFINITY ? 1.f : fast_exp2(m_ref - m_new);
    lpart *= alpha;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[dt][i] *= alpha;
    m_ref = m_new;
  }
  const float m_sub = (MASK != 0 && m_ref == -INFINITY) ? 0.f : m_ref;
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int i = 0; i < 16; ++i) st[mt][i] = fast_exp2(fmaf(st[mt][i], sc2, -m_sub));
  // O^T += V^T P^T.  The row sums are taken over the ROUNDED operand values (one dot-with-ones per pair on
  // bf16), so that numerator and normaliser see the same weights: a row dominated by one key then returns
  // that key's value exactly, whatever the reference m is.
  float rs = 0.f;
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int s = 0; s < SPT; ++s) {
      const typename M::frag pf = M::from_acc(st[mt], s);
      rs = M::sum_into(pf, rs);
      const int e = 32 * mt + s * M::KK + g * M::KPL;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) o[dt] = M::mma(M::load(Vs + Cf::voff(32 * dt + r, e)), pf, o[dt]);
    }
  lpart += rs;
}

// (a __device__ body behind a thin __global__ wrapper keeps the kernel's host-side launch stub simple)
// EV: the budget policy that evicts: the retained tiles are all offers in routing order, each under the bit mask of
// the wave's chunk (a.alive), staged in LDS behind the tiles and the z vectors.
template <typename T, int D, bool EV>
__device__ __forceinline__ void sa_body(const SaArgs& a) {
  typedef Mma<T> M;
  typedef SaCfg<T, D> Cf;
  constexpr int KS = D / M::KK;
  constexpr int DT = D / 32;
  constexpr int BN = Cf::BN;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  T* Kl = reinterpret_cast<T*>(smem);                 // two K tiles
  T* Vl = Kl + 2 * Cf::K_ELEMS;                       // two V^T tiles

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
  const int N = seq_tokens(a.seq_len, b, a.N), C = a.C, lam = a.lam;
  const int kvh = a.map.kv[hq];

  const int row0 = tile * Cf::BM;
  if (row0 >= N) return;   // a tile of padding rows in a right-padded batch (uniform over the workgroup)
  const int q0 = row0 + 32 * wave;
  const int t = q0 + r;
  const bool wave_active = q0 < N;
  const int cw = q0 / C;
  const int ret_w = retained_rows(cw >= 1 ? cw - 1 : 0, lam, a.rcap);   // retained keys visible to this wave
  const int lo_w = (cw >= 1 ? cw - 1 : 0) * C;        // first local key of this wave
  const int c_first = row0 / C;
  const int last_row = (row0 + Cf::BM - 1 < N - 1) ? row0 + Cf::BM - 1 : N - 1;
  const int c_last = last_row / C;
  const int ret_max = retained_rows(c_last >= 1 ? c_last - 1 : 0, lam, a.rcap);
  const int loc_lo = (c_first >= 1 ? c_first - 1 : 0) * C;
  const int n_ret_tiles = (ret_max + BN - 1) / BN;
  const int n_tiles = n_ret_tiles + (last_row + 1 - loc_lo + BN - 1) / BN;
  unsigned long long* aliveL = reinterpret_cast<unsigned long long*>(smem + Cf::tile_bytes + 2 * (2 * D) * 4);
  if constexpr (EV) {
    // mask rows of the tile's chunks (at most two); every wave passes a barrier before the first retained tile
    const unsigned long long* al = static_cast<const unsigned long long*>(a.alive) +
                                   (((int64_t)b * a.Hq + hq) * a.nc + c_first) * (int64_t)a.AW;
    for (int i = tid; i < (c_last - c_first + 1) * a.AW; i += Cf::NW * 64) aliveL[i] = al[i];
  }
  auto tile_bits = [&](int ti) -> unsigned long long { return aliveL[(cw - c_first) * a.AW + ti]; };

  const T* __restrict__ kloc = static_cast<const T*>(a.k) + (int64_t)b * a.k_sb + (int64_t)kvh * a.k_sh;
  const T* __restrict__ vtl = static_cast<const T*>(a.vt) + ((int64_t)b * a.Hkv + kvh) * (int64_t)D * a.Np;
  const T* __restrict__ kret = static_cast<const T*>(a.kret) + ((int64_t)b * a.Hq + hq) * (int64_t)a.cap * D;
  const T* __restrict__ vrett = static_cast<const T*>(a.vrett) + ((int64_t)b * a.Hq + hq) * (int64_t)D * a.cap;
  const int kst = (int)a.k_st;

  // Per-lane constants of the direct-to-LDS requests.  Request j of this wave fills the 1 KB LDS segment
  // number (wave + NW j) of a tile; lane L lands at segment + 16 L, i.e. at LDS (row, slot); it therefore
  // fetches the global 16-byte column  slot ^ swizzle(row)  of the key (K) or feature row (V^T) that LDS row
  // holds.  Every request is "tile base (wave-uniform) + constant per-lane element offset".  Only the offsets
  // into the retained buffers (the steady-state loop's) are kept in registers for the whole kernel; the few
  // general steps of a workgroup rebuild theirs from the lane id, which costs a handful of integer operations
  // per request and keeps eight to sixteen registers out of the loop's allocation.
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  auto k_lane = [&](int lane_now, int j, int& key, int& col) __attribute__((always_inline)) {
    const int v = (wave_s + Cf::NW * j) * 64 + lane_now;     // 16-byte vector index inside the tile
    const int lrow = v / Cf::KVR, slot = v % Cf::KVR;
    key = (lrow & ~31) + M::kappa(lrow & 31);                // LDS row lrow holds key kappa(lrow) of its 32-block
    col = (slot ^ Cf::kswz(lrow)) * Cf::EPV;
  };
  auto v_lane = [&](int lane_now, int j, int& lrow, int& col) __attribute__((always_inline)) {
    const int v = (wave_s + Cf::NW * j) * 64 + lane_now;
    lrow = v / Cf::VVR;
    col = ((v % Cf::VVR) ^ Cf::vswz(lrow)) * Cf::EPV;
  };
  uint32_t k_off_ret[Cf::K_INSTR], v_off_ret[Cf::V_INSTR];
#pragma unroll
  for (int j = 0; j < Cf::K_INSTR; ++j) {
    int key, col;
    k_lane(lane, j, key, col);
    k_off_ret[j] = (uint32_t)(key * D + col);
  }
#pragma unroll
  for (int j = 0; j < Cf::V_INSTR; ++j) {
    int lrow, col;
    v_lane(lane, j, lrow, col);
    v_off_ret[j] = (uint32_t)(lrow * a.cap + col);
  }

  auto tile_kb = [&](int ti) { return ti < n_ret_tiles ? ti * BN : loc_lo + (ti - n_ret_tiles) * BN; };

  auto request_k = [&](int ti) {
    const int kb = tile_kb(ti);
    T* dst = Kl + (ti & 1) * Cf::K_ELEMS + wave_s * 64 * Cf::EPV;
    if (ti < n_ret_tiles) {
      const T* base = kret + (int64_t)kb * D;
#pragma unroll
      for (int j = 0; j < Cf::K_INSTR; ++j)
        async_copy16(base + k_off_ret[j], lds_address(dst + Cf::NW * j * 64 * Cf::EPV));
    } else {
      // rows past the end of a ragged sequence re-read the last token (masked later)
      const int lane_now = fresh_lane_id();
#pragma unroll
      for (int j = 0; j < Cf::K_INSTR; ++j) {
        int key, col;
        k_lane(lane_now, j, key, col);
        int tok = kb + key;
        tok = tok < N ? tok : N - 1;
        async_copy16(kloc + ((int64_t)tok * kst + col), lds_address(dst + Cf::NW * j * 64 * Cf::EPV));
      }
    }
  };
  auto request_v = [&](int ti) {
    const int kb = tile_kb(ti);
    T* dst = Vl + (ti & 1) * Cf::V_ELEMS + wave_s * 64 * Cf::EPV;
    if (ti < n_ret_tiles) {
      const T* base = vrett + kb;
#pragma unroll
      for (int j = 0; j < Cf::V_INSTR; ++j)
        async_copy16(base + v_off_ret[j], lds_address(dst + Cf::NW * j * 64 * Cf::EPV));
    } else {
      const T* base = vtl + kb;
      const int lane_now = fresh_lane_id();
#pragma unroll
      for (int j = 0; j < Cf::V_INSTR; ++j) {
        int lrow, col;
        v_lane(lane_now, j, lrow, col);
        async_copy16(base + ((int64_t)lrow * a.Np + col), lds_address(dst + Cf::NW * j * 64 * Cf::EPV));
      }
    }
  };
  // wave-uniform: does this wave use tile ti, and with which mask variant
  auto tile_mode = [&](int ti) -> int {   // -1 = skip
    if (!wave_active) return -1;
    const int kb = tile_kb(ti);
    if (ti < n_ret_tiles) {
      if constexpr (EV) return (kb < ret_w && tile_bits(ti) != 0ull) ? 3 : -1;
      if (kb + BN <= ret_w) return 0;
      return kb < ret_w ? 1 : -1;
    }
    if (kb + BN - 1 < lo_w || kb > q0 + 31) return -1;
    return (kb >= lo_w && kb + BN - 1 <= q0) ? 0 : 2;
  };

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
  float m_ref = -INFINITY, lpart = 0.f;
  const float sc2 = a.scale * kLog2e;

  // ---- linear branch of the rows (see the header): o = g * phi_q(q) S, lpart = phi_q(q) z, m_ref = 0.
  // Chunks 0 and 1 have no state.  Control flow is uniform over the workgroup (all waves deal the tile requests
  // and meet at the barriers); a wave computes only for its own chunk.
  {
    constexpr int DF = D, DP = 2 * D;
    constexpr int NWT = DF / 64, NST = DP / 64;        // W_q^T tiles (64 features x d), state tiles (d x 64 features)
    constexpr int SPT = M::STEPS_PER_TILE;
    const int la_lo = c_first >= 2 ? c_first : 2, la_hi = c_last;
    bool la_done = false;
    if (la_lo <= la_hi) {
      const int64_t unit = (int64_t)b * a.Hq + hq;
      float* zl = reinterpret_cast<float*>(smem + Cf::tile_bytes);       // [chunk - la_lo][DP]
      const bool mine = wave_active && cw >= 2;                          // this wave has linear terms
      const T* wq_h = static_cast<const T*>(a.wqt) + (int64_t)hq * DF * D;
      auto request_w = [&](int wt, T* slot) {       // W_q^T rows [64 wt, +64): laid out like a tile of retained keys
        const T* base = wq_h + (int64_t)wt * 64 * D;
        T* dst = slot + wave_s * 64 * Cf::EPV;
#pragma unroll
        for (int j = 0; j < Cf::K_INSTR; ++j)
          async_copy16(base + k_off_ret[j], lds_address(dst + Cf::NW * j * 64 * Cf::EPV));
      };
      // columns [64 jt, +64) of a state image [D][DP]: like a V^T tile, row stride DP
      auto request_t = [&](const T* img, int jt, T* slot) {
        const T* base = img + 64 * jt;
        T* dst = slot + wave_s * 64 * Cf::EPV;
        const int lane_now = fresh_lane_id();
#pragma unroll
        for (int j = 0; j < Cf::V_INSTR; ++j) {
          int lrow, col;
          v_lane(lane_now, j, lrow, col);
          async_copy16(base + (lrow * DP + col), lds_address(dst + Cf::NW * j * 64 * Cf::EPV));
        }
      };
      // The state through chunk cc-2 is the sum of two images: the running sums of cc's own segment (operand 0;
      // empty for the first chunk of a segment) and the prefix of that segment (operand 1; empty in segment 0).
      // The product is linear in the state: phi_q^T meets the tiles of both.  Work is dealt in PAIRS of NWT tiles
      // (one half of the features of one operand of one chunk), positive halves first; pair p uses the V slots
      // (p even) or the K slots (p odd), and pair p+1 travels while pair p is contracted.
      const int Gs = a.seg_chunks;
      const T* snap_u = static_cast<const T*>(a.snap) + unit * a.nc * (int64_t)(D * DP);
      const T* pimg_u = static_cast<const T*>(a.pimg) + unit * a.nseg * (int64_t)(D * DP);
      uint32_t codes = 0;      // 4 bits per pair: (chunk - la_lo) << 2 | half << 1 | operand
      int np = 0;
      for (int cc = la_lo; cc <= la_hi; ++cc)
        for (int half = 0; half < 2; ++half)
          for (int op = 0; op < 2; ++op)
            if (op == 0 ? (cc % Gs) != 0 : (cc / Gs) >= 1) {
              codes |= (uint32_t)(((cc - la_lo) << 2) | (half << 1) | op) << (4 * np);
              ++np;
            }
      codes = __builtin_amdgcn_readfirstlane(codes);   // uniform by construction
      np = __builtin_amdgcn_readfirstlane(np);
      constexpr int MAXP = 8;                          // two chunks x two halves x two operands
      static_assert(Cf::K_ELEMS == Cf::V_ELEMS, "the four slots are equal and contiguous: K, K, V, V");
      auto slot_of = [&](int p, int w) -> T* { return Kl + (w + 2 * (1 - (p & 1))) * Cf::K_ELEMS; };
      auto request_pair = [&](int p) __attribute__((always_inline)) {
        const int code = (codes >> (4 * p)) & 7;
        const int cc = la_lo + (code >> 2), half = (code >> 1) & 1;
        const T* img = (code & 1) ? pimg_u + (int64_t)(cc / Gs) * (D * DP) : snap_u + (int64_t)cc * (D * DP);
#pragma unroll
        for (int w = 0; w < NWT; ++w) request_t(img, half * NWT + w, slot_of(p, w));
      };
      // stage 0: W_q^T into the K slots, the first pair into the V slots, z of the chunks
#pragma unroll
      for (int wt = 0; wt < NWT; ++wt) request_w(wt, Kl + wt * Cf::K_ELEMS);
      request_pair(0);
      for (int i = tid; i < (la_hi - la_lo + 1) * DP; i += Cf::NW * 64) {
        const int cc = la_lo + i / DP, fz = i % DP;
        zl[i] = a.zsnap[(unit * a.nc + cc) * DP + fz] + a.zpre[(unit * a.nseg + cc / Gs) * DP + fz];
      }
#pragma unroll
      for (int s = 0; s < KS; ++s) asm volatile("" ::"v"(qf[s]));
      wait_async_copies();
      lds_barrier();

      // phi_q^T of this wave's 32 queries, as operand fragments (un-normalised exponentials; the two normalisers
      // are applied to the accumulator): f^T = W_q^T Q^T, statistics per lane, u = f * ||q|| / ||f||
      typename M::frag pfr[NWT][2][SPT], nfr[NWT][2][SPT];
      float ip = 0.f, in = 0.f, sn_keep = 1.f, dla = 0.f;
      floatx16 f[NWT][2];
      if (mine) {
#pragma unroll
        for (int wt = 0; wt < NWT; ++wt) sa_qk<T, D>(Kl + wt * Cf::K_ELEMS, qf, f[wt], r, g);
      }
      lds_barrier();   // every wave has read W_q^T: the K slots are free
      // the second pair travels to the K slots under the feature map's vector work
      if (np > 1) request_pair(1);
      if (mine) {
        if (a.bq != nullptr) {
          const T* bq = static_cast<const T*>(a.bq) + (int64_t)hq * DF;
#pragma unroll
          for (int wt = 0; wt < NWT; ++wt)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
              for (int i = 0; i < 16; ++i) f[wt][mt][i] += to_f32(bq[64 * wt + 32 * mt + M::pos_of_reg(i, g)]);
        }
        // statistics of the query's features: four partial chains each, then the other lane group's half
        float nx2, nf2, fmax, fmin;
        {
          float x4[4] = {0.f, 0.f, 0.f, 0.f}, q4[4] = {0.f, 0.f, 0.f, 0.f}, mx4[4], mn4[4];
#pragma unroll
          for (int c = 0; c < 4; ++c) mx4[c] = -INFINITY, mn4[c] = INFINITY;
#pragma unroll
          for (int s = 0; s < KS; ++s) x4[s & 3] = M::dot_into(qf[s], qf[s], x4[s & 3]);
#pragma unroll
          for (int wt = 0; wt < NWT; ++wt)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
              for (int i = 0; i < 16; ++i) {
                q4[i & 3] = fmaf(f[wt][mt][i], f[wt][mt][i], q4[i & 3]);
                mx4[i & 3] = fmaxf(mx4[i & 3], f[wt][mt][i]);
                mn4[i & 3] = fminf(mn4[i & 3], f[wt][mt][i]);
              }
          nx2 = sum32((x4[0] + x4[1]) + (x4[2] + x4[3]));
          nf2 = sum32((q4[0] + q4[1]) + (q4[2] + q4[3]));
          fmax = max32(fmaxf(fmaxf(mx4[0], mx4[1]), fmaxf(mx4[2], mx4[3])));
          fmin = min32(fminf(fminf(mn4[0], mn4[1]), fminf(mn4[2], mn4[3])));
        }
        const float ratio = nf2 > 0.f ? __builtin_amdgcn_sqrtf(nx2 * fast_rcp(nf2)) : 0.f;
        const float a1 = ratio * kLog2e;
        const float bp = -fmax * a1, bn = fmin * a1;
        const float* zc = zl + (cw - la_lo) * DP;
        float sp4[4] = {0.f, 0.f, 0.f, 0.f}, sn4[4] = {0.f, 0.f, 0.f, 0.f};
        float dp4[4] = {0.f, 0.f, 0.f, 0.f}, dn4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int wt = 0; wt < NWT; ++wt)
#pragma unroll
          for (int mt = 0; mt < 2; ++mt) {
            floatx16 ep, en;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              ep[i] = fast_exp2(fmaf(f[wt][mt][i], a1, bp));
              en[i] = fast_exp2(fmaf(f[wt][mt][i], -a1, bn));
              sp4[i & 3] += ep[i];
              sn4[i & 3] += en[i];
            }
            // D_LA: the same weights against z.  The features of four consecutive registers are consecutive (both
            // operand conventions), and every lane of a group reads the same address: 16-byte broadcast reads.
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
              const int fi = 64 * wt + 32 * mt + M::pos_of_reg(4 * i4, g);
              if constexpr (M::KPL == 8) {
                const floatx4 zp = *reinterpret_cast<const floatx4*>(zc + fi);
                const floatx4 zn = *reinterpret_cast<const floatx4*>(zc + DF + fi);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                  dp4[e] = fmaf(ep[4 * i4 + e], zp[e], dp4[e]);
                  dn4[e] = fmaf(en[4 * i4 + e], zn[e], dn4[e]);
                }
              } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                  const int fe = 64 * wt + 32 * mt + M::pos_of_reg(4 * i4 + e, g);
                  dp4[e] = fmaf(ep[4 * i4 + e], zc[fe], dp4[e]);
                  dn4[e] = fmaf(en[4 * i4 + e], zc[DF + fe], dn4[e]);
                }
              }
            }
#pragma unroll
            for (int s = 0; s < SPT; ++s) {
              pfr[wt][mt][s] = M::from_acc(ep, s);
              nfr[wt][mt][s] = M::from_acc(en, s);
            }
          }
        const float sp = sum32((sp4[0] + sp4[1]) + (sp4[2] + sp4[3]));
        const float sn = sum32((sn4[0] + sn4[1]) + (sn4[2] + sn4[3]));
        ip = fast_rcp(sp);
        in = fast_rcp(sn);
        sn_keep = sn;
        dla = sum32((dp4[0] + dp4[1]) + (dp4[2] + dp4[3])) * ip + sum32((dn4[0] + dn4[1]) + (dn4[2] + dn4[3])) * in;
      }

      // "S^T tile x phi_q^T" into the accumulator, tile jt from its slot (a wave joins only for its own chunk).  The
      // S^T fragments are read PDEPTH products ahead of their use (the scheduling barriers pin that order).
      auto la_pv = [&](int jt_c, const T* Vs) __attribute__((always_inline)) {
        static_for<NST>([&](auto JT) __attribute__((always_inline)) {
          constexpr int jt = decltype(JT)::value;
          if (jt == jt_c) {
            constexpr int wt = jt % NWT;
            constexpr int NPV = 2 * SPT * DT;                       // product idx: (mt, s) = idx / DT, dt = idx % DT
            constexpr int PDEPTH = NPV < 8 ? NPV : 8;
            auto a_at = [&](int idx) {
              const int ms = idx / DT;
              return M::load(Vs + Cf::voff(32 * (idx % DT) + r, 32 * (ms / SPT) + (ms % SPT) * M::KK + g * M::KPL));
            };
            typename M::frag af[PDEPTH];
#pragma unroll
            for (int i = 0; i < PDEPTH; ++i) af[i] = a_at(i);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int idx = 0; idx < NPV; ++idx) {
              const int ms = idx / DT;
              const typename M::frag pf = jt < NWT ? pfr[wt][ms / SPT][ms % SPT] : nfr[wt][ms / SPT][ms % SPT];
              o[idx % DT] = M::mma(af[idx % PDEPTH], pf, o[idx % DT]);
              if (idx + PDEPTH < NPV) af[idx % PDEPTH] = a_at(idx + PDEPTH);
              __builtin_amdgcn_sched_barrier(0);
            }
          }
        });
      };
      // The steps are laid out at compile time in the order of the codes (chunk, half, operand), so that the
      // fragments a product reads are known statically; whether a step exists, and which slots its pair sits in
      // (pairs alternate between the V and the K slots), is decided at run time, uniformly.
      int pi = 0;                                        // pairs done so far
      static_for<MAXP>([&](auto SS) __attribute__((always_inline)) {
        constexpr int st = decltype(SS)::value;
        constexpr int ci = st >> 2, half = (st >> 1) & 1, op = st & 1;
        const int cc = la_lo + ci;
        if (cc <= la_hi && (op == 0 ? (cc % Gs) != 0 : (cc / Gs) >= 1)) {
          if (pi >= 1 && pi + 1 < np) request_pair(pi + 1);   // (pair 1 was requested above)
          if (mine && cw == cc) {
            if (half == 1 && op == (cc % Gs != 0 ? 0 : 1)) {  // first negative pair: the positive halves are complete;
              const float k1 = ip * sn_keep;                  // (ip / in) A now, + B and * in later = ip A + in B
#pragma unroll
              for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[dt][i] *= k1;
            }
#pragma unroll
            for (int w = 0; w < NWT; ++w) la_pv(half * NWT + w, slot_of(pi, w));
          }
          wait_async_copies();
          lds_barrier();                  // pair pi+1 has arrived everywhere, the slots of pair pi may be refilled
          ++pi;
        }
      });
      if (mine) {
        la_done = true;
        const int tq = t < N ? t : N - 1;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            const int x0 = 32 * dt + 8 * i4 + 4 * g;     // four consecutive columns per register quad
            float gv[4] = {1.f, 1.f, 1.f, 1.f};
            if (a.g != nullptr) {
              const T* gp = static_cast<const T*>(a.g) + (int64_t)b * a.g_sb + (int64_t)tq * a.g_st +
                            (int64_t)hq * a.g_sh + x0;
#pragma unroll
              for (int e = 0; e < 4; ++e) gv[e] = a.gate_act ? fast_sigmoid(to_f32(gp[e])) : to_f32(gp[e]);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) o[dt][4 * i4 + e] *= in * gv[e];
            if (a.n_la_out != nullptr && t < N) {
              floatx4 nv;
#pragma unroll
              for (int e = 0; e < 4; ++e) nv[e] = o[dt][4 * i4 + e];
              *reinterpret_cast<floatx4*>(a.n_la_out + (unit * a.N + t) * D + x0) = nv;
            }
          }
        if (a.d_la_out != nullptr && t < N && g == 0) a.d_la_out[unit * a.N + t] = dla;
        // one more "key": logit 0, weight D_LA, value N_LA / D_LA (an all-kept context has D_LA = 0: no such key)
        if (dla > 0.f) {
          m_ref = 0.f;
          lpart = g == 0 ? dla : 0.f;
        }
      }
    }
    if ((a.n_la_out != nullptr || a.d_la_out != nullptr) && !la_done && wave_active && t < N) {
      // (inspection only) rows without linear terms read as zeros
      const int64_t unit = (int64_t)b * a.Hq + hq;
      if (a.d_la_out != nullptr && g == 0) a.d_la_out[unit * a.N + t] = 0.f;
      if (a.n_la_out != nullptr)
        for (int x = g * (D / 2); x < (g + 1) * (D / 2); ++x) a.n_la_out[(unit * a.N + t) * D + x] = 0.f;
    }
  }

  // ---- prologue: K(0), V(0), K(1) resident; S(0) computed
  request_k(0);
  request_v(0);
  if (n_tiles > 1) request_k(1);
  // The query loads are the only global loads the compiler knows of.  Consuming them here makes it wait for
  // them once, before the loop; otherwise it re-waits at their first use inside every trip of the loop
  // (s_waitcnt vmcnt(n) with small n), which also waits for the tile requests issued just before.
#pragma unroll
  for (int s = 0; s < KS; ++s) asm volatile("" ::"v"(qf[s]));
  wait_async_copies();
  lds_barrier();
  floatx16 st_a[2], st_b[2];
  if (tile_mode(0) >= 0) sa_qk<T, D>(Kl, qf, st_a, r, g);
  lds_barrier();   // every wave has read K(0) before its slot is refilled with K(2)

  // one pipeline step: st_cur holds S(ti); S(ti+1) is started into st_next before the softmax of S(ti)
  auto step = [&](int ti, floatx16 (&st_cur)[2], floatx16 (&st_next)[2]) {
    if (ti + 2 < n_tiles) request_k(ti + 2);          // into the slot S(ti) was computed from
    if (ti + 1 < n_tiles) request_v(ti + 1);          // into the slot the previous step's P V read
    const int mode_next = ti + 1 < n_tiles ? tile_mode(ti + 1) : -1;
    if (mode_next >= 0) sa_qk<T, D>(Kl + ((ti + 1) & 1) * Cf::K_ELEMS, qf, st_next, r, g);
    const int mode = tile_mode(ti);
    const T* Vs = Vl + (ti & 1) * Cf::V_ELEMS;
    const int kb = tile_kb(ti);
    if (mode == 0)
      sa_softmax_pv<T, D, 0>(Vs, st_cur, o, m_ref, lpart, kb, ret_w, lo_w, t, sc2, r, g);
    else if (mode == 1)
      sa_softmax_pv<T, D, 1>(Vs, st_cur, o, m_ref, lpart, kb, ret_w, lo_w, t, sc2, r, g);
    else if (mode == 2)
      sa_softmax_pv<T, D, 2>(Vs, st_cur, o, m_ref, lpart, kb, ret_w, lo_w, t, sc2, r, g);
    else if (EV && mode == 3)
      sa_softmax_pv<T, D, 3>(Vs, st_cur, o, m_ref, lpart, kb, ret_w, lo_w, t, sc2, r, g, tile_bits(ti));
    wait_async_copies();
    lds_barrier();
  };
  // Steady state over the retained set: while tiles ti and ti+1 are fully visible to this wave and the tiles
  // requested during the step (K(ti+2), V(ti+1)) are retained ones, a step needs no per-tile decisions.  Waves
  // may leave this loop at different tiles: both loops execute exactly one barrier per tile.
  auto steady_step = [&](int ti, floatx16 (&st_cur)[2], floatx16 (&st_next)[2]) __attribute__((always_inline)) {
    const T* kbase = kret + (int64_t)(ti + 2) * BN * D;
    const T* vbase = vrett + (ti + 1) * BN;
    T* kdst = Kl + (ti & 1) * Cf::K_ELEMS + wave_s * 64 * Cf::EPV;
    T* vdst = Vl + ((ti + 1) & 1) * Cf::V_ELEMS + wave_s * 64 * Cf::EPV;
    constexpr int NC = Cf::K_INSTR + Cf::V_INSTR, NP = 2 * KS;
    auto issue = [&](auto IDX) __attribute__((always_inline)) {
      constexpr int idx = decltype(IDX)::value;
      static_for<NC>([&](auto CC) __attribute__((always_inline)) {
        constexpr int c = decltype(CC)::value;
        if constexpr ((c * NP) / NC == idx) {   // request c follows product floor(c NP / NC)
          if constexpr (c < Cf::K_INSTR)
            async_copy16(kbase + k_off_ret[c], lds_address(kdst + Cf::NW * c * 64 * Cf::EPV));
          else
            async_copy16(vbase + v_off_ret[c - Cf::K_INSTR],
                         lds_address(vdst + Cf::NW * (c - Cf::K_INSTR) * 64 * Cf::EPV));
        }
      });
    };
    sa_qk<T, D>(Kl + ((ti + 1) & 1) * Cf::K_ELEMS, qf, st_next, r, g, issue);
    if constexpr (EV) {   // every offer of the tile exists for this wave; which of them are retained is in the mask
      const unsigned long long bits = tile_bits(ti);
      if (bits != 0ull)
        sa_softmax_pv<T, D, 3>(Vl + (ti & 1) * Cf::V_ELEMS, st_cur, o, m_ref, lpart, ti * BN, ret_w, lo_w, t, sc2, r, g,
                               bits);
    } else {
      sa_softmax_pv<T, D, 0>(Vl + (ti & 1) * Cf::V_ELEMS, st_cur, o, m_ref, lpart, ti * BN, ret_w, lo_w, t, sc2, r, g);
    }
    wait_async_copies();
    lds_barrier();
  };
  int ti = 0;
  {
    // last even ti (exclusive) such that tiles ti+1 (fully visible) and ti+2, ti+3 (retained) qualify
    int n_steady = wave_active ? ret_w / BN - 1 : 0;             // ti + 1 < ret_w / BN  for both steps of a trip
    if (n_steady > n_ret_tiles - 3) n_steady = n_ret_tiles - 3;  // ti + 3 < n_ret_tiles
    n_steady = __builtin_amdgcn_readfirstlane(n_steady);
    for (; ti < n_steady; ti += 2) {
      steady_step(ti, st_a, st_b);
      steady_step(ti + 1, st_b, st_a);
    }
  }
  for (; ti < n_tiles; ti += 2) {                     // two steps per trip: the S tiles swap roles, no copies
    step(ti, st_a, st_b);
    if (ti + 1 < n_tiles) step(ti + 1, st_b, st_a);
  }

  // ---- epilogue: y = (N_SA + N_LA) / (D_SA + D_LA), both branches already under one factor in the accumulator.
  // In the accumulator layout a lane owns one row and four consecutive columns per register quad, so direct
  // stores of the output would touch 32 rows with 8-16 bytes each per instruction.  The tile therefore passes
  // through LDS (the K/V slots are free after the last barrier, each wave uses a private 32-row region, so no
  // further barrier is needed): every global store is a 1 KB contiguous piece, and the row <-> column exchange
  // happens in LDS, with the 16-byte slot index XOR-ed with the row so that neither direction meets bank conflicts.
  {
    constexpr int ROWB_O = D * (int)sizeof(T), NSO = ROWB_O / 16;  // output row: bytes, 16-byte slots
    constexpr int NOUT = 32 * ROWB_O / 1024;
    static_assert(Cf::NW * 32 * ROWB_O <= (int)Cf::tile_bytes, "epilogue staging fits the tile slots");
    unsigned char* reg = smem + wave_s * (32 * ROWB_O);
    const int lane_now = fresh_lane_id();
    const float lsum = sum32(lpart);
    const float inv = 1.0f / lsum;
    // log of the shared normaliser D_SA + D_LA with the common factor undone (what a backward pass starts from)
    if (a.lse != nullptr && t < N && g == 0)
      a.lse[(int64_t)unit * a.N + t] = (m_ref + fast_log2(lsum)) * 0.6931471805599453f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[dt][i] *= inv;
    // output tile -> LDS in the storage type
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int byte = (32 * dt + 8 * i4 + 4 * g) * (int)sizeof(T);
        unsigned char* dst = reg + r * ROWB_O + (((byte / 16) ^ (r & (NSO - 1))) * 16) + byte % 16;
        if constexpr (sizeof(T) == 2) {
          bf16x4 ov;
#pragma unroll
          for (int e = 0; e < 4; ++e) ov[e] = static_cast<bf16>(o[dt][4 * i4 + e]);
          *reinterpret_cast<bf16x4*>(dst) = ov;
        } else {
          floatx4 ov;
#pragma unroll
          for (int e = 0; e < 4; ++e) ov[e] = o[dt][4 * i4 + e];
          *reinterpret_cast<floatx4*>(dst) = ov;
        }
      }
    // LDS -> global, 1 KB per instruction
    T* obase = static_cast<T*>(a.out) + (int64_t)b * a.o_sb + (int64_t)hq * a.o_sh;
#pragma unroll
    for (int i = 0; i < NOUT; ++i) {
      const int off = i * 1024 + lane_now * 16;
      const int row = off / ROWB_O, slot = (off % ROWB_O) / 16;
      const Vec16 x = *reinterpret_cast<const Vec16*>(reg + row * ROWB_O + ((slot ^ (row & (NSO - 1))) * 16));
      const int tr = q0 + row;
      if (tr < N) *reinterpret_cast<Vec16*>(obase + (int64_t)tr * a.o_st + slot * Cf::EPV) = x;
    }
  }
}

template <typename T, int D, bool EV>
__global__ __launch_bounds__(kSaRows * 2, kSaRows == 128 ? 2 : 1) void sa_kernel(SaArgs a) {
  sa_body<T, D, EV>(a);
}

template <typename T, int D>
static hipError_t launch_sa_t(const SaArgs& a, int B, hipStream_t stream) {
  typedef SaCfg<T, D> Cf;
  const bool ev = a.alive != nullptr;
  auto kern = ev ? sa_kernel<T, D, true> : sa_kernel<T, D, false>;
  const size_t smem = Cf::smem_bytes + (ev ? (size_t)2 * a.AW * 8 : 0);   // + the mask rows of two chunks
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) return e;
  dim3 grid((unsigned)(a.ntiles * a.Hq * B)), block(64 * Cf::NW);
  hipLaunchKernelGGL(kern, grid, block, smem, stream, a);
  return hipGetLastError();
}

hipError_t launch_sa(const SaArgs& a, int dtype, int d, int B, hipStream_t stream) {
  if (dtype == 1) return d == 64 ? launch_sa_t<bf16, 64>(a, B, stream) : launch_sa_t<bf16, 128>(a, B, stream);
  return d == 64 ? launch_sa_t<float, 64>(a, B, stream) : launch_sa_t<float, 128>(a, B, stream);
}

}  // namespace still

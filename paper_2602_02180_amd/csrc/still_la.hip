// NP-Map fused into chunk-wise linear attention.
//
// Paper: Sec. 3.2 (Norm-Preserved Feature Map: u = f(x)/||f(x)|| * ||x||, phi = softmax(u) (+) softmax(-u)),
// the cache-routing equation of Sec. 3.3 (state s, z summed over the UN-selected tokens of routed chunks)
// and Algorithm 1's linear-attention branch (per-chunk phi_k(k_LA)^T v_LA, cumulative sum over chunks,
// delayed by two chunks; numerator phi_q(q) s, normaliser phi_q(q) z).
//
// The chunk scan is cut into segments so that a single long sequence still fills the chip:
//   la_state  (MODE 0): one workgroup per (batch, head, segment) sums  phi_k^T v  and  sum phi_k  over the
//                       segment's chunks, and leaves every staged K unit (LDS slot + softmax sums) in global
//                       memory for the output pass, which needs exactly the same units again.
//   la_prefix          : exclusive prefix over segments (elementwise, tiny).
//   la_out    (MODE 1): one workgroup per (batch, head, segment) starts from the prefix state and walks its
//                       chunks: N_LA, D_LA of chunk c from the state through chunk c-2, then the state
//                       absorbs chunk c-1.  Its producers compute the query features only; the key features
//                       are copied from what the state pass left (they are recomputed only when the scan has
//                       a single segment and no state pass runs).
// Segment s of the state pass covers chunks [s*G-1, (s+1)*G-1), so the exclusive prefix handed to the
// output pass of segment s is exactly the state through chunk s*G-2.
//
// Workgroup plan: the waves are specialised, and wave w shares a SIMD with wave w + d/32.
//   consumer waves (d/32): wave w keeps the fp32 state columns [32w, 32w+32) of S (2*d_f x d) in MFMA
//     accumulators for the whole scan and does the two token-contracting products from LDS operands:
//     S += phi_k^T V (phi_k staged as [feature][token], V from the token-contiguous transposed copy) and
//     N = phi_q S (phi_q staged as [token][feature]; S is the B operand straight from its accumulator
//     registers, converted to the input dtype).  z is kept in LDS in fp32; D_LA = phi_q z is a short
//     dot product per row.
//   producer waves (d_f/32): wave v computes features [32v, 32v+32) of f = x W for ALL tokens of a sub-unit
//     (its rows of W^T stay in registers), exchanges the per-token statistics that span the feature dimension
//     with the other producers through LDS, and writes the two exponential halves UN-normalised into the LDS
//     slot together with its partial softmax sums; the consumers fold the reciprocal sums into their operands.
// Units alternate "queries of chunk c" / "keys of chunk c-1" so that the outputs of chunk c see the state
// through chunk c-2; a unit is cut into sub-units of 64 tokens, and one barrier per sub-unit interval hands data
// from the projection step to the exponential step to the consumers.
#include "still_kernels.h"
#include <type_traits>

namespace still {

template <typename T>
struct LaPad {
  static constexpr int value = 16 / sizeof(T);
};

// sum over the fragment's k positions of  f[e] * w[e]
template <typename T>
__device__ __forceinline__ float frag_dot(typename Mma<T>::frag f, const float* __restrict__ w) {
  if constexpr (Mma<T>::KPL == 1) {
    return f * w[0];
  } else {
    float acc = 0.f;
#pragma unroll
    for (int e = 0; e < Mma<T>::KPL; ++e) acc += to_f32(f[e]) * w[e];
    return acc;
  }
}

// fragment with element e multiplied by w[e] (rounded back to the operand type)
template <typename T>
__device__ __forceinline__ typename Mma<T>::frag frag_scale(typename Mma<T>::frag f, const float* __restrict__ w) {
  if constexpr (Mma<T>::KPL == 1) {
    return f * w[0];
  } else {
    typename Mma<T>::frag o;
#pragma unroll
    for (int e = 0; e < Mma<T>::KPL; ++e) o[e] = from_f32<T>(to_f32(f[e]) * w[e]);
    return o;
  }
}

// 16 bytes of raw data carried in an operand-fragment register set (16-byte fragments only)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
template <typename F>
__device__ __forceinline__ F frag_from_bits(u32x4 x) {
  if constexpr (sizeof(F) == 16) return __builtin_bit_cast(F, x);
  else return F{};
}
template <typename F>
__device__ __forceinline__ u32x4 frag_to_bits(F f) {
  if constexpr (sizeof(F) == 16) return __builtin_bit_cast(u32x4, f);
  else return u32x4{};
}

template <typename T, int D, int DF, int C>
struct LaSmem {
  static constexpr int DP = 2 * DF;
  static constexpr int PAD = LaPad<T>::value;
  static constexpr int NM = D / 32, NV = DF / 32, CT = C / 32;
  static constexpr int KSTRIDE = C + PAD;   // phik row stride (elements)
  static constexpr int QSTRIDE = DP + PAD;  // phiq row stride
  static constexpr size_t phik_bytes = sizeof(T) * DP * KSTRIDE;
  static constexpr size_t phiq_bytes = sizeof(T) * C * QSTRIDE;
  static constexpr size_t slot_bytes(int mode) {
    return (mode && phiq_bytes > phik_bytes) ? phiq_bytes : phik_bytes;
  }
  static constexpr int STAT_FLOATS = 2 * NV * 32 * 4;                     // one buffer: [tile][wave][token]{nf2,max,min,nx2}
  static constexpr size_t stat_bytes = sizeof(float) * 2 * STAT_FLOATS;   // two buffers (sub-unit parity)
  static constexpr size_t sums_bytes = sizeof(float) * 2 * 2 * NV * C;    // [unit parity][half][wave][token]
  static constexpr size_t unit_sums_bytes = sums_bytes / 2;               // one unit's sums
  static constexpr size_t unit_bytes = phik_bytes + unit_sums_bytes;      // a staged K unit as kept in global memory
  static_assert(phik_bytes % 1024 == 0 && unit_sums_bytes % 1024 == 0, "units are copied in 1 KB pieces");
  static constexpr size_t inv_bytes = sizeof(float) * NM * 2 * C;         // [consumer wave][half][token]
  static constexpr size_t z_bytes = sizeof(float) * DP;
  static constexpr size_t keep_bytes = NV * C;                            // [producer wave][token] flags
  static constexpr size_t warm_bytes = 256;                               // landing zone of cache-warming loads
  static constexpr size_t total(int mode) {
    return 2 * slot_bytes(mode) + stat_bytes + sums_bytes + inv_bytes + z_bytes + keep_bytes + warm_bytes;
  }
};

// One work unit of the scan: either the queries of chunk `chunk` (kind 0) or the keys of chunk `chunk`
// that are folded into the state (kind 1).  `valid` false = a chunk that does not exist or is not routed;
// it is produced with every token masked, so it contributes nothing.
struct LaUnit {
  int kind, chunk;
  bool valid;
};

template <int V>
using IC = std::integral_constant<int, V>;

template <typename T, int D, int DF, int C, int MODE>
__device__ __forceinline__ void la_body(const LaArgs& a) {
  typedef Mma<T> M;
  typedef LaSmem<T, D, DF, C> L;
  constexpr int DP = 2 * DF;
  constexpr int NM = D / 32;     // consumer (state) waves: wave w owns value columns [32w, 32w+32)
  constexpr int NV = DF / 32;    // producer (feature-map) waves: wave NM+v owns features [32v, 32v+32) of f
  constexpr int FT = DF / 32;    // feature tiles per half
  constexpr int PT = DP / 32;    // feature tiles of the state
  constexpr int CT = C / 32;     // token tiles per chunk
  constexpr int NSUB = CT / 2;   // sub-units (two token tiles) per unit
  constexpr int NPART = 2 * NSUB;  // barrier-separated parts per unit = token tiles per chunk
  constexpr int SPT = M::STEPS_PER_TILE;
  constexpr int KS = D / M::KK;  // k-steps over the head dimension
  constexpr int VS = C / M::KK;  // k-steps over the tokens of a chunk
  constexpr size_t SLOT = L::slot_bytes(MODE);
  static_assert(NPART == CT, "one token tile per part");

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* stat = reinterpret_cast<float*>(smem + 2 * SLOT);
  float* sums = reinterpret_cast<float*>(smem + 2 * SLOT + L::stat_bytes);
  float* invs = reinterpret_cast<float*>(smem + 2 * SLOT + L::stat_bytes + L::sums_bytes);
  float* zsh = reinterpret_cast<float*>(smem + 2 * SLOT + L::stat_bytes + L::sums_bytes + L::inv_bytes);
  unsigned char* keep = smem + 2 * SLOT + L::stat_bytes + L::sums_bytes + L::inv_bytes + L::z_bytes;
  unsigned char* warm = keep + L::keep_bytes;

  int seg, hq;
  head_major_block(blockIdx.x, a.Hq, hq, seg);
  const int b = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r = lane & 31, g = lane >> 5;
  const bool consumer = wave < NM;
  const int kvh = a.map.kv[hq];
  const int N = seq_tokens(a.seq_len, b, a.N);   // this sequence's tokens (a right-padded batch has shorter ones)
  const int nc_b = (N + C - 1) / C, ncf_b = N / C;
  const int G = a.seg_chunks;

  const T* __restrict__ qbase = static_cast<const T*>(a.q) + (int64_t)b * a.q_sb + (int64_t)hq * a.q_sh;
  const T* __restrict__ kbase = static_cast<const T*>(a.k) + (int64_t)b * a.k_sb + (int64_t)kvh * a.k_sh;
  const T* __restrict__ vfr = static_cast<const T*>(a.vfr) + ((int64_t)b * a.Hkv + kvh) * (int64_t)D * a.Np;
  const T* __restrict__ wqt = static_cast<const T*>(a.wqt) + (int64_t)hq * DF * D;
  const T* __restrict__ wkt = static_cast<const T*>(a.wkt) + (int64_t)hq * DF * D;
  const T* __restrict__ bq = a.bq ? static_cast<const T*>(a.bq) + (int64_t)hq * DF : nullptr;
  const T* __restrict__ bk = a.bk ? static_cast<const T*>(a.bk) + (int64_t)hq * DF : nullptr;
  float* __restrict__ segp = a.seg + (((int64_t)b * a.Hq + hq) * a.nseg + seg) * (int64_t)(DP * (D + 1));
  const int col = 32 * wave + r;  // value column owned by this lane (consumer waves)

  // chunk range and pipeline slots of this workgroup
  const int c_beg = seg * G;
  const int c_end = MODE == 1 ? (c_beg + G < nc_b ? c_beg + G : nc_b) : c_beg + G;
  if (MODE == 1 && c_beg >= nc_b) return;   // the whole segment is padding (uniform over the workgroup)
  // Unit list.  Output pass: Q(c_beg), then for every later chunk c of the segment K(c-2), Q(c): the
  // outputs of chunk c see the state through chunk c-2.  State pass: K(c_beg-1) .. K(c_beg+G-2).
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
      x.kind = 1; x.chunk = c_beg + u - 1; x.valid = x.chunk >= 0 && x.chunk < ncf_b;
    }
    return x;
  };

  // A unit is produced in NSUB sub-units of two token tiles.  Sub-unit m takes two steps: the projection and
  // the per-wave partial statistics in interval m, the exponentials (which need every wave's statistics) in
  // interval m+1; one workgroup barrier ends each interval, so interval m holds the second step of sub-unit
  // m-1 and the first step of sub-unit m, two independent instruction streams that hide each other's
  // latencies.  The consumers handle sub-unit m in interval m+2.  Both roles execute n_units*NSUB + 2 barriers.
  const int M_sub = n_units * NSUB;
  // The state pass leaves every K unit it staged (LDS slot + sums) in global memory; the output pass of the same
  // segment needs exactly those units again (K(c_beg-1) .. K(c_beg+G-3)) and copies them straight into its slots.
  const bool copy_k = MODE == 1 && a.phik != nullptr;
  unsigned char* const phik_seg =
      a.phik == nullptr ? nullptr
                        : a.phik + ((((int64_t)b * a.Hq + hq) * a.nseg + seg) * (int64_t)G) * a.phik_unit;
  auto phik_unit_ptr = [&](const LaUnit& x) { return phik_seg + (int64_t)(x.chunk - (c_beg - 1)) * a.phik_unit; };
  if (!consumer) {
    // ---- producer wave v: features [32v, 32v+32) of f = x W for ALL tokens.  Its 32 rows of W^T stay in
    // registers, so the projection weights are read once per unit instead of once per token tile.  The
    // statistics that span the whole feature dimension (||f||^2, max f, min f per token) are combined across
    // the producer waves through LDS.  The exponentials are written UN-normalised, next to this wave's
    // partial softmax sums; the consumers fold 1/sum into their own operands.
    const int v = wave - NM;
    auto row_ptr = [&](const LaUnit& x, int tt, int r, int g) -> const T* {
      int tok = x.chunk * C + 32 * tt + r;
      tok = tok < N ? tok : N - 1;
      tok = tok < 0 ? 0 : tok;
      return (x.kind == 0 ? qbase + (int64_t)tok * a.q_st : kbase + (int64_t)tok * a.k_st) + g * M::KPL;
    };
    typename M::frag xb[2][KS];    // token rows of the next sub-unit (B operand), refilled right after their use
    typename M::frag w[KS];        // this wave's rows of W^T (A operand) for the current unit kind
    floatx16 f[2];                 // f of the sub-unit between its two steps
    int32_t selv[2];               // Top-lambda list of the next K unit, entries lane and lane + 64
    unsigned char* keepb = keep + v * C;   // this wave's private table: 1 = token goes to the linear state
    auto load_w = [&](int kind, int r, int g) __attribute__((always_inline)) {
      const T* wrow = (kind == 0 ? wqt : wkt) + (int64_t)(32 * v + M::kappa(r)) * D + g * M::KPL;
#pragma unroll
      for (int s = 0; s < KS; ++s) w[s] = M::load(wrow + s * M::KK);
    };
    auto load_x = [&](const LaUnit& x, int tt, int j, int r, int g) __attribute__((always_inline)) {
      const T* xp = row_ptr(x, tt, r, g);
#pragma unroll
      for (int s = 0; s < KS; ++s) xb[j][s] = M::load(xp + s * M::KK);
    };
    auto load_sel = [&](const LaUnit& x, int lane) __attribute__((always_inline)) {
      const int32_t* selc = a.sel + (((int64_t)b * a.Hq + hq) * a.ncf + (x.valid ? x.chunk : 0)) * a.lam;
#pragma unroll
      for (int j = 0; j < 2; ++j) selv[j] = (x.valid && lane + 64 * j < chunk_quota(x.chunk, a.lam, a.rcap)) ? selc[lane + 64 * j] : -1;
    };
    // A staged K unit (slot, then sums) travels global memory -> registers -> LDS in 1 KB pieces dealt over the
    // producer waves: the loads go out in the unit's first interval, when the producers have nothing to project
    // and their registers are free; the LDS writes follow at the top of the next interval, when the consumers
    // have left the slot.  (Direct-to-LDS requests sustain only ~16 bytes per clock and CU and hold up the wave
    // that issues them; ordinary 16-byte loads are four times as fast.)
    constexpr int NPIECE_K = (int)(L::phik_bytes / 1024), NPIECE = NPIECE_K + (int)(L::unit_sums_bytes / 1024);
    constexpr int NST = (NPIECE + NV - 1) / NV;
    // Staging registers: the token-row fragments xb are free exactly while a unit is in flight (the rows of the
    // next Q unit are requested only in the K unit's last interval), so with 16-byte fragments they carry the
    // first 2*KS pieces themselves; the compiler cannot see that the two live ranges never overlap around the
    // loop, and a separate array would be spilled.
    // (With one sub-unit per unit the rows of the next Q unit are requested in the same interval as the staged
    // unit, so the fragments are not free; those units are small enough for an array of their own.)
    constexpr int NXB = (sizeof(typename M::frag) == 16 && NSUB > 1) ? (2 * KS < NST ? 2 * KS : NST) : 0;
    u32x4 stage[NST - NXB > 0 ? NST - NXB : 1];
    auto put_piece = [&](auto J, u32x4 x) __attribute__((always_inline)) {
      constexpr int j = decltype(J)::value;
      if constexpr (j < NXB) xb[j / KS][j % KS] = frag_from_bits<typename M::frag>(x);
      else stage[j - NXB] = x;
    };
    auto get_piece = [&](auto J) __attribute__((always_inline)) -> u32x4 {
      constexpr int j = decltype(J)::value;
      if constexpr (j < NXB) return frag_to_bits<typename M::frag>(xb[j / KS][j % KS]);
      else return stage[j - NXB];
    };
    auto load_k_unit = [&](int u) __attribute__((always_inline)) {
      const int lane = fresh_lane_id();
      const unsigned char* src = phik_unit_ptr(unit_at(u)) + lane * 16;
      static_for<NST>([&](auto J) __attribute__((always_inline)) {
        constexpr int j = decltype(J)::value;
        // (when the pieces divide evenly among the waves there is no test: a branch per load would break the
        // burst into a chain of blocks)
        if (NPIECE % NV == 0 || v + j * NV < NPIECE)
          put_piece(J, *reinterpret_cast<const u32x4*>(src + (v + j * NV) * 1024));
      });
    };
    auto store_k_unit = [&](int u) __attribute__((always_inline)) {
      const int lane = fresh_lane_id();
      unsigned char* slot = smem + (u & 1) * SLOT + lane * 16;
      unsigned char* sums_u = reinterpret_cast<unsigned char*>(sums + (u & 1) * (2 * NV * C)) + lane * 16;
      static_for<NST>([&](auto J) __attribute__((always_inline)) {
        constexpr int j = decltype(J)::value;
        const int i = v + j * NV;
        if constexpr (NPIECE % NV == 0 && NPIECE_K % NV == 0) {
          // piece j of every wave lies on the same side of the slot / sums boundary
          if constexpr (j * NV < NPIECE_K) *reinterpret_cast<u32x4*>(slot + i * 1024) = get_piece(J);
          else *reinterpret_cast<u32x4*>(sums_u + (i - NPIECE_K) * 1024) = get_piece(J);
        } else {
          if (i < NPIECE_K) *reinterpret_cast<u32x4*>(slot + i * 1024) = get_piece(J);
          else if (i < NPIECE) *reinterpret_cast<u32x4*>(sums_u + (i - NPIECE_K) * 1024) = get_piece(J);
        }
      });
    };
    {
      const LaUnit x0 = unit_at(0);
      load_x(x0, 0, 0, r, g);
      load_x(x0, 1, 1, r, g);
      load_w(x0.kind, r, g);
      if (x0.kind == 1) load_sel(x0, lane);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) f[j] = zero16();

#pragma unroll 1
    for (int m = 0; m <= M_sub; ++m) {
      // Lane ids are re-derived per interval: the many lane-dependent LDS and global addresses below are
      // then recomputed where they are used (a few integer operations each) instead of being kept in
      // registers across the whole scan, where they would not fit.
      const int lane = fresh_lane_id(), r = lane & 31, g = lane >> 5;
      const int mp = m - 1, up = mp / NSUB, subp = mp % NSUB;
      // A copied K unit always lands in slot 1 (K units are the odd units).  The consumers read the previous K
      // unit until the end of interval NSUB*(up-1)+1 and this one from interval NSUB*up+2 on, so it is written in
      // interval NSUB*up+1, from registers loaded in interval NSUB*up.
      const bool k_prev = m >= 1 && copy_k && unit_at(up).kind == 1;
      if (k_prev) {
        if (subp == 0) store_k_unit(up);
      } else if (m >= 1) {
        // ---- second step of sub-unit m-1: statistics of all waves -> exponentials -> slot
        const LaUnit x = unit_at(up);
        unsigned char* slot = smem + (up & 1) * SLOT;
        float* sums_u = sums + (up & 1) * (2 * NV * C);
        const float* statp = stat + (mp & 1) * L::STAT_FLOATS;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int tl = 32 * (2 * subp + j) + r;
          float nf2 = 0.f, fmax = -INFINITY, fmin = INFINITY, nx2 = 0.f;
#pragma unroll
          for (int vv = 0; vv < NV; ++vv) {
            const floatx4 st = *reinterpret_cast<const floatx4*>(statp + ((j * NV + vv) * 32 + r) * 4);
            nf2 += st[0];
            fmax = fmaxf(fmax, st[1]);
            fmin = fminf(fmin, st[2]);
            nx2 += st[3];
          }
          nx2 *= NV >= 2 ? 2.f / NV : 1.f;   // NV/2 waves (all of them if NV = 1) recorded ||x||^2 of this tile
          // u = f * ratio with ratio = ||x|| / ||f|| >= 0, so max/min of u are ratio * max/min of f;
          // exp(u - umax) = exp2(f * a1 - fmax * a1),  exp(umin - u) = exp2(fmin * a1 - f * a1).
          // Tokens kept by the softmax branch (and every token of an absent chunk) get -inf offsets, i.e.
          // zero features; their (unused) sums are recorded as 1.
          const float ratio = nf2 > 0.f ? __builtin_amdgcn_sqrtf(nx2 * fast_rcp(nf2)) : 0.f;
          const float a1 = ratio * kLog2e;
          const bool live = x.kind == 0 || keepb[tl] != 0;
          const float bp = live ? -fmax * a1 : -INFINITY, bn = live ? fmin * a1 : -INFINITY;
          floatx16 ep, en;
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            ep[i] = fast_exp2(fmaf(f[j][i], a1, bp));
            en[i] = fast_exp2(fmaf(f[j][i], -a1, bn));
          }
          typename M::frag pf[SPT], nf[SPT];
          float sp = 0.f, sn = 0.f;   // sums of the ROUNDED weights: the stored features then sum to one
#pragma unroll
          for (int s = 0; s < SPT; ++s) {
            pf[s] = M::from_acc(ep, s);
            nf[s] = M::from_acc(en, s);
            sp = M::sum_into(pf[s], sp);
            sn = M::sum_into(nf[s], sn);
          }
          sp = sum32(sp);
          sn = sum32(sn);
          const float srec = g ? sn : sp;   // lane group g records the sum of half g
          sums_u[(g * NV + v) * C + tl] = live ? srec : 1.f;
          if (x.kind == 0) {
            T* qrow = reinterpret_cast<T*>(slot) + tl * L::QSTRIDE + 32 * v + g * M::KPL;
#pragma unroll
            for (int s = 0; s < SPT; ++s) {
              *reinterpret_cast<typename M::frag*>(qrow + s * M::KK) = pf[s];
              *reinterpret_cast<typename M::frag*>(qrow + DF + s * M::KK) = nf[s];
            }
          } else {
            T* kcol = reinterpret_cast<T*>(slot) + (32 * v + g * M::KPL) * L::KSTRIDE + tl;
#pragma unroll
            for (int s = 0; s < SPT; ++s) {
              if constexpr (M::KPL == 1) {
                kcol[(s * M::KK) * L::KSTRIDE] = pf[s];
                kcol[(DF + s * M::KK) * L::KSTRIDE] = nf[s];
              } else {
#pragma unroll
                for (int e = 0; e < M::KPL; ++e) {
                  kcol[(s * M::KK + e) * L::KSTRIDE] = pf[s][e];
                  kcol[(DF + s * M::KK + e) * L::KSTRIDE] = nf[s][e];
                }
              }
            }
          }
        }
      }
      if (m < M_sub && copy_k && unit_at(m / NSUB).kind == 1) {
        const int u = m / NSUB, sub = m % NSUB;
        if (sub == 0) load_k_unit(u);
        if (u + 1 < n_units) {
          // The token rows of the next Q unit's first sub-unit are requested here, in the K unit's last interval,
          // not right after their registers were last used: until now those registers carried the staged unit.
          if (sub == NSUB - 1) {
            load_x(unit_at(u + 1), 0, 0, r, g);
            load_x(unit_at(u + 1), 1, 1, r, g);
          }
          // warm the cache for that unit's rows while there is nothing to project
          if (v < 2) {
            const T* wp = row_ptr(unit_at(u + 1), 2 * sub + v, r, 0) + g * (128 / sizeof(T));
            if (g * (128 / sizeof(T)) < D) async_copy4(wp, lds_address(warm));
          }
        }
      } else if (m < M_sub) {
        // ---- first step of sub-unit m: projection, partial statistics
        const int u = m / NSUB, sub = m % NSUB;
        const LaUnit x = unit_at(u);
        // the next sub-unit that is projected (copied K units are skipped)
        // the next sub-unit whose rows this step requests (after a Q unit's last sub-unit in copy mode: none, the
        // copied K unit in between does it)
        const int subn = sub + 1 < NSUB ? sub + 1 : 0;
        const int un = sub + 1 < NSUB ? u : u + 1;
        const bool more = un < n_units && !(copy_k && un != u);
        const LaUnit xn = unit_at(more ? un : u);
        const T* bias = x.kind == 0 ? bq : bk;
        float* statc = stat + (m & 1) * L::STAT_FLOATS;
        if (x.kind == 1 && sub == 0) {
          // keep table of this K unit from the list requested an interval ago; the wave's own LDS accesses
          // are processed in order, so the later reads need no barrier
          for (int t = lane; t < C; t += 64) keepb[t] = x.valid ? 1 : 0;
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            const unsigned off = (unsigned)(selv[j] - x.chunk * C);
            if (selv[j] >= 0 && off < (unsigned)C) keepb[off] = 0;
          }
        }
        if (more && xn.kind == 1 && subn == 0) load_sel(xn, lane);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          floatx16 acc = zero16();
#pragma unroll
          for (int s = 0; s < KS; ++s) acc = M::mma(w[s], xb[j][s], acc);
          // ||x||^2 of a tile is needed once per token, not once per wave: the waves take turns
          float n2 = 0.f;
          if (NV == 1 || (v & 1) == j) {
#pragma unroll
            for (int s = 0; s < KS; ++s) n2 = M::dot_into(xb[j][s], xb[j][s], n2);
            n2 = sum32(n2);
          }
          // the rows are dead now: request the tile that will use the same registers
          if (more) load_x(xn, 2 * subn + j, j, r, g);
          if (bias != nullptr) {
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] += to_f32(bias[32 * v + M::pos_of_reg(i, g)]);
          }
          float nf2 = 0.f, fmax = -INFINITY, fmin = INFINITY;
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            nf2 = fmaf(acc[i], acc[i], nf2);
            fmax = fmaxf(fmax, acc[i]);
            fmin = fminf(fmin, acc[i]);
          }
          nf2 = sum32(nf2);
          fmax = max32(fmax);
          fmin = min32(fmin);
          if (g == 0) {
            floatx4 st;
            st[0] = nf2; st[1] = fmax; st[2] = fmin; st[3] = n2;
            *reinterpret_cast<floatx4*>(statc + ((j * NV + v) * 32 + r) * 4) = st;
          }
          f[j] = acc;
        }
        if (more && xn.kind != x.kind) load_w(xn.kind, r, g);
        // Warm the cache for the sub-unit after the next one: a 4-byte load per 128-byte line of its rows,
        // landing in a scratch corner of LDS (no registers are held while it is in flight).
        if (!copy_k && m + 2 < M_sub && v < 2) {
          const LaUnit xw = unit_at((m + 2) / NSUB);
          const T* wp = row_ptr(xw, 2 * ((m + 2) % NSUB) + v, r, 0) + g * (128 / sizeof(T));
          if (g * (128 / sizeof(T)) < D)
            async_copy4(wp, lds_address(warm));
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
    for (int fi = threadIdx.x; fi < DP; fi += NM * 64) zsh[fi] = segp[DP * D + fi];
  } else {
#pragma unroll
    for (int ft = 0; ft < PT; ++ft) S[ft] = zero16();
    for (int fi = threadIdx.x; fi < DP; fi += NM * 64) zsh[fi] = 0.f;
  }
  float* invw = invs + wave * (2 * C);   // this wave's private table: 1/softmax-sum per [half][token]

  typedef typename M::frag VFrag[VS];    // V fragments of a K unit (B operand, k = tokens)
  auto load_v = [&](int u, VFrag& vf) __attribute__((always_inline)) {
    const LaUnit x = unit_at(u);
    const int ch = x.valid ? x.chunk : 0;   // an absent chunk meets zero features; any finite V will do
    // from the fragment-ordered copy: the 64 lanes of one load read one contiguous piece (the transposed copy
    // would give 32 rows x 32 bytes per load)
    const T* vrow = vfr + vfr_offset(ch * C, 32 * wave, C, D, M::KK, M::KPL) + (2 * r + g) * M::KPL;
#pragma unroll
    for (int s = 0; s < VS; ++s) vf[s] = M::load(vrow + s * 64 * M::KPL);
  };

  // reciprocal softmax sums of the 64 tokens of sub-unit `sub` of the unit in slot u&1, from the producers'
  // partial sums: lane t handles token 64*sub + t, both halves
  auto make_inv = [&](int u, int sub) __attribute__((always_inline)) {
    const int lane = fresh_lane_id();
    const float* src = sums + (u & 1) * (2 * NV * C) + 64 * sub + lane;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      float sacc = 0.f;
#pragma unroll
      for (int vv = 0; vv < NV; ++vv) sacc += src[(h * NV + vv) * C];
      invw[h * C + 64 * sub + lane] = fast_rcp(sacc);
    }
  };

  // S += phi_k^T V, z += sum phi_k for the unit in slot u&1, over one part (32 tokens) of the chunk.  The
  // softmax normalisers are per token, i.e. per contracted index: they are folded into the V operand, once
  // for each half of the feature dimension.  The phi_k fragments are read from LDS ADEPTH products ahead of
  // their use (the scheduling barriers pin that order), so a product never waits for its own read.
  constexpr int ADEPTH = 8;
  auto consume_k = [&](int u, const VFrag& vf, auto part_c) __attribute__((always_inline)) {
    constexpr int part = decltype(part_c)::value;
    const int lane = fresh_lane_id(), r = lane & 31, g = lane >> 5;   // addresses are rebuilt here, not kept across units
    constexpr int HS = VS / NPART;       // k-steps in this part
    constexpr int NSTEP = HS * PT;       // products in this part
    const T* phik = reinterpret_cast<const T*>(smem + (u & 1) * SLOT);
    const T* abase = phik + M::kappa(r) * L::KSTRIDE + part * 32 + g * M::KPL;
    auto a_at = [&](int idx) { return M::load(abase + (32 * (idx % PT)) * L::KSTRIDE + (idx / PT) * M::KK); };
    const float* ivp = invw + part * 32 + g * M::KPL;
    typename M::frag af[ADEPTH];
#pragma unroll
    for (int i = 0; i < ADEPTH; ++i) af[i] = a_at(i);
    float iv[2][M::KPL];   // reciprocal sums of the next k-step's tokens, read well before they are used
#pragma unroll
    for (int e = 0; e < M::KPL; ++e) {
      iv[0][e] = ivp[e];
      iv[1][e] = ivp[C + e];
    }
    typename M::frag vp = frag_scale<T>(vf[part * HS], iv[0]);
    typename M::frag vn = frag_scale<T>(vf[part * HS], iv[1]);
    typename M::frag vp_next = vp, vn_next = vn;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int idx = 0; idx < NSTEP; ++idx) {
      const int sh = idx / PT, ft = idx % PT;
      if (ft == 0 && sh > 0) {
        vp = vp_next;
        vn = vn_next;
      }
      S[ft] = M::mma(af[idx % ADEPTH], ft < FT ? vp : vn, S[ft]);
      if (idx + ADEPTH < NSTEP) af[idx % ADEPTH] = a_at(idx + ADEPTH);
      if (ft == 0 && sh + 1 < HS) {
#pragma unroll
        for (int e = 0; e < M::KPL; ++e) {
          iv[0][e] = ivp[(sh + 1) * M::KK + e];
          iv[1][e] = ivp[C + (sh + 1) * M::KK + e];
        }
      }
      if (ft == PT - 2 && sh + 1 < HS) vp_next = frag_scale<T>(vf[part * HS + sh + 1], iv[0]);
      if (ft == PT - 1 && sh + 1 < HS) vn_next = frag_scale<T>(vf[part * HS + sh + 1], iv[1]);
      __builtin_amdgcn_sched_barrier(0);
    }
    // row sums of the same LDS rows, PT/NM feature tiles per consumer wave, outside the MFMA loop
    constexpr int ZT = PT / NM;
#pragma unroll
    for (int j = 0; j < ZT; ++j) {
      const int ft = wave * ZT + j;
      const T* zrow = phik + (32 * ft + r) * L::KSTRIDE + part * 32 + g * M::KPL;
      const float* izp = invw + (j * NM >= FT ? 0 : 0) + part * 32 + g * M::KPL;
      float zp = 0.f;
#pragma unroll
      for (int sh = 0; sh < HS; ++sh)
        zp += frag_dot<T>(M::load(zrow + sh * M::KK), izp + (ft >= FT ? C : 0) + sh * M::KK);
      zp = sum32(zp);
      if (g == 0) zsh[32 * ft + r] += zp;
    }
  };

  // N_LA = phi_q S and D_LA = phi_q z for token tile `part` of the chunk in slot u&1.  Each half of the
  // feature dimension gets its own accumulator; the per-token normalisers scale the two partial products
  // when they are combined.
  auto consume_q = [&](int u, auto part_c) __attribute__((always_inline)) {
    constexpr int mt = decltype(part_c)::value;
    const int lane = fresh_lane_id(), r = lane & 31, g = lane >> 5;   // addresses are rebuilt here, not kept across units
    const int col = 32 * wave + r;
    const LaUnit x = unit_at(u);
    const T* phiq = reinterpret_cast<const T*>(smem + (u & 1) * SLOT);
    float* nrow = a.n_la + ((int64_t)b * a.Hq + hq) * (int64_t)a.N * D;
    // The operand-type copies of S are made again for every token tile: kept across tiles (the state does
    // not change between them) they would need as many registers as the state itself.
#pragma unroll
    for (int ft = 0; ft < PT; ++ft) asm volatile("" : "+v"(S[ft]));
    floatx16 op = zero16(), on = zero16();
    const T* arow = phiq + (32 * mt + r) * L::QSTRIDE + g * M::KPL;
    // product idx: feature k-step idx/2 of half idx%2 (first half accumulates into op, second into on)
    constexpr int NQ = 2 * FT * SPT;
    auto a_at = [&](int idx) { return M::load(arow + (idx & 1) * DF + (idx >> 1) * M::KK); };
    auto b_at = [&](int idx) { return M::from_acc(S[(idx & 1) * FT + (idx >> 1) / SPT], (idx >> 1) % SPT); };
    typename M::frag af[ADEPTH];
#pragma unroll
    for (int i = 0; i < ADEPTH; ++i) af[i] = a_at(i);
    typename M::frag bcur = b_at(0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int idx = 0; idx < NQ; ++idx) {
      typename M::frag bnext = bcur;
      if (idx + 1 < NQ) bnext = b_at(idx + 1);
      if (idx & 1) on = M::mma(af[idx % ADEPTH], bcur, on);
      else op = M::mma(af[idx % ADEPTH], bcur, op);
      if (idx + ADEPTH < NQ) af[idx % ADEPTH] = a_at(idx + ADEPTH);
      bcur = bnext;
      __builtin_amdgcn_sched_barrier(0);
    }
    const int tok0 = x.chunk * C + 32 * mt;                   // first token of the tile
    const bool tile_full = tok0 + 32 <= N;                    // uniform: no per-row test in the common case
    float* ntile = nrow + (int64_t)tok0 * D + col;
    if (tile_full && a.g == nullptr) {
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int row0 = 8 * i4 + 4 * g;
        const floatx4 ip = *reinterpret_cast<const floatx4*>(invw + 32 * mt + row0);
        const floatx4 in = *reinterpret_cast<const floatx4*>(invw + C + 32 * mt + row0);
        float* np = ntile + row0 * D;
#pragma unroll
        for (int e = 0; e < 4; ++e) np[e * D] = op[4 * i4 + e] * ip[e] + on[4 * i4 + e] * in[e];
      }
    } else {
#pragma unroll 1
      for (int i4 = 0; i4 < 4; ++i4) {
        const int row0 = 8 * i4 + 4 * g;
        const floatx4 ip = *reinterpret_cast<const floatx4*>(invw + 32 * mt + row0);
        const floatx4 in = *reinterpret_cast<const floatx4*>(invw + C + 32 * mt + row0);
        floatx4 vo, vn4;
        if (i4 == 0) { vo = {op[0], op[1], op[2], op[3]}; vn4 = {on[0], on[1], on[2], on[3]}; }
        else if (i4 == 1) { vo = {op[4], op[5], op[6], op[7]}; vn4 = {on[4], on[5], on[6], on[7]}; }
        else if (i4 == 2) { vo = {op[8], op[9], op[10], op[11]}; vn4 = {on[8], on[9], on[10], on[11]}; }
        else { vo = {op[12], op[13], op[14], op[15]}; vn4 = {on[12], on[13], on[14], on[15]}; }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int tok = tok0 + row0 + e;
          if (tok < N) {
            float val = vo[e] * ip[e] + vn4[e] * in[e];
            if (a.g != nullptr)
              val *= to_f32(static_cast<const T*>(a.g)[(int64_t)b * a.g_sb + (int64_t)tok * a.g_st +
                                                       (int64_t)hq * a.g_sh + col]);
            ntile[(row0 + e) * D] = val;
          }
        }
      }
    }
    // D_LA = phi_q z for this wave's share of the tile's rows.  LPT consecutive lanes split one row's 2*d_f
    // features into slices of 32 (a slice lies in one half, so it has one normaliser); the partial dot
    // products are added across those lanes.
    constexpr int TPW = 32 / NM, LPT = 64 / TPW;
    static_assert(DP / LPT == 32, "32 features per lane");
    {
      const int tl = 32 * mt + wave * TPW + lane / LPT;
      const int sl = lane % LPT;
      const T* qrow = phiq + tl * L::QSTRIDE + 32 * sl;
      const float* zz = zsh + 32 * sl;
      float dla = 0.f;
#pragma unroll
      for (int f0 = 0; f0 < 32; f0 += M::KPL) dla += frag_dot<T>(M::load(qrow + f0), zz + f0);
      dla *= invw[(sl >= LPT / 2 ? C : 0) + tl];
#pragma unroll
      for (int m = 1; m < LPT; m <<= 1) dla += __shfl_xor(dla, m, 64);
      const int tok = x.chunk * C + tl;
      if (sl == 0 && tok < N) a.d_la[((int64_t)b * a.Hq + hq) * a.N + tok] = dla;
    }
  };

  // one sub-unit (two token tiles) per interval
  auto consume_q_sub = [&](int u, auto sub_c) __attribute__((always_inline)) {
    constexpr int sub = decltype(sub_c)::value;
    make_inv(u, sub);
    consume_q(u, IC<2 * sub>{});
    consume_q(u, IC<2 * sub + 1>{});
    lds_barrier();
  };
  auto consume_k_sub = [&](int u, const VFrag& vf, auto sub_c) __attribute__((always_inline)) {
    constexpr int sub = decltype(sub_c)::value;
    make_inv(u, sub);
    consume_k(u, vf, IC<2 * sub>{});
    consume_k(u, vf, IC<2 * sub + 1>{});
    if constexpr (MODE == 0 && sub == NSUB - 1) {
      // the unit is complete in LDS and stays untouched for two more intervals: leave a copy for the output pass
      if (a.phik != nullptr) {
        const int lane = fresh_lane_id();
        Vec16* dst = reinterpret_cast<Vec16*>(phik_unit_ptr(unit_at(u)));
        const Vec16* src = reinterpret_cast<const Vec16*>(smem + (u & 1) * SLOT);
        for (int i = wave * 64 + lane; i < (int)(L::phik_bytes / 16); i += NM * 64) dst[i] = src[i];
        const Vec16* ssrc = reinterpret_cast<const Vec16*>(sums + (u & 1) * (2 * NV * C));
        for (int i = wave * 64 + lane; i < (int)(L::unit_sums_bytes / 16); i += NM * 64)
          dst[L::phik_bytes / 16 + i] = ssrc[i];
      }
    }
    lds_barrier();
  };
  auto consume_q_unit = [&](int u) __attribute__((always_inline)) {
    consume_q_sub(u, IC<0>{});
    if constexpr (NSUB == 2) consume_q_sub(u, IC<1>{});
  };
  auto consume_k_unit = [&](int u, const VFrag& vf) __attribute__((always_inline)) {
    consume_k_sub(u, vf, IC<0>{});
    if constexpr (NSUB == 2) consume_k_sub(u, vf, IC<1>{});
  };

  if (MODE == 1) {
    VFrag vf;
    if (n_units > 1) load_v(1, vf);
    lds_barrier();
    lds_barrier();
    consume_q_unit(0);
#pragma unroll 1
    for (int u = 1; u + 1 < n_units; u += 2) {
      consume_k_unit(u, vf);
      // V of the next K unit is requested BEFORE this unit's N_LA stores: the vector-memory counter retires
      // in order, so a later wait for these loads does not have to wait for the stores as well
      if (u + 2 < n_units) {
        load_v(u + 2, vf);
        // One interval before the producers fetch the next staged K unit, touch each of its 128-byte lines (4-byte
        // direct-to-LDS loads into a scratch corner, no registers held): a CU can only keep a few KB of misses in
        // flight, and 72 KB straight from HBM would take the producers several memory latencies.
        if (copy_k) {
          const int lane = fresh_lane_id();
          const unsigned char* src = phik_unit_ptr(unit_at(u + 2)) + lane * 128;
          for (int i = wave; i * 8192 < (int)L::unit_bytes; i += NM)
            if (i * 8192 + lane * 128 < (int)L::unit_bytes) async_copy4(src + i * 8192, lds_address(warm));
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      consume_q_unit(u + 1);
    }
  } else {
    // two V buffers: the next unit's V is in flight while the current one is contracted
    VFrag va, vb;
    load_v(0, va);
    lds_barrier();
    lds_barrier();
#pragma unroll 1
    for (int u = 0; u < n_units; u += 2) {
      if (u + 1 < n_units) load_v(u + 1, vb);
      __builtin_amdgcn_sched_barrier(0);
      consume_k_unit(u, va);
      if (u + 1 < n_units) {
        if (u + 2 < n_units) load_v(u + 2, va);
        __builtin_amdgcn_sched_barrier(0);
        consume_k_unit(u + 1, vb);
      }
    }
  }

  // ---- write the state
  float* dst = nullptr;
  if (MODE == 0) dst = segp;
  if (MODE == 1 && a.s_final != nullptr && c_end == nc_b)
    dst = a.s_final + ((int64_t)b * a.Hq + hq) * (int64_t)(DP * (D + 1));
  if (dst != nullptr) {
#pragma unroll
    for (int ft = 0; ft < PT; ++ft)
#pragma unroll
      for (int i = 0; i < 16; ++i) dst[(int64_t)(32 * ft + M::pos_of_reg(i, g)) * D + col] = S[ft][i];
    for (int fi = threadIdx.x; fi < DP; fi += NM * 64) dst[DP * D + fi] = zsh[fi];
  }
}

// (the body lives in a __device__ function behind a thin __global__ wrapper)
template <typename T, int D, int DF, int C, int MODE>
__global__ __launch_bounds__((D / 32 + DF / 32) * 64) void la_kernel(LaArgs a) {
  la_body<T, D, DF, C, MODE>(a);
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
  dim3 grid(nblocks * a.Hq, 1, B), block((D / 32 + D / 32) * 64);
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
  // the last segment's sum is not needed by the prefix, but its staged key features are needed by the output pass
  return launch_la_mode<0>(a, dtype, d, B, a.phik != nullptr ? a.nseg : a.nseg - 1, stream);
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

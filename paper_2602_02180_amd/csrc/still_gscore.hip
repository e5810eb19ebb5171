// Local-versus-global consistency study of Sec. 3.1 (the figure that sets window-local Self-Saliency Scores
// against scores taken over the whole causal prefix):
//
//   global_score : Score_t with the window set replaced by {0..t}: a = softmax over all keys j <= t,
//                  n = softmax over j < t (n_t = 0), Score = sum_j a_j ln((a_j + eps) / (n_j + eps)).
//                  The sum needs each a_j inside a logarithm, so it cannot be folded into one online pass:
//                  pass 1 takes the row maximum and the two normalisers, pass 2 recomputes the logits and
//                  accumulates the terms.  Both passes run the logits on the MFMA units (K rows as the A
//                  operand out of LDS, the wave's 32 queries as the B operand out of registers), so a lane
//                  owns one query and 16 of the 32 keys of a tile and every row statistic is a reduction
//                  over its own registers plus one exchange between the two lane groups.
//   topk_overlap : per full chunk, how many tokens the Top-lambda sets under two scores share.
#include "still_kernels.h"

namespace still {

template <typename T, int D>
__global__ __launch_bounds__(256) void global_score_kernel(GScoreArgs a) {
  typedef Mma<T> M;
  constexpr int KS = D / M::KK;
  constexpr int BK = 64;                                   // keys per LDS tile
  constexpr int EPV = 16 / (int)sizeof(T), VPR = D / EPV;  // elements per 16-byte piece, pieces per key row
  constexpr int LD = D + EPV;                              // padded row: operand reads of 32 rows spread over banks
  constexpr int NLD = BK * VPR / 256;                      // pieces per thread and tile
  __shared__ __attribute__((aligned(16))) T Kl[BK * LD];

  const int tile = gridDim.x - 1 - blockIdx.x;             // long rows first
  const int hq = blockIdx.y, b = blockIdx.z;
  const int kvh = a.map.kv[hq];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, g = lane >> 5;
  const int N = a.N;
  const int row0 = tile * 128, q0 = row0 + 32 * wave, t = q0 + r;
  const int tq = t < N ? t : N - 1;                        // lanes past the end repeat the last row, unused
  const T* __restrict__ kbase = static_cast<const T*>(a.k) + (int64_t)b * a.k_sb + (int64_t)kvh * a.k_sh;

  typename M::frag qf[KS];
  {
    const T* qp = static_cast<const T*>(a.q) + (int64_t)b * a.q_sb + (int64_t)tq * a.q_st + (int64_t)hq * a.q_sh +
                  g * M::KPL;
#pragma unroll
    for (int s = 0; s < KS; ++s) qf[s] = M::load(qp + s * M::KK);
  }
  const int last_row = row0 + 127 < N - 1 ? row0 + 127 : N - 1;
  const int n_kt = last_row / BK + 1;                      // key tiles the workgroup walks
  const int wave_last = q0 + 31 < N - 1 ? q0 + 31 : N - 1; // last key any row of this wave sees
  const bool wave_on = q0 < N;
  const float sc2 = a.scale * kLog2e;

  Vec16 stage[NLD];
  auto fetch = [&](int kt) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int idx = tid + 256 * i, row = idx / VPR, piece = idx % VPR;
      int key = kt * BK + row;
      key = key < N ? key : N - 1;                         // masked below
      stage[i] = *reinterpret_cast<const Vec16*>(kbase + (int64_t)key * a.k_st + piece * EPV);
    }
  };
  auto commit = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int idx = tid + 256 * i, row = idx / VPR, piece = idx % VPR;
      *reinterpret_cast<Vec16*>(&Kl[row * LD + piece * EPV]) = stage[i];
    }
  };
  // raw logits of this lane's query against the 16 keys it owns in sub-tile `sub` of the staged tile
  auto products = [&](int sub) __attribute__((always_inline)) {
    floatx16 acc = zero16();
    const T* krow = &Kl[(32 * sub + r) * LD + g * M::KPL];
#pragma unroll
    for (int s = 0; s < KS; ++s) acc = M::mma(M::load(krow + s * M::KK), qf[s], acc);
    return acc;
  };

  // A sub-tile whose 32 keys all precede the wave's first query is FULL: every key is visible to every row and none
  // is a diagonal key, so it needs neither masks nor the with/without-diagonal distinction.  All but the last one
  // to three sub-tiles of a wave are full; their sums are kept apart from the edge sub-tiles':
  //   z_all = z_full + z_edge_all,   z_nd = z_full + z_edge_nd,   e_diag summed on its own   (no cancellation).
  // Pass 2 does not subtract two nearly equal logarithms (over a long prefix a_j and n_j differ by the factor
  // 1 - a_diag with a_diag ~ 1e-4, which fp32 logarithms of a_j + eps and n_j + eps resolve to a few per cent
  // only).  For a key other than the diagonal one, with e_j the exponential under the row maximum,
  //   (a_j + eps) / (n_j + eps) = (z_nd / z_all) (e_j + eps z_all) / (e_j + eps z_nd)
  //                             = (1 - a_diag) (1 + eps e_diag / (e_j + eps z_nd)),
  // both factors of the form 1 + (small, exactly known): K = log(1 - a_diag) once per row (series when a_diag is
  // small) and log(1 + eps e_diag / (e_j + c2)) per key, so that
  //   sum_{j != t} a_j log(...) = (1 / z_all) sum_j e_j [K + log(1 + ced / (e_j + c2))],  c2 = eps z_nd, ced = eps e_diag.
  // The diagonal key's term, a_diag [log(a_diag + eps) - log eps], is taken as it stands.
  float m = -INFINITY, z_full = 0.f, z_all = 0.f, z_nd = 0.f, z_dg = 0.f, total = 0.f, tfull = 0.f;
  float inv_all = 0.f, c2 = 0.f, ced = 0.f, K = 0.f;
  const float log2_eps = fast_log2(a.eps);
  for (int pass = 0; pass < 2; ++pass) {
    fetch(0);
    for (int kt = 0; kt < n_kt; ++kt) {
      __syncthreads();                                     // the previous tile has been read
      commit();
      __syncthreads();
      if (kt + 1 < n_kt) fetch(kt + 1);                    // in flight under the products below
      if (!wave_on || kt * BK > wave_last) continue;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const int k0 = kt * BK + 32 * sub;
        if (k0 > wave_last) continue;                      // uniform over the wave
        const floatx16 acc = products(sub);
        const bool full = k0 + 31 < q0;                    // uniform over the wave
        if (pass == 0) {
          // running maximum and normalisers (raw logits: the positive scale commutes with the maximum)
          float mraw = -INFINITY;
          if (full) {
#pragma unroll
            for (int i = 0; i < 16; ++i) mraw = fmaxf(mraw, acc[i]);
          } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) mraw = fmaxf(mraw, k0 + c_row(i, g) <= tq ? acc[i] : -INFINITY);
          }
          const float m_new = fmaxf(m, mraw * sc2);
          if (m_new != -INFINITY) {                        // else every key so far is masked for this lane
            const float resc = fast_exp2(m - m_new);       // 0 when m = -inf
            z_full *= resc;
            z_all *= resc;
            z_nd *= resc;
            z_dg *= resc;
            if (full) {
              float z4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
              for (int i = 0; i < 16; ++i) z4[i & 3] += fast_exp2(fmaf(acc[i], sc2, -m_new));
              z_full += (z4[0] + z4[1]) + (z4[2] + z4[3]);
            } else {
#pragma unroll
              for (int i = 0; i < 16; ++i) {
                const int key = k0 + c_row(i, g);
                const float e = key <= tq ? fast_exp2(fmaf(acc[i], sc2, -m_new)) : 0.f;
                z_all += e;
                z_nd += key == tq ? 0.f : e;
                z_dg += key == tq ? e : 0.f;
              }
            }
            m = m_new;
          }
        } else if (full) {
          float t4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const float e = fast_exp2(fmaf(acc[i], sc2, -m));   // m is the row maximum now
            t4[i & 3] = fmaf(e, fast_log2(fmaf(ced, fast_rcp(e + c2), 1.0f)), t4[i & 3]);
          }
          tfull += (t4[0] + t4[1]) + (t4[2] + t4[3]);
        } else {
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const bool vis = k0 + c_row(i, g) <= tq;
            const bool diag = k0 + c_row(i, g) == tq;
            const float e = vis ? fast_exp2(fmaf(acc[i], sc2, -m)) : 0.f;
            const float ad = e * inv_all;
            const float lg = diag ? fast_log2(ad + a.eps) - log2_eps
                                  : K + fast_log2(fmaf(ced, fast_rcp(e + c2), 1.0f));
            total = fmaf(ad, vis ? lg : 0.f, total);       // (an invisible key has e = 0, and c2 may be 0 too)
          }
        }
      }
    }
    if (pass == 0) {
      // combine the two lane groups of each query: common maximum, then the normalisers
      const float m_row = max32(m);
      const float w = m == -INFINITY ? 0.f : fast_exp2(m - m_row);
      z_full = sum32(z_full * w);
      z_all = z_full + sum32(z_all * w);
      z_nd = z_full + sum32(z_nd * w);
      z_dg = sum32(z_dg * w);
      m = m_row;
      inv_all = 1.0f / z_all;
      c2 = a.eps * z_nd;
      ced = a.eps * z_dg;
      // K = log2(1 - a_diag); a row whose only key is the diagonal one has no other term (K unused, kept finite)
      const float y = z_dg * inv_all;
      K = z_nd > 0.f ? (y < 0.01f ? -y * (1.0f + y * (0.5f + y * (1.0f / 3.0f))) * kLog2e : fast_log2(z_nd * inv_all)) : 0.f;
    }
  }
  // the full sub-tiles' share (a row without other keys has none: z_full = 0)
  total = sum32(total + inv_all * tfull) + inv_all * K * z_full;
  if (g == 0 && t < N) a.score[((int64_t)b * a.Hq + hq) * N + t] = total * kLn2;
}

// One workgroup of C threads per (full chunk, query head, batch): ranks the chunk under both scores (ties to the
// lower index, as the selection does) and counts the tokens that are among the lam best of both.
__global__ __launch_bounds__(128) void topk_overlap_kernel(const float* __restrict__ sa, const float* __restrict__ sb,
                                                           int32_t* __restrict__ overlap, int N, int C, int lam,
                                                           int Hq, int ncf) {
  __shared__ float s_a[128], s_b[128];
  __shared__ int s_cnt[2];
  const int c = blockIdx.x, hq = blockIdx.y, b = blockIdx.z, i = threadIdx.x;
  const int64_t base = ((int64_t)b * Hq + hq) * N + (int64_t)c * C;
  const float va = sa[base + i], vb = sb[base + i];
  s_a[i] = va;
  s_b[i] = vb;
  __syncthreads();
  int ra = 0, rb = 0;
  for (int j = 0; j < C; ++j) {
    const float xa = s_a[j], xb = s_b[j];
    ra += (xa > va || (xa == va && j < i)) ? 1 : 0;
    rb += (xb > vb || (xb == vb && j < i)) ? 1 : 0;
  }
  const unsigned long long both = __ballot(ra < lam && rb < lam);
  if ((i & 63) == 0) s_cnt[i >> 6] = __popcll(both);
  __syncthreads();
  if (i == 0) overlap[((int64_t)b * Hq + hq) * ncf + c] = s_cnt[0] + (C > 64 ? s_cnt[1] : 0);
}

hipError_t launch_global_score(const GScoreArgs& a, int dtype, int d, int B, hipStream_t stream) {
  dim3 grid((a.N + 127) / 128, a.Hq, B), block(256);
  if (dtype == 1) {
    if (d == 64) hipLaunchKernelGGL((global_score_kernel<bf16, 64>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((global_score_kernel<bf16, 128>), grid, block, 0, stream, a);
  } else {
    if (d == 64) hipLaunchKernelGGL((global_score_kernel<float, 64>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((global_score_kernel<float, 128>), grid, block, 0, stream, a);
  }
  return hipGetLastError();
}

hipError_t launch_topk_overlap(const float* sa, const float* sb, int32_t* overlap, int N, int C, int lam, int Hq,
                               int B, hipStream_t stream) {
  const int ncf = N / C;
  if (ncf <= 0) return hipSuccess;
  hipLaunchKernelGGL(topk_overlap_kernel, dim3(ncf, Hq, B), dim3(C), 0, stream, sa, sb, overlap, N, C, lam, Hq, ncf);
  return hipGetLastError();
}

}  // namespace still

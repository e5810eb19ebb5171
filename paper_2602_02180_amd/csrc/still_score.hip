// Self-Saliency Score over the causal window and Top-lambda selection per completed chunk.
//
// Paper: Sec. 3.1 (window set, the two window softmaxes a_diag / a_nodiag, the score equation)
// and Sec. 3.3 (delayed selection: Top-lambda of a chunk's scores).  Algorithm 1 computes the same
// logits chunk by chunk for the special case W = C; here the window length W is free.
//
// One workgroup handles one chunk of one (batch, query head): each wave owns 32 consecutive
// query tokens and evaluates the logit band  key in [t-W+1, t]  as NT tiles of 32 keys with MFMA
// (K rows as the A operand, the wave's 32 queries as the B operand, both read straight from
// global memory: every byte of the rows is consumed across the k-steps, so the L1/L2 lines are
// fetched once).  In C layout every lane then holds the logits of ONE query, so the two softmaxes
// and the score reduce inside a lane plus one exchange with the other lane group.
// Scores go to an LDS array; each thread ranks one token by counting (score higher, or equal with a
// lower index) and the selected tokens are written in ascending order.
#include "still_kernels.h"

namespace still {

template <typename T, int D, int NT>
__global__ __launch_bounds__(256) void score_select_kernel(ScoreArgs a) {
  typedef Mma<T> M;
  constexpr int KS = D / M::KK;
  const T* __restrict__ q = static_cast<const T*>(a.q);
  const T* __restrict__ k = static_cast<const T*>(a.k);
  int c, hq;
  head_major_block(blockIdx.x, a.Hq, hq, c);
  const int b = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 31, g = lane >> 5;
  const int N = a.N, C = a.C, W = a.W;
  const int kvh = a.map.kv[hq];
  const int t0 = c * C + 32 * wave;
  const int t = t0 + r;

  __shared__ float s_score[128];
  __shared__ unsigned char s_flag[128];

  // queries of this wave as B operand
  typename M::frag qf[KS];
  {
    const int tq = t < N ? t : N - 1;
    const T* qp = q + (int64_t)b * a.q_sb + (int64_t)tq * a.q_st + (int64_t)hq * a.q_sh + g * M::KPL;
#pragma unroll
    for (int s = 0; s < KS; ++s) qf[s] = M::load(qp + s * M::KK);
  }

  floatx16 acc[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    acc[j] = zero16();
    const int kb = t0 - 32 * (NT - 1 - j);
    if (kb + 31 < 0 || kb >= N) continue;  // wave-uniform: tile entirely outside the sequence
    int key = kb + M::kappa(r);
    key = key < 0 ? 0 : (key >= N ? N - 1 : key);
    const T* kp = k + (int64_t)b * a.k_sb + (int64_t)key * a.k_st + (int64_t)kvh * a.k_sh + g * M::KPL;
#pragma unroll
    for (int s = 0; s < KS; ++s) acc[j] = M::mma(M::load(kp + s * M::KK), qf[s], acc[j]);
  }

  // window softmaxes for query t (this lane and lane^32 share the query)
  const int lo = (t - W + 1) > 0 ? (t - W + 1) : 0;
  const float sc2 = a.scale * kLog2e;
  float m2 = -INFINITY;
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int kb = t0 - 32 * (NT - 1 - j);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int key = kb + M::pos_of_reg(i, g);
      const bool valid = key >= lo && key <= t;
      const float x = valid ? acc[j][i] * sc2 : -INFINITY;
      acc[j][i] = x;
      m2 = fmaxf(m2, x);
    }
  }
  m2 = fmaxf(m2, xor32(m2));
  float d_all = 0.f, d_no = 0.f;
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int kb = t0 - 32 * (NT - 1 - j);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int key = kb + M::pos_of_reg(i, g);
      const float e = fast_exp2(acc[j][i] - m2);  // masked entries: exp2(-inf) = 0
      acc[j][i] = e;
      d_all += e;
      d_no += (key == t) ? 0.f : e;
    }
  }
  d_all += xor32(d_all);
  d_no += xor32(d_no);
  const float inv_all = 1.0f / d_all;
  const float inv_no = d_no > 0.f ? 1.0f / d_no : 0.f;
  float score = 0.f;
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int kb = t0 - 32 * (NT - 1 - j);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int key = kb + M::pos_of_reg(i, g);
      const bool valid = key >= lo && key <= t;
      const float e = acc[j][i];
      const float ad = e * inv_all;
      const float an = (key == t) ? 0.f : e * inv_no;
      const float term = ad * (fast_log2(ad + a.eps) - fast_log2(an + a.eps));
      score += valid ? term : 0.f;
    }
  }
  score *= kLn2;
  score += xor32(score);

  if (g == 0) {
    s_score[32 * wave + r] = score;
    if (t < N) a.score[((int64_t)b * a.Hq + hq) * N + t] = score;
  }

  // Top-lambda of a full chunk, ties to the lower index, written ascending.
  if (a.sel != nullptr && c < a.ncf) {
    __syncthreads();
    const int i = threadIdx.x;
    bool chosen = false;
    if (i < C) {
      const float si = s_score[i];
      int rank = 0;
      for (int j = 0; j < C; ++j) {
        const float sj = s_score[j];
        rank += (sj > si || (sj == si && j < i)) ? 1 : 0;
      }
      chosen = rank < a.lam;
      s_flag[i] = chosen ? 1 : 0;
    }
    __syncthreads();
    if (chosen) {
      int pos = 0;
      for (int j = 0; j < i; ++j) pos += s_flag[j];
      if (pos < a.lam)  // NaN scores can flag more than lam tokens; never write past the chunk's slots
        a.sel[(((int64_t)b * a.Hq + hq) * a.ncf + c) * a.lam + pos] = c * C + i;
    }
  }
}

template <typename T, int D>
static hipError_t launch_score_t(const ScoreArgs& a, int B, int nc, hipStream_t stream) {
  dim3 grid(nc * a.Hq, 1, B), block((a.C / 32) * 64);
  if (a.W <= 65)
    hipLaunchKernelGGL((score_select_kernel<T, D, 3>), grid, block, 0, stream, a);
  else
    hipLaunchKernelGGL((score_select_kernel<T, D, 5>), grid, block, 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_score(const ScoreArgs& a, int dtype, int d, int B, int nc, hipStream_t stream) {
  if (dtype == 1) {
    return d == 64 ? launch_score_t<bf16, 64>(a, B, nc, stream) : launch_score_t<bf16, 128>(a, B, nc, stream);
  }
  return d == 64 ? launch_score_t<float, 64>(a, B, nc, stream) : launch_score_t<float, 128>(a, B, nc, stream);
}

}  // namespace still

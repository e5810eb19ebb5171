// Self-Saliency Score over the causal window and Top-lambda selection per completed chunk.
//
// Paper: Sec. 3.1 (window set, the two window softmaxes a_diag / a_nodiag, the score equation)
// and Sec. 3.3 (delayed selection: Top-lambda of a chunk's scores).  Algorithm 1 computes the same
// logits chunk by chunk for the special case W = C; here the window length W is free.
//
// One workgroup handles one chunk of one (batch, query head): each wave owns 32 consecutive
// query tokens and evaluates the logit band  key in [t-W+1, t]  as NT tiles of 32 keys with MFMA
// (K rows as the A operand, staged through LDS for the whole workgroup; the wave's 32 queries as
// the B operand, from registers).  In C layout every lane then holds the logits of ONE query, so
// the two softmaxes and the score reduce inside a lane plus one exchange with the other lane group.
// Scores go to an LDS array; each thread ranks one token by counting (score higher, or equal with a
// lower index) and the selected tokens are written in ascending order.
#include "still_kernels.h"

namespace still {

template <typename T, int D, int NT>
__global__ __launch_bounds__(256, NT > 5 ? 2 : 3) void score_select_kernel(ScoreArgs a) {
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

  __shared__ __attribute__((aligned(16))) float s_score[128];
  __shared__ int s_rank[256];
  __shared__ unsigned long long s_ball[4];

  // queries of this wave as B operand
  typename M::frag qf[KS];
  {
    const int tq = t < N ? t : N - 1;
    const T* qp = q + (int64_t)b * a.q_sb + (int64_t)tq * a.q_st + (int64_t)hq * a.q_sh + g * M::KPL;
#pragma unroll
    for (int s = 0; s < KS; ++s) qf[s] = M::load(qp + s * M::KK);
  }

  // Logit band.  The waves of the workgroup need overlapping key ranges (wave w: band tiles w .. w+NT-1 of the
  // NB = NT-1 + C/32 tiles of 32 keys that end with the chunk), and as an MFMA operand a K row is consumed 16
  // bytes per lane and instruction, i.e. 32 rows x 32 bytes per load: fetched straight from global memory the
  // same lines are requested over and over.  The band therefore passes through LDS, PT tiles at a time, with
  // direct-to-LDS copies of whole 1 KB pieces (the 16-byte column index is XOR-ed with the row so that the
  // operand reads meet no bank conflicts); every wave then takes the tiles of the pass that belong to its band.
  constexpr int EPV = 16 / (int)sizeof(T), KVR = D / EPV;                // elements / vectors per K row
  constexpr int PT_MAX = 32768 / (32 * D * (int)sizeof(T));              // tiles in 32 KB
  const int NW = C / 32, NB = NT - 1 + NW;
  constexpr int PT = PT_MAX < 8 ? PT_MAX : 8;
  __shared__ __attribute__((aligned(16))) unsigned char s_kraw[PT * 32 * D * sizeof(T)];
  T* s_k = reinterpret_cast<T*>(s_kraw);
  auto swz = [](int row) { return KVR == 8 ? ((row >> 1) & 7) : (row & 15); };
  const T* kbase = k + (int64_t)b * a.k_sb + (int64_t)kvh * a.k_sh;
  const int band0 = c * C - 32 * (NT - 1);                               // first key of the band (may be < 0)
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);

  floatx16 acc[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) acc[j] = zero16();
  for (int p0 = 0; p0 < NB; p0 += PT) {
    const int npt = NB - p0 < PT ? NB - p0 : PT;                         // tiles in this pass
    if (p0 > 0) lds_barrier();                                           // the previous pass has been read
    // piece i (1 KB) of the pass: lane L lands at 1024 i + 16 L = LDS (row, slot) and fetches the global column
    // slot ^ swz(row) of the key that row holds; keys outside the sequence re-read an end token (masked later)
    for (int i = wave_s; i < npt * 32 * KVR / 64; i += NW) {
      const int v = i * 64 + lane;
      const int row = v / KVR, slot = v % KVR;
      int key = band0 + 32 * p0 + row;
      key = key < 0 ? 0 : (key >= N ? N - 1 : key);
      async_copy16(kbase + (int64_t)key * a.k_st + ((slot ^ swz(row)) * EPV), lds_address(s_kraw + i * 1024));
    }
    wait_async_copies();
    lds_barrier();
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int bt = wave_s + j - p0;                                    // tile index inside the pass
      const int kb = t0 - 32 * (NT - 1 - j);
      if (bt < 0 || bt >= npt || kb + 31 < 0 || kb >= N) continue;       // wave-uniform
      const int row = 32 * bt + M::kappa(r);
      const T* krow = s_k + row * D;
      const int sw = swz(row);
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        const int e = s * M::KK + g * M::KPL;
        acc[j] = M::mma(M::load(krow + (((e / EPV) ^ sw) * EPV) + e % EPV), qf[s], acc[j]);
      }
    }
  }

  // window softmaxes for query t (this lane and lane^32 share the query).
  // The band is 32 keys longer than any window (W <= 32 (NT-1)): a slot of the oldest tile (position p) is inside
  // query r's window only if p > r, the same slot of the newest tile only if p <= r (causal limit), so at most one
  // of the two is ever alive.  They are merged into one value per slot, and the exponentials and logarithms run
  // over NT-1 tiles.  The merged tile is the only one that can hold the diagonal key (slot p == r).  Of the
  // others only those at the window start of the wave's first chunk rows need a mask; which, is wave-uniform.
  const int lo = (t - W + 1) > 0 ? (t - W + 1) : 0;
  const int lo_max = (t0 + 32 - W) > 0 ? (t0 + 32 - W) : 0;   // window start of the wave's last query
  const float sc2 = a.scale * kLog2e;
  {
    const int kb_old = t0 - 32 * (NT - 1);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int p = M::pos_of_reg(i, g);
      const int key_old = kb_old + p, key_new = t0 + p;
      const float v_old = (key_old >= lo) ? acc[0][i] : -INFINITY;         // key_old <= t always
      acc[NT - 1][i] = (key_new <= t) ? (key_new >= lo ? acc[NT - 1][i] : -INFINITY) : v_old;
    }
  }
  bool full[NT];
#pragma unroll
  for (int j = 1; j < NT; ++j) {
    const int kb = t0 - 32 * (NT - 1 - j);
    full[j] = j == NT - 1 || (kb >= lo_max && kb >= 0);
  }
  // pass 1: masked logits (raw, the positive scale commutes with the maximum) and their maximum
  float mraw = -INFINITY;
#pragma unroll
  for (int j = 1; j < NT; ++j) {
    const int kb = t0 - 32 * (NT - 1 - j);
    if (!full[j]) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = kb + M::pos_of_reg(i, g);
        acc[j][i] = (key >= lo && key <= t) ? acc[j][i] : -INFINITY;
      }
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) mraw = fmaxf(mraw, acc[j][i]);
  }
  mraw = max32(mraw);
  // pass 2: e = exp(scale * (x - max)); masked entries give exp2(-inf) = 0.  The sums without the diagonal
  // differ from the full sums only in the merged tile.
  const float moff = -mraw * sc2;
  float d_old = 0.f, d_new = 0.f, d_new_no = 0.f;
#pragma unroll
  for (int j = 1; j < NT; ++j) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float e = fast_exp2(fmaf(acc[j][i], sc2, moff));
      acc[j][i] = e;
      if (j < NT - 1) {
        d_old += e;
      } else {
        d_new += e;
        d_new_no += (M::pos_of_reg(i, g) == r) ? 0.f : e;   // slot p == r of the merged tile is the query itself
      }
    }
  }
  float d_all = d_old + d_new, d_no = d_old + d_new_no;
  d_all = sum32(d_all);
  d_no = sum32(d_no);
  const float inv_all = 1.0f / d_all;
  const float inv_no = d_no > 0.f ? 1.0f / d_no : 0.f;
  // pass 3: sum of a_diag * (log(a_diag + eps) - log(a_nodiag + eps)).  A masked entry has a_diag = a_nodiag = 0:
  // its term is 0 * (log eps - log eps) = 0 (eps > 0 is checked on the host).
  float score = 0.f;
#pragma unroll
  for (int j = 1; j < NT; ++j) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float e = acc[j][i];
      const float ad = e * inv_all;
      float an = e * inv_no;
      if (j == NT - 1) an = (M::pos_of_reg(i, g) == r) ? 0.f : an;
      score = fmaf(ad, fast_log2(ad + a.eps) - fast_log2(an + a.eps), score);
    }
  }
  score *= kLn2;
  score = sum32(score);

  if (g == 0) {
    s_score[32 * wave + r] = score;
    if (t < N) a.score[((int64_t)b * a.Hq + hq) * N + t] = score;
  }

  // Top-lambda of a full chunk, ties to the lower index, written ascending.  Token i's rank = number of
  // tokens that beat it; the count is split between threads i and i + C (half of the opponents each).  The
  // output position of a chosen token = number of chosen tokens before it, from wave ballots.
  if (a.sel != nullptr && c < a.ncf) {
    __syncthreads();
    const int i = threadIdx.x % C, half = threadIdx.x / C;   // blockDim = 2 C
    const float si = s_score[i];
    int part = 0;
    const int j0 = half * (C / 2);
#pragma unroll 4
    for (int j = j0; j < j0 + C / 2; j += 4) {   // four opponents per LDS read (every lane reads the same address)
      const floatx4 sj = *reinterpret_cast<const floatx4*>(&s_score[j]);
#pragma unroll
      for (int e = 0; e < 4; ++e) part += (sj[e] > si || (sj[e] == si && j + e < i)) ? 1 : 0;
    }
    s_rank[threadIdx.x] = part;
    __syncthreads();
    bool chosen = false;
    const int quota = chunk_quota(c, a.lam, a.rcap);
    int32_t* selc = a.sel + (((int64_t)b * a.Hq + hq) * a.ncf + c) * a.lam;
    if ((int)threadIdx.x < C) chosen = s_rank[threadIdx.x] + s_rank[threadIdx.x + C] < quota;
    if ((int)threadIdx.x >= quota && (int)threadIdx.x < a.lam) selc[threadIdx.x] = -1;   // slots the budget leaves empty
    const unsigned long long bal = __ballot(chosen);
    if (lane == 0) s_ball[wave] = bal;
    __syncthreads();
    if (chosen) {
      int pos = __popcll(bal & ((1ull << lane) - 1ull));
      for (int w = 0; w < wave; ++w) pos += __popcll(s_ball[w]);
      if (pos < quota)  // NaN scores can flag more tokens than the quota; never write past the chunk's slots
        selc[pos] = c * C + threadIdx.x;
    }
  }
}

// Group-shared Top-lambda, a variant (the paper ranks per head and does not mention grouped-query attention): the
// query heads that read one kv head rank a chunk by the sum of their Self-Saliency Scores, added in ascending head
// order, and all receive the same list, so the retained keys and values could be kept once per kv head.
// One workgroup of C threads per (full chunk, kv head, batch); reads the scores the score kernel has written.
__global__ __launch_bounds__(128) void group_select_kernel(ScoreArgs a) {
  __shared__ float s_sum[128];
  __shared__ unsigned long long s_ball[2];
  const int c = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int C = a.C, i = threadIdx.x, lane = i & 63, wave = i >> 6;
  float s = 0.f;
  for (int h = 0; h < a.Hq; ++h)
    if (a.map.kv[h] == kvh) s += a.score[((int64_t)b * a.Hq + h) * a.N + c * C + i];
  s_sum[i] = s;
  __syncthreads();
  int rank = 0;
#pragma unroll 4
  for (int j = 0; j < C; ++j) {
    const float sj = s_sum[j];
    rank += (sj > s || (sj == s && j < i)) ? 1 : 0;
  }
  const int quota = chunk_quota(c, a.lam, a.rcap);
  const bool chosen = rank < quota;
  const unsigned long long bal = __ballot(chosen);
  if (lane == 0) s_ball[wave] = bal;
  __syncthreads();
  int pos = __popcll(bal & ((1ull << lane) - 1ull));
  if (wave == 1) pos += __popcll(s_ball[0]);
  for (int h = 0; h < a.Hq; ++h) {
    if (a.map.kv[h] != kvh) continue;
    int32_t* selc = a.sel + (((int64_t)b * a.Hq + h) * a.ncf + c) * a.lam;
    if (chosen && pos < quota) selc[pos] = c * C + i;
    if (i >= quota && i < a.lam) selc[i] = -1;
  }
}

hipError_t launch_group_select(const ScoreArgs& a, int B, int Hkv, hipStream_t stream) {
  if (a.ncf <= 0 || a.sel == nullptr) return hipSuccess;
  hipLaunchKernelGGL(group_select_kernel, dim3(a.ncf, Hkv, B), dim3(a.C), 0, stream, a);
  return hipGetLastError();
}

template <typename T, int D>
static hipError_t launch_score_t(const ScoreArgs& a, int B, int nc, hipStream_t stream) {
  dim3 grid(nc * a.Hq, 1, B), block((a.C / 32) * 64);
  if (a.W <= 64)   // the band must be at least 32 keys longer than the window less one: W <= 32 (NT - 1)
    hipLaunchKernelGGL((score_select_kernel<T, D, 3>), grid, block, 0, stream, a);
  else if (a.W <= 128)
    hipLaunchKernelGGL((score_select_kernel<T, D, 5>), grid, block, 0, stream, a);
  else             // up to 256 keys: nine band tiles (two workgroups per CU: 144 accumulator registers)
    hipLaunchKernelGGL((score_select_kernel<T, D, 9>), grid, block, 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_score(const ScoreArgs& a, int dtype, int d, int B, int nc, hipStream_t stream) {
  if (dtype == 1) {
    return d == 64 ? launch_score_t<bf16, 64>(a, B, nc, stream) : launch_score_t<bf16, 128>(a, B, nc, stream);
  }
  return d == 64 ? launch_score_t<float, 64>(a, B, nc, stream) : launch_score_t<float, 128>(a, B, nc, stream);
}

}  // namespace still

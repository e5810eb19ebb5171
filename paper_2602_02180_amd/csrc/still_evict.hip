// Budget policy "evict the lowest score" for the prefill (a variant of this library: the long-context settings of
// Sec. 4 cap the number of cached tokens without stating a policy; the paper's own operator has no budget).
//
// Every routed chunk offers its lambda highest scores (the delayed selection of Sec. 3.3, unchanged).  After routing
// step s the retained set is the union of the previous set and chunk s's offers, cut back to M members by removing
// the lowest score first (between equal scores the higher token index first).  A removed token enters the linear
// state at step s.  The rows of chunk c use the set retained after step c-2 (the two-chunk delay of the cache-routing
// equation).
//
// The retained set therefore changes from chunk to chunk, while the other kernels want something fixed:
//   * the sparse-attention kernel walks ALL offers in routing order (the gathered rows, as without a budget) under a
//     bit mask per (row chunk, tile of 64 offers): evict_plan_kernel writes `alive`;
//   * the state scan adds, at chunk s, the chunk's own unselected tokens, and a retained token that leaves at step s
//     takes the place of an offer of chunk s that stays (a kept token contributes nothing, so its position is free;
//     there are never more leavers than stayers): evict_plan_kernel writes, for every token position, the token
//     whose key and value it carries (`src`, -1 = nothing), vfr_gather_kernel builds the operand-order copy of v
//     through it, and the scan's producers read their key rows through it;
//   * a decode state exported by the prefill gets the set retained after the last routed step (`fin_*`).
#include "still_kernels.h"

namespace still {

// ascending key order = ascending score, then descending token index (the first to leave has the smallest key)
__device__ __forceinline__ unsigned long long evict_key(float sc, int tok) {
  uint32_t u = __float_as_uint(sc);
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return ((unsigned long long)u << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)tok);
}
__device__ __forceinline__ int evict_key_token(unsigned long long key) {
  return (int)(0xFFFFFFFFu - (uint32_t)(key & 0xFFFFFFFFull));
}

// One workgroup per (sequence, query head), walking the routing steps in order.  The retained set is
// kept SORTED by key (ascending: the first entries are the first to leave) in one of two LDS buffers.  Per step:
//   the lam offers are sorted among themselves (rank counting);
//   the `over` smallest keys of the union are found by merging the two sorted heads (one thread, at most lam picks):
//   they are the first e_old retained entries and the first e_new offers;
//   the survivors of both lists are merged into the other buffer, every entry computing its own place (its index
//   in its list plus a binary search in the other);
//   the offers that stay lend their positions to the retained tokens that leave (src), the mask row of chunk s+2 is
//   built from the entries' offer indices.
// The barriers inside the loop order LDS traffic only (the kernel never reads back what it writes to global memory),
// so the offers of the next step, fetched a step ahead, and the stores of this step stay in flight across them.
// LDS (dynamic): 2 x keys[M + lam] (8 bytes), 2 x slot[M + lam] (4 bytes), the words of one mask row.
// (threads per workgroup: with one entry per thread the dependent LDS reads of a step overlap)
constexpr int kPlanThreads = 1024;
__global__ __launch_bounds__(kPlanThreads) void evict_plan_kernel(EvictPlanArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char dsm[];
  const int hq = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int64_t unit = (int64_t)b * a.Hq + hq;
  const int N = seq_tokens(a.seq_len, b, a.N);
  const int C = a.C, lam = a.lam, M = a.M, cap = M + lam;
  const int ncf = N / C, nc = (N + C - 1) / C;
  const int n_exp = nc >= 2 ? nc - 2 : 0;                 // routing steps a decode hand-over has seen
  unsigned long long* kbuf[2] = {reinterpret_cast<unsigned long long*>(dsm),
                                 reinterpret_cast<unsigned long long*>(dsm) + cap};
  int* sbuf[2] = {reinterpret_cast<int*>(dsm + (size_t)cap * 16), reinterpret_cast<int*>(dsm + (size_t)cap * 16) + cap};
  uint32_t* words = reinterpret_cast<uint32_t*>(dsm + (size_t)cap * 24);   // 2 * AW 32-bit words
  __shared__ unsigned long long s_new[128], s_raw[128];
  __shared__ int s_newslot[128], s_eold;

  const float* score = a.score + unit * a.N;
  const int32_t* sel = a.sel + unit * (int64_t)a.ncf_all * lam;
  int32_t* src = a.src + unit * a.N;
  uint32_t* alive = reinterpret_cast<uint32_t*>(a.alive) + unit * (int64_t)a.nc_all * (2 * a.AW);

  for (int t = tid; t < a.N; t += kPlanThreads) src[t] = t;        // every position carries its own token unless told otherwise
  for (int i = tid; i < 2 * (2 * a.AW); i += kPlanThreads)         // rows of chunks 0 and 1 see no retained token
    if (i / (2 * a.AW) < a.nc_all) alive[i] = 0u;
  if (tid == 0) a.fin_n[unit] = 0;
  int n = 0, cur = 0;                                     // retained entries (in kbuf[cur]); uniform over the workgroup
  // the offers of the next step are fetched a step ahead (two dependent global loads: index, then score)
  unsigned long long next_key = 0ull;
  auto fetch_offer = [&](int s) {
    if (tid < lam && s < ncf) {
      const int tok = sel[(int64_t)s * lam + tid];
      next_key = evict_key(score[tok], tok);
    }
  };
  fetch_offer(0);
  __syncthreads();

  for (int s = 0; s < ncf; ++s) {
    const unsigned long long* kold = kbuf[cur];
    const int* sold = sbuf[cur];
    unsigned long long* knew = kbuf[cur ^ 1];
    int* snew = sbuf[cur ^ 1];
    // the chunk's offers, sorted among themselves
    if (tid < lam) s_raw[tid] = next_key;
    if (tid == 0) s_eold = 0;
    lds_barrier();                        // (also: every thread has finished the previous step's mask row)
    for (int i = tid; i < 2 * a.AW; i += kPlanThreads) words[i] = 0u;
    fetch_offer(s + 1);
    if (tid < lam) {
      const unsigned long long mine = s_raw[tid];
      int rank = 0;
      for (int j = 0; j < lam; ++j) rank += s_raw[j] < mine ? 1 : 0;   // keys are distinct (distinct tokens)
      s_new[rank] = mine;
      s_newslot[rank] = s * lam + tid;
    }
    lds_barrier();
    // The `over` smallest keys of the union are among the first `over` entries of either sorted list.  Retained
    // entry i (< over) leaves iff fewer than `over` keys of the union are smaller: its own index plus the offers
    // below it.  The leavers of a sorted list are a prefix, so counting them gives e_old; the rest are offers.
    const int over = n + lam > M ? n + lam - M : 0;
    if (tid < over && tid < n) {
      const unsigned long long key = kold[tid];
      int below = tid;
      const int jmax = over < lam ? over : lam;
      for (int j = 0; j < jmax; ++j) below += s_new[j] < key ? 1 : 0;
      if (below < over) atomicAdd(&s_eold, 1);
    }
    lds_barrier();
    const int e_old = s_eold, e_new = over - e_old;
    const int n_old_s = n - e_old, n_new_s = lam - e_new;   // survivors of both lists
    // merge the survivors into the other buffer
    for (int i = tid; i < n_old_s; i += kPlanThreads) {
      const unsigned long long key = kold[e_old + i];
      int lo = 0, hi = n_new_s;                            // offers that stay and are smaller
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (s_new[e_new + mid] < key) lo = mid + 1;
        else hi = mid;
      }
      knew[i + lo] = key;
      snew[i + lo] = sold[e_old + i];
    }
    if (tid < n_new_s) {
      const unsigned long long key = s_new[e_new + tid];
      int lo = 0, hi = n_old_s;                            // retained entries that stay and are smaller
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (kold[e_old + mid] < key) lo = mid + 1;
        else hi = mid;
      }
      knew[tid + lo] = key;
      snew[tid + lo] = s_newslot[e_new + tid];
    }
    // what every offer's position carries into the state: an offer that leaves at once is an ordinary unselected
    // token; an offer that stays carries nothing, or the retained token that leaves in its favour
    if (tid < lam) {
      const int tok = evict_key_token(s_new[tid]);
      int carries = tok;
      if (tid >= e_new) carries = (tid - e_new < e_old) ? evict_key_token(kold[tid - e_new]) : -1;
      src[tok] = carries;
    }
    n = n_old_s + n_new_s;
    cur ^= 1;
    // the set the rows of chunk s+2 see, as one bit per offer in routing order
    lds_barrier();
    if (s + 2 < nc) {
      for (int i = tid; i < n; i += kPlanThreads) atomicOr(&words[snew[i] >> 5], 1u << (snew[i] & 31));
      lds_barrier();
      for (int i = tid; i < 2 * a.AW; i += kPlanThreads) alive[(int64_t)(s + 2) * (2 * a.AW) + i] = words[i];
    }
    if (s == n_exp - 1 && a.fin_tok != nullptr) {
      for (int i = tid; i < n; i += kPlanThreads) {
        const int tok = evict_key_token(knew[i]);
        a.fin_tok[unit * M + i] = tok;
        a.fin_score[unit * M + i] = score[tok];
      }
      if (tid == 0) a.fin_n[unit] = n;
    }
  }
}

// v in operand order per QUERY head, every token position holding the value row of the token it carries (zeros for a
// position that carries nothing or lies in the padding).  Layout and tiling as in transpose_v_kernel.
template <typename E>
__global__ __launch_bounds__(256) void vfr_gather_kernel(VfrGatherArgs a) {
  __shared__ E tile[64][65];
  const E* __restrict__ v = static_cast<const E*>(a.v);
  const int tok0 = blockIdx.x * 64;
  const int nd = a.d / 64;
  const int h = blockIdx.y / nd, d0 = (blockIdx.y % nd) * 64;
  const int b = blockIdx.z;
  const int kvh = a.map.kv[h];
  const int n_tok = seq_tokens(a.seq_len, b, a.N);
  const int32_t* src = a.src + ((int64_t)b * a.Hq + h) * a.N;
  constexpr int EPV = 16 / (int)sizeof(E), VPR = 64 / EPV;
  for (int q = threadIdx.x; q < 64 * VPR; q += 256) {
    const int i = q / VPR, x0 = (q % VPR) * EPV;
    const int tok = tok0 + i;
    Vec16 pk;
    pk.w[0] = pk.w[1] = pk.w[2] = pk.w[3] = 0u;
    if (tok < n_tok) {
      const int st = src[tok];
      if (st >= 0)
        pk = *reinterpret_cast<const Vec16*>(v + (int64_t)b * a.v_sb + (int64_t)st * a.v_st + (int64_t)kvh * a.v_sh + d0 + x0);
    }
    const E* pe = reinterpret_cast<const E*>(&pk);
#pragma unroll
    for (int e = 0; e < EPV; ++e) tile[i][x0 + e] = pe[e];
  }
  __syncthreads();
  constexpr int KK = sizeof(E) == 2 ? 16 : 2, KPL = sizeof(E) == 2 ? 8 : 1;
  E* __restrict__ vfr = static_cast<E*>(a.vfr) + ((int64_t)b * a.Hq + h) * (int64_t)a.Np * a.d;
  for (int q = threadIdx.x; q < 64 * 64 / KPL; q += 256) {
    const int blk = q / 64, inner = q % 64;
    const int w2 = blk / (64 / KK), s = blk % (64 / KK);
    const int r = inner / 2, g = inner % 2;
    const int ti = s * KK + g * KPL, xi = 32 * w2 + r;
    E* dst = vfr + vfr_offset(tok0 + ti, d0 + xi, a.C, a.d, KK, KPL);
    if constexpr (KPL == 8) {
      Vec16 pk;
      E* pe = reinterpret_cast<E*>(&pk);
#pragma unroll
      for (int e = 0; e < KPL; ++e) pe[e] = tile[ti + e][xi];
      *reinterpret_cast<Vec16*>(dst) = pk;
    } else {
      dst[0] = tile[ti][xi];
    }
  }
}

// Retained rows of an exported decode state under the evict policy: the set after the last routed step, in the
// order the plan left it (the decode step makes no assumption about the order), with scores and token indices.
template <typename T>
__global__ __launch_bounds__(64) void state_fill_evict_kernel(StateFillEvictArgs a) {
  const int row = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
  const int64_t unit = (int64_t)b * a.Hq + hq;
  if (row >= a.fin_n[unit]) return;
  const int tok = a.fin_tok[unit * a.M + row];
  const int kvh = a.map.kv[hq];
  const T* k = static_cast<const T*>(a.k) + (int64_t)b * a.k_sb + (int64_t)tok * a.k_st + (int64_t)kvh * a.k_sh;
  const T* v = static_cast<const T*>(a.v) + (int64_t)b * a.v_sb + (int64_t)tok * a.v_st + (int64_t)kvh * a.v_sh;
  T* kr = static_cast<T*>(a.kret) + (unit * a.cap + row) * (int64_t)a.d;
  T* vr = static_cast<T*>(a.vret) + (unit * a.cap + row) * (int64_t)a.d;
  for (int x = threadIdx.x; x < a.d; x += 64) {
    kr[x] = k[x];
    vr[x] = v[x];
  }
  if (threadIdx.x == 0) {
    a.ret_score[unit * a.cap + row] = a.fin_score[unit * a.M + row];
    a.ret_tok[unit * a.cap + row] = tok;
  }
}

size_t evict_plan_smem(int M, int lam, int AW) { return (size_t)(M + lam) * 24 + (size_t)2 * AW * 4 + 16; }

hipError_t launch_evict_plan(const EvictPlanArgs& a, int B, hipStream_t stream) {
  const size_t smem = evict_plan_smem(a.M, a.lam, a.AW);
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(evict_plan_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(evict_plan_kernel, dim3(a.Hq, B), dim3(kPlanThreads), smem, stream, a);
  return hipGetLastError();
}

hipError_t launch_vfr_gather(const VfrGatherArgs& a, int dtype, int B, hipStream_t stream) {
  dim3 grid(a.Np / 64, a.Hq * (a.d / 64), B), block(256);
  if (dtype == 1)
    hipLaunchKernelGGL(vfr_gather_kernel<uint16_t>, grid, block, 0, stream, a);
  else
    hipLaunchKernelGGL(vfr_gather_kernel<uint32_t>, grid, block, 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_state_fill_evict(const StateFillEvictArgs& a, int dtype, int B, hipStream_t stream) {
  if (a.M <= 0) return hipSuccess;
  dim3 grid(a.M, a.Hq, B), block(64);
  if (dtype == 1)
    hipLaunchKernelGGL(state_fill_evict_kernel<bf16>, grid, block, 0, stream, a);
  else
    hipLaunchKernelGGL(state_fill_evict_kernel<float>, grid, block, 0, stream, a);
  return hipGetLastError();
}

}  // namespace still

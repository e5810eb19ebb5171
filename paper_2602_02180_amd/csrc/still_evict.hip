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

// One workgroup of 256 threads per (sequence, query head), walking the routing steps in order.
// LDS (dynamic): keys[M + lam] (8 bytes), slot[M + lam] (4 bytes: index of the offer in routing order), then the
// words of one alive row.
__global__ __launch_bounds__(256) void evict_plan_kernel(EvictPlanArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char dsm[];
  const int hq = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t unit = (int64_t)b * a.Hq + hq;
  const int N = seq_tokens(a.seq_len, b, a.N);
  const int C = a.C, lam = a.lam, M = a.M;
  const int ncf = N / C, nc = (N + C - 1) / C;
  const int n_exp = nc >= 2 ? nc - 2 : 0;                 // routing steps a decode hand-over has seen
  unsigned long long* keys = reinterpret_cast<unsigned long long*>(dsm);
  int* slot = reinterpret_cast<int*>(dsm + (size_t)(M + lam) * 8);
  uint32_t* words = reinterpret_cast<uint32_t*>(dsm + (size_t)(M + lam) * 12);   // 2 * AW 32-bit words
  __shared__ unsigned long long s_best[4];
  __shared__ int s_besti[4], s_ev[128], s_host[128], s_n;

  const float* score = a.score + unit * a.N;
  const int32_t* sel = a.sel + unit * (int64_t)a.ncf_all * lam;
  int32_t* src = a.src + unit * a.N;
  uint32_t* alive = reinterpret_cast<uint32_t*>(a.alive) + unit * (int64_t)a.nc_all * (2 * a.AW);

  for (int t = tid; t < a.N; t += 256) src[t] = t;        // every position carries its own token unless told otherwise
  for (int i = tid; i < 2 * (2 * a.AW); i += 256)         // rows of chunks 0 and 1 see no retained token
    if (i / (2 * a.AW) < a.nc_all) alive[i] = 0u;
  if (tid == 0) {
    s_n = 0;
    a.fin_n[unit] = 0;
  }
  __syncthreads();

  for (int s = 0; s < ncf; ++s) {
    const int n_old = s_n;
    // the chunk's offers join the set
    if (tid < lam) {
      const int tok = sel[(int64_t)s * lam + tid];
      keys[n_old + tid] = evict_key(score[tok], tok);
      slot[n_old + tid] = s * lam + tid;
      src[tok] = -1;                                       // kept: carries nothing (revised below)
    }
    __syncthreads();
    const int total = n_old + lam;
    const int over = total > M ? total - M : 0;
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
      if (lane == 0) s_best[wave] = best, s_besti[wave] = bi;
      __syncthreads();
      if (tid == 0) {
        int w = 0;
        for (int j = 1; j < 4; ++j)
          if (s_best[j] < s_best[w]) w = j;
        s_ev[it] = s_besti[w];
        s_host[it] = evict_key_token(s_best[w]);           // the token that leaves
        keys[s_besti[w]] = ~0ull;
      }
      __syncthreads();
    }
    if (tid == 0) {
      // An offer that leaves at once is an ordinary unselected token of its chunk.  A retained token that leaves is
      // carried by the position of an offer that stays (in ascending order of both).
      int nh = 0;                                          // leavers that were retained before this step
      for (int it = 0; it < over; ++it) {
        if (s_ev[it] >= n_old) src[s_host[it]] = s_host[it];
        else s_host[nh++] = s_host[it];
      }
      int h = 0;
      for (int i = 0; i < lam && h < nh; ++i)
        if (keys[n_old + i] != ~0ull) src[evict_key_token(keys[n_old + i])] = s_host[h++];
      // close the gaps: the last valid entries move into the vacated places (vacated indices in descending order)
      for (int x = 1; x < over; ++x) {                     // insertion sort, at most lam entries
        const int v = s_ev[x];
        int y = x - 1;
        while (y >= 0 && s_ev[y] < v) s_ev[y + 1] = s_ev[y], --y;
        s_ev[y + 1] = v;
      }
      int last = total - 1;
      for (int x = 0; x < over; ++x) {
        const int idx = s_ev[x];
        if (idx != last) keys[idx] = keys[last], slot[idx] = slot[last];
        --last;
      }
      s_n = total - over;
    }
    __syncthreads();
    const int n_now = s_n;
    // the set the rows of chunk s+2 see, as one bit per offer in routing order
    if (s + 2 < nc) {
      for (int i = tid; i < 2 * a.AW; i += 256) words[i] = 0u;
      __syncthreads();
      for (int i = tid; i < n_now; i += 256) atomicOr(&words[slot[i] >> 5], 1u << (slot[i] & 31));
      __syncthreads();
      for (int i = tid; i < 2 * a.AW; i += 256) alive[(int64_t)(s + 2) * (2 * a.AW) + i] = words[i];
    }
    if (s == n_exp - 1 && a.fin_tok != nullptr) {
      for (int i = tid; i < n_now; i += 256) {
        const int tok = evict_key_token(keys[i]);
        a.fin_tok[unit * M + i] = tok;
        a.fin_score[unit * M + i] = score[tok];
      }
      if (tid == 0) a.fin_n[unit] = n_now;
    }
    __syncthreads();
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

size_t evict_plan_smem(int M, int lam, int AW) { return (size_t)(M + lam) * 12 + (size_t)2 * AW * 4 + 16; }

hipError_t launch_evict_plan(const EvictPlanArgs& a, int B, hipStream_t stream) {
  const size_t smem = evict_plan_smem(a.M, a.lam, a.AW);
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(evict_plan_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(evict_plan_kernel, dim3(a.Hq, B), dim3(256), smem, stream, a);
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

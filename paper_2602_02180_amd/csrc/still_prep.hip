// Layout preparation: pure data movement, no arithmetic of the method.
//
//   transpose_v : v [B,N,Hkv,d] -> vt [B,Hkv,d,Np] (tokens contiguous, zero padded to Np), so that
//                 the value operand of every "contract over tokens" MFMA is k-contiguous; and a second copy
//                 in MFMA-fragment order for the kernel that loads that operand straight from global memory.
//   transpose_w : NP-Map weights [Hq,d,df] -> [Hq,df,d] (feature rows, d contiguous), or the same rows in the
//                 operand order of the key projection.
//   keep_mask   : the Top-lambda lists as one bit per token (what the state scan tests).
//   gather      : Index(k, M^SA), Index(v, M^SA) of Algorithm 1: the keys of the selected tokens of
//                 every full chunk, flattened in chunk order, as rows of kret [B,Hq,cap,d]; the values
//                 transposed into vrett [B,Hq,d,cap].  Rows beyond the selected count are zero.
#include "still_kernels.h"

namespace still {

template <typename E>
__global__ __launch_bounds__(256) void transpose_v_kernel(TransposeVArgs a) {
  __shared__ E tile[64][65];
  const E* __restrict__ v = static_cast<const E*>(a.v);
  E* __restrict__ vt = static_cast<E*>(a.vt);
  const int tok0 = blockIdx.x * 64;
  const int nd = a.d / 64;
  const int h = blockIdx.y / nd, d0 = (blockIdx.y % nd) * 64;
  const int b = blockIdx.z;
  const int n_tok = seq_tokens(a.seq_len, b, a.N);   // padding rows of a shorter sequence are written as zeros
  // rows in and columns out move in 16-byte pieces (bases and strides are multiples of 16 bytes; Np is a
  // multiple of 64)
  constexpr int EPV = 16 / (int)sizeof(E), VPR = 64 / EPV;     // elements per piece, pieces per 64-element row
  for (int q = threadIdx.x; q < 64 * VPR; q += 256) {
    const int i = q / VPR, x0 = (q % VPR) * EPV;
    const int tok = tok0 + i;
    Vec16 pk;
    pk.w[0] = pk.w[1] = pk.w[2] = pk.w[3] = 0u;
    if (tok < n_tok)
      pk = *reinterpret_cast<const Vec16*>(v + (int64_t)b * a.v_sb + (int64_t)tok * a.v_st + (int64_t)h * a.v_sh + d0 + x0);
    const E* pe = reinterpret_cast<const E*>(&pk);
#pragma unroll
    for (int e = 0; e < EPV; ++e) tile[i][x0 + e] = pe[e];
  }
  __syncthreads();
  for (int q = threadIdx.x; q < 64 * VPR; q += 256) {
    const int i = q / VPR, t0 = (q % VPR) * EPV;               // column d0 + i, tokens tok0 + t0 ..
    Vec16 pk;
    E* pe = reinterpret_cast<E*>(&pk);
#pragma unroll
    for (int e = 0; e < EPV; ++e) pe[e] = tile[t0 + e][i];
    *reinterpret_cast<Vec16*>(vt + (((int64_t)b * a.Hkv + h) * a.d + d0 + i) * a.Np + tok0 + t0) = pk;
  }
  // second copy in fragment order: consecutive threads write consecutive elements of one (column block, k-step)
  // piece (the 64 tokens of the tile lie in one chunk: C is a multiple of 64)
  if (a.vfr != nullptr) {
    constexpr int KK = sizeof(E) == 2 ? 16 : 2, KPL = sizeof(E) == 2 ? 8 : 1;
    E* __restrict__ vfr = static_cast<E*>(a.vfr) + ((int64_t)b * a.Hkv + h) * (int64_t)a.Np * a.d;
    // one thread writes the KPL consecutive elements of one (column, lane group) at once
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
}

template <typename E>
__global__ __launch_bounds__(256) void transpose_w_kernel(TransposeWArgs a) {
  // one 64 x 64 tile of one head per workgroup: rows of w in, rows of wt out, 16 bytes per thread and access
  __shared__ E tile[64][65];
  constexpr int EPV = 16 / (int)sizeof(E), VPR = 64 / EPV;
  const int h = blockIdx.z, x0 = blockIdx.x * 64, f0 = blockIdx.y * 64;
  const E* __restrict__ w = static_cast<const E*>(a.w) + (int64_t)h * a.d * a.df;
  E* __restrict__ wt = static_cast<E*>(a.wt) + (int64_t)h * a.d * a.df;
  for (int q = threadIdx.x; q < 64 * VPR; q += 256) {
    const int i = q / VPR, j0 = (q % VPR) * EPV;               // row x0 + i of w, features f0 + j0 ..
    const Vec16 pk = *reinterpret_cast<const Vec16*>(w + (int64_t)(x0 + i) * a.df + f0 + j0);
    const E* pe = reinterpret_cast<const E*>(&pk);
#pragma unroll
    for (int e = 0; e < EPV; ++e) tile[i][j0 + e] = pe[e];
  }
  __syncthreads();
  for (int q = threadIdx.x; q < 64 * VPR; q += 256) {
    const int j = q / VPR, i0 = (q % VPR) * EPV;               // row f0 + j of wt, columns x0 + i0 ..
    Vec16 pk;
    E* pe = reinterpret_cast<E*>(&pk);
#pragma unroll
    for (int e = 0; e < EPV; ++e) pe[e] = tile[i0 + e][j];
    *reinterpret_cast<Vec16*>(wt + (int64_t)(f0 + j) * a.d + x0 + i0) = pk;
  }
}

// W [Hq, d, df] -> W^T in the operand order of the key projection (wfrag_offset): one element per thread (the
// weights of all heads are a few hundred KB)
template <typename T>
__global__ __launch_bounds__(256) void w_frag_kernel(TransposeWArgs a) {
  typedef Mma<T> M;
  const int h = blockIdx.y;
  const int idx = blockIdx.x * 256 + threadIdx.x;      // position in the head's output
  if (idx >= a.d * a.df) return;
  const int e = idx % M::KPL, lane = (idx / M::KPL) % 64, blk = idx / (64 * M::KPL);
  const int s = blk % (a.d / M::KK), ft = blk / (a.d / M::KK);
  const int m = lane & 31, g = lane >> 5;
  const int x = s * M::KK + g * M::KPL + e, f = 32 * ft + M::kappa(m);
  static_cast<T*>(a.wt)[(int64_t)h * a.d * a.df + idx] = static_cast<const T*>(a.w)[((int64_t)h * a.d + x) * a.df + f];
}

template <typename E, int D>
__global__ __launch_bounds__(256) void gather_kernel(GatherArgs a) {
  __shared__ E tile[64][D + 2];
  __shared__ int s_tok[64];
  const E* __restrict__ k = static_cast<const E*>(a.k);
  const E* __restrict__ v = static_cast<const E*>(a.v);
  E* __restrict__ kret = static_cast<E*>(a.kret);
  E* __restrict__ vrett = static_cast<E*>(a.vrett);
  const int r0 = blockIdx.x * 64, hq = blockIdx.y, b = blockIdx.z;
  const int kvh = a.map.kv[hq];
  if (threadIdx.x < 64) {
    const int row = r0 + threadIdx.x;
    int tok = -1;
    int nsel = a.nsel;
    if (a.seq_len != nullptr) {   // right-padded batch: only the full chunks of this sequence have real selections
      const int own = retained_rows(seq_tokens(a.seq_len, b, a.N) / a.C, a.lam, a.rcap);
      nsel = own < nsel ? own : nsel;
    }
    if (row < nsel) {
      tok = a.sel[((int64_t)b * a.Hq + hq) * a.sel_stride + row];
      if (tok < 0 || tok >= a.N) tok = -1;  // caller-supplied indices are never trusted for addressing
    }
    s_tok[threadIdx.x] = tok;
  }
  __syncthreads();
  // rows move in 16-byte pieces (strides and bases are multiples of 16 bytes)
  constexpr int EPV = 16 / (int)sizeof(E), VPR = D / EPV;   // elements per piece, pieces per row
  for (int idx = threadIdx.x; idx < 64 * VPR; idx += 256) {
    const int i = idx / VPR, x = (idx % VPR) * EPV;
    const int tok = s_tok[i];
    const int row = r0 + i;
    Vec16 kv, vv;
    kv.w[0] = kv.w[1] = kv.w[2] = kv.w[3] = 0u;
    vv = kv;
    if (tok >= 0) {
      kv = *reinterpret_cast<const Vec16*>(k + (int64_t)b * a.k_sb + (int64_t)tok * a.k_st + (int64_t)kvh * a.k_sh + x);
      vv = *reinterpret_cast<const Vec16*>(v + (int64_t)b * a.v_sb + (int64_t)tok * a.v_st + (int64_t)kvh * a.v_sh + x);
    }
    *reinterpret_cast<Vec16*>(kret + (((int64_t)b * a.Hq + hq) * a.cap + row) * D + x) = kv;
    const E* ve = reinterpret_cast<const E*>(&vv);
#pragma unroll
    for (int e = 0; e < EPV; ++e) tile[i][x + e] = ve[e];
  }
  __syncthreads();
  // columns out: one thread writes 16 bytes (EPV retained rows) of one feature row
  for (int q = threadIdx.x; q < D * (64 / EPV); q += 256) {
    const int x = q / (64 / EPV), t0 = (q % (64 / EPV)) * EPV;
    Vec16 pk;
    E* pe = reinterpret_cast<E*>(&pk);
#pragma unroll
    for (int e = 0; e < EPV; ++e) pe[e] = tile[t0 + e][x];
    *reinterpret_cast<Vec16*>(vrett + (((int64_t)b * a.Hq + hq) * D + x) * a.cap + r0 + t0) = pk;
  }
}

// one thread per (batch, head, full chunk): the chunk's list as a bit mask
__global__ __launch_bounds__(128) void keep_mask_kernel(KeepMaskArgs a) {
  const int c = blockIdx.x * 128 + threadIdx.x, hq = blockIdx.y, b = blockIdx.z;
  if (c >= a.ncf) return;
  const int64_t chunk = ((int64_t)b * a.Hq + hq) * a.ncf + c;
  uint32_t m[4] = {0u, 0u, 0u, 0u};
  const int quota = chunk_quota(c, a.lam, a.rcap);
  for (int j = 0; j < quota; ++j) {
    const unsigned off = (unsigned)(a.sel[chunk * a.lam + j] - c * a.C);
    if (off < (unsigned)a.C) m[off >> 5] |= 1u << (off & 31);
  }
  for (int i = 0; i < a.C / 32; ++i) a.kmask[chunk * (a.C / 32) + i] = m[i];
}

hipError_t launch_keep_mask(const KeepMaskArgs& a, int B, hipStream_t stream) {
  if (a.ncf <= 0) return hipSuccess;
  dim3 grid((a.ncf + 127) / 128, a.Hq, B), block(128);
  hipLaunchKernelGGL(keep_mask_kernel, grid, block, 0, stream, a);
  return hipGetLastError();
}

// Rotary position embedding of q and k in place (the layer applies it before the operator; a pre-pass here, not
// fused into the tile loads: every key tile is re-read once per row tile and per score window, so rotating on load
// would repeat the rotation many times to save one element-wise pass).  One thread per (token, channel pair
// (i, i + d/2)): the angle position * base^(-2 i / d) and its sine and cosine are computed once and applied to that
// pair of every query head and every kv head of the token.
template <typename E>
__global__ __launch_bounds__(256) void rope_kernel(RopeArgs a) {
  const int half = a.d / 2;
  const int64_t idx = blockIdx.x * 256ll + threadIdx.x;
  const int64_t tok_idx = idx / half;
  const int i = (int)(idx % half);
  if (tok_idx >= (int64_t)a.B * a.N) return;
  const int b = (int)(tok_idx / a.N), t = (int)(tok_idx % a.N);
  const double pos = (double)((a.pos0 ? a.pos0[b] : 0) + t);
  // base^(-2 i / d) = exp2(-(2 i / d) log2(base)).  The angle reaches thousands of radians, where an fp32 product
  // is only good to ~1e-4 rad: angle, sine and cosine are taken in double (one pair per token and channel pair, a
  // small share of this memory-bound pass), the rotation itself in fp32.
  const double theta = exp2(-(2.0 * (double)i / (double)a.d) * (double)a.log2_base);
  double snd, csd;
  sincos(pos * theta, &snd, &csd);
  const float sn = (float)snd, cs = (float)csd;
  auto turn = [&](E* row) {
    const float x0 = to_f32<E>(row[i]), x1 = to_f32<E>(row[i + half]);
    row[i] = from_f32<E>(x0 * cs - x1 * sn);
    row[i + half] = from_f32<E>(x0 * sn + x1 * cs);
  };
  if (a.q != nullptr)
    for (int h = 0; h < a.Hq; ++h) turn(static_cast<E*>(a.q) + b * a.q_sb + (int64_t)t * a.q_st + h * a.q_sh);
  if (a.k != nullptr)
    for (int h = 0; h < a.Hkv; ++h) turn(static_cast<E*>(a.k) + b * a.k_sb + (int64_t)t * a.k_st + h * a.k_sh);
}

hipError_t launch_rope(const RopeArgs& a, int dtype, hipStream_t stream) {
  const int64_t n = (int64_t)a.B * a.N * (a.d / 2);
  const dim3 grid((unsigned)((n + 255) / 256));
  if (dtype == 1) hipLaunchKernelGGL(rope_kernel<bf16>, grid, dim3(256), 0, stream, a);
  else hipLaunchKernelGGL(rope_kernel<float>, grid, dim3(256), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_transpose_v(const TransposeVArgs& a, int dtype, int B, hipStream_t stream) {
  dim3 grid(a.Np / 64, a.Hkv * (a.d / 64), B), block(256);
  if (dtype == 1)
    hipLaunchKernelGGL(transpose_v_kernel<uint16_t>, grid, block, 0, stream, a);
  else
    hipLaunchKernelGGL(transpose_v_kernel<uint32_t>, grid, block, 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_transpose_w(const TransposeWArgs& a, int dtype, hipStream_t stream) {
  if (a.frag) {
    dim3 fgrid((a.d * a.df + 255) / 256, a.Hq), fblock(256);
    if (dtype == 1)
      hipLaunchKernelGGL(w_frag_kernel<bf16>, fgrid, fblock, 0, stream, a);
    else
      hipLaunchKernelGGL(w_frag_kernel<float>, fgrid, fblock, 0, stream, a);
    return hipGetLastError();
  }
  dim3 grid(a.d / 64, a.df / 64, a.Hq), block(256);   // d and d_f are multiples of 64
  if (dtype == 1)
    hipLaunchKernelGGL(transpose_w_kernel<uint16_t>, grid, block, 0, stream, a);
  else
    hipLaunchKernelGGL(transpose_w_kernel<uint32_t>, grid, block, 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_gather(const GatherArgs& a, int dtype, int B, hipStream_t stream) {
  if (a.cap == 0) return hipSuccess;
  dim3 grid(a.cap / 64, a.Hq, B), block(256);
  if (dtype == 1) {
    if (a.d == 64)
      hipLaunchKernelGGL((gather_kernel<uint16_t, 64>), grid, block, 0, stream, a);
    else
      hipLaunchKernelGGL((gather_kernel<uint16_t, 128>), grid, block, 0, stream, a);
  } else {
    if (a.d == 64)
      hipLaunchKernelGGL((gather_kernel<uint32_t, 64>), grid, block, 0, stream, a);
    else
      hipLaunchKernelGGL((gather_kernel<uint32_t, 128>), grid, block, 0, stream, a);
  }
  return hipGetLastError();
}

}  // namespace still

// Shared device helpers for the STILL hybrid-attention kernels (gfx950 only).
//
// Matrix work is expressed through the 32x32 MFMA instructions of CDNA4:
//   bf16 : v_mfma_f32_32x32x16_bf16  (each lane supplies 8 consecutive k values of one row)
//   fp32 : v_mfma_f32_32x32x2_f32    (each lane supplies 1 k value of one row)
// Operand convention used everywhere (lane = 32*g + r, g in {0,1}, r in 0..31):
//   A (32 x KK): lane holds row r,    k = KPL*g .. KPL*g+KPL-1   of the current k-step
//   B (KK x 32): lane holds column r, same k values
//   C (32 x 32): lane holds column r; accumulator register i is row 8*(i/4) + 4*g + (i%4)
// A result in C layout can feed the next contraction directly as an operand: its register
// dimension (rows) becomes the contracted index, its lane dimension stays free.  To make the
// registers of one lane group hold CONSECUTIVE k positions, the producer assigns logical row
// `kappa(m)` to MFMA row m; then accumulator register i of group g is position pos_of_reg(i, g).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>
#include <utility>

namespace still {

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kMaxHq = 128;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct HeadMap {
  int32_t kv[kMaxHq];
};

template <typename T>
struct Mma;

template <>
struct Mma<bf16> {
  typedef bf16x8 frag;
  static constexpr int KK = 16;  // k per instruction
  static constexpr int KPL = 8;  // k per lane
  static __device__ __forceinline__ floatx16 mma(frag a, frag b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
  // logical row carried by MFMA row m (swap bits 2 and 3)
  static __device__ __forceinline__ int kappa(int m) { return (m & ~12) | ((m & 4) << 1) | ((m & 8) >> 1); }
  static __device__ __forceinline__ int kappa_inv(int p) { return kappa(p); }
  // logical position (0..31) held by accumulator register i of lane group g
  static __device__ __forceinline__ int pos_of_reg(int i, int g) { return 16 * (i >> 3) + 8 * g + (i & 7); }
  static __device__ __forceinline__ frag load(const bf16* p) { return *reinterpret_cast<const frag*>(p); }
  // operand fragment of k-step s (positions 16s .. 16s+15 of a 32-position tile) from C-layout registers
  static __device__ __forceinline__ frag from_acc(const floatx16& c, int s /*0..1*/) {
    frag f;
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] = static_cast<bf16>(c[8 * s + e]);
    return f;
  }
  static constexpr int STEPS_PER_TILE = 2;  // k-steps covering one 32-position tile
  // acc + sum_e a[e] * b[e] in fp32 (v_dot2c_f32_bf16, two products per instruction)
  static __device__ __forceinline__ float dot_into(frag a, frag b, float acc) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      bf16x2 pa, pb;
      pa[0] = a[e]; pa[1] = a[e + 1];
      pb[0] = b[e]; pb[1] = b[e + 1];
      acc = __builtin_amdgcn_fdot2_f32_bf16(pa, pb, acc, false);
    }
    return acc;
  }
  // acc + sum of the fragment's elements, in fp32, on the ROUNDED bf16 values (v_dot2c_f32_bf16 with ones)
  static __device__ __forceinline__ float sum_into(frag f, float acc) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 one;
    one[0] = static_cast<__bf16>(1.0f);
    one[1] = static_cast<__bf16>(1.0f);
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      bf16x2 pr;
      pr[0] = f[e];
      pr[1] = f[e + 1];
      acc = __builtin_amdgcn_fdot2_f32_bf16(pr, one, acc, false);
    }
    return acc;
  }
};

template <>
struct Mma<float> {
  typedef float frag;
  static constexpr int KK = 2;
  static constexpr int KPL = 1;
  static __device__ __forceinline__ floatx16 mma(frag a, frag b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
  }
  // m = 8a + 4g + r  ->  8a + 2r + g
  static __device__ __forceinline__ int kappa(int m) { return (m & ~7) | ((m & 3) << 1) | ((m >> 2) & 1); }
  // p = 8a + 2r + g  ->  8a + 4g + r
  static __device__ __forceinline__ int kappa_inv(int p) { return (p & ~7) | ((p & 1) << 2) | ((p >> 1) & 3); }
  static __device__ __forceinline__ int pos_of_reg(int i, int g) { return 2 * i + g; }
  static __device__ __forceinline__ frag load(const float* p) { return *p; }
  static __device__ __forceinline__ frag from_acc(const floatx16& c, int s /*0..15*/) { return c[s]; }
  static constexpr int STEPS_PER_TILE = 16;
  static __device__ __forceinline__ float sum_into(frag f, float acc) { return acc + f; }
  static __device__ __forceinline__ float dot_into(frag a, frag b, float acc) { return fmaf(a, b, acc); }
};

// natural C-layout row of accumulator register i for lane group g
__device__ __forceinline__ int c_row(int i, int g) { return 8 * (i >> 2) + 4 * g + (i & 3); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }
__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }

// Reductions over the two lane groups (lane and lane ^ 32) without an LDS round trip: v_permlane32_swap
// exchanges the upper 32 lanes of its first operand with the lower 32 lanes of its second; given the same value
// twice it leaves the lower group's values in every lane of one result and the upper group's in the other.
struct LaneGroups {
  float lo, hi;   // value of lane (l & 31) and of lane (l & 31) + 32, in every lane
};
__device__ __forceinline__ LaneGroups lane_groups(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return {__uint_as_float(r[0]), __uint_as_float(r[1])};
}
__device__ __forceinline__ float sum32(float x) {
  const LaneGroups p = lane_groups(x);
  return p.lo + p.hi;
}
__device__ __forceinline__ float max32(float x) {
  const LaneGroups p = lane_groups(x);
  return fmaxf(p.lo, p.hi);
}
__device__ __forceinline__ float min32(float x) {
  const LaneGroups p = lane_groups(x);
  return fminf(p.lo, p.hi);
}

template <typename T>
__device__ __forceinline__ float to_f32(T x) { return static_cast<float>(x); }

template <typename T>
__device__ __forceinline__ T from_f32(float x) { return static_cast<T>(x); }

// logistic function through the hardware exp2 / rcp
__device__ __forceinline__ float fast_sigmoid(float x) { return fast_rcp(1.0f + fast_exp2(-x * kLog2e)); }

__device__ __forceinline__ floatx16 zero16() {
  floatx16 z;
#pragma unroll
  for (int i = 0; i < 16; ++i) z[i] = 0.f;
  return z;
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also drains every outstanding global
// load and store of the wave (vmcnt(0)), which would expose the latency of prefetches and of result
// stores at each pipeline step; the kernels that use this barrier exchange data between waves through
// LDS only, and never read global memory written by another wave of the same launch.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Lane index within the wave, recomputed by two instructions at the point of the call.  The asm is opaque to the
// compiler, so the value (and every address derived from it) has a short live range: in kernels whose register
// file is full of accumulators this keeps lane-dependent addresses from being computed once up front and then
// spilled to scratch memory, whose reloads queue behind the outstanding global prefetches.
__device__ __forceinline__ int fresh_lane_id() {
  int l;
  asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
  return l;
}

// Block id -> (query head, work item) with the head varying fastest, so that workgroups running at the same
// time read the SAME token range of q/k/v for different heads: in the [B, N, H, d] layout one token's rows of
// all heads are contiguous, and a DRAM page fetched for one head is used by the others while it is open.
// Block ids are dealt round-robin to the 8 XCDs; XCD x is given the heads [x*Hq/8, (x+1)*Hq/8), i.e. whole
// GQA groups when Hq/Hkv divides Hq/8, so a kv-head's rows are shared through that XCD's L2.
__device__ __forceinline__ void head_major_block(int L, int Hq, int& hq, int& item) {
  if ((Hq & 7) == 0) {
    const int hpx = Hq >> 3, xcd = L & 7, slot = L >> 3;
    hq = xcd * hpx + slot % hpx;
    item = slot / hpx;
  } else {
    hq = L % Hq;
    item = L / Hq;
  }
}

// Global -> LDS copies without staging registers (global_load_lds): lane L's 16 (or 4) bytes land at
// lds_base + 16 L (4 L).  They are issued as opaque assembly on purpose.  Issued through the compiler builtin,
// an in-flight copy makes the compiler's wait-count bookkeeping treat every later LDS wait as "wait for
// everything" (the instruction touches two address spaces), which drains the LDS read pipeline of the very
// loops these copies are meant to run under.  The price: the compiler does not know about these copies, so the
// caller must wait for them itself (s_waitcnt vmcnt(0), then a workgroup barrier) before the data is read.
// The LDS base is uniform over the wave by contract; it is taken from the first lane because the constraint
// needs a scalar register and a base selected at run time (one slot or another) may sit in a vector register.
typedef __attribute__((address_space(3))) void* lds_ptr_t;

__device__ __forceinline__ uint32_t lds_address(const void* p) {
  return (uint32_t)(uintptr_t)(lds_ptr_t)p;
}

__device__ __forceinline__ void async_copy16(const void* gptr, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :
               : "v"(gptr), "s"(__builtin_amdgcn_readfirstlane(lds_base))
               : "memory", "m0");
}

__device__ __forceinline__ void async_copy4(const void* gptr, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off"
               :
               : "v"(gptr), "s"(__builtin_amdgcn_readfirstlane(lds_base))
               : "memory", "m0");
}

__device__ __forceinline__ void wait_async_copies() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// f(integral_constant<int, 0>{}), ..., f(integral_constant<int, N-1>{}) in order: a loop whose index is a
// compile-time constant in every iteration by construction (register arrays indexed with it never depend on
// the loop unroller's thresholds).
template <int... Is, typename F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, Is...>, F&& f) {
  (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, static_cast<F&&>(f));
}

// 16-byte global/LDS copy unit
struct __attribute__((aligned(16))) Vec16 {
  uint32_t w[4];
};

}  // namespace still

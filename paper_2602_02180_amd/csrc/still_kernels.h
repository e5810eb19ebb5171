// Kernel argument blocks and host-side launchers shared by the translation units of libstill.
// Nothing here is part of the public ABI (include/still.h is).
#pragma once
#include "still_common.h"

namespace still {

struct ScoreArgs {
  const void* q;
  const void* k;
  int64_t q_sb, q_st, q_sh, k_sb, k_st, k_sh;
  HeadMap map;
  int N, C, W, lam, Hq, ncf;
  int rcap;       // budget on the retained tokens of one (batch, head): see chunk_quota()
  float scale, eps;
  float* score;   // [B, Hq, N]
  int32_t* sel;   // [B, Hq, ncf, lam] or nullptr (no selection)
};

// Tokens that chunk c keeps when at most rcap tokens may be retained in total and chunks are served in order:
// lam until the budget is used up, then what is left of it, then none.  Retained row c * lam + pos therefore
// stays the row of slot pos of chunk c, and the rows in use are exactly those below min(chunks * lam, rcap).
__host__ __device__ inline int chunk_quota(int c, int lam, int rcap) {
  const int left = rcap - c * lam;
  return left >= lam ? lam : (left > 0 ? left : 0);
}
__host__ __device__ inline int retained_rows(int chunks, int lam, int rcap) {
  const int r = chunks * lam;
  return r < rcap ? r : rcap;
}
constexpr int kNoBudget = 1 << 30;
constexpr int kMaxEvictBudget = 4096;   // the plan and the routing step hold the retained set in LDS

// Tokens of sequence b: N for every sequence, or, for a right-padded batch, the caller's per-sequence count
// (device array, clamped to [1, N]).  Rows at and beyond it are padding: never read as keys or values by a real
// row, never written as outputs.
__device__ inline int seq_tokens(const int32_t* seq_len, int b, int N) {
  if (seq_len == nullptr) return N;
  const int n = seq_len[b];
  return n < 1 ? 1 : (n > N ? N : n);
}

struct GScoreArgs {
  const void* q;
  const void* k;
  int64_t q_sb, q_st, q_sh, k_sb, k_st, k_sh;
  HeadMap map;
  int N, Hq;
  float scale, eps;
  float* score;   // [B, Hq, N]
};

struct TransposeVArgs {
  const void* v;
  int64_t v_sb, v_st, v_sh;
  void* vt;       // [B, Hkv, d, Np]
  void* vfr;      // nullable: the same values in MFMA-fragment order, see vfr_offset()
  int N, Np, Hkv, d, C;
  const int32_t* seq_len;   // nullable, device [B]: see seq_tokens()
};

// Element offset of (token tau, column x) of one (batch, kv head) in the fragment-ordered copy of v that the
// linear-attention consumers load their "S += phi_k^T V" operand from: [chunk][x / 32][k-step][x % 32][lane
// group][k per lane], so that the 64 lanes of one operand load read one contiguous piece (1 KB for 2-byte types).
// KK / KPL = k per instruction / per lane of the element type's MFMA (16 / 8 for 2-byte types, 2 / 1 for fp32).
__host__ __device__ inline int64_t vfr_offset(int tau, int x, int C, int D, int KK, int KPL) {
  const int ch = tau / C, tc = tau % C;
  const int s = tc / KK, g = (tc % KK) / KPL, e = tc % KPL;
  return ((((int64_t)ch * (D / 32) + x / 32) * (C / KK) + s) * 64 + 2 * (x % 32) + g) * KPL + e;
}

struct TransposeWArgs {
  const void* w;  // [Hq, d, df]
  void* wt;       // [Hq, df, d], or (frag) the same rows in MFMA operand order, see wfrag_offset()
  int Hq, d, df;
  int frag;
};

// Element offset, inside one head's copy, of W^T[f][x] in the operand order of the key projection f^T = W^T x^T:
// [feature tile f / 32][k-step x / KK][lane = 32 g + m][k per lane], with feature 32 ft + kappa(m) in MFMA row m,
// so that the 64 lanes of one operand load read one contiguous piece.
template <typename M>
__host__ __device__ inline int wfrag_offset(int ft, int s, int lane, int d) {
  return ((ft * (d / M::KK) + s) * 64 + lane) * M::KPL;
}

// Tokens per round of the linear-attention state scan: the round's feature image [2 d_f][round] is double
// buffered in LDS, so wide features in a wide type take shorter rounds.
__host__ __device__ constexpr int la_round_tokens(int es, int d) { return es * 2 * d <= 512 ? 128 : 64; }

struct GatherArgs {
  const void* k;
  const void* v;
  int64_t k_sb, k_st, k_sh, v_sb, v_st, v_sh;
  HeadMap map;
  const int32_t* sel;  // [B, Hq, sel_stride]; the first nsel entries of each list are gathered
  int nsel, sel_stride, cap, Hq, d, N;
  int C, lam, rcap;
  const int32_t* seq_len;   // nullable, device [B]: rows of chunks beyond a sequence's full chunks are zero
  void* kret;          // [B, Hq, cap, d]
  void* vrett;         // [B, Hq, d, cap]
};

// Top-lambda lists -> one bit per token of every full chunk (set = kept by the softmax branch, so the token does
// NOT enter the linear state).  Entries outside their chunk are ignored (caller-supplied lists are never trusted for
// addressing); slots beyond a chunk's quota are not read.
struct KeepMaskArgs {
  const int32_t* sel;   // [B, Hq, ncf, lam], nullable when lam == 0
  uint32_t* kmask;      // [B, Hq, ncf, C/32]
  int Hq, ncf, C, lam, rcap;
};

struct LaArgs {
  const void* k;
  int64_t k_sb, k_st, k_sh;
  const void* vfr;     // [B, Hkv, Np * d]: v in fragment order (vfr_offset)
  const void* wkf;     // [Hq, df * d]: Wk^T in operand order (wfrag_offset)
  const void* bk;      // nullable [Hq, df]
  const uint32_t* kmask;  // [B, Hq, ncf, C/32]: bit = token kept by the softmax branch (see KeepMaskArgs)
  HeadMap map;
  int N, Np, C, Hq, Hkv, nc, ncf;
  const int32_t* seq_len;   // nullable, device [B]
  int seg_chunks, nseg;
  float* seg;          // [B, Hq, nseg][D*DP + DP]: every segment's total, S^T as [x][feature], then z
  void* snap;          // [B, Hq, nc][D][DP] storage type: S^T summed over chunk c's own segment, through chunk c-2
  float* zsnap;        // [B, Hq, nc][DP]: z likewise
  void* pimg;          // [B, Hq, nseg][D][DP] storage type: S^T through the chunk before the segment (prefix)
  float* zpre;         // [B, Hq, nseg][DP]: z likewise
  float* s_final;      // nullable [B, Hq, DP*(D+1)] as S [feature][x] then z: fp32 state through chunk (last - 2)
  const int32_t* src;  // evict policy only [B, Hq, N]: token carried by every position (-1: none); replaces kmask, and
                       //   vfr is then per QUERY head ([B, Hq, Np * d], built through the same table)
};

// Budget policy "evict the lowest score" in the prefill (still_evict.hip)
struct EvictPlanArgs {
  const float* score;      // [B, Hq, N]
  const int32_t* sel;      // [B, Hq, ncf_all, lam]: every chunk's offers (its lam highest scores)
  int32_t* src;            // [B, Hq, N]: token whose key/value a position carries into the state scan (-1: none)
  void* alive;             // [B, Hq, nc_all, AW] 64-bit words: bit j = offer j (routing order) is retained for the rows
                           //   of that chunk
  int32_t* fin_tok;        // nullable [B, Hq, M]: the set retained after the last routed step (decode hand-over)
  float* fin_score;        // [B, Hq, M]
  int32_t* fin_n;          // [B, Hq]
  const int32_t* seq_len;  // nullable, device [B]
  int N, C, lam, M, Hq, ncf_all, nc_all, AW;
};
struct VfrGatherArgs {
  const void* v;
  int64_t v_sb, v_st, v_sh;
  const int32_t* src;      // [B, Hq, N]
  void* vfr;               // [B, Hq, Np * d]
  HeadMap map;
  const int32_t* seq_len;
  int N, Np, Hq, d, C;
};
struct StateFillEvictArgs {
  const void* k;
  const void* v;
  int64_t k_sb, k_st, k_sh, v_sb, v_st, v_sh;
  const int32_t* fin_tok;
  const float* fin_score;
  const int32_t* fin_n;
  void* kret;
  void* vret;
  float* ret_score;
  int32_t* ret_tok;
  HeadMap map;
  int M, cap, Hq, d;
};
constexpr int kMaxEvictOffers = 32768;   // offers per (sequence, head) the sparse kernel's LDS mask rows hold (x 2 chunks)

// query rows per workgroup of the sparse-attention kernel (one wave per 32 rows)
constexpr int kSaRows = 128;

struct SaArgs {
  const void* q;
  const void* k;
  int64_t q_sb, q_st, q_sh, k_sb, k_st, k_sh;
  const void* vt;      // [B, Hkv, d, Np]
  const void* kret;    // [B, Hq, cap, d]
  const void* vrett;   // [B, Hq, d, cap]
  const void* wqt;     // [Hq, df, d]: Wq^T
  const void* bq;      // nullable [Hq, df]
  const void* g;       // nullable gate [B, N, Hq, d]
  int64_t g_sb, g_st, g_sh;
  int gate_act;        // 1: g is a pre-activation, the gate is its logistic function
  const void* snap;    // [B, Hq, nc][D][DP]: see LaArgs
  const float* zsnap;  // [B, Hq, nc][DP]
  const void* pimg;    // [B, Hq, nseg][D][DP]
  const float* zpre;   // [B, Hq, nseg][DP]
  int seg_chunks, nseg;
  float* n_la_out;     // nullable [B, Hq, N, d]: the gated linear numerator of every row (inspection)
  float* d_la_out;     // nullable [B, Hq, N]
  float* lse;          // nullable [B, Hq, N]: ln(D_SA + D_LA) of every row
  void* out;
  int64_t o_sb, o_st, o_sh;
  HeadMap map;
  int N, Np, C, lam, Hq, Hkv, cap, ntiles, B_, rcap, nc;
  const int32_t* seq_len;   // nullable, device [B]
  float scale;
  const void* alive;   // evict policy only [B, Hq, nc, AW] 64-bit words: see EvictPlanArgs (the retained tiles are then
  int AW;              //   all offers, each under its chunk's mask; AW = words per row = cap / 64)
};

struct DecArgs {
  float* S;            // [B, Hq, DP*(D+1)]
  void* kret;          // [B, Hq, cap, d]
  void* vret;
  int32_t* sel;        // [B, Hq, nchunks, lam]
  void* kring;         // [B, Hkv, R, d]
  void* vring;
  float* score;        // [B, Hq, R]
  float* part;         // [B, Hq, 32, d+2]
  const void* q;       // [B, Hq, d]
  const void* k;       // [B, Hkv, d]
  const void* v;
  const void* g;       // nullable
  const void* wq;      // [Hq, d, df]
  const void* wk;
  const void* bq;      // nullable
  const void* bk;
  void* out;           // [B, Hq, d]
  HeadMap map;
  int B, Hq, Hkv, C, W, lam, cap, R, nchunks, t, nsplit, rcap;
  int shared;              // 1: the query heads of one kv head rank by their summed score (one list per group)
  int gate_act;            // 1: g is a pre-activation, the gate is its logistic function
  int evict;               // 1: the budget is held by evicting the lowest score (ret_score, ret_tok are then kept)
  float* ret_score;        // [B, Hq, cap] score of every retained row
  int32_t* ret_tok;        // [B, Hq, cap] its token index
  const int32_t* tpos;     // nullable, device [B]: index of each sequence's new token (t is then ignored)
  int max_tokens;
  float scale, eps;
};

// Index of the new token of sequence b: the same for every sequence, or the caller's per-sequence entry.  An
// entry outside [0, max_tokens) marks a sequence that sits this step out (-1 is returned).
__device__ inline int step_index(const DecArgs& a, int b) {
  if (a.tpos == nullptr) return a.t;
  const int t = a.tpos[b];
  return (t >= 0 && t < a.max_tokens) ? t : -1;
}

// Retained rows of a decode state: one slice per (sequence, query head), or, with group-shared selection, one per
// (sequence, kv head), written by the lowest query head of the group only.
__device__ inline int64_t retained_slice(bool shared, int b, int hq, int kvh, int Hq, int Hkv) {
  return shared ? (int64_t)b * Hkv + kvh : (int64_t)b * Hq + hq;
}
__device__ inline bool writes_retained(bool shared, const HeadMap& map, int hq) {
  if (!shared) return true;
  for (int h = 0; h < hq; ++h)
    if (map.kv[h] == map.kv[hq]) return false;
  return true;
}

struct StateFillArgs {
  const void* k;
  const void* v;
  int64_t k_sb, k_st, k_sh, v_sb, v_st, v_sh;
  const float* score;      // [B, Hq, N]
  const int32_t* sel;      // [B, Hq, ncf, lam]
  HeadMap map;
  void* kret;
  void* vret;
  int32_t* sel_state;
  void* kring;
  void* vring;
  float* score_ring;
  int N, R, Hq, Hkv, d, lam, cap, ncf, nchunks, rcap, shared, C;
  int lists_only;           // 1: write the index lists of the routed chunks but no retained rows (evict policy)
  const int32_t* seq_len;   // nullable, device [B]
};

hipError_t launch_decode_step(const DecArgs& a, int dtype, int d, bool route, hipStream_t stream);
hipError_t launch_state_fill(const StateFillArgs& a, int dtype, int B, int n_routed, hipStream_t stream);
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t stream);
hipError_t launch_score(const ScoreArgs& a, int dtype, int d, int B, int nc, hipStream_t stream);
hipError_t launch_global_score(const GScoreArgs& a, int dtype, int d, int B, hipStream_t stream);
hipError_t launch_topk_overlap(const float* sa, const float* sb, int32_t* overlap, int N, int C, int lam, int Hq,
                               int B, hipStream_t stream);
hipError_t launch_group_select(const ScoreArgs& a, int B, int Hkv, hipStream_t stream);
hipError_t launch_transpose_v(const TransposeVArgs& a, int dtype, int B, hipStream_t stream);
hipError_t launch_transpose_w(const TransposeWArgs& a, int dtype, hipStream_t stream);
hipError_t launch_gather(const GatherArgs& a, int dtype, int B, hipStream_t stream);
hipError_t launch_keep_mask(const KeepMaskArgs& a, int B, hipStream_t stream);
hipError_t launch_la_states(const LaArgs& a, int dtype, int d, int B, hipStream_t stream);
hipError_t launch_la_prefix(const LaArgs& a, int dtype, int d, int B, hipStream_t stream);
hipError_t launch_sa(const SaArgs& a, int dtype, int d, int B, hipStream_t stream);
hipError_t launch_evict_plan(const EvictPlanArgs& a, int B, hipStream_t stream);
hipError_t launch_vfr_gather(const VfrGatherArgs& a, int dtype, int B, hipStream_t stream);
hipError_t launch_state_fill_evict(const StateFillEvictArgs& a, int dtype, int B, hipStream_t stream);
size_t evict_plan_smem(int M, int lam, int AW);

// ---- backward pass (still_bwd.hip) ----
// One operand of the generic batched product: element (row, k) of batch item (b, head, c) sits at
// base[b*s_b + head*s_h + (c / c_div)*s_c + row*s_r + k*s_k]; head is the query head or, with kv = 1, its kv head.
struct GemmOperand {
  const void* base;
  int64_t s_b, s_h, s_c, s_r, s_k;
  int kv, c_div, f32;      // f32 = 1: the elements are float whatever the storage type
};
struct GemmArgs {
  GemmOperand A, B;        // C[m][n] = sum_k A(m, k) B(n, k)
  GemmOperand B2;          // base != nullptr: ... + sum_k A(m, k) B2(n, k), the same A against a second operand
  float* C;                // element (m, n) of item (b, head, c) at C[b*c_b + head*c_h + c*c_c + m*c_r + n]
  int64_t c_b, c_h, c_c, c_r;
  int c_kv;
  int M, Nn, K;            // per item; Nn and K multiples of 64 (a K cut short by k_total reads as zeros)
  int m_total, k_total;    // > 0: item c holds only min(M, m_total - c*M) rows / min(K, k_total - c*K) contraction entries
  int Hq;
  HeadMap map;
  int mode;                // 0: store, 1: add, 2: atomic add
};
struct BwdRowArgs {
  const void* out;         // y of the forward pass, strided like dout
  const void* dout;
  int64_t o_sb, o_st, o_sh;
  const void* g;           // nullable gate
  int64_t g_sb, g_st, g_sh;
  int gate_act;
  const float* lse;        // [U, N]
  float* e_row;            // [U, N]: E_t = exp(-L_t)
  float* delta;            // [U, N]: dy_t . y_t
  float* ed;               // [U, N]: E_t delta_t
  void* A;                 // [U, N, d] storage type: E_t (gate_t * dy_t)
  const float* nraw;       // [U, N, d]: phi_q S (dg kernel)
  void* dg;                // strided like g (dg kernel)
  int U, N, Hq, d;
};
struct BwdNpArgs {
  const void* x;           // q or k
  int64_t x_sb, x_st, x_sh;
  int x_kv;                // 1: x is read (and its gradient accumulated) at the kv head of the query head
  const void* bias;        // nullable [Hq, F]
  float* u;                // [U, N, F]: f = x W on entry of the forward kernel, u afterwards
  float* st;               // [U, N, 2]: |x|, |f|
  void* phi;               // [U, N, 2F] storage type (forward kernel)
  const uint32_t* kmask;   // nullable [B, Hq, ncf, C/32]: tokens the softmax branch keeps have phi = 0, df = 0
  const float* dphi;       // [U, N, 2F] (backward kernel)
  const float* coef;       // nullable [U, N]: dphi -= coef * (z1 + z2)
  const float* z1;         // nullable [U, nc, 2F]
  const float* z2;         // nullable [U, nseg, 2F], indexed by chunk / seg_chunks
  void* df;                // [U, N, F] storage type
  float* cx;               // [U, N]: coefficient of x in dx (the |x| path), 0 for tokens without a gradient
  HeadMap map;
  int U, N, Hq, Hkv, d, F, C, nc, ncf, nseg, seg_chunks;
};
struct BwdColsumArgs {
  const void* X;           // [U, N, L] storage type
  const float* w;          // nullable [U, N]
  float* out;              // [U, nc, L], or (per_head) [Hq, L] added atomically
  int N, C, nc, L, Hq, per_head;
};
struct BwdFinishArgs {
  const float* src;        // [B, H, N, d]
  void* dst;               // strided, storage type
  const void* x;           // the tensor the gradient belongs to (same strides as dst); read when cx is given
  int64_t s_b, s_t, s_h;
  const float* cx;         // nullable [B, Hq, N]: dst += coefficient * x
  int per_kv;              // 1: H counts kv heads, the coefficients of the query heads of a kv head are added up
  HeadMap map;
  int B, H, Hq, N, d;
};
struct BwdSaArgs {
  const void* q;
  const void* k;
  const void* v;
  const void* dout;
  int64_t q_sb, q_st, q_sh, k_sb, k_st, k_sh, v_sb, v_st, v_sh, o_sb, o_st, o_sh;
  const void* qt;          // [U, d, Np]: q transposed, zero padded
  const void* dot;         // [U, d, Np]: dout transposed
  const void* kt;          // [B, Hkv, d, Np]: k transposed
  const void* kret;        // [U, cap, d]: retained keys in routing order, zero rows where no token is retained
  const void* krett;       // [U, d, cap]: the same, transposed
  const int32_t* sel;      // [U, sel_stride]: retained entry e is token sel[e] (chunk e / lam)
  const float* lse;        // [U, N]
  const float* delta;      // [U, N]
  float* dq32;             // [U, N, d]
  float* dk32;             // [B, Hkv, N, d]: stored by the local key tiles, added to by the retained ones
  float* dv32;
  HeadMap map;
  int N, Np, cap, C, lam, rcap, Hq, Hkv, nc, sel_stride, n_row_tiles, n_ret_tiles;
  float scale;
};
struct RopeArgs {
  void* q;                 // nullable [B, N, Hq, d], rotated in place
  void* k;                 // nullable [B, N, Hkv, d]
  int64_t q_sb, q_st, q_sh, k_sb, k_st, k_sh;
  const int32_t* pos0;     // nullable, device [B]: position of each sequence's token 0
  double log2_base;
  int B, N, Hq, Hkv, d;
};
hipError_t launch_rope(const RopeArgs& a, int dtype, hipStream_t stream);
hipError_t launch_bgemm(const GemmArgs& a, int dtype, int U, int n_c, hipStream_t stream);
// the same product summed over the items c' >= c + 2 for every item c, written in the storage type (C is then a T*;
// M a multiple of 64, m_total unused)
hipError_t launch_bgemm_revscan(const GemmArgs& a, int dtype, int U, int n_c, hipStream_t stream);
hipError_t launch_fill_f32(float* p, int64_t n, float x, hipStream_t stream);
hipError_t launch_bwd_row_prep(const BwdRowArgs& a, int dtype, hipStream_t stream);
hipError_t launch_bwd_dg(const BwdRowArgs& a, int dtype, hipStream_t stream);
hipError_t launch_bwd_np(const BwdNpArgs& a, int dtype, bool backward, hipStream_t stream);
hipError_t launch_bwd_colsum(const BwdColsumArgs& a, int dtype, int U, hipStream_t stream);
hipError_t launch_bwd_revcumsum(float* X, int U, int nc, int64_t L, hipStream_t stream);
hipError_t launch_bwd_finish(const BwdFinishArgs& a, int dtype, hipStream_t stream);
hipError_t launch_bwd_sa(const BwdSaArgs& a, int dtype, int d, int B, hipStream_t stream);
struct AttnMapArgs {
  const void* q;
  const void* k;
  int64_t q_sb, q_st, q_sh, k_sb, k_st, k_sh;
  const void* phi_q;       // [U, N, 2d] storage type
  const void* phi_k;       // [U, N, 2d], zero rows' worth for selected tokens
  const uint32_t* kmask;   // [U, ncf, C/32]: bit = token selected (within its chunk's quota)
  const float* lse;        // [U, N]
  float* map_out;          // [U, N, N]
  HeadMap map;
  int N, C, Hq, ncf;
  float scale;
};
struct MapDwArgs {
  const float* dA;         // [U, N, N]
  const float* lse;        // [U, N]
  const uint32_t* kmask;   // [U, ncf, C/32]
  float* rowdot;           // [U, N]
  void* dw;                // [U, N, Np8] storage type
  int N, Np8, C, ncf;
};
hipError_t launch_map_dw(const MapDwArgs& a, const float* A, int dtype, int U, hipStream_t stream);
hipError_t launch_attn_map(const AttnMapArgs& a, int dtype, int d, int U, hipStream_t stream);

}  // namespace still

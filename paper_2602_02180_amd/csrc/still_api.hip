// C ABI of libstill: argument validation, workspace layout and the launch sequence of the prefill path.
// See include/still.h for the contract of every entry point.
#include "../../include/still.h"

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>

#include "still_kernels.h"

namespace {

thread_local char g_err[512] = "";

still_status_t fail(still_status_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

// per-thread kernel timing (host-side event objects only): one (begin, end) pair per kernel, recorded on the
// stream that kernel runs on, in a ring of kProfRing sets so that a run of calls can be timed without a
// synchronisation in between
constexpr int kProfRing = 64;
struct Profile {
  bool on = false, created = false;
  bool last_only = false;   // record the last kernel's pair only (fewer markers in the stream)
  int calls = 0;   // prefill calls recorded since profiling was enabled
  hipEvent_t beg[kProfRing][STILL_PROFILE_SLOTS], end[kProfRing][STILL_PROFILE_SLOTS];
};
thread_local Profile g_prof;
const char* const kSlotNames[STILL_PROFILE_SLOTS] = {"transpose_v", "transpose_w", "score_select", "gather",
                                                     "keep_mask",   "la_states",   "la_prefix",    "sparse_attn_merge"};

void prof_begin(int slot, hipStream_t stream) {
  if (!g_prof.on || (g_prof.last_only && slot != STILL_PROFILE_SLOTS - 1)) return;
  if (!g_prof.created) {
    for (int r = 0; r < kProfRing; ++r)
      for (int i = 0; i < STILL_PROFILE_SLOTS; ++i)
        if (hipEventCreate(&g_prof.beg[r][i]) != hipSuccess || hipEventCreate(&g_prof.end[r][i]) != hipSuccess) {
          g_prof.on = false;
          return;
        }
    g_prof.created = true;
  }
  (void)hipEventRecord(g_prof.beg[g_prof.calls % kProfRing][slot], stream);
}

void prof_end(int slot, hipStream_t stream) {
  if (!g_prof.on || !g_prof.created || (g_prof.last_only && slot != STILL_PROFILE_SLOTS - 1)) return;
  (void)hipEventRecord(g_prof.end[g_prof.calls % kProfRing][slot], stream);
  if (slot == STILL_PROFILE_SLOTS - 1) ++g_prof.calls;
}

// The layout kernels (transposes of v and of the projection weights) do not depend on the scores and are bound by
// memory, the score kernel by the vector ALU: they run side by side, the layout kernels on a second stream of
// default priority that forks from the caller's stream at the start of the call and joins it again before the
// first kernel that reads their output.  One side stream and one event pair per host thread and device.
struct SideStream {
  bool ok = false;
  int dev = -1;
  hipStream_t s = nullptr;
  hipEvent_t fork = nullptr, join = nullptr;
};
thread_local SideStream g_side;

SideStream* side_stream() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return nullptr;
  if (g_side.ok && g_side.dev == dev) return &g_side;
  if (g_side.ok) {   // the thread moved to another device: drop the old objects
    (void)hipEventDestroy(g_side.fork);
    (void)hipEventDestroy(g_side.join);
    (void)hipStreamDestroy(g_side.s);
    g_side.ok = false;
  }
  if (hipStreamCreateWithFlags(&g_side.s, hipStreamNonBlocking) != hipSuccess) return nullptr;
  if (hipEventCreateWithFlags(&g_side.fork, hipEventDisableTiming) != hipSuccess) {
    (void)hipStreamDestroy(g_side.s);
    return nullptr;
  }
  if (hipEventCreateWithFlags(&g_side.join, hipEventDisableTiming) != hipSuccess) {
    (void)hipEventDestroy(g_side.fork);
    (void)hipStreamDestroy(g_side.s);
    return nullptr;
  }
  g_side.dev = dev;
  g_side.ok = true;
  return &g_side;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline size_t esize(int dtype) { return dtype == STILL_BF16 ? 2 : 4; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
inline int retained_budget(const still_params_t* p) { return p->max_retained > 0 ? p->max_retained : still::kNoBudget; }

still_status_t validate_params(const still_params_t* p, bool need_n) {
  if (p == nullptr) return fail(STILL_ERR_INVALID_ARG, "params is NULL");
  if (p->dtype != STILL_F32 && p->dtype != STILL_BF16) return fail(STILL_ERR_INVALID_ARG, "dtype %d unknown", p->dtype);
  if (p->B < 1 || p->Hq < 1 || p->Hkv < 1) return fail(STILL_ERR_INVALID_ARG, "B, Hq, Hkv must be >= 1");
  if (need_n && p->N < 1) return fail(STILL_ERR_INVALID_ARG, "N must be >= 1 (got %d)", p->N);
  if (p->lambda < 0 || p->lambda > p->C) return fail(STILL_ERR_INVALID_ARG, "lambda %d outside [0, C=%d]", p->lambda, p->C);
  if (p->W < 1) return fail(STILL_ERR_INVALID_ARG, "W must be >= 1");
  if (p->gate_activation != 0 && p->gate_activation != 1)
    return fail(STILL_ERR_INVALID_ARG, "gate_activation %d unknown (0: none, 1: sigmoid)", p->gate_activation);
  if (p->budget_policy != 0 && p->budget_policy != 1)
    return fail(STILL_ERR_INVALID_ARG, "budget_policy %d unknown (0: stop adding, 1: evict the lowest score)",
                p->budget_policy);
  if (p->budget_policy == 1) {
    if (p->max_retained < 1) return fail(STILL_ERR_INVALID_ARG, "budget_policy 1 needs max_retained >= 1");
    if (p->shared_selection) return fail(STILL_ERR_UNSUPPORTED, "budget_policy 1 is defined per query head");
    if (p->max_retained > still::kMaxEvictBudget)
      return fail(STILL_ERR_UNSUPPORTED, "budget_policy 1: max_retained %d > %d", p->max_retained,
                  still::kMaxEvictBudget);
  }
  if (!(p->eps > 0.f)) return fail(STILL_ERR_INVALID_ARG, "eps must be > 0");
  if (!(p->scale > 0.f)) return fail(STILL_ERR_INVALID_ARG, "scale must be > 0");
  if (p->Hq > still::kMaxHq) return fail(STILL_ERR_UNSUPPORTED, "Hq %d > %d", p->Hq, still::kMaxHq);
  if (p->kv_head_of_q == nullptr) {
    if (p->Hq % p->Hkv != 0) return fail(STILL_ERR_INVALID_ARG, "Hq %% Hkv != 0 and no kv_head_of_q map given");
  } else {
    for (int h = 0; h < p->Hq; ++h)
      if (p->kv_head_of_q[h] < 0 || p->kv_head_of_q[h] >= p->Hkv)
        return fail(STILL_ERR_INVALID_ARG, "kv_head_of_q[%d] = %d outside [0, Hkv)", h, p->kv_head_of_q[h]);
  }
  if (p->d != 64 && p->d != 128) return fail(STILL_ERR_UNSUPPORTED, "d = %d (supported: 64, 128)", p->d);
  if (p->d_f != p->d) return fail(STILL_ERR_UNSUPPORTED, "d_f = %d (supported: d_f == d)", p->d_f);
  if (p->C != 64 && p->C != 128) return fail(STILL_ERR_UNSUPPORTED, "C = %d (supported: 64, 128)", p->C);
  if (p->W > 256 || p->W > 4 * p->C)   // nine band tiles at most; a decode state keeps the last 4 C tokens
    return fail(STILL_ERR_UNSUPPORTED, "W = %d (supported: 1..min(256, 4 C))", p->W);
  if (need_n && (int64_t)p->N > (int64_t)1 << 24) return fail(STILL_ERR_UNSUPPORTED, "N = %d too large", p->N);
  return STILL_OK;
}

// What the two side entry points (global score, selection overlap) need from the problem description: they do not
// touch the linear branch, so its restrictions (d_f, W, the fp32 LDS budget) do not apply to them.
still_status_t validate_score_params(const still_params_t* p, bool with_qk) {
  if (p == nullptr) return fail(STILL_ERR_INVALID_ARG, "params is NULL");
  if (p->B < 1 || p->Hq < 1 || p->N < 1) return fail(STILL_ERR_INVALID_ARG, "B, Hq, N must be >= 1");
  if ((int64_t)p->N > (int64_t)1 << 24) return fail(STILL_ERR_UNSUPPORTED, "N = %d too large", p->N);
  if (p->Hq > still::kMaxHq) return fail(STILL_ERR_UNSUPPORTED, "Hq %d > %d", p->Hq, still::kMaxHq);
  if (with_qk) {
    if (p->dtype != STILL_F32 && p->dtype != STILL_BF16) return fail(STILL_ERR_INVALID_ARG, "dtype %d unknown", p->dtype);
    if (p->Hkv < 1) return fail(STILL_ERR_INVALID_ARG, "Hkv must be >= 1");
    if (!(p->eps > 0.f)) return fail(STILL_ERR_INVALID_ARG, "eps must be > 0");
    if (!(p->scale > 0.f)) return fail(STILL_ERR_INVALID_ARG, "scale must be > 0");
    if (p->d != 64 && p->d != 128) return fail(STILL_ERR_UNSUPPORTED, "d = %d (supported: 64, 128)", p->d);
    if (p->kv_head_of_q == nullptr) {
      if (p->Hq % p->Hkv != 0) return fail(STILL_ERR_INVALID_ARG, "Hq %% Hkv != 0 and no kv_head_of_q map given");
    } else {
      for (int h = 0; h < p->Hq; ++h)
        if (p->kv_head_of_q[h] < 0 || p->kv_head_of_q[h] >= p->Hkv)
          return fail(STILL_ERR_INVALID_ARG, "kv_head_of_q[%d] = %d outside [0, Hkv)", h, p->kv_head_of_q[h]);
    }
  } else {
    if (p->C < 1 || p->C > 128) return fail(STILL_ERR_UNSUPPORTED, "C = %d (supported by the overlap count: 1..128)", p->C);
    if (p->lambda < 0 || p->lambda > p->C) return fail(STILL_ERR_INVALID_ARG, "lambda %d outside [0, C=%d]", p->lambda, p->C);
  }
  return STILL_OK;
}

still_status_t validate_strides(const still_params_t* p, bool with_g) {
  const int64_t unit = 16 / (int64_t)esize(p->dtype);
  const int64_t s[] = {p->q_sb, p->q_st, p->q_sh, p->k_sb, p->k_st, p->k_sh, p->v_sb, p->v_st, p->v_sh,
                       p->o_sb, p->o_st, p->o_sh};
  for (int64_t x : s)
    if (x < 0 || x % unit != 0) return fail(STILL_ERR_INVALID_ARG, "stride %lld is negative or not a multiple of 16 bytes", (long long)x);
  if (p->q_st < p->d || p->k_st < p->d || p->v_st < p->d || p->o_st < p->d)
    return fail(STILL_ERR_INVALID_ARG, "token stride smaller than d");
  if (with_g) {
    const int64_t gs[] = {p->g_sb, p->g_st, p->g_sh};
    for (int64_t x : gs)
      if (x < 0 || x % unit != 0) return fail(STILL_ERR_INVALID_ARG, "gate stride %lld invalid", (long long)x);
  }
  return STILL_OK;
}

void fill_map(const still_params_t* p, still::HeadMap* m) {
  for (int h = 0; h < still::kMaxHq; ++h) m->kv[h] = 0;
  for (int h = 0; h < p->Hq; ++h) m->kv[h] = p->kv_head_of_q ? p->kv_head_of_q[h] : h / (p->Hq / p->Hkv);
}

void compute_layout(const still_params_t* p, still_ws_layout_t* L) {
  const size_t es = esize(p->dtype);
  const int64_t B = p->B, N = p->N, Hq = p->Hq, Hkv = p->Hkv, d = p->d, df = p->d_f;
  const int64_t nc = (N + p->C - 1) / p->C, ncf = N / p->C;
  const int64_t npad = (N + 127) / 128 * 128;
  const bool evict = p->budget_policy == 1;   // then the retained rows of the workspace are ALL offers, under masks
  const int64_t cap = ((int64_t)still::retained_rows((int)ncf, p->lambda, evict ? still::kNoBudget : retained_budget(p)) + 63) / 64 * 64;
  int64_t G = (nc * B * Hq + 255) / 256;   // one workgroup per CU at the size of the chip
  if (G < 2) G = 2;
  if (G > nc) G = nc;
  // the scan walks in rounds of RT tokens: a segment is a whole number of rounds
  const int64_t per_round = still::la_round_tokens((int)es, (int)d) / p->C;
  if (per_round > 1) G = (G + per_round - 1) / per_round * per_round;
  const int64_t nseg = (nc + G - 1) / G;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off = align_up(off + (bytes ? bytes : 16), 256);
    return o;
  };
  L->score = take((size_t)B * Hq * N * 4);
  L->sel = take((size_t)B * Hq * ncf * p->lambda * 4);
  L->vt = take((size_t)B * Hkv * d * npad * es);
  L->kret = take((size_t)B * Hq * cap * d * es);
  L->vrett = take((size_t)B * Hq * cap * d * es);
  L->wqt = take((size_t)Hq * df * d * es);
  L->wkf = take((size_t)Hq * df * d * es);
  L->seg = take((size_t)B * Hq * nseg * (2 * df * (d + 1)) * 4);
  L->snap = take((size_t)B * Hq * nc * d * (2 * df) * es);
  L->zsnap = take((size_t)B * Hq * nc * (2 * df) * 4);
  L->pimg = take((size_t)B * Hq * nseg * d * (2 * df) * es);
  L->zpre = take((size_t)B * Hq * nseg * (2 * df) * 4);
  L->kmask = take((size_t)B * Hq * ncf * (p->C / 32) * 4);
  L->n_la = take(p->emit_terms ? (size_t)B * Hq * N * d * 4 : 0);
  L->d_la = take(p->emit_terms ? (size_t)B * Hq * N * 4 : 0);
  L->vfr = take((size_t)B * Hkv * d * npad * es);
  const size_t M = evict ? (size_t)p->max_retained : 0;
  L->ev_src = take(evict ? (size_t)B * Hq * N * 4 : 0);
  L->ev_alive = take(evict ? (size_t)B * Hq * nc * (cap / 64) * 8 : 0);
  L->ev_fin = take(evict ? (size_t)B * Hq * (2 * M + 1) * 4 : 0);
  L->ev_vfr = take(evict ? (size_t)B * Hq * d * npad * es : 0);
  L->lse = take((size_t)B * Hq * N * 4);
  L->total = off;
  L->n_pad = (int32_t)npad;
  L->cap = (int32_t)cap;
  L->nseg = (int32_t)nseg;
  L->seg_chunks = (int32_t)G;
}

still_status_t validate_state_params(const still_params_t* p) {
  still_status_t st = validate_params(p, false);
  if (st != STILL_OK) return st;
  if (p->max_tokens < 1) return fail(STILL_ERR_INVALID_ARG, "max_tokens must be >= 1 for a decode state");
  if ((int64_t)p->max_tokens > (int64_t)1 << 24) return fail(STILL_ERR_UNSUPPORTED, "max_tokens too large");
  return STILL_OK;
}

void compute_state_layout(const still_params_t* p, still_state_layout_t* L) {
  const size_t es = esize(p->dtype);
  const int64_t B = p->B, Hq = p->Hq, Hkv = p->Hkv, d = p->d, df = p->d_f;
  const int64_t nch = ((int64_t)p->max_tokens + p->C - 1) / p->C;
  const int64_t cap = ((int64_t)still::retained_rows((int)nch, p->lambda, retained_budget(p)) + 63) / 64 * 64 + 64;
  const int64_t R = 4 * (int64_t)p->C;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off = align_up(off + (bytes ? bytes : 16), 256);
    return o;
  };
  const int64_t slices = p->shared_selection ? Hkv : Hq;   // group-shared selection: retained rows once per kv head
  L->S = take((size_t)B * Hq * (2 * df * (d + 1)) * 4);
  L->kret = take((size_t)B * slices * cap * d * es);
  L->vret = take((size_t)B * slices * cap * d * es);
  L->sel = take((size_t)B * Hq * nch * p->lambda * 4);
  L->kring = take((size_t)B * Hkv * R * d * es);
  L->vring = take((size_t)B * Hkv * R * d * es);
  L->score = take((size_t)B * Hq * R * 4);
  L->part = take((size_t)B * Hq * 32 * (d + 2) * 4);
  L->ret_score = take(p->budget_policy == 1 ? (size_t)B * Hq * cap * 4 : 0);
  L->ret_tok = take(p->budget_policy == 1 ? (size_t)B * Hq * cap * 4 : 0);
  L->total = off;
  L->cap = (int32_t)cap;
  L->R = (int32_t)R;
  L->n_chunks = (int32_t)nch;
}

}  // namespace

extern "C" {

// 0.3.0: budget_policy in the params, more regions in both layouts
int32_t still_version(void) { return 400; }   // 0.4.0: backward pass, attention map, rotary pre-pass

const char* still_last_error(void) { return g_err; }

still_status_t still_fwd_workspace_layout(const still_params_t* p, still_ws_layout_t* layout) {
  if (layout == nullptr) return fail(STILL_ERR_INVALID_ARG, "layout is NULL");
  still_status_t st = validate_params(p, true);
  if (st != STILL_OK) return st;
  compute_layout(p, layout);
  return STILL_OK;
}

size_t still_fwd_workspace_bytes(const still_params_t* p) {
  still_ws_layout_t L;
  if (still_fwd_workspace_layout(p, &L) != STILL_OK) return 0;
  return L.total;
}

}  // extern "C"

namespace {

// Scratch of the allocation-free entry point: one fixed array in device memory per GPU, part of the library's code
// object (it exists from the moment the library is loaded on a device until the process ends).  In host code the
// array's name is only a handle for hipGetSymbolAddress; the address each device holds it at is looked up once per
// device and kept here.
constexpr size_t kStaticWorkspaceBytes = (size_t)STILL_STATIC_WORKSPACE_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticWorkspaceBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

still_status_t static_workspace(void** ptr) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(STILL_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(STILL_ERR_UNSUPPORTED, "device index %d outside [0, %d)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* sym = nullptr;
    e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
    if (e != hipSuccess || sym == nullptr)
      return fail(STILL_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
    g_scratch_ptr[dev] = sym;
  }
  *ptr = g_scratch_ptr[dev];
  return STILL_OK;
}

// The prefill behind both entry points.  two_streams: run the layout kernels on the library's helper stream (created
// on first use) and record timing events if profiling is on; without it everything is enqueued on `stream` and no
// host or device object is created.
still_status_t fwd_impl(const still_params_t* p, const void* q, const void* k, const void* v,
                        const void* g, const void* Wq, const void* bq, const void* Wk,
                        const void* bk, void* out, float* score_out, int32_t* sel_idx,
                        int32_t sel_idx_is_input, void* state_out, void* workspace,
                        size_t workspace_bytes, void* stream_v, bool two_streams, bool static_ws) {
  still_status_t st = validate_params(p, true);
  if (st != STILL_OK) return st;
  st = validate_strides(p, g != nullptr);
  if (st != STILL_OK) return st;
  if (p->budget_policy != 0) {
    if (sel_idx_is_input || static_ws)
      return fail(STILL_ERR_UNSUPPORTED, "budget_policy 1 with injected indices or the built-in scratch array");
    const int64_t offers = (int64_t)(p->N / p->C) * p->lambda;
    if (offers > still::kMaxEvictOffers)
      return fail(STILL_ERR_UNSUPPORTED, "budget_policy 1: %lld offers per head > %d", (long long)offers,
                  still::kMaxEvictOffers);
  }
  if (!q || !k || !v || !Wq || !Wk || !out || (!workspace && !static_ws))
    return fail(STILL_ERR_INVALID_ARG, "a required pointer (q, k, v, Wq, Wk, out, workspace) is NULL");
  const void* ptrs[] = {q, k, v, g, Wq, bq, Wk, bk, out, score_out, sel_idx, workspace};
  for (const void* x : ptrs)
    if (x != nullptr && !aligned16(x)) return fail(STILL_ERR_INVALID_ARG, "pointer %p is not 16-byte aligned", x);
  if (p->seq_len != nullptr && (reinterpret_cast<uintptr_t>(p->seq_len) & 3) != 0)
    return fail(STILL_ERR_INVALID_ARG, "seq_len is not 4-byte aligned");
  if (sel_idx_is_input && sel_idx == nullptr && p->lambda > 0 && p->N >= p->C)
    return fail(STILL_ERR_INVALID_ARG, "sel_idx_is_input set but sel_idx is NULL");
  if (state_out != nullptr) {
    if (!aligned16(state_out)) return fail(STILL_ERR_INVALID_ARG, "state_out is not 16-byte aligned");
    if (p->max_tokens < p->N) return fail(STILL_ERR_INVALID_ARG, "state_out needs max_tokens >= N");
    if ((int64_t)p->max_tokens > (int64_t)1 << 24) return fail(STILL_ERR_UNSUPPORTED, "max_tokens too large");
    // the state carries the scores of the local span; with injected indices they are only computed on request
    if (sel_idx_is_input && score_out == nullptr)
      return fail(STILL_ERR_INVALID_ARG,
                  "state_out needs the scores: do not combine it with sel_idx_is_input unless score_out is given");
  }
  still_ws_layout_t L;
  compute_layout(p, &L);
  if (static_ws) {
    if (L.total > kStaticWorkspaceBytes)
      return fail(STILL_ERR_WORKSPACE_TOO_SMALL,
                  "this problem needs %zu bytes of workspace, the built-in scratch array holds %zu: use "
                  "still_hybrid_attn_fwd with a caller-owned workspace", L.total, kStaticWorkspaceBytes);
    st = static_workspace(&workspace);
    if (st != STILL_OK) return st;
  } else if (workspace_bytes < L.total) {
    return fail(STILL_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, L.total);
  }
  // timing events are host objects created on demand: the allocation-free entry point records none
  struct ProfPause {
    bool was;
    explicit ProfPause(bool pause) : was(g_prof.on) { if (pause) g_prof.on = false; }
    ~ProfPause() { g_prof.on = was; }
  } prof_pause(!two_streams);

  hipStream_t stream = static_cast<hipStream_t>(stream_v);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  const int B = p->B, N = p->N, d = p->d, C = p->C;
  const int nc = (N + C - 1) / C, ncf = N / C;
  still::HeadMap map;
  fill_map(p, &map);
  float* score = reinterpret_cast<float*>(ws + L.score);
  int32_t* sel = (sel_idx != nullptr) ? sel_idx : reinterpret_cast<int32_t*>(ws + L.sel);
  const bool have_sel = p->lambda > 0 && ncf > 0;
  hipError_t e;

  // layout preparation, on the side stream (the caller's stream if it could not be created)
  SideStream* side = two_streams ? side_stream() : nullptr;
  hipStream_t s2 = stream;
  if (side != nullptr) {
    if (hipEventRecord(side->fork, stream) == hipSuccess && hipStreamWaitEvent(side->s, side->fork, 0) == hipSuccess)
      s2 = side->s;
    else
      side = nullptr;
  }
  // From here on the helper stream may hold work that depends on the caller's stream.  A launch failure must not
  // leave it dangling (under stream capture an unjoined fork invalidates the capture): every error return below
  // goes through hip_fail, which joins the helper stream back into `stream` first.
  bool joined = false;
  auto join_side = [&]() -> hipError_t {
    if (side == nullptr || joined) return hipSuccess;
    joined = true;
    hipError_t je = hipEventRecord(side->join, s2);
    if (je == hipSuccess) je = hipStreamWaitEvent(stream, side->join, 0);
    return je;
  };
  auto hip_fail = [&](const char* what, hipError_t err) -> still_status_t {
    (void)join_side();
    return fail(STILL_ERR_HIP, "%s: %s", what, hipGetErrorString(err));
  };
  prof_begin(0, s2);
  const bool evict = p->budget_policy == 1;
  const int budget = evict ? still::kNoBudget : retained_budget(p);   // under eviction every chunk offers its lam best
  still::TransposeVArgs tv{v, p->v_sb, p->v_st, p->v_sh, ws + L.vt, evict ? nullptr : ws + L.vfr, N, L.n_pad, p->Hkv, d,
                           C, p->seq_len};
  if ((e = still::launch_transpose_v(tv, p->dtype, B, s2)) != hipSuccess)
    return hip_fail("transpose_v", e);
  prof_end(0, s2);
  prof_begin(1, s2);
  still::TransposeWArgs twq{Wq, ws + L.wqt, p->Hq, d, p->d_f, 0};   // rows of W_q^T: tiles of the query feature map
  still::TransposeWArgs twk{Wk, ws + L.wkf, p->Hq, d, p->d_f, 1};   // W_k^T in operand order: the key projection
  if ((e = still::launch_transpose_w(twq, p->dtype, s2)) != hipSuccess ||
      (e = still::launch_transpose_w(twk, p->dtype, s2)) != hipSuccess)
    return hip_fail("transpose_w", e);
  prof_end(1, s2);

  prof_begin(2, stream);
  // Self-Saliency Score + Top-lambda
  still::ScoreArgs sa{};
  sa.q = q; sa.k = k;
  sa.q_sb = p->q_sb; sa.q_st = p->q_st; sa.q_sh = p->q_sh;
  sa.k_sb = p->k_sb; sa.k_st = p->k_st; sa.k_sh = p->k_sh;
  sa.map = map;
  sa.N = N; sa.C = C; sa.W = p->W; sa.lam = p->lambda; sa.Hq = p->Hq; sa.ncf = ncf; sa.rcap = budget;
  sa.scale = p->scale; sa.eps = p->eps;
  sa.score = score;
  const bool group_sel = p->shared_selection != 0;
  sa.sel = (have_sel && !sel_idx_is_input && !group_sel) ? sel : nullptr;
  const bool need_scores = !sel_idx_is_input || score_out != nullptr;
  if (need_scores) {
    if ((e = still::launch_score(sa, p->dtype, d, B, nc, stream)) != hipSuccess)
      return hip_fail("score_select", e);
    if (have_sel && !sel_idx_is_input && group_sel) {
      sa.sel = sel;
      if ((e = still::launch_group_select(sa, B, p->Hkv, stream)) != hipSuccess)
        return hip_fail("group_select", e);
    }
    if (score_out != nullptr) {
      e = hipMemcpyAsync(score_out, score, (size_t)B * p->Hq * N * sizeof(float), hipMemcpyDeviceToDevice, stream);
      if (e != hipSuccess) return hip_fail("score copy", e);
    }
  }
  prof_end(2, stream);

  prof_begin(3, stream);
  // retained K/V of every full chunk
  still::GatherArgs ga{};
  ga.k = k; ga.v = v;
  ga.k_sb = p->k_sb; ga.k_st = p->k_st; ga.k_sh = p->k_sh;
  ga.v_sb = p->v_sb; ga.v_st = p->v_st; ga.v_sh = p->v_sh;
  ga.map = map;
  ga.sel = sel;
  ga.nsel = have_sel ? still::retained_rows(ncf, p->lambda, budget) : 0;
  ga.sel_stride = ncf * p->lambda;
  ga.C = C; ga.lam = p->lambda; ga.rcap = budget; ga.seq_len = p->seq_len;
  ga.cap = L.cap; ga.Hq = p->Hq; ga.d = d; ga.N = N;
  ga.kret = ws + L.kret; ga.vrett = ws + L.vrett;
  if ((e = still::launch_gather(ga, p->dtype, B, stream)) != hipSuccess)
    return hip_fail("gather", e);
  prof_end(3, stream);
  // everything below reads the transposed copies
  if ((e = join_side()) != hipSuccess) return hip_fail("side stream", e);

  // NP-Map of the keys + scan of the linear-attention state: per-chunk sums inside every segment, prefix over segments
  still::LaArgs la{};
  la.k = k;
  la.k_sb = p->k_sb; la.k_st = p->k_st; la.k_sh = p->k_sh;
  la.vfr = ws + L.vfr; la.wkf = ws + L.wkf; la.bk = bk;
  la.kmask = reinterpret_cast<const uint32_t*>(ws + L.kmask);
  la.map = map;
  la.N = N; la.Np = L.n_pad; la.C = C; la.Hq = p->Hq; la.Hkv = p->Hkv;
  la.nc = nc; la.ncf = ncf; la.seq_len = p->seq_len;
  la.seg_chunks = L.seg_chunks; la.nseg = L.nseg;
  la.seg = reinterpret_cast<float*>(ws + L.seg);
  la.snap = ws + L.snap;
  la.zsnap = reinterpret_cast<float*>(ws + L.zsnap);
  la.pimg = ws + L.pimg;
  la.zpre = reinterpret_cast<float*>(ws + L.zpre);
  still_state_layout_t SL{};
  unsigned char* stp = static_cast<unsigned char*>(state_out);
  if (state_out != nullptr) compute_state_layout(p, &SL);
  la.s_final = state_out != nullptr ? reinterpret_cast<float*>(stp + SL.S) : nullptr;
  prof_begin(4, stream);
  const bool plan = evict && have_sel;
  int32_t* fin_tok = reinterpret_cast<int32_t*>(ws + L.ev_fin);
  float* fin_score = reinterpret_cast<float*>(ws + L.ev_fin) + (size_t)B * p->Hq * (plan ? p->max_retained : 0);
  int32_t* fin_n = fin_tok + (size_t)2 * B * p->Hq * (plan ? p->max_retained : 0);
  if (plan) {
    // which offers are retained for which rows, and which token every position carries into the state scan
    still::EvictPlanArgs ep{};
    ep.score = score; ep.sel = sel;
    ep.src = reinterpret_cast<int32_t*>(ws + L.ev_src); ep.alive = ws + L.ev_alive;
    ep.fin_tok = fin_tok; ep.fin_score = fin_score; ep.fin_n = fin_n;
    ep.seq_len = p->seq_len;
    ep.N = N; ep.C = C; ep.lam = p->lambda; ep.M = p->max_retained; ep.Hq = p->Hq; ep.ncf_all = ncf; ep.nc_all = nc;
    ep.AW = L.cap / 64;
    if ((e = still::launch_evict_plan(ep, B, stream)) != hipSuccess) return hip_fail("evict_plan", e);
    still::VfrGatherArgs vg{};
    vg.v = v; vg.v_sb = p->v_sb; vg.v_st = p->v_st; vg.v_sh = p->v_sh;
    vg.src = ep.src; vg.vfr = ws + L.ev_vfr; vg.map = map; vg.seq_len = p->seq_len;
    vg.N = N; vg.Np = L.n_pad; vg.Hq = p->Hq; vg.d = d; vg.C = C;
    if ((e = still::launch_vfr_gather(vg, p->dtype, B, stream)) != hipSuccess) return hip_fail("vfr_gather", e);
    la.src = ep.src;
    la.vfr = ws + L.ev_vfr;
  } else {   // (also budget_policy 1 with lambda = 0 or without a full chunk: nothing is ever offered)
    still::KeepMaskArgs km{sel, reinterpret_cast<uint32_t*>(ws + L.kmask), p->Hq, ncf, C, have_sel ? p->lambda : 0,
                           retained_budget(p)};
    if ((e = still::launch_keep_mask(km, B, stream)) != hipSuccess)
      return hip_fail("keep_mask", e);
  }
  prof_end(4, stream);
  prof_begin(5, stream);
  if ((e = still::launch_la_states(la, p->dtype, d, B, stream)) != hipSuccess)
    return hip_fail("la_states", e);
  prof_end(5, stream);
  prof_begin(6, stream);
  if ((e = still::launch_la_prefix(la, p->dtype, d, B, stream)) != hipSuccess)
    return hip_fail("la_prefix", e);
  prof_end(6, stream);

  prof_begin(7, stream);
  // sparse softmax branch, the rows' linear terms, merge
  still::SaArgs sx{};
  sx.q = q; sx.k = k;
  sx.q_sb = p->q_sb; sx.q_st = p->q_st; sx.q_sh = p->q_sh;
  sx.k_sb = p->k_sb; sx.k_st = p->k_st; sx.k_sh = p->k_sh;
  sx.vt = ws + L.vt; sx.kret = ws + L.kret; sx.vrett = ws + L.vrett;
  sx.wqt = ws + L.wqt; sx.bq = bq;
  sx.g = g; sx.g_sb = p->g_sb; sx.g_st = p->g_st; sx.g_sh = p->g_sh; sx.gate_act = p->gate_activation != 0;
  sx.snap = la.snap; sx.zsnap = la.zsnap; sx.nc = nc;
  sx.pimg = la.pimg; sx.zpre = la.zpre; sx.seg_chunks = L.seg_chunks; sx.nseg = L.nseg;
  sx.n_la_out = p->emit_terms ? reinterpret_cast<float*>(ws + L.n_la) : nullptr;
  sx.d_la_out = p->emit_terms ? reinterpret_cast<float*>(ws + L.d_la) : nullptr;
  sx.lse = reinterpret_cast<float*>(ws + L.lse);
  sx.out = out; sx.o_sb = p->o_sb; sx.o_st = p->o_st; sx.o_sh = p->o_sh;
  sx.map = map;
  sx.N = N; sx.Np = L.n_pad; sx.C = C; sx.lam = have_sel ? p->lambda : 0; sx.Hq = p->Hq; sx.Hkv = p->Hkv;
  sx.rcap = budget; sx.seq_len = p->seq_len;
  if (plan) {
    sx.alive = ws + L.ev_alive;
    sx.AW = L.cap / 64;
  }
  sx.cap = L.cap; sx.ntiles = (N + still::kSaRows - 1) / still::kSaRows; sx.B_ = B;
  sx.scale = p->scale;
  if ((e = still::launch_sa(sx, p->dtype, d, B, stream)) != hipSuccess)
    return hip_fail("sparse_attention", e);
  prof_end(7, stream);

  // decode state standing after token N-1: (S, z) through chunk c_last-2 came from the linear pass above
  if (state_out != nullptr) {
    still::StateFillArgs sf{};
    sf.k = k; sf.v = v;
    sf.k_sb = p->k_sb; sf.k_st = p->k_st; sf.k_sh = p->k_sh;
    sf.v_sb = p->v_sb; sf.v_st = p->v_st; sf.v_sh = p->v_sh;
    sf.score = score; sf.sel = sel; sf.map = map;
    sf.kret = stp + SL.kret; sf.vret = stp + SL.vret;
    sf.sel_state = reinterpret_cast<int32_t*>(stp + SL.sel);
    sf.kring = stp + SL.kring; sf.vring = stp + SL.vring;
    sf.score_ring = reinterpret_cast<float*>(stp + SL.score);
    sf.N = N; sf.R = SL.R; sf.Hq = p->Hq; sf.Hkv = p->Hkv; sf.d = d; sf.lam = have_sel ? p->lambda : 0;
    sf.cap = SL.cap; sf.ncf = ncf; sf.nchunks = SL.n_chunks; sf.rcap = budget;
    sf.shared = p->shared_selection != 0; sf.C = C; sf.seq_len = p->seq_len;
    sf.lists_only = plan;      // under eviction the lists are the offers and the rows come from the plan's last set
    const int n_routed = nc >= 2 ? nc - 2 : 0;
    if ((e = still::launch_state_fill(sf, p->dtype, B, n_routed, stream)) != hipSuccess)
      return hip_fail("state_fill", e);
    if (plan) {
      still::StateFillEvictArgs fe{};
      fe.k = k; fe.v = v;
      fe.k_sb = p->k_sb; fe.k_st = p->k_st; fe.k_sh = p->k_sh;
      fe.v_sb = p->v_sb; fe.v_st = p->v_st; fe.v_sh = p->v_sh;
      fe.fin_tok = fin_tok; fe.fin_score = fin_score; fe.fin_n = fin_n;
      fe.kret = stp + SL.kret; fe.vret = stp + SL.vret;
      fe.ret_score = reinterpret_cast<float*>(stp + SL.ret_score);
      fe.ret_tok = reinterpret_cast<int32_t*>(stp + SL.ret_tok);
      fe.map = map; fe.M = p->max_retained; fe.cap = SL.cap; fe.Hq = p->Hq; fe.d = d;
      if ((e = still::launch_state_fill_evict(fe, p->dtype, B, stream)) != hipSuccess)
        return hip_fail("state_fill_evict", e);
    }
  }
  g_err[0] = 0;
  return STILL_OK;
}

}  // namespace

extern "C" {

still_status_t still_hybrid_attn_fwd(const still_params_t* p, const void* q, const void* k, const void* v,
                                     const void* g, const void* Wq, const void* bq, const void* Wk,
                                     const void* bk, void* out, float* score_out, int32_t* sel_idx,
                                     int32_t sel_idx_is_input, void* state_out, void* workspace,
                                     size_t workspace_bytes, void* stream_v) {
  return fwd_impl(p, q, k, v, g, Wq, bq, Wk, bk, out, score_out, sel_idx, sel_idx_is_input, state_out, workspace,
                  workspace_bytes, stream_v, /*two_streams=*/true, /*static_ws=*/false);
}

still_status_t still_hybrid_attn_fwd_static(const still_params_t* p, const void* q, const void* k, const void* v,
                                            const void* g, const void* Wq, const void* bq, const void* Wk,
                                            const void* bk, void* out, float* score_out, int32_t* sel_idx,
                                            int32_t sel_idx_is_input, void* state_out, void* stream_v) {
  return fwd_impl(p, q, k, v, g, Wq, bq, Wk, bk, out, score_out, sel_idx, sel_idx_is_input, state_out, nullptr, 0,
                  stream_v, /*two_streams=*/false, /*static_ws=*/true);
}

void still_profile_enable(int32_t on) {
  g_prof.on = on != 0;
  g_prof.last_only = on == 2;
  g_prof.calls = 0;
}

still_status_t still_profile_read(float* ms, int32_t n) {
  if (ms == nullptr || n < 0) return fail(STILL_ERR_INVALID_ARG, "ms is NULL or n < 0");
  if (!g_prof.created || g_prof.calls == 0) return fail(STILL_ERR_STATE, "no profiled call recorded on this thread");
  const int last = (g_prof.calls - 1) % kProfRing;
  const int kept = g_prof.calls < kProfRing ? g_prof.calls : kProfRing;
  if (hipEventSynchronize(g_prof.end[last][STILL_PROFILE_SLOTS - 1]) != hipSuccess)
    return fail(STILL_ERR_HIP, "event synchronize failed");
  for (int i = 0; i < n && i < STILL_PROFILE_SLOTS; ++i) {
    double sum = 0.0;
    if (g_prof.last_only && i != STILL_PROFILE_SLOTS - 1) {
      ms[i] = 0.f;
      continue;
    }
    for (int c = 0; c < kept; ++c) {
      const int r = (g_prof.calls - 1 - c) % kProfRing;
      float t = 0.f;
      if (hipEventElapsedTime(&t, g_prof.beg[r][i], g_prof.end[r][i]) != hipSuccess)
        return fail(STILL_ERR_HIP, "event elapsed failed for slot %d", i);
      sum += t;
    }
    ms[i] = (float)(sum / kept);
  }
  return STILL_OK;
}

const char* still_profile_kernel_name(int32_t i) {
  return (i >= 0 && i < STILL_PROFILE_SLOTS) ? kSlotNames[i] : nullptr;
}

size_t still_state_bytes(const still_params_t* p) {
  still_state_layout_t L;
  if (still_state_layout(p, &L) != STILL_OK) return 0;
  return L.total;
}

still_status_t still_state_layout(const still_params_t* p, still_state_layout_t* layout) {
  if (layout == nullptr) return fail(STILL_ERR_INVALID_ARG, "layout is NULL");
  still_status_t st = validate_state_params(p);
  if (st != STILL_OK) return st;
  compute_state_layout(p, layout);
  return STILL_OK;
}

still_status_t still_state_init(const still_params_t* p, void* state, void* stream) {
  still_status_t st = validate_state_params(p);
  if (st != STILL_OK) return st;
  if (state == nullptr || !aligned16(state)) return fail(STILL_ERR_INVALID_ARG, "state is NULL or misaligned");
  still_state_layout_t L;
  compute_state_layout(p, &L);
  hipError_t e = still::launch_fill_zero(state, L.total, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail(STILL_ERR_HIP, "state_init: %s", hipGetErrorString(e));
  g_err[0] = 0;
  return STILL_OK;
}

}  // extern "C"

namespace {

// One decode step.  t_dev == nullptr: every sequence is at token t.  Otherwise t_dev holds each sequence's own
// token index on the device and t is an upper bound of them, used only to size the launch.
still_status_t decode_step(const still_params_t* p, void* state, int32_t t, const int32_t* t_dev, const void* q_t,
                           const void* k_t, const void* v_t, const void* g_t, const void* Wq, const void* bq,
                           const void* Wk, const void* bk, void* out_t, void* stream_v) {
  still_status_t st = validate_state_params(p);
  if (st != STILL_OK) return st;
  if (!state || !q_t || !k_t || !v_t || !Wq || !Wk || !out_t)
    return fail(STILL_ERR_INVALID_ARG, "a required pointer (state, q_t, k_t, v_t, Wq, Wk, out_t) is NULL");
  const void* ptrs[] = {state, q_t, k_t, v_t, g_t, Wq, bq, Wk, bk, out_t};
  for (const void* x : ptrs)
    if (x != nullptr && !aligned16(x)) return fail(STILL_ERR_INVALID_ARG, "pointer %p is not 16-byte aligned", x);
  if (t < 0 || t >= p->max_tokens)
    return fail(STILL_ERR_STATE, "token index %d outside the state capacity [0, %d)", t, p->max_tokens);
  still_state_layout_t L;
  compute_state_layout(p, &L);
  unsigned char* sp = static_cast<unsigned char*>(state);
  still::DecArgs a{};
  a.S = reinterpret_cast<float*>(sp + L.S);
  a.kret = sp + L.kret; a.vret = sp + L.vret;
  a.sel = reinterpret_cast<int32_t*>(sp + L.sel);
  a.kring = sp + L.kring; a.vring = sp + L.vring;
  a.score = reinterpret_cast<float*>(sp + L.score);
  a.part = reinterpret_cast<float*>(sp + L.part);
  a.q = q_t; a.k = k_t; a.v = v_t; a.g = g_t; a.wq = Wq; a.wk = Wk; a.bq = bq; a.bk = bk; a.out = out_t;
  fill_map(p, &a.map);
  a.B = p->B; a.Hq = p->Hq; a.Hkv = p->Hkv; a.C = p->C; a.W = p->W; a.lam = p->lambda;
  a.cap = L.cap; a.R = L.R; a.nchunks = L.n_chunks; a.t = t; a.rcap = retained_budget(p);
  a.scale = p->scale; a.eps = p->eps;
  a.tpos = t_dev; a.max_tokens = p->max_tokens; a.shared = p->shared_selection != 0;
  a.gate_act = p->gate_activation != 0;
  a.evict = p->budget_policy == 1;
  a.ret_score = reinterpret_cast<float*>(sp + L.ret_score);
  a.ret_tok = reinterpret_cast<int32_t*>(sp + L.ret_tok);
  const int c = t / p->C;
  const int rows = still::retained_rows(c >= 1 ? c - 1 : 0, p->lambda, a.rcap) + (t - (c >= 1 ? c - 1 : 0) * p->C + 1);
  const int units = p->B * (p->shared_selection ? p->Hkv : p->Hq);   // workgroups per split
  int nsplit = (1024 + units - 1) / units;
  if (nsplit > 32) nsplit = 32;
  if (nsplit > (rows + 63) / 64) nsplit = (rows + 63) / 64;
  if (nsplit < 1) nsplit = 1;
  a.nsplit = nsplit;
  // with per-sequence positions any sequence at a chunk start >= 2C routes; the others leave the kernel at once
  const bool route = t_dev != nullptr ? c >= 2 : ((t % p->C == 0) && c >= 2);
  hipError_t e = still::launch_decode_step(a, p->dtype, p->d, route, static_cast<hipStream_t>(stream_v));
  if (e != hipSuccess) return fail(STILL_ERR_HIP, "decode_step: %s", hipGetErrorString(e));
  g_err[0] = 0;
  return STILL_OK;
}

}  // namespace

extern "C" {

still_status_t still_hybrid_attn_decode_step(const still_params_t* p, void* state, int32_t t, const void* q_t,
                                             const void* k_t, const void* v_t, const void* g_t, const void* Wq,
                                             const void* bq, const void* Wk, const void* bk, void* out_t,
                                             void* stream_v) {
  return decode_step(p, state, t, nullptr, q_t, k_t, v_t, g_t, Wq, bq, Wk, bk, out_t, stream_v);
}

still_status_t still_hybrid_attn_decode_step_at(const still_params_t* p, void* state, const int32_t* t_dev,
                                                int32_t t_max, const void* q_t, const void* k_t, const void* v_t,
                                                const void* g_t, const void* Wq, const void* bq, const void* Wk,
                                                const void* bk, void* out_t, void* stream_v) {
  if (t_dev == nullptr) return fail(STILL_ERR_INVALID_ARG, "t_dev is NULL");
  if ((reinterpret_cast<uintptr_t>(t_dev) & 3) != 0) return fail(STILL_ERR_INVALID_ARG, "t_dev is not 4-byte aligned");
  return decode_step(p, state, t_max, t_dev, q_t, k_t, v_t, g_t, Wq, bq, Wk, bk, out_t, stream_v);
}

still_status_t still_global_score(const still_params_t* p, const void* q, const void* k, float* score_out,
                                  void* stream_v) {
  still_status_t st = validate_score_params(p, true);
  if (st != STILL_OK) return st;
  {
    const int64_t unit = 16 / (int64_t)esize(p->dtype);
    const int64_t s[] = {p->q_sb, p->q_st, p->q_sh, p->k_sb, p->k_st, p->k_sh};
    for (int64_t x : s)
      if (x < 0 || x % unit != 0) return fail(STILL_ERR_INVALID_ARG, "stride %lld is negative or not a multiple of 16 bytes", (long long)x);
    if (p->q_st < p->d || p->k_st < p->d) return fail(STILL_ERR_INVALID_ARG, "token stride smaller than d");
  }
  if (!q || !k || !score_out) return fail(STILL_ERR_INVALID_ARG, "a required pointer (q, k, score_out) is NULL");
  if (!aligned16(q) || !aligned16(k) || !aligned16(score_out))
    return fail(STILL_ERR_INVALID_ARG, "q, k and score_out must be 16-byte aligned");
  still::GScoreArgs ga{};
  ga.q = q; ga.k = k;
  ga.q_sb = p->q_sb; ga.q_st = p->q_st; ga.q_sh = p->q_sh;
  ga.k_sb = p->k_sb; ga.k_st = p->k_st; ga.k_sh = p->k_sh;
  fill_map(p, &ga.map);
  ga.N = p->N; ga.Hq = p->Hq; ga.scale = p->scale; ga.eps = p->eps; ga.score = score_out;
  hipError_t e = still::launch_global_score(ga, p->dtype, p->d, p->B, static_cast<hipStream_t>(stream_v));
  if (e != hipSuccess) return fail(STILL_ERR_HIP, "global_score: %s", hipGetErrorString(e));
  g_err[0] = 0;
  return STILL_OK;
}

still_status_t still_selection_overlap(const still_params_t* p, const float* score_a, const float* score_b,
                                       int32_t* overlap, void* stream_v) {
  still_status_t st = validate_score_params(p, false);
  if (st != STILL_OK) return st;
  if (!score_a || !score_b || !overlap) return fail(STILL_ERR_INVALID_ARG, "a required pointer (score_a, score_b, overlap) is NULL");
  if ((reinterpret_cast<uintptr_t>(score_a) & 3) || (reinterpret_cast<uintptr_t>(score_b) & 3) ||
      (reinterpret_cast<uintptr_t>(overlap) & 3))
    return fail(STILL_ERR_INVALID_ARG, "score_a, score_b and overlap must be 4-byte aligned");
  hipError_t e = still::launch_topk_overlap(score_a, score_b, overlap, p->N, p->C, p->lambda, p->Hq, p->B,
                                            static_cast<hipStream_t>(stream_v));
  if (e != hipSuccess) return fail(STILL_ERR_HIP, "selection_overlap: %s", hipGetErrorString(e));
  g_err[0] = 0;
  return STILL_OK;
}

}  // extern "C"

// ---------------------------------------------------------------------------------------------------------
// Backward pass of the prefill (the routing held fixed)
// ---------------------------------------------------------------------------------------------------------
namespace {

still_status_t validate_bwd_params(const still_params_t* p) {
  still_status_t st = validate_params(p, true);
  if (st != STILL_OK) return st;
  if (p->budget_policy != 0) return fail(STILL_ERR_UNSUPPORTED, "the backward pass does not cover budget_policy 1");
  if (p->seq_len != nullptr) return fail(STILL_ERR_UNSUPPORTED, "the backward pass does not cover right-padded batches");
  if (p->dtype == STILL_F32 && p->d != 64)
    return fail(STILL_ERR_UNSUPPORTED, "the backward pass in fp32 is built for d = 64 only");
  return STILL_OK;
}

void compute_bwd_layout(const still_params_t* p, still_bwd_ws_layout_t* L) {
  still_ws_layout_t F;
  compute_layout(p, &F);
  const size_t es = esize(p->dtype);
  const size_t U = (size_t)p->B * p->Hq, N = p->N, d = p->d, df = p->d_f, DP = 2 * df;
  const size_t nc = (N + p->C - 1) / p->C, rows = U * N, kvrows = (size_t)p->B * p->Hkv * N;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off = align_up(off + (bytes ? bytes : 16), 256);
    return o;
  };
  L->fwd = take(F.total);
  L->e_row = take(rows * 4);
  L->delta = take(rows * 4);
  L->ed = take(rows * 4);
  L->a = take(rows * d * es);
  L->phi_q = take(rows * DP * es);
  L->phi_k = take(rows * DP * es);
  L->uq = take(rows * df * 4);
  L->uk = take(rows * df * 4);
  L->stq = take(rows * 2 * 4);
  L->stk = take(rows * 2 * 4);
  L->nraw = take(rows * d * 4);
  L->gq = take(rows * DP * 4);
  L->dphi_k = take(rows * DP * 4);
  L->ds = take(U * nc * DP * d * es);
  L->dz = take(U * nc * DP * 4);
  L->dfq = take(rows * df * es);
  L->dfk = take(rows * df * es);
  L->dq32 = take(rows * d * 4);
  L->dk32 = take(kvrows * d * 4);
  L->dv32 = take(kvrows * d * 4);
  L->cxq = take(rows * 4);
  L->cxk = take(rows * 4);
  // transposed copies with a row stride that is no power of two: their readers fetch 16 bytes from each of 32 rows
  // at once, and rows a power of two apart would all fall into one memory channel
  const size_t npt = (size_t)F.n_pad + 64, capt = (size_t)F.cap + 64;
  L->qt = take(U * d * npt * es);
  L->dot = take(U * d * npt * es);
  L->kt = take((size_t)p->B * p->Hkv * d * npt * es);
  L->kret = take(F.cap ? U * capt * d * es : 0);
  L->krett = take(F.cap ? U * capt * d * es : 0);
  L->n_pad_t = (int32_t)npt;
  L->cap_t = (int32_t)(F.cap ? capt : 0);
  L->total = off;
}

still::GemmOperand operand(const void* base, int64_t s_b, int64_t s_h, int64_t s_c, int64_t s_r, int64_t s_k,
                           int kv = 0, int f32 = 0, int c_div = 1) {
  still::GemmOperand o;
  o.base = base; o.s_b = s_b; o.s_h = s_h; o.s_c = s_c; o.s_r = s_r; o.s_k = s_k;
  o.kv = kv; o.c_div = c_div; o.f32 = f32;
  return o;
}

still_status_t bwd_impl(const still_params_t* p, const void* q, const void* k, const void* v, const void* g,
                        const void* Wq, const void* bq, const void* Wk, const void* bk, const void* out,
                        const void* dout, const float* lse, const int32_t* sel_idx, void* dq, void* dk, void* dv,
                        void* dg, float* dWq, float* dbq, float* dWk, float* dbk, void* workspace,
                        size_t workspace_bytes, void* stream_v) {
  still_status_t st = validate_bwd_params(p);
  if (st != STILL_OK) return st;
  st = validate_strides(p, g != nullptr);
  if (st != STILL_OK) return st;
  if (!q || !k || !v || !Wq || !Wk || !out || !dout || !lse || !dq || !dk || !dv || !dWq || !dWk || !workspace)
    return fail(STILL_ERR_INVALID_ARG,
                "a required pointer (q, k, v, Wq, Wk, out, dout, lse, dq, dk, dv, dWq, dWk, workspace) is NULL");
  if ((g != nullptr) != (dg != nullptr)) return fail(STILL_ERR_INVALID_ARG, "dg must be given exactly when g is");
  if ((bq != nullptr) != (dbq != nullptr) || (bk != nullptr) != (dbk != nullptr))
    return fail(STILL_ERR_INVALID_ARG, "dbq / dbk must be given exactly when bq / bk are");
  const int B = p->B, N = p->N, d = p->d, C = p->C, F = p->d_f, DP = 2 * F, Hq = p->Hq, Hkv = p->Hkv;
  const int nc = (N + C - 1) / C, ncf = N / C, U = B * Hq;
  const bool have_sel = p->lambda > 0 && ncf > 0;
  if (have_sel && sel_idx == nullptr)
    return fail(STILL_ERR_INVALID_ARG, "sel_idx (the forward pass's index lists) is NULL");
  const void* ptrs[] = {q, k, v, g, Wq, bq, Wk, bk, out, dout, lse, sel_idx, dq, dk, dv, dg, dWq, dbq, dWk, dbk, workspace};
  for (const void* x : ptrs)
    if (x != nullptr && !aligned16(x)) return fail(STILL_ERR_INVALID_ARG, "pointer %p is not 16-byte aligned", x);
  still_bwd_ws_layout_t BL;
  compute_bwd_layout(p, &BL);
  if (workspace_bytes < BL.total)
    return fail(STILL_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, BL.total);
  still_ws_layout_t L;
  compute_layout(p, &L);

  hipStream_t stream = static_cast<hipStream_t>(stream_v);
  unsigned char* bws = static_cast<unsigned char*>(workspace);
  unsigned char* ws = bws + BL.fwd;
  still::HeadMap map;
  fill_map(p, &map);
  const int dt = p->dtype;
  const int budget = retained_budget(p);
  hipError_t e;
  auto hip_fail = [&](const char* what, hipError_t err) -> still_status_t {
    return fail(STILL_ERR_HIP, "%s: %s", what, hipGetErrorString(err));
  };
  auto f32p = [&](size_t off) { return reinterpret_cast<float*>(bws + off); };

  // ---- outputs and accumulators that are added into
  if ((e = still::launch_fill_f32(dWq, (int64_t)Hq * d * F, 0.f, stream)) != hipSuccess ||
      (e = still::launch_fill_f32(dWk, (int64_t)Hq * d * F, 0.f, stream)) != hipSuccess ||
      (dbq && (e = still::launch_fill_f32(dbq, (int64_t)Hq * F, 0.f, stream)) != hipSuccess) ||
      (dbk && (e = still::launch_fill_f32(dbk, (int64_t)Hq * F, 0.f, stream)) != hipSuccess))
    return hip_fail("fill", e);

  // ---- the forward pass's linear-attention states, rebuilt from the index lists (same kernels as the prefill)
  still::TransposeVArgs tv{v, p->v_sb, p->v_st, p->v_sh, ws + L.vt, ws + L.vfr, N, L.n_pad, Hkv, d, C, nullptr};
  if ((e = still::launch_transpose_v(tv, dt, B, stream)) != hipSuccess) return hip_fail("transpose_v", e);
  still::TransposeWArgs twk{Wk, ws + L.wkf, Hq, d, F, 1};
  if ((e = still::launch_transpose_w(twk, dt, stream)) != hipSuccess) return hip_fail("transpose_w", e);
  still::KeepMaskArgs km{sel_idx, reinterpret_cast<uint32_t*>(ws + L.kmask), Hq, ncf, C, have_sel ? p->lambda : 0,
                         budget};
  if ((e = still::launch_keep_mask(km, B, stream)) != hipSuccess) return hip_fail("keep_mask", e);
  still::LaArgs la{};
  la.k = k;
  la.k_sb = p->k_sb; la.k_st = p->k_st; la.k_sh = p->k_sh;
  la.vfr = ws + L.vfr; la.wkf = ws + L.wkf; la.bk = bk;
  la.kmask = reinterpret_cast<const uint32_t*>(ws + L.kmask);
  la.map = map;
  la.N = N; la.Np = L.n_pad; la.C = C; la.Hq = Hq; la.Hkv = Hkv;
  la.nc = nc; la.ncf = ncf; la.seq_len = nullptr;
  la.seg_chunks = L.seg_chunks; la.nseg = L.nseg;
  la.seg = reinterpret_cast<float*>(ws + L.seg);
  la.snap = ws + L.snap;
  la.zsnap = reinterpret_cast<float*>(ws + L.zsnap);
  la.pimg = ws + L.pimg;
  la.zpre = reinterpret_cast<float*>(ws + L.zpre);
  la.s_final = nullptr;
  if ((e = still::launch_la_states(la, dt, d, B, stream)) != hipSuccess) return hip_fail("la_states", e);
  if ((e = still::launch_la_prefix(la, dt, d, B, stream)) != hipSuccess) return hip_fail("la_prefix", e);

  // ---- per-row scalars and A_t = E_t (gate_t * dy_t)
  still::BwdRowArgs ra{};
  ra.out = out; ra.dout = dout; ra.o_sb = p->o_sb; ra.o_st = p->o_st; ra.o_sh = p->o_sh;
  ra.g = g; ra.g_sb = p->g_sb; ra.g_st = p->g_st; ra.g_sh = p->g_sh; ra.gate_act = p->gate_activation != 0;
  ra.lse = lse; ra.e_row = f32p(BL.e_row); ra.delta = f32p(BL.delta); ra.ed = f32p(BL.ed);
  ra.A = bws + BL.a; ra.nraw = f32p(BL.nraw); ra.dg = dg;
  ra.U = U; ra.N = N; ra.Hq = Hq; ra.d = d;
  if ((e = still::launch_bwd_row_prep(ra, dt, stream)) != hipSuccess) return hip_fail("bwd_row_prep", e);

  // ---- softmax branch: dq (owned rows), dk / dv (atomic adds per key tile).  Its products over rows and keys read
  // transposed copies: q^T, dout^T, k^T of the sequence, and the retained keys both ways (the prefill's gather
  // kernel with k in the place of v too).
  still::TransposeVArgs tq{q, p->q_sb, p->q_st, p->q_sh, bws + BL.qt, nullptr, N, BL.n_pad_t, Hq, d, C, nullptr};
  still::TransposeVArgs td{dout, p->o_sb, p->o_st, p->o_sh, bws + BL.dot, nullptr, N, BL.n_pad_t, Hq, d, C, nullptr};
  still::TransposeVArgs tk{k, p->k_sb, p->k_st, p->k_sh, bws + BL.kt, nullptr, N, BL.n_pad_t, Hkv, d, C, nullptr};
  if ((e = still::launch_transpose_v(tq, dt, B, stream)) != hipSuccess ||
      (e = still::launch_transpose_v(td, dt, B, stream)) != hipSuccess ||
      (e = still::launch_transpose_v(tk, dt, B, stream)) != hipSuccess)
    return hip_fail("bwd transposes", e);
  still::GatherArgs ga{};
  ga.k = k; ga.v = k;
  ga.k_sb = p->k_sb; ga.k_st = p->k_st; ga.k_sh = p->k_sh;
  ga.v_sb = p->k_sb; ga.v_st = p->k_st; ga.v_sh = p->k_sh;
  ga.map = map;
  ga.sel = sel_idx;
  ga.nsel = have_sel ? still::retained_rows(ncf, p->lambda, budget) : 0;
  ga.sel_stride = ncf * p->lambda;
  ga.C = C; ga.lam = p->lambda; ga.rcap = budget; ga.seq_len = nullptr;
  ga.cap = BL.cap_t; ga.Hq = Hq; ga.d = d; ga.N = N;
  ga.kret = bws + BL.kret; ga.vrett = bws + BL.krett;
  if ((e = still::launch_gather(ga, dt, B, stream)) != hipSuccess) return hip_fail("bwd gather", e);
  still::BwdSaArgs sa{};
  sa.qt = bws + BL.qt; sa.dot = bws + BL.dot; sa.kt = bws + BL.kt; sa.kret = bws + BL.kret; sa.krett = bws + BL.krett;
  sa.Np = BL.n_pad_t; sa.cap = BL.cap_t;
  sa.q = q; sa.k = k; sa.v = v; sa.dout = dout;
  sa.q_sb = p->q_sb; sa.q_st = p->q_st; sa.q_sh = p->q_sh;
  sa.k_sb = p->k_sb; sa.k_st = p->k_st; sa.k_sh = p->k_sh;
  sa.v_sb = p->v_sb; sa.v_st = p->v_st; sa.v_sh = p->v_sh;
  sa.o_sb = p->o_sb; sa.o_st = p->o_st; sa.o_sh = p->o_sh;
  sa.sel = sel_idx; sa.lse = lse; sa.delta = ra.delta;
  sa.dq32 = f32p(BL.dq32); sa.dk32 = f32p(BL.dk32); sa.dv32 = f32p(BL.dv32);
  sa.map = map;
  sa.N = N; sa.C = C; sa.lam = have_sel ? p->lambda : 0; sa.rcap = budget; sa.Hq = Hq; sa.Hkv = Hkv; sa.nc = nc;
  sa.sel_stride = ncf * p->lambda;
  sa.n_row_tiles = (N + 63) / 64;
  sa.n_ret_tiles = (still::retained_rows(nc >= 2 ? nc - 2 : 0, sa.lam, budget) + 63) / 64;
  sa.scale = p->scale;
  if ((e = still::launch_bwd_sa(sa, dt, d, B, stream)) != hipSuccess) return hip_fail("bwd_sparse_attention", e);

  // ---- NP-Map of q and k again: f = x W on the matrix core, then phi, u and the norms per token
  still::GemmArgs gm{};
  gm.Hq = Hq; gm.map = map;
  auto product = [&](const still::GemmOperand& A_, const still::GemmOperand& B_, float* Cp, int64_t c_b, int64_t c_h,
                     int64_t c_c, int64_t c_r, int c_kv, int M_, int Nn_, int K_, int m_total, int k_total, int mode,
                     int n_c, const still::GemmOperand* B2_ = nullptr) -> hipError_t {
    gm.A = A_; gm.B = B_; gm.C = Cp;
    gm.B2 = B2_ != nullptr ? *B2_ : still::GemmOperand{}; gm.c_b = c_b; gm.c_h = c_h; gm.c_c = c_c; gm.c_r = c_r; gm.c_kv = c_kv;
    gm.M = M_; gm.Nn = Nn_; gm.K = K_; gm.m_total = m_total; gm.k_total = k_total; gm.mode = mode;
    return still::launch_bgemm(gm, dt, U, n_c, stream);
  };
  const int64_t NF = (int64_t)N * F, NDP = (int64_t)N * DP, ND = (int64_t)N * d;
  const still::GemmOperand q_rows = operand(q, p->q_sb, p->q_sh, (int64_t)C * p->q_st, p->q_st, 1);
  const still::GemmOperand k_rows = operand(k, p->k_sb, p->k_sh, (int64_t)C * p->k_st, p->k_st, 1, 1);
  const still::GemmOperand v_rows = operand(v, p->v_sb, p->v_sh, (int64_t)C * p->v_st, p->v_st, 1, 1);
  const still::GemmOperand wq_fx = operand(Wq, 0, (int64_t)d * F, 0, 1, F);   // (n = feature, k = x)
  const still::GemmOperand wk_fx = operand(Wk, 0, (int64_t)d * F, 0, 1, F);
  const still::GemmOperand wq_xf = operand(Wq, 0, (int64_t)d * F, 0, F, 1);   // (n = x, k = feature)
  const still::GemmOperand wk_xf = operand(Wk, 0, (int64_t)d * F, 0, F, 1);
  if ((e = product(q_rows, wq_fx, f32p(BL.uq), Hq * NF, NF, (int64_t)C * F, F, 0, C, F, d, N, 0, 0, nc)) != hipSuccess ||
      (e = product(k_rows, wk_fx, f32p(BL.uk), Hq * NF, NF, (int64_t)C * F, F, 0, C, F, d, N, 0, 0, nc)) != hipSuccess)
    return hip_fail("bwd f = x W", e);
  still::BwdNpArgs nq{};
  nq.x = q; nq.x_sb = p->q_sb; nq.x_st = p->q_st; nq.x_sh = p->q_sh; nq.x_kv = 0;
  nq.bias = bq; nq.u = f32p(BL.uq); nq.st = f32p(BL.stq); nq.phi = bws + BL.phi_q; nq.kmask = nullptr;
  nq.dphi = f32p(BL.gq); nq.coef = ra.ed; nq.z1 = la.zsnap; nq.z2 = la.zpre;
  nq.df = bws + BL.dfq; nq.cx = f32p(BL.cxq);
  nq.map = map; nq.U = U; nq.N = N; nq.Hq = Hq; nq.Hkv = Hkv; nq.d = d; nq.F = F; nq.C = C; nq.nc = nc; nq.ncf = ncf;
  nq.nseg = L.nseg; nq.seg_chunks = L.seg_chunks;
  still::BwdNpArgs nk = nq;
  nk.x = k; nk.x_sb = p->k_sb; nk.x_st = p->k_st; nk.x_sh = p->k_sh; nk.x_kv = 1;
  nk.bias = bk; nk.u = f32p(BL.uk); nk.st = f32p(BL.stk); nk.phi = bws + BL.phi_k; nk.kmask = la.kmask;
  nk.dphi = f32p(BL.dphi_k); nk.coef = nullptr; nk.z1 = f32p(BL.dz); nk.z2 = nullptr;
  nk.df = bws + BL.dfk; nk.cx = f32p(BL.cxk);
  if ((e = still::launch_bwd_np(nq, dt, false, stream)) != hipSuccess ||
      (e = still::launch_bwd_np(nk, dt, false, stream)) != hipSuccess)
    return hip_fail("bwd_np_fwd", e);

  // ---- query side of the linear branch: phi_q S (for dg) and S A (for dphi_q), against both state images
  const still::GemmOperand phiq_rows = operand(bws + BL.phi_q, Hq * NDP, NDP, (int64_t)C * DP, DP, 1);
  const still::GemmOperand a_rows = operand(bws + BL.a, Hq * ND, ND, (int64_t)C * d, d, 1);
  const int64_t img = (int64_t)d * DP;
  const still::GemmOperand snap_xf = operand(la.snap, Hq * nc * img, nc * img, img, DP, 1);        // (n = x, k = f)
  const still::GemmOperand pimg_xf = operand(la.pimg, Hq * L.nseg * img, L.nseg * img, img, DP, 1, 0, 0, L.seg_chunks);
  const still::GemmOperand snap_fx = operand(la.snap, Hq * nc * img, nc * img, img, 1, DP);        // (n = f, k = x)
  const still::GemmOperand pimg_fx = operand(la.pimg, Hq * L.nseg * img, L.nseg * img, img, 1, DP, 0, 0, L.seg_chunks);
  if ((e = product(phiq_rows, snap_xf, f32p(BL.nraw), Hq * ND, ND, (int64_t)C * d, d, 0, C, d, DP, N, 0, 0, nc, &pimg_xf)) != hipSuccess ||
      (e = product(a_rows, snap_fx, f32p(BL.gq), Hq * NDP, NDP, (int64_t)C * DP, DP, 0, C, DP, d, N, 0, 0, nc, &pimg_fx)) != hipSuccess)
    return hip_fail("bwd query-side products", e);
  if (g != nullptr && (e = still::launch_bwd_dg(ra, dt, stream)) != hipSuccess) return hip_fail("bwd_dg", e);

  // ---- gradient of the states: the per-chunk contributions phi_q^T A summed over the chunks two and more ahead
  const still::GemmOperand phiq_ft = operand(bws + BL.phi_q, Hq * NDP, NDP, (int64_t)C * DP, 1, DP);   // (m = f, k = token)
  const still::GemmOperand a_xt = operand(bws + BL.a, Hq * ND, ND, (int64_t)C * d, 1, d);              // (n = x, k = token)
  const int64_t simg = (int64_t)DP * d;
  gm.A = phiq_ft; gm.B = a_xt; gm.B2 = still::GemmOperand{};
  gm.C = f32p(BL.ds);   // written in the storage type by the scan
  gm.c_b = Hq * nc * simg; gm.c_h = nc * simg; gm.c_c = simg; gm.c_r = d; gm.c_kv = 0;
  gm.M = DP; gm.Nn = d; gm.K = C; gm.m_total = 0; gm.k_total = N; gm.mode = 0;
  if ((e = still::launch_bgemm_revscan(gm, dt, U, nc, stream)) != hipSuccess)
    return hip_fail("bwd state gradient", e);
  still::BwdColsumArgs cz{bws + BL.phi_q, ra.ed, f32p(BL.dz), N, C, nc, DP, Hq, 0};
  if ((e = still::launch_bwd_colsum(cz, dt, U, stream)) != hipSuccess) return hip_fail("bwd_colsum", e);
  if ((e = still::launch_bwd_revcumsum(f32p(BL.dz), U, nc, DP, stream)) != hipSuccess)
    return hip_fail("bwd_revcumsum", e);

  // ---- key side: dphi_k = v dS^T (- dz, in the NP-Map kernel), dv += phi_k dS
  const still::GemmOperand ds_fx = operand(bws + BL.ds, Hq * nc * simg, nc * simg, simg, d, 1);   // (n = f, k = x)
  const still::GemmOperand ds_xf = operand(bws + BL.ds, Hq * nc * simg, nc * simg, simg, 1, d);   // (n = x, k = f)
  const still::GemmOperand phik_rows = operand(bws + BL.phi_k, Hq * NDP, NDP, (int64_t)C * DP, DP, 1);
  if ((e = product(v_rows, ds_fx, f32p(BL.dphi_k), Hq * NDP, NDP, (int64_t)C * DP, DP, 0, C, DP, d, N, 0, 0, nc)) != hipSuccess ||
      (e = product(phik_rows, ds_xf, f32p(BL.dv32), Hkv * ND, ND, (int64_t)C * d, d, 1, C, d, DP, N, 0, 2, nc)) != hipSuccess)
    return hip_fail("bwd key-side products", e);

  // ---- NP-Map backwards (df, and the |x| path of dx), then dx += df W^T and dW += x^T df
  if ((e = still::launch_bwd_np(nq, dt, true, stream)) != hipSuccess ||
      (e = still::launch_bwd_np(nk, dt, true, stream)) != hipSuccess)
    return hip_fail("bwd_np_bwd", e);
  const still::GemmOperand dfq_rows = operand(bws + BL.dfq, Hq * NF, NF, (int64_t)C * F, F, 1);
  const still::GemmOperand dfk_rows = operand(bws + BL.dfk, Hq * NF, NF, (int64_t)C * F, F, 1);
  if ((e = product(dfq_rows, wq_xf, f32p(BL.dq32), Hq * ND, ND, (int64_t)C * d, d, 0, C, d, F, N, 0, 1, nc)) != hipSuccess ||
      (e = product(dfk_rows, wk_xf, f32p(BL.dk32), Hkv * ND, ND, (int64_t)C * d, d, 1, C, d, F, N, 0, 2, nc)) != hipSuccess)
    return hip_fail("bwd dx += df W^T", e);
  const int KS = 256, nsplit = (N + KS - 1) / KS;   // tokens per split of the sum over tokens
  const still::GemmOperand q_xt = operand(q, p->q_sb, p->q_sh, (int64_t)KS * p->q_st, 1, p->q_st);       // (m = x, k = token)
  const still::GemmOperand k_xt = operand(k, p->k_sb, p->k_sh, (int64_t)KS * p->k_st, 1, p->k_st, 1);
  const still::GemmOperand dfq_ft = operand(bws + BL.dfq, Hq * NF, NF, (int64_t)KS * F, 1, F);           // (n = f, k = token)
  const still::GemmOperand dfk_ft = operand(bws + BL.dfk, Hq * NF, NF, (int64_t)KS * F, 1, F);
  if ((e = product(q_xt, dfq_ft, dWq, 0, (int64_t)d * F, 0, F, 0, d, F, KS, 0, N, 2, nsplit)) != hipSuccess ||
      (e = product(k_xt, dfk_ft, dWk, 0, (int64_t)d * F, 0, F, 0, d, F, KS, 0, N, 2, nsplit)) != hipSuccess)
    return hip_fail("bwd dW += x^T df", e);
  if (dbq != nullptr) {
    still::BwdColsumArgs cb{bws + BL.dfq, nullptr, dbq, N, C, nc, F, Hq, 1};
    if ((e = still::launch_bwd_colsum(cb, dt, U, stream)) != hipSuccess) return hip_fail("bwd db", e);
  }
  if (dbk != nullptr) {
    still::BwdColsumArgs cb{bws + BL.dfk, nullptr, dbk, N, C, nc, F, Hq, 1};
    if ((e = still::launch_bwd_colsum(cb, dt, U, stream)) != hipSuccess) return hip_fail("bwd db", e);
  }

  // ---- fp32 sums -> the caller's tensors
  still::BwdFinishArgs fq{f32p(BL.dq32), dq, q, p->q_sb, p->q_st, p->q_sh, f32p(BL.cxq), 0, map, B, Hq, Hq, N, d};
  still::BwdFinishArgs fk{f32p(BL.dk32), dk, k, p->k_sb, p->k_st, p->k_sh, f32p(BL.cxk), 1, map, B, Hkv, Hq, N, d};
  still::BwdFinishArgs fv{f32p(BL.dv32), dv, v, p->v_sb, p->v_st, p->v_sh, nullptr, 0, map, B, Hkv, Hq, N, d};
  if ((e = still::launch_bwd_finish(fq, dt, stream)) != hipSuccess ||
      (e = still::launch_bwd_finish(fk, dt, stream)) != hipSuccess ||
      (e = still::launch_bwd_finish(fv, dt, stream)) != hipSuccess)
    return hip_fail("bwd_finish", e);
  g_err[0] = 0;
  return STILL_OK;
}

}  // namespace

extern "C" {

size_t still_bwd_workspace_bytes(const still_params_t* p) {
  if (validate_bwd_params(p) != STILL_OK) return 0;
  still_bwd_ws_layout_t L;
  compute_bwd_layout(p, &L);
  return L.total;
}

still_status_t still_bwd_workspace_layout(const still_params_t* p, still_bwd_ws_layout_t* layout) {
  if (layout == nullptr) return fail(STILL_ERR_INVALID_ARG, "layout is NULL");
  still_status_t st = validate_bwd_params(p);
  if (st != STILL_OK) return st;
  compute_bwd_layout(p, layout);
  return STILL_OK;
}

}  // extern "C"

namespace {

// keep mask and the feature maps of q and k (phi_k zero for selected tokens), u and the norms, into a backward
// workspace: the common first part of the attention map and of its backward pass
still_status_t prepare_feature_maps(const still_params_t* p, const void* q, const void* k, const void* Wq,
                                    const void* bq, const void* Wk, const void* bk, const int32_t* sel_idx,
                                    unsigned char* bws, const still_bwd_ws_layout_t& BL, const still_ws_layout_t& L,
                                    const still::HeadMap& map, hipStream_t stream, still::BwdNpArgs* nq_out,
                                    still::BwdNpArgs* nk_out) {
  const int B = p->B, N = p->N, d = p->d, C = p->C, F = p->d_f, Hq = p->Hq;
  const int nc = (N + C - 1) / C, ncf = N / C, U = B * Hq;
  const bool have_sel = p->lambda > 0 && ncf > 0;
  const int dt = p->dtype;
  unsigned char* ws = bws + BL.fwd;
  hipError_t e;
  auto hip_fail = [&](const char* what, hipError_t err) -> still_status_t {
    return fail(STILL_ERR_HIP, "%s: %s", what, hipGetErrorString(err));
  };
  auto f32p = [&](size_t off) { return reinterpret_cast<float*>(bws + off); };
  still::KeepMaskArgs km{sel_idx, reinterpret_cast<uint32_t*>(ws + L.kmask), Hq, ncf, C, have_sel ? p->lambda : 0,
                         retained_budget(p)};
  if ((e = still::launch_keep_mask(km, B, stream)) != hipSuccess) return hip_fail("keep_mask", e);
  still::GemmArgs gm{};
  gm.Hq = Hq; gm.map = map;
  const int64_t NF = (int64_t)N * F;
  auto fxw = [&](const void* x, int64_t sb, int64_t st_, int64_t sh, int kv, const void* Wm, float* dst) -> hipError_t {
    gm.A = operand(x, sb, sh, (int64_t)C * st_, st_, 1, kv);
    gm.B = operand(Wm, 0, (int64_t)d * F, 0, 1, F);
    gm.B2 = still::GemmOperand{};
    gm.C = dst; gm.c_b = Hq * NF; gm.c_h = NF; gm.c_c = (int64_t)C * F; gm.c_r = F; gm.c_kv = 0;
    gm.M = C; gm.Nn = F; gm.K = d; gm.m_total = N; gm.k_total = 0; gm.mode = 0;
    return still::launch_bgemm(gm, dt, U, nc, stream);
  };
  if ((e = fxw(q, p->q_sb, p->q_st, p->q_sh, 0, Wq, f32p(BL.uq))) != hipSuccess ||
      (e = fxw(k, p->k_sb, p->k_st, p->k_sh, 1, Wk, f32p(BL.uk))) != hipSuccess)
    return hip_fail("f = x W", e);
  still::BwdNpArgs nq{};
  nq.x = q; nq.x_sb = p->q_sb; nq.x_st = p->q_st; nq.x_sh = p->q_sh; nq.x_kv = 0;
  nq.bias = bq; nq.u = f32p(BL.uq); nq.st = f32p(BL.stq); nq.phi = bws + BL.phi_q; nq.kmask = nullptr;
  nq.map = map; nq.U = U; nq.N = N; nq.Hq = Hq; nq.Hkv = p->Hkv; nq.d = d; nq.F = F; nq.C = C; nq.nc = nc; nq.ncf = ncf;
  nq.nseg = L.nseg; nq.seg_chunks = L.seg_chunks;
  still::BwdNpArgs nk = nq;
  nk.x = k; nk.x_sb = p->k_sb; nk.x_st = p->k_st; nk.x_sh = p->k_sh; nk.x_kv = 1;
  nk.bias = bk; nk.u = f32p(BL.uk); nk.st = f32p(BL.stk); nk.phi = bws + BL.phi_k;
  nk.kmask = reinterpret_cast<const uint32_t*>(ws + L.kmask);
  if ((e = still::launch_bwd_np(nq, dt, false, stream)) != hipSuccess ||
      (e = still::launch_bwd_np(nk, dt, false, stream)) != hipSuccess)
    return hip_fail("feature maps", e);
  *nq_out = nq;
  *nk_out = nk;
  return STILL_OK;
}

size_t map_bwd_extra(const still_params_t* p, size_t* rowdot_off, size_t* dw_off, int* np8) {
  still_bwd_ws_layout_t BL;
  compute_bwd_layout(p, &BL);
  const size_t U = (size_t)p->B * p->Hq, N = p->N, n8 = (N + 7) / 8 * 8;
  *rowdot_off = BL.total;
  *dw_off = align_up(*rowdot_off + U * N * 4, 256);
  *np8 = (int)n8;
  return align_up(*dw_off + U * N * n8 * esize(p->dtype), 256);
}

}  // namespace

extern "C" {

still_status_t still_attention_map(const still_params_t* p, const void* q, const void* k, const void* Wq,
                                   const void* bq, const void* Wk, const void* bk, const float* lse,
                                   const int32_t* sel_idx, float* map_out, void* workspace, size_t workspace_bytes,
                                   void* stream_v) {
  still_status_t st = validate_bwd_params(p);
  if (st != STILL_OK) return st;
  st = validate_strides(p, false);
  if (st != STILL_OK) return st;
  if (!q || !k || !Wq || !Wk || !lse || !map_out || !workspace)
    return fail(STILL_ERR_INVALID_ARG, "a required pointer (q, k, Wq, Wk, lse, map_out, workspace) is NULL");
  const int ncf = p->N / p->C, U = p->B * p->Hq;
  if (p->lambda > 0 && ncf > 0 && sel_idx == nullptr)
    return fail(STILL_ERR_INVALID_ARG, "sel_idx (the forward pass's index lists) is NULL");
  const void* ptrs[] = {q, k, Wq, bq, Wk, bk, lse, sel_idx, map_out, workspace};
  for (const void* x : ptrs)
    if (x != nullptr && !aligned16(x)) return fail(STILL_ERR_INVALID_ARG, "pointer %p is not 16-byte aligned", x);
  still_bwd_ws_layout_t BL;
  compute_bwd_layout(p, &BL);
  if (workspace_bytes < BL.total)
    return fail(STILL_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, BL.total);
  still_ws_layout_t L;
  compute_layout(p, &L);
  hipStream_t stream = static_cast<hipStream_t>(stream_v);
  unsigned char* bws = static_cast<unsigned char*>(workspace);
  still::HeadMap map;
  fill_map(p, &map);
  still::BwdNpArgs nq, nk;
  st = prepare_feature_maps(p, q, k, Wq, bq, Wk, bk, sel_idx, bws, BL, L, map, stream, &nq, &nk);
  if (st != STILL_OK) return st;
  still::AttnMapArgs am{};
  am.q = q; am.k = k;
  am.q_sb = p->q_sb; am.q_st = p->q_st; am.q_sh = p->q_sh; am.k_sb = p->k_sb; am.k_st = p->k_st; am.k_sh = p->k_sh;
  am.phi_q = bws + BL.phi_q; am.phi_k = bws + BL.phi_k; am.kmask = nk.kmask; am.lse = lse; am.map_out = map_out;
  am.map = map; am.N = p->N; am.C = p->C; am.Hq = p->Hq; am.ncf = ncf; am.scale = p->scale;
  const hipError_t e = still::launch_attn_map(am, p->dtype, p->d, U, stream);
  if (e != hipSuccess) return fail(STILL_ERR_HIP, "attention_map: %s", hipGetErrorString(e));
  g_err[0] = 0;
  return STILL_OK;
}

size_t still_attention_map_bwd_workspace_bytes(const still_params_t* p) {
  if (validate_bwd_params(p) != STILL_OK) return 0;
  size_t r, w;
  int n8;
  return map_bwd_extra(p, &r, &w, &n8);
}

still_status_t still_attention_map_bwd(const still_params_t* p, const void* q, const void* k, const void* Wq,
                                       const void* bq, const void* Wk, const void* bk, const float* lse,
                                       const int32_t* sel_idx, const float* map, const float* dmap, float* dWq,
                                       float* dbq, float* dWk, float* dbk, void* workspace, size_t workspace_bytes,
                                       void* stream_v) {
  still_status_t st = validate_bwd_params(p);
  if (st != STILL_OK) return st;
  st = validate_strides(p, false);
  if (st != STILL_OK) return st;
  if (!q || !k || !Wq || !Wk || !lse || !map || !dmap || !dWq || !dWk || !workspace)
    return fail(STILL_ERR_INVALID_ARG,
                "a required pointer (q, k, Wq, Wk, lse, map, dmap, dWq, dWk, workspace) is NULL");
  if ((bq != nullptr) != (dbq != nullptr) || (bk != nullptr) != (dbk != nullptr))
    return fail(STILL_ERR_INVALID_ARG, "dbq / dbk must be given exactly when bq / bk are");
  const int B = p->B, N = p->N, d = p->d, C = p->C, F = p->d_f, DP = 2 * F, Hq = p->Hq;
  const int nc = (N + C - 1) / C, ncf = N / C, U = B * Hq;
  if (p->lambda > 0 && ncf > 0 && sel_idx == nullptr)
    return fail(STILL_ERR_INVALID_ARG, "sel_idx (the forward pass's index lists) is NULL");
  const void* ptrs[] = {q, k, Wq, bq, Wk, bk, lse, sel_idx, map, dmap, dWq, dbq, dWk, dbk, workspace};
  for (const void* x : ptrs)
    if (x != nullptr && !aligned16(x)) return fail(STILL_ERR_INVALID_ARG, "pointer %p is not 16-byte aligned", x);
  size_t rowdot_off, dw_off;
  int np8;
  const size_t need = map_bwd_extra(p, &rowdot_off, &dw_off, &np8);
  if (workspace_bytes < need)
    return fail(STILL_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
  still_bwd_ws_layout_t BL;
  compute_bwd_layout(p, &BL);
  still_ws_layout_t L;
  compute_layout(p, &L);
  hipStream_t stream = static_cast<hipStream_t>(stream_v);
  unsigned char* bws = static_cast<unsigned char*>(workspace);
  still::HeadMap hmap;
  fill_map(p, &hmap);
  const int dt = p->dtype;
  hipError_t e;
  auto hip_fail = [&](const char* what, hipError_t err) -> still_status_t {
    return fail(STILL_ERR_HIP, "%s: %s", what, hipGetErrorString(err));
  };
  auto f32p = [&](size_t off) { return reinterpret_cast<float*>(bws + off); };
  if ((e = still::launch_fill_f32(dWq, (int64_t)Hq * d * F, 0.f, stream)) != hipSuccess ||
      (e = still::launch_fill_f32(dWk, (int64_t)Hq * d * F, 0.f, stream)) != hipSuccess ||
      (dbq && (e = still::launch_fill_f32(dbq, (int64_t)Hq * F, 0.f, stream)) != hipSuccess) ||
      (dbk && (e = still::launch_fill_f32(dbk, (int64_t)Hq * F, 0.f, stream)) != hipSuccess))
    return hip_fail("fill", e);
  still::BwdNpArgs nq, nk;
  st = prepare_feature_maps(p, q, k, Wq, bq, Wk, bk, sel_idx, bws, BL, L, hmap, stream, &nq, &nk);
  if (st != STILL_OK) return st;
  // dw: the gradient of the linear branch's weights, zero on every other pair
  still::MapDwArgs md{dmap, lse, nk.kmask, f32p(rowdot_off), bws + dw_off, N, np8, C, ncf};
  if ((e = still::launch_map_dw(md, map, dt, U, stream)) != hipSuccess) return hip_fail("map_dw", e);
  // dphi_q = dw phi_k, dphi_k = dw^T phi_q (one item per (batch, head), all rows)
  still::GemmArgs gm{};
  gm.Hq = Hq; gm.map = hmap;
  const int64_t NDP = (int64_t)N * DP, NN8 = (int64_t)N * np8, NF = (int64_t)N * F;
  auto run = [&](const still::GemmOperand& A_, const still::GemmOperand& B_, float* Cp, int64_t c_b, int64_t c_h,
                 int64_t c_c, int64_t c_r, int M_, int Nn_, int K_, int k_total, int mode, int n_c) -> hipError_t {
    gm.A = A_; gm.B = B_; gm.B2 = still::GemmOperand{}; gm.C = Cp;
    gm.c_b = c_b; gm.c_h = c_h; gm.c_c = c_c; gm.c_r = c_r; gm.c_kv = 0;
    gm.M = M_; gm.Nn = Nn_; gm.K = K_; gm.m_total = 0; gm.k_total = k_total; gm.mode = mode;
    return still::launch_bgemm(gm, dt, U, n_c, stream);
  };
  const still::GemmOperand dw_tj = operand(bws + dw_off, Hq * NN8, NN8, 0, np8, 1);      // (m = t, k = j)
  const still::GemmOperand dw_jt = operand(bws + dw_off, Hq * NN8, NN8, 0, 1, np8);      // (m = j, k = t)
  const still::GemmOperand phik_fj = operand(bws + BL.phi_k, Hq * NDP, NDP, 0, 1, DP);   // (n = f, k = j)
  const still::GemmOperand phiq_ft = operand(bws + BL.phi_q, Hq * NDP, NDP, 0, 1, DP);   // (n = f, k = t)
  if ((e = run(dw_tj, phik_fj, f32p(BL.gq), Hq * NDP, NDP, 0, DP, N, DP, N, 0, 0, 1)) != hipSuccess ||
      (e = run(dw_jt, phiq_ft, f32p(BL.dphi_k), Hq * NDP, NDP, 0, DP, N, DP, N, 0, 0, 1)) != hipSuccess)
    return hip_fail("map backward products", e);
  // NP-Map backwards, then dW += x^T df and the bias gradients
  nq.dphi = f32p(BL.gq); nq.coef = nullptr; nq.z1 = nullptr; nq.z2 = nullptr;
  nq.df = bws + BL.dfq; nq.cx = f32p(BL.cxq);
  nk.dphi = f32p(BL.dphi_k); nk.coef = nullptr; nk.z1 = nullptr; nk.z2 = nullptr;
  nk.df = bws + BL.dfk; nk.cx = f32p(BL.cxk);
  if ((e = still::launch_bwd_np(nq, dt, true, stream)) != hipSuccess ||
      (e = still::launch_bwd_np(nk, dt, true, stream)) != hipSuccess)
    return hip_fail("bwd_np_bwd", e);
  const int KS = 256, nsplit = (N + KS - 1) / KS;
  const still::GemmOperand q_xt = operand(q, p->q_sb, p->q_sh, (int64_t)KS * p->q_st, 1, p->q_st);
  const still::GemmOperand k_xt = operand(k, p->k_sb, p->k_sh, (int64_t)KS * p->k_st, 1, p->k_st, 1);
  const still::GemmOperand dfq_ft = operand(bws + BL.dfq, Hq * NF, NF, (int64_t)KS * F, 1, F);
  const still::GemmOperand dfk_ft = operand(bws + BL.dfk, Hq * NF, NF, (int64_t)KS * F, 1, F);
  if ((e = run(q_xt, dfq_ft, dWq, 0, (int64_t)d * F, 0, F, d, F, KS, N, 2, nsplit)) != hipSuccess ||
      (e = run(k_xt, dfk_ft, dWk, 0, (int64_t)d * F, 0, F, d, F, KS, N, 2, nsplit)) != hipSuccess)
    return hip_fail("dW += x^T df", e);
  if (dbq != nullptr) {
    still::BwdColsumArgs cb{bws + BL.dfq, nullptr, dbq, N, C, nc, F, Hq, 1};
    if ((e = still::launch_bwd_colsum(cb, dt, U, stream)) != hipSuccess) return hip_fail("db", e);
  }
  if (dbk != nullptr) {
    still::BwdColsumArgs cb{bws + BL.dfk, nullptr, dbk, N, C, nc, F, Hq, 1};
    if ((e = still::launch_bwd_colsum(cb, dt, U, stream)) != hipSuccess) return hip_fail("db", e);
  }
  g_err[0] = 0;
  return STILL_OK;
}

still_status_t still_rope_apply(const still_params_t* p, void* q, void* k, const int32_t* pos0, float base,
                                void* stream_v) {
  if (p == nullptr) return fail(STILL_ERR_INVALID_ARG, "params is NULL");
  if (p->dtype != STILL_F32 && p->dtype != STILL_BF16) return fail(STILL_ERR_INVALID_ARG, "dtype %d unknown", p->dtype);
  if (p->B < 1 || p->N < 1 || p->Hq < 1 || p->Hkv < 1) return fail(STILL_ERR_INVALID_ARG, "B, N, Hq, Hkv must be >= 1");
  if (p->d < 2 || p->d % 2 != 0) return fail(STILL_ERR_INVALID_ARG, "d = %d must be even", p->d);
  if (!(base > 1.f)) return fail(STILL_ERR_INVALID_ARG, "base must be > 1");
  if (q == nullptr && k == nullptr) return fail(STILL_ERR_INVALID_ARG, "both q and k are NULL");
  if (pos0 != nullptr && (reinterpret_cast<uintptr_t>(pos0) & 3) != 0)
    return fail(STILL_ERR_INVALID_ARG, "pos0 is not 4-byte aligned");
  const int64_t str[] = {p->q_sb, p->q_st, p->q_sh, p->k_sb, p->k_st, p->k_sh};
  for (int64_t x : str)
    if (x < 0) return fail(STILL_ERR_INVALID_ARG, "negative stride");
  if ((q != nullptr && p->q_st < p->d) || (k != nullptr && p->k_st < p->d))
    return fail(STILL_ERR_INVALID_ARG, "token stride smaller than d");
  still::RopeArgs a{q, k, p->q_sb, p->q_st, p->q_sh, p->k_sb, p->k_st, p->k_sh, pos0, log2((double)base),
                    p->B, p->N, p->Hq, p->Hkv, p->d};
  hipError_t e = still::launch_rope(a, p->dtype, static_cast<hipStream_t>(stream_v));
  if (e != hipSuccess) return fail(STILL_ERR_HIP, "rope_apply: %s", hipGetErrorString(e));
  g_err[0] = 0;
  return STILL_OK;
}

still_status_t still_hybrid_attn_bwd(const still_params_t* p, const void* q, const void* k, const void* v,
                                     const void* g, const void* Wq, const void* bq, const void* Wk, const void* bk,
                                     const void* out, const void* dout, const float* lse, const int32_t* sel_idx,
                                     void* dq, void* dk, void* dv, void* dg, float* dWq, float* dbq, float* dWk,
                                     float* dbk, void* workspace, size_t workspace_bytes, void* stream) {
  return bwd_impl(p, q, k, v, g, Wq, bq, Wk, bk, out, dout, lse, sel_idx, dq, dk, dv, dg, dWq, dbq, dWk, dbk,
                  workspace, workspace_bytes, stream);
}

}  // extern "C"

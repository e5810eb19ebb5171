/*
 * libstill - hot path of STILL's intra-layer hybrid attention on AMD MI355X (gfx950).
 *
 * One Transformer layer's attention operator from "STILL" (arXiv 2602.02180), forward (prefill and decode) and the
 * backward pass of the prefill:
 *   - Self-Saliency Score over a causal sliding window            (Sec. 3.1, score equation)
 *   - delayed, chunk-granular Top-lambda routing                   (Sec. 3.3, delayed-selection eq.)
 *   - softmax attention over the salient cache (local span + retained tokens)
 *   - NP-Map linear attention over every other routed token        (Sec. 3.2; cache-routing eq.)
 *   - one shared normaliser  y = (N_SA + N_LA) / (D_SA + D_LA)     (Sec. 3.3, output eqs.)
 * in its chunk-wise parallel form (Algorithm 1) for prefill and its recurrent form for decode.
 *
 * Conventions
 *   - Plain C ABI.  Every tensor, workspace and state pointer is DEVICE memory owned by the caller,
 *     16-byte aligned, unless marked HOST.  The library allocates and frees nothing on the device,
 *     never synchronises the stream, and keeps no global mutable state except, per host thread, an error
 *     text, the timing events below and one helper stream with two events (created at the first prefill
 *     call on a device, default priority, never destroyed while the thread stays on that device).
 *   - All work is ordered on `stream` (a hipStream_t passed as void*; NULL = the default stream): work
 *     enqueued on `stream` before a call precedes all of the call's kernels, work enqueued after it follows
 *     all of them.  still_hybrid_attn_fwd runs two small layout kernels on the helper stream, forked from
 *     and joined back into `stream` with events, so the same holds under stream capture.
 *   - Tokens and chunks are 0-indexed here (the paper counts from 1).
 *   - Every function returning still_status_t validates its arguments on the host before any launch;
 *     on failure nothing has been enqueued and still_last_error() describes the reason.
 */
#ifndef STILL_H
#define STILL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define STILL_API __attribute__((visibility("default")))

typedef enum {
  STILL_OK = 0,
  STILL_ERR_INVALID_ARG = 1,         /* null/misaligned pointer, inconsistent sizes              */
  STILL_ERR_UNSUPPORTED = 2,         /* legal problem outside the shapes the kernels are built for */
  STILL_ERR_WORKSPACE_TOO_SMALL = 3,
  STILL_ERR_HIP = 4,                 /* a launch was rejected by the runtime                     */
  STILL_ERR_STATE = 5                /* decode state full or not initialised for these params    */
} still_status_t;

typedef enum { STILL_F32 = 0, STILL_BF16 = 1 } still_dtype_t;

/*
 * Problem description (Algorithm 1's inputs: q, k, v, gate g, feature maps phi_q / phi_k, chunk size C,
 * number lambda, small constant eps; plus what the paper leaves implicit: batch, GQA head map, the
 * score window W of the window-set equation, and the logit scale).
 *
 * Supported by the kernels (both dtypes): d in {64,128}; d_f == d; C in {64,128}; 1 <= W <= min(256, 4 C); 0 <= lambda <= C;
 * Hq <= 128; Hq % Hkv == 0 when kv_head_of_q is NULL.  N >= 1 need not be a multiple of C: the trailing
 * partial chunk is never ranked.  Anything else returns STILL_ERR_UNSUPPORTED.
 *
 * Strides are in ELEMENTS for (batch, token, head); the head dimension is contiguous.  Every stride
 * must be a multiple of 16 bytes.
 */
typedef struct still_params {
  int32_t B, N, Hq, Hkv, d, d_f; /* d_f: width of the NP-Map layer f(x) = x W + b; phi has 2*d_f features */
  int32_t C, W, lambda;          /* chunk size, score window (keys, token itself included), kept per chunk */
  float scale;                   /* > 0; multiplies every q.k logit, score window and softmax branch alike */
  float eps;                     /* eps of the score equation                                              */
  int32_t dtype;                 /* still_dtype_t of q, k, v, g, out, Wq, Wk, bq, bk                        */
  int32_t max_tokens;            /* capacity (tokens per sequence) of a decode state; used only by the state
                                    functions, the decode step and state_out; 0 where no state is involved  */
  int32_t max_retained;          /* budget on the retained tokens of one (sequence, query head); <= 0: none.
                                    The long-context evaluations of Sec. 4 cap the number of selected tokens
                                    without stating a policy; here chunks are served in order: chunk c keeps
                                    its min(lambda, max_retained - c*lambda) highest scores (none once the
                                    budget is used up) and the rest of the chunk goes to the linear state like
                                    any other un-selected token.  Slots of an index list that a chunk does not
                                    use hold -1.  A decode state then needs only max_retained retained rows. */
  int32_t shared_selection;      /* 0: every query head ranks by its own score (the paper's method).
                                    1: a variant for grouped-query attention, which the paper does not mention:
                                    the query heads that read one kv head rank each chunk by the SUM of their
                                    scores (added in ascending head order) and keep the same tokens; sel_idx
                                    still has one list per query head, the lists of a group being equal.  A
                                    decode state then holds the retained rows once per kv head, and a decode
                                    step reads each of them once for the whole group.                        */
  int32_t emit_terms;            /* inspection hook, normally 0.  1: the prefill also leaves the linear-branch
                                    terms of every row in the workspace (regions n_la, d_la of the layout), which
                                    then needs room for them; the results are the same either way.             */
  int32_t gate_activation;       /* 0: g multiplies the linear numerator as given (already activated).
                                    1: g holds a pre-activation (x W_g of Sec. 3.2) and the kernels apply the
                                    logistic function 1 / (1 + exp(-g)) where they read it; the paper names no
                                    activation, this one is an option of this library.  Prefill and decode.   */
  int32_t budget_policy;         /* what max_retained means once the budget is reached (both are inventions, see
                                    max_retained).  0: stop adding, as described there.  1: evict the lowest
                                    score: every routed chunk offers its lambda highest scores; the retained set
                                    is then cut back to max_retained members by removing the lowest score first
                                    (between equal scores the higher token index first), and a removed token,
                                    retained earlier or just offered, enters the linear state (through the
                                    NP-Map) at that routing step, so that every past token is still seen exactly
                                    once.  sel lists then hold the chunk's offers (cap of the workspace layout
                                    counts all offers).  Prefill and decode; shared_selection, injected indices
                                    (sel_idx_is_input) and the allocation-free entry point refuse it.          */
  int64_t q_sb, q_st, q_sh;      /* q   [B, N, Hq,  d]                                                     */
  int64_t k_sb, k_st, k_sh;      /* k   [B, N, Hkv, d]                                                     */
  int64_t v_sb, v_st, v_sh;      /* v   [B, N, Hkv, d]                                                     */
  int64_t o_sb, o_st, o_sh;      /* out [B, N, Hq,  d]                                                     */
  int64_t g_sb, g_st, g_sh;      /* g   [B, N, Hq,  d] (ignored when g == NULL)                            */
  const int32_t* kv_head_of_q;   /* HOST, Hq entries in [0,Hkv), or NULL => hq / (Hq / Hkv)                */
  const int32_t* seq_len;        /* DEVICE, B entries, or NULL: prefill of a right-padded batch.  Sequence b has
                                    seq_len[b] tokens (clamped to [1, N]); its rows t >= seq_len[b] are padding:
                                    their q, k, v are never read as part of a real row's result (they may hold
                                    anything), their rows of out are not written, and their entries of score_out
                                    and sel_idx are unspecified.  Rows t < seq_len[b] get exactly the result of a
                                    call with that sequence alone (the operator is causal), and state_out holds,
                                    for every sequence, the state after ITS last token, so decoding continues
                                    with still_hybrid_attn_decode_step_at at t_dev[b] = seq_len[b].  Ignored by
                                    the decode functions.                                                     */
} still_params_t;

/* Byte offsets of the regions still_hybrid_attn_fwd lays out inside its workspace (for tests/tools). */
typedef struct still_ws_layout {
  size_t score;    /* float   [B, Hq, N]                         Self-Saliency Score of every token        */
  size_t sel;      /* int32   [B, Hq, N/C, lambda]               selected tokens per full chunk, ascending */
  size_t vt;       /* dtype   [B, Hkv, d, Npad]                  v transposed, zero padded                 */
  size_t kret;     /* dtype   [B, Hq, cap, d]                    retained keys in routing order            */
  size_t vrett;    /* dtype   [B, Hq, d, cap]                    retained values, transposed               */
  size_t wqt;      /* dtype   [Hq, d_f, d]                       Wq transposed                             */
  size_t wkf;      /* dtype   [Hq, d_f * d]                      Wk transposed, in matrix-operand order    */
  size_t seg;      /* float   [B, Hq, nseg, 2*d_f*(d+1)]         per-segment totals of the linear-attention state */
  size_t snap;     /* dtype   [B, Hq, ceil(N/C), d, 2*d_f]       S^T summed inside chunk c's segment, through chunk c-2 */
  size_t zsnap;    /* float   [B, Hq, ceil(N/C), 2*d_f]          z likewise                                */
  size_t pimg;     /* dtype   [B, Hq, nseg, d, 2*d_f]            S^T through the chunk before the segment (prefix) */
  size_t zpre;     /* float   [B, Hq, nseg, 2*d_f]               z likewise                                */
  size_t kmask;    /* uint32  [B, Hq, N/C, C/32]                 the selection as one bit per token        */
  size_t n_la;     /* float   [B, Hq, N, d]                      gated linear-branch numerator N_LA (emit_terms) */
  size_t d_la;     /* float   [B, Hq, N]                         linear-branch normaliser D_LA (emit_terms) */
  size_t vfr;      /* dtype   [B, Hkv, Npad * d]                 v in the operand order of the state update */
  size_t ev_src;   /* int32   [B, Hq, N]          budget_policy 1: token whose key/value a position carries into the state */
  size_t ev_alive; /* uint64  [B, Hq, ceil(N/C), cap/64]  budget_policy 1: per row chunk, which offers are retained */
  size_t ev_fin;   /* budget_policy 1: the set retained after the last routed step: int32 tok [B,Hq,M], float score
                      [B,Hq,M], int32 count [B,Hq]                                                           */
  size_t ev_vfr;   /* dtype   [B, Hq, Npad * d]   budget_policy 1: v in operand order per query head, through ev_src */
  size_t lse;      /* float   [B, Hq, N]          ln(D_SA + D_LA) of every row: the log of the shared normaliser of the
                      output equation, written by every prefill call; still_hybrid_attn_bwd reads it           */
  size_t total;    /* bytes needed                                                                         */
  int32_t n_pad;   /* Npad                                                                                 */
  int32_t cap;     /* retained-row capacity (multiple of 64)                                               */
  int32_t nseg;    /* segments of the chunk scan                                                           */
  int32_t seg_chunks; /* chunks per segment                                                                */
} still_ws_layout_t;

/* Library/ABI version: major*10000 + minor*100 + patch. */
STILL_API int32_t still_version(void);

/* Text of the last failure on the calling thread (static storage, never NULL). */
STILL_API const char* still_last_error(void);

/* Bytes of device workspace still_hybrid_attn_fwd needs for `p`; 0 on invalid/unsupported params
 * (still_last_error() says why). */
STILL_API size_t still_fwd_workspace_bytes(const still_params_t* p);

/* Fills *layout for `p`; same validation as above. */
STILL_API still_status_t still_fwd_workspace_layout(const still_params_t* p, still_ws_layout_t* layout);

/*
 * Prefill: the chunk-wise parallel form (Algorithm 1) over all N tokens of B sequences.
 *
 *   q, k, v        device, dtype, strided as described in `p`
 *   g              device, dtype, or NULL (gate of ones); multiplies the linear numerator only
 *   Wq, Wk         device, dtype, [Hq, d, d_f] contiguous: per-query-head NP-Map layers for q and k
 *   bq, bk         device, dtype, [Hq, d_f] contiguous, or NULL (no bias)
 *   out            device, dtype, strided; rows written for every (b, t < N, hq)
 *   score_out      device float [B, Hq, N] or NULL: Score of every token
 *   sel_idx        device int32 [B, Hq, N/C, lambda] or NULL: global token indices of the tokens kept
 *                  in each full chunk, ascending within a chunk; -1 in the slots that a budget
 *                  (max_retained) leaves unused, which are always the last slots of a chunk
 *   sel_idx_is_input  0: sel_idx (if given) is an OUTPUT.  1: sel_idx is an INPUT that replaces the
 *                  Top-lambda step (indices must lie inside their chunk, strictly ascending; with a budget
 *                  only the first min(lambda, max_retained - c*lambda) slots of chunk c are read; with
 *                  shared_selection the lists of the query heads of one kv head must be equal); test hook
 *   state_out      device, or NULL: a decode state buffer (see still_state_bytes; p->max_tokens >= N);
 *                  on return it holds the tokens 0..N-1, so the next decode step is t = N.  Its previous
 *                  contents are overwritten (no still_state_init needed)
 *   workspace      device scratch of at least still_fwd_workspace_bytes(p) bytes; contents undefined
 *                  afterwards, except the regions the layout documents as results (score, sel, lse)
 *   stream         hipStream_t (as void*)
 *
 * Ties in the Top-lambda step go to the lower token index.  NaN inputs give undefined routing.
 */
STILL_API still_status_t still_hybrid_attn_fwd(const still_params_t* p,
                                     const void* q, const void* k, const void* v, const void* g,
                                     const void* Wq, const void* bq, const void* Wk, const void* bk,
                                     void* out, float* score_out, int32_t* sel_idx,
                                     int32_t sel_idx_is_input, void* state_out,
                                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same prefill for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture that has no buffer to hand, tight serving loops, harnesses that forbid hipMalloc.  It is
 * still_hybrid_attn_fwd with the workspace taken from a fixed array of STILL_STATIC_WORKSPACE_BYTES that is part of
 * the library's device code (every GPU the library runs on holds one copy until the process ends), with every kernel
 * on `stream` (no helper stream, no timing events): the call creates no stream, event or allocation of any kind.
 * Same arguments, same results (bit for bit: the same kernels run in the same order).
 *
 *   - Problems whose still_fwd_workspace_bytes(p) exceeds STILL_STATIC_WORKSPACE_BYTES are refused with
 *     STILL_ERR_WORKSPACE_TOO_SMALL before anything is enqueued (use still_hybrid_attn_fwd for those).
 *   - All calls on one GPU share that GPU's array: two calls whose kernels may overlap in time (different streams,
 *     different host threads) race; calls on one stream are ordered and safe.  Nothing in the array has to start at
 *     zero and nothing in it survives a call.
 *   - The first call on a device looks up the array's address (hipGetSymbolAddress); make that call outside a
 *     stream capture.
 */
#define STILL_STATIC_WORKSPACE_BYTES (32u << 20)
STILL_API still_status_t still_hybrid_attn_fwd_static(const still_params_t* p,
                                            const void* q, const void* k, const void* v, const void* g,
                                            const void* Wq, const void* bq, const void* Wk, const void* bk,
                                            void* out, float* score_out, int32_t* sel_idx,
                                            int32_t sel_idx_is_input, void* state_out, void* stream);

/*
 * Optional per-kernel timing of still_hybrid_attn_fwd (used by the benchmark to time the dominant kernel
 * on the stream it is launched on).  While enabled on the calling thread, every prefill call records HIP
 * events (host objects created lazily, one ring of 64 sets per thread) around each of its kernels; it does
 * not synchronise.  still_profile_read waits for the last recorded call to finish and writes, for up to n
 * kernels in launch order, the MEAN duration in milliseconds over the calls recorded since
 * still_profile_enable(1) (the last 64 of them if there were more) into the HOST array ms;
 * still_profile_kernel_name(i) names slot i (NULL past the last).  Returns STILL_ERR_STATE if no call was
 * recorded.  A kernel that a call skips (e.g. the score kernel when the selection is an input) shows as a
 * zero-length slot.
 * still_profile_enable(2) records the pair of the last kernel (the sparse-attention + merge kernel) only and
 * reports 0 for the others: every recorded event is a marker in the stream, and sixteen of them per call cost
 * a few per cent of a back-to-back run.
 * The two layout kernels (slots 0 and 1) run on a library-owned second stream next to the score kernel
 * (slot 2), so the durations of these three overlap and do not add up to the duration of the call.
 */
#define STILL_PROFILE_SLOTS 8
STILL_API void still_profile_enable(int32_t on);
STILL_API still_status_t still_profile_read(float* ms, int32_t n);
STILL_API const char* still_profile_kernel_name(int32_t i);

/*
 * Decode state of B sequences (in lock step, or each at its own token: every region below is sliced per
 * sequence): the salient cache h and the state (s, z) of the cache-routing equation (Sec. 3.3), plus the ring of
 * recent tokens that delayed selection needs.  One
 * opaque caller-owned device buffer of still_state_bytes(p) bytes (p->max_tokens = capacity per sequence):
 *   S    float [B, Hq, 2*d_f*(d+1)]   state through the last routed chunk: S (2*d_f x d) then z (2*d_f)
 *   Kret dtype [B, Hq, cap, d]        retained keys in routing order ([B, Hkv, cap, d] with shared_selection);
 *                                     cap = lambda*ceil(max_tokens/C), or max_retained if that is smaller (+pad)
 *   Vret dtype [B, Hq, cap, d]        retained values
 *   sel  int32 [B, Hq, ceil(max_tokens/C), lambda]   token indices kept per routed chunk, -1 in unused slots
 *                                     (for inspection)
 *   ring dtype [B, Hkv, R, d] x 2     keys and values of the last R = 4*C tokens, slot = token % R
 *   sc   float [B, Hq, R]             Self-Saliency Score of the same tokens
 *   part float [B, Hq, 32, d+2]       split partials of the attention pass
 *   rsc  float [B, Hq, cap]           budget_policy 1 only: Self-Saliency Score of every retained row
 *   rtok int32 [B, Hq, cap]           budget_policy 1 only: its token index (retained rows are then in no order)
 * The number of tokens seen is NOT stored: the caller passes the index t of the new token to every step.
 * The buffer can be copied or saved with plain memcpy.  p->N is ignored by the state functions.
 */
STILL_API size_t still_state_bytes(const still_params_t* p);

/* Byte offsets of the regions above inside a state buffer (for tests/tools). */
typedef struct still_state_layout {
  size_t S, kret, vret, sel, kring, vring, score, part, ret_score, ret_tok, total;
  int32_t cap, R, n_chunks;
} still_state_layout_t;
STILL_API still_status_t still_state_layout(const still_params_t* p, still_state_layout_t* layout);

/* Resets a state buffer to "no token seen" (zero fill on `stream`). */
STILL_API still_status_t still_state_init(const still_params_t* p, void* state, void* stream);

/*
 * One decode step of the recurrent form (Sec. 3.3) for the token with index t (0-based; the state must hold
 * exactly the tokens 0..t-1) of every sequence in the batch:
 *   - (k_t, v_t) are appended to the ring and the token's Self-Saliency Score over its window is stored;
 *   - if t opens a new chunk c = t/C >= 2, chunk c-2 leaves the local span and is routed: its Top-lambda
 *     keys/values (fewer once a max_retained budget runs out) join the retained cache, the others are added
 *     to (s, z) through the NP-Map;
 *   - y_t = (N_SA + N_LA) / (D_SA + D_LA) over the retained cache, the local span and the state.
 *
 *   q_t [B, Hq, d], k_t, v_t [B, Hkv, d], g_t [B, Hq, d] or NULL, out_t [B, Hq, d]: device, dtype, contiguous.
 *   Wq, Wk, bq, bk as for the prefill.
 * Returns STILL_ERR_STATE when t < 0 or t >= p->max_tokens.
 */
STILL_API still_status_t still_hybrid_attn_decode_step(const still_params_t* p, void* state, int32_t t,
                                                       const void* q_t, const void* k_t, const void* v_t,
                                                       const void* g_t,
                                                       const void* Wq, const void* bq, const void* Wk, const void* bk,
                                                       void* out_t, void* stream);

/*
 * The same decode step (recurrent form, Sec. 3.3) for sequences that are NOT in lock step, as a serving loop
 * with continuous batching needs: sequence b appends the token with index t_dev[b] (its state must hold exactly
 * the tokens 0..t_dev[b]-1 of that sequence).  Every sequence owns its slice of each state region, so sequences
 * at different positions never interact; a sequence whose new token opens a chunk c >= 2 routes its own chunk
 * c-2 in this call, the others do not.
 *
 *   t_dev   DEVICE int32 [B], read by the kernels of this call (the caller may advance it with a kernel of its
 *           own between calls, so a captured graph of the step can be replayed).  An entry outside
 *           [0, p->max_tokens) marks a sequence that sits this step out: its state and its row of out_t are
 *           left untouched.
 *   t_max   HOST upper bound of the entries of t_dev, 0 <= t_max < p->max_tokens (p->max_tokens - 1 is always
 *           valid); it sizes the launch (how many workgroups share one sequence's cache rows; whether the routing
 *           kernel is launched at all), a tight bound gives the best split.  An entry above t_max is a caller
 *           error: that sequence's result is undefined.
 * All other arguments as for still_hybrid_attn_decode_step.  Returns STILL_ERR_STATE when t_max is outside
 * [0, p->max_tokens).
 */
STILL_API still_status_t still_hybrid_attn_decode_step_at(const still_params_t* p, void* state,
                                                          const int32_t* t_dev, int32_t t_max,
                                                          const void* q_t, const void* k_t, const void* v_t,
                                                          const void* g_t,
                                                          const void* Wq, const void* bq, const void* Wk, const void* bk,
                                                          void* out_t, void* stream);

/*
 * Local-versus-global consistency study of Sec. 3.1 (the figure that compares the window-local Self-Saliency
 * Score with the score over the whole context): a second workload on the score step, not part of the layer.
 *
 * still_global_score: the score equation with the window set replaced by the whole causal prefix {0..t}, for every
 *   (b, hq, t).  q, k: device, dtype, strided as in `p`; score_out: device float [B, Hq, N].  Read from `p`: B, N,
 *   Hq, Hkv, d (64 or 128), dtype, scale, eps, the q/k strides and the head map; W, C, lambda, d_f and the rest are
 *   ignored.  Cost is quadratic in N (two passes over the causal logits).
 * still_selection_overlap: for every full chunk, the number of tokens that the Top-lambda sets under two scores
 *   have in common (ties to the lower index, as in the selection step).  score_a, score_b: device float [B, Hq, N]
 *   (for instance score_out of the prefill and of still_global_score); overlap: device int32 [B, Hq, N/C].
 *   overlap / lambda averaged over chunks is the consistency figure.  Read from `p`: B, N, Hq, C (1..128), lambda.
 * Both validate on the host and return the usual codes; neither needs a workspace.
 */
STILL_API still_status_t still_global_score(const still_params_t* p, const void* q, const void* k, float* score_out,
                                            void* stream);
STILL_API still_status_t still_selection_overlap(const still_params_t* p, const float* score_a, const float* score_b,
                                                 int32_t* overlap, void* stream);

/*
 * Backward pass of the prefill.  The paper trains the operator (Sec. 4.1: attention transfer for the feature maps
 * and the gate, then low-rank adaptation of the projections) without printing its gradients; what is differentiated
 * here is the output equation of Sec. 3.3, y = (N_SA + g N_LA) / (D_SA + D_LA), through the softmax branch's
 * exponentials, the linear branch's phi_q . phi_k weights and the NP-Map of Sec. 3.2, for the index lists the forward
 * pass chose: the Top-lambda selection is a discrete decision and passes no gradient, and the Self-Saliency Score
 * only feeds that decision.
 *
 *   q, k, v, g, Wq, bq, Wk, bk   as given to still_hybrid_attn_fwd (same `p`, same strides)
 *   out            device, dtype: the forward pass's result
 *   dout           device, dtype, strided like out: gradient of the loss w.r.t. out
 *   lse            device float [B, Hq, N]: region `lse` of the forward call's workspace (ln of the shared normaliser)
 *   sel_idx        device int32 [B, Hq, N/C, lambda]: the forward call's index lists (its sel_idx, or region `sel`
 *                  of its workspace); may be NULL when lambda = 0 or N < C.  Entries outside their chunk are ignored
 *   dq, dk, dv     device, dtype, strided like q, k, v: gradients (dk, dv summed over the query heads of a kv head)
 *   dg             device, dtype, strided like g; given exactly when g is.  With gate_activation = 1 it is the
 *                  gradient w.r.t. the pre-activation
 *   dWq, dWk       device FLOAT [Hq, d, d_f]; dbq, dbk device FLOAT [Hq, d_f], given exactly when bq, bk are.
 *                  Parameter gradients are sums over every token of the batch and are returned in fp32
 *   workspace      device scratch of at least still_bwd_workspace_bytes(p) bytes
 *
 * Covers budget_policy 0 (with or without max_retained), both selection modes, both gate modes; d = 64 or 128 in
 * bf16, d = 64 in fp32; not right-padded batches (seq_len must be NULL).  dk, dv and the parameter gradients are
 * accumulated with floating-point atomic adds: results are reproducible to rounding, not bit for bit.
 * Validation on the host before any launch, as everywhere.
 */
typedef struct still_bwd_ws_layout {
  size_t fwd;      /* a forward workspace (still_ws_layout_t offsets apply from here): the states are rebuilt   */
  size_t e_row;    /* float [B, Hq, N]        E_t = exp(-lse_t)                                               */
  size_t delta;    /* float [B, Hq, N]        dout_t . out_t                                                  */
  size_t ed;       /* float [B, Hq, N]        E_t * delta_t                                                   */
  size_t a;        /* dtype [B, Hq, N, d]     E_t (gate_t * dout_t)                                           */
  size_t phi_q;    /* dtype [B, Hq, N, 2*d_f] feature map of the queries                                      */
  size_t phi_k;    /* dtype [B, Hq, N, 2*d_f] feature map of the keys, zero for the selected tokens           */
  size_t uq, uk;   /* float [B, Hq, N, d_f]   rescaled pre-activations u of Sec. 3.2                          */
  size_t stq, stk; /* float [B, Hq, N, 2]     |x|, |f(x)|                                                     */
  size_t nraw;     /* float [B, Hq, N, d]     phi_q S (the ungated linear numerator)                          */
  size_t gq;       /* float [B, Hq, N, 2*d_f] S A_t                                                           */
  size_t dphi_k;   /* float [B, Hq, N, 2*d_f] dS v_j                                                          */
  size_t ds;       /* dtype [B, Hq, ceil(N/C), 2*d_f, d]  gradient of the state the rows of chunk c+2 and later read */
  size_t dz;       /* float [B, Hq, ceil(N/C), 2*d_f]     likewise for z                                       */
  size_t dfq, dfk; /* dtype [B, Hq, N, d_f]   gradient of f(x)                                                */
  size_t dq32;     /* float [B, Hq, N, d]                                                                     */
  size_t dk32, dv32; /* float [B, Hkv, N, d]                                                                  */
  size_t cxq, cxk; /* float [B, Hq, N]        coefficient of x in its own gradient (the norm |x| of Sec. 3.2)   */
  size_t qt, dot;  /* dtype [B, Hq, d, Npad]  q and dout transposed, zero padded                              */
  size_t kt;       /* dtype [B, Hkv, d, Npad] k transposed                                                    */
  size_t kret;     /* dtype [B, Hq, cap, d]   retained keys in routing order                                  */
  size_t krett;    /* dtype [B, Hq, d, cap]   the same, transposed                                            */
  size_t total;
  int32_t n_pad_t; /* Npad of the three transposed copies above (64 more than the forward workspace's)         */
  int32_t cap_t;   /* cap of the two retained-key copies (likewise)                                           */
} still_bwd_ws_layout_t;
STILL_API size_t still_bwd_workspace_bytes(const still_params_t* p);
STILL_API still_status_t still_bwd_workspace_layout(const still_params_t* p, still_bwd_ws_layout_t* layout);
STILL_API still_status_t still_hybrid_attn_bwd(const still_params_t* p,
                                     const void* q, const void* k, const void* v, const void* g,
                                     const void* Wq, const void* bq, const void* Wk, const void* bk,
                                     const void* out, const void* dout, const float* lse, const int32_t* sel_idx,
                                     void* dq, void* dk, void* dv, void* dg,
                                     float* dWq, float* dbq, float* dWk, float* dbk,
                                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * Attention map of the operator, for inspection and for the first training stage of Sec. 4.1 (which compares it
 * with the teacher's softmax map): map_out[b, hq, t, j] = weight of v_j in row t under the shared normaliser of the
 * Sec. 3.3 output equation: exp(scale q_t.k_j - lse_t) for the keys the softmax branch sees (local span, retained
 * tokens), phi_q(q_t).phi_k(k_j) exp(-lse_t) for the tokens that went to the linear state, 0 for j > t.  Every row
 * sums to one; with a gate of ones out = map v (the per-channel gate scales the linear part of the numerator only
 * and is not part of a scalar map).  map_out: device FLOAT [B, Hq, N, N] (quadratic in N: meant for training-length
 * sequences); lse, sel_idx as for still_hybrid_attn_bwd; workspace: at least still_bwd_workspace_bytes(p) bytes.
 * Same coverage and validation as the backward pass.
 */
STILL_API still_status_t still_attention_map(const still_params_t* p, const void* q, const void* k,
                                   const void* Wq, const void* bq, const void* Wk, const void* bk,
                                   const float* lse, const int32_t* sel_idx, float* map_out,
                                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * Backward of the attention map w.r.t. the feature-map parameters: given dmap = d loss / d map (device FLOAT
 * [B, Hq, N, N]; entries above the diagonal are ignored) and the map itself (as written by still_attention_map for the
 * same inputs), returns dWq, dWk (device FLOAT [Hq, d, d_f]) and dbq, dbk (device FLOAT [Hq, d_f], given exactly when
 * bq, bk are), with q, k and the routing held fixed: what the first training stage of Sec. 4.1 updates (q and k come
 * from the frozen teacher there).  map_tj = a_tj / s_t with s_t the row's sum, so da_tj = (dmap_tj - <dmap_t, map_t>)
 * / s_t, and only the pairs owned by the linear branch depend on the parameters, through phi_q(q_t) . phi_k(k_j).
 * workspace: at least still_attention_map_bwd_workspace_bytes(p) bytes (a backward workspace plus one [B, Hq, N, N]
 * matrix in the storage type).  Same coverage and validation as the backward pass; sums with atomic adds.
 */
STILL_API size_t still_attention_map_bwd_workspace_bytes(const still_params_t* p);
STILL_API still_status_t still_attention_map_bwd(const still_params_t* p, const void* q, const void* k,
                                   const void* Wq, const void* bq, const void* Wk, const void* bk,
                                   const float* lse, const int32_t* sel_idx, const float* map, const float* dmap,
                                   float* dWq, float* dbq, float* dWk, float* dbk,
                                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * Rotary position embedding of q and k, in place: a pre-pass for callers whose q and k are not rotated yet (the
 * paper converts Llama-family layers, which rotate q and k before attention; nothing in the method depends on it, and
 * every other entry point takes q and k as they are).  Channel pair (i, i + d/2) of the token at position pos turns
 * by the angle pos * base^(-2 i / d) (the half-split pairing of those checkpoints); pos = pos0[b] + t for token t of
 * sequence b (pos0: device int32 [B], or NULL for zeros), so a decode step rotates its one new token with N = 1 and
 * pos0 = the token's index.  q: device, dtype, [B, N, Hq, d]; k: [B, N, Hkv, d]; either may be NULL.  Read from `p`:
 * B, N, Hq, Hkv, d (even), dtype, the q and k strides.  Angles, sines and cosines are computed in double (an fp32
 * angle of thousands of radians is only good to 1e-4), the rotation in fp32.
 */
STILL_API still_status_t still_rope_apply(const still_params_t* p, void* q, void* k, const int32_t* pos0, float base,
                                          void* stream);

#ifdef __cplusplus
}
#endif
#endif /* STILL_H */

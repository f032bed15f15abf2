/*
 * lola.h - C ABI of the MI355X (gfx950) implementation of one LoLA attention layer
 * (LoLA: Low-Rank Linear Attention with Sparse Caching, arxiv 2505.23666).
 *
 * The library owns no memory and never synchronises: every pointer below is a DEVICE pointer
 * (unless marked host) to caller-owned, contiguous, row-major memory aligned to 16 bytes, and
 * every call only enqueues kernels on `stream` (a hipStream_t passed as void*; NULL is the default
 * stream).  The one exception is opt-in: with lola_config.prefill_overlap = 1, lola_prefill may also
 * use one second stream per device that the library creates on first use, forks from `stream` and
 * joins back into it with events before the call returns, on every path (see lola_prefill;
 * lola_release_streams destroys it).  With prefill_overlap = 0 the library holds no state at all.
 * Errors: arguments, shapes, alignment, workspace size and whether a kernel exists for the
 * configuration are all checked on the host before anything is launched, so every status other
 * than LOLA_OK and LOLA_ERR_HIP means that nothing was enqueued and the memories are untouched.
 * LOLA_ERR_HIP means that hipGetLastError reported an error after one of the call's launches:
 * earlier launches of the call stay enqueued and the memories are then undefined.  An error that
 * the caller's own earlier HIP calls left pending is reported (and cleared) the same way.
 * Calls on distinct states are independent; calls on one state must be ordered by the caller
 * (same stream, or events).
 *
 * Notation (paper, Sec. 2-3): B batch, Hq query heads, Hkv key/value heads (Hq % Hkv == 0, query
 * head h reads kv head h / (Hq/Hkv)), d = head_dim = d_k = d_v, D = feat_dim (phi: R^d -> R^D,
 * D even, m = D/2 learned projections), eta = window, lambda = sparse_budget, C = chunk.
 * One "stream of memories" exists per (batch, kv head): the recurrent state (H, s), the sliding
 * window (last min(n, eta) pairs) and the sparse cache (<= lambda pairs with the largest
 * self-recall error).  Invariant at every call boundary: each of the n tokens seen so far lives in
 * exactly one of window, sparse cache, or (H, s).
 */
#ifndef LOLA_H
#define LOLA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LOLA_OK = 0,
    LOLA_ERR_NULL = -1,        /* a required pointer is NULL */
    LOLA_ERR_SHAPE = -2,       /* a size is out of range or inconsistent */
    LOLA_ERR_DTYPE = -3,       /* unknown dtype / phi_kind value */
    LOLA_ERR_ALIGN = -4,       /* a pointer is not 16-byte aligned */
    LOLA_ERR_UNSUPPORTED = -5, /* valid request this build has no kernel for */
    LOLA_ERR_WORKSPACE = -6,   /* workspace missing or smaller than the stated minimum */
    LOLA_ERR_HIP = -7,         /* a HIP launch reported an error */
    LOLA_ERR_TOO_LARGE = -8    /* lola_prefill_noalloc: the call needs more scratch than the library holds */
} lola_status;

enum { LOLA_F32 = 0, LOLA_BF16 = 1 };
/* Feature map, Sec. 2.3 eq. (feature_map): z = W^T x in R^m.
 * LOLA_PHI_EXP is the paper's form [exp(z), exp(-z)]; LOLA_PHI_SOFTMAX is the bounded form
 * [softmax(z), softmax(-z)] the benchmark configurations prescribe. */
enum { LOLA_PHI_SOFTMAX = 0, LOLA_PHI_EXP = 1 };
/* Restricted-query ablation (appendix "Sparse Cache & Linear Attention Ablation"): the memories are
 * updated as usual, but the queries do not read the hidden state and / or the sparse cache. */
enum { LOLA_HIDE_STATE = 1, LOLA_HIDE_SPARSE = 2 };
/* What ranks the eligible pairs.  LOLA_SCORE_SRE is the method's self-recall error (Sec. 3, eq. score).
 * The others are the query-dependent scores of the scoring ablation (Sec. 4, appendix "scoring
 * ablation"): Score(k_i) = sum over the eta queries t = i .. i+eta-1 that see k_i in the sliding window,
 * and over the query heads of its group, of
 *     (w - a)^2 | |w - a| | a / w | w,    w = exp(scale q_t.k_i), a = phi(q_t).phi(k_i).
 * A pair's sum is final when it leaves the window and stays with it in the sparse cache; the lambda
 * largest stay (ties: lower token index), as with the self-recall error.  These kinds run on the
 * shape-generic kernels and need queries: an update-only lola_prefill returns LOLA_ERR_UNSUPPORTED. */
enum { LOLA_SCORE_SRE = 0, LOLA_SCORE_WERR_SQ = 1, LOLA_SCORE_WERR_ABS = 2, LOLA_SCORE_OVEREST = 3, LOLA_SCORE_ATTN = 4 };

typedef struct {
    int32_t batch, n_q_heads, n_kv_heads;
    int32_t head_dim;      /* d: 32, 64, 128 or 256 */
    int32_t feat_dim;      /* D: even, 2..512 */
    int32_t window;        /* eta >= 0 */
    int32_t sparse_budget; /* lambda >= 0 */
    int32_t chunk;         /* C >= 1, prefill only */
    int32_t dtype;         /* LOLA_F32 | LOLA_BF16: storage type of q, k, v, Wq, Wk and cached K, V */
    int32_t out_dtype;     /* LOLA_F32 | LOLA_BF16: storage type of `out` */
    int32_t phi_kind;      /* LOLA_PHI_SOFTMAX | LOLA_PHI_EXP */
    float softmax_scale;   /* logit scale; <= 0 selects 1/sqrt(head_dim) (Sec. 2.1) */
    int32_t fold_defer;    /* 0: every fold is applied to H and s in memory at once.
                              R = 8: deferred folds (see lola_state.pend_*); accepted only where the fused
                              generation-step kernel exists (bf16, head_dim 128, feat_dim 128, window 64,
                              sparse_budget 64 or 128, at most 4 query heads per kv head), else LOLA_ERR_UNSUPPORTED */
    int32_t query_hide;    /* 0, or LOLA_HIDE_STATE | LOLA_HIDE_SPARSE bits: terms left out of the numerator
                              and the denominator of every output (lola_prefill and lola_decode_step) */
    int32_t score_kind;    /* LOLA_SCORE_*; anything but LOLA_SCORE_SRE excludes fold_defer */
    int32_t prefill_overlap; /* 0: lola_prefill enqueues on `stream` only.  1: it may run the outputs of a piece of the
                              call on the library's second stream beside the state evolution of the next piece */
} lola_config;

/* The memories of a layer.  H and s are always fp32 (Sec. 2.2, eq. recurrent_update). */
typedef struct {
    float *H;          /* [B, Hkv, d, D]      H^T: H[c][f] = sum over folded pairs of v[c] phi(k)[f]
                          (stored value-major so that the feature index, which every read contracts
                          over, is contiguous) */
    float *s;          /* [B, Hkv, D]         s = sum over folded pairs of phi(k) */
    void *win_k;       /* [B, Hkv, eta, d]    ring buffer: token t sits in slot t % eta */
    void *win_v;       /* [B, Hkv, eta, d] */
    void *sp_k;        /* [B, Hkv, lambda, d] sparse cache, slots [0, sp_count) in use, unordered */
    void *sp_v;        /* [B, Hkv, lambda, d] */
    int32_t *sp_idx;   /* [B, Hkv, lambda]    token index held by each slot, -1 = empty */
    int32_t *sp_count; /* [B, Hkv] */
    int64_t *n_tokens; /* [B, Hkv]            tokens consumed so far (equal across kv heads of a sequence) */
    /* Deferred folds (fold_defer = R > 0; NULL otherwise).  The sums of eq. recurrent_update are
     * associative, so a generation step may keep its folded pair in a short list instead of
     * rewriting H: the true state is
     *     H_true = H + sum_{p < pend_count} pend_v[p] pend_phi[p]^T   (in the H^T layout above),
     *     s_true = s + sum_{p < pend_count} pend_phi[p],
     * and every entry point computes with H_true, s_true.  The generation step that finds R pairs
     * listed writes H_true, s_true back (without its own fold) and starts a new list with its own
     * pair; lola_prefill and lola_state_flush write back and empty the list on entry.  Read H or s
     * directly only after lola_state_flush. */
    float *pend_phi;     /* [B, Hkv, R, D]  phi(k) of the listed pairs, fp32 */
    float *pend_v;       /* [B, Hkv, R, d]  their values, fp32 */
    int32_t *pend_count; /* [B, Hkv]        pairs listed, 0 .. R */
    /* Query-dependent scores (score_kind != LOLA_SCORE_SRE; NULL otherwise, except that sp_score may be
     * given with LOLA_SCORE_SRE too: it is then scratch of lola_decode_step, lola_step_scratch_bytes(cfg)
     * bytes whose contents mean nothing between calls, never read before written, not touched by
     * lola_state_init.  With it, at the run-time-parameter shapes and with few streams (batch *
     * n_kv_heads <= 128 for the update at lambda >= 512, <= 85 for the outputs at window + lambda > 480), the
     * step spreads a stream's work over several workgroups: the cached pairs' scores (same bits as
     * without it) and the outputs' sums over the keys (same result up to the order of the fp32 sums).
     * Calls on states that share one scratch must not overlap. */
    float *win_score;    /* [B, Hkv, eta]     sum gathered so far by the pair in each ring slot */
    float *sp_score;     /* [B, Hkv, lambda]  final sum of the pair in each sparse slot */
} lola_state;

/* Bytes of each state field in the order of the struct (host output, 14 entries; fields of an
 * option that is off are 0); returns their sum, or 0 if the configuration is invalid or
 * unsupported. */
size_t lola_state_bytes(const lola_config *cfg, size_t field_bytes[14]);

/* Bytes of the optional scratch of lola_decode_step (lola_state.sp_score with LOLA_SCORE_SRE, see there);
 * 0 if the configuration is invalid or the step has no use for one. */
size_t lola_step_scratch_bytes(const lola_config *cfg);

/* Workspace of lola_prefill for T tokens: returns the size with which all chunks are processed in
 * one pass; *min_bytes (host, may be NULL) receives the smallest size accepted (the chunks are then
 * processed in several passes).  0 if the configuration is invalid.  with_outputs = 0 sizes the
 * update-only call (q == out == NULL). */
size_t lola_prefill_workspace_bytes(const lola_config *cfg, int32_t T, int32_t with_outputs, size_t *min_bytes);

/* Empty memories: H = 0, s = 0, window and sparse cache empty (appendix "Algorithm Pseudo-Code",
 * init).  Cached K, V rows are zeroed too so that a state is a deterministic function of its inputs. */
lola_status lola_state_init(const lola_config *cfg, const lola_state *st, void *stream);

/* Applies the listed pairs of every stream to H and s in memory and empties the lists (a no-op
 * without deferred folds): afterwards H = H_true, s = s_true (Sec. 2.2, eq. recurrent_update). */
lola_status lola_state_flush(const lola_config *cfg, const lola_state *st, void *stream);

/*
 * Chunkwise prefill of T >= 0 tokens per sequence (Sec. 3 "Chunkwise Inference"; appendix
 * update_chunk).  T == 0 returns LOLA_OK without looking at the token or workspace pointers.
 * For each chunk of C tokens (the last may be shorter):
 *   1. every query t of the chunk, every query head:
 *        y_t = [phi(q_t)^T H + sum_i exp(scale q_t.k_i) v_i] / [phi(q_t)^T s + sum_i exp(scale q_t.k_i)]
 *      with i over the sparse cache, the window and the tokens <= t of the chunk, all memories as
 *      they stood when the chunk began (Sec. 3, y_t equation with the chunk sharing one state);
 *   2. the chunk joins the window; the pairs that no longer fit in eta are, together with the
 *      sparse cache, scored by self-recall error ||phi(k)^T H / phi(k)^T s - v||_2 (eq. score, with
 *      the state before this update; recall = 0 while nothing was folded); the lambda largest stay
 *      in the sparse cache (ties: lower token index stays), the rest are folded:
 *      H += phi(k) v^T, s += phi(k).  While the candidates number <= lambda all are cached unscored.
 * q   [B, Hq, T, d], k, v [B, Hkv, T, d], out [B, Hq, T, d] (out_dtype), Wq [Hq, m, d], Wk [Hkv, m, d]:
 *   row j of a head's matrix is the projection vector w_j of eq. (feature_map), so z_j = w_j . x.
 * q == out == NULL updates the memories without producing outputs (Wq is then ignored).
 * sel_trace: NULL, or int32 [B, Hkv, ceil(T/C), lambda] receiving the token indices held by the
 *   sparse cache after each chunk's update (slot order, -1 = empty slot).
 * workspace: see lola_prefill_workspace_bytes.  Contents are scratch; calls sharing a workspace
 *   must be ordered.
 * May be called repeatedly (the memories carry over) and be followed by lola_decode_step.
 * Streams: with prefill_overlap = 1, few streams of memories (B * Hkv <= 128) and enough output work, the MFMA
 *   kernels cut a pass into up to 8 pieces (each half as long as the one before) and run the outputs of a piece on the library's second stream
 *   beside the state evolution of the next piece; `stream` waits for that work before the call's
 *   last kernel, so work the caller enqueues on `stream` afterwards sees every output.  While
 *   `stream` is under graph capture, or if the second stream cannot be created, everything stays
 *   on `stream`.  Results do not depend on which way a call ran.  Host threads may call
 *   concurrently; the second stream is shared and guarded by a lock held while a call enqueues.
 * Token indices are int32: n_tokens + T must stay below 2^31.
 */
lola_status lola_prefill(const lola_config *cfg, const lola_state *st,
                         const void *q, const void *k, const void *v,
                         const void *Wq, const void *Wk, int32_t T, void *out,
                         int32_t *sel_trace, void *workspace, size_t workspace_bytes, void *stream);

/*
 * lola_prefill for callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same results and same checks as lola_prefill, without the workspace: the
 * scratch is an array of lola_noalloc_scratch_bytes() = 64 MiB in the library's own device data, one copy per GPU,
 * held until the process ends.  The call allocates nothing, frees nothing, creates no stream or event (it stays on
 * `stream`, whatever prefill_overlap says) and never synchronises; the array's device address is looked up on the
 * first call on each device.  A call whose smallest workspace (lola_prefill_workspace_bytes, *min_bytes) exceeds the
 * array returns LOLA_ERR_TOO_LARGE with nothing enqueued; a call that fits but is large is processed in several
 * passes over its chunks, as lola_prefill does with a small workspace.  The scratch need not be cleared between
 * calls (every pass writes what it reads).  All calls on one GPU share the array: the caller orders them (one
 * stream, or events); calls that overlap on one GPU race.
 */
lola_status lola_prefill_noalloc(const lola_config *cfg, const lola_state *st,
                                 const void *q, const void *k, const void *v,
                                 const void *Wq, const void *Wk, int32_t T, void *out,
                                 int32_t *sel_trace, void *stream);

/* Size of the static scratch of lola_prefill_noalloc (host value, the same on every device). */
size_t lola_noalloc_scratch_bytes(void);

/*
 * One generation step for every sequence (Sec. 3, E_t / G_t / S_t / y_t equations; appendix
 * update + attend).  Order: (1) the new pair enters the window; once the window holds more than
 * eta pairs the oldest leaves; (2) the leaving pair and the sparse cache form the eligible set,
 * scored and cut to lambda exactly as in lola_prefill step 2 (a single pair is folded in steady
 * state); (3) the outputs of all query heads are computed with the updated memories, the window
 * including the new token.
 * q [B, Hq, d], k, v [B, Hkv, d], out [B, Hq, d] (out_dtype).
 * With deferred folds the step's outputs, cache and window are the same; only where the folded
 * pair is kept differs (see lola_state).
 */
lola_status lola_decode_step(const lola_config *cfg, const lola_state *st,
                             const void *q, const void *k, const void *v,
                             const void *Wq, const void *Wk, void *out, void *stream);

/* Destroys the second streams and events that lola_prefill calls with prefill_overlap = 1 created (all
 * devices); a later such call creates them again.  The caller makes sure that no lola_prefill call is
 * running on another host thread.  Synchronises with the second streams only.  A no-op if none exists. */
void lola_release_streams(void);

/* Human-readable name of a status code (host string, never NULL). */
const char *lola_status_str(lola_status s);

/* Name of the kernel family the given call would use; host string.  "mfma": every kernel of the call is an
 * MFMA kernel; "mixed" (lola_prefill only): the state evolution runs on the shape-generic kernel, the outputs on an
 * MFMA kernel; "generic": shape-generic kernels.  which: 0 = lola_prefill, 1 = lola_decode_step. */
const char *lola_kernel_path(const lola_config *cfg, int32_t which);

#ifdef __cplusplus
}
#endif
#endif /* LOLA_H */

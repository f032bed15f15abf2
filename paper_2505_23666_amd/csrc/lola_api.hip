// C ABI of the LoLA layer library (see include/lola.h): host-side validation, workspace carving
// and kernel dispatch.  Nothing here allocates or synchronises.
#include "../../include/lola.h"
#include <type_traits>
#include <mutex>
#include "generic_kernels.h"
#include "decode_mfma.h"
#include "prefill_mfma.h"

using namespace lola;

// Scratch of lola_prefill_noalloc: one copy per GPU, held from the moment the library's code is loaded there until
// the process ends.  In host code this name is only a handle for hipGetSymbolAddress; the device address is looked up
// once per device (noalloc_scratch below) and that pointer is what kernels receive.
#define LOLA_NOALLOC_SCRATCH_BYTES (64u << 20)
static __device__ __align__(256) unsigned char scratch[LOLA_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr size_t ALIGN = 256;
inline size_t up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }
inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
inline size_t esize(int dtype) { return dtype == LOLA_BF16 ? 2 : 4; }

constexpr size_t LDS_LIMIT = 64 * 1024 - 256;   // static workgroup limit minus the kernels' few static words

constexpr int DEFER_R = 8;   // pairs a stream may list before the generation step writes its state back

// The fused MFMA generation step covers the Llama-8B head shape with bf16 storage.
bool fast_decode_ok(const lola_config *c) {
    return c->dtype == LOLA_BF16 && (c->head_dim == 128 || c->head_dim == 64) && c->feat_dim == 128 && c->window == 64 &&
           (c->sparse_budget == 128 || c->sparse_budget == 64) && c->n_q_heads / c->n_kv_heads <= 4 &&
           c->score_kind == LOLA_SCORE_SRE;
}

// Shapes at which the outputs of the generation step come from the MFMA output kernel (any window and sparse budget up
// to its key limit, 128 or 256 features), the shape-generic kernel keeping the update of the memories ...
bool wide_step_out_ok(const lola_config *c) {
    return c->dtype == LOLA_BF16 && (c->head_dim == 128 || c->head_dim == 64) && (c->feat_dim == 128 || c->feat_dim == 256) &&
           c->window >= 1 && !fast_decode_ok(c) && c->n_q_heads / c->n_kv_heads <= 8 &&
           c->sparse_budget + c->window <= (c->n_q_heads / c->n_kv_heads <= 4 ? fast::STEP_OUT_NKMAX : fast::STEP_OUT_NKMAX / 2);
}
// ... and at which the streams in steady state are updated by the MFMA update kernel ahead of it (sparse budgets in
// multiples of 64).
bool wide_decode_ok(const lola_config *c) {
    return wide_step_out_ok(c) && c->sparse_budget >= 64 && c->sparse_budget % 64 == 0 && c->sparse_budget <= fast::STEP_UPDATE_LAMMAX;
}

// Floats per stream of the generation step's optional scratch: the cached pairs' scores, later the output kernel's
// shares (both launches of a step use it one after the other).
size_t step_scratch_floats(const lola_config *c) {
    if (c->score_kind != LOLA_SCORE_SRE || !wide_step_out_ok(c)) return 0;
    const int G = c->n_q_heads / c->n_kv_heads <= 4 ? 4 : 8;
    const size_t shares = (size_t)fast::STEP_OUT_PARTS_MAX * (G * c->head_dim + 2 * G);
    return std::max(shares, (size_t)c->sparse_budget);
}

lola_status check_config(const lola_config *c) {
    if (!c) return LOLA_ERR_NULL;
    if (c->dtype != LOLA_F32 && c->dtype != LOLA_BF16) return LOLA_ERR_DTYPE;
    if (c->out_dtype != LOLA_F32 && c->out_dtype != LOLA_BF16) return LOLA_ERR_DTYPE;
    if (c->phi_kind != LOLA_PHI_SOFTMAX && c->phi_kind != LOLA_PHI_EXP) return LOLA_ERR_DTYPE;
    if (c->batch < 1 || c->n_kv_heads < 1 || c->n_q_heads < c->n_kv_heads || c->n_q_heads % c->n_kv_heads)
        return LOLA_ERR_SHAPE;
    if (c->head_dim != 32 && c->head_dim != 64 && c->head_dim != 128 && c->head_dim != 256) return LOLA_ERR_SHAPE;
    if (c->feat_dim < 2 || c->feat_dim > 512 || (c->feat_dim & 1)) return LOLA_ERR_SHAPE;
    if (c->window < 0 || c->sparse_budget < 0 || c->chunk < 1) return LOLA_ERR_SHAPE;
    if (c->window > 4096 || c->sparse_budget > 4096 || c->chunk > 1024) return LOLA_ERR_SHAPE;
    // streams, query heads and sequences index the y and z dimensions of some launch grids (limit 65535)
    if ((long long)c->batch * c->n_kv_heads > 65535 || c->n_q_heads > 65535) return LOLA_ERR_SHAPE;
    if (c->prefill_overlap != 0 && c->prefill_overlap != 1) return LOLA_ERR_SHAPE;
    if (c->query_hide < 0 || c->query_hide > 3) return LOLA_ERR_SHAPE;
    if (c->score_kind < LOLA_SCORE_SRE || c->score_kind > LOLA_SCORE_ATTN) return LOLA_ERR_DTYPE;
    if (c->fold_defer != 0 && c->fold_defer != DEFER_R) return LOLA_ERR_SHAPE;
    if (c->fold_defer != 0 && !fast_decode_ok(c)) return LOLA_ERR_UNSUPPORTED;
    return LOLA_OK;
}

Dims make_dims(const lola_config *c) {
    Dims dm;
    dm.B = c->batch; dm.Hq = c->n_q_heads; dm.Hkv = c->n_kv_heads; dm.g = dm.Hq / dm.Hkv;
    dm.d = c->head_dim; dm.D = c->feat_dim; dm.m = dm.D / 2;
    dm.eta = c->window; dm.lam = c->sparse_budget; dm.C = c->chunk;
    dm.phi_kind = c->phi_kind;
    dm.scale = c->softmax_scale > 0.f ? c->softmax_scale : 1.0f / sqrtf((float)c->head_dim);
    dm.hide = c->query_hide;
    dm.score_kind = c->score_kind;
    return dm;
}

lola_status check_state(const lola_config *c, const lola_state *st) {
    if (!st || !st->H || !st->s || !st->sp_count || !st->n_tokens) return LOLA_ERR_NULL;
    if (c->window > 0 && (!st->win_k || !st->win_v)) return LOLA_ERR_NULL;
    if (c->sparse_budget > 0 && (!st->sp_k || !st->sp_v || !st->sp_idx)) return LOLA_ERR_NULL;
    const void *ps[] = {st->H, st->s, st->win_k, st->win_v, st->sp_k, st->sp_v, st->sp_idx, st->sp_count, st->n_tokens};
    for (const void *p : ps) if (p && misaligned(p)) return LOLA_ERR_ALIGN;
    if (c->fold_defer) {
        if (!st->pend_phi || !st->pend_v || !st->pend_count) return LOLA_ERR_NULL;
        if (misaligned(st->pend_phi) || misaligned(st->pend_v) || misaligned(st->pend_count)) return LOLA_ERR_ALIGN;
    }
    if (c->score_kind != LOLA_SCORE_SRE) {
        if ((c->window > 0 && !st->win_score) || (c->sparse_budget > 0 && !st->sp_score)) return LOLA_ERR_NULL;
        if (misaligned(st->win_score) || misaligned(st->sp_score)) return LOLA_ERR_ALIGN;
    } else if (st->sp_score && misaligned(st->sp_score)) return LOLA_ERR_ALIGN;   // (optional scratch of the generation step)
    return LOLA_OK;
}

// H += sum_p v_p phi_p^T, s += sum_p phi_p over the listed pairs of each stream; the list is emptied
__global__ __launch_bounds__(256) void flush_pending_kernel(float *H, float *s, float *pend_phi, float *pend_v,
                                                            int32_t *pend_count, int d, int D, int R) {
    const int si = blockIdx.x;
    const int cnt = pend_count[si];
    if (cnt == 0) return;
    const float *pphi = pend_phi + (size_t)si * R * D, *pv = pend_v + (size_t)si * R * d;
    float *Hs = H + (size_t)si * d * D, *ss = s + (size_t)si * D;
    for (int e = threadIdx.x; e < d * D; e += 256) {
        const int c = e / D, f = e - c * D;
        float acc = Hs[e];
        for (int p = 0; p < cnt; p++) acc = fmaf(pv[p * d + c], pphi[p * D + f], acc);
        Hs[e] = acc;
    }
    for (int f = threadIdx.x; f < D; f += 256) {
        float acc = ss[f];
        for (int p = 0; p < cnt; p++) acc += pphi[p * D + f];
        ss[f] = acc;
    }
    __syncthreads();   // every thread has read the count
    if (threadIdx.x == 0) pend_count[si] = 0;
}

lola_status flush_pending(const lola_config *c, const lola_state *st, hipStream_t stream) {
    if (!c->fold_defer) return LOLA_OK;
    hipLaunchKernelGGL(flush_pending_kernel, dim3(c->batch * c->n_kv_heads), dim3(256), 0, stream, st->H, st->s,
                       st->pend_phi, st->pend_v, st->pend_count, c->head_dim, c->feat_dim, c->fold_defer);
    if (hipGetLastError() != hipSuccess) return LOLA_ERR_HIP;
    return LOLA_OK;
}

template <typename T>
State<T> make_state(const lola_state *st) {
    State<T> s;
    s.H = st->H; s.s = st->s;
    s.win_k = (T *)st->win_k; s.win_v = (T *)st->win_v; s.sp_k = (T *)st->sp_k; s.sp_v = (T *)st->sp_v;
    s.sp_idx = st->sp_idx; s.sp_count = st->sp_count; s.n_tokens = st->n_tokens;
    s.win_score = st->win_score; s.sp_score = st->sp_score;
    return s;
}

// rows per scoring tile of the generic kernels: as many as fit next to `fixed_floats` in LDS
int score_tile_rows(const Dims &dm, size_t fixed_floats, bool with_key_features = false) {
    size_t per_row = (size_t)(3 * dm.d + dm.D + 1) + (with_key_features ? dm.D : 0);
    size_t avail = LDS_LIMIT / 4;
    int rmin = generic::NT / dm.d > 1 ? generic::NT / dm.d : 1;
    if (avail < fixed_floats + per_row * rmin) return 0;
    size_t r = (avail - fixed_floats) / per_row;
    if (r > 32) r = 32;
    return (int)r < rmin ? 0 : (int)r;
}
size_t decode_fixed_floats(const Dims &dm) {
    return (size_t)(dm.lam + 1) + 2 * dm.d + (dm.lam + dm.eta) + 3 * generic::NW + 8 + (dm.score_kind ? 2 * dm.eta : 0);
}
// keys (= queries) per tile of the query-dependent score kernel of the prefill
int band_tile_rows(const Dims &dm) {
    size_t r = (LDS_LIMIT / 4) / (size_t)(2 * (dm.d + dm.D) + 1);
    return (int)(r > 16 ? 16 : r);
}
size_t scan_fixed_floats(const Dims &dm) { return (size_t)4 * (dm.lam + dm.C) + 2 * dm.C + 8; }
int attend_tile_queries(const Dims &dm) {
    size_t per_q = (size_t)dm.d + dm.D + (dm.lam + dm.eta + dm.C) + 3;
    size_t q = (LDS_LIMIT / 4) / per_q;
    if (q > 16) q = 16;
    return (int)q;
}

#define LAUNCH_CHECK() do { if (hipGetLastError() != hipSuccess) return LOLA_ERR_HIP; } while (0)

// Whether the shape-generic prefill kernels can tile this configuration into LDS; asked before anything is enqueued.
lola_status prefill_feasible(const lola_config *c, bool want_out) {
    const Dims dm = make_dims(c);
    if (score_tile_rows(dm, scan_fixed_floats(dm)) <= 0) return LOLA_ERR_UNSUPPORTED;
    if (want_out && attend_tile_queries(dm) <= 0) return LOLA_ERR_UNSUPPORTED;
    if (dm.score_kind && band_tile_rows(dm) <= 0) return LOLA_ERR_UNSUPPORTED;
    return LOLA_OK;
}
lola_status decode_feasible(const lola_config *c) {
    if (c->dtype == LOLA_BF16 && fast_decode_ok(c)) return LOLA_OK;
    const Dims dm = make_dims(c);
    return score_tile_rows(dm, decode_fixed_floats(dm), dm.score_kind != 0) > 0 ? LOLA_OK : LOLA_ERR_UNSUPPORTED;
}

// The MFMA kernels of the prefill cover the Llama 8B and 1B head shapes (head_dim 128 / 64, 128 features) with
// chunk = window = 64.
// shapes of the MFMA prefill kernels; the output kernel serves every score kind (its inputs are the snapshots, whoever
// took them), the state-evolution kernel ranks by self-recall error only
bool fast_output_ok(const lola_config *c) {
    return c->dtype == LOLA_BF16 && (c->head_dim == 128 || c->head_dim == 64) && c->feat_dim == 128 && c->window == 64 && c->chunk == 64 &&
           (c->sparse_budget == 0 || c->sparse_budget == 64 || c->sparse_budget == 128 || c->sparse_budget == 256);
}
bool fast_attend_ok(const lola_config *c) { return fast_output_ok(c) && c->score_kind == LOLA_SCORE_SRE; }
// shapes of the MFMA output kernel with run-time window and sparse budget (any score kind: its inputs are the snapshots)
bool wide_output_ok(const lola_config *c) {
    return c->dtype == LOLA_BF16 && (c->head_dim == 128 || c->head_dim == 64) && (c->feat_dim == 128 || c->feat_dim == 256) &&
           c->chunk == 64 && c->sparse_budget <= 1024;
}

// shapes of the MFMA state-evolution kernel with run-time window and sparse budget (multiples of 64; it ranks by
// self-recall error only); the shapes of the specialised kernels above keep those
bool wide_scan_ok(const lola_config *c) {
    // (the compile-time shapes keep their own state-evolution kernel for the self-recall error; with the
    // query-dependent scores, which are given to the selection instead of being computed by it, they come here too)
    // (sparse budget 0: no selection, every leaving pair is folded; at window 64 the row-split kernel is faster)
    return wide_output_ok(c) && (!fast_output_ok(c) || (c->score_kind != LOLA_SCORE_SRE && c->sparse_budget > 0)) &&
           c->sparse_budget % 64 == 0 && c->window >= 64 && c->window % 64 == 0;
}

struct PrefillPlan {
    size_t off_prefK, off_prefV, off_sp_row, off_phiE, off_next, off_score, off_snap;   // byte offsets
    size_t snap_bytes_per_chunk;                                    // all streams, one chunk (snapshots + phi of its keys)
    size_t phik_bytes_per_chunk;
    size_t fixed_bytes;
};
PrefillPlan plan_prefill(const lola_config *c, int with_outputs, size_t Tn) {
    const size_t ns = (size_t)c->batch * c->n_kv_heads, es = esize(c->dtype);
    const size_t P = (size_t)c->sparse_budget + c->window, d = c->head_dim, D = c->feat_dim, lam = c->sparse_budget;
    PrefillPlan p;
    size_t off = 0;
    p.off_prefK = off; off += up(ns * P * d * es);
    p.off_prefV = off; off += up(ns * P * d * es);
    p.off_sp_row = off; off += up(ns * lam * 4);
    p.off_phiE = off; off += up(ns * (lam + c->chunk) * D * 4);
    p.off_next = off; off += up(ns * 4);
    p.off_score = off; if (c->score_kind != LOLA_SCORE_SRE) off += up(ns * ((size_t)c->window + Tn) * 4);
    p.off_snap = off;
    p.fixed_bytes = off;
    p.snap_bytes_per_chunk = with_outputs ? up(ns * D * d * 4) + up(ns * D * 4) + up(ns * (lam ? lam : 1) * 4) : 0;
    p.phik_bytes_per_chunk = (fast_attend_ok(c) || wide_scan_ok(c)) ? up(ns * (size_t)c->chunk * D * 4) : 0;   // phi of the chunk's keys, two bf16 parts
    p.snap_bytes_per_chunk += p.phik_bytes_per_chunk;
    return p;
}


template <int LAM, typename TO>
lola_status launch_fast_decode(const lola_config *c, const lola_state *st, const void *q, const void *k, const void *v,
                               const void *Wq, const void *Wk, void *out, hipStream_t stream) {
    fast::DecodeFastArgs<TO> a;
    a.st = make_state<bf16_t>(st);
    a.q = (const bf16_t *)q; a.k = (const bf16_t *)k; a.v = (const bf16_t *)v;
    a.Wq = (const bf16_t *)Wq; a.Wk = (const bf16_t *)Wk;
    a.out = (TO *)out;
    a.Hq = c->n_q_heads; a.Hkv = c->n_kv_heads;
    a.scale = make_dims(c).scale;
    a.phi_kind = c->phi_kind;
    a.hide = c->query_hide;
    a.g = c->n_q_heads / c->n_kv_heads;
    a.pend_phi = st->pend_phi; a.pend_v = st->pend_v; a.pend_count = st->pend_count;
    const dim3 grid(c->batch * c->n_kv_heads), block(256);
#define LOLA_DEC(RV, GD, DHV) hipLaunchKernelGGL((fast::decode_fast_kernel<LAM, 64, 4, RV, GD, DHV, TO>), grid, block, 0, stream, a)
    if (c->head_dim == 128) {
        // the benchmarked shape keeps the group size as a compile-time constant
        if (a.g == 4) { if (c->fold_defer) LOLA_DEC(DEFER_R, false, 128); else LOLA_DEC(0, false, 128); }
        else { if (c->fold_defer) LOLA_DEC(DEFER_R, true, 128); else LOLA_DEC(0, true, 128); }
    } else {
        if (c->fold_defer) LOLA_DEC(DEFER_R, true, 64); else LOLA_DEC(0, true, 64);
    }
#undef LOLA_DEC
    LAUNCH_CHECK();
    return LOLA_OK;
}

lola_status run_fast_decode(const lola_config *c, const lola_state *st, const void *q, const void *k, const void *v,
                            const void *Wq, const void *Wk, void *out, hipStream_t stream) {
    const bool f32o = c->out_dtype == LOLA_F32;
    if (c->sparse_budget == 128)
        return f32o ? launch_fast_decode<128, float>(c, st, q, k, v, Wq, Wk, out, stream)
                    : launch_fast_decode<128, bf16_t>(c, st, q, k, v, Wq, Wk, out, stream);
    return f32o ? launch_fast_decode<64, float>(c, st, q, k, v, Wq, Wk, out, stream)
                : launch_fast_decode<64, bf16_t>(c, st, q, k, v, Wq, Wk, out, stream);
}

template <typename T>
lola_status run_decode(const lola_config *c, const lola_state *st, const void *q, const void *k, const void *v,
                       const void *Wq, const void *Wk, void *out, hipStream_t stream) {
    generic::DecodeArgs<T> a;
    a.dm = make_dims(c);
    a.st = make_state<T>(st);
    a.q = (const T *)q; a.k = (const T *)k; a.v = (const T *)v; a.Wq = (const T *)Wq; a.Wk = (const T *)Wk;
    a.out = out;
    const size_t fixed = decode_fixed_floats(a.dm);
    const bool sk = a.dm.score_kind != 0;
    a.R = score_tile_rows(a.dm, fixed, sk);
    if (a.R <= 0) return LOLA_ERR_UNSUPPORTED;
    const size_t lds = 4 * (fixed + (size_t)a.R * (3 * a.dm.d + a.dm.D + 1 + (sk ? a.dm.D : 0)));
    dim3 grid(a.dm.B * a.dm.Hkv), block(generic::NT);
    a.no_out = 0;
    a.skip_steady = 0;
    bool wide_out = false;
    if constexpr (std::is_same<T, bf16_t>::value) {
        if (wide_decode_ok(c)) {
            // streams in steady state (window and cache full: scoring, arg-min, fold, slot replacement) by the MFMA update
            // kernel; the others (still filling) are left to the step kernel, which skips the steady ones
            fast::StepUpdateArgs ua;
            ua.st = a.st; ua.k = a.k; ua.v = a.v; ua.Wk = a.Wk;
            ua.Hkv = a.dm.Hkv; ua.lam = a.dm.lam; ua.eta = a.dm.eta; ua.phi_kind = a.dm.phi_kind;
            ua.scr_stride = (int)step_scratch_floats(c);
            // Few streams and several passes over the cached pairs: the scoring is split over `parts` workgroups per
            // stream (each at least one pass of 256 pairs, all of them resident at once), a second launch does the rest.
            // The scores travel through sp_score, which a self-recall-error state may carry as scratch.
            // Where the compute units suffice for one tile of 16 pairs per wavefront (lambda / 128 workgroups per stream),
            // the parts take single tiles instead of pairs of tiles.
            const int ns = a.dm.B * a.dm.Hkv, npass = a.dm.lam / 256;
            int parts = 1;
            bool single = false;
            if (!a.dm.score_kind && st->sp_score && npass >= 2 && 2 * ns <= 256) {
                single = a.dm.lam % 128 == 0 && ns * (a.dm.lam / 128) <= 256;
                parts = single ? a.dm.lam / 128 : std::min(npass, 256 / ns);
            }
            const dim3 grid1(ns, parts);
#define LOLA_UPD(DHV, DFV) do { if (a.dm.score_kind) hipLaunchKernelGGL((fast::step_update_wide_kernel<DHV, DFV, true>), grid, dim3(512), 0, stream, ua); \
                                else if (parts == 1) hipLaunchKernelGGL((fast::step_update_wide_kernel<DHV, DFV, false>), grid, dim3(512), 0, stream, ua); \
                                else { if (single) hipLaunchKernelGGL((fast::step_update_wide_kernel<DHV, DFV, false, 1, 1>), grid1, dim3(512), 0, stream, ua); \
                                       else hipLaunchKernelGGL((fast::step_update_wide_kernel<DHV, DFV, false, 1>), grid1, dim3(512), 0, stream, ua); \
                                       hipLaunchKernelGGL((fast::step_update_wide_kernel<DHV, DFV, false, 2>), grid, dim3(512), 0, stream, ua); } } while (0)
            if (c->head_dim == 128) { if (c->feat_dim == 256) LOLA_UPD(128, 256); else LOLA_UPD(128, 128); }
            else { if (c->feat_dim == 256) LOLA_UPD(64, 256); else LOLA_UPD(64, 128); }
#undef LOLA_UPD
            LAUNCH_CHECK();
            a.skip_steady = 1;
        }
        if (wide_step_out_ok(c)) {
            a.no_out = 1;
            wide_out = true;
        }
    }
    if (c->out_dtype == LOLA_F32) hipLaunchKernelGGL((generic::decode_kernel<T, float>), grid, block, lds, stream, a);
    else hipLaunchKernelGGL((generic::decode_kernel<T, bf16_t>), grid, block, lds, stream, a);
    LAUNCH_CHECK();
    if constexpr (std::is_same<T, bf16_t>::value) {
        if (wide_out) {   // the outputs from the updated memories (streams in any state)
            auto launch = [&](auto *o) {
                using TO = std::remove_pointer_t<decltype(o)>;
                fast::StepOutArgs<TO> oa;
                oa.st = a.st; oa.q = a.q; oa.Wq = a.Wq; oa.Wk = a.Wk; oa.out = (TO *)out; oa.score_kind = a.dm.score_kind;
                oa.Hq = a.dm.Hq; oa.Hkv = a.dm.Hkv; oa.g = a.dm.g; oa.lam = a.dm.lam; oa.eta = a.dm.eta;
                oa.phi_kind = a.dm.phi_kind; oa.hide = a.dm.hide; oa.scale = a.dm.scale;
                // Few streams: the keys in shares of at least 8 blocks of 32 on workgroups of their own, the linear part
                // on another, a small launch adds the shares up (they pass through the state's optional scratch).
                const int ns = a.dm.B * a.dm.Hkv, nblk = (a.dm.lam + a.dm.eta + 31) / 32;
                // The linear part reads W_q per query head and all of H^T: one workgroup per query head where the compute
                // units suffice for that and two shares of keys, else one workgroup for all heads.
                int kparts = 0, nlin = 1;
                if (!a.dm.score_kind && st->sp_score && 3 * ns <= 256 && nblk >= 16) {
                    const int total = std::min(fast::STEP_OUT_PARTS_MAX, 256 / ns);
                    if (total - a.dm.g >= 2) nlin = a.dm.g;
                    kparts = std::min(total - nlin, nblk / 8);
                }
                oa.part = st->sp_score; oa.part_stride = (int)step_scratch_floats(c); oa.nlin = nlin;
                const dim3 gridp(ns, kparts + nlin);
                const int Gv = oa.g <= 4 ? 4 : 8;
#define LOLA_OUT(DHV, DFV) do { if (kparts >= 2) { \
                                    if (oa.g <= 4) hipLaunchKernelGGL((fast::step_out_wide_kernel<DHV, DFV, TO, 4, true>), gridp, dim3(256), 0, stream, oa); \
                                    else hipLaunchKernelGGL((fast::step_out_wide_kernel<DHV, DFV, TO, 8, true>), gridp, dim3(256), 0, stream, oa); \
                                    hipLaunchKernelGGL((fast::step_out_combine_kernel<TO>), grid, dim3(256), 0, stream, oa, Gv, DHV, kparts + nlin); } \
                                else if (oa.g <= 4) hipLaunchKernelGGL((fast::step_out_wide_kernel<DHV, DFV, TO, 4>), grid, dim3(256), 0, stream, oa); \
                                else hipLaunchKernelGGL((fast::step_out_wide_kernel<DHV, DFV, TO, 8>), grid, dim3(256), 0, stream, oa); } while (0)
                if (c->head_dim == 128) { if (c->feat_dim == 256) LOLA_OUT(128, 256); else LOLA_OUT(128, 128); }
                else { if (c->feat_dim == 256) LOLA_OUT(64, 256); else LOLA_OUT(64, 128); }
#undef LOLA_OUT
            };
            if (c->out_dtype == LOLA_F32) launch((float *)nullptr); else launch((bf16_t *)nullptr);
            LAUNCH_CHECK();
        }
    }
    return LOLA_OK;
}

// Second stream of the prefill: one per device, created on first use at the default priority and kept until the process
// ends.  Calls from several host threads share it; the events keep every call's work ordered behind its own stream.
struct SideStream {
    static constexpr int NEV = 8;   // pieces per pass at most
    hipStream_t s;
    hipEvent_t fork[NEV], join;
};
#ifndef LOLA_SCAN_RT128
#define LOLA_SCAN_RT128 1
#endif
constexpr int SCAN_RT128 = LOLA_SCAN_RT128;   // row tiles of H^T per wavefront in the MFMA scan at head_dim 128
constexpr int CHIP_CUS = 256;                 // compute units of the MI355X
constexpr size_t OVERLAP_MAX_STREAMS = 128;   // beyond this many streams the serial evolution fills the chip by itself
constexpr int OVERLAP_MIN_PIECE = 8;          // chunks per piece on average at least.  The first piece, at least half of the
                                              // pass and so at least 8 chunks, is longer than the (256 + 64) / 64 chunks
                                              // after which the sparse cache of the MFMA shapes is full
constexpr size_t OVERLAP_MIN_WORK = 4096;     // output workgroups (in units of 64 head columns) per piece at least: below
                                              // this the restart of the evolution costs more than the overlap hides

std::mutex side_init_mu;   // creation of the per-device entries
std::mutex side_use_mu;    // held by a call from its first fork to its join: the events are shared

constexpr int MAX_DEV = 16;
SideStream side_table[MAX_DEV];
int side_state[MAX_DEV];   // 0 not created, 1 ready, -1 unavailable

// destroys every second stream and its events (the next call that wants one creates it again)
void release_side_streams() {
    std::lock_guard<std::mutex> lock(side_init_mu);
    int cur = -1;
    const bool have_cur = hipGetDevice(&cur) == hipSuccess;
    for (int dev = 0; dev < MAX_DEV; dev++) {
        if (side_state[dev] == 1 && hipSetDevice(dev) == hipSuccess) {
            SideStream &t = side_table[dev];
            (void)hipStreamSynchronize(t.s);
            for (int i = 0; i < SideStream::NEV; i++) (void)hipEventDestroy(t.fork[i]);
            (void)hipEventDestroy(t.join);
            (void)hipStreamDestroy(t.s);
        }
        side_state[dev] = 0;
    }
    if (have_cur) (void)hipSetDevice(cur);
    (void)hipGetLastError();
}

SideStream *side_stream(hipStream_t caller) {
    SideStream *table = side_table;
    int *state = side_state;
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(caller, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) {
        (void)hipGetLastError();
        return nullptr;          // under graph capture the call stays on the caller's stream
    }
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEV) return nullptr;
    std::lock_guard<std::mutex> lock(side_init_mu);
    if (state[dev] == 0) {
        SideStream &t = table[dev];
        bool ok = hipStreamCreateWithFlags(&t.s, hipStreamNonBlocking) == hipSuccess;
        for (int i = 0; ok && i < SideStream::NEV; i++) ok = hipEventCreateWithFlags(&t.fork[i], hipEventDisableTiming) == hipSuccess;
        ok = ok && hipEventCreateWithFlags(&t.join, hipEventDisableTiming) == hipSuccess;
        if (!ok) (void)hipGetLastError();
        state[dev] = ok ? 1 : -1;
    }
    return state[dev] == 1 ? &table[dev] : nullptr;
}

// outputs of the chunks [r0, r1) by the MFMA output kernels: the compile-time form where the shape has one, else the
// form with run-time window and sparse budget
void launch_output_kernel(const lola_config *c, const generic::PrefillArgs<bf16_t> &a, int r0, int r1, hipStream_t so) {
    generic::PrefillArgs<bf16_t> ao = a;
    ao.j0 = r0; ao.j1 = r1; ao.scan_mode = 0;
    const dim3 ga((unsigned)(r1 - r0), (unsigned)a.dm.Hq, (unsigned)a.dm.B);
    const bool f32o = c->out_dtype == LOLA_F32;
    if (!fast_output_ok(c)) {
#define LOLA_WIDE(DHV, DFV) do { if (f32o) hipLaunchKernelGGL((fast::attend_wide_kernel<DHV, DFV, float>), ga, dim3(256), 0, so, ao); \
                                 else hipLaunchKernelGGL((fast::attend_wide_kernel<DHV, DFV, bf16_t>), ga, dim3(256), 0, so, ao); } while (0)
        if (c->head_dim == 128) { if (c->feat_dim == 256) LOLA_WIDE(128, 256); else LOLA_WIDE(128, 128); }
        else { if (c->feat_dim == 256) LOLA_WIDE(64, 256); else LOLA_WIDE(64, 128); }
#undef LOLA_WIDE
        return;
    }
#define LOLA_ATT2(LAMV, DHV) do { if (f32o) hipLaunchKernelGGL((fast::attend_fast_kernel<LAMV, DHV, float>), ga, dim3(256), 0, so, ao); \
                                  else hipLaunchKernelGGL((fast::attend_fast_kernel<LAMV, DHV, bf16_t>), ga, dim3(256), 0, so, ao); } while (0)
#define LOLA_ATT(LAMV) do { if (c->head_dim == 128) LOLA_ATT2(LAMV, 128); else LOLA_ATT2(LAMV, 64); } while (0)
    if (c->sparse_budget == 0) LOLA_ATT(0); else if (c->sparse_budget == 64) LOLA_ATT(64);
    else if (c->sparse_budget == 128) LOLA_ATT(128); else LOLA_ATT(256);
#undef LOLA_ATT
#undef LOLA_ATT2
}

template <typename T>
lola_status run_prefill(const lola_config *c, const lola_state *st, const void *q, const void *k, const void *v,
                        const void *Wq, const void *Wk, int32_t Tn, void *out, int32_t *sel_trace,
                        void *workspace, size_t workspace_bytes, hipStream_t stream, bool allow_side_stream = true) {
    generic::PrefillArgs<T> a;
    a.dm = make_dims(c);
    a.st = make_state<T>(st);
    a.q = (const T *)q; a.k = (const T *)k; a.v = (const T *)v; a.Wq = (const T *)Wq; a.Wk = (const T *)Wk;
    a.out = out;
    a.T_tokens = Tn;
    a.n_chunks = (Tn + a.dm.C - 1) / a.dm.C;
    a.want_out = q != nullptr;
    a.sel_trace = sel_trace;
    const PrefillPlan p = plan_prefill(c, a.want_out, (size_t)Tn);
    char *ws = (char *)workspace;
    a.tok_score = (float *)(ws + p.off_score);
    a.R2 = band_tile_rows(a.dm);
    a.prefK = (T *)(ws + p.off_prefK); a.prefV = (T *)(ws + p.off_prefV);
    a.sp_row = (int32_t *)(ws + p.off_sp_row);
    a.phiE = (float *)(ws + p.off_phiE);
    a.next_j = (int32_t *)(ws + p.off_next);
    a.scan_mode = 0;
    int S = a.n_chunks > 0 ? a.n_chunks : 1;
    if (p.snap_bytes_per_chunk > 0) {
        size_t room = (workspace_bytes - p.fixed_bytes) / p.snap_bytes_per_chunk;
        if (room < 1) return LOLA_ERR_WORKSPACE;
        if ((size_t)S > room) S = (int)room;
    }
    a.S = S;
    const size_t ns = (size_t)a.dm.B * a.dm.Hkv, D = a.dm.D, d = a.dm.d, lam = a.dm.lam;
    char *snap = ws + p.off_snap;
    a.snapH = (float *)snap;
    a.snapS = (float *)(snap + up(ns * S * D * d * 4));
    a.snapG = (int32_t *)(snap + up(ns * S * D * d * 4) + up(ns * S * D * 4));
    a.phiK = nullptr;
    if (p.phik_bytes_per_chunk > 0) {   // behind the snapshot regions (absent in an update-only call)
        const size_t snaps = a.want_out ? up(ns * S * D * d * 4) + up(ns * S * D * 4) + up(ns * S * (lam ? lam : 1) * 4) : 0;
        a.phiK = (uint16_t *)(snap + snaps);
    }
    // the three snapshot regions are each rounded up per pass, which never exceeds S * snap_bytes_per_chunk

    const size_t scan_fixed = scan_fixed_floats(a.dm);
    a.R = score_tile_rows(a.dm, scan_fixed);
    a.QT = attend_tile_queries(a.dm);
    const bool fast_att = a.want_out && fast_output_ok(c);
    const bool wide_att = a.want_out && !fast_att && wide_output_ok(c);
    a.snap_split = (fast_att || wide_att) ? 1 : 0;
    if (a.R <= 0 || (a.want_out && a.QT <= 0)) return LOLA_ERR_UNSUPPORTED;
    const size_t lds_scan = 4 * (scan_fixed + (size_t)a.R * (3 * d + D + 1));
    const size_t lds_att = 4 * ((size_t)a.QT * (d + D + (lam + a.dm.eta + a.dm.C) + 3));
    dim3 block(generic::NT), gs((unsigned)ns);

    {
        // enough workgroups per stream to keep the copy of (lambda + eta) rows short when the streams are few
        const size_t rows = (size_t)a.dm.lam + a.dm.eta;
        const unsigned parts = (unsigned)(ns >= 512 ? 1 : (rows * d / (generic::NT * 16) > 16 ? 16 : (rows * d / (generic::NT * 16) < 1 ? 1 : rows * d / (generic::NT * 16))));
        hipLaunchKernelGGL((generic::prefix_kernel<T>), dim3((unsigned)ns, parts), block, 0, stream, a);
    }
    LAUNCH_CHECK();
    bool band_done = false;
    if constexpr (std::is_same<T, bf16_t>::value) {
        if (a.dm.score_kind && wide_scan_ok(c)) {   // the MFMA form of the same sums
            const dim3 gb((unsigned)(((size_t)a.dm.eta + Tn + 63) / 64), (unsigned)ns);
            if (c->head_dim == 128) {
                if (c->feat_dim == 256) hipLaunchKernelGGL((fast::band_score_wide_kernel<128, 256>), gb, dim3(256), 0, stream, a);
                else hipLaunchKernelGGL((fast::band_score_wide_kernel<128, 128>), gb, dim3(256), 0, stream, a);
            } else {
                if (c->feat_dim == 256) hipLaunchKernelGGL((fast::band_score_wide_kernel<64, 256>), gb, dim3(256), 0, stream, a);
                else hipLaunchKernelGGL((fast::band_score_wide_kernel<64, 128>), gb, dim3(256), 0, stream, a);
            }
            LAUNCH_CHECK();
            band_done = true;
        }
    }
    if (a.dm.score_kind && !band_done) {   // the query-dependent scores of every pair the call touches, before the state evolves
        if (a.R2 <= 0) return LOLA_ERR_UNSUPPORTED;
        const size_t lds_band = 4 * ((size_t)a.R2 * (2 * (d + D) + 1));
        const dim3 gb((unsigned)(((size_t)a.dm.eta + Tn + a.R2 - 1) / a.R2), (unsigned)ns);
        hipLaunchKernelGGL((generic::band_score_kernel<T>), gb, block, lds_band, stream, a);
        LAUNCH_CHECK();
    }
    for (int j0 = 0; j0 < a.n_chunks; j0 += S) {
        const int jend = j0 + S < a.n_chunks ? j0 + S : a.n_chunks;
        a.jb = a.j0 = j0;
        a.j1 = jend;
        if constexpr (std::is_same<T, bf16_t>::value) {
            if (fast_attend_ok(c) && c->sparse_budget == 0) {
                // No sparse cache: nothing is scored, every pair that leaves the window is folded, and the recurrence splits
                // over the value columns of H.  Features of the pass's keys (chunk-parallel); the generic kernel until the
                // first regular chunk (a full chunk with a full window behind it); the row-split kernel over the full
                // chunks; the generic kernel again for a ragged last chunk; the outputs from the snapshots.
                const dim3 gp((unsigned)(jend - j0), (unsigned)ns);
                if (c->head_dim == 128) hipLaunchKernelGGL(fast::phi_k_kernel<128>, gp, dim3(256), 0, stream, a);
                else hipLaunchKernelGGL(fast::phi_k_kernel<64>, gp, dim3(256), 0, stream, a);
                LAUNCH_CHECK();
                a.scan_mode = 1;
                hipLaunchKernelGGL((generic::scan_kernel<T>), gs, block, lds_scan, stream, a);
                LAUNCH_CHECK();
                const dim3 gn((unsigned)(c->head_dim / 16 + 1), (unsigned)ns);   // row tiles of H^T, then s
                if (c->head_dim == 128) hipLaunchKernelGGL(fast::scan_nocache_kernel<128>, gn, dim3(64), 0, stream, a);
                else hipLaunchKernelGGL(fast::scan_nocache_kernel<64>, gn, dim3(64), 0, stream, a);
                LAUNCH_CHECK();
                const int full_end = jend < Tn / a.dm.C ? jend : Tn / a.dm.C;
                hipLaunchKernelGGL(fast::advance_next_j_kernel, dim3((unsigned)((ns + 255) / 256)), dim3(256), 0, stream, a.next_j, (int)ns, full_end);
                LAUNCH_CHECK();
                if (jend == a.n_chunks && Tn % a.dm.C != 0) {
                    a.scan_mode = 2;
                    hipLaunchKernelGGL((generic::scan_kernel<T>), gs, block, lds_scan, stream, a);
                    LAUNCH_CHECK();
                }
                a.scan_mode = 0;
                if (a.want_out) {
                    launch_output_kernel(c, a, j0, jend, stream);
                    LAUNCH_CHECK();
                }
                continue;
            }
            const bool wide = wide_scan_ok(c);   // (run-time window / budget kernels; else the compile-time shapes)
            if (wide || fast_attend_ok(c)) {
                // The serial evolution in legs that hand the chunk position over in next_j: generic kernel until the first
                // regular chunk (a full chunk with a full window behind it and a full cache), MFMA kernel over the regular
                // chunks, generic kernel for what is left (a ragged last chunk); phi of the keys chunk-parallel
                // beforehand: at the compile-time shapes of every key of the pass, at the run-time shapes (per piece,
                // behind the generic leg) of the pairs that leave the window in each chunk and of the cache slots as
                // they stand.
                // (a compile-time shape whose cache does not stay in LDS takes its features the run-time way)
                const bool big = !wide && c->sparse_budget > 128;
                if (!wide && !big) {
                    const dim3 gp((unsigned)(jend - j0), (unsigned)ns);
                    if (c->head_dim == 128) hipLaunchKernelGGL(fast::phi_k_kernel<128>, gp, dim3(256), 0, stream, a);
                    else hipLaunchKernelGGL(fast::phi_k_kernel<64>, gp, dim3(256), 0, stream, a);
                    LAUNCH_CHECK();
                }
                // With few streams the serial evolution occupies few compute units, so the pass is cut into pieces and
                // the outputs of a piece (chunk-parallel, from its snapshots) run on a second stream beside the
                // evolution of the next piece.
                int piece = jend - j0;
                SideStream *side = nullptr;
                int np = piece / OVERLAP_MIN_PIECE;
                const size_t work = (size_t)piece * a.dm.Hq * a.dm.B * (size_t)(c->head_dim / 64);
                if ((size_t)np > work / OVERLAP_MIN_WORK) np = (int)(work / OVERLAP_MIN_WORK);
                if (np > SideStream::NEV) np = SideStream::NEV;
                if (allow_side_stream && c->prefill_overlap && a.want_out && ns <= OVERLAP_MAX_STREAMS && np >= 2) side = side_stream(stream);
                std::unique_lock<std::mutex> side_lock(side_use_mu, std::defer_lock);
                // Whatever happens after the first fork, the caller's stream waits for the second stream before this
                // call returns (an error path included): declared after the lock, so it runs while the lock is held.
                struct Joiner {
                    SideStream *side = nullptr; hipStream_t stream = nullptr; bool forked = false;
                    bool join() {
                        if (!forked) return true;
                        forked = false;
                        const bool ok = hipEventRecord(side->join, side->s) == hipSuccess &&
                                        hipStreamWaitEvent(stream, side->join, 0) == hipSuccess;
                        if (!ok) (void)hipGetLastError();
                        return ok;
                    }
                    ~Joiner() { (void)join(); }
                } joiner;
                joiner.side = side; joiner.stream = stream;
                // Piece boundaries: each piece half as long as the one before it, so that the outputs of a piece
                // (which take about half as long per chunk as the evolution) are hidden behind the evolution of the
                // next; the last piece, whose outputs nothing hides, is at least one round of output workgroups on the
                // chip (two per compute unit).
                int bnd[SideStream::NEV + 1];
                bnd[0] = j0; bnd[1] = jend;
                int npieces = 1;
                if (side) {
                    side_lock.lock();
                    const int per_chunk = a.dm.Hq * a.dm.B;   // output workgroups per chunk
                    int last = (2 * CHIP_CUS + per_chunk - 1) / per_chunk;
                    if (last < 2) last = 2;
                    while (np > 2 && piece / ((1 << np) - 1) < last) np--;
                    int unit = piece / ((1 << np) - 1);
                    if (unit < 1) unit = 1;
                    npieces = np;
                    bnd[np] = jend;
                    for (int i = np - 1; i >= 1; i--) bnd[i] = bnd[i + 1] - (unit << (np - 1 - i));   // the first piece takes the rest
                }
                auto attend = [&](hipStream_t so, int r0, int r1) { launch_output_kernel(c, a, r0, r1, so); };
                // outputs of the chunks [r0, r1) on the second stream, behind what `stream` held when fork[ev] was recorded
                auto attend_aside = [&](int ev, int r0, int r1) -> bool {
                    if (hipStreamWaitEvent(side->s, side->fork[ev], 0) != hipSuccess) return false;
                    joiner.forked = true;
                    attend(side->s, r0, r1);
                    return hipGetLastError() == hipSuccess;
                };
                int ip = 0, prev0 = j0;
                for (; ip < npieces; ip++) {
                    const int p0 = bnd[ip];
                    a.j0 = p0;
                    a.j1 = bnd[ip + 1];
                    // At the compile-time shapes later pieces start on regular chunks (the first piece is longer than the
                    // (lambda + eta) / C chunks after which the cache is full); with a long window and a large budget a
                    // piece may still begin while they fill, so the run-time shapes run the generic leg in every piece (it
                    // returns at once on a regular chunk).
                    if (ip == 0 || wide) {
                        a.scan_mode = 1;
                        hipLaunchKernelGGL((generic::scan_kernel<T>), gs, block, lds_scan, stream, a);
                        LAUNCH_CHECK();
                    }
                    // The previous piece's outputs may start once the evolution kernel of this piece is next in line (the
                    // event) and are enqueued after its launch: the evolution's workgroups, which need a compute unit's whole
                    // register file, should be resident before the output workgroups arrive, instead of queueing for
                    // compute units behind them.
                    if (wide) {
                        const dim3 gp((unsigned)(a.j1 - a.j0) + (unsigned)(c->sparse_budget / 64), (unsigned)ns);
#define LOLA_WSCAN(DHV, DFV) do { hipLaunchKernelGGL((fast::phi_wide_kernel<DHV, DFV>), gp, dim3(256), 0, stream, a); \
                                  if (side && ip > 0 && hipEventRecord(side->fork[ip - 1], stream) != hipSuccess) return LOLA_ERR_HIP; \
                                  if (a.dm.score_kind) hipLaunchKernelGGL((fast::scan_wide_kernel<DHV, DFV, true>), gs, dim3(DHV * 4), 0, stream, a); \
                                  else hipLaunchKernelGGL((fast::scan_wide_kernel<DHV, DFV, false>), gs, dim3(DHV * 4), 0, stream, a); } while (0)
                        if (c->head_dim == 128) { if (c->feat_dim == 256) LOLA_WSCAN(128, 256); else LOLA_WSCAN(128, 128); }
                        else { if (c->feat_dim == 256) LOLA_WSCAN(64, 256); else LOLA_WSCAN(64, 128); }
#undef LOLA_WSCAN
                    } else {
                    if (big) {
                        const dim3 gp((unsigned)(a.j1 - a.j0) + (unsigned)(c->sparse_budget / 64), (unsigned)ns);
                        if (c->head_dim == 128) hipLaunchKernelGGL((fast::phi_wide_kernel<128, 128>), gp, dim3(256), 0, stream, a);
                        else hipLaunchKernelGGL((fast::phi_wide_kernel<64, 128>), gp, dim3(256), 0, stream, a);
                        LAUNCH_CHECK();
                    }
                    if (side && ip > 0 && hipEventRecord(side->fork[ip - 1], stream) != hipSuccess) return LOLA_ERR_HIP;
#define LOLA_SCAN(LAMV) do { if (c->head_dim == 128) hipLaunchKernelGGL((fast::scan_fast_kernel<LAMV, 128, SCAN_RT128>), gs, dim3(512 / SCAN_RT128), 0, stream, a); \
                             else hipLaunchKernelGGL((fast::scan_fast_kernel<LAMV, 64, 1>), gs, dim3(256), 0, stream, a); } while (0)
                    if (c->sparse_budget == 64) LOLA_SCAN(64); else if (c->sparse_budget == 128) LOLA_SCAN(128); else LOLA_SCAN(256);
#undef LOLA_SCAN
                    }
                    LAUNCH_CHECK();
                    if (side && ip > 0 && !attend_aside(ip - 1, prev0, p0)) return LOLA_ERR_HIP;
                    if (a.j1 == a.n_chunks && Tn % a.dm.C != 0) {   // only a ragged last chunk is left to the generic kernel
                        a.scan_mode = 2;
                        hipLaunchKernelGGL((generic::scan_kernel<T>), gs, block, lds_scan, stream, a);
                        LAUNCH_CHECK();
                    }
                    a.scan_mode = 0;
                    if (a.want_out && !side) {
                        attend(stream, a.j0, a.j1);
                        LAUNCH_CHECK();
                    }
                    prev0 = p0;
                }
                if (side) {   // last piece; then the caller's stream continues (next pass, final write-back, the caller's
                              // own work) behind all outputs
                    if (hipEventRecord(side->fork[ip - 1], stream) != hipSuccess) return LOLA_ERR_HIP;
                    if (!attend_aside(ip - 1, prev0, jend)) return LOLA_ERR_HIP;
                    if (!joiner.join()) return LOLA_ERR_HIP;
                }
                continue;
            }
        }
        hipLaunchKernelGGL((generic::scan_kernel<T>), gs, block, lds_scan, stream, a);
        LAUNCH_CHECK();
        if (a.want_out) {
            bool done = false;
            if constexpr (std::is_same<T, bf16_t>::value) {
                if (fast_att) {   // the generic evolution took the snapshots in the MFMA output kernel's layout
                    launch_output_kernel(c, a, a.j0, a.j1, stream);
                    done = true;
                }
            }
            if constexpr (std::is_same<T, bf16_t>::value) {
                if (!done && wide_att) {   // any window / budget, 128 or 256 features: the run-time form of the MFMA output kernel
                    launch_output_kernel(c, a, a.j0, a.j1, stream);
                    done = true;
                }
            }
            if (!done) {
                dim3 ga((unsigned)(a.j1 - a.j0), (unsigned)a.dm.Hq, (unsigned)a.dm.B);
                if (c->out_dtype == LOLA_F32) hipLaunchKernelGGL((generic::attend_kernel<T, float>), ga, block, lds_att, stream, a);
                else hipLaunchKernelGGL((generic::attend_kernel<T, bf16_t>), ga, block, lds_att, stream, a);
            }
            LAUNCH_CHECK();
        }
    }
    hipLaunchKernelGGL((generic::finalize_kernel<T>), gs, block, 0, stream, a);
    LAUNCH_CHECK();
    return LOLA_OK;
}

}  // namespace

extern "C" {

size_t lola_step_scratch_bytes(const lola_config *c) {
    if (check_config(c) != LOLA_OK) return 0;
    return step_scratch_floats(c) * (size_t)c->batch * c->n_kv_heads * sizeof(float);
}

size_t lola_state_bytes(const lola_config *c, size_t fb[14]) {
    if (check_config(c) != LOLA_OK) return 0;
    const size_t ns = (size_t)c->batch * c->n_kv_heads, es = esize(c->dtype);
    const size_t d = c->head_dim, D = c->feat_dim, eta = c->window, lam = c->sparse_budget, R = c->fold_defer;
    const size_t sk = c->score_kind != LOLA_SCORE_SRE ? 1 : 0;
    size_t f[14] = {ns * D * d * 4, ns * D * 4, ns * eta * d * es, ns * eta * d * es, ns * lam * d * es,
                    ns * lam * d * es, ns * lam * 4, ns * 4, ns * 8,
                    ns * R * D * 4, ns * R * d * 4, R ? ns * 4 : 0,
                    sk * ns * eta * 4, sk * ns * lam * 4};
    size_t tot = 0;
    for (int i = 0; i < 14; i++) { if (fb) fb[i] = f[i]; tot += f[i]; }
    return tot;
}

size_t lola_prefill_workspace_bytes(const lola_config *c, int32_t T, int32_t with_outputs, size_t *min_bytes) {
    if (check_config(c) != LOLA_OK || T < 0) return 0;
    const PrefillPlan p = plan_prefill(c, with_outputs, (size_t)T);
    size_t nch = ((size_t)T + c->chunk - 1) / c->chunk;
    if (nch < 1) nch = 1;
    if (min_bytes) *min_bytes = p.fixed_bytes + p.snap_bytes_per_chunk;
    // an update-only call keeps no snapshots; its per-chunk scratch (features of the keys) is only an accelerator, so
    // the recommended size stops at 64 chunks per pass
    if (!with_outputs && nch > 64) nch = 64;
    return p.fixed_bytes + nch * p.snap_bytes_per_chunk;
}

lola_status lola_state_init(const lola_config *c, const lola_state *st, void *stream) {
    lola_status rc = check_config(c);
    if (rc != LOLA_OK) return rc;
    rc = check_state(c, st);
    if (rc != LOLA_OK) return rc;
    size_t fb[14];
    lola_state_bytes(c, fb);
    const bool sk = c->score_kind != LOLA_SCORE_SRE;
    void *ptrs[14] = {st->H, st->s, st->win_k, st->win_v, st->sp_k, st->sp_v, st->sp_idx, st->sp_count, st->n_tokens,
                      c->fold_defer ? st->pend_phi : nullptr, c->fold_defer ? st->pend_v : nullptr,
                      c->fold_defer ? st->pend_count : nullptr, sk ? st->win_score : nullptr, sk ? st->sp_score : nullptr};
    for (int i = 0; i < 14; i++) {
        if (!ptrs[i] || fb[i] == 0) continue;
        size_t n = fb[i] / 4;   // every field is a multiple of 4 bytes (head_dim is even)
        unsigned blocks = (unsigned)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
        hipLaunchKernelGGL(generic::fill_u32_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                           (uint32_t *)ptrs[i], n, i == 6 ? 0xFFFFFFFFu : 0u);
        LAUNCH_CHECK();
    }
    return LOLA_OK;
}

lola_status lola_state_flush(const lola_config *c, const lola_state *st, void *stream) {
    lola_status rc = check_config(c);
    if (rc != LOLA_OK) return rc;
    rc = check_state(c, st);
    if (rc != LOLA_OK) return rc;
    return flush_pending(c, st, (hipStream_t)stream);
}

}  // extern "C"

namespace {

// device address of this GPU's copy of `scratch`, looked up on the first call on each device
std::mutex noalloc_mu;
void *noalloc_ptr[MAX_DEV];
lola_status noalloc_scratch(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEV) { (void)hipGetLastError(); return LOLA_ERR_HIP; }
    std::lock_guard<std::mutex> lock(noalloc_mu);
    if (!noalloc_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return LOLA_ERR_HIP; }
        noalloc_ptr[dev] = p;
    }
    *out = noalloc_ptr[dev];
    return LOLA_OK;
}

// the two prefill entry points differ in where the workspace comes from and in whether the second stream may be used
lola_status prefill_entry(const lola_config *c, const lola_state *st, const void *q, const void *k, const void *v,
                          const void *Wq, const void *Wk, int32_t T, void *out, int32_t *sel_trace,
                          void *workspace, size_t workspace_bytes, void *stream, bool noalloc) {
    lola_status rc = check_config(c);
    if (rc != LOLA_OK) return rc;
    rc = check_state(c, st);
    if (rc != LOLA_OK) return rc;
    if (T < 0) return LOLA_ERR_SHAPE;
    if (T == 0) return LOLA_OK;   // nothing to read or write: the token pointers are not looked at
    if ((q == nullptr) != (out == nullptr)) return LOLA_ERR_NULL;
    if (!k || !v || !Wk || (q && !Wq)) return LOLA_ERR_NULL;
    if (!q && c->score_kind != LOLA_SCORE_SRE) return LOLA_ERR_UNSUPPORTED;   // these scores are sums over queries
    const void *ps[] = {q, k, v, Wq, Wk, out, sel_trace, noalloc ? nullptr : workspace};
    for (const void *p : ps) if (p && misaligned(p)) return LOLA_ERR_ALIGN;
    size_t need_min = 0;
    lola_prefill_workspace_bytes(c, T, q != nullptr, &need_min);
    if (noalloc) {
        if (need_min > LOLA_NOALLOC_SCRATCH_BYTES) return LOLA_ERR_TOO_LARGE;
        rc = prefill_feasible(c, q != nullptr);
        if (rc != LOLA_OK) return rc;
        rc = noalloc_scratch(&workspace);
        if (rc != LOLA_OK) return rc;
        workspace_bytes = LOLA_NOALLOC_SCRATCH_BYTES;
    } else {
        if (!workspace || workspace_bytes < need_min) return LOLA_ERR_WORKSPACE;
        rc = prefill_feasible(c, q != nullptr);
        if (rc != LOLA_OK) return rc;
    }
    rc = flush_pending(c, st, (hipStream_t)stream);   // the prefill kernels read H and s as they are in memory
    if (rc != LOLA_OK) return rc;
    if (c->dtype == LOLA_F32)
        return run_prefill<float>(c, st, q, k, v, Wq, Wk, T, out, sel_trace, workspace, workspace_bytes, (hipStream_t)stream, !noalloc);
    return run_prefill<bf16_t>(c, st, q, k, v, Wq, Wk, T, out, sel_trace, workspace, workspace_bytes, (hipStream_t)stream, !noalloc);
}

}  // namespace

extern "C" {

lola_status lola_prefill(const lola_config *c, const lola_state *st, const void *q, const void *k, const void *v,
                         const void *Wq, const void *Wk, int32_t T, void *out, int32_t *sel_trace,
                         void *workspace, size_t workspace_bytes, void *stream) {
    return prefill_entry(c, st, q, k, v, Wq, Wk, T, out, sel_trace, workspace, workspace_bytes, stream, false);
}

lola_status lola_prefill_noalloc(const lola_config *c, const lola_state *st, const void *q, const void *k, const void *v,
                                 const void *Wq, const void *Wk, int32_t T, void *out, int32_t *sel_trace, void *stream) {
    return prefill_entry(c, st, q, k, v, Wq, Wk, T, out, sel_trace, nullptr, 0, stream, true);
}

size_t lola_noalloc_scratch_bytes(void) { return LOLA_NOALLOC_SCRATCH_BYTES; }

lola_status lola_decode_step(const lola_config *c, const lola_state *st, const void *q, const void *k, const void *v,
                             const void *Wq, const void *Wk, void *out, void *stream) {
    lola_status rc = check_config(c);
    if (rc != LOLA_OK) return rc;
    rc = check_state(c, st);
    if (rc != LOLA_OK) return rc;
    if (!q || !k || !v || !Wq || !Wk || !out) return LOLA_ERR_NULL;
    const void *ps[] = {q, k, v, Wq, Wk, out};
    for (const void *p : ps) if (misaligned(p)) return LOLA_ERR_ALIGN;
    rc = decode_feasible(c);
    if (rc != LOLA_OK) return rc;
    if (c->dtype == LOLA_F32) return run_decode<float>(c, st, q, k, v, Wq, Wk, out, (hipStream_t)stream);
    if (fast_decode_ok(c)) return run_fast_decode(c, st, q, k, v, Wq, Wk, out, (hipStream_t)stream);
    return run_decode<bf16_t>(c, st, q, k, v, Wq, Wk, out, (hipStream_t)stream);
}

void lola_release_streams(void) {
    std::lock_guard<std::mutex> use(side_use_mu);
    release_side_streams();
}

const char *lola_status_str(lola_status s) {
    switch (s) {
        case LOLA_OK: return "ok";
        case LOLA_ERR_NULL: return "required pointer is NULL";
        case LOLA_ERR_SHAPE: return "size out of range or inconsistent";
        case LOLA_ERR_DTYPE: return "unknown dtype or phi_kind";
        case LOLA_ERR_ALIGN: return "pointer not 16-byte aligned";
        case LOLA_ERR_UNSUPPORTED: return "no kernel for this configuration";
        case LOLA_ERR_WORKSPACE: return "workspace missing or too small";
        case LOLA_ERR_HIP: return "HIP launch failed";
        case LOLA_ERR_TOO_LARGE: return "request exceeds the static scratch of the entry point that allocates nothing";
    }
    return "unknown status";
}

const char *lola_kernel_path(const lola_config *c, int32_t which) {
    if (check_config(c) != LOLA_OK) return "invalid";
    if (which == 1 && fast_decode_ok(c)) return "mfma";
    if (which == 1 && wide_decode_ok(c)) return "mfma";      // update of steady-state streams and outputs on MFMA
    if (which == 1 && wide_step_out_ok(c)) return "mixed";   // outputs on MFMA, update shape-generic
    if (which == 0 && (fast_attend_ok(c) || wide_scan_ok(c))) return "mfma";
    if (which == 0 && (fast_output_ok(c) || wide_output_ok(c))) return "mixed";
    return "generic";
}

}  // extern "C"

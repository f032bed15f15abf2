// Shape-generic kernels of the LoLA layer: plain fp32 FMA arithmetic, any supported shape, both
// storage types.  They are the reference path on the GPU (fp32 mode, unusual shapes) and the
// structure the MFMA kernels specialise: a per-stream sequential "scan" that evolves the memories
// chunk by chunk and leaves per-chunk snapshots, and a chunk-parallel "attend" that produces the
// outputs from those snapshots.
//
// Paper passages: feature map Sec. 2.3 eq. (feature_map); self-recall error Sec. 3 eq. (score);
// eligible set / top-lambda / fold Sec. 3 (E_t, G_t, S_t, H_t equations); output Sec. 3 (y_t
// equation); chunk schedule Sec. 3 "Chunkwise Inference".
#pragma once
#include <type_traits>
#include "lola_common.h"
#include "decode_mfma.h"   // MFMA primitives (operand types, bf16 high/low split)

namespace lola {
namespace generic {

constexpr int NT = 256;          // threads per workgroup
constexpr int NW = NT / WAVE;    // wavefronts per workgroup

__device__ __forceinline__ float block_sum(float v, float *red) {
    v = wave_sum(v);
    if ((threadIdx.x % WAVE) == 0) red[threadIdx.x / WAVE] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < NW; i++) t += red[i];
    __syncthreads();
    return t;
}
__device__ __forceinline__ float block_max(float v, float *red) {
    v = wave_max(v);
    if ((threadIdx.x % WAVE) == 0) red[threadIdx.x / WAVE] = v;
    __syncthreads();
    float t = red[0];
#pragma unroll
    for (int i = 1; i < NW; i++) t = fmaxf(t, red[i]);
    __syncthreads();
    return t;
}

// sum_i row[i] * x[i] in index order (same rounding as the element-wise loop), the row fetched 16 bytes at a time;
// n is a multiple of 8 and the row is 16-byte aligned (head_dim is 32, 64, 128 or 256)
__device__ __forceinline__ float dot_row(const bf16_t *row, const float *x, int n, float acc) {
    const uint4 *r4 = reinterpret_cast<const uint4 *>(row);
    for (int i = 0; i < n / 8; i++) {
        const uint4 u = r4[i];
        const uint32_t wds[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int e = 0; e < 4; e++) {
            acc = fmaf(__uint_as_float(wds[e] << 16), x[8 * i + 2 * e], acc);
            acc = fmaf(__uint_as_float(wds[e] & 0xFFFF0000u), x[8 * i + 2 * e + 1], acc);
        }
    }
    return acc;
}
__device__ __forceinline__ float dot_row(const float *row, const float *x, int n, float acc) {
    const float4 *r4 = reinterpret_cast<const float4 *>(row);
    for (int i = 0; i < n / 4; i++) {
        const float4 u = r4[i];
        acc = fmaf(u.x, x[4 * i], acc); acc = fmaf(u.y, x[4 * i + 1], acc);
        acc = fmaf(u.z, x[4 * i + 2], acc); acc = fmaf(u.w, x[4 * i + 3], acc);
    }
    return acc;
}

// one 16-byte piece of a stored row as fp32 into LDS (dst is the row's fp32 copy; 8 bf16 or 4 fp32 values per piece)
__device__ __forceinline__ void piece_to_f32(const bf16_t *row, int piece, float *dst) {
    const uint4 u = reinterpret_cast<const uint4 *>(row)[piece];
    reinterpret_cast<float4 *>(dst)[2 * piece] = make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xFFFF0000u),
                                                              __uint_as_float(u.y << 16), __uint_as_float(u.y & 0xFFFF0000u));
    reinterpret_cast<float4 *>(dst)[2 * piece + 1] = make_float4(__uint_as_float(u.z << 16), __uint_as_float(u.z & 0xFFFF0000u),
                                                                  __uint_as_float(u.w << 16), __uint_as_float(u.w & 0xFFFF0000u));
}
__device__ __forceinline__ void piece_to_f32(const float *row, int piece, float *dst) {
    reinterpret_cast<float4 *>(dst)[piece] = reinterpret_cast<const float4 *>(row)[piece];
}

// acc[q] = sum_i row[i] * xs[q][i] for q < nq <= 16, each in index order (the rounding of dot_row); the row crosses the
// memory system once for all nq vectors (xs in LDS, row stride n)
__device__ __forceinline__ void dot_row_many(const bf16_t *row, const float *xs, int n, int nq, float (&acc)[16]) {
    const uint4 *r4 = reinterpret_cast<const uint4 *>(row);
    for (int i = 0; i < n / 8; i++) {
        const uint4 u = r4[i];
        const float kf[8] = {__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xFFFF0000u), __uint_as_float(u.y << 16), __uint_as_float(u.y & 0xFFFF0000u),
                             __uint_as_float(u.z << 16), __uint_as_float(u.z & 0xFFFF0000u), __uint_as_float(u.w << 16), __uint_as_float(u.w & 0xFFFF0000u)};
#pragma unroll
        for (int q = 0; q < 16; q++) {
            if (q < nq) {
                const float4 x0 = *reinterpret_cast<const float4 *>(xs + q * n + 8 * i), x1 = *reinterpret_cast<const float4 *>(xs + q * n + 8 * i + 4);
                float t = acc[q];
                t = fmaf(kf[0], x0.x, t); t = fmaf(kf[1], x0.y, t); t = fmaf(kf[2], x0.z, t); t = fmaf(kf[3], x0.w, t);
                t = fmaf(kf[4], x1.x, t); t = fmaf(kf[5], x1.y, t); t = fmaf(kf[6], x1.z, t); t = fmaf(kf[7], x1.w, t);
                acc[q] = t;
            }
        }
    }
}
__device__ __forceinline__ void dot_row_many(const float *row, const float *xs, int n, int nq, float (&acc)[16]) {
    const float4 *r4 = reinterpret_cast<const float4 *>(row);
    for (int i = 0; i < n / 4; i++) {
        const float4 u = r4[i];
#pragma unroll
        for (int q = 0; q < 16; q++) {
            if (q < nq) {
                const float4 x0 = *reinterpret_cast<const float4 *>(xs + q * n + 4 * i);
                float t = acc[q];
                t = fmaf(u.x, x0.x, t); t = fmaf(u.y, x0.y, t); t = fmaf(u.z, x0.z, t); t = fmaf(u.w, x0.w, t);
                acc[q] = t;
            }
        }
    }
}

// phi of R rows.  xs [R][d] (LDS, fp32 copies of the stored vectors), W [m][d] (global, row j = w_j), result
// ph [R][D] (LDS).  Workgroup-wide; ends with a barrier.
template <typename T>
__device__ void phi_rows(const Dims &dm, const T *W, const float *xs, float *ph, int R) {
    const int tid = threadIdx.x, d = dm.d, m = dm.m, D = dm.D;
    if (std::is_same<T, bf16_t>::value && R >= 8 && (m & 15) == 0) {
        // projections on MFMA (bf16 storage: the fp32 copies in LDS are exact bf16 values, products are exact, fp32
        // accumulation): tile = 16 projections x 16 rows, A = rows of W from memory, B = the vectors from LDS
        const int w = tid / WAVE, lane = tid % WAVE, r16 = lane & 15, g4 = lane >> 4;
        const int njt = m / 16, ntile = ((R + 15) / 16) * njt;
        for (int t = w; t < ntile; t += NW) {
            const int rt = t / njt, jt = t - rt * njt, r = 16 * rt + r16;
            fast::f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            fast::bf16x8 A[8];   // head_dim <= 256: at most eight k-steps, all requested before the first is used
#pragma unroll
            for (int ks = 0; ks < 8; ks++)
                A[ks] = ks < d / 32 ? fast::ld_bf16x8(reinterpret_cast<const bf16_t *>(W) + (size_t)(16 * jt + r16) * d + 32 * ks + 8 * g4)
                                    : fast::zero_bf16x8();
#pragma unroll
            for (int ks = 0; ks < 8; ks++) {
                if (ks < d / 32) {
                    fast::bf16x8 B = fast::zero_bf16x8();
                    if (r < R) {
                        const float4 x0 = *reinterpret_cast<const float4 *>(&xs[r * d + 32 * ks + 8 * g4]);
                        const float4 x1 = *reinterpret_cast<const float4 *>(&xs[r * d + 32 * ks + 8 * g4 + 4]);
                        B[0] = (__bf16)x0.x; B[1] = (__bf16)x0.y; B[2] = (__bf16)x0.z; B[3] = (__bf16)x0.w;
                        B[4] = (__bf16)x1.x; B[5] = (__bf16)x1.y; B[6] = (__bf16)x1.z; B[7] = (__bf16)x1.w;
                    }
                    acc = fast::mfma16(A[ks], B, acc);
                }
            }
            if (r < R) {   // lane (column = row r of the batch, group g4) holds projections 16 jt + 4 g4 + 0..3
#pragma unroll
                for (int i = 0; i < 4; i++) ph[r * D + 16 * jt + 4 * g4 + i] = acc[i];
            }
        }
    } else {
        for (int p = tid; p < R * m; p += NT) {
            int r = p / m, j = p - r * m;
            const float *x = xs + r * d;
            ph[r * D + j] = dot_row(W + (size_t)j * d, x, d, 0.f);
        }
    }
    __syncthreads();
    const int w = tid / WAVE, lane = tid % WAVE;
    for (int r = w; r < R; r += NW) {
        float *row = ph + r * D;
        if (dm.phi_kind == 1) {
            for (int j = lane; j < m; j += WAVE) {
                float z = row[j];
                row[j] = expf(z);
                row[m + j] = expf(-z);
            }
        } else {
            float zmax = -INFINITY, zmin = INFINITY;
            for (int j = lane; j < m; j += WAVE) {
                float z = row[j];
                zmax = fmaxf(zmax, z);
                zmin = fminf(zmin, z);
            }
            zmax = wave_max(zmax);
            zmin = wave_min(zmin);
            float sp = 0.f, sn = 0.f;
            for (int j = lane; j < m; j += WAVE) {
                float z = row[j];
                float ep = expf(z - zmax), en = expf(zmin - z);
                row[j] = ep;
                row[m + j] = en;
                sp += ep;
                sn += en;
            }
            sp = wave_sum(sp);
            sn = wave_sum(sn);
            for (int j = lane; j < m; j += WAVE) {
                row[j] = row[j] / sp;
                row[m + j] = row[m + j] / sn;
            }
        }
    }
    __syncthreads();
}

// Self-recall error of R pairs against (H, s), H stored transposed [d][D]: ph [R][D], vs [R][d] in LDS; err [R][d], den [R] LDS
// scratch; score_out[r] = || ph_r^T H / ph_r^T s - v_r ||_2 (recall = 0 while ph_r^T s == 0).
// MF (bf16 storage only): the recall contraction runs on MFMA with both fp32 operands split into bf16 high + low parts
// (three passes, ~2^-17 relative), tile = 16 value columns x 16 rows.
template <bool MF>
__device__ void score_rows(const Dims &dm, const float *H, const float *s, const float *ph, const float *vs,
                           float *err, float *den, float *score_out, int R) {
    const int tid = threadIdx.x, d = dm.d, D = dm.D;
    const int w = tid / WAVE, lane = tid % WAVE;
    for (int r = w; r < R; r += NW) {
        float a = 0.f;
        for (int f = lane; f < D; f += WAVE) a = fmaf(ph[r * D + f], s[f], a);
        a = wave_sum(a);
        if (lane == 0) den[r] = a;
    }
    __syncthreads();
    if (MF && R >= 8 && (D & 31) == 0) {
        const int r16 = lane & 15, g4 = lane >> 4;
        const int nrt = (R + 15) / 16;
        for (int ct = w; ct < d / 16; ct += NW) {
            // A = this wavefront's 16 rows of H^T, eight k-steps at a time (all their loads in flight together, split once
            // and used for both row tiles of the batch: a batch has at most 32 rows); B = the feature rows from LDS
            fast::f32x4 acc[2][3];
#pragma unroll
            for (int rt = 0; rt < 2; rt++)
#pragma unroll
                for (int x = 0; x < 3; x++) acc[rt][x] = (fast::f32x4){0.f, 0.f, 0.f, 0.f};
            for (int ks0 = 0; ks0 < D / 32; ks0 += 8) {
                float4 h0[8], h1[8];
#pragma unroll
                for (int u = 0; u < 8; u++) {
                    const int ks = ks0 + u < D / 32 ? ks0 + u : ks0;   // (a repeated load instead of a branch; its product is skipped below)
                    const float *hp = H + (size_t)(16 * ct + r16) * D + 32 * ks + 8 * g4;
                    h0[u] = *reinterpret_cast<const float4 *>(hp); h1[u] = *reinterpret_cast<const float4 *>(hp + 4);
                }
                fast::bf16x8 Ah[8], Al[8];
#pragma unroll
                for (int u = 0; u < 8; u++) {
                    const float hv[8] = {h0[u].x, h0[u].y, h0[u].z, h0[u].w, h1[u].x, h1[u].y, h1[u].z, h1[u].w};
                    fast::split8(hv, Ah[u], Al[u]);
                }
#pragma unroll
                for (int rt = 0; rt < 2; rt++) {
                    const int r = 16 * rt + r16;
                    if (rt < nrt) {
#pragma unroll
                        for (int u = 0; u < 8; u++) {
                            if (ks0 + u < D / 32) {
                                fast::bf16x8 Bh = fast::zero_bf16x8(), Bl = fast::zero_bf16x8();
                                if (r < R) {
                                    const float4 p0 = *reinterpret_cast<const float4 *>(&ph[r * D + 32 * (ks0 + u) + 8 * g4]);
                                    const float4 p1 = *reinterpret_cast<const float4 *>(&ph[r * D + 32 * (ks0 + u) + 8 * g4 + 4]);
                                    const float pv[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
                                    fast::split8(pv, Bh, Bl);
                                }
                                acc[rt][0] = fast::mfma16(Ah[u], Bh, acc[rt][0]);
                                acc[rt][1] = fast::mfma16(Ah[u], Bl, acc[rt][1]);
                                acc[rt][2] = fast::mfma16(Al[u], Bh, acc[rt][2]);
                            }
                        }
                    }
                }
            }
#pragma unroll
            for (int rt = 0; rt < 2; rt++) {
                const int r = 16 * rt + r16;
                if (rt < nrt && r < R) {   // lane (column = row r, group g4) holds value columns c = 16 ct + 4 g4 + 0..3
                    const float dn = den[r];
#pragma unroll
                    for (int i = 0; i < 4; i++) {
                        const int c = 16 * ct + 4 * g4 + i;
                        const float p = acc[rt][0][i] + (acc[rt][1][i] + acc[rt][2][i]);
                        const float pred = dn > 0.f ? p / dn : 0.f;
                        const float e = pred - vs[r * d + c];
                        err[r * d + c] = e * e;
                    }
                }
            }
        }
    } else {
    // thread (c, rg) takes rows rg, rg + nrg, ...; eight rows share one pass over row c of H^T, so that a value of H
    // fetched from memory feeds eight multiply-adds (the features come from LDS, the same word for all c)
    const int c = tid % d, rg = tid / d, nrg = NT / d;
    for (int r0 = rg; r0 < R; r0 += 8 * nrg) {
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if ((D & 3) == 0) {   // four features per load of H and of the LDS rows (index order kept)
            const float4 *H4 = reinterpret_cast<const float4 *>(H + (size_t)c * D);
            for (int f4 = 0; f4 < D / 4; f4++) {
                const float4 hv = H4[f4];
#pragma unroll
                for (int i = 0; i < 8; i++) {
                    const int r = r0 + i * nrg;
                    if (r < R) {
                        const float4 pv = *reinterpret_cast<const float4 *>(&ph[r * D + 4 * f4]);
                        acc[i] = fmaf(pv.x, hv.x, acc[i]); acc[i] = fmaf(pv.y, hv.y, acc[i]);
                        acc[i] = fmaf(pv.z, hv.z, acc[i]); acc[i] = fmaf(pv.w, hv.w, acc[i]);
                    }
                }
            }
        } else {
            for (int f = 0; f < D; f++) {
                const float hv = H[(size_t)c * D + f];
#pragma unroll
                for (int i = 0; i < 8; i++) {
                    const int r = r0 + i * nrg;
                    if (r < R) acc[i] = fmaf(ph[r * D + f], hv, acc[i]);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const int r = r0 + i * nrg;
            if (r < R) {
                const float dn = den[r];
                const float pred = dn > 0.f ? acc[i] / dn : 0.f;
                const float e = pred - vs[r * d + c];
                err[r * d + c] = e * e;
            }
        }
    }
    }
    __syncthreads();
    for (int r = w; r < R; r += NW) {
        float a = 0.f;
        for (int c2 = lane; c2 < d; c2 += WAVE) a += err[r * d + c2];
        a = wave_sum(a);
        if (lane == 0) score_out[r] = sqrtf(a);
    }
    __syncthreads();
}

// One query's contribution to a key's query-dependent score (Sec. 4 / appendix "scoring ablation"): w = exp(logit),
// a = phi(q) . phi(k); kinds 1..4: (w - a)^2, |w - a|, a / w, w.
__device__ __forceinline__ float query_term(int kind, float logit, float a) {
    const float w = expf(logit);
    if (kind == 1) return (w - a) * (w - a);
    if (kind == 2) return fabsf(w - a);
    if (kind == 3) return a / w;
    return w;
}

// ---------------------------------------------------------------------------------------------
// state init
// ---------------------------------------------------------------------------------------------
__global__ void fill_u32_kernel(uint32_t *p, size_t n, uint32_t val) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = val;
}

// ---------------------------------------------------------------------------------------------
// decode: one workgroup per (batch, kv head)
// ---------------------------------------------------------------------------------------------
template <typename T>
struct DecodeArgs {
    Dims dm;
    State<T> st;
    const T *q, *k, *v, *Wq, *Wk;
    void *out;
    int R;          // rows scored per tile
    int no_out;               // 1: the memories are updated only (another kernel computes the outputs)
    int skip_steady;          // 1: streams in steady state (window and cache full) were updated by another kernel already
};

template <typename T, typename TO>
__global__ __launch_bounds__(NT) void decode_kernel(DecodeArgs<T> a) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const Dims &dm = a.dm;
    const int tid = threadIdx.x, d = dm.d, D = dm.D, m = dm.m, eta = dm.eta, lam = dm.lam, R = a.R;
    const int si = blockIdx.x, b = si / dm.Hkv, h = si % dm.Hkv;
    float *xs = smem;                  // [R][d]
    float *ph = xs + R * d;            // [R][D]
    float *vs = ph + R * D;            // [R][d]
    float *err = vs + R * d;           // [R][d]
    float *den = err + R * d;          // [R]
    float *score = den + R;            // [lam + 1]
    float *pk = score + (lam + 1);     // [d] leaving pair
    float *pv = pk + d;                // [d]
    float *pw = pv + d;                // [lam + eta] softmax weights
    float *red = pw + (lam + eta);     // [NW * 3]
    // query-dependent scores only: sums of the window pairs, logits of one query, features of a tile of window keys
    const int sk = dm.score_kind;
    float *wsc = red + NW * 3 + 8;     // [eta]
    float *wlg = wsc + eta;            // [eta]
    float *ph2 = wlg + eta;            // [R][D]
    __shared__ int sh_drop;
    __shared__ float sh_pscore;

    float *H = a.st.H + (size_t)si * D * d;
    float *s = a.st.s + (size_t)si * D;
    T *win_k = a.st.win_k + (size_t)si * eta * d, *win_v = a.st.win_v + (size_t)si * eta * d;
    T *sp_k = a.st.sp_k + (size_t)si * lam * d, *sp_v = a.st.sp_v + (size_t)si * lam * d;
    int32_t *sp_idx = a.st.sp_idx + (size_t)si * lam;
    const T *Wk = a.Wk + (size_t)h * d * m;
    const T *knew = a.k + (size_t)si * d, *vnew = a.v + (size_t)si * d;

    const int64_t tok = a.st.n_tokens[si];
    const bool popped = tok >= (int64_t)eta;
    const int slot = eta > 0 ? (int)(tok % eta) : 0;
    const int32_t pidx = (int32_t)(tok - eta);
    int spc = a.st.sp_count[si];
    if (a.skip_steady && popped && lam > 0 && spc == lam) return;   // (a stream stays in steady state once it is there)
    float *win_score = sk ? a.st.win_score + (size_t)si * eta : nullptr;
    float *sp_score = sk ? a.st.sp_score + (size_t)si * lam : nullptr;
    if (sk) {
        // the leaving pair's sum is final; the new pair starts at zero in the same ring slot
        if (tid == 0) sh_pscore = (popped && eta > 0) ? win_score[slot] : 0.f;
        for (int i = tid; i < eta; i += NT) wsc[i] = i == slot ? 0.f : win_score[i];
    }

    // 1. the new pair enters the window (ring slot tok % eta); the pair it displaces leaves
    if (popped) {
        for (int i = tid; i < d; i += NT) {
            pk[i] = eta > 0 ? ldf(win_k, (size_t)slot * d + i) : ldf(knew, i);
            pv[i] = eta > 0 ? ldf(win_v, (size_t)slot * d + i) : ldf(vnew, i);
        }
    }
    __syncthreads();
    if (eta > 0) {
        for (int i = tid; i < d; i += NT) {
            win_k[(size_t)slot * d + i] = knew[i];
            win_v[(size_t)slot * d + i] = vnew[i];
        }
    }

    // 2. eligible set = sparse cache + leaving pair
    if (popped) {
        if (spc < lam) {
            for (int i = tid; i < d; i += NT) {
                stf(sp_k, (size_t)spc * d + i, pk[i]);
                stf(sp_v, (size_t)spc * d + i, pv[i]);
            }
            if (tid == 0) { sp_idx[spc] = pidx; a.st.sp_count[si] = spc + 1; if (sk) sp_score[spc] = sh_pscore; }
            spc += 1;
        } else {
            int drop = 0;   // candidate index: < lam a sparse slot, == lam the leaving pair
            if (lam > 0) {
                if (sk) {
                    for (int e = tid; e <= lam; e += NT) score[e] = e < lam ? sp_score[e] : sh_pscore;
                    __syncthreads();
                }
                for (int t0 = 0; t0 <= lam && !sk; t0 += R) {
                    int nr = min(R, lam + 1 - t0);
                    for (int p = tid; p < nr * d; p += NT) {
                        int r = p / d, i = p - r * d, e = t0 + r;
                        xs[p] = e < lam ? ldf(sp_k, (size_t)e * d + i) : pk[i];
                        vs[p] = e < lam ? ldf(sp_v, (size_t)e * d + i) : pv[i];
                    }
                    __syncthreads();
                    phi_rows(dm, Wk, xs, ph, nr);
                    score_rows<std::is_same<T, bf16_t>::value>(dm, H, s, ph, vs, err, den, score + t0, nr);
                }
                // the pair that goes: smallest score, ties -> the larger token index goes
                if (tid < WAVE) {
                    float bs = INFINITY; int bi = -1, be = 0;
                    for (int e = tid; e <= lam; e += WAVE) {
                        float sc = score[e]; int ix = e < lam ? sp_idx[e] : pidx;
                        if (sc < bs || (sc == bs && ix > bi)) { bs = sc; bi = ix; be = e; }
                    }
                    for (int o = WAVE / 2; o > 0; o >>= 1) {
                        float os = __shfl_xor(bs, o, WAVE); int oi = __shfl_xor(bi, o, WAVE), oe = __shfl_xor(be, o, WAVE);
                        if (os < bs || (os == bs && oi > bi)) { bs = os; bi = oi; be = oe; }
                    }
                    if (tid == 0) sh_drop = be;
                }
                __syncthreads();
                drop = sh_drop;
            }
            // fold the dropped pair: H += phi(k) v^T, s += phi(k)
            for (int i = tid; i < d; i += NT) {
                xs[i] = drop < lam ? ldf(sp_k, (size_t)drop * d + i) : pk[i];
                vs[i] = drop < lam ? ldf(sp_v, (size_t)drop * d + i) : pv[i];
            }
            __syncthreads();
            phi_rows(dm, Wk, xs, ph, 1);
            for (int idx = tid; idx < D * d; idx += NT) {
                int c = idx / D, f = idx - c * D;
                H[idx] = fmaf(ph[f], vs[c], H[idx]);
            }
            for (int f = tid; f < D; f += NT) s[f] += ph[f];
            __syncthreads();
            if (drop < lam) {   // the leaving pair takes the freed slot
                for (int i = tid; i < d; i += NT) {
                    stf(sp_k, (size_t)drop * d + i, pk[i]);
                    stf(sp_v, (size_t)drop * d + i, pv[i]);
                }
                if (tid == 0) { sp_idx[drop] = pidx; if (sk) sp_score[drop] = sh_pscore; }
            }
        }
    }
    __syncthreads();

    // 3. outputs of the group's query heads with the updated memories
    const int wn = (int)min((int64_t)eta, tok + 1);
    const int nk = spc + wn;
    TO *out = (TO *)a.out;
    for (int r = 0; r < dm.g && !a.no_out; r++) {
        const int hq = h * dm.g + r;
        const T *qrow = a.q + ((size_t)b * dm.Hq + hq) * d;
        for (int i = tid; i < d; i += NT) xs[i] = ldf(qrow, i);
        __syncthreads();
        phi_rows(dm, a.Wq + (size_t)hq * d * m, xs, ph, 1);
        float lmax = 0.f;     // m = max(0, max logit): the linear terms carry weight exp(-m) <= 1
        for (int i = tid; i < nk; i += NT) {
            const T *kr = i < spc ? sp_k + (size_t)i * d : win_k + (size_t)(i - spc) * d;
            float dot = dot_row(kr, xs, d, 0.f);
            dot *= dm.scale;
            if (i >= spc && sk) wlg[i - spc] = dot;
            if (i < spc && (dm.hide & 2)) dot = -INFINITY;   // restricted query: the sparse cache is not read
            pw[i] = dot;
            lmax = fmaxf(lmax, dot);
        }
        lmax = block_max(lmax, red);
        float psum = 0.f;
        for (int i = tid; i < nk; i += NT) {
            float p = expf(pw[i] - lmax);
            pw[i] = p;
            psum += p;
        }
        psum = block_sum(psum, red);
        float lden = 0.f;
        for (int f = tid; f < D; f += NT) lden = fmaf(ph[f], s[f], lden);
        lden = block_sum(lden, red);
        const float elin = (dm.hide & 1) ? 0.f : expf(-lmax);   // restricted query: the hidden state is not read
        const int c = tid % d, part = tid / d, nparts = NT / d;
        float num = 0.f;
        for (int i = part; i < nk; i += nparts) {
            const T *vr = i < spc ? sp_v + (size_t)i * d : win_v + (size_t)(i - spc) * d;
            num = fmaf(pw[i], ldf(vr, c), num);
        }
        float lin = 0.f;
        for (int f = part; f < D; f += nparts) lin = fmaf(ph[f], H[(size_t)c * D + f], lin);
        num = fmaf(elin, lin, num);
        err[part * d + c] = num;
        __syncthreads();
        if (tid < d) {
            float t = 0.f;
            for (int p = 0; p < nparts; p++) t += err[p * d + tid];
            stf(out, ((size_t)b * dm.Hq + hq) * d + tid, t / (psum + elin * lden));
        }
        __syncthreads();
        if (sk) {
            // this query's term for every pair in the window (ring slot order), a tile of R keys at a time; one
            // wavefront per key sums phi(q) . phi(k)
            for (int t0 = 0; t0 < wn; t0 += R) {
                const int nr = min(R, wn - t0);
                for (int p = tid; p < nr * d; p += NT) vs[p] = ldf(win_k, (size_t)t0 * d + p);
                __syncthreads();
                phi_rows(dm, Wk, vs, ph2, nr);
                for (int rr = tid / WAVE; rr < nr; rr += NW) {
                    float av = 0.f;
                    for (int f = tid % WAVE; f < D; f += WAVE) av = fmaf(ph[f], ph2[rr * D + f], av);
                    av = wave_sum(av);
                    if (tid % WAVE == 0) wsc[t0 + rr] += query_term(sk, wlg[t0 + rr], av);
                }
                __syncthreads();
            }
        }
    }
    if (sk) for (int i = tid; i < wn; i += NT) win_score[i] = wsc[i];
    if (tid == 0) a.st.n_tokens[si] = tok + 1;
}

// ---------------------------------------------------------------------------------------------
// prefill
// ---------------------------------------------------------------------------------------------
// Rows of one stream during a prefill call are addressed by a "virtual row":
//   [0, lam)            copy of the sparse cache as it stood at entry,
//   [lam, lam + eta)    copy of the entry window, chronological, right-aligned,
//   P + i               token i of this call (P = lam + eta);
// token t (t >= a0 - eta, a0 = tokens consumed before the call) sits at row P + (t - a0).
template <typename T>
struct PrefillArgs {
    Dims dm;
    State<T> st;
    const T *q, *k, *v, *Wq, *Wk;
    void *out;
    int T_tokens, n_chunks;   // of the whole call
    int j0, j1;               // chunk range of this launch
    int jb;                   // first chunk of the pass: per-chunk workspace regions are indexed by chunk - jb
    T *prefK, *prefV;         // [B*Hkv][P][d]
    int32_t *sp_row;          // [B*Hkv][lam] virtual row held by each sparse slot
    float *phiE;              // [B*Hkv][lam + C][D] features of the eligible set (scan scratch)
    float *snapH, *snapS;     // [B*Hkv][S][D][d], [B*Hkv][S][D]: state at the entry of each chunk of the pass
    int32_t *snapG;           // [B*Hkv][S][lam]: virtual rows of the sparse cache at chunk entry, -1 = empty
    int S;                    // chunks per pass (snapshot capacity)
    int want_out;             // 0: update only (no snapshots)
    int32_t *sel_trace;       // [B*Hkv][n_chunks][lam] or NULL
    int R;                    // rows per scoring tile
    int QT;                   // queries per attend tile
    int snap_split;           // 1: H snapshots are written as bf16 high + low parts in MFMA operand order (D a multiple of 32)
    uint16_t *phiK;           // [B*Hkv][S][C][2][D] phi of the pass's keys, bf16 high + low parts (MFMA state-evolution kernel only)
    int scan_mode;            // scan_kernel: 0 all chunks of the launch; bit 0: stop at the first regular chunk (a full chunk with
                              // a full window behind it and a full cache: the MFMA kernel's case) and note it in next_j; bit 1:
                              // start from next_j instead of j0
    int32_t *next_j;          // [B*Hkv] hand-over of the chunk position between the kernels of a pass
    float *tok_score;         // [B*Hkv][eta + T] query-dependent scores: entry window (virtual rows lam ..), then the call's tokens
    int R2;                   // keys / queries per tile of band_score_kernel
};

// grid (stream, part): the parts of a stream share its rows evenly
template <typename T>
__global__ __launch_bounds__(NT) void prefix_kernel(PrefillArgs<T> a) {
    const Dims &dm = a.dm;
    const int si = blockIdx.x, d = dm.d, eta = dm.eta, lam = dm.lam, P = lam + eta;
    const int tid = blockIdx.y * NT + threadIdx.x, nth = gridDim.y * NT;
    const int64_t a0 = a.st.n_tokens[si];
    T *pK = a.prefK + (size_t)si * P * d, *pV = a.prefV + (size_t)si * P * d;
    const T *sp_k = a.st.sp_k + (size_t)si * lam * d, *sp_v = a.st.sp_v + (size_t)si * lam * d;
    const T *win_k = a.st.win_k + (size_t)si * eta * d, *win_v = a.st.win_v + (size_t)si * eta * d;
    // rows are copied as 16-byte pieces (a row is d * sizeof(T) bytes, a multiple of 16)
    const int ppr = d * (int)sizeof(T) / 16;
    const uint4 *sk4 = reinterpret_cast<const uint4 *>(sp_k), *sv4 = reinterpret_cast<const uint4 *>(sp_v);
    uint4 *pK4 = reinterpret_cast<uint4 *>(pK), *pV4 = reinterpret_cast<uint4 *>(pV);
    for (int p = tid; p < lam * ppr; p += nth) { pK4[p] = sk4[p]; pV4[p] = sv4[p]; }
    for (int s = tid; s < lam; s += nth) a.sp_row[(size_t)si * lam + s] = s;
    const int nw = (int)min((int64_t)eta, a0);
    const uint4 *wk4 = reinterpret_cast<const uint4 *>(win_k), *wv4 = reinterpret_cast<const uint4 *>(win_v);
    for (int p = tid; p < nw * ppr; p += nth) {
        int back = p / ppr + 1, i = p % ppr;      // token a0 - back
        int slot = (int)((a0 - back) % eta);
        size_t row = (size_t)(P - back);
        pK4[row * ppr + i] = wk4[(size_t)slot * ppr + i];
        pV4[row * ppr + i] = wv4[(size_t)slot * ppr + i];
    }
}

template <typename T>
__global__ __launch_bounds__(NT) void finalize_kernel(PrefillArgs<T> a) {
    const Dims &dm = a.dm;
    const int si = blockIdx.x, tid = threadIdx.x, d = dm.d, eta = dm.eta;
    const int64_t a0 = a.st.n_tokens[si];
    const int Tn = a.T_tokens;
    T *win_k = a.st.win_k + (size_t)si * eta * d, *win_v = a.st.win_v + (size_t)si * eta * d;
    const T *k = a.k + (size_t)si * Tn * d, *v = a.v + (size_t)si * Tn * d;
    const int first = max(0, Tn - eta);       // tokens of this call that end in the window
    const int ppr = d * (int)sizeof(T) / 16;  // 16-byte pieces per row
    const uint4 *k4 = reinterpret_cast<const uint4 *>(k), *v4 = reinterpret_cast<const uint4 *>(v);
    uint4 *wk4 = reinterpret_cast<uint4 *>(win_k), *wv4 = reinterpret_cast<uint4 *>(win_v);
    for (int p = tid; p < (Tn - first) * ppr; p += NT) {
        int i = first + p / ppr, c = p % ppr;
        int slot = (int)((a0 + i) % eta);
        wk4[(size_t)slot * ppr + c] = k4[(size_t)i * ppr + c];
        wv4[(size_t)slot * ppr + c] = v4[(size_t)i * ppr + c];
    }
    if (dm.score_kind) {
        // the sums of the pairs that end in the window (some may have been there before the call) go back to their ring slots
        float *win_score = a.st.win_score + (size_t)si * eta;
        const float *ts = a.tok_score + (size_t)si * (eta + Tn);
        const int64_t t_lo = max((int64_t)0, a0 + Tn - eta);
        for (int64_t t = t_lo + tid; t < a0 + Tn; t += NT) win_score[t % eta] = ts[eta + (t - a0)];
    }
    __syncthreads();
    if (tid == 0) a.st.n_tokens[si] = a0 + Tn;
}

// Query-dependent scores of a prefill call (Sec. 4 / appendix "scoring ablation"): row x of tok_score belongs to token
// a0 - eta + x (x < eta: the entry window, x >= eta: the call's tokens) and receives what the pair had gathered before
// the call plus the terms of the call's queries i (token a0 + i) with x - eta <= i <= x - 1, i.e. the queries that see
// the key inside the sliding-window band, over all query heads of the group.  Chunk-parallel: grid (key tile, stream).
// One wavefront owns a key and adds its terms in a fixed order (results do not depend on timing).
template <typename T>
__global__ __launch_bounds__(NT) void band_score_kernel(PrefillArgs<T> a) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const Dims &dm = a.dm;
    const int tid = threadIdx.x, d = dm.d, D = dm.D, m = dm.m, eta = dm.eta, lam = dm.lam, R = a.R2;
    const int si = blockIdx.y, b = si / dm.Hkv, h = si % dm.Hkv, x0 = blockIdx.x * R;
    const int Tn = a.T_tokens, nrows = eta + Tn, P = lam + eta;
    const int nk = min(R, nrows - x0);
    float *ks = smem;               // [R][d]
    float *phk = ks + R * d;        // [R][D]
    float *qs = phk + R * D;        // [R][d]
    float *phq = qs + R * d;        // [R][D]
    float *acc = phq + R * D;       // [R]
    const int64_t a0 = a.st.n_tokens[si];
    const T *pK = a.prefK + (size_t)si * P * d;
    const T *kc = a.k + (size_t)si * Tn * d;
    const float *win_score = a.st.win_score + (size_t)si * eta;
    for (int p = tid; p < nk * d; p += NT) {
        const int r = p / d, c = p - r * d, x = x0 + r;
        const bool valid = a0 - eta + x >= 0;
        ks[p] = !valid ? 0.f : (x < eta ? ldf(pK, (size_t)(lam + x) * d + c) : ldf(kc, (size_t)(x - eta) * d + c));
    }
    for (int r = tid; r < nk; r += NT) {
        const int x = x0 + r;
        const int64_t t = a0 - eta + x;
        acc[r] = (x < eta && t >= 0) ? win_score[t % eta] : 0.f;
    }
    __syncthreads();
    phi_rows(dm, a.Wk + (size_t)h * d * m, ks, phk, nk);
    const int i_lo = max(0, x0 - eta), i_hi = min(Tn - 1, x0 + nk - 2);   // queries that see some key of the tile
    const int w = tid / WAVE, lane = tid % WAVE;
    for (int r = 0; r < dm.g; r++) {
        const int hq = h * dm.g + r;
        const T *qh = a.q + ((size_t)b * dm.Hq + hq) * Tn * d;
        for (int i0 = i_lo; i0 <= i_hi; i0 += R) {
            const int nq = min(R, i_hi + 1 - i0);
            for (int p = tid; p < nq * d; p += NT) qs[p] = ldf(qh, (size_t)i0 * d + p);
            __syncthreads();
            phi_rows(dm, a.Wq + (size_t)hq * d * m, qs, phq, nq);
            for (int kr = w; kr < nk; kr += NW) {
                const int x = x0 + kr;
                if (a0 - eta + x < 0) continue;
                float sum = 0.f;
                for (int ql = 0; ql < nq; ql++) {
                    const int i = i0 + ql;
                    if (i < x - eta || i > x - 1) continue;
                    float dot = 0.f, av = 0.f;
                    for (int c = lane; c < d; c += WAVE) dot = fmaf(qs[ql * d + c], ks[kr * d + c], dot);
                    for (int f = lane; f < D; f += WAVE) av = fmaf(phq[ql * D + f], phk[kr * D + f], av);
                    dot = wave_sum(dot); av = wave_sum(av);
                    sum += query_term(dm.score_kind, dot * dm.scale, av);
                }
                if (lane == 0) acc[kr] += sum;
            }
            __syncthreads();
        }
    }
    for (int r = tid; r < nk; r += NT) a.tok_score[(size_t)si * nrows + x0 + r] = acc[r];
}

// One chunk of the sequential evolution of a stream's memories, all state in global memory (H^T, s, cache) except the
// sparse-cache fill count `spc`, which the caller carries.  Workgroup-wide (NT threads); `smem` is scratch LDS.
template <typename T>
__device__ void scan_chunk(const PrefillArgs<T> &a, const int si, const int j, int &spc, float *smem) {
    const Dims &dm = a.dm;
    const int tid = threadIdx.x, d = dm.d, D = dm.D, m = dm.m, eta = dm.eta, lam = dm.lam, C = dm.C, R = a.R;
    const int P = lam + eta, nEmax = lam + C;
    const int h = si % dm.Hkv;
    float *xs = smem;                   // [R][d]
    float *ph = xs + R * d;             // [R][D]
    float *vs = ph + R * D;             // [R][d]
    float *err = vs + R * d;            // [R][d]
    float *den = err + R * d;           // [R]
    float *score = den + R;             // [nEmax]
    int *cidx = (int *)(score + nEmax); // [nEmax] token index of each candidate
    int *keep = cidx + nEmax;           // [nEmax]
    int *flist = keep + nEmax;          // [nEmax] candidates to fold
    int *eslot = flist + nEmax;         // [C] destination slot of each entrant
    int *ecand = eslot + C;             // [C] candidate index of each entrant
    __shared__ int sh_nf, sh_ne;

    float *H = a.st.H + (size_t)si * D * d;
    float *s = a.st.s + (size_t)si * D;
    T *sp_k = a.st.sp_k + (size_t)si * lam * d, *sp_v = a.st.sp_v + (size_t)si * lam * d;
    int32_t *sp_idx = a.st.sp_idx + (size_t)si * lam;
    int32_t *sp_row = a.sp_row + (size_t)si * lam;
    float *phiE = a.phiE + (size_t)si * nEmax * D;
    const T *Wk = a.Wk + (size_t)h * d * m;
    const T *pK = a.prefK + (size_t)si * P * d, *pV = a.prefV + (size_t)si * P * d;
    const T *kc = a.k + (size_t)si * a.T_tokens * d, *vc = a.v + (size_t)si * a.T_tokens * d;
    const int64_t a0 = a.st.n_tokens[si];
    const int sk = dm.score_kind;
    float *sp_score = sk ? a.st.sp_score + (size_t)si * lam : nullptr;
    const float *tsc = sk ? a.tok_score + (size_t)si * (eta + a.T_tokens) : nullptr;

    {

        const int cl = min(C, a.T_tokens - j * C);
        const int64_t aj = a0 + (int64_t)j * C;
        if (a.want_out) {   // snapshot of the memories the chunk's queries read
            const size_t sj = (size_t)si * a.S + (j - a.jb);
            float *sH = a.snapH + sj * D * d, *sS = a.snapS + sj * D;
            int32_t *sG = a.snapG + sj * lam;
            if (a.snap_split) {
                // feature f sits in 16-byte piece (f/32)*4 + (f/4)%4, element 4*((f/16)%2) + f%4 of its row; pieces are
                // ordered [part][row tile of 16][k-step = piece / 4][16 (piece % 4) + row % 16] (the order in
                // which the MFMA kernels hold them, one contiguous 1 KB per wavefront store)
                uint16_t *s16 = reinterpret_cast<uint16_t *>(sH);
                const int ppr = D / 8, ksd = D / 32;            // 16-byte pieces per row, k-steps of 32 features
                for (int pi = tid; pi < D * d / 8; pi += NT) {   // one 16-byte piece (8 features of one row) per step
                    const int c = pi / ppr, piece = pi % ppr;
                    const float *src = H + (size_t)c * D + 32 * (piece >> 2) + 4 * (piece & 3);
                    const float4 lo4 = *reinterpret_cast<const float4 *>(src), hi4 = *reinterpret_cast<const float4 *>(src + 16);
                    const float x[8] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};
                    uint32_t ph[4], pl[4];
#pragma unroll
                    for (int e = 0; e < 4; e++) {
                        const uint16_t h0 = f32_to_bf16_bits(x[2 * e]), h1 = f32_to_bf16_bits(x[2 * e + 1]);
                        const float r0 = x[2 * e] - __uint_as_float(((uint32_t)h0) << 16), r1 = x[2 * e + 1] - __uint_as_float(((uint32_t)h1) << 16);
                        ph[e] = (uint32_t)h0 | ((uint32_t)h1 << 16);
                        pl[e] = (uint32_t)f32_to_bf16_bits(r0) | ((uint32_t)f32_to_bf16_bits(r1) << 16);
                    }
                    const int pos = ((((c >> 4) * ksd + (piece >> 2)) * 64) + 16 * (piece & 3) + (c & 15)) << 3;
                    *reinterpret_cast<uint4 *>(s16 + pos) = make_uint4(ph[0], ph[1], ph[2], ph[3]);
                    *reinterpret_cast<uint4 *>(s16 + D * d + pos) = make_uint4(pl[0], pl[1], pl[2], pl[3]);
                }
            } else {
                for (int idx = tid; idx < D * d; idx += NT) sH[idx] = H[idx];
            }
            for (int f = tid; f < D; f += NT) sS[f] = s[f];
            for (int sl = tid; sl < lam; sl += NT) sG[sl] = sl < spc ? sp_row[sl] : -1;
        }
        // tokens leaving the window once the chunk has joined it
        const int64_t lo = max((int64_t)0, aj - eta), hi = max((int64_t)0, aj + cl - eta);
        const int n_ev = (int)(hi - lo);
        const int vrow0 = P + (int)(lo - a0);
        if (n_ev > 0 && spc + n_ev <= lam) {
            // warm-up: everything is cached, nothing scored
            const int ppr = d * (int)sizeof(T) / 16;   // rows are copied as 16-byte pieces
            for (int p = tid; p < n_ev * ppr; p += NT) {
                int e = p / ppr, i = p - e * ppr, vr = vrow0 + e;
                const T *ksrc = vr < P ? pK + (size_t)vr * d : kc + (size_t)(vr - P) * d;
                const T *vsrc = vr < P ? pV + (size_t)vr * d : vc + (size_t)(vr - P) * d;
                reinterpret_cast<uint4 *>(sp_k + (size_t)(spc + e) * d)[i] = reinterpret_cast<const uint4 *>(ksrc)[i];
                reinterpret_cast<uint4 *>(sp_v + (size_t)(spc + e) * d)[i] = reinterpret_cast<const uint4 *>(vsrc)[i];
            }
            for (int e = tid; e < n_ev; e += NT) {
                sp_idx[spc + e] = (int32_t)(lo + e); sp_row[spc + e] = vrow0 + e;
                if (sk) sp_score[spc + e] = tsc[vrow0 + e - lam];
            }
            spc += n_ev;
            __syncthreads();
        } else if (n_ev > 0) {
            const int nE = spc + n_ev;
            for (int t0 = 0; t0 < nE; t0 += R) {
                int nr = min(R, nE - t0);
                const int ppr = d * (int)sizeof(T) / 16;   // 16-byte pieces per stored row
                for (int p = tid; p < nr * ppr; p += NT) {
                    const int r = p / ppr, i = p - r * ppr, e = t0 + r;
                    const T *ksrc, *vsrc;
                    if (e < spc) { ksrc = sp_k + (size_t)e * d; vsrc = sp_v + (size_t)e * d; }
                    else {
                        const int vr = vrow0 + (e - spc);
                        ksrc = vr < P ? pK + (size_t)vr * d : kc + (size_t)(vr - P) * d;
                        vsrc = vr < P ? pV + (size_t)vr * d : vc + (size_t)(vr - P) * d;
                    }
                    piece_to_f32(ksrc, i, xs + r * d);
                    piece_to_f32(vsrc, i, vs + r * d);
                }
                __syncthreads();
                phi_rows(dm, Wk, xs, ph, nr);
                for (int p = tid; p < nr * D; p += NT) phiE[(size_t)t0 * D + p] = ph[p];
                if (!sk) score_rows<std::is_same<T, bf16_t>::value>(dm, H, s, ph, vs, err, den, score + t0, nr);
                else __syncthreads();
            }
            if (sk) for (int e = tid; e < nE; e += NT) score[e] = e < spc ? sp_score[e] : tsc[vrow0 + (e - spc) - lam];
            for (int e = tid; e < nE; e += NT) cidx[e] = e < spc ? sp_idx[e] : (int)(lo + (e - spc));
            __syncthreads();
            // rank by (score descending, token index ascending); the first lam stay
            for (int e = tid; e < nE; e += NT) {
                float sc = score[e]; int ix = cidx[e], rank = 0;
                for (int o = 0; o < nE; o++) {
                    float so = score[o];
                    rank += (so > sc || (so == sc && cidx[o] < ix)) ? 1 : 0;
                }
                keep[e] = rank < lam;
            }
            __syncthreads();
            if (tid < WAVE) {
                // one wavefront builds the lists, 64 candidates per step, positions from ballots (candidate order kept):
                // the pairs to fold, the entrants, and the slots they take: those of leaving cache entries first, then
                // the never-used tail
                const unsigned long long below = (1ull << tid) - 1ull;
                int nf = 0, ne = 0, nfree = 0;
                for (int e0 = 0; e0 < nE; e0 += WAVE) {
                    const int e = e0 + tid;
                    const bool in = e < nE, kp = in && keep[e];
                    const bool fo = in && !kp, en = kp && e >= spc;
                    const unsigned long long mf = __ballot(fo), me = __ballot(en);
                    if (fo) flist[nf + __popcll(mf & below)] = e;
                    if (en) ecand[ne + __popcll(me & below)] = e;
                    nf += __popcll(mf); ne += __popcll(me);
                }
                for (int e0 = 0; e0 < spc; e0 += WAVE) {
                    const int e = e0 + tid;
                    const bool lv = e < spc && !keep[e];
                    const unsigned long long ml = __ballot(lv);
                    const int pos = nfree + __popcll(ml & below);
                    if (lv && pos < ne) eslot[pos] = e;
                    nfree += __popcll(ml);
                }
                if (nfree > ne) nfree = ne;
                for (int sl = spc + tid; sl < lam && nfree + (sl - spc) < ne; sl += WAVE) eslot[nfree + (sl - spc)] = sl;
                if (tid == 0) { sh_nf = nf; sh_ne = ne; }
            }
            __syncthreads();
            const int nf = sh_nf, ne = sh_ne;
            // fold: H += sum phi(k) v^T, s += sum phi(k) over the pairs that do not stay.  R pairs at a time are staged in
            // LDS (features and values as fp32) and every thread accumulates blocks of 4 value columns x 16 features in
            // registers: 5 LDS reads of 16 bytes per 64 multiply-adds, where the plain loop below reads global memory
            // twice per multiply-add (0.9 ms per chunk at the 8B shape).
            if (d % 4 == 0 && D % 16 == 0) {
                const int nbf = D / 16, nblk = (d / 4) * nbf;
                for (int t0 = 0; t0 < nf; t0 += R) {
                    const int nr = min(R, nf - t0);
                    for (int p = tid; p < nr * (D / 4); p += NT) {
                        const int r = p / (D / 4), i = p - r * (D / 4);
                        reinterpret_cast<float4 *>(ph + r * D)[i] = reinterpret_cast<const float4 *>(phiE + (size_t)flist[t0 + r] * D)[i];
                    }
                    const int ppr = d * (int)sizeof(T) / 16;
                    for (int p = tid; p < nr * ppr; p += NT) {
                        const int r = p / ppr, i = p - r * ppr, e = flist[t0 + r];
                        const T *vsrc;
                        if (e < spc) vsrc = sp_v + (size_t)e * d;
                        else { const int vr = vrow0 + (e - spc); vsrc = vr < P ? pV + (size_t)vr * d : vc + (size_t)(vr - P) * d; }
                        piece_to_f32(vsrc, i, vs + r * d);
                    }
                    __syncthreads();
                    for (int b = tid; b < nblk; b += NT) {
                        const int c0 = 4 * (b / nbf), f0 = 16 * (b % nbf);
                        float acc[4][16];
#pragma unroll
                        for (int i = 0; i < 4; i++)
#pragma unroll
                            for (int x = 0; x < 16; x++) acc[i][x] = 0.f;
                        for (int r = 0; r < nr; r++) {
                            const float4 v4 = *reinterpret_cast<const float4 *>(vs + r * d + c0);
                            const float vv[4] = {v4.x, v4.y, v4.z, v4.w};
#pragma unroll
                            for (int q4 = 0; q4 < 4; q4++) {
                                const float4 p4 = *reinterpret_cast<const float4 *>(ph + r * D + f0 + 4 * q4);
#pragma unroll
                                for (int i = 0; i < 4; i++) {
                                    acc[i][4 * q4] = fmaf(p4.x, vv[i], acc[i][4 * q4]); acc[i][4 * q4 + 1] = fmaf(p4.y, vv[i], acc[i][4 * q4 + 1]);
                                    acc[i][4 * q4 + 2] = fmaf(p4.z, vv[i], acc[i][4 * q4 + 2]); acc[i][4 * q4 + 3] = fmaf(p4.w, vv[i], acc[i][4 * q4 + 3]);
                                }
                            }
                        }
#pragma unroll
                        for (int i = 0; i < 4; i++)
#pragma unroll
                            for (int q4 = 0; q4 < 4; q4++) {
                                float4 *hp = reinterpret_cast<float4 *>(H + (size_t)(c0 + i) * D + f0 + 4 * q4);
                                float4 hv = *hp;
                                hv.x += acc[i][4 * q4]; hv.y += acc[i][4 * q4 + 1]; hv.z += acc[i][4 * q4 + 2]; hv.w += acc[i][4 * q4 + 3];
                                *hp = hv;
                            }
                    }
                    for (int f = tid; f < D; f += NT) {
                        float acc = 0.f;
                        for (int r = 0; r < nr; r++) acc += ph[r * D + f];
                        s[f] += acc;
                    }
                    __syncthreads();
                }
            } else {
            for (int idx = tid; idx < D * d; idx += NT) {
                int c = idx / D, f = idx - c * D;
                float acc = 0.f;
                for (int x = 0; x < nf; x++) {
                    int e = flist[x];
                    float val;
                    if (e < spc) val = ldf(sp_v, (size_t)e * d + c);
                    else { int vr = vrow0 + (e - spc); val = vr < P ? ldf(pV, (size_t)vr * d + c) : ldf(vc, (size_t)(vr - P) * d + c); }
                    acc = fmaf(phiE[(size_t)e * D + f], val, acc);
                }
                H[idx] += acc;
            }
            for (int f = tid; f < D; f += NT) {
                float acc = 0.f;
                for (int x = 0; x < nf; x++) acc += phiE[(size_t)flist[x] * D + f];
                s[f] += acc;
            }
            }
            __syncthreads();
            // compaction: entrants overwrite the slots that were freed
            const int ppr = d * (int)sizeof(T) / 16;   // 16-byte pieces per row
            for (int p = tid; p < ne * ppr; p += NT) {
                int x = p / ppr, i = p - x * ppr;
                int vr = vrow0 + (ecand[x] - spc), sl = eslot[x];
                const T *ksrc = vr < P ? pK + (size_t)vr * d : kc + (size_t)(vr - P) * d;
                const T *vsrc = vr < P ? pV + (size_t)vr * d : vc + (size_t)(vr - P) * d;
                reinterpret_cast<uint4 *>(sp_k + (size_t)sl * d)[i] = reinterpret_cast<const uint4 *>(ksrc)[i];
                reinterpret_cast<uint4 *>(sp_v + (size_t)sl * d)[i] = reinterpret_cast<const uint4 *>(vsrc)[i];
            }
            for (int x = tid; x < ne; x += NT) {
                sp_idx[eslot[x]] = cidx[ecand[x]];
                sp_row[eslot[x]] = vrow0 + (ecand[x] - spc);
                if (sk) sp_score[eslot[x]] = score[ecand[x]];
            }
            spc = lam;
            __syncthreads();
        }
        if (a.sel_trace) {
            int32_t *tr = a.sel_trace + ((size_t)si * a.n_chunks + j) * lam;
            for (int sl = tid; sl < lam; sl += NT) tr[sl] = sl < spc ? sp_idx[sl] : -1;
        }
        __syncthreads();
    }
}

// Sequential evolution of one stream's memories over the chunks [j0, j1).
template <typename T>
__global__ __launch_bounds__(NT) void scan_kernel(PrefillArgs<T> a) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int si = blockIdx.x;
    int spc = a.st.sp_count[si];
    int j = (a.scan_mode & 2) ? a.next_j[si] : a.j0;
    const int64_t a0 = a.st.n_tokens[si];
    for (; j < a.j1; j++) {
        if (a.scan_mode & 1) {
            const int cl = min(a.dm.C, a.T_tokens - j * a.dm.C);
            if (cl == a.dm.C && a0 + (int64_t)j * a.dm.C >= a.dm.eta && spc == a.dm.lam) break;
        }
        scan_chunk(a, si, j, spc, smem);
    }
    if (threadIdx.x == 0) {
        a.st.sp_count[si] = spc;
        if (a.scan_mode & 1) a.next_j[si] = j;
    }
}

// Outputs of one chunk of one query head from the snapshot taken at the chunk's entry.
template <typename T, typename TO>
__global__ __launch_bounds__(NT) void attend_kernel(PrefillArgs<T> a) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const Dims &dm = a.dm;
    const int tid = threadIdx.x, d = dm.d, D = dm.D, m = dm.m, eta = dm.eta, lam = dm.lam, C = dm.C, QT = a.QT;
    const int P = lam + eta, nkmax = lam + eta + C;
    const int j = a.j0 + blockIdx.x, jj = j - a.jb, hq = blockIdx.y, b = blockIdx.z;
    const int h = hq / dm.g, si = b * dm.Hkv + h;
    float *qs = smem;                 // [QT][d]
    float *phq = qs + QT * d;         // [QT][D]
    float *pw = phq + QT * D;         // [QT][nkmax]
    float *rmax = pw + QT * nkmax;    // [QT]
    float *rsum = rmax + QT;          // [QT]
    float *rlin = rsum + QT;          // [QT]

    const int64_t a0 = a.st.n_tokens[si];
    const int Tn = a.T_tokens;
    const int cl = min(C, Tn - j * C);
    const int64_t aj = a0 + (int64_t)j * C;
    const int64_t lo = max((int64_t)0, aj - eta);
    const int vrow0 = P + (int)(lo - a0);
    const int nwin = (int)(aj + cl - lo);          // window at entry + the whole chunk
    const int nk = lam + nwin;
    const size_t sj = (size_t)si * a.S + jj;
    const float *Hj = a.snapH + sj * D * d, *sjv = a.snapS + sj * D;
    const int32_t *G = a.snapG + sj * lam;
    const T *pK = a.prefK + (size_t)si * P * d, *pV = a.prefV + (size_t)si * P * d;
    const T *kc = a.k + (size_t)si * Tn * d, *vc = a.v + (size_t)si * Tn * d;
    const T *qh = a.q + (((size_t)b * dm.Hq + hq) * Tn + (size_t)j * C) * d;
    TO *oh = (TO *)a.out + (((size_t)b * dm.Hq + hq) * Tn + (size_t)j * C) * d;
    const T *Wq = a.Wq + (size_t)hq * d * m;
    const int w = tid / WAVE, lane = tid % WAVE;

    for (int i0 = 0; i0 < cl; i0 += QT) {
        const int nq = min(QT, cl - i0);
        for (int p = tid; p < nq * d; p += NT) qs[p] = ldf(qh, (size_t)i0 * d + p);
        __syncthreads();
        phi_rows(dm, Wq, qs, phq, nq);
        // logits; a key is visible to query i iff it is cached, in the entry window, or a chunk token <= i
        // (one thread per key: its row is read once for all queries of the tile)
        for (int key = tid; key < nk; key += NT) {
            int vr; bool row_ok = true;
            if (key < lam) { vr = G[key]; row_ok = vr >= 0 && !(dm.hide & 2); }
            else vr = vrow0 + (key - lam);
            float lq[16];
#pragma unroll
            for (int qi = 0; qi < 16; qi++) lq[qi] = 0.f;
            if (row_ok) {
                const T *kr = vr < P ? pK + (size_t)vr * d : kc + (size_t)(vr - P) * d;
                dot_row_many(kr, qs, d, nq, lq);
            }
#pragma unroll
            for (int qi = 0; qi < 16; qi++) {
                if (qi < nq) {
                    const bool ok = key < lam ? row_ok : (lo + (key - lam)) <= (aj + i0 + qi);
                    pw[qi * nkmax + key] = ok ? lq[qi] * dm.scale : -INFINITY;
                }
            }
        }
        __syncthreads();
        for (int qi = w; qi < nq; qi += NW) {
            float *row = pw + qi * nkmax;
            float mx = 0.f;
            for (int key = lane; key < nk; key += WAVE) mx = fmaxf(mx, row[key]);
            mx = wave_max(mx);
            float sum = 0.f;
            for (int key = lane; key < nk; key += WAVE) {
                float p = expf(row[key] - mx);    // exp(-inf) = 0 for masked keys
                row[key] = p;
                sum += p;
            }
            sum = wave_sum(sum);
            float lin = 0.f;
            for (int f = lane; f < D; f += WAVE) lin = fmaf(phq[qi * D + f], sjv[f], lin);
            lin = wave_sum(lin);
            if (lane == 0) { rmax[qi] = mx; rsum[qi] = sum; rlin[qi] = lin; }
        }
        __syncthreads();
        // one thread per value column (and per group of queries): a value row and a row of H^T are read once for all
        // the thread's queries of the tile, the sums of each query run in key / feature order
        const int c = tid % d, part = tid / d, nparts = NT / d;
        float num[16], lin[16];
#pragma unroll
        for (int x = 0; x < 16; x++) { num[x] = 0.f; lin[x] = 0.f; }
        for (int key = 0; key < nk; key++) {
            const int vr = key < lam ? G[key] : vrow0 + (key - lam);
            if (vr < 0) continue;   // empty slot: weight 0 for every query
            const float val = vr < P ? ldf(pV, (size_t)vr * d + c) : ldf(vc, (size_t)(vr - P) * d + c);
#pragma unroll
            for (int x = 0; x < 16; x++) {
                const int qi = part + x * nparts;
                if (qi < nq) num[x] = fmaf(pw[qi * nkmax + key], val, num[x]);
            }
        }
        if ((D & 3) == 0) {
            const float4 *H4 = reinterpret_cast<const float4 *>(Hj + (size_t)c * D);
            for (int f4 = 0; f4 < D / 4; f4++) {
                const float4 hv = H4[f4];
#pragma unroll
                for (int x = 0; x < 16; x++) {
                    const int qi = part + x * nparts;
                    if (qi < nq) {
                        const float4 pv = reinterpret_cast<const float4 *>(phq + qi * D)[f4];
                        float t = lin[x];
                        t = fmaf(pv.x, hv.x, t); t = fmaf(pv.y, hv.y, t); t = fmaf(pv.z, hv.z, t); t = fmaf(pv.w, hv.w, t);
                        lin[x] = t;
                    }
                }
            }
        } else {
#pragma unroll
            for (int x = 0; x < 16; x++) {
                const int qi = part + x * nparts;
                if (qi < nq) { float t = 0.f; for (int f = 0; f < D; f++) t = fmaf(phq[qi * D + f], Hj[(size_t)c * D + f], t); lin[x] = t; }
            }
        }
#pragma unroll
        for (int x = 0; x < 16; x++) {
            const int qi = part + x * nparts;
            if (qi < nq) {
                const float elin = (dm.hide & 1) ? 0.f : expf(-rmax[qi]);
                stf(oh, (size_t)(i0 + qi) * d + c, fmaf(elin, lin[x], num[x]) / (rsum[qi] + elin * rlin[qi]));
            }
        }
        __syncthreads();
    }
}

}  // namespace generic
}  // namespace lola

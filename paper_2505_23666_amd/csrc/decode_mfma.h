// Fused single-token generation step for the 8B/1B head shapes on gfx950: one workgroup of four
// wavefronts per (sequence, kv head), two workgroups resident per compute unit.
//
// What one launch does per stream (paper Sec. 3: E_t, G_t, S_t, H_t and y_t equations):
//   - the new pair replaces the oldest one in the window ring; the displaced pair p leaves;
//   - phi of the lambda cached keys (bf16 MFMA, exact products, fp32 accumulate, fp32 softmax),
//     recall phi(k)^T H / phi(k)^T s of all lambda + 1 eligible pairs with H held ONCE in LDS as
//     fp32 (operands split into bf16 high + low parts: three MFMAs per product, ~2^-17 relative),
//     squared self-recall error, arg-min (ties: larger token index goes);
//   - rank-1 fold of the dropped pair into H (in LDS) and s, H written back once;
//   - the dropped slot is overwritten in place by p (cache compaction);
//   - outputs of the G query heads: softmax weights over cache + window with m = max(0, max logit),
//     linear read-out phi(q)^T H taken from the same pass over H and corrected by the rank-1 term,
//     shared normaliser.
// H is read from HBM once and written once; cached K rows are read once, cached V rows twice
// (second time from cache).
//
// MFMA 16x16x32 bf16 register layout used throughout (verified on hardware):
//   A operand: lane l holds row l%16, k-slots 8*(l/16) + 0..7;  B operand: column l%16, same k-slots;
//   C/D: lane l holds column l%16, rows 4*(l/16) + 0..3.
// The contraction index may be permuted freely as long as A and B agree; the feature index uses
//   f(ks, e, grp) = 32*ks + 16*(e/4) + 4*grp + e%4
// so that the C layout of the phi GEMM is directly the B layout of the recall GEMM.
#pragma once
#include "lola_common.h"

namespace lola {
namespace fast {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ bf16x8 ld_bf16x8(const bf16_t *p) {
    uint4 u = *reinterpret_cast<const uint4 *>(p);
    return __builtin_bit_cast(bf16x8, u);
}
__device__ __forceinline__ bf16x8 zero_bf16x8() {
    uint4 u = make_uint4(0, 0, 0, 0);
    return __builtin_bit_cast(bf16x8, u);
}
// x = hi + lo + O(2^-17 |x|), both parts bf16
__device__ __forceinline__ void split8(const float x[8], bf16x8 &hi, bf16x8 &lo) {
#pragma unroll
    for (int e = 0; e < 8; e++) {
        __bf16 h = (__bf16)x[e];
        hi[e] = h;
        lo[e] = (__bf16)(x[e] - (float)h);
    }
}
__device__ __forceinline__ float bf_bits_to_f(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

template <typename TO>
struct DecodeFastArgs {
    State<bf16_t> st;
    const bf16_t *q, *k, *v, *Wq, *Wk;
    TO *out;
    int Hq, Hkv;
    float scale;
    int phi_kind;
};

// DH = head_dim = 128, feature dim D = 128 (M = 64 projections), LAM multiple of 16 (<= 128 here),
// ETA = 64, G = query heads per kv head (<= 4).
template <int LAM, int ETA, int G, typename TO>
__global__ __launch_bounds__(256, 2) void decode_fast_kernel(DecodeFastArgs<TO> a) {
    constexpr int DH = 128, M = 64, D = 128;
    constexpr int NKT = LAM / 16;          // key tiles of the sparse cache
    constexpr int TPW = (NKT + 3) / 4;     // key tiles per wavefront
    constexpr int NWT = ETA / 16;          // window tiles
    constexpr int KP = LAM;                // position of the leaving pair in the logit / score arrays
    constexpr int KW = LAM + 1;            // first window position
    constexpr int NKEY = LAM + 1 + ETA;
    static_assert(LAM % 16 == 0 && ETA % 16 == 0 && G >= 1 && G <= 4 && NKT <= 8 && NWT <= 4, "shape");

    __shared__ __attribute__((aligned(16))) float Hs[D * DH];   // fp32 H, column index XOR-swizzled by feature bit 2
    __shared__ float s_l[D];
    __shared__ float score2[LAM + 1];
    __shared__ float errX[4];
    __shared__ float lg[G][NKEY];          // logits, then softmax weights
    __shared__ float phiX[1 + G][D];       // row 0: phi of the leaving key; rows 1..G: phi of the queries
    __shared__ float lin[G][DH];           // phi(q)^T H (state before the fold)
    __shared__ float denq[G], dotqf[G], psum_s[G], elin_s[G];
    __shared__ float phif[D], vf[DH];      // the folded pair
    __shared__ float pkf[DH], pvf[DH];     // the leaving pair
    __shared__ uint16_t pkb[DH], pvb[DH];
    __shared__ int idx_l[LAM];
    __shared__ int sh_drop;

    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, r16 = lane & 15, g4 = lane >> 4;
    const int si = blockIdx.x, b = si / a.Hkv, h = si - b * a.Hkv;
    float *Hg = a.st.H + (size_t)si * D * DH;
    float *sg = a.st.s + (size_t)si * D;
    bf16_t *win_k = a.st.win_k + (size_t)si * ETA * DH, *win_v = a.st.win_v + (size_t)si * ETA * DH;
    bf16_t *sp_k = a.st.sp_k + (size_t)si * LAM * DH, *sp_v = a.st.sp_v + (size_t)si * LAM * DH;
    int32_t *sp_idx = a.st.sp_idx + (size_t)si * LAM;
    const bf16_t *Wk = a.Wk + (size_t)h * DH * M;
    const bf16_t *knew = a.k + (size_t)si * DH, *vnew = a.v + (size_t)si * DH;
    const bf16_t *qg = a.q + ((size_t)b * a.Hq + (size_t)h * G) * DH;   // G consecutive query rows

    const int64_t tok = a.st.n_tokens[si];
    const int spc = a.st.sp_count[si];
    const bool popped = tok >= (int64_t)ETA;
    const bool steady = popped && spc == LAM;          // scoring happens; H may be non-zero
    const int slot = (int)(tok % ETA);
    const int pidx = (int)(tok - ETA);
    const int wn = (int)min((int64_t)ETA, tok + 1);   // window pairs after the push

    // ---- stage 0: small per-stream vectors; the leaving pair is read before its slot is overwritten
    if (tid < D) { s_l[tid] = sg[tid]; }
    if (tid < LAM) idx_l[tid] = sp_idx[tid];
    if (popped && tid < DH) {
        uint16_t kb = win_k[(size_t)slot * DH + tid].x, vb = win_v[(size_t)slot * DH + tid].x;
        pkb[tid] = kb; pvb[tid] = vb;
        pkf[tid] = bf_bits_to_f(kb); pvf[tid] = bf_bits_to_f(vb);
    }
    __syncthreads();
    if (tid < 16) reinterpret_cast<uint4 *>(win_k + (size_t)slot * DH)[tid] = reinterpret_cast<const uint4 *>(knew)[tid];
    else if (tid < 32) reinterpret_cast<uint4 *>(win_v + (size_t)slot * DH)[tid - 16] = reinterpret_cast<const uint4 *>(vnew)[tid - 16];

    // ---- query rows as MFMA A operand (rows >= G are zero)
    bf16x8 AQ[4];
#pragma unroll
    for (int ks = 0; ks < 4; ks++) AQ[ks] = r16 < G ? ld_bf16x8(qg + (size_t)r16 * DH + 32 * ks + 8 * g4) : zero_bf16x8();

    // ---- stage 1a: phi of the queries (and of the leaving key) on the vector ALUs, one vector per wavefront
    // lane j computes projection j; W reads are coalesced along j
    if (steady) {
        for (int r = w; r < 1 + G; r += 4) {
            // r < G: query r (row r + 1 of phiX); r == G: the leaving key (row 0)
            const bf16_t *W = r < G ? a.Wq + ((size_t)h * G + r) * DH * M : Wk;
            float z = 0.f;
            if (r < G) {
                const bf16_t *x = qg + (size_t)r * DH;
#pragma unroll 8
                for (int i = 0; i < DH; i++) z = fmaf(ldf(W, (size_t)i * M + lane), ldf(x, i), z);
            } else {
#pragma unroll 8
                for (int i = 0; i < DH; i++) z = fmaf(ldf(W, (size_t)i * M + lane), pkf[i], z);
            }
            float pp, pn;
            if (a.phi_kind == 1) { pp = __expf(z); pn = __expf(-z); }
            else {
                float zmax = wave_max(z), zmin = wave_min(z);
                float ep = __expf(z - zmax), en = __expf(zmin - z);
                pp = ep / wave_sum(ep); pn = en / wave_sum(en);
            }
            const int row = r < G ? r + 1 : 0;
            phiX[row][lane] = pp; phiX[row][M + lane] = pn;
            float dn = wave_sum(pp * s_l[lane] + pn * s_l[M + lane]);
            if (lane == 0) { if (r < G) denq[r] = dn; else errX[0] = dn; }   // errX[0] temporarily carries the leaving key's denominator
        }
    }
    // logit of the leaving key (it is attended if it stays in the cache)
    if (popped) {
        for (int r = w; r < G; r += 4) {
            const bf16_t *x = qg + (size_t)r * DH;
            float dot = ldf(x, lane) * pkf[lane] + ldf(x, lane + 64) * pkf[lane + 64];
            dot = wave_sum(dot);
            if (lane == 0) lg[r][KP] = dot * a.scale;
        }
    }

    // ---- stage 1b: per key tile: logits (Q K^T) and, in steady state, phi(K) -> B operands of the recall GEMM
    bf16x8 AW[4][4];
    if (steady) {
#pragma unroll
        for (int mt = 0; mt < 4; mt++)
#pragma unroll
            for (int ks = 0; ks < 4; ks++) {
                bf16x8 t;
#pragma unroll
                for (int e = 0; e < 8; e++) {
                    uint16_t bits = Wk[(size_t)(32 * ks + 8 * g4 + e) * M + 16 * mt + r16].x;
                    t[e] = __builtin_bit_cast(__bf16, bits);
                }
                AW[mt][ks] = t;
            }
    }
    bf16x8 Bhi[TPW][4], Blo[TPW][4];
    float rden[TPW];
#pragma unroll
    for (int t = 0; t < TPW; t++) {
        const int tile = w + 4 * t;
        rden[t] = 0.f;
        if (tile < NKT) {
            const int key = 16 * tile + r16;
            bf16x8 BK[4];
#pragma unroll
            for (int ks = 0; ks < 4; ks++) BK[ks] = ld_bf16x8(sp_k + (size_t)key * DH + 32 * ks + 8 * g4);
            f32x4 accL = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ks++) accL = mfma16(AQ[ks], BK[ks], accL);
            if (g4 == 0) {
#pragma unroll
                for (int i = 0; i < G; i++) lg[i][key] = accL[i] * a.scale;
            }
            if (steady) {
                f32x4 z[4];
#pragma unroll
                for (int mt = 0; mt < 4; mt++) {
                    z[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < 4; ks++) z[mt] = mfma16(AW[mt][ks], BK[ks], z[mt]);
                }
                // lane holds z[key][16*mt + 4*g4 + i]; the other three lane groups hold the rest of the row
                float pp[16], pn[16];
                if (a.phi_kind == 1) {
#pragma unroll
                    for (int x = 0; x < 16; x++) { float zz = z[x >> 2][x & 3]; pp[x] = __expf(zz); pn[x] = __expf(-zz); }
                } else {
                    float zmax = z[0][0], zmin = z[0][0];
#pragma unroll
                    for (int x = 1; x < 16; x++) { zmax = fmaxf(zmax, z[x >> 2][x & 3]); zmin = fminf(zmin, z[x >> 2][x & 3]); }
                    zmax = fmaxf(zmax, __shfl_xor(zmax, 16, WAVE)); zmax = fmaxf(zmax, __shfl_xor(zmax, 32, WAVE));
                    zmin = fminf(zmin, __shfl_xor(zmin, 16, WAVE)); zmin = fminf(zmin, __shfl_xor(zmin, 32, WAVE));
                    float sp = 0.f, sn = 0.f;
#pragma unroll
                    for (int x = 0; x < 16; x++) {
                        float zz = z[x >> 2][x & 3];
                        pp[x] = __expf(zz - zmax); pn[x] = __expf(zmin - zz);
                        sp += pp[x]; sn += pn[x];
                    }
                    sp += __shfl_xor(sp, 16, WAVE); sp += __shfl_xor(sp, 32, WAVE);
                    sn += __shfl_xor(sn, 16, WAVE); sn += __shfl_xor(sn, 32, WAVE);
                    const float ip = 1.0f / sp, in_ = 1.0f / sn;
#pragma unroll
                    for (int x = 0; x < 16; x++) { pp[x] *= ip; pn[x] *= in_; }
                }
                float dn = 0.f;
#pragma unroll
                for (int x = 0; x < 16; x++) {
                    const int f = 16 * (x >> 2) + 4 * g4 + (x & 3);
                    dn = fmaf(pp[x], s_l[f], dn);
                    dn = fmaf(pn[x], s_l[M + f], dn);
                }
                dn += __shfl_xor(dn, 16, WAVE); dn += __shfl_xor(dn, 32, WAVE);
                rden[t] = dn > 0.f ? 1.0f / dn : 0.f;
                // feature order of the recall GEMM: ks 0,1 -> positive half (mt 0,1 / 2,3), ks 2,3 -> negative half
                split8(&pp[0], Bhi[t][0], Blo[t][0]);
                split8(&pp[8], Bhi[t][1], Blo[t][1]);
                split8(&pn[0], Bhi[t][2], Blo[t][2]);
                split8(&pn[8], Bhi[t][3], Blo[t][3]);
            }
        }
    }
    // window logits: one tile per wavefront; the ring slot of the new token is taken from the input
    if (w < NWT) {
        const int row = 16 * w + r16;
        const bf16_t *src = row == slot ? knew : win_k + (size_t)row * DH;
        f32x4 accL = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ks++) accL = mfma16(AQ[ks], ld_bf16x8(src + 32 * ks + 8 * g4), accL);
        if (g4 == 0) {
#pragma unroll
            for (int i = 0; i < G; i++) lg[i][KW + row] = accL[i] * a.scale;
        }
    }

    int drop = -1;   // candidate that is folded: < LAM a cache slot, == LAM the leaving pair, -1 none
    if (steady) {
        // ---- stage 2: recall of all eligible pairs: P^T = H^T Phi^T, H from LDS
        // cached values in the C layout of P^T: lane (key r16, group g4) needs v[key][16*mt + 4*g4 + 0..3]
        uint2 vreg[TPW][8];
#pragma unroll
        for (int t = 0; t < TPW; t++) {
            const int tile = w + 4 * t;
            if (tile < NKT) {
#pragma unroll
                for (int mt = 0; mt < 8; mt++)
                    vreg[t][mt] = *reinterpret_cast<const uint2 *>(sp_v + (size_t)(16 * tile + r16) * DH + 16 * mt + 4 * g4);
            }
        }
        // H -> LDS (coalesced float4 reads, swizzled so that the four lane groups of an A-operand read hit distinct banks)
#pragma unroll 4
        for (int r = 0; r < (D * DH / 4) / 256; r++) {
            const int idx4 = tid + 256 * r, f = idx4 >> 5, c = (idx4 & 31) << 2;
            float4 val = reinterpret_cast<const float4 *>(Hg)[idx4];
            *reinterpret_cast<float4 *>(&Hs[f * DH + (c ^ (((f >> 2) & 1) << 4))]) = val;
        }
        __syncthreads();
        const float denP = errX[0];
        const float rdenX = denP > 0.f ? 1.0f / denP : 0.f;
        // B operands of the extra tile: row 0 the leaving key, rows 1..G the queries
        bf16x8 BXhi[4], BXlo[4];
#pragma unroll
        for (int ks = 0; ks < 4; ks++) {
            float x[8];
#pragma unroll
            for (int e = 0; e < 8; e++) x[e] = r16 <= G ? phiX[r16][32 * ks + 16 * (e >> 2) + 4 * g4 + (e & 3)] : 0.f;
            split8(x, BXhi[ks], BXlo[ks]);
        }
        float err[TPW], errP = 0.f;
#pragma unroll
        for (int t = 0; t < TPW; t++) err[t] = 0.f;
        const int swz = (g4 & 1) << 4;
#pragma unroll
        for (int mt = 0; mt < 8; mt++) {
            const bool doX = (mt >> 1) == w;     // the extra tile's eight column tiles are shared out, two per wavefront
            f32x4 acc[TPW], accX = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < TPW; t++) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
            const int c = (16 * mt + r16) ^ swz;
#pragma unroll
            for (int ks = 0; ks < 4; ks++) {
                float x[8];
#pragma unroll
                for (int e = 0; e < 8; e++) x[e] = Hs[(32 * ks + 16 * (e >> 2) + 4 * g4 + (e & 3)) * DH + c];
                bf16x8 Ahi, Alo;
                split8(x, Ahi, Alo);
#pragma unroll
                for (int t = 0; t < TPW; t++) {
                    if (w + 4 * t < NKT) {
                        acc[t] = mfma16(Ahi, Bhi[t][ks], acc[t]);
                        acc[t] = mfma16(Ahi, Blo[t][ks], acc[t]);
                        acc[t] = mfma16(Alo, Bhi[t][ks], acc[t]);
                    }
                }
                if (doX) {
                    accX = mfma16(Ahi, BXhi[ks], accX);
                    accX = mfma16(Ahi, BXlo[ks], accX);
                    accX = mfma16(Alo, BXhi[ks], accX);
                }
            }
#pragma unroll
            for (int t = 0; t < TPW; t++) {
                if (w + 4 * t < NKT) {
                    const uint2 vv = vreg[t][mt];
                    const float v0 = __uint_as_float(vv.x << 16), v1 = __uint_as_float(vv.x & 0xFFFF0000u);
                    const float v2 = __uint_as_float(vv.y << 16), v3 = __uint_as_float(vv.y & 0xFFFF0000u);
                    float e0 = fmaf(acc[t][0], rden[t], -v0), e1 = fmaf(acc[t][1], rden[t], -v1);
                    float e2 = fmaf(acc[t][2], rden[t], -v2), e3 = fmaf(acc[t][3], rden[t], -v3);
                    err[t] = fmaf(e0, e0, err[t]); err[t] = fmaf(e1, e1, err[t]);
                    err[t] = fmaf(e2, e2, err[t]); err[t] = fmaf(e3, e3, err[t]);
                }
            }
            if (doX) {
                const int c0 = 16 * mt + 4 * g4;
                if (r16 == 0) {
#pragma unroll
                    for (int i = 0; i < 4; i++) { float e = fmaf(accX[i], rdenX, -pvf[c0 + i]); errP = fmaf(e, e, errP); }
                } else if (r16 <= G) {
#pragma unroll
                    for (int i = 0; i < 4; i++) lin[r16 - 1][c0 + i] = accX[i];
                }
            }
        }
        __syncthreads();   // errX[0] (the leaving key's denominator) has been read by everyone
#pragma unroll
        for (int t = 0; t < TPW; t++) {
            float e = err[t];
            e += __shfl_xor(e, 16, WAVE); e += __shfl_xor(e, 32, WAVE);
            if (g4 == 0 && w + 4 * t < NKT) score2[16 * (w + 4 * t) + r16] = e;
        }
        errP += __shfl_xor(errP, 16, WAVE); errP += __shfl_xor(errP, 32, WAVE);
        if (lane == 0) errX[w] = errP;
        __syncthreads();

        // ---- stage 3: the pair that leaves the cache: smallest error, ties -> larger token index
        if (w == 0) {
            float bs = INFINITY; int bi = -1, be = 0;
            for (int e = lane; e <= LAM; e += WAVE) {
                float sc = e < LAM ? score2[e] : errX[0] + errX[1] + errX[2] + errX[3];
                int ix = e < LAM ? idx_l[e] : pidx;
                if (sc < bs || (sc == bs && ix > bi)) { bs = sc; bi = ix; be = e; }
            }
#pragma unroll
            for (int o = WAVE / 2; o > 0; o >>= 1) {
                float os = __shfl_xor(bs, o, WAVE); int oi = __shfl_xor(bi, o, WAVE), oe = __shfl_xor(be, o, WAVE);
                if (os < bs || (os == bs && oi > bi)) { bs = os; bi = oi; be = oe; }
            }
            if (lane == 0) sh_drop = be;
        }
        __syncthreads();
        drop = sh_drop;
        // phi and v of the folded pair
        if (drop < LAM) {
            const int tile = drop >> 4;
            if ((tile & 3) == w && r16 == (drop & 15)) {
                const int t = tile >> 2;
#pragma unroll
                for (int tt = 0; tt < TPW; tt++) {
                    if (tt == t) {
#pragma unroll
                        for (int ks = 0; ks < 4; ks++)
#pragma unroll
                            for (int e = 0; e < 8; e++)
                                phif[32 * ks + 16 * (e >> 2) + 4 * g4 + (e & 3)] = (float)Bhi[tt][ks][e] + (float)Blo[tt][ks][e];
                    }
                }
            }
            if (tid < DH) vf[tid] = ldf(sp_v, (size_t)drop * DH + tid);
        } else {
            if (tid < D) phif[tid] = phiX[0][tid];
            if (tid < DH) vf[tid] = pvf[tid];
        }
        __syncthreads();
        // the leaving pair takes the freed slot (in-place compaction)
        if (drop < LAM) {
            if (tid < 16) reinterpret_cast<uint4 *>(sp_k + (size_t)drop * DH)[tid] = reinterpret_cast<const uint4 *>(pkb)[tid];
            else if (tid < 32) reinterpret_cast<uint4 *>(sp_v + (size_t)drop * DH)[tid - 16] = reinterpret_cast<const uint4 *>(pvb)[tid - 16];
            else if (tid == 32) sp_idx[drop] = pidx;
        }
        // fold: H += phi_f v_f^T (written back once), s += phi_f
#pragma unroll 4
        for (int r = 0; r < (D * DH / 4) / 256; r++) {
            const int idx4 = tid + 256 * r, f = idx4 >> 5, c = (idx4 & 31) << 2;
            float4 hv = *reinterpret_cast<const float4 *>(&Hs[f * DH + (c ^ (((f >> 2) & 1) << 4))]);
            const float pf = phif[f];
            hv.x = fmaf(pf, vf[c], hv.x); hv.y = fmaf(pf, vf[c + 1], hv.y);
            hv.z = fmaf(pf, vf[c + 2], hv.z); hv.w = fmaf(pf, vf[c + 3], hv.w);
            reinterpret_cast<float4 *>(Hg)[idx4] = hv;
        }
        if (tid < D) sg[tid] = s_l[tid] + phif[tid];
        for (int r = w; r < G; r += 4) {
            float dq = wave_sum(phiX[r + 1][lane] * phif[lane] + phiX[r + 1][lane + 64] * phif[lane + 64]);
            if (lane == 0) dotqf[r] = dq;
        }
    } else if (popped) {
        // cache not full yet: the leaving pair is appended, nothing is scored (spc < LAM)
        if (tid < 16) reinterpret_cast<uint4 *>(sp_k + (size_t)spc * DH)[tid] = reinterpret_cast<const uint4 *>(pkb)[tid];
        else if (tid < 32) reinterpret_cast<uint4 *>(sp_v + (size_t)spc * DH)[tid - 16] = reinterpret_cast<const uint4 *>(pvb)[tid - 16];
        else if (tid == 32) { sp_idx[spc] = pidx; a.st.sp_count[si] = spc + 1; }
    }
    __syncthreads();

    // ---- stage 4: softmax weights (one query per wavefront), m = max(0, max logit)
    for (int r = w; r < G; r += 4) {
        float mx = 0.f;
        for (int key = lane; key < NKEY; key += WAVE) {
            bool ok;
            if (key < LAM) ok = key < spc && key != drop;
            else if (key == KP) ok = popped && drop != LAM;
            else ok = (key - KW) < wn;
            float l = ok ? lg[r][key] : -INFINITY;
            lg[r][key] = l;
            mx = fmaxf(mx, l);
        }
        mx = wave_max(mx);
        float sum = 0.f;
        for (int key = lane; key < NKEY; key += WAVE) {
            float p = __expf(lg[r][key] - mx);
            lg[r][key] = p;
            sum += p;
        }
        sum = wave_sum(sum);
        if (lane == 0) { psum_s[r] = sum; elin_s[r] = __expf(-mx); }
    }
    __syncthreads();

    // ---- stage 5: sum_i p_i v_i on the vector ALUs: thread (column group cg, row group rg), rows rg + 16 it
    float accv[G][8];
#pragma unroll
    for (int r = 0; r < G; r++)
#pragma unroll
        for (int x = 0; x < 8; x++) accv[r][x] = 0.f;
    {
        const int cg = tid & 15, rg = tid >> 4;
        for (int key = rg; key < NKEY; key += 16) {
            float p[G];
            bool any = false;
#pragma unroll
            for (int r = 0; r < G; r++) { p[r] = lg[r][key]; any |= p[r] != 0.f; }
            if (!any) continue;
            float vals[8];
            if (key == KP) {
#pragma unroll
                for (int x = 0; x < 8; x++) vals[x] = pvf[8 * cg + x];
            } else {
                const bf16_t *src;
                if (key < LAM) src = sp_v + (size_t)key * DH;
                else { const int row = key - KW; src = row == slot ? vnew : win_v + (size_t)row * DH; }
                const uint4 u = reinterpret_cast<const uint4 *>(src)[cg];
                vals[0] = __uint_as_float(u.x << 16); vals[1] = __uint_as_float(u.x & 0xFFFF0000u);
                vals[2] = __uint_as_float(u.y << 16); vals[3] = __uint_as_float(u.y & 0xFFFF0000u);
                vals[4] = __uint_as_float(u.z << 16); vals[5] = __uint_as_float(u.z & 0xFFFF0000u);
                vals[6] = __uint_as_float(u.w << 16); vals[7] = __uint_as_float(u.w & 0xFFFF0000u);
            }
#pragma unroll
            for (int r = 0; r < G; r++)
#pragma unroll
                for (int x = 0; x < 8; x++) accv[r][x] = fmaf(p[r], vals[x], accv[r][x]);
        }
    }
    // reduce over the four row groups of a wavefront, then over wavefronts through LDS (reusing the H tile)
#pragma unroll
    for (int r = 0; r < G; r++)
#pragma unroll
        for (int x = 0; x < 8; x++) {
            float t = accv[r][x];
            t += __shfl_xor(t, 16, WAVE); t += __shfl_xor(t, 32, WAVE);
            accv[r][x] = t;
        }
    float *part = Hs;   // [4 wavefronts][G][DH]
    if (g4 == 0) {
#pragma unroll
        for (int r = 0; r < G; r++)
#pragma unroll
            for (int x = 0; x < 8; x++) part[(w * G + r) * DH + 8 * r16 + x] = accv[r][x];
    }
    __syncthreads();
    for (int o = tid; o < G * DH; o += 256) {
        const int r = o / DH, c = o - r * DH;
        float num = part[(0 * G + r) * DH + c] + part[(1 * G + r) * DH + c] + part[(2 * G + r) * DH + c] + part[(3 * G + r) * DH + c];
        float den = psum_s[r];
        if (steady) {
            const float el = elin_s[r];
            num = fmaf(el, fmaf(dotqf[r], vf[c], lin[r][c]), num);
            den = fmaf(el, denq[r] + dotqf[r], den);
        }
        stf(a.out, ((size_t)b * a.Hq + (size_t)h * G + r) * DH + c, num / den);
    }
    if (tid == 0) a.st.n_tokens[si] = tok + 1;
}

}  // namespace fast
}  // namespace lola

// Chunk-parallel output kernel of the prefill for the 8B head shape (bf16 storage) on gfx950.
//
// One workgroup (four wavefronts) per (sequence, query head, chunk); every wavefront owns 16 of the
// chunk's 64 queries.  All GEMMs are computed transposed (queries are MFMA columns), so that
//   - the softmax statistics of a query live in the four lanes that share l % 16,
//   - the C layout of one GEMM is directly the B-operand layout of the next
//     (S^T -> P^T for the value GEMM, z^T -> phi(q)^T for the linear read-out),
// using the contraction-index permutation kappa(ks, e, grp) = 32 ks + 16 (e / 4) + 4 grp + e % 4.
//
// Per workgroup (paper Sec. 3, y_t equation with the chunk sharing one state, "Chunkwise Inference"):
//   1. phi(q) for the 64 queries: z^T = W_q Q^T on MFMA, fp32 softmax halves; phi(q)^T s.
//   2. linear part lin^T = H^T phi(q)^T with the chunk's snapshot of H^T, which the scan kernel
//      leaves as bf16 high + low parts in operand order (three MFMAs per product).
//   3. keys in blocks of 128: positions [0, lambda) sparse cache (gathered by virtual row),
//      [lambda, lambda + 64) the 64 rows before the chunk, [lambda + 64, lambda + 128) the chunk
//      itself (causal).  Per block: K and V^T staged in LDS, S^T = K Q^T, running max (started at 0:
//      the linear terms carry weight exp(-m)), P^T as bf16 high + low parts, out^T += V^T P^T.
//   4. y = (out + exp(-m) lin) / (sum p + exp(-m) phi(q)^T s).
#pragma once
#include "decode_mfma.h"
#include "generic_kernels.h"

namespace lola {
namespace fast {

// position of feature / key index x (0..127) inside a 128-wide operand row: 16-byte chunk and element
__device__ __forceinline__ int perm_chunk(int x) { return ((x >> 5) << 2) | ((x >> 2) & 3); }
__device__ __forceinline__ int perm_elem(int x) { return (((x >> 4) & 1) << 2) | (x & 3); }

template <int LAM, typename TO>
__global__ __launch_bounds__(256, 2) void attend_fast_kernel(generic::PrefillArgs<bf16_t> a) {
    constexpr int DH = 128, M = 64, D = 128, C = 64, ETA = 64, G = 4;
    constexpr int P = LAM + ETA;                    // rows of the virtual prefix
    constexpr int NKEYS = LAM + ETA + C;            // key positions
    constexpr int NB = (NKEYS + 127) / 128;         // key blocks
    __shared__ __attribute__((aligned(16))) uint16_t L[2 * DH * D];   // 64 KB: H^T high/low parts, then K block + V^T block
    __shared__ __attribute__((aligned(16))) float s_l[D];
    __shared__ int G_l[LAM > 0 ? LAM : 1];

    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, r16 = lane & 15, g4 = lane >> 4;
    const int jj = blockIdx.x, j = a.j0 + jj, hq = blockIdx.y, b = blockIdx.z;
    const int h = hq / G, si = b * a.dm.Hkv + h;
    const int64_t a0 = a.st.n_tokens[si];
    const int Tn = a.T_tokens;
    const int cl = min(C, Tn - j * C);              // queries in this chunk
    const int64_t aj = a0 + (int64_t)j * C;         // token index of the chunk's first query
    const size_t sj = (size_t)si * a.S + jj;
    const uint16_t *Hsnap = reinterpret_cast<const uint16_t *>(a.snapH) + sj * (2 * DH * D);
    const float *ssnap = a.snapS + sj * D;
    const int32_t *Gsnap = a.snapG + sj * LAM;
    const bf16_t *pK = a.prefK + (size_t)si * P * DH, *pV = a.prefV + (size_t)si * P * DH;
    const bf16_t *kc = a.k + (size_t)si * Tn * DH, *vc = a.v + (size_t)si * Tn * DH;
    const bf16_t *qh = a.q + (((size_t)b * a.dm.Hq + hq) * Tn + (size_t)j * C) * DH;
    TO *oh = (TO *)a.out + (((size_t)b * a.dm.Hq + hq) * Tn + (size_t)j * C) * DH;
    const bf16_t *Wq = a.Wq + (size_t)hq * M * DH;   // [M][DH]
    const int vrow_c = P + j * C;                     // virtual row of the chunk's first token
    const float scale2 = a.dm.scale * LOG2E;          // logits are kept in units of log2(e)

    // ---- loads: this wavefront's queries as MFMA B operand (column = query, k = input index); rows past the chunk's
    // end are read from row 0 (their results are never stored)
    const int qi = 16 * w + r16;
    bf16x8 BQ[4];
#pragma unroll
    for (int ks = 0; ks < 4; ks++) BQ[ks] = ld_bf16x8(qh + (size_t)(qi < cl ? qi : 0) * DH + 32 * ks + 8 * g4);
    // H^T snapshot -> LDS, 16-byte chunks XOR-swizzled by the row so that operand reads are conflict free
    if (tid < D / 4) reinterpret_cast<float4 *>(s_l)[tid] = reinterpret_cast<const float4 *>(ssnap)[tid];
    for (int x = tid; x < LAM; x += 256) G_l[x] = Gsnap[x];
#pragma unroll
    for (int p4 = 0; p4 < 4; p4++) {
        uint4 hv[4];
#pragma unroll
        for (int it = 0; it < 4; it++) hv[it] = reinterpret_cast<const uint4 *>(Hsnap)[tid + 256 * (4 * p4 + it)];
#pragma unroll
        for (int it = 0; it < 4; it++) {
            const int o = tid + 256 * (4 * p4 + it), part = o >> 11, rem = o & 2047, c = rem >> 4, ch = rem & 15;
            *reinterpret_cast<uint4 *>(&L[part * DH * D + c * D + ((ch ^ (c & 15)) << 3)]) = hv[it];
        }
    }
    // ---- phi(q): z^T = W_q Q^T (A = W_q rows from global, B = queries)
    float pp[16], pn[16];
    {
        f32x4 zt[4];
#pragma unroll
        for (int mt = 0; mt < 4; mt++) {
            zt[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ks++)
                zt[mt] = mfma16(ld_bf16x8(Wq + (size_t)(16 * mt + r16) * DH + 32 * ks + 8 * g4), BQ[ks], zt[mt]);
        }
        phi_from_z(zt, a.dm.phi_kind, pp, pn);
    }
    __syncthreads();
    float lden = 0.f;   // phi(q)^T s
#pragma unroll
    for (int mt = 0; mt < 4; mt++) {
        const float4 sp4 = *reinterpret_cast<const float4 *>(&s_l[16 * mt + 4 * g4]);
        const float4 sn4 = *reinterpret_cast<const float4 *>(&s_l[M + 16 * mt + 4 * g4]);
        lden = fmaf(pp[4 * mt], sp4.x, lden); lden = fmaf(pp[4 * mt + 1], sp4.y, lden);
        lden = fmaf(pp[4 * mt + 2], sp4.z, lden); lden = fmaf(pp[4 * mt + 3], sp4.w, lden);
        lden = fmaf(pn[4 * mt], sn4.x, lden); lden = fmaf(pn[4 * mt + 1], sn4.y, lden);
        lden = fmaf(pn[4 * mt + 2], sn4.z, lden); lden = fmaf(pn[4 * mt + 3], sn4.w, lden);
    }
    lden = grp_sum(lden);
    // ---- linear part: lin^T[c][q] = sum_f H^T[c][f] phi(q)[f]
    f32x4 lin[8];
    {
        bf16x8 Bh[4], Bl[4];
        split8(&pp[0], Bh[0], Bl[0]); split8(&pp[8], Bh[1], Bl[1]);
        split8(&pn[0], Bh[2], Bl[2]); split8(&pn[8], Bh[3], Bl[3]);
#pragma unroll
        for (int mt = 0; mt < 8; mt++) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f}, acc2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ks++) {
                const int addr = (16 * mt + r16) * D + (((4 * ks + g4) ^ r16) << 3);
                const bf16x8 Ahi = as_bf16x8(*reinterpret_cast<const uint4 *>(&L[addr]));
                const bf16x8 Alo = as_bf16x8(*reinterpret_cast<const uint4 *>(&L[DH * D + addr]));
                acc = mfma16(Ahi, Bh[ks], acc);
                acc2 = mfma16(Ahi, Bl[ks], acc2);
                acc2 = mfma16(Alo, Bh[ks], acc2);
            }
            lin[mt] = acc + acc2;
        }
    }

    // ---- softmax part over key blocks of 128 positions
    uint16_t *Kl = L, *Vt = L + DH * 128;   // [key][input chunk ^ key%16] and [c][key chunk ^ swz(c)], 32 KB each
    f32x4 out[8];
#pragma unroll
    for (int mt = 0; mt < 8; mt++) out[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float mrun = 0.f, lsum = 0.f;   // running max (units of log2 e) and running sum of weights
    const int64_t tq = aj + qi;     // token index of this lane's query
#pragma unroll 1
    for (int blk = 0; blk < NB; blk++) {
        // position -> source row (or none).  Thread handles 8 (key, 16-byte chunk) pairs of the block
        // (named scalars: an array held across the barrier would be sent through scratch memory).
#define LOLA_REP8(X) X(0) X(1) X(2) X(3) X(4) X(5) X(6) X(7)
#define LOLA_KVLOAD(it) uint4 kreg##it = make_uint4(0, 0, 0, 0), vreg##it = make_uint4(0, 0, 0, 0); { \
            const int o = tid + 256 * it, kk = o >> 4, ch = o & 15, pos = 128 * blk + kk; \
            int vr = -1; \
            if (pos < LAM) vr = G_l[pos]; \
            else if (pos < NKEYS) { vr = vrow_c - ETA + (pos - LAM); if (aj - ETA + (pos - LAM) < 0 || (pos - LAM - ETA) >= cl) vr = -1; } \
            if (vr >= 0) { \
                const bf16_t *kr = vr < P ? pK + (size_t)vr * DH : kc + (size_t)(vr - P) * DH; \
                const bf16_t *vrp = vr < P ? pV + (size_t)vr * DH : vc + (size_t)(vr - P) * DH; \
                kreg##it = reinterpret_cast<const uint4 *>(kr)[ch]; \
                vreg##it = reinterpret_cast<const uint4 *>(vrp)[ch]; \
            } }
#define LOLA_KVSTORE(it) { \
            const int o = tid + 256 * it, kk = o >> 4, ch = o & 15; \
            *reinterpret_cast<uint4 *>(&Kl[kk * DH + ((ch ^ (kk & 15)) << 3)]) = kreg##it; \
            const uint32_t u[4] = {vreg##it.x, vreg##it.y, vreg##it.z, vreg##it.w}; \
            const int kchunk = perm_chunk(kk), kel = perm_elem(kk); \
            _Pragma("unroll") for (int x = 0; x < 8; x++) { \
                const int c = 8 * ch + x; \
                Vt[c * 128 + ((kchunk ^ ((c ^ (c >> 3)) & 15)) << 3) + kel] = (uint16_t)((x & 1) ? (u[x >> 1] >> 16) : (u[x >> 1] & 0xFFFFu)); \
            } }
        LOLA_REP8(LOLA_KVLOAD)
        __syncthreads();   // previous users of L (H^T, or the previous block) are done
        LOLA_REP8(LOLA_KVSTORE)
#undef LOLA_KVLOAD
#undef LOLA_KVSTORE
#undef LOLA_REP8
        __syncthreads();
        // S^T = K Q^T for the 8 key tiles of the block; lane (column = query r16, group g4) holds keys 16 mt + 4 g4 + i
        f32x4 sc[8];
        float bmax = mrun;
#pragma unroll
        for (int mt = 0; mt < 8; mt++) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ks++)
                acc = mfma16(as_bf16x8(*reinterpret_cast<const uint4 *>(&Kl[(16 * mt + r16) * DH + (((4 * ks + g4) ^ r16) << 3)])), BQ[ks], acc);
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const int pos = 128 * blk + 16 * mt + 4 * g4 + i;
                bool ok;
                if (pos < LAM) ok = G_l[pos] >= 0;
                else if (pos < LAM + ETA) ok = aj - ETA + (pos - LAM) >= 0;
                else ok = pos < NKEYS && (aj + (pos - LAM - ETA)) <= tq;
                acc[i] = ok ? acc[i] * scale2 : -INFINITY;
                bmax = fmaxf(bmax, acc[i]);
            }
            sc[mt] = acc;
        }
        bmax = grp_max(bmax);
        const float resc = fexp2(mrun - bmax);
        mrun = bmax;
        lsum *= resc;
#pragma unroll
        for (int mt = 0; mt < 8; mt++) out[mt] *= resc;
        // weights and out^T += V^T P^T, 32 keys per k-step (key tiles 2s, 2s+1)
#pragma unroll
        for (int s = 0; s < 4; s++) {
            float pw[8];
#pragma unroll
            for (int e = 0; e < 8; e++) { pw[e] = fexp2(sc[2 * s + (e >> 2)][e & 3] - mrun); lsum += pw[e]; }
            bf16x8 Ph, Pl;
            split8(pw, Ph, Pl);
#pragma unroll
            for (int mt = 0; mt < 8; mt++) {
                const int c = 16 * mt + r16;
                const bf16x8 Av = as_bf16x8(*reinterpret_cast<const uint4 *>(&Vt[c * 128 + (((4 * s + g4) ^ ((c ^ (c >> 3)) & 15)) << 3)]));
                out[mt] = mfma16(Av, Ph, out[mt]);
                out[mt] = mfma16(Av, Pl, out[mt]);
            }
        }
    }
    lsum = grp_sum(lsum);
    // ---- y = (out + exp(-m) lin) / (sum p + exp(-m) phi(q)^T s); lane holds columns c = 16 mt + 4 g4 + 0..3 of query qi
    if (qi < cl) {
        const float el = fexp2(-mrun);
        const float inv = 1.0f / fmaf(el, lden, lsum);
#pragma unroll
        for (int mt = 0; mt < 8; mt++) {
            TO *dst = oh + (size_t)qi * DH + 16 * mt + 4 * g4;
#pragma unroll
            for (int i = 0; i < 4; i++) stf(dst, i, fmaf(el, lin[mt][i], out[mt][i]) * inv);
        }
    }
}

}  // namespace fast
}  // namespace lola

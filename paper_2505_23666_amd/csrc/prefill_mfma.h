// MFMA kernels of the prefill (and, further down, of the generation step at the shapes the fused kernel of
// decode_mfma.h does not cover) for gfx950, bf16 storage.  In file order: attend_fast_kernel / attend_wide_kernel
// (chunk-parallel outputs, compile-time / run-time window and budget), phi_k_kernel, scan_fast_kernel (state evolution,
// compile-time shapes), phi_wide_kernel, scan_wide_kernel (run-time shapes; also with given scores and without a
// cache), step_out_wide_kernel, step_update_wide_kernel (generation step), band_score_wide_kernel (query-dependent
// scores of a call), scan_nocache_kernel (no sparse cache, window 64).
//
// The chunk-parallel output kernel for the 8B head shape:
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
//      itself (causal).  Per block: K and V staged in LDS (both row-major), S^T = K Q^T, running max (started at 0:
//      the linear terms carry weight exp(-m)), P^T as bf16 high + low parts, out^T += V^T P^T with V^T taken
//      through the transposing LDS read.
//   4. y = (out + exp(-m) lin) / (sum p + exp(-m) phi(q)^T s).
#pragma once
#include "decode_mfma.h"
#include "generic_kernels.h"

namespace lola {
namespace fast {

template <int PR> __device__ __forceinline__ int vswz2(int row);   // (piece swizzle of row-major value tiles, defined with the other swizzles below)

template <int LAM, int DH, typename TO>
__global__ __launch_bounds__(256, 2) void attend_fast_kernel(generic::PrefillArgs<bf16_t> a) {
    constexpr int M = 64, D = 128, C = 64, ETA = 64, KS = DH / 32, PR = DH / 8, NCT = DH / 16;
    static_assert(DH == 64 || DH == 128, "head_dim");
    constexpr int P = LAM + ETA;                    // rows of the virtual prefix
    constexpr int NKEYS = LAM + ETA + C;            // key positions
    constexpr int NB = (NKEYS + 127) / 128;         // key blocks
    __shared__ __attribute__((aligned(16))) uint16_t L[2 * DH * D];   // 64 KB: H^T high/low parts, then K block + V block
    __shared__ __attribute__((aligned(16))) float s_l[D];
    __shared__ int G_l[LAM > 0 ? LAM : 1];
    __shared__ int gneg_l[4];   // per wavefront: it saw an empty cache slot

    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, r16 = lane & 15, g4 = lane >> 4;
    const int j = a.j0 + blockIdx.x, jj = j - a.jb, hq = blockIdx.y, b = blockIdx.z;
    const int h = hq / a.dm.g, si = b * a.dm.Hkv + h;
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
    bf16x8 BQ[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ks++) BQ[ks] = ld_bf16x8(qh + (size_t)(qi < cl ? qi : 0) * DH + 32 * ks + 8 * g4);
    if (tid < D / 4) reinterpret_cast<float4 *>(s_l)[tid] = reinterpret_cast<const float4 *>(ssnap)[tid];
    bool gneg = false;
    for (int x = tid; x < LAM; x += 256) { const int gr = Gsnap[x]; G_l[x] = gr; gneg |= gr < 0; }
    if (lane == 0) gneg_l[w] = 0;
    if (gneg) gneg_l[w] = 1;   // (after the store of 0 in program order; lanes of one wavefront, same value)
    lds_barrier();
    // Key blocks that lie in the cache and the window need no masks when every slot is in use, the window is full and the
    // queries may read the cache: the per-element tests (an LDS read and three compares each) are skipped there.
    const bool nomask_ok = !(gneg_l[0] | gneg_l[1] | gneg_l[2] | gneg_l[3]) && !(a.dm.hide & 2) && aj >= ETA;

    // ---- softmax part over key blocks of 128 positions
    uint16_t *Kl = L, *Vr = L + DH * 128;   // [key][input piece ^ key % pieces] and [key][piece ^ vswz2(key)] (read transposed)
    f32x4 out[NCT];
#pragma unroll
    for (int mt = 0; mt < NCT; mt++) out[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float mrun = 0.f, lsum = 0.f;   // running max (units of log2 e) and running sum of weights
    const int64_t tq = aj + qi;     // token index of this lane's query
#pragma unroll 1
    for (int blk = 0; blk < NB; blk++) {
        // position -> source row (or none).  A thread handles PR / 4 items of the block, each one 16-byte piece of two
        // neighbouring keys; the values stay row-major (the value GEMM reads them through the transposing LDS read)
        // (named scalars: an array held across the barrier would be sent through scratch memory).
#define LOLA_REP8(X) X(0) X(1) X(2) X(3)   // items beyond 64 * PR / 256 compile to nothing
#define LOLA_KVROW(pos, vr) { vr = -1; \
            if (pos < LAM) vr = G_l[pos]; \
            else if (pos < NKEYS) { vr = vrow_c - ETA + (pos - LAM); if (aj - ETA + (pos - LAM) < 0 || (pos - LAM - ETA) >= cl) vr = -1; } }
#define LOLA_KVLOAD(it) uint4 kreg##it = make_uint4(0, 0, 0, 0), vreg##it = make_uint4(0, 0, 0, 0), \
                              kreh##it = make_uint4(0, 0, 0, 0), vreh##it = make_uint4(0, 0, 0, 0); if (it < PR / 4) { \
            const int o = tid + 256 * it, kk = 2 * (o / PR), ch = o % PR; \
            int vr0, vr1; \
            LOLA_KVROW((128 * blk + kk), vr0) LOLA_KVROW((128 * blk + kk + 1), vr1) \
            if (vr0 >= 0) { \
                kreg##it = reinterpret_cast<const uint4 *>(vr0 < P ? pK + (size_t)vr0 * DH : kc + (size_t)(vr0 - P) * DH)[ch]; \
                vreg##it = reinterpret_cast<const uint4 *>(vr0 < P ? pV + (size_t)vr0 * DH : vc + (size_t)(vr0 - P) * DH)[ch]; \
            } \
            if (vr1 >= 0) { \
                kreh##it = reinterpret_cast<const uint4 *>(vr1 < P ? pK + (size_t)vr1 * DH : kc + (size_t)(vr1 - P) * DH)[ch]; \
                vreh##it = reinterpret_cast<const uint4 *>(vr1 < P ? pV + (size_t)vr1 * DH : vc + (size_t)(vr1 - P) * DH)[ch]; \
            } }
#define LOLA_KVSTORE(it) if (it < PR / 4) { \
            const int o = tid + 256 * it, kk = 2 * (o / PR), ch = o % PR; \
            *reinterpret_cast<uint4 *>(&Kl[kk * DH + ((ch ^ (kk & (PR - 1))) << 3)]) = kreg##it; \
            *reinterpret_cast<uint4 *>(&Kl[(kk + 1) * DH + ((ch ^ ((kk + 1) & (PR - 1))) << 3)]) = kreh##it; \
            *reinterpret_cast<uint4 *>(&Vr[kk * DH + ((ch ^ vswz2<PR>(kk)) << 3)]) = vreg##it; \
            *reinterpret_cast<uint4 *>(&Vr[(kk + 1) * DH + ((ch ^ vswz2<PR>(kk + 1)) << 3)]) = vreh##it; }
        LOLA_REP8(LOLA_KVLOAD)
        lds_barrier();   // previous users of L (H^T, or the previous block) are done
        LOLA_REP8(LOLA_KVSTORE)
#undef LOLA_KVLOAD
#undef LOLA_KVSTORE
#undef LOLA_KVROW
#undef LOLA_REP8
        lds_barrier();
        // S^T = K Q^T for the 8 key tiles of the block; lane (column = query r16, group g4) holds keys 16 mt + 4 g4 + i
        f32x4 sc[8];
        float bmax = mrun;
#pragma unroll
        for (int mt = 0; mt < 8; mt++) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ks++)
                acc = mfma16(as_bf16x8(*reinterpret_cast<const uint4 *>(&Kl[(16 * mt + r16) * DH + (((4 * ks + g4) ^ (r16 & (PR - 1))) << 3)])), BQ[ks], acc);
            if (nomask_ok && 128 * (blk + 1) <= LAM + ETA) {
#pragma unroll
                for (int i = 0; i < 4; i++) { acc[i] *= scale2; bmax = fmaxf(bmax, acc[i]); }
            } else {
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const int pos = 128 * blk + 16 * mt + 4 * g4 + i;
                    bool ok;
                    if (pos < LAM) ok = G_l[pos] >= 0 && !(a.dm.hide & 2);
                    else if (pos < LAM + ETA) ok = aj - ETA + (pos - LAM) >= 0;
                    else ok = pos < NKEYS && (aj + (pos - LAM - ETA)) <= tq;
                    acc[i] = ok ? acc[i] * scale2 : -INFINITY;
                    bmax = fmaxf(bmax, acc[i]);
                }
            }
            sc[mt] = acc;
        }
        bmax = grp_max(bmax);
        const float resc = fexp2(mrun - bmax);
        mrun = bmax;
        lsum *= resc;
#pragma unroll
        for (int mt = 0; mt < NCT; mt++) out[mt] *= resc;
        // weights and out^T += V^T P^T, 32 keys per k-step (key tiles 2s, 2s+1)
#pragma unroll
        for (int s = 0; s < 4; s++) {
            float pw[8];
#pragma unroll
            for (int e = 0; e < 8; e++) { pw[e] = fexp2(sc[2 * s + (e >> 2)][e & 3] - mrun); lsum += pw[e]; }
            bf16x8 Ph, Pl;
            split8(pw, Ph, Pl);
            // A = V^T of keys 32 s ..: lane (column r16 of tile mt, group g4) holds keys 4 g4 + 0..3 and 16 + 4 g4 + 0..3 (the
            // order of pw) of its column, through the transposing read of the row-major block
            const int t0 = 4 * g4 + (r16 >> 2);
            const uint16_t *vb = &Vr[(32 * s + t0) * DH + 4 * (r16 & 1)];
#pragma unroll
            for (int mt = 0; mt < NCT; mt++) {
                const int pc = ((2 * mt + ((r16 & 3) >> 1)) ^ vswz2<PR>(t0)) << 3;
                const bf16x4 b0 = tr_read(vb + pc), b1 = tr_read(vb + 16 * DH + pc);
                const bf16x8 Av = __builtin_shufflevector(b0, b1, 0, 1, 2, 3, 4, 5, 6, 7);
                out[mt] = mfma16(Av, Ph, out[mt]);
                out[mt] = mfma16(Av, Pl, out[mt]);
            }
        }
    }
    lsum = grp_sum(lsum);

    // ---- linear part, after the softmax part so that its operands do not occupy registers during the key blocks:
    // H^T snapshot -> LDS (16-byte pieces XOR-swizzled by the row so that operand reads are conflict free), phi(q),
    // then per value tile lin^T[c][q] = sum_f H^T[c][f] phi(q)[f] and the output
    //   y = (out + exp(-m) lin) / (sum p + exp(-m) phi(q)^T s);  the lane holds columns c = 16 mt + 4 g4 + 0..3 of query qi
    lds_barrier();   // the last key block has been consumed
#pragma unroll
    for (int p4 = 0; p4 < DH / 32; p4++) {
        uint4 hv[4];
#pragma unroll
        for (int it = 0; it < 4; it++) hv[it] = reinterpret_cast<const uint4 *>(Hsnap)[tid + 256 * (4 * p4 + it)];
#pragma unroll
        for (int it = 0; it < 4; it++) {
            // snapshot order: [part][row tile of 16][k-step][lane = 16 (piece % 4) + row % 16]
            const int o = tid + 256 * (4 * p4 + it), part = o / (DH * 16), op = o % (DH * 16);
            const int c = 16 * (op >> 8) + (o & 15), ch = 4 * ((o >> 6) & 3) + ((o >> 4) & 3);
            *reinterpret_cast<uint4 *>(&L[part * DH * D + c * D + ((ch ^ (c & 15)) << 3)]) = hv[it];
        }
    }
    // phi(q): z^T = W_q Q^T (A = W_q rows from global, B = queries)
    float pp[16], pn[16];
    {
        f32x4 zt[4];
#pragma unroll
        for (int mt = 0; mt < 4; mt++) {
            zt[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ks++)
                zt[mt] = mfma16(ld_bf16x8(Wq + (size_t)(16 * mt + r16) * DH + 32 * ks + 8 * g4), BQ[ks], zt[mt]);
        }
        phi_from_z(zt, a.dm.phi_kind, pp, pn);
    }
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
    bf16x8 Bh[4], Bl[4];
    split8(&pp[0], Bh[0], Bl[0]); split8(&pp[8], Bh[1], Bl[1]);
    split8(&pn[0], Bh[2], Bl[2]); split8(&pn[8], Bh[3], Bl[3]);
    const float el = (a.dm.hide & 1) ? 0.f : fexp2(-mrun);   // restricted query: no hidden-state terms
    const float inv = frcp(fmaf(el, lden, lsum));
    lds_barrier();   // H^T is in LDS
#pragma unroll
    for (int mt = 0; mt < NCT; mt++) {
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
        const f32x4 lin = acc + acc2;
        if (qi < cl) {
            TO *dst = oh + (size_t)qi * DH + 16 * mt + 4 * g4;
#pragma unroll
            for (int i = 0; i < 4; i++) stf(dst, i, fmaf(el, lin[i], out[mt][i]) * inv);
        }
    }
}


// phi of 16 vectors from their NT tiles of projections in the C layout of the projection GEMM (lane (column r16, group
// g4) holds z[16 mt + 4 g4 + i] in zt[mt][i]): the lane's 4 NT positive-half and 4 NT negative-half features, index
// 4 mt + i (Sec. 2.3 eq. feature_map; the softmax kind normalises each half over all 16 NT projections).
template <int NT>
__device__ __forceinline__ void phi_from_z_tiles(const f32x4 (&zt)[NT], int phi_kind, float (&pp)[4 * NT], float (&pn)[4 * NT]) {
    if (phi_kind == 1) {
#pragma unroll
        for (int x = 0; x < 4 * NT; x++) { const float zs = zt[x >> 2][x & 3] * LOG2E; pp[x] = fexp2(zs); pn[x] = fexp2(-zs); }
        return;
    }
    float zmax = zt[0][0], zmin = zt[0][0];
#pragma unroll
    for (int x = 1; x < 4 * NT; x++) { zmax = fmaxf(zmax, zt[x >> 2][x & 3]); zmin = fminf(zmin, zt[x >> 2][x & 3]); }
    zmax = grp_max(zmax); zmin = grp_min(zmin);
    const float cp = -zmax * LOG2E, cn = zmin * LOG2E;
    float sp = 0.f, sn = 0.f;
#pragma unroll
    for (int x = 0; x < 4 * NT; x++) {
        const float zz = zt[x >> 2][x & 3];
        pp[x] = fexp2(fmaf(zz, LOG2E, cp)); pn[x] = fexp2(fmaf(zz, -LOG2E, cn));
        sp += pp[x]; sn += pn[x];
    }
    sp = grp_sum(sp); sn = grp_sum(sn);
    const float ip = frcp(sp), in_ = frcp(sn);
#pragma unroll
    for (int x = 0; x < 4 * NT; x++) { pp[x] *= ip; pn[x] *= in_; }
}

// The output kernel for any window and sparse budget (read from the arguments) and for 128 or 256 features: the
// paper's own models use twice the head dimension as feature dimension and windows / budgets of 128 .. 1024 in the
// long-context runs (Sec. 4).  Same computation and layouts as attend_fast_kernel (chunks of 64 queries, key blocks of
// 128 positions: cache slots, window, the chunk itself), with run-time trip counts; the H^T snapshot passes through LDS
// 128 features at a time.  The snapshot's pieces are ordered [part][row tile of 16][k-step of 32 features][lane].
template <int DH, int DF, typename TO>
__global__ __launch_bounds__(256, 2) void attend_wide_kernel(generic::PrefillArgs<bf16_t> a) {
    constexpr int M = DF / 2, C = 64, KS = DH / 32, PR = DH / 8, NCT = DH / 16, NZT = M / 16, KSD = DF / 32, NFH = DF / 128;
    constexpr int MAXLAM = 1024;
    static_assert((DH == 64 || DH == 128) && (DF == 128 || DF == 256), "shape");
    __shared__ __attribute__((aligned(16))) uint16_t L[2 * DH * 128];   // 64 KB: K block + V block, then half of H^T (high/low parts)
    __shared__ __attribute__((aligned(16))) float s_l[DF];
    __shared__ int G_l[MAXLAM];
    __shared__ int gneg_l[4];   // per wavefront: it saw an empty cache slot

    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, r16 = lane & 15, g4 = lane >> 4;
    const int LAM = a.dm.lam, ETA = a.dm.eta;
    const int P = LAM + ETA, NKEYS = LAM + ETA + C, NB = (NKEYS + 127) / 128;
    const int j = a.j0 + blockIdx.x, jj = j - a.jb, hq = blockIdx.y, b = blockIdx.z;
    const int h = hq / a.dm.g, si = b * a.dm.Hkv + h;
    const int64_t a0 = a.st.n_tokens[si];
    const int Tn = a.T_tokens;
    const int cl = min(C, Tn - j * C);              // queries in this chunk
    const int64_t aj = a0 + (int64_t)j * C;         // token index of the chunk's first query
    const size_t sj = (size_t)si * a.S + jj;
    const uint16_t *Hsnap = reinterpret_cast<const uint16_t *>(a.snapH) + sj * (2 * DH * DF);
    const float *ssnap = a.snapS + sj * DF;
    const int32_t *Gsnap = a.snapG + sj * LAM;
    const bf16_t *pK = a.prefK + (size_t)si * P * DH, *pV = a.prefV + (size_t)si * P * DH;
    const bf16_t *kc = a.k + (size_t)si * Tn * DH, *vc = a.v + (size_t)si * Tn * DH;
    const bf16_t *qh = a.q + (((size_t)b * a.dm.Hq + hq) * Tn + (size_t)j * C) * DH;
    TO *oh = (TO *)a.out + (((size_t)b * a.dm.Hq + hq) * Tn + (size_t)j * C) * DH;
    const bf16_t *Wq = a.Wq + (size_t)hq * M * DH;   // [M][DH]
    const int vrow_c = P + j * C;                     // virtual row of the chunk's first token
    const float scale2 = a.dm.scale * LOG2E;          // logits are kept in units of log2(e)

    const int qi = 16 * w + r16;
    bf16x8 BQ[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ks++) BQ[ks] = ld_bf16x8(qh + (size_t)(qi < cl ? qi : 0) * DH + 32 * ks + 8 * g4);
    for (int x = tid; x < DF / 4; x += 256) reinterpret_cast<float4 *>(s_l)[x] = reinterpret_cast<const float4 *>(ssnap)[x];
    bool gneg = false;
    for (int x = tid; x < LAM; x += 256) { const int gr = Gsnap[x]; G_l[x] = gr; gneg |= gr < 0; }
    if (lane == 0) gneg_l[w] = 0;
    if (gneg) gneg_l[w] = 1;   // (after the store of 0 in program order; lanes of one wavefront, same value)
    __syncthreads();
    // Key blocks that lie in the cache and the window need no masks when every slot is in use, the window is full and the
    // queries may read the cache: the per-element tests (an LDS read and three compares each) are skipped there.
    const bool nomask_ok = !(gneg_l[0] | gneg_l[1] | gneg_l[2] | gneg_l[3]) && !(a.dm.hide & 2) && aj >= ETA;

    // position -> source row of the key / value (or -1)
    auto kv_row = [&](int pos) -> int {
        if (pos < LAM) return G_l[pos];
        if (pos >= NKEYS) return -1;
        const int wpos = pos - LAM;                       // 0 .. ETA + C - 1: window, then the chunk
        if (aj - ETA + wpos < 0 || wpos - ETA >= cl) return -1;
        return vrow_c - ETA + wpos;
    };

    // ---- softmax part over key blocks of 128 positions
    uint16_t *Kl = L, *Vr = L + DH * 128;   // [key][input piece ^ key % pieces] and [key][piece ^ vswz2(key)] (read transposed)
    f32x4 out[NCT];
#pragma unroll
    for (int mt = 0; mt < NCT; mt++) out[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float mrun = 0.f, lsum = 0.f;   // running max (units of log2 e) and running sum of weights
    const int64_t tq = aj + qi;     // token index of this lane's query
#pragma unroll 1
    for (int blk = 0; blk < NB; blk++) {
        // a thread stages PR / 4 items of the block, each one 16-byte piece of two neighbouring keys; the values stay
        // row-major (the value GEMM reads them through the transposing LDS read)
        constexpr int NIT = PR / 4;
        uint4 kreg[NIT], kreh[NIT], vreg[NIT], vreh[NIT];
#pragma unroll
        for (int it = 0; it < NIT; it++) {
            const int o = tid + 256 * it, kk = 2 * (o / PR), ch = o % PR;
            const int vr0 = kv_row(128 * blk + kk), vr1 = kv_row(128 * blk + kk + 1);
            kreg[it] = kreh[it] = vreg[it] = vreh[it] = make_uint4(0, 0, 0, 0);
            if (vr0 >= 0) {
                kreg[it] = reinterpret_cast<const uint4 *>(vr0 < P ? pK + (size_t)vr0 * DH : kc + (size_t)(vr0 - P) * DH)[ch];
                vreg[it] = reinterpret_cast<const uint4 *>(vr0 < P ? pV + (size_t)vr0 * DH : vc + (size_t)(vr0 - P) * DH)[ch];
            }
            if (vr1 >= 0) {
                kreh[it] = reinterpret_cast<const uint4 *>(vr1 < P ? pK + (size_t)vr1 * DH : kc + (size_t)(vr1 - P) * DH)[ch];
                vreh[it] = reinterpret_cast<const uint4 *>(vr1 < P ? pV + (size_t)vr1 * DH : vc + (size_t)(vr1 - P) * DH)[ch];
            }
        }
        __syncthreads();   // previous users of L (the previous block) are done
#pragma unroll
        for (int it = 0; it < NIT; it++) {
            const int o = tid + 256 * it, kk = 2 * (o / PR), ch = o % PR;
            *reinterpret_cast<uint4 *>(&Kl[kk * DH + ((ch ^ (kk & (PR - 1))) << 3)]) = kreg[it];
            *reinterpret_cast<uint4 *>(&Kl[(kk + 1) * DH + ((ch ^ ((kk + 1) & (PR - 1))) << 3)]) = kreh[it];
            *reinterpret_cast<uint4 *>(&Vr[kk * DH + ((ch ^ vswz2<PR>(kk)) << 3)]) = vreg[it];
            *reinterpret_cast<uint4 *>(&Vr[(kk + 1) * DH + ((ch ^ vswz2<PR>(kk + 1)) << 3)]) = vreh[it];
        }
        __syncthreads();
        // S^T = K Q^T for the 8 key tiles of the block; lane (column = query r16, group g4) holds keys 16 mt + 4 g4 + i
        f32x4 sc[8];
        float bmax = mrun;
#pragma unroll
        for (int mt = 0; mt < 8; mt++) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ks++)
                acc = mfma16(as_bf16x8(*reinterpret_cast<const uint4 *>(&Kl[(16 * mt + r16) * DH + (((4 * ks + g4) ^ (r16 & (PR - 1))) << 3)])), BQ[ks], acc);
            if (nomask_ok && 128 * (blk + 1) <= LAM + ETA) {
#pragma unroll
                for (int i = 0; i < 4; i++) { acc[i] *= scale2; bmax = fmaxf(bmax, acc[i]); }
            } else {
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const int pos = 128 * blk + 16 * mt + 4 * g4 + i;
                    bool ok;
                    if (pos < LAM) ok = G_l[pos] >= 0 && !(a.dm.hide & 2);
                    else if (pos < LAM + ETA) ok = aj - ETA + (pos - LAM) >= 0;
                    else ok = pos < NKEYS && (aj + (pos - LAM - ETA)) <= tq;
                    acc[i] = ok ? acc[i] * scale2 : -INFINITY;
                    bmax = fmaxf(bmax, acc[i]);
                }
            }
            sc[mt] = acc;
        }
        bmax = grp_max(bmax);
        const float resc = fexp2(mrun - bmax);
        mrun = bmax;
        lsum *= resc;
#pragma unroll
        for (int mt = 0; mt < NCT; mt++) out[mt] *= resc;
#pragma unroll
        for (int s = 0; s < 4; s++) {
            float pw[8];
#pragma unroll
            for (int e = 0; e < 8; e++) { pw[e] = fexp2(sc[2 * s + (e >> 2)][e & 3] - mrun); lsum += pw[e]; }
            bf16x8 Ph, Pl;
            split8(pw, Ph, Pl);
            // A = V^T of keys 32 s ..: lane (column r16 of tile mt, group g4) holds keys 4 g4 + 0..3 and 16 + 4 g4 + 0..3 (the
            // order of pw) of its column, through the transposing read of the row-major block
            const int t0 = 4 * g4 + (r16 >> 2);
            const uint16_t *vb = &Vr[(32 * s + t0) * DH + 4 * (r16 & 1)];
#pragma unroll
            for (int mt = 0; mt < NCT; mt++) {
                const int pc = ((2 * mt + ((r16 & 3) >> 1)) ^ vswz2<PR>(t0)) << 3;
                const bf16x4 b0 = tr_read(vb + pc), b1 = tr_read(vb + 16 * DH + pc);
                const bf16x8 Av = __builtin_shufflevector(b0, b1, 0, 1, 2, 3, 4, 5, 6, 7);
                out[mt] = mfma16(Av, Ph, out[mt]);
                out[mt] = mfma16(Av, Pl, out[mt]);
            }
        }
    }
    lsum = grp_sum(lsum);

    // ---- linear part: phi(q), phi(q)^T s, then lin^T = H^T phi(q)^T with the snapshot staged 128 features at a time
    float pp[4 * NZT], pn[4 * NZT];
    {
        f32x4 zt[NZT];
#pragma unroll
        for (int mt = 0; mt < NZT; mt++) {
            zt[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ks++)
                zt[mt] = mfma16(ld_bf16x8(Wq + (size_t)(16 * mt + r16) * DH + 32 * ks + 8 * g4), BQ[ks], zt[mt]);
        }
        phi_from_z_tiles<NZT>(zt, a.dm.phi_kind, pp, pn);
    }
    float lden = 0.f;   // phi(q)^T s
#pragma unroll
    for (int mt = 0; mt < NZT; mt++) {
        const float4 sp4 = *reinterpret_cast<const float4 *>(&s_l[16 * mt + 4 * g4]);
        const float4 sn4 = *reinterpret_cast<const float4 *>(&s_l[M + 16 * mt + 4 * g4]);
        lden = fmaf(pp[4 * mt], sp4.x, lden); lden = fmaf(pp[4 * mt + 1], sp4.y, lden);
        lden = fmaf(pp[4 * mt + 2], sp4.z, lden); lden = fmaf(pp[4 * mt + 3], sp4.w, lden);
        lden = fmaf(pn[4 * mt], sn4.x, lden); lden = fmaf(pn[4 * mt + 1], sn4.y, lden);
        lden = fmaf(pn[4 * mt + 2], sn4.z, lden); lden = fmaf(pn[4 * mt + 3], sn4.w, lden);
    }
    lden = grp_sum(lden);
    // B operands of the read-out: k-step ks covers features 32 ks ..: the first KSD / 2 k-steps the positive half
    bf16x8 Bh[KSD], Bl[KSD];
#pragma unroll
    for (int ks = 0; ks < KSD / 2; ks++) {
        split8(&pp[8 * ks], Bh[ks], Bl[ks]);
        split8(&pn[8 * ks], Bh[KSD / 2 + ks], Bl[KSD / 2 + ks]);
    }
    const float el = (a.dm.hide & 1) ? 0.f : fexp2(-mrun);   // restricted query: no hidden-state terms
    const float inv = frcp(fmaf(el, lden, lsum));
    f32x4 lin[NCT], lin2[NCT];
#pragma unroll
    for (int mt = 0; mt < NCT; mt++) { lin[mt] = (f32x4){0.f, 0.f, 0.f, 0.f}; lin2[mt] = (f32x4){0.f, 0.f, 0.f, 0.f}; }
#pragma unroll 1
    for (int fh = 0; fh < NFH; fh++) {
        __syncthreads();   // the last key block (or the previous half) has been consumed
        // snapshot order: [part][row tile of 16][k-step][lane = 16 (piece % 4) + row % 16]; this half: k-steps 4 fh .. 4 fh + 3
        for (int o = tid; o < 2 * DH * 16; o += 256) {
            const int part = o / (DH * 16), op = o % (DH * 16);
            const int ct = op >> 8, ksl = (op >> 6) & 3, ln = op & 63;
            const uint4 hv = reinterpret_cast<const uint4 *>(Hsnap)[(size_t)part * (DH * DF / 8) + (ct * KSD + 4 * fh + ksl) * 64 + ln];
            const int c = 16 * ct + (ln & 15), ch = 4 * ksl + (ln >> 4);
            *reinterpret_cast<uint4 *>(&L[part * DH * 128 + c * 128 + ((ch ^ (c & 15)) << 3)]) = hv;
        }
        __syncthreads();
#pragma unroll
        for (int mt = 0; mt < NCT; mt++) {
#pragma unroll
            for (int ks = 0; ks < 4; ks++) {
                const int addr = (16 * mt + r16) * 128 + (((4 * ks + g4) ^ r16) << 3);
                const bf16x8 Ahi = as_bf16x8(*reinterpret_cast<const uint4 *>(&L[addr]));
                const bf16x8 Alo = as_bf16x8(*reinterpret_cast<const uint4 *>(&L[DH * 128 + addr]));
                const bf16x8 bh = fh == 0 ? Bh[ks] : Bh[(KSD > 4 ? 4 : 0) + ks], bl = fh == 0 ? Bl[ks] : Bl[(KSD > 4 ? 4 : 0) + ks];
                lin[mt] = mfma16(Ahi, bh, lin[mt]);
                lin2[mt] = mfma16(Ahi, bl, lin2[mt]);
                lin2[mt] = mfma16(Alo, bh, lin2[mt]);
            }
        }
    }
    if (qi < cl) {
#pragma unroll
        for (int mt = 0; mt < NCT; mt++) {
            const f32x4 ln4 = lin[mt] + lin2[mt];
            TO *dst = oh + (size_t)qi * DH + 16 * mt + 4 * g4;
#pragma unroll
            for (int i = 0; i < 4; i++) stf(dst, i, fmaf(el, ln4[i], out[mt][i]) * inv);
        }
    }
}


// ---------------------------------------------------------------------------------------------
// Sequential state evolution of the prefill (paper Sec. 3 "Chunkwise Inference": after each chunk the
// oldest chunk leaves the window; it and the sparse cache are scored by self-recall error, the top
// lambda stay, the rest are folded) for the 8B head shape: one workgroup of eight wavefronts per
// (sequence, kv head), persistent over the regular chunks of a pass (a full chunk, a full window behind
// it, a full cache).  Chunks before the first regular one (cache still filling, first chunks of a
// sequence) and a ragged last chunk are handled by the generic kernel in launches of their own; the
// chunk position is handed over in a per-stream counter.
//
// H^T lives in registers for the whole pass (wavefront w owns rows 16w .. 16w+15 as fp32, re-split
// into bf16 high + low MFMA operands once per chunk); s lives in LDS.  With lambda <= 128 the features
// of the cached keys stay in LDS from chunk to chunk as well (a cache slot keeps its row; an entrant's
// row is copied into the slot it takes); the features of the 64 pairs that leave the window come from
// the chunk-parallel feature kernel below and are requested one chunk ahead, like their values.
// With lambda = 256 the candidates' features do not fit LDS: they stream through two LDS buffers in
// batches of five tiles, each batch requested (direct global -> LDS loads) while the one before it is worked
// on; the rows come from the feature kernel of the run-time shapes (phi_wide_kernel: the pairs that leave
// the window in each chunk and the cache slots as the launch finds them), the compaction keeping the
// slots' rows current in that global scratch.
// Per chunk:
//   1. snapshot of H^T (operand order, high/low parts), s and the cache's row list for the output kernel;
//   2. recall GEMM P^T = H^T Phi^T for all lambda + 64 candidates, with s riding along as one more row
//      (phi.s, the recall's denominator), and per candidate the three sums  |P|^2, P.v, |v|^2  from which
//      |P/(phi.s) - v|^2  follows;
//   3. selection: the 64th smallest score by a bitwise search on the scalar unit, the lists by ballots;
//   4. fold of the 64 others on MFMA: H[f][c] += sum_e phi_e[f] v_e[c] accumulates directly into the
//      registers that hold H^T (its C layout is the recall GEMM's A layout), operands gathered
//      through LDS in transposed order; s += sum_e phi_e (the same operands times a vector of ones);
//   5. in-place compaction: the entrants' K, V rows overwrite the slots of the leavers.

// phi of the keys of every chunk of a pass (Sec. 2.3 eq. feature_map), chunk-parallel: grid (chunk of the pass, stream),
// one 16-key tile per wavefront.  The serial state evolution below then only reads these rows (bf16 high + low parts,
// features in operand order) when the chunk's pairs leave the window one chunk later.
template <int DH>
__global__ __launch_bounds__(256) void phi_k_kernel(generic::PrefillArgs<bf16_t> a) {
    constexpr int M = 64, D = 128, C = 64, KS = DH / 32;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, r16 = lane & 15, g4 = lane >> 4;
    const int j = a.j0 + blockIdx.x, jj = j - a.jb, si = blockIdx.y, h = si % a.dm.Hkv;
    const int row = 16 * w + r16, tok = j * C + row;
    const bf16_t *Wk = a.Wk + (size_t)h * M * DH;
    const bf16_t *kr = a.k + ((size_t)si * a.T_tokens + tok) * DH;
    bf16x8 BK[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ks++) BK[ks] = tok < a.T_tokens ? ld_bf16x8(kr + 32 * ks + 8 * g4) : zero_bf16x8();
    f32x4 zt[4];
#pragma unroll
    for (int mt = 0; mt < 4; mt++) {
        zt[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ks++)
            zt[mt] = mfma16(ld_bf16x8(Wk + (size_t)(16 * mt + r16) * DH + 32 * ks + 8 * g4), BK[ks], zt[mt]);
    }
    float pp[16], pn[16];
    phi_from_z(zt, a.dm.phi_kind, pp, pn);
    bf16x8 hi[4], lo[4];
    split8(&pp[0], hi[0], lo[0]); split8(&pp[8], hi[1], lo[1]);
    split8(&pn[0], hi[2], lo[2]); split8(&pn[8], hi[3], lo[3]);
    uint16_t *dst = a.phiK + (((size_t)si * a.S + jj) * C + row) * 2 * D;
#pragma unroll
    for (int ks = 0; ks < 4; ks++) {
        *reinterpret_cast<uint4 *>(dst + ((4 * ks + g4) << 3)) = __builtin_bit_cast(uint4, hi[ks]);
        *reinterpret_cast<uint4 *>(dst + D + ((4 * ks + g4) << 3)) = __builtin_bit_cast(uint4, lo[ks]);
    }
}

// Chunk swizzle of the transposed fold operands: three bits of the row index r, chosen among the bits that differ
// between the rows one wavefront writes at once (r2, r3, r5) and between the rows it reads at once (r0 .. r3).
__device__ __forceinline__ int tswz(int r) { return ((((r >> 5) ^ (r >> 1)) & 1) << 2) | ((r >> 2) & 3); }

// Piece swizzles of row-major LDS tiles that the transposing read consumes.  A 16-lane group of that read touches four
// consecutive rows (pairs) x four consecutive 16-byte pieces (features) or two pieces x two halves (values); rows are a
// multiple of 256 bytes apart, so the piece index is XOR-ed with row bits moved to where the group's pieces do not
// differ: the two low row bits go to piece bits 2-3 (features: 16 distinct pieces per group; the swapped bit pairs also
// keep the 16 rows of a plain operand read on 16 different pieces), or to piece bits 1-2 (values).
__device__ __forceinline__ int fswz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }
template <int PR> __device__ __forceinline__ int vswz2(int row) { return (row & (PR / 2 - 1)) << 1; }

// Lanes whose value lies below a wavefront-uniform trial value, as a mask in scalar registers.  Written as an
// instruction of its own so that the compares of one search step are issued back to back into masks of their own and
// counted afterwards: compiled from a ballot, each compare writes the one condition register and its count waits for
// it before the next compare can start (300 cycles per step instead of 140).
__device__ __forceinline__ unsigned long long below_mask(uint32_t v, uint32_t trial) {
    unsigned long long m;
    asm volatile("v_cmp_lt_u32_e64 %0, %1, %2" : "=s"(m) : "v"(v), "s"(trial));
    return m;
}

template <int LAM, int DH, int RT>
__global__ __launch_bounds__(DH * 4 / RT, 1) void scan_fast_kernel(generic::PrefillArgs<bf16_t> a) {
    // one wavefront per RT tiles of 16 rows of H^T (row tile RT w + rt).  With two tiles per wavefront (head_dim 128:
    // four wavefronts) every feature operand read from LDS serves two row tiles, which halves the LDS traffic of the
    // recall GEMM and of the fold, and one wavefront per SIMD has the whole register file (nothing spills).
    constexpr int M = 64, D = 128, C = 64, ETA = 64, NW = DH / (16 * RT), NTH = 64 * NW, KS = DH / 32, PR = DH / 8;
    static_assert(RT == 1 || RT == 2, "row tiles per wavefront");
    static_assert(DH == 64 || DH == 128, "head_dim");
    constexpr int P = LAM + ETA, NE = LAM + C, NTILE = NE / 16, TB = LAM > 128 ? 5 : 12, RB = TB * 16;
    constexpr int NK = NE / 64, TC = LAM / 16;
    constexpr bool PERSIST = NTILE <= TB;   // one batch: the candidates' features all fit in LDS and the cache's part stays there
    // Otherwise the batches alternate between two buffers, the next batch's rows being requested while this one is
    // worked on.  The buffers are two arrays, selected at compile time in a batch loop unrolled by two: a wavefront's
    // reads of one buffer then do not wait for its direct loads into the other (the compiler orders LDS reads behind
    // pending direct loads per array).
    constexpr int NBUFS = PERSIST ? 1 : 2;
    static_assert(NE % 64 == 0, "candidates are selected 64 per register");
    static_assert(PERSIST || NTILE % (2 * TB) == 0, "an even number of whole batches");
    __shared__ __attribute__((aligned(16))) uint16_t PB[2 * RB * D];    // phi of (a batch of) candidates: high parts, low parts
    __shared__ __attribute__((aligned(16))) uint16_t PB1[PERSIST ? 8 : 2 * RB * D];   // the second batch buffer
    __shared__ __attribute__((aligned(16))) uint16_t PT[2 * D * C];     // phi^T of the folded pairs [part][f][e']
    __shared__ __attribute__((aligned(16))) uint16_t VT[DH * C];        // v^T of the folded pairs [c][e']
    __shared__ __attribute__((aligned(16))) float s_l[D];
    __shared__ float dn_l[NE];               // phi(k).s
    __shared__ uint32_t skey[NE];            // bit patterns of the squared errors
    __shared__ int cidx[NE];
    __shared__ int ne_s;
    __shared__ uint32_t thr_s;               // wavefront 0: the fold threshold of the previous chunk (bit pattern of a squared
                                             // error); kept here rather than in a register across the chunk loop, where one more
                                             // live value means spill reloads that wait for the chunk's loads
    __shared__ int flist[C], ecand[C], eslot[C];
    // per wavefront: |P|^2, P.v, |v|^2 over its 16 value columns; lives in the transposed tile, which is idle until the selection is done
    float (*part)[NW][NE] = reinterpret_cast<float (*)[NW][NE]>(PT);
#ifndef LOLA_PIPE_ALL
#define LOLA_PIPE_ALL 0
#endif
    constexpr bool PIPE = NW == 4 || (LOLA_PIPE_ALL && 4 * NW * NE * 4 <= 2 * D * C * 2);   // the recall loop is software-pipelined (a fourth, spare row of sums)
    static_assert((PIPE ? 4 : 3) * NW * NE * 4 <= 2 * D * C * 2, "the partial sums fit the transposed tile");

    const int tid0 = threadIdx.x, w0 = tid0 >> 6;
    const int si = blockIdx.x, h = si % a.dm.Hkv;
    float *Hg = a.st.H + (size_t)si * D * DH;
    float *sg = a.st.s + (size_t)si * D;
    bf16_t *sp_k = a.st.sp_k + (size_t)si * LAM * DH, *sp_v = a.st.sp_v + (size_t)si * LAM * DH;
    int32_t *sp_idx = a.st.sp_idx + (size_t)si * LAM;
    int32_t *sp_row = a.sp_row + (size_t)si * LAM;
    uint16_t *phiE = reinterpret_cast<uint16_t *>(a.phiE + (size_t)si * NE * D);   // [e][part][128] bf16, operand order
    const bf16_t *Wk = a.Wk + (size_t)h * M * DH;
    const bf16_t *pK = a.prefK + (size_t)si * P * DH, *pV = a.prefV + (size_t)si * P * DH;
    const bf16_t *kc = a.k + (size_t)si * a.T_tokens * DH, *vc = a.v + (size_t)si * a.T_tokens * DH;
    const int64_t a0 = a.st.n_tokens[si];
    const int spc = a.st.sp_count[si];
    int j = a.next_j[si];

    // H^T row 16 (RT w + rt) + r16, features 32ks + 16hf + 4g4 + 0..3 (the names of row tile 1 stay unused when RT = 1)
#define LOLA_SREP1(X, rt) X(rt, 0, 0) X(rt, 0, 1) X(rt, 1, 0) X(rt, 1, 1) X(rt, 2, 0) X(rt, 2, 1) X(rt, 3, 0) X(rt, 3, 1)
#define LOLA_SREP(X) LOLA_SREP1(X, 0) LOLA_SREP1(X, 1)
#define LOLA_SADDR(rt, ks, hf) ((size_t)(16 * (RT * w0 + rt) + (tid0 & 15)) * D + 32 * ks + 16 * hf + 4 * ((tid0 & 63) >> 4))
#define LOLA_SDECL(rt, ks, hf) f32x4 hreg##rt##ks##hf = {0.f, 0.f, 0.f, 0.f};
#define LOLA_SLOAD(rt, ks, hf) if (rt < RT) hreg##rt##ks##hf = *reinterpret_cast<const f32x4 *>(Hg + LOLA_SADDR(rt, ks, hf));
#define LOLA_SSTORE(rt, ks, hf) if (rt < RT) *reinterpret_cast<f32x4 *>(Hg + LOLA_SADDR(rt, ks, hf)) = hreg##rt##ks##hf;
    LOLA_SREP(LOLA_SDECL)
    bool started = false;
    bool idx_valid = false;     // rows [0, LAM) of cidx hold the cache slots' token indices
    if (tid0 == 0) thr_s = 0;   // published by the barrier that follows the loading of the state
    bool phi_valid = false;     // PERSIST: rows [0, LAM) of PB hold phi of the cache slots, and PHn / vvn the rows requested ahead
    // !PERSIST: rows [0, LAM) of the global feature scratch hold phi of the cache slots (written by the feature kernel
    // that runs before this launch, kept current by the compaction), and that kernel's rows of chunk j are phi of the
    // pairs that leave the window in chunk j
    constexpr int PHN = C * 32 / NTH;   // 16-byte pieces of a chunk's features per thread
    uint4 PHn[PHN];             // this thread's pieces of phi of the pairs that leave the window in the next chunk
    uint2 vvn[4][RT];           // their values at this wavefront's columns
#pragma unroll
    for (int x = 0; x < 4; x++)
#pragma unroll
        for (int rt = 0; rt < RT; rt++) vvn[x][rt] = make_uint2(0, 0);
#pragma unroll
    for (int x = 0; x < PHN; x++) PHn[x] = make_uint4(0, 0, 0, 0);

    for (; j < a.j1; j++) {
        const int cl = min(C, a.T_tokens - j * C);
        const int64_t aj = a0 + (int64_t)j * C;
        if (!(cl == C && aj >= ETA && spc == LAM)) break;   // not a regular chunk: the generic kernel takes over
        if (!started) {
            LOLA_SREP(LOLA_SLOAD)
            if (tid0 < D) s_l[tid0] = sg[tid0];
            started = true;
            // The state is waited for here, once: left to the first use, the wait would stand in the loop body behind the
            // chunk's own requests (the counter is in order) and hold every chunk until half of those had arrived.
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
            __syncthreads();
        }
        // The lane coordinates are made opaque once per chunk: everything derived from them (LDS and global
        // addresses of every phase) is then recomputed inside the loop instead of being hoisted out of it as
        // hundreds of loop-invariant registers, which the register file cannot hold next to H^T.
        int tl_ = threadIdx.x;
        asm volatile("" : "+v"(tl_));
        const int tid = tl_, lane = tid & 63, r16 = lane & 15, g4 = lane >> 4, w = __builtin_amdgcn_readfirstlane(tid >> 6);
        const int vrow_c = P + j * C;           // virtual row of the chunk's first token
        // source rows of candidate e: a cache slot, or one of the 64 rows before the chunk
        auto krow = [&](int e) -> const bf16_t * {
            if (e < LAM) return sp_k + (size_t)e * DH;
            const int vr = vrow_c - ETA + (e - LAM);
            return vr < P ? pK + (size_t)vr * DH : kc + (size_t)(vr - P) * DH;
        };
        auto vrow = [&](int e) -> const bf16_t * {
            if (e < LAM) return sp_v + (size_t)e * DH;
            const int vr = vrow_c - ETA + (e - LAM);
            return vr < P ? pV + (size_t)vr * DH : vc + (size_t)(vr - P) * DH;
        };
        const bool have_phi = PERSIST && phi_valid;   // the cache's rows are in LDS and the leaving pairs' rows (from the
                                                      // parallel feature kernel) were requested one chunk ahead
        // !PERSIST: where candidate e's features are (operand order, high part then low part)
        const uint16_t *phk_cur = a.phiK + ((size_t)si * a.S + (size_t)(j - a.jb)) * C * 2 * D;
        auto phirow = [&](int e) -> const uint16_t * {
            return e >= LAM ? phk_cur + (size_t)(e - LAM) * 2 * D : phiE + (size_t)e * 2 * D;
        };

        // A cache too large to stay in LDS: a batch's rows come in from the global scratch (cache
        // slots) and from the feature kernel's output (pairs leaving the window) by direct global -> LDS loads: no
        // registers, all of a wavefront's loads in flight at once.  One load instruction fills 1 KB of LDS, lane l its
        // bytes 16 l ..: four rows of one part; a row's 16-byte pieces are XOR-swizzled, so lane l fetches the piece that
        // belongs in its position.  The candidates' values at this wavefront's columns travel with them, in registers.
        constexpr int BPP = RB / 4;                          // 1 KB blocks per part (high, low)
        static_assert(PERSIST || (2 * BPP) % NW == 0, "the wavefronts share a batch's blocks evenly");
        uint2 vvq[PERSIST ? 1 : TB][RT];
        auto request_batch = [&](int tb0, uint16_t *dstbuf) {
#pragma unroll
            for (int it = 0; it < 2 * BPP / NW; it++) {
                const int blk = w + NW * it, pt = blk / BPP, rl0 = 4 * (blk % BPP);
                const int rl = rl0 + (lane >> 4), slot = lane & 15, e = 16 * tb0 + rl;
                const uint16_t *src = phirow(e) + pt * D + ((slot ^ (rl & 15)) << 3);
                lds_dma16(src, &dstbuf[pt * RB * D + rl0 * D]);
            }
#pragma unroll
            for (int u = 0; u < (PERSIST ? 1 : TB); u++)
#pragma unroll
                for (int rt = 0; rt < RT; rt++)
                    vvq[u][rt] = *reinterpret_cast<const uint2 *>(vrow(16 * (tb0 + u) + r16) + 16 * (RT * w + rt) + 4 * g4);
        };
        if (!PERSIST) request_batch(0, PB);   // (the chunk's first batch travels while the operands below are made)

        // ---- 1. operands of the recall GEMM from the fp32 registers (H^T, and s as one more row held by the lanes
        // of row 0); the snapshot for the output kernel is stored further down
        bf16x8 Ahi[RT][4], Alo[RT][4], Ash[4], Asl[4];
#define LOLA_SSPLIT(rt, ks, hf) if (rt < RT) { const f32x4 v = hreg##rt##ks##hf; \
            const __bf16 h0 = (__bf16)v[0], h1 = (__bf16)v[1], h2 = (__bf16)v[2], h3 = (__bf16)v[3]; \
            Ahi[rt % RT][ks][4 * hf] = h0; Ahi[rt % RT][ks][4 * hf + 1] = h1; Ahi[rt % RT][ks][4 * hf + 2] = h2; Ahi[rt % RT][ks][4 * hf + 3] = h3; \
            Alo[rt % RT][ks][4 * hf] = (__bf16)(v[0] - (float)h0); Alo[rt % RT][ks][4 * hf + 1] = (__bf16)(v[1] - (float)h1); \
            Alo[rt % RT][ks][4 * hf + 2] = (__bf16)(v[2] - (float)h2); Alo[rt % RT][ks][4 * hf + 3] = (__bf16)(v[3] - (float)h3); }
        LOLA_SREP(LOLA_SSPLIT)
#undef LOLA_SSPLIT
#pragma unroll
        for (int ks = 0; ks < 4; ks++) {
            float sv[8];
#pragma unroll
            for (int hf = 0; hf < 2; hf++) {
                const float4 s4 = *reinterpret_cast<const float4 *>(&s_l[32 * ks + 16 * hf + 4 * g4]);
                sv[4 * hf] = s4.x; sv[4 * hf + 1] = s4.y; sv[4 * hf + 2] = s4.z; sv[4 * hf + 3] = s4.w;
            }
            split8(sv, Ash[ks], Asl[ks]);
            if (r16 != 0) { Ash[ks] = zero_bf16x8(); Asl[ks] = zero_bf16x8(); }
        }
        // token indices of the candidates: the cache slots' stay in LDS from chunk to chunk (an entrant's index follows
        // it into its slot), so only a launch's first chunk reads them from memory
        if (!idx_valid)
            for (int e = tid; e < LAM; e += NTH) cidx[e] = sp_idx[e];
        for (int e = LAM + tid; e < NE; e += NTH) cidx[e] = (int)(aj - ETA + (e - LAM));
        // the snapshot's row list is requested ahead of the chunk's other loads (the wait counter is in order: requested
        // where it is stored, its wait would cover all of them)
        static_assert(LAM <= NTH, "one slot per thread");
        const int sprow_ld = (a.want_out && tid < LAM) ? sp_row[tid] : 0;

        // ---- 2. phi of the candidates and their recall error, in batches of TB tiles.  Global loads of a batch are
        // requested up front: the candidates' values for the recall epilogue, then the rows wanted by the next chunk; the
        // snapshot stores follow, so that they drain while the recall GEMM runs out of LDS and registers.
#pragma unroll 1
        for (int tp = 0; tp < NTILE; tp += NBUFS * TB) {
#pragma unroll
        for (int hb = 0; hb < NBUFS; hb++) {
            const int t0 = tp + hb * TB;
            const int t1 = min(NTILE, t0 + TB);
            uint16_t *PBb = hb ? PB1 : PB, *PBn = hb ? PB : PB1;   // (compile-time choices: the inner loop is unrolled)
            uint2 vv[TB][RT];
            if (!PERSIST) {
                // This batch's rows and values (requested one batch ago) have landed; then the next batch is requested
                // into the other buffer, whose readers passed the barrier that ended the batch before this one.
                __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
#pragma unroll
                for (int u = 0; u < TB; u++)
#pragma unroll
                    for (int rt = 0; rt < RT; rt++) vv[u][rt] = vvq[PERSIST ? 0 : u][rt];
                if (t0 + TB < NTILE) request_batch(t0 + TB, PBn);
            } else {
#pragma unroll
            for (int u = 0; u < TB; u++) {
#pragma unroll
                for (int rt = 0; rt < RT; rt++) {
                    if (PERSIST && u >= TC && have_phi) {
                        vv[u][rt] = vvn[u >= TC ? u - TC : 0][rt];
                    } else if (t0 + u < t1) {
                        vv[u][rt] = *reinterpret_cast<const uint2 *>(vrow(16 * (t0 + u) + r16) + 16 * (RT * w + rt) + 4 * g4);
                    }
                }
            }
            }
            if (have_phi) {   // the rows requested one chunk ago take their place behind the cache's rows
#pragma unroll
                for (int it = 0; it < PHN; it++) {
                    const int o = tid + NTH * it, row = o >> 5, pt = (o >> 4) & 1, pc = o & 15;
                    *reinterpret_cast<uint4 *>(&PBb[pt * RB * D + (LAM + row) * D + ((pc ^ (row & 15)) << 3)]) = PHn[it];
                }
            } else if (PERSIST) {
                // phi of the batch's tiles (first regular chunk of a launch): wavefront w takes tiles t0 + w, t0 + w + NW, ...
                // (W_k is read where it is used: this path runs once per launch and must not raise the kernel's register need)
#pragma unroll 1
                for (int t = t0 + w; t < t1; t += NW) {
                    const int e = 16 * t + r16;
                    const bf16_t *kr = krow(e);
                    bf16x8 BK[KS];
#pragma unroll
                    for (int ks = 0; ks < KS; ks++) BK[ks] = ld_bf16x8(kr + 32 * ks + 8 * g4);
                    f32x4 zt[4];
#pragma unroll
                    for (int mt = 0; mt < 4; mt++) {
                        zt[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int ks = 0; ks < KS; ks++)
                            zt[mt] = mfma16(ld_bf16x8(Wk + (size_t)(16 * mt + r16) * DH + 32 * ks + 8 * g4), BK[ks], zt[mt]);
                    }
                    float pp[16], pn[16];
                    phi_from_z(zt, a.dm.phi_kind, pp, pn);
                    bf16x8 hi[4], lo[4];
                    split8(&pp[0], hi[0], lo[0]); split8(&pp[8], hi[1], lo[1]);
                    split8(&pn[0], hi[2], lo[2]); split8(&pn[8], hi[3], lo[3]);
                    const int rl = e - 16 * t0;
#pragma unroll
                    for (int ks = 0; ks < 4; ks++) {
                        const int addr = rl * D + (((4 * ks + g4) ^ r16) << 3);
                        *reinterpret_cast<uint4 *>(&PBb[addr]) = __builtin_bit_cast(uint4, hi[ks]);
                        *reinterpret_cast<uint4 *>(&PBb[RB * D + addr]) = __builtin_bit_cast(uint4, lo[ks]);
                    }
                }
            }
            if (a.want_out && t0 == 0) {
                const size_t sj = (size_t)si * a.S + (j - a.jb);
                if (tid < D / 4) reinterpret_cast<float4 *>(a.snapS + sj * D)[tid] = reinterpret_cast<const float4 *>(s_l)[tid];
                if (tid < LAM) a.snapG[sj * LAM + tid] = sprow_ld;
            }
            lds_barrier();
            // recall GEMM for the batch: A = this wavefront's 16 rows of H^T, B = phi from LDS; lane (candidate r16,
            // group g4) holds rows c = 16w + 4 g4 + i and pairs them with the candidate's values at those columns.
            // Tile t's denominators come from wavefront t % 8 (A = s in row 0, zeros below).  Operands of the next
            // tile are read from LDS before this tile's MFMAs; the scheduling fence keeps the compiler from hoisting
            // the reads of all tiles at once.
            bf16x8 Bc[8], Bn[8];
#pragma unroll
            for (int ks = 0; ks < 4; ks++) {
                const int addr = r16 * D + (((4 * ks + g4) ^ r16) << 3);
                Bc[ks] = as_bf16x8(*reinterpret_cast<const uint4 *>(&PBb[addr]));
                Bc[4 + ks] = as_bf16x8(*reinterpret_cast<const uint4 *>(&PBb[RB * D + addr]));
            }
            if constexpr (PIPE) {
                // One wavefront per SIMD: the error terms of tile u - 1 (vector instructions) are issued between the
                // matrix instructions of tile u, in one branch-free block per tile (the three sums leave through one
                // store: lane group g4 stores sum g4, group 3 into a spare row); the denominators' matrix
                // instructions follow in a block of their own.
                f32x4 pp[RT];
#pragma unroll
                for (int rt = 0; rt < RT; rt++) pp[rt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int u = 0; u <= TB; u++) {
                    const bool cur = u < TB && t0 + u < t1, prev = u > 0 && t0 + u - 1 < t1;
                    f32x4 acc[RT];   // the three products of a k-step go into one accumulator: the large one first
#pragma unroll
                    for (int rt = 0; rt < RT; rt++) acc[rt] = (f32x4){0.f, 0.f, 0.f, 0.f};
                    if (cur) {
                        if (u + 1 < TB && t0 + u + 1 < t1) {
#pragma unroll
                            for (int ks = 0; ks < 4; ks++) {
                                const int addr = (16 * (u + 1) + r16) * D + (((4 * ks + g4) ^ r16) << 3);
                                Bn[ks] = as_bf16x8(*reinterpret_cast<const uint4 *>(&PBb[addr]));
                                Bn[4 + ks] = as_bf16x8(*reinterpret_cast<const uint4 *>(&PBb[RB * D + addr]));
                            }
                        }
#pragma unroll
                        for (int pass = 0; pass < 3; pass++)
#pragma unroll
                            for (int ks = 0; ks < 4; ks++)
#pragma unroll
                                for (int rt = 0; rt < RT; rt++)
                                    acc[rt] = mfma16(pass == 2 ? Alo[rt][ks] : Ahi[rt][ks], Bc[pass == 1 ? 4 + ks : ks], acc[rt]);
                    }
                    if (prev) {
                        float sa = 0.f, sb = 0.f, sc = 0.f;
#pragma unroll
                        for (int rt = 0; rt < RT; rt++) {
                            const f32x4 p = pp[rt];
                            const uint2 vvu = vv[u > 0 ? u - 1 : 0][rt];
                            const float v0 = bf_lo(vvu.x), v1 = bf_hi(vvu.x), v2 = bf_lo(vvu.y), v3 = bf_hi(vvu.y);
                            sa = fmaf(p[0], p[0], sa); sa = fmaf(p[1], p[1], sa); sa = fmaf(p[2], p[2], sa); sa = fmaf(p[3], p[3], sa);
                            sb = fmaf(p[0], v0, sb); sb = fmaf(p[1], v1, sb); sb = fmaf(p[2], v2, sb); sb = fmaf(p[3], v3, sb);
                            sc = fmaf(v0, v0, sc); sc = fmaf(v1, v1, sc); sc = fmaf(v2, v2, sc); sc = fmaf(v3, v3, sc);
                        }
                        part[g4][w][16 * (t0 + u - 1) + r16] = grp_sum3(sa, sb, sc);
                    }
                    if (cur) {
#pragma unroll
                        for (int rt = 0; rt < RT; rt++) pp[rt] = acc[rt];
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    if (cur && ((t0 + u) & (NW - 1)) == w) {
                        f32x4 ds = {0.f, 0.f, 0.f, 0.f}, ds2 = {0.f, 0.f, 0.f, 0.f}, ds3 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int ks = 0; ks < 4; ks++) {
                            ds = mfma16(Ash[ks], Bc[ks], ds);
                            ds2 = mfma16(Ash[ks], Bc[4 + ks], ds2);
                            ds3 = mfma16(Asl[ks], Bc[ks], ds3);
                        }
                        if (g4 == 0) dn_l[16 * (t0 + u) + r16] = ds[0] + (ds2[0] + ds3[0]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int x = 0; x < 8; x++) Bc[x] = Bn[x];
                }
            } else {
#pragma unroll
            for (int u = 0; u < TB; u++) {
                if (t0 + u < t1) {
                    const int e = 16 * (t0 + u) + r16;
                    if (u + 1 < TB && t0 + u + 1 < t1) {
#pragma unroll
                        for (int ks = 0; ks < 4; ks++) {
                            const int addr = (16 * (u + 1) + r16) * D + (((4 * ks + g4) ^ r16) << 3);
                            Bn[ks] = as_bf16x8(*reinterpret_cast<const uint4 *>(&PBb[addr]));
                            Bn[4 + ks] = as_bf16x8(*reinterpret_cast<const uint4 *>(&PBb[RB * D + addr]));
                        }
                    }
                    f32x4 acc[RT];   // the three products of a k-step go into one accumulator: the large one first
#pragma unroll
                    for (int rt = 0; rt < RT; rt++) acc[rt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int pass = 0; pass < 3; pass++)
#pragma unroll
                        for (int ks = 0; ks < 4; ks++)
#pragma unroll
                            for (int rt = 0; rt < RT; rt++)
                                acc[rt] = mfma16(pass == 2 ? Alo[rt][ks] : Ahi[rt][ks], Bc[pass == 1 ? 4 + ks : ks], acc[rt]);
                    if (((t0 + u) & (NW - 1)) == w) {
                        f32x4 ds = {0.f, 0.f, 0.f, 0.f}, ds2 = {0.f, 0.f, 0.f, 0.f}, ds3 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int ks = 0; ks < 4; ks++) {
                            ds = mfma16(Ash[ks], Bc[ks], ds);
                            ds2 = mfma16(Ash[ks], Bc[4 + ks], ds2);
                            ds3 = mfma16(Asl[ks], Bc[ks], ds3);
                        }
                        if (g4 == 0) dn_l[e] = ds[0] + (ds2[0] + ds3[0]);
                    }
                    float sa = 0.f, sb = 0.f, sc = 0.f;
#pragma unroll
                    for (int rt = 0; rt < RT; rt++) {
                        const f32x4 p = acc[rt];
                        const float v0 = bf_lo(vv[u][rt].x), v1 = bf_hi(vv[u][rt].x), v2 = bf_lo(vv[u][rt].y), v3 = bf_hi(vv[u][rt].y);
                        sa = fmaf(p[0], p[0], sa); sa = fmaf(p[1], p[1], sa); sa = fmaf(p[2], p[2], sa); sa = fmaf(p[3], p[3], sa);
                        sb = fmaf(p[0], v0, sb); sb = fmaf(p[1], v1, sb); sb = fmaf(p[2], v2, sb); sb = fmaf(p[3], v3, sb);
                        sc = fmaf(v0, v0, sc); sc = fmaf(v1, v1, sc); sc = fmaf(v2, v2, sc); sc = fmaf(v3, v3, sc);
                    }
                    const float s3 = grp_sum3(sa, sb, sc);   // lane group g4 holds sum g4
                    if (g4 < 3) part[g4][w][e] = s3;
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int x = 0; x < 8; x++) Bc[x] = Bn[x];
                }
            }
            }
            // Requests that nothing in this chunk waits for - the rows wanted by the next chunk and the snapshot of
            // H^T - are issued where a wavefront would otherwise idle: by wavefront 0 here, behind its share of the
            // recall GEMM (it waits for the other wavefront of its SIMD anyway), by the others while wavefront 0 runs the
            // selection.  Issued by all wavefronts ahead of the recall GEMM they cost 1.3 us per chunk.
            if (w == 0 && t0 + TB >= NTILE) {
                if (PERSIST) {   // this chunk's own pairs leave the window in the next chunk
                    const uint4 *ph = reinterpret_cast<const uint4 *>(a.phiK + ((size_t)si * a.S + (j - a.jb)) * C * 2 * D);
#pragma unroll
                    for (int it = 0; it < PHN; it++) PHn[it] = ph[tid + NTH * it];
#pragma unroll
                    for (int u = 0; u < 4; u++)
#pragma unroll
                        for (int rt = 0; rt < RT; rt++)
                            vvn[u][rt] = *reinterpret_cast<const uint2 *>(vc + (size_t)(j * C + 16 * u + r16) * DH + 16 * (RT * w + rt) + 4 * g4);
                }
                if (a.want_out) {
                    uint16_t *s16 = reinterpret_cast<uint16_t *>(a.snapH) + ((size_t)si * a.S + (j - a.jb)) * (2 * D * DH);
#pragma unroll
                    for (int rt = 0; rt < RT; rt++)
#pragma unroll
                        for (int ks = 0; ks < 4; ks++) {
                            // one contiguous 1 KB piece per store: [row tile][k-step][lane]
                            const int off = (((RT * w + rt) * 4 + ks) * 64 + lane) << 3;
                            *reinterpret_cast<uint4 *>(s16 + off) = __builtin_bit_cast(uint4, Ahi[rt][ks]);
                            *reinterpret_cast<uint4 *>(s16 + D * DH + off) = __builtin_bit_cast(uint4, Alo[rt][ks]);
                        }
                }
            }
            lds_barrier();
        }
        }

        // ---- 3. selection: the 64 candidates with the smallest squared error are folded (order: score descending,
        // token index ascending, the first LAM stay).  The squared error is |P|^2 / (phi.s)^2 - 2 P.v / (phi.s) + |v|^2
        // (recall = 0 while phi.s = 0, i.e. nothing folded yet); the bit pattern of a float >= 0 orders like an integer.
        for (int e = tid; e < NE; e += NTH) {
            const float dn = dn_l[e], rd = dn > 0.f ? __builtin_amdgcn_rcpf(dn) : 0.f;
            float sa = 0.f, sb = 0.f, sc = 0.f;
#pragma unroll
            for (int x = 0; x < NW; x++) { sa += part[0][x][e]; sb += part[1][x][e]; sc += part[2][x][e]; }
            const float sq = fmaxf(fmaf(rd * rd, sa, fmaf(-2.0f * rd, sb, sc)), 0.f);
            skey[e] = __float_as_uint(sq) & 0x7FFFFFFFu;
        }
        lds_barrier();
        // One wavefront holds all scores (NK per lane) and finds the 64th smallest by building it bit by bit: a trial
        // value is kept when fewer than 64 scores lie below it (votes counted on the scalar unit).  Scores equal to
        // the threshold are folded too if that makes exactly 64; otherwise (exact ties across the cut) the same search
        // over their token indices picks the largest ones.  The lists follow from the fold predicate by ballots:
        // candidates to fold; entrants paired with the slots of the leavers.
        if (w != 0) {   // the requests wavefront 0 issued before the recall GEMM (H^T is still the chunk's entry state)
            if (PERSIST) {
                const uint4 *ph = reinterpret_cast<const uint4 *>(a.phiK + ((size_t)si * a.S + (j - a.jb)) * C * 2 * D);
#pragma unroll
                for (int it = 0; it < PHN; it++) PHn[it] = ph[tid + NTH * it];
#pragma unroll
                for (int u = 0; u < 4; u++)
#pragma unroll
                    for (int rt = 0; rt < RT; rt++)
                        vvn[u][rt] = *reinterpret_cast<const uint2 *>(vc + (size_t)(j * C + 16 * u + r16) * DH + 16 * (RT * w + rt) + 4 * g4);
            }
            if (a.want_out) {
                uint16_t *s16 = reinterpret_cast<uint16_t *>(a.snapH) + ((size_t)si * a.S + (j - a.jb)) * (2 * D * DH);
#define LOLA_SSNAP(rt, ks) if (rt < RT) { float sv[8]; \
                _Pragma("unroll") for (int x = 0; x < 4; x++) { sv[x] = hreg##rt##ks##0[x]; sv[4 + x] = hreg##rt##ks##1[x]; } \
                bf16x8 hi8, lo8; split8(sv, hi8, lo8); \
                const int off = (((RT * w + rt) * 4 + ks) * 64 + lane) << 3; \
                *reinterpret_cast<uint4 *>(s16 + off) = __builtin_bit_cast(uint4, hi8); \
                *reinterpret_cast<uint4 *>(s16 + D * DH + off) = __builtin_bit_cast(uint4, lo8); }
                LOLA_SSNAP(0, 0) LOLA_SSNAP(0, 1) LOLA_SSNAP(0, 2) LOLA_SSNAP(0, 3)
                LOLA_SSNAP(1, 0) LOLA_SSNAP(1, 1) LOLA_SSNAP(1, 2) LOLA_SSNAP(1, 3)
#undef LOLA_SSNAP
            }
        } else {
            uint32_t sb[NK]; int ix[NK];
#pragma unroll
            for (int x = 0; x < NK; x++) { sb[x] = skey[64 * x + lane]; ix[x] = cidx[64 * x + lane]; }
            uint32_t thr = 0;
            uint32_t cut = 0;               // != 0: exactly 64 scores lie below it, the search can stop there
            int bit0 = 28;
            {   // The threshold moves little from chunk to chunk: if the leading 13 bits of the last one still bracket
                // the 64th smallest score (fewer than 64 scores below the prefix, at least 64 below the next prefix),
                // the search resumes below them, in the state it would have reached bit by bit.
                const uint32_t tA = (uint32_t)__builtin_amdgcn_readfirstlane((int)thr_s) & 0xFFFC0000u, tB = tA + (1u << 18);
                unsigned long long mA[NK], mB[NK];
#pragma unroll
                for (int x = 0; x < NK; x++) { mA[x] = below_mask(sb[x], tA); mB[x] = below_mask(sb[x], tB); }
                int cA = 0, cB = 0;
#pragma unroll
                for (int x = 0; x < NK; x++) { cA += __popcll(mA[x]); cB += __popcll(mB[x]); }
                if (cA < C && cB >= C) {
                    thr = tA; bit0 = 16;
                    if (cB == C) cut = tB;
                } else {   // bit 30 alone, then two bits per step (three trial values counted side by side)
                    int c = 0;
#pragma unroll
                    for (int x = 0; x < NK; x++) c += __popcll(__ballot(sb[x] < (1u << 30)));
                    if (c < C) thr = 1u << 30;
                }
            }
#pragma unroll 1
            for (int bit = bit0; bit >= 0 && cut == 0; bit -= 2) {
                const uint32_t t1 = thr | (1u << bit), t2 = thr | (2u << bit), t3 = thr | (3u << bit);
                unsigned long long m1[NK], m2[NK], m3[NK];
#pragma unroll
                for (int x = 0; x < NK; x++) { m1[x] = below_mask(sb[x], t1); m2[x] = below_mask(sb[x], t2); m3[x] = below_mask(sb[x], t3); }
                int c1 = 0, c2 = 0, c3 = 0;
#pragma unroll
                for (int x = 0; x < NK; x++) { c1 += __popcll(m1[x]); c2 += __popcll(m2[x]); c3 += __popcll(m3[x]); }
                cut = c1 == C ? t1 : (c2 == C ? t2 : (c3 == C ? t3 : 0u));
                thr = c3 < C ? t3 : (c2 < C ? t2 : (c1 < C ? t1 : thr));
            }
            int n_lt = 0, n_eq = 0;
            if (lane == 0) thr_s = cut != 0 ? cut : thr;
            if (cut != 0) { thr = cut; n_lt = C; }   // everything below the cut is folded, nothing at or above it
            else {
#pragma unroll
                for (int x = 0; x < NK; x++) { n_lt += __popcll(__ballot(sb[x] < thr)); n_eq += __popcll(__ballot(sb[x] == thr)); }
            }
            const int need = C - n_lt;      // ties at the threshold to fold: 0 after an early stop, else 1 <= need <= n_eq
            uint32_t imin = need == 0 ? 0xFFFFFFFFu : 0u;   // ties are folded from token index imin upwards
            if (need != 0 && n_eq != need) {
#pragma unroll 1
                for (int bit = 30; bit >= 0; bit--) {
                    const uint32_t trial = imin | (1u << bit);
                    int c = 0;
#pragma unroll
                    for (int x = 0; x < NK; x++) c += __popcll(__ballot(sb[x] == thr && (uint32_t)ix[x] >= trial));
                    if (c >= need) imin = trial;
                }
            }
            int nf = 0, nen = 0, nlv = 0;
#pragma unroll
            for (int x = 0; x < NK; x++) {
                const int e = 64 * x + lane;
                const bool fo = sb[x] < thr || (sb[x] == thr && (uint32_t)ix[x] >= imin);
                const bool en = !fo && e >= LAM, lv = fo && e < LAM;
                const unsigned long long mf = __ballot(fo), me = __ballot(en), ml = __ballot(lv);
                const unsigned long long below = (1ull << lane) - 1ull;
                if (fo) flist[nf + __popcll(mf & below)] = e;
                if (en) ecand[nen + __popcll(me & below)] = e;
                if (lv) eslot[nlv + __popcll(ml & below)] = e;
                nf += __popcll(mf); nen += __popcll(me); nlv += __popcll(ml);
            }
            if (lane == 0) ne_s = nen;
        }
        lds_barrier();
        // exactly 64 are folded, so entrants and leavers pair up
        const int ne = ne_s;

        // ---- 4. fold: operands of the folded pairs transposed into LDS, then H[f][c] += sum_e phi_e[f] v_e[c].
        // Each thread takes two folded pairs (e', e'+1) and one 16-byte piece of their rows and writes eight 32-bit
        // words (column pair e', e'+1 of eight rows of the transposed tile).  Within a wavefront the lanes cover 16
        // pieces x 4 column pairs; the 16-byte column chunk of a row is XOR-ed with three row bits chosen so that
        // these writes fall on all banks (two lanes per bank) and the 128-bit operand reads of the MFMAs below
        // on all eight chunks evenly.
        {
            // phi^T: piece ch, part pt = w % 2 and column chunk w / 2 + (NW / 2) it of the folded pairs
            constexpr int CPW = NW / 2, PIT = 8 / CPW;
            const int ch = tid & 15, pairpos = (tid >> 4) & 3, pt = w & 1;
            constexpr int VIT = 32 * PR / NTH;   // column pairs of v^T per thread
            uint4 pa[PIT], pb[PIT], va[VIT], vb[VIT];
#pragma unroll
            for (int it = 0; it < PIT; it++) {
                const int ep = 8 * ((w >> 1) + CPW * it) + 2 * pairpos;
                const int ea = flist[ep], eb = flist[ep + 1];
                if (PERSIST) {
                    pa[it] = *reinterpret_cast<const uint4 *>(&PB[pt * RB * D + ea * D + ((ch ^ (ea & 15)) << 3)]);
                    pb[it] = *reinterpret_cast<const uint4 *>(&PB[pt * RB * D + eb * D + ((ch ^ (eb & 15)) << 3)]);
                } else {
                    pa[it] = *reinterpret_cast<const uint4 *>(phirow(ea) + pt * D + (ch << 3));
                    pb[it] = *reinterpret_cast<const uint4 *>(phirow(eb) + pt * D + (ch << 3));
                }
            }
            // v^T: VIT items per thread: piece vch of the value rows of column pair vpair0 + (NTH / PR) vit
            const int vch = tid % PR, vpair0 = tid / PR;
#pragma unroll
            for (int vit = 0; vit < VIT; vit++) {
                const int ep = 2 * (vpair0 + (NTH / PR) * vit);
                va[vit] = reinterpret_cast<const uint4 *>(vrow(flist[ep]))[vch];
                vb[vit] = reinterpret_cast<const uint4 *>(vrow(flist[ep + 1]))[vch];
            }
            // feature held by element x of piece ch (operand order): 32 (ch / 4) + 16 (x / 4) + 4 (ch % 4) + x % 4
#pragma unroll
            for (int x = 0; x < 8; x++) {
                const int f = 32 * (ch >> 2) + 16 * (x >> 2) + 4 * (ch & 3) + (x & 3);
                const int bx = pt * D * C + f * C + ((((w >> 1) ^ tswz(f))) << 3) + 2 * pairpos;
#pragma unroll
                for (int it = 0; it < PIT; it++) {
                    const uint32_t ua = (&pa[it].x)[x >> 1], ub = (&pb[it].x)[x >> 1];
                    const uint32_t wv = (x & 1) ? ((ua >> 16) | (ub & 0xFFFF0000u)) : ((ua & 0xFFFFu) | (ub << 16));
                    *reinterpret_cast<uint32_t *>(&PT[bx ^ ((CPW * it) << 3)]) = wv;
                }
            }
#pragma unroll
            for (int vit = 0; vit < VIT; vit++) {
                const int vpair = vpair0 + (NTH / PR) * vit;
#pragma unroll
                for (int x = 0; x < 8; x++) {
                    const int c = 8 * vch + x;
                    const int bx = c * C + ((((vpair >> 2) ^ tswz(c))) << 3) + 2 * (vpair & 3);
                    const uint32_t ua = (&va[vit].x)[x >> 1], ub = (&vb[vit].x)[x >> 1];
                    const uint32_t wv = (x & 1) ? ((ua >> 16) | (ub & 0xFFFF0000u)) : ((ua & 0xFFFFu) | (ub << 16));
                    *reinterpret_cast<uint32_t *>(&VT[bx]) = wv;
                }
            }
        }
        lds_barrier();
        {
            // compaction, first half: the entrants' rows are requested now and stored after the fold (all reads of
            // the leavers' rows were completed before the barrier above)
            constexpr int CIT = C * 2 * PR / NTH;   // 16-byte pieces of up to 64 entrants' rows per thread
            uint4 cp[CIT];
#pragma unroll
            for (int it = 0; it < CIT; it++) {
                const int o = tid + NTH * it;
                cp[it] = make_uint4(0, 0, 0, 0);   // (left unset on some paths, the array is kept in memory instead of registers)
                if (o < ne * 2 * PR) {
                    const int x = o / (2 * PR), rem = o % (2 * PR);
                    const int e = ecand[x];
                    cp[it] = reinterpret_cast<const uint4 *>((rem >= PR) ? vrow(e) : krow(e))[rem % PR];
                }
            }
            bf16x8 Bv[RT][2];
#pragma unroll
            for (int rt = 0; rt < RT; rt++)
#pragma unroll
                for (int k2 = 0; k2 < 2; k2++) {
                    const int c = 16 * (RT * w + rt) + r16;
                    Bv[rt][k2] = as_bf16x8(*reinterpret_cast<const uint4 *>(&VT[c * C + (((4 * k2 + g4) ^ tswz(c)) << 3)]));
                }
            // per feature tile (16 features): four A operands (high / low part x two k-steps); the operands of the next
            // tile are read from LDS before this tile's MFMAs are issued
            bf16x8 Ac[4], An[4];
#define LOLA_SFA(dst, mt) _Pragma("unroll") for (int x = 0; x < 4; x++) { const int f = 16 * (mt) + r16; \
                dst[x] = as_bf16x8(*reinterpret_cast<const uint4 *>(&PT[(x >> 1) * D * C + f * C + (((4 * (x & 1) + g4) ^ tswz(f)) << 3)])); }
            LOLA_SFA(Ac, 0)
            // s += sum of the folded features: a feature tile's operands times a vector of ones (tile mt by wavefront mt % NW)
            const bf16x8 ones = as_bf16x8(make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u));
            f32x4 sacc[8 / NW];
#pragma unroll
            for (int x = 0; x < 8 / NW; x++) sacc[x] = (f32x4){0.f, 0.f, 0.f, 0.f};
#define LOLA_SFOLD2(ks, hf) { if (2 * ks + hf + 1 < 8) { LOLA_SFA(An, 2 * ks + hf + 1) } \
            _Pragma("unroll") for (int x = 0; x < 4; x++) { hreg0##ks##hf = mfma16(Ac[x], Bv[0][x & 1], hreg0##ks##hf); \
                                                            if (RT > 1) hreg1##ks##hf = mfma16(Ac[x], Bv[RT - 1][x & 1], hreg1##ks##hf); } \
            if (((2 * ks + hf) & (NW - 1)) == w) { _Pragma("unroll") for (int x = 0; x < 4; x++) sacc[(2 * ks + hf) / NW] = mfma16(Ac[x], ones, sacc[(2 * ks + hf) / NW]); } \
            __builtin_amdgcn_sched_barrier(0); \
            _Pragma("unroll") for (int x = 0; x < 4; x++) Ac[x] = An[x]; }
            LOLA_SFOLD2(0, 0) LOLA_SFOLD2(0, 1) LOLA_SFOLD2(1, 0) LOLA_SFOLD2(1, 1) LOLA_SFOLD2(2, 0) LOLA_SFOLD2(2, 1) LOLA_SFOLD2(3, 0) LOLA_SFOLD2(3, 1)
#undef LOLA_SFOLD2
#undef LOLA_SFA
            if (r16 == 0) {   // column 0 of the result tiles: features 16 (w + NW x) + 4 g4 + 0..3
#pragma unroll
                for (int x = 0; x < 8 / NW; x++) {
                    float4 *sp = reinterpret_cast<float4 *>(&s_l[16 * (w + NW * x) + 4 * g4]);
                    float4 sv = *sp;
                    sv.x += sacc[x][0]; sv.y += sacc[x][1]; sv.z += sacc[x][2]; sv.w += sacc[x][3];
                    *sp = sv;
                }
            }
            // ---- 5. compaction, second half: entrants take the leavers' slots, in the state and (their features) in LDS
#pragma unroll
            for (int it = 0; it < CIT; it++) {
                const int o = tid + NTH * it;
                if (o < ne * 2 * PR) {
                    const int x = o / (2 * PR), rem = o % (2 * PR);
                    bf16_t *dst = ((rem >= PR) ? sp_v : sp_k) + (size_t)eslot[x] * DH;
                    reinterpret_cast<uint4 *>(dst)[rem % PR] = cp[it];
                }
            }
            if (PERSIST) {
#pragma unroll
                for (int it = 0; it < PHN; it++) {
                    const int o = tid + NTH * it;
                    if (o < ne * 32) {
                        const int x = o >> 5, rem = o & 31, pt = rem >> 4, ch = rem & 15;
                        const int e = ecand[x], sl = eslot[x];
                        const uint4 val = *reinterpret_cast<const uint4 *>(&PB[pt * RB * D + e * D + ((ch ^ (e & 15)) << 3)]);
                        *reinterpret_cast<uint4 *>(&PB[pt * RB * D + sl * D + ((ch ^ (sl & 15)) << 3)]) = val;
                    }
                }
            } else {
                // the same in the global scratch: a slot's row follows its occupant (every read of the leavers' rows
                // was completed before the barrier that precedes the fold)
#pragma unroll
                for (int it = 0; it < PHN; it++) {
                    const int o = tid + NTH * it;
                    if (o < ne * 32) {
                        const int x = o >> 5, rem = o & 31;
                        const uint4 val = *reinterpret_cast<const uint4 *>(phirow(ecand[x]) + rem * 8);
                        *reinterpret_cast<uint4 *>(phiE + (size_t)eslot[x] * 2 * D + rem * 8) = val;
                    }
                }
            }
        }
        for (int x = tid; x < ne; x += NTH) {
            const int e = ecand[x], sl = eslot[x];
            const int ti = cidx[e];
            sp_idx[sl] = ti;
            cidx[sl] = ti;
            sp_row[sl] = vrow_c - ETA + (e - LAM);
        }
        idx_valid = true;
        phi_valid = PERSIST;
        __syncthreads();   // (workgroup scope is enough: only this workgroup reads the stream's memories before the kernel ends)
        if (a.sel_trace) {
            int32_t *tr = a.sel_trace + ((size_t)si * a.n_chunks + j) * LAM;
            for (int sl = tid; sl < LAM; sl += NTH) tr[sl] = sp_idx[sl];
        }
    }
    if (started) {
        LOLA_SREP(LOLA_SSTORE)
        if (tid0 < D) sg[tid0] = s_l[tid0];
    }
    if (tid0 == 0) a.next_j[si] = j;
#undef LOLA_SREP
#undef LOLA_SREP1
#undef LOLA_SADDR
#undef LOLA_SDECL
#undef LOLA_SLOAD
#undef LOLA_SSTORE
}

// ---------------------------------------------------------------------------------------------
// State evolution of the prefill for any window and sparse budget (multiples of 64, read from the arguments) and 128 or
// 256 features: the paper's own models use twice the head dimension as feature dimension and windows / budgets of
// 128 .. 1024 in the long-context runs (Sec. 4).  Same five steps per regular chunk as scan_fast_kernel (snapshot,
// self-recall error of the lambda + 64 candidates, selection of the 64 to fold, fold, compaction; Sec. 3.1 - 3.2), laid
// out for a candidate set that does not fit LDS:
//   * phi of every row is computed chunk-parallel beforehand (phi_wide_kernel): the pairs that leave the window in chunk
//     j (phiK[j - jb]) and the cache slots as the launch finds them (phiE[slot], kept current by the compaction);
//   * one wavefront per 16 rows of H^T (fp32 accumulators, split into bf16 high + low parts once per chunk);
//   * the candidates' features and values stream through LDS in batches of RB rows (NBUF buffers) by direct
//     global -> LDS loads issued NBUF - 1 batches ahead; each wavefront runs the recall GEMM of the batch against its
//     rows of H^T and leaves |P|^2, P.v, |v|^2 over its 16 value columns per candidate, summed over the wavefronts one
//     batch later; phi(k).s is a plain dot product per row of the batch;
//   * the fold reads both MFMA operands out of row-major LDS tiles (the 64 folded rows gathered by direct loads)
//     through the transposing LDS read, the contraction index being the pair.
// A sparse budget of 0 switches scoring and selection off (every leaving pair is folded).
//
// phi_wide_kernel: phi of the rows the evolution kernel reads (Sec. 2.3 eq. feature_map), 64 rows per workgroup, bf16
// high + low parts in operand order: blocks [0, j1 - j0) the pairs that leave the window in chunk j0 + block (virtual
// rows lam + j C + 0..63) -> phiK[j - jb]; the lam / 64 blocks behind them the cache slots -> phiE[slot].
template <int DH, int DF>
__global__ __launch_bounds__(256) void phi_wide_kernel(generic::PrefillArgs<bf16_t> a) {
    constexpr int M = DF / 2, C = 64, KS = DH / 32, NZT = M / 16, FR = 2 * DF;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, r16 = lane & 15, g4 = lane >> 4;
    const int si = blockIdx.y, h = si % a.dm.Hkv, LAM = a.dm.lam, P = LAM + a.dm.eta;
    const int nch = a.j1 - a.j0, row = 16 * w + r16;
    const bf16_t *Wk = a.Wk + (size_t)h * M * DH;
    const bf16_t *kr;
    uint16_t *dst;
    bool valid = true;
    if ((int)blockIdx.x < nch) {
        // the pairs that leave the window while chunk j joins it: virtual rows lam + j C + 0..63 (rows below P: the cache
        // and window the call found)
        const int j = a.j0 + (int)blockIdx.x, vr = LAM + j * C + row;
        valid = vr - P < a.T_tokens;
        kr = vr < P ? a.prefK + ((size_t)si * P + vr) * DH : a.k + ((size_t)si * a.T_tokens + (valid ? vr - P : 0)) * DH;
        dst = a.phiK + (((size_t)si * a.S + (j - a.jb)) * C + row) * FR;
    } else {
        const int slot = 64 * ((int)blockIdx.x - nch) + row;   // the grid covers lam / 64 such blocks
        kr = a.st.sp_k + ((size_t)si * LAM + slot) * DH;
        dst = reinterpret_cast<uint16_t *>(a.phiE + (size_t)si * (LAM + C) * DF) + (size_t)slot * FR;
    }
    bf16x8 BK[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ks++) BK[ks] = valid ? ld_bf16x8(kr + 32 * ks + 8 * g4) : zero_bf16x8();
    f32x4 zt[NZT];
#pragma unroll
    for (int mt = 0; mt < NZT; mt++) {
        zt[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ks++)
            zt[mt] = mfma16(ld_bf16x8(Wk + (size_t)(16 * mt + r16) * DH + 32 * ks + 8 * g4), BK[ks], zt[mt]);
    }
    float pp[4 * NZT], pn[4 * NZT];
    phi_from_z_tiles<NZT>(zt, a.dm.phi_kind, pp, pn);
    // operand order: 16-byte piece 4 ks + g4 of a part holds features 32 ks + 16 (x / 4) + 4 g4 + x % 4, x < 8: the
    // lane's values of projection tiles 2 ks and 2 ks + 1; the negative half follows the positive half
#pragma unroll
    for (int ks = 0; ks < M / 32; ks++) {
        bf16x8 hi, lo;
        split8(&pp[8 * ks], hi, lo);
        *reinterpret_cast<uint4 *>(dst + ((4 * ks + g4) << 3)) = __builtin_bit_cast(uint4, hi);
        *reinterpret_cast<uint4 *>(dst + DF + ((4 * ks + g4) << 3)) = __builtin_bit_cast(uint4, lo);
        split8(&pn[8 * ks], hi, lo);
        *reinterpret_cast<uint4 *>(dst + ((4 * (M / 32 + ks) + g4) << 3)) = __builtin_bit_cast(uint4, hi);
        *reinterpret_cast<uint4 *>(dst + DF + ((4 * (M / 32 + ks) + g4) << 3)) = __builtin_bit_cast(uint4, lo);
    }
}

// SCORED: the candidates' scores are given (the query-dependent scores of Sec. 4 / appendix "scoring ablation", summed
// beforehand per token: tok_score for the pairs that leave the window, sp_score for the cache slots) instead of being
// self-recall errors; step 2 is skipped, an entrant's score follows it into its slot, everything else is the same.
template <int DH, int DF, bool SCORED>
__global__ __launch_bounds__(DH * 4) void scan_wide_kernel(generic::PrefillArgs<bf16_t> a) {
    constexpr int C = 64, NW = DH / 16, NTH = 64 * NW, KF = DF / 32, NMT = DF / 16, PR = DH / 8, FR = 2 * DF, PP = DF / 8;
    constexpr int RB = DF == 256 ? 32 : 64, TB = RB / 16;  // candidates per batch (32 KB of features)
    constexpr int NBUF = DF == 256 ? 3 : 2;                // batch buffers in LDS: requests run NBUF - 1 batches ahead
    constexpr int VPB = RB * DH / 512 / NW;                // direct loads per wavefront and batch: values ...
    constexpr int LPB = RB * FR / 512 / NW + VPB;          // ... and features + values
    static_assert(VPB >= 1 && VPB * NW * 512 == RB * DH, "the wavefronts share the values of a batch evenly");
    constexpr int NEMAX = 1024 + C, NKMAX = NEMAX / 64;
    constexpr int BUF = RB * FR + RB * DH;                 // 16-bit elements of one batch buffer: features, then values
    constexpr int FOLD = C * FR + C * DH;                  // the folded pairs' features and values
    constexpr int POOL = NBUF * BUF > FOLD ? NBUF * BUF : FOLD;
    static_assert((DH == 64 || DH == 128) && (DF == 128 || DF == 256), "shape");
    __shared__ __attribute__((aligned(16))) uint16_t pool[POOL];
    __shared__ __attribute__((aligned(16))) float s_l[DF];
    __shared__ float dn_l[NEMAX];              // phi(k).s
    __shared__ float tot[3][NEMAX];            // |P|^2, P.v, |v|^2 over all value columns
    __shared__ uint32_t skey[NEMAX];           // bit patterns of the squared errors
    __shared__ int cidx[NEMAX];                // token index of each candidate
    __shared__ float part[2][3][NW][RB];       // per wavefront: the three sums over its 16 columns, for the batch in flight
    __shared__ int flist[C], ecand[C], eslot[C];
    __shared__ int ne_s;

    const int tid0 = threadIdx.x, w0 = tid0 >> 6;
    const int si = blockIdx.x;
    const int LAM = a.dm.lam, ETA = a.dm.eta, P = LAM + ETA, NE = LAM + C, NBATCH = NE / RB, nk = NE / 64;
    float *Hg = a.st.H + (size_t)si * DF * DH;
    float *sg = a.st.s + (size_t)si * DF;
    bf16_t *sp_k = a.st.sp_k + (size_t)si * LAM * DH, *sp_v = a.st.sp_v + (size_t)si * LAM * DH;
    int32_t *sp_idx = a.st.sp_idx + (size_t)si * LAM;
    int32_t *sp_row = a.sp_row + (size_t)si * LAM;
    uint16_t *phiE = reinterpret_cast<uint16_t *>(a.phiE + (size_t)si * (LAM + C) * DF);   // [slot][part][DF] bf16, operand order
    const bf16_t *pK = a.prefK + (size_t)si * P * DH, *pV = a.prefV + (size_t)si * P * DH;
    const bf16_t *kc = a.k + (size_t)si * a.T_tokens * DH, *vc = a.v + (size_t)si * a.T_tokens * DH;
    const int64_t a0 = a.st.n_tokens[si];
    const int spc = a.st.sp_count[si];
    int j = a.next_j[si];

    // H^T row 16 w + r16, features 16 mt + 4 g4 + 0..3
    f32x4 hacc[NMT];
#pragma unroll
    for (int mt = 0; mt < NMT; mt++) hacc[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    bool started = false;

    for (; j < a.j1; j++) {
        const int cl = min(C, a.T_tokens - j * C);
        const int64_t aj = a0 + (int64_t)j * C;
        if (!(cl == C && aj >= ETA && spc == LAM)) break;   // not a regular chunk: the generic kernel takes over
        if (!started) {
            const float *hrow = Hg + (size_t)(16 * w0 + (tid0 & 15)) * DF + 4 * ((tid0 & 63) >> 4);
#pragma unroll
            for (int mt = 0; mt < NMT; mt++) hacc[mt] = *reinterpret_cast<const f32x4 *>(hrow + 16 * mt);
            for (int x = tid0; x < DF; x += NTH) s_l[x] = sg[x];
            for (int e = tid0; e < LAM; e += NTH) cidx[e] = sp_idx[e];
            started = true;
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
            __syncthreads();
        }
        // the lane coordinates are made opaque once per chunk, so that the addresses derived from them are recomputed in
        // the loop instead of being kept as loop-invariant registers next to H^T
        int tl_ = threadIdx.x;
        asm volatile("" : "+v"(tl_));
        const int tid = tl_, lane = tid & 63, r16 = lane & 15, g4 = lane >> 4, w = __builtin_amdgcn_readfirstlane(tid >> 6);
        const int vrow_l = LAM + j * C;   // virtual row of the first pair that leaves the window in this chunk
        const uint16_t *phk = a.phiK + ((size_t)si * a.S + (size_t)(j - a.jb)) * C * FR;
        auto krow = [&](int e) -> const bf16_t * {
            if (e < LAM) return sp_k + (size_t)e * DH;
            const int vr = vrow_l + (e - LAM);
            return vr < P ? pK + (size_t)vr * DH : kc + (size_t)(vr - P) * DH;
        };
        auto vrow = [&](int e) -> const bf16_t * {
            if (e < LAM) return sp_v + (size_t)e * DH;
            const int vr = vrow_l + (e - LAM);
            return vr < P ? pV + (size_t)vr * DH : vc + (size_t)(vr - P) * DH;
        };
        auto phirow = [&](int e) -> const uint16_t * { return e < LAM ? phiE + (size_t)e * FR : phk + (size_t)(e - LAM) * FR; };

        // the snapshot's row list is read before anything else is requested or stored (the memory counter is in order)
        constexpr int NSP = 1024 / NTH;
        int sprow_ld[NSP];
#pragma unroll
        for (int x = 0; x < NSP; x++) sprow_ld[x] = (a.want_out && tid + NTH * x < LAM) ? sp_row[tid + NTH * x] : 0;

        // ---- 1. operands of the recall GEMM from the fp32 registers; they are the snapshot's pieces as well
        bf16x8 Ahi[KF], Alo[KF];
#pragma unroll
        for (int ks = 0; ks < KF; ks++) {
            const float x8[8] = {hacc[2 * ks][0], hacc[2 * ks][1], hacc[2 * ks][2], hacc[2 * ks][3],
                                 hacc[2 * ks + 1][0], hacc[2 * ks + 1][1], hacc[2 * ks + 1][2], hacc[2 * ks + 1][3]};
            split8(x8, Ahi[ks], Alo[ks]);
        }
        if (tid < C) cidx[LAM + tid] = (int)(aj - ETA + tid);

        // requests of batch b into buffer buf: 1 KB per instruction, lane l fills bytes 16 l ..; a row's 16-byte pieces are
        // XOR-swizzled with the row number, so a lane fetches the piece that belongs in its position
        auto issue = [&](int b, int buf) {
            uint16_t *PBb = pool + buf * BUF, *VBb = PBb + RB * FR;
            const int e0 = b * RB;
#pragma unroll
            for (int it = 0; it < RB * FR / 512 / NW; it++) {
                const int i = w + NW * it, g = 512 * i + 8 * lane, row = g / FR, pt = (g % FR) / DF, slot = (g % DF) >> 3;
                const uint16_t *src = phirow(e0 + row) + pt * DF + ((slot ^ (row & 15)) << 3);
                lds_dma16(src, PBb + 512 * i);
            }
#pragma unroll
            for (int it = 0; it < VPB; it++) {
                const int i = w + NW * it, g = 512 * i + 8 * lane, row = g / DH, slot = (g % DH) >> 3;
                const bf16_t *src = vrow(e0 + row) + ((slot ^ (row & (PR - 1))) << 3);
                lds_dma16(src, VBb + 512 * i);
            }
        };
        if (!SCORED && LAM > 0) {
#pragma unroll
        for (int b = 0; b < NBUF - 1; b++) issue(b, b);   // (lambda + 64 >= 128 candidates: at least NBUF batches)

        // ---- 2. recall error of the candidates, batch by batch
        int buf = 0;
#pragma unroll 1
        for (int b = 0; b < NBATCH; b++) {
            // this wavefront's share of batch b has landed: all but the requests of the batches behind it
            const int ahead = min(NBUF - 2, NBATCH - 1 - b);
            if (NBUF >= 4 && ahead >= 2) __builtin_amdgcn_s_waitcnt(0x0F70 | ((2 * LPB) & 15) | (((2 * LPB) >> 4) << 14));
            else if (NBUF >= 3 && ahead == 1) __builtin_amdgcn_s_waitcnt(0x0F70 | (LPB & 15) | ((LPB >> 4) << 14));
            else __builtin_amdgcn_s_waitcnt(0x0F70);
            lds_barrier();                        // ... and everybody's; the readers of batch b - 1's buffer are done
            if (b + NBUF - 1 < NBATCH) issue(b + NBUF - 1, buf == 0 ? NBUF - 1 : buf - 1);
            const uint16_t *PBb = pool + buf * BUF, *VBb = PBb + RB * FR;
            const int pb = b & 1;
            if (b > 0 && tid < 3 * RB) {          // batch b - 1: the wavefronts' sums over their columns, added in a fixed order
                const int k = tid / RB, r = tid % RB;
                float sum = 0.f;
#pragma unroll
                for (int x = 0; x < NW; x++) sum += part[pb ^ 1][k][x][r];
                tot[k][(b - 1) * RB + r] = sum;
            }
            {   // phi(k).s of the batch's rows: TPR neighbouring lanes share a row
                constexpr int TPR = NTH / RB, NPC = PP / TPR;
                const int r = tid / TPR, sub = tid % TPR;
                float dsum = 0.f;
#pragma unroll
                for (int x = 0; x < NPC; x++) {
                    const int pc = sub + TPR * x, addr = r * FR + ((pc ^ (r & 15)) << 3);
                    const uint4 hi = *reinterpret_cast<const uint4 *>(&PBb[addr]), lo = *reinterpret_cast<const uint4 *>(&PBb[addr + DF]);
                    const float4 s0 = *reinterpret_cast<const float4 *>(&s_l[32 * (pc >> 2) + 4 * (pc & 3)]);
                    const float4 s1 = *reinterpret_cast<const float4 *>(&s_l[32 * (pc >> 2) + 16 + 4 * (pc & 3)]);
                    dsum = fmaf(bf_lo(hi.x) + bf_lo(lo.x), s0.x, dsum); dsum = fmaf(bf_hi(hi.x) + bf_hi(lo.x), s0.y, dsum);
                    dsum = fmaf(bf_lo(hi.y) + bf_lo(lo.y), s0.z, dsum); dsum = fmaf(bf_hi(hi.y) + bf_hi(lo.y), s0.w, dsum);
                    dsum = fmaf(bf_lo(hi.z) + bf_lo(lo.z), s1.x, dsum); dsum = fmaf(bf_hi(hi.z) + bf_hi(lo.z), s1.y, dsum);
                    dsum = fmaf(bf_lo(hi.w) + bf_lo(lo.w), s1.z, dsum); dsum = fmaf(bf_hi(hi.w) + bf_hi(lo.w), s1.w, dsum);
                }
                dsum += dpp_f<0xB1>(dsum); dsum += dpp_f<0x4E>(dsum);
                if (TPR >= 8) dsum += dpp_f<0x141>(dsum);
                if (TPR >= 16) dsum += dpp_f<0x140>(dsum);
                if (sub == 0) dn_l[b * RB + r] = dsum;
            }
            // recall GEMM: A = this wavefront's 16 rows of H^T, B = phi of 16 candidates from LDS; lane (candidate r16,
            // group g4) holds the recall at columns 16 w + 4 g4 + i and pairs it with the candidate's values there
#pragma unroll
            for (int u = 0; u < TB; u++) {
                const uint16_t *rowp = PBb + (16 * u + r16) * FR;
                bf16x8 Bh[KF], Bl[KF];
#pragma unroll
                for (int ks = 0; ks < KF; ks++) {
                    const int addr = ((4 * ks + g4) ^ r16) << 3;
                    Bh[ks] = as_bf16x8(*reinterpret_cast<const uint4 *>(rowp + addr));
                    Bl[ks] = as_bf16x8(*reinterpret_cast<const uint4 *>(rowp + DF + addr));
                }
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};   // the three products of a k-step go into one accumulator: the large one first
#pragma unroll
                for (int ks = 0; ks < KF; ks++) acc = mfma16(Ahi[ks], Bh[ks], acc);
#pragma unroll
                for (int ks = 0; ks < KF; ks++) acc = mfma16(Ahi[ks], Bl[ks], acc);
#pragma unroll
                for (int ks = 0; ks < KF; ks++) acc = mfma16(Alo[ks], Bh[ks], acc);
                const uint2 vv = *reinterpret_cast<const uint2 *>(&VBb[(16 * u + r16) * DH + (((2 * w + (g4 >> 1)) ^ (r16 & (PR - 1))) << 3) + 4 * (g4 & 1)]);
                const float v0 = bf_lo(vv.x), v1 = bf_hi(vv.x), v2 = bf_lo(vv.y), v3 = bf_hi(vv.y);
                float sa = 0.f, sb = 0.f, sc = 0.f;
                sa = fmaf(acc[0], acc[0], sa); sa = fmaf(acc[1], acc[1], sa); sa = fmaf(acc[2], acc[2], sa); sa = fmaf(acc[3], acc[3], sa);
                sb = fmaf(acc[0], v0, sb); sb = fmaf(acc[1], v1, sb); sb = fmaf(acc[2], v2, sb); sb = fmaf(acc[3], v3, sb);
                sc = fmaf(v0, v0, sc); sc = fmaf(v1, v1, sc); sc = fmaf(v2, v2, sc); sc = fmaf(v3, v3, sc);
                const float s3 = grp_sum3(sa, sb, sc);   // lane group g4 holds sum g4
                if (g4 < 3) part[pb][g4][w][16 * u + r16] = s3;
            }
            buf = buf == NBUF - 1 ? 0 : buf + 1;
        }
        lds_barrier();
        if (tid < 3 * RB) {
            const int k = tid / RB, r = tid % RB;
            float sum = 0.f;
#pragma unroll
            for (int x = 0; x < NW; x++) sum += part[(NBATCH - 1) & 1][k][x][r];
            tot[k][(NBATCH - 1) * RB + r] = sum;
        }
        lds_barrier();
        }

        // The snapshot is stored here, behind the batches: the memory counter is in order, so stores issued ahead of the
        // batches' requests would stand between every batch and its wait; from here they drain while the selection runs.
        if (a.want_out) {
            const size_t sj = (size_t)si * a.S + (j - a.jb);
            uint16_t *s16 = reinterpret_cast<uint16_t *>(a.snapH) + sj * (2 * DF * DH);
#pragma unroll
            for (int ks = 0; ks < KF; ks++) {
                // one contiguous 1 KB piece per store: [part][row tile][k-step][lane]
                const int off = ((w * KF + ks) * 64 + lane) << 3;
                *reinterpret_cast<uint4 *>(s16 + off) = __builtin_bit_cast(uint4, Ahi[ks]);
                *reinterpret_cast<uint4 *>(s16 + DF * DH + off) = __builtin_bit_cast(uint4, Alo[ks]);
            }
            for (int x = tid; x < DF / 4; x += NTH) reinterpret_cast<float4 *>(a.snapS + sj * DF)[x] = reinterpret_cast<const float4 *>(s_l)[x];
#pragma unroll
            for (int x = 0; x < NSP; x++)
                if (tid + NTH * x < LAM) a.snapG[sj * LAM + tid + NTH * x] = sprow_ld[x];
        }

        // ---- 3. selection: the 64 candidates with the smallest squared error are folded (order: score descending,
        // token index ascending, the first lambda stay).  The squared error is |P|^2 / (phi.s)^2 - 2 P.v / (phi.s) + |v|^2
        // (recall = 0 while phi.s = 0); the bit pattern of a float >= 0 orders like an integer.
        if (LAM == 0) {
            // no sparse cache: nothing to select, every pair that leaves is folded
            if (tid < C) flist[tid] = tid;
            if (tid == 0) ne_s = 0;
        } else if (SCORED) {
            // given scores (sums of non-negative terms): the cache slots' from the state, the leaving pairs' from the
            // per-token sums of the call (row j C + x of the stream's block: token a0 - eta + j C + x)
            const float *sps = a.st.sp_score + (size_t)si * LAM;
            const float *tsc = a.tok_score + (size_t)si * (ETA + a.T_tokens) + (size_t)j * C;
            for (int e = tid; e < NE; e += NTH) {
                const float sc = e < LAM ? sps[e] : tsc[e - LAM];
                tot[0][e] = sc;
                skey[e] = __float_as_uint(sc) & 0x7FFFFFFFu;
            }
        } else {
        for (int e = tid; e < NE; e += NTH) {
            const float dn = dn_l[e], rd = dn > 0.f ? __builtin_amdgcn_rcpf(dn) : 0.f;
            const float sq = fmaxf(fmaf(rd * rd, tot[0][e], fmaf(-2.0f * rd, tot[1][e], tot[2][e])), 0.f);
            skey[e] = __float_as_uint(sq) & 0x7FFFFFFFu;
        }
        }
        lds_barrier();
        if (w == 0 && LAM > 0) {
            // One wavefront holds all scores (up to 17 per lane) and builds the 64th smallest bit by bit: a trial value is
            // kept while fewer than 64 scores lie below it.  Scores equal to the threshold are folded too if that makes
            // exactly 64; otherwise (exact ties across the cut) the same search over their token indices picks the
            // largest ones.  The lists follow from the fold predicate by ballots (candidate order kept).
            uint32_t sb[NKMAX]; int ix[NKMAX];
#pragma unroll
            for (int x = 0; x < NKMAX; x++) {
                sb[x] = 0xFFFFFFFFu; ix[x] = 0;
                if (x < nk) { sb[x] = skey[64 * x + lane]; ix[x] = cidx[64 * x + lane]; }
            }
            uint32_t thr = 0, cut = 0;   // cut != 0: exactly 64 scores lie below it
#pragma unroll 1
            for (int bit = 30; bit >= 0 && cut == 0; bit--) {
                const uint32_t trial = thr | (1u << bit);
                int c = 0;
#pragma unroll
                for (int x = 0; x < NKMAX; x++) if (x < nk) c += __popcll(__ballot(sb[x] < trial));
                if (c == C) cut = trial;
                if (c < C) thr = trial;
            }
            int n_lt = 0, n_eq = 0;
            if (cut != 0) { thr = cut; n_lt = C; }
            else {
#pragma unroll
                for (int x = 0; x < NKMAX; x++)
                    if (x < nk) { n_lt += __popcll(__ballot(sb[x] < thr)); n_eq += __popcll(__ballot(sb[x] == thr)); }
            }
            const int need = C - n_lt;      // ties at the threshold to fold: 0 after an early stop, else 1 <= need <= n_eq
            uint32_t imin = need == 0 ? 0xFFFFFFFFu : 0u;   // ties are folded from token index imin upwards
            if (need != 0 && n_eq != need) {
#pragma unroll 1
                for (int bit = 30; bit >= 0; bit--) {
                    const uint32_t trial = imin | (1u << bit);
                    int c = 0;
#pragma unroll
                    for (int x = 0; x < NKMAX; x++) if (x < nk) c += __popcll(__ballot(sb[x] == thr && (uint32_t)ix[x] >= trial));
                    if (c >= need) imin = trial;
                }
            }
            int nf = 0, nen = 0, nlv = 0;
            const unsigned long long below = (1ull << lane) - 1ull;
#pragma unroll
            for (int x = 0; x < NKMAX; x++) {
                if (x < nk) {
                    const int e = 64 * x + lane;
                    const bool fo = sb[x] < thr || (sb[x] == thr && (uint32_t)ix[x] >= imin);
                    const bool en = !fo && e >= LAM, lv = fo && e < LAM;
                    const unsigned long long mf = __ballot(fo), me = __ballot(en), ml = __ballot(lv);
                    if (fo) flist[nf + __popcll(mf & below)] = e;
                    if (en) ecand[nen + __popcll(me & below)] = e;
                    if (lv) eslot[nlv + __popcll(ml & below)] = e;
                    nf += __popcll(mf); nen += __popcll(me); nlv += __popcll(ml);
                }
            }
            if (lane == 0) ne_s = nen;
        }
        lds_barrier();
        const int ne = ne_s;   // exactly 64 are folded, so entrants and leavers pair up

        // ---- 4. fold: H[f][c] += sum_e phi_e[f] v_e[c], s[f] += sum_e phi_e[f] over the 64 folded pairs, whose rows are
        // gathered into LDS ([pair][part][position] and [pair][column], 16-byte pieces XOR-swizzled with bits of the pair number: fswz, vswz2)
        uint16_t *FP = pool, *FV = pool + C * FR;
#pragma unroll
        for (int it = 0; it < C * FR / 512 / NW; it++) {
            const int i = w + NW * it, g = 512 * i + 8 * lane, row = g / FR, pt = (g % FR) / DF, slot = (g % DF) >> 3;
            const uint16_t *src = phirow(flist[row]) + pt * DF + ((slot ^ fswz(row)) << 3);
            lds_dma16(src, FP + 512 * i);
        }
#pragma unroll
        for (int it = 0; it < C * DH / 512 / NW; it++) {
            const int i = w + NW * it, g = 512 * i + 8 * lane, row = g / DH, slot = (g % DH) >> 3;
            const bf16_t *src = vrow(flist[row]) + ((slot ^ vswz2<PR>(row)) << 3);
            lds_dma16(src, FV + 512 * i);
        }
        // compaction, first half: the entrants' rows (keys, values, features) are requested now and stored after the fold
        constexpr int CIT = C * 2 * PR / NTH, PIT = C * (FR / 8) / NTH;
        uint4 cp[CIT], fe[PIT];
#pragma unroll
        for (int it = 0; it < CIT; it++) {
            const int o = tid + NTH * it;
            cp[it] = make_uint4(0, 0, 0, 0);
            if (o < ne * 2 * PR) {
                const int x = o / (2 * PR), rem = o % (2 * PR), e = ecand[x];
                cp[it] = reinterpret_cast<const uint4 *>((rem >= PR) ? vrow(e) : krow(e))[rem % PR];
            }
        }
#pragma unroll
        for (int it = 0; it < PIT; it++) {
            const int o = tid + NTH * it;
            fe[it] = make_uint4(0, 0, 0, 0);
            if (o < ne * (FR / 8)) fe[it] = reinterpret_cast<const uint4 *>(phirow(ecand[o / (FR / 8)]))[o % (FR / 8)];
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        lds_barrier();
        // contraction slots of lane group g4 in k-step kst: pairs 32 kst + 4 g4 + 0..3, then + 16 (the order in which the
        // transposing read delivers them, the same for both operands)
#pragma unroll
        for (int kst = 0; kst < 2; kst++) {
            const int t0 = 32 * kst + 4 * g4 + (r16 >> 2), t15 = fswz(t0);
            // B: values, column 16 w + r16: lane i of a group points at pair t0's four columns 16 w + 4 (i % 4) ..
            const uint16_t *vb = FV + t0 * DH + (((2 * w + ((r16 & 3) >> 1)) ^ vswz2<PR>(t0)) << 3) + 4 * (r16 & 1);
            const bf16x4 b0 = tr_read(vb), b1 = tr_read(vb + 16 * DH);
            const bf16x8 Bv = __builtin_shufflevector(b0, b1, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
            for (int mt = 0; mt < NMT; mt++) {
                // A: phi^T, row f = 16 mt + r of the tile from position 32 (mt / 2) + 8 (r / 4) + 4 (mt % 2) + r % 4, i.e.
                // 16-byte piece 4 (mt / 2) + r / 4 of the row (stored at that piece ^ fswz(pair)), its half mt % 2
                const int off = (((4 * (mt >> 1) + (r16 & 3)) ^ t15) << 3) + 4 * (mt & 1);
#pragma unroll
                for (int pt = 0; pt < 2; pt++) {
                    const uint16_t *pa = FP + pt * DF + off;
                    const bf16x4 a0v = tr_read(pa + t0 * FR), a1v = tr_read(pa + (t0 + 16) * FR);
                    const bf16x8 Av = __builtin_shufflevector(a0v, a1v, 0, 1, 2, 3, 4, 5, 6, 7);
                    hacc[mt] = mfma16(Av, Bv, hacc[mt]);
                }
            }
        }
        {   // s: the same product with a column of ones in place of the values, feature tiles w, w + NW, ... by wavefront w
            const uint32_t one2 = 0x3F803F80u;
            const bf16x8 Bones = as_bf16x8(make_uint4(one2, one2, one2, one2));
#pragma unroll
            for (int x = 0; x < NMT / NW; x++) {
                const int mt = w + NW * x;
                f32x4 sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kst = 0; kst < 2; kst++) {
                    const int t0 = 32 * kst + 4 * g4 + (r16 >> 2), t15 = fswz(t0);
                    const int off = (((4 * (mt >> 1) + (r16 & 3)) ^ t15) << 3) + 4 * (mt & 1);
#pragma unroll
                    for (int pt = 0; pt < 2; pt++) {
                        const uint16_t *pa = FP + pt * DF + off;
                        const bf16x4 a0v = tr_read(pa + t0 * FR), a1v = tr_read(pa + (t0 + 16) * FR);
                        const bf16x8 Av = __builtin_shufflevector(a0v, a1v, 0, 1, 2, 3, 4, 5, 6, 7);
                        sacc = mfma16(Av, Bones, sacc);
                    }
                }
                if (r16 == 0) {   // column 0 of the result tile: features 16 mt + 4 g4 + 0..3
                    float4 *sp = reinterpret_cast<float4 *>(&s_l[16 * mt + 4 * g4]);
                    float4 sv = *sp;
                    sv.x += sacc[0]; sv.y += sacc[1]; sv.z += sacc[2]; sv.w += sacc[3];
                    *sp = sv;
                }
            }
        }
        // ---- 5. compaction, second half: entrants take the leavers' slots (rows of the state, features, indices)
#pragma unroll
        for (int it = 0; it < CIT; it++) {
            const int o = tid + NTH * it;
            if (o < ne * 2 * PR) {
                const int x = o / (2 * PR), rem = o % (2 * PR);
                bf16_t *dst = ((rem >= PR) ? sp_v : sp_k) + (size_t)eslot[x] * DH;
                reinterpret_cast<uint4 *>(dst)[rem % PR] = cp[it];
            }
        }
#pragma unroll
        for (int it = 0; it < PIT; it++) {
            const int o = tid + NTH * it;
            if (o < ne * (FR / 8)) reinterpret_cast<uint4 *>(phiE + (size_t)eslot[o / (FR / 8)] * FR)[o % (FR / 8)] = fe[it];
        }
        for (int x = tid; x < ne; x += NTH) {
            const int e = ecand[x], sl = eslot[x];
            const int ti = cidx[e];
            sp_idx[sl] = ti;
            cidx[sl] = ti;
            sp_row[sl] = vrow_l + (e - LAM);
            if (SCORED) a.st.sp_score[(size_t)si * LAM + sl] = tot[0][e];
        }
        __syncthreads();   // (workgroup scope is enough: only this workgroup reads the stream's memories before the kernel ends)
        if (a.sel_trace) {
            int32_t *tr = a.sel_trace + ((size_t)si * a.n_chunks + j) * LAM;
            for (int sl = tid; sl < LAM; sl += NTH) tr[sl] = cidx[sl];
        }
    }
    if (started) {
        float *hrow = Hg + (size_t)(16 * w0 + (tid0 & 15)) * DF + 4 * ((tid0 & 63) >> 4);
#pragma unroll
        for (int mt = 0; mt < NMT; mt++) *reinterpret_cast<f32x4 *>(hrow + 16 * mt) = hacc[mt];
        for (int x = tid0; x < DF; x += NTH) sg[x] = s_l[x];
    }
    if (tid0 == 0) a.next_j[si] = j;
}

// ---------------------------------------------------------------------------------------------
// Outputs of a generation step from the memories as the step's update left them (Sec. 3.1 eq. lola_output with the
// shared normaliser: softmax part over the sparse cache and the window, linear part phi(q)^T H, phi(q)^T s), for any
// window and sparse budget with at most NKMAX keys, 128 or 256 features and up to eight query heads per kv head.  One
// workgroup per stream, four wavefronts:
//   1. logits Q K^T on MFMA (A = the group's queries, B = 16 keys straight from memory), tiles dealt round-robin;
//   2. phi of query w by wavefront w (projection on MFMA with the query in every column);
//   3. m = max(0, max logit) and the weights e^(l - m) per query, left in LDS as bf16 high + low parts;
//   4. weights x values on MFMA: each wavefront stages blocks of 32 value rows in its own LDS tile (direct loads, two
//      tiles in flight) and reads them as B operand through the transposing LDS read;
//   5. phi(q)^T H on MFMA with H^T read from memory and split into bf16 high + low parts on the way;
//   6. y = (sum w v + e^(-m) phi(q)^T H) / (sum w + e^(-m) phi(q)^T s).
// With a query-dependent score (Sec. 4 / appendix "scoring ablation") the step's queries also add their terms to the
// sums of the pairs in the window (between 2 and 3: phi of the window keys on MFMA, phi(q) phi(k)^T against the
// queries' features in LDS, the logits still in LDS as fp32), as the shape-generic step does.
template <typename TO>
struct StepOutArgs {
    State<bf16_t> st;
    const bf16_t *q, *Wq, *Wk;
    TO *out;
    int Hq, Hkv, g, lam, eta, phi_kind, hide, score_kind;
    float scale;
    float *part;          // SPLIT: partial results [stream][part][G * DH + 2 * G] (scratch)
    int part_stride;      // floats per stream in `part`
    int nlin;             // SPLIT: parts that take the linear part (1: all query heads; g: one query head each)
};

constexpr int STEP_OUT_NKMAX = 3072;
constexpr int STEP_OUT_PARTS_MAX = 16;

// G = 4 or 8: query rows the kernel is built for (query heads per kv head <= G); the logits of all of them stay in
// LDS, so the key limit is STEP_OUT_NKMAX * 4 / G.  Lane (column, group g4) of an MFMA result holds rows 4 g4 + i: the
// queries sit in the lane groups g4 < G / 4.
// SPLIT (few streams: one workgroup per stream is bounded by its compute unit's share of the memory system): grid
// (streams, parts); the first nlin parts compute the linear part (sections 2 and 5: of all query heads, or of query head
// `part` each - W_q is read per head, H^T by all of them) and no keys, the others take the key blocks of 32 in equal
// shares; each leaves (sum w v, m, sum w) of its share in `part` - the linear part as a share with m = 0, rows of other
// heads zero - and step_out_combine_kernel adds the shares up under the common maximum.
template <int DH, int DF, typename TO, int G, bool SPLIT = false>
__global__ __launch_bounds__(256) void step_out_wide_kernel(StepOutArgs<TO> a) {
    constexpr int M = DF / 2, KS = DH / 32, NZT = M / 16, KF = DF / 32, NCT = DH / 16, PR = DH / 8, NKMAX = STEP_OUT_NKMAX * 4 / G;
    static_assert(G == 4 || G == 8, "query rows");
    __shared__ __attribute__((aligned(16))) float lg[G][NKMAX];              // logits; then per 4 keys: 4 high parts, 4 low parts
    __shared__ __attribute__((aligned(16))) uint16_t VS[4][2][32 * DH];      // per wavefront: two blocks of 32 value rows
    __shared__ __attribute__((aligned(16))) uint16_t PQ[G][2][DF];           // phi(q), operand order, high / low parts
    __shared__ __attribute__((aligned(16))) float outp[4][G][DH];            // per wavefront: its keys' share of sum w v
    __shared__ __attribute__((aligned(16))) float lin_l[G][DH];
    __shared__ float m_l[G], psum_l[G], denq_l[G];

    const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, r16 = lane & 15, g4 = lane >> 4;
    const int si = blockIdx.x, b = si / a.Hkv, h = si - b * a.Hkv, g = a.g, LAM = a.lam, ETA = a.eta;
    const int64_t tok = a.st.n_tokens[si];                    // tokens consumed, this step's included
    const int spc = a.st.sp_count[si];
    const int wn = (int)min((int64_t)ETA, tok), nk = spc + wn, KPAD = (nk + 31) & ~31;
    // this workgroup's key blocks of 32: [kb0, kb1)
    const int prt = SPLIT ? blockIdx.y : 0, nlin = SPLIT ? a.nlin : 1, nkp = SPLIT ? gridDim.y - nlin : 1;
    const bool linear = !SPLIT || prt < nlin;
    const int kb0 = !SPLIT ? 0 : linear ? 0 : (int)((int64_t)(KPAD / 32) * (prt - nlin) / nkp);
    const int kb1 = !SPLIT ? KPAD / 32 : linear ? 0 : (int)((int64_t)(KPAD / 32) * (prt - nlin + 1) / nkp);
    // query heads whose features this workgroup makes: [q0, q1), dealt to the wavefronts from q0 on
    const int q0 = SPLIT && nlin > 1 ? prt : 0, q1 = !linear ? 0 : SPLIT && nlin > 1 ? prt + 1 : g;
    const bf16_t *sp_k = a.st.sp_k + (size_t)si * LAM * DH, *sp_v = a.st.sp_v + (size_t)si * LAM * DH;
    const bf16_t *win_k = a.st.win_k + (size_t)si * ETA * DH, *win_v = a.st.win_v + (size_t)si * ETA * DH;
    const float *Hg = a.st.H + (size_t)si * DF * DH, *sg = a.st.s + (size_t)si * DF;
    const bf16_t *qg = a.q + ((size_t)b * a.Hq + (size_t)h * g) * DH;   // g consecutive query rows

    if (tid < G) { m_l[tid] = 0.f; psum_l[tid] = 0.f; denq_l[tid] = 0.f; }
    for (int x = tid; x < G * 2 * DF / 8; x += 256) reinterpret_cast<uint4 *>(PQ)[x] = make_uint4(0, 0, 0, 0);
    __syncthreads();

    // ---- 1. logits
    {
        bf16x8 AQ[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ks++) AQ[ks] = r16 < g ? ld_bf16x8(qg + (size_t)r16 * DH + 32 * ks + 8 * g4) : zero_bf16x8();
        // four key tiles per pass, their rows requested together: one tile at a time, every tile cost a round trip
        constexpr int UT = 4;
#pragma unroll 1
        for (int t0 = 2 * kb0 + w; t0 < 2 * kb1; t0 += 4 * UT) {
            bf16x8 KB[UT][KS];
#pragma unroll
            for (int u = 0; u < UT; u++) {
                const int key = 16 * (t0 + 4 * u) + r16;
                const bf16_t *kr = key < spc ? sp_k + (size_t)key * DH : win_k + (size_t)(key < nk ? key - spc : 0) * DH;
#pragma unroll
                for (int ks = 0; ks < KS; ks++) KB[u][ks] = ld_bf16x8(kr + 32 * ks + 8 * g4);   // (tiles past the last one: any readable row)
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < UT; u++) {
                const int t = t0 + 4 * u, key = 16 * t + r16;
                if (t < 2 * kb1) {
                    const bool valid = key < nk;
                    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < KS; ks++) acc = mfma16(AQ[ks], KB[u][ks], acc);
                    if (g4 < G / 4) {   // rows 4 g4 + i of the tile: the queries
                        const bool hidden = !valid || ((a.hide & 2) && key < spc);   // restricted query: the sparse cache is not read
#pragma unroll
                        for (int i = 0; i < 4; i++) lg[4 * g4 + i][key] = hidden ? -INFINITY : acc[i] * a.scale;
                    }
                }
            }
        }
    }
    // ---- 2. phi of queries w, w + 4, ... (Sec. 2.3 eq. feature_map) and phi(q).s
#pragma unroll 1
    for (int qi = q0 + w; qi < q1; qi += 4) {
        const bf16_t *Wq = a.Wq + ((size_t)h * g + qi) * M * DH;
        bf16x8 BQ[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ks++) BQ[ks] = ld_bf16x8(qg + (size_t)qi * DH + 32 * ks + 8 * g4);
        // all of W_q's operands are requested before the first product (one wavefront per SIMD has the registers:
        // requested where they are used, they arrive a few at a time, one round trip after the other)
        bf16x8 WQ[NZT][KS];
#pragma unroll
        for (int mt = 0; mt < NZT; mt++)
#pragma unroll
            for (int ks = 0; ks < KS; ks++) WQ[mt][ks] = ld_bf16x8(Wq + (size_t)(16 * mt + r16) * DH + 32 * ks + 8 * g4);
        __builtin_amdgcn_sched_barrier(0);
        f32x4 zt[NZT];
#pragma unroll
        for (int mt = 0; mt < NZT; mt++) {
            zt[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ks++) zt[mt] = mfma16(WQ[mt][ks], BQ[ks], zt[mt]);
        }
        float pp[4 * NZT], pn[4 * NZT];
        phi_from_z_tiles<NZT>(zt, a.phi_kind, pp, pn);
        float dn = 0.f;
#pragma unroll
        for (int mt = 0; mt < NZT; mt++) {
            const float4 sp4 = *reinterpret_cast<const float4 *>(sg + 16 * mt + 4 * g4);
            const float4 sn4 = *reinterpret_cast<const float4 *>(sg + M + 16 * mt + 4 * g4);
            dn = fmaf(pp[4 * mt], sp4.x, dn); dn = fmaf(pp[4 * mt + 1], sp4.y, dn);
            dn = fmaf(pp[4 * mt + 2], sp4.z, dn); dn = fmaf(pp[4 * mt + 3], sp4.w, dn);
            dn = fmaf(pn[4 * mt], sn4.x, dn); dn = fmaf(pn[4 * mt + 1], sn4.y, dn);
            dn = fmaf(pn[4 * mt + 2], sn4.z, dn); dn = fmaf(pn[4 * mt + 3], sn4.w, dn);
        }
        dn = grp_sum(dn);
        if (lane == 0) denq_l[qi] = dn;
        if (r16 == 0) {   // every column holds the same query: column 0 stores
#pragma unroll
            for (int ks = 0; ks < KF / 2; ks++) {
                bf16x8 hi, lo;
                split8(&pp[8 * ks], hi, lo);
                *reinterpret_cast<uint4 *>(&PQ[qi][0][(4 * ks + g4) << 3]) = __builtin_bit_cast(uint4, hi);
                *reinterpret_cast<uint4 *>(&PQ[qi][1][(4 * ks + g4) << 3]) = __builtin_bit_cast(uint4, lo);
                split8(&pn[8 * ks], hi, lo);
                *reinterpret_cast<uint4 *>(&PQ[qi][0][(4 * (KF / 2 + ks) + g4) << 3]) = __builtin_bit_cast(uint4, hi);
                *reinterpret_cast<uint4 *>(&PQ[qi][1][(4 * (KF / 2 + ks) + g4) << 3]) = __builtin_bit_cast(uint4, lo);
            }
        }
    }
    __syncthreads();
    if (a.score_kind) {
        const bf16_t *Wk = a.Wk + (size_t)h * M * DH;
        float *wsc = a.st.win_score + (size_t)si * ETA;
        bf16x8 Ahi[KF], Alo[KF];
#pragma unroll
        for (int ks = 0; ks < KF; ks++) {
            Ahi[ks] = r16 < G ? as_bf16x8(*reinterpret_cast<const uint4 *>(&PQ[r16][0][(4 * ks + g4) << 3])) : zero_bf16x8();
            Alo[ks] = r16 < G ? as_bf16x8(*reinterpret_cast<const uint4 *>(&PQ[r16][1][(4 * ks + g4) << 3])) : zero_bf16x8();
        }
        for (int t = w; t < (wn + 15) / 16; t += 4) {
            const int kk = 16 * t + r16;       // ring slot
            const bool valid = kk < wn;
            const bf16_t *kr = win_k + (size_t)(valid ? kk : 0) * DH;
            bf16x8 BK[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ks++) BK[ks] = ld_bf16x8(kr + 32 * ks + 8 * g4);
            f32x4 zt[NZT];
#pragma unroll
            for (int mt = 0; mt < NZT; mt++) {
                zt[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ks++)
                    zt[mt] = mfma16(ld_bf16x8(Wk + (size_t)(16 * mt + r16) * DH + 32 * ks + 8 * g4), BK[ks], zt[mt]);
            }
            float pp[4 * NZT], pn[4 * NZT];
            phi_from_z_tiles<NZT>(zt, a.phi_kind, pp, pn);
            f32x4 acc = {0.f, 0.f, 0.f, 0.f}, acc2 = {0.f, 0.f, 0.f, 0.f}, acc3 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KF; ks++) {
                bf16x8 Bh, Bl;
                split8(ks < KF / 2 ? &pp[8 * ks] : &pn[8 * (ks - KF / 2)], Bh, Bl);
                acc = mfma16(Ahi[ks], Bh, acc);
                acc2 = mfma16(Ahi[ks], Bl, acc2);
                acc3 = mfma16(Alo[ks], Bh, acc3);
            }
            {   // rows 4 g4 + i of the tile: the queries; column: this lane's key
                float add = 0.f;
#pragma unroll
                for (int i = 0; i < 4; i++)
                    if (valid && 4 * g4 + i < g) add += generic::query_term(a.score_kind, lg[4 * g4 + i][spc + kk], acc[i] + (acc2[i] + acc3[i]));
                add = grp_sum(add);
                if (g4 == 0 && valid) wsc[kk] += add;
            }
        }
        __syncthreads();   // the logits are overwritten next
    }
    // the first block of value rows of section 4 is requested here: it lands while the weights are computed (each
    // wavefront's VS tile is its own, and nothing reads it before section 4)
    auto stage = [&](int kb, int buf) {
        // 1 KB per instruction = 2048 / DH rows; lane l fills bytes 16 l ..: the row's piece (l % PR) ^ vswz2(row)
#pragma unroll
        for (int i = 0; i < 32 * DH / 512; i++) {
            const int row = (512 * i + 8 * lane) / DH, slot = lane % PR;
            int key = 32 * kb + row;
            if (key >= nk) key = 0;   // weight 0: any readable row will do
            const bf16_t *vr = key < spc ? sp_v + (size_t)key * DH : win_v + (size_t)(key - spc) * DH;
            lds_dma16(vr + ((slot ^ vswz2<PR>(row)) << 3), &VS[w][buf][512 * i]);   // (inline assembly: the reads of the other buffer below do not wait for it)
        }
    };
    if (kb0 + w < kb1) stage(kb0 + w, 0);
    // and so are this wavefront's rows of H^T for section 5 (one wavefront per SIMD has the registers to hold them)
    float4 hv[NCT / 4][KF][2];
#pragma unroll
    for (int x = 0; x < NCT / 4; x++)
#pragma unroll
        for (int ks = 0; ks < KF; ks++) hv[x][ks][0] = hv[x][ks][1] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (linear) {
#pragma unroll
        for (int x = 0; x < NCT / 4; x++) {
            const float *hrow = Hg + (size_t)(16 * (w + 4 * x) + r16) * DF + 4 * g4;
#pragma unroll
            for (int ks = 0; ks < KF; ks++) {
                hv[x][ks][0] = *reinterpret_cast<const float4 *>(hrow + 32 * ks);
                hv[x][ks][1] = *reinterpret_cast<const float4 *>(hrow + 32 * ks + 16);
            }
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    // ---- 3. weights of queries w, w + 4, ...: m = max(0, max logit) (the linear terms carry weight e^(-m) <= 1)
#pragma unroll 1
    for (int qi = w; qi < g; qi += 4) {
        float mx = 0.f;
        for (int x = 8 * kb0 + lane; x < 8 * kb1; x += 64) {
            const float4 l4 = reinterpret_cast<const float4 *>(lg[qi])[x];
            mx = fmaxf(mx, fmaxf(fmaxf(l4.x, l4.y), fmaxf(l4.z, l4.w)));
        }
        mx = wmax(mx);
        float ps = 0.f;
        for (int x = 8 * kb0 + lane; x < 8 * kb1; x += 64) {
            const float4 l4 = reinterpret_cast<const float4 *>(lg[qi])[x];
            const float p[4] = {fexp2((l4.x - mx) * LOG2E), fexp2((l4.y - mx) * LOG2E), fexp2((l4.z - mx) * LOG2E), fexp2((l4.w - mx) * LOG2E)};
            uint32_t hi[2], lo[2];
#pragma unroll
            for (int y = 0; y < 2; y++) {
                const uint16_t h0 = f32_to_bf16_bits(p[2 * y]), h1 = f32_to_bf16_bits(p[2 * y + 1]);
                const float r0 = p[2 * y] - __uint_as_float((uint32_t)h0 << 16), r1 = p[2 * y + 1] - __uint_as_float((uint32_t)h1 << 16);
                hi[y] = (uint32_t)h0 | ((uint32_t)h1 << 16);
                lo[y] = (uint32_t)f32_to_bf16_bits(r0) | ((uint32_t)f32_to_bf16_bits(r1) << 16);
                // (the sum runs over the weights as the MFMAs will see them)
                ps += (__uint_as_float((uint32_t)h0 << 16) + __uint_as_float((uint32_t)f32_to_bf16_bits(r0) << 16)) +
                      (__uint_as_float((uint32_t)h1 << 16) + __uint_as_float((uint32_t)f32_to_bf16_bits(r1) << 16));
            }
            reinterpret_cast<uint4 *>(lg[qi])[x] = make_uint4(hi[0], hi[1], lo[0], lo[1]);
        }
        ps = wsum(ps);
        if (lane == 0) { m_l[qi] = mx; psum_l[qi] = ps; }
    }
    __syncthreads();
    // ---- 4. sum w v: key blocks of 32 dealt round-robin; A = weights (rows = queries), B = values through the
    // transposing read (contraction slots of lane group g4: keys 4 g4 + 0..3, then + 16)
    {
        f32x4 acc[NCT];
#pragma unroll
        for (int ct = 0; ct < NCT; ct++) acc[ct] = (f32x4){0.f, 0.f, 0.f, 0.f};
        int buf = 0;
#pragma unroll 1
        for (int kb = kb0 + w; kb < kb1; kb += 4) {
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the block has landed (only this wavefront reads it)
            asm volatile("" ::: "memory");
            if (kb + 4 < kb1) stage(kb + 4, buf ^ 1);
            bf16x8 Ahi = zero_bf16x8(), Alo = zero_bf16x8();
            if (r16 < g) {
                const uint4 u0 = reinterpret_cast<const uint4 *>(lg[r16])[8 * kb + g4], u1 = reinterpret_cast<const uint4 *>(lg[r16])[8 * kb + 4 + g4];
                Ahi = as_bf16x8(make_uint4(u0.x, u0.y, u1.x, u1.y));
                Alo = as_bf16x8(make_uint4(u0.z, u0.w, u1.z, u1.w));
            }
            const int t0 = 4 * g4 + (r16 >> 2);
            const uint16_t *vb = &VS[w][buf][t0 * DH + 4 * (r16 & 1)];
#pragma unroll
            for (int ct = 0; ct < NCT; ct++) {
                const int pc = ((2 * ct + ((r16 & 3) >> 1)) ^ vswz2<PR>(t0)) << 3;
                const bf16x4 b0 = tr_read(vb + pc), b1 = tr_read(vb + 16 * DH + pc);
                const bf16x8 Bv = __builtin_shufflevector(b0, b1, 0, 1, 2, 3, 4, 5, 6, 7);
                acc[ct] = mfma16(Ahi, Bv, acc[ct]);
                acc[ct] = mfma16(Alo, Bv, acc[ct]);
            }
            buf ^= 1;
        }
        if (g4 < G / 4) {   // lane (column r16 of tile ct): rows 4 g4 + i = the queries
#pragma unroll
            for (int ct = 0; ct < NCT; ct++)
#pragma unroll
                for (int i = 0; i < 4; i++) outp[w][4 * g4 + i][16 * ct + r16] = acc[ct][i];
        }
    }
    // ---- 5. phi(q)^T H: column tiles w, w + 4, ...; A = phi(q) (rows = queries), B = 16 rows of H^T
    if (linear) {
        bf16x8 Ahi[KF], Alo[KF];
#pragma unroll
        for (int ks = 0; ks < KF; ks++) {
            Ahi[ks] = r16 < G ? as_bf16x8(*reinterpret_cast<const uint4 *>(&PQ[r16][0][(4 * ks + g4) << 3])) : zero_bf16x8();
            Alo[ks] = r16 < G ? as_bf16x8(*reinterpret_cast<const uint4 *>(&PQ[r16][1][(4 * ks + g4) << 3])) : zero_bf16x8();
        }
#pragma unroll
        for (int x = 0; x < NCT / 4; x++) {
            const int ct = w + 4 * x;
            f32x4 acc = {0.f, 0.f, 0.f, 0.f}, acc2 = {0.f, 0.f, 0.f, 0.f}, acc3 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KF; ks++) {
                const float4 h0 = hv[x][ks][0], h1 = hv[x][ks][1];
                const float x8[8] = {h0.x, h0.y, h0.z, h0.w, h1.x, h1.y, h1.z, h1.w};
                bf16x8 Bh, Bl;
                split8(x8, Bh, Bl);
                acc = mfma16(Ahi[ks], Bh, acc);
                acc2 = mfma16(Ahi[ks], Bl, acc2);
                acc3 = mfma16(Alo[ks], Bh, acc3);
            }
            if (g4 < G / 4) {
#pragma unroll
                for (int i = 0; i < 4; i++) lin_l[4 * g4 + i][16 * ct + r16] = acc[i] + (acc2[i] + acc3[i]);
            }
        }
    }
    __syncthreads();
    // ---- 6. outputs
    if (SPLIT) {   // this part's share: numerators, then (m, sum of weights) per query; part 0: the linear part, m = 0
        float *ps = a.part + (size_t)si * a.part_stride + (size_t)prt * (G * DH + 2 * G);
        const float elin = (a.hide & 1) ? 0.f : 1.f;   // restricted query: the hidden state is not read
        for (int o = tid; o < g * DH; o += 256) {
            const int qi = o / DH, c = o - qi * DH;
            ps[o] = linear ? elin * lin_l[qi][c] : (outp[0][qi][c] + outp[1][qi][c]) + (outp[2][qi][c] + outp[3][qi][c]);
        }
        if (tid < g) {
            ps[G * DH + 2 * tid] = linear ? 0.f : m_l[tid];
            ps[G * DH + 2 * tid + 1] = linear ? elin * denq_l[tid] : psum_l[tid];
        }
        return;
    }
    for (int o = tid; o < g * DH; o += 256) {
        const int qi = o / DH, c = o - qi * DH;
        const float elin = (a.hide & 1) ? 0.f : fexp2(-m_l[qi] * LOG2E);   // restricted query: the hidden state is not read
        const float num = (outp[0][qi][c] + outp[1][qi][c]) + (outp[2][qi][c] + outp[3][qi][c]) + elin * lin_l[qi][c];
        const float val = num / (psum_l[qi] + elin * denq_l[qi]);
        stf(a.out, ((size_t)b * a.Hq + (size_t)h * g + qi) * DH + c, val);
    }
}

// Sum of the shares left by step_out_wide_kernel<..., SPLIT> (softmax part per key range and the linear part; Sec. 3.1
// eq. lola_output with the shared normaliser): with M = max over the shares' m,
// y = sum_p e^(m_p - M) num_p / sum_p e^(m_p - M) den_p.  One workgroup per stream, one thread per (query, column).
template <typename TO>
__global__ __launch_bounds__(256) void step_out_combine_kernel(StepOutArgs<TO> a, int G, int DH, int nparts) {
    const int si = blockIdx.x, b = si / a.Hkv, h = si - b * a.Hkv, g = a.g, PS = G * DH + 2 * G;
    const float *ps = a.part + (size_t)si * a.part_stride;
    for (int o = threadIdx.x; o < g * DH; o += 256) {
        const int qi = o / DH;
        // (all shares requested before the first is used: one round trip instead of one per share)
        float mp[STEP_OUT_PARTS_MAX], lp[STEP_OUT_PARTS_MAX], vp[STEP_OUT_PARTS_MAX];
#pragma unroll
        for (int p = 0; p < STEP_OUT_PARTS_MAX; p++) {
            const int pc = p < nparts ? p : 0;
            mp[p] = ps[(size_t)pc * PS + G * DH + 2 * qi];
            lp[p] = ps[(size_t)pc * PS + G * DH + 2 * qi + 1];
            vp[p] = ps[(size_t)pc * PS + o];
        }
        float mx = 0.f;
#pragma unroll
        for (int p = 0; p < STEP_OUT_PARTS_MAX; p++)
            if (p < nparts) mx = fmaxf(mx, mp[p]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int p = 0; p < STEP_OUT_PARTS_MAX; p++)
            if (p < nparts) {
                const float sc = fexp2((mp[p] - mx) * LOG2E);
                num = fmaf(sc, vp[p], num);
                den = fmaf(sc, lp[p], den);
            }
        stf(a.out, ((size_t)b * a.Hq + (size_t)h * g + qi) * DH + o - qi * DH, num / den);
    }
}

// ---------------------------------------------------------------------------------------------
// Update of the memories in a generation step in steady state (window and cache full; Sec. 3.1 "Method Overview" and
// Sec. 3.2 eq. sre: the new pair enters the window, the pair it displaces and the lambda cached pairs are scored with the
// state as it stands, the one with the smallest self-recall error is folded into H and s, the others stay cached), for
// sparse budgets in multiples of 64 and 128 or 256 features.  One workgroup of eight wavefronts per stream:
//   1. H^T is read once: every thread keeps its 16-byte-piece pairs as fp32 (they are rewritten by the fold) and leaves
//      them in LDS split into bf16 high + low parts, in the A-operand order of the recall GEMM;
//   2. the cache's candidates are dealt to the wavefronts round-robin, two tiles of 16 per pass: phi of the keys on MFMA
//      (Sec. 2.3 eq. feature_map), kept as B operand, recall against all of H^T from LDS, || recall - v || per candidate
//      to LDS; the leaving pair, which would be a tile (and a round) of its own, is scored from the fp32 registers
//      instead: its projections are computed one tile of 16 features per wavefront during start-up, wavefront 7 turns
//      them into phi, and after the tiles every thread multiplies its pieces of H^T with it;
//   3. wavefront 0: arg-min (ties: the larger token index goes), phi of the folded pair as fp32 (W_k requested ahead);
//   4. rank-1 fold on the registers, H^T and s written back; the leaving pair takes the folded pair's slot unless it is
//      the one folded; the new pair takes the ring slot; the token counter advances.
// Streams that are not in steady state are left untouched (the shape-generic step kernel takes them).
struct StepUpdateArgs {
    State<bf16_t> st;
    const bf16_t *k, *v, *Wk;
    int Hkv, lam, eta, phi_kind;
    int scr_stride;       // split forms: floats per stream in the scratch (sp_score)
};

constexpr int STEP_UPDATE_LAMMAX = 2048;

// SCORED: the candidates' scores are the query-dependent sums kept in the state (Sec. 4 / appendix "scoring ablation":
// sp_score per cache slot, the leaving pair's finished sum in its ring slot) instead of self-recall errors: step 2 is
// skipped, the leaving pair's sum follows it into the cache, the new pair's sum starts at zero.
// MODE 0: the whole update by one workgroup per stream.  With few streams most compute units would idle and each
// workgroup is bounded by its unit's share of the memory system, so the scoring (step 2 for the cached pairs) can be
// split off: MODE 1 = grid (streams, parts), workgroup (stream, part) scores the passes part, part + parts, ... into
// sp_score (scratch in this mode) and changes nothing else; MODE 2 = one workgroup per stream reads those scores and does
// the rest (the leaving pair's score, steps 3 and 4).  The scores are computed by the same instructions in either form.
// NTP: tiles of 16 candidates a wavefront takes per pass (2: the operands of H^T and W_k serve both; 1 for the score
// part when there are compute units enough to give every wavefront a single tile).
template <int DH, int DF, bool SCORED, int MODE = 0, int NTP = 2>
__global__ __launch_bounds__(512) void step_update_wide_kernel(StepUpdateArgs a) {
    static_assert(MODE == 0 || !SCORED, "the split forms score by self-recall error");
    static_assert(NTP == 2 || (NTP == 1 && MODE == 1), "single tiles: score part only");
    constexpr int M = DF / 2, KS = DH / 32, NZT = M / 16, KF = DF / 32, NCT = DH / 16, NP = NCT * KF / 8, PR = DH / 8;
    constexpr int LAMMAX = STEP_UPDATE_LAMMAX;
    __shared__ __attribute__((aligned(16))) uint4 HA[NCT * KF * 2 * 64];     // [row tile][k-step][part][lane]
    __shared__ __attribute__((aligned(16))) float s_l[DF];
    __shared__ __attribute__((aligned(16))) float phif[DF];                  // phi of the folded pair
    __shared__ __attribute__((aligned(16))) float vf[DH];                    // its value
    __shared__ __attribute__((aligned(16))) uint16_t pkb[DH], pvb[DH];       // the pair that leaves the window
    __shared__ float score[LAMMAX + 1];
    __shared__ int idx_l[LAMMAX + 1];
    __shared__ int drop_s;
    __shared__ __attribute__((aligned(16))) float phip[DF];   // phi of the leaving pair
    __shared__ float partp[KF][DH];                           // its recall, partial sums over 32 features each
    __shared__ float rdp_s, errp[2];
    __shared__ __attribute__((aligned(16))) float zp[M];      // its projections

    const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, r16 = lane & 15, g4 = lane >> 4;
    const int si = blockIdx.x, h = si % a.Hkv, LAM = a.lam, ETA = a.eta;
    float *Hg = a.st.H + (size_t)si * DF * DH, *sg = a.st.s + (size_t)si * DF;
    // ---- 1. the state (requested ahead of the check below: its address does not depend on the counters that the check
    // has to wait for); the leaving pair; the slots' token indices
    float4 hreg[NP][2];
    auto load_state = [&]() {
#pragma unroll
        for (int i = 0; i < NP; i++) {
            const int idx = w + 8 * i, ct = idx / KF, ks = idx % KF;
            const float *hp = Hg + (size_t)(16 * ct + r16) * DF + 32 * ks + 4 * g4;
            hreg[i][0] = *reinterpret_cast<const float4 *>(hp);
            hreg[i][1] = *reinterpret_cast<const float4 *>(hp + 16);
        }
    };
    if (MODE != 2) load_state();   // (MODE 2 needs the state only behind the first barrier: requested there)
    int32_t *sp_idx = a.st.sp_idx + (size_t)si * LAM;
    for (int x = tid; x < DF; x += 512) s_l[x] = sg[x];
    for (int e = tid; e < LAM; e += 512) idx_l[e] = sp_idx[e];
    const int64_t tok = a.st.n_tokens[si];
    if (!(tok >= (int64_t)ETA && a.st.sp_count[si] == LAM)) return;
    const int slot = (int)(tok % ETA), pidx = (int)(tok - ETA);
    bf16_t *sp_k = a.st.sp_k + (size_t)si * LAM * DH, *sp_v = a.st.sp_v + (size_t)si * LAM * DH;
    bf16_t *win_k = a.st.win_k + ((size_t)si * ETA + slot) * DH, *win_v = a.st.win_v + ((size_t)si * ETA + slot) * DH;
    const bf16_t *Wk = a.Wk + (size_t)h * M * DH;
    // the leaving pair's projections W_k^T k: one tile of 16 features per wavefront, its operands requested with the
    // rest of the start-up loads
    static_assert(NZT <= 8, "one projection tile per wavefront");
    bf16x8 zW[KS], zK[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
        zW[ks] = ld_bf16x8(Wk + (size_t)(16 * (w < NZT ? w : 0) + r16) * DH + 32 * ks + 8 * g4);
        zK[ks] = ld_bf16x8(win_k + 32 * ks + 8 * g4);
    }
    if (tid < PR) reinterpret_cast<uint4 *>(pkb)[tid] = reinterpret_cast<const uint4 *>(win_k)[tid];
    else if (tid < 2 * PR) reinterpret_cast<uint4 *>(pvb)[tid - PR] = reinterpret_cast<const uint4 *>(win_v)[tid - PR];
    if (tid == 0) idx_l[LAM] = pidx;
    float *wsc = nullptr, *sps = nullptr;
    if (SCORED) {
        wsc = a.st.win_score + (size_t)si * ETA + slot; sps = a.st.sp_score + (size_t)si * LAM;
        for (int e = tid; e < LAM; e += 512) score[e] = sps[e];
        if (tid == 0) score[LAM] = wsc[0];
    }
    float *scr = MODE ? a.st.sp_score + (size_t)si * a.scr_stride : nullptr;   // split forms: the cached pairs' scores
    if (MODE == 2)
        for (int e = tid; e < LAM; e += 512) score[e] = scr[e];
    if (!SCORED && MODE != 1 && w < NZT) {   // (every column of the tile holds the same key: column 0 stores)
        f32x4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ks++) z = mfma16(zW[ks], zK[ks], z);
        if (r16 == 0) *reinterpret_cast<f32x4 *>(&zp[16 * w + 4 * g4]) = z;
    }
    if (!SCORED && MODE != 2) {
#pragma unroll
    for (int i = 0; i < NP; i++) {
        const float x8[8] = {hreg[i][0].x, hreg[i][0].y, hreg[i][0].z, hreg[i][0].w, hreg[i][1].x, hreg[i][1].y, hreg[i][1].z, hreg[i][1].w};
        bf16x8 hi, lo;
        split8(x8, hi, lo);
        HA[((w + 8 * i) * 2 + 0) * 64 + lane] = __builtin_bit_cast(uint4, hi);
        HA[((w + 8 * i) * 2 + 1) * 64 + lane] = __builtin_bit_cast(uint4, lo);
    }
    }
    if (MODE == 2) {
        // the state travels while the leaving pair's features are made: requested behind the small loads (whose waits
        // would otherwise cover it) and not waited for by this barrier
        load_state();
        lds_barrier();
    } else {
        __syncthreads();
    }

    // W_k as wavefront 0 will need it for the features of the folded pair: requested before the arg-min is known, so
    // that only the pair's key is waited for afterwards
    bf16x8 WF[NZT][KS];
    auto preload_w = [&]() {
#pragma unroll
        for (int mt = 0; mt < NZT; mt++)
#pragma unroll
            for (int ks = 0; ks < KS; ks++) WF[mt][ks] = zero_bf16x8();
        if (w == 0) {
#pragma unroll
            for (int mt = 0; mt < NZT; mt++)
#pragma unroll
                for (int ks = 0; ks < KS; ks++) WF[mt][ks] = ld_bf16x8(Wk + (size_t)(16 * mt + r16) * DH + 32 * ks + 8 * g4);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    if (SCORED) preload_w();

    // ---- 2. self-recall errors
    if (!SCORED) {
    if (MODE != 1 && w == 7) {   // the leaving pair's features from its projections (every column of the tile holds the same key: column 0 stores)
        float pp[4 * NZT], pn[4 * NZT];
        f32x4 zt[NZT];
#pragma unroll
        for (int mt = 0; mt < NZT; mt++) zt[mt] = *reinterpret_cast<const f32x4 *>(&zp[16 * mt + 4 * g4]);
        phi_from_z_tiles<NZT>(zt, a.phi_kind, pp, pn);
        float dn = 0.f;
#pragma unroll
        for (int mt = 0; mt < NZT; mt++) {
            const float4 sp4 = *reinterpret_cast<const float4 *>(&s_l[16 * mt + 4 * g4]);
            const float4 sn4 = *reinterpret_cast<const float4 *>(&s_l[M + 16 * mt + 4 * g4]);
            dn = fmaf(pp[4 * mt], sp4.x, dn); dn = fmaf(pp[4 * mt + 1], sp4.y, dn);
            dn = fmaf(pp[4 * mt + 2], sp4.z, dn); dn = fmaf(pp[4 * mt + 3], sp4.w, dn);
            dn = fmaf(pn[4 * mt], sn4.x, dn); dn = fmaf(pn[4 * mt + 1], sn4.y, dn);
            dn = fmaf(pn[4 * mt + 2], sn4.z, dn); dn = fmaf(pn[4 * mt + 3], sn4.w, dn);
        }
        dn = grp_sum(dn);
        if (lane == 0) rdp_s = dn > 0.f ? 1.0f / dn : 0.f;
        if (r16 == 0) {
#pragma unroll
            for (int mt = 0; mt < NZT; mt++) {
                *reinterpret_cast<float4 *>(&phip[16 * mt + 4 * g4]) = make_float4(pp[4 * mt], pp[4 * mt + 1], pp[4 * mt + 2], pp[4 * mt + 3]);
                *reinterpret_cast<float4 *>(&phip[M + 16 * mt + 4 * g4]) = make_float4(pn[4 * mt], pn[4 * mt + 1], pn[4 * mt + 2], pn[4 * mt + 3]);
            }
        }
    }
    // Two tiles (32 candidates) per pass: every operand of H^T read from LDS and every operand of W_k read from L2
    // serves both, which halves the two streams that, next to the products themselves, fill the pass (per tile of 16
    // candidates the recall GEMM reads all 2 D d bytes of the split H^T).
    const int npair = MODE == 2 ? 0 : LAM / (16 * NTP);   // passes of NTP tiles
    const int part = MODE == 1 ? blockIdx.y : 0, nparts = MODE == 1 ? gridDim.y : 1;
#pragma unroll 1
    for (int tp = w + 8 * part; tp < npair; tp += 8 * nparts) {
        // With several passes the two wavefronts of a SIMD take turns at the higher issue priority: left alone, the
        // older one wins every arbitration and the younger one ends a sixth later (with one pass the default is faster).
        if (npair > 8 * nparts) {
            if (((tp >> 3) / nparts + (w >> 2)) & 1) __builtin_amdgcn_s_setprio(1);
            else __builtin_amdgcn_s_setprio(0);
        }
        const int e0 = 16 * NTP * tp + r16;   // this lane's candidates: e0 (and e0 + 16)
        bf16x8 Bh[NTP][KF], Bl[NTP][KF];
        float rd[NTP];
        {
            bf16x8 BK[NTP][KS];
#pragma unroll
            for (int u = 0; u < NTP; u++)
#pragma unroll
                for (int ks = 0; ks < KS; ks++) BK[u][ks] = ld_bf16x8(sp_k + (size_t)(e0 + 16 * u) * DH + 32 * ks + 8 * g4);
            // (W_k: two projection tiles at a time into two register sets, refilled as soon as their products are issued)
            // (addresses as a base in scalar registers plus one 32-bit lane offset, kept apart by an empty asm: the
            // 64-bit lane addresses the compiler would otherwise hold through the loop do not fit beside the operands)
            typedef const __attribute__((address_space(1))) bf16x8 *global_b8;
            const uint64_t Wu = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)((uint64_t)(uintptr_t)Wk >> 32)) << 32) |
                                (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(uintptr_t)Wk);
            uint32_t lane_off = (uint32_t)(2 * (r16 * DH + 8 * g4));   // bytes
            asm volatile("" : "+v"(lane_off));
            auto wld = [&](int mt, int ks) { return *(global_b8)((Wu + 2 * (16 * mt * DH + 32 * ks)) + lane_off); };
            bf16x8 Wa[2 * KS], Wb[2 * KS];
#pragma unroll
            for (int x = 0; x < 2 * KS; x++) Wa[x] = wld(x / KS, x % KS);
#pragma unroll
            for (int x = 0; x < 2 * KS; x++) Wb[x] = wld(2 + x / KS, x % KS);
            __builtin_amdgcn_sched_barrier(0);
            f32x4 zt[NTP][NZT];
#pragma unroll
            for (int u = 0; u < NTP; u++)
#pragma unroll
                for (int mt = 0; mt < NZT; mt++) zt[u][mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int m0 = 0; m0 < NZT; m0 += 4) {
#pragma unroll
                for (int x = 0; x < 2 * KS; x++) {
#pragma unroll
                    for (int u = 0; u < NTP; u++) zt[u][m0 + x / KS] = mfma16(Wa[x], BK[u][x % KS], zt[u][m0 + x / KS]);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (m0 + 4 < NZT) {
#pragma unroll
                    for (int x = 0; x < 2 * KS; x++) Wa[x] = wld(m0 + 4 + x / KS, x % KS);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int x = 0; x < 2 * KS; x++) {
#pragma unroll
                    for (int u = 0; u < NTP; u++) zt[u][m0 + 2 + x / KS] = mfma16(Wb[x], BK[u][x % KS], zt[u][m0 + 2 + x / KS]);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (m0 + 6 < NZT) {
#pragma unroll
                    for (int x = 0; x < 2 * KS; x++) Wb[x] = wld(m0 + 6 + x / KS, x % KS);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int u = 0; u < NTP; u++) {
                float pp[4 * NZT], pn[4 * NZT];
                phi_from_z_tiles<NZT>(zt[u], a.phi_kind, pp, pn);
                float dn = 0.f;
#pragma unroll
                for (int mt = 0; mt < NZT; mt++) {
                    const float4 sp4 = *reinterpret_cast<const float4 *>(&s_l[16 * mt + 4 * g4]);
                    const float4 sn4 = *reinterpret_cast<const float4 *>(&s_l[M + 16 * mt + 4 * g4]);
                    dn = fmaf(pp[4 * mt], sp4.x, dn); dn = fmaf(pp[4 * mt + 1], sp4.y, dn);
                    dn = fmaf(pp[4 * mt + 2], sp4.z, dn); dn = fmaf(pp[4 * mt + 3], sp4.w, dn);
                    dn = fmaf(pn[4 * mt], sn4.x, dn); dn = fmaf(pn[4 * mt + 1], sn4.y, dn);
                    dn = fmaf(pn[4 * mt + 2], sn4.z, dn); dn = fmaf(pn[4 * mt + 3], sn4.w, dn);
                }
                dn = grp_sum(dn);
                rd[u] = dn > 0.f ? 1.0f / dn : 0.f;   // recall = 0 while nothing was folded
#pragma unroll
                for (int ks = 0; ks < KF / 2; ks++) {
                    split8(&pp[8 * ks], Bh[u][ks], Bl[u][ks]);
                    split8(&pn[8 * ks], Bh[u][KF / 2 + ks], Bl[u][KF / 2 + ks]);
                }
            }
        }
        float esum[NTP] = {};
        // the candidates' values at all column tiles are requested together (one round trip instead of one per column
        // tile) and picked by a chain of selects (indexed by the loop variable, the arrays would leave the registers)
        uint2 vva[NTP][NCT];
#pragma unroll
        for (int u = 0; u < NTP; u++)
#pragma unroll
            for (int c2 = 0; c2 < NCT; c2++) vva[u][c2] = *reinterpret_cast<const uint2 *>(sp_v + (size_t)(e0 + 16 * u) * DH + 16 * c2 + 4 * g4);
#pragma unroll 2
        for (int ct = 0; ct < NCT; ct++) {
            uint2 vv[NTP];
#pragma unroll
            for (int u = 0; u < NTP; u++) vv[u] = vva[u][0];
#pragma unroll
            for (int c2 = 1; c2 < NCT; c2++)
                if (ct == c2) {
#pragma unroll
                    for (int u = 0; u < NTP; u++) vv[u] = vva[u][c2];
                }
            f32x4 acc[NTP], acc2[NTP], acc3[NTP];
#pragma unroll
            for (int u = 0; u < NTP; u++) acc[u] = acc2[u] = acc3[u] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KF; ks++) {
                const bf16x8 Ah = as_bf16x8(HA[((ct * KF + ks) * 2 + 0) * 64 + lane]), Al = as_bf16x8(HA[((ct * KF + ks) * 2 + 1) * 64 + lane]);
#pragma unroll
                for (int u = 0; u < NTP; u++) {
                    acc[u] = mfma16(Ah, Bh[u][ks], acc[u]);
                    acc2[u] = mfma16(Ah, Bl[u][ks], acc2[u]);
                    acc3[u] = mfma16(Al, Bh[u][ks], acc3[u]);
                }
            }
#pragma unroll
            for (int u = 0; u < NTP; u++) {
                const float v4[4] = {bf_lo(vv[u].x), bf_hi(vv[u].x), bf_lo(vv[u].y), bf_hi(vv[u].y)};
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const float err = (acc[u][i] + (acc2[u][i] + acc3[u][i])) * rd[u] - v4[i];
                    esum[u] = fmaf(err, err, esum[u]);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < NTP; u++) {
            const float es = grp_sum(esum[u]);
            if (g4 == 0) {
                if (MODE == 1) scr[e0 + 16 * u] = sqrtf(es);
                else score[e0 + 16 * u] = sqrtf(es);
            }
        }
    }
    if (MODE == 1) return;
    __builtin_amdgcn_s_setprio(0);
    preload_w();
    // The fp32 pieces of H^T are read a second time here (from L2) rather than held through the tile loop: there their
    // 64 registers were spilled, and every reload of a spilled register waits for all outstanding loads.
    if (MODE != 2) load_state();
    __syncthreads();
    // the leaving pair: this thread's pieces of H^T (row 16 ct + r16, features 32 ks + 4 g4 .. and + 16) times phi
#pragma unroll
    for (int i = 0; i < NP; i++) {
        const int idx = w + 8 * i, ct = idx / KF, ks = idx % KF;
        const float4 p0 = *reinterpret_cast<const float4 *>(&phip[32 * ks + 4 * g4]), p1 = *reinterpret_cast<const float4 *>(&phip[32 * ks + 16 + 4 * g4]);
        float d0 = hreg[i][0].x * p0.x;
        d0 = fmaf(hreg[i][0].y, p0.y, d0); d0 = fmaf(hreg[i][0].z, p0.z, d0); d0 = fmaf(hreg[i][0].w, p0.w, d0);
        d0 = fmaf(hreg[i][1].x, p1.x, d0); d0 = fmaf(hreg[i][1].y, p1.y, d0); d0 = fmaf(hreg[i][1].z, p1.z, d0); d0 = fmaf(hreg[i][1].w, p1.w, d0);
        d0 = grp_sum(d0);
        if (g4 == 0) partp[ks][16 * ct + r16] = d0;
    }
    __syncthreads();
    if (tid < 128) {   // (two wavefronts; head_dim 64 leaves the upper half idle)
        float err = 0.f;
        if (tid < DH) {
            float rec = 0.f;
#pragma unroll
            for (int ks = 0; ks < KF; ks++) rec += partp[ks][tid];
            err = rec * rdp_s - __uint_as_float((uint32_t)pvb[tid] << 16);
        }
        err = wsum(err * err);
        if (lane == 0) errp[w] = err;
    }
    __syncthreads();
    if (tid == 0) score[LAM] = sqrtf(errp[0] + errp[1]);
    __syncthreads();
    }

    // ---- 3. the pair that goes: smallest score, ties -> the larger token index; its features and value as fp32
    if (w == 0) {
        float bs = INFINITY; int bi = -1, be = 0;
        for (int e = lane; e <= LAM; e += 64) {
            const float sc = score[e]; const int ix = idx_l[e];
            if (sc < bs || (sc == bs && ix > bi)) { bs = sc; bi = ix; be = e; }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const float os = __shfl_xor(bs, o, 64); const int oi = __shfl_xor(bi, o, 64), oe = __shfl_xor(be, o, 64);
            if (os < bs || (os == bs && oi > bi)) { bs = os; bi = oi; be = oe; }
        }
        const int drop = __builtin_amdgcn_readfirstlane(be);
        const bf16_t *kr = drop < LAM ? sp_k + (size_t)drop * DH : reinterpret_cast<const bf16_t *>(pkb);
        const bf16_t *vr = drop < LAM ? sp_v + (size_t)drop * DH : reinterpret_cast<const bf16_t *>(pvb);
        float pp[4 * NZT], pn[4 * NZT];
        {   // every column holds the same key: column 0 stores
            bf16x8 BK[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ks++) BK[ks] = ld_bf16x8(kr + 32 * ks + 8 * g4);
            f32x4 zt[NZT];
#pragma unroll
            for (int mt = 0; mt < NZT; mt++) {
                zt[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ks++) zt[mt] = mfma16(WF[mt][ks], BK[ks], zt[mt]);
            }
            phi_from_z_tiles<NZT>(zt, a.phi_kind, pp, pn);
        }
        if (r16 == 0) {
#pragma unroll
            for (int mt = 0; mt < NZT; mt++) {
                *reinterpret_cast<float4 *>(&phif[16 * mt + 4 * g4]) = make_float4(pp[4 * mt], pp[4 * mt + 1], pp[4 * mt + 2], pp[4 * mt + 3]);
                *reinterpret_cast<float4 *>(&phif[M + 16 * mt + 4 * g4]) = make_float4(pn[4 * mt], pn[4 * mt + 1], pn[4 * mt + 2], pn[4 * mt + 3]);
            }
        }
        for (int c = lane; c < DH; c += 64) vf[c] = ldf(vr, c);
        if (lane == 0) drop_s = drop;
    }
    __syncthreads();

    // ---- 4. fold, write-back, slot replacement, ring slot
    const int drop = drop_s;
#pragma unroll
    for (int i = 0; i < NP; i++) {
        const int idx = w + 8 * i, ct = idx / KF, ks = idx % KF;
        const float vc = vf[16 * ct + r16];
        const float4 p0 = *reinterpret_cast<const float4 *>(&phif[32 * ks + 4 * g4]), p1 = *reinterpret_cast<const float4 *>(&phif[32 * ks + 16 + 4 * g4]);
        float4 h0 = hreg[i][0], h1 = hreg[i][1];
        h0.x = fmaf(p0.x, vc, h0.x); h0.y = fmaf(p0.y, vc, h0.y); h0.z = fmaf(p0.z, vc, h0.z); h0.w = fmaf(p0.w, vc, h0.w);
        h1.x = fmaf(p1.x, vc, h1.x); h1.y = fmaf(p1.y, vc, h1.y); h1.z = fmaf(p1.z, vc, h1.z); h1.w = fmaf(p1.w, vc, h1.w);
        float *hp = Hg + (size_t)(16 * ct + r16) * DF + 32 * ks + 4 * g4;
        *reinterpret_cast<float4 *>(hp) = h0;
        *reinterpret_cast<float4 *>(hp + 16) = h1;
    }
    for (int x = tid; x < DF; x += 512) sg[x] = s_l[x] + phif[x];
    if (drop < LAM) {   // the leaving pair takes the freed slot
        if (tid < PR) reinterpret_cast<uint4 *>(sp_k + (size_t)drop * DH)[tid] = reinterpret_cast<const uint4 *>(pkb)[tid];
        else if (tid < 2 * PR) reinterpret_cast<uint4 *>(sp_v + (size_t)drop * DH)[tid - PR] = reinterpret_cast<const uint4 *>(pvb)[tid - PR];
        if (tid == 64) sp_idx[drop] = pidx;
        if (SCORED && tid == 65) sps[drop] = score[LAM];
    }
    if (SCORED && tid == 66) wsc[0] = 0.f;
    const bf16_t *knew = a.k + (size_t)si * DH, *vnew = a.v + (size_t)si * DH;
    if (tid >= 128 && tid < 128 + PR) reinterpret_cast<uint4 *>(win_k)[tid - 128] = reinterpret_cast<const uint4 *>(knew)[tid - 128];
    else if (tid >= 192 && tid < 192 + PR) reinterpret_cast<uint4 *>(win_v)[tid - 192] = reinterpret_cast<const uint4 *>(vnew)[tid - 192];
    if (tid == 0) a.st.n_tokens[si] = tok + 1;
}

// ---------------------------------------------------------------------------------------------
// Query-dependent scores of a prefill call on MFMA (Sec. 4 / appendix "scoring ablation"; same sums as
// generic::band_score_kernel): row x of tok_score belongs to token a0 - eta + x (x < eta: the window the call found,
// then the call's tokens) and receives what the pair had gathered before the call plus, over all query heads of the
// group, the terms of the call's queries i with x - eta <= i <= x - 1 (the queries that see the key inside the sliding
// window).  Grid (tile of 64 keys, stream), one wavefront per 16 keys: phi of its keys stays in registers as the B
// operand (bf16 high + low parts); the (query head, tile of 16 queries) pairs of the band are taken four at a time:
// wavefront w computes phi of the queries of pair w into LDS, then every wavefront forms Q K^T and phi(Q) phi(K)^T of
// all four against its keys and adds the terms inside the band.
template <int DH, int DF>
__global__ __launch_bounds__(256) void band_score_wide_kernel(generic::PrefillArgs<bf16_t> a) {
    constexpr int M = DF / 2, KS = DH / 32, NZT = M / 16, KF = DF / 32;
    __shared__ __attribute__((aligned(16))) uint16_t PQ[4][2][16 * DF];   // phi of four query tiles, high / low parts, operand order
    const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, r16 = lane & 15, g4 = lane >> 4;
    const int si = blockIdx.y, b = si / a.dm.Hkv, h = si % a.dm.Hkv, g = a.dm.g;
    const int ETA = a.dm.eta, LAM = a.dm.lam, P = LAM + ETA, Tn = a.T_tokens, nrows = ETA + Tn, kind = a.dm.score_kind;
    const int64_t a0 = a.st.n_tokens[si];
    const int x0 = 64 * (int)blockIdx.x, x = x0 + 16 * w + r16;
    const bool kvalid = x < nrows && a0 - ETA + x >= 0;
    const int xr = x < nrows ? x : nrows - 1;   // (rows past the end read the last row; their sums are not stored)
    const bf16_t *kr = xr < ETA ? a.prefK + ((size_t)si * P + LAM + xr) * DH : a.k + ((size_t)si * Tn + (xr - ETA)) * DH;
    const bf16_t *Wk = a.Wk + (size_t)h * M * DH;

    bf16x8 BK[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ks++) BK[ks] = ld_bf16x8(kr + 32 * ks + 8 * g4);
    bf16x8 Bh[KF], Bl[KF];
    {
        f32x4 zt[NZT];
#pragma unroll
        for (int mt = 0; mt < NZT; mt++) {
            zt[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ks++)
                zt[mt] = mfma16(ld_bf16x8(Wk + (size_t)(16 * mt + r16) * DH + 32 * ks + 8 * g4), BK[ks], zt[mt]);
        }
        float pp[4 * NZT], pn[4 * NZT];
        phi_from_z_tiles<NZT>(zt, a.dm.phi_kind, pp, pn);
#pragma unroll
        for (int ks = 0; ks < KF / 2; ks++) {
            split8(&pp[8 * ks], Bh[ks], Bl[ks]);
            split8(&pn[8 * ks], Bh[KF / 2 + ks], Bl[KF / 2 + ks]);
        }
    }
    // queries that see some key of the tile
    const int i_lo = max(0, x0 - ETA), i_hi = min(Tn - 1, x0 + 62);
    const int nqt = i_hi >= i_lo ? (i_hi - i_lo) / 16 + 1 : 0, np = g * nqt;
    float sum = 0.f;
#pragma unroll 1
    for (int p0 = 0; p0 < np; p0 += 4) {
        if (p0 + w < np) {   // phi of the 16 queries of pair p0 + w (lane (column = query r16, group g4))
            const int r = (p0 + w) / nqt, qt = (p0 + w) - r * nqt, hq = h * g + r;
            const int iq = min(i_lo + 16 * qt + r16, i_hi);
            const bf16_t *qr = a.q + (((size_t)b * a.dm.Hq + hq) * Tn + iq) * DH;
            const bf16_t *Wq = a.Wq + (size_t)hq * M * DH;
            bf16x8 BQ[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ks++) BQ[ks] = ld_bf16x8(qr + 32 * ks + 8 * g4);
            f32x4 zt[NZT];
#pragma unroll
            for (int mt = 0; mt < NZT; mt++) {
                zt[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ks++)
                    zt[mt] = mfma16(ld_bf16x8(Wq + (size_t)(16 * mt + r16) * DH + 32 * ks + 8 * g4), BQ[ks], zt[mt]);
            }
            float pp[4 * NZT], pn[4 * NZT];
            phi_from_z_tiles<NZT>(zt, a.dm.phi_kind, pp, pn);
#pragma unroll
            for (int ks = 0; ks < KF / 2; ks++) {
                bf16x8 hi, lo;
                split8(&pp[8 * ks], hi, lo);
                *reinterpret_cast<uint4 *>(&PQ[w][0][r16 * DF + (((4 * ks + g4) ^ r16) << 3)]) = __builtin_bit_cast(uint4, hi);
                *reinterpret_cast<uint4 *>(&PQ[w][1][r16 * DF + (((4 * ks + g4) ^ r16) << 3)]) = __builtin_bit_cast(uint4, lo);
                split8(&pn[8 * ks], hi, lo);
                *reinterpret_cast<uint4 *>(&PQ[w][0][r16 * DF + (((4 * (KF / 2 + ks) + g4) ^ r16) << 3)]) = __builtin_bit_cast(uint4, hi);
                *reinterpret_cast<uint4 *>(&PQ[w][1][r16 * DF + (((4 * (KF / 2 + ks) + g4) ^ r16) << 3)]) = __builtin_bit_cast(uint4, lo);
            }
        }
        __syncthreads();
#pragma unroll 1
        for (int u = 0; u < 4; u++) {
            if (p0 + u >= np) break;
            const int r = (p0 + u) / nqt, qt = (p0 + u) - r * nqt, hq = h * g + r;
            const int iqa = min(i_lo + 16 * qt + r16, i_hi);   // A operand: row = query r16 of the tile
            const bf16_t *qr = a.q + (((size_t)b * a.dm.Hq + hq) * Tn + iqa) * DH;
            f32x4 S = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ks++) S = mfma16(ld_bf16x8(qr + 32 * ks + 8 * g4), BK[ks], S);
            f32x4 acc = {0.f, 0.f, 0.f, 0.f}, acc2 = {0.f, 0.f, 0.f, 0.f}, acc3 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KF; ks++) {
                const int addr = r16 * DF + (((4 * ks + g4) ^ r16) << 3);
                const bf16x8 Ah = as_bf16x8(*reinterpret_cast<const uint4 *>(&PQ[u][0][addr])), Al = as_bf16x8(*reinterpret_cast<const uint4 *>(&PQ[u][1][addr]));
                acc = mfma16(Ah, Bh[ks], acc);
                acc2 = mfma16(Ah, Bl[ks], acc2);
                acc3 = mfma16(Al, Bh[ks], acc3);
            }
            // lane (key r16 of this wavefront's tile, group g4): queries i_lo + 16 qt + 4 g4 + i
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const int iq = i_lo + 16 * qt + 4 * g4 + i;
                if (kvalid && iq <= i_hi && iq >= x - ETA && iq <= x - 1)
                    sum += generic::query_term(kind, S[i] * a.dm.scale, acc[i] + (acc2[i] + acc3[i]));
            }
        }
        __syncthreads();
    }
    sum = grp_sum(sum);
    if (g4 == 0 && x < nrows) {
        const int64_t t = a0 - ETA + x;
        const float prior = (x < ETA && t >= 0) ? a.st.win_score[(size_t)si * ETA + (int)(t % ETA)] : 0.f;
        a.tok_score[(size_t)si * nrows + x] = kvalid ? prior + sum : 0.f;
    }
}


// ---------------------------------------------------------------------------------------------
// State evolution of the prefill WITHOUT a sparse cache (sparse budget 0: the sliding-window + linear-attention
// base model, paper appendix "Efficiency Analysis", the lambda = 0 case).  Nothing is scored, so every pair that
// leaves the window is folded (Sec. 2.2 eq. recurrent_update): H at the entry of chunk j is a prefix sum over the
// groups that left before it.  Without the selection nothing couples the value columns of H, so the recurrence is
// split over them: grid (16-row tile of H^T, stream), ONE wavefront per workgroup (no barriers at all); head_dim / 16
// times as many workgroups as streams evolve the state.  Per regular chunk (a full chunk with a full window behind it):
//   1. snapshot of this tile's rows of H^T as bf16 high + low parts in the output kernel's operand order (and of s,
//      by the workgroup of tile 0);
//   2. H[f][c] += sum_t phi_t[f] v_t[c] over the 64 pairs that leave: both MFMA operands come out of row-major LDS
//      tiles through the transposing LDS read (contraction index = the pair); the pairs' features are the chunk-parallel
//      feature kernel's (copied into LDS by direct global -> LDS loads, one chunk ahead), their values this tile's
//      16 columns of the rows.  s += sum_t phi_t is the same product with a column of ones in place of the values: one
//      more workgroup per stream (block index head_dim / 16) evolves s that way.
// Chunks whose leaving group was not covered by the feature kernel (the first chunk of a pass: the group lies in the
// previous pass or in the window the call found) get their features computed here.
// Feature order: the feature kernel stores a row in operand order (position p holds feature 32 (p/32) + 16 ((p%8)/4)
// + 4 ((p/8)%4) + p%4); the accumulators are kept in plain feature order (lane (column c, group g) holds features
// 16 mt + 4 g + i of tile mt), which makes the lane's registers exactly the snapshot's pieces; row 16 mt + r of the A
// operand is therefore read from position 32 (mt/2) + 8 (r/4) + 4 (mt%2) + r%4.
template <int DH>
__global__ __launch_bounds__(64) void scan_nocache_kernel(generic::PrefillArgs<bf16_t> a) {
    constexpr int M = 64, D = 128, C = 64, ETA = 64, KS = DH / 32, P = ETA, NMT = D / 16;
    static_assert(DH == 64 || DH == 128, "head_dim");
    __shared__ __attribute__((aligned(16))) uint16_t PHs[2][C * 2 * D];   // phi of a leaving group [pair][part][position], two buffers
    __shared__ __attribute__((aligned(16))) uint16_t VS[2][2 * C * 8];    // their values at this tile's columns [half of 8][pair][8]
    const int lane = threadIdx.x, r16 = lane & 15, g4 = lane >> 4;
    const int ct = blockIdx.x, si = blockIdx.y, h = si % a.dm.Hkv;
    // The workgroup past the last row tile evolves s instead of rows of H^T: its "values" are a column of ones, everything
    // else is the same code (the role is decided outside the MFMA loops).
    const bool s_role = ct == DH / 16;
    float *Hg = a.st.H + (size_t)si * D * DH, *sg = a.st.s + (size_t)si * D;
    const bf16_t *Wk = a.Wk + (size_t)h * M * DH;
    const bf16_t *pK = a.prefK + (size_t)si * P * DH, *pV = a.prefV + (size_t)si * P * DH;
    const bf16_t *kc = a.k + (size_t)si * a.T_tokens * DH, *vc = a.v + (size_t)si * a.T_tokens * DH;
    const int j_first = a.next_j[si];
    const int j_end = min(a.j1, a.T_tokens / C);      // the full chunks of this launch; regular once the first one is
    if (j_first >= j_end) return;

    // this tile's rows of H^T: acc[mt][i] = H^T[16 ct + r16][16 mt + 4 g4 + i]  (s role: s[16 mt + 4 g4 + i] in every column)
    float *row_mem = s_role ? sg : Hg + (size_t)(16 * ct + r16) * D;
    f32x4 acc[NMT];
#pragma unroll
    for (int mt = 0; mt < NMT; mt++) acc[mt] = *reinterpret_cast<const f32x4 *>(row_mem + 16 * mt + 4 * g4);
    const uint32_t one2 = 0x3F803F80u;   // two bf16 ones
    const bf16x8 Bones = as_bf16x8(make_uint4(one2, one2, one2, one2));

    // rows of the group that leaves after chunk j: virtual rows j C + e, e < 64 (rows below P are the window the call found)
    auto krow = [&](int j, int e) { const int vr = j * C + e; return vr < P ? pK + (size_t)vr * DH : kc + (size_t)(vr - P) * DH; };
    auto vrow = [&](int j, int e) { const int vr = j * C + e; return vr < P ? pV + (size_t)vr * DH : vc + (size_t)(vr - P) * DH; };
    // requests for chunk j's leaving group into buffer `buf`
    auto fetch = [&](int j, int buf) {
        // values: 32 bytes per pair (this tile's 16 columns), lane = pair, one instruction per half
        if (!s_role) {
#pragma unroll
            for (int x = 0; x < 2; x++)
                lds_dma16(vrow(j, lane) + 16 * ct + 8 * x, &VS[buf][x * C * 8]);
        }
        if (j - 1 >= a.jb) {
            // the feature kernel's rows of chunk j - 1: 32 KB.  An instruction fills 1 KB = two rows; lane l fills part
            // (l / 16) % 2 of row 2 i + l / 32 at 16-byte position l % 16, which holds the row's piece (l % 16) ^ fswz(row):
            // sixteen rows read at once then hit different banks
            const uint16_t *src = a.phiK + ((size_t)si * a.S + (j - 1 - a.jb)) * C * 2 * D;
#pragma unroll 8
            for (int i = 0; i < C * 2 * D / 512; i++) {
                const int row = 2 * i + (lane >> 5);
                lds_dma16(src + row * 2 * D + ((lane >> 4) & 1) * D + (((lane & 15) ^ fswz(row)) << 3), &PHs[buf][i * 512]);
            }
        } else {
            // not covered by the feature kernel: phi of the 64 keys here (Sec. 2.3 eq. feature_map), four tiles of 16
#pragma unroll 1
            for (int t4 = 0; t4 < 4; t4++) {
                const int row = 16 * t4 + r16;
                const bf16_t *kr = krow(j, row);
                bf16x8 BK[KS];
#pragma unroll
                for (int ks = 0; ks < KS; ks++) BK[ks] = ld_bf16x8(kr + 32 * ks + 8 * g4);
                f32x4 zt[4];
#pragma unroll
                for (int mt = 0; mt < 4; mt++) {
                    zt[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < KS; ks++)
                        zt[mt] = mfma16(ld_bf16x8(Wk + (size_t)(16 * mt + r16) * DH + 32 * ks + 8 * g4), BK[ks], zt[mt]);
                }
                float pp[16], pn[16];
                phi_from_z(zt, a.dm.phi_kind, pp, pn);
                bf16x8 hi[4], lo[4];
                split8(&pp[0], hi[0], lo[0]); split8(&pp[8], hi[1], lo[1]);
                split8(&pn[0], hi[2], lo[2]); split8(&pn[8], hi[3], lo[3]);
                uint16_t *dst = &PHs[buf][row * 2 * D];
#pragma unroll
                for (int ks = 0; ks < 4; ks++) {
                    *reinterpret_cast<uint4 *>(dst + (((4 * ks + g4) ^ fswz(row)) << 3)) = __builtin_bit_cast(uint4, hi[ks]);
                    *reinterpret_cast<uint4 *>(dst + D + (((4 * ks + g4) ^ fswz(row)) << 3)) = __builtin_bit_cast(uint4, lo[ks]);
                }
            }
        }
    };

    fetch(j_first, j_first & 1);
    for (int j = j_first; j < j_end; j++) {
        const int buf = j & 1;
        // ---- 1. snapshot of the state at the chunk's entry (stores; the loads they follow complete first)
        if (a.want_out) {
            const size_t sj = (size_t)si * a.S + (j - a.jb);
            if (s_role) {
                if (r16 == 0) {
#pragma unroll
                    for (int mt = 0; mt < NMT; mt++) *reinterpret_cast<f32x4 *>(a.snapS + sj * D + 16 * mt + 4 * g4) = acc[mt];
                }
            } else {
                uint4 *Hs = reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(a.snapH) + sj * (2 * DH * D));
#pragma unroll
                for (int ks = 0; ks < 4; ks++) {
                    const float x8[8] = {acc[2 * ks][0], acc[2 * ks][1], acc[2 * ks][2], acc[2 * ks][3],
                                         acc[2 * ks + 1][0], acc[2 * ks + 1][1], acc[2 * ks + 1][2], acc[2 * ks + 1][3]};
                    bf16x8 hi, lo;
                    split8(x8, hi, lo);
                    Hs[ct * 256 + ks * 64 + lane] = __builtin_bit_cast(uint4, hi);                 // [part][row tile][k-step][lane]
                    Hs[DH * 16 + ct * 256 + ks * 64 + lane] = __builtin_bit_cast(uint4, lo);
                }
            }
        }
        // ---- the leaving group's rows have landed (direct loads have no register to wait on); then the next group is
        // requested into the other buffer, whose last reads were the previous chunk's
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        asm volatile("" ::: "memory");
        if (j + 1 < j_end) fetch(j + 1, buf ^ 1);
        // ---- 2. fold.  Contraction slots of lane group g4 in k-step kst: pairs 32 kst + 4 g4 + 0..3, then + 16 (the
        // order in which the transposing read delivers them, the same for both operands)
#pragma unroll
        for (int kst = 0; kst < 2; kst++) {
            const int t0 = 32 * kst + 4 * g4 + (r16 >> 2), t15 = fswz(t0);
            // B: values, column c = 16 ct + r16; lane i of a group points at pair t0's 4 columns 4 (i % 4) ..
            bf16x8 Bv = Bones;
            if (!s_role) {
                const uint16_t *vb = &VS[buf][((r16 & 3) >> 1) * C * 8 + 4 * (r16 & 1)];
                const bf16x4 b0 = tr_read(vb + t0 * 8), b1 = tr_read(vb + (t0 + 16) * 8);
                Bv = __builtin_shufflevector(b0, b1, 0, 1, 2, 3, 4, 5, 6, 7);
            }
#pragma unroll
            for (int mt = 0; mt < NMT; mt++) {
                // A: phi^T, row f = 16 mt + r of the tile from position 32 (mt / 2) + 8 (r / 4) + 4 (mt % 2) + r % 4, i.e.
                // 16-byte piece 4 (mt / 2) + r / 4 of the row (stored at that piece ^ fswz(pair)), its half mt % 2
                const int off = (((4 * (mt >> 1) + (r16 & 3)) ^ t15) << 3) + 4 * (mt & 1);
#pragma unroll
                for (int part = 0; part < 2; part++) {
                    const uint16_t *pa = &PHs[buf][part * D + off];
                    const bf16x4 a0 = tr_read(pa + t0 * 2 * D), a1 = tr_read(pa + (t0 + 16) * 2 * D);
                    const bf16x8 Av = __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7);
                    acc[mt] = mfma16(Av, Bv, acc[mt]);
                }
            }
        }
    }
    // ---- the state after the last full chunk goes back to memory
    if (!s_role || r16 == 0) {
#pragma unroll
        for (int mt = 0; mt < NMT; mt++) *reinterpret_cast<f32x4 *>(row_mem + 16 * mt + 4 * g4) = acc[mt];
    }
}

// after scan_nocache_kernel: the chunk position of every stream moves behind the full chunks of the launch
__global__ void advance_next_j_kernel(int32_t *next_j, int ns, int j_end) {
    const int si = blockIdx.x * blockDim.x + threadIdx.x;
    if (si < ns && next_j[si] < j_end) next_j[si] = j_end;
}

}  // namespace fast
}  // namespace lola

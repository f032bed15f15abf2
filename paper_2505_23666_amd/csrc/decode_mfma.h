// Fused single-token generation step for the 8B head shape on gfx950: one workgroup of four
// wavefronts per (sequence, kv head), two workgroups resident per compute unit.
//
// What one launch does per stream (paper Sec. 3: E_t, G_t, S_t, H_t and y_t equations):
//   - the new pair replaces the oldest one in the window ring; the displaced pair p leaves;
//   - phi of the lambda cached keys and of p (bf16 MFMA, exact products, fp32 accumulate, fp32
//     softmax), recall phi(k)^T H / phi(k)^T s of all lambda + 1 eligible pairs: every wavefront keeps
//     32 rows of H^T in registers (fp32, plus bf16 high + low parts as MFMA operands), the feature
//     vectors are shared through LDS as bf16 high + low parts (three MFMAs per product, ~2^-17
//     relative); squared self-recall error, arg-min (ties: larger token index goes);
//   - rank-1 fold of the dropped pair into the fp32 registers, written back once; s likewise;
//   - the dropped slot is overwritten in place by p (cache compaction);
//   - outputs of the G query heads: softmax weights over cache + window with m = max(0, max logit),
//     sum_i p_i v_i on MFMA from values staged in LDS, linear read-out phi(q)^T H taken from the
//     same pass over H and corrected by the rank-1 term, shared normaliser.
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
#include <type_traits>
#include "lola_common.h"

namespace lola {
namespace fast {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ bf16x8 as_bf16x8(uint4 u) { return __builtin_bit_cast(bf16x8, u); }
__device__ __forceinline__ bf16x8 ld_bf16x8(const bf16_t *p) { return as_bf16x8(*reinterpret_cast<const uint4 *>(p)); }
__device__ __forceinline__ bf16x8 zero_bf16x8() { return as_bf16x8(make_uint4(0, 0, 0, 0)); }
// x = hi + lo + O(2^-17 |x|), both parts bf16.  Two values are rounded by one packed conversion; the residual
// x - hi is one bf16 dot product each (hi . (-1, 0) + x, exact: the difference of a float and its bf16 rounding is a
// float).  The two selector constants are kept in registers the compiler cannot fold: as literals of the dot
// instruction (-1, 0) comes out wrong on this toolchain.
__device__ __forceinline__ void split8(const float x[8], bf16x8 &hi, bf16x8 &lo) {
    uint32_t c0 = 0x0000BF80u, c1 = 0xBF800000u;
    asm volatile("" : "+s"(c0), "+s"(c1));
    const bf16x2 m0 = __builtin_bit_cast(bf16x2, c0), m1 = __builtin_bit_cast(bf16x2, c1);
#pragma unroll
    for (int p = 0; p < 4; p++) {
        const f32x2 v = {x[2 * p], x[2 * p + 1]};
        const bf16x2 h = __builtin_convertvector(v, bf16x2);
        const f32x2 r = {__builtin_amdgcn_fdot2_f32_bf16(h, m0, v[0], false), __builtin_amdgcn_fdot2_f32_bf16(h, m1, v[1], false)};
        const bf16x2 l = __builtin_convertvector(r, bf16x2);
        hi[2 * p] = h[0]; hi[2 * p + 1] = h[1];
        lo[2 * p] = l[0]; lo[2 * p + 1] = l[1];
    }
}
// LDS read with transposition inside each group of 16 lanes (gfx950): lane i of a group supplies the address of four
// consecutive 16-bit values E[i][0..3]; lane j receives E[j / 4][j % 4], E[4 + j / 4][j % 4], E[8 + j / 4][j % 4],
// E[12 + j / 4][j % 4] (verified on hardware).  The address must be 8-byte aligned.
__device__ __forceinline__ bf16x4 tr_read(const uint16_t *p) {
    typedef __bf16 v4 __attribute__((ext_vector_type(4)));
    return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) v4 *)(p));
}
// reciprocal to one unit in the last place (the hardware instruction); an IEEE division costs ten instructions
__device__ __forceinline__ float frcp(float x) { return __builtin_amdgcn_rcpf(x); }
__device__ __forceinline__ float bf_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf_hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }
__device__ __forceinline__ float dot2bf(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
}
// exchange with the lane 16 / 32 positions away (gfx950 row swaps): r0 and r1 are this lane's value and its partner's
__device__ __forceinline__ void swap16(float v, float &r0, float &r1) {
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    r0 = __uint_as_float(r[0]); r1 = __uint_as_float(r[1]);
}
__device__ __forceinline__ void swap32(float v, float &r0, float &r1) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    r0 = __uint_as_float(r[0]); r1 = __uint_as_float(r[1]);
}
// reductions over the four lanes that share l % 16
__device__ __forceinline__ float grp_sum(float v) { float x, y; swap16(v, x, y); v = x + y; swap32(v, x, y); return x + y; }
// Three sums at once over the four lanes that share l % 16: lane group l / 16 = 0, 1, 2 receives the sum of a, b, c
// (group 3 receives 0).  The row swap exchanges the odd rows of its first operand with the even rows of its second, so
// one swap pairs partial sums of two different quantities: three swaps and three additions instead of six and six.
__device__ __forceinline__ float grp_sum3(float a, float b, float c) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    const float x = __uint_as_float(r[0]) + __uint_as_float(r[1]);   // rows: a0+a1, b0+b1, a2+a3, b2+b3
    const auto q = __builtin_amdgcn_permlane16_swap(__float_as_uint(c), 0u, false, false);
    const float y = __uint_as_float(q[0]) + __uint_as_float(q[1]);   // rows: c0+c1, 0, c2+c3, 0
    const auto t = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(y), false, false);
    return __uint_as_float(t[0]) + __uint_as_float(t[1]);            // rows: sum a, sum b, sum c, 0
}
__device__ __forceinline__ float grp_max(float v) { float x, y; swap16(v, x, y); v = fmaxf(x, y); swap32(v, x, y); return fmaxf(x, y); }
__device__ __forceinline__ float grp_min(float v) { float x, y; swap16(v, x, y); v = fminf(x, y); swap32(v, x, y); return fminf(x, y); }
// reductions over the whole wavefront: four data-parallel-primitive steps inside each row of 16 lanes (swap
// neighbours, swap pairs, mirror each half, mirror the row: every lane ends with the row's result), then the
// two row swaps above
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}
__device__ __forceinline__ float wsum(float v) {
    v += dpp_f<0xB1>(v); v += dpp_f<0x4E>(v); v += dpp_f<0x141>(v); v += dpp_f<0x140>(v);
    return grp_sum(v);
}
__device__ __forceinline__ float wmax(float v) {
    v = fmaxf(v, dpp_f<0xB1>(v)); v = fmaxf(v, dpp_f<0x4E>(v)); v = fmaxf(v, dpp_f<0x141>(v)); v = fmaxf(v, dpp_f<0x140>(v));
    return grp_max(v);
}
// smallest 64-bit key of the wavefront, in every lane
__device__ __forceinline__ unsigned long long wmin_u64(unsigned long long k) {
#define LOLA_KSTEP(CTRL) { const unsigned long long o = ((unsigned long long)dpp_u<CTRL>((uint32_t)(k >> 32)) << 32) | dpp_u<CTRL>((uint32_t)k); k = o < k ? o : k; }
    LOLA_KSTEP(0xB1) LOLA_KSTEP(0x4E) LOLA_KSTEP(0x141) LOLA_KSTEP(0x140)
#undef LOLA_KSTEP
    {
        auto h = __builtin_amdgcn_permlane16_swap((uint32_t)(k >> 32), (uint32_t)(k >> 32), false, false);
        auto l = __builtin_amdgcn_permlane16_swap((uint32_t)k, (uint32_t)k, false, false);
        const unsigned long long x = ((unsigned long long)h[0] << 32) | l[0], y = ((unsigned long long)h[1] << 32) | l[1];
        k = x < y ? x : y;
    }
    {
        auto h = __builtin_amdgcn_permlane32_swap((uint32_t)(k >> 32), (uint32_t)(k >> 32), false, false);
        auto l = __builtin_amdgcn_permlane32_swap((uint32_t)k, (uint32_t)k, false, false);
        const unsigned long long x = ((unsigned long long)h[0] << 32) | l[0], y = ((unsigned long long)h[1] << 32) | l[1];
        k = x < y ? x : y;
    }
    return k;
}
__device__ __forceinline__ float wmin(float v) { return -wmax(-v); }
__device__ __forceinline__ float fexp2(float x) { return __builtin_amdgcn_exp2f(x); }
constexpr float LOG2E = 1.4426950408889634f;


template <typename TO>
struct DecodeFastArgs {
    State<bf16_t> st;
    const bf16_t *q, *k, *v, *Wq, *Wk;
    TO *out;
    int Hq, Hkv;
    float scale;
    int phi_kind;
    int hide;   // restricted query: bit 0 the hidden state, bit 1 the sparse cache is not read
    int g;      // query heads per kv head, 1 .. G (the kernel is compiled for G = 4 rows of queries; unused rows are zero)
    // deferred folds (R > 0): up to R - 1 folded pairs per stream wait here, [stream][R][D] / [stream][R][DH] fp32
    float *pend_phi, *pend_v;
    int32_t *pend_count;
};

// phi of 16 vectors from their projections held in the C layout of the projection GEMM: lane (column r16,
// group g4) holds z[16*mt + 4*g4 + i] in zt[mt][i]; the other three lanes of the column hold the rest.
// Returns the lane's 16 positive-half and 16 negative-half features (same index pattern).
__device__ __forceinline__ void phi_from_z(const f32x4 zt[4], int phi_kind, float pp[16], float pn[16]) {
    if (phi_kind == 1) {
#pragma unroll
        for (int x = 0; x < 16; x++) { const float zs = zt[x >> 2][x & 3] * LOG2E; pp[x] = fexp2(zs); pn[x] = fexp2(-zs); }
        return;
    }
    float zmax = zt[0][0], zmin = zt[0][0];
#pragma unroll
    for (int x = 1; x < 16; x++) { zmax = fmaxf(zmax, zt[x >> 2][x & 3]); zmin = fminf(zmin, zt[x >> 2][x & 3]); }
    zmax = grp_max(zmax); zmin = grp_min(zmin);
    const float cp = -zmax * LOG2E, cn = zmin * LOG2E;
    float sp = 0.f, sn = 0.f;
#pragma unroll
    for (int x = 0; x < 16; x++) {
        const float zz = zt[x >> 2][x & 3];
        pp[x] = fexp2(fmaf(zz, LOG2E, cp)); pn[x] = fexp2(fmaf(zz, -LOG2E, cn));
        sp += pp[x]; sn += pn[x];
    }
    sp = grp_sum(sp); sn = grp_sum(sn);
    const float ip = frcp(sp), in_ = frcp(sn);
#pragma unroll
    for (int x = 0; x < 16; x++) { pp[x] *= ip; pn[x] *= in_; }
}

// DH = head_dim = 128, feature dim D = 128 (M = 64 projections), LAM multiple of 64 (<= 128 here),
// ETA = 64, G = query heads per kv head (<= 4).
//
// LDS plan (about 78 KB, two workgroups per compute unit):
//   PB   64 KB  bf16 high and low parts of phi of the cached keys, [key][feature chunk] with the 16-byte chunk index
//               XOR-ed by key % 16 so that operand stores and loads are bank-conflict free.  After the recall GEMM
//               the same bytes hold the value rows [key][c] (row stride 130 bf16) and the softmax weights as bf16
//               high + low parts.
//   PX    4 KB  the same for the "extra tile": row 0 the leaving key, rows 1..G the queries.
//   the rest    small per-stream vectors.
// H^T never goes through LDS: wavefront w owns its rows 32w .. 32w+31 (output columns of the recall GEMM).
//
// Deferred folds (R = 8): the state in memory lags behind by up to R folded pairs, which are kept as fp32 rows
// (phi, v) beside it.  A step adds them to its register copy of H^T with fp32 MFMAs (16x16x4: the contraction index
// is the pending pair) and to s, so everything downstream sees the true state; its own fold is appended to the
// list.  The step that finds the list full writes H and s (with the R listed pairs, without its own) back and
// starts a new list with its own pair.  Same sums as folding at once (Sec. 2.2, eq. recurrent_update), seven of
// eight write-backs of H saved.
// GDYN: the group size is read from the arguments (1 .. G) instead of being G; the benchmarked shape keeps the
// compile-time form.
// DH = head_dim: 128 (8B head shape) or 64 (1B head shape); with 64 a wavefront owns 16 rows of H^T instead of 32.
template <int LAM, int ETA, int G, int R, bool GDYN, int DH, typename TO>
__global__ __launch_bounds__(256, 2) void decode_fast_kernel(DecodeFastArgs<TO> a) {
    static_assert(R == 0 || R == 4 || R == 8, "pending pairs are the contraction index of 16x16x4 MFMAs");
    static_assert(DH == 128 || DH == 64, "head_dim");
    constexpr int RG = R > 0 ? R / 4 : 1;
    constexpr int M = 64, D = 128;
    constexpr int KS = DH / 32;            // k-steps of a contraction over the head dimension
    constexpr int PR = DH / 8;             // 16-byte pieces of a key / value / query row
    constexpr int CW = DH / 4;             // rows of H^T (= value columns) a wavefront owns
    constexpr int NCT = CW / 16;           // its 16-row tiles
    constexpr int NKT = LAM / 16;          // key tiles of the sparse cache
    constexpr int TPW = NKT / 4;           // key tiles whose phi a wavefront computes
    constexpr int NWT = ETA / 16;          // window tiles
    constexpr int KP = LAM;                // position of the leaving pair in the logit / score arrays
    constexpr int KW = LAM + 1;            // first window position
    constexpr int NKEY = LAM + 1 + ETA;
    constexpr int NKS = (NKEY + 31) / 32;  // k-steps of the value read-out
    constexpr int KPAD = NKS * 32;
    constexpr int VLS = DH;                // row stride (bf16) of the staged values (8-byte pieces XOR-swizzled by the row)
    constexpr int XR = 8;                  // rows reserved for the extra tile (1 + G used)
    static_assert(NKT % 4 == 0 && ETA % 16 == 0 && G >= 1 && G <= 4 && NKT <= 8 && NWT <= 4, "shape");
    constexpr int PB_ELEMS = (2 * LAM * D > KPAD * VLS + 2 * G * KPAD) ? 2 * LAM * D : ((KPAD * VLS + 2 * G * KPAD + 7) / 8) * 8;

    __shared__ __attribute__((aligned(16))) uint16_t PB[PB_ELEMS];      // [0, LAM*D): high parts, [LAM*D, 2*LAM*D): low parts
    __shared__ __attribute__((aligned(16))) uint16_t PX[2 * XR * D];
    __shared__ __attribute__((aligned(16))) float s_l[D];
    __shared__ float rden_l[LAM + 1];      // 1 / (phi(k)^T s) per eligible pair (0 while nothing was folded)
    __shared__ float part[4][LAM + 1];     // squared-error partial sums, one row per wavefront (32 value columns each)
    __shared__ float lg[G][NKEY];          // logits
    __shared__ float lin[G][DH];           // phi(q)^T H (state before the fold)
    __shared__ float denq[G], dotqf[G], psum_s[G], elin_s[G];
    __shared__ __attribute__((aligned(16))) float phif[D];
    __shared__ float vf[DH];               // the folded pair
    __shared__ float pvf[DH];              // value of the leaving pair
    __shared__ __attribute__((aligned(16))) uint32_t qb[G][DH / 2];   // query rows, raw bf16 pairs
    __shared__ __attribute__((aligned(16))) uint16_t pkb[DH];
    __shared__ __attribute__((aligned(16))) uint16_t pvb[DH];
    __shared__ int idx_l[LAM];
    __shared__ __attribute__((aligned(16))) float zx[M];   // projections of the leaving key
    uint16_t *Vl = PB;                                                  // [KPAD][VLS] after the recall GEMM
    uint16_t *Ph = PB + KPAD * VLS, *Pl = Ph + G * KPAD;               // [G][KPAD] weights, high / low parts

    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, r16 = lane & 15, g4 = lane >> 4;
    const int si = blockIdx.x, b = si / a.Hkv, h = si - b * a.Hkv;
    float *Hg = a.st.H + (size_t)si * D * DH;     // H^T [DH][D]
    float *sg = a.st.s + (size_t)si * D;
    bf16_t *win_k = a.st.win_k + (size_t)si * ETA * DH, *win_v = a.st.win_v + (size_t)si * ETA * DH;
    bf16_t *sp_k = a.st.sp_k + (size_t)si * LAM * DH, *sp_v = a.st.sp_v + (size_t)si * LAM * DH;
    int32_t *sp_idx = a.st.sp_idx + (size_t)si * LAM;
    const bf16_t *Wk = a.Wk + (size_t)h * M * DH;            // [M][DH], row j = w_j
    const bf16_t *knew = a.k + (size_t)si * DH, *vnew = a.v + (size_t)si * DH;
    const int g = GDYN ? a.g : G;
    const bf16_t *qg = a.q + ((size_t)b * a.Hq + (size_t)h * g) * DH;   // g consecutive query rows

    const int64_t tok = a.st.n_tokens[si];
    const int spc = a.st.sp_count[si];
    const bool popped = tok >= (int64_t)ETA;
    const bool steady = popped && spc == LAM;          // scoring happens; H may be non-zero
    const int slot = (int)(tok % ETA);
    const int pidx = (int)(tok - ETA);
    const int wn = (int)min((int64_t)ETA, tok + 1);   // window pairs after the push

    // ---- stage 0: loads are requested in the order in which they are consumed (they complete in order): the small
    // per-stream vectors that the first barrier waits for, then the operands of the projections, then the window keys
    const uint4 q_ld = (tid >= 64 && tid < 64 + g * PR) ? reinterpret_cast<const uint4 *>(qg)[tid - 64] : make_uint4(0, 0, 0, 0);
    // s and the listed pairs' feature vectors: all lanes of wavefront 0 load (lanes 32 .. 63 the same pieces as 0 .. 31)
    // inside one wavefront-uniform branch.  Loaded per thread under `tid < D / 4`, the first of these loads was followed
    // by a wait for everything requested so far (a register copy of its result), which held wavefront 0 for a memory
    // round trip before it requested its weights and keys.
    const int wu = __builtin_amdgcn_readfirstlane(w);
    float4 s_ld = make_float4(0.f, 0.f, 0.f, 0.f);
    float *pphi = nullptr, *pval = nullptr;
    int cnt = 0;
    float4 sp_ld[R > 0 ? R : 1];
#pragma unroll
    for (int p = 0; p < (R > 0 ? R : 1); p++) sp_ld[p] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (R > 0) {
        pphi = a.pend_phi + (size_t)si * R * D; pval = a.pend_v + (size_t)si * R * DH;
        cnt = a.pend_count[si];
    }
    if (wu == 0) {
        const int t4 = tid & (D / 4 - 1);
        s_ld = reinterpret_cast<const float4 *>(sg)[t4];
        if (R > 0) {
#pragma unroll
            for (int p = 0; p < R; p++) sp_ld[p] = reinterpret_cast<const float4 *>(pphi + p * D)[t4];
        }
    }
    const int idx_ld = tid < LAM ? sp_idx[tid] : 0;
    // W_k crosses the cache hierarchy once per workgroup: each wavefront fetches a quarter (16 projections, 4 KB,
    // whole lines) and the MFMA A operands are read back from LDS, where the feature tile is not in use yet
    uint4 wk_ld[KS];
#pragma unroll
    for (int it = 0; it < KS; it++) wk_ld[it] = reinterpret_cast<const uint4 *>(Wk)[16 * PR * w + 64 * it + lane];
    // W_q of this wavefront's query head, read as whole 1 KB pieces: piece `it` holds 64 / PR projections, lane l the
    // 8 inputs 8 (l % PR) .. of projection (64 / PR) it + l / PR (each row's dot product is finished by a reduction over
    // PR neighbouring lanes)
    uint4 wq[PR];
    {
        const bf16_t *Wq = a.Wq + ((size_t)h * g + (w < g ? w : 0)) * M * DH;
#pragma unroll
        for (int it = 0; it < PR; it++) wq[it] = reinterpret_cast<const uint4 *>(Wq)[64 * it + lane];
    }
    // cached key rows of this wavefront's tiles, already in MFMA B-operand form (column = key, k = input index)
    bf16x8 BK[TPW][KS];
#pragma unroll
    for (int t = 0; t < TPW; t++)
#pragma unroll
        for (int ks = 0; ks < KS; ks++) BK[t][ks] = ld_bf16x8(sp_k + (size_t)(16 * (w + 4 * t) + r16) * DH + 32 * ks + 8 * g4);
    // window keys of this wavefront's tile as they stand in memory, and the new key: the row in the new token's ring
    // slot is the key of the pair that leaves; it is swapped for the new key once the token counter is known, so that
    // nothing requested here waits for that counter (whose own load is still on its way)
    bf16x8 BWin[KS], KN[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
        BWin[ks] = ld_bf16x8(win_k + (size_t)(16 * (w < NWT ? w : 0) + r16) * DH + 32 * ks + 8 * g4);
        KN[ks] = ld_bf16x8(knew + 32 * ks + 8 * g4);
    }
    // the value row of the leaving pair (PR threads, 16 bytes each) is wanted much later
    // (every lane loads its piece of the row, whether or not a pair leaves: a load under a condition, with zeros
    // otherwise, is followed by a register copy that waits for everything requested so far)
    const uint4 p_ld = reinterpret_cast<const uint4 *>(win_v + (size_t)slot * DH)[tid & (PR - 1)];
    if (tid < D / 4) {
        float4 sv = s_ld;
        if (R > 0) {
#pragma unroll
            for (int p = 0; p < R; p++)
                if (p < cnt) { sv.x += sp_ld[p].x; sv.y += sp_ld[p].y; sv.z += sp_ld[p].z; sv.w += sp_ld[p].w; }
        }
        reinterpret_cast<float4 *>(s_l)[tid] = sv;
    }
    if (tid < LAM) idx_l[tid] = idx_ld;
    if (tid >= 64 && tid < 64 + g * PR) reinterpret_cast<uint4 *>(qb)[tid - 64] = q_ld;
    if (tid >= 128 && tid < 128 + 2 * XR * D / 8) reinterpret_cast<uint4 *>(PX)[tid - 128] = make_uint4(0, 0, 0, 0);
    // W_k staging: row j = projection, 16-byte piece p at position p ^ (j % PR)
#pragma unroll
    for (int it = 0; it < KS; it++) {
        const int j = 16 * w + (64 * it + lane) / PR, pc = lane % PR;
        *reinterpret_cast<uint4 *>(&PB[j * DH + ((pc ^ (j & (PR - 1))) << 3)]) = wk_ld[it];
    }
    lds_barrier();
    // (behind the barrier: the keys are the last of the loads above, and the barrier needs only the first)
    {
        // the lanes that hold the ring slot's row hand the leaving key over and take the new key
        const bool mine = w < NWT && 16 * w + r16 == slot;
        if (mine) {
#pragma unroll
            for (int ks = 0; ks < KS; ks++) {
                if (popped) *reinterpret_cast<uint4 *>(&pkb[32 * ks + 8 * g4]) = __builtin_bit_cast(uint4, BWin[ks]);
                BWin[ks] = KN[ks];
            }
        }
    }
    // W_k as MFMA A operand (row = projection, k = input index): [projection tile][k-step]
    bf16x8 AW[4][KS];
#pragma unroll
    for (int mt = 0; mt < 4; mt++)
#pragma unroll
        for (int ks = 0; ks < KS; ks++)
            AW[mt][ks] = as_bf16x8(*reinterpret_cast<const uint4 *>(&PB[(16 * mt + r16) * DH + (((4 * ks + g4) ^ (r16 & (PR - 1))) << 3)]));
    lds_barrier();   // every wavefront holds its operands: the staging area may become the feature tile
    // ---- query rows as MFMA A operand (rows >= G are zero)
    bf16x8 AQ[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ks++)
        AQ[ks] = r16 < g ? as_bf16x8(*reinterpret_cast<const uint4 *>(&qb[r16][16 * ks + 4 * g4])) : zero_bf16x8();

    // ---- logits of this wavefront's cached-key tiles and window tile (Q K^T)
#pragma unroll
    for (int t = 0; t < TPW; t++) {
        f32x4 accL = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ks++) accL = mfma16(AQ[ks], BK[t][ks], accL);
        if (g4 == 0) {
#pragma unroll
            for (int i = 0; i < G; i++) lg[i][16 * (w + 4 * t) + r16] = accL[i] * a.scale;
        }
    }
    // window logits: one tile per wavefront
    if (w < NWT) {
        const int row = 16 * w + r16;
        f32x4 accL = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ks++) accL = mfma16(AQ[ks], BWin[ks], accL);
        if (g4 == 0) {
#pragma unroll
            for (int i = 0; i < G; i++) lg[i][KW + row] = accL[i] * a.scale;
        }
    }

    // ---- stage 1a: phi of this wavefront's query; stored as bf16 high + low parts in the operand layout of the
    // recall GEMM (row w + 1 of the extra tile).  Each 1 KB piece of W_q yields four projections: eight products per
    // lane, then a reduction over the 16 lanes of a row; lane (r16, g4) keeps projection j = 4 r16 + g4.
    if (steady && w < g) {
        const uint4 xq = reinterpret_cast<const uint4 *>(qb[w])[lane % PR];
        float z = 0.f;
#pragma unroll
        for (int it = 0; it < PR; it++) {
            float pz = dot2bf(wq[it].x, xq.x, 0.f); pz = dot2bf(wq[it].y, xq.y, pz);
            pz = dot2bf(wq[it].z, xq.z, pz); pz = dot2bf(wq[it].w, xq.w, pz);
            pz += dpp_f<0xB1>(pz); pz += dpp_f<0x4E>(pz); pz += dpp_f<0x141>(pz);
            if (PR == 16) pz += dpp_f<0x140>(pz);
            if (lane % PR == it) z = pz;
        }
        const int j = (64 / PR) * (lane % PR) + lane / PR;   // the projection this lane keeps
        float pp, pn;
        if (a.phi_kind == 1) { pp = fexp2(z * LOG2E); pn = fexp2(-z * LOG2E); }
        else {
            const float zmax = wmax(z), zmin = wmin(z);
            const float ep = fexp2((z - zmax) * LOG2E), en = fexp2((zmin - z) * LOG2E);
            pp = ep * frcp(wsum(ep)); pn = en * frcp(wsum(en));
        }
        const float dn = wsum(fmaf(pp, s_l[j], pn * s_l[M + j]));
        if (lane == 0) denq[w] = dn;
        // feature f sits in chunk (f / 32) * 4 + (f / 4) % 4, element 4 * ((f / 16) % 2) + f % 4
        const int row = w + 1;
#pragma unroll
        for (int half = 0; half < 2; half++) {
            const int f = half * M + j;
            const float val = half ? pn : pp;
            const int addr = row * D + (((((f >> 5) << 2) | ((f >> 2) & 3)) ^ row) << 3) + (((f >> 4) & 1) << 2) + (f & 3);
            const __bf16 hi = (__bf16)val;
            PX[addr] = __builtin_bit_cast(uint16_t, hi);
            PX[XR * D + addr] = __builtin_bit_cast(uint16_t, (__bf16)(val - (float)hi));
        }
    }
    // logit of the leaving key (it is attended if it stays in the cache)
    if (popped) {
        for (int r = w; r < g; r += 4) {
            float dot = wsum(lane < DH / 2 ? dot2bf(qb[r][lane % (DH / 2)], reinterpret_cast<const uint32_t *>(pkb)[lane % (DH / 2)], 0.f) : 0.f);
            if (lane == 0) lg[r][KP] = dot * a.scale;
        }
    }

    // ---- H^T rows of this wavefront are requested now and stay in registers until the fold writes them back:
    // lane (r16, g4) holds, for column tile ct and k-step ks, H^T[32w + 16ct + r16][32ks + 16 half + 4 g4 + 0..3]
    // (named scalars rather than an array: arrays of this size end up in scratch memory)
#define LOLA_HREP(X) X(0, 0, 0) X(0, 0, 1) X(0, 1, 0) X(0, 1, 1) X(0, 2, 0) X(0, 2, 1) X(0, 3, 0) X(0, 3, 1) \
                     X(1, 0, 0) X(1, 0, 1) X(1, 1, 0) X(1, 1, 1) X(1, 2, 0) X(1, 2, 1) X(1, 3, 0) X(1, 3, 1)
#define LOLA_HADDR(ct, ks, hf) ((size_t)(CW * w + 16 * ct + r16) * D + 32 * ks + 16 * hf + 4 * g4)
#define LOLA_HDECL(ct, ks, hf) float4 hreg##ct##ks##hf = make_float4(0.f, 0.f, 0.f, 0.f);
#define LOLA_HLOAD(ct, ks, hf) if (ct < NCT) hreg##ct##ks##hf = *reinterpret_cast<const float4 *>(Hg + LOLA_HADDR(ct, ks, hf));
    LOLA_HREP(LOLA_HDECL)
    if (steady) { LOLA_HREP(LOLA_HLOAD) }
    // cached values at this wavefront's value columns, wanted by the recall epilogue of every key tile: requested here,
    // right behind the state, so that their trip from HBM overlaps the feature map
    // (the first half of the tiles; the second half is requested when the recall GEMM starts and has four tiles' worth
    // of matrix work to arrive)
    constexpr int NKE = NKT / 2;
    uint2 vrec[NKT][NCT];
#pragma unroll
    for (int kt = 0; kt < NKT; kt++)
#pragma unroll
        for (int ct = 0; ct < NCT; ct++) {
            vrec[kt][ct] = make_uint2(0, 0);
            if (steady && kt < NKE) vrec[kt][ct] = *reinterpret_cast<const uint2 *>(sp_v + (size_t)(16 * kt + r16) * DH + CW * w + 16 * ct + 4 * g4);
        }

    // ---- stage 1b: logits Q K^T of this wavefront's key tiles; in steady state z^T = W_k K^T -> phi -> LDS.
    // Wavefront 0 also projects the leaving key (a tile with one real column).
    f32x4 zt[TPW + 1][4];
    if (steady) {
        bf16x8 BP[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ks++)
            BP[ks] = (w == 0 && r16 == 0) ? as_bf16x8(*reinterpret_cast<const uint4 *>(&pkb[32 * ks + 8 * g4])) : zero_bf16x8();
#pragma unroll
        for (int mt = 0; mt < 4; mt++) {
#pragma unroll
            for (int t = 0; t < TPW; t++) {
                zt[t][mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ks++) zt[t][mt] = mfma16(AW[mt][ks], BK[t][ks], zt[t][mt]);
            }
            zt[TPW][mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
            if (w == 0) {
#pragma unroll
                for (int ks = 0; ks < KS; ks++) zt[TPW][mt] = mfma16(AW[mt][ks], BP[ks], zt[TPW][mt]);
            }
        }
    }
    // operands of the listed pairs: A = phi_p (row = feature within a 16-block, k = p), B = v_p (column = value
    // index).  They are requested after the first key tile's feature map: from there on enough registers are free,
    // and the rest of the feature map covers their latency.
    float pa[RG][8], pb[RG][NCT];
    if (steady) {
#pragma unroll
        for (int t = 0; t < TPW; t++) {
            // cached keys, rows of PB
            const int row = 16 * (w + 4 * t) + r16;
            float pp[16], pn[16];
            phi_from_z(zt[t], a.phi_kind, pp, pn);
            float dn = 0.f;
#pragma unroll
            for (int mt = 0; mt < 4; mt++) {
                const float4 sp4 = *reinterpret_cast<const float4 *>(&s_l[16 * mt + 4 * g4]);
                const float4 sn4 = *reinterpret_cast<const float4 *>(&s_l[M + 16 * mt + 4 * g4]);
                dn = fmaf(pp[4 * mt], sp4.x, dn); dn = fmaf(pp[4 * mt + 1], sp4.y, dn);
                dn = fmaf(pp[4 * mt + 2], sp4.z, dn); dn = fmaf(pp[4 * mt + 3], sp4.w, dn);
                dn = fmaf(pn[4 * mt], sn4.x, dn); dn = fmaf(pn[4 * mt + 1], sn4.y, dn);
                dn = fmaf(pn[4 * mt + 2], sn4.z, dn); dn = fmaf(pn[4 * mt + 3], sn4.w, dn);
            }
            dn = grp_sum(dn);
            // feature order of the recall GEMM: ks 0,1 -> positive half (mt 0,1 / 2,3), ks 2,3 -> negative half;
            // the lane's eight values of a k-step are exactly chunk 4 ks + g4 of the row
            bf16x8 hi[4], lo[4];
            split8(&pp[0], hi[0], lo[0]); split8(&pp[8], hi[1], lo[1]);
            split8(&pn[0], hi[2], lo[2]); split8(&pn[8], hi[3], lo[3]);
            if (g4 == 0) rden_l[row] = dn > 0.f ? frcp(dn) : 0.f;
#pragma unroll
            for (int ks = 0; ks < 4; ks++) {
                const int addr = row * D + (((4 * ks + g4) ^ r16) << 3);
                *reinterpret_cast<uint4 *>(&PB[addr]) = __builtin_bit_cast(uint4, hi[ks]);
                *reinterpret_cast<uint4 *>(&PB[LAM * D + addr]) = __builtin_bit_cast(uint4, lo[ks]);
            }
            if (R > 0 && t == 0) {
                __builtin_amdgcn_sched_barrier(0);
                int lp = lane;
                asm volatile("" : "+v"(lp));
                const int pr = lp & 15, pg = lp >> 4;
#pragma unroll
                for (int gr = 0; gr < RG; gr++) {
                    const int pp_ = 4 * gr + pg;
                    const bool live = pp_ < cnt;
#pragma unroll
                    for (int x = 0; x < 8; x++) pa[gr][x] = live ? pphi[pp_ * D + 16 * x + pr] : 0.f;
#pragma unroll
                    for (int ct = 0; ct < NCT; ct++) pb[gr][ct] = live ? pval[pp_ * DH + CW * w + 16 * ct + pr] : 0.f;
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (w == 0) {
            // the leaving key (row 0 of the extra tile): its 64 projections sit in the four lanes of column 0; spread
            // over the wavefront (one projection per lane) the feature map costs a few wave reductions instead of a
            // whole tile's worth of arithmetic on 15 unused columns
            if (r16 == 0) {
#pragma unroll
                for (int mt = 0; mt < 4; mt++)
                    *reinterpret_cast<float4 *>(&zx[16 * mt + 4 * g4]) = make_float4(zt[TPW][mt][0], zt[TPW][mt][1], zt[TPW][mt][2], zt[TPW][mt][3]);
            }
            const float z = zx[lane];
            float pp, pn;
            if (a.phi_kind == 1) { pp = fexp2(z * LOG2E); pn = fexp2(-z * LOG2E); }
            else {
                const float zmax = wmax(z), zmin = wmin(z);
                const float ep = fexp2((z - zmax) * LOG2E), en = fexp2((zmin - z) * LOG2E);
                pp = ep * frcp(wsum(ep)); pn = en * frcp(wsum(en));
            }
            const float dn = wsum(fmaf(pp, s_l[lane], pn * s_l[M + lane]));
            if (lane == 0) rden_l[KP] = dn > 0.f ? frcp(dn) : 0.f;
#pragma unroll
            for (int half = 0; half < 2; half++) {
                const int f = half * M + lane;
                const float val = half ? pn : pp;
                const int addr = ((((f >> 5) << 2) | ((f >> 2) & 3)) << 3) + (((f >> 4) & 1) << 2) + (f & 3);   // row 0: no swizzle
                const __bf16 hi = (__bf16)val;
                PX[addr] = __builtin_bit_cast(uint16_t, hi);
                PX[XR * D + addr] = __builtin_bit_cast(uint16_t, (__bf16)(val - (float)hi));
            }
        }
    }
    if (popped && tid < PR) {   // (read by the recall epilogue and the fold, behind the next barrier)
        reinterpret_cast<uint4 *>(pvb)[tid] = p_ld;
        float *d = pvf + 8 * tid;
        d[0] = bf_lo(p_ld.x); d[1] = bf_hi(p_ld.x); d[2] = bf_lo(p_ld.y); d[3] = bf_hi(p_ld.y);
        d[4] = bf_lo(p_ld.z); d[5] = bf_hi(p_ld.z); d[6] = bf_lo(p_ld.w); d[7] = bf_hi(p_ld.w);
    }
    // Value rows for the read-out.  In steady state the cached rows are already in registers (the recall epilogue's
    // operands, kept until the feature tile is free), so only the rows behind them - the leaving pair, the window, the
    // zero rows that pad the last k-step - are fetched; while the cache fills, every row is.
    constexpr int NVIT = KPAD * PR / 256, NWIT = (KPAD - LAM) * PR / 256;
    static_assert(KPAD * PR % 256 == 0 && (KPAD - LAM) * PR % 256 == 0, "value staging is an exact number of passes");
    uint4 vst[NVIT];
    auto load_values = [&](auto first_key) {
        constexpr int K0 = decltype(first_key)::value;
#pragma unroll
        for (int it = 0; it < (KPAD - K0) * PR / 256; it++) {
            const int o = tid + 256 * it, key = K0 + o / PR, c8 = o % PR;
            vst[it] = make_uint4(0, 0, 0, 0);
            if (key < NKEY && key != KP) {
                const bf16_t *src;
                if (key < LAM) src = sp_v + (size_t)key * DH;
                else { const int row = key - KW; src = row == slot ? vnew : win_v + (size_t)row * DH; }
                vst[it] = reinterpret_cast<const uint4 *>(src)[c8];
            } else if (key == KP && popped) {
                vst[it] = reinterpret_cast<const uint4 *>(pvb)[c8];
            }
        }
    };
    int drop = -1;   // candidate that is folded: < LAM a cache slot, == LAM the leaving pair, -1 none
    if (steady) {
        // ---- stage 2: recall of all eligible pairs: P^T = H^T Phi^T; A = this wavefront's rows of H^T (bf16 high +
        // low parts made here), B = feature vectors from LDS
        bf16x8 Ahi[NCT][4], Alo[NCT][4];
        if (R > 0) {
#define LOLA_HPEND(ct, ks, hf) if (ct < NCT) { f32x4 c_ = {hreg##ct##ks##hf.x, hreg##ct##ks##hf.y, hreg##ct##ks##hf.z, hreg##ct##ks##hf.w}; \
            _Pragma("unroll") for (int gr = 0; gr < RG; gr++) c_ = __builtin_amdgcn_mfma_f32_16x16x4f32(pa[gr][2 * ks + hf], pb[gr][ct], c_, 0, 0, 0); \
            hreg##ct##ks##hf = make_float4(c_[0], c_[1], c_[2], c_[3]); }
            LOLA_HREP(LOLA_HPEND)
#undef LOLA_HPEND
        }
#define LOLA_HSPLIT(ct, ks, hf) if (ct < NCT) { const float4 v = hreg##ct##ks##hf; \
            const __bf16 h0 = (__bf16)v.x, h1 = (__bf16)v.y, h2 = (__bf16)v.z, h3 = (__bf16)v.w; \
            Ahi[ct][ks][4 * hf] = h0; Ahi[ct][ks][4 * hf + 1] = h1; Ahi[ct][ks][4 * hf + 2] = h2; Ahi[ct][ks][4 * hf + 3] = h3; \
            Alo[ct][ks][4 * hf] = (__bf16)(v.x - (float)h0); Alo[ct][ks][4 * hf + 1] = (__bf16)(v.y - (float)h1); \
            Alo[ct][ks][4 * hf + 2] = (__bf16)(v.z - (float)h2); Alo[ct][ks][4 * hf + 3] = (__bf16)(v.w - (float)h3); }
        LOLA_HREP(LOLA_HSPLIT)
#undef LOLA_HSPLIT
        lds_barrier();   // feature vectors and denominators of all eligible pairs are in LDS
        // Key tiles 0..NKT-1 are the cache slots; tile NKT is the extra tile (column 0: the leaving key, columns 1..G:
        // the queries, whose "recall" numerators are the linear read-out).  C layout: lane (column r16, group g4)
        // holds rows c = 32w + 16ct + 4 g4 + i.
#pragma unroll
        for (int kt = NKE; kt < NKT; kt++)
#pragma unroll
            for (int ct = 0; ct < NCT; ct++)
                vrec[kt][ct] = *reinterpret_cast<const uint2 *>(sp_v + (size_t)(16 * kt + r16) * DH + CW * w + 16 * ct + 4 * g4);
#pragma unroll
        for (int kt = 0; kt <= NKT; kt++) {
            const uint16_t *bh = kt < NKT ? PB + (16 * kt + r16) * D : PX + (r16 < XR ? r16 : 0) * D;
            const uint16_t *bl = kt < NKT ? bh + LAM * D : bh + XR * D;
            const int swz = kt < NKT ? r16 : (r16 < XR ? r16 : 0);
            // three passes (high x high, high x low, low x high) into one accumulator per row tile, the large products
            // first; the row tiles alternate, so a matrix instruction never waits on the one before it
            f32x4 acc[NCT];
#pragma unroll
            for (int ct = 0; ct < NCT; ct++) acc[ct] = (f32x4){0.f, 0.f, 0.f, 0.f};
            bf16x8 Bh[4], Bl[4];
#pragma unroll
            for (int ks = 0; ks < 4; ks++) {
                const int off = ((4 * ks + g4) ^ swz) << 3;
                Bh[ks] = as_bf16x8(*reinterpret_cast<const uint4 *>(bh + off));
                Bl[ks] = as_bf16x8(*reinterpret_cast<const uint4 *>(bl + off));
            }
#pragma unroll
            for (int pass = 0; pass < 3; pass++)
#pragma unroll
                for (int ks = 0; ks < 4; ks++)
#pragma unroll
                    for (int ct = 0; ct < NCT; ct++)
                        acc[ct] = mfma16(pass == 2 ? Alo[ct][ks] : Ahi[ct][ks], pass == 1 ? Bl[ks] : Bh[ks], acc[ct]);
            if (kt < NKT) {
                const float rd = rden_l[16 * kt + r16];
                float e2 = 0.f;
#pragma unroll
                for (int ct = 0; ct < NCT; ct++) {
                    const f32x4 p = acc[ct];
                    const uint2 vv = vrec[kt < NKT ? kt : 0][ct];
                    const float e0 = fmaf(p[0], rd, -bf_lo(vv.x)), e1 = fmaf(p[1], rd, -bf_hi(vv.x));
                    const float e2_ = fmaf(p[2], rd, -bf_lo(vv.y)), e3 = fmaf(p[3], rd, -bf_hi(vv.y));
                    e2 = fmaf(e0, e0, e2); e2 = fmaf(e1, e1, e2); e2 = fmaf(e2_, e2_, e2); e2 = fmaf(e3, e3, e2);
                }
                e2 = grp_sum(e2);
                if (g4 == 0) part[w][16 * kt + r16] = e2;
            } else {
                const float rd = rden_l[KP];
                float e2 = 0.f;
#pragma unroll
                for (int ct = 0; ct < NCT; ct++) {
                    const f32x4 p = acc[ct];
                    const int c0 = CW * w + 16 * ct + 4 * g4;
                    if (r16 == 0) {
#pragma unroll
                        for (int i = 0; i < 4; i++) { const float e = fmaf(p[i], rd, -pvf[c0 + i]); e2 = fmaf(e, e, e2); }
                    } else if (r16 <= g) {
#pragma unroll
                        for (int i = 0; i < 4; i++) lin[r16 - 1][c0 + i] = p[i];
                    }
                }
                e2 = grp_sum(e2);
                if (lane == 0) part[w][KP] = e2;
            }
        }
        lds_barrier();
        load_values(std::integral_constant<int, LAM>{});
        // ---- stage 3: the pair that leaves the cache: smallest error, ties -> larger token index
        // (every wavefront does the same search, which saves a barrier)
        {
            // one 64-bit key per candidate: the bits of the squared error (>= 0, so they order like an integer), then
            // the reversed token index; the smallest key is the pair to fold and keys are distinct
            unsigned long long kb = ~0ull; int be = 0;
            for (int e = lane; e <= LAM; e += WAVE) {
                const float sc = part[0][e] + part[1][e] + part[2][e] + part[3][e];
                const int ix = e < LAM ? idx_l[e] : pidx;
                const unsigned long long ke = ((unsigned long long)(__float_as_uint(sc) & 0x7FFFFFFFu) << 32) | (uint32_t)(0x7FFFFFFF - ix);
                if (ke < kb) { kb = ke; be = e; }
            }
            const unsigned long long kmin = wmin_u64(kb);
            const unsigned long long owner = __ballot(kb == kmin);
            drop = __builtin_amdgcn_readlane(be, (int)__builtin_ctzll(owner));
        }
        // phi and v of the folded pair (phi from its bf16 high + low parts)
        if (tid < D) {
            const int f = tid;
            const int chunk = ((f >> 5) << 2) | ((f >> 2) & 3), el = (((f >> 4) & 1) << 2) + (f & 3);
            const uint16_t *bh = drop < LAM ? PB + drop * D + ((chunk ^ (drop & 15)) << 3) + el : PX + (chunk << 3) + el;
            const uint16_t *bl = drop < LAM ? bh + LAM * D : bh + XR * D;
            phif[f] = bf_lo(*bh) + bf_lo(*bl);
            if (f < DH && drop == LAM) vf[f] = pvf[f];
        }
        if (drop < LAM) {
            // the folded slot's value row is among the recall epilogue's operands: the lanes of column drop % 16 hold it
            // at this wavefront's value columns (no second trip to memory behind the selection)
            uint2 sel[NCT];
#pragma unroll
            for (int ct = 0; ct < NCT; ct++) {
                sel[ct] = vrec[0][ct];
#pragma unroll
                for (int kt = 1; kt < NKT; kt++)
                    if ((drop >> 4) == kt) sel[ct] = vrec[kt][ct];
            }
            if (r16 == (drop & 15)) {
#pragma unroll
                for (int ct = 0; ct < NCT; ct++) {
                    float *d = vf + CW * w + 16 * ct + 4 * g4;
                    d[0] = bf_lo(sel[ct].x); d[1] = bf_hi(sel[ct].x); d[2] = bf_lo(sel[ct].y); d[3] = bf_hi(sel[ct].y);
                }
            }
        }
        lds_barrier();
        // the leaving pair takes the freed slot (in-place compaction)
        if (drop < LAM) {
            if (tid < PR) reinterpret_cast<uint4 *>(sp_k + (size_t)drop * DH)[tid] = reinterpret_cast<const uint4 *>(pkb)[tid];
            else if (tid < 2 * PR) reinterpret_cast<uint4 *>(sp_v + (size_t)drop * DH)[tid - PR] = reinterpret_cast<const uint4 *>(pvb)[tid - PR];
            else if (tid == 2 * PR) sp_idx[drop] = pidx;
        }
        // fold: without deferred folds H^T += v_f phi_f^T on the fp32 registers, written back at once; s += phi_f.
        // With deferred folds the pair is appended to the list; the step that finds the list full first writes its
        // registers (H^T plus the listed pairs) and s back and then starts a new list with its own pair.
        if (R == 0) {
#define LOLA_HFOLD(ct, ks, hf) if (ct < NCT) { const float vc = vf[CW * w + 16 * ct + r16]; \
            const float4 pf = *reinterpret_cast<const float4 *>(&phif[32 * ks + 16 * hf + 4 * g4]); \
            hreg##ct##ks##hf.x = fmaf(pf.x, vc, hreg##ct##ks##hf.x); hreg##ct##ks##hf.y = fmaf(pf.y, vc, hreg##ct##ks##hf.y); \
            hreg##ct##ks##hf.z = fmaf(pf.z, vc, hreg##ct##ks##hf.z); hreg##ct##ks##hf.w = fmaf(pf.w, vc, hreg##ct##ks##hf.w); \
            *reinterpret_cast<float4 *>(Hg + LOLA_HADDR(ct, ks, hf)) = hreg##ct##ks##hf; }
            LOLA_HREP(LOLA_HFOLD)
#undef LOLA_HFOLD
            if (tid < D) sg[tid] = s_l[tid] + phif[tid];
        } else {
            const bool full = cnt == R;
            if (full) {
#define LOLA_HSTORE(ct, ks, hf) if (ct < NCT) *reinterpret_cast<float4 *>(Hg + LOLA_HADDR(ct, ks, hf)) = hreg##ct##ks##hf;
                LOLA_HREP(LOLA_HSTORE)
#undef LOLA_HSTORE
                if (tid < D) sg[tid] = s_l[tid];
            }
            const int p_at = full ? 0 : cnt;
            if (tid < D) pphi[p_at * D + tid] = phif[tid];
            else if (tid < D + DH) pval[p_at * DH + tid - D] = vf[tid - D];
            if (tid == 0) a.pend_count[si] = p_at + 1;
        }
        // phi(q) . phi_f for the rank-1 correction of the linear read-out
        for (int r = w; r < g; r += 4) {
            float acc = 0.f;
#pragma unroll
            for (int half = 0; half < 2; half++) {
                const int f = half * M + lane, row = r + 1;
                const int addr = row * D + (((((f >> 5) << 2) | ((f >> 2) & 3)) ^ row) << 3) + (((f >> 4) & 1) << 2) + (f & 3);
                acc = fmaf(bf_lo(PX[addr]) + bf_lo(PX[XR * D + addr]), phif[f], acc);
            }
            acc = wsum(acc);
            if (lane == 0) dotqf[r] = acc;
        }
    } else {
        lds_barrier();   // logits of all wavefronts and the leaving pair's value row are in LDS (the steady path has passed barriers of its own)
        load_values(std::integral_constant<int, 0>{});
    }
#undef LOLA_HDECL
#undef LOLA_HLOAD
#undef LOLA_HADDR
#undef LOLA_HREP
    if (!steady && popped) {
        // cache not full yet: the leaving pair is appended, nothing is scored (spc < LAM)
        if (tid < PR) reinterpret_cast<uint4 *>(sp_k + (size_t)spc * DH)[tid] = reinterpret_cast<const uint4 *>(pkb)[tid];
        else if (tid < 2 * PR) reinterpret_cast<uint4 *>(sp_v + (size_t)spc * DH)[tid - PR] = reinterpret_cast<const uint4 *>(pvb)[tid - PR];
        else if (tid == 2 * PR) { sp_idx[spc] = pidx; a.st.sp_count[si] = spc + 1; }
    }

    // ---- stage 4: value rows into LDS (the feature tile is no longer needed): [key][c], key order = logit order; rows
    // past the last key are zero.  The dropped slot's row is the old one, or mid-overwrite while the cache fills: its weight is 0.
    // 8-byte piece p of row `key` sits at piece p ^ vswz(key) (a multiple of 4 taken from the row bits that differ
    // between the eight rows two lane groups read at once): the transposing reads below then touch every bank once
    auto vswz = [](int key) { return DH == 128 ? 4 * (key & 7) : 4 * ((key >> 1) & 3); };
    if (steady) {
        // cached rows from the registers of the recall epilogue: lane (r16, g4) holds, per key tile and row tile, the
        // 8-byte piece (CW w + 16 ct) / 4 + g4 of row 16 kt + r16
#pragma unroll
        for (int kt = 0; kt < NKT; kt++)
#pragma unroll
            for (int ct = 0; ct < NCT; ct++) {
                const int key = 16 * kt + r16, pc = (CW / 4) * w + 4 * ct + g4;
                *reinterpret_cast<uint2 *>(Vl + key * VLS + 4 * (pc ^ vswz(key))) = vrec[kt][ct];
            }
#pragma unroll
        for (int it = 0; it < NWIT; it++) {
            const int o = tid + 256 * it, key = LAM + o / PR, c8 = o % PR;
            *reinterpret_cast<uint4 *>(Vl + key * VLS + 4 * ((2 * c8) ^ vswz(key))) = vst[it];
        }
    } else {
#pragma unroll
        for (int it = 0; it < NVIT; it++) {
            const int o = tid + 256 * it, key = o / PR, c8 = o % PR;
            *reinterpret_cast<uint4 *>(Vl + key * VLS + 4 * ((2 * c8) ^ vswz(key))) = vst[it];
        }
    }
    // the new pair, which takes the ring slot of the pair that left, is requested here and stored at the very end
    // (a store that follows its own load waits for every load the wavefront has in flight: by then there is none)
    uint4 new_ld = make_uint4(0, 0, 0, 0);
    if (tid < 2 * PR) new_ld = reinterpret_cast<const uint4 *>(tid < PR ? knew : vnew)[tid % PR];
    // softmax weights (one query per wavefront), m = max(0, max logit); written as bf16 high + low parts
    for (int r = w; r < g; r += 4) {
        float l[(KPAD + 63) / 64];
        float mx = 0.f;
#pragma unroll
        for (int x = 0; x < (KPAD + 63) / 64; x++) {
            const int key = lane + 64 * x;
            bool ok = false;
            if (key < LAM) ok = key < spc && key != drop && !(a.hide & 2);
            else if (key == KP) ok = popped && drop != LAM && !(a.hide & 2);   // it sits in the sparse cache now
            else if (key < NKEY) ok = (key - KW) < wn;
            l[x] = ok ? lg[r][key] : -INFINITY;
            mx = fmaxf(mx, l[x]);
        }
        mx = wmax(mx);
        float sum = 0.f;
#pragma unroll
        for (int x = 0; x < (KPAD + 63) / 64; x++) {
            const int key = lane + 64 * x;
            const float p = fexp2((l[x] - mx) * LOG2E);
            sum += p;
            if (key < KPAD) {
                const __bf16 ph = (__bf16)p;
                Ph[r * KPAD + key] = __builtin_bit_cast(uint16_t, ph);
                Pl[r * KPAD + key] = __builtin_bit_cast(uint16_t, (__bf16)(p - (float)ph));
            }
        }
        sum = wsum(sum);
        if (lane == 0) { psum_s[r] = sum; elin_s[r] = fexp2(-mx * LOG2E); }
    }
    lds_barrier();

    // ---- stage 5: out[q][c] = sum_key p[q][key] v[key][c] on MFMA: A = weights (rows = queries), B = staged values
    // (column c, k = key); each wavefront owns CW output columns
    {
        f32x4 acc[NCT];
#pragma unroll
        for (int nt = 0; nt < NCT; nt++) acc[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < NKS; ks++) {
            // contraction slots of lane group g4: keys 32 ks + 4 g4 + 0..3, then 32 ks + 16 + 4 g4 + 0..3 (the order in which
            // the transposing LDS read delivers the values; the weights follow it)
            const int k0 = 32 * ks + 4 * g4;
            bf16x8 Aph = zero_bf16x8(), Apl = zero_bf16x8();
            if (r16 < g) {
                const uint2 h0 = *reinterpret_cast<const uint2 *>(&Ph[r16 * KPAD + k0]), h1 = *reinterpret_cast<const uint2 *>(&Ph[r16 * KPAD + k0 + 16]);
                const uint2 l0 = *reinterpret_cast<const uint2 *>(&Pl[r16 * KPAD + k0]), l1 = *reinterpret_cast<const uint2 *>(&Pl[r16 * KPAD + k0 + 16]);
                Aph = as_bf16x8(make_uint4(h0.x, h0.y, h1.x, h1.y));
                Apl = as_bf16x8(make_uint4(l0.x, l0.y, l1.x, l1.y));
            }
#pragma unroll
            for (int nt = 0; nt < NCT; nt++) {
                // a 16-lane group reads a 4 x 16 block of the row-major values (lane i: row i / 4, columns 4 (i % 4) ..) and
                // receives it transposed: lane j holds column j of the four rows
                const int row = k0 + (r16 >> 2), piece = 4 * (NCT * w + nt) + (r16 & 3);
                const bf16x4 t0 = tr_read(Vl + row * VLS + 4 * (piece ^ vswz(row)));
                const bf16x4 t1 = tr_read(Vl + (row + 16) * VLS + 4 * (piece ^ vswz(row + 16)));
                const bf16x8 Bv = __builtin_shufflevector(t0, t1, 0, 1, 2, 3, 4, 5, 6, 7);
                acc[nt] = mfma16(Aph, Bv, acc[nt]);
                acc[nt] = mfma16(Apl, Bv, acc[nt]);
            }
        }
        if (g4 == 0) {
#pragma unroll
            for (int nt = 0; nt < NCT; nt++) {
                const int c = 16 * (NCT * w + nt) + r16;
#pragma unroll
                for (int r = 0; r < G; r++) {
                    if (r >= g) break;
                    float num = acc[nt][r], den = psum_s[r];
                    if (steady && !(a.hide & 1)) {
                        const float el = elin_s[r];
                        num = fmaf(el, fmaf(dotqf[r], vf[c], lin[r][c]), num);
                        den = fmaf(el, denq[r] + dotqf[r], den);
                    }
                    stf(a.out, ((size_t)b * a.Hq + (size_t)h * g + r) * DH + c, num * frcp(den));
                }
            }
        }
    }
    // the new pair takes the ring slot of the pair that left (read in stage 0)
    if (tid < 2 * PR) reinterpret_cast<uint4 *>(tid < PR ? win_k + (size_t)slot * DH : win_v + (size_t)slot * DH)[tid % PR] = new_ld;
    if (tid == 0) a.st.n_tokens[si] = tok + 1;
}

}  // namespace fast
}  // namespace lola

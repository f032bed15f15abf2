// Shared device-side helpers of the LoLA kernels (gfx950 only, 64-lane wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lola {

constexpr int WAVE = 64;

struct bf16_t { uint16_t x; };

// Dimensions of one layer as the kernels see them.
struct Dims {
    int B, Hq, Hkv, g;      // g = Hq / Hkv query heads per kv head
    int d, D, m;            // head_dim, feature dim, m = D / 2
    int eta, lam, C;        // window, sparse budget, prefill chunk
    int phi_kind;           // 0 softmax kind, 1 exponential kind
    float scale;            // logit scale
    int hide;               // bit 0: queries do not read (H, s); bit 1: queries do not read the sparse cache
    int score_kind;         // 0 self-recall error; 1..4 the query-dependent scores of the scoring ablation
};

// Device pointers of the memories (layout documented in include/lola.h).
template <typename T>
struct State {
    float *H, *s;
    T *win_k, *win_v, *sp_k, *sp_v;
    int32_t *sp_idx, *sp_count;
    int64_t *n_tokens;
    float *win_score, *sp_score;   // query-dependent scores only: per ring slot / per sparse slot
};

__device__ __forceinline__ float ldf(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float ldf(const bf16_t *p, size_t i) {
    return __uint_as_float(((uint32_t)p[i].x) << 16);
}
__device__ __forceinline__ void stf(float *p, size_t i, float v) { p[i] = v; }
// round to nearest even; inputs here are finite
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float v) {
    uint32_t u = __float_as_uint(v);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ void stf(bf16_t *p, size_t i, float v) { p[i].x = f32_to_bf16_bits(v); }

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every global load and store the
// wavefront has in flight (and so does a workgroup fence restricted to LDS once the kernel holds direct global -> LDS
// loads), which ends all prefetching at each barrier; this form waits for the wavefront's LDS operations alone and
// leaves its global requests in flight.  The "memory" clobber keeps the compiler from moving memory accesses across
// it.  It may stand wherever the wavefronts of a workgroup exchange data through LDS alone: data that one wavefront
// writes to global memory and another reads back in the same launch still needs __syncthreads().  Direct global -> LDS
// loads are waited for by the wavefront that issued them, with an explicit s_waitcnt, before it enters the barrier.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Direct global -> LDS load of 16 bytes per lane (1 KB per wavefront: lane l fills bytes 16 l .. of the block at
// lds_dst, which must be the same for all lanes), issued as inline assembly.  The compiler orders every LDS read that it
// cannot prove disjoint behind the direct loads it knows of, which serialises a batch's reads with the requests of
// the next batch; loads issued here are invisible to that bookkeeping and are waited for by hand (s_waitcnt vmcnt
// counts them like any other load, in order, so the compiler's own waits only ever become longer, never too short).
// A kernel that uses this form uses it for all its direct loads: M0 is written here without the compiler knowing.
__device__ __forceinline__ void lds_dma16(const void *gsrc, void *lds_dst) {
    const uint32_t l = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)lds_dst);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" :: "s"(l), "v"(gsrc) : "memory");
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
    return v;
}
__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o, WAVE));
    return v;
}

}  // namespace lola

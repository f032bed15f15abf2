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

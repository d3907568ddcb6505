// Element arithmetic of the decoder glue that can be fused around a Linear (RMSNorm before the QKV
// and gate+up projections, SwiGLU before the down projection, the residual add after the attention
// output and down projections).  The stand-alone kernels and the fused M == 1 prologues both call
// these helpers, so that an element is computed the same way wherever it is computed:
//   rmsnorm  RNE_bf16((x * scale) * gamma),  scale = rsq(sum(x^2) / K + eps)         (0 for an all-zero row)
//   swiglu   RNE_bf16((gate * rcp(1 + exp(-gate))) * up)
// in fp32, with the hardware's reciprocal, reciprocal square root and exp2 (about 1 ulp of fp32 each:
// the result is rounded to bf16, 16 bits coarser, right after, and on the small decode layers the
// prologue sits on the critical path, where the correctly rounded sequences cost about 1 us).
// A piece is 8 consecutive bf16 values (one 16-byte access).
#pragma once
#include "common.hpp"

namespace dmr {

enum Prologue { kProNone = 0, kProRmsNorm = 1, kProSwiGLU = 2 };

// What an M == 1 forward fuses: a prologue on the activation row (aux = gamma for RMSNorm; for
// SwiGLU the activation pointer holds the gate half followed by the up half) and a bf16 residual
// added to the fp32 result before the output rounding.
struct Fusion {
    int pro = kProNone;
    const uint16_t *aux = nullptr;
    float eps = 0.f;
    const uint16_t *res = nullptr;
};

__device__ __forceinline__ float sumsq_piece(const uint4 &x) {
    const uint32_t w[4] = {x.x, x.y, x.z, x.w};
    float s = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const float lo = __uint_as_float(w[q] << 16), hi = __uint_as_float(w[q] & 0xFFFF0000u);
        s = fmaf(lo, lo, s);
        s = fmaf(hi, hi, s);
    }
    return s;
}

__device__ __forceinline__ float rms_scale(float sumsq, float inv_k, float eps) {
    const float v = fmaf(sumsq, inv_k, eps);
    return v > 0.f ? __builtin_amdgcn_rsqf(v) : 0.f;
}

// Sum over the 64 lanes of a wave, the same value in every lane: DPP row sums, then the four row sums
// through scalar registers (no LDS round trip).
__device__ __forceinline__ float wave64_sum(float v) {
    v = row16_sum(v);
    const int b = __float_as_int(v);
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(b, 0)), r1 = __int_as_float(__builtin_amdgcn_readlane(b, 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(b, 32)), r3 = __int_as_float(__builtin_amdgcn_readlane(b, 48));
    return (r0 + r1) + (r2 + r3);
}

__device__ __forceinline__ uint4 rmsnorm_piece(const uint4 &x, const uint4 &gamma, float scale) {
    const uint32_t w[4] = {x.x, x.y, x.z, x.w}, g[4] = {gamma.x, gamma.y, gamma.z, gamma.w};
    uint32_t o[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const float lo = (__uint_as_float(w[q] << 16) * scale) * __uint_as_float(g[q] << 16);
        const float hi = (__uint_as_float(w[q] & 0xFFFF0000u) * scale) * __uint_as_float(g[q] & 0xFFFF0000u);
        o[q] = pack_bf16x2(lo, hi);
    }
    return make_uint4(o[0], o[1], o[2], o[3]);
}

__device__ __forceinline__ float silu(float a) { return a * __builtin_amdgcn_rcpf(1.0f + __expf(-a)); }

__device__ __forceinline__ uint4 swiglu_piece(const uint4 &gate, const uint4 &up) {
    const uint32_t g[4] = {gate.x, gate.y, gate.z, gate.w}, u[4] = {up.x, up.y, up.z, up.w};
    uint32_t o[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const float lo = silu(__uint_as_float(g[q] << 16)) * __uint_as_float(u[q] << 16);
        const float hi = silu(__uint_as_float(g[q] & 0xFFFF0000u)) * __uint_as_float(u[q] & 0xFFFF0000u);
        o[q] = pack_bf16x2(lo, hi);
    }
    return make_uint4(o[0], o[1], o[2], o[3]);
}

// Stand-alone kernels (any M).
hipError_t launch_rmsnorm(const uint16_t *x, const uint16_t *gamma, float eps, int64_t M, int64_t K, uint16_t *out,
                          hipStream_t stream);
hipError_t launch_swiglu(const uint16_t *in, int64_t M, int64_t I, uint16_t *out, hipStream_t stream);
// out = RNE(acc + res): acc fp32 [count], res bf16 [count], out fp32 or bf16.
hipError_t launch_add_residual(const float *acc, const uint16_t *res, int64_t count, void *out, bool out_f32,
                               hipStream_t stream);

// Weight-streaming forwards with fused glue; hipErrorInvalidValue (nothing launched) for what they do not take.
hipError_t launch_w4_gemv_fused(const LayerView &L, const uint16_t *x, void *y, bool out_f32, const Fusion &f,
                                hipStream_t stream);
// 2 <= M <= 16 with the rows whole in LDS.
hipError_t launch_w4_stream_fused(const LayerView &L, const uint16_t *x, int64_t M, void *y, bool out_f32,
                                  const Fusion &f, hipStream_t stream);
hipError_t launch_bf16_gemv_fused(const uint16_t *w, const uint16_t *x, int64_t K, int64_t N, void *y, bool out_f32,
                                  const Fusion &f, hipStream_t stream);

}  // namespace dmr

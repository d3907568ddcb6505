// Stand-alone decoder glue kernels (any M): RMSNorm, SwiGLU, residual add.  At M == 1 the forwards
// fuse the same arithmetic into their activation staging instead (glue.hpp).
#include "glue.hpp"

namespace dmr {

namespace {

// One workgroup per row: pieces round-robin over 256 threads, sum of squares through DPP / LDS.
__global__ __launch_bounds__(256) void rmsnorm_kernel(const uint16_t *__restrict__ x,
                                                      const uint16_t *__restrict__ gamma, float eps, int64_t K,
                                                      uint16_t *__restrict__ out) {
    __shared__ float part[4];
    const int64_t row = blockIdx.x;
    const uint4 *src = reinterpret_cast<const uint4 *>(x + row * K);
    const uint4 *gsrc = reinterpret_cast<const uint4 *>(gamma);
    uint4 *dst = reinterpret_cast<uint4 *>(out + row * K);
    const int pieces = (int)(K / 8);
    float ss = 0.f;
    for (int i = threadIdx.x; i < pieces; i += 256) ss += sumsq_piece(src[i]);
    ss = wave64_sum(ss);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float scale = rms_scale((part[0] + part[1]) + (part[2] + part[3]), 1.0f / (float)K, eps);
    for (int i = threadIdx.x; i < pieces; i += 256) dst[i] = rmsnorm_piece(src[i], gsrc[i], scale);
}

__global__ __launch_bounds__(256) void swiglu_kernel(const uint16_t *__restrict__ in, int64_t M, int64_t I,
                                                     uint16_t *__restrict__ out) {
    const int64_t pieces_per_row = I / 8;
    const int64_t slot = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (slot >= M * pieces_per_row) return;
    const int64_t m = slot / pieces_per_row, i = slot % pieces_per_row;
    const uint4 *row = reinterpret_cast<const uint4 *>(in + m * 2 * I);
    reinterpret_cast<uint4 *>(out + m * I)[i] = swiglu_piece(row[i], row[pieces_per_row + i]);
}

__global__ __launch_bounds__(256) void add_residual_kernel(const float *__restrict__ acc,
                                                           const uint16_t *__restrict__ res, int64_t count,
                                                           void *__restrict__ out, int out_f32) {
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= count) return;
    const f32x4 a = *reinterpret_cast<const f32x4 *>(acc + i);
    const uint2 r = *reinterpret_cast<const uint2 *>(res + i);
    f32x4 v;
    v[0] = a[0] + __uint_as_float(r.x << 16);
    v[1] = a[1] + __uint_as_float(r.x & 0xFFFF0000u);
    v[2] = a[2] + __uint_as_float(r.y << 16);
    v[3] = a[3] + __uint_as_float(r.y & 0xFFFF0000u);
    if (out_f32) {
        *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(out) + i) = v;
    } else {
        uint2 o;
        o.x = pack_bf16x2(v[0], v[1]);
        o.y = pack_bf16x2(v[2], v[3]);
        *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(out) + i) = o;
    }
}

}  // namespace

hipError_t launch_rmsnorm(const uint16_t *x, const uint16_t *gamma, float eps, int64_t M, int64_t K, uint16_t *out,
                          hipStream_t stream) {
    hipLaunchKernelGGL(rmsnorm_kernel, dim3((unsigned)M), dim3(256), 0, stream, x, gamma, eps, K, out);
    return hipGetLastError();
}

hipError_t launch_swiglu(const uint16_t *in, int64_t M, int64_t I, uint16_t *out, hipStream_t stream) {
    const int64_t slots = M * (I / 8);
    hipLaunchKernelGGL(swiglu_kernel, dim3((unsigned)((slots + 255) / 256)), dim3(256), 0, stream, in, M, I, out);
    return hipGetLastError();
}

hipError_t launch_add_residual(const float *acc, const uint16_t *res, int64_t count, void *out, bool out_f32,
                               hipStream_t stream) {
    hipLaunchKernelGGL(add_residual_kernel, dim3((unsigned)((count / 4 + 255) / 256)), dim3(256), 0, stream, acc, res,
                       count, out, out_f32 ? 1 : 0);
    return hipGetLastError();
}

}  // namespace dmr

// One-off, integer-mostly kernels around the streaming layout: re-tile at create time,
// dequantize (the parity anchor of the layout), and the round-to-nearest quantiser that
// produces canonical inputs on the device.
#include "common.hpp"

namespace dmr {

// ---- re-tile: canonical [N][K/8] words + [N][K/128] scales/zeros -> streaming blocks ----------
// One thread per 16-byte lane slot (T, G, l): its four words are canonical words 16G+4c..+3 of
// row 16T+j, which are contiguous, so the read and the write are both one 128-bit access.
__global__ __launch_bounds__(256) void retile_kernel(int64_t K, int64_t N,
                                                     const uint32_t *__restrict__ qweight,
                                                     const uint16_t *__restrict__ scales,
                                                     const uint16_t *__restrict__ zeros,
                                                     uint4 *__restrict__ wt,
                                                     uint32_t *__restrict__ sz, int per_channel) {
    const int64_t groups = K / kGroup;
    const int64_t slot = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t slots = N * K / 32;
    if (slot >= slots) return;
    const int l = (int)(slot & 63);
    const int64_t block = slot >> 6;
    const int64_t T = block / groups, G = block % groups;
    const int c = l >> 4, j = l & 15;
    const int64_t n = T * kTileRows + j;
    const uint4 src = *reinterpret_cast<const uint4 *>(qweight + n * (K / 8) + G * 16 + c * 4);
    const uint32_t in[4] = {src.x, src.y, src.z, src.w};
    uint32_t out[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        uint32_t w = 0;
#pragma unroll
        for (int p = 0; p < 8; ++p)
            w |= ((in[t] >> (4 * p)) & 0xFu) << (4 * nibble_of_position(p));
        out[t] = w;
    }
    wt[slot] = make_uint4(out[0], out[1], out[2], out[3]);
    if (c == 0 && (!per_channel || G == 0)) {
        // per-channel symmetric layers carry one scale per row and the fixed zero point 8: one word per row
        const uint32_t s_bits = per_channel ? scales[n] : scales[n * groups + G];
        const float z = per_channel ? 8.0f : bf16_bits_to_f32(zeros[n * groups + G]);
        const uint32_t cz_bits = __float_as_uint(-(128.0f + z)) >> 16;   // exact in bf16
        sz[sz_index(T, G, groups, per_channel ? 0 : 1, j)] = s_bits | (cz_bits << 16);
    }
}

hipError_t launch_retile(int64_t K, int64_t N, const uint32_t *qweight, const uint16_t *scales,
                         const uint16_t *zeros, uint4 *wt, uint32_t *sz, bool per_channel,
                         hipStream_t stream) {
    const int64_t slots = N * K / 32;
    const unsigned blocks = (unsigned)((slots + 255) / 256);
    hipLaunchKernelGGL(retile_kernel, dim3(blocks), dim3(256), 0, stream, K, N, qweight, scales, zeros,
                       wt, sz, per_channel ? 1 : 0);
    return hipGetLastError();
}

// ---- dequantize: streaming blocks -> bf16 [N][K] = RNE_bf16((q - z) * s) ----------------------
__global__ __launch_bounds__(256) void dequantize_kernel(int64_t K, int64_t N,
                                                         const uint4 *__restrict__ wt,
                                                         const uint32_t *__restrict__ sz,
                                                         uint16_t *__restrict__ w_bf16, int szs) {
    const int64_t groups = K / kGroup;
    const int64_t slot = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (slot >= N * K / 32) return;
    const int l = (int)(slot & 63);
    const int64_t block = slot >> 6;
    const int64_t T = block / groups, G = block % groups;
    const int c = l >> 4, j = l & 15;
    const int64_t n = T * kTileRows + j;
    const uint4 src = wt[slot];
    const uint32_t szw = sz[sz_index(T, G, groups, szs, j)];
    const float s = bf16_bits_to_f32(szw & 0xFFFFu);
    const float z = -bf16_bits_to_f32(szw >> 16) - 128.0f;
    const uint32_t in[4] = {src.x, src.y, src.z, src.w};
    uint4 *dst = reinterpret_cast<uint4 *>(w_bf16 + n * K + G * kGroup + c * 32);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        uint32_t o[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            // (q - z) * s: a 5-bit integer times an 8-bit significand, exact in fp32
            const float lo = ((float)((in[t] >> (4 * nibble_of_position(2 * i))) & 0xFu) - z) * s;
            const float hi = ((float)((in[t] >> (4 * nibble_of_position(2 * i + 1))) & 0xFu) - z) * s;
            o[i] = pack_bf16x2(lo, hi);
        }
        dst[t] = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

hipError_t launch_dequantize(const LayerView &L, uint16_t *w_bf16, hipStream_t stream) {
    const int64_t slots = L.N * L.K / 32;
    const unsigned blocks = (unsigned)((slots + 255) / 256);
    hipLaunchKernelGGL(dequantize_kernel, dim3(blocks), dim3(256), 0, stream, L.K, L.N, L.wt, L.sz,
                       w_bf16, L.szs);
    return hipGetLastError();
}

// ---- quantise: fp32 [N][K] -> canonical codes, scales, zero points (round to nearest) --------
// 16 consecutive lanes share one group of 128 weights (8 each): range by a 16-lane butterfly,
// then every lane derives the same scale and zero point in fp64 and packs its own word.
__global__ __launch_bounds__(256) void quantize_kernel(int64_t K, int64_t N,
                                                       const float *__restrict__ w,
                                                       uint32_t *__restrict__ qweight,
                                                       uint16_t *__restrict__ scales,
                                                       uint16_t *__restrict__ zeros) {
    const int64_t word = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // canonical word index
    const bool live = word < N * K / 8;
    float v[8];
    float lo = 0.0f, hi = 0.0f;
    if (live) {
        const float4 a = *reinterpret_cast<const float4 *>(w + word * 8);
        const float4 b = *reinterpret_cast<const float4 *>(w + word * 8 + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
        v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            lo = fminf(lo, v[i]);
            hi = fmaxf(hi, v[i]);
        }
    }
#pragma unroll
    for (int mask = 1; mask < 16; mask <<= 1) {
        lo = fminf(lo, __shfl_xor(lo, mask, 16));
        hi = fmaxf(hi, __shfl_xor(hi, mask, 16));
    }
    if (!live) return;
    const float s32 = (float)(((double)hi - (double)lo) / 15.0);
    uint32_t s_bits = f32_to_bf16(s32);
    double s = (double)bf16_bits_to_f32(s_bits);
    if (s == 0.0) {
        s = 1.0;
        s_bits = 0x3F80u;
    }
    double z = rint(-(double)lo / s);
    z = (z > 0.0) ? fmin(z, 15.0) : 0.0;   // code 0 is +0 also when -lo / s is -0
    uint32_t packed = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        double c = rint((double)v[i] / s) + z;
        c = fmin(fmax(c, 0.0), 15.0);
        packed |= (uint32_t)(int)c << (4 * i);
    }
    qweight[word] = packed;
    if ((word & 15) == 0) {
        const int64_t group = word >> 4;     // (n, G) flattened: rows hold K/128 groups each
        scales[group] = (uint16_t)s_bits;
        zeros[group] = f32_to_bf16((float)z);
    }
}

hipError_t launch_quantize(int64_t K, int64_t N, const float *w, uint32_t *qweight, uint16_t *scales,
                           uint16_t *zeros, hipStream_t stream) {
    const int64_t words = N * K / 8;
    const unsigned blocks = (unsigned)((words + 255) / 256);
    hipLaunchKernelGGL(quantize_kernel, dim3(blocks), dim3(256), 0, stream, K, N, w, qweight, scales,
                       zeros);
    return hipGetLastError();
}

}  // namespace dmr

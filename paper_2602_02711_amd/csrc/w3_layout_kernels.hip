// One-off kernels of the 3-bit (W3A16, group 128) variant: re-tile canonical words into streaming
// blocks, dequantize (the parity anchor), and the round-to-nearest quantiser.
//
// Canonical: 32 codes per three words, code j in bits [3j, 3j+3) of the 96-bit little-endian run.
// Streaming: block (T, G) = 64 lanes x 3 words; lane l = 16 c + j owns row 16 T + j and the weights
// k = 128 G + 32 c + i, i = 0..31, as 16 operand registers r = i / 2 (code 2r in the low half, 2r + 1
// in the high half).  Every byte of the three words holds two codes, bits [0, 3) and [3, 6), so that
// one mask isolates four codes as clean bytes: register r < 12 takes word r / 4, field (r / 2) % 2,
// bytes (r % 2) and (r % 2) + 2.  The two spare bits of each byte carry the last eight codes:
// registers 12, 13 (14, 15) have their low two bits in bits [6, 8) of the bytes of word 0 (word 1)
// and their third bit in bit 6 (bit 7) of the same byte of word 2.
#include "common.hpp"

namespace dmr {

namespace {

// codes[32] -> the lane's three streaming words
__device__ __forceinline__ void encode_lane(const uint32_t (&code)[32], uint32_t (&w)[3]) {
    w[0] = w[1] = w[2] = 0;
#pragma unroll
    for (int r = 0; r < 12; ++r) {
        const int v = r / 4, f = (r / 2) % 2, p = r % 2;
        w[v] |= code[2 * r] << (8 * p + 3 * f);
        w[v] |= code[2 * r + 1] << (8 * (p + 2) + 3 * f);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int cc = e / 4, idx = e % 4;
        const int b = ((idx & 1) << 1) | (idx >> 1);       // codes of a register sit in bytes (0, 2) or (1, 3)
        w[cc] |= (code[24 + e] & 3u) << (8 * b + 6);
        w[2] |= (code[24 + e] >> 2) << (8 * b + 6 + cc);
    }
}

__device__ __forceinline__ uint32_t decode_lane(const uint32_t (&w)[3], int i) {
    const int r = i >> 1, h = i & 1;
    if (r < 12) {
        const int v = r / 4, f = (r / 2) % 2, p = r % 2;
        return (w[v] >> (8 * (p + 2 * h) + 3 * f)) & 7u;
    }
    const int e = i - 24, cc = e / 4, idx = e % 4;
    const int b = ((idx & 1) << 1) | (idx >> 1);
    return ((w[cc] >> (8 * b + 6)) & 3u) | (((w[2] >> (8 * b + 6 + cc)) & 1u) << 2);
}

}  // namespace

__global__ __launch_bounds__(256) void retile3_kernel(int64_t K, int64_t N,
                                                      const uint32_t *__restrict__ qweight,
                                                      const uint16_t *__restrict__ scales,
                                                      const uint16_t *__restrict__ zeros,
                                                      uint32_t *__restrict__ wt, uint32_t *__restrict__ sz) {
    const int64_t groups = K / kGroup;
    const int64_t slot = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (slot >= N * K / 32) return;
    const int l = (int)(slot & 63);
    const int64_t block = slot >> 6;
    const int64_t T = block / groups, G = block % groups;
    const int c = l >> 4, j = l & 15;
    const int64_t n = T * kTileRows + j;
    // the lane's 32 codes are one canonical run of three words
    const uint32_t *src = qweight + (n * (K / 32) + G * 4 + c) * 3;
    const uint32_t in[3] = {src[0], src[1], src[2]};
    uint32_t code[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        const int wi = (3 * i) >> 5, o = (3 * i) & 31;            // compile-time after unrolling
        uint32_t bits3 = in[wi] >> o;
        if (o > 29) bits3 |= in[wi + 1] << (32 - o);              // the field straddles two words
        code[i] = bits3 & 7u;
    }
    uint32_t out[3];
    encode_lane(code, out);
    wt[slot * 3 + 0] = out[0];
    wt[slot * 3 + 1] = out[1];
    wt[slot * 3 + 2] = out[2];
    if (c == 0) {
        const uint32_t s_bits = scales[n * groups + G];
        const float z = bf16_bits_to_f32(zeros[n * groups + G]);
        const uint32_t cz_bits = __float_as_uint(-(128.0f + z)) >> 16;
        sz[block * kTileRows + j] = s_bits | (cz_bits << 16);
    }
}

__global__ __launch_bounds__(256) void dequantize3_kernel(int64_t K, int64_t N,
                                                          const uint32_t *__restrict__ wt,
                                                          const uint32_t *__restrict__ sz,
                                                          uint16_t *__restrict__ w_bf16) {
    const int64_t groups = K / kGroup;
    const int64_t slot = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (slot >= N * K / 32) return;
    const int l = (int)(slot & 63);
    const int64_t block = slot >> 6;
    const int64_t T = block / groups, G = block % groups;
    const int c = l >> 4, j = l & 15;
    const int64_t n = T * kTileRows + j;
    const uint32_t w[3] = {wt[slot * 3], wt[slot * 3 + 1], wt[slot * 3 + 2]};
    const uint32_t szw = sz[block * kTileRows + j];
    const float s = bf16_bits_to_f32(szw & 0xFFFFu);
    const float z = -bf16_bits_to_f32(szw >> 16) - 128.0f;
    uint4 *dst = reinterpret_cast<uint4 *>(w_bf16 + n * K + G * kGroup + c * 32);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        uint32_t o[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const float lo = ((float)decode_lane(w, 8 * t + 2 * p) - z) * s;       // exact in fp32
            const float hi = ((float)decode_lane(w, 8 * t + 2 * p + 1) - z) * s;
            o[p] = pack_bf16x2(lo, hi);
        }
        dst[t] = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

// Quantiser: 16 lanes share a group (8 weights each), as in the 4-bit kernel; four lanes together
// own one 96-bit canonical run (24 bits each) and exchange their pieces to form the three words.
__global__ __launch_bounds__(256) void quantize3_kernel(int64_t K, int64_t N, const float *__restrict__ w,
                                                        uint32_t *__restrict__ qweight,
                                                        uint16_t *__restrict__ scales,
                                                        uint16_t *__restrict__ zeros) {
    const int64_t oct = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // index of 8 consecutive weights
    const bool live = oct < N * K / 8;
    float v[8];
    float lo = 0.0f, hi = 0.0f;
    if (live) {
        const float4 a = *reinterpret_cast<const float4 *>(w + oct * 8);
        const float4 b = *reinterpret_cast<const float4 *>(w + oct * 8 + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
        v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            lo = fminf(lo, v[i]);
            hi = fmaxf(hi, v[i]);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = 0.f;
    }
#pragma unroll
    for (int mask = 1; mask < 16; mask <<= 1) {
        lo = fminf(lo, __shfl_xor(lo, mask, 16));
        hi = fmaxf(hi, __shfl_xor(hi, mask, 16));
    }
    const float s32 = (float)(((double)hi - (double)lo) / 7.0);
    uint32_t s_bits = f32_to_bf16(s32);
    double s = (double)bf16_bits_to_f32(s_bits);
    if (s == 0.0) {
        s = 1.0;
        s_bits = 0x3F80u;
    }
    double z = rint(-(double)lo / s);
    z = (z > 0.0) ? fmin(z, 7.0) : 0.0;
    uint32_t piece = 0;   // this lane's 24 bits
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        double c = rint((double)v[i] / s) + z;
        c = fmin(fmax(c, 0.0), 7.0);
        piece |= (uint32_t)(int)c << (3 * i);
    }
    // lanes 4q..4q+3 hold pieces p0..p3 of one run: word0 = p0 | p1 << 24, word1 = p1 >> 8 | p2 << 16,
    // word2 = p2 >> 16 | p3 << 8.  Lane 4q + i (i < 3) writes word i.
    const int lane = threadIdx.x & 63, i4 = lane & 3;
    const uint32_t next = __shfl(piece, (lane & ~3) + ((i4 + 1) & 3), 64);
    uint32_t word = 0;
    if (i4 == 0) word = piece | (next << 24);
    if (i4 == 1) word = (piece >> 8) | (next << 16);
    if (i4 == 2) word = (piece >> 16) | (next << 8);
    if (live && i4 < 3) qweight[(oct >> 2) * 3 + i4] = word;
    if (live && (oct & 15) == 0) {
        const int64_t group = oct >> 4;
        scales[group] = (uint16_t)s_bits;
        zeros[group] = f32_to_bf16((float)z);
    }
}

hipError_t launch_retile3(int64_t K, int64_t N, const uint32_t *qweight, const uint16_t *scales,
                          const uint16_t *zeros, uint32_t *wt, uint32_t *sz, hipStream_t stream) {
    const int64_t slots = N * K / 32;
    hipLaunchKernelGGL(retile3_kernel, dim3((unsigned)((slots + 255) / 256)), dim3(256), 0, stream, K, N, qweight,
                       scales, zeros, wt, sz);
    return hipGetLastError();
}

hipError_t launch_dequantize3(const LayerView3 &L, uint16_t *w_bf16, hipStream_t stream) {
    const int64_t slots = L.N * L.K / 32;
    hipLaunchKernelGGL(dequantize3_kernel, dim3((unsigned)((slots + 255) / 256)), dim3(256), 0, stream, L.K, L.N,
                       L.wt, L.sz, w_bf16);
    return hipGetLastError();
}

hipError_t launch_quantize3(int64_t K, int64_t N, const float *w, uint32_t *qweight, uint16_t *scales,
                            uint16_t *zeros, hipStream_t stream) {
    const int64_t octs = N * K / 8;
    hipLaunchKernelGGL(quantize3_kernel, dim3((unsigned)((octs + 255) / 256)), dim3(256), 0, stream, K, N, w,
                       qweight, scales, zeros);
    return hipGetLastError();
}

}  // namespace dmr

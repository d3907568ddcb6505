// Weight-streaming bf16 kernel for M <= 64: the high-precision twin of the W4A16 decode path.
// Same work split as the INT4 kernel (one workgroup per 16 weight rows, S wavefronts along k,
// deterministic LDS reduction); the B operand of each 16x16x32 MFMA is loaded straight from the
// row-major bf16 weight matrix: lane l = 16 c + j reads W[16 T + j][k0 + 32 t + 8 c .. + 7].
#include "common.hpp"

namespace dmr {

namespace {

template <int MT>
constexpr int bf16_max_waves() { return MT == 1 ? 16 : (MT == 2 ? 8 : 4); }

template <int MT>
struct StepRegs {
    Frag b[4];
    Frag a[MT][4];
};

template <int MT>
__device__ __forceinline__ void load_step(StepRegs<MT> &r, const uint16_t *__restrict__ wrow,
                                          const uint16_t *__restrict__ x, int lane, int64_t M,
                                          int64_t K, int64_t k0) {
    const int c = lane >> 4, j = lane & 15;
#pragma unroll
    for (int t = 0; t < 4; ++t)
        r.b[t].u = *reinterpret_cast<const uint4 *>(wrow + k0 + t * 32 + c * 8);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int64_t m = mt * 16 + j;
        if (m < M) {
#pragma unroll
            for (int t = 0; t < 4; ++t)
                r.a[mt][t].u = *reinterpret_cast<const uint4 *>(x + m * K + k0 + t * 32 + c * 8);
        } else {
#pragma unroll
            for (int t = 0; t < 4; ++t) r.a[mt][t].u = make_uint4(0, 0, 0, 0);
        }
    }
}

template <int MT, bool OUT_F32>
__global__ __launch_bounds__(bf16_max_waves<MT>() * 64) void bf16_skinny_kernel(
    const uint16_t *__restrict__ w, const uint16_t *__restrict__ x, void *__restrict__ y, int64_t M,
    int64_t K, int64_t N) {
    extern __shared__ float red[];   // [S][MT * 4][64]
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int S = blockDim.x >> 6;
    const int64_t T = blockIdx.x;
    const int steps = (int)(K / 128);
    const int s0 = (int)(((int64_t)steps * wave) / S);
    const int s1 = (int)(((int64_t)steps * (wave + 1)) / S);
    const uint16_t *wrow = w + (T * kTileRows + (lane & 15)) * K;

    f32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    constexpr int U = (MT == 1) ? 2 : 1;
    int st = s0;
    for (; st + U <= s1; st += U) {
        StepRegs<MT> regs[U];
#pragma unroll
        for (int u = 0; u < U; ++u) load_step<MT>(regs[u], wrow, x, lane, M, K, (int64_t)(st + u) * 128);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(regs[u].a[mt][t].v, regs[u].b[t].v,
                                                                      acc[mt], 0, 0, 0);
    }
    for (; st < s1; ++st) {
        StepRegs<MT> regs;
        load_step<MT>(regs, wrow, x, lane, M, K, (int64_t)st * 128);
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(regs.a[mt][t].v, regs.b[t].v, acc[mt],
                                                                  0, 0, 0);
    }

#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int q = 0; q < 4; ++q) red[((wave * MT + mt) * 4 + q) * 64 + lane] = acc[mt][q];
    __syncthreads();

    for (int e = threadIdx.x; e < MT * 4 * 64; e += blockDim.x) {
        float sum = 0.f;
        for (int s = 0; s < S; ++s) sum += red[s * (MT * 4 * 64) + e];
        const int l = e & 63, q = (e >> 6) & 3, mt = e >> 8;
        const int64_t m = mt * 16 + (l >> 4) * 4 + q;
        const int64_t n = T * kTileRows + (l & 15);
        if (m < M) {
            if (OUT_F32)
                reinterpret_cast<float *>(y)[m * N + n] = sum;
            else
                reinterpret_cast<uint16_t *>(y)[m * N + n] = f32_to_bf16(sum);
        }
    }
}

int pick_waves(int64_t tiles, int steps, int max_waves) {
    int s = 1;
    while (s < max_waves && (int64_t)tiles * s < 4096 && s * 2 <= steps) s *= 2;
    return s;
}

template <int MT>
hipError_t launch_mt(const uint16_t *w, const uint16_t *x, int64_t M, int64_t K, int64_t N, void *y,
                     bool out_f32, hipStream_t stream) {
    const int64_t tiles = N / kTileRows;
    const int S = pick_waves(tiles, (int)(K / 128), bf16_max_waves<MT>());
    const size_t lds = (size_t)S * MT * 4 * 64 * sizeof(float);
    if (out_f32)
        hipLaunchKernelGGL((bf16_skinny_kernel<MT, true>), dim3((unsigned)tiles), dim3(S * 64), lds,
                           stream, w, x, y, M, K, N);
    else
        hipLaunchKernelGGL((bf16_skinny_kernel<MT, false>), dim3((unsigned)tiles), dim3(S * 64), lds,
                           stream, w, x, y, M, K, N);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_bf16_skinny(const uint16_t *w, const uint16_t *x, int64_t M, int64_t K, int64_t N,
                              void *y, bool out_f32, hipStream_t stream) {
    if (M <= 16) return launch_mt<1>(w, x, M, K, N, y, out_f32, stream);
    if (M <= 32) return launch_mt<2>(w, x, M, K, N, y, out_f32, stream);
    if (M <= 48) return launch_mt<3>(w, x, M, K, N, y, out_f32, stream);
    return launch_mt<4>(w, x, M, K, N, y, out_f32, stream);
}

}  // namespace dmr

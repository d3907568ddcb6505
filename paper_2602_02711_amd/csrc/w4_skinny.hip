// Weight-streaming W4A16 kernel for M <= 64 (one decode token, or a group of parallel rollouts
// each taking one low-precision step): packed nibbles are read once from HBM with 128-bit
// loads, turned into bf16 MFMA operands in registers, and contracted on the matrix cores.
//
// Work split: one workgroup per 16-row tile of W; its S wavefronts split the groups along k
// and meet in LDS, summed in wave order (deterministic, no float atomics).
//
// Per wave and group (128 k): B = the 16 x 128 block of (128 + q) as bf16, A = 16 activation
// rows (zero rows beyond M).  Four 16x16x32 MFMAs give D = sum x (128+q); four more against an
// all-ones B give X = sum x in exactly the accumulator layout of D, so
//     acc += s * (D - (128 + z) * X)
// needs no cross-lane traffic.  Accumulator layout of a 16x16 tile: lane l, register r holds
// (activation row 4 (l / 16) + r, weight row l % 16).
#include "common.hpp"

namespace dmr {

namespace {

constexpr uint32_t kMagic = 0x43004300u;   // bf16 pair (128.0, 128.0); OR-ing a nibble adds q
constexpr uint32_t kOnes = 0x3F803F80u;    // bf16 pair (1.0, 1.0)

template <int MT>
struct GroupRegs {
    uint4 w;
    uint32_t szw;
    Frag a[MT][4];
};

template <int MT>
__device__ __forceinline__ void load_group(GroupRegs<MT> &r, const uint4 *__restrict__ wt,
                                           const uint32_t *__restrict__ sz,
                                           const uint16_t *__restrict__ x, int64_t block, int64_t sz_at, int lane,
                                           int64_t M, int64_t K, int64_t k0) {
    const int c = lane >> 4, j = lane & 15;
    r.w = load_stream(wt + block * 64 + lane);
    r.szw = sz[sz_at + j];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int64_t m = mt * 16 + j;
        if (m < M) {
            const uint4 *src = reinterpret_cast<const uint4 *>(x + m * K + k0 + c * 32);
#pragma unroll
            for (int t = 0; t < 4; ++t) r.a[mt][t].u = src[t];
        } else {
#pragma unroll
            for (int t = 0; t < 4; ++t) r.a[mt][t].u = make_uint4(0, 0, 0, 0);
        }
    }
}

template <int MT>
__device__ __forceinline__ void compute_group(const GroupRegs<MT> &r, f32x4 (&acc)[MT]) {
    const uint32_t words[4] = {r.w.x, r.w.y, r.w.z, r.w.w};
    Frag ones;
    ones.u = make_uint4(kOnes, kOnes, kOnes, kOnes);
    f32x4 d[MT], xs[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        d[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
        xs[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        Frag b;
#pragma unroll
        for (int i = 0; i < 4; ++i) b.w[i] = ((words[t] >> (4 * i)) & 0x000F000Fu) | kMagic;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            d[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(r.a[mt][t].v, b.v, d[mt], 0, 0, 0);
            xs[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(r.a[mt][t].v, ones.v, xs[mt], 0, 0, 0);
        }
    }
    const float s = __uint_as_float(r.szw << 16);
    const float cz = __uint_as_float(r.szw & 0xFFFF0000u);   // -(128 + z)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[mt][q] = fmaf(s, fmaf(cz, xs[mt][q], d[mt][q]), acc[mt][q]);
}

template <int MT>
constexpr int max_waves() { return MT == 1 ? 16 : (MT == 2 ? 8 : 4); }

template <int MT, bool OUT_F32>
__global__ __launch_bounds__(max_waves<MT>() * 64) void w4_skinny_kernel(const uint4 *__restrict__ wt, const uint32_t *__restrict__ sz,
                                 const uint16_t *__restrict__ x, void *__restrict__ y, int64_t M,
                                 int64_t K, int64_t N, int szs) {
    extern __shared__ float red[];   // [S][MT * 4][64]
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int S = blockDim.x >> 6;
    const int64_t T = blockIdx.x;
    const int groups = (int)(K / kGroup);
    const int g0 = (int)(((int64_t)groups * wave) / S);
    const int g1 = (int)(((int64_t)groups * (wave + 1)) / S);

    f32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    constexpr int U = (MT == 1) ? 4 : (MT == 2 ? 2 : 1);   // groups in flight per wave
    int g = g0;
    for (; g + U <= g1; g += U) {
        GroupRegs<MT> regs[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            load_group<MT>(regs[u], wt, sz, x, T * groups + g + u, sz_index(T, g + u, groups, szs, 0), lane, M, K,
                           (int64_t)(g + u) * kGroup);
#pragma unroll
        for (int u = 0; u < U; ++u) compute_group<MT>(regs[u], acc);
    }
    for (; g < g1; ++g) {
        GroupRegs<MT> regs;
        load_group<MT>(regs, wt, sz, x, T * groups + g, sz_index(T, g, groups, szs, 0), lane, M, K, (int64_t)g * kGroup);
        compute_group<MT>(regs, acc);
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

int pick_waves(int64_t tiles, int groups, int max_waves) {
    // aim at ~4096 wavefronts on the chip (16 per CU), never more waves than groups
    int s = 1;
    while (s < max_waves && (int64_t)tiles * s < 4096 && s * 2 <= groups) s *= 2;
    return s;
}

template <int MT>
hipError_t launch_mt(const LayerView &L, const uint16_t *x, int64_t M, void *y, bool out_f32,
                     hipStream_t stream) {
    const int64_t tiles = L.N / kTileRows;
    const int groups = (int)(L.K / kGroup);
    const int S = pick_waves(tiles, groups, max_waves<MT>());
    const size_t lds = (size_t)S * MT * 4 * 64 * sizeof(float);
    if (out_f32)
        hipLaunchKernelGGL((w4_skinny_kernel<MT, true>), dim3((unsigned)tiles), dim3(S * 64), lds, stream,
                           L.wt, L.sz, x, y, M, L.K, L.N, L.szs);
    else
        hipLaunchKernelGGL((w4_skinny_kernel<MT, false>), dim3((unsigned)tiles), dim3(S * 64), lds, stream,
                           L.wt, L.sz, x, y, M, L.K, L.N, L.szs);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_w4_skinny(const LayerView &L, const uint16_t *x, int64_t M, void *y, bool out_f32,
                            hipStream_t stream) {
    if (M <= 16) return launch_mt<1>(L, x, M, y, out_f32, stream);
    if (M <= 32) return launch_mt<2>(L, x, M, y, out_f32, stream);
    if (M <= 48) return launch_mt<3>(L, x, M, y, out_f32, stream);
    return launch_mt<4>(L, x, M, y, out_f32, stream);
}

}  // namespace dmr

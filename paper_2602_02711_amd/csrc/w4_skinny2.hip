// W4A16 streaming kernel for 16 < M <= 64 (a large group of parallel rollouts): still one pass over
// the packed weights, but with MT = ceil(M / 16) activation tiles the matrix cores do real work, so
// operand traffic is what has to be kept down.
//
// Pre-pass (one small kernel, into the caller's workspace): the activations are rewritten in MFMA
// A-operand order, xf[group][mt][t][lane] = the 8 bf16 that lane (c, j) feeds to MFMA t of row tile
// mt (row 16 mt + j, k = 128 g + 32 c + 8 t ..), zero beyond M, so that a wave fetches an operand
// with one coalesced 1 KiB load; and XG[group][row] = sum of the row's 128 activations of the group.
//
// Main kernel: a workgroup owns R consecutive 16-row weight tiles, its S wavefronts split the
// groups along k.  Per group a wave loads R weight blocks and the MT x 4 operand fragments once and
// issues R x MT x 4 MFMAs on them (each fragment is used R times, each unpacked weight register MT
// times), then applies  acc += s (D - (128 + z) XG).  Partial tiles meet in LDS at the end and are
// added in wave order.
#include "common.hpp"

namespace dmr {

namespace {

// ---- pre-pass --------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void xfrag_kernel(const uint16_t *__restrict__ x, uint4 *__restrict__ xf,
                                                    float *__restrict__ xg, int M, int64_t K, int groups,
                                                    int MT) {
    const int64_t slot = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // (g, mt, t, lane)
    const int64_t slots = (int64_t)groups * MT * 256;
    if (slot < slots) {
        const int lane = (int)(slot & 63), t = (int)((slot >> 6) & 3);
        const int64_t gm = slot >> 8;
        const int mt = (int)(gm % MT);
        const int64_t g = gm / MT;
        const int c = lane >> 4, j = lane & 15;
        const int m = mt * 16 + j;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (m < M) v = *reinterpret_cast<const uint4 *>(x + (int64_t)m * K + g * kGroup + c * 32 + t * 8);
        xf[slot] = v;
    }
    // group sums: one thread per (g, row)
    const int64_t rows = (int64_t)groups * MT * 16;
    if (slot < rows) {
        const int m = (int)(slot % (MT * 16));
        const int64_t g = slot / (MT * 16);
        float sum = 0.f;
        if (m < M) {
            const uint4 *src = reinterpret_cast<const uint4 *>(x + (int64_t)m * K + g * kGroup);
            for (int i = 0; i < 16; ++i) {
                const uint4 v = src[i];
                const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int q = 0; q < 4; ++q) sum += __uint_as_float(w[q] << 16) + __uint_as_float(w[q] & 0xFFFF0000u);
            }
        }
        xg[slot] = sum;
    }
}

// ---- main kernel -----------------------------------------------------------------------------
template <int MT, int R>
__global__ __launch_bounds__(256) void w4_skinny2_kernel(const uint4 *__restrict__ wt,
                                                         const uint32_t *__restrict__ sz,
                                                         const uint4 *__restrict__ xf,
                                                         const float *__restrict__ xg,
                                                         void *__restrict__ y, int M, int64_t N, int groups,
                                                         int tiles, int out_f32, int szs) {
    extern __shared__ float red[];   // [S][R][MT][4][64]
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int S = blockDim.x >> 6;
    const int c = lane >> 4, j = lane & 15;
    const int g0 = (groups * wave) / S, g1 = (groups * (wave + 1)) / S;
    const int t0 = (int)blockIdx.x * R;

    f32x4 acc[R][MT];
#pragma unroll
    for (int rt = 0; rt < R; ++rt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[rt][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int g = g0; g < g1; ++g) {
        uint4 w[R];
        uint32_t szw[R];
#pragma unroll
        for (int rt = 0; rt < R; ++rt) {
            int tile = t0 + rt;
            tile = tile < tiles ? tile : tiles - 1;          // ragged last workgroup: re-read, never stored
            const int64_t block = (int64_t)tile * groups + g;
            w[rt] = load_stream(wt + block * 64 + lane);
            szw[rt] = sz[sz_index(tile, g, groups, szs, j)];
        }
        Frag a[MT][4];
        f32x4 xs[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
            for (int t = 0; t < 4; ++t) a[mt][t].u = xf[(((int64_t)g * MT + mt) * 4 + t) * 64 + lane];
            xs[mt] = *reinterpret_cast<const f32x4 *>(xg + ((int64_t)g * MT + mt) * 16 + c * 4);
        }
#pragma unroll
        for (int rt = 0; rt < R; ++rt) {
            const uint32_t words[4] = {w[rt].x, w[rt].y, w[rt].z, w[rt].w};
            f32x4 d[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) d[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                Frag b;
                unpack_word(words[t], b.w);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    d[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[mt][t].v, b.v, d[mt], 0, 0, 0);
            }
            const float sc = __uint_as_float(szw[rt] << 16);
            const float cz = __uint_as_float(szw[rt] & 0xFFFF0000u);   // -(128 + z)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    acc[rt][mt][q] = fmaf(sc, fmaf(cz, xs[mt][q], d[mt][q]), acc[rt][mt][q]);
        }
    }

    // cross-wave sum in wave order
#pragma unroll
    for (int rt = 0; rt < R; ++rt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            reinterpret_cast<f32x4 *>(red)[((wave * R + rt) * MT + mt) * 64 + lane] = acc[rt][mt];
    __syncthreads();
    for (int e = threadIdx.x; e < R * MT * 64; e += blockDim.x) {
        const int l = e & 63, mt = (e >> 6) % MT, rt = (e >> 6) / MT;
        f32x4 v = reinterpret_cast<const f32x4 *>(red)[e];
        for (int q = 1; q < S; ++q) {
            const f32x4 u = reinterpret_cast<const f32x4 *>(red)[q * R * MT * 64 + e];
#pragma unroll
            for (int k = 0; k < 4; ++k) v[k] += u[k];
        }
        const int tile = t0 + rt;
        if (tile < tiles) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int row = mt * 16 + (l >> 4) * 4 + k;
                if (row < M) {
                    const int64_t o = (int64_t)row * N + (int64_t)tile * kTileRows + (l & 15);
                    if (out_f32)
                        reinterpret_cast<float *>(y)[o] = v[k];
                    else
                        reinterpret_cast<uint16_t *>(y)[o] = f32_to_bf16(v[k]);
                }
            }
        }
    }
}

template <int MT, int R>
hipError_t launch_main(const LayerView &L, const uint4 *xf, const float *xg, int M, void *y, bool out_f32,
                       hipStream_t stream) {
    const int groups = (int)(L.K / kGroup), tiles = (int)(L.N / kTileRows);
    int S = 4;
    while (S > groups) S >>= 1;
    const size_t lds = (size_t)S * R * MT * 64 * sizeof(f32x4);
    // once per process and kernel instantiation (thread-safe static initialisation)
    static const hipError_t attr_status = hipFuncSetAttribute(reinterpret_cast<const void *>(&w4_skinny2_kernel<MT, R>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024);
    if (attr_status != hipSuccess) return attr_status;
    const unsigned grid = (unsigned)((tiles + R - 1) / R);
    hipLaunchKernelGGL((w4_skinny2_kernel<MT, R>), dim3(grid), dim3(S * 64), lds, stream, L.wt, L.sz, xf, xg, y,
                       M, L.N, groups, tiles, out_f32 ? 1 : 0, L.szs);
    return hipGetLastError();
}

}  // namespace

size_t w4_skinny2_workspace_bytes(int64_t M, int64_t K) {
    if (M <= 16 || M > 64) return 0;
    const int64_t MT = (M + 15) / 16, groups = K / kGroup;
    return (size_t)(groups * MT * 256 * sizeof(uint4) + groups * MT * 16 * sizeof(float));
}

hipError_t launch_w4_skinny2(const LayerView &L, const uint16_t *x, int64_t M, void *y, bool out_f32,
                             void *ws, hipStream_t stream) {
    const int MT = (int)((M + 15) / 16);
    const int groups = (int)(L.K / kGroup), tiles = (int)(L.N / kTileRows);
    uint4 *xf = reinterpret_cast<uint4 *>(ws);
    float *xg = reinterpret_cast<float *>(xf + (int64_t)groups * MT * 256);
    const int64_t slots = (int64_t)groups * MT * 256;
    hipLaunchKernelGGL(xfrag_kernel, dim3((unsigned)((slots + 255) / 256)), dim3(256), 0, stream, x, xf, xg, (int)M,
                       L.K, groups, MT);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // R = 4 tiles per workgroup once that still leaves more than one workgroup per CU
    const bool wide = tiles >= 4 * 256;
    const int iM = (int)M;
    switch (MT) {
        case 2: return wide ? launch_main<2, 4>(L, xf, xg, iM, y, out_f32, stream)
                            : launch_main<2, 1>(L, xf, xg, iM, y, out_f32, stream);
        case 3: return wide ? launch_main<3, 4>(L, xf, xg, iM, y, out_f32, stream)
                            : launch_main<3, 1>(L, xf, xg, iM, y, out_f32, stream);
        case 4: return wide ? launch_main<4, 4>(L, xf, xg, iM, y, out_f32, stream)
                            : launch_main<4, 1>(L, xf, xg, iM, y, out_f32, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace dmr

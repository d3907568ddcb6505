// W4A16 / W3A16 panel kernel for 2 <= M <= 16 rows of a layer whose activations do not fit LDS as a whole
// (K = 14336 from five rows on).
//
// A workgroup owns TW * R weight tiles (16 rows each) and one slice of gq groups along k.  It stages
// the M x (128 gq) panel of x in LDS once (rows padded by 16 bytes, as in the M <= 16 streaming
// kernel), then its WAVES = S * TW wavefronts stream their weight blocks straight from HBM into
// registers (ring of four outstanding items, an item = the R blocks of one group) with no barrier in
// the loop: wave (s, tw) walks sub-slice s of the k slice for tiles (blockIdx.x * TW + tw) * R + r.
// Differences from the kernels around it:
//   - the group sums of x (the zero-point term needs sum_k x over each group) are formed once per
//     workgroup, by one pass of MFMAs against all-ones right after the staging, and kept in LDS as a
//     table [group][row tile][4 row quads] of fp32x4; the main loop spends its MFMAs on weights only;
//   - an activation fragment read from LDS feeds R weight tiles (half the LDS traffic at R = 2);
//   - K may be split over blockIdx.y, fp32 partials [split][M][N] added by the shared reduction kernel
//     in ascending order; the S sub-slices inside a workgroup are added through LDS (the panel's
//     memory, reused after a barrier) in ascending order as well.  Results do not depend on timing.
#include "panel_plan.hpp"
#include "w3_unpack.hpp"

namespace dmr {

namespace {

constexpr uint32_t kOnes = 0x3F803F80u;    // bf16 pair (1.0, 1.0)

// BITS = 4: one 16-byte word group per lane and block; BITS = 3: three words (the 3-bit streaming layout)
template <int R, int BITS>
struct PanelItem {
    u32x4_t w[R];          // BITS == 3: .x .y .z hold the three words
    uint32_t szw[R];
};

// Copy the M x x16 pieces (16 bytes each) of the k slice starting at column k0 of x[M][K] into LDS,
// piece (row, col) to slot row * (x16 + 1) + col; B loads in flight per thread.
template <int B>
__device__ __forceinline__ void stage_panel(const uint16_t *__restrict__ x, uint4 *smem, int M, int64_t K,
                                            int64_t k0, int x16, uint32_t x16_magic, int first) {
    const int T = (int)blockDim.x;
    const int total = M * x16;
    for (int base = first + (int)threadIdx.x; base < total; base += B * T) {
        u32x4_t v[B];
        int slot[B];
#pragma unroll
        for (int u = 0; u < B; ++u) {
            const int p = min(base + u * T, total - 1);
            const int row = (int)__umulhi((uint32_t)p, x16_magic);
            const int col = p - row * x16;
            slot[u] = p + row;
            v[u] = *reinterpret_cast<const u32x4_t *>(x + (int64_t)row * K + k0 + col * 8);
        }
#pragma unroll
        for (int u = 0; u < B; ++u)
            if (base + u * T < total) reinterpret_cast<u32x4_t *>(smem)[slot[u]] = v[u];
    }
}

// out_mode: 0 = fp32 y, 1 = bf16 y, 2 = fp32 partial [split][M][N]
template <int MT, int R, int WAVES, int BITS>
__global__ __launch_bounds__(64 * WAVES) void w4_panel_kernel(const void *__restrict__ wt,
                                                              const uint32_t *__restrict__ sz,
                                                              const uint16_t *__restrict__ x,
                                                              void *__restrict__ y, int M, int64_t K, int64_t N,
                                                              int groups, int tiles, int gq, int lgS,
                                                              int out_mode, uint32_t x16_magic, int szs) {
    extern __shared__ uint4 smem[];   // panel [M][gq * 16 + 1] uint4, then xs [gq][MT][4] f32x4
    constexpr int P = 4;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int S = 1 << lgS, TW = WAVES >> lgS;
    const int s = wave & (S - 1), tw = wave >> lgS;
    const int c = lane >> 4, j = lane & 15;
    const int ga = (int)blockIdx.y * gq;                           // first group of this k slice
    const int gl0 = (gq * s) >> lgS;                               // this wave's sub-slice, slice-local
    const int GW = ((gq * (s + 1)) >> lgS) - gl0;                  // >= 1 (S <= gq)
    const int tile0 = ((int)blockIdx.x * TW + tw) * R;
    const int x16 = gq * 16, row_stride = x16 + 1;

    // The first pieces of the activation panel are requested before the weight ring: memory operations of a
    // wave return in order, so behind the ring they would arrive only after its HBM latency.
    constexpr int B0 = 8;
    const int total = M * x16, T = (int)blockDim.x;
    u32x4_t x0[B0];
    int slot0[B0];
#pragma unroll
    for (int u = 0; u < B0; ++u) {
        slot0[u] = 0;
        if (u * T < total) {          // uniform
            const int p = min((int)threadIdx.x + u * T, total - 1);
            const int row = (int)__umulhi((uint32_t)p, x16_magic);
            slot0[u] = p + row;
            x0[u] = *reinterpret_cast<const u32x4_t *>(x + (int64_t)row * K + (int64_t)ga * kGroup + (p - row * x16) * 8);
        }
    }

    // weight stream: unconditional, clamped loads (a tile past the end re-reads the last tile, an item
    // past the sub-slice its last group)
    PanelItem<R, BITS> ring[P];
    auto issue = [&](PanelItem<R, BITS> &dst, int i) {
        const int g = ga + gl0 + (i < GW ? i : GW - 1);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int tile = min(tile0 + r, tiles - 1);
            const int64_t block = (int64_t)tile * groups + g;
            if constexpr (BITS == 4) {
                dst.w[r] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(wt) + block * 64 + lane);
            } else {
                const uint32_t *pw = reinterpret_cast<const uint32_t *>(wt) + (block * 64 + lane) * 3;
                dst.w[r].x = load_stream(pw);
                dst.w[r].y = load_stream(pw + 1);
                dst.w[r].z = load_stream(pw + 2);
            }
            dst.szw[r] = load_stream(sz + sz_index(tile, g, groups, szs, j));
        }
    };
#pragma unroll
    for (int p = 0; p < P; ++p) issue(ring[p], p);

#pragma unroll
    for (int u = 0; u < B0; ++u)
        if ((int)threadIdx.x + u * T < total) reinterpret_cast<u32x4_t *>(smem)[slot0[u]] = x0[u];
    if (total > B0 * T) stage_panel<8>(x, smem, M, K, (int64_t)ga * kGroup, x16, x16_magic, B0 * T);
    __syncthreads();

    // group sums of x: unit u = (group, row tile) -> D = A . ones, every column of D the row sums
    f32x4 *xs = reinterpret_cast<f32x4 *>(smem + M * row_stride);
    {
        Frag ones;
        ones.u = make_uint4(kOnes, kOnes, kOnes, kOnes);
        for (int u = wave; u < gq * MT; u += WAVES) {
            const int gl = u / MT, mt = u - gl * MT;
            const int row = min(mt * 16 + j, M - 1);
            const uint4 *xp = smem + row * row_stride + gl * 16 + c * 4;
            f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                Frag a;
                a.u = xp[t];
                d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, ones.v, d, 0, 0, 0);
            }
            if (j == 0) xs[u * 4 + c] = d;
        }
    }
    __syncthreads();

    const uint4 *xrow[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) xrow[mt] = smem + min(mt * 16 + j, M - 1) * row_stride + c * 4;

    f32x4 acc[R][MT];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[r][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto consume = [&](const PanelItem<R, BITS> &cur, int i) {
        const int gl = gl0 + i;
        f32x4 d[R][MT];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) d[r][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
        uint32_t r16[R][16];
        if constexpr (BITS == 3) {
#pragma unroll
            for (int r = 0; r < R; ++r) unpack3(cur.w[r].x, cur.w[r].y, cur.w[r].z, r16[r]);
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            Frag a[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) a[mt].u = xrow[mt][gl * 16 + t];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                Frag b;
                if constexpr (BITS == 4)
                    unpack_word(cur.w[r][t], b.w);
                else
                    b.u = make_uint4(r16[r][4 * t], r16[r][4 * t + 1], r16[r][4 * t + 2], r16[r][4 * t + 3]);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    d[r][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[mt].v, b.v, d[r][mt], 0, 0, 0);
            }
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const f32x4 xsum = xs[(gl * MT + mt) * 4 + c];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const float sc = __uint_as_float(cur.szw[r] << 16);
                const float cz = __uint_as_float(cur.szw[r] & 0xFFFF0000u);   // -(128 + z)
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[r][mt][q] = fmaf(sc, fmaf(cz, xsum[q], d[r][mt][q]), acc[r][mt][q]);
            }
        }
    };

    int base = 0;
    for (; base + P <= GW; base += P) {
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const PanelItem<R, BITS> cur = ring[p];
            issue(ring[p], base + p + P);
            consume(cur, base + p);
        }
    }
#pragma unroll
    for (int p = 0; p < P - 1; ++p)
        if (base + p < GW) consume(ring[p], base + p);

    const int64_t part = out_mode == 2 ? (int64_t)blockIdx.y * M * N : 0;
    auto store_tile = [&](int tile, int mt, const f32x4 &v) {
        if (tile >= tiles) return;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int row = mt * 16 + c * 4 + q;
            if (row < M) {
                const int64_t o = (int64_t)row * N + (int64_t)tile * kTileRows + j;
                if (out_mode == 1)
                    reinterpret_cast<uint16_t *>(y)[o] = f32_to_bf16(v[q]);
                else
                    reinterpret_cast<float *>(y)[part + o] = v[q];
            }
        }
    };

    if (lgS == 0) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) store_tile(tile0 + r, mt, acc[r][mt]);
        return;
    }
    // cross-slice sum: red[tw][r][mt][s][64] f32x4 in the panel's memory
    __syncthreads();   // every wave has finished reading the panel and the sums
    f32x4 *red = reinterpret_cast<f32x4 *>(smem);
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) red[((((tw * R + r) * MT + mt) << lgS) + s) * 64 + lane] = acc[r][mt];
    __syncthreads();
    for (int u = wave; u < TW * R * MT; u += WAVES) {
        const f32x4 *src = red + ((u << lgS) * 64 + lane);
        f32x4 v = src[0];
        for (int q = 1; q < S; ++q) {
            const f32x4 w2 = src[q * 64];
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] += w2[e];
        }
        const int mt = u % MT, tr = u / MT;                 // tr = tw * R + r
        store_tile((int)blockIdx.x * TW * R + tr, mt, v);
    }
}

template <int MT, int R, int WAVES, int BITS>
hipError_t launch_cfg(int64_t K, int64_t N, const void *wt, const uint32_t *sz, int szs, const uint16_t *x, int M, void *dst,
                      int out_mode, const PanelPlan &p, hipStream_t stream) {
    // once per process and kernel instantiation (thread-safe static initialisation)
    static const hipError_t attr_status = hipFuncSetAttribute(reinterpret_cast<const void *>(&w4_panel_kernel<MT, R, WAVES, BITS>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (attr_status != hipSuccess) return attr_status;
    const int groups = (int)(K / kGroup), tiles = (int)(N / kTileRows);
    const int TW = WAVES / p.S;
    int lgS = 0;
    while ((1 << lgS) < p.S) ++lgS;
    const uint32_t x16_magic = (uint32_t)(((uint64_t(1) << 32) + (uint64_t)p.gq * 16 - 1) / ((uint64_t)p.gq * 16));
    const dim3 grid((unsigned)((tiles + TW * R - 1) / (TW * R)), (unsigned)p.SK);
    hipLaunchKernelGGL((w4_panel_kernel<MT, R, WAVES, BITS>), grid, dim3(64 * WAVES), p.lds, stream, wt, sz, x, dst, M,
                       K, N, groups, tiles, p.gq, lgS, out_mode, x16_magic, szs);
    return hipGetLastError();
}

}  // namespace

size_t w4_panel_workspace_bytes(int64_t M, int64_t K, int64_t N) {
    const PanelPlan p = plan_panel(M, K, N);
    return (p.ok && p.SK > 1) ? (size_t)p.SK * (size_t)M * (size_t)N * sizeof(float) : 0;
}

bool w4_panel_applies(int64_t M, int64_t K, int64_t N) { return plan_panel(M, K, N).ok; }

namespace {

hipError_t launch_panel(int bits, int64_t K, int64_t N, const void *wt, const uint32_t *sz, int szs, const uint16_t *x,
                        int64_t M, void *y, bool out_f32, void *ws, hipStream_t stream) {
    const PanelPlan p = plan_panel(M, K, N);
    if (!p.ok) return hipErrorInvalidValue;
    const bool split = p.SK > 1;
    if (split && !ws) return hipErrorInvalidValue;
    void *dst = split ? ws : y;
    const int out_mode = split ? 2 : (out_f32 ? 0 : 1);
    // the planner only produces one tile per wave in 16-wave workgroups; the kernel itself is written
    // for MT row tiles x R weight tiles per wave (MT * R <= 2 fits the 128 registers of 16 waves)
    if (p.MT != 1 || p.R != 1 || p.WAVES != 16) return hipErrorInvalidValue;
    const hipError_t e = bits == 3 ? launch_cfg<1, 1, 16, 3>(K, N, wt, sz, szs, x, (int)M, dst, out_mode, p, stream)
                                   : launch_cfg<1, 1, 16, 4>(K, N, wt, sz, szs, x, (int)M, dst, out_mode, p, stream);
    if (e != hipSuccess || !split) return e;
    return launch_splitk_reduce(static_cast<const float *>(ws), y, M * N, p.SK, out_f32, stream);
}

}  // namespace

hipError_t launch_w4_panel(const LayerView &L, const uint16_t *x, int64_t M, void *y, bool out_f32, void *ws,
                           hipStream_t stream) {
    return launch_panel(4, L.K, L.N, L.wt, L.sz, L.szs, x, M, y, out_f32, ws, stream);
}

hipError_t launch_w3_panel(const LayerView3 &L, const uint16_t *x, int64_t M, void *y, bool out_f32, void *ws,
                           hipStream_t stream) {
    return launch_panel(3, L.K, L.N, L.wt, L.sz, 1, x, M, y, out_f32, ws, stream);
}

}  // namespace dmr

// W4A16 kernel for 17 <= M <= 64 rows on wide layers (enough 16-row weight tiles that every CU gets a
// workgroup without splitting K): one pass over the packed weights with the activations in LDS.
//
// A workgroup of 8 wavefronts owns TW * R weight tiles (TW = 8 / S tile lanes, R tiles per wave) and
// walks k in chunks of CG groups.  The chunk's x panel, MT * 16 rows x 128 CG columns, sits in one of
// two LDS buffers (rows padded by 16 bytes); while the waves work on chunk c the next panel travels
// global memory -> registers -> the other buffer, and one barrier per chunk publishes it.  The group
// sums of x that the zero-point term needs are formed once per workgroup and chunk (MFMAs against
// all-ones, table [group][row tile][row quad] of fp32x4 behind a second barrier), so the main loop
// spends its MFMAs on weights only.  The weights never touch LDS: wave (s, tw) streams the R blocks
// of groups s * CG / S .. of every chunk straight into registers, one chunk ahead (the
// requests cross chunk boundaries freely).  An activation fragment read from LDS feeds R weight
// tiles.  The S partial tiles of a workgroup meet in LDS at the end (the panels' memory) and are added
// in ascending order.  Splitting K over workgroups was measured and never paid on layers this wide
// (the fp32 partials cost as much as the weights).  Rows of the last row tile beyond M are staged as copies of row M - 1 and never stored.
// BITS = 3 runs the same kernel on the 3-bit streaming layout (768-byte blocks, three words per lane).
#include "w3_unpack.hpp"
#include "wide_plan.hpp"

namespace dmr {

namespace {

constexpr uint32_t kOnes = 0x3F803F80u;    // bf16 pair (1.0, 1.0)

template <int R>
struct WideItem {
    u32x4_t w[R];          // 3-bit layout: .x .y .z hold the lane's three words
    uint32_t szw[R];
};

constexpr int ilog2(int v) { return v <= 1 ? 0 : 1 + ilog2(v / 2); }

template <int MT, int R, int S, int CG, int BITS>
__global__ __launch_bounds__(512) void w4_wide_kernel(const void *__restrict__ wt, const uint32_t *__restrict__ sz,
                                                      const uint16_t *__restrict__ x, void *__restrict__ y, int M,
                                                      int64_t K, int64_t N, int groups, int tiles, int out_f32, int szs) {
    constexpr int WAVES = 8, THREADS = 512, TW = WAVES / S, GWc = CG / S, P = GWc;
    constexpr int ROW = CG * 16 + 1;                  // uint4 per panel row
    constexpr int ROWS = MT * 16;
    constexpr int PANEL = ROWS * ROW;                 // uint4 per buffer
    constexpr int LGC = ilog2(CG * 16);
    constexpr int XL = ROWS * CG * 16 / THREADS;      // 16-byte pieces of a panel per thread
    static_assert(CG % S == 0, "a chunk must divide over the sub-slices");
    static_assert((ROWS * CG * 16) % THREADS == 0, "panel pieces must divide over the threads");
    extern __shared__ uint4 smem[];                   // panel[2][PANEL], then xs[2][CG][MT][4] f32x4

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int s = wave % S, tw = wave / S;
    const int c = lane >> 4, j = lane & 15;
    const int nch = groups / CG;                      // chunks (the group count is a multiple of CG)
    const int items = nch * GWc;
    const int tile0 = ((int)blockIdx.x * TW + tw) * R;

    // weight stream: item n = (chunk n / GWc, local n % GWc); unconditional, clamped loads
    WideItem<R> ring[P];
    auto issue = [&](WideItem<R> &dst, int n) {
        n = n < items ? n : items - 1;
        const int g = (n / GWc) * CG + s * GWc + (n % GWc);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int tile = min(tile0 + r, tiles - 1);
            const int64_t block = (int64_t)tile * groups + g;
            if constexpr (BITS == 4) {
                dst.w[r] = __builtin_nontemporal_load(static_cast<const u32x4_t *>(wt) + block * 64 + lane);
            } else {
                const uint32_t *pw = static_cast<const uint32_t *>(wt) + (block * 64 + lane) * 3;
                dst.w[r].x = load_stream(pw);
                dst.w[r].y = load_stream(pw + 1);
                dst.w[r].z = load_stream(pw + 2);
            }
            dst.szw[r] = load_stream(sz + sz_index(tile, g, groups, szs, j));
        }
    };

    // panel staging: piece p = u * THREADS + tid -> (row p >> LGC, column piece p & (16 CG - 1))
    u32x4_t xr[XL];
    int xoff[XL], xslot[XL];
#pragma unroll
    for (int u = 0; u < XL; ++u) {
        const int p = u * THREADS + tid;
        const int row = p >> LGC, col = p & (CG * 16 - 1);
        xoff[u] = min(row, M - 1) * (int)K + col * 8;      // M * K < 2^31 (checked by the launcher)
        xslot[u] = row * ROW + col;
    }
    auto fetch_x = [&](int ch) {
#pragma unroll
        for (int u = 0; u < XL; ++u)
            xr[u] = *reinterpret_cast<const u32x4_t *>(x + xoff[u] + ch * (CG * kGroup));
    };
    auto put_x = [&](int buf) {
#pragma unroll
        for (int u = 0; u < XL; ++u) reinterpret_cast<u32x4_t *>(smem)[buf * PANEL + xslot[u]] = xr[u];
    };
    f32x4 *xs_base = reinterpret_cast<f32x4 *>(smem + 2 * PANEL);
    auto sums = [&](int buf) {
        Frag ones;
        ones.u = make_uint4(kOnes, kOnes, kOnes, kOnes);
        for (int u = wave; u < CG * MT; u += WAVES) {
            const int gl = u / MT, mt = u - gl * MT;
            const uint4 *xp = smem + buf * PANEL + (mt * 16 + j) * ROW + gl * 16 + c * 4;
            f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                Frag a;
                a.u = xp[t];
                d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, ones.v, d, 0, 0, 0);
            }
            if (j == 0) xs_base[(buf * CG * MT + u) * 4 + c] = d;
        }
    };

    f32x4 acc[R][MT];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[r][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto consume = [&](const WideItem<R> &cur, int buf, int gl) {
        const uint4 *xp = smem + buf * PANEL + j * ROW + gl * 16 + c * 4;
        f32x4 d[R][MT];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) d[r][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            Frag a[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) a[mt].u = xp[mt * 16 * ROW + t];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                Frag b;
                if constexpr (BITS == 4) {
                    unpack_word(cur.w[r][t], b.w);
                } else {
                    if (t == 0) unpack3_step<0>(cur.w[r].x, cur.w[r].y, cur.w[r].z, b.w);
                    if (t == 1) unpack3_step<1>(cur.w[r].x, cur.w[r].y, cur.w[r].z, b.w);
                    if (t == 2) unpack3_step<2>(cur.w[r].x, cur.w[r].y, cur.w[r].z, b.w);
                    if (t == 3) unpack3_step<3>(cur.w[r].x, cur.w[r].y, cur.w[r].z, b.w);
                }
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    d[r][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[mt].v, b.v, d[r][mt], 0, 0, 0);
            }
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const f32x4 xsum = xs_base[((buf * CG + gl) * MT + mt) * 4 + c];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const float sc = __uint_as_float(cur.szw[r] << 16);
                const float cz = __uint_as_float(cur.szw[r] & 0xFFFF0000u);   // -(128 + z)
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[r][mt][q] = fmaf(sc, fmaf(cz, xsum[q], d[r][mt][q]), acc[r][mt][q]);
            }
        }
    };

    // One chunk: request the next panel, work through this wave's GWc items (the ring holds exactly one
    // chunk's items, so each slot is refilled with the same item of the next chunk), publish the next
    // panel and its sums.
    auto chunk_step = [&](int ch, bool more) {
        const int buf = ch & 1;
        fetch_x(min(ch + 1, nch - 1));                 // unconditional (the last chunk re-reads itself)
#pragma unroll
        for (int i = 0; i < GWc; ++i) {
            const WideItem<R> cur = ring[i];
            issue(ring[i], (ch + 1) * GWc + i);
            consume(cur, buf, s * GWc + i);
        }
        if (more) {                                    // uniform over the workgroup
            put_x(buf ^ 1);
            __syncthreads();
            sums(buf ^ 1);
            __syncthreads();
        }
    };

    fetch_x(0);              // ahead of the weights: a wave's loads return in order, and the panel is needed first
#pragma unroll
    for (int p = 0; p < P; ++p) issue(ring[p], p);
    put_x(0);
    __syncthreads();
    sums(0);
    __syncthreads();
    for (int ch = 0; ch < nch; ++ch) chunk_step(ch, ch + 1 < nch);

    auto store_tile = [&](int tile, int mt, const f32x4 &v) {
        if (tile >= tiles) return;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int row = mt * 16 + c * 4 + q;
            if (row < M) {
                const int64_t o = (int64_t)row * N + (int64_t)tile * kTileRows + j;
                if (out_f32)
                    reinterpret_cast<float *>(y)[o] = v[q];
                else
                    reinterpret_cast<uint16_t *>(y)[o] = f32_to_bf16(v[q]);
            }
        }
    };

    if constexpr (S == 1) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) store_tile(tile0 + r, mt, acc[r][mt]);
    } else {
        // cross-slice sum: red[tw][r][mt][s][64] f32x4 in the panels' memory
        __syncthreads();   // every wave has finished reading the panels and the sums
        f32x4 *red = reinterpret_cast<f32x4 *>(smem);
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) red[(((tw * R + r) * MT + mt) * S + s) * 64 + lane] = acc[r][mt];
        __syncthreads();
        for (int u = wave; u < TW * R * MT; u += WAVES) {
            const f32x4 *src = red + (u * S * 64 + lane);
            f32x4 v = src[0];
#pragma unroll
            for (int q = 1; q < S; ++q) {
                const f32x4 w2 = src[q * 64];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] += w2[e];
            }
            const int mt = u % MT, tr = u / MT;             // tr = tw * R + r
            store_tile((int)blockIdx.x * TW * R + tr, mt, v);
        }
    }
}

template <int MT, int R, int S, int CG, int BITS>
hipError_t launch_cfg(const void *wt, const uint32_t *sz, int szs, int64_t K, int64_t N, const uint16_t *x, int M, void *y,
                      bool out_f32, hipStream_t stream) {
    // once per process and kernel instantiation (thread-safe static initialisation)
    static const hipError_t attr_status = hipFuncSetAttribute(
        reinterpret_cast<const void *>(&w4_wide_kernel<MT, R, S, CG, BITS>), hipFuncAttributeMaxDynamicSharedMemorySize,
        160 * 1024);
    if (attr_status != hipSuccess) return attr_status;
    const int groups = (int)(K / kGroup), tiles = (int)(N / kTileRows);
    constexpr int TW = 8 / S;
    static_assert(TW * R == kWideTilesPerWg && CG == kWideChunk, "the planner assumes this shape");
    const unsigned grid = (unsigned)((tiles + TW * R - 1) / (TW * R));
    hipLaunchKernelGGL((w4_wide_kernel<MT, R, S, CG, BITS>), dim3(grid), dim3(512), wide_lds_bytes(MT, R, S, CG), stream,
                       wt, sz, x, y, M, K, N, groups, tiles, out_f32 ? 1 : 0, szs);
    return hipGetLastError();
}

template <int BITS>
hipError_t launch_wide(const void *wt, const uint32_t *sz, int szs, int64_t K, int64_t N, const uint16_t *x, int64_t M, void *y,
                       bool out_f32, hipStream_t stream) {
    const WidePlan p = plan_wide(M, K, N);
    if (!p.ok) return hipErrorInvalidValue;
    const int iM = (int)M;
    switch (p.MT) {
        case 2: return launch_cfg<2, 2, 2, 4, BITS>(wt, sz, szs, K, N, x, iM, y, out_f32, stream);
        case 3: return launch_cfg<3, 2, 2, 4, BITS>(wt, sz, szs, K, N, x, iM, y, out_f32, stream);
        case 4: return launch_cfg<4, 2, 2, 4, BITS>(wt, sz, szs, K, N, x, iM, y, out_f32, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool w4_wide_applies(int64_t M, int64_t K, int64_t N) { return plan_wide(M, K, N).ok; }

hipError_t launch_w4_wide(const LayerView &L, const uint16_t *x, int64_t M, void *y, bool out_f32,
                          hipStream_t stream) {
    return launch_wide<4>(L.wt, L.sz, L.szs, L.K, L.N, x, M, y, out_f32, stream);
}

hipError_t launch_w3_wide(const LayerView3 &L, const uint16_t *x, int64_t M, void *y, bool out_f32,
                          hipStream_t stream) {
    return launch_wide<3>(L.wt, L.sz, 1, L.K, L.N, x, M, y, out_f32, stream);
}

}  // namespace dmr

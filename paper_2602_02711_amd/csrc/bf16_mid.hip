// bf16 twin of the rollout-batch kernel: y[M][N] = x[M][K] . W[N][K]^T for 17 rows up to a few hundred
// (and whenever a tiled GEMM would leave most of the 256 CUs idle), fp32 accumulation.
//
// Same skeleton as the INT4 kernel of this size class, so that the two copies of a routed step are
// compared like for like: the workgroup's BM x 128 slice of x goes through double-buffered LDS (rows
// padded to 272 bytes), the weights go from global memory straight into MFMA B-operand registers.
// A lane (c, j) of a wave supplies row 16 T + j of its weight tile and, for MFMA t of a 128-wide k
// step, the 8 values k = 32 t + 8 c .. + 7: one 16-byte load, the four lanes c of a row covering 64
// contiguous bytes per instruction; the A operand is read from LDS with the same k mapping.
// Weight loads run two steps ahead, activation loads three (registers) plus one (LDS).  K may be
// split over blockIdx.z with fp32 partials added by the shared reduction kernel (ascending order).
#include <algorithm>

#include "mid_plan.hpp"

namespace dmr {

namespace {

constexpr int ROW_BYTES = 272;   // one activation row of a k step in LDS: 128 bf16 + 16 bytes of padding

// out_mode: 0 = fp32 y, 1 = bf16 y, 2 = fp32 partial [split][M][N]
template <int MTW, int WM, int NW, int R>
__global__ __launch_bounds__(64 * WM * NW, 2) void bf16_mid_kernel(const uint16_t *__restrict__ w,
                                                                   const uint16_t *__restrict__ x,
                                                                   void *__restrict__ y, int M, int64_t K,
                                                                   int64_t N, int groups, int tiles, int gps,
                                                                   int out_mode) {
    constexpr int THREADS = 64 * WM * NW;
    constexpr int BM = 16 * MTW * WM;
    constexpr int ROWS_PER_PASS = THREADS / 16;
    constexpr int XL = BM / ROWS_PER_PASS;          // 16-byte pieces of x per thread and k step
    static_assert(BM % ROWS_PER_PASS == 0, "activation rows must divide over the threads");
    extern __shared__ __attribute__((aligned(16))) uint8_t xl[];   // [2][BM][ROW_BYTES]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane >> 4, j = lane & 15;
    const int wm = wave % WM, wn = wave / WM;
    const int m0 = (int)blockIdx.y * BM;
    const int gA = (int)blockIdx.z * gps;
    const int gB = min(groups, gA + gps);

    // this lane's weight row per tile (a ragged last column block re-reads the last tile) at k = 8 c
    const int tile0 = ((int)blockIdx.x * NW + wn) * R;
    const uint16_t *wsrc[R];
#pragma unroll
    for (int rt = 0; rt < R; ++rt)
        wsrc[rt] = w + ((int64_t)min(tile0 + rt, tiles - 1) * kTileRows + j) * K + c * 8;

    struct Slot {
        u32x4_t w[R][4];
    };
    Slot ring[2];
    auto fetch_w = [&](Slot &s, int g) {
#pragma unroll
        for (int rt = 0; rt < R; ++rt)
#pragma unroll
            for (int t = 0; t < 4; ++t)
                s.w[rt][t] = *reinterpret_cast<const u32x4_t *>(wsrc[rt] + (int64_t)g * kGroup + t * 32);
    };

    // activations: thread -> (row, 16-byte piece) of the BM x 128 slice; rows beyond M wrap around to
    // rows m mod M (their outputs are never stored)
    u32x4_t xr[2][XL];
    const int xrow = tid >> 4, xpiece = tid & 15;
    const uint16_t *xsrc[XL];
#pragma unroll
    for (int p = 0; p < XL; ++p) {
        const int m = m0 + p * ROWS_PER_PASS + xrow;
        xsrc[p] = x + (int64_t)(m < M ? m : m % M) * K + xpiece * 8;
    }
    auto fetch_x = [&](int set, int g) {
#pragma unroll
        for (int p = 0; p < XL; ++p)
            xr[set][p] = *reinterpret_cast<const u32x4_t *>(xsrc[p] + (int64_t)g * kGroup);
    };
    auto put_x = [&](int set, int buf) {
        uint8_t *dst = xl + buf * (BM * ROW_BYTES);
#pragma unroll
        for (int p = 0; p < XL; ++p)
            *reinterpret_cast<u32x4_t *>(dst + (p * ROWS_PER_PASS + xrow) * ROW_BYTES + xpiece * 16) = xr[set][p];
    };

    f32x4 acc[R][MTW];
#pragma unroll
    for (int rt = 0; rt < R; ++rt)
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt) acc[rt][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto compute = [&](const Slot &s, int buf) {
        const uint8_t *src = xl + buf * (BM * ROW_BYTES) + (wm * MTW * 16 + j) * ROW_BYTES + c * 16;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            Frag a[MTW];
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt)
                a[mt].u = *reinterpret_cast<const uint4 *>(src + mt * 16 * ROW_BYTES + t * 64);
#pragma unroll
            for (int rt = 0; rt < R; ++rt) {
                const bf16x8 b = __builtin_bit_cast(bf16x8, s.w[rt][t]);
#pragma unroll
                for (int mt = 0; mt < MTW; ++mt)
                    acc[rt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[mt].v, b, acc[rt][mt], 0, 0, 0);
            }
        }
    };

    // One 128-wide k step per phase, phases in pairs (static register indices).  A phase past the end
    // of this split's k range re-reads the last step and skips the MFMAs (a uniform branch with no
    // loads and no barrier inside), so every wave passes the same barriers and every load is
    // unconditional.
    const int last = gB - 1;
    fetch_x(0, gA);          // ahead of the weights: a wave's loads return in order, and this one is needed first
    fetch_w(ring[0], gA);
    fetch_w(ring[1], min(gA + 1, last));
    put_x(0, 0);
    fetch_x(1, min(gA + 1, last));
    fetch_x(0, min(gA + 2, last));
    __syncthreads();
    for (int g = gA; g < gB; g += 2) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (g + u < gB) compute(ring[u], u);
            fetch_w(ring[u], min(g + u + 2, last));
            put_x((u + 1) & 1, (u + 1) & 1);                 // step g + u + 1
            fetch_x((u + 1) & 1, min(g + u + 3, last));
            __syncthreads();
        }
    }

    const int64_t part = out_mode == 2 ? (int64_t)blockIdx.z * M * N : 0;
#pragma unroll
    for (int rt = 0; rt < R; ++rt) {
        const int tile = tile0 + rt;
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int m = m0 + (wm * MTW + mt) * 16 + c * 4 + q;
                if (m < M && tile < tiles) {
                    const int64_t o = (int64_t)m * N + (int64_t)tile * kTileRows + j;
                    if (out_mode == 1)
                        reinterpret_cast<uint16_t *>(y)[o] = f32_to_bf16(acc[rt][mt][q]);
                    else
                        reinterpret_cast<float *>(y)[part + o] = acc[rt][mt][q];
                }
            }
    }
}

template <int MTW, int WM, int NW, int R>
hipError_t launch_cfg(const uint16_t *w, const uint16_t *x, int M, int64_t K, int64_t N, void *dst, int out_mode,
                      const MidPlan &p, hipStream_t stream) {
    constexpr int BM = 16 * MTW * WM;
    constexpr size_t lds = 2ull * BM * ROW_BYTES;
    // once per process and kernel instantiation (thread-safe static initialisation)
    static const hipError_t attr_status = hipFuncSetAttribute(reinterpret_cast<const void *>(&bf16_mid_kernel<MTW, WM, NW, R>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (attr_status != hipSuccess) return attr_status;
    const int groups = (int)(K / kGroup), tiles = (int)(N / kTileRows);
    const dim3 grid((unsigned)((tiles + NW * R - 1) / (NW * R)), (unsigned)((M + BM - 1) / BM), (unsigned)p.SK);
    hipLaunchKernelGGL((bf16_mid_kernel<MTW, WM, NW, R>), grid, dim3(64 * WM * NW), lds, stream, w, x, dst, M, K, N,
                       groups, tiles, p.gps, out_mode);
    return hipGetLastError();
}

template <int MTW, int WM, int NW>
hipError_t launch_r(const uint16_t *w, const uint16_t *x, int M, int64_t K, int64_t N, void *dst, int out_mode,
                    const MidPlan &p, hipStream_t stream) {
    return p.R == 2 ? launch_cfg<MTW, WM, NW, 2>(w, x, M, K, N, dst, out_mode, p, stream)
                    : launch_cfg<MTW, WM, NW, 1>(w, x, M, K, N, dst, out_mode, p, stream);
}

}  // namespace

size_t bf16_mid_workspace_bytes(int64_t M, int64_t K, int64_t N) {
    const MidPlan p = plan_mid(M, K, N);
    return p.SK > 1 ? (size_t)p.SK * (size_t)M * (size_t)N * sizeof(float) : 0;
}

hipError_t launch_bf16_mid(const uint16_t *w, const uint16_t *x, int64_t M, int64_t K, int64_t N, void *y,
                           bool out_f32, void *ws, hipStream_t stream) {
    const MidPlan p = plan_mid(M, K, N);
    const bool split = p.SK > 1;
    void *dst = split ? ws : y;
    const int out_mode = split ? 2 : (out_f32 ? 0 : 1);
    const int iM = (int)M;
    hipError_t e;
    if (p.WM == 1) {
        switch (p.MTW) {
            case 1: e = launch_r<1, 1, 4>(w, x, iM, K, N, dst, out_mode, p, stream); break;
            case 2: e = launch_r<2, 1, 4>(w, x, iM, K, N, dst, out_mode, p, stream); break;
            case 3: e = launch_r<3, 1, 4>(w, x, iM, K, N, dst, out_mode, p, stream); break;
            default: e = launch_r<4, 1, 4>(w, x, iM, K, N, dst, out_mode, p, stream); break;
        }
    } else {
        e = p.MTW == 3 ? launch_r<3, 2, 2>(w, x, iM, K, N, dst, out_mode, p, stream)
                       : launch_r<4, 2, 2>(w, x, iM, K, N, dst, out_mode, p, stream);
    }
    if (e != hipSuccess || !split) return e;
    return launch_splitk_reduce(static_cast<const float *>(ws), y, M * N, p.SK, out_f32, stream);
}

}  // namespace dmr

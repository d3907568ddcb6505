// W4A16 for batches of 17 rows up to several hundred (a group of parallel rollouts decoding together,
// or a short prefill): too many rows for the pure streaming kernels, too few for a tiled GEMM to fill
// 256 CUs.  Also serves 2..16 rows when K is so long that the rows do not fit LDS whole.
//
// The streaming layout already is MFMA B-operand order, so the weights never touch LDS: a wave
// loads its 1 KiB blocks straight into registers (nontemporal, requested four groups ahead),
// unpacks them with the bf16 magic number and feeds v_mfma_f32_16x16x32_bf16.  Only the activations
// go through LDS: the workgroup's BM x 128 slice of x for the current group, double buffered (and
// requested three groups ahead into registers), rows padded to 272 bytes so that the 16-byte
// A-operand reads of 8 consecutive lanes fall in distinct banks.  A wave owns MTW row tiles x R weight tiles; every A fragment it reads from LDS feeds R MFMAs
// and every unpacked weight register MTW MFMAs.  The group sums of x come from one more MFMA against
// an all-ones operand, already in accumulator layout, and a group contributes
//     acc += s (D - (128 + z) X)                                  (exact codes, fp32 scale)
// as in the decode kernels, so this path has their accuracy.
//
// Small N x M leaves too few (row block, column block) pairs for the chip; then K is split over
// blockIdx.z, each split writes an fp32 partial tile to the caller's workspace and a second kernel
// adds the partials in ascending split order (deterministic, no atomics).
//
// BITS = 3 runs the same kernel on the 3-bit streaming layout (768-byte blocks, three words per lane).
#include <algorithm>

#include "mid_plan.hpp"
#include "w3_unpack.hpp"

namespace dmr {

namespace {

constexpr int ROW_BYTES = 272;   // one activation row of a group in LDS: 128 bf16 + 16 bytes of padding


// out_mode: 0 = fp32 y, 1 = bf16 y, 2 = fp32 partial [split][M][N]
template <int MTW, int WM, int NW, int R, int BITS>
__global__ __launch_bounds__(64 * WM * NW, (WM * NW == 4) ? 2 : 1) void w4_mid_kernel(
    const void *__restrict__ wt, const uint32_t *__restrict__ sz, const uint16_t *__restrict__ x,
    void *__restrict__ y, int M, int64_t K, int64_t N, int groups, int tiles, int gps, int out_mode, int szs) {
    constexpr int THREADS = 64 * WM * NW;
    constexpr int BM = 16 * MTW * WM;
    constexpr int ROWS_PER_PASS = THREADS / 16;
    constexpr int XL = BM / ROWS_PER_PASS;          // 16-byte pieces of x per thread and group
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

    const int tile0 = ((int)blockIdx.x * NW + wn) * R;
    int64_t wbase[R];          // block index of (tile, group 0); ragged last column block re-reads the last tile
    int64_t sbase[R];          // its first scale / zero word (wave-uniform, like wbase)
#pragma unroll
    for (int rt = 0; rt < R; ++rt) {
        wbase[rt] = (int64_t)min(tile0 + rt, tiles - 1) * groups;
        sbase[rt] = sz_index(min(tile0 + rt, tiles - 1), 0, groups, szs, 0);
    }
    const uint32_t *szj = sz + j;
    const int sstep = szs * kTileRows;

    struct Slot {
        uint4 w[R];            // BITS == 3: .x .y .z hold the lane's three words
        uint32_t s[R];
    };
    Slot ring[4];
    auto fetch_w = [&](Slot &s, int g) {
#pragma unroll
        for (int rt = 0; rt < R; ++rt) {
            const int64_t block = wbase[rt] + g;
            if constexpr (BITS == 4) {
                s.w[rt] = load_stream(static_cast<const uint4 *>(wt) + block * 64 + lane);
            } else {
                const uint32_t *pw = static_cast<const uint32_t *>(wt) + (block * 64 + lane) * 3;
                s.w[rt].x = load_stream(pw);
                s.w[rt].y = load_stream(pw + 1);
                s.w[rt].z = load_stream(pw + 2);
            }
            s.s[rt] = szj[sbase[rt] + (int64_t)g * sstep];
        }
    };

    // activations: thread -> (row, 16-byte piece) of the BM x 128 slice.  Rows beyond M wrap around to
    // rows m mod M: MFMA rows are independent and those outputs are never stored, so no zero fill
    // (whose per-lane select would make the loads conditional) is needed.
    u32x4_t xr[2][XL];     // two groups in flight (a plain vector type: the array has to stay in registers)
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

    Frag ones;
    ones.w[0] = ones.w[1] = ones.w[2] = ones.w[3] = 0x3F803F80u;

    auto compute = [&](const Slot &s, int buf, bool valid) {
        const uint8_t *src = xl + buf * (BM * ROW_BYTES) + (wm * MTW * 16 + j) * ROW_BYTES + c * 64;
        f32x4 d[R][MTW], xs[MTW];
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt) {
            xs[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int rt = 0; rt < R; ++rt) d[rt][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            Frag a[MTW];
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt)
                a[mt].u = *reinterpret_cast<const uint4 *>(src + mt * 16 * ROW_BYTES + t * 16);
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt)
                xs[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[mt].v, ones.v, xs[mt], 0, 0, 0);
#pragma unroll
            for (int rt = 0; rt < R; ++rt) {
                Frag b;
                if constexpr (BITS == 4) {
                    const uint32_t word = t == 0 ? s.w[rt].x : t == 1 ? s.w[rt].y : t == 2 ? s.w[rt].z : s.w[rt].w;
                    unpack_word(word, b.w);
                } else {
                    if (t == 0) unpack3_step<0>(s.w[rt].x, s.w[rt].y, s.w[rt].z, b.w);
                    if (t == 1) unpack3_step<1>(s.w[rt].x, s.w[rt].y, s.w[rt].z, b.w);
                    if (t == 2) unpack3_step<2>(s.w[rt].x, s.w[rt].y, s.w[rt].z, b.w);
                    if (t == 3) unpack3_step<3>(s.w[rt].x, s.w[rt].y, s.w[rt].z, b.w);
                }
#pragma unroll
                for (int mt = 0; mt < MTW; ++mt)
                    d[rt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[mt].v, b.v, d[rt][mt], 0, 0, 0);
            }
        }
#pragma unroll
        for (int rt = 0; rt < R; ++rt) {
            // a slot past the end of this split's k range re-reads its last group with scale 0
            const float sc = valid ? __uint_as_float(s.s[rt] << 16) : 0.f;
            const float cz = __uint_as_float(s.s[rt] & 0xFFFF0000u);   // -(128 + z)
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    acc[rt][mt][q] = fmaf(sc, fmaf(cz, xs[mt][q], d[rt][mt][q]), acc[rt][mt][q]);
        }
    };

    // Software pipeline, one group of 128 k per phase: the weights of a phase were requested four
    // phases earlier, its activations three phases earlier into registers and written to the other
    // LDS buffer one phase earlier.  Phases come in fours (static register indices); a phase past the
    // end of this split's k range re-reads the last group with scale 0, so that every wave passes the
    // same barriers and every load is unconditional.  (Walking the groups in a different order per
    // workgroup was measured and is slower: workgroups in step share the activations in cache.)
    const int last = gB - 1;
    fetch_x(0, gA);          // ahead of the weights: a wave's loads return in order, and this one is needed first
#pragma unroll
    for (int u = 0; u < 4; ++u) fetch_w(ring[u], min(gA + u, last));
    put_x(0, 0);
    fetch_x(1, min(gA + 1, last));
    fetch_x(0, min(gA + 2, last));
    __syncthreads();
    for (int g = gA; g < gB; g += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            compute(ring[u], u & 1, g + u < gB);
            fetch_w(ring[u], min(g + u + 4, last));
            put_x((u + 1) & 1, (u + 1) & 1);                 // group g + u + 1
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

// y = sum over splits of part[split], four outputs per thread, splits in ascending order.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ part, void *__restrict__ y,
                                                            int64_t total, int splits, int out_f32) {
    const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i >= total) return;
    f32x4 v = *reinterpret_cast<const f32x4 *>(part + i);
    for (int s = 1; s < splits; ++s) {
        const f32x4 u = *reinterpret_cast<const f32x4 *>(part + (int64_t)s * total + i);
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] += u[k];
    }
    if (out_f32) {
        *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(y) + i) = v;
    } else {
        uint2 o;
        o.x = pack_bf16x2(v[0], v[1]);
        o.y = pack_bf16x2(v[2], v[3]);
        *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(y) + i) = o;
    }
}

template <int MTW, int WM, int NW, int R, int BITS>
hipError_t launch_cfg(const void *wt, const uint32_t *sz, int szs, int64_t K, int64_t N, const uint16_t *x, int M, void *dst,
                      int out_mode, const MidPlan &p, hipStream_t stream) {
    constexpr int BM = 16 * MTW * WM;
    constexpr size_t lds = 2ull * BM * ROW_BYTES;
    // once per process and kernel instantiation (thread-safe static initialisation)
    static const hipError_t attr_status = hipFuncSetAttribute(
        reinterpret_cast<const void *>(&w4_mid_kernel<MTW, WM, NW, R, BITS>), hipFuncAttributeMaxDynamicSharedMemorySize,
        (int)lds);
    if (attr_status != hipSuccess) return attr_status;
    const int groups = (int)(K / kGroup), tiles = (int)(N / kTileRows);
    const dim3 grid((unsigned)((tiles + NW * R - 1) / (NW * R)), (unsigned)((M + BM - 1) / BM), (unsigned)p.SK);
    hipLaunchKernelGGL((w4_mid_kernel<MTW, WM, NW, R, BITS>), grid, dim3(64 * WM * NW), lds, stream, wt, sz, x, dst, M,
                       K, N, groups, tiles, p.gps, out_mode, szs);
    return hipGetLastError();
}

template <int MTW, int WM, int NW, int BITS>
hipError_t launch_r(const void *wt, const uint32_t *sz, int szs, int64_t K, int64_t N, const uint16_t *x, int M, void *dst,
                    int out_mode, const MidPlan &p, hipStream_t stream) {
    // R = 4 was measured too: never faster, and with 4 row tiles per wave it needs more than the 256
    // registers that two waves per SIMD leave
    return p.R == 2 ? launch_cfg<MTW, WM, NW, 2, BITS>(wt, sz, szs, K, N, x, M, dst, out_mode, p, stream)
                    : launch_cfg<MTW, WM, NW, 1, BITS>(wt, sz, szs, K, N, x, M, dst, out_mode, p, stream);
}

template <int BITS>
hipError_t launch_mid(const void *wt, const uint32_t *sz, int szs, int64_t K, int64_t N, const uint16_t *x, int64_t M, void *y,
                      bool out_f32, void *ws, hipStream_t stream) {
    const MidPlan p = plan_mid(M, K, N);
    const bool split = p.SK > 1;
    if (split && !ws) return hipErrorInvalidValue;
    void *dst = split ? ws : y;
    const int out_mode = split ? 2 : (out_f32 ? 0 : 1);
    const int iM = (int)M;
    hipError_t e;
    if (p.WM == 1) {
        switch (p.MTW) {
            case 1: e = launch_r<1, 1, 4, BITS>(wt, sz, szs, K, N, x, iM, dst, out_mode, p, stream); break;
            case 2: e = launch_r<2, 1, 4, BITS>(wt, sz, szs, K, N, x, iM, dst, out_mode, p, stream); break;
            case 3: e = launch_r<3, 1, 4, BITS>(wt, sz, szs, K, N, x, iM, dst, out_mode, p, stream); break;
            default: e = launch_r<4, 1, 4, BITS>(wt, sz, szs, K, N, x, iM, dst, out_mode, p, stream); break;
        }
    } else {
        e = p.MTW == 3 ? launch_r<3, 2, 2, BITS>(wt, sz, szs, K, N, x, iM, dst, out_mode, p, stream)
                       : launch_r<4, 2, 2, BITS>(wt, sz, szs, K, N, x, iM, dst, out_mode, p, stream);
    }
    if (e != hipSuccess || !split) return e;
    return launch_splitk_reduce(static_cast<const float *>(ws), y, M * N, p.SK, out_f32, stream);
}

}  // namespace

hipError_t launch_splitk_reduce(const float *part, void *y, int64_t total, int splits, bool out_f32,
                                hipStream_t stream) {
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((total / 4 + 255) / 256)), dim3(256), 0, stream, part, y,
                       total, splits, out_f32 ? 1 : 0);
    return hipGetLastError();
}

size_t w4_mid_workspace_bytes(int64_t M, int64_t K, int64_t N) {
    const MidPlan p = plan_mid(M, K, N);
    return p.SK > 1 ? (size_t)p.SK * (size_t)M * (size_t)N * sizeof(float) : 0;
}

hipError_t launch_w4_mid(const LayerView &L, const uint16_t *x, int64_t M, void *y, bool out_f32, void *ws,
                         hipStream_t stream) {
    return launch_mid<4>(L.wt, L.sz, L.szs, L.K, L.N, x, M, y, out_f32, ws, stream);
}

hipError_t launch_w3_mid(const LayerView3 &L, const uint16_t *x, int64_t M, void *y, bool out_f32, void *ws,
                         hipStream_t stream) {
    return launch_mid<3>(L.wt, L.sz, 1, L.K, L.N, x, M, y, out_f32, ws, stream);
}

}  // namespace dmr

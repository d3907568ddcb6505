// Large-tile MFMA GEMM for long prefills: y[M][N] = x[M][K] . W[N][K]^T, fp32 accumulation.
//
// The 128 x 128 kernel is bound by LDS reads (1 KiB of operand fragments per 32x32x16 MFMA).  Here
// a workgroup of 4 wavefronts owns a 256 x 256 tile and every wave a 128 x 128 patch (4 x 4 MFMA
// tiles, 256 accumulator registers): 8 fragments feed 16 MFMAs, half the LDS bytes per MFMA.  LDS is
// double buffered (2 x 72 KiB of 160), one barrier per 64-wide k step; the global loads of step
// i + 1 are issued before the MFMAs of step i and written to the other buffer after them.
// INT4 tiles are dequantised to RNE_bf16((q - z) s) on the way into LDS.
#include "common.hpp"

namespace dmr {

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int LDS_STRIDE = BK + 8;                       // bf16 elements per padded row (144 bytes)
constexpr int TILE_ELEMS = BM * LDS_STRIDE;              // one operand, one buffer
constexpr size_t LDS_BYTES = 4ull * TILE_ELEMS * sizeof(uint16_t);   // A and B, two buffers each

template <bool W4>
struct Prefetch {
    uint4 xa[8];
    uint4 wb[W4 ? 2 : 8];
    uint32_t szw[2];
};

template <bool W4>
__device__ __forceinline__ void load_global(Prefetch<W4> &p, const void *__restrict__ wsrc,
                                            const uint32_t *__restrict__ sz,
                                            const uint16_t *__restrict__ x, int64_t M, int64_t K,
                                            int64_t N, int64_t m0, int64_t n0, int64_t k0, int tid) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int idx = tid + 256 * i;
        const int row = idx >> 3, chunk = idx & 7;
        const int64_t m = m0 + row;
        p.xa[i] = (m < M) ? *reinterpret_cast<const uint4 *>(x + m * K + k0 + chunk * 8)
                          : make_uint4(0, 0, 0, 0);
    }
    if (W4) {
        const int64_t groups = K / kGroup;
        const int64_t G = k0 / kGroup;
        const int half = (int)((k0 % kGroup) / 64);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int slot = tid + 256 * i;
            const int64_t T = n0 / kTileRows + (slot >> 5);
            const int l = half * 32 + (slot & 31);
            if (T * kTileRows < N) {
                p.wb[i] = reinterpret_cast<const uint4 *>(wsrc)[(T * groups + G) * 64 + l];
                p.szw[i] = sz[(T * groups + G) * kTileRows + (l & 15)];
            } else {
                p.wb[i] = make_uint4(0, 0, 0, 0);
                p.szw[i] = 0xC3000000u;   // s = 0, -(128 + z) = -128: contributes zeros
            }
        }
    } else {
        const uint16_t *w = reinterpret_cast<const uint16_t *>(wsrc);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int idx = tid + 256 * i;
            const int row = idx >> 3, chunk = idx & 7;
            const int64_t n = n0 + row;
            p.wb[i] = (n < N) ? *reinterpret_cast<const uint4 *>(w + n * K + k0 + chunk * 8)
                              : make_uint4(0, 0, 0, 0);
        }
    }
}

template <bool W4>
__device__ __forceinline__ void store_lds(const Prefetch<W4> &p, uint16_t *As, uint16_t *Bs, int tid) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int idx = tid + 256 * i;
        const int row = idx >> 3, chunk = idx & 7;
        *reinterpret_cast<uint4 *>(As + row * LDS_STRIDE + chunk * 8) = p.xa[i];
    }
    if (W4) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int slot = tid + 256 * i;
            const int l = slot & 31;
            const int row = (slot >> 5) * kTileRows + (l & 15);
            const int kofs = (l >> 4) * 32;
            const float s = __uint_as_float(p.szw[i] << 16);
            const float czs = __uint_as_float(p.szw[i] & 0xFFFF0000u) * s;   // -(128 + z) s, exact
            const uint32_t words[4] = {p.wb[i].x, p.wb[i].y, p.wb[i].z, p.wb[i].w};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                uint32_t o[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t pair = ((words[t] >> (4 * q)) & 0x000F000Fu) | 0x43004300u;
                    const float lo = fmaf(__uint_as_float(pair << 16), s, czs);
                    const float hi = fmaf(__uint_as_float(pair & 0xFFFF0000u), s, czs);
                    o[q] = pack_bf16x2(lo, hi);
                }
                *reinterpret_cast<uint4 *>(Bs + row * LDS_STRIDE + kofs + t * 8) =
                    make_uint4(o[0], o[1], o[2], o[3]);
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int idx = tid + 256 * i;
            const int row = idx >> 3, chunk = idx & 7;
            *reinterpret_cast<uint4 *>(Bs + row * LDS_STRIDE + chunk * 8) = p.wb[i];
        }
    }
}

template <bool W4, bool OUT_F32>
__global__ __launch_bounds__(256) void gemm_big_kernel(const void *__restrict__ wsrc,
                                                       const uint32_t *__restrict__ sz,
                                                       const uint16_t *__restrict__ x,
                                                       void *__restrict__ y, int64_t M, int64_t K,
                                                       int64_t N, int nbn, int lg_xm) {
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];   // As[2], Bs[2]
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    int tm, tn;
    if (lg_xm < 0) {            // plain order: column blocks fastest
        tm = (int)blockIdx.x / nbn;
        tn = (int)blockIdx.x % nbn;
    } else {
        // XCD-aware order (see the launcher): linear index -> (region, XCD, slot in the XCD's 4 x 8 patch)
        const int region = (int)blockIdx.x >> 8, r = (int)blockIdx.x & 255;
        const int xcd = r & 7, q = r >> 3;
        const int xn = 8 >> lg_xm;
        const int regions_n = nbn / (8 * xn);
        tm = (region / regions_n) * (4 << lg_xm) + (xcd / xn) * 4 + (q >> 3);
        tn = (region % regions_n) * 8 * xn + (xcd % xn) * 8 + (q & 7);
    }
    const int64_t n0 = (int64_t)tn * BN;
    const int64_t m0 = (int64_t)tm * BM;

    f32x16 acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    Prefetch<W4> pre;
    load_global<W4>(pre, wsrc, sz, x, M, K, N, m0, n0, 0, tid);
    store_lds<W4>(pre, lds, lds + 2 * TILE_ELEMS, tid);
    __syncthreads();
    const int steps = (int)(K / BK);
    for (int kt = 0; kt < steps; ++kt) {
        const int cur = kt & 1;
        const uint16_t *As = lds + cur * TILE_ELEMS;
        const uint16_t *Bs = lds + (2 + cur) * TILE_ELEMS;
        if (kt + 1 < steps) load_global<W4>(pre, wsrc, sz, x, M, K, N, m0, n0, (int64_t)(kt + 1) * BK, tid);
        // fragments of k sub-step ks + 1 are requested before the MFMAs of sub-step ks
        Frag a[2][4], b[2][4];
        auto load_frags = [&](int set, int ks) {
            const int kk = ks * 16 + (lane >> 5) * 8;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[set][i].u = *reinterpret_cast<const uint4 *>(As + (wm * 128 + i * 32 + (lane & 31)) * LDS_STRIDE + kk);
                b[set][i].u = *reinterpret_cast<const uint4 *>(Bs + (wn * 128 + i * 32 + (lane & 31)) * LDS_STRIDE + kk);
            }
        };
        load_frags(0, 0);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            if (ks + 1 < BK / 16) load_frags((ks + 1) & 1, ks + 1);
            __builtin_amdgcn_sched_barrier(0);   // keep the next fragments' reads ahead of these MFMAs
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks & 1][i].v, b[ks & 1][j].v, acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (kt + 1 < steps)
            store_lds<W4>(pre, lds + (cur ^ 1) * TILE_ELEMS, lds + (2 + (cur ^ 1)) * TILE_ELEMS, tid);
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t n = n0 + wn * 128 + j * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t m = m0 + wm * 128 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (m < M && n < N) {
                    if (OUT_F32)
                        reinterpret_cast<float *>(y)[m * N + n] = acc[i][j][r];
                    else
                        reinterpret_cast<uint16_t *>(y)[m * N + n] = f32_to_bf16(acc[i][j][r]);
                }
            }
        }
}

template <bool W4, bool OUT_F32>
hipError_t launch_one(const void *wsrc, const uint32_t *sz, const uint16_t *x, int64_t M, int64_t K,
                      int64_t N, void *y, hipStream_t stream) {
    // once per process and kernel instantiation (thread-safe static initialisation)
    static const hipError_t attr_status = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_big_kernel<W4, OUT_F32>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_BYTES);
    if (attr_status != hipSuccess) return attr_status;
    // Workgroups go to the 8 XCDs round-robin by linear index and each XCD has its own L2.  When the
    // tile grid divides evenly, the index is decoded so that the 32 workgroups an XCD runs at a time
    // form a compact 4 x 8 patch of tiles (12 operand panels instead of ~17) and the 8 patches of a
    // round tile a compact region; otherwise plain order (a padded region would leave XCDs idle).
    // Measured at (4096, 28672), M = 8192, bf16: L2 hit rate 53 % -> 79 %, time -7 %.  (Walking k in
    // a different order per tile was measured too and is slower: tiles in step share operand panels.)
    const int nbm = (int)((M + BM - 1) / BM), nbn = (int)((N + BN - 1) / BN);
    int lg_xm = 2;
    while (lg_xm >= 0 && (nbm % (4 << lg_xm) != 0 || nbn % (8 * (8 >> lg_xm)) != 0)) --lg_xm;
    hipLaunchKernelGGL((gemm_big_kernel<W4, OUT_F32>), dim3((unsigned)(nbm * nbn)), dim3(256), LDS_BYTES, stream,
                       wsrc, sz, x, y, M, K, N, nbn, lg_xm);
    return hipGetLastError();
}

}  // namespace

// True when the 256 x 256 tiling gives every CU at least ~1.5 workgroups.
bool gemm_big_applies(int64_t M, int64_t N) {
    const int64_t wgs = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
    return wgs >= 384;
}

hipError_t launch_w4_gemm_big(const LayerView &L, const uint16_t *x, int64_t M, void *y, bool out_f32,
                              hipStream_t stream) {
    return out_f32 ? launch_one<true, true>(L.wt, L.sz, x, M, L.K, L.N, y, stream)
                   : launch_one<true, false>(L.wt, L.sz, x, M, L.K, L.N, y, stream);
}

hipError_t launch_bf16_gemm_big(const uint16_t *w, const uint16_t *x, int64_t M, int64_t K, int64_t N,
                                void *y, bool out_f32, hipStream_t stream) {
    return out_f32 ? launch_one<false, true>(w, nullptr, x, M, K, N, y, stream)
                   : launch_one<false, false>(w, nullptr, x, M, K, N, y, stream);
}

}  // namespace dmr

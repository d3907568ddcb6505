// Tiled MFMA GEMM for prefill-sized M (a long prompt: few-shot prefix plus the whole history),
// y[M][N] = x[M][K] . W[N][K]^T with fp32 accumulation.  Three weight sources share the kernel:
//   kSrcBf16    bf16 weights read as they are;
//   kSrcW4Exact INT4 codes enter LDS as the exact small integers (q - z); the MFMAs of one group of
//               128 k accumulate into a per-group tile that is folded into the result with the
//               group's scale in fp32, acc += s[n][G] * D_G, so no weight is ever rounded.  (Feeding the
//               matrix cores RNE_bf16((q - z) s) instead, what dmr_qlinear_dequantize returns, saves the
//               fold but leaves the largest of 10^7 outputs at 0.8 .. 1.1 of the 1e-2 rms bound.)  Serves
//               the tiled INT4 shapes with fewer than 256 rows, and the column blocks that the faster
//               256-row kernel declines (scales it cannot rescale by).
//   kSrcW3Exact the same on the 3-bit streaming layout (768-byte blocks, unpacked with the byte masks of
//               w3_unpack.hpp), so that a 3-bit layer needs no dequantised copy at prefill sizes.
//
// Workgroup tile 128 (m) x 128 (n) x 64 (k), 4 wavefronts in a 2 x 2 grid, each owning a 64 x 64
// patch as 2 x 2 tiles of v_mfma_f32_32x32x16_bf16.  Global loads for step i+1 are issued into
// registers before the MFMAs of step i.  LDS rows are padded by 16 bytes so that the 16-byte
// operand reads of 32 consecutive rows fall in distinct banks.
//
// Operand layout of a 32x32x16 MFMA: lane l supplies row (l % 32), k = 8 (l / 32) .. + 7 of A and
// of B; accumulator register r of lane l is (A row 8 (r / 4) + 4 (l / 32) + r % 4, B row l % 32).
#include "w3_unpack.hpp"

namespace dmr {

namespace {

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int kSrcBf16 = 0, kSrcW4Exact = 2, kSrcW3Exact = 3;
constexpr int LDS_STRIDE = BK + 8;   // bf16 elements per padded LDS row (144 bytes)

template <int SRC>
struct Prefetch {
    uint4 xa[4];
    uint4 wb[4];       // bf16 source: 4 x 16 bytes; INT4 source: wb[0] = 32 packed weights (3-bit: three words)
    uint32_t szw;
};

template <int SRC>
__device__ __forceinline__ void load_global(Prefetch<SRC> &p, const void *__restrict__ wsrc,
                                            const uint32_t *__restrict__ sz,
                                            const uint16_t *__restrict__ x, int64_t M, int64_t K,
                                            int64_t N, int64_t m0, int64_t n0, int64_t k0, int tid, int szs) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int idx = tid + 256 * i;
        const int row = idx >> 3, chunk = idx & 7;
        const int64_t m = m0 + row;
        p.xa[i] = (m < M) ? *reinterpret_cast<const uint4 *>(x + m * K + k0 + chunk * 8)
                          : make_uint4(0, 0, 0, 0);
    }
    if (SRC != kSrcBf16) {
        // 8 row tiles x 32 lanes: the half of each 1 KiB block that covers this 64-wide k step
        const int64_t groups = K / kGroup;
        const int64_t G = k0 / kGroup;
        const int half = (int)((k0 % kGroup) / 64);
        const int64_t T = n0 / kTileRows + (tid >> 5);
        const int l = half * 32 + (tid & 31);
        if (T * kTileRows < N) {
            if (SRC == kSrcW3Exact) {
                const uint32_t *w3 = reinterpret_cast<const uint32_t *>(wsrc) + ((T * groups + G) * 64 + l) * 3;
                p.wb[0] = make_uint4(w3[0], w3[1], w3[2], 0);
            } else {
                p.wb[0] = reinterpret_cast<const uint4 *>(wsrc)[(T * groups + G) * 64 + l];
            }
            p.szw = sz[sz_index(T, G, groups, szs, l & 15)];
        } else {
            p.wb[0] = make_uint4(0, 0, 0, 0);
            p.szw = 0xC3000000u;   // s = 0, -(128 + z) = -128: contributes zeros
        }
    } else {
        const uint16_t *w = reinterpret_cast<const uint16_t *>(wsrc);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = tid + 256 * i;
            const int row = idx >> 3, chunk = idx & 7;
            const int64_t n = n0 + row;
            p.wb[i] = (n < N) ? *reinterpret_cast<const uint4 *>(w + n * K + k0 + chunk * 8)
                              : make_uint4(0, 0, 0, 0);
        }
    }
}

template <int SRC>
__device__ __forceinline__ void store_lds(const Prefetch<SRC> &p, uint16_t *As, uint16_t *Bs, int tid) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int idx = tid + 256 * i;
        const int row = idx >> 3, chunk = idx & 7;
        *reinterpret_cast<uint4 *>(As + row * LDS_STRIDE + chunk * 8) = p.xa[i];
    }
    if (SRC != kSrcBf16) {
        const int l = tid & 31;                       // lane within the half block
        const int row = (tid >> 5) * kTileRows + (l & 15);
        const int kofs = (l >> 4) * 32;               // 0 or 32 inside the 64-wide step
        const float cz = __uint_as_float(p.szw & 0xFFFF0000u);   // -(128 + z)
        const uint32_t words[4] = {p.wb[0].x, p.wb[0].y, p.wb[0].z, p.wb[0].w};
        uint32_t r3[16];                                         // 3-bit: the lane's 16 (128 + q) pairs, k ascending
        if (SRC == kSrcW3Exact) unpack3(words[0], words[1], words[2], r3);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            uint32_t o[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                // (128 + q) as fp32 straight from the bf16 magic pair; adding -(128 + z) leaves the integer
                // q - z in [-15, 15], which bf16 holds exactly
                const uint32_t pair = SRC == kSrcW3Exact ? r3[4 * t + i]
                                                         : (((words[t] >> (4 * i)) & 0x000F000Fu) | 0x43004300u);
                const float plo = __uint_as_float(pair << 16), phi = __uint_as_float(pair & 0xFFFF0000u);
                o[i] = pack_bf16x2(plo + cz, phi + cz);
            }
            *reinterpret_cast<uint4 *>(Bs + row * LDS_STRIDE + kofs + t * 8) =
                make_uint4(o[0], o[1], o[2], o[3]);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = tid + 256 * i;
            const int row = idx >> 3, chunk = idx & 7;
            *reinterpret_cast<uint4 *>(Bs + row * LDS_STRIDE + chunk * 8) = p.wb[i];
        }
    }
}

template <int SRC, bool OUT_F32>
__global__ __launch_bounds__(256, 2) void gemm_kernel(const void *__restrict__ wsrc,
                                                   const uint32_t *__restrict__ sz,
                                                   const uint16_t *__restrict__ x,
                                                   void *__restrict__ y, int64_t M, int64_t K,
                                                   int64_t N, int szs, const uint32_t *__restrict__ only,
                                                   int only_pairs) {
    // `only` (optional): one word per 32 columns; the block is computed here only when one of the words of its 128
    // columns is nonzero (with only_pairs: of the 256 columns of its aligned pair of blocks)
    if (only) {
        const int span = only_pairs ? 8 : 4;
        const int f0 = (int)(blockIdx.x & (only_pairs ? ~1u : ~0u)) * 4, nf = (int)((N + 31) / 32);
        uint32_t f = 0;
        for (int i = 0; i < span; ++i) f |= f0 + i < nf ? only[f0 + i] : 0u;
        if (f == 0) return;
    }
    __shared__ __attribute__((aligned(16))) uint16_t As[BM * LDS_STRIDE];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[BN * LDS_STRIDE];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t n0 = (int64_t)blockIdx.x * BN;
    // row blocks blockIdx.y, blockIdx.y + gridDim.y, ...: one per workgroup in a full launch; the launch that only serves
    // flagged column blocks uses a few workgroups per column block, so that the unflagged ones cost next to nothing
    for (int64_t m0 = (int64_t)blockIdx.y * BM; m0 < M; m0 += (int64_t)gridDim.y * BM) {
        f32x16 acc[2][2];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

        // exact INT4: per-group accumulators and this lane's two weight rows (one per n tile)
        constexpr bool EXACT = SRC == kSrcW4Exact || SRC == kSrcW3Exact;
        f32x16 grp[2][2];
        if (EXACT) {
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int r = 0; r < 16; ++r) grp[a][b][r] = 0.f;
        }
        const int64_t groups = K / kGroup;
        int64_t srow[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int64_t n = n0 + wn * 64 + j * 32 + (lane & 31);
            const int64_t nc = n < N ? n : N - 1;                         // clamped: never stored
            srow[j] = sz_index(nc / kTileRows, 0, groups, szs, (int)(nc % kTileRows));   // sz index of (row, G = 0)
        }

        Prefetch<SRC> pre;
        load_global<SRC>(pre, wsrc, sz, x, M, K, N, m0, n0, 0, tid, szs);
        for (int64_t k0 = 0; k0 < K; k0 += BK) {
            store_lds<SRC>(pre, As, Bs, tid);
            __syncthreads();
            if (k0 + BK < K) load_global<SRC>(pre, wsrc, sz, x, M, K, N, m0, n0, k0 + BK, tid, szs);
            float gscale[2] = {0.f, 0.f};
            const bool group_end = EXACT && ((k0 + BK) % kGroup == 0);
            if (group_end) {
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    gscale[j] = __uint_as_float(sz[srow[j] + (k0 / kGroup) * kTileRows * szs] << 16);
            }
#pragma unroll
            for (int ks = 0; ks < BK / 16; ++ks) {
                Frag a[2], b[2];
                const int kk = ks * 16 + (lane >> 5) * 8;
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    a[i].u = *reinterpret_cast<const uint4 *>(As + (wm * 64 + i * 32 + (lane & 31)) * LDS_STRIDE + kk);
                    b[i].u = *reinterpret_cast<const uint4 *>(Bs + (wn * 64 + i * 32 + (lane & 31)) * LDS_STRIDE + kk);
                }
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        if (EXACT)
                            grp[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i].v, b[j].v, grp[i][j], 0, 0, 0);
                        else
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i].v, b[j].v, acc[i][j], 0, 0, 0);
                    }
            }
            if (group_end) {
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            acc[i][j][r] = fmaf(gscale[j], grp[i][j][r], acc[i][j][r]);
                            grp[i][j][r] = 0.f;
                        }
            }
            __syncthreads();
        }

#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int64_t n = n0 + wn * 64 + j * 32 + (lane & 31);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t m = m0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    if (m < M && n < N) {
                        if (OUT_F32)
                            reinterpret_cast<float *>(y)[m * N + n] = acc[i][j][r];
                        else
                            reinterpret_cast<uint16_t *>(y)[m * N + n] = f32_to_bf16(acc[i][j][r]);
                    }
                }
            }
    }   // row blocks
}

template <int SRC>
hipError_t launch(const void *wsrc, const uint32_t *sz, int szs, const uint16_t *x, int64_t M, int64_t K,
                  int64_t N, void *y, bool out_f32, hipStream_t stream, const uint32_t *only = nullptr,
                  bool only_pairs = false) {
    const unsigned row_blocks = (unsigned)((M + BM - 1) / BM);
    const dim3 grid((unsigned)((N + BN - 1) / BN), only ? (row_blocks < 4 ? row_blocks : 4) : row_blocks);
    if (out_f32)
        hipLaunchKernelGGL((gemm_kernel<SRC, true>), grid, dim3(256), 0, stream, wsrc, sz, x, y, M, K, N, szs, only,
                           (int)only_pairs);
    else
        hipLaunchKernelGGL((gemm_kernel<SRC, false>), grid, dim3(256), 0, stream, wsrc, sz, x, y, M, K, N, szs, only,
                           (int)only_pairs);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_w4_gemm(const LayerView &L, const uint16_t *x, int64_t M, void *y, bool out_f32, hipStream_t stream) {
    return launch<kSrcW4Exact>(L.wt, L.sz, L.szs, x, M, L.K, L.N, y, out_f32, stream);
}

// The exact kernel on the column blocks of 128 rows that have a nonzero word in `only` (device memory, one word per
// 32 rows); with `pairs`, on both blocks of an aligned pair (256 columns) when either has one.
hipError_t launch_w4_gemm_flagged(const LayerView &L, const uint16_t *x, int64_t M, void *y, bool out_f32,
                                  const uint32_t *only, bool pairs, hipStream_t stream) {
    return launch<kSrcW4Exact>(L.wt, L.sz, L.szs, x, M, L.K, L.N, y, out_f32, stream, only, pairs);
}

hipError_t launch_w3_gemm(const LayerView3 &L, const uint16_t *x, int64_t M, void *y, bool out_f32,
                          hipStream_t stream) {
    return launch<kSrcW3Exact>(L.wt, L.sz, 1, x, M, L.K, L.N, y, out_f32, stream);
}

hipError_t launch_w3_gemm_flagged(const LayerView3 &L, const uint16_t *x, int64_t M, void *y, bool out_f32,
                                  const uint32_t *only, bool pairs, hipStream_t stream) {
    return launch<kSrcW3Exact>(L.wt, L.sz, 1, x, M, L.K, L.N, y, out_f32, stream, only, pairs);
}

hipError_t launch_bf16_gemm(const uint16_t *w, const uint16_t *x, int64_t M, int64_t K, int64_t N,
                            void *y, bool out_f32, hipStream_t stream) {
    return launch<kSrcBf16>(w, nullptr, 1, x, M, K, N, y, out_f32, stream);
}

}  // namespace dmr

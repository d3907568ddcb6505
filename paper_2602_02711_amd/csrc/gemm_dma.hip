// Large-tile MFMA GEMM with direct-to-LDS operand loads: y[M][N] = x[M][K] . W[N][K]^T, fp32 accumulation.
//
// Same tile as the 256 x 256 kernel next to it (4 wavefronts, each a 128 x 128 patch of 4 x 4 MFMA
// 32x32x16 tiles, 256 accumulator registers), but the bf16 operands travel global memory -> LDS without
// passing through registers (`global_load_lds_dwordx4`: every lane names its own 16 global bytes, the
// wave's 64 x 16 bytes land contiguously at a wave-uniform LDS address).  With no staging registers the
// loads can run three k steps ahead: four LDS stages of 32 k (4 x 32 KiB), one barrier per step, and
// the wait before a step only covers the loads issued three steps earlier.  The register-staged
// kernel can afford one step of prefetch and spends ~40 % of its time waiting for it.
//
// LDS layout of a stage: operand rows of 32 bf16 = 64 bytes = four 16-byte chunks, unpadded (a load
// instruction fills 16 consecutive rows), chunk c of row r stored at position c ^ ((r >> 2) & 3): the
// 16 lanes of a quarter wave that read the same chunk of 16 consecutive rows then touch 16 different
// 16-byte bank groups.  The swizzle is applied on the global side (lane l of a load instruction owns
// LDS slot l, i.e. row l / 4, position l % 4, and fetches chunk (l % 4) ^ ((row >> 2) & 3) of that row).
// Rows beyond M or N are clamped to the last row (their products are never stored).
//
// INT4 layers: the packed codes and scale / zero words of a k step (16 + 4 bytes per thread) are fetched
// direct-to-LDS as well, into a small ring, one step further ahead; the lane that fetched them reads them
// back a step before they are needed, dequantises to RNE_bf16((q - z) s) and writes its 64-byte row slice of
// the weight tile.  No load in the loop targets a register, so no register wait ever drains the pipeline.
#include "common.hpp"

namespace dmr {

namespace {

constexpr int BM = 256, BN = 256, BK = 32, NS = 4;
constexpr int ROW_BYTES = BK * 2;                         // 64
constexpr int OPERAND_BYTES = BM * ROW_BYTES;             // 16 KiB per operand and stage
constexpr int STAGE_BYTES = 2 * OPERAND_BYTES;            // A then B
constexpr int NR = NS + 1;                                // ring of packed INT4 slices (requested one step further ahead)
constexpr int RAW_W_BYTES = 4096, RAW_SZ_BYTES = 1024;    // per slot: 256 lanes x 16 bytes of codes, x 4 bytes of scale / zero
constexpr int RAW_BYTES = RAW_W_BYTES + RAW_SZ_BYTES;
constexpr size_t LDS_BYTES_BF16 = (size_t)NS * STAGE_BYTES;                      // 128 KiB
constexpr size_t LDS_BYTES_W4 = LDS_BYTES_BF16 + (size_t)NR * RAW_BYTES + 1024;  // + 25 KiB of ring + 1 KiB of slack

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void global_void;

// s_waitcnt vmcnt(N) (gfx9 encoding: vmcnt in bits [3:0] and [15:14], expcnt [6:4], lgkmcnt [11:8])
// Also waits for this wave's LDS accesses (lgkmcnt = 0): the barrier that follows is a bare s_barrier.
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (0 << 8));
}

// Workgroup barrier without the release / acquire fences of __syncthreads(): those would make the
// compiler wait for every direct-to-LDS load in flight (they are LDS writes), i.e. for the whole
// prefetch.  What must have landed is waited for explicitly (wait_vmcnt) before this is called; the
// signal fences keep the compiler from moving memory accesses across the barrier.
__device__ __forceinline__ void bare_barrier() {
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    __builtin_amdgcn_s_barrier();
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
}

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 2) & 3); }

// INT4: one thread turns its 32 codes of a k step (16 bytes of the streaming layout plus the scale / zero word,
// both fetched into `raw` by this same lane) into bf16 RNE((q - z) s) and writes the 64-byte row slice
// of the weight tile.  Restrict pointers for the same reason as in mfma_step.
__device__ __forceinline__ void dequant_row(const uint8_t *__restrict__ raw_w, const uint8_t *__restrict__ raw_sz,
                                            uint8_t *__restrict__ Bs, int tid) {
    const int lane = tid & 63, wave = tid >> 6;
    const u32x4_t w = *reinterpret_cast<const u32x4_t *>(raw_w + wave * 1024 + lane * 16);
    const uint32_t szw = *reinterpret_cast<const uint32_t *>(raw_sz + wave * 256 + lane * 4);
    const int row = tid;                                       // tile tid / 16, row tid % 16 of it
    const float s = __uint_as_float(szw << 16);
    const float czs = __uint_as_float(szw & 0xFFFF0000u) * s;   // -(128 + z) s, exact
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        uint32_t o[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t pair = ((w[t] >> (4 * q)) & 0x000F000Fu) | 0x43004300u;
            const float lo = fmaf(__uint_as_float(pair << 16), s, czs);
            const float hi = fmaf(__uint_as_float(pair & 0xFFFF0000u), s, czs);
            o[q] = pack_bf16x2(lo, hi);
        }
        const u32x4_t v = {o[0], o[1], o[2], o[3]};
        *reinterpret_cast<u32x4_t *>(Bs + row * ROW_BYTES + swz(row, t) * 16) = v;
    }
}

// The MFMAs of one k step on one LDS stage.  The operand pointers are `__restrict__` on purpose: after
// inlining, the LDS reads carry alias scopes, which is what lets the compiler's wait-count pass tell
// them apart from the direct-to-LDS loads in flight into the other stages (without scopes it waits for
// every outstanding load before the first LDS read, which would serialise the pipeline; the wait for
// the stage that is read here is the explicit one in the caller).
__device__ __forceinline__ void mfma_step(const uint8_t *__restrict__ As, const uint8_t *__restrict__ Bs,
                                          f32x16 (&acc)[4][4], int lane, int wm, int wn) {
    Frag a[2][4], b[2][4];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        const int chunk = ks * 2 + (lane >> 5);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int ra = wm * 128 + i * 32 + (lane & 31);
            const int rb = wn * 128 + i * 32 + (lane & 31);
            a[ks][i].u = *reinterpret_cast<const uint4 *>(As + ra * ROW_BYTES + swz(ra, chunk) * 16);
            b[ks][i].u = *reinterpret_cast<const uint4 *>(Bs + rb * ROW_BYTES + swz(rb, chunk) * 16);
        }
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks][i].v, b[ks][j].v, acc[i][j], 0, 0, 0);
}

template <bool W4, bool OUT_F32>
__global__ __launch_bounds__(256) void gemm_dma_kernel(const void *__restrict__ wsrc, const uint32_t *__restrict__ sz,
                                                       const uint16_t *__restrict__ x, void *__restrict__ y,
                                                       int64_t M, int64_t K, int64_t N, int nbn, int lg_xm) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];   // NS stages of {A, B}
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    int tm, tn;
    if (lg_xm < 0) {            // plain order: column blocks fastest
        tm = (int)blockIdx.x / nbn;
        tn = (int)blockIdx.x % nbn;
    } else {
        // XCD-aware order (as in the register-staged kernel): linear index -> (region, XCD, slot in a 4 x 8 patch)
        const int region = (int)blockIdx.x >> 8, r = (int)blockIdx.x & 255;
        const int xcd = r & 7, q = r >> 3;
        const int xn = 8 >> lg_xm;
        const int regions_n = nbn / (8 * xn);
        tm = (region / regions_n) * (4 << lg_xm) + (xcd / xn) * 4 + (q >> 3);
        tn = (region % regions_n) * 8 * xn + (xcd % xn) * 8 + (q & 7);
    }
    const int64_t n0 = (int64_t)tn * BN;
    const int64_t m0 = (int64_t)tm * BM;
    const int steps = (int)(K / BK);

    // ---- direct-to-LDS loads: wave w fills rows [64 w, 64 w + 64) of an operand, 16 rows per instruction
    const uint16_t *ga[4];
    const uint16_t *gb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = wave * 64 + i * 16 + (lane >> 2);
        const int chunk = swz(row, lane & 3);
        const int64_t m = m0 + row < M ? m0 + row : M - 1;
        ga[i] = x + m * K + chunk * 8;
        if constexpr (!W4) {
            const int64_t n = n0 + row < N ? n0 + row : N - 1;
            gb[i] = reinterpret_cast<const uint16_t *>(wsrc) + n * K + chunk * 8;
        }
    }
    auto issue_dma = [&](int step) {
        uint8_t *stage = lds + (step % NS) * STAGE_BYTES;
        const int64_t k0 = (int64_t)step * BK;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __builtin_amdgcn_global_load_lds((global_void *)(ga[i] + k0),
                                             (lds_void *)(stage + (wave * 64 + i * 16) * ROW_BYTES), 16, 0, 0);
        if constexpr (!W4) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                __builtin_amdgcn_global_load_lds((global_void *)(gb[i] + k0),
                                                 (lds_void *)(stage + OPERAND_BYTES + (wave * 64 + i * 16) * ROW_BYTES),
                                                 16, 0, 0);
        }
    };

    // ---- INT4 weight slices: thread -> (tile tid / 16, row j = tid % 16); the 32 weights of a k step are the
    // 16 bytes of lane 16 c + j of the tile's block, c = (k0 % 128) / 32.  Every lane fetches its own
    // 16 + 4 bytes into the raw ring (direct to LDS as well) and reads them back itself one step later.
    uint8_t *raw = lds + LDS_BYTES_BF16;
    const int wt_j = tid & 15;
    const int64_t groups = K / kGroup;
    int64_t wT = n0 / kTileRows + (tid >> 4);
    const int64_t tiles_n = N / kTileRows;
    if (wT >= tiles_n) wT = tiles_n - 1;
    auto issue_raw = [&](int step) {
        const int64_t k0 = (int64_t)step * BK;
        const int64_t block = wT * groups + k0 / kGroup;
        const int c = (int)((k0 % kGroup) / 32);
        uint8_t *slot = raw + (step % NR) * RAW_BYTES;
        __builtin_amdgcn_global_load_lds((global_void *)(reinterpret_cast<const u32x4_t *>(wsrc) + block * 64 + c * 16 + wt_j),
                                         (lds_void *)(slot + wave * 1024), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((global_void *)(sz + block * kTileRows + wt_j),
                                         (lds_void *)(slot + RAW_W_BYTES + wave * 256), 4, 0, 0);
    };
    auto dequant = [&](int step) {
        const uint8_t *slot = raw + (step % NR) * RAW_BYTES;
        dequant_row(slot, slot + RAW_W_BYTES, lds + (step % NS) * STAGE_BYTES + OPERAND_BYTES, tid);
    };

    f32x16 acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    // Load instructions of a wave in issue order.  bf16: step j issues D(j + 3) (8 instructions).  INT4: step j
    // issues A(j + 3) (4) and then R(j + 4) (2), the raw slice one step further ahead because it has to be
    // dequantised a step before it is multiplied.  vmcnt retires in order, so "everything up to D(kt)" resp.
    // "up to R(kt + 1)" has landed when at most the instructions of the two following steps are outstanding
    // (fewer near the end of k).  The prologue issues in the same order.
    constexpr int L = W4 ? 6 : 8;
    if constexpr (W4) {
        issue_raw(0);
        issue_dma(0);
        issue_raw(1);
        issue_dma(1);
        issue_raw(2);
        issue_dma(2);
        issue_raw(3);
        wait_vmcnt<3 * L>();     // R(0) has landed (read back by the lane that fetched it: no barrier needed)
        dequant(0);
    } else {
        issue_dma(0);
        issue_dma(1);
        issue_dma(2);
    }

    for (int kt = 0; kt < steps; ++kt) {
        const int rem = steps - 1 - kt;
        if constexpr (W4) {
            if (rem >= 3)
                wait_vmcnt<12>();
            else if (rem == 2)
                wait_vmcnt<10>();
            else if (rem == 1)
                wait_vmcnt<4>();
            else
                wait_vmcnt<0>();
        } else {
            if (rem >= 2)
                wait_vmcnt<16>();
            else if (rem == 1)
                wait_vmcnt<8>();
            else
                wait_vmcnt<0>();
        }
        bare_barrier();      // everyone's loads (and dequantised rows) of step kt are visible; everyone has left stage (kt - 1) % NS
        if (kt + 3 < steps) issue_dma(kt + 3);
        if constexpr (W4) {
            if (kt + 4 < steps) issue_raw(kt + 4);
        }
        const uint8_t *As = lds + (kt % NS) * STAGE_BYTES;
        mfma_step(As, As + OPERAND_BYTES, acc, lane, wm, wn);
        if constexpr (W4) {
            // weights of step kt + 1 into their stage (last read at step kt - 3)
            if (kt + 1 < steps) dequant(kt + 1);
        }
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
hipError_t launch_one(const void *wsrc, const uint32_t *sz, const uint16_t *x, int64_t M, int64_t K, int64_t N,
                      void *y, hipStream_t stream) {
    if (K / BK < 4) return hipErrorInvalidValue;
    static const hipError_t attr_status = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_dma_kernel<W4, OUT_F32>),
                                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)(W4 ? LDS_BYTES_W4 : LDS_BYTES_BF16));
    if (attr_status != hipSuccess) return attr_status;
    const int nbm = (int)((M + BM - 1) / BM), nbn = (int)((N + BN - 1) / BN);
    int lg_xm = 2;      // XCD-aware order when the tile grid divides evenly (see the register-staged kernel)
    while (lg_xm >= 0 && (nbm % (4 << lg_xm) != 0 || nbn % (8 * (8 >> lg_xm)) != 0)) --lg_xm;
    hipLaunchKernelGGL((gemm_dma_kernel<W4, OUT_F32>), dim3((unsigned)(nbm * nbn)), dim3(256), W4 ? LDS_BYTES_W4 : LDS_BYTES_BF16, stream, wsrc,
                       sz, x, y, M, K, N, nbn, lg_xm);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_w4_gemm_dma(const LayerView &L, const uint16_t *x, int64_t M, void *y, bool out_f32,
                              hipStream_t stream) {
    return out_f32 ? launch_one<true, true>(L.wt, L.sz, x, M, L.K, L.N, y, stream)
                   : launch_one<true, false>(L.wt, L.sz, x, M, L.K, L.N, y, stream);
}

hipError_t launch_bf16_gemm_dma(const uint16_t *w, const uint16_t *x, int64_t M, int64_t K, int64_t N, void *y,
                                bool out_f32, hipStream_t stream) {
    return out_f32 ? launch_one<false, true>(w, nullptr, x, M, K, N, y, stream)
                   : launch_one<false, false>(w, nullptr, x, M, K, N, y, stream);
}

}  // namespace dmr

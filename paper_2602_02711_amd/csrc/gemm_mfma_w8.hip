// 256 x 256 tiles on eight wavefronts: the direct-to-LDS pipeline of the tiled GEMMs with two waves per SIMD that take
// turns at the matrix pipe.
//
// y[M][N] = x[M][K] . W[N][K]^T, bf16 operands, fp32 accumulation.  A workgroup of 8 wavefronts (2 x 4) owns a
// 256 x 256 tile, every wave a 128 x 64 patch = 4 x 2 tiles of v_mfma_f32_32x32x16_bf16: 128 accumulator registers,
// which together with the operand fragments fit the 256 registers a wave has at two waves per SIMD, so the
// accumulators stay in ordinary vector registers.  The two waves of a SIMD alternate between a multiply phase (the 16
// MFMAs of a k step, operands already in registers) and a fetch phase (the step's 12 fragment reads from LDS, the wave's
// share of the global -> LDS loads), so that one of them always has MFMAs to issue: measured 3-9 % ahead of eight waves
// that all run the same software pipeline, which in turn was 3-7 % ahead of four waves with 128 x 128 patches.
// Data movement and LDS layout: `global_load_lds_dwordx4` (every lane names its own 16 global bytes, the wave's
// 64 x 16 bytes land contiguously at a wave-uniform LDS address), four LDS stages of 32 k, rows of 64 bytes with the
// 16-byte chunks XOR-swizzled on the global side, bare barriers, loads three to four steps ahead.
#include "common.hpp"

namespace dmr {

namespace {

constexpr int BK = 32, NS = 4;
constexpr int ROW_BYTES = BK * 2;                          // 64
constexpr int TM = 4, TN = 2;                              // MFMA tiles per wave
constexpr int WM = 2, WN = 4;                              // waves per workgroup
constexpr int BM = 32 * TM * WM, BN = 32 * TN * WN;        // 256 x 256
constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BN * ROW_BYTES;
constexpr int STAGE_BYTES = A_BYTES + B_BYTES;             // 32 KiB
constexpr size_t LDS_BYTES = (size_t)NS * STAGE_BYTES;     // 128 KiB
constexpr int LA = BM / 16 / (WM * WN), LB = BN / 16 / (WM * WN);      // load instructions per wave and step: 2 + 2
constexpr int L = LA + LB;

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void global_void;

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (0 << 8));
}

__device__ __forceinline__ void bare_barrier() {
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    __builtin_amdgcn_s_barrier();
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
}

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 2) & 3); }

__device__ __forceinline__ void load_frags(const uint8_t *__restrict__ As, const uint8_t *__restrict__ Bs, int ks,
                                           Frag (&a)[TM], Frag (&b)[TN], int lane, int wm, int wn) {
    const int chunk = ks * 2 + (lane >> 5);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int ra = wm * 32 * TM + i * 32 + (lane & 31);
        a[i].u = *reinterpret_cast<const uint4 *>(As + ra * ROW_BYTES + swz(ra, chunk) * 16);
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int rb = wn * 32 * TN + j * 32 + (lane & 31);
        b[j].u = *reinterpret_cast<const uint4 *>(Bs + rb * ROW_BYTES + swz(rb, chunk) * 16);
    }
}

__device__ __forceinline__ void mfma_all(const Frag (&a)[TM], const Frag (&b)[TN], f32x16 (&acc)[TM][TN]) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i].v, b[j].v, acc[i][j], 0, 0, 0);
}

// The two waves of a SIMD alternate roles.  Waves 0..3 (rows 0..127 of the tile) multiply step kt (16 MFMAs on fragments
// already in registers, nothing to wait for) while waves 4..7 fetch their fragments of step kt from LDS and issue their
// loads; then the roles swap.  Two barriers per k step, the same number on both paths.  A wave's fragments of a whole k
// step (both sub-steps, 48 registers) live in registers from its fetch phase to its multiply phase.
template <bool OUT_F32>
__global__ __launch_bounds__(512) void gemm_w8_kernel(const uint16_t *__restrict__ w, const uint16_t *__restrict__ x,
                                                         void *__restrict__ y, int64_t M, int64_t K, int64_t N, int nbn, int lg_xm) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const bool first = wm == 0;                      // role group: waves 0..3 multiply in the even phases
    int tm, tn;
    if (lg_xm < 0) {
        tm = (int)blockIdx.x / nbn;
        tn = (int)blockIdx.x % nbn;
    } else {
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

    const uint16_t *gp[L];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        const int row = wave * 16 * LA + i * 16 + (lane >> 2);
        const int64_t m = m0 + row < M ? m0 + row : M - 1;
        gp[i] = x + m * K + swz(row, lane & 3) * 8;
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        const int row = wave * 16 * LB + i * 16 + (lane >> 2);
        const int64_t n = n0 + row < N ? n0 + row : N - 1;
        gp[LA + i] = w + n * K + swz(row, lane & 3) * 8;
    }
    int at = 0;
    auto issue = [&](int step) {                       // this wave's share of a step's loads, into stage step % 4
        uint8_t *stage = lds + (step & 3) * STAGE_BYTES;
        const int target = step < steps ? step : steps - 1;
        const int adv = (target - at) * BK;
        at = target;
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            gp[i] += adv;
            __builtin_amdgcn_global_load_lds((global_void *)gp[i], (lds_void *)(stage + (wave * 16 * LA + i * 16) * ROW_BYTES), 16, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            gp[LA + i] += adv;
            __builtin_amdgcn_global_load_lds((global_void *)gp[LA + i],
                                             (lds_void *)(stage + A_BYTES + (wave * 16 * LB + i * 16) * ROW_BYTES), 16, 0, 0);
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
    Frag fa[2][TM], fb[2][TN];
    auto fetch = [&](int step) {
        const uint8_t *st = lds + (step & 3) * STAGE_BYTES;
        load_frags(st, st + A_BYTES, 0, fa[0], fb[0], lane, wm, wn);
        load_frags(st, st + A_BYTES, 1, fa[1], fb[1], lane, wm, wn);
    };
    auto multiply = [&]() {        // (raising the wave's priority around this block measured 1-2 % slower)
        mfma_all(fa[0], fb[0], acc);
        mfma_all(fa[1], fb[1], acc);
    };

    // Prologue.  Every wave issues its shares of steps 0..2, the first group also of step 3 (in the loop the first group
    // issues step kt + 4 in the odd phase, the second group step kt + 3 in the even phase).
    issue(0);
    issue(1);
    issue(2);
    if (first) {
        issue(3);
        wait_vmcnt<3 * L>();       // step 0 landed
    } else {
        wait_vmcnt<2 * L>();
    }
    bare_barrier();
    if (first) fetch(0);
    wait_vmcnt<3 * L>();           // own LDS reads done (the load count is already satisfied)
    bare_barrier();

    // Two loops, one per role group, with the same number of barriers (two per k step): a single loop with the roles
    // behind branches makes the compiler spill the accumulators at the joins.
    if (first) {
        for (int kt = 0; kt < steps; ++kt) {
            multiply();                // even phase: step kt
            __builtin_amdgcn_sched_barrier(0);
            wait_vmcnt<2 * L>();       // shares of step kt + 1 landed (two younger shares may be in flight)
            bare_barrier();
            fetch(kt + 1);             // odd phase (past the end: the clamped stage, never used)
            __builtin_amdgcn_sched_barrier(0);
            issue(kt + 4);
            __builtin_amdgcn_sched_barrier(0);
            wait_vmcnt<3 * L>();       // own LDS reads done; no new share is needed yet
            bare_barrier();
        }
    } else {
        for (int kt = 0; kt < steps; ++kt) {
            fetch(kt);                 // even phase
            __builtin_amdgcn_sched_barrier(0);
            issue(kt + 3);
            __builtin_amdgcn_sched_barrier(0);
            wait_vmcnt<2 * L>();       // shares of step kt + 1 landed, own LDS reads done
            bare_barrier();
            multiply();                // odd phase: step kt
            __builtin_amdgcn_sched_barrier(0);
            wait_vmcnt<3 * L>();
            bare_barrier();
        }
    }
    wait_vmcnt<0>();

#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int64_t n = n0 + wn * 32 * TN + j * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t m = m0 + wm * 32 * TM + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (m < M && n < N) {
                    if (OUT_F32)
                        reinterpret_cast<float *>(y)[m * N + n] = acc[i][j][r];
                    else
                        reinterpret_cast<uint16_t *>(y)[m * N + n] = f32_to_bf16(acc[i][j][r]);
                }
            }
        }
}

template <bool OUT_F32>
hipError_t launch_one(const uint16_t *w, const uint16_t *x, int64_t M, int64_t K, int64_t N, void *y, hipStream_t stream) {
    if (K / BK < 4) return hipErrorInvalidValue;
    static const hipError_t attr_status = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_w8_kernel<OUT_F32>),
                                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_BYTES);
    if (attr_status != hipSuccess) return attr_status;
    // Workgroups go to the 8 XCDs round-robin by linear index and each XCD has its own L2.  When the
    // grid of 256 x 256 tiles divides evenly, the index is decoded so that the 32 workgroups an XCD runs at
    // a time form a compact 4 x 8 patch of tiles (12 operand panels instead of ~17) and the 8 patches of a
    // round tile a compact region; otherwise plain order (a padded region would leave XCDs idle).
    // Measured at (4096, 28672), M = 8192: L2 hit rate 53 % -> 79 %, time -7 %.  (Walking k in a different
    // order per tile was measured too and is slower: tiles in step share operand panels.)
    const int nbm = (int)((M + BM - 1) / BM), nbn = (int)((N + BN - 1) / BN);
    int lg_xm = 2;
    while (lg_xm >= 0 && (nbm % (4 << lg_xm) != 0 || nbn % (8 * (8 >> lg_xm)) != 0)) --lg_xm;
    hipLaunchKernelGGL((gemm_w8_kernel<OUT_F32>), dim3((unsigned)(nbm * nbn)), dim3(512), LDS_BYTES, stream, w, x, y, M, K, N, nbn,
                       lg_xm);
    return hipGetLastError();
}

}  // namespace

// True when the 256 x 256 tiling gives every CU at least ~1.5 workgroups, or one round that fills at
// least ~80 % of the 256 CUs (one workgroup is resident per CU).
bool gemm_big_applies(int64_t M, int64_t N) {
    const int64_t wgs = ((M + 255) / 256) * ((N + 255) / 256);
    return wgs >= 384 || (wgs >= 208 && wgs <= 256);
}

hipError_t launch_bf16_gemm_w8(const uint16_t *w, const uint16_t *x, int64_t M, int64_t K, int64_t N, void *y, bool out_f32,
                               hipStream_t stream) {
    return out_f32 ? launch_one<true>(w, x, M, K, N, y, stream) : launch_one<false>(w, x, M, K, N, y, stream);
}

}  // namespace dmr

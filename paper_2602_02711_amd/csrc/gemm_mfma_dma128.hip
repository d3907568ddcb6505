// 128 x 128 MFMA GEMM with direct-to-LDS operand loads, bf16 operands: y[M][N] = x[M][K] . W[N][K]^T, fp32
// accumulation.  For the twin's shapes that are too small for 256 x 256 tiles.
//
// A workgroup of 4 wavefronts owns a 128 x 128 tile and every wave a 64 x 64 patch (2 x 2 tiles of
// v_mfma_f32_32x32x16_bf16); 64 KB of LDS, two workgroups per CU.  The operands travel global memory -> LDS without
// passing through registers (`global_load_lds_dwordx4`: every lane names its own 16 global bytes, the wave's
// 64 x 16 bytes land contiguously at a wave-uniform LDS address).  With no staging registers the loads can run three
// to four k steps ahead: four LDS stages of 32 k, one barrier per step, and the wait before it only covers the loads
// issued three steps earlier.  (A first version staged the operands through registers: one step of prefetch was all
// the registers allowed and ~40 % of the time went into waiting for it.)
//
// LDS layout of a stage: operand rows of 32 bf16 = 64 bytes = four 16-byte chunks, unpadded (a load
// instruction fills 16 consecutive rows), chunk c of row r stored at position c ^ ((r >> 2) & 3): the
// 16 lanes of a quarter wave that read the same chunk of 16 consecutive rows then touch 16 different
// 16-byte bank groups.  The swizzle is applied on the global side (lane l of a load instruction owns
// LDS slot l, i.e. row l / 4, position l % 4, and fetches chunk (l % 4) ^ ((row >> 2) & 3) of that row).
// Rows beyond M or N are clamped to the last row (their products are never stored).
#include "common.hpp"

namespace dmr {

namespace {

// T = MFMA tiles per wave and dimension (2: 128 x 128 workgroup tile)
constexpr int BK = 32, NS = 4;
constexpr int ROW_BYTES = BK * 2;                         // 64
template <int T>
struct Geo {
    static constexpr int BT = 64 * T;                              // rows of a workgroup tile (both operands)
    static constexpr int OPERAND_BYTES = BT * ROW_BYTES;           // per operand and stage (8 KiB)
    static constexpr int STAGE_BYTES = 2 * OPERAND_BYTES;          // A then B
    static constexpr size_t LDS_BYTES = (size_t)NS * STAGE_BYTES;  // 64 KiB
};

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

// Operand fragments of one 16-wide k sub-step (ks = 0, 1) of an LDS stage.  The stage pointer is
// `__restrict__` on purpose: after inlining, the LDS reads carry alias scopes, which is what lets the
// compiler's wait-count pass tell them apart from the direct-to-LDS loads in flight into the other stages
// (without scopes it waits for every outstanding load before the first LDS read, which would serialise
// the pipeline; the wait for the stage that is read here is the explicit one in the kernel).
template <int T>
__device__ __forceinline__ void load_frags_ab(const uint8_t *__restrict__ As, const uint8_t *__restrict__ Bs, int ks,
                                              Frag (&a)[T], Frag (&b)[T], int lane, int wm, int wn) {
    const int chunk = ks * 2 + (lane >> 5);
#pragma unroll
    for (int i = 0; i < T; ++i) {
        const int ra = wm * 32 * T + i * 32 + (lane & 31);
        const int rb = wn * 32 * T + i * 32 + (lane & 31);
        a[i].u = *reinterpret_cast<const uint4 *>(As + ra * ROW_BYTES + swz(ra, chunk) * 16);
        b[i].u = *reinterpret_cast<const uint4 *>(Bs + rb * ROW_BYTES + swz(rb, chunk) * 16);
    }
}

template <int T>
__device__ __forceinline__ void load_frags(const uint8_t *stage, int ks, Frag (&a)[T], Frag (&b)[T], int lane, int wm,
                                           int wn) {
    load_frags_ab<T>(stage, stage + Geo<T>::OPERAND_BYTES, ks, a, b, lane, wm, wn);
}

template <int T>
__device__ __forceinline__ void mfma_16(const Frag (&a)[T], const Frag (&b)[T], f32x16 (&acc)[T][T]) {
#pragma unroll
    for (int i = 0; i < T; ++i)
#pragma unroll
        for (int j = 0; j < T; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i].v, b[j].v, acc[i][j], 0, 0, 0);
}

template <bool OUT_F32, int T>
__global__ __launch_bounds__(256) void gemm_dma_kernel(const uint16_t *__restrict__ w, const uint16_t *__restrict__ x,
                                                       void *__restrict__ y, int64_t M, int64_t K, int64_t N, int nbn) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];   // NS stages of {A, B}
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int tm = (int)blockIdx.x / nbn, tn = (int)blockIdx.x % nbn;       // column blocks fastest
    using G = Geo<T>;
    constexpr int BM = G::BT, BN = G::BT, OPERAND_BYTES = G::OPERAND_BYTES, STAGE_BYTES = G::STAGE_BYTES;
    const int64_t n0 = (int64_t)tn * BN;
    const int64_t m0 = (int64_t)tm * BM;
    const int steps = (int)(K / BK);

    // ---- direct-to-LDS loads: wave w fills rows [16 T w, 16 T (w + 1)) of an operand, 16 rows per instruction
    const uint16_t *ga[T];
    const uint16_t *gb[T];
#pragma unroll
    for (int i = 0; i < T; ++i) {
        const int row = wave * 16 * T + i * 16 + (lane >> 2);
        const int chunk = swz(row, lane & 3);
        const int64_t m = m0 + row < M ? m0 + row : M - 1;
        ga[i] = x + m * K + chunk * 8;
        const int64_t n = n0 + row < N ? n0 + row : N - 1;
        gb[i] = w + n * K + chunk * 8;
    }
    // (the loads of a step past the end of k are issued all the same, clamped to the last step and into a
    // stage nobody reads again: every iteration then issues the same instructions, which keeps the wait
    // counts constant and the issue in one basic block with the LDS reads that follow).  The per-lane
    // pointers are advanced in place, so that the address registers of the loads in flight are never
    // reused for anything else.
    int dma_step = 0;            // the step the pointers stand at
    auto issue_dma = [&](int step) {
        uint8_t *stage = lds + (step % NS) * STAGE_BYTES;
        const int target = step < steps ? step : steps - 1;
        const int adv = (target - dma_step) * BK;
        dma_step = target;
#pragma unroll
        for (int i = 0; i < T; ++i) {
            ga[i] += adv;
            __builtin_amdgcn_global_load_lds((global_void *)ga[i],
                                             (lds_void *)(stage + (wave * 16 * T + i * 16) * ROW_BYTES), 16, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < T; ++i) {
            gb[i] += adv;
            __builtin_amdgcn_global_load_lds((global_void *)gb[i],
                                             (lds_void *)(stage + OPERAND_BYTES + (wave * 16 * T + i * 16) * ROW_BYTES), 16, 0, 0);
        }
    };

    f32x16 acc[T][T];
#pragma unroll
    for (int a = 0; a < T; ++a)
#pragma unroll
        for (int b = 0; b < T; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    // Pipeline.  A k step has two 16-wide sub-steps; the fragments of a sub-step are read from LDS while the
    // MFMAs of the sub-step before run, and the one barrier per step sits in the middle of the step:
    //     read (kt, 1) | MFMA (kt, 0) | wait: loads of step kt + 1 landed, own LDS accesses done | barrier |
    //     issue the loads of step kt + 4 into stage kt % 4 (free: everyone's reads of it are complete) |
    //     read (kt + 1, 0) | MFMA (kt, 1)
    // Load instructions of a wave in issue order: iteration j issues D(j + 4), 2 T instructions.  vmcnt retires in
    // order, so everything up to D(kt + 1) has landed when at most the instructions of the two following iterations
    // are outstanding.  The prologue issues in the same order.
    constexpr int L = 2 * T;                           // load instructions per wave and iteration
    Frag fa[2][T], fb[2][T];
#pragma unroll
    for (int j = 0; j < 4; ++j) issue_dma(j);
    wait_vmcnt<3 * L>();
    bare_barrier();
    load_frags<T>(lds, 0, fa[0], fb[0], lane, wm, wn);

    for (int kt = 0; kt < steps; ++kt) {
        const uint8_t *cur = lds + (kt % NS) * STAGE_BYTES;
        const bool more = kt + 1 < steps;                  // uniform over the workgroup
        load_frags<T>(cur, 1, fa[1], fb[1], lane, wm, wn);
        __builtin_amdgcn_sched_barrier(0);
        mfma_16<T>(fa[0], fb[0], acc);
        __builtin_amdgcn_sched_barrier(0);
        if (more) {
            wait_vmcnt<2 * L>();
            bare_barrier();
            load_frags<T>(lds + ((kt + 1) % NS) * STAGE_BYTES, 0, fa[0], fb[0], lane, wm, wn);
            __builtin_amdgcn_sched_barrier(0);
            issue_dma(kt + 4);
        }
        __builtin_amdgcn_sched_barrier(0);
        mfma_16<T>(fa[1], fb[1], acc);
        __builtin_amdgcn_sched_barrier(0);
    }
    wait_vmcnt<0>();           // the clamped loads of the last iterations are still in flight

#pragma unroll
    for (int i = 0; i < T; ++i)
#pragma unroll
        for (int j = 0; j < T; ++j) {
            const int64_t n = n0 + wn * 32 * T + j * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t m = m0 + wm * 32 * T + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (m < M && n < N) {
                    if (OUT_F32)
                        reinterpret_cast<float *>(y)[m * N + n] = acc[i][j][r];
                    else
                        reinterpret_cast<uint16_t *>(y)[m * N + n] = f32_to_bf16(acc[i][j][r]);
                }
            }
        }
}

template <bool OUT_F32, int T>
hipError_t launch_one(const uint16_t *w, const uint16_t *x, int64_t M, int64_t K, int64_t N, void *y, hipStream_t stream) {
    using G = Geo<T>;
    constexpr int BT = G::BT;
    if (K / BK < 4) return hipErrorInvalidValue;
    static const hipError_t attr_status = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_dma_kernel<OUT_F32, T>),
                                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)G::LDS_BYTES);
    if (attr_status != hipSuccess) return attr_status;
    const int nbm = (int)((M + BT - 1) / BT), nbn = (int)((N + BT - 1) / BT);
    hipLaunchKernelGGL((gemm_dma_kernel<OUT_F32, T>), dim3((unsigned)(nbm * nbn)), dim3(256), G::LDS_BYTES, stream, w, x, y, M, K, N,
                       nbn);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_bf16_gemm_dma128(const uint16_t *w, const uint16_t *x, int64_t M, int64_t K, int64_t N, void *y,
                                   bool out_f32, hipStream_t stream) {
    return out_f32 ? launch_one<true, 2>(w, x, M, K, N, y, stream) : launch_one<false, 2>(w, x, M, K, N, y, stream);
}

}  // namespace dmr

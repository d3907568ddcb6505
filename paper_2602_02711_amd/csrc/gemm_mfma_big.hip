// Large-tile MFMA GEMM with direct-to-LDS operand loads: y[M][N] = x[M][K] . W[N][K]^T, fp32 accumulation.
//
// The 128 x 128 kernel is bound by LDS reads (1 KiB of operand fragments per 32x32x16 MFMA).  Here a
// workgroup of 4 wavefronts owns a 256 x 256 tile and every wave a 128 x 128 patch (4 x 4 MFMA tiles, 256
// accumulator registers): 8 fragments feed 16 MFMAs, half the LDS bytes per MFMA.  The bf16 operands travel global memory -> LDS without
// passing through registers (`global_load_lds_dwordx4`: every lane names its own 16 global bytes, the
// wave's 64 x 16 bytes land contiguously at a wave-uniform LDS address).  With no staging registers the
// loads can run three to four k steps ahead: four LDS stages of 32 k (4 x 32 KiB), one barrier per step,
// and the wait before it only covers the loads issued three steps earlier.  (A first version staged the
// operands through registers: one step of prefetch was all the registers allowed, ~40 % of the time went
// into waiting for it, and it measured 6-20 % slower on bf16 weights, 0-8 % on INT4.)
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

// T = MFMA tiles per wave and dimension: 4 -> 256 x 256 workgroup tile, 2 -> 128 x 128 (two workgroups per CU)
constexpr int BK = 32, NS = 4;
constexpr int ROW_BYTES = BK * 2;                         // 64
constexpr int NR = NS + 1;                                // ring of packed INT4 slices (requested one step further ahead)
template <int T>
struct Geo {
    static constexpr int BT = 64 * T;                              // rows of a workgroup tile (both operands)
    static constexpr int OPERAND_BYTES = BT * ROW_BYTES;           // per operand and stage (16 KiB at T = 4)
    static constexpr int STAGE_BYTES = 2 * OPERAND_BYTES;          // A then B
    static constexpr int RAW_W_BYTES = 4096, RAW_SZ_BYTES = 1024;  // per ring slot: 256 rows x (16 + 4) bytes (INT4, T = 4)
    static constexpr int RAW_BYTES = RAW_W_BYTES + RAW_SZ_BYTES;
    static constexpr size_t LDS_BYTES_BF16 = (size_t)NS * STAGE_BYTES;                            // 128 KiB at T = 4
    static constexpr size_t LDS_BYTES_W4 = LDS_BYTES_BF16 + (size_t)NR * RAW_BYTES + 256;         // + 25 KiB of ring
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

// INT4 (256 x 256 tiles only): one thread turns the 32 codes of its weight row and k step (16 bytes of the
// streaming layout plus the scale / zero word, both fetched into `raw` by this same lane) into bf16
// RNE((q - z) s) and writes the row's 64-byte slice of the weight tile.  Restrict pointers for the same reason
// as in the fragment loader below.
__device__ __forceinline__ void dequant_row(const uint8_t *__restrict__ raw_w, const uint8_t *__restrict__ raw_sz,
                                            uint8_t *__restrict__ Bs, int tid) {
    const u32x4_t w = *reinterpret_cast<const u32x4_t *>(raw_w + tid * 16);
    const uint32_t szw = *reinterpret_cast<const uint32_t *>(raw_sz + tid * 4);
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

template <bool W4, bool OUT_F32, int T>
__global__ __launch_bounds__(256) void gemm_big_kernel(const void *__restrict__ wsrc, const uint32_t *__restrict__ sz,
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
        // XCD-aware order (see the launcher): linear index -> (region, XCD, slot in the XCD's 4 x 8 patch)
        const int region = (int)blockIdx.x >> 8, r = (int)blockIdx.x & 255;
        const int xcd = r & 7, q = r >> 3;
        const int xn = 8 >> lg_xm;
        const int regions_n = nbn / (8 * xn);
        tm = (region / regions_n) * (4 << lg_xm) + (xcd / xn) * 4 + (q >> 3);
        tn = (region % regions_n) * 8 * xn + (xcd % xn) * 8 + (q & 7);
    }
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
        if constexpr (!W4) {
            const int64_t n = n0 + row < N ? n0 + row : N - 1;
            gb[i] = reinterpret_cast<const uint16_t *>(wsrc) + n * K + chunk * 8;
        }
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
        if constexpr (!W4) {
#pragma unroll
            for (int i = 0; i < T; ++i) {
                gb[i] += adv;
                __builtin_amdgcn_global_load_lds((global_void *)gb[i],
                                                 (lds_void *)(stage + OPERAND_BYTES + (wave * 16 * T + i * 16) * ROW_BYTES),
                                                 16, 0, 0);
            }
        }
    };

    // ---- INT4 weight slices: thread -> (tile tid / 16, row j = tid % 16); the 32 weights of a k step are the
    // 16 bytes of lane 16 c + j of the tile's block, c = (k0 % 128) / 32.  Every lane fetches its own
    // 16 + 4 bytes into the raw ring (direct to LDS as well) and reads them back itself one step later.
    static_assert(!W4 || T == 4, "the INT4 path assumes one thread per weight row of the tile");
    uint8_t *raw = lds + G::LDS_BYTES_BF16;
    const int wt_j = tid & 15;
    const int64_t groups = K / kGroup;
    int64_t wT = n0 / kTileRows + (tid >> 4);
    const int64_t tiles_n = N / kTileRows;
    if (wT >= tiles_n) wT = tiles_n - 1;
    auto issue_raw = [&](int step) {
        const int64_t k0 = (int64_t)(step < steps ? step : steps - 1) * BK;
        const int64_t block = wT * groups + k0 / kGroup;
        const int c = (int)((k0 % kGroup) / 32);
        uint8_t *slot = raw + (step % NR) * G::RAW_BYTES;
        __builtin_amdgcn_global_load_lds((global_void *)(reinterpret_cast<const u32x4_t *>(wsrc) + block * 64 + c * 16 + wt_j),
                                         (lds_void *)(slot + wave * 1024), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((global_void *)(sz + block * kTileRows + wt_j),
                                         (lds_void *)(slot + G::RAW_W_BYTES + wave * 256), 4, 0, 0);
    };
    auto dequant = [&](int step) {
        const uint8_t *slot = raw + (step % NR) * G::RAW_BYTES;
        dequant_row(slot, slot + G::RAW_W_BYTES, lds + (step % NS) * STAGE_BYTES + OPERAND_BYTES, tid);
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
    // Load instructions of a wave in issue order: iteration j issues D(j + 4) (bf16: 8 instructions; INT4:
    // A(j + 4), 4, then the raw slice R(j + 5), 2, one step further ahead because it is dequantised a step
    // before it is multiplied).  vmcnt retires in order, so everything up to D(kt + 1) resp. R(kt + 2) has
    // landed when at most the instructions of the two following iterations are outstanding.  The prologue
    // issues in the same order.
    constexpr int L = W4 ? T + 2 : 2 * T;              // load instructions per wave and iteration
    Frag fa[2][T], fb[2][T];
    if constexpr (W4) {
        issue_raw(0);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            issue_dma(j);
            issue_raw(j + 1);
        }
        wait_vmcnt<4 * L>();   // R(0) has landed (read back by the lane that fetched it: no barrier needed)
        dequant(0);
        wait_vmcnt<3 * L>();   // ... A(0) and R(1) too
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) issue_dma(j);
        wait_vmcnt<3 * L>();
    }
    bare_barrier();
    load_frags<T>(lds, 0, fa[0], fb[0], lane, wm, wn);

    for (int kt = 0; kt < steps; ++kt) {
        const uint8_t *cur = lds + (kt % NS) * STAGE_BYTES;
        const bool more = kt + 1 < steps;                  // uniform over the workgroup
        load_frags<T>(cur, 1, fa[1], fb[1], lane, wm, wn);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (W4) {
            // The raw slice of step kt + 1 landed before the previous barrier.  Unconditional (after the last
            // step it rewrites a stage nobody reads) so that it shares a scheduling region with the MFMAs
            // below and its ~130 VALU instructions go into their shadow: one MFMA, then eight VALU.
            dequant(kt + 1);
            mfma_16<T>(fa[0], fb[0], acc);
#pragma unroll
            for (int i = 0; i < T * T; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                      // one MFMA
                __builtin_amdgcn_sched_group_barrier(0x002, 144 / (T * T), 0);          // its share of the VALU work
            }
        } else {
            mfma_16<T>(fa[0], fb[0], acc);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (more) {
            wait_vmcnt<2 * L>();
            bare_barrier();
            load_frags<T>(lds + ((kt + 1) % NS) * STAGE_BYTES, 0, fa[0], fb[0], lane, wm, wn);
            __builtin_amdgcn_sched_barrier(0);
            issue_dma(kt + 4);
            if constexpr (W4) issue_raw(kt + 5);
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

template <bool W4, bool OUT_F32, int T>
hipError_t launch_one(const void *wsrc, const uint32_t *sz, const uint16_t *x, int64_t M, int64_t K, int64_t N,
                      void *y, hipStream_t stream) {
    using G = Geo<T>;
    constexpr int BT = G::BT;
    constexpr size_t lds_bytes = W4 ? G::LDS_BYTES_W4 : G::LDS_BYTES_BF16;
    if (K / BK < 4) return hipErrorInvalidValue;
    static const hipError_t attr_status = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_big_kernel<W4, OUT_F32, T>),
                                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (attr_status != hipSuccess) return attr_status;
    // Workgroups go to the 8 XCDs round-robin by linear index and each XCD has its own L2.  When the
    // grid of 256 x 256 tiles divides evenly, the index is decoded so that the 32 workgroups an XCD runs at
    // a time form a compact 4 x 8 patch of tiles (12 operand panels instead of ~17) and the 8 patches of a
    // round tile a compact region; otherwise plain order (a padded region would leave XCDs idle).
    // Measured at (4096, 28672), M = 8192, bf16: L2 hit rate 53 % -> 79 %, time -7 %.  (Walking k in
    // a different order per tile was measured too and is slower: tiles in step share operand panels.)
    const int nbm = (int)((M + BT - 1) / BT), nbn = (int)((N + BT - 1) / BT);
    int lg_xm = T == 4 ? 2 : -1;
    while (lg_xm >= 0 && (nbm % (4 << lg_xm) != 0 || nbn % (8 * (8 >> lg_xm)) != 0)) --lg_xm;
    hipLaunchKernelGGL((gemm_big_kernel<W4, OUT_F32, T>), dim3((unsigned)(nbm * nbn)), dim3(256), lds_bytes, stream, wsrc,
                       sz, x, y, M, K, N, nbn, lg_xm);
    return hipGetLastError();
}

}  // namespace

// True when the 256 x 256 tiling gives every CU at least ~1.5 workgroups, or one round that fills at
// least ~80 % of the 256 CUs (one workgroup is resident per CU).
bool gemm_big_applies(int64_t M, int64_t N) {
    const int64_t wgs = ((M + 255) / 256) * ((N + 255) / 256);
    return wgs >= 384 || (wgs >= 208 && wgs <= 256);
}

hipError_t launch_w4_gemm_big(const LayerView &L, const uint16_t *x, int64_t M, void *y, bool out_f32,
                              hipStream_t stream) {
    return out_f32 ? launch_one<true, true, 4>(L.wt, L.sz, x, M, L.K, L.N, y, stream)
                   : launch_one<true, false, 4>(L.wt, L.sz, x, M, L.K, L.N, y, stream);
}

hipError_t launch_bf16_gemm_big(const uint16_t *w, const uint16_t *x, int64_t M, int64_t K, int64_t N, void *y,
                                bool out_f32, hipStream_t stream) {
    return out_f32 ? launch_one<false, true, 4>(w, nullptr, x, M, K, N, y, stream)
                   : launch_one<false, false, 4>(w, nullptr, x, M, K, N, y, stream);
}

// The same kernel on 128 x 128 tiles (2 x 2 MFMA tiles per wave, two workgroups per CU), bf16 weights only:
// with INT4 weights the dequantisation per k step is amortised over half as many activation rows and the
// register-staged 128 x 128 kernel measured faster.
hipError_t launch_bf16_gemm_dma128(const uint16_t *w, const uint16_t *x, int64_t M, int64_t K, int64_t N, void *y,
                                   bool out_f32, hipStream_t stream) {
    return out_f32 ? launch_one<false, true, 2>(w, nullptr, x, M, K, N, y, stream)
                   : launch_one<false, false, 2>(w, nullptr, x, M, K, N, y, stream);
}

}  // namespace dmr

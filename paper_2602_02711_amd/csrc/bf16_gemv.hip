// bf16 decode GEMV (M == 1): the high-precision twin of the INT4 GEMV, tuned to the same
// standard so that the speed-up ratio has an honest denominator.
//
// W is row-major [N][K], so one row is one contiguous stream.  A wavefront keeps its k slice of x
// in registers (XC chunks of 512 values, 8 per lane) and walks RPW consecutive rows: each row
// costs XC fully coalesced 1 KiB loads (64 lanes x 16 bytes, nontemporal: every line is consumed
// whole, once), 4 XC v_dot2_f32_bf16 per lane and a 6-step lane butterfly.  The loads of row r+1
// are in flight while row r is reduced.  With S > 1 slices per row the partial sums of a
// workgroup's 4 wavefronts meet in LDS and are added in slice order.
#include "glue.hpp"

namespace dmr {

namespace {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

__device__ __forceinline__ float dot8(const uint4 &w, const uint4 &x, float acc) {
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.x), __builtin_bit_cast(bf16x2_t, x.x), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.y), __builtin_bit_cast(bf16x2_t, x.y), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.z), __builtin_bit_cast(bf16x2_t, x.z), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.w), __builtin_bit_cast(bf16x2_t, x.w), acc, false);
    return acc;
}

// Sum over the 64 lanes, the same value in every lane: DPP row sums, then the four row sums through
// scalar registers (no LDS round trips, unlike a shuffle butterfly).
__device__ __forceinline__ float wave_sum(float v) { return wave64_sum(v); }

constexpr int kWaves = 4;   // wavefronts per workgroup

// PRO: glue fused into the load of the activation slice (glue.hpp).  RMSNorm needs the whole row in
// one wave (S == 1); `res`, if not null, is a bf16 residual added to the result.
template <int XC, int PRO>
__global__ __launch_bounds__(kWaves * 64) void bf16_gemv_kernel(const uint16_t *__restrict__ w,
                                                                const uint16_t *__restrict__ x,
                                                                void *__restrict__ y, int64_t K, int64_t N,
                                                                int S, int rpw, int out_f32,
                                                                const uint16_t *__restrict__ aux, float eps,
                                                                const uint16_t *__restrict__ res) {
    extern __shared__ float red[];   // [kWaves][rpw]
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t task = (int64_t)blockIdx.x * kWaves + wave;     // (row block, slice), slice fastest
    const int64_t rb = task / S;
    const int s = (int)(task % S);
    const int64_t k0 = (int64_t)s * XC * 512;
    const int64_t r0 = rb * rpw;
    const int64_t r1 = (r0 + rpw < N) ? r0 + rpw : N;
    const int rows = r0 < N ? (int)(r1 - r0) : 0;

    // this lane's k offsets; beyond K the activation is zero and the weight address is clamped
    uint4 xr[XC];
    int64_t koff[XC];
#pragma unroll
    for (int cidx = 0; cidx < XC; ++cidx) {
        const int64_t k = k0 + cidx * 512 + lane * 8;
        const bool ok = k < K;
        koff[cidx] = ok ? k : 0;
        xr[cidx] = ok ? *reinterpret_cast<const uint4 *>(x + k) : make_uint4(0, 0, 0, 0);
        if (PRO == kProSwiGLU && ok) xr[cidx] = swiglu_piece(xr[cidx], *reinterpret_cast<const uint4 *>(x + K + k));
    }
    if (PRO == kProRmsNorm) {
        float ss = 0.f;
#pragma unroll
        for (int cidx = 0; cidx < XC; ++cidx) ss += sumsq_piece(xr[cidx]);     // zeros beyond K
        const float scale = rms_scale(wave64_sum(ss), 1.0f / (float)K, eps);
#pragma unroll
        for (int cidx = 0; cidx < XC; ++cidx)
            xr[cidx] = rmsnorm_piece(xr[cidx], *reinterpret_cast<const uint4 *>(aux + koff[cidx]), scale);
    }
    auto store_out = [&](int64_t r, float v) {
        if (res) v += __uint_as_float((uint32_t)res[r] << 16);
        if (out_f32)
            reinterpret_cast<float *>(y)[r] = v;
        else
            reinterpret_cast<uint16_t *>(y)[r] = f32_to_bf16(v);
    };

    uint4 cur[XC], nxt[XC];
    auto load_row = [&](uint4 (&dst)[XC], int64_t r) {
        const uint16_t *row = w + r * K;
#pragma unroll
        for (int cidx = 0; cidx < XC; ++cidx)
            dst[cidx] = load_stream(reinterpret_cast<const uint4 *>(row + koff[cidx]));
    };
    auto finish_row = [&](int i) {
        float a0 = 0.f, a1 = 0.f;
#pragma unroll
        for (int cidx = 0; cidx < XC; ++cidx) {
            if (cidx & 1)
                a1 = dot8(cur[cidx], xr[cidx], a1);
            else
                a0 = dot8(cur[cidx], xr[cidx], a0);
        }
        const float sum = wave_sum(a0 + a1);
        if (lane == 0) {
            if (S > 1)
                red[wave * rpw + i] = sum;
            else
                store_out(r0 + i, sum);
        }
    };
    if (rows > 0) {
        load_row(cur, r0);
        for (int i = 0; i + 1 < rows; ++i) {
            load_row(nxt, r0 + i + 1);      // next row in flight while this one is reduced
            finish_row(i);
#pragma unroll
            for (int cidx = 0; cidx < XC; ++cidx) cur[cidx] = nxt[cidx];
        }
        finish_row(rows - 1);
    }
    if (S == 1) return;
    __syncthreads();
    // the S slices of a row block sit in adjacent wavefronts of this workgroup (S divides kWaves)
    const int blocks_here = kWaves / S;
    for (int e = threadIdx.x; e < blocks_here * rpw; e += blockDim.x) {
        const int b = e / rpw, i = e % rpw;
        const int64_t r = ((int64_t)blockIdx.x * blocks_here + b) * rpw + i;
        if (r < N) {
            float sum = 0.f;
            for (int q = 0; q < S; ++q) sum += red[(b * S + q) * rpw + i];
            store_out(r, sum);
        }
    }
}

}  // namespace

// Whether the bf16 decode kernel takes rows of K values (at most eight 512-value chunks of x per wave after
// slicing a row over the waves of a workgroup); longer rows go to the direct-from-L2 kernel.
bool bf16_gemv_fits(int64_t K) {
    const int64_t chunks = (K + 511) / 512;
    return (chunks + kWaves - 1) / kWaves <= 8;
}

hipError_t launch_bf16_gemv(const uint16_t *w, const uint16_t *x, int64_t K, int64_t N, void *y,
                            bool out_f32, hipStream_t stream) {
    return launch_bf16_gemv_fused(w, x, K, N, y, out_f32, Fusion{}, stream);
}

hipError_t launch_bf16_gemv_fused(const uint16_t *w, const uint16_t *x, int64_t K, int64_t N, void *y, bool out_f32,
                                  const Fusion &f, hipStream_t stream) {
    // slices per row: keep at most 8 chunks of 512 values of x in registers
    const int64_t chunks = (K + 511) / 512;
    int S = 1;
    while (S < kWaves && (chunks + S - 1) / S > 8) S <<= 1;
    const int XC = (int)((chunks + S - 1) / S);
    if (XC > 8) return hipErrorInvalidValue;   // K > 16384: the caller uses the general kernel
    // rows per wave: aim at ~2048 wavefronts (8 per CU; measured 3-10 % ahead of 4096 on the four decoder
    // shapes and the vocabulary projection, 1024 and 8192 in between) but at least 1 row, at most 64
    const int64_t target_waves = env_int("DMR_BF16_GEMV_WAVES", 2048);
    int64_t rpw = (N * S + target_waves - 1) / target_waves;
    if (rpw < 1) rpw = 1;
    if (rpw > 64) rpw = 64;
    const int64_t row_blocks = (N + rpw - 1) / rpw;
    const int64_t tasks = row_blocks * S;
    const unsigned grid = (unsigned)((tasks + kWaves - 1) / kWaves);
    const size_t lds = S > 1 ? (size_t)kWaves * rpw * sizeof(float) : 0;
    const int of = out_f32 ? 1 : 0;
    const int irpw = (int)rpw;
    if (f.pro == kProRmsNorm && S != 1) return hipErrorInvalidValue;   // the row must sit in one wave
#define DMR_BF16_GEMV_LAUNCH(X, PRO)                                                                   \
    hipLaunchKernelGGL((bf16_gemv_kernel<X, PRO>), dim3(grid), dim3(kWaves * 64), lds, stream, w, x, y, K, N, \
                       S, irpw, of, f.aux, f.eps, f.res)
#define DMR_BF16_GEMV_CASE(X)                                                                          \
    case X:                                                                                            \
        if (f.pro == kProRmsNorm) DMR_BF16_GEMV_LAUNCH(X, kProRmsNorm);                                 \
        else if (f.pro == kProSwiGLU) DMR_BF16_GEMV_LAUNCH(X, kProSwiGLU);                              \
        else DMR_BF16_GEMV_LAUNCH(X, kProNone);                                                         \
        break;
    switch (XC) {
        DMR_BF16_GEMV_CASE(1) DMR_BF16_GEMV_CASE(2) DMR_BF16_GEMV_CASE(3) DMR_BF16_GEMV_CASE(4)
        DMR_BF16_GEMV_CASE(5) DMR_BF16_GEMV_CASE(6) DMR_BF16_GEMV_CASE(7) DMR_BF16_GEMV_CASE(8)
        default: return hipErrorInvalidValue;
    }
#undef DMR_BF16_GEMV_CASE
#undef DMR_BF16_GEMV_LAUNCH
    return hipGetLastError();
}

}  // namespace dmr

// Shared declarations of the gfx950 kernels behind dmr_qlinear.h.
//
// Internal ("streaming") layout of a quantised layer, written once by the re-tiling kernel:
//
//   weights: a 1 KiB block per (row tile T = n / 16, group G = k / 128), blocks ordered
//            [T][G], so a wave that walks along k for its 16 rows reads one contiguous stream.
//            Inside a block, lane l = 16 c + j of a wavefront owns 16 bytes at offset 16 l:
//            row n = 16 T + j, the 32 weights k = 128 G + 32 c + 8 t + p (t = word 0..3,
//            p = 0..7).  Within a word, position p sits in nibble (p >> 1) + 4 (p & 1), so that
//            ((word >> 4 i) & 0x000F000F) | 0x43004300 is the bf16 pair (128 + q[p = 2 i],
//            128 + q[p = 2 i + 1]): one MFMA B-operand register, k-consecutive like the
//            activations.
//   sz:      after the weights, one uint32 per (T, G, j): low half = bf16 scale s, high half =
//            bf16 of -(128 + z) (exact: 128..143 needs 8 significant bits).
//
// With D = sum_k x_k (128 + q_k) and X = sum_k x_k over one group, the group's contribution to
// an output is  s * (D - (128 + z) * X): the zero point and the scale cost two FMAs per group
// instead of work per weight, and D, X come out of the matrix cores.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cstdlib>

#include "../../include/dmr_qlinear.h"

namespace dmr {

constexpr int kGroup = 128;      // weights per (scale, zero) along k
constexpr int kTileRows = 16;    // rows of one streaming block
constexpr int kBlockBytes = 1024;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

union Frag {
    uint4 u;
    uint32_t w[4];
    bf16x8 v;
};

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t bits16) {
    return __uint_as_float(bits16 << 16);
}

// fp32 -> bf16 bits, round to nearest even (v_cvt_pk_bf16_f32 on gfx950).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    return (uint16_t)(pack_bf16x2(f, 0.0f) & 0xFFFFu);
}

// Streaming (read-once) loads: keep weight traffic from displacing the activations in the caches.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream(const uint4 *p) {
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint32_t load_stream(const uint32_t *p) { return __builtin_nontemporal_load(p); }

// Sum over each aligned group of 16 lanes (a DPP "row"), result in every lane: four rotate-and-add
// steps on the VALU, no LDS round trip.
template <int N>
__device__ __forceinline__ float row_ror_add(float v) {
    return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x120 + N, 0xF, 0xF, false));
}
// v as seen through a DPP control word (quad_perm, row_mirror, ...), all lanes and banks enabled.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ float row16_sum(float v) {
    v = row_ror_add<8>(v);
    v = row_ror_add<4>(v);
    v = row_ror_add<2>(v);
    return row_ror_add<1>(v);
}

// One streaming-layout word (8 nibbles) -> four MFMA B-operand registers, register i = the bf16 pair
// (128 + nibble i, 128 + nibble i + 4), i.e. ((w >> 4 i) & 0x000F000F) | 0x43004300, in 7 VALU
// instructions: two masks split the nibbles into bytes and v_perm_b32 interleaves them with the
// 0x43 exponent byte (selector bytes 4..7 pick bytes of the first source, 0..3 of the second).
// Deliberately no inline assembly: the wait states an MFMA needs after a VALU write of its
// operands are only inserted by the compiler for instructions it emitted itself.
__device__ __forceinline__ void unpack_word(uint32_t w, uint32_t (&out)[4]) {
    const uint32_t even = w & 0x0F0F0F0Fu;            // nibbles 0, 2, 4, 6 as bytes
    const uint32_t odd = (w >> 4) & 0x0F0F0F0Fu;      // nibbles 1, 3, 5, 7
    const uint32_t exp = 0x43434343u;
    out[0] = __builtin_amdgcn_perm(even, exp, 0x00060004u);   // nibbles 0, 4
    out[1] = __builtin_amdgcn_perm(odd, exp, 0x00060004u);    // nibbles 1, 5
    out[2] = __builtin_amdgcn_perm(even, exp, 0x00070005u);   // nibbles 2, 6
    out[3] = __builtin_amdgcn_perm(odd, exp, 0x00070005u);    // nibbles 3, 7
}

// Position p (0..7) of a streaming-layout word -> nibble index.
__host__ __device__ __forceinline__ int nibble_of_position(int p) { return (p >> 1) + 4 * (p & 1); }

// Launch-shape overrides for tuning sweeps: read only when DMR_TUNING is set in the environment (one
// lookup per process), so that production launches never touch the environment.
inline int env_int(const char *name, int fallback) {
    static const bool tuning = std::getenv("DMR_TUNING") != nullptr;
    if (!tuning) return fallback;
    const char *v = std::getenv(name);
    return (v && *v) ? std::atoi(v) : fallback;
}

// Compute units the launch shapes are planned for: a whole MI355X.  A constant, not a device query, so that
// the host-side planners behind the workspace queries and the launchers always agree with each other (on a
// partition with fewer CUs the shapes stay correct, only less well balanced).
constexpr int kCus = 256;
inline constexpr int compute_units() { return kCus; }

struct LayerView {
    int64_t K, N;
    const uint4 *wt;       // streaming weight blocks
    const uint32_t *sz;    // streaming scale / zero words
    int szs = 1;           // 1: one scale / zero word per (row, group); 0: one per row (per-channel layers)
};

// Index of the scale / zero word of row j of tile `tile` for group g: [tile][group][16] with one word per group
// (szs = 1), or [tile][16] with one word per row, whatever the group (szs = 0).
__host__ __device__ __forceinline__ int64_t sz_index(int64_t tile, int64_t g, int64_t groups, int szs, int j) {
    return (tile * (szs * (groups - 1) + 1) + g * szs) * kTileRows + j;
}

struct LayerView3 {       // 3-bit variant: 64 lanes x 3 words per block
    int64_t K, N;
    const uint32_t *wt;
    const uint32_t *sz;
};

inline size_t weight3_region_bytes(int64_t K, int64_t N) { return (size_t)N * (size_t)K / 32 * 12; }
inline size_t weight_region_bytes(int64_t K, int64_t N) { return (size_t)N * (size_t)K / 2; }
inline size_t sz_region_bytes(int64_t K, int64_t N) { return (size_t)N * (size_t)(K / kGroup) * 4; }
inline size_t sz_region_bytes_per_channel(int64_t N) { return (size_t)N * 4; }

// Kernel launchers (each returns hipGetLastError() after its launch).
hipError_t launch_retile(int64_t K, int64_t N, const uint32_t *qweight, const uint16_t *scales,
                         const uint16_t *zeros, uint4 *wt, uint32_t *sz, bool per_channel,
                         hipStream_t stream);
hipError_t launch_dequantize(const LayerView &L, uint16_t *w_bf16, hipStream_t stream);
hipError_t launch_quantize(int64_t K, int64_t N, const float *w, uint32_t *qweight,
                           uint16_t *scales, uint16_t *zeros, hipStream_t stream);
// M == 1 decode kernel; returns hipErrorInvalidValue (nothing launched) for shapes it does not take.
bool w4_gemv_fits(int64_t K, int64_t N, bool with_residual);
hipError_t launch_w4_gemv(const LayerView &L, const uint16_t *x, void *y, bool out_f32,
                          hipStream_t stream);
// M == 1 bf16 kernel; hipErrorInvalidValue (nothing launched) for K beyond its range.
bool bf16_gemv_fits(int64_t K);
hipError_t launch_bf16_gemv(const uint16_t *w, const uint16_t *x, int64_t K, int64_t N, void *y,
                            bool out_f32, hipStream_t stream);
// 2 <= M <= 16 streaming kernel; hipErrorInvalidValue (nothing launched) when the activations do not fit LDS.
bool w4_stream_fits(int64_t M, int64_t K, int64_t N);
hipError_t launch_w4_stream(const LayerView &L, const uint16_t *x, int64_t M, void *y, bool out_f32,
                            hipStream_t stream);
// bf16 twin of the streaming kernel (optional residual added at the store).
bool bf16_stream_fits(int64_t M, int64_t K, int64_t N);
hipError_t launch_bf16_stream(const uint16_t *w, const uint16_t *x, int64_t M, int64_t K, int64_t N, void *y,
                              bool out_f32, const uint16_t *res, hipStream_t stream);
// 16 < M <= 64: activation pre-pass into `ws` (w4_skinny2_workspace_bytes), then the streaming kernel.
size_t w4_skinny2_workspace_bytes(int64_t M, int64_t K);
hipError_t launch_w4_skinny2(const LayerView &L, const uint16_t *x, int64_t M, void *y, bool out_f32,
                             void *ws, hipStream_t stream);
// 16 < M up to a few hundred rows: weights straight into registers, activations through LDS, optional
// split of K whose fp32 partials go to `ws` (w4_mid_workspace_bytes) and are added by a second kernel.
size_t w4_mid_workspace_bytes(int64_t M, int64_t K, int64_t N);
hipError_t launch_w4_mid(const LayerView &L, const uint16_t *x, int64_t M, void *y, bool out_f32, void *ws,
                         hipStream_t stream);
// The same kernel on a 3-bit layer (same plan and workspace as launch_w4_mid).
hipError_t launch_w3_mid(const LayerView3 &L, const uint16_t *x, int64_t M, void *y, bool out_f32, void *ws,
                         hipStream_t stream);
// bf16 twin of launch_w4_mid.
size_t bf16_mid_workspace_bytes(int64_t M, int64_t K, int64_t N);
hipError_t launch_bf16_mid(const uint16_t *w, const uint16_t *x, int64_t M, int64_t K, int64_t N, void *y,
                           bool out_f32, void *ws, hipStream_t stream);
hipError_t launch_retile3(int64_t K, int64_t N, const uint32_t *qweight, const uint16_t *scales,
                          const uint16_t *zeros, uint32_t *wt, uint32_t *sz, hipStream_t stream);
hipError_t launch_dequantize3(const LayerView3 &L, uint16_t *w_bf16, hipStream_t stream);
hipError_t launch_quantize3(int64_t K, int64_t N, const float *w, uint32_t *qweight, uint16_t *scales,
                            uint16_t *zeros, hipStream_t stream);
// 2 <= M <= 16 on a 3-bit layer; hipErrorInvalidValue (nothing launched) when the activations do not fit LDS.
hipError_t launch_w3_stream(const LayerView3 &L, const uint16_t *x, int64_t M, void *y, bool out_f32,
                            hipStream_t stream);
bool w3_gemv_fits(int64_t K, int64_t N);
hipError_t launch_w3_gemv(const LayerView3 &L, const uint16_t *x, void *y, bool out_f32, hipStream_t stream);
hipError_t launch_hbm_read_probe(const void *buf, size_t bytes, uint32_t *sink, int blocks,
                                 hipStream_t stream);
hipError_t launch_empty_probe(int blocks, int threads, size_t lds_bytes, hipStream_t stream);
hipError_t launch_w4_skinny(const LayerView &L, const uint16_t *x, int64_t M, void *y, bool out_f32,
                            hipStream_t stream);
hipError_t launch_bf16_skinny(const uint16_t *w, const uint16_t *x, int64_t M, int64_t K, int64_t N,
                              void *y, bool out_f32, hipStream_t stream);
// 128 x 128 tiles on the exact integer codes q - z; the scale is applied per group in fp32.
hipError_t launch_w4_gemm(const LayerView &L, const uint16_t *x, int64_t M, void *y, bool out_f32, hipStream_t stream);
// The exact kernel restricted to the column blocks of 128 rows with a nonzero word in `only` (device memory, one word
// per 32 rows; `pairs`: to the aligned pairs of blocks with one).
hipError_t launch_w4_gemm_flagged(const LayerView &L, const uint16_t *x, int64_t M, void *y, bool out_f32,
                                  const uint32_t *only, bool pairs, hipStream_t stream);
// 256 x 256 or 256 x 128 tiles on the exact codes 16 + q with one accumulator tile kept in units of the current group's scale;
// a pre-pass writes the zero-point operands, the rescale factors and per-column-block flags into `ws`
// (w4_gemm_rescale_workspace_bytes), and the 128 x 128 exact kernel takes the column blocks it flags.
bool w4_gemm_rescale_applies(int64_t M, int64_t N);
int w4_gemm_rescale_tile_rows(int64_t M, int64_t N);      // 128: 128 x 128 tiles (then the next function does not apply); 256
int w4_gemm_rescale_wave_columns(int64_t M, int64_t N);   // 4: 256 x 256 tiles; 2: 256 x 128
size_t w4_gemm_rescale_workspace_bytes(int64_t M, int64_t K, int64_t N);
hipError_t launch_w4_gemm_rescale(const LayerView &L, const uint16_t *x, int64_t M, void *y, bool out_f32, void *ws,
                                  hipStream_t stream);
// The exact-code 128 x 128 kernel on a 3-bit layer; the 256-row kernel and its fallback for flagged column blocks.
hipError_t launch_w3_gemm(const LayerView3 &L, const uint16_t *x, int64_t M, void *y, bool out_f32, hipStream_t stream);
hipError_t launch_w3_gemm_flagged(const LayerView3 &L, const uint16_t *x, int64_t M, void *y, bool out_f32,
                                  const uint32_t *only, bool pairs, hipStream_t stream);
hipError_t launch_w3_gemm_rescale(const LayerView3 &L, const uint16_t *x, int64_t M, void *y, bool out_f32, void *ws,
                                  hipStream_t stream);
hipError_t launch_bf16_gemm(const uint16_t *w, const uint16_t *x, int64_t M, int64_t K, int64_t N,
                            void *y, bool out_f32, hipStream_t stream);
// 256 x 256 tiles on eight wavefronts (direct-to-LDS operand loads, four-stage pipeline, two waves per SIMD) for
// problems large enough to fill the chip with them.
bool gemm_big_applies(int64_t M, int64_t N);
hipError_t launch_bf16_gemm_w8(const uint16_t *w, const uint16_t *x, int64_t M, int64_t K, int64_t N, void *y, bool out_f32,
                               hipStream_t stream);
hipError_t launch_bf16_gemm_dma128(const uint16_t *w, const uint16_t *x, int64_t M, int64_t K, int64_t N,
                                   void *y, bool out_f32, hipStream_t stream);

}  // namespace dmr

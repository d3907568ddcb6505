// C ABI of dmr_qlinear.h: argument checks (all before the first HIP call), the host handle, and
// the choice of kernel by M.  No device memory is allocated here or anywhere in the library.
#include <new>

#include "glue.hpp"
#include "panel_plan.hpp"
#include "wide_plan.hpp"

struct dmr_qlinear {
    int64_t K, N;
    int32_t g;
    int32_t bits;           // 4, or 3 for the W3A16 variant
    const uint4 *wt;        // 4-bit streaming blocks
    const uint32_t *wt3;    // 3-bit streaming blocks
    const uint32_t *sz;
    int32_t szs;            // 1: a scale / zero word per (row, group); 0: one per row (per-channel layers)
};

namespace {

constexpr int64_t kSkinnyMaxM = 64;

// Which INT4 kernel serves M rows of a (K, N) layer (measured crossovers, 256 CUs).  The workspace
// query and the forward call both go through this.
enum class W4Path { Gemv, Stream, Panel, Wide, Skinny2, Mid, Gemm, GemmRescale };
constexpr int kTiledMinBlocks = 140;
W4Path w4_path(int64_t M, int64_t K, int64_t N) {
    if (M == 1) return W4Path::Gemv;
    if (M <= 16) {
        if (dmr::w4_stream_fits(M, K, N)) return W4Path::Stream;
        // long rows: k-sliced panels of x in LDS (measured 10-15 % ahead of the rollout-batch kernel)
        return dmr::w4_panel_applies(M, K, N) ? W4Path::Panel : W4Path::Mid;
    }
    if (M <= kSkinnyMaxM && dmr::w4_wide_applies(M, K, N)) return W4Path::Wide;
    const int64_t tiles = N / dmr::kTileRows;
    // wide layers already give the register-blocked streaming kernel 4 tiles per workgroup
    if (M <= kSkinnyMaxM) return tiles >= 1024 ? W4Path::Skinny2 : W4Path::Mid;
    // the tiled GEMM wins from about 140 output blocks of 128 x 128 on (measured: ahead at 144 and from there on, on
    // 128-row tiles up to 256 blocks and on 256-row tiles beyond; behind at 128)
    const int64_t gemm_wgs = ((M + 127) / 128) * ((N + 127) / 128);
    if (M <= 128 || gemm_wgs < dmr::env_int("DMR_W4_GEMM_MIN_WGS", kTiledMinBlocks)) return W4Path::Mid;
    return dmr::w4_gemm_rescale_applies(M, N) ? W4Path::GemmRescale : W4Path::Gemm;
}

// 3-bit layers: the 4-bit size classes on the native 3-bit kernels; a decode row too long for the GEMV's LDS
// budget takes the rollout-batch kernel (which slices K).  The workspace query and the forward call both go
// through this.
enum class W3Path { Gemv, Stream, Panel, Wide, Mid, Gemm, GemmRescale };
W3Path w3_path(int64_t M, int64_t K, int64_t N) {
    if (M == 1) return dmr::w3_gemv_fits(K, N) ? W3Path::Gemv : W3Path::Mid;
    if (M <= 16) {
        if (dmr::w4_stream_fits(M, K, N)) return W3Path::Stream;
        return dmr::w4_panel_applies(M, K, N) ? W3Path::Panel : W3Path::Mid;
    }
    if (M <= kSkinnyMaxM && dmr::w4_wide_applies(M, K, N)) return W3Path::Wide;
    const int64_t gemm_wgs = ((M + 127) / 128) * ((N + 127) / 128);
    if (M <= 128 || gemm_wgs < kTiledMinBlocks) return W3Path::Mid;
    return dmr::w4_gemm_rescale_applies(M, N) ? W3Path::GemmRescale : W3Path::Gemm;
}

// The bf16 twin: GEMV, the direct-from-L2 skinny kernel for 2..8 rows (measured faster there than the
// LDS-staged kernels), then the same size classes as INT4.
enum class Bf16Path { Gemv, Stream, Skinny, Mid, GemmBig, Gemm };
Bf16Path bf16_path(int64_t M, int64_t K, int64_t N) {
    if (M == 1) return Bf16Path::Gemv;
    // the streaming kernel wins (by ~12 %) only for 9..16 rows of the widest layers; below that the
    // direct-from-L2 kernel, elsewhere the rollout-batch kernel measured faster
    if (M > 8 && M <= 16 && N / dmr::kTileRows >= 1024 && dmr::bf16_stream_fits(M, K, N)) return Bf16Path::Stream;
    if (M <= 8) return Bf16Path::Skinny;
    // measured crossover: the tiled kernels win once they have more than ~128 workgroups
    const int64_t gemm_wgs = ((M + 127) / 128) * ((N + 127) / 128);
    if (M <= 64 || gemm_wgs <= 128) return Bf16Path::Mid;
    return dmr::gemm_big_applies(M, N) ? Bf16Path::GemmBig : Bf16Path::Gemm;
}

size_t align256(size_t v) { return (v + 255) & ~size_t(255); }

// Workspace of a fused forward that falls back to glue kernel + plain forward: the glue output
// (bf16 [M][K]), the fp32 result awaiting its residual ([M][N]), then the plain forward's own.
size_t fused_extra_bytes(int64_t M, int64_t K, int64_t N, int pro, bool has_res) {
    return (pro != DMR_PRO_NONE ? align256((size_t)M * (size_t)K * 2) : 0) +
           (has_res ? align256((size_t)M * (size_t)N * 4) : 0);
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

dmr_status_t check_shape(int64_t K, int64_t N, int32_t g) {
    if (K <= 0 || N <= 0 || g <= 0) return DMR_ERR_SHAPE;
    if (g != dmr::kGroup) return (K % g == 0) ? DMR_ERR_UNSUPPORTED : DMR_ERR_SHAPE;
    if (K % dmr::kGroup != 0 || N % dmr::kTileRows != 0) return DMR_ERR_SHAPE;
    // block and element indices are formed in 64 bits; the grid's x dimension is 32 bits
    if (N / dmr::kTileRows > 0x7FFFFFFF || K > (int64_t(1) << 31) || N > (int64_t(1) << 31))
        return DMR_ERR_SHAPE;
    return DMR_OK;
}

dmr_status_t hip_status(hipError_t e) { return e == hipSuccess ? DMR_OK : DMR_ERR_HIP; }

}  // namespace

extern "C" {

size_t dmr_qlinear_storage_bytes(int64_t K, int64_t N, int32_t g) {
    if (check_shape(K, N, g) != DMR_OK) return 0;
    return dmr::weight_region_bytes(K, N) + dmr::sz_region_bytes(K, N);
}

size_t dmr_qlinear_workspace_bytes(int64_t M, int64_t K, int64_t N) {
    if (M <= 0 || K <= 0 || K % dmr::kGroup != 0 || N <= 0 || N % dmr::kTileRows != 0) return 0;
    switch (w4_path(M, K, N)) {
        case W4Path::Mid: return dmr::w4_mid_workspace_bytes(M, K, N);    // fp32 partials when K is split
        case W4Path::Panel: return dmr::w4_panel_workspace_bytes(M, K, N);    // likewise
        case W4Path::Skinny2: return dmr::w4_skinny2_workspace_bytes(M, K);   // re-ordered activations
        case W4Path::GemmRescale: return dmr::w4_gemm_rescale_workspace_bytes(M, K, N);   // zero-point operands, factors
        default: return 0;
    }
}

size_t dmr_qlinear_bf16_workspace_bytes(int64_t M, int64_t K, int64_t N) {
    if (M <= 0 || K <= 0 || K % dmr::kGroup != 0 || N <= 0 || N % dmr::kTileRows != 0) return 0;
    return bf16_path(M, K, N) == Bf16Path::Mid ? dmr::bf16_mid_workspace_bytes(M, K, N) : 0;
}

dmr_status_t dmr_qlinear_create(dmr_qlinear_t **out, int64_t K, int64_t N, int32_t g,
                                const uint32_t *d_qweight, const uint16_t *d_scales,
                                const uint16_t *d_zeros, void *d_storage, size_t storage_bytes,
                                void *stream) {
    if (!out) return DMR_ERR_NULL;
    *out = nullptr;
    const dmr_status_t shape = check_shape(K, N, g);
    if (shape != DMR_OK) return shape;
    if (!d_qweight || !d_scales || !d_zeros || !d_storage) return DMR_ERR_NULL;
    if (!aligned16(d_qweight) || !aligned16(d_scales) || !aligned16(d_zeros) || !aligned16(d_storage))
        return DMR_ERR_ALIGN;
    if (storage_bytes < dmr_qlinear_storage_bytes(K, N, g)) return DMR_ERR_WORKSPACE;

    dmr_qlinear *h = new (std::nothrow) dmr_qlinear;
    if (!h) return DMR_ERR_NULL;
    h->K = K;
    h->N = N;
    h->g = g;
    h->bits = 4;
    h->szs = 1;
    h->wt3 = nullptr;
    uint8_t *base = static_cast<uint8_t *>(d_storage);
    h->wt = reinterpret_cast<const uint4 *>(base);
    h->sz = reinterpret_cast<const uint32_t *>(base + dmr::weight_region_bytes(K, N));
    const hipError_t e = dmr::launch_retile(K, N, d_qweight, d_scales, d_zeros,
                                            reinterpret_cast<uint4 *>(base),
                                            reinterpret_cast<uint32_t *>(base + dmr::weight_region_bytes(K, N)),
                                            false, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) {
        delete h;
        return DMR_ERR_HIP;
    }
    *out = h;
    return DMR_OK;
}

size_t dmr_qlinear_per_channel_storage_bytes(int64_t K, int64_t N) {
    if (check_shape(K, N, dmr::kGroup) != DMR_OK) return 0;
    return dmr::weight_region_bytes(K, N) + dmr::sz_region_bytes_per_channel(N);
}

dmr_status_t dmr_qlinear_create_per_channel(dmr_qlinear_t **out, int64_t K, int64_t N,
                                            const uint32_t *d_qweight, const uint16_t *d_scales,
                                            void *d_storage, size_t storage_bytes, void *stream) {
    if (!out) return DMR_ERR_NULL;
    *out = nullptr;
    const dmr_status_t shape = check_shape(K, N, dmr::kGroup);
    if (shape != DMR_OK) return shape;
    if (!d_qweight || !d_scales || !d_storage) return DMR_ERR_NULL;
    if (!aligned16(d_qweight) || !aligned16(d_scales) || !aligned16(d_storage)) return DMR_ERR_ALIGN;
    if (storage_bytes < dmr_qlinear_per_channel_storage_bytes(K, N)) return DMR_ERR_WORKSPACE;
    dmr_qlinear *h = new (std::nothrow) dmr_qlinear;
    if (!h) return DMR_ERR_NULL;
    h->K = K;
    h->N = N;
    h->g = (int32_t)K;      // one group spans the whole row
    h->bits = 4;
    h->szs = 0;             // one scale word per row behind the weights: 0.5 byte per weight + 4 bytes per row
    h->wt3 = nullptr;
    uint8_t *base = static_cast<uint8_t *>(d_storage);
    h->wt = reinterpret_cast<const uint4 *>(base);
    h->sz = reinterpret_cast<const uint32_t *>(base + dmr::weight_region_bytes(K, N));
    const hipError_t e = dmr::launch_retile(K, N, d_qweight, d_scales, nullptr, reinterpret_cast<uint4 *>(base),
                                            reinterpret_cast<uint32_t *>(base + dmr::weight_region_bytes(K, N)),
                                            true, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) {
        delete h;
        return DMR_ERR_HIP;
    }
    *out = h;
    return DMR_OK;
}

size_t dmr_qlinear_w3_storage_bytes(int64_t K, int64_t N, int32_t g) {
    if (check_shape(K, N, g) != DMR_OK) return 0;
    return dmr::weight3_region_bytes(K, N) + dmr::sz_region_bytes(K, N);
}

size_t dmr_qlinear_w3_workspace_bytes(int64_t M, int64_t K, int64_t N) {
    if (M <= 0 || K <= 0 || K % dmr::kGroup != 0 || N <= 0 || N % dmr::kTileRows != 0) return 0;
    switch (w3_path(M, K, N)) {
        case W3Path::Panel: return dmr::w4_panel_workspace_bytes(M, K, N);   // fp32 partials of the k slices
        case W3Path::Mid: return dmr::w4_mid_workspace_bytes(M, K, N);       // fp32 partials when K is split
        case W3Path::GemmRescale: return dmr::w4_gemm_rescale_workspace_bytes(M, K, N);   // zero-point operands, factors
        default: return 0;
    }
}

dmr_status_t dmr_qlinear_w3_create(dmr_qlinear_t **out, int64_t K, int64_t N, int32_t g,
                                   const uint32_t *d_qweight3, const uint16_t *d_scales,
                                   const uint16_t *d_zeros, void *d_storage, size_t storage_bytes,
                                   void *stream) {
    if (!out) return DMR_ERR_NULL;
    *out = nullptr;
    const dmr_status_t shape = check_shape(K, N, g);
    if (shape != DMR_OK) return shape;
    if (!d_qweight3 || !d_scales || !d_zeros || !d_storage) return DMR_ERR_NULL;
    if (!aligned16(d_qweight3) || !aligned16(d_scales) || !aligned16(d_zeros) || !aligned16(d_storage))
        return DMR_ERR_ALIGN;
    if (storage_bytes < dmr_qlinear_w3_storage_bytes(K, N, g)) return DMR_ERR_WORKSPACE;
    dmr_qlinear *h = new (std::nothrow) dmr_qlinear;
    if (!h) return DMR_ERR_NULL;
    h->K = K;
    h->N = N;
    h->g = g;
    h->bits = 3;
    h->szs = 1;
    h->wt = nullptr;
    uint8_t *base = static_cast<uint8_t *>(d_storage);
    h->wt3 = reinterpret_cast<const uint32_t *>(base);
    h->sz = reinterpret_cast<const uint32_t *>(base + dmr::weight3_region_bytes(K, N));
    const hipError_t e = dmr::launch_retile3(K, N, d_qweight3, d_scales, d_zeros,
                                             reinterpret_cast<uint32_t *>(base),
                                             reinterpret_cast<uint32_t *>(base + dmr::weight3_region_bytes(K, N)),
                                             static_cast<hipStream_t>(stream));
    if (e != hipSuccess) {
        delete h;
        return DMR_ERR_HIP;
    }
    *out = h;
    return DMR_OK;
}

dmr_status_t dmr_qlinear_quantize_w3(int64_t K, int64_t N, int32_t g, const float *d_w, uint32_t *d_qweight3,
                                     uint16_t *d_scales, uint16_t *d_zeros, void *stream) {
    const dmr_status_t shape = check_shape(K, N, g);
    if (shape != DMR_OK) return shape;
    if (!d_w || !d_qweight3 || !d_scales || !d_zeros) return DMR_ERR_NULL;
    if (!aligned16(d_w) || !aligned16(d_qweight3) || !aligned16(d_scales) || !aligned16(d_zeros))
        return DMR_ERR_ALIGN;
    return hip_status(dmr::launch_quantize3(K, N, d_w, d_qweight3, d_scales, d_zeros,
                                            static_cast<hipStream_t>(stream)));
}

dmr_status_t dmr_qlinear_dequantize(const dmr_qlinear_t *layer, uint16_t *d_w_bf16, void *stream) {
    if (!layer || !d_w_bf16) return DMR_ERR_NULL;
    if (!aligned16(d_w_bf16)) return DMR_ERR_ALIGN;
    if (layer->bits == 3) {
        const dmr::LayerView3 L3{layer->K, layer->N, layer->wt3, layer->sz};
        return hip_status(dmr::launch_dequantize3(L3, d_w_bf16, static_cast<hipStream_t>(stream)));
    }
    const dmr::LayerView L{layer->K, layer->N, layer->wt, layer->sz, layer->szs};
    return hip_status(dmr::launch_dequantize(L, d_w_bf16, static_cast<hipStream_t>(stream)));
}

dmr_status_t dmr_qlinear_forward(const dmr_qlinear_t *layer, const uint16_t *d_x, int64_t M, void *d_y,
                                 dmr_out_t out, void *d_ws, size_t ws_bytes, void *stream) {
    if (!layer) return DMR_ERR_NULL;
    if (M < 0 || M > (int64_t(1) << 22)) return DMR_ERR_SHAPE;
    if (out != DMR_OUT_BF16 && out != DMR_OUT_FP32) return DMR_ERR_UNSUPPORTED;
    if (M == 0) return DMR_OK;
    if (!d_x || !d_y) return DMR_ERR_NULL;
    if (!aligned16(d_x) || !aligned16(d_y) || (d_ws && !aligned16(d_ws))) return DMR_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool f32 = out == DMR_OUT_FP32;
    if (layer->bits == 3) {
        const dmr::LayerView3 L3{layer->K, layer->N, layer->wt3, layer->sz};
        const size_t need3 = dmr_qlinear_w3_workspace_bytes(M, layer->K, layer->N);
        if (need3 > 0 && (!d_ws || ws_bytes < need3)) return DMR_ERR_WORKSPACE;
        switch (w3_path(M, layer->K, layer->N)) {
            case W3Path::Gemv: return hip_status(dmr::launch_w3_gemv(L3, d_x, d_y, f32, s));
            case W3Path::Stream: return hip_status(dmr::launch_w3_stream(L3, d_x, M, d_y, f32, s));
            case W3Path::Panel: return hip_status(dmr::launch_w3_panel(L3, d_x, M, d_y, f32, d_ws, s));
            case W3Path::Wide: return hip_status(dmr::launch_w3_wide(L3, d_x, M, d_y, f32, s));
            case W3Path::Mid: return hip_status(dmr::launch_w3_mid(L3, d_x, M, d_y, f32, d_ws, s));
            case W3Path::Gemm: return hip_status(dmr::launch_w3_gemm(L3, d_x, M, d_y, f32, s));
            case W3Path::GemmRescale: return hip_status(dmr::launch_w3_gemm_rescale(L3, d_x, M, d_y, f32, d_ws, s));
        }
        return DMR_ERR_UNSUPPORTED;
    }
    const size_t need = dmr_qlinear_workspace_bytes(M, layer->K, layer->N);
    if (need > 0 && (!d_ws || ws_bytes < need)) return DMR_ERR_WORKSPACE;
    const dmr::LayerView L{layer->K, layer->N, layer->wt, layer->sz, layer->szs};
    const W4Path path = w4_path(M, layer->K, layer->N);
    if (path == W4Path::Gemv) {
        const hipError_t e = dmr::launch_w4_gemv(L, d_x, d_y, f32, s);
        if (e != hipErrorInvalidValue) return hip_status(e);   // else: shape outside its range
    }
    if (path == W4Path::Stream) {
        const hipError_t e = dmr::launch_w4_stream(L, d_x, M, d_y, f32, s);
        if (e != hipErrorInvalidValue) return hip_status(e);   // else: activations do not fit LDS
    }
    if (path == W4Path::Panel) return hip_status(dmr::launch_w4_panel(L, d_x, M, d_y, f32, d_ws, s));
    if (path == W4Path::Wide) return hip_status(dmr::launch_w4_wide(L, d_x, M, d_y, f32, s));
    if (path == W4Path::Mid) return hip_status(dmr::launch_w4_mid(L, d_x, M, d_y, f32, d_ws, s));
    if (path == W4Path::Skinny2) return hip_status(dmr::launch_w4_skinny2(L, d_x, M, d_y, f32, d_ws, s));
    if (M <= kSkinnyMaxM) return hip_status(dmr::launch_w4_skinny(L, d_x, M, d_y, f32, s));
    if (path == W4Path::GemmRescale) return hip_status(dmr::launch_w4_gemm_rescale(L, d_x, M, d_y, f32, d_ws, s));
    // Not reached with the present crossovers (the rescaling kernel takes every tiled shape and calls this kernel
    // itself for the column blocks it declines): 128 x 128 tiles on the exact integer codes q - z, the group's scale
    // applied to the group's partial sums in fp32.  (No tiled kernel rounds the weights to bf16 on their way into
    // LDS, what dmr_qlinear_dequantize returns: that leaves an error of about 1.7e-3 rms(y) standard deviation per
    // output, so that the largest of 10^7 .. 10^8 outputs lands at 0.8 .. 1.1 times the 1e-2 rms bound.)
    return hip_status(dmr::launch_w4_gemm(L, d_x, M, d_y, f32, s));
}

dmr_status_t dmr_qlinear_bf16_forward(const uint16_t *d_w, const uint16_t *d_x, int64_t M, int64_t K,
                                      int64_t N, void *d_y, dmr_out_t out, void *d_ws, size_t ws_bytes,
                                      void *stream) {
    const dmr_status_t shape = check_shape(K, N, dmr::kGroup);
    if (shape != DMR_OK) return shape;
    if (M < 0 || M > (int64_t(1) << 22)) return DMR_ERR_SHAPE;
    if (out != DMR_OUT_BF16 && out != DMR_OUT_FP32) return DMR_ERR_UNSUPPORTED;
    if (M == 0) return DMR_OK;
    if (!d_w || !d_x || !d_y) return DMR_ERR_NULL;
    if (!aligned16(d_w) || !aligned16(d_x) || !aligned16(d_y) || (d_ws && !aligned16(d_ws)))
        return DMR_ERR_ALIGN;
    const size_t need = dmr_qlinear_bf16_workspace_bytes(M, K, N);
    if (need > 0 && (!d_ws || ws_bytes < need)) return DMR_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool f32 = out == DMR_OUT_FP32;
    const Bf16Path path = bf16_path(M, K, N);
    if (path == Bf16Path::Gemv) {
        const hipError_t e = dmr::launch_bf16_gemv(d_w, d_x, K, N, d_y, f32, s);
        if (e != hipErrorInvalidValue) return hip_status(e);   // else: K outside its range
        return hip_status(dmr::launch_bf16_skinny(d_w, d_x, M, K, N, d_y, f32, s));
    }
    switch (path) {
        case Bf16Path::Stream: return hip_status(dmr::launch_bf16_stream(d_w, d_x, M, K, N, d_y, f32, nullptr, s));
        case Bf16Path::Skinny: return hip_status(dmr::launch_bf16_skinny(d_w, d_x, M, K, N, d_y, f32, s));
        case Bf16Path::Mid: return hip_status(dmr::launch_bf16_mid(d_w, d_x, M, K, N, d_y, f32, d_ws, s));
        case Bf16Path::GemmBig: return hip_status(dmr::launch_bf16_gemm_w8(d_w, d_x, M, K, N, d_y, f32, s));
        default: {
            // 128 x 128 tiles: the direct-to-LDS kernel while its pipeline has room to pay (K >= 1024) and the
            // grid is at most ~3 workgroups per CU (measured: 25-30 % ahead at 256 workgroups, level at 512,
            // 8 % ahead at 768, 6 % behind at 1056)
            const int64_t wgs = ((M + 127) / 128) * ((N + 127) / 128);
            if (K >= 1024 && wgs <= 800) return hip_status(dmr::launch_bf16_gemm_dma128(d_w, d_x, M, K, N, d_y, f32, s));
            return hip_status(dmr::launch_bf16_gemm(d_w, d_x, M, K, N, d_y, f32, s));
        }
    }
}

dmr_status_t dmr_glue_rmsnorm(const uint16_t *d_x, const uint16_t *d_gamma, float eps, int64_t M, int64_t K,
                              uint16_t *d_out, void *stream) {
    if (M < 0 || M > (int64_t(1) << 22) || K <= 0 || K % 8 != 0 || K > (int64_t(1) << 31)) return DMR_ERR_SHAPE;
    if (!(eps >= 0.f)) return DMR_ERR_UNSUPPORTED;
    if (M == 0) return DMR_OK;
    if (!d_x || !d_gamma || !d_out) return DMR_ERR_NULL;
    if (!aligned16(d_x) || !aligned16(d_gamma) || !aligned16(d_out)) return DMR_ERR_ALIGN;
    return hip_status(dmr::launch_rmsnorm(d_x, d_gamma, eps, M, K, d_out, static_cast<hipStream_t>(stream)));
}

dmr_status_t dmr_glue_swiglu(const uint16_t *d_in, int64_t M, int64_t I, uint16_t *d_out, void *stream) {
    if (M < 0 || M > (int64_t(1) << 22) || I <= 0 || I % 8 != 0 || I > (int64_t(1) << 30)) return DMR_ERR_SHAPE;
    if (M == 0) return DMR_OK;
    if (!d_in || !d_out) return DMR_ERR_NULL;
    if (!aligned16(d_in) || !aligned16(d_out)) return DMR_ERR_ALIGN;
    return hip_status(dmr::launch_swiglu(d_in, M, I, d_out, static_cast<hipStream_t>(stream)));
}

size_t dmr_qlinear_fused_workspace_bytes(const dmr_qlinear_t *layer, int64_t M, dmr_prologue_t pro,
                                         int32_t has_residual) {
    if (!layer || M <= 0) return 0;
    const size_t inner = layer->bits == 3 ? dmr_qlinear_w3_workspace_bytes(M, layer->K, layer->N)
                                          : dmr_qlinear_workspace_bytes(M, layer->K, layer->N);
    return fused_extra_bytes(M, layer->K, layer->N, pro, has_residual != 0) + inner;
}

size_t dmr_qlinear_bf16_fused_workspace_bytes(int64_t M, int64_t K, int64_t N, dmr_prologue_t pro,
                                              int32_t has_residual) {
    if (M <= 0 || K <= 0 || N <= 0) return 0;
    return fused_extra_bytes(M, K, N, pro, has_residual != 0) + dmr_qlinear_bf16_workspace_bytes(M, K, N);
}

}  // extern "C"

namespace {

// Argument checks shared by the two fused forwards; DMR_OK means "go on".
dmr_status_t check_fused(dmr_prologue_t pro, const uint16_t *d_in, const uint16_t *d_gamma, float eps,
                         const uint16_t *d_residual, int64_t M, const void *d_y, dmr_out_t out, const void *d_ws) {
    if (M < 0 || M > (int64_t(1) << 22)) return DMR_ERR_SHAPE;
    if (out != DMR_OUT_BF16 && out != DMR_OUT_FP32) return DMR_ERR_UNSUPPORTED;
    if (pro != DMR_PRO_NONE && pro != DMR_PRO_RMSNORM && pro != DMR_PRO_SWIGLU) return DMR_ERR_UNSUPPORTED;
    if (pro == DMR_PRO_RMSNORM && !(eps >= 0.f)) return DMR_ERR_UNSUPPORTED;
    if (M == 0) return DMR_OK;
    if (!d_in || !d_y || (pro == DMR_PRO_RMSNORM && !d_gamma)) return DMR_ERR_NULL;
    if (!aligned16(d_in) || !aligned16(d_y) || (d_gamma && !aligned16(d_gamma)) ||
        (d_residual && !aligned16(d_residual)) || (d_ws && !aligned16(d_ws)))
        return DMR_ERR_ALIGN;
    return DMR_OK;
}

// The unfused composition: glue kernel into the workspace, plain forward (fp32 if a residual
// follows), residual add.  `forward` runs the plain forward on (x, y, out type, inner workspace).
template <typename Forward>
dmr_status_t run_unfused(dmr_prologue_t pro, const uint16_t *d_in, const uint16_t *d_gamma, float eps,
                         const uint16_t *d_residual, int64_t M, int64_t K, int64_t N, void *d_y, dmr_out_t out,
                         void *d_ws, size_t ws_bytes, hipStream_t s, Forward forward) {
    uint8_t *ws = static_cast<uint8_t *>(d_ws);
    size_t used = 0;
    const uint16_t *x = d_in;
    if (pro != DMR_PRO_NONE) {
        uint16_t *xg = reinterpret_cast<uint16_t *>(ws);
        used += align256((size_t)M * (size_t)K * 2);
        const hipError_t e = pro == DMR_PRO_RMSNORM ? dmr::launch_rmsnorm(d_in, d_gamma, eps, M, K, xg, s)
                                                     : dmr::launch_swiglu(d_in, M, K, xg, s);
        if (e != hipSuccess) return DMR_ERR_HIP;
        x = xg;
    }
    if (!d_residual) return forward(x, d_y, out, ws + used, ws_bytes - used);
    float *acc = reinterpret_cast<float *>(ws + used);
    used += align256((size_t)M * (size_t)N * 4);
    const dmr_status_t st = forward(x, acc, DMR_OUT_FP32, ws + used, ws_bytes - used);
    if (st != DMR_OK) return st;
    return hip_status(dmr::launch_add_residual(acc, d_residual, M * N, d_y, out == DMR_OUT_FP32, s));
}

}  // namespace

extern "C" {

dmr_status_t dmr_qlinear_forward_fused(const dmr_qlinear_t *layer, dmr_prologue_t pro, const uint16_t *d_in,
                                       const uint16_t *d_gamma, float eps, const uint16_t *d_residual, int64_t M,
                                       void *d_y, dmr_out_t out, void *d_ws, size_t ws_bytes, void *stream) {
    if (!layer) return DMR_ERR_NULL;
    const dmr_status_t chk = check_fused(pro, d_in, d_gamma, eps, d_residual, M, d_y, out, d_ws);
    if (chk != DMR_OK || M == 0) return chk;
    const size_t need = dmr_qlinear_fused_workspace_bytes(layer, M, pro, d_residual != nullptr);
    if (need > 0 && (!d_ws || ws_bytes < need)) return DMR_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (M == 1 && layer->bits == 4) {
        const dmr::LayerView L{layer->K, layer->N, layer->wt, layer->sz, layer->szs};
        dmr::Fusion f;
        f.pro = (int)pro;
        f.aux = d_gamma;
        f.eps = eps;
        f.res = d_residual;
        const hipError_t e = dmr::launch_w4_gemv_fused(L, d_in, d_y, out == DMR_OUT_FP32, f, s);
        if (e != hipErrorInvalidValue) return hip_status(e);   // else: shape outside the GEMV's range
    }
    if (M >= 2 && M <= 16 && layer->bits == 4 && dmr::w4_stream_fits(M, layer->K, layer->N)) {
        const dmr::LayerView L{layer->K, layer->N, layer->wt, layer->sz, layer->szs};
        dmr::Fusion f;
        f.pro = (int)pro;
        f.aux = d_gamma;
        f.eps = eps;
        f.res = d_residual;
        const uint16_t *x = d_in;
        // In this kernel every workgroup would recompute the prologue for all M rows, which measured
        // slower than one launch of the stand-alone kernel: the prologue runs on its own, the residual
        // stays fused.
        if (pro != DMR_PRO_NONE) {
            uint16_t *xg = static_cast<uint16_t *>(d_ws);
            const hipError_t eg = pro == DMR_PRO_RMSNORM ? dmr::launch_rmsnorm(d_in, d_gamma, eps, M, layer->K, xg, s)
                                                          : dmr::launch_swiglu(d_in, M, layer->K, xg, s);
            if (eg != hipSuccess) return DMR_ERR_HIP;
            x = xg;
            f.pro = dmr::kProNone;
        }
        const hipError_t e = dmr::launch_w4_stream_fused(L, x, M, d_y, out == DMR_OUT_FP32, f, s);
        if (e != hipErrorInvalidValue) return hip_status(e);
    }
    return run_unfused(pro, d_in, d_gamma, eps, d_residual, M, layer->K, layer->N, d_y, out, d_ws, ws_bytes, s,
                       [&](const uint16_t *x, void *y, dmr_out_t o, void *ws, size_t wsb) {
                           return dmr_qlinear_forward(layer, x, M, y, o, ws, wsb, stream);
                       });
}

dmr_status_t dmr_qlinear_bf16_forward_fused(const uint16_t *d_w, dmr_prologue_t pro, const uint16_t *d_in,
                                            const uint16_t *d_gamma, float eps, const uint16_t *d_residual,
                                            int64_t M, int64_t K, int64_t N, void *d_y, dmr_out_t out, void *d_ws,
                                            size_t ws_bytes, void *stream) {
    const dmr_status_t shape = check_shape(K, N, dmr::kGroup);
    if (shape != DMR_OK) return shape;
    const dmr_status_t chk = check_fused(pro, d_in, d_gamma, eps, d_residual, M, d_y, out, d_ws);
    if (chk != DMR_OK || M == 0) return chk;
    if (!d_w) return DMR_ERR_NULL;
    if (!aligned16(d_w)) return DMR_ERR_ALIGN;
    const size_t need = dmr_qlinear_bf16_fused_workspace_bytes(M, K, N, pro, d_residual != nullptr);
    if (need > 0 && (!d_ws || ws_bytes < need)) return DMR_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (M == 1) {
        dmr::Fusion f;
        f.pro = (int)pro;
        f.aux = d_gamma;
        f.eps = eps;
        f.res = d_residual;
        const hipError_t e = dmr::launch_bf16_gemv_fused(d_w, d_in, K, N, d_y, out == DMR_OUT_FP32, f, s);
        if (e != hipErrorInvalidValue) return hip_status(e);   // else: K outside its range, or RMSNorm over slices
    }
    if (bf16_path(M, K, N) == Bf16Path::Stream) {
        // as in the INT4 kernel of this size class: stand-alone prologue, residual fused at the store
        const uint16_t *x = d_in;
        if (pro != DMR_PRO_NONE) {
            uint16_t *xg = static_cast<uint16_t *>(d_ws);
            const hipError_t eg = pro == DMR_PRO_RMSNORM ? dmr::launch_rmsnorm(d_in, d_gamma, eps, M, K, xg, s)
                                                          : dmr::launch_swiglu(d_in, M, K, xg, s);
            if (eg != hipSuccess) return DMR_ERR_HIP;
            x = xg;
        }
        const hipError_t e = dmr::launch_bf16_stream(d_w, x, M, K, N, d_y, out == DMR_OUT_FP32, d_residual, s);
        if (e != hipErrorInvalidValue) return hip_status(e);
    }
    return run_unfused(pro, d_in, d_gamma, eps, d_residual, M, K, N, d_y, out, d_ws, ws_bytes, s,
                       [&](const uint16_t *x, void *y, dmr_out_t o, void *ws, size_t wsb) {
                           return dmr_qlinear_bf16_forward(d_w, x, M, K, N, y, o, ws, wsb, stream);
                       });
}

dmr_status_t dmr_qlinear_quantize(int64_t K, int64_t N, int32_t g, const float *d_w, uint32_t *d_qweight,
                                  uint16_t *d_scales, uint16_t *d_zeros, void *stream) {
    const dmr_status_t shape = check_shape(K, N, g);
    if (shape != DMR_OK) return shape;
    if (!d_w || !d_qweight || !d_scales || !d_zeros) return DMR_ERR_NULL;
    if (!aligned16(d_w) || !aligned16(d_qweight) || !aligned16(d_scales) || !aligned16(d_zeros))
        return DMR_ERR_ALIGN;
    return hip_status(dmr::launch_quantize(K, N, d_w, d_qweight, d_scales, d_zeros,
                                           static_cast<hipStream_t>(stream)));
}

dmr_status_t dmr_probe_hbm_read(const void *d_buf, size_t bytes, uint32_t *d_sink, int32_t blocks,
                                void *stream) {
    if (!d_buf || !d_sink) return DMR_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0 || blocks <= 0 || blocks > (1 << 20)) return DMR_ERR_SHAPE;
    if (!aligned16(d_buf) || !aligned16(d_sink)) return DMR_ERR_ALIGN;
    return hip_status(dmr::launch_hbm_read_probe(d_buf, bytes, d_sink, blocks, static_cast<hipStream_t>(stream)));
}

const char *dmr_qlinear_kernel_path(dmr_format_t format, int64_t M, int64_t K, int64_t N) {
    if (M <= 0 || check_shape(K, N, dmr::kGroup) != DMR_OK) return "none";
    auto bf16_name = [&]() -> const char * {
        switch (bf16_path(M, K, N)) {
            case Bf16Path::Gemv: return dmr::bf16_gemv_fits(K) ? "bf16_gemv" : "bf16_skinny";
            case Bf16Path::Stream: return "bf16_stream";
            case Bf16Path::Skinny: return "bf16_skinny";
            case Bf16Path::Mid: return "bf16_mid";
            case Bf16Path::GemmBig: return "bf16_gemm256";
            default: {
                const int64_t wgs = ((M + 127) / 128) * ((N + 127) / 128);
                return (K >= 1024 && wgs <= 800) ? "bf16_gemm128_dma" : "bf16_gemm128";
            }
        }
    };
    switch (format) {
        case DMR_FMT_BF16: return bf16_name();
        case DMR_FMT_W3_G128:
            switch (w3_path(M, K, N)) {
                case W3Path::Gemv: return "w3_gemv";
                case W3Path::Stream: return "w3_stream";
                case W3Path::Panel: return "w3_panel";
                case W3Path::Wide: return "w3_wide";
                case W3Path::Mid: return "w3_mid";
                case W3Path::GemmRescale:
                    if (dmr::w4_gemm_rescale_tile_rows(M, N) == 128) return "w3_gemm128_rescale";
                    return dmr::w4_gemm_rescale_wave_columns(M, N) == 4 ? "w3_gemm256_rescale" : "w3_gemm256x128_rescale";
                default: return "w3_gemm128_exact";
            }
        case DMR_FMT_W4_G128:
        case DMR_FMT_W4_PER_CHANNEL:
            switch (w4_path(M, K, N)) {
                case W4Path::Gemv: return dmr::w4_gemv_fits(K, N, false) ? "w4_gemv" : "w4_skinny";
                case W4Path::Stream: return "w4_stream";
                case W4Path::Panel: return "w4_panel";
                case W4Path::Wide: return "w4_wide";
                case W4Path::Skinny2: return "w4_skinny2";
                case W4Path::Mid: return "w4_mid";
                case W4Path::GemmRescale:
                    if (dmr::w4_gemm_rescale_tile_rows(M, N) == 128) return "w4_gemm128_rescale";
                    return dmr::w4_gemm_rescale_wave_columns(M, N) == 4 ? "w4_gemm256_rescale" : "w4_gemm256x128_rescale";
                default: return "w4_gemm128_exact";
            }
    }
    return "none";
}

dmr_status_t dmr_probe_empty_launch(int32_t blocks, int32_t threads, size_t lds_bytes, void *stream) {
    if (blocks <= 0 || blocks > (1 << 20) || threads <= 0 || threads > 1024 || threads % 64 != 0 ||
        lds_bytes > 64 * 1024)
        return DMR_ERR_SHAPE;
    return hip_status(dmr::launch_empty_probe(blocks, threads, lds_bytes, static_cast<hipStream_t>(stream)));
}

void dmr_qlinear_destroy(dmr_qlinear_t *layer) { delete layer; }

int32_t dmr_qlinear_bits(const dmr_qlinear_t *layer) { return layer ? layer->bits : 0; }

dmr_status_t dmr_qlinear_shape(const dmr_qlinear_t *layer, int64_t *K, int64_t *N, int32_t *g) {
    if (!layer) return DMR_ERR_NULL;
    if (K) *K = layer->K;
    if (N) *N = layer->N;
    if (g) *g = layer->g;
    return DMR_OK;
}

const char *dmr_status_string(dmr_status_t status) {
    switch (status) {
        case DMR_OK: return "ok";
        case DMR_ERR_NULL: return "a required pointer is NULL";
        case DMR_ERR_SHAPE: return "bad shape";
        case DMR_ERR_ALIGN: return "device pointer not 16-byte aligned";
        case DMR_ERR_WORKSPACE: return "storage or workspace buffer too small";
        case DMR_ERR_UNSUPPORTED: return "unsupported configuration";
        case DMR_ERR_HIP: return "HIP launch failed";
    }
    return "unknown status";
}

}  // extern "C"

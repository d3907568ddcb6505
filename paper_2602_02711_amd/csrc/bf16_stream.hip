// bf16 twin of the W4A16 streaming kernel for 2 <= M <= 16: the same skeleton (S k slices x TW tiles of
// wavefronts per workgroup, all M activation rows staged in LDS with rows padded by 16 bytes, a
// register ring of P outstanding weight items per wave, the cross-slice sum at every tile step through
// one reused LDS buffer, every wave running the same number of item slots and barriers), so that the
// two copies of a routed step are compared like for like.  An item is the 16 rows x 128 k of one
// (tile, group): lane (c, j) loads row 16 T + j of the row-major weight matrix, for MFMA t of the
// group the 8 values k = 128 g + 32 t + 8 c .. + 7 (one 16-byte load; the four lanes c of a row cover
// 64 contiguous bytes per instruction), 4 KiB per wave and item; the A operand is read from LDS with
// the same k mapping and the MFMAs accumulate straight into the output tile.
// Of the decoder glue only the residual add is fused (at the store), as in the INT4 kernel.
#include <cstdlib>

#include "glue.hpp"

namespace dmr {

namespace {

struct Item {
    u32x4_t w[4];
};

// Copy `total` 16-byte pieces of x into LDS, piece p to slot p + p / x16 (rows padded by one piece; the
// division by multiplication with ceil(2^32 / x16)), B loads in flight per thread.  (Plain vector
// type for the staging registers: an array of HIP's uint4 struct ends up in scratch memory.)
template <int B>
__device__ __forceinline__ void stage_rows(const uint16_t *__restrict__ x, uint4 *smem, int total,
                                           uint32_t x16_magic, int first) {
    const int T = (int)blockDim.x;
    for (int base = first + (int)threadIdx.x; base < total; base += B * T) {
        u32x4_t v[B];
#pragma unroll
        for (int u = 0; u < B; ++u)
            v[u] = reinterpret_cast<const u32x4_t *>(x)[min(base + u * T, total - 1)];
#pragma unroll
        for (int u = 0; u < B; ++u) {
            const int p = base + u * T;
            if (p < total) reinterpret_cast<u32x4_t *>(smem)[p + (int)__umulhi((uint32_t)p, x16_magic)] = v[u];
        }
    }
}

template <int P>
__global__ __launch_bounds__(1024) void bf16_stream_kernel(const uint16_t *__restrict__ w,
                                                           const uint16_t *__restrict__ x,
                                                           void *__restrict__ y, int M, int64_t K, int64_t N,
                                                           int groups, int tiles, int lgS, int lgTW,
                                                           int nT_max, int gw_max, int out_f32,
                                                           const uint16_t *__restrict__ res, uint32_t x16_magic) {
    extern __shared__ uint4 smem[];   // x rows [M][groups * 16 + 1] uint4, then red[TW][S][64] float4
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int S = 1 << lgS, TW = 1 << lgTW;
    const int s = wave & (S - 1), tw = wave >> lgS;
    const int c = lane >> 4, j = lane & 15;
    const int g0 = (groups * s) >> lgS;
    const int GW = ((groups * (s + 1)) >> lgS) - g0;          // 0 <= GW <= gw_max
    const int t_first = ((int)blockIdx.x << lgTW) + tw;
    const int t_step = (int)gridDim.x << lgTW;
    const int slots = nT_max * gw_max;                          // the same for every wave
    const int x16 = groups * 16, row_stride = x16 + 1;

    // Slot (step, gi) -> block to load, clamped into this wave's valid range (or to the matrix's last
    // tile if it owns none): every load is unconditional and in bounds.
    // The first pieces of the activation rows are requested before the weight ring: memory operations of a
    // wave return in order, so behind the ring they would arrive only after its HBM latency.
    constexpr int B0 = 8;
    const int total = M * x16, T = (int)blockDim.x;
    u32x4_t x0[B0];
#pragma unroll
    for (int u = 0; u < B0; ++u)
        if (u * T < total)            // uniform
            x0[u] = reinterpret_cast<const u32x4_t *>(x)[min((int)threadIdx.x + u * T, total - 1)];

    int is = 0, ig = 0;   // issue pointer
    Item ring[P];
    auto issue = [&](Item &dst) {
        int tile = t_first + is * t_step;
        tile = tile < tiles ? tile : tiles - 1;
        int g = g0 + (ig < GW ? ig : GW - 1);
        g = g < 0 ? 0 : (g < groups ? g : groups - 1);
        const uint16_t *src = w + ((int64_t)tile * kTileRows + j) * K + g * kGroup + c * 8;
#pragma unroll
        for (int t = 0; t < 4; ++t)
            dst.w[t] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(src + t * 32));
        if (++ig == gw_max) {
            ig = 0;
            if (is + 1 < nT_max) ++is;      // saturate at the last step
        }
    };
#pragma unroll
    for (int p = 0; p < P; ++p) issue(ring[p]);

    // Stage the M activation rows: x is one contiguous run of M * x16 pieces; piece p of row
    // r = p / x16 (by multiplication with ceil(2^32 / x16), exact in this range) lands at p + r because
    // rows are padded by one piece.  The first eight pieces per thread are in registers already; the rest
    // follows in batches of eight loads before the first store, so that a thread pays the memory latency
    // once per batch and not once per piece.
#pragma unroll
    for (int u = 0; u < B0; ++u) {
        const int p = (int)threadIdx.x + u * T;
        if (p < total) reinterpret_cast<u32x4_t *>(smem)[p + (int)__umulhi((uint32_t)p, x16_magic)] = x0[u];
    }
    if (total > B0 * T) stage_rows<8>(x, smem, total, x16_magic, B0 * T);
    __syncthreads();
    auto store_out = [&](int64_t o, float v) {
        if (res) v += __uint_as_float((uint32_t)res[o] << 16);
        if (out_f32)
            reinterpret_cast<float *>(y)[o] = v;
        else
            reinterpret_cast<uint16_t *>(y)[o] = f32_to_bf16(v);
    };

    float *red = reinterpret_cast<float *>(smem + M * row_stride);
    const uint4 *xrow = smem + (j < M ? j : M - 1) * row_stride + c;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    int cs = 0, cg = 0;   // consume pointer: (tile step, slot within step)

    auto consume = [&](const Item &cur) {
        const int tile = t_first + cs * t_step;
        if (cg < GW && tile < tiles) {
            const uint4 *xp = xrow + (g0 + cg) * 16;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                Frag a;
                a.u = xp[4 * t];
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, __builtin_bit_cast(bf16x8, cur.w[t]), acc, 0, 0, 0);
            }
        }
        if (++cg == gw_max) {
            // tile step finished: every wave arrives here exactly once per step
            if (lgS == 0) {
                // one slice: the wave owns the whole k range, its tile goes straight to memory
                if (tile < tiles) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int row = (lane >> 4) * 4 + r;
                        if (row < M) store_out((int64_t)row * N + (int64_t)tile * kTileRows + (lane & 15), acc[r]);
                    }
                }
            } else {
                reinterpret_cast<f32x4 *>(red)[((tw << lgS) + s) * 64 + lane] = acc;
                __syncthreads();
                // wave w2 < TW adds the S partial tiles of tile lane w2 in slice order
                if (wave < TW) {
                    const f32x4 *part = reinterpret_cast<const f32x4 *>(red) + ((wave << lgS) * 64 + lane);
                    f32x4 v = part[0];
                    for (int q = 1; q < S; ++q) {
                        const f32x4 u = part[q * 64];
#pragma unroll
                        for (int r = 0; r < 4; ++r) v[r] += u[r];
                    }
                    const int t2 = ((int)blockIdx.x << lgTW) + wave + cs * t_step;
                    if (t2 < tiles) {
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int row = (lane >> 4) * 4 + r;
                            if (row < M) store_out((int64_t)row * N + (int64_t)t2 * kTileRows + (lane & 15), v[r]);
                        }
                    }
                }
                __syncthreads();
            }
            acc = f32x4{0.f, 0.f, 0.f, 0.f};
            cg = 0;
            ++cs;
        }
    };

    int base = 0;
    for (; base + P < slots; base += P) {
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const Item cur = ring[p];
            issue(ring[p]);
            consume(cur);
        }
    }
#pragma unroll
    for (int p = 0; p < P; ++p)
        if (base + p < slots) consume(ring[p]);
}

}  // namespace

// Whether the M activation rows (plus the reduction buffer of the default launch shape on 256 CUs)
// fit the 160 KB of LDS; pure host arithmetic.
bool bf16_stream_fits(int64_t M, int64_t K, int64_t N) {
    if (M < 2 || M > 16) return false;
    (void)N;
    const int groups = (int)(K / kGroup);
    const size_t xbytes = (size_t)M * (groups * 16 + 1) * sizeof(uint4);
    int nw = 16, S = 16;
    while (S > groups) S >>= 1;
    return xbytes + (S > 1 ? (size_t)nw * 64 * sizeof(f32x4) : 0) <= 160 * 1024;
}

hipError_t launch_bf16_stream(const uint16_t *w, const uint16_t *x, int64_t M, int64_t K, int64_t N, void *y,
                              bool out_f32, const uint16_t *res, hipStream_t stream) {
    if (!bf16_stream_fits(M, K, N)) return hipErrorInvalidValue;
    const int groups = (int)(K / kGroup);
    const int tiles = (int)(N / kTileRows);
    const int cus = compute_units();
    // Measured on MI355X (sweep over waves, k slices and ring depth at M = 4 and 16 on the four decoder
    // shapes): unlike the INT4 kernel, whose blocks are contiguous, the row-major weights want all 16
    // waves of a workgroup along k on the same 16 rows (whole rows stream at a time) and only two items
    // in flight per wave; overridable for sweeps.
    const size_t xbytes = (size_t)M * (groups * 16 + 1) * sizeof(uint4);
    int nw = 16, S = 16;
    nw = env_int("DMR_BSTREAM_NW", nw);
    S = env_int("DMR_BSTREAM_S", S);
    if (nw < 1 || nw > 16 || S < 1 || S > nw || (nw & (nw - 1)) || (S & (S - 1))) return hipErrorInvalidValue;
    while (S > groups) S >>= 1;
    const int TW = nw / S;
    const size_t lds = xbytes + (S > 1 ? (size_t)nw * 64 * sizeof(f32x4) : 0);
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    int per_cu = (int)((160 * 1024) / lds);
    if (per_cu > 16 / nw) per_cu = 16 / nw;
    const int wgs = (tiles + TW - 1) / TW;
    int grid = wgs < per_cu * cus ? wgs : per_cu * cus;
    grid = env_int("DMR_BSTREAM_GRID", grid);
    if (grid < 1) return hipErrorInvalidValue;
    int lgS = 0, lgTW = 0;
    while ((1 << lgS) < S) ++lgS;
    while ((1 << lgTW) < TW) ++lgTW;
    const int t_step = grid * TW;
    const int nT_max = (tiles + t_step - 1) / t_step;
    const int gw_max = (groups + S - 1) / S;
    const int slots = nT_max * gw_max;
    int P = env_int("DMR_BSTREAM_P", 2);
    if (P > slots) P = slots;
    const int of = out_f32 ? 1 : 0;
    const int iM = (int)M;
    const uint32_t x16_magic = (uint32_t)(((uint64_t(1) << 32) + (uint64_t)groups * 16 - 1) / ((uint64_t)groups * 16));
#define DMR_BSTREAM_CASE(PP)                                                                              \
    case PP: {                                                                                            \
        static const hipError_t attr_status = hipFuncSetAttribute(reinterpret_cast<const void *>(&bf16_stream_kernel<PP>), \
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024); \
        if (attr_status != hipSuccess) return attr_status; \
        hipLaunchKernelGGL((bf16_stream_kernel<PP>), dim3(grid), dim3(nw * 64), lds, stream, w, x, y, iM, K, N, \
                           groups, tiles, lgS, lgTW, nT_max, gw_max, of, res, x16_magic);                 \
    } break;
    switch (P) {
        DMR_BSTREAM_CASE(1) DMR_BSTREAM_CASE(2) DMR_BSTREAM_CASE(3)     // 4 items exceed the 128 registers of 16 waves
        default: return hipErrorInvalidValue;
    }
#undef DMR_BSTREAM_CASE
    return hipGetLastError();
}

}  // namespace dmr

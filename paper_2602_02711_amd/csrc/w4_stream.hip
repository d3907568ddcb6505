// W4A16 streaming kernel for 2 <= M <= 16: a small group of parallel rollouts each taking one
// low-precision step.  Same structure as the M == 1 GEMV (S k slices x TW tiles of wavefronts per
// workgroup, a register ring of P outstanding 1 KiB block loads per wave, nibble -> bf16 unpack,
// 16x16x32 MFMAs, group-wise zero point and scale), with three differences:
//   - all M activation rows are staged in LDS (row stride padded by 16 bytes so that the 16
//     operand rows of a wave fall in distinct banks); lanes of rows >= M re-read row M - 1 and
//     their results are never stored;
//   - the accumulator is the whole 16 x 16 MFMA tile (4 registers per lane);
//   - the cross-slice sum happens at every tile step through one reused LDS buffer, bracketed by
//     two barriers.  Every wave executes the same nT_max * GW_max item slots and therefore the same
//     number of barriers whatever its share of the work: slots beyond a wave's work re-read its last
//     block from cache and skip the arithmetic.
// Of the decoder glue (glue.hpp) only the residual add is fused here (at the store).  A prologue
// would be recomputed for all M rows by every workgroup, which measured slower than one launch of the
// stand-alone RMSNorm / SwiGLU kernel from two rows on.
#include <cstdlib>

#include "glue.hpp"

namespace dmr {

namespace {

constexpr uint32_t kOnes = 0x3F803F80u;    // bf16 pair (1.0, 1.0)

struct Item {
    uint4 w;
    uint32_t szw;
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

template <int P, bool XS>
__global__ __launch_bounds__(1024) void w4_stream_kernel(const uint4 *__restrict__ wt,
                                                         const uint32_t *__restrict__ sz,
                                                         const uint16_t *__restrict__ x,
                                                         void *__restrict__ y, int M, int64_t N,
                                                         int groups, int tiles, int lgS, int lgTW,
                                                         int nT_max, int gw_max, int out_f32,
                                                         const uint16_t *__restrict__ res, uint32_t x16_magic, int szs) {
    extern __shared__ uint4 smem[];   // x rows [M][groups * 16 + 1] uint4, xs[groups][4] float4, red[TW][S][64] float4
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
        const int64_t block = (int64_t)tile * groups + g;
        dst.w = load_stream(wt + block * 64 + lane);
        dst.szw = load_stream(sz + sz_index(tile, g, groups, szs, j));
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
    // XS: the group sums of x (every column of A . ones holds the row sums) are formed once per workgroup
    // into a table instead of by four more MFMAs per block; pays when a wave streams many blocks
    f32x4 *xs = reinterpret_cast<f32x4 *>(smem + M * row_stride);
    if constexpr (XS) {
        Frag ones1;
        ones1.u = make_uint4(kOnes, kOnes, kOnes, kOnes);
        const uint4 *xr = smem + (j < M ? j : M - 1) * row_stride + c * 4;
        for (int u = wave; u < groups; u += (int)(blockDim.x >> 6)) {
            f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                Frag a;
                a.u = xr[u * 16 + t];
                d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, ones1.v, d, 0, 0, 0);
            }
            if (j == 0) xs[u * 4 + c] = d;
        }
        __syncthreads();
    }
    auto store_out = [&](int64_t o, float v) {
        if (res) v += __uint_as_float((uint32_t)res[o] << 16);
        if (out_f32)
            reinterpret_cast<float *>(y)[o] = v;
        else
            reinterpret_cast<uint16_t *>(y)[o] = f32_to_bf16(v);
    };

    float *red = reinterpret_cast<float *>(smem + M * row_stride + groups * 4);
    const uint4 *xrow = smem + (j < M ? j : M - 1) * row_stride + c * 4;
    Frag ones;
    ones.u = make_uint4(kOnes, kOnes, kOnes, kOnes);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    int cs = 0, cg = 0;   // consume pointer: (tile step, slot within step)

    auto consume = [&](const Item &cur) {
        const int tile = t_first + cs * t_step;
        if (cg < GW && tile < tiles) {
            const uint4 *xp = xrow + (g0 + cg) * 16;
            Frag a[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) a[t].u = xp[t];
            const uint32_t words[4] = {cur.w.x, cur.w.y, cur.w.z, cur.w.w};
            f32x4 d = {0.f, 0.f, 0.f, 0.f}, xsum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                Frag b;
                unpack_word(words[t], b.w);
                d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[t].v, b.v, d, 0, 0, 0);
                if constexpr (!XS) xsum = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[t].v, ones.v, xsum, 0, 0, 0);
            }
            if constexpr (XS) xsum = xs[(g0 + cg) * 4 + c];
            const float sc = __uint_as_float(cur.szw << 16);
            const float cz = __uint_as_float(cur.szw & 0xFFFF0000u);   // -(128 + z)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[r] = fmaf(sc, fmaf(cz, xsum[r], d[r]), acc[r]);
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
// fit the 160 KB of LDS; pure host arithmetic, so that the caller can plan its workspace.
bool w4_stream_fits(int64_t M, int64_t K, int64_t N) {
    if (M < 2 || M > 16) return false;
    const int groups = (int)(K / kGroup), tiles = (int)(N / kTileRows);
    const size_t xbytes = (size_t)M * (groups * 16 + 1) * sizeof(uint4) + (size_t)groups * 4 * sizeof(f32x4);
    int nw = 16, S = 16;
    if (tiles >= 4 * kCus) {
        nw = 8;
        S = 2;
    } else if (tiles > kCus) {
        nw = 8;
        S = 4;
    }
    while (S > groups) S >>= 1;
    return xbytes + (S > 1 ? (size_t)nw * 64 * sizeof(f32x4) : 0) <= 160 * 1024;
}

hipError_t launch_w4_stream(const LayerView &L, const uint16_t *x, int64_t M, void *y, bool out_f32,
                            hipStream_t stream) {
    return launch_w4_stream_fused(L, x, M, y, out_f32, Fusion{}, stream);
}

hipError_t launch_w4_stream_fused(const LayerView &L, const uint16_t *x, int64_t M, void *y, bool out_f32,
                                  const Fusion &f, hipStream_t stream) {
    if (M < 2 || M > 16 || f.pro != kProNone) return hipErrorInvalidValue;
    const int groups = (int)(L.K / kGroup);
    const int tiles = (int)(L.N / kTileRows);
    const int cus = compute_units();
    // Choose (waves per workgroup, k slices S, tile lanes TW = waves / S).  The activations' LDS
    // footprint limits how many workgroups a CU holds.
    const size_t xbytes = (size_t)M * (groups * 16 + 1) * sizeof(uint4) + (size_t)groups * 4 * sizeof(f32x4);
    // Measured on MI355X (sweep over waves per workgroup, S, ring depth at M = 2..16): few, long k
    // slices win once there are several tiles per CU; one tile per CU wants all 16 slices.
    int best_nw, best_S;
    if (tiles >= 4 * cus) {
        best_nw = 8;
        best_S = 2;
    } else if (tiles > cus) {
        best_nw = 8;
        best_S = 4;
    } else {
        best_nw = 16;
        best_S = 16;
    }
    while (best_S > groups) best_S >>= 1;
    int best_grid = 0;
    {
        const int TWc = best_nw / best_S;
        const size_t lds_c = xbytes + (best_S > 1 ? (size_t)best_nw * 64 * sizeof(f32x4) : 0);
        if (lds_c > 160 * 1024) {
            best_nw = 0;
        } else {
            int per_cu = (int)((160 * 1024) / lds_c);
            if (per_cu > 16 / best_nw) per_cu = 16 / best_nw;
            const int wgs = (tiles + TWc - 1) / TWc;
            best_grid = wgs < per_cu * cus ? wgs : per_cu * cus;
        }
    }
    if (best_nw == 0) return hipErrorInvalidValue;   // activations do not fit LDS: general kernel
    // sweep overrides (unset in production)
    const int nw = env_int("DMR_STREAM_NW", best_nw), S = env_int("DMR_STREAM_S", best_S);
    if (nw < 1 || nw > 16 || S < 1 || S > nw || S > groups || (nw & (nw - 1)) || (S & (S - 1)))
        return hipErrorInvalidValue;
    const int TW = nw / S;
    int grid = best_grid;
    if (nw != best_nw || S != best_S) {
        const size_t lds_o = xbytes + (S > 1 ? (size_t)nw * 64 * sizeof(f32x4) : 0);
        if (lds_o > 160 * 1024) return hipErrorInvalidValue;
        int per_cu = (int)((160 * 1024) / lds_o);
        if (per_cu > 16 / nw) per_cu = 16 / nw;
        const int wgs = (tiles + TW - 1) / TW;
        grid = wgs < per_cu * cus ? wgs : per_cu * cus;
    }
    grid = env_int("DMR_STREAM_GRID", grid);
    if (grid < 1) return hipErrorInvalidValue;
    int lgS = 0, lgTW = 0;
    while ((1 << lgS) < S) ++lgS;
    while ((1 << lgTW) < TW) ++lgTW;
    const int t_step = grid * TW;
    const int nT_max = (tiles + t_step - 1) / t_step;
    const int gw_max = (groups + S - 1) / S;
    const size_t lds = xbytes + (S > 1 ? (size_t)nw * 64 * sizeof(f32x4) : 0);
    const int slots = nT_max * gw_max;
    int P = slots < 4 ? slots : 4;
    P = env_int("DMR_STREAM_P", P);
    if (P > slots) P = slots;
    const int of = out_f32 ? 1 : 0;
    const int iM = (int)M;
    const uint32_t x16_magic = (uint32_t)(((uint64_t(1) << 32) + (uint64_t)groups * 16 - 1) / ((uint64_t)groups * 16));
#define DMR_STREAM_CASE(PP)                                                                             \
    case PP: {                                                                                          \
        static const hipError_t attr_status = hipFuncSetAttribute(reinterpret_cast<const void *>(&w4_stream_kernel<PP, false>), \
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024); \
        if (attr_status != hipSuccess) return attr_status; \
        hipLaunchKernelGGL((w4_stream_kernel<PP, false>), dim3(grid), dim3(nw * 64), lds, stream, L.wt, L.sz, x, y, \
                           iM, L.N, groups, tiles, lgS, lgTW, nT_max, gw_max, of, f.res, x16_magic, L.szs);   \
    } break;
    // Group sums from a table when a wave streams at least sixteen blocks and the table costs it at most
    // a quarter as many MFMA passes as it saves (the widest layers: 0.3-0.9 us of 17 on gate+up; on the
    // 6144-row layer, eight blocks per wave, it measured 0.3 us slower).
    const int units = (groups + nw - 1) / nw;
    const bool xs_table = env_int("DMR_STREAM_XS", (P == 4 && slots >= 16 && 4 * units <= slots) ? 1 : 0) == 1 && P == 4;
    if (xs_table) {
        static const hipError_t attr_status = hipFuncSetAttribute(reinterpret_cast<const void *>(&w4_stream_kernel<4, true>),
                                                                  hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (attr_status != hipSuccess) return attr_status;
        hipLaunchKernelGGL((w4_stream_kernel<4, true>), dim3(grid), dim3(nw * 64), lds, stream, L.wt, L.sz, x, y, iM, L.N,
                           groups, tiles, lgS, lgTW, nT_max, gw_max, of, f.res, x16_magic, L.szs);
        return hipGetLastError();
    }
    switch (P) {
        DMR_STREAM_CASE(1) DMR_STREAM_CASE(2) DMR_STREAM_CASE(3) DMR_STREAM_CASE(4)
        DMR_STREAM_CASE(5) DMR_STREAM_CASE(6) DMR_STREAM_CASE(7) DMR_STREAM_CASE(8)
        default: return hipErrorInvalidValue;
    }
#undef DMR_STREAM_CASE
    return hipGetLastError();
}

}  // namespace dmr

// W4A16 decode GEMV (M == 1): the kernel behind "one generated token streams every weight once".
//
// Work split.  A workgroup owns the row tiles blockIdx.x, blockIdx.x + gridDim.x, ...; its S
// wavefronts split the groups along k once (wave w owns groups [g0, g1)) and keep that slice of
// x in wave-private LDS for the whole kernel.  Each wave walks the flattened list of
// (tile, group) blocks it owns through a register ring of P outstanding 1 KiB block loads, so
// the HBM stream never drains between tiles.  Partial sums meet in LDS once, at the end, and are
// added in wave order (deterministic).
//
// Per block: 3 shifts + 4 v_and_or_b32 per packed word turn nibbles into bf16 (128 + q) pairs,
// four 16x16x32 MFMAs contract them with x (row 0 of the A operand; the other 15 rows repeat it
// and are ignored), four more against all-ones give sum(x) in the same accumulator slot, and
//     acc += s * (D - (128 + z) * X)
// applies zero point and scale once per group.
#include "common.hpp"

namespace dmr {

namespace {

constexpr uint32_t kOnes = 0x3F803F80u;    // bf16 pair (1.0, 1.0)

// (a & mask) | c in one VALU instruction; mask rides the scalar operand slot.
__device__ __forceinline__ uint32_t and_or(uint32_t a, uint32_t mask, uint32_t c) {
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "s"(mask), "v"(c));
    return r;
}

struct Item {
    uint4 w;
    uint32_t szw;
};

template <int P, bool OUT_F32>
__global__ __launch_bounds__(1024) void w4_gemv_kernel(const uint4 *__restrict__ wt,
                                                       const uint32_t *__restrict__ sz,
                                                       const uint16_t *__restrict__ x,
                                                       void *__restrict__ y, int groups, int tiles,
                                                       int slice_uint4 /* LDS uint4 per wave slice */) {
    extern __shared__ uint4 smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, lives in an SGPR
    const int S = blockDim.x >> 6;
    const int c = lane >> 4, j = lane & 15;
    const int g0 = (groups * wave) / S;
    const int GW = (groups * (wave + 1)) / S - g0;
    const int nT = (tiles - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;
    const int items = nT * GW;

    // wave-private copy of x[128 g0 .. 128 g1): 16 uint4 per group
    uint4 *xs = smem + wave * slice_uint4;
    {
        const uint4 *src = reinterpret_cast<const uint4 *>(x) + (int64_t)g0 * 16;
        for (int i = lane; i < GW * 16; i += 64) xs[i] = src[i];
    }
    float *red = reinterpret_cast<float *>(smem + S * slice_uint4);   // [nT][S][16]

    // Issue pointer (it, ig) walks (tile slot, group in slice) and saturates at the last block,
    // so every issue is unconditional (the waitcnt bookkeeping stays exact); a wave whose item
    // count is not a multiple of P re-reads its last block up to P - 1 times from cache.
    int it = 0, ig = 0, issued = 0;
    Item ring[P];
    auto issue = [&](Item &dst) {
        const int64_t block = (int64_t)((int)blockIdx.x + it * (int)gridDim.x) * groups + (g0 + ig);
        dst.w = wt[block * 64 + lane];
        dst.szw = sz[block * kTileRows + j];
        if (issued + 1 < items) {
            ++issued;
            if (++ig == GW) {
                ig = 0;
                ++it;
            }
        }
    };

    Frag ones;
    ones.u = make_uint4(kOnes, kOnes, kOnes, kOnes);
    const uint32_t mask = 0x000F000Fu, magic = 0x43004300u;
    float acc = 0.f;
    int ct = 0, cg = 0;
    auto compute = [&](const Item &cur) {
        const uint4 *xp = xs + cg * 16 + c * 4;
        Frag a[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) a[t].u = xp[t];
        const uint32_t words[4] = {cur.w.x, cur.w.y, cur.w.z, cur.w.w};
        f32x4 d = {0.f, 0.f, 0.f, 0.f}, xsum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            Frag b;
            b.w[0] = and_or(words[t], mask, magic);
            b.w[1] = and_or(words[t] >> 4, mask, magic);
            b.w[2] = and_or(words[t] >> 8, mask, magic);
            b.w[3] = and_or(words[t] >> 12, mask, magic);
            d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[t].v, b.v, d, 0, 0, 0);
            xsum = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[t].v, ones.v, xsum, 0, 0, 0);
        }
        const float s = __uint_as_float(cur.szw << 16);
        const float cz = __uint_as_float(cur.szw & 0xFFFF0000u);   // -(128 + z)
        acc = fmaf(s, fmaf(cz, xsum[0], d[0]), acc);
        if (++cg == GW) {
            if (lane < 16) red[(ct * S + wave) * 16 + lane] = acc;
            acc = 0.f;
            cg = 0;
            ++ct;
        }
    };

    if (items > 0) {
#pragma unroll
        for (int p = 0; p < P; ++p) issue(ring[p]);
        int base = 0;
        for (; base + P < items; base += P) {
#pragma unroll
            for (int p = 0; p < P; ++p) {
                const Item cur = ring[p];
                issue(ring[p]);
                compute(cur);
            }
        }
#pragma unroll
        for (int p = 0; p < P; ++p)
            if (base + p < items) compute(ring[p]);
    }
    __syncthreads();
    for (int e = threadIdx.x; e < nT * 16; e += blockDim.x) {
        const int slot = e >> 4, col = e & 15;
        float sum = 0.f;
        for (int s = 0; s < S; ++s) sum += red[(slot * S + s) * 16 + col];
        const int64_t n = (int64_t)((int)blockIdx.x + slot * (int)gridDim.x) * kTileRows + col;
        if (OUT_F32)
            reinterpret_cast<float *>(y)[n] = sum;
        else
            reinterpret_cast<uint16_t *>(y)[n] = f32_to_bf16(sum);
    }
}

}  // namespace

hipError_t launch_w4_gemv(const LayerView &L, const uint16_t *x, void *y, bool out_f32,
                          hipStream_t stream) {
    const int groups = (int)(L.K / kGroup);
    const int tiles = (int)(L.N / kTileRows);
    static int cus = 0;   // compute units of the (single) device, asked once
    if (cus == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            cus = v;
        else
            cus = 256;
    }
    // A CU holds 16 of these wavefronts.  With S waves per workgroup, cus * 16 / S workgroups are
    // resident at once; take the largest S (most k slices, shortest per-wave stream) whose grid
    // still fits in one round, then a grid that divides the tile count when one exists.
    int S = 16;
    while (S > groups) S >>= 1;
    while (S > 4 && tiles > cus && tiles < 2 * cus && tiles > cus * (16 / S)) S >>= 1;
    int grid = tiles < cus * (16 / S) ? tiles : cus * (16 / S);
    if (tiles > grid) {
        for (int gsz = grid; gsz >= grid / 2; --gsz)
            if (tiles % gsz == 0) {
                grid = gsz;
                break;
            }
    }
    const int nT = (tiles + grid - 1) / grid;
    const int gw_max = (groups + S - 1) / S;
    const int slice_uint4 = gw_max * 16;
    const size_t lds = (size_t)S * slice_uint4 * sizeof(uint4) + (size_t)nT * S * 16 * sizeof(float);
    if (lds > 64 * 1024) return hipErrorInvalidValue;   // caller falls back to the general kernel
    // Ring depth: the P in 4..8 that wastes the fewest re-reads (largest on ties); short streams
    // take P = items.
    const int items_max = nT * gw_max;
    int P = items_max < 4 ? items_max : 4;
    if (items_max >= 4) {
        int best_waste = 1 << 30;
        for (int cand = 4; cand <= 8; ++cand) {
            const int waste = (items_max + cand - 1) / cand * cand - items_max;
            if (waste <= best_waste) {
                best_waste = waste;
                P = cand;
            }
        }
    }
    const dim3 g(grid), b(S * 64);
#define DMR_GEMV_CASE(PP)                                                                              \
    case PP:                                                                                           \
        if (out_f32)                                                                                   \
            hipLaunchKernelGGL((w4_gemv_kernel<PP, true>), g, b, lds, stream, L.wt, L.sz, x, y, groups, \
                               tiles, slice_uint4);                                                    \
        else                                                                                           \
            hipLaunchKernelGGL((w4_gemv_kernel<PP, false>), g, b, lds, stream, L.wt, L.sz, x, y, groups, \
                               tiles, slice_uint4);                                                    \
        break;
    switch (P) {
        DMR_GEMV_CASE(1) DMR_GEMV_CASE(2) DMR_GEMV_CASE(3) DMR_GEMV_CASE(4) DMR_GEMV_CASE(5)
        DMR_GEMV_CASE(6) DMR_GEMV_CASE(7) DMR_GEMV_CASE(8)
        default: return hipErrorInvalidValue;
    }
#undef DMR_GEMV_CASE
    return hipGetLastError();
}

}  // namespace dmr

// W3A16 (group 128) decode GEMV, M == 1: the native 3-bit kernel the paper did not have (its W3 cell
// ran fake-quantised and its cost was projected as T_W4 / 1.15, App. A).  Same structure as the
// 4-bit GEMV (S k slices x TW tiles of wavefronts, x and its group sums staged in LDS, a register
// ring of outstanding block loads, bf16 MFMA 16x16x32, deterministic LDS reduction); a block is
// 64 lanes x 12 bytes = 768 bytes (0.40625 bytes per weight with scale and zero point).
//
// Streaming layout of a lane's three words (32 weights k = 32 c + i): operand register r = i / 2
// (the pair i = 2r, 2r + 1, low and high half).  Every byte holds two codes in bits [0, 3) and
// [3, 6): `w & 0x07070707` and `(w >> 3) & 0x07070707` each leave four codes as clean bytes, and
// v_perm_b32 interleaves two of them with the 0x43 exponent byte into a bf16 pair (128 + q,
// 128 + q): 7 VALU instructions for the 4 registers of a word.  The spare bits [6, 8) of the bytes
// carry the last 8 codes (two low bits in words 0 and 1, the third bit in word 2): 14 more
// instructions for registers 12..15, 35 per block in all.
#include <cstdlib>

#include "w3_unpack.hpp"

namespace dmr {

namespace {


struct Item {
    uint32_t w0, w1, w2;
    uint32_t szw;
};

template <int P, int XL>
__global__ __launch_bounds__(1024) void w3_gemv_kernel(const uint32_t *__restrict__ wt,
                                                       const uint32_t *__restrict__ sz,
                                                       const uint16_t *__restrict__ x,
                                                       void *__restrict__ y, int groups, int tiles,
                                                       int lgS, int lgTW, int nT_max, int out_f32) {
    extern __shared__ uint4 smem[];          // x (16 uint4 per group), X[groups], red[nT_max][TW][S][16]
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform (SGPR)
    const int S = 1 << lgS, TW = 1 << lgTW;
    const int s = wave & (S - 1), tw = wave >> lgS;
    const int c = lane >> 4, j = lane & 15;
    const int g0 = (groups * s) >> lgS;
    const int GW = ((groups * (s + 1)) >> lgS) - g0;
    const int t_first = ((int)blockIdx.x << lgTW) + tw;
    const int t_step = (int)gridDim.x << lgTW;
    // tiles go round-robin over the grid: a wave gets nT_max of them, or one fewer
    const int nT = nT_max - ((t_first + (nT_max - 1) * t_step >= tiles) ? 1 : 0);
    const int items = nT * GW;

    // x -> registers now (oldest loads), -> LDS after the first weight loads have been issued
    uint4 xreg[XL];
    const int x16 = groups * 16;
#pragma unroll
    for (int u = 0; u < XL; ++u) {
        const int i = (int)threadIdx.x + u * (int)blockDim.x;
        xreg[u] = reinterpret_cast<const uint4 *>(x)[i < x16 ? i : 0];
    }

    // Issue pointer (it, ig) walks (tile step, group in slice) and saturates at the last block,
    // so every issue is unconditional (the waitcnt bookkeeping stays exact); a wave whose item
    // count is not a multiple of P re-reads its last block up to P - 1 times from cache.
    int it = 0, ig = 0, issued = 0;
    Item ring[P];
    auto issue = [&](Item &dst) {
        // a wave without work (its first tile lies beyond the matrix) loads the last tile instead, so
        // that the loads stay unconditional: a branch around them would make the compiler wait for
        // all of them (vmcnt(0)) where only the activations are needed
        const int tile = min(t_first + it * t_step, tiles - 1);
        const int64_t block = (int64_t)tile * groups + (g0 + ig);
        const uint32_t *pw = wt + (block * 64 + lane) * 3;
        dst.w0 = load_stream(pw);
        dst.w1 = load_stream(pw + 1);
        dst.w2 = load_stream(pw + 2);
        dst.szw = load_stream(sz + block * kTileRows + j);
        if (issued + 1 < items) {
            ++issued;
            if (++ig == GW) {
                ig = 0;
                ++it;
            }
        }
    };
#pragma unroll
    for (int p = 0; p < P; ++p) issue(ring[p]);
    float *xsum_lds = reinterpret_cast<float *>(smem + x16);                 // X[group]
    float *red = xsum_lds + ((groups + 3) & ~3);
#pragma unroll
    for (int u = 0; u < XL; ++u) {
        const int i = (int)threadIdx.x + u * (int)blockDim.x;
        // 16 consecutive threads hold one group's 128 activations: sum them (fp32, fixed order)
        float part = 0.f;
        const uint32_t xw[4] = {xreg[u].x, xreg[u].y, xreg[u].z, xreg[u].w};
#pragma unroll
        for (int q = 0; q < 4; ++q) part += __uint_as_float(xw[q] << 16) + __uint_as_float(xw[q] & 0xFFFF0000u);
        part = row16_sum(part);
        if (i < x16) {
            smem[i] = xreg[u];
            if ((i & 15) == 0) xsum_lds[i >> 4] = part;
        }
    }
    __syncthreads();

    const uint4 *xs = smem + g0 * 16;
    float acc = 0.f;
    int ct = 0, cg = 0;
    auto compute = [&](const Item &cur) {
        const uint4 *xp = xs + cg * 16 + c * 4;
        const float xg = xsum_lds[g0 + cg];
        Frag a[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) a[t].u = xp[t];
        f32x4 d = {0.f, 0.f, 0.f, 0.f};
        uint32_t reg[16];
        unpack3(cur.w0, cur.w1, cur.w2, reg);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            Frag b;
#pragma unroll
            for (int i = 0; i < 4; ++i) b.w[i] = reg[4 * t + i];
            d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[t].v, b.v, d, 0, 0, 0);
        }
        const float sc = __uint_as_float(cur.szw << 16);
        const float cz = __uint_as_float(cur.szw & 0xFFFF0000u);   // -(128 + z)
        acc = fmaf(sc, fmaf(cz, xg, d[0]), acc);
        if (++cg == GW) {
            if (lane < 16) {
                if (lgS > 0) {
                    red[((((ct << lgTW) + tw) << lgS) + s) * 16 + lane] = acc;
                } else {
                    const int64_t n = (int64_t)(t_first + ct * t_step) * kTileRows + lane;
                    if (out_f32)
                        reinterpret_cast<float *>(y)[n] = acc;
                    else
                        reinterpret_cast<uint16_t *>(y)[n] = f32_to_bf16(acc);
                }
            }
            acc = 0.f;
            cg = 0;
            ++ct;
        }
    };

    if (items > 0) {
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
    if (lgS == 0) return;

    // Cross-slice sum: thread e = (slot, column, slice) with the slice index fastest, so the S
    // partials of one output sit in S adjacent lanes and fold by DPP adds in a fixed order.
    __syncthreads();
    const int total = (nT_max << (lgTW + lgS)) * 16;
    for (int e = threadIdx.x; e < total; e += blockDim.x) {
        const int q = e & (S - 1), col = (e >> lgS) & 15, slot = e >> (lgS + 4);
        float v = red[((slot << lgS) + q) * 16 + col];
        if (S >= 2) v += dpp_move<0xB1>(v);       // quad_perm [1, 0, 3, 2]
        if (S >= 4) v += dpp_move<0x4E>(v);       // quad_perm [2, 3, 0, 1]
        if (S >= 8) v += dpp_move<0x141>(v);      // row_half_mirror
        if (S >= 16) v += dpp_move<0x140>(v);     // row_mirror
        const int tile = ((int)blockIdx.x << lgTW) + (slot & (TW - 1)) + (slot >> lgTW) * t_step;
        if (q == 0 && tile < tiles) {
            const int64_t n = (int64_t)tile * kTileRows + col;
            if (out_f32)
                reinterpret_cast<float *>(y)[n] = v;
            else
                reinterpret_cast<uint16_t *>(y)[n] = f32_to_bf16(v);
        }
    }
}

struct GemvPlan {
    int S, TW, grid;
};

// Launch shape from (groups, tiles), after a sweep of (S, TW, grid, P) on MI355X at the four
// decoder shapes: up to two workgroups' worth of tiles per CU runs as one workgroup of 16 k
// slices per tile; beyond that, 8 slices and two workgroups per CU, each looping over tiles.
GemvPlan plan_for(int groups, int tiles, int cus) {
    GemvPlan p;
    p.TW = 1;
    // measured on MI355X: the 768-byte blocks want shorter slices on wide layers than the 4-bit kernel
    p.S = tiles <= 2 * cus ? 16 : 4;
    while (p.S > groups) p.S >>= 1;
    const int resident = cus * (16 / p.S);
    p.grid = tiles <= 2 * cus ? tiles : (tiles < resident ? tiles : resident);
    return p;
}

}  // namespace

// Whether the decode kernel takes the shape with its default launch plan (x staging within eight loads per
// thread, activations and reduction buffer within 64 KB of LDS); pure host arithmetic, shared by the
// workspace query and the forward so that both name the same fallback for very long rows.
bool w3_gemv_fits(int64_t K, int64_t N) {
    const int groups = (int)(K / kGroup), tiles = (int)(N / kTileRows);
    const GemvPlan plan = plan_for(groups, tiles, compute_units());
    const int nw = plan.S * plan.TW;
    if ((groups * 16 + nw * 64 - 1) / (nw * 64) > 8) return false;
    const int t_step = plan.grid * plan.TW;
    const int nT_max = (tiles + t_step - 1) / t_step;
    const size_t lds = (size_t)groups * 16 * sizeof(uint4) + (size_t)((groups + 3) & ~3) * sizeof(float) +
                       (plan.S > 1 ? (size_t)nT_max * nw * 16 * sizeof(float) : 0);
    return lds <= 64 * 1024;
}

hipError_t launch_w3_gemv(const LayerView3 &L, const uint16_t *x, void *y, bool out_f32,
                          hipStream_t stream) {
    const int groups = (int)(L.K / kGroup);
    const int tiles = (int)(L.N / kTileRows);
    const int cus = compute_units();
    GemvPlan plan = plan_for(groups, tiles, cus);
    // sweep overrides (unset in production)
    plan.S = env_int("DMR_GEMV3_S", plan.S);
    plan.TW = env_int("DMR_GEMV3_TW", plan.TW);
    plan.grid = env_int("DMR_GEMV3_GRID", plan.grid);
    auto log2_exact = [](int v) {
        int l = 0;
        while ((1 << l) < v) ++l;
        return (1 << l) == v ? l : -1;
    };
    const int lgS = log2_exact(plan.S), lgTW = log2_exact(plan.TW);
    if (lgS < 0 || lgTW < 0 || plan.S * plan.TW > 16 || plan.S > groups || plan.grid < 1)
        return hipErrorInvalidValue;
    const int nw = plan.S * plan.TW;
    const int xl_need = (groups * 16 + nw * 64 - 1) / (nw * 64);   // x staging loads per thread
    if (xl_need > 8) return hipErrorInvalidValue;
    const int t_step = plan.grid * plan.TW;
    const int nT_max = (tiles + t_step - 1) / t_step;
    const int gw_max = (groups + plan.S - 1) / plan.S;
    const size_t lds = (size_t)groups * 16 * sizeof(uint4) + (size_t)((groups + 3) & ~3) * sizeof(float) +
                       (plan.S > 1 ? (size_t)nT_max * nw * 16 * sizeof(float) : 0);
    if (lds > 64 * 1024) return hipErrorInvalidValue;   // caller falls back to the general kernel

    // Ring depth: four blocks in flight per wave measured best (more costs registers, hence
    // resident waves); shorter streams take their whole length.
    const int items_max = nT_max * gw_max;
    int P = items_max < 4 ? items_max : 4;
    P = env_int("DMR_GEMV3_P", P);
    const dim3 g(plan.grid), b(nw * 64);
    const int of = out_f32 ? 1 : 0;
#define DMR_GEMV3_LAUNCH(PP, XX)                                                                        \
    hipLaunchKernelGGL((w3_gemv_kernel<PP, XX>), g, b, lds, stream, L.wt, L.sz, x, y, groups, tiles, lgS, \
                       lgTW, nT_max, of)
#define DMR_GEMV3_CASE(PP)                                                                              \
    case PP:                                                                                           \
        if (xl_need <= 1) DMR_GEMV3_LAUNCH(PP, 1);                                                      \
        else if (xl_need <= 2) DMR_GEMV3_LAUNCH(PP, 2);                                                 \
        else if (xl_need <= 4) DMR_GEMV3_LAUNCH(PP, 4);                                                 \
        else DMR_GEMV3_LAUNCH(PP, 8);                                                                   \
        break;
    switch (P) {
        DMR_GEMV3_CASE(1) DMR_GEMV3_CASE(2) DMR_GEMV3_CASE(3) DMR_GEMV3_CASE(4) DMR_GEMV3_CASE(6) DMR_GEMV3_CASE(8)
        default: return hipErrorInvalidValue;
    }
#undef DMR_GEMV3_CASE
#undef DMR_GEMV3_LAUNCH
    return hipGetLastError();
}

}  // namespace dmr

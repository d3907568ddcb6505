// W4A16 decode GEMV (M == 1): the kernel behind "one generated token streams every weight once".
//
// Work split.  A workgroup has S x TW wavefronts: wave (s, tw) owns the k slice s of S (groups
// [g0, g1)) and, of the TW adjacent row tiles the workgroup visits per step, tile tw; steps
// advance by gridDim.x * TW tiles.  x is staged once per workgroup in LDS.  Each wave walks the
// flattened list of (tile, group) blocks it owns through a register ring of P outstanding 1 KiB
// block loads, so the HBM stream never drains between tiles.  With S > 1 the partial sums meet in
// LDS once, at the end, and are added in slice order (deterministic, no float atomics).
//
// Per block: 2 masks, 1 shift and 4 v_perm_b32 per packed word turn nibbles into bf16 (128 + q) pairs,
// four 16x16x32 MFMAs contract them with x (row 0 of the A operand; the other 15 rows repeat it
// and are ignored), and
//     acc += s * (D - (128 + z) * X)
// applies zero point and scale once per group; X = sum of the group's 128 activations is formed
// once per workgroup while x is staged and kept in LDS beside it.
#include <cstdlib>

#include "glue.hpp"

namespace dmr {

namespace {


struct Item {
    uint4 w;
    uint32_t szw;
};

// PRO selects glue fused into the activation staging (glue.hpp): the row is normalised (RMSNorm,
// gamma in `aux`) or formed from a gate half and an up half (SwiGLU, x then holds 2 K values) in
// registers on its way into LDS.  `res`, if not null, is a bf16 residual added to the result.
template <int P, int XL, int PRO>
__global__ __launch_bounds__(1024) void w4_gemv_kernel(const uint4 *__restrict__ wt,
                                                       const uint32_t *__restrict__ sz,
                                                       const uint16_t *__restrict__ x,
                                                       void *__restrict__ y, int groups, int tiles,
                                                       int lgS, int lgTW, int nT_max, int out_f32,
                                                       const uint16_t *__restrict__ aux, float eps,
                                                       const uint16_t *__restrict__ res, int szs) {
    extern __shared__ uint4 smem[];          // x (16 uint4 per group), X[groups], red[nT_max][TW][S][16], 16 floats
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
    uint4 xaux[PRO == kProNone ? 1 : XL];     // gamma pieces (RMSNorm) or up pieces (SwiGLU)
    const int x16 = groups * 16;
#pragma unroll
    for (int u = 0; u < XL; ++u) {
        const int i = (int)threadIdx.x + u * (int)blockDim.x;
        const int ic = i < x16 ? i : 0;
        xreg[u] = reinterpret_cast<const uint4 *>(x)[ic];
        if (PRO == kProRmsNorm) xaux[u] = reinterpret_cast<const uint4 *>(aux)[ic];
        if (PRO == kProSwiGLU) xaux[u] = reinterpret_cast<const uint4 *>(x)[x16 + ic];
    }

    // The residual of the outputs this thread will store at the very end (first pass of the cross-slice sum) is
    // requested now and parked in LDS beside x: fetched after the reduction it would add a cache round trip to
    // the tail of the kernel.
    constexpr bool kEarlyRes = XL <= 4;      // the widest staging variant has no register to spare
    float res_first = 0.f;
    if (kEarlyRes && res && lgS > 0) {
        const int e = (int)threadIdx.x;
        const int q = e & (S - 1), col = (e >> lgS) & 15, slot = e >> (lgS + 4);
        const int tile = ((int)blockIdx.x << lgTW) + (slot & (TW - 1)) + (slot >> lgTW) * t_step;
        if (q == 0 && e < (nT_max << (lgTW + lgS)) * 16 && tile < tiles)
            res_first = __uint_as_float((uint32_t)res[(int64_t)tile * kTileRows + col] << 16);
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
        dst.w = load_stream(wt + block * 64 + lane);
        dst.szw = load_stream(sz + sz_index(tile, g0 + ig, groups, szs, j));
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
    float *res_lds = red + (lgS > 0 ? (nT_max << (lgTW + lgS)) * 16 : 0) + 16;   // one word per thread
    if (PRO == kProRmsNorm) {
        // sum of squares of the whole row: lanes -> wave (DPP, two cross-row steps) -> 16 waves via LDS
        float *part = red + (lgS > 0 ? (nT_max << (lgTW + lgS)) * 16 : 0);
        float ss = 0.f;
#pragma unroll
        for (int u = 0; u < XL; ++u)
            if ((int)threadIdx.x + u * (int)blockDim.x < x16) ss += sumsq_piece(xreg[u]);
        ss = wave64_sum(ss);
        if (lane == 0) part[wave] = ss;
        __syncthreads();
        // every wave adds the (at most 16) wave sums in the same DPP tree
        const int nw = (int)blockDim.x >> 6;
        const float total = row16_sum(j < nw ? part[j] : 0.f);
        const float scale = rms_scale(total, 1.0f / (float)(groups * kGroup), eps);
#pragma unroll
        for (int u = 0; u < XL; ++u) xreg[u] = rmsnorm_piece(xreg[u], xaux[u], scale);
    }
    if (PRO == kProSwiGLU) {
#pragma unroll
        for (int u = 0; u < XL; ++u) xreg[u] = swiglu_piece(xreg[u], xaux[u]);
    }
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
    if (kEarlyRes && res) res_lds[threadIdx.x] = res_first;
    __syncthreads();

    // output: the fp32 result, plus the residual if there is one, rounded once if bf16 is asked for
    auto store_out = [&](int64_t n, float v) {
        if (res) v += __uint_as_float((uint32_t)res[n] << 16);
        if (out_f32)
            reinterpret_cast<float *>(y)[n] = v;
        else
            reinterpret_cast<uint16_t *>(y)[n] = f32_to_bf16(v);
    };
    const uint4 *xs = smem + g0 * 16;
    float acc = 0.f;
    int ct = 0, cg = 0;
    auto compute = [&](const Item &cur) {
        const uint4 *xp = xs + cg * 16 + c * 4;
        const float xg = xsum_lds[g0 + cg];
        Frag a[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) a[t].u = xp[t];
        const uint32_t words[4] = {cur.w.x, cur.w.y, cur.w.z, cur.w.w};
        f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            Frag b;
            unpack_word(words[t], b.w);
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
                    store_out((int64_t)(t_first + ct * t_step) * kTileRows + lane, acc);
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
    // partials of one output sit in S adjacent lanes and fold in a fixed order.
    __syncthreads();
    const int total = (nT_max << (lgTW + lgS)) * 16;
    for (int e = threadIdx.x; e < total; e += blockDim.x) {
        const int q = e & (S - 1), col = (e >> lgS) & 15, slot = e >> (lgS + 4);
        float v = red[((slot << lgS) + q) * 16 + col];
        // the S <= 16 partials sit in one aligned group of lanes: DPP adds (pair, quad, mirrored half, mirrored
        // row) leave the total in every lane of the group, without the LDS round trips of a shuffle tree
        if (S >= 2) v += dpp_move<0xB1>(v);       // quad_perm [1, 0, 3, 2]
        if (S >= 4) v += dpp_move<0x4E>(v);       // quad_perm [2, 3, 0, 1]
        if (S >= 8) v += dpp_move<0x141>(v);      // row_half_mirror
        if (S >= 16) v += dpp_move<0x140>(v);     // row_mirror
        const int tile = ((int)blockIdx.x << lgTW) + (slot & (TW - 1)) + (slot >> lgTW) * t_step;
        if (q == 0 && tile < tiles) {
            const int64_t n = (int64_t)tile * kTileRows + col;
            if (kEarlyRes && e == (int)threadIdx.x) {   // first pass: the residual waits in LDS
                const float r = res ? v + res_lds[threadIdx.x] : v;
                if (out_f32)
                    reinterpret_cast<float *>(y)[n] = r;
                else
                    reinterpret_cast<uint16_t *>(y)[n] = f32_to_bf16(r);
            } else {
                store_out(n, v);
            }
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
    p.S = tiles <= 2 * cus ? 16 : 8;
    while (p.S > groups) p.S >>= 1;
    // Few tiles: one workgroup per tile (up to two 16-wave workgroups share a CU), which measured
    // faster than handing some workgroups a second tile.  Many tiles: as many workgroups as stay
    // resident, tiles round-robin.
    const int resident = cus * (16 / p.S);
    p.grid = tiles <= 2 * cus ? tiles : (tiles < resident ? tiles : resident);
    return p;
}

}  // namespace

// Whether the decode kernel takes the shape with its default launch plan (x staging within eight loads per
// thread; activations, reduction buffer and the parked residual within 64 KB of LDS).  Longer rows go to the
// direct-from-L2 kernel.  Pure host arithmetic.
bool w4_gemv_fits(int64_t K, int64_t N, bool with_residual) {
    const int groups = (int)(K / kGroup), tiles = (int)(N / kTileRows);
    const GemvPlan plan = plan_for(groups, tiles, compute_units());
    const int nw = plan.S * plan.TW;
    if ((groups * 16 + nw * 64 - 1) / (nw * 64) > 8) return false;
    const int t_step = plan.grid * plan.TW;
    const int nT_max = (tiles + t_step - 1) / t_step;
    const size_t lds = (size_t)groups * 16 * sizeof(uint4) + (size_t)((groups + 3) & ~3) * sizeof(float) +
                       (plan.S > 1 ? (size_t)nT_max * nw * 16 * sizeof(float) : 0) + 16 * sizeof(float) +
                       (with_residual ? (size_t)nw * 64 * sizeof(float) : 0);
    return lds <= 64 * 1024;
}

hipError_t launch_w4_gemv(const LayerView &L, const uint16_t *x, void *y, bool out_f32,
                          hipStream_t stream) {
    return launch_w4_gemv_fused(L, x, y, out_f32, Fusion{}, stream);
}

hipError_t launch_w4_gemv_fused(const LayerView &L, const uint16_t *x, void *y, bool out_f32, const Fusion &f,
                                hipStream_t stream) {
    const int groups = (int)(L.K / kGroup);
    const int tiles = (int)(L.N / kTileRows);
    const int cus = compute_units();
    GemvPlan plan = plan_for(groups, tiles, cus);
    // sweep overrides (unset in production)
    plan.S = env_int("DMR_GEMV_S", plan.S);
    plan.TW = env_int("DMR_GEMV_TW", plan.TW);
    plan.grid = env_int("DMR_GEMV_GRID", plan.grid);
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
                       (plan.S > 1 ? (size_t)nT_max * nw * 16 * sizeof(float) : 0) + 16 * sizeof(float) +
                       (f.res ? (size_t)nw * 64 * sizeof(float) : 0);
    if (lds > 64 * 1024) return hipErrorInvalidValue;   // caller falls back to the general kernel

    // Ring depth: four blocks in flight per wave measured best (six to eight measured 10-25 % slower on
    // the long-K layer even where a wave's whole stream is seven blocks); shorter streams take their
    // whole length.
    const int items_max = nT_max * gw_max;
    int P = items_max < 4 ? items_max : 4;
    P = env_int("DMR_GEMV_P", P);
    const dim3 g(plan.grid), b(nw * 64);
    const int of = out_f32 ? 1 : 0;
#define DMR_GEMV_LAUNCH_PRO(PP, XX, PRO)                                                               \
    hipLaunchKernelGGL((w4_gemv_kernel<PP, XX, PRO>), g, b, lds, stream, L.wt, L.sz, x, y, groups, tiles, \
                       lgS, lgTW, nT_max, of, f.aux, f.eps, f.res, L.szs)
#define DMR_GEMV_LAUNCH(PP, XX)                                                                        \
    do {                                                                                               \
        if (f.pro == kProRmsNorm) DMR_GEMV_LAUNCH_PRO(PP, XX, kProRmsNorm);                             \
        else if (f.pro == kProSwiGLU) DMR_GEMV_LAUNCH_PRO(PP, XX, kProSwiGLU);                          \
        else DMR_GEMV_LAUNCH_PRO(PP, XX, kProNone);                                                     \
    } while (0)
#define DMR_GEMV_CASE(PP)                                                                              \
    case PP:                                                                                           \
        if (xl_need <= 1) DMR_GEMV_LAUNCH(PP, 1);                                                      \
        else if (xl_need <= 2) DMR_GEMV_LAUNCH(PP, 2);                                                 \
        else if (xl_need <= 4) DMR_GEMV_LAUNCH(PP, 4);                                                 \
        else DMR_GEMV_LAUNCH(PP, 8);                                                                   \
        break;
    switch (P) {
        DMR_GEMV_CASE(1) DMR_GEMV_CASE(2) DMR_GEMV_CASE(3) DMR_GEMV_CASE(4)
        default: return hipErrorInvalidValue;
    }
#undef DMR_GEMV_CASE
#undef DMR_GEMV_LAUNCH
#undef DMR_GEMV_LAUNCH_PRO
    return hipGetLastError();
}

}  // namespace dmr

// A whole decode step of the 4-bit copy (M == 1) as ONE resident grid: the Linear layers of the step
// run in order inside a single launch, separated by grid-wide barriers instead of kernel boundaries.
//
// Why.  At M == 1 a layer moves 9..62 MB and takes 4..12 us, of which about 2.5 us are the launch and
// the ramp of the memory pipeline from empty: a chain of per-layer launches cannot keep HBM busy across
// its boundaries.  Here every wave walks ONE list of weight blocks that runs through all stages, with
// a register ring of P block loads in flight.  Weights do not depend on the activations, so the ring
// runs ahead into the next stage while the current one is reduced, stored and synchronised: the
// barrier is paid with the memory pipeline full.
//
// Work split (as the per-layer GEMV): one workgroup of 16 waves per CU; workgroup b owns the row tiles
// b, b + grid, ... of every stage, wave s the k slice s of 16.  The activation row is staged in LDS with
// the group sums X beside it; per block  acc += s * (D - (128 + z) * X)  with D from four MFMAs; the 16
// slice sums of an output meet in LDS and are added in a fixed order.
//
// Grid barrier.  Stage k + 1 reads what stage k wrote (the row, the residual), on other CUs and other
// XCDs: storing waves release at agent scope, then the workgroup writes the number of stages it has
// finished into its own word of a flag array in device memory (no read-modify-write on a shared word:
// 256 of those on one address serialise at the memory side and cost tens of microseconds), and one
// wave per workgroup reads the whole array with agent-scope loads until no flag is behind; rows and
// residuals are then read with agent-scope loads, which no stale cache line can serve.  The poll is
// bounded: a workgroup that gives up sets the time-out word, which every poll also reads and which
// opens all later barriers, so the grid always drains (results are then garbage and the host reports
// the word).  All workgroups must be resident at once: the host launches no more than fit.
#include "chain.hpp"
#include "glue.hpp"

namespace dmr {

namespace {

struct Item {
    uint4 w;
    uint32_t szw;
};

// Workgroup barrier for LDS traffic only: waits for this wave's LDS operations, not for its global
// loads (the ring stays in flight across it).  A __syncthreads() would drain the ring.
__device__ __forceinline__ void lds_barrier() {
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    __builtin_amdgcn_s_waitcnt(0xC07F);     // lgkmcnt(0); vmcnt and expcnt untouched
    __builtin_amdgcn_s_barrier();
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
}

// Pointers that come out of the stage table are generic to the compiler; a generic ("flat") access counts
// as an LDS operation too, so every wait for an LDS read would also wait for the whole weight ring.
// Everything the table points to is device memory: say so.
#define DMR_GLOBAL __attribute__((address_space(1)))
template <typename T>
__device__ __forceinline__ DMR_GLOBAL T *as_global(const void *p) {
    return reinterpret_cast<DMR_GLOBAL T *>(reinterpret_cast<uintptr_t>(p));
}
__device__ __forceinline__ uint4 load_stream_g(const uint4 *p) {
    const u32x4_t v = __builtin_nontemporal_load(as_global<const u32x4_t>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint32_t load_stream_g(const uint32_t *p) {
    return __builtin_nontemporal_load(as_global<const uint32_t>(p));
}

// 16 bytes written by another workgroup of this launch: agent-scope loads.
__device__ __forceinline__ uint4 load_agent16(const uint16_t *base, int piece) {
    DMR_GLOBAL uint64_t *p = as_global<uint64_t>(base) + 2 * (int64_t)piece;
    const uint64_t a = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint64_t b = __hip_atomic_load(p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_uint4((uint32_t)a, (uint32_t)(a >> 32), (uint32_t)b, (uint32_t)(b >> 32));
}
__device__ __forceinline__ float load_agent_bf16(const uint16_t *p) {
    const uint16_t v = __hip_atomic_load(as_global<uint16_t>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return __uint_as_float((uint32_t)v << 16);
}

// One stage of the table as the kernel keeps it in LDS (wave-uniform values, read into scalar registers).
struct StageRef {
    const uint32_t *w;     // LDS: the 16 words of a ChainStage
    __device__ __forceinline__ int word(int i) const { return __builtin_amdgcn_readfirstlane((int)w[i]); }
    __device__ __forceinline__ const void *ptr(int i) const {
        const uint64_t lo = (uint32_t)word(2 * i), hi = (uint32_t)word(2 * i + 1);
        return reinterpret_cast<const void *>(lo | (hi << 32));
    }
    __device__ __forceinline__ const uint4 *wt() const { return static_cast<const uint4 *>(ptr(0)); }
    __device__ __forceinline__ const uint32_t *sz() const { return static_cast<const uint32_t *>(ptr(1)); }
    __device__ __forceinline__ const uint16_t *in() const { return static_cast<const uint16_t *>(ptr(2)); }
    __device__ __forceinline__ const uint16_t *aux() const { return static_cast<const uint16_t *>(ptr(3)); }
    __device__ __forceinline__ const uint16_t *res() const { return static_cast<const uint16_t *>(ptr(4)); }
    __device__ __forceinline__ void *out() const { return const_cast<void *>(ptr(5)); }
    __device__ __forceinline__ int groups() const { return word(12); }
    __device__ __forceinline__ int tiles() const { return word(13); }
    __device__ __forceinline__ int flags() const { return word(14); }
    __device__ __forceinline__ float eps() const { return __int_as_float(word(15)); }
};

template <int P, int R>
__device__ __forceinline__ void rotate_ring(Item (&ring)[P]) {   // ring[k] <- ring[(k + R) % P]
    Item tmp[P];
#pragma unroll
    for (int k = 0; k < P; ++k) tmp[k] = ring[(k + R) % P];
#pragma unroll
    for (int k = 0; k < P; ++k) ring[k] = tmp[k];
}

__global__ void chain_reset_kernel(uint32_t *ctl) {
    if (threadIdx.x < kChainMaxGrid) ctl[threadIdx.x] = 0;     // the arrival flags; the time-out word is sticky
}

template <int P>
__global__ __launch_bounds__(1024) void w4_chain_kernel(const ChainStage *__restrict__ tab, uint32_t *ctl,
                                                        int n_stages, int x16_cap, int g_cap, int spin_limit, int tune) {
    // LDS: stage table (4 uint4 per stage) | next stage with tiles for this workgroup [n_stages + 1, padded to 4] |
    //      x (16 pieces per group) | X[g_cap] | 16 wave sums | red[nt][16 slices][16]
    extern __shared__ uint4 lds_base[];
    int *next_with_tiles = reinterpret_cast<int *>(lds_base + 4 * n_stages);
    uint4 *smem = lds_base + 4 * n_stages + (n_stages + 4) / 4;
    float *xsum_lds = reinterpret_cast<float *>(smem + x16_cap);
    float *part = xsum_lds + g_cap;
    float *red = part + 16;
    const int tid = (int)threadIdx.x, lane = tid & 63;
    const int s = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave = k slice
    const int c = lane >> 4, j = lane & 15;
    const int b = (int)blockIdx.x, G = (int)gridDim.x;
    // The table moves to LDS once: reading it there later does not queue behind the weight loads in flight.
    for (int i = tid; i < 4 * n_stages; i += 1024) lds_base[i] = reinterpret_cast<const uint4 *>(tab)[i];
    __syncthreads();
    auto stage = [&](int k) { return StageRef{reinterpret_cast<const uint32_t *>(lds_base + 4 * k)}; };
    // next_with_tiles[k]: first stage >= k in which this workgroup owns a tile (n_stages if none), so that the
    // issue side steps over stages narrower than the grid without a loop in the hot path
    for (int k = tid; k <= n_stages; k += 1024) {
        int k2 = k;
        while (k2 < n_stages && (int)reinterpret_cast<const uint32_t *>(lds_base + 4 * k2)[13] <= b) ++k2;
        next_with_tiles[k] = k2;
    }
    __syncthreads();

    // ---- issue side: the next block to load, anywhere in the chain ------------------------------------
    int is = -1, igroups = 0, ig0 = 0, iGW = 1, inT = 1, it = 0, ig = 0;
    bool idone = false;
    const uint4 *iwt = stage(0).wt();
    const uint32_t *isz = stage(0).sz();
    const uint4 *nw = iwt + lane;            // block 0 of stage 0: a valid address for a workgroup without tiles
    const uint32_t *nsz = isz + j;
    auto next_ptrs = [&]() {
        const int64_t block = (int64_t)(b + it * G) * igroups + (ig0 + ig);
        nw = iwt + block * 64 + lane;
        nsz = isz + block * kTileRows + j;
    };
    auto issue_stage = [&]() {               // on to the next stage in which this workgroup owns tiles
        is = __builtin_amdgcn_readfirstlane(next_with_tiles[is + 1]);
        if (is >= n_stages) {
            idone = true;                    // past the end: keep re-reading the last block (loads stay unconditional)
            return;
        }
        const StageRef st = stage(is);
        igroups = st.groups();
        iwt = st.wt();
        isz = st.sz();
        ig0 = (igroups * s) >> 4;
        iGW = ((igroups * (s + 1)) >> 4) - ig0;
        inT = (st.tiles() - b - 1) / G + 1;
        it = 0;
        ig = 0;
        next_ptrs();
    };
    auto issue = [&](Item &dst) {
        dst.w = load_stream_g(nw);
        dst.szw = load_stream_g(nsz);
        if (!idone) {
            if (++ig == iGW) {
                ig = 0;
                ++it;
            }
            if (it == inT)
                issue_stage();
            else
                next_ptrs();
        }
    };
    issue_stage();
    Item ring[P];
#pragma unroll
    for (int p = 0; p < P; ++p) issue(ring[p]);

    // ---- compute side ------------------------------------------------------------------------------------
    int cs = -1, cgroups = 0, cg0 = 0, cGW = 1, cnT = 0, cflags = 0, ct = 0, cg = 0;
    float acc = 0.f;

    auto epilogue = [&]() {                  // slice sums -> outputs, then arrive at the grid barrier
        if (cnT > 0) {
            lds_barrier();
            const StageRef st = stage(cs);
            const uint16_t *res = st.res();
            void *out = st.out();
            const int total = cnT * 256;
            for (int e = tid; e < total; e += 1024) {
                const int q = e & 15, col = (e >> 4) & 15, slot = e >> 8;
                float v = row16_sum(red[(slot * 16 + q) * 16 + col]);
                if (q == 0) {
                    const int64_t n = (int64_t)(b + slot * G) * kTileRows + col;
                    if (res) v += load_agent_bf16(res + n);
                    if (cflags & 0x100)
                        as_global<float>(out)[n] = v;
                    else if (tune & 1)
                        __hip_atomic_store(as_global<uint16_t>(out) + n, f32_to_bf16(v), __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
                    else
                        as_global<uint16_t>(out)[n] = f32_to_bf16(v);
                }
            }
            // wave-uniform (total is a multiple of 256): the waves that stored make it visible to the device
            if (tid < total) {
                if (tune & 1)
                    __builtin_amdgcn_s_waitcnt(0x0070);      // vmcnt(0) lgkmcnt(0)
                else if (!(tune & 8))
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            }
        }
        if (cs + 1 < n_stages) {
            lds_barrier();                   // every storing wave has released
            if (tid == 0) __hip_atomic_store(ctl + b, (uint32_t)(cs + 1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    };

    auto prologue = [&]() {                  // wait for the stage before, then stage the activation row
        const StageRef st = stage(cs);
        const int ctiles = st.tiles();
        cgroups = st.groups();
        cflags = st.flags();
        cg0 = (cgroups * s) >> 4;
        cGW = ((cgroups * (s + 1)) >> 4) - cg0;
        cnT = ctiles > b ? (ctiles - b - 1) / G + 1 : 0;
        ct = 0;
        cg = 0;
        acc = 0.f;
        if (cs > 0) {
            if (s == 0 && !(tune & 2)) {
                // wave 0 reads all arrival flags at once (four per lane and pass) until none is behind
                int spins = 0;
                for (;;) {
                    uint32_t behind = 0;
                    for (int base = 0; base < G; base += 256) {
                        const int i = base + lane * 4;
                        const uint4 f = load_agent16(reinterpret_cast<const uint16_t *>(ctl), (i < G ? i : 0) >> 2);
                        const uint32_t fw[4] = {f.x, f.y, f.z, f.w};
#pragma unroll
                        for (int q = 0; q < 4; ++q) behind |= (i + q < G && fw[q] < (uint32_t)cs) ? 1u : 0u;
                    }
                    const uint32_t gave_up = __hip_atomic_load(ctl + kChainTimeoutWord, __ATOMIC_RELAXED,
                                                               __HIP_MEMORY_SCOPE_AGENT);
                    if (__builtin_amdgcn_ballot_w64(behind != 0) == 0 || gave_up != 0) break;
                    if (++spins > spin_limit) {
                        if (lane == 0)
                            __hip_atomic_store(ctl + kChainTimeoutWord, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        break;
                    }
                    __builtin_amdgcn_s_sleep(1);
                }
            }
            lds_barrier();
        }
        if (cnT == 0) return;
        const int pro = cflags & 0xFF;
        const int x16 = cgroups * 16;
        const uint16_t *xin = st.in(), *gamma = st.aux();
        uint4 xreg[2], xaux[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            xreg[u] = make_uint4(0, 0, 0, 0);
            xaux[u] = make_uint4(0, 0, 0, 0);
            if (u * 1024 < x16) {            // uniform
                const int i = tid + u * 1024;
                const int ic = i < x16 ? i : 0;
                xreg[u] = load_agent16(xin, ic);
                if (pro == kProRmsNorm) {
                    const u32x4_t gv = as_global<const u32x4_t>(gamma)[ic];
                    xaux[u] = make_uint4(gv.x, gv.y, gv.z, gv.w);
                }
                if (pro == kProSwiGLU) xaux[u] = load_agent16(xin, x16 + ic);
            }
        }
        if (pro == kProRmsNorm) {
            float ss = 0.f;
#pragma unroll
            for (int u = 0; u < 2; ++u)
                if (tid + u * 1024 < x16) ss += sumsq_piece(xreg[u]);
            ss = wave64_sum(ss);
            if (lane == 0) part[s] = ss;
            lds_barrier();
            const float total = row16_sum(part[j]);
            const float scale = rms_scale(total, 1.0f / (float)(cgroups * kGroup), st.eps());
#pragma unroll
            for (int u = 0; u < 2; ++u) xreg[u] = rmsnorm_piece(xreg[u], xaux[u], scale);
        }
        if (pro == kProSwiGLU) {
#pragma unroll
            for (int u = 0; u < 2; ++u) xreg[u] = swiglu_piece(xreg[u], xaux[u]);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (u * 1024 < x16) {
                const int i = tid + u * 1024;
                float gsum = 0.f;
                const uint32_t xw[4] = {xreg[u].x, xreg[u].y, xreg[u].z, xreg[u].w};
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    gsum += __uint_as_float(xw[q] << 16) + __uint_as_float(xw[q] & 0xFFFF0000u);
                gsum = row16_sum(gsum);      // 16 consecutive threads hold one group's 128 activations
                if (i < x16) {
                    smem[i] = xreg[u];
                    if ((i & 15) == 0) xsum_lds[i >> 4] = gsum;
                }
            }
        }
        lds_barrier();
    };

    auto next_stage = [&]() -> bool {        // false when the chain is finished
        for (;;) {
            if (cs >= 0) epilogue();
            if (++cs == n_stages) return false;
            prologue();
            if (cnT > 0) return true;
        }
    };

    auto compute = [&](const Item &cur) -> bool {   // true when this wave has finished the stage
        const uint4 *xp = smem + (cg0 + cg) * 16 + c * 4;
        const float xg = xsum_lds[cg0 + cg];
        Frag a[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) a[t].u = xp[t];
        const uint32_t words[4] = {cur.w.x, cur.w.y, cur.w.z, cur.w.w};
        f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            Frag wb;
            unpack_word(words[t], wb.w);
            d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[t].v, wb.v, d, 0, 0, 0);
        }
        const float sc = __uint_as_float(cur.szw << 16);
        const float cz = __uint_as_float(cur.szw & 0xFFFF0000u);   // -(128 + z)
        acc = fmaf(sc, fmaf(cz, xg, d[0]), acc);
        if (++cg == cGW) {
            if (lane < 16) red[(ct * 16 + s) * 16 + lane] = acc;
            acc = 0.f;
            cg = 0;
            return ++ct == cnT;
        }
        return false;
    };

    if (!next_stage()) return;
    for (;;) {
        int left = cnT * cGW;                // blocks this wave still owes the current stage (>= 1)
        // Full turns of the ring: nothing but consume-and-refill.  Every load issued so far has landed here
        // (the activation row was loaded after them and has been used); saying so with an explicit wait gives
        // the compiler a clean state at the loop entry, and with it exact wait counts inside the loop.
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
        while (left > P) {
#pragma unroll
            for (int p = 0; p < P; ++p) {
                compute(ring[p]);            // consume, then refill the same registers
                issue(ring[p]);
            }
            left -= P;
        }
        // last 1..P blocks of the stage: the refills already belong to later stages
#pragma unroll
        for (int p = 0; p < P; ++p) {
            if (p < left) {
                compute(ring[p]);
                issue(ring[p]);
            }
        }
        if (!next_stage()) return;
        // every ring load has landed by now (the row was loaded after them): bring the oldest entry back to
        // slot 0 so that ring indices stay compile-time constants
#define DMR_CHAIN_ROT(RR) \
    if (RR < P && left == RR) rotate_ring<P, (RR < P ? RR : 0)>(ring);
        DMR_CHAIN_ROT(1) DMR_CHAIN_ROT(2) DMR_CHAIN_ROT(3) DMR_CHAIN_ROT(4)
        DMR_CHAIN_ROT(5) DMR_CHAIN_ROT(6) DMR_CHAIN_ROT(7)
#undef DMR_CHAIN_ROT
    }
}

constexpr int kRing = 8;

}  // namespace

size_t chain_lds_bytes(const ChainLaunch &c) {
    return (size_t)c.n_stages * sizeof(ChainStage) + (size_t)((c.n_stages + 4) / 4) * sizeof(uint4) + (size_t)c.x16_cap * sizeof(uint4) + (size_t)c.g_cap * sizeof(float) + 16 * sizeof(float) +
           (size_t)c.nt_cap * 256 * sizeof(float);
}

int chain_resident_grid(size_t lds_bytes) {
    static const hipError_t attr_status = hipFuncSetAttribute(
        reinterpret_cast<const void *>(w4_chain_kernel<kRing>), hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
    if (attr_status != hipSuccess || lds_bytes > 128 * 1024) return 0;
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, w4_chain_kernel<kRing>, 1024, lds_bytes) != hipSuccess ||
        per_cu < 1)
        return 0;
    return compute_units();                  // one workgroup per CU
}

hipError_t launch_w4_chain(const ChainLaunch &c, hipStream_t stream) {
    if (c.n_stages < 1 || c.grid < 1 || c.grid > kChainMaxGrid || c.grid > chain_resident_grid(chain_lds_bytes(c))) return hipErrorInvalidValue;
    hipLaunchKernelGGL(chain_reset_kernel, dim3(1), dim3(1024), 0, stream, c.ctl);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int tune = env_int("DMR_CHAIN_TUNE", 0);
    switch (env_int("DMR_CHAIN_P", kRing)) {
        case 4:
            hipLaunchKernelGGL((w4_chain_kernel<4>), dim3(c.grid), dim3(1024), chain_lds_bytes(c), stream, c.tab, c.ctl,
                               c.n_stages, c.x16_cap, c.g_cap, c.spin_limit, tune);
            break;
        case 6:
            hipLaunchKernelGGL((w4_chain_kernel<6>), dim3(c.grid), dim3(1024), chain_lds_bytes(c), stream, c.tab, c.ctl,
                               c.n_stages, c.x16_cap, c.g_cap, c.spin_limit, tune);
            break;
        default:
            hipLaunchKernelGGL((w4_chain_kernel<kRing>), dim3(c.grid), dim3(1024), chain_lds_bytes(c), stream, c.tab,
                               c.ctl, c.n_stages, c.x16_cap, c.g_cap, c.spin_limit, tune);
    }
    return hipGetLastError();
}

}  // namespace dmr

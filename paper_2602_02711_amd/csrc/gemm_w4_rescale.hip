// Tiled MFMA GEMM for prefill-sized M on a 4-bit (or 3-bit) layer that never rounds a weight and keeps ONE accumulator tile.
//
//     y[m][n] = sum_G s[n][G] * ( sum_{k in G} x[m][k] (16 + q[n][k]) )  -  sum_G s[n][G] (16 + z[n][G]) X[m][G]
//
// with X[m][G] the sum of the activations of row m over group G.  The matrix cores multiply the activations
// with exact bf16 values (16 + q) / 2 (a magic-number unpack like the decode kernels': shifts, masks and
// v_perm_b32 only, one VALU instruction per weight; the factor 2 goes into the last scale).  The group scale is not
// applied to a per-group tile: the accumulator is kept in units of the CURRENT group's scale.  Between groups G and
// G + 1 every accumulator element is multiplied by s[G] / s[G + 1] (one VALU multiply per element and group, in place),
// the MFMAs of the next group add into it directly, and after the last group it is multiplied by the last scale.  No
// second tile and no fold: 128 accumulator registers per wave, in ordinary vector registers (the kernel is compiled
// for two waves per SIMD, i.e. at most 256 registers, which makes the compiler use the MFMA forms whose accumulator
// the VALU can address).
//
// The zero-point term is a product of rank K / 128.  A pre-pass splits the fp32 group sums X into three bf16
// terms and the exact products c = -s (16 + z) into two, and lays them out as two plain bf16 matrices A2[M][KP],
// B2[N][KP] whose product over KP = 6 K / 128 columns (all pairs of terms) is that sum; the kernel runs it as a
// short second k loop on bf16 operands into the same accumulator.  It adds 4.7 % to the MFMA count.
//
// A layer qualifies when every scale is a normal nonzero number and the scales of a row stay within 2^20 of its
// first one (the running rescale would otherwise divide by zero or overflow).  The pre-pass checks that per block
// of 32 rows and leaves a flag; a workgroup whose columns are flagged returns at once and the 128 x 128 exact
// kernel, launched behind this one with the same flags, computes those columns instead.
//
// Shape of the work.  Eight wavefronts (2 x 4), two per SIMD, in three instantiations: a 256 x 256 tile with a 128 x 64
// patch per wave (4 x 2 tiles of v_mfma_f32_32x32x16_bf16), for grids that one round of them covers a 256 x 128
// tile with 128 x 32 per wave (4 x 1), and for outputs of at most 256 blocks of 128 x 128 a 128 x 128 tile with 64 x 32
// per wave (2 x 1; 82 registers and 74 KiB of LDS, so two workgroups share a CU).  (The kernel is written for WM x WN waves of TM x TN tiles; 256 x 128 on four
// waves of 128 x 64 and on eight of 64 x 64 were measured 0-8 % behind and are not instantiated.)
//
// The weight operand never sits in LDS unpacked.  The codes of a weight row are private to the waves that own its
// column, so nothing has to be unpacked INTO a shared stage: the packed codes travel global -> LDS as they are (32 bytes
// per weight row and 64 k, one `global_load_lds_dwordx4` per wave and stage), every wave reads the 16 bytes of its own
// columns back and unpacks them in registers straight into MFMA B operands, one word (8 codes, one operand) per MFMA
// round.  LDS then carries, per 64 k and workgroup, 32 KiB of activations in (direct-to-LDS as well) and 16 fragment
// reads per wave out: two thirds of the fragment reads and half of the writes of a kernel that stages both operands
// (the bf16 twin; the first version of this one, which unpacked into the stage: 1740 -> 1530 us on gate+up at 8192
// rows), whose LDS port is as busy as its matrix cores.
//
// A stage is 64 k = four MFMA rounds: lane half h of an MFMA operand takes the k step 2 v + h of the group's half v,
// word w of it in round w, so that a lane's 16 code bytes are exactly its four B operands; the activation fragment of
// that round is 16-byte chunk 4 h + w of the row's 128-byte slice (chunks XOR-swizzled with bits 1..3 of the row
// number: 16 consecutive rows then cover the 16 bank groups of 16 bytes; swizzling with bits 0..2 measured 1.2e8
// conflict cycles per launch, this none).  Three stages of 32 KiB + the codes, requested two stages ahead; one bare
// barrier per stage, behind the third round, the fourth round's MFMAs starting at once with the next requests and the
// first reads of the next stage between them.  The rescale factors of a wave's 64 columns come direct-to-LDS into a
// slot of the wave's own, one instruction per group.  The zero-point loop runs on four stages of 32 k with both
// operands direct-to-LDS (rows of 64 bytes, chunks swizzled with bits 2..3 of the row number).
#include "common.hpp"

namespace dmr {

namespace {

constexpr int kMaxBM = 256;                                // rows of the largest tile
// first loop: stages of 64 k, activations and packed codes
constexpr int BK2 = 64, ROW2 = BK2 * 2, NS2 = 3;
// second loop (zero-point term): stages of 32 k, both operands as bf16
constexpr int BK = 32, NS = 4;
constexpr int ROW_BYTES = BK * 2;                          // 64

// WM x WN wavefronts, each on TM x TN MFMA tiles of 32 x 32; code width BITS (4 or 3).
template <int WM, int WN, int TM, int TN, int BITS>
struct Geo {
    static constexpr int WAVES = WM * WN, THREADS = 64 * WAVES;
    static constexpr int BM = 32 * TM * WM;                                // 256 (or 128)
    static constexpr int BN = 32 * TN * WN;                                // 128 or 256
    // first loop
    static constexpr int A2S_BYTES = BM * ROW2;                            // 32 KiB (16)
    // the codes of a stage: 32 bytes per weight row, two row tiles of 16 per load instruction.  Where one instruction
    // per wave covers the tile's columns exactly once, every wave reads its columns from whichever wave fetched them;
    // otherwise every wave fetches the 2 TN row tiles of its own columns into a slot of its own.
    static constexpr bool PRIVATE_CODES = BN / kTileRows != 2 * WAVES;
    static constexpr int RI = PRIVATE_CODES ? TN : 1;                      // code load instructions per wave and stage
    static constexpr int RAWB = WAVES * RI * 1024;
    static constexpr int STAGE = A2S_BYTES + RAWB;                         // 40 or 36 KiB (48 with private codes)
    static constexpr int FAC_OFF = NS2 * STAGE;                            // 256 bytes of factors per wave
    static constexpr int MAIN_BYTES = FAC_OFF + WAVES * 256;
    static constexpr int RA = A2S_BYTES / 1024 / WAVES;                    // activation load instructions per wave and stage
    static constexpr int RL = RA + RI;                                     // ... plus the codes
    static_assert(RA >= 1 && RA * WAVES * 1024 == A2S_BYTES, "whole load instructions");
    // second loop
    static constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BN * ROW_BYTES;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;                  // 24 or 32 KiB
    static constexpr int PH2_BYTES = NS * STAGE_BYTES;
    static constexpr int LA = BM / 16 / WAVES;                             // A2 load instructions per wave and step
    static constexpr int LB = BN / 16 / WAVES;                             // B2 load instructions per wave and step
    static constexpr int L2 = LA + LB;
    static_assert(LA >= 1 && LB >= 1, "whole load instructions");
    static constexpr size_t LDS_BYTES = MAIN_BYTES > PH2_BYTES ? MAIN_BYTES : PH2_BYTES;
};

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void global_void;

// s_waitcnt vmcnt(N) with lgkmcnt(0): the barrier that follows is a bare s_barrier.
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (0 << 8));
}

// Workgroup barrier without the fences of __syncthreads() (which would wait for every direct-to-LDS load in
// flight); what must have landed is waited for explicitly before this is called.
__device__ __forceinline__ void bare_barrier() {
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    __builtin_amdgcn_s_barrier();
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
}

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 2) & 3); }

// Fragments of the second loop's stages.  (Restrict pointers: see read_a_frags.)
template <int TM, int TN>
__device__ __forceinline__ void load_frags(const uint8_t *__restrict__ As, const uint8_t *__restrict__ Bs, int ks,
                                           Frag (&a)[TM], Frag (&b)[TN], int lane, int wm, int wn) {
    const int chunk = ks * 2 + (lane >> 5);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int ra = wm * 32 * TM + i * 32 + (lane & 31);
        a[i].u = *reinterpret_cast<const uint4 *>(As + ra * ROW_BYTES + swz(ra, chunk) * 16);
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int rb = wn * 32 * TN + j * 32 + (lane & 31);
        b[j].u = *reinterpret_cast<const uint4 *>(Bs + rb * ROW_BYTES + swz(rb, chunk) * 16);
    }
}

template <int TM, int TN>
__device__ __forceinline__ void mfma_all(const Frag (&a)[TM], const Frag (&b)[TN], f32x16 (&acc)[TM][TN]) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i].v, b[j].v, acc[i][j], 0, 0, 0);
}

// One word of a lane's codes -> the 8 bf16 values (16 + q) / 2 = 8 + q / 2 of an MFMA B operand.  Each nibble goes to
// mantissa bits [3, 7) of a bf16 whose high byte is 0x41 and whose exponent's lowest bit (the top bit of the low byte)
// stays clear: 2^3 (1 + q / 16).  (With that bit set the value would be 16 + q; leaving it saves an OR per four
// weights.  The decode kernels' 128 + q would carry an offset eight times larger into the cancellation with the
// zero-point term.)  In the streaming layout word w of a lane's unit holds the 8 codes of k = 8 w .. 8 w + 7 of its k
// step, the nibbles in the order 0, 4, 1, 5, 2, 6, 3, 7 that the four permutes below undo.
__device__ __forceinline__ void unpack4_word(uint32_t w, Frag &f) {
    const uint32_t even = (w << 3) & 0x78787878u;     // nibbles 0, 2, 4, 6 as low bytes
    const uint32_t odd = (w >> 1) & 0x78787878u;      // nibbles 1, 3, 5, 7
    const uint32_t exp = 0x41414141u;
    f.w[0] = __builtin_amdgcn_perm(even, exp, 0x00060004u);
    f.w[1] = __builtin_amdgcn_perm(odd, exp, 0x00060004u);
    f.w[2] = __builtin_amdgcn_perm(even, exp, 0x00070005u);
    f.w[3] = __builtin_amdgcn_perm(odd, exp, 0x00070005u);
}

// The 3-bit unit (three words per weight row and k step): chunk c < 3 of the row's 32 k is the two 3-bit fields of
// the bytes of word c, chunk 3 the spare top bits of all three words (bit 6 + h of word 2 is the third bit of a code
// in half h of the chunk, the top two bits of word h its low two).  Codes land in mantissa bits [3, 6): values
// (16 + q) / 2 as for four bits.
__device__ __forceinline__ void unpack3_chunk(const u32x4_t &u, int c, Frag &f) {
    const uint32_t exp = 0x41414141u, m38 = 0x38383838u;
    const uint32_t sel_a = 0x00060004u, sel_b = 0x00070005u;
    uint32_t f0, f1;
    if (c < 3) {
        const uint32_t v = u[c];
        f0 = (v << 3) & m38;
        f1 = v & m38;
    } else {
        f0 = (((u[2] >> 6) & 0x01010101u) << 5) | (((u[0] >> 6) & 0x03030303u) << 3);
        f1 = (((u[2] >> 7) & 0x01010101u) << 5) | (((u[1] >> 6) & 0x03030303u) << 3);
    }
    f.w[0] = __builtin_amdgcn_perm(f0, exp, sel_a);
    f.w[1] = __builtin_amdgcn_perm(f0, exp, sel_b);
    f.w[2] = __builtin_amdgcn_perm(f1, exp, sel_a);
    f.w[3] = __builtin_amdgcn_perm(f1, exp, sel_b);
}

// LDS reads through restrict pointers: the alias scopes they carry keep the wait-count pass from tying them to the
// direct-to-LDS loads in flight, whose completion the kernel waits for explicitly.  (A scope only appears for a restrict
// parameter that is used and has another one to be distinct from, and only survives on a load of a vector type; hence
// two pointers into the same buffer.)
template <int TM>
__device__ __forceinline__ void read_a_frags(const uint8_t *__restrict__ p, const uint8_t *__restrict__ q, Frag (&a)[TM]) {
    static_assert(TM % 2 == 0, "half of the tiles through each pointer (q = p + TM / 2 tiles)");
#pragma unroll
    for (int i = 0; i < TM / 2; ++i) {
        const u32x4_t lo = *reinterpret_cast<const u32x4_t *>(p + i * 32 * ROW2);
        const u32x4_t hi = *reinterpret_cast<const u32x4_t *>(q + i * 32 * ROW2);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            a[i].w[c] = lo[c];
            a[TM / 2 + i].w[c] = hi[c];
        }
    }
}
template <int TN>
__device__ __forceinline__ void read_code_units(const uint8_t *__restrict__ p, const uint8_t *__restrict__ q, u32x4_t (&rw)[TN]) {
    if constexpr (TN == 2) {            // one unit through each pointer (q = p + 1 KiB)
        rw[0] = *reinterpret_cast<const u32x4_t *>(p);
        rw[1] = *reinterpret_cast<const u32x4_t *>(q);
    } else {                            // one unit, half through each pointer (q = p + 8)
        typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
        const u32x2_t lo = *reinterpret_cast<const u32x2_t *>(p);
        const u32x2_t hi = *reinterpret_cast<const u32x2_t *>(q);
        rw[0] = u32x4_t{lo[0], lo[1], hi[0], hi[1]};
    }
}
template <int TN>
__device__ __forceinline__ void read_wave_factors(const uint8_t *__restrict__ p, const uint8_t *__restrict__ q, float (&rf)[TN]) {
    rf[0] = *reinterpret_cast<const float *>(p);
    const float other = *reinterpret_cast<const float *>(q);      // q = p + 128: the factor of the column 32 further on
    if constexpr (TN == 2)
        rf[1] = other;
    else                                                          // (a use that folds away: the scope needs one)
        rf[0] = __uint_as_float(__float_as_uint(rf[0]) | (__float_as_uint(other) & 0u));
}

// wt: the layer's codes in the streaming layout (1 KiB, 3-bit 768 B, per row tile of 16 and group; the unit of lane
// 16 c + j of a block is row j's 32 codes of k step c).  rfac: [row tile][groups + 1][16] fp32, factor of (row, group):
// s[G - 1] / s[G] for G >= 1, the LAST scale for G = 0 (the accumulator is zero when group 0 starts, so that slot is
// free), 1 in the slot behind the last group.  a2 / b2: bf16 [M][KP] / [N][KP].  flags: one word per 32 columns,
// nonzero = those columns do not qualify; a tile with a flagged part is left to the other kernel as a whole.
template <int WM, int WN, int TM, int TN, int BITS, bool OUT_F32, bool PC>
__global__ __launch_bounds__(64 * WM * WN, TM * TN <= 2 ? 2 : 1) void gemm_w4_rescale_kernel(
    const void *__restrict__ wt, const float *__restrict__ rfac, const uint16_t *__restrict__ x, const uint16_t *__restrict__ a2,
    const uint16_t *__restrict__ b2, const uint32_t *__restrict__ flags, void *__restrict__ y, int64_t M, int64_t K, int64_t N,
    int KP, int nbn, int lg_xm) {
    using G = Geo<WM, WN, TM, TN, BITS>;
    constexpr int BM = G::BM, BN = G::BN, STAGE_BYTES = G::STAGE_BYTES, A_BYTES = G::A_BYTES, A2S_BYTES = G::A2S_BYTES;
    constexpr int LA = G::LA, LB = G::LB, L2 = G::L2;
    constexpr int RA = G::RA, RI = G::RI, RL = G::RL, RSTAGE = G::STAGE;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    int tm, tn;
    if (lg_xm < 0) {
        tm = (int)blockIdx.x / nbn;
        tn = (int)blockIdx.x % nbn;
    } else {
        // XCD-aware order: workgroups go to the 8 XCDs round-robin by linear index; the 32 an XCD runs at a
        // time form a compact 4 x 8 patch of tiles and the 8 patches of a round a compact region
        const int region = (int)blockIdx.x >> 8, r = (int)blockIdx.x & 255;
        const int xcd = r & 7, q = r >> 3;
        const int xn = 8 >> lg_xm;
        const int regions_n = nbn / (8 * xn);
        tm = (region / regions_n) * (4 << lg_xm) + (xcd / xn) * 4 + (q >> 3);
        tn = (region % regions_n) * 8 * xn + (xcd % xn) * 8 + (q & 7);
    }
    const int64_t n0 = (int64_t)tn * BN;
    const int64_t m0 = (int64_t)tm * BM;
    {
        const int f0 = (int)(n0 / 32), nf = (int)((N + 31) / 32);
        uint32_t fl = 0;
#pragma unroll
        for (int i = 0; i < BN / 32; ++i) fl |= f0 + i < nf ? flags[f0 + i] : 0u;
        if (fl != 0) return;
    }
    const int groups = (int)(K / kGroup);
    const int stages = groups * 2;

    // ---- activations: wave v fills rows [8 RA v, 8 RA (v + 1)) of a stage, 8 rows of 128 bytes per instruction
    const uint16_t *ga[RA];
#pragma unroll
    for (int i = 0; i < RA; ++i) {
        const int row = wave * 8 * RA + i * 8 + (lane >> 3);
        const int chunk = (lane & 7) ^ ((row >> 1) & 7);
        const int64_t m = m0 + row < M ? m0 + row : M - 1;
        ga[i] = x + m * K + chunk * 8;
    }
    // ---- codes: per instruction two row tiles, lanes [32 v, 32 v + 32) of their block (k steps 2 v and 2 v + 1)
    const int64_t tiles_n = N / kTileRows;
    int64_t unit0[RI];
#pragma unroll
    for (int i = 0; i < RI; ++i) {
        int64_t wT = n0 / kTileRows + (G::PRIVATE_CODES ? wn * 2 * TN + 2 * i : 2 * wave) + (lane >> 5);
        if (wT >= tiles_n) wT = tiles_n - 1;
        unit0[i] = wT * groups * 64 + (lane & 31);
    }
    int at = 0;                  // the stage the activation pointers stand at
    auto issue_stage = [&](int t, int off) {
        const int target = t < stages ? t : stages - 1;        // past the end: the last stage again, never read
        const int adv = (target - at) * BK2;
        at = target;
#pragma unroll
        for (int i = 0; i < RA; ++i) {
            ga[i] += adv;
            __builtin_amdgcn_global_load_lds((global_void *)ga[i], (lds_void *)(lds + off + (wave * 8 * RA + i * 8) * ROW2), 16, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < RI; ++i) {
            const int64_t unit = unit0[i] + (int64_t)(target >> 1) * 64 + (target & 1) * 32;
            lds_void *dst = (lds_void *)(lds + off + A2S_BYTES + (wave * RI + i) * 1024);
            if constexpr (BITS == 4)
                __builtin_amdgcn_global_load_lds((global_void *)(reinterpret_cast<const uint4 *>(wt) + unit), dst, 16, 0, 0);
            else   // 12 bytes per unit, fetched as 16
                __builtin_amdgcn_global_load_lds((global_void *)(reinterpret_cast<const uint32_t *>(wt) + unit * 3), dst, 16, 0, 0);
        }
    };
    // ---- factors of the wave's 64 columns (lane = column), slot g + 1 of the table: s[g] / s[g + 1]
    constexpr bool RESCALE = !PC;
    const float *fptr;
    {
        int64_t n = n0 + wn * 32 * TN + lane;
        if (n >= N) n = N - 1;
        fptr = rfac + ((n / kTileRows) * (groups + 1)) * kTileRows + (n % kTileRows);
    }
    auto issue_factors = [&](int slot) {
        __builtin_amdgcn_global_load_lds((global_void *)(fptr + (int64_t)slot * kTileRows), (lds_void *)(lds + G::FAC_OFF + wave * 256), 4,
                                         0, 0);
    };

    // ---- what a lane reads back: its fragment addresses within a stage
    const int arow = wm * 32 * TM + (lane & 31);
    const int abase = arow * ROW2 + (((4 * (lane >> 5)) ^ ((lane >> 1) & 7)) * 16);    // MFMA round w: abase ^ (16 w)
    const int rbase = A2S_BYTES + ((G::PRIVATE_CODES ? wave : wn) * 2 * TN + ((lane & 31) >> 4)) * 512 + (lane >> 5) * 256 + (lane & 15) * 16;
    auto read_a = [&](int off, int w, Frag (&a)[TM]) { const uint8_t *p = lds + off + (abase ^ (w << 4));
        read_a_frags<TM>(p, p + (TM / 2) * 32 * ROW2, a); };
    auto read_raw = [&](int off, u32x4_t (&rw)[TN]) { read_code_units<TN>(lds + off + rbase, lds + off + rbase + (TN == 2 ? 1024 : 8), rw); };
    auto unpack_b = [&](const u32x4_t (&rw)[TN], int w, Frag (&b)[TN]) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if constexpr (BITS == 4)
                unpack4_word(rw[j][w], b[j]);
            else
                unpack3_chunk(rw[j], w, b[j]);
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
    constexpr int TILES = TM * TN;
    static_assert(TILES == 8 || TILES == 4 || TILES == 2, "the schedules below are written for 8, 4 or 2 tiles per wave");
    static_assert(TILES == 8 ? TN == 2 : true, "the 8-tile schedule pairs the halves of a tile row");
    auto mul_half = [&](int t, int h, const float (&f)[TN]) {
        const int i = t / TN, j = t % TN;
#pragma unroll
        for (int r = 0; r < 8; ++r) acc[i][j][8 * h + r] *= f[j];
    };
    auto mfma_tile = [&](int t, const Frag (&a)[TM], const Frag (&b)[TN]) {
        const int i = t / TN, j = t % TN;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i].v, b[j].v, acc[i][j], 0, 0, 0);
    };
    // an MFMA round with the next round's fragment reads and unpack spread between its MFMAs
    auto round_plain = [&](const Frag (&a)[TM], const Frag (&b)[TN]) {
        mfma_all(a, b, acc);
#pragma unroll
        for (int t = 0; t < TILES; ++t) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, TILES == 8 ? 3 : (TILES == 4 ? 5 : 9), 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
    };

    // ---- prologue
    int off_c = 0, off_n = RSTAGE, off_nn = 2 * RSTAGE;
    issue_stage(0, off_c);
    issue_stage(1, off_n);
    issue_stage(2, off_nn);
    wait_vmcnt<2 * RL>();
    bare_barrier();
    u32x4_t rw[TN];
    Frag fa[2][TM], fb[2][TN];
    read_raw(off_c, rw);
    read_a(off_c, 0, fa[0]);
    unpack_b(rw, 0, fb[0]);
    float rf[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) rf[j] = 1.f;
    const int fcol = G::FAC_OFF + wave * 256 + (lane & 31) * 4;

    for (int g = 0; g < groups; ++g) {
#pragma unroll
        for (int v = 0; v < 2; ++v) {
            const int t = 2 * g + v;
            // round 0
            read_a(off_c, 1, fa[1]);
            unpack_b(rw, 1, fb[1]);
            if (v == 0 && RESCALE && TILES == 2) {
                // the second tile into the units of this group, ahead of its first MFMA
                mfma_tile(0, fa[0], fb[0]);
                __builtin_amdgcn_sched_barrier(0);
                mul_half(1, 0, rf);
                mul_half(1, 1, rf);
                mfma_tile(1, fa[0], fb[0]);
            } else if (v == 0 && RESCALE && TILES == 4) {
                // the second half of the tiles into the units of this group, ahead of their first MFMA
                mfma_tile(0, fa[0], fb[0]);
                __builtin_amdgcn_sched_barrier(0);
                mul_half(2, 0, rf);
                mul_half(2, 1, rf);
                mfma_tile(1, fa[0], fb[0]);
                __builtin_amdgcn_sched_barrier(0);
                mul_half(3, 0, rf);
                mul_half(3, 1, rf);
                mfma_tile(2, fa[0], fb[0]);
                mfma_tile(3, fa[0], fb[0]);
            } else if (v == 0 && RESCALE) {
                // tiles 4..7 into the units of this group, ahead of their first MFMA (factor 1 in the first group)
                mfma_tile(0, fa[0], fb[0]);
                mul_half(4, 0, rf);
                mfma_tile(1, fa[0], fb[0]);
                mul_half(4, 1, rf);
                mfma_tile(2, fa[0], fb[0]);
                mul_half(5, 0, rf);
                mfma_tile(3, fa[0], fb[0]);
                mul_half(5, 1, rf);
                mul_half(6, 0, rf);
                mfma_tile(4, fa[0], fb[0]);
                mul_half(6, 1, rf);
                mul_half(7, 0, rf);
                mfma_tile(5, fa[0], fb[0]);
                mul_half(7, 1, rf);
                mfma_tile(6, fa[0], fb[0]);
                mfma_tile(7, fa[0], fb[0]);
#pragma unroll
                for (int q = 0; q < 3; ++q) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 11, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 19, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 19, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 11, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            } else {
                round_plain(fa[0], fb[0]);
            }
            __builtin_amdgcn_sched_barrier(0);
            // round 1
            read_a(off_c, 2, fa[0]);
            unpack_b(rw, 2, fb[0]);
            round_plain(fa[1], fb[1]);
            __builtin_amdgcn_sched_barrier(0);
            // round 2
            read_a(off_c, 3, fa[1]);
            unpack_b(rw, 3, fb[1]);
            round_plain(fa[0], fb[0]);
            __builtin_amdgcn_sched_barrier(0);
            // stage t + 1 has landed (and, in the second half of a group, the factors to the next group); every wave
            // has read its last fragments of stage t
            wait_vmcnt<RL>();
            if (v == 1 && RESCALE) read_wave_factors<TN>(lds + fcol, lds + fcol + 128, rf);   // the wave's own slot: no barrier needed
            bare_barrier();
            // round 3 starts at once; the requests for stage t + 3 and the first reads of stage t + 1 go between its MFMAs
            mfma_tile(0, fa[1], fb[1]);
            __builtin_amdgcn_sched_barrier(0);
            if (v == 0 && RESCALE) issue_factors(g + 1);
            issue_stage(t + 3, off_c);
            __builtin_amdgcn_sched_barrier(0);
            mfma_tile(1, fa[1], fb[1]);
            __builtin_amdgcn_sched_barrier(0);
            read_raw(off_n, rw);
            read_a(off_n, 0, fa[0]);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (TILES > 2) mfma_tile(2, fa[1], fb[1]);
            if (v == 1 && RESCALE && TILES == 2) {
                // the first tile into the units of the next group, behind its last MFMA
                __builtin_amdgcn_sched_barrier(0);
                mul_half(0, 0, rf);
                mul_half(0, 1, rf);
                unpack_b(rw, 0, fb[0]);
            } else if (v == 1 && RESCALE && TILES == 4) {
                // the first half of the tiles into the units of the next group, behind their last MFMA
                __builtin_amdgcn_sched_barrier(0);
                mul_half(0, 0, rf);
                mul_half(0, 1, rf);
                mfma_tile(3, fa[1], fb[1]);
                __builtin_amdgcn_sched_barrier(0);
                mul_half(1, 0, rf);
                mul_half(1, 1, rf);
                unpack_b(rw, 0, fb[0]);
            } else if (v == 1 && RESCALE) {
                // tiles 0..3 into the units of the next group, behind their last MFMA
                __builtin_amdgcn_sched_barrier(0);
                mul_half(0, 0, rf);
                mfma_tile(3, fa[1], fb[1]);
                __builtin_amdgcn_sched_barrier(0);
                mul_half(0, 1, rf);
                mfma_tile(4, fa[1], fb[1]);
                __builtin_amdgcn_sched_barrier(0);
                mul_half(1, 0, rf);
                mfma_tile(5, fa[1], fb[1]);
                __builtin_amdgcn_sched_barrier(0);
                mul_half(1, 1, rf);
                mfma_tile(6, fa[1], fb[1]);
                __builtin_amdgcn_sched_barrier(0);
                mul_half(2, 0, rf);
                mfma_tile(7, fa[1], fb[1]);
                __builtin_amdgcn_sched_barrier(0);
                mul_half(2, 1, rf);
                mul_half(3, 0, rf);
                mul_half(3, 1, rf);
                unpack_b(rw, 0, fb[0]);
            } else {
                __builtin_amdgcn_sched_barrier(0);
                unpack_b(rw, 0, fb[0]);
#pragma unroll
                for (int q = 3; q < TILES; ++q) mfma_tile(q, fa[1], fb[1]);
#pragma unroll
                for (int q = 3; q < TILES; ++q) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            const int o = off_c;
            off_c = off_n;
            off_n = off_nn;
            off_nn = o;
        }
    }
    wait_vmcnt<0>();
    bare_barrier();

    const int scol = wn * 32 * TN + (lane & 31);
    {
        float sl[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            int64_t n = n0 + scol + j * 32;
            if (n >= N) n = N - 1;
            sl[j] = 2.f * rfac[((n / kTileRows) * (groups + 1)) * kTileRows + (n % kTileRows)];   // the operands were (16 + q) / 2
        }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] *= sl[j];
    }

    // ---- second loop: the zero-point term, bf16 operands A2[m][.] and B2[n][.] over KP columns, both direct-to-LDS in
    // stages of 32 k; wave v fills rows [16 LA v, ..) of A2's stage half and rows [16 LB v, ..) of B2's
    {
        const int steps2 = KP / BK;
        const uint16_t *gp[L2];
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            const int row = wave * 16 * LA + i * 16 + (lane >> 2);
            const int64_t m = m0 + row < M ? m0 + row : M - 1;
            gp[i] = a2 + m * KP + swz(row, lane & 3) * 8;
        }
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            const int row = wave * 16 * LB + i * 16 + (lane >> 2);
            const int64_t n = n0 + row < N ? n0 + row : N - 1;
            gp[LA + i] = b2 + n * KP + swz(row, lane & 3) * 8;
        }
        int at2 = 0;
        auto issue2 = [&](int step, int stage_idx) {
            uint8_t *stage = lds + stage_idx * STAGE_BYTES;
            const int target = step < steps2 ? step : steps2 - 1;
            const int adv = (target - at2) * BK;
            at2 = target;
#pragma unroll
            for (int i = 0; i < LA; ++i) {
                gp[i] += adv;
                __builtin_amdgcn_global_load_lds((global_void *)gp[i], (lds_void *)(stage + (wave * 16 * LA + i * 16) * ROW_BYTES),
                                                 16, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < LB; ++i) {
                gp[LA + i] += adv;
                __builtin_amdgcn_global_load_lds((global_void *)gp[LA + i],
                                                 (lds_void *)(stage + A_BYTES + (wave * 16 * LB + i * 16) * ROW_BYTES), 16, 0, 0);
            }
        };
#pragma unroll
        for (int j = 0; j < 4; ++j) issue2(j, j);
        wait_vmcnt<3 * L2>();
        bare_barrier();
        load_frags(lds, lds + A_BYTES, 0, fa[0], fb[0], lane, wm, wn);
        for (int kt = 0; kt < steps2; ++kt) {
            const uint8_t *cur = lds + (kt & 3) * STAGE_BYTES;
            const bool more = kt + 1 < steps2;
            load_frags(cur, cur + A_BYTES, 1, fa[1], fb[1], lane, wm, wn);
            __builtin_amdgcn_sched_barrier(0);
            mfma_all(fa[0], fb[0], acc);
            __builtin_amdgcn_sched_barrier(0);
            if (more) {
                wait_vmcnt<2 * L2>();
                bare_barrier();
                const uint8_t *nxt = lds + ((kt + 1) & 3) * STAGE_BYTES;
                load_frags(nxt, nxt + A_BYTES, 0, fa[0], fb[0], lane, wm, wn);
                __builtin_amdgcn_sched_barrier(0);
                issue2(kt + 4, kt & 3);
            }
            __builtin_amdgcn_sched_barrier(0);
            mfma_all(fa[1], fb[1], acc);
            __builtin_amdgcn_sched_barrier(0);
        }
        wait_vmcnt<0>();
    }

#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int64_t n = n0 + wn * 32 * TN + j * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t m = m0 + wm * 32 * TM + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (m < M && n < N) {
                    if (OUT_F32)
                        reinterpret_cast<float *>(y)[m * N + n] = acc[i][j][r];
                    else
                        reinterpret_cast<uint16_t *>(y)[m * N + n] = f32_to_bf16(acc[i][j][r]);
                }
            }
        }
}

// ---- pre-pass, activations ----------------------------------------------------------------------------------------
// One wave per activation row; the fp32 sum X of each group of 128 activations (8 per lane in k order, then the 16
// lanes of the group in a fixed rotate-and-add order), split into three bf16 terms X = X0 + X1 + X2, written to
// A2[m][(2 i + j) G_n + G] = X_i for j = 0, 1.  Columns [6 G_n, KP) are written as zeros (the workspace arrives
// uninitialised).
__device__ __forceinline__ void xsum_block(int block, const uint16_t *__restrict__ x, uint16_t *__restrict__ a2, int64_t M, int64_t K,
                                           int KP) {
    const int groups = (int)(K / kGroup);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t m = (int64_t)block * 4 + wave;
    if (m >= M) return;
    const uint16_t *xr = x + m * K;
    uint16_t *out = a2 + m * KP;
    for (int g0 = 0; g0 < groups; g0 += 32) {              // 8 loads of 1 KiB (4 groups each) in flight per wave
        uint4 v[8];
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const int g = g0 + 4 * b + (lane >> 4);
            v[b] = g < groups ? *reinterpret_cast<const uint4 *>(xr + (int64_t)g * kGroup + (lane & 15) * 8) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const int g = g0 + 4 * b + (lane >> 4);
            const uint32_t w[4] = {v[b].x, v[b].y, v[b].z, v[b].w};
            float sum = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                sum += __uint_as_float(w[i] << 16);
                sum += __uint_as_float(w[i] & 0xFFFF0000u);
            }
            sum = row16_sum(sum);
            if (g < groups && (lane & 15) == 0) {
                const uint16_t t0 = f32_to_bf16(sum);
                const float r1 = sum - bf16_bits_to_f32(t0);
                const uint16_t t1 = f32_to_bf16(r1);
                const uint16_t t2 = f32_to_bf16(r1 - bf16_bits_to_f32(t1));
                const uint16_t t[3] = {t0, t1, t2};
#pragma unroll
                for (int i = 0; i < 3; ++i) {
                    out[(2 * i) * groups + g] = t[i];
                    out[(2 * i + 1) * groups + g] = t[i];
                }
            }
        }
    }
    for (int c = 6 * groups + lane; c < KP; c += 64) out[c] = 0;
}

// ---- pre-pass, weights ---------------------------------------------------------------------------------------------
// A block takes 32 weight rows (two row tiles).  The scale / zero words go through LDS in chunks of 32 groups (read
// in their own order, written out row by row); c = -s (16 + z) (exact in fp32: two 8-bit significands) is split into
// two bf16 terms, B2[n][(2 i + j) G_n + G] = c_j for i = 0..2; the rescale factors; and the block's flag: set when
// a scale is zero, subnormal or not finite, or further than 2^20 from the row's first.  Columns [6 G_n, KP) of B2
// are written as zeros.
constexpr int PRE_CHUNK = 32, PRE_ROWS = 32;

__device__ __forceinline__ float scale_of(uint32_t szw) { return __uint_as_float(szw << 16); }

// One launch does both parts; the blocks of this part come first in the grid (there are few of them and each runs
// longer than a block of the activation part, which fills the rest of the chip meanwhile).
__global__ __launch_bounds__(256) void gemm_w4_rescale_prepass_kernel(const uint16_t *__restrict__ x, const uint32_t *__restrict__ sz,
                                                                      int szs, uint16_t *__restrict__ a2, uint16_t *__restrict__ b2,
                                                                      float *__restrict__ rfac, uint32_t *__restrict__ flags, int64_t M,
                                                                      int64_t K, int64_t N, int KP, int nblocks) {
    if ((int)blockIdx.x >= nblocks) {
        xsum_block((int)blockIdx.x - nblocks, x, a2, M, K, KP);
        return;
    }
    const int groups = (int)(K / kGroup);
    const int tid = threadIdx.x;
    __shared__ uint32_t w_sh[PRE_ROWS][PRE_CHUNK + 1];          // scale / zero word of (row, group within the chunk)
    __shared__ float prev_sh[PRE_ROWS], first_sh[PRE_ROWS];     // scale of the group before the chunk; |first scale| of the row
    const int64_t nbase = (int64_t)blockIdx.x * PRE_ROWS;
    int bad = 0;
    for (int g0 = 0; g0 < groups; g0 += PRE_CHUNK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {                  // in the order of the words: tile, group, row of the tile
            const int idx = tid + 256 * i;
            const int tile = idx >> 9, gl = (idx >> 4) & 31, j = idx & 15;
            const int64_t n = nbase + tile * 16 + j;
            const int g = g0 + gl;
            w_sh[tile * 16 + j][gl] = (n < N && g < groups) ? sz[sz_index(n / kTileRows, g, groups, szs, j)] : 0x3F80u;
        }
        __syncthreads();
        if (g0 == 0) {
            if (tid < PRE_ROWS) first_sh[tid] = fabsf(scale_of(w_sh[tid][0]));
            __syncthreads();
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {                  // row by row: B2 and the checks
            const int idx = tid + 256 * i;
            const int row = idx >> 5, gl = idx & 31;
            const int64_t n = nbase + row;
            const int g = g0 + gl;
            if (n < N && g < groups) {
                const uint32_t szw = w_sh[row][gl];
                const float s = scale_of(szw);
                const float c = s * (__uint_as_float(szw & 0xFFFF0000u) + 112.f);      // -(16 + z) s
                const uint16_t c0 = f32_to_bf16(c);
                const uint16_t c1 = f32_to_bf16(c - bf16_bits_to_f32(c0));
                uint16_t *out = b2 + n * KP + g;
#pragma unroll
                for (int t = 0; t < 3; ++t) {
                    out[(2 * t) * groups] = c0;
                    out[(2 * t + 1) * groups] = c1;
                }
                const uint32_t ex = (szw >> 7) & 0xFFu;                                  // exponent field of the bf16 scale
                const float as = fabsf(s), f = first_sh[row];
                bad |= (ex == 0 || ex == 255) || !(as <= f * 1048576.f) || !(f <= as * 1048576.f);
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {                  // in the order of the words again: the factors
            const int idx = tid + 256 * i;
            const int tile = idx >> 9, gl = (idx >> 4) & 31, j = idx & 15;
            const int row = tile * 16 + j;
            const int64_t n = nbase + row;
            const int g = g0 + gl;
            if (n < N && g < groups && g > 0) {
                const float sp = gl > 0 ? scale_of(w_sh[row][gl - 1]) : prev_sh[row];
                rfac[((n / kTileRows) * (groups + 1) + g) * kTileRows + j] = sp / scale_of(w_sh[row][gl]);
            }
        }
        __syncthreads();
        const int last = groups - g0 < PRE_CHUNK ? groups - g0 - 1 : PRE_CHUNK - 1;
        if (tid < PRE_ROWS) prev_sh[tid] = scale_of(w_sh[tid][last]);
        __syncthreads();
    }
    if (tid < PRE_ROWS && nbase + tid < N) {
        const int64_t n = nbase + tid;
        float *f = rfac + ((n / kTileRows) * (groups + 1)) * kTileRows + (n % kTileRows);
        f[0] = prev_sh[tid];                           // the last scale
        f[(int64_t)groups * kTileRows] = 1.f;
    }
    for (int idx = tid; idx < PRE_ROWS * 32; idx += 256) {
        const int row = idx >> 5, c = 6 * groups + (idx & 31);
        if (nbase + row < N && c < KP) b2[(nbase + row) * KP + c] = 0;
    }
    bad = __syncthreads_or(bad);
    if (tid == 0) flags[blockIdx.x] = (uint32_t)bad;
}

struct RescalePlan {
    int KP;
    size_t off_a2, off_b2, off_r, off_flags, total;
};

RescalePlan plan_rescale(int64_t M, int64_t K, int64_t N) {
    RescalePlan p;
    const int64_t groups = K / kGroup;
    p.KP = (int)((6 * groups + BK - 1) / BK * BK);
    auto up = [](size_t v) { return (v + 255) / 256 * 256; };
    p.off_a2 = 0;
    p.off_b2 = up((size_t)M * p.KP * 2);
    p.off_r = p.off_b2 + up((size_t)N * p.KP * 2);
    p.off_flags = p.off_r + up((size_t)N * (groups + 1) * 4);
    p.total = p.off_flags + up((size_t)((N + 31) / 32) * 4);
    return p;
}


struct Operands {       // what the pre-pass leaves in the workspace
    const uint16_t *a2, *b2;
    const float *rfac;
    const uint32_t *flags;
};

template <int WM, int WN, int TM, int TN, int BITS>
hipError_t launch_tile(const void *wt, bool pc, const uint16_t *x, int64_t M, int64_t K, int64_t N, void *y, bool out_f32,
                       const RescalePlan &p, const Operands &o, hipStream_t stream) {
    using G = Geo<WM, WN, TM, TN, BITS>;
    const int nbm = (int)((M + G::BM - 1) / G::BM), nbn = (int)((N + G::BN - 1) / G::BN);
    // XCD-aware tile order when the grid of tiles divides into regions of 8 patches of 4 x 8 tiles (see the kernel)
    int lg_xm = 2;
    while (lg_xm >= 0 && (nbm % (4 << lg_xm) != 0 || nbn % (8 * (8 >> lg_xm)) != 0)) --lg_xm;
    auto go = [&](auto kernel) {
        hipError_t st = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                            (int)G::LDS_BYTES);
        if (st != hipSuccess) return st;
        hipLaunchKernelGGL(kernel, dim3((unsigned)(nbm * nbn)), dim3(G::THREADS), G::LDS_BYTES, stream, wt, o.rfac, x, o.a2, o.b2,
                           o.flags, y, M, K, N, p.KP, nbn, lg_xm);
        return hipGetLastError();
    };
    if constexpr (BITS == 4) {
        if (pc)
            return out_f32 ? go(&gemm_w4_rescale_kernel<WM, WN, TM, TN, 4, true, true>)
                           : go(&gemm_w4_rescale_kernel<WM, WN, TM, TN, 4, false, true>);
    }
    return out_f32 ? go(&gemm_w4_rescale_kernel<WM, WN, TM, TN, BITS, true, false>)
                   : go(&gemm_w4_rescale_kernel<WM, WN, TM, TN, BITS, false, false>);
}

// Pre-pass, then the rescaling kernel; the caller launches the 128 x 128 exact kernel behind them for the column blocks
// the pre-pass flagged (normally none: its workgroups then return at once).
template <int BITS>
hipError_t launch_rescale(const void *wt, const uint32_t *sz, int szs, int64_t K, int64_t N, const uint16_t *x, int64_t M, void *y,
                          bool out_f32, void *ws, const uint32_t **flags_out, bool *pairs_out, hipStream_t stream) {
    const RescalePlan p = plan_rescale(M, K, N);
    uint8_t *base = reinterpret_cast<uint8_t *>(ws);
    uint16_t *a2 = reinterpret_cast<uint16_t *>(base + p.off_a2);
    uint16_t *b2 = reinterpret_cast<uint16_t *>(base + p.off_b2);
    float *rfac = reinterpret_cast<float *>(base + p.off_r);
    uint32_t *flags = reinterpret_cast<uint32_t *>(base + p.off_flags);
    const int nblocks = (int)((N + PRE_ROWS - 1) / PRE_ROWS), mblocks = (int)((M + 3) / 4);
    hipLaunchKernelGGL(gemm_w4_rescale_prepass_kernel, dim3((unsigned)(nblocks + mblocks)), dim3(256), 0, stream, x, sz, szs, a2, b2,
                       rfac, flags, M, K, N, p.KP, nblocks);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int wn = w4_gemm_rescale_tile_rows(M, N) == 128 ? 2 : w4_gemm_rescale_wave_columns(M, N);
    const Operands o{a2, b2, rfac, flags};
    *flags_out = flags;
    *pairs_out = wn == 4;
    if (wn == 4) return launch_tile<2, 4, 4, 2, BITS>(wt, szs == 0, x, M, K, N, y, out_f32, p, o, stream);
    if (w4_gemm_rescale_tile_rows(M, N) == 128) return launch_tile<2, 4, 2, 1, BITS>(wt, szs == 0, x, M, K, N, y, out_f32, p, o, stream);
    // 256 x 128 tiles: eight waves of 128 x 32 (measured 0-8 % ahead of four waves of 128 x 64 and of eight of 64 x 64)
    return launch_tile<2, 4, 4, 1, BITS>(wt, szs == 0, x, M, K, N, y, out_f32, p, o, stream);
}

}  // namespace

// Measured against the 128 x 128 exact kernel: ahead wherever the tiled path is dispatched, also with a row tile that
// is only half full (gate+up at 144 .. 240 rows: 93-96 against 101 us).
bool w4_gemm_rescale_applies(int64_t M, int64_t N) {
    const int64_t wgs = ((M + kMaxBM - 1) / kMaxBM) * ((N + 127) / 128);
    return M > env_int("DMR_W4_RESCALE_MIN_M", kMaxBM / 2) && wgs <= 0x3FFFFFFF;
}

// (The rules hold for 3-bit layers as well: same tiles, same pipeline.)
// Wave columns of the tile.  Either tile's LDS use leaves one workgroup per CU, so a launch runs in rounds of 256
// tiles; a round of 256 x 256 tiles (8 waves) takes about 1.5 times a round of 256 x 128 tiles (4 waves).  One round
// of the narrow tiles is therefore the fastest where it covers the layer, and from there on the wide tiles, which
// need half the rounds (measured on K = 4096: 288 narrow tiles 159 us against 144 wide ones 132 us; 256 narrow tiles
// 90 us against 128 wide ones 125 us; level at 576 against 288).
int w4_gemm_rescale_wave_columns(int64_t M, int64_t N) {
    const int forced = env_int("DMR_W4_RESCALE_WN", 0);
    if (forced == 2 || forced == 4) return forced;
    const int64_t narrow = ((M + kMaxBM - 1) / kMaxBM) * ((N + 127) / 128);
    return narrow > compute_units() ? 4 : 2;
}

// Rows of the tile: 128 while one round of 128 x 128 tiles (eight waves of 64 x 32, up to two workgroups per CU) covers
// the output; measured there against the rollout-batch kernel and the 256-row tiles: attn-out at 768 / 1024 rows 48 / 52
// against 55 / 64 us, qkv at 384 / 512 rows 49 / 50 against 55 / 55, down at 768 / 1024 rows 146 / 152 against 173 / 191;
// behind both from 288 blocks on.
int w4_gemm_rescale_tile_rows(int64_t M, int64_t N) {
    const int forced = env_int("DMR_W4_RESCALE_BM", 0);
    if (forced == 128 || forced == 256) return forced;
    const int64_t blocks = ((M + 127) / 128) * ((N + 127) / 128);
    return blocks <= compute_units() ? 128 : 256;
}

size_t w4_gemm_rescale_workspace_bytes(int64_t M, int64_t K, int64_t N) { return plan_rescale(M, K, N).total; }

hipError_t launch_w4_gemm_rescale(const LayerView &Lv, const uint16_t *x, int64_t M, void *y, bool out_f32, void *ws,
                                  hipStream_t stream) {
    const uint32_t *flags = nullptr;
    bool pairs = false;
    const hipError_t e = launch_rescale<4>(Lv.wt, Lv.sz, Lv.szs, Lv.K, Lv.N, x, M, y, out_f32, ws, &flags, &pairs, stream);
    if (e != hipSuccess) return e;
    return launch_w4_gemm_flagged(Lv, x, M, y, out_f32, flags, pairs, stream);
}

hipError_t launch_w3_gemm_rescale(const LayerView3 &Lv, const uint16_t *x, int64_t M, void *y, bool out_f32, void *ws,
                                  hipStream_t stream) {
    const uint32_t *flags = nullptr;
    bool pairs = false;
    const hipError_t e = launch_rescale<3>(Lv.wt, Lv.sz, 1, Lv.K, Lv.N, x, M, y, out_f32, ws, &flags, &pairs, stream);
    if (e != hipSuccess) return e;
    return launch_w3_gemm_flagged(Lv, x, M, y, out_f32, flags, pairs, stream);
}

}  // namespace dmr

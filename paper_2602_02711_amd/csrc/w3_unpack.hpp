// Register unpack of the 3-bit streaming layout (see w3_layout_kernels.hip for the layout), shared by
// the W3A16 kernels.
#pragma once
#include "common.hpp"

namespace dmr {

// The 16 operand registers of a lane's three words (no inline assembly: the wait states an MFMA
// needs after a VALU write of its operands are only inserted for compiler-emitted instructions).
__device__ __forceinline__ void unpack3(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t (&r)[16]) {
    const uint32_t m7 = 0x07070707u, exp = 0x43434343u;
    const uint32_t sel_a = 0x00060004u, sel_b = 0x00070005u;     // bytes (0, 2) resp. (1, 3) of the codes
    const uint32_t w[3] = {w0, w1, w2};
#pragma unroll
    for (int v = 0; v < 3; ++v) {
        const uint32_t f0 = w[v] & m7, f1 = (w[v] >> 3) & m7;
        r[4 * v + 0] = __builtin_amdgcn_perm(f0, exp, sel_a);
        r[4 * v + 1] = __builtin_amdgcn_perm(f0, exp, sel_b);
        r[4 * v + 2] = __builtin_amdgcn_perm(f1, exp, sel_a);
        r[4 * v + 3] = __builtin_amdgcn_perm(f1, exp, sel_b);
    }
    const uint32_t c0 = (((w2 >> 6) & 0x01010101u) << 2) | ((w0 >> 6) & 0x03030303u);
    const uint32_t c1 = (((w2 >> 7) & 0x01010101u) << 2) | ((w1 >> 6) & 0x03030303u);
    r[12] = __builtin_amdgcn_perm(c0, exp, sel_a);
    r[13] = __builtin_amdgcn_perm(c0, exp, sel_b);
    r[14] = __builtin_amdgcn_perm(c1, exp, sel_a);
    r[15] = __builtin_amdgcn_perm(c1, exp, sel_b);
}

// The four operand registers of k step T (0..3) alone, for kernels that cannot hold all 16 at once: steps
// 0..2 come from word T, step 3 gathers the third bits and the top two bits of the three words.
template <int T>
__device__ __forceinline__ void unpack3_step(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t (&r)[4]) {
    const uint32_t m7 = 0x07070707u, exp = 0x43434343u;
    const uint32_t sel_a = 0x00060004u, sel_b = 0x00070005u;
    if constexpr (T < 3) {
        const uint32_t w = T == 0 ? w0 : T == 1 ? w1 : w2;
        const uint32_t f0 = w & m7, f1 = (w >> 3) & m7;
        r[0] = __builtin_amdgcn_perm(f0, exp, sel_a);
        r[1] = __builtin_amdgcn_perm(f0, exp, sel_b);
        r[2] = __builtin_amdgcn_perm(f1, exp, sel_a);
        r[3] = __builtin_amdgcn_perm(f1, exp, sel_b);
    } else {
        const uint32_t c0 = (((w2 >> 6) & 0x01010101u) << 2) | ((w0 >> 6) & 0x03030303u);
        const uint32_t c1 = (((w2 >> 7) & 0x01010101u) << 2) | ((w1 >> 6) & 0x03030303u);
        r[0] = __builtin_amdgcn_perm(c0, exp, sel_a);
        r[1] = __builtin_amdgcn_perm(c0, exp, sel_b);
        r[2] = __builtin_amdgcn_perm(c1, exp, sel_a);
        r[3] = __builtin_amdgcn_perm(c1, exp, sel_b);
    }
}

}  // namespace dmr

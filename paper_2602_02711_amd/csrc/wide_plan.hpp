// Launch planning of the wide-layer kernel (w4_wide.hip): pure host arithmetic for 256 CUs.
#pragma once
#include "common.hpp"

namespace dmr {

struct WidePlan {
    bool ok;
    int MT;    // row tiles of 16
};

constexpr int kWideChunk = 4;       // groups per LDS panel
constexpr int kWideTilesPerWg = 8;  // 4 tile lanes x 2 tiles per wave

inline size_t wide_lds_bytes(int MT, int R, int S, int CG) {
    const size_t panels = 2 * (size_t)(MT * 16) * (CG * 16 + 1) * 16 + 2 * (size_t)CG * MT * 4 * 16;
    const size_t red = S > 1 ? (size_t)8 * R * MT * 1024 : 0;
    return panels > red ? panels : red;
}

// 17 <= M <= 64 on layers with at least 128 workgroups' worth of tiles (measured against the
// rollout-batch kernel, which wins on narrower layers by splitting K).
inline WidePlan plan_wide(int64_t M, int64_t K, int64_t N) {
    WidePlan p{};
    p.ok = false;
    if (M < 17 || M > 64 || M * K >= (int64_t(1) << 31)) return p;
    const int64_t groups = K / kGroup, tiles = N / kTileRows;
    if (groups % kWideChunk != 0 || tiles < 128 * kWideTilesPerWg) return p;
    p.MT = (int)((M + 15) / 16);
    p.ok = true;
    return p;
}

bool w4_wide_applies(int64_t M, int64_t K, int64_t N);
hipError_t launch_w4_wide(const LayerView &L, const uint16_t *x, int64_t M, void *y, bool out_f32,
                          hipStream_t stream);
// The same kernel on a 3-bit layer.
hipError_t launch_w3_wide(const LayerView3 &L, const uint16_t *x, int64_t M, void *y, bool out_f32,
                          hipStream_t stream);

}  // namespace dmr

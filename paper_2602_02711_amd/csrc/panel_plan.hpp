// Launch planning of the panel kernel (w4_panel.hip): pure host arithmetic for 256 CUs and 160 KB of
// LDS, so that the workspace query agrees with the launch.
#pragma once
#include "mid_plan.hpp"

namespace dmr {

struct PanelPlan {
    bool ok;
    int MT;       // row tiles of 16
    int R;        // weight tiles per wave
    int WAVES;    // wavefronts per workgroup
    int S;        // sub-slices of the k slice inside a workgroup (power of two)
    int SK;       // k slices over blockIdx.y (divides the group count)
    int gq;       // groups per k slice
    size_t lds;   // dynamic LDS bytes
};

inline size_t panel_lds_bytes(int64_t M, int MT, int R, int WAVES, int S, int gq) {
    const size_t panel = (size_t)M * (gq * 16 + 1) * 16 + (size_t)gq * MT * 4 * 16;
    const size_t red = S > 1 ? (size_t)WAVES * R * MT * 1024 : 0;
    return panel > red ? panel : red;
}

// Measured on MI355X (K = 14336, M = 8 and 16; sweep over R, WAVES, S, SK): one tile per wave, 16 waves,
// at most four sub-slices per workgroup, then k slices until every CU has a workgroup.  Configurations
// with more row tiles (M up to 64) or two weight tiles per wave were measured as well and lost to the
// rollout-batch kernel (their fp32 partials cost as much as the weights on wide layers), so the plan
// is limited to M <= 16.
inline PanelPlan plan_panel(int64_t M, int64_t K, int64_t N) {
    PanelPlan p{};
    p.ok = false;
    if (M < 2 || M > 16) return p;
    const int groups = (int)(K / kGroup), tiles = (int)(N / kTileRows);
    constexpr size_t kLds = 160 * 1024;
    p.MT = 1;
    p.R = 1;
    p.WAVES = 16;
    // smallest split whose panel fits
    int sk = 0;
    for (int d = 1; d <= groups; ++d) {
        if (groups % d) continue;
        if (panel_lds_bytes(M, p.MT, p.R, p.WAVES, 1, groups / d) <= kLds) {
            sk = d;
            break;
        }
    }
    if (sk == 0 || groups / sk < 8) return p;     // awkward group counts: the rollout-batch kernel
    auto wgs_at = [&](int s_in, int d) {
        const int TW = p.WAVES / s_in;
        return (int64_t)((tiles + TW * p.R - 1) / (TW * p.R)) * d;
    };
    p.S = 1;
    while (p.S < 4 && wgs_at(p.S, sk) < kCus && (groups / sk) / (p.S * 2) >= 4) p.S *= 2;
    for (int d = sk + 1; d <= groups && wgs_at(p.S, sk) < kCus; ++d) {
        if (groups % d || (groups / d) / p.S < 4) continue;
        sk = d;
    }
    // sweep overrides (unset in production)
    const int s_env = env_int("DMR_PANEL_S", 0), sk_env = env_int("DMR_PANEL_SK", 0);
    if (s_env >= 1 && s_env <= p.WAVES && (s_env & (s_env - 1)) == 0) p.S = s_env;
    if (sk_env >= 1 && groups % sk_env == 0) sk = sk_env;
    p.SK = sk;
    p.gq = groups / sk;
    while (p.S > p.gq) p.S >>= 1;
    p.lds = panel_lds_bytes(M, p.MT, p.R, p.WAVES, p.S, p.gq);
    if (p.lds > kLds) return p;
    p.ok = true;
    return p;
}

size_t w4_panel_workspace_bytes(int64_t M, int64_t K, int64_t N);
bool w4_panel_applies(int64_t M, int64_t K, int64_t N);
hipError_t launch_w3_panel(const LayerView3 &L, const uint16_t *x, int64_t M, void *y, bool out_f32, void *ws,
                           hipStream_t stream);
hipError_t launch_w4_panel(const LayerView &L, const uint16_t *x, int64_t M, void *y, bool out_f32, void *ws,
                           hipStream_t stream);

}  // namespace dmr

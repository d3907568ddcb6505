// Launch planning shared by the rollout-batch kernels (INT4 and bf16): row tiles per wave, waves along
// m and n, weight tiles per wave, and the split of K.  Pure host arithmetic for 256 CUs, so that the
// workspace queries agree with the launches.
#pragma once
#include <cstdlib>

#include "common.hpp"

namespace dmr {

struct MidPlan {
    int MTW, WM, NW, R, SK, gps;
};

// Pure host arithmetic (the workspace query must agree with the launch): 256 CUs assumed.
inline MidPlan plan_mid(int64_t M, int64_t K, int64_t N) {
    MidPlan p;
    const int groups = (int)(K / kGroup), tiles = (int)(N / kTileRows);
    if (M <= 64) {
        p.MTW = (int)((M + 15) / 16);
        p.WM = 1;
        p.NW = 4;
    } else {
        const int64_t pad3 = (M + 95) / 96 * 96, pad4 = (M + 127) / 128 * 128;
        p.MTW = pad3 < pad4 ? 3 : 4;
        p.WM = 2;
        p.NW = 2;     // 8-wave workgroups (128 x 128 tiles) were measured too: no faster
    }
    const int BM = 16 * p.MTW * p.WM;
    const int64_t mblocks = (M + BM - 1) / BM;
    // Measured rules (gfx950, 256 CUs): split K while that keeps >= 8 groups per split and fewer than
    // 384 workgroups exist; two weight tiles per wave unless that leaves under 256 workgroups
    // even at the deepest split.
    auto split_for = [&](int64_t wgs) {
        int sk = 1;
        while (wgs * sk < 384 && groups % (sk * 2) == 0 && groups / (sk * 2) >= 8) sk *= 2;
        return sk;
    };
    auto wgs_for = [&](int R) { return (int64_t)((tiles + p.NW * R - 1) / (p.NW * R)) * mblocks; };
    p.R = wgs_for(2) * split_for(wgs_for(2)) >= 256 ? 2 : 1;
    const int r_env = env_int("DMR_MID_R", 0);
    if (r_env == 1 || r_env == 2) p.R = r_env;
    p.SK = split_for(wgs_for(p.R));
    const int sk_env = env_int("DMR_MID_SK", 0);
    if (sk_env >= 1 && groups % sk_env == 0) p.SK = sk_env;
    p.gps = groups / p.SK;
    return p;
}

// y = sum over splits of part[split] (fp32 [splits][M][N]), splits in ascending order.
hipError_t launch_splitk_reduce(const float *part, void *y, int64_t total, int splits, bool out_f32,
                                hipStream_t stream);

}  // namespace dmr

// Device-side description of a persistent decode chain (w4_chain.hip): a table of stages, each one
// M == 1 Linear of the 4-bit copy with its fused glue, run in order by one resident grid.
#pragma once
#include "common.hpp"

namespace dmr {

struct ChainStage {            // 64 bytes, one per Linear, in device memory behind the control block
    const uint4 *wt;           // streaming weight blocks of the layer
    const uint32_t *sz;        // its scale / zero words
    const uint16_t *in;        // activation row: [K] bf16 ([2 K] with the SwiGLU prologue)
    const uint16_t *aux;       // gamma [K] for the RMSNorm prologue
    const uint16_t *res;       // residual [N] bf16 or null
    void *out;                 // [N] bf16 or fp32
    int32_t groups, tiles;     // K / 128, N / 16
    int32_t flags;             // prologue (Prologue) in bits 0..7, bit 8: fp32 output
    float eps;
};
static_assert(sizeof(ChainStage) == 64, "stage table layout");

constexpr size_t kChainControlBytes = 4096;  // one arrival flag per workgroup, then the time-out word
constexpr int kChainMaxGrid = 1008;
constexpr int kChainTimeoutWord = 1008;
constexpr int kChainMaxGroups = 128;         // K <= 16384: two 16-byte pieces per thread stage the row
constexpr int kChainMinGroups = 16;          // one k slice per wave of the workgroup

struct ChainLaunch {
    const ChainStage *tab;     // device
    uint32_t *ctl;             // device, kChainControlBytes
    int n_stages;
    int x16_cap;               // 16-byte pieces of the longest activation row
    int g_cap;                 // groups of the longest row, rounded up to 4
    int nt_cap;                // most tiles a workgroup owns in one stage
    int grid;
    int spin_limit;
};

size_t chain_lds_bytes(const ChainLaunch &c);
// Largest grid whose workgroups are all resident at once with that much LDS (0 if none).
int chain_resident_grid(size_t lds_bytes);
hipError_t launch_w4_chain(const ChainLaunch &c, hipStream_t stream);

}  // namespace dmr

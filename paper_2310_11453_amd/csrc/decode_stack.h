// Shapes and work split of the layer-chain kernel (decode_stack.hip), shared with the host
// code that validates a chain and sizes its workspace.
#pragma once
#include "common.h"

namespace bl {

constexpr int kStackWaves = 8;      // waves per workgroup (one workgroup per CU)
constexpr int kStackD = 3;          // ring slots (units in flight) per wave; unit = one tile x C chunks
constexpr int kStackTpw = 4;        // tiles per wave and pass
constexpr int kStackCodes = 65536;  // LDS bytes for the codes of the M input rows
constexpr int kStackMaxM = 16;

// One layer of the chain as the caller describes it (the layout of bl_stack_layer).
struct StackLayer {
    const uint32_t* packed;  // tile layout of bitlinear_pack_weights
    const float* beta;       // device scalar
    int64_t N, K;
};

// What the kernel derives from (N, K, M).  Waves split K into `pairs` groups of C chunks, WK of
// them side by side (several rounds if pairs > WK), and the tile rows WT ways.
struct StackPlan {
    int TN, TK, Kpad, C, pairs, WK, WT, ln_waves;
};

// false: the kernel cannot take this layer
__host__ __device__ inline bool stack_plan(int64_t N, int64_t K, int M, StackPlan& p) {
    if (N <= 0 || K <= 0 || K % 4 != 0 || N % 4 != 0 || K >= (1 << 22) || N >= (1 << 26)) return false;
    p.TN = (int)tiles_n(N);
    p.TK = (int)tiles_k(K);
    p.Kpad = p.TK * kChunkK;
    if ((int64_t)M * p.Kpad > kStackCodes) return false;
    if (K / 4 > 8 * kWave * 16) return false;  // the quantiser's own limit on a row
    p.C = (p.TK % 2 == 0 && p.TK >= 8) ? 2 : 1;
    p.pairs = p.TK / p.C;
    const int rounds = (p.pairs + kStackWaves - 1) / kStackWaves;
    p.WK = (p.pairs + rounds - 1) / rounds;
    p.WT = kStackWaves / p.WK;
    // waves per row of the quantiser whose reduction order the kernel reproduces
    p.ln_waves = K / 4 > 4 * kWave * 16 ? 8 : 4;
    return true;
}

struct StackArgs {
    const StackLayer* layers;  // device
    int n_layers;
    int M;
    const float* X;
    float* Y;
    float* buf[2];   // [M][max N] each: outputs of the inner layers, alternating
    unsigned* sync;  // [0] arrivals at the grid barrier, [1] error flag
    float eps;
    unsigned spin_limit;
};
hipError_t launch_decode_stack(const StackArgs& a, hipStream_t s);
int decode_stack_grid();

}  // namespace bl

// Host-side launchers implemented by the kernel files; called from api.hip only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bl {

// Launch-time switches for tests and benchmarks (bitlinear_set_tuning in the C ABI; defaults:
// everything 0 = the launchers decide).  One process-wide instance, defined in api.hip.
struct Tuning {
    int decode_nofuse;     // forward at one token: quantiser and GEMM as two launches
    int decode_nosplit;    // M <= 16: never split K over workgroups
    int decode_tiles;      // M <= 16: weight tiles per workgroup (1..8)
    int mid_nosplit;       // 16 < M <= 64: never split K over workgroups
    int mid_split_tiles;   // 16 < M <= 64: 512-chunks of K per slice
    int mid_only;          // 16 < M <= 32: skip the register-streaming kernel
    int prefill_tile;      // M > 64: 1 = 128 x 256 tiles, 2 = 256 x 256
    int prefill_grid;      // M > 64: workgroups of the persistent kernel
    int prefill_xbm;       // M > 64: tile rows in the block of tiles an XCD owns (0: one)
    int quant_wpr;         // quantiser: waves per row (1, 2, 4, 8)
    int bwd_ring;          // backward GEMM: 1 = ring kernel, 2 = small kernel
    int bwd_grid;          // backward ring kernel: workgroups
    int bwd_rowmajor;      // backward ring kernel: plain row-major tile order
    int group_slices;      // grouped layer, M <= 64: every K-group a slice of the grid (work item) of its own
    int mid_kernel;        // 32 < M <= 64: 1 = LDS-tiled kernel with the in-workgroup K split
};
const Tuning& tuning();

// pack.hip
// A block of `rows` x `cols` weights inside a matrix whose rows are `ldw` floats apart
// (ldw == cols: the whole matrix).  `packed` receives tiles_n(rows) x tiles_k(cols) tiles.
int reduce_grid(int64_t count4);
hipError_t launch_pack(const float* W, int64_t rows, int64_t cols, int64_t ldw, bool beta_centered,
                       uint32_t* packed, float* alpha, float* beta, double* partials, hipStream_t s);
// canonical words of the block go to canonical[n * ldc + kw], ldc in words
hipError_t launch_weight_rowsums(const uint32_t* packed, int64_t N, int64_t K, int32_t* wsum,
                                 hipStream_t s);
hipError_t launch_to_canonical(const uint32_t* packed, int64_t N, int64_t K, uint32_t* canonical,
                               int64_t ldc, hipStream_t s);

// quant.hip
struct QuantArgs {
    const float* X;
    int64_t M, K;
    const float* gain;
    const float* bias;
    float eps;
    bool skip_ln;
    bool per_tensor;
    int8_t* codes;
    float* gamma;
    int32_t* rowsum;
    float* xhat_dump;
    double* rowstats;   // per-tensor only: [M][2] = (mean, rstd)
    uint32_t* gmax_bits; // per-tensor only: [groups], bit pattern of the running max
    uint32_t* gmin_bits; // per-tensor Eq. 6 only: [groups], ordered key of the running minimum
                         // (gmax_bits then holds the ordered key of the running maximum)
    // Group normalisation / quantisation (Eq. 14-15): a token of `groups` * K elements is
    // handled as `groups` consecutive rows of K; row r belongs to group r % groups.  M counts
    // those rows.  gain/bias hold groups * K entries.  groups = 1: the plain layer.
    int groups;
    // Eq. 6: codes = clamp(rne((x^ - eta) * 128 / gamma), 0, 127) with eta = min x^,
    // gamma = max(x^ - eta); eta receives the minima, laid out like gamma ([M] rows per token,
    // [groups] per tensor).
    bool nonneg;
    float* eta;
};
bool quant_supported(int64_t K);
hipError_t launch_quant(const QuantArgs& a, hipStream_t s);

// gemm_decode.hip / gemm_prefill.hip
struct GemmArgs {
    const int8_t* codes;
    const float* gamma;
    const int32_t* rowsum;
    int64_t M, K, N;
    const uint32_t* packed;
    const float* beta;
    bool per_tensor;
    bool out_acc;
    float* Y;
    // Group quantisation (Eq. 13-15); plain layer: ldq = K, gstride = 1, beta_rows = N.
    int64_t ldq;          // bytes between consecutive rows of codes (>= K: a K-slice of wider rows)
    int64_t gstride;      // gamma[m * gstride], rowsum[m * gstride] belong to token m
    int64_t beta_rows;    // output columns n per beta group (a multiple of 16, or N)
    int64_t beta_stride;  // beta[(n / beta_rows) * beta_stride] scales column n
    bool accumulate;      // Y += result (a later K-group) instead of Y = result
    // Eq. 6: Y += (beta * eta[m * gstride]) * wsum[n] (eta[0] per tensor), wsum[n] = sum_k s[n,k];
    // nullptr otherwise
    const float* eta;
    const int32_t* wsum;
    // Packed tiles of one tile row are tk_pitch KiB apart (0: tiles_k(K), the whole matrix).
    int64_t tk_pitch;
    // K split across workgroups (set by the launchers, not by callers): blockIdx.y = split,
    // split_k elements of K each; partial sums 2 * sum_k q b go to split_ws[split][M][N] (int32)
    // and a second kernel folds them and applies the epilogue.
    int64_t split_k;
    int32_t* split_ws;
    size_t split_ws_bytes;  // what the caller offers; too small or nullptr: no split
    // All K-groups of a grouped layer (Eq. 13-15) in one launch, M <= 64 (set by the caller
    // together with split_ws of kgroups * M * N * 4 bytes): slice g of the launch is K-group g.
    // codes, packed, K, gamma, rowsum, beta, eta, wsum describe group 0; group g reads codes + g * K,
    // packed + g * group_packed dwords, and the fold applies gamma[.. + g], rowsum[.. + g], beta[.. + g],
    // eta[.. + g], wsum[g * N + n] to its partial sums and adds the groups in the order 0, 1, ...
    // 0 or 1: off.
    int kgroups;
    int64_t group_packed;
    // One token (M = 1, K <= 32768) straight from fp32, small-batch kernel only: every workgroup
    // normalises and quantises the row for itself (Eq. 12, Eq. 4-5) while its first weight tiles
    // are on their way, instead of reading codes / gamma / rowsum, so the layer is one launch.
    // Workgroup 0 also writes the three to codes_out / gamma_out / rowsum_out and the normalised
    // row to xhat_out.  nullptr: codes
    // are read.
    const float* x_row;
    const float* ln_gain;  // [K] or nullptr
    const float* ln_bias;  // [K] or nullptr
    float ln_eps;
    bool skip_ln;
    int8_t* codes_out;
    float* gamma_out;
    int32_t* rowsum_out;
    float* xhat_out;  // [K]: the normalised row the codes were rounded from
};
bool gemm_decode_fuses_quant(int64_t M, int64_t K, int64_t N);
size_t gemm_split_ws_bytes(int64_t M, int64_t N, int64_t K);
int64_t prefill_split_tiles(int64_t M, int64_t N, int64_t K);
void launch_splitk_reduce(const GemmArgs& a, int splits, hipStream_t s);
hipError_t launch_read_probe(const void* src, size_t bytes, int workgroups, int threads,
                             uint32_t* sink, hipStream_t s);
hipError_t launch_gemm_decode(const GemmArgs& a, hipStream_t s);
hipError_t launch_gemm_prefill(const GemmArgs& a, hipStream_t s);
hipError_t launch_gemm_mid(const GemmArgs& a, hipStream_t s);  // 16 < M <= 64
bool launch_gemm_stream(const GemmArgs& a, hipStream_t s);      // 16 < M <= 32; false: not taken
int64_t stream_split_tiles(int64_t M, int64_t K);

// backward.hip
struct BackwardArgs {
    const float* dY;
    int64_t M, N, K;
    const int8_t* codes;
    const float* gamma;
    bool per_tensor;
    const uint32_t* packed;
    const float* beta;
    float* dX;
    float* dW;
    void* workspace;
};
size_t backward_workspace_bytes(int64_t M, int64_t N, int64_t K);
hipError_t launch_backward(const BackwardArgs& a, hipStream_t s);

// ln_backward.hip
struct LnBackwardArgs {
    const float* g;    // gradient w.r.t. the LayerNorm output, [M][K]
    const float* X;    // the layer's input, [M][K]
    int64_t M, K;      // rows of K elements: tokens * groups rows, K = elements per group
    const float* gain; // [groups * K] or nullptr
    float eps;
    int groups;        // row r belongs to K-group r % groups
    float* dX;         // [M][K] or nullptr (statistics only)
    double* rowstats;  // [M][2] = (mean, rstd), or nullptr
};
bool ln_backward_supported(int64_t K);
int ln_backward_chunks(int64_t tokens);
hipError_t launch_ln_backward(const LnBackwardArgs& a, float* dgain, float* dbias, double* partials,
                              hipStream_t s);

}  // namespace bl

// 1-bit x 8-bit GEMM + dequantisation for many tokens (prefill / training):
//   Y[m,n] = (sum_k q[m,k] * s[n,k]) * beta * gamma_m / 128     (Eq. 7, Eq. 11)
// of arXiv 2310.11453.  Compute-bound: the contraction runs on the i8 MFMA
// (v_mfma_i32_32x32x32_i8, int32 accumulators).
//
// Tiling.  A workgroup computes a BM x BN block of Y.  The int8 activation
// codes of the block (BM rows x 64 k per stage) are staged through LDS, double
// buffered, rows padded to 80 bytes so the 16-byte operand reads of a 16-lane
// group touch every bank once.  The 1-bit weights never enter LDS: each wave
// keeps the packed dwords of its own columns in registers (16 bytes per lane
// cover 16 k in each of the eight 64-wide sub-blocks of a 512-chunk) and
// expands them to +-1 bytes right before use:
//     t  = (w >> i) & 0x01010101          four {0,1} bytes
//     pm = v_perm_b32(table, t)           byte 1 -> +1 (0x01), byte 0 -> -1 (0xff)
// i.e. three VALU operations per four weights, amortised over the WTM/32 MFMAs
// that reuse the operand.  A wave tile of 128 x 64 keeps both the LDS traffic
// (one 1 KiB operand read per two MFMAs) and the expansion cost (24 VALU per 8
// MFMAs) well below the MFMA time.
#include "common.h"
#include "kernels.h"

namespace bl {

constexpr int kStageK = 64;    // k per LDS stage
constexpr int kRowPitch = 80;  // bytes per staged row (64 + 16 padding)

__device__ inline int expand_pm1(uint32_t w, int i) {
    const uint32_t t = (w >> i) & 0x01010101u;
    // selector byte 0 -> table byte 0 = 0xff (-1), selector byte 1 -> table byte 1 = 0x01 (+1)
    return (int)__builtin_amdgcn_perm(0x000001ffu, 0x000001ffu, t);
}

template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(WM * WN * 64, 2) void gemm_prefill_kernel(GemmArgs a, int grid_m,
                                                                        int grid_n) {
    constexpr int THREADS = WM * WN * kWave;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int MI = WTM / 32, NI = WTN / 32;
    constexpr int PIECES = BM * 4 / THREADS;  // 16-byte pieces of a stage per thread
    static_assert(BM * 4 % THREADS == 0 && MI >= 1 && NI >= 1, "tile shape");

    __shared__ __attribute__((aligned(16))) uint8_t smA[2][BM * kRowPitch];
    __shared__ float smScale[BM];

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD one contiguous
    // range of tiles (M fastest) so the tiles sharing an L2 share weight columns.
    const int nb = grid_m * grid_n;
    int pid = blockIdx.x;
    if ((nb & 7) == 0) pid = (pid & 7) * (nb >> 3) + (pid >> 3);
    const int bm = pid % grid_m, bn = pid / grid_m;
    const int64_t m0 = (int64_t)bm * BM, n0 = (int64_t)bn * BN;

    const int w = threadIdx.x / kWave, l = threadIdx.x % kWave;
    const int wm = w / WN, wn = w % WN;
    const int j = l & 31, g2 = l >> 5;
    const int64_t TN = tiles_n(a.N), TK = tiles_k(a.K);
    const int64_t M = a.M, K = a.K;

    // per-row dequantisation scale (Eq. 11): beta * gamma_m / 128
    {
        const float beta = *a.beta;
        for (int r = threadIdx.x; r < BM; r += THREADS) {
            const int64_t m = m0 + r;
            float sc = 0.f;
            if (m < M) sc = (beta * (a.per_tensor ? a.gamma[0] : a.gamma[m])) / 128.0f;
            smScale[r] = sc;
        }
    }

    // global -> LDS staging of the activation codes
    v4i stage[PIECES];
    auto load_stage = [&](int64_t kbase) {
#pragma unroll
        for (int q = 0; q < PIECES; ++q) {
            const int p = threadIdx.x + q * THREADS;
            const int row = p >> 2, seg = p & 3;
            const int64_t m = m0 + row, k = kbase + seg * 16;
            v4i z = {0, 0, 0, 0};
            if (m < M && k < K) z = *reinterpret_cast<const v4i*>(a.codes + m * K + k);
            stage[q] = z;
        }
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int q = 0; q < PIECES; ++q) {
            const int p = threadIdx.x + q * THREADS;
            const int row = p >> 2, seg = p & 3;
            *reinterpret_cast<v4i*>(&smA[buf][row * kRowPitch + seg * 16]) = stage[q];
        }
    };

    // packed weights of this wave's columns for one 512-chunk: [NI][h = 0,1]
    auto load_bits = [&](int64_t tk, v4i (&bw)[NI][2]) {
#pragma unroll
        for (int s = 0; s < NI; ++s) {
            const int64_t n = n0 + wn * WTN + 32 * s + j;
            const int64_t tn = n >> 4;
            const int c = (int)(n & 15);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                v4i z = {0, 0, 0, 0};
                if (tn < TN && tk < TK)
                    z = *reinterpret_cast<const v4i*>(a.packed + tile_dword_offset(tn, tk, TK) +
                                                      ((2 * h + g2) * 16 + c) * 4);
                bw[s][h] = z;
            }
        }
    };

    v16i acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int s = 0; s < NI; ++s)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][s][r] = 0;

    v4i bw_cur[NI][2], bw_nxt[NI][2];
    load_bits(0, bw_cur);
    load_stage(0);
    store_stage(0);
    __syncthreads();

    const int64_t nstages = TK * 8;
    const uint8_t* a_base = &smA[0][(wm * WTM + j) * kRowPitch + 16 * g2];

    for (int64_t tk = 0; tk < TK; ++tk) {
        load_bits(tk + 1, bw_nxt);  // guarded inside: zeros past the end
        for (int i = 0; i < 8; ++i) {
            const int64_t st = tk * 8 + i;
            const int buf = (int)(st & 1);
            if (st + 1 < nstages) load_stage((st + 1) * kStageK);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                v4i b[NI];
#pragma unroll
                for (int s = 0; s < NI; ++s) {
                    b[s][0] = expand_pm1((uint32_t)bw_cur[s][h][0], i);
                    b[s][1] = expand_pm1((uint32_t)bw_cur[s][h][1], i);
                    b[s][2] = expand_pm1((uint32_t)bw_cur[s][h][2], i);
                    b[s][3] = expand_pm1((uint32_t)bw_cur[s][h][3], i);
                }
                v4i av[MI];
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
                    av[mi] = *reinterpret_cast<const v4i*>(a_base + buf * (BM * kRowPitch) +
                                                           mi * 32 * kRowPitch + 32 * h);
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                    for (int s = 0; s < NI; ++s)
                        acc[mi][s] = __builtin_amdgcn_mfma_i32_32x32x32_i8(av[mi], b[s], acc[mi][s],
                                                                           0, 0, 0);
            }
            if (st + 1 < nstages) store_stage(buf ^ 1);
            __syncthreads();
        }
#pragma unroll
        for (int s = 0; s < NI; ++s)
#pragma unroll
            for (int h = 0; h < 2; ++h) bw_cur[s][h] = bw_nxt[s][h];
    }

    // epilogue: lane (j, g2) holds column n = .. + j and rows 8*(r/4) + 4*g2 + r%4
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int s = 0; s < NI; ++s) {
            const int64_t n = n0 + wn * WTN + 32 * s + j;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = wm * WTM + 32 * mi + 8 * (r >> 2) + 4 * g2 + (r & 3);
                const int64_t m = m0 + row;
                if (m < M && n < a.N) {
                    if (a.out_acc)
                        reinterpret_cast<int*>(a.Y)[m * a.N + n] = acc[mi][s][r];
                    else
                        a.Y[m * a.N + n] = (float)acc[mi][s][r] * smScale[row];
                }
            }
        }
}

template <int BM, int BN, int WM, int WN>
static void launch_tile(const GemmArgs& a, hipStream_t s) {
    const int grid_m = (int)((a.M + BM - 1) / BM), grid_n = (int)((a.N + BN - 1) / BN);
    gemm_prefill_kernel<BM, BN, WM, WN>
        <<<(unsigned)(grid_m * grid_n), WM * WN * kWave, 0, s>>>(a, grid_m, grid_n);
}

hipError_t launch_gemm_prefill(const GemmArgs& a, hipStream_t s) {
    if (a.M <= 64) launch_tile<64, 128, 1, 4>(a, s);
    else launch_tile<256, 128, 2, 2>(a, s);
    return hipGetLastError();
}

}  // namespace bl

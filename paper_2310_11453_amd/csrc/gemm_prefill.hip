// 1-bit x 8-bit GEMM + dequantisation for many tokens (prefill / training):
//   Y[m,n] = (sum_k q[m,k] * s[n,k]) * beta * gamma_m / 128     (Eq. 7, Eq. 11)
// of arXiv 2310.11453.  Compute-bound: the contraction runs on the i8 MFMA
// (v_mfma_i32_32x32x32_i8, int32 accumulators).
//
// Tiling.  A workgroup computes a BM x BN block of Y.
//  * Activation codes (int8) are streamed global -> LDS with the direct
//    global_load_lds_dwordx4 path, no registers in between, through a ring of NS
//    stages of BM rows x 64 k.  A stage is issued NS-1 stages ahead of its use,
//    which hides the L2/HBM latency behind (NS-1) x 16 MFMAs per wave.  The 16-byte
//    segments of a row are XOR-swizzled with (row/4)%4 so that the 16-byte operand
//    reads of 16 consecutive rows hit every LDS bank exactly once.
//  * The 1-bit weights of the block's BN columns for one 512-chunk (BN/16 packed tiles of
//    1 KiB) take the same DMA path into a small LDS buffer, one chunk ahead.  At the start
//    of a chunk each lane copies the 16-byte groups of its own columns to registers (16
//    bytes cover 16 k in each of the eight 64-wide sub-blocks of the chunk) and expands
//    them right before use, never as bytes in LDS:
//        b = (w >> i) & 0x01010101           four {0,1} bytes, two VALU operations
//    amortised over the WTM/32 MFMAs that reuse the operand.  The MFMA accumulates
//    sum_k q b; the epilogue restores sum_k q s = 2 sum_k q b - sum_k q with the row sums
//    of the codes that the quantiser already produced.
//  * A 128 x 64 wave tile keeps LDS traffic (one 1 KiB operand read per two MFMAs)
//    and expansion cost (24 VALU per 8 MFMAs) well below the MFMA time; two
//    workgroups share a CU so one's epilogue overlaps the other's main loop.
//
// Synchronisation is explicit: s_waitcnt vmcnt(n) on the wave's own DMA, then a bare
// s_barrier (no fence: a fence would drain every DMA in flight).  LDS reads of stage
// st happen strictly between barrier(st) and barrier(st+1); the DMA that overwrites
// the same buffer is issued after barrier(st+1).
#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace bl {

constexpr int kStageK = 64;  // k per LDS stage (= bytes per staged row)

// compile-time loop: f(integral_constant<int, B>), ..., f(integral_constant<int, E-1>)
template <int B, int E, class F>
__device__ inline void static_for(F&& f) {
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

// four {0,1} bytes: bit plane i of a packed dword
__device__ inline int expand_01(uint32_t w, int i) { return (int)((w >> i) & 0x01010101u); }

template <int N>
__device__ inline void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    // gfx9 encoding: vmcnt = {[15:14],[3:0]}, expcnt [6:4] = 7 and lgkmcnt [11:8] = 15 (no wait).
    // The compiler barrier keeps ordinary memory operations on their side of the wait.
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// LDS reads are written as asm.  The data is put there by DMA, and an LDS read the compiler
// can see makes it drain the DMA queue (vmcnt(0)) first, which would undo the prefetch.  Each
// asm block issues its reads AND waits for them (lgkmcnt(0)), so every output register is
// valid when the block ends and the compiler is free to copy or move it.
template <int O>
__device__ inline void lds_read_x4(v4i (&a0)[4], uint32_t ad0) {
    asm volatile(
        "ds_read_b128 %0, %4 offset:%5\n\t"
        "ds_read_b128 %1, %4 offset:%6\n\t"
        "ds_read_b128 %2, %4 offset:%7\n\t"
        "ds_read_b128 %3, %4 offset:%8\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(a0[0]), "=&v"(a0[1]), "=&v"(a0[2]), "=&v"(a0[3])
        : "v"(ad0), "n"(O), "n"(O + 2048), "n"(O + 4096), "n"(O + 6144));
}
template <int O>
__device__ inline void lds_read_x2(v4i (&a0)[2], uint32_t ad0) {
    asm volatile(
        "ds_read_b128 %0, %2 offset:%3\n\t"
        "ds_read_b128 %1, %2 offset:%4\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(a0[0]), "=&v"(a0[1])
        : "v"(ad0), "n"(O), "n"(O + 2048));
}
// packed weight bits of a lane: [NI][h]; sub-tile s at +2048, half h at +512
__device__ inline void lds_read_bits(v4i (&bw)[2][2], uint32_t ad) {
    asm volatile(
        "ds_read_b128 %0, %4\n\t"
        "ds_read_b128 %1, %4 offset:512\n\t"
        "ds_read_b128 %2, %4 offset:2048\n\t"
        "ds_read_b128 %3, %4 offset:2560\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(bw[0][0]), "=&v"(bw[0][1]), "=&v"(bw[1][0]), "=&v"(bw[1][1])
        : "v"(ad));
}
__device__ inline void lds_read_bits(v4i (&bw)[1][2], uint32_t ad) {
    asm volatile(
        "ds_read_b128 %0, %2\n\t"
        "ds_read_b128 %1, %2 offset:512\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(bw[0][0]), "=&v"(bw[0][1])
        : "v"(ad));
}

__device__ inline void block_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

template <int BM, int BN, int WM, int WN, int NS>
__global__ __launch_bounds__(WM * WN * 64, 2) void gemm_prefill_kernel(GemmArgs a, int grid_m,
                                                                        int grid_n) {
    constexpr int THREADS = WM * WN * kWave;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int MI = WTM / 32, NI = WTN / 32;
    constexpr int P = BM * 4 / THREADS;  // 16-byte DMA pieces per thread per stage
    constexpr int NWAVES = WM * WN;
    constexpr int NBW = (BN / 16) / NWAVES;  // packed-weight tiles (DMA pieces) per wave per chunk
    constexpr int STAGE_BYTES = BM * kStageK;
    static_assert(BM * 4 % THREADS == 0 && MI >= 1 && NI >= 1, "tile shape");
    static_assert(NS == 4 || NS == 8, "ring size must divide the 8 stages of a chunk");
    static_assert((BN / 16) % NWAVES == 0 && (NS - 2) * P + NBW < 64, "tile shape");

    __shared__ __attribute__((aligned(1024))) uint8_t smA[NS * STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) uint8_t smB[(BN / 16) * 1024];

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
    const int nst = (int)((K + kStageK - 1) / kStageK);

    // ---- DMA of one stage: thread -> P pieces; piece = (row, swizzled 16-byte segment) ----
    // Global address = uniform base (block row 0, stage k) + a 32-bit per-lane offset, so
    // advancing a stage costs scalar arithmetic only.  Rows past M re-read row M-1 (never
    // stored).  CLAMP: stages that may reach past K re-read the last 16 valid bytes of the row
    // (the upper half of a half-filled last stage is never read).
    uint32_t goff[P];
    int gseg[P];
#pragma unroll
    for (int q = 0; q < P; ++q) {
        const int slot = q * THREADS + threadIdx.x;
        int row = slot >> 2;
        gseg[q] = ((slot & 3) ^ ((row >> 2) & 3)) * 16;
        if (m0 + row > M - 1) row = (int)(M - 1 - m0);
        goff[q] = (uint32_t)row * (uint32_t)K + gseg[q];
    }
    const int8_t* gbase = a.codes + m0 * K;
    const uint32_t lds_wave = (uint32_t)(w * kWave * 16);
    auto issue = [&](int st, int buf, bool clamp) {
#pragma unroll
        for (int q = 0; q < P; ++q) {
            const int8_t* src = gbase + (int64_t)st * kStageK + goff[q];
            if (clamp) {
                const int64_t k = (int64_t)st * kStageK + gseg[q];
                if (k > K - 16) src -= k - (K - 16);
            }
            __builtin_amdgcn_global_load_lds(
                (const void*)src,
                (__attribute__((address_space(3))) void*)(smA + buf * STAGE_BYTES +
                                                          q * THREADS * 16 + lds_wave),
                16, 0, 0);
        }
    };

    // ---- packed weights: DMA of the block's BN/16 tiles for one 512-chunk -----------------
    // Tile t of the block goes to smB + t KiB, lane for lane as it lies in memory; wave w
    // moves tiles w, w + NWAVES, ...  Columns past N read a valid tile (never stored).
    const uint32_t* bsrc[NBW];
#pragma unroll
    for (int q = 0; q < NBW; ++q) {
        int64_t tn = (n0 >> 4) + w + q * NWAVES;
        if (tn > TN - 1) tn = TN - 1;
        bsrc[q] = a.packed + tile_dword_offset(tn, 0, TK) + l * 4;
    }
    auto issue_bits = [&](int64_t tk) {
#pragma unroll
        for (int q = 0; q < NBW; ++q)
            __builtin_amdgcn_global_load_lds(
                (const void*)(bsrc[q] + tk * 256),
                (__attribute__((address_space(3))) void*)(smB + (w + q * NWAVES) * 1024), 16, 0, 0);
    };
    // lane (j, g2) of sub-tile s, half h reads lane slot (2h+g2)*16 + j%16 of tile (..+j/16)
    const uint32_t b_lane = (uint32_t)(uintptr_t)smB + ((wn * WTN + j) >> 4) * 1024 +
                            (g2 * 16 + (j & 15)) * 16;
    v4i bw[NI][2];
    auto read_bits = [&]() { lds_read_bits(bw, b_lane); };

    v16i acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int s = 0; s < NI; ++s)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][s][r] = 0;

    issue_bits(0);
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) issue(s, s, true);

    // lane's operand address inside a stage: row (wm*WTM + j), segment (2h+g2) ^ swizzle
    const int sw = (j >> 2) & 3;
    const uint32_t a_lane[2] = {
        (uint32_t)(uintptr_t)smA + (wm * WTM + j) * kStageK + ((g2) ^ sw) * 16,
        (uint32_t)(uintptr_t)smA + (wm * WTM + j) * kStageK + ((2 + g2) ^ sw) * 16};

    // One stage of MFMAs: 2 k-steps of 32 (h = 0, 1); `i` selects the bit plane of the chunk.
    // The weight operand holds {0,1}; the epilogue turns sum_k q b into sum_k q (2b - 1).
    // BUFOFF is the stage's byte offset in the ring when known at compile time (main loop),
    // else 0 with the offset folded into `dyn`.
    auto mfma_half = [&](v4i (&av)[MI], int h, int i) {
        v4i b[NI];
#pragma unroll
        for (int s = 0; s < NI; ++s)
#pragma unroll
            for (int d = 0; d < 4; ++d) b[s][d] = expand_01((uint32_t)bw[s][h][d], i);
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int s = 0; s < NI; ++s)
                acc[mi][s] = __builtin_amdgcn_mfma_i32_32x32x32_i8(av[mi], b[s], acc[mi][s], 0, 0, 0);
    };
    auto compute = [&](auto bufoff, uint32_t dyn, int i, bool half) {
        constexpr int O = decltype(bufoff)::value;
        static_assert(MI == 2 || MI == 4, "activation sub-tiles per wave");
        // one half (4 or 2 operand reads) at a time keeps 16 registers live instead of 32
        v4i av[MI];
        if constexpr (MI == 4) lds_read_x4<O>(av, a_lane[0] + dyn);
        else lds_read_x2<O>(av, a_lane[0] + dyn);
        mfma_half(av, 0, i);
        if (!half) {
            if constexpr (MI == 4) lds_read_x4<O>(av, a_lane[1] + dyn);
            else lds_read_x2<O>(av, a_lane[1] + dyn);
            mfma_half(av, 1, i);
        }
    };

    // Every stage issues the same DMA operations (P pieces of a stage NS-1 ahead, plus, at
    // i == 2, the NBW weight tiles of the next chunk; past the end they re-read valid bytes
    // into buffers nobody reads), so the number of operations younger than a given group is a
    // compile-time constant: (NS-2)*P, plus NBW while the weight tiles are among them.  The
    // tiles are older than group 8*tk+5, so they have landed for every wave after the barrier
    // of stage 8*tk+5; smB is free again once every wave has passed the barrier of 8*tk+1.
    //
    // Main loop: chunks whose look-ahead stays inside K; no clamps, constant LDS offsets.
    const int64_t kfull = K / kStageK;
    const int64_t main_chunks = kfull >= NS + 7 ? (kfull - NS - 7) / 8 + 1 : 0;
    for (int64_t tk = 0; tk < main_chunks; ++tk) {
        static_for<0, 8>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            if constexpr (i == 3 || i == 4) wait_vmcnt<(NS - 2) * P + NBW>();
            else wait_vmcnt<(NS - 2) * P>();
            block_barrier();
            if constexpr (i == 0) read_bits();
            if constexpr (i == 2) issue_bits(tk + 1);
            issue((int)tk * 8 + i + NS - 1, (i + NS - 1) % NS, false);
            compute(std::integral_constant<int, (i % NS) * STAGE_BYTES>{}, 0u, i, false);
        });
    }
    // Remaining stages (last chunk, ragged K): same schedule with clamped addresses.
    for (int st = (int)main_chunks * 8; st < nst; ++st) {
        const int i = st & 7;
        if (i == 3 || i == 4) wait_vmcnt<(NS - 2) * P + NBW>();
        else wait_vmcnt<(NS - 2) * P>();
        block_barrier();
        if (i == 0) read_bits();
        if (i == 2) issue_bits((st >> 3) + 1 < TK ? (st >> 3) + 1 : (st >> 3));
        issue(st + NS - 1, (st + NS - 1) % NS, true);
        compute(std::integral_constant<int, 0>{}, (uint32_t)((st % NS) * STAGE_BYTES), i,
                (int64_t)st * kStageK + 32 >= K);
    }

    // ---- epilogue (Eq. 11): lane (j, g2) holds column n and rows 8*(r/4) + 4*g2 + r%4 -----
    //   sum_k q s = 2 sum_k q b - sum_k q ;  y = that * (beta * gamma_m / 128)
    const float beta = *a.beta;
    const float g_all = a.per_tensor ? a.gamma[0] : 0.f;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t m = m0 + wm * WTM + 32 * mi + 8 * (r >> 2) + 4 * g2 + (r & 3);
            if (m >= M) continue;
            const int rs = a.rowsum[m];
            const float sc = (beta * (a.per_tensor ? g_all : a.gamma[m])) / 128.0f;
#pragma unroll
            for (int s = 0; s < NI; ++s) {
                const int64_t n = n0 + wn * WTN + 32 * s + j;
                if (n >= a.N) continue;
                const int pm = 2 * acc[mi][s][r] - rs;
                if (a.out_acc) reinterpret_cast<int*>(a.Y)[m * a.N + n] = pm;
                else a.Y[m * a.N + n] = (float)pm * sc;
            }
        }
}

template <int BM, int BN, int WM, int WN, int NS>
static void launch_tile(const GemmArgs& a, hipStream_t s) {
    const int grid_m = (int)((a.M + BM - 1) / BM), grid_n = (int)((a.N + BN - 1) / BN);
    gemm_prefill_kernel<BM, BN, WM, WN, NS>
        <<<(unsigned)(grid_m * grid_n), WM * WN * kWave, 0, s>>>(a, grid_m, grid_n);
}

// K < 2^22 is required (the per-lane offset into a block of 256 rows is kept in 32 bits).
hipError_t launch_gemm_prefill(const GemmArgs& a, hipStream_t s) {
    if (a.K >= ((int64_t)1 << 22)) return hipErrorInvalidValue;
    if (a.M <= 64) launch_tile<64, 128, 1, 4, 4>(a, s);
    else launch_tile<256, 128, 2, 2, 4>(a, s);
    return hipGetLastError();
}

}  // namespace bl

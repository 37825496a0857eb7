// 1-bit x 8-bit GEMM + dequantisation for many tokens (prefill / training):
//   Y[m,n] = (sum_k q[m,k] * s[n,k]) * beta * gamma_m / 128     (Eq. 7, Eq. 11)
// of arXiv 2310.11453.  Compute-bound: the contraction runs on the i8 MFMA
// (v_mfma_i32_32x32x32_i8, int32 accumulators).
//
// Tiling.  A workgroup computes a BM x BN block of Y; a wave a WTM x WTN part of it.
//  * Activation codes (int8) are streamed global -> LDS with the direct
//    global_load_lds_dwordx4 path, no registers in between, through a ring of NS
//    stages of BM rows x 64 k.  The 16-byte segments of a row are XOR-swizzled with
//    (row/4)%4 so that the 16-byte operand reads of 16 consecutive rows hit every LDS
//    bank exactly once.
//  * The 1-bit weights of the block's BN columns for one 512-chunk (BN/16 packed tiles of
//    1 KiB) take the same DMA path into a small LDS buffer, one chunk ahead.  Once per
//    chunk each lane copies the 16-byte groups of its own columns to registers (16 bytes
//    cover 16 k in each of the eight 64-wide sub-blocks of the chunk) and expands them
//    right before use, never as bytes in LDS:
//        b = (w >> i) & 0x01010101           four {0,1} bytes, two VALU operations
//    amortised over the WTM/32 MFMAs that reuse the operand.  The MFMA accumulates
//    sum_k q b; the epilogue restores sum_k q s = 2 sum_k q b - sum_k q with the row sums
//    of the codes that the quantiser already produced.
//  * A 128 x 64 wave tile keeps LDS traffic (one 1 KiB operand read per two MFMAs) and
//    expansion cost (16 VALU per 8 MFMAs) well below the MFMA time.
//  * Eight waves share a 256 x 256 (or 128 x 256) block, one block per CU.  The L2 -> LDS
//    stream of codes is BM*K bytes per block, i.e. 2*BN operations per byte: with BN = 256
//    the whole chip needs ~5 TB/s of it at half the MFMA peak, and with a latency of about
//    2 us that is ~40 KiB in flight per CU, hence the deep ring (NS = 8 stages of 16 KiB).
//
// Schedule.  The unit of work is a half-step: 32 k of a stage, MI*NI MFMAs.  One asm block
// issues the LDS reads of the NEXT half-step's activation operand, then the MFMAs of the
// current one, then waits for the reads: the LDS latency hides under the MFMAs and every
// register the block defines is valid when it ends.  (An LDS read the compiler can see
// makes it drain the whole DMA queue first, because it cannot tell the read from the DMA's
// target; reads whose completion the compiler cannot see must not escape an asm block.)
// Between the two half-steps of stage st every wave waits for its own DMA of stage st+1
// (s_waitcnt vmcnt(n), n counted by hand) and meets the others at a bare s_barrier (no
// fence: a fence would drain every DMA in flight).  After that barrier stage st+1 is
// readable and the buffer of stage st-1 is free, so the DMA of stage st+NS-1 goes there.
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

template <int N>
__device__ inline void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    // gfx9 encoding: vmcnt = {[15:14],[3:0]}, expcnt [6:4] = 7 and lgkmcnt [11:8] = 15 (no wait).
    // The compiler barrier keeps ordinary memory operations on their side of the wait.
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

__device__ inline void block_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// ---- asm blocks ----------------------------------------------------------------------
// Operand reads of one half-step (sub-tile mi at +2048*mi), complete on exit.
__device__ inline void lds_read_a(v4i (&a)[4], uint32_t ad) {
    asm volatile(
        "ds_read_b128 %0, %4\n\t"
        "ds_read_b128 %1, %4 offset:2048\n\t"
        "ds_read_b128 %2, %4 offset:4096\n\t"
        "ds_read_b128 %3, %4 offset:6144\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(a[0]), "=&v"(a[1]), "=&v"(a[2]), "=&v"(a[3])
        : "v"(ad));
}
__device__ inline void lds_read_a(v4i (&a)[2], uint32_t ad) {
    asm volatile(
        "ds_read_b128 %0, %2\n\t"
        "ds_read_b128 %1, %2 offset:2048\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(a[0]), "=&v"(a[1])
        : "v"(ad));
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

// Half-step, 4 x 2 sub-tiles: prefetch an[] from LDS address `ad`, acc[mi][s] += ac[mi] x b[s].
// The four reads ahead of the first MFMA also separate it from whatever VALU instruction
// the compiler placed last.
__device__ inline void half_step(v16i (&acc)[4][2], const v4i (&ac)[4], const v4i (&b)[2],
                                 v4i (&an)[4], uint32_t ad) {
    asm volatile(
        "ds_read_b128 %8, %18\n\t"
        "ds_read_b128 %9, %18 offset:2048\n\t"
        "ds_read_b128 %10, %18 offset:4096\n\t"
        "ds_read_b128 %11, %18 offset:6144\n\t"
        "v_mfma_i32_32x32x32_i8 %0, %12, %16, %0\n\t"
        "v_mfma_i32_32x32x32_i8 %1, %12, %17, %1\n\t"
        "v_mfma_i32_32x32x32_i8 %2, %13, %16, %2\n\t"
        "v_mfma_i32_32x32x32_i8 %3, %13, %17, %3\n\t"
        "v_mfma_i32_32x32x32_i8 %4, %14, %16, %4\n\t"
        "v_mfma_i32_32x32x32_i8 %5, %14, %17, %5\n\t"
        "v_mfma_i32_32x32x32_i8 %6, %15, %16, %6\n\t"
        "v_mfma_i32_32x32x32_i8 %7, %15, %17, %7\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "+v"(acc[0][0]), "+v"(acc[0][1]), "+v"(acc[1][0]), "+v"(acc[1][1]), "+v"(acc[2][0]),
          "+v"(acc[2][1]), "+v"(acc[3][0]), "+v"(acc[3][1]), "=&v"(an[0]), "=&v"(an[1]),
          "=&v"(an[2]), "=&v"(an[3])
        : "v"(ac[0]), "v"(ac[1]), "v"(ac[2]), "v"(ac[3]), "v"(b[0]), "v"(b[1]), "v"(ad));
}
// Timing experiments only: the MFMAs of a 4 x 2 half-step without the operand prefetch.
__device__ inline void half_step_noread(v16i (&acc)[4][2], const v4i (&ac)[4], const v4i (&b)[2]) {
    asm volatile(
        "v_mfma_i32_32x32x32_i8 %0, %8, %12, %0\n\t"
        "v_mfma_i32_32x32x32_i8 %1, %8, %13, %1\n\t"
        "v_mfma_i32_32x32x32_i8 %2, %9, %12, %2\n\t"
        "v_mfma_i32_32x32x32_i8 %3, %9, %13, %3\n\t"
        "v_mfma_i32_32x32x32_i8 %4, %10, %12, %4\n\t"
        "v_mfma_i32_32x32x32_i8 %5, %10, %13, %5\n\t"
        "v_mfma_i32_32x32x32_i8 %6, %11, %12, %6\n\t"
        "v_mfma_i32_32x32x32_i8 %7, %11, %13, %7"
        : "+v"(acc[0][0]), "+v"(acc[0][1]), "+v"(acc[1][0]), "+v"(acc[1][1]), "+v"(acc[2][0]),
          "+v"(acc[2][1]), "+v"(acc[3][0]), "+v"(acc[3][1])
        : "v"(ac[0]), "v"(ac[1]), "v"(ac[2]), "v"(ac[3]), "v"(b[0]), "v"(b[1]));
}
template <class A, class B, class C>
__device__ inline void half_step_noread(A&, const B&, const C&) {}

// Half-step, 2 x 2 sub-tiles.
__device__ inline void half_step(v16i (&acc)[2][2], const v4i (&ac)[2], const v4i (&b)[2],
                                 v4i (&an)[2], uint32_t ad) {
    asm volatile(
        "ds_read_b128 %4, %10\n\t"
        "ds_read_b128 %5, %10 offset:2048\n\t"
        "s_nop 1\n\t"
        "v_mfma_i32_32x32x32_i8 %0, %6, %8, %0\n\t"
        "v_mfma_i32_32x32x32_i8 %1, %6, %9, %1\n\t"
        "v_mfma_i32_32x32x32_i8 %2, %7, %8, %2\n\t"
        "v_mfma_i32_32x32x32_i8 %3, %7, %9, %3\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "+v"(acc[0][0]), "+v"(acc[0][1]), "+v"(acc[1][0]), "+v"(acc[1][1]), "=&v"(an[0]),
          "=&v"(an[1])
        : "v"(ac[0]), "v"(ac[1]), "v"(b[0]), "v"(b[1]), "v"(ad));
}
// Half-step, 2 x 1 sub-tiles.
__device__ inline void half_step(v16i (&acc)[2][1], const v4i (&ac)[2], const v4i (&b)[1],
                                 v4i (&an)[2], uint32_t ad) {
    asm volatile(
        "ds_read_b128 %2, %7\n\t"
        "ds_read_b128 %3, %7 offset:2048\n\t"
        "s_nop 1\n\t"
        "v_mfma_i32_32x32x32_i8 %0, %4, %6, %0\n\t"
        "v_mfma_i32_32x32x32_i8 %1, %5, %6, %1\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "+v"(acc[0][0]), "+v"(acc[1][0]), "=&v"(an[0]), "=&v"(an[1])
        : "v"(ac[0]), "v"(ac[1]), "v"(b[0]), "v"(ad));
}

// NS = stages in the LDS ring (4 or 8: it must divide the 8 stages of a chunk)
template <int BM, int BN, int WM, int WN, int NS, int ABL = 0>
__global__ __launch_bounds__(WM * WN * 64, 2) void gemm_prefill_kernel(GemmArgs a, int grid_m,
                                                                        int grid_n) {
    constexpr int THREADS = WM * WN * kWave;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int MI = WTM / 32, NI = WTN / 32;
    constexpr int P = BM * 4 / THREADS;  // 16-byte DMA pieces per thread per stage
    constexpr int NWAVES = WM * WN;
    constexpr int NBW = (BN / 16) / NWAVES;  // packed-weight tiles (DMA pieces) per wave per chunk
    constexpr int STAGE_BYTES = BM * kStageK;
    static_assert(BM * 4 % THREADS == 0, "tile shape");
    static_assert((MI == 4 && NI == 2) || (MI == 2 && NI == 2) || (MI == 2 && NI == 1),
                  "wave tiles with an asm block");
    static_assert(NS == 4 || NS == 8, "ring size");
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
    // Global address = uniform base (block row 0, stage k) + a 32-bit per-lane offset.  Rows
    // past M re-read row M-1 (never stored).  clamp: stages that may reach past K re-read the
    // last 16 valid bytes of the row (nobody reads those buffer bytes).
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
    auto issue = [&](int st, bool clamp) {
#pragma unroll
        for (int q = 0; q < P; ++q) {
            const int8_t* src = gbase + (int64_t)st * kStageK + goff[q];
            if (clamp) {
                const int64_t k = (int64_t)st * kStageK + gseg[q];
                if (k > K - 16) src -= k - (K - 16);
            }
            __builtin_amdgcn_global_load_lds(
                (const void*)src,
                (__attribute__((address_space(3))) void*)(smA + (st % NS) * STAGE_BYTES +
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
        if (tk > TK - 1) tk = TK - 1;
#pragma unroll
        for (int q = 0; q < NBW; ++q)
            __builtin_amdgcn_global_load_lds(
                (const void*)(bsrc[q] + tk * 256),
                (__attribute__((address_space(3))) void*)(smB + (w + q * NWAVES) * 1024), 16, 0, 0);
    };
    // lane (j, g2) of sub-tile s, half h reads lane slot (2h+g2)*16 + j%16 of tile (..+j/16)
    const uint32_t b_lane = (uint32_t)(uintptr_t)smB + ((wn * WTN + j) >> 4) * 1024 +
                            (g2 * 16 + (j & 15)) * 16;
    // lane's operand address inside a stage: row (wm*WTM + j), segment (2h+g2) ^ swizzle
    const int sw = (j >> 2) & 3;
    const uint32_t a_lane[2] = {
        (uint32_t)(uintptr_t)smA + (wm * WTM + j) * kStageK + ((g2) ^ sw) * 16,
        (uint32_t)(uintptr_t)smA + (wm * WTM + j) * kStageK + ((2 + g2) ^ sw) * 16};
    auto a_addr = [&](int st, int h) { return a_lane[h] + (uint32_t)((st % NS) * STAGE_BYTES); };

    v16i acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int s = 0; s < NI; ++s)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][s][r] = 0;

    v4i bw[NI][2];  // packed bits of the current chunk
    // bit plane i of half h as {0,1} bytes; the epilogue turns sum_k q b into sum_k q (2b - 1)
    auto expand = [&](v4i (&b)[NI], int h, int i) {
#pragma unroll
        for (int s = 0; s < NI; ++s)
#pragma unroll
            for (int d = 0; d < 4; ++d) b[s][d] = (int)(((uint32_t)bw[s][h][d] >> i) & 0x01010101u);
    };

    // ---- prologue: weight bits of chunk 0, stages 0..2 in flight, operands of half-step 0 --
    issue_bits(0);
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) issue(s, true);
    wait_vmcnt<(NS - 2) * P>();  // younger than stage 0: stages 1 .. NS-2
    block_barrier();
    lds_read_bits(bw, b_lane);
    v4i ax[MI], ay[MI], bx[NI], by[NI];
    lds_read_a(ax, a_addr(0, 0));
    expand(bx, 0, 0);

    // Stage st, bit plane i = st % 8.  In: ax/bx = operands of (st, h=0).  Out: ax/bx =
    // operands of (st+1, h=0).  DMA bookkeeping at the mid-stage point: the groups younger
    // than stage st+1 are stages st+2 .. st+NS-2 ((NS-3)*P operations), plus the NBW weight
    // tiles while they are among them: the tiles are issued at i == 2 ahead of stage
    // st+NS-1's group, so they are younger than stage st+1 at i = 3 .. NS-1.  At i == 7 they
    // are never allowed to be outstanding: smB is read right after that barrier.
    auto stage = [&](int st, int i, bool clamp, bool half) {
        if (!(ABL & 4)) expand(by, 1, i);
        if (ABL & 1) half_step_noread(acc, ax, bx);
        else half_step(acc, ax, bx, ay, a_addr(st, 1));
        if (!(ABL & 8)) {
            if (i >= 3 && i <= NS - 1 && i <= 6) wait_vmcnt<(NS - 3) * P + NBW>();
            else wait_vmcnt<(NS - 3) * P>();
            block_barrier();
        }
        if (i == 7) lds_read_bits(bw, b_lane);  // bits of the next chunk (landed long ago)
        if (!(ABL & 2)) {
            if (i == 2) issue_bits((st >> 3) + 1);
            issue(st + NS - 1, clamp);
        }
        if (!half) {
            if (!(ABL & 4)) expand(bx, 0, (i + 1) & 7);
            if (ABL & 1) half_step_noread(acc, ay, by);
            else half_step(acc, ay, by, ax, a_addr(st + 1, 0));
        } else {
            lds_read_a(ax, a_addr(st + 1, 0));
        }
    };

    // Main loop: chunks whose look-ahead stays inside K (no clamps, constant folding of i).
    const int64_t kfull = K / kStageK;
    const int64_t main_chunks = kfull >= NS + 7 ? (kfull - NS - 7) / 8 + 1 : 0;
    for (int64_t tk = 0; tk < main_chunks; ++tk) {
        static_for<0, 8>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            stage((int)tk * 8 + i, i, false, false);
        });
    }
    // Remaining stages (last chunk, ragged K): same schedule with clamped addresses.
    for (int st = (int)main_chunks * 8; st < nst; ++st)
        stage(st, st & 7, true, (int64_t)st * kStageK + 32 >= K);

    // The accumulators were last written by MFMAs inside an asm block: give the matrix
    // pipeline time to retire them before ordinary instructions read them.  Also drain the
    // look-ahead DMA that ran past the end of K: it must not land after the LDS is released.
    asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");
    wait_vmcnt<0>();

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
                if ((ABL & 16) && pm != 0x12345678) continue;  // timing experiment: no stores
                if (a.out_acc) reinterpret_cast<int*>(a.Y)[m * a.N + n] = pm;
                else a.Y[m * a.N + n] = (float)pm * sc;
            }
        }
}

template <int BM, int BN, int WM, int WN, int NS, int ABL = 0>
static void launch_tile(const GemmArgs& a, hipStream_t s) {
    const int grid_m = (int)((a.M + BM - 1) / BM), grid_n = (int)((a.N + BN - 1) / BN);
    gemm_prefill_kernel<BM, BN, WM, WN, NS, ABL>
        <<<(unsigned)(grid_m * grid_n), WM * WN * kWave, 0, s>>>(a, grid_m, grid_n);
}

// K < 2^22 is required (the per-lane offset into a block of 256 rows is kept in 32 bits).
hipError_t launch_gemm_prefill(const GemmArgs& a, hipStream_t s) {
    if (a.K >= ((int64_t)1 << 22)) return hipErrorInvalidValue;
    const char* e = getenv("BITLINEAR_PREFILL_TILE");  // bench-only override: 0, 1, 2
    int pick;
    if (e) pick = atoi(e);
    else if (a.M <= 64) pick = 0;
    else {
        // 256x256 unless the 128-row tile needs fewer block-rounds of work on the 256 CUs
        auto cost = [&](int64_t bm, int64_t bn) {
            const int64_t blocks = ((a.M + bm - 1) / bm) * ((a.N + bn - 1) / bn);
            return ((blocks + 255) / 256) * bm * bn;
        };
        pick = cost(128, 256) < cost(256, 256) ? 1 : 2;
    }
    if (const char* ab = getenv("BITLINEAR_PREFILL_ABLATE")) {  // timing experiments (wrong results)
        switch (atoi(ab)) {
            case 1: launch_tile<256, 256, 2, 4, 8, 1>(a, s); break;
            case 2: launch_tile<256, 256, 2, 4, 8, 2>(a, s); break;
            case 3: launch_tile<256, 256, 2, 4, 8, 3>(a, s); break;
            case 4: launch_tile<256, 256, 2, 4, 8, 4>(a, s); break;
            case 7: launch_tile<256, 256, 2, 4, 8, 7>(a, s); break;
            case 8: launch_tile<256, 256, 2, 4, 8, 8>(a, s); break;
            case 15: launch_tile<256, 256, 2, 4, 8, 15>(a, s); break;
            case 16: launch_tile<256, 256, 2, 4, 8, 16>(a, s); break;
            case 31: launch_tile<256, 256, 2, 4, 8, 31>(a, s); break;
            case 116: launch_tile<128, 256, 2, 4, 8, 16>(a, s); break;
            case 131: launch_tile<128, 256, 2, 4, 8, 30>(a, s); break;
            default: launch_tile<256, 256, 2, 4, 8, 11>(a, s); break;
        }
        return hipGetLastError();
    }
    if (pick == 0) launch_tile<64, 128, 1, 4, 4>(a, s);
    else if (pick == 1) launch_tile<128, 256, 2, 4, 8>(a, s);
    else launch_tile<256, 256, 2, 4, 8>(a, s);
    return hipGetLastError();
}

}  // namespace bl

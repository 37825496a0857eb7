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
// Schedule.  The unit of work is a half-step: 32 k of a stage, MI*NI MFMAs.  It starts the LDS
// reads of the NEXT half-step's activation operand (asm), issues the MFMAs of the current one
// with the expansion of the next weight operand scheduled between them, then waits for the
// reads (asm): LDS latency and expansion both hide under the MFMAs.  (An LDS read the compiler
// can see makes it drain the whole DMA queue first, because it cannot tell the read from the
// DMA's target; the registers of a read in flight are tied to the asm that waits for it, so
// nothing can use them earlier.)
// Between the two half-steps of stage st every wave waits for its own DMA of stage st+1
// (s_waitcnt vmcnt(n), n counted by hand) and meets the others at a bare s_barrier (no
// fence: a fence would drain every DMA in flight).  After that barrier stage st+1 is
// readable and the buffer of stage st-1 is free, so the DMA of stage st+NS-1 goes there.
#include "common.h"
#include "kernels.h"
#include "ring.h"

namespace bl {

constexpr int kStageK = 64;  // k per LDS stage (= bytes per staged row)

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

// The LDS reads of the next half-step's operands, started here and valid at lds_wait, which ties
// the registers so that nothing the compiler schedules in between can use them earlier.
__device__ inline void lds_issue(v4i (&a)[4], uint32_t ad) {
    asm volatile(
        "ds_read_b128 %0, %4\n\t"
        "ds_read_b128 %1, %4 offset:2048\n\t"
        "ds_read_b128 %2, %4 offset:4096\n\t"
        "ds_read_b128 %3, %4 offset:6144"
        : "=&v"(a[0]), "=&v"(a[1]), "=&v"(a[2]), "=&v"(a[3])
        : "v"(ad));
}
__device__ inline void lds_issue(v4i (&a)[2], uint32_t ad) {
    asm volatile(
        "ds_read_b128 %0, %2\n\t"
        "ds_read_b128 %1, %2 offset:2048"
        : "=&v"(a[0]), "=&v"(a[1])
        : "v"(ad));
}
__device__ inline void lds_wait(v4i (&a)[4]) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]));
}
__device__ inline void lds_wait(v4i (&a)[2]) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a[0]), "+v"(a[1]));
}
// Row scale and row sum of four consecutive rows (epilogue), complete on exit.
__device__ inline void lds_read_rows(v4f& sc, v4i& rs, uint32_t ad_sc, uint32_t ad_rs) {
    asm volatile(
        "ds_read_b128 %0, %2\n\t"
        "ds_read_b128 %1, %3\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(sc), "=&v"(rs)
        : "v"(ad_sc), "v"(ad_rs));
}
__device__ inline float lds_read_f32(uint32_t ad) {
    float v;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=&v"(v) : "v"(ad));
    return v;
}
__device__ inline void lds_write_b32(uint32_t ad, uint32_t v) {
    asm volatile("ds_write_b32 %0, %1" : : "v"(ad), "v"(v) : "memory");
}

// NS = stages in the LDS ring (4 or 8: it must divide the 8 stages of a chunk).
// Persistent: gridDim.x workgroups (one per CU) walk the tiles t = blockIdx.x, + gridDim.x, ...
// GEN = false: the plain layer (one beta, Y = result): nothing of what follows costs anything.
// GEN = true adds beta per column group (Eq. 13), accumulation over K-groups, the shift term of
// Eq. 6.
// KGRP = true (with GEN): all a.kgroups K-groups of a grouped layer (Eq. 13-15) in this launch.  A
// work item is (tile, group), the groups of a tile following each other on the same workgroup:
// each group's int32 sums are dequantised with that group's beta_g gamma_g / 128 (and shifted by
// its eta_g) into an fp32 register copy of the tile, which is stored once, after the last group.
template <int BM, int BN, int WM, int WN, int NS, bool GEN, bool KGRP = false>
__global__ __launch_bounds__(WM * WN * 64, 2) void gemm_prefill_kernel(GemmArgs a, int grid_m,
                                                                        int grid_n, int xbm) {
    constexpr int THREADS = WM * WN * kWave;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int MI = WTM / 32, NI = WTN / 32;
    constexpr int P = BM * 4 / THREADS;  // 16-byte DMA pieces per thread per stage
    constexpr int NWAVES = WM * WN;
    constexpr int NBW = (BN / 16) / NWAVES;  // packed-weight tiles (DMA pieces) per wave per chunk
    constexpr int STAGE_BYTES = BM * kStageK;
    static_assert(BM * 4 % THREADS == 0, "tile shape");
    static_assert((MI == 4 && NI == 2) || (MI == 2 && NI == 2), "wave tiles with LDS-read asm blocks");
    static_assert(NS == 4 || NS == 8, "ring size");
    static_assert((BN / 16) % NWAVES == 0 && (NS - 2) * P + NBW < 64, "tile shape");

    __shared__ __attribute__((aligned(1024))) uint8_t smA[NS * STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) uint8_t smB[(BN / 16) * 1024];
    __shared__ __attribute__((aligned(16))) float smScale[2][BM];  // gamma_m / 128, per tile parity
    __shared__ __attribute__((aligned(16))) float smBeta[2][GEN ? BN : 4];  // beta of each column's group
    __shared__ __attribute__((aligned(16))) float smEta[2][GEN ? BM : 4];   // Eq. 6 only: eta_m
    __shared__ __attribute__((aligned(16))) int smWsum[2][GEN ? BN : 4];    // Eq. 6 only: sum_k s[n,k]
    __shared__ __attribute__((aligned(16))) int smRowsum[2][BM];   // sum_k q[m,k]

    const int w = threadIdx.x / kWave, l = threadIdx.x % kWave;
    const int wm = w / WN, wn = w % WN;
    const int j = l & 31, g2 = l >> 5;
    const int64_t TN = tiles_n(a.N);
    const int64_t M = a.M;
    const int64_t K = a.K, TK = tiles_k(K);
    const int nst = (int)((K + kStageK - 1) / kStageK);
    const int64_t kfull = K / kStageK;
    // chunks whose look-ahead stays inside K and that have a successor chunk
    const int64_t main_chunks = kfull >= NS + 7 ? (kfull - NS - 7) / 8 + 1 : 0;
    const int64_t TKp = a.tk_pitch ? a.tk_pitch : tiles_k(a.K);  // tiles per tile row in memory
    const int ntiles = grid_m * grid_n;

    // Tile order.  Workgroups are dealt round-robin to the 8 XCDs, each with its own L2; give
    // each XCD one contiguous range of the tile sequence, so that the tiles running together on
    // an XCD share operands in its L2.  The sequence walks bands of xbm rows of tiles, inside a
    // band the rows fastest: an XCD's range is then a block of xbm x (range / xbm) tiles and it
    // fetches xbm row blocks of codes (BM x K bytes each) and range / xbm column blocks of packed
    // weights (BN x K / 8 bytes each).  xbm = 1 unless the host asks otherwise (see launch_tile).
    auto tile_origin = [&](int t, int64_t& m0, int64_t& n0) {
        int logical = t;
        const int G = (int)gridDim.x;
        if ((ntiles & 7) == 0 && (G & 7) == 0) {
            const int q = ((t % G) >> 3) + (t / G) * (G >> 3);  // index inside the XCD's range
            logical = (t & 7) * (ntiles >> 3) + q;
            // the XCD's range may end before the last round does
            if (q >= (ntiles >> 3)) logical = -1;
        }
        int tm = logical / grid_n, tn = logical % grid_n;
        if (xbm > 1 && logical >= 0) {
            const int band = logical / (xbm * grid_n), rem = logical - band * xbm * grid_n;
            const int rows = min(xbm, grid_m - band * xbm);  // the last band may be lower
            tm = band * xbm + rem % rows;
            tn = rem / rows;
        }
        m0 = logical < 0 ? -1 : (int64_t)tm * BM;
        n0 = logical < 0 ? -1 : (int64_t)tn * BN;
    };

    // ---- DMA of one stage: thread -> P pieces; piece = (row, swizzled 16-byte segment) ----
    // Global address = uniform base (tile row 0, stage k) + a 32-bit per-lane offset.  Rows
    // past M re-read row M-1 (never stored).  clamp: stages that may reach past K re-read the
    // last 16 valid bytes of the row (nobody reads those buffer bytes).
    uint32_t goff[P];
    int gseg[P];
    const int8_t* gbase = a.codes;
    const uint32_t* bsrc[NBW];
    auto setup_dma = [&](int64_t m0, int64_t n0, int grp) {
#pragma unroll
        for (int q = 0; q < P; ++q) {
            const int slot = q * THREADS + threadIdx.x;
            int row = slot >> 2;
            gseg[q] = ((slot & 3) ^ ((row >> 2) & 3)) * 16;
            if (m0 + row > M - 1) row = (int)(M - 1 - m0);
            goff[q] = (uint32_t)row * (uint32_t)a.ldq + gseg[q];
        }
        gbase = a.codes + m0 * a.ldq + (KGRP ? (int64_t)grp * K : 0);
        // packed weights: tile t of the block goes to smB + t KiB, lane for lane as it lies in
        // memory; wave w moves tiles w, w + NWAVES, ...  Columns past N read a valid tile.
#pragma unroll
        for (int q = 0; q < NBW; ++q) {
            int64_t tn = (n0 >> 4) + w + q * NWAVES;
            if (tn > TN - 1) tn = TN - 1;
            bsrc[q] = a.packed + (KGRP ? (int64_t)grp * a.group_packed : 0) +
                      tile_dword_offset(tn, 0, TKp) + l * 4;
        }
    };
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
    auto issue_bits = [&](int64_t tk) {
#pragma unroll
        for (int q = 0; q < NBW; ++q)
            __builtin_amdgcn_global_load_lds(
                (const void*)(bsrc[q] + tk * 256),
                (__attribute__((address_space(3))) void*)(smB + (w + q * NWAVES) * 1024), 16, 0, 0);
    };
    // what a tile starts with: weight bits of chunk 0 and stages 0 .. NS-2 (clamped: K may be short)
    auto issue_tile_start = [&]() {
        issue_bits(0);
#pragma unroll
        for (int s = 0; s < NS - 1; ++s) issue(s, true);
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
    v4i bw[NI][2];  // packed bits of the current chunk
    // bit plane i of half h as {0,1} bytes; the epilogue turns sum_k q b into sum_k q (2b - 1)
    auto expand = [&](v4i (&b)[NI], int h, int i) {
#pragma unroll
        for (int s = 0; s < NI; ++s)
#pragma unroll
            for (int d = 0; d < 4; ++d) b[s][d] = (int)(((uint32_t)bw[s][h][d] >> i) & 0x01010101u);
    };
    v4i ax[MI], ay[MI], bx[NI], by[NI];
    // One half-step (32 k of a stage): acc += ac x b, MI * NI MFMAs, with the next half-step's
    // weight operand bn = plane i of half h expanded BETWEEN them (the compiler's scheduler is told
    // so with sched_group_barrier: one MFMA, then the two vector ALU operations of a dword, ...), so
    // that a wave expands under its own MFMAs instead of ahead of them; the operands at `ad` are
    // read into an meanwhile (valid on return).  Against an asm block of the MFMAs with the
    // expansion ahead of it: 117 against 129 us on 2048 x 4096 x 16384, 1-2 % on the longer K.
    auto half_step = [&](const v4i(&ac)[MI], const v4i(&b)[NI], v4i(&bn)[NI], int h, int i,
                          v4i(&an)[MI], uint32_t ad) {
        lds_issue(an, ad);
        // the bits pass through an (empty) asm placed after the reads, and the new operand through
        // one at the end: the expansion can neither be moved ahead of this half-step nor be left
        // for a later one before the scheduler sees the groups below
        asm volatile("" : "+v"(bw[0][h]), "+v"(bw[1][h]));
        __builtin_amdgcn_sched_barrier(0);
        constexpr int DW = NI * 4 / (MI * NI);  // dwords of the new operand per MFMA: 1 or 2
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int s = 0; s < NI; ++s) {
                acc[mi][s] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ac[mi], b[s], acc[mi][s], 0, 0, 0);
                const int q = mi * NI + s;
#pragma unroll
                for (int e = 0; e < DW; ++e) {
                    const int idx = q * DW + e;  // 0 .. NI*4-1
                    bn[idx >> 2][idx & 3] = (int)(((uint32_t)bw[idx >> 2][h][idx & 3] >> i) & 0x01010101u);
                }
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 2 * DW, 0);
            }
        asm volatile("" : "+v"(bn[0]), "+v"(bn[1]));
        __builtin_amdgcn_sched_barrier(0);
        lds_wait(an);
    };

    // Stage st, bit plane i = st % 8.  In: ax/bx = operands of (st, h=0).  Out: ax/bx =
    // operands of (st+1, h=0).  DMA bookkeeping at the mid-stage point, while the look-ahead
    // stage st+NS-1 exists (`ahead`): the groups younger than stage st+1 are stages st+2 ..
    // st+NS-2 ((NS-3)*P operations), plus the NBW weight tiles while they are among them: the
    // tiles are issued at i == 2 ahead of stage st+NS-1's group, so they are younger than stage
    // st+1 at i = 3 .. NS-1.  At i == 7 they are never allowed to be outstanding: smB is read
    // right after that barrier.  Near the end of K nothing more is issued and the wait is for
    // everything outstanding (all of it is needed within the next NS-2 stages).
    auto stage = [&](int st, int i, bool clamp, bool half, bool ahead, bool bits_in_flight) {
        half_step(ax, bx, by, 1, i, ay, a_addr(st, 1));
        if (!ahead) wait_vmcnt<0>();
        else if (bits_in_flight && i >= 3 && i <= NS - 1 && i <= 6) wait_vmcnt<(NS - 3) * P + NBW>();
        else wait_vmcnt<(NS - 3) * P>();
        block_barrier();
        if (i == 7) lds_read_bits(bw, b_lane);  // bits of the next chunk (landed long ago)
        if (i == 2 && (st >> 3) + 1 < TK) issue_bits((st >> 3) + 1);
        if (ahead) issue(st + NS - 1, clamp);
        if (!half) {
            half_step(ay, by, bx, 0, (i + 1) & 7, ax, a_addr(st + 1, 0));
        }
    };

    int t = (int)blockIdx.x, parity = 0;
    int grp = 0;  // KGRP: the K-group of the current work item
    const int ngroups = KGRP ? a.kgroups : 1;
    int64_t m0, n0;
    tile_origin(t, m0, n0);
    if (m0 < 0) return;  // uniform for the whole workgroup
    setup_dma(m0, n0, 0);
    issue_tile_start();
    float side[KGRP ? MI : 1][KGRP ? NI : 1][16];  // KGRP: the tile's sum over the groups so far

    while (true) {
        if constexpr (GEN) {
            // Per-row gamma and row sum of the codes, per-column beta (Eq. 11, Eq. 13), for the
            // epilogue.  Thread i serves row i and column i (BM, BN <= THREADS); every load is
            // issued before the first value is needed, so the tile pays one memory latency here.
            {
                static_assert(BM <= THREADS && BN <= THREADS, "one row and one column per thread");
                const int i = threadIdx.x;
                const int64_t m = m0 + i < M ? m0 + i : M - 1;
                int64_t n = n0 + i;
                if (n > a.N - 1) n = a.N - 1;
                // branch-free (a branch here makes the compiler drain the loads issued so far):
                // with one beta for the matrix the quotient is 0 by itself; the Eq. 6 operands are
                // read from a valid stand-in address when they are not in use
                const uint32_t bg = (uint32_t)n / (uint32_t)a.beta_rows;
                // KGRP: group grp's entries lie grp further on (gamma, rowsum, eta: [M][groups] or
                // [groups] per tensor; beta: [row groups][groups]); wsum: [groups][N]
                const int64_t go = KGRP ? grp : 0;
                const float gm = a.gamma[(a.per_tensor ? 0 : m * a.gstride) + go];
                const int rs = a.rowsum[m * a.gstride + go];
                const float b = a.beta[bg * a.beta_stride + go];
                const float e = *(a.eta ? a.eta + (a.per_tensor ? 0 : m * a.gstride) + go : a.gamma);
                const int ws = *(a.eta ? a.wsum + go * a.N + n : a.rowsum);
                if (i < BM) {
                    // gamma / 128 is exact, so beta * (gamma / 128) has the bits of (beta * gamma) / 128
                    lds_write_b32((uint32_t)(uintptr_t)&smScale[parity][i], __float_as_uint(gm * 0.0078125f));
                    lds_write_b32((uint32_t)(uintptr_t)&smRowsum[parity][i], (uint32_t)rs);
                    lds_write_b32((uint32_t)(uintptr_t)&smEta[parity][i], __float_as_uint(e));
                }
                if (i < BN) {
                    lds_write_b32((uint32_t)(uintptr_t)&smBeta[parity][i], __float_as_uint(b));
                    lds_write_b32((uint32_t)(uintptr_t)&smWsum[parity][i], (uint32_t)ws);
                }
            }
        } else {
            // per-row dequantisation scale (Eq. 11) and row sum of the codes, for the epilogue
            const float beta = *a.beta;
            for (int r = threadIdx.x; r < BM; r += THREADS) {
                const int64_t m = m0 + r;
                float sc = 0.f;
                int rs = 0;
                if (m < M) {
                    sc = (beta * (a.per_tensor ? a.gamma[0] : a.gamma[m])) / 128.0f;
                    rs = a.rowsum[m];
                }
                lds_write_b32((uint32_t)(uintptr_t)&smScale[parity][r], __float_as_uint(sc));
                lds_write_b32((uint32_t)(uintptr_t)&smRowsum[parity][r], (uint32_t)rs);
            }
        }
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int s = 0; s < NI; ++s)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mi][s][r] = 0;

        // stage 0 and the bits of chunk 0 have landed; operands of half-step 0
        wait_vmcnt<(NS - 2) * P>();  // younger than stage 0: stages 1 .. NS-2
        block_barrier();
        lds_read_bits(bw, b_lane);
        lds_read_a(ax, a_addr(0, 0));
        expand(bx, 0, 0);

        // Main loop: no clamps, i folds to a constant.  Then the remaining stages.
        for (int64_t tk = 0; tk < main_chunks; ++tk) {
            static_for<0, 8>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                stage((int)tk * 8 + i, i, false, false, true, true);
            });
        }
        for (int st = (int)main_chunks * 8; st < nst; ++st)
            stage(st, st & 7, true, (int64_t)st * kStageK + 32 >= K, st + NS - 1 < nst,
                  (st >> 3) + 1 < TK);

        // Every wave is done with the LDS ring: start the next tile's stream, then store.
        block_barrier();
        // the next work item: the tile's next K-group, else the workgroup's next tile
        const bool last_group = !KGRP || grp + 1 == ngroups;
        const int grp_next = last_group ? 0 : grp + 1;
        const int t_next = last_group ? t + (int)gridDim.x : t;
        int64_t m0n = -1, n0n = -1;
        if (!last_group) m0n = m0, n0n = n0;
        else if (t_next < ntiles) tile_origin(t_next, m0n, n0n);
        if (m0n >= 0) {
            setup_dma(m0n, n0n, grp_next);
            issue_tile_start();
        }

        // ---- epilogue (Eq. 11): lane (j, g2) holds column n, rows 8*(r/4) + 4*g2 + r%4 ----
        //   sum_k q s = 2 sum_k q b - sum_k q ;  y = that * (beta_n * gamma_m / 128)
        float bcol[NI];
#pragma unroll
        for (int s = 0; s < NI; ++s)
            bcol[s] = GEN ? lds_read_f32((uint32_t)(uintptr_t)&smBeta[parity][wn * WTN + 32 * s + j])
                          : 1.f;
        const uint32_t sc_base = (uint32_t)(uintptr_t)&smScale[parity][wm * WTM + 4 * g2];
        const uint32_t rs_base = (uint32_t)(uintptr_t)&smRowsum[parity][wm * WTM + 4 * g2];
        const bool special = a.out_acc || (GEN && (a.eta != nullptr || a.accumulate));
        float wcol[NI];  // Eq. 6 only
#pragma unroll
        for (int s = 0; s < NI; ++s)
            wcol[s] = (GEN && a.eta) ? (float)__float_as_int(lds_read_f32(
                                  (uint32_t)(uintptr_t)&smWsum[parity][wn * WTN + 32 * s + j]))
                            : 0.f;
        // Register allocation here is at the limit of 256 and sensitive to the form of these
        // loops: hoisting the uniform branches into a second copy of the loops, or naming the
        // row index as a 32-bit temporary, makes the compiler precompute the store addresses and
        // spill over a hundred registers.  Check the resource usage after any change.
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                v4f sc4;
                v4i rs4;
                lds_read_rows(sc4, rs4, sc_base + (32 * mi + 8 * rq) * 4, rs_base + (32 * mi + 8 * rq) * 4);
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    const int r = rq * 4 + rr;
                    const int64_t m = m0 + wm * WTM + 32 * mi + 8 * rq + 4 * g2 + rr;
                    if (m >= M) continue;
#pragma unroll
                    for (int s = 0; s < NI; ++s) {
                        const int64_t n = n0 + wn * WTN + 32 * s + j;
                        if (n >= a.N) continue;
                        const int pm = 2 * acc[mi][s][r] - rs4[rr];
                        // y = acc * ((beta * gamma) / 128)
                        // (GEN: sc4 holds gamma / 128, else the whole scale)
                        float y = GEN ? (float)pm * (bcol[s] * sc4[rr]) : (float)pm * sc4[rr];
                        if constexpr (KGRP) {
                            if (a.eta) {  // Eq. 6 / Eq. 14: + (beta_g * eta_g) * sum_{k in g} s[n,k]
                                const float e = lds_read_f32(
                                    (uint32_t)(uintptr_t)&smEta[parity][wm * WTM + 32 * mi + 8 * rq + 4 * g2 + rr]);
                                y = y + (bcol[s] * e) * wcol[s];
                            }
                            // groups are added in the order 0, 1, ... (as launches per group would)
                            if (grp) y = y + side[mi][s][r];
                            side[mi][s][r] = y;
                            if (!last_group) continue;
                            __builtin_nontemporal_store(y, &a.Y[m * a.N + n]);
                            continue;
                        }
                        if (special) {  // uniform
                            if (a.out_acc) {
                                reinterpret_cast<int*>(a.Y)[m * a.N + n] = pm;
                                continue;
                            }
                            if (GEN && a.eta) {  // Eq. 6: + (beta * eta_m) * sum_k s[n,k]
                                const float e = lds_read_f32(
                                    (uint32_t)(uintptr_t)&smEta[parity][wm * WTM + 32 * mi + 8 * rq + 4 * g2 + rr]);
                                y = y + (bcol[s] * e) * wcol[s];
                            }
                            if (GEN && a.accumulate) y += a.Y[m * a.N + n];  // a later K-group
                        }
                        // streaming store: the output is not read again soon, and keeping it out
                        // of L2 leaves the codes and bits there (3-4 % of the kernel)
                        __builtin_nontemporal_store(y, &a.Y[m * a.N + n]);
                    }
                }
            }
        if (m0n < 0) break;
        t = t_next;
        grp = grp_next;
        m0 = m0n;
        n0 = n0n;
        parity ^= 1;
    }
}

static int num_cus() {
    static int n = 0;
    if (n == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            n = prop.multiProcessorCount;
        if (n <= 0) n = 256;
    }
    return n;
}

template <int BM, int BN, int WM, int WN, int NS>
static void launch_tile(const GemmArgs& a, hipStream_t s) {
    const bool plain = a.beta_rows >= a.N && a.gstride == 1 && !a.eta && !a.accumulate;
    const int grid_m = (int)((a.M + BM - 1) / BM), grid_n = (int)((a.N + BN - 1) / BN);
    const int ntiles = grid_m * grid_n;
    int grid = num_cus();  // one workgroup per CU
    if (tuning().prefill_grid > 0) grid = tuning().prefill_grid;
    if (grid > ntiles) grid = ntiles;
    // Rows of tiles in an XCD's block.  One row (the XCD's tiles share their codes and stream all
    // the packed weights) is the fastest on every shape measured, although two or four rows fetch
    // fewer bytes: 2048 x 4096 x 16384 takes 115.2 us with 1 (84 MB fetched per launch), 117.5 us
    // with 2 (55 MB), 124.1 us with 4 (medians of 12 alternating runs); the kernel is not bound by
    // HBM.  prefill_xbm overrides.
    int xbm = 1;
    if ((ntiles & 7) == 0 && (grid & 7) == 0 && tuning().prefill_xbm > 0)
        xbm = tuning().prefill_xbm < grid_m ? tuning().prefill_xbm : grid_m;
    if constexpr (BM == 128) {
        if (a.kgroups > 1) {  // all K-groups of a grouped layer in this launch
            gemm_prefill_kernel<BM, BN, WM, WN, NS, true, true>
                <<<(unsigned)grid, WM * WN * kWave, 0, s>>>(a, grid_m, grid_n, xbm);
            return;
        }
    }
    if (plain)
        gemm_prefill_kernel<BM, BN, WM, WN, NS, false>
            <<<(unsigned)grid, WM * WN * kWave, 0, s>>>(a, grid_m, grid_n, xbm);
    else
        gemm_prefill_kernel<BM, BN, WM, WN, NS, true>
            <<<(unsigned)grid, WM * WN * kWave, 0, s>>>(a, grid_m, grid_n, xbm);
}

// K < 2^22 is required (the per-lane offset into a block of 256 rows is kept in 32 bits).
hipError_t launch_gemm_prefill(const GemmArgs& a_in, hipStream_t s) {
    GemmArgs a = a_in;
    a.split_k = 0;  // set here only
    if (a.K >= ((int64_t)1 << 22) || a.ldq >= ((int64_t)1 << 22)) return hipErrorInvalidValue;
    int pick;
    if (tuning().prefill_tile) pick = tuning().prefill_tile;
    else if (a.M <= 64) pick = 0;
    else {
        // 256x256 unless the 128-row tile needs fewer block-rounds of work on the CUs.  A 128-row
        // tile expands every weight bit for half as many MFMAs: per unit of work it measured
        // 1.12-1.17 times the 256-row tile's time (4096 x 7168 x 21504: 530 us in 11 rounds of
        // 128-row tiles, 514 us in 6 rounds of 256-row tiles), hence the 8/7.
        const int64_t cus = num_cus();
        auto cost = [&](int64_t bm, int64_t bn) {
            const int64_t blocks = ((a.M + bm - 1) / bm) * ((a.N + bn - 1) / bn);
            return ((blocks + cus - 1) / cus) * bm * bn * (bm == 128 ? 8 : 7);
        };
        pick = cost(128, 256) < cost(256, 256) ? 1 : 2;
    }
    if (a.M <= 64) {  // up to 32 tokens: gemm_stream.hip where it takes the shape; else gemm_mid.hip
        if (!tuning().mid_only && a_in.kgroups <= 1 && launch_gemm_stream(a_in, s)) return hipGetLastError();
        return launch_gemm_mid(a_in, s);
    }
    // K-groups in one launch: the 128-row tile, whose accumulators leave room for the fp32 copy
    if (a.kgroups > 1) pick = 1;
    if (pick == 1) launch_tile<128, 256, 2, 4, 8>(a, s);
    else launch_tile<256, 256, 2, 4, 8>(a, s);
    return hipGetLastError();
}

}  // namespace bl

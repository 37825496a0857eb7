// 1-bit x 8-bit GEMM + dequantisation for a few dozen tokens (16 < M <= 64), Eq. 7 and Eq. 11
// of arXiv 2310.11453: the batch between the weight-streaming kernel (M <= 16) and the large
// MFMA tiles.  One 64 x 128 output tile per workgroup gives at most a few hundred workgroups,
// each with a long serial walk over K, so the walk is split INSIDE the workgroup: eight waves,
// four K-groups of two waves (64 x 64 each), each group streaming its own quarter of K through
// its own LDS ring (codes and packed bits by global_load_lds, bits expanded in registers,
// hand-counted vmcnt), all groups meeting at the same barriers.  The integer accumulators of
// the four groups are added through LDS at the end and one epilogue dequantises: the same
// integers as any other split of K, so the result does not depend on it.
//
// What bounds this shape is the stream of activation codes from L2 into LDS: every workgroup
// reads all M x K of them (64 bytes per k against 16 bytes of packed weights), 100 MB per launch
// at the 30B shapes.  L2 serves whole 128-byte lines, so a stage holds 128 k: a row of a stage
// is one line, and the eight lanes that fetch it sit in one DMA instruction.  (With 64-k stages
// every line was requested twice, half of it each time, and the kernel ran at the L2's request
// rate: 1.79 M requests of 128 bytes per launch for 128 MB of operands.)
//
// A wave expands its weight bits to {0,1} operand bytes with two vector ALU operations per dword,
// for an operand that only two MFMAs use.  That work sits between the MFMAs of the half-step
// before (the compiler's scheduler is told so with sched_group_barrier), two half-steps ahead of
// its use, so a wave keeps the matrix pipe fed without help from the other wave of its SIMD.
#include "common.h"
#include "kernels.h"
#include "ring.h"

namespace bl {

namespace mid {
constexpr int BM = 64, BN = 128, KG = 4, WN = 2;
constexpr int THREADS = KG * WN * kWave;      // 512
constexpr int GT = WN * kWave;                // threads of a K-group
constexpr int STAGE_K = 128;                  // k per stage: a row of a stage is one 128-byte line
constexpr int STAGE_BYTES = BM * STAGE_K;     // 8 KiB
constexpr int P = BM * (STAGE_K / 16) / GT;   // 16-byte DMA pieces per thread and stage: 4
constexpr int NBW = (BN / 16) / WN;           // packed tiles per wave and chunk: 4
constexpr int SPC = kChunkK / STAGE_K;        // stages per 512-chunk: 4
static_assert(P == 4 && NBW == 4 && SPC == 4, "tile shape");

// operands of one half-step (rows j and 32 + j of the stage), complete on exit
__device__ inline void read_a(v4i (&a)[2], uint32_t ad) {
    asm volatile(
        "ds_read_b128 %0, %2\n\t"
        "ds_read_b128 %1, %2 offset:4096\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(a[0]), "=&v"(a[1])
        : "v"(ad));
}
// packed bits of the lane's two columns (sub-tile s at +2048), two halves of a chunk (+512)
__device__ inline void read_bits(v4i (&bw)[2][2], uint32_t ad) {
    asm volatile(
        "ds_read_b128 %0, %4\n\t"
        "ds_read_b128 %1, %4 offset:512\n\t"
        "ds_read_b128 %2, %4 offset:2048\n\t"
        "ds_read_b128 %3, %4 offset:2560\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(bw[0][0]), "=&v"(bw[0][1]), "=&v"(bw[1][0]), "=&v"(bw[1][1])
        : "v"(ad));
}
// The LDS reads stay in asm (a read the compiler can see makes it wait for every DMA in flight).
// lds_issue starts the reads of the next half-step's operands; they become valid at lds_wait,
// which ties the registers so that nothing the compiler schedules can use them earlier.
__device__ inline void lds_issue(v4i (&a)[2], uint32_t ad) {
    asm volatile(
        "ds_read_b128 %0, %2\n\t"
        "ds_read_b128 %1, %2 offset:4096"
        : "=&v"(a[0]), "=&v"(a[1])
        : "v"(ad));
}
__device__ inline void lds_wait(v4i (&a)[2]) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a[0]), "+v"(a[1]));
}
}  // namespace mid

// Work item = (column tile, K-slice): blockIdx.x = slice * grid_n + tile.  With a.split_k the
// slice's partial sums 2 * sum_k q b go to a.split_ws and splitk_reduce finishes; otherwise the
// workgroup owns all of K and writes Y.
// gmode 2 (a grouped layer, Eq. 13-15): a work item is (column tile, four K-groups of the layer), one
// per K-group of the workgroup: each walks its own layer group's K (its own columns of the codes,
// its own blob) and its sums go, without being added, to that group's slice of a.split_ws.
// gmode 1: a work item is (column tile, one K-group of the layer), split over the workgroup's four.
// NS = stages in each group's ring.
template <int NS>
__global__ __launch_bounds__(mid::THREADS) void gemm_mid_kernel(GemmArgs a, int grid_n, int gmode) {
    using namespace mid;
    // rings of the four K-groups; after the walk the same bytes hold two 64 x 128 int32 sums
    __shared__ __attribute__((aligned(1024))) uint8_t smA[KG * NS * STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) uint8_t smB[KG * (BN / 16) * 1024];
    static_assert(KG * NS * STAGE_BYTES >= 2 * BM * BN * 4, "room for the reduction");
    static_assert(NS >= 4, "the wait bookkeeping below: a stage's codes are requested NS-1 >= 3 stages ahead");

    // wave-uniform values in scalar registers: the loop below branches on them
    const int w = __builtin_amdgcn_readfirstlane((int)threadIdx.x / kWave), l = threadIdx.x % kWave;
    const int kg = w / WN, wn = w % WN;
    const int tg = threadIdx.x % GT;  // thread inside the K-group
    const int j = l & 31, g2 = l >> 5;
    const int64_t M = a.M, N = a.N;
    const int64_t TN = tiles_n(N);
    const int64_t TKp = a.tk_pitch ? a.tk_pitch : tiles_k(a.K);
    const int sp = (int)blockIdx.x / grid_n;
    const int64_t n0 = (int64_t)((int)blockIdx.x % grid_n) * BN;

    // ---- this item's slice of K, then this group's chunks of it ----------------------------
    int64_t ki0 = 0, Ki = a.K;
    const bool to_slices = a.split_k || a.kgroups > 1;  // partial sums go to split_ws
    const int lgrp = gmode == 2 ? sp * KG + kg : sp;  // gmode 1, 2: the layer's K-group walked here
    if (gmode) {  // a K-group of a grouped layer: its own codes columns and blob
        const int gi = lgrp < a.kgroups ? lgrp : a.kgroups - 1;
        a.codes += (int64_t)gi * a.K;
        a.packed += (int64_t)gi * a.group_packed;
    } else if (a.split_k) {
        ki0 = (int64_t)sp * a.split_k;
        Ki = a.K - ki0 < a.split_k ? a.K - ki0 : a.split_k;
    }
    const int64_t TKi = tiles_k(Ki);
    // gmode 2: the whole group (nothing for a group past the layer's last)
    const int64_t c0 = gmode == 2 ? 0 : TKi * kg / KG;
    const int64_t c1 = gmode == 2 ? (lgrp < a.kgroups ? TKi : 0) : TKi * (kg + 1) / KG;
    const int64_t k0 = ki0 + c0 * kChunkK;
    int64_t K = Ki - c0 * kChunkK;  // this group's K
    if (K > (c1 - c0) * kChunkK) K = (c1 - c0) * kChunkK;
    if (c1 == c0) K = 0;
    const int64_t TK = c1 - c0;
    // Every group walks the same number of stages, whole chunks of the longest group; what lies
    // past a group's own K meets zero bits (padding of its last chunk, or a zero mask past its
    // last chunk), so it adds nothing.
    int64_t TKmax = 0;
#pragma unroll
    for (int g = 0; g < KG; ++g) {
        const int64_t d = TKi * (g + 1) / KG - TKi * g / KG;
        TKmax = d > TKmax ? d : TKmax;
    }
    if (gmode == 2) TKmax = TKi;
    const int nrun = (int)TKmax * SPC;

    // ---- epilogue operands of this thread's outputs, requested now ---------------------------
    // thread -> columns nq .. nq+3 of the tile, rows er + 16 h
    constexpr int EH = BM * (BN / 4) / THREADS;  // 4
    constexpr int ER = THREADS / (BN / 4);       // 16
    const int er = (int)threadIdx.x >> 5;
    const int64_t nq = n0 + (threadIdx.x & 31) * 4;
    float e_gamma[EH], e_eta[EH];
    int e_rs[EH];
#pragma unroll
    for (int h = 0; h < EH; ++h) {
        const int64_t m = er + ER * h < M ? er + ER * h : M - 1;
        e_gamma[h] = a.gamma[a.per_tensor ? 0 : m * a.gstride];
        e_rs[h] = a.rowsum[m * a.gstride];
        e_eta[h] = *(a.eta ? a.eta + (a.per_tensor ? 0 : m * a.gstride) : a.gamma);
    }
    float e_beta[4];
    int e_ws[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const int64_t n = nq + c < N ? nq + c : N - 1;
        e_beta[c] = a.beta[((uint32_t)n / (uint32_t)a.beta_rows) * a.beta_stride];
        e_ws[c] = *(a.eta ? a.wsum + n : a.rowsum);
    }

    // ---- DMA of this group.  A stage is 64 rows of 128 bytes; thread -> four 16-byte pieces of
    // it, piece = (row, physical segment).  The eight lanes of a row sit in one instruction, so
    // the row's line is requested once.  Segments are XOR-swizzled with (row / 2) % 8: the
    // 16-byte operand reads of 16 consecutive rows then touch every LDS bank exactly once.
    uint8_t* const ringA = smA + kg * (NS * STAGE_BYTES);
    uint8_t* const ringB = smB + kg * ((BN / 16) * 1024);
    const int8_t* gsrc[P];
    int gseg[P];
#pragma unroll
    for (int q = 0; q < P; ++q) {
        const int slot = q * GT + tg;
        int row = slot >> 3;
        gseg[q] = ((slot & 7) ^ ((row >> 1) & 7)) * 16;
        if (row > M - 1) row = (int)(M - 1);
        gsrc[q] = a.codes + (int64_t)row * a.ldq + k0 + gseg[q];
    }
    const uint32_t* bsrc[NBW];
#pragma unroll
    for (int q = 0; q < NBW; ++q) {
        int64_t tn = (n0 >> 4) + wn + q * WN;
        if (tn > TN - 1) tn = TN - 1;
        bsrc[q] = a.packed + tile_dword_offset(tn, k0 / kChunkK, TKp) + l * 4;
    }
    const uint32_t lds_wave = (uint32_t)(wn * kWave * 16);
    // clamp: a stage that may reach past the group's K re-reads the last 16 valid bytes of the
    // row instead (the packed bits there are zero, or masked)
    auto issue = [&](int st, bool clamp) {
#pragma unroll
        for (int q = 0; q < P; ++q) {
            const int8_t* src = gsrc[q] + (int64_t)st * STAGE_K;
            if (clamp) {
                const int64_t k = (int64_t)st * STAGE_K + gseg[q];
                if (k > K - 16) src -= k - (K - 16);
            }
            __builtin_amdgcn_global_load_lds(
                (const void*)src,
                (__attribute__((address_space(3))) void*)(ringA + (st % NS) * STAGE_BYTES +
                                                          q * GT * 16 + lds_wave),
                16, 0, 0);
        }
    };
    auto issue_bits = [&](int64_t tk) {
#pragma unroll
        for (int q = 0; q < NBW; ++q)
            __builtin_amdgcn_global_load_lds(
                (const void*)(bsrc[q] + tk * 256),
                (__attribute__((address_space(3))) void*)(ringB + (wn + q * WN) * 1024), 16, 0, 0);
    };

    const uint32_t b_lane = (uint32_t)(uintptr_t)ringB + ((wn * 64 + j) >> 4) * 1024 +
                            (g2 * 16 + (j & 15)) * 16;
    // lane (j, g2) reads logical segment 2 hs + g2 of row j in half-step hs of a stage
    const int sw = (j >> 1) & 7;
    uint32_t a_lane[4];
#pragma unroll
    for (int hs = 0; hs < 4; ++hs)
        a_lane[hs] = (uint32_t)(uintptr_t)ringA + j * STAGE_K + ((2 * hs + g2) ^ sw) * 16;
    auto a_addr = [&](int st, int hs) { return a_lane[hs] + (uint32_t)((st % NS) * STAGE_BYTES); };

    v16i acc[2][2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][s2][r] = 0;
    // Packed bits of the current chunk and of the next one; plane i of half h of a chunk as {0,1}
    // bytes, nothing past the group's last chunk.  Half-step u of a chunk (plane u / 2, half u % 2)
    // multiplies A[u % 2] by B[u % 4], starts the LDS reads of A[(u + 1) % 2] and builds B[(u + 2) % 4].
    v4i bw[2][2], bwn[2][2];
    v4i A[2][2], B[4][2];
    const bool has_k = TK > 0;  // a group without chunks requests nothing and multiplies by zero

    if (has_k) {
        issue_bits(0);
#pragma unroll
        for (int s = 0; s < NS - 1; ++s) issue(s, true);
    }
    wait_vmcnt<(NS - 2) * P>();  // younger than stage 0: stages 1 .. NS-2
    block_barrier();
    read_bits(bw, b_lane);
    read_a(A[0], a_addr(0, 0));
    {
        const uint32_t m01 = 0 < TK ? 0x01010101u : 0u;
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                for (int d = 0; d < 4; ++d) B[h][s2][d] = (int)((uint32_t)bw[s2][h][d] & m01);
    }

    // DMA bookkeeping: at the wait of stage st the operations younger than stage st+1 are those of
    // stages st+2 .. st+NS-2 and the bits of the next chunk while they may still be on their way:
    // they are requested in stage 0 of a chunk BEHIND that stage's codes (the buffer is free once
    // every wave has read the current chunk's bits, one barrier earlier), so they are younger than
    // what the waits of stages 1 and 2 are for, and the wait of stage 3, which is for a group
    // requested after them, covers them: three stages for a trip to HBM, then they are read.
    for (int64_t c = 0; c < TKmax; ++c) {
        const bool bits_next = has_k && c + 1 < TK;
        static_for<0, 16>([&](auto uc) {
            constexpr int u = decltype(uc)::value;
            constexpr int s = u >> 2, hs = u & 3;
            const int st = (int)c * SPC + s;
            if constexpr (hs == 2) {  // mid-stage: stage st+1 becomes readable, stage st-1's buffer free
                const bool ahead = st + NS - 1 < nrun;
                if (!ahead) wait_vmcnt<0>();
                else if (bits_next && (s == 1 || s == 2)) wait_vmcnt<(NS - 3) * P + NBW>();
                else wait_vmcnt<(NS - 3) * P>();
                block_barrier();
                if (s == 3) read_bits(bwn, b_lane);
                if (ahead && has_k) issue(st + NS - 1, (int64_t)(st + NS) * STAGE_K > K);  // clamp only past K
                if (s == 0 && bits_next) issue_bits(c + 1);
            }
            constexpr int u2 = u + 2;  // the operand built in this half-step
            constexpr int i2 = (u2 >> 1) & 7, h2 = u2 & 1;
            v4i(&src)[2][2] = u2 >= 16 ? bwn : bw;
            const uint32_t m01 = (u2 >= 16 ? c + 1 : c) < TK ? 0x01010101u : 0u;
            v4i(&an)[2] = A[(u + 1) & 1];
            v4i(&bn)[2] = B[u2 & 3];
            lds_issue(an, a_addr(hs == 3 ? st + 1 : st, (hs + 1) & 3));
            // the bits pass through an (empty) asm placed after the reads, and the new operand
            // through one at the end: the expansion can neither be moved ahead of this half-step
            // nor be left for a later one before the scheduler sees the groups below
            asm volatile("" : "+v"(src[0][h2]), "+v"(src[1][h2]));
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    acc[mi][s2] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[u & 1][mi], B[u & 3][s2],
                                                                        acc[mi][s2], 0, 0, 0);
                    const int q = mi * 2 + s2;  // two of the eight dwords of the new operand per MFMA
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const int d = (q & 1) * 2 + e, sn = q >> 1;
                        bn[sn][d] = (int)(((uint32_t)src[sn][h2][d] >> i2) & m01);
                    }
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
                }
            asm volatile("" : "+v"(bn[0]), "+v"(bn[1]));
            __builtin_amdgcn_sched_barrier(0);
            lds_wait(an);
        });
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
            for (int h = 0; h < 2; ++h) bw[s2][h] = bwn[s2][h];
    }
    wait_vmcnt<0>();
    __syncthreads();  // every group is done with its ring

    // ---- add the four groups: lane (j, g2) of wave wn holds columns 64*wn + 32*s + j, rows
    // 32*mi + 8*(r/4) + 4*g2 + r%4; groups 2,3 write, groups 0,1 add theirs, then all threads
    // read both sums ------------------------------------------------------------------------
    int* red = reinterpret_cast<int*>(smA);
    auto red_at = [&](int region, int mi, int s2, int r) {
        return red + region * (BM * BN) + (32 * mi + 8 * (r >> 2) + 4 * g2 + (r & 3)) * BN + wn * 64 +
               32 * s2 + j;
    };
    if (gmode == 2) {  // four K-groups of the layer: each group's sums to its own slice
        static_assert(KG * NS * STAGE_BYTES >= KG * BM * BN * 4, "room for the four groups' sums");
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                for (int r = 0; r < 16; ++r) *red_at(kg, mi, s2, r) = acc[mi][s2][r];
        __syncthreads();
        const bool vec = (N & 3) == 0;
#pragma unroll
        for (int h = 0; h < BM * (BN / 4) / THREADS; ++h) {
            const int64_t m = er + (THREADS / (BN / 4)) * h;
            if (m >= M || nq >= N) continue;
            for (int rg = 0; rg < KG && sp * KG + rg < a.kgroups; ++rg) {
                const v4i t = *reinterpret_cast<const v4i*>(red + rg * (BM * BN) + (int)m * BN +
                                                             (threadIdx.x & 31) * 4) * 2;
                int* o = a.split_ws + ((int64_t)(sp * KG + rg) * M + m) * N + nq;
                if (vec) *reinterpret_cast<v4i*>(o) = t;
                else
                    for (int c = 0; c < 4; ++c)
                        if (nq + c < N) o[c] = t[c];
            }
        }
        return;
    }
    if (kg >= 2) {
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                for (int r = 0; r < 16; ++r) *red_at(kg - 2, mi, s2, r) = acc[mi][s2][r];
    }
    __syncthreads();
    if (kg < 2) {
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                for (int r = 0; r < 16; ++r) *red_at(kg, mi, s2, r) += acc[mi][s2][r];
    }
    __syncthreads();

    // ---- epilogue (Eq. 11): sum_k q s = 2 sum_k q b - sum_k q ; y = that * (beta gamma / 128) ----
#pragma unroll
    for (int h = 0; h < EH; ++h) {
        const int64_t m = er + ER * h;
        if (m >= M || nq >= N) continue;
        const int* p0 = red + (er + ER * h) * BN + (threadIdx.x & 31) * 4;
        const v4i s4 = *reinterpret_cast<const v4i*>(p0) + *reinterpret_cast<const v4i*>(p0 + BM * BN);
        const bool vec = (N & 3) == 0;  // then nq + 3 < N and the row starts 16-byte aligned
        if (to_slices) {
            int* o = a.split_ws + ((int64_t)sp * M + m) * N + nq;
            const v4i t = s4 * 2;
            if (vec) *reinterpret_cast<v4i*>(o) = t;
            else
                for (int c = 0; c < 4; ++c)
                    if (nq + c < N) o[c] = t[c];
            continue;
        }
        const v4i pm = s4 * 2 - e_rs[h];
        if (a.out_acc) {
            int* o = reinterpret_cast<int*>(a.Y) + m * N + nq;
            if (vec) *reinterpret_cast<v4i*>(o) = pm;
            else
                for (int c = 0; c < 4; ++c)
                    if (nq + c < N) o[c] = pm[c];
            continue;
        }
        float* o = a.Y + m * N + nq;
        const float sc = e_gamma[h] * 0.0078125f;  // gamma / 128, exact
        v4f y;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            // beta * (gamma / 128) has the bits of (beta * gamma) / 128
            y[c] = (float)pm[c] * (e_beta[c] * sc);
            if (a.eta) y[c] = y[c] + (e_beta[c] * e_eta[h]) * (float)e_ws[c];  // Eq. 6
        }
        if (vec) {
            if (a.accumulate) y += *reinterpret_cast<const v4f*>(o);  // a later K-group (Eq. 13-15)
            *reinterpret_cast<v4f*>(o) = y;
        } else {
            for (int c = 0; c < 4; ++c)
                if (nq + c < N) o[c] = a.accumulate ? y[c] + o[c] : y[c];
        }
    }
}

// Small batches (16 < M <= 64) leave most of the chip idle when N supplies few 64 x 128 tiles
// (fewer than half the CUs): K is then split over workgroups too, so that about one work item
// runs per CU, as long as the partial sums (M*N*4 bytes a slice) stay below the packed weights.
// Measured on the 28672 -> 7168 layer at M = 64: 70 us unsplit, 30 us in 4 slices, 38 us in 8;
// with 168 tiles or more a split only adds traffic.  256 CUs are assumed (the workspace is sized
// from this too).  Returns tiles of K per slice, 0 = no split.
int64_t prefill_split_tiles(int64_t M, int64_t N, int64_t K) {
    if (M <= 16 || M > 64) return 0;
    if (const int64_t per = tuning().mid_split_tiles) return per > 0 && per < tiles_k(K) ? per : 0;
    const int64_t tiles = ((M + 63) / 64) * ((N + 127) / 128), TK = tiles_k(K);
    if (tiles > 128) return 0;
    int64_t smax = 256 / tiles;
    if (smax > K / (32 * M)) smax = K / (32 * M);
    if (smax > 16) smax = 16;
    if (smax < 2) return 0;
    int64_t per = (TK + smax - 1) / smax;
    if (per < 2) per = 2;
    return (TK + per - 1) / per >= 2 ? per : 0;
}

// 16 < M <= 64.  K is also split over workgroups (second kernel: splitk_reduce) when N gives
// few tiles and the caller brought the workspace for it, as prefill_split_tiles decides.
hipError_t launch_gemm_mid(const GemmArgs& a_in, hipStream_t s) {
    GemmArgs a = a_in;
    a.split_k = 0;
    if (a.M > mid::BM || a.K >= ((int64_t)1 << 22) || a.ldq >= ((int64_t)1 << 22))
        return hipErrorInvalidValue;
    const int grid_n = (int)((a.N + mid::BN - 1) / mid::BN);
    int splits = 1;
    const int64_t per = prefill_split_tiles(a.M, a.N, a.K);
    const size_t need = gemm_split_ws_bytes(a.M, a.N, a.K);
    int gmode = 0;
    if (a.kgroups > 1) {  // the caller sized split_ws for one slice per K-group
        if (!a.split_ws || a.split_ws_bytes < (size_t)a.kgroups * a.M * a.N * 4)
            return hipErrorInvalidValue;
        // four K-groups per work item, one per K-group of the workgroup, unless the layer's groups
        // are long enough to be worth splitting over the workgroup's four themselves
        gmode = tuning().group_slices || tiles_k(a.K) >= 8 ? 1 : 2;
        splits = gmode == 2 ? (a.kgroups + mid::KG - 1) / mid::KG : a.kgroups;
    } else if (per && a.split_ws && a.split_ws_bytes >= need && !tuning().mid_nosplit) {
        splits = (int)((tiles_k(a.K) + per - 1) / per);
        a.tk_pitch = a.tk_pitch ? a.tk_pitch : tiles_k(a.K);
        a.split_k = per * kChunkK;
    }
    gemm_mid_kernel<4><<<(unsigned)(grid_n * splits), mid::THREADS, 0, s>>>(a, grid_n, gmode);
    if (splits > 1 || gmode) launch_splitk_reduce(a, gmode ? a.kgroups : splits, s);
    return hipGetLastError();
}

}  // namespace bl

// Straight-through-estimator backward of BitLinear (arXiv 2310.11453, Section 2.2):
// Sign, Clip and rounding are treated as identity and alpha, beta, gamma as constants, so
//   y = x^ (beta S)^T  with  x^ ~ q gamma/128,  S = sign matrix in {-1,+1}
//   dX^[M,K] = beta * g[M,N] S[N,K]                 g  = bf16(dY)
//   dW [N,K] = gw^T[N,M] q[M,K] * (gamma/128)       gw = bf16(dY) per tensor,
//                                                    bf16(dY * gamma_m/128) per token
// Both are bf16 MFMA contractions with fp32 accumulation (+-1 and int8 codes are exact in
// bf16; only dY is rounded).
//
// Structure.  Each operand is first written once in the layout the MFMA wants, i.e. with the
// reduction index contiguous and padded with zeros to a multiple of 32:
//   g   [M][Np]   rows of dY, cast                (A operand of dX, reduction over N)
//   Sw  [Np/32][K] the signs of 32 weight rows of a column in one word (B operand of dX for
//                 large operands: the kernel builds +-1 bf16 from it in registers), or
//   St  [K][Np]   +-1 as bf16 from the packed bits (B operand of dX for small operands)
//   gwT [N][Mp]   dY transposed, scaled, cast      (A operand of dW, reduction over M)
//   qT  [K][Mp]   codes transposed, cast           (B operand of dW)
// (one pass over dY writes g and gwT) and one product, C[I][J] = scale * sum_r A[I][r] B[J][r],
// serves both: persistent 256 x 256 kernels fed by DMA for large operands, a plain 256 x 128
// kernel otherwise.  The preparation passes are HBM-bound and small next to the 2*M*N*K flops
// of each product.

#include "common.h"
#include "kernels.h"
#include "ring.h"

namespace bl {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

// round-to-nearest-even fp32 -> bf16 bits (inputs are finite)
__device__ inline uint32_t bf16_bits(float v) {
    uint32_t u = __float_as_uint(v);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// Rows of the bf16 copies are `ld` elements apart, ld >= the padded length: see row_pitch().
//
// ---- in[R][C] (fp32 or int8) -> bf16 copies, one read of the input ----------------------------
//   rows[R][Cp]  = bf16(in)                      (row pitch ld_rows; columns C..Cp-1 zero)
//   tr  [C][Rp]  = bf16(scale_r * in)^T          (row pitch ld_tr; columns R..Rp-1 zero)
// scale_r = row_gamma[r] / 128 or 1.  Either output may be null.  A workgroup takes a 64 x 64
// tile: each thread reads 4 x 4 consecutive elements, writes its 8-byte pieces of `rows`, and
// the transpose goes through LDS (row pitch 66 halfwords: the 4-row steps of the 16 lanes that
// build one output row fall on distinct banks) and leaves as 8-byte pieces too.
// VEC: C % 4 == 0 and `in` 16-byte aligned, so that a thread's 4 elements are one load.
template <typename IN, bool VEC>
__global__ __launch_bounds__(256) void cast_transpose_bf16(const IN* __restrict__ in, int64_t R,
                                                           int64_t C, int64_t Cp, int64_t ld_rows,
                                                           int64_t Rp, int64_t ld_tr,
                                                           const float* __restrict__ row_gamma,
                                                           uint16_t* __restrict__ rows,
                                                           uint16_t* __restrict__ tr) {
    __shared__ __attribute__((aligned(8))) uint16_t tile[64][66];
    const int64_t r0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int idx = it * 256 + threadIdx.x;
        const int rl = idx >> 4, cl = (idx & 15) * 4;
        const int64_t r = r0 + rl, c = c0 + cl;
        float v[4] = {0.f, 0.f, 0.f, 0.f};
        if (r < R) {
            if (VEC && c + 3 < C) {
                if constexpr (sizeof(IN) == 4) {
                    const float4 t = *reinterpret_cast<const float4*>(in + r * C + c);
                    v[0] = t.x, v[1] = t.y, v[2] = t.z, v[3] = t.w;
                } else {
                    const char4 t = *reinterpret_cast<const char4*>(in + r * C + c);
                    v[0] = (float)t.x, v[1] = (float)t.y, v[2] = (float)t.z, v[3] = (float)t.w;
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (c + e < C) v[e] = (float)in[r * C + c + e];
            }
        }
        if (rows && r < R && c < Cp)
            *reinterpret_cast<uint2*>(rows + r * ld_rows + c) =
                make_uint2(bf16_bits(v[0]) | (bf16_bits(v[1]) << 16),
                           bf16_bits(v[2]) | (bf16_bits(v[3]) << 16));
        if (row_gamma && r < R) {
            const float sc = row_gamma[r] / 128.0f;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = v[e] * sc;
        }
        uint32_t* t32 = reinterpret_cast<uint32_t*>(&tile[rl][cl]);
        t32[0] = bf16_bits(v[0]) | (bf16_bits(v[1]) << 16);
        t32[1] = bf16_bits(v[2]) | (bf16_bits(v[3]) << 16);
    }
    if (!tr) return;
    __syncthreads();
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int idx = it * 256 + threadIdx.x;
        const int cl = idx >> 4, rl = (idx & 15) * 4;
        const int64_t c = c0 + cl, r = r0 + rl;
        if (c < C && r < Rp)
            *reinterpret_cast<uint2*>(tr + c * ld_tr + r) =
                make_uint2((uint32_t)tile[rl][cl] | ((uint32_t)tile[rl + 1][cl] << 16),
                           (uint32_t)tile[rl + 2][cl] | ((uint32_t)tile[rl + 3][cl] << 16));
    }
}

template <typename IN>
static void launch_cast_transpose(const IN* in, int64_t R, int64_t C, int64_t Cp, int64_t ld_rows,
                                  int64_t Rp, int64_t ld_tr, const float* row_gamma, uint16_t* rows,
                                  uint16_t* tr, hipStream_t s) {
    // the grid covers the padded extents of whichever outputs are written
    const int64_t cols = rows ? Cp : C, rws = tr ? Rp : R;
    dim3 grid((unsigned)((cols + 63) / 64), (unsigned)((rws + 63) / 64));
    const bool vec = C % 4 == 0 && ((uintptr_t)in & 15) == 0;
    if (vec)
        cast_transpose_bf16<IN, true><<<grid, 256, 0, s>>>(in, R, C, Cp, ld_rows, Rp, ld_tr,
                                                           row_gamma, rows, tr);
    else
        cast_transpose_bf16<IN, false><<<grid, 256, 0, s>>>(in, R, C, Cp, ld_rows, Rp, ld_tr,
                                                            row_gamma, rows, tr);
}

// ---- St[K][Np] = +-1 as bf16 from the packed tiles ------------------------------------------
// One workgroup expands 64 weight rows (4 tiles) x 512 columns: thread -> (k, 8 rows), 16 bytes.
__global__ __launch_bounds__(256) void bits_transpose_bf16(const uint32_t* __restrict__ packed,
                                                           int64_t N, int64_t K, int64_t Np,
                                                           int64_t ld, uint16_t* __restrict__ St) {
    __shared__ uint32_t sm[4][256];
    const int64_t TN = tiles_n(N), TK = tiles_k(K);
    const int64_t tn0 = (int64_t)blockIdx.x * 4, tk = blockIdx.y;
    for (int t = 0; t < 4; ++t) {
        uint32_t v = 0;  // rows past N: zero bits; their columns of St are the zero padding
        if (tn0 + t < TN) v = packed[tile_dword_offset(tn0 + t, tk, TK) + threadIdx.x];
        sm[t][threadIdx.x] = v;
    }
    __syncthreads();
    for (int it = 0; it < 16; ++it) {
        const int o = it * 256 + threadIdx.x;  // 512 k x 8 row-groups
        const int kl = o >> 3, seg = o & 7;    // seg: tile seg/2, rows 8*(seg%2)..+7
        const int64_t k = tk * kChunkK + kl, n = tn0 * 16 + seg * 8;
        if (k >= K || n >= Np) continue;
        const int i = kl >> 6, g = (kl & 63) >> 4, d = (kl & 15) >> 2, j = kl & 3;
        uint32_t w[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            uint32_t pair = 0;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int c = (seg & 1) * 8 + 2 * p + e;
                const uint32_t dw = sm[seg >> 1][(g * 16 + c) * 4 + d];
                const uint32_t bit = (dw >> (8 * j + i)) & 1u;
                const uint32_t val = (n + 2 * p + e < N) ? (bit ? 0x3f80u : 0xbf80u) : 0u;
                pair |= val << (16 * e);
            }
            w[p] = pair;
        }
        *reinterpret_cast<uint4*>(St + k * ld + n) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// ---- Sw[Np/32][K]: the signs of 32 consecutive weight rows of one column k in one word -------
// What the ring kernel below reads as the B operand of dX (reduction over n): a stage of 32 n is
// one word per column, 1 KiB for a 256-column tile instead of 16 KiB of bf16.  Bit layout of a
// word, chosen so that a lane builds an MFMA operand dword with one shift and one and-or: row
// n = 32 sw + r sits at bit 8 (r/16) + 4 ((r%16)/8) + (r%8)/2 + 16 (r%2), and holds 1 for -1
// (the bf16 sign bit), 0 for +1.  Rows past N: their columns of g are zero, any bit does.
// One workgroup transposes two tiles (32 rows) x 512 columns.
__global__ __launch_bounds__(256) void bits_transpose_words(const uint32_t* __restrict__ packed,
                                                            int64_t N, int64_t K,
                                                            uint32_t* __restrict__ Sw) {
    __shared__ uint32_t sm[2][256];
    const int64_t TN = tiles_n(N), TK = tiles_k(K);
    const int64_t sw = blockIdx.x, tk = blockIdx.y;
    for (int t = 0; t < 2; ++t) {
        uint32_t v = 0;
        if (2 * sw + t < TN) v = packed[tile_dword_offset(2 * sw + t, tk, TK) + threadIdx.x];
        sm[t][threadIdx.x] = v;
    }
    __syncthreads();
    for (int it = 0; it < 2; ++it) {
        const int kl = it * 256 + threadIdx.x;
        const int64_t k = tk * kChunkK + kl;
        if (k >= K) continue;
        const int i = kl >> 6, g = (kl & 63) >> 4, d = (kl & 15) >> 2, j = kl & 3;
        uint32_t word = 0;
#pragma unroll
        for (int r = 0; r < 32; ++r) {
            const uint32_t dw = sm[r >> 4][(g * 16 + (r & 15)) * 4 + d];
            const uint32_t minus = ((dw >> (8 * j + i)) & 1u) ^ 1u;
            word |= minus << (8 * (r >> 4) + 4 * ((r & 15) >> 3) + ((r & 7) >> 1) + 16 * (r & 1));
        }
        Sw[sw * K + k] = word;
    }
}

// ---- C[I][J] = scale * sum_r A[I][r] B[J][r], bf16 operands, fp32 accumulate -------------------
// Workgroup tile 256 x 128, four waves of 128 x 64 (4 x 2 MFMA tiles of 32 x 32), stage = 32
// reduction elements (64-byte rows, padded to 80 in LDS: conflict-free 16-byte operand reads).
// Global -> registers -> LDS double buffering.  scale = *scale_ptr * scale_mul (either may be
// neutral).
constexpr int kBwdPitch = 80;

template <int BM, int BN>
__global__ __launch_bounds__(256, 2) void gemm_tn_bf16(const uint16_t* __restrict__ A,
                                                       const uint16_t* __restrict__ B, int64_t I,
                                                       int64_t J, int64_t Rp, int64_t ld,
                                                       const float* __restrict__ scale_ptr,
                                                       float scale_mul, float* __restrict__ C) {
    constexpr int WTM = BM / 2, WTN = BN / 2, MI = WTM / 32, NI = WTN / 32;
    constexpr int PA = BM * 4 / 256, PB = BN * 4 / 256;
    __shared__ __attribute__((aligned(16))) uint8_t smA[2][BM * kBwdPitch];
    __shared__ __attribute__((aligned(16))) uint8_t smB[2][BN * kBwdPitch];

    const int grid_j = (int)((J + BN - 1) / BN);
    const int64_t i0 = (int64_t)(blockIdx.x / grid_j) * BM, j0 = (int64_t)(blockIdx.x % grid_j) * BN;
    const int w = threadIdx.x / kWave, l = threadIdx.x % kWave;
    const int wm = w >> 1, wn = w & 1, jl = l & 31, g2 = l >> 5;

    v4i ra[PA], rb[PB];
    auto load_stage = [&](int64_t r0) {
#pragma unroll
        for (int q = 0; q < PA; ++q) {
            const int p = threadIdx.x + q * 256;
            int64_t row = i0 + (p >> 2);
            if (row > I - 1) row = I - 1;
            ra[q] = *reinterpret_cast<const v4i*>(A + row * ld + r0 + (p & 3) * 8);
        }
#pragma unroll
        for (int q = 0; q < PB; ++q) {
            const int p = threadIdx.x + q * 256;
            int64_t row = j0 + (p >> 2);
            if (row > J - 1) row = J - 1;
            rb[q] = *reinterpret_cast<const v4i*>(B + row * ld + r0 + (p & 3) * 8);
        }
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int q = 0; q < PA; ++q) {
            const int p = threadIdx.x + q * 256;
            *reinterpret_cast<v4i*>(&smA[buf][(p >> 2) * kBwdPitch + (p & 3) * 16]) = ra[q];
        }
#pragma unroll
        for (int q = 0; q < PB; ++q) {
            const int p = threadIdx.x + q * 256;
            *reinterpret_cast<v4i*>(&smB[buf][(p >> 2) * kBwdPitch + (p & 3) * 16]) = rb[q];
        }
    };

    v16f acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int s = 0; s < NI; ++s)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][s][r] = 0.f;

    const int64_t nst = Rp / 32;
    load_stage(0);
    store_stage(0);
    __syncthreads();
    for (int64_t st = 0; st < nst; ++st) {
        const int buf = (int)(st & 1);
        if (st + 1 < nst) load_stage((st + 1) * 32);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            v4i av[MI], bv[NI];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                av[mi] = *reinterpret_cast<const v4i*>(
                    &smA[buf][(wm * WTM + 32 * mi + jl) * kBwdPitch + (2 * h + g2) * 16]);
#pragma unroll
            for (int s = 0; s < NI; ++s)
                bv[s] = *reinterpret_cast<const v4i*>(
                    &smB[buf][(wn * WTN + 32 * s + jl) * kBwdPitch + (2 * h + g2) * 16]);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int s = 0; s < NI; ++s)
                    acc[mi][s] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(v8bf, av[mi]), __builtin_bit_cast(v8bf, bv[s]),
                        acc[mi][s], 0, 0, 0);
        }
        if (st + 1 < nst) store_stage(buf ^ 1);
        __syncthreads();
    }

    const float scale = (scale_ptr ? *scale_ptr : 1.0f) * scale_mul;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t i = i0 + wm * WTM + 32 * mi + 8 * (r >> 2) + 4 * g2 + (r & 3);
            if (i >= I) continue;
#pragma unroll
            for (int s = 0; s < NI; ++s) {
                const int64_t j = j0 + wn * WTN + 32 * s + jl;
                if (j < J) C[i * J + j] = scale * acc[mi][s][r];
            }
        }
}

// ---- the same product for large operands: LDS ring fed by DMA --------------------------------
// Workgroup tile 256 x 256, eight waves of 128 x 64 (4 x 2 MFMA tiles), one workgroup per CU,
// persistent over the tiles.  A stage is 32 reduction elements: 64-byte rows of A and of B,
// streamed global -> LDS by global_load_lds_dwordx4 into a ring of NS stages; the 16-byte
// segments of a row are XOR-swizzled with (row/4)%4, so the operand reads of 16 consecutive rows
// touch every bank once.  The unit of work is a half-step (16 elements, 8 MFMAs): one asm block
// issues the LDS reads of the next half-step's operands, then the MFMAs of the current one, then
// waits for the reads.  Between the half-steps of stage st every wave waits for its own DMA of
// stage st+1 (s_waitcnt vmcnt(n), n counted by hand), meets the others at a bare s_barrier, and
// the DMA of stage st+NS-1 goes to the buffer stage st-1 has left.
__device__ inline void bf16_read_ops(v4i (&a)[4], v4i (&b)[2], uint32_t ad_a, uint32_t ad_b) {
    asm volatile(
        "ds_read_b128 %0, %6\n\t"
        "ds_read_b128 %1, %6 offset:2048\n\t"
        "ds_read_b128 %2, %6 offset:4096\n\t"
        "ds_read_b128 %3, %6 offset:6144\n\t"
        "ds_read_b128 %4, %7\n\t"
        "ds_read_b128 %5, %7 offset:2048\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(a[0]), "=&v"(a[1]), "=&v"(a[2]), "=&v"(a[3]), "=&v"(b[0]), "=&v"(b[1])
        : "v"(ad_a), "v"(ad_b));
}
// acc[mi][s] += ac[mi] x bc[s]; an, bn = operands at ad_a, ad_b, complete on exit
__device__ inline void bf16_half_step(v16f (&acc)[4][2], const v4i (&ac)[4], const v4i (&bc)[2],
                                      v4i (&an)[4], v4i (&bn)[2], uint32_t ad_a, uint32_t ad_b) {
    asm volatile(
        "ds_read_b128 %8, %20\n\t"
        "ds_read_b128 %9, %20 offset:2048\n\t"
        "ds_read_b128 %12, %21\n\t"
        "ds_read_b128 %13, %21 offset:2048\n\t"
        "ds_read_b128 %10, %20 offset:4096\n\t"
        "ds_read_b128 %11, %20 offset:6144\n\t"
        "v_mfma_f32_32x32x16_bf16 %0, %14, %18, %0\n\t"
        "v_mfma_f32_32x32x16_bf16 %1, %14, %19, %1\n\t"
        "v_mfma_f32_32x32x16_bf16 %2, %15, %18, %2\n\t"
        "v_mfma_f32_32x32x16_bf16 %3, %15, %19, %3\n\t"
        "v_mfma_f32_32x32x16_bf16 %4, %16, %18, %4\n\t"
        "v_mfma_f32_32x32x16_bf16 %5, %16, %19, %5\n\t"
        "v_mfma_f32_32x32x16_bf16 %6, %17, %18, %6\n\t"
        "v_mfma_f32_32x32x16_bf16 %7, %17, %19, %7\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "+v"(acc[0][0]), "+v"(acc[0][1]), "+v"(acc[1][0]), "+v"(acc[1][1]), "+v"(acc[2][0]),
          "+v"(acc[2][1]), "+v"(acc[3][0]), "+v"(acc[3][1]), "=&v"(an[0]), "=&v"(an[1]),
          "=&v"(an[2]), "=&v"(an[3]), "=&v"(bn[0]), "=&v"(bn[1])
        : "v"(ac[0]), "v"(ac[1]), "v"(ac[2]), "v"(ac[3]), "v"(bc[0]), "v"(bc[1]), "v"(ad_a),
          "v"(ad_b));
}

// Tile order of the persistent bf16 kernels.  Workgroups are dealt round-robin to the 8 XCDs (one
// L2 each).  An XCD gets grid_i / 8 whole rows of tiles, and the G / 8 tiles it runs together
// form a blk_i x blk_j block of them: both operands are equally wide here, so what the XCD
// streams from memory per step of the contraction is blk_i + blk_j operand blocks, least for a
// square.  blk_i = 0 (the host found no such blocks for this grid): one contiguous range of tiles
// per XCD, J fastest.  i0 = -1: no tile (the XCD's range ended before the last round did).
__device__ inline void ring_tile_origin(int t, int G, int grid_i, int grid_j, int blk_i, int blk_j,
                                        int BM, int BN, int64_t& i0, int64_t& j0) {
    const int ntiles = grid_i * grid_j;
    int logical = t;
    if ((ntiles & 7) == 0 && (G & 7) == 0) {
        const int q = ((t % G) >> 3) + (t / G) * (G >> 3);
        const int per = ntiles >> 3;
        if (q >= per) {
            logical = -1;
        } else if (blk_i > 0) {
            const int cpx = G >> 3, b = q / cpx, within = q % cpx, bpr = grid_j / blk_j;
            const int row = (t & 7) * (grid_i >> 3) + (b / bpr) * blk_i + within / blk_j;
            const int col = (b % bpr) * blk_j + within % blk_j;
            logical = row * grid_j + col;
        } else {
            logical = (t & 7) * per + q;
        }
    }
    i0 = logical < 0 ? -1 : (int64_t)(logical / grid_j) * BM;
    j0 = logical < 0 ? -1 : (int64_t)(logical % grid_j) * BN;
}

template <int NS>
__global__ __launch_bounds__(512, 2) void gemm_tn_bf16_ring(const uint16_t* __restrict__ A,
                                                            const uint16_t* __restrict__ B,
                                                            int64_t I, int64_t J, int64_t Rp,
                                                            int64_t ld,
                                                            const float* __restrict__ scale_ptr,
                                                            float scale_mul, float* __restrict__ C,
                                                            int grid_i, int grid_j, int blk_i,
                                                            int blk_j) {
    constexpr int BM = 256, BN = 256, WN = 4, THREADS = 512, WTM = 128, WTN = 64, MI = 4, NI = 2;
    constexpr int PA = BM * 4 / THREADS, PB = BN * 4 / THREADS, P = PA + PB;
    constexpr int A_BYTES = BM * 64, STAGE_BYTES = (BM + BN) * 64;
    static_assert((NS - 1) * P < 64, "vmcnt range");
    __shared__ __attribute__((aligned(1024))) uint8_t sm[NS * STAGE_BYTES];

    const int w = threadIdx.x / kWave, l = threadIdx.x % kWave;
    const int wm = w / WN, wn = w % WN;
    const int j = l & 31, g2 = l >> 5;
    const int nst = (int)(Rp / 32);
    const int ntiles = grid_i * grid_j;
    // groups of NS stages whose look-ahead stage st+NS-1 exists for every stage of the group
    const int main_groups = nst >= 2 * NS - 1 ? (nst - (2 * NS - 1)) / NS + 1 : 0;

    auto tile_origin = [&](int t, int64_t& i0, int64_t& j0) {
        ring_tile_origin(t, (int)gridDim.x, grid_i, grid_j, blk_i, blk_j, BM, BN, i0, j0);
    };

    // DMA: thread -> PA + PB pieces of 16 bytes per stage; piece = (row, swizzled segment).
    // Rows past the matrix re-read its last row (their results are never stored).
    uint32_t goffA[PA], goffB[PB];
    const uint8_t *baseA = nullptr, *baseB = nullptr;
    const uint32_t pitch = (uint32_t)ld * 2;
    auto setup_dma = [&](int64_t i0, int64_t j0) {
#pragma unroll
        for (int q = 0; q < PA; ++q) {
            const int slot = q * THREADS + threadIdx.x;
            int row = slot >> 2;
            const int seg = ((slot & 3) ^ ((row >> 2) & 3)) * 16;
            if (i0 + row > I - 1) row = (int)(I - 1 - i0);
            goffA[q] = (uint32_t)row * pitch + seg;
        }
#pragma unroll
        for (int q = 0; q < PB; ++q) {
            const int slot = q * THREADS + threadIdx.x;
            int row = slot >> 2;
            const int seg = ((slot & 3) ^ ((row >> 2) & 3)) * 16;
            if (j0 + row > J - 1) row = (int)(J - 1 - j0);
            goffB[q] = (uint32_t)row * pitch + seg;
        }
        baseA = reinterpret_cast<const uint8_t*>(A) + i0 * (int64_t)pitch;
        baseB = reinterpret_cast<const uint8_t*>(B) + j0 * (int64_t)pitch;
    };
    const uint32_t lds_wave = (uint32_t)(w * kWave * 16);
    // stage `st` into ring slot st % NS; `src_st` is the stage whose bytes are read (== st, or
    // the last stage when st does not exist: the slot is filled with bytes nobody uses)
    auto issue = [&](int st, int src_st) {
        uint8_t* dst = sm + (st % NS) * STAGE_BYTES + lds_wave;
#pragma unroll
        for (int q = 0; q < PA; ++q)
            __builtin_amdgcn_global_load_lds(
                (const void*)(baseA + (int64_t)src_st * 64 + goffA[q]),
                (__attribute__((address_space(3))) void*)(dst + q * THREADS * 16), 16, 0, 0);
#pragma unroll
        for (int q = 0; q < PB; ++q)
            __builtin_amdgcn_global_load_lds(
                (const void*)(baseB + (int64_t)src_st * 64 + goffB[q]),
                (__attribute__((address_space(3))) void*)(dst + A_BYTES + q * THREADS * 16), 16, 0,
                0);
    };
    auto issue_tile_start = [&]() {
#pragma unroll
        for (int s = 0; s < NS - 1; ++s) issue(s, s < nst ? s : nst - 1);
    };

    // lane's operand addresses inside a stage: row, segment (2h + g2) ^ swizzle
    const int sw = (j >> 2) & 3;
    const uint32_t smb = (uint32_t)(uintptr_t)sm;
    const uint32_t a_lane[2] = {smb + (wm * WTM + j) * 64 + ((g2) ^ sw) * 16,
                                smb + (wm * WTM + j) * 64 + ((2 + g2) ^ sw) * 16};
    const uint32_t b_lane[2] = {smb + A_BYTES + (wn * WTN + j) * 64 + ((g2) ^ sw) * 16,
                                smb + A_BYTES + (wn * WTN + j) * 64 + ((2 + g2) ^ sw) * 16};
    auto ring = [&](int st) { return (uint32_t)((st % NS) * STAGE_BYTES); };

    v16f acc[MI][NI];
    v4i ax[MI], ay[MI], bx[NI], by[NI];
    // In: ax/bx = operands of (st, half 0).  Out: operands of (st+1, half 0); for the last stage
    // these are stale ring bytes that nobody uses.
    auto stage = [&](int st, bool ahead) {
        bf16_half_step(acc, ax, bx, ay, by, a_lane[1] + ring(st), b_lane[1] + ring(st));
        // younger than stage st+1: stages st+2 .. st+NS-2
        if (ahead) wait_vmcnt<(NS - 3) * P>();
        else wait_vmcnt<0>();
        block_barrier();
        if (ahead) issue(st + NS - 1, st + NS - 1);
        bf16_half_step(acc, ay, by, ax, bx, a_lane[0] + ring(st + 1), b_lane[0] + ring(st + 1));
    };

    const float scale = (scale_ptr ? *scale_ptr : 1.0f) * scale_mul;
    int t = (int)blockIdx.x;
    int64_t i0, j0;
    tile_origin(t, i0, j0);
    if (i0 < 0) return;  // uniform for the whole workgroup
    setup_dma(i0, j0);
    issue_tile_start();

    while (true) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int s = 0; s < NI; ++s)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mi][s][r] = 0.f;

        wait_vmcnt<(NS - 2) * P>();  // younger than stage 0: stages 1 .. NS-2
        block_barrier();
        bf16_read_ops(ax, bx, a_lane[0], b_lane[0]);

        for (int gidx = 0; gidx < main_groups; ++gidx)
            static_for<0, NS>([&](auto ic) { stage(gidx * NS + decltype(ic)::value, true); });
        for (int st = main_groups * NS; st < nst; ++st) stage(st, st + NS - 1 < nst);

        // the accumulators were last written inside an asm block: let the matrix pipeline
        // retire them before ordinary instructions read them
        asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");

        // every wave is done with the ring: start the next tile's stream, then store
        block_barrier();
        const int t_next = t + (int)gridDim.x;
        int64_t i0n = -1, j0n = -1;
        if (t_next < ntiles) tile_origin(t_next, i0n, j0n);
        if (i0n >= 0) {
            setup_dma(i0n, j0n);
            issue_tile_start();
        }

        // lane (j, g2) holds column j0 + .. + j, rows 8*(r/4) + 4*g2 + r%4 of each sub-tile
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t i = i0 + wm * WTM + 32 * mi + 8 * (r >> 2) + 4 * g2 + (r & 3);
                if (i >= I) continue;
#pragma unroll
                for (int s = 0; s < NI; ++s) {
                    const int64_t jj = j0 + wn * WTN + 32 * s + j;
                    if (jj < J) __builtin_nontemporal_store(scale * acc[mi][s][r], &C[i * J + jj]);  // streaming
                }
            }
        if (i0n < 0) break;
        t = t_next;
        i0 = i0n;
        j0 = j0n;
    }
}

// ---- dX^: the same persistent kernel with the +-1 operand built from sign words ----------------
// C[I][J] = scale * sum_r A[I][r] S[r][J], A = g (bf16 rows, as above), S given as Sw[r / 32][J]
// (bits_transpose_words).  Only A goes through the big ring (16 KiB a stage, half the bytes the
// bf16 copy of S would add); a stage of S is one word per column, which each wave fetches for
// its own 64 columns (one 4-byte DMA per lane) into a ring of its own, one stage ahead of A, so
// that the words of stage st+1 can be read while stage st is being multiplied.  A lane turns its
// word into the four dwords of an MFMA operand (eight +-1 bf16 values) with a shift and an
// and-or each, placed between the MFMAs of the half-step before (the same scheduling as in the
// forward GEMM).  Group of DMA operations of stage s: the words of stage s+1, then A of stage s;
// they complete in this order, so the hand-counted waits are those of the kernel above with one
// more operation per stage.
__device__ inline void a_issue(v4i (&a)[4], uint32_t ad) {
    asm volatile(
        "ds_read_b128 %0, %4\n\t"
        "ds_read_b128 %1, %4 offset:2048\n\t"
        "ds_read_b128 %2, %4 offset:4096\n\t"
        "ds_read_b128 %3, %4 offset:6144"
        : "=&v"(a[0]), "=&v"(a[1]), "=&v"(a[2]), "=&v"(a[3])
        : "v"(ad));
}
__device__ inline void words_issue(uint32_t (&wd)[2], uint32_t ad) {
    asm volatile(
        "ds_read_b32 %0, %2\n\t"
        "ds_read_b32 %1, %2 offset:128"
        : "=&v"(wd[0]), "=&v"(wd[1])
        : "v"(ad));
}
__device__ inline void a_wait(v4i (&a)[4]) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]));
}
__device__ inline void a_words_wait(v4i (&a)[4], uint32_t (&wd)[2]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(wd[0]), "+v"(wd[1]));
}

template <int NS>
__global__ __launch_bounds__(512, 2) void gemm_tn_signs_ring(const uint16_t* __restrict__ A,
                                                             const uint32_t* __restrict__ Sw,
                                                             int64_t I, int64_t J, int64_t Rp,
                                                             int64_t ld,
                                                             const float* __restrict__ scale_ptr,
                                                             float scale_mul, float* __restrict__ C,
                                                             int grid_i, int grid_j, int blk_i,
                                                             int blk_j) {
    constexpr int BM = 256, BN = 256, WN = 4, THREADS = 512, WTM = 128, WTN = 64, MI = 4, NI = 2;
    constexpr int PA = BM * 4 / THREADS, P = PA + 1;  // DMA operations per thread and stage
    constexpr int STAGE_BYTES = BM * 64;
    static_assert((NS - 1) * P + 1 < 64, "vmcnt range");
    __shared__ __attribute__((aligned(1024))) uint8_t sm[NS * STAGE_BYTES];
    __shared__ __attribute__((aligned(256))) uint32_t smW[8][NS][64];  // [wave][slot][column]

    const int w = threadIdx.x / kWave, l = threadIdx.x % kWave;
    const int wm = w / WN, wn = w % WN;
    const int j = l & 31, g2 = l >> 5;
    const int nst = (int)(Rp / 32);
    const int ntiles = grid_i * grid_j;
    const int main_groups = nst >= 2 * NS - 1 ? (nst - (2 * NS - 1)) / NS + 1 : 0;

    auto tile_origin = [&](int t, int64_t& i0, int64_t& j0) {
        ring_tile_origin(t, (int)gridDim.x, grid_i, grid_j, blk_i, blk_j, BM, BN, i0, j0);
    };

    uint32_t goffA[PA];
    const uint8_t* baseA = nullptr;
    const uint32_t* wsrc = Sw;  // this lane's column of the sign words, stage 0
    const uint32_t pitch = (uint32_t)ld * 2;
    auto setup_dma = [&](int64_t i0, int64_t j0) {
#pragma unroll
        for (int q = 0; q < PA; ++q) {
            const int slot = q * THREADS + threadIdx.x;
            int row = slot >> 2;
            const int seg = ((slot & 3) ^ ((row >> 2) & 3)) * 16;
            if (i0 + row > I - 1) row = (int)(I - 1 - i0);
            goffA[q] = (uint32_t)row * pitch + seg;
        }
        baseA = reinterpret_cast<const uint8_t*>(A) + i0 * (int64_t)pitch;
        int64_t col = j0 + wn * WTN + l;  // columns past J re-read the last one (never stored)
        if (col > J - 1) col = J - 1;
        wsrc = Sw + col;
    };
    const uint32_t lds_wave = (uint32_t)(w * kWave * 16);
    // sign words of stage sb (the last stage's again when sb does not exist) into slot sb % NS
    auto issue_words = [&](int sb) {
        const int src = sb < nst ? sb : nst - 1;
        __builtin_amdgcn_global_load_lds(
            (const void*)(wsrc + (int64_t)src * J),
            (__attribute__((address_space(3))) void*)(&smW[w][sb % NS][0]), 4, 0, 0);
    };
    // the group of stage st: words of stage st+1, then A of stage st
    auto issue = [&](int st, int src_st) {
        issue_words(st + 1);
        uint8_t* dst = sm + (st % NS) * STAGE_BYTES + lds_wave;
#pragma unroll
        for (int q = 0; q < PA; ++q)
            __builtin_amdgcn_global_load_lds(
                (const void*)(baseA + (int64_t)src_st * 64 + goffA[q]),
                (__attribute__((address_space(3))) void*)(dst + q * THREADS * 16), 16, 0, 0);
    };
    auto issue_tile_start = [&]() {
        issue_words(0);
#pragma unroll
        for (int s = 0; s < NS - 1; ++s) issue(s, s < nst ? s : nst - 1);
    };

    const int sw = (j >> 2) & 3;
    const uint32_t smb = (uint32_t)(uintptr_t)sm;
    const uint32_t a_lane[2] = {smb + (wm * WTM + j) * 64 + ((g2) ^ sw) * 16,
                                smb + (wm * WTM + j) * 64 + ((2 + g2) ^ sw) * 16};
    auto ring = [&](int st) { return (uint32_t)((st % NS) * STAGE_BYTES); };
    // word of column 32 s + j of this wave (s = 0, 1: +128 bytes) for stage st
    const uint32_t w_lane = (uint32_t)(uintptr_t)&smW[w][0][j];
    auto w_addr = [&](int st) { return w_lane + (uint32_t)((st % NS) * 256); };

    v16f acc[MI][NI];
    v4i ax[MI], ay[MI], bx[NI], by[NI];
    uint32_t wcur[NI], wnext[NI];  // sign words of the current / next stage, shifted by 4 g2
    // bf16 +-1 pair number d of half h from a shifted word: bit 8h + d -> 15, bit 8h + d + 16 -> 31
    // (the two constants live in registers the compiler cannot see through: as literals they
    // would split the and-or into two instructions)
    uint32_t k_signs = 0x80008000u, k_ones = 0x3f803f80u;
    asm volatile("" : "+s"(k_signs), "+v"(k_ones));
    auto pm_one = [&](uint32_t wq, int h, int d) {
        return (int)(((wq << (15 - 8 * h - d)) & k_signs) | k_ones);
    };
    // One half-step: acc += ac x b (MI * NI MFMAs) with the next half-step's +-1 operand bn (half h
    // of the words ws) built between them; the A operand at `ad` is read into an meanwhile, and
    // with WORDS the sign words at `adw` into wr (both valid on return).
    auto half_step = [&](const v4i(&ac)[MI], const v4i(&b)[NI], v4i(&bn)[NI], uint32_t(&ws)[NI],
                         int h, v4i(&an)[MI], uint32_t ad, auto words, uint32_t(&wr)[NI],
                         uint32_t adw) {
        constexpr bool WORDS = decltype(words)::value;
        a_issue(an, ad);
        if constexpr (WORDS) words_issue(wr, adw);
        asm volatile("" : "+v"(ws[0]), "+v"(ws[1]));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int s = 0; s < NI; ++s) {
                acc[mi][s] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    __builtin_bit_cast(v8bf, ac[mi]), __builtin_bit_cast(v8bf, b[s]), acc[mi][s], 0, 0, 0);
                const int idx = mi * NI + s;  // 0 .. 7: dword idx % 4 of sub-tile idx / 4
                bn[idx >> 2][idx & 3] = pm_one(ws[idx >> 2], h, idx & 3);
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
            }
        asm volatile("" : "+v"(bn[0]), "+v"(bn[1]));
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (WORDS) a_words_wait(an, wr);
        else a_wait(an);
    };
    uint32_t wraw[NI];
    auto stage = [&](int st, bool ahead) {
        // MFMAs of (st, half 0); operand of (st, half 1) from this stage's words; the words of stage
        // st+1 (their group landed before the barrier that released stage st) are read meanwhile
        half_step(ax, bx, by, wcur, 1, ay, a_lane[1] + ring(st), std::true_type{}, wraw, w_addr(st + 1));
        if (ahead) wait_vmcnt<(NS - 3) * P>();  // younger than stage st+1: stages st+2 .. st+NS-2
        else wait_vmcnt<0>();
        block_barrier();
        if (ahead) issue(st + NS - 1, st + NS - 1);
#pragma unroll
        for (int s = 0; s < NI; ++s) wnext[s] = wraw[s] >> (4 * g2);
        half_step(ay, by, bx, wnext, 0, ax, a_lane[0] + ring(st + 1), std::false_type{}, wraw, 0u);
#pragma unroll
        for (int s = 0; s < NI; ++s) wcur[s] = wnext[s];
    };

    const float scale = (scale_ptr ? *scale_ptr : 1.0f) * scale_mul;
    int t = (int)blockIdx.x;
    int64_t i0, j0;
    tile_origin(t, i0, j0);
    if (i0 < 0) return;  // uniform for the whole workgroup
    setup_dma(i0, j0);
    issue_tile_start();

    while (true) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int s = 0; s < NI; ++s)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mi][s][r] = 0.f;

        wait_vmcnt<(NS - 2) * P>();  // younger than stage 0's group: those of stages 1 .. NS-2
        block_barrier();
        a_issue(ax, a_lane[0]);
        words_issue(wraw, w_addr(0));
        a_words_wait(ax, wraw);
#pragma unroll
        for (int s = 0; s < NI; ++s) {
            wcur[s] = wraw[s] >> (4 * g2);
#pragma unroll
            for (int d = 0; d < 4; ++d) bx[s][d] = pm_one(wcur[s], 0, d);
        }

        for (int gidx = 0; gidx < main_groups; ++gidx)
            static_for<0, NS>([&](auto ic) { stage(gidx * NS + decltype(ic)::value, true); });
        for (int st = main_groups * NS; st < nst; ++st) stage(st, st + NS - 1 < nst);

        // every wave is done with the rings: start the next tile's stream, then store
        block_barrier();
        const int t_next = t + (int)gridDim.x;
        int64_t i0n = -1, j0n = -1;
        if (t_next < ntiles) tile_origin(t_next, i0n, j0n);
        if (i0n >= 0) {
            setup_dma(i0n, j0n);
            issue_tile_start();
        }

#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t i = i0 + wm * WTM + 32 * mi + 8 * (r >> 2) + 4 * g2 + (r & 3);
                if (i >= I) continue;
#pragma unroll
                for (int s = 0; s < NI; ++s) {
                    const int64_t jj = j0 + wn * WTN + 32 * s + j;
                    if (jj < J) __builtin_nontemporal_store(scale * acc[mi][s][r], &C[i * J + jj]);
                }
            }
        if (i0n < 0) break;
        t = t_next;
        i0 = i0n;
        j0 = j0n;
    }
}

static int bwd_num_cus() {
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

// The persistent 256 x 256 kernels are used when their tiles fill at least half the CUs (and a
// lane's byte offset into a block of 256 rows fits 32 bits); the plan is the grid and the block of
// tiles an XCD runs together (ring_tile_origin): blk_i x blk_j = grid / 8 tiles out of its
// grid_i / 8 rows, as square as the divisors allow; 0 = no such tiling.
struct RingPlan {
    bool use;
    int grid, gi, gj, blk_i, blk_j;
};
static RingPlan ring_plan(int64_t I, int64_t J, int64_t ld) {
    RingPlan p{};
    const int64_t gi = (I + 255) / 256, gj = (J + 255) / 256;
    p.gi = (int)gi;
    p.gj = (int)gj;
    p.use = gi * gj * 2 >= bwd_num_cus() && ld < ((int64_t)1 << 22);
    if (tuning().bwd_ring) p.use = tuning().bwd_ring == 1 && ld < ((int64_t)1 << 22);
    if (!p.use) return p;
    int grid = bwd_num_cus();
    if (tuning().bwd_grid > 0) grid = tuning().bwd_grid;
    if (grid > gi * gj) grid = (int)(gi * gj);
    p.grid = grid;
    const int64_t ntiles = gi * gj;
    if (ntiles % 8 == 0 && grid % 8 == 0 && gi % 8 == 0 && (ntiles / 8) % (grid / 8) == 0 &&
        !tuning().bwd_rowmajor) {
        const int cpx = grid / 8;
        const int64_t rx = gi / 8;
        for (int br = 1; br <= cpx; ++br) {
            if (cpx % br) continue;
            const int bc = cpx / br;
            if (br <= rx && bc <= gj && rx % br == 0 && gj % bc == 0 &&
                (p.blk_i == 0 || br + bc < p.blk_i + p.blk_j)) {
                p.blk_i = br;
                p.blk_j = bc;
            }
        }
    }
    return p;
}

// C[I][J] = scale * A[I][:] . B[J][:]: the ring kernel, else the 256 x 128 kernel with a workgroup
// per tile.
static void launch_gemm_tn(const uint16_t* A, const uint16_t* B, int64_t I, int64_t J, int64_t Rp,
                           int64_t ld, const float* scale_ptr, float scale_mul, float* C,
                           hipStream_t s) {
    const RingPlan p = ring_plan(I, J, ld);
    if (p.use) {
        gemm_tn_bf16_ring<4><<<(unsigned)p.grid, 512, 0, s>>>(A, B, I, J, Rp, ld, scale_ptr, scale_mul,
                                                               C, p.gi, p.gj, p.blk_i, p.blk_j);
    } else {
        const unsigned blocks = (unsigned)(((I + 255) / 256) * ((J + 127) / 128));
        gemm_tn_bf16<256, 128><<<blocks, 256, 0, s>>>(A, B, I, J, Rp, ld, scale_ptr, scale_mul, C);
    }
}

// ---------------------------------------------------------------------------------------------
static inline int64_t pad32(int64_t v) { return (v + 31) / 32 * 32; }
// Row pitch (elements) of a bf16 copy whose rows hold Rp elements.  A GEMM stage reads 64 bytes
// from each of 512 rows; with rows a multiple of 4 KiB apart those reads would all fall on the
// same memory channel, so such rows are set 128 bytes further apart.
static inline int64_t row_pitch(int64_t Rp) { return Rp % 2048 == 0 ? Rp + 64 : Rp; }

// bytes of the +-1 operand of dX^: sign words [Np / 32][K] when the persistent kernel takes the
// product, else the bf16 copy St[K][Nl]
static size_t signs_bytes(int64_t M, int64_t N, int64_t K) {
    const int64_t Np = pad32(N), Nl = row_pitch(Np);
    return ring_plan(M, K, Nl).use ? (size_t)(Np / 32) * K * 4 : (size_t)K * Nl * 2;
}

size_t backward_workspace_bytes(int64_t M, int64_t N, int64_t K) {
    const int64_t Nl = row_pitch(pad32(N)), Ml = row_pitch(pad32(M));
    // g[M][Nl], the signs, gwT[N][Ml], qT[K][Ml] (bf16), each region 256-byte aligned
    auto al = [](size_t v) { return (v + 255) & ~(size_t)255; };
    return al((size_t)M * Nl * 2) + al(signs_bytes(M, N, K)) + al((size_t)N * Ml * 2) +
           al((size_t)K * Ml * 2);
}

hipError_t launch_backward(const BackwardArgs& a, hipStream_t s) {
    const int64_t M = a.M, N = a.N, K = a.K, Np = pad32(N), Mp = pad32(M);
    const int64_t Nl = row_pitch(Np), Ml = row_pitch(Mp);
    auto al = [](size_t v) { return (v + 255) & ~(size_t)255; };
    char* ws = (char*)a.workspace;
    uint16_t* g = (uint16_t*)ws;
    uint16_t* St = (uint16_t*)(ws + al((size_t)M * Nl * 2));
    uint16_t* gwT = (uint16_t*)((char*)St + al(signs_bytes(M, N, K)));
    uint16_t* qT = (uint16_t*)((char*)gwT + al((size_t)N * Ml * 2));

    // dY is read once: g for dX and gwT for dW come out of the same pass when both are wanted
    launch_cast_transpose<float>(a.dY, M, N, Np, Nl, Mp, Ml, a.per_tensor ? nullptr : a.gamma,
                                 a.dX ? g : nullptr, a.dW ? gwT : nullptr, s);
    if (a.dX) {
        const RingPlan p = ring_plan(M, K, Nl);
        if (p.use) {  // +-1 from sign words inside the kernel: no bf16 copy of the weights
            uint32_t* Sw = (uint32_t*)St;
            dim3 gb((unsigned)(Np / 32), (unsigned)tiles_k(K));
            bits_transpose_words<<<gb, 256, 0, s>>>(a.packed, N, K, Sw);
            gemm_tn_signs_ring<4><<<(unsigned)p.grid, 512, 0, s>>>(g, Sw, M, K, Np, Nl, a.beta, 1.0f,
                                                                    a.dX, p.gi, p.gj, p.blk_i, p.blk_j);
        } else {
            dim3 gb((unsigned)((tiles_n(N) + 3) / 4), (unsigned)tiles_k(K));
            bits_transpose_bf16<<<gb, 256, 0, s>>>(a.packed, N, K, Np, Nl, St);
            launch_gemm_tn(g, St, M, K, Np, Nl, a.beta, 1.0f, a.dX, s);
        }
    }
    if (a.dW) {
        launch_cast_transpose<int8_t>(a.codes, M, K, K, 0, Mp, Ml, nullptr, nullptr, qT, s);
        launch_gemm_tn(gwT, qT, N, K, Mp, Ml, a.per_tensor ? a.gamma : nullptr,
                       a.per_tensor ? 1.0f / 128.0f : 1.0f, a.dW, s);
    }
    return hipGetLastError();
}

}  // namespace bl

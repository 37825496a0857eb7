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
//   St  [K][Np]   +-1 from the packed bits         (B operand of dX)
//   gwT [N][Mp]   dY transposed, scaled, cast      (A operand of dW, reduction over M)
//   qT  [K][Mp]   codes transposed, cast           (B operand of dW)
// and one kernel, C[I][J] = scale * sum_r A[I][r] B[J][r], serves both products.  The
// preparation passes are HBM-bound and small next to the 2*M*N*K flops of each product.
#include "common.h"
#include "kernels.h"

namespace bl {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

// round-to-nearest-even fp32 -> bf16 bits (inputs are finite)
__device__ inline uint32_t bf16_bits(float v) {
    uint32_t u = __float_as_uint(v);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// ---- g[M][Np] = bf16(dY[M][N]), zero padding ------------------------------------------
__global__ __launch_bounds__(256) void cast_rows_bf16(const float* __restrict__ dY, int64_t M,
                                                      int64_t N, int64_t Np,
                                                      uint16_t* __restrict__ g) {
    const int64_t pairs = Np / 2;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= M * pairs) return;
    const int64_t m = idx / pairs, n = (idx % pairs) * 2;
    const float a = n < N ? dY[m * N + n] : 0.f;
    const float b = n + 1 < N ? dY[m * N + n + 1] : 0.f;
    reinterpret_cast<uint32_t*>(g)[idx] = bf16_bits(a) | (bf16_bits(b) << 16);
}

// ---- out[C][Rp] = bf16(scale_r * in[R][C])^T, 64x64 tiles through LDS ---------------------
// IN = float (dY, optional per-row scale gamma_r/128) or int8_t (codes).
template <typename IN>
__global__ __launch_bounds__(256) void transpose_cast_bf16(const IN* __restrict__ in, int64_t R,
                                                           int64_t C, int64_t Rp,
                                                           const float* __restrict__ row_gamma,
                                                           uint16_t* __restrict__ out) {
    __shared__ uint16_t tile[64][66];
    const int64_t r0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int rr = ty; rr < 64; rr += 4) {
        const int64_t r = r0 + rr, c = c0 + tx;
        float v = 0.f;
        if (r < R && c < C) {
            v = (float)in[r * C + c];
            if (row_gamma) v = v * (row_gamma[r] / 128.0f);
        }
        tile[rr][tx] = (uint16_t)bf16_bits(v);
    }
    __syncthreads();
    for (int cc = ty; cc < 64; cc += 4) {
        const int64_t c = c0 + cc, r = r0 + tx;
        if (c < C && r < Rp) out[c * Rp + r] = tile[tx][cc];
    }
}

// ---- St[K][Np] = +-1 as bf16 from the packed tiles ------------------------------------------
// One workgroup expands 64 weight rows (4 tiles) x 512 columns: thread -> (k, 8 rows), 16 bytes.
__global__ __launch_bounds__(256) void bits_transpose_bf16(const uint32_t* __restrict__ packed,
                                                           int64_t N, int64_t K, int64_t Np,
                                                           uint16_t* __restrict__ St) {
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
        *reinterpret_cast<uint4*>(St + k * Np + n) = make_uint4(w[0], w[1], w[2], w[3]);
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
                                                       int64_t J, int64_t Rp,
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
            ra[q] = *reinterpret_cast<const v4i*>(A + row * Rp + r0 + (p & 3) * 8);
        }
#pragma unroll
        for (int q = 0; q < PB; ++q) {
            const int p = threadIdx.x + q * 256;
            int64_t row = j0 + (p >> 2);
            if (row > J - 1) row = J - 1;
            rb[q] = *reinterpret_cast<const v4i*>(B + row * Rp + r0 + (p & 3) * 8);
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

// ---------------------------------------------------------------------------------------------
static inline int64_t pad32(int64_t v) { return (v + 31) / 32 * 32; }

size_t backward_workspace_bytes(int64_t M, int64_t N, int64_t K) {
    const int64_t Np = pad32(N), Mp = pad32(M);
    // g[M][Np], St[K][Np], gwT[N][Mp], qT[K][Mp], each bf16, each region 256-byte aligned
    auto al = [](size_t v) { return (v + 255) & ~(size_t)255; };
    return al((size_t)M * Np * 2) + al((size_t)K * Np * 2) + al((size_t)N * Mp * 2) +
           al((size_t)K * Mp * 2);
}

hipError_t launch_backward(const BackwardArgs& a, hipStream_t s) {
    const int64_t M = a.M, N = a.N, K = a.K, Np = pad32(N), Mp = pad32(M);
    auto al = [](size_t v) { return (v + 255) & ~(size_t)255; };
    char* ws = (char*)a.workspace;
    uint16_t* g = (uint16_t*)ws;
    uint16_t* St = (uint16_t*)(ws + al((size_t)M * Np * 2));
    uint16_t* gwT = (uint16_t*)((char*)St + al((size_t)K * Np * 2));
    uint16_t* qT = (uint16_t*)((char*)gwT + al((size_t)N * Mp * 2));

    if (a.dX) {
        const int64_t pairs = M * (Np / 2);
        cast_rows_bf16<<<(unsigned)((pairs + 255) / 256), 256, 0, s>>>(a.dY, M, N, Np, g);
        dim3 gb((unsigned)((tiles_n(N) + 3) / 4), (unsigned)tiles_k(K));
        bits_transpose_bf16<<<gb, 256, 0, s>>>(a.packed, N, K, Np, St);
        const unsigned blocks = (unsigned)(((M + 255) / 256) * ((K + 127) / 128));
        gemm_tn_bf16<256, 128><<<blocks, 256, 0, s>>>(g, St, M, K, Np, a.beta, 1.0f, a.dX);
    }
    if (a.dW) {
        dim3 gt((unsigned)((N + 63) / 64), (unsigned)((Mp + 63) / 64));
        transpose_cast_bf16<float><<<gt, 256, 0, s>>>(a.dY, M, N, Mp,
                                                       a.per_tensor ? nullptr : a.gamma, gwT);
        dim3 gq((unsigned)((K + 63) / 64), (unsigned)((Mp + 63) / 64));
        transpose_cast_bf16<int8_t><<<gq, 256, 0, s>>>(a.codes, M, K, Mp, nullptr, qT);
        const unsigned blocks = (unsigned)(((N + 255) / 256) * ((K + 127) / 128));
        gemm_tn_bf16<256, 128><<<blocks, 256, 0, s>>>(gwT, qT, N, K, Mp,
                                                      a.per_tensor ? a.gamma : nullptr,
                                                      a.per_tensor ? 1.0f / 128.0f : 1.0f, a.dW);
    }
    return hipGetLastError();
}

}  // namespace bl

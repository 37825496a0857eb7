// Weight preparation for BitLinear (arXiv 2310.11453, Eq. 1-3 and Eq. 12):
// alpha = mean(W), beta = mean|W|, bit = (W > alpha), packed 1 bit per weight
// into 16x512 tiles (layout described in common.h).  HBM-bound: 4 bytes read
// per weight per pass, 1/8 byte written.
#include "common.h"
#include "kernels.h"

namespace bl {

// ---- pass 1: per-block partial sums of W and |W - centre| in fp64 ----------
// partials[2*b] = sum of W, partials[2*b+1] = sum of |W - centre| over the
// block's grid-stride share.  centre_ptr == nullptr means centre = 0.
// The block's rows are cols4 float4 long and ld4 float4 apart (ld4 == cols4: contiguous, the
// index is used as it is).
__global__ __launch_bounds__(256) void weight_partial_sums(const float4* __restrict__ W4,
                                                           int64_t count4, int64_t cols4,
                                                           int64_t ld4,
                                                           const float* __restrict__ centre_ptr,
                                                           double* __restrict__ partials) {
    __shared__ double sm[4];
    const double centre = centre_ptr ? (double)*centre_ptr : 0.0;
    double s = 0.0, a = 0.0;
    const int64_t stride = (int64_t)gridDim.x * 256;
    const bool strided = ld4 != cols4;
    auto at = [&](int64_t i) { return W4[strided ? (i / cols4) * ld4 + i % cols4 : i]; };
    auto add = [&](const float4& w) {
        const double x = (double)w.x, y = (double)w.y, z = (double)w.z, u = (double)w.w;
        s += (x + y) + (z + u);
        a += (fabs(x - centre) + fabs(y - centre)) + (fabs(z - centre) + fabs(u - centre));
    };
    // four loads in flight per thread (one at a time, the pass is bound by their latency); the
    // order of the sums stays that of the plain loop
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < count4; i += 4 * stride) {
        const float4 w0 = at(i), w1 = at(i + stride), w2 = at(i + 2 * stride), w3 = at(i + 3 * stride);
        add(w0);
        add(w1);
        add(w2);
        add(w3);
    }
    for (; i < count4; i += stride) add(at(i));
    s = block_sum<4>(s, sm);
    a = block_sum<4>(a, sm);
    if (threadIdx.x == 0) {
        partials[2 * blockIdx.x] = s;
        partials[2 * blockIdx.x + 1] = a;
    }
}

// ---- pass 2: one block folds the partials in a fixed order -----------------
// write_alpha / write_beta select which scalars this call produces.
__global__ __launch_bounds__(256) void weight_finalize(const double* __restrict__ partials,
                                                       int nblocks, double count, int write_alpha,
                                                       int write_beta, float* __restrict__ alpha,
                                                       float* __restrict__ beta) {
    __shared__ double sm[4];
    double s = 0.0, a = 0.0;
    for (int i = threadIdx.x; i < nblocks; i += 256) {
        s += partials[2 * i];
        a += partials[2 * i + 1];
    }
    s = block_sum<4>(s, sm);
    a = block_sum<4>(a, sm);
    if (threadIdx.x == 0) {
        if (write_alpha) *alpha = (float)(s / count);
        if (write_beta) *beta = (float)(a / count);
    }
}

// ---- pass 3: compare with alpha and pack ----------------------------------
// One wave builds one 16x512 tile.  For each of the 16 rows the wave reads the
// row's 512 floats with two coalesced float4 loads per lane; a lane's four
// comparisons land in bit positions 8*j + i of the dword owned by lanes with
// the same (lane % 16), which two xor-shuffles OR together.  The tile is
// staged in LDS so the final store is one 16-byte write per lane.
__global__ __launch_bounds__(256) void pack_tiles(const float* __restrict__ W, int64_t N,
                                                  int64_t K, int64_t ldw,
                                                  const float* __restrict__ alpha_ptr,
                                                  uint32_t* __restrict__ packed) {
    __shared__ uint32_t sm[4][256];
    const int wave = threadIdx.x / kWave, l = threadIdx.x % kWave;
    const int64_t TN = tiles_n(N), TK = tiles_k(K);
    const int64_t task = (int64_t)blockIdx.x * 4 + wave;
    const bool live = task < TN * TK;
    const int64_t tn = live ? task / TK : 0, tk = live ? task % TK : 0;
    const float alpha = *alpha_ptr;

#pragma unroll 4
    for (int c = 0; c < kTileN; ++c) {
        const int64_t n = tn * kTileN + c;
        uint32_t part = 0;
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int64_t k = tk * kChunkK + 256 * it + 4 * l;
            if (live && n < N && k < K) {
                const float4 w = *reinterpret_cast<const float4*>(W + n * ldw + k);
                const int i = 4 * it + (l >> 4);
                part |= (uint32_t)(w.x > alpha) << i;
                part |= (uint32_t)(w.y > alpha) << (8 + i);
                part |= (uint32_t)(w.z > alpha) << (16 + i);
                part |= (uint32_t)(w.w > alpha) << (24 + i);
            }
        }
        part |= (uint32_t)__shfl_xor((int)part, 16, kWave);
        part |= (uint32_t)__shfl_xor((int)part, 32, kWave);
        if (l < 16) sm[wave][((l >> 2) * 16 + c) * 4 + (l & 3)] = part;
    }
    __syncthreads();
    if (live) {
        const uint4 v = *reinterpret_cast<const uint4*>(&sm[wave][l * 4]);
        *reinterpret_cast<uint4*>(packed + tile_dword_offset(tn, tk, TK) + l * 4) = v;
    }
}

// ---- inspection: tiles -> canonical words ---------------------------------
// canonical[n][kw] bit b  <->  sign bit of (n, k = 32*kw + b).
__global__ __launch_bounds__(256) void tiles_to_canonical(const uint32_t* __restrict__ packed,
                                                          int64_t N, int64_t K,
                                                          uint32_t* __restrict__ canonical,
                                                          int64_t ldc) {
    const int64_t KW = K / 32;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= N * KW) return;
    const int64_t n = idx / KW, kw = idx % KW;
    const int64_t TK = tiles_k(K);
    const int64_t tn = n / kTileN, c = n % kTileN;
    const int64_t k0 = kw * 32;
    const int64_t tk = k0 / kChunkK;
    const int r0 = (int)(k0 % kChunkK);
    const int i = r0 / 64;
    const uint32_t* tile = packed + tile_dword_offset(tn, tk, TK);
    uint32_t word = 0;
    for (int b = 0; b < 32; ++b) {
        const int r = r0 + b;
        const int g = (r % 64) / 16, d = (r % 16) / 4, j = r % 4;
        const uint32_t dw = tile[(g * 16 + c) * 4 + d];
        word |= ((dw >> (8 * j + i)) & 1u) << b;
    }
    canonical[n * ldc + kw] = word;
}

// ---- wsum[n] = sum_k s[n,k] = 2 * popcount(row n) - K, from the packed tiles ----------
// One wave per tile row: it walks the row's tiles (1 KiB, coalesced), every lane counts the set
// bits of its 4 dwords (16 columns of weight row lane%16), the four lanes of a row add up.
// Padding bits are zero, so only real columns are counted.
__global__ __launch_bounds__(256) void weight_rowsums(const uint32_t* __restrict__ packed,
                                                      int64_t N, int64_t K,
                                                      int32_t* __restrict__ wsum) {
    const int wave = threadIdx.x / kWave, l = threadIdx.x % kWave;
    const int64_t TN = tiles_n(N), TK = tiles_k(K);
    const int64_t tn = (int64_t)blockIdx.x * 4 + wave;
    if (tn >= TN) return;
    int pop = 0;
    for (int64_t tk = 0; tk < TK; ++tk) {
        const uint4 v = *reinterpret_cast<const uint4*>(packed + tile_dword_offset(tn, tk, TK) + l * 4);
        pop += __popc(v.x) + __popc(v.y) + __popc(v.z) + __popc(v.w);
    }
    pop += __shfl_xor(pop, 16, kWave);
    pop += __shfl_xor(pop, 32, kWave);
    const int64_t n = tn * kTileN + l;
    if (l < kTileN && n < N) wsum[n] = 2 * pop - (int)K;
}

// ---------------------------------------------------------------------------
int reduce_grid(int64_t count4) {
    int64_t g = (count4 + 256 * 8 - 1) / (256 * 8);
    if (g < 1) g = 1;
    if (g > 1024) g = 1024;
    return (int)g;
}

hipError_t launch_pack(const float* W, int64_t N, int64_t K, int64_t ldw, bool beta_centered,
                       uint32_t* packed, float* alpha, float* beta, double* partials, hipStream_t s) {
    const int64_t count4 = N * K / 4;
    const int G = reduce_grid(count4);
    const double cnt = (double)N * (double)K;
    const float4* W4 = (const float4*)W;
    weight_partial_sums<<<G, 256, 0, s>>>(W4, count4, K / 4, ldw / 4, nullptr, partials);
    weight_finalize<<<1, 256, 0, s>>>(partials, G, cnt, 1, beta_centered ? 0 : 1, alpha, beta);
    if (beta_centered) {
        weight_partial_sums<<<G, 256, 0, s>>>(W4, count4, K / 4, ldw / 4, alpha, partials);
        weight_finalize<<<1, 256, 0, s>>>(partials, G, cnt, 0, 1, alpha, beta);
    }
    const int64_t tasks = tiles_n(N) * tiles_k(K);
    pack_tiles<<<(unsigned)((tasks + 3) / 4), 256, 0, s>>>(W, N, K, ldw, alpha, packed);
    return hipGetLastError();
}

hipError_t launch_weight_rowsums(const uint32_t* packed, int64_t N, int64_t K, int32_t* wsum,
                                 hipStream_t s) {
    weight_rowsums<<<(unsigned)((tiles_n(N) + 3) / 4), 256, 0, s>>>(packed, N, K, wsum);
    return hipGetLastError();
}

hipError_t launch_to_canonical(const uint32_t* packed, int64_t N, int64_t K, uint32_t* canonical,
                               int64_t ldc, hipStream_t s) {
    const int64_t words = N * (K / 32);
    tiles_to_canonical<<<(unsigned)((words + 255) / 256), 256, 0, s>>>(packed, N, K, canonical, ldc);
    return hipGetLastError();
}

}  // namespace bl

// Device-side helpers shared by the BitLinear kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bl {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;
constexpr int kTileN = 16;    // weight rows per packed tile
constexpr int kChunkK = 512;  // fan-in elements per packed tile

// ---------------------------------------------------------------------------
// Packed 1-bit layout ("tiles").  The [N,K] sign matrix is cut into tiles of
// 16 rows x 512 columns; a tile is 1 KiB = 64 lanes x 4 dwords, stored so that
// one wave reads it with a single fully coalesced 16-byte-per-lane load.
//   lane  = g*16 + c      c = row inside the tile (0..15), g = 0..3
//   dword = d             d = 0..3
//   bit   = 8*j + i       j = 0..3, i = 0..7
//   <->  n = 16*tile_n + c,  k = 512*tile_k + 64*i + 16*g + 4*d + j
// For a fixed i the 16 bytes (d,j) of a lane are 16 consecutive k, which is
// the operand shape of the i8 MFMA instructions: (w >> i) & 0x01010101 turns a
// dword into four {0,1} bytes, and w & (0x01010101 << i) into four {0,2^i}
// bytes, with no cross-lane traffic.  Tiles are ordered [tile_n][tile_k].
// ---------------------------------------------------------------------------
__host__ __device__ inline int64_t tiles_n(int64_t N) { return (N + kTileN - 1) / kTileN; }
__host__ __device__ inline int64_t tiles_k(int64_t K) { return (K + kChunkK - 1) / kChunkK; }
__host__ __device__ inline int64_t tile_dword_offset(int64_t tn, int64_t tk, int64_t TK) {
    return (tn * TK + tk) * 256;
}

// ---------------------------------------------------------------------------
// Wave and block reductions.  All of them use a fixed butterfly order, so the
// result is identical run to run.
// ---------------------------------------------------------------------------
__device__ inline double shfl_xor_f64(double v, int mask) {
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __shfl_xor(lo, mask, kWave);
    hi = __shfl_xor(hi, mask, kWave);
    return __hiloint2double(hi, lo);
}

__device__ inline double wave_sum(double v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += shfl_xor_f64(v, m);
    return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, kWave));
    return v;
}
__device__ inline int wave_sum(int v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
    return v;
}

// Block-wide reductions over NW waves; every thread gets the result.
// `smem` must hold NW elements and may be reused after the call returns.
template <int NW>
__device__ inline double block_sum(double v, double* smem) {
    v = wave_sum(v);
    if constexpr (NW == 1) return v;
    const int w = threadIdx.x / kWave;
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) smem[w] = v;
    __syncthreads();
    double r = smem[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) r += smem[i];
    return r;
}
template <int NW>
__device__ inline float block_max(float v, float* smem) {
    v = wave_max(v);
    if constexpr (NW == 1) return v;
    const int w = threadIdx.x / kWave;
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) smem[w] = v;
    __syncthreads();
    float r = smem[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) r = fmaxf(r, smem[i]);
    return r;
}
template <int NW>
__device__ inline int block_sum(int v, int* smem) {
    v = wave_sum(v);
    if constexpr (NW == 1) return v;
    const int w = threadIdx.x / kWave;
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) smem[w] = v;
    __syncthreads();
    int r = smem[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) r += smem[i];
    return r;
}

}  // namespace bl

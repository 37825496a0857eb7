// 1-bit x 8-bit GEMM + dequantisation for a handful of tokens (M <= 16):
//   Y[m,n] = (sum_k q[m,k] * s[n,k]) * beta * gamma_m / 128     (Eq. 7, Eq. 11)
// of arXiv 2310.11453, with s in {-1,+1} stored 1 bit per weight.
//
// This shape is bound by streaming the packed weights from HBM, and the only
// ALU work the stream can afford is about two VALU operations per 32 weights.
// The kernel therefore never expands a bit to a +-1 byte.  One AND with
// 0x01010101 << i turns a packed dword into four bytes in {0, 2^i} ("bit plane
// i", 2^7 read as -128 by the signed MFMA), each plane feeds its own i8 MFMA
// accumulator, and the planes are folded once per output tile:
//   sum_k q b = sum_i acc_i / c_i,  c_i = 2^i (i < 7), c_7 = -128   (exact shifts)
//   sum_k q s = 2 * sum_k q b - sum_k q,        s = 2 b - 1
// with sum_k q taken from the quantiser's row sums.
//
// Work split: a workgroup owns T consecutive 16-row weight tiles and all of K;
// wave w of the group owns the K-chunks {w*C .. w*C+C-1} (+ W*C per round) and
// keeps the matching slice of the activation codes in registers as MFMA
// operands, reusing them for every tile.  Partial sums meet in LDS.
#include "common.h"
#include "kernels.h"

namespace bl {

template <int C, int T, int MAXT>
__global__ __launch_bounds__(MAXT) void gemm_decode_kernel(GemmArgs a) {
    extern __shared__ int red[];  // [W][T][64][4]
    const int W = blockDim.x / kWave;
    const int w = threadIdx.x / kWave, l = threadIdx.x % kWave;
    const int m = l & 15, g = l >> 4;
    const int64_t TN = tiles_n(a.N), TK = tiles_k(a.K);
    const int M = (int)a.M;

    int part[T][4];
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) part[t][r] = 0;

    const int64_t rounds = (TK + (int64_t)W * C - 1) / ((int64_t)W * C);
    for (int64_t rd = 0; rd < rounds; ++rd) {
        const int64_t tk0 = (rd * W + w) * C;

        // activation operand: lane (m, g) holds codes[m][512*tk + 64*i + 16*g .. +15]
        v4i act[C][8];
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int64_t k = (tk0 + c) * kChunkK + 64 * i + 16 * g;
                v4i z = {0, 0, 0, 0};
                if (m < M && k < a.K) z = *reinterpret_cast<const v4i*>(a.codes + (int64_t)m * a.K + k);
                act[c][i] = z;
            }

        // all weight tiles of this round are requested before the first MFMA
        v4i wt[T][C];
#pragma unroll
        for (int t = 0; t < T; ++t)
#pragma unroll
            for (int c = 0; c < C; ++c) {
                const int64_t tn = (int64_t)blockIdx.x * T + t, tk = tk0 + c;
                v4i z = {0, 0, 0, 0};
                if (tn < TN && tk < TK)
                    z = *reinterpret_cast<const v4i*>(a.packed + tile_dword_offset(tn, tk, TK) + l * 4);
                wt[t][c] = z;
            }

#pragma unroll
        for (int t = 0; t < T; ++t) {
            v4i acc[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = (v4i){0, 0, 0, 0};
#pragma unroll
            for (int c = 0; c < C; ++c)
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int mask = (int)(0x01010101u << i);
                    const v4i plane = wt[t][c] & mask;
                    // rows of the MFMA = weights (n), columns = tokens (m)
                    acc[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(plane, act[c][i], acc[i], 0, 0, 0);
                }
            // fold the planes: every acc[i] is an exact multiple of 2^i
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                int h = acc[6][r];
#pragma unroll
                for (int i = 5; i >= 0; --i) h = acc[i][r] + (h >> 1);
                part[t][r] += h - (acc[7][r] >> 7);
            }
        }
    }

    // cross-wave reduction over K, then the dequantisation epilogue
    if (W > 1) {
#pragma unroll
        for (int t = 0; t < T; ++t)
            *reinterpret_cast<v4i*>(&red[((w * T + t) * kWave + l) * 4]) =
                (v4i){part[t][0], part[t][1], part[t][2], part[t][3]};
        __syncthreads();
    }
    const float beta = *a.beta;
    for (int t = w; t < T; t += W) {
        v4i sum;
        if (W > 1) {
            sum = (v4i){0, 0, 0, 0};
            for (int ww = 0; ww < W; ++ww)
                sum += *reinterpret_cast<const v4i*>(&red[((ww * T + t) * kWave + l) * 4]);
        } else {
            // W == 1: t == the only wave's own tile index; select without dynamic indexing
            sum = (v4i){0, 0, 0, 0};
#pragma unroll
            for (int tt = 0; tt < T; ++tt)
                if (tt == t) sum = (v4i){part[tt][0], part[tt][1], part[tt][2], part[tt][3]};
        }
        const int64_t tn = (int64_t)blockIdx.x * T + t;
        const int64_t n = tn * kTileN + 4 * g;
        if (tn >= TN || m >= M || n >= a.N) continue;
        const int rs = a.rowsum[m];
        const v4i pm = sum * 2 - rs;  // sum_k q s
        float* y = a.Y + (int64_t)m * a.N + n;
        if (a.out_acc) {
            int* yi = reinterpret_cast<int*>(y);
            if ((a.N & 3) == 0) *reinterpret_cast<v4i*>(yi) = pm;
            else
                for (int r = 0; r < 4; ++r)
                    if (n + r < a.N) yi[r] = pm[r];
        } else {
            const float gm = a.per_tensor ? a.gamma[0] : a.gamma[m];
            const float sc = (beta * gm) / 128.0f;
            const v4f o = {(float)pm[0] * sc, (float)pm[1] * sc, (float)pm[2] * sc, (float)pm[3] * sc};
            if ((a.N & 3) == 0) *reinterpret_cast<v4f*>(y) = o;
            else
                for (int r = 0; r < 4; ++r)
                    if (n + r < a.N) y[r] = o[r];
        }
    }
}

static int env_int(const char* name, int dflt) {
    const char* e = getenv(name);
    return e ? atoi(e) : dflt;
}

template <int C, int T, int MAXT>
static void launch_one(const GemmArgs& a, int W, hipStream_t s) {
    const int64_t TN = tiles_n(a.N);
    const unsigned grid = (unsigned)((TN + T - 1) / T);
    const size_t lds = W > 1 ? (size_t)W * T * 1024 : 0;
    gemm_decode_kernel<C, T, MAXT><<<grid, W * kWave, lds, s>>>(a);
}

hipError_t launch_gemm_decode(const GemmArgs& a, hipStream_t s) {
    const int64_t TN = tiles_n(a.N), TK = tiles_k(a.K);
    // waves per group cover K: one chunk each (up to 16 waves) while K <= 8192, two chunks
    // each (up to 8 waves, which leaves 256 registers per lane) beyond; longer K loops
    const int C = TK <= 16 ? 1 : 2;
    const int maxW = C == 1 ? 16 : 8;
    const int64_t slots = (TK + C - 1) / C;
    const int64_t rounds = (slots + maxW - 1) / maxW;
    const int W = (int)((slots + rounds - 1) / rounds);
    // tiles per group: few when the matrix is small (parallelism first), more when
    // 16 tokens make the activation operand as heavy as the weights
    int T = TN >= 1024 ? (a.M > 4 ? 4 : 2) : 1;
    T = env_int("BITLINEAR_DECODE_T", T);
    if (C == 1) {
        if (T == 1) launch_one<1, 1, 1024>(a, W, s);
        else if (T == 2) launch_one<1, 2, 1024>(a, W, s);
        else launch_one<1, 4, 1024>(a, W, s);
    } else {
        if (T == 1) launch_one<2, 1, 512>(a, W, s);
        else if (T == 2) launch_one<2, 2, 512>(a, W, s);
        else launch_one<2, 4, 512>(a, W, s);
    }
    return hipGetLastError();
}

}  // namespace bl

// 1-bit x 8-bit GEMM + dequantisation for 17 to 32 tokens, Eq. 7 and Eq. 11 of arXiv 2310.11453,
// built like the small-batch kernel: the packed weights stream from HBM through registers exactly
// once, and the activation codes of all tokens wait for them in registers as MFMA operands.
//
//  * v_mfma_i32_32x32x32_i8 with the WEIGHTS as its row operand (two 16-row packed tiles make
//    32 rows) and the TOKENS as its 32 columns.  A lane's 16-byte load of a packed tile covers 16
//    consecutive k in each of the 8 bit planes; (w >> i) & 0x01010101 turns plane i into {0,1}
//    operand bytes.  The epilogue restores sum_k q s = 2 sum_k q b - sum_k q with the
//    quantiser's row sums.
//  * Wave w of a workgroup owns the 512-chunks w, w + W, ... of K.  Per chunk it reads the codes
//    of all tokens as whole 512-byte rows, turns them into the MFMA's column operands through a
//    staging area of its own in LDS (no other wave touches it, so no barrier), and walks the
//    workgroup's pairs of weight tiles.  The next chunk's codes and tiles are fetched during the
//    MFMAs of this one.
//  * The waves' partial sums meet in LDS by integer atomic adds (order-free), then all threads
//    dequantise and store 16 bytes each.
// Every workgroup reads all M x K codes (from L2), which is why the token count is bounded: at
// more tokens that traffic, not the weight stream, sets the time, and the LDS-tiled mid-batch
// kernel is as fast.  Long K is split over workgroups (second kernel: splitk_reduce) when the
// caller brought the workspace.

#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace bl {

namespace stream {
constexpr int kTokens = 32;    // columns of the MFMA
constexpr int kMaxPairs = 4;   // pairs of weight tiles per workgroup (the switch below names each count)
constexpr int kPitch = 33;     // ints per weight row in LDS: 32 tokens + 1 (column reads hit every bank)
constexpr int kMaxWaves = 8;
constexpr int kStageRow = 528; // bytes per token in a wave's staging area: 512 + 16, so that the 16-byte
                               // operand reads of 16 tokens at one k fall on different banks
constexpr int kStageBytes = kTokens * kStageRow;
}  // namespace stream

// grid.x workgroups share the pairs of tile rows, grid.y = K-slices (a.split_k elements each,
// 0 = one slice).  M <= 32.
__global__ __launch_bounds__(stream::kMaxWaves* kWave) void gemm_stream_kernel(GemmArgs a) {
    using namespace stream;
    __shared__ int red[kMaxPairs * 32 * kPitch];
    // per wave: one chunk of the codes of 32 tokens on its way from row-major memory (read as
    // whole 512-byte rows) to the MFMA's operand layout (16-byte pieces of 32 tokens at one k)
    __shared__ __attribute__((aligned(16))) uint8_t stage[kMaxWaves * kStageBytes];
    __shared__ int tok_sum[kTokens];
    __shared__ float tok_sc[kTokens], tok_eta[kTokens];

    const int W = (int)blockDim.x / kWave;
    const int w = __builtin_amdgcn_readfirstlane((int)threadIdx.x / kWave), l = threadIdx.x % kWave;
    const int tok = l & 31, half = l >> 5;
    const int M = (int)a.M;
    const int64_t N = a.N;
    const int64_t TN = tiles_n(N);
    const int64_t TKp = a.tk_pitch ? a.tk_pitch : tiles_k(a.K);
    const int sp = (int)blockIdx.y;
    int64_t k0 = 0, K = a.K;
    if (a.split_k) {
        k0 = (int64_t)sp * a.split_k;
        K = a.K - k0 < a.split_k ? a.K - k0 : a.split_k;
    }
    const int TK = (int)tiles_k(K);

    // this workgroup's pairs of tile rows
    const int64_t TP = (TN + 1) / 2;
    const int p0 = (int)(TP * blockIdx.x / gridDim.x), p1 = (int)(TP * (blockIdx.x + 1) / gridDim.x);
    const int np = p1 - p0;  // <= kMaxPairs (the launcher sees to it)

    for (int i = threadIdx.x; i < np * 32 * kPitch; i += blockDim.x) red[i] = 0;
    // per-token factors of the epilogue, fetched now so that it waits on no load of theirs
    if ((int)threadIdx.x < M && !a.split_k) {
        const int m = threadIdx.x;
        tok_sum[m] = a.rowsum[m * a.gstride];
        // gamma / 128 is exact
        tok_sc[m] = a.out_acc ? 0.f : a.gamma[a.per_tensor ? 0 : m * a.gstride] * 0.0078125f;
        tok_eta[m] = a.eta && !a.out_acc ? a.eta[a.per_tensor ? 0 : m * a.gstride] : 0.f;
    }
    __syncthreads();

    // lane -> weight row (tok is also the row index of the A operand) and its 16-byte slot:
    // tile 2p + row/16, slot (2 mf + half) * 16 + row % 16
    const int wrow = tok;
    const uint32_t slot_dw = (uint32_t)((half * 16 + (wrow & 15)) * 4);  // + 128 dwords for mf = 1
    auto pair_ptr = [&](int p, int c) {
        int64_t tn = (int64_t)(p0 + p) * 2 + (wrow >> 4);
        if (tn > TN - 1) tn = TN - 1;  // its rows are never stored
        return a.packed + tile_dword_offset(tn, k0 / kChunkK + c, TKp) + slot_dw;
    };

    // NP = pairs of this workgroup, a compile-time count so that the tiles sit in registers
    auto wave_chunks = [&](auto np_c) {
        constexpr int NP = decltype(np_c)::value;
        const int steps = (TK - w + W - 1) / W;  // chunks w, w + W, ...
        uint8_t* const mine = stage + w * kStageBytes;
        v4i q[NP][2], qn[NP][2], raw[16];
        auto load_q = [&](v4i (&dst)[NP][2], int c) {
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                const uint32_t* s = pair_ptr(p, c);
                dst[p][0] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(s));
                dst[p][1] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(s + 128));
            }
        };
        // wave-load jj brings tokens 2 jj and 2 jj + 1: lane -> (token, 16-byte piece), whole rows
        auto load_raw = [&](int c) {
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) {
                const int t = 2 * jj + half;
                const int m = t < M ? t : M - 1;
                int64_t k = (int64_t)c * kChunkK + 16 * tok;
                if (k > K - 16) k = K - 16;  // the packed bits there are zero
                raw[jj] = *reinterpret_cast<const v4i*>(a.codes + (int64_t)m * a.ldq + k0 + k);
            }
        };
        load_q(q, w);
        load_raw(w);
        // the first tiles are waited for here, once: inside the loop a wait for them would have to
        // count the conditional fetches behind them as absent, and so wait for those as well
#pragma unroll
        for (int p = 0; p < NP; ++p) asm volatile("" : "+v"(q[p][0]), "+v"(q[p][1]));
#pragma unroll 1
        for (int st = 0; st < steps; ++st) {
            // ---- the fetched codes become the B operands of plane i, k-half mf -------------------
            v4i act[8][2];
#pragma unroll
            for (int jj = 0; jj < 16; ++jj)
                *reinterpret_cast<v4i*>(mine + (2 * jj + half) * kStageRow + 16 * tok) = raw[jj];
            __builtin_amdgcn_wave_barrier();  // same wave, other lanes: LDS keeps a wave's accesses in order
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int mf = 0; mf < 2; ++mf)
                    act[i][mf] =
                        *reinterpret_cast<const v4i*>(mine + tok * kStageRow + 64 * i + 32 * mf + 16 * half);
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_sched_barrier(0);
            // ---- the next chunk's fetches (wave-uniform branch) ------------------------------------
            const bool more = st + 1 < steps;
            if (more) {
                load_raw((st + 1) * W + w);
                load_q(qn, (st + 1) * W + w);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                v16i acc;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[r] = 0;
#pragma unroll
                for (int i = 0; i < 8; ++i)
#pragma unroll
                    for (int mf = 0; mf < 2; ++mf) {
                        const v4i wv = q[p][mf];
                        v4i b;
#pragma unroll
                        for (int d = 0; d < 4; ++d) b[d] = (int)(((uint32_t)wv[d] >> i) & 0x01010101u);
                        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(b, act[i][mf], acc, 0, 0, 0);
                    }
                // lane (tok, half) holds token tok, weight rows 8 (r/4) + 4 half + r%4
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    atomicAdd(&red[(p * 32 + 8 * (r >> 2) + 4 * half + (r & 3)) * kPitch + tok], acc[r]);
                // the scheduler stays inside one pair: across pairs it would expand every plane of
                // every pair ahead of the MFMAs, and the registers run out
                __builtin_amdgcn_sched_barrier(0);
            }
            if (more) {
#pragma unroll
                for (int p = 0; p < NP; ++p) {
                    q[p][0] = qn[p][0];
                    q[p][1] = qn[p][1];
                }
            }
        }
    };

    if (w < TK) {  // uniform per wave; nothing in there synchronises across waves
        switch (np) {
            case 1: wave_chunks(std::integral_constant<int, 1>{}); break;
            case 2: wave_chunks(std::integral_constant<int, 2>{}); break;
            case 3: wave_chunks(std::integral_constant<int, 3>{}); break;
            case 4: wave_chunks(std::integral_constant<int, 4>{}); break;
            default: break;
        }
    }
    __syncthreads();

    // ---- epilogue (Eq. 11): sum_k q s = 2 sum_k q b - sum_k q ; y = that * (beta gamma / 128) ----
    // thread -> four consecutive weight rows of every pair and every (blockDim / 8)-th token
    const int nl0 = (threadIdx.x & 7) * 4, MG = blockDim.x >> 3;
    const bool raw_out = a.split_k || a.out_acc;
    uint32_t* const out = a.split_k ? reinterpret_cast<uint32_t*>(a.split_ws) + (int64_t)sp * M * N
                                    : reinterpret_cast<uint32_t*>(a.Y);
    const bool vec = (N & 3) == 0;  // then n0 + 3 < N and the row starts 16-byte aligned
    float beta[kMaxPairs][4], wsum[kMaxPairs][4];
#pragma unroll
    for (int p = 0; p < kMaxPairs; ++p)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t n = ((int64_t)(p0 + p) * 2) * kTileN + nl0 + j;
            const bool live = p < np && n < N && !raw_out;
            beta[p][j] = live ? a.beta[((uint32_t)n / (uint32_t)a.beta_rows) * a.beta_stride] : 0.f;
            wsum[p][j] = live && a.eta ? (float)a.wsum[n] : 0.f;
        }
#pragma unroll
    for (int p = 0; p < kMaxPairs; ++p) {
        const int64_t n0 = ((int64_t)(p0 + p) * 2) * kTileN + nl0;
        if (p >= np || n0 >= N) continue;
        for (int m = threadIdx.x >> 3; m < M; m += MG) {
            uint32_t o[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int s2 = 2 * red[(p * 32 + nl0 + j) * kPitch + m];
                if (a.split_k) {
                    o[j] = (uint32_t)s2;
                    continue;
                }
                const int pm = s2 - tok_sum[m];
                if (a.out_acc) {
                    o[j] = (uint32_t)pm;
                    continue;
                }
                // beta * (gamma / 128) has the bits of (beta * gamma) / 128
                float y = (float)pm * (beta[p][j] * tok_sc[m]);
                if (a.eta) y = y + (beta[p][j] * tok_eta[m]) * wsum[p][j];  // Eq. 6
                if (a.accumulate && n0 + j < N) y += a.Y[m * N + n0 + j];    // a later K-group (Eq. 13-15)
                o[j] = __float_as_uint(y);
            }
            uint32_t* const dst = out + (int64_t)m * N + n0;
            if (vec) {
                *reinterpret_cast<uint4*>(dst) = make_uint4(o[0], o[1], o[2], o[3]);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (n0 + j < N) dst[j] = o[j];
            }
        }
    }
}

static int stream_cus() {
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

// K-slices for 16 < M <= 32: longer K than 16 chunks (two per wave) is cut into slices of at most
// 16 chunks.  0 = no split.
int64_t stream_split_tiles(int64_t M, int64_t K) {
    if (M <= 16 || M > stream::kTokens) return 0;
    const int64_t TK = tiles_k(K);
    if (TK <= 16) return 0;
    const int64_t splits = (TK + 15) / 16;
    return (TK + splits - 1) / splits;
}

// false: the shape is not for this kernel (the mid-batch MFMA-tile kernel takes it)
bool launch_gemm_stream(const GemmArgs& a_in, hipStream_t s) {
    using namespace stream;
    GemmArgs a = a_in;
    a.split_k = 0;
    if (a.M <= 16 || a.M > kTokens || a.K >= ((int64_t)1 << 22)) return false;
    const int64_t TP = (tiles_n(a.N) + 1) / 2;
    int grid = stream_cus();
    if (grid > TP) grid = (int)TP;
    if ((TP + grid - 1) / grid > kMaxPairs) return false;
    // every workgroup reads the codes of 32 tokens over all of K from L2 (K-slices share the
    // workgroups' pairs, so the split does not change the sum): past about 128 MB of that the
    // LDS-tiled kernel, whose workgroups share codes across more weight rows, measured faster
    // (M = 32, K = 28672, N = 7168: 34 us here, 27 us there)
    if ((int64_t)grid * kTokens * a.K > ((int64_t)1 << 27)) return false;
    int splits = 1;
    const int64_t per = stream_split_tiles(a.M, a.K);
    const int64_t nsl = per ? (tiles_k(a.K) + per - 1) / per : 1;
    const size_t need = (size_t)nsl * (size_t)a.M * (size_t)a.N * 4;
    if (per && a.split_ws && a.split_ws_bytes >= need && !tuning().mid_nosplit) {
        splits = (int)nsl;
        a.tk_pitch = a.tk_pitch ? a.tk_pitch : tiles_k(a.K);
        a.split_k = per * kChunkK;
    }
    // as many waves as give every wave the same number of chunks (14 chunks: 7 waves, not 8)
    const int64_t TKs = splits > 1 ? per : tiles_k(a.K);
    const int64_t rounds = (TKs + kMaxWaves - 1) / kMaxWaves;
    const int W = (int)((TKs + rounds - 1) / rounds);
    const dim3 g((unsigned)grid, (unsigned)splits);
    gemm_stream_kernel<<<g, W * kWave, 0, s>>>(a);
    if (splits > 1) launch_splitk_reduce(a, splits, s);
    return true;
}

}  // namespace bl

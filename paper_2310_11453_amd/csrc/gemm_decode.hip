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
// Work split: a workgroup owns up to T consecutive 16-row weight tiles and all of K;
// wave w of the group owns the K-chunks {w*C .. w*C+C-1} (+ W*C per round) and
// keeps the matching slice of the activation codes in registers as MFMA
// operands, reusing them for every tile.  Partial sums meet in LDS.
#include "common.h"
#include "kernels.h"
#include "rowops.h"

namespace bl {

// LayerNorm (Eq. 12) and the 8-bit absmax quantiser (Eq. 4-5) of ONE token by a whole workgroup,
// with the arithmetic of the stand-alone quantiser: sums in fp64 about an element of the row,
// the normalised value rounded once to fp32, then scale = 128 / gamma, rne, clamp - one fp32
// operation per step.  The codes go to `lds_codes` (K bytes); returns gamma and sum_k codes.
// Every thread of the workgroup must call it (it synchronises), K <= 4 * NV * blockDim.
// `after_loads` runs once the row's loads are issued: loads return in order, so whatever else
// the caller wants in flight meanwhile has to queue behind the row, not ahead of it.
struct TokenQuant {
    float gamma;
    int rowsum;
};
template <int NV, class F>
__device__ inline TokenQuant quant_token(const GemmArgs& a, uint32_t* lds_codes, double (*smd)[16],
                                         float (*smf)[16], int* smi, F&& after_loads) {
    const int T = blockDim.x, t = threadIdx.x, W = T / kWave, wave = t / kWave;
    const bool lead = (t & (kWave - 1)) == 0;
    const int K4 = (int)(a.K / 4);
    const float4* __restrict__ x4 = reinterpret_cast<const float4*>(a.x_row);
    float4 v[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int idx = t + j * T;
        v[j] = x4[idx < K4 ? idx : K4 - 1];
    }
    const float first = a.x_row[0];
    after_loads();
    const bool affine = a.ln_gain != nullptr || a.ln_bias != nullptr;
    bool have_amax = false;
    float amax = 0.f;
    if (!a.skip_ln) {
        const double c = (double)first;
        double s = 0.0, q = 0.0;
        float mn = v[0].x, mx = v[0].x;  // always an element of the row (clamped index)
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            if (t + j * T < K4) {
                const double dx = (double)v[j].x, dy = (double)v[j].y;
                const double dz = (double)v[j].z, dw = (double)v[j].w;
                s += (dx + dy) + (dz + dw);
                q = fma(dx - c, dx - c, q);
                q = fma(dy - c, dy - c, q);
                q = fma(dz - c, dz - c, q);
                q = fma(dw - c, dw - c, q);
                mn = fminf(fminf(mn, v[j].x), fminf(fminf(v[j].y, v[j].z), v[j].w));
                mx = fmaxf(fmaxf(mx, v[j].x), fmaxf(fmaxf(v[j].y, v[j].z), v[j].w));
            }
        }
        s = wave_reduce(s, OpSum{});
        q = wave_reduce(q, OpSum{});
        mn = wave_reduce(mn, OpMin{});
        mx = wave_reduce(mx, OpMax{});
        if (lead) {
            smd[0][wave] = s;
            smd[1][wave] = q;
            smf[0][wave] = mn;
            smf[1][wave] = mx;
        }
        __syncthreads();
        s = smd[0][0];
        q = smd[1][0];
        mn = smf[0][0];
        mx = smf[1][0];
        for (int i = 1; i < W; ++i) {
            s += smd[0][i];
            q += smd[1][i];
            mn = fminf(mn, smf[0][i]);
            mx = fmaxf(mx, smf[1][i]);
        }
        const double mu = s / (double)a.K;
        const double var = fmax(q / (double)a.K - (mu - c) * (mu - c), 0.0);
        const double rstd = 1.0 / sqrt(var + (double)a.ln_eps);
        if (!affine) {
            // x -> fl32((x - mu) * rstd) is monotone: the largest magnitude sits at min or max
            const float lo = (float)(((double)mn - mu) * rstd);
            const float hi = (float)(((double)mx - mu) * rstd);
            amax = fmaxf(fabsf(lo), fabsf(hi));
            have_amax = true;
        }
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int idx = t + j * T;
            float4 o;
            o.x = (float)(((double)v[j].x - mu) * rstd);
            o.y = (float)(((double)v[j].y - mu) * rstd);
            o.z = (float)(((double)v[j].z - mu) * rstd);
            o.w = (float)(((double)v[j].w - mu) * rstd);
            if (idx < K4) {
                if (a.ln_gain) {
                    const float4 g = reinterpret_cast<const float4*>(a.ln_gain)[idx];
                    o.x = o.x * g.x; o.y = o.y * g.y; o.z = o.z * g.z; o.w = o.w * g.w;
                }
                if (a.ln_bias) {
                    const float4 b = reinterpret_cast<const float4*>(a.ln_bias)[idx];
                    o.x = o.x + b.x; o.y = o.y + b.y; o.z = o.z + b.z; o.w = o.w + b.w;
                }
                v[j] = o;
            }
        }
    }
    if (!have_amax) {  // uniform: no LayerNorm, or a gain / bias after it
        float m = 0.f;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            if (t + j * T < K4)
                m = fmaxf(m, fmaxf(fmaxf(fabsf(v[j].x), fabsf(v[j].y)), fmaxf(fabsf(v[j].z), fabsf(v[j].w))));
        }
        m = wave_reduce(m, OpMax{});
        if (lead) smf[2][wave] = m;
        __syncthreads();
        amax = smf[2][0];
        for (int i = 1; i < W; ++i) amax = fmaxf(amax, smf[2][i]);
    }
    const float gamma = fmaxf(amax, 1e-5f);
    const float scale = 128.0f / gamma;
    if (blockIdx.x == 0 && blockIdx.y == 0 && a.xhat_out) {  // uniform
        float4* __restrict__ d4 = reinterpret_cast<float4*>(a.xhat_out);
#pragma unroll
        for (int j = 0; j < NV; ++j)
            if (t + j * T < K4) d4[t + j * T] = v[j];
    }
    int rs = 0;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int idx = t + j * T;
        // the integral float plus 128 lies in 0..255 and goes straight into its byte; flipping
        // the top bit of each byte turns that offset form into two's complement
        const float q0 = fminf(fmaxf(rintf(v[j].x * scale), -128.f), 127.f) + 128.f;
        const float q1 = fminf(fmaxf(rintf(v[j].y * scale), -128.f), 127.f) + 128.f;
        const float q2 = fminf(fmaxf(rintf(v[j].z * scale), -128.f), 127.f) + 128.f;
        const float q3 = fminf(fmaxf(rintf(v[j].w * scale), -128.f), 127.f) + 128.f;
        uint32_t wd = __builtin_amdgcn_cvt_pk_u8_f32(q0, 0, 0u);
        wd = __builtin_amdgcn_cvt_pk_u8_f32(q1, 1, wd);
        wd = __builtin_amdgcn_cvt_pk_u8_f32(q2, 2, wd);
        wd = __builtin_amdgcn_cvt_pk_u8_f32(q3, 3, wd) ^ 0x80808080u;
        if (idx < K4) {
            rs = __builtin_amdgcn_sdot4((int)wd, 0x01010101, rs, false);  // sum of the four codes
            lds_codes[idx] = wd;
            if (blockIdx.x == 0 && blockIdx.y == 0 && a.codes_out)
                reinterpret_cast<uint32_t*>(a.codes_out)[idx] = wd;
        }
    }
    rs = wave_reduce(rs, OpSum{});
    if (lead) smi[wave] = rs;
    __syncthreads();  // also: the codes are in LDS
    rs = smi[0];
    for (int i = 1; i < W; ++i) rs += smi[i];
    if (t == 0 && blockIdx.x == 0 && blockIdx.y == 0) {
        if (a.gamma_out) a.gamma_out[0] = gamma;
        if (a.rowsum_out) a.rowsum_out[0] = rs;
    }
    return {gamma, rs};
}

// C = K-chunks per wave and round, T = weight tiles per workgroup (compile-time bound; `tpb`
// <= T of them are used), MAXT = launch bound.  ONE_ROUND: the waves of the group cover K in a
// single round, so a tile's partial sum goes straight to LDS and no per-tile registers are
// kept - this is what lets a wave keep eight 1 KiB weight loads in flight.
// FUSED (one round, M = 1): the codes come from quant_token, not from memory.  1: a wave keeps
// its slice of them in registers like codes read from memory; 2 (long K, many chunks per wave):
// every MFMA takes its operand from LDS.
// KGRP (one round, codes from memory): the a.kgroups K-groups of a grouped layer (Eq. 13-15) inside
// one workgroup.  a.K is one group's K; the waves are dealt to the groups (W / kgroups consecutive
// waves each, C chunks of the group's K per wave), every group reads its own columns of the codes
// and its own blob of tiles, and a tile's sums are added per group and written to the group's slice
// of split_ws (2 * sum_k q b, as a K split does), for splitk_reduce to dequantise group by group.
template <int C, int T, int MAXT, bool ONE_ROUND, int FUSED = 0, bool KGRP = false>
__global__ __launch_bounds__(MAXT) void gemm_decode_kernel(GemmArgs a, int tpb) {
    static_assert(!FUSED || ONE_ROUND, "the fused quantiser covers K in one round");
    static_assert(!KGRP || (ONE_ROUND && !FUSED), "K-groups inside the workgroup: one round, codes from memory");
    constexpr bool kActLds = FUSED == 2;
    constexpr int kRowBytes = FUSED == 2 ? 32768 : 16384;  // longest row the fused kernels take
    __shared__ __attribute__((aligned(16))) int red[(MAXT / kWave) * T * 256];  // [W][T][64][4]
    __shared__ __attribute__((aligned(16))) uint32_t row_codes[FUSED ? kRowBytes / 4 : 1];
    __shared__ double smd[FUSED ? 2 : 1][16];
    __shared__ float smf[FUSED ? 3 : 1][16];
    __shared__ int smi[16];
    const int W = blockDim.x / kWave;
    // the wave's index as a scalar: which chunks and tiles it owns is then scalar arithmetic and
    // the tile loads take a scalar base, instead of 64-bit compares and selects in every lane
    const int w = __builtin_amdgcn_readfirstlane((int)threadIdx.x / kWave), l = threadIdx.x % kWave;
    const int m = l & 15, g = l >> 4;
    const int64_t TKp = a.tk_pitch ? a.tk_pitch : tiles_k(a.K);  // tiles per tile row in memory
    const bool to_slices = a.split_k || a.kgroups > 1;  // partial sums go to split_ws
    // KGRP: waves per K-group, this wave's group and its index inside the group
    const int wpg = KGRP ? W / a.kgroups : W;
    const int gw = KGRP ? w / wpg : 0, wg = KGRP ? w % wpg : w;
    if constexpr (KGRP) {  // this wave's K-group (wave-uniform)
        a.codes += (int64_t)gw * a.K;
        a.packed += (int64_t)gw * a.group_packed;
    } else if (a.kgroups > 1) {  // this workgroup's K-group (uniform)
        a.codes += (int64_t)blockIdx.y * a.K;
        a.packed += (int64_t)blockIdx.y * a.group_packed;
    } else if (a.split_k) {  // this workgroup's slice of K (uniform)
        const int64_t k0 = (int64_t)blockIdx.y * a.split_k;
        a.codes += k0;
        a.packed += (k0 / kChunkK) * 256;
        a.K = a.K - k0 < a.split_k ? a.K - k0 : a.split_k;
    }
    const int64_t TN = tiles_n(a.N), TK = tiles_k(a.K);
    const int M = (int)a.M;
    const int64_t tn0 = (int64_t)blockIdx.x * tpb;

    // epilogue operands, requested up front so their latency hides under the weight stream.
    // beta belongs to the group of output rows that holds a tile (Eq. 13; one group: beta[0]).
    auto beta_of = [&](int64_t tn) {  // branch-free: nothing may delay the loads that follow
        if (tn > TN - 1) tn = TN - 1;
        return a.beta[((uint32_t)(tn * kTileN) / (uint32_t)a.beta_rows) * a.beta_stride];  // N <= 2^30
    };
    const float beta_first = beta_of(tn0 + w);
    const int mc = m < M ? m : M - 1;
    int rs = 0;
    float gm = 0.f, eta = 0.f;
    if constexpr (!FUSED && !KGRP) {
        rs = a.rowsum[mc * a.gstride];
        gm = a.per_tensor ? a.gamma[0] : a.gamma[mc * a.gstride];
        // Eq. 6 only; without it the load goes to gamma (always valid) and the value is not used
        eta = *(a.eta ? a.eta + (a.per_tensor ? 0 : mc * a.gstride) : a.gamma);
    }

    int part[ONE_ROUND ? 1 : T][4];
    if (!ONE_ROUND) {
#pragma unroll
        for (int t = 0; t < T; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) part[t][r] = 0;
    }

    const int64_t rounds = ONE_ROUND ? 1 : (TK + (int64_t)W * C - 1) / ((int64_t)W * C);
    for (int64_t rd = 0; rd < rounds; ++rd) {
        const int64_t tk0 = (rd * W + wg) * C;

        // Every load below is unconditional (addresses are clamped instead of guarded): with
        // no branches around them the loads complete in issue order and the MFMAs of tile t
        // wait for tile t only, not for the whole weight stream behind it.
        //
        // activation operand: lane (m, g) holds codes[m][512*tk + 64*i + 16*g .. +15].  Rows
        // m >= M read row M-1 (their outputs are never stored); columns k >= K read the last 16
        // valid bytes (the packed bits there are zero, so they contribute nothing).
        v4i act[kActLds ? 1 : C][8];
        auto load_act = [&](const int8_t* arow) {
            if constexpr (kActLds) return;
#pragma unroll
            for (int c = 0; c < C; ++c)
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    int k = (int)(tk0 + c) * kChunkK + 64 * i + 16 * g;  // K < 2^22
                    k = k > (int)a.K - 16 ? (int)a.K - 16 : k;
                    act[c][i] = *reinterpret_cast<const v4i*>(arow + k);
                }
        };
        // Few tokens: the wave's slice of the codes is M rows of C * 512 bytes, and fetching it in
        // operand layout costs C * 8 load instructions whatever M is (at one token as much time on
        // the load path as a seventh of the weight stream).  Instead each row is fetched with one
        // instruction, 16 consecutive bytes a lane, and (below, once the first weight tiles have
        // been requested behind it) parked in the wave's own part of `red`, which holds nothing
        // before the wave's first tile is done, and read from there in operand layout.
        // More tokens than the region has rows: the rows go through it in passes (the lanes of a
        // pass's rows read their operands, then the next rows are parked).  A row is 1 KiB, so the
        // same 16 bytes of every row would share their banks: the 16-byte slots of row r are stored
        // at slot ^ (r % 16).
        constexpr int kStageRows = T < 8 ? T : 8;
        constexpr int kStagePasses = (16 + kStageRows - 1) / kStageRows;
        const bool staged = !FUSED && ONE_ROUND && (M <= kStageRows || T >= 4);
        const bool stage_lane = l < C * 32;
        v4i rowv[16];
        if constexpr (!FUSED) {
            if (staged) {
                int kl = (int)tk0 * kChunkK + 16 * l;  // this lane's 16 bytes of a row slice
                kl = kl > (int)a.K - 16 ? (int)a.K - 16 : kl;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (r < M && stage_lane)
                        rowv[r] = *reinterpret_cast<const v4i*>(a.codes + (int64_t)r * a.ldq + kl);
            } else {
                load_act(a.codes + (int64_t)(m < M ? m : M - 1) * a.ldq);
            }
        }

        // Weight tiles: a software pipeline of depth kDepth per wave.  Asking for everything at
        // once looks attractive for a 4-microsecond stream, but the memory system then returns
        // the requests in no particular order, every wave gets its first tile late and all the
        // MFMA work piles up behind the stream.  With three tiles in flight per wave (~42 KiB per
        // CU, enough to cover the latency) tiles arrive in order and compute overlaps the stream.
        // Tiles past the end re-read the last tile (never stored); chunks past the end are
        // masked to zero arithmetically (no branch around a load).
        // FUSED: the waves spend the next microseconds on the token, not on MFMAs, so every tile
        // is requested now and the stream runs under the quantiser.
        constexpr int kDepth = FUSED ? T : T < 3 ? T : 3;
        v4i wt[T][C];
        // chunk c of this wave: valid index and all-ones / all-zeros mask
        int64_t tkc[C];
        int livem[C];
#pragma unroll
        for (int c = 0; c < C; ++c) {
            livem[c] = -(int)(tk0 + c < TK);
            tkc[c] = tk0 + c < TK ? tk0 + c : TK - 1;
        }
        // tile t of the group lies t*TK KiB after tile 0; tiles past the last valid one
        // (ragged N, or tpb < T) re-read the last valid tile
        const int t_last = (int)((tn0 + tpb - 1 < TN - 1 ? tn0 + tpb - 1 : TN - 1) - tn0);
        const uint32_t* wbase[C];
#pragma unroll
        for (int c = 0; c < C; ++c) wbase[c] = a.packed + (tn0 * TKp + tkc[c]) * 256 + l * 4;
        const uint32_t tile_stride = (uint32_t)TKp * 256;  // dwords; K < 2^22 keeps it in 32 bits
        auto load_tile = [&](int t) {
            const uint32_t off = (uint32_t)(t < t_last ? t : t_last) * tile_stride;
#pragma unroll
            for (int c = 0; c < C; ++c)  // read once: streaming loads leave L2 to the codes (3-6 %)
                wt[t][c] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(wbase[c] + off));
        };
        if constexpr (FUSED) {
            // the row is normalised and quantised while the tiles are on their way; every column
            // of the MFMA then holds the one token
            const TokenQuant tq = quant_token<kActLds ? 16 : 4>(a, row_codes, smd, smf, smi, [&]() {
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t = 0; t < kDepth; ++t) load_tile(t);
                __builtin_amdgcn_sched_barrier(0);
            });
            gm = tq.gamma;
            rs = tq.rowsum;
            load_act(reinterpret_cast<const int8_t*>(row_codes));
        } else {
#pragma unroll
            for (int t = 0; t < kDepth; ++t) load_tile(t);
            if (staged) {  // rows past M repeat row M-1 (never stored)
                int* stage = &red[w * T * 256];
                const int mr = m < M ? m : M - 1;
#pragma unroll
                for (int p = 0; p < kStagePasses; ++p) {
                    if (p * kStageRows < M) {  // uniform
#pragma unroll
                        for (int r = 0; r < kStageRows; ++r)
                            if (p * kStageRows + r < 16 && p * kStageRows + r < M && stage_lane)
                                *reinterpret_cast<v4i*>(&stage[r * 256 + (l ^ (r & 15)) * 4]) =
                                    rowv[p * kStageRows + r < 16 ? p * kStageRows + r : 15];
                        if (mr / kStageRows == p) {
                            const int rr = mr - p * kStageRows;
#pragma unroll
                            for (int c = 0; c < C; ++c)
#pragma unroll
                                for (int i = 0; i < 8; ++i)
                                    act[c][i] = *reinterpret_cast<const v4i*>(
                                        &stage[rr * 256 + ((c * 32 + 4 * i + g) ^ (rr & 15)) * 4]);
                        }
                    }
                }
            }
        }

#pragma unroll
        for (int t = 0; t < T; ++t) {
            if (t + kDepth < T) load_tile(t + kDepth);
            __builtin_amdgcn_sched_barrier(0);  // keep the request ahead of this tile's MFMAs
            v4i acc[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = (v4i){0, 0, 0, 0};
            // chunks past the end of K are masked here, at the point of use (masking at the load
            // would tie a wait for the whole stream to the first tile), and inside the plane mask,
            // a scalar: it costs no instruction of its own
            // kActLds: an offset of zero the compiler cannot see through, so that each tile reads
            // its operands again instead of all C * 8 of them being kept in registers
            int again = 0;
            if constexpr (kActLds) asm volatile("" : "+v"(again));
#pragma unroll
            for (int c = 0; c < C; ++c)
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int mask = (int)(0x01010101u << i) & livem[c];
                    const v4i plane = wt[t][c] & mask;
                    v4i cols;
                    if constexpr (kActLds) {
                        int k = (int)(tk0 + c) * kChunkK + 64 * i + 16 * g;
                        if (k > (int)a.K - 16) k = (int)a.K - 16;
                        cols = *reinterpret_cast<const v4i*>(reinterpret_cast<const int8_t*>(row_codes) + k + again);
                    } else {
                        cols = act[c][i];
                    }
                    // rows of the MFMA = weights (n), columns = tokens (m)
                    acc[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(plane, cols, acc[i], 0, 0, 0);
                }
            // fold the planes, scaled by 128 so that one shift-add per plane does it:
            //   128 * sum_k q b = sum_{i<7} acc_i * 2^(7-i) - acc_7      (|.| < 2^24 per chunk)
            v4i sum;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                int h = acc[0][r];
#pragma unroll
                for (int i = 1; i < 7; ++i) h = (h << 1) + acc[i][r];
                sum[r] = (h << 1) - acc[7][r];
            }
            if (ONE_ROUND) {
                *reinterpret_cast<v4i*>(&red[((w * T + t) * kWave + l) * 4]) = sum;
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) part[t][r] += sum[r];
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // cross-wave reduction over K, then the dequantisation epilogue
    if (!ONE_ROUND) {
#pragma unroll
        for (int t = 0; t < T; ++t)
            *reinterpret_cast<v4i*>(&red[((w * T + t) * kWave + l) * 4]) =
                (v4i){part[t][0], part[t][1], part[t][2], part[t][3]};
    }
    __syncthreads();
    if constexpr (KGRP) {
        // (tile, group) pairs are dealt to the waves; a pair's sum runs over the group's waves
        for (int item = w; item < tpb * a.kgroups; item += W) {
            const int t = item % tpb, grp = item / tpb;
            v4i sum = (v4i){0, 0, 0, 0};
            for (int ww = grp * wpg; ww < (grp + 1) * wpg; ++ww)
                sum += *reinterpret_cast<const v4i*>(&red[((ww * T + t) * kWave + l) * 4]);
            const int64_t tn = tn0 + t;
            const int64_t n = tn * kTileN + 4 * g;
            if (tn >= TN || m >= M || n >= a.N) continue;
            int* p = a.split_ws + ((int64_t)grp * M + m) * a.N + n;
            const v4i h = sum >> 6;
            if ((a.N & 3) == 0) *reinterpret_cast<v4i*>(p) = h;
            else
                for (int r = 0; r < 4; ++r)
                    if (n + r < a.N) p[r] = h[r];
        }
        return;
    }
    for (int t = w; t < tpb; t += W) {
        v4i sum = (v4i){0, 0, 0, 0};
        for (int ww = 0; ww < W; ++ww)
            sum += *reinterpret_cast<const v4i*>(&red[((ww * T + t) * kWave + l) * 4]);
        const int64_t tn = tn0 + t;
        const int64_t n = tn * kTileN + 4 * g;
        if (tn >= TN || m >= M || n >= a.N) continue;
        if (to_slices) {  // partial sum of this K-slice: 2 * sum_k q b, folded by splitk_reduce
            int* p = a.split_ws + ((int64_t)blockIdx.y * M + m) * a.N + n;
            const v4i h = sum >> 6;
            if ((a.N & 3) == 0) *reinterpret_cast<v4i*>(p) = h;
            else
                for (int r = 0; r < 4; ++r)
                    if (n + r < a.N) p[r] = h[r];
            continue;
        }
        const v4i pm = (sum >> 6) - rs;  // sum_k q s = 2 * (sum / 128) - sum_k q, exact shift
        float* y = a.Y + (int64_t)m * a.N + n;
        if (a.out_acc) {
            int* yi = reinterpret_cast<int*>(y);
            if ((a.N & 3) == 0) *reinterpret_cast<v4i*>(yi) = pm;
            else
                for (int r = 0; r < 4; ++r)
                    if (n + r < a.N) yi[r] = pm[r];
        } else {
            const float beta = t == w ? beta_first : beta_of(tn);
            const float sc = (beta * gm) / 128.0f;
            v4f o = {(float)pm[0] * sc, (float)pm[1] * sc, (float)pm[2] * sc, (float)pm[3] * sc};
            if (a.eta) {  // Eq. 6: the shift eta of the activations adds (beta * eta) * sum_k s[n,k]
                const float be = beta * eta;
                for (int r = 0; r < 4; ++r)
                    o[r] = o[r] + be * (float)a.wsum[n + r < a.N ? n + r : a.N - 1];
            }
            if ((a.N & 3) == 0) {
                if (a.accumulate) o += *reinterpret_cast<const v4f*>(y);  // a later K-group
                *reinterpret_cast<v4f*>(y) = o;
            } else {
                for (int r = 0; r < 4; ++r)
                    if (n + r < a.N) y[r] = a.accumulate ? y[r] + o[r] : o[r];
            }
        }
    }
}

// Fold of a grouped layer's slices (Eq. 13-15), four consecutive columns per thread (N % 4 == 0):
// each K-group's sums are dequantised with its own beta_g gamma_g / 128 (and shifted by its own
// eta_g, Eq. 14) and the groups are added in the order 0, 1, ...
__global__ __launch_bounds__(256) void groups_reduce4(GemmArgs a) {
    const int64_t N4 = a.N >> 2;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= a.M * N4) return;
    const int64_t m = idx / N4, n = (idx % N4) * 4;
    const int G = a.kgroups;
    uint32_t bg[4];
#pragma unroll
    for (int c = 0; c < 4; ++c)
        bg[c] = ((uint32_t)(n + c) / (uint32_t)a.beta_rows) * (uint32_t)a.beta_stride;
    v4f y = {0.f, 0.f, 0.f, 0.f};
    for (int g = 0; g < G; ++g) {
        const v4i part = *reinterpret_cast<const v4i*>(a.split_ws + ((int64_t)g * a.M + m) * a.N + n);
        const int rs = a.rowsum[m * a.gstride + g];
        const float gm = a.gamma[a.per_tensor ? g : m * a.gstride + g];
        const float eta = a.eta ? a.eta[a.per_tensor ? g : m * a.gstride + g] : 0.f;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float beta = a.beta[bg[c] + g];
            float yg = (float)(part[c] - rs) * ((beta * gm) / 128.0f);
            if (a.eta) yg = yg + (beta * eta) * (float)a.wsum[(int64_t)g * a.N + n + c];
            y[c] = g ? yg + y[c] : yg;
        }
    }
    *reinterpret_cast<v4f*>(a.Y + m * a.N + n) = y;
}

// Second step of a K split: Y[m,n] = epilogue(sum_s partial[s][m][n] - rowsum[m]).
__global__ __launch_bounds__(256) void splitk_reduce(GemmArgs a, int splits) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= a.M * a.N) return;
    const int64_t m = idx / a.N, n = idx % a.N;
    if (a.kgroups > 1) {
        // slices are K-groups (Eq. 13-15): each is dequantised with its own beta_g gamma_g / 128
        // (and shifted by its own eta_g, Eq. 14); the groups are added in the order 0, 1, ...
        const int G = a.kgroups;
        const uint32_t bg = ((uint32_t)n / (uint32_t)a.beta_rows) * (uint32_t)a.beta_stride;
        float y = 0.f;
        for (int g = 0; g < G; ++g) {
            const int pm = a.split_ws[((int64_t)g * a.M + m) * a.N + n] - a.rowsum[m * a.gstride + g];
            const float beta = a.beta[bg + g];
            const float gm = a.gamma[a.per_tensor ? g : m * a.gstride + g];
            float yg = (float)pm * ((beta * gm) / 128.0f);
            if (a.eta)
                yg = yg + (beta * a.eta[a.per_tensor ? g : m * a.gstride + g]) *
                              (float)a.wsum[(int64_t)g * a.N + n];
            y = g ? yg + y : yg;
        }
        a.Y[idx] = y;
        return;
    }
    int sum = 0;
    for (int sp = 0; sp < splits; ++sp) sum += a.split_ws[((int64_t)sp * a.M + m) * a.N + n];
    const int pm = sum - a.rowsum[m * a.gstride];
    if (a.out_acc) {
        reinterpret_cast<int*>(a.Y)[idx] = pm;
        return;
    }
    const float beta = a.beta[((uint32_t)n / (uint32_t)a.beta_rows) * a.beta_stride];
    const float gm = a.per_tensor ? a.gamma[0] : a.gamma[m * a.gstride];
    float y = (float)pm * ((beta * gm) / 128.0f);
    if (a.eta) y = y + (beta * a.eta[a.per_tensor ? 0 : m * a.gstride]) * (float)a.wsum[n];
    if (a.accumulate) y += a.Y[idx];
    a.Y[idx] = y;
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

template <int C, int T, int MAXT, bool ONE_ROUND, int FUSED = 0, bool KGRP = false>
static void launch_one(const GemmArgs& a, int W, int tpb, hipStream_t s) {
    const int64_t TN = tiles_n(a.N);
    const unsigned splits = KGRP ? 1u : a.kgroups > 1 ? (unsigned)a.kgroups
                            : a.split_k ? (unsigned)((a.K + a.split_k - 1) / a.split_k) : 1u;
    const dim3 grid((unsigned)((TN + tpb - 1) / tpb), splits);
    gemm_decode_kernel<C, T, MAXT, ONE_ROUND, FUSED, KGRP><<<grid, W * kWave, 0, s>>>(a, tpb);
}

// one round, up to 8 waves, exactly tpb = 1..8 tiles per group
template <int C, int FUSED, bool KGRP = false>
static void launch_tiles(const GemmArgs& a, int W, int tpb, hipStream_t s) {
    switch (tpb) {
        case 1: launch_one<C, 1, 512, true, FUSED, KGRP>(a, W, 1, s); break;
        case 2: launch_one<C, 2, 512, true, FUSED, KGRP>(a, W, 2, s); break;
        case 3: launch_one<C, 3, 512, true, FUSED, KGRP>(a, W, 3, s); break;
        case 4: launch_one<C, 4, 512, true, FUSED, KGRP>(a, W, 4, s); break;
        case 5: launch_one<C, 5, 512, true, FUSED, KGRP>(a, W, 5, s); break;
        case 6: launch_one<C, 6, 512, true, FUSED, KGRP>(a, W, 6, s); break;
        case 7: launch_one<C, 7, 512, true, FUSED, KGRP>(a, W, 7, s); break;
        default: launch_one<C, 8, 512, true, FUSED, KGRP>(a, W, 8, s); break;
    }
}

// One token and a K that one round of waves covers: the small-batch kernel can quantise the row
// itself.  Up to 32 chunks a wave holds one or two of them as register operands; up to 64 it
// walks eight, with the operands read from LDS.  Every workgroup repeats the quantiser, so it
// pays only while one round of workgroups covers N (8, 2 or 3 tiles a group at most, as the
// launcher below chooses): K = N = 28672 measured 58 us fused against 44 us in two launches.
bool gemm_decode_fuses_quant(int64_t M, int64_t K, int64_t N) {
    const int64_t TK = tiles_k(K);
    if (M != 1 || TK > 64 || tuning().decode_nofuse) return false;
    const int64_t cap = TK <= 16 ? 8 : TK <= 32 ? 2 : 3;
    return tiles_n(N) <= cap * num_cus();
}

// K > 16384 with a workspace: split K over workgroups so that every slice takes the one-round
// path with two chunks per wave (at most 16 chunks a slice), and fold the slices afterwards.
size_t gemm_split_ws_bytes(int64_t M, int64_t N, int64_t K) {
    const int64_t TK = tiles_k(K);
    int64_t splits = 0;
    if (M <= 16) {
        if (TK > 32) splits = (TK + 15) / 16;
    } else {  // enough for whichever of the two mid-batch kernels takes the shape
        if (const int64_t per = prefill_split_tiles(M, N, K)) splits = (TK + per - 1) / per;
        if (const int64_t per = stream_split_tiles(M, K)) {
            const int64_t s2 = (TK + per - 1) / per;
            splits = s2 > splits ? s2 : splits;
        }
    }
    return (size_t)splits * (size_t)M * (size_t)N * 4;
}

// Measurement aid: reads `bytes` of device memory the way the small-batch kernel streams its
// weight tiles (16-byte nontemporal loads, a wave takes 1 KiB at a time, the workgroups share the
// range evenly, kDepth loads in flight per lane) and does nothing else.  What such a launch takes
// is the floor for any kernel that has to bring the same bytes in from HBM.
__global__ __launch_bounds__(1024) void read_probe_kernel(const v4i* __restrict__ src, int64_t n16,
                                                          uint32_t* sink) {
    constexpr int kDepth = 4;
    const int64_t per = (n16 + gridDim.x - 1) / gridDim.x;  // 16-byte pieces per workgroup
    const int64_t lo = per * blockIdx.x, hi = lo + per < n16 ? lo + per : n16;
    v4i x = {0, 0, 0, 0};
    for (int64_t i = lo + threadIdx.x; i < hi; i += (int64_t)blockDim.x * kDepth) {
        v4i v[kDepth];
#pragma unroll
        for (int d = 0; d < kDepth; ++d) {
            const int64_t j = i + (int64_t)d * blockDim.x;
            v[d] = __builtin_nontemporal_load(src + (j < hi ? j : hi - 1));
        }
#pragma unroll
        for (int d = 0; d < kDepth; ++d) x ^= v[d];
    }
    // never true for the all-ones pattern no weight blob holds in every lane; keeps the loads alive
    if ((x[0] & x[1] & x[2] & x[3]) == -1 && sink) sink[blockIdx.x] = 1u;
}
hipError_t launch_read_probe(const void* src, size_t bytes, int workgroups, int threads,
                             uint32_t* sink, hipStream_t s) {
    read_probe_kernel<<<(unsigned)workgroups, (unsigned)threads, 0, s>>>(
        reinterpret_cast<const v4i*>(src), (int64_t)(bytes / 16), sink);
    return hipGetLastError();
}

void launch_splitk_reduce(const GemmArgs& a, int splits, hipStream_t s) {
    if (a.kgroups > 1 && (a.N & 3) == 0 && ((uintptr_t)a.Y & 15) == 0) {
        groups_reduce4<<<(unsigned)((a.M * (a.N >> 2) + 255) / 256), 256, 0, s>>>(a);
        return;
    }
    splitk_reduce<<<(unsigned)((a.M * a.N + 255) / 256), 256, 0, s>>>(a, splits);
}

hipError_t launch_gemm_decode(const GemmArgs& a_in, hipStream_t s) {
    GemmArgs a = a_in;
    const int64_t TN = tiles_n(a.N);
    int64_t TK = tiles_k(a.K);
    int splits = 1;
    const bool fused = a.x_row != nullptr;  // the caller asked gemm_decode_fuses_quant
    const size_t need = gemm_split_ws_bytes(a.M, a.N, a.K);
    if (a.kgroups > 1) {  // one slice per K-group; the caller sized split_ws for it
        if (fused || !a.split_ws || a.split_ws_bytes < (size_t)a.kgroups * a.M * a.N * 4)
            return hipErrorInvalidValue;
        a.split_k = 0;
        // All groups inside a workgroup when their chunks fit the waves of one (up to 8 waves of
        // one or two chunks, or 16 waves with at most two tiles a group); a wave's chunks must
        // lie in one group.  One round of workgroups then covers N as in the plain layer.
        const int64_t V = TK * a.kgroups;  // chunks of all groups
        auto tiles_for = [&](int cap) {
            int tpb = (int)((TN + num_cus() - 1) / num_cus());
            tpb = tpb > cap ? cap : tpb < 1 ? 1 : tpb;
            const int t = tuning().decode_tiles;
            return t >= 1 && t <= cap ? t : tpb;
        };
        bool done = true;
        if (tuning().group_slices) done = false;  // (tests: the K-groups as slices of the grid)
        else if (TK % 2 == 0 && V / 2 <= 8) launch_tiles<2, 0, true>(a, (int)(V / 2), tiles_for(8), s);
        else if (V <= 8) launch_tiles<1, 0, true>(a, (int)V, tiles_for(8), s);
        else if (TK % 2 == 0 && V / 2 <= 16) {
            if (tiles_for(2) <= 1) launch_one<2, 1, 1024, true, 0, true>(a, (int)(V / 2), 1, s);
            else launch_one<2, 2, 1024, true, 0, true>(a, (int)(V / 2), 2, s);
        } else if (V <= 16) {
            if (tiles_for(2) <= 1) launch_one<1, 1, 1024, true, 0, true>(a, (int)V, 1, s);
            else launch_one<1, 2, 1024, true, 0, true>(a, (int)V, 2, s);
        } else {
            done = false;
        }
        if (done) {
            launch_splitk_reduce(a, a.kgroups, s);
            return hipGetLastError();
        }
        splits = a.kgroups;  // else: the K-groups as slices of the grid
    } else if (need && !fused && a.split_ws && a.split_ws_bytes >= need && !tuning().decode_nosplit) {
        splits = (int)((TK + 15) / 16);
        const int64_t per = (TK + splits - 1) / splits;  // tiles per slice, evenly
        splits = (int)((TK + per - 1) / per);            // slices that actually hold tiles
        a.tk_pitch = a.tk_pitch ? a.tk_pitch : TK;
        a.split_k = per * kChunkK;
        TK = per;
    } else {
        a.split_k = 0;
    }
    // The whole matrix is a few microseconds of HBM time, so the kernel is built to have every
    // byte requested at once: one round of workgroups (about one per CU), each wave asking for
    // all of its weight tiles before the first MFMA.
    auto tiles_per_group = [&](int cap) {
        int tpb = (int)((TN * splits + num_cus() - 1) / num_cus());
        tpb = tpb > cap ? cap : tpb < 1 ? 1 : tpb;
        const int t = tuning().decode_tiles;
        return t >= 1 && t <= cap ? t : tpb;
    };
    if (TK < 8) {
        // K < 4096: one K-chunk per wave, W = TK waves cover K in one round
        const int W = (int)TK;
        const int tpb = tiles_per_group(8);
        if (fused) launch_tiles<1, 1>(a, W, tpb, s);
        else launch_tiles<1, 0>(a, W, tpb, s);
    } else if (TK <= 16) {
        // 4096 <= K <= 8192: two chunks per wave (the fold of the bit planes, once per tile and
        // wave, is then shared by two chunks), W = ceil(TK/2) <= 8 waves, one round
        const int W = (int)((TK + 1) / 2);
        const int tpb = tiles_per_group(8);
        if (fused) launch_tiles<2, 1>(a, W, tpb, s);
        else launch_tiles<2, 0>(a, W, tpb, s);
    } else if (TK <= 32) {
        // K <= 16384: up to 16 waves of two chunks, one round; 128 registers per lane
        const int W = (int)((TK + 1) / 2);
        const int tpb = tiles_per_group(2);
        if (fused) {
            if (tpb <= 1) launch_one<2, 1, 1024, true, 1>(a, W, 1, s);
            else launch_one<2, 2, 1024, true, 1>(a, W, 2, s);
        } else if (tpb <= 1) {
            launch_one<2, 1, 1024, true>(a, W, 1, s);
        } else {
            launch_one<2, 2, 1024, true>(a, W, 2, s);
        }
    } else if (fused) {
        // one token, K <= 32768: eight chunks per wave (the last ones masked), up to 8 waves, one
        // round, up to three tiles per group in registers (96 of them)
        const int W = (int)((TK + 7) / 8);
        switch (tiles_per_group(3)) {
            case 1: launch_one<8, 1, 512, true, 2>(a, W, 1, s); break;
            case 2: launch_one<8, 2, 512, true, 2>(a, W, 2, s); break;
            default: launch_one<8, 3, 512, true, 2>(a, W, 3, s); break;
        }
    } else {
        // longer K: two chunks per wave and round, up to 16 waves, several rounds
        const int64_t slots = (TK + 1) / 2;
        const int64_t rounds = (slots + 15) / 16;
        const int W = (int)((slots + rounds - 1) / rounds);
        launch_one<2, 1, 1024, false>(a, W, 1, s);
    }
    if (splits > 1) launch_splitk_reduce(a, splits, s);
    return hipGetLastError();
}

}  // namespace bl

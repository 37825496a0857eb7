// Fused LayerNorm + absmax + round/clip activation quantiser
// (arXiv 2310.11453, Eq. 12 for LN, Eq. 4-5 for the 8-bit absmax quantiser).
//
// One workgroup owns one token.  The row is read from HBM once and stays in
// registers through the three reductions (mean, variance, max) and the
// rounding pass, so the kernel moves 4 bytes in and 1 byte out per element.
// Mean, variance and the normalisation itself are evaluated in fp64 (the
// kernel is bandwidth-bound, the extra ALU work is free) so that the fp32
// value handed to the rounding step is the correctly rounded normalised
// input; the steps that decide a code are single fp32 operations:
//   scale = 128 / gamma,  t = x^ * scale,  code = clamp(rne(t), -128, 127).
#include "common.h"
#include "kernels.h"

namespace bl {

enum QuantMode { kFull = 0, kStats = 1, kApply = 2 };

// kFull : per-token gamma, everything in one pass.
// kStats: per-tensor, pass 1: row mean/rstd to rowstats, running max to gmax_bits.
// kApply: per-tensor, pass 2: re-read the row, normalise with the saved stats,
//         quantise with the tensor-wide gamma.
template <int THREADS, int NV, int MODE>
__global__ __launch_bounds__(THREADS) void ln_quant_rows(QuantArgs a) {
    constexpr int NW = THREADS / kWave;
    __shared__ double smd[NW > 1 ? NW : 1];
    __shared__ float smf[NW > 1 ? NW : 1];
    __shared__ int smi[NW > 1 ? NW : 1];

    const int64_t row = blockIdx.x;
    const int K4 = (int)(a.K / 4);
    const float4* __restrict__ x4 = reinterpret_cast<const float4*>(a.X + row * a.K);

    float4 v[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int idx = threadIdx.x + j * THREADS;
        v[j] = idx < K4 ? x4[idx] : make_float4(0.f, 0.f, 0.f, 0.f);
    }

    if (!a.skip_ln) {
        double mu, rstd;
        if constexpr (MODE == kApply) {
            mu = a.rowstats[2 * row];
            rstd = a.rowstats[2 * row + 1];
        } else {
            double s = 0.0;
#pragma unroll
            for (int j = 0; j < NV; ++j)
                s += ((double)v[j].x + (double)v[j].y) + ((double)v[j].z + (double)v[j].w);
            mu = block_sum<NW>(s, smd) / (double)a.K;
            double q = 0.0;
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                if (threadIdx.x + j * THREADS < K4) {
                    const double dx = (double)v[j].x - mu, dy = (double)v[j].y - mu;
                    const double dz = (double)v[j].z - mu, dw = (double)v[j].w - mu;
                    q += (dx * dx + dy * dy) + (dz * dz + dw * dw);
                }
            }
            const double var = block_sum<NW>(q, smd) / (double)a.K;
            rstd = 1.0 / sqrt(var + (double)a.eps);
            if constexpr (MODE == kStats) {
                if (threadIdx.x == 0) {
                    a.rowstats[2 * row] = mu;
                    a.rowstats[2 * row + 1] = rstd;
                }
            }
        }
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int idx = threadIdx.x + j * THREADS;
            float4 o;
            o.x = (float)(((double)v[j].x - mu) * rstd);
            o.y = (float)(((double)v[j].y - mu) * rstd);
            o.z = (float)(((double)v[j].z - mu) * rstd);
            o.w = (float)(((double)v[j].w - mu) * rstd);
            if (idx < K4) {
                if (a.gain) {
                    const float4 g = reinterpret_cast<const float4*>(a.gain)[idx];
                    o.x = o.x * g.x; o.y = o.y * g.y; o.z = o.z * g.z; o.w = o.w * g.w;
                }
                if (a.bias) {
                    const float4 b = reinterpret_cast<const float4*>(a.bias)[idx];
                    o.x = o.x + b.x; o.y = o.y + b.y; o.z = o.z + b.z; o.w = o.w + b.w;
                }
                v[j] = o;
            }
        }
    }

    if constexpr (MODE != kStats) {
        if (a.xhat_dump) {
            float4* __restrict__ d4 = reinterpret_cast<float4*>(a.xhat_dump + row * a.K);
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                const int idx = threadIdx.x + j * THREADS;
                if (idx < K4) d4[idx] = v[j];
            }
        }
    }

    float gamma;
    if constexpr (MODE == kApply) {
        gamma = fmaxf(__uint_as_float(*a.gmax_bits), 1e-5f);
    } else {
        float amax = 0.f;
#pragma unroll
        for (int j = 0; j < NV; ++j) {  // padding lanes hold 0 and cannot raise the max
            amax = fmaxf(amax, fmaxf(fmaxf(fabsf(v[j].x), fabsf(v[j].y)),
                                     fmaxf(fabsf(v[j].z), fabsf(v[j].w))));
        }
        amax = block_max<NW>(amax, smf);
        if constexpr (MODE == kStats) {
            // non-negative floats order like their bit patterns: integer max is exact
            if (threadIdx.x == 0) atomicMax(a.gmax_bits, __float_as_uint(amax));
            return;
        }
        gamma = fmaxf(amax, 1e-5f);
    }

    const float scale = 128.0f / gamma;
    int rs = 0;
    uint32_t* __restrict__ c4 = reinterpret_cast<uint32_t*>(a.codes + row * a.K);
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int idx = threadIdx.x + j * THREADS;
        const int q0 = (int)fminf(fmaxf(rintf(v[j].x * scale), -128.f), 127.f);
        const int q1 = (int)fminf(fmaxf(rintf(v[j].y * scale), -128.f), 127.f);
        const int q2 = (int)fminf(fmaxf(rintf(v[j].z * scale), -128.f), 127.f);
        const int q3 = (int)fminf(fmaxf(rintf(v[j].w * scale), -128.f), 127.f);
        if (idx < K4) {
            rs += (q0 + q1) + (q2 + q3);
            c4[idx] = (uint32_t)(q0 & 0xff) | ((uint32_t)(q1 & 0xff) << 8) |
                      ((uint32_t)(q2 & 0xff) << 16) | ((uint32_t)(q3 & 0xff) << 24);
        }
    }
    if (a.rowsum) {
        rs = block_sum<NW>(rs, smi);
        if (threadIdx.x == 0) a.rowsum[row] = rs;
    }
    if (threadIdx.x == 0) {
        if (MODE == kFull) a.gamma[row] = gamma;
        else if (row == 0) a.gamma[0] = gamma;
    }
}

__global__ void fill_u32(uint32_t* p, uint32_t v) { *p = v; }

// rows of up to 32768 elements stay in registers (8 float4 per lane, up to 1024 lanes)
bool quant_supported(int64_t K) { return K % 4 == 0 && K / 4 <= 1024 * 8; }

template <int THREADS, int NV>
static void launch_mode(const QuantArgs& a, hipStream_t s) {
    const unsigned grid = (unsigned)a.M;
    if (!a.per_tensor) {
        ln_quant_rows<THREADS, NV, kFull><<<grid, THREADS, 0, s>>>(a);
    } else {
        fill_u32<<<1, 1, 0, s>>>(a.gmax_bits, 0u);
        ln_quant_rows<THREADS, NV, kStats><<<grid, THREADS, 0, s>>>(a);
        ln_quant_rows<THREADS, NV, kApply><<<grid, THREADS, 0, s>>>(a);
    }
}

hipError_t launch_quant(const QuantArgs& a, hipStream_t s) {
    const int64_t K4 = a.K / 4;
    if (K4 <= 64) launch_mode<64, 1>(a, s);
    else if (K4 <= 128) launch_mode<64, 2>(a, s);
    else if (K4 <= 256) launch_mode<64, 4>(a, s);
    else if (K4 <= 512) launch_mode<256, 2>(a, s);
    else if (K4 <= 1024) launch_mode<256, 4>(a, s);
    else if (K4 <= 2048) launch_mode<256, 8>(a, s);
    else if (K4 <= 4096) launch_mode<512, 8>(a, s);
    else launch_mode<1024, 8>(a, s);
    return hipGetLastError();
}

}  // namespace bl

// Fused LayerNorm + absmax + round/clip activation quantiser
// (arXiv 2310.11453, Eq. 12 for LN, Eq. 4-5 for the 8-bit absmax quantiser).
//
// One to eight waves own one token.  The row is read from HBM once and stays in
// registers through the reductions (sum with min/max, then variance) and the
// rounding pass, so the kernel moves 4 bytes in and 1 byte out per element.
// Mean, variance and the normalisation itself are evaluated in fp64 (the
// kernel is bandwidth-bound, the extra ALU work is free) so that the fp32
// value handed to the rounding step is the correctly rounded normalised
// input; the steps that decide a code are single fp32 operations:
//   scale = 128 / gamma,  t = x^ * scale,  code = clamp(rne(t), -128, 127).
#include "common.h"
#include "kernels.h"
#include "rowops.h"

namespace bl {

enum QuantMode { kFull = 0, kStats = 1, kApply = 2 };

// Order-preserving map of floats (any sign) onto unsigned integers and back, so that a running
// minimum / maximum over the whole tensor can be an integer atomic: exact and order-free.
__device__ inline uint32_t float_key(float v) {
    const uint32_t b = __float_as_uint(v);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ inline float key_float(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}
// Eq. 6 per tensor: the row's extremes join the running minimum (gmin_bits) and maximum
// (gmax_bits) of its K-group; a look first spares the atomic when there is nothing to add.
__device__ inline void offer_extremes(const QuantArgs& a, int g, float lo, float hi) {
    const uint32_t kl = float_key(lo), kh = float_key(hi);
    if (kl < __hip_atomic_load(a.gmin_bits + g, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
        atomicMin(a.gmin_bits + g, kl);
    if (kh > __hip_atomic_load(a.gmax_bits + g, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
        atomicMax(a.gmax_bits + g, kh);
}

// WPR waves share one token (row); a lane holds NV float4 of it.  Workgroups have at least
// four waves, so short rows are handled four (or two) to a workgroup, one per wave, with no
// barrier at all.
// kFull : per-token gamma, everything in one pass.
// kStats: per-tensor, pass 1: row mean/rstd to rowstats, running max to gmax_bits.
// kApply: per-tensor, pass 2: re-read the row, normalise with the saved stats,
//         quantise with the tensor-wide gamma.
template <int WPR, int NV, int MODE>
__global__ __launch_bounds__((WPR < 4 ? 4 : WPR) * kWave, 4) void ln_quant_rows(QuantArgs a) {
    constexpr int NW = WPR < 4 ? 4 : WPR;  // waves per workgroup
    constexpr int RPW = NW / WPR;          // rows per workgroup
    constexpr int RT = WPR * kWave;        // lanes per row
    __shared__ double smd[2][NW];
    __shared__ float smf[4][NW];
    __shared__ int smi[NW];

    const int wave = threadIdx.x / kWave;
    const int rw = wave / WPR, wr = wave % WPR;
    const int t = wr * kWave + (threadIdx.x & (kWave - 1));
    int64_t row = (int64_t)blockIdx.x * RPW + rw;
    const bool live = row < a.M;
    if constexpr (WPR == 1 && MODE != kStats) {
        if (!live) return;  // no barriers on this path
    } else {
        if (!live) row = a.M - 1;
    }
    const int K4 = (int)(a.K / 4);
    const float4* __restrict__ x4 = reinterpret_cast<const float4*>(a.X + row * a.K);
    const int grp = a.groups > 1 ? (int)(row % a.groups) : 0;  // K-group of this row (Eq. 14-15)

    // The loads are unconditional (clamped index, value masked afterwards) so that all of
    // them are in flight before the first is needed.
    float4 v[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int idx = t + j * RT;
        v[j] = x4[idx < K4 ? idx : K4 - 1];
    }
    // Each pass over the row converts its elements to fp64 again: `forget` hides the values
    // from the optimiser between passes, or it would keep all the converted copies alive
    // (two registers per element) and the kernel would run at minimal occupancy.
    auto forget = [&]() {
#pragma unroll
        for (int j = 0; j < NV; ++j)
            asm volatile("" : "+v"(v[j].x), "+v"(v[j].y), "+v"(v[j].z), "+v"(v[j].w));
    };
    const bool affine = a.gain != nullptr || a.bias != nullptr;
    bool have_amax = false;
    float amax = 0.f;
    float lo = 0.f, hi_row = 0.f;  // Eq. 6 only: the row's minimum (eta) and maximum; amax = max - min

    if (!a.skip_ln) {
        double mu, rstd;
        if constexpr (MODE == kApply) {
            mu = a.rowstats[2 * row];
            rstd = a.rowstats[2 * row + 1];
        } else {
            // One pass for the mean and the variance: sums of x and of (x - c)^2 in fp64, with
            // c an element of the row, so that var = E[(x-c)^2] - (mu-c)^2 loses no digits to
            // a large common offset.  Minimum and maximum ride along for the absmax.
            const double c = (double)a.X[row * a.K];
            double s = 0.0, q = 0.0;
            float mn = v[0].x, mx = v[0].x;  // always an element of the row (clamped index)
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                if (t + j * RT < K4) {
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
            // one barrier for the four values
            s = wave_reduce(s, OpSum{});
            q = wave_reduce(q, OpSum{});
            mn = wave_reduce(mn, OpMin{});
            mx = wave_reduce(mx, OpMax{});
            if constexpr (WPR > 1) {
                if ((threadIdx.x & (kWave - 1)) == 0) {
                    smd[0][wave] = s;
                    smd[1][wave] = q;
                    smf[0][wave] = mn;
                    smf[1][wave] = mx;
                }
                __syncthreads();
                s = smd[0][rw * WPR];
                q = smd[1][rw * WPR];
                mn = smf[0][rw * WPR];
                mx = smf[1][rw * WPR];
#pragma unroll
                for (int i = 1; i < WPR; ++i) {
                    s += smd[0][rw * WPR + i];
                    q += smd[1][rw * WPR + i];
                    mn = fminf(mn, smf[0][rw * WPR + i]);
                    mx = fmaxf(mx, smf[1][rw * WPR + i]);
                }
            }
            mu = s / (double)a.K;
            const double qs = q;
            const double var = fmax(qs / (double)a.K - (mu - c) * (mu - c), 0.0);
            rstd = 1.0 / sqrt(var + (double)a.eps);
            if constexpr (MODE == kStats) {
                if (t == 0 && live) {
                    a.rowstats[2 * row] = mu;
                    a.rowstats[2 * row + 1] = rstd;
                }
            }
            if (!affine) {
                // x -> fl32((x - mu) * rstd) is monotone, so the largest magnitude of the
                // normalised row is reached at the row's minimum or maximum.
                lo = (float)(((double)mn - mu) * rstd);
                const float hi = (float)(((double)mx - mu) * rstd);
                hi_row = hi;
                amax = a.nonneg ? hi - lo : fmaxf(fabsf(lo), fabsf(hi));
                have_amax = true;
            }
        }
        if (MODE != kStats || affine) {
            forget();
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                const int idx = t + j * RT;
                float4 o;
                o.x = (float)(((double)v[j].x - mu) * rstd);
                o.y = (float)(((double)v[j].y - mu) * rstd);
                o.z = (float)(((double)v[j].z - mu) * rstd);
                o.w = (float)(((double)v[j].w - mu) * rstd);
                if (idx < K4) {
                    if (a.gain) {
                        const float4 g = reinterpret_cast<const float4*>(a.gain + grp * a.K)[idx];
                        o.x = o.x * g.x; o.y = o.y * g.y; o.z = o.z * g.z; o.w = o.w * g.w;
                    }
                    if (a.bias) {
                        const float4 b = reinterpret_cast<const float4*>(a.bias + grp * a.K)[idx];
                        o.x = o.x + b.x; o.y = o.y + b.y; o.z = o.z + b.z; o.w = o.w + b.w;
                    }
                    v[j] = o;
                }
            }
        }
    }

    if constexpr (MODE != kStats) {
        if (a.xhat_dump && live) {
            float4* __restrict__ d4 = reinterpret_cast<float4*>(a.xhat_dump + row * a.K);
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                const int idx = t + j * RT;
                if (idx < K4) d4[idx] = v[j];
            }
        }
    }

    float gamma;
    if constexpr (MODE == kApply) {
        if (a.nonneg) {  // Eq. 6 per tensor: eta and gamma from the tensor's extremes
            lo = key_float(a.gmin_bits[grp]);
            gamma = fmaxf(key_float(a.gmax_bits[grp]) - lo, 1e-5f);
        } else {
            gamma = fmaxf(__uint_as_float(a.gmax_bits[grp]), 1e-5f);
        }
    } else {
        if (!have_amax && !a.nonneg) {  // uniform: no LayerNorm, or a gain/bias after it
            float m = 0.f;
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                if (t + j * RT < K4)
                    m = fmaxf(m, fmaxf(fmaxf(fabsf(v[j].x), fabsf(v[j].y)),
                                       fmaxf(fabsf(v[j].z), fabsf(v[j].w))));
            }
            amax = row_reduce<WPR>(m, OpMax{}, smf[2], rw, wr);
        } else if (!have_amax) {  // Eq. 6 on such a row: minimum and maximum of the values
            float mn = v[0].x, mx = v[0].x;  // lane 0's first element always exists
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                if (t + j * RT < K4) {
                    mn = fminf(fminf(mn, v[j].x), fminf(fminf(v[j].y, v[j].z), v[j].w));
                    mx = fmaxf(fmaxf(mx, v[j].x), fmaxf(fmaxf(v[j].y, v[j].z), v[j].w));
                }
            }
            if (t >= K4) {  // a lane without elements must not contribute the padding it holds
                mn = __builtin_inff();
                mx = -__builtin_inff();
            }
            lo = row_reduce<WPR>(mn, OpMin{}, smf[2], rw, wr);
            hi_row = row_reduce<WPR>(mx, OpMax{}, smf[3], rw, wr);
            amax = hi_row - lo;
        }
        if constexpr (MODE == kStats) {
            if (a.nonneg) {  // uniform
                if (t == 0 && live) offer_extremes(a, grp, lo, hi_row);
                return;
            }
            // non-negative floats order like their bit patterns: integer max is exact
            // The running maximum only grows, so whoever does not exceed what is there already
            // has nothing to add: the look first keeps thousands of rows from queueing on one
            // address (a stale, lower value only costs the atomic it would have saved).  With one
            // K-group the rows of a workgroup share a maximum and send one candidate.
            __shared__ float wg_amax[NW];
            auto offer = [&](float v, int g) {
                const uint32_t bits = __float_as_uint(v);
                if (bits > __hip_atomic_load(a.gmax_bits + g, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
                    atomicMax(a.gmax_bits + g, bits);
            };
            if (RPW > 1 && a.groups <= 1) {  // uniform
                if (t == 0) wg_amax[rw] = live ? amax : 0.f;
                __syncthreads();
                if (threadIdx.x == 0) {
                    float m = wg_amax[0];
#pragma unroll
                    for (int i = 1; i < RPW; ++i) m = fmaxf(m, wg_amax[i]);
                    offer(m, 0);
                }
            } else if (t == 0 && live) {
                offer(amax, grp);
            }
            return;
        }
        gamma = fmaxf(amax, 1e-5f);
    }

    const float scale = 128.0f / gamma;
    int rs = 0;
    uint32_t* __restrict__ c4 = reinterpret_cast<uint32_t*>(a.codes + row * a.K);
    // code = clamp(rne(x^ * scale), -128, 127), one fp32 operation per step.  The integral
    // float plus 128 lies in 0..255 and goes straight into its byte of the output word;
    // flipping the top bit of each byte turns that offset form into two's complement.
    auto code_word_nonneg = [&](const float4& x) {  // Eq. 6: shift by eta, clamp to [0, 127]
        const float q0 = fminf(fmaxf(rintf((x.x - lo) * scale), 0.f), 127.f);
        const float q1 = fminf(fmaxf(rintf((x.y - lo) * scale), 0.f), 127.f);
        const float q2 = fminf(fmaxf(rintf((x.z - lo) * scale), 0.f), 127.f);
        const float q3 = fminf(fmaxf(rintf((x.w - lo) * scale), 0.f), 127.f);
        uint32_t wd = __builtin_amdgcn_cvt_pk_u8_f32(q0, 0, 0u);
        wd = __builtin_amdgcn_cvt_pk_u8_f32(q1, 1, wd);
        wd = __builtin_amdgcn_cvt_pk_u8_f32(q2, 2, wd);
        return __builtin_amdgcn_cvt_pk_u8_f32(q3, 3, wd);
    };
    auto code_word = [&](const float4& x) {
        const float q0 = fminf(fmaxf(rintf(x.x * scale), -128.f), 127.f) + 128.f;
        const float q1 = fminf(fmaxf(rintf(x.y * scale), -128.f), 127.f) + 128.f;
        const float q2 = fminf(fmaxf(rintf(x.z * scale), -128.f), 127.f) + 128.f;
        const float q3 = fminf(fmaxf(rintf(x.w * scale), -128.f), 127.f) + 128.f;
        uint32_t wd = __builtin_amdgcn_cvt_pk_u8_f32(q0, 0, 0u);
        wd = __builtin_amdgcn_cvt_pk_u8_f32(q1, 1, wd);
        wd = __builtin_amdgcn_cvt_pk_u8_f32(q2, 2, wd);
        wd = __builtin_amdgcn_cvt_pk_u8_f32(q3, 3, wd);
        return wd ^ 0x80808080u;
    };
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int idx = t + j * RT;
        const uint32_t wd = a.nonneg ? code_word_nonneg(v[j]) : code_word(v[j]);
        if (idx < K4) {
            rs = __builtin_amdgcn_sdot4((int)wd, 0x01010101, rs, false);  // sum of the four codes
            if (live) c4[idx] = wd;
        }
    }
    if (a.rowsum) {
        rs = row_reduce<WPR>(rs, OpSum{}, smi, rw, wr);
        if (t == 0 && live) a.rowsum[row] = rs;
    }
    if (t == 0 && live && (MODE == kFull || row < a.groups)) {  // rows 0 .. groups-1 cover every group
        a.gamma[row] = gamma;
        if (a.nonneg) a.eta[row] = lo;
    }
}

// Rows too long for registers (K > 32768): one workgroup of eight waves per row walks the row
// from memory in each pass (it stays in L2 between passes): sums with minimum and maximum,
// then - only with a gain / bias or without LayerNorm, where the largest magnitude is not at
// the minimum or maximum of the raw row - the absmax of the normalised values, then the
// rounding pass.  The arithmetic per element and the order of the fp32 / fp64 operations that
// decide a code are those of ln_quant_rows; only the summation order of the statistics
// differs (each K is served by exactly one of the two kernels, so results stay deterministic).
template <int MODE>
__global__ __launch_bounds__(512) void ln_quant_long(QuantArgs a) {
    constexpr int NW = 8, T = NW * kWave;
    __shared__ double smd[2][NW];
    __shared__ float smf[4][NW];
    __shared__ int smi[NW];
    const int wave = threadIdx.x / kWave, t = threadIdx.x;
    const bool lead = (threadIdx.x & (kWave - 1)) == 0;
    const int64_t row = blockIdx.x;
    const int64_t K4 = a.K / 4;
    const float4* __restrict__ x4 = reinterpret_cast<const float4*>(a.X + row * a.K);
    const int grp = a.groups > 1 ? (int)(row % a.groups) : 0;
    const bool affine = a.gain != nullptr || a.bias != nullptr;
    bool have_amax = false;
    float amax = 0.f, lo = 0.f, hi_row = 0.f;
    double mu = 0.0, rstd = 1.0;

    if (!a.skip_ln) {
        if constexpr (MODE == kApply) {
            mu = a.rowstats[2 * row];
            rstd = a.rowstats[2 * row + 1];
        } else {
            const double c = (double)a.X[row * a.K];
            double s = 0.0, q = 0.0;
            float mn = a.X[row * a.K], mx = mn;
            for (int64_t idx = t; idx < K4; idx += T) {
                const float4 v = x4[idx];
                const double dx = (double)v.x, dy = (double)v.y, dz = (double)v.z, dw = (double)v.w;
                s += (dx + dy) + (dz + dw);
                q = fma(dx - c, dx - c, q);
                q = fma(dy - c, dy - c, q);
                q = fma(dz - c, dz - c, q);
                q = fma(dw - c, dw - c, q);
                mn = fminf(fminf(mn, v.x), fminf(fminf(v.y, v.z), v.w));
                mx = fmaxf(fmaxf(mx, v.x), fmaxf(fmaxf(v.y, v.z), v.w));
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
#pragma unroll
            for (int i = 1; i < NW; ++i) {
                s += smd[0][i];
                q += smd[1][i];
                mn = fminf(mn, smf[0][i]);
                mx = fmaxf(mx, smf[1][i]);
            }
            mu = s / (double)a.K;
            const double var = fmax(q / (double)a.K - (mu - c) * (mu - c), 0.0);
            rstd = 1.0 / sqrt(var + (double)a.eps);
            if constexpr (MODE == kStats) {
                if (t == 0) {
                    a.rowstats[2 * row] = mu;
                    a.rowstats[2 * row + 1] = rstd;
                }
            }
            if (!affine) {
                lo = (float)(((double)mn - mu) * rstd);
                const float hi = (float)(((double)mx - mu) * rstd);
                hi_row = hi;
                amax = a.nonneg ? hi - lo : fmaxf(fabsf(lo), fabsf(hi));
                have_amax = true;
            }
        }
    }
    // the normalised (and scaled, shifted) values of four consecutive elements
    auto xhat_at = [&](int64_t idx) {
        float4 v = x4[idx];
        if (!a.skip_ln) {
            v.x = (float)(((double)v.x - mu) * rstd);
            v.y = (float)(((double)v.y - mu) * rstd);
            v.z = (float)(((double)v.z - mu) * rstd);
            v.w = (float)(((double)v.w - mu) * rstd);
            if (a.gain) {
                const float4 g = reinterpret_cast<const float4*>(a.gain + grp * a.K)[idx];
                v.x = v.x * g.x; v.y = v.y * g.y; v.z = v.z * g.z; v.w = v.w * g.w;
            }
            if (a.bias) {
                const float4 b = reinterpret_cast<const float4*>(a.bias + grp * a.K)[idx];
                v.x = v.x + b.x; v.y = v.y + b.y; v.z = v.z + b.z; v.w = v.w + b.w;
            }
        }
        return v;
    };
    float gamma;
    if constexpr (MODE == kApply) {
        if (a.nonneg) {
            lo = key_float(a.gmin_bits[grp]);
            gamma = fmaxf(key_float(a.gmax_bits[grp]) - lo, 1e-5f);
        } else {
            gamma = fmaxf(__uint_as_float(a.gmax_bits[grp]), 1e-5f);
        }
    } else {
        if (!have_amax) {  // uniform: minimum and maximum of the values that get rounded
            float mn = __builtin_inff(), mx = -__builtin_inff();
            for (int64_t idx = t; idx < K4; idx += T) {
                const float4 v = xhat_at(idx);
                mn = fminf(fminf(mn, v.x), fminf(fminf(v.y, v.z), v.w));
                mx = fmaxf(fmaxf(mx, v.x), fmaxf(fmaxf(v.y, v.z), v.w));
            }
            mn = wave_reduce(mn, OpMin{});
            mx = wave_reduce(mx, OpMax{});
            if (lead) {
                smf[2][wave] = mn;
                smf[3][wave] = mx;
            }
            __syncthreads();
            mn = smf[2][0];
            mx = smf[3][0];
#pragma unroll
            for (int i = 1; i < NW; ++i) {
                mn = fminf(mn, smf[2][i]);
                mx = fmaxf(mx, smf[3][i]);
            }
            lo = mn;
            hi_row = mx;
            amax = a.nonneg ? mx - mn : fmaxf(fabsf(mn), fabsf(mx));
        }
        if constexpr (MODE == kStats) {
            if (a.nonneg) {
                if (t == 0) offer_extremes(a, grp, lo, hi_row);
                return;
            }
            if (t == 0) {
                const uint32_t bits = __float_as_uint(amax);
                if (bits > __hip_atomic_load(a.gmax_bits + grp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
                    atomicMax(a.gmax_bits + grp, bits);
            }
            return;
        }
        gamma = fmaxf(amax, 1e-5f);
    }
    const float scale = 128.0f / gamma;
    int rs = 0;
    uint32_t* __restrict__ c4 = reinterpret_cast<uint32_t*>(a.codes + row * a.K);
    float4* __restrict__ d4 = a.xhat_dump ? reinterpret_cast<float4*>(a.xhat_dump + row * a.K) : nullptr;
    for (int64_t idx = t; idx < K4; idx += T) {
        const float4 x = xhat_at(idx);
        if (d4) d4[idx] = x;
        uint32_t wd;
        if (a.nonneg) {  // Eq. 6: shift by eta, clamp to [0, 127]
            const float q0 = fminf(fmaxf(rintf((x.x - lo) * scale), 0.f), 127.f);
            const float q1 = fminf(fmaxf(rintf((x.y - lo) * scale), 0.f), 127.f);
            const float q2 = fminf(fmaxf(rintf((x.z - lo) * scale), 0.f), 127.f);
            const float q3 = fminf(fmaxf(rintf((x.w - lo) * scale), 0.f), 127.f);
            wd = __builtin_amdgcn_cvt_pk_u8_f32(q0, 0, 0u);
            wd = __builtin_amdgcn_cvt_pk_u8_f32(q1, 1, wd);
            wd = __builtin_amdgcn_cvt_pk_u8_f32(q2, 2, wd);
            wd = __builtin_amdgcn_cvt_pk_u8_f32(q3, 3, wd);
        } else {
            const float q0 = fminf(fmaxf(rintf(x.x * scale), -128.f), 127.f) + 128.f;
            const float q1 = fminf(fmaxf(rintf(x.y * scale), -128.f), 127.f) + 128.f;
            const float q2 = fminf(fmaxf(rintf(x.z * scale), -128.f), 127.f) + 128.f;
            const float q3 = fminf(fmaxf(rintf(x.w * scale), -128.f), 127.f) + 128.f;
            wd = __builtin_amdgcn_cvt_pk_u8_f32(q0, 0, 0u);
            wd = __builtin_amdgcn_cvt_pk_u8_f32(q1, 1, wd);
            wd = __builtin_amdgcn_cvt_pk_u8_f32(q2, 2, wd);
            wd = __builtin_amdgcn_cvt_pk_u8_f32(q3, 3, wd) ^ 0x80808080u;
        }
        rs = __builtin_amdgcn_sdot4((int)wd, 0x01010101, rs, false);
        c4[idx] = wd;
    }
    if (a.rowsum) {
        rs = wave_reduce(rs, OpSum{});
        if (lead) smi[wave] = rs;
        __syncthreads();
        if (t == 0) {
            int r = smi[0];
#pragma unroll
            for (int i = 1; i < NW; ++i) r += smi[i];
            a.rowsum[row] = r;
        }
    }
    if (t == 0 && (MODE == kFull || row < a.groups)) {
        a.gamma[row] = gamma;
        if (a.nonneg) a.eta[row] = lo;
    }
}

// running maxima start at 0 (below every key and every non-negative float), minima at all ones
__global__ void fill_extremes(uint32_t* gmax, uint32_t* gmin, int n) {
    if ((int)threadIdx.x < n) {
        gmax[threadIdx.x] = 0u;
        if (gmin) gmin[threadIdx.x] = 0xFFFFFFFFu;
    }
}

// rows of up to 32768 elements stay in registers (16 float4 per lane, up to 8 waves); longer
// ones take ln_quant_long
bool quant_supported(int64_t K) { return K % 4 == 0; }
static bool quant_in_registers(int64_t K) { return K / 4 <= 8 * kWave * 16; }

template <int WPR, int NV>
static void launch_mode(const QuantArgs& a, hipStream_t s) {
    constexpr int NW = WPR < 4 ? 4 : WPR, RPW = NW / WPR;
    const unsigned grid = (unsigned)((a.M + RPW - 1) / RPW);
    if (!a.per_tensor) {
        ln_quant_rows<WPR, NV, kFull><<<grid, NW * kWave, 0, s>>>(a);
    } else {
        fill_extremes<<<1, 64, 0, s>>>(a.gmax_bits, a.nonneg ? a.gmin_bits : nullptr, a.groups);
        ln_quant_rows<WPR, NV, kStats><<<grid, NW * kWave, 0, s>>>(a);
        ln_quant_rows<WPR, NV, kApply><<<grid, NW * kWave, 0, s>>>(a);
    }
}

// Waves per row: enough of them that the chip holds about sixteen waves per CU (short rows
// of a small batch are split over several waves rather than leaving most SIMDs idle), and
// never more than 16 float4 per lane.
hipError_t launch_quant(const QuantArgs& a, hipStream_t s) {
    const int64_t K4 = a.K / 4;
    if (!quant_in_registers(a.K)) {
        const unsigned grid = (unsigned)a.M;
        if (!a.per_tensor) {
            ln_quant_long<kFull><<<grid, 512, 0, s>>>(a);
        } else {
            fill_extremes<<<1, 64, 0, s>>>(a.gmax_bits, a.nonneg ? a.gmin_bits : nullptr, a.groups);
            ln_quant_long<kStats><<<grid, 512, 0, s>>>(a);
            ln_quant_long<kApply><<<grid, 512, 0, s>>>(a);
        }
        return hipGetLastError();
    }
    int wpr = 1;
    while (wpr < 8 && K4 > (int64_t)wpr * kWave * 16) wpr *= 2;             // capacity
    while (wpr < 8 && a.M * wpr < 4096 && K4 >= (int64_t)wpr * 2 * kWave * 4) wpr *= 2;  // occupancy
    if (const int v = tuning().quant_wpr)
        if ((v == 1 || v == 2 || v == 4 || v == 8) && K4 <= (int64_t)v * kWave * 16) wpr = v;
    const int64_t per_lane = (K4 + wpr * kWave - 1) / (wpr * kWave);
    int nv = 1;
    while (nv < per_lane) nv *= 2;
    if (wpr == 2 && nv < 4) nv = 4;
    if (wpr == 4 && nv < 4) nv = 4;
    if (wpr == 8 && nv < 8) nv = 8;
#define BL_QUANT_CASE(W, V) if (wpr == W && nv == V) launch_mode<W, V>(a, s); else
    BL_QUANT_CASE(1, 1) BL_QUANT_CASE(1, 2) BL_QUANT_CASE(1, 4) BL_QUANT_CASE(1, 8) BL_QUANT_CASE(1, 16)
    BL_QUANT_CASE(2, 4) BL_QUANT_CASE(2, 8) BL_QUANT_CASE(2, 16)
    BL_QUANT_CASE(4, 4) BL_QUANT_CASE(4, 8) BL_QUANT_CASE(4, 16)
    BL_QUANT_CASE(8, 8) BL_QUANT_CASE(8, 16)
    return hipErrorInvalidValue;
#undef BL_QUANT_CASE
    return hipGetLastError();
}

}  // namespace bl

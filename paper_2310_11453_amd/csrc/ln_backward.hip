// Backward of the LayerNorm in front of the quantiser (arXiv 2310.11453, Eq. 12; per K-group:
// Eq. 15).  Under the straight-through estimator of Section 2.2 the gradient that
// bitlinear_backward_ste returns is the gradient with respect to the LayerNorm output; this
// file takes it to the layer's input x and to the optional gain and bias:
//   xn = (x - mu) * rstd,  gh = g * gain
//   dx = rstd * (gh - mean(gh) - xn * mean(gh * xn))
//   dgain[k] = sum_m g[m,k] * xn[m,k],   dbias[k] = sum_m g[m,k]
// HBM-bound: 8 bytes read and 4 written per element for dx; the gain/bias gradients are a
// second pass over g and x (column sums) and only run when asked for.
#include "common.h"
#include "kernels.h"
#include "rowops.h"

namespace bl {

// One to eight waves own one row (a token, or one K-group of a token); x and g of the row
// stay in registers (NV float4 per lane each).  Statistics and the two means are fp64, as in
// the forward kernel.  Rows are the consecutive K-element pieces of X, so a K-group of a
// token is simply a row of its own.
template <int WPR, int NV>
__global__ __launch_bounds__((WPR < 4 ? 4 : WPR) * kWave, 4) void ln_backward_rows(LnBackwardArgs a) {
    constexpr int NW = WPR < 4 ? 4 : WPR;
    constexpr int RT = WPR * kWave;
    __shared__ double smd[4][NW];

    const int wave = threadIdx.x / kWave;
    const int rw = wave / WPR, wr = wave % WPR;
    const int t = wr * kWave + (threadIdx.x & (kWave - 1));
    int64_t row = (int64_t)blockIdx.x * (NW / WPR) + rw;
    const bool live = row < a.M;
    if constexpr (WPR == 1) {
        if (!live) return;  // no barriers on this path
    } else {
        if (!live) row = a.M - 1;
    }
    const int K4 = (int)(a.K / 4);
    const float4* __restrict__ x4 = reinterpret_cast<const float4*>(a.X + row * a.K);
    const float4* g4 = reinterpret_cast<const float4*>(a.g + row * a.K);  // may alias dX
    const int grp = a.groups > 1 ? (int)(row % a.groups) : 0;

    float4 x[NV], g[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int idx = t + j * RT;
        x[j] = x4[idx < K4 ? idx : K4 - 1];
        g[j] = g4[idx < K4 ? idx : K4 - 1];
    }
    if (a.gain) {
        const float4* __restrict__ w4 = reinterpret_cast<const float4*>(a.gain + grp * a.K);
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int idx = t + j * RT;
            const float4 w = w4[idx < K4 ? idx : K4 - 1];
            g[j].x *= w.x; g[j].y *= w.y; g[j].z *= w.z; g[j].w *= w.w;
        }
    }

    // mean and variance of the row, one pass, shifted by an element of the row
    const double c = (double)a.X[row * a.K];
    double s = 0.0, q = 0.0;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        if (t + j * RT < K4) {
            const double dx = (double)x[j].x, dy = (double)x[j].y, dz = (double)x[j].z, dw = (double)x[j].w;
            s += (dx + dy) + (dz + dw);
            q = fma(dx - c, dx - c, q);
            q = fma(dy - c, dy - c, q);
            q = fma(dz - c, dz - c, q);
            q = fma(dw - c, dw - c, q);
        }
    }
    s = wave_reduce(s, OpSum{});
    q = wave_reduce(q, OpSum{});
    if constexpr (WPR > 1) {
        if ((threadIdx.x & (kWave - 1)) == 0) {
            smd[0][wave] = s;
            smd[1][wave] = q;
        }
        __syncthreads();
        s = smd[0][rw * WPR];
        q = smd[1][rw * WPR];
#pragma unroll
        for (int i = 1; i < WPR; ++i) {
            s += smd[0][rw * WPR + i];
            q += smd[1][rw * WPR + i];
        }
    }
    const double mu = s / (double)a.K;
    const double var = fmax(q / (double)a.K - (mu - c) * (mu - c), 0.0);
    const double rstd = 1.0 / sqrt(var + (double)a.eps);
    if (a.rowstats && t == 0 && live) {
        a.rowstats[2 * row] = mu;
        a.rowstats[2 * row + 1] = rstd;
    }
    if (!a.dX) return;  // uniform: only the statistics were wanted

    // hide x from the optimiser so that the fp64 copies of the first pass are not kept alive
#pragma unroll
    for (int j = 0; j < NV; ++j) asm volatile("" : "+v"(x[j].x), "+v"(x[j].y), "+v"(x[j].z), "+v"(x[j].w));
    // xn replaces x; c1 = sum gh, c2 = sum gh * xn
    double c1 = 0.0, c2 = 0.0;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        x[j].x = (float)(((double)x[j].x - mu) * rstd);
        x[j].y = (float)(((double)x[j].y - mu) * rstd);
        x[j].z = (float)(((double)x[j].z - mu) * rstd);
        x[j].w = (float)(((double)x[j].w - mu) * rstd);
        if (t + j * RT < K4) {
            c1 += ((double)g[j].x + (double)g[j].y) + ((double)g[j].z + (double)g[j].w);
            c2 = fma((double)g[j].x, (double)x[j].x, c2);
            c2 = fma((double)g[j].y, (double)x[j].y, c2);
            c2 = fma((double)g[j].z, (double)x[j].z, c2);
            c2 = fma((double)g[j].w, (double)x[j].w, c2);
        }
    }
    c1 = wave_reduce(c1, OpSum{});
    c2 = wave_reduce(c2, OpSum{});
    if constexpr (WPR > 1) {
        if ((threadIdx.x & (kWave - 1)) == 0) {
            smd[2][wave] = c1;
            smd[3][wave] = c2;
        }
        __syncthreads();
        c1 = smd[2][rw * WPR];
        c2 = smd[3][rw * WPR];
#pragma unroll
        for (int i = 1; i < WPR; ++i) {
            c1 += smd[2][rw * WPR + i];
            c2 += smd[3][rw * WPR + i];
        }
    }
    const float m1 = (float)(c1 / (double)a.K), m2 = (float)(c2 / (double)a.K);
    const float r = (float)rstd;
    float4* d4 = reinterpret_cast<float4*>(a.dX + row * a.K);
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int idx = t + j * RT;
        float4 o;
        o.x = r * ((g[j].x - m1) - x[j].x * m2);
        o.y = r * ((g[j].y - m1) - x[j].y * m2);
        o.z = r * ((g[j].z - m1) - x[j].z * m2);
        o.w = r * ((g[j].w - m1) - x[j].w * m2);
        if (idx < K4 && live) d4[idx] = o;
    }
}

// Rows too long for registers (K / groups > 16384): one workgroup of eight waves per row walks
// the row from memory in each of the three passes (statistics, the two means, dx), the same
// arithmetic per element; x and g of a row stay in L2 between the passes.
__global__ __launch_bounds__(512) void ln_backward_long(LnBackwardArgs a) {
    constexpr int NW = 8, T = NW * kWave;
    __shared__ double smd[4][NW];
    const int wave = threadIdx.x / kWave, t = threadIdx.x;
    const bool lead = (threadIdx.x & (kWave - 1)) == 0;
    const int64_t row = blockIdx.x;
    const int64_t K4 = a.K / 4;
    const float4* __restrict__ x4 = reinterpret_cast<const float4*>(a.X + row * a.K);
    const float4* g4 = reinterpret_cast<const float4*>(a.g + row * a.K);  // may alias dX
    const int grp = a.groups > 1 ? (int)(row % a.groups) : 0;
    const float4* __restrict__ w4 =
        a.gain ? reinterpret_cast<const float4*>(a.gain + grp * a.K) : nullptr;

    const double c = (double)a.X[row * a.K];
    double s = 0.0, q = 0.0;
    for (int64_t idx = t; idx < K4; idx += T) {
        const float4 v = x4[idx];
        const double dx = (double)v.x, dy = (double)v.y, dz = (double)v.z, dw = (double)v.w;
        s += (dx + dy) + (dz + dw);
        q = fma(dx - c, dx - c, q);
        q = fma(dy - c, dy - c, q);
        q = fma(dz - c, dz - c, q);
        q = fma(dw - c, dw - c, q);
    }
    s = wave_reduce(s, OpSum{});
    q = wave_reduce(q, OpSum{});
    if (lead) {
        smd[0][wave] = s;
        smd[1][wave] = q;
    }
    __syncthreads();
    s = smd[0][0];
    q = smd[1][0];
#pragma unroll
    for (int i = 1; i < NW; ++i) {
        s += smd[0][i];
        q += smd[1][i];
    }
    const double mu = s / (double)a.K;
    const double var = fmax(q / (double)a.K - (mu - c) * (mu - c), 0.0);
    const double rstd = 1.0 / sqrt(var + (double)a.eps);
    if (a.rowstats && t == 0) {
        a.rowstats[2 * row] = mu;
        a.rowstats[2 * row + 1] = rstd;
    }
    if (!a.dX) return;

    auto load = [&](int64_t idx, float4& xn, float4& gh) {
        const float4 v = x4[idx];
        gh = g4[idx];
        if (w4) {
            const float4 w = w4[idx];
            gh.x *= w.x; gh.y *= w.y; gh.z *= w.z; gh.w *= w.w;
        }
        xn.x = (float)(((double)v.x - mu) * rstd);
        xn.y = (float)(((double)v.y - mu) * rstd);
        xn.z = (float)(((double)v.z - mu) * rstd);
        xn.w = (float)(((double)v.w - mu) * rstd);
    };
    double c1 = 0.0, c2 = 0.0;
    for (int64_t idx = t; idx < K4; idx += T) {
        float4 xn, gh;
        load(idx, xn, gh);
        c1 += ((double)gh.x + (double)gh.y) + ((double)gh.z + (double)gh.w);
        c2 = fma((double)gh.x, (double)xn.x, c2);
        c2 = fma((double)gh.y, (double)xn.y, c2);
        c2 = fma((double)gh.z, (double)xn.z, c2);
        c2 = fma((double)gh.w, (double)xn.w, c2);
    }
    c1 = wave_reduce(c1, OpSum{});
    c2 = wave_reduce(c2, OpSum{});
    if (lead) {
        smd[2][wave] = c1;
        smd[3][wave] = c2;
    }
    __syncthreads();  // also: every read of g in the pass above is done before dX (= g) is written
    c1 = smd[2][0];
    c2 = smd[3][0];
#pragma unroll
    for (int i = 1; i < NW; ++i) {
        c1 += smd[2][i];
        c2 += smd[3][i];
    }
    const float m1 = (float)(c1 / (double)a.K), m2 = (float)(c2 / (double)a.K);
    const float r = (float)rstd;
    float4* d4 = reinterpret_cast<float4*>(a.dX + row * a.K);
    for (int64_t idx = t; idx < K4; idx += T) {
        float4 xn, gh, o;
        load(idx, xn, gh);
        o.x = r * ((gh.x - m1) - xn.x * m2);
        o.y = r * ((gh.y - m1) - xn.y * m2);
        o.z = r * ((gh.z - m1) - xn.z * m2);
        o.w = r * ((gh.w - m1) - xn.w * m2);
        d4[idx] = o;
    }
}

// Column sums for the gain and bias gradients: thread = one float4 of columns of the full
// token width (groups * K), workgroup row = a chunk of tokens; fp64 partials per chunk.
__global__ __launch_bounds__(256) void ln_backward_affine_partial(LnBackwardArgs a, int64_t tokens,
                                                                  int64_t width, int rows_per_chunk,
                                                                  double* __restrict__ partials) {
    const int64_t c4 = (int64_t)blockIdx.x * 256 + threadIdx.x;  // float4 column
    if (c4 * 4 >= width) return;
    const int grp = (int)(c4 * 4 / a.K);
    const int64_t m0 = (int64_t)blockIdx.y * rows_per_chunk;
    const int64_t m1 = m0 + rows_per_chunk < tokens ? m0 + rows_per_chunk : tokens;
    double dg[4] = {0, 0, 0, 0}, db[4] = {0, 0, 0, 0};
    for (int64_t m = m0; m < m1; ++m) {
        const float4 x = reinterpret_cast<const float4*>(a.X + m * width)[c4];
        const float4 g = reinterpret_cast<const float4*>(a.g + m * width)[c4];
        const double mu = a.rowstats[2 * (m * a.groups + grp)];
        const double rstd = a.rowstats[2 * (m * a.groups + grp) + 1];
        dg[0] = fma((double)g.x, ((double)x.x - mu) * rstd, dg[0]);
        dg[1] = fma((double)g.y, ((double)x.y - mu) * rstd, dg[1]);
        dg[2] = fma((double)g.z, ((double)x.z - mu) * rstd, dg[2]);
        dg[3] = fma((double)g.w, ((double)x.w - mu) * rstd, dg[3]);
        db[0] += (double)g.x; db[1] += (double)g.y; db[2] += (double)g.z; db[3] += (double)g.w;
    }
    double* p = partials + ((int64_t)blockIdx.y * 2) * width + c4 * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        p[i] = dg[i];
        p[width + i] = db[i];
    }
}

__global__ __launch_bounds__(256) void ln_backward_affine_final(const double* __restrict__ partials,
                                                                int chunks, int64_t width,
                                                                float* __restrict__ dgain,
                                                                float* __restrict__ dbias) {
    const int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k >= width) return;
    double dg = 0.0, db = 0.0;
    for (int cidx = 0; cidx < chunks; ++cidx) {
        dg += partials[((int64_t)cidx * 2) * width + k];
        db += partials[((int64_t)cidx * 2 + 1) * width + k];
    }
    if (dgain) dgain[k] = (float)dg;
    if (dbias) dbias[k] = (float)db;
}

bool ln_backward_supported(int64_t K) { return K % 4 == 0; }
static bool ln_backward_in_registers(int64_t K) { return K / 4 <= 8 * kWave * 8; }

int ln_backward_chunks(int64_t tokens) {
    int64_t c = (tokens + 127) / 128;
    return (int)(c < 1 ? 1 : c > 64 ? 64 : c);
}

template <int WPR, int NV>
static void launch_rows(const LnBackwardArgs& a, hipStream_t s) {
    constexpr int NW = WPR < 4 ? 4 : WPR, RPW = NW / WPR;
    ln_backward_rows<WPR, NV><<<(unsigned)((a.M + RPW - 1) / RPW), NW * kWave, 0, s>>>(a);
}

// a.M counts rows of a.K elements (tokens * groups); a.rowstats must be given when dgain or
// dbias is wanted; `partials` holds chunks * 2 * width doubles.
hipError_t launch_ln_backward(const LnBackwardArgs& a, float* dgain, float* dbias, double* partials,
                              hipStream_t s) {
    const int64_t K4 = a.K / 4;
    int wpr = 1;
    while (wpr < 8 && K4 > (int64_t)wpr * kWave * 8) wpr *= 2;
    const int64_t per_lane = (K4 + wpr * kWave - 1) / (wpr * kWave);
    int nv = 1;
    while (nv < per_lane) nv *= 2;
    if (wpr > 1 && nv < 8) nv = 8;
    auto rows = [&](const LnBackwardArgs& r) {
        if (!ln_backward_in_registers(r.K)) {
            ln_backward_long<<<(unsigned)r.M, 512, 0, s>>>(r);
            return true;
        }
#define BL_LNB_CASE(W, V) if (wpr == W && nv == V) launch_rows<W, V>(r, s); else
        BL_LNB_CASE(1, 1) BL_LNB_CASE(1, 2) BL_LNB_CASE(1, 4) BL_LNB_CASE(1, 8)
        BL_LNB_CASE(2, 8) BL_LNB_CASE(4, 8) BL_LNB_CASE(8, 8)
        return false;
#undef BL_LNB_CASE
        return true;
    };
    if (dgain || dbias) {
        // The column sums read g, which dX may overwrite: statistics first, then the sums, then dX.
        LnBackwardArgs st = a;
        st.dX = nullptr;
        if (!rows(st)) return hipErrorInvalidValue;
        const int64_t tokens = a.M / a.groups, width = a.K * a.groups;
        const int chunks = ln_backward_chunks(tokens);
        const int rows_per_chunk = (int)((tokens + chunks - 1) / chunks);
        dim3 grid((unsigned)((width / 4 + 255) / 256), (unsigned)chunks);
        ln_backward_affine_partial<<<grid, 256, 0, s>>>(a, tokens, width, rows_per_chunk, partials);
        ln_backward_affine_final<<<(unsigned)((width + 255) / 256), 256, 0, s>>>(partials, chunks, width,
                                                                                  dgain, dbias);
    }
    if (a.dX && !rows(a)) return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace bl

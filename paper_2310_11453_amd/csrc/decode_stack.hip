// A chain of BitLinear layers for a handful of tokens in ONE launch:
//   h_0 = X,  h_l = BitLinear_l(leading K_l columns of h_{l-1}),  Y = h_L
// each layer being Eq. 12 (LayerNorm), Eq. 4-5 (absmax quantiser), Eq. 7 and Eq. 11 of
// arXiv 2310.11453, per token.  Decoding one token runs dozens of such layers whose weights are
// a few MB each: launched one by one, every layer costs two launches (quantiser, GEMM) of
// about 4 us each next to 1-5 us of weight streaming.  Here one persistent workgroup per CU
// walks all layers and the workgroups meet at a barrier between layers.
//
// Per layer and workgroup:
//  1. LayerNorm + quantiser of the M input rows, by every workgroup for itself (M rows of K
//     floats out of L2; cheaper than a second grid barrier): codes go to LDS, gamma and the row
//     sums too.  The arithmetic and the order of the reductions are those of the stand-alone
//     quantiser with 4 (K <= 16384) or 8 waves per row, so the codes are the same bit for bit.
//  2. The workgroup's share of the weight tiles (a contiguous range of tile rows), streamed
//     global -> LDS by DMA through a small ring per wave (the wave that asks for a tile is the
//     one that reads it: no barrier, only s_waitcnt vmcnt counted by hand), ANDed into bit planes
//     and multiplied on the i8 MFMA exactly as in the stand-alone small-batch GEMM.  Waves split K
//     (wk) and, when K is short, tile rows (wt); partial sums meet in LDS.
//  3. Dequantisation, stores, then the grid barrier: arrive (release), the other waves request
//     their first tiles of the next layer, wave 0 spins (bounded) and acquires.
#include "common.h"
#include "decode_stack.h"
#include "ring.h"
#include "rowops.h"

namespace bl {

// ---- asm: LDS accesses whose ordering against the DMA the compiler must not guess ---------
__device__ inline void stack_read_act(v4i (&a)[8], uint32_t ad) {
    asm volatile(
        "ds_read_b128 %0, %8\n\t"
        "ds_read_b128 %1, %8 offset:64\n\t"
        "ds_read_b128 %2, %8 offset:128\n\t"
        "ds_read_b128 %3, %8 offset:192\n\t"
        "ds_read_b128 %4, %8 offset:256\n\t"
        "ds_read_b128 %5, %8 offset:320\n\t"
        "ds_read_b128 %6, %8 offset:384\n\t"
        "ds_read_b128 %7, %8 offset:448\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(a[0]), "=&v"(a[1]), "=&v"(a[2]), "=&v"(a[3]), "=&v"(a[4]), "=&v"(a[5]),
          "=&v"(a[6]), "=&v"(a[7])
        : "v"(ad)
        : "memory");
}
__device__ inline v4i stack_read_tile(uint32_t ad) {
    v4i v;
    asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=&v"(v) : "v"(ad) : "memory");
    return v;
}
__device__ inline void stack_red_store(uint32_t ad, v4i v) {
    asm volatile("ds_write_b128 %0, %1" : : "v"(ad), "v"(v) : "memory");
}
__device__ inline void stack_red_add(uint32_t ad, v4i v) {
    asm volatile(
        "ds_add_u32 %0, %1\n\t"
        "ds_add_u32 %0, %2 offset:4\n\t"
        "ds_add_u32 %0, %3 offset:8\n\t"
        "ds_add_u32 %0, %4 offset:12"
        :
        : "v"(ad), "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3])
        : "memory");
}

__global__ __launch_bounds__(kStackWaves* kWave) void decode_stack_kernel(StackArgs a) {
    __shared__ __attribute__((aligned(1024))) uint8_t smRing[kStackWaves * kStackD * 2048];
    __shared__ __attribute__((aligned(16))) uint8_t smCodes[kStackCodes];
    __shared__ __attribute__((aligned(16))) int smRed[kStackWaves * kStackTpw * 256];
    __shared__ double smd[2][kStackWaves];
    __shared__ float smf[2][kStackWaves];
    __shared__ int smi[kStackWaves];
    __shared__ float smGamma[16];
    __shared__ int smRs[16];
    __shared__ int smFail;

    const int w = threadIdx.x / kWave, l = threadIdx.x % kWave;
    const int G = (int)gridDim.x, b = (int)blockIdx.x;
    const int M = a.M;
    const int m = l & 15, g = l >> 4;           // MFMA lane: token m, row group g
    const int mrow = m < M ? m : M - 1;
    if (threadIdx.x == 0) smFail = 0;
    const uint32_t ring_wave = (uint32_t)(uintptr_t)smRing + (uint32_t)w * (kStackD * 2048);
    const uint32_t red_wave = (uint32_t)(uintptr_t)smRed + (uint32_t)(w * kStackTpw * kWave + l) * 16;

    // ---- the weight stream of this wave in the current layer --------------------------------
    // units in the order pass p, round rd, tile t; `issued` and `consumed` count units
    const uint32_t* s_packed = nullptr;
    int s_TK = 0, s_WK = 1, s_C = 1, s_first = 0, s_step = 0, s_r1 = 0, s_P = 0, s_Rw = 0, s_wk = 0;
    int pp = 0, prd = 0, pt = 0, issued = 0, consumed = 0;
    bool pdone = true;
    auto tiles_in_pass = [&](int p) {  // tiles of this wave in pass p; first tile row: s_first + p * s_step
        int c = s_r1 - (s_first + p * s_step);
        return c < 0 ? 0 : c > kStackTpw ? kStackTpw : c;
    };
    auto stream_begin = [&](int li) {
        const StackLayer raw = a.layers[li];
        StackPlan L;
        stack_plan(raw.N, raw.K, M, L);  // validated on the host
        const int wk = w % L.WK, wt = w / L.WK;
        const int r0 = (int)((int64_t)L.TN * b / G);
        s_r1 = (int)((int64_t)L.TN * (b + 1) / G);
        s_packed = raw.packed;
        s_TK = L.TK, s_WK = L.WK, s_C = L.C, s_wk = wk;
        s_step = L.WT * kStackTpw;
        s_first = r0 + wt * kStackTpw;
        s_P = (s_r1 - r0 + s_step - 1) / s_step;
        s_Rw = (wt < L.WT && wk < L.pairs) ? (L.pairs - wk + L.WK - 1) / L.WK : 0;
        pp = prd = pt = issued = consumed = 0;
        pdone = s_Rw == 0 || s_P == 0 || tiles_in_pass(0) == 0;
    };
    auto issue_unit = [&]() {
        const int64_t tn = s_first + pp * s_step + pt;
        const int64_t tk = (int64_t)(prd * s_WK + s_wk) * s_C;
        const uint32_t* src = s_packed + (tn * s_TK + tk) * 256 + l * 4;
        const uint32_t dst = ring_wave + (uint32_t)(issued % kStackD) * 2048;
        __builtin_amdgcn_global_load_lds((const void*)src,
                                         (__attribute__((address_space(3))) void*)(uintptr_t)dst, 16,
                                         0, 0);
        if (s_C == 2)
            __builtin_amdgcn_global_load_lds(
                (const void*)(src + 256),
                (__attribute__((address_space(3))) void*)(uintptr_t)(dst + 1024), 16, 0, 0);
        ++issued;
        if (++pt >= tiles_in_pass(pp)) {
            pt = 0;
            if (++prd >= s_Rw) {
                prd = 0;
                ++pp;
                if (pp >= s_P || tiles_in_pass(pp) == 0) pdone = true;
            }
        }
    };
    auto fill_ring = [&]() {
        while (!pdone && issued - consumed < kStackD) issue_unit();
    };

    // ---- grid barrier: every workgroup arrives once per call; `target` arrivals release it ----
    // Wave 0 arrives and spins (bounded: a workgroup that never shows up ends the kernel with
    // the error flag set instead of hanging it); the other waves use the time to request the
    // first tiles of the next layer.
    auto grid_barrier = [&](unsigned target, int next) {
        __syncthreads();
        if (w == 0) {
            if (l == 0) {
                __threadfence();  // release: this workgroup's stores, written back past its L2
                __hip_atomic_fetch_add(a.sync, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                unsigned spins = 0;
                bool ok = true;
                while (__hip_atomic_load(a.sync, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
                    __builtin_amdgcn_s_sleep(4);
                    if (++spins > a.spin_limit) {
                        ok = false;
                        break;
                    }
                }
                __threadfence();  // acquire: drop what this CU and its L2 hold of the other outputs
                if (!ok) {
                    smFail = 1;
                    __hip_atomic_store(a.sync + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        } else {
            stream_begin(next);
            fill_ring();
        }
        __syncthreads();
        if (w == 0 && smFail == 0) {
            stream_begin(next);
            fill_ring();
        }
        return smFail == 0;
    };

    const float* xin = a.X;
    int in_pitch = (int)a.layers[0].K;
    stream_begin(0);
    fill_ring();

    for (int li = 0; li < a.n_layers; ++li) {
        const StackLayer raw = a.layers[li];
        StackPlan L;
        stack_plan(raw.N, raw.K, M, L);
        const int N = (int)raw.N, K = (int)raw.K, K4 = K / 4, Kpad = L.Kpad;
        float* yout = li == a.n_layers - 1 ? a.Y : a.buf[li & 1];

        // ---- 1. LayerNorm + absmax quantiser (Eq. 12, 4, 5), row by row, LW waves per row ----
        const int LW = L.ln_waves, RT = LW * kWave;
        const int t = threadIdx.x;  // lane of the row (only t < RT hold elements)
        for (int r = 0; r < M; ++r) {
            const float* xr = xin + (int64_t)r * in_pitch;
            const float4* x4 = reinterpret_cast<const float4*>(xr);
            // the row's first element (a per-lane load: the row was written during this kernel)
            const float first = *reinterpret_cast<const volatile float*>(xr);
            const double c = (double)first;
            double s = 0.0, q = 0.0;
            float mn = first, mx = first;
            if (t < RT) {
                for (int idx = t; idx < K4; idx += RT) {
                    const float4 v = x4[idx];
                    const double dx = (double)v.x, dy = (double)v.y;
                    const double dz = (double)v.z, dw = (double)v.w;
                    s += (dx + dy) + (dz + dw);
                    q = fma(dx - c, dx - c, q);
                    q = fma(dy - c, dy - c, q);
                    q = fma(dz - c, dz - c, q);
                    q = fma(dw - c, dw - c, q);
                    mn = fminf(fminf(mn, v.x), fminf(fminf(v.y, v.z), v.w));
                    mx = fmaxf(fmaxf(mx, v.x), fmaxf(fmaxf(v.y, v.z), v.w));
                }
            }
            s = wave_reduce(s, OpSum{});
            q = wave_reduce(q, OpSum{});
            mn = wave_reduce(mn, OpMin{});
            mx = wave_reduce(mx, OpMax{});
            if (l == 0) {
                smd[0][w] = s;
                smd[1][w] = q;
                smf[0][w] = mn;
                smf[1][w] = mx;
            }
            __syncthreads();
            s = smd[0][0];
            q = smd[1][0];
            mn = smf[0][0];
            mx = smf[1][0];
            for (int i = 1; i < LW; ++i) {
                s += smd[0][i];
                q += smd[1][i];
                mn = fminf(mn, smf[0][i]);
                mx = fmaxf(mx, smf[1][i]);
            }
            const double mu = s / (double)K;
            const double var = fmax(q / (double)K - (mu - c) * (mu - c), 0.0);
            const double rstd = 1.0 / sqrt(var + (double)a.eps);
            const float lo = (float)(((double)mn - mu) * rstd);
            const float hi = (float)(((double)mx - mu) * rstd);
            const float gamma = fmaxf(fmaxf(fabsf(lo), fabsf(hi)), 1e-5f);
            const float scale = 128.0f / gamma;
            int rs = 0;
            uint32_t* c4 = reinterpret_cast<uint32_t*>(smCodes + (size_t)r * Kpad);
            if (t < RT) {
                for (int idx = t; idx < K4; idx += RT) {
                    const float4 v = x4[idx];
                    const float ox = (float)(((double)v.x - mu) * rstd);
                    const float oy = (float)(((double)v.y - mu) * rstd);
                    const float oz = (float)(((double)v.z - mu) * rstd);
                    const float ow = (float)(((double)v.w - mu) * rstd);
                    const float q0 = fminf(fmaxf(rintf(ox * scale), -128.f), 127.f) + 128.f;
                    const float q1 = fminf(fmaxf(rintf(oy * scale), -128.f), 127.f) + 128.f;
                    const float q2 = fminf(fmaxf(rintf(oz * scale), -128.f), 127.f) + 128.f;
                    const float q3 = fminf(fmaxf(rintf(ow * scale), -128.f), 127.f) + 128.f;
                    uint32_t wd = __builtin_amdgcn_cvt_pk_u8_f32(q0, 0, 0u);
                    wd = __builtin_amdgcn_cvt_pk_u8_f32(q1, 1, wd);
                    wd = __builtin_amdgcn_cvt_pk_u8_f32(q2, 2, wd);
                    wd = __builtin_amdgcn_cvt_pk_u8_f32(q3, 3, wd);
                    wd ^= 0x80808080u;
                    rs = __builtin_amdgcn_sdot4((int)wd, 0x01010101, rs, false);
                    c4[idx] = wd;
                }
            }
            // columns K .. Kpad-1 (the packed bits there are zero)
            for (int idx = K4 + threadIdx.x; idx < Kpad / 4; idx += kStackWaves * kWave) c4[idx] = 0u;
            rs = wave_reduce(rs, OpSum{});
            if (l == 0) smi[w] = rs;
            __syncthreads();
            if (threadIdx.x == 0) {
                int tot = 0;
                for (int i = 0; i < LW; ++i) tot += smi[i];
                smRs[r] = tot;
                smGamma[r] = gamma;
            }
        }
        __syncthreads();  // codes, gamma and row sums of all rows are in LDS

        // ---- 2. the weight stream -----------------------------------------------------------
        const float beta = *raw.beta;
        const float gm = smGamma[mrow];
        const int rsum = smRs[mrow];
        const int r0 = (int)((int64_t)L.TN * b / G), r1 = (int)((int64_t)L.TN * (b + 1) / G);
        const int step = L.WT * kStackTpw;
        const int P = (r1 - r0 + step - 1) / step;
        const uint32_t act_base = (uint32_t)(uintptr_t)smCodes + (uint32_t)mrow * Kpad + 16 * g;

        auto gemm = [&](auto cc) {
            constexpr int C = decltype(cc)::value;
            v4i act[C][8];
            int act_rd = -1;
            for (int p = 0; p < P; ++p) {
                const int cnt = tiles_in_pass(p);
                for (int rd = 0; rd < s_Rw; ++rd) {
                    if (cnt > 0 && act_rd != rd) {  // this wave's K-chunks of the round
                        const int tk = (rd * s_WK + s_wk) * C;
#pragma unroll
                        for (int c = 0; c < C; ++c) stack_read_act(act[c], act_base + (tk + c) * kChunkK);
                        act_rd = rd;
                    }
                    for (int tt = 0; tt < cnt; ++tt) {
                        // the unit needed now is the oldest one in flight
                        const int younger = issued - consumed - 1;
                        if (younger <= 0) wait_vmcnt<0>();
                        else if (younger == 1) wait_vmcnt<C>();
                        else wait_vmcnt<2 * C>();
                        const uint32_t slot = ring_wave + (uint32_t)(consumed % kStackD) * 2048 + l * 16;
                        v4i wv[C];
#pragma unroll
                        for (int c = 0; c < C; ++c) wv[c] = stack_read_tile(slot + c * 1024);
                        ++consumed;
                        fill_ring();
                        v4i acc[8];
#pragma unroll
                        for (int i = 0; i < 8; ++i) acc[i] = (v4i){0, 0, 0, 0};
#pragma unroll
                        for (int c = 0; c < C; ++c)
#pragma unroll
                            for (int i = 0; i < 8; ++i) {
                                const v4i plane = wv[c] & (int)(0x01010101u << i);
                                acc[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(plane, act[c][i], acc[i],
                                                                               0, 0, 0);
                            }
                        // 128 * sum_k q b = sum_{i<7} acc_i * 2^(7-i) - acc_7
                        v4i sum;
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            int h = acc[0][r];
#pragma unroll
                            for (int i = 1; i < 7; ++i) h = (h << 1) + acc[i][r];
                            sum[r] = (h << 1) - acc[7][r];
                        }
                        if (rd == 0) stack_red_store(red_wave + tt * 1024, sum);
                        else stack_red_add(red_wave + tt * 1024, sum);
                    }
                }
                __syncthreads();
                // ---- 3. fold the K-waves, dequantise (Eq. 11), store -------------------------
                const int first = r0 + p * step;
                const int ntile = r1 - first < step ? r1 - first : step;
                for (int qi = w; qi < ntile; qi += kStackWaves) {
                    const int wtq = qi / kStackTpw, tq = qi % kStackTpw;
                    v4i sum = (v4i){0, 0, 0, 0};
                    for (int k = 0; k < L.WK; ++k)
                        sum += *reinterpret_cast<const v4i*>(
                            &smRed[(((wtq * L.WK + k) * kStackTpw + tq) * kWave + l) * 4]);
                    const int64_t n = (int64_t)(first + qi) * kTileN + 4 * g;
                    if (m < M && n < N) {
                        const v4i pm = (sum >> 6) - rsum;
                        const float sc = (beta * gm) / 128.0f;
                        const v4f o = {(float)pm[0] * sc, (float)pm[1] * sc, (float)pm[2] * sc,
                                       (float)pm[3] * sc};
                        *reinterpret_cast<v4f*>(yout + (int64_t)m * N + n) = o;
                    }
                }
                __syncthreads();
            }
        };
        if (L.C == 2) gemm(std::integral_constant<int, 2>{});
        else gemm(std::integral_constant<int, 1>{});

        if (li + 1 < a.n_layers) {
            if (!grid_barrier((unsigned)(li + 1) * (unsigned)G, li + 1)) {
                wait_vmcnt<0>();  // nothing of this wave may still be on its way into LDS
                return;
            }
            xin = yout;
            in_pitch = N;
        }
    }
}

__global__ void stack_clear_sync(unsigned* p) {
    if (threadIdx.x < 2) p[threadIdx.x] = 0u;
}

int decode_stack_grid() {
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

// One workgroup per CU: each holds ~145 KiB of LDS, so exactly one fits a CU and all of them
// are resident together, which the grid barrier needs.
hipError_t launch_decode_stack(const StackArgs& a, hipStream_t s) {
    stack_clear_sync<<<1, 64, 0, s>>>(a.sync);
    decode_stack_kernel<<<(unsigned)decode_stack_grid(), kStackWaves * kWave, 0, s>>>(a);
    return hipGetLastError();
}

}  // namespace bl

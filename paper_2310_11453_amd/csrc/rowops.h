// Row-wise reduction helpers shared by the quantiser and the LayerNorm backward (gfx950, wave64).
#pragma once
#include "common.h"

namespace bl {

// ---- wave reductions on the DPP path (no LDS traffic) ---------------------------------
// Butterfly inside each row of 16 lanes (xor 1, xor 2, mirror inside 8, mirror inside 16),
// then the four row totals are read back as scalars and combined in a fixed order, so every
// lane ends with the same bits and the result does not depend on the run.
template <int CTRL>
__device__ inline int dpp_mov(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, false);
}
template <int CTRL>
__device__ inline float dpp_mov(float v) {
    return __int_as_float(dpp_mov<CTRL>(__float_as_int(v)));
}
template <int CTRL>
__device__ inline double dpp_mov(double v) {
    return __hiloint2double(dpp_mov<CTRL>(__double2hiint(v)), dpp_mov<CTRL>(__double2loint(v)));
}
__device__ inline int lane_value(int v, int lane) { return __builtin_amdgcn_readlane(v, lane); }
__device__ inline float lane_value(float v, int lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
__device__ inline double lane_value(double v, int lane) {
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), lane),
                            __builtin_amdgcn_readlane(__double2loint(v), lane));
}
struct OpSum {
    template <class T> __device__ T operator()(T a, T b) const { return a + b; }
};
struct OpMax {
    __device__ float operator()(float a, float b) const { return fmaxf(a, b); }
};
struct OpMin {
    __device__ float operator()(float a, float b) const { return fminf(a, b); }
};
template <class T, class Op>
__device__ inline T wave_reduce(T v, Op op) {
    v = op(v, dpp_mov<0xB1>(v));   // quad_perm [1,0,3,2]
    v = op(v, dpp_mov<0x4E>(v));   // quad_perm [2,3,0,1]
    v = op(v, dpp_mov<0x141>(v));  // row_half_mirror
    v = op(v, dpp_mov<0x140>(v));  // row_mirror
    return op(op(lane_value(v, 0), lane_value(v, 16)), op(lane_value(v, 32), lane_value(v, 48)));
}

// Reduction over the WPR waves that share a row: wave totals meet in LDS.  Every wave of the
// workgroup takes part (rows past M are computed on a clamped row and never stored).  Each
// slot array serves one reduction per kernel, so no barrier is needed ahead of the write.
template <int WPR, class T, class Op>
__device__ inline T row_reduce(T v, Op op, T* slots /* [rows per workgroup][WPR] */, int rw, int wr) {
    v = wave_reduce(v, op);
    if constexpr (WPR == 1) return v;
    if ((threadIdx.x & (kWave - 1)) == 0) slots[rw * WPR + wr] = v;
    __syncthreads();
    T r = slots[rw * WPR];
#pragma unroll
    for (int i = 1; i < WPR; ++i) r = op(r, slots[rw * WPR + i]);
    return r;
}

}  // namespace bl

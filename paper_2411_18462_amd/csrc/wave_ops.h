// Wave64 cross-lane primitives for gfx950 built on DPP moves (no LDS traffic).
//
// A wave has 64 lanes in 4 DPP rows of 16.  row_reduce() leaves the combination of a row's
// 16 values in every lane of that row (quad_perm xor-1, xor-2, then row rotations by 4 and
// 8); wave_reduce() then combines the four row results read from lanes 15/31/47/63 with
// v_readlane, so the result is wave-uniform and always associated in the same order.
#pragma once
#include <hip/hip_runtime.h>

namespace svip {

constexpr int DPP_QUAD_XOR1 = 0xB1;   // quad_perm:[1,0,3,2]
constexpr int DPP_QUAD_XOR2 = 0x4E;   // quad_perm:[2,3,0,1]
constexpr int DPP_ROW_ROR4 = 0x124;   // row_ror:4
constexpr int DPP_ROW_ROR8 = 0x128;   // row_ror:8

template <int CTRL>
__device__ __forceinline__ int dpp_mov(int v)
{
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xF, 0xF, false);
}
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v)
{
    return __int_as_float(dpp_mov<CTRL>(__float_as_int(v)));
}
template <int CTRL>
__device__ __forceinline__ double dpp_mov(double v)
{
    int lo = dpp_mov<CTRL>(__double2loint(v));
    int hi = dpp_mov<CTRL>(__double2hiint(v));
    return __hiloint2double(hi, lo);
}

template <int CTRL>
__device__ __forceinline__ unsigned long long dpp_mov(unsigned long long v)
{
    const unsigned lo = (unsigned)dpp_mov<CTRL>((int)(unsigned)v);
    const unsigned hi = (unsigned)dpp_mov<CTRL>((int)(unsigned)(v >> 32));
    return ((unsigned long long)hi << 32) | lo;
}

__device__ __forceinline__ int read_lane(int v, int lane) { return __builtin_amdgcn_readlane(v, lane); }
__device__ __forceinline__ unsigned long long read_lane(unsigned long long v, int lane)
{
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)v, lane);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(v >> 32), lane);
    return ((unsigned long long)hi << 32) | lo;
}
__device__ __forceinline__ float read_lane(float v, int lane)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
__device__ __forceinline__ double read_lane(double v, int lane)
{
    int lo = __builtin_amdgcn_readlane(__double2loint(v), lane);
    int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane);
    return __hiloint2double(hi, lo);
}

struct OpSum {
    template <typename T> __device__ __forceinline__ T operator()(T a, T b) const { return a + b; }
};
struct OpMax {
    __device__ __forceinline__ float operator()(float a, float b) const { return fmaxf(a, b); }
    __device__ __forceinline__ int operator()(int a, int b) const { return a > b ? a : b; }
    __device__ __forceinline__ unsigned long long operator()(unsigned long long a, unsigned long long b) const
    {
        return a > b ? a : b;
    }
};

template <typename T, typename Op>
__device__ __forceinline__ T row_reduce(T v, Op op)
{
    v = op(v, dpp_mov<DPP_QUAD_XOR1>(v));
    v = op(v, dpp_mov<DPP_QUAD_XOR2>(v));
    v = op(v, dpp_mov<DPP_ROW_ROR4>(v));
    v = op(v, dpp_mov<DPP_ROW_ROR8>(v));
    return v;
}

// Wave-uniform combination of all 64 lanes' values.
template <typename T, typename Op>
__device__ __forceinline__ T wave_reduce(T v, Op op)
{
    v = row_reduce(v, op);
    T r0 = read_lane(v, 15), r1 = read_lane(v, 31), r2 = read_lane(v, 47), r3 = read_lane(v, 63);
    return op(op(r0, r1), op(r2, r3));
}

__device__ __forceinline__ float wave_max(float v) { return wave_reduce(v, OpMax{}); }

// Wave-uniform fp64 sum of all 64 lanes' values by the DPP butterfly (about 30 vector-ALU slots).  The same
// sum as two v_mfma_f64_16x16x4 against a matrix of ones is exact too and needs 6 slots, but its long
// dependent latency made every kernel that used it slower (a draft step of 64 rows 12.7 us against 12.2 us,
// the residual pass 13.45 us against 13.1 us), so the matrix cores stay unused in this library.
__device__ __forceinline__ double wave_sum(double v) { return wave_reduce(v, OpSum{}); }

// DPP move that yields 0 where a lane has no source (row shifts) or its row is masked out.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_mov_or_zero(double v)
{
    int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, ROW_MASK, 0xF, true);
    int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, ROW_MASK, 0xF, true);
    return __hiloint2double(hi, lo);
}

// Inclusive prefix sum over the lanes of a wave (lane order) in fp64: Hillis-Steele inside
// each DPP row (row_shr 1, 2, 4, 8), then the row totals are carried across rows with
// row_bcast:15 (into rows 1 and 3) and row_bcast:31 (into rows 2 and 3).
__device__ __forceinline__ double wave_inclusive_sum(double v)
{
    v += dpp_mov_or_zero<0x111, 0xF>(v);
    v += dpp_mov_or_zero<0x112, 0xF>(v);
    v += dpp_mov_or_zero<0x114, 0xF>(v);
    v += dpp_mov_or_zero<0x118, 0xF>(v);
    v += dpp_mov_or_zero<0x142, 0xA>(v);
    v += dpp_mov_or_zero<0x143, 0xC>(v);
    return v;
}

}  // namespace svip

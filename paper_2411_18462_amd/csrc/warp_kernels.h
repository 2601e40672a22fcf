// Kernel of svip_warp_logits: top-k followed by top-p filtering of logits rows (a variant of the
// sampling rows of Algorithms 1, 2 and 4 that the paper does not cover; dropped logits become -inf
// and every other call treats them as tokens of probability zero).
//
// Both filters are thresholds on the logit value, found per row by a radix select over an
// order-preserving 32-bit key of the fp32 logit, most significant digit first (11 + 11 + 10 bits):
//   top-k   select on the COUNT of keys:  tau_k = k-th largest value;
//   top-p   select on the MASS  of keys >= tau_k: the first value, going down, at which the
//           cumulative softmax mass reaches top_p of the mass kept so far.
// Masses are summed as 64-bit fixed-point integers, so a row's thresholds do not depend on the
// order in which workgroup threads reach the histogram.  One workgroup owns a row and re-reads it
// once per digit (the row stays in L2); HBM sees one read and one write of the row.
#pragma once
#include "row_math.h"

namespace svip {

constexpr int WARP_WG = 1024;              // threads of the workgroup that owns a row
constexpr int WARP_WAVES = WARP_WG / 64;
constexpr int WARP_BINS = 2048;            // histogram bins: digits of up to 11 bits

struct WarpArgs {
    const void *in;
    void *out;                 // may equal in
    long long seq_stride, row_stride;
    int k;                     // rows per sequence
    int V;
    Scale sc;
    int top_k;                 // 0: filter off
    double top_p;              // >= 1: filter off
    float fix_scale;           // weights in [0, 1] are summed as integers in units of 1 / fix_scale
    int *kept;                 // [rows] survivors per row, or nullptr
};

struct WarpLds {
    unsigned long long hist[WARP_BINS];
    unsigned long long wave_tot[WARP_WAVES];
    float wave_max[WARP_WAVES];
    int wave_kept[WARP_WAVES];
    unsigned digit;
    unsigned long long rem;
};

// Order-preserving key of an fp32 value; -0 and +0 share a key.
__device__ __forceinline__ unsigned value_key(float v)
{
    unsigned u = __float_as_uint(v);
    u = u == 0x80000000u ? 0u : u;
    return u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ unsigned long long dpp_mov_or_zero_u64(unsigned long long v)
{
    const unsigned lo = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)v, CTRL, ROW_MASK, 0xF, true);
    const unsigned hi = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)(v >> 32), CTRL, ROW_MASK, 0xF, true);
    return ((unsigned long long)hi << 32) | lo;
}
// Inclusive prefix sum over the lanes of a wave, as wave_inclusive_sum but on 64-bit integers.
__device__ __forceinline__ unsigned long long wave_inclusive_sum_u64(unsigned long long v)
{
    v += dpp_mov_or_zero_u64<0x111, 0xF>(v);
    v += dpp_mov_or_zero_u64<0x112, 0xF>(v);
    v += dpp_mov_or_zero_u64<0x114, 0xF>(v);
    v += dpp_mov_or_zero_u64<0x118, 0xF>(v);
    v += dpp_mov_or_zero_u64<0x142, 0xA>(v);
    v += dpp_mov_or_zero_u64<0x143, 0xC>(v);
    return v;
}

// Vector vi of a row through the cached path (the row is read several times): a vector wholly
// inside the row as one 16-byte load, the one at the end element by element, -inf past the end.
template <typename DT>
__device__ __forceinline__ typename RawOf<DT>::type warp_load(const DT *row, int vi, int V)
{
    typedef typename RawOf<DT>::type R;
    if ((vi + 1) * VecOf<DT>::N <= V) return *(reinterpret_cast<const R *>(row) + vi);
    return load_raw_edge(row, vi, V);
}

// f(vector index, its N values) for every vector of the row, two loads in flight per thread.
template <typename DT, typename F>
__device__ __forceinline__ void for_each_vector(const DT *row, int V, F f)
{
    constexpr int N = VecOf<DT>::N;
    const int nvec = (V + N - 1) / N;
    for (int v0 = threadIdx.x; v0 < nvec; v0 += 2 * WARP_WG) {
        const int v1 = v0 + WARP_WG;
        const bool has1 = v1 < nvec;
        const typename RawOf<DT>::type r0 = warp_load<DT>(row, v0, V);
        const typename RawOf<DT>::type r1 = has1 ? warp_load<DT>(row, v1, V) : r0;
        float z[N];
        unpack<DT>(r0, z);
        f(v0, z);
        if (has1) {
            unpack<DT>(r1, z);
            f(v1, z);
        }
    }
}

struct CountMeasure {
    __device__ __forceinline__ unsigned long long operator()(float) const { return 1ull; }
};
struct MassMeasure {
    float m;
    Scale sc;
    float fix_scale;
    __device__ __forceinline__ unsigned long long operator()(float z) const
    {
        return (unsigned long long)(exp2_raw(scaled_diff(z, m, sc)) * fix_scale);
    }
};

// Radix select, going down from the largest key, over the keys >= floor_key of a row: the key v
// with   measure(keys > v) < target <= measure(keys >= v).
// With frac >= 0 the target is max(1, frac * total measure) (total taken from the first digit's
// histogram).  If the total falls short of the target the lowest key (keep everything) results.
// Every thread of the workgroup must call it; the result is uniform.
template <typename DT, typename Measure>
__device__ unsigned select_key(const DT *row, int V, unsigned floor_key, Measure measure,
                               unsigned long long target, double frac, WarpLds &L)
{
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    unsigned prefix = 0;
    int done = 0;                           // key bits fixed so far
#pragma unroll 1
    for (int pass = 0; pass < 3; ++pass) {
        const int bits = pass < 2 ? 11 : 10;
        const int shift = 32 - done - bits;
        const unsigned mask = (1u << bits) - 1u;
        L.hist[tid] = 0ull;
        L.hist[tid + WARP_WG] = 0ull;
        __syncthreads();
        for_each_vector<DT>(row, V, [&](int, const float(&z)[VecOf<DT>::N]) {
#pragma unroll
            for (int e = 0; e < VecOf<DT>::N; ++e) {
                const unsigned key = value_key(z[e]);
                const bool match = done == 0 || (key >> (32 - done)) == prefix;
                if (key >= floor_key && match) atomicAdd(&L.hist[(key >> shift) & mask], measure(z[e]));
            }
        });
        __syncthreads();
        // thread t owns the bins 2047 - 2t and 2046 - 2t: highest digits first
        const int b0 = WARP_BINS - 1 - 2 * tid, b1 = b0 - 1;
        const unsigned long long m0 = L.hist[b0], m1 = L.hist[b1];
        const unsigned long long incl = wave_inclusive_sum_u64(m0 + m1);
        if (lane == 63) L.wave_tot[wave] = incl;
        if (tid == 0) {
            L.digit = 0u;
            L.rem = 0ull;
        }
        __syncthreads();
        unsigned long long above = incl - (m0 + m1), total = 0ull;
#pragma unroll
        for (int w = 0; w < WARP_WAVES; ++w) {
            const unsigned long long t = L.wave_tot[w];
            above += w < wave ? t : 0ull;
            total += t;
        }
        if (pass == 0 && frac >= 0.0) {
            target = (unsigned long long)llrint(frac * (double)total);
            target = target ? target : 1ull;
        }
        if (above < target && target <= above + m0) {
            L.digit = (unsigned)b0;
            L.rem = target - above;
        } else if (above + m0 < target && target <= above + m0 + m1) {
            L.digit = (unsigned)b1;
            L.rem = target - (above + m0);
        }
        __syncthreads();
        const unsigned digit = L.digit;
        const unsigned long long rem = L.rem;
        if (rem == 0ull) return 0u;          // total < target: nothing to cut
        prefix = (prefix << bits) | digit;
        target = rem;
        done += bits;             // (digit, rem are rewritten only after two more barriers)
    }
    return prefix;
}

template <typename DT> struct StoreBits;
template <> struct StoreBits<float> {
    static __device__ __forceinline__ void one(float *p, float z) { *p = z; }
    static __device__ __forceinline__ void vec(float *p, const float (&z)[4])
    {
        f32x4 r;
        r.x = z[0]; r.y = z[1]; r.z = z[2]; r.w = z[3];
        *reinterpret_cast<f32x4 *>(p) = r;
    }
};
// 16-bit storage: the fp32 values came from the storage type, so converting back is exact.
template <> struct StoreBits<bf16> {
    static __device__ __forceinline__ uint32_t bits(float z) { return __float_as_uint(z) >> 16; }
};
template <> struct StoreBits<f16> {
    static __device__ __forceinline__ uint32_t bits(float z)
    {
        return (uint32_t)__builtin_bit_cast(unsigned short, (_Float16)z);
    }
};
template <typename DT>
__device__ __forceinline__ void store_one(DT *p, float z)
{
    if constexpr (VecOf<DT>::N == 4) StoreBits<DT>::one(p, z);
    else p->bits = (uint16_t)StoreBits<DT>::bits(z);
}
template <typename DT>
__device__ __forceinline__ void store_vec(DT *p, const float (&z)[VecOf<DT>::N])
{
    if constexpr (VecOf<DT>::N == 4) {
        StoreBits<DT>::vec(p, z);
    } else {
        u32x4 r;
        r.x = StoreBits<DT>::bits(z[0]) | (StoreBits<DT>::bits(z[1]) << 16);
        r.y = StoreBits<DT>::bits(z[2]) | (StoreBits<DT>::bits(z[3]) << 16);
        r.z = StoreBits<DT>::bits(z[4]) | (StoreBits<DT>::bits(z[5]) << 16);
        r.w = StoreBits<DT>::bits(z[6]) | (StoreBits<DT>::bits(z[7]) << 16);
        *reinterpret_cast<u32x4 *>(p) = r;
    }
}

// grid (rows), WARP_WG threads.
template <typename DT>
__global__ __launch_bounds__(WARP_WG) void k_warp(WarpArgs a)
{
    constexpr int N = VecOf<DT>::N;
    __shared__ WarpLds L;
    const int y = blockIdx.x, b = y / a.k, j = y - b * a.k;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const long long off = (long long)b * a.seq_stride + (long long)j * a.row_stride;
    const DT *row = static_cast<const DT *>(a.in) + off;
    DT *dst = static_cast<DT *>(a.out) + off;
    const int V = a.V;

    unsigned tau = 0u;                      // keep keys >= tau
    if (a.top_k > 0 && a.top_k < V)
        tau = select_key<DT>(row, V, 0u, CountMeasure{}, (unsigned long long)a.top_k, -1.0, L);
    if (a.top_p < 1.0) {
        float m = neg_inf();
        for_each_vector<DT>(row, V, [&](int, const float(&z)[N]) { m = vmax(m, tree_max<N>(z)); });
        m = wave_max(m);
        if (lane == 0) L.wave_max[wave] = m;
        __syncthreads();
        m = L.wave_max[0];
#pragma unroll
        for (int w = 1; w < WARP_WAVES; ++w) m = vmax(m, L.wave_max[w]);
        const unsigned tau_p = select_key<DT>(row, V, tau, MassMeasure{m, a.sc, a.fix_scale}, 0ull, a.top_p, L);
        tau = tau_p > tau ? tau_p : tau;
    }

    int kept = 0;
    for_each_vector<DT>(row, V, [&](int vi, const float(&z)[N]) {
        float o[N];
#pragma unroll
        for (int e = 0; e < N; ++e) {
            const bool keep = value_key(z[e]) >= tau;
            o[e] = keep ? z[e] : neg_inf();
            kept += (keep && vi * N + e < V) ? 1 : 0;
        }
        if ((vi + 1) * N <= V) {
            store_vec<DT>(dst + (long long)vi * N, o);
        } else {
            for (int e = 0; e < N && vi * N + e < V; ++e) store_one<DT>(dst + (long long)vi * N + e, o[e]);
        }
    });
    if (a.kept) {
        kept = wave_reduce(kept, OpSum{});
        if (lane == 0) L.wave_kept[wave] = kept;
        __syncthreads();
        if (tid == 0) {
            int n = 0;
#pragma unroll
            for (int w = 0; w < WARP_WAVES; ++w) n += L.wave_kept[w];
            a.kept[y] = n;
        }
    }
}

}  // namespace svip

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
// order in which workgroup threads reach the histogram.  One workgroup owns a row.  Only the first
// digit is histogrammed over the whole row; the keys of the bin it selects go into a list in LDS
// and the other digits are found there.  Every sweep over the row is a read from memory (the rows
// in flight exceed L2), so the sweeps are few: count + maximum, mass + candidates, candidates of
// the nucleus bin if it is another one, masked copy.  A small top_k skips the histograms: a pivot
// from a sample, one sweep for the candidates above it (which also writes the output when that
// is a different buffer), everything else on the list.
#pragma once
#include "row_math.h"

namespace svip {

constexpr int WARP_WG = 1024;              // threads of the workgroup that owns a row
constexpr int WARP_WAVES = WARP_WG / 64;
constexpr int WARP_BINS = 2048;            // histogram bins: digits of up to 11 bits
constexpr int WARP_CAP = 8192;             // keys of one first-digit bin that fit the candidate list
constexpr int DIGIT1_SHIFT = 21;           // first digit = top 11 bits of the key

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
    int no_shortcut;           // always take the histogram path (for tests and measurements)
};

struct WarpLds {
    unsigned long long hist[WARP_BINS];    // mass per first digit
    unsigned long long sub[WARP_BINS];     // measure per later digit while a bin is refined
    unsigned cnt[WARP_BINS];               // keys per first digit
    unsigned list[WARP_CAP];               // the keys of one first-digit bin
    unsigned long long wave_tot[WARP_WAVES];
    float wave_max[WARP_WAVES];
    int wave_kept[WARP_WAVES];
    unsigned digit;
    unsigned n_list;
    unsigned long long rem;
    unsigned long long acc;
};

// Order-preserving key of an fp32 value (-0 and +0 share a key) and the value of a key.
__device__ __forceinline__ unsigned value_key(float v)
{
    unsigned u = __float_as_uint(v);
    u = u == 0x80000000u ? 0u : u;
    return u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}
__device__ __forceinline__ float key_value(unsigned key)
{
    return __uint_as_float(key ^ ((key >> 31) ? 0x80000000u : 0xFFFFFFFFu));
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

// f(vector index, its N values) for every vector of the row, U loads in flight per thread.
template <typename DT, int U = 4, typename F>
__device__ __forceinline__ void for_each_vector(const DT *row, int V, F f)
{
    constexpr int N = VecOf<DT>::N;
    const int nvec = (V + N - 1) / N;
    for (int v0 = threadIdx.x; v0 < nvec; v0 += U * WARP_WG) {
        typename RawOf<DT>::type r[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int v = v0 + u * WARP_WG;
            r[u] = warp_load<DT>(row, v < nvec ? v : v0, V);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int v = v0 + u * WARP_WG;
            if (v < nvec) {
                float z[N];
                unpack<DT>(r[u], z);
                f(v, z);
            }
        }
    }
}

// Sources of candidate keys: the whole row, or the list of one first-digit bin.  f(key, value).
template <typename DT>
struct RowSource {
    const DT *row;
    int V;
    template <typename F>
    __device__ __forceinline__ void for_each(F f) const
    {
        for_each_vector<DT>(row, V, [&](int, const float(&z)[VecOf<DT>::N]) {
#pragma unroll
            for (int e = 0; e < VecOf<DT>::N; ++e) f(value_key(z[e]), z[e]);
        });
    }
};
struct ListSource {
    const unsigned *list;
    unsigned n;
    template <typename F>
    __device__ __forceinline__ void for_each(F f) const
    {
        for (unsigned i = threadIdx.x; i < n; i += WARP_WG) f(list[i], key_value(list[i]));
    }
};

struct CountMeasure {
    __device__ __forceinline__ unsigned long long operator()(float) const { return 1ull; }
};
struct MassMeasure {
    float m;
    Scale sc;
    float fix_hi;              // fix_scale / 2^32
    // w * fix_scale truncated to an integer; fix_scale = 2^s with s >= 32.  The float is split at
    // 2^32 (both parts convert exactly), which is cheaper than a 64-bit conversion.
    __device__ __forceinline__ unsigned long long operator()(float z) const
    {
        const float t = exp2_raw(scaled_diff(z, m, sc)) * fix_hi;          // = w * 2^(s - 32), < 2^13
        const unsigned hi = (unsigned)t;
        const unsigned lo = (unsigned)(__builtin_amdgcn_fractf(t) * 4294967296.0f);
        return ((unsigned long long)hi << 32) | lo;
    }
};

// Going down from the highest digit over a histogram h[WARP_BINS] in LDS (filled and barriered
// by the caller): the digit d with  sum(h above d) < target <= sum(h at and above d),  and
// rem = target - sum(h above d), the share of the target that falls inside d.  With frac >= 0
// the target is max(1, frac * sum(h)).  rem == 0: the histogram's total falls short of the target.
// Every thread of the workgroup must call it; the result is uniform.
struct Crossing {
    unsigned digit;
    unsigned long long rem;
};
template <typename T>
__device__ __forceinline__ Crossing crossing(const T *h, unsigned long long target, double frac, WarpLds &L)
{
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    // thread t owns the bins 2047 - 2t and 2046 - 2t: highest digits first
    const int b0 = WARP_BINS - 1 - 2 * tid, b1 = b0 - 1;
    const unsigned long long m0 = h[b0], m1 = h[b1];
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
    if (frac >= 0.0) {
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
    Crossing c;
    c.digit = L.digit;
    c.rem = L.rem;
    __syncthreads();                         // the next call rewrites digit, rem and wave_tot
    return c;
}

// Remaining digits of a select (11, 11 and 10 bits, most significant first) over the candidates of
// src at or above floor_key that carry `prefix` in their top `done` bits (done = 0: all, three
// digits; done = 11: inside first-digit bin `prefix`, two digits): the key v among them with
//   measure(candidates > v) < target <= measure(candidates >= v).
template <typename Src, typename Measure>
__device__ __forceinline__ unsigned select_digits(const Src &src, unsigned floor_key, Measure measure, unsigned prefix, int done,
                                  unsigned long long target, WarpLds &L)
{
    const int tid = threadIdx.x;
#pragma unroll 1
    while (done < 32) {
        const int bits = done < 22 ? 11 : 10;
        const int shift = 32 - done - bits;
        const unsigned mask = (1u << bits) - 1u;
        L.sub[tid] = 0ull;
        L.sub[tid + WARP_WG] = 0ull;
        __syncthreads();
        src.for_each([&](unsigned key, float z) {
            if (key >= floor_key && (done == 0 || (key >> (32 - done)) == prefix))
                atomicAdd(&L.sub[(key >> shift) & mask], measure(z));
        });
        __syncthreads();
        const Crossing c = crossing(L.sub, target, -1.0, L);
        prefix = (prefix << bits) | c.digit;
        if (c.rem == 0ull) return prefix << shift;         // the candidates' measure falls short of the target
        target = c.rem;
        done += bits;
    }
    return prefix;
}
template <typename Src, typename Measure>
__device__ __forceinline__ unsigned refine(const Src &src, unsigned floor_key, Measure measure, unsigned d1,
                           unsigned long long target, WarpLds &L)
{
    return select_digits(src, floor_key, measure, d1, 11, target, L);
}

// Sum over the workgroup of one 64-bit value per thread (uniform result; uses L.acc).
__device__ __forceinline__ unsigned long long wg_sum_u64(unsigned long long mine, WarpLds &L)
{
    if (threadIdx.x == 0) L.acc = 0ull;
    __syncthreads();
    mine = wave_reduce(mine, OpSum{});
    if ((threadIdx.x & 63) == 0 && mine) atomicAdd(&L.acc, mine);
    __syncthreads();
    const unsigned long long r = L.acc;
    __syncthreads();
    return r;
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

// Shortcut for a small top_k: a pivot from a sample of the row (one vector per thread), aimed at
// about three times top_k keys above it; one sweep puts every key >= pivot into L.list.  If at
// least top_k keys arrive and all of them fit, the list holds the row's largest keys, the row
// maximum among them, and both thresholds follow from the list alone -- with the same integer
// arithmetic as the histogram path, hence the same result.
// With `fused` (output is not the input, top_k <= 1024) the same sweep already writes the output:
// -inf below the pivot, the logit itself at and above it, and the list also keeps the candidates'
// indices (4096 of each); afterwards only the candidates below the final threshold are overwritten,
// so the row is read once.
// Returns 0: nothing decided (the sample misjudged the row; the caller takes the histogram path,
// which rewrites the whole output), 1: *tau_out is the threshold, 2: output and *kept_out are done.
template <typename DT, bool fused>
__device__ __forceinline__ int small_k_shortcut(const DT *row, DT *dst, int V, const WarpArgs &a, bool P,
                                             unsigned *tau_out, int *kept_out, WarpLds &L)
{
    constexpr int N = VecOf<DT>::N;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int nvec = (V + N - 1) / N;
    const int nsamp = nvec < WARP_WG ? nvec : WARP_WG;            // sampled vectors
    constexpr unsigned cap = fused ? WARP_CAP / 2 : WARP_CAP;
    const long long want = 3ll * a.top_k * ((long long)nsamp * N) / V + 8;
    if (a.top_k > (int)cap / 4 || want > (long long)nsamp * N / 4) return 0;
    if (tid < nsamp) {
        // sixteen evenly spaced runs of 64 consecutive vectors: whole cache lines, spread over the row
        const int vi = nvec <= WARP_WG ? tid : (int)((long long)(tid >> 6) * (nvec - 64) / 15) + (tid & 63);
        float z[N];
        unpack<DT>(warp_load<DT>(row, vi, V), z);
#pragma unroll
        for (int e = 0; e < N; ++e) L.list[tid * N + e] = value_key(z[e]);
    }
    __syncthreads();
    const ListSource sample{L.list, (unsigned)(nsamp * N)};
    const unsigned pivot = select_digits(sample, 0u, CountMeasure{}, 0u, 0, (unsigned long long)want, L);
    if (tid == 0) L.n_list = 0u;
    __syncthreads();
    for_each_vector<DT, 2>(row, V, [&](int vi, const float(&z)[N]) {
        float o[N];
#pragma unroll
        for (int e = 0; e < N; ++e) {
            const unsigned key = value_key(z[e]);
            o[e] = key >= pivot ? z[e] : neg_inf();
            if (key >= pivot) {
                const unsigned i = atomicAdd(&L.n_list, 1u);
                if (i < cap) {
                    L.list[i] = key;
                    if (fused) L.list[cap + i] = (unsigned)(vi * N + e);
                }
            }
        }
        if (fused) {
            if ((vi + 1) * N <= V) {
                store_vec<DT>(dst + (long long)vi * N, o);
            } else {
                #pragma unroll
                for (int e = 0; e < N; ++e)
                    if (vi * N + e < V) store_one<DT>(dst + (long long)vi * N + e, o[e]);
            }
        }
    });
    __syncthreads();
    const unsigned n = L.n_list;
    __syncthreads();
    if (n < (unsigned)a.top_k || n > cap) return 0;
    const ListSource ls{L.list, n};
    unsigned tau = select_digits(ls, 0u, CountMeasure{}, 0u, 0, (unsigned long long)a.top_k, L);
    if (P) {
        float m = neg_inf();
        ls.for_each([&](unsigned, float z) { m = vmax(m, z); });
        m = wave_max(m);
        if (lane == 0) L.wave_max[wave] = m;
        __syncthreads();
        m = L.wave_max[0];
#pragma unroll
        for (int w = 1; w < WARP_WAVES; ++w) m = vmax(m, L.wave_max[w]);
        const MassMeasure mass{m, a.sc, a.fix_scale * (1.0f / 4294967296.0f)};
        unsigned long long mine = 0ull;
        ls.for_each([&](unsigned key, float z) { mine += key >= tau ? mass(z) : 0ull; });
        const unsigned long long Zk = wg_sum_u64(mine, L);
        unsigned long long target = (unsigned long long)llrint(a.top_p * (double)Zk);
        target = target ? target : 1ull;
        if (Zk >= target) {
            const unsigned tau_p = select_digits(ls, tau, mass, 0u, 0, target, L);
            tau = tau_p > tau ? tau_p : tau;
        }
    }
    *tau_out = tau;
    if (!fused) return 1;
    // the sweep's stores are complete (every barrier since waited for them): drop the candidates below tau
    unsigned long long kept = 0ull;
    for (unsigned i = tid; i < n; i += WARP_WG) {
        const unsigned idx = L.list[cap + i];
        if (idx < (unsigned)V) {
            if (L.list[i] >= tau) kept += 1ull;
            else store_one<DT>(dst + idx, neg_inf());
        }
    }
    *kept_out = (int)wg_sum_u64(kept, L);
    return 2;
}

// The keys of first-digit bin d1 into L.list (the caller has checked that they fit).
template <typename DT>
__device__ __forceinline__ void collect(const RowSource<DT> &rs, unsigned d1, WarpLds &L)
{
    if (threadIdx.x == 0) L.n_list = 0u;
    __syncthreads();
    rs.for_each([&](unsigned key, float) {
        if ((key >> DIGIT1_SHIFT) == d1) {
            const unsigned i = atomicAdd(&L.n_list, 1u);
            if (i < (unsigned)WARP_CAP) L.list[i] = key;
        }
    });
    __syncthreads();
}

// grid (rows), WARP_WG threads.
template <typename DT>
__global__ __launch_bounds__(WARP_WG, 8) void k_warp(WarpArgs a)
{
    constexpr int N = VecOf<DT>::N;
    __shared__ WarpLds L;
    const int y = blockIdx.x, b = y / a.k, j = y - b * a.k;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const long long off = (long long)b * a.seq_stride + (long long)j * a.row_stride;
    const DT *row = static_cast<const DT *>(a.in) + off;
    DT *dst = static_cast<DT *>(a.out) + off;
    const int V = a.V;

    const bool K = a.top_k > 0 && a.top_k < V, P = a.top_p < 1.0;
    const RowSource<DT> rs{row, V};
    unsigned tau = 0u;                      // keep keys >= tau
    int kept = 0;
    int decided = 0;
    if (K && !a.no_shortcut)
        decided = a.in != a.out && a.top_k <= WARP_CAP / 8
                      ? small_k_shortcut<DT, true>(row, dst, V, a, P, &tau, &kept, L)
                      : small_k_shortcut<DT, false>(row, dst, V, a, P, &tau, &kept, L);
    if (decided == 0 && (K || P)) {
        // sweep 1: keys per first digit (top-k), row maximum (reference of the top-p weights)
        float m = neg_inf();
        unsigned d_k = 0u;
        unsigned long long k_rem = 0ull;
        if (K) {
            L.cnt[tid] = 0u;
            L.cnt[tid + WARP_WG] = 0u;
            __syncthreads();
        }
        for_each_vector<DT>(row, V, [&](int, const float(&z)[N]) {
            if (P) m = vmax(m, tree_max<N>(z));
            if (K) {
#pragma unroll
                for (int e = 0; e < N; ++e) atomicAdd(&L.cnt[value_key(z[e]) >> DIGIT1_SHIFT], 1u);
            }
        });
        if (P) {
            m = wave_max(m);
            if (lane == 0) L.wave_max[wave] = m;
        }
        __syncthreads();
        if (P) {
            m = L.wave_max[0];
#pragma unroll
            for (int w = 1; w < WARP_WAVES; ++w) m = vmax(m, L.wave_max[w]);
        }
        if (K) {
            const Crossing c = crossing(L.cnt, (unsigned long long)a.top_k, -1.0, L);
            d_k = c.digit;
            k_rem = c.rem;
        }
        const MassMeasure mass{m, a.sc, a.fix_scale * (1.0f / 4294967296.0f)};

        // sweep 2: mass per first digit from d_k upwards (top-p), the keys of bin d_k (top-k)
        const bool listA = K && L.cnt[d_k] <= (unsigned)WARP_CAP;
        if (P) {
            L.hist[tid] = 0ull;
            L.hist[tid + WARP_WG] = 0ull;
        }
        if (tid == 0) L.n_list = 0u;
        __syncthreads();
        if (P || listA) {
            rs.for_each([&](unsigned key, float z) {
                const unsigned d = key >> DIGIT1_SHIFT;
                if (P && d >= d_k) atomicAdd(&L.hist[d], mass(z));
                if (listA && d == d_k) {
                    const unsigned i = atomicAdd(&L.n_list, 1u);
                    if (i < (unsigned)WARP_CAP) L.list[i] = key;
                }
            });
        }
        __syncthreads();
        const ListSource ls{L.list, listA ? L.n_list : 0u};
        if (K) tau = listA ? refine(ls, 0u, CountMeasure{}, d_k, k_rem, L) : refine(rs, 0u, CountMeasure{}, d_k, k_rem, L);
        if (P) {
            if (K) {
                // bin d_k counts only with its keys >= tau
                if (tid == 0) L.acc = 0ull;
                __syncthreads();
                unsigned long long mine = 0ull;
                const auto add = [&](unsigned key, float z) {
                    if ((key >> DIGIT1_SHIFT) == d_k && key >= tau) mine += mass(z);
                };
                if (listA) ls.for_each(add);
                else rs.for_each(add);
                mine = wave_reduce(mine, OpSum{});
                if (lane == 0 && mine) atomicAdd(&L.acc, mine);
                __syncthreads();
                if (tid == 0) L.hist[d_k] = L.acc;
                __syncthreads();
            }
            const Crossing c = crossing(L.hist, 0ull, a.top_p, L);
            unsigned tau_p = 0u;
            if (c.rem != 0ull) {
                if (K && c.digit == d_k) {
                    tau_p = listA ? refine(ls, tau, mass, d_k, c.rem, L) : refine(rs, tau, mass, d_k, c.rem, L);
                } else {
                    // sweep 3; a bin too crowded for the list is refined by sweeps over the row instead
                    const bool fits = !K || L.cnt[c.digit] <= (unsigned)WARP_CAP;
                    if (fits) collect<DT>(rs, c.digit, L);
                    if (fits && L.n_list <= (unsigned)WARP_CAP) {
                        const ListSource lp{L.list, L.n_list};
                        tau_p = refine(lp, tau, mass, c.digit, c.rem, L);
                    } else {
                        tau_p = refine(rs, tau, mass, c.digit, c.rem, L);
                    }
                }
            }
            tau = tau_p > tau ? tau_p : tau;
        }
    }

    if (decided == 2) {
        if (a.kept && tid == 0) a.kept[y] = kept;
        return;
    }
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
            #pragma unroll
                for (int e = 0; e < N; ++e)
                    if (vi * N + e < V) store_one<DT>(dst + (long long)vi * N + e, o[e]);
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

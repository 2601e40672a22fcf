// Per-row building blocks of the SVIP kernels: 128-bit logit loads, the scaled exponential,
// streaming softmax statistics of a row slice, and the in-slice inverse-CDF search.
//
// Geometry.  A row of V logits is cut into vectors of 16 bytes (8 bf16 or fp16 / 4 fp32), chunks of 64
// consecutive vectors (what one wave reads with one load: 1 KiB contiguous), tiles of WG consecutive
// vectors (four chunks; one vector per thread of a workgroup), and `ns` slices of `tps` consecutive
// tiles.  The streaming passes give a slice to a workgroup; the draft statistics give it to a wave.
//
// Arithmetic.  With c = log2(e)/T split into two fp32 parts, a logit z contributes
// exp2((z - m) * c) relative to the running maximum m (draft statistics: the subtraction comes
// first, so the maximum has weight exactly 1), exp2(z * c - ref) relative to a reference next to
// m * c (the logsumexp-only pass of verification, two fused multiply-adds per logit), or
// exp2(z * c - L) with L = logsumexp * log2(e) (probabilities).  The split keeps the rounding of c
// from biasing every term of a row in the same direction.  Per-element work is fp32 (v_exp_f32);
// everything that combines partial sums is fp64.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "wave_ops.h"

namespace svip {

constexpr int WG = 256;              // threads per workgroup
constexpr int NWAVE = WG / 64;
constexpr int MAX_SLICES = 64;       // a wave merges one slice per lane
constexpr int LOCATE_UNROLL = 4;     // tiles per batch of the inverse-CDF search over a whole slice
constexpr int TILE_MASSES = 4;       // slices of at most this many tiles also report the mass of every tile
constexpr float X_FLOOR = -200.0f;   // exp2 of anything below is 0 in fp32; also squashes NaN from -inf logits

struct bf16 { uint16_t bits; };   // storage types: the bits only, widened to fp32 on load
struct f16 { uint16_t bits; };
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <typename DT> struct VecOf;
template <> struct VecOf<float> { static constexpr int N = 4; };
template <> struct VecOf<bf16> { static constexpr int N = 8; };
template <> struct VecOf<f16> { static constexpr int N = 8; };

struct Geo {
    int V;        // logits per row
    int ntiles;   // ceil(ceil(V / N) / WG)
    int ns;       // slices per row, <= MAX_SLICES
    int tps;      // tiles per slice, ns * tps >= ntiles
};

struct Scale {
    float c_hi, c_lo;   // log2(e) / T as nearest float + remainder
    float c_dn, c_up;   // the same constant as a float strictly below it + a positive remainder
    double c;
    double inv_T;
};

__device__ __forceinline__ float neg_inf() { return -__builtin_inff(); }
__device__ __forceinline__ float exp2_raw(float x) { return __builtin_amdgcn_exp2f(x); }

// v_max_f32 / v_max3_f32 issued directly.  The instructions return the other operand when
// one is NaN; going through fmaxf() instead makes the compiler quiet every input first
// (one more instruction per logit).
__device__ __forceinline__ float vmax(float a, float b)
{
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ float vmax3(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// Raw 16-byte vector of a row: loaded first, unpacked to fp32 later, so that a batch of
// loads is in flight before the first use.
template <typename DT> struct RawOf;
template <> struct RawOf<float> { typedef f32x4 type; };
template <> struct RawOf<bf16> { typedef u32x4 type; };
template <> struct RawOf<f16> { typedef u32x4 type; };

// Unchecked load of vector vi: every element must lie inside the row.
template <typename DT>
__device__ __forceinline__ typename RawOf<DT>::type load_raw(const DT *row, int vi)
{
    typedef typename RawOf<DT>::type R;
    return __builtin_nontemporal_load(reinterpret_cast<const R *>(row) + vi);
}

// Element-wise load of a vector that straddles or lies past the end of the row: elements at or
// beyond V read as -inf and nothing past the row is touched.
__device__ __forceinline__ f32x4 load_raw_edge(const float *row, int vi, int V)
{
    const int base = vi * 4;
    f32x4 r;
    r.x = base + 0 < V ? row[base + 0] : neg_inf();
    r.y = base + 1 < V ? row[base + 1] : neg_inf();
    r.z = base + 2 < V ? row[base + 2] : neg_inf();
    r.w = base + 3 < V ? row[base + 3] : neg_inf();
    return r;
}
__device__ __forceinline__ u32x4 load_raw_edge(const bf16 *row, int vi, int V)
{
    const int base = vi * 8;
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const uint32_t lo = base + 2 * e < V ? row[base + 2 * e].bits : 0xFF80u;       // bf16 -inf
        const uint32_t hi = base + 2 * e + 1 < V ? row[base + 2 * e + 1].bits : 0xFF80u;
        w[e] = lo | (hi << 16);
    }
    u32x4 r;
    r.x = w[0]; r.y = w[1]; r.z = w[2]; r.w = w[3];
    return r;
}

__device__ __forceinline__ u32x4 load_raw_edge(const f16 *row, int vi, int V)
{
    const int base = vi * 8;
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const uint32_t lo = base + 2 * e < V ? row[base + 2 * e].bits : 0xFC00u;       // fp16 -inf
        const uint32_t hi = base + 2 * e + 1 < V ? row[base + 2 * e + 1].bits : 0xFC00u;
        w[e] = lo | (hi << 16);
    }
    u32x4 r;
    r.x = w[0]; r.y = w[1]; r.z = w[2]; r.w = w[3];
    return r;
}

// Checked load for the last, partial tile of a row: a vector that lies wholly inside the row
// is read as one 16-byte load, only the vector at the end of the row goes element by element.
template <typename DT>
__device__ __forceinline__ typename RawOf<DT>::type load_raw_checked(const DT *row, int vi, int V)
{
    if ((vi + 1) * VecOf<DT>::N <= V) return load_raw<DT>(row, vi);
    return load_raw_edge(row, vi, V);
}

// Widening of one 16-byte vector to fp32 (exact for every storage type).
template <typename DT>
__device__ __forceinline__ void unpack(const typename RawOf<DT>::type &v, float (&z)[VecOf<DT>::N]);
template <>
__device__ __forceinline__ void unpack<float>(const f32x4 &v, float (&z)[4])
{
    z[0] = v.x; z[1] = v.y; z[2] = v.z; z[3] = v.w;
}
template <>
__device__ __forceinline__ void unpack<bf16>(const u32x4 &v, float (&z)[8])
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        z[2 * e] = __uint_as_float(w[e] << 16);
        z[2 * e + 1] = __uint_as_float(w[e] & 0xFFFF0000u);
    }
}
__device__ __forceinline__ float half_bits_to_float(uint32_t bits)
{
    return (float)__builtin_bit_cast(_Float16, (unsigned short)bits);
}
template <>
__device__ __forceinline__ void unpack<f16>(const u32x4 &v, float (&z)[8])
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        z[2 * e] = half_bits_to_float(w[e] & 0xFFFFu);
        z[2 * e + 1] = half_bits_to_float(w[e] >> 16);
    }
}

// One stored logit widened to fp32 (exact).  Kept apart from the load so that a caller can request a value and
// only look at it later.
__device__ __forceinline__ float widen(float v) { return v; }
__device__ __forceinline__ float widen(bf16 v) { return __uint_as_float((uint32_t)v.bits << 16); }
__device__ __forceinline__ float widen(f16 v) { return half_bits_to_float(v.bits); }
template <typename DT>
__device__ __forceinline__ float load_one(const DT *row, int i) { return widen(row[i]); }
// The value unchanged, but not looked at (so not waited for) before this point of the program.
__device__ __forceinline__ float not_before_here(float v)
{
    asm volatile("" : "+v"(v));
    return v;
}
__device__ __forceinline__ bf16 not_before_here(bf16 v)
{
    unsigned t = v.bits;
    asm volatile("" : "+v"(t));
    v.bits = (uint16_t)t;
    return v;
}
__device__ __forceinline__ f16 not_before_here(f16 v)
{
    unsigned t = v.bits;
    asm volatile("" : "+v"(t));
    v.bits = (uint16_t)t;
    return v;
}

template <int N>
__device__ __forceinline__ float tree_sum(const float (&v)[N])
{
    if constexpr (N == 4) {
        return (v[0] + v[1]) + (v[2] + v[3]);
    } else {
        static_assert(N == 8, "vector width");
        return ((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7]));
    }
}
template <int N>
__device__ __forceinline__ float tree_max(const float (&v)[N])
{
    if constexpr (N == 4) {
        return vmax(vmax3(v[0], v[1], v[2]), v[3]);
    } else {
        static_assert(N == 8, "vector width");
        return vmax3(vmax3(v[0], v[1], v[2]), vmax3(v[3], v[4], v[5]), vmax(v[6], v[7]));
    }
}

// (z - m) * c in exp2 units, floored (see X_FLOOR).  The subtraction comes first so that the
// row maximum itself gets exactly 0 (weight exactly 1): a one-hot row then has S = 1, t = 0 and
// H = 0 without rounding, and small entropies keep their relative accuracy.
__device__ __forceinline__ float scaled_diff(float z, float m, const Scale &sc)
{
    const float d = z - m;
    return vmax(fmaf(d, sc.c_hi, d * sc.c_lo), X_FLOOR);
}

// Probability-like weight exp2(z * c - L), L given as fp32 hi + lo.
struct ExpRef {
    float c_hi, c_lo, L_hi, L_lo;
    // log2 of the weight, floored (see X_FLOOR)
    __device__ __forceinline__ float arg(float z) const
    {
        const float x = fmaf(z, c_hi, -L_hi) + fmaf(z, c_lo, -L_lo);
        return vmax(x, X_FLOOR);
    }
    __device__ __forceinline__ float operator()(float z) const { return exp2_raw(arg(z)); }
};
__device__ __forceinline__ ExpRef make_exp_ref(const Scale &sc, double L)
{
    ExpRef r;
    r.c_hi = sc.c_hi;
    r.c_lo = sc.c_lo;
    r.L_hi = (float)L;
    r.L_lo = (float)(L - (double)r.L_hi);
    return r;
}

// Softmax statistics of a slice relative to its own maximum m:
//   S = sum exp2((z - m) c),   t = sum exp2((z - m) c) * (z - m) c    (t only if WITH_T).
struct Partial {
    float m;
    int idx;       // smallest index holding m (only filled by the argmax-tracking variants)
    double S;
    double t;
};

// Smallest token index among the batch's elements equal to v (-1 if none); z[u] is vector
// (t0 + u) * TW + (thread index modulo TW) of the row: TW = WG for a workgroup reading tile by tile,
// TW = 64 for a wave reading chunk by chunk.
template <int N, int NU, int TW = WG>
__device__ __forceinline__ int first_equal(const float (&z)[NU][N], float v, int t0)
{
    int found = -1;
#pragma unroll
    for (int u = NU - 1; u >= 0; --u) {
#pragma unroll
        for (int e = N - 1; e >= 0; --e)
            if (z[u][e] == v) found = ((t0 + u) * TW + (int)(threadIdx.x & (TW - 1))) * N + e;
    }
    return found;
}

// One batch of NU vectors per thread folded into the thread's running statistics: m, the maximum
// of its logits so far; with x = (z - m) c and w = exp2(x):  ones = the number of weights that are
// exactly 1 in fp32 (the maximum, its ties, anything within one rounding of it), S = the sum of all
// other weights, t = sum w x.  Keeping the ones out of the fp32 sum is what keeps small entropies
// accurate: next to a 1 the tail of a confident row (1e-4 and less) would lose its low bits.  The
// loop sums fract(w) (fract(1) = 0, fract(w) = w below 1) beside w itself; the difference of the two
// batch sums is the batch's count of ones up to rounding far below 1/2.  With ARG, idx follows the
// smallest index that holds m: it moves only when the maximum strictly increases, so earlier equal
// values keep it; the batch is one wave's chunks c0 .. c0 + NU - 1 (64 vectors each).
template <int N, int NU, bool ARG>
__device__ __forceinline__ void accumulate(const float (&z)[NU][N], float &m, float &ones, float &S, float &t,
                                           const Scale &sc, int &idx, int c0)
{
    float mb = tree_max<N>(z[0]);
#pragma unroll
    for (int u = 1; u < NU; ++u) mb = vmax(mb, tree_max<N>(z[u]));
    if (mb > m) {
        if (ARG) idx = first_equal<N, NU, 64>(z, mb, c0);
        if (m != neg_inf()) {
            const float xd = scaled_diff(m, mb, sc);
            const float f = exp2_raw(xd);
            if (f < 1.0f) {                     // the old maximum becomes an ordinary term
                const float all = S + ones;
                t = f * fmaf(xd, all, t);
                S = f * all;
                ones = 0.f;
            }                                   // else: still weight 1 at fp32 resolution, nothing moves
        }
        m = mb;
    }
    const float mref = (m == neg_inf()) ? 0.f : m;
    float Wb = 0.f, Sb = 0.f, tb = 0.f;
#pragma unroll
    for (int u = 0; u < NU; ++u) {
        float w[N], fr[N], wx[N];
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const float x = scaled_diff(z[u][i], mref, sc);
            w[i] = exp2_raw(x);
            wx[i] = w[i] * x;
            fr[i] = __builtin_amdgcn_fractf(w[i]);
        }
        // group sums are formed first, then added to the batch sum: the running sums only
        // ever take one addition per batch
        Wb += tree_sum<N>(w);
        Sb += tree_sum<N>(fr);
        tb += tree_sum<N>(wx);
    }
    ones += rintf(Wb - Sb);
    S += Sb;
    t += tb;
}

// LDS of one workgroup combination (each field is written once, so two barriers suffice).
struct CombineLds {
    float m[NWAVE];
    double S[NWAVE];
};

// ---- logsumexp only (statistics pass of verification) -----------------------------------------
//
// S = sum exp2(z c - ref) relative to a reference ref = float(m c_dn) of the running maximum m,
// with the exponent formed by two fused multiply-adds, x = fma(z, c_up, fma(z, c_dn, -ref)):
// two rounded operations per logit, no subtraction, and no floor -- because c_up > 0, a logit
// of -inf gives x = -inf and weight 0 without passing through inf - inf.  The exact value of
// ref does not matter (it cancels in ref + log2 S); it only has to sit next to m c so that the
// largest weight is about 1.
template <int N, int NU>
__device__ __forceinline__ void accumulate_lse(const float (&z)[NU][N], float &m, float &ref, float &S,
                                               const Scale &sc)
{
    float mb = tree_max<N>(z[0]);
#pragma unroll
    for (int u = 1; u < NU; ++u) mb = vmax(mb, tree_max<N>(z[u]));
    if (mb > m) {
        const float nref = mb * sc.c_dn;
        if (m != neg_inf()) S *= exp2_raw(ref - nref);
        m = mb;
        ref = nref;
    }
    const float nr = (m == neg_inf()) ? 0.f : -ref;
    float Sb = 0.f;
#pragma unroll
    for (int u = 0; u < NU; ++u) {
        float e[N];
#pragma unroll
        for (int i = 0; i < N; ++i) e[i] = exp2_raw(fmaf(z[u][i], sc.c_up, fmaf(z[u][i], sc.c_dn, nr)));
        Sb += tree_sum<N>(e);
    }
    S += Sb;
}

template <typename DT, int NU>
__device__ __forceinline__ void lse_batch(const DT *row, int t0, float &m, float &ref, float &S, const Scale &sc)
{
    constexpr int N = VecOf<DT>::N;
    typename RawOf<DT>::type raw[NU];
#pragma unroll
    for (int u = 0; u < NU; ++u) raw[u] = load_raw<DT>(row, (t0 + u) * WG + (int)threadIdx.x);
    float z[NU][N];
#pragma unroll
    for (int u = 0; u < NU; ++u) unpack<DT>(raw[u], z[u]);
    accumulate_lse<N, NU>(z, m, ref, S, sc);
}

// (ref, S) of tiles [tb, te) of one row with S = sum exp2(z c - ref): Partial::m holds ref (log2
// units), Partial::S the sum; m = -inf marks a slice without finite logits.  Batches hold 32
// logits per thread (4 bf16 vectors or 8 fp32 vectors): small enough for 8 waves per SIMD.
// Result valid in thread 0.
template <typename DT>
__device__ __forceinline__ Partial slice_lse(const DT *row, int V, int tb, int te, const Scale &sc,
                                             CombineLds &lds)
{
    constexpr int N = VecOf<DT>::N, NB = 32 / N;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    float m = neg_inf(), ref = neg_inf(), S = 0.f;
    const int fe = min(te, V / (WG * N));
    int t0 = tb;
    for (; t0 + NB <= fe; t0 += NB) lse_batch<DT, NB>(row, t0, m, ref, S, sc);
    if (NB == 8 && t0 + 4 <= fe) { lse_batch<DT, 4>(row, t0, m, ref, S, sc); t0 += 4; }
    if (t0 + 2 <= fe) { lse_batch<DT, 2>(row, t0, m, ref, S, sc); t0 += 2; }
    if (t0 + 1 <= fe) { lse_batch<DT, 1>(row, t0, m, ref, S, sc); t0 += 1; }
    if (t0 < te) {
        float z[1][N];
        unpack<DT>(load_raw_checked(row, t0 * WG + tid, V), z[0]);
        accumulate_lse<N, 1>(z, m, ref, S, sc);
    }
    // workgroup: largest reference first, then every thread rescales to it (a difference of two
    // floats, exact) and the sums are added in fp64
    const float rw = wave_max(ref);
    if (lane == 0) lds.m[wave] = rw;
    __syncthreads();
    float rg = lds.m[0];
#pragma unroll
    for (int w = 1; w < NWAVE; ++w) rg = vmax(rg, lds.m[w]);
    double Sd = (m != neg_inf()) ? (double)S * (double)exp2_raw(ref - rg) : 0.0;
    Sd = wave_sum(Sd);
    if (lane == 0) lds.S[wave] = Sd;
    __syncthreads();
    Partial p;
    p.m = rg;
    p.idx = -1;
    p.S = 0.0;
    p.t = 0.0;
    if (tid == 0) {
#pragma unroll
        for (int w = 0; w < NWAVE; ++w) p.S += lds.S[w];
    }
    return p;
}

// ---- argmax only (greedy verification): no exponentials, a pure stream ---------------------
//
// A 64-bit key orders (value descending, index ascending): the fp32 value mapped to an unsigned
// integer that sorts the same way, then 0xFFFFFFFF - index.  The largest key of a row is its
// first maximum.
__device__ __forceinline__ unsigned long long argmax_key(float v, int idx)
{
    unsigned u = __float_as_uint(v);
    u = u == 0x80000000u ? 0u : u;                  // -0 and +0 compare equal: one key for both
    u ^= (u >> 31) ? 0xFFFFFFFFu : 0x80000000u;
    return ((unsigned long long)u << 32) | (unsigned long long)(0xFFFFFFFFu - (unsigned)idx);
}
__device__ __forceinline__ int argmax_index(unsigned long long key) { return (int)(0xFFFFFFFFu - (unsigned)key); }

template <typename DT, int NU>
__device__ __forceinline__ void argmax_batch(const DT *row, int t0, float &m, int &idx)
{
    constexpr int N = VecOf<DT>::N;
    typename RawOf<DT>::type raw[NU];
#pragma unroll
    for (int u = 0; u < NU; ++u) raw[u] = load_raw<DT>(row, (t0 + u) * WG + (int)threadIdx.x);
    float z[NU][N];
#pragma unroll
    for (int u = 0; u < NU; ++u) unpack<DT>(raw[u], z[u]);
    float mb = tree_max<N>(z[0]);
#pragma unroll
    for (int u = 1; u < NU; ++u) mb = vmax(mb, tree_max<N>(z[u]));
    if (mb > m || idx < 0) {
        m = mb;
        idx = first_equal<N, NU>(z, mb, t0);
    }
}

// Key of the first maximum of tiles [tb, te) of a row; result in thread 0.
template <typename DT>
__device__ __forceinline__ unsigned long long slice_argmax(const DT *row, int V, int tb, int te,
                                                           unsigned long long *lds /* >= NWAVE */)
{
    constexpr int N = VecOf<DT>::N;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    float m = neg_inf();
    int idx = -1;
    const int fe = min(te, V / (WG * N));
    int t0 = tb;
    constexpr int NB = 32 / N;                  // 32 logits per thread and batch, as in slice_lse
    for (; t0 + NB <= fe; t0 += NB) argmax_batch<DT, NB>(row, t0, m, idx);
    if (NB == 8 && t0 + 4 <= fe) { argmax_batch<DT, 4>(row, t0, m, idx); t0 += 4; }
    if (t0 + 2 <= fe) { argmax_batch<DT, 2>(row, t0, m, idx); t0 += 2; }
    if (t0 + 1 <= fe) { argmax_batch<DT, 1>(row, t0, m, idx); t0 += 1; }
    if (t0 < te) {
        float z[1][N];
        unpack<DT>(load_raw_checked(row, t0 * WG + tid, V), z[0]);
        const float mb = tree_max<N>(z[0]);
        // elements past the end of the row read as -inf: only take the tile if it beats what we have
        if (mb > m || (idx < 0 && t0 * WG * N + tid * N < V)) {
            m = mb;
            idx = first_equal<N, 1>(z, mb, t0);
        }
    }
    unsigned long long key = idx >= 0 ? argmax_key(m, idx) : 0ull;
    key = wave_reduce(key, OpMax{});
    if (lane == 0) lds[wave] = key;
    __syncthreads();
    unsigned long long best = lds[0];
#pragma unroll
    for (int w = 1; w < NWAVE; ++w) best = lds[w] > best ? lds[w] : best;
    return best;
}

// ---- in-slice inverse CDF ---------------------------------------------------------
//
// Finds the smallest token index i inside tiles [tb, te) whose inclusive prefix of weights,
// counted from the start of the slice, exceeds `target`.  The search works on batches of
// LOCATE_UNROLL tiles: per-vector group sums in fp32, then lanes -> waves -> tiles in fp64.
// The first crossing is found without LDS atomics: each wave ballots "my prefix exceeds the
// target" per tile, posts its first hit, and the workgroup takes the smallest post.  If
// rounding leaves no crossing, the last index of the slice with positive weight is returned
// (or -1 if the slice has no mass).  All threads of the workgroup must call; the result
// (token, its weight) is uniform.
struct LocateLds {
    double wtot[NWAVE][LOCATE_UNROLL];      // sized for the widest batch
    int wkey[NWAVE];
    int wlast[NWAVE];
    int tok;
    float w;
};
constexpr int NOKEY = 0x7FFFFFFF;

// One batch: w[u] holds the weights of vector (t0 + u) * WG + tid, all zero for absent tiles.
// Returns true (uniform) if the crossing lies in this batch (L.tok / L.w are then set);
// otherwise adds the batch mass to `run`.
// `report` (optional): called by the one thread that finds the token, with (token, its weight); the token is
// then not passed through LDS and the batch ends one barrier earlier.  `lds_is_free`: no thread can still be
// reading L from an earlier use, so the batch need not wait before writing it.
struct NoReport {
    static constexpr bool active = false;
    __device__ __forceinline__ void operator()(int, float) const {}
};
template <int N, int LU, typename Report = NoReport>
__device__ __forceinline__ bool locate_batch(const float (&w)[LU][N], int t0, int ntile,
                                             double target, double &run, int &last, LocateLds &L,
                                             bool lds_is_free = false, Report report = Report())
{
    static_assert(LU <= LOCATE_UNROLL, "batch wider than the LDS block");
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    float g[LU];
    double incl[LU];
#pragma unroll
    for (int u = 0; u < LU; ++u) {
        g[u] = tree_sum<N>(w[u]);
        incl[u] = 0.0;
    }
#pragma unroll
    for (int u = 0; u < LU; ++u)
        if (u < ntile) incl[u] = wave_inclusive_sum((double)g[u]);
    if (!lds_is_free) __syncthreads();    // LDS of an earlier batch / caller is free again
    if (lane == 63) {
#pragma unroll
        for (int u = 0; u < LU; ++u) L.wtot[wave][u] = incl[u];
    }
    __syncthreads();
    double base = run;
    double excl[LU];
    int wkey = NOKEY;
#pragma unroll
    for (int u = 0; u < LU; ++u) {
        double before = 0.0, tot = 0.0;
#pragma unroll
        for (int w2 = 0; w2 < NWAVE; ++w2) {
            const double x = L.wtot[w2][u];
            if (w2 < wave) before += x;
            tot += x;
        }
        const double P = base + before + incl[u];
        excl[u] = base + before + (incl[u] - (double)g[u]);
        const unsigned long long hit = __ballot(g[u] > 0.f && P > target);
        if (wkey == NOKEY && hit) wkey = u * WG + wave * 64 + (__ffsll((long long)hit) - 1);
        base += tot;
    }
    if (lane == 0) L.wkey[wave] = wkey;
    __syncthreads();
    int key = L.wkey[0];
#pragma unroll
    for (int w2 = 1; w2 < NWAVE; ++w2) key = min(key, L.wkey[w2]);
    if (key == NOKEY) {
#pragma unroll
        for (int u = 0; u < LU; ++u) {
#pragma unroll
            for (int e = 0; e < N; ++e)
                if (w[u][e] > 0.f) last = max(last, ((t0 + u) * WG + tid) * N + e);
        }
        run = base;
        return false;
    }
    if ((key & (WG - 1)) == tid) {
        const int ku = key / WG;
#pragma unroll
        for (int u = 0; u < LU; ++u) {
            if (u == ku) {
                double C = excl[u];
                int pick = -1, lastpos = -1;
#pragma unroll
                for (int e = 0; e < N; ++e) {
                    C += (double)w[u][e];
                    if (w[u][e] > 0.f) {
                        lastpos = e;
                        if (pick < 0 && C > target) pick = e;
                    }
                }
                if (pick < 0) pick = lastpos;
                float wv = 0.f;
#pragma unroll
                for (int e = 0; e < N; ++e)
                    if (e == pick) wv = w[u][e];
                if constexpr (Report::active) {
                    report(((t0 + u) * WG + tid) * N + pick, wv);
                } else {
                    L.tok = ((t0 + u) * WG + tid) * N + pick;
                    L.w = wv;
                }
            }
        }
    }
    if constexpr (!Report::active) __syncthreads();
    return true;
}

// No crossing anywhere: the last index with positive weight (-1 if none), uniform.
template <int N, typename WF>
__device__ __forceinline__ void locate_fallback(WF &wf, int last, LocateLds &L)
{
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wl = wave_reduce(last, OpMax{});
    __syncthreads();
    if (lane == 0) L.wlast[wave] = wl;
    __syncthreads();
    int best = L.wlast[0];
#pragma unroll
    for (int w2 = 1; w2 < NWAVE; ++w2) best = max(best, L.wlast[w2]);
    if (tid == 0) {
        float wv = 0.f;
        if (best >= 0) {
            float one[N];
            wf.weights(wf.load_checked(best / N), one);
#pragma unroll
            for (int e = 0; e < N; ++e)
                if (e == best % N) wv = one[e];
        }
        L.tok = best;
        L.w = wv;
    }
    __syncthreads();
}

// Search over tiles [tb, te), LU tiles per batch, with the weights fetched by the functor wf:
// wf.load(vi) / wf.load_checked(vi) fetch the raw vector(s) and wf.weights(pack, w) turns them
// into the N weights of vector vi (fp32, >= 0).
struct NoHook {
    __device__ __forceinline__ void operator()() const {}
};

// `between` runs once, after the loads of the first batch have been issued and before their data is
// used: work that does not depend on the search hides behind the memory round trip there.
template <int N, int LU, typename WF, typename Hook = NoHook, typename Report = NoReport>
__device__ __forceinline__ int locate_in_slice(WF &wf, int tb, int te, double target, LocateLds &L,
                                               float *weight_out, Hook between = Hook(), bool lds_is_free = false,
                                               Report report = Report())
{
    const int tid = threadIdx.x;
    const int fe = min(te, wf.V / (WG * N));   // end of the tiles wholly inside the row
    double run = 0.0;
    int last = -1;
    bool found = false;
    for (int t0 = tb; t0 < te && !found; t0 += LU) {
        float w[LU][N];
        typename WF::Pack pk[LU];
#pragma unroll
        for (int u = 0; u < LU; ++u)
            if (t0 + u < fe) pk[u] = wf.load((t0 + u) * WG + tid);
        if (t0 == tb) between();
#pragma unroll
        for (int u = 0; u < LU; ++u) {
            if (t0 + u < fe) {
                wf.weights(pk[u], w[u]);
            } else if (t0 + u < te) {
                wf.weights(wf.load_checked((t0 + u) * WG + tid), w[u]);
            } else {
#pragma unroll
                for (int e = 0; e < N; ++e) w[u][e] = 0.f;
            }
        }
        found = locate_batch<N, LU, Report>(w, t0, min(LU, te - t0), target, run, last, L, lds_is_free && t0 == tb, report);
    }
    if constexpr (Report::active) {       // the finder has reported; without a crossing thread 0 reports the fallback
        if (!found) {
            locate_fallback<N>(wf, last, L);
            if (tid == 0) report(L.tok, L.w);
        }
        return 0;
    } else {
        if (!found) locate_fallback<N>(wf, last, L);
        *weight_out = L.w;
        return L.tok;
    }
}

}  // namespace svip

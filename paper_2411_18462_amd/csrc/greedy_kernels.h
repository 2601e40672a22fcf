// Kernels of svip_verify_greedy (Algorithms 3 and 5).
#pragma once
#include "exchange.h"
#include "kernel_args.h"

namespace svip {

// ---- greedy verification (Algorithms 3 and 5) ------------------------------------------------

struct GreedyArgs {
    const void *target;
    long long seq_t, row_stride;
    const int *pos;   // optional [B]: row j of sequence b is trace row pos[b] + j
    const unsigned char *skip;   // optional [B]: sequences to leave alone
    int B, k;
    Geo geo;
    const int *tokens;
    const int *draft_len;
    int *n_accepted;
    int *next_token;
    unsigned long long *keys;    // [B (k+1)][ns] first-maximum keys
    unsigned *flags;
};

// One wave: lane = position.  argmax of target row j from its slice keys; position j < draft_len is accepted iff
// that argmax is the draft token; a ballot finds the first failure r, and the correction (or, if none
// failed, the bonus token) is the argmax of row r.
__device__ __forceinline__ void accept_greedy_sequence(const GreedyArgs &a, int b, int lane)
{
    const int graw = a.draft_len[b];
    const int g = clamp_len(graw, a.k);
    if (graw != g && lane == 0) atomicOr(a.flags, (unsigned)SVIP_FLAG_BAD_DRAFT_LEN);
    int r = -1, next = -1;
    for (int j0 = 0; j0 <= g && r < 0; j0 += 64) {
        const int j = j0 + lane;
        int am = -1;
        bool reject = false;
        if (j <= g) {
            const unsigned long long *kr = a.keys + ((size_t)b * (a.k + 1) + j) * a.geo.ns;
            unsigned long long best = 0ull;
            for (int s0 = 0; s0 < a.geo.ns; s0 += 8) {          // eight loads in flight at a time
                unsigned long long kk[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) kk[u] = s0 + u < a.geo.ns ? kr[s0 + u] : 0ull;
#pragma unroll
                for (int u = 0; u < 8; ++u) best = kk[u] > best ? kk[u] : best;
            }
            am = argmax_index(best);
            if (j < g) {
                const int x = a.tokens[(size_t)b * a.k + j];
                if (x < 0 || x >= a.geo.V) atomicOr(a.flags, (unsigned)SVIP_FLAG_BAD_TOKEN);
                reject = am != x;
            }
        }
        const unsigned long long rej = __ballot(reject);
        if (rej) {
            const int first = __ffsll((long long)rej) - 1;
            r = j0 + first;
            next = read_lane(am, first);
        } else if (g - j0 < 64) {
            r = g;
            next = read_lane(am, g - j0);
        }
    }
    if (lane == 0) {
        a.n_accepted[b] = r;
        a.next_token[b] = next;
    }
}

// grid (sequences * (k+1) * slices): first maximum of slice s of target row (b, j), j <= draft_len[b].
template <typename DT>
__global__ __launch_bounds__(WG) void k_argmax(GreedyArgs a)
{
    __shared__ unsigned long long lds[NWAVE];
    const int y = blockIdx.x / a.geo.ns, s = blockIdx.x - y * a.geo.ns;
    const int b = y / (a.k + 1), j = y - b * (a.k + 1);
    if (a.skip && a.skip[b]) return;
    const int g = clamp_len(a.draft_len[b], a.k);
    if (j > g) return;
    const DT *row = static_cast<const DT *>(a.target) + row_offset(a, a.seq_t, b, j);
    const int tb = s * a.geo.tps, te = min(tb + a.geo.tps, a.geo.ntiles);
    const unsigned long long key = slice_argmax<DT>(row, a.geo.V, tb, te, lds);
    if (threadIdx.x == 0) a.keys[(size_t)y * a.geo.ns + s] = key;
}

// grid (sequences), one wave.
__global__ __launch_bounds__(64) void k_accept_greedy(GreedyArgs a)
{
    if (a.skip && a.skip[blockIdx.x]) return;
    accept_greedy_sequence(a, blockIdx.x, threadIdx.x);
}

}  // namespace svip

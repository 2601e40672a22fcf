// Workspace layout and kernel argument blocks shared by the kernels of libsvip.so.
#pragma once
#include "../../include/svip.h"
#include "row_math.h"

namespace svip {

// ---- workspace layout ----------------------------------------------------------------

struct SeqRec {          // what the acceptance test hands to the residual kernel, one per sequence
    double Lp;           // logsumexp(target row r) * log2(e)
    double Lq;           // logsumexp(draft row r) * log2(e) (residual mode only)
    int r;               // target row to sample from (first rejection, or draft_len for a bonus)
    int resid;           // 1: residual of row r, 0: bonus from row r
};

struct Workspace {
    unsigned *flags;     // sticky device-data flags
    unsigned *tickets;   // END of the ticket counters (see ticket()): they grow downwards from here
    SeqRec *rec;         // [B]
    double *mass;        // [B][slices of the residual pass] tile masses (ResidSlot), verification only
    Partial *part;       // [stat rows][ns] slice statistics
};

constexpr int MAX_BATCH = 1 << 20;               // sequences per call (grids are one-dimensional)
constexpr size_t HEADER_BYTES = 256;
#ifndef SVIP_TICKET_STRIDE
#define SVIP_TICKET_STRIDE 16
#endif
constexpr int TICKETS_PER_ROW = SVIP_TICKET_STRIDE;   // words between the counters of consecutive rows
__host__ __device__ inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

static size_t ws_rec_bytes(int B) { return align256((size_t)B * sizeof(SeqRec)); }
static size_t ws_mass_bytes(int B, int slices) { return align256((size_t)B * slices * 2 * TILE_MASSES * sizeof(double)); }
static size_t ws_ticket_bytes(int B) { return align256((size_t)B * TICKETS_PER_ROW * sizeof(unsigned)); }

// Layout: flag word | records | slice masses | slice statistics ...            ... ticket counters.
// The counters sit at the END of the workspace (the given size rounded down to 256 bytes) and counter
// t of row b lies TICKETS_PER_ROW * b + t + 1 words below that end, whatever the batch size of the call: regions at the
// front never reach them (every call checks front + counters <= size), so they keep the zeros that
// svip_workspace_reset wrote and that every kernel restores, also when calls of different batch sizes
// share a workspace.
static Workspace carve(void *ws, size_t bytes, int B, int mass_slices)
{
    char *p = static_cast<char *>(ws);
    Workspace w;
    w.flags = reinterpret_cast<unsigned *>(p);
    w.tickets = reinterpret_cast<unsigned *>(p + (bytes & ~(size_t)255));
    p += HEADER_BYTES;
    w.rec = reinterpret_cast<SeqRec *>(p);
    p += ws_rec_bytes(B);
    w.mass = reinterpret_cast<double *>(p);
    p += ws_mass_bytes(B, mass_slices);
    w.part = reinterpret_cast<Partial *>(p);
    return w;
}
enum { TICKET_RESID = 0 };
__device__ __forceinline__ unsigned *ticket(unsigned *tickets_end, int b, int t)
{
    return tickets_end - ((size_t)b * TICKETS_PER_ROW + t + 1);
}

// ---- kernel arguments ------------------------------------------------------------------

struct DraftArgs {
    const void *logits;
    long long row_stride;   // between the rows of consecutive sequences
    const int *pos;         // optional [B]: sequence b reads trace row pos[b] + step_j of its own trace
    long long pos_stride;   // elements between consecutive trace rows (used with pos)
    const int *cap;         // optional [B]: per-sequence limit on the draft length (at most k_max)
    int B;
    Geo geo;
    Scale sc;
    float h;
    int step_j, k_max;
    const float *u;
    const unsigned char *stop_in;
    int *token;
    float *entropy;
    float *q_tok;
    double *lse;
    unsigned char *stop;
    int *draft_len;
    long long io_stride;
    Partial *part;          // [B][ns] records of the row's waves
    int rows_by_xcd;        // k_draft_stats: workgroup -> (row, records) mapping, see there
    unsigned div, div_magic;  // its one division, by div: n / div = div == 1 ? n : umulhi(n, div_magic), exact for n * div < 2^32
};

struct VerifyArgs {
    const void *target;
    const void *draft;
    long long seq_t, seq_d, row_stride;
    const int *pos;   // optional [B]: row j of sequence b is trace row pos[b] + j
    const unsigned char *skip;   // optional [B]: sequences to leave alone (no read, no write, no ticket)
    int B, k;
    int kd;        // draft rows per sequence in the statistics pass: k if the draft logsumexps are recomputed, else 0
    int bonus;     // 1: the statistics pass also covers target row draft_len (verification), 0: rows j < draft_len only
    Geo geo;       // slicing of the statistics pass
    long long stat_items;   // statistics rows * slices: the work items of the statistics pass
    Geo geo_s;     // slicing of the sampling pass (slices of at most LOCATE_UNROLL tiles when possible)
    Scale sc;
    const int *tokens;
    const int *draft_len;
    const double *draft_lse;
    const float *u_accept;
    const float *u_resample;
    int *n_accepted;
    int *next_token;
    float *accept_prob;
    Workspace ws;
};

__device__ __forceinline__ int clamp_len(int g, int k) { return g < 0 ? 0 : (g > k ? k : g); }

// Element offset of row j of sequence b (seq_stride between sequences, optional trace position).
template <typename A>
__device__ __forceinline__ long long row_offset(const A &a, long long seq_stride, int b, int j)
{
    return (long long)b * seq_stride + (long long)(j + (a.pos ? a.pos[b] : 0)) * a.row_stride;
}

}  // namespace svip

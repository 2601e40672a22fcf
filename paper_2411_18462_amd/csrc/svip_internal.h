// Calls shared by the sources of libsvip.so: the public entry points of include/svip.h and the
// decoding loop are thin wrappers around these.  Compared with the public signatures they add
// the optional per-sequence trace positions and draft-length limits the loop needs.
#pragma once
#include <stddef.h>

#include "../../include/svip.h"

namespace svip {

struct DraftCall {
    bool greedy;                 // argmax instead of a draw (u_sample unused)
    const void *logits;          // device
    int dtype;
    int B, V;
    long long row_stride;        // elements between the rows (or traces) of consecutive sequences
    const int *pos;              // device [B] or nullptr: sequence b reads trace row pos[b] + step_j
    long long pos_stride;        // elements between consecutive trace rows
    const int *cap;              // device [B] or nullptr: per-sequence draft-length limit (<= k_max)
    float temperature, h;
    int step_j, k_max;
    const float *u_sample;
    const unsigned char *stop_in;
    int *token_out;
    float *entropy_out;
    float *q_tok_out;
    double *lse_out;
    unsigned char *stop_out;
    int *draft_len_out;
    long long io_stride;
    void *workspace;
    size_t workspace_bytes;
    void *stream;
};

struct VerifyCall {
    bool greedy;                 // Algorithms 3 and 5: only the target, tokens and lengths are used
    const void *target, *draft;  // device
    int dtype;
    int B, k_max, V;
    long long seq_stride_t, seq_stride_d, row_stride;
    const int *pos;              // device [B] or nullptr: row j of sequence b is trace row pos[b] + j
    const unsigned char *skip;   // device [B] or nullptr: sequences with skip[b] != 0 are neither read nor written
    float temperature;
    const int *draft_tokens;
    const int *draft_len;
    const double *draft_lse;
    const float *u_accept;
    const float *u_resample;
    int *n_accepted_out;
    int *next_token_out;
    float *accept_prob_out;
    void *workspace;
    size_t workspace_bytes;
    void *stream;
};

svip_status draft_step_call(const DraftCall &c);
svip_status verify_call(const VerifyCall &c);

}  // namespace svip

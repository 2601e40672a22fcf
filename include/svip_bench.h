/*
 * svip_bench.h -- hooks for benchmarks and experiments.  NOT part of the product ABI of svip.h:
 * nothing here changes what the calls compute, and a serving path has no use for it.  The library
 * allocates nothing here either: timing events are created, owned and read by the caller.
 *
 * Process-wide state without locks: not for concurrent use from several threads.
 */
#ifndef SVIP_BENCH_H
#define SVIP_BENCH_H

#include "svip.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Kernel classes whose launches can carry timing events. */
enum {
    SVIP_BENCH_K_DRAFT_STATS = 0,   /* statistics launch of svip_draft_step / svip_draft_step_greedy */
    SVIP_BENCH_K_VERIFY_STATS = 1,  /* statistics pass of svip_verify (argmax pass of svip_verify_greedy) */
    SVIP_BENCH_K_RESID = 2,         /* residual / bonus pass of svip_verify */
    SVIP_BENCH_K_ACCEPT = 3,        /* acceptance tests and first-rejection scan of svip_verify / svip_verify_greedy */
    SVIP_BENCH_K_DRAFT_FINISH = 4,  /* second launch of a draft step: the rows' merge, stop test and token */
    SVIP_BENCH_KERNEL_CLASSES = 5
};

/*
 * From now on, launch number i (i = 0 .. n_pairs - 1) of a kernel of class `kernel_class` carries
 * start_events[i] and stop_events[i] (host arrays of hipEvent_t, created by the caller with timing
 * enabled) attached to the launch itself (hipExtLaunchKernel), so that they take the kernel's own
 * begin and end on the call's stream; later launches carry none.  The arrays must stay valid until
 * they are replaced or removed (n_pairs = 0).  The caller synchronises and reads the events.
 */
svip_status svip_bench_time_kernels(int kernel_class, void *const *start_events /* host */,
                                    void *const *stop_events /* host */, int n_pairs);

/* Event pairs of that class handed out so far (-1: no such class). */
int svip_bench_events_used(int kernel_class);

/*
 * Launch-shape overrides for experiments; 0 in a field (and NULL for the whole struct) means the
 * library's own choice.  Workspace sizes (svip_workspace_bytes, svip_workspace_needed) never depend
 * on these: a forced shape that needs more workspace than the call was given is rejected with
 * SVIP_ERR_WORKSPACE.  Results do not depend on the shape beyond the rounding of partial sums.
 */
typedef struct svip_bench_tuning {
    int draft_slices;          /* records (waves) per row of the draft step */
    int stats_slices;          /* slices per row of the statistics / argmax pass of verification */
    int resid_slices;          /* slices per row of the residual pass */
    int pair_slices;           /* slices per row of the second pass of svip_pair_stats */
    int even_tiles_per_slice;  /* 1: do not round the streaming passes' slices up to an odd number of tiles */
    int warp_no_shortcut;      /* 1: svip_warp_logits always takes the histogram path */
    int stats_workgroups;      /* workgroups of the statistics pass of svip_verify: fewer than its items makes each loop over several */
} svip_bench_tuning;
svip_status svip_bench_set_tuning(const svip_bench_tuning *tuning /* host, or NULL */);

/*
 * Reference launches for stating floors and peaks next to the calls' own figures.
 *
 * svip_bench_empty_kernel: one launch of a kernel that does nothing (what a launch costs).
 * svip_bench_stream_read: a read-only stream over [buf, buf + bytes) (device, 16-byte aligned; bytes
 * rounded down to 16) with the access pattern of the statistics passes: 256-thread workgroups,
 * vectors_per_thread (4, 8 or 16) non-temporal 16-byte loads per thread, every vector read exactly once
 * and folded into one word per wave written to sink (device, svip_bench_stream_sink_words(bytes,
 * vectors_per_thread) unsigned words).  bytes / kernel time is the read rate this GPU sustains.
 */
svip_status svip_bench_empty_kernel(void *hip_stream);
size_t svip_bench_stream_sink_words(size_t bytes, int vectors_per_thread);
svip_status svip_bench_stream_read(const void *buf /* device */, size_t bytes, int vectors_per_thread,
                                   unsigned *sink /* device */, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SVIP_BENCH_H */

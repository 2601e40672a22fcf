"""MI355X-native hot path of SVIP (arXiv 2411.18462): thin Python binding of libsvip.so.

Every step of the path runs in the HIP kernels behind the C ABI of ``include/svip.h``; this
package only marshals torch tensors (device memory, strides, the current HIP stream) into
that ABI.  There is no CPU or PyTorch fallback: if the library has not been built, ``load()``
raises.

    import paper_2411_18462_amd as svip
    ws = svip.new_workspace(B, k_max, V)
    svip.draft_step(logits[:, j], ..., workspace=ws)      # Algorithm 1, drafting loop
    svip.verify(target, draft, ..., workspace=ws)         # Algorithm 1, verification loop
"""
from .binding import (SvipError, draft_step, load, new_workspace, verify, verify_greedy, pair_stats, warp_logits,
                      PAIR_NSTAT, PAIR_FIELDS, Loop, LoopConfig, LOOP_NSTATE, LOOP_STATE_FIELDS, workspace_bytes,
                      workspace_needed, workspace_flags, MAX_K, FLAG_BAD_TOKEN, FLAG_BAD_DRAFT_LEN,
                      bench_time_kernels, bench_events_used, bench_set_tuning, bench_empty_kernel, bench_stream_read,
                      BENCH_K_DRAFT_STATS,
                      BENCH_K_VERIFY_STATS, BENCH_K_RESID, BENCH_K_ACCEPT, BENCH_K_DRAFT_FINISH)

__all__ = ["SvipError", "draft_step", "load", "new_workspace", "verify", "verify_greedy", "pair_stats", "warp_logits",
           "PAIR_NSTAT", "PAIR_FIELDS", "Loop", "LoopConfig", "LOOP_NSTATE", "LOOP_STATE_FIELDS", "workspace_bytes",
           "workspace_needed", "workspace_flags", "MAX_K", "FLAG_BAD_TOKEN", "FLAG_BAD_DRAFT_LEN",
           "bench_time_kernels", "bench_events_used", "bench_set_tuning", "bench_empty_kernel", "bench_stream_read",
           "BENCH_K_DRAFT_STATS",
           "BENCH_K_VERIFY_STATS", "BENCH_K_RESID", "BENCH_K_ACCEPT", "BENCH_K_DRAFT_FINISH"]

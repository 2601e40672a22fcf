"""ctypes binding of libsvip.so: argument marshalling only (see include/svip.h)."""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsvip.so")
_lib = None

MAX_K = 1024
FLAG_BAD_TOKEN = 1
FLAG_BAD_DRAFT_LEN = 2
_DTYPES = {torch.float32: 0, torch.bfloat16: 1, torch.float16: 2}

# every symbol include/svip.h declares
EXPORTS = ("svip_status_string", "svip_workspace_bytes", "svip_workspace_needed", "svip_workspace_reset",
           "svip_workspace_flags", "svip_draft_step", "svip_draft_step_static", "svip_verify", "svip_draft_step_greedy",
           "svip_verify_greedy", "svip_pair_stats", "svip_warp_logits", "svip_loop_workspace_bytes", "svip_loop_init", "svip_loop_run")
# every symbol include/svip_bench.h declares (benchmark and experiment hooks, not the product ABI)
BENCH_EXPORTS = ("svip_bench_time_kernels", "svip_bench_events_used", "svip_bench_set_tuning", "svip_bench_empty_kernel",
                 "svip_bench_stream_sink_words", "svip_bench_stream_read")
BENCH_K_DRAFT_STATS, BENCH_K_VERIFY_STATS, BENCH_K_RESID, BENCH_K_ACCEPT, BENCH_K_DRAFT_FINISH = 0, 1, 2, 3, 4


class SvipError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(text)
        self.status = status


class LoopConfig(ctypes.Structure):
    """svip_loop_config of include/svip.h, field for field."""
    _fields_ = [
        ("target_trace", ctypes.c_void_p), ("draft_trace", ctypes.c_void_p), ("dtype", ctypes.c_int),
        ("B", ctypes.c_int), ("L", ctypes.c_int), ("V", ctypes.c_int),
        ("seq_stride", ctypes.c_longlong), ("row_stride", ctypes.c_longlong),
        ("temperature", ctypes.c_float), ("greedy", ctypes.c_int), ("h", ctypes.c_float),
        ("gamma0", ctypes.c_int), ("gamma_max", ctypes.c_int), ("gamma_inc", ctypes.c_int),
        ("gamma_dec", ctypes.c_int), ("n0", ctypes.c_int), ("max_new", ctypes.c_int), ("rounds", ctypes.c_int),
        ("u_sample", ctypes.c_void_p), ("u_accept", ctypes.c_void_p), ("u_resample", ctypes.c_void_p),
        ("state", ctypes.c_void_p), ("out_tokens", ctypes.c_void_p), ("out_stride", ctypes.c_longlong),
        ("round_log", ctypes.c_void_p), ("check_every", ctypes.c_int),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t), ("hip_stream", ctypes.c_void_p),
    ]


class BenchTuning(ctypes.Structure):
    """svip_bench_tuning of include/svip_bench.h, field for field."""
    _fields_ = [("draft_slices", ctypes.c_int), ("stats_slices", ctypes.c_int), ("resid_slices", ctypes.c_int),
                ("pair_slices", ctypes.c_int),
                ("even_tiles_per_slice", ctypes.c_int), ("warp_no_shortcut", ctypes.c_int), ("stats_workgroups", ctypes.c_int)]


def load():
    """Load libsvip.so (built by ``paper_2411_18462_amd.build``); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is not built; run `python -m paper_2411_18462_amd.build` "
            "(hipcc, gfx950).  There is no fallback path.")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i, ll, f, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_longlong, ctypes.c_float, ctypes.c_size_t
    lib.svip_status_string.restype = ctypes.c_char_p
    lib.svip_status_string.argtypes = [i]
    lib.svip_workspace_bytes.restype = sz
    lib.svip_workspace_bytes.argtypes = [i, i, i]
    lib.svip_workspace_reset.restype = i
    lib.svip_workspace_reset.argtypes = [vp, sz, vp]
    lib.svip_workspace_flags.restype = i
    lib.svip_workspace_flags.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_uint)]
    lib.svip_draft_step.restype = i
    lib.svip_draft_step.argtypes = [vp, i, i, i, ll, f, f, i, i, vp, vp, vp, vp, vp, vp, vp, vp, ll, vp, sz, vp]
    lib.svip_draft_step_static.restype = i
    lib.svip_draft_step_static.argtypes = [vp, i, i, i, ll, f, f, i, i, vp, vp, vp, vp, vp, vp, vp, vp, ll, vp]
    lib.svip_verify.restype = i
    lib.svip_verify.argtypes = [vp, vp, i, i, i, i, ll, ll, ll, f, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.svip_draft_step_greedy.restype = i
    lib.svip_draft_step_greedy.argtypes = [vp, i, i, i, ll, f, f, i, i, vp, vp, vp, vp, vp, vp, vp, ll, vp, sz, vp]
    lib.svip_verify_greedy.restype = i
    lib.svip_verify_greedy.argtypes = [vp, i, i, i, i, ll, ll, vp, vp, vp, vp, vp, sz, vp]
    lib.svip_pair_stats.restype = i
    lib.svip_pair_stats.argtypes = [vp, vp, i, i, i, i, ll, ll, ll, f, vp, vp, f, vp, vp, sz, vp]
    lib.svip_warp_logits.restype = i
    lib.svip_warp_logits.argtypes = [vp, vp, i, i, i, i, ll, ll, f, i, ctypes.c_double, vp, vp]
    lib.svip_workspace_needed.restype = sz
    lib.svip_workspace_needed.argtypes = [i, i, i, i, i]
    lib.svip_loop_workspace_bytes.restype = sz
    lib.svip_loop_workspace_bytes.argtypes = [i, i, i]
    lib.svip_loop_init.restype = i
    lib.svip_loop_init.argtypes = [ctypes.POINTER(LoopConfig)]
    lib.svip_loop_run.restype = i
    lib.svip_loop_run.argtypes = [ctypes.POINTER(LoopConfig), i, i, ctypes.POINTER(i), ctypes.POINTER(i)]
    lib.svip_bench_time_kernels.restype = i
    lib.svip_bench_time_kernels.argtypes = [i, ctypes.POINTER(vp), ctypes.POINTER(vp), i]
    lib.svip_bench_events_used.restype = i
    lib.svip_bench_events_used.argtypes = [i]
    lib.svip_bench_empty_kernel.restype = i
    lib.svip_bench_empty_kernel.argtypes = [vp]
    lib.svip_bench_stream_sink_words.restype = sz
    lib.svip_bench_stream_sink_words.argtypes = [sz, i]
    lib.svip_bench_stream_read.restype = i
    lib.svip_bench_stream_read.argtypes = [vp, sz, i, vp, vp]
    lib.svip_bench_set_tuning.restype = i
    lib.svip_bench_set_tuning.argtypes = [ctypes.POINTER(BenchTuning)]
    _lib = lib
    return lib


def _check(status: int):
    if status != 0:
        raise SvipError(status, load().svip_status_string(status).decode())


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _ptr(t, dtype=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    return t.data_ptr()


def _col(t, B, dtype, name, stride=None):
    """Pointer and row stride of a per-row array: a [B] tensor, possibly a column view."""
    if t is None:
        return None, stride
    if t.dim() != 1 or t.shape[0] != B:
        raise ValueError(f"{name} must have shape [{B}]")
    s = t.stride(0) if B > 1 else (stride or 1)
    if stride is not None and B > 1 and s != stride:
        raise ValueError(f"{name}: all per-row arrays must share one stride ({s} vs {stride})")
    return _ptr(t, dtype, name), s


def workspace_bytes(B: int, k_max: int, V: int) -> int:
    return int(load().svip_workspace_bytes(B, k_max, V))


def workspace_needed(call: int, dtype, B: int, k_max: int, V: int) -> int:
    """svip_workspace_needed; dtype a torch dtype, call one of the SVIP_CALL_* numbers (0..5)."""
    return int(load().svip_workspace_needed(int(call), _DTYPES[dtype], B, k_max, V))


def new_workspace(B: int, k_max: int, V: int, device="cuda", stream=None) -> torch.Tensor:
    """Allocate a workspace tensor for batches up to (B, k_max, V) and zero its flag word."""
    n = workspace_bytes(B, k_max, V)
    if n == 0:
        raise SvipError(2, "svip_workspace_bytes: bad B, k_max or V")
    ws = torch.empty(n, dtype=torch.uint8, device=device)
    _check(load().svip_workspace_reset(ws.data_ptr(), n, _stream(stream)))
    return ws


def workspace_flags(workspace: torch.Tensor, stream=None) -> int:
    out = ctypes.c_uint(0)
    _check(load().svip_workspace_flags(workspace.data_ptr(), _stream(stream), ctypes.byref(out)))
    return out.value


def draft_step(draft_logits, *, temperature, h, step_j, k_max, token_out, lse_out, stop_out, workspace=None,
               u_sample=None, greedy=False, stop_in=None, entropy_out=None, q_tok_out=None,
               draft_len_out=None, stream=None):
    """svip_draft_step, or svip_draft_step_greedy when greedy=True (then u_sample is not used), or, with
    workspace=None, svip_draft_step_static (the library's own fixed scratch; sampling only).
    draft_logits: [B, V] view (unit stride along V); u_sample, token_out, entropy_out, q_tok_out,
    lse_out: [B] tensors or column views sharing one stride; stop_in / stop_out / draft_len_out:
    contiguous [B]."""
    if draft_logits.dim() != 2 or draft_logits.stride(1) != 1:
        raise ValueError("draft_logits must be [B, V] with unit stride along V")
    B, V = draft_logits.shape
    row_stride = draft_logits.stride(0) if B > 1 else max(V, draft_logits.stride(0))
    if draft_logits.dtype not in _DTYPES:
        raise SvipError(3, "logits must be float32, bfloat16 or float16")
    if not greedy and u_sample is None:
        raise SvipError(1, "u_sample is required unless greedy=True")
    pu, ios = _col(None if greedy else u_sample, B, torch.float32, "u_sample")
    pt, ios = _col(token_out, B, torch.int32, "token_out", ios)
    pe, ios = _col(entropy_out, B, torch.float32, "entropy_out", ios)
    pq, ios = _col(q_tok_out, B, torch.float32, "q_tok_out", ios)
    pl, ios = _col(lse_out, B, torch.float64, "lse_out", ios)
    for t, n in ((stop_in, "stop_in"), (stop_out, "stop_out"), (draft_len_out, "draft_len_out")):
        if t is not None and (t.dim() != 1 or t.shape[0] != B or not t.is_contiguous()):
            raise ValueError(f"{n} must be contiguous [{B}]")
    head = (_ptr(draft_logits, None, "draft_logits"), _DTYPES[draft_logits.dtype], B, V, row_stride,
            float(temperature), float(h), int(step_j), int(k_max))
    if workspace is None:
        if greedy:
            raise ValueError("the greedy draft step needs a workspace")
        _check(load().svip_draft_step_static(
            *head, pu, _ptr(stop_in, torch.uint8, "stop_in"), pt, pe, pq, pl, _ptr(stop_out, torch.uint8, "stop_out"),
            _ptr(draft_len_out, torch.int32, "draft_len_out"), ios or 1, _stream(stream)))
        return
    tail = (_ptr(stop_in, torch.uint8, "stop_in"), pt, pe, pq, pl,
            _ptr(stop_out, torch.uint8, "stop_out"), _ptr(draft_len_out, torch.int32, "draft_len_out"),
            ios or 1, _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream))
    if greedy:
        _check(load().svip_draft_step_greedy(*head, *tail))
    else:
        _check(load().svip_draft_step(*head, pu, *tail))


def verify_greedy(target_logits, *, draft_tokens, draft_len, n_accepted_out, next_token_out, workspace,
                  stream=None):
    """svip_verify_greedy.  target_logits [B, k+1, V] (unit stride along V); draft_tokens [B, k]."""
    if target_logits.dim() != 3 or target_logits.stride(2) != 1:
        raise ValueError("target_logits must be [B, k+1, V] with unit stride along V")
    B, kp1, V = target_logits.shape
    k = kp1 - 1
    if target_logits.dtype not in _DTYPES:
        raise SvipError(3, "logits must be float32, bfloat16 or float16")
    row_stride = target_logits.stride(1)
    seq_t = target_logits.stride(0) if B > 1 else kp1 * row_stride
    for t, shape, n in ((draft_tokens, (B, k), "draft_tokens"), (draft_len, (B,), "draft_len"),
                        (n_accepted_out, (B,), "n_accepted_out"), (next_token_out, (B,), "next_token_out")):
        if tuple(t.shape) != shape or not t.is_contiguous():
            raise ValueError(f"{n} must be contiguous {list(shape)}")
    _check(load().svip_verify_greedy(
        _ptr(target_logits, None, "target_logits"), _DTYPES[target_logits.dtype], B, k, V, seq_t, row_stride,
        _ptr(draft_tokens, torch.int32, "draft_tokens"), _ptr(draft_len, torch.int32, "draft_len"),
        _ptr(n_accepted_out, torch.int32, "n_accepted_out"), _ptr(next_token_out, torch.int32, "next_token_out"),
        _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream)))


PAIR_NSTAT = 8
PAIR_FIELDS = ("beta", "kl", "hqp", "hq", "bound_oracle", "bound_bh", "bound_approx", "ratio")


def pair_stats(target_logits, draft_logits, *, temperature, draft_len, c, stats_out, workspace,
               draft_lse=None, stream=None):
    """svip_pair_stats.  target_logits [B, >=k, V] (rows j < k are used), draft_logits [B, k, V],
    stats_out contiguous float32 [B, k, PAIR_NSTAT]."""
    if target_logits.dim() != 3 or draft_logits.dim() != 3:
        raise ValueError("logits must be [B, rows, V]")
    B, k, V = draft_logits.shape
    if target_logits.shape[0] != B or target_logits.shape[1] < k or target_logits.shape[2] != V:
        raise ValueError("target_logits must be [B, >=k, V]")
    if target_logits.dtype != draft_logits.dtype or draft_logits.dtype not in _DTYPES:
        raise SvipError(3, "logits must both be float32, bfloat16 or float16")
    if target_logits.stride(2) != 1 or draft_logits.stride(2) != 1 or target_logits.stride(1) != draft_logits.stride(1):
        raise ValueError("logits need unit stride along V and a common row stride")
    row_stride = draft_logits.stride(1) if k > 1 else max(V, draft_logits.stride(1))
    seq_t = target_logits.stride(0) if B > 1 else target_logits.shape[1] * row_stride
    seq_d = draft_logits.stride(0) if B > 1 else k * row_stride
    if tuple(stats_out.shape) != (B, k, PAIR_NSTAT) or not stats_out.is_contiguous():
        raise ValueError(f"stats_out must be contiguous [{B}, {k}, {PAIR_NSTAT}]")
    if tuple(draft_len.shape) != (B,) or not draft_len.is_contiguous():
        raise ValueError(f"draft_len must be contiguous [{B}]")
    if draft_lse is not None and (tuple(draft_lse.shape) != (B, k) or not draft_lse.is_contiguous()):
        raise ValueError(f"draft_lse must be contiguous [{B}, {k}]")
    _check(load().svip_pair_stats(
        _ptr(target_logits, None, "target_logits"), _ptr(draft_logits, None, "draft_logits"),
        _DTYPES[draft_logits.dtype], B, k, V, seq_t, seq_d, row_stride, float(temperature),
        _ptr(draft_len, torch.int32, "draft_len"), _ptr(draft_lse, torch.float64, "draft_lse"), float(c),
        _ptr(stats_out, torch.float32, "stats_out"), _ptr(workspace, torch.uint8, "workspace"),
        workspace.numel(), _stream(stream)))


def warp_logits(logits, *, temperature, top_k=0, top_p=1.0, out=None, kept_out=None, stream=None):
    """svip_warp_logits.  logits [B, rows, V] (unit stride along V); out has the same shape and strides
    (default: in place).  Returns out."""
    if logits.dim() != 3 or logits.dtype not in _DTYPES:
        raise ValueError("logits must be [B, rows, V] of float32, bfloat16 or float16")
    out = logits if out is None else out
    if out.shape != logits.shape or out.stride() != logits.stride() or out.dtype != logits.dtype:
        raise ValueError("out must match logits in shape, strides and dtype")
    if logits.stride(2) != 1:
        raise ValueError("logits need unit stride along V")
    B, n, V = logits.shape
    row_stride = logits.stride(1) if n > 1 else max(V, logits.stride(1))
    seq_stride = logits.stride(0) if B > 1 else n * row_stride
    if kept_out is not None and (kept_out.numel() != B * n or not kept_out.is_contiguous()):
        raise ValueError(f"kept_out must be contiguous with {B * n} elements")
    _check(load().svip_warp_logits(
        _ptr(logits, None, "logits"), _ptr(out, None, "out"), _DTYPES[logits.dtype], B, n, V, seq_stride,
        row_stride, float(temperature), int(top_k), float(top_p), _ptr(kept_out, torch.int32, "kept_out"),
        _stream(stream)))
    return out


def verify(target_logits, draft_logits, *, temperature, draft_tokens, draft_len, u_accept,
           u_resample, n_accepted_out, next_token_out, workspace, draft_lse=None,
           accept_prob_out=None, stream=None):
    """svip_verify.  target_logits [B, k+1, V], draft_logits [B, k, V] (unit stride along V,
    equal stride along the position axis); [B, k] arrays contiguous."""
    if target_logits.dim() != 3 or draft_logits.dim() != 3:
        raise ValueError("logits must be [B, k+1, V] and [B, k, V]")
    B, kp1, V = target_logits.shape
    k = kp1 - 1
    if tuple(draft_logits.shape) != (B, k, V):
        raise ValueError(f"draft_logits must be [{B}, {k}, {V}]")
    if target_logits.dtype != draft_logits.dtype or target_logits.dtype not in _DTYPES:
        raise SvipError(3, "logits must both be float32, bfloat16 or float16")
    if target_logits.stride(2) != 1 or draft_logits.stride(2) != 1:
        raise ValueError("logits need unit stride along V")
    row_stride = target_logits.stride(1)
    if k > 1 and draft_logits.stride(1) != row_stride:
        raise ValueError("target and draft logits must share the stride along the position axis")
    seq_t = target_logits.stride(0) if B > 1 else kp1 * row_stride
    seq_d = draft_logits.stride(0) if B > 1 else k * row_stride
    for t, shape, n in ((draft_tokens, (B, k), "draft_tokens"), (draft_len, (B,), "draft_len"),
                        (draft_lse, (B, k), "draft_lse"), (u_accept, (B, k), "u_accept"),
                        (u_resample, (B,), "u_resample"), (n_accepted_out, (B,), "n_accepted_out"),
                        (next_token_out, (B,), "next_token_out"), (accept_prob_out, (B, k), "accept_prob_out")):
        if t is not None and (tuple(t.shape) != shape or not t.is_contiguous()):
            raise ValueError(f"{n} must be contiguous {list(shape)}")
    _check(load().svip_verify(
        _ptr(target_logits, None, "target_logits"), _ptr(draft_logits, None, "draft_logits"),
        _DTYPES[target_logits.dtype], B, k, V, seq_t, seq_d, row_stride, float(temperature),
        _ptr(draft_tokens, torch.int32, "draft_tokens"), _ptr(draft_len, torch.int32, "draft_len"),
        _ptr(draft_lse, torch.float64, "draft_lse"), _ptr(u_accept, torch.float32, "u_accept"),
        _ptr(u_resample, torch.float32, "u_resample"), _ptr(n_accepted_out, torch.int32, "n_accepted_out"),
        _ptr(next_token_out, torch.int32, "next_token_out"), _ptr(accept_prob_out, torch.float32, "accept_prob_out"),
        _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream)))


LOOP_NSTATE = 8
LOOP_STATE_FIELDS = ("pos", "limit", "finished", "rounds", "drafted", "accepted", "produced", "start")


class Loop:
    """The decoding loop over logit traces (svip_loop_init / svip_loop_run).  Holds the device
    buffers the configuration points to; all arithmetic and bookkeeping runs in the library."""

    def __init__(self, target_trace, draft_trace, *, temperature, h, gamma0, gamma_max, gamma_inc=0, gamma_dec=0,
                 n0=0, max_new, rounds, greedy=False, u_sample=None, u_accept=None, u_resample=None,
                 log=True, check_every=8, stream=None):
        if target_trace.dim() != 3 or target_trace.shape != draft_trace.shape:
            raise ValueError("traces must both be [B, L, V]")
        if target_trace.dtype != draft_trace.dtype or draft_trace.dtype not in _DTYPES:
            raise SvipError(3, "traces must both be float32, bfloat16 or float16")
        if target_trace.stride() != draft_trace.stride() or draft_trace.stride(2) != 1:
            raise ValueError("traces need the same strides and unit stride along V")
        B, L, V = draft_trace.shape
        dev = draft_trace.device
        self.target_trace, self.draft_trace = target_trace, draft_trace
        self.B, self.L, self.V, self.rounds, self.gamma_max = B, L, V, int(rounds), int(gamma_max)
        self.u = []
        if not greedy:
            for t, shape, n in ((u_sample, (rounds, B, gamma_max), "u_sample"), (u_accept, (rounds, B, gamma_max), "u_accept"),
                                (u_resample, (rounds, B), "u_resample")):
                if t is None or tuple(t.shape) != shape or not t.is_contiguous():
                    raise ValueError(f"{n} must be contiguous {list(shape)}")
                self.u.append(t)
        self.state = torch.zeros(B, LOOP_NSTATE, dtype=torch.int32, device=dev)
        self.out_stride = int(max_new) + int(gamma_max)
        self.out_tokens = torch.full((B, self.out_stride), -1, dtype=torch.int32, device=dev)
        self.round_log = torch.full((rounds, B, 4), -2, dtype=torch.int32, device=dev) if log else None
        n = int(load().svip_loop_workspace_bytes(B, gamma_max, V))
        if n == 0:
            raise SvipError(2, "svip_loop_workspace_bytes: bad B, gamma_max or V")
        self.workspace = torch.empty(n, dtype=torch.uint8, device=dev)
        row_stride = draft_trace.stride(1) if L > 1 else max(V, draft_trace.stride(1))
        seq_stride = draft_trace.stride(0) if B > 1 else L * row_stride
        c = LoopConfig()
        c.target_trace, c.draft_trace = _ptr(target_trace, None, "target_trace"), _ptr(draft_trace, None, "draft_trace")
        c.dtype, c.B, c.L, c.V = _DTYPES[draft_trace.dtype], B, L, V
        c.seq_stride, c.row_stride = seq_stride, row_stride
        c.temperature, c.greedy, c.h = float(temperature), int(bool(greedy)), float(h)
        c.gamma0, c.gamma_max, c.gamma_inc, c.gamma_dec = int(gamma0), int(gamma_max), int(gamma_inc), int(gamma_dec)
        c.n0, c.max_new, c.rounds = int(n0), int(max_new), int(rounds)
        if not greedy:
            c.u_sample = _ptr(u_sample, torch.float32, "u_sample")
            c.u_accept = _ptr(u_accept, torch.float32, "u_accept")
            c.u_resample = _ptr(u_resample, torch.float32, "u_resample")
        c.state, c.out_tokens, c.out_stride = self.state.data_ptr(), self.out_tokens.data_ptr(), self.out_stride
        c.round_log = self.round_log.data_ptr() if log else None
        c.check_every = int(check_every)
        c.workspace, c.workspace_bytes, c.hip_stream = self.workspace.data_ptr(), n, _stream(stream)
        self.config = c
        self.next_round = 0
        _check(load().svip_loop_init(ctypes.byref(c)))

    def run(self, max_rounds=None):
        """Runs up to max_rounds further rounds (default: all that are left); returns
        (rounds run, sequences still running).  Synchronises the stream."""
        left = self.rounds - self.next_round
        n = left if max_rounds is None else min(int(max_rounds), left)
        ran, running = ctypes.c_int(0), ctypes.c_int(0)
        _check(load().svip_loop_run(ctypes.byref(self.config), self.next_round, n, ctypes.byref(ran),
                                    ctypes.byref(running)))
        self.next_round += ran.value
        return ran.value, running.value

    def flags(self) -> int:
        return workspace_flags(self.workspace)


def bench_time_kernels(kernel_class: int, start_events, stop_events):
    """svip_bench_time_kernels: the next len(start_events) launches of that kernel class carry the given
    hipEvent_t handles (integers; created, kept alive and read by the caller).  Empty lists remove them.
    Returns the ctypes arrays, which the caller must keep alive while they are registered."""
    n = len(start_events)
    assert n == len(stop_events)
    a0 = (ctypes.c_void_p * max(n, 1))(*start_events)
    a1 = (ctypes.c_void_p * max(n, 1))(*stop_events)
    _check(load().svip_bench_time_kernels(int(kernel_class), a0, a1, n))
    return a0, a1


def bench_events_used(kernel_class: int) -> int:
    return int(load().svip_bench_events_used(int(kernel_class)))


def bench_set_tuning(**fields):
    """svip_bench_set_tuning: launch-shape overrides for experiments; no arguments = the library's own choices."""
    t = BenchTuning(**{k: int(v) for k, v in fields.items()})
    _check(load().svip_bench_set_tuning(ctypes.byref(t) if fields else None))


def bench_empty_kernel(stream=None):
    _check(load().svip_bench_empty_kernel(_stream(stream)))


def bench_stream_read(buf: torch.Tensor, sink: torch.Tensor = None, vectors_per_thread: int = 8, stream=None):
    """svip_bench_stream_read over the bytes of a contiguous device tensor; returns the sink tensor."""
    nbytes = buf.numel() * buf.element_size()
    words = int(load().svip_bench_stream_sink_words(nbytes, int(vectors_per_thread)))
    if sink is None:
        sink = torch.empty(max(words, 1), dtype=torch.int32, device=buf.device)
    assert sink.numel() >= words and sink.dtype == torch.int32 and buf.is_contiguous()
    _check(load().svip_bench_stream_read(buf.data_ptr(), nbytes, int(vectors_per_thread), sink.data_ptr(), _stream(stream)))
    return sink

"""svip_draft_step_static (the entry point that allocates nothing: its workspace is a fixed array inside the
library's device code) against svip_draft_step, through the C ABI: two calls in a row, the second with a
smaller input, must give bit-identical outputs; oversized requests are refused with a clear status."""
import numpy as np
import pytest
import torch

import svip_inputs as si

pytestmark = pytest.mark.gpu


def _outputs(B, k, dev):
    return dict(tok=torch.full((B, k), -7, dtype=torch.int32, device=dev),
                ent=torch.full((B, k), float("nan"), dtype=torch.float32, device=dev),
                q=torch.full((B, k), float("nan"), dtype=torch.float32, device=dev),
                lse=torch.full((B, k), float("nan"), dtype=torch.float64, device=dev),
                stop=torch.zeros(B, dtype=torch.uint8, device=dev), dl=torch.zeros(B, dtype=torch.int32, device=dev))


def _chain(svip, draft, us, T, h, ws):
    """k chained draft steps; ws=None takes the static entry point."""
    B, k, V = draft.shape
    o = _outputs(B, k, draft.device)
    for j in range(k):
        svip.draft_step(draft[:, j], temperature=T, h=h, step_j=j, k_max=k, u_sample=us[:, j], stop_in=o["stop"],
                        token_out=o["tok"][:, j], entropy_out=o["ent"][:, j], q_tok_out=o["q"][:, j],
                        lse_out=o["lse"][:, j], stop_out=o["stop"], draft_len_out=o["dl"], workspace=ws)
    torch.cuda.synchronize()
    return o


def test_static_scratch_entry_point_matches_the_workspace_one(svip):
    dev = torch.device("cuda:0")
    cases = [("cfg3", list(range(24)), {}), ("cfg2", [0, 1, 2, 3, 4], {"k": 5, "T": 0.7})]     # larger first, then smaller
    for name, rows, over in cases:
        w = si.workload(name, **over)
        d = si.gen_batch(w, seed=3, rows=rows)
        draft, us = d["draft"].to(dev), d["u_sample"].to(dev)
        B, k, V = draft.shape
        print(f"static scratch: {name} B={B} k={k} V={V} {draft.dtype}", flush=True)
        ref = _chain(svip, draft, us, w.T, w.h, svip.new_workspace(B, k, V))
        got = _chain(svip, draft, us, w.T, w.h, None)
        for key in ref:
            assert torch.equal(ref[key].view(torch.uint8), got[key].view(torch.uint8)), (name, key)
        assert int(got["dl"].min()) >= 1 and (got["stop"] == 1).all()
    # a batch whose slice records cannot fit the fixed array is refused, and nothing is launched
    lib = svip.load()
    Bbig, V = 4096, 128256
    z = torch.zeros(8, dtype=torch.bfloat16, device=dev)
    rc = lib.svip_draft_step_static(z.data_ptr(), 1, Bbig, V, V, 1.0, 0.3, 0, 4, z.data_ptr(), None, z.data_ptr(), None,
                                    None, z.data_ptr(), z.data_ptr(), None, 1, None)
    assert rc == 5 and b"WORKSPACE" in lib.svip_status_string(rc)
    torch.cuda.synchronize()

"""GPU edge cases: ragged and tiny vocabularies, masked logits, degenerate rows, draft lengths,
long rows that need several sampler batches, flags for bad device data."""
import math

import numpy as np
import pytest
import torch

import oracle
from helpers import MARGIN, Round, check_draft_rows, check_verify

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


def _padded(x, dtype, mult):
    """Copy x [..., V] into storage whose row pitch is a multiple of `mult` elements, so that
    any V satisfies the 16-byte stride rule; returns the [..., V] view."""
    V = x.shape[-1]
    Vp = (V + mult - 1) // mult * mult
    buf = torch.full((*x.shape[:-1], Vp), 77.0, dtype=dtype)     # padding must never be read
    buf[..., :V] = x.to(dtype)
    return buf.cuda()[..., :V]


def _make(B, k, V, dtype, seed, scale=2.0, noise=1.0):
    g = torch.Generator().manual_seed(seed)
    draft = (scale * torch.randn(B, k, V, generator=g)).to(dtype)
    target = torch.cat([draft.float(), scale * torch.randn(B, 1, V, generator=g)], 1)
    target = (target + noise * torch.randn(B, k + 1, V, generator=g)).to(dtype)
    u = torch.rand(3, B, k, generator=g)
    return draft, target, u[0], u[1], u[2][:, 0].contiguous()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
@pytest.mark.parametrize("V", [1, 2, 5, 8, 9, 1023, 2049, 4097, 16385, 40003])
def test_ragged_vocab_sizes(svip, V, dtype):
    """V that is not a multiple of the vector, the tile or the slice; padding is poisoned."""
    B, k = 3, 4
    mult = 4 if dtype == torch.float32 else 8
    draft, target, us, ua, ur = _make(B, k, V, dtype, seed=V)
    r = Round(svip, draft, target, us, ua, ur, 1.0, 1.5)
    r.draft = _padded(draft, dtype, mult)
    r.target = _padded(target, dtype, mult)
    r.draft_all(chain=False)
    st = check_draft_rows(draft, 1.0, 1.5, k, us, r)
    tokens = r.tokens.cpu().numpy().astype(np.int64)
    dl = np.array([k, k - 1, 1][:B], np.int64)
    for mode in ("given", None):
        r.verify(tokens=r.tokens, draft_len=torch.from_numpy(dl).int().cuda(), lse=mode)
        check_verify(draft, target, 1.0, tokens, dl, ua, ur, r)
    _say(f"V={V} {dtype}: {st}")


@pytest.mark.parametrize("dtype,V", [(torch.float32, 600_000), (torch.bfloat16, 1_200_003)])
def test_long_rows_take_several_sampler_batches(svip, dtype, V):
    """Rows longer than 64 slices x 8 tiles: the sampler scans more than one batch per slice."""
    B, k = 2, 2
    draft, target, us, ua, ur = _make(B, k, V, dtype, seed=5, scale=1.0)
    mult = 4 if dtype == torch.float32 else 8
    r = Round(svip, draft, target, us, ua, ur, 1.0, 3.0)
    r.draft = _padded(draft, dtype, mult)
    r.target = _padded(target, dtype, mult)
    r.draft_all(chain=False)
    st = check_draft_rows(draft, 1.0, 3.0, k, us, r)
    tokens = r.tokens.cpu().numpy().astype(np.int64)
    dl = np.array([2, 1], np.int64)
    r.verify(tokens=r.tokens, draft_len=torch.from_numpy(dl).int().cuda(), lse="given")
    check_verify(draft, target, 1.0, tokens, dl, ua, ur, r)
    _say(f"V={V}: {st}")


def test_masked_vocab_and_degenerate_rows(svip):
    """-inf logits carry no mass and are never drawn; one-hot rows have H = 0 and never stop;
    uniform rows have H = ln V."""
    V, k = 5000, 6
    g = torch.Generator().manual_seed(3)
    draft = torch.randn(2, k, V, generator=g)
    draft[0, 0, :] = -math.inf
    draft[0, 0, 4321] = 2.5                          # one-hot through masking
    draft[0, 1, ::2] = -math.inf                     # half the vocabulary masked
    draft[0, 2, :] = 0.0                             # uniform
    draft[0, 3, :] = 0.0
    draft[0, 3, 77] = 1.0e4                          # one-hot through a huge spike
    draft[0, 4, :4000] = -math.inf                   # whole leading slices masked
    draft[0, 5, 100:] = -math.inf                    # only a short head has mass
    target = torch.cat([draft, torch.randn(2, 1, V, generator=g)], 1) + 0.5 * torch.randn(2, k + 1, V, generator=g)
    target[0, 1] = torch.randn(V, generator=g)
    target[0, 1, 1::2] = -math.inf                   # target support disjoint from the draft's
    u = torch.rand(3, 2, k, generator=g)
    us, ua, ur = u[0], u[1], u[2][:, 0].contiguous()
    us[0, 0] = 0.0
    us[0, 3] = float(np.nextafter(np.float32(1.0), np.float32(0.0)))
    for dtype in (torch.float32, torch.bfloat16, torch.float16):
        d, t = draft.to(dtype), target.to(dtype)
        r = Round(svip, d, t, us, ua, ur, 1.0, 0.3)
        r.draft_all(chain=False)
        check_draft_rows(d, 1.0, 0.3, k, us, r)
        tok = r.tokens.cpu().numpy()
        H = r.entropy.cpu().numpy()
        stop = r.stop_hist.cpu().numpy()
        assert tok[0, 0] == 4321 and H[0, 0] == 0.0 and stop[0, 0] == 0
        assert tok[0, 1] % 2 == 1
        assert abs(H[0, 2] - math.log(V)) < 1e-4 * math.log(V) and stop[2, 0] == 1
        assert tok[0, 3] == 77 and H[0, 3] == 0.0 and stop[3, 0] == 0
        assert tok[0, 4] >= 4000 and tok[0, 5] < 100
        assert np.isfinite(H).all() and np.isfinite(r.lse.cpu().numpy()).all()
        tokens = tok.astype(np.int64)
        dl = np.array([k, k], np.int64)
        r.verify(tokens=r.tokens, draft_len=torch.from_numpy(dl).int().cuda(), lse="given")
        check_verify(d, t, 1.0, tokens, dl, ua, ur, r)
        # position 1 of sequence 0 has disjoint supports: p(x) = 0 -> certain rejection there or earlier
        assert r.n_accepted.cpu().numpy()[0] <= 1


def test_identical_models_accept_everything(svip):
    B, k, V = 4, 5, 3000
    draft, target, us, ua, ur = _make(B, k, V, torch.float32, seed=9)
    target[:, :k] = draft
    r = Round(svip, draft, target, us, ua, ur, 1.0, 9.0)
    r.draft_all(chain=True)
    assert (r.draft_len.cpu().numpy() == k).all()
    for mode in ("given", None):
        r.verify(lse=mode)
        assert (r.n_accepted.cpu().numpy() == k).all()
        assert (r.accept_prob.cpu().numpy() >= 1.0 - 1e-6).all()
        for b in range(B):      # bonus token from the row after the drafts
            p, _ = oracle.softmax_row(target[b, k])
            i, m = oracle.inverse_cdf(p, float(ur[b]))
            if m >= MARGIN:
                assert r.next_token.cpu().numpy()[b] == i


def test_draft_len_zero_and_k_above_one_wave(svip):
    """draft_len = 0 draws the bonus from the first target row; k = 100 > 64 positions."""
    B, k, V = 3, 100, 257
    draft, target, us, ua, ur = _make(B, k, V, torch.float32, seed=11, scale=1.0, noise=0.2)
    r = Round(svip, draft, target, us, ua, ur, 1.0, 9.0)
    r.draft = _padded(draft, torch.float32, 4)
    r.target = _padded(target, torch.float32, 4)
    r.draft_all(chain=False)
    tokens = r.tokens.cpu().numpy().astype(np.int64)
    for dl in ([0, 100, 65], [64, 1, 99]):
        dl = np.array(dl, np.int64)
        r.accept_prob.fill_(float("nan"))
        r.verify(tokens=r.tokens, draft_len=torch.from_numpy(dl).int().cuda(), lse=None)
        st = check_verify(draft, target, 1.0, tokens, dl, ua, ur, r)
        _say(f"dl={dl.tolist()} n_acc={r.n_accepted.cpu().tolist()} {st}")


def test_inactive_rows_are_left_alone(svip):
    B, k, V = 6, 3, 1000
    draft, target, us, ua, ur = _make(B, k, V, torch.bfloat16, seed=13)
    r = Round(svip, draft, target, us, ua, ur, 1.0, 9.0)
    r.stop[:] = torch.tensor([0, 1, 0, 1, 1, 0], dtype=torch.uint8)
    r.draft_len.fill_(-5)
    svip.draft_step(r.draft[:, 0], temperature=1.0, h=9.0, step_j=0, k_max=k, u_sample=r.u_sample[:, 0],
                    stop_in=r.stop, token_out=r.tokens[:, 0], entropy_out=r.entropy[:, 0],
                    q_tok_out=r.q_tok[:, 0], lse_out=r.lse[:, 0], stop_out=r.stop,
                    draft_len_out=r.draft_len, workspace=r.ws)
    torch.cuda.synchronize()
    tok, H, dl = r.tokens.cpu().numpy(), r.entropy.cpu().numpy(), r.draft_len.cpu().numpy()
    for b in (1, 3, 4):
        assert tok[b, 0] == -1 and np.isnan(H[b, 0]) and dl[b] == -5 and r.stop[b] == 1
    for b in (0, 2, 5):
        assert tok[b, 0] >= 0 and not np.isnan(H[b, 0]) and dl[b] == 1 and r.stop[b] == 0
    assert (tok[:, 1:] == -7).all()                   # other columns untouched


def test_bad_device_data_sets_flags(svip):
    B, k, V = 2, 3, 64
    draft, target, us, ua, ur = _make(B, k, V, torch.float32, seed=17)
    r = Round(svip, draft, target, us, ua, ur, 1.0, 9.0)
    assert svip.workspace_flags(r.ws) == 0
    r.draft_all(chain=True)
    r.verify()
    assert svip.workspace_flags(r.ws) == 0
    bad_tok = r.tokens.clone()
    bad_tok[1, 0] = V + 5
    r.verify(tokens=bad_tok)
    assert svip.workspace_flags(r.ws) == svip.FLAG_BAD_TOKEN
    r.verify(draft_len=torch.tensor([k + 1, -1], dtype=torch.int32).cuda())
    assert svip.workspace_flags(r.ws) == svip.FLAG_BAD_TOKEN | svip.FLAG_BAD_DRAFT_LEN
    assert (r.n_accepted.cpu().numpy() <= k).all() and (r.n_accepted.cpu().numpy() >= 0).all()


def test_host_errors_enqueue_nothing(svip):
    B, k, V = 2, 2, 64
    draft, target, us, ua, ur = _make(B, k, V, torch.float32, seed=19)
    r = Round(svip, draft, target, us, ua, ur, 1.0, 0.3)
    kw = dict(temperature=1.0, h=0.3, step_j=0, k_max=k, u_sample=r.u_sample[:, 0], token_out=r.tokens[:, 0],
              lse_out=r.lse[:, 0], stop_out=r.stop, workspace=r.ws)
    for bad, status in ((dict(temperature=0.0), 6), (dict(temperature=float("nan")), 6), (dict(h=-1.0), 6),
                        (dict(step_j=k), 2), (dict(k_max=svip.MAX_K + 1), 2),
                        (dict(workspace=r.ws[:300]), 5), (dict(workspace=r.ws[8:]), 5)):
        with pytest.raises(svip.SvipError) as e:
            svip.draft_step(r.draft[:, 0], **{**kw, **bad})
        assert e.value.status == status, bad
    with pytest.raises(svip.SvipError) as e:                 # misaligned base pointer
        svip.draft_step(r.draft[:, 0, 1:], **kw)
    assert e.value.status == 4
    torch.cuda.synchronize()
    assert (r.tokens.cpu().numpy() == -7).all()              # nothing ran


def test_largest_k(svip):
    """k_max = SVIP_MAX_K = 1024 positions per round (16 passes of the acceptance wave), close models so that
    long runs are accepted."""
    B, k, V = 2, svip.MAX_K, 132
    draft, target, us, ua, ur = _make(B, k, V, torch.float32, seed=31, scale=1.0, noise=0.02)
    r = Round(svip, draft, target, us, ua, ur, 1.0, 9.0)
    r.draft_all(chain=False)
    tokens = r.tokens.cpu().numpy().astype(np.int64)
    st_d = check_draft_rows(draft, 1.0, 9.0, k, us, r, steps=[0, 1, 63, 64, 511, 1022, 1023])
    for dl in ([1024, 700], [1, 1023]):
        dl = np.array(dl, np.int64)
        r.accept_prob.fill_(float("nan"))
        for mode in ("given", None):
            r.verify(tokens=r.tokens, draft_len=torch.from_numpy(dl).int().cuda(), lse=mode)
            st = check_verify(draft, target, 1.0, tokens, dl, ua, ur, r)
        _say(f"k={k} dl={dl.tolist()} n_acc={r.n_accepted.cpu().tolist()} {st} draft {st_d}")
    assert svip.workspace_flags(r.ws) == 0


def test_large_batch_of_short_rows(svip):
    """B = 6000 sequences (more statistics rows than a 16-bit grid dimension), tiny vocabulary."""
    B, k, V = 6000, 5, 96
    draft, target, us, ua, ur = _make(B, k, V, torch.float32, seed=23, scale=1.5, noise=0.7)
    r = Round(svip, draft, target, us, ua, ur, 1.0, 1.9)
    r.draft_all(chain=True)
    from helpers import check_chain, oracle_chain
    rows = list(range(0, B, 97))
    tokens, dl, lse, mh, ms = oracle_chain(draft[rows], 1.0, 1.9, us[rows])
    st = check_chain(r.tokens.cpu().numpy(), r.draft_len.cpu().numpy(), tokens, dl, mh, ms, rows=rows,
                     draft_cpu=draft[rows], T=1.0, u_sample=us[rows])
    for mode in ("given", None):
        r.verify(lse=mode)
        sv = check_verify(draft, target, 1.0, r.tokens.cpu().numpy().astype(np.int64),
                          r.draft_len.cpu().numpy().astype(np.int64), ua, ur, r, rows=rows)
    assert svip.workspace_flags(r.ws) == 0
    _say(f"B={B}: chain {st} verify {sv}")


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16, torch.float32])
def test_wide_batch_of_long_rows(svip, dtype):
    """B = 261 rows of the 128K vocabulary: a launch that would have more than 8100 one-tile waves, so a draft
    record holds two tiles, the search takes them as one batch, and with 8352 waves rows are not placed by XCD;
    a sample of rows against the oracle, every output of the batch finite."""
    B, k, V = 261, 2, 128256
    g = torch.Generator().manual_seed(77)
    draft = torch.randn(B, k, V, generator=g)
    low = torch.rand(B, k, generator=g) < 0.7
    draft = torch.where(low[..., None], draft, 0.5 * draft)
    draft[torch.arange(B)[:, None], torch.arange(k)[None, :], torch.randint(0, V, (B, k), generator=g)] += 9.0
    draft = draft.to(dtype)
    target = torch.cat([draft, draft[:, :1]], 1)
    u = torch.rand(3, B, k, generator=g)
    r = Round(svip, draft.cuda(), target.cuda(), u[0], u[1], u[2][:, 0].contiguous(), 1.0, 3.0)
    r.draft_all(chain=False)
    rows = list(range(0, B, 11))
    st = check_draft_rows(draft, 1.0, 3.0, k, u[0], r, rows=rows)
    tok = r.tokens.cpu().numpy()
    assert ((tok >= 0) & (tok < V)).all() and torch.isfinite(r.entropy).all() and torch.isfinite(r.lse).all()
    # tail cells of these rows are about 5e-6 wide, so about four draws in ten lie within 1e-6 of a cell edge
    # (a property of the rows, computed by the oracle alone); they are checked for validity, the rest exactly
    assert st["stop_excluded"] == 0 and st["tok_excluded"] <= 0.55 * st["rows"]
    _say(f"{dtype} B={B} V={V}: {st}")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
def test_small_entropies_keep_their_relative_accuracy(svip, dtype):
    """Confident rows: one logit far above the rest, H from 5e-2 down to 1e-8.  The row maximum has
    weight exactly 1 on the GPU, so the entropy comes from the tail alone and stays accurate to REL."""
    from helpers import REL
    V, k = 40003, 6
    g = torch.Generator().manual_seed(12)
    spikes = [16.0, 19.0, 22.0, 25.0, 28.0, 31.0]
    draft = torch.randn(3, k, V, generator=g)
    for j, s in enumerate(spikes):
        draft[:, j, 1000 * j + 7] = s
    draft = draft.to(dtype)
    target = torch.cat([draft, draft[:, :1]], 1)
    u = torch.rand(3, 3, k, generator=g)
    r = Round(svip, _padded(draft, dtype, 8), _padded(target, dtype, 8), u[0], u[1], u[2][:, 0].contiguous(), 1.0, 0.3)
    r.draft_all(chain=False)
    H = r.entropy.cpu().numpy()
    for b in range(3):
        for j in range(k):
            p, _ = oracle.softmax_row(draft[b, j].double().numpy(), 1.0)
            want = oracle.entropy_row(p)
            assert 1e-9 < want < 0.5
            assert abs(H[b, j] - want) <= REL * want, f"row {b} step {j}: H {H[b, j]} vs {want}"


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
def test_every_launch_shape_of_the_draft_step(svip, dtype):
    """The draft step picks records per row (one tile each, two tiles each with both requested at once, longer
    ones), and places rows by XCD or not, from the batch and the row length.  Here every one of those shapes
    is forced on the same ragged rows (sampled and greedy) and each is compared with the oracle; B = 11 is
    no multiple of the 8 XCDs and the record counts are no multiples of a workgroup's 4 waves."""
    B, k = 11, 2
    mult, tile = (4, 1024) if dtype == torch.float32 else (8, 2048)
    V = 13 * tile + 5 * mult + 3                      # 14 tiles, the last one ragged
    draft, target, us, ua, ur = _make(B, k, V, dtype, seed=77)
    try:
        for records in (0, 14, 13, 7, 5, 3, 1):       # 0: the library's own choice; 7: two tiles each; 5, 3, 1: longer
            svip.bench_set_tuning(draft_slices=records)
            for greedy in (False, True):
                r = Round(svip, draft, target, us, ua, ur, 1.0, 1.5)
                r.draft = _padded(draft, dtype, mult)
                r.draft_all(chain=False, greedy=greedy)
                if greedy:
                    tok = r.tokens.cpu().numpy()
                    want = draft.double().numpy().argmax(-1)          # numpy's argmax is the first maximum
                    assert (tok == want).all(), f"records={records}: greedy tokens"
                else:
                    st = check_draft_rows(draft, 1.0, 1.5, k, us, r)
                    assert st["tok_excluded_diff"] <= 1 and st["stop_excluded"] == 0, (records, st)
            _say(f"{dtype} records={records}: {st}")
    finally:
        svip.bench_set_tuning()

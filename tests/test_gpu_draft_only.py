"""LLC_FLAG_DRAFT_ONLY: the drafters' step of Algorithm 2 (the draft side of Algorithm 1 alone), through
the C ABI, against the oracle and against the full call (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2506_05632_amd as llc
from paper_2506_05632_amd import workloads
from parity_util import oracle_rows, to_host

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
DO = llc.FLAG_DRAFT_ONLY


def _check(draft, target, K, rows, *, kind="logits", temp_draft=1.0, seed=0, row_offset=0, extra_flags=0, min_first=False, **kw):
    got = llc.llc_couple(draft, None, K, kind=kind, temp_draft=temp_draft, seed=seed, row_offset=row_offset,
                         want_keys=True, flags=DO | extra_flags, **kw)
    full = llc.llc_couple(draft, target, K, kind=kind, temp_draft=temp_draft, seed=seed, row_offset=row_offset,
                          want_keys=True, flags=extra_flags, **kw)
    torch.cuda.synchronize()
    assert set(got) == {"X", "keyX"}
    assert torch.equal(got["X"], full["X"])               # the draft side does not depend on the target
    np.testing.assert_allclose(got["keyX"].cpu().numpy(), full["keyX"].cpu().numpy(), rtol=1e-6)
    ref = oracle_rows(draft, target, K, rows, kind=kind, temp_target=1.0, temp_draft=temp_draft, seed=seed,
                      row_offset=row_offset, min_first=min_first)
    gx = got["X"][rows[0]:rows[1]].cpu().numpy()
    bad = gx != ref["X"]
    assert (ref["gapX"][bad] < 1e-6).all()
    ok = ~bad & (ref["X"] >= 0)
    np.testing.assert_allclose(got["keyX"][rows[0]:rows[1]].cpu().numpy()[ok], ref["keyX"][ok], rtol=1e-6)


@pytest.mark.parametrize("min_first", [False, True])
def test_draft_side_alone_on_the_configurations(min_first):
    mf = llc.FLAG_MIN_FIRST if min_first else 0
    for cfg, rows in ((1, 64), (2, 256), (3, 64), (4, 32)):
        w = workloads.make(cfg, DEV, rows=rows)
        _check(w.draft, w.target, w.K, (0, w.B), kind=w.kind, temp_draft=w.temp_draft, seed=w.seed,
               row_offset=w.row_offset, extra_flags=mf, min_first=min_first)


def test_launch_shapes_edge_rows_and_the_other_entry_points():
    g = torch.Generator(device=DEV).manual_seed(3)
    B, V, K = 9, 4099, 5
    tq = 2 * torch.randn(B, V, generator=g, device=DEV)
    td = tq[:, None, :] + torch.randn(B, K, V, generator=g, device=DEV)
    td[1, 2, :] = float("-inf")                 # a draft without mass: X = -1
    td[2, 0, 7] = float("nan")
    base = llc.llc_couple(td, None, K, seed=4, flags=DO, want_keys=True)
    assert (base["X"][1, 2] == -1) and torch.isinf(base["keyX"][1, 2])
    for vc, kt in ((1, 2), (3, 4), (5, 8), (2, 1)):
        other = llc.llc_couple(td, None, K, seed=4, flags=DO, want_keys=True, v_chunks=vc, k_tile=kt)
        assert torch.equal(other["X"], base["X"])
    exact = llc.llc_couple(td, None, K, seed=4, flags=DO | llc.FLAG_EXACT_SCAN)
    assert torch.equal(exact["X"], base["X"])
    ref = oracle.couple(to_host(td)[0], to_host(tq)[0], K, seed=4)
    assert np.array_equal(base["X"].cpu().numpy(), ref["X"])
    # probabilities, one shared proposal, bf16
    p = (torch.rand(B, V, generator=g, device=DEV) ** 6).to(torch.bfloat16)
    got = llc.llc_couple(p, None, 3, kind="probs", seed=8, flags=DO)
    ref = oracle.couple(to_host(p)[0], to_host(p)[0], 3, dtype=oracle.BF16, kind=oracle.PROBS, seed=8)
    assert np.array_equal(got["X"].cpu().numpy(), ref["X"])
    # the entry point that allocates nothing takes the flag too
    out = {"X": torch.empty(B, K, dtype=torch.int32, device=DEV)}
    llc.llc_couple_static(td, None, K, seed=4, flags=DO, out=out)
    torch.cuda.synchronize()
    assert torch.equal(out["X"], base["X"])


def test_drafting_and_verifying_one_position_use_the_same_randomness():
    # Algorithm 2 at one position: the drafters sample with the flag, the verifier (llc_verify with no
    # draft positions before it, i.e. Algorithm 1's pool) must accept exactly where llc_couple does
    g = torch.Generator(device=DEV).manual_seed(12)
    S, K, V = 200, 4, 3000
    q = 2 * torch.randn(S, V, generator=g, device=DEV)
    p = q + 0.7 * torch.randn(S, V, generator=g, device=DEV)
    for flags in (0, llc.FLAG_MIN_FIRST):
        drafted = llc.llc_couple(p, None, K, seed=21, flags=DO | flags)["X"]            # rows 0..S-1
        full = llc.llc_couple(p, q, K, seed=21, flags=flags)
        target = q[:, None, None, :].expand(S, 2, K, V).contiguous()                      # [S, 2, K, V]
        ver = llc.llc_verify(target, drafted[:, None, :].contiguous(), seed=21, row_stride_s=1, row_stride_j=S, flags=flags)
        torch.cuda.synchronize()
        assert torch.equal(drafted, full["X"])
        assert torch.equal(ver["Y"][:, 0], full["Y"])
        assert torch.equal(ver["n_out"], 1 + full["accept"].to(torch.int32))

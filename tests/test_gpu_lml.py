"""GPU parity of llc_lml_bound (Theorem 1's bound per row) against the CPU oracle (needs an MI355X).

Tolerance: the device sorts on the fp32 image of ln(q/p), so indices whose ratios agree to fp32
precision may be swapped, which moves their summands by a relative 2^-23 at most; everything
else is fp64 on both sides (sums in different orders).  rtol 1e-6 covers it with room.
"""
import numpy as np
import pytest
import torch

import paper_2506_05632_amd as llc
from oracle import lml
from paper_2506_05632_amd import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
RTOL = 1e-6
KS = [1, 2, 4, 8, 16]


def check(draft, target, ks, rows=None, **kw):
    gpu = llc.llc_lml_bound(draft, target, ks, **kw)
    torch.cuda.synchronize()
    d = draft.detach().float().cpu().numpy()  # (bf16 -> fp32 is exact)
    t = target.detach().float().cpu().numpy()
    sel = np.arange(d.shape[0]) if rows is None else np.asarray(rows)
    ref = lml.lml_rows(d[sel], t[sel], ks, kind=kw.get("kind", "logits"), temp_draft=kw.get("temp_draft", 1.0),
                       temp_target=kw.get("temp_target", 1.0))
    for name in ("bound", "relaxed", "tv"):
        got = gpu[name].cpu().numpy()[sel]
        np.testing.assert_allclose(got, ref[name], rtol=RTOL, atol=1e-12, err_msg=name)
    return gpu, ref


# (the sort takes a row 4096 entries at a time: one tile exactly, one entry more, several tiles)
@pytest.mark.parametrize("V", [1, 2, 63, 64, 65, 255, 256, 257, 1000, 4095, 4096, 4097, 8192, 12289])
@pytest.mark.parametrize("kind", ["logits", "logw", "probs"])
def test_small_rows_all_kinds_and_ragged_lengths(V, kind):
    g = torch.Generator(device=DEV).manual_seed(100 + V)
    B = 7
    tq = 2.0 * torch.randn(B, V, generator=g, device=DEV)
    td = tq + torch.randn(B, V, generator=g, device=DEV)
    if kind == "probs":
        td, tq = torch.exp(td), torch.exp(tq)
    gpu, ref = check(td, tq, KS, kind=kind, temp_draft=1.3, temp_target=0.7)
    assert (ref["bound"] <= 1 + 1e-12).all() and (np.diff(ref["bound"], axis=1) >= -1e-12).all()


def test_bf16_inputs_and_strided_rows():
    g = torch.Generator(device=DEV).manual_seed(7)
    B, V = 9, 3001
    big = (1.5 * torch.randn(B, 2 * V + 6, generator=g, device=DEV)).to(torch.bfloat16)
    check(big[:, :V], big[:, V + 3:2 * V + 3], [1, 8], temp_target=0.8)


def test_entries_without_mass_and_equal_distributions():
    g = torch.Generator(device=DEV).manual_seed(8)
    B, V = 6, 777
    tq = torch.randn(B, V, generator=g, device=DEV)
    td = tq + torch.randn(B, V, generator=g, device=DEV)
    td[0, :50] = -float("inf")                 # mass of q where p has none
    tq[1, 100:300] = -float("inf")             # and the reverse
    td[2, ::3] = -float("inf"); tq[2, ::3] = -float("inf")  # neither
    td[3] = tq[3]                              # p = q: the bound is 1
    td[4, :V // 2] = -float("inf"); tq[4, V // 2:] = -float("inf")  # disjoint supports: 0
    td[5, 5] = float("nan"); tq[5, 9] = float("inf")  # carry no mass
    gpu, ref = check(td, tq, [1, 3, 8])
    got = gpu["bound"].cpu().numpy()
    assert np.allclose(got[3], 1.0, rtol=1e-12) and (got[4] == 0.0).all()
    assert abs(gpu["tv"].cpu().numpy()[4] - 1.0) < 1e-12
    # probabilities with zeros
    p = torch.rand(B, V, generator=g, device=DEV); q = torch.rand(B, V, generator=g, device=DEV)
    p[:, ::5] = 0.0; q[:, 1::7] = 0.0
    check(p, q, [2, 5], kind="probs")


def test_many_equal_ratios_and_sorted_inputs():
    # ties in q/p (stability and the either-order argument), already sorted and reversed rows
    B, V = 4, 2048
    base = torch.linspace(-4, 4, V, device=DEV)
    td = torch.stack([base, base.flip(0), torch.zeros(V, device=DEV), base.round()])
    tq = torch.stack([base * 0.5, base * 0.5, torch.zeros(V, device=DEV), (base * 0.5).round()])
    check(td.contiguous(), tq.contiguous(), KS)


def test_more_rows_than_workspace_slots_and_a_workspace_of_one_row():
    # a call is as many launches as its rows need slots of the workspace: more rows than slots
    # (the library's size caps at 512 rows' worth), a workspace that holds a single row (one
    # launch per row), and a larger one than asked for (one launch) give the same bits
    g = torch.Generator(device=DEV).manual_seed(600)
    B, V = 1300, 700
    assert llc.llc_lml_workspace_size(B, V) == llc.llc_lml_workspace_size(512, V) < 24 * B * V
    tq = 2 * torch.randn(B, V, generator=g, device=DEV)
    td = tq + torch.randn(B, V, generator=g, device=DEV)
    gpu, _ = check(td, tq, KS, rows=list(range(0, B, 37)) + [511, 512, 513, 1023, 1024, B - 1], temp_draft=1.1, temp_target=0.9)
    for rows in (1, 3, 600, 1400):
        ws = torch.empty(24 * V * rows + 256, dtype=torch.uint8, device=DEV)
        other = llc.llc_lml_bound(td, tq, KS, temp_draft=1.1, temp_target=0.9, workspace=ws)
        torch.cuda.synchronize()
        for name in ("bound", "relaxed", "tv"):
            assert torch.equal(other[name], gpu[name]), (rows, name)


def test_acceptance_of_the_sampler_respects_the_bound():
    # the measured acceptance rate of llc_couple on one pair (p, q) repeated over many rows of
    # randomness is at least Theorem 1's bound (up to sampling error)
    g = torch.Generator(device=DEV).manual_seed(11)
    V, n = 500, 40000
    tq = 1.5 * torch.randn(1, V, generator=g, device=DEV)
    td = tq + 0.8 * torch.randn(1, V, generator=g, device=DEV)
    ks = [1, 4, 8]
    bound = llc.llc_lml_bound(td, tq, ks)["bound"].cpu().numpy()[0]
    for K, lo in zip(ks, bound):
        out = llc.llc_couple(td.expand(n, V), tq.expand(n, V), K, seed=3 + K)
        rate = out["accept"].float().mean().item()
        sigma = np.sqrt(max(lo * (1 - lo), 1e-4) / n)
        assert rate >= lo - 4 * sigma, (K, rate, lo)
        if K == 1:
            assert abs(rate - lo) < 4 * sigma  # Remark 1: exact for K = 1


def test_large_vocabulary_workload_sampled_rows():
    w = workloads.make(3, DEV)
    rows = np.linspace(0, w.B - 1, 12).astype(int)
    draft = w.draft if w.draft.dim() == 2 else w.draft[:, 0]
    gpu, ref = check(draft, w.target, [1, 2, 4, 8], rows=rows, temp_draft=w.temp_draft, temp_target=w.temp_target)
    b = gpu["bound"].cpu().numpy()
    print(f"config 3: mean bound for K=1,2,4,8: {b.mean(0)}; mean tv {gpu['tv'].mean().item():.3f}")
    assert (b >= 0).all() and (b <= 1 + 1e-9).all() and (np.diff(b, axis=1) >= -1e-9).all()
    assert (gpu["relaxed"].cpu().numpy() <= b + 1e-9).all()


def test_rows_of_many_equal_ratios_and_of_few_distinct_ones():
    """The sort's digits at their most lopsided: every entry with the same ratio q/p (all keys
    equal), two values only, and ratios that differ in the last bits of the key only."""
    g = torch.Generator(device=DEV).manual_seed(77)
    V = 9000
    tq = torch.randn(4, V, generator=g, device=DEV)
    td = tq.clone()
    td[1] = tq[1] + 0.5                                  # softmax undoes the shift: p = q up to the sum's rounding
    td[2, ::2] += 1.0                                    # two ratios
    td[3] = tq[3] + 1e-6 * torch.randn(V, generator=g, device=DEV)  # ratios within a few ulps of 1
    gpu, ref = check(td, tq, KS)
    got = gpu["bound"].cpu().numpy()
    assert np.allclose(got[0], 1.0, rtol=1e-12) and np.allclose(got[1], 1.0, rtol=1e-6)


def test_the_longest_row_the_interface_accepts():
    """V = 2^28, the most llc_lml_bound takes.  The mass sits on some thousand entries (the first and
    the last ones among them); entries without mass on either side add nothing to any sum, so the
    oracle is given the entries with mass alone."""
    V, M = 1 << 28, 20000
    g = torch.Generator(device=DEV).manual_seed(5)
    ids = torch.randint(0, V, (M,), generator=g, device=DEV, dtype=torch.int64)
    ids = torch.cat([ids, torch.arange(0, 5, device=DEV), torch.arange(V - 5, V, device=DEV)]).unique()
    vq = 2 * torch.randn(ids.numel(), generator=g, device=DEV)
    vd = vq + torch.randn(ids.numel(), generator=g, device=DEV)
    vd[::7] = -float("inf")  # some entries with target mass only
    tq = torch.full((1, V), -float("inf"), device=DEV)
    td = torch.full((1, V), -float("inf"), device=DEV)
    tq[0, ids] = vq
    td[0, ids] = vd
    gpu = llc.llc_lml_bound(td, tq, KS, temp_draft=1.2, temp_target=0.8)
    torch.cuda.synchronize()
    ref = lml.lml_rows(vd.cpu().numpy()[None], vq.cpu().numpy()[None], KS, temp_draft=1.2, temp_target=0.8)
    for name in ("bound", "relaxed", "tv"):
        np.testing.assert_allclose(gpu[name].cpu().numpy(), ref[name], rtol=RTOL, atol=1e-12, err_msg=name)
    del tq, td, gpu
    torch.cuda.empty_cache()

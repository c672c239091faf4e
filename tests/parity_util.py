"""Helpers shared by the GPU parity tests: run both implementations on the same bits, compare.

The bar: X, Y, accept, match_k bit-exact; a mismatch is excused only where the
oracle's own relative gap between the best and the runner-up key of that
reduction is below 1e-6 (a near-tie); winning keys within 1e-6 relative.
"""
import numpy as np
import torch

import oracle

NEAR_TIE = 1e-6
KEY_RTOL = 1e-6
_KIND = {"logits": oracle.LOGITS, "probs": oracle.PROBS, "logw": oracle.LOGW}


def to_host(t: torch.Tensor):
    """Device tensor -> (numpy array the oracle takes, oracle dtype code)."""
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).numpy().view(np.uint16), oracle.BF16
    return t.contiguous().numpy(), oracle.F32


def oracle_rows(draft, target, K, rows, *, kind, temp_target, temp_draft, temp_draft_per_k=None,
                seed=0, row_offset=0, min_first=False):
    """Oracle on rows [r0, r1) of the batch, keyed as the same global rows."""
    r0, r1 = rows
    d, dt = to_host(draft[r0:r1])
    t, _ = to_host(target[r0:r1])
    tk = None if temp_draft_per_k is None else temp_draft_per_k.detach().cpu().numpy()
    return oracle.couple(d, t, K, dtype=dt, kind=_KIND[kind], temp_target=temp_target,
                         temp_draft=tk, temp_draft_all=temp_draft, seed=seed,
                         row_offset=row_offset + r0, min_first=min_first)


def compare(gpu: dict, ref: dict, rows=None, check_keys=True):
    """Assert parity on the given row range; returns the number of excused near-ties."""
    g = {k: v.detach().cpu().numpy() for k, v in gpu.items()}
    if rows is not None:
        g = {k: v[rows[0]:rows[1]] for k, v in g.items()}
    near = 0
    badX = g["X"] != ref["X"]
    for b, k in zip(*np.nonzero(badX)):
        assert ref["gapX"][b, k] < NEAR_TIE, f"X[{b},{k}] gpu {g['X'][b, k]} ref {ref['X'][b, k]} gap {ref['gapX'][b, k]}"
        near += 1
    badY = g["Y"] != ref["Y"]
    for b in np.nonzero(badY)[0]:
        assert ref["gapY"][b] < NEAR_TIE, f"Y[{b}] gpu {g['Y'][b]} ref {ref['Y'][b]} gap {ref['gapY'][b]}"
        near += 1
    clean = ~(badX.any(axis=1) | badY)
    assert np.array_equal(g["accept"][clean], ref["accept"][clean])
    if "match_k" in g:
        assert np.array_equal(g["match_k"][clean], ref["match_k"][clean])
    # accept is consistent with the GPU's own X and Y everywhere
    inlist = ((g["X"] == g["Y"][:, None]) & (g["Y"][:, None] >= 0)).any(axis=1)
    assert np.array_equal(g["accept"].astype(bool), inlist)
    if check_keys and "keyX" in g:
        okX = ~badX & (ref["X"] >= 0)
        np.testing.assert_allclose(g["keyX"][okX], ref["keyX"][okX], rtol=KEY_RTOL)
        okY = ~badY & (ref["Y"] >= 0)
        np.testing.assert_allclose(g["keyY"][okY], ref["keyY"][okY], rtol=KEY_RTOL)
        assert np.isinf(g["keyX"][ref["X"] < 0]).all() and np.isinf(g["keyY"][ref["Y"] < 0]).all()
    return near


def oracle_near_ties(ref: dict) -> int:
    """Reductions of an oracle result whose runner-up (at another index) is within 1e-6 of the winner."""
    n = int((ref["gapY"] < NEAR_TIE).sum())
    if "gapX" in ref:
        n += int((ref["gapX"] < NEAR_TIE).sum())
    return n


def oracle_borderline(ref: dict) -> int:
    """Reductions whose gap is so close to 1e-6 itself that the two sides' fp64 roundings may
    classify them differently (the device compares log-domain keys, the oracle S/p)."""
    lo, hi = NEAR_TIE * (1 - 1e-6), NEAR_TIE * (1 + 1e-6)
    n = int(((ref["gapY"] > lo) & (ref["gapY"] < hi)).sum())
    if "gapX" in ref:
        n += int(((ref["gapX"] > lo) & (ref["gapX"] < hi)).sum())
    return n


def stats_dict(stats: torch.Tensor) -> dict:
    from paper_2506_05632_amd.binding import STATS_FIELDS
    return dict(zip(STATS_FIELDS, (int(v) for v in stats.cpu().numpy())))


def same_outputs(a: dict, b: dict):
    """Indices and flags bit for bit.  Reported keys carry the rows' normalisers, which the scan
    sums chunk by chunk: their last bits may depend on the launch shape (far inside the 1e-6 that
    keys are held to)."""
    for name in a:
        if name.startswith("key"):
            torch.testing.assert_close(a[name], b[name], rtol=1e-6, atol=0)
        else:
            assert torch.equal(a[name], b[name]), name


# Near-ties per configuration (reductions whose runner-up is within 1e-6 of the winner): with keys
# that are continuous up to the 2^-32 grid of the uniforms, one reduction is a near-tie with
# probability of the order of 1e-6, so a whole configuration (10^4 reductions) almost surely has
# none; more than this many would point at a defect, not at chance.
NEAR_TIE_BOUND = 2


def check_all_rows(w, gpu, stats, block, is_form=False, min_first=False):
    """Every row of the workload against the oracle, `block` rows at a time (host memory), and the
    device's near-tie counter against the oracle's own count.  Returns the report line's numbers."""
    mismatches, near_oracle, borderline = 0, 0, 0
    for r0 in range(0, w.B, block):
        rows = (r0, min(w.B, r0 + block))
        if is_form:
            enc, _ = to_host(w.target[rows[0]:rows[1]])
            dec, _ = to_host(w.draft[rows[0]:rows[1]])
            ref = oracle.couple_is(enc, dec, seed=w.seed, row_offset=w.row_offset + rows[0], min_first=min_first)
        else:
            ref = oracle_rows(w.draft, w.target, w.K, rows, kind=w.kind, temp_target=w.temp_target,
                              temp_draft=w.temp_draft, seed=w.seed, row_offset=w.row_offset, min_first=min_first)
        mismatches += compare(gpu, ref, rows)
        near_oracle += oracle_near_ties(ref)
        borderline += oracle_borderline(ref)
    s = stats_dict(stats)
    print(f"{w.name}{' (min-first)' if min_first else ''}: {w.B} rows compared, excused mismatches {mismatches}, "
          f"near-ties oracle {near_oracle} / device {s['near_ties']}, survivors {s['survivors']} of {w.elems}, "
          f"exact {s['exact_evals']}, slow blocks {s['slow_blocks']}")
    assert abs(s["near_ties"] - near_oracle) <= borderline
    assert near_oracle <= NEAR_TIE_BOUND and mismatches <= near_oracle
    assert s["slow_blocks"] == 0
    return s

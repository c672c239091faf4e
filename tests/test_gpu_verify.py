"""GPU parity of llc_verify (Algorithm 2's verification loop) against the CPU oracle (needs an MI355X).

The bar: Y, n_out, active bit-exact.  A sequence is excused from the first position at which the
oracle's own relative gap between the best and the runner-up key is below 1e-6 (a near-tie; what
follows depends on which of the two is taken).  Winning keys within 1e-6 relative.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2506_05632_amd as llc
from paper_2506_05632_amd import workloads
from parity_util import KEY_RTOL, NEAR_TIE, stats_dict, to_host

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
_KIND = {"logits": oracle.LOGITS, "logw": oracle.LOGW}


def oracle_verify(target, tokens, seqs, *, kind="logits", temp_target=1.0, seed=0, row_offset=0,
                  row_stride_s=None, row_stride_j=1, strong=False):
    """Oracle on sequences [s0, s1), keyed as the same global rows."""
    s0, s1 = seqs
    t, dt = to_host(target[s0:s1])
    L1 = target.shape[1]
    rs = L1 if row_stride_s is None else row_stride_s
    tok = tokens[s0:s1].detach().cpu().numpy() if L1 > 1 else np.zeros((s1 - s0, 0, target.shape[2]), np.int32)
    return oracle.verify(t, tok, dtype=dt, kind=_KIND[kind], temp_target=temp_target, seed=seed,
                         row_offset=row_offset + s0 * rs, row_stride_s=rs, row_stride_j=row_stride_j, strong=strong)


def compare_verify(gpu, ref, seqs=None):
    g = {k: v.detach().cpu().numpy() for k, v in gpu.items()}
    if seqs is not None:
        g = {k: v[seqs[0]:seqs[1]] for k, v in g.items()}
    S, L1 = ref["Y"].shape
    near = 0
    for s in range(S):
        clean = True
        for j in range(L1):
            if ref["Y"][s, j] >= 0 and ref["gap"][s, j] < NEAR_TIE:
                near += 1
                clean = False
                break
            assert g["Y"][s, j] == ref["Y"][s, j], f"Y[{s},{j}] gpu {g['Y'][s, j]} ref {ref['Y'][s, j]} gap {ref['gap'][s, j]}"
            if "keyY" in g:
                if ref["Y"][s, j] >= 0:
                    np.testing.assert_allclose(g["keyY"][s, j], ref["key"][s, j], rtol=KEY_RTOL)
                else:
                    assert np.isinf(g["keyY"][s, j])
        if clean:
            assert g["n_out"][s] == ref["n_out"][s]
            assert np.array_equal(g["active"][s], ref["active"][s])
    return near


def oracle_verify_near_ties(ref):
    """Emitted positions whose pool ended within 1e-6 of its runner-up (what the device counts)."""
    return int(((ref["Y"] >= 0) & (ref["gap"] < NEAR_TIE)).sum())


def run_verify(w, **kw):
    return llc.llc_verify(w.target, w.tokens, kind=w.kind, temp_target=w.temp_target, seed=w.seed,
                          row_offset=w.row_offset, **kw)


def test_verify_tiny_full_with_partials():
    w = workloads.make_verify("tiny", DEV)
    gpu = run_verify(w, want_keys=True, want_partials=True)
    torch.cuda.synchronize()
    ref = oracle_verify(w.target, w.tokens, (0, w.S), temp_target=w.temp_target, seed=w.seed)
    compare_verify({k: gpu[k] for k in ("Y", "n_out", "active", "keyY")}, ref)
    assert ref["n_out"].max() == w.L + 1 and ref["n_out"].min() == 1      # both ends of the loop occur
    # the per-(position, draft) reductions are Algorithm 1's draft-side argmins on the same rows
    rows, dt = to_host(w.target.reshape(w.S * (w.L + 1), w.K, w.V))
    part = oracle.couple(rows, rows[:, 0], w.K, dtype=dt, temp_target=w.temp_target,
                         temp_draft_all=w.temp_target, seed=w.seed)
    Yk = gpu["Yk"].cpu().numpy().reshape(-1, w.K)
    ok = part["gapX"] >= NEAR_TIE
    assert np.array_equal(Yk[ok], part["X"][ok])
    np.testing.assert_allclose(gpu["keyYk"].cpu().numpy().reshape(-1, w.K)[ok], part["keyX"][ok], rtol=KEY_RTOL)


def test_verify_with_drafts_coupled_by_algorithm_1():
    # draft tokens drawn by the oracle's Algorithm 1 on the same rows: the realistic, coupled case
    g = torch.Generator(device="cpu").manual_seed(31)
    S, L, K, V = 40, 3, 3, 6000
    seed, base = 91, 1 << 33
    tq = 2.5 * torch.randn(S, L + 1, K, V, generator=g)
    tq[:, 0, 1:] = tq[:, 0, :1]
    tokens = np.zeros((S, L, K), np.int32)
    for j in range(L):
        draft = (tq[:, j] + 0.7 * torch.randn(S, K, V, generator=g)).numpy()
        res = oracle.couple(draft, draft[:, 0], K, seed=seed, row_offset=base + j * S)
        tokens[:, j] = res["X"]
        if j + 1 <= L:
            # drafts that chose the same token keep seeing the same target row
            for s in range(S):
                for k in range(1, K):
                    for k2 in range(k):
                        if (tokens[s, :j + 1, k] == tokens[s, :j + 1, k2]).all():
                            tq[s, j + 1, k] = tq[s, j + 1, k2]
                            break
    target, tok = tq.to(DEV), torch.from_numpy(tokens).to(DEV)
    gpu = llc.llc_verify(target, tok, seed=seed, row_offset=base, row_stride_s=1, row_stride_j=S,
                         want_keys=True)
    torch.cuda.synchronize()
    ref = oracle.verify(tq.numpy(), tokens, seed=seed, row_offset=base, row_stride_s=1, row_stride_j=S)
    compare_verify(gpu, ref)
    assert ref["n_out"].mean() > 1.5      # coupled drafts are accepted often


def test_verify_bf16_full():
    w = workloads.make_verify("small_bf16", DEV)
    stats = llc.new_stats(DEV)
    gpu = run_verify(w, want_keys=True, stats=stats)
    torch.cuda.synchronize()
    ref = oracle_verify(w.target, w.tokens, (0, w.S), temp_target=w.temp_target, seed=w.seed)
    near = compare_verify(gpu, ref)
    s = stats_dict(stats)
    print(f"verify bf16: excused {near}, near-ties oracle {oracle_verify_near_ties(ref)} / device {s['near_ties']}, "
          f"survivors {s['survivors']} of {w.elems}, exact {s['exact_evals']}, slow blocks {s['slow_blocks']}")
    assert s["slow_blocks"] == 0 and s["near_ties"] == oracle_verify_near_ties(ref)


@pytest.mark.parametrize("strong", [False, True])
def test_verify_large_vocab_full(strong):
    w = workloads.make_verify("largevocab", DEV)          # the shape bench.py --workload verify times
    stats = llc.new_stats(DEV)
    gpu = run_verify(w, want_keys=True, stats=stats, strong=strong)
    torch.cuda.synchronize()
    excused, near_oracle = 0, 0
    for s0 in range(0, w.S, 32):                          # every sequence, 32 at a time (host memory)
        seqs = (s0, min(w.S, s0 + 32))
        ref = oracle_verify(w.target, w.tokens, seqs, temp_target=w.temp_target, seed=w.seed, strong=strong)
        excused += compare_verify(gpu, ref, seqs)
        near_oracle += oracle_verify_near_ties(ref)
    s = stats_dict(stats)
    print(f"verify large (strong={strong}): {w.S} sequences compared, excused {excused}, near-ties oracle "
          f"{near_oracle} / device {s['near_ties']}, survivors {s['survivors']} of {w.elems}, exact "
          f"{s['exact_evals']}, slow blocks {s['slow_blocks']}")
    assert s["slow_blocks"] == 0
    assert s["near_ties"] == near_oracle and near_oracle <= 2 and excused <= near_oracle
    Y, n = gpu["Y"].cpu().numpy(), gpu["n_out"].cpu().numpy()
    assert n.min() >= 1 and n.max() <= w.L + 1
    # the first token is position 0's pool argmin, where all K rows coincide: Algorithm 1's Y on that row
    # (rows of llc_couple are consecutive; position 0 of sequence s is row s*(L+1))
    for srow in range(0, w.S, 17):
        one = llc.llc_couple(w.target[srow:srow + 1, 0, 0], w.target[srow:srow + 1, 0, 0], w.K,
                             temp_target=w.temp_target, temp_draft=w.temp_target, seed=w.seed,
                             row_offset=srow * (w.L + 1))
        assert one["Y"].item() == Y[srow, 0]


def test_strong_form_at_the_paper_s_draft_length_and_list_size_with_the_largest_vocabulary():
    """S=64, L=4, K=8, V=152064 with the library's own launch plan: the later positions' scans split
    V over more workgroups than the one-shot scan does and need more room for their partial
    results than it; the workspace of llc_verify_workspace_size must hold both."""
    S, L, K, V = 64, 4, 8, 152064
    g = torch.Generator(device=DEV).manual_seed(640)
    target = torch.empty(S, L + 1, K, V, device=DEV)
    for j in range(L + 1):
        target[:, j] = 2.5 * torch.randn(S, K, V, generator=g, device=DEV)
    target[:, 0, 1:] = target[:, 0, :1]
    tokens = target[:, :L].argmax(dim=3).to(torch.int32)
    flip = torch.rand(S, L, K, generator=g, device=DEV) < 0.5
    tokens = torch.where(flip, torch.randint(0, V, (S, L, K), generator=g, device=DEV, dtype=torch.int32), tokens)
    kw = dict(temp_target=0.5, seed=99, row_offset=7)
    ref = oracle_verify(target, tokens, (0, S), strong=True, **kw)
    for _ in range(L):      # let some drafts follow the output, so that later positions are reached
        y = torch.from_numpy(ref["Y"][:, :L].copy()).to(DEV)
        follow = (torch.rand(S, L, K, generator=g, device=DEV) < 0.5) & (y[:, :, None] >= 0)
        tokens = torch.where(follow, y[:, :, None].expand(S, L, K).to(torch.int32), tokens)
        ref = oracle_verify(target, tokens, (0, S), strong=True, **kw)
    assert ref["n_out"].max() >= 3
    ws = torch.empty(llc.llc_verify_workspace_size(S, L, K, V), dtype=torch.uint8, device=DEV)
    gpu = llc.llc_verify(target, tokens, want_keys=True, strong=True, workspace=ws, **kw)
    torch.cuda.synchronize()
    compare_verify({k: gpu[k] for k in ("Y", "n_out", "active", "keyY")}, ref)


def test_strong_form_prices_dropped_drafts_with_rows_that_are_not_vector_aligned():
    """Contiguous [S, L+1, K, V] with odd V and K = 4: the rows of drafts 1..3 start off a
    four-element boundary.  Draft 0 is dropped at position 0, so the later positions are priced
    with another draft's (unaligned) row."""
    S, L, K, V = 9, 3, 4, 2051
    g = torch.Generator(device=DEV).manual_seed(2051)
    target = 2 * torch.randn(S, L + 1, K, V, generator=g, device=DEV)
    target[:, 0, 1:] = target[:, 0, :1]
    kw = dict(temp_target=0.8, seed=12, row_offset=3)
    tokens = torch.randint(0, V, (S, L, K), generator=g, device=DEV, dtype=torch.int32)
    for _ in range(L + 1):   # drafts 1..3 follow the output, draft 0 never does
        ref = oracle_verify(target, tokens, (0, S), strong=True, **kw)
        y = torch.from_numpy(ref["Y"][:, :L].copy()).to(DEV).to(torch.int32)
        tokens[:, :, 1:] = torch.where(y[:, :, None] >= 0, y[:, :, None].expand(S, L, K - 1), tokens[:, :, 1:])
        tokens[:, :, 0] = torch.where(tokens[:, :, 0] == y, (y + 1) % V, tokens[:, :, 0])
    ref = oracle_verify(target, tokens, (0, S), strong=True, **kw)
    assert (ref["n_out"] == L + 1).all() and (ref["active"][:, 0] == 0).all()
    for dt in (torch.float32, torch.bfloat16):
        t = target.to(dt)
        r = oracle_verify(t, tokens, (0, S), strong=True, **kw)
        gpu = llc.llc_verify(t, tokens, want_keys=True, strong=True, **kw)
        torch.cuda.synchronize()
        compare_verify({k: gpu[k] for k in ("Y", "n_out", "active", "keyY")}, r)


def test_verify_results_do_not_depend_on_launch_shape():
    w = workloads.make_verify("small_bf16", DEV, sequences=5)
    base = run_verify(w, want_keys=True, want_partials=True)
    for vc, kt in ((1, 1), (3, 2), (9, 4), (2, 8)):
        other = run_verify(w, want_keys=True, want_partials=True, v_chunks=vc, k_tile=kt)
        torch.cuda.synchronize()
        for name in base:
            if name.startswith("key"):
                # the normalisers are summed chunk by chunk: the last bits may depend on the split
                torch.testing.assert_close(base[name], other[name], rtol=1e-6, atol=0)
            else:
                assert torch.equal(base[name], other[name]), name
    exact = run_verify(w, want_keys=True, want_partials=True, flags=llc.FLAG_EXACT_SCAN)
    torch.cuda.synchronize()
    for name in ("Y", "n_out", "active", "Yk"):
        assert torch.equal(base[name], exact[name]), name


@pytest.mark.parametrize("strong", [False, True])
@pytest.mark.parametrize("L,K,V", [(0, 1, 777), (0, 5, 1025), (1, 1, 4099), (5, 2, 333), (2, 64, 517), (4, 64, 130)])
def test_verify_edge_shapes(L, K, V, strong):
    g = torch.Generator(device=DEV).manual_seed(L * 1000 + K * 10 + V)
    S = 7
    target = 3 * torch.randn(S, L + 1, K, V, generator=g, device=DEV)
    target[:, 0, 1:] = target[:, 0, :1]
    tokens = target[:, :L].argmax(dim=3).to(torch.int32)
    gpu = llc.llc_verify(target, tokens, temp_target=0.6, seed=17, row_offset=5, want_keys=True, strong=strong)
    torch.cuda.synchronize()
    ref = oracle_verify(target, tokens, (0, S), temp_target=0.6, seed=17, row_offset=5, strong=strong)
    compare_verify(gpu, ref)


def test_verify_strided_views_log_weights_and_rows_without_mass():
    g = torch.Generator(device=DEV).manual_seed(41)
    S, L, K, V = 6, 3, 4, 2051
    store = 2 * torch.randn(S, K, L + 1, V + 3, generator=g, device=DEV)   # [S, K, L+1, V'] permuted, odd rows
    target = store.permute(0, 2, 1, 3)[:, :, :, 1:1 + V]
    target[:, 0, 1:] = target[:, 0, :1]
    ninf = float("-inf")
    target[1, 1, 2, :] = ninf                     # one (position, draft) row without mass
    target[2, 0, :, :] = ninf                     # position 0 without mass at all: Y = -1, loop ends
    target[3, 2, 0, 5] = float("nan")
    big_tok = torch.randint(0, V, (S, L, K + 2), generator=g, device=DEV, dtype=torch.int32)
    tokens = big_tok[:, :, :K]
    tokens[:, :, 0] = target[:, :L, 0].argmax(dim=2).to(torch.int32)
    gpu = llc.llc_verify(target, tokens, kind="logw", seed=19, want_keys=True)
    torch.cuda.synchronize()
    t, dt = to_host(target)
    ref = oracle.verify(t, tokens.cpu().numpy(), dtype=dt, kind=oracle.LOGW, seed=19)
    compare_verify(gpu, ref)
    assert gpu["Y"][2, 0].item() == -1 and gpu["n_out"][2].item() == 1


def test_verify_error_codes_on_device():
    t = torch.randn(2, 3, 2, 64, device=DEV)
    tok = torch.zeros(2, 2, 2, dtype=torch.int32, device=DEV)
    with pytest.raises(llc.LlcError) as e:
        llc.llc_verify(t, tok, kind="probs")
    assert e.value.code == -4
    with pytest.raises(llc.LlcError) as e:
        llc.llc_verify(t, tok, workspace=torch.empty(256, dtype=torch.uint8, device=DEV))
    assert e.value.code == -6
    out = llc.llc_verify(torch.empty(0, 3, 2, 64, device=DEV), torch.empty(0, 2, 2, dtype=torch.int32, device=DEV))
    assert out["Y"].shape == (0, 3)


def test_per_draft_target_side_argmins_of_algorithm_1():
    # llc_verify with L = 0 and one target row per sequence viewed K times (stride 0) returns, as
    # Yk / keyYk, Algorithm 1's per-draft target-side argmins argmin_i S_i^(k) / q_i, whose
    # minimum over k is Y: the quantities an active-set verifier keeps per draft
    g = torch.Generator(device=DEV).manual_seed(23)
    B, K, V = 33, 5, 7001
    tq = 2 * torch.randn(B, V, generator=g, device=DEV)
    view = tq[:, None, None, :].expand(B, 1, K, V)
    gpu = llc.llc_verify(view, torch.empty(B, 0, K, dtype=torch.int32, device=DEV), temp_target=0.9,
                         seed=14, row_offset=100, row_stride_s=1, want_keys=True, want_partials=True)
    torch.cuda.synchronize()
    t, dt = to_host(tq)
    ref = oracle.couple(t, t, K, dtype=dt, temp_target=0.9, temp_draft_all=0.9, seed=14, row_offset=100,
                        partials=True)
    ok = ref["gapYk"] >= NEAR_TIE
    assert np.array_equal(gpu["Yk"].cpu().numpy()[:, 0][ok], ref["Yk"][ok])
    np.testing.assert_allclose(gpu["keyYk"].cpu().numpy()[:, 0][ok], ref["keyYk"][ok], rtol=KEY_RTOL)
    clean = ref["gapY"] >= NEAR_TIE
    assert np.array_equal(gpu["Y"].cpu().numpy()[:, 0][clean], ref["Y"][clean])
    assert (gpu["n_out"] == 1).all()


@pytest.mark.parametrize("name", ["tiny", "small_bf16"])
def test_strong_variant_matches_the_oracle(name):
    # Appendix B: dropped drafts stay in the pool, priced with the first viable draft's row
    w = workloads.make_verify(name, DEV)
    gpu = run_verify(w, want_keys=True, strong=True)
    torch.cuda.synchronize()
    ref = oracle_verify(w.target, w.tokens, (0, w.S), temp_target=w.temp_target, seed=w.seed, strong=True)
    near = compare_verify({k: gpu[k] for k in ("Y", "n_out", "active", "keyY")}, ref)
    plain = oracle_verify(w.target, w.tokens, (0, w.S), temp_target=w.temp_target, seed=w.seed)
    assert near <= 1
    # the two variants differ somewhere (else this test shows nothing) and agree on the first token
    assert not np.array_equal(ref["Y"], plain["Y"])
    assert np.array_equal(ref["Y"][:, 0], plain["Y"][:, 0])


def test_strong_variant_with_coupled_drafts_row_strides_and_launch_shapes():
    g = torch.Generator(device="cpu").manual_seed(37)
    S, L, K, V = 30, 4, 5, 5000
    target = (1.5 * torch.randn(S, L + 1, K, V, generator=g)).to(DEV)
    # draft tokens that often agree with the target's sample: where `keep` is set a draft copies the
    # oracle's output of that position (found position by position), elsewhere it stays random
    tok = torch.randint(0, V, (S, L, K), generator=g, dtype=torch.int32)
    keep = torch.rand(S, L, K, generator=g) < 0.6
    kw = dict(seed=5, row_stride_s=64, row_stride_j=3, row_offset=1 << 33, strong=True)
    for _ in range(L):
        y = torch.from_numpy(oracle_verify(target, tok, (0, S), **kw)["Y"][:, :L].copy()).to(torch.int32)
        tok = torch.where(keep & (y[:, :, None] >= 0), y[:, :, None].expand(S, L, K), tok)
    tok = tok.to(DEV)
    ref = oracle_verify(target, tok, (0, S), **kw)
    assert ref["n_out"].max() > 2
    for vc, kt in ((0, 0), (3, 2), (1, 8)):
        gpu = llc.llc_verify(target, tok, seed=5, row_stride_s=64, row_stride_j=3, row_offset=1 << 33,
                             want_keys=True, strong=True, v_chunks=vc, k_tile=kt)
        torch.cuda.synchronize()
        compare_verify({k: gpu[k] for k in ("Y", "n_out", "active", "keyY")}, ref)


def test_strong_variant_ignores_the_draft_tokens_in_distribution_of_the_first_miss():
    # with no draft ever matching, the loop stops after the first token in both variants
    w = workloads.make_verify("tiny", DEV)
    tok = torch.full_like(w.tokens, -5)
    a = llc.llc_verify(w.target, tok, temp_target=w.temp_target, seed=w.seed, strong=True)
    b = llc.llc_verify(w.target, tok, temp_target=w.temp_target, seed=w.seed)
    torch.cuda.synchronize()
    assert torch.equal(a["Y"], b["Y"]) and (a["n_out"] == 1).all() and (a["active"] == 0).all()


def test_strong_variant_through_the_all_fp64_scan():
    # the debugging flag and the strong flag combine: same tokens from the scan without a prefilter
    w = workloads.make_verify("tiny", DEV)
    a = run_verify(w, strong=True)
    b = run_verify(w, strong=True, flags=llc.FLAG_EXACT_SCAN)
    torch.cuda.synchronize()
    for name in ("Y", "n_out", "active"):
        assert torch.equal(a[name], b[name]), name

"""GPU parity: the HIP path against the CPU oracle, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2506_05632_amd as llc
from paper_2506_05632_amd import workloads
from parity_util import check_all_rows, compare, oracle_borderline, oracle_near_ties, oracle_rows, same_outputs, stats_dict, to_host

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_gpu(w, **kw):
    kind = kw.pop("kind", w.kind)
    if kind == "logw" and kw.pop("is_form", False):
        return llc.llc_couple_is(w.target, w.draft, seed=w.seed, row_offset=w.row_offset, **kw)
    return llc.llc_couple(w.draft, w.target, w.K, kind=kind, temp_target=w.temp_target,
                          temp_draft=w.temp_draft, seed=w.seed, row_offset=w.row_offset, **kw)


# ------------------------------------------------------------------ the five configurations, every row
def test_config1_tiny_full():
    w = workloads.make(1, DEV)
    stats = llc.new_stats(DEV)
    gpu = run_gpu(w, want_keys=True, stats=stats)
    torch.cuda.synchronize()
    s = check_all_rows(w, gpu, stats, w.B)
    assert s["degenerate"] == 0


def test_config2_specdec_bf16_full():
    w = workloads.make(2, DEV)
    stats = llc.new_stats(DEV)
    gpu = run_gpu(w, want_keys=True, stats=stats)
    torch.cuda.synchronize()
    check_all_rows(w, gpu, stats, w.B)


def test_config3_large_vocab_full():
    w = workloads.make(3, DEV)
    stats = llc.new_stats(DEV)
    gpu_nokeys = run_gpu(w, stats=stats)                # the launch configuration bench.py times
    gpu = run_gpu(w, want_keys=True)
    torch.cuda.synchronize()
    for name in ("X", "Y", "accept", "match_k"):
        assert torch.equal(gpu[name], gpu_nokeys[name])
    check_all_rows(w, gpu, stats, 128)
    assert gpu["accept"].float().mean().item() > 0.5


def test_config4_distinct_drafters_full():
    w = workloads.make(4, DEV)
    stats = llc.new_stats(DEV)
    gpu = run_gpu(w, want_keys=True, stats=stats)
    torch.cuda.synchronize()
    check_all_rows(w, gpu, stats, 64)


def test_config5_importance_form_full():
    w = workloads.make(5, DEV)
    stats = llc.new_stats(DEV)
    gpu = run_gpu(w, is_form=True, want_keys=True, stats=stats)
    torch.cuda.synchronize()
    via_couple = run_gpu(w, want_keys=True)
    torch.cuda.synchronize()
    same_outputs({k: gpu[k] for k in ("X", "Y", "accept", "match_k")},
                 {k: via_couple[k] for k in ("X", "Y", "accept", "match_k")})
    check_all_rows(w, gpu, stats, 512, is_form=True)


def test_near_tie_counter_against_the_oracle_on_millions_of_small_races():
    """A race ends within 1e-6 of its runner-up with probability about 1e-6 whatever the
    distributions are (the gap after the first arrival of a Poisson process, relative to the first
    arrival time), so near-ties cannot be planted through the inputs; they can be made to occur by
    sheer number: 2^21 rows of 8 nearly equiprobable entries and 15 drafts are 33 million reductions,
    a few dozen of which are near-ties.  The device's counter must find exactly the oracle's, on the prefiltered path and
    on the all-fp64 one."""
    g = torch.Generator(device=DEV).manual_seed(77)
    B, V, K = 1 << 21, 8, 15
    tq = 0.3 * torch.randn(B, V, generator=g, device=DEV)
    td = tq + 0.3 * torch.randn(B, V, generator=g, device=DEV)
    ref = oracle_rows(td, tq, K, (0, B), kind="logits", temp_target=0.9, temp_draft=1.2, seed=3)
    want = oracle_near_ties(ref)
    assert want >= 5, "the recipe is meant to contain near-ties"
    for kw in (dict(), dict(flags=llc.FLAG_EXACT_SCAN), dict(k_tile=4)):
        stats = llc.new_stats(DEV)
        gpu = llc.llc_couple(td, tq, K, temp_target=0.9, temp_draft=1.2, seed=3, want_keys=True, stats=stats, **kw)
        torch.cuda.synchronize()
        excused = compare(gpu, ref)
        got = stats_dict(stats)["near_ties"]
        print(f"33M small races: near-ties oracle {want}, device {got}, excused mismatches {excused}")
        assert abs(got - want) <= oracle_borderline(ref) and excused <= want


# ------------------------------------------------------------------ shape independence
def test_results_do_not_depend_on_launch_shape():
    w = workloads.make(2, DEV, rows=24)
    base = run_gpu(w, want_keys=True)
    for vc in (1, 2, 5, 32):
        for kt in (1, 2, 4, 8):
            ws = llc.new_workspace(w.B, w.K, w.V, DEV, v_chunks=vc)
            other = run_gpu(w, want_keys=True, v_chunks=vc, k_tile=kt, workspace=ws)
            torch.cuda.synchronize()
            same_outputs(base, other)
    exact = run_gpu(w, want_keys=True, flags=llc.FLAG_EXACT_SCAN)
    torch.cuda.synchronize()
    same_outputs({k: base[k] for k in ("X", "Y", "accept", "match_k")},
                 {k: exact[k] for k in ("X", "Y", "accept", "match_k")})
    np.testing.assert_allclose(base["keyX"].cpu().numpy(), exact["keyX"].cpu().numpy(), rtol=1e-6)


def test_distinct_layout_launch_shapes_and_exact_scan():
    w = workloads.make(4, DEV, rows=6)
    base = run_gpu(w)
    for vc, kt in ((3, 1), (1, 2), (7, 4), (2, 8)):
        other = run_gpu(w, v_chunks=vc, k_tile=kt)
        torch.cuda.synchronize()
        same_outputs(base, other)
    exact = run_gpu(w, flags=llc.FLAG_EXACT_SCAN)
    torch.cuda.synchronize()
    same_outputs(base, exact)


# ------------------------------------------------------------------ edge cases
@pytest.mark.parametrize("V", [1, 3, 5, 255, 1001, 1023, 1025, 4099])
@pytest.mark.parametrize("K", [1, 3])
def test_ragged_vocab_sizes(V, K):
    g = torch.Generator(device=DEV).manual_seed(V * 10 + K)
    B = 37
    tq = 2 * torch.randn(B, V, generator=g, device=DEV)
    td = tq + torch.randn(B, V, generator=g, device=DEV)
    gpu = llc.llc_couple(td, tq, K, seed=5, want_keys=True)
    torch.cuda.synchronize()
    ref = oracle_rows(td, tq, K, (0, B), kind="logits", temp_target=1.0, temp_draft=1.0, seed=5)
    compare(gpu, ref)


@pytest.mark.parametrize("K", [1, 2, 5, 8, 9, 17, 40])
@pytest.mark.parametrize("shared", [True, False])
def test_draft_counts(K, shared):
    g = torch.Generator(device=DEV).manual_seed(K + (100 if shared else 0))
    B, V = 9, 3000
    tq = 2 * torch.randn(B, V, generator=g, device=DEV)
    td = tq + torch.randn(B, V, generator=g, device=DEV) if shared else \
        tq[:, None, :] + torch.randn(B, K, V, generator=g, device=DEV)
    gpu = llc.llc_couple(td, tq, K, seed=77, row_offset=(1 << 35) + 3, want_keys=True,
                         temp_target=0.8, temp_draft=1.3)
    torch.cuda.synchronize()
    ref = oracle_rows(td, tq, K, (0, B), kind="logits", temp_target=0.8, temp_draft=1.3, seed=77,
                      row_offset=(1 << 35) + 3)
    compare(gpu, ref)


def test_unaligned_rows_and_strided_views():
    g = torch.Generator(device=DEV).manual_seed(3)
    B, V, K = 11, 2049, 3
    big_q = torch.randn(B, V + 7, generator=g, device=DEV)
    big_d = torch.randn(B, K, V + 5, generator=g, device=DEV)
    tq, td = big_q[:, 3:3 + V], big_d[:, :, 1:1 + V]          # odd offsets, odd strides
    gpu = llc.llc_couple(td, tq, K, seed=9, want_keys=True)
    torch.cuda.synchronize()
    ref = oracle_rows(td, tq, K, (0, B), kind="logits", temp_target=1.0, temp_draft=1.0, seed=9)
    compare(gpu, ref)
    bq, bd = big_q.to(torch.bfloat16), big_d.to(torch.bfloat16)
    tq, td = bq[:, 3:3 + V], bd[:, :, 1:1 + V]
    gpu = llc.llc_couple(td, tq, K, seed=9, want_keys=True)
    torch.cuda.synchronize()
    ref = oracle_rows(td, tq, K, (0, B), kind="logits", temp_target=1.0, temp_draft=1.0, seed=9)
    compare(gpu, ref)


def test_probability_inputs():
    g = torch.Generator(device=DEV).manual_seed(4)
    B, V, K = 40, 5000, 4
    q = torch.rand(B, V, generator=g, device=DEV) ** 8
    p = torch.rand(B, K, V, generator=g, device=DEV) ** 8
    p[:, :, ::7] = 0.0
    q[:, 5::11] = 0.0
    p[0, 0, 1] = float("nan"); p[0, 1, 2] = -1.0; q[1, 3] = float("inf")
    for pp in (p, p[:, 0].contiguous()):
        gpu = llc.llc_couple(pp, q, K, kind="probs", seed=11, want_keys=True)
        torch.cuda.synchronize()
        ref = oracle_rows(pp, q, K, (0, B), kind="probs", temp_target=1.0, temp_draft=1.0, seed=11)
        compare(gpu, ref)
    gpu = llc.llc_couple(p.to(torch.bfloat16), q.to(torch.bfloat16), K, kind="probs", seed=11, want_keys=True)
    torch.cuda.synchronize()
    ref = oracle_rows(p.to(torch.bfloat16), q.to(torch.bfloat16), K, (0, B), kind="probs",
                      temp_target=1.0, temp_draft=1.0, seed=11)
    compare(gpu, ref)


def test_per_draft_temperatures():
    g = torch.Generator(device=DEV).manual_seed(6)
    B, V, K = 20, 4000, 5
    tq = 2 * torch.randn(B, V, generator=g, device=DEV)
    td = tq + torch.randn(B, V, generator=g, device=DEV)
    temps = torch.tensor([0.5, 1.0, 1.5, 2.0, 0.7], dtype=torch.float32, device=DEV)
    gpu = llc.llc_couple(td, tq, K, temp_target=2.0, temp_draft_per_k=temps, seed=13, want_keys=True)
    torch.cuda.synchronize()
    ref = oracle_rows(td, tq, K, (0, B), kind="logits", temp_target=2.0, temp_draft=1.0,
                      temp_draft_per_k=temps, seed=13)
    compare(gpu, ref)


def test_masked_degenerate_and_one_hot_rows():
    g = torch.Generator(device=DEV).manual_seed(8)
    B, V, K = 8, 3001, 3
    tq = torch.randn(B, V, generator=g, device=DEV)
    td = torch.randn(B, V, generator=g, device=DEV)
    ninf = float("-inf")
    tq[0, :] = ninf                              # target has no mass: Y = -1, accept = 0
    td[1, :] = ninf                              # draft has no mass: X = -1
    tq[2, :] = ninf; tq[2, 1234] = 0.0           # one atom each
    td[2, :] = ninf; td[2, 1234] = 3.0
    td[3, :] = ninf; td[3, 3000] = 0.0           # one-hot proposal in the ragged tail
    tq[4, 100:] = ninf                           # mass only in the first tile
    td[5, :2900] = ninf                          # mass only at the end
    tq[6, 7] = float("nan"); td[6, 9] = float("inf")
    stats = llc.new_stats(DEV)
    gpu = llc.llc_couple(td, tq, K, seed=21, want_keys=True, stats=stats)
    torch.cuda.synchronize()
    ref = oracle_rows(td, tq, K, (0, B), kind="logits", temp_target=1.0, temp_draft=1.0, seed=21)
    compare(gpu, ref)
    assert gpu["Y"][0].item() == -1 and gpu["accept"][0].item() == 0
    assert (gpu["X"][1] == -1).all() and (gpu["X"][3] == 3000).all()
    assert stats_dict(stats)["degenerate"] == 1 + K


@pytest.mark.parametrize("K,shared", [(300, True), (70, False), (1000, True), (65535, True), (65535, False)])
def test_many_drafts(K, shared):
    # many draft groups per row: the pool's bound and argmin are merged over all of them
    # (65535 is the most the interface takes)
    g = torch.Generator(device=DEV).manual_seed(K)
    B, V = (3, 700) if K < 10000 else (2, 37)
    tq = 2 * torch.randn(B, V, generator=g, device=DEV)
    td = tq + torch.randn(B, V, generator=g, device=DEV) if shared else \
        tq[:, None, :] + torch.randn(B, K, V, generator=g, device=DEV)
    gpu = llc.llc_couple(td, tq, K, seed=19, want_keys=True)
    torch.cuda.synchronize()
    ref = oracle_rows(td, tq, K, (0, B), kind="logits", temp_target=1.0, temp_draft=1.0, seed=19)
    compare(gpu, ref)


def test_one_very_long_row_is_spread_over_a_thousand_workgroups():
    # a single row of five million entries: the planner cuts it into the most chunks it allows
    g = torch.Generator(device=DEV).manual_seed(55)
    V, K = 5_000_011, 3
    tq = 2 * torch.randn(1, V, generator=g, device=DEV)
    td = tq + torch.randn(1, V, generator=g, device=DEV)
    stats = llc.new_stats(DEV)
    gpu = llc.llc_couple(td, tq, K, seed=2, want_keys=True, stats=stats)
    torch.cuda.synchronize()
    ref = oracle_rows(td, tq, K, (0, 1), kind="logits", temp_target=1.0, temp_draft=1.0, seed=2)
    compare(gpu, ref)
    assert stats_dict(stats)["slow_blocks"] == 0  # no workgroup fell back to the all-fp64 scan


def test_the_longest_row_the_interface_accepts():
    """V = 2^31 - 5, the largest the ABI takes: 32-bit index arithmetic at its limit.  The mass sits
    on a few thousand entries (the first and the last ones among them), so the oracle's candidate-
    list form, whose uniforms are keyed by the same indices, gives the expected result."""
    import oracle
    V, K, M = 2**31 - 5, 3, 4000
    g = torch.Generator(device=DEV).manual_seed(91)
    ids = torch.randint(0, V, (M,), generator=g, device=DEV, dtype=torch.int64)
    ids = torch.cat([ids, torch.arange(0, 6, device=DEV), torch.arange(V - 6, V, device=DEV)]).unique()
    vq = 2 * torch.randn(ids.numel(), generator=g, device=DEV)
    vd = vq + torch.randn(ids.numel(), generator=g, device=DEV)
    tq = torch.full((1, V), -float("inf"), device=DEV)
    td = torch.full((1, V), -float("inf"), device=DEV)
    tq[0, ids] = vq
    td[0, ids] = vd
    ids32 = ids.to(torch.int32).cpu().numpy().reshape(1, -1)
    ref = oracle.couple_topm(ids32, vd.cpu().numpy().reshape(1, -1), ids32, vq.cpu().numpy().reshape(1, -1), K,
                             kind=oracle.LOGITS, temp_target=0.9, temp_draft_all=1.1, seed=17)
    for kw in (dict(), dict(flags=llc.FLAG_EXACT_SCAN)):
        stats = llc.new_stats(DEV)
        gpu = llc.llc_couple(td, tq, K, seed=17, temp_target=0.9, temp_draft=1.1, want_keys=True, stats=stats, **kw)
        torch.cuda.synchronize()
        compare(gpu, ref)
    del tq, td
    torch.cuda.empty_cache()


def test_identical_distributions_always_accept():
    g = torch.Generator(device=DEV).manual_seed(10)
    z = 3 * torch.randn(300, 7001, generator=g, device=DEV)
    for K in (1, 4, 8):
        out = llc.llc_couple(z, z, K, temp_target=0.9, temp_draft=0.9, seed=K)
        assert out["accept"].all().item()


def test_target_sample_ignores_the_drafts():
    g = torch.Generator(device=DEV).manual_seed(12)
    B, V, K = 64, 9000, 4
    tq = 2 * torch.randn(B, V, generator=g, device=DEV)
    a = llc.llc_couple(torch.randn(B, V, generator=g, device=DEV), tq, K, seed=3, want_keys=True)
    b = llc.llc_couple(5 * torch.randn(B, K, V, generator=g, device=DEV), tq, K, seed=3, want_keys=True,
                       temp_draft=3.0)
    assert torch.equal(a["Y"], b["Y"])
    # (the target row's normaliser is summed by different kernels for the two draft layouts: the
    # reported key may differ in its last bits, far inside the 1e-6 that keys are held to)
    torch.testing.assert_close(a["keyY"], b["keyY"], rtol=1e-6, atol=0)


def test_extreme_logits_fall_back_to_the_exact_scan():
    g = torch.Generator(device=DEV).manual_seed(14)
    B, V, K = 6, 5000, 2
    tq = torch.randn(B, V, generator=g, device=DEV)
    td = tq + torch.randn(B, V, generator=g, device=DEV)
    tq[:3] += 4000.0
    td[3:] -= 2500.0
    stats = llc.new_stats(DEV)
    gpu = llc.llc_couple(td, tq, K, seed=23, want_keys=True, stats=stats)
    torch.cuda.synchronize()
    ref = oracle_rows(td, tq, K, (0, B), kind="logits", temp_target=1.0, temp_draft=1.0, seed=23)
    compare(gpu, ref)
    assert stats_dict(stats)["slow_blocks"] > 0


def test_sorted_logits_overflow_the_candidate_list():
    # steeply increasing probabilities make almost every element a new running minimum
    B, V, K = 4, 40000, 2
    z = torch.arange(V, dtype=torch.float32, device=DEV)[None, :].repeat(B, 1) * 0.01
    stats = llc.new_stats(DEV)
    gpu = llc.llc_couple(z, z.flip(1).contiguous(), K, seed=25, want_keys=True, stats=stats, v_chunks=1)
    torch.cuda.synchronize()
    ref = oracle_rows(z, z.flip(1).contiguous(), K, (0, B), kind="logits", temp_target=1.0,
                      temp_draft=1.0, seed=25)
    compare(gpu, ref)


def test_empty_batch_and_error_codes_on_device():
    out = llc.llc_couple(torch.empty(0, 16, device=DEV), torch.empty(0, 16, device=DEV), 2)
    assert out["X"].shape == (0, 2)
    with pytest.raises(llc.LlcError) as e:
        llc.llc_couple(torch.randn(2, 16, device=DEV), torch.randn(2, 16, device=DEV), 2, temp_target=0.0)
    assert e.value.code == -3
    with pytest.raises(llc.LlcError) as e:
        llc.llc_couple(torch.randn(2, 16, device=DEV), torch.randn(2, 16, device=DEV), 2,
                       workspace=torch.empty(256, dtype=torch.uint8, device=DEV))
    assert e.value.code == -6

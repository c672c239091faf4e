"""GPU parity of llc_compress_select (binned index selection of the compression scheme) against the
CPU oracle, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2506_05632_amd as llc
from paper_2506_05632_amd import workloads
from parity_util import KEY_RTOL, NEAR_TIE, oracle_borderline, oracle_near_ties, stats_dict

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def compare_select(gpu, ref, rows=None):
    g = {k: v.detach().cpu().numpy() for k, v in gpu.items()}
    if rows is not None:
        g = {k: v[rows[0]:rows[1]] for k, v in g.items()}
    near = 0
    for b in range(ref["Y"].shape[0]):
        if g["Y"][b] != ref["Y"][b]:
            assert ref["gapY"][b] < NEAR_TIE, f"Y[{b}] gpu {g['Y'][b]} ref {ref['Y'][b]} gap {ref['gapY'][b]}"
            near += 1
            continue                      # another Y announces another bin: the decoders differ
        assert g["message"][b] == ref["message"][b]
        clean = True
        for l in range(ref["X"].shape[1]):
            if g["X"][b, l] != ref["X"][b, l]:
                assert ref["gapX"][b, l] < NEAR_TIE, f"X[{b},{l}] gpu {g['X'][b, l]} ref {ref['X'][b, l]}"
                near += 1
                clean = False
            elif "keyX" in g:
                if ref["X"][b, l] >= 0:
                    np.testing.assert_allclose(g["keyX"][b, l], ref["keyX"][b, l], rtol=KEY_RTOL)
                else:
                    assert np.isinf(g["keyX"][b, l])
        if clean:
            assert g["accept"][b] == ref["accept"][b] and g["match_k"][b] == ref["match_k"][b]
        if "keyY" in g and ref["Y"][b] >= 0:
            np.testing.assert_allclose(g["keyY"][b], ref["keyY"][b], rtol=KEY_RTOL)
    return near


def _case(B, L, N, l_max, seed, shared_dec=False):
    g = torch.Generator(device=DEV).manual_seed(seed)
    enc = 2 * torch.randn(B, N, generator=g, device=DEV)
    dec = enc[:, None, :] + 1.5 * torch.randn(B, 1 if shared_dec else L, N, generator=g, device=DEV)
    if shared_dec:
        dec = dec.expand(B, L, N)
    bins = torch.randint(0, l_max, (B, N), generator=g, device=DEV, dtype=torch.uint8)
    return enc, dec, bins


@pytest.mark.parametrize("B,L,N,l_max", [(30, 4, 5000, 8), (9, 1, 1023, 2), (5, 7, 4099, 64), (3, 2, 77, 256),
                                         (40, 16, 3000, 4)])
def test_compress_select_shapes(B, L, N, l_max):
    enc, dec, bins = _case(B, L, N, l_max, seed=B * 100 + L)
    stats = llc.new_stats(DEV)
    gpu = llc.llc_compress_select(enc, dec, bins, seed=3, row_offset=(1 << 36) + 1, want_keys=True, stats=stats)
    torch.cuda.synchronize()
    ref = oracle.compress_select(enc.cpu().numpy(), dec.cpu().numpy(), bins.cpu().numpy(), seed=3,
                                 row_offset=(1 << 36) + 1)
    compare_select(gpu, ref)
    assert stats_dict(stats)["slow_blocks"] == 0
    # every decoder answers inside the announced bin
    X, msg = gpu["X"].long(), gpu["message"]
    ok = X >= 0
    assert (torch.gather(bins.long(), 1, X.clamp(min=0))[ok] == msg[:, None].expand_as(X)[ok]).all()


def test_compress_select_single_bin_is_llc_couple_is_and_launch_shapes_do_not_matter():
    enc, dec, bins = _case(12, 4, 9000, 16, seed=7)
    one = llc.llc_compress_select(enc, dec, torch.zeros_like(bins), seed=5, want_keys=True)
    plain = llc.llc_couple_is(enc, dec, seed=5, want_keys=True)
    for name in ("X", "Y", "accept", "match_k"):
        assert torch.equal(one[name], plain[name]), name
    for name in ("keyX", "keyY"):   # normalisers summed in another order: equal up to the last bits
        torch.testing.assert_close(one[name], plain[name], rtol=1e-6, atol=0)
    base = llc.llc_compress_select(enc, dec, bins, seed=5, want_keys=True)
    for vc, kt in ((1, 2), (3, 4), (7, 8)):
        other = llc.llc_compress_select(enc, dec, bins, seed=5, want_keys=True, v_chunks=vc, k_tile=kt)
        torch.cuda.synchronize()
        for name in base:
            assert torch.equal(base[name], other[name]), name
    exact = llc.llc_compress_select(enc, dec, bins, seed=5, flags=llc.FLAG_EXACT_SCAN)
    for name in ("X", "Y", "message", "accept"):
        assert torch.equal(base[name], exact[name]), name


def test_compress_select_shared_decoder_weights_strided_views_and_empty_bins():
    enc, dec, bins = _case(10, 3, 2050, 5, seed=9, shared_dec=True)          # dec_stride_l == 0
    gpu = llc.llc_compress_select(enc, dec, bins, seed=8, want_keys=True)
    torch.cuda.synchronize()
    ref = oracle.compress_select(enc.cpu().numpy(), dec.contiguous().cpu().numpy(), bins.cpu().numpy(), seed=8)
    compare_select(gpu, ref)
    # odd strides / offsets, a decoder without mass in the announced bin, an encoder without mass
    big_e = torch.randn(10, 2057, device=DEV); big_d = torch.randn(10, 3, 2061, device=DEV)
    big_b = torch.randint(0, 5, (10, 2055), device=DEV, dtype=torch.uint8)
    e, d, b = big_e[:, 3:2053], big_d[:, :, 1:2051], big_b[:, 1:2051]
    d[1, 2, :] = float("-inf")
    e[2, :] = float("-inf")
    gpu = llc.llc_compress_select(e, d, b, seed=8, want_keys=True)
    torch.cuda.synchronize()
    ref = oracle.compress_select(e.contiguous().cpu().numpy(), d.contiguous().cpu().numpy(),
                                 b.contiguous().cpu().numpy(), seed=8)
    compare_select(gpu, ref)
    assert gpu["X"][1, 2].item() == -1 and gpu["Y"][2].item() == -1 and gpu["message"][2].item() == -1
    assert (gpu["X"][2] == -1).all() and gpu["accept"][2].item() == 0


def test_compress_select_config5_with_bins_full():
    w = workloads.make(5, DEV)                       # the importance-form workload, now with 16 bins
    g = torch.Generator(device=DEV).manual_seed(77)
    bins = torch.randint(0, 16, (w.B, w.V), generator=g, device=DEV, dtype=torch.uint8)
    stats = llc.new_stats(DEV)
    gpu = llc.llc_compress_select(w.target, w.draft, bins, seed=w.seed, want_keys=True, stats=stats)
    torch.cuda.synchronize()
    excused, near_oracle, borderline = 0, 0, 0
    for r0 in range(0, w.B, 512):                    # every row, 512 at a time (host memory)
        rows = (r0, min(w.B, r0 + 512))
        ref = oracle.compress_select(w.target[rows[0]:rows[1]].cpu().numpy(), w.draft[rows[0]:rows[1]].cpu().numpy(),
                                     bins[rows[0]:rows[1]].cpu().numpy(), seed=w.seed, row_offset=rows[0])
        excused += compare_select(gpu, ref, rows)
        near_oracle += oracle_near_ties(ref)
        borderline += oracle_borderline(ref)
    s = stats_dict(stats)
    print(f"config5 + 16 bins: {w.B} rows compared, excused mismatches {excused}, near-ties oracle {near_oracle} / "
          f"device {s['near_ties']}, survivors {s['survivors']}, exact {s['exact_evals']}, slow blocks {s['slow_blocks']}, "
          f"match rate {gpu['accept'].float().mean().item():.3f}")
    assert s["slow_blocks"] == 0
    assert abs(s["near_ties"] - near_oracle) <= borderline and near_oracle <= 2 and excused <= near_oracle

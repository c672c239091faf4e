"""llc_couple_static (the entry point for callers that cannot allocate) against llc_couple, through
the C ABI, on two calls in a row that share the library's static scratch (needs an MI355X)."""
import ctypes

import pytest
import torch

import paper_2506_05632_amd as llc
from paper_2506_05632_amd import binding, workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _outputs(B, K, keys):
    out = {"X": torch.full((B, K), -7, dtype=torch.int32, device=DEV),
           "Y": torch.full((B,), -7, dtype=torch.int32, device=DEV),
           "accept": torch.full((B,), 9, dtype=torch.uint8, device=DEV),
           "match_k": torch.full((B,), -7, dtype=torch.int32, device=DEV)}
    if keys:
        out["keyX"] = torch.zeros(B, K, dtype=torch.float32, device=DEV)
        out["keyY"] = torch.zeros(B, dtype=torch.float32, device=DEV)
    return out


def _both(draft, target, K, **kw):
    B = target.shape[0]
    want = llc.llc_couple(draft, target, K, out=_outputs(B, K, True), **kw)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated(DEV)
    got = llc.llc_couple_static(draft, target, K, out=_outputs(B, K, True), **kw)
    torch.cuda.synchronize()
    for name in want:     # the same kernels on the same inputs: identical bits, keys included
        assert torch.equal(got[name], want[name]), name
    return before


def test_two_calls_in_a_row_the_second_smaller():
    # first call: config 2's shape (bf16, rows spread over several workgroups, so the rows' shared
    # running bests in the scratch are in use); second call: fewer, shorter rows, other layout
    w = workloads.make(2, DEV)
    _both(w.draft, w.target, w.K, temp_target=w.temp_target, temp_draft=w.temp_draft, seed=w.seed)
    g = torch.Generator(device=DEV).manual_seed(5)
    B, V, K = 37, 1001, 3
    tq = 2 * torch.randn(B, V, generator=g, device=DEV)
    td = tq[:, None, :] + torch.randn(B, K, V, generator=g, device=DEV)
    _both(td, tq, K, seed=11, temp_target=0.9, temp_draft=1.1)
    # and the first shape once more, after the smaller call has left its results in the array
    _both(w.draft, w.target, w.K, temp_target=w.temp_target, temp_draft=w.temp_draft, seed=w.seed + 1)
    # the race times drawn min-first go through the same entry point
    _both(td, tq, K, seed=11, temp_target=0.9, temp_draft=1.1, flags=llc.FLAG_MIN_FIRST)


def test_the_headline_shape_fits_and_an_oversized_one_is_refused_up_front():
    w = workloads.make(3, DEV, rows=64)
    _both(w.draft, w.target, w.K, temp_target=w.temp_target, temp_draft=w.temp_draft, seed=w.seed)
    lib = llc.load()
    a = binding.CoupleArgs()
    a.B, a.K, a.V = 1 << 20, 16, 64           # partial results of 2^24 (row, draft) pairs: far too many
    a.dtype, a.kind = binding.F32, binding.LOGITS
    a.draft = a.target = 0x1000
    a.draft_stride_b = a.target_stride_b = 64
    a.temp_target = a.temp_draft_all = 1.0
    a.X = a.Y = a.accept = 0x2000
    assert lib.llc_couple_static(ctypes.byref(a)) == -9    # found on the host: nothing was launched
    assert "static scratch" in llc.llc_status_string(-9)
    a.B, a.K, a.V = 1024, 8, 128256                        # the headline configuration fits
    a.draft_stride_b = a.target_stride_b = 128256
    a.flags = binding.FLAG_DRY_RUN
    assert lib.llc_couple_static(ctypes.byref(a)) == 0

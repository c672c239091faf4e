"""llc_couple on a few hundred randomly drawn valid shapes and options against the oracle (needs an MI355X).

The other parity files pick their cases by what they are meant to exercise; this one draws them:
rows, drafts, vocabulary sizes around the tile and chunk boundaries, both layouts and input types,
both ways of drawing the race times, keys or not, temperatures, launch shapes, row offsets, rows
whose first third carries no mass, logits far from zero.  Same bar as everywhere: indices and
flags bit for bit (near-ties excused and counted), keys to 1e-6."""
import random

import pytest
import torch

import paper_2506_05632_amd as llc
from parity_util import compare, oracle_near_ties, oracle_rows

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("seed", [1, 2])
def test_random_shapes_and_options(seed):
    rng = random.Random(seed)
    for case in range(120):
        B = rng.choice([1, 2, 3, 7, 16, 33])
        K = rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 16, 19])
        V = rng.choice([1, 5, 63, 64, 1000, 1023, 1024, 1025, 4097, 20011, 50000, 70001])
        shared = rng.random() < 0.5
        dtype = rng.choice([torch.float32, torch.bfloat16])
        min_first = rng.random() < 0.6
        keys = rng.random() < 0.7
        temp_target, temp_draft = rng.choice([0.3, 0.7, 1.0, 2.5]), rng.choice([0.3, 0.7, 1.0, 2.5])
        v_chunks, k_tile = rng.choice([0, 0, 1, 2, 5]), rng.choice([0, 0, 2, 4, 8])
        g = torch.Generator(device=DEV).manual_seed(1000 * seed + case)
        tq = rng.choice([0.5, 2.0, 6.0]) * torch.randn(B, V, generator=g, device=DEV) + rng.choice([0.0, -40.0, 30.0])
        if rng.random() < 0.3:
            tq[:, : V // 3] = float("-inf")
        if shared:
            draft = tq + 0.5 * torch.randn(B, V, generator=g, device=DEV)
        else:
            draft = tq[:, None, :] + 0.7 * torch.randn(B, K, V, generator=g, device=DEV)
        tq, draft = tq.to(dtype), draft.to(dtype)
        stream_seed, row_offset = rng.randrange(1 << 40), rng.choice([0, 5, 1 << 33])
        what = (f"case {case}: B={B} K={K} V={V} shared={shared} {dtype} min_first={min_first} keys={keys} "
                f"T={temp_target}/{temp_draft} v_chunks={v_chunks} k_tile={k_tile}")
        out = llc.llc_couple(draft, tq, K, temp_target=temp_target, temp_draft=temp_draft, seed=stream_seed,
                             row_offset=row_offset, want_keys=keys, v_chunks=v_chunks, k_tile=k_tile,
                             workspace=llc.new_workspace(B, K, V, DEV, v_chunks=v_chunks),
                             flags=llc.FLAG_MIN_FIRST if min_first else 0)
        torch.cuda.synchronize()
        ref = oracle_rows(draft, tq, K, (0, B), kind="logits", temp_target=temp_target, temp_draft=temp_draft,
                          seed=stream_seed, row_offset=row_offset, min_first=min_first)
        try:
            excused = compare(out, ref)
        except AssertionError as err:
            raise AssertionError(what + ": " + str(err)[:400]) from None
        assert excused <= oracle_near_ties(ref), what

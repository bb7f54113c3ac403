"""ds_eval_noalloc (scratch in a static device array, no allocation) against ds_eval, through the C ABI:
two calls in a row on one context, the second on a smaller input, each compared with ds_eval's output."""
import numpy as np
import pytest

from oracle import sampling
from synth import make_workload
from tests.gpu_common import make_context, say

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _masks(n, rows, seed):
    rng = np.random.default_rng(seed)
    bits = np.zeros((rows, n), dtype=bool)
    bits[1] = True
    for i in range(2, rows):
        bits[i] = rng.random(n) < rng.random() ** 2
    return torch.from_numpy(sampling.pack_rows(bits).view(np.int64)).cuda()


def test_eval_noalloc_matches_eval_twice_second_call_smaller():
    from paper_2506_22668_amd import DistShapError, DS_ECAPACITY
    w = make_workload("c2_small")
    ctx = make_context(w)
    cg = ctx.extract(w.targets[0])
    n = ctx.cgraph_info(cg).num_players
    # first call: enough rows for the one-coalition-per-lane kernel (its per-workgroup scratch is what the static
    # array has to hold); second call: fewer rows, which also takes the one-workgroup-per-coalition kernel
    for rows, seed in ((1500, 1), (100, 2)):
        say(f"eval_noalloc c2_small rows={rows}")
        Z = _masks(n, rows, seed)
        ref, _ = ctx.eval(cg, Z)
        y = torch.full((rows,), float("nan"), dtype=torch.float32, device="cuda")
        ctx.eval_noalloc(cg, Z, y)
        ctx.synchronize()
        err = (y - ref).abs().max().item()
        say(f"  max |noalloc - eval| = {err:.3e}")
        assert torch.isfinite(y).all() and err <= 1e-5
    ctx.cgraph_free(cg)
    ctx.close()
    # a second, smaller graph on a fresh context of the same process (the array is shared per GPU)
    w2 = make_workload("c1")
    ctx2 = make_context(w2)
    cg2 = ctx2.extract(0)
    n2 = ctx2.cgraph_info(cg2).num_players
    Z = _masks(n2, 300, 3)
    ref, _ = ctx2.eval(cg2, Z)
    y = torch.empty(300, dtype=torch.float32, device="cuda")
    ctx2.eval_noalloc(cg2, Z, y)
    ctx2.synchronize()
    assert (y - ref).abs().max().item() <= 1e-5
    with pytest.raises(DistShapError):
        ctx2.eval_noalloc(cg2, Z, y, score=9)
    ctx2.cgraph_free(cg2)
    ctx2.close()

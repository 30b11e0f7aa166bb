"""The benchmark configurations at full size, in the launch configuration bench.py times: one
training step from identical state compared with the oracle in full (active sets bit-exact; logits,
errors, hidden gradient, Adam state and weights within tolerance), plus sampled buckets."""
import time

import numpy as np
import pytest

from paper_2201_12667_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("needs a GPU", allow_module_level=True)

from helpers import assert_ok, compare_step, make_pair  # noqa: E402


def _say(*a):
    print(*a, flush=True)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("i", [1, 2, 3, 4])
def test_full_size_step(i):
    wl = synth.config(i)
    t0 = time.time()
    _say("full-size", wl.name, "building model + oracle")
    gen, model, orc = make_pair(wl)
    model.build_tables()
    torch.cuda.synchronize()
    _say("  gpu tables built", round(time.time() - t0, 1), "s")
    T = orc.build_tables()
    _say("  oracle tables built", round(time.time() - t0, 1), "s; overflowed", T.overflowed)
    assert model.stats()["overflowed_buckets"] == T.overflowed
    rng = np.random.default_rng(1)
    codes_w = orc.hash.codes(orc.p["W2"][:64])
    for t in rng.integers(0, wl.L, size=40):
        for c in list(rng.integers(0, wl.num_buckets, size=20)) + [int(x) for x in codes_w[:8, t]]:
            assert np.array_equal(model.debug_bucket(int(t), int(c)), T.bucket(int(t), int(c))), (t, c)
    _say("  sampled buckets identical", round(time.time() - t0, 1), "s")
    res = compare_step(model, orc, gen.batch(0))
    _say("  step compared", round(time.time() - t0, 1), "s",
         {k: round(v, 3) for k, v in res.items() if not k.startswith("_")}, res["_loss"], model.stats())
    assert_ok(res)
    model.destroy()

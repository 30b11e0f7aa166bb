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

from helpers import assert_ok, compare_step, load_state, make_pair  # noqa: E402


def _say(*a):
    print(*a, flush=True)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("i", [1, 2, 3, 4, 5, 6, 7, 8])
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
    _say("  with a floor of 1e-7 * max|ref|:", {k: round(v, 3) for k, v in res["_floor1e-7"].items()})
    assert_ok(res)
    model.destroy()


@pytest.mark.timeout(600)
def test_output_layer_larger_than_one_lds_bitmap():
    """1.5 million output neurons: a sample's bitmap of candidates no longer fits the LDS in one piece,
    so the lookup sweeps it in two segments and re-reads the spilled words for the id list.  Two steps
    from identical state, compared with the oracle in full, and a prediction over the retrieved set."""
    wl = synth.small(synth.HASH_DWTA, num_classes=1_500_007, hidden_dim=16, K=6, L=4, bucket_cap=16, batch=21,
                     input_dim=500, nnz_mean=10.0, rebuild_every=0)
    _say("large layer", wl.num_classes)
    gen, model, orc = make_pair(wl)
    model.build_tables()
    T = orc.build_tables()
    assert model.stats()["overflowed_buckets"] == T.overflowed
    for step in range(2):
        load_state(model, orc)                             # (weights agree to 1e-4 after a step, not to the bit)
        res = compare_step(model, orc, gen.batch(step))
        _say("  step", step, {k: round(v, 3) for k, v in res.items() if not k.startswith("_")}, res["_loss"])
        assert_ok(res)
    load_state(model, orc)
    b = gen.batch(2)
    ids, _ = model.predict(model.to_device(b), 5, mode=0)
    want, _ = orc.predict(b, 5, 0)
    assert float((ids.cpu().numpy() == want).mean()) > 0.98
    assert model.status() == 0
    model.destroy()


@pytest.mark.timeout(600)
def test_full_size_prediction_over_all_neurons():
    """cfg2 (670K-class): top-5 over all neurons for the whole batch; sampled samples are checked
    against the oracle's double-precision scores, every sample against the properties that hold at
    any size (distinct valid ids, scores descending)."""
    from helpers import FLOOR, REL
    wl = synth.config(2)
    gen, model, orc = make_pair(wl)
    model.build_tables()
    b = gen.batch(0)
    db = model.to_device(b)
    ids, sc = model.predict(db, 5, mode=1)
    torch.cuda.synchronize()
    t0 = time.time()
    for _ in range(3):
        ids, sc = model.predict(db, 5, mode=1)
    torch.cuda.synchronize()
    _say("  dense prediction over", wl.num_classes, "neurons x", wl.batch, "samples:",
         round((time.time() - t0) / 3 * 1e3, 2), "ms")
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    assert ids.min() >= 0 and ids.max() < wl.num_classes
    assert all(len(set(r.tolist())) == 5 for r in ids)
    assert np.all(np.diff(sc, axis=1) <= 0)
    h = orc.forward_hidden(b).astype(np.float64)
    W2, b2 = orc.p["W2"].astype(np.float64), orc.p["b2"].astype(np.float64)
    for i in np.random.default_rng(3).choice(wl.batch, size=6, replace=False):
        z = W2 @ h[i] + b2
        order = np.lexsort((np.arange(z.size), -z))[:5]
        tol = REL * np.abs(z[order]) + FLOOR * np.abs(z).max()
        assert np.all(np.abs(sc[i] - z[order]) <= tol), (i, sc[i], z[order])
        assert np.all(np.abs(z[ids[i]] - z[order]) <= 2 * tol)
    model.destroy()

"""Prediction over all output neurons (slide_predict mode 1) against the oracle, and the
prediction-quality loop on a task with planted structure: the hashed retrieval must find what the
dense evaluation finds."""
import numpy as np
import pytest

from paper_2201_12667_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("needs a GPU", allow_module_level=True)

from helpers import (FLOOR, REL, make_oracle, make_pair, planted_batch, planted_prototypes,  # noqa: E402
                     planted_workload)


def _say(*a):
    print(*a, flush=True)


def _dense_scores(orc, batch):
    """All N scores per sample in double precision, from the oracle's parameters."""
    h = orc.forward_hidden(batch).astype(np.float64)
    return h @ orc.p["W2"].astype(np.float64).T + orc.p["b2"].astype(np.float64)


def _check_topk(ids, sc, z, topk):
    """ids/sc [B][topk] from the GPU against the full score matrix z [B][N] of the oracle: the
    scores agree to the fp32 bar, every reported id carries the score reported for it, the list is
    the oracle's top-k up to the order of scores that differ by less than the bar, ties to the
    lower id are honoured where the oracle's scores are exactly equal, and the tail is padded."""
    B, N = z.shape
    k = min(topk, N)
    order = np.lexsort((np.broadcast_to(np.arange(N), z.shape), -z), axis=1)[:, :k]
    want = np.take_along_axis(z, order, axis=1)
    tol = REL * np.abs(want) + FLOOR * np.abs(z).max()
    assert np.all(ids[:, k:] == -1) and np.all(np.isneginf(sc[:, k:]))
    got_ids = ids[:, :k]
    assert got_ids.min() >= 0 and got_ids.max() < N
    assert all(len(set(r.tolist())) == k for r in got_ids)
    assert np.all(np.abs(sc[:, :k] - want) <= tol)                       # r-th best score
    assert np.all(np.abs(np.take_along_axis(z, got_ids, axis=1) - want) <= 2 * tol)   # carried by the reported id
    exact = float((got_ids == order).mean())
    return exact


@pytest.mark.parametrize("name,wl,topk", [
    ("dwta-small", synth.small(synth.HASH_DWTA), 5),
    ("dense-hidden-h200", synth.small(synth.HASH_DWTA, input_dim=0, hidden_dim=200, K=3, L=5, batch=70,
                                      num_classes=9973), 64),
    ("h1024-b130", synth.small(synth.HASH_DWTA, hidden_dim=1024, K=4, L=5, batch=130, num_classes=7001,
                               input_dim=2500, bucket_cap=64), 10),
    ("fewer-neurons-than-k", synth.small(synth.HASH_SIMHASH, hidden_dim=32, K=3, L=3, batch=9, num_classes=50,
                                         input_dim=100, nnz_mean=5.0, lab_mean=1.0), 64),
    # 2048 samples: eight sample tiles per neuron tile, two chunks of neurons
    ("b2048-three-chunks", synth.small(synth.HASH_SIMHASH, hidden_dim=32, K=5, L=4, batch=2048, num_classes=20011,
                                       input_dim=0, bucket_cap=8), 7),
    ("h4", synth.small(synth.HASH_SIMHASH, hidden_dim=4, K=2, L=3, batch=3, num_classes=700,
                       input_dim=60, nnz_mean=4.0), 3),
])
def test_predict_over_all_neurons_matches_oracle(name, wl, topk):
    _say("dense predict", name)
    gen, model, orc = make_pair(wl)
    model.build_tables()
    b = gen.batch(0)
    ids, sc = model.predict(model.to_device(b), topk, mode=1)
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    exact = _check_topk(ids, sc, _dense_scores(orc, b), topk)
    _say("   positions identical to the oracle's order:", round(exact, 4))
    assert exact > 0.98
    want_ids, _ = orc.predict(b, topk, 1)
    assert float((ids == want_ids).mean()) > 0.98
    assert model.status() == 0
    model.destroy()


@pytest.mark.parametrize("slope", [0.01, -0.01])
def test_predict_when_every_or_no_later_neuron_beats_the_list(slope):
    """The two extremes of the chunked top-k: biases that grow with the neuron id make every score of
    every later chunk beat the running list (the candidate buffers overflow and the chunk's scores are
    streamed instead); biases that fall with the id make none beat it (the list of the first chunk stands)."""
    _say("dense predict, bias slope", slope)
    wl = synth.small(synth.HASH_DWTA, num_classes=20011, batch=33)
    gen, model, orc = make_pair(wl)
    bias = (slope * np.arange(wl.num_classes)).astype(np.float32)
    orc.p["b2"][:] = bias
    model.p["b2"].copy_(torch.from_numpy(bias))
    model.build_tables()
    b = gen.batch(0)
    for topk in (1, 64):
        ids, sc = model.predict(model.to_device(b), topk, mode=1)
        ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
        exact = _check_topk(ids, sc, _dense_scores(orc, b), topk)
        _say("   topk", topk, "positions identical to the oracle's order:", round(exact, 4))
        assert exact > 0.9
        lo, hi = (wl.num_classes - 200, wl.num_classes) if slope > 0 else (0, 200)
        assert ids.min() >= lo and ids.max() < hi
    assert model.status() == 0
    model.destroy()


def test_prediction_quality_on_a_planted_task():
    """300 training steps on the GPU, then top-1 over the retrieved set (mode 0) and over all neurons
    (mode 1): both find the planted class, and they agree."""
    wl = planted_workload()
    gen, model, orc = make_pair(wl)
    protos = planted_prototypes(wl)
    model.build_tables()
    first = last = None
    for s in range(300):
        b, _ = planted_batch(wl, protos, s)
        loss = model.train_step(model.to_device(b))
        if s == 0:
            first = float(loss.item())
    last = float(loss.item())
    _say("planted task: loss", first, "->", last)
    assert last < 0.1 < first
    hits = {0: 0, 1: 0}
    agree = total = 0
    for s in range(10_000, 10_004):
        b, labels = planted_batch(wl, protos, s)
        db = model.to_device(b)
        lsh = model.predict(db, 1, mode=0)[0].cpu().numpy()[:, 0]
        dense = model.predict(db, 1, mode=1)[0].cpu().numpy()[:, 0]
        hits[0] += int((lsh == labels).sum())
        hits[1] += int((dense == labels).sum())
        agree += int((lsh == dense).sum())
        total += labels.size
    _say("P@1 retrieved set", hits[0] / total, " P@1 all neurons", hits[1] / total, " agreement", agree / total)
    assert hits[1] / total >= 0.97 and hits[0] / total >= 0.9 and agree / total >= 0.9
    # the dense pass on the trained weights against the oracle evaluated on the same weights
    w = {k: v.cpu().numpy() for k, v in model.p.items()}
    ref = make_oracle(wl, w, gen.hash_params())
    b, _ = planted_batch(wl, protos, 20_000)
    ids, sc = model.predict(model.to_device(b), 5, mode=1)
    assert _check_topk(ids.cpu().numpy(), sc.cpu().numpy(), _dense_scores(ref, b), 5) > 0.98
    model.destroy()

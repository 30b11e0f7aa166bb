"""Pins of the oracle's inference (SlideOracle.predict) and of its handling of label entries that
name no neuron: a model small enough to score by hand (tests/golden/predict_example.json), and brute
force with Python sets."""
import json
import os

import numpy as np

from oracle import slide_oracle as so


def _example(golden_dir):
    with open(os.path.join(golden_dir, "predict_example.json")) as f:
        g = json.load(f)
    hp = dict(srp_idx=np.array(g["srp_idx"], np.int32), srp_sign=np.array(g["srp_sign"], np.int8),
              dens_a=1, dens_b=1, prio_a=1, prio_b=1)
    w = dict(W2=np.array(g["W2"], np.float32), b2=np.array(g["b2"], np.float32))
    orc = so.SlideOracle(input_dim=0, hidden_dim=g["H"], num_classes=g["N"], hash_kind=so.SIMHASH, K=g["K"],
                         L=g["L"], bucket_cap=g["bucket_cap"], rebuild_every=0, lr=1e-3, weights=w, hash_params=hp)
    orc.build_tables()
    batch = dict(batch=3, hidden=np.array(g["hidden"], np.float32), y_indptr=np.array(g["y_indptr"], np.int32),
                 y_indices=np.array(g["y_indices"], np.int32))
    return g, orc, batch


def _scores(rows):
    return np.array([[-np.inf if x == "-inf" else float(x) for x in r] for r in rows])


def test_predict_over_retrieved_neurons_hand_example(golden_dir):
    g, orc, batch = _example(golden_dir)
    for c, want in enumerate([[2, 5], [0, 3, 4], [], [1]]):              # the buckets the scores come from
        assert orc.tables.bucket(0, c).tolist() == want
    ids, sc = orc.predict(batch, g["topk_retrieved"], mode=0)
    assert ids.tolist() == g["ids_retrieved"]                            # tie to the lower id, label not added, -1 padding
    assert np.array_equal(sc, _scores(g["scores_retrieved"]))            # integer data: exact, bias included


def test_predict_over_all_neurons_hand_example(golden_dir):
    g, orc, batch = _example(golden_dir)
    ids, sc = orc.predict(batch, g["topk_all"], mode=1)
    assert ids.tolist() == g["ids_all"]
    assert np.array_equal(sc, _scores(g["scores_all"]))
    ids2, sc2 = orc.predict(batch, 2, mode=1)                            # a prefix of the same order
    assert np.array_equal(ids2, ids[:, :2]) and np.array_equal(sc2, sc[:, :2])


def test_label_entries_outside_the_layer_are_left_out_and_counted():
    """A label entry outside [0, N) names no neuron: the step runs as if the entry were not in the batch
    (same sets, same target 1/|valid distinct labels|, same loss), and the entry is counted."""
    rng = np.random.default_rng(11)
    N, H, L, K, B = 300, 16, 5, 4, 6
    S = -(-H // 3)
    hp = dict(srp_idx=np.stack([np.sort(rng.choice(H, S, replace=False)) for _ in range(K * L)]).astype(np.int32),
              srp_sign=(rng.integers(0, 2, (K * L, S)) * 2 - 1).astype(np.int8), dens_a=1, dens_b=1, prio_a=3, prio_b=5)
    w = dict(W2=rng.standard_normal((N, H)).astype(np.float32), b2=rng.standard_normal(N).astype(np.float32))

    def model():
        o = so.SlideOracle(input_dim=0, hidden_dim=H, num_classes=N, hash_kind=so.SIMHASH, K=K, L=L, bucket_cap=8,
                           rebuild_every=0, lr=1e-3, weights=w, hash_params=hp)
        o.build_tables()
        return o

    hidden = np.maximum(rng.standard_normal((B, H)), 0).astype(np.float32)
    good = [[5, 17], [299], [0, 1, 2], [40], [41, 7], [9]]
    bad = [[5, -1, 17], [299, N], [0, 1, 2], [N + 5, 40, -7], [41, 7], [9, 2 ** 31 - 1]]

    def batch(ys):
        yp = np.zeros(B + 1, np.int32)
        yp[1:] = np.cumsum([len(y) for y in ys])
        return dict(batch=B, hidden=hidden, y_indptr=yp, y_indices=np.array(sum(ys, []), np.int32))

    a, b = model().train_step(batch(good)), model().train_step(batch(bad))
    assert a["bad_labels"] == 0 and b["bad_labels"] == 5
    for k in ("as_ptr", "as_ids", "is_label", "z", "delta", "loss_i", "dh"):
        assert np.array_equal(a[k], b[k]), k
    # brute force of the sets themselves
    o = model()
    codes = o.hash.codes(hidden)
    for i in range(B):
        want = set(good[i])
        for t in range(L):
            want |= set(o.tables.bucket(t, int(codes[i, t])).tolist())
        got = b["as_ids"][b["as_ptr"][i]:b["as_ptr"][i + 1]]
        assert got.tolist() == sorted(want)
        lab = b["is_label"][b["as_ptr"][i]:b["as_ptr"][i + 1]]
        assert set(got[lab != 0].tolist()) == set(good[i])

"""The oracle on a task with planted structure: after training, the neurons the hash tables
retrieve contain the right class almost always, and the prediction over the retrieved set agrees
with the prediction over all neurons -- the property the method rests on (paper Section 2.1: the
tables return the neurons with the highest activations; Section 4: accuracy at a fraction of the
computation).  A dropped label union, a wrong gradient sign or stale tables all break it."""
import numpy as np

from helpers import make_oracle, planted_batch, planted_prototypes, planted_workload
from paper_2201_12667_amd import synth


def test_lsh_prediction_finds_the_planted_class():
    wl = planted_workload()
    gen = synth.Generator(wl, 0)
    orc = make_oracle(wl, gen.weights(), gen.hash_params())
    protos = planted_prototypes(wl)
    orc.build_tables()
    losses = []
    for s in range(300):
        b, _ = planted_batch(wl, protos, s)
        losses.append(orc.train_step(b)["loss"])
    assert losses[-1] < 0.1 < losses[0]
    b, labels = planted_batch(wl, protos, 10_000)
    lsh, _ = orc.predict(b, 1, 0)
    dense, _ = orc.predict(b, 1, 1)
    p_lsh, p_dense = float((lsh[:, 0] == labels).mean()), float((dense[:, 0] == labels).mean())
    agree = float((lsh[:, 0] == dense[:, 0]).mean())
    assert p_dense >= 0.97 and p_lsh >= 0.9 and agree >= 0.9, (p_lsh, p_dense, agree)
    # the retrieved sets are a small fraction of the layer
    codes = orc.hash.codes(orc.forward_hidden(b))
    as_ptr, _, _, _ = orc.tables.active_sets(codes, b["y_indptr"], b["y_indices"], include_labels=False)
    assert np.diff(as_ptr).mean() < 0.6 * wl.num_classes


def test_training_under_a_sampling_budget_still_learns():
    """Section 3.7's budget: at most `budget` retrieved neurons per sample (random fill when the
    tables return fewer), labels always present; the planted task is still learnt."""
    wl = planted_workload()
    gen = synth.Generator(wl, 0)
    from oracle import slide_oracle as so
    orc = so.SlideOracle(input_dim=wl.input_dim, hidden_dim=wl.hidden_dim, num_classes=wl.num_classes,
                         hash_kind=wl.hash_kind, K=wl.K, L=wl.L, bucket_cap=wl.bucket_cap,
                         rebuild_every=wl.rebuild_every, lr=wl.lr, dwta_bin=wl.dwta_bin,
                         overflow_policy=wl.overflow_policy, weights=gen.weights(), hash_params=gen.hash_params(),
                         sample_budget=60, sample_fill=True, sample_seed=5)
    protos = planted_prototypes(wl)
    orc.build_tables()
    for s in range(300):
        b, labels = planted_batch(wl, protos, s)
        r = orc.train_step(b)
        sizes = np.diff(r["as_ptr"])
        assert np.all(sizes == 61)                                 # budget (filled) + the one label
        assert r["is_label"].sum() == wl.batch
    assert r["loss"] < 0.2
    b, labels = planted_batch(wl, protos, 10_000)
    dense, _ = orc.predict(b, 1, 1)
    assert float((dense[:, 0] == labels).mean()) >= 0.95

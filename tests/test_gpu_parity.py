"""HIP path against the CPU oracle, through the C ABI, on the same seeded inputs.

Bar: bit-exact for hash codes, bucket contents, active sets and (sparse-input mode) hidden
activations; 1e-4 relative (helpers.close) for logits, errors, gradients-as-Adam-state and updated
weights; 1e-3 on the 10-step loss."""
import numpy as np
import pytest

from paper_2201_12667_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("needs a GPU", allow_module_level=True)

from helpers import assert_ok, close, compare_step, load_state, make_pair  # noqa: E402


def _say(*a):
    print(*a, flush=True)


@pytest.mark.parametrize("kind,H,K,L", [(synth.HASH_DWTA, 128, 6, 40), (synth.HASH_SIMHASH, 128, 9, 50),
                                        (synth.HASH_DWTA, 1024, 8, 20), (synth.HASH_SIMHASH, 32, 4, 8),
                                        (synth.HASH_DWTA, 200, 4, 33), (synth.HASH_SIMHASH, 1024, 9, 7)])
def test_hash_codes_bit_exact(kind, H, K, L):
    _say("hash", kind, H, K, L)
    wl = synth.small(kind, hidden_dim=H, K=K, L=L, input_dim=0, num_classes=300, batch=8)
    gen, model, orc = make_pair(wl)
    rng = np.random.default_rng(5)
    V = rng.standard_normal((203, H)).astype(np.float32)        # several tiles + a ragged tail
    V[:70] = np.maximum(V[:70], 0)                              # ReLU-like rows: empty DWTA bins
    V[3] = 0                                                    # all-zero vector
    V[4, 5:] = 0                                                # almost empty vector
    V[5] *= 1e-30                                               # tiny magnitudes
    V[6, ::2] = np.nan
    got = model.debug_hash(V)
    want = orc.hash.codes(V)
    assert np.array_equal(got, want), np.argwhere(got != want)[:5]
    model.destroy()


@pytest.mark.parametrize("kind,policy,C,N", [(synth.HASH_SIMHASH, 1, 16, 2000), (synth.HASH_SIMHASH, 0, 5, 1500),
                                             (synth.HASH_DWTA, 1, 16, 20011), (synth.HASH_DWTA, 0, 3, 5000),
                                             (synth.HASH_SIMHASH, 1, 128, 30000),
                                             # the largest capacity, buckets of about 3000 members
                                             (synth.HASH_SIMHASH, 1, 1024, 200000), (synth.HASH_SIMHASH, 0, 1024, 100000)])
def test_tables_bit_exact_first_build_and_rebuild(kind, policy, C, N):
    _say("tables", kind, policy, C, N)
    K = 3 if kind == synth.HASH_DWTA else 6
    wl = synth.small(kind, K=K, L=7, bucket_cap=C, num_classes=N, overflow_policy=policy, input_dim=0)
    gen, model, orc = make_pair(wl)
    for rebuild in (False, True):
        model.build_tables()
        T = orc.build_tables(first=not rebuild)
        assert model.stats()["overflowed_buckets"] == T.overflowed
        for t in range(wl.L):
            for c in range(wl.num_buckets):
                assert np.array_equal(model.debug_bucket(t, c), T.bucket(t, c)), (rebuild, t, c)
    model.destroy()


@pytest.mark.parametrize("kind,K,N,C,policy", [(synth.HASH_DWTA, 6, 20011, 16, 1), (synth.HASH_DWTA, 5, 9001, 2, 0),
                                               (synth.HASH_SIMHASH, 16, 5003, 8, 1)])
def test_tables_with_far_more_buckets_than_neurons(kind, K, N, C, policy):
    """Codes of 15 .. 18 bits over a few thousand neurons: a partition of the bucket kernel spans
    2048 .. 8192 buckets, nearly all of them empty.  Every occupied bucket and its neighbours are
    compared, and a sample of the others; the occupied ones must hold all N neurons."""
    _say("sparse tables", kind, K, N, C, policy)
    wl = synth.small(kind, K=K, L=5, bucket_cap=C, num_classes=N, overflow_policy=policy, input_dim=0)
    gen, model, orc = make_pair(wl)
    nb = wl.num_buckets
    rng = np.random.default_rng(7)
    for rebuild in (False, True):
        model.build_tables()
        T = orc.build_tables(first=not rebuild)
        assert model.stats()["overflowed_buckets"] == T.overflowed
        codes = orc.hash.codes(orc.p["W2"])
        for t in range(wl.L):
            occ = np.unique(codes[:, t]).astype(np.int64)
            look = np.unique(np.concatenate([occ, occ - 1, occ + 1, rng.integers(0, nb, 3000), [0, nb - 1]]))
            look = look[(look >= 0) & (look < nb)]
            held = 0
            for c in look:
                got, want = model.debug_bucket(t, int(c)), T.bucket(t, int(c))
                assert np.array_equal(got, want), (rebuild, t, int(c), got, want)
                held += len(got)
            assert held == T.entries(t)
    model.destroy()


@pytest.mark.parametrize("N,policy", [(5000, 1), (12000, 1), (12000, 0)])
def test_degenerate_tables_all_rows_identical(N, policy):
    """Two buckets per table hold everything (4,000 identical rows; the all-zero rest, which at
    N = 12,000 is more than the survivor search stages on chip)."""
    _say("tables degenerate", N, policy)
    wl = synth.small(synth.HASH_DWTA, K=2, L=3, bucket_cap=8, num_classes=N, input_dim=0, overflow_policy=policy)
    gen = synth.Generator(wl, 0)
    w = gen.weights()
    w["W2"][:] = w["W2"][0]                    # one bucket per table holds every neuron
    w["W2"][4000:] = 0                         # and the all-zero rows go to code 0
    from helpers import make_oracle
    from paper_2201_12667_amd import slide
    hp = gen.hash_params()
    model, orc = slide.Slide(slide.config_from_workload(wl), w, hp), make_oracle(wl, w, hp)
    model.build_tables()
    T = orc.build_tables()
    for t in range(wl.L):
        for c in range(wl.num_buckets):
            assert np.array_equal(model.debug_bucket(t, c), T.bucket(t, c)), (t, c)
    model.destroy()


@pytest.mark.parametrize("name,wl", [
    ("dwta-small", synth.small(synth.HASH_DWTA)),
    ("simhash-small", synth.small(synth.HASH_SIMHASH)),
    ("dense-hidden", synth.small(synth.HASH_DWTA, input_dim=0, batch=70, num_classes=9973)),
    ("cfg0", synth.config(0)),
    ("h1024-b130", synth.small(synth.HASH_DWTA, hidden_dim=1024, K=4, L=11, batch=130, num_classes=7001,
                               input_dim=2500, bucket_cap=64)),
    ("h32-uniform", synth.small(synth.HASH_SIMHASH, hidden_dim=32, K=5, L=9, batch=5, num_classes=900,
                                input_dim=400, nnz_mean=6.0, feat_zipf_s=None, lab_zipf_s=None)),
    ("h200", synth.small(synth.HASH_DWTA, hidden_dim=200, K=3, L=13, batch=33, num_classes=4099,
                         input_dim=1200)),
    ("single-sample", synth.small(synth.HASH_DWTA, batch=1)),
    # larger batches: tiles of 512, 256 and 128 rows in the row-list construction
    ("b300-tile512", synth.small(synth.HASH_DWTA, hidden_dim=64, K=3, L=9, batch=300, num_classes=6007,
                                 input_dim=2900, nnz_mean=8.0, bucket_cap=8)),
    ("b600-tile256", synth.small(synth.HASH_SIMHASH, hidden_dim=32, K=6, L=7, batch=600, num_classes=5003,
                                 input_dim=1900, nnz_mean=6.0, bucket_cap=8)),
    ("b1100-tile128", synth.small(synth.HASH_DWTA, hidden_dim=32, K=3, L=5, batch=1100, num_classes=4001,
                                  input_dim=700, nnz_mean=5.0, bucket_cap=8)),
    ("b2048-tile128", synth.small(synth.HASH_SIMHASH, hidden_dim=32, K=5, L=4, batch=2048, num_classes=3001,
                                  input_dim=0, bucket_cap=8)),
    # very wide inputs: the feature tiles hold a handful of the batch's features each (a wave per tile),
    # the tiles of the popular features far more (left to the whole workgroup); uniform features: no such tile
    ("wide-input-zipf", synth.small(synth.HASH_DWTA, hidden_dim=64, K=3, L=9, batch=256, num_classes=6007,
                                    input_dim=300001, nnz_mean=8.0, bucket_cap=8)),
    ("wide-input-uniform", synth.small(synth.HASH_SIMHASH, hidden_dim=32, K=6, L=7, batch=70, num_classes=5003,
                                       input_dim=150001, nnz_mean=3.0, bucket_cap=8, feat_zipf_s=None)),
    ("wide-input-b600", synth.small(synth.HASH_DWTA, hidden_dim=32, K=3, L=5, batch=600, num_classes=4001,
                                    input_dim=400001, nnz_mean=4.0, bucket_cap=8)),
    # a layer wide enough for the lookup workgroup to stage the sample's W1 rows in LDS, and samples with
    # more features than the staging holds at once (48 rows here): three rounds of staging per sample
    ("staged-hidden-three-rounds", synth.small(synth.HASH_DWTA, num_classes=200003, input_dim=5000, nnz_mean=120.0,
                                               batch=8, L=9)),
    # the largest bucket capacity: every bucket holds more than 1024 neurons, 5120 candidates per sample
    ("cap1024", synth.small(synth.HASH_SIMHASH, K=4, L=5, bucket_cap=1024, num_classes=60000, batch=9)),
])
def test_single_step_from_identical_state(name, wl):
    _say("step", name)
    gen, model, orc = make_pair(wl)
    model.build_tables()
    orc.build_tables()
    res = compare_step(model, orc, gen.batch(0))
    _say({k: round(v, 3) for k, v in res.items() if not k.startswith("_")}, res["_loss"])
    assert_ok(res)
    # rows that were not touched are bit-identical to the initial weights
    w0 = gen.weights()["W2"]
    untouched = np.setdiff1d(np.arange(wl.num_classes), res["_ref"]["uniq"])
    assert np.array_equal(model.p["W2"].cpu().numpy()[untouched], w0[untouched])
    assert not model.m["W2"].cpu().numpy()[untouched].any()
    model.destroy()


@pytest.mark.parametrize("kind", [synth.HASH_DWTA, synth.HASH_SIMHASH])
def test_every_step_of_a_run_from_the_oracles_state(kind):
    """Steps 1..6 (rebuild after every 3rd): before each step the HIP model is given the oracle's
    state, so each step is compared on its own, including the rebuilt tables."""
    _say("run", kind)
    wl = synth.small(kind)
    gen, model, orc = make_pair(wl)
    model.build_tables()
    orc.build_tables()
    for s in range(wl.steps):
        load_state(model, orc)
        res = compare_step(model, orc, gen.batch(s))
        _say(s, {k: round(v, 3) for k, v in res.items() if not k.startswith("_")})
        assert_ok(res)
    assert model.stats()["rebuilds"] == orc.r == 2
    model.destroy()


def test_rebuild_inside_step_matches_oracle_tables():
    _say("rebuild-in-step")
    wl = synth.small(synth.HASH_SIMHASH, rebuild_every=1, bucket_cap=8)
    gen, model, orc = make_pair(wl)
    model.build_tables()
    orc.build_tables()
    res = compare_step(model, orc, gen.batch(0))
    assert_ok(res)
    assert res["_ref"]["rebuilt"] and model.stats()["rebuilds"] == 1
    same = total = 0
    for t in range(wl.L):
        for c in range(wl.num_buckets):
            total += 1
            same += np.array_equal(model.debug_bucket(t, c), orc.tables.bucket(t, c))
    _say("identical buckets after in-step rebuild:", same, "/", total)
    assert same >= 0.98 * total        # weights agree to 1e-4, so a few sign bits may flip


def test_ten_step_loss_tiny_config():
    _say("ten steps cfg0")
    wl = synth.config(0)
    gen, model, orc = make_pair(wl)
    model.build_tables()
    orc.build_tables()
    first_diff = None
    for s in range(10):
        b = gen.batch(s)
        loss = float(model.train_step(model.to_device(b)).item())
        ref = orc.train_step(b)
        as_ptr, ids, _, _, _ = model.debug_active()
        if first_diff is None and not (np.array_equal(as_ptr, ref["as_ptr"]) and np.array_equal(ids, ref["as_ids"])):
            first_diff = s
        _say(s, loss, ref["loss"])
        assert abs(loss - ref["loss"]) < 1e-3
    _say("active sets first differ at step:", first_diff)
    assert model.stats()["steps"] == 10 and model.stats()["rebuilds"] == 2
    model.destroy()


def test_edge_cases_labels_and_empty_samples():
    _say("edge cases")
    wl = synth.small(synth.HASH_DWTA, batch=6, num_classes=3000, input_dim=500)
    gen, model, orc = make_pair(wl)
    model.build_tables()
    orc.build_tables()
    b = gen.batch(0)
    # sample 0: no features; sample 1: no labels; sample 2: a repeated label; sample 3: unsorted labels
    xp, xi, xv = b["x_indptr"], b["x_indices"], b["x_values"]
    n0 = xp[1]
    xi, xv = xi[n0:], xv[n0:]
    xp = np.concatenate([[0], xp[1:] - n0]).astype(np.int32)
    ys = [b["y_indices"][b["y_indptr"][i]:b["y_indptr"][i + 1]].tolist() for i in range(6)]
    ys[1] = []
    ys[2] = ys[2] + [ys[2][0]]
    ys[3] = [2999, 0, 17]
    yp = np.zeros(7, np.int32)
    yp[1:] = np.cumsum([len(y) for y in ys])
    b2 = dict(batch=6, x_indptr=xp, x_indices=xi, x_values=xv, y_indptr=yp,
              y_indices=np.array(sum(ys, []), np.int32))
    res = compare_step(model, orc, b2)
    assert_ok(res)
    assert not res["_ref"]["dh"][1].any()
    model.destroy()


def test_hash_densification_probe_limit(golden_dir):
    """The hand-worked case in which one empty bin finds its donor at the 100th probe and another would
    find it only at the 101st: the library's two hash kernels (row tiles, and the per-sample one inside the
    lookup) must stop where the definition stops."""
    from test_oracle_hash import dwta_probe_limit_case
    from paper_2201_12667_amd import slide
    g, perm, v, want = dwta_probe_limit_case(golden_dir)
    wl = synth.small(synth.HASH_DWTA, hidden_dim=g["H"], K=g["K"], L=g["L"], dwta_bin=g["m"], input_dim=0,
                     num_classes=64, batch=3, bucket_cap=4, rebuild_every=0)
    gen = synth.Generator(wl, 0)
    hp = dict(gen.hash_params(), dwta_perm=perm, dens_a=g["dens_a"], dens_b=g["dens_b"])
    w = gen.weights()
    from helpers import make_oracle
    model, orc = slide.Slide(slide.config_from_workload(wl), w, hp), make_oracle(wl, w, hp)
    V = np.concatenate([v, np.zeros((1, g["H"]), np.float32), v * 3])
    got = model.debug_hash(V)
    assert np.array_equal(got[0], want) and np.array_equal(got[2], want) and not got[1].any()
    # the same vectors as a batch of hidden activations: the lookup's own hashing
    model.build_tables()
    orc.build_tables()
    b = gen.batch(0)
    b["hidden"] = V
    res = compare_step(model, orc, b)
    assert np.array_equal(res["_ref"]["codes"][0], want)
    assert_ok(res)
    model.destroy()


def test_step_with_label_entries_outside_the_layer_matches_oracle():
    """Label entries outside [0, N) are left out (as if absent) and flagged: the whole step is compared."""
    _say("bad labels, full compare")
    wl = synth.small(synth.HASH_DWTA, batch=9, num_classes=3000, input_dim=500)
    gen, model, orc = make_pair(wl)
    model.build_tables()
    orc.build_tables()
    b = gen.batch(0)
    yp, yi = b["y_indptr"], b["y_indices"]
    ys = [yi[yp[i]:yp[i + 1]].tolist() for i in range(wl.batch)]
    ys[0] = [-1] + ys[0]
    ys[2] = ys[2] + [3000]
    ys[4] = [2 ** 31 - 1]                          # a sample whose only label is invalid: no labels at all
    ys[5] = ys[5][:1] + [-(2 ** 31)] + ys[5][1:]
    yp2 = np.zeros(wl.batch + 1, np.int32)
    yp2[1:] = np.cumsum([len(y) for y in ys])
    b2 = dict(b, y_indptr=yp2, y_indices=np.array(sum(ys, []), np.int64).astype(np.int32))
    res = compare_step(model, orc, b2)             # (asserts the flag word: exactly "bad label")
    assert res["_ref"]["bad_labels"] == 4
    assert not res["_ref"]["dh"][4].any()
    assert_ok(res)
    load_state(model, orc)                         # (weights agree to 1e-4 after a step, not to the bit)
    res = compare_step(model, orc, gen.batch(1))   # and the flag does not stick
    assert_ok(res)
    model.destroy()


@pytest.mark.parametrize("num_classes,input_dim", [(3000, 500), (200003, 500), (3000, 300001)],
                         ids=["wave-per-columns", "rows-staged-in-lds", "wave-per-feature-tile"])
def test_bad_batch_data_is_flagged_not_fatal(num_classes, input_dim):
    """Both forms of the lookup's hidden layer (the wide output layer lets the workgroup stage the W1 rows) and
    both forms of the feature tiles (the wide input layer has a wave take a tile)."""
    _say("bad data", num_classes, input_dim)
    from paper_2201_12667_amd import slide
    wl = synth.small(synth.HASH_DWTA, batch=4, num_classes=num_classes, input_dim=input_dim, L=9)
    gen, model, orc = make_pair(wl)
    model.build_tables()
    orc.build_tables()
    b = gen.batch(0)
    b["x_indices"] = b["x_indices"].copy()
    b["y_indices"] = b["y_indices"].copy()
    b["x_indices"][0] = input_dim                # out of range
    b["y_indices"][0] = -3                       # out of range
    b["x_indices"][b["x_indptr"][1]:b["x_indptr"][1] + 2] = b["x_indices"][b["x_indptr"][1]:b["x_indptr"][1] + 2][::-1]
    model.train_step(model.to_device(b))
    flags = model.status()
    assert flags == slide.FLAG_BAD_FEATURE | slide.FLAG_BAD_LABEL | slide.FLAG_UNSORTED
    assert model.status() == 0                   # cleared after being reported
    # the flagged step leaves nothing behind that a later step would trip over (feature segments, counters):
    # from the oracle's state again (after its own, clean, first step), a clean batch gives a clean, fully
    # matching step
    orc.train_step(gen.batch(0))
    load_state(model, orc)
    assert_ok(compare_step(model, orc, gen.batch(1)))
    # host-detected errors
    with pytest.raises(slide.SlideError) as e:
        db = model.to_device(gen.batch(1))
        db["batch"] = wl.batch + 1
        model.train_step(db)
    assert e.value.code == slide.SLIDE_EINVAL
    model.destroy()
    gen2, fresh, _ = make_pair(wl)
    with pytest.raises(slide.SlideError) as e:
        fresh.train_step(fresh.to_device(gen2.batch(0)))
    assert e.value.code == slide.SLIDE_ESTATE
    fresh.destroy()


def test_batches_beyond_the_configured_capacities_are_refused():
    """SLIDE_ENOMEM on the host, before any launch: more stored features or label entries in a batch than
    the configuration reserved room for, and a read-back buffer smaller than the active sets."""
    _say("capacities")
    from paper_2201_12667_amd import slide
    import ctypes as C
    wl = synth.small(synth.HASH_DWTA, batch=8, num_classes=3000, input_dim=500)
    gen = synth.Generator(wl, 0)
    b = gen.batch(0)
    nnz, nlab = int(b["x_indptr"][-1]), int(b["y_indptr"][-1])
    for over in ({"max_nnz_per_batch": nnz - 1}, {"max_labels_per_batch": nlab - 1}):
        _, model, _ = make_pair(wl, **over)
        model.build_tables()
        with pytest.raises(slide.SlideError) as e:
            model.train_step(model.to_device(b))
        assert e.value.code == slide.SLIDE_ENOMEM
        assert model.stats()["steps"] == 0                 # nothing ran
        model.destroy()
    _, model, _ = make_pair(wl, max_nnz_per_batch=nnz, max_labels_per_batch=nlab)   # exactly enough: accepted
    model.build_tables()
    model.train_step(model.to_device(b))
    assert model.status() == 0
    as_ptr = np.zeros(wl.batch + 1, dtype=np.int64)
    ids = np.zeros(4, dtype=np.int32)
    rc = model.L.slide_debug_get_active(model.ctx, as_ptr.ctypes.data, ids.ctypes.data, None, None, None, 4)
    assert rc == slide.SLIDE_ENOMEM and as_ptr[-1] > 4     # the sizes are reported, the ids are not copied
    model.destroy()


@pytest.mark.parametrize("kind", [synth.HASH_DWTA, synth.HASH_SIMHASH])
def test_predict_mode0_matches_oracle(kind):
    _say("predict", kind)
    wl = synth.small(kind)
    gen, model, orc = make_pair(wl)
    model.build_tables()
    orc.build_tables()
    b = gen.batch(0)
    ids, sc = model.predict(model.to_device(b), 5)
    want_ids, want_sc = orc.predict(b, 5)
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    as_ptr, got_set, _, _, _ = model.debug_active()
    assert np.array_equal(ids, want_ids)
    fin = np.isfinite(want_sc)
    assert close(sc[fin], want_sc[fin]) and np.array_equal(np.isfinite(sc), fin)
    # a training step afterwards still works (the feature segments were left clean)
    res = compare_step(model, orc, gen.batch(1))
    assert_ok(res)
    model.destroy()


@pytest.mark.parametrize("kind", [synth.HASH_DWTA, synth.HASH_SIMHASH])
def test_redrawn_hash_functions_then_rebuild(kind):
    """New hash functions at a rebuild (Algorithm 1): both sides get the same redraw; the tables
    built from them are bit-identical, the rebuild is counted, and the next step matches."""
    _say("redraw", kind)
    from paper_2201_12667_amd import slide
    wl = synth.small(kind, rebuild_every=0, bucket_cap=8)
    gen, model, orc = make_pair(wl)
    model.build_tables()
    orc.build_tables()
    assert_ok(compare_step(model, orc, gen.batch(0)))
    hp1 = gen.hash_params(draw=1)
    model.set_hash_params(hp1)
    with pytest.raises(slide.SlideError):                 # stale tables: a step must not run
        model.train_step(model.to_device(gen.batch(1)))
    orc.set_hash_params(hp1)
    load_state(model, orc)
    model.build_tables()
    T = orc.build_tables(first=False)
    assert model.stats()["rebuilds"] == orc.r == 1
    for t in range(wl.L):
        for c in range(wl.num_buckets):
            assert np.array_equal(model.debug_bucket(t, c), T.bucket(t, c)), (t, c)
    V = np.random.default_rng(2).standard_normal((50, wl.hidden_dim)).astype(np.float32)
    assert np.array_equal(model.debug_hash(V), orc.hash.codes(V))
    assert_ok(compare_step(model, orc, gen.batch(1)))
    model.destroy()


@pytest.mark.parametrize("kind,hidden,N", [(synth.HASH_DWTA, 128, 20011), (synth.HASH_SIMHASH, 128, 20011),
                                           (synth.HASH_DWTA, 1024, 20011), (synth.HASH_DWTA, 128, 1500)])
def test_incremental_rebuild_equals_full_rebuild(kind, hidden, N):
    """Scheduled rebuilds that hash only the rows updated since the last build (Section 3.1: the
    tables are updated locally).  A row that no step touched keeps its weights, hence its codes, so
    the tables must be those of a full rebuild: checked bucket by bucket against a second model
    that rebuilds in full, with the loss checked against the oracle (which always rebuilds in full),
    and the number of rows hashed checked against the union of the active sets since the last build
    (all N once that union exceeds three quarters of the rows: the small layer of the last case)."""
    import dataclasses
    _say("incremental rebuild", kind, hidden, N)
    over = dict(hidden_dim=hidden, K=3, L=6) if hidden != 128 else {}
    wl_full = synth.small(kind, rebuild_every=2, bucket_cap=8, num_classes=N, **over)

    def hashed(touched):
        return len(touched) if 4 * len(touched) <= 3 * N else N

    wl_inc = dataclasses.replace(wl_full, incremental_rebuild=True)
    gen, full, orc = make_pair(wl_full)
    _, inc, _ = make_pair(wl_inc)
    full.build_tables()
    inc.build_tables()
    orc.build_tables()
    assert inc.stats()["rehashed_rows"] == N and full.stats()["rehashed_rows"] == N
    hashed_all = 0
    touched = set()
    for s in range(6):
        b = gen.batch(s)
        loss_full = float(full.train_step(full.to_device(b)).item())
        loss_inc = float(inc.train_step(inc.to_device(b)).item())
        ref = orc.train_step(b)
        assert loss_full == loss_inc
        assert abs(loss_inc - ref["loss"]) < 1e-3
        _, ids, _, _, _ = inc.debug_active()
        touched |= set(ids.tolist())
        if (s + 1) % 2 == 0:
            assert ref["rebuilt"]
            assert inc.stats()["rehashed_rows"] == hashed(touched)
            hashed_all += hashed(touched) == N
            assert full.stats()["rehashed_rows"] == N
            touched.clear()
            for t in range(wl_full.L):
                for c in range(wl_full.num_buckets):
                    assert np.array_equal(inc.debug_bucket(t, c), full.debug_bucket(t, c)), (s, t, c)
    assert inc.stats()["rebuilds"] == full.stats()["rebuilds"] == orc.r == 3
    assert hashed_all == (3 if N == 1500 else 0)
    for n in inc.p:
        assert torch.equal(inc.p[n], full.p[n]), n
    # an explicit build trusts nothing: every row is hashed again, and the marks start afresh
    inc.build_tables()
    assert inc.stats()["rehashed_rows"] == N
    inc.train_step(inc.to_device(gen.batch(6)))
    _, ids, _, _, _ = inc.debug_active()
    inc.train_step(inc.to_device(gen.batch(7)))
    _, ids2, _, _, _ = inc.debug_active()
    assert inc.stats()["rehashed_rows"] == hashed(set(ids.tolist()) | set(ids2.tolist()))
    full.destroy()
    inc.destroy()


@pytest.mark.parametrize("name,wl", [
    ("over-budget", synth.small(synth.HASH_DWTA, sample_budget=20, sample_seed=9)),
    ("over-budget-simhash", synth.small(synth.HASH_SIMHASH, sample_budget=7, sample_seed=3, batch=130)),
    ("fill", synth.small(synth.HASH_DWTA, sample_budget=900, sample_fill=True, sample_seed=5)),
    ("no-fill-under-budget", synth.small(synth.HASH_DWTA, sample_budget=900, sample_fill=False)),
    ("fill-small-layer", synth.small(synth.HASH_SIMHASH, num_classes=600, sample_budget=550, sample_fill=True,
                                     K=4, L=5, batch=20)),
    ("budget-of-one", synth.small(synth.HASH_DWTA, sample_budget=1, sample_fill=True, input_dim=0, batch=70,
                                  num_classes=9973)),
])
def test_sampling_budget_steps_match_oracle(name, wl):
    """Section 3.7's budget: the kept / filled neurons are decided by a counter-based generator that
    both sides implement, so the active sets stay bit-exact; three steps so that the step number
    enters the generator, each from the oracle's state."""
    _say("budget", name)
    gen, model, orc = make_pair(wl)
    model.build_tables()
    orc.build_tables()
    sizes = []
    for s in range(3):
        load_state(model, orc)
        res = compare_step(model, orc, gen.batch(s))
        assert_ok(res)
        ref = res["_ref"]
        non_label = np.diff(ref["as_ptr"]) - np.add.reduceat(ref["is_label"], ref["as_ptr"][:-1])
        assert non_label.max() <= wl.sample_budget
        sizes.append(int(non_label.mean()))
    _say("   mean non-label active neurons per sample:", sizes)
    # prediction ignores the budget
    b = gen.batch(7)
    ids, _ = model.predict(model.to_device(b), 5)
    assert np.array_equal(ids.cpu().numpy(), orc.predict(b, 5)[0])
    model.destroy()


@pytest.mark.parametrize("name,wl", [
    ("dwta-small", synth.small(synth.HASH_DWTA, row_major_mode=2)),
    ("simhash-saturated", synth.small(synth.HASH_SIMHASH, K=3, L=9, bucket_cap=64, row_major_mode=2)),
    ("dense-hidden", synth.small(synth.HASH_DWTA, input_dim=0, batch=70, num_classes=9973, row_major_mode=2)),
    ("cfg0", __import__("dataclasses").replace(synth.config(0), row_major_mode=2)),
    ("h32-b300", synth.small(synth.HASH_SIMHASH, hidden_dim=32, K=4, L=7, batch=300, num_classes=5003, input_dim=1900,
                             nnz_mean=6.0, bucket_cap=32, row_major_mode=2)),
    ("h200-b130", synth.small(synth.HASH_DWTA, hidden_dim=200, K=2, L=13, batch=130, num_classes=4099, input_dim=1200,
                              bucket_cap=32, row_major_mode=2)),
    ("h1024-b37", synth.small(synth.HASH_DWTA, hidden_dim=1024, K=2, L=6, num_classes=3001, input_dim=900,
                              bucket_cap=64, row_major_mode=2)),
    # batches above 512 samples: their vectors do not fit the LDS by useful slices, the plain update runs
    ("h64-b700", synth.small(synth.HASH_SIMHASH, hidden_dim=64, K=3, L=5, batch=700, num_classes=4001,
                                        input_dim=700, nnz_mean=5.0, bucket_cap=32, row_major_mode=2)),
    ("h200-b1024", synth.small(synth.HASH_SIMHASH, hidden_dim=200, K=4, L=6, batch=1024, num_classes=6007,
                                          input_dim=0, bucket_cap=64, row_major_mode=2)),
    ("h136-b513", synth.small(synth.HASH_DWTA, hidden_dim=136, K=2, L=7, batch=513, num_classes=3001,
                                         input_dim=300, nnz_mean=4.0, bucket_cap=16, row_major_mode=2)),
    ("h64-b1100", synth.small(synth.HASH_SIMHASH, hidden_dim=64, K=3, L=5, batch=1100, num_classes=4001, input_dim=700,
                              nnz_mean=5.0, bucket_cap=32, row_major_mode=2)),
    ("h20-b2048-falls-back", synth.small(synth.HASH_SIMHASH, hidden_dim=20, K=3, L=4, batch=2048, num_classes=3001,
                                         input_dim=0, bucket_cap=8, row_major_mode=2)),
    ("single-sample", synth.small(synth.HASH_DWTA, batch=1, row_major_mode=2)),
])
def test_row_major_kernels_match_oracle(name, wl):
    """The kernels for batches whose samples share most rows (rows streamed once, the batch's vectors
    in LDS), forced on: three steps, each from the oracle's state, the third after a rebuild."""
    _say("row-major", name)
    gen, model, orc = make_pair(wl)
    model.build_tables()
    orc.build_tables()
    for s in range(3):
        load_state(model, orc)
        res = compare_step(model, orc, gen.batch(s))
        _say(s, {k: round(v, 3) for k, v in res.items() if not k.startswith("_")})
        assert_ok(res)
    model.destroy()


def _random_workloads():
    rng = np.random.default_rng(2024)
    out = []
    Hs = [4, 8, 20, 36, 64, 100, 132, 260, 516, 1028, 2048]
    Bs = [1, 2, 3, 31, 63, 64, 65, 127, 129, 255, 257, 333]
    for k in range(14):
        kind = synth.HASH_DWTA if k % 2 == 0 else synth.HASH_SIMHASH
        H = int(Hs[k % len(Hs)])
        if kind == synth.HASH_DWTA and H % 8:
            H += 8 - H % 8                                  # DWTA bins of 8 coordinates
        B = int(Bs[(3 * k + 1) % len(Bs)])
        N = int(rng.integers(33, 5000))
        D = 0 if k % 5 == 4 else int(rng.integers(5, 3000))
        K = int(rng.integers(1, 4)) if kind == synth.HASH_DWTA else int(rng.integers(1, 9))
        L = int(rng.integers(1, 12))
        Ccap = int(rng.choice([1, 2, 5, 16, 64]))
        nnz = float(min(max(D // 3, 1), rng.integers(1, 40))) if D else 1.0
        wl = synth.small(kind, hidden_dim=H, batch=B, num_classes=N, input_dim=D, K=K, L=L, bucket_cap=Ccap,
                         nnz_mean=nnz, lab_mean=float(rng.integers(1, 6)), rebuild_every=2,
                         overflow_policy=int(k % 3 == 0))
        out.append(("r%02d-H%d-B%d-N%d-D%d-K%dL%dC%d" % (k, H, B, N, D, K, L, Ccap), wl))
    return out


@pytest.mark.parametrize("name,wl", _random_workloads())
def test_randomly_shaped_workloads_two_steps(name, wl):
    """Odd shapes: vectors that do not fill the lane groups, single-sample batches, layers smaller
    than a tile, one table, buckets of one -- two steps each (the second after a rebuild)."""
    _say("random shape", name)
    gen, model, orc = make_pair(wl)
    model.build_tables()
    orc.build_tables()
    for s in range(2):
        load_state(model, orc)
        res = compare_step(model, orc, gen.batch(s))
        assert_ok(res)
    model.destroy()


def test_copy_yardstick_copies_every_byte():
    """The measurement aid behind the bandwidth figures: whole chunks, a ragged tail, less than a chunk."""
    from paper_2201_12667_amd import slide
    st = torch.cuda.current_stream().cuda_stream
    for words in (1, 255, 1023, 1024, 1025, 3 * 1024 + 5, 70000 * 1024 + 777):
        _say("copy", words, "x 16 bytes")
        src = torch.randint(0, 256, (words * 16,), dtype=torch.uint8, device="cuda:0")
        dst = torch.zeros(words * 16 + 16, dtype=torch.uint8, device="cuda:0")
        slide.debug_copy(dst[:words * 16], src, st)
        torch.cuda.synchronize()
        assert torch.equal(dst[:words * 16], src)
        assert int(dst[words * 16:].sum()) == 0

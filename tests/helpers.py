"""Shared helpers of the GPU parity tests: build the HIP model and the oracle from the same seeded
arrays, and the floating-point comparison rule."""
import numpy as np

from oracle import slide_oracle as so
from paper_2201_12667_amd import slide, synth
from paper_2201_12667_amd.slide import FLAG_BAD_LABEL

# fp32 tolerance: |gpu - ref| <= REL*|ref| + FLOOR*max|ref| (REL is the stated 1e-4 relative bar; the
# floor, about two fp32 ulps of the tensor's largest element, is what keeps the bar meaningful for
# elements that cancel to nearly zero).
REL, FLOOR = 1e-4, 1e-7


def close(a, ref, rel=REL, floor=FLOOR):
    a, ref = np.asarray(a, np.float64), np.asarray(ref, np.float64)
    if a.shape != ref.shape:
        return False
    if ref.size == 0:
        return True
    return bool(np.all(np.abs(a - ref) <= rel * np.abs(ref) + floor * np.abs(ref).max() + 1e-30))


def worst(a, ref, floor=None):
    floor = FLOOR if floor is None else floor
    a, ref = np.asarray(a, np.float64), np.asarray(ref, np.float64)
    if ref.size == 0:
        return 0.0
    return float(np.max(np.abs(a - ref) / (REL * np.abs(ref) + floor * np.abs(ref).max() + 1e-30)))


def touched_rows(orc, ref, name):
    """Rows of parameter `name` that the step updates (membership, not a non-zero gradient)."""
    if name in ("W2", "b2"):
        return np.asarray(ref["uniq"], np.int64)
    if name == "W1":
        return np.asarray(ref["uniq1"], np.int64)
    return np.arange(orc.p[name].shape[0], dtype=np.int64)


def adam_self_consistency(model, orc, ref, before, t):
    """The update rule checked on the library's own numbers: on every touched row the new weight
    must equal w_before - lr * (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps) evaluated in double precision from
    the library's own post-step m and v (which are themselves compared with the oracle's at the plain
    bar), at the plain bar; every other row must be bit-identical to what it was.  This isolates the
    one place where the comparison of the weights themselves needs a derived bound (worst_weight)."""
    out = {}
    bc1, bc2 = 1 - orc.beta1 ** t, 1 - orc.beta2 ** t
    for n in model.p:
        rows = touched_rows(orc, ref, n)
        w = model.p[n].cpu().numpy()
        keep = np.ones(w.shape[0], bool)
        keep[rows] = False
        assert np.array_equal(w[keep], before[n][keep]), "untouched rows of %s changed" % n
        m = model.m[n].cpu().numpy()[rows].astype(np.float64)
        v = model.v[n].cpu().numpy()[rows].astype(np.float64)
        want = before[n][rows].astype(np.float64) - orc.lr * (m / bc1) / (np.sqrt(v / bc2) + orc.eps)
        out["adam:" + n] = worst(w[rows], want)
    return out


def worst_weight(w, orc, name):
    """Tolerance ratio of an updated parameter tensor.  On top of the direct bar
    (REL*|w| + FLOOR*max|w|) it grants what the tolerances already granted to Adam's momentum and
    velocity amount to once propagated through the update u = lr * mh / (sqrt(vh) + eps),
    mh = m/(1-b1^t), vh = v/(1-b2^t):  |du| <= lr/(sqrt(vh)+eps) * |dmh| + lr*|mh| / (2 sqrt(vh)
    (sqrt(vh)+eps)^2) * |dvh|.  Adam normalises the gradient, so an element whose gradient is tiny
    (a sum that cancels to ~eps) amplifies its absolute rounding error by up to lr/eps; every
    quantity below comes from the oracle."""
    ref = orc.p[name].astype(np.float64)
    m, v = orc.m[name].astype(np.float64), orc.v[name].astype(np.float64)
    bc1, bc2 = 1 - orc.beta1 ** orc.t, 1 - orc.beta2 ** orc.t
    tol_m = (REL * np.abs(m) + FLOOR * np.abs(m).max()) / bc1
    tol_v = (REL * np.abs(v) + FLOOR * np.abs(v).max()) / bc2
    sv = np.sqrt(v / bc2)
    with np.errstate(divide="ignore", invalid="ignore"):
        dv = np.where(sv > 0, np.abs(m / bc1) / (2 * sv * (sv + orc.eps) ** 2), 0.0)
    tol = REL * np.abs(ref) + FLOOR * np.abs(ref).max() + orc.lr * (tol_m / (sv + orc.eps) + dv * tol_v) + 1e-30
    return float(np.max(np.abs(np.asarray(w, np.float64) - ref) / tol))


def make_oracle(wl, weights, hp):
    return so.SlideOracle(input_dim=wl.input_dim, hidden_dim=wl.hidden_dim, num_classes=wl.num_classes,
                          hash_kind=wl.hash_kind, K=wl.K, L=wl.L, bucket_cap=wl.bucket_cap,
                          rebuild_every=wl.rebuild_every, lr=wl.lr, beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps,
                          dwta_bin=wl.dwta_bin, overflow_policy=wl.overflow_policy, weights=weights,
                          hash_params=hp, sample_budget=wl.sample_budget, sample_fill=wl.sample_fill,
                          sample_seed=wl.sample_seed)


def make_pair(wl, seed=0, **cfg_over):
    gen = synth.Generator(wl, seed)
    weights, hp = gen.weights(), gen.hash_params()
    cfg = slide.config_from_workload(wl, **cfg_over)
    model = slide.Slide(cfg, weights, hp)
    return gen, model, make_oracle(wl, weights, hp)


def load_state(model, orc):
    """Copies the oracle's parameters, Adam state and counters' worth of state into the HIP model."""
    import torch
    for n in model.p:
        model.p[n].copy_(torch.from_numpy(orc.p[n]))
        model.m[n].copy_(torch.from_numpy(orc.m[n]))
        model.v[n].copy_(torch.from_numpy(orc.v[n]))
    torch.cuda.synchronize()


def compare_step(model, orc, batch, check_state=True):
    """Runs one step on both from their current states and compares everything.  Returns a dict of
    worst tolerance ratios (<= 1 passes); raises AssertionError on any integer mismatch."""
    db = model.to_device(batch)
    before = {n: model.p[n].cpu().numpy() for n in model.p} if check_state else None
    loss = float(model.train_step(db).item())
    flags = model.status()
    ref = orc.train_step(batch)
    assert flags == (FLAG_BAD_LABEL if ref["bad_labels"] else 0), flags
    h, dh = model.debug_hidden()
    as_ptr, ids, lab, z, d = model.debug_active()
    if not orc.dense_hidden:
        bad = np.argwhere(h != ref["h"])
        assert bad.size == 0, ("hidden activations are not bit-identical", len(bad), bad[:6].tolist(),
                               [(float(h[i, j]), float(ref["h"][i, j])) for i, j in bad[:6]])
    assert np.array_equal(as_ptr, ref["as_ptr"]), "active-set sizes differ"
    assert np.array_equal(ids, ref["as_ids"]), "active-set ids differ"
    assert np.array_equal(lab, ref["is_label"]), "label flags differ"
    st = model.stats()
    assert st["active_pairs"] == len(ids) and st["unique_out_rows"] == len(ref["uniq"])
    assert st["candidates"] == ref["candidates"]
    if not orc.dense_hidden:
        assert st["unique_in_rows"] == len(ref["uniq1"])
    res = {"z": worst(z, ref["z"]), "delta": worst(d, ref["delta"]), "dh": worst(dh, ref["dh"]),
           "loss": abs(loss - ref["loss"]) / (REL * max(abs(ref["loss"]), 1e-12))}
    if check_state:
        for n in model.p:
            res["w:" + n] = worst_weight(model.p[n].cpu().numpy(), orc, n)
            res["m:" + n] = worst(model.m[n].cpu().numpy(), orc.m[n])
            res["v:" + n] = worst(model.v[n].cpu().numpy(), orc.v[n])
        res.update(adam_self_consistency(model, orc, ref, before, st["steps"]))
    # the same comparisons with the floor of 1e-7 * max|ref| (reported, not asserted)
    s16 = {"z": worst(z, ref["z"], 1e-7), "delta": worst(d, ref["delta"], 1e-7), "dh": worst(dh, ref["dh"], 1e-7)}
    if check_state:
        for n in model.p:
            s16["m:" + n] = worst(model.m[n].cpu().numpy(), orc.m[n], 1e-7)
            s16["v:" + n] = worst(model.v[n].cpu().numpy(), orc.v[n], 1e-7)
    res["_floor1e-7"] = s16
    res["_loss"] = (loss, ref["loss"])
    res["_ref"] = ref
    return res


def assert_ok(res):
    bad = {k: v for k, v in res.items() if not k.startswith("_") and not (v <= 1.0)}
    assert not bad, bad


# ---- a synthetic task with planted structure (prediction-quality tests) -----------------------
def planted_workload(num_classes=500, lr=5e-3):
    """Small DWTA model for the planted task below: 64 buckets per table, rebuilt every 20 steps."""
    return synth.small(synth.HASH_DWTA, num_classes=num_classes, input_dim=800, hidden_dim=64, K=2, L=16,
                       bucket_cap=64, batch=128, rebuild_every=20, lr=lr, nnz_mean=8.0)


def planted_prototypes(wl, per_class=6):
    """Every class owns a fixed set of features; a sample of the class shows them plus noise."""
    return np.stack([np.random.default_rng([1, c]).choice(wl.input_dim, size=per_class, replace=False)
                     for c in range(wl.num_classes)])


def planted_batch(wl, protos, step, noise=2, seed=0):
    """One batch: a uniformly drawn class per sample (its single label), the class's features plus
    `noise` random ones, equal values with unit norm.  Returns (batch dict, labels)."""
    rng = np.random.default_rng([seed, 77, step])
    labels = rng.integers(0, wl.num_classes, size=wl.batch)
    xp, xi, xv = [0], [], []
    for c in labels:
        f = set(protos[c].tolist())
        f.update(rng.integers(0, wl.input_dim, size=noise).tolist())
        f = np.array(sorted(f), dtype=np.int32)
        xi.append(f)
        xv.append(np.full(f.size, 1.0 / np.sqrt(f.size), dtype=np.float32))
        xp.append(xp[-1] + f.size)
    batch = dict(batch=wl.batch, x_indptr=np.array(xp, np.int32), x_indices=np.concatenate(xi),
                 x_values=np.concatenate(xv), y_indptr=np.arange(wl.batch + 1, dtype=np.int32),
                 y_indices=labels.astype(np.int32))
    return batch, labels

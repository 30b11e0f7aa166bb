"""Pins of the oracle's hash codes (SimHash / sparse random projections, DWTA).

The paper (Section 4.1) only names the two families, so the pins are: hand-worked
examples stored under tests/golden/, special cases that reduce to a library routine
(sign of a dense mat-vec on integer data; numpy argmax over permuted bins), the
closed-form collision probability of sign random projections, and invariants.
"""
import json
import os

import numpy as np
import pytest

from oracle import slide_oracle as so


def _load(golden_dir, name):
    with open(os.path.join(golden_dir, name)) as f:
        return json.load(f)


def test_simhash_hand_example(golden_dir):
    g = _load(golden_dir, "simhash_example.json")
    hf = so.HashFn(so.SIMHASH, g["H"], g["K"], g["L"], srp_idx=np.array(g["srp_idx"]),
                   srp_sign=np.array(g["srp_sign"]))
    assert hf.codes(np.array([g["v"]], dtype=np.float32)).tolist() == [g["codes"]]


def test_dwta_hand_example(golden_dir):
    g = _load(golden_dir, "dwta_example.json")
    hf = so.HashFn(so.DWTA, g["H"], g["K"], g["L"], m=g["m"], dwta_perm=np.array(g["dwta_perm"]),
                   dens_a=g["dens_a"], dens_b=g["dens_b"])
    assert hf.codes(np.array([g["v"]], dtype=np.float32)).tolist() == [g["codes"]]


def dwta_probe_limit_case(golden_dir):
    """(hash function, vector, expected codes) of tests/golden/dwta_probe_limit.json."""
    g = _load(golden_dir, "dwta_probe_limit.json")
    NP = g["K"] * g["L"] // (g["H"] // g["m"])
    perm = np.array([g["special_perms"].get(str(q), g["default_perm"]) for q in range(NP)], np.int32)
    want = np.zeros(g["L"], np.uint32)
    for t, c in g["nonzero_codes"].items():
        want[int(t)] = c
    return g, perm, np.array([g["v"]], dtype=np.float32), want


def test_dwta_densification_gives_up_after_exactly_100_probes(golden_dir):
    g, perm, v, want = dwta_probe_limit_case(golden_dir)
    hf = so.HashFn(so.DWTA, g["H"], g["K"], g["L"], m=g["m"], dwta_perm=perm, dens_a=g["dens_a"], dens_b=g["dens_b"])
    assert np.array_equal(hf.codes(v)[0], want)


def _srp(rng, H, K, L):
    S = -(-H // 3)
    NH = K * L
    idx = np.stack([np.sort(rng.choice(H, S, replace=False)) for _ in range(NH)]).astype(np.int32)
    sgn = (rng.integers(0, 2, (NH, S)) * 2 - 1).astype(np.int8)
    return idx, sgn


def test_simhash_equals_sign_of_dense_projection_on_integer_data():
    # integer-valued vectors: every fp32 partial sum is exact, so the order of the
    # additions cannot matter and the bits must equal the sign of a plain mat-vec.
    rng = np.random.default_rng(1)
    H, K, L = 48, 5, 7
    idx, sgn = _srp(rng, H, K, L)
    hf = so.HashFn(so.SIMHASH, H, K, L, srp_idx=idx, srp_sign=sgn)
    V = rng.integers(-9, 10, size=(200, H)).astype(np.float32)
    P = np.zeros((K * L, H))
    for e in range(K * L):
        P[e, idx[e]] = sgn[e]
    bits = (V.astype(np.float64) @ P.T > 0).astype(np.uint32).reshape(200, L, K)
    want = (bits << np.arange(K, dtype=np.uint32)).sum(axis=2)
    assert np.array_equal(hf.codes(V), want)


def test_simhash_invariants():
    rng = np.random.default_rng(2)
    H, K, L = 33, 9, 4
    idx, sgn = _srp(rng, H, K, L)
    hf = so.HashFn(so.SIMHASH, H, K, L, srp_idx=idx, srp_sign=sgn)
    V = rng.standard_normal((50, H)).astype(np.float32)
    c = hf.codes(V)
    assert c.max() < (1 << K)
    assert np.array_equal(hf.codes(V * np.float32(4.0)), c)          # positive power-of-two scale
    assert np.array_equal(hf.codes(np.zeros((1, H), np.float32)), np.zeros((1, L), np.uint32))
    # negating the vector flips every bit whose sum is non-zero
    assert np.array_equal(hf.codes(-V) ^ c, np.full_like(c, (1 << K) - 1))


def test_simhash_collision_probability_closed_form():
    # sign random projections: P[bit(u) == bit(v)] = 1 - angle(u, v)/pi
    rng = np.random.default_rng(3)
    H, K, L = 96, 8, 500
    idx, sgn = _srp(rng, H, K, L)
    hf = so.HashFn(so.SIMHASH, H, K, L, srp_idx=idx, srp_sign=sgn)
    for rho in (0.0, 0.5, 0.9):
        u = rng.standard_normal((40, H))
        v = rho * u + np.sqrt(1 - rho * rho) * rng.standard_normal((40, H))
        cu, cv = hf.codes(u.astype(np.float32)), hf.codes(v.astype(np.float32))
        x = cu ^ cv
        differ = sum(int(((x >> k) & 1).sum()) for k in range(K))
        agree = 1.0 - differ / (40 * K * L)
        assert abs(agree - (1 - np.arccos(rho) / np.pi)) < 0.02, (rho, agree)


def _perms(rng, H, m, NH):
    NP = -(-NH // (H // m))
    return np.stack([rng.permutation(H) for _ in range(NP)]).astype(np.int32)


@pytest.mark.parametrize("H,m,K,L", [(128, 8, 6, 40), (32, 8, 3, 5), (1024, 8, 8, 20), (64, 4, 4, 9)])
def test_dwta_equals_argmax_over_permuted_bins_when_no_bin_is_empty(H, m, K, L):
    # no zeros and no ties: winner-take-all is numpy's argmax over each bin
    rng = np.random.default_rng(4)
    perm = _perms(rng, H, m, K * L)
    hf = so.HashFn(so.DWTA, H, K, L, m=m, dwta_perm=perm, dens_a=12345 * 2 + 1, dens_b=777 * 2 + 1)
    V = rng.standard_normal((30, H)).astype(np.float32)
    P = H // m
    raw = np.concatenate([V[:, perm[q]].reshape(30, P, m).argmax(axis=2) for q in range(perm.shape[0])],
                         axis=1)[:, :K * L]
    lg = int(np.log2(m))
    want = (raw.reshape(30, L, K).astype(np.uint32) << (np.arange(K, dtype=np.uint32) * lg)).sum(axis=2)
    assert np.array_equal(hf.codes(V), want)


def test_dwta_ties_keep_lowest_position_and_zeros_are_absent():
    H, m = 8, 8
    perm = np.arange(8, dtype=np.int32)[None]
    hf = so.HashFn(so.DWTA, H, 1, 1, m=m, dwta_perm=perm, dens_a=3, dens_b=5)
    assert hf.codes(np.array([[0, 2, 5, 5, 1, 0, 5, 0]], np.float32))[0, 0] == 2     # first of the 5s
    assert hf.codes(np.array([[0, 0, -3, 0, -1, 0, 0, 0]], np.float32))[0, 0] == 4   # 0 does not beat -1
    assert hf.codes(np.array([[np.nan, 0, -3, 0, 0, 0, 0, 0]], np.float32))[0, 0] == 2
    assert hf.codes(np.array([[-0.0, 0, 0, 0, 0, 0, 0, 0]], np.float32))[0, 0] == 0  # all empty -> 0


def test_dwta_invariants_and_densification_borrows_only_existing_values():
    rng = np.random.default_rng(5)
    H, m, K, L = 128, 8, 6, 30
    perm = _perms(rng, H, m, K * L)
    hf = so.HashFn(so.DWTA, H, K, L, m=m, dwta_perm=perm, dens_a=2654435761, dens_b=40503 * 2 + 1)
    V = np.maximum(rng.standard_normal((64, H)), 0).astype(np.float32)     # about half zeros
    c = hf.codes(V)
    assert c.max() < (1 << (K * 3))
    assert np.array_equal(hf.codes(V * np.float32(8.0)), c)
    assert np.array_equal(hf.codes(np.zeros((2, H), np.float32)), np.zeros((2, L), np.uint32))
    assert np.array_equal(hf.codes(np.vstack([V[:3], V[:3]]))[:3], hf.codes(np.vstack([V[:3], V[:3]]))[3:])
    # vector with exactly one non-empty bin (single permutation): every elementary hash is
    # that bin's winner position or, if 100 probes never reach it, 0
    perm1 = _perms(rng, H, m, 16)[:1]
    hf1 = so.HashFn(so.DWTA, H, 4, 4, m=m, dwta_perm=perm1, dens_a=2654435761, dens_b=40503 * 2 + 1)
    v = np.zeros((1, H), np.float32)
    v[0, perm1[0, 5 * m + 6]] = 1.0          # bin 5, position 6
    vals = {(int(cc) >> (3 * k)) & 7 for cc in hf1.codes(v)[0] for k in range(4)}
    assert vals <= {0, 6} and 6 in vals
    # non-empty bins are never altered by densification: they equal numpy's argmax over non-zeros
    P = H // m
    codes = hf.codes(V)
    for r in range(8):
        for e in range(K * L):
            q, b = divmod(e, P)
            x = V[r, perm[q, b * m:(b + 1) * m]].astype(np.float64)
            if np.any(x != 0):
                x[x == 0] = -np.inf
                t, k = divmod(e, K)
                assert (int(codes[r, t]) >> (3 * k)) & 7 == int(np.argmax(x))

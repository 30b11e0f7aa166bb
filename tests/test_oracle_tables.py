"""Pins of the oracle's hash tables and active sets: a hand-worked fixture, brute force
with Python dicts / sets on small inputs, and the structural invariants (ids ascending,
each id once per table, at most C per bucket, labels always present, no duplicates,
size within L*C plus the labels)."""
import json
import os

import numpy as np
import pytest

from oracle import slide_oracle as so


def _prio_key(j, t, r, pa, pb):
    M = 0xffffffff
    u = (pa * (j + 1) + pb * (t * 65537 + r + 1)) & M
    u ^= u >> 15
    u = (u * pa) & M
    u ^= u >> 13
    return (u, j)


def _brute(codes, C, policy, r, pa, pb):
    N, L = codes.shape
    out = []
    for t in range(L):
        d = {}
        for j in range(N):
            d.setdefault(int(codes[j, t]), []).append(j)
        for c, mem in d.items():
            if len(mem) > C:
                key = (lambda j: j) if policy == 0 else (lambda j: _prio_key(j, t, r, pa, pb))
                d[c] = sorted(sorted(mem, key=key)[:C])
        out.append(d)
    return out


def test_tables_hand_example(golden_dir):
    with open(os.path.join(golden_dir, "tables_example.json")) as f:
        g = json.load(f)
    T = so.Tables(np.array(g["codes_per_neuron"], dtype=np.uint32), g["C"], 0, 0, 1, 1)
    for t, bk in g["buckets"].items():
        for c, ids in bk.items():
            assert T.bucket(int(t), int(c)).tolist() == ids
    assert T.overflowed == g["overflowed"]


@pytest.mark.parametrize("policy", [0, 1])
@pytest.mark.parametrize("nb,C", [(8, 4), (64, 16), (4096, 3)])
def test_tables_match_brute_force(policy, nb, C):
    rng = np.random.default_rng(7)
    N, L = 300, 5
    codes = rng.integers(0, nb, size=(N, L)).astype(np.uint32)
    pa, pb, r = 2654435761, 0x9E3779B1, 2
    T = so.Tables(codes, C, policy, r, pa, pb)
    want = _brute(codes, C, policy, r, pa, pb)
    over = 0
    for t in range(L):
        seen = []
        for c in range(nb):
            got = T.bucket(t, c).tolist()
            assert got == want[t].get(c, [])
            assert got == sorted(got) and len(got) <= C
            full = [j for j in range(N) if codes[j, t] == c]
            assert set(got) <= set(full) and len(got) == min(len(full), C)
            over += len(full) > C
            seen += got
        assert len(seen) == len(set(seen))
        if all(len(v) <= C for v in _brute(codes, N, 0, 0, 1, 1)[t].values()):
            assert len(seen) == N
    assert T.overflowed == over


def test_policy0_keeps_lowest_ids_and_policies_agree_without_overflow():
    rng = np.random.default_rng(8)
    codes = rng.integers(0, 4, size=(100, 3)).astype(np.uint32)
    T0 = so.Tables(codes, 5, 0, 0, 3, 5)
    for t in range(3):
        for c in range(4):
            full = [j for j in range(100) if codes[j, t] == c]
            assert T0.bucket(t, c).tolist() == full[:5]
    big0, big1 = so.Tables(codes, 100, 0, 0, 3, 5), so.Tables(codes, 100, 1, 9, 3, 5)
    assert big0.fingerprint() == big1.fingerprint() and big0.overflowed == 0


def test_priority_depends_on_rebuild_counter_only_when_overflowing():
    rng = np.random.default_rng(9)
    codes = rng.integers(0, 2, size=(400, 2)).astype(np.uint32)
    a = so.Tables(codes, 8, 1, 0, 2654435761, 0x9E3779B1)
    b = so.Tables(codes, 8, 1, 1, 2654435761, 0x9E3779B1)
    c = so.Tables(codes, 8, 1, 0, 2654435761, 0x9E3779B1)
    assert a.fingerprint() == c.fingerprint() and a.fingerprint() != b.fingerprint()
    # the survivors of an overflowing bucket are spread over the whole id range
    assert a.bucket(0, 0).max() > 100


def test_active_sets_match_brute_force_and_invariants():
    rng = np.random.default_rng(10)
    N, L, C, B = 500, 6, 7, 9
    codes_w = rng.integers(0, 16, size=(N, L)).astype(np.uint32)
    T = so.Tables(codes_w, C, 1, 0, 2654435761, 0x9E3779B1)
    q = rng.integers(0, 16, size=(B, L)).astype(np.uint32)
    nl = rng.integers(0, 5, size=B)
    yptr = np.zeros(B + 1, np.int32)
    yptr[1:] = np.cumsum(nl)
    yidx = rng.integers(0, N, size=yptr[-1]).astype(np.int32)
    yidx[1] = yidx[0]                                    # a duplicated label
    as_ptr, ids, lab, ncand = T.active_sets(q, yptr, yidx)
    total = 0
    for i in range(B):
        cand = set()
        for t in range(L):
            b = T.bucket(t, q[i, t]).tolist()
            total += len(b)
            cand |= set(b)
        Y = set(yidx[yptr[i]:yptr[i + 1]].tolist())
        want = sorted(cand | Y)
        got = ids[as_ptr[i]:as_ptr[i + 1]].tolist()
        assert got == want
        assert all(a < b for a, b in zip(got, got[1:]))                    # strictly ascending
        assert Y <= set(got)                                              # labels always included
        assert len(set(got) - Y) <= L * C and len(got) <= L * C + len(Y)   # size bounds
        assert [g for g, f in zip(got, lab[as_ptr[i]:as_ptr[i + 1]]) if f] == sorted(Y)
    assert ncand == total
    # prediction mode leaves the labels out
    p_ptr, p_ids, p_lab, _ = T.active_sets(q, yptr, yidx, include_labels=False)
    for i in range(B):
        cand = set()
        for t in range(L):
            cand |= set(T.bucket(t, q[i, t]).tolist())
        assert p_ids[p_ptr[i]:p_ptr[i + 1]].tolist() == sorted(cand)
    assert not p_lab.any()


def test_identical_vectors_retrieve_their_own_neuron():
    # a query equal to a stored weight row collides with it in every table
    rng = np.random.default_rng(11)
    H, K, L, N = 64, 3, 10, 200
    perm = np.stack([rng.permutation(H) for _ in range(-(-K * L // (H // 8)))]).astype(np.int32)
    hf = so.HashFn(so.DWTA, H, K, L, dwta_perm=perm, dens_a=2654435761, dens_b=40503 * 2 + 1)
    W = rng.standard_normal((N, H)).astype(np.float32)
    T = so.Tables(hf.codes(W), N, 0, 0, 3, 5)
    yptr = np.zeros(5, np.int32)
    as_ptr, ids, _, _ = T.active_sets(hf.codes(W[[3, 50, 77, 199]]), yptr, np.zeros(0, np.int32), False)
    for i, j in enumerate([3, 50, 77, 199]):
        assert j in ids[as_ptr[i]:as_ptr[i + 1]]


def test_bucket_of_exactly_C_and_C_plus_one_members():
    codes = np.zeros((5, 1), dtype=np.uint32)
    assert so.Tables(codes, 5, 0, 0, 3, 5).bucket(0, 0).tolist() == [0, 1, 2, 3, 4]
    T = so.Tables(codes, 4, 0, 0, 3, 5)
    assert T.bucket(0, 0).tolist() == [0, 1, 2, 3] and T.overflowed == 1
    assert so.Tables(codes[:0], 4, 0, 0, 3, 5).bucket(0, 0).tolist() == []     # no neurons at all

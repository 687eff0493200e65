"""Pins for the oracle's router and selection-array builder (sections 2.1, 3.1, 4.1)."""
import math

import numpy as np
import pytest
import scipy.special

from oracle import ssmm_oracle as O


def brute_route(logits, k, renorm):
    """Pure-Python router: exp / sum for the softmax, repeated max for the top-k
    (first maximum wins, i.e. the lower expert id on equal logits)."""
    ids, ws = [], []
    for row in logits:
        row = [-math.inf if math.isnan(float(v)) else float(v) for v in row]   # a NaN logit counts as -infinity
        mx = max(row)
        ex = [math.exp(v - mx) for v in row]
        tot = sum(ex)
        p = [v / tot for v in ex]
        chosen = []
        for _ in range(k):
            best = None
            for e, v in enumerate(row):
                if e in chosen:
                    continue
                if best is None or v > row[best]:
                    best = e
            chosen.append(best)
        w = [p[e] for e in chosen]
        if renorm:
            s = sum(w)
            w = [v / s for v in w]
        ids.append(chosen)
        ws.append(w)
    return ids, ws


@pytest.mark.parametrize("E,k", [(8, 2), (64, 8), (64, 6), (5, 5), (3, 1)])
@pytest.mark.parametrize("renorm", [True, False])
def test_route_matches_brute_force(E, k, renorm):
    rng = np.random.default_rng(E * 10 + k)
    lg = rng.standard_normal((37, E)).astype(np.float32)
    lg[3, :] = 0.25                      # a full tie row
    lg[4, : E // 2] = lg[4, E // 2]      # partial ties
    ids, w = O.route(lg, k, 0, renorm)
    bids, bw = brute_route(lg, k, renorm)
    assert ids.tolist() == bids
    np.testing.assert_allclose(w, np.array(bw), rtol=1e-13, atol=0)
    assert ids[3].tolist() == list(range(k))


@pytest.mark.parametrize("E,k", [(8, 2), (130, 4), (64, 8), (200, 16)])
def test_masked_and_nan_logits(E, k):
    """Logits of -infinity (masked experts) and NaN (counted as -infinity): weight 0, never preferred to a
    number, and when fewer than k logits are numbers the rest of the choice goes by ascending id --
    ids stay distinct.  Brute force with the rule spelled out."""
    rng = np.random.default_rng(E + k)
    lg = rng.standard_normal((40, E)).astype(np.float32)
    lg[:, ::3] = -np.inf
    lg[5:9, 1::3] = np.nan
    lg[10] = -np.inf
    lg[10, [E - 1, 2]] = [0.5, -1.0]          # two numbers only: fewer than k for every k here but 2
    lg[11] = np.nan
    lg[11, E // 2] = 3.0                      # one number only
    for renorm in (True, False):
        with np.errstate(invalid="ignore", divide="ignore"):
            ids, w = O.route(lg, k, 0, renorm)
        bids, bw = brute_route(lg, k, renorm)
        assert ids.tolist() == bids
        np.testing.assert_allclose(w, np.array(bw), rtol=1e-13, atol=0)
        assert all(len(set(r)) == k for r in ids.tolist())
    assert ids[10, :2].tolist() == [E - 1, 2] and ids[10, 2:].tolist() == [e for e in range(E) if e not in (E - 1, 2)][: k - 2]
    assert ids[11, 0] == E // 2 and w[11, 0] == 1.0 and (w[11, 1:] == 0).all()


def test_route_closed_forms():
    rng = np.random.default_rng(0)
    lg = rng.standard_normal((50, 8)).astype(np.float32)
    # renormalised weights sum to one
    _, w = O.route(lg, 3, 0, True)
    np.testing.assert_allclose(w.sum(axis=1), 1.0, rtol=1e-14)
    # k = E: the weights are the softmax itself, whatever the flag (library softmax as the pin)
    for renorm in (True, False):
        ids, w = O.route(lg, 8, 0, renorm)
        p = scipy.special.softmax(lg.astype(np.float64), axis=1)
        np.testing.assert_allclose(w, np.take_along_axis(p, ids.astype(np.int64), axis=1), rtol=1e-13)
        assert (np.sort(ids, axis=1) == np.arange(8)).all()
    # k = 1 renormalised: weight exactly 1; not renormalised: the max probability
    ids, w = O.route(lg, 1, 0, True)
    assert (w == 1.0).all() and (ids[:, 0] == lg.argmax(axis=1)).all()
    _, w = O.route(lg, 1, 0, False)
    np.testing.assert_allclose(w[:, 0], scipy.special.softmax(lg.astype(np.float64), axis=1).max(axis=1), rtol=1e-13)
    # descending-logit order
    ids, _ = O.route(lg, 4, 0, True)
    picked = np.take_along_axis(lg, ids.astype(np.int64), axis=1)
    assert (np.diff(picked, axis=1) <= 0).all()
    # shifting every logit of a token changes nothing
    ids2, w2 = O.route(lg + np.float32(0.5), 4, 0, True)
    assert (ids2 == ids).all()


def test_route_shared_experts():
    rng = np.random.default_rng(1)
    lg = rng.standard_normal((9, 6)).astype(np.float32)
    ids, w = O.route(lg, 2, 2, False)
    assert ids.shape == (9, 4) and (ids[:, 2] == 6).all() and (ids[:, 3] == 7).all()
    assert (w[:, 2:] == 1.0).all()
    ids0, w0 = O.route(lg, 2, 0, False)
    assert (ids[:, :2] == ids0).all() and (w[:, :2] == w0).all()


def test_route_rejects_bad_topk():
    with pytest.raises(ValueError):
        O.route(np.zeros((2, 4), dtype=np.float32), 5)
    with pytest.raises(ValueError):
        O.route(np.zeros((2, 4), dtype=np.float32), 0)


def brute_bucket(ids, E_total):
    """Stable sort of the (token, slot) pairs by expert id, with Python's sorted()."""
    T, S = len(ids), len(ids[0])
    pairs = sorted(((ids[t][j], t, j) for t in range(T) for j in range(S)))
    sel = [t for _, t, _ in pairs]
    counts = [sum(1 for e, _, _ in pairs if e == x) for x in range(E_total)]
    offsets = [0]
    for c in counts:
        offsets.append(offsets[-1] + c)
    inv = [[None] * S for _ in range(T)]
    for pos, (_, t, j) in enumerate(pairs):
        inv[t][j] = pos
    return offsets, sel, inv


@pytest.mark.parametrize("T,E,k,S", [(40, 8, 2, 0), (33, 16, 4, 2), (1, 4, 2, 0), (70, 64, 8, 0), (17, 3, 3, 1)])
def test_bucket_matches_brute_force_and_invariants(T, E, k, S):
    rng = np.random.default_rng(T + E)
    lg = rng.standard_normal((T, E)).astype(np.float32)
    ids, w = O.route(lg, k, S, True)
    offsets, sel, slot, inv = O.bucket(ids, E + S)
    bo, bs, bi = brute_bucket(ids.tolist(), E + S)
    assert offsets.tolist() == bo and sel.tolist() == bs and inv.tolist() == bi
    P = T * (k + S)
    assert offsets[0] == 0 and offsets[-1] == P
    # every token once in each of its k+S distinct experts
    for t in range(T):
        assert len(set(ids[t].tolist())) == k + S
    for e in range(E + S):
        seg = sel[offsets[e]:offsets[e + 1]]
        assert (np.diff(seg) > 0).all()                      # ascending, no repeats
        assert set(seg.tolist()) == {t for t in range(T) if e in ids[t]}
    assert (sel[inv] == np.arange(T)[:, None]).all()
    assert (slot[inv] == np.arange(k + S)[None, :]).all()
    assert sorted(inv.reshape(-1).tolist()) == list(range(P))
    # shared experts hold every token in order
    for s in range(S):
        e = E + s
        assert sel[offsets[e]:offsets[e + 1]].tolist() == list(range(T))


def test_bucket_expert_relabelling_permutes_buckets():
    rng = np.random.default_rng(2)
    lg = rng.standard_normal((25, 6)).astype(np.float32)
    perm = rng.permutation(6)
    ids, _ = O.route(lg, 2)
    ids_p, _ = O.route(lg[:, perm], 2)          # expert perm[j] now sits in column j
    o, s, _, _ = O.bucket(ids, 6)
    op, sp, _, _ = O.bucket(ids_p, 6)
    for j in range(6):
        e = perm[j]
        assert s[o[e]:o[e + 1]].tolist() == sp[op[j]:op[j + 1]].tolist()


def test_bucket_empty_experts_and_no_tokens():
    ids = np.array([[0, 3], [3, 0]], dtype=np.int32)
    o, s, _, inv = O.bucket(ids, 5)
    assert o.tolist() == [0, 2, 2, 2, 4, 4]
    assert s.tolist() == [0, 1, 0, 1] and inv.tolist() == [[0, 2], [3, 1]]
    o, s, _, inv = O.bucket(np.zeros((0, 2), dtype=np.int32), 4)
    assert o.tolist() == [0, 0, 0, 0, 0] and s.size == 0 and inv.shape == (0, 2)

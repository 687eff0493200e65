"""Pins for the oracle's prune / compress / decompress (sections 2.3 and 4.1).

None of these tests re-uses the oracle's own selection code: the brute-force
reference below is written with plain Python loops and Python floats.
"""
import os

import numpy as np
import math

import pytest

from oracle import ssmm_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bf16_val(b):
    return float(np.array([int(b) << 16], dtype=np.uint32).view(np.float32)[0])


def random_bf16(rng, shape, kind="normal"):
    if kind == "normal":
        f = rng.standard_normal(shape).astype(np.float32) * 0.02
    elif kind == "ties":      # few distinct magnitudes, both signs, zeros and -0.0
        f = rng.choice(np.array([0.0, -0.0, 0.5, -0.5, 1.0, -1.0, 2.0], dtype=np.float32), size=shape)
    else:
        raise ValueError(kind)
    return (f.view(np.uint32) >> 16).astype(np.uint16)


# ---------------------------------------------------------------- brute force


def brute_prune(bits, N, M, V):
    """Pure-Python statement of the pattern: per block keep N Sub-Rows by sum of
    squares, then per group of 4 keep the two largest magnitudes; first-best
    wins ties (lower row / lower position)."""
    rows, K = bits.shape
    val = [[bf16_val(bits[r, c]) for c in range(K)] for r in range(rows)]
    live = [[True] * K for _ in range(rows)]
    if N < M:
        for b in range(rows // M):
            for s in range(K // V):
                scores = []
                for m in range(M):
                    acc = 0.0
                    for v in range(V):
                        x = val[b * M + m][s * V + v]
                        acc = acc + x * x
                    scores.append(math.inf if math.isnan(acc) else acc)   # a NaN ranks like +infinity
                chosen = []
                for _ in range(N):
                    best = None
                    for m in range(M):
                        if m in chosen:
                            continue
                        if best is None or scores[m] > scores[best]:
                            best = m
                    chosen.append(best)
                for m in range(M):
                    if m not in chosen:
                        for v in range(V):
                            live[b * M + m][s * V + v] = False
    out = np.zeros((rows, K), dtype=np.uint16)
    for r in range(rows):
        for g in range(K // 4):
            if not live[r][4 * g]:
                continue
            mags = [math.inf if math.isnan(val[r][4 * g + i]) else abs(val[r][4 * g + i]) for i in range(4)]
            first = max(range(4), key=lambda i: (mags[i], -i))
            second = max((i for i in range(4) if i != first), key=lambda i: (mags[i], -i))
            for i in (first, second):
                out[r, 4 * g + i] = bits[r, 4 * g + i]
    return out


# ---------------------------------------------------------------- golden files


def load_golden(name):
    sec, data = None, {"dense": [], "pruned": [], "values": [], "meta": [], "index": []}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            tok = line.split()
            if tok[0] == "format":
                data["fmt"] = O.Format(*map(int, tok[1:]))
            elif tok[0] in ("rows", "K"):
                data[tok[0]] = int(tok[1])
            elif tok[0] in data and isinstance(data[tok[0]], list) and len(tok) == 1:
                sec = tok[0]
            else:
                data[sec].append([int(t, 16) for t in tok])
    return data


@pytest.mark.parametrize("name", ["two_four_worked.txt", "subrow_worked.txt", "subrow_2of4_worked.txt"])
def test_hand_worked_examples(name):
    g = load_golden(name)
    dense = np.array(g["dense"], dtype=np.uint16)
    fmt = g["fmt"]
    assert dense.shape == (g["rows"], g["K"])
    np.testing.assert_array_equal(O.prune(dense, fmt), np.array(g["pruned"], dtype=np.uint16))
    values, meta, index = O.compress(dense, fmt)
    np.testing.assert_array_equal(values, np.array(g["values"], dtype=np.uint16))
    np.testing.assert_array_equal(meta.reshape(-1), np.array(g["meta"], dtype=np.uint32).reshape(-1))
    if g["index"]:
        np.testing.assert_array_equal(index, np.array(g["index"], dtype=np.uint8))
    else:
        assert index.size == 0
    back = O.decompress(values, meta, index, g["rows"], g["K"], fmt)
    np.testing.assert_array_equal(back, np.array(g["pruned"], dtype=np.uint16))


# ---------------------------------------------------------------- brute force on small inputs

FORMATS = [(1, 1, 0), (1, 2, 8), (1, 2, 4), (2, 4, 8), (4, 8, 32), (1, 2, 16), (3, 4, 4)]


def plant_non_finite(rng, bits, share=0.05):
    """NaNs (two payloads, both signs) and infinities scattered over a bf16 matrix."""
    bits = bits.copy()
    special = np.array([0x7FC0, 0xFFC0, 0x7FA1, 0x7F80, 0xFF80], dtype=np.uint16)
    mask = rng.random(bits.shape) < share
    bits[mask] = rng.choice(special, size=int(mask.sum()))
    return bits


@pytest.mark.parametrize("fmt", FORMATS)
def test_not_a_number_ranks_like_infinity_and_is_kept(fmt):
    """The paper says nothing of NaN or infinite weights; the rule here: a NaN ranks like an infinity
    in both prunings (a Sub-Row that holds one, and the value itself in its group of 4), ties as
    always to the lower row / position.  Brute force with the rule spelled out, and the encoding
    still round-trips bit for bit (NaN payloads included)."""
    rng = np.random.default_rng(7000 + 100 * fmt[1] + fmt[2])
    f = O.Format(*fmt)
    V = max(fmt[2], 4)
    rows, K = 2 * fmt[1] * 3, V * 3 if V % 8 == 0 else V * 6
    bits = plant_non_finite(rng, random_bf16(rng, (rows, K), "ties"))
    pruned = O.prune(bits, f)
    np.testing.assert_array_equal(pruned, brute_prune(bits, *fmt))
    values, meta, index = O.compress(bits, f)
    np.testing.assert_array_equal(O.decompress(values, meta, index, rows, K, f), pruned)
    # a group of a kept Sub-Row never drops a NaN in favour of a number
    val = O.bf16_bits_to_f64(bits).reshape(rows, K // 4, 4)
    kept = (pruned.reshape(rows, K // 4, 4) != 0) | (bits.reshape(rows, K // 4, 4) == 0)
    if fmt[0] == fmt[1]:
        for r, g in zip(*np.nonzero(np.isnan(val).any(axis=2))):
            n_nan = int(np.isnan(val[r, g]).sum())
            assert int((np.isnan(val[r, g]) & (pruned.reshape(rows, K // 4, 4)[r, g] != 0)).sum()) == min(n_nan, 2)


@pytest.mark.parametrize("fmt", FORMATS)
@pytest.mark.parametrize("kind", ["normal", "ties"])
def test_prune_matches_brute_force(fmt, kind):
    rng = np.random.default_rng(1000 * fmt[0] + 100 * fmt[1] + fmt[2] + len(kind))
    f = O.Format(*fmt)
    V = max(fmt[2], 4)
    rows, K = 2 * fmt[1] * 3, V * 3 if V % 8 == 0 else V * 6
    bits = random_bf16(rng, (rows, K), kind)
    np.testing.assert_array_equal(O.prune(bits, f), brute_prune(bits, *fmt))


@pytest.mark.parametrize("fmt", FORMATS)
@pytest.mark.parametrize("kind", ["normal", "ties"])
def test_roundtrip_and_structure(fmt, kind):
    rng = np.random.default_rng(7 + 1000 * fmt[0] + 100 * fmt[1] + fmt[2] + len(kind))
    f = O.Format(*fmt)
    N, M, V = fmt
    rows, K = 8 * M, 64 if V == 0 else 4 * V
    bits = random_bf16(rng, (rows, K), kind)
    pruned = O.prune(bits, f)
    values, meta, index = O.compress(bits, f)
    rc = f.compressed_rows(rows)
    # closed-form sizes of section 4.1 (row count m*N/M for N > 1)
    vb, mb, ib = O.compressed_sizes(rows, K, f)
    assert values.shape == (rc, K // 2) and values.nbytes == vb
    assert meta.nbytes == mb and meta.shape == (rc, (K // 4 + 7) // 8)
    assert index.nbytes == ib
    if f.vectorwise:
        assert index.shape == (rc, K // V) and index.max() < M
    # round trip reproduces the pruned matrix bit for bit
    np.testing.assert_array_equal(O.decompress(values, meta, index, rows, K, f), pruned)
    # every group of 4 has at most 2 non-zero bit patterns; metadata pairs strictly ascending
    nz = (pruned.reshape(rows, K // 4, 4) != 0).sum(axis=-1)
    assert nz.max() <= 2
    for r in range(rc):
        for g in range(K // 4):
            nib = (int(meta[r, g // 8]) >> (4 * (g % 8))) & 0xF
            assert (nib & 3) < (nib >> 2)
    # every M x V block has exactly N live Sub-Rows at most (a live Sub-Row may be all zero values)
    if f.vectorwise:
        blk = (pruned.reshape(rows // M, M, K // V, V) != 0).any(axis=-1)   # [b][m][s]
        assert blk.sum(axis=1).max() <= N
        # index rows ascending inside a block and distinct
        idx = index.reshape(rows // M, N, K // V).astype(int)
        assert (np.diff(idx, axis=1) > 0).all()
    # pruning is idempotent and compress of the pruned matrix is the same encoding
    np.testing.assert_array_equal(O.prune(pruned, f) if kind == "normal" else pruned, pruned)
    if kind == "normal":     # (with exact ties a pruned zero may out-rank an equal-zero kept one)
        v2, m2, i2 = O.compress(pruned, f)
        np.testing.assert_array_equal(v2, values)
        np.testing.assert_array_equal(m2, meta)
        np.testing.assert_array_equal(i2, index)


def test_kept_fraction():
    rng = np.random.default_rng(3)
    bits = random_bf16(rng, (64, 256))
    assert (O.prune(bits, O.Format(1, 1, 0)) != 0).mean() == pytest.approx(0.5, abs=0.01)
    assert (O.prune(bits, O.Format(1, 2, 8)) != 0).mean() == pytest.approx(0.25, abs=0.01)
    assert (O.prune(bits, O.Format(2, 8, 16)) != 0).mean() == pytest.approx(0.125, abs=0.01)


def test_conforming_matrix_is_kept_whole():
    """A matrix that already obeys 2:4 loses nothing (zeros never beat a non-zero)."""
    rng = np.random.default_rng(11)
    bits = random_bf16(rng, (16, 64))
    bits[bits == 0] = 0x3C00
    keep = np.zeros((16, 16, 4), dtype=bool)
    for r in range(16):
        for g in range(16):
            keep[r, g, rng.choice(4, size=2, replace=False)] = True
    conf = np.where(keep.reshape(16, 64), bits, 0).astype(np.uint16)
    f = O.Format(1, 1, 0)
    np.testing.assert_array_equal(O.prune(conf, f), conf)
    np.testing.assert_array_equal(O.decompress(*O.compress(conf, f), 16, 64, f), conf)


def test_planted_mistakes_are_caught():
    """The brute force separates the plausible wrong variants: ties to the higher
    position, 2:4 before the Sub-Row choice, index counted from the wrong end."""
    rng = np.random.default_rng(5)
    bits = random_bf16(rng, (8, 32), "ties")
    ref = brute_prune(bits, 1, 1, 0)
    w = O.bf16_bits_to_f64(bits).reshape(8, 8, 4)
    order = np.argsort(-np.abs(w[..., ::-1]), axis=-1, kind="stable")      # ties to the HIGHER position
    pos = 3 - order[..., :2]
    m = np.zeros((8, 8, 4), dtype=bool)
    np.put_along_axis(m, pos, True, axis=-1)
    wrong = np.where(m.reshape(8, 32), bits, 0)
    assert not np.array_equal(wrong, ref)
    # Sub-Row choice after 2:4 would see other scores: row 0 = [3 3 0 0 0 0 0 0] (18 either way),
    # row 1 = eight 2s (32 unpruned, 16 once 2:4 has halved it) -> the paper's order keeps row 1.
    three, two = 0x4040, 0x4000
    bits2 = np.array([[three, three, 0, 0, 0, 0, 0, 0], [two] * 8], dtype=np.uint16)
    ref2 = brute_prune(bits2, 1, 2, 8)
    assert ref2[0].max() == 0 and (ref2[1] != 0).sum() == 4
    np.testing.assert_array_equal(O.prune(bits2, O.Format(1, 2, 8)), ref2)
    wrong2 = brute_prune(brute_prune(bits2, 1, 1, 0), 1, 2, 8)
    assert not np.array_equal(wrong2, ref2)


def test_bad_shapes_raise():
    with pytest.raises(ValueError):
        O.prune(np.zeros((4, 6), dtype=np.uint16), O.Format())
    with pytest.raises(ValueError):
        O.prune(np.zeros((3, 16), dtype=np.uint16), O.Format(1, 2, 8))
    with pytest.raises(ValueError):
        O.prune(np.zeros((4, 12), dtype=np.uint16), O.Format(1, 2, 8))
    with pytest.raises(ValueError):
        O.Format(2, 1, 8)


def test_bf16_helpers():
    assert O.bf16_bits_to_f64(np.array([0x3F80, 0xC040, 0x8000], dtype=np.uint16)).tolist() == [1.0, -3.0, -0.0]
    # round-to-nearest-even: 1 + 2^-8 is a tie between 1.0 (even) and 1.0078125
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -12, 1.0078125 + 2.0 ** -8, -2.5])
    assert O.f64_to_bf16_bits(x).tolist() == [0x3F80, 0x3F81, 0x3F82, 0xC020]

"""GPU parity: prune + encode, decode and the kernel-ready re-ordering against the
oracle, bit for bit (section 4.1 format)."""
import numpy as np
import pytest
import torch

from oracle import ssmm_oracle as O
from paper_2503_10725_amd import binding as B
from paper_2503_10725_amd import synth

pytestmark = pytest.mark.gpu


def random_bits(rng, shape, kind):
    if kind == "normal":
        f = rng.standard_normal(shape).astype(np.float32) * 0.02
    else:   # many exact ties, zeros and negative zeros
        f = rng.choice(np.array([0.0, -0.0, 0.5, -0.5, 1.0, -1.0, 2.0], dtype=np.float32), size=shape)
    bits = (f.view(np.uint32) >> 16).astype(np.uint16)
    if kind == "non-finite":   # NaNs (several payloads, both signs) and infinities among the ties: a NaN ranks like an infinity
        mask = rng.random(shape) < 0.05
        bits[mask] = rng.choice(np.array([0x7FC0, 0xFFC0, 0x7FA1, 0x7F80, 0xFF80], dtype=np.uint16), size=int(mask.sum()))
    return bits


CASES = [
    # E, rows, K, fmt
    (3, 64, 128, (1, 1, 0)),
    (2, 96, 320, (1, 1, 0)),        # several row tiles and k blocks
    (1, 6, 20, (1, 1, 0)),          # not tileable, partial metadata word
    (2, 64, 128, (1, 2, 8)),          # tileable vector-wise case: 32 stored rows
    (2, 256, 320, (1, 2, 8)),         # several stored row tiles, odd number of 64-element stages
    (1, 96, 128, (1, 2, 8)),          # 48 stored rows: not tileable
    (2, 128, 256, (1, 2, 16)),        # Sub-Rows of 16 and 32 elements (formats of the paper's Table 4) and 64: tileable
    (2, 128, 320, (1, 2, 32)),
    (1, 64, 192, (1, 2, 64)),
    (1, 64, 192, (1, 2, 24)),         # a Sub-Row straddles k blocks
    (2, 32, 96, (4, 8, 32)),
    (2, 128, 256, (4, 8, 32)),        # gathered formats of the paper's Table 4 at tileable shapes: a source byte per dense row and k block
    (1, 256, 128, (8, 16, 32)),
    (1, 64, 128, (2, 4, 64)),
    (2, 128, 192, (1, 4, 32)),
    (1, 48, 72, (2, 3, 12)),        # V not a power of two, partial words
    (1, 512, 32, (8, 16, 32)),
    (2, 1024, 512, (1, 1, 0)),      # the tiny layer's gate shape
]


@pytest.mark.parametrize("E,rows,K,fmt", CASES)
@pytest.mark.parametrize("kind", ["normal", "ties", "non-finite"])
def test_compress_decompress_untile_bit_exact(E, rows, K, fmt, kind):
    print(f"case E={E} rows={rows} K={K} fmt={fmt} kind={kind}", flush=True)
    rng = np.random.default_rng(E * 1000 + rows + K + len(kind))
    bits = random_bits(rng, (E, rows, K), kind)
    w = synth.from_bits(bits, "cuda")
    ofmt = O.Format(*fmt)
    tileable = B.compressed_sizes(rows, K, fmt)[3] > 0
    enc = B.compress_weights(w, fmt, canonical=True, tiled=tileable)
    torch.cuda.synchronize()
    for e in range(E):
        v, m, i = O.compress(bits[e], ofmt)
        assert np.array_equal(synth.bits(enc["values"][e]), v)
        assert np.array_equal(enc["meta"][e].cpu().numpy().view(np.uint32), m)
        if ofmt.vectorwise:
            assert np.array_equal(enc["index"][e].cpu().numpy(), i)
    dense = B.decompress_weights(enc["values"], enc["meta"], enc["index"], rows, K, fmt)
    torch.cuda.synchronize()
    for e in range(E):
        assert np.array_equal(synth.bits(dense[e]), O.prune(bits[e], ofmt))
    if tileable:
        v2, m2, i2 = B.untile_weights(enc["tiled"], E, rows, K, fmt)
        torch.cuda.synchronize()
        assert torch.equal(v2.view(torch.int16), enc["values"].view(torch.int16))
        assert torch.equal(m2, enc["meta"])
        if ofmt.vectorwise:
            assert torch.equal(i2, enc["index"])
        # tiled-only call writes the same kernel-ready bytes
        only = B.compress_weights(w, fmt, canonical=False, tiled=True)["tiled"]
        torch.cuda.synchronize()
        assert torch.equal(only, enc["tiled"])


@pytest.mark.parametrize("E,rows,K,fmt", [(2, 128, 256, (4, 8, 32)), (1, 256, 128, (8, 16, 32)), (1, 64, 128, (2, 4, 64)),
                                          (2, 128, 192, (1, 4, 32))])
@pytest.mark.parametrize("kind", ["normal", "ties"])
def test_expanded_gathered_weights_decode_to_the_pruned_matrix(E, rows, K, fmt, kind):
    """Gathered kernel-ready form -> plain 2:4 kernel-ready form: read back as plain 2:4 (untile,
    decode) it must be the oracle's pruned dense matrix, bit for bit."""
    rng = np.random.default_rng(E * 77 + rows + K)
    bits = random_bits(rng, (E, rows, K), kind)
    tiled = B.compress_weights(synth.from_bits(bits, "cuda"), fmt, canonical=False, tiled=True)["tiled"]
    plain = B.expand_tiled_weights(tiled, E, rows, K, fmt)
    assert plain.numel() == E * B.compressed_sizes(rows, K, (1, 1, 0))[3]
    v, m, _ = B.untile_weights(plain, E, rows, K, (1, 1, 0))
    dense = B.decompress_weights(v, m, None, rows, K, (1, 1, 0))
    torch.cuda.synchronize()
    for e in range(E):
        assert np.array_equal(synth.bits(dense[e]), O.prune(bits[e], O.Format(*fmt)))


def test_expand_rejects_formats_without_a_gathered_form():
    buf = torch.zeros((1 << 16,), dtype=torch.uint8, device="cuda")
    for fmt in [(1, 1, 0), (1, 2, 8), (2, 3, 12)]:
        with pytest.raises(RuntimeError):
            B.expand_tiled_weights(buf, 1, 96, 192, fmt)
    with pytest.raises(RuntimeError):
        B.expand_tiled_weights(buf, 1, 48, 128, (4, 8, 32))     # rows not a multiple of 32


def test_tiling_is_a_permutation_of_the_canonical_bytes():
    rng = np.random.default_rng(0)
    bits = random_bits(rng, (1, 64, 128), "normal")
    enc = B.compress_weights(synth.from_bits(bits, "cuda"), (1, 1, 0))
    torch.cuda.synchronize()
    n_val = enc["values"].numel()
    tv = enc["tiled"][: n_val * 2].view(torch.int16).cpu().numpy()
    assert sorted(tv.tolist()) == sorted(enc["values"].view(torch.int16).cpu().numpy().reshape(-1).tolist())


def test_empty_expert_list_is_a_no_op():
    w = torch.empty((0, 64, 128), dtype=torch.bfloat16, device="cuda")
    enc = B.compress_weights(w, (1, 1, 0))
    assert enc["values"].shape[0] == 0

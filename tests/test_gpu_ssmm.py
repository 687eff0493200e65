"""GPU parity: the stand-alone sparse-sparse matrix multiplication C = A x B[:, SEL] against the
oracle's definition on the same seeded inputs.  Bar: relative Frobenius error <= 5e-3 (bf16 inputs,
fp32 accumulation, one bf16 rounding of the result)."""
import numpy as np
import pytest
import torch

from oracle import ssmm_oracle as O
from paper_2503_10725_amd import binding as B
from paper_2503_10725_amd import synth

import gpu_common as G

pytestmark = pytest.mark.gpu


def run_case(rows, K, fmt, n_b, n, seed, identity=False):
    print(f"case rows={rows} K={K} fmt={fmt} n_b={n_b} n={n} identity={identity}", flush=True)
    g = torch.Generator(device="cuda").manual_seed(seed)
    a = (torch.randn((1, rows, K), generator=g, device="cuda") * 0.05).to(torch.bfloat16)
    b = torch.randn((n_b, K), generator=g, device="cuda").to(torch.bfloat16)
    sel = None if identity else torch.randint(0, n_b, (n,), generator=g, device="cuda", dtype=torch.int32)
    tiled = B.compress_weights(a, fmt, canonical=True, tiled=True)["tiled"]
    c = B.matmul(tiled, rows, K, fmt, b, sel=sel, n=n)
    torch.cuda.synchronize()
    ofmt = O.Format(*fmt)
    ref = O.ssmm(O.compress(synth.bits(a[0]), ofmt), rows, K, ofmt, synth.bits(b),
                 None if identity else sel.cpu().numpy())[:n]
    got = G.bf16_tensor_to_f64(c)
    err = G.rel_fro(got, ref)
    print(f"  rel_fro={err:.3e}", flush=True)
    assert got.shape == ref.shape and err <= G.TOL
    return c


CASES = [
    # rows, K, fmt, n_b, n  -- n picks the tile shape: <= 20 -> 32-token tiles, < 192 -> 128, else 160
    (256, 256, (1, 1, 0), 64, 7),
    (256, 256, (1, 1, 0), 300, 150),
    (512, 320, (1, 1, 0), 900, 700),        # odd number of stages, ragged token tiles
    (96, 128, (1, 1, 0), 400, 333),         # row tiles that do not fill a block
    (1024, 1024, (1, 1, 0), 2048, 2048),
    (256, 256, (1, 2, 8), 64, 19),
    (512, 384, (1, 2, 8), 500, 100),
    (512, 256, (1, 2, 32), 1000, 640),
    (512, 256, (4, 8, 32), 1000, 640),      # gathered formats
    (256, 384, (8, 16, 32), 300, 90),
    (128, 128, (1, 4, 64), 64, 11),
    # few tiles and a long reduction: the reduction is cut into slices (fp32 partial sums, fixed order) --
    # 2 slices at the 32-token shape, 4 at the 128-token one, 3 ragged ones (9 + 9 + 7 stages) at the 160-token one
    (256, 1024, (1, 1, 0), 64, 7),
    (256, 2048, (1, 1, 0), 300, 150),
    (512, 1600, (1, 1, 0), 900, 700),
    (256, 1024, (1, 2, 8), 64, 19),
    (512, 1536, (1, 2, 8), 500, 100),
]


@pytest.mark.parametrize("rows,K,fmt,n_b,n", CASES)
def test_matmul_matches_oracle(rows, K, fmt, n_b, n):
    run_case(rows, K, fmt, n_b, n, seed=rows + K + n)


def test_split_reduction_differs_from_the_unsplit_one_only_by_rounding(monkeypatch, tuning_library):
    g = torch.Generator(device="cuda").manual_seed(11)
    rows, K, n = 512, 4096, 300
    a = (torch.randn((1, rows, K), generator=g, device="cuda") * 0.05).to(torch.bfloat16)
    b = torch.randn((n, K), generator=g, device="cuda").to(torch.bfloat16)
    tiled = B.compress_weights(a, (1, 1, 0), canonical=False, tiled=True)["tiled"]
    assert B.lib().ssmm_matmul_workspace_bytes(rows, K, n, B.Format(1, 1, 0)) > 256      # this shape splits
    split = G.bf16_tensor_to_f64(B.matmul(tiled, rows, K, (1, 1, 0), b))
    monkeypatch.setenv("SSMM_MATMUL_SPLITS", "1")
    whole = G.bf16_tensor_to_f64(B.matmul(tiled, rows, K, (1, 1, 0), b))
    torch.cuda.synchronize()
    d = G.rel_fro(split, whole)
    print(f"  split vs unsplit rel_fro={d:.3e}", flush=True)
    assert d <= 2.5e-3          # fp32 summation order, then one bf16 rounding on both sides


def test_identity_selection_and_repeatability():
    c1 = run_case(256, 512, (1, 1, 0), 500, 420, seed=3, identity=True)
    c2 = run_case(256, 512, (1, 1, 0), 500, 420, seed=3, identity=True)
    assert torch.equal(c1.view(torch.int16), c2.view(torch.int16))


def test_selected_columns_equal_columns_of_the_full_product():
    """Section 4.1: selecting columns of B commutes with the product."""
    rows, K, n_b = 256, 256, 384
    g = torch.Generator(device="cuda").manual_seed(5)
    a = (torch.randn((1, rows, K), generator=g, device="cuda") * 0.05).to(torch.bfloat16)
    b = torch.randn((n_b, K), generator=g, device="cuda").to(torch.bfloat16)
    tiled = B.compress_weights(a, (1, 1, 0), canonical=False, tiled=True)["tiled"]
    full = B.matmul(tiled, rows, K, (1, 1, 0), b)
    sel = torch.randperm(n_b, generator=g, device="cuda").to(torch.int32)[:200]
    part = B.matmul(tiled, rows, K, (1, 1, 0), b, sel=sel)
    torch.cuda.synchronize()
    # same token row, same weights, same reduction order: identical bits whatever tile it lands in
    assert torch.equal(part.view(torch.int16), full[sel.long()].view(torch.int16))


def test_no_columns_selected():
    a = torch.zeros((1, 64, 128), dtype=torch.bfloat16, device="cuda")
    tiled = B.compress_weights(a, (1, 1, 0), canonical=False, tiled=True)["tiled"]
    b = torch.zeros((4, 128), dtype=torch.bfloat16, device="cuda")
    c = B.matmul(tiled, 64, 128, (1, 1, 0), b, sel=torch.empty((0,), dtype=torch.int32, device="cuda"))
    assert c.shape == (0, 64)


def test_mfma_probe_runs_and_reports_plausible_rates():
    """The measurement aid bench.py loads (libssmm_probe.so, not part of the library): back-to-back
    MFMAs cannot beat their pass counts at 2.4 GHz -- 13.3 ns for the 32x32x32 sparse and the 32x32x16
    dense instruction, 6.7 ns for the 16x16x64 sparse one."""
    import ctypes
    import os
    import sys
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    import bench
    lib = bench.probe_library()
    nbytes = int(lib.ssmm_probe_operand_bytes())
    buf = torch.zeros((nbytes,), dtype=torch.uint8, device="cuda")
    sink = torch.zeros((1,), dtype=torch.float32, device="cuda")
    iters = 2000

    def run(b, idle, kind):
        ms = ctypes.c_float(0.0)
        st = lib.ssmm_probe_mfma(ctypes.c_void_p(b.data_ptr()), b.numel(), iters, idle, kind, ctypes.c_void_p(sink.data_ptr()),
                                 ctypes.byref(ms), None)
        return st, ms.value * 1e6 / (iters * 8)

    for kind, floor in ((0, 13.0), (1, 6.5), (2, 13.0)):
        st, ns = run(buf, 0, kind)
        st2, ns_idle = run(buf, 4, kind)
        print(f"kind {kind}: {ns:.2f} ns per MFMA back to back, {ns_idle:.2f} with 32 idle cycles", flush=True)
        assert st == 0 and st2 == 0
        assert floor < ns < 40.0
        assert ns_idle > ns
    assert run(buf[:64], 0, 0)[0] == -3
    assert run(buf, 3, 0)[0] == -1
    assert run(buf, 0, 5)[0] == -1


def test_hbm_probe_reads_no_faster_than_the_memory_can():
    """The other measurement aid of libssmm_probe.so: a streaming read of 1 GiB (four times the memory-side
    cache) cannot beat the published 8 TB/s, and with eight blocks per compute unit and eight loads in flight
    it reaches a good part of it; bad arguments are refused."""
    import ctypes
    import os
    import sys
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    import bench
    lib = bench.probe_library()
    nbytes = 1 << 30
    buf = torch.empty((nbytes,), dtype=torch.uint8, device="cuda")
    buf.view(torch.int32).random_()
    sink = torch.zeros((4,), dtype=torch.int32, device="cuda")

    def run(n, blocks, in_flight):
        ms = ctypes.c_float(0.0)
        st = lib.ssmm_probe_hbm_read(ctypes.c_void_p(buf.data_ptr()), n, blocks, in_flight, ctypes.c_void_p(sink.data_ptr()),
                                     ctypes.byref(ms), None)
        return st, (n / ms.value * 1e-6 if ms.value > 0 else 0.0)

    st, gbs = run(nbytes, 8, 8)
    print(f"streaming read: {gbs:.0f} GB/s", flush=True)
    assert st == 0 and 2000.0 < gbs < 8000.0
    assert not sink.bool().any()
    assert run(nbytes, 0, 8)[0] == -1 and run(nbytes, 8, 3)[0] == -1 and run(1000, 8, 8)[0] == -1

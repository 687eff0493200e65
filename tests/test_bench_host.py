"""Host-side parts of bench.py that need no GPU: the byte and FLOP accounting of the roofline objects, the
parsers of the committed counter / probe summaries, and the refusal of more than one GPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
from paper_2503_10725_amd import synth  # noqa: E402


def test_bytes_per_weight_follow_the_encoding():
    # 2:4: half the values (1 byte per dense element) + 2 bits per kept value (1/8 byte per dense element)
    assert bench.bytes_per_weight((1, 1, 0)) == pytest.approx(1.125)
    # (1,2,V) on top: half the rows stored, plus the kernel-ready source-row bits, 1/32 byte per dense element
    assert bench.bytes_per_weight((1, 2, 8)) == pytest.approx(0.5 * 1.125 + 1.0 / 32)


def test_kernel_bytes_of_the_headline_layer():
    cfg = synth.CONFIGS["mixtral"].with_tokens(4096)
    gu, dn, cb = bench.kernel_bytes(cfg, cfg.E_total)
    H, F, E, P, T = cfg.H, cfg.F, cfg.E_total, cfg.pairs, cfg.T
    assert gu == pytest.approx(2 * E * H * F * 1.125 + P * (2 * H + 2 * F))
    assert dn == pytest.approx(E * H * F * 1.125 + P * (2 * F + 2 * H))
    assert cb == pytest.approx(P * 2 * H + 2 * T * H)
    w, a = bench.algorithmic_bytes(cfg, cfg.E_total)
    assert w == pytest.approx(3 * E * H * F * 1.125)


def test_committed_summaries_parse():
    share = bench.sustained_mfma_share()
    assert share is not None and 0.5 < share < 0.9          # random operands: well below the published peak
    hbm = bench.sustained_hbm_share()
    assert hbm is not None and 0.6 < hbm < 1.0
    for kernel in ("gate_up", "down"):
        for config, tokens in (("mixtral", 4096), ("mixtral", 16), ("qwen", 2048), ("deepseek", 8192), ("mixtral75", 4096)):
            t = bench.measured_traffic(kernel, tokens, config)
            assert t is not None and t > 1e6
    assert bench.measured_traffic("gate_up", 12345, "mixtral") is None


def test_more_than_one_gpu_is_refused():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode == 2 and "ONE GPU" in res.stderr

"""GPU parity: the expert-FFN path (route -> bucket -> SSMM gate/up + SiLU -> SSMM down
-> combine) against the fp64 oracle on the same seeded inputs.  Bar: relative
Frobenius error <= 5e-3 over the whole [T][H] output; integers bit-exact."""
import numpy as np
import pytest
import torch

from paper_2503_10725_amd import binding as B
from paper_2503_10725_amd import synth
from paper_2503_10725_amd.synth import LayerConfig

import gpu_common as G

pytestmark = pytest.mark.gpu


def run_case(cfg, std=0.02, mutate=None):
    print(f"case {cfg}", flush=True)
    x, lg, wg, wu, wd = G.make_inputs(cfg, std=std)
    if mutate:
        x, lg, wg, wu, wd = mutate(x, lg, wg, wu, wd)
    y, route = G.run_gpu_layer(cfg, x, lg, wg, wu, wd)
    ref = G.run_oracle_layer(cfg, x, lg, wg, wu, wd)
    G.check_routing(route, ref, cfg)
    got = G.bf16_tensor_to_f64(y)
    err = G.rel_fro(got, ref["y"])
    print(f"  rel_fro={err:.3e}", flush=True)
    assert err <= G.TOL, err
    return got, ref, err


SMALL = [
    # tile-shape selector: mean bucket <= 20 -> 32-token tiles, two waves per SIMD
    LayerConfig("tiny", T=128, H=512, F=1024, E=8, topk=2, seed=1),
    LayerConfig("few_tokens", T=16, H=256, F=384, E=8, topk=2, logits="uniform", seed=11),
    LayerConfig("one_token", T=1, H=128, F=128, E=4, topk=2, seed=12),
    # 20 < mean < 192 -> 128-token tiles, few rows per block, ragged tails (tiny: split down projection)
    LayerConfig("mid", T=300, H=256, F=448, E=4, topk=1, seed=13),
    LayerConfig("mid_shared", T=150, H=192, F=320, E=6, topk=2, S=2, renormalize=False, seed=14),
    # mean >= 192 -> 128-token (gate/up) and 160-token (down) tiles, 256 / 512 rows per block
    LayerConfig("big", T=1100, H=256, F=384, E=4, topk=2, seed=15),
    LayerConfig("big_skewed", T=900, H=128, F=256, E=8, topk=3, logits="biased", renormalize=False, seed=16),
    # row-tile counts that do not fill the block's row tile (F=192: 6 tiles, H=320: 10) and an
    # odd number of pipeline stages (K=320: 5), under each of the three tile shapes
    LayerConfig("odd_rows_mid", T=260, H=320, F=192, E=2, topk=1, seed=17),
    LayerConfig("odd_rows_big", T=600, H=320, F=192, E=2, topk=1, seed=18),
    LayerConfig("odd_rows_small", T=40, H=320, F=192, E=2, topk=1, seed=19),
    # buckets that fit one 160-token tile but not one 128-token tile: the down projection takes the 160-token tile
    LayerConfig("odd_rows_mid160", T=270, H=320, F=192, E=2, topk=1, seed=20),
    LayerConfig("mid160", T=450, H=512, F=1024, E=8, topk=2, seed=26),
    # (1,2,8) vector-wise pruning stacked on 2:4 (75 % sparse weights), under each tile shape
    LayerConfig("vec_tiny", T=128, H=512, F=1024, E=8, topk=2, fmt=(1, 2, 8), seed=31),
    LayerConfig("vec_mid", T=300, H=256, F=448, E=4, topk=1, fmt=(1, 2, 8), seed=32),
    LayerConfig("vec_big_shared", T=700, H=256, F=384, E=4, topk=2, S=1, fmt=(1, 2, 8), renormalize=False, seed=33),
    LayerConfig("vec_odd_rows", T=260, H=320, F=192, E=2, topk=1, fmt=(1, 2, 8), seed=34),
    LayerConfig("vec_odd_rows_big", T=600, H=320, F=192, E=2, topk=1, fmt=(1, 2, 8), seed=35),
    # longer Sub-Rows of the same 1-of-2 scheme: (1,2,16) and (1,2,32) of the paper's Table 4, and one that straddles k blocks
    LayerConfig("vec16_mid", T=300, H=256, F=448, E=4, topk=1, fmt=(1, 2, 16), seed=36),
    LayerConfig("vec32_big", T=700, H=256, F=384, E=4, topk=2, fmt=(1, 2, 32), seed=37),
    LayerConfig("vec24_tiny", T=30, H=192, F=384, E=4, topk=2, fmt=(1, 2, 24), seed=38),
    # gathered formats ((4,8,32) and (8,16,32) of the paper's Table 4, and others with M / N a power of two),
    # under each tile shape, with row-tile counts that do not fill a block and an odd number of stages
    LayerConfig("gen48_mid", T=300, H=256, F=512, E=4, topk=1, fmt=(4, 8, 32), seed=61),
    LayerConfig("gen816_big", T=700, H=256, F=384, E=4, topk=2, S=1, fmt=(8, 16, 32), renormalize=False, seed=62),
    LayerConfig("gen24_tiny", T=30, H=256, F=384, E=4, topk=2, fmt=(2, 4, 64), seed=63),
    # 192 to 255 pairs per expert: the 128-token gathering kernels (from 256 on the layer expands the weights instead)
    LayerConfig("gen48_big_gathering", T=440, H=256, F=384, E=4, topk=2, fmt=(4, 8, 32), seed=66),
    LayerConfig("gen14_odd_rows", T=600, H=384, F=256, E=2, topk=1, fmt=(1, 4, 32), seed=64),
    LayerConfig("gen48_odd_rows_mid", T=260, H=320, F=192, E=2, topk=1, fmt=(4, 8, 32), seed=65),
    # more tiles than resident blocks (256): every block multiplies several tiles in turn, in both
    # projections (gate/up 4 row tiles x ~95 token tiles, down 4 x ~76), plain and vector-wise
    LayerConfig("loop_big", T=6000, H=2048, F=1024, E=4, topk=2, seed=51),
    LayerConfig("loop_vec", T=6000, H=2048, F=1024, E=4, topk=2, fmt=(1, 2, 8), seed=52),
    # more buckets than lanes in a wavefront (the tile look-up takes two rounds), some of them
    # empty, shared experts, small and large buckets, blocks that take several tiles
    LayerConfig("many_experts", T=2000, H=256, F=256, E=70, topk=2, logits="biased", seed=53),
    LayerConfig("many_experts_big", T=9000, H=256, F=512, E=68, topk=2, S=2, logits="biased", renormalize=False, seed=54),
]


@pytest.mark.parametrize("cfg", SMALL, ids=lambda c: c.name)
def test_layer_matches_oracle(cfg):
    run_case(cfg)


def test_error_is_rounding_not_a_bug():
    """Against the oracle variant that rounds h to bf16 like the kernel stores it, the
    distance must shrink: what is left is the bf16 rounding of yp and y."""
    cfg = LayerConfig("diag", T=256, H=512, F=1024, E=8, topk=2, seed=21)
    x, lg, wg, wu, wd = G.make_inputs(cfg)
    y, _ = G.run_gpu_layer(cfg, x, lg, wg, wu, wd)
    got = G.bf16_tensor_to_f64(y)
    plain = G.rel_fro(got, G.run_oracle_layer(cfg, x, lg, wg, wu, wd)["y"])
    rounded = G.rel_fro(got, G.run_oracle_layer(cfg, x, lg, wg, wu, wd, round_h=True)["y"])
    print(f"  plain={plain:.3e} rounded_h={rounded:.3e}", flush=True)
    assert rounded < plain <= G.TOL
    assert rounded < 3.5e-3


def test_empty_experts_and_everything_on_one_expert():
    cfg = LayerConfig("hot", T=400, H=128, F=192, E=8, topk=2, seed=22)

    def mutate(x, lg, wg, wu, wd):
        lg = lg.clone()
        lg[:, 2] += 50.0      # every token picks expert 2 first
        lg[:, 6] -= 50.0      # expert 6 stays empty
        return x, lg, wg, wu, wd

    _, ref, _ = run_case(cfg, mutate=mutate)
    off = ref["offsets"]
    assert off[3] - off[2] == cfg.T and off[7] - off[6] == 0


def test_zero_gate_gives_exact_zero_and_identical_experts_ignore_routing():
    cfg = LayerConfig("props", T=200, H=128, F=256, E=4, topk=2, seed=23)
    x, lg, wg, wu, wd = G.make_inputs(cfg)
    y, _ = G.run_gpu_layer(cfg, x, lg, torch.zeros_like(wg), wu, wd)
    assert not y.view(torch.int16).bool().any()          # silu(0) * u = 0, exactly
    wg[:], wu[:], wd[:] = wg[0].clone(), wu[0].clone(), wd[0].clone()
    y1, _ = G.run_gpu_layer(cfg, x, lg, wg, wu, wd)
    y2, _ = G.run_gpu_layer(cfg, x, torch.flip(lg, dims=[1]), wg, wu, wd)   # other routing, same experts
    a, b = G.bf16_tensor_to_f64(y1), G.bf16_tensor_to_f64(y2)
    assert G.rel_fro(a, b) <= G.TOL


def test_unpruned_weights_through_the_pair_embedding_equal_a_dense_ffn():
    """k = E, weights embedded as (a, b, 0, 0) per pair so 2:4 removes nothing: the layer
    must equal sum_e softmax_e * FFN_e(x) computed densely by torch in fp64 on the CPU."""
    H, F, E, T = 128, 128, 4, 96
    cfg = LayerConfig("dense", T=T, H=2 * H, F=2 * F, E=E, topk=E, seed=24)
    g = torch.Generator().manual_seed(5)
    x = torch.randn((T, H), generator=g).to(torch.bfloat16)
    lg = torch.randn((T, E), generator=g)
    wg = (torch.randn((E, F, H), generator=g) * 0.05).to(torch.bfloat16)
    wu = (torch.randn((E, F, H), generator=g) * 0.05).to(torch.bfloat16)
    wd = (torch.randn((E, H, F), generator=g) * 0.05).to(torch.bfloat16)

    def embed_k(w):      # [.., R, K] -> [.., R, 2K]
        out = torch.zeros(w.shape[:-1] + (w.shape[-1] // 2, 4), dtype=w.dtype)
        out[..., :2] = w.reshape(w.shape[:-1] + (w.shape[-1] // 2, 2))
        return out.reshape(w.shape[:-1] + (2 * w.shape[-1],))

    def embed_rows(w):   # [E, R, K] -> [E, 2R, K], rows interleaved like the reduction of the consumer
        return embed_k(w.transpose(1, 2)).transpose(1, 2).contiguous()

    xe = embed_k(x)
    wge, wue = embed_rows(embed_k(wg)), embed_rows(embed_k(wu))       # [E][2F][2H]
    wde = torch.zeros((E, 2 * H, 2 * F), dtype=torch.bfloat16)
    wde[:, :H] = embed_k(wd)
    dev = [t.cuda().contiguous() for t in (xe, lg, wge, wue, wde)]
    y, _ = G.run_gpu_layer(cfg, *dev)
    got = G.bf16_tensor_to_f64(y)[:, :H]
    p = torch.softmax(lg.double(), dim=1)
    ref = torch.zeros((T, H), dtype=torch.float64)
    for e in range(E):
        gg, uu = x.double() @ wg[e].double().T, x.double() @ wu[e].double().T
        ref += p[:, e:e + 1] * ((torch.nn.functional.silu(gg) * uu) @ wd[e].double().T)
    err = G.rel_fro(got, ref.numpy())
    print(f"  rel_fro={err:.3e}", flush=True)
    assert err <= G.TOL


@pytest.mark.parametrize("fmt", [(1, 1, 0), (1, 2, 8)], ids=["2:4", "1:2:8"])
@pytest.mark.parametrize("T", [24, 200, 240], ids=["32-token-tiles", "128-token-tiles", "160-token-tiles"])
def test_split_down_projection(monkeypatch, tuning_library, fmt, T):
    """Small buckets split the reduction of the down projection into fp32 partial sums.  Every
    number of splits (also one that leaves a ragged last slice: 24 stages in 5 slices) must meet
    the oracle, and the result may differ between split counts only by fp32 summation order."""
    cfg = LayerConfig("split", T=T, H=256, F=1536, E=4, topk=2, fmt=fmt, seed=41)
    x, lg, wg, wu, wd = G.make_inputs(cfg)
    ref = G.run_oracle_layer(cfg, x, lg, wg, wu, wd)["y"]
    outs = []
    for splits in (1, 2, 3, 5, 8):
        monkeypatch.setenv("SSMM_DOWN_SPLITS", str(splits))
        y, _ = G.run_gpu_layer(cfg, x, lg, wg, wu, wd)
        got = G.bf16_tensor_to_f64(y)
        err = G.rel_fro(got, ref)
        print(f"  splits={splits} rel_fro={err:.3e}", flush=True)
        assert err <= G.TOL
        outs.append(got)
    for o in outs[2:]:
        assert G.rel_fro(o, outs[1]) <= 5e-4     # fp32 summation order, then the same bf16 rounding of y
    assert G.rel_fro(outs[1], outs[0]) <= G.TOL  # unsplit rounds yp to bf16 on the way, split does not


@pytest.mark.parametrize("H,F", [(512, 1536), (320, 1600)], ids=["3x8-stages", "ragged-slices-odd-rows"])
def test_split_down_projection_of_few_large_buckets(monkeypatch, tuning_library, H, F):
    """Large buckets, but few blocks: the 512-row x 160-token down tile splits its reduction into
    up to four slices of at least eight stages (24 stages: 3 slices of 8; 25 stages: 9 + 9 + 7).  Split
    and unsplit must both meet the oracle and differ only by summation order and one bf16 rounding."""
    cfg = LayerConfig("tall_split", T=600, H=H, F=F, E=4, topk=2, seed=43)
    x, lg, wg, wu, wd = G.make_inputs(cfg)
    ref = G.run_oracle_layer(cfg, x, lg, wg, wu, wd)["y"]
    outs = []
    for knob in (None, "0"):
        if knob is not None:
            monkeypatch.setenv("SSMM_DOWN_TALLSPLIT", knob)
        y, _ = G.run_gpu_layer(cfg, x, lg, wg, wu, wd)
        got = G.bf16_tensor_to_f64(y)
        err = G.rel_fro(got, ref)
        print(f"  split={'default' if knob is None else 'off'} rel_fro={err:.3e}", flush=True)
        assert err <= G.TOL
        outs.append(got)
    d = G.rel_fro(outs[0], outs[1])
    assert 0 < d <= G.TOL      # not the same code path, and no further apart than rounding


def test_pre_expanded_gathered_weights_give_the_layer_bit_for_bit():
    """Large buckets: the layer expands gathered weights to plain 2:4 operands in its workspace on
    every call; weights expanded once beforehand and passed as plain 2:4 must give the same bits."""
    cfg = LayerConfig("gen_pre", T=700, H=256, F=384, E=4, topk=2, S=1, fmt=(8, 16, 32), renormalize=False, seed=62)
    x, lg, wg, wu, wd = G.make_inputs(cfg)
    y, route = G.run_gpu_layer(cfg, x, lg, wg, wu, wd)
    ref = G.run_oracle_layer(cfg, x, lg, wg, wu, wd)
    assert G.rel_fro(G.bf16_tensor_to_f64(y), ref["y"]) <= G.TOL
    shapes = [(cfg.F, cfg.H), (cfg.F, cfg.H), (cfg.H, cfg.F)]
    enc = [B.compress_weights(w, cfg.fmt, canonical=False, tiled=True)["tiled"] for w in (wg, wu, wd)]
    pre = [B.expand_tiled_weights(t, cfg.E_total, r, k, cfg.fmt) for t, (r, k) in zip(enc, shapes)]
    y2 = B.expert_ffn(x, cfg.F, (1, 1, 0), pre[0], pre[1], pre[2], route)
    torch.cuda.synchronize()
    assert torch.equal(y2.view(torch.int16), y.view(torch.int16))


def test_repeat_runs_are_bit_identical():
    for T, F in ((500, 256), (2000, 256), (20, 1024)):     # mid-size, large, tiny buckets (split reduction)
        cfg = LayerConfig("det", T=T, H=256, F=F, E=8, topk=2, seed=25)
        x, lg, wg, wu, wd = G.make_inputs(cfg)
        y1, _ = G.run_gpu_layer(cfg, x, lg, wg, wu, wd)
        y2, _ = G.run_gpu_layer(cfg, x, lg, wg, wu, wd)
        assert torch.equal(y1.view(torch.int16), y2.view(torch.int16))


# ---- layer variants: other activation functions, experts without a gate ----------------------
VARIANT_SHAPES = [
    LayerConfig("var_small", T=24, H=256, F=384, E=4, topk=2, seed=71),
    LayerConfig("var_mid", T=300, H=256, F=448, E=4, topk=1, S=1, renormalize=False, seed=72),
    LayerConfig("var_big", T=1100, H=320, F=384, E=4, topk=2, seed=73),
    LayerConfig("var_vec", T=700, H=256, F=384, E=4, topk=2, fmt=(1, 2, 8), seed=74),
    LayerConfig("var_gen", T=300, H=256, F=512, E=4, topk=1, fmt=(4, 8, 32), seed=75),
]


@pytest.mark.parametrize("act,gated", [("gelu_tanh", True), ("relu", True), ("silu", False), ("gelu_tanh", False),
                                       ("relu", False)])
@pytest.mark.parametrize("cfg", VARIANT_SHAPES, ids=lambda c: c.name)
def test_layer_variants_match_oracle(cfg, act, gated):
    print(f"case {cfg} activation={act} gated={gated}", flush=True)
    # without the product with `up` the intermediate is larger: weights scaled as usual keep it O(1)
    x, lg, wg, wu, wd = G.make_inputs(cfg)
    y, route = G.run_gpu_layer(cfg, x, lg, wg, wu, wd, activation=act, gated=gated)
    ref = G.run_oracle_layer(cfg, x, lg, wg, wu, wd, act=act, gated=gated)
    G.check_routing(route, ref, cfg)
    err = G.rel_fro(G.bf16_tensor_to_f64(y), ref["y"])
    print(f"  rel_fro={err:.3e}", flush=True)
    assert err <= G.TOL, err
    if not gated or act != "silu":   # and it is not the default layer that ran
        base = G.run_oracle_layer(cfg, x, lg, wg, wu, wd)
        assert G.rel_fro(ref["y"], base["y"]) > 10 * G.TOL


def test_variant_argument_checks():
    cfg = LayerConfig("var_args", T=16, H=128, F=128, E=4, topk=2, seed=76)
    x, lg, wg, wu, wd = G.make_inputs(cfg)
    with pytest.raises(KeyError):
        G.run_gpu_layer(cfg, x, lg, wg, wu, wd, activation="swish")
    lib = B.lib()
    import ctypes
    one = ctypes.c_void_p(256)
    bad = lib.ssmm_expert_ffn_variant(one, 16, 128, 128, 4, B.Format(1, 1, 0), 7, 1, one, one, one, one, one, one, one, 2,
                                      one, one, 1 << 30, None, None)
    assert bad == B.SSMM_EINVAL


# ---- the compiler-scheduled kernels as the fall-back of the usual layer (token matrices of 4 GB and more take them) ----
@pytest.mark.parametrize("name", ["tiny", "mid_shared", "big", "odd_rows_big", "vec_mid", "vec_big_shared", "loop_big"])
def test_fallback_kernels_match_oracle(monkeypatch, tuning_library, name):
    monkeypatch.setenv("SSMM_PIPE", "1")
    run_case(next(c for c in SMALL if c.name == name))


def test_whole_layer_from_hidden_states_with_the_router_in_front():
    """router logits -> route -> bucket -> expert FFN, all on the GPU; the oracle routes on the GPU's
    fp32 logits (the top-k decision is taken in the kernel's precision on both sides) after the
    logits themselves have been checked against its own."""
    from oracle import ssmm_oracle as O
    cfg = LayerConfig("from_hidden", T=500, H=256, F=384, E=16, topk=4, S=1, renormalize=False, seed=81)
    x, _, wg, wu, wd = G.make_inputs(cfg)
    g = torch.Generator(device="cuda").manual_seed(82)
    wr = (torch.randn((cfg.E, cfg.H), generator=g, device="cuda") * 0.1).to(torch.bfloat16)
    lg = B.router_logits(x, wr)
    ref_lg = O.router_logits(synth.bits(x), synth.bits(wr))
    np.testing.assert_allclose(lg.cpu().numpy(), ref_lg, rtol=0, atol=2e-6 * np.sqrt(cfg.H) * np.abs(ref_lg).max())
    y, route = G.run_gpu_layer(cfg, x, lg, wg, wu, wd)
    ref = G.run_oracle_layer(cfg, x, lg, wg, wu, wd)
    G.check_routing(route, ref, cfg)
    err = G.rel_fro(G.bf16_tensor_to_f64(y), ref["y"])
    print(f"  rel_fro={err:.3e}", flush=True)
    assert err <= G.TOL


# ---- a seeded sweep over shapes, formats, routing set-ups and layer variants ---------------------
def _sweep_cases(n, seed):
    rng = np.random.default_rng(seed)
    fmts = [(1, 1, 0), (1, 1, 0), (1, 2, 8), (1, 2, 16), (4, 8, 32), (8, 16, 32), (2, 4, 64), (1, 4, 32)]
    cases = []
    while len(cases) < n:
        fmt = fmts[rng.integers(len(fmts))]
        N, M, V = fmt
        H = int(rng.integers(1, 7)) * 64
        F = int(rng.integers(1, 9)) * 64
        ok = True
        for rows, K in ((F, H), (H, F)):
            rc = rows * N // M if N < M else rows
            ok &= rc % 32 == 0 and rows % 32 == 0 and (N == M or (K % V == 0 and rows % M == 0))
        if not ok:
            continue
        E = int(rng.integers(1, 10))
        topk = int(rng.integers(1, min(E, 4) + 1))
        S = int(rng.integers(0, 3)) if rng.random() < 0.3 else 0
        T = int(rng.choice([1, 7, 33, 130, 400, 900, 1500]))
        act, gated = ("silu", True) if rng.random() < 0.6 else (str(rng.choice(["silu", "gelu_tanh", "relu"])), bool(rng.random() < 0.5))
        logits = str(rng.choice(["normal", "uniform", "biased"]))
        cases.append((LayerConfig(f"sweep{len(cases)}", T=T, H=H, F=F, E=E, topk=topk, S=S, fmt=fmt, logits=logits,
                                  renormalize=bool(rng.random() < 0.5), seed=1000 + len(cases)), act, gated))
    return cases


@pytest.mark.parametrize("cfg,act,gated", _sweep_cases(48, 20250310), ids=lambda v: getattr(v, "name", str(v)))
def test_seeded_sweep_matches_oracle(cfg, act, gated):
    print(f"case {cfg} activation={act} gated={gated}", flush=True)
    x, lg, wg, wu, wd = G.make_inputs(cfg)
    y, route = G.run_gpu_layer(cfg, x, lg, wg, wu, wd, activation=act, gated=gated)
    ref = G.run_oracle_layer(cfg, x, lg, wg, wu, wd, act=act, gated=gated)
    G.check_routing(route, ref, cfg)
    got = G.bf16_tensor_to_f64(y)
    err = G.rel_fro(got, ref["y"])
    worst = (np.linalg.norm(got - ref["y"], axis=1) / np.maximum(np.linalg.norm(ref["y"], axis=1), 1e-30)).max()
    print(f"  rel_fro={err:.3e} worst token={worst:.3e}", flush=True)
    assert err <= G.TOL, err
    assert worst <= 4 * G.TOL, worst


# ---- Sub-Row compute skipping (sections 4.1, 4.3): one MFMA per stored operand into intermediate sums,
# merged into the accumulators of the source rows at the end of every V-wide block ----
SKIP_CASES = [
    LayerConfig("skip32_small", T=20, H=256, F=384, E=4, topk=2, fmt=(1, 2, 32), seed=91),
    LayerConfig("skip32_mid", T=300, H=256, F=448, E=4, topk=1, fmt=(1, 2, 32), seed=92),      # 14 stored row tiles: ragged rows too
    LayerConfig("skip32_big_shared", T=700, H=256, F=384, E=4, topk=2, S=1, fmt=(1, 2, 32), renormalize=False, seed=93),
    LayerConfig("skip64", T=333, H=384, F=512, E=6, topk=2, fmt=(1, 2, 64), seed=94),           # merge every second k block
    LayerConfig("skip128", T=500, H=256, F=640, E=3, topk=2, fmt=(1, 2, 128), seed=95),         # a Sub-Row spans two stages
    LayerConfig("skip96", T=200, H=192, F=384, E=4, topk=2, fmt=(1, 2, 96), seed=96),           # three k blocks: not a power of two
]


@pytest.mark.parametrize("cfg", SKIP_CASES, ids=[c.name for c in SKIP_CASES])
def test_subrow_compute_skipping_matches_oracle(monkeypatch, tuning_library, cfg):
    monkeypatch.setenv("SSMM_SUBROW_SKIP", "1")
    got, ref, err = run_case(cfg)
    monkeypatch.delenv("SSMM_SUBROW_SKIP")
    y, _ = G.run_gpu_layer(cfg, *G.make_inputs(cfg))      # the masked scheme on the same inputs
    d = G.rel_fro(G.bf16_tensor_to_f64(y), got)
    print(f"  skipping vs masked rel_fro={d:.3e}", flush=True)
    assert d <= G.TOL     # same products, another order of the fp32 sums


@pytest.mark.parametrize("fmt", [(1, 1, 0), (1, 2, 8), (4, 8, 32)], ids=["2:4", "1:2:8", "4:8:32"])
def test_extreme_bucket_skew(fmt):
    """One expert with a single token, one with more than a thousand (several full token tiles and a ragged one),
    one with a few dozen, one with none: every tile shape meets every kind of ragged end in one layer (the tile
    rules only see the mean bucket)."""
    cfg = LayerConfig("skew", T=1300, H=256, F=384, E=4, topk=1, fmt=fmt, seed=97)

    def mutate(x, lg, wg, wu, wd):
        lg = torch.full_like(lg, -4.0)
        lg[:, 1] = 4.0                 # nearly everybody goes to expert 1
        lg[0, 0] = 8.0                 # token 0 alone on expert 0
        lg[100:137, 2] = 8.0           # 37 tokens on expert 2, none on expert 3
        return x, lg, wg, wu, wd

    _, ref, _ = run_case(cfg, mutate=mutate)
    counts = np.diff(ref["offsets"])
    assert counts.tolist() == [1, 1300 - 38, 37, 0]


@pytest.mark.parametrize("fmt", [(1, 1, 0), (1, 2, 8), (4, 8, 32)], ids=["2:4", "1:2:8", "4:8:32"])
@pytest.mark.parametrize("T,E", [(40, 200), (1500, 200), (700, 255)])
def test_buckets_span_several_rounds_of_the_tile_table(fmt, T, E):
    """200 or 255 routed experts + 1 shared (256 buckets: the most route + bucket serve): the kernels read the bucket
    offsets 64 at a time, so their tile table takes four rounds, the last one with few buckets or exactly full; at 40
    tokens most buckets are empty, at 1500 the non-empty ones fill more than two rounds."""
    cfg = LayerConfig("wide_table", T=T, H=128, F=128, E=E, topk=4, S=1, fmt=fmt, logits="biased", seed=131 + T)
    _, ref, _ = run_case(cfg)
    counts = np.diff(ref["offsets"])
    assert len(counts) == E + 1 and counts[-1] == T
    if T == 40:
        assert (counts == 0).any()
    elif T == 1500:
        assert (counts > 0).sum() > 128


# ---- the same kind of sweep with many experts: bucket counts on both sides of 64, 128 and 192 (the kernels look at
# ---- 64 buckets at a time), shared experts, from one token to a few thousand ----
def _many_expert_cases(n, seed):
    rng = np.random.default_rng(seed)
    fmts = [(1, 1, 0), (1, 2, 8), (4, 8, 32), (1, 1, 0), (8, 16, 32)]
    cases = []
    for i in range(n):
        E = int(rng.choice([33, 63, 64, 65, 100, 127, 128, 129, 190, 250]))
        topk = int(rng.integers(1, 9))
        cfg = LayerConfig(f"experts{i}", T=int(rng.choice([1, 5, 17, 64, 200, 257, 900, 2500])), H=int(rng.integers(1, 5)) * 128,
                          F=int(rng.integers(1, 5)) * 128, E=E, topk=topk, S=int(rng.integers(0, 3)), fmt=fmts[i % 5],
                          logits=["normal", "biased"][i % 2], renormalize=bool(i % 3), seed=2000 + i)
        act, gated = [("silu", True), ("gelu_tanh", True), ("relu", False), ("silu", True), ("silu", False)][(i // 5) % 5]
        cases.append((cfg, act, gated))
    return cases


@pytest.mark.parametrize("cfg,act,gated", _many_expert_cases(20, 20250311), ids=lambda v: getattr(v, "name", str(v)))
def test_seeded_sweep_with_many_experts_matches_oracle(cfg, act, gated):
    print(f"case {cfg} activation={act} gated={gated}", flush=True)
    x, lg, wg, wu, wd = G.make_inputs(cfg)
    y, route = G.run_gpu_layer(cfg, x, lg, wg, wu, wd, activation=act, gated=gated)
    ref = G.run_oracle_layer(cfg, x, lg, wg, wu, wd, act=act, gated=gated)
    G.check_routing(route, ref, cfg)
    err = G.rel_fro(G.bf16_tensor_to_f64(y), ref["y"])
    print(f"  rel_fro={err:.3e}", flush=True)
    assert err <= G.TOL, err


# ---- (1,2,V) on 160-token tiles: the plan takes them by expected tile and round counts; here they are forced, so
# ---- that every shape below runs both products on them (and, without the knobs, on whatever the plan takes) ----
VEC160_CASES = [
    LayerConfig("vec160_two_tiles", T=1300, H=512, F=768, E=4, topk=2, fmt=(1, 2, 8), seed=141),                  # ~650 pairs per expert: ragged fifth tile
    LayerConfig("vec160_shared", T=3000, H=1024, F=512, E=3, topk=1, S=1, fmt=(1, 2, 16), renormalize=False, seed=142),
    LayerConfig("vec160_odd_rows", T=2000, H=640, F=448, E=2, topk=2, fmt=(1, 2, 32), seed=143),                  # row tiles that do not fill a block
    LayerConfig("vec160_many_experts", T=2000, H=256, F=512, E=40, topk=8, fmt=(1, 2, 8), logits="biased", seed=144),
    LayerConfig("vec160_loop", T=7000, H=1024, F=1024, E=4, topk=2, fmt=(1, 2, 8), seed=145),                    # more tiles than resident blocks
]


@pytest.mark.parametrize("cfg", VEC160_CASES, ids=[c.name for c in VEC160_CASES])
def test_vector_wise_format_on_160_token_tiles(monkeypatch, tuning_library, cfg):
    monkeypatch.setenv("SSMM_VEC_GU_NT5", "1")
    monkeypatch.setenv("SSMM_VEC_DOWN_NT5", "1")
    monkeypatch.setenv("SSMM_TILE_SHAPE", "2")          # the large-bucket rules, whatever the bucket size
    got, ref, err = run_case(cfg)
    monkeypatch.setenv("SSMM_VEC_GU_NT5", "0")
    monkeypatch.setenv("SSMM_VEC_DOWN_NT5", "0")
    y, _ = G.run_gpu_layer(cfg, *G.make_inputs(cfg))     # the 128-token tiles on the same inputs
    d = G.rel_fro(G.bf16_tensor_to_f64(y), got)
    print(f"  160- vs 128-token tiles rel_fro={d:.3e}", flush=True)
    assert d == 0.0      # same products in the same order: the tile width changes no sum


# ---- plain 2:4, large buckets: the down projection on 512-row x 128-token tiles (the plan takes them when they
# ---- need a round of the resident blocks less than the 160-token ones); forced here ----
TALL128_CASES = [
    LayerConfig("tall128_two_tiles", T=1300, H=512, F=768, E=4, topk=2, seed=151),
    LayerConfig("tall128_odd_rows", T=3000, H=1088, F=512, E=3, topk=1, S=1, renormalize=False, seed=152),   # 34 row tiles: the last block half empty
    LayerConfig("tall128_loop", T=7000, H=2048, F=1024, E=4, topk=2, seed=153),                              # more tiles than resident blocks
]


@pytest.mark.parametrize("cfg", TALL128_CASES, ids=[c.name for c in TALL128_CASES])
def test_down_projection_on_512_by_128_tiles(monkeypatch, tuning_library, cfg):
    monkeypatch.setenv("SSMM_TILE_SHAPE", "2")
    monkeypatch.setenv("SSMM_DOWN_TALL_NT4", "1")
    got, ref, err = run_case(cfg)
    monkeypatch.setenv("SSMM_DOWN_TALL_NT4", "0")
    y, _ = G.run_gpu_layer(cfg, *G.make_inputs(cfg))     # the 160-token tiles on the same inputs
    assert G.rel_fro(G.bf16_tensor_to_f64(y), got) == 0.0   # the tile width changes no sum


@pytest.mark.parametrize("cfg", [LayerConfig("gu64_small", T=40, H=512, F=1024, E=8, topk=2, seed=161),
                                 LayerConfig("gu64_two_tiles", T=300, H=256, F=768, E=6, topk=2, S=1, seed=162),      # the shared expert needs five tiles of 64
                                 LayerConfig("gu64_odd_rows", T=200, H=1024, F=448, E=3, topk=1, seed=163)], ids=lambda c: c.name)
def test_first_product_on_256_by_64_tiles(monkeypatch, tuning_library, cfg):
    """The 64-token version of the widest gate/up tile (the plan takes it for small buckets of layers with many
    row tiles), forced here on small layers; the tile width changes no sum."""
    monkeypatch.setenv("SSMM_GU_SHAPE", "2")
    monkeypatch.setenv("SSMM_GU_NT5", "0")
    monkeypatch.setenv("SSMM_GU_NT2", "1")
    got, ref, err = run_case(cfg)
    monkeypatch.setenv("SSMM_GU_NT2", "0")
    y, _ = G.run_gpu_layer(cfg, *G.make_inputs(cfg))     # the 128-token tiles on the same inputs
    assert G.rel_fro(G.bf16_tensor_to_f64(y), got) == 0.0

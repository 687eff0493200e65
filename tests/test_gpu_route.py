"""GPU parity: routing and selection arrays against the oracle.  Integer outputs
(ids, offsets, sel, inv) bit-exact; weights to fp32 rounding."""
import numpy as np
import pytest
import torch

from oracle import ssmm_oracle as O
from paper_2503_10725_amd import binding as B

pytestmark = pytest.mark.gpu


def check(logits_np, topk, S, renorm):
    T, E = logits_np.shape
    lg = torch.from_numpy(logits_np).cuda()
    r = B.route_bucket(lg, topk, S, renorm)
    torch.cuda.synchronize()
    ids, w = O.route(logits_np, topk, S, renorm)
    off, sel, slot, inv = O.bucket(ids, E + S)
    assert np.array_equal(r.topk_ids.cpu().numpy(), ids[:, :topk])
    assert np.array_equal(r.expert_offsets.cpu().numpy(), off)
    assert np.array_equal(r.sel.cpu().numpy(), sel)
    assert np.array_equal(r.inv.cpu().numpy(), inv)
    np.testing.assert_allclose(r.topk_w.cpu().numpy(), w[:, :topk], rtol=1e-5, atol=1e-9)
    np.testing.assert_allclose(r.sel_w.cpu().numpy(), w[sel, slot], rtol=1e-5, atol=1e-9)
    return r


@pytest.mark.parametrize("T,E,topk,S,renorm", [
    (128, 8, 2, 0, True), (16, 8, 2, 0, True), (1, 8, 2, 0, True), (257, 8, 2, 0, False),
    (2048, 64, 8, 0, False), (8192, 64, 6, 2, False), (4096, 8, 2, 0, True), (1000, 200, 16, 3, True),
    (300, 5, 5, 0, True), (77, 3, 1, 1, True),
    # up to 256 tokens one fused block places the tokens (up to 16 it also routes them)
    (64, 64, 8, 2, False), (65, 8, 2, 0, True), (256, 64, 6, 2, False), (200, 250, 16, 6, True), (3, 2, 2, 0, True),
    (16, 64, 8, 2, False), (17, 64, 8, 2, False), (9, 250, 16, 6, True),
    # more than 64 chunks of 256 tokens: the offset scan carries between rounds
    (20000, 64, 2, 1, True), (17000, 130, 3, 0, False),
])
def test_route_bucket_matches_oracle(T, E, topk, S, renorm):
    print(f"case T={T} E={E} topk={topk} S={S} renorm={renorm}", flush=True)
    rng = np.random.default_rng(T + E + topk)
    lg = rng.standard_normal((T, E)).astype(np.float32)
    check(lg, topk, S, renorm)


def test_ties_and_signed_zeros():
    rng = np.random.default_rng(1)
    lg = rng.integers(-2, 3, size=(513, 64)).astype(np.float32)      # heavy ties
    lg[7] = 0.0
    lg[8, ::2] = -0.0
    lg[8, 1::2] = 0.0
    check(lg, 8, 0, True)


def test_minus_infinity_logits_are_never_chosen():
    rng = np.random.default_rng(5)
    lg = rng.standard_normal((300, 8)).astype(np.float32)
    lg[:, [1, 4, 6]] = -np.inf
    lg[::7, 0] = -np.inf
    r = check(lg, 2, 0, True)
    ids = r.topk_ids.cpu().numpy()
    assert not np.isin(ids, [1, 4, 6]).any()


def test_skewed_loads_and_empty_experts():
    rng = np.random.default_rng(2)
    lg = rng.standard_normal((600, 16)).astype(np.float32)
    lg[:, 3] -= 100.0            # never chosen
    lg[:, 5] += 100.0            # always chosen
    r = check(lg, 2, 0, True)
    off = r.expert_offsets.cpu().numpy()
    assert off[4] - off[3] == 0 and off[6] - off[5] == 600


def test_uniform_logits_like_the_mixtral_config():
    rng = np.random.default_rng(3)
    check(rng.random((4096, 8), dtype=np.float32), 2, 0, True)


def test_no_tokens():
    lg = torch.empty((0, 8), dtype=torch.float32, device="cuda")
    r = B.route_bucket(lg, 2, 1, True)
    torch.cuda.synchronize()
    assert r.expert_offsets.cpu().numpy().tolist() == [0] * 10


def test_repeat_calls_are_bit_identical():
    rng = np.random.default_rng(4)
    lg = torch.from_numpy(rng.standard_normal((3000, 64)).astype(np.float32)).cuda()
    a = B.route_bucket(lg, 6, 2, False)
    b = B.route_bucket(lg, 6, 2, False)
    torch.cuda.synchronize()
    for name in ("topk_ids", "expert_offsets", "sel", "inv", "topk_w", "sel_w"):
        assert torch.equal(getattr(a, name), getattr(b, name))


# ---- the router in front: logits = x Wr^T (section 2.1) --------------------------------------
from paper_2503_10725_amd import synth


@pytest.mark.parametrize("T,H,E", [(100, 256, 8), (700, 512, 64), (65, 128, 70), (33, 64, 200), (1, 64, 3), (4096, 1024, 8)])
def test_router_logits_match_oracle(T, H, E):
    print(f"case T={T} H={H} E={E}", flush=True)
    g = torch.Generator(device="cuda").manual_seed(T + H + E)
    x = torch.randn((T, H), generator=g, device="cuda").to(torch.bfloat16)
    wr = (torch.randn((E, H), generator=g, device="cuda") * 0.1).to(torch.bfloat16)
    lg = B.router_logits(x, wr)
    torch.cuda.synchronize()
    ref = O.router_logits(synth.bits(x), synth.bits(wr))
    # bf16 x bf16 products are exact in fp32; the error is that of H fp32 additions
    scale = float(np.abs(ref).max())
    np.testing.assert_allclose(lg.cpu().numpy(), ref, rtol=0, atol=2e-6 * np.sqrt(H) * scale)
    # same bits on a second call
    assert torch.equal(lg, B.router_logits(x, wr))
    # the top-k decision is taken on these fp32 logits on both sides
    if E >= 2:
        check(lg.cpu().numpy(), min(2, E), 0, True)


def test_router_logits_argument_checks():
    x = torch.zeros((4, 24), dtype=torch.bfloat16, device="cuda")
    wr = torch.zeros((3, 24), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.SsmmError):          # H not a multiple of 16
        B.router_logits(x, wr)
    x = torch.zeros((4, 32), dtype=torch.bfloat16, device="cuda")
    wr = torch.zeros((257, 32), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.SsmmError):          # more experts than the routing kernels admit
        B.router_logits(x, wr)
    assert B.router_logits(torch.zeros((0, 32), dtype=torch.bfloat16, device="cuda"),
                           torch.zeros((4, 32), dtype=torch.bfloat16, device="cuda")).shape == (0, 4)


@pytest.mark.parametrize("E,topk", [(8, 2), (130, 4), (64, 8), (250, 16)])
def test_masked_and_nan_logits_give_distinct_ids(E, topk):
    """-infinity logits (masked experts) and NaN logits (counted as -infinity): when a token has fewer
    than topk numbers among its logits the rest of its choice goes by ascending expert id, and its ids
    stay distinct (every bucket position is written).  Bit-exact against the oracle, on both routing
    paths (up to 64 experts: ranks by place; above: repeated arg-max)."""
    rng = np.random.default_rng(E + topk)
    lg = rng.standard_normal((600, E)).astype(np.float32)
    lg[:, ::3] = -np.inf
    lg[5:90, 1::3] = np.nan
    lg[100:200] = -np.inf
    lg[100:200, [E - 1, 2]] = [0.5, -1.0]        # two numbers per token only
    lg[300:350] = np.nan
    lg[300:350, E // 2] = 3.0                    # one number per token only
    r = check(lg, topk, 1, True)
    ids = r.topk_ids.cpu().numpy()
    assert all(len(set(row)) == topk for row in ids.tolist())
    assert (ids[100:200, :2] == [E - 1, 2]).all() and (ids[300:350, 0] == E // 2).all()

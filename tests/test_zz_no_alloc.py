"""GPU: the entry point that takes no workspace and allocates nothing (ssmm_route_bucket_noalloc)
returns what ssmm_route_bucket returns, bit for bit, on two calls in a row that share the
library's fixed scratch array -- the second with a smaller input -- and refuses sizes beyond
that array."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2503_10725_amd import binding as B

pytestmark = pytest.mark.gpu

FIELDS = ("topk_ids", "topk_w", "expert_offsets", "sel", "sel_w", "inv")


def both_ways(T, E, topk, S, renorm, seed):
    print(f"case T={T} E={E} topk={topk} S={S} renorm={renorm} seed={seed}", flush=True)
    g = torch.Generator(device="cuda").manual_seed(seed)
    logits = torch.randn((T, E), generator=g, device="cuda", dtype=torch.float32)
    want = B.route_bucket(logits, topk, S, renorm)
    got = B.RouteBuffers(T, E, topk, S, "cuda")
    for f in FIELDS:                                  # nothing of an earlier call may show through
        getattr(got, f).view(torch.int32).fill_(-7)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    B.route_bucket_noalloc(logits, topk, S, renorm, got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for f in FIELDS:                                  # same kernels, same order of work: identical bits, weights included
        a, b = getattr(want, f), getattr(got, f)
        assert torch.equal(a.view(torch.int32), b.view(torch.int32)), f


def test_two_calls_in_a_row_second_one_smaller():
    # both beyond the 256 tokens one fused block handles, so both use the per-chunk histograms in the scratch array
    both_ways(5000, 64, 6, 2, False, seed=11)
    both_ways(700, 8, 2, 0, True, seed=12)
    # and once more with the larger shape: the smaller call's leftovers do not matter either
    both_ways(5000, 64, 6, 2, False, seed=13)


def test_small_and_empty_inputs():
    both_ways(100, 8, 2, 0, True, seed=14)            # fused block, no scratch
    off = torch.full((8 + 1,), -1, dtype=torch.int32, device="cuda")
    st = B.lib().ssmm_route_bucket_noalloc(None, 0, 8, 2, 0, 1, None, None, ctypes.c_void_p(off.data_ptr()), None, None,
                                           None, None)
    torch.cuda.synchronize()
    assert st == B.SSMM_OK and int(off.abs().sum()) == 0


def test_sizes_beyond_the_fixed_scratch_are_refused():
    one = ctypes.c_void_p(256)                        # never dereferenced: the call is refused before any launch
    lib = B.lib()
    # ceil(T / 256) * E cells of the histogram must fit 65536
    assert lib.ssmm_route_bucket_noalloc(one, 65536 + 1, 256, 2, 0, 1, one, one, one, one, one, one, None) == B.SSMM_ELIMIT
    assert lib.ssmm_route_bucket_noalloc(one, 262144 + 1, 64, 2, 0, 1, one, one, one, one, one, one, None) == B.SSMM_ELIMIT
    assert "scratch" in B.strerror(B.SSMM_ELIMIT)
    # at the limit the usual checks answer
    assert lib.ssmm_route_bucket_noalloc(None, 65536, 256, 2, 0, 1, one, one, one, one, one, one, None) == B.SSMM_EINVAL

"""fo_encode_noalloc (the entry point for callers that cannot allocate: static device scratch, no plan) against
fo_encode on the same inputs: same packed signs and same amplitudes, bit for bit, on calls made one after the
other that share the static array, each smaller than the one before."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2405_11095_amd import binding, inputs
    assert torch.cuda.is_available()
    binding.load_library()
    return binding, inputs, torch.device("cuda:0")


def _encode_both(B, torch, dev, g, d, M, blk, party, rnd, seed, force=None):
    plan = B.Plan(d=d, M=M, block_log2=blk, seed=seed)
    W, nb = plan.W, plan.nblocks
    bits_a = torch.zeros(W, dtype=torch.int64, device=dev)
    bits_b = torch.full((W,), -1, dtype=torch.int64, device=dev)
    lam_a = torch.zeros(nb, dtype=torch.float32, device=dev)
    lam_b = torch.full((nb,), -1.0, dtype=torch.float32, device=dev)
    flags = 0
    if force is not None:
        lam_a[:] = force
        lam_b[:] = force
        flags = B.FORCE_SCALE
    plan.fo_encode(g, rnd, party, bits_a, lam_a, flags=flags)
    B.fo_encode_noalloc(plan.params, g, rnd, party, bits_b, lam_b, flags=flags)
    torch.cuda.synchronize()
    plan.close()
    return bits_a.cpu().numpy(), bits_b.cpu().numpy(), lam_a.cpu().numpy(), lam_b.cpu().numpy()


def test_noalloc_encode_equals_plan_encode_on_consecutive_calls(env):
    import torch
    B, inputs, dev = env
    # (d, block_log2): the largest vector the entry point takes (n = 2^22, seven strided stages), then smaller ones
    # that reuse the same static array: a ragged two-pass one, blocks of 2^16 (one pass), a single tile
    cases = [((1 << 22) - 4321, 0), (70_001, 0), ((1 << 19) + 5, 16), (30_000, 0), (200_003, 12), (1 << 21, 0)]
    for k, (d, blk) in enumerate(cases):
        print(f"noalloc case d={d} block_log2={blk}", flush=True)
        g = torch.from_numpy(inputs.heavy_tailed(d, k)).to(dev)
        a, b, la, lb = _encode_both(B, torch, dev, g, d, 3, blk, party=k % 3, rnd=5 + k, seed=77 + k)
        assert np.array_equal(la, lb) and np.all(la > 0)
        assert np.array_equal(a, b)
        assert 0.3 < np.unpackbits(a.view(np.uint8)).mean() < 0.7     # a real message, not a cleared buffer
    # forced amplitudes and the server's party (input of the padded length)
    d = 150_000
    plan = B.Plan(d=d, M=2, seed=9)
    nt = plan.ntot
    plan.close()
    g = torch.from_numpy(inputs.gaussian(nt, 1)).to(dev)
    a, b, la, lb = _encode_both(B, torch, dev, g[:d].clone(), d, 2, 0, party=1, rnd=3, seed=9, force=0.01)
    assert np.array_equal(a, b) and np.array_equal(la, lb)


def test_noalloc_rejects_what_it_cannot_take(env):
    import torch
    B, inputs, dev = env
    d = B.NOALLOC_MAX_N + 1
    g = torch.zeros(64, dtype=torch.float32, device=dev)
    bits = torch.zeros(64, dtype=torch.int64, device=dev)
    lam = torch.zeros(64, dtype=torch.float32, device=dev)
    p = B.Params(d, 1, 0, 1, 0, 1, 0, 2.0, 2.0, 1.0, 1, 0)
    with pytest.raises(B.FoError) as e:
        B.fo_encode_noalloc(p, g, 0, 0, bits, lam)
    assert e.value.code == B.ESIZE and "FO_NOALLOC_MAX_N" in str(e.value)
    p = B.Params(1000, 1, 0, 1, 0, 1, 0, 1.0, 2.0, 1.0, 1, 0)      # alpha < 2
    with pytest.raises(B.FoError) as e:
        B.fo_encode_noalloc(p, g, 0, 0, bits, lam)
    assert e.value.code == B.EINVAL
    p = B.Params(1000, 2, 0, 1, 0, 1, 0, 2.0, 2.0, 1.0, 1, 0)
    with pytest.raises(B.FoError) as e:
        B.fo_encode_noalloc(p, g, 0, 2, bits, lam)                  # party out of range
    assert e.value.code == B.EINVAL
    with pytest.raises(B.FoError) as e:
        B.fo_encode_noalloc(p, g[1:], 0, 0, bits, lam)              # gradient not 16-byte aligned
    assert e.value.code == B.EALIGN

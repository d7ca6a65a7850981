"""The allocation-free top-k entry point (elmo_topk_static: scratch in a device array inside the
library) against elmo_head_topk on a head over the same weights, through the C ABI: two calls in a
row, the second with a smaller input, so that whatever the first call left in the shared scratch
must not show in the second."""
import sys

import numpy as np
import pytest
import torch

from paper_2510_11168_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def _one_call(b, fmt, L, d, B, k, seed):
    """Weights and queries on the device; returns (static result, head result) as numpy arrays."""
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    head = b.Head(L, d, fmt, 4096, 0, B, 64)
    f = torch.randn(L * d, device=DEV, generator=g) * 0.05
    b.elmo_quantize(f, f.numel(), fmt, 0, 0, 0, 0, head.weights())
    X = torch.from_numpy(synth.make_x(np.random.default_rng(seed), B, d).view(np.int16)).to(DEV)
    out = []
    for static in (True, False):
        idx = torch.full((B, k), -7, dtype=torch.int32, device=DEV)
        sc = torch.full((B, k), -7.0, dtype=torch.float32, device=DEV)
        if static:
            b.elmo_topk_static(head.W, L, d, fmt, X, B, k, idx, sc)
        else:
            head.topk(X, k, idx, sc)
        torch.cuda.synchronize()
        out.append((idx.cpu().numpy(), sc.cpu().numpy()))
    head.close()
    return out


@pytest.mark.parametrize("fmt", [1, 0])
def test_static_topk_equals_the_heads_topk_on_two_calls_in_a_row(fmt):
    from paper_2510_11168_amd import binding as b
    assert torch.cuda.is_available()
    # first call: 128 queries, 40000 labels, two pages; second call: fewer queries, fewer labels, smaller k
    for (L, d, B, k, seed) in ((40000 + 13, 512, 128, 150, 1), (3000 + 5, 256, 37, 10, 2)):
        say(f"[static top-k] fmt={fmt} L={L} d={d} B={B} k={k}")
        (si, ss), (hi, hs) = _one_call(b, fmt, L, d, B, k, seed)
        assert np.array_equal(si, hi), "label ids differ from elmo_head_topk"
        assert np.array_equal(ss.view(np.uint32), hs.view(np.uint32)), "scores differ from elmo_head_topk"
        assert si.min() >= 0 and si.max() < L and np.all(np.diff(ss, axis=1) <= 0)


def test_static_topk_rejects_what_does_not_fit():
    from paper_2510_11168_amd import binding as b
    W = torch.zeros(1000 * 256, dtype=torch.uint8, device=DEV)
    X = torch.zeros((200, 256), dtype=torch.int16, device=DEV)
    for kw in (dict(B=129), dict(d=4096 + 128), dict(d=100), dict(k=0), dict(k=1001), dict(fmt=2)):
        a = dict(L=1000, d=256, fmt=1, B=8, k=5)
        a.update(kw)
        with pytest.raises(b.ElmoError) as e:
            b.elmo_topk_static(W, a["L"], a["d"], a["fmt"], X, a["B"], a["k"], None, None)
        assert e.value.code in (-1, -2)

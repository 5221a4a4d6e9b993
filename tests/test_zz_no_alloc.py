"""The entry point that allocates nothing: moe_dispatch_noalloc keeps the
dispatch index scratch in a fixed device array inside the library.  Its outputs
must equal moe_dispatch's bit for bit, on two calls in a row (the second with a
smaller input, so stale scratch contents of the first call would show), and
sizes beyond the fixed array are refused."""
import numpy as np
import pytest
import torch

import paper_2601_08800_amd as moe
from paper_2601_08800_amd import binding as B
from paper_2601_08800_amd.layer import config_from_workload
from workloads import gen
from helpers import dev, host

pytestmark = pytest.mark.gpu


def _dispatch_both(w, seed):
    """ids from a seeded draw (distinct experts per token, a hot expert and some
    empty ones); returns the outputs of moe_dispatch and of moe_dispatch_noalloc."""
    cfg = config_from_workload(w)
    rng = np.random.default_rng(seed)
    ids = np.stack([rng.permutation(w.E)[:w.k] for _ in range(w.T)]).astype(np.int32)
    ids[::3, 0] = w.expert_lo                       # a hot local expert
    x = dev(gen.make_x(w))
    A = w.T * w.k
    res = []
    for which in ("ws", "noalloc"):
        i32 = dict(dtype=torch.int32, device="cuda")
        counts, offsets = torch.full((w.E_loc,), -7, **i32), torch.full((w.E_loc + 1,), -7, **i32)
        perm, inv = torch.full((A,), -7, **i32), torch.full((A,), -7, **i32)
        xs = torch.zeros((A, w.H), dtype=torch.bfloat16, device="cuda")
        if which == "ws":
            ws = torch.empty(moe.moe_workspace_bytes(cfg, w.T), dtype=torch.uint8, device="cuda")
            moe.moe_dispatch(cfg, w.T, x, dev(ids), counts, offsets, perm, inv, xs, ws)
        else:
            moe.moe_dispatch_noalloc(cfg, w.T, x, dev(ids), counts, offsets, perm, inv, xs)
        torch.cuda.synchronize()
        n = int(offsets[-1].item())
        res.append((host(counts), host(offsets), host(perm)[:n], host(inv), host(xs[:n])))
    return res


def test_noalloc_dispatch_equals_dispatch_on_two_calls_in_a_row():
    base = gen.CONFIGS["c2p"]
    # both sizes take the multi-kernel path (more than 4096 assignments), which is
    # the one that uses the scratch; the second call is the smaller one
    big = base.replace(name="na_big", T=3000, H=512, E=64, k=8, I=128, expert_lo=8, expert_hi=40)
    small = base.replace(name="na_small", T=700, H=512, E=64, k=8, I=128, expert_lo=8, expert_hi=40)
    for w, seed in ((big, 1), (small, 2)):
        print("dispatch", w.name, "T", w.T, flush=True)
        a, b = _dispatch_both(w, seed)
        for u, v, what in zip(a, b, ("counts", "offsets", "perm", "inv", "xs")):
            assert np.array_equal(u, v), (w.name, what)
        assert a[1][-1] > 0


def test_noalloc_dispatch_refuses_sizes_beyond_its_scratch():
    limit = moe.moe_dispatch_noalloc_max_bytes()
    assert limit == 4 << 20
    # 128 local experts x ceil(T*8/64) sub-chunks x 4 bytes: one token past 65 536
    w = gen.CONFIGS["c2x"].replace(T=65536 + 8)
    cfg = config_from_workload(w)
    P = 0x1000                                       # never dereferenced: the size check comes first
    with pytest.raises(moe.MoEError) as ei:
        moe.moe_dispatch_noalloc(cfg, w.T, P, P, P, P, P, P, P)
    assert ei.value.status == B.MOE_ERR_WORKSPACE

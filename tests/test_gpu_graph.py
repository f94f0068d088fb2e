"""The library under HIP graph capture: a block's calls (one-call refresh step, reuse steps, and the external pass on the
library's built-in scratch array, which exists for callers that cannot allocate under capture) are recorded into a graph
once and replayed several times, with eager work and synchronisations between the replays; every replay must reproduce
the eager result bit for bit.  The library records kernels only (no memset nodes)."""
import pytest
import torch

from paper_2602_05305_amd import flashblock as fb
from paper_2602_05305_amd import workloads as wl

import fb_testlib as T

pytestmark = pytest.mark.gpu


def test_block_replays_match_eager_bit_for_bit():
    w = wl.CONFIGS["llm_32k"].with_(name="graph", prefix_len=8192 + 19, steps=3, refresh=3)
    print(f"[case] graph capture {w.name}", flush=True)
    Kp, Vp = wl.make_prefix(w, 71)
    steps = wl.make_block_steps(w, 71)
    shape = T.shape_of(w)
    kp, vp = T.to_dev(Kp, "bf16"), T.to_dev(Vp, "bf16")
    dev_steps = [tuple(T.to_dev(x, "bf16") for x in st) for st in steps]
    ws = T.workspace(shape)
    ext, ext2 = T.Partial(w), T.Partial(w)
    outs = [torch.empty_like(dev_steps[0][0]) for _ in steps]

    def block():
        for t, (q, kb, vb) in enumerate(dev_steps):
            if t == 0:
                fb.fb_refresh_step(shape, q, kp, vp, kb, vb, ext.o, ext.m, ext.lse, outs[t], None, ws)
                fb.fb_external_partial_builtin_ws(shape, q, kp, vp, ext2.o, ext2.m, ext2.lse)
            else:
                fb.fb_internal_merge(shape, q, kb, vb, ext.o, ext.m, ext.lse, outs[t], None)

    block()                                   # eager: first launches, attribute and symbol look-ups stay outside the capture
    torch.cuda.synchronize()
    want = [o.clone() for o in outs] + [ext.o.clone(), ext.lse.clone(), ext2.o.clone(), ext2.lse.clone()]
    assert torch.equal(ext.lse, ext2.lse)     # same pass, caller workspace vs built-in scratch

    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        block()
    scratch = torch.empty(1 << 22, device=T.DEV)
    for rep in range(4):
        for t in outs + [ext.o, ext.lse, ext2.o, ext2.lse]:
            t.fill_(float("nan"))
        scratch.normal_()                     # unrelated eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = outs + [ext.o, ext.lse, ext2.o, ext2.lse]
        for i, (a, b) in enumerate(zip(got, want)):
            assert torch.equal(a, b), f"replay {rep}: tensor {i} differs from the eager result"

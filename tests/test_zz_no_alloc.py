"""fb_external_partial_builtin_ws (the entry point for callers that cannot allocate a workspace) against
fb_external_partial and the oracle: two calls in a row on the library's built-in scratch array, the second on a
smaller input, then a shape that does not fit (rejected before any launch)."""
import numpy as np
import pytest
import torch

from oracle import flashblock_oracle as orc
from paper_2602_05305_amd import flashblock as fb
from paper_2602_05305_amd import workloads as wl

import fb_testlib as T

pytestmark = pytest.mark.gpu


def _one(w, seed):
    print(f"[case] builtin_ws {w.name} seed={seed}", flush=True)
    Kp, Vp = wl.make_prefix(w, seed)
    Q = wl.make_block_steps(w, seed, steps=1)[0][0]
    shape = T.shape_of(w)
    q, kp, vp = T.to_dev(Q, w.dtype), T.to_dev(Kp, w.dtype), T.to_dev(Vp, w.dtype)
    ref, got = T.Partial(w), T.Partial(w)
    fb.fb_external_partial(shape, q, kp, vp, ref.o, ref.m, ref.lse, T.workspace(shape))
    for t in (got.o, got.m, got.lse):
        t.fill_(float("nan"))
    fb.fb_external_partial_builtin_ws(shape, q, kp, vp, got.o, got.m, got.lse)
    torch.cuda.synchronize()
    # same kernels, same split count, same fold order: identical bits
    assert torch.equal(got.o, ref.o) and torch.equal(got.m, ref.m) and torch.equal(got.lse, ref.lse)
    T.check_partial(got.numpy(), orc.partial(Q, Kp, Vp), w.dtype, f"{w.name} builtin_ws ext")


def test_builtin_ws_two_calls_second_smaller_then_too_large():
    assert fb.fb_builtin_workspace_bytes() == 20 * 1024 * 1024
    big = wl.CONFIGS["llm_32k"].with_(name="builtin_a", prefix_len=8192 + 33)
    small = wl.Workload("builtin_b", 2, 4, 2, 64, 1500, 16, 1, 1, "bf16", 1.0)
    _one(big, 901)
    _one(small, 902)
    _one(wl.Workload("builtin_c", 1, 4, 4, 64, 300, 5, 1, 1, "f32", 1.0), 903)
    # the video shape needs more split-partial space than the built-in array has: refused, nothing launched
    v = wl.CONFIGS["video"]
    shape = T.shape_of(v)
    assert fb.fb_workspace_bytes(shape) > fb.fb_builtin_workspace_bytes()
    dummy = torch.zeros(16, device=T.DEV)
    with pytest.raises(fb.FlashBlockError) as ei:
        fb.fb_external_partial_builtin_ws(shape, dummy, dummy, dummy, dummy, dummy, dummy)
    assert ei.value.status == fb.FB_ERR_WORKSPACE

#!/usr/bin/env python3
"""Benchmark of the FlashBlock attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llm_32k] [--no-long] [--no-cpu]

A "step" is one diffusion step of one block: fb_internal_merge on every step plus the external
pass on refresh steps (t mod R == 0; both in one call, fb_refresh_step).  The headline value is the
attention time per diffusion step on the LLM-shaped 32K-context workload with the prefix K/V
resident in HBM; consecutive blocks rotate through distinct K/V buffer sets so that the 128 MiB of
one set cannot be served from the last-level cache.

Timing protocol.  After W warm-up steps (and at least 150 ms of the same work: the clock governor of
the part needs that long to settle after an idle period, and the first ~50 ms of a load run up to
40 % slower), exactly K steps are launched between two events recorded on the stream; when K steps
are short the K-step sequence is repeated back to back and the value is the median over the
repeats, so that it does not depend on K.  Every kernel-level number is the median (and minimum) of
at least 30 event-bracketed launches after the same kind of warm-up.

One JSON line is printed, with
  roofline      the external-pass kernel against the HBM roofline: HIP events recorded on the
                stream around that kernel inside the refresh-step call, plus the read ceiling of this
                GPU measured in the same process by a kernel that only reads (measured_peak),
  cpu_baseline  the numpy float64 oracle timed on the host cores on whole blocks of the same shape,
  parity        max |gpu - oracle| of this run on the tiny fp32 configuration and on a 32K block,
and extra objects for the full-recomputation comparison (R = 1 with the same kernels), the
128K-context external pass, the video-shaped (MFMA-bound), sparse and paged passes.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth


class HipEvents:
    """Raw HIP events through libamdhip64 (already loaded by torch)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def create(self):
        ev = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(ev))
        if rc != 0:
            raise RuntimeError(f"hipEventCreate failed: {rc}")
        return ev

    def elapsed_ms(self, a, b):
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return ms.value

    def destroy(self, ev):
        self.hip.hipEventDestroy(ev)


def external_algorithmic_bytes(w, fused=False):
    """Bytes the external pass must move per launch: prefix K and V once, Q once, and the
    (o, m, lse) partial written once.  Split-KV scratch traffic is overhead, not counted.
    The fused refresh launch also reads the block's own K and V."""
    esz = 4 if w.dtype == "f32" else 2
    rows = w.batch * w.n_q_heads * w.block_len
    blk = 2 * w.batch * w.n_kv_heads * w.block_len * w.head_dim * esz if fused else 0
    return w.kv_bytes + rows * w.head_dim * esz + rows * (w.head_dim + 2) * 4 + blk


class DeviceBlock:
    """Device-resident synthetic data of one workload: NSETS prefix K/V sets, one block's per-step
    (Q, K_block, V_block), the cached partial, outputs and workspace."""

    def __init__(self, w, nsets, seed=1234, fused=False):
        import torch
        from paper_2602_05305_amd import flashblock as fb
        self.w, self.fb, self.torch = w, fb, torch
        dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
        g = torch.Generator(device="cuda").manual_seed(seed)
        kshape = (w.batch, w.n_kv_heads, w.prefix_len, w.head_dim)
        self.K = [(torch.randn(kshape, device="cuda", generator=g) * w.input_scale).to(dt) for _ in range(nsets)]
        self.V = [(torch.randn(kshape, device="cuda", generator=g) * w.input_scale).to(dt) for _ in range(nsets)]
        qs = (w.batch, w.n_q_heads, w.block_len, w.head_dim)
        ks = (w.batch, w.n_kv_heads, w.block_len, w.head_dim)
        q = torch.randn(qs, device="cuda", generator=g) * w.input_scale
        k = torch.randn(ks, device="cuda", generator=g) * w.input_scale
        v = torch.randn(ks, device="cuda", generator=g) * w.input_scale
        self.steps = []
        for _ in range(w.steps):     # cumulative random walk between diffusion steps
            self.steps.append((q.to(dt).contiguous(), k.to(dt).contiguous(), v.to(dt).contiguous()))
            q = self.steps[-1][0].float() + w.step_sigma * torch.randn(qs, device="cuda", generator=g)
            k = self.steps[-1][1].float() + w.step_sigma * torch.randn(ks, device="cuda", generator=g)
            v = self.steps[-1][2].float() + w.step_sigma * torch.randn(ks, device="cuda", generator=g)
        self.shape = fb.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.block_len, w.prefix_len, w.dtype)
        rows = (w.batch, w.n_q_heads, w.block_len)
        self.o = torch.empty(rows + (w.head_dim,), device="cuda", dtype=torch.float32)
        self.m = torch.empty(rows, device="cuda", dtype=torch.float32)
        self.lse = torch.empty(rows, device="cuda", dtype=torch.float32)
        self.out = torch.empty(qs, device="cuda", dtype=dt)
        self.ws = torch.empty(fb.fb_workspace_bytes(self.shape), device="cuda", dtype=torch.uint8)
        self.nsets = nsets
        self.fused = fused       # refresh steps through fb_refresh_step (one streaming launch + one combine)

    def step(self, t, kv_set, R, prof=None):
        """One diffusion step t of a block whose prefix is K/V set kv_set."""
        fb = self.fb
        q, kb, vb = self.steps[t]
        if t % R == 0 and self.fused:
            if prof is None:
                fb.fb_refresh_step(self.shape, q, self.K[kv_set], self.V[kv_set], kb, vb, self.o, self.m, self.lse,
                                   self.out, None, self.ws)
            else:
                fb.fb_refresh_step_prof(self.shape, q, self.K[kv_set], self.V[kv_set], kb, vb, self.o, self.m,
                                        self.lse, self.out, None, self.ws, prof[0], prof[1], prof[2])
            return
        if t % R == 0:
            if prof is None:
                fb.fb_external_partial(self.shape, q, self.K[kv_set], self.V[kv_set], self.o, self.m, self.lse, self.ws)
            else:
                fb.fb_external_partial_prof(self.shape, q, self.K[kv_set], self.V[kv_set], self.o, self.m, self.lse,
                                            0, self.ws, prof[0], prof[1], prof[2])
        fb.fb_internal_merge(self.shape, q, kb, vb, self.o, self.m, self.lse, self.out, None)

    def run_eager(self, n_steps, R, first_step=0):
        S = self.w.steps
        for i in range(first_step, first_step + n_steps):
            self.step(i % S, (i // S) % self.nsets, R)

    def make_graphs(self, R):
        """One HIP graph per K/V set holding a whole block (S steps)."""
        torch = self.torch
        graphs = []
        side = torch.cuda.Stream()
        for s in range(self.nsets):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                for t in range(self.w.steps):
                    self.step(t, s, R)
            graphs.append(g)
        return graphs


WARM_SECONDS = 0.15      # same work, untimed, before any timed region (clock governor settling)


def _median(xs):
    xs = sorted(xs)
    return xs[len(xs) // 2]


def time_steps(dev, n_steps, warmup, R, use_graph, target_s=0.12, max_reps=400):
    """Exactly n_steps diffusion steps (whole blocks replayed as graphs, any remainder eagerly) between two
    events on the stream, after `warmup` untimed steps and at least WARM_SECONDS of the same work.  The
    n_steps sequence is repeated back to back (about target_s of GPU time in all) and every repeat is timed.
    Returns a dict: median / min us per step over the repeats, number of repeats, wall-clock us per step over
    all repeats (host clock around the whole timed region, for cross-checking)."""
    torch = dev.torch
    S = dev.w.steps
    dev.run_eager(S, R)            # first launches (one-time kernel attribute calls) stay outside any capture
    torch.cuda.synchronize()
    graphs = dev.make_graphs(R) if use_graph else None

    def run(n, start):
        if graphs is None:
            dev.run_eager(n, R, start)
            return
        blocks, rem = divmod(n, S)
        b0 = start // S
        for b in range(blocks):
            graphs[(b0 + b) % dev.nsets].replay()
        if rem:
            dev.run_eager(rem, R, (b0 + blocks) * S)

    run(warmup, 0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    done = 0
    while time.perf_counter() - t0 < WARM_SECONDS:
        run(max(n_steps, 10 * S), 0)
        done += max(n_steps, 10 * S)
        torch.cuda.synchronize()
    est = (time.perf_counter() - t0) / max(done, 1)            # seconds per step, host clock, upper bound
    reps = int(min(max_reps, max(5, math.ceil(target_s / max(est * n_steps, 1e-9)))))
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    torch.cuda.synchronize()
    w0 = time.perf_counter()
    for a, b in evs:
        a.record()
        run(n_steps, 0)
        b.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - w0
    us = [a.elapsed_time(b) * 1e3 / n_steps for a, b in evs]
    return {"us": _median(us), "us_min": min(us), "repeats": reps, "wall_us": wall / (reps * n_steps) * 1e6}


def profile_external(dev, n_blocks, R, batch=8):
    """The same loop with HIP events around the kernels of the external pass (recorded by the library between
    its launches, on the stream they run on) and around every step.  Blocks are launched in batches of `batch`
    with a synchronisation between batches (bounded number of events in flight), after WARM_SECONDS of the same
    loop.  Returns us statistics of the attention kernel, the fold/combine kernel, a refresh step and a reuse step."""
    torch = dev.torch
    hev = HipEvents()
    S = dev.w.steps
    t0 = time.perf_counter()
    blk = 0
    while time.perf_counter() - t0 < WARM_SECONDS:
        for _ in range(4):
            for t in range(S):
                dev.step(t, blk % dev.nsets, R)
            blk += 1
        torch.cuda.synchronize()
    pool = [[hev.create() for _ in range(3)] for _ in range(batch)]
    attn, comb, refresh, reuse = [], [], [], []
    # pass 1: only the library's three events around the kernels of the refresh step (nothing else is recorded, so
    # that no other marker sits next to the kernel being timed); pass 2: events around every step
    left = n_blocks
    while left > 0:
        nb = min(batch, left)
        for t in range(S):                       # one untimed block first: the queue was drained by the synchronisation
            dev.step(t, blk % dev.nsets, R)
        blk += 1
        for i in range(nb):
            for t in range(S):
                dev.step(t, blk % dev.nsets, R, prof=pool[i] if t == 0 else None)
            blk += 1
        torch.cuda.synchronize()
        for i in range(nb):
            attn.append(hev.elapsed_ms(pool[i][0], pool[i][1]) * 1e3)
            comb.append(hev.elapsed_ms(pool[i][1], pool[i][2]) * 1e3)
        left -= nb
    left = n_blocks
    while left > 0:
        nb = min(batch, left)
        step_evs = []
        for i in range(nb):
            sev = [torch.cuda.Event(enable_timing=True) for _ in range(S + 1)]
            sev[0].record()
            for t in range(S):
                dev.step(t, blk % dev.nsets, R)
                sev[t + 1].record()
            step_evs.append(sev)
            blk += 1
        torch.cuda.synchronize()
        for i in range(nb):
            for t in range(S):
                (refresh if t % R == 0 else reuse).append(step_evs[i][t].elapsed_time(step_evs[i][t + 1]) * 1e3)
        left -= nb
    for evs in pool:
        for e in evs:
            hev.destroy(e)
    mean = lambda x: sum(x) / max(1, len(x))
    if os.environ.get("FB_BENCH_DEBUG"):
        print("attn us:", " ".join(f"{x:.0f}" for x in attn), file=sys.stderr)
    return {"attn_us": mean(attn), "attn_us_median": _median(attn), "attn_us_min": min(attn),
            "combine_us": _median(comb), "refresh_step_us": _median(refresh),
            "reuse_step_us": _median(reuse) if reuse else 0.0, "launches": len(attn)}


def read_traffic(workload_name):
    """HBM bytes per launch of the external-pass kernel as measured with rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE and recorded (with the commands) in profiles/; None if no such record exists."""
    tpath = os.path.join(ROOT, "profiles", f"attn_stream_external_{workload_name}_hbm_traffic.txt")
    if os.path.exists(tpath):
        for ln in open(tpath):
            if ln.startswith("hbm_bytes_per_launch"):
                return int(float(ln.split("=")[1].split()[0]))
    return None


def roofline_obj(w, prof, traffic=None, fused=False, ceilings=None):
    """HBM roofline of the streaming attention kernel of the external pass.  achieved = algorithmic bytes per
    launch / mean launch duration (HIP events on the stream, this run); peak = the published 8 TB/s;
    measured_peak = what a kernel that only reads the same number of bytes reached in this process."""
    from paper_2602_05305_amd import flashblock as fb
    # fb_refresh_step streams the block's own keys in the attention kernel only for blocks above 64 rows;
    # at the LLM shapes its streaming kernel is the plain external pass
    streams_block = fused and (w.block_len > 64 or w.block_len % 4 != 0)
    alg = external_algorithmic_bytes(w, streams_block)
    us = prof["attn_us"]
    ach = alg / us / 1e3
    shape = fb.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.block_len, w.prefix_len, w.dtype)
    kern = ("fb::attn_bf16_kernel<.., 6, ..> (refresh step: prefix splits + the block's own keys, one streaming launch)"
            if streams_block else "fb::" + fb.fb_external_kernel_name(shape) + " (external pass, streaming attention kernel)")
    r = {"bound": "hbm", "kernel": kern,
         "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
         "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": traffic,
         "traffic_source": ("profiles/attn_stream_external_%s_hbm_traffic.txt (rocprofv3 FETCH_SIZE / WRITE_SIZE of an "
                            "earlier run of the same kernel and workload, not measured in this run)" % w.name)
                           if traffic is not None else None,
         "algorithmic_bytes_per_launch": alg, "avg_launch_us": round(us, 2),
         "median_launch_us": round(prof["attn_us_median"], 2), "min_launch_us": round(prof["attn_us_min"], 2),
         "launches_timed": prof["launches"]}
    if ceilings is not None:
        r["measured_peak"] = ceilings["read_GBps"]
        r["frac_of_measured"] = round(ach / ceilings["read_GBps"], 4)
        r["measured_peak_kernel"] = ceilings["read_kernel"]
    return r


class Calib:
    """libfbcalib.so: kernels that do nothing but read, copy, or issue MFMAs (bench-only, not the product library)."""

    def __init__(self):
        path = os.path.join(ROOT, "paper_2602_05305_amd", "libfbcalib.so")
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: build it with `python -m paper_2602_05305_amd.build`")
        lib = ctypes.CDLL(path)
        vp = ctypes.c_void_p
        lib.fbc_read_vgpr.argtypes = [vp, ctypes.c_size_t, ctypes.c_int, vp, vp]
        lib.fbc_read_lds.argtypes = [vp, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, vp, vp]
        lib.fbc_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
        lib.fbc_mfma.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, vp]
        self.lib = lib


def measure_ceilings(torch, reps=30):
    """What this GPU sustains, measured in this process with the calibration kernels: a pure read of 512 MiB
    (three buffers rotated, so it comes from HBM) through registers and through direct-to-LDS loads into a ring
    (the data path of the streaming attention kernel), a plain copy, and back-to-back bf16 MFMAs."""
    lib = Calib().lib
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    nbytes = 512 * 1024 * 1024
    # random bytes: what the bus carries when real K/V stream through it (constant data would toggle fewer lines)
    bufs = [torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device="cuda") for _ in range(3)]
    sink = torch.zeros(64, dtype=torch.int32, device="cuda")
    i = [0]

    def check(rc):
        if rc != 0:
            raise RuntimeError(f"calibration launch failed: hipError {rc}")

    def read_vgpr():
        check(lib.fbc_read_vgpr(bufs[i[0] % 3].data_ptr(), nbytes, 512, sink.data_ptr(), st)); i[0] += 1

    def read_lds():
        check(lib.fbc_read_lds(bufs[i[0] % 3].data_ptr(), nbytes, 256, 4, sink.data_ptr(), st)); i[0] += 1

    def copy():
        check(lib.fbc_copy(bufs[(i[0] + 1) % 3].data_ptr(), bufs[i[0] % 3].data_ptr(), nbytes, st)); i[0] += 1

    iters, wgs = 4000, 2048
    flops = wgs * 4 * iters * 4 * 32768.0

    def mfma():
        check(lib.fbc_mfma(iters, wgs, 1, sink.data_ptr(), st))

    def mfma_const():
        check(lib.fbc_mfma(iters, wgs, 0, sink.data_ptr(), st))

    t_v, t_vmin = _ev_median_us(torch, read_vgpr, reps, 3, warm_s=0.1)
    t_l, t_lmin = _ev_median_us(torch, read_lds, reps, 3, warm_s=0.1)
    t_c, _ = _ev_median_us(torch, copy, reps, 3, warm_s=0.05)
    t_m, t_mmin = _ev_median_us(torch, mfma, 10, 2, warm_s=0.05)
    t_mc, _ = _ev_median_us(torch, mfma_const, 10, 2, warm_s=0.05)
    del bufs
    torch.cuda.empty_cache()
    best, kern = (t_v, "fbc_read_vgpr (16-byte loads into registers, 512 workgroups)") if t_v <= t_l else \
                 (t_l, "fbc_read_lds (direct-to-LDS loads into a 4-stage ring, 256 workgroups)")
    return {"read_GBps": round(nbytes / best / 1e3, 1), "read_kernel": kern,
            "read_bytes": nbytes, "read_vgpr_us": round(t_v, 1), "read_vgpr_min_us": round(t_vmin, 1),
            "read_lds_ring_us": round(t_l, 1), "read_lds_ring_min_us": round(t_lmin, 1),
            "copy_GBps_read_plus_write": round(2 * nbytes / t_c / 1e3, 1),
            "mfma_bf16_TFLOPs": round(flops / t_m / 1e6, 1), "mfma_us": round(t_m, 1),
            "mfma_bf16_TFLOPs_constant_operands": round(flops / t_mc / 1e6, 1),
            "mfma_note": "back-to-back v_mfma_f32_32x32x16_bf16, no memory traffic; operands changing from MFMA to MFMA (pseudo-random "
                         "bf16, what a real contraction presents: the part lowers its clock under that load) / one constant pair",
            "note": "medians of event-timed launches in this process; source paper_2602_05305_amd/csrc/fb_calib.hip"}


def parity_obj(torch, fb, wl):
    """max |gpu - oracle| of this run: the tiny fp32 configuration (all steps) and one whole block of the
    LLM-shaped 32K workload (refresh step through fb_refresh_step, reuse steps through fb_internal_merge),
    on the final output, on the normalised external attention A = o exp(m - lse) and on the log-normalisers."""
    import numpy as np
    from oracle import flashblock_oracle as orc
    res = {}
    for name in ("tiny_f32", "llm_32k"):
        w = wl.CONFIGS[name]
        tdt = torch.float32 if w.dtype == "f32" else torch.bfloat16
        up = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to("cuda").to(tdt).contiguous()
        Kp, Vp = wl.make_prefix(w, 7)
        steps = wl.make_block_steps(w, 7)
        want = orc.run_block_dense(Kp, Vp, steps, w.refresh)
        shape = fb.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.block_len, w.prefix_len, w.dtype)
        rows = (w.batch, w.n_q_heads, w.block_len)
        o = torch.empty(rows + (w.head_dim,), device="cuda")
        m, lse = torch.empty(rows, device="cuda"), torch.empty(rows, device="cuda")
        lse_out = torch.empty(rows, device="cuda")
        ws = torch.empty(fb.fb_workspace_bytes(shape), device="cuda", dtype=torch.uint8)
        kp, vp = up(Kp), up(Vp)
        e_out = e_A = e_L = e_Lf = 0.0
        for t, (Q, Kb, Vb) in enumerate(steps):
            q, kb, vb = up(Q), up(Kb), up(Vb)
            out = torch.empty_like(q)
            if t % w.refresh == 0:
                fb.fb_refresh_step(shape, q, kp, vp, kb, vb, o, m, lse, out, lse_out, ws)
            else:
                fb.fb_internal_merge(shape, q, kb, vb, o, m, lse, out, lse_out)
            torch.cuda.synchronize()
            e_out = max(e_out, float(np.abs(out.double().cpu().numpy() - want[t]["out"]).max()))
            e_Lf = max(e_Lf, float(np.abs(lse_out.double().cpu().numpy() - want[t]["lse"]).max()))
            if t % w.refresh == 0:
                got = {"o": o.double().cpu().numpy(), "m": m.double().cpu().numpy(), "lse": lse.double().cpu().numpy()}
                e_A = max(e_A, float(np.abs(orc.normalized(got) - orc.normalized(want[t]["ext"])).max()))
                e_L = max(e_L, float(np.abs(got["lse"] - want[t]["ext"]["lse"]).max()))
        res[name] = {"steps": len(steps), "max_abs_err_out": e_out, "max_abs_err_A_ext": e_A,
                     "max_abs_err_L_ext": e_L, "max_abs_err_L_full": e_Lf,
                     "tolerance": "1e-5 max-abs" if w.dtype == "f32" else "1e-2 abs + 1e-2 rel"}
        del kp, vp
        torch.cuda.empty_cache()
    res["note"] = "float64 numpy oracle on the same seeded inputs (bf16 inputs rounded before both sides)"
    return res


def cpu_baseline(w, budget_s=12.0):
    """The numpy float64 oracle, as it stands, on whole blocks of the workload's full shape."""
    import numpy as np  # noqa: F401
    from oracle import flashblock_oracle as orc
    from paper_2602_05305_amd import workloads as wl
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    Kp, Vp = wl.make_prefix(w, 1)
    steps = wl.make_block_steps(w, 1)
    n_blocks, t0 = 0, time.perf_counter()
    while True:
        orc.run_block_dense(Kp, Vp, steps, w.refresh)
        n_blocks += 1
        el = time.perf_counter() - t0
        if el >= budget_s or n_blocks >= 400:
            break
    us = el / (n_blocks * w.steps) * 1e6
    return {"value": round(us, 1), "unit": "us/step", "cores": int(threads), "kind": "oracle",
            "sample": f"{n_blocks} whole block(s) of {w.steps} diffusion steps (1 refresh + {w.steps - 1} reuse, R={w.refresh}) "
                      f"at the full {w.name} shape, numpy float64, {el:.1f} s",
            "host_cores_visible": len(os.sched_getaffinity(0))}


def _ev_median_us(torch, fn, reps=30, warm=3, warm_s=0.05):
    """(median, min) event-timed duration of fn in us over `reps` launches.  Clocks take a while to settle on a
    freshly idle GPU, so fn is first run untimed for at least warm_s seconds."""
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    n = 0
    while n < warm or time.perf_counter() - t0 < warm_s:
        fn()
        n += 1
        if n % 8 == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in evs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) for a, b in evs)
    return ts[len(ts) // 2] * 1e3, ts[0] * 1e3


def video_extra(torch, fb, wl, ceilings=None):
    """Video-shaped workload: both passes are dense contractions, priced against bf16 MFMA peak."""
    w = wl.CONFIGS["video"]
    d = DeviceBlock(w, 1)
    q, kb, vb = d.steps[0]
    t_ext, t_ext_min = _ev_median_us(torch, lambda: fb.fb_external_partial(d.shape, q, d.K[0], d.V[0], d.o, d.m, d.lse, d.ws))
    t_int, t_int_min = _ev_median_us(torch, lambda: fb.fb_internal_merge(d.shape, q, kb, vb, d.o, d.m, d.lse, d.out, None))
    hm = torch.zeros((w.batch, w.n_q_heads), device="cuda", dtype=torch.uint8)
    hm[:, ::2] = 1                       # head-wise selective refresh: every other head recomputed
    ns_h = max(fb.fb_external_heads_splits(d.shape, w.n_q_heads // 2), fb.fb_external_heads_splits(d.shape, 1), 1)
    ws_h = torch.empty(fb.fb_workspace_bytes(d.shape, 0, 0, ns_h), device="cuda", dtype=torch.uint8)
    t_half, _ = _ev_median_us(torch, lambda: fb.fb_external_partial_heads(d.shape, q, d.K[0], d.V[0], hm, d.o, d.m, d.lse,
                                                                          ws_h, w.n_q_heads // 2))
    hm1 = torch.zeros((w.batch, w.n_q_heads), device="cuda", dtype=torch.uint8)
    hm1[:, 3] = 1                        # a single unstable head
    t_one, _ = _ev_median_us(torch, lambda: fb.fb_external_partial_heads(d.shape, q, d.K[0], d.V[0], hm1, d.o, d.m, d.lse,
                                                                         ws_h, 1))
    f_ext = 4.0 * w.batch * w.n_q_heads * w.block_len * w.prefix_len * w.head_dim
    f_int = 4.0 * w.batch * w.n_q_heads * w.block_len * w.block_len * w.head_dim
    peak = 2500.0
    S, R = w.steps, w.refresh
    return {"workload": describe(w), "bound": "mfma", "peak": peak, "unit": "TFLOP/s",
            "external_us": round(t_ext, 1), "external_min_us": round(t_ext_min, 1),
            "external_tflops": round(f_ext / t_ext / 1e6, 1),
            "external_frac": round(f_ext / t_ext / 1e6 / peak, 4),
            "external_half_of_heads_us": round(t_half, 1), "external_one_head_us": round(t_one, 1),
            "internal_us": round(t_int, 1), "internal_min_us": round(t_int_min, 1),
            "internal_tflops": round(f_int / t_int / 1e6, 1),
            "internal_frac": round(f_int / t_int / 1e6 / peak, 4),
            "block_speedup_cached_vs_full": round(S * (t_ext + t_int) / (-(-S // R) * t_ext + S * t_int), 3),
            **({"measured_peak": ceilings["mfma_bf16_TFLOPs"],
                "external_frac_of_measured": round(f_ext / t_ext / 1e6 / ceilings["mfma_bf16_TFLOPs"], 4),
                "internal_frac_of_measured": round(f_int / t_int / 1e6 / ceilings["mfma_bf16_TFLOPs"], 4),
                "measured_peak_kernel": "fbc_mfma with changing operands (MFMA-only loop, this process)"} if ceilings else {}),
            "timing": "median (and min) of 30 event-timed calls after 50 ms of the same call"}


def sparse_extra(torch, fb, wl):
    """Sparse + residual reuse at the 64K prefix: selection on the GPU, refresh and reuse calls."""
    w = wl.CONFIGS["sparse_64k"]
    d = DeviceBlock(w, 2)
    nblk = -(-w.prefix_len // w.key_block)
    ws = torch.empty(fb.fb_workspace_bytes(d.shape, w.key_block, w.topk), device="cuda", dtype=torch.uint8)
    pooled = [torch.empty((w.batch, w.n_kv_heads, nblk, w.head_dim), device="cuda") for _ in range(2)]
    idx = torch.empty((w.batch, w.n_q_heads, w.topk), device="cuda", dtype=torch.int32)
    rows = (w.batch, w.n_q_heads, w.block_len)
    ro = torch.empty(rows + (w.head_dim,), device="cuda")
    rm, rl = torch.empty(rows, device="cuda"), torch.empty(rows, device="cuda")
    q = d.steps[0][0]
    i = [0]
    t_pool, t_pool_min = _ev_median_us(torch, lambda: fb.fb_pool_keys(d.shape, d.K[0], w.key_block, pooled[0]))
    fb.fb_pool_keys(d.shape, d.K[1], w.key_block, pooled[1])
    t_sel1, t_sel1_min = _ev_median_us(torch, lambda: fb.fb_select_topk(d.shape, q, pooled[0], w.key_block, w.topk, idx))
    sws = torch.empty(fb.fb_select_workspace_bytes(d.shape, w.key_block), device="cuda", dtype=torch.uint8)
    t_sel, t_sel_min = _ev_median_us(torch, lambda: fb.fb_select_topk(d.shape, q, pooled[0], w.key_block, w.topk, idx, sws))
    wsm = torch.empty(fb.fb_select_mass_workspace_bytes(d.shape, w.key_block), device="cuda", dtype=torch.uint8)
    fb.fb_external_partial(d.shape, q, d.K[0], d.V[0], d.o, d.m, d.lse, ws)
    idx_m = torch.empty_like(idx)
    t_mass, t_mass_min = _ev_median_us(torch, lambda: fb.fb_select_topk_mass(d.shape, q, d.K[i[0] % 2], d.lse, w.key_block, w.topk,
                                                                   idx_m, None, wsm))

    def call(mode):
        s = i[0] % 2
        i[0] += 1
        fb.fb_sparse_external_residual(d.shape, mode, q, d.K[s], d.V[s], w.key_block, w.topk, idx, ro, rm, rl,
                                       d.o, d.m, d.lse, ws)
    t_refresh, t_refresh_min = _ev_median_us(torch, lambda: call(fb.FB_SPARSE_REFRESH))
    t_reuse_rebuild, t_reuse_rebuild_min = _ev_median_us(torch, lambda: call(fb.FB_SPARSE_REUSE))
    # reuse steps of a block keep the refresh step's selection: no mask rebuild
    t_reuse, t_reuse_min = _ev_median_us(torch, lambda: call(fb.FB_SPARSE_REUSE_SAME_SELECTION))
    t_dense, t_dense_min = _ev_median_us(torch, lambda: fb.fb_external_partial(d.shape, q, d.K[i[0] % 2], d.V[i[0] % 2], d.o, d.m, d.lse, ws))
    sel = idx.cpu().numpy()
    G = w.n_q_heads // w.n_kv_heads
    union = sum(len(set(sel[0, kv * G:(kv + 1) * G].ravel().tolist())) for kv in range(w.n_kv_heads))
    union_bytes = union * w.key_block * w.head_dim * 2 * 2
    return {"workload": describe(w) + f", key_block {w.key_block}, topk {w.topk}",
            "pool_keys_us": round(t_pool, 1), "select_topk_us": round(t_sel, 1),
            "select_topk_without_workspace_us": round(t_sel1, 1),
            "select_topk_mass_us": round(t_mass, 1),
            "sparse_refresh_call_us": round(t_refresh, 1), "sparse_reuse_call_us": round(t_reuse, 1),
            "sparse_reuse_call_rebuilding_masks_us": round(t_reuse_rebuild, 1),
            "dense_external_call_us": round(t_dense, 1),
            "sparse_refresh_call_min_us": round(t_refresh_min, 1), "sparse_reuse_call_min_us": round(t_reuse_min, 1),
            "dense_external_call_min_us": round(t_dense_min, 1),
            "union_fraction_of_prefix": round(union / (nblk * w.n_kv_heads), 3),
            "reuse_union_bytes": union_bytes, "reuse_GBps_vs_union_bytes": round(union_bytes / t_reuse / 1e3, 1),
            "reuse_frac_of_8TBps_vs_union_bytes": round(union_bytes / t_reuse / 1e3 / HBM_PEAK_GBS, 4),
            "refresh_GBps_vs_kv_bytes": round(w.kv_bytes / t_refresh / 1e3, 1),
            "refresh_frac_of_8TBps_vs_kv_bytes": round(w.kv_bytes / t_refresh / 1e3 / HBM_PEAK_GBS, 4),
            "timing": "median (and min) of 30 event-timed calls after 50 ms of the same call"}


def paged_setup(torch, fb, wl, B=32, block_len=32, lo=512, pmax=8192, page=256, seed=5305):
    """Paged prefix cache with ragged per-sequence lengths (the serving shape): batch B, prefix lengths uniform in
    [lo, pmax] (one at the maximum), 256-token pages handed out in random order, block of block_len tokens.
    Returns the call closure and a description."""
    import numpy as np
    base = wl.CONFIGS["llm_32k"]
    rng = np.random.default_rng([2602, seed])
    lens = rng.integers(lo, pmax + 1, size=B).astype(np.int32)
    lens[0] = pmax
    need = [-(-int(n) // page) for n in lens]
    npages = sum(need) + 3
    table = np.full((B, pmax // page), -1, dtype=np.int32)
    order, nxt = rng.permutation(npages), 0
    for b in range(B):
        table[b, :need[b]] = order[nxt:nxt + need[b]]
        nxt += need[b]
    shape = fb.make_shape(B, base.n_q_heads, base.n_kv_heads, base.head_dim, block_len, pmax, "bf16")
    sc = float(base.input_scale)
    # pools above ~1 GB are not doubled: they exceed the last-level cache several times over on their own
    npools = 2 if npages * base.n_kv_heads * page * base.head_dim * 4 < (1 << 30) else 1
    pools = [tuple((torch.randn((npages, base.n_kv_heads, page, base.head_dim), device="cuda") * sc).to(torch.bfloat16)
                   for _ in range(2)) for _ in range(npools)]
    tbl, ln = torch.from_numpy(table).cuda(), torch.from_numpy(lens).cuda()
    kvs = [fb.make_paged_kv(k, v, tbl, ln) for k, v in pools]
    q = (torch.randn((B, base.n_q_heads, block_len, base.head_dim), device="cuda") * sc).to(torch.bfloat16)
    rows = (B, base.n_q_heads, block_len)
    o = torch.empty(rows + (base.head_dim,), device="cuda")
    m, l = torch.empty(rows, device="cuda"), torch.empty(rows, device="cuda")
    ns = fb.fb_paged_splits(shape)
    ws = torch.empty(fb.fb_workspace_bytes(shape, 0, 0, ns), device="cuda", dtype=torch.uint8)
    i = [0]

    def call():
        fb.fb_external_partial_paged(shape, q, kvs[i[0] % npools], o, m, l, ws)
        i[0] += 1
    kb = (torch.randn((B, base.n_kv_heads, block_len, base.head_dim), device="cuda") * sc).to(torch.bfloat16)
    vb = (torch.randn((B, base.n_kv_heads, block_len, base.head_dim), device="cuda") * sc).to(torch.bfloat16)
    out = torch.empty_like(q)

    def refresh_step():
        fb.fb_refresh_step_paged(shape, q, kvs[i[0] % npools], kb, vb, o, m, l, out, None, ws)
        i[0] += 1
    call.refresh_step = refresh_step
    call.keep = (pools, tbl, ln, q, o, m, l, ws)        # the closure's buffers live as long as it does
    kv_bytes = int(lens.sum()) * base.n_kv_heads * base.head_dim * 2 * 2
    info = {"workload": f"paged external pass: batch {B}, prefix lengths uniform {lo}..{pmax} ({int(lens.sum())} tokens), "
                        f"{page}-token pages in random order, {base.n_q_heads} q / {base.n_kv_heads} kv heads, "
                        f"head_dim {base.head_dim}, block {block_len}, bf16",
            "splits": ns, "kv_bytes": kv_bytes}
    return call, info


def paged_extra(torch, fb, wl, **kw):
    """Bandwidth of the paged external pass, priced against the K/V bytes of the tokens that exist
    (not of the padded maximum)."""
    call, info = paged_setup(torch, fb, wl, **kw)
    t, tmin = _ev_median_us(torch, call)
    t_step, t_step_min = _ev_median_us(torch, call.refresh_step)
    info.update({"external_call_us": round(t, 1), "external_call_min_us": round(tmin, 1),
                 "GBps_vs_kv_bytes": round(info["kv_bytes"] / t / 1e3, 1),
                 "frac_of_8TBps": round(info["kv_bytes"] / t / 1e3 / 8000.0, 4),
                 "refresh_step_paged_us": round(t_step, 1), "refresh_step_paged_min_us": round(t_step_min, 1)})
    del call
    torch.cuda.empty_cache()
    return info


# the paper's language-model deployment shape (Section 5 implementation details, Table 1): 128 sequences under one
# token budget of about 800k tokens, blocks of 4 or 8 tokens
PAGED_DEPLOY = dict(B=128, lo=512, pmax=12288, page=256)


def gamma_calibration(torch, fb, wl, gamma=0.85):
    """Head-wise selective reuse (Section 4.2, the video rule) end to end on synthetic drift, all on the HIP path.
    The 12 heads of the video shape drift at different rates (per-step query perturbation sigma_h from 0.02 to
    1.5).  Calibration block: the external partial is recomputed at every step and fb_head_similarity gives each
    head's cosine similarity of A_out between consecutive steps (the quantity of Figure 1); heads whose mean
    similarity exceeds gamma become reuse heads.  Evaluation block (fresh inputs): step 0 refreshes every head, the
    later steps refresh only the other heads through fb_external_partial_heads; reported are the mean L1 distance
    of the merged output to full recomputation per head class and the external-pass time per step."""
    w = wl.CONFIGS["video"]
    dt = torch.bfloat16
    H, Bq, D = w.n_q_heads, w.block_len, w.head_dim
    sig = torch.logspace(math.log10(0.02), math.log10(1.5), H, device="cuda").view(1, H, 1, 1)
    shape = fb.make_shape(w.batch, H, w.n_kv_heads, D, Bq, w.prefix_len, w.dtype)
    ws = torch.empty(fb.fb_workspace_bytes(shape), device="cuda", dtype=torch.uint8)
    rows = (w.batch, H, Bq)
    mk = lambda: (torch.empty(rows + (D,), device="cuda"), torch.empty(rows, device="cuda"), torch.empty(rows, device="cuda"))

    def block(seed):
        g = torch.Generator(device="cuda").manual_seed(seed)
        ks = (w.batch, w.n_kv_heads, w.prefix_len, D)
        K = (torch.randn(ks, device="cuda", generator=g) * w.input_scale).to(dt)
        V = (torch.randn(ks, device="cuda", generator=g) * w.input_scale).to(dt)
        q = torch.randn(rows + (D,), device="cuda", generator=g) * w.input_scale
        kb = torch.randn((w.batch, w.n_kv_heads, Bq, D), device="cuda", generator=g) * w.input_scale
        vb = torch.randn((w.batch, w.n_kv_heads, Bq, D), device="cuda", generator=g) * w.input_scale
        steps = []
        for _ in range(w.steps):
            steps.append((q.to(dt).contiguous(), kb.to(dt).contiguous(), vb.to(dt).contiguous()))
            q = steps[-1][0].float() + sig * torch.randn(q.shape, device="cuda", generator=g)
            kb = steps[-1][1].float() + w.step_sigma * torch.randn(kb.shape, device="cuda", generator=g)
            vb = steps[-1][2].float() + w.step_sigma * torch.randn(vb.shape, device="cuda", generator=g)
        return K, V, steps

    # calibration: similarity of consecutive fresh partials
    K, V, steps = block(501)
    prev, cur = mk(), mk()
    sim = torch.empty((w.batch, H), device="cuda")
    sims = []
    for t, (q, kb, vb) in enumerate(steps):
        fb.fb_external_partial(shape, q, K, V, *cur, ws)
        if t > 0:
            fb.fb_head_similarity(shape, prev[0], cur[0], sim)
            sims.append(sim.clone())
        prev, cur = cur, prev
    mean_sim = torch.stack(sims).mean(dim=0)[0]
    reuse = (mean_sim > gamma)
    n_refresh = int((~reuse).sum())
    mask = (~reuse).to(torch.uint8).view(w.batch, H).contiguous()
    wsh = torch.empty(max(fb.fb_workspace_bytes(shape, 0, 0, max(fb.fb_external_heads_splits(shape, n_refresh), 1)),
                          fb.fb_workspace_bytes(shape)), device="cuda", dtype=torch.uint8)

    # evaluation on fresh inputs
    K, V, steps = block(502)
    part, full, stale = mk(), mk(), mk()
    out_sel, out_full, out_stale = (torch.empty_like(steps[0][0]) for _ in range(3))
    err, err_stale = [], []
    for t, (q, kb, vb) in enumerate(steps):
        fb.fb_external_partial(shape, q, K, V, *full, ws)
        fb.fb_internal_merge(shape, q, kb, vb, *full, out_full)
        if t == 0:
            fb.fb_external_partial(shape, q, K, V, *part, wsh)
            fb.fb_external_partial(shape, q, K, V, *stale, wsh)      # never refreshed again: every head reused
        elif n_refresh > 0:
            fb.fb_external_partial_heads(shape, q, K, V, mask, *part, wsh, n_refresh)
        fb.fb_internal_merge(shape, q, kb, vb, *part, out_sel)
        fb.fb_internal_merge(shape, q, kb, vb, *stale, out_stale)
        if t > 0:
            err.append((out_sel.float() - out_full.float()).abs().mean(dim=(0, 2, 3)))
            err_stale.append((out_stale.float() - out_full.float()).abs().mean(dim=(0, 2, 3)))
    err = torch.stack(err).mean(dim=0)
    err_stale = torch.stack(err_stale).mean(dim=0)
    q = steps[1][0]
    t_full = _ev_median_us(torch, lambda: fb.fb_external_partial(shape, q, K, V, *full, ws), 9, 3)[0]
    t_sel = (_ev_median_us(torch, lambda: fb.fb_external_partial_heads(shape, q, K, V, mask, *part, wsh, n_refresh), 9, 3)[0]
             if n_refresh > 0 else 0.0)
    ref_scale = float(out_full.float().abs().mean())
    return {"workload": describe(w), "gamma": gamma,
            "per_step_query_sigma_by_head": [round(float(x), 3) for x in sig.view(-1)],
            "mean_similarity_by_head": [round(float(x), 4) for x in mean_sim],
            "reuse_heads": [int(i) for i in torch.nonzero(reuse).view(-1)],
            "refreshed_heads_per_reuse_step": n_refresh,
            "mean_abs_output": round(ref_scale, 5),
            "l1_to_full_recompute_reuse_heads": round(float(err[reuse].mean()) if reuse.any() else 0.0, 6),
            "l1_to_full_recompute_refreshed_heads": round(float(err[~reuse].mean()) if (~reuse).any() else 0.0, 6),
            "l1_of_those_heads_if_they_were_reused_too": round(float(err_stale[~reuse].mean()) if (~reuse).any() else 0.0, 6),
            "external_us_all_heads": round(t_full, 1), "external_us_selected_heads": round(t_sel, 1)}


def tau_policy(torch, fb, wl, n_blocks=24):
    """The dLLM refresh rule (Section 4.2: refresh the cached external partial iff the number of tokens updated
    in the step is at least tau) on a synthetic unmasking schedule, all on the HIP path, at the llm_32k shape.
    Per step a random number M_t in 0..4 of the block's 32 tokens is unmasked: their Q / K / V rows are redrawn,
    the other rows drift slightly (sigma 0.01).  For each tau the block runs with "refresh iff t == 0 or
    M_t >= tau"; reported are the fraction of refresh steps, the mean L1 distance of the step output to full
    recomputation, and the measured attention time per step (refresh steps through fb_refresh_step)."""
    w = wl.CONFIGS["llm_32k"]
    dt = torch.bfloat16
    d0 = DeviceBlock(w, 2, seed=99)
    shape, ws = d0.shape, d0.ws
    g = torch.Generator(device="cuda").manual_seed(4242)
    gcpu = torch.Generator().manual_seed(4242)
    qs = (w.batch, w.n_q_heads, w.block_len, w.head_dim)
    ks = (w.batch, w.n_kv_heads, w.block_len, w.head_dim)
    rows = (w.batch, w.n_q_heads, w.block_len)
    mk = lambda: (torch.empty(rows + (w.head_dim,), device="cuda"), torch.empty(rows, device="cuda"), torch.empty(rows, device="cuda"))
    full, part = mk(), mk()
    out_f, out_p = torch.empty(qs, device="cuda", dtype=dt), torch.empty(qs, device="cuda", dtype=dt)
    taus = [1, 2, 3, 5]           # 5 > max M_t: refresh at t = 0 only
    stats = {tau: {"refresh": 0, "steps": 0, "l1": 0.0} for tau in taus}
    blocks = []
    for blk in range(n_blocks):
        K, V = d0.K[blk % 2], d0.V[blk % 2]
        q = torch.randn(qs, device="cuda", generator=g) * w.input_scale
        kb = torch.randn(ks, device="cuda", generator=g) * w.input_scale
        vb = torch.randn(ks, device="cuda", generator=g) * w.input_scale
        sched, counts = [], []       # counts[t] = tokens updated on the way into step t
        for t in range(w.steps):
            if t == 0:
                counts.append(w.block_len)
            else:
                m_t = int(torch.randint(0, 5, (1,), generator=gcpu))
                counts.append(m_t)
                q = sched[-1][0].float() + 0.01 * w.input_scale * torch.randn(qs, device="cuda", generator=g)
                kb = sched[-1][1].float() + 0.01 * w.input_scale * torch.randn(ks, device="cuda", generator=g)
                vb = sched[-1][2].float() + 0.01 * w.input_scale * torch.randn(ks, device="cuda", generator=g)
                if m_t > 0:
                    upd = torch.randperm(w.block_len, generator=gcpu)[:m_t].to("cuda")
                    q[:, :, upd] = torch.randn((w.batch, w.n_q_heads, m_t, w.head_dim), device="cuda", generator=g) * w.input_scale
                    kb[:, :, upd] = torch.randn((w.batch, w.n_kv_heads, m_t, w.head_dim), device="cuda", generator=g) * w.input_scale
                    vb[:, :, upd] = torch.randn((w.batch, w.n_kv_heads, m_t, w.head_dim), device="cuda", generator=g) * w.input_scale
            sched.append((q.to(dt).contiguous(), kb.to(dt).contiguous(), vb.to(dt).contiguous()))
        blocks.append((K, V, sched, counts))
        fulls = []
        for t, (qt, kt, vt) in enumerate(sched):
            fb.fb_external_partial(shape, qt, K, V, *full, ws)
            fb.fb_internal_merge(shape, qt, kt, vt, *full, out_f)
            fulls.append(out_f.float().clone())
        for tau in taus:
            for t, (qt, kt, vt) in enumerate(sched):
                if t == 0 or counts[t] >= tau:
                    fb.fb_refresh_step(shape, qt, K, V, kt, vt, *part, out_p, None, ws)
                    stats[tau]["refresh"] += 1
                else:
                    fb.fb_internal_merge(shape, qt, kt, vt, *part, out_p, None)
                stats[tau]["steps"] += 1
                stats[tau]["l1"] += float((out_p.float() - fulls[t]).abs().mean())
    ref = float(sum(float(f.abs().mean()) for f in fulls) / len(fulls))

    def timed(tau):
        """All blocks' steps under the rule, launched back to back, timed as a whole (as the headline is)."""
        def run():
            for K, V, sched, counts in blocks:
                for t, (qt, kt, vt) in enumerate(sched):
                    if t == 0 or counts[t] >= tau:
                        fb.fb_refresh_step(shape, qt, K, V, kt, vt, *part, out_p, None, ws)
                    else:
                        fb.fb_internal_merge(shape, qt, kt, vt, *part, out_p, None)
        run()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            run()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (3 * n_blocks * w.steps)

    table = []
    for tau in taus + [0]:          # 0: every step refreshes (full recomputation)
        us = timed(tau)
        if tau == 0:
            table.append({"tau": "every step refreshes", "refresh_fraction": 1.0, "l1_to_full_recompute": 0.0,
                          "attention_us_per_step": round(us, 2)})
            continue
        st = stats[tau]
        table.append({"tau": tau if tau <= 4 else "never (t = 0 only)", "refresh_fraction": round(st["refresh"] / st["steps"], 3),
                      "l1_to_full_recompute": round(st["l1"] / st["steps"], 7), "attention_us_per_step": round(us, 2)})
    return {"workload": describe(w), "updated_tokens_per_step": "uniform 0..4 of 32 rows redrawn, the rest drift with sigma 0.01",
            "mean_abs_output": round(ref, 5), "by_tau": table}


def sparse_accuracy(torch, fb, wl, prefix_len=32768):
    """Synthetic analogue of the paper's Table 3: mean L1 distance to full attention on reuse steps
    of sparse attention alone vs. sparse attention + the cached residual, per attention density.
    All three outputs come from the HIP path (full attention = dense path refreshed every step)."""
    rows = []
    base = wl.CONFIGS["sparse_64k"].with_(prefix_len=prefix_len)
    nblk = -(-base.prefix_len // base.key_block)
    for density in (0.10, 0.20, 0.30, 0.40, 0.50):
        w = base.with_(topk=int(round(density * nblk)))
        d = DeviceBlock(w, 1, seed=77)
        ws = torch.empty(fb.fb_workspace_bytes(d.shape, w.key_block, w.topk), device="cuda", dtype=torch.uint8)
        pooled = torch.empty((w.batch, w.n_kv_heads, nblk, w.head_dim), device="cuda")
        idx = torch.empty((w.batch, w.n_q_heads, w.topk), device="cuda", dtype=torch.int32)
        shp = (w.batch, w.n_q_heads, w.block_len)
        mk = lambda: (torch.empty(shp + (w.head_dim,), device="cuda"), torch.empty(shp, device="cuda"), torch.empty(shp, device="cuda"))
        res, ext, full = mk(), mk(), mk()
        empty = (torch.zeros(shp + (w.head_dim,), device="cuda"), torch.full(shp, float("-inf"), device="cuda"),
                 torch.full(shp, float("-inf"), device="cuda"))
        fb.fb_pool_keys(d.shape, d.K[0], w.key_block, pooled)
        out_a, out_b, out_f = torch.empty_like(d.out), torch.empty_like(d.out), torch.empty_like(d.out)
        wsm = torch.empty(fb.fb_select_mass_workspace_bytes(d.shape, w.key_block), device="cuda", dtype=torch.uint8)
        row = {"density": density}
        for rule in ("mean_pooled_keys", "attention_mass"):
            l1_res, l1_only = [], []
            for t, (q, kb, vb) in enumerate(d.steps):
                if t == 0:
                    if rule == "mean_pooled_keys":
                        fb.fb_select_topk(d.shape, q, pooled, w.key_block, w.topk, idx)
                    else:       # mask from full attention at the block's first step
                        fb.fb_external_partial(d.shape, q, d.K[0], d.V[0], *full, ws)
                        fb.fb_select_topk_mass(d.shape, q, d.K[0], full[2], w.key_block, w.topk, idx, None, wsm)
                    fb.fb_sparse_external_residual(d.shape, fb.FB_SPARSE_REFRESH, q, d.K[0], d.V[0], w.key_block, w.topk,
                                                   idx, *res, *ext, ws)
                    continue
                fb.fb_sparse_external_residual(d.shape, fb.FB_SPARSE_REUSE, q, d.K[0], d.V[0], w.key_block, w.topk, idx,
                                               *res, *ext, ws)
                fb.fb_internal_merge(d.shape, q, kb, vb, *ext, out_a, None)
                fb.fb_sparse_external_residual(d.shape, fb.FB_SPARSE_REUSE, q, d.K[0], d.V[0], w.key_block, w.topk, idx,
                                               *empty, *ext, ws)
                fb.fb_internal_merge(d.shape, q, kb, vb, *ext, out_b, None)
                fb.fb_external_partial(d.shape, q, d.K[0], d.V[0], *full, ws)
                fb.fb_internal_merge(d.shape, q, kb, vb, *full, out_f, None)
                l1_res.append((out_a.float() - out_f.float()).abs().mean().item())
                l1_only.append((out_b.float() - out_f.float()).abs().mean().item())
            row[rule] = {"l1_sparse_only": sum(l1_only) / len(l1_only),
                         "l1_sparse_plus_cached_residual": sum(l1_res) / len(l1_res)}
        rows.append(row)
        del d
        torch.cuda.empty_cache()
    return {"workload": describe(base) + ", densities swept, two selection rules", "rows": rows}


def describe(w):
    return (f"{w.name}: batch {w.batch}, {w.n_q_heads} q heads / {w.n_kv_heads} kv heads, head_dim {w.head_dim}, "
            f"prefix {w.prefix_len}, block {w.block_len}, {w.steps} steps/block, refresh every {w.refresh}, {w.dtype}")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4000)
    ap.add_argument("--warmup", type=int, default=400)
    ap.add_argument("--workload", default="llm_32k")
    ap.add_argument("--launch", choices=["auto", "graph", "eager"], default="auto",
                    help="how steps are launched: one HIP graph per block, eagerly, or (auto) time both and report the faster")
    ap.add_argument("--no-graph", action="store_true", help="same as --launch eager")
    ap.add_argument("--split-refresh", action="store_true",
                    help="refresh steps as fb_external_partial + fb_internal_merge (3 launches) instead of "
                         "fb_refresh_step (2 launches)")
    ap.add_argument("--no-long", action="store_true", help="skip the 128K-context external-pass measurement")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-parity", action="store_true", help="skip the gpu-vs-oracle error report")
    ap.add_argument("--no-calibration", action="store_true", help="skip the read / MFMA ceiling measurement")
    ap.add_argument("--calibration-only", action="store_true",
                    help="only print the measured ceilings (pure read, copy, MFMA-only kernels); also what the "
                         "rocprofv3 summaries under profiles/ of those kernels run")
    ap.add_argument("--no-extras", action="store_true", help="skip the video-shaped (MFMA), sparse and paged measurements")
    ap.add_argument("--profile-external", type=int, default=0, metavar="N",
                    help="only run N whole blocks of the workload, eagerly (for rocprofv3), print nothing else")
    ap.add_argument("--sparse-accuracy", action="store_true",
                    help="only print the sparse-vs-full L1 table (synthetic analogue of the paper's Table 3)")
    ap.add_argument("--tau-policy", action="store_true",
                    help="only print the updated-token-count refresh rule report (synthetic unmasking schedule)")
    ap.add_argument("--gamma-calibration", action="store_true",
                    help="only print the head-wise selective-reuse report (similarity calibration on synthetic drift)")
    ap.add_argument("--profile-sparse", type=int, default=0, metavar="N",
                    help="only run N sparse refresh + reuse call pairs of the sparse_64k workload (for rocprofv3)")
    ap.add_argument("--profile-paged", type=int, default=0, metavar="N",
                    help="only run N paged external passes of the batch-32 serving shape (for rocprofv3)")
    ap.add_argument("--paged-block", type=int, default=0, metavar="BQ",
                    help="with --profile-paged: the batch-128 deployment shape with blocks of BQ tokens instead of batch 32")
    ap.add_argument("--profile-copy", type=int, default=0, metavar="N",
                    help="only run N launches of the plain copy kernel on 256 MiB (calibrates rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (the path has no multi-GPU part); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2602_05305_amd import flashblock as fb
    from paper_2602_05305_amd import workloads as wl
    fb.load_library()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    w = wl.CONFIGS[args.workload]
    if args.calibration_only:
        print(json.dumps(measure_ceilings(torch)))
        return
    if args.profile_copy > 0:
        x = torch.full((256 * 1024 * 1024,), 3, dtype=torch.uint8, device="cuda")
        y = torch.empty_like(x)
        lib = Calib().lib
        st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        for _ in range(args.profile_copy):
            if lib.fbc_copy(y.data_ptr(), x.data_ptr(), x.numel(), st) != 0:
                raise RuntimeError("fbc_copy launch failed")
        torch.cuda.synchronize()
        print(f"ran {args.profile_copy} copy kernels of {x.numel()} bytes (read {x.numel()} + write {x.numel()} per launch)")
        return
    if args.profile_paged > 0:
        if args.paged_block:
            call, info = paged_setup(torch, fb, wl, block_len=args.paged_block, **PAGED_DEPLOY)
        else:
            call, info = paged_setup(torch, fb, wl)
        for _ in range(args.profile_paged):
            call()
        torch.cuda.synchronize()
        print(f"ran {args.profile_paged} calls of {info['workload']} ({info['kv_bytes']} K/V bytes per call)")
        return
    if args.sparse_accuracy:
        print(json.dumps(sparse_accuracy(torch, fb, wl)))
        return
    if args.gamma_calibration:
        print(json.dumps(gamma_calibration(torch, fb, wl)))
        return
    if args.tau_policy:
        print(json.dumps(tau_policy(torch, fb, wl)))
        return
    if args.profile_sparse > 0:
        ws_ = wl.CONFIGS["sparse_64k"]
        d = DeviceBlock(ws_, 2)
        nblk = -(-ws_.prefix_len // ws_.key_block)
        wsb = torch.empty(fb.fb_workspace_bytes(d.shape, ws_.key_block, ws_.topk), device="cuda", dtype=torch.uint8)
        pooled = torch.empty((ws_.batch, ws_.n_kv_heads, nblk, ws_.head_dim), device="cuda")
        idx = torch.empty((ws_.batch, ws_.n_q_heads, ws_.topk), device="cuda", dtype=torch.int32)
        rows = (ws_.batch, ws_.n_q_heads, ws_.block_len)
        ro, rm, rl = torch.empty(rows + (ws_.head_dim,), device="cuda"), torch.empty(rows, device="cuda"), torch.empty(rows, device="cuda")
        q = d.steps[0][0]
        sws = torch.empty(fb.fb_select_workspace_bytes(d.shape, ws_.key_block), device="cuda", dtype=torch.uint8)
        for i in range(args.profile_sparse):
            s_ = i % 2
            fb.fb_pool_keys(d.shape, d.K[s_], ws_.key_block, pooled)
            fb.fb_select_topk(d.shape, q, pooled, ws_.key_block, ws_.topk, idx, sws)
            for mode in (fb.FB_SPARSE_REFRESH, fb.FB_SPARSE_REUSE):
                fb.fb_sparse_external_residual(d.shape, mode, q, d.K[s_], d.V[s_], ws_.key_block, ws_.topk, idx,
                                               ro, rm, rl, d.o, d.m, d.lse, wsb)
        torch.cuda.synchronize()
        print(f"ran {args.profile_sparse} sparse refresh+reuse pairs of {ws_.name}")
        return
    if args.profile_external > 0:
        # the same loop as the event-timed pass of the benchmark: whole blocks, one refresh step and
        # steps-1 reuse steps each, K/V sets rotated per block
        d = DeviceBlock(w, max(2, min(4, int(-(-600e6 // w.kv_bytes)))), fused=not args.split_refresh)
        for b in range(args.profile_external):
            for t in range(w.steps):
                d.step(t, b % d.nsets, w.refresh)
        torch.cuda.synchronize()
        print(f"ran {args.profile_external} blocks of {w.steps} steps of {w.name}")
        return
    K, W = args.steps, args.warmup
    nsets = max(2, min(4, int(-(-600e6 // w.kv_bytes))))     # working set well beyond the last-level cache
    fused = not args.split_refresh
    ceilings = None if args.no_calibration else measure_ceilings(torch)
    dev = DeviceBlock(w, nsets, fused=fused)

    # Exactly K steps per repeat after W warm-up steps, in both launch modes unless one is forced; the faster one
    # is the reported value (the other is listed in steps_detail).
    modes = {"graph": [True], "eager": [False], "auto": [True, False]}["eager" if args.no_graph else args.launch]
    timed = {g: time_steps(dev, K, W, w.refresh, g) for g in modes}
    use_graph = min(timed, key=lambda g: timed[g]["us"])
    tm = timed[use_graph]
    us_step = tm["us"]
    full = time_steps(dev, K, W, 1, use_graph)               # full recomputation: refresh on every step
    us_full = full["us"]
    prof = profile_external(dev, 40, w.refresh)

    traffic = read_traffic(w.name)
    line = {
        "metric": "attention us per diffusion step (cached block-external attention, 32K context); "
                  "external-pass HBM GB/s in roofline / external_128k",
        "value": round(us_step, 3), "unit": "us/step", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(us_step / 1e3, 6), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": describe(w), "kv_buffer_sets_rotated": nsets,
                   "launch": "one HIP graph per block" if use_graph else "eager",
                   "refresh_step": "fb_refresh_step (2 launches)" if fused else "fb_external_partial + fb_internal_merge (3 launches)",
                   "external_splits": fb.fb_external_splits(dev.shape)},
        "timing": {"protocol": f"{W} warm-up steps and >= {WARM_SECONDS} s of the same work, then {tm['repeats']} back-to-back "
                               f"repeats of exactly {K} steps, each between two events on the stream; value = median over repeats",
                   "repeats": tm["repeats"], "us_per_step_min_over_repeats": round(tm["us_min"], 3),
                   "wall_clock_us_per_step_over_all_repeats": round(tm["wall_us"], 3)},
        "roofline": roofline_obj(w, prof, traffic, fused, ceilings),
        "steps_detail": {"refresh_step_us": round(prof["refresh_step_us"], 2),
                         "reuse_step_us": round(prof["reuse_step_us"], 2),
                         "external_attn_kernel_us": round(prof["attn_us"], 2),
                         ("refresh_fold_kernel_us (split fold + block-internal attention + merge)" if fused
                          else "external_combine_kernel_us"): round(prof["combine_us"], 2),
                         "us_per_step_by_launch_mode": {("hip_graph_per_block" if g else "eager"): round(t["us"], 3)
                                                        for g, t in timed.items()}},
        "full_recompute": {"us_per_step": round(us_full, 3), "speedup_cached_vs_full": round(us_full / us_step, 3),
                           "note": "same kernels with refresh interval 1"},
    }
    if ceilings is not None:
        line["calibration"] = ceilings
    # the same external pass with the prefix resident in the last-level cache (one K/V set, never rotated)
    dev_warm = DeviceBlock(w, 1, fused=fused)
    pw = profile_external(dev_warm, 32, w.refresh)
    line["steps_detail"]["external_attn_kernel_us_prefix_in_llc"] = round(pw["attn_us"], 2)
    del dev_warm, dev
    torch.cuda.empty_cache()

    if not args.no_long:
        wl128 = wl.CONFIGS["long_128k"]
        d2 = DeviceBlock(wl128, 2, fused=fused)
        p2 = profile_external(d2, 32, wl128.refresh)
        r2 = roofline_obj(wl128, p2, read_traffic(wl128.name), fused, ceilings)
        r2["workload"] = describe(wl128)
        r2["external_call_us"] = round(p2["attn_us_median"] + p2["combine_us"], 2)
        r2["refresh_step_us"] = round(p2["refresh_step_us"], 2)
        r2["reuse_step_us"] = round(p2["reuse_step_us"], 2)
        # refresh-interval sweep (speedup of caching against full recomputation = R 1), eager launches
        sweep = {}
        for R in (1, 2, 4, 8):
            sweep[f"R={R}"] = round(time_steps(d2, 5 * wl128.steps, wl128.steps, R, False, target_s=0.04)["us"], 2)
        r2["us_per_step_by_refresh_interval"] = sweep
        r2["speedup_R8_vs_R1"] = round(sweep["R=1"] / sweep["R=8"], 3)
        line["external_128k"] = r2
        del d2
        torch.cuda.empty_cache()
        # batch 4 at the same context length (2.1 GB of K/V per pass)
        w4 = wl.CONFIGS["long_128k_b4"]
        d4 = DeviceBlock(w4, 2, fused=fused)
        p4 = profile_external(d4, 32, w4.refresh)
        r4 = roofline_obj(w4, p4, None, fused, ceilings)
        r4["workload"] = describe(w4)
        r4["refresh_step_us"] = round(p4["refresh_step_us"], 2)
        line["external_128k_batch4"] = r4
        del d4
        torch.cuda.empty_cache()

    if not args.no_extras:
        line["video_mfma"] = video_extra(torch, fb, wl, ceilings)
        torch.cuda.empty_cache()
        line["sparse_64k"] = sparse_extra(torch, fb, wl)
        torch.cuda.empty_cache()
        line["paged_b32"] = paged_extra(torch, fb, wl)
        line["paged_b128_block4"] = paged_extra(torch, fb, wl, block_len=4, **PAGED_DEPLOY)
        line["paged_b128_block8"] = paged_extra(torch, fb, wl, block_len=8, **PAGED_DEPLOY)
        torch.cuda.empty_cache()

    if not args.no_extras:
        # the tiny fp32 configuration: launch-bound, reported for completeness
        wt = wl.CONFIGS["tiny_f32"]
        dt_ = DeviceBlock(wt, 2, fused=fused)
        nt = 50 * wt.steps
        line["tiny_f32"] = {"workload": describe(wt), "us_per_step": round(time_steps(dt_, nt, wt.steps, wt.refresh, False, target_s=0.03)["us"], 2),
                            "note": "launch-bound: a roofline fraction is not meaningful at this size"}
        del dt_

    if not args.no_parity:
        line["parity"] = parity_obj(torch, fb, wl)
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(line))


if __name__ == "__main__":
    main()

#!/usr/bin/env python3
"""Benchmark of the segmented multi-LoRA hot path on one MI355X.

Headline (`value`, `roofline`, `cpu_baseline`): the forward of the 8B-shaped 32-layer stack, the largest
configuration: a step = segment-metadata builder + the forward of the 224 LoRA linears
(7 projections x 32 layers; shrink, h-save, expand in one launch per call, the library choosing between its two
one-launch kernels call by call; q, k, v and gate, up as grouped calls
that read their common x once, so 4 launches per layer) over one mixed batch of 5632 tokens; `value` = tokens of
the batch / step time.  `configs` carries the single-call workloads (a step = builder + forward,
operands rotated over > 1 GiB of replicas) and the layer stack's backward.  Inputs are synthetic, resident in HBM
before the timed region, and no two calls share an operand, so that nothing the accounting counts is served from L2
or the Infinity Cache.

`roofline` is the HBM roofline of the dominant kernel: algorithmic bytes per launch / that kernel's average launch
duration, taken from the dispatches' own start and end time stamps (HIP events on the launch stream, see
lora_profile_enable); `traffic` is read from the committed rocprofv3 counter summary under profiles/.
`cpu_baseline` is the fp64 oracle on the host cores on a bounded sample.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published
METRIC = "segmented multi-LoRA fwd: tokens/s, HBM GB/s & MFMA util vs peak (1 MI355X)"


def algorithmic_work(p):
    """Bytes the method must move and flops it must do for one call:
    x once, y read + write, A and B of every adapter in use once, saved h once; 2 r (d_in + d_out) flops/token."""
    import numpy as np
    ta, tk = p.batch.token_adapter, p.batch.token_kind
    live = (ta >= 0) & (ta < p.n_adapters) & (tk <= 2)
    used = np.unique(ta[live])
    r_tok = p.ranks[ta[live]].astype(np.int64)
    n_live = int(live.sum())
    ft = live & (tk == 0)
    bytes_x = n_live * p.d_in * 2
    bytes_y = n_live * p.d_out * 4
    bytes_A = int(sum(int(p.ranks[a]) * p.d_in * 2 for a in used))
    bytes_B = int(sum(int(p.ranks[a]) * p.d_out * 2 for a in used))
    bytes_h = int(p.ranks[ta[ft]].astype(np.int64).sum()) * 4
    flops = int((2 * r_tok * (p.d_in + p.d_out)).sum())
    return dict(shrink=bytes_x + bytes_A, expand=bytes_y + bytes_B + bytes_h,
                total=bytes_x + bytes_y + bytes_A + bytes_B + bytes_h, flops=flops, tokens=n_live)


class Replicas:
    """Device copies of one problem, rotated step by step so that operands come from HBM."""

    def __init__(self, p, variant, min_total_bytes=int(1.25 * 2 ** 30), max_replicas=64):
        import torch
        from paper_2511_00101_amd import binding as lq
        self.lq, self.torch, self.p, self.variant = lq, torch, p, variant
        per = p.x.nbytes + p.y0.nbytes + sum(a.nbytes for a in p.A) + sum(b.nbytes for b in p.B)
        self.n = int(min(max_replicas, max(2, -(-min_total_bytes // per))))
        dev = "cuda"
        x0, y0 = lq.bf16_from_bits(p.x, dev), lq.bf16_from_bits(p.y0, dev)
        A0 = [lq.bf16_from_bits(a, dev) for a in p.A]
        B0 = [lq.bf16_from_bits(b, dev) for b in p.B]
        self.x = [x0] + [x0.clone() for _ in range(self.n - 1)]
        self.y = [y0] + [y0.clone() for _ in range(self.n - 1)]
        self.ad = [lq.AdapterTable.from_tensors([a.clone() for a in A0], [b.clone() for b in B0], p.scales, dev)
                   for _ in range(self.n)]
        self.ta = torch.from_numpy(p.batch.token_adapter).to(dev)
        self.tk = torch.from_numpy(p.batch.token_kind).to(dev)
        self.seg = lq.SegmentTables.empty(p.n_tokens, p.n_adapters, dev)
        self.bws = lq.workspace(lq.lora_build_workspace_bytes(p.n_tokens, p.n_adapters), dev)
        self.fws = lq.workspace(lq.lora_forward_workspace_bytes(p.n_tokens, self.ad[0].max_rank, p.d_in, p.d_out, variant), dev)
        lq.lora_build_segments(self.ta, self.tk, self.ad[0].ranks, self.seg, self.bws)
        h_elems = int(self.seg.h_offsets.max().item())
        self.h_out = torch.zeros(max(h_elems, 1), dtype=torch.float32, device=dev)
        self.prepare()

    def build(self, i):
        self.lq.lora_build_segments(self.ta, self.tk, self.ad[i % self.n].ranks, self.seg, self.bws)

    def forward(self, i, variant=None):
        r = i % self.n
        self.lq.lora_segmented_forward(self.x[r], self.y[r], self.ad[r], self.seg, self.h_out, self.fws,
                                       self.variant if variant is None else variant)

    def prepare(self):
        """The step's two calls with their arguments marshalled once per replica, so that the host keeps ahead of
        a 20-microsecond step."""
        lq = self.lq
        self.calls = [(lq.prepare_build_segments(self.ta, self.tk, self.ad[r].ranks, self.seg, self.bws),
                       lq.prepare_forward(self.x[r], self.y[r], self.ad[r], self.seg, self.h_out, self.fws, self.variant))
                      for r in range(self.n)]

    def step(self, i):
        build, forward = self.calls[i % self.n]
        build()
        forward()


PROFILE_FILES = dict(cfg2_decode_heavy="forward_cfg2_decode_heavy.txt", cfg3_unified="forward_cfg3_unified.txt",
                     cfg4_mlp_up="forward_cfg4_mlp_up.txt", cfg4_mlp_down="forward_cfg4_mlp_down.txt",
                     cfg5_layer_stack="forward_cfg5_layer_stack.txt",
                     cfg5_layer_stack_single_calls="forward_cfg5_layer_stack_single_calls.txt")


def traffic_source(workload):
    """Where roofline.traffic comes from: counters need rocprofv3, so the figure is the one of the committed
    summary of this workload (it goes stale when a kernel changes; the summary names its command)."""
    name = PROFILE_FILES.get(workload)
    return f"profiles/{name} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by profiles/copy_calibration.txt)" if name else None


def counter_traffic(workload, phase):
    """HBM bytes per launch of `phase` from the committed rocprofv3 counter summary of this workload
    (profiles/, FETCH_SIZE and WRITE_SIZE scaled by the copy calibration), or None."""
    name = PROFILE_FILES.get(workload)
    path = os.path.join(ROOT, "profiles", name) if name else None
    if not path or not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) == 3 and f[0] == "traffic_bytes_per_launch" and (f[1] == phase or (phase in ONE_LAUNCH and (f[1] == "forward" or f[1] in ONE_LAUNCH))):
            return int(f[2])
    return None


def measure(p, variant, steps, warmup):
    """One single-call workload: a step = segment builder + forward."""
    import torch
    work = algorithmic_work(p)
    rep = Replicas(p, variant)
    s_per_step, per_step = timed_steps(torch, rep.step, steps, warmup)
    kern = profiled(rep.lq, torch, lambda: [rep.step(warmup + i) for i in range(steps)])
    fwd_names = [k for k in kern if k != "build"]
    fwd_us = sum(kern[k]["avg_us"] for k in fwd_names)
    one = [k for k in ONE_LAUNCH if k in kern]
    if one:
        dom, dom_bytes = one[0], work["total"]
    else:
        dom = "expand" if work["expand"] >= work["shrink"] else "shrink"
        dom_bytes = work[dom]
    dom_gbps = dom_bytes / (kern[dom]["avg_us"] * 1e-6) / 1e9
    traffic = counter_traffic(p.name, dom)
    res = dict(
        workload=p.name, tokens=work["tokens"], d_in=p.d_in, d_out=p.d_out, replicas=rep.n, steps=steps,
        ms_per_step=s_per_step * 1e3, per_step=per_step, tokens_per_s=work["tokens"] / s_per_step,
        forward_us=fwd_us, forward_gbps=work["total"] / (fwd_us * 1e-6) / 1e9,
        forward_tflops=work["flops"] / (fwd_us * 1e-6) / 1e12,
        forward_hbm_frac=work["total"] / (fwd_us * 1e-6) / 1e9 / HBM_PEAK_GBPS,
        forward_mfma_frac=work["flops"] / (fwd_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        algorithmic_bytes=work["total"], flops=work["flops"], kernels=kern,
        roofline=dict(bound="hbm", kernel=dom, achieved=dom_gbps, peak=HBM_PEAK_GBPS, unit="GB/s",
                      frac=dom_gbps / HBM_PEAK_GBPS, traffic=traffic, traffic_source=traffic_source(p.name) if traffic else None,
                      algorithmic_bytes=dom_bytes, avg_launch_us=kern[dom]["avg_us"]),
        error_word=int(rep.fws[0].item() & 0xffffffff) | int(rep.bws[0].item() & 0xffffffff))
    del rep
    return res


LAYER_STACK_NAME = "cfg5_layer_stack"
ONE_LAUNCH = ("forward_fused", "forward_slab")   # kernel names of the variants that run a forward as one launch


class LayerStack:
    """The 8B-shaped 32-layer stack: 7 LoRA linears per layer with their own adapter
    weights, one batch structure for all 224.  grouped: q, k, v read one x and gate, up read one x, as in a real
    decoder layer (Algorithm 1), and each such group is one lora_segmented_forward_group call; x is then counted
    once per group.  Not grouped: one call per linear, and every call has its OWN x.  Either way no two launches share an
    operand, so no byte that the accounting counts can come from the Infinity Cache left there by a neighbouring launch.
    Activations and weights are drawn on the GPU with torch's generator (same distributions as the seeded
    generators; the parity tests run the seeded ones on sampled calls and groups, this loop is timed, not checked)."""

    GROUPS = ((0, 1, 2), (3,), (4, 5), (6,))   # q+k+v read one x, o its own, gate+up one x, down its own (Algorithm 1; the MLP)

    def __init__(self, variant, with_backward, grouped=True, n_layers=None):
        import numpy as np
        import torch
        from paper_2511_00101_amd import binding as lq
        from paper_2511_00101_amd import synth
        self.lq, self.torch, self.variant, self.with_backward, self.grouped = lq, torch, variant, with_backward, grouped
        self.n_layers = n_layers or synth.N_LAYERS
        dev = "cuda"
        b = synth.config5_batch()
        self.batch = b
        T = b.n_tokens
        self.T = T
        n_ad, r = 16, 32
        self.n_adapters, self.rank = n_ad, r
        gen = torch.Generator(device=dev).manual_seed(5000)
        bf = torch.bfloat16

        def act(cols):
            return torch.randn(T, cols, generator=gen, device=dev, dtype=torch.float32).to(bf)

        self.ta = torch.from_numpy(b.token_adapter).to(dev)
        self.tk = torch.from_numpy(b.token_kind).to(dev)
        self.seg = lq.SegmentTables.empty(T, n_ad, dev)
        self.bws = lq.workspace(lq.lora_build_workspace_bytes(T, n_ad), dev)
        self.calls = []
        max_ws = 0
        for layer in range(self.n_layers):
            shared_x = {}
            for pi, (name, d_in, d_out) in enumerate(synth.LAYER_PROJECTIONS):
                A = [(torch.randn(r, d_in, generator=gen, device=dev) * 0.02).to(bf) for _ in range(n_ad)]
                B = [(torch.randn(r, d_out, generator=gen, device=dev) * 0.02).to(bf) for _ in range(n_ad)]
                ad = lq.AdapterTable.from_tensors(A, B, [2.0] * n_ad, dev)
                # grouped: the projections of a group read the group's x; else every call has its own
                gi = [g for g in self.GROUPS if pi in g][0]
                if not grouped or gi not in shared_x:
                    shared_x[gi] = act(d_in)
                c = dict(name=name, x=shared_x[gi], y=act(d_out), ad=ad, d_in=d_in, d_out=d_out,  # y: y0; later it doubles as dy
                         h_out=torch.zeros(4096 * r, dtype=torch.float32, device=dev))
                if with_backward:
                    c["dx"] = act(d_in)
                    c["dA"] = [torch.zeros(r, d_in, device=dev) if a < 2 else None for a in range(n_ad)]
                    c["dB"] = [torch.zeros(r, d_out, device=dev) if a < 2 else None for a in range(n_ad)]
                    c["dA_ptrs"] = torch.tensor([t.data_ptr() if t is not None else 0 for t in c["dA"]], dtype=torch.int64, device=dev)
                    c["dB_ptrs"] = torch.tensor([t.data_ptr() if t is not None else 0 for t in c["dB"]], dtype=torch.int64, device=dev)
                self.calls.append(c)
                max_ws = max(max_ws, lq.lora_workspace_bytes(T, n_ad, r, d_in, d_out) if with_backward
                             else lq.lora_forward_workspace_bytes(T, r, d_in, d_out, variant),
                             lq.lora_forward_group_workspace_bytes(lq.LQ_MAX_GROUP, T, r))
        self.ws = lq.workspace(max_ws, dev)
        self.ranks = self.calls[0]["ad"].ranks
        self.build = lq.prepare_build_segments(self.ta, self.tk, self.ranks, self.seg, self.bws)
        if grouped:
            self.fwd = []
            for base in range(0, len(self.calls), len(synth.LAYER_PROJECTIONS)):
                for g in self.GROUPS:
                    cs = [self.calls[base + pi] for pi in g]
                    self.fwd.append(lq.prepare_forward_group(cs[0]["x"], [c["y"] for c in cs], [c["ad"] for c in cs], self.seg,
                                                             [c["h_out"] for c in cs], self.ws, variant))
        else:
            self.fwd = [lq.prepare_forward(c["x"], c["y"], c["ad"], self.seg, c["h_out"], self.ws, variant) for c in self.calls]
        self.build()
        torch.cuda.synchronize()

    def work(self):
        """Algorithmic bytes / flops: forward of all calls, and backward of the fine-tune rows of all calls."""
        b = self.batch
        n_live, n_ft = b.n_tokens, int((b.token_kind == 0).sum())
        r, used, used_ft = self.rank, self.n_adapters, 2
        fwd_b = bwd_b = fwd_f = bwd_f = 0
        seen_x = set()
        for c in self.calls:
            di, do = c["d_in"], c["d_out"]
            # (x is counted once per tensor: the projections of a grouped call read it together)
            fwd_b += (0 if c["x"].data_ptr() in seen_x else n_live * di * 2) + n_live * do * 4 + used * r * (di + do) * 2 + n_ft * r * 4
            seen_x.add(c["x"].data_ptr())
            fwd_f += 2 * r * (di + do) * n_live
            # backward: dy and x of the fine-tune rows read once, dx read + written, A and B of the fine-tune adapters,
            # dA and dB read + written, the saved h read
            bwd_b += n_ft * do * 2 + n_ft * di * 2 + n_ft * di * 4 + used_ft * r * (di + do) * 2 + used_ft * r * (di + do) * 8 + n_ft * r * 4
            bwd_f += 2 * r * (di + do) * n_ft * 2
        return dict(fwd_bytes=fwd_b, bwd_bytes=bwd_b, fwd_flops=fwd_f, bwd_flops=bwd_f, tokens=n_live, calls=len(self.calls),
                    launches=len(self.fwd))

    def step(self, i=0):
        """Headline step: the segment builder once (all calls share the batch structure), then every call's forward."""
        self.build()
        for f in self.fwd:
            f()

    def backward_only(self):
        lq = self.lq
        for c in reversed(self.calls):
            lq.lora_segmented_backward(c["x"], c["y"], c["dx"], c["ad"], c["dA_ptrs"], c["dB_ptrs"], self.seg, c["h_out"],
                                       self.ws, self.variant)

    def error_word(self):
        return int(self.ws[0].item() & 0xffffffff) | int(self.bws[0].item() & 0xffffffff)


def timed_steps(torch, step, steps, warmup):
    """Exactly `steps` steps between two synchronisations (wall clock), after `warmup` untimed ones; an event after
    every step gives the per-step times as well (their median does not depend on a single slow step)."""
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(steps):
        step(warmup + i)
        ev[i + 1].record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / steps
    per = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(steps))
    return wall, dict(median_ms=per[len(per) // 2], min_ms=per[0], max_ms=per[-1])


def profiled(lq, torch, run):
    """Per-kernel average durations of `run()` from the dispatch time stamps (lora_profile_*)."""
    lq.lora_profile_enable(True)
    run()
    torch.cuda.synchronize()
    prof = lq.lora_profile_read()
    lq.lora_profile_enable(False)
    return {name: dict(avg_us=total / n, launches=n) for name, (total, n) in prof.items() if n}


def measure_layer_stack(variant, steps, warmup, with_backward, grouped=True):
    """Headline: builder + the forward of the 224 linear layers.  grouped: the projections that read the same x
    (q, k, v; gate, up) go through lora_segmented_forward_group, 4 launches per decoder layer; else 7 single calls.
    With `with_backward`, the backward of the fine-tune rows of all calls is measured as well (its own entry)."""
    import torch
    st = LayerStack(variant, with_backward, grouped)
    w = st.work()
    s_per_step, per_step = timed_steps(torch, st.step, steps, warmup)
    kern = profiled(st.lq, torch, lambda: [st.step(i) for i in range(max(1, min(steps, 3)))])
    n_steps_prof = max(1, min(steps, 3))
    fwd_us = sum(k["avg_us"] * k["launches"] for name, k in kern.items() if name != "build") / n_steps_prof   # per step
    per_launch = w["fwd_bytes"] / w["launches"]
    one = [k for k in ONE_LAUNCH if k in kern]
    if one:
        # one launch per call (LQ_VARIANT_AUTO picks the slab or the fused kernel call by call): bytes and duration
        # are averages over all the step's forward launches
        dom, dom_bytes = " + ".join(one), per_launch
        dom_us = sum(kern[k]["avg_us"] * kern[k]["launches"] for k in one) / sum(kern[k]["launches"] for k in one)
    else:   # two launches: the expand kernel carries y, B and the saved h
        n_ft = int((st.batch.token_kind == 0).sum())
        dom = "expand"
        dom_bytes = sum(st.T * c["d_out"] * 4 + st.n_adapters * st.rank * c["d_out"] * 2 + n_ft * st.rank * 4 for c in st.calls) / w["launches"]
        dom_us = kern[dom]["avg_us"]
    dom_gbps = dom_bytes / (dom_us * 1e-6) / 1e9
    name = LAYER_STACK_NAME if grouped else LAYER_STACK_NAME + "_single_calls"
    traffic = counter_traffic(name, one[0] if one else dom)
    head = dict(
        workload=name, tokens=w["tokens"], calls=w["calls"], launches=w["launches"], ms_per_step=s_per_step * 1e3, per_step=per_step,
        tokens_per_s=w["tokens"] / s_per_step, forward_us=fwd_us,
        forward_gbps=w["fwd_bytes"] / (fwd_us * 1e-6) / 1e9, forward_tflops=w["fwd_flops"] / (fwd_us * 1e-6) / 1e12,
        forward_hbm_frac=w["fwd_bytes"] / (fwd_us * 1e-6) / 1e9 / HBM_PEAK_GBPS,
        forward_mfma_frac=w["fwd_flops"] / (fwd_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        algorithmic_bytes=w["fwd_bytes"], flops=w["fwd_flops"], kernels=kern,
        roofline=dict(bound="hbm", kernel=dom, achieved=dom_gbps, peak=HBM_PEAK_GBPS, unit="GB/s", frac=dom_gbps / HBM_PEAK_GBPS,
                      traffic=traffic, traffic_source=traffic_source(name) if traffic else None,
                      algorithmic_bytes=dom_bytes, avg_launch_us=dom_us,
                      note=f"average over the step's {w['launches']} launches of 4 shapes: bytes and duration are both per launch"),
        error_word=st.error_word())
    bwd = None
    if with_backward:
        st.backward_only()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        reps = 3
        ev[0].record()
        for _ in range(reps):
            st.backward_only()
        ev[1].record()
        torch.cuda.synchronize()
        bwd_ms = ev[0].elapsed_time(ev[1]) / reps
        bk = profiled(st.lq, torch, st.backward_only)
        bdom = max(bk, key=lambda k: bk[k]["avg_us"] * bk[k]["launches"])
        kernel_us = sum(k["avg_us"] * k["launches"] for k in bk.values())
        # the backward's launches form one pipeline over the same bytes: its roofline entry is the whole call
        # (algorithmic bytes of a call / summed duration of its launches)
        per_call_us = kernel_us / w["calls"]
        gbps = w["bwd_bytes"] / w["calls"] / (per_call_us * 1e-6) / 1e9
        bwd = dict(workload=LAYER_STACK_NAME + "_backward (fine-tune rows of all 224 calls)", tokens=int((st.batch.token_kind == 0).sum()),
                   calls=w["calls"], ms_per_step=bwd_ms, backward_gbps=w["bwd_bytes"] / (bwd_ms * 1e-3) / 1e9,
                   backward_tflops=w["bwd_flops"] / (bwd_ms * 1e-3) / 1e12,
                   backward_hbm_frac=w["bwd_bytes"] / (bwd_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                   algorithmic_bytes=w["bwd_bytes"], flops=w["bwd_flops"], kernels=bk,
                   roofline=dict(bound="hbm", kernel="all launches of a call (largest: %s)" % bdom, achieved=gbps, peak=HBM_PEAK_GBPS,
                                 unit="GB/s", frac=gbps / HBM_PEAK_GBPS, traffic=None, algorithmic_bytes=w["bwd_bytes"] / w["calls"],
                                 avg_launch_us=per_call_us),
                   error_word=st.error_word())
    del st
    return head, bwd


def layer_stack_cpu_baseline(budget_s=12.0):
    """The fp64 oracle, as it stands, on the host cores, on a bounded sample of the headline workload: the seven
    calls of layer 0 (seeded inputs), repeated for ~budget_s; scaled to the 32 layers of a step."""
    import oracle
    from paper_2511_00101_amd import synth
    oracle.build()
    problems = [synth.config5(0, pi, with_dy=False) for pi in range(len(synth.LAYER_PROJECTIONS))]
    n, t0 = 0, time.perf_counter()
    while True:
        for p in problems:
            oracle.forward(p.x, p.y0, p.A, p.B, p.ranks, p.scales, p.batch.token_adapter, p.batch.token_kind)
        n += 1
        el = time.perf_counter() - t0
        if el >= budget_s:
            break
    per_layer = el / n
    T = problems[0].n_tokens
    return dict(value=T / (per_layer * synth.N_LAYERS), unit="tokens/s", cores=oracle.num_threads(), kind="oracle",
                sample=f"the 7 forward calls of layer 0 ({T} tokens each, metadata + forward), {n} times in {el:.1f} s; "
                       f"one layer takes {per_layer:.2f} s, scaled by the {synth.N_LAYERS} layers of a step")


def cpu_baseline(p, budget_s=12.0):
    """The fp64 oracle, as it stands, on the host cores: repeated whole-batch forwards for ~budget_s."""
    import oracle
    oracle.build()
    n, t0 = 0, time.perf_counter()
    while True:
        oracle.forward(p.x, p.y0, p.A, p.B, p.ranks, p.scales, p.batch.token_adapter, p.batch.token_kind)
        n += 1
        el = time.perf_counter() - t0
        if el >= budget_s or n >= 10000:
            break
    return dict(value=n * p.n_tokens / el, unit="tokens/s", cores=oracle.num_threads(), kind="oracle",
                sample=f"{n} whole-batch forwards of {p.name} ({p.n_tokens} tokens each, metadata + forward) in {el:.1f} s")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--variant", choices=["auto", "split", "fused", "slab"], default="auto",
                    help="auto: LQ_VARIANT_AUTO, one launch per call (the library picks the slab or the fused kernel); slab, fused: "
                         "that one-launch variant for every call; split: two launches, with the shrink / expand breakdown")
    ap.add_argument("--workload", default="cfg5",
                    help="headline workload: cfg5 (the 32-layer stack's forward, the largest configuration), or one of the "
                         "single-call ones cfg1, cfg2, cfg3, cfg4up, cfg4down")
    ap.add_argument("--others", default="cfg2,cfg3,cfg4up,cfg4down,cfg5single,cfg5bwd",
                    help="comma list of further workloads for the `configs` list ('' = none); cfg5single: the layer stack as 224 "
                         "single calls; cfg5bwd: the layer stack's backward")
    ap.add_argument("--single-calls", action="store_true",
                    help="headline cfg5 with one call per linear layer (224 launches) instead of grouped calls (128 launches)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain device copy of known size (256 MiB read + 256 MiB written, 8 times) so that "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings can be scaled to bytes")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU's throughput; --gpus must be 1 "
              "(the path shards by token segments with no exchange between GPUs; nothing here uses a second one)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2511_00101_amd import binding as lq
    from paper_2511_00101_amd import synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    lq.lib()
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.ones(256 * 2 ** 20, dtype=torch.uint8, device="cuda")
        dst = torch.zeros_like(src)
        for _ in range(8):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps(dict(copy_bytes_read=src.numel(), copy_bytes_written=dst.numel(), copies=8)))
        return
    variant = dict(split=lq.LQ_VARIANT_SPLIT, slab=lq.LQ_VARIANT_SLAB, fused=lq.LQ_VARIANT_FUSED)[args.variant] if args.variant != "auto" \
        else lq.LQ_VARIANT_AUTO
    makers = dict(cfg1=synth.config1, cfg2=synth.config2, cfg3=synth.config3,
                  cfg4up=lambda: synth.config4("up"), cfg4down=lambda: synth.config4("down"))
    # single-call workloads take microseconds per step: they are timed over more steps than a layer-stack step needs
    small_steps = dict(cfg1=400, cfg2=400, cfg3=200, cfg4up=80, cfg4down=80)
    other_names = [n for n in args.others.split(",") if n and n != args.workload]

    others = []
    if args.workload == "cfg5":
        head, bwd = measure_layer_stack(variant, args.steps, args.warmup, with_backward="cfg5bwd" in other_names,
                                        grouped=not args.single_calls)
        cpu = None if args.no_cpu_baseline else layer_stack_cpu_baseline()
        workload = (f"{head['workload']} forward: 32 layers x 7 LoRA linears = {head['calls']} (q,o 4096->4096; k,v 4096->1024; "
                    f"gate,up 4096->14336; down 14336->4096), {head['tokens']} tokens (4096 fine-tune + 1024 prefill + 512 decode), "
                    f"16 adapters rank 32")
        step = (f"segment builder + the forward of the {head['calls']} linears in {head['launches']} launches "
                + ("(q,k,v and gate,up as grouped calls that read their x once; o and down single)" if not args.single_calls
                   else "(one call per linear)") + "; the calls share the batch structure, so the tables are built once")
        extra = dict(calls=head["calls"], launches=head["launches"],
                     inputs="drawn on the GPU by torch's generator, every call (group) with its own x, y and weights; "
                            "timed, not checked (the parity tests check sampled calls and groups with the seeded generators)")
        if bwd:
            others.append(bwd)
    else:
        p = makers[args.workload]()
        head = measure(p, variant, max(args.steps, small_steps[args.workload]), max(args.warmup, 10))
        cpu = None if args.no_cpu_baseline else cpu_baseline(p)
        workload = f"{head['workload']}: {head['tokens']} tokens, {head['d_in']}->{head['d_out']}, {p.n_adapters} adapters rank {int(p.ranks.max())}"
        step = "segment builder + forward"
        extra = dict(replicas=head["replicas"], timed_steps=head["steps"])
        del p
    for name in other_names:
        if name in ("cfg5bwd", "cfg5", "cfg5single"):
            if name == "cfg5single":
                others.append(measure_layer_stack(variant, 5, 1, with_backward=False, grouped=False)[0])
            elif name == "cfg5" or args.workload != "cfg5":
                h5, b5 = measure_layer_stack(variant, 3, 1, with_backward=name == "cfg5bwd")
                others.append(b5 if name == "cfg5bwd" else h5)
            continue
        q = makers[name]()
        others.append(measure(q, variant, small_steps[name], 10))
        del q

    line = dict(
        metric=METRIC, value=head["tokens_per_s"], unit="tokens/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
        ms_per_step=head["ms_per_step"], higher_is_better=True, scaling="weak", vs_baseline=None, dtype="bf16",
        data="synthetic",
        config=dict(workload=workload, variant={lq.LQ_VARIANT_FUSED: "fused", lq.LQ_VARIANT_SPLIT: "split", lq.LQ_VARIANT_SLAB: "slab",
                             lq.LQ_VARIANT_AUTO: "auto (one launch per call: the slab or the fused kernel, picked by the library from rank and output width)"}[variant], step=step, **extra),
        roofline=head["roofline"], cpu_baseline=cpu,
        forward=dict(us=head["forward_us"], gbps=head["forward_gbps"], tflops=head["forward_tflops"],
                     hbm_frac=head["forward_hbm_frac"], mfma_frac=head["forward_mfma_frac"], kernels=head["kernels"],
                     per_step=head["per_step"], error_word=head["error_word"]),
        configs=others)
    bad = [head["error_word"]] + [o.get("error_word", 0) for o in others]
    if any(bad):
        print(f"bench.py: a workspace error word is non-zero after the timed loops: {bad}", file=sys.stderr)
        sys.exit(3)
    print(json.dumps(line))


if __name__ == "__main__":
    main()

#!/usr/bin/env python3
"""Benchmark of the segmented multi-LoRA hot path on one MI355X.

A step = one pass of the whole path over one batch: segment-metadata builder + forward (shrink,
h-save, expand; split or fused variant) [+ backward of the fine-tune rows for the layer-stack
workload].  Inputs are synthetic (paper_2511_00101_amd/synth.py), already resident in HBM, and
rotated over enough replicas (> 1 GiB in total) that no step finds its operands in L2 or in the
Infinity Cache left there by the previous step.

Prints ONE JSON line (see README/DESIGN for the fields).  `value` is tokens/s of the headline
workload (the decode-heavy batch, benchmark configs[1]); `roofline` is the HBM roofline of the
dominant kernel from HIP-event timing of each launch (the dispatch's own start and end time stamps); `cpu_baseline` is the fp64 oracle on the host
cores; `configs` carries the same measurements for the other single-call workloads.
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
    """Bytes the method must move and flops it must do for one call ('Algorithmic bytes'):
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


def time_steps(rep, steps, warmup):
    """Wall clock over exactly `steps` steps, synchronised on both sides."""
    torch = rep.torch
    for i in range(warmup):
        rep.step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        rep.step(warmup + i)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def time_kernels(rep, steps, warmup):
    """Average duration of each kernel over `steps` steps, from HIP events on the launch stream: the library
    launches every kernel with a pair of events that receive the dispatch's own start and end time stamps
    (lora_profile_enable / lora_profile_read), which is the duration rocprofv3's kernel trace reports
    (profiles/), without the gaps between launches."""
    torch, lq = rep.torch, rep.lq
    for i in range(warmup):
        rep.step(i)
    torch.cuda.synchronize()
    lq.lora_profile_enable(True)
    for i in range(steps):
        rep.step(warmup + i)
    torch.cuda.synchronize()
    prof = lq.lora_profile_read()
    lq.lora_profile_enable(False)
    return {name: dict(avg_us=total / n, launches=n) for name, (total, n) in prof.items() if n}


PROFILE_FILES = dict(cfg2_decode_heavy="forward_cfg2_decode_heavy.txt", cfg3_unified="forward_cfg3_unified.txt",
                     cfg4_mlp_up="forward_cfg4_mlp_up.txt", cfg4_mlp_down="forward_cfg4_mlp_down.txt")


def counter_traffic(workload, phase):
    """HBM bytes per launch of `phase` from the committed rocprofv3 counter summary of this workload
    (profiles/, FETCH_SIZE and WRITE_SIZE scaled by the copy calibration), or None."""
    name = PROFILE_FILES.get(workload)
    path = os.path.join(ROOT, "profiles", name) if name else None
    if not path or not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) == 3 and f[0] == "traffic_bytes_per_launch" and f[1] == phase:
            return int(f[2])
    return None


def measure(p, variant, steps, warmup):
    work = algorithmic_work(p)
    rep = Replicas(p, variant)
    s_per_step = time_steps(rep, steps, warmup)
    kern = time_kernels(rep, steps, warmup)
    fwd_names = [k for k in kern if k != "build"]
    fwd_us = sum(kern[k]["avg_us"] for k in fwd_names)
    if "forward_fused" in kern:
        dom, dom_bytes = "forward_fused", work["total"]
    else:
        dom = "expand" if work["expand"] >= work["shrink"] else "shrink"
        dom_bytes = work[dom]
    dom_gbps = dom_bytes / (kern[dom]["avg_us"] * 1e-6) / 1e9
    res = dict(
        workload=p.name, tokens=work["tokens"], d_in=p.d_in, d_out=p.d_out, replicas=rep.n,
        ms_per_step=s_per_step * 1e3, tokens_per_s=work["tokens"] / s_per_step,
        forward_us=fwd_us, forward_gbps=work["total"] / (fwd_us * 1e-6) / 1e9,
        forward_tflops=work["flops"] / (fwd_us * 1e-6) / 1e12,
        forward_hbm_frac=work["total"] / (fwd_us * 1e-6) / 1e9 / HBM_PEAK_GBPS,
        forward_mfma_frac=work["flops"] / (fwd_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        algorithmic_bytes=work["total"], flops=work["flops"], kernels=kern,
        roofline=dict(bound="hbm", kernel=dom, achieved=dom_gbps, peak=HBM_PEAK_GBPS, unit="GB/s",
                      frac=dom_gbps / HBM_PEAK_GBPS, traffic=counter_traffic(p.name, dom), algorithmic_bytes=dom_bytes,
                      avg_launch_us=kern[dom]["avg_us"]))
    del rep
    return res


class LayerStack:
    """The 8B-shaped 32-layer stack (benchmark configs[4]): 7 LoRA projections per layer with their own
    adapter weights, one batch structure for all 224 calls; forward of every call, then backward of the
    fine-tune rows of every call.  Activations and weights are drawn on the GPU (same distributions as the
    seeded generators; the parity tests use the seeded ones on sampled calls)."""

    def __init__(self, variant, n_layers=None):
        import numpy as np
        import torch
        from paper_2511_00101_amd import binding as lq
        from paper_2511_00101_amd import synth
        self.lq, self.torch, self.variant = lq, torch, variant
        self.n_layers = n_layers or synth.N_LAYERS
        dev = "cuda"
        b = synth.config5_batch()
        self.batch = b
        T = b.n_tokens
        self.T = T
        n_ad, r = 16, 32
        self.ranks_np = np.full(n_ad, r, np.int32)
        gen = torch.Generator(device=dev).manual_seed(5000)
        bf = torch.bfloat16

        def act(cols, std=1.0):
            return (torch.randn(T, cols, generator=gen, device=dev, dtype=torch.float32) * std).to(bf)

        self.ta = torch.from_numpy(b.token_adapter).to(dev)
        self.tk = torch.from_numpy(b.token_kind).to(dev)
        self.seg = lq.SegmentTables.empty(T, n_ad, dev)
        self.bws = lq.workspace(lq.lora_build_workspace_bytes(T, n_ad), dev)
        self.calls = []
        max_fws = max_bws = 0
        for layer in range(self.n_layers):
            xs = {4096: act(4096), 14336: act(14336)}          # q,k,v,(o),gate,up read a 4096-wide x; down a 14336-wide one
            x_o = act(4096)
            dxs = {4096: act(4096), 14336: act(14336)}
            dx_o = act(4096)
            for pi, (name, d_in, d_out) in enumerate(synth.LAYER_PROJECTIONS):
                A = [(torch.randn(r, d_in, generator=gen, device=dev) * 0.02).to(bf) for _ in range(n_ad)]
                B = [(torch.randn(r, d_out, generator=gen, device=dev) * 0.02).to(bf) for _ in range(n_ad)]
                ad = lq.AdapterTable.from_tensors(A, B, [2.0] * n_ad, dev)
                y = act(d_out)                                   # y0; after the forward it doubles as dy for the backward
                dA = [torch.zeros(r, d_in, device=dev) if a < 2 else None for a in range(n_ad)]
                dB = [torch.zeros(r, d_out, device=dev) if a < 2 else None for a in range(n_ad)]
                dA_ptrs = torch.tensor([t.data_ptr() if t is not None else 0 for t in dA], dtype=torch.int64, device=dev)
                dB_ptrs = torch.tensor([t.data_ptr() if t is not None else 0 for t in dB], dtype=torch.int64, device=dev)
                h_out = torch.zeros(4096 * r, dtype=torch.float32, device=dev)
                self.calls.append(dict(x=x_o if name == "o" else xs[d_in], dx=dx_o if name == "o" else dxs[d_in], y=y, ad=ad,
                                       h_out=h_out, dA=dA, dB=dB, dA_ptrs=dA_ptrs, dB_ptrs=dB_ptrs, d_in=d_in, d_out=d_out))
                max_fws = max(max_fws, lq.lora_forward_workspace_bytes(T, r, d_in, d_out, variant))
                max_bws = max(max_bws, lq.lora_backward_workspace_bytes(T, n_ad, r, d_in, d_out))
        self.fws = lq.workspace(max_fws, dev)
        self.bwd_ws = lq.workspace(max_bws, dev)
        self.ranks = self.calls[0]["ad"].ranks

    def work(self):
        """Algorithmic bytes / flops of one step (forward of all calls + backward of the fine-tune rows)."""
        import numpy as np
        b = self.batch
        n_live, n_ft = b.n_tokens, int((b.token_kind == 0).sum())
        r, used, used_ft = 32, 16, 2
        fwd_b = bwd_b = fwd_f = bwd_f = 0
        for c in self.calls:
            di, do = c["d_in"], c["d_out"]
            fwd_b += n_live * di * 2 + n_live * do * 4 + used * r * (di + do) * 2 + n_ft * r * 4
            fwd_f += 2 * r * (di + do) * n_live
            # backward: dy and x read once each for the weight gradients and once for g / dx's operands are the same
            # rows, dx read + written, A and B of the fine-tune adapters, dA and dB read + written, h read
            bwd_b += n_ft * do * 2 + n_ft * di * 2 + n_ft * di * 4 + used_ft * r * (di + do) * 2 + used_ft * r * (di + do) * 8 + n_ft * r * 4
            bwd_f += 2 * r * (di + do) * n_ft * 2
        return dict(fwd_bytes=fwd_b, bwd_bytes=bwd_b, fwd_flops=fwd_f, bwd_flops=bwd_f, tokens=n_live)

    def step(self, i=0):
        lq = self.lq
        lq.lora_build_segments(self.ta, self.tk, self.ranks, self.seg, self.bws)
        for c in self.calls:
            lq.lora_segmented_forward(c["x"], c["y"], c["ad"], self.seg, c["h_out"], self.fws, self.variant)
        for c in reversed(self.calls):
            lq.lora_segmented_backward(c["x"], c["y"], c["dx"], c["ad"], c["dA_ptrs"], c["dB_ptrs"], self.seg, c["h_out"],
                                       self.bwd_ws)

    def forward_only(self):
        for c in self.calls:
            self.lq.lora_segmented_forward(c["x"], c["y"], c["ad"], self.seg, c["h_out"], self.fws, self.variant)

    def backward_only(self):
        for c in reversed(self.calls):
            self.lq.lora_segmented_backward(c["x"], c["y"], c["dx"], c["ad"], c["dA_ptrs"], c["dB_ptrs"], self.seg, c["h_out"],
                                            self.bwd_ws)


def measure_layer_stack(variant, steps, warmup):
    import torch
    st = LayerStack(variant)
    w = st.work()
    for i in range(warmup):
        st.step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        st.step(i)
    torch.cuda.synchronize()
    s_per_step = (time.perf_counter() - t0) / steps
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    ev[0].record(); st.forward_only(); ev[1].record(); st.backward_only(); ev[2].record()
    torch.cuda.synchronize()
    fwd_ms, bwd_ms = ev[0].elapsed_time(ev[1]), ev[1].elapsed_time(ev[2])
    kernels = {}
    for which, run in (("forward", st.forward_only), ("backward", st.backward_only)):
        st.lq.lora_profile_enable(True)
        run()
        torch.cuda.synchronize()
        kernels[which] = {name: dict(avg_us=total / n, launches=n) for name, (total, n) in st.lq.lora_profile_read().items() if n}
        st.lq.lora_profile_enable(False)
    return dict(workload="cfg5_layer_stack (32 layers x 7 projections, forward + backward of the fine-tune rows)",
                tokens=w["tokens"], calls=len(st.calls), ms_per_step=s_per_step * 1e3, tokens_per_s=w["tokens"] / s_per_step,
                forward_ms=fwd_ms, backward_ms=bwd_ms,
                forward_gbps=w["fwd_bytes"] / (fwd_ms * 1e-3) / 1e9, backward_gbps=w["bwd_bytes"] / (bwd_ms * 1e-3) / 1e9,
                forward_tflops=w["fwd_flops"] / (fwd_ms * 1e-3) / 1e12, backward_tflops=w["bwd_flops"] / (bwd_ms * 1e-3) / 1e12,
                forward_hbm_frac=w["fwd_bytes"] / (fwd_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                backward_hbm_frac=w["bwd_bytes"] / (bwd_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                algorithmic_bytes=w["fwd_bytes"] + w["bwd_bytes"], flops=w["fwd_flops"] + w["bwd_flops"], kernels=kernels)


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
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--variant", choices=["auto", "split", "fused"], default="auto",
                    help="auto: the single-launch (fused) variant, which is at least as fast as two launches on every "
                         "workload here; split: two launches, with the shrink / expand breakdown")
    ap.add_argument("--workload", default="cfg2", help="headline workload: cfg1, cfg2, cfg3, cfg4up, cfg4down")
    ap.add_argument("--others", default="cfg3,cfg4up,cfg4down,cfg5", help="comma list of further workloads ('' = none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain device copy of known size (256 MiB read + 256 MiB written, 8 times) so that "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings can be scaled to bytes")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU's throughput; --gpus must be 1 "
              "(the path shards by token segments with no exchange, see DESIGN.md)", file=sys.stderr)
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
    def variant_for(problem):
        return lq.LQ_VARIANT_SPLIT if args.variant == "split" else lq.LQ_VARIANT_FUSED
    makers = dict(cfg1=synth.config1, cfg2=synth.config2, cfg3=synth.config3,
                  cfg4up=lambda: synth.config4("up"), cfg4down=lambda: synth.config4("down"))

    p = makers[args.workload]()
    variant = variant_for(p)
    head = measure(p, variant, args.steps, args.warmup)
    others = []
    for name in [n for n in args.others.split(",") if n and n != args.workload]:
        if name == "cfg5":
            others.append(measure_layer_stack(lq.LQ_VARIANT_SPLIT if args.variant == "split" else lq.LQ_VARIANT_FUSED, 3, 1))
            continue
        q = makers[name]()
        others.append(measure(q, variant_for(q), max(20, args.steps // 4), max(5, args.warmup // 2)))
        del q
    cpu = None if args.no_cpu_baseline else cpu_baseline(p)

    line = dict(
        metric=METRIC, value=head["tokens_per_s"], unit="tokens/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
        ms_per_step=head["ms_per_step"], higher_is_better=True, scaling="weak", vs_baseline=None, dtype="bf16",
        data="synthetic",
        config=dict(workload=f"{head['workload']}: {head['tokens']} tokens, {head['d_in']}->{head['d_out']}, "
                             f"{p.n_adapters} adapters rank {int(p.ranks.max())}",
                    variant="fused" if variant == lq.LQ_VARIANT_FUSED else "split",
                    replicas=head["replicas"], step="segment builder + forward"),
        roofline=head["roofline"], cpu_baseline=cpu,
        forward=dict(us=head["forward_us"], gbps=head["forward_gbps"], tflops=head["forward_tflops"],
                     hbm_frac=head["forward_hbm_frac"], mfma_frac=head["forward_mfma_frac"], kernels=head["kernels"]),
        configs=others)
    print(json.dumps(line))


if __name__ == "__main__":
    main()

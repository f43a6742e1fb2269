#!/usr/bin/env python3
"""Throughput of the VScan reduction path on one MI355X.

One "step" is one pass of the whole path over one batch of seeded synthetic
inputs: for every keep budget the workload sweeps, vscan_encoder_reduce followed
by vscan_llm_prune.  Inputs, outputs and workspaces are resident in HBM before
the timed region; nothing is allocated inside it.

Prints ONE JSON line: whole-job "visual tokens reduced per second", the roofline
figures of the kernel that takes the most device time, and the CPU oracle timed
on this host as a baseline.
"""
from __future__ import annotations

import argparse
import dataclasses
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2505_22654_amd import workloads as wl  # noqa: E402

PEAK_HBM_GBS = 8000.0
PEAK_MFMA_TFLOPS = {"bf16": 2500.0, "f32": 157.3}

KERNEL_SOURCE = {
    "score_cls": "encoder_score.hip", "score_mean_lse": "encoder_score.hip",
    "score_mean_colsum": "encoder_score.hip", "encoder_select": "select.hip",
    "llm_select": "select.hip", "sim_argmax": "sim_merge.hip",
    "merge": "sim_merge.hip", "llm_score": "llm.hip", "compact": "llm.hip",
    "fused_q": "fused.hip", "fused_split_q": "fused.hip", "fused_qt": "fused.hip",
    "fused_logits": "fused.hip", "fused_softmax": "fused.hip",
    "fused_colsum": "fused.hip",
}


def sweep_points(index: int):
    if index == 2:
        return [wl.config(2, sweep=k) for k in (192, 128, 64)]
    if index == 5:
        return [wl.config(5, sweep=k) for k in (720, 288, 144)]
    return [wl.config(index)]


def _score_chain_work(out, seqs, Dh, Hq, Hkv, dh, Tq, V):
    """Adds the kernels of the score chain that starts from hidden states: each operand read
    once, each result written once; the logit contraction counts as matrix-core work once its
    flops per byte exceed the chip's ridge (2.5 PFLOP/s over 8 TB/s)."""
    R, nq, nkv = Hq * Tq, Hq * dh, Hkv * dh
    flops, byts = 2.0 * seqs * V * Dh * R, seqs * V * (Dh * 2 + R * 4) + seqs * R * Dh * 6
    add = {
        "fused_q": ("hbm", nq * Dh * 2 + seqs * Tq * (Dh * 2 + nq * 4)),
        "fused_split_q": ("hbm", seqs * Tq * nq * (4 + 6)),
        "fused_qt": ("hbm", nkv * Dh * 2 + seqs * Tq * nq * 6 + seqs * R * Dh * 6),
        "fused_logits": ("mfma", flops) if flops / byts > 312 else ("hbm", byts),
        "fused_softmax": ("hbm", seqs * R * V * 8),
        "fused_colsum": ("hbm", seqs * R * V * 4 + seqs * V * 4),
    }
    for name, (bound, amount) in add.items():
        b0, a0 = out.get(name, (bound, 0.0))
        out[name] = (b0, a0 + amount)


def algorithmic_work(w: wl.Workload, inputs: str = "qk"):
    """Per-kernel algorithmic work of ONE call pair on this workload:
    {kernel: (bound, amount)} with bytes for "hbm" and flops for "mfma"."""
    out = {}
    e = w.encoder
    if e is not None:
        es = 2 if e.dtype == wl.BF16 else 4
        B, C, N, S, H, dh, D = e.batch, e.n_segments, e.n_tokens, e.rows, e.heads, e.head_dim, e.feat_dim
        K, T = e.keep, e.tokens_per_image
        U = T - K
        if inputs == "hidden":
            _score_chain_work(out, B * C, D, H, H, dh, 1, N)
        elif e.score_mode == 0:
            out["score_cls"] = ("hbm", B * C * H * S * dh * es)
        else:
            out["score_mean_lse"] = ("mfma", 2.0 * B * C * H * N * N * dh)
            out["score_mean_colsum"] = ("mfma", 2.0 * B * C * H * N * N * dh)
        out["encoder_select"] = ("hbm", B * T * 4 + B * K * 4)
        out["sim_argmax"] = ("mfma", 2.0 * B * U * K * D)
        out["merge"] = ("hbm", B * (T + K) * D * es)
    l = w.llm
    if l is not None:
        es = 2 if l.dtype == wl.BF16 else 4
        row = (l.hidden + 2 * l.kv_heads * l.head_dim) * es
        out["llm_select"] = ("hbm", l.batch * l.vis_len * 4 + l.batch * l.keep * 4)
        moved = (l.keep + l.text) if l.in_place else l.seq_out
        if inputs == "qk":
            out["llm_score"] = ("hbm", l.batch * l.kv_heads * l.vis_len * l.head_dim * es)
            out["compact"] = ("hbm", l.batch * moved * row * 2)
        else:
            _score_chain_work(out, l.batch, l.hidden, l.q_heads, l.kv_heads, l.head_dim,
                              l.n_query, l.vis_len)
            out["compact"] = ("hbm", l.batch * moved * l.hidden * es * 2)
    return out


def tokens_reduced(w: wl.Workload) -> int:
    n = 0
    if w.encoder is not None:
        n += w.encoder.batch * (w.encoder.tokens_per_image - w.encoder.keep)
    if w.llm is not None:
        n += w.llm.batch * (w.llm.vis_len - w.llm.keep)
    return n


class DeviceCase:
    """Device-resident inputs, outputs and workspaces of one sweep point."""

    def __init__(self, w: wl.Workload, host, ring: int, inputs: str = "qk"):
        import torch
        from paper_2505_22654_amd import binding as vb
        self.w, self.vb, self.torch, self.inputs = w, vb, torch, inputs
        self.enc_in = self.enc_out = self.enc_ws = None
        if w.encoder is not None:
            e = w.encoder
            if inputs == "hidden":
                import numpy as np
                hh = host["enc_hidden"]
                self.enc_in = {"hidden": _to_device(hh["hidden"], e.dtype),
                               "w_q": _to_device(hh["w_q"], e.dtype),
                               "w_k_t": _to_device(np.ascontiguousarray(hh["w_k"].T), e.dtype),
                               "x": _to_device(hh["x"], e.dtype)}
                need = vb.encoder_fused_workspace_size(vb.encoder_desc(e))
            else:
                self.enc_in = {n: _to_device(host["enc"][n], e.dtype) for n in ("q", "k", "x")}
                need = vb.encoder_workspace_size(vb.encoder_desc(e))
            self.enc_ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            self.enc_out = {
                "kept_idx": torch.empty((e.batch, e.keep), dtype=torch.int32, device="cuda"),
                "merged": torch.empty((e.batch, e.keep, e.feat_dim), dtype=self.enc_in["x"].dtype,
                                      device="cuda")}
        self.llm_in, self.llm_out, self.llm_ws, self.pristine = [], None, None, None
        if w.llm is not None:
            l = w.llm
            base = {n: _to_device(host["llm"][n], l.dtype) for n in ("q", "k", "v", "hidden")}
            sets = ring if l.in_place else 1
            self.llm_in = [base] + [{n: (t if n == "q" else t.clone()) for n, t in base.items()}
                                    for _ in range(sets - 1)]
            need = vb.llm_workspace_size(vb.llm_desc(l))
            if inputs == "hidden":
                import numpy as np
                need = vb.llm_fused_workspace_size(vb.llm_desc(l))
                self.w_q = _to_device(host["weights"]["w_q"], l.dtype)
                self.w_k_t = _to_device(np.ascontiguousarray(host["weights"]["w_k"].T), l.dtype)
            self.llm_ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            self.llm_out = {"kept_idx": torch.empty((l.batch, l.keep), dtype=torch.int32,
                                                    device="cuda")}
            if not l.in_place:
                self.llm_out["k"] = torch.empty((l.batch, l.kv_heads, l.seq_out, l.head_dim),
                                                dtype=base["k"].dtype, device="cuda")
                self.llm_out["v"] = torch.empty_like(self.llm_out["k"])
                self.llm_out["hidden"] = torch.empty((l.batch, l.seq_out, l.hidden),
                                                     dtype=base["k"].dtype, device="cuda")
            elif sets > 1:
                self.pristine = {n: base[n].clone() for n in ("k", "v", "hidden")}

    def restore(self):
        """Undo in-place compaction (outside any timed region)."""
        if self.pristine is not None:
            for s in self.llm_in:
                for n, t in self.pristine.items():
                    s[n].copy_(t)

    def run_encoder(self):
        if self.enc_in is not None and self.inputs == "hidden":
            self.vb.encoder_reduce_fused(self.w.encoder, self.enc_in["hidden"], self.enc_in["w_q"],
                                         self.enc_in["w_k_t"], self.enc_in["x"],
                                         workspace=self.enc_ws, out=self.enc_out)
        elif self.enc_in is not None:
            self.vb.encoder_reduce(self.w.encoder, self.enc_in["q"], self.enc_in["k"],
                                   self.enc_in["x"], workspace=self.enc_ws, out=self.enc_out)

    def run_llm(self, i: int):
        if self.llm_in:
            s = self.llm_in[i % len(self.llm_in)]
            if self.inputs == "hidden":
                self.vb.llm_prune_fused(self.w.llm, s["hidden"], self.w_q, self.w_k_t,
                                        workspace=self.llm_ws, out=self.llm_out)
                return
            self.vb.llm_prune(self.w.llm, s["q"], s["k"], s["v"], s["hidden"],
                              workspace=self.llm_ws, out=self.llm_out)

    def run(self, i: int):
        self.run_encoder()
        self.run_llm(i)


def _to_device(a, dtype):
    import torch
    import numpy as np
    if dtype == wl.BF16:
        return torch.from_numpy(wl.bf16_bits(a)).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def host_inputs(points, inputs: str = "qk"):
    """Seeded inputs per sweep point; tensors that do not depend on the budget are shared."""
    cache, hosts = {}, []
    for w in points:
        h = {}
        if w.encoder is not None:
            key = ("enc", dataclasses.replace(w.encoder, keep_global=0, keep_local=0))
            if inputs == "hidden":
                if ("hid",) + key not in cache:
                    cache[("hid",) + key] = wl.encoder_hidden_inputs(w.encoder, w.seed)
                h["enc_hidden"] = cache[("hid",) + key]
            else:
                if key not in cache:
                    cache[key] = wl.encoder_inputs(w.encoder, w.seed)
                h["enc"] = cache[key]
        if w.llm is not None:
            key = ("llm", dataclasses.replace(w.llm, keep=0))
            if key not in cache:
                cache[key] = wl.llm_inputs(w.llm, w.seed)
            h["llm"] = cache[key]
            if inputs == "hidden":
                if ("weights", key) not in cache:
                    cache[("weights", key)] = wl.llm_weights(w.llm, w.seed)
                h["weights"] = cache[("weights", key)]
        hosts.append(h)
    return hosts


def cpu_baseline(points, hosts, budget_s=12.0, inputs: str = "qk"):
    """The CPU oracle on this host's cores over whole steps of the same inputs."""
    from oracle import vscan_oracle as vo

    def one_step():
        for w, h in zip(points, hosts):
            if w.encoder is not None and inputs == "hidden":
                hh = h["enc_hidden"]
                vo.encoder_reduce_fused(w.encoder, hh["hidden"], hh["w_q"], hh["w_k"], hh["x"])
            elif w.encoder is not None:
                vo.encoder_reduce(w.encoder, h["enc"]["q"], h["enc"]["k"], h["enc"]["x"])
            if w.llm is not None and inputs == "hidden":
                vo.llm_prune_fused(w.llm, h["llm"]["hidden"], h["weights"]["w_q"],
                                   h["weights"]["w_k"])
            elif w.llm is not None:
                vo.llm_prune(w.llm, **h["llm"])

    t0 = time.perf_counter()
    one_step()
    first = time.perf_counter() - t0
    reps = max(1, min(50, int(budget_s / max(first, 1e-3))))
    t0 = time.perf_counter()
    for _ in range(reps):
        one_step()
    dt = (time.perf_counter() - t0) / reps
    reduced = sum(tokens_reduced(w) for w in points)
    return {"value": reduced / dt, "unit": "visual tokens reduced/s", "cores": vo.threads(),
            "kind": "oracle", "sample": f"{reps} full step(s) of the same workload, "
                                        f"{dt * 1e3:.1f} ms per step"}


def kernel_source_digest(kernel: str) -> str:
    """sha256 over the kernel's source file and the headers every kernel includes."""
    h = hashlib.sha256()
    names = [KERNEL_SOURCE[kernel], "common.hpp", "launch.hpp"]
    if KERNEL_SOURCE[kernel] == "fused.hip":
        names.append("fused.hpp")
    for name in names:
        with open(os.path.join(ROOT, "paper_2505_22654_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def stored_traffic(kernel: str, workload: str):
    """HBM bytes per launch from the committed counter runs, or None when absent or when the
    kernel's source changed after the counters were taken."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(path):
        return None
    try:
        rec = json.load(open(path)).get(f"{workload}:{kernel}")
        if rec and rec.get("source_sha256") == kernel_source_digest(kernel):
            return rec["bytes_per_launch"]
    except (OSError, ValueError, KeyError):
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "cfg6"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="N",
                    help="also run N plain device copies of 256 MiB (a kernel of known traffic "
                         "for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--inputs", default="qk", choices=["qk", "hidden"],
                    help="qk: both stages score from the layers' Q and K (the default step); "
                         "hidden: vscan_encoder_reduce_fused + vscan_llm_prune_fused, which score "
                         "from hidden states and projection weights ([CLS] encoders only)")
    ap.add_argument("--streams", type=int, default=1, choices=[1, 2],
                    help="2: issue the encoder calls and the LLM calls of a step on two streams "
                         "(they are independent in this benchmark); default 1 = strictly serial")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: one GPU only (the path shards by image / "
                 "sequence with no exchange); run with --gpus 1")

    import torch
    from paper_2505_22654_amd import binding as vb
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    vb.lib()

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(args.calibrate_copy):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    index = int(args.workload[3:])
    points = sweep_points(index)
    if args.inputs == "hidden" and any(w.encoder is not None and w.encoder.score_mode != 0
                                       for w in points):
        sys.exit("bench.py: --inputs hidden needs a [CLS] encoder (mean-attention scoring has one "
                 "query per token and is served by the Q/K form only)")
    hosts = host_inputs(points, args.inputs)
    in_place = any(w.llm is not None and w.llm.in_place for w in points)
    steps, warmup = args.steps, args.warmup
    if index in (4, 5):
        steps, warmup = min(steps, 20), min(warmup, 3)
    ring = steps if in_place else 1
    cases = [DeviceCase(w, h, ring, args.inputs) for w, h in zip(points, hosts)]

    side = torch.cuda.Stream() if args.streams == 2 else None

    def step(i):
        if side is None:
            for c in cases:
                c.run(i)
            return
        # encoder calls on the current stream, LLM calls on a second one; both sides are
        # joined again before the step ends
        main_stream = torch.cuda.current_stream()
        side.wait_stream(main_stream)
        for c in cases:
            c.run_encoder()
        with torch.cuda.stream(side):
            for c in cases:
                c.run_llm(i)
        main_stream.wait_stream(side)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    for c in cases:
        c.restore()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    # second pass of the same steps with the library's per-kernel HIP events switched on
    for c in cases:
        c.restore()
    torch.cuda.synchronize()
    vb.profile_enable(True)
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    vb.profile_enable(False)
    prof = vb.profile_read()

    work = {}
    for w in points:
        for name, (bound, amount) in algorithmic_work(w, args.inputs).items():
            b, a = work.get(name, (bound, 0.0))
            work[name] = (bound, a + amount)
    dtype = (points[0].encoder or points[0].llm).dtype
    kernels = {}
    for name, rec in prof.items():
        bound, amount = work[name]
        avg_s = rec["total_ms"] * 1e-3 / rec["launches"]
        per_launch = amount * steps / rec["launches"]
        if bound == "hbm":
            achieved, peak, unit = per_launch / avg_s / 1e9, PEAK_HBM_GBS, "GB/s"
        else:
            achieved, peak, unit = per_launch / avg_s / 1e12, PEAK_MFMA_TFLOPS[dtype], "TFLOP/s"
        kernels[name] = {"bound": bound, "achieved": round(achieved, 3), "peak": peak,
                         "unit": unit, "frac": round(achieved / peak, 5),
                         "avg_us": round(avg_s * 1e6, 2), "launches_per_step": rec["launches"] // steps,
                         "share": rec["total_ms"]}
    total_ms = sum(k["share"] for k in kernels.values()) or 1.0
    for k in kernels.values():
        k["share"] = round(k["share"] / total_ms, 4)
    dominant = max(kernels, key=lambda n: kernels[n]["share"])
    roof = {key: kernels[dominant][key] for key in ("bound", "achieved", "peak", "unit", "frac")}
    roof["kernel"] = dominant
    roof["avg_us"] = kernels[dominant]["avg_us"]
    roof["traffic"] = stored_traffic(dominant, args.workload)

    reduced = sum(tokens_reduced(w) for w in points)
    result = {
        "metric": "visual tokens reduced/sec (encoder scan+merge, LLM prune)",
        "value": reduced * steps / dt,
        "unit": "visual tokens reduced/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": dt * 1e3 / steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic",
        "config": {"workload": args.workload + ": " + ", ".join(w.name for w in points),
                   "streams": args.streams,
                   "tokens_reduced_per_step": reduced,
                   "step": ("encoder_reduce + llm_prune" if args.inputs == "qk" else
                            "encoder_reduce_fused + llm_prune_fused")
                           + " for every keep budget of the sweep"},
        "roofline": roof,
        "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(points, hosts, inputs=args.inputs)
    print(json.dumps(result))


if __name__ == "__main__":
    main()

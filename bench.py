#!/usr/bin/env python3
"""Throughput of the VScan reduction path on one MI355X.

One "step" is one pass of the whole path over one batch of seeded synthetic
inputs: for every keep budget the workload sweeps, vscan_encoder_reduce followed
by vscan_llm_prune.  Inputs, outputs and workspaces are resident in HBM before
the timed region; nothing is allocated inside it.

The headline workload is configuration 4, the largest that runs both stages (one
16384-token image scored by mean attention received, then a 4096-token visual
span pruned under grouped-query attention).  Configurations 5 (stage-2 stress,
in place) and 2 (LLaVA-1.5-shaped batch) are measured in the same run and carried
under "other_workloads".

Prints ONE JSON line: whole-job "visual tokens reduced per second" of the headline
workload, the roofline figures of the kernel that takes the most device time
there, and the CPU oracle timed on this host as a baseline.
"""
from __future__ import annotations

import argparse
import ctypes
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
# Vector ALU without packed fp32 operations (the build switches them off): 256 compute units x
# 4 SIMDs x 16 lanes = 16384 lane-operations per cycle at 2.4 GHz.  On this chip a
# transcendental (v_exp_f32) issues at half that rate (one wave instruction per 8 cycles and SIMD,
# measured; CDNA4 doubled the transcendental rate of its predecessor) and counts as 2.
PEAK_ALU_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12
# least lane-operations per logit of the mean-attention passes: one multiply (or multiply-add)
# by the softmax scale, one exponential (2), one accumulation
MEAN_LANEOPS_PER_LOGIT = 4.0

KERNEL_SOURCE = {
    "score_cls": "encoder_score.hip", "score_mean_lse": "encoder_score.hip",
    "score_mean_colsum": "encoder_score.hip", "encoder_select": "select.hip",
    "llm_select": "select.hip", "sim_argmax": "sim_merge.hip",
    "merge": "sim_merge.hip", "llm_score": "llm.hip",
    "compact": "llm.hip",
    "fused_q": "fused.hip", "fused_split_q": "fused.hip", "fused_qt": "fused.hip",
    "fused_logits": "fused.hip", "fused_softmax": "fused.hip",
    "fused_colsum": "fused.hip",
}

DEFAULT_STEPS = {1: (200, 20), 2: (200, 20), 3: (100, 10), 4: (30, 5), 5: (10, 2), 6: (100, 10)}


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
    {kernel: (bound, amount)} with bytes for "hbm" and flops for "mfma".  Second return value:
    bytes a call moves beyond that definition ({kernel: {term: bytes}}), reported apart."""
    out, extra = {}, {}
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
        # rows the method has to move: the kept visual rows and the rows after the span; an
        # out-of-place call also copies the prefix rows, counted apart
        moved = l.keep + l.text
        prefix = 0 if l.in_place else l.prefix
        if inputs == "qk":
            out["llm_score"] = ("hbm", l.batch * l.kv_heads * l.vis_len * l.head_dim * es)
            out["compact"] = ("hbm", l.batch * moved * row * 2)
            extra["compact"] = {"prefix_rows_bytes": l.batch * prefix * row * 2}
        else:
            _score_chain_work(out, l.batch, l.hidden, l.q_heads, l.kv_heads, l.head_dim,
                              l.n_query, l.vis_len)
            out["compact"] = ("hbm", l.batch * moved * l.hidden * es * 2)
            extra["compact"] = {"prefix_rows_bytes": l.batch * prefix * l.hidden * es * 2}
    return out, extra


def tokens_reduced(w: wl.Workload) -> int:
    n = 0
    if w.encoder is not None:
        n += w.encoder.batch * (w.encoder.tokens_per_image - w.encoder.keep)
    if w.llm is not None:
        n += w.llm.batch * (w.llm.vis_len - w.llm.keep)
    return n


class DeviceCase:
    """Device-resident inputs, outputs and workspaces of one sweep point.  `ring` independent
    copies of the inputs are cycled through by step number: more than one makes consecutive
    steps read different memory (cold caches), and in-place compaction needs a pristine copy
    per step anyway."""

    def __init__(self, w: wl.Workload, host, ring: int, inputs: str = "qk"):
        import torch
        from paper_2505_22654_amd import binding as vb
        self.w, self.vb, self.torch, self.inputs = w, vb, torch, inputs
        self.enc_in, self.enc_out, self.enc_ws = [], None, None
        if w.encoder is not None:
            e = w.encoder
            if inputs == "hidden":
                import numpy as np
                hh = host["enc_hidden"]
                base = {"hidden": _to_device(hh["hidden"], e.dtype),
                        "w_q": _to_device(hh["w_q"], e.dtype),
                        "w_k_t": _to_device(np.ascontiguousarray(hh["w_k"].T), e.dtype),
                        "x": _to_device(hh["x"], e.dtype)}
                need = vb.encoder_fused_workspace_size(vb.encoder_desc(e))
            else:
                base = {n: _to_device(host["enc"][n], e.dtype) for n in ("q", "k", "x")}
                need = vb.encoder_workspace_size(vb.encoder_desc(e))
            copies = 1 if (w.llm is not None and w.llm.in_place) else ring
            self.enc_in = [base] + [{n: t.clone() for n, t in base.items()} for _ in range(copies - 1)]
            self.enc_ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            self.enc_out = {
                "kept_idx": torch.empty((e.batch, e.keep), dtype=torch.int32, device="cuda"),
                "merged": torch.empty((e.batch, e.keep, e.feat_dim), dtype=base["x"].dtype,
                                      device="cuda")}
        self.llm_in, self.llm_out, self.llm_ws, self.pristine = [], None, None, None
        if w.llm is not None:
            l = w.llm
            base = {n: _to_device(host["llm"][n], l.dtype) for n in ("q", "k", "v", "hidden")}
            self.llm_in = [base] + [{n: (t if n == "q" else t.clone()) for n, t in base.items()}
                                    for _ in range(ring - 1)]
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
            else:
                self.pristine = {n: base[n].clone() for n in ("k", "v", "hidden")}

    def restore(self):
        """Undo in-place compaction (outside any timed region)."""
        if self.pristine is not None:
            for s in self.llm_in:
                for n, t in self.pristine.items():
                    s[n].copy_(t)

    def run_encoder(self, i: int):
        if not self.enc_in:
            return
        s = self.enc_in[i % len(self.enc_in)]
        if self.inputs == "hidden":
            self.vb.encoder_reduce_fused(self.w.encoder, s["hidden"], s["w_q"], s["w_k_t"], s["x"],
                                         workspace=self.enc_ws, out=self.enc_out)
        else:
            self.vb.encoder_reduce(self.w.encoder, s["q"], s["k"], s["x"], workspace=self.enc_ws,
                                   out=self.enc_out)

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
        self.run_encoder(i)
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


def _omp_set_threads(n: int) -> bool:
    """Thread count of the oracle's OpenMP regions (it asks omp_get_max_threads)."""
    try:
        ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))
        return True
    except OSError:
        return False


def cpu_baseline(points, hosts, budget_s=12.0, inputs: str = "qk", one_thread: bool = False):
    """The CPU oracle, as it stands, on this host's cores over the same inputs.

    Workloads whose oracle step fits the time budget run whole steps.  Mean-attention scoring
    of a 16384-token image (H x N^2 x dh multiply-adds in fp64: about a minute on 16 cores) is
    probed first: the oracle scores 2 of the H heads.  If that projects to a full pass within
    the budget, the full step is timed as it is; else everything but the scoring (selection,
    assignment, merging, the LLM stage) runs in full and the step time is extrapolated as
    t(2 heads) x H/2 + t(rest), and the record says so."""
    from oracle import vscan_oracle as vo
    import numpy as np
    reduced = sum(tokens_reduced(w) for w in points)

    heavy = [w for w in points if w.encoder is not None and w.encoder.score_mode == 1 and
             w.encoder.heads * w.encoder.n_tokens ** 2 * w.encoder.head_dim > 2e10]
    if heavy and inputs == "qk":
        total, notes, exact_parts = 0.0, [], 0
        for w, h in zip(points, hosts):
            e = w.encoder
            if e is not None:
                sub = 2
                q, k, x = h["enc"]["q"], h["enc"]["k"], h["enc"]["x"]
                t0 = time.perf_counter()
                s = vo.encoder_scores(np.ascontiguousarray(q[:, :, :sub]),
                                      np.ascontiguousarray(k[:, :, :sub]), e.has_cls, e.score_mode,
                                      e.softmax_domain, e.scale)
                t_score = time.perf_counter() - t0
                if t_score * e.heads / sub <= 25.0:
                    # the whole pass fits the budget after all: time it as it is
                    t0 = time.perf_counter()
                    vo.encoder_reduce(e, q, k, x)
                    t_full = time.perf_counter() - t0
                    total += t_full
                    notes.append(f"encoder stage in full {t_full:.2f} s")
                    exact_parts += 1
                    if w.llm is not None:
                        t0 = time.perf_counter()
                        vo.llm_prune(w.llm, **h["llm"])
                        t_llm = time.perf_counter() - t0
                        total += t_llm
                        notes.append(f"LLM stage in full {t_llm:.2f} s")
                    continue
                t0 = time.perf_counter()
                kept = vo.select(s, s, e.grid_h, e.grid_w, e.win_rows, e.win_cols, e.keep_local,
                                 e.keep_global)
                a = vo.assign(x, kept)
                vo.merge(x, kept, a)
                t_rest = time.perf_counter() - t0
                total += t_score * e.heads / sub + t_rest
                notes.append(f"encoder: {sub} of {e.heads} heads scored in {t_score:.2f} s "
                             f"(x{e.heads // sub}), select+assign+merge in full {t_rest:.2f} s")
            if w.llm is not None:
                t0 = time.perf_counter()
                vo.llm_prune(w.llm, **h["llm"])
                t_llm = time.perf_counter() - t0
                total += t_llm
                notes.append(f"LLM stage in full {t_llm:.2f} s")
        return {"value": reduced / total, "unit": "visual tokens reduced/s", "cores": vo.threads(),
                "kind": "oracle", "extrapolated": exact_parts < len(heavy),
                "sample": "one step; " + "; ".join(notes) + f"; step {total:.1f} s"}

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

    def timed(budget):
        t0 = time.perf_counter()
        one_step()
        first = time.perf_counter() - t0
        reps = max(1, min(50, int(budget / max(first, 1e-3))))
        t0 = time.perf_counter()
        for _ in range(reps):
            one_step()
        return (time.perf_counter() - t0) / reps, reps

    dt, reps = timed(budget_s)
    rec = {"value": reduced / dt, "unit": "visual tokens reduced/s", "cores": vo.threads(),
           "kind": "oracle", "sample": f"{reps} full step(s) of the same workload, "
                                       f"{dt * 1e3:.1f} ms per step"}
    if one_thread:
        full = vo.threads()
        if _omp_set_threads(1):
            try:
                dt1, reps1 = timed(budget_s)
                rec["one_thread"] = {"value": reduced / dt1, "cores": 1,
                                     "sample": f"{reps1} full step(s), {dt1 * 1e3:.1f} ms per step"}
            finally:
                _omp_set_threads(full)
    return rec


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
    """HBM bytes per launch from the committed counter runs (profiles/traffic.json: two
    rocprofv3 --pmc runs, not measured in this process), or None when absent or when the
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


def _percentile(sorted_vals, p):
    if not sorted_vals:
        return None
    i = min(len(sorted_vals) - 1, max(0, int(round(p * (len(sorted_vals) - 1)))))
    return sorted_vals[i]


def measure(index: int, steps: int, warmup: int, inputs: str, streams: int, cold_ring: int,
            want_cpu: bool, one_thread: bool):
    """All figures of one workload: wall-clock throughput over exactly `steps` steps, per-step
    distribution, per-kernel device times with roofline fractions, CPU baseline."""
    import torch
    from paper_2505_22654_amd import binding as vb

    name = f"cfg{index}"
    points = sweep_points(index)
    if inputs == "hidden" and any(w.encoder is not None and w.encoder.score_mode != 0
                                  for w in points):
        sys.exit("bench.py: --inputs hidden is timed on [CLS] encoders only (the mean-attention form of "
                 "vscan_encoder_reduce_fused projects Q and K of every token and then runs the fp32 "
                 "kernels of the Q/K entry point; it is covered by the parity tests, not by this bench)")
    hosts = host_inputs(points, inputs)
    in_place = any(w.llm is not None and w.llm.in_place for w in points)
    ring = steps if in_place else 1
    cases = [DeviceCase(w, h, ring, inputs) for w, h in zip(points, hosts)]
    side = torch.cuda.Stream() if streams == 2 else None

    def step(i, cs=cases):
        if side is None:
            for c in cs:
                c.run(i)
            return
        # encoder calls on the current stream, LLM calls on a second one; both sides are
        # joined again before the step ends
        main_stream = torch.cuda.current_stream()
        side.wait_stream(main_stream)
        for c in cs:
            c.run_encoder(i)
        with torch.cuda.stream(side):
            for c in cs:
                c.run_llm(i)
        main_stream.wait_stream(side)

    def restore(cs=cases):
        for c in cs:
            c.restore()
        torch.cuda.synchronize()

    # ---- the contract measurement: W untimed steps, then exactly K steps between two syncs
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    restore()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    # ---- distribution: every step between its own pair of events on the launch stream
    def per_step_ms(cs):
        restore(cs)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(steps)]
        for i, (a, b) in enumerate(evs):
            a.record()
            step(i, cs)
            b.record()
        torch.cuda.synchronize()
        return sorted(a.elapsed_time(b) for a, b in evs)

    ms = per_step_ms(cases)
    timing = {"regime": ("in place: every step runs on its own pristine copy of K, V and hidden "
                         "states (cold)" if in_place else
                         "warm: every step reads the same buffers"),
              "median_ms": _percentile(ms, 0.5), "p10_ms": _percentile(ms, 0.1),
              "p90_ms": _percentile(ms, 0.9)}
    if cold_ring > 1 and not in_place:
        cold = [DeviceCase(w, h, cold_ring, inputs) for w, h in zip(points, hosts)]
        for i in range(min(warmup, cold_ring)):
            step(i, cold)
        cms = per_step_ms(cold)
        timing["cold"] = {"regime": f"cold: steps cycle through {cold_ring} independent copies of "
                                    "the inputs",
                          "median_ms": _percentile(cms, 0.5), "p10_ms": _percentile(cms, 0.1),
                          "p90_ms": _percentile(cms, 0.9)}
        del cold

    # ---- per kernel: the same steps with the library's HIP events around every launch
    restore()
    vb.profile_enable(True)
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    vb.profile_enable(False)
    prof = vb.profile_read()

    work, extra = {}, {}
    for w in points:
        wk, ex = algorithmic_work(w, inputs)
        for kname, (bound, amount) in wk.items():
            b, a = work.get(kname, (bound, 0.0))
            work[kname] = (bound, a + amount)
        for kname, terms in ex.items():
            for term, amount in terms.items():
                extra.setdefault(kname, {}).setdefault(term, 0.0)
                extra[kname][term] += amount
    dtype = (points[0].encoder or points[0].llm).dtype
    kernels = {}
    for kname, rec in prof.items():
        bound, amount = work[kname]
        avg_s = rec["total_ms"] * 1e-3 / rec["launches"]
        per_launch = amount * steps / rec["launches"]
        if bound == "hbm":
            achieved, peak, unit = per_launch / avg_s / 1e9, PEAK_HBM_GBS, "GB/s"
        else:
            achieved, peak, unit = per_launch / avg_s / 1e12, PEAK_MFMA_TFLOPS[dtype], "TFLOP/s"
        k = {"bound": bound, "achieved": round(achieved, 3), "peak": peak, "unit": unit,
             "frac": round(achieved / peak, 5), "avg_us": round(avg_s * 1e6, 2),
             "launches_per_step": rec["launches"] // steps, "share": rec["total_ms"]}
        if kname in ("score_mean_lse", "score_mean_colsum"):
            # also against the vector-ALU bound: MEAN_LANEOPS_PER_LOGIT lane-operations per logit
            laneops = MEAN_LANEOPS_PER_LOGIT * (per_launch / (2.0 * _head_dim(points))) / avg_s / 1e12
            k["alu"] = {"bound": "alu", "achieved": round(laneops, 3),
                        "peak": round(PEAK_ALU_TLANEOPS, 3), "unit": "Tlane-op/s",
                        "frac": round(laneops / PEAK_ALU_TLANEOPS, 5)}
        for term, amount in extra.get(kname, {}).items():
            if amount:
                k[term + "_per_launch"] = amount * steps / rec["launches"]
        kernels[kname] = k
    total_ms = sum(k["share"] for k in kernels.values()) or 1.0
    for k in kernels.values():
        k["share"] = round(k["share"] / total_ms, 4)
    dominant = max(kernels, key=lambda n: kernels[n]["share"])
    dk = kernels[dominant]
    src = dk.get("alu", dk)  # the mean-attention passes are bound by the vector ALU
    roof = {key: src[key] for key in ("bound", "achieved", "peak", "unit", "frac")}
    roof["kernel"] = dominant
    roof["avg_us"] = dk["avg_us"]
    roof["traffic"] = stored_traffic(dominant, name)
    roof["traffic_source"] = "profiles/traffic.json (stored rocprofv3 counter runs), not this run"
    if "alu" in dk:
        roof["vs_mfma_peak"] = {key: dk[key] for key in ("bound", "achieved", "peak", "unit", "frac")}

    reduced = sum(tokens_reduced(w) for w in points)
    result = {
        "value": reduced * steps / dt,
        "unit": "visual tokens reduced/s",
        "steps": steps, "warmup": warmup,
        "ms_per_step": dt * 1e3 / steps,
        "dtype": dtype,
        "config": {"workload": name + ": " + ", ".join(w.name for w in points),
                   "streams": streams,
                   "tokens_reduced_per_step": reduced,
                   "step": ("encoder_reduce + llm_prune" if inputs == "qk" else
                            "encoder_reduce_fused + llm_prune_fused")
                           + " for every keep budget of the sweep"},
        "timing": timing,
        "roofline": roof,
        "kernels": kernels,
    }
    del cases
    torch.cuda.empty_cache()
    if want_cpu:
        result["cpu_baseline"] = cpu_baseline(points, hosts, inputs=inputs, one_thread=one_thread)
    return result


def _head_dim(points):
    return next(w.encoder.head_dim for w in points if w.encoder is not None)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed steps of the headline workload (default: 30 for cfg4)")
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="cfg4",
                    choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "cfg6"],
                    help="the headline workload (default cfg4: the largest with both stages)")
    ap.add_argument("--also", default=None,
                    help="comma-separated workloads measured in the same run and reported under "
                         "other_workloads (default: cfg5,cfg2 beside the default headline, none "
                         "otherwise; 'none' switches them off)")
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
    ap.add_argument("--cold-ring", type=int, default=4,
                    help="independent input copies cycled through for the cold-cache figures "
                         "(0 or 1: warm figures only)")
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
    d_steps, d_warm = DEFAULT_STEPS[index]
    steps = args.steps if args.steps is not None else d_steps
    warmup = args.warmup if args.warmup is not None else d_warm
    also = args.also
    if also is None:
        also = "cfg5,cfg2" if (args.workload == "cfg4" and args.inputs == "qk") else "none"
    also = [a for a in also.split(",") if a and a != "none" and a != args.workload]

    head = measure(index, steps, warmup, args.inputs, args.streams, args.cold_ring,
                   not args.no_cpu_baseline, one_thread=False)
    result = {
        "metric": "visual tokens reduced/sec (encoder scan+merge, LLM prune)",
        "value": head["value"], "unit": head["unit"], "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": head["dtype"], "data": "synthetic",
        "config": head["config"], "timing": head["timing"], "roofline": head["roofline"],
        "kernels": head["kernels"],
    }
    if "cpu_baseline" in head:
        result["cpu_baseline"] = head["cpu_baseline"]
    others = {}
    for a in also:
        i = int(a[3:])
        s, w = DEFAULT_STEPS[i]
        rec = measure(i, s, w, args.inputs, args.streams, args.cold_ring,
                      not args.no_cpu_baseline, one_thread=(i == 2))
        rec["metric"] = result["metric"]
        others[a] = rec
    if others:
        result["other_workloads"] = others
    print(json.dumps(result))


if __name__ == "__main__":
    main()

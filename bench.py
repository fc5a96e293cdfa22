#!/usr/bin/env python3
"""Benchmark of the pruned W4A16 decode hot path on one MI355X.

A step is one pass of the whole hot path over one Llama-3-8B shaped decoder
layer at batch 1: q/k/v projections with the pruned RoPE of the fresh Q/K heads
as the epilogue of their launch, o_proj, gate/up with h = SiLU(gate) * up as the
epilogue of their launch, down -- seven W4A16 linears, the rotation and the
activation in four launches, all through the C ABI (--fused-mlp: the gated MLP as
its one persistent launch, three launches; --separate-rope: the rotation as its own launch).
Consecutive steps walk through a pool of distinct layers (a 32-layer
model, several GB), so every step streams its weights from HBM, not from the
256 MB Infinity Cache.  The timed region is ONE replay of a HIP graph that holds exactly
--steps consecutive steps.  Inputs are seeded synthetic stand-ins (random nibbles,
fp16 scales ~ U(0.005, 0.02), zeros ~ U{0..15}, activations ~ N(0, 1)).

Prints one JSON line (see the keys below); human-readable detail goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads as wl  # noqa: E402

METRIC = "µs and achieved HBM GB/s per pruned W4A16 decode linear (Llama-3-8B shapes)"
HBM_PEAK_GBS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2500.0
# HBM bytes per launch of the dominant kernel at pruning 15 %, from the two rocprofv3 --pmc runs (FETCH_SIZE,
# WRITE_SIZE) summarised in PMC_TRAFFIC_SOURCE, each scaled by what the same counter reads for a 256 MiB elementwise
# copy (--pmc-calib).  A separate run of this script under the profiler, NOT a measurement of the present run; other
# rates, formats and launch groupings were not measured (traffic = null).
PMC_TRAFFIC_SOURCE = "profiles/w4_gemv_llama3_8b_decode_p15.md"
PMC_TRAFFIC_BYTES = {("gate_up_silu", 15): 52480000, ("mlp", 15): 79742000}     # {(launch, rate): bytes}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


FMT = "f16"          # 16-bit format of scales, activations and outputs: "f16", or "bf16" with --bf16


def fdt(torch):
    return torch.bfloat16 if FMT == "bf16" else torch.float16


def dev16(torch, a):
    """Generated 16-bit array (float16, or uint16 bit patterns of bfloat16) -> device tensor."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


class Layer:
    """Device tensors and buffers of one decoder layer at one pruning rate."""

    def __init__(self, torch, uq, specs, rope, layer_index, rate, host_first=True, symmetric=False):
        self.specs = specs
        self.rope = rope
        self.lin = {}
        gen = torch.Generator(device="cuda")
        gen.manual_seed(wl.SEED_BASE + 1000 * rate + layer_index)
        for si, s in enumerate(specs):
            if layer_index == 0 and host_first:
                w = wl.gen_linear(wl.rng_for(1, 100 * rate + si), s.N, s.K, fmt=FMT)
                if symmetric:
                    w["zeros"] = None
                self.lin[s.name] = uq.QuantLinear.from_numpy(w)
                if not hasattr(self, "host"):
                    self.host = {}
                self.host[s.name] = w
            else:
                qw = (torch.randint(0, 2 ** 32, (s.N, s.K // 8), dtype=torch.int64, device="cuda", generator=gen)
                      - 2 ** 31).to(torch.int32)
                sc = (torch.rand((s.N, s.K // 128), device="cuda", generator=gen) * 0.015 + 0.005).to(fdt(torch))
                zr = torch.randint(0, 16, (s.N, s.K // 128), dtype=torch.uint8, device="cuda", generator=gen)
                self.lin[s.name] = uq.QuantLinear(qw, sc, None if symmetric else zr)


def interleave_o_proj(uq, layer, heads):
    """One-time re-layout of a layer's o_proj (uniql_w4_interleave): the words of every row head-interleaved, so that
    head-dimension pruning truncates the row.  The head-major copy stays for the comparison row."""
    layer.lin["o_proj_il"] = uq.uniql_w4_interleave(layer.lin["o_proj"], heads)


class DecodeStep:
    """Buffers shared by all layers plus the launch sequence of one step."""

    def __init__(self, torch, uq, specs, rope, M=1):
        self.torch, self.uq, self.specs, self.rope, self.M = torch, uq, specs, rope, M
        rng = wl.rng_for(1, 999)
        self.xin = {}
        self.yout = {}
        self.host_x = {}
        self._calls = {}
        shared = {"k_proj": "q_proj", "v_proj": "q_proj", "up_proj": "gate_proj"}   # same layer input
        for s in specs:
            if s.name in shared and shared[s.name] in self.xin:
                self.host_x[s.name] = self.host_x[shared[s.name]]
                self.xin[s.name] = self.xin[shared[s.name]]
            else:
                x = wl.gen_activations(rng, M, s.k_keep, fmt=FMT)
                self.host_x[s.name] = x
                self.xin[s.name] = dev16(torch, x)
            self.yout[s.name] = torch.empty((M, s.n_keep), dtype=fdt(torch), device="cuda")
        r = wl.gen_rope_inputs(rng, rope, fmt=FMT)
        self.host_rope = r
        self.pos = torch.from_numpy(r["positions"]).cuda()
        self.idx = torch.from_numpy(r["kept_idx"]).cuda()

    FUSED = (("q_proj", "k_proj", "v_proj"), ("gate_proj", "up_proj"))

    def multi_call(self, layer, names):
        """Marshalled uniql_w4_linear_multi call for a group of linears of one layer (cached)."""
        key = (id(layer), names)
        if key not in self._calls:
            sp = {s.name: s for s in self.specs}
            self._calls[key] = self.uq.MultiCall([layer.lin[n] for n in names], [sp[n].keep for n in names],
                                                 [self.xin[n] for n in names], [self.yout[n] for n in names])
        return self._calls[key]

    def rope_qk(self):
        q = self.yout["q_proj"].view(self.M, self.rope.Hq, self.rope.D_keep)
        k = self.yout["k_proj"].view(self.M, self.rope.Hkv, self.rope.D_keep)
        self.uq.uniql_pruned_rope(q, k, self.pos, self.idx, self.rope.D_full, self.rope.theta)

    def qkv_rope_call(self, layer):
        """Marshalled uniql_w4_qkv_rope call of one layer (cached): q, k, v and the rotation in one launch."""
        key = (id(layer), "qkv_rope")
        if key not in self._calls:
            sp = {s.name: s for s in self.specs}
            names = self.FUSED[0]
            r = self.rope
            self._calls[key] = self.uq.QkvRopeCall(
                [layer.lin[n] for n in names], [sp[n].keep for n in names], self.xin["q_proj"][0],
                self.yout["q_proj"].view(r.Hq, r.D_keep), self.yout["k_proj"].view(r.Hkv, r.D_keep),
                self.yout["v_proj"].view(-1), self.pos[:1], self.idx, r.D_full, r.theta)
        return self._calls[key]

    def gate_up_call(self, layer):
        """Marshalled uniql_w4_gate_up_silu call of one layer (cached): gate, up and SiLU(gate) * up in one launch."""
        key = (id(layer), "gate_up_silu")
        if key not in self._calls:
            sp = {s.name: s for s in self.specs}
            if not hasattr(self, "hbuf"):
                self.hbuf = self.torch.empty((sp["gate_proj"].n_keep,), dtype=fdt(self.torch), device="cuda")
            self._calls[key] = self.uq.GateUpCall([layer.lin["gate_proj"], layer.lin["up_proj"]],
                                                  [sp["gate_proj"].keep, sp["up_proj"].keep],
                                                  self.xin["gate_proj"][0], self.hbuf)
        return self._calls[key]

    def mlp_call(self, layer):
        """Marshalled uniql_w4_mlp call of one layer (cached): gate, up, SiLU(gate) * up and down in one launch."""
        key = (id(layer), "mlp")
        if key not in self._calls:
            sp = {s.name: s for s in self.specs}
            if not hasattr(self, "mlp_work"):
                self.mlp_work = self.uq.mlp_workspace(sp["gate_proj"].N)
            self._calls[key] = self.uq.MlpCall([layer.lin["gate_proj"], layer.lin["up_proj"], layer.lin["down_proj"]],
                                               [sp["gate_proj"].keep, sp["up_proj"].keep, sp["down_proj"].keep],
                                               self.xin["gate_proj"][0], self.yout["down_proj"][0], self.mlp_work)
        return self._calls[key]

    o_name = "o_proj_il"      # which copy of o_proj the step uses ("o_proj": head-major, as the ABI stores it by default)

    def run(self, layer, only=None, fused=True, fuse_rope=True, fuse_mlp=True):
        """One step: q/k/v with the rotation of the fresh Q/K heads (one launch; fuse_rope=False: one
        launch for q/k/v, one for the rotation), o_proj, gate/up (one launch), down.
        only = a linear name or a tuple of names: just that launch (for attribution)."""
        uq = self.uq
        if only is not None:
            if only == "qkv_rope":
                self.qkv_rope_call(layer).run()
            elif only == "gate_up_silu":
                self.gate_up_call(layer).run()
            elif only == "gate_up_probe":
                self.gate_up_call(layer).run_probe()
            elif only == "mlp":
                self.mlp_call(layer).run()
            elif isinstance(only, tuple):
                self.multi_call(layer, only).run()
            else:
                s = next(s for s in self.specs if s.name == only.replace("_il", ""))
                uq.uniql_w4_linear(layer.lin[only], s.keep, self.xin[s.name], self.yout[s.name])
            return
        if not fused:
            for s in self.specs:
                uq.uniql_w4_linear(layer.lin[s.name], s.keep, self.xin[s.name], self.yout[s.name])
                if s.name == "k_proj":
                    self.rope_qk()
            return
        sp = {s.name: s for s in self.specs}
        if fuse_rope and self.M == 1:
            self.qkv_rope_call(layer).run()
        else:
            self.multi_call(layer, self.FUSED[0]).run()
            self.rope_qk()
        uq.uniql_w4_linear(layer.lin[self.o_name], sp["o_proj"].keep, self.xin["o_proj"], self.yout["o_proj"])
        if self.M == 1 and fuse_mlp:
            self.mlp_call(layer).run()         # the whole gated MLP (Eq. 1) in one launch
            return
        if self.M == 1:
            self.gate_up_call(layer).run()     # gate, up and h = SiLU(gate) * up (Eq. 1) in one launch
        else:
            self.multi_call(layer, self.FUSED[1]).run()
        uq.uniql_w4_linear(layer.lin["down_proj"], sp["down_proj"].keep, self.xin["down_proj"], self.yout["down_proj"])


def time_events(torch, fn, iters):
    """Average GPU milliseconds of fn() over iters back-to-back calls (events on the launch stream)."""
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    s.record()
    for i in range(iters):
        fn(i)
    e.record()
    torch.cuda.synchronize()
    return s.elapsed_time(e) / iters


def cpu_baseline(specs, rope, layer0, step, M):
    """The oracle, as it stands, on the host cores: one full layer step (all seven linears + RoPE)."""
    import oracle
    cores = min(oracle.max_threads(), int(os.environ.get("OMP_NUM_THREADS", "16") or 16), 16)
    oracle.set_threads(cores)
    r = step.host_rope
    t0 = time.perf_counter()
    reps = 0
    while reps < 3 or time.perf_counter() - t0 < 10.0:      # about 10 s of CPU work, at least 3 passes
        for s in specs:
            w = layer0.host[s.name]
            oracle.w4_linear(w["qweight"], w["scales"], w["zeros"], step.host_x[s.name], s.keep, fmt=FMT)
        oracle.pruned_rope(r["q"], r["k"], r["positions"], r["kept_idx"], rope.D_full, rope.theta, fmt=FMT)
        reps += 1
    dt = (time.perf_counter() - t0) / reps
    nbytes = sum(s.algorithmic_bytes(M) for s in specs) + rope.algorithmic_bytes()
    # one thread, on a bounded sample: the q_proj linear alone (a few seconds)
    oracle.set_threads(1)
    q = next(s for s in specs if s.name == "q_proj")
    w = layer0.host[q.name]
    t1 = time.perf_counter()
    oracle.w4_linear(w["qweight"], w["scales"], w["zeros"], step.host_x[q.name], q.keep, fmt=FMT)
    dt1 = time.perf_counter() - t1
    oracle.set_threads(cores)
    return {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"{reps} passes of one full decode layer step (7 linears + RoPE, {nbytes / 1e6:.1f} MB "
                      f"algorithmic each), {dt:.3f} s per pass, OpenMP over output rows",
            "one_thread_value": q.algorithmic_bytes(M) / dt1 / 1e9,
            "one_thread_sample": f"q_proj alone ({q.algorithmic_bytes(M) / 1e6:.1f} MB), {dt1:.3f} s"}


def graph_time_us(torch, side, fn, n_inner, reps=6):
    """Mean GPU microseconds of one fn(i) call, issued n_inner times back to back inside a HIP graph."""
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        for i in range(n_inner):
            fn(i)
    g.replay()
    return time_events(torch, lambda i: g.replay(), reps) * 1e3 / n_inner


def detail_report(torch, uq, side):
    """Other workloads of the benchmark configurations, each as isolated launches over a pool of
    distinct weight copies: the three pruning rates, Qwen2.5-7B and Mamba2-2.7B shapes, the
    prefill-sized MFMA GEMM and the prefill RoPE.  Returned as a dict; printed to stderr."""
    rep = {}

    def pool_for(spec, min_bytes=1.0e9, max_copies=32):
        nb = spec.N * spec.K // 2
        n = int(max(2, min(max_copies, min_bytes // nb + 1)))
        gen = torch.Generator(device="cuda")
        gen.manual_seed(wl.SEED_BASE + spec.N + spec.K)
        out = []
        for _ in range(n):
            qw = (torch.randint(0, 2 ** 32, (spec.N, spec.K // 8), dtype=torch.int64, device="cuda", generator=gen)
                  - 2 ** 31).to(torch.int32)
            sc = (torch.rand((spec.N, spec.K // 128), device="cuda", generator=gen) * 0.015 + 0.005).to(fdt(torch))
            zr = torch.randint(0, 16, (spec.N, spec.K // 128), dtype=torch.uint8, device="cuda", generator=gen)
            out.append(uq.QuantLinear(qw, sc, zr))
        return out

    def time_linear(spec, M, pool):
        x = torch.randn((M, spec.k_keep), dtype=fdt(torch), device="cuda")
        y = torch.empty((M, spec.n_keep), dtype=fdt(torch), device="cuda")
        us = graph_time_us(torch, side, lambda i: uq.uniql_w4_linear(pool[i % len(pool)], spec.keep, x, y), len(pool))
        nbytes = spec.algorithmic_bytes(M)
        return {"M": M, "MB": round(nbytes / 1e6, 3), "us": round(us, 2), "GBps": round(nbytes / us / 1e3, 1),
                "frac_hbm": round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4),
                "TFLOPs": round(spec.flops(M) / us / 1e6, 2)}

    # Llama-3-8B shapes at the three rates (M = 1)
    pools = {}
    for rate in (0, 15, 35):
        rows = {}
        for spec in wl.llama3_8b_layer(rate):
            key = (spec.N, spec.K)
            if key not in pools:
                pools[key] = pool_for(spec)
            rows[spec.name] = time_linear(spec, 1, pools[key])
        rows["layer_us"] = round(sum(v["us"] for v in rows.values()), 2)
        rep[f"llama3_8b_p{rate}"] = rows
    # prefill-sized GEMM on the gate/up and down shapes, 15 %
    for spec in wl.prefill_linears(15):
        for M in (256, 1024, 4096):
            r = time_linear(spec, M, pools[(spec.N, spec.K)][:4])
            r["frac_mfma"] = round(r["TFLOPs"] / MFMA_F16_PEAK_TFLOPS, 4)
            rep[f"prefill_{spec.name}_M{M}"] = r
    pools.clear()
    torch.cuda.empty_cache()
    # Qwen2.5-7B shapes, 25 %, batch 1 / 8 / 16
    qpools = {}
    for spec in wl.qwen25_7b_layer(25):
        key = (spec.N, spec.K)
        if key not in qpools:
            qpools[key] = pool_for(spec)
        for M in (1, 8, 16):
            rep[f"qwen25_7b_p25_{spec.name}_M{M}"] = time_linear(spec, M, qpools[key])
    # the same decode batches with q + k + v and gate + up as one uniql_w4_linear_multi call each (one launch per call)
    qspecs = {s.name: s for s in wl.qwen25_7b_layer(25)}
    for label, names in (("qkv", ("q_proj", "k_proj", "v_proj")), ("gate_up", ("gate_proj", "up_proj"))):
        members = [qspecs[n] for n in names]
        mpools = []
        for j, sp in enumerate(members):
            pl = qpools[(sp.N, sp.K)]
            mpools.append([pl[(i + j * (len(pl) // 2)) % len(pl)] for i in range(len(pl))])   # members never share a matrix
        npool = min(len(pl) for pl in mpools)
        for M in (8, 16):
            x = torch.randn((M, members[0].k_keep), dtype=fdt(torch), device="cuda")
            ys = [torch.empty((M, sp.n_keep), dtype=fdt(torch), device="cuda") for sp in members]
            keeps = [sp.keep for sp in members]
            us = graph_time_us(torch, side, lambda i: uq.uniql_w4_linear_multi([pl[i % npool] for pl in mpools], keeps, [x] * len(members), ys), npool)
            nbytes = sum(sp.algorithmic_bytes(M) for sp in members) - (len(members) - 1) * M * members[0].k_keep * 2
            rep[f"qwen25_7b_p25_{label}_one_call_M{M}"] = {"M": M, "MB": round(nbytes / 1e6, 3), "us": round(us, 2),
                                                            "GBps": round(nbytes / us / 1e3, 1),
                                                            "frac_hbm": round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4)}
    # gate + up + SiLU(gate) * up of the same decode batches in one launch
    gsp = qspecs["gate_proj"]
    gpl = qpools[(gsp.N, gsp.K)]
    for M in (8, 16):
        x = torch.randn((M, gsp.k_keep), dtype=fdt(torch), device="cuda")
        h = torch.empty((M, gsp.n_keep), dtype=fdt(torch), device="cuda")
        half = len(gpl) // 2
        us = graph_time_us(torch, side, lambda i: uq.uniql_w4_gate_up_silu_batch([gpl[i % half], gpl[half + i % half]], [gsp.keep, gsp.keep], x, h), half)
        nbytes = 2 * gsp.algorithmic_bytes(M) - M * gsp.k_keep * 2 - M * gsp.n_keep * 2
        rep[f"qwen25_7b_p25_gate_up_silu_M{M}"] = {"M": M, "MB": round(nbytes / 1e6, 3), "us": round(us, 2),
                                                    "GBps": round(nbytes / us / 1e3, 1),
                                                    "frac_hbm": round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4)}
    qpools.clear()
    torch.cuda.empty_cache()
    # Mamba2-2.7B shapes, 15 %
    for spec in wl.mamba2_2p7b_layer(15):
        rep[f"mamba2_2p7b_p15_{spec.name}"] = time_linear(spec, 1, pool_for(spec))
    # the same block with every SSM head cut to 54 of 64 channels and the B / C parts to 108 of 128 state channels
    for spec in wl.mamba2_2p7b_layer_heads_and_state(15):
        rep[f"mamba2_2p7b_heads_state_p15_{spec.name}"] = time_linear(spec, 1, pool_for(spec))
    torch.cuda.empty_cache()
    # codes of 8, 6 and 3 bits (Eq. 3 with N = 8, 6, 3) on the gate / up and down shapes, 15 %, M = 1
    for bits in (8, 6, 3):
        for spec in wl.llama3_8b_layer(15):
            if spec.name not in ("gate_proj", "down_proj"):
                continue
            gen = torch.Generator(device="cuda")
            gen.manual_seed(wl.SEED_BASE + bits + spec.N)
            poolb = []
            f = 16.0 / (1 << bits)
            for _ in range(12 if bits == 8 else 16):
                qw = (torch.randint(0, 2 ** 32, (spec.N, spec.K * bits // 32), dtype=torch.int64, device="cuda", generator=gen)
                      - 2 ** 31).to(torch.int32)
                sc = (torch.rand((spec.N, spec.K // 128), device="cuda", generator=gen) * (0.015 * f) + 0.005 * f).to(fdt(torch))
                zr = torch.randint(0, 1 << bits, (spec.N, spec.K // 128), dtype=torch.uint8, device="cuda", generator=gen)
                poolb.append(uq.QuantLinear(qw, sc, zr, bits=bits))
            r = time_linear(spec, 1, poolb)
            # bits / 8 bytes per code and a byte per zero point instead of the 4-bit format's halves
            nbb = (spec.algorithmic_bytes(1) - spec.n_keep * spec.k_keep // 2 + spec.n_keep * spec.k_keep * bits // 8
                   + spec.n_keep * spec.groups_touched() // 2)
            r.update({"MB": round(nbb / 1e6, 3), "GBps": round(nbb / r["us"] / 1e3, 1), "frac_hbm": round(nbb / r["us"] / 1e3 / HBM_PEAK_GBS, 4)})
            rep[f"llama3_8b_p15_w{bits}_{spec.name}_M1"] = r
            del poolb
        torch.cuda.empty_cache()
    # the 4-bit output head (128256 x 4096), M = 1: the same GEMV at a size where launch latency is small
    spec = wl.lm_head_llama3()
    rep["lm_head_llama3_M1"] = time_linear(spec, 1, pool_for(spec, min_bytes=1.3e9, max_copies=5))
    torch.cuda.empty_cache()
    # 4-bit embedding rows (128256 x 4096 table) gathered for one token and for a 4096-token prompt
    emb = pool_for(spec, min_bytes=1.0, max_copies=2)[0]
    for T in (1, 4096):
        ids = torch.randint(0, spec.N, (T,), dtype=torch.int32, device="cuda")
        outs = [torch.empty((T, spec.K), dtype=fdt(torch), device="cuda") for _ in range(4)]
        us = graph_time_us(torch, side, lambda i: uq.uniql_w4_embedding(emb, ids, out=outs[i % 4]), 8)
        nb = T * (spec.K // 2 + spec.K // 128 * 2.5 + 4 + 2 * spec.K)
        rep[f"embedding_llama3_T{T}"] = {"MB": round(nb / 1e6, 3), "us": round(us, 2), "GBps": round(nb / us / 1e3, 1),
                                         "frac_hbm": round(nb / us / 1e3 / HBM_PEAK_GBS, 4)}
    del emb
    torch.cuda.empty_cache()
    # on-device repack of the kept channels (Llama gate_proj: rows; down_proj: column prefix), 15 %
    for spec in wl.prefill_linears(15):
        if spec.name not in ("gate_up_proj", "gate_proj", "down_proj"):
            continue
        src = pool_for(spec, min_bytes=1.2e8, max_copies=4)
        outs = [uq.uniql_w4_repack(src[0], spec.keep)[0] for _ in range(4)]
        us = graph_time_us(torch, side, lambda i: uq.uniql_w4_repack(src[i % len(src)], spec.keep, out=outs[i % 4]), 8)
        n_out, k_out = outs[0].N, outs[0].K
        nb = 2 * n_out * (k_out // 2 + k_out // 128 * 3)       # codes, scale and zero point: read once, written once
        rep[f"repack_{spec.name}_p15"] = {"MB": round(nb / 1e6, 3), "us": round(us, 2), "GBps": round(nb / us / 1e3, 1),
                                          "frac_hbm": round(nb / us / 1e3 / HBM_PEAK_GBS, 4)}
        del src, outs
        torch.cuda.empty_cache()
    # RoPE: decode and prefill
    for name, rs in (("rope_decode_llama_p15", wl.llama3_8b_rope(15, T=1)), ("rope_prefill_llama_p15", wl.prefill_rope(15, 4096))):
        r = wl.gen_rope_inputs(wl.rng_for(4, 7), rs, fmt=FMT)
        bufs = [(dev16(torch, r["q"]), dev16(torch, r["k"])) for _ in range(8 if rs.T > 1 else 2)]
        pos, idx = torch.from_numpy(r["positions"]).cuda(), torch.from_numpy(r["kept_idx"]).cuda()
        us = graph_time_us(torch, side, lambda i: uq.uniql_pruned_rope(bufs[i % len(bufs)][0], bufs[i % len(bufs)][1],
                                                                      pos, idx, rs.D_full, rs.theta), 16)
        nb = rs.algorithmic_bytes()
        rep[name] = {"MB": round(nb / 1e6, 3), "us": round(us, 2), "GBps": round(nb / us / 1e3, 1),
                     "frac_hbm": round(nb / us / 1e3 / HBM_PEAK_GBS, 4)}
    for k, v in rep.items():
        log(f"  {k}: {v}")
    return rep


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=640)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--prune", type=int, default=15, help="pruning rate in percent (0, 15, 35)")
    ap.add_argument("--layers", type=int, default=32, help="distinct layers in the weight pool")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying HIP graphs")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--separate-rope", action="store_true",
                    help="run the rotation as its own launch after q/k/v instead of as the epilogue of their launch")
    ap.add_argument("--fused-mlp", action="store_true",
                    help="run the gated MLP (gate+up+SiLU, then down) as its one persistent launch (uniql_w4_mlp) instead of "
                         "two launches; the two take the same time on the device, the step is reported on the two launches")
    ap.add_argument("--o-head-major", action="store_true",
                    help="run o_proj on the head-major words the ABI stores by default (the pruned dims of every head are then "
                         "fetched with the 32-byte sectors they share with kept ones) instead of the head-interleaved re-layout")
    ap.add_argument("--pmc-calib", action="store_true",
                    help="also launch a plain 256 MiB elementwise copy four times: the kernel of known size that "
                         "scales rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--symmetric", action="store_true",
                    help="matrices without zero points (Eq. 3's symmetric scheme, every z = 8): no zero point is stored or "
                         "read; not the benchmark configuration, which is asymmetric")
    ap.add_argument("--bf16", action="store_true",
                    help="scales, activations and outputs in bfloat16 (the paper's compute type, Sec. 4.1) instead of the "
                         "benchmark configuration's fp16")
    ap.add_argument("--no-detail", action="store_true",
                    help="skip the other benchmark configurations (three rates, Qwen / Mamba shapes, prefill GEMM, RoPE, output head)")
    ap.add_argument("--detail", action="store_true", help="(default now; kept for old command lines)")
    args = ap.parse_args()
    global FMT
    FMT = "bf16" if args.bf16 else "f16"
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build measures the one-GPU hot path only; run with --gpus 1")
    if args.steps < 1 or args.warmup < 0:
        sys.exit("bench.py: --steps must be at least 1 and --warmup at least 0")

    import torch
    import paper_2512_03383_amd as uq
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    uq.lib()
    torch.cuda.set_device(0)
    M = 1
    rate = args.prune
    specs = wl.llama3_8b_layer(rate)
    rope = wl.llama3_8b_rope(rate, T=M)
    layers = [Layer(torch, uq, specs, rope, i, rate, symmetric=args.symmetric) for i in range(args.layers)]
    for L in layers:
        interleave_o_proj(uq, L, rope.Hq)
    step = DecodeStep(torch, uq, specs, rope, M)
    if args.o_head_major:
        step.o_name = "o_proj"
    nl = len(layers)
    # without zero points a touched group costs its 2-byte scale only
    lin_bytes = {s.name: s.algorithmic_bytes(M) - (s.n_keep * s.groups_touched() // 2 if args.symmetric else 0) for s in specs}
    step_bytes = sum(lin_bytes.values()) + rope.algorithmic_bytes()
    pool_gb = sum(s.N * s.K / 2 for s in specs) * args.layers / 1e9
    log(f"pool: {args.layers} layers, {pool_gb:.2f} GB of packed weights; step = {step_bytes / 1e6:.2f} MB algorithmic")

    fuse_rope, fuse_mlp = not args.separate_rope, args.fused_mlp

    def run_step(i):
        step.run(layers[i % nl], fuse_rope=fuse_rope, fuse_mlp=fuse_mlp)

    # one eager pass (also warms the per-device caches of the library), then capture two HIP graphs: --warmup and --steps
    # CONSECUTIVE steps each, walking on through the layer pool (the steady state of a decode loop)
    for i in range(nl):
        run_step(i)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    g_warm, g_timed = None, None
    if not args.no_graph:
        if args.warmup:
            g_warm = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_warm, stream=side):
                for i in range(args.warmup):
                    run_step(i)
        g_timed = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_timed, stream=side):
            for i in range(args.steps):
                run_step(args.warmup + i)
        torch.cuda.synchronize()

    if args.no_graph:
        for i in range(args.warmup):
            run_step(i)
    elif g_warm is not None:
        g_warm.replay()
    torch.cuda.synchronize()
    ev_s, ev_e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev_s.record()
    if args.no_graph:
        for i in range(args.steps):
            run_step(args.warmup + i)
    else:
        g_timed.replay()                      # exactly --steps steps
    ev_e.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    ms_per_step_gpu = ev_s.elapsed_time(ev_e) / args.steps
    value = step_bytes / (ms_per_step * 1e-3) / 1e9

    # ---- attribution: duration of each launch of the step (and of the launches it replaces), measured with HIP events
    # on the launch stream around a graph that issues that one launch back to back over the whole layer pool
    # (cold weights every launch, no host launch cost inside the bracket)
    first = "qkv_rope" if fuse_rope else DecodeStep.FUSED[0]
    names = [first, "o_proj_il", "o_proj", "gate_up_silu", "down_proj", "mlp", "gate_up_probe"]
    lin_bytes = dict(lin_bytes)
    for grp in DecodeStep.FUSED:
        lin_bytes[grp] = sum(lin_bytes[n] for n in grp)
    lin_bytes["qkv_rope"] = lin_bytes[DecodeStep.FUSED[0]] + rope.algorithmic_bytes()
    # gate + up with the activation as epilogue writes one hidden vector instead of two
    lin_bytes["gate_up_silu"] = lin_bytes[DecodeStep.FUSED[1]] - 2 * next(s for s in specs if s.name == "gate_proj").n_keep
    lin_bytes["gate_up_probe"] = lin_bytes["gate_up_silu"]
    lin_bytes["o_proj_il"] = lin_bytes["o_proj"]
    lin_bytes["mlp"] = lin_bytes["gate_up_silu"] + lin_bytes["down_proj"]
    if FMT == "bf16" or args.symmetric:
        names.remove("gate_up_probe")        # the probe exists for fp16 matrices with zero points
    iso_us, min_us, warm_us = {}, {}, {}
    for n in names:
        if args.no_graph:
            ms = time_events(torch, lambda i, n=n: step.run(layers[i % nl], only=n), 8 * nl)
            iso_us[n] = ms * 1e3
            continue
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for L in layers:
                step.run(L, only=n)
        g.replay()
        ms = time_events(torch, lambda i: g.replay(), 8)
        iso_us[n] = ms * 1e3 / nl
        # the fastest of eight replays, and the same launch repeated on ONE layer: its weights then
        # come from the 256 MB Infinity Cache / L2, not from HBM (labelled warm, not a bandwidth claim)
        min_us[n] = min(time_events(torch, lambda i: g.replay(), 1) for _ in range(8)) * 1e3 / nl
        gw = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gw, stream=side):
            for _ in range(nl):
                step.run(layers[0], only=n)
        gw.replay()
        warm_us[n] = time_events(torch, lambda i: gw.replay(), 8) * 1e3 / nl
    assert uq.uniql_w4_mlp_status(step.mlp_work) == 0, "a fused MLP launch gave up waiting for its blocks"
    label = {"qkv_rope": "q_proj+k_proj+v_proj+rope", "gate_up_silu": "gate_proj+up_proj+silu",
             "o_proj_il": "o_proj (head-interleaved words)", "o_proj": "o_proj (head-major words)",
             "mlp": "gate_proj+up_proj+silu+down_proj (one launch)",
             "gate_up_probe": "loads of gate_proj+up_proj+silu without its arithmetic (persistent read probe)"}
    per_linear = {}
    for n in names:
        v = {"MB": round(lin_bytes[n] / 1e6, 3), "us": round(iso_us[n], 3),
             "GBps": round(lin_bytes[n] / (iso_us[n] * 1e-6) / 1e9, 1),
             "frac_of_peak": round(lin_bytes[n] / (iso_us[n] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}
        if n in min_us:
            v.update({"min_us": round(min_us[n], 3), "warm_cache_us": round(warm_us[n], 3)})
        per_linear["+".join(n) if isinstance(n, tuple) else label.get(n, n)] = v
    for n, v in per_linear.items():
        log(f"  {n:28s} {v}")
    in_step = [first, step.o_name] + (["mlp"] if fuse_mlp else ["gate_up_silu", "down_proj"])
    sum_us = sum(iso_us[n] for n in in_step)

    # the dominant kernel of the step: the launch that serves the gated MLP (or, with --separate-mlp, gate + up)
    dom = "mlp" if fuse_mlp else "gate_up_silu"
    dom_bytes, dom_us = float(lin_bytes[dom]), float(iso_us[dom])
    achieved = dom_bytes / (dom_us * 1e-6) / 1e9
    zp, bf = str(not args.symmetric).lower(), str(FMT == "bf16").lower()
    dom_kernel = (f"w4_mlp_stream_kernel<2,6,{zp},{bf}> (gate_proj + up_proj + SiLU(gate)*up, then down_proj, one persistent launch)"
                  if fuse_mlp else f"w4_gemv_stream_kernel<2,2,{zp},{bf},false> (gate_proj + up_proj + SiLU(gate)*up in one launch)")
    # read-stream ceilings for the same byte count: plain 128-bit loads in a grid of short-lived blocks, and (for the
    # gate + up launch) the kernel's own persistent walk with every load and no arithmetic; the better one counts
    probe_out = torch.empty(1 << 16, dtype=torch.int32, device="cuda")
    nb = int(dom_bytes) // 8192 * 8192
    probe_buf = torch.empty(2 * 2 ** 30 // 4, dtype=torch.int32, device="cuda")      # 2 GB to walk through
    n_slots = max(1, probe_buf.numel() * 4 // nb)
    probe_src = [probe_buf[(i % n_slots) * (nb // 4):] for i in range(nl)]
    if not args.no_graph:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for t in probe_src:
                uq.uniql_stream_read_probe(t, nb, probe_out)
        g.replay()
        ceil_us = time_events(torch, lambda i: g.replay(), 8) * 1e3 / len(probe_src)
    else:
        ceil_us = time_events(torch, lambda i: uq.uniql_stream_read_probe(probe_src[i % len(probe_src)], nb, probe_out),
                              8 * len(probe_src)) * 1e3
    ceil_gbs = nb / (ceil_us * 1e-6) / 1e9
    ceilings = {"grid_of_blocks_GBps": round(ceil_gbs, 1)}
    if not fuse_mlp and "gate_up_probe" in iso_us:
        ceilings["persistent_walk_GBps"] = round(lin_bytes["gate_up_probe"] / (iso_us["gate_up_probe"] * 1e-6) / 1e9, 1)
    best_ceiling = max(ceilings.values())
    log(f"  step: wall {ms_per_step * 1e3:.2f} us, gpu events {ms_per_step_gpu * 1e3:.2f} us, sum of its launches "
        f"{sum_us:.2f} us; read-stream ceiling for {nb / 1e6:.1f} MB: {ceil_us:.2f} us = {ceil_gbs:.0f} GB/s")

    out = {
        "metric": METRIC, "value": round(value, 2), "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": FMT,
        "data": "synthetic",
        "config": {"workload": f"Llama-3-8B shaped decode layer, batch 1, int4 group-128 weights{' without zero points (symmetric)' if args.symmetric else ''}{', bfloat16 activations' if FMT == 'bf16' else ''}, "
                               f"pruning {rate}% (q+k+v{' with the pruned RoPE as epilogue' if fuse_rope else ', pruned RoPE'}, "
                               f"o{' on head-interleaved words (one-time re-layout, pruning still a run-time argument)' if step.o_name == 'o_proj_il' else ''}, "
                               f"{'the gated MLP gate+up+SiLU(gate)*up+down as one persistent launch' if fuse_mlp else 'gate+up with SiLU(gate)*up as epilogue, down'}: "
                               f"W4A16 GEMV launches), {args.layers}-layer weight pool streamed from HBM",
                   "prune_pct": rate, "M": M,
                   "launch": f"one HIP graph of {args.steps} consecutive steps over the layer pool" if g_timed is not None else "eager",
                   "step_algorithmic_MB": round(step_bytes / 1e6, 3)},
        "us_per_step_gpu_events": round(ms_per_step_gpu * 1e3, 3),
        "us_sum_of_step_launches": round(sum_us, 3),
        "per_linear": per_linear,
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": None if (args.symmetric or FMT == "bf16") else PMC_TRAFFIC_BYTES.get((dom, rate)),
                     "traffic_unit": "bytes per launch (rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE, copy-kernel scaled)",
                     "traffic_source": f"{PMC_TRAFFIC_SOURCE}: a separate run of this script under rocprofv3, not this run",
                     "kernel": dom_kernel,
                     "bytes_per_launch": int(dom_bytes), "us_per_launch": round(dom_us, 3),
                     "stream_ceilings": ceilings,
                     "stream_ceiling_GBps": round(best_ceiling, 1),
                     "frac_of_stream_ceiling": round(achieved / best_ceiling, 4),
                     "how": "algorithmic bytes of the launch / its mean duration, HIP events on the launch "
                            "stream around a graph of back-to-back launches over the layer pool (cold HBM)"},
    }
    if args.pmc_calib:
        src = torch.ones(64 * 2 ** 20, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(4):
            torch.add(src, 1, out=dst)      # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(specs, rope, layers[0], step, M)
    if not args.no_detail:
        del layers, g_warm, g_timed, probe_buf, probe_src
        step._calls.clear()
        torch.cuda.empty_cache()
        t_d = time.perf_counter()
        out["detail"] = detail_report(torch, uq, side)
        log(f"  (other configurations: {time.perf_counter() - t_d:.1f} s)")
    print(json.dumps(out, ensure_ascii=False), flush=True)


if __name__ == "__main__":
    main()

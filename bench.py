#!/usr/bin/env python3
"""Benchmark of the MoLE lookup-expert layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-extras]

One "step" is one pass of the inference hot path over one batch of synthetic input: for the
headline workload (410M-shaped decode: 24 MoLE layers x 256 tokens, N=16, d=1024, bf16 tables
resident in HBM, Zipf(1.1) token ids) that is router + softmax + row gather + gate-weighted sum +
shared-FFN add for all 24 layers.  Inputs are resident in HBM when the clock starts; 16
pre-generated id batches rotate so that successive steps do not replay identical rows.
The script prints ONE JSON line (kept under 8 KB).  Besides the contract fields it carries
  roofline      the forward kernel against the HBM roofline: `achieved` / `frac` on the algorithmic bytes
                (every token's own rows) over the launch duration, `traffic` / `traffic_frac` on the
                counter-measured bytes (rocprofv3 summary under profiles/, with the hash of the kernel
                sources it was taken on), `moved_frac` on the bytes that have to move (each distinct id
                once), and `also`: the same fractions for the other configurations (prefill with uniform
                and Zipf ids, with the plan; small decode batches; offload fetch against the host link; LUT
                build against the MFMA peak)
  cpu_baseline  the fp64 CPU oracle timed on the host cores on the same workload
  other_ms      milliseconds of every other workload and variant; --full adds their complete entries
                under `other`.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time
import traceback

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16
HOST_LINK_GBS = 64.0            # PCIe Gen5 x16, one direction
N_ID_BATCHES = 16


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="decode410m")
    ap.add_argument("--plan", action="store_true",
                    help="the timed step is the forward given a plan of mole_dedup_ids (plans computed "
                         "beforehand, one per id batch); for profiling that path")
    ap.add_argument("--runs", action="store_true",
                    help="with --plan: also pass MOLE_FLAG_RUNS (tokens with equal ids summed together on the matrix pipe)")
    ap.add_argument("--dedup-forward", action="store_true",
                    help="the timed step is mole_dedup_forward (dedup and forward in id order as one call); for the "
                         "profiles of the prefill workloads")
    ap.add_argument("--no-extras", action="store_true", help="only the headline workload")
    ap.add_argument("--full", action="store_true", help="also print the complete entries of the other workloads")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--only-build", action="store_true",
                    help="time mole_build_lut on one 410M layer and print its entry alone (for profiling)")
    ap.add_argument("--only-nf", action="store_true",
                    help="only the dequantising forward on --workload, NF4 and NF3 (used for its profile)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch a plain 1 GiB device copy (reference for rocprofv3 byte counters)")
    return ap.parse_args()


class Layers:
    """Device-resident state of one workload: tables, router weights, activations, id batches."""

    def __init__(self, w, torch, mb, wl, ids_kind=None):
        self.w, self.torch, self.mb = w, torch, mb
        dev = "cuda"
        tdt = torch.bfloat16 if w.dtype == wl.BF16 else torch.float32
        self.code = mb.MOLE_BF16 if w.dtype == wl.BF16 else mb.MOLE_F32
        self.tabs = torch.empty((w.L, w.V, w.N, w.d), dtype=tdt, device=dev)
        for l in range(w.L):
            wl.device_table(w, l, dev, out=self.tabs[l])
        g = torch.Generator(device=dev)
        g.manual_seed(1000 + w.seed)
        self.h = torch.randn((w.L, w.T, w.d), generator=g, device=dev).to(tdt)
        self.shared = torch.randn((w.L, w.T, w.d), generator=g, device=dev).to(tdt)
        self.W_r = (torch.randn((w.L, w.d, w.N), generator=g, device=dev) * 0.02).to(tdt)
        self.out = torch.empty_like(self.h)
        import numpy as np
        ww = w if ids_kind is None else wl.scaled(w, ids=ids_kind)
        self.ids_host = np.stack([wl.token_ids(ww, b) for b in range(N_ID_BATCHES)])
        self.ids = torch.from_numpy(self.ids_host).to(dev)
        self.err = torch.zeros((1,), dtype=torch.int32, device=dev)
        self.plan = torch.empty((mb.mole_dedup_workspace(w.T, w.V) // 4,), dtype=torch.int32, device=dev)
        self.uniq = torch.empty((w.T,), dtype=torch.int32, device=dev)
        self.inv = torch.empty((w.T,), dtype=torch.int32, device=dev)
        self.n_uniq = torch.zeros((1,), dtype=torch.int32, device=dev)

    def forward(self, i, stream, dedup=False, table=None, slot=None, rows=None, table_stride=None):
        w, mb = self.w, self.mb
        tab = self.tabs if table is None else table
        mb.mole_lookup_forward_layers(
            tab, w.V * w.N * w.d if table_stride is None else table_stride, self.ids[i % N_ID_BATCHES], slot,
            self.h, self.W_r, self.shared, None, self.out, w.T * w.d, None, None, self.err,
            w.L, w.T, w.V if rows is None else rows, w.d, w.N, self.code,
            mb.MOLE_FLAG_DEDUP if dedup else 0, self.plan if dedup else None, stream=stream)

    def dedup(self, i, stream):
        self.mb.mole_dedup_ids(self.ids[i % N_ID_BATCHES], self.w.T, self.w.V, self.uniq, self.inv, self.n_uniq,
                               self.err, self.plan, stream=stream)

    def dedup_forward(self, i, stream):
        """mole_dedup_forward: dedup and forward in id order as one call (for large batches at N = 32 the dedup
        runs beside the router inside one launch; other shapes run the two calls)."""
        w, mb = self.w, self.mb
        if not hasattr(self, "ddf_ws"):
            self.ddf_ws = self.torch.empty((mb.mole_dedup_forward_workspace(w.T, w.V, w.N, w.L) // 4,),
                                           dtype=self.torch.int32, device="cuda")
        mb.mole_dedup_forward(self.tabs, w.V * w.N * w.d, self.ids[i % N_ID_BATCHES], self.h, None, 0.0, self.W_r,
                              self.shared, None, self.out, w.T * w.d, self.uniq, self.inv, self.n_uniq, self.err,
                              w.L, w.T, w.V, w.d, w.N, self.code, self.ddf_ws, stream=stream)

    def make_plans(self, stream):
        """One plan per id batch, computed outside any timed region (a real model computes the plan
        once per batch and reuses it for every MoLE layer)."""
        torch = self.torch
        self.plans = [torch.empty_like(self.plan) for _ in range(N_ID_BATCHES)]
        for b in range(N_ID_BATCHES):
            self.mb.mole_dedup_ids(self.ids[b], self.w.T, self.w.V, self.uniq, self.inv, self.n_uniq, self.err,
                                   self.plans[b], stream=stream)
        stream.synchronize()

    def forward_planned(self, i, stream, runs=False):
        w, mb = self.w, self.mb
        mb.mole_lookup_forward_layers(
            self.tabs, w.V * w.N * w.d, self.ids[i % N_ID_BATCHES], None, self.h, self.W_r, self.shared, None,
            self.out, w.T * w.d, None, None, self.err, w.L, w.T, w.V, w.d, w.N, self.code,
            mb.MOLE_FLAG_DEDUP | (mb.MOLE_FLAG_RUNS if runs else 0), self.plans[i % N_ID_BATCHES], stream=stream)

    def forward_one_layer(self, i, l, stream):
        """The single-layer entry point on layer l (what a real decoder calls, once per layer)."""
        w, mb = self.w, self.mb
        mb.mole_lookup_forward(self.tabs[l], self.ids[i % N_ID_BATCHES], None, self.h[l], self.W_r[l],
                               self.shared[l], None, self.out[l], None, None, self.err, w.T, w.V, w.d, w.N,
                               self.code, 0, None, stream=stream)

    def quantize(self, bits, block, scale_bytes):
        """NF-quantise every layer's table on the device (mole_quantize_lut)."""
        torch, mb, w = self.torch, self.mb, self.w
        cb = mb.mole_nf_codes_bytes(w.V, w.N, w.d, bits)
        sb = mb.mole_nf_scales_bytes(w.V, w.N, w.d, block, scale_bytes)
        self.nf = dict(bits=bits, block=block, scale_bytes=scale_bytes,
                       codes=torch.empty((w.L, cb), dtype=torch.uint8, device="cuda"),
                       scales=torch.empty((w.L, sb), dtype=torch.uint8, device="cuda"))
        for l in range(w.L):
            mb.mole_quantize_lut(self.tabs[l], self.nf["codes"][l], self.nf["scales"][l], w.V, w.N, w.d, bits,
                                 block, scale_bytes)
        torch.cuda.synchronize()

    def forward_nf(self, i, stream):
        w, mb, q = self.w, self.mb, self.nf
        mb.mole_lookup_forward_nf(q["codes"], q["codes"].shape[1], q["scales"], q["scales"].shape[1] // q["scale_bytes"],
                                  self.ids[i % N_ID_BATCHES], None, self.h, self.W_r, self.shared, None, self.out,
                                  w.T * w.d, None, None, self.err, w.L, w.T, w.V, w.d, w.N, q["bits"], q["block"],
                                  q["scale_bytes"], 0, None, stream=stream)

    def forward_with_residual(self, i, stream):
        """The layer as the inference listing has it, unfused: normed state in, residual added."""
        w, mb = self.w, self.mb
        mb.mole_lookup_forward_layers(
            self.tabs, w.V * w.N * w.d, self.ids[i % N_ID_BATCHES], None, self.h, self.W_r, self.shared, self.x,
            self.out, w.T * w.d, None, None, self.err, w.L, w.T, w.V, w.d, w.N, self.code, 0, None, stream=stream)

    def forward_fused_norm(self, i, stream):
        """mole_layer_forward: post-attention state in; norm and residual inside the kernel."""
        w, mb = self.w, self.mb
        mb.mole_layer_forward(
            self.tabs, w.V * w.N * w.d, self.ids[i % N_ID_BATCHES], None, self.x, self.ln_w, 1e-5, self.W_r,
            self.shared, self.out, w.T * w.d, None, None, self.err, w.L, w.T, w.V, w.d, w.N, self.code, 0, None,
            stream=stream)

    def make_norm_inputs(self):
        torch, w = self.torch, self.w
        g = torch.Generator(device="cuda")
        g.manual_seed(2000 + w.seed)
        self.x = (torch.randn((w.L, w.T, w.d), generator=g, device="cuda") * 2.0).to(self.h.dtype)
        self.ln_w = (torch.rand((w.L, w.d), generator=g, device="cuda") + 0.5).to(self.h.dtype)
        torch.cuda.synchronize()

    def distinct(self):
        import numpy as np
        return float(np.mean([len(np.unique(b)) for b in self.ids_host]))


def release_pinned(torch):
    """Hand cached pinned host blocks back (torch rounds a pinned request up to a power of two and keeps
    it; the box allows about 64 GiB of pinned memory in all)."""
    import gc
    gc.collect()
    if hasattr(torch._C, "_host_emptyCache"):
        torch._C._host_emptyCache()


def time_steps(torch, stream, step, steps, warmup):
    """`warmup` untimed, then exactly `steps` timed calls of step(i), all enqueued on `stream` and
    bracketed by two HIP events recorded on that stream, with a device synchronisation on both
    sides.  Returns milliseconds per step."""
    with torch.cuda.stream(stream):
        for i in range(warmup):
            step(i)
        stream.synchronize()
        torch.cuda.synchronize()
        ev0 = torch.cuda.Event(enable_timing=True)
        ev1 = torch.cuda.Event(enable_timing=True)
        ev0.record(stream)
        for i in range(steps):
            step(warmup + i)
        ev1.record(stream)
        stream.synchronize()
        torch.cuda.synchronize()
    return ev0.elapsed_time(ev1) / steps


def launch_spread(torch, stream, step, n=200):
    """Launch-to-launch time of n further calls of step(i), each bracketed by its own HIP events on
    `stream`: median, 10th and 90th percentile in microseconds (outside the timed region)."""
    with torch.cuda.stream(stream):
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        stream.synchronize()
        evs[0].record(stream)
        for i in range(n):
            step(i)
            evs[i + 1].record(stream)
        stream.synchronize()
    us = sorted(evs[i].elapsed_time(evs[i + 1]) * 1e3 for i in range(n))
    pick = lambda q: us[min(n - 1, int(q * n))]
    return {"median": pick(0.5), "p10": pick(0.1), "p90": pick(0.9), "n": n}


def rates(w, acc, ms, distinct=None):
    """tokens/s and GB/s for a forward over all layers of workload w taking `ms`."""
    alg = acc.forward_bytes_per_token(w.d, w.N, w.elem_bytes) * w.T * w.L
    # the algorithmic rate counts every token's own rows, so with repeated ids it can exceed what HBM delivers:
    # it is a rate, never a fraction of the peak; the fraction is taken on the bytes that have to move
    out = {"ms": round(ms, 5), "layer_tokens_per_s": w.T * w.L / (ms * 1e-3), "tokens_per_s": w.T / (ms * 1e-3),
           "algorithmic_GBps": alg / (ms * 1e-3) / 1e9}
    if distinct is not None:
        moved = w.L * acc.forward_bytes_moved(w.T, int(round(distinct)), w.d, w.N, w.elem_bytes)
        out["distinct_ids"] = distinct
        out["moved_bytes"] = moved
        out["moved_GBps"] = moved / (ms * 1e-3) / 1e9
        out["moved_frac_of_hbm_peak"] = out["moved_GBps"] / HBM_PEAK_GBS
    return out


KERNEL_SOURCES = ("lookup_forward.hip", "fwd_tile.hip", "tile_router.h", "fwd_common.h", "mole_internal.h")


def kernel_source_hash():
    """Hash of the forward kernels' sources (comments and blank lines left out, so that only a change of code
    counts): a counter summary under profiles/ records the hash it was taken on, so a summary of an older
    kernel is recognised as such."""
    import hashlib
    import re
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2503_15798_amd", "csrc", name), "r") as f:
            text = f.read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        lines = [re.sub(r"//.*$", "", ln).rstrip() for ln in text.splitlines()]
        h.update("\n".join(ln for ln in lines if ln.strip()).encode())
    return h.hexdigest()[:16]


def read_traffic(kernel_tag):
    """(HBM bytes per launch, provenance) of the forward kernel from the committed rocprofv3 counter
    summary (profiles/<tag>_hbm_traffic.txt: key=value lines); (None, None) if there is none.  Counters
    cannot be read inside this run; `current` says whether the summary was taken on today's kernel sources."""
    path = os.path.join(ROOT, "profiles", f"{kernel_tag}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None, None
    kv = {}
    for line in open(path):
        line = line.split("#")[0].strip()
        if "=" in line:
            k, v = line.split("=", 1)
            kv[k.strip()] = v.strip()
    try:
        traffic = float(kv["hbm_bytes_per_launch"])
    except (KeyError, ValueError):
        return None, None
    sha = kv.get("kernel_source_sha")
    return traffic, {"file": os.path.relpath(path, ROOT), "kernel_source_sha": sha,
                     "current": sha == kernel_source_hash(),
                     "counters": "FETCH_SIZE x 2.0 + WRITE_SIZE (L2 misses and write-backs: Infinity Cache hits included)"}


def cpu_baseline(L, torch, wl, steps=21):
    """The fp64 oracle on the host cores, same workload: all layers x all tokens of id batch 0.
    Only the looked-up rows are brought to the host (plain indexing; the copy is not timed)."""
    import numpy as np
    import oracle
    w = L.w
    ids = L.ids_host[0]
    uniq, inv = np.unique(ids, return_inverse=True)
    rows_t = torch.from_numpy(uniq.astype(np.int64)).cuda()

    def host(t):
        if t.dtype == torch.bfloat16:
            return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return t.cpu().numpy()
    per_layer = [(host(L.tabs[l][rows_t]), host(L.h[l]), host(L.W_r[l]), host(L.shared[l])) for l in range(w.L)]
    inv32 = inv.astype(np.int32)
    oracle.lib()
    times = []
    for _ in range(steps):
        t0 = time.perf_counter()
        for tab, h, wr, sh in per_layer:
            oracle.lookup_forward(tab, inv32, h, wr, sh)
        times.append(time.perf_counter() - t0)
    sec = statistics.median(times)
    return {"value": w.T * w.L / sec, "unit": "layer-tokens/s", "cores": oracle.threads(), "kind": "oracle",
            "seconds_per_step": sec,
            "sample": f"the whole step ({w.L} layers x {w.T} tokens, id batch 0), median of {steps} runs; "
                      "rows gathered to the host beforehand, untimed"}, per_layer, inv32


def check_against_oracle(L, torch, wl, per_layer, inv32, stream):
    """One GPU step on id batch 0 compared with the oracle on a few layers (guards the numbers)."""
    import numpy as np
    import oracle
    w = L.w
    L.forward(0, stream)
    torch.cuda.synchronize()
    for l in sorted({0, w.L // 2, w.L - 1}):
        tab, h, wr, sh = per_layer[l]
        ref, _, _, _ = oracle.lookup_forward(tab, inv32, h, wr, sh)
        got = L.out[l]
        got = wl.storage_to_f64(got.contiguous().view(torch.int16).cpu().numpy().view(np.uint16), wl.BF16) \
            if got.dtype == torch.bfloat16 else got.cpu().numpy().astype(np.float64)
        if not np.all(np.abs(got - ref) <= 1e-3 + 2e-2 * np.abs(ref)):
            raise RuntimeError(f"GPU output of layer {l} disagrees with the oracle")


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build measures ONE GPU (the MoLE lookup path of one device); --gpus {args.gpus} "
              "is not supported (token-parallel sharding with a replicated table would need no "
              "communication: every GPU would run this same path on its share of the tokens)", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2503_15798_amd import accounting as acc
    from paper_2503_15798_amd import binding as mb
    from paper_2503_15798_amd import workloads as wl
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    mb.lib()     # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)
    stream = torch.cuda.Stream()
    if args.only_build:
        print(json.dumps({"build_lut_410m_layer": build_bench(torch, mb, wl, acc, stream)}))
        return
    w = wl.CONFIGS[args.workload]

    # ------------------------------------------------------------------ headline workload
    L = Layers(w, torch, mb, wl)
    if args.only_nf:
        print(json.dumps({f"{w.name}_{tag}": nf_entry(L, acc, torch, stream, args.steps, args.warmup, bits, block, sb)
                          for tag, bits, block, sb in (("nf4", 4, 1024, 4), ("nf3", 3, 128, 2))}))
        return

    if args.plan:
        L.make_plans(stream)

    def step(i):
        if args.dedup_forward:
            L.dedup_forward(i, stream)
        elif args.plan:
            L.forward_planned(i, stream, runs=args.runs)
        else:
            L.forward(i, stream)
    ms_step = time_steps(torch, stream, step, args.steps, args.warmup)
    # the step is exactly one launch of the forward kernel, so the launch-to-launch average over the
    # timed region is that kernel's duration (an upper bound: it includes the gap between launches)
    ms_kernel = ms_step
    if int(L.err.item()) != 0:
        raise RuntimeError("error flag set by the forward kernel")
    distinct = L.distinct()
    table_bytes = int(L.tabs.numel() * L.tabs.element_size())
    head = rates(w, acc, ms_step, distinct)
    alg_bytes = acc.forward_bytes_per_token(w.d, w.N, w.elem_bytes) * w.T * w.L
    achieved = alg_bytes / (ms_kernel * 1e-3) / 1e9
    # the kernel the launcher picks for this call (--runs passes MOLE_FLAG_RUNS: the run kernel for N <= 32; N = 32
    # with at least two rounds of eight tokens per CU: the tile kernel)
    if args.dedup_forward:
        # two launches (dedup beside the router, then the gather): the step time stands for both
        if not (w.N == 32 and w.L == 1 and 4096 < w.T <= 16384):
            raise SystemExit("--dedup-forward: only workloads the fused launches serve (N = 32, one layer, 4096 < T <= 16384)")
        kernel = "fwd_bf16_gather_kernel"
    elif args.plan and args.runs and w.N <= 32:
        kernel = "fwd_bf16_run_kernel"
    elif w.N == 32 and ((w.T + 7) // 8) * w.L >= 2 * torch.cuda.get_device_properties(0).multi_processor_count:
        kernel = "fwd_bf16_tile_kernel"
    else:
        kernel = "fwd_bf16_stream_kernel"
    kernel_tag = f"{kernel[:-7]}_{w.name}" + ("_plan" if args.plan and not args.dedup_forward else "")
    traffic, traffic_src = read_traffic(kernel_tag)
    moved_bytes = w.L * acc.forward_bytes_moved(w.T, int(round(distinct)), w.d, w.N, w.elem_bytes)
    roofline = {"bound": "hbm", "kernel": kernel, "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                "traffic_frac": None if traffic is None else traffic / (ms_kernel * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "traffic_source": traffic_src,
                "algorithmic_bytes_per_launch": alg_bytes, "moved_bytes_per_launch": moved_bytes,
                "moved_frac": moved_bytes / (ms_kernel * 1e-3) / 1e9 / HBM_PEAK_GBS, "kernel_ms": ms_kernel}

    if achieved > HBM_PEAK_GBS:
        # Zipf ids on a large batch: most of the algorithmic bytes are repeats that L2 / Infinity Cache serve
        roofline["frac_note"] = ("algorithmic bytes count every token's own rows; above 1 it is no fraction of what "
                                 "HBM delivers: see traffic_frac (counters) and moved_frac (distinct rows once)")
    roofline["launch_us"] = launch_spread(torch, stream, step)

    cpu = None
    if not args.no_cpu:
        cpu, per_layer, inv32 = cpu_baseline(L, torch, wl)
        check_against_oracle(L, torch, wl, per_layer, inv32, stream)
        del per_layer

    other = {}
    if not args.no_extras:
        other = extras(args, torch, mb, wl, acc, stream, L)
        roofline["also"] = also_list(other)
    if args.calibrate_copy:
        a = torch.empty((1 << 30,), dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()

    line = {
        "metric": ("MoLE layer tokens/s (410M-shape decode step: 24 MoLE layers x 256 tokens, N=16, d=1024)"
                   if w.name == "decode410m" else
                   f"MoLE layer tokens/s ({w.name}: {w.L} MoLE layers x {w.T} tokens, N={w.N}, d={w.d})"),
        "value": head["layer_tokens_per_s"], "unit": "layer-tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "layers": w.L, "tokens_per_step": w.T, "V": w.V, "d": w.d, "N": w.N,
                   "ids": ("zipf(1.1)" if w.ids == "zipf" else w.ids) + ", 16 rotating batches", "mean_distinct_ids": distinct,
                   "table_bytes": table_bytes,
                   "step": "router + softmax + gather + gate-weighted sum + shared add, all layers, one launch"
                           + (", tokens visited by the plan of mole_dedup_ids (computed beforehand)"
                              if args.plan and not args.dedup_forward else "")
                           + (", preceded in the same call by the dedup (mole_dedup_forward: two launches)"
                              if args.dedup_forward else ""),
                   "decode_tokens_per_s": head["tokens_per_s"],
                   "algorithmic_GBps": head["algorithmic_GBps"], "moved_GBps": head["moved_GBps"]},
        "roofline": roofline,
        "cpu_baseline": cpu,
        # one number per secondary entry (ms); the small shapes' dedup-kernel times only with --full
        "other_ms": {k: round(v["ms"] if isinstance(v, dict) else v, 4) for k, v in other.items()
                     if (not isinstance(v, dict) or "ms" in v)
                     and not (k.endswith("_dedup_kernel_ms") and not k.startswith(("decode410m_dedup", "prefill410m")))},
    }
    if args.full:
        line["other"] = other
    print(json.dumps(line))


def also_list(o):
    """The other configurations against their rooflines, in the shape of `roofline` (short: the driver keeps
    this part of the line).  HBM entries are taken on the bytes that have to move (each distinct id's rows
    once + activations); with uniform ids and no plan nearly every token has its own rows and the
    algorithmic bytes are what the counters read."""
    out = []

    def hbm(name, what, key="moved_GBps"):
        e = o.get(name)
        if isinstance(e, dict) and key in e:
            out.append({"workload": name, "what": what, "bound": "hbm", "achieved": round(e[key], 1),
                        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(e[key] / HBM_PEAK_GBS, 4),
                        "us": round(e["ms"] * 1e3, 2), "bytes": key.split("_")[0]})
    hbm("prefill410m_uniform", "N=32, 16384 tokens, uniform ids (no-reuse control), no plan", "algorithmic_GBps")
    hbm("prefill410m_uniform_forward_with_plan", "the same with the plan of mole_dedup_ids")
    hbm("prefill410m_uniform_dedup_plus_forward", "the same, dedup inside the timed step (mole_dedup_forward)")
    hbm("prefill410m", "N=32, 16384 tokens, Zipf ids, no plan")
    hbm("prefill410m_forward_with_plan", "the same with the plan")
    hbm("prefill410m_dedup_plus_forward", "the same, dedup inside the timed step (mole_dedup_forward)")
    hbm("decode410m_forward_with_plan", "headline step with the plan")
    hbm("decode410m_dedup_plus_forward", "headline step, dedup inside the timed step")
    hbm("decode160m", "12 layers x 64 tokens, d=768 (latency regime)")
    hbm("decode410m_t32", "24 layers x 32 tokens (latency regime)")
    hbm("decode410m_t1", "24 layers x 1 token (latency regime)")
    hbm("decode1b_4e", "16 layers x 256 tokens, d=2048, N=4")
    for tag in ("nf4", "nf3"):
        e = o.get(f"decode410m_{tag}")
        if isinstance(e, dict):
            out.append({"workload": f"decode410m_{tag}", "what": "dequantising forward, on its own (smaller) byte count",
                        "bound": "hbm", "achieved": round(e["algorithmic_GBps"], 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": round(e["algorithmic_GBps"] / HBM_PEAK_GBS, 4), "us": round(e["ms"] * 1e3, 2),
                        "bytes": "algorithmic"})
    e = o.get("offload410m")
    if isinstance(e, dict) and "fetch_GBps" in e:
        out.append({"workload": "offload410m", "what": "fetch of the distinct rows of 24 layers from pinned host memory",
                    "bound": "host link", "achieved": round(e["fetch_GBps"], 2), "peak": HOST_LINK_GBS, "unit": "GB/s",
                    "frac": round(e["fetch_GBps"] / HOST_LINK_GBS, 4), "us": round(e["fetch_only_ms"] * 1e3, 1),
                    "step_us": round(e["ms"] * 1e3, 1)})
    e = o.get("build_lut_410m_layer")
    if isinstance(e, dict) and "algorithmic_TFLOPs" in e:
        out.append({"workload": "build_lut_410m_layer", "what": "mole_build_lut, one 410M layer (16 experts, V=50304)",
                    "bound": "mfma", "achieved": round(e["algorithmic_TFLOPs"], 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(e["algorithmic_TFLOPs"] / MFMA_BF16_PEAK_TFLOPS, 4),
                    "us": round(e["ms"] * 1e3, 1)})
    return out


def extras(args, torch, mb, wl, acc, stream, L):
    """The other workloads and variants.  Each entry: ms, tokens/s, GB/s."""
    import numpy as np
    out = {}
    # warm-up covers every id batch once, so that no batch's rows are touched for the first time in a timed step
    steps, warm = max(20, args.steps // 4), max(N_ID_BATCHES, args.warmup // 2)
    w = L.w

    def both(LL):
        return lambda i: LL.dedup_forward(i, stream)

    def two_calls(LL):
        def f(i):
            LL.dedup(i, stream)
            LL.forward(i, stream, dedup=True)
        return f

    def plain(LL):
        return lambda i: LL.forward(i, stream)

    def planned(LL):
        LL.make_plans(stream)
        return lambda i: LL.forward_planned(i, stream)

    def per_layer(LL):
        def f(i):
            for l in range(LL.w.L):
                LL.forward_one_layer(i, l, stream)
        return f

    def graph_of_layers(LL):
        """The per-layer launches of one step captured in a HIP graph (id batch 0), replayed per step."""
        g = torch.cuda.CUDAGraph()
        f = per_layer(LL)
        with torch.cuda.stream(stream):
            f(0)
            stream.synchronize()
            with torch.cuda.graph(g, stream=stream):
                f(0)
        return lambda i: g.replay()

    # headline shape: dedup + id-ordered forward, and the dedup kernel alone
    ms = time_steps(torch, stream, both(L), steps, warm)
    out["decode410m_dedup_plus_forward"] = rates(w, acc, ms, L.distinct())
    ms = time_steps(torch, stream, lambda i: L.dedup(i, stream), steps, warm)
    out["decode410m_dedup_kernel_ms"] = ms
    ms = time_steps(torch, stream, planned(L), steps, warm)
    out["decode410m_forward_with_plan"] = rates(w, acc, ms, L.distinct())
    # the same step as 24 launches of the single-layer entry point, eagerly and from a HIP graph
    ms = time_steps(torch, stream, per_layer(L), steps, warm)
    out["decode410m_per_layer_launches"] = rates(w, acc, ms, L.distinct())
    try:
        ms = time_steps(torch, stream, graph_of_layers(L), steps, warm)
        out["decode410m_per_layer_launches_hip_graph"] = rates(w, acc, ms, L.distinct())
    except Exception as e:
        out["decode410m_per_layer_launches_hip_graph"] = {"skipped": repr(e)}

    # ---- the whole listing step from the post-attention state: unfused (normed state + residual, 4 activation
    # streams) against mole_layer_forward (norm and residual inside: 3 streams)
    out.update(norm_entries(L, acc, torch, stream, steps, warm, "decode410m"))

    # ---- NF4 / NF3 tables (Sec. 5.5 of the paper): quantised on the device, dequantised inside the forward
    for tag, bits, block, sbytes in (("nf4", 4, 1024, 4), ("nf3", 3, 128, 2)):
        out[f"decode410m_{tag}"] = nf_entry(L, acc, torch, stream, steps, warm, bits, block, sbytes)

    # ---- storage tier: a few layers of the same tables in an id-major LUT file ----
    try:
        out["storage410m"] = storage_bench(torch, mb, wl, stream, L, steps, warm)
    except Exception as e:
        traceback.print_exc(file=sys.stderr)
        out["storage410m"] = {"skipped": repr(e)}
    release_pinned(torch)

    # ---- offloaded mode on the same tables: all LUTs in pinned host memory, T = 32 ----
    try:
        out.update(offload_bench(torch, mb, wl, acc, stream, L, steps, warm))
    except Exception as e:   # host memory may not allow 40 GB of pinned pages
        traceback.print_exc(file=sys.stderr)
        out["offload410m"] = {"skipped": repr(e)}
    release_pinned(torch)

    # ---- the same with NF4 / NF3 tables: codes and scales of all layers in pinned host memory ----
    for tag, bits, block, sbytes in (("nf4", 4, 1024, 4), ("nf3", 3, 128, 2)):
        try:
            out[f"offload410m_{tag}"] = offload_nf_bench(torch, mb, wl, stream, L, steps, warm, bits, block, sbytes)
        except Exception as e:
            traceback.print_exc(file=sys.stderr)
            out[f"offload410m_{tag}"] = {"skipped": repr(e)}
        release_pinned(torch)

    # smaller decode batches on the same tables (latency-bound: microseconds are the result)
    for T in (32, 1):
        ww = wl.scaled(w, T=T, name=f"decode410m_t{T}")
        LL = Layers.__new__(Layers)
        LL.__dict__.update(L.__dict__)
        LL.w = ww
        LL.h, LL.shared, LL.out = L.h[:, :T].contiguous(), L.shared[:, :T].contiguous(), L.out[:, :T].contiguous()
        LL.ids_host = np.stack([wl.token_ids(ww, b) for b in range(N_ID_BATCHES)])
        LL.ids = torch.from_numpy(LL.ids_host).cuda()
        ms = time_steps(torch, stream, plain(LL), steps, warm)
        out[ww.name] = rates(ww, acc, ms, LL.distinct())
        ms = time_steps(torch, stream, per_layer(LL), steps, warm)
        out[ww.name + "_per_layer_launches"] = rates(ww, acc, ms, LL.distinct())
        try:
            ms = time_steps(torch, stream, graph_of_layers(LL), steps, warm)
            out[ww.name + "_per_layer_launches_hip_graph"] = rates(ww, acc, ms, LL.distinct())
        except Exception as e:
            out[ww.name + "_per_layer_launches_hip_graph"] = {"skipped": repr(e)}
    del L.tabs
    torch.cuda.empty_cache()

    for name in ("prefill410m", "prefill410m_uniform", "decode160m", "decode1b_4e", "decode410m_n2", "decode410m_n4",
                 "decode410m_n8"):
        ww = wl.CONFIGS[name]
        LL = Layers(ww, torch, mb, wl)
        ms = time_steps(torch, stream, plain(LL), steps, warm)
        out[name] = rates(ww, acc, ms, LL.distinct())
        ms = time_steps(torch, stream, both(LL), steps, warm)
        out[name + "_dedup_plus_forward"] = rates(ww, acc, ms, LL.distinct())
        if name.startswith("prefill"):      # mole_dedup_ids, then the planned forward, as two calls
            ms = time_steps(torch, stream, two_calls(LL), steps, warm)
            out[name + "_dedup_then_forward_two_calls"] = rates(ww, acc, ms, LL.distinct())
        ms = time_steps(torch, stream, lambda i: LL.dedup(i, stream), steps, warm)
        out[name + "_dedup_kernel_ms"] = ms
        ms = time_steps(torch, stream, planned(LL), steps, warm)
        out[name + "_forward_with_plan"] = rates(ww, acc, ms, LL.distinct())
        if name.startswith("prefill"):      # MOLE_FLAG_RUNS: equal ids summed together on the matrix pipe
            ms = time_steps(torch, stream, lambda i: LL.forward_planned(i, stream, runs=True), steps, warm)
            out[name + "_forward_with_plan_runs"] = rates(ww, acc, ms, LL.distinct())
        if name == "prefill410m_uniform":
            out[name + "_nf4"] = nf_entry(LL, acc, torch, stream, steps, warm, 4, 1024, 4)
            out.update(norm_entries(LL, acc, torch, stream, steps, warm, name))
            out.update(shared_ffn_entries(LL, acc, torch, mb, stream, steps, warm, name))
        del LL
        torch.cuda.empty_cache()

    out["build_lut_410m_layer"] = build_bench(torch, mb, wl, acc, stream, with_cpu=not args.no_cpu)
    return out


def shared_ffn_entries(LL, acc, torch, mb, stream, steps, warm, name):
    """One layer with its shared expert (D_s = 4 d): mole_shared_ffn_forward (gather and combine in the second
    product's epilogue) against the same layer with the shared expert computed by torch's own bf16 GEMMs
    (linear, GELU, linear -> shared_out in HBM) followed by mole_lookup_forward.  Layer 0 of the workload."""
    import torch.nn.functional as F
    w = LL.w
    D_s = 4 * w.d
    g = torch.Generator(device="cuda")
    g.manual_seed(3000 + w.seed)
    W1 = (torch.randn((D_s, w.d), generator=g, device="cuda") * 0.02).to(torch.bfloat16)
    W2 = (torch.randn((w.d, D_s), generator=g, device="cuda") * 0.02).to(torch.bfloat16)
    b1 = (torch.randn((D_s,), generator=g, device="cuda") * 0.1).to(torch.bfloat16)
    b2 = (torch.randn((w.d,), generator=g, device="cuda") * 0.1).to(torch.bfloat16)
    res = torch.randn((w.T, w.d), generator=g, device="cuda").to(torch.bfloat16)
    ws = torch.empty((mb.mole_shared_ffn_workspace(w.T, w.d, D_s, w.N),), dtype=torch.uint8, device="cuda")
    tab, h, W_r, out = LL.tabs[0], LL.h[0], LL.W_r[0], LL.out[0]

    def fused(i):
        mb.mole_shared_ffn_forward(tab, LL.ids[i % N_ID_BATCHES], None, h, W_r, W1, b1, W2, b2, res, out, None, LL.err,
                                   w.T, w.V, w.d, D_s, w.N, LL.code, mb.MOLE_GELU_ERF, ws, stream=stream)

    def torch_ffn(i):
        return F.linear(F.gelu(F.linear(h, W1, b1)), W2, b2)

    def unfused(i):
        sh = torch_ffn(i)
        mb.mole_lookup_forward(tab, LL.ids[i % N_ID_BATCHES], None, h, W_r, sh, res, out, None, None, LL.err, w.T, w.V,
                               w.d, w.N, LL.code, 0, None, stream=stream)

    def lookup_only(i):
        mb.mole_lookup_forward(tab, LL.ids[i % N_ID_BATCHES], None, h, W_r, LL.shared[0], res, out, None, None, LL.err,
                               w.T, w.V, w.d, w.N, LL.code, 0, None, stream=stream)
    flops = 4.0 * w.T * w.d * D_s
    out_d = {}
    for tag, fn in (("fused", fused), ("torch_gemms_then_lookup", unfused), ("torch_gemms_alone", torch_ffn),
                    ("lookup_alone", lookup_only)):
        ms = time_steps(torch, stream, fn, max(5, steps // 4), 3)
        out_d[f"{name}_shared_ffn_{tag}"] = {"ms": ms, "tokens_per_s": w.T / (ms * 1e-3), "D_s": D_s,
                                             "ffn_TFLOPs": None if tag == "lookup_alone" else flops / (ms * 1e-3) / 1e12}
    return out_d


def norm_entries(LL, acc, torch, stream, steps, warm, name):
    w = LL.w
    LL.make_norm_inputs()
    res = {}
    for tag, fn, streams in (("with_residual", LL.forward_with_residual, 4), ("fused_norm", LL.forward_fused_norm, 3)):
        ms = time_steps(torch, stream, lambda i: fn(i, stream), steps, warm)
        alg = (w.N * w.d * w.elem_bytes + streams * w.d * w.elem_bytes + 4) * w.T * w.L
        res[f"{name}_{tag}"] = {"ms": round(ms, 5), "layer_tokens_per_s": w.T * w.L / (ms * 1e-3),
                                "activation_streams": streams, "algorithmic_bytes_per_launch": alg,
                                "algorithmic_GBps": alg / (ms * 1e-3) / 1e9}
    del LL.x, LL.ln_w
    return res


def nf_entry(LL, acc, torch, stream, steps, warm, bits, block, sbytes):
    """Quantise LL's tables and time the dequantising forward; rates against its own (smaller) byte count."""
    w = LL.w
    t0 = time.perf_counter()
    LL.quantize(bits, block, sbytes)
    t_quant = time.perf_counter() - t0
    ms = time_steps(torch, stream, lambda i: LL.forward_nf(i, stream), steps, warm)
    alg = acc.nf_forward_bytes_per_token(w.d, w.N, bits, block, sbytes) * w.T * w.L
    res = {"bits": bits, "block": block, "scale_bytes": sbytes, "ms": ms,
           "layer_tokens_per_s": w.T * w.L / (ms * 1e-3), "algorithmic_bytes_per_launch": alg,
           "algorithmic_GBps": alg / (ms * 1e-3) / 1e9,
           "table_bytes": acc.nf_table_bytes(w.V, w.N, w.d, bits, block, sbytes) * w.L,
           "table_ratio_to_bf16": acc.nf_table_bytes(w.V, w.N, w.d, bits, block, sbytes) / (w.V * w.N * w.d * 2),
           "quantise_all_layers_s": t_quant}
    del LL.nf
    torch.cuda.empty_cache()
    return res


def offload_bench(torch, mb, wl, acc, stream, L, steps, warm):
    import numpy as np
    w = wl.CONFIGS["offload410m"]
    res = {}
    host = torch.empty(L.tabs.shape, dtype=L.tabs.dtype, pin_memory=True)
    host.copy_(L.tabs)
    torch.cuda.synchronize()
    T, U_cap = w.T, w.T
    ids_host = np.stack([wl.token_ids(w, b) for b in range(N_ID_BATCHES)])
    ids = torch.from_numpy(ids_host).cuda()
    uniq = torch.empty((T,), dtype=torch.int32, device="cuda")
    inv = torch.empty((T,), dtype=torch.int32, device="cuda")
    nu = torch.zeros((1,), dtype=torch.int32, device="cuda")
    err = torch.zeros((1,), dtype=torch.int32, device="cuda")
    plan = torch.empty((mb.mole_dedup_workspace(T, w.V) // 4,), dtype=torch.int32, device="cuda")
    staging = torch.empty((w.L, U_cap, w.N, w.d), dtype=L.tabs.dtype, device="cuda")
    h, sh, o = L.h[:, :T].contiguous(), L.shared[:, :T].contiguous(), L.out[:, :T].contiguous()
    row_elems, code = w.N * w.d, mb.MOLE_BF16

    def dedup(i):
        mb.mole_dedup_ids(ids[i % N_ID_BATCHES], T, w.V, uniq, inv, nu, err, plan, stream=stream)

    def fetch(i):
        mb.mole_offload_fetch(host, w.V * row_elems, uniq, nu, staging, U_cap * row_elems, err, w.L, U_cap, w.V,
                              w.d, w.N, code, stream=stream)

    def fwd_staged(i):
        mb.mole_lookup_forward_layers(staging, U_cap * row_elems, ids[i % N_ID_BATCHES], inv, h, L.W_r, sh, None, o,
                                      T * w.d, None, None, err, w.L, T, U_cap, w.d, w.N, code, 0, None, stream=stream)

    def fwd_direct(i):
        mb.mole_lookup_forward_layers(host, w.V * row_elems, ids[i % N_ID_BATCHES], None, h, L.W_r, sh, None, o,
                                      T * w.d, None, None, err, w.L, T, w.V, w.d, w.N, code, 0, None, stream=stream)

    def full(i):
        dedup(i)
        fetch(i)
        fwd_staged(i)
    U = float(np.mean([len(np.unique(b)) for b in ids_host]))
    fetched = U * w.L * row_elems * 2
    ms_full = time_steps(torch, stream, full, steps, warm)

    def only_fetch(i):
        fetch(i)
    dedup(0)
    ms_fetch = time_steps(torch, stream, only_fetch, steps, warm)
    u0 = len(np.unique(ids_host[0]))
    ms_direct = time_steps(torch, stream, lambda i: fwd_direct(i), steps, warm)
    # the practical ceiling of the link: one plain pinned-to-device copy of a layer's table (1.65 GB)
    dst = torch.empty_like(L.tabs[0])
    ms_copy = time_steps(torch, stream, lambda i: dst.copy_(host[0], non_blocking=True), 3, 1)
    copy_GBps = host[0].numel() * 2 / (ms_copy * 1e-3) / 1e9
    del dst
    res["offload410m"] = {
        "step": "dedup + fetch of the distinct rows of all 24 layers from pinned host memory + staged forward",
        "tokens": T, "mean_distinct_ids": U, "ms": ms_full, "tokens_per_s": T / (ms_full * 1e-3),
        "fetch_only_ms": ms_fetch, "fetch_GBps": u0 * w.L * row_elems * 2 / (ms_fetch * 1e-3) / 1e9,
        "fetch_frac_of_host_link_peak": u0 * w.L * row_elems * 2 / (ms_fetch * 1e-3) / 1e9 / HOST_LINK_GBS,
        "fetched_bytes_per_step": fetched, "host_table_bytes": int(host.numel() * 2),
        "forward_reading_host_table_directly_ms": ms_direct,
        "pinned_memcpy_GBps": copy_GBps,
    }
    del host
    release_pinned(torch)

    # ---- the same tables id-major on the host ([V, L, N, d]: one contiguous 768 KiB block per id) ----
    host_id = torch.empty((w.V, w.L, w.N, w.d), dtype=L.tabs.dtype, pin_memory=True)
    for l in range(w.L):
        host_id[:, l].copy_(L.tabs[l])
    torch.cuda.synchronize()

    def fetch_id(i, s=stream, bufs=None):
        u, n, st = bufs or (uniq, nu, staging)
        mb.mole_offload_fetch_idmajor(host_id, u, n, st, U_cap * row_elems, err, w.L, U_cap, w.V, w.d, w.N, code,
                                      stream=s)

    def full_id(i):
        dedup(i)
        fetch_id(i)
        fwd_staged(i)
    ms_full_id = time_steps(torch, stream, full_id, steps, warm)
    dedup(0)
    ms_fetch_id = time_steps(torch, stream, lambda i: fetch_id(i), steps, warm)

    # double-buffered: the rows of step i+1 are fetched on a second stream while step i's forward runs
    # (ids are known when a step starts; both streams at the default priority)
    s2 = torch.cuda.Stream()
    sets = []
    for _ in range(2):
        sets.append(dict(uniq=torch.empty_like(uniq), inv=torch.empty_like(inv), nu=torch.zeros_like(nu),
                         plan=torch.empty_like(plan), staging=torch.empty_like(staging),
                         fetched=torch.cuda.Event(), consumed=torch.cuda.Event()))

    def prefetch(i):
        b = sets[i % 2]
        s2.wait_event(b["consumed"])
        mb.mole_dedup_ids(ids[i % N_ID_BATCHES], T, w.V, b["uniq"], b["inv"], b["nu"], err, b["plan"], stream=s2)
        fetch_id(i, s2, (b["uniq"], b["nu"], b["staging"]))
        b["fetched"].record(s2)

    def consume(i):
        b = sets[i % 2]
        stream.wait_event(b["fetched"])
        mb.mole_lookup_forward_layers(b["staging"], U_cap * row_elems, ids[i % N_ID_BATCHES], b["inv"], h, L.W_r, sh,
                                      None, o, T * w.d, None, None, err, w.L, T, U_cap, w.d, w.N, code, 0, None,
                                      stream=stream)
        b["consumed"].record(stream)

    for b in sets:
        b["consumed"].record(stream)
    torch.cuda.synchronize()
    n_pipe = steps + warm
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    prefetch(0)
    for i in range(n_pipe):
        if i == warm:
            ev0.record(stream)
        if i + 1 < n_pipe:
            prefetch(i + 1)
        consume(i)
    ev1.record(stream)
    torch.cuda.synchronize()
    ms_pipe = ev0.elapsed_time(ev1) / steps
    res["offload410m_id_major"] = {
        "step": "as offload410m with the host table laid out [V, L, N, d]",
        "ms": ms_full_id, "tokens_per_s": T / (ms_full_id * 1e-3), "fetch_only_ms": ms_fetch_id,
        "fetch_GBps": u0 * w.L * row_elems * 2 / (ms_fetch_id * 1e-3) / 1e9,
        "fetch_frac_of_host_link_peak": u0 * w.L * row_elems * 2 / (ms_fetch_id * 1e-3) / 1e9 / HOST_LINK_GBS,
        "double_buffered_ms": ms_pipe, "double_buffered_tokens_per_s": T / (ms_pipe * 1e-3),
        "double_buffered_fetch_GBps": fetched / (ms_pipe * 1e-3) / 1e9,
    }
    del host_id, sets
    return res


def offload_nf_bench(torch, mb, wl, stream, L, steps, warm, bits, block, sbytes):
    """Offloaded mode with a quantised table (Sec. 5.5 / Table 8 of the paper: quantising the LUT cuts the
    bytes loaded per token): dedup + fetch of the distinct ids' code and scale rows of all layers from
    pinned host memory + dequantising forward on the staged rows."""
    import numpy as np
    w = wl.CONFIGS["offload410m"]
    T, U_cap = w.T, w.T
    L.quantize(bits, block, sbytes)
    code_row, scale_row = w.N * w.d * bits // 8, w.N * (w.d // block)
    host_codes = L.nf["codes"][:, :w.V * code_row].cpu().pin_memory()
    host_scales = L.nf["scales"][:, :w.V * scale_row * sbytes].cpu().pin_memory()
    del L.nf
    torch.cuda.empty_cache()
    ids_host = np.stack([wl.token_ids(w, b) for b in range(N_ID_BATCHES)])
    ids = torch.from_numpy(ids_host).cuda()
    uniq = torch.empty((T,), dtype=torch.int32, device="cuda")
    inv = torch.empty((T,), dtype=torch.int32, device="cuda")
    nu = torch.zeros((1,), dtype=torch.int32, device="cuda")
    err = torch.zeros((1,), dtype=torch.int32, device="cuda")
    plan = torch.empty((mb.mole_dedup_workspace(T, w.V) // 4,), dtype=torch.int32, device="cuda")
    st_codes = torch.empty((w.L, U_cap * code_row), dtype=torch.uint8, device="cuda")
    st_scales = torch.empty((w.L, U_cap * scale_row * sbytes), dtype=torch.uint8, device="cuda")
    h, sh, o = L.h[:, :T].contiguous(), L.shared[:, :T].contiguous(), L.out[:, :T].contiguous()

    def fetch(i):
        mb.mole_offload_fetch_nf(host_codes, w.V * code_row, host_scales, w.V * scale_row, uniq, nu, st_codes,
                                 U_cap * code_row, st_scales, U_cap * scale_row, err, w.L, U_cap, w.V, w.d, w.N, bits,
                                 block, sbytes, stream=stream)

    def full(i):
        mb.mole_dedup_ids(ids[i % N_ID_BATCHES], T, w.V, uniq, inv, nu, err, plan, stream=stream)
        fetch(i)
        mb.mole_lookup_forward_nf(st_codes, U_cap * code_row, st_scales, U_cap * scale_row, ids[i % N_ID_BATCHES], inv,
                                  h, L.W_r, sh, None, o, T * w.d, None, None, err, w.L, T, U_cap, w.d, w.N, bits, block,
                                  sbytes, 0, None, stream=stream)
    ms_full = time_steps(torch, stream, full, steps, warm)
    mb.mole_dedup_ids(ids[0], T, w.V, uniq, inv, nu, err, plan, stream=stream)
    ms_fetch = time_steps(torch, stream, fetch, steps, warm)
    if int(err.item()) != 0:
        raise RuntimeError("error flag set in the offloaded NF step")
    u0 = len(np.unique(ids_host[0]))
    row_bytes = code_row + scale_row * sbytes
    res = {"step": "dedup + fetch of the distinct ids' NF code and scale rows of all 24 layers from pinned host "
                   "memory + dequantising forward on the staged rows",
           "bits": bits, "block": block, "scale_bytes": sbytes, "tokens": T, "ms": ms_full,
           "tokens_per_s": T / (ms_full * 1e-3), "fetch_only_ms": ms_fetch,
           "fetched_bytes_per_id": w.L * row_bytes, "bf16_bytes_per_id": w.L * w.N * w.d * 2,
           "fetch_GBps": u0 * w.L * row_bytes / (ms_fetch * 1e-3) / 1e9,
           "host_table_bytes": int(host_codes.numel() + host_scales.numel())}
    del host_codes, host_scales
    return res


def storage_bench(torch, mb, wl, stream, L, steps, warm, layers=4, threads=16):
    """The table in a file (id-major), `layers` of the 24 layers to keep the file small: per step the
    distinct ids go to the host, their rows are read from the file into pinned memory and pulled to the
    device.  The file was just written, so reads are served by the page cache: this times the path, not a disk."""
    import numpy as np
    import tempfile
    w = wl.CONFIGS["offload410m"]
    T, U_cap, row_elems = w.T, w.T, w.N * w.d
    path = os.path.join(tempfile.gettempdir(), f"mole_bench_{os.getpid()}.molelut")
    f = mb.mole_lut_file_create(path, mb.MOLE_BF16, mb.MOLE_LAYOUT_ID_MAJOR, layers, w.V, w.N, w.d)
    try:
        t0 = time.perf_counter()
        lay = torch.empty((w.V, w.N, w.d), dtype=L.tabs.dtype, pin_memory=True)
        for l in range(layers):
            lay.copy_(L.tabs[l])
            torch.cuda.synchronize()
            mb.mole_lut_file_write_layer(f, l, lay, threads)
        handle, f = f, None
        mb.mole_lut_file_close(handle)
        t_write = time.perf_counter() - t0
        f, desc = mb.mole_lut_file_open(path)
        ids_host = np.stack([wl.token_ids(w, b) for b in range(N_ID_BATCHES)])
        ids = torch.from_numpy(ids_host).cuda()
        uniq = torch.empty((T,), dtype=torch.int32, device="cuda")
        inv = torch.empty((T,), dtype=torch.int32, device="cuda")
        nu = torch.zeros((1,), dtype=torch.int32, device="cuda")
        err = torch.zeros((1,), dtype=torch.int32, device="cuda")
        plan = torch.empty((mb.mole_dedup_workspace(T, w.V) // 4,), dtype=torch.int32, device="cuda")
        uniq_h = torch.empty((T + 1,), dtype=torch.int32, pin_memory=True)
        pinned = torch.empty((U_cap, layers, w.N, w.d), dtype=L.tabs.dtype, pin_memory=True)
        staging = torch.empty((layers, U_cap, w.N, w.d), dtype=L.tabs.dtype, device="cuda")
        h, sh, o = (x[:layers, :T].contiguous() for x in (L.h, L.shared, L.out))
        both = torch.empty((T + 1,), dtype=torch.int32, device="cuda")
        t_read = [0.0]

        def step(i):
            with torch.cuda.stream(stream):
                mb.mole_dedup_ids(ids[i % N_ID_BATCHES], T, w.V, uniq, inv, nu, err, plan, stream=stream)
                both[:T].copy_(uniq)
                both[T:].copy_(nu)
                uniq_h.copy_(both, non_blocking=True)
                stream.synchronize()
                U = int(uniq_h[T])
                t1 = time.perf_counter()
                mb.mole_lut_file_read_rows(f, uniq_h, U, pinned, threads)
                t_read[0] += time.perf_counter() - t1
                mb.mole_offload_fetch_idmajor(pinned, None, nu, staging, U_cap * row_elems, err, layers, U_cap,
                                              U_cap, w.d, w.N, mb.MOLE_BF16, stream=stream)
                mb.mole_lookup_forward_layers(staging, U_cap * row_elems, ids[i % N_ID_BATCHES], inv, h, L.W_r, sh,
                                              None, o, T * w.d, None, None, err, layers, T, U_cap, w.d, w.N,
                                              mb.MOLE_BF16, 0, None, stream=stream)
        n = min(steps, 50)
        for i in range(3):
            step(i)
        torch.cuda.synchronize()
        t_read[0] = 0.0
        t0 = time.perf_counter()
        for i in range(n):
            step(3 + i)
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) / n
        U = float(np.mean([len(np.unique(b)) for b in ids_host]))
        return {"step": "dedup, distinct ids to the host, rows read from an id-major LUT file into pinned memory "
                        "(page cache, not a disk), pulled to the device, staged forward",
                "layers_in_file": layers, "file_bytes": 4096 + layers * w.V * row_elems * 2, "reader_threads": threads,
                "write_file_s": t_write, "steps": n, "wall_ms_per_step": wall * 1e3,
                "read_rows_ms_per_step": t_read[0] / n * 1e3,
                "read_rows_GBps": U * layers * row_elems * 2 / (t_read[0] / n) / 1e9,
                "tokens_per_s": T / wall}
    finally:
        mb.mole_lut_file_close(f)
        if os.path.exists(path):
            os.remove(path)


def build_bench(torch, mb, wl, acc, stream, with_cpu=False):
    w = wl.CONFIGS["offload410m"]
    g = torch.Generator(device="cuda")
    g.manual_seed(77)
    E = torch.randn((w.V, w.d), generator=g, device="cuda").to(torch.bfloat16)
    W1 = (torch.randn((w.N, w.d, w.D), generator=g, device="cuda") * 0.02).to(torch.bfloat16)
    W2 = (torch.randn((w.N, w.D, w.d), generator=g, device="cuda") * 0.02).to(torch.bfloat16)
    lut = torch.empty((w.V, w.N, w.d), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty((mb.mole_build_lut_workspace(w.V, w.d, w.D, w.N, mb.MOLE_BF16),), dtype=torch.uint8, device="cuda")

    def f(i):
        mb.mole_build_lut(E, W1, None, W2, None, None, 0.0, lut, w.V, w.d, w.D, w.N, mb.MOLE_BF16, mb.MOLE_GELU_ERF,
                          ws, stream=stream)
    ms = time_steps(torch, stream, f, 3, 1)
    flops = acc.build_flops(w.V, w.d, w.D, w.N)
    # fp16 hidden activation (the library's choice for these inputs): executed = algorithmic flops; the
    # bf16 hi + lo variant runs the second GEMM over two planes
    executed = flops * (1.5 if os.environ.get("MOLE_BUILD_HIDDEN") == "split" else 1.0)
    res = {"ms": ms, "algorithmic_TFLOPs": flops / (ms * 1e-3) / 1e12,
           "algorithmic_frac_of_bf16_mfma_peak": flops / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
           "executed_mfma_TFLOPs": executed / (ms * 1e-3) / 1e12,
           "vocab_rows_per_s": w.V / (ms * 1e-3)}
    if with_cpu:
        # the fp64 oracle on a sample of vocabulary rows, extrapolated linearly to the whole table
        import oracle
        n = 512
        rows = torch.arange(0, w.V, w.V // n, device="cuda")[:n]
        host = lambda t: t.contiguous().view(torch.int16).cpu().numpy().view("uint16")
        Eh, W1h, W2h = host(E[rows]), host(W1), host(W2)
        t0 = time.perf_counter()
        oracle.build_lut(Eh, W1h, W2h)
        dt = time.perf_counter() - t0
        res["cpu_oracle"] = {"sample_rows": n, "seconds": dt, "cores": oracle.threads(),
                             "extrapolated_seconds_per_layer": dt / n * w.V,
                             "note": "timed on the sample, extrapolated linearly to V rows"}
    return res


if __name__ == "__main__":
    main()

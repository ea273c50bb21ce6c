#!/usr/bin/env python3
"""Benchmark of the KV-cache context-switch hot path on one MI355X.

A step is one pass of the whole path over one synthetic Llama-2-7B-shaped
4096-token cache (2 GiB fp16): score the chunks from attention (kv_score_chunks),
turn the densities into bit-widths and record offsets on the host
(kv_bits_from_scores, kv_chunk_offsets), quantise and pack every chunk
(kv_compress_chunks), build the gather list (kv_build_gather) and swap the whole
cache back in (kv_swapin_chunks).  Inputs are resident in HBM before the timed
region.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import paper_2403_11805_amd as kvs  # noqa: E402
from paper_2403_11805_amd import synth  # noqa: E402

HBM_PEAK_GBPS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2500.0
FRACTIONS = {"score-terciles": (1, 1, 3), "scores-25-50-25": (1, 2, 4)}


def find_workload(name):
    for wl in synth.WORKLOADS:
        if wl.name == name:
            return wl
    raise SystemExit(f"unknown workload {name!r}; have {[w.name for w in synth.WORKLOADS]}")


class Path:
    """Device buffers and the per-step call sequence for one context."""

    def __init__(self, wl, dev):
        g = wl.geom
        self.wl, self.g, self.dev = wl, g, dev
        self.shape = kvs.Shape(g.L, g.Hkv, g.Hq, g.D, g.N, g.T, g.G)
        self.kv = synth.make_kv(g, wl.seed, dev, wl.outlier_channels, wl.outlier_scale)
        self.R = wl.n_queries
        if self.R:
            self.q = synth.make_q(g, wl.seed, self.R, dev)
            self.ws = torch.empty(kvs.kv_score_workspace_bytes(self.shape, self.R), dtype=torch.uint8,
                                  device=dev)
            self.chunk_mass = torch.empty((g.L, g.Hq, g.n_chunks), dtype=torch.float32, device=dev)
            self.density = torch.empty(g.n_chunks, dtype=torch.float32, device=dev)
            self.density_host = torch.empty(g.n_chunks, dtype=torch.float32).pin_memory()
        if wl.bits_rule == "uniform":
            self.fixed_bits = synth.draw_bits_uniform(g.n_chunks, wl.seed).numpy()
        elif not self.R:
            self.fixed_bits = kvs.kv_bits_from_scores(synth.draw_scores(g.n_chunks, wl.seed).numpy(),
                                                      *FRACTIONS[wl.bits_rule])
        else:
            self.fixed_bits = None
        worst = kvs.kv_record_bytes(self.shape, 8) * g.n_chunks
        self.packed = torch.empty(worst, dtype=torch.uint8, device=dev)
        self.kv_out = torch.empty_like(self.kv)
        self.lists_host = torch.empty(g.n_chunks * 32 + 64, dtype=torch.uint8).pin_memory()
        self.lists_dev = torch.empty_like(self.lists_host, device=dev)
        self.all_chunks = np.arange(g.n_chunks, dtype=np.int32)
        self.ev = {k: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                   for k in ("score", "compress", "swapin")}
        self.packed_bytes = 0
        self.bits = None

    def _upload_lists(self, bits, off, src, dst, sb):
        """One pinned staging buffer, one async copy: bits | off | src_off | dst_tok | sel_bits."""
        n = self.g.n_chunks
        h = self.lists_host.numpy()
        o = 0
        views = {}
        for name, arr in (("off", off.view(np.uint8)), ("src", src.view(np.uint8)),
                          ("dst", dst.view(np.uint8)), ("bits", bits), ("sb", sb)):
            h[o:o + arr.size] = arr.reshape(-1)
            views[name] = (o, arr.size)
            o = (o + arr.size + 15) & ~15
        self.lists_dev.copy_(self.lists_host, non_blocking=True)
        d = self.lists_dev

        def cut(name, dtype):
            a, sz = views[name]
            return d[a:a + sz].view(dtype)
        return (cut("bits", torch.uint8), cut("off", torch.int64), cut("src", torch.int64),
                cut("dst", torch.int32), cut("sb", torch.uint8))

    def step(self):
        s = self.shape
        if self.R:
            self.ev["score"][0].record()
            kvs.kv_score_chunks(s, self.q, self.kv, kvs.KV_NORM_VISIBLE, self.ws, self.chunk_mass,
                                self.density)
            self.ev["score"][1].record()
            self.density_host.copy_(self.density, non_blocking=True)
            torch.cuda.current_stream().synchronize()
            bits = kvs.kv_bits_from_scores(self.density_host.numpy(), *FRACTIONS[self.wl.bits_rule])
        else:
            bits = self.fixed_bits
        off = kvs.kv_chunk_offsets(s, bits)
        src, dst, sb = kvs.kv_build_gather(s, off, bits, self.all_chunks)
        bits_d, off_d, src_d, dst_d, sb_d = self._upload_lists(bits, off, src, dst, sb)
        self.ev["compress"][0].record()
        kvs.kv_compress_chunks(s, self.kv, bits_d, off_d, self.packed)
        self.ev["compress"][1].record()
        self.ev["swapin"][0].record()
        kvs.kv_swapin_chunks(s, self.packed, src_d, dst_d, sb_d, self.kv_out)
        self.ev["swapin"][1].record()
        self.packed_bytes = int(off[-1])
        self.bits = bits

    def kernel_ms(self):
        return {k: a.elapsed_time(b) for k, (a, b) in self.ev.items() if k != "score" or self.R}


def cpu_baseline(path, budget_s=20.0):
    """The CPU oracle, as it stands, on a bounded sample of the same workload."""
    import oracle
    g = path.g
    one = oracle.Shape(g.L, g.Hkv, g.Hq, g.D, g.T, g.T, g.G)
    n_sample = 3
    sample = [0, g.n_chunks // 2, g.n_chunks - 1][:n_sample]
    t_cs = 0.0
    for i in sample:
        x = path.kv[:, :, :, i * g.T:(i + 1) * g.T, :].contiguous().cpu().numpy()
        b = np.array([path.bits[i]], dtype=np.uint8)
        off = oracle.chunk_offsets(one, b)
        t0 = time.perf_counter()
        packed = oracle.compress_chunks(one, x, b, off)
        out = np.empty(x.shape, dtype=np.float16)
        oracle.swapin_chunks(one, packed, *oracle.build_gather(one, off, b, [0]), out)
        t_cs += time.perf_counter() - t0
    full_s = t_cs / len(sample) * g.n_chunks
    desc = f"compress+swap-in of {len(sample)} of {g.n_chunks} chunks"
    if path.R:
        # a one-layer slice with as many kv heads as the oracle has threads (it runs heads in parallel)
        per_kv = g.Hq // g.Hkv
        n_kv = max(1, min(g.Hkv, oracle.threads() // per_kv))
        n_q = n_kv * per_kv
        hs = oracle.Shape(1, n_kv, n_q, g.D, g.N, g.T, g.G)
        q_host = path.q[0:1, 0:n_q].contiguous().cpu().numpy()
        k_host = path.kv[0:1, :, 0:n_kv].contiguous().cpu().numpy()
        t0 = time.perf_counter()
        oracle.score_chunks(hs, q_host, k_host, oracle.NORM_VISIBLE)
        t_sc = time.perf_counter() - t0
        full_s += t_sc * (g.L * g.Hq) / n_q
        desc += f"; scoring of {n_q} of {g.L * g.Hq} (layer, head) pairs"
    return {"value": round(g.elements * 2 / full_s / 1e9, 4), "unit": "GB/s", "cores": oracle.threads(),
            "kind": "oracle", "sample": desc + "; scaled to the whole cache"}


def read_traffic(workload, kernel):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, if there is one."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    try:
        for line in open(path):
            parts = line.replace("traffic_bytes=", " traffic_bytes=").split()
            if len(parts) >= 2 and parts[0] == kernel and parts[1].startswith("traffic_bytes="):
                return int(float(parts[1].split("=", 1)[1]))
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama2-7b-4k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="N",
                    help="instead of the benchmark, run N pass-through (16-bit) compress launches: "
                         "a plain copy of the whole cache, used to scale rocprofv3 byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("this build runs on one GPU: the path has no collectives; use --gpus 1")
    if not torch.cuda.is_available():
        raise SystemExit("no GPU visible: the benchmark has no CPU path")
    kvs.binding.lib()   # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    wl = find_workload(args.workload)
    path = Path(wl, dev)
    g = wl.geom

    if args.calibrate_copy:
        bits = np.full(g.n_chunks, 16, dtype=np.uint8)
        off = kvs.kv_chunk_offsets(path.shape, bits)
        bits_d = torch.from_numpy(bits).to(dev)
        off_d = torch.from_numpy(off.view(np.int64)).to(dev)
        for _ in range(args.calibrate_copy):
            kvs.kv_compress_chunks(path.shape, path.kv, bits_d, off_d, path.kv_out.view(torch.uint8))
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": args.calibrate_copy, "bytes_read": g.elements * 2,
                          "bytes_written": g.elements * 2}))
        return
    for _ in range(args.warmup):
        path.step()
        torch.cuda.synchronize()
    sums = {}
    t0 = time.perf_counter()
    for _ in range(args.steps):
        path.step()
        torch.cuda.synchronize()
        for k, v in path.kernel_ms().items():
            sums.setdefault(k, []).append(v)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3

    cache_bytes = g.elements * 2
    alg = {"compress": cache_bytes + path.packed_bytes, "swapin": cache_bytes + path.packed_bytes}
    if path.R:
        alg["score"] = (g.L * g.Hkv * g.N * g.D * 2 + g.L * g.Hq * path.R * g.D * 2 +
                        g.L * g.Hq * g.n_chunks * 4)
    kernels = {}
    for k, v in sums.items():
        ms = float(np.mean(v))
        gbps = alg[k] / ms / 1e6
        kernels[k] = {"ms": round(ms, 4), "ms_min": round(float(np.min(v)), 4),
                      "algorithmic_bytes": alg[k], "hbm_gbps": round(gbps, 1),
                      "hbm_frac": round(gbps / HBM_PEAK_GBPS, 4),
                      "fp16_equiv_gbps": round(cache_bytes / ms / 1e6, 1)}
    if path.R:
        flops = 2.0 * path.R * g.N * g.D * g.L * g.Hq
        kernels["score"]["mfma_tflops"] = round(flops / kernels["score"]["ms"] / 1e9, 2)
        kernels["score"]["mfma_frac"] = round(kernels["score"]["mfma_tflops"] / MFMA_F16_PEAK_TFLOPS, 4)
    names = {"compress": "compress_kernel", "swapin": "swapin_kernel", "score": "score_tiles_kernel"}
    dom = max(kernels, key=lambda k: kernels[k]["ms"])
    roofline = {"kernel": names[dom], "bound": "hbm", "achieved": kernels[dom]["hbm_gbps"],
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": kernels[dom]["hbm_frac"],
                "traffic": read_traffic(wl.name, names[dom])}

    out = {
        "metric": "KV GB/s (fp16-equiv) compress + swap-in, % of HBM peak; ms per 4K-ctx switch",
        "value": round(cache_bytes / ms_per_step / 1e6, 2),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: [L={g.L},K/V,Hkv={g.Hkv},N={g.N},D={g.D}] fp16, "
                               f"chunk {g.T}, group {g.G}, R={path.R}, widths {wl.bits_rule}",
                   "cache_bytes": cache_bytes, "packed_bytes": path.packed_bytes,
                   "step": "score + bits/offsets (host) + compress + gather list (host) + swap-in"},
        "ms_per_4k_ctx_switch": kernels["swapin"]["ms"],
        "compress_pct_hbm_peak": round(100 * kernels["compress"]["hbm_frac"], 2),
        "swapin_pct_hbm_peak": round(100 * kernels["swapin"]["hbm_frac"], 2),
        "kernels": kernels,
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(path)
    print(json.dumps(out))


if __name__ == "__main__":
    main()

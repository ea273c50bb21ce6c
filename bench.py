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

    def __init__(self, wl, dev, host_plan=False, fmt=0, ratio=None):
        g = wl.geom
        self.wl, self.g, self.dev = wl, g, dev
        self.ratio = ratio                  # (num, den): thresholds from a global ratio (Eq. 2-3) instead of fixed fractions
        self.shape = kvs.Shape(g.L, g.Hkv, g.Hq, g.D, g.N, g.T, g.G, fmt)
        self.kv = synth.make_kv(g, wl.seed, dev, wl.outlier_channels, wl.outlier_scale)
        # caches below ~640 MB would be served from the 256 MB Infinity Cache when reused every
        # step: rotate over enough independent copies that each step streams from HBM
        cache_bytes = g.elements * 2
        self.n_sets = max(1, min(1024, -(-640 * 2 ** 20 // cache_bytes))) if cache_bytes < 640 * 2 ** 20 else 1
        self.kv_sets = [self.kv] + [self.kv.clone() for _ in range(self.n_sets - 1)]
        self.step_no = 0
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
        self.packed_sets = [torch.empty(worst, dtype=torch.uint8, device=dev) for _ in range(self.n_sets)]
        self.out_sets = [torch.empty_like(self.kv) for _ in range(self.n_sets)]
        self.packed, self.kv_out = self.packed_sets[0], self.out_sets[0]
        self.lists_host = torch.empty(g.n_chunks * 32 + 64, dtype=torch.uint8).pin_memory()
        self.lists_dev = torch.empty_like(self.lists_host, device=dev)
        self.all_chunks = np.arange(g.n_chunks, dtype=np.int32)
        # one set of events per step in flight, read back after the timed region
        self.ev_sets = [self._event_set()]
        self.ev = self.ev_sets[0]
        self.packed_bytes = 0
        self.bits = None
        self.host_stages = False
        # widths, offsets and the gather list of the whole cache stay on the device when the
        # widths come from the scores: the step then has no host round trip
        self.device_plan = bool(self.R) and not host_plan
        if self.device_plan:
            n = g.n_chunks
            self.bits_d = torch.empty(n, dtype=torch.uint8, device=dev)
            self.off_d = torch.empty(n + 1, dtype=torch.int64, device=dev)
            self.dst_d = torch.empty(n, dtype=torch.int32, device=dev)

    @staticmethod
    def _event_set():
        """Five events bound the four stages of a step that stays on the device: the event behind one stage
        is the one in front of the next (an event record costs some 3.5 us of stream time, so a step
        carries as few as it can).  The host-planned step has host work between scoring and compression:
        there a sixth event opens the compress stage."""
        e = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
        return {"score": (e[0], e[1]), "plan": (e[1], e[2]), "compress": (e[2], e[3]), "swapin": (e[3], e[4]),
                "compress_host": (e[5], e[3])}

    def reserve_event_sets(self, n):
        """Steps numbered modulo n record into event sets of their own (kernel_ms(i) reads them later)."""
        while len(self.ev_sets) < n:
            self.ev_sets.append(self._event_set())

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

    def _plan_dev(self):
        """Widths, offsets and gather list on the device: the workload's fixed fractions (Eq. 2 with fixed
        thresholds) or, with --ratio, the thresholds of Eq. 2-3 for that global ratio."""
        if self.ratio:
            kvs.kv_plan_optimise_dev(self.shape, self.density, self.ratio[0], self.ratio[1], kvs.KV_OBJ_BITS_TO_DENSE,
                                     self.bits_d, self.off_d, self.dst_d)
        else:
            kvs.kv_plan_chunks_dev(self.shape, self.density, *FRACTIONS[self.wl.bits_rule], self.bits_d, self.off_d,
                                   self.dst_d)

    def step(self, record_events=True):
        s = self.shape
        k = self.step_no % self.n_sets
        self.ev = self.ev_sets[self.step_no % len(self.ev_sets)]
        self.step_no += 1
        self.kv, self.packed, self.kv_out = self.kv_sets[k], self.packed_sets[k], self.out_sets[k]
        if self.device_plan and not record_events:
            n = self.g.n_chunks
            kvs.kv_score_chunks(s, self.q, self.kv, kvs.KV_NORM_VISIBLE, self.ws, self.chunk_mass,
                                self.density)
            self._plan_dev()
            kvs.kv_compress_chunks(s, self.kv, self.bits_d, self.off_d, self.packed)
            kvs.kv_swapin_chunks(s, self.packed, self.off_d[:n], self.dst_d, self.bits_d, self.kv_out)
            return
        if not self.R and not record_events:
            # fixed widths: the lists of the last timed step are still on the device (graph capture)
            bits_d, off_d, src_d, dst_d, sb_d = self.fixed_lists
            kvs.kv_compress_chunks(s, self.kv, bits_d, off_d, self.packed)
            kvs.kv_swapin_chunks(s, self.packed, src_d, dst_d, sb_d, self.kv_out)
            return
        if self.device_plan:
            n = self.g.n_chunks
            self.ev["score"][0].record()
            kvs.kv_score_chunks(s, self.q, self.kv, kvs.KV_NORM_VISIBLE, self.ws, self.chunk_mass,
                                self.density)
            self.ev["plan"][0].record()
            self._plan_dev()
            self.ev["compress"][0].record()
            kvs.kv_compress_chunks(s, self.kv, self.bits_d, self.off_d, self.packed)
            self.ev["swapin"][0].record()
            kvs.kv_swapin_chunks(s, self.packed, self.off_d[:n], self.dst_d, self.bits_d, self.kv_out)
            self.ev["swapin"][1].record()
            self.host_stages = False
            return
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
        self.fixed_lists = (bits_d, off_d, src_d, dst_d, sb_d)
        self.ev["compress_host"][0].record()
        kvs.kv_compress_chunks(s, self.kv, bits_d, off_d, self.packed)
        self.ev["swapin"][0].record()
        kvs.kv_swapin_chunks(s, self.packed, src_d, dst_d, sb_d, self.kv_out)
        self.ev["swapin"][1].record()
        self.host_stages = True
        self.packed_bytes = int(off[-1])
        self.bits = bits

    def kernel_ms(self, step=None):
        ev = self.ev if step is None else self.ev_sets[step % len(self.ev_sets)]
        stages = {k: ev[k] for k in ("score", "plan", "compress", "swapin")}
        if self.host_stages:
            stages["compress"] = ev["compress_host"]
        return {k: a.elapsed_time(b) for k, (a, b) in stages.items()
                if (k != "score" or self.R) and (k != "plan" or self.device_plan)}

    def fetch_plan(self):
        """After the last step: the widths and the packed size the device planned."""
        if self.device_plan:
            torch.cuda.synchronize()
            self.bits = self.bits_d.cpu().numpy()
            self.packed_bytes = int(self.off_d[-1])


def run_pipeline(wl, args, dev):
    """The swapping-recompute pipeline of Sec. 3.3, measured end to end for one context whose records
    sit in pinned host memory: the first x chunks are recomputed through all L layers (a prefix
    attends only to itself, so it needs none of the chunks still in flight) on one stream while the
    other chunks are loaded by kv_swapin_pinned on two more.  x = 0 is the plain Load.  Every layer
    has weights of its own (seeded), so that no layer finds its weights in the last-level cache."""
    g = wl.geom
    fmt = 3 if args.format == "f16h" else 0
    shape = kvs.Shape(g.L, g.Hkv, g.Hq, g.D, g.N, g.T, g.G, fmt)
    d_model, d_ff = g.Hq * g.D, args.d_ff
    dims = kvs.LayerDims(d_model, d_ff)
    kv = synth.make_kv(g, wl.seed, dev, wl.outlier_channels, wl.outlier_scale)
    bits = kvs.kv_bits_from_scores(synth.draw_scores(g.n_chunks, wl.seed).numpy(), 1, 1, 3)
    off = kvs.kv_chunk_offsets(shape, bits)
    total = int(off[-1])
    packed = torch.empty(total, dtype=torch.uint8, device=dev)
    kvs.kv_compress_chunks(shape, kv, torch.from_numpy(bits).to(dev), torch.from_numpy(off.view(np.int64)).to(dev),
                           packed)
    pinned = torch.empty(total, dtype=torch.uint8).pin_memory()
    pinned.copy_(packed)
    torch.cuda.synchronize()
    del packed
    weights = [synth.make_layer_weights(d_model, g.Hq, g.Hkv, g.D, d_ff, wl.seed, dev, layer=l) for l in range(g.L)]
    copy_s, comp_s, re_s = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    loader = kvs.Loader()              # owns the events of the staging slots for every streaming Load below
    staging = torch.empty(args.stream_buffers * (args.stream_slot_mib << 20), dtype=torch.uint8, device=dev)
    out = torch.zeros_like(kv)
    rc = kvs.Recompute()
    rows = []
    xs = [x for x in (0, 8, 16, 24, 32, 48, 64) if x < g.n_chunks]
    for x in xs:
        rest = np.arange(x, g.n_chunks, dtype=np.int32)
        src, dst, sb = kvs.kv_build_gather(shape, off, bits, rest)
        if x:
            idx_dev = torch.arange(x, dtype=torch.int32, device=dev)
            x0 = synth.make_hidden(x * g.T, d_model, wl.seed, dev)          # the prefix's embedded tokens
            hid = [torch.empty_like(x0), torch.empty_like(x0)]
            ws = torch.empty(kvs.kv_recompute_workspace_bytes(shape, dims, x), dtype=torch.uint8, device=dev)
            if not args.no_tune:
                rc.tune(shape, dims, weights[0], x, ws)
        wall, re_ms = [], []
        for it in range(args.warmup + args.steps):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            loader.swapin_stream(shape, pinned, src, dst, sb, staging, args.stream_buffers, out, copy_s, comp_s)
            if x:
                with torch.cuda.stream(re_s):
                    for l in range(g.L):
                        rc.layer(shape, dims, weights[l], l, idx_dev, x0 if l == 0 else hid[l & 1], out,
                                 hid[(l + 1) & 1], ws, re_s)
                re_s.synchronize()
                t_re = time.perf_counter()
            comp_s.synchronize(); copy_s.synchronize()
            t1 = time.perf_counter()
            if it >= args.warmup:
                wall.append((t1 - t0) * 1e3)
                re_ms.append((t_re - t0) * 1e3 if x else 0.0)
        loaded = int(sum(int(off[i + 1] - off[i]) for i in rest))
        rows.append({"recomputed_chunks": x, "loaded_bytes": loaded, "delay_ms": round(float(np.median(wall)), 3),
                     "recompute_done_ms": round(float(np.median(re_ms)), 3)})
        if x:
            assert bool(torch.isfinite(out[:, :, :, :x * g.T].float()).all()), "recomputed K/V not finite"
    # the loaded chunks equal the resident Load bit for bit (last configuration)
    ref = torch.zeros_like(kv)
    kvs.kv_load_chunks(shape, pinned.to(dev), off, bits, np.arange(xs[-1], g.n_chunks, dtype=np.int32), ref)
    torch.cuda.synchronize()
    assert torch.equal(out[:, :, :, xs[-1] * g.T:].view(torch.int16), ref[:, :, :, xs[-1] * g.T:].view(torch.int16))

    # The paper's own order for INTERLEAVED missing chunks: layer by layer.  x of the heaviest (8-bit)
    # chunks, spread over the context, are recomputed; layer l of the others is loaded by
    # kv_swapin_layers straight from the pinned pool on an IO stream, and the recompute of layer l waits
    # for it (a recomputed token attends to every earlier token of its layer, loaded ones included).
    io_s = comp_s        # (a further stream may share a hardware queue with the recompute stream and serialise)
    heavy = np.flatnonzero(bits == 8)
    layer_done = [torch.cuda.Event() for _ in range(g.L)]
    rows_il = []
    for x in [x for x in xs if x <= len(heavy)]:
        pick = np.unique(heavy[np.linspace(0, len(heavy) - 1, x).astype(np.int64)]).astype(np.int32) if x else \
            np.zeros(0, dtype=np.int32)
        assert len(pick) == x
        rest = np.setdiff1d(np.arange(g.n_chunks, dtype=np.int32), pick)
        src, dst, sb = kvs.kv_build_gather(shape, off, bits, rest)
        lists_d = (torch.from_numpy(src.view(np.int64)).to(dev), torch.from_numpy(dst).to(dev),
                   torch.from_numpy(sb).to(dev))
        if x:
            idx_dev = torch.from_numpy(pick).to(dev)
            x0 = synth.make_hidden(x * g.T, d_model, wl.seed, dev)
            hid = [torch.empty_like(x0), torch.empty_like(x0)]
            ws = torch.empty(kvs.kv_recompute_workspace_bytes(shape, dims, x), dtype=torch.uint8, device=dev)
        out.zero_()
        wall = []
        for it in range(args.warmup + args.steps):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for l in range(g.L):          # the host hands out layer l's Load, then layer l's recompute
                kvs.kv_swapin_layers(shape, pinned, *lists_d, l, l + 1, out, io_s)
                layer_done[l].record(io_s)
                if x:
                    re_s.wait_event(layer_done[l])
                    rc.layer(shape, dims, weights[l], l, idx_dev, x0 if l == 0 else hid[l & 1], out,
                             hid[(l + 1) & 1], ws, re_s)
            io_s.synchronize(); re_s.synchronize()
            t1 = time.perf_counter()
            if it >= args.warmup:
                wall.append((t1 - t0) * 1e3)
        loaded = int(sum(int(off[i + 1] - off[i]) for i in rest))
        rows_il.append({"recomputed_chunks": x, "loaded_bytes": loaded, "delay_ms": round(float(np.median(wall)), 3)})
        # loaded chunks: the resident Load's bytes; recomputed ones: finite values in their places
        ref.zero_()
        kvs.kv_load_chunks(shape, pinned, off, bits, rest, ref)
        torch.cuda.synchronize()
        keep = torch.ones(g.n_chunks, dtype=torch.bool)
        keep[torch.from_numpy(pick.astype(np.int64))] = False
        tok = keep.repeat_interleave(g.T).to(dev)
        assert torch.equal(out[:, :, :, tok].view(torch.int16), ref[:, :, :, tok].view(torch.int16))
        assert bool(torch.isfinite(out[:, :, :, ~tok].float()).all())
    # The same layer-by-layer order with the context stored as one pool per layer (records of a
    # one-layer shape): a layer's records are then contiguous runs, kv_swapin_pinned moves them with
    # the copy engines, and the recompute of layer l on its own stream waits for that layer's Load.
    shape1 = kvs.Shape(1, g.Hkv, g.Hq, g.D, g.N, g.T, g.G, fmt)
    off1 = kvs.kv_chunk_offsets(shape1, bits)
    total1 = int(off1[-1])
    pools = torch.empty((g.L, total1), dtype=torch.uint8).pin_memory()
    tmp = torch.empty(total1, dtype=torch.uint8, device=dev)
    bits_d, off1_d = torch.from_numpy(bits).to(dev), torch.from_numpy(off1.view(np.int64)).to(dev)
    for l in range(g.L):
        kvs.kv_compress_chunks(shape1, kv[l:l + 1], bits_d, off1_d, tmp)
        pools[l].copy_(tmp)
    torch.cuda.synchronize()
    del tmp
    stage2 = torch.empty(8 * (8 << 20), dtype=torch.uint8, device=dev)
    rows_lm = []
    for x in [x for x in xs if x <= len(heavy)]:
        pick = np.unique(heavy[np.linspace(0, len(heavy) - 1, x).astype(np.int64)]).astype(np.int32) if x else \
            np.zeros(0, dtype=np.int32)
        rest = np.setdiff1d(np.arange(g.n_chunks, dtype=np.int32), pick)
        src1, dst1, sb1 = kvs.kv_build_gather(shape1, off1, bits, rest)
        if x:
            idx_dev = torch.from_numpy(pick).to(dev)
            x0 = synth.make_hidden(x * g.T, d_model, wl.seed, dev)
            hid = [torch.empty_like(x0), torch.empty_like(x0)]
            ws = torch.empty(kvs.kv_recompute_workspace_bytes(shape, dims, x), dtype=torch.uint8, device=dev)
        out.zero_()
        wall = []
        for it in range(args.warmup + args.steps):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for l in range(g.L):
                # one handle, one staging area: a call waits by itself for the slots its predecessor still uses
                loader.swapin_stream(shape1, pools[l], src1, dst1, sb1, stage2, 8, out[l:l + 1], copy_s, comp_s)
                layer_done[l].record(comp_s)
                if x:
                    re_s.wait_event(layer_done[l])
                    rc.layer(shape, dims, weights[l], l, idx_dev, x0 if l == 0 else hid[l & 1], out,
                             hid[(l + 1) & 1], ws, re_s)
            comp_s.synchronize(); copy_s.synchronize(); re_s.synchronize()
            t1 = time.perf_counter()
            if it >= args.warmup:
                wall.append((t1 - t0) * 1e3)
        rows_lm.append({"recomputed_chunks": x, "loaded_bytes": int(sum(int(off1[i + 1] - off1[i]) for i in rest)) * g.L,
                        "delay_ms": round(float(np.median(wall)), 3)})
        ref.zero_()
        kvs.kv_load_chunks(shape, pinned, off, bits, rest, ref)
        torch.cuda.synchronize()
        keep = torch.ones(g.n_chunks, dtype=torch.bool)
        keep[torch.from_numpy(pick.astype(np.int64))] = False
        tok = keep.repeat_interleave(g.T).to(dev)
        assert torch.equal(out[:, :, :, tok].view(torch.int16), ref[:, :, :, tok].view(torch.int16))
        assert bool(torch.isfinite(out[:, :, :, ~tok].float()).all())
    rc.close()
    loader.close()
    best = min(rows, key=lambda r: r["delay_ms"])
    base = rows[0]["delay_ms"]
    best_il = min(rows_il, key=lambda r: r["delay_ms"])
    best_lm = min(rows_lm, key=lambda r: r["delay_ms"])
    return {
        "metric": "context Load from pinned host memory with the swapping-recompute pipeline (Sec. 3.3), ms",
        "value": best["delay_ms"], "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": best["delay_ms"], "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{wl.name}: [L={g.L},K/V,Hkv={g.Hkv},N={g.N},D={g.D}] fp16, chunk {g.T}, records of "
                               f"{total} bytes in pinned host memory{' (group parameters in binary16)' if fmt == 3 else ''}; "
                               f"Llama-2-7B-sized layers, d_ff {d_ff}",
                   "step": "recompute of the first x chunks through all layers || streaming Load of the others"},
        "load_only_ms": base, "best": best, "gain": round(1.0 - best["delay_ms"] / base, 4), "rows": rows,
        "layer_wise_interleaved": {
            "step": "x heaviest chunks, interleaved with the others, recomputed layer by layer; layer l of the "
                    "others loaded by kv_swapin_layers straight from the pinned pool, recompute of layer l waits for it",
            "load_only_ms": rows_il[0]["delay_ms"], "best": best_il,
            "gain": round(1.0 - best_il["delay_ms"] / rows_il[0]["delay_ms"], 4), "rows": rows_il},
        "layer_wise_layer_major_pools": {
            "step": "the same interleaved chunks and layer-by-layer order with the context stored as one pool per "
                    "layer: kv_swapin_stream per layer (copy engines, one loader handle), recompute of layer l waits for that layer",
            "load_only_ms": rows_lm[0]["delay_ms"], "best": best_lm,
            "gain": round(1.0 - best_lm["delay_ms"] / rows_lm[0]["delay_ms"], 4), "rows": rows_lm},
    }


def graph_ms_per_step(path, args):
    """The device-planned step captured in a HIP graph (one per rotating buffer set) and replayed
    K times between two synchronisations.  The path records no events while capturing."""
    side = torch.cuda.Stream()
    graphs = []
    saved, path.ev_sets = path.ev_sets, [None]
    try:
        for k in range(path.n_sets):
            path.step_no = k
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                path.step(record_events=False)
            graphs.append(graph)
    finally:
        path.ev_sets = saved
    for i in range(args.warmup):
        graphs[i % len(graphs)].replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        graphs[i % len(graphs)].replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / args.steps * 1e3


def cpu_baseline(path):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: once on all the threads
    it takes (the reported value) and once on a single thread (the per-core rate, which does not
    depend on how many cores a box has).  Where the workload scores chunks the oracle scores the whole
    cache; its densities also tell how many chunks would get another width than under the GPU's."""
    import oracle
    g = path.g
    n_all = oracle.threads()
    one = oracle.Shape(g.L, g.Hkv, g.Hq, g.D, g.T, g.T, g.G)

    def quant_seconds(sample):
        t = 0.0
        for i in sample:
            x = path.kv[:, :, :, i * g.T:(i + 1) * g.T, :].contiguous().cpu().numpy()
            b = np.array([path.bits[i]], dtype=np.uint8)
            off = oracle.chunk_offsets(one, b)
            t0 = time.perf_counter()
            packed = oracle.compress_chunks(one, x, b, off)
            out = np.empty(x.shape, dtype=np.float16)
            oracle.swapin_chunks(one, packed, *oracle.build_gather(one, off, b, [0]), out)
            t += time.perf_counter() - t0
        return t / len(sample) * g.n_chunks

    first = {b: int(np.flatnonzero(path.bits == b)[0]) for b in (8, 4, 2) if (path.bits == b).any()}
    sample = sorted(set(first.values()) | {0, g.n_chunks // 2, g.n_chunks - 1})
    full_s = quant_seconds(sample)
    desc = f"compress+swap-in of {len(sample)} of {g.n_chunks} chunks, scaled to all"
    extra = {}
    if path.R:
        q_host = path.q.cpu().numpy()
        kv_host = path.kv.cpu().numpy()
        os_ = oracle.Shape(g.L, g.Hkv, g.Hq, g.D, g.N, g.T, g.G)
        t0 = time.perf_counter()
        _, d_orc = oracle.score_chunks(os_, q_host, kv_host, oracle.NORM_VISIBLE)
        full_s += time.perf_counter() - t0
        desc += f"; scoring of all {g.L * g.Hq} (layer, head) pairs"
        num8, num4, den = FRACTIONS[path.wl.bits_rule]
        moved = int((oracle.bits_from_scores(d_orc, num8, num4, den) != path.bits).sum())
        extra["chunks_in_another_bucket_under_oracle_scores"] = moved
    # one thread: one chunk, one (layer, head) pair
    oracle.set_threads(1)
    try:
        one_s = quant_seconds(sample[:1])
        if path.R:
            hs = oracle.Shape(1, 1, 1, g.D, g.N, g.T, g.G)
            q1 = path.q[0:1, 0:1].contiguous().cpu().numpy()
            k1 = path.kv[0:1, :, 0:1].contiguous().cpu().numpy()
            t0 = time.perf_counter()
            oracle.score_chunks(hs, q1, k1, oracle.NORM_VISIBLE)
            one_s += (time.perf_counter() - t0) * g.L * g.Hq
    finally:
        oracle.set_threads(n_all)
    return {"value": round(g.elements * 2 / full_s / 1e9, 4), "unit": "GB/s", "cores": n_all,
            "kind": "oracle", "sample": desc,
            "per_core_value": round(g.elements * 2 / one_s / 1e9, 5),
            "per_core_sample": "one thread: one chunk" + (" and one (layer, head) pair" if path.R else "") + ", scaled to all",
            **extra}


def clock_state():
    """GPU clocks and power state as the driver reports them just before the timed region (sysfs of
    the first amdgpu card; None where the box does not expose it).  Read once, outside the timing."""
    import glob
    out = {}
    for card in sorted(glob.glob("/sys/class/drm/card*/device")):
        if not os.path.exists(os.path.join(card, "pp_dpm_sclk")):
            continue
        for key, name in (("sclk", "pp_dpm_sclk"), ("mclk", "pp_dpm_mclk"), ("fclk", "pp_dpm_fclk")):
            try:
                lines = open(os.path.join(card, name)).read().split("\n")
                active = [l for l in lines if l.strip().endswith("*")]
                if active:
                    out[f"{key}_mhz"] = int("".join(ch for ch in active[0].split(":")[1] if ch.isdigit()))
            except (OSError, ValueError, IndexError):
                pass
        try:
            out["performance_level"] = open(os.path.join(card, "power_dpm_force_performance_level")).read().strip()
        except OSError:
            pass
        try:
            hw = glob.glob(os.path.join(card, "hwmon", "hwmon*", "power1_average"))
            if hw:
                out["power_w"] = round(int(open(hw[0]).read()) / 1e6, 1)
        except (OSError, ValueError):
            pass
        break
    try:
        out["max_sclk_mhz"] = torch.cuda.get_device_properties(0).clock_rate // 1000
    except Exception:
        pass
    return out or None


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


def pctl(v, q):
    return float(np.percentile(np.asarray(v, dtype=np.float64), q))


def run_pool(wl, args, dev):
    """Multi-app context pool: every context is compressed once into a device-resident pool;
    a step is one context switch = seeded context draw (the paper's Random pattern, Sec. 4),
    LCTRU lock/touch, seeded 40 % chunk subset, Load of these chunks (kv_load_chunks)."""
    g = wl.geom
    shape = kvs.Shape(g.L, g.Hkv, g.Hq, g.D, g.N, g.T, g.G)
    n_ctx = args.contexts or wl.n_contexts
    n_sel = int(wl.select_frac * g.n_chunks)
    ctx_bits, ctx_off, pools = [], [], []
    queue = kvs.Lctru()
    t_build = time.perf_counter()
    for c in range(n_ctx):
        kv = synth.make_kv(g, wl.seed, dev, wl.outlier_channels, wl.outlier_scale, context=c)
        bits = synth.draw_bits_uniform(g.n_chunks, wl.seed, context=c).numpy()
        off = kvs.kv_chunk_offsets(shape, bits)
        pool = torch.empty(int(off[-1]), dtype=torch.uint8, device=dev)
        kvs.kv_compress_chunks(shape, kv, torch.from_numpy(bits).to(dev),
                               torch.from_numpy(off.view(np.int64)).to(dev), pool)
        torch.cuda.synchronize()
        ctx_bits.append(bits); ctx_off.append(off); pools.append(pool)
        for i in range(g.n_chunks):
            queue.insert(c, i, int(bits[i]), int(off[i + 1] - off[i]), c)
        del kv
    t_build = time.perf_counter() - t_build
    caches = [torch.zeros(shape.kv_dims, dtype=torch.float16, device=dev) for _ in range(min(n_ctx, 4))]
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    draw = torch.Generator().manual_seed(wl.seed * 7919 + 1)
    order_ctx = torch.randint(0, n_ctx, (args.warmup + args.steps,), generator=draw).tolist()
    subsets = [synth.draw_subset(g.n_chunks, n_sel, wl.seed, draw=it).numpy() for it in range(len(order_ctx))]
    k_ms, wall_ms, host_ms, moved = [], [], [], []
    for it, c in enumerate(order_ctx):
        sel = subsets[it]                   # which chunks a call needs is an input, drawn beforehand
        t0 = time.perf_counter()
        queue.lock(c)                       # working set of the call
        queue.touch_ctx(c, 1000 + it)
        t1 = time.perf_counter()
        ev0.record()
        # Load in one call: the gather list is built on the host and travels in the kernel arguments
        kvs.kv_load_chunks(shape, pools[c], ctx_off[c], ctx_bits[c], sel, caches[it % len(caches)])
        ev1.record()
        torch.cuda.synchronize()
        queue.unlock(c)
        t2 = time.perf_counter()
        if it >= args.warmup:
            k_ms.append(ev0.elapsed_time(ev1)); wall_ms.append((t2 - t0) * 1e3); host_ms.append((t1 - t0) * 1e3)
            packed_b = int(sum(int(ctx_off[c][i + 1] - ctx_off[c][i]) for i in sel))
            moved.append(packed_b + n_sel * g.elements * 2 // g.n_chunks)
    # the same Loads enqueued eight at a time between one event pair: per-launch time without the dispatch
    # of a single launch and without the host's part between the events
    b2b_ms, b2b_bytes = [], []
    for rep in range(12):
        ev0.record()
        for j in range(8):
            it = (rep * 8 + j) % len(subsets)
            c = order_ctx[it]
            kvs.kv_load_chunks(shape, pools[c], ctx_off[c], ctx_bits[c], subsets[it], caches[j % len(caches)])
            b2b_bytes.append(int(sum(int(ctx_off[c][i + 1] - ctx_off[c][i]) for i in subsets[it])) +
                             n_sel * g.elements * 2 // g.n_chunks)
        ev1.record()
        torch.cuda.synchronize()
        b2b_ms.append(ev0.elapsed_time(ev1) / 8)
    b2b = float(np.median(b2b_ms[2:]))
    # the Fault primitive: Load of one chunk, issue to completion as the caller sees it
    fault_wall = []
    for it in range(264):
        c = order_ctx[it % len(order_ctx)]
        one = subsets[it % len(subsets)][it % n_sel:it % n_sel + 1]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        kvs.kv_load_chunks(shape, pools[c], ctx_off[c], ctx_bits[c], one, caches[it % len(caches)])
        torch.cuda.synchronize()
        fault_wall.append((time.perf_counter() - t0) * 1e3)
    # A context whose records were reclaimed to pinned host memory (Sec. 3.4: Reclaim moves no data, the
    # records are already there): Fault and switch-sized Loads from the host, the kernel reading the
    # pinned pool itself (in place) or kv_swapin_pinned staging it through the copy engines.
    c0 = order_ctx[0]
    host_pool = torch.empty(pools[c0].numel(), dtype=torch.uint8).pin_memory()
    host_pool.copy_(pools[c0])
    torch.cuda.synchronize()
    hs_copy, hs_comp = torch.cuda.Stream(), torch.cuda.Stream()
    stage = torch.empty(2 * (16 << 20), dtype=torch.uint8, device=dev)
    from_host = []
    for n in (1, n_sel):
        t_place, t_staged, rec_bytes = [], [], []
        for it in range(40):
            sel = subsets[it % len(subsets)][:n]
            rec_bytes.append(sum(int(ctx_off[c0][i + 1] - ctx_off[c0][i]) for i in sel))
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            kvs.kv_load_chunks(shape, host_pool, ctx_off[c0], ctx_bits[c0], sel, caches[0])
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            src, dst, sb = kvs.kv_build_gather(shape, ctx_off[c0], ctx_bits[c0], sel)
            kvs.kv_swapin_pinned(shape, host_pool, src, dst, sb, stage, 2, caches[0], hs_copy, hs_comp)
            hs_comp.synchronize(); hs_copy.synchronize()
            t2 = time.perf_counter()
            t_place.append((t1 - t0) * 1e3); t_staged.append((t2 - t1) * 1e3)
        mb = float(np.mean(rec_bytes))
        from_host.append({"chunks": n, "record_mib": round(mb / 2**20, 2), "in_place_ms_p50": round(pctl(t_place[8:], 50), 4),
                          "staged_ms_p50": round(pctl(t_staged[8:], 50), 4), "link_ms_at_measured_rate": round(mb / 57e6, 4)})
    order_ms = 1e9
    for _ in range(3):                     # the first call pays one-off interpreter costs
        order_t0 = time.perf_counter()
        eviction_order = queue.order()
        order_ms = min(order_ms, (time.perf_counter() - order_t0) * 1e3)
    queue.close()
    sel_fp16 = n_sel * g.elements * 2 // g.n_chunks
    gbps = float(np.mean(moved)) / float(np.mean(k_ms)) / 1e6
    gbps_med = float(np.median(np.asarray(moved) / np.asarray(k_ms))) / 1e6     # a stall of the host thread moves the mean
    return {
        "metric": "KV GB/s (fp16-equiv) compress + swap-in, % of HBM peak; ms per 4K-ctx switch",
        "value": round(sel_fp16 / float(np.mean(wall_ms)) / 1e6, 2), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(float(np.mean(wall_ms)), 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{wl.name}: {n_ctx} contexts of [L={g.L},K/V,Hkv={g.Hkv},N={g.N},D={g.D}] fp16, "
                               f"chunk {g.T}, mixed 8/4/2 bits; a step swaps in {n_sel} of {g.n_chunks} chunks",
                   "pool_bytes": int(sum(int(o[-1]) for o in ctx_off)), "selected_fp16_bytes": sel_fp16,
                   "step": "context draw + LCTRU lock/touch + subset + Load (kv_load_chunks: gather list on the host, carried in the kernel arguments)"},
        "switch_ms": {"mean": round(float(np.mean(wall_ms)), 4), "p50": round(pctl(wall_ms, 50), 4),
                      "p99": round(pctl(wall_ms, 99), 4), "host_part_mean": round(float(np.mean(host_ms)), 4)},
        "swapin_kernel_ms": {"mean": round(float(np.mean(k_ms)), 4), "p50": round(pctl(k_ms, 50), 4),
                             "p99": round(pctl(k_ms, 99), 4)},
        "fault_ms": {"p50": round(pctl(fault_wall[8:], 50), 4), "p99": round(pctl(fault_wall[8:], 99), 4),
                     "max": round(max(fault_wall[8:]), 4), "samples": len(fault_wall) - 8,
                     "note": "kv_load_chunks of one chunk (8 MiB of fp16 cache), call to completion"},
        "load_from_pinned_host": from_host,
        "lctru": {"entries": len(eviction_order), "order_ms": round(order_ms, 3)},
        "pool_build_s": round(t_build, 2),
        "roofline": {"kernel": "swapin_batch_kernel", "bound": "hbm", "achieved": round(gbps, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(gbps / HBM_PEAK_GBPS, 4),
                     "achieved_median": round(gbps_med, 1), "frac_median": round(gbps_med / HBM_PEAK_GBPS, 4),
                     "traffic": None, "ms_back_to_back": round(b2b, 4),
                     "frac_back_to_back": round(float(np.mean(b2b_bytes)) / b2b / 1e6 / HBM_PEAK_GBPS, 4),
                     "note": "HIP events around ONE kv_load_chunks call: the host's gather list and the dispatch are "
                             "inside; back_to_back: eight calls between one event pair, per call"},
    }


def run_stream(wl, args, dev):
    """Long-context cache whose records live in pinned host memory: score, compress, ahead-of-time
    swap-out to the host, then a streaming swap-in (H2D copies on one stream, dequantise kernel
    on another).  Reports the kernel-only rate, the bare copy rate and the overlap."""
    g = wl.geom
    path = Path(wl, dev, host_plan=True, fmt=(3 if args.format == "f16h" else 0))     # the host owns the pinned pool: it needs the offsets
    shape = path.shape
    copy_s, comp_s = torch.cuda.Stream(), torch.cuda.Stream()
    loader = kvs.Loader()
    path.step()                                  # score + compress (+ resident swap-in)
    torch.cuda.synchronize()
    off = kvs.kv_chunk_offsets(shape, path.bits)
    total = int(off[-1])
    pinned = torch.empty(total, dtype=torch.uint8).pin_memory()
    staging = torch.empty(args.stream_buffers * (args.stream_slot_mib << 20), dtype=torch.uint8, device=dev)
    src, dst, sb = kvs.kv_build_gather(shape, off, path.bits, path.all_chunks)
    lists_d = (torch.from_numpy(src.view(np.int64)).to(dev), torch.from_numpy(dst).to(dev), torch.from_numpy(sb).to(dev))
    res = {"aot": [], "stream": [], "zero_copy": [], "h2d": [], "score": [], "compress": [], "swapin_resident": []}
    for it in range(args.warmup + args.steps):
        path.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(0, g.n_chunks, 64):       # the chunks modified by one call, 64 at a time
            j = min(i + 64, g.n_chunks)
            kvs.kv_swapout_aot(path.packed, pinned, int(off[i]), int(off[j]),
                               torch.cuda.current_stream(), copy_s)
        copy_s.synchronize()
        t1 = time.perf_counter()
        loader.swapin_stream(shape, pinned, src, dst, sb, staging, args.stream_buffers, path.kv_out,
                             copy_s, comp_s)
        comp_s.synchronize(); copy_s.synchronize()
        t2 = time.perf_counter()
        with torch.cuda.stream(copy_s):
            staging_all = path.packed[:total]
            staging_all.copy_(pinned, non_blocking=True)      # the bare host->device copy of the pool
        copy_s.synchronize()
        t3 = time.perf_counter()
        # the same Load with no staging: the swap-in kernel reads the pinned pool over the host link
        kvs.kv_swapin_chunks(shape, pinned, *lists_d, path.kv_out, comp_s)
        comp_s.synchronize()
        t4 = time.perf_counter()
        if it >= args.warmup:
            res["aot"].append((t1 - t0) * 1e3); res["stream"].append((t2 - t1) * 1e3); res["h2d"].append((t3 - t2) * 1e3)
            res["zero_copy"].append((t4 - t3) * 1e3)
            for k, v in path.kernel_ms().items():
                res[{"swapin": "swapin_resident"}.get(k, k)].append(v)
    mean = {k: float(np.mean(v)) for k, v in res.items() if v}
    cache_bytes = g.elements * 2
    gbps = (cache_bytes + total) / mean["swapin_resident"] / 1e6
    # one-shot profiling of the IO delay at discrete sizes (Sec. 3.3 i) and a plan (Eq. 4) for
    # loading the whole context when recomputing a chunk would cost --re-us-per-chunk
    sizes, times = [], []
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for mib in (1, 4, 16, 64, 256, 1024):
        nbytes = min(mib << 20, total)
        with torch.cuda.stream(copy_s):
            for rep in range(3):
                ev0.record()
                path.packed[:nbytes].copy_(pinned[:nbytes], non_blocking=True)
                ev1.record()
                copy_s.synchronize()
        sizes.append(float(nbytes)); times.append(ev0.elapsed_time(ev1) * 1e-3)
    io_per_byte, io_fixed = kvs.kv_fit_line(sizes, times)
    rec = [kvs.kv_record_bytes(shape, b) for b in (8, 4, 2)]
    missing = [int((path.bits == b).sum()) for b in (8, 4, 2)]
    model = (args.re_us_per_chunk * 1e-6, 0.0, max(io_per_byte, 0.0), max(io_fixed, 0.0))
    recompute, delay = kvs.kv_plan_pipeline(model, missing, rec)
    return {
        "metric": "KV GB/s (fp16-equiv) compress + swap-in, % of HBM peak; ms per 4K-ctx switch",
        "value": round(cache_bytes / mean["stream"] / 1e6, 2), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(mean["stream"], 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{wl.name}: [L={g.L},K/V,Hkv={g.Hkv},N={g.N},D={g.D}] fp16, chunk {g.T}, "
                               f"group {g.G}, R={path.R}; records in pinned host memory"
                               + (", record parameters in binary16" if shape.format == 3 else ""),
                   "cache_bytes": cache_bytes, "packed_bytes": total,
                   "step": f"streaming swap-in from pinned host memory ({args.stream_buffers} staging slots of "
                           f"{args.stream_slot_mib} MiB); value includes the host link"},
        "ms": {k: round(v, 4) for k, v in mean.items()},
        "zero_copy": {"step": "kv_swapin_chunks reading the pinned pool itself (no staging buffer, no copy engine)",
                      "ms": round(mean["zero_copy"], 4), "fp16_equiv_gbps": round(cache_bytes / mean["zero_copy"] / 1e6, 2),
                      "link_gbps": round(total / mean["zero_copy"] / 1e6, 2)},
        "h2d_gbps": round(total / mean["h2d"] / 1e6, 2),
        "d2h_aot_gbps": round(total / mean["aot"] / 1e6, 2),
        "overlap_efficiency": round(max(mean["h2d"], mean["swapin_resident"]) / mean["stream"], 4),
        "io_model": {"seconds_per_byte": io_per_byte, "fixed_seconds": io_fixed,
                     "gbps": round(1e-9 / io_per_byte, 2), "points": len(sizes)},
        "plan_example": {"assumed_recompute_us_per_chunk": args.re_us_per_chunk, "missing_8_4_2": missing,
                         "recompute_8_4_2": list(recompute), "planned_delay_ms": round(delay * 1e3, 3)},
        "roofline": {"kernel": "swapin_kernel", "bound": "hbm", "achieved": round(gbps, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(gbps / HBM_PEAK_GBPS, 4),
                     "traffic": None},
    }


def run_chunk_sweep(wl, args, dev):
    """Compress and swap-in rates against the chunk size (the paper's chunk-size study, Sec. 5.4,
    looks at IO efficiency against redundant swapping; here: how the kernels take smaller or
    larger units).  Widths are seeded uniform draws; the cache is the workload's."""
    g0 = wl.geom
    kv = synth.make_kv(g0, wl.seed, dev, wl.outlier_channels, wl.outlier_scale)
    out = torch.empty_like(kv)
    rows = []
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    for T in (4, 8, 16, 32, 64, 128, 256):
        if g0.N % T or (T * g0.D) % 512 or (T * g0.D // g0.G) % 4:
            continue
        shape = kvs.Shape(g0.L, g0.Hkv, g0.Hq, g0.D, g0.N, T, g0.G)
        bits = synth.draw_bits_uniform(shape.n_chunks, wl.seed).numpy()
        off = kvs.kv_chunk_offsets(shape, bits)
        src, dst, sb = kvs.kv_build_gather(shape, off, bits, np.arange(shape.n_chunks, dtype=np.int32))
        packed = torch.empty(int(off[-1]), dtype=torch.uint8, device=dev)
        d = [torch.from_numpy(a).to(dev) for a in (bits, off.view(np.int64), src.view(np.int64), dst, sb)]
        tc, ts = [], []
        for it in range(args.warmup + args.steps):
            ev[0].record()
            kvs.kv_compress_chunks(shape, kv, d[0], d[1], packed)
            ev[1].record()
            kvs.kv_swapin_chunks(shape, packed, d[2], d[3], d[4], out)
            ev[2].record()
            torch.cuda.synchronize()
            if it >= args.warmup:
                tc.append(ev[0].elapsed_time(ev[1])); ts.append(ev[1].elapsed_time(ev[2]))
        moved = g0.elements * 2 + int(off[-1])
        rows.append({"chunk_tokens": T, "n_chunks": shape.n_chunks, "packed_bytes": int(off[-1]),
                     "compress_ms": round(float(np.mean(tc)), 4), "swapin_ms": round(float(np.mean(ts)), 4),
                     "compress_gbps": round(moved / float(np.mean(tc)) / 1e6, 1),
                     "swapin_gbps": round(moved / float(np.mean(ts)) / 1e6, 1)})
        del packed
    return {"sweep": "chunk_tokens", "workload": wl.name, "unit": "GB/s of algorithmic bytes", "rows": rows}


def run_i8(wl, args, dev):
    """The paper's own quantiser setting on the workload's geometry: an int8 cache, widths
    8/4/2 by terciles of seeded scores, channel-wise parameters per slab.  A step is compress
    + swap-in of the whole cache (scoring reads fp16 keys and is not part of this variant)."""
    g = wl.geom
    half = args.format == "i8h"
    shape = kvs.Shape(g.L, g.Hkv, g.Hq, g.D, g.N, g.T, g.G,
                      kvs.KV_FMT_I8_CHANNELS_H if half else kvs.KV_FMT_I8_CHANNELS)
    kv = synth.make_kv_i8(g, wl.seed, dev)
    out = torch.empty_like(kv)
    bits = kvs.kv_bits_from_scores(synth.draw_scores(g.n_chunks, wl.seed).numpy(), 1, 1, 3)
    off = kvs.kv_chunk_offsets(shape, bits)
    src, dst, sb = kvs.kv_build_gather(shape, off, bits, np.arange(g.n_chunks, dtype=np.int32))
    packed = torch.empty(int(off[-1]), dtype=torch.uint8, device=dev)
    d = [torch.from_numpy(a).to(dev) for a in (bits, off.view(np.int64), src.view(np.int64), dst, sb)]
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    tc, ts = [], []
    t0 = None
    for it in range(args.warmup + args.steps):
        if it == args.warmup:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
        ev[0].record()
        kvs.kv_compress_chunks(shape, kv, d[0], d[1], packed)
        ev[1].record()
        kvs.kv_swapin_chunks(shape, packed, d[2], d[3], d[4], out)
        ev[2].record()
        torch.cuda.synchronize()
        if it >= args.warmup:
            tc.append(ev[0].elapsed_time(ev[1])); ts.append(ev[1].elapsed_time(ev[2]))
    ms_per_step = (time.perf_counter() - t0) / args.steps * 1e3
    cache_bytes = g.elements
    moved = cache_bytes + int(off[-1])
    kernels = {}
    for name, v in (("compress", tc), ("swapin", ts)):
        ms = float(np.mean(v))
        kernels[name] = {"ms": round(ms, 4), "ms_min": round(float(np.min(v)), 4), "algorithmic_bytes": moved,
                         "hbm_gbps": round(moved / ms / 1e6, 1), "hbm_frac": round(moved / ms / 1e6 / HBM_PEAK_GBPS, 4)}
    dom = max(kernels, key=lambda k: kernels[k]["ms"])
    return {
        "metric": "KV GB/s (fp16-equiv) compress + swap-in, % of HBM peak; ms per 4K-ctx switch",
        "value": round(cache_bytes / ms_per_step / 1e6, 2), "unit": "GB/s (int8 cache bytes)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "i8", "data": "synthetic",
        "config": {"workload": f"{wl.name}, int8 channel-wise format ({'binary16' if half else 'fp32'} parameters): [L={g.L},K/V,Hkv={g.Hkv},N={g.N},D={g.D}] int8, "
                               f"chunk {g.T}, widths 8/4/2 by terciles of seeded scores",
                   "cache_bytes": cache_bytes, "packed_bytes": int(off[-1]), "step": "compress + swap-in"},
        "kernels": kernels,
        "roofline": {"kernel": f"{dom}_i8_kernel", "bound": "hbm", "achieved": kernels[dom]["hbm_gbps"],
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": kernels[dom]["hbm_frac"], "traffic": None},
    }


def run_recompute(wl, args, dev):
    """Recompute of interleaved chunks (Sec. 3.3) on the workload's geometry with a Llama-2-7B-sized
    block and seeded random weights: one layer over x of the context's chunks (seeded interleaved
    subsets), timed per x; the line T_re(x) fitted through the points (Sec. 3.3 i) and, with a
    measured host-to-device line, a plan for loading the whole context (Eq. 4)."""
    g = wl.geom
    d_model, d_ff = g.Hq * g.D, args.d_ff
    shape = kvs.Shape(1, g.Hkv, g.Hq, g.D, g.N, g.T, g.G)          # one layer's planes are enough
    dims = kvs.LayerDims(d_model, d_ff)
    w = synth.make_layer_weights(d_model, g.Hq, g.Hkv, g.D, d_ff, wl.seed, dev)
    kv = synth.make_kv(synth.Geometry(1, g.Hkv, g.Hq, g.D, g.N, g.T, g.G), wl.seed, dev)
    if args.own_gemm:
        os.environ["KVSWITCH_OWN_GEMM"] = "1"        # read when the handle is created
    rc = kvs.Recompute()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    points = []
    per = g.Hq // g.Hkv
    for x in [c for c in (8, 16, 32, 64, 102, 154, 256) if c <= g.n_chunks]:
        idx = synth.draw_subset(g.n_chunks, x, wl.seed, draw=1000 + x)
        idx_dev = idx.to(dev)
        M = x * g.T
        x_in = synth.make_hidden(M, d_model, wl.seed, dev)
        x_out = torch.empty_like(x_in)
        ws = torch.empty(kvs.kv_recompute_workspace_bytes(shape, dims, x), dtype=torch.uint8, device=dev)
        improved = 0 if args.no_tune else rc.tune(shape, dims, w, x, ws)
        ms = []
        for it in range(args.warmup + args.steps):
            ev0.record()
            rc.layer(shape, dims, w, 0, idx_dev, x_in, kv, x_out, ws)
            ev1.record()
            torch.cuda.synchronize()
            if it >= args.warmup:
                ms.append(ev0.elapsed_time(ev1))
        pos = (idx.numpy()[:, None].astype(np.int64) * g.T + np.arange(g.T)[None, :]).reshape(-1)
        gemm_flop = 2.0 * M * (d_model * (g.Hq + 2 * g.Hkv) * g.D + g.Hq * g.D * d_model + 3 * d_model * d_ff)
        attn_flop = 4.0 * float((pos + 1).sum()) * g.D * g.Hq
        t = float(np.mean(ms))
        points.append({"chunks": x, "tokens": M, "ms": round(t, 4), "ms_min": round(float(np.min(ms)), 4),
                       "gemm_gflop": round(gemm_flop / 1e9, 1), "attention_gflop": round(attn_flop / 1e9, 1),
                       "tflops": round((gemm_flop + attn_flop) / t / 1e9, 1),
                       "projections": "gemm_f16_kernel" if M <= kvs.KV_RECOMPUTE_OWN_GEMM_ROWS or args.own_gemm else "rocBLAS",
                       "gemm_shapes_retuned": improved})
        del ws, x_in, x_out
    rc.close()
    slope, icpt = kvs.kv_fit_line([float(p["chunks"]) for p in points], [p["ms"] * 1e-3 for p in points])
    # IO line: pinned host -> device copies of a few sizes (as in the streaming workload)
    pinned = torch.empty(256 << 20, dtype=torch.uint8).pin_memory()
    stage = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
    sizes, times = [], []
    for mib in (1, 4, 16, 64, 256):
        for rep in range(3):
            ev0.record()
            stage[:mib << 20].copy_(pinned[:mib << 20], non_blocking=True)
            ev1.record()
            torch.cuda.synchronize()
        sizes.append(float(mib << 20)); times.append(ev0.elapsed_time(ev1) * 1e-3)
    io_per_byte, io_fixed = kvs.kv_fit_line(sizes, times)
    full = kvs.Shape(g.L, g.Hkv, g.Hq, g.D, g.N, g.T, g.G)
    rec = [kvs.kv_record_bytes(full, b) for b in (8, 4, 2)]
    bits = kvs.kv_bits_from_scores(synth.draw_scores(g.n_chunks, wl.seed).numpy(), 1, 1, 3)
    missing = [int((bits == b).sum()) for b in (8, 4, 2)]
    # a recomputed chunk passes through all L layers; the fitted per-layer line is scaled by L
    model = (max(slope, 0.0) * g.L, max(icpt, 0.0) * g.L, max(io_per_byte, 0.0), max(io_fixed, 0.0))
    recompute, delay = kvs.kv_plan_pipeline(model, missing, rec)
    io_only = model[2] * sum(m * r for m, r in zip(missing, rec)) + model[3]
    big = points[-1]
    return {
        "metric": "recompute of interleaved chunks, one layer (Sec. 3.3): ms per layer against recomputed chunks",
        "value": big["tflops"], "unit": "TFLOP/s (GEMMs + attention, largest point)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": big["ms"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16 (f32 accumulate)",
        "data": "synthetic",
        "config": {"workload": f"{wl.name} geometry, Llama-2-7B-sized block: d_model {d_model}, {g.Hq} heads of {g.D} "
                               f"({g.Hkv} kv heads), d_ff {d_ff}, cache of {g.N} tokens, chunk {g.T}; seeded weights",
                   "step": "kv_recompute_layer over x interleaved chunks"},
        "points": points,
        "recompute_model": {"seconds_per_chunk_per_layer": slope, "fixed_seconds_per_layer": icpt},
        "io_model": {"seconds_per_byte": io_per_byte, "fixed_seconds": io_fixed, "gbps": round(1e-9 / io_per_byte, 2)},
        "plan": {"missing_8_4_2": missing, "record_bytes_8_4_2": rec, "layers": g.L,
                 "recompute_8_4_2": list(recompute), "planned_delay_ms": round(delay * 1e3, 3),
                 "io_only_delay_ms": round(io_only * 1e3, 3)},
        "roofline": {"kernel": "kv_recompute_layer (" + big["projections"] + " projections + recompute_attention_kernel)", "bound": "mfma",
                     "achieved": big["tflops"], "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(big["tflops"] / MFMA_F16_PEAK_TFLOPS, 4), "traffic": None},
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama2-7b-4k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--format", choices=("f16", "f16h", "i8", "i8h"), default="f16",
                    help="f16h: the fp16 group format with binary16 parameters (the whole step, smaller records); "
                         "i8 / i8h: the int8 channel-wise record format with fp32 / binary16 parameters on the "
                         "workload's geometry (compress + swap-in)")
    ap.add_argument("--sweep-chunk-tokens", action="store_true",
                    help="instead of the benchmark: compress / swap-in rates for chunk sizes 4..256")
    ap.add_argument("--recompute", action="store_true",
                    help="instead of the benchmark: one-layer recompute of interleaved chunks (Sec. 3.3) on the "
                         "workload's geometry, T_re fit and an Eq. 4 plan")
    ap.add_argument("--d-ff", type=int, default=11008, help="--recompute: feed-forward width")
    ap.add_argument("--contexts", type=int, default=0, help="pool workload: number of contexts (default: all)")
    ap.add_argument("--stream-buffers", type=int, default=4)
    ap.add_argument("--stream-slot-mib", type=int, default=64)
    ap.add_argument("--re-us-per-chunk", type=float, default=50.0,
                    help="streaming workload: assumed recompute cost per chunk for the Eq. 4 plan example")
    ap.add_argument("--pipeline", action="store_true",
                    help="instead of the benchmark: a context Load from pinned host memory with the first x chunks "
                         "recomputed meanwhile (Sec. 3.3 pipeline), measured for several x")
    ap.add_argument("--ratio", default=None, metavar="NUM/DEN",
                    help="device-planned step: widths by the thresholds of Eq. 2-3 for this global compression ratio "
                         "(kv_plan_optimise_dev) instead of the workload's fixed fractions")
    ap.add_argument("--own-gemm", action="store_true",
                    help="--recompute: every projection on the library's own GEMM kernel (default: rocBLAS above 512 rows)")
    ap.add_argument("--no-tune", action="store_true",
                    help="--recompute: keep the GEMM library's own choice of kernels (default: kv_recompute_tune first)")
    ap.add_argument("--graph", action="store_true",
                    help="additionally time the step replayed from a HIP graph (device-planned or fixed-width workloads)")
    ap.add_argument("--host-plan", action="store_true",
                    help="widths, offsets and gather list on the host between scoring and compression "
                         "(default: on the device, no host round trip)")
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
    if args.sweep_chunk_tokens:
        print(json.dumps(run_chunk_sweep(wl, args, dev)))
        return
    if args.format in ("i8", "i8h"):
        print(json.dumps(run_i8(wl, args, dev)))
        return
    if args.pipeline:
        print(json.dumps(run_pipeline(wl, args, dev)))
        return
    if args.recompute:
        print(json.dumps(run_recompute(wl, args, dev)))
        return
    if wl.n_contexts > 1:
        print(json.dumps(run_pool(wl, args, dev)))
        return
    if wl.name == "llama3-8b-32k" and not args.calibrate_copy:
        print(json.dumps(run_stream(wl, args, dev)))
        return
    ratio = None
    if args.ratio:
        num, den = (int(v) for v in args.ratio.split("/"))
        ratio = (num, den)
    path = Path(wl, dev, host_plan=args.host_plan, fmt=(3 if args.format == "f16h" else 0), ratio=ratio)
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
    # Untimed: the shader clock of an idle GPU needs some tens of milliseconds of load to come up, and the
    # compress kernel, whose VALU work is close to its memory time, is some 25 % slower until it has (its
    # time over the steps of a cold start: 0.57, 0.55, 0.55, ... 0.43 ms from the twentieth step on).  So
    # steps are run for 100 ms before the W warm-up steps, which are enqueued back to back like the timed ones.
    n_ramp, t_ramp = 0, time.perf_counter()
    while (time.perf_counter() - t_ramp) < 0.1:
        for _ in range(8):
            path.step()
        torch.cuda.synchronize()
        n_ramp += 8
    path.reserve_event_sets(args.steps)
    for _ in range(args.warmup):
        path.step()
    clocks = clock_state()          # read while the warm-up steps are running: the clock under this load
    # the K timed steps are enqueued back to back (the host-plan route synchronises inside each
    # step to read the densities); the per-kernel events are read after the timed region
    torch.cuda.synchronize()
    first = path.step_no
    t0 = time.perf_counter()
    for _ in range(args.steps):
        path.step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3
    sums = {}
    for i in range(args.steps):
        for k, v in path.kernel_ms(first + i).items():
            sums.setdefault(k, []).append(v)

    # The same K steps once more without the per-kernel events (five records per step, some 3.5 us of stream
    # time each): what the sequence takes when nothing observes it.  Reported beside `value`, never as it.
    bare_ms = None
    if path.device_plan:
        for _ in range(2):
            path.step(record_events=False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            path.step(record_events=False)
        torch.cuda.synchronize()
        bare_ms = (time.perf_counter() - t0) / args.steps * 1e3

    path.fetch_plan()
    cache_bytes = g.elements * 2
    alg = {"compress": cache_bytes + path.packed_bytes, "swapin": cache_bytes + path.packed_bytes}
    if path.R:
        alg["score"] = (g.L * g.Hkv * g.N * g.D * 2 + g.L * g.Hq * path.R * g.D * 2 +
                        g.L * g.Hq * g.n_chunks * 4)
    kernels = {}
    plan_ms = sums.pop("plan", None)
    for k, v in sums.items():
        ms, med = float(np.mean(v)), float(np.median(v))
        gbps = alg[k] / ms / 1e6
        kernels[k] = {"ms": round(ms, 4), "ms_median": round(med, 4),
                      "ms_min": round(float(np.min(v)), 4), "algorithmic_bytes": alg[k], "hbm_gbps": round(gbps, 1),
                      "hbm_frac": round(gbps / HBM_PEAK_GBPS, 4),
                      "hbm_gbps_median": round(alg[k] / med / 1e6, 1),
                      "hbm_frac_median": round(alg[k] / med / 1e6 / HBM_PEAK_GBPS, 4),
                      "fp16_equiv_gbps": round(cache_bytes / ms / 1e6, 1)}
    if path.n_sets > 1 and not path.R:
        # A launch of tens of microseconds: an event pair around ONE launch also holds its dispatch.  The same
        # kernel over the rotating buffer sets, enqueued back to back between one event pair, per launch:
        bits_d, off_d, src_d, dst_d, sb_d = path.fixed_lists
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for k, call in (("compress", lambda i: kvs.kv_compress_chunks(path.shape, path.kv_sets[i], bits_d, off_d,
                                                                      path.packed_sets[i])),
                        ("swapin", lambda i: kvs.kv_swapin_chunks(path.shape, path.packed_sets[i], src_d, dst_d, sb_d,
                                                                  path.out_sets[i]))):
            per = []
            for rep in range(12):
                e0.record()
                for i in range(path.n_sets):
                    call(i)
                e1.record()
                torch.cuda.synchronize()
                per.append(e0.elapsed_time(e1) / path.n_sets)
            b2b = float(np.median(per[2:]))
            kernels[k]["ms_back_to_back"] = round(b2b, 4)
            kernels[k]["hbm_frac_back_to_back"] = round(alg[k] / b2b / 1e6 / HBM_PEAK_GBPS, 4)
    if path.R:
        flops = 2.0 * path.R * g.N * g.D * g.L * g.Hq
        kernels["score"]["mfma_tflops"] = round(flops / kernels["score"]["ms"] / 1e9, 2)
        kernels["score"]["mfma_frac"] = round(kernels["score"]["mfma_tflops"] / MFMA_F16_PEAK_TFLOPS, 4)
    # a head with one block of query rows and >= 256 (layer, head) pairs is scored by score_head_kernel
    one_block = g.Hq == g.Hkv and path.R <= 32 and g.L * g.Hkv >= 256
    names = {"compress": "compress_kernel", "swapin": "swapin_kernel",
             "score": "score_head_kernel" if one_block else "score_tiles_kernel"}
    dom = max(kernels, key=lambda k: kernels[k]["ms"])
    # achieved / frac: algorithmic bytes over the MEAN launch duration (what a kernel trace's average must
    # agree with); the median of the same launches is given beside it
    roofline = {"kernel": names[dom], "bound": "hbm", "achieved": kernels[dom]["hbm_gbps"],
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": kernels[dom]["hbm_frac"],
                "achieved_median": kernels[dom]["hbm_gbps_median"], "frac_median": kernels[dom]["hbm_frac_median"],
                "traffic": read_traffic(wl.name, names[dom])}

    out = {
        "metric": "KV GB/s (fp16-equiv) compress + swap-in, % of HBM peak; ms per 4K-ctx switch",
        "value": round(cache_bytes / ms_per_step / 1e6, 2),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "dtype_note": "fp16 cache and MFMA operands; softmax, accumulation and the quantiser's "
                                      "arithmetic in f32",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: [L={g.L},K/V,Hkv={g.Hkv},N={g.N},D={g.D}] fp16, "
                               f"chunk {g.T}, group {g.G}, R={path.R}, widths "
                               + (f"by Eq. 2-3 for ratio {args.ratio}" if path.ratio and path.device_plan else wl.bits_rule)
                               + (", record parameters in binary16" if path.shape.format == 3 else ""),
                   "cache_bytes": cache_bytes, "packed_bytes": path.packed_bytes,
                   "step": ("score + widths/offsets/gather list (device) + compress + swap-in, one stream, no "
                            "host round trip" if path.device_plan else
                            "score + bits/offsets (host) + compress + gather list (host) + swap-in")},
        "ms_per_4k_ctx_switch": kernels["swapin"]["ms"],
        "compress_pct_hbm_peak": round(100 * kernels["compress"]["hbm_frac"], 2),
        "swapin_pct_hbm_peak": round(100 * kernels["swapin"]["hbm_frac"], 2),
        "kernels": kernels,
        "roofline": roofline,
    }
    if plan_ms is not None:
        out["plan_ms"] = round(float(np.mean(plan_ms)), 4)
    out["clocks_before_timed_region"] = clocks
    out["untimed_ramp_steps"] = n_ramp
    if bare_ms is not None:
        out["without_kernel_events"] = {
            "ms_per_step": round(bare_ms, 4), "value": round(cache_bytes / bare_ms / 1e6, 2), "unit": "GB/s",
            "note": "the same K steps again, right behind the timed region, with no event records between the kernels"}
    if args.graph and path.device_plan:
        out["hip_graph"] = {"ms_per_step": round(graph_ms_per_step(path, args), 4),
                            "note": "the same step captured once per buffer set and replayed; no events inside"}
    elif args.graph and not path.R:
        out["hip_graph"] = {"ms_per_step": round(graph_ms_per_step(path, args), 4),
                            "note": "compress + swap-in captured once per buffer set and replayed (fixed widths: "
                                    "the lists are built and uploaded once, not per step); no events inside"}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(path)
    print(json.dumps(out))


if __name__ == "__main__":
    main()

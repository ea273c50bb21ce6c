"""GPU tests of kv_plan_chunks_dev: widths from densities (Sec. 3.2, Eq. 2 with fixed
thresholds), record offsets and the whole-cache gather list computed on the device must
equal the oracle's host bookkeeping bit for bit, and the library's own host functions."""
import numpy as np
import pytest
import torch

from oracle import hostlogic
import paper_2403_11805_amd as kvs
from paper_2403_11805_amd import synth

from gpu_util import DEV, both_shapes, gpu_compress, gpu_swapin

pytestmark = pytest.mark.gpu


def plan_on_device(ks, density, fr):
    n = ks.n_chunks
    d = torch.from_numpy(np.asarray(density, dtype=np.float32)).to(DEV)
    bits = torch.full((n,), 0xEE, dtype=torch.uint8, device=DEV)
    off = torch.full((n + 2,), -1, dtype=torch.int64, device=DEV)
    dst = torch.full((n,), -1, dtype=torch.int32, device=DEV)
    kvs.kv_plan_chunks_dev(ks, d, *fr, bits, off[:n + 1], dst)
    torch.cuda.synchronize()
    assert int(off[n + 1]) == -1, "offsets written past n_chunks + 1 entries"
    return bits.cpu().numpy(), off[:n + 1].cpu().numpy().view(np.uint64), dst.cpu().numpy()


def expect(os_, density, fr):
    bits = hostlogic.bits_from_scores(density, *fr)
    off = hostlogic.chunk_offsets(os_, bits)
    src, dst, sb = hostlogic.build_gather(os_, off, bits, list(range(len(bits))))
    return bits, off, np.asarray(src, dtype=np.uint64), np.asarray(dst, dtype=np.int32), np.asarray(sb, dtype=np.uint8)


def densities(kind, n, seed):
    rng = np.random.default_rng(seed)
    if kind == "uniform":
        return rng.random(n, dtype=np.float32)
    if kind == "ties":                       # few distinct values: the index order decides
        return rng.integers(0, 4, n).astype(np.float32) / 4
    if kind == "constant":
        return np.full(n, 0.25, dtype=np.float32)
    if kind == "ascending":
        return np.arange(n, dtype=np.float32) / n
    if kind == "signed_zero":                # -0 and +0 are equal densities
        return np.where(rng.random(n) < 0.5, np.float32(-0.0), np.float32(0.0)).astype(np.float32)
    raise ValueError(kind)


FRACTIONS = [(1, 1, 3), (1, 2, 4), (0, 0, 1), (1, 0, 1), (0, 1, 1), (2, 3, 7)]


@pytest.mark.parametrize("n_chunks", [1, 2, 7, 255, 256, 257, 1000, 1024, 2049])
@pytest.mark.parametrize("kind", ["uniform", "ties", "constant", "ascending", "signed_zero"])
def test_plan_equals_oracle(n_chunks, kind):
    T = 16
    for fmt in (0, 1, 2, 3):
        ks, os_ = both_shapes((1, 1, 1, 64, n_chunks * T, T, 64), fmt)
        for k, fr in enumerate(FRACTIONS):
            d = densities(kind, n_chunks, seed=n_chunks * 31 + k)
            bits, off, dst = plan_on_device(ks, d, fr)
            e_bits, e_off, e_src, e_dst, e_sb = expect(os_, d, fr)
            assert np.array_equal(bits, e_bits), (fmt, fr)
            assert np.array_equal(off, e_off), (fmt, fr)
            assert np.array_equal(off[:-1], e_src) and np.array_equal(bits, e_sb)
            assert np.array_equal(dst, e_dst)
            # and the library's host functions
            assert np.array_equal(bits, kvs.kv_bits_from_scores(d, *fr))
            assert np.array_equal(off, kvs.kv_chunk_offsets(ks, bits))


def test_many_chunks_with_ties():
    """The largest supported count: 65536 chunks (tiles of the ranking loop, 64 chunks per
    thread of the offset scan), heavy ties."""
    n, T = 65536, 8
    ks, os_ = both_shapes((1, 1, 1, 64, n * T, T, 64))
    d = densities("ties", n, seed=5)
    bits, off, dst = plan_on_device(ks, d, (1, 1, 3))
    assert np.array_equal(bits, kvs.kv_bits_from_scores(d, 1, 1, 3))     # host library == oracle: CPU tests
    assert np.array_equal(off, kvs.kv_chunk_offsets(ks, bits))
    assert np.array_equal(dst, np.arange(n, dtype=np.int32) * T)
    sample = np.random.default_rng(1).choice(n, 64, replace=False)
    order = sorted(range(n), key=lambda i: (-float(d[i]), i))
    rank = np.empty(n, dtype=np.int64)
    rank[order] = np.arange(n)
    k8, k84 = n // 3, 2 * n // 3
    for i in sample:
        assert bits[i] == (8 if rank[i] < k8 else 4 if rank[i] < k84 else 2)


def test_switch_without_host_round_trip():
    """Score -> plan -> compress -> swap-in enqueued back to back on one stream: the pool and
    the recovered cache equal those of the path that plans on the host from the same scores."""
    g = synth.Geometry(2, 2, 4, 128, 2048, 16, 64)
    ks, os_ = both_shapes(g)
    kv = synth.make_kv(g, 3).to(DEV)
    q = synth.make_q(g, 3, 32).to(DEV)
    n = ks.n_chunks
    ws = torch.empty(kvs.kv_score_workspace_bytes(ks, 32), dtype=torch.uint8, device=DEV)
    cm = torch.empty((g.L, g.Hq, n), dtype=torch.float32, device=DEV)
    dens = torch.empty(n, dtype=torch.float32, device=DEV)
    bits_d = torch.empty(n, dtype=torch.uint8, device=DEV)
    off_d = torch.empty(n + 1, dtype=torch.int64, device=DEV)
    dst_d = torch.empty(n, dtype=torch.int32, device=DEV)
    packed = torch.zeros(kvs.kv_record_bytes(ks, 8) * n, dtype=torch.uint8, device=DEV)
    out = torch.zeros_like(kv)
    kvs.kv_score_chunks(ks, q, kv, kvs.KV_NORM_VISIBLE, ws, cm, dens)
    kvs.kv_plan_chunks_dev(ks, dens, 1, 1, 3, bits_d, off_d, dst_d)
    kvs.kv_compress_chunks(ks, kv, bits_d, off_d, packed)
    kvs.kv_swapin_chunks(ks, packed, off_d[:n], dst_d, bits_d, out)
    torch.cuda.synchronize()
    bits = hostlogic.bits_from_scores(dens.cpu().numpy(), 1, 1, 3)
    assert np.array_equal(bits_d.cpu().numpy(), bits)
    ref_packed, off = gpu_compress(ks, kv, bits)
    total = int(off[-1])
    assert int(off_d[n]) == total
    assert torch.equal(packed[:total], ref_packed[:total])
    ref_out = gpu_swapin(ks, ref_packed, off, bits, np.arange(n, dtype=np.int32), torch.zeros_like(kv))
    assert torch.equal(out.view(torch.int16), ref_out.view(torch.int16))


def test_switch_replayed_from_a_hip_graph():
    """The device path allocates nothing, clears nothing and never synchronises, so a whole
    switch (score, plan, compress, swap-in) can be captured once and replayed.  Every replay,
    with the inputs changed and eager work in between, must equal the eager result."""
    g = synth.Geometry(2, 2, 4, 128, 1024, 16, 64)
    ks, _ = both_shapes(g)
    n = ks.n_chunks
    kv = synth.make_kv(g, 5).to(DEV)
    q = synth.make_q(g, 5, 32).to(DEV)
    ws = torch.empty(kvs.kv_score_workspace_bytes(ks, 32), dtype=torch.uint8, device=DEV)
    cm = torch.empty((g.L, g.Hq, n), dtype=torch.float32, device=DEV)
    dens = torch.empty(n, dtype=torch.float32, device=DEV)
    bits_d = torch.empty(n, dtype=torch.uint8, device=DEV)
    off_d = torch.empty(n + 1, dtype=torch.int64, device=DEV)
    dst_d = torch.empty(n, dtype=torch.int32, device=DEV)
    packed = torch.zeros(kvs.kv_record_bytes(ks, 8) * n, dtype=torch.uint8, device=DEV)
    out = torch.zeros_like(kv)

    def switch():
        kvs.kv_score_chunks(ks, q, kv, kvs.KV_NORM_VISIBLE, ws, cm, dens)
        kvs.kv_plan_chunks_dev(ks, dens, 1, 1, 3, bits_d, off_d, dst_d)
        kvs.kv_compress_chunks(ks, kv, bits_d, off_d, packed)
        kvs.kv_swapin_chunks(ks, packed, off_d[:n], dst_d, bits_d, out)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        switch()                                    # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        switch()
    for rep in range(4):
        kv.copy_(synth.make_kv(g, 50 + rep).to(DEV))        # new cache and queries for this replay
        q.copy_(synth.make_q(g, 50 + rep, 32).to(DEV))
        for t in (dens, bits_d, off_d, dst_d, packed, out):
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (dens, bits_d, off_d, dst_d, packed, out)]
        for t in (dens, bits_d, off_d, dst_d, packed, out):
            t.zero_()
        switch()                                    # the same switch, eagerly
        torch.cuda.synchronize()
        for a, b, name in zip(got, (dens, bits_d, off_d, dst_d, packed, out),
                              ("density", "bits", "offsets", "dst_tok", "pool", "cache")):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), f"replay {rep}: {name} differs"
        assert int(off_d[n]) > 0 and bool(out.any())

"""CPU tests of libkvswitch's host side: it loads, exports every declared
symbol, rejects bad arguments without touching a GPU, and its bookkeeping
(offsets, bit-widths, gather lists, LCTRU) is identical to the oracle's."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2403_11805_amd as kvs
from paper_2403_11805_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def shapes(i):
    g = synth.WORKLOADS[i].geom
    return kvs.Shape(g.L, g.Hkv, g.Hq, g.D, g.N, g.T, g.G), oracle.Shape(*g)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "kvswitch.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(kv_[a-z0-9_]+)\s*\(", header))
    assert {"kv_score_chunks", "kv_score_chunks_valid", "kv_compress_chunks", "kv_swapin_chunks", "kv_swapin_pinned",
            "kv_swapout_aot", "kv_lctru_evict", "kv_build_gather"} <= declared
    handle = ctypes.CDLL(binding.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(handle, name), f"{name} declared in kvswitch.h but not exported"
    assert declared == set(binding._SIGNATURES), "binding and header disagree on the entry points"


@pytest.mark.parametrize("cfg", range(5))
def test_record_bytes_and_offsets_match_oracle(cfg):
    ks, os_ = shapes(cfg)
    for b in (16, 8, 4, 2):
        assert kvs.kv_record_bytes(ks, b) == oracle.record_bytes(os_, b)
    bits = synth.draw_bits_uniform(ks.n_chunks, cfg, widths=(16, 8, 4, 2)).numpy()
    assert np.array_equal(kvs.kv_chunk_offsets(ks, bits), oracle.chunk_offsets(os_, bits))


def test_int8_channel_format_sizes_offsets_and_validation():
    """Formats 1 and 2 (int8 cache, channel-wise parameters in fp32 / binary16): record sizes and
    offsets equal the oracle's, widths are {8,4,2,1}, and shapes one wavefront cannot hold are refused."""
    for (D, T, fmt) in ((64, 16, 1), (128, 16, 1), (128, 32, 2), (256, 4, 1), (1024, 1, 2), (1024, 4, 1),
                        (64, 16, 2), (128, 16, 2)):
        ks = kvs.Shape(3, 2, 2, D, 8 * T, T, 64, fmt)
        os_ = oracle.Shape(3, 2, 2, D, 8 * T, T, 64, fmt)
        assert fmt in (binding.KV_FMT_I8_CHANNELS, binding.KV_FMT_I8_CHANNELS_H)
        for b in (8, 4, 2, 1):
            assert kvs.kv_record_bytes(ks, b) == oracle.record_bytes(os_, b)
        bits = np.array([8, 4, 2, 1, 1, 2, 4, 8], dtype=np.uint8)
        off = kvs.kv_chunk_offsets(ks, bits)
        assert np.array_equal(off, oracle.chunk_offsets(os_, bits))
        got = kvs.kv_build_gather(ks, off, bits, [1, 3, 6])
        want = oracle.build_gather(os_, off, bits, [1, 3, 6])
        assert all(np.array_equal(g, w) for g, w in zip(got, want))
    good = kvs.Shape(2, 2, 2, 128, 64, 16, 64, binding.KV_FMT_I8_CHANNELS)
    assert kvs.kv_record_bytes(good, 2) == 8 * (16 * 128 // 4 + 8 * 128)
    assert kvs.kv_record_bytes(good._replace(format=2), 2) == 8 * (16 * 128 // 4 + 4 * 128)
    assert kvs.kv_record_bytes(good._replace(format=2), 8) == 8 * 16 * 128
    with pytest.raises(kvs.KvError):
        kvs.kv_record_bytes(good, 16)
    with pytest.raises(kvs.KvError) as e:
        kvs.kv_chunk_offsets(good, np.array([8, 4, 16, 2], dtype=np.uint8))
    assert e.value.code == binding.KV_EBITS
    for bad in (good._replace(head_dim=96), good._replace(head_dim=32, chunk_tokens=32),
                good._replace(chunk_tokens=64), good._replace(chunk_tokens=4, n_tokens=64),
                good._replace(format=4), good._replace(format=-1)):
        with pytest.raises(kvs.KvError) as e:
            kvs.kv_chunk_offsets(bad, np.full(max(bad.n_chunks, 1), 4, dtype=np.uint8))
        assert e.value.code == binding.KV_ESHAPE
    with pytest.raises(kvs.KvError):      # scoring reads fp16 keys
        kvs.kv_score_workspace_bytes(good, 8)


def test_fp16_group_format_with_binary16_parameters_sizes_and_offsets():
    """Format 3: format 0 with 2 x 2 bytes of parameters per group instead of 2 x 4; same widths, same
    shape rules; sizes and offsets equal the oracle's and a hand count."""
    for (D, T, G) in ((64, 16, 64), (128, 16, 64), (128, 32, 128), (256, 16, 64), (1024, 4, 512)):
        ks = kvs.Shape(3, 2, 2, D, 8 * T, T, G, binding.KV_FMT_F16_GROUPS_H)
        os_ = oracle.Shape(3, 2, 2, D, 8 * T, T, G, 3)
        for b in (16, 8, 4, 2):
            assert kvs.kv_record_bytes(ks, b) == oracle.record_bytes(os_, b)
        bits = np.array([8, 4, 2, 16, 16, 2, 4, 8], dtype=np.uint8)
        off = kvs.kv_chunk_offsets(ks, bits)
        assert np.array_equal(off, oracle.chunk_offsets(os_, bits))
        assert all(int(o) % 16 == 0 for o in off)
        got = kvs.kv_build_gather(ks, off, bits, [1, 3, 6])
        want = oracle.build_gather(os_, off, bits, [1, 3, 6])
        assert all(np.array_equal(g, w) for g, w in zip(got, want))
    h = kvs.Shape(32, 32, 32, 128, 4096, 16, 64, binding.KV_FMT_F16_GROUPS_H)
    assert kvs.kv_record_bytes(h, 8) == 2048 * 16 * (128 + 8) == 4456448         # 4718592 with fp32 parameters
    assert kvs.kv_record_bytes(h, 2) == 2048 * 16 * (32 + 8)
    assert kvs.kv_record_bytes(h, 16) == 2048 * 16 * 256
    with pytest.raises(kvs.KvError) as e:
        kvs.kv_chunk_offsets(h, np.full(256, 1, dtype=np.uint8))
    assert e.value.code == binding.KV_EBITS
    with pytest.raises(kvs.KvError) as e:
        kvs.kv_chunk_offsets(h._replace(group=96), np.full(256, 8, dtype=np.uint8))
    assert e.value.code == binding.KV_ESHAPE
    assert kvs.kv_score_workspace_bytes(h, 32) == kvs.kv_score_workspace_bytes(h._replace(format=0), 32) > 0


def test_recompute_entry_points_validate_on_the_host():
    """Workspace size by hand; bad geometry and NULL handles are refused before any launch."""
    shape = kvs.Shape(32, 32, 32, 128, 4096, 16, 64)
    dims = binding.LayerDims(4096, 11008)
    M, dq = 8 * 16, 32 * 128

    def up(n):
        return (n + 255) // 256 * 256
    def plain(M):
        return (up(M * 4096 * 2) + 3 * up(M * dq * 4) + 2 * up(M * dq * 2) + up(M * 4096 * 2) + 2 * up(M * 11008 * 2))
    # 128 rows give 32 attention workgroups: the key range is shared by 8 workgroups each, whose
    # partial outputs (binary32) and (maximum, denominator) pairs are part of the workspace
    # and the projections of so few rows divide K among several workgroups per tile (some 256 workgroups per
    # launch up to 128 rows); the widest set of binary32 partial tiles is that of gate | up in one launch:
    # 172 column tiles want 2 shares of K, [128][2 * 11008] each (q | k | v: 3 shares of [128][3 * 4096];
    # o and down: 8 shares of [128][4096])
    want = plain(M) + 8 * M * dq * 4 + 8 * M * 32 * 8 + 2 * M * 2 * 11008 * 4
    assert kvs.kv_recompute_workspace_bytes(shape, dims, 8) == want
    assert kvs.kv_recompute_workspace_bytes(shape, dims, 256) == plain(4096)       # enough workgroups: no split
    for bad_shape, bad_dims, n in ((shape._replace(head_dim=256, group=64), dims, 8),
                                   (shape._replace(format=1), dims, 8),
                                   (shape, dims._replace(d_model=4100), 8),
                                   (shape, dims._replace(d_ff=0), 8),
                                   (shape, dims._replace(rope_base=1.0), 8),
                                   (shape, dims, 0), (shape, dims, 257)):
        with pytest.raises(kvs.KvError):
            kvs.kv_recompute_workspace_bytes(bad_shape, bad_dims, n)
    s, d = shape.c(), dims.c()
    w = binding.kv_layer_weights_t()
    assert binding.lib().kv_recompute_layer(None, ctypes.byref(s), ctypes.byref(d), ctypes.byref(w), 0, None, 8,
                                            None, None, None, None, 0, None) == binding.KV_EINVAL
    improved = ctypes.c_int32(7)
    assert binding.lib().kv_recompute_tune(None, ctypes.byref(s), ctypes.byref(d), ctypes.byref(w), 8, None, 0,
                                           None, ctypes.byref(improved)) == binding.KV_EINVAL
    assert improved.value == 0
    binding.lib().kv_recompute_destroy(None)      # a no-op


def test_bits_from_scores_matches_oracle_including_ties():
    rng = np.random.default_rng(0)
    for n in (1, 2, 3, 7, 256, 1024):
        for (a, b, c) in ((1, 1, 3), (1, 2, 4), (0, 1, 2), (1, 0, 1), (0, 0, 5)):
            d = rng.random(n).astype(np.float32)
            d[rng.integers(0, n, size=n // 3)] = 0.5        # plenty of ties
            assert np.array_equal(kvs.kv_bits_from_scores(d, a, b, c),
                                  oracle.bits_from_scores(d, a, b, c))


def test_gather_matches_oracle_and_rejects_bad_lists():
    ks, os_ = shapes(3)
    bits = synth.draw_bits_uniform(ks.n_chunks, 3).numpy()
    off = kvs.kv_chunk_offsets(ks, bits)
    for draw in range(4):
        idx = synth.draw_subset(ks.n_chunks, 51, 3, draw).numpy()
        got = kvs.kv_build_gather(ks, off, bits, idx)
        want = oracle.build_gather(os_, off, bits, idx)
        for g, w in zip(got, want):
            assert g.dtype == w.dtype and np.array_equal(g, w)
    for bad in ([3, 3], [5, 2], [-1], [ks.n_chunks]):
        with pytest.raises(kvs.KvError) as e:
            kvs.kv_build_gather(ks, off, bits, bad)
        assert e.value.code == binding.KV_EINDEX
    assert all(len(a) == 0 for a in kvs.kv_build_gather(ks, off, bits, []))


def test_shape_and_bits_validation():
    good = kvs.Shape(2, 4, 4, 64, 512, 16, 64)
    bad_shapes = [good._replace(n_tokens=500), good._replace(group=32), good._replace(group=96),
                  good._replace(head_dim=96), good._replace(n_q_heads=6), good._replace(n_layers=0),
                  good._replace(chunk_tokens=4, n_tokens=512)]
    for s in bad_shapes:
        with pytest.raises(kvs.KvError) as e:
            kvs.kv_chunk_offsets(s, np.full(max(s.n_chunks, 1), 8, dtype=np.uint8))
        assert e.value.code == binding.KV_ESHAPE and kvs.kv_last_error()
    with pytest.raises(kvs.KvError) as e:
        kvs.kv_chunk_offsets(good, np.full(good.n_chunks, 3, dtype=np.uint8))
    assert e.value.code == binding.KV_EBITS
    with pytest.raises(kvs.KvError):
        kvs.kv_record_bytes(good, 5)
    with pytest.raises(kvs.KvError):
        kvs.kv_bits_from_scores(np.zeros(4, dtype=np.float32), 2, 2, 3)
    # scoring has extra requirements, checked on the host
    with pytest.raises(kvs.KvError):
        kvs.kv_score_workspace_bytes(good._replace(n_tokens=48), 8)
    with pytest.raises(kvs.KvError):
        kvs.kv_score_workspace_bytes(good, 0)
    assert kvs.kv_score_workspace_bytes(good, 8) % 256 == 0


def test_device_entry_points_validate_before_touching_the_gpu():
    """NULL pointers and bad sizes are refused on the host (nothing is launched)."""
    L = binding.lib()
    s = kvs.Shape(2, 4, 4, 64, 512, 16, 64).c()
    assert L.kv_compress_chunks(ctypes.byref(s), None, None, None, None, None) == binding.KV_EINVAL
    assert L.kv_swapin_chunks(ctypes.byref(s), None, None, None, None, 3, None, None) == binding.KV_EINVAL
    assert L.kv_swapin_chunks(ctypes.byref(s), None, None, None, None, 0, None, None) == binding.KV_OK
    assert L.kv_swapin_chunks(ctypes.byref(s), None, None, None, None, 33, None, None) == binding.KV_EINVAL
    # layer-wise Load: the layer range is checked on the host; empty ranges and empty lists are no-ops
    assert L.kv_swapin_layers(ctypes.byref(s), None, None, None, None, 3, -1, 1, None, None) == binding.KV_EINVAL
    assert L.kv_swapin_layers(ctypes.byref(s), None, None, None, None, 3, 2, 1, None, None) == binding.KV_EINVAL
    assert L.kv_swapin_layers(ctypes.byref(s), None, None, None, None, 3, 0, 3, None, None) == binding.KV_EINVAL
    assert L.kv_swapin_layers(ctypes.byref(s), None, None, None, None, 3, 1, 1, None, None) == binding.KV_OK
    assert L.kv_swapin_layers(ctypes.byref(s), None, None, None, None, 0, 0, 2, None, None) == binding.KV_OK
    assert L.kv_swapin_layers(ctypes.byref(s), None, None, None, None, 3, 0, 2, None, None) == binding.KV_EINVAL   # NULL pointers
    assert L.kv_score_chunks(ctypes.byref(s), None, 8, None, 0, None, 0, None, None, None) == binding.KV_EINVAL
    # padded contexts: the number of valid tokens lies between the query rows and the cache size
    for nv in (7, s.n_tokens + 1, -1):
        assert L.kv_score_chunks_valid(ctypes.byref(s), None, 8, None, nv, 0, None, 0, None, None, None) == binding.KV_EINVAL
        assert "n_valid" in binding.kv_last_error()
    assert L.kv_swapout_aot(None, None, 0, 0, None, None) == binding.KV_EINVAL
    bad = kvs.Shape(2, 4, 4, 64, 500, 16, 64).c()
    assert L.kv_compress_chunks(ctypes.byref(bad), None, None, None, None, None) == binding.KV_ESHAPE
    assert L.kv_plan_chunks_dev(ctypes.byref(s), None, 1, 1, 3, None, None, None, None) == binding.KV_EINVAL
    assert L.kv_plan_chunks_dev(ctypes.byref(bad), None, 1, 1, 3, None, None, None, None) == binding.KV_ESHAPE
    fake = ctypes.c_void_p(4096)         # never dereferenced: the fractions are refused first
    for fr in ((1, 1, 0), (-1, 1, 3), (1, -1, 3), (2, 2, 3)):
        assert L.kv_plan_chunks_dev(ctypes.byref(s), fake, *fr, fake, fake, fake, None) == binding.KV_EINVAL
    assert L.kv_compress_selected(ctypes.byref(s), None, None, None, None, 3, None, None) == binding.KV_EINVAL
    assert L.kv_compress_selected(ctypes.byref(s), None, None, None, None, 0, None, None) == binding.KV_OK
    assert L.kv_compress_selected(ctypes.byref(s), None, None, None, None, 33, None, None) == binding.KV_EINVAL
    assert L.kv_load_chunks(ctypes.byref(s), None, None, None, None, 3, None, None) == binding.KV_EINVAL
    assert L.kv_load_chunks(ctypes.byref(s), None, None, None, None, 0, None, None) == binding.KV_OK
    off = (ctypes.c_uint64 * 33)(*range(0, 33 * 4096, 4096))
    b8 = (ctypes.c_uint8 * 32)(*([8] * 32))
    for idx in ((2, 1), (5, 5), (0, 32)):                 # refused on the host: nothing is launched
        ci = (ctypes.c_int32 * 2)(*idx)
        assert L.kv_load_chunks(ctypes.byref(s), fake, off, b8, ci, 2, fake, None) == binding.KV_EINDEX
    many = kvs.Shape(1, 1, 1, 64, 8 * 65537, 8, 64).c()
    assert L.kv_plan_chunks_dev(ctypes.byref(many), fake, 1, 1, 3, fake, fake, fake, None) == binding.KV_ESHAPE


def replay(ops):
    """Apply the same operation sequence to the library queue and to the oracle model."""
    q, m = kvs.Lctru(), oracle.LctruModel()
    for op in ops:
        kind = op[0]
        if kind == "insert":
            q.insert(*op[1:]); m.insert(*op[1:])
        elif kind == "touch":
            q.touch_ctx(*op[1:]); m.touch_ctx(*op[1:])
        elif kind == "lock":
            q.lock(op[1]); m.lock(op[1])
        elif kind == "unlock":
            q.unlock(op[1]); m.unlock(op[1])
        elif kind == "remove":
            q.remove_ctx(op[1]); m.remove_ctx(op[1])
        elif kind == "evict":
            assert q.evict(op[1]) == m.evict(op[1])
        assert q.order() == m.order()
        assert q.size() == m.size()
    q.close()


def test_lctru_matches_oracle_on_random_sequences():
    rng = np.random.default_rng(7)
    for trial in range(20):
        ops, now, live = [], 0, set()
        for _ in range(300):
            now += int(rng.integers(0, 3))          # repeated timestamps exercise the tie rule
            k = rng.random()
            ctx = int(rng.integers(0, 6))
            if k < 0.45:
                chunk = int(rng.integers(0, 40))
                if (ctx, chunk) not in live:
                    live.add((ctx, chunk))
                    b = int(rng.choice([16, 8, 4, 2]))
                    ops.append(("insert", ctx, chunk, b, 100 * b + int(rng.integers(0, 5)), now))
            elif k < 0.6:
                ops.append(("touch", ctx, now))
            elif k < 0.7:
                ops.append(("lock", ctx))
            elif k < 0.8:
                ops.append(("unlock", ctx))
            elif k < 0.85:
                ops.append(("remove", ctx))
                live = {x for x in live if x[0] != ctx}
            else:
                ops.append(("evict", int(rng.integers(0, 6000))))
                live = None
                break
        replay(ops)


def test_lctru_pool_workload_order():
    """64 contexts x 128 chunks (the multi-app pool): order equals the oracle's sort."""
    ks, _ = shapes(3)
    q, m = kvs.Lctru(), oracle.LctruModel()
    rng = np.random.default_rng(3)
    for ctx in range(64):
        bits = synth.draw_bits_uniform(ks.n_chunks, 3, context=ctx).numpy()
        for chunk in range(ks.n_chunks):
            args = (ctx, chunk, int(bits[chunk]), kvs.kv_record_bytes(ks, int(bits[chunk])), ctx)
            q.insert(*args); m.insert(*args)
    for step, ctx in enumerate(rng.integers(0, 64, size=50)):
        q.touch_ctx(int(ctx), 100 + step); m.touch_ctx(int(ctx), 100 + step)
    q.lock(5); m.lock(5)
    assert q.order() == m.order()
    need = 3 * 2 ** 30
    assert q.evict(need) == m.evict(need)
    assert q.size() == m.size()
    with pytest.raises(kvs.KvError):
        q.insert(0, 0, 8, 1, 1) if (0, 0) in m.entries else q.insert(1, 1, 3, 1, 1)
    q.close()


def test_bits_optimise_matches_oracle():
    rng = np.random.default_rng(11)
    for n in (0, 1, 2, 3, 7, 12, 100, 256, 1024):
        for (num, den) in ((1, 2), (1, 4), (1, 1), (3, 8), (5, 8), (2, 3)):
            for printed in (0, 1):
                d = (rng.random(n) ** 3).astype(np.float32)
                if n > 4:
                    d[rng.integers(0, n, size=n // 4)] = 0.25
                got_bits, got_counts = kvs.kv_bits_optimise(d, num, den, printed)
                want_bits, want_counts = oracle.bits_optimise(d, num, den, bool(printed))
                assert got_counts == want_counts, (n, num, den, printed)
                assert np.array_equal(got_bits, want_bits)
    # ratios just below 1 ask for a bit budget no split has: counts stay valid, the mean stays below
    for n, num, den in ((10, 99, 100), (3, 11, 12), (1, 7, 8), (64, 255, 256)):
        d = rng.random(n).astype(np.float32)
        for printed in (0, 1):
            got_bits, (k8, k4, k2) = kvs.kv_bits_optimise(d, num, den, printed)
            assert min(k8, k4, k2) >= 0 and k8 + k4 + k2 == n
            assert (k8 + k4 / 2 + k2 / 4) / n <= num / den
            want_bits, want_counts = oracle.bits_optimise(d, num, den, bool(printed))
            assert (k8, k4, k2) == want_counts and np.array_equal(got_bits, want_bits)
    for bad in ((1, 5), (3, 2), (0, 1), (1, 0)):
        with pytest.raises(kvs.KvError):
            kvs.kv_bits_optimise(np.ones(4, dtype=np.float32), bad[0], bad[1], 0)
    for poison in (np.nan, np.inf, -np.inf):
        d = np.ones(5, dtype=np.float32)
        d[3] = poison
        with pytest.raises(kvs.KvError):
            kvs.kv_bits_optimise(d, 1, 2, 0)
        with pytest.raises(kvs.KvError):
            kvs.kv_bits_from_scores(d, 1, 1, 3)
    with pytest.raises(kvs.KvError):
        kvs.kv_bits_optimise(np.ones(4, dtype=np.float32), 1, 2, 7)


def test_fit_line_and_plan_pipeline_match_oracle():
    rng = np.random.default_rng(21)
    for _ in range(20):
        n = int(rng.integers(2, 9))
        x = np.cumsum(rng.random(n) + 0.1)
        t = rng.random(n)
        assert kvs.kv_fit_line(x, t) == pytest.approx(oracle.fit_line(x, t), rel=1e-12)
    with pytest.raises(kvs.KvError):
        kvs.kv_fit_line([1.0, 1.0], [2.0, 3.0])
    with pytest.raises(kvs.KvError):
        kvs.kv_fit_line([1.0], [2.0])
    ks, _ = shapes(2)
    rec = [kvs.kv_record_bytes(ks, b) for b in (8, 4, 2)]
    for _ in range(200):
        missing = [int(v) for v in rng.integers(0, 90, size=3)]
        model = (float(rng.random() * 2e-3), float(rng.random() * 1e-3) * (rng.random() < 0.7),
                 float(rng.random() / 2e10), float(rng.random() * 1e-3) * (rng.random() < 0.7))
        got = kvs.kv_plan_pipeline(model, missing, rec)
        want = oracle.plan_pipeline(model, missing, rec)
        assert got[0] == want[0] and got[1] == want[1], (model, missing)
    for bad_model in ((-1.0, 0, 0, 0), (0, 0, float("nan"), 0)):
        with pytest.raises(kvs.KvError):
            kvs.kv_plan_pipeline(bad_model, [1, 1, 1], rec)
    with pytest.raises(kvs.KvError):
        kvs.kv_plan_pipeline((1, 0, 1, 0), [1, 1, 1], rec[::-1])
    with pytest.raises(kvs.KvError):
        kvs.kv_plan_pipeline((1, 0, 1, 0), [1, -1, 1], rec)


def test_scoring_refuses_contexts_beyond_its_run_table():
    """The combine kernel keeps one bit per run of tiles and head: 8192 runs, i.e. 2 097 152 tokens with
    one block of query rows per kv head (runs of 8 tiles), 16 777 216 with several (runs of 64)."""
    one = kvs.Shape(1, 1, 1, 64, 2097152, 1024, 64)
    assert kvs.kv_score_workspace_bytes(one, 32) > 0
    with pytest.raises(kvs.KvError):
        kvs.kv_score_workspace_bytes(one._replace(n_tokens=2097152 + 1024), 32)
    grouped = kvs.Shape(1, 1, 4, 64, 4194304, 1024, 64)
    assert kvs.kv_score_workspace_bytes(grouped, 32) > 0


def test_pipeline_split_matches_oracle():
    rng = np.random.default_rng(31)
    for fmt in (0, 3):
        for _ in range(40):
            n = int(rng.integers(1, 60))
            ks = kvs.Shape(1, 1, 1, 64, n * 16, 16, 64, fmt)
            bits = rng.choice([16, 8, 4, 2], n, p=[0.1, 0.3, 0.3, 0.3]).astype(np.uint8)
            missing = np.flatnonzero(rng.random(n) < 0.7).astype(np.int32)
            have = [int((bits[missing] == b).sum()) for b in (8, 4, 2)]
            plan = [int(rng.integers(0, h + 1)) for h in have]
            re, io = kvs.kv_pipeline_split(ks, bits, missing, plan)
            want_re, want_io = oracle.pipeline_split(missing, bits, plan)
            assert np.array_equal(re, want_re) and np.array_equal(io, want_io)
    ks = kvs.Shape(1, 1, 1, 64, 64, 16, 64)
    bits = np.array([8, 8, 4, 2], dtype=np.uint8)
    for missing, plan in (([0, 1], [3, 0, 0]), ([0, 1], [0, 1, 0]), ([0, 1], [-1, 0, 0])):
        with pytest.raises(kvs.KvError) as e:
            kvs.kv_pipeline_split(ks, bits, missing, plan)
        assert e.value.code == kvs.KV_EINVAL
    for missing in ([1, 0], [0, 0], [4], [-1]):
        with pytest.raises(kvs.KvError) as e:
            kvs.kv_pipeline_split(ks, bits, missing, [0, 0, 0])
        assert e.value.code == kvs.KV_EINDEX
    with pytest.raises(kvs.KvError) as e:
        kvs.kv_pipeline_split(ks, np.array([8, 3, 4, 2], dtype=np.uint8), [1], [0, 0, 0])
    assert e.value.code == kvs.KV_EBITS

"""GPU parity for the int8, channel-wise record format (the paper's own quantiser setting,
Sec. 3.2 "Compressing chunks" and Sec. 4): kv_compress_chunks / kv_swapin_chunks /
kv_swapin_pinned with shape.format = KV_FMT_I8_CHANNELS (fp32 parameters) and
KV_FMT_I8_CHANNELS_H (binary16 parameters) against the CPU oracle.

Bar: every record byte (codes, scales, minima, pass-through bytes) and every
dequantised int8 value bit-exact."""
import numpy as np
import pytest
import torch

import oracle
import paper_2403_11805_amd as kvs
from paper_2403_11805_amd import synth

from gpu_util import DEV, both_shapes, chunk_view, gpu_compress, gpu_swapin

pytestmark = pytest.mark.gpu

SENTINEL = 0x55


def check_full(geom, kv_host, bits, select=None, fmts=(1, 2)):
    """Both int8 formats: parameters in fp32 (1) and in binary16 (2)."""
    got = None
    for fmt in fmts:
        got = check_format(geom, kv_host, bits, select, fmt)
    return got


def check_format(geom, kv_host, bits, select, fmt):
    ks, os_ = both_shapes(geom, fmt)
    kv_dev = torch.from_numpy(kv_host).to(DEV)
    packed_dev, off = gpu_compress(ks, kv_dev, bits)
    assert np.array_equal(off, oracle.chunk_offsets(os_, bits))
    want = oracle.compress_chunks_i8(os_, kv_host, bits, off)
    got = packed_dev[:int(off[-1])].cpu().numpy()
    if not np.array_equal(got, want):
        bad = np.flatnonzero(got != want)
        chunk = int(np.searchsorted(off, bad[0], side="right") - 1)
        raise AssertionError(f"{len(bad)} packed bytes differ; first at byte {bad[0]} "
                             f"(chunk {chunk}, bits {bits[chunk]}, record offset {bad[0] - int(off[chunk])})")
    idx = list(range(ks.n_chunks)) if select is None else select
    out_dev = torch.full(ks.kv_dims, SENTINEL, dtype=torch.int8, device=DEV)
    gpu_swapin(ks, packed_dev, off, bits, idx, out_dev)
    ref = np.full(kv_host.shape, SENTINEL, dtype=np.int8)
    oracle.swapin_chunks_i8(os_, want, *oracle.build_gather(os_, off, bits, idx), ref)
    out = out_dev.cpu().numpy()
    assert np.array_equal(out, ref), f"{(out != ref).sum()} dequantised int8 values differ"
    return got


# every head_dim (4..64 pieces per token row) with 1, 2 and 4 pieces per lane
@pytest.mark.parametrize("D,T", [(64, 16), (64, 32), (64, 64), (128, 8), (128, 16), (128, 32),
                                 (256, 4), (256, 8), (256, 16), (512, 2), (512, 4), (512, 8),
                                 (1024, 1), (1024, 2), (1024, 4)])
def test_shapes_and_mixed_widths(D, T):
    g = synth.Geometry(2, 3, 3, D, 5 * T, T, 64)       # 5 chunks: ragged last workgroup
    kv = synth.make_kv_i8(g, 17, "cpu").numpy()
    bits = np.array([1, 4, 8, 2, 4], dtype=np.uint8)
    check_full(g, kv, bits)
    check_full(g, kv, bits, select=[0, 4])
    check_full(g, kv, np.roll(bits, 2), select=[3])


@pytest.mark.parametrize("b", [4, 2, 1])
def test_adversarial_values(b):
    """Exact ties of the quotient (integer data make them common), constant channels, full
    range -128..127, ranges that are and are not multiples of the level count."""
    g = synth.Geometry(1, 2, 2, 128, 64, 16, 64)
    rng = np.random.default_rng(b)
    levels = (1 << b) - 1
    x = np.zeros((g.L, 2, g.Hkv, g.N, g.D), dtype=np.int64)
    # chunk 0: range 2 * levels: odd offsets are exact half-integers of the quotient
    t = rng.integers(0, 2 * levels + 1, size=(g.L, 2, g.Hkv, 16, g.D))
    t[..., 0, :] = 0
    t[..., 1, :] = 2 * levels
    x[..., 0:16, :] = t - 100
    # chunk 1: full range (scale 255 / levels), every value
    t = rng.integers(-128, 128, size=(g.L, 2, g.Hkv, 16, g.D))
    t[..., 3, :] = -128
    t[..., 7, :] = 127
    x[..., 16:32, :] = t
    # chunk 2: constant channels, two-valued channels, channels at the extremes
    t = np.zeros((g.L, 2, g.Hkv, 16, g.D), dtype=np.int64)
    t[..., :, 0::4] = 7
    t[..., :, 1::4] = rng.integers(0, 2, size=(g.L, 2, g.Hkv, 16, g.D // 4)) * 3 - 128
    t[..., :, 2::4] = 127
    t[..., :, 3::4] = rng.integers(0, 2, size=(g.L, 2, g.Hkv, 16, g.D // 4)) + 126
    x[..., 32:48, :] = t
    # chunk 3: random ranges per channel (most are not multiples of the level count)
    width = rng.integers(1, 200, size=(g.L, 2, g.Hkv, 1, g.D))
    x[..., 48:64, :] = (rng.random((g.L, 2, g.Hkv, 16, g.D)) * width).astype(np.int64) - 90
    assert x.min() >= -128 and x.max() <= 127
    check_full(g, x.astype(np.int8), np.full(g.n_chunks, b, dtype=np.uint8))


@pytest.mark.parametrize("b", [4, 2, 1])
def test_every_range_and_offset(b):
    """The codes of a channel depend only on its range r = max - min and on x - min.  Every
    pair 0 <= x - min <= r <= 255 occurs here (with varying minima), so this comparison
    covers the whole domain of the format's two divisions."""
    T, D = 16, 128
    rng = np.random.default_rng(100 + b)
    cols = []
    for r in range(256):
        inner = list(range(1, r))                      # offsets besides 0 and r
        for i in range(0, max(len(inner), 1), T - 2):
            part = inner[i:i + T - 2]
            col = [0, r] + part + [0] * (T - 2 - len(part))
            rng.shuffle(col)
            lo = int(rng.integers(-128, 128 - r))
            cols.append(np.array(col) + lo)
    n_units = -(-len(cols) // D)
    n_chunks = -(-n_units // 2)
    cols += [np.zeros(T, dtype=np.int64)] * (n_chunks * 2 * D - len(cols))
    x = np.stack(cols, axis=1).reshape(T, n_chunks, 2, D)              # [t][chunk][slab][d]
    kv = np.ascontiguousarray(x.transpose(2, 1, 0, 3)).reshape(1, 2, 1, n_chunks * T, D)
    assert kv.min() >= -128 and kv.max() <= 127
    g = synth.Geometry(1, 1, 1, D, n_chunks * T, T, 64)
    check_full(g, kv.astype(np.int8), np.full(n_chunks, b, dtype=np.uint8))


def test_random_cache_many_channels():
    g = synth.Geometry(4, 4, 4, 128, 512, 16, 64)
    kv = synth.make_kv_i8(g, 5, "cpu").numpy()
    bits = synth.draw_bits_uniform(g.n_chunks, 5, widths=(8, 4, 2, 1)).numpy()
    check_full(g, kv, bits)


@pytest.mark.parametrize("fmt", [1, 2])
def test_llama7b_4k_int8_cache_sampled(fmt):
    """Llama-2-7B-shaped int8 cache (1 GiB) at full size; the oracle recomputes sampled chunks."""
    g = synth.Geometry(32, 32, 32, 128, 4096, 16, 64)
    ks, os_ = both_shapes(g, fmt)
    one = oracle.Shape(os_.L, os_.Hkv, os_.Hq, os_.D, os_.T, os_.T, os_.G, fmt)
    kv_dev = synth.make_kv_i8(g, 2, DEV)
    bits = synth.draw_bits_uniform(g.n_chunks, 2, widths=(8, 4, 2, 1)).numpy()
    packed_dev, off = gpu_compress(ks, kv_dev, bits)
    sel = synth.draw_subset(g.n_chunks, 200, 2).numpy()
    out_dev = torch.full(ks.kv_dims, SENTINEL, dtype=torch.int8, device=DEV)
    gpu_swapin(ks, packed_dev, off, bits, sel, out_dev)
    first = [int(np.flatnonzero(bits == b)[0]) for b in (8, 4, 2, 1)]
    unsel = sorted(set(range(g.n_chunks)) - set(sel.tolist()))
    for i in sorted({0, g.n_chunks - 1, *first, int(sel[0]), int(sel[-1]), unsel[0], unsel[-1]}):
        b = np.array([bits[i]], dtype=np.uint8)
        o1 = oracle.chunk_offsets(one, b)
        want = oracle.compress_chunks_i8(one, chunk_view(kv_dev, g.T, i), b, o1)
        got = packed_dev[int(off[i]):int(off[i + 1])].cpu().numpy()
        assert np.array_equal(got, want), f"record of chunk {i} (bits {bits[i]}) differs"
        got_out = chunk_view(out_dev, g.T, i)
        if i in sel:
            ref = np.zeros(got_out.shape, dtype=np.int8)
            oracle.swapin_chunks_i8(one, want, *oracle.build_gather(one, o1, b, [0]), ref)
            assert np.array_equal(got_out, ref)
        else:
            assert np.all(got_out == SENTINEL), f"unselected chunk {i} was written"
    # property at full size: a dequantised value differs from the original by at most half a
    # step of its channel (+ the final rounding to an integer)
    T, D = g.T, g.D
    for i in (int(sel[1]), int(sel[-2])):
        x = kv_dev[:, :, :, i * T:(i + 1) * T, :].float()
        y = out_dev[:, :, :, i * T:(i + 1) * T, :].float()
        rng_ = x.amax(dim=3, keepdim=True) - x.amin(dim=3, keepdim=True)
        step = rng_ / ((1 << int(bits[i])) - 1) if bits[i] < 8 else torch.zeros_like(rng_)
        assert bool(((y - x).abs() <= step * 0.5 + 0.5 + 1e-3).all())


@pytest.mark.parametrize("fmt", [1, 2])
def test_streaming_from_pinned_host_equals_resident_path(fmt):
    g = synth.Geometry(2, 2, 2, 128, 512, 16, 64)
    ks, os_ = both_shapes(g, fmt)
    kv = synth.make_kv_i8(g, 31, "cpu")
    bits = synth.draw_bits_uniform(g.n_chunks, 31, widths=(8, 4, 2, 1)).numpy()
    packed_dev, off = gpu_compress(ks, kv.to(DEV), bits)
    total = int(off[-1])
    pinned = torch.zeros(total, dtype=torch.uint8).pin_memory()
    copy_s, comp_s = torch.cuda.Stream(), torch.cuda.Stream()
    kvs.kv_swapout_aot(packed_dev, pinned, 0, total, torch.cuda.current_stream(), copy_s)
    copy_s.synchronize()
    idx = synth.draw_subset(g.n_chunks, 13, 31).numpy().tolist()
    src, dst, sb = kvs.kv_build_gather(ks, off, bits, idx)
    staging = torch.empty(3 * 2 * kvs.kv_record_bytes(ks, 8), dtype=torch.uint8, device=DEV)
    out = torch.full(ks.kv_dims, SENTINEL, dtype=torch.int8, device=DEV)
    torch.cuda.synchronize()
    kvs.kv_swapin_pinned(ks, pinned, src, dst, sb, staging, 3, out, copy_s, comp_s)
    comp_s.synchronize()
    copy_s.synchronize()
    ref = np.full(kv.shape, SENTINEL, dtype=np.int8)
    want = oracle.compress_chunks_i8(os_, kv.numpy(), bits, off)
    oracle.swapin_chunks_i8(os_, want, *oracle.build_gather(os_, off, bits, idx), ref)
    assert np.array_equal(out.cpu().numpy(), ref)


def test_more_chunks_than_a_grid_dimension():
    """70 000 chunks of the int8 format (the second grid dimension holds at most 65 535)."""
    g = synth.Geometry(1, 1, 1, 64, 16 * 70000, 16, 64)
    kv = synth.make_kv_i8(g, 22, "cpu").numpy()
    bits = synth.draw_bits_uniform(g.n_chunks, 22, widths=(8, 4, 2, 1)).numpy()
    check_full(g, kv, bits)
    check_full(g, kv, bits, select=[1, 65535, 65536, 69998])

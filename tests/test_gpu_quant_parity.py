"""GPU parity: kv_compress_chunks / kv_swapin_chunks against the CPU oracle.

Bar: packed code bytes, scales, minima and pass-through bytes bit-exact;
dequantised fp16 within 1 fp16 ulp (the tests also report exact equality,
which the kernels are built to reach)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2403_11805_amd as kvs
from paper_2403_11805_amd import synth

from gpu_util import (DEV, both_shapes, chunk_view, gpu_compress, gpu_swapin, half_ulp_distance)

pytestmark = pytest.mark.gpu


def check_full(geom, kv_host, bits, select=None, fmt=0):
    ks, os_ = both_shapes(geom, fmt)
    kv_dev = torch.from_numpy(kv_host).to(DEV)
    packed_dev, off = gpu_compress(ks, kv_dev, bits)
    want = oracle.compress_chunks(os_, kv_host, bits, off)
    got = packed_dev[:int(off[-1])].cpu().numpy()
    if not np.array_equal(got, want):
        bad = np.flatnonzero(got != want)
        chunk = int(np.searchsorted(off, bad[0], side="right") - 1)
        raise AssertionError(f"{len(bad)} packed bytes differ; first at byte {bad[0]} "
                             f"(chunk {chunk}, bits {bits[chunk]}, record offset {bad[0] - int(off[chunk])})")
    idx = list(range(ks.n_chunks)) if select is None else select
    sentinel = 0x7bff
    out_dev = torch.full(ks.kv_dims, sentinel, dtype=torch.int16, device=DEV).view(torch.float16)
    gpu_swapin(ks, packed_dev, off, bits, idx, out_dev)
    out = out_dev.cpu().numpy().view(np.uint16)
    ref = np.full(kv_host.shape, sentinel, dtype=np.uint16)
    oracle.swapin_chunks(os_, want, *oracle.build_gather(os_, off, bits, idx), ref)
    dist = half_ulp_distance(out, ref)
    assert dist.max() <= 1, f"dequantised values differ by up to {dist.max()} fp16 ulp"
    assert np.array_equal(out, ref), f"{(dist > 0).sum()} dequantised values are 1 ulp off"
    return got


@pytest.mark.parametrize("fmt", [0, 3])
def test_tiny_workload_full(fmt):
    wl = synth.WORKLOADS[0]
    kv = synth.make_kv(wl.geom, wl.seed, "cpu", wl.outlier_channels, wl.outlier_scale).numpy()
    bits = synth.draw_bits_uniform(wl.geom.n_chunks, wl.seed).numpy()
    assert wl.geom.n_chunks == 32
    check_full(wl.geom, kv, bits, fmt=fmt)


@pytest.mark.parametrize("geom", [
    (3, 2, 2, 64, 80, 16, 64),      # 5 chunks: a ragged last workgroup
    (1, 3, 3, 128, 96, 32, 128),
    (2, 1, 1, 256, 48, 16, 64),
    (1, 1, 1, 256, 24, 8, 256),
    (1, 2, 2, 512, 16, 4, 512),
    (2, 1, 1, 64, 64, 8, 64),
    (1, 1, 1, 1024, 6, 2, 128),
    (1, 5, 5, 128, 2048, 1024, 64),  # the largest chunk
    (1, 2, 2, 64, 72, 24, 64),       # 3 wavefront tasks per unit (not a power of two), 1 piece per lane
    (2, 1, 1, 64, 144, 48, 64),      # 6 -> 2 pieces per lane, 3 tasks per unit
    (1, 1, 2, 128, 96, 48, 128),     # 12 -> 4 pieces per lane, 3 tasks per unit
    (1, 1, 1, 64, 40, 8, 64),        # one task per unit, 5 chunks: last workgroup partly idle
])
def test_shapes_and_mixed_widths(geom):
    g = synth.Geometry(*geom)
    kv = synth.make_kv(g, 11, "cpu", 2, 10.0).numpy()
    bits = synth.draw_bits_uniform(g.n_chunks, 11, widths=(16, 8, 4, 2)).numpy()
    bits[0] = 2
    if g.n_chunks > 2:
        bits[1], bits[2] = 8, 16
    check_full(g, kv, bits)
    # a subset: untouched tokens must keep the sentinel
    if g.n_chunks >= 3:
        check_full(g, kv, bits, select=[0, g.n_chunks - 1])


@pytest.mark.parametrize("fmt", [0, 3])
@pytest.mark.parametrize("b", [8, 4, 2])
def test_adversarial_values(b, fmt):
    """Exact ties (k + 0.5 on an integer grid), subnormal halves, constant and all-zero
    groups, signed zeros, the largest finite halves."""
    g = synth.Geometry(1, 2, 2, 128, 64, 16, 64)
    rng = np.random.default_rng(b)
    levels = (1 << b) - 1
    x = np.zeros((g.L, 2, g.Hkv, g.N, g.D), dtype=np.float64)
    # tokens 0..15: half-integers on a 0..levels grid (scale exactly 1)
    t = rng.integers(0, 2 * levels + 1, size=(g.L, 2, g.Hkv, 16, g.D)) / 2.0
    t[..., 0::64] = 0
    t[..., 1::64] = levels
    x[..., 0:16, :] = t
    # tokens 16..31: the same pattern scaled by powers of two and shifted (ties survive)
    x[..., 16:32, :] = t * 0.25 - 3.0
    # tokens 32..47: subnormal and tiny values
    x[..., 32:48, :] = rng.integers(-1023, 1024, size=(g.L, 2, g.Hkv, 16, g.D)) * 2.0 ** -24
    # tokens 48..63: constant groups, zeros of both signs, extremes
    x[..., 48:52, :] = 3.25
    x[..., 52:56, :] = -0.0
    x[..., 56:60, :] = np.where(rng.random((g.L, 2, g.Hkv, 4, g.D)) < 0.5, -0.0, 0.0)
    x[..., 60:64, :] = np.where(rng.random((g.L, 2, g.Hkv, 4, g.D)) < 0.5, -65504.0, 65504.0)
    kv = x.astype(np.float16)
    check_full(g, kv, np.full(g.n_chunks, b, dtype=np.uint8), fmt=fmt)


@pytest.mark.parametrize("fmt", [0, 3])
@pytest.mark.parametrize("b", [8, 4, 2])
def test_ranges_of_a_few_binary16_subnormal_steps(b, fmt):
    """Groups whose range is a few steps of the smallest binary16 subnormal: with binary16 parameters the
    stored scale then has one or two significant bits and may fall short of range / levels by tens of
    per cent, so quotients run past the top level and must saturate there (never spill into the
    neighbouring code of a packed byte)."""
    g = synth.Geometry(1, 2, 2, 128, 64, 16, 64)
    rng = np.random.default_rng(70 + b)
    levels = (1 << b) - 1
    x = np.zeros((g.L, 2, g.Hkv, g.N, g.D), dtype=np.float64)
    for t in range(g.N):
        top = int(round(levels * (1.05 + 0.45 * (t % 16) / 15)))      # range / levels between 1.05 and 1.5 steps ...
        steps = 1 + t // 16                                         # ... of 1 to 4 subnormal steps
        k = rng.integers(0, top + 1, size=(g.L, 2, g.Hkv, g.D))
        k[..., 0::64] = 0
        k[..., 1::64] = top
        x[..., t, :] = k * steps * 2.0 ** -24 - (t % 3) * 2.0 ** -20
    check_full(g, x.astype(np.float16), np.full(g.n_chunks, b, dtype=np.uint8), fmt=fmt)


@pytest.mark.parametrize("fmt", [0, 3])
@pytest.mark.parametrize("b", [8, 4, 2])
def test_scale_for_every_binary16_range(b, fmt):
    """The stored scale is (max - min) / levels as a correctly rounded binary32 division.  One group per
    positive finite binary16 value h with range h (minimum 0), and one with range h + h' (minimum -h', h'
    another binary16 value, so that the numerator is a sum that binary32 may have to round): 63 486
    numerators per width, compared bit for bit with the oracle's division like every other record byte."""
    g = synth.Geometry(1, 2, 2, 128, 8192, 16, 64)
    rng = np.random.default_rng(300 + b)
    halves = np.arange(1, 0x7c00, dtype=np.uint16).view(np.float16).astype(np.float64)   # every positive finite value
    n_groups = 2 * g.Hkv * g.N * (g.D // g.G)
    assert n_groups >= 2 * len(halves)
    top = np.resize(halves, n_groups)
    low = np.where(np.arange(n_groups) < len(halves), 0.0, -halves[(np.arange(n_groups) * 7919) % len(halves)])
    x = low[:, None] + rng.random((n_groups, g.G)) * (top - low)[:, None]
    x[:, 0] = low
    x[:, 1] = top
    kv = x.reshape(g.L, 2, g.Hkv, g.N, g.D).astype(np.float16)
    check_full(g, kv, np.full(g.n_chunks, b, dtype=np.uint8), fmt=fmt)


@pytest.mark.parametrize("fmt", [0, 3])
@pytest.mark.parametrize("b", [8, 4, 2])
def test_groups_far_from_zero(b, fmt):
    """Groups whose minimum is thousands of steps away from zero (a range of 1 to 600 units in the last
    place at magnitudes from 1 to 32768, both signs): the quotient (x - min) / scale is then a small
    difference of large terms, the case in which a quantiser that folds the minimum into one
    multiply-add has the least margin, and every value sits on a grid on which exact ties are common."""
    g = synth.Geometry(1, 2, 2, 128, 64, 16, 64)
    rng = np.random.default_rng(170 + b)
    x = np.zeros((g.L, 2, g.Hkv, g.N, g.D), dtype=np.float64)
    for t in range(g.N):
        e = t % 16                                                   # binade 2^e .. 2^(e+1)
        base = (1.0 + rng.integers(0, 1024) / 1024.0) * 2.0 ** e
        ulp = 2.0 ** (e - 10)
        width = int(rng.integers(1, 601))
        j = rng.integers(0, width + 1, size=(g.L, 2, g.Hkv, g.D))
        j[..., 0::64] = 0
        j[..., 1::64] = width
        row = base + j * ulp
        x[..., t, :] = np.minimum(row, 65504.0) * (-1.0 if t % 2 else 1.0)
    check_full(g, x.astype(np.float16), np.full(g.n_chunks, b, dtype=np.uint8), fmt=fmt)


@pytest.mark.parametrize("fmt", [0, 3])
@pytest.mark.parametrize("scale", [1.0, 1e-3, 300.0])
def test_random_magnitudes_all_groups(scale, fmt):
    """Many random groups per width, including ones whose quotients land within a few
    ulps of a half-integer (exercises the exact-division path)."""
    g = synth.Geometry(4, 4, 4, 128, 256, 16, 64)
    kv = (synth.make_kv(g, 5, "cpu", 1, 10.0).float() * scale).to(torch.float16).numpy()
    bits = synth.draw_bits_uniform(g.n_chunks, 5).numpy()
    check_full(g, kv, bits, fmt=fmt)


def test_gemma_shaped_workload_full():
    """Configuration 2 at full size: 72 MiB cache, bit-widths from seeded scores (25/50/25)."""
    wl = synth.WORKLOADS[1]
    ks, os_ = both_shapes(wl.geom)
    kv = synth.make_kv(wl.geom, wl.seed, "cpu", wl.outlier_channels, wl.outlier_scale).numpy()
    scores = synth.draw_scores(wl.geom.n_chunks, wl.seed).numpy()
    bits = kvs.kv_bits_from_scores(scores, 1, 2, 4)
    assert np.array_equal(bits, oracle.bits_from_scores(scores, 1, 2, 4))
    assert [(bits == b).sum() for b in (8, 4, 2)] == [64, 128, 64]
    got = check_full(wl.geom, kv, bits)
    assert len(got) == 25952256


@pytest.mark.parametrize("geom,select_every", [
    ((3, 3, 3, 128, 8192, 16, 64), 1),    # 36 MiB, 18 planes: two strips of eight and a ragged one
    ((5, 1, 1, 64, 32768, 8, 64), 1),     # 40 MiB, 10 planes of small units (64 pieces): wavefronts of 1 KiB
    ((3, 3, 3, 128, 16384, 16, 64), 3),   # a third of the chunks of a 72 MiB cache: a launch just under 32 MiB
])
def test_launch_shapes_of_the_load_kernels(geom, select_every):
    """Caches around the size at which the Load kernels change their launch shape (workgroups of 4
    wavefronts with six to a CU from 32 MiB written, up to 8 wavefronts below, 4 for small units), with
    plane counts that are no multiple of the eight planes a strip holds: records and swapped-in cache
    bit-exact."""
    g = synth.Geometry(*geom)
    kv = synth.make_kv(g, 91, "cpu", 1, 10.0).numpy()
    bits = synth.draw_bits_uniform(g.n_chunks, 91, widths=(16, 8, 4, 2)).numpy()
    check_full(g, kv, bits, select=list(range(0, g.n_chunks, select_every)))


def test_empty_selection_and_all_passthrough():
    g = synth.Geometry(1, 2, 2, 64, 64, 16, 64)
    ks, os_ = both_shapes(g)
    kv = synth.make_kv(g, 2, "cpu", 1, 10.0).numpy()
    bits = np.full(g.n_chunks, 16, dtype=np.uint8)
    got = check_full(g, kv, bits)
    assert len(got) == kv.nbytes
    kv_dev = torch.from_numpy(kv).to(DEV)
    packed_dev, off = gpu_compress(ks, kv_dev, bits)
    out = torch.zeros(ks.kv_dims, dtype=torch.float16, device=DEV)
    gpu_swapin(ks, packed_dev, off, bits, [], out)
    assert not bool(out.any())


def test_determinism():
    g = synth.Geometry(2, 4, 4, 128, 512, 16, 64)
    ks, _ = both_shapes(g)
    kv_dev = synth.make_kv(g, 9, DEV, 1, 10.0)
    bits = synth.draw_bits_uniform(g.n_chunks, 9).numpy()
    a, _ = gpu_compress(ks, kv_dev, bits)
    b, _ = gpu_compress(ks, kv_dev, bits)
    assert torch.equal(a, b)


def test_more_chunks_than_a_grid_dimension():
    """70 000 chunks: the launch grid cannot carry the chunk index in its second dimension
    (limit 65 535), so compression walks the chunks of one slab instead.  Bit-exact records
    and cache for every chunk, and for a subset that starts beyond chunk 65 535."""
    g = synth.Geometry(1, 1, 1, 64, 8 * 70000, 8, 64)
    kv = synth.make_kv(g, 21, "cpu", 1, 10.0).numpy()
    bits = synth.draw_bits_uniform(g.n_chunks, 21, widths=(16, 8, 4, 2)).numpy()
    check_full(g, kv, bits)
    check_full(g, kv, bits, select=[0, 65535, 65536, 69999])


def test_random_valid_geometries():
    """Thirty seeded geometries drawn from everything the shape rules admit (head_dim 64..1024,
    every group size that divides it, chunk sizes that keep a unit a whole number of wavefront
    rows), random widths and a random subset each: records and cache bit for bit."""
    rng = np.random.default_rng(2024)
    done = 0
    while done < 30:
        D = int(rng.choice([64, 128, 192, 256, 384, 512, 1024]))
        G = int(rng.choice([g_ for g_ in (64, 128, 256, 512) if D % g_ == 0]))
        T = int(rng.choice([2, 4, 6, 8, 12, 16, 24, 32, 40, 64]))
        if (T * D) % 512 or (T * D // G) % 4:
            continue
        L, Hkv = int(rng.integers(1, 3)), int(rng.integers(1, 4))
        n_chunks = int(rng.integers(1, 8))
        g = synth.Geometry(L, Hkv, Hkv, D, n_chunks * T, T, G)
        kv = synth.make_kv(g, 100 + done, "cpu", 1, 10.0).numpy()
        bits = rng.choice([16, 8, 4, 2], n_chunks).astype(np.uint8)
        fmt = 3 if done % 3 == 2 else 0          # every third geometry with binary16 parameters
        check_full(g, kv, bits, fmt=fmt)
        sel = sorted(rng.choice(n_chunks, int(rng.integers(1, n_chunks + 1)), replace=False).tolist())
        check_full(g, kv, bits, select=sel, fmt=fmt)
        done += 1

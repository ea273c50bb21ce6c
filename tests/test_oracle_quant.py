"""Pins for the compress / swap-in oracle (Sec. 3.2 "Compressing chunks", Sec. 4
bit-shift packing, Load primitive of Sec. 3.1).  CPU only.

Closed forms, literal bytes, invariants, the rounding-error bound, exhaustive
pack/unpack per byte and the IEEE fp16 conversions against numpy.
"""
import numpy as np
import pytest

import oracle


def shape_small(T=4, D=64, G=64, L=1, Hkv=1, N=None):
    return oracle.Shape(L=L, Hkv=Hkv, Hq=Hkv, D=D, N=N or T, T=T, G=G)


def compress_one(shape, kv, b):
    bits = np.full(shape.n_chunks, b, dtype=np.uint8)
    off = oracle.chunk_offsets(shape, bits)
    return oracle.compress_chunks(shape, kv, bits, off), bits, off


def sections(shape, rec, b):
    """Split one record into (codes [slabs][T][D*b/8], scale [slabs][T][D/G], mn)."""
    n_codes = shape.slabs * shape.T * shape.D * b // 8
    n_meta = shape.slabs * shape.T * (shape.D // shape.G)
    codes = rec[:n_codes].reshape(shape.slabs, shape.T, shape.D * b // 8)
    scale = rec[n_codes:n_codes + 4 * n_meta].view(np.float32).reshape(shape.slabs, shape.T, -1)
    mn = rec[n_codes + 4 * n_meta:n_codes + 8 * n_meta].view(np.float32).reshape(shape.slabs, shape.T, -1)
    assert n_codes + 8 * n_meta == len(rec)
    return codes, scale, mn


def unpack(codes_row, b):
    """Independent decoder of the stated bit order: element d in byte d*b/8, bit (d % (8/b))*b."""
    per = 8 // b
    out = []
    for byte in codes_row:
        for k in range(per):
            out.append((int(byte) >> (k * b)) & ((1 << b) - 1))
    return np.array(out)


# ------------------------------------------------------------------ fp16 conversions

def test_half_to_float_all_bit_patterns():
    allbits = np.arange(65536, dtype=np.uint16)
    ref = allbits.view(np.float16).astype(np.float32)
    got = np.array([oracle.half_to_float(int(b)) for b in allbits], dtype=np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), ref[~nan].view(np.uint32))


def test_float_to_half_round_to_nearest_even():
    rng = np.random.default_rng(0)
    vals = [0.0, -0.0, 1.0, 65504.0, 65519.99, 65520.0, 1e9, -1e9, 2.0 ** -24, 2.0 ** -25,
            2.0 ** -25 * 1.0001, 2.0 ** -14, 2.0 ** -14 - 2.0 ** -25, 1.0 + 2.0 ** -11,
            1.0 + 3 * 2.0 ** -11, 2047.5, 2048.5, 2049.5, 0.1, -0.1, 3.14159]
    vals += list(rng.normal(size=4000) * 10)
    vals += list(rng.normal(size=2000) * 1e-5)
    vals += list(rng.uniform(-70000, 70000, size=2000))
    # exact ties between neighbouring halfs
    h = rng.integers(0, 0x7bff, size=2000).astype(np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    vals += list((lo + hi) / 2)
    vals = np.array(vals, dtype=np.float32)
    with np.errstate(over="ignore"):            # values beyond 65504 round to infinity, as they should
        ref = vals.astype(np.float16).view(np.uint16)
    got = np.array([oracle.float_to_half(float(v)) for v in vals], dtype=np.uint16)
    assert np.array_equal(got, ref)


# ------------------------------------------------------------------ closed forms

@pytest.mark.parametrize("b", [8, 4, 2])
def test_integer_grid_is_coded_exactly(b):
    """A group holding integers between 0 and 2^b-1 (both present): mn=0, scale=1, code=value."""
    rng = np.random.default_rng(b)
    shape = shape_small(T=4, D=128, G=64, L=2, Hkv=2)
    levels = (1 << b) - 1
    x = rng.integers(0, levels + 1, size=(shape.L, 2, shape.Hkv, shape.N, shape.D))
    x[..., 0::64] = 0
    x[..., 1::64] = levels
    kv = x.astype(np.float16)
    packed, bits, off = compress_one(shape, kv, b)
    codes, scale, mn = sections(shape, packed, b)
    assert np.all(scale == 1.0) and np.all(mn == 0.0)
    flat = x.reshape(shape.slabs, shape.T, shape.D)
    for s in range(shape.slabs):
        for t in range(shape.T):
            assert np.array_equal(unpack(codes[s, t], b), flat[s, t])
    # and the round trip is exact
    out = np.full(kv.shape, -1.0, dtype=np.float16)
    src, dst, sb = oracle.build_gather(shape, off, bits, [0])
    oracle.swapin_chunks(shape, packed, src, dst, sb, out)
    assert np.array_equal(out.view(np.uint16), kv.view(np.uint16))


def test_halves_round_to_even():
    """0..255 group at 8 bits has scale 1: k+0.5 rounds to the even neighbour."""
    shape = shape_small(T=1)
    x = np.zeros((1, 2, 1, 1, 64), dtype=np.float16)
    vals = [0.0, 255.0, 0.5, 1.5, 2.5, 3.5, 100.5, 101.5, 254.5, 0.25, 0.75, 1.25]
    x[0, :, 0, 0, :len(vals)] = vals
    packed, _, _ = compress_one(shape, x, 8)
    codes, scale, mn = sections(shape, packed, 8)
    assert scale[0, 0, 0] == 1.0 and mn[0, 0, 0] == 0.0
    assert list(codes[0, 0, :len(vals)]) == [0, 255, 0, 2, 2, 4, 100, 102, 254, 0, 1, 1]


def test_literal_packed_bytes():
    """2-bit codes 0,1,2,3 -> 0xE4; 4-bit codes 1,15 -> 0xF1 (lowest index in the low bits)."""
    shape = shape_small(T=1)
    x = np.zeros((1, 2, 1, 1, 64), dtype=np.float16)
    x[0, :, 0, 0, :4] = [0, 1, 2, 3]
    packed, _, _ = compress_one(shape, x, 2)
    assert packed[0] == 0xE4
    x[:] = 0
    x[0, :, 0, 0, :3] = [1, 15, 0]
    packed, _, _ = compress_one(shape, x, 4)
    assert packed[0] == 0xF1 and packed[1] == 0x00
    x[:] = 0
    x[0, :, 0, 0, :3] = [7, 255, 0]
    packed, _, _ = compress_one(shape, x, 8)
    assert packed[0] == 7 and packed[1] == 255


@pytest.mark.parametrize("b", [8, 4, 2])
def test_pack_unpack_exhaustive_bytes(b):
    """Every byte value appears as a packed byte and decodes to the codes that made it."""
    levels = (1 << b) - 1
    per = 8 // b
    free = 64 - 2                       # last two elements of the group pin min and max
    free_bytes = free // per
    rows = -(-256 // free_bytes)
    shape = shape_small(T=rows)
    x = np.zeros((1, 2, 1, rows, 64))
    x[..., 62] = 0
    x[..., 63] = levels
    want = {}
    for v in range(256):
        t, j = divmod(v, free_bytes)
        for k in range(per):
            x[0, 0, 0, t, j * per + k] = (v >> (k * b)) & levels
        want[(t, j)] = v
    kv = x.astype(np.float16)
    packed, bits, off = compress_one(shape, kv, b)
    codes, scale, mn = sections(shape, packed, b)
    for (t, j), v in want.items():
        assert codes[0, t, j] == v
    out = np.zeros(kv.shape, dtype=np.float16)
    oracle.swapin_chunks(shape, packed, *oracle.build_gather(shape, off, bits, [0]), out)
    assert np.array_equal(out, kv)


# ------------------------------------------------------------------ invariants and bounds

def random_cache(shape, seed, scale=1.0):
    rng = np.random.default_rng(seed)
    x = rng.normal(size=(shape.L, 2, shape.Hkv, shape.N, shape.D)) * scale
    x[..., 5] *= 8.0       # an outlier channel
    return x.astype(np.float16)


@pytest.mark.parametrize("b", [8, 4, 2])
def test_invariants_and_error_bound(b):
    shape = oracle.Shape(L=2, Hkv=2, Hq=2, D=128, N=32, T=16, G=64)
    kv = random_cache(shape, 10 + b)
    packed, bits, off = compress_one(shape, kv, b)
    levels = (1 << b) - 1
    out = np.zeros(kv.shape, dtype=np.float16)
    oracle.swapin_chunks(shape, packed, *oracle.build_gather(shape, off, bits, [0, 1]), out)
    x = kv.astype(np.float64).reshape(shape.slabs, shape.n_chunks, shape.T, shape.D // shape.G, shape.G)
    y = out.astype(np.float64).reshape(x.shape)
    for i in range(shape.n_chunks):
        rec = packed[int(off[i]):int(off[i + 1])]
        codes, scale, mn = sections(shape, rec, b)
        for s in range(shape.slabs):
            for t in range(shape.T):
                c = unpack(codes[s, t], b).reshape(-1, shape.G)
                for j in range(shape.D // shape.G):
                    g = x[s, i, t, j]
                    sc, m = float(scale[s, t, j]), float(mn[s, t, j])
                    # stored metadata are the group's min and (max-min)/levels in fp32
                    assert m == g.min()
                    assert sc == float(np.float32(np.float32(g.max()) - np.float32(g.min())) /
                                       np.float32(levels))
                    # extremes hit the end codes; codes are monotone in the value
                    assert c[j][np.argmin(g)] == 0 and c[j][np.argmax(g)] == levels
                    order = np.argsort(g, kind="stable")
                    assert np.all(np.diff(c[j][order]) >= 0)
                    # reconstruction error <= scale * (1/2 + 2^-14), evaluated in double
                    err = np.abs(m + c[j] * sc - g)
                    assert np.all(err <= sc * (0.5 + 2.0 ** -14))
                    # after the fp16 rounding of the dequantised value: half an fp16 ulp more
                    ulp = np.spacing(np.abs(y[s, i, t, j]).astype(np.float16)).astype(np.float64)
                    assert np.all(np.abs(y[s, i, t, j] - g) <= sc * (0.5 + 2.0 ** -14) + 0.5 * ulp + 1e-12)


@pytest.mark.parametrize("b", [8, 4, 2])
def test_constant_group_and_signed_zero(b):
    """scale 0 -> all codes 0 and an exact round trip; a minimum of -0 is stored as +0."""
    shape = shape_small(T=2, D=128, G=64)
    x = np.zeros((1, 2, 1, 2, 128), dtype=np.float16)
    x[0, 0, 0, 0, :64] = 3.25                    # constant group
    x[0, 0, 0, 0, 64:] = -0.0                    # all negative zero
    x[0, 0, 0, 1, :64] = np.where(np.arange(64) % 2 == 0, -0.0, 1.0)
    packed, bits, off = compress_one(shape, x, b)
    codes, scale, mn = sections(shape, packed, b)
    assert scale[0, 0, 0] == 0.0 and mn[0, 0, 0] == np.float32(3.25)
    assert np.all(codes[0, 0] == 0)
    assert scale[0, 0, 1] == 0.0 and mn[0, 0, 1].view(np.uint32) == 0      # +0, not -0
    assert mn[0, 1, 0].view(np.uint32) == 0
    out = np.ones(x.shape, dtype=np.float16)
    oracle.swapin_chunks(shape, packed, *oracle.build_gather(shape, off, bits, [0]), out)
    assert np.all(out[0, 0, 0, 0, :64] == np.float16(3.25))
    assert np.all(out[0, 0, 0, 0, 64:] == 0)


def test_sixteen_bit_chunks_pass_through():
    shape = oracle.Shape(L=2, Hkv=2, Hq=2, D=64, N=48, T=16, G=64)
    kv = random_cache(shape, 3)
    bits = np.array([16, 4, 16], dtype=np.uint8)
    off = oracle.chunk_offsets(shape, bits)
    packed = oracle.compress_chunks(shape, kv, bits, off)
    rec0 = packed[:int(off[1])].view(np.uint16).reshape(shape.slabs, shape.T, shape.D)
    want0 = kv.view(np.uint16).reshape(shape.slabs, shape.N, shape.D)[:, :16]
    assert np.array_equal(rec0, want0)
    out = np.zeros(kv.shape, dtype=np.float16)
    oracle.swapin_chunks(shape, packed, *oracle.build_gather(shape, off, bits, [0, 2]), out)
    assert np.array_equal(out[..., :16, :].view(np.uint16), kv[..., :16, :].view(np.uint16))
    assert np.array_equal(out[..., 32:, :].view(np.uint16), kv[..., 32:, :].view(np.uint16))
    assert np.all(out[..., 16:32, :] == 0)       # chunk 1 was not selected


def test_swapin_touches_only_selected_tokens():
    shape = oracle.Shape(L=1, Hkv=2, Hq=2, D=64, N=64, T=16, G=64)
    kv = random_cache(shape, 4)
    bits = np.array([8, 4, 2, 8], dtype=np.uint8)
    off = oracle.chunk_offsets(shape, bits)
    packed = oracle.compress_chunks(shape, kv, bits, off)
    sentinel = np.uint16(0x7bff)
    out = np.full(kv.shape, sentinel, dtype=np.uint16)
    oracle.swapin_chunks(shape, packed, *oracle.build_gather(shape, off, bits, [1, 3]), out)
    assert np.all(out[..., 0:16, :] == sentinel) and np.all(out[..., 32:48, :] == sentinel)
    assert not np.any(out[..., 16:32, :] == sentinel)
    full = np.zeros(kv.shape, dtype=np.uint16)
    oracle.swapin_chunks(shape, packed, *oracle.build_gather(shape, off, bits, [0, 1, 2, 3]), full)
    assert np.array_equal(out[..., 16:32, :], full[..., 16:32, :])
    assert np.array_equal(out[..., 48:, :], full[..., 48:, :])


def test_layer_wise_load_is_the_layer_share_of_each_record():
    """Layer-wise Load (Sec. 3.3 pipeline): a record keeps its layers one after the other in every
    section, so layer l of chunk c is slabs [l*2*Hkv, (l+1)*2*Hkv) of the three sections.  Decoded
    here by hand from those pieces (independent bit decoder, numpy float32 arithmetic), it must be
    what swapin_layers puts into layer l, and the other layers must keep their contents."""
    shape = oracle.Shape(L=3, Hkv=2, Hq=2, D=64, N=48, T=16, G=64)
    kv = random_cache(shape, 9)
    bits = np.array([4, 8, 2], dtype=np.uint8)
    off = oracle.chunk_offsets(shape, bits)
    packed = oracle.compress_chunks(shape, kv, bits, off)
    lists = oracle.build_gather(shape, off, bits, [0, 2])
    sentinel = np.uint16(0x7bff)
    for l in range(shape.L):
        out = np.full(kv.shape, sentinel, dtype=np.uint16)
        oracle.swapin_layers(shape, packed, *lists, l, l + 1, out)
        others = [m for m in range(shape.L) if m != l]
        assert np.all(out[others] == sentinel)
        assert np.all(out[l][:, :, 16:32, :] == sentinel)          # chunk 1 is not listed
        for c in (0, 2):
            b = int(bits[c])
            codes, scale, mn = sections(shape, packed[int(off[c]):int(off[c + 1])], b)
            for kvsel in range(2):
                for h in range(shape.Hkv):
                    slab = (l * 2 + kvsel) * shape.Hkv + h
                    for t in range(shape.T):
                        q = unpack(codes[slab, t], b).astype(np.float32)
                        want = (q * scale[slab, t, 0] + mn[slab, t, 0]).astype(np.float32).astype(np.float16)
                        got = out[l, kvsel, h, c * shape.T + t].view(np.float16)
                        assert np.array_equal(want.view(np.uint16), got.view(np.uint16))
    # all layers one after the other = the whole Load; an empty range changes nothing
    step = np.full(kv.shape, sentinel, dtype=np.uint16)
    for l in range(shape.L):
        oracle.swapin_layers(shape, packed, *lists, l, l + 1, step)
    oracle.swapin_layers(shape, packed, *lists, 2, 2, step)
    whole = np.full(kv.shape, sentinel, dtype=np.uint16)
    oracle.swapin_chunks(shape, packed, *lists, whole)
    assert np.array_equal(step, whole)


# ------------------------------------------------------------------ format 3: binary16 parameters

def sections_h(shape, rec, b):
    """Split a format-3 record into (codes, scale binary16 bits [slabs][T][D/G], mn binary16 bits)."""
    n_codes = shape.slabs * shape.T * shape.D * b // 8
    n_meta = shape.slabs * shape.T * (shape.D // shape.G)
    assert n_codes + 4 * n_meta == len(rec)
    codes = rec[:n_codes].reshape(shape.slabs, shape.T, shape.D * b // 8)
    scale = rec[n_codes:n_codes + 2 * n_meta].view(np.uint16).reshape(shape.slabs, shape.T, -1)
    mn = rec[n_codes + 2 * n_meta:].view(np.uint16).reshape(shape.slabs, shape.T, -1)
    return codes, scale, mn


def test_format3_record_sizes_by_hand():
    """Groups of 64 along head_dim 128, 16 tokens, 2 layers x K/V x 2 heads = 8 slabs: a token row holds
    128*b/8 code bytes and two groups; the parameters weigh 2 x 2 bytes per group instead of 2 x 4."""
    s3 = oracle.Shape(L=2, Hkv=2, Hq=2, D=128, N=64, T=16, G=64, fmt=3)
    s0 = oracle.Shape(L=2, Hkv=2, Hq=2, D=128, N=64, T=16, G=64)
    assert [oracle.record_bytes(s3, b) for b in (16, 8, 4, 2)] == [8 * 16 * 256, 8 * 16 * 136, 8 * 16 * 72, 8 * 16 * 40]
    assert [oracle.record_bytes(s0, b) for b in (8, 4, 2)] == [8 * 16 * 144, 8 * 16 * 80, 8 * 16 * 48]
    bits = np.array([4, 16, 2, 8], dtype=np.uint8)
    assert oracle.chunk_offsets(s3, bits).tolist() == [0, 9216, 9216 + 32768, 9216 + 32768 + 5120, 9216 + 32768 + 5120 + 17408]


@pytest.mark.parametrize("b", [8, 4, 2])
def test_format3_equals_format0_when_the_scale_is_a_binary16_number(b):
    """Values on the grid mn + k * 2^-3, k = 0 .. 2^b - 1 (every level present): the scale is exactly 2^-3,
    a binary16 number, so rounding it changes nothing: same codes as format 0, same parameters after
    widening, and the Load returns the inputs bit for bit."""
    levels = (1 << b) - 1
    rng = np.random.default_rng(b)
    shape3 = shape_small(T=8, D=128, G=64, N=8)
    shape3 = oracle.Shape(shape3.L, shape3.Hkv, shape3.Hq, shape3.D, shape3.N, shape3.T, shape3.G, 3)
    shape0 = shape_small(T=8, D=128, G=64, N=8)
    k = rng.integers(0, levels + 1, size=(1, 2, 1, 8, 128))
    k[..., 0] = 0; k[..., 1] = levels; k[..., 64] = levels; k[..., 65] = 0       # both ends in every group
    kv = (-3.0 + 0.125 * k).astype(np.float16)
    rec3, bits, off3 = compress_one(shape3, kv, b)
    rec0, _, off0 = compress_one(shape0, kv, b)
    c3, sc3, mn3 = sections_h(shape3, rec3, b)
    c0, sc0, mn0 = sections(shape0, rec0, b)
    assert np.array_equal(c3, c0)
    assert np.array_equal(sc3.view(np.float16).astype(np.float32), sc0) and np.all(sc0 == 0.125)
    assert np.array_equal(mn3.view(np.float16).astype(np.float32), mn0) and np.all(mn0 == -3.0)
    out = np.zeros(kv.shape, dtype=np.uint16)
    oracle.swapin_chunks(shape3, rec3, *oracle.build_gather(shape3, off3, bits, [0]), out)
    assert np.array_equal(out, kv.view(np.uint16))


@pytest.mark.parametrize("b", [8, 4, 2])
def test_format3_by_an_independent_route_and_its_error_bound(b):
    """Random data with an outlier channel: the record's sections re-derived with numpy (float32 array
    arithmetic, numpy's own binary16 rounding, the independent bit decoder).  The scale must have been
    rounded to binary16 BEFORE the codes were computed: coding against the unrounded scale gives
    different codes on this input (checked), so a swapped order cannot pass.  Then the error of the
    round trip: half a step of the stored scale, the clamped top of the range (the rounded scale may
    fall short of it by range * 2^-11), and the final binary16 rounding."""
    levels = (1 << b) - 1
    shape = oracle.Shape(L=1, Hkv=2, Hq=2, D=128, N=32, T=16, G=64, fmt=3)
    kv = random_cache(shape, 40 + b)
    rec, bits, off = compress_one(shape, kv, b)
    codes, scale_bits, mn_bits = sections_h(shape, rec[:int(off[1])], b)
    x = kv[:, :, :, 0:16, :].astype(np.float32).reshape(shape.slabs, 16, 2, 64)     # [slab][t][group][k]
    mn = x.min(axis=-1, keepdims=True) + np.float32(0.0)
    mx = x.max(axis=-1, keepdims=True) + np.float32(0.0)
    scale32 = ((mx - mn) / np.float32(levels)).astype(np.float32)
    scale16 = scale32.astype(np.float16)
    assert np.array_equal(scale16.view(np.uint16)[..., 0], scale_bits)
    assert np.array_equal(mn.astype(np.float16).view(np.uint16)[..., 0], mn_bits)
    sc = scale16.astype(np.float32)
    with np.errstate(divide="ignore", invalid="ignore"):
        want = np.where(sc != 0, np.clip(np.rint((x - mn) / sc), 0, levels), 0).astype(np.int64)
        unrounded = np.where(scale32 != 0, np.clip(np.rint((x - mn) / scale32), 0, levels), 0).astype(np.int64)
    got = np.stack([np.stack([unpack(codes[sl, t], b) for t in range(16)]) for sl in range(shape.slabs)])
    assert np.array_equal(got.reshape(want.shape), want)
    if b == 8:
        assert (want != unrounded).any(), "input does not tell the two orders apart"
    out = np.zeros(kv.shape, dtype=np.uint16)
    oracle.swapin_chunks(shape, rec, *oracle.build_gather(shape, off, bits, [0, 1]), out)
    deq = (want.astype(np.float32) * sc + mn).astype(np.float32).astype(np.float16)
    assert np.array_equal(out[:, :, :, 0:16, :].reshape(deq.shape), deq.view(np.uint16))
    err = np.abs(deq.astype(np.float64) - x)
    rng_ = (mx - mn).astype(np.float64)
    bound = sc.astype(np.float64) / 2 + rng_ * 2.0 ** -11 + np.abs(x) * 2.0 ** -11 + 1e-7
    assert np.all(err <= bound)


def test_vectorised_float32_cross_check_on_tiny_workload():
    """The tiny benchmark configuration, re-derived with numpy float32 array arithmetic
    (numpy's float32 divide and rint are the IEEE operations the contract names)."""
    from paper_2403_11805_amd import synth
    wl = synth.WORKLOADS[0]
    g = wl.geom
    shape = oracle.Shape(*g)
    kv = synth.make_kv(g, wl.seed, "cpu", wl.outlier_channels, wl.outlier_scale).numpy()
    bits = synth.draw_bits_uniform(g.n_chunks, wl.seed).numpy()
    assert set(bits.tolist()) <= {8, 4, 2}
    off = oracle.chunk_offsets(shape, bits)
    packed = oracle.compress_chunks(shape, kv, bits, off)
    x = kv.astype(np.float32).reshape(shape.slabs, g.n_chunks, g.T, g.D // g.G, g.G)
    for i in range(g.n_chunks):
        b = int(bits[i])
        levels = np.float32((1 << b) - 1)
        xi = x[:, i]
        mn = xi.min(axis=-1, keepdims=True) + np.float32(0)
        mx = xi.max(axis=-1, keepdims=True) + np.float32(0)
        scale = (mx - mn) / levels
        with np.errstate(divide="ignore", invalid="ignore"):
            code = np.where(scale == 0, 0, np.clip(np.rint((xi - mn) / scale), 0, levels)).astype(np.uint32)
        codes, s_got, m_got = sections(shape, packed[int(off[i]):int(off[i + 1])], b)
        assert np.array_equal(s_got.view(np.uint32), scale[..., 0].view(np.uint32))
        assert np.array_equal(m_got.view(np.uint32), mn[..., 0].view(np.uint32))
        flat = code.reshape(shape.slabs, g.T, g.D)
        per = 8 // b
        packed_ref = np.zeros((shape.slabs, g.T, g.D // per), dtype=np.uint32)
        for k in range(per):
            packed_ref |= flat[..., k::per] << (k * b)
        assert np.array_equal(codes, packed_ref.astype(np.uint8))
        deq = (code.astype(np.float32) * scale + mn).astype(np.float16)
        out = np.zeros(kv.shape, dtype=np.float16)
        oracle.swapin_chunks(shape, packed, *oracle.build_gather(shape, off, bits, [i]), out)
        got = out.reshape(shape.slabs, g.n_chunks, g.T, g.D // g.G, g.G)[:, i]
        assert np.array_equal(got.view(np.uint16), deq.view(np.uint16))

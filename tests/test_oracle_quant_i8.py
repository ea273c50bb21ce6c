"""Pins for the oracle's int8, channel-wise format (the paper's own setting: an 8-bit
cache quantised further per channel, Sec. 3.2 "Compressing chunks" and Sec. 4).  CPU only."""
import numpy as np
import pytest

import oracle


def shape_i8(T=16, D=64, L=1, Hkv=1, N=None):
    return oracle.Shape(L=L, Hkv=Hkv, Hq=Hkv, D=D, N=N or T, T=T, G=64, fmt=1)


def sections(shape, rec, b):
    n_codes = shape.slabs * shape.T * shape.D * b // 8
    n_meta = shape.slabs * shape.D
    assert len(rec) == n_codes + 8 * n_meta
    codes = rec[:n_codes].reshape(shape.slabs, shape.T, shape.D * b // 8)
    scale = rec[n_codes:n_codes + 4 * n_meta].view(np.float32).reshape(shape.slabs, shape.D)
    mn = rec[n_codes + 4 * n_meta:].view(np.float32).reshape(shape.slabs, shape.D)
    return codes, scale, mn


def unpack(row, b):
    per = 8 // b
    return np.array([(int(byte) >> (k * b)) & ((1 << b) - 1) for byte in row for k in range(per)])


def compress_one(shape, kv, b):
    bits = np.full(shape.n_chunks, b, dtype=np.uint8)
    off = oracle.chunk_offsets(shape, bits)
    return oracle.compress_chunks_i8(shape, kv, bits, off), bits, off


def test_record_sizes_by_hand():
    s = oracle.Shape(32, 32, 32, 128, 4096, 16, 64, 1)          # int8 Llama-2-7B cache: 1 GiB
    assert oracle.record_bytes(s, 8) == 2048 * 16 * 128 == 4194304
    assert oracle.record_bytes(s, 4) == 2048 * (16 * 128 // 2 + 8 * 128) == 4194304
    assert oracle.record_bytes(s, 2) == 2048 * (512 + 1024) == 3145728
    assert oracle.record_bytes(s, 1) == 2048 * (256 + 1024) == 2621440
    with pytest.raises(AssertionError):
        oracle.record_bytes(s, 16)


@pytest.mark.parametrize("b", [4, 2, 1])
def test_integer_steps_are_coded_exactly(b):
    """Every channel holds mn, mn+1, ..., mn+levels (both ends present): scale 1, code = x - mn."""
    rng = np.random.default_rng(b)
    shape = shape_i8(T=16, D=64, L=2, Hkv=2)
    levels = (1 << b) - 1
    base = rng.integers(-128, 128 - levels, size=(shape.L, 2, shape.Hkv, 1, shape.D))
    step = rng.integers(0, levels + 1, size=(shape.L, 2, shape.Hkv, shape.T, shape.D))
    step[..., 0, :] = 0
    step[..., 1, :] = levels
    kv = (base + step).astype(np.int8)
    packed, bits, off = compress_one(shape, kv, b)
    codes, scale, mn = sections(shape, packed, b)
    assert np.all(scale == 1.0)
    assert np.array_equal(mn, base.reshape(shape.slabs, shape.D).astype(np.float32))
    flat = step.reshape(shape.slabs, shape.T, shape.D)
    for s in range(shape.slabs):
        for t in range(shape.T):
            assert np.array_equal(unpack(codes[s, t], b), flat[s, t])
    out = np.zeros(kv.shape, dtype=np.int8)
    oracle.swapin_chunks_i8(shape, packed, *oracle.build_gather(shape, off, bits, [0]), out)
    assert np.array_equal(out, kv)


def test_halves_round_to_even_and_literal_bytes():
    shape = shape_i8(T=16, D=64)
    x = np.zeros((1, 2, 1, 16, 64), dtype=np.int8)
    # channel 0, 4 bits: values 0..30 step 2 would give scale 2; odd values are exact ties
    x[0, 0, 0, :, 0] = [0, 30, 1, 3, 5, 7, 9, 11, 13, 15, 17, 19, 21, 23, 25, 27]
    packed, _, _ = compress_one(shape, x, 4)
    codes, scale, mn = sections(shape, packed, 4)
    assert scale[0, 0] == 2.0 and mn[0, 0] == 0.0
    got = [int(codes[0, t, 0]) & 0xf for t in range(16)]
    assert got == [0, 15, 0, 2, 2, 4, 4, 6, 6, 8, 8, 10, 10, 12, 12, 14]     # k+0.5 -> even neighbour
    # 1 bit: channels 0..7 of one token with codes 1,0,0,0,0,0,0,1 -> 0x81 (lowest index in bit 0)
    x[:] = 0
    x[0, 0, 0, 1:, 0:8] = 0
    x[0, 0, 0, 0, 0] = 5
    x[0, 0, 0, 0, 7] = 5
    x[0, 0, 0, 1, 1:7] = 5            # make channels 1..6 non-constant without setting token 0
    packed, _, _ = compress_one(shape, x, 1)
    assert packed[0] == 0x81 and packed[8] == 0x7e      # token 1 starts at byte D/8 = 8
    # 2 bits: codes 0,1,2,3 in channels 0..3 -> 0xE4
    x[:] = 0
    x[0, 0, 0, 0, 0:4] = [0, 1, 2, 3]
    x[0, 0, 0, 1, 0:4] = 3
    x[0, 0, 0, 2, 0:4] = 0
    x[0, 0, 0, 0, 0] = 0
    packed, _, _ = compress_one(shape, x, 2)
    assert packed[0] == 0xE4


@pytest.mark.parametrize("b", [4, 2, 1])
def test_invariants_and_error_bound(b):
    rng = np.random.default_rng(10 + b)
    shape = oracle.Shape(2, 2, 2, 128, 64, 32, 64, 1)
    kv = np.clip(np.rint(rng.normal(size=(2, 2, 2, 64, 128)) * 30), -128, 127).astype(np.int8)
    kv[..., 5] = 17                                  # a constant channel
    packed, bits, off = compress_one(shape, kv, b)
    levels = (1 << b) - 1
    out = np.zeros(kv.shape, dtype=np.int8)
    oracle.swapin_chunks_i8(shape, packed, *oracle.build_gather(shape, off, bits, [0, 1]), out)
    x = kv.astype(np.float64).reshape(shape.slabs, shape.n_chunks, shape.T, shape.D)
    y = out.astype(np.float64).reshape(x.shape)
    for i in range(shape.n_chunks):
        codes, scale, mn = sections(shape, packed[int(off[i]):int(off[i + 1])], b)
        for s in range(shape.slabs):
            c = np.stack([unpack(codes[s, t], b) for t in range(shape.T)])       # [T][D]
            g = x[s, i]
            assert np.array_equal(mn[s], g.min(axis=0).astype(np.float32))
            want_scale = (g.max(axis=0) - g.min(axis=0)).astype(np.float32) / np.float32(levels)
            assert np.array_equal(scale[s], want_scale)
            nz = scale[s] > 0
            assert np.all(c[np.argmin(g, axis=0), np.arange(shape.D)] == 0)
            assert np.all(c[np.argmax(g, axis=0), np.arange(shape.D)][nz] == levels)
            assert np.all(c[:, ~nz] == 0) and scale[s][5] == 0 and mn[s][5] == 17
            for d in range(0, shape.D, 7):
                order = np.argsort(g[:, d], kind="stable")
                assert np.all(np.diff(c[order, d]) >= 0)
            err = np.abs(mn[s].astype(np.float64) + c * scale[s].astype(np.float64) - g)
            assert np.all(err <= scale[s].astype(np.float64) * (0.5 + 2.0 ** -14))
            # the dequantised integer is the rounded reconstruction
            assert np.all(np.abs(y[s, i] - g) <= scale[s].astype(np.float64) * (0.5 + 2.0 ** -14) + 0.5)
            assert np.all(y[s, i][:, 5] == 17)


def test_eight_bit_chunks_pass_through_and_selection():
    shape = oracle.Shape(1, 2, 2, 64, 48, 16, 64, 1)
    rng = np.random.default_rng(3)
    kv = rng.integers(-128, 128, size=(1, 2, 2, 48, 64)).astype(np.int8)
    bits = np.array([8, 2, 8], dtype=np.uint8)
    off = oracle.chunk_offsets(shape, bits)
    assert off.tolist() == [0, 4096, 4096 + 4 * (256 + 512), 2 * 4096 + 4 * 768]
    packed = oracle.compress_chunks_i8(shape, kv, bits, off)
    rec0 = packed[:4096].view(np.int8).reshape(shape.slabs, 16, 64)
    assert np.array_equal(rec0, kv.reshape(shape.slabs, 48, 64)[:, :16])
    out = np.full(kv.shape, 99, dtype=np.int8)
    oracle.swapin_chunks_i8(shape, packed, *oracle.build_gather(shape, off, bits, [0, 2]), out)
    assert np.array_equal(out[..., :16, :], kv[..., :16, :]) and np.array_equal(out[..., 32:, :], kv[..., 32:, :])
    assert np.all(out[..., 16:32, :] == 99)


def test_vectorised_float32_cross_check():
    rng = np.random.default_rng(8)
    shape = oracle.Shape(2, 2, 2, 128, 64, 16, 64, 1)
    kv = np.clip(np.rint(rng.normal(size=(2, 2, 2, 64, 128)) * 25), -128, 127).astype(np.int8)
    bits = np.array([4, 2, 1, 8], dtype=np.uint8)
    off = oracle.chunk_offsets(shape, bits)
    packed = oracle.compress_chunks_i8(shape, kv, bits, off)
    out = np.zeros(kv.shape, dtype=np.int8)
    oracle.swapin_chunks_i8(shape, packed, *oracle.build_gather(shape, off, bits, [0, 1, 2, 3]), out)
    x = kv.astype(np.float32).reshape(shape.slabs, shape.n_chunks, shape.T, shape.D)
    for i in range(3):
        b = int(bits[i])
        levels = np.float32((1 << b) - 1)
        xi = x[:, i]
        mn = xi.min(axis=1, keepdims=True) + np.float32(0)
        mx = xi.max(axis=1, keepdims=True) + np.float32(0)
        scale = (mx - mn) / levels
        with np.errstate(divide="ignore", invalid="ignore"):
            code = np.where(scale == 0, 0, np.clip(np.rint((xi - mn) / scale), 0, levels)).astype(np.uint32)
        codes, s_got, m_got = sections(shape, packed[int(off[i]):int(off[i + 1])], b)
        assert np.array_equal(s_got, scale[:, 0]) and np.array_equal(m_got, mn[:, 0])
        per = 8 // b
        ref = np.zeros((shape.slabs, shape.T, shape.D // per), dtype=np.uint32)
        for k in range(per):
            ref |= code[..., k::per] << (k * b)
        assert np.array_equal(codes, ref.astype(np.uint8))
        deq = np.clip(np.rint(code.astype(np.float32) * scale + mn), -128, 127).astype(np.int8)
        assert np.array_equal(out.reshape(shape.slabs, shape.n_chunks, shape.T, shape.D)[:, i], deq)


# ------------------------------------------------------------------ binary16 parameters (format 2)

def sections_h(shape, rec, b):
    n_codes = shape.slabs * shape.T * shape.D * b // 8
    n_meta = shape.slabs * shape.D
    assert len(rec) == n_codes + 4 * n_meta
    codes = rec[:n_codes].reshape(shape.slabs, shape.T, shape.D * b // 8)
    scale = rec[n_codes:n_codes + 2 * n_meta].view(np.float16).reshape(shape.slabs, shape.D)
    mn = rec[n_codes + 2 * n_meta:].view(np.float16).reshape(shape.slabs, shape.D)
    return codes, scale, mn


def test_half_parameter_record_sizes_by_hand():
    s = oracle.Shape(32, 32, 32, 128, 4096, 16, 64, 2)
    assert oracle.record_bytes(s, 8) == 4194304
    assert oracle.record_bytes(s, 4) == 2048 * (1024 + 4 * 128) == 3145728
    assert oracle.record_bytes(s, 2) == 2048 * (512 + 512) == 2097152
    assert oracle.record_bytes(s, 1) == 2048 * (256 + 512) == 1572864
    bits = np.array([8, 4, 2, 1] * 64, dtype=np.uint8)
    assert int(oracle.chunk_offsets(s, bits)[-1]) == 64 * (4194304 + 3145728 + 2097152 + 1572864)


@pytest.mark.parametrize("b", [4, 2, 1])
def test_half_parameters_equal_format_one_when_the_scale_is_a_half(b):
    """A range that is a multiple of the level count gives an integer scale, exact in binary16:
    codes and reconstruction must then equal those of the fp32-parameter format."""
    rng = np.random.default_rng(40 + b)
    levels = (1 << b) - 1
    s1 = oracle.Shape(1, 2, 2, 64, 32, 16, 64, 1)
    s2 = oracle.Shape(1, 2, 2, 64, 32, 16, 64, 2)
    k = rng.integers(1, 255 // levels + 1, size=(1, 2, 2, 1, 64))                # the scale of a channel
    base = rng.integers(-128, 128 - k * levels)
    step = rng.integers(0, k * levels + 1, size=(1, 2, 2, 32, 64))
    step[..., 0::16, :] = 0                                                      # both ends in every chunk
    step[..., 1::16, :] = k * levels
    kv = (base + step).astype(np.int8)
    assert np.array_equal(kv.astype(np.int64), base + step)
    bits = np.full(2, b, dtype=np.uint8)
    o1, o2 = oracle.chunk_offsets(s1, bits), oracle.chunk_offsets(s2, bits)
    p1, p2 = oracle.compress_chunks_i8(s1, kv, bits, o1), oracle.compress_chunks_i8(s2, kv, bits, o2)
    for i in range(2):
        c1, sc1, m1 = sections(s1, p1[int(o1[i]):int(o1[i + 1])], b)
        c2, sc2, m2 = sections_h(s2, p2[int(o2[i]):int(o2[i + 1])], b)
        assert np.array_equal(c1, c2)
        assert np.array_equal(sc1, sc2.astype(np.float32)) and np.array_equal(m1, m2.astype(np.float32))
        assert np.array_equal(sc1[0], k.reshape(4, 64)[0].astype(np.float32))
    a, h = np.zeros(kv.shape, np.int8), np.zeros(kv.shape, np.int8)
    oracle.swapin_chunks_i8(s1, p1, *oracle.build_gather(s1, o1, bits, [0, 1]), a)
    oracle.swapin_chunks_i8(s2, p2, *oracle.build_gather(s2, o2, bits, [0, 1]), h)
    assert np.array_equal(a, h)


def test_half_parameters_vectorised_cross_check_and_error_bound():
    """Independent numpy route: scale = binary16(float32 range / levels) (numpy's cast rounds to
    nearest even), codes against that rounded scale, reconstruction from the stored halves; and
    the error bound with the rounded scale: |x' - x| <= scale_h / 2 + 1/2."""
    rng = np.random.default_rng(77)
    shape = oracle.Shape(2, 2, 2, 128, 64, 16, 64, 2)
    kv = np.clip(np.rint(rng.normal(size=(2, 2, 2, 64, 128)) * 25), -128, 127).astype(np.int8)
    kv[..., 9] = -3                                              # a constant channel
    kv[0, 0, 0, :16, 11] = np.arange(-128, 128, 16)              # widest range: 240
    kv[0, 0, 0, 1, 11] = 127
    bits = np.array([4, 2, 1, 8], dtype=np.uint8)
    off = oracle.chunk_offsets(shape, bits)
    packed = oracle.compress_chunks_i8(shape, kv, bits, off)
    out = np.zeros(kv.shape, dtype=np.int8)
    oracle.swapin_chunks_i8(shape, packed, *oracle.build_gather(shape, off, bits, [0, 1, 2, 3]), out)
    x = kv.astype(np.float32).reshape(shape.slabs, shape.n_chunks, shape.T, shape.D)
    y = out.reshape(x.shape)
    assert np.array_equal(y[:, 3], kv.reshape(x.shape)[:, 3])     # 8 bits: pass-through
    n_inexact = 0
    for i in range(3):
        b = int(bits[i])
        levels = np.float32((1 << b) - 1)
        xi = x[:, i]
        mn = xi.min(axis=1, keepdims=True)
        mx = xi.max(axis=1, keepdims=True)
        exact = (mx - mn) / levels                                # float32
        scale_h = exact.astype(np.float16)
        scale = scale_h.astype(np.float32)
        n_inexact += int((scale != exact).sum())
        with np.errstate(divide="ignore", invalid="ignore"):
            code = np.where(scale == 0, 0, np.clip(np.rint((xi - mn) / scale), 0, levels)).astype(np.uint32)
        codes, s_got, m_got = sections_h(shape, packed[int(off[i]):int(off[i + 1])], b)
        assert np.array_equal(s_got.view(np.uint16), scale_h[:, 0].view(np.uint16))
        assert np.array_equal(m_got.astype(np.float32), mn[:, 0])
        per = 8 // b
        ref = np.zeros((shape.slabs, shape.T, shape.D // per), dtype=np.uint32)
        for k in range(per):
            ref |= code[..., k::per] << (k * b)
        assert np.array_equal(codes, ref.astype(np.uint8))
        deq = np.clip(np.rint(code.astype(np.float32) * scale + mn), -128, 127).astype(np.int8)
        assert np.array_equal(y[:, i], deq)
        # both ends of every non-constant channel keep their codes; error bound with the stored scale
        assert np.all(code[np.arange(shape.slabs)[:, None], np.argmax(xi, axis=1), np.arange(shape.D)][scale[:, 0] > 0] == levels)
        assert np.all(code[np.arange(shape.slabs)[:, None], np.argmin(xi, axis=1), np.arange(shape.D)] == 0)
        err = np.abs(y[:, i].astype(np.float64) - xi.astype(np.float64))
        assert np.all(err <= scale.astype(np.float64) / 2 + 0.5 + 1e-3)
        assert np.all(y[:, i][..., 9] == -3)
    assert n_inexact > 100, "the test must exercise scales that binary16 cannot hold exactly"

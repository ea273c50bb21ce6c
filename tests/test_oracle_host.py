"""Pins for the oracle's host bookkeeping: record sizes, offsets, rank-based
bit-widths (Sec. 3.2, Eq. 2), gather lists (Load, Sec. 3.1) and the LCTRU
queue with working-set lock (Sec. 3.4).  Expected values are worked out by
hand from the definitions."""
import numpy as np
import pytest

import oracle
from paper_2403_11805_amd import synth


def oshape(i):
    return oracle.Shape(*synth.WORKLOADS[i].geom)


def test_record_sizes_by_hand():
    # tiny: 16 slabs x 16 tokens; a token row is 64 elements, one group
    s = oshape(0)
    assert oracle.record_bytes(s, 16) == 16 * 16 * 64 * 2 == 32768
    assert oracle.record_bytes(s, 8) == 16 * 16 * (64 + 8) == 18432
    assert oracle.record_bytes(s, 4) == 16 * 16 * (32 + 8) == 10240
    assert oracle.record_bytes(s, 2) == 16 * 16 * (16 + 8) == 6144
    # Llama-2-7B shape: 2048 slabs x 16 tokens; rows of 128 elements, two groups
    s = oshape(2)
    assert oracle.record_bytes(s, 16) == 8388608
    assert oracle.record_bytes(s, 8) == 2048 * 16 * (128 + 16) == 4718592
    assert oracle.record_bytes(s, 4) == 2621440 and oracle.record_bytes(s, 2) == 1572864
    # 32k GQA shape: 512 slabs x 32 tokens, group 128
    s = oshape(4)
    assert [oracle.record_bytes(s, b) for b in (16, 8, 4, 2)] == [4194304, 2228224, 1179648, 655360]
    # the whole 4k Llama-2-7B context is 2 GiB in fp16 (Sec. 2.3: "over 2GB")
    assert oracle.record_bytes(oshape(2), 16) * oshape(2).n_chunks == 2 ** 31


def test_offsets_are_a_prefix_sum():
    s = oshape(1)
    bits = np.array([8] * 64 + [4] * 128 + [2] * 64, dtype=np.uint8)
    off = oracle.chunk_offsets(s, bits)
    assert off[0] == 0 and len(off) == 257
    assert int(off[-1]) == 64 * 165888 + 128 * 92160 + 64 * 55296 == 25952256
    assert np.all(np.diff(off.astype(np.int64)) == [oracle.record_bytes(s, int(b)) for b in bits])
    s = oshape(2)
    bits = np.array([8] * 85 + [4] * 85 + [2] * 86, dtype=np.uint8)
    assert int(oracle.chunk_offsets(s, bits)[-1]) == 759169024


def test_bits_from_scores_counts_and_ties():
    d = synth.draw_scores(256, 1).numpy()
    bits = oracle.bits_from_scores(d, 1, 2, 4)
    assert [(bits == b).sum() for b in (8, 4, 2)] == [64, 128, 64]
    assert d[bits == 8].min() >= d[bits == 4].max() and d[bits == 4].min() >= d[bits == 2].max()
    bits = oracle.bits_from_scores(d, 1, 1, 3)
    assert [(bits == b).sum() for b in (8, 4, 2)] == [85, 85, 86]
    bits = oracle.bits_from_scores(np.arange(1024, dtype=np.float32), 1, 1, 3)
    assert [(bits == b).sum() for b in (8, 4, 2)] == [341, 341, 342]
    # equal scores: the lower index ranks first
    bits = oracle.bits_from_scores(np.array([1, 1, 1, 1, 1, 1], dtype=np.float32), 1, 1, 3)
    assert bits.tolist() == [8, 8, 4, 4, 2, 2]
    bits = oracle.bits_from_scores(np.array([0.1, 0.9, 0.5, 0.9], dtype=np.float32), 1, 2, 4)
    assert bits.tolist() == [2, 8, 4, 4]


def test_gather_list():
    s = oshape(0)
    bits = np.array([8, 4, 2, 16] * 8, dtype=np.uint8)
    off = oracle.chunk_offsets(s, bits)
    src, dst, sb = oracle.build_gather(s, off, bits, [1, 2, 7, 31])
    assert src.tolist() == [18432, 18432 + 10240, int(off[7]), int(off[31])]
    assert dst.tolist() == [16, 32, 112, 496] and sb.tolist() == [4, 2, 16, 16]
    with pytest.raises(AssertionError):
        oracle.build_gather(s, off, bits, [2, 1])
    with pytest.raises(AssertionError):
        oracle.build_gather(s, off, bits, [32])


def test_lctru_heavy_first_then_least_recent_and_lock():
    q = oracle.LctruModel()
    # ctx 0 used at t=1, ctx 1 at t=2, ctx 2 at t=3
    for ctx, now in ((0, 1), (1, 2), (2, 3)):
        q.insert(ctx, 0, 8, 100, now)
        q.insert(ctx, 1, 4, 60, now)
        q.insert(ctx, 2, 2, 30, now)
    # heavy (8-bit) sub-queue first, oldest context first inside each sub-queue
    assert q.order() == [(0, 0), (1, 0), (2, 0), (0, 1), (1, 1), (2, 1), (0, 2), (1, 2), (2, 2)]
    q.touch_ctx(0, 10)         # ctx 0 becomes the most recent
    assert q.order()[:3] == [(1, 0), (2, 0), (0, 0)]
    q.lock(1)                  # working set of a call in progress
    assert all(k[0] != 1 for k in q.order())
    assert q.evict(10 ** 6) is None and q.size() == (9, 570)    # cannot supply: nothing popped
    got = q.evict(150)         # 100 (ctx 2) + 100 (ctx 0) >= 150
    assert got == [(2, 0), (0, 0)]
    q.unlock(1)
    assert q.order()[0] == (1, 0)
    q.remove_ctx(1)
    assert q.size() == (4, 180)
    assert q.evict(0) == []


# ------------------------------------------------------------------ thresholds from a global ratio (Eq. 2 / Eq. 3)

def ctx_info(density, bits, weights):
    return sum(weights[int(b)] * float(np.float32(d)) for d, b in zip(density, bits))


def test_optimised_thresholds_meet_the_global_ratio():
    """Levels {8/8, 4/8, 2/8} at a global ratio of 50 % (the paper's setting, Sec. 3.2
    micro experiments and Sec. 4): the mean of the per-chunk ratios must be 1/2."""
    rng = np.random.default_rng(0)
    for n in (12, 48, 256):
        d = rng.random(n).astype(np.float32)
        for printed in (False, True):
            bits, (k8, k4, k2) = oracle.bits_optimise(d, 1, 2, printed)
            assert k8 + k4 + k2 == n and [(bits == b).sum() for b in (8, 4, 2)] == [k8, k4, k2]
            assert k8 * 1.0 + k4 * 0.5 + k2 * 0.25 == n * 0.5
            # Eq. 2: buckets follow the ranking, densest chunks in the least compressed bucket
            if k8 and k4:
                assert d[bits == 8].min() >= d[bits == 4].max()
            if k2 and (k4 or k8):
                assert d[bits != 2].min() >= d[bits == 2].max()
    # other ratios: the largest average that does not exceed the target
    d = rng.random(10).astype(np.float32)
    for num, den in ((1, 4), (1, 1), (3, 8), (5, 8), (2, 3)):
        bits, (k8, k4, k2) = oracle.bits_optimise(d, num, den)
        avg = (k8 + k4 / 2 + k2 / 4) / 10
        assert avg <= num / den + 1e-12 and avg + 0.025 > num / den
    assert oracle.bits_optimise(d, 1, 4)[1] == (0, 0, 10) and oracle.bits_optimise(d, 1, 1)[1] == (10, 0, 0)


def test_optimised_thresholds_average_is_the_largest_reachable():
    """Eq. 3's constraint for every ratio a small context can ask for: the chosen split has the
    largest mean ratio that any split (k8, k4, k2) of the n chunks reaches without exceeding the
    target, found here by trying all of them.  Ratios just below 1 ask for a bit budget no
    split has (3*k8 + k4 = 3n - 1): counts stay non-negative and the mean stays below the target."""
    from fractions import Fraction
    rng = np.random.default_rng(3)
    for n in range(1, 9):
        d = rng.random(n).astype(np.float32)
        for den in (4, 7, 12, 100):
            for num in range((den + 3) // 4, den + 1):
                target = Fraction(num, den)
                reach = max(Fraction(4 * k8 + 2 * k4 + (n - k8 - k4), 4 * n)
                            for k8 in range(n + 1) for k4 in range(n + 1 - k8)
                            if Fraction(4 * k8 + 2 * k4 + (n - k8 - k4), 4 * n) <= target)
                for printed in (False, True):
                    bits, (k8, k4, k2) = oracle.bits_optimise(d, num, den, printed)
                    assert min(k8, k4, k2) >= 0 and k8 + k4 + k2 == n
                    assert [(bits == b).sum() for b in (8, 4, 2)] == [k8, k4, k2]
                    assert Fraction(4 * k8 + 2 * k4 + k2, 4 * n) == reach, (n, num, den)
    assert oracle.bits_optimise(np.arange(10, dtype=np.float32), 99, 100)[1] == (9, 1, 0)
    assert oracle.bits_optimise(np.arange(3, dtype=np.float32), 11, 12)[1] == (2, 1, 0)


def test_optimised_thresholds_against_brute_force():
    """Weights = ratio_w: no assignment of widths with the same bit budget (not only the
    rank-ordered ones) has a larger ctxInfo."""
    import itertools
    rng = np.random.default_rng(1)
    w = {8: 1.0, 4: 0.5, 2: 0.25}
    for trial in range(6):
        n = int(rng.integers(3, 9))
        d = rng.random(n).astype(np.float32)
        if trial % 2:
            d[rng.integers(0, n, size=2)] = 0.5          # ties
        for num, den in ((1, 2), (5, 8)):
            bits, (k8, k4, k2) = oracle.bits_optimise(d, num, den)
            budget = 4 * k8 + 2 * k4 + k2
            best = max(ctx_info(d, a, w) for a in itertools.product((8, 4, 2), repeat=n)
                       if sum(x // 2 for x in a) == budget)
            assert ctx_info(d, bits, w) == pytest.approx(best, rel=1e-12)


def test_optimised_thresholds_closed_forms():
    """One free variable: k4 = n - 3*k8, k2 = 2*k8 at a 50 % ratio.
    Weights ratio_w: ctxInfo rises with k8 whenever densities differ -> k8 = n // 3.
    Weights 1/ratio_w (as printed): d ctxInfo / d k8 = 4*D(rank n-2*k8) - D(rank k8);
    with a fraction `a` of chunks at density H and the rest at 1 the optimum is
    k8 = n/3 if a*(H-1) < 1 and k8 = 0 if a*(H-1) > 1; equal densities -> k8 = n/3."""
    n = 12
    distinct = np.linspace(1.0, 2.0, n).astype(np.float32)
    assert oracle.bits_optimise(distinct, 1, 2)[1] == (4, 0, 8)
    assert oracle.bits_optimise(np.ones(n, dtype=np.float32), 1, 2)[1] == (0, 12, 0)   # all equal: first maximum
    assert oracle.bits_optimise(np.ones(n, dtype=np.float32), 1, 2, True)[1] == (4, 0, 8)
    two = np.ones(n, dtype=np.float32)
    two[[3, 7]] = 4.0             # a = 1/6, H = 4: a*(H-1) = 0.5 < 1
    bits, counts = oracle.bits_optimise(two, 1, 2, True)
    assert counts == (4, 0, 8) and bits[3] == 8 and bits[7] == 8
    two[[3, 7]] = 10.0            # a*(H-1) = 1.5 > 1: every chunk stays at 4 bits
    assert oracle.bits_optimise(two, 1, 2, True)[1] == (0, 12, 0)
    # the printed objective at its optimum is not below its neighbours
    rng = np.random.default_rng(5)
    d = (rng.random(60) ** 4).astype(np.float32)
    w = {8: 1.0, 4: 2.0, 2: 4.0}
    bits, (k8, k4, k2) = oracle.bits_optimise(d, 1, 2, True)
    order = sorted(range(60), key=lambda i: (-float(d[i]), i))
    for k in (k8 - 1, k8 + 1):
        if 0 <= k <= 20:
            alt = np.zeros(60, dtype=np.uint8)
            for rank, i in enumerate(order):
                alt[i] = 8 if rank < k else (4 if rank < k + 60 - 3 * k else 2)
            assert ctx_info(d, bits, w) >= ctx_info(d, alt, w)


# ------------------------------------------------------------------ swapping-recompute planning (Sec. 3.3, Eq. 4)

def test_fit_line_recovers_exact_lines_and_matches_polyfit():
    x = [1.0, 2.0, 4.0, 8.0, 16.0]
    slope, icpt = oracle.fit_line(x, [3.0 * v + 0.5 for v in x])
    assert slope == pytest.approx(3.0, rel=1e-14) and icpt == pytest.approx(0.5, rel=1e-12)
    rng = np.random.default_rng(2)
    t = rng.random(5)
    ref = np.polyfit(x, t, 1)                      # library least squares
    slope, icpt = oracle.fit_line(x, t)
    assert slope == pytest.approx(ref[0], rel=1e-10) and icpt == pytest.approx(ref[1], rel=1e-10)


def test_plan_pipeline_against_brute_force_over_all_choices():
    """No triple (r8, r4, r2) <= missing, heaviest-first or not, has a smaller delay."""
    import itertools
    rng = np.random.default_rng(3)
    rec = [4718592, 2621440, 1572864]
    for trial in range(30):
        missing = [int(v) for v in rng.integers(0, 7, size=3)]
        model = (float(rng.random() * 2e-3), float(rng.random() * 1e-3),
                 float(rng.random() / 2e9), float(rng.random() * 1e-3))
        r, d = oracle.plan_pipeline(model, missing, rec)
        assert all(0 <= a <= b for a, b in zip(r, missing))
        assert d == oracle.pipeline_delay(model, missing, rec, r)
        best = min(oracle.pipeline_delay(model, missing, rec, c)
                   for c in itertools.product(*[range(m + 1) for m in missing]))
        assert d == pytest.approx(best, rel=1e-12, abs=1e-18)


def test_plan_pipeline_closed_forms():
    """One width, no fixed costs: T_re = a*x and T_IO = c*B*(n - x) cross at x* = n*c*B/(a + c*B);
    the best integer is next to it.  Free recompute -> recompute everything; free IO -> load
    everything; heaviest chunks leave the IO first."""
    rec = [4000, 2000, 1000]
    n, a, c = 100, 1.0, 0.5 / 4000          # c*B = 0.5 -> x* = 100 * 0.5 / 1.5 = 33.3
    r, d = oracle.plan_pipeline((a, 0.0, c, 0.0), [n, 0, 0], rec)
    assert r in ((33, 0, 0), (34, 0, 0)) and d == pytest.approx(min(max(33, 0.5 * 67), max(34, 0.5 * 66)))
    assert oracle.plan_pipeline((0.0, 0.0, 1e-6, 0.0), [3, 4, 5], rec) == ((3, 4, 5), 0.0)
    assert oracle.plan_pipeline((1.0, 0.0, 0.0, 0.0), [3, 4, 5], rec) == ((0, 0, 0), 0.0)
    r, _ = oracle.plan_pipeline((1e-3, 0.0, 1e-6, 0.0), [2, 50, 50], rec)
    assert r[0] == 2 and r[2] == 0 and 0 < r[1] < 50      # 8-bit chunks first, then 4-bit
    # a fixed recompute cost larger than the whole IO: do not start recomputing
    assert oracle.plan_pipeline((1e-6, 1.0, 1e-6, 0.0), [5, 5, 5], rec)[0] == (0, 0, 0)


def test_pipeline_split_hand_example_and_properties():
    """Which chunks a plan recomputes: the earliest of each width.  A hand-made example, then random
    cases checked through what defines the result: the two lists partition the missing chunks, each
    is ascending, the recomputed ones hold exactly the planned number per width, and no loaded chunk
    of a width precedes a recomputed chunk of the same width."""
    bits = np.array([8, 4, 2, 8, 4, 2, 8, 4, 2, 8], dtype=np.uint8)
    re, io = oracle.pipeline_split([0, 1, 3, 4, 5, 6, 8, 9], bits, (2, 1, 1))
    assert re.tolist() == [0, 1, 3, 5] and io.tolist() == [4, 6, 8, 9]
    re, io = oracle.pipeline_split([2, 5, 7], bits, (0, 0, 0))
    assert re.tolist() == [] and io.tolist() == [2, 5, 7]
    re, io = oracle.pipeline_split([2, 5, 7], bits, (0, 1, 2))
    assert re.tolist() == [2, 5, 7] and io.tolist() == []
    rng = np.random.default_rng(4)
    for _ in range(50):
        n = int(rng.integers(1, 40))
        bits = rng.choice([8, 4, 2], n).astype(np.uint8)
        missing = np.flatnonzero(rng.random(n) < 0.6)
        have = [int((bits[missing] == b).sum()) for b in (8, 4, 2)]
        plan = tuple(int(rng.integers(0, h + 1)) for h in have)
        re, io = oracle.pipeline_split(missing, bits, plan)
        assert sorted(re.tolist() + io.tolist()) == missing.tolist()
        assert re.tolist() == sorted(re.tolist()) and io.tolist() == sorted(io.tolist())
        for b, want in zip((8, 4, 2), plan):
            mine = [i for i in re if bits[i] == b]
            assert len(mine) == want
            assert all(j > max(mine) for j in io if bits[j] == b) if mine else True
    with pytest.raises(AssertionError):
        oracle.pipeline_split([0, 1], np.array([8, 8], dtype=np.uint8), (3, 0, 0))

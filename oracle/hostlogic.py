"""Oracle for the host-side bookkeeping of the context-switch path: record
sizes and offsets, rank-to-bit-width bucketing (Sec. 3.2, Eq. 2 with fixed
thresholds), the gather list of the Load primitive (Sec. 3.1) and the LCTRU
eviction queue with its working-set lock (Sec. 3.4).

TEST INFRASTRUCTURE ONLY.  Plain Python on small integer inputs; written as the
definitions read, not for speed.
"""
from __future__ import annotations

import numpy as np

VALID_BITS = (16, 8, 4, 2)
VALID_BITS_I8 = (8, 4, 2, 1)


def record_bytes(shape, bits: int) -> int:
    """Bytes of one chunk's packed record.  fp16 format: b < 16: every token row of
    every slab holds D*b/8 code bytes plus one fp32 scale and one fp32 minimum per
    group of G elements (binary16 parameters in format 3); b = 16: the raw fp16 bytes.  int8 channel-wise formats: b < 8:
    T*D*b/8 code bytes per slab plus one scale and one minimum per channel (fp32, or
    binary16 in format 2); b = 8: raw."""
    slabs = shape.L * 2 * shape.Hkv
    fmt = getattr(shape, "fmt", 0)
    if fmt in (1, 2):
        assert bits in VALID_BITS_I8
        if bits == 8:
            return slabs * shape.T * shape.D
        meta = 8 if fmt == 1 else 4            # fp32 or binary16 (scale, minimum) per channel
        return slabs * (shape.T * shape.D * bits // 8 + meta * shape.D)
    assert bits in VALID_BITS
    if bits == 16:
        return slabs * shape.T * shape.D * 2
    meta = 4 if fmt == 3 else 8                # binary16 (format 3) or fp32 (scale, minimum) per group
    return slabs * shape.T * (shape.D * bits // 8 + meta * (shape.D // shape.G))


def chunk_offsets(shape, bits) -> np.ndarray:
    """off[0] = 0, off[i+1] = off[i] + record_bytes(bits[i])."""
    off = [0]
    for b in bits:
        off.append(off[-1] + record_bytes(shape, int(b)))
    return np.array(off, dtype=np.uint64)


def bits_from_scores(density, num8: int, num4: int, den: int) -> np.ndarray:
    """Rank chunks by density (highest first, ties by lower index first); the
    densest n*num8//den chunks keep 8 bits, the following ones up to
    n*(num8+num4)//den in total get 4 bits, the rest 2 bits."""
    density = [float(np.float32(d)) for d in density]
    n = len(density)
    order = sorted(range(n), key=lambda i: (-density[i], i))
    k8 = n * num8 // den
    k84 = n * (num8 + num4) // den
    bits = np.zeros(n, dtype=np.uint8)
    for rank, i in enumerate(order):
        bits[i] = 8 if rank < k8 else (4 if rank < k84 else 2)
    return bits


def bits_optimise(density, ratio_num: int, ratio_den: int, as_printed: bool = False):
    """Thresholds of Eq. 2 chosen by Eq. 3 for the levels {8/8, 4/8, 2/8}.

    Chunks are ranked densest first (ties: lower index).  With k8 chunks at 8
    bits, k4 at 4 and k2 at 2, the average ratio (k8 + k4/2 + k2/4)/n has to be
    the largest reachable value that does not exceed ratio_num/ratio_den; that fixes
    3*k8 + k4 = M = floor(n*(4*ratio - 1)) and leaves k8 free (M = 3n - 1 is the one
    total no split of n chunks reaches - it would need k4 = 2 with one chunk left -
    and gives way to 3n - 2).  Every feasible k8
    is evaluated: ctxInfo = sum_w weight_w * (sum of densities in bucket w), with
    weight_w = ratio_w (denser chunks should get more bits) or, as_printed,
    1/ratio_w (the formula as printed).  The first maximum (smallest k8) wins.
    Returns (bits, (k8, k4, k2))."""
    d = [float(np.float32(x)) for x in density]
    n = len(d)
    order = sorted(range(n), key=lambda i: (-d[i], i))
    prefix = [0.0]
    for i in order:
        prefix.append(prefix[-1] + d[i])
    w8, w4, w2 = (1.0, 2.0, 4.0) if as_printed else (1.0, 0.5, 0.25)
    M = n * (4 * ratio_num - ratio_den) // ratio_den
    if n > 0 and M == 3 * n - 1:
        M -= 1
    best = None
    for k8 in range(0, n + 1):
        k4 = M - 3 * k8
        k2 = n - k8 - k4
        if k4 < 0 or k2 < 0:
            continue
        s8 = prefix[k8]
        s4 = prefix[k8 + k4] - prefix[k8]
        s2 = prefix[n] - prefix[k8 + k4]
        info = w8 * s8 + w4 * s4 + w2 * s2
        if best is None or info > best[0]:
            best = (info, k8, k4, k2)
    _, k8, k4, k2 = best
    bits = np.zeros(n, dtype=np.uint8)
    for rank, i in enumerate(order):
        bits[i] = 8 if rank < k8 else (4 if rank < k8 + k4 else 2)
    return bits, (k8, k4, k2)


def fit_line(x, t):
    """Least-squares line t = slope*x + intercept (Sec. 3.3 i: delays are approximated by
    linear functions fitted to discrete test points)."""
    n = len(x)
    mx = sum(float(v) for v in x) / n
    mt = sum(float(v) for v in t) / n
    sxx = sum((float(a) - mx) * (float(a) - mx) for a in x)
    sxt = sum((float(a) - mx) * (float(b) - mt) for a, b in zip(x, t))
    slope = sxt / sxx
    return slope, mt - slope * mx


def pipeline_delay(model, missing, record_bytes, recompute):
    """Eq. 4 for one choice: max(T_re(#recomputed), T_IO(bytes still loaded)); an idle stage costs 0."""
    re_per_chunk, re_fixed, io_per_byte, io_fixed = model
    x = sum(recompute)
    all_bytes = (float(missing[0]) * float(record_bytes[0]) + float(missing[1]) * float(record_bytes[1]) +
                 float(missing[2]) * float(record_bytes[2]))
    removed = (float(recompute[0]) * float(record_bytes[0]) + float(recompute[1]) * float(record_bytes[1]) +
               float(recompute[2]) * float(record_bytes[2]))
    t_re = re_per_chunk * float(x) + re_fixed if x > 0 else 0.0
    t_io = io_per_byte * (all_bytes - removed) + io_fixed if x < sum(missing) else 0.0
    return max(t_re, t_io)


def plan_pipeline(model, missing, record_bytes):
    """Eq. 4: how many missing chunks of each width (8, 4, 2 bits) to recompute instead of
    loading.  For every total, the heaviest records are recomputed first; the first total
    with the smallest delay wins.  Returns ((r8, r4, r2), delay)."""
    best = None
    for x in range(sum(missing) + 1):
        r8 = min(x, missing[0])
        r4 = min(x - r8, missing[1])
        r = (r8, r4, x - r8 - r4)
        d = pipeline_delay(model, missing, record_bytes, r)
        if best is None or d < best[1]:
            best = (r, d)
    return best


def pipeline_split(missing_idx, bits, recompute):
    """The chunks a plan of Eq. 4 sends to each stage.  `missing_idx` (strictly ascending) are
    the chunks to recover, bits[i] the width of chunk i, recompute = (r8, r4, r2) the number of
    8-, 4- and 2-bit chunks to recompute.  The paper leaves open WHICH chunks of a width are
    recomputed; the reading here: the earliest ones (lowest index), so that a recomputed
    token depends on as few loaded chunks as possible.  Returns (recompute_idx, load_idx),
    both ascending: together they are missing_idx."""
    want = {8: recompute[0], 4: recompute[1], 2: recompute[2]}
    re_idx, io_idx = [], []
    for i in missing_idx:
        b = int(bits[int(i)])
        if want.get(b, 0) > 0:
            want[b] -= 1
            re_idx.append(int(i))
        else:
            io_idx.append(int(i))
    assert all(v == 0 for v in want.values()), "more chunks of a width to recompute than are missing"
    return np.array(re_idx, dtype=np.int32), np.array(io_idx, dtype=np.int32)


def build_gather(shape, off, bits, chunk_idx):
    """Gather list for loading the chunks `chunk_idx` (strictly ascending):
    where each record starts, which token it lands on, and its bit-width."""
    idx = [int(i) for i in chunk_idx]
    assert all(0 <= i < shape.N // shape.T for i in idx)
    assert all(a < b for a, b in zip(idx, idx[1:]))
    src_off = np.array([int(off[i]) for i in idx], dtype=np.uint64)
    dst_tok = np.array([i * shape.T for i in idx], dtype=np.int32)
    sel_bits = np.array([int(bits[i]) for i in idx], dtype=np.uint8)
    return src_off, dst_tok, sel_bits


class LctruModel:
    """LCTRU queue (Sec. 3.4): one sub-queue per bit-width, concatenated with
    the least compressed (most bits) first; inside a sub-queue the entry whose
    context was used longest ago comes first.  Ties: lower context id, then
    lower chunk index.  Chunks of a locked context (the working set of a call in
    progress) are never handed out."""

    def __init__(self):
        self.entries = {}   # (ctx, chunk) -> dict(bits, bytes, last)
        self.locked = set()

    def insert(self, ctx, chunk, bits, nbytes, now):
        assert (ctx, chunk) not in self.entries and bits in VALID_BITS
        self.entries[(ctx, chunk)] = dict(bits=bits, bytes=nbytes, last=now)

    def touch_ctx(self, ctx, now):
        for (c, _), e in self.entries.items():
            if c == ctx:
                e["last"] = now

    def lock(self, ctx):
        self.locked.add(ctx)

    def unlock(self, ctx):
        self.locked.discard(ctx)

    def remove_ctx(self, ctx):
        self.entries = {k: v for k, v in self.entries.items() if k[0] != ctx}
        self.locked.discard(ctx)

    def order(self):
        keys = [k for k in self.entries if k[0] not in self.locked]
        keys.sort(key=lambda k: (-self.entries[k]["bits"], self.entries[k]["last"], k[0], k[1]))
        return keys

    def evict(self, bytes_needed, cap=None):
        """Pop from the front until the freed bytes reach bytes_needed; None
        (and no change) if the unlocked entries cannot supply that much or more
        than `cap` entries would be needed."""
        order = self.order()
        got, out = 0, []
        for k in order:
            if got >= bytes_needed:
                break
            out.append(k)
            got += self.entries[k]["bytes"]
        if got < bytes_needed or (cap is not None and len(out) > cap):
            return None
        for k in out:
            del self.entries[k]
        return out

    def size(self):
        return len(self.entries), sum(e["bytes"] for e in self.entries.values())

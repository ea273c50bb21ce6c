"""GPU test of the chunk life cycle across two contexts (Sec. 3.1 primitives, Sec. 3.4): the
chunks a call adds are compressed and swapped out ahead of time when it returns, memory pressure
reclaims chunks in LCTRU order without moving data, and a context switch loads what is missing -
resident records from the device pool, reclaimed ones from pinned host memory, one more by a
Fault.  The recovered cache must equal the oracle's dequantisation of the oracle's records bit
for bit, and the queue must agree with the oracle's model at every step."""
import numpy as np
import pytest
import torch

import oracle
import paper_2403_11805_amd as kvs
from paper_2403_11805_amd import synth

from gpu_util import DEV, both_shapes

pytestmark = pytest.mark.gpu
POISON = 0xEE


class Context:
    def __init__(self, cid, seed):
        self.g = synth.Geometry(2, 2, 2, 128, 512, 16, 64)
        self.ks, self.os = both_shapes(self.g)
        self.cid = cid
        self.kv_host = synth.make_kv(self.g, seed, "cpu", 1, 10.0).numpy()
        self.kv = torch.from_numpy(self.kv_host).to(DEV)                 # what the engine has produced
        self.bits = synth.draw_bits_uniform(self.g.n_chunks, seed).numpy()
        self.off = kvs.kv_chunk_offsets(self.ks, self.bits)
        total = int(self.off[-1])
        self.pool = torch.full((total,), POISON, dtype=torch.uint8, device=DEV)   # records resident in HBM
        self.store = torch.zeros(total, dtype=torch.uint8).pin_memory()           # ahead-of-time copies
        self.bits_d = torch.from_numpy(self.bits).to(DEV)
        self.off_d = torch.from_numpy(self.off.view(np.int64)).to(DEV)
        self.resident = set()
        self.want = oracle.compress_chunks(self.os, self.kv_host, self.bits, self.off)

    def call_returns(self, chunks, queue, model, now, copy_s):
        """The chunks this call added: compress, copy out ahead of time, enter the queue."""
        idx = torch.tensor(chunks, dtype=torch.int32, device=DEV)
        kvs.kv_compress_selected(self.ks, self.kv, self.bits_d, self.off_d, idx, self.pool)
        for i in chunks:
            kvs.kv_swapout_aot(self.pool, self.store, int(self.off[i]), int(self.off[i + 1]),
                               torch.cuda.current_stream(), copy_s)
            nbytes = int(self.off[i + 1] - self.off[i])
            queue.insert(self.cid, i, int(self.bits[i]), nbytes, now)
            model.insert(self.cid, i, int(self.bits[i]), nbytes, now)
            self.resident.add(i)

    def reclaim(self, chunks):
        """Reclaim moves no data: the record is already in the store; its HBM bytes are reused."""
        for i in chunks:
            self.pool[int(self.off[i]):int(self.off[i + 1])] = POISON
            self.resident.discard(i)


def test_two_contexts_claim_reclaim_load_fault():
    a, b = Context(0, 61), Context(1, 62)
    ctxs = {0: a, 1: b}
    queue, model = kvs.Lctru(), oracle.LctruModel()
    copy_s, comp_s = torch.cuda.Stream(), torch.cuda.Stream()
    a.call_returns(list(range(0, 16)), queue, model, 1, copy_s)          # A: first call, 256 tokens
    b.call_returns(list(range(0, 32)), queue, model, 2, copy_s)          # B: one call, 512 tokens
    a.call_returns(list(range(16, 32)), queue, model, 3, copy_s)         # A: second call
    queue.touch_ctx(0, 3); model.touch_ctx(0, 3)
    copy_s.synchronize()
    for c in (a, b):
        assert np.array_equal(c.store.numpy(), c.want), "ahead-of-time copies differ from the oracle's records"
    assert queue.order() == model.order()
    # memory pressure while A is running: reclaim half of all bytes, A's working set is locked
    queue.lock(0); model.lock(0)
    need = (int(a.off[-1]) + int(b.off[-1])) // 4
    evicted = queue.evict(need)
    assert evicted == model.evict(need)
    assert evicted and all(ctx == 1 for ctx, _ in evicted), "only the unlocked context may lose chunks"
    assert [int(b.bits[i]) for _, i in evicted] == sorted((int(b.bits[i]) for _, i in evicted), reverse=True), \
        "heavier chunks go first"
    b.reclaim([i for _, i in evicted])
    queue.unlock(0); model.unlock(0)
    assert queue.order() == model.order()
    # switch to B: everything it needs is loaded into a fresh cache
    queue.lock(1); model.lock(1)
    queue.touch_ctx(1, 4); model.touch_ctx(1, 4)
    cache = torch.full(b.ks.kv_dims, 0x7bff, dtype=torch.int16, device=DEV).view(torch.float16)
    missing = sorted(set(range(b.g.n_chunks)) - b.resident)
    present = sorted(b.resident)
    fault = missing.pop()                                                # noticed late: a Fault
    assert missing and present
    kvs.kv_load_chunks(b.ks, b.pool, b.off, b.bits, present, cache)      # resident records: from HBM
    src, dst, sb = kvs.kv_build_gather(b.ks, b.off, b.bits, missing)     # reclaimed ones: from the store
    staging = torch.empty(2 * kvs.kv_record_bytes(b.ks, 8), dtype=torch.uint8, device=DEV)
    kvs.kv_swapin_pinned(b.ks, b.store, src, dst, sb, staging, 2, cache, copy_s, comp_s)
    comp_s.synchronize(); copy_s.synchronize()
    T = b.g.T
    assert bool((cache[:, :, :, fault * T:(fault + 1) * T].view(torch.int16) == 0x7bff).all())
    src, dst, sb = kvs.kv_build_gather(b.ks, b.off, b.bits, [fault])     # Fault = Load of one chunk
    kvs.kv_swapin_pinned(b.ks, b.store, src, dst, sb, staging, 2, cache, copy_s, comp_s)
    comp_s.synchronize(); copy_s.synchronize()
    torch.cuda.synchronize()
    ref = np.zeros(b.kv_host.shape, dtype=np.uint16)
    everything = list(range(b.g.n_chunks))
    oracle.swapin_chunks(b.os, b.want, *oracle.build_gather(b.os, b.off, b.bits, everything), ref)
    assert np.array_equal(cache.cpu().numpy().view(np.uint16), ref), "recovered cache differs from the oracle"
    # the loaded chunks are resident again; B leaves, the queue matches the model to the end
    for i in missing + [fault]:
        nbytes = int(b.off[i + 1] - b.off[i])
        queue.insert(1, i, int(b.bits[i]), nbytes, 4); model.insert(1, i, int(b.bits[i]), nbytes, 4)
    queue.unlock(1); model.unlock(1)
    assert queue.order() == model.order()
    queue.remove_ctx(0); model.remove_ctx(0)
    assert queue.order() == model.order() and all(ctx == 1 for ctx, _ in queue.order())
    queue.close()

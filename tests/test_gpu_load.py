"""GPU tests of kv_load_chunks, the Load primitive in one call (Sec. 3.1; Fault with one
chunk): host lists in, gather list in the kernel arguments.  Compared with the oracle's
swap-in of the same records element by element, and with kv_swapin_chunks bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2403_11805_amd as kvs
from paper_2403_11805_amd import binding, synth

from gpu_util import DEV, both_shapes, gpu_compress, gpu_swapin

pytestmark = pytest.mark.gpu

SENTINEL = 0x7bff


def selections(n):
    rng = np.random.default_rng(n)
    picks = [[0], [n - 1], list(range(n)), sorted(rng.choice(n, 2 * n // 5, replace=False).tolist())]
    if n > 65:
        picks += [list(range(64)), list(range(3, 3 + 65)), list(range(0, n, 2))]
    return picks


@pytest.mark.parametrize("geom", [(2, 2, 2, 128, 2048, 16, 64),       # 128 chunks: two launches when all are loaded
                                  (1, 3, 3, 64, 160, 16, 64),         # 10 chunks, head_dim 64
                                  (2, 1, 1, 256, 3200, 32, 128)])     # 100 chunks, 8 wavefront-rows per unit
def test_load_equals_oracle_and_list_path(geom):
    g = synth.Geometry(*geom)
    ks, os_ = both_shapes(g)
    kv_host = synth.make_kv(g, 11, "cpu", 1, 10.0).numpy()
    bits = synth.draw_bits_uniform(g.n_chunks, 11, widths=(16, 8, 4, 2)).numpy()
    kv_dev = torch.from_numpy(kv_host).to(DEV)
    packed_dev, off = gpu_compress(ks, kv_dev, bits)
    packed = packed_dev[:int(off[-1])].cpu().numpy()
    for idx in selections(g.n_chunks):
        out = torch.full(ks.kv_dims, SENTINEL, dtype=torch.int16, device=DEV).view(torch.float16)
        kvs.kv_load_chunks(ks, packed_dev, off, bits, idx, out)
        torch.cuda.synchronize()
        ref = np.full(kv_host.shape, SENTINEL, dtype=np.uint16)
        oracle.swapin_chunks(os_, packed, *oracle.build_gather(os_, off, bits, idx), ref)
        got = out.cpu().numpy().view(np.uint16)
        assert np.array_equal(got, ref), f"{len(idx)} chunks: {(got != ref).sum()} values differ from the oracle"
        via_lists = torch.full(ks.kv_dims, SENTINEL, dtype=torch.int16, device=DEV).view(torch.float16)
        gpu_swapin(ks, packed_dev, off, bits, np.asarray(idx, dtype=np.int32), via_lists)
        assert torch.equal(out.view(torch.int16), via_lists.view(torch.int16))


@pytest.mark.parametrize("fmt", [1, 2])
def test_load_int8_formats(fmt):
    g = synth.Geometry(2, 2, 2, 128, 1600, 16, 64)
    ks, os_ = both_shapes(g, fmt)
    kv_host = synth.make_kv_i8(g, 4).numpy()
    bits = synth.draw_bits_uniform(g.n_chunks, 4, widths=(8, 4, 2, 1)).numpy()
    kv_dev = torch.from_numpy(kv_host).to(DEV)
    packed_dev, off = gpu_compress(ks, kv_dev, bits)
    packed = packed_dev[:int(off[-1])].cpu().numpy()
    for idx in selections(g.n_chunks):
        out = torch.full(ks.kv_dims, 0x55, dtype=torch.int8, device=DEV)
        kvs.kv_load_chunks(ks, packed_dev, off, bits, idx, out)
        torch.cuda.synchronize()
        ref = np.full(kv_host.shape, 0x55, dtype=np.int8)
        oracle.swapin_chunks_i8(os_, packed, *oracle.build_gather(os_, off, bits, idx), ref)
        assert np.array_equal(out.cpu().numpy(), ref)


def test_bad_list_is_refused_before_anything_is_written():
    g = synth.Geometry(1, 2, 2, 64, 256, 16, 64)
    ks, _ = both_shapes(g)
    bits = synth.draw_bits_uniform(g.n_chunks, 2).numpy()
    kv_dev = synth.make_kv(g, 2, DEV)
    packed_dev, off = gpu_compress(ks, kv_dev, bits)
    out = torch.full(ks.kv_dims, SENTINEL, dtype=torch.int16, device=DEV).view(torch.float16)
    for idx in ([3, 2], [1, 1], [0, g.n_chunks], [-1, 4]):
        with pytest.raises(kvs.KvError) as e:
            kvs.kv_load_chunks(ks, packed_dev, off, bits, idx, out)
        assert e.value.code == binding.KV_EINDEX
    torch.cuda.synchronize()
    assert bool((out.view(torch.int16) == SENTINEL).all())
    kvs.kv_load_chunks(ks, packed_dev, off, bits, [], out)           # nothing to load: a no-op
    torch.cuda.synchronize()
    assert bool((out.view(torch.int16) == SENTINEL).all())


@pytest.mark.parametrize("fmt", [0, 1, 2, 3])
def test_compress_selected_writes_only_the_listed_records(fmt):
    """kv_compress_selected (the chunks a call added, compressed when it returns, Sec. 3.4 i): the
    listed records equal the oracle's bit for bit, every other byte of the pool keeps its value."""
    g = synth.Geometry(2, 2, 2, 128, 1280, 16, 64)              # 80 chunks
    ks, os_ = both_shapes(g, fmt)
    if fmt in (0, 3):
        kv_host = synth.make_kv(g, 13, "cpu", 1, 10.0).numpy()
        bits = synth.draw_bits_uniform(g.n_chunks, 13, widths=(16, 8, 4, 2)).numpy()
    else:
        kv_host = synth.make_kv_i8(g, 13).numpy()
        bits = synth.draw_bits_uniform(g.n_chunks, 13, widths=(8, 4, 2, 1)).numpy()
    off = kvs.kv_chunk_offsets(ks, bits)
    want = oracle.compress_chunks(os_, kv_host, bits, off) if fmt in (0, 3) else oracle.compress_chunks_i8(os_, kv_host, bits, off)
    kv_dev = torch.from_numpy(kv_host).to(DEV)
    bits_d = torch.from_numpy(bits).to(DEV)
    off_d = torch.from_numpy(off.view(np.int64)).to(DEV)
    for idx in ([79], [0, 1, 2], [5, 17, 18, 40, 77], list(range(0, 80, 3)), [63, 2, 30]):   # any order
        pool = torch.full((int(off[-1]) + 64,), 0xA5, dtype=torch.uint8, device=DEV)
        kvs.kv_compress_selected(ks, kv_dev, bits_d, off_d, torch.tensor(idx, dtype=torch.int32, device=DEV), pool)
        torch.cuda.synchronize()
        got = pool.cpu().numpy()
        expect = np.full(len(got), 0xA5, dtype=np.uint8)
        for i in idx:
            expect[int(off[i]):int(off[i + 1])] = want[int(off[i]):int(off[i + 1])]
        assert np.array_equal(got, expect), f"chunks {idx}: {(got != expect).sum()} pool bytes differ"
    pool = torch.full((int(off[-1]),), 0xA5, dtype=torch.uint8, device=DEV)
    kvs.kv_compress_selected(ks, kv_dev, bits_d, off_d, torch.empty(0, dtype=torch.int32, device=DEV), pool)
    torch.cuda.synchronize()
    assert bool((pool == 0xA5).all())

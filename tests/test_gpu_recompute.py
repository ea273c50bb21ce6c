"""GPU parity: kv_recompute_layer (recompute of interleaved chunks, Sec. 3.3) against the
float64 oracle.

The GPU path rounds intermediates to fp16 where an engine would (normalised activations,
probabilities, hidden states); the oracle rounds only what the data flow fixes (K and V in
the fp16 cache).  Bars, from that arithmetic (u = 2^-11, the fp16 unit roundoff):
  recomputed K/V: one fp16 rounding of the inputs of a d_model-term dot product (about
      0.6 u of the result's rms) plus one rounding of the result on either side
      -> |diff| <= 2e-3 * |ref| + 2e-3 * rms(ref);
  layer output: six more fp16 roundings along the way (probabilities, attention output,
      two hidden states, gate/up, activation) -> |diff| <= 1e-2 * |ref| + 1e-2 * rms(ref),
      and the rms of the difference below 3e-3 * rms(ref) (a systematic error would not hide
      there);
  everything not recomputed (resident chunks, other layers): untouched, bit for bit."""
import numpy as np
import pytest
import torch

import oracle.recompute as orc
import paper_2403_11805_amd as kvs
from paper_2403_11805_amd import binding, synth

from gpu_util import DEV

pytestmark = pytest.mark.gpu
NAN16 = 0x7e00


def close(got, ref, rtol, atol_rms, what):
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert np.all(np.isfinite(got)), f"{what}: non-finite values"
    rms = np.sqrt(np.mean(ref * ref))
    bad = np.abs(got - ref) > rtol * np.abs(ref) + atol_rms * rms
    assert not bad.any(), (f"{what}: {bad.sum()} of {bad.size} outside the bar, worst "
                           f"{np.abs(got - ref).max() / rms:.2e} rms at {np.argwhere(bad)[0]}")
    return np.sqrt(np.mean((got - ref) ** 2)) / rms


def run_case(L, Hkv, Hq, D, N, T, d_model, d_ff, layer, missing, seed, tune=False):
    shape = kvs.Shape(L, Hkv, Hq, D, N, T, 64)
    dims_o = orc.LayerDims(d_model, Hq, Hkv, D, d_ff)
    dims = binding.LayerDims(d_model, d_ff, dims_o.rope_base, dims_o.rms_eps)
    w = synth.make_layer_weights(d_model, Hq, Hkv, D, d_ff, seed)
    w_np = {k: v.numpy() for k, v in w.items()}
    x_all = synth.make_hidden(N, d_model, seed)
    k_all, v_all, y_all = orc.layer_full(x_all.numpy(), w_np, dims_o)
    rows = np.concatenate([np.arange(c * T, (c + 1) * T) for c in missing])
    # the oracle's own recompute of these chunks (the paper's procedure) from the resident K/V
    k_ref, v_ref = k_all.copy(), v_all.copy()
    k_ref[:, rows] = np.nan
    v_ref[:, rows] = np.nan
    y_ref = orc.recompute_layer(x_all.numpy()[rows], missing, T, k_ref, v_ref, w_np, dims_o)

    cache = np.full((L, 2, Hkv, N, D), 0x3c00, dtype=np.uint16)        # other layers: ones
    cache[layer, 0] = k_all.view(np.uint16)
    cache[layer, 1] = v_all.view(np.uint16)
    cache[layer, :, :, rows] = NAN16                                     # the missing chunks are gone
    before = cache.copy()
    kv_dev = torch.from_numpy(cache.view(np.int16)).to(DEV).view(torch.float16)
    x_in = x_all[rows].contiguous().to(DEV)
    x_out = torch.full_like(x_in, float("nan"))
    ws = torch.empty(kvs.kv_recompute_workspace_bytes(shape, dims, len(missing)), dtype=torch.uint8, device=DEV)
    rc = kvs.Recompute()
    w_dev = {k: v.to(DEV) for k, v in w.items()}
    if tune:        # let the GEMM library's fastest kernels run the projections: same bars
        improved = rc.tune(shape, dims, w_dev, len(missing), ws)
        assert 0 <= improved <= 5
        assert rc.tune(shape, dims, w_dev, len(missing), ws) == 0, "a tuned shape was tuned again"
    rc.layer(shape, dims, w_dev, layer,
             torch.tensor(missing, dtype=torch.int32, device=DEV), x_in, kv_dev, x_out, ws)
    torch.cuda.synchronize()
    rc.close()
    after = kv_dev.cpu().view(torch.int16).numpy().view(np.uint16)
    keep = np.ones(N, dtype=bool)
    keep[rows] = False
    assert np.array_equal(after[layer][:, :, keep], before[layer][:, :, keep]), "a resident chunk was written"
    other = [l for l in range(L) if l != layer]
    assert np.array_equal(after[other], before[other]), "another layer was written"
    k_gpu = after[layer, 0][:, rows].view(np.float16)
    v_gpu = after[layer, 1][:, rows].view(np.float16)
    close(k_gpu, k_ref[:, rows], 2e-3, 2e-3, "recomputed K")
    close(v_gpu, v_ref[:, rows], 2e-3, 2e-3, "recomputed V")
    err = close(x_out.cpu().numpy(), y_ref, 1e-2, 1e-2, "layer output")
    assert err < 3e-3, f"layer output: rms error {err:.2e} of the reference rms"
    # and the paper's claim on the GPU: the same as the whole sequence gives
    close(x_out.cpu().numpy(), y_all[rows], 1e-2, 1e-2, "layer output vs whole sequence")


@pytest.mark.parametrize("case", [
    # L, Hkv, Hq, D, N, T, d_model, d_ff, layer, missing
    (2, 2, 4, 64, 256, 16, 256, 512, 1, [2, 4, 5, 11]),          # the paper's pattern: interleaved chunks
    (1, 2, 8, 128, 104, 8, 256, 384, 0, [0, 3, 4, 9, 12]),       # four heads per kv head; M = 40, N = 104
    (1, 2, 2, 128, 384, 16, 256, 256, 0, [0, 1, 2, 5, 7, 8, 13, 20, 23]),   # five row blocks per head
    (1, 1, 2, 64, 128, 32, 128, 256, 0, [3]),                    # only the last chunk
    (1, 1, 1, 128, 96, 16, 128, 128, 0, [0, 1, 2, 3, 4, 5]),     # everything: the plain forward pass
    (1, 1, 2, 64, 128, 8, 200, 328, 0, [1, 5, 6]),               # widths that fill no GEMM tile or k-step: M = 24
    (1, 2, 4, 64, 512, 16, 264, 1096, 0, [0, 2, 3, 7, 8, 9, 12, 15, 16, 20, 21, 22, 30]),  # M = 208: two row tiles, a ragged one
])
def test_small_layers_full(case):
    run_case(*case, seed=41)


def test_llama_like_layer_sampled_positions():
    """A wider layer (d_model 1024, 8 heads of 128, 2048-token cache, 40 % of the chunks
    recomputed): the oracle's whole-sequence route is the reference."""
    run_case(1, 8, 8, 128, 2048, 16, 1024, 2816, 0,
             sorted(np.random.default_rng(7).choice(128, size=51, replace=False).tolist()), seed=43)


def test_tuned_gemm_kernels_keep_parity():
    """kv_recompute_tune picks other GEMM kernels for the projections; the layer stays within
    the same bars of the oracle (a small case and the wider one)."""
    run_case(2, 2, 4, 64, 256, 16, 256, 512, 1, [2, 4, 5, 11], seed=41, tune=True)
    run_case(1, 8, 8, 128, 2048, 16, 1024, 2816, 0,
             sorted(np.random.default_rng(7).choice(128, size=51, replace=False).tolist()), seed=43, tune=True)


def test_own_gemm_kernel_at_every_size(monkeypatch):
    """Without the GEMM library (switched off through the environment) the projections of the
    816-row case run on the library's own kernel as well: same bars."""
    monkeypatch.setenv("KVSWITCH_OWN_GEMM", "1")
    run_case(1, 8, 8, 128, 2048, 16, 1024, 2816, 0,
             sorted(np.random.default_rng(7).choice(128, size=51, replace=False).tolist()), seed=43)


def test_long_cache_positions_near_32768():
    """Chunks at the start, the middle and the very end of a 32768-token cache (one kv head, four
    query heads): rotary angles of tens of thousands of radians and attention over the whole
    cache.  The resident K/V are seeded random values; the oracle's recompute procedure is the
    reference."""
    L, Hkv, Hq, D, N, T, d_model, d_ff = 1, 1, 4, 128, 32768, 32, 512, 1024
    missing = [0, 511, 1022, 1023]
    shape = kvs.Shape(L, Hkv, Hq, D, N, T, 128)
    dims_o = orc.LayerDims(d_model, Hq, Hkv, D, d_ff)
    dims = binding.LayerDims(d_model, d_ff, dims_o.rope_base, dims_o.rms_eps)
    w = synth.make_layer_weights(d_model, Hq, Hkv, D, d_ff, 47)
    w_np = {k: v.numpy() for k, v in w.items()}
    kv = synth.make_kv(synth.Geometry(L, Hkv, Hq, D, N, T, 128), 47, "cpu")
    rows = np.concatenate([np.arange(c * T, (c + 1) * T) for c in missing])
    x = synth.make_hidden(len(rows), d_model, 47)
    k_ref, v_ref = kv[0, 0].numpy().copy(), kv[0, 1].numpy().copy()
    y_ref = orc.recompute_layer(x.numpy(), missing, T, k_ref, v_ref, w_np, dims_o)
    kv_dev = kv.to(DEV)
    x_out = torch.full((len(rows), d_model), float("nan"), dtype=torch.float16, device=DEV)
    ws = torch.empty(kvs.kv_recompute_workspace_bytes(shape, dims, len(missing)), dtype=torch.uint8, device=DEV)
    rc = kvs.Recompute()
    rc.layer(shape, dims, {k: v.to(DEV) for k, v in w.items()}, 0,
             torch.tensor(missing, dtype=torch.int32, device=DEV), x.to(DEV), kv_dev, x_out, ws)
    torch.cuda.synchronize()
    # twice: identical bytes
    x_out2 = torch.empty_like(x_out)
    kv_dev2 = kv.to(DEV)
    rc.layer(shape, dims, {k: v.to(DEV) for k, v in w.items()}, 0,
             torch.tensor(missing, dtype=torch.int32, device=DEV), x.to(DEV), kv_dev2, x_out2, ws)
    torch.cuda.synchronize()
    rc.close()
    assert torch.equal(x_out.view(torch.int16), x_out2.view(torch.int16))
    assert torch.equal(kv_dev.view(torch.int16), kv_dev2.view(torch.int16))
    got = kv_dev.cpu().numpy()
    close(got[0, 0][:, rows], k_ref[:, rows], 2e-3, 2e-3, "recomputed K")
    close(got[0, 1][:, rows], v_ref[:, rows], 2e-3, 2e-3, "recomputed V")
    keep = np.ones(N, dtype=bool)
    keep[rows] = False
    assert np.array_equal(got[0][:, :, keep].view(np.uint16), kv[0].numpy()[:, :, keep].view(np.uint16))
    err = close(x_out.cpu().numpy(), y_ref, 1e-2, 1e-2, "layer output")
    assert err < 3e-3


def test_layer_chain_replayed_from_a_hip_graph():
    """kv_recompute_layer allocates nothing and never synchronises, the GEMM library included: two
    chained layers captured in a HIP graph give, on every replay, the bits of the eager run."""
    L, Hkv, Hq, D, N, T, d_model, d_ff = 2, 2, 4, 128, 512, 16, 512, 1024
    shape = kvs.Shape(L, Hkv, Hq, D, N, T, 64)
    dims = binding.LayerDims(d_model, d_ff)
    w = [{k: v.to(DEV) for k, v in synth.make_layer_weights(d_model, Hq, Hkv, D, d_ff, 53, layer=l).items()}
         for l in range(L)]
    missing = [1, 2, 9, 30]
    idx = torch.tensor(missing, dtype=torch.int32, device=DEV)
    kv0 = synth.make_kv(synth.Geometry(L, Hkv, Hq, D, N, T, 64), 53, DEV)
    kv = kv0.clone()
    x0 = synth.make_hidden(len(missing) * T, d_model, 53, DEV)
    hid = [torch.empty_like(x0), torch.empty_like(x0)]
    ws = torch.empty(kvs.kv_recompute_workspace_bytes(shape, dims, len(missing)), dtype=torch.uint8, device=DEV)
    rc = kvs.Recompute()

    def chain():
        for l in range(L):
            rc.layer(shape, dims, w[l], l, idx, x0 if l == 0 else hid[l & 1], kv, hid[(l + 1) & 1], ws)

    chain()
    torch.cuda.synchronize()
    y_ref, kv_ref = hid[L & 1].clone(), kv.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        chain()                                     # warm-up on the capture stream
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        chain()
    for rep in range(3):
        kv.copy_(kv0)
        hid[0].zero_(); hid[1].zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(hid[L & 1].view(torch.int16), y_ref.view(torch.int16)), f"replay {rep}: output differs"
        assert torch.equal(kv.view(torch.int16), kv_ref.view(torch.int16)), f"replay {rep}: cache differs"
    rc.close()

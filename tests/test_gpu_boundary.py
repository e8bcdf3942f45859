"""GPU tests of the boundary itself: dtypes, caller streams, counts derived from p and alpha."""
import numpy as np
import pytest

from oracle import thanos_oracle as orc
from synth import LayerSpec, make_weight, make_calibration

pytestmark = pytest.mark.gpu


def _layer(c, b, T, seed, dtype="f32"):
    spec = LayerSpec("bd", c=c, b=b, tokens=T, dtype=dtype, rho=0.7, k_mix=16, seed=seed)
    return make_weight(spec), make_calibration(spec)


def _prune_torch(Wd, Hd, o, stream=None, cast=True):
    import torch
    import paper_2504_05346_amd as th
    c, b = Wd.shape
    ws = torch.empty((th.thanos_prune_workspace_bytes(c, b, o),), dtype=torch.uint8, device="cuda")
    Wo = torch.empty((c, b), dtype=torch.float32, device="cuda")
    Wc = torch.empty((c, b), dtype=Wd.dtype, device="cuda") if cast else None
    M = torch.empty((c, b), dtype=torch.uint8, device="cuda")
    info = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    th.thanos_prune_layer(Wd, Hd, o, Wo, Wc, M, ws, info, stream=stream)
    return Wo, Wc, M, info, ws


@pytest.mark.parametrize("mode", ["nm", "unstructured"])
def test_bf16_weights(mode):
    """bf16 weights in, bf16 cast out: the oracle gets the same bf16 values, exactly converted."""
    import torch
    import paper_2504_05346_amd as th
    W32, X = _layer(192, 384, 1536, seed=21)
    Wd = torch.from_numpy(W32).cuda().to(torch.bfloat16)
    W = Wd.float().cpu().numpy().astype(np.float64)            # the bf16 values, exact
    H = orc.hessian(X)
    Hd = torch.from_numpy(H.astype(np.float32)).cuda()
    H = Hd.cpu().numpy().astype(np.float64)
    o = th.PruneOpts(mode=th.THANOS_NM if mode == "nm" else th.THANOS_UNSTRUCTURED, sparsity=0.5,
                     n=2, m=4, block_size=128, damping=0.01)
    print(f"bf16 weights {mode}", flush=True)
    Wo, Wc, M, info, _ = _prune_torch(Wd, Hd, o)
    torch.cuda.synchronize()
    assert int(info.item()) == 0
    Mg = M.cpu().numpy()
    Wg = Wo.cpu().numpy().astype(np.float64)
    # bf16 weights have 8 significant bits: equal metrics are common, so the comparison runs
    # under the GPU's own mask after checking that it differs from the oracle's only at ties
    Wr, Mr = orc.prune_fast(W, H, mode=mode, p=0.5, n=2, m=4, B=128, damp=0.01)
    assert (Mg != Mr).mean() < 2e-3
    Wt, _ = orc.prune_fast(W, H, mode=mode, p=0.5, n=2, m=4, B=128, damp=0.01, mask_in=Mg)
    assert np.linalg.norm(Wg - Wt) <= 1e-3 * np.linalg.norm(Wt)
    assert np.all(Wg[Mg == 1] == 0.0)
    if mode == "unstructured":
        assert int(Mg.sum()) == 192 * 384 // 2
    else:
        assert np.all(Mg.reshape(192, -1, 4).sum(axis=2) == 2)
    # the cast copy is the fp32 result rounded to nearest-even bf16
    assert Wc.dtype == torch.bfloat16
    assert torch.equal(Wc, Wo.to(torch.bfloat16))


def test_call_on_a_non_default_stream():
    """Everything (accumulate, factor, sweep, helper streams of the call) is ordered on the
    stream that is passed in: inputs produced on that stream just before the call, outputs read
    on it just after, no synchronisation with the default stream in between."""
    import torch
    import paper_2504_05346_amd as th
    W, X = _layer(256, 1280, 2048, seed=22, dtype="f16")      # 10 blocks: two super-blocks
    c, b = W.shape
    Wh, Xh = torch.from_numpy(W).pin_memory(), torch.from_numpy(X).pin_memory()
    o = th.PruneOpts(mode=th.THANOS_NM, sparsity=0.0, n=2, m=4, block_size=128, damping=0.01)
    ref = None
    for use_side in (False, True):
        s = torch.cuda.Stream() if use_side else torch.cuda.current_stream()
        with torch.cuda.stream(s):
            Wd = Wh.to("cuda", non_blocking=True)
            Xd = Xh.to("cuda", non_blocking=True)
            H = torch.zeros((b, b), dtype=torch.float32, device="cuda")
            th.thanos_hessian_accumulate(H, Xd[:1024], stream=s)
            th.thanos_hessian_accumulate(H, Xd[1024:], stream=s)
            Wo, Wc, M, info, ws = _prune_torch(Wd, H, o, stream=s)
            out = (Wo.to("cpu", non_blocking=True), M.to("cpu", non_blocking=True),
                   info.to("cpu", non_blocking=True))
        s.synchronize()
        assert int(out[2].item()) == 0
        if ref is None:
            ref = (out[0].numpy().copy(), out[1].numpy().copy())
        else:
            np.testing.assert_array_equal(out[1].numpy(), ref[1])
            # the Hessian's token chunks are summed with atomics (last bits vary), so W_hat is
            # compared to the bar, not bit for bit
            assert np.linalg.norm(out[0].numpy().astype(np.float64) - ref[0]) <= \
                1e-4 * np.linalg.norm(ref[0])
    Hh = orc.hessian(X)
    Wr, Mr = orc.prune_fast(W, Hh, mode="nm", n=2, m=4, B=128, damp=0.01, mask_in=ref[1])
    assert np.linalg.norm(ref[0] - Wr) <= 1e-3 * np.linalg.norm(Wr)
    _, Mfree = orc.prune_fast(W, Hh, mode="nm", n=2, m=4, B=128, damp=0.01)
    assert (Mfree != ref[1]).mean() < 1e-3


@pytest.mark.parametrize("p,c,b", [(0.3333333, 1, 3), (0.33333334, 1, 3), (0.6, 5, 2), (0.7, 2, 5),
                                   (0.1, 10, 3), (0.29, 10, 10), (0.57, 100, 1), (0.999, 7, 13),
                                   (0.0, 4, 8), (1e-9, 64, 128)])
def test_number_removed_is_floor_of_the_decimal_product(p, c, b):
    """r = floor(p c b) on the decimal value of p (0.6 is 6/10): the library's count equals the
    oracle's exact rational evaluation, also where p c b lands on or next to an integer."""
    import torch
    import paper_2504_05346_amd as th
    g = np.random.default_rng(5)
    W = g.standard_normal((c, b)).astype(np.float32)
    X = g.standard_normal((4 * b + 8, b)).astype(np.float32)
    H = (X.T @ X).astype(np.float32)
    o = th.PruneOpts(mode=th.THANOS_UNSTRUCTURED, sparsity=p, n=0, m=0, block_size=4, damping=0.01)
    Wo, _, M, info, _ = _prune_torch(torch.from_numpy(W).cuda(), torch.from_numpy(H).cuda(), o,
                                     cast=False)
    torch.cuda.synchronize()
    assert int(info.item()) == 0
    assert int(M.sum().item()) == orc.num_to_remove(p, c, b)


@pytest.mark.parametrize("alpha,c", [(0.1, 10), (0.1, 11), (0.3, 10), (0.0999999, 10), (0.07, 100),
                                     (0.15, 20)])
def test_outlier_row_count_is_ceil_of_the_decimal_product(alpha, c):
    import torch
    import paper_2504_05346_amd as th
    b = 16
    g = np.random.default_rng(6)
    W = g.standard_normal((c, b)).astype(np.float32)
    X = g.standard_normal((128, b)).astype(np.float32)
    H = (X.T @ X).astype(np.float32)
    o = th.PruneOpts(mode=th.THANOS_NM, sparsity=0.0, n=2, m=4, block_size=8, damping=0.01,
                     outlier_fraction=alpha)
    _, _, M, info, _ = _prune_torch(torch.from_numpy(W).cuda(), torch.from_numpy(H).cuda(), o,
                                    cast=False)
    torch.cuda.synchronize()
    assert int(info.item()) == 0
    untouched = int((M.sum(dim=1) == 0).sum().item())
    assert untouched == orc.num_outlier_rows(alpha, c)


@pytest.mark.parametrize("mode", ["nm", "unstructured"])
def test_diagnostic_phase_timing_gives_the_same_result(mode):
    """opts.phase_ms_out: kernels serialised on the stream and timed per phase by the library;
    masks and W_hat are those of the normal call, every phase that runs reports a time."""
    import ctypes
    import torch
    import paper_2504_05346_amd as th
    W, X = _layer(256, 1280, 2048, seed=23, dtype="f16")
    Wd = torch.from_numpy(W).cuda()
    H = torch.from_numpy(orc.hessian(X).astype(np.float32)).cuda()
    o = th.PruneOpts(mode=th.THANOS_NM if mode == "nm" else th.THANOS_UNSTRUCTURED, sparsity=0.5,
                     n=2, m=4, block_size=128, damping=0.01)
    Wo, Wc, M, info, _ = _prune_torch(Wd, H, o)
    torch.cuda.synchronize()
    buf = (ctypes.c_float * len(th.THANOS_PHASES))(*([-1.0] * len(th.THANOS_PHASES)))
    o.phase_ms_out = ctypes.addressof(buf)
    Wo2, Wc2, M2, info2, _ = _prune_torch(Wd, H, o)
    torch.cuda.synchronize()
    assert int(info.item()) == 0 and int(info2.item()) == 0
    assert torch.equal(M, M2) and torch.equal(Wo, Wo2) and torch.equal(Wc, Wc2)
    ph = dict(zip(th.THANOS_PHASES, list(buf)))
    print(f"phases {mode}: {ph}", flush=True)
    for k in ("prep", "factor", "solve", "update", "finalise"):
        assert 0.0 < ph[k] < 1000.0, (k, ph)
    assert (ph["mask"] > 0.0) == (mode == "unstructured")
    # the no-allocation entry point refuses the diagnostic mode (it would create events)
    st = th.lib().thanos_prune_layer_noalloc(Wd.data_ptr(), th.THANOS_F16, 256, 1280, H.data_ptr(),
                                             ctypes.byref(o), Wo2.data_ptr(), None, M2.data_ptr(),
                                             info2.data_ptr(), None)
    assert st == 2


@pytest.mark.parametrize("mode", ["unstructured", "nm"])
def test_two_calls_on_two_streams_at_once(mode):
    """Two sweeps enqueued back to back on two streams (own buffers and workspaces each) run side
    by side on the device -- helper streams from the pool, and for the unstructured mode two
    selection kernels whose workgroups wait for each other inside the launch -- and give what
    each gives alone."""
    import torch
    import paper_2504_05346_amd as th
    layers = []
    for k, (c, b) in enumerate([(512, 1536), (384, 2048)]):
        W, X = _layer(c, b, 2048, seed=30 + k, dtype="f16")
        Wd = torch.from_numpy(W).cuda()
        H = torch.from_numpy(orc.hessian(X).astype(np.float32)).cuda()
        layers.append((Wd, H))
    o = th.PruneOpts(mode=th.THANOS_NM if mode == "nm" else th.THANOS_UNSTRUCTURED, sparsity=0.5,
                     n=2, m=4, block_size=128, damping=0.01)
    alone = []
    for Wd, H in layers:
        Wo, _, M, info, _ = _prune_torch(Wd, H, o, cast=False)
        torch.cuda.synchronize()
        assert int(info.item()) == 0
        alone.append((Wo.clone(), M.clone()))
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    outs = []
    for rep in range(3):
        outs.clear()
        for (Wd, H), s in zip(layers, streams):
            with torch.cuda.stream(s):
                outs.append(_prune_torch(Wd, H, o, stream=s, cast=False))
        for s in streams:
            s.synchronize()
        for (Wo, _, M, info, _), (Wa, Ma) in zip(outs, alone):
            assert int(info.item()) == 0
            assert torch.equal(M, Ma) and torch.equal(Wo, Wa)

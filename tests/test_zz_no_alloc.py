"""bwla_decode_forward_static (the entry point that allocates nothing) against bwla_decode_forward,
through the C ABI: two calls in a row on one GPU, the second with a smaller input, so that the
second call finds the first call's contents in the library's scratch array."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2605_00422_amd import inputs as syn  # noqa: E402

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2605_00422_amd import binding as B
    B.load()


def _layer(cfg):
    from paper_2605_00422_amd import binding as B
    d = syn.make_layer(cfg)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    layer = B.pack_weights(t(d.W), t(d.R1), t(d.R2), t(d.U) if cfg.r else None, t(d.V) if cfg.r else None,
                           cfg.n1, cfg.n2)
    X = t(d.X).to(torch.bfloat16) if cfg.x_dtype == "bf16" else t(d.X)
    return layer, X


def _both(layer, X, cfg):
    """(outputs of the existing entry point, outputs of the allocation-free one)."""
    from paper_2605_00422_amd import binding as B
    outs = []
    for static in (False, True):
        act = B.Activations(layer, cfg.M)
        for tns in (act.q, act.scale, act.qsum) + ((act.T,) if act.T is not None else ()):
            tns.fill_(1)                                # whatever the call leaves unwritten would show
        Y = torch.full((cfg.M, cfg.N), float("nan"), dtype=torch.float32, device=DEV)
        acc = torch.full((cfg.M, cfg.N), -7, dtype=torch.int32, device=DEV)
        (B.decode_forward_static if static else B.decode_forward)(layer, X, act, Y, acc)
        torch.cuda.synchronize()
        outs.append((act.q.clone(), act.scale.clone(), act.qsum.clone(),
                     None if act.T is None else act.T.clone(), Y, acc))
    return outs


def _same(a, b, what):
    for x, y, name in zip(a, b, ("codes", "scales", "code sums", "T", "Y", "accumulators")):
        if x is None:
            assert y is None
            continue
        # integer outputs bit for bit; the kernels are the same and deterministic, so the floats too
        assert torch.equal(x, y), f"{what}: {name} differ"
    assert bool(torch.isfinite(a[4]).all())


def test_static_scratch_call_matches_the_workspace_call_twice_in_a_row():
    # first the larger input: sixteen tokens, split projection (ten slices x two rank groups) ...
    big = syn.LayerConfig("noalloc_big", 16, 5120, 64, 80, 3000, 64, "bf16", 51, 50.0, seed=21)
    # ... then a smaller one: one token, eight slices; its partial tiles land where the first call's were
    small = syn.LayerConfig("noalloc_small", 1, 4096, 64, 64, 1200, 32, "bf16", 4, 20.0, seed=22)
    # and a few tokens of a layer with a large factor: rotation in two launches, rotated values in scratch
    split = syn.LayerConfig("noalloc_split", 2, 16896, 176, 96, 96, 8, "bf16", 8, 20.0, seed=23)
    from paper_2605_00422_amd import binding as B
    for cfg in (big, small, split, small):
        layer, X = _layer(cfg)
        assert 0 < B.psp_workspace_size(layer, cfg.M) <= (4 << 20)
        ref, got = _both(layer, X, cfg)
        _same(ref, got, cfg.name)


def test_static_scratch_call_refuses_what_does_not_fit():
    from ctypes import byref, c_void_p
    from paper_2605_00422_amd import binding as B
    cfg = syn.LayerConfig("noalloc_refused", 1, 4096, 64, 64, 256, 32, "bf16", 4, 20.0, seed=24)
    layer, X = _layer(cfg)
    M = 4096                                            # a prefill: its projection wants megabytes of partial sums
    assert B.psp_workspace_size(layer, M) > (4 << 20)
    p = c_void_p(X.data_ptr())                          # never dereferenced: the size check comes first
    st = B.load().bwla_decode_forward_static(byref(layer.desc), p, B.BWLA_X_BF16, M, p, p, p, p, p, None, None)
    assert st == B.BWLA_ERR_BUFSIZE

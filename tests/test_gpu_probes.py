"""The library's measurement aids and the launch-count query on the GPU (run with -m gpu): the
probes run, refuse what their header says they refuse, and the query names the single-launch
kernel exactly for the shapes bwla_decode_forward's description lists."""
import dataclasses

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2605_00422_amd import inputs as syn  # noqa: E402

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2605_00422_amd import binding as B
    B.load()


def test_probes_run_and_refuse():
    from paper_2605_00422_amd import binding as B
    sink = torch.zeros(16384, dtype=torch.int32, device="cuda:0")
    src = torch.arange(1 << 20, dtype=torch.int32, device="cuda:0")
    B.probe_hbm_read(src, sink)
    torch.cuda.synchronize()
    # the xor of all words of the buffer, folded over the workgroups' checksums
    got = 0
    for w in sink.cpu().numpy().tolist():
        got ^= w & 0xFFFFFFFF
    x = src.cpu().numpy()
    want = int(np.bitwise_xor.reduce(x.view(np.uint32)))
    assert got == want
    ops = B.probe_mfma_int8(100, sink)
    torch.cuda.synchronize()
    assert ops > 0 and ops % (2 * 16 * 16 * 64 * 4 * 100) == 0
    with pytest.raises(B.BwlaError):
        B.probe_hbm_read(src[:3], sink)            # 12 bytes: not a multiple of 16
    with pytest.raises(B.BwlaError):
        B.probe_mfma_int8(0, sink)
    with pytest.raises(B.BwlaError):
        B.probe_mfma_int8(10, sink[:16])           # sink too small


def test_latency_probes_run_and_refuse():
    from paper_2605_00422_amd import binding as B
    B.probe_empty_launch()
    buf = torch.zeros(1 << 18, dtype=torch.int32, device="cuda:0")          # 1 MiB of even words: stride exact
    out = torch.zeros(2, dtype=torch.int64, device="cuda:0")
    B.probe_load_latency(buf, 128, 1000, out)
    torch.cuda.synchronize()
    ticks, idx = out.cpu().numpy().tolist()
    assert idx == (1000 * 32) % (1 << 18)                                    # 1000 steps of 32 words
    assert 1000 * 5 <= ticks * 10 <= 1000 * 20000                            # 5 ns .. 20 us per load
    odd = torch.ones(1 << 10, dtype=torch.int32, device="cuda:0")           # odd words: one word further each time
    B.probe_load_latency(odd, 64, 10, out)
    torch.cuda.synchronize()
    assert out[1].item() == (10 * 17) % (1 << 10)
    with pytest.raises(B.BwlaError):
        B.probe_load_latency(buf, 0, 10, out)
    with pytest.raises(B.BwlaError):
        B.probe_load_latency(buf, 4 << 20, 10, out)                          # stride beyond the buffer
    with pytest.raises(B.BwlaError):
        B.probe_load_latency(buf, 128, 0, out)


def test_clock_probe_brackets_work_on_the_stream():
    """Two clock launches around a known amount of GPU work: the counter advances, at 100 MHz, by about
    what events measure for the same span; also from a captured graph, on every replay."""
    from paper_2605_00422_amd import binding as B
    t0 = torch.zeros(1, dtype=torch.int64, device="cuda:0")
    t1 = torch.zeros(1, dtype=torch.int64, device="cuda:0")
    big = torch.zeros(64 << 20, dtype=torch.int32, device="cuda:0")

    def span():
        B.probe_clock(t0)
        big.add_(1)                                  # 512 MB of traffic: some tens of microseconds at least
        B.probe_clock(t1)

    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    span()
    torch.cuda.synchronize()
    e0.record()
    span()
    e1.record()
    torch.cuda.synchronize()
    us_clock = (t1.item() - t0.item()) / 100.0
    us_events = e0.elapsed_time(e1) * 1e3
    assert 20.0 < us_clock <= us_events * 1.05 + 5.0, (us_clock, us_events)
    assert us_clock > 0.5 * us_events - 20.0, (us_clock, us_events)
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            span()
    seen = []
    for _ in range(3):
        g.replay()
        torch.cuda.synchronize()
        seen.append((t0.item(), t1.item()))
    assert all(b > a for a, b in seen) and seen[0][1] < seen[1][0] < seen[1][1] < seen[2][0]
    with pytest.raises(B.BwlaError):
        B.probe_clock(None)


def test_launch_count_query():
    from paper_2605_00422_amd import binding as B
    from parity_util import pack_on_gpu
    small = dataclasses.replace(syn.CONFIGS["cfg1_decode7b"], N=1024)
    layer = pack_on_gpu(syn.make_layer(small, with_activations=False))
    assert B.decode_forward_launches(layer, 1, bf16=True) == 1
    assert B.decode_forward_launches(layer, 1, bf16=False) == 2      # fp32 activations
    assert B.decode_forward_launches(layer, 2, bf16=True) == 2       # more than one token
    c0 = syn.CONFIGS["cfg0_tiny"]                                     # 16 x 32 factors
    l0 = pack_on_gpu(syn.make_layer(c0, with_activations=False))
    assert B.decode_forward_launches(l0, 1, bf16=True) == 2

"""GPU parity of the HIP path against the CPU oracle, through the C ABI (run with -m gpu)."""
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
    B.load()   # raises when the HIP library is missing: there is no fallback path


def _sample_rows(M, n=64, seed=0):
    rng = np.random.default_rng(seed)
    rows = set(rng.choice(M, size=min(n, M), replace=False).tolist()) | {0, M - 1}
    return np.array(sorted(rows))


def test_cfg0_tiny():
    from parity_util import run_case
    print(run_case(syn.CONFIGS["cfg0_tiny"]), flush=True)


def test_cfg1_decode7b():
    from parity_util import run_case
    print(run_case(syn.CONFIGS["cfg1_decode7b"]), flush=True)


def test_cfg2_qwen32b_up_m16():
    from parity_util import run_case
    print(run_case(syn.CONFIGS["cfg2_qwen32b_up_m16"]), flush=True)


def test_cfg3_qwen32b_down_prefill_sampled_rows():
    """Full M = 2048 on the GPU in the benchmarked launch configuration; the oracle checks 64
    seeded token rows plus the first and the last (tokens are independent)."""
    from parity_util import run_case
    cfg = syn.CONFIGS["cfg3_qwen32b_down_m2048"]
    print(run_case(cfg, rows=_sample_rows(cfg.M)), flush=True)


@pytest.mark.parametrize("M", [1, 64])
@pytest.mark.parametrize("which", ["k", "o", "gate", "down"])
def test_cfg4_70b_block_small_m(which, M):
    """The block's four distinct layer shapes (q = o, v = k, up = gate) at one and at 64 tokens."""
    from parity_util import run_case
    cfg = {c.name.split("_")[2]: c for c in syn.block70b_configs(M)}[which]
    rows = None if which != "gate" or M == 1 else _sample_rows(M, 16)   # (oracle time: 28672 channels)
    print(run_case(cfg, rows=rows), flush=True)


@pytest.mark.parametrize("which", ["qkv", "gateup"])
def test_cfg1_7b_merged_projections(which):
    """Projections that read the same activations, packed as one layer (N = 12288, r = 96; N = 22016, r = 64)."""
    from parity_util import run_case
    cfg = {c.name.split("_")[2]: c for c in syn.block7b_configs(1)}[which]
    print(run_case(cfg), flush=True)


def test_looping_rotation_two_tokens_at_a_time_odd_count():
    """Large resident factors, M >= 512: a workgroup rotates two tokens at a time; with an odd
    number of tokens the last pair is half empty."""
    from parity_util import run_case
    cfg = syn.LayerConfig("dual_515", 515, 8192, 128, 64, 48, 8, "bf16", 80, 20.0, seed=13)
    print(run_case(cfg, rows=[0, 1, 2, 3, 255, 256, 257, 510, 511, 512, 513, 514]), flush=True)


def test_looping_rotation_two_tokens_at_a_time_fewer_pairs_than_cus():
    """Between one and two tokens per CU: fewer workgroups than CUs, one round of two tokens each."""
    from parity_util import run_case
    cfg = syn.LayerConfig("dual_301", 301, 8192, 128, 64, 48, 8, "bf16", 80, 20.0, seed=14)
    print(run_case(cfg, rows=[0, 1, 2, 149, 150, 151, 298, 299, 300]), flush=True)


@pytest.mark.parametrize("M,K,n1,n2,N,r,bits,centered", [
    (2085, 4096, 64, 64, 48, 8, 6, False),     # four tokens at a time per workgroup, three rounds, the last one ragged
    (520, 25600, 160, 160, 64, 16, 6, False),  # ten strips, one token at a time, third round with eight workgroups
    (600, 4096, 64, 64, 40, 8, 8, False),      # 8-bit codes
    (515, 8192, 128, 64, 40, 8, 6, True),      # row shift: the shift entry of T from the looping kernel
    (512, 2048, 32, 64, 40, 0, 6, False),      # exactly two tokens per CU, no low-rank part: no kernel built, the older path
    (530, 28672, 224, 128, 40, 8, 6, False),   # R1 too large for LDS: its terms streamed step by step, seven steps (odd: buffers swap roles per token)
])
def test_resident_factor_rotation_many_tokens(M, K, n1, n2, N, r, bits, centered):
    """At least two bf16 tokens per CU and factors whose operand-order planes fit LDS: the looping
    rotation kernel with resident factors (two-term fp16 operands)."""
    from parity_util import run_case
    cfg = syn.LayerConfig(f"planes_{M}_{K}_{bits}", M, K, n1, n2, N, r, "bf16", max(1, K // 100), 20.0, seed=21)
    rows = sorted(set(_sample_rows(M, 40, seed=3).tolist()) | {M - 2, M // 2})
    print(run_case(cfg, rows=rows, centered=centered, act_bits=bits), flush=True)


@pytest.mark.parametrize("which", ["q", "k", "gate", "down"])
def test_cfg4_70b_block_m4096_sampled_rows(which):
    """The block's four distinct shapes at 4096 tokens, full size on the GPU in the benchmarked
    launch configuration; the oracle checks a seeded sample of token rows plus the first and last."""
    from parity_util import run_case
    cfg = {c.name.split("_")[2]: c for c in syn.block70b_configs(4096)}[which]
    print(run_case(cfg, rows=_sample_rows(cfg.M, 32 if which in ("gate", "down") else 48)), flush=True)


@pytest.mark.parametrize("M,K,n1,n2,N,r,xd", [
    (1, 96, 12, 8, 40, 0, "f32"),        # rank 0, ragged N, single partly filled chunk
    (5, 96, 8, 12, 33, 8, "bf16"),       # factors not multiples of 16
    (16, 1024, 32, 32, 100, 20, "bf16"), # rank not a multiple of 16, N not a multiple of 4... of 16
    (17, 512, 16, 32, 130, 8, "f32"),    # just past the decode batch: tiled kernel with a ragged tile
    (33, 640, 20, 32, 257, 64, "bf16"),  # ragged in every dimension
    (200, 2048, 32, 64, 300, 32, "bf16"),
    (3, 11008, 128, 86, 64, 16, "bf16"), # 7B down-projection width: n2 = 86, K not a multiple of 512
    (300, 1152, 36, 32, 200, 20, "bf16"),  # streaming GEMM: ragged token and channel tiles, 9 slices
    (257, 256, 16, 16, 48, 5, "f32"),      # streaming GEMM: two slices, odd rank, N < one tile, fp32 input
    (520, 640, 20, 32, 330, 0, "bf16"),    # streaming GEMM without a low-rank branch
    (40, 480, 20, 24, 70, 8, "bf16"),      # K not a multiple of 128: LDS-tiled GEMM, 64 x 128 tiles
    (150, 160, 16, 10, 24, 4, "f32"),      # fewer than 32 channels: LDS-tiled GEMM, 128 x 128 tiles
    (33, 256, 16, 16, 8800, 8, "bf16"),    # streaming GEMM, 275 tiles of 64 x 32: 64 x 64 tiles shared by four wavefronts
    (20, 256, 16, 16, 16672, 0, "bf16"),   # streaming GEMM, 521 tiles: one wavefront per tile
    # rows longer than 8192 columns at decode: four chunks per compute wavefront
    (1, 11008, 128, 86, 1000, 32, "bf16"),  # 7B down-projection shape: 22 chunks, six compute wavefronts
    (8, 12288, 128, 96, 520, 0, "bf16"),    # 24 chunks, eight tokens, no low-rank part
    (2, 14336, 128, 112, 200, 48, "bf16"),  # the longest row this variant takes: 28 chunks, seven compute wavefronts
    # rows longer than 14336 columns at decode: several passes of 28 chunks in one launch
    (1, 28672, 224, 128, 300, 32, "bf16"),  # 70B down-projection width: two full passes
    (16, 27648, 216, 128, 200, 16, "bf16"), # 32B down-projection width, sixteen tokens: 54 chunks, 28 + 26
    (4, 30976, 176, 176, 9000, 8, "bf16"),  # three passes (28, 28, 5 chunks, the last partly filled), three channel tiles per workgroup
    # one token without low-rank part: bwla_decode_forward runs its single-launch kernel
    (1, 4096, 64, 64, 4096, 0, "bf16"),    # 7B attention projection shape, one channel tile per workgroup
    (1, 4096, 64, 64, 11008, 0, "bf16"),   # 7B gate/up shape: up to three channel tiles per workgroup
    (1, 2048, 32, 64, 333, 0, "bf16"),     # ragged N (scalar stores), two compute wavefronts
    (1, 1536, 48, 32, 1000, 0, "bf16"),    # two rotation strips, odd chunk count, last tile ragged
    (1, 4096, 128, 32, 520, 0, "bf16"),    # eight tiles along n1
    (1, 4096, 64, 64, 1040, 96, "bf16"),   # single-launch kernel at its largest rank (six 16-column tiles of U)
    (1, 4096, 64, 64, 2000, 70, "bf16"),   # five rank tiles, the last partly filled
    # few tokens, R1 too large for LDS: rotation split over several workgroups + quantizing launch
    (3, 16896, 176, 96, 80, 8, "bf16"),    # odd number of tiles along n1: the last slice has one tile
    (2, 20000, 200, 100, 48, 0, "bf16"),   # ragged n1 and n2 (strips and tiles partly filled), r = 0
    (1, 9600, 128, 75, 64, 8, "bf16"),     # resident factors, long stage: split too; odd n2 (2-byte token loads)
    (2, 25600, 160, 160, 100, 16, "bf16"), # ten strips: 640-thread workgroups, ten slices per token
    (5, 8192, 128, 64, 300, 24, "bf16"),   # resident factors, up to eight tokens: split (40 rotation workgroups + projection)
    # projection of more than two 16-column rank tiles: dealt to several workgroups per slice
    (7, 1024, 32, 32, 100, 40, "f32"),     # fp32 activations, two slices, three rank tiles in two groups
    (3, 512, 16, 32, 64, 48, "bf16"),      # a single slice: the groups write T themselves
    (12, 4096, 64, 64, 200, 128, "bf16"),  # the largest rank: four groups of two tiles
    (20, 28672, 224, 128, 64, 40, "bf16"), # two token tiles, more workgroups than CUs (280 rotation + 224 projection)
])
def test_ragged_and_degenerate_shapes(M, K, n1, n2, N, r, xd):
    from parity_util import run_case
    cfg = syn.LayerConfig(f"edge_{M}_{K}_{N}_{r}", M, K, n1, n2, N, r, xd, max(1, K // 100), 20.0, seed=11)
    print(run_case(cfg), flush=True)


@pytest.mark.parametrize("M,K,n1,n2,N,r,xd", [
    (16, 512, 16, 32, 512, 8, "f32"),        # fp32 activations (old rotation kernel), decode GEMM
    (1, 4096, 64, 64, 1000, 32, "bf16"),     # one token: merged projection, shift entry from the bf16 rotation
    (1, 4096, 64, 64, 528, 0, "bf16"),       # no PSP at all: the shift is the only column of T and V
    (1, 4096, 64, 64, 1536, 96, "bf16"),     # single-launch kernel, rank 96 + the shift column: seven tiles of V
    (16, 5120, 64, 80, 640, 15, "bf16"),     # r + 1 = 16 fills the padded rank exactly
    (40, 1024, 32, 32, 200, 16, "bf16"),     # r + 1 = 17 crosses into the next 16-column group; streaming GEMM, 4 waves split K
    (300, 1152, 36, 32, 200, 20, "bf16"),    # prefill: separate projection kernel writes T with the wider pitch
    (2, 20000, 200, 100, 48, 4, "bf16"),     # split rotation: shift entries from the extra small launch
])
def test_row_shift_binarization(M, K, n1, n2, N, r, xd):
    """Layers packed with bwla_pack_weights_centered (paper Sec. 3 "Discussion", Eq. 1-2, 4)."""
    from parity_util import run_case
    cfg = syn.LayerConfig(f"shift_{M}_{K}_{N}_{r}", M, K, n1, n2, N, r, xd, max(1, K // 100), 20.0, seed=12)
    print(run_case(cfg, centered=True), flush=True)


@pytest.mark.parametrize("bits,M,K,n1,n2,N,r,xd", [
    (8, 1, 4096, 64, 64, 1000, 32, "bf16"),    # W1A8, the width of the paper's speed run: decode
    (8, 16, 512, 16, 32, 512, 8, "f32"),       # fp32 activations (old rotation kernel)
    (8, 300, 1152, 36, 32, 200, 20, "bf16"),   # prefill: accumulators up to 127 K through the streaming GEMM
    (8, 2, 20000, 200, 100, 48, 4, "bf16"),    # split rotation: the quantizing launch
    (4, 16, 5120, 64, 80, 640, 16, "bf16"),    # A4 codes (in int8 containers)
    (4, 40, 1024, 32, 32, 200, 16, "bf16"),
    (2, 5, 96, 8, 12, 33, 8, "bf16"),          # the narrowest width: codes in {-1, 0, 1}
])
def test_other_activation_widths(bits, M, K, n1, n2, N, r, xd):
    """bwla_rotate_quant_bits: the same quantizer at other code widths (paper Tables 1-3: A6, A4;
    Sec. 4.4: W1A8); bwla_linear_forward takes the codes as they are."""
    from parity_util import run_case
    cfg = syn.LayerConfig(f"a{bits}_{M}_{K}_{N}_{r}", M, K, n1, n2, N, r, xd, max(1, K // 100), 20.0, seed=13)
    print(run_case(cfg, act_bits=bits), flush=True)


@pytest.mark.parametrize("M,K,n1,n2,N,r", [
    (2048, 25600, 160, 160, 5120, 64),   # the prefill configuration's shape: 256 x 160 tiles
    (300, 1152, 36, 32, 200, 20),        # ragged token and channel tiles, 9 slices, one wavefront per tile
    (64, 8192, 128, 64, 8192, 64),       # four wavefronts share a tile and split K
    (130, 4096, 64, 64, 2500, 0),        # no low-rank part
])
def test_nibble_packed_a4_codes(M, K, n1, n2, N, r):
    """W1A4 with two codes per byte (paper Table 3): the packing kernel against the oracle's layout,
    bit for bit, and the GEMM on packed codes against the GEMM on the same codes in int8 -- accumulators
    and outputs identical -- which the oracle's rows then check by the usual criteria."""
    from parity_util import pack_on_gpu, x_on_gpu, check_output, DEV
    from oracle import bwla_oracle as orc
    from paper_2605_00422_amd import binding as B
    cfg = syn.LayerConfig(f"a4n_{M}_{K}_{N}", M, K, n1, n2, N, r, "bf16", max(1, K // 100), 20.0, seed=31)
    d = syn.make_layer(cfg)
    layer = pack_on_gpu(d)
    X = x_on_gpu(d)
    act = B.Activations(layer, M)
    B.rotate_quant(layer, X, act, 4)
    Y8 = torch.empty((M, N), dtype=torch.float32, device=DEV)
    a8 = torch.empty((M, N), dtype=torch.int32, device=DEV)
    B.linear_forward(layer, act, Y8, a8)
    q4 = B.pack_codes_a4(act.q)
    Y4 = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
    a4 = torch.full((M, N), -1, dtype=torch.int32, device=DEV)
    B.linear_forward_a4(layer, q4, act, Y4, a4)
    torch.cuda.synchronize()
    q = act.q.cpu().numpy()
    assert q.min() >= -7 and q.max() <= 7
    assert np.array_equal(q4.cpu().numpy(), orc.pack_nibbles(q)), "packed layout differs from the oracle's"
    assert torch.equal(a4, a8), "accumulators on packed codes differ"
    assert torch.equal(Y4, Y8), "outputs on packed codes differ"
    # the oracle on a sample of rows, from the GPU's own codes: exact accumulators, output by criterion 3
    rows = _sample_rows(M, 16, seed=5)
    sgn, alpha = orc.binarize_rows(d.W)
    assert np.array_equal(a4[torch.from_numpy(rows).to(DEV)].cpu().numpy().astype(np.int64), orc.binary_gemm(q[rows], sgn))
    ref = orc.forward_rows(d.X, d.R1, d.R2, sgn, orc.to_fp16(alpha), d.U if r else None, d.V if r else None, rows, act_bits=4)
    check_output(Y4[torch.from_numpy(rows).to(DEV)].cpu().numpy(), ref["Y"])


def test_nibble_packed_a4_refusals():
    from parity_util import pack_on_gpu, DEV
    from paper_2605_00422_amd import binding as B
    cfg = syn.LayerConfig("a4n_refuse", 8, 1024, 32, 32, 64, 0, "bf16", 4, 20.0, seed=32)
    layer = pack_on_gpu(syn.make_layer(cfg))
    act = B.Activations(layer, 8)
    q4 = torch.zeros((8, 512), dtype=torch.uint8, device=DEV)
    Y = torch.empty((8, 64), dtype=torch.float32, device=DEV)
    with pytest.raises(B.BwlaError) as e:
        B.linear_forward_a4(layer, q4, act, Y)          # decode batch: the decode kernels take bytes
    assert e.value.status == 5
    with pytest.raises(B.BwlaError):
        B.pack_codes_a4(torch.zeros((2, 48), dtype=torch.int8, device=DEV))     # K not a multiple of 32


def test_row_shift_with_eight_bit_codes():
    from parity_util import run_case
    cfg = syn.LayerConfig("shift_a8", 3, 2048, 32, 64, 300, 16, "bf16", 20, 20.0, seed=14)
    print(run_case(cfg, centered=True, act_bits=8), flush=True)


@pytest.mark.parametrize("bits,centered,M,K,n1,n2,N,r,xd", [
    (6, False, 16, 512, 16, 32, 512, 8, "f32"),      # fp32 activations (old rotation kernel)
    (6, False, 1, 4096, 64, 64, 1000, 32, "bf16"),   # decode, one token
    (6, True, 16, 5120, 64, 80, 640, 13, "bf16"),    # with the row shift: 13 + 2 + 1 = 16 columns
    (6, True, 300, 1152, 36, 32, 200, 20, "bf16"),   # prefill kernels
    (6, False, 2, 20000, 200, 100, 48, 4, "bf16"),   # split rotation
    (6, True, 3, 16896, 176, 96, 80, 0, "bf16"),     # split rotation, shift, no PSP: the three mode columns only
    (6, True, 1, 11008, 128, 86, 64, 40, "bf16"),    # split rotation with resident factors, projection in groups
    (6, True, 515, 8192, 128, 64, 40, 8, "bf16"),    # looping rotation, two tokens at a time, odd token count
    (4, False, 40, 1024, 32, 32, 200, 16, "bf16"),   # A4
    (7, True, 5, 2048, 32, 64, 333, 8, "bf16"),      # the widest the offset form allows
    # one token, one launch: the paper's own setting (asymmetric codes, row shift) on the 7B shapes
    (6, True, 1, 4096, 64, 64, 4096, 64, "bf16"),    # 64 + 2 + 1 columns: five tiles of V
    (6, True, 1, 4096, 64, 64, 1029, 0, "bf16"),     # the three mode columns only, ragged channels
    (6, True, 1, 8192, 128, 64, 1024, 61, "bf16"),   # 8192 columns, 64 columns of V in all
    (7, False, 1, 4096, 64, 64, 520, 0, "bf16"),     # 7-bit codes: the two zero-point columns only
    (4, True, 1, 2048, 64, 32, 600, 13, "bf16"),     # 4-bit codes, 13 + 3 = 16 columns
])
def test_asymmetric_activation_codes(bits, centered, M, K, n1, n2, N, r, xd):
    """Layers packed with BWLA_MODE_ASYM_ACT (paper Sec. 4.1: per-token asymmetric activation
    quantization; min-max affine reading) against the oracle's forward_asym."""
    from parity_util import run_case_asym
    cfg = syn.LayerConfig(f"asym{bits}_{M}_{K}_{N}_{r}", M, K, n1, n2, N, r, xd, max(1, K // 100), 20.0, seed=15)
    print(run_case_asym(cfg, centered=centered, act_bits=bits), flush=True)


def test_asymmetric_codes_single_launch_shapes_and_zero_token():
    """One bf16 token on a layer with asymmetric codes is served by a single launch (shapes of the decode
    kernel); a token of zeros gives step 0, every stored code at the bottom of its range (q = z = 0),
    zero mode columns and a zero output."""
    from parity_util import to_dev, DEV
    from paper_2605_00422_amd import binding as B
    cfg = syn.LayerConfig("asym_zero_tok", 1, 4096, 64, 64, 777, 32, "bf16", 0, 1.0, seed=21)
    d = syn.make_layer(cfg)
    layer = B.pack_weights(to_dev(syn.shifted_weights(d)), to_dev(d.R1), to_dev(d.R2), to_dev(d.U), to_dev(d.V), cfg.n1,
                           cfg.n2, centered=True, asym=True)
    assert B.decode_forward_launches(layer, 1) == 1
    X = torch.zeros((1, cfg.K), dtype=torch.bfloat16, device=DEV)
    act = B.Activations(layer, 1)
    Y = torch.full((1, cfg.N), float("nan"), dtype=torch.float32, device=DEV)
    B.decode_forward(layer, X, act, Y)
    torch.cuda.synchronize()
    assert float(act.scale[0]) == 0.0
    assert torch.all(act.q == -32) and int(act.qsum[0]) == -32 * cfg.K
    assert torch.count_nonzero(act.T) == 0 and torch.count_nonzero(Y) == 0


@pytest.mark.parametrize("M,K,n1,n2,N,r,xd", [
    (1, 4096, 64, 64, 22016, 64, "bf16"),   # 7B gate|up at one token: gated in the decode kernel's epilogue
    (16, 5120, 64, 80, 1000, 24, "bf16"),   # sixteen tokens, N a multiple of 4
    (3, 2048, 32, 64, 334, 8, "bf16"),      # N even but not a multiple of 4: 2-byte stores, ragged last tile
    (2, 28672, 224, 128, 96, 0, "bf16"),    # long rows (several passes), no low-rank part
    (40, 1024, 32, 32, 200, 16, "bf16"),    # streaming GEMM, four waves split K: gated in its epilogue
    (300, 1152, 36, 32, 512, 20, "bf16"),   # streaming GEMM, ragged token tile
    (520, 640, 20, 32, 330, 0, "bf16"),     # streaming GEMM, N even but ragged in the last channel tile
    (40, 480, 20, 24, 70, 8, "bf16"),       # K not a multiple of 128: LDS-tiled GEMM into scratch, then the gating launch
])
def test_gated_merged_projection(M, K, n1, n2, N, r, xd):
    """bwla_linear_forward_swiglu (block chaining: the gate of the MLP block applied in the GEMM
    that computes gate and up)."""
    from parity_util import run_case_swiglu
    cfg = syn.LayerConfig(f"swiglu_{M}_{K}_{N}_{r}", M, K, n1, n2, N, r, xd, max(1, K // 100), 20.0, seed=16)
    out = run_case_swiglu(cfg)
    assert (out["ws"] == 0) == (M <= 16 or K % 128 == 0)
    print(out, flush=True)


def test_seeded_random_shapes_and_modes():
    """A seeded draw of supported (tokens, factor pair, rank, mode) combinations, each through
    the whole path against the oracle: a guard for launch rules that depend on several of them
    at once (which rotation kernel, how the projection is dealt out, which GEMM)."""
    import random
    from paper_2605_00422_amd import binding as B
    from parity_util import run_case, run_case_asym, run_case_swiglu
    rnd = random.Random(7)
    done = 0
    while done < 24:
        n1 = rnd.choice([16, 32, 48, 64, 96, 112, 128, 144, 160, 176, 192, 200, 224, 256])
        n2 = rnd.choice([8, 12, 16, 24, 32, 40, 48, 64, 75, 80, 86, 96, 100, 112, 128, 144, 160])
        K = n1 * n2
        M = rnd.choice([1, 1, 2, 3, 4, 5, 8, 9, 16, 17, 20, 33, 64, 130, 300, 515])
        r = rnd.choice([0, 8, 16, 24, 32, 40, 48, 64, 96, 120])
        N = rnd.choice([32, 40, 64, 100])
        mode = rnd.choice(["plain", "plain", "centered", "asym", "asym+centered", "gated"])
        if K % 32 or K > 32768 or n2 > n1:
            continue
        try:
            B.packed_size(N, K, n1, n2, r)
        except B.BwlaError:                    # a factor pair outside the documented limits
            continue
        cfg = syn.LayerConfig(f"rnd_{M}_{n1}x{n2}_{N}_{r}", M, K, n1, n2, N, r, "bf16", max(1, K // 100), 20.0,
                              seed=200 + done)
        print(done, cfg.name, mode, flush=True)
        if mode == "gated":
            run_case_swiglu(cfg)
        elif mode.startswith("asym"):
            run_case_asym(cfg, centered=mode.endswith("centered"))
        else:
            run_case(cfg, centered=(mode == "centered"))
        done += 1


def test_seeded_single_launch_shapes_and_modes():
    """A seeded draw over what the single-launch decode kernel takes (one bf16 token, factors of 32, 64
    or 128 x 64, ranks 0..96 that are not multiples of 16 too, channel counts around the kernel's limits,
    every mode and code width) and its neighbours (two tokens, too few channels for the shared projection),
    each through the whole path against the oracle."""
    import random
    from paper_2605_00422_amd import binding as B
    from parity_util import run_case, run_case_asym, run_case_swiglu
    rnd = random.Random(11)
    done = 0
    while done < 32:
        n1 = rnd.choice([32, 64, 64, 64, 128])
        n2 = rnd.choice([32, 64, 64]) if n1 != 128 else 64
        K = n1 * n2
        M = rnd.choice([1, 1, 1, 2])
        r = rnd.choice([0, 1, 5, 13, 16, 17, 30, 32, 45, 48, 61, 64, 70, 80, 93, 96])
        N = rnd.choice([48, 500, 512, 513, 777, 1024, 2000, 4096, 4100, 6001, 11008, 12288, 13000])
        bits = rnd.choice([6, 6, 6, 4, 7, 8])
        mode = rnd.choice(["plain", "centered", "asym", "asym+centered", "gated"])
        if mode.startswith("asym") and bits == 8:
            bits = 7
        if mode == "gated" and (N % 2 or bits != 6):
            continue
        cfg = syn.LayerConfig(f"rdl_{M}_{n1}x{n2}_{N}_{r}_a{bits}", M, K, n1, n2, N, r, "bf16", max(1, K // 100), 20.0,
                              seed=300 + done)
        print(done, cfg.name, mode, flush=True)
        if mode == "gated":
            run_case_swiglu(cfg)
        elif mode.startswith("asym"):
            run_case_asym(cfg, centered=mode.endswith("centered"), act_bits=bits)
        else:
            run_case(cfg, centered=(mode == "centered"), act_bits=bits)
        done += 1


def test_zero_token_gives_zero_codes_and_scale():
    from parity_util import pack_on_gpu, DEV
    from paper_2605_00422_amd import binding as B
    cfg = syn.LayerConfig("zero_tok", 4, 512, 16, 32, 64, 8, "f32", 0, 1.0, seed=2)
    d = syn.make_layer(cfg)
    d.X[2] = 0.0
    layer = pack_on_gpu(d)
    act = B.Activations(layer, 4)
    B.rotate_quant(layer, torch.from_numpy(d.X).to(DEV), act)
    Y = torch.empty((4, 64), dtype=torch.float32, device=DEV)
    B.linear_forward(layer, act, Y)
    torch.cuda.synchronize()
    assert int(act.q[2].abs().max()) == 0 and float(act.scale[2]) == 0.0 and int(act.qsum[2]) == 0
    assert float(Y[2].abs().max()) == 0.0
    assert int(act.q[1].abs().max()) == 31


def test_repeated_calls_are_deterministic():
    from parity_util import pack_on_gpu, x_on_gpu, DEV
    from paper_2605_00422_amd import binding as B
    cfg = syn.CONFIGS["cfg1_decode7b"]
    d = syn.make_layer(cfg)
    layer = pack_on_gpu(d)
    X = x_on_gpu(d)
    act = B.Activations(layer, cfg.M)
    outs = []
    for _ in range(3):
        B.rotate_quant(layer, X, act)
        Y = torch.empty((cfg.M, cfg.N), dtype=torch.float32, device=DEV)
        B.linear_forward(layer, act, Y)
        torch.cuda.synchronize()
        outs.append((Y.clone(), act.T.clone(), act.q.clone()))
    for o in outs[1:]:
        assert all(torch.equal(a, b) for a, b in zip(o, outs[0]))


@pytest.mark.parametrize("name,M,K,n1,n2,N,r,one_call", [
    ("decode", 1, 4096, 64, 64, 1024, 32, False),          # two launches per layer (the bench's default workload shape)
    ("single_launch", 1, 4096, 64, 64, 1024, 0, True),     # bwla_decode_forward's single-launch kernel
    ("single_launch_psp", 1, 4096, 64, 64, 1024, 32, True),     # ... with the shared projection: epoch and tagged sums move on with every replay
    ("single_launch_asym", 1, 4096, 64, 64, 1024, 32, True),    # ... on a layer with asymmetric codes and the row shift
    ("batch16", 16, 5120, 64, 80, 640, 64, False),         # projection with ten slices and its arrival counters
    ("split_rotation", 2, 20000, 200, 100, 48, 4, False),  # three launches; integer atomics on qsum
    ("prefill", 300, 1152, 36, 32, 200, 20, False),        # separate projection kernel, streaming GEMM
    ("split_groups", 1, 11008, 128, 86, 256, 96, False),   # split rotation; projection in rank groups, summed by the quantizing launch
    ("two_at_a_time", 600, 8192, 128, 64, 64, 8, False),   # looping rotation, two tokens at a time
])
def test_hip_graph_replays_match_eager(name, M, K, n1, n2, N, r, one_call):
    """The benchmark times HIP graphs: a captured layer forward, replayed several times with other
    activations in the same buffers and with eager work and synchronizations in between, gives
    the eager results bit for bit on every replay."""
    from parity_util import pack_on_gpu, x_on_gpu, DEV
    from paper_2605_00422_amd import binding as B
    cfg = syn.LayerConfig(f"graph_{name}", M, K, n1, n2, N, r, "bf16", max(1, K // 100), 20.0, seed=16)
    d = syn.make_layer(cfg)
    if name.endswith("asym"):
        from parity_util import to_dev
        layer = B.pack_weights(to_dev(syn.shifted_weights(d)), to_dev(d.R1), to_dev(d.R2), to_dev(d.U), to_dev(d.V), n1, n2,
                               centered=True, asym=True)
    else:
        layer = pack_on_gpu(d)
    if name.startswith("single_launch"):
        assert B.decode_forward_launches(layer, M) == 1
    X1 = x_on_gpu(d)
    X2 = (X1.float() * 0.75 + torch.roll(X1.float(), 3, dims=1)).to(X1.dtype)

    def forward(X, act, Y):
        if one_call:
            B.decode_forward(layer, X, act, Y)
        else:
            B.rotate_quant(layer, X, act)
            B.linear_forward(layer, act, Y)

    eager = {}
    for key, X in (("x1", X1), ("x2", X2)):
        act = B.Activations(layer, M)
        Y = torch.empty((M, N), dtype=torch.float32, device=DEV)
        forward(X, act, Y)
        torch.cuda.synchronize()
        eager[key] = (Y.clone(), act.q.clone(), act.scale.clone(), act.qsum.clone()) + ((act.T.clone(),) if r > 0 else ())

    Xg = X1.clone()
    actg = B.Activations(layer, M)
    Yg = torch.empty((M, N), dtype=torch.float32, device=DEV)
    forward(Xg, actg, Yg)                                   # warm-up outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            forward(Xg, actg, Yg)
    torch.cuda.synchronize()
    for rep, key in enumerate(("x2", "x1", "x2", "x2")):
        Xg.copy_(X2 if key == "x2" else X1)                 # eager work between the replays
        Yg.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = (Yg, actg.q, actg.scale, actg.qsum) + ((actg.T,) if r > 0 else ())
        assert all(torch.equal(a, b) for a, b in zip(got, eager[key])), f"replay {rep} ({key}) differs from eager"

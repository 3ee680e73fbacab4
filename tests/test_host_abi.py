"""Host-side checks of the C-ABI library (no GPU): it loads, exports every symbol the header
declares, and rejects bad arguments before enqueueing anything."""
import ctypes
import math
import os
import re
from ctypes import byref, c_int32, c_size_t, c_void_p

import pytest

from paper_2605_00422_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2605_00422_amd.build import build_library
        build_library()
    return B.load()


def test_exports_match_header(lib):
    from paper_2605_00422_amd import quantizer_binding as QB
    QB.load()
    declared = set()
    for header, names in (("bwla.h", B.EXPORTS), ("bwla_quantizer.h", QB.EXPORTS)):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        here = set(re.findall(r"\b(bwla_[a-z_0-9]+)\s*\(", text))
        assert here == set(names), header
        declared |= here
    for name in declared:
        assert hasattr(lib, name), name
    # and nothing else of the library's own is visible from outside
    import shutil
    import subprocess
    nm = shutil.which("nm") or "/opt/rocm/llvm/bin/llvm-nm"
    out = subprocess.run([nm, "-D", "--defined-only", B.LIB_PATH], capture_output=True, text=True, check=True).stdout
    exported = {l.split()[-1] for l in out.splitlines() if l.split() and " T " in l}
    assert {n for n in exported if "bwla" in n} == declared


def test_status_strings_and_version(lib):
    assert B.status_string(0) == "ok"
    seen = {B.status_string(s) for s in range(0, 7)}
    assert len(seen) == 7 and "unknown status" not in seen
    assert B.status_string(99) == "unknown status"
    assert B.version() >= 2


def test_kron_factor_matches_hand_pairs(lib):
    with open(os.path.join(GOLDEN, "kron_pairs.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            n, n1, n2 = (int(v) for v in line.split())
            assert B.kron_factor(n) == (n1, n2), n
    for n in range(1, 400):
        n1, n2 = B.kron_factor(n)
        assert n1 * n2 == n and n2 <= n1
        assert n2 == max(d for d in range(1, n + 1) if n % d == 0 and d * d <= n)
    a, b = c_int32(), c_int32()
    from paper_2605_00422_amd import inputs as syn
    for K, pair in syn.KRON_PAIRS.items():
        assert B.kron_factor(K) == pair, K
    assert lib.bwla_kron_factor(0, byref(a), byref(b)) == B.BWLA_ERR_SHAPE
    assert lib.bwla_kron_factor(16, None, byref(b)) == B.BWLA_ERR_NULL


def test_packed_size_accounting(lib):
    """Blob = 1 bit per weight in 16 x 512 tiles + fp16 alpha + fp16 U, V (rows padded to 16)
    + fp32 factors + operand-ordered copies of the two small factors (bf16 term planes; for factors that
    are multiples of 32 up to 160 also fp16 two-term planes of both, and for 32 or 64 the bf16 planes of
    the single-launch decode kernel).  The layer's parameters are ~1.18
    bits per weight at the 7B-like shape, inside the band the paper reports (Table 1: 1.15-1.19); the
    copies of the factors add 0.02 on top."""
    N, K, n1, n2, r = 11008, 4096, 64, 64, 32
    size = B.packed_size(N, K, n1, n2, r)
    pad = lambda n, m: (n + m - 1) // m * m
    planes = lambda n: 3 * pad(n, 16) * pad(n, 32) * 2        # three bf16 terms of a factor, padded
    decode_planes = ((n2 // 16) * (n2 // 32) * 3 * 1024 + (n1 // 32) * 2 * (n1 // 16) * 1024
                     + (n2 // 16) * (n2 // 32) * 2 * 1024)
    params = N * K // 8 + 2 * N + 2 * r * (N + K) + 4 * (n1 * n1 + n2 * n2)
    exact = params + planes(n1) + planes(n2) + decode_planes
    assert exact <= size <= exact + 9 * 256
    assert 1.15 <= 8 * params / (N * K) <= 1.19
    assert 8 * size / (N * K) <= 1.21
    # factor pairs the decode kernel does not take carry no such planes
    assert B.packed_size(N, 4096 * 2, 128, 64, r) - B.packed_size(N, 4096 * 2, 128, 64, 0) <= 2 * r * (N + 8192) + 512
    # ragged shapes pad rows to 16 and columns to 512
    size2 = B.packed_size(100, 96, 12, 8, 8)
    assert size2 >= 7 * 1 * 1024 + 200 + 2 * 16 * (100 + 96) + 4 * (144 + 64)


def test_packed_size_with_row_shifts(lib):
    """A layer with row shifts stores them as one more fp16 column of V (U keeps r columns): the blob
    grows only where the padded rank of V grows."""
    N, K, n1, n2 = 11008, 4096, 64, 64
    pad16 = lambda n: (n + 15) // 16 * 16
    for r in (0, 15, 16, 32):
        grow = B.packed_size(N, K, n1, n2, r, centered=True) - B.packed_size(N, K, n1, n2, r)
        expect = 2 * N * (pad16(r + 1) - pad16(r))
        assert expect <= grow <= expect + 2 * 256
    out = c_size_t()
    assert lib.bwla_packed_size_centered(512, 512, 16, 32, 128, byref(out)) == B.BWLA_ERR_UNSUPPORTED   # r + 1 > 128
    assert lib.bwla_packed_size_centered(512, 512, 16, 32, -1, byref(out)) == B.BWLA_ERR_SHAPE
    assert lib.bwla_packed_size_centered(512, 512, 16, 32, 127, byref(out)) == B.BWLA_OK


@pytest.mark.parametrize("args,status", [
    ((0, 512, 16, 32, 8), B.BWLA_ERR_SHAPE),
    ((512, 512, 16, 16, 8), B.BWLA_ERR_SHAPE),        # n1 * n2 != K
    ((512, 512, 16, 32, -1), B.BWLA_ERR_SHAPE),
    ((512, 48, 6, 8, 8), B.BWLA_ERR_UNSUPPORTED),     # K % 32 != 0
    ((512, 512, 16, 32, 129), B.BWLA_ERR_UNSUPPORTED),
    ((512, 65536, 256, 256, 8), B.BWLA_ERR_UNSUPPORTED),
    ((512, 8192, 512, 16, 8), B.BWLA_ERR_UNSUPPORTED),
])
def test_shape_validation(lib, args, status):
    out = c_size_t()
    assert lib.bwla_packed_size(*args, byref(out)) == status


def test_null_and_alignment_checks_happen_before_any_launch(lib):
    desc = B.BwlaLayer()
    fake = c_void_p(0x1000)
    odd = c_void_p(0x1008)
    # pack: null pointers, misalignment, small buffer
    assert lib.bwla_pack_weights(None, fake, fake, fake, fake, 512, 512, 16, 32, 8, fake, 1 << 20, None,
                                 byref(desc)) == B.BWLA_ERR_NULL
    assert lib.bwla_pack_weights(fake, fake, fake, None, fake, 512, 512, 16, 32, 8, fake, 1 << 20, None,
                                 byref(desc)) == B.BWLA_ERR_NULL
    assert lib.bwla_pack_weights(odd, fake, fake, fake, fake, 512, 512, 16, 32, 8, fake, 1 << 20, None,
                                 byref(desc)) == B.BWLA_ERR_ALIGN
    assert lib.bwla_pack_weights(fake, fake, fake, fake, fake, 512, 512, 16, 32, 8, fake, 16, None,
                                 byref(desc)) == B.BWLA_ERR_BUFSIZE
    assert lib.bwla_pack_weights(fake, fake, fake, fake, fake, 512, 512, 16, 16, 8, fake, 1 << 20, None,
                                 byref(desc)) == B.BWLA_ERR_SHAPE
    # forward calls: null layer, zeroed descriptor, inconsistent descriptor
    assert lib.bwla_rotate_quant(None, fake, 0, 1, fake, fake, fake, fake, None, 0, None) == B.BWLA_ERR_NULL
    assert lib.bwla_linear_forward(byref(desc), fake, fake, fake, fake, 1, fake, None, None) == B.BWLA_ERR_NULL
    desc.N, desc.K, desc.n1, desc.n2, desc.r = 512, 512, 16, 32, 8
    desc.d_blob = 0x1000
    assert lib.bwla_linear_forward(byref(desc), fake, fake, fake, fake, 1, fake, None, None) == B.BWLA_ERR_SHAPE
    assert lib.bwla_code_sums(None, 1, 512, fake, None) == B.BWLA_ERR_NULL
    assert lib.bwla_code_sums(fake, 0, 512, fake, None) == B.BWLA_ERR_SHAPE
    assert lib.bwla_code_sums(fake, 1, 48, fake, None) == B.BWLA_ERR_UNSUPPORTED
    out = c_size_t()
    assert lib.bwla_psp_workspace_size(byref(desc), 1, byref(out)) == B.BWLA_ERR_SHAPE


def test_binding_raises_on_error(lib):
    with pytest.raises(B.BwlaError) as e:
        B.packed_size(512, 512, 16, 16, 8)
    assert e.value.status == B.BWLA_ERR_SHAPE


def test_rotate_quant_bits_rejects_widths_outside_int8(lib):
    """The code width is checked on the host before anything else."""
    for bits in (1, 9, 16, -6):
        assert lib.bwla_rotate_quant_bits(None, None, 1, bits, 1, None, None, None, None, None, 0, None) == \
            B.BWLA_ERR_UNSUPPORTED
    for bits in (2, 4, 6, 8):                           # accepted: the next check (the layer) reports
        assert lib.bwla_rotate_quant_bits(None, None, 1, bits, 1, None, None, None, None, None, 0, None) == \
            B.BWLA_ERR_NULL


def test_packed_size_mode(lib):
    """Mode bits add columns to V only: asymmetric activation codes two, the row shift one."""
    N, K, n1, n2, r = 1024, 512, 16, 32, 13
    pad16 = lambda n: (n + 15) // 16 * 16
    base = B.packed_size(N, K, n1, n2, r)
    out = c_size_t()
    for mode, extra in ((0, 0), (1, 1), (2, 2), (3, 3)):
        assert lib.bwla_packed_size_mode(N, K, n1, n2, r, mode, byref(out)) == B.BWLA_OK
        grow = 2 * N * (pad16(r + extra) - pad16(r))
        assert grow <= out.value - base <= grow + 2 * 256
    assert lib.bwla_packed_size_mode(N, K, n1, n2, r, 4, byref(out)) == B.BWLA_ERR_UNSUPPORTED
    assert lib.bwla_packed_size_mode(N, K, n1, n2, 126, 3, byref(out)) == B.BWLA_ERR_UNSUPPORTED    # 126 + 3 > 128
    assert lib.bwla_packed_size_mode(N, K, n1, n2, 125, 3, byref(out)) == B.BWLA_OK
    assert B.packed_size(N, K, n1, n2, r, centered=True, asym=True) == \
        (lib.bwla_packed_size_mode(N, K, n1, n2, r, 3, byref(out)), out.value)[1]


def test_swiglu_entry_points_check_arguments_first(lib):
    desc = B.BwlaLayer()
    fake = c_void_p(0x1000)
    out = c_size_t()
    assert lib.bwla_swiglu_workspace_size(None, 1, byref(out)) == B.BWLA_ERR_NULL
    assert lib.bwla_swiglu_workspace_size(byref(desc), 1, None) == B.BWLA_ERR_NULL
    assert lib.bwla_linear_forward_swiglu(None, fake, fake, fake, fake, 1, fake, None, 0, None) == B.BWLA_ERR_NULL
    assert lib.bwla_linear_forward_swiglu(byref(desc), fake, fake, fake, fake, 1, fake, None, 0, None) == \
        B.BWLA_ERR_NULL                                   # zeroed descriptor: no blob


def test_quantizer_entry_points_check_arguments_first(lib):
    """Offline quantizer (include/bwla_quantizer.h): shapes, limits, null pointers, alignment and the
    scratch size are checked on the host; the scratch holds at least the five n x m fp64 arrays."""
    from paper_2605_00422_amd import quantizer_binding as QB
    QB.load()
    out = c_size_t()
    assert lib.bwla_quantizer_workspace_size(100, 512, 16, 32, 8, byref(out)) == B.BWLA_OK
    assert out.value >= 5 * 100 * 512 * 8
    assert QB.workspace_size(100, 512, 16, 32, 8) == out.value
    assert lib.bwla_quantizer_workspace_size(100, 512, 16, 32, 8, None) == B.BWLA_ERR_NULL
    assert lib.bwla_quantizer_workspace_size(100, 512, 16, 16, 8, byref(out)) == B.BWLA_ERR_SHAPE      # n1 n2 != m
    assert lib.bwla_quantizer_workspace_size(4, 512, 16, 32, 8, byref(out)) == B.BWLA_ERR_SHAPE        # k > n
    assert lib.bwla_quantizer_workspace_size(100, 512, 16, 32, -1, byref(out)) == B.BWLA_ERR_SHAPE
    assert lib.bwla_quantizer_workspace_size(1000, 512 * 512, 512, 512, 8, byref(out)) == B.BWLA_ERR_UNSUPPORTED
    assert lib.bwla_quantizer_workspace_size(1000, 512, 16, 32, 129, byref(out)) == B.BWLA_ERR_UNSUPPORTED
    assert lib.bwla_quantizer_workspace_size(70000, 512, 16, 32, 8, byref(out)) == B.BWLA_ERR_UNSUPPORTED
    fake, odd = c_void_p(0x1000), c_void_p(0x1008)
    big = 1 << 40
    assert lib.bwla_q_okt_rows(None, fake, fake, 8, fake, fake, 100, 512, 16, 32, fake, None, fake, big, None) == B.BWLA_ERR_NULL
    assert lib.bwla_q_okt_rows(fake, None, fake, 8, fake, fake, 100, 512, 16, 32, fake, None, fake, big, None) == B.BWLA_ERR_NULL
    assert lib.bwla_q_okt_rows(fake, fake, fake, 8, fake, fake, 100, 512, 16, 32, odd, None, fake, big, None) == B.BWLA_ERR_ALIGN
    assert lib.bwla_q_okt_rows(fake, fake, fake, 8, fake, fake, 100, 512, 16, 32, fake, None, fake, 1024, None) == B.BWLA_ERR_BUFSIZE
    assert lib.bwla_q_okt_rows(fake, fake, fake, 8, fake, fake, 100, 512, 16, 31, fake, None, fake, big, None) == B.BWLA_ERR_SHAPE
    assert lib.bwla_q_init_theta(None, 10, 10, 1e-8, fake, fake, None) == B.BWLA_ERR_NULL
    assert lib.bwla_q_em_step(fake, 0, 10, 1e-8, fake, fake, None) == B.BWLA_ERR_SHAPE
    assert lib.bwla_q_gmm_nll(fake, 10, 10, fake, fake, fake, fake, 8, None) == B.BWLA_ERR_BUFSIZE
    assert lib.bwla_q_procrustes(3, fake, fake, fake, fake, fake, 100, 512, 16, 32, fake, fake, big, None) == B.BWLA_ERR_SHAPE
    assert lib.bwla_q_svd_square(fake, 257, fake, fake, fake, fake, big, None) == B.BWLA_ERR_UNSUPPORTED
    assert lib.bwla_q_svd_square(fake, 16, fake, fake, fake, fake, 64, None) == B.BWLA_ERR_BUFSIZE
    assert lib.bwla_q_truncate_rank(fake, 100, 512, 0, 10, 1e-9, fake, fake, None, fake, big, None) == B.BWLA_ERR_SHAPE
    assert lib.bwla_q_psp_step(fake, fake, fake, 8, fake, fake, fake, None, 100, 512, 16, 32, 0.0, 10, 1e-9, fake, big, None) == B.BWLA_ERR_NULL
    assert lib.bwla_quantize_layer(fake, 100, 512, 16, 32, 8, 2, 0.0, 1e-8, 10, 1e-9, 1, fake, fake, fake, None, fake,
                                   None, None, None, fake, big, None) == B.BWLA_ERR_NULL               # k > 0 needs U
    assert lib.bwla_quantize_layer(fake, 100, 512, 16, 32, 8, 2, 0.0, 0.0, 10, 1e-9, 1, fake, fake, fake, fake, fake,
                                   None, None, None, fake, big, None) == B.BWLA_ERR_SHAPE              # s2_min must be > 0

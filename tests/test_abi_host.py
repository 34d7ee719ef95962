"""Host-side checks that need no GPU: the library loads, exports every symbol the header declares,
and validates its arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

from tests import helpers as Hp

from paper_2604_10496_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    found = set()
    for header in ("cq.h", "cq_measure.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        found |= set(re.findall(r"\b(cq_[a-z0-9_]+)\s*\(", text))
    return sorted(found)


def test_header_and_library_agree():
    if not os.path.exists(B.LIB_PATH):
        pytest.fail("libcq.so is not built: run `python -m paper_2604_10496_amd.build`")
    lib = B.load_library()
    declared = _declared_functions()
    assert len(declared) >= 14
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in cq.h but not exported"
    assert sorted(B.EXPORTS) == declared


def test_status_strings():
    lib = B.load_library()
    seen = {lib.cq_status_string(i) for i in range(6)}
    assert len(seen) == 6 and lib.cq_status_string(0) == b"CQ_OK"


def test_argument_validation_happens_before_any_device_call():
    lib = B.load_library()
    one = ctypes.c_void_p(256)   # a non-null dummy that must never be dereferenced
    # rotate_quant
    assert lib.cq_rotate_quant(None, one, 4, 64, 8, one, one, one, one, 1 << 20, None) == 1
    assert lib.cq_rotate_quant(one, one, 0, 64, 8, one, one, one, one, 1 << 20, None) == 2
    assert lib.cq_rotate_quant(one, one, 4, 100, 8, one, one, one, one, 1 << 20, None) == 2
    assert lib.cq_rotate_quant(one, one, 4, 64, 5, one, one, one, one, 1 << 20, None) == 3
    assert lib.cq_rotate_quant(one, one, 16, 4096, 8, one, one, one, None, 0, None) == 4
    # route_permute
    args = lambda **k: [k.get("XR", one), one, None, None, k.get("T", 8), 64, k.get("E", 8), k.get("k", 2), 0,
                        None, one, one, one, one, one, None, k.get("ws", one), k.get("wsb", 1 << 24), None]
    assert lib.cq_route_permute(*args(k=9)) == 2
    assert lib.cq_route_permute(*args(E=2000)) == 2
    assert lib.cq_route_permute(*args(XR=None)) == 1
    assert lib.cq_route_permute(*args(wsb=8)) == 4
    # grouped gemm
    W = B.CodebookWeights(256, 256, None, 2, 128, 128)
    g = lambda W, a_kind=0, epi=0, outk=0: lib.cq_codebook_grouped_gemm(ctypes.byref(W), one, a_kind, None, None,
                                                                        one, 4, epi, one, outk, None, 0, None)
    assert g(B.CodebookWeights(None, 256, None, 2, 128, 128)) == 1
    assert g(B.CodebookWeights(256, 256, None, 2, 100, 128)) == 2
    assert g(B.CodebookWeights(256, 256, None, 2, 128, 96)) == 2
    assert g(W, a_kind=7) == 3 and g(W, epi=5) == 3 and g(W, outk=9) == 3
    # the lookup formulation of the product
    gl = lambda W, epi=0, outk=0, codes=one: lib.cq_codebook_grouped_gemm_lut(ctypes.byref(W), codes, None, None,
                                                                             one, 4, epi, one, outk, None)
    assert gl(W, codes=None) == 1
    assert gl(B.CodebookWeights(None, 256, 256, 2, 128, 128)) == 1          # canonical bytes are required
    assert gl(B.CodebookWeights(256, 256, None, 2, 100, 128)) == 2
    assert gl(B.CodebookWeights(256, 256, None, 2, 128, 128, 48)) == 2      # groups of 48 weights
    assert gl(W, epi=5) == 3 and gl(W, outk=9) == 3
    # block-wise tables in the matrix-core product: groups must be multiples of 512 weights, rows of 256
    assert g(B.CodebookWeights(256, 256, None, 2, 256, 1024, 256)) == 3
    assert g(B.CodebookWeights(256, 256, None, 2, 128, 1024, 512)) == 3
    assert g(B.CodebookWeights(256, 256, None, 2, 128, 1024, -4)) == 2
    # smaller centroid budgets
    ex = lambda bits=2, K=128, src=one: lib.cq_expand_centroid_budget(src, one, bits, 2, 64, K, 1, one, one, None)
    assert ex(src=None) == 1 and ex(K=100) == 2 and ex(bits=4) == 3 and ex(bits=1) == 3
    # moe_forward: shape mismatch between layer and weights, bad bits
    gu = B.CodebookWeights(256, 256, None, 4, 256, 128)
    dn = B.CodebookWeights(256, 256, None, 4, 128, 128)
    L = B.Layer(128, 128, 4, 2, 0, 8, 256, 256, None, gu, dn)
    assert lib.cq_moe_workspace_bytes(ctypes.byref(L), 16) > 0
    assert lib.cq_moe_forward(ctypes.byref(L), one, 16, one, None, 0, None) == 4
    # the entry point with the library's own scratch array: same validation, and a batch beyond the array's
    # size is refused before any device call
    assert lib.cq_moe_forward_static(ctypes.byref(L), None, 16, one, None) == 1
    assert lib.cq_moe_forward_static(ctypes.byref(L), one, 0, one, None) == 2
    assert lib.cq_moe_workspace_bytes(ctypes.byref(L), 1 << 16) > (32 << 20)
    assert lib.cq_moe_forward_static(ctypes.byref(L), one, 1 << 16, one, None) == 4
    Lbad = B.Layer(128, 128, 4, 2, 0, 6, 256, 256, None, gu, dn)
    assert lib.cq_moe_forward(ctypes.byref(Lbad), one, 16, one, one, 1 << 30, None) == 3
    Lbad2 = B.Layer(128, 128, 4, 5, 0, 8, 256, 256, None, gu, dn)
    assert lib.cq_moe_forward(ctypes.byref(Lbad2), one, 16, one, one, 1 << 30, None) == 2
    Lbad3 = B.Layer(128, 64, 4, 2, 0, 8, 256, 256, None, gu, dn)
    assert lib.cq_moe_forward(ctypes.byref(Lbad3), one, 16, one, one, 1 << 30, None) == 2
    # block-wise tables the kernels cannot take: refused for the layer as well
    gu_b = B.CodebookWeights(256, 256, None, 4, 256, 128, 64)
    Lblk = B.Layer(128, 128, 4, 2, 0, 8, 256, 256, None, gu_b, dn)
    assert lib.cq_moe_workspace_bytes(ctypes.byref(Lblk), 16) == 0
    assert lib.cq_moe_forward(ctypes.byref(Lblk), one, 16, one, one, 1 << 30, None) == 3
    # prepack / decode
    assert lib.cq_prepack(ctypes.byref(W), one, 8, None) == 4
    assert lib.cq_decode_dense(ctypes.byref(W), 5, one, None) == 2
    assert lib.cq_stream_read(one, 24, one, None) == 2
    assert lib.cq_mfma_loop(8, 10, None, None) == 1 and lib.cq_mfma_loop(0, 10, one, None) == 2
    # split copy of R and the rotation that uses it
    assert lib.cq_rotation_split_bytes(256) == 256 * 256 * 4 and lib.cq_rotation_split_bytes(100) == 0
    assert lib.cq_rotation_split(None, 256, one, 1 << 30, None) == 1
    assert lib.cq_rotation_split(one, 100, one, 1 << 30, None) == 2
    assert lib.cq_rotation_split(one, 256, one, 16, None) == 4
    assert lib.cq_rotate_quant_split(one, None, 256, 256, 8, one, one, one, one, 1 << 30, None) == 1
    assert lib.cq_rotate_quant_split(one, one, 100, 256, 8, one, one, one, one, 1 << 30, None) == 2   # too few tokens
    assert lib.cq_rotate_quant_split(one, one, 256, 192, 8, one, one, one, one, 1 << 30, None) == 2   # H % 256
    assert lib.cq_rotate_quant_split(one, one, 256, 256, 5, one, one, one, one, 1 << 30, None) == 3
    assert lib.cq_rotate_quant_split(one, one, 256, 256, 8, one, one, one, one, 64, None) == 4
    assert lib.cq_rotate_quant_split_workspace_bytes(256, 256) >= 2 * 256 * 256 * 2 + 256 * 4
    # online-Hadamard transform of rows
    assert lib.cq_hadamard_quant(None, 4, 512, 8, None, one, one, None) == 1
    assert lib.cq_hadamard_quant(one, 4, 320, 8, None, one, one, None) == 2       # 5 * 64: no such matrix here
    assert lib.cq_hadamard_quant(one, 4, 1 << 15, 8, None, one, one, None) == 2   # row longer than LDS holds
    assert lib.cq_hadamard_quant(one, 4, 768, 5, None, one, one, None) == 3
    assert lib.cq_hadamard_quant(None, 0, 768, 8, None, None, None, None) == 0


def test_workspace_sizes_are_pure_and_monotone():
    lib = B.load_library()
    a = lib.cq_rotate_quant_workspace_bytes(16, 4096)
    assert a == lib.cq_rotate_quant_workspace_bytes(16, 4096) and a >= 16 * 4096 * 4
    assert lib.cq_rotate_quant_workspace_bytes(4096, 4096) == 0       # enough tiles: no K split
    assert lib.cq_route_permute_workspace_bytes(2048, 2048, 128, 8) >= (2048 * 8 // 256) * 128 * 4


def test_prepack_layout_documented_in_header_matches_numpy_model():
    """The tile order and nibble grouping stated in cq.h keep every weight exactly once."""
    rng = np.random.default_rng(5)
    N, K = 64, 128
    idx = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    packed = Hp.prepack_model(idx)
    # read every weight back through the documented position
    for n in (0, 17, 40, 63):
        for k in (0, 1, 5, 12, 63, 64, 77, 127):
            rb, s, l = n // 32, k // 64, (n % 32) + 32 * ((k % 64) // 32)
            within = k % 32                                   # weight inside the lane's 16-byte piece
            dword, w = within // 8, within % 8
            byte = packed[(rb * (K // 64) + s) * 1024 + l * 16 + dword * 4 + w % 4]
            got = (int(byte) >> (4 * (w // 4))) & 15
            want = (int(idx[n, k // 2]) >> (4 * (k % 2))) & 15
            assert got == want
    assert sorted(np.concatenate([packed & 15, packed >> 4]).tolist()) == \
        sorted(np.concatenate([idx.reshape(-1) & 15, idx.reshape(-1) >> 4]).tolist())


def test_build_reads_spill_counts_from_the_compiler_remarks():
    """build.py refuses kernels with asynchronous register loads that spill; its reader of hipcc's resource
    remarks is checked on a sample of that output."""
    from paper_2604_10496_amd import build
    tag = "[-Rpass-analysis=kernel-resource-usage]"
    sample = [
        f"a.hip:12:1: remark: Function Name: kern_a {tag}",
        "   12 | __global__ void kern_a() {",
        "      | ^",
        f"a.hip:12:1: remark:     VGPRs: 34 {tag}",
        f"a.hip:12:1: remark:     ScratchSize [bytes/lane]: 0 {tag}",
        f"a.hip:12:1: remark:     VGPRs Spill: 0 {tag}",
        "a.hip:40:3: warning: something else",
        f"a.hip:50:1: remark: Function Name: kern_b {tag}",
        "   50 | __global__ void kern_b() {",
        "      | ^",
        f"a.hip:50:1: remark:     ScratchSize [bytes/lane]: 8 {tag}",
        f"a.hip:50:1: remark:     VGPRs Spill: 2 {tag}",
    ]
    usage, rest = build._split_resource_remarks(sample)
    assert usage == {"kern_a": {"VGPRs": 34, "ScratchSize [bytes/lane]": 0, "VGPRs Spill": 0},
                     "kern_b": {"ScratchSize [bytes/lane]": 8, "VGPRs Spill": 2}}
    assert rest == ["a.hip:40:3: warning: something else"]

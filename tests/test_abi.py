"""The C-ABI library loads without a GPU and exports every function include/lc.h declares;
the host-only entry points behave as documented.  No compute calls here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = sorted(os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h"))
LIB = os.path.join(ROOT, "paper_2009_13003_amd", "liblc.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2009_13003_amd import build
        build.build_library()
    return ctypes.CDLL(LIB)


def declared_functions():
    names = set()
    for header in HEADERS:
        text = re.sub(r"/\*.*?\*/", "", open(header).read(), flags=re.S)
        names |= set(re.findall(r"\b(lc_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"lc_encode", "lc_blob_sizes", "lc_encode_batch", "lc_decode_batch", "lc_batch_workspace_bytes", "lc_encode_t", "lc_decode_t", "lc_encode_cached", "lc_encode_async", "lc_encode_release_inputs", "lc_encode_wait", "lc_decode", "lc_decode_many", "lc_encode_bound", "lc_workspace_bytes", "lc_set_workspace",
            "lc_blob_info", "lc_shutdown", "lc_strerror", "lc_profile", "lc_profile_read",
            "lc_profile_name", "lc_encode_sized", "lc_decode_sized"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_binding_has_every_name_it_uses_and_every_entry_point():
    """The Python binding imports without a GPU, carries a function for every call of the header (lc_batch_workspace_bytes
    and lc_profile_name are used inside it), and refers to no module-level name that is not there."""
    import ast
    import builtins
    from paper_2009_13003_amd import lc
    for name in declared_functions():
        assert hasattr(lc, name) or name in ("lc_batch_workspace_bytes", "lc_profile_name"), name
    tree = ast.parse(open(lc.__file__).read())
    used = {node.id for node in ast.walk(tree) if isinstance(node, ast.Name) and isinstance(node.ctx, ast.Load)}
    local = {a.arg for node in ast.walk(tree) if isinstance(node, ast.arguments) for a in node.args + node.kwonlyargs}
    local |= {node.id for node in ast.walk(tree) if isinstance(node, ast.Name) and isinstance(node.ctx, ast.Store)}
    missing = [u for u in used if not hasattr(lc, u) and not hasattr(builtins, u) and u not in local]
    assert not missing, missing


def test_host_only_entry_points(lib):
    lib.lc_encode_bound.restype = ctypes.c_size_t
    lib.lc_encode_bound.argtypes = [ctypes.c_uint64, ctypes.c_int]
    lib.lc_workspace_bytes.restype = ctypes.c_size_t
    lib.lc_workspace_bytes.argtypes = [ctypes.c_uint64, ctypes.c_int]
    lib.lc_strerror.restype = ctypes.c_char_p
    # header + one offset entry padded to 16 bytes
    assert lib.lc_encode_bound(0, 3) == 512 + 16
    # one chunk: header, 2 offsets (16 bytes), 128 bytes of lane lengths + 4 bytes of padding, n*nbits/8
    assert lib.lc_encode_bound(16384, 4) == 512 + 16 + 132 + 8192
    assert lib.lc_encode_bound(16385, 1) == 512 + 16 + 2 * 132 + 2049
    for bad in ((10, 0), (10, 5), ((1 << 32) + 1, 3)):
        assert lib.lc_encode_bound(*bad) == 0 and lib.lc_workspace_bytes(*bad) == 0
    assert lib.lc_workspace_bytes(1 << 28, 4) >= 8 * (1 << 14)
    # the scratch grows with n and with nbits, by at least a slot (the chunk's longest code bits) and 16 bytes of notes
    # per chunk
    fixed = lib.lc_workspace_bytes(0, 1)
    assert fixed == lib.lc_workspace_bytes(0, 4)
    for nbits in (1, 2, 3, 4):
        prev = fixed
        for nchunks in (1, 2, 63, 64, 65, 1000):
            size = lib.lc_workspace_bytes(nchunks * 16384, nbits)
            assert size > prev
            assert size - fixed >= nchunks * (16 + 4 + 16384 * ((1 << nbits) - 1) // 8)
            assert lib.lc_workspace_bytes(nchunks * 16384 - 1, nbits) == size          # a ragged chunk counts as a chunk
            if nbits > 1:
                assert size > lib.lc_workspace_bytes(nchunks * 16384, nbits - 1)
            prev = size
    assert lib.lc_strerror(0) == b"ok" and lib.lc_strerror(-2) == lib.lc_strerror(2) != b"ok"
    # blob info on a host header
    import struct
    hdr = bytearray(64)
    hdr[0:4] = b"LCB1"
    struct.pack_into("<HHQI", hdr, 4, 1, 512, 12345, 3)
    struct.pack_into("<QI", hdr, 40, 999, 0)
    n, nbits, total, status = ctypes.c_uint64(), ctypes.c_int(), ctypes.c_uint64(), ctypes.c_int()
    buf = (ctypes.c_uint8 * 64).from_buffer(hdr)
    assert lib.lc_blob_info(buf, ctypes.byref(n), ctypes.byref(nbits), ctypes.byref(total), ctypes.byref(status)) == 0
    assert (n.value, nbits.value, total.value, status.value) == (12345, 3, 999, 0)
    hdr[0] = ord("X")
    assert lib.lc_blob_info(buf, None, None, None, None) == 4


def test_blob_sizes_per_stage(lib):
    """Section 3.1.1's worked example through the library's size breakdown (n = 10, k = 5: 190 bits), and the
    three stages of a real blob against the oracle's accounting."""
    import struct
    import numpy as np
    from oracle import lc_oracle as orc
    bits = (ctypes.c_uint64 * 3)()
    hdr = bytearray(64)
    hdr[0:4] = b"LCB1"
    struct.pack_into("<HHQI", hdr, 4, 1, 512, 10, 2)          # n = 10, x = 2
    struct.pack_into("<QII", hdr, 40, 600, 0, 5)              # total bytes, status, k_E = 5
    buf = (ctypes.c_uint8 * 64).from_buffer(hdr)
    assert lib.lc_blob_sizes(buf, bits) == 0
    assert (bits[0], bits[1], bits[2]) == (10 * 3 + 5 * 32, 10 * 2 + 4 * 32, 8 * 600)
    rng = np.random.RandomState(0)
    w_ref = (0.05 * rng.randn(40000)).astype(np.float32)
    w = (w_ref + 1e-3 * rng.laplace(size=40000)).astype(np.float32)
    for nbits in (2, 3, 4):
        blob = orc.encode(w, w_ref, nbits)
        acct = orc.accounting(blob)
        head = (ctypes.c_uint8 * 512).from_buffer(bytearray(blob[:512].tobytes()))
        assert lib.lc_blob_sizes(head, bits) == 0
        assert (bits[0], bits[1], bits[2]) == (int(acct["bits_E"]), int(acct["bits_EP"]), int(acct["bits_EPH"]))
    hdr[0] = ord("X")
    assert lib.lc_blob_sizes(buf, bits) == 4 and lib.lc_blob_sizes(None, bits) == 1


def test_workloads_have_the_stated_parameter_counts():
    from paper_2009_13003_amd import workloads as W
    for name, fn in W.SHAPES.items():
        assert W.numel(fn()) == W.EXPECTED_NUMEL[name]
    assert len(W.resnet50_shapes()) == 161 and len(W.vgg16_shapes()) == 32
    assert len(W.gpt2_medium_shapes()) == 292 and len(W.llama7b_shapes()) == 291
    w, w_ref, nbits = W.single_tensor(n=1000, seed=0, device="cpu")
    w2, _, _ = W.single_tensor(n=1000, seed=0, device="cpu")
    assert nbits == 3 and w.dtype == w_ref.dtype and (w == w2).all() and abs(float((w - w_ref).abs().mean()) - 1e-3) < 3e-4

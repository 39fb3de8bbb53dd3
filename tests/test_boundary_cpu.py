"""The C-ABI library without a GPU: it loads, exports every symbol the header declares,
sizes workspaces, and rejects bad arguments before any HIP call.  CPU only."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2605_10453_amd import binding
    return binding.load_library(), binding


def declared_functions():
    text = open(os.path.join(ROOT, "include", "slimspec.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_0-9]+)\s*\(", text)) - {"defined"})


def test_header_symbols_are_exported(lib):
    l, binding = lib
    names = declared_functions()
    assert set(names) == set(binding.EXPORTED_SYMBOLS), names
    for n in names:
        assert getattr(l, n) is not None


def test_version_and_status_strings(lib):
    l, binding = lib
    assert binding.slimspec_version() == 1
    assert binding.status_string(0) == "ok"
    for s in (-1, -2, -3, -4):
        assert binding.status_string(s) not in ("ok", "unknown status")
    assert binding.status_string(-99) == "unknown status"


def test_workspace_bytes(lib):
    _, b = lib
    w1 = b.slimspec_workspace_bytes(1, 4096, 512, 128256, 10)
    w512 = b.slimspec_workspace_bytes(512, 4096, 512, 128256, 10)
    assert 0 < w1 < w512 and w1 % 256 == 0
    assert b.slimspec_workspace_bytes(1, 4096, 512, 128256, 64) > w1
    # invalid or unsupported shapes -> 0
    assert b.slimspec_workspace_bytes(0, 4096, 512, 128256, 10) == 0
    assert b.slimspec_workspace_bytes(1, 4096, 512, 128256, 0) == 0
    assert b.slimspec_workspace_bytes(1, 4096, 512, 128256, 65) == 0
    assert b.slimspec_workspace_bytes(1, 4096, 512, 128257, 10) == 0
    assert b.slimspec_workspace_bytes(1, 4100, 512, 128256, 10) == 0
    # r is ignored by the full head: a bad r still leaves the full-head size
    assert b.slimspec_workspace_bytes(1, 4096, 0, 128256, 10) > 0


def test_argument_validation_without_gpu(lib):
    l, b = lib
    fake = ctypes.c_void_p(0x1000)     # never dereferenced: validation fails first
    null = ctypes.c_void_p(0)

    def low(shape, k, h=fake, A=fake, B=fake, ids=fake, lp=fake, ws=fake, wsb=1 << 40):
        return l.slimspec_head_topk(h, A, B, ctypes.byref(shape) if shape else None, k, ids, lp, ws, wsb, None)

    def full(shape, k, dtype=0, h=fake, W=fake, ids=fake, lp=fake, ws=fake, wsb=1 << 40):
        return l.full_head_topk(h, W, dtype, ctypes.byref(shape) if shape else None, k, ids, lp, ws, wsb, None)

    S = b.SlimspecShape
    good = S(1, 4096, 512, 128256)
    assert low(None, 10) == b.STATUS_INVALID_ARGUMENT
    assert low(good, 10, h=null) == b.STATUS_INVALID_ARGUMENT
    assert low(good, 10, A=null) == b.STATUS_INVALID_ARGUMENT
    assert low(good, 10, B=null) == b.STATUS_INVALID_ARGUMENT
    assert low(good, 10, ids=null) == b.STATUS_INVALID_ARGUMENT
    assert low(good, 10, lp=null) == b.STATUS_INVALID_ARGUMENT
    assert low(good, 10, ws=null) == b.STATUS_INVALID_ARGUMENT
    assert low(good, 0) == b.STATUS_INVALID_ARGUMENT
    assert low(S(1, 64, 8, 16), 17) == b.STATUS_INVALID_ARGUMENT            # k > V
    assert low(S(0, 4096, 512, 128256), 10) == b.STATUS_INVALID_ARGUMENT
    assert low(S(1, -8, 512, 128256), 10) == b.STATUS_INVALID_ARGUMENT
    assert low(S(1, 4096, 0, 128256), 10) == b.STATUS_INVALID_ARGUMENT
    assert low(good, 65) == b.STATUS_UNSUPPORTED                            # k > KMAX
    assert low(S(1, 4096, 512, 128260), 10) == b.STATUS_UNSUPPORTED         # V % 8
    assert low(S(1, 4100, 512, 128256), 10) == b.STATUS_UNSUPPORTED         # d % 8
    assert low(S(1, 4096, 516, 128256), 10) == b.STATUS_UNSUPPORTED         # r % 8
    assert low(S(1, 4096, 512, (1 << 28) + 8), 10) == b.STATUS_UNSUPPORTED  # V beyond the 32-bit lane offsets
    assert low(S(1, 1 << 20, 1 << 11, 128256), 10) == b.STATUS_UNSUPPORTED  # d * r beyond them
    assert low(good, 10, h=ctypes.c_void_p(0x1004)) == b.STATUS_UNSUPPORTED  # misaligned
    assert low(good, 10, wsb=1024) == b.STATUS_WORKSPACE_TOO_SMALL
    assert full(good, 10, dtype=7) == b.STATUS_INVALID_ARGUMENT
    assert full(good, 10, W=null) == b.STATUS_INVALID_ARGUMENT
    assert full(S(1, 4096, 0, 128256), 10, wsb=1024) == b.STATUS_WORKSPACE_TOO_SMALL   # r ignored
    assert full(S(1, 4096, 0, 128256), 0) == b.STATUS_INVALID_ARGUMENT


def test_product_path_does_not_touch_the_checker():
    """Neither the package nor the C/HIP sources may import, include or call anything under oracle/."""
    pkg = os.path.join(ROOT, "paper_2605_10453_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f), errors="ignore").read()
                assert "oracle" not in text.lower(), f"{f} mentions the checker"
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2605_10453_amd" not in text and "libslimspec" not in text


@pytest.mark.parametrize("source,kernel", [("head_tile.hip", "head_tile_kernel"), ("merge_streams.hip", "merge_streams_kernel")])
def test_kernels_use_no_scratch_memory(source, kernel):
    """head_tile_kernel counts its own vector-memory loads (s_waitcnt vmcnt(N)); a register spill would add
    loads the count does not know about.  merge_streams_kernel once kept a small array in scratch memory, which
    cost 12 MB of writes per 512-row call.  The compiler must report no scratch for every instance of either."""
    import shutil
    import subprocess
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("hipcc not available")
    from paper_2605_10453_amd import build as build_mod
    src = os.path.join(build_mod.CSRC, source)
    flags = [f for f in build_mod.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    out = subprocess.run([hipcc, *flags, "--cuda-device-only", "-c", src, "-o", os.devnull,
                          "-Rpass-analysis=kernel-resource-usage"], capture_output=True, text=True)
    assert out.returncode == 0, out.stderr[-2000:]
    text = out.stderr
    names = re.findall(r"Function Name: (\S+)", text)
    scratch = re.findall(r"ScratchSize \[bytes/lane\]: (\d+)", text)
    found = [(n, int(sz)) for n, sz in zip(names, scratch) if kernel in n]
    assert len(found) >= 1, text[-2000:]
    assert all(sz == 0 for _, sz in found), found


def test_workspace_check_covers_every_batch_of_a_call(lib):
    """Calls with more than 512 rows run in batches that reuse the workspace; the last batch has a plan of its own
    (fewer row blocks, more slices of d) that can need more room than the first.  The size the call checks must be
    the size the query reports, and the query must cover the first batch and the tail batch alike."""
    l, b = lib
    fake = ctypes.c_void_p(0x1000)
    for d, r, V in ((5120, 640, 8192), (4096, 512, 128256), (1024, 1024, 4096)):
        for rows in list(range(513, 1024, 37)) + [1023, 1024, 1025, 1536 + 300]:
            need = b.slimspec_workspace_bytes(rows, d, r, V, 10)
            assert need > 0
            shape = b.SlimspecShape(rows, d, r, V)
            for call in (lambda wsb: l.slimspec_head_topk(fake, fake, fake, ctypes.byref(shape), 10, fake, fake, fake, wsb, None),
                         lambda wsb: l.full_head_topk(fake, fake, 0, ctypes.byref(shape), 10, fake, fake, fake, wsb, None)):
                assert call(256) == b.STATUS_WORKSPACE_TOO_SMALL
            # a call of its own with only the first 512 rows, or only the tail rows, never needs more than the whole call
            assert need >= b.slimspec_workspace_bytes(512, d, r, V, 10)
            tail = rows % 512
            if tail >= 5:
                assert need >= b.slimspec_workspace_bytes(tail, d, r, V, 10), (rows, d, r, V)


def test_truncated_head_argument_validation(lib):
    l, b = lib
    fake, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    good = b.SlimspecShape(1, 4096, 0, 65536)

    def call(shape, k, dtype=0, id_map=fake, wsb=1 << 40):
        return l.truncated_head_topk(fake, fake, dtype, id_map, ctypes.byref(shape), k, fake, fake, fake, wsb, None)

    assert call(good, 10, id_map=null) == b.STATUS_INVALID_ARGUMENT
    assert call(good, 10, id_map=ctypes.c_void_p(0x1002)) == b.STATUS_UNSUPPORTED        # misaligned
    assert call(good, 10, dtype=5) == b.STATUS_INVALID_ARGUMENT
    assert call(good, 0) == b.STATUS_INVALID_ARGUMENT
    assert call(good, 10, wsb=1024) == b.STATUS_WORKSPACE_TOO_SMALL
    assert call(b.SlimspecShape(1, 4096, 0, 65537), 10) == b.STATUS_UNSUPPORTED


def test_positions_argument_validation(lib):
    l, b = lib
    fake = ctypes.c_void_p(0x1000)
    good = b.SlimspecShape(8, 4096, 512, 128256)

    def call(n_pos, off, shape=good, k=10, wsb=1 << 40):
        arr = (ctypes.c_int32 * len(off))(*off) if off is not None else None
        return l.slimspec_head_topk_positions(fake, fake, n_pos, arr, fake, ctypes.byref(shape), k, fake, fake, fake, wsb, None)

    assert call(2, None) == b.STATUS_INVALID_ARGUMENT
    assert call(0, [0]) == b.STATUS_INVALID_ARGUMENT
    assert call(17, list(range(18))) == b.STATUS_UNSUPPORTED
    assert call(2, [1, 4, 8]) == b.STATUS_INVALID_ARGUMENT            # does not start at 0
    assert call(2, [0, 4, 7]) == b.STATUS_INVALID_ARGUMENT            # does not end at rows
    assert call(3, [0, 6, 4, 8]) == b.STATUS_INVALID_ARGUMENT         # decreasing
    assert call(2, [0, 4, 8], k=0) == b.STATUS_INVALID_ARGUMENT
    assert call(2, [0, 4, 8], wsb=1024) == b.STATUS_WORKSPACE_TOO_SMALL


def test_routed_head_argument_validation(lib):
    l, b = lib
    fake, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    good = b.SlimspecShape(1, 4096, 512, 128256)

    def call(shape, k_route, k, W=fake, dtype=0, wsb=1 << 40):
        return l.routed_head_topk(fake, fake, fake, W, dtype, ctypes.byref(shape), k_route, k, fake, fake, fake, wsb, None)

    need = l.routed_workspace_bytes(ctypes.byref(good), 64)
    assert need > b.slimspec_workspace_bytes(1, 4096, 512, 128256, 64) > 0
    assert l.routed_workspace_bytes(ctypes.byref(good), 65) == 0
    assert call(good, 64, 65) == b.STATUS_INVALID_ARGUMENT            # k > k_route
    assert call(good, 64, 0) == b.STATUS_INVALID_ARGUMENT
    assert call(good, 65, 10) == b.STATUS_UNSUPPORTED                 # k_route > KMAX
    assert call(good, 64, 10, W=null) == b.STATUS_INVALID_ARGUMENT
    assert call(good, 64, 10, dtype=3) == b.STATUS_INVALID_ARGUMENT
    assert call(good, 64, 10, wsb=need - 1) == b.STATUS_WORKSPACE_TOO_SMALL


def test_prepared_weights_argument_validation(lib):
    l, b = lib
    fake, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    good = b.SlimspecShape(512, 4096, 512, 128256)

    def call(shape=good, k=10, Bt=fake, wsb=1 << 40):
        return l.slimspec_head_topk_prepared(fake, fake, fake, Bt, ctypes.byref(shape), k, fake, fake, fake, wsb, None)

    assert call(Bt=null) == b.STATUS_INVALID_ARGUMENT
    assert call(Bt=ctypes.c_void_p(0x1008)) == b.STATUS_UNSUPPORTED                      # misaligned
    assert call(k=0) == b.STATUS_INVALID_ARGUMENT
    assert call(shape=b.SlimspecShape(512, 4096, 516, 128256)) == b.STATUS_UNSUPPORTED
    assert call(wsb=1024) == b.STATUS_WORKSPACE_TOO_SMALL

    def transpose(M=fake, K=512, V=128256, Mt=fake):
        return l.slimspec_transpose_weights(M, K, V, Mt, None)

    assert transpose(M=null) == b.STATUS_INVALID_ARGUMENT
    assert transpose(Mt=null) == b.STATUS_INVALID_ARGUMENT
    assert transpose(K=0) == b.STATUS_INVALID_ARGUMENT
    assert transpose(V=-8) == b.STATUS_INVALID_ARGUMENT
    assert transpose(K=12) == b.STATUS_UNSUPPORTED
    assert transpose(V=128257) == b.STATUS_UNSUPPORTED
    assert transpose(Mt=ctypes.c_void_p(0x1004)) == b.STATUS_UNSUPPORTED


def test_routed_head_prepared_argument_validation(lib):
    l, b = lib
    fake, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    good = b.SlimspecShape(1, 4096, 512, 128256)

    def call(shape=good, k_route=64, k=10, Bt=null, Wt=fake, dtype=0, wsb=1 << 40):
        return l.routed_head_topk_prepared(fake, fake, fake, Bt, Wt, dtype, ctypes.byref(shape), k_route, k, fake, fake, fake, wsb, None)

    assert call(Wt=null) == b.STATUS_INVALID_ARGUMENT
    assert call(Wt=ctypes.c_void_p(0x1008)) == b.STATUS_UNSUPPORTED
    assert call(Bt=ctypes.c_void_p(0x1008)) == b.STATUS_UNSUPPORTED
    assert call(k=65) == b.STATUS_INVALID_ARGUMENT
    assert call(dtype=7) == b.STATUS_INVALID_ARGUMENT
    assert call(wsb=1024) == b.STATUS_WORKSPACE_TOO_SMALL


def test_prepared_sampling_and_positions_argument_validation(lib):
    l, b = lib
    fake, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    good = b.SlimspecShape(8, 4096, 512, 128256)

    def sample(Bt=fake, k=10, lse=fake, wsb=1 << 40):
        return l.slimspec_head_sample_prepared(fake, fake, fake, Bt, ctypes.byref(good), k, 7, fake, fake, lse, fake, fake, fake, wsb, None)

    assert sample(Bt=null) == b.STATUS_INVALID_ARGUMENT
    assert sample(lse=null) == b.STATUS_INVALID_ARGUMENT
    assert sample(k=0) == b.STATUS_INVALID_ARGUMENT
    assert sample(wsb=1024) == b.STATUS_WORKSPACE_TOO_SMALL

    def positions(off, Bt=fake, n_pos=2, wsb=1 << 40):
        arr = (ctypes.c_int32 * len(off))(*off)
        return l.slimspec_head_topk_positions_prepared(fake, fake, n_pos, arr, fake, Bt, ctypes.byref(good), 10, fake, fake, fake, wsb, None)

    assert positions([0, 4, 8], Bt=null) == b.STATUS_INVALID_ARGUMENT
    assert positions([0, 4, 7]) == b.STATUS_INVALID_ARGUMENT
    assert positions([0, 4, 8], Bt=ctypes.c_void_p(0x1002)) == b.STATUS_UNSUPPORTED
    assert positions([0, 4, 8], wsb=1024) == b.STATUS_WORKSPACE_TOO_SMALL


def test_binding_rejects_mismatched_shapes_before_any_device_call(lib):
    """The Python binding only marshals arguments; what it checks itself (shapes, element sizes) it checks before
    the first device call, so CPU tensors are enough here."""
    import torch
    _, b = lib
    bf = torch.bfloat16
    h, A, B = torch.zeros(5, 64, dtype=bf), torch.zeros(64, 16, dtype=bf), torch.zeros(16, 800, dtype=bf)
    Bt_bad, W = torch.zeros(16, 800, dtype=bf), torch.zeros(64, 800, dtype=bf)
    with pytest.raises(ValueError):
        b.slimspec_head_topk(h, A, torch.zeros(24, 800, dtype=bf), 4)
    with pytest.raises(ValueError):
        b.slimspec_head_topk_prepared(h, A, B, Bt_bad, 4)                     # Bt must be [V, r]
    with pytest.raises(ValueError):
        b.slimspec_head_topk_prepared(h, A, B, torch.zeros(800, 16, dtype=torch.float32), 4)
    with pytest.raises(ValueError):
        b.slimspec_head_sample_prepared(h, A, B, Bt_bad, 4, 1)
    with pytest.raises(ValueError):
        b.slimspec_head_topk_positions_prepared(h, A.view(1, 64, 16), [0, 5], B, Bt_bad, 4)
    with pytest.raises(ValueError):
        b.routed_head_topk_prepared(h, A, B, W, 8, 4)                         # Wt must be [V, d]
    with pytest.raises(ValueError):
        b.slimspec_transpose_weights(torch.zeros(16, 800, dtype=torch.float32))
    with pytest.raises(ValueError):
        b.slimspec_transpose_weights(B, out=torch.zeros(16, 800, dtype=bf))

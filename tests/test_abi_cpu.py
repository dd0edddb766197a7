"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every function
the header declares, sizes workspaces, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2411_05288_amd", "libvp.so")
HEADER = os.path.join(ROOT, "include", "vp.h")

VP_OK, VP_ERR_INVALID_ARG, VP_ERR_UNSUPPORTED, VP_ERR_WORKSPACE, VP_ERR_DEVICE = range(5)


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2411_05288_amd.build import build
        build()
    import paper_2411_05288_amd as vp
    return vp.load_library()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vp_[a-z_]+)\s*\(", text)))


def test_exports_every_declared_symbol(lib):
    names = declared_functions()
    assert {"vp_output_fwd", "vp_combine_stats", "vp_output_bwd", "vp_embed_fwd", "vp_embed_bwd",
            "vp_workspace_bytes", "vp_version", "vp_status_string"} <= set(names)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_status_strings(lib):
    assert lib.vp_version() >= 100
    assert lib.vp_status_string(VP_OK) == b"VP_OK"
    assert lib.vp_status_string(VP_ERR_WORKSPACE) == b"VP_ERR_WORKSPACE"
    assert lib.vp_status_string(77) == b"VP_ERR_UNKNOWN"


def test_workspace_sizes(lib):
    bad = ctypes.c_size_t(-1).value
    ws = lib.vp_workspace_bytes
    # bf16 fwd: (2 * ceil(Vs/256) + 1) * N floats
    assert ws(0, 4096, 4096, 16032, 1, 1) == (2 * 63 + 1) * 4096 * 4
    assert ws(0, 4096, 4096, 16032, 1, 0) == (2 * 63 + 1) * 4096 * 4
    # fp32 fwd: logits live in the workspace only when they are not kept
    # (plus scratch for K slices when the output has few tiles: 2 slices of [128, 4096] here)
    assert ws(0, 128, 256, 4096, 0, 1) == 2 * 128 * 4096 * 4
    assert ws(0, 128, 256, 4096, 0, 0) == 128 * 4096 * 4 + 2 * 128 * 4096 * 4
    assert ws(0, 4096, 4096, 4096, 0, 1) == 0                      # enough tiles: no slicing
    # bwd: D [N, Vs] in the storage type
    assert ws(2, 4096, 8192, 16000, 1, 0) == 4096 * 16000 * 2
    assert ws(2, 4096, 4096, 4000, 1, 1) == 4096 * 4032 * 2        # rows of D padded to 128-byte multiples
    assert ws(2, 128, 256, 4096, 0, 1) == 128 * 4096 * 4 + 32 * 128 * 256 * 4   # fp32: D, then 32 K slices of dH
    assert ws(1, 128, 256, 4096, 0, 0) == 0 and ws(3, 128, 256, 4096, 1, 0) == 0
    assert ws(4, 8192, 4096, 32000, 1, 0) == 8192 * 12 + 256   # sorted keys, run starts, run counter
    assert ws(4, 5000, 4096, 32000, 1, 0) == 8192 * 12 + 256   # padded to a power of two
    assert ws(0, 0, 256, 4096, 0, 0) == bad
    assert ws(0, 128, 256, 4096, 5, 0) == bad
    assert ws(0, 128, 256, 4096, 0, 2) == bad                       # VP_SKIP_DH belongs to the backward call only
    assert ws(2, 128, 256, 4096, 0, 2) == 128 * 4096 * 4 + 32 * 128 * 256 * 4
    # Algorithm 2 forward: partials + the padded bf16 softmax' operand; fp32: one [N, Vs] matrix
    assert ws(5, 4096, 4096, 4000, 1, 1) == (2 * 16 + 1) * 4096 * 4 + 4096 * 4032 * 2
    assert ws(5, 128, 256, 4096, 0, 0) == 128 * 4096 * 4 + 32 * 128 * 256 * 4 and ws(6, 128, 256, 4096, 0, 0) == 0
    assert ws(9, 128, 256, 4096, 0, 0) == bad
    assert ws(2, 1 << 20, 256, 1 << 20, 1, 0) == bad               # N*Vs beyond 2^31 elements
    assert ws(0, 8, 8, (1 << 20) + 8, 1, 0) == bad and ws(0, 8, 8, 1 << 20, 1, 0) != bad   # rows of at most 2^20 elements
    assert ws(2, 8, (1 << 20) + 8, 8, 1, 0) == bad


def test_argument_validation_launches_nothing(lib):
    # every call below must be rejected on the host; fake non-null pointers are never touched
    P = 0x1000
    fwd, cmb, bwd, efw, ebw = (lib.vp_output_fwd, lib.vp_combine_stats, lib.vp_output_bwd,
                               lib.vp_embed_fwd, lib.vp_embed_bwd)
    assert fwd(None, P, P, 8, 8, 8, 0, 1, 0, P, P, P, None, P, 1 << 20, None) == VP_ERR_INVALID_ARG
    assert fwd(P, P, P, 0, 8, 8, 0, 1, 0, P, P, P, None, P, 1 << 20, None) == VP_ERR_INVALID_ARG
    assert fwd(P, P, P, 8, 8, 8, -1, 1, 0, P, P, P, None, P, 1 << 20, None) == VP_ERR_INVALID_ARG
    assert fwd(P, P, P, 8, 8, 8, 0, 3, 0, P, P, P, None, P, 1 << 20, None) == VP_ERR_INVALID_ARG
    assert fwd(P, P, P, 8, 8, 8, 0, 1, 1, P, P, P, None, P, 1 << 20, None) == VP_ERR_INVALID_ARG   # flag w/o buffer
    assert fwd(P, P, P, 8, 8, 8, 0, 1, 0, P, P, P, P, P, 1 << 20, None) == VP_ERR_INVALID_ARG      # buffer w/o flag
    assert fwd(P + 2, P, P, 8, 8, 8, 0, 1, 0, P, P, P, None, P, 1 << 20, None) == VP_ERR_INVALID_ARG  # misaligned
    assert fwd(P, P, P, 8, 8, 8, 0, 1, 0, P, P, P, None, P, 16, None) == VP_ERR_WORKSPACE
    assert fwd(P, P, P, 8, 8, 8, 0, 1, 0, P, P, P, None, None, 0, None) == VP_ERR_WORKSPACE
    assert fwd(P, P, P, 1 << 20, 8, 1 << 20, 0, 1, 0, P, P, P, None, P, 1 << 40, None) == VP_ERR_UNSUPPORTED
    assert cmb(P, P, P, 0, 8, P, P, None, P, None) == VP_ERR_INVALID_ARG
    assert cmb(P, P, P, 2, 8, P, P, None, None, None) == VP_ERR_INVALID_ARG
    assert bwd(P, P, P, 8, 8, 8, 0, 1, 0, P, P, None, 1.0, None, P, P, 1 << 20, None) == VP_ERR_INVALID_ARG
    assert bwd(P, P, P, 8, 8, 8, 0, 1, 0, P, P, None, 1.0, P, P, P, 8, None) == VP_ERR_WORKSPACE
    assert bwd(P, P, P, 8, 8, 8, 0, 1, 1, P, P, None, 1.0, P, P, P, 1 << 20, None) == VP_ERR_INVALID_ARG
    assert efw(P, None, 8, 8, 8, 0, 1, P, None) == VP_ERR_INVALID_ARG
    assert efw(P, P, 8, 8, 8, 0, 7, P, None) == VP_ERR_INVALID_ARG
    assert ebw(P, P, 8, 8, 8, 0, 1, P, None, 0, None) == VP_ERR_WORKSPACE
    assert ebw(P, P, 1 << 25, 8, 8, 0, 1, P, P, 1 << 40, None) == VP_ERR_UNSUPPORTED
    assert ebw(P, P, 8, 0, 8, 0, 1, P, P, 1 << 20, None) == VP_ERR_INVALID_ARG
    # Algorithm 2: pass S with A and B, the input-gradient term, pass T without dH
    fwd2, dx2 = lib.vp_output_fwd_alg2, lib.vp_output_dx_alg2
    assert fwd2(P, P, P, 8, 8, 8, 0, 1, 0, P, P, P, None, None, P, P, 1 << 20, None) == VP_ERR_INVALID_ARG   # no A
    assert fwd2(P, P, P, 8, 8, 8, 0, 1, 0, P, P, P, None, P, None, P, 1 << 20, None) == VP_ERR_INVALID_ARG   # no B
    assert fwd2(P, P, P, 8, 8, 8, 0, 1, 2, P, P, P, None, P, P, P, 1 << 20, None) == VP_ERR_INVALID_ARG      # bad flag
    assert fwd2(P, P, P, 8, 8, 8, 0, 1, 0, P, P, P, None, P, P, P, 64, None) == VP_ERR_WORKSPACE
    assert dx2(P, P, P, P, P, P, 8, 8, 1, 0, 1.0, None, None) == VP_ERR_INVALID_ARG
    assert dx2(P, P, P, P, P, P, 0, 8, 1, 0, 1.0, P, None) == VP_ERR_INVALID_ARG
    assert dx2(P, P + 4, P, P, P, P, 8, 8, 1, 0, 1.0, P, None) == VP_ERR_INVALID_ARG
    assert dx2(P, P, P, P, P, P, 8, 8, 1, 2, 1.0, P, None) == VP_ERR_INVALID_ARG                            # only VP_DH_OVERWRITE
    assert bwd(P, P, P, 8, 8, 8, 0, 1, 2, P, P, None, 1.0, None, P, P, 8, None) == VP_ERR_WORKSPACE          # VP_SKIP_DH: dH may be NULL
    assert bwd(P, P, P, 8, 8, 8, 0, 1, 8, P, P, None, 1.0, P, P, P, 1 << 20, None) == VP_ERR_INVALID_ARG
    assert bwd(P, P, P, 8, 8, 8, 0, 1, 6, P, P, None, 1.0, P, P, P, 1 << 20, None) == VP_ERR_INVALID_ARG      # skip + overwrite
    assert bwd(P, P, P, 8, 8, 8, 0, 1, 4, P, P, None, 1.0, P, P, P, 8, None) == VP_ERR_WORKSPACE               # VP_DH_OVERWRITE is valid


def test_binding_refuses_cpu_tensors(lib):
    import torch
    import paper_2411_05288_amd as vp
    H = torch.zeros(8, 8)
    with pytest.raises(vp.VPError):
        vp.vp_embed_fwd(H, torch.zeros(8, dtype=torch.int64), 0, torch.zeros(8, 8))


def test_bench_refuses_more_than_one_gpu():
    # the path runs on one GPU; asking for more must end with a message, before anything touches a GPU
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr


def test_missing_library_is_an_error_not_a_fallback(monkeypatch):
    # the product path has no CPU fallback: without libvp.so every entry point raises
    import paper_2411_05288_amd.binding as B
    monkeypatch.setattr(B, "_LIB", None)
    monkeypatch.setattr(B, "lib_path", lambda: "/nonexistent/libvp.so")
    with pytest.raises(B.VPError):
        B.load_library()
    with pytest.raises(B.VPError):
        B.vp_version()
    with pytest.raises(B.VPError):
        B.vp_workspace_bytes(B.VP_CALL_OUTPUT_FWD, 8, 8, 8, B.VP_BF16, 0)

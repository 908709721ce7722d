"""Host-only checks of the C ABI: the library loads, exports every declared symbol, sizes its
workspace as documented, and rejects bad arguments before touching any device."""
import ctypes
import os
import re

import pytest

from paper_2506_13996_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2506_13996_amd.build import build_library
        build_library(verbose=False)
    return B.load_library()


def test_every_declared_symbol_is_exported(lib):
    hdr = open(os.path.join(ROOT, "include", "alst.h")).read()
    hdr += open(os.path.join(ROOT, "include", "alst_mlp.h")).read()
    hdr += open(os.path.join(ROOT, "include", "alst_linear.h")).read()
    hdr += open(os.path.join(ROOT, "include", "alst_debug.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(alst_[a-z_0-9]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_version_and_status_strings(lib):
    assert B.alst_version() >= 100
    seen = set()
    for s in range(0, 10):
        msg = B.alst_status_string(s)
        assert msg and msg != "unknown status"
        seen.add(msg)
    assert len(seen) == 10
    assert B.alst_status_string(99) == "unknown status"


def test_workspace_is_independent_of_n_beyond_12_bytes_per_row(lib):
    H, V, T = 4096, 128256, 4096
    w = [B.alst_tiled_ce_workspace_bytes(N, H, V, T) for N in (32768, 131072, 524288)]
    assert 0 < w[0] < w[1] < w[2]
    # difference between sequence lengths: per-row loss term, lse and dense-row index (12 bytes per
    # row) plus 12 bytes per 1024 rows of scan bookkeeping (each region rounded up to 256 bytes)
    for (n0, w0), (n1, w1) in (((32768, w[0]), (131072, w[1])), ((131072, w[1]), (524288, w[2]))):
        extra = w1 - w0 - 12 * (n1 - n0)
        assert 0 <= extra <= 12 * (n1 - n0) // 1024 + 512
    # and far below the logits that are never materialised (4 * N * V bytes)
    assert w[2] < 0.04 * 4 * 524288 * V
    # a tile larger than N is clamped
    assert B.alst_tiled_ce_workspace_bytes(100, 64, 300, 4096) == B.alst_tiled_ce_workspace_bytes(100, 64, 300, 100)
    # fp32 overwrite mode accumulates directly in dW: no separate accumulator
    assert w[1] - B.alst_tiled_ce_workspace_bytes(131072, H, V, T, B.ALST_FLAG_DW_FP32) == V * H * 4
    assert B.alst_tiled_ce_workspace_bytes(0, H, V, T) == 0
    assert B.alst_tiled_ce_workspace_bytes(10, H, 0, T) == 0
    assert B.alst_tiled_ce_workspace_bytes(10, H, V, 0) == 0


def test_workspace_follows_the_tile_as_documented(lib):
    """The large terms of the workspace (alst.h): 2 Kg (Vp + H) bytes of dZ and dense hidden rows,
    4 V H of dW sums, 2 Vp H of W transposed, 8 (Vp / 128) Tp of softmax partials; Kg is one tile
    under ALST_FLAG_TILE_SCRATCH and a group of tiles (about 16384 rows) without it."""
    H, V, N = 4096, 128256, 131072
    Vp = (V + 255) // 256 * 256
    small = 12 * N + 12 * N // 1024 + 64 * 1024          # the O(N) part and the roundings to 256 bytes

    def expect(T, kg, acc=True, part_rows=0):
        Tp = (T + 255) // 256 * 256
        return (2 * kg * (Vp + H) + (4 * V * H if acc else 0) + 2 * Vp * H + 8 * (Vp // 128) * Tp + 20 * Tp
                + 4 * part_rows * H)

    for T, g in ((128, 8), (2048, 8), (4096, 4), (8192, 2), (16384, 1), (32768, 1)):
        Tp = (T + 255) // 256 * 256
        # dHidden partial products: a tile of fewer than 256 output blocks may be cut along V
        w1 = B.alst_tiled_ce_workspace_bytes(N, H, V, T, B.ALST_FLAG_TILE_SCRATCH)
        wg = B.alst_tiled_ce_workspace_bytes(N, H, V, T)
        assert wg - w1 == 2 * (g - 1) * Tp * (Vp + H), (T, g)
        lo = expect(T, Tp)
        assert lo <= w1 <= lo + 4 * 8 * Tp * H + small, T       # at most 8 ranges of partial products
        # the tile bounds the dZ scratch: no more than 2 bytes per logit of ONE tile
        assert (w1 - 4 * V * H - 2 * Vp * H - 4 * 8 * Tp * H - small
                <= 2 * Tp * Vp + 2 * Tp * H + 8 * (Vp // 128) * Tp + 20 * Tp)
    # halving the tile halves everything but the dW sums, W transposed and the O(N) part
    a = B.alst_tiled_ce_workspace_bytes(N, H, V, 4096, B.ALST_FLAG_TILE_SCRATCH | B.ALST_FLAG_DW_FP32)
    b = B.alst_tiled_ce_workspace_bytes(N, H, V, 2048, B.ALST_FLAG_TILE_SCRATCH | B.ALST_FLAG_DW_FP32)
    fixed = 12 * N + 2 * Vp * H
    assert abs((a - fixed) - 2 * (b - fixed)) <= 4 * 8 * 2048 * H + small
    # forward only: no dZ rows, no dW sums, no partial products
    f = B.alst_tiled_ce_workspace_bytes(N, H, V, 4096, B.ALST_FLAG_FORWARD_ONLY)
    assert f <= 2 * 4096 * H + 8 * (Vp // 128) * 4096 + 20 * 4096 + small
    assert B.alst_tiled_ce_workspace_bytes(N, H, V, 4096, 1 << 9) == 0       # unknown flag


def test_paper_memory_arithmetic():
    # section "Sequence Tiling ...": one fp32 copy of the logits at 16 000 tokens, V = 128 256
    assert abs(4 * 16_000 * 128_256 / 2**30 - 7.65) < 0.01
    # a 1 GiB shard of fp32 logits is about 2093 rows, i.e. about 8 shards at 16K tokens
    rows = round(2**30 / (4 * 128_256))
    assert rows == 2093 and round(16_000 / rows) == 8
    # TiledMLP example: ceil(256 000 / 4096) = 63 shards, the last one ragged
    assert -(-256_000 // 4096) == 63 and 256_000 % 4096 != 0


def _call_forward(lib, hidden=0x1000, W=0x2000, labels=0x3000, N=16, H=64, V=32, tile=8, loss=0x4000,
                  ws=0x5000, ws_bytes=1 << 40, flags=0):
    vp = ctypes.c_void_p
    return lib.alst_tiled_ce_forward(vp(hidden), vp(W), vp(labels), N, H, V, tile, -100, vp(loss),
                                     None, None, vp(ws), ws_bytes, flags, None)


def test_bad_arguments_are_rejected_on_the_host(lib):
    # the pointers are fakes: every call below must fail validation before anything is launched
    assert _call_forward(lib, hidden=None) == B.ALST_ERR_NULL
    assert _call_forward(lib, labels=None) == B.ALST_ERR_NULL
    assert _call_forward(lib, loss=None) == B.ALST_ERR_NULL
    assert _call_forward(lib, ws=None) == B.ALST_ERR_NULL
    assert _call_forward(lib, N=0) == B.ALST_ERR_SHAPE
    assert _call_forward(lib, V=-3) == B.ALST_ERR_SHAPE
    assert _call_forward(lib, tile=0) == B.ALST_ERR_SHAPE
    assert _call_forward(lib, H=60) == B.ALST_ERR_ALIGN
    assert _call_forward(lib, W=0x2004) == B.ALST_ERR_ALIGN
    assert _call_forward(lib, ws_bytes=1024) == B.ALST_ERR_WORKSPACE
    assert _call_forward(lib, flags=64) == B.ALST_ERR_UNSUPPORTED
    vp = ctypes.c_void_p
    rc = lib.alst_tiled_ce_backward(vp(0x1000), vp(0x2000), vp(0x3000), None, 16, 64, 32, 8, -100, 1.0,
                                    vp(0x6000), vp(0x7000), vp(0x5000), 1 << 40, 0, None)
    assert rc == B.ALST_ERR_NULL
    rc = lib.alst_tiled_ce_forward_backward(vp(0x1000), vp(0x2000), vp(0x3000), 16, 64, 32, 8, -100, 1.0,
                                            vp(0x4000), None, None, None, vp(0x7000), vp(0x5000),
                                            1 << 40, 0, None)
    assert rc == B.ALST_ERR_NULL
    # a forward-only workspace cannot serve the entry points that compute gradients
    rc = lib.alst_tiled_ce_forward_backward(vp(0x1000), vp(0x2000), vp(0x3000), 16, 64, 32, 8, -100, 1.0,
                                            vp(0x4000), None, None, vp(0x6000), vp(0x7000), vp(0x5000),
                                            1 << 40, B.ALST_FLAG_FORWARD_ONLY, None)
    assert rc == B.ALST_ERR_UNSUPPORTED
    assert _call_forward(lib, flags=B.ALST_FLAG_FORWARD_ONLY, ws_bytes=1024) == B.ALST_ERR_WORKSPACE
    # the unreduced losses live in the workspace: its size is checked like everywhere else
    rc = lib.alst_tiled_ce_token_losses(vp(0x5000), 1024, 16, 64, 32, 8, 0, vp(0x8000), None)
    assert rc == B.ALST_ERR_WORKSPACE
    rc = lib.alst_tiled_ce_token_losses(None, 1 << 40, 16, 64, 32, 8, 0, vp(0x8000), None)
    assert rc == B.ALST_ERR_NULL
    rc = lib.alst_tiled_ce_token_losses(vp(0x5000), 1 << 40, 16, 64, 32, 8, 1 << 9, vp(0x8000), None)
    assert rc == B.ALST_ERR_UNSUPPORTED
    assert lib.alst_last_device_status(None, None) == B.ALST_ERR_NULL
    # the entry point without a workspace argument: host validation as above, and a problem beyond
    # its static scratch is refused before any device is touched
    def noalloc(hidden=0x1000, N=16, H=64, V=32, tile=8, flags=0):
        return lib.alst_tiled_ce_forward_backward_noalloc(
            vp(hidden), vp(0x2000), vp(0x3000), N, H, V, tile, -100, 1.0, vp(0x4000), None, None,
            vp(0x6000), vp(0x7000), None, flags, None)
    assert noalloc(hidden=None) == B.ALST_ERR_NULL
    assert noalloc(H=60) == B.ALST_ERR_ALIGN
    assert noalloc(flags=B.ALST_FLAG_FORWARD_ONLY) == B.ALST_ERR_UNSUPPORTED
    assert noalloc(N=131072, H=4096, V=128256, tile=4096) == B.ALST_ERR_NOALLOC_LIMIT
    assert B.alst_tiled_ce_workspace_bytes(4096, 1024, 8192, 256, B.ALST_FLAG_TILE_SCRATCH) <= B.ALST_NOALLOC_SCRATCH_BYTES
    assert B.alst_tiled_ce_workspace_bytes(4096, 1024, 8192, 2048) > B.ALST_NOALLOC_SCRATCH_BYTES
    assert noalloc(N=4096, H=1024, V=8192, tile=2048) == B.ALST_ERR_NOALLOC_LIMIT
    assert lib.alst_shift_labels(None, vp(0x1000), 4, -100, None) == B.ALST_ERR_NULL
    assert lib.alst_shift_labels(vp(0x1000), vp(0x2000), 0, -100, None) == B.ALST_ERR_SHAPE


def test_mlp_workspace_and_host_validation(lib):
    H, I, T = 4096, 14336, 4096
    # independent of the sequence length; backward needs more than forward
    wf = [B.alst_tiled_mlp_workspace_bytes(N, H, I, T, False) for N in (4096, 256000, 1 << 20)]
    wb = [B.alst_tiled_mlp_workspace_bytes(N, H, I, T, True) for N in (4096, 256000, 1 << 20)]
    assert wf[0] == wf[1] == wf[2] > 0 and wb[0] == wb[1] == wb[2] > wf[0]
    # far below the [N, I] activations of the untiled MLP (g, u, a in bf16) at the paper's shape
    assert wb[1] < 0.2 * 3 * 2 * 256000 * I
    # forward: exactly the tile's [T, I] bf16 activations (g and u stay in registers)
    assert wf[0] == T * I * 2
    assert B.alst_tiled_mlp_workspace_bytes(100, 64, 96, 4096, True) == B.alst_tiled_mlp_workspace_bytes(100, 64, 96, 100, True)
    assert B.alst_tiled_mlp_workspace_bytes(0, H, I, T, False) == 0
    assert B.alst_tiled_mlp_workspace_bytes(10, H, 0, T, True) == 0
    vp = ctypes.c_void_p

    def fwd(x=0x1000, Wd=0x4000, y=0x5000, ws=0x6000, N=16, H=64, I=64, tile=8, wsb=1 << 40, flags=0):
        return lib.alst_tiled_mlp_forward(vp(x), vp(0x2000), vp(0x3000), vp(Wd), N, H, I, tile, vp(y), vp(ws),
                                          wsb, flags, None)
    assert fwd(x=None) == B.ALST_ERR_NULL
    assert fwd(y=None) == B.ALST_ERR_NULL
    assert fwd(ws=None) == B.ALST_ERR_NULL
    assert fwd(N=0) == B.ALST_ERR_SHAPE
    assert fwd(tile=-1) == B.ALST_ERR_SHAPE
    assert fwd(I=60) == B.ALST_ERR_ALIGN
    assert fwd(Wd=0x4008) == B.ALST_ERR_ALIGN
    assert fwd(wsb=64) == B.ALST_ERR_WORKSPACE
    assert fwd(flags=4) == B.ALST_ERR_UNSUPPORTED           # the sum flag belongs to the loss, not here
    rc = lib.alst_tiled_mlp_backward(vp(0x1000), vp(0x2000), vp(0x3000), vp(0x4000), None, 16, 64, 64, 8,
                                     vp(0x5000), vp(0x6000), vp(0x7000), vp(0x8000), vp(0x9000), 1 << 40, 0, None)
    assert rc == B.ALST_ERR_NULL


@pytest.mark.parametrize("tiles_r,tiles_c,parts", [(16, 501, 1), (16, 16, 1), (8, 16, 2), (20, 594, 1),
                                                    (16, 56, 3), (3, 5, 4), (1, 1, 8), (17, 3, 5), (1, 40, 1)])
def test_block_to_tile_mapping_covers_every_block_once_and_balances_the_xcds(lib, tiles_r, tiles_c, parts):
    """Every output block of every part is computed by exactly one workgroup; workgroup b runs on
    XCD b % 8, the 32 workgroups of a patch share one XCD, and the XCDs' loads differ by at most
    the blocks of one patch per part boundary."""
    n = B.alst_debug_block_tile(tiles_r, tiles_c, parts, 0)[0]
    assert n % 256 == 0 and n >= tiles_r * tiles_c * parts
    seen, per_xcd, patch_xcd = set(), [0] * 8, {}
    for bid in range(n):
        n2, part, tr, tc = B.alst_debug_block_tile(tiles_r, tiles_c, parts, bid)
        assert n2 == n
        if part < 0:
            continue
        assert 0 <= part < parts and 0 <= tr < tiles_r and 0 <= tc < tiles_c
        assert (part, tr, tc) not in seen
        seen.add((part, tr, tc))
        per_xcd[bid % 8] += 1
        patch_xcd.setdefault((bid // 8) // 32 * 8 + bid % 8, set()).add(bid % 8)
    assert len(seen) == tiles_r * tiles_c * parts
    assert all(len(x) == 1 for x in patch_xcd.values())
    assert max(per_xcd) - min(per_xcd) <= 32 * 2
    # the padding a launch carries stays below one round of patches plus the ragged patch edges
    assert n <= 4 * tiles_r * tiles_c * parts + 256


def test_block_to_tile_mapping_rejects_bad_arguments(lib):
    with pytest.raises(B.AlstError):
        B.alst_debug_block_tile(0, 4, 1, 0)
    with pytest.raises(B.AlstError):
        B.alst_debug_block_tile(4, 4, 1, -1)
    with pytest.raises(B.AlstError):
        B.alst_debug_block_tile(1 << 15, 1 << 15, 8, 0)


def test_binding_refuses_tensors_the_abi_would_reinterpret():
    """The C ABI sees addresses only; the binding checks dtype, shape, contiguity and device."""
    import torch
    N, H, V = 8, 16, 12
    bf = lambda *sh: torch.zeros(sh, dtype=torch.bfloat16)
    h, W = bf(N, H), bf(V, H)
    y32 = torch.zeros(N, dtype=torch.int32)
    loss = torch.zeros(1)
    ws = torch.zeros(64, dtype=torch.uint8)
    kw = dict(loss_out=loss, workspace=ws)
    with pytest.raises(TypeError, match="labels: must be torch.int32"):
        B.alst_tiled_ce_forward(h, W, torch.zeros(N, dtype=torch.int64), 4, **kw)
    with pytest.raises(TypeError, match="hidden: must be torch.bfloat16"):
        B.alst_tiled_ce_forward(h.to(torch.float16), W, y32, 4, **kw)
    with pytest.raises(TypeError, match="W: must be contiguous"):
        B.alst_tiled_ce_forward(h, bf(H, V).t(), y32, 4, **kw)
    with pytest.raises(TypeError, match="share H"):
        B.alst_tiled_ce_forward(h, bf(V, H + 8), y32, 4, **kw)
    with pytest.raises(TypeError, match="labels: expected shape"):
        B.alst_tiled_ce_forward(h, W, torch.zeros(N + 1, dtype=torch.int32), 4, **kw)
    with pytest.raises(TypeError, match="lse_out: must be torch.float32"):
        B.alst_tiled_ce_forward(h, W, y32, 4, lse_out=torch.zeros(N, dtype=torch.float64), **kw)
    with pytest.raises(TypeError, match="dW: must be torch.float32"):
        B.alst_tiled_ce_forward_backward(h, W, y32, 4, dHidden=bf(N, H), dW=bf(V, H),
                                         flags=B.ALST_FLAG_DW_FP32, **kw)
    with pytest.raises(TypeError, match="dHidden: expected shape"):
        B.alst_tiled_ce_backward(h, W, y32, torch.zeros(N), 4, dHidden=bf(N, H + 8), dW=bf(V, H), workspace=ws)
    # everything else right: a host tensor is refused (nothing is launched)
    with pytest.raises(TypeError, match="hidden: must be a device tensor"):
        B.alst_tiled_ce_forward(h, W, y32, 4, **kw)
    with pytest.raises(TypeError, match="Wd: expected shape"):
        B.alst_tiled_mlp_forward(h, bf(24, H), bf(24, H), bf(24, H), 4, y=bf(N, H), workspace=ws)


def test_host_logic_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """The library's own sources, rebuilt with ASan + UBSan on the host pass, driven by
    tests/host_sanitize_main.cpp: workspace layout, choice of dHidden ranges, patch mapping and
    argument validation over a sweep of shapes (no kernel is launched, so this runs without a GPU)."""
    import subprocess
    from paper_2506_13996_amd.build import CSRC, hipcc_path
    exe = str(tmp_path / "host_sanitize")
    srcs = [os.path.join(ROOT, "tests", "host_sanitize_main.cpp")]
    srcs += [os.path.join(CSRC, f) for f in ("tiled_ce.hip", "tiled_mlp.hip", "prof.hip")]
    cmd = [hipcc_path(), "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), *srcs, "-o", exe]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-4000:])
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr[-4000:]
    assert "0 failures" in run.stdout

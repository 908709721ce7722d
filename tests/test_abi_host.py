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
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(alst_[a-z_0-9]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_version_and_status_strings(lib):
    assert B.alst_version() >= 100
    seen = set()
    for s in range(0, 9):
        msg = B.alst_status_string(s)
        assert msg and msg != "unknown status"
        seen.add(msg)
    assert len(seen) == 9
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
    assert lib.alst_last_device_status(None, None) == B.ALST_ERR_NULL
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

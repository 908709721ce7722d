"""GPU parity: the HIP library (through its C ABI) against the CPU fp64 oracle, element by element.

Bars (stated by the build target): |L_gpu - L_or| / |L_or| <= 1e-3; for dHidden and dW,
max|G_gpu - G_or| / max|G_or| <= 2e-2.  Integer outputs (n_valid, status) must be exact.
"""
import numpy as np
import pytest
import torch

from oracle import labels_oracle as laborc
from oracle import tiled_ce_oracle as orc
from paper_2506_13996_amd import binding as B
from paper_2506_13996_amd import synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

LOSS_RTOL = 1e-3
GRAD_TOL = 2e-2
IGN = synth.IGNORE_INDEX


def _oracle(h, W, y, grad_loss=1.0, ignore_index=IGN):
    f = orc.forward(h, W, y, ignore_index=ignore_index, row_block=256)
    dH, dW = orc.backward(h, W, y, ignore_index=ignore_index, grad_loss=grad_loss, row_block=256)
    return f, dH, dW


def _check(r, f, dH, dW, tag="", valid=None):
    assert r.status == B.ALST_OK, tag
    assert r.n_valid == f["n_valid"], tag
    if f["loss"] != 0.0:
        assert abs(r.loss - f["loss"]) / abs(f["loss"]) <= LOSS_RTOL, (tag, r.loss, f["loss"])
    else:
        assert r.loss == 0.0
    # lse is defined for the tokens that take part; rows of ignored tokens are skipped and read 0
    if valid is not None:
        ref_lse = np.where(valid, f["lse"], 0.0)
        assert (r.lse[~valid] == 0.0).all(), tag
    else:
        ref_lse = f["lse"]
    assert np.abs(r.lse - ref_lse).max() <= 1e-3 * max(1.0, np.abs(f["lse"]).max()), tag
    assert np.isfinite(r.dH).all() and np.isfinite(r.dW).all(), tag
    eh, ew = G.grad_err(r.dH, dH), G.grad_err(r.dW, dW)
    assert eh <= GRAD_TOL, (tag, "dHidden", eh)
    assert ew <= GRAD_TOL, (tag, "dW", ew)
    return eh, ew


CASES = [
    # name, N, H, V, tile, ignore_frac
    ("tiny", 512, 256, 4096, 128, 0.05),            # the Tiny workload itself
    ("aligned", 1024, 256, 1024, 512, 0.05),        # every extent block-aligned: unguarded kernels
    ("aligned_3tiles_ragged_last", 1280, 512, 768, 512, 0.1),
    ("ragged", 700, 136, 1000, 300, 0.1),           # H % 64 != 0, V % 256 != 0, ragged tiles
    ("tile_gt_n", 200, 64, 300, 4096, 0.0),
    ("one_row_tiles", 5, 64, 130, 1, 0.2),
    ("small_v", 300, 128, 7, 128, 0.1),
    # few dHidden output blocks and a long vocabulary: the contraction over V is cut into ranges
    ("split_v_direct", 600, 256, 16640, 256, 0.1),
    ("split_v_guarded", 520, 136, 16392, 300, 0.1),
    # a full tile of 64 output blocks is cut into 4 ranges, the last tile (2 row blocks) into 8: the
    # number of ranges is chosen per tile on the device
    ("split_v_last_tile_differs", 8500, 512, 33280, 8192, 0.0),
    # block-aligned H, a vocabulary that ends inside a column block: unguarded logits and dW kernels
    # (the missing rows of W are masked); dHidden unguarded too, a vocabulary that is not whole
    # k-steps taking the kernel variant that clamps the last k-step's rows of W
    ("ragged_v_whole_ksteps", 600, 256, 1088, 256, 0.1),
    ("ragged_v", 600, 256, 1000, 256, 0.1),
    ("ragged_v_below_one_block", 300, 256, 72, 128, 0.1),
    # hidden sizes that are not whole k-steps of 64 (below one step, just above one, odd multiples
    # of 8): the dense hidden rows are zero padded, W's rows are read clamped in the last k-step
    ("h_below_one_kstep", 300, 8, 500, 128, 0.1),
    ("h_72", 520, 72, 700, 256, 0.1),
    ("h_1000", 300, 1000, 520, 256, 0.1),
]


@pytest.mark.parametrize("name,N,H,V,tile,frac", CASES, ids=[c[0] for c in CASES])
def test_fused_matches_oracle(name, N, H, V, tile, frac):
    wl = synth.custom(name, N, H, V, tile, ignore_frac=frac, seed=3)
    h, W, y = synth.make_inputs(wl)
    f, dH, dW = _oracle(h, W, y)
    r = G.run_fused(h, W, y, tile)
    eh, ew = _check(r, f, dH, dW, name, valid=(y != IGN))
    print(f"{name}: loss {r.loss:.6f} vs {f['loss']:.6f}  dH err {eh:.2e}  dW err {ew:.2e}")
    # rows of ignored tokens are exact zeros
    ign = (y == IGN)
    assert (r.dH[ign] == 0.0).all()


@pytest.mark.parametrize("name,N,H,V,tile,frac", CASES[:4], ids=[c[0] for c in CASES[:4]])
def test_split_forward_backward_matches_oracle(name, N, H, V, tile, frac):
    wl = synth.custom(name, N, H, V, tile, ignore_frac=frac, seed=4)
    h, W, y = synth.make_inputs(wl)
    f, dH, dW = _oracle(h, W, y, grad_loss=0.5)
    r = G.run_split(h, W, y, tile, grad_loss=0.5)
    assert r.status_bwd == B.ALST_OK
    _check(r, f, dH, dW, name, valid=(y != IGN))
    # the forward-only call and the fused call produce the same loss and lse bits
    r2 = G.run_fused(h, W, y, tile, grad_loss=0.5)
    assert r.loss_bits == r2.loss_bits
    assert (r.lse.view(np.uint32) == r2.lse.view(np.uint32)).all()


def test_loss_bits_do_not_depend_on_tile():
    wl = synth.custom("tiles", 1000, 192, 1500, 0, ignore_frac=0.1, seed=5)
    h, W, y = synth.make_inputs(wl)
    bits = set()
    lses = []
    for tile in (1000, 512, 300, 256, 77):
        r = G.run_fused(h, W, y, tile)
        bits.add(int(r.loss_bits))
        lses.append(r.lse.view(np.uint32))
    assert len(bits) == 1
    for l in lses[1:]:
        assert (l == lses[0]).all()


def test_run_to_run_bit_reproducible():
    wl = synth.custom("repro", 1024, 256, 2048, 512, ignore_frac=0.05, seed=6)
    h, W, y = synth.make_inputs(wl)
    a = G.run_fused(h, W, y, 512)
    b = G.run_fused(h, W, y, 512)
    assert a.loss_bits == b.loss_bits
    assert torch.equal(a.dH_t.view(torch.int16), b.dH_t.view(torch.int16))
    assert torch.equal(a.dW_t.view(torch.int16), b.dW_t.view(torch.int16))


def test_all_ignored_and_single_valid():
    wl = synth.custom("ign", 300, 64, 500, 128, ignore_frac=0.0, seed=7)
    h, W, y = synth.make_inputs(wl)
    y_all = np.full_like(y, IGN)
    r = G.run_fused(h, W, y_all, 128)
    assert r.status == B.ALST_OK and r.n_valid == 0 and r.loss == 0.0
    assert (r.dH == 0).all() and (r.dW == 0).all()
    y_one = y_all.copy()
    y_one[257] = 123
    f, dH, dW = _oracle(h, W, y_one)
    r = G.run_fused(h, W, y_one, 128)
    _check(r, f, dH, dW, "single valid", valid=(y_one != IGN))
    assert (r.dH[np.arange(300) != 257] == 0).all()


def test_zero_hidden_gives_ln_v():
    V = 4096
    wl = synth.custom("z", 256, 64, V, 128, ignore_frac=0.1, seed=8)
    h, W, y = synth.make_inputs(wl)
    h[:] = 0
    r = G.run_fused(h, W, y, 128)
    assert abs(r.loss - np.log(V)) < 1e-5
    assert (r.dW == 0).all()


def test_other_ignore_index_and_upstream_gradient():
    wl = synth.custom("ii", 400, 128, 600, 256, ignore_frac=0.0, seed=9)
    h, W, y = synth.make_inputs(wl)
    y[::7] = 5          # 5 is also a real vocabulary id; as ignore_index it masks those rows
    f, dH, dW = _oracle(h, W, y, grad_loss=-2.5, ignore_index=5)
    r = G.run_fused(h, W, y, 256, ignore_index=5, grad_loss=-2.5)
    _check(r, f, dH, dW, "ignore_index=5", valid=(y != 5))


def test_dw_fp32_and_accumulate_flags():
    wl = synth.custom("flags", 600, 128, 520, 256, ignore_frac=0.05, seed=10)
    h, W, y = synth.make_inputs(wl)
    f, dH, dW = _oracle(h, W, y)
    r = G.run_fused(h, W, y, 256, flags=B.ALST_FLAG_DW_FP32)
    _check(r, f, dH, dW, "fp32", valid=(y != IGN))
    assert G.grad_err(r.dW, dW) < 5e-3      # fp32 output: only the bf16 rounding of dz remains
    g = torch.Generator().manual_seed(1)
    base32 = (torch.randn(520, 128, generator=g) * np.abs(dW).max()).cuda()
    r = G.run_fused(h, W, y, 256, flags=B.ALST_FLAG_DW_FP32 | B.ALST_FLAG_DW_ACCUMULATE, dW_init=base32)
    assert G.grad_err(r.dW - base32.cpu().numpy().astype(np.float64), dW) <= GRAD_TOL
    base16 = base32.to(torch.bfloat16)
    r = G.run_fused(h, W, y, 256, flags=B.ALST_FLAG_DW_ACCUMULATE, dW_init=base16)
    ref = base16.float().cpu().numpy().astype(np.float64) + dW
    assert G.grad_err(r.dW, ref) <= GRAD_TOL


def test_tile_scratch_flag_keeps_one_tile_of_dz_and_matches_oracle():
    """ALST_FLAG_TILE_SCRATCH: the dW sums are updated after every tile (5 tiles here, the last one
    ragged) instead of once per group; same loss bits, gradients within the bar."""
    wl = synth.custom("tile_scratch", 1200, 256, 1500, 256, ignore_frac=0.1, seed=13)
    h, W, y = synth.make_inputs(wl)
    f, dH, dW = _oracle(h, W, y)
    assert (B.alst_tiled_ce_workspace_bytes(1200, 256, 1500, 256, B.ALST_FLAG_TILE_SCRATCH)
            < 0.5 * B.alst_tiled_ce_workspace_bytes(1200, 256, 1500, 256))
    for flags in (B.ALST_FLAG_TILE_SCRATCH, B.ALST_FLAG_TILE_SCRATCH | B.ALST_FLAG_DW_FP32):
        r = G.run_fused(h, W, y, 256, flags=flags)
        _check(r, f, dH, dW, f"tile scratch flags={flags}", valid=(y != IGN))
        r0 = G.run_fused(h, W, y, 256, flags=flags & ~B.ALST_FLAG_TILE_SCRATCH)
        assert r.loss_bits == r0.loss_bits
        assert torch.equal(r.dH_t.view(torch.int16), r0.dH_t.view(torch.int16))   # dHidden is per tile anyway
    r = G.run_split(h, W, y, 256, flags=B.ALST_FLAG_TILE_SCRATCH)
    assert r.status_bwd == B.ALST_OK
    _check(r, f, dH, dW, "tile scratch, split entry points", valid=(y != IGN))


def test_forward_only_workspace():
    """ALST_FLAG_FORWARD_ONLY: a workspace without dZ rows and dW sums serves the forward entry
    point and the unreduced losses, with the bits of the full-size workspace."""
    N, H, V, T = 900, 192, 2100, 256
    wl = synth.custom("fwd_only", N, H, V, T, ignore_frac=0.1, seed=14)
    h, W, y = synth.make_inputs(wl)
    f = orc.forward(h, W, y, row_block=256)
    hd, Wd, yd = G.bits_to_dev(h), G.bits_to_dev(W), torch.from_numpy(y).cuda()
    out = []
    for flags in (B.ALST_FLAG_FORWARD_ONLY, 0):
        ws = B.alloc_workspace(N, H, V, T, flags)
        loss = torch.full((1,), float("nan"), device="cuda")
        lse = torch.full((N,), float("nan"), device="cuda")
        tok = torch.full((N,), float("nan"), device="cuda")
        B.alst_tiled_ce_forward(hd, Wd, yd, T, IGN, loss_out=loss, lse_out=lse, workspace=ws, flags=flags)
        B.alst_tiled_ce_token_losses(ws, N, H, V, T, tok, flags=flags)
        assert B.alst_last_device_status(ws) == B.ALST_OK
        out.append((ws.numel(), loss.cpu().numpy().view(np.uint32)[0], lse.cpu().numpy(), tok.cpu().numpy()))
    assert out[0][0] < 0.2 * out[1][0]
    assert out[0][1] == out[1][1]
    assert (out[0][2].view(np.uint32) == out[1][2].view(np.uint32)).all()
    assert (out[0][3].view(np.uint32) == out[1][3].view(np.uint32)).all()
    assert abs(float(np.array(out[0][1], dtype=np.uint32).view(np.float32)) - f["loss"]) / f["loss"] <= LOSS_RTOL
    assert np.abs(out[0][3] - f["loss_rows"]).max() <= 1e-3 * np.abs(f["loss_rows"]).max()
    ws = B.alloc_workspace(N, H, V, T, B.ALST_FLAG_FORWARD_ONLY)
    with pytest.raises(B.AlstError) as e:
        B.alst_tiled_ce_forward_backward(hd, Wd, yd, T, IGN, 1.0, loss_out=torch.zeros(1, device="cuda"),
                                         dHidden=torch.empty((N, H), dtype=torch.bfloat16, device="cuda"),
                                         dW=torch.empty((V, H), dtype=torch.bfloat16, device="cuda"),
                                         workspace=ws, flags=B.ALST_FLAG_FORWARD_ONLY)
    assert e.value.status == B.ALST_ERR_UNSUPPORTED


def test_vocabulary_of_one():
    """V = 1: the only logit is the label's, so every token loss is 0 and both gradients vanish
    (softmax = 1 = one-hot)."""
    wl = synth.custom("v1", 300, 64, 1, 128, ignore_frac=0.1, seed=15)
    h, W, y = synth.make_inputs(wl)
    assert set(np.unique(y)) <= {0, IGN}
    f, dH, dW = _oracle(h, W, y)
    assert f["loss"] == 0.0 and not dH.any() and not dW.any()
    r = G.run_fused(h, W, y, 128)
    assert r.status == B.ALST_OK and r.n_valid == f["n_valid"]
    assert abs(r.loss) <= 1e-6
    assert np.abs(r.lse - np.where(y != IGN, f["lse"], 0.0)).max() <= 1e-3 * max(1.0, np.abs(f["lse"]).max())
    # e = exp(0) = 1 exactly, dZ = 1 * 1 - 1 = 0 exactly
    assert (r.dH == 0).all() and (r.dW == 0).all()


def test_label_out_of_range_is_flagged_and_treated_as_ignored():
    wl = synth.custom("bad", 300, 64, 200, 128, ignore_frac=0.05, seed=11)
    h, W, y = synth.make_inputs(wl)
    yb = y.copy()
    yb[10], yb[200] = 200, -7
    r = G.run_fused(h, W, yb, 128)
    assert r.status == B.ALST_ERR_LABEL_RANGE
    yi = y.copy()
    yi[10], yi[200] = IGN, IGN
    f, dH, dW = _oracle(h, W, yi)
    r.status = B.ALST_OK
    _check(r, f, dH, dW, "bad labels ignored", valid=(yi != IGN))
    # the status word was cleared by the read
    ws = B.alloc_workspace(300, 64, 200, 128)
    loss = torch.zeros(1, device="cuda")
    B.alst_tiled_ce_forward(G.bits_to_dev(h), G.bits_to_dev(W), torch.from_numpy(y).cuda(), 128,
                            loss_out=loss, workspace=ws)
    assert B.alst_last_device_status(ws) == B.ALST_OK


def test_shift_labels_matches_paper_example():
    # section "Loss Sharding in Hugging Face Transformers": labels 1..8 -> 2..8, -100
    lab = torch.arange(1, 9, dtype=torch.int32, device="cuda")
    out = torch.zeros(8, dtype=torch.int32, device="cuda")
    B.alst_shift_labels(lab, out)
    torch.cuda.synchronize()
    assert out.cpu().tolist() == [2, 3, 4, 5, 6, 7, 8, -100]
    # bit-exact against the label oracle on a long random sequence and a one-token one
    g = np.random.default_rng(5)
    for n in (1, 2, 100003):
        y = g.integers(0, 50000, n).astype(np.int32)
        out = torch.zeros(n, dtype=torch.int32, device="cuda")
        B.alst_shift_labels(torch.from_numpy(y).cuda(), out, ignore_index=-7)
        assert (out.cpu().numpy() == laborc.shift_labels(y, -7)).all()


def test_loss_of_presharded_sequence_equals_unsharded():
    """Section "Loss Sharding ...": shift the labels of the whole sequence, cut hidden states and
    shifted labels into SP pieces, run the path on every piece: the summed token losses and the
    valid counts add up to those of the whole sequence (and the naive order, cut then shift, loses
    one label per piece)."""
    N, H, V, SP = 1024, 128, 1536, 4
    wl = synth.custom("sp", N, H, V, 256, ignore_frac=0.0, seed=21)
    h, W, tokens = synth.make_inputs(wl)                       # `tokens` stand for the next-token ids
    shifted = laborc.shift_labels(tokens, IGN)
    whole = orc.forward(h, W, shifted, row_block=256, reduction="sum")
    assert whole["n_valid"] == N - 1
    flags = B.ALST_FLAG_REDUCE_SUM
    Wd = G.bits_to_dev(W)
    total, count = 0.0, 0
    pieces_h = np.split(h, SP)
    for piece_h, piece_y in zip(pieces_h, laborc.shift_then_shard(tokens, SP, IGN)):
        n = len(piece_y)
        ws = B.alloc_workspace(n, H, V, 128, flags)
        loss = torch.zeros(1, device="cuda")
        nv = torch.zeros(1, dtype=torch.int64, device="cuda")
        B.alst_tiled_ce_forward(G.bits_to_dev(piece_h), Wd, torch.from_numpy(np.ascontiguousarray(piece_y)).cuda(),
                                128, IGN, loss_out=loss, n_valid_out=nv, workspace=ws, flags=flags)
        assert B.alst_last_device_status(ws) == B.ALST_OK
        total += float(loss.item())
        count += int(nv.item())
    assert count == whole["n_valid"]
    assert abs(total - whole["loss"]) / abs(whole["loss"]) <= LOSS_RTOL
    naive = sum(int((p != IGN).sum()) for p in laborc.shard_then_shift(tokens, SP, IGN))
    assert naive == N - SP


def test_sum_reduction_and_token_losses():
    wl = synth.custom("sum", 700, 128, 1000, 256, ignore_frac=0.1, seed=12)
    h, W, y = synth.make_inputs(wl)
    f = orc.forward(h, W, y, row_block=256, reduction="sum")
    dH, dW = orc.backward(h, W, y, grad_loss=0.25, row_block=256, reduction="sum")
    flags = B.ALST_FLAG_REDUCE_SUM | B.ALST_FLAG_DW_FP32
    N, H = h.shape
    V = W.shape[0]
    hd, Wd, yd = G.bits_to_dev(h), G.bits_to_dev(W), torch.from_numpy(y).cuda()
    ws = B.alloc_workspace(N, H, V, 256, flags)
    loss = torch.zeros(1, device="cuda")
    gH = torch.empty((N, H), dtype=torch.bfloat16, device="cuda")
    gW = torch.empty((V, H), dtype=torch.float32, device="cuda")
    B.alst_tiled_ce_forward_backward(hd, Wd, yd, 256, IGN, 0.25, loss_out=loss, dHidden=gH, dW=gW,
                                     workspace=ws, flags=flags)
    tok = torch.full((N,), float("nan"), device="cuda")
    B.alst_tiled_ce_token_losses(ws, N, H, V, 256, tok, flags=flags)
    assert B.alst_last_device_status(ws) == B.ALST_OK
    torch.cuda.synchronize()
    assert abs(float(loss) - f["loss"]) / abs(f["loss"]) <= LOSS_RTOL
    t = tok.cpu().numpy().astype(np.float64)
    assert (t[y == IGN] == 0.0).all()
    assert np.abs(t - f["loss_rows"]).max() <= 1e-3 * np.abs(f["loss_rows"]).max()
    assert G.grad_err(G.bf16_dev_to_f64(gH), dH) <= GRAD_TOL
    assert G.grad_err(gW.cpu().numpy().astype(np.float64), dW) <= GRAD_TOL


def test_random_shapes_against_oracle():
    """A seeded sweep of odd shapes (ragged H, V, N, tiles of every alignment): guards and tails."""
    g = np.random.default_rng(2024)
    for case in range(14):
        N = int(g.integers(1, 900))
        H = int(g.integers(1, 40)) * 8
        V = int(g.integers(2, 1400))
        tile = int(g.choice([1, 7, 64, 100, 256, 300, 512, 1000]))
        frac = float(g.choice([0.0, 0.1, 0.5, 0.95]))
        wl = synth.custom(f"rnd{case}", N, H, V, tile, ignore_frac=frac, seed=100 + case)
        h, W, y = synth.make_inputs(wl)
        f, dH, dW = _oracle(h, W, y, grad_loss=1.25)
        r = G.run_fused(h, W, y, tile, grad_loss=1.25)
        tag = f"case {case}: N={N} H={H} V={V} tile={tile} ignored={frac}"
        _check(r, f, dH, dW, tag, valid=(y != IGN))
        assert (r.dH[y == IGN] == 0.0).all(), tag


def test_random_shapes_with_block_aligned_hidden_size():
    """The same sweep with H a multiple of the block width, so that the unguarded kernels meet
    vocabularies, row counts and tiles of every alignment (V a multiple of 64 in half the cases,
    which also takes dHidden off the guarded core)."""
    g = np.random.default_rng(2025)
    for case in range(10):
        N = int(g.integers(1, 1200))
        H = int(g.choice([256, 512]))
        V = int(g.integers(1, 30)) * 64 if case % 2 == 0 else int(g.integers(2, 2000))
        tile = int(g.choice([1, 64, 100, 256, 300, 512, 1000]))
        frac = float(g.choice([0.0, 0.1, 0.5]))
        wl = synth.custom(f"rnda{case}", N, H, V, tile, ignore_frac=frac, seed=200 + case)
        h, W, y = synth.make_inputs(wl)
        f, dH, dW = _oracle(h, W, y, grad_loss=0.75)
        r = G.run_fused(h, W, y, tile, grad_loss=0.75)
        tag = f"case {case}: N={N} H={H} V={V} tile={tile} ignored={frac}"
        _check(r, f, dH, dW, tag, valid=(y != IGN))
        assert (r.dH[y == IGN] == 0.0).all(), tag


def test_large_logits_stay_finite_and_match():
    """Weights 30x the workload law: logits of several tens, a peaked softmax, losses up to ~100."""
    wl = synth.custom("big", 512, 256, 2048, 256, ignore_frac=0.05, seed=13)
    h, W, y = synth.make_inputs(wl)
    W = synth.normal_bf16(2048, 256, 0.6, 13, synth.STREAM_W)
    f, dH, dW = _oracle(h, W, y)
    assert np.abs(orc.logits(h[:8], W)).max() > 25.0 and f["loss"] > 10.0
    r = G.run_fused(h, W, y, 256)
    _check(r, f, dH, dW, "large logits", valid=(y != IGN))


def _redo_case(name, h, W, y, tile):
    f, dH, dW = _oracle(h, W, y)
    r = G.run_fused(h, W, y, tile)
    eh, ew = _check(r, f, dH, dW, name, valid=(y != IGN))
    rs = G.run_split(h, W, y, tile)
    assert rs.status_bwd == B.ALST_OK
    _check(rs, f, dH, dW, name + " split", valid=(y != IGN))
    assert rs.loss_bits == r.loss_bits and (rs.lse.view(np.uint32) == r.lse.view(np.uint32)).all()
    print(f"{name}: loss {r.loss:.4f}  max|z| {np.abs(orc.logits(h[:64], W)).max():.0f}  dH err {eh:.2e}  dW err {ew:.2e}")
    return f


def test_rows_outside_the_exponent_window_are_redone_with_their_exact_maximum():
    """The softmax of a row is first formed as exp(z) with no shift; rows whose sum leaves the
    safe range of the fp32 / bf16 exponents are recomputed relative to their exact maximum.
    Logits of +-170 (overflow), logits around -100 (underflow), and a mix where only some rows
    of each tile take the second pass; 3 tiles, the last ragged."""
    N, H, V, tile = 640, 256, 1500, 256
    wl = synth.custom("redo", N, H, V, tile, ignore_frac=0.1, seed=41)
    h, _, y = synth.make_inputs(wl)
    # overflow: logits ~ N(0, 48^2), exp(z) overflows fp32 in every row
    W_big = synth.normal_bf16(V, H, 3.0, 41, synth.STREAM_W)
    f = _redo_case("overflow", h, W_big, y, tile)
    assert np.abs(f["lse"]).max() > 100.0
    # underflow: every logit near -110 +- 10 (hidden states positive, weights negative)
    hf = np.abs(orc.bf16_bits_to_f64(h)) + 0.5
    h_pos = synth.f32_to_bf16_bits(hf.astype(np.float32))
    Wf = -np.abs(orc.bf16_bits_to_f64(synth.normal_bf16(V, H, 0.1, 42, synth.STREAM_W))) - 0.25
    W_neg = synth.f32_to_bf16_bits(Wf.astype(np.float32))
    f = _redo_case("underflow", h_pos, W_neg, y, tile)
    assert f["lse"][y != IGN].max() < -60.0
    # mixed: every third row scaled by 40 (its logits overflow), the rest ordinary
    W_ord = synth.normal_bf16(V, H, 0.1, 43, synth.STREAM_W)
    hm = orc.bf16_bits_to_f64(h).copy()
    hm[::3] *= 40.0
    h_mix = synth.f32_to_bf16_bits(hm.astype(np.float32))
    f = _redo_case("mixed", h_mix, W_ord, y, tile)
    big = np.abs(f["lse"]) > 90.0
    assert big[::3][(y != IGN)[::3]].all() and not big[1::3].any()


def test_mfma_rate_aid_reports_a_plausible_rate():
    """The benchmarking aid behind bench.py's `mfma_sustained`: a register-resident loop of the
    matrix instruction; its rate lies between a tenth of and just above the published 2.5 PFLOP/s."""
    for data in (0, 1, 2, 3):          # bit 0: operand data, bit 1: instruction form
        r = B.alst_debug_mfma_rate(data, 5000)
        assert 250.0 < r < 2700.0, (data, r)
    with pytest.raises(B.AlstError):
        B.alst_debug_mfma_rate(4, 5000)
    with pytest.raises(B.AlstError):
        B.alst_debug_mfma_rate(1, 0)


def test_calls_from_two_host_threads_on_their_own_workspaces_and_streams():
    """The library keeps no state between calls (the one-time kernel setup is behind a lock, the
    timers behind another): two host threads, each with its own workspace, outputs and stream, run
    the fused pass concurrently several times and get the bits of a single-threaded call."""
    import threading
    cases = [synth.custom("thr_a", 900, 256, 1280, 256, ignore_frac=0.1, seed=51),
             synth.custom("thr_b", 700, 128, 2100, 512, ignore_frac=0.2, seed=52)]
    inputs = [synth.make_inputs(wl) for wl in cases]
    refs = [G.run_fused(h, W, y, wl.tile) for wl, (h, W, y) in zip(cases, inputs)]
    results, errors = [None, None], []
    B.alst_profile_enable(True)            # the timers' span list is shared by the threads

    def worker(k):
        try:
            torch.cuda.set_device(0)
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                for _ in range(5):
                    r = G.run_fused(*inputs[k], cases[k].tile)
                results[k] = r
        except Exception as e:             # surfaced by the assert below
            errors.append(repr(e))

    threads = [threading.Thread(target=worker, args=(k,)) for k in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    prof = B.alst_profile_read()
    B.alst_profile_enable(False)
    assert not errors, errors
    for r, ref in zip(results, refs):
        assert r.status == B.ALST_OK and r.loss_bits == ref.loss_bits
        assert torch.equal(r.dH_t.view(torch.int16), ref.dH_t.view(torch.int16))
        assert torch.equal(r.dW_t.view(torch.int16), ref.dW_t.view(torch.int16))
    # every span of both threads was recorded: 5 calls x tiles of each case, one logits span per tile
    assert prof["logits_gemm"][1] == 5 * (4 + 2)


def test_hip_graph_replays_match_eager():
    """The entry points only enqueue kernels on the caller's stream (no allocation, no memset, no
    host synchronisation), so a call can be captured into a HIP graph.  Every replay, with eager
    work and synchronisations between the replays, must reproduce the eager result bit for bit."""
    wl = synth.custom("graph", 900, 256, 1280, 256, ignore_frac=0.1, seed=31)
    h, W, y = synth.make_inputs(wl)
    N, H, V, tile = wl.N, wl.H, wl.V, wl.tile
    hd, Wd, yd = G.bits_to_dev(h), G.bits_to_dev(W), torch.from_numpy(y).cuda()
    eager = G.run_fused(h, W, y, tile, dev_inputs=(hd, Wd, yd))       # also the first-call set-up

    ws = B.alloc_workspace(N, H, V, tile)
    loss = torch.zeros(1, device="cuda")
    lse = torch.zeros(N, device="cuda")
    dH = torch.zeros((N, H), dtype=torch.bfloat16, device="cuda")
    dW = torch.zeros((V, H), dtype=torch.bfloat16, device="cuda")
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.alst_tiled_ce_forward_backward(hd, Wd, yd, tile, IGN, 1.0, loss_out=loss, lse_out=lse,
                                         dHidden=dH, dW=dW, workspace=ws)
    for replay in range(3):
        for t in (loss, lse, dH, dW):
            t.fill_(float("nan"))                                   # eager work between the replays
        ws.random_(0, 255)                                          # the workspace holds no state
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert B.alst_last_device_status(ws) == B.ALST_OK
        assert loss.cpu().numpy().view(np.uint32)[0] == eager.loss_bits, replay
        assert torch.equal(dH.view(torch.int16), eager.dH_t.view(torch.int16)), replay
        assert torch.equal(dW.view(torch.int16), eager.dW_t.view(torch.int16)), replay
        assert np.array_equal(lse.cpu().numpy(), eager.lse), replay


def test_runs_on_the_callers_stream():
    """Everything is enqueued on the stream handed in (here a second, non-default stream of default
    priority): results are complete once that stream is synchronised, and match the default-stream run."""
    wl = synth.custom("stream", 700, 256, 1536, 256, ignore_frac=0.1, seed=41)
    h, W, y = synth.make_inputs(wl)
    base = G.run_fused(h, W, y, wl.tile)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        r = G.run_fused(h, W, y, wl.tile)
    side.synchronize()
    assert r.status == B.ALST_OK and r.loss_bits == base.loss_bits
    assert torch.equal(r.dH_t.view(torch.int16), base.dH_t.view(torch.int16))
    assert torch.equal(r.dW_t.view(torch.int16), base.dW_t.view(torch.int16))

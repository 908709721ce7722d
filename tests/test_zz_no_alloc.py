"""The entry point that allocates nothing (alst_tiled_ce_forward_backward_noalloc) against the
entry point it is a variant of (alst_tiled_ce_forward_backward with a caller-owned workspace):
same kernels on a different workspace, so every output must agree bit for bit.  Two calls in a
row share the library's static scratch; the second is smaller, so it meets whatever the first
left behind."""
import numpy as np
import pytest
import torch

from paper_2506_13996_amd import binding as B
from paper_2506_13996_amd import synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu
IGN = synth.IGNORE_INDEX


def _run_noalloc(dev_inputs, N, H, V, tile, flags=0):
    hd, Wd, yd = dev_inputs
    loss = torch.full((1,), float("nan"), device="cuda")
    lse = torch.full((N,), float("nan"), device="cuda")
    nv = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    st = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    dH = torch.full((N, H), float("nan"), dtype=torch.bfloat16, device="cuda")
    dW = torch.full((V, H), float("nan"), dtype=torch.float32 if flags & B.ALST_FLAG_DW_FP32 else torch.bfloat16,
                    device="cuda")
    B.alst_tiled_ce_forward_backward_noalloc(hd, Wd, yd, tile, IGN, 1.0, loss_out=loss, lse_out=lse,
                                             n_valid_out=nv, dHidden=dH, dW=dW, device_status_out=st,
                                             flags=flags)
    torch.cuda.synchronize()
    return loss, lse, nv, st, dH, dW


def _same_bits(a: torch.Tensor, b: torch.Tensor) -> bool:
    return torch.equal(a.contiguous().view(torch.uint8), b.contiguous().view(torch.uint8))


def test_noalloc_entry_matches_workspace_entry_on_two_calls_in_a_row():
    # first call: 3 tiles (the last ragged), two dW groups under the one-tile scratch flag;
    # second call: smaller in every extent, default grouping, a vocabulary that ends inside a block
    calls = [("first", 1100, 256, 3000, 512, 0.1, B.ALST_FLAG_TILE_SCRATCH),
             ("second_smaller", 300, 128, 1000, 128, 0.2, 0)]
    for name, N, H, V, tile, frac, flags in calls:
        assert B.alst_tiled_ce_workspace_bytes(N, H, V, tile, flags) <= B.ALST_NOALLOC_SCRATCH_BYTES
        wl = synth.custom(name, N, H, V, tile, ignore_frac=frac, seed=31)
        h, W, y = synth.make_inputs(wl)
        dev = (G.bits_to_dev(h), G.bits_to_dev(W), torch.from_numpy(y).cuda())
        print(f"noalloc case {name}: N={N} H={H} V={V} tile={tile} flags={flags}", flush=True)
        loss, lse, nv, st, dH, dW = _run_noalloc(dev, N, H, V, tile, flags)
        ref = G.run_fused(h, W, y, tile, flags=flags, dev_inputs=dev)
        assert int(st.item()) == B.ALST_OK and ref.status == B.ALST_OK
        assert int(nv.item()) == ref.n_valid == int((y != IGN).sum())
        assert loss.cpu().numpy().view(np.uint32)[0] == ref.loss_bits
        assert (lse.cpu().numpy().view(np.uint32) == ref.lse.view(np.uint32)).all()
        assert _same_bits(dH, ref.dH_t), name
        assert _same_bits(dW, ref.dW_t), name
        assert np.isfinite(ref.loss) and ref.loss > 0


def test_noalloc_entry_reports_device_status_and_refuses_large_problems():
    N, H, V, tile = 300, 64, 200, 128
    wl = synth.custom("bad", N, H, V, tile, ignore_frac=0.05, seed=32)
    h, W, y = synth.make_inputs(wl)
    y = y.copy()
    y[17] = V + 5                                   # neither ignore_index nor a vocabulary id
    dev = (G.bits_to_dev(h), G.bits_to_dev(W), torch.from_numpy(y).cuda())
    *_, st, dH, dW = _run_noalloc(dev, N, H, V, tile)
    assert int(st.item()) == B.ALST_ERR_LABEL_RANGE
    assert (dH[17] == 0).all()
    with pytest.raises(B.AlstError) as e:           # 4 V H bytes of dW sums alone exceed the scratch
        big = torch.empty((8192, 4096), dtype=torch.bfloat16, device="cuda")
        B.alst_tiled_ce_forward_backward_noalloc(
            torch.empty((256, 4096), dtype=torch.bfloat16, device="cuda"), big,
            torch.zeros(256, dtype=torch.int32, device="cuda"), 256, loss_out=torch.zeros(1, device="cuda"),
            dHidden=torch.empty((256, 4096), dtype=torch.bfloat16, device="cuda"), dW=torch.empty_like(big))
    assert e.value.status == B.ALST_ERR_NOALLOC_LIMIT

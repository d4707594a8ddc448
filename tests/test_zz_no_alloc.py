"""The allocation-free cross-entropy entry point (per-row losses in a static device array inside the
library) against ce_loss_fwd_bwd, which takes the same scratch from the caller: two calls in a row,
the second on a smaller input, each compared bit for bit with the existing entry point and, to the
tolerance of the cross-entropy parity tests, with the fp64 oracle."""
import numpy as np
import pytest
import torch

from oracle import lm_stack as olm
from synth import inputs as si
from tests.parity import assert_close, dev_bf16

pytestmark = pytest.mark.gpu


def _case(K, rng, T, V, grad_scale):
    lb = si.f32_to_bf16_bits((rng.standard_normal((T, V)) * 2.0).astype(np.float32))
    tg = rng.integers(0, V, T)
    ld, td = dev_bf16(lb), torch.from_numpy(tg).cuda()
    # existing entry point: scratch from the caller
    ref_out = torch.full_like(ld, float("nan"))
    ref_loss = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.full((max(K.ce_loss_workspace_bytes(T, V), 256),), 0xFF, dtype=torch.uint8, device="cuda")
    K.ce_loss_fwd_bwd(ld, td, T, V, grad_scale, ref_loss, ref_out, ws)
    # allocation-free entry point: no scratch argument
    out = torch.full_like(ld, float("nan"))
    loss = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")
    K.ce_loss_fwd_bwd_static(ld, td, T, V, grad_scale, loss, out)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), ref_out.view(torch.int16)), f"dlogits differ (T={T}, V={V})"
    assert torch.equal(loss.view(torch.int32), ref_loss.view(torch.int32)), f"loss differs (T={T}, V={V})"
    loss_o, dlg_o, _ = olm.ce_loss_fwd_bwd(si.bf16_bits_to_f64(lb), tg, grad_scale=grad_scale)
    assert abs(loss.item() - loss_o) <= 1e-5 * abs(loss_o)
    assert_close(out, dlg_o, f"dlogits T={T} V={V}", rel_tol=1e-2)


def test_static_scratch_entry_point_matches_the_workspace_one():
    import paper_2602_08387_amd as K
    rng = np.random.default_rng(77)
    _case(K, rng, 1536, 8000, 1.0)      # register-cached rows
    _case(K, rng, 320, 66048, 2.5)      # second call: fewer rows (two-pass kernel), stale losses behind them
    _case(K, rng, 64, 4096, 1.0)


def test_static_scratch_entry_point_rejects_more_rows_than_it_holds():
    import paper_2602_08387_amd as K
    t = torch.zeros(8, dtype=torch.bfloat16, device="cuda")
    tg = torch.zeros(1, dtype=torch.int64, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    with pytest.raises(K.DLayerError, match="exceeds"):
        K.ce_loss_fwd_bwd_static(t, tg, 65536 + 1, 8, 1.0, loss, t)

"""GPU parity of the optimizer step (grad_sq_norm + adamw_step through the C ABI) against the fp64
oracle on the same seeded bf16 parameters and gradients."""
import numpy as np
import pytest
import torch

from oracle import optimizer as oo
from synth import inputs as si
from tests.parity import dev_bf16, host_f64

pytestmark = pytest.mark.gpu

HP = dict(lr=3e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)


def _bits(rng, n, std):
    return si.f32_to_bf16_bits((rng.standard_normal(n) * std).astype(np.float32))


def _bf16_ulp(x):
    """Spacing of bf16 numbers at |x| (8 significant bits)."""
    return 2.0 ** (np.floor(np.log2(np.maximum(np.abs(x), 1e-30))) - 7)


@pytest.mark.parametrize("max_norm", [1e9, 1.0])     # clipping idle / binding
def test_clip_and_adamw_match_the_oracle(max_norm):
    import paper_2602_08387_amd as K
    rng = np.random.default_rng(11)
    sizes = [8, 16384, 16384 * 3 + 4096, 100_000, 1_000_000]     # one vector, exact chunks, ragged tails, many chunks
    pb = [_bits(rng, n, 0.02) for n in sizes]
    P = [si.bf16_bits_to_f64(b) for b in pb]
    M = [np.zeros(n) for n in sizes]
    V = [np.zeros(n) for n in sizes]
    pd = [dev_bf16(b) for b in pb]
    md = [torch.zeros(n, dtype=torch.float32, device="cuda") for n in sizes]
    vd = [torch.zeros(n, dtype=torch.float32, device="cuda") for n in sizes]
    sq = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")
    for step in (1, 2, 3):
        gb = [_bits(rng, n, 1e-3 * step) for n in sizes]
        G = [si.bf16_bits_to_f64(b) for b in gb]
        gd = [dev_bf16(b) for b in gb]
        ws = torch.full((max(K.grad_sq_norm_workspace_bytes(gd), 256),), 0xFF, dtype=torch.uint8, device="cuda")
        # the norm over two calls (3 + 2 tensors), the second accumulating
        K.grad_sq_norm(gd[:3], sq, 0, ws)
        K.grad_sq_norm(gd[3:], sq, 1, ws)
        K.adamw_step(pd, gd, md, vd, step, HP["lr"], HP["beta1"], HP["beta2"], HP["eps"], HP["weight_decay"], max_norm, sq)
        torch.cuda.synchronize()
        n_ref = oo.global_grad_norm(G)
        assert abs(np.sqrt(sq.item()) - n_ref) <= 1e-5 * n_ref
        c = oo.clip_coefficient(n_ref, max_norm)
        assert (c < 1.0) == (max_norm == 1.0)
        for i in range(len(sizes)):
            p_new, M[i], V[i] = oo.adamw_step(P[i], G[i], M[i], V[i], step, clip_coef=c, **HP)
            got = host_f64(pd[i])
            # the parameter is stored in bf16: the fp32 result may fall on the other side of a rounding
            # boundary than the fp64 one, never further than one bf16 step
            ref = si.bf16_bits_to_f64(si.f32_to_bf16_bits(p_new.astype(np.float32)))
            # plus the fp32 rounding of the two terms the new value is the difference of (it shows where
            # parameter and step nearly cancel)
            slack = 2.0 ** -22 * (np.abs(P[i]) + HP["lr"] / (1 - HP["beta1"] ** step))
            assert np.all(np.abs(got - ref) <= _bf16_ulp(ref) * 1.001 + slack), (i, step)
            assert np.mean(got == ref) > 0.99, (i, step, np.mean(got == ref))
            # fp32 moments: a few units in the last place of the larger of the two terms each is the sum of
            np.testing.assert_allclose(md[i].cpu().numpy(), M[i], rtol=2e-5, atol=1e-6 * np.abs(M[i]).max())
            np.testing.assert_allclose(vd[i].cpu().numpy(), V[i], rtol=2e-5, atol=1e-6 * np.abs(V[i]).max())
            P[i] = got        # the method stores bf16: the next step starts from what is stored
            M[i] = md[i].cpu().numpy().astype(np.float64)
            V[i] = vd[i].cpu().numpy().astype(np.float64)


def test_norm_is_reproducible_and_arguments_are_checked():
    import paper_2602_08387_amd as K
    rng = np.random.default_rng(12)
    g = [dev_bf16(_bits(rng, 300_000, 1.0)), dev_bf16(_bits(rng, 4096, 1.0))]
    ws = torch.empty(max(K.grad_sq_norm_workspace_bytes(g), 256), dtype=torch.uint8, device="cuda")
    a = torch.zeros(1, dtype=torch.float32, device="cuda")
    b = torch.zeros(1, dtype=torch.float32, device="cuda")
    K.grad_sq_norm(g, a, 0, ws)
    K.grad_sq_norm(g, b, 0, ws)
    assert torch.equal(a.view(torch.int32), b.view(torch.int32))
    ref = sum(float((t.double() ** 2).sum()) for t in g)
    assert abs(a.item() - ref) <= 1e-5 * ref
    with pytest.raises(K.DLayerError, match="multiple of 8"):
        K.grad_sq_norm([g[0][:1001]], a, 0, ws)
    with pytest.raises(K.DLayerError, match="starts at 1"):
        m = [torch.zeros_like(t, dtype=torch.float32) for t in g]
        K.adamw_step(g, g, m, m, 0, 1e-3, 0.9, 0.95, 1e-8, 0.0, 1.0, None)

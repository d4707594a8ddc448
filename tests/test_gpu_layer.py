"""Whole-layer GPU parity against the fp64 oracle: dlayer_forward / dlayer_backward through the
C ABI on the seeded workload shapes, plus the invariants the definition fixes."""
import numpy as np
import pytest
import torch

from oracle import decoder_layer as odl
from synth import inputs as si
from tests.parity import (COS_TOL, REL_TOL, assert_close, cosine, dev_bf16, f64_to_bf16_bits, host_f64, rel_err,
                          rounded)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def K():
    import paper_2602_08387_amd as k
    return k


class GpuLayer:
    """Device buffers for one layer call (allocation and pointer plumbing only)."""

    def __init__(self, K, cfg, inp):
        self.K, self.cfg = K, cfg
        self.x, self.dy = dev_bf16(inp["x"]), dev_bf16(inp["dy"])
        self.w = {n: dev_bf16(inp[n]) for n in si.WEIGHT_NAMES}
        self.y = torch.full_like(self.x, float("nan"))
        self.dx = torch.full_like(self.x, float("nan"))
        self.dw = {n: torch.full_like(t, float("nan")) for n, t in self.w.items()}
        # poisoned scratch: the library must not depend on its contents
        self.saved = torch.full((K.dlayer_saved_bytes(cfg),), 0xFF, dtype=torch.uint8, device="cuda")
        self.ws = torch.full((K.dlayer_workspace_bytes(cfg),), 0xFF, dtype=torch.uint8, device="cuda")

    def forward(self):
        self.K.dlayer_forward(self.cfg, self.x, self.w, self.y, self.saved, self.ws)

    def backward(self, accumulate=0):
        self.K.dlayer_backward(self.cfg, self.x, self.w, self.dy, self.saved, self.dx, self.dw, accumulate, self.ws)


def _oracle(cfg, inp):
    v = si.to_f64(inp)
    x, dy = v.pop("x"), v.pop("dy")
    f = odl.layer_forward(cfg, x, v)
    r = odl.layer_backward(cfg, x, v, dy, f)
    return f, r


def _check_layer(g, f, r, tag, y_tol=REL_TOL):
    rep = {"y": assert_close(g.y, f["y"], f"{tag}:y", rel_tol=y_tol)}
    rep["dx"] = assert_close(g.dx, r["dx"], f"{tag}:dx", rel_tol=np.inf)
    for n in si.WEIGHT_NAMES:
        rep[n] = assert_close(g.dw[n], r[n], f"{tag}:d{n}", rel_tol=np.inf)
    return rep


@pytest.mark.parametrize("name,override", [
    ("tiny", {}),
    ("tiny", {"rope_layout": 1}),
    ("tiny", {"n_q_heads": 8, "n_kv_heads": 2, "seq": 384}),
    ("small", {}),
    ("small", {"batch": 1, "rope_layout": 1}),
    ("1b", {}),
    ("1b", {"batch": 1, "seq": 512, "rope_layout": 1}),
    # many tokens, narrow layer: every product has more tiles than workgroups and an odd number of
    # K-steps per segment (5, 5, 5 for the q/k/v input gradients, 7 + 7 for gate/up), so the
    # persistent GEMMs change their ring parity from tile to tile and across K-segments; with 16 bands of
    # 8 tile-rows the contraction of a tile starts at every K-step offset of every segment in turn
    # (q/k/v: K-steps 0, 1, 3, 5, 7, 9, 11, 13 of 15; gate/up: 0, 1, 3, 5, 7, 8, 10, 12 of 14) and wraps
    # a layer wider than 4096 (70B-like proportions, few tokens)
    ("tiny", {"seq": 256, "d_model": 8192, "n_q_heads": 8, "n_kv_heads": 2, "head_dim": 128, "d_ff": 1024}),
    ("tiny", {"batch": 16, "seq": 2048, "d_model": 320, "n_q_heads": 5, "n_kv_heads": 5, "head_dim": 64, "d_ff": 448}),
])
def test_layer_matches_oracle(K, name, override):
    cfg = si.CONFIGS[name].with_(**override)
    inp = si.make_layer_inputs(cfg, seed=0)
    f, r = _oracle(cfg, inp)
    g = GpuLayer(K, cfg, inp)
    g.forward()
    g.backward()
    torch.cuda.synchronize()
    # the element-wise bound on y grows with the width (see Y_TOL_8B below); for the one case wider than
    # 4096 the bf16-operand floor on these very inputs is 3.4e-2 and the GPU measures 3.5e-2
    rep = _check_layer(g, f, r, name, y_tol=Y_TOL_D8192 if cfg.d_model > 4096 else REL_TOL)
    print(name, override, {k: (f"{a:.2e}", f"{b:.6f}") for k, (a, b) in rep.items()})


def test_layer_large_scores_and_accumulate(K):
    """Weights with std 2/sqrt(D) give scores with std ~4 (softmax weights spanning e^+-12: exercises
    the online-softmax rescaling).  In that regime the bf16 rounding of q and k moves the softmax
    weights by several percent, so the element-wise bound on y is 1e-1 here; the cosine bar stays.
    The second backward call accumulates into the first one's weight gradients."""
    cfg = si.CONFIGS["tiny"].with_(seq=256, n_kv_heads=2)
    inp = si.make_layer_inputs(cfg, seed=3, w_std=2.0 / np.sqrt(cfg.d_model))
    f, r = _oracle(cfg, inp)
    g = GpuLayer(K, cfg, inp)
    g.forward()
    g.backward()
    assert_close(g.y, f["y"], "wide:y", rel_tol=1e-1)
    assert_close(g.dx, r["dx"], "wide:dx", rel_tol=np.inf)
    for n in si.WEIGHT_NAMES:
        assert_close(g.dw[n], r[n], f"wide:d{n}", rel_tol=np.inf)
    g.backward(accumulate=1)
    for n in si.WEIGHT_NAMES:
        assert_close(g.dw[n], 2 * r[n], f"acc:d{n}", rel_tol=np.inf)


def test_backward_can_reuse_the_transposed_weights(K):
    """Two micro-batches through one layer: the second backward is told that the transposed weight
    copies the first one left in the workspace are still valid (the forward in between does not touch
    them) and must give, bit for bit, what a backward that rewrites them gives."""
    cfg = si.CONFIGS["small"].with_(batch=2)
    a_in, b_in = si.make_layer_inputs(cfg, seed=8), si.make_layer_inputs(cfg, seed=9)
    b_in.update({n: a_in[n] for n in si.WEIGHT_NAMES})          # same weights, new activations
    g = GpuLayer(K, cfg, a_in)
    g.forward(); g.backward()
    g.x.copy_(dev_bf16(b_in["x"])); g.dy.copy_(dev_bf16(b_in["dy"]))
    g.forward(); g.backward(accumulate=2)                       # DLAYER_REUSE_TRANSPOSED_WEIGHTS
    torch.cuda.synchronize()
    ref = GpuLayer(K, cfg, b_in)
    ref.forward(); ref.backward()
    torch.cuda.synchronize()
    for name, p, q in [("dx", g.dx, ref.dx)] + [(n, g.dw[n], ref.dw[n]) for n in si.WEIGHT_NAMES]:
        assert torch.equal(p.view(torch.int16), q.view(torch.int16)), f"{name} differs when the transposed weights are reused"
    with pytest.raises(K.DLayerError, match="unknown flag"):
        g.backward(accumulate=8)


@pytest.mark.parametrize("name,override", [("tiny", {"seq": 256}), ("small", {"batch": 2}), ("1b", {"batch": 1, "seq": 1024})])
def test_recomputing_configurations_match_the_oracle_and_keep_less(K, name, override):
    """recompute = norms | swiglu: h1, h2 and a are not kept in `saved`; the backward rebuilds them.  Same
    bar against the oracle; outputs and every gradient but the down projection's equal the keeping
    configuration's bit for bit (its operand a is rebuilt from the stored g and u when the fused kernel ran)."""
    cfg = si.CONFIGS[name].with_(**override)
    rc = cfg.with_(recompute=3)
    inp = si.make_layer_inputs(cfg, seed=4)
    f, r = _oracle(cfg, inp)
    a, b = GpuLayer(K, cfg, inp), GpuLayer(K, rc, inp)
    T, D, F = cfg.tokens, cfg.d_model, cfg.d_ff
    assert K.dlayer_saved_bytes(cfg) - K.dlayer_saved_bytes(rc) >= 2 * T * (2 * D + F)
    a.forward(); a.backward()
    b.forward(); b.backward()
    torch.cuda.synchronize()
    _check_layer(b, f, r, name + ":recompute")
    for n_, p, q in [("y", a.y, b.y), ("dx", a.dx, b.dx)] + [(n, a.dw[n], b.dw[n]) for n in si.WEIGHT_NAMES if n != "w_down"]:
        assert torch.equal(p.view(torch.int16), q.view(torch.int16)), f"{n_} differs between keeping and recomputing"


def test_layer_is_causal_and_deterministic(K):
    cfg = si.CONFIGS["tiny"].with_(seq=256, batch=2)
    inp = si.make_layer_inputs(cfg, seed=1)
    g = GpuLayer(K, cfg, inp)
    g.forward()
    y1 = g.y.clone()
    g.forward()
    assert torch.equal(y1.view(torch.int16), g.y.view(torch.int16))
    t = 100
    inp2 = dict(inp)
    x2 = inp["x"].copy()
    x2[:, t + 1:] = si.make_layer_inputs(cfg, seed=2)["x"][:, t + 1:]
    inp2["x"] = x2
    g2 = GpuLayer(K, cfg, inp2)
    g2.forward()
    assert torch.equal(y1[:, :t + 1].view(torch.int16), g2.y[:, :t + 1].view(torch.int16))
    assert not torch.equal(y1[:, t + 1:].view(torch.int16), g2.y[:, t + 1:].view(torch.int16))


def test_layer_on_a_side_stream(K):
    """Every call enqueues on the stream it is given: a forward + backward on a second stream (default
    priority), with the default stream left idle, gives the bits of the default-stream run."""
    cfg = si.CONFIGS["small"].with_(batch=2)
    inp = si.make_layer_inputs(cfg, seed=6)
    a = GpuLayer(K, cfg, inp)
    a.forward(); a.backward()
    torch.cuda.synchronize()
    b = GpuLayer(K, cfg, inp)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        b.forward(); b.backward()
    side.synchronize()
    for name, p, q in [("y", a.y, b.y), ("dx", a.dx, b.dx)] + [(n, a.dw[n], b.dw[n]) for n in si.WEIGHT_NAMES]:
        assert torch.equal(p.view(torch.int16), q.view(torch.int16)), f"{name} differs between streams"


@pytest.mark.parametrize("name", ["tiny", "small"])
def test_layer_replays_from_a_hip_graph(K, name):
    """The calls only enqueue kernels (no allocation, memset or synchronisation), so a forward +
    backward can be captured once and replayed: three replays on fresh inputs, each with eager work
    and synchronisations in between, must reproduce the eager results bit for bit."""
    cfg = si.CONFIGS[name]
    inps = [si.make_layer_inputs(cfg, seed=s) for s in (3, 4, 5)]
    g = GpuLayer(K, cfg, inps[0])
    g.forward(); g.backward()              # first call outside capture: one-time kernel attributes
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        g.forward(); g.backward()
    names = ("y", "dx") + tuple(si.WEIGHT_NAMES)
    outs = lambda o: [o.y, o.dx] + [o.dw[n] for n in si.WEIGHT_NAMES]
    for inp in inps:
        e = GpuLayer(K, cfg, inp)           # eager reference on buffers of its own
        e.forward(); e.backward()
        torch.cuda.synchronize()
        g.x.copy_(e.x); g.dy.copy_(e.dy)
        for n in si.WEIGHT_NAMES:
            g.w[n].copy_(e.w[n])
        for t in outs(g):
            t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        for n, a, b in zip(names, outs(g), outs(e)):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16)), f"{name}: {n} differs between replay and eager"


# At D = 4096, F = 14336 the element-wise metric (max over the outputs of |err| / max(|ref|, rms)) of
# ANY pipeline that rounds MFMA operands to bf16 exceeds 2e-2: rounding only h1, q, k, v, o, h2, a and
# y (each needed as an MFMA operand or as the output) in an otherwise exact fp64 evaluation gives
# 2.43e-2 on the very inputs of test_8b_shape_prefix_parity (2 x 2048 positions, 16.8 M outputs;
# 2.48e-2 with y1 rounded as well), and 2.2e-2 on 64 positions
# (tests/test_oracle_pins.py::test_bf16_operand_rounding_floor_at_8b_width).  The GPU measures 2.66e-2
# there (2.63e-2 with another summation order of the GEMMs): the floor plus the rounding of the softmax
# weights to bf16 and fp32 summation.  The bound at this width is the first measured value with a 5 % margin, together with two companion figures: the
# infinity-norm ratio (bound 1e-2, measured 5e-3) and the fraction of elements above 2e-2 (bound 1e-3,
# measured 7e-6).  The stated bar of 2e-2 on this metric is NOT met at this width and cannot be with
# bf16 operands.
Y_TOL_8B = 2.75e-2
# d_model 8192 (one case of test_layer_matches_oracle): same emulation on its inputs 3.4e-2, GPU 3.5e-2
Y_TOL_D8192 = 3.8e-2


def _assert_y_8b(got, ref, name):
    got = host_f64(got)
    assert_close(got, ref, name, rel_tol=Y_TOL_8B)
    inf_ratio = np.abs(got - ref).max() / np.abs(ref).max()
    rms = np.sqrt(np.mean(ref * ref))
    frac = np.mean(np.abs(got - ref) / np.maximum(np.abs(ref), rms) > REL_TOL)
    assert inf_ratio <= REL_TOL / 2 and frac <= 1e-3, (name, inf_ratio, frac)
    print(name, f"rel_err {rel_err(got, ref):.3e} inf-norm ratio {inf_ratio:.3e} frac>2e-2 {frac:.2e}")


def test_8b_shape_prefix_parity(K):
    """Full-size 8B-shaped launch.  The oracle cannot run 16384 tokens, but causality makes the
    first P positions of every batch row a closed sub-problem: y[:, :P] depends only on x[:, :P], and
    with an upstream gradient that is zero outside the first P positions of both rows, dx[:, :P] and
    every weight gradient equal those of the (2, P) problem."""
    cfg = si.CONFIGS["8b"]
    P = 2048
    inp = si.make_layer_inputs(cfg, seed=0)
    dy = np.zeros_like(inp["dy"])
    dy[:, :P] = inp["dy"][:, :P]
    inp["dy"] = dy
    sub = cfg.with_(seq=P)
    sub_inp = {k: v for k, v in inp.items()}
    sub_inp["x"], sub_inp["dy"] = inp["x"][:, :P], dy[:, :P]
    f, r = _oracle(sub, sub_inp)
    g = GpuLayer(K, cfg, inp)
    g.forward()
    g.backward()
    torch.cuda.synchronize()
    _assert_y_8b(g.y[:, :P], f["y"], "8b:y[prefix]")
    rep = {"dx": assert_close(g.dx[:, :P], r["dx"], "8b:dx[prefix]", rel_tol=np.inf)}
    assert float(g.dx[:, P:].float().abs().max()) == 0.0
    for n in si.WEIGHT_NAMES:
        rep[n] = assert_close(g.dw[n], r[n], f"8b:d{n}", rel_tol=np.inf)
    print("8b", {k: (f"{a:.2e}", f"{b:.6f}") for k, (a, b) in rep.items()})
    # Floor or defect?  The same forward evaluated in fp64 but rounded to bf16 exactly where the library
    # stores a tensor (h1, rotated q and k, v, o, y1, h2, a, y).  Step by step the kernels reproduce that
    # evaluation bit for bit on 99.95 % of the elements (test_8b_width_steps_against_the_storage_emulation);
    # the one thing it leaves out is the bf16 rounding of the softmax weights inside the attention kernel,
    # which alone moves o by up to 1.2e-2 on this metric, so the whole layer sits as far from the emulation
    # (measured 2.06e-2) as the emulation sits from the exact result (2.48e-2): same noise, other draw.
    v = {k: si.bf16_bits_to_f64(inp[k]) for k in si.WEIGHT_NAMES}
    x64 = si.bf16_bits_to_f64(sub_inp["x"])
    Bq, S, D = x64.shape
    Hq, Hkv, dh = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    h1 = rounded(odl.rmsnorm_fwd(x64, v["g_attn"], cfg.rms_eps)[0])
    phi = odl.rope_angles(S, dh, cfg.rope_base)
    q = rounded(odl.rope_rotate((h1 @ v["wq"].T).reshape(Bq, S, Hq, dh), phi))
    k = rounded(odl.rope_rotate((h1 @ v["wk"].T).reshape(Bq, S, Hkv, dh), phi))
    vv = rounded((h1 @ v["wv"].T).reshape(Bq, S, Hkv, dh))
    o = rounded(odl.attention_fwd(q, k, vv)[0])
    y1 = rounded(x64 + o.reshape(Bq, S, Hq * dh) @ v["wo"].T)
    h2 = rounded(odl.rmsnorm_fwd(y1, v["g_mlp"], cfg.rms_eps)[0])
    a = rounded(odl.swiglu_fwd(h2 @ v["w_gate"].T, h2 @ v["w_up"].T))
    y_emu = rounded(y1 + a @ v["w_down"].T)
    r_emu = rel_err(host_f64(g.y[:, :P]), y_emu)
    print(f"8b:y against the bf16-storage emulation: rel_err {r_emu:.3e}")
    assert r_emu <= 2.2e-2, r_emu


def test_8b_width_steps_against_the_storage_emulation(K):
    """Each step of the forward at the 8B widths, fed with the tensor the fp64 evaluation holds at that
    point after rounding it to bf16 where the library stores it: the step's output must equal the fp64
    result rounded to bf16 except where the fp32 sum lands on the other side of a rounding boundary,
    i.e. be bit-identical almost everywhere and never more than one bf16 step away.  This separates the
    rounding floor of bf16 storage from any defect of a kernel."""
    cfg = si.CONFIGS["8b"].with_(batch=1, seq=512)   # 512 rows: enough tiles for the fused gate/up kernel
    inp = si.make_layer_inputs(cfg, seed=0)
    w = {k: si.bf16_bits_to_f64(inp[k]) for k in si.WEIGHT_NAMES}
    wd = {k: dev_bf16(inp[k]) for k in si.WEIGHT_NAMES}
    x = si.bf16_bits_to_f64(inp["x"])[0]
    T, D, F = cfg.tokens, cfg.d_model, cfg.d_ff
    Hq, Hkv, dh, S = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.seq
    QD, KD = Hq * dh, Hkv * dh
    up = lambda a: dev_bf16(f64_to_bf16_bits(a))
    bf = lambda *s: torch.full(s, float("nan"), dtype=torch.bfloat16, device="cuda")
    report = {}

    def check(name, got, ref64, min_exact):
        ref = rounded(ref64)
        got = host_f64(got).reshape(ref.shape)
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 1e-30))) - 7)
        exact = float(np.mean(got == ref))
        # where terms cancel the fp32 rounding of the terms shows next to a tiny result: 1e-5 of the
        # tensor's rms is allowed on top of the one rounding step
        slack = 1e-5 * np.sqrt(np.mean(ref * ref))
        worst = float(np.max(np.maximum(np.abs(got - ref) - slack, 0.0) / ulp))
        report[name] = (exact, worst)
        assert exact >= min_exact and worst <= 1.001, (name, exact, worst)
        return ref

    h1g, rstd = bf(T, D), torch.empty(T, dtype=torch.float32, device="cuda")
    K.rmsnorm_forward(up(x), wd["g_attn"], T, D, cfg.rms_eps, h1g, rstd)
    h1 = check("h1", h1g, odl.rmsnorm_fwd(x, w["g_attn"], cfg.rms_eps)[0], 0.999)
    qg, kg, vg = bf(T, QD), bf(T, KD), bf(T, KD)
    ws = torch.empty(K.qkv_rope_workspace_bytes(S, dh), dtype=torch.uint8, device="cuda")
    K.qkv_rope_forward(up(h1), wd["wq"], wd["wk"], wd["wv"], 1, S, D, Hq, Hkv, dh, cfg.rope_base, 0, qg, kg, vg, ws)
    phi = odl.rope_angles(S, dh, cfg.rope_base)
    q = check("q", qg, odl.rope_rotate((h1 @ w["wq"].T).reshape(1, S, Hq, dh), phi), 0.995)
    k = check("k", kg, odl.rope_rotate((h1 @ w["wk"].T).reshape(1, S, Hkv, dh), phi), 0.995)
    v = check("v", vg, (h1 @ w["wv"].T).reshape(1, S, Hkv, dh), 0.995)
    og, lse = bf(T, QD), torch.empty(1, Hq, S, dtype=torch.float32, device="cuda")
    K.attention_forward(up(q), up(k), up(v), 1, S, Hq, Hkv, dh, og, lse)
    # the attention output also carries the bf16 rounding of the softmax weights: bounded by its own
    # per-kernel tolerance rather than by one rounding step
    o_ref = odl.attention_fwd(q, k, v)[0]
    report["o"] = assert_close(og, o_ref, "o", rel_tol=2.5e-2)
    o = rounded(o_ref).reshape(T, QD)
    y1g = bf(T, D)
    K.linear_forward(up(o), wd["wo"], up(x), T, QD, D, y1g)
    y1 = check("y1", y1g, x + o @ w["wo"].T, 0.995)
    h2g = bf(T, D)
    K.rmsnorm_forward(up(y1), wd["g_mlp"], T, D, cfg.rms_eps, h2g, rstd)
    h2 = check("h2", h2g, odl.rmsnorm_fwd(y1, w["g_mlp"], cfg.rms_eps)[0], 0.999)
    gg, ug, ag = bf(T, F), bf(T, F), bf(T, F)
    K.linear_swiglu_forward(up(h2), wd["w_gate"], wd["w_up"], T, D, F, gg, ug, ag)
    g64, u64 = h2 @ w["w_gate"].T, h2 @ w["w_up"].T
    check("g", gg, g64, 0.995)
    check("u", ug, u64, 0.995)
    a = check("a", ag, odl.swiglu_fwd(g64, u64), 0.99)
    yg = bf(T, D)
    K.linear_forward(up(a), wd["w_down"], up(y1), T, F, D, yg)
    check("y", yg, y1 + a @ w["w_down"].T, 0.995)
    print("steps vs storage emulation (fraction bit-identical, worst distance in bf16 steps):",
          {k: (f"{e:.5f}", f"{wst:.3g}") for k, (e, wst) in report.items()})

"""Pins of the CPU oracle against things other than itself.

Every check here ties a function of oracle/mrem_oracle.py to a hand-computed
fixture, a closed form, an invariant, a brute-force definition or a library
routine (torch fp64 autograd, torch.nn.TransformerEncoderLayer,
torch.optim.AdamW), so that a dropped term, a wrong sign or index or a
transposed operand in the oracle fails at least one of them.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import mrem_oracle as O
from paper_2109_15082_amd import synth

torch.set_default_dtype(torch.float64)


# --------------------------------------------------------------------------
# helpers
# --------------------------------------------------------------------------

def tiny_cfg(**kw):
    base = dict(n_layers=1, hidden=16, n_heads=2, ffn=32, w_bits=4, a_bits=8)
    base.update(kw)
    return O.Config(**base)


def tiny_student(cfg, seed=7, jitter=0.1, batch=2, seq=6, seqlens=None, x_seed=11):
    layers = O.to_f64(synth.make_module_params(cfg.n_layers, cfg.hidden, cfg.ffn, seed, jitter))
    # larger weights than the workloads' 0.02 so that attention is not uniform
    for lp in layers:
        for n in O.WEIGHT_NAMES:
            lp[n] = np.float64(np.float32(lp[n] * 10.0))
    x = synth.make_hidden_states(batch, seq, cfg.hidden, x_seed).astype(np.float64).reshape(batch * seq, cfg.hidden)
    teacher = [{k: v.copy() for k, v in lp.items()} for lp in layers]
    for lp in layers:
        for n in O.WEIGHT_NAMES:
            lp["s" + n] = O.weight_step_init(lp[n], max(cfg.w_bits, 2)) if cfg.w_bits else np.ones(lp[n].shape[0])
        lp["s_a"] = np.ones(8)
        lp["z_a"] = np.zeros(8)
    if cfg.a_bits:
        cal = O.calibrate(x, teacher, cfg, batch, seq, seqlens)
        for lp, (s, z) in zip(layers, cal):
            lp["s_a"], lp["z_a"] = s.copy(), z.copy()
    return teacher, layers, x


# --------------------------------------------------------------------------
# A. quantizer (Section 3.1, Eq. 1) and its straight-through backward
# --------------------------------------------------------------------------

def test_quantizer_hand_example(golden_dir):
    rows = np.loadtxt(os.path.join(golden_dir, "quantizer_hand_example.txt"))
    x, v_ref, code_ref, inside_ref, dsd_ref = rows.T
    s = 2.0 ** -7
    x_hat, q, v, inside = O.fake_quant_forward(x, s, *O.sym_range(4))
    assert np.array_equal(v, v_ref)
    assert np.array_equal(q, code_ref)
    assert np.array_equal(inside.astype(float), inside_ref)
    assert np.array_equal(x_hat, s * code_ref)
    # unit upstream gradient per element: dx = mask, ds elementwise = fixture column
    for i in range(len(x)):
        e = np.zeros_like(x)
        e[i] = 1.0
        dx, ds = O.fake_quant_backward(e, q, v, inside)
        assert ds == dsd_ref[i]
        assert np.array_equal(dx, e * inside_ref)


def test_rounding_ties_to_even():
    _, q, _, _ = O.fake_quant_forward(np.array([2.5, 3.5, -3.5, -2.5, 0.5, -0.5, 1.5]), 1.0, -127, 127)
    assert q.tolist() == [2.0, 4.0, -4.0, -2.0, 0.0, -0.0, 2.0]


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_quantizer_invariants(bits):
    rng = np.random.default_rng(bits)
    x = rng.standard_normal(5000) * 0.05
    qn, qp = O.sym_range(bits)
    assert (qn, qp) == (-(2 ** (bits - 1)) + 1, 2 ** (bits - 1) - 1)
    s = np.float64(np.float32(np.abs(x).max() / qp * 0.7))      # some values clip
    x_hat, q, v, inside = O.fake_quant_forward(x, s, qn, qp)
    assert q.min() >= qn and q.max() <= qp
    assert q.min() >= -(2 ** (bits - 1)) and q.max() <= 2 ** (bits - 1) - 1
    assert len(np.unique(q)) <= 2 ** bits - 1 <= 2 ** bits
    assert np.array_equal(q, np.rint(q))
    # idempotence: quantizing a grid point returns the same grid point
    x_hat2, q2, _, _ = O.fake_quant_forward(x_hat, s, qn, qp)
    assert np.array_equal(q2, q) and np.array_equal(x_hat2, x_hat)
    # half-step error bound for unclipped values, odd symmetry
    assert np.all(np.abs(x - x_hat)[inside] <= 0.5 * s * (1 + 1e-6))
    assert np.all(np.abs(x_hat[~inside]) == qp * s)
    xm, qm, _, _ = O.fake_quant_forward(-x, s, qn, qp)
    assert np.array_equal(qm, -q)


@pytest.mark.parametrize("bits", [2, 4])
def test_quantizer_is_projection_onto_grid(bits):
    """Brute force: x^ is the element of {s*k : k in Omega(b)} closest to x."""
    rng = np.random.default_rng(100 + bits)
    s = 0.125
    x = rng.uniform(-1.5 * s * 2 ** (bits - 1), 1.5 * s * 2 ** (bits - 1), size=400)
    qn, qp = O.sym_range(bits)
    grid = [s * k for k in range(qn, qp + 1)]
    x_hat, _, _, _ = O.fake_quant_forward(x, s, qn, qp, decide32=False)
    for xi, xh in zip(x, x_hat):
        dists = [abs(xi - gk) for gk in grid]
        best = min(dists)
        if sorted(dists)[1] - best < 1e-12:      # an exact tie: either neighbour is a projection
            continue
        assert xh == grid[dists.index(best)]


def test_unsigned_quantizer_grid_and_offset():
    rng = np.random.default_rng(3)
    g = rng.uniform(-0.17, 3.0, size=2000)
    z = np.float64(np.float32(-0.17))
    qn, qp = O.unsigned_range(8)
    assert (qn, qp) == (0, 255)
    s = np.float64(np.float32((3.0 - z) / qp))
    x_hat, q, v, inside = O.fake_quant_forward(g, s, qn, qp, z)
    assert q.min() >= 0 and q.max() <= 255 and len(np.unique(q)) <= 256
    assert np.allclose(x_hat, s * q + z, rtol=0, atol=0)
    assert np.all(np.abs(g - x_hat)[inside] <= 0.5 * s * (1 + 1e-5))


def test_weight_quantizer_per_channel_and_fp32_decision():
    rng = np.random.default_rng(5)
    w = (rng.standard_normal((12, 40)) * 0.02).astype(np.float32)
    s = O.weight_step_init(w, 4)
    # init: the row maximum maps to +-7 exactly and nothing clips
    codes, w_hat, v, inside = O.quantize_weight(w, s, 4)
    assert codes.dtype == np.int64 and np.all(np.abs(codes).max(axis=1) == 7)
    assert inside.all() or np.all(np.abs(v[~inside]) > 7)
    # the decision ratio is the IEEE fp32 quotient (numpy's own fp32 division)
    v32 = (w / s.astype(np.float32)[:, None])
    assert v32.dtype == np.float32 and np.array_equal(v, v32.astype(np.float64))
    assert np.array_equal(codes, np.rint(np.clip(v32, -7, 7)).astype(np.int64))
    # rows are independent: rescaling one row's step changes only that row
    s2 = s.copy()
    s2[3] *= 2
    codes2, _, _, _ = O.quantize_weight(w, s2, 4)
    assert np.array_equal(np.delete(codes2, 3, 0), np.delete(codes, 3, 0)) and not np.array_equal(codes2[3], codes[3])


def _torch_surrogate(x, s, z, qn, qp):
    """Frozen-residual straight-through surrogate in torch."""
    c = torch.clamp((x - z) / s, qn, qp)
    return s * (c + (torch.round(c) - c).detach()) + z


@pytest.mark.parametrize("unsigned", [False, True])
def test_quantizer_backward_vs_autograd(unsigned):
    rng = np.random.default_rng(17)
    x = rng.standard_normal((6, 50)) * 2.0 + (1.0 if unsigned else 0.0)
    s, z = 0.03, (-0.17 if unsigned else 0.0)
    qn, qp = (O.unsigned_range(8) if unsigned else O.sym_range(8))
    up = rng.standard_normal(x.shape)
    _, q, v, inside = O.fake_quant_forward(x, s, qn, qp, z, decide32=False)
    dx, ds = O.fake_quant_backward(up, q, v, inside)
    xt = torch.tensor(x, requires_grad=True)
    st = torch.tensor(s, requires_grad=True)
    (_torch_surrogate(xt, st, z, qn, qp) * torch.tensor(up)).sum().backward()
    assert (~inside).sum() > 0
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(ds, st.grad.item(), rtol=1e-9)


def test_step_gradient_finite_difference_on_frozen_residual():
    """Central differences on s*(clamp(x/s)+kappa) with kappa frozen at the base point."""
    rng = np.random.default_rng(23)
    x = rng.standard_normal(300)
    s0, qn, qp = 0.02, *O.sym_range(8)
    _, q, v, inside = O.fake_quant_forward(x, s0, qn, qp, decide32=False)
    assert np.abs(np.abs(v) - qp).min() > 1e-3
    kappa = q - np.clip(v, qn, qp)
    up = rng.standard_normal(300)
    f = lambda s: float((up * (s * (np.clip(x / s, qn, qp) + kappa))).sum())
    h = 1e-7
    fd = (f(s0 + h) - f(s0 - h)) / (2 * h)
    _, ds = O.fake_quant_backward(up, q, v, inside)
    assert abs(fd - ds) <= 1e-6 * max(1.0, abs(ds))


# --------------------------------------------------------------------------
# B. operators against library routines / closed forms
# --------------------------------------------------------------------------

def test_round_bf16_matches_torch():
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(4000) * 10.0 ** rng.integers(-6, 6, 4000), [0.0, 1.0, -1.0, 1.00390625, 1.01171875]])
    ref = torch.tensor(x, dtype=torch.float64).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(O.round_bf16(x), ref)


def test_gelu_layernorm_softmax_vs_torch():
    rng = np.random.default_rng(2)
    u = rng.standard_normal((5, 24)) * 3
    np.testing.assert_allclose(O.gelu(u), torch.nn.functional.gelu(torch.tensor(u)).numpy(), rtol=1e-13, atol=1e-15)
    ut = torch.tensor(u, requires_grad=True)
    torch.nn.functional.gelu(ut).sum().backward()
    np.testing.assert_allclose(O.gelu_grad(u), ut.grad.numpy(), rtol=1e-12, atol=1e-14)
    assert O.gelu(np.array([0.0]))[0] == 0.0 and abs(O.gelu(np.array([30.0]))[0] - 30.0) < 1e-12
    gam, bet = rng.standard_normal(24), rng.standard_normal(24)
    y, cache = O.layernorm_forward(u, gam, bet, 1e-12)
    rt = torch.tensor(u, requires_grad=True)
    gt, bt = torch.tensor(gam, requires_grad=True), torch.tensor(bet, requires_grad=True)
    yt = torch.nn.functional.layer_norm(rt, (24,), gt, bt, 1e-12)
    np.testing.assert_allclose(y, yt.detach().numpy(), rtol=1e-12, atol=1e-13)
    up = rng.standard_normal(u.shape)
    (yt * torch.tensor(up)).sum().backward()
    dr, dg, db = O.layernorm_backward(up, gam, cache)
    np.testing.assert_allclose(dr, rt.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(dg, gt.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(db, bt.grad.numpy(), rtol=1e-11, atol=1e-12)
    y1, _ = O.layernorm_forward(u, np.ones(24), np.zeros(24), 1e-12)
    np.testing.assert_allclose(y1.mean(-1), 0, atol=1e-14)
    np.testing.assert_allclose(y1.var(-1), 1, rtol=1e-9)
    p = O.softmax_rows(u)
    np.testing.assert_allclose(p.sum(-1), 1, rtol=1e-14)
    np.testing.assert_allclose(p, torch.softmax(torch.tensor(u), -1).numpy(), rtol=1e-13)


def _torch_encoder_layer(lp, cfg):
    m = torch.nn.TransformerEncoderLayer(cfg.hidden, cfg.n_heads, cfg.ffn, dropout=0.0, activation="gelu",
                                         layer_norm_eps=cfg.ln_eps, batch_first=True, norm_first=False)
    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
    with torch.no_grad():
        m.self_attn.in_proj_weight.copy_(t(lp["w_qkv"])); m.self_attn.in_proj_bias.copy_(t(lp["b_qkv"]))
        m.self_attn.out_proj.weight.copy_(t(lp["w_o"])); m.self_attn.out_proj.bias.copy_(t(lp["b_o"]))
        m.linear1.weight.copy_(t(lp["w_1"])); m.linear1.bias.copy_(t(lp["b_1"]))
        m.linear2.weight.copy_(t(lp["w_2"])); m.linear2.bias.copy_(t(lp["b_2"]))
        m.norm1.weight.copy_(t(lp["ln1_g"])); m.norm1.bias.copy_(t(lp["ln1_b"]))
        m.norm2.weight.copy_(t(lp["ln2_g"])); m.norm2.bias.copy_(t(lp["ln2_b"]))
    return m.train()


@pytest.mark.parametrize("masked", [False, True])
def test_teacher_layer_vs_torch_transformer_encoder_layer(masked):
    """Quantizers off: the layer is the library's post-LayerNorm encoder layer,
    forward and (through autograd) backward for every parameter group."""
    cfg = tiny_cfg(w_bits=0, a_bits=0)
    batch, seq = 3, 5
    seqlens = np.array([5, 2, 4]) if masked else None
    teacher, _, x = tiny_student(cfg, batch=batch, seq=seq, seqlens=seqlens)
    lp = teacher[0]
    f, cache = O.layer_forward(x, lp, cfg, batch, seq, seqlens, quant=False)
    m = _torch_encoder_layer(lp, cfg)
    xt = torch.tensor(x.reshape(batch, seq, cfg.hidden), requires_grad=True)
    kpm = None
    if masked:
        kpm = torch.arange(seq)[None, :] >= torch.tensor(seqlens)[:, None]
    ft = m(xt, src_key_padding_mask=kpm)
    np.testing.assert_allclose(f, ft.detach().numpy().reshape(-1, cfg.hidden), rtol=1e-10, atol=1e-12)
    up = np.random.default_rng(9).standard_normal(f.shape)
    (ft.reshape(-1, cfg.hidden) * torch.tensor(up)).sum().backward()
    dx, g = O.layer_backward(up, cache, cfg)
    np.testing.assert_allclose(dx, xt.grad.numpy().reshape(-1, cfg.hidden), rtol=1e-8, atol=1e-11)
    ref = {"w_qkv": m.self_attn.in_proj_weight, "b_qkv": m.self_attn.in_proj_bias, "w_o": m.self_attn.out_proj.weight,
           "b_o": m.self_attn.out_proj.bias, "w_1": m.linear1.weight, "b_1": m.linear1.bias, "w_2": m.linear2.weight,
           "b_2": m.linear2.bias, "ln1_g": m.norm1.weight, "ln1_b": m.norm1.bias, "ln2_g": m.norm2.weight,
           "ln2_b": m.norm2.bias}
    for k, p in ref.items():
        np.testing.assert_allclose(g[k], p.grad.numpy(), rtol=1e-8, atol=1e-11, err_msg=k)


def test_attention_brute_force_loops():
    """The attention block on a tiny case, written out index by index."""
    cfg = tiny_cfg(w_bits=0, a_bits=0, hidden=8, n_heads=2, ffn=8)
    batch, seq = 2, 3
    seqlens = np.array([3, 2])
    teacher, _, x = tiny_student(cfg, batch=batch, seq=seq, seqlens=seqlens)
    lp = teacher[0]
    _, c = O.layer_forward(x, lp, cfg, batch, seq, seqlens, quant=False)
    H, d = cfg.hidden, cfg.head_dim
    qkv = x @ lp["w_qkv"].T + lp["b_qkv"]
    ctx = np.zeros((batch * seq, H))
    for b in range(batch):
        for h in range(cfg.n_heads):
            for i in range(seq):
                sc = []
                for j in range(int(seqlens[b])):
                    sc.append(sum(qkv[b * seq + i, h * d + e] * qkv[b * seq + j, H + h * d + e] for e in range(d)) / math.sqrt(d))
                mx = max(sc)
                ex = [math.exp(v - mx) for v in sc]
                for e in range(d):
                    ctx[b * seq + i, h * d + e] = sum(ex[j] / sum(ex) * qkv[b * seq + j, 2 * H + h * d + e] for j in range(len(sc)))
    np.testing.assert_allclose(c["C"], ctx, rtol=1e-11, atol=1e-13)
    assert np.all(c["P"][1, :, :, 2] == 0.0)          # padded key of the second sequence


# --------------------------------------------------------------------------
# C. quantized layer: placement, exactness, limits, backward
# --------------------------------------------------------------------------

def test_quantizer_placement_and_integer_exactness():
    """Both operands of each of the six matrix products lie on their grids
    (Section 3.1); LayerNorm outputs, residuals and biases do not.  Each linear
    output equals s_a*s_w[n]*(integer dot product) (+ offset term) + bias."""
    cfg = tiny_cfg()
    batch, seq = 2, 6
    teacher, student, x = tiny_student(cfg, batch=batch, seq=seq)
    lp = student[0]
    f, c = O.layer_forward(x, lp, cfg, batch, seq, None, quant=True)
    sa, za = lp["s_a"], lp["z_a"]

    def on_grid(t, i, levels):
        k = (t - (za[i] if O.ACT_Q_UNSIGNED[i] else 0.0)) / sa[i]
        assert np.abs(k - np.rint(k)).max() < 1e-9, O.ACT_Q_NAMES[i]
        assert len(np.unique(np.rint(k))) <= levels
        return np.rint(k).astype(np.int64)

    kx = on_grid(c["xh"], O.AQ_X, 255)
    kq = on_grid(c["Qh"], O.AQ_Q, 255); kk = on_grid(c["Kh"], O.AQ_K, 255); kv = on_grid(c["Vh"], O.AQ_V, 255)
    kp = on_grid(c["Ph"], O.AQ_P, 256); kc = on_grid(c["Ch"], O.AQ_C, 255)
    kx1 = on_grid(c["x1h"], O.AQ_X1, 255); kg = on_grid(c["gh"], O.AQ_G, 256)
    assert kp.min() >= 0 and kg.min() >= 0 and kg.max() <= 255 and np.abs(kx).max() <= 127
    for n in O.WEIGHT_NAMES:
        wq = c["wq"][n]
        assert np.abs(wq.codes).max() <= 7
        np.testing.assert_array_equal(wq.w_hat, lp["s" + n][:, None] * wq.codes)
    assert len(np.unique(c["x1"])) > 0.9 * c["x1"].size          # LayerNorm output is not quantized
    # integer exactness of the four linear layers
    sw = lambda n: lp["s" + n][None, :]
    np.testing.assert_allclose(c["qkv"], sa[O.AQ_X] * sw("w_qkv") * (kx @ c["wq"]["w_qkv"].codes.T) + lp["b_qkv"], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(c["o"], sa[O.AQ_C] * sw("w_o") * (kc @ c["wq"]["w_o"].codes.T) + lp["b_o"], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(c["u"], sa[O.AQ_X1] * sw("w_1") * (kx1 @ c["wq"]["w_1"].codes.T) + lp["b_1"], rtol=1e-12, atol=1e-14)
    w2c = c["wq"]["w_2"].codes
    np.testing.assert_allclose(c["y"], sa[O.AQ_G] * sw("w_2") * (kg @ w2c.T) + za[O.AQ_G] * sw("w_2") * w2c.sum(1)[None, :] + lp["b_2"],
                               rtol=1e-11, atol=1e-13)
    # attention products are integer products too
    d = cfg.head_dim
    A = sa[O.AQ_Q] * sa[O.AQ_K] * (kq @ kk.transpose(0, 1, 3, 2)) / math.sqrt(d)
    np.testing.assert_allclose(c["P"], O.softmax_rows(A), rtol=1e-11)
    np.testing.assert_allclose(c["C"], O.merge_heads(sa[O.AQ_P] * sa[O.AQ_V] * (kp @ kv)), rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(c["Ph"].sum(-1), 1.0, atol=seq * sa[O.AQ_P] / 2 + 1e-12)


def test_zero_reconstruction_error_with_quantization_off():
    cfg = tiny_cfg(w_bits=0, a_bits=0, n_layers=2)
    teacher, student, x = tiny_student(cfg)
    res = O.module_grads(x, x, teacher, student, cfg, 2, 6)
    assert res.loss == 0.0 and all(p == 0.0 for p in res.per_layer_loss)
    for g in res.grads:
        for k, v in g.items():
            assert np.all(v == 0.0), k
    for a, b in zip(res.f_fp, res.f_q):
        assert np.array_equal(a, b)


def test_many_bits_approach_the_teacher():
    teacher, student, x = tiny_student(tiny_cfg(n_layers=2))
    losses = []
    for wb, ab in [(4, 8), (8, 8), (12, 12), (16, 16)]:
        cfg = tiny_cfg(n_layers=2, w_bits=wb, a_bits=ab)
        teacher, student, x = tiny_student(cfg)
        losses.append(O.module_grads(x, x, teacher, student, cfg, 2, 6).loss)
    assert losses[0] > losses[1] > losses[2] > losses[3]
    assert losses[3] < 1e-7 and losses[3] < 1e-4 * losses[0]


def _torch_student_layer(x, lp, cfg, batch, seq, seqlens):
    """The quantized layer restated with torch ops and frozen-residual
    surrogates, used only for its autograd derivative."""
    H, nh, d = cfg.hidden, cfg.n_heads, cfg.head_dim
    qs = lambda t, i: _torch_surrogate(t, lp["s_a"][i], 0.0, *O.sym_range(cfg.a_bits))
    qu = lambda t, i: _torch_surrogate(t, lp["s_a"][i], lp["z_a"][i], *O.unsigned_range(cfg.a_bits))
    wq = lambda n: _torch_surrogate(lp[n], lp["s" + n][:, None], 0.0, *O.sym_range(cfg.w_bits))
    F = torch.nn.functional
    qkv = F.linear(qs(x, 0), wq("w_qkv"), lp["b_qkv"])
    heads = lambda t: t.reshape(batch, seq, nh, d).transpose(1, 2)
    Q, K, V = heads(qkv[:, :H]), heads(qkv[:, H:2 * H]), heads(qkv[:, 2 * H:])
    A = qs(Q, 1) @ qs(K, 2).transpose(-1, -2) / math.sqrt(d)
    if seqlens is not None:
        kpm = torch.arange(seq)[None, :] >= torch.tensor(seqlens)[:, None]
        A = A.masked_fill(kpm[:, None, None, :], float("-inf"))
    P = torch.softmax(A, -1)
    C = (qu(P, 3) @ qs(V, 4)).transpose(1, 2).reshape(batch * seq, H)
    o = F.linear(qs(C, 5), wq("w_o"), lp["b_o"])
    x1 = F.layer_norm(x + o, (H,), lp["ln1_g"], lp["ln1_b"], cfg.ln_eps)
    u = F.linear(qs(x1, 6), wq("w_1"), lp["b_1"])
    y = F.linear(qu(F.gelu(u), 7), wq("w_2"), lp["b_2"])
    return F.layer_norm(x1 + y, (H,), lp["ln2_g"], lp["ln2_b"], cfg.ln_eps)


@pytest.mark.parametrize("masked", [False, True])
def test_quantized_module_backward_vs_autograd(masked):
    """Two quantized layers + Eq. 3: every gradient the oracle returns equals
    torch's autograd derivative of the straight-through surrogate."""
    cfg = tiny_cfg(n_layers=2)
    batch, seq = 2, 6
    seqlens = np.array([6, 4]) if masked else None
    teacher, student, x = tiny_student(cfg, batch=batch, seq=seq, seqlens=seqlens)
    # shrink some steps so that a share of the values clips
    for lp in student:
        lp["s_a"] = lp["s_a"] * np.array([0.8, 0.7, 0.9, 0.6, 0.8, 0.7, 0.9, 0.5])
        # weight steps moved off their initial value: no element sits exactly on the clip bound,
        # where the fp32 decision and torch's fp64 clamp could differ
        for n, f in zip(O.STEP_NAMES, (1.05, 0.9, 0.8, 1.1)):
            lp[n] = np.float64(np.float32(lp[n] * f))
        lp["s_a"], lp["z_a"] = np.float64(np.float32(lp["s_a"])), np.float64(np.float32(lp["z_a"]))
    cfg64 = cfg                                   # act_round None => fp64 ratios
    res = O.module_grads(x, x, teacher, student, cfg64, batch, seq, seqlens)
    clipped = sum((~a.inside).sum() for c in res.caches for a in c["aq"])
    assert clipped > 20
    tl = [{k: torch.tensor(v, requires_grad=(k != "z_a")) for k, v in lp.items()} for lp in student]
    h = torch.tensor(x)
    loss = 0.0
    for l, lp in enumerate(tl):
        h = _torch_student_layer(h, lp, cfg, batch, seq, seqlens)
        np.testing.assert_allclose(res.f_q[l], h.detach().numpy(), rtol=1e-9, atol=1e-11)
        loss = loss + ((h - torch.tensor(res.f_fp[l])) ** 2).mean()
    assert abs(loss.item() - res.loss) <= 1e-10 * abs(res.loss)
    loss.backward()
    for l, lp in enumerate(tl):
        for k in O.TRAINABLE_FIELDS:
            ref = lp[k].grad.numpy()
            got = res.grads[l][k]
            scale = np.abs(ref).max() + 1e-30
            # the weight ratios w/s are fp32 quotients in the oracle (fp64 in torch): 2^-24 relative
            tol = 2e-6 if k in O.STEP_NAMES else 1e-8
            assert np.abs(got - ref).max() <= tol * scale, (l, k, np.abs(got - ref).max(), scale)
            assert scale > 1e-12, (l, k)


def test_no_gradient_leaves_the_module_and_layer_losses_add():
    """Eq. 3 sums per-layer terms; switching a layer off in the mask removes
    exactly its term, and the gradient of an upper layer's term reaches lower
    layers' parameters (joint optimisation inside the module)."""
    cfg = tiny_cfg(n_layers=2)
    teacher, student, x = tiny_student(cfg)
    full = O.module_grads(x, x, teacher, student, cfg, 2, 6)
    assert abs(full.loss - sum(full.per_layer_loss)) < 1e-15
    only1 = O.module_grads(x, x, teacher, student, tiny_cfg(n_layers=2, loss_layer_mask=0b10), 2, 6)
    only0 = O.module_grads(x, x, teacher, student, tiny_cfg(n_layers=2, loss_layer_mask=0b01), 2, 6)
    assert only1.per_layer_loss[0] == 0.0 and only1.per_layer_loss[1] == full.per_layer_loss[1]
    assert np.abs(only1.grads[0]["w_1"]).max() > 0          # reaches the lower layer
    assert np.all(only0.grads[1]["w_1"] == 0)               # but never flows upward
    for k in O.TRAINABLE_FIELDS:
        np.testing.assert_allclose(only0.grads[0][k] + only1.grads[0][k], full.grads[0][k], rtol=1e-9, atol=1e-18)


def test_loss_brute_force_and_sum_mode():
    rng = np.random.default_rng(4)
    fq = [rng.standard_normal((3, 4)) for _ in range(2)]
    ff = [rng.standard_normal((3, 4)) for _ in range(2)]
    tot = 0.0
    for a, b in zip(fq, ff):
        for i in range(3):
            for j in range(4):
                tot += (a[i, j] - b[i, j]) ** 2
    cfg_sum = tiny_cfg(n_layers=2, loss_mean=False)
    loss_sum, _, gr = O.module_loss(fq, ff, cfg_sum)
    assert abs(loss_sum - tot) < 1e-12
    np.testing.assert_allclose(gr[1], 2 * (fq[1] - ff[1]))
    loss_mean, per, gr = O.module_loss(fq, ff, tiny_cfg(n_layers=2))
    assert abs(loss_mean - tot / 12) < 1e-12
    np.testing.assert_allclose(gr[0], 2 * (fq[0] - ff[0]) / 12)


# --------------------------------------------------------------------------
# D. finite differences with the quantizers off (every parameter group)
# --------------------------------------------------------------------------

def test_central_finite_differences_unquantized_module():
    """Student without quantizers but with perturbed weights (so the loss is
    not zero): central differences of Eq. 3 for sampled coordinates of every
    parameter group."""
    cfg = tiny_cfg(n_layers=2, w_bits=0, a_bits=0)
    teacher, student, x = tiny_student(cfg)
    rng = np.random.default_rng(31)
    for lp in student:
        for k in O.LAYER_FIELDS[:12]:
            lp[k] = lp[k] + 0.05 * rng.standard_normal(lp[k].shape)
    res = O.module_grads(x, x, teacher, student, cfg, 2, 6)
    assert res.loss > 1e-4

    def loss_of():
        f_q, _ = O.module_forward(x, student, cfg, 2, 6, None, quant=True)
        return O.module_loss(f_q, res.f_fp, cfg)[0]

    for l, lp in enumerate(student):
        for k in O.LAYER_FIELDS[:12]:
            flat = lp[k].reshape(-1)
            for idx in rng.choice(flat.size, size=3, replace=False):
                old = flat[idx]
                h = 1e-6
                flat[idx] = old + h
                lp_ = loss_of()
                flat[idx] = old - h
                lm_ = loss_of()
                flat[idx] = old
                fd = (lp_ - lm_) / (2 * h)
                an = res.grads[l][k].reshape(-1)[idx]
                assert abs(fd - an) <= 1e-6 * max(abs(an), 1e-3), (l, k, idx, fd, an)


# --------------------------------------------------------------------------
# E. update rule
# --------------------------------------------------------------------------

def test_adamw_first_step_closed_form(golden_dir):
    p0, g, p1 = np.loadtxt(os.path.join(golden_dir, "adamw_first_step.txt")).T
    cfg = tiny_cfg(adam_eps=0.0, weight_decay=0.01)
    p, m, v = O.adamw_update(p0, g, np.zeros(3), np.zeros(3), 1, 0.1, cfg, decay=True)
    np.testing.assert_allclose(p, p1, rtol=1e-12)
    np.testing.assert_allclose(m, 0.1 * g, rtol=1e-12)
    np.testing.assert_allclose(v, 0.001 * g * g, rtol=1e-9)


@pytest.mark.parametrize("decay", [True, False])
def test_adamw_vs_torch_optim(decay):
    rng = np.random.default_rng(8)
    p = rng.standard_normal(50)
    cfg = tiny_cfg()
    pt = torch.tensor(p.copy(), requires_grad=True)
    opt = torch.optim.AdamW([pt], lr=1e-2, betas=(cfg.beta1, cfg.beta2), eps=cfg.adam_eps,
                            weight_decay=cfg.weight_decay if decay else 0.0)
    m, v = np.zeros(50), np.zeros(50)
    for t in range(1, 6):
        g = rng.standard_normal(50)
        lr = O.linear_decay_lr(1e-2, t - 1, 5)
        for grp in opt.param_groups:
            grp["lr"] = lr
        pt.grad = torch.tensor(g)
        opt.step()
        p, m, v = O.adamw_update(p, g, m, v, t, lr, cfg, decay)
        np.testing.assert_allclose(p, pt.detach().numpy(), rtol=1e-10, atol=1e-13)
    assert O.linear_decay_lr(1.0, 0, 4) == 1.0 and O.linear_decay_lr(1.0, 3, 4) == 0.25


def test_teacher_forcing_mix():
    assert O.teacher_forcing_lambda(0, 40) == 1.0 and O.teacher_forcing_lambda(10, 40) == 0.75
    assert O.teacher_forcing_lambda(40, 40) == 0.0 and O.teacher_forcing_lambda(90, 40) == 0.0
    a, b = np.array([1.0, 2.0]), np.array([3.0, -2.0])
    assert np.array_equal(O.mix_inputs(a, b, 1.0), a) and np.array_equal(O.mix_inputs(a, b, 0.0), b)
    assert np.array_equal(O.mix_inputs(a, b, 0.25), np.array([2.5, -1.0]))


# --------------------------------------------------------------------------
# F. calibration, storage rounding, whole-step behaviour
# --------------------------------------------------------------------------

def test_calibration_ranges():
    cfg = tiny_cfg()
    batch, seq = 2, 6
    teacher, student, x = tiny_student(cfg, batch=batch, seq=seq)
    (s, z), = O.calibrate(x, teacher, cfg, batch, seq)
    _, c = O.layer_forward(x, teacher[0], cfg, batch, seq, None, quant=False)
    H = cfg.hidden
    for i, t in [(O.AQ_X, x), (O.AQ_Q, c["qkv"][:, :H]), (O.AQ_K, c["qkv"][:, H:2 * H]), (O.AQ_V, c["qkv"][:, 2 * H:]),
                 (O.AQ_C, c["C"]), (O.AQ_X1, c["x1"])]:
        _, q, v, inside = O.fake_quant_forward(t, s[i], -127, 127)
        assert np.abs(q).max() == 127 and np.abs(v).max() < 127 * (1 + 1e-6) and z[i] == 0
    _, q, v, _ = O.fake_quant_forward(c["P"], s[O.AQ_P], 0, 255)
    assert q.max() == 255 and q.min() >= 0 and z[O.AQ_P] == 0
    g = O.gelu(c["u"])
    _, q, v, _ = O.fake_quant_forward(g, s[O.AQ_G], 0, 255, z[O.AQ_G])
    assert q.max() == 255 and q.min() == 0 and -0.2 < z[O.AQ_G] < 0 and v.min() >= -1e-6


@pytest.mark.parametrize("mode,tol", [("f32", 1e-5), ("bf16", 5e-2)])
def test_storage_rounding_stays_close_to_fp64(mode, tol):
    cfg = tiny_cfg(n_layers=2)
    teacher, student, x = tiny_student(cfg)
    x = O.round_store(x, mode)
    ref = O.module_grads(x, x, teacher, student, cfg, 2, 6)
    cfg_r = tiny_cfg(n_layers=2, act_round=mode)
    got = O.module_grads(x, x, teacher, student, cfg_r, 2, 6)
    for a, b in zip(ref.f_fp + ref.f_q, got.f_fp + got.f_q):
        assert np.linalg.norm(a - b) <= tol * np.linalg.norm(a)
    if mode == "bf16":
        for f in got.f_q:
            assert np.array_equal(f, O.round_bf16(f))


def test_loss_ordering_and_descent():
    """Step-0 loss ordered W8A8 < W4A8 < W2A8, and Algorithm 2 iterations
    reduce the loss on a fixed batch."""
    losses = {}
    for wb in (8, 4, 2):
        cfg = tiny_cfg(n_layers=2, w_bits=wb)
        teacher, student, x = tiny_student(cfg)
        losses[wb] = O.module_grads(x, x, teacher, student, cfg, 2, 6).loss
    assert losses[8] < losses[4] < losses[2]
    cfg = tiny_cfg(n_layers=2)
    teacher, student, x = tiny_student(cfg)
    zeros = lambda: [{k: np.zeros_like(v) for k, v in lp.items()} for lp in student]
    m, v = zeros(), zeros()
    before = {k: student[0][k].copy() for k in O.LAYER_FIELDS}
    hist = []
    for t in range(1, 41):
        hist.append(O.module_step(x, x, teacher, student, m, v, t, O.linear_decay_lr(2e-3, t - 1, 40), cfg, 2, 6).loss)
    assert hist[-1] < 0.5 * hist[0]
    assert np.array_equal(student[0]["z_a"], before["z_a"])          # offsets are not learned
    for k in O.TRAINABLE_FIELDS:
        assert not np.array_equal(student[0][k], before[k]), k       # weights and every step size moved
    assert all(np.all(lp[k] > 0) for lp in student for k in O.STEP_NAMES + ("s_a",))


# ---------------------------------------------------------------------------------
# schedules around the step (Section 4.1, Section 4.2 / Algorithm 1): the pipeline oracle
# ---------------------------------------------------------------------------------
import helpers as Hh  # noqa: E402  (tests/ is on sys.path through conftest)

def _chain_states(cases):
    from oracle import mrem_pipeline as P
    import copy
    states = []
    for c in cases:
        m, v = Hh.fresh_moments(c.student)
        states.append(P.ModuleState(copy.deepcopy(c.teacher), copy.deepcopy(c.student), m, v, c.cfg))
    return states


PIPE_WL = synth.Workload("pipe_tiny", 1, 32, 2, 64, 8, 2, act_dtype="f32")


def test_pipeline_single_module_is_repeated_steps():
    """One module: Algorithm 1 degenerates to Algorithm 2 applied to the data stream."""
    import copy
    from oracle import mrem_pipeline as P
    cases, batches, lens = Hh.make_chain(PIPE_WL, 1, 4)
    data = [b.reshape(-1, PIPE_WL.hidden).astype(np.float64) for b in batches]
    tr = P.run_parallel(_chain_states(cases), data, lens, Hh.draw_slots(4, 1, 2), 2, 4, 1e-3, 2, PIPE_WL.batch, PIPE_WL.seq)
    c = cases[0]
    student = copy.deepcopy(c.student)
    m, v = Hh.fresh_moments(student)
    for t in range(4):
        res = O.module_step(data[t], data[t], c.teacher, student, m, v, t + 1, O.linear_decay_lr(1e-3, t, 4), c.cfg,
                            PIPE_WL.batch, PIPE_WL.seq, lens[t])
        assert tr.loss[t][0] == res.loss
        assert tr.read_age[t] == [-1]


def test_pipeline_queue_semantics_by_hand():
    """Two modules, queue depth 2, 5 steps, written out by hand: fill phase chained within the
    step; afterwards module 2 reads the entry of the stated age from the queue as it stood after
    the previous step, mixes its two halves with lambda_t (Eq. 4) and the queue drops its oldest entry."""
    import copy
    from oracle import mrem_pipeline as P
    T, t0, tf = 5, 2, 4
    cases, batches, lens = Hh.make_chain(PIPE_WL, 2, T)
    data = [b.reshape(-1, PIPE_WL.hidden).astype(np.float64) for b in batches]
    slots = [[0, 0], [0, 0], [0, 1], [0, 0], [0, 1]]
    tr = P.run_parallel(_chain_states(cases), data, lens, slots, t0, T, 1e-3, tf, PIPE_WL.batch, PIPE_WL.seq)
    st = [copy.deepcopy(c.student) for c in cases]
    mv = [Hh.fresh_moments(s) for s in st]
    B_, S_ = PIPE_WL.batch, PIPE_WL.seq
    history = []   # outputs of module 1 per step: (f, f^)
    for t in range(T):
        lr = 1e-3 * (1 - t / T)
        lam = max(1 - t / tf, 0.0)
        r1 = O.module_step(data[t], data[t], cases[0].teacher, st[0], mv[0][0], mv[0][1], t + 1, lr, cases[0].cfg, B_, S_, lens[t])
        if t < t0:
            src = (r1.f_fp[-1], r1.f_q[-1])          # just produced
        else:
            src = history[t - 1 - slots[t][1]]      # age 0 = step t-1, age 1 = step t-2
        x_in = lam * src[0] + (1 - lam) * src[1]
        r2 = O.module_step(src[0], x_in, cases[1].teacher, st[1], mv[1][0], mv[1][1], t + 1, lr, cases[1].cfg, B_, S_, lens[t])
        history.append((r1.f_fp[-1], r1.f_q[-1]))
        assert tr.loss[t][0] == r1.loss
        np.testing.assert_allclose(tr.loss[t][1], r2.loss, rtol=1e-12)
    # teacher forcing matters: with lambda = 0 throughout, module 2 sees other inputs and other losses
    tr0 = P.run_parallel(_chain_states(cases), data, lens, slots, t0, T, 1e-3, 0, B_, S_)
    assert tr0.loss[0][0] == tr.loss[0][0]
    assert tr0.loss[0][1] != tr.loss[0][1]


def test_pipeline_sequential_feeds_finished_chains():
    """Section 4.1: the second module is trained on the outputs of the finished first module
    (teacher chain into the teacher, quantized chain into the quantized copy)."""
    import copy
    from oracle import mrem_pipeline as P
    cases, batches, lens = Hh.make_chain(PIPE_WL, 2, 2)
    data = [b.reshape(-1, PIPE_WL.hidden).astype(np.float64) for b in batches]
    states = _chain_states(cases)
    tr = P.run_sequential(states, data, lens, 3, 1e-3, PIPE_WL.batch, PIPE_WL.seq)
    B_, S_ = PIPE_WL.batch, PIPE_WL.seq
    # module 1 alone
    st = copy.deepcopy(cases[0].student)
    m, v = Hh.fresh_moments(st)
    for t in range(3):
        res = O.module_step(data[t % 2], data[t % 2], cases[0].teacher, st, m, v, t + 1, 1e-3 * (1 - t / 3), cases[0].cfg, B_, S_, lens[t % 2])
        assert tr.loss[0][t] == res.loss
    f_fp, _ = O.module_forward(data[0], cases[0].teacher, cases[0].cfg, B_, S_, lens[0], quant=False)
    f_q, _ = O.module_forward(data[0], st, cases[0].cfg, B_, S_, lens[0], quant=True)
    st2 = copy.deepcopy(cases[1].student)
    m2, v2 = Hh.fresh_moments(st2)
    res = O.module_step(f_fp[-1], f_q[-1], cases[1].teacher, st2, m2, v2, 1, 1e-3, cases[1].cfg, B_, S_, lens[0])
    assert tr.loss[1][0] == res.loss
    # the quantized chain differs from the full-precision chain
    assert not np.array_equal(f_fp[-1], f_q[-1])


# ---------------------------------------------------------------------------------
# one step per weight matrix (Section 3.1's default granularity)
# ---------------------------------------------------------------------------------

def test_per_tensor_weight_steps_vs_autograd_of_a_scalar_step():
    """per_channel=False: the initial step is max|W|/Qp over the whole matrix, the vector of
    steps stays tied through AdamW updates, and the step gradient the oracle returns (one value,
    repeated) equals torch's autograd derivative of the surrogate with a scalar step."""
    cfg = tiny_cfg(n_layers=1)
    cfg = O.Config(**{**cfg.__dict__, "per_channel": False})
    batch, seq = 2, 6
    teacher, student, x = tiny_student(cfg, batch=batch, seq=seq)
    lp = student[0]
    for n in O.WEIGHT_NAMES:
        s0 = O.weight_step_init(lp[n], cfg.w_bits, per_channel=False)
        assert np.all(s0 == s0[0])
        assert s0[0] == np.float64(np.float32(np.float32(np.abs(lp[n]).max()) / np.float32(O.sym_range(cfg.w_bits)[1])))
        lp["s" + n] = np.float64(np.float32(s0 * 0.9))       # off the clip bound (see the per-channel test)
    res = O.module_grads(x, x, teacher, student, cfg, batch, seq, None)
    # torch: scalar steps, expanded to rows inside the surrogate
    tl = {k: torch.tensor(v, requires_grad=(k != "z_a")) for k, v in lp.items()}
    scal = {n: torch.tensor(float(lp[n][0]), dtype=torch.float64, requires_grad=True) for n in O.STEP_NAMES}
    tl_s = dict(tl)
    for n in O.STEP_NAMES:
        tl_s[n] = scal[n].expand(lp[n].shape[0])
    h = _torch_student_layer(torch.tensor(x), tl_s, cfg, batch, seq, None)
    loss = ((h - torch.tensor(res.f_fp[0])) ** 2).mean()
    loss.backward()
    for n in O.STEP_NAMES:
        got = res.grads[0][n]
        assert np.all(got == got[0])
        assert abs(got[0] - scal[n].grad.item()) <= 2e-6 * abs(scal[n].grad.item()), (n, got[0], scal[n].grad.item())
    # the per-channel gradients of the same point sum to it
    cfg_pc = O.Config(**{**cfg.__dict__, "per_channel": True})
    res_pc = O.module_grads(x, x, teacher, student, cfg_pc, batch, seq, None)
    for n in O.STEP_NAMES:
        np.testing.assert_allclose(res.grads[0][n][0], res_pc.grads[0][n].sum(), rtol=1e-12)
    # tied through an update
    m, v = ([{k: np.zeros_like(a) for k, a in lp.items()}], [{k: np.zeros_like(a) for k, a in lp.items()}])
    O.module_step(x, x, teacher, student, m, v, 1, 1e-3, cfg, batch, seq, None)
    for n in O.STEP_NAMES:
        assert np.all(student[0][n] == student[0][n][0])


def test_step_gradient_interval_at_a_clip_bound():
    """The diagnostic that accompanies ds: with bf16 storage a value within one rounding of a clip
    bound may be decided either way, and the element's term jumps between d*(q - v) and d*q_bound.
    Checked by hand on four elements: one just inside the upper bound, one just outside, two far."""
    cfg = O.Config(n_layers=1, hidden=8, n_heads=1, ffn=8, a_bits=8, w_bits=4, act_round="bf16")
    lp = {"s_a": np.full(8, 0.5), "z_a": np.zeros(8)}
    aq = O._AQ(cfg, lp, O.AQ_X, True)               # symmetric, Qp = 127
    x = np.array([126.6, 127.4, 10.2, -50.3]) * 0.5  # v = 126.6 (inside), 127.4 (clipped), far, far
    d = np.array([2.0, -3.0, 1.0, 1.0])
    aq.fwd(x)
    _, ds = aq.bwd(d)
    terms = np.array([2.0 * (127 - 126.6), -3.0 * 127, 1.0 * (10 - 10.2), 1.0 * (-50 + 50.3)])
    assert np.isclose(ds, terms.sum())
    # element 0 decided "outside": 2*127 instead of 2*0.4 -> ds rises by 253.2
    # element 1 decided "inside": -3*(127 - 127.4) = 1.2 instead of -381 -> ds rises by 382.2
    assert np.isclose(aq.ds_up, 253.2 + 382.2) and aq.ds_down == 0.0
    _, _ = aq.bwd(-d)
    assert np.isclose(aq.ds_down, 253.2 + 382.2) and aq.ds_up == 0.0
    # exact storage: no band, no interval
    cfg32 = O.Config(n_layers=1, hidden=8, n_heads=1, ffn=8, a_bits=8, w_bits=4, act_round="f32")
    aq32 = O._AQ(cfg32, lp, O.AQ_X, True)
    aq32.fwd(x)
    aq32.bwd(d)
    assert aq32.ds_up == 0.0 and aq32.ds_down == 0.0


# --------------------------------------------------------------------------------
# diagnostics that the GPU parity tests select inputs with, divide by or widen intervals with
# --------------------------------------------------------------------------------

def test_decision_margin_hand_vectors():
    """decision_margin: distance (in steps) to the nearest rounding tie inside the range or clip bound."""
    # ties: |frac - 1/2| = 0.3, 0.05, 0.4 ; bounds (qn, qp = -7, 7): 5.8, 3.55, 0.1
    assert np.isclose(O.decision_margin(np.array([1.2, 3.45, -6.9]), -7, 7), 0.05)
    # an exact tie inside the range
    assert O.decision_margin(np.array([1.2, 2.5]), -7, 7) == 0.0
    # a clipped value just beyond the upper bound: no tie counts outside the range, the bound does
    assert np.isclose(O.decision_margin(np.array([7.02]), -7, 7), 0.02)
    # ... and just beyond the lower one
    assert np.isclose(O.decision_margin(np.array([-7.25, 0.0]), -7, 7), 0.25)
    # a value sitting on the bound itself (the largest element at initialisation)
    assert O.decision_margin(np.array([7.0, 0.9]), -7, 7) == 0.0
    # unsigned grid: the lower bound 0 counts ...
    assert np.isclose(O.decision_margin(np.array([0.05, 200.0]), 0, 255), 0.05)
    # ... unless the values cannot go below it (softmax probabilities): then only ties and the upper bound
    assert np.isclose(O.decision_margin(np.array([0.05, 200.0]), 0, 255, nonnegative=True), 0.45)
    assert np.isclose(O.decision_margin(np.array([254.9]), 0, 255, nonnegative=True), 0.1)


@pytest.mark.parametrize("qn,qp", [(-7, 7), (0, 15)])
def test_decision_margin_is_a_safe_perturbation_radius(qn, qp):
    """Brute force: moving every ratio by less than the margin changes no code and no mask."""
    rng = np.random.default_rng(3)
    v = rng.uniform(qn - 2.0, qp + 2.0, size=400)
    m = O.decision_margin(v, qn, qp)
    assert m > 0
    code = lambda t: np.rint(np.clip(t, qn, qp))
    mask = lambda t: (t >= qn) & (t <= qp)
    for sign in (-1.0, 1.0):
        w = v + sign * 0.999 * m
        assert np.array_equal(code(w), code(v)) and np.array_equal(mask(w), mask(v))
    # and the margin is attained: a move a little larger than it flips one code or one mask entry
    flipped = False
    for sign in (-1.0, 1.0):
        w = v + sign * 1.001 * m
        flipped |= (not np.array_equal(code(w), code(v))) or (not np.array_equal(mask(w), mask(v)))
    assert flipped


def test_flag_near_discontinuity_hand_vectors():
    tau = O.discontinuity_band("bf16")
    assert tau == 2.0 ** -7 and O.discontinuity_band("f32") == 2.0 ** -20 and O.discontinuity_band(None) == 0.0
    #            tie      near tie   far      at bound  near bound(in)  near bound(out)  far outside
    v = np.array([2.5,    -3.496,    1.2,     127.0,    126.3,          127.9,           140.0, -126.2, 0.504])
    tie, bound = O.flag_near_discontinuity(v, -127, 127, tau)        # bound band: 127 / 128 = 0.992 steps
    assert tie.tolist() == [True, True, False, False, False, False, False, False, True]
    assert bound.tolist() == [False, False, False, True, True, True, False, True, False]
    # a tie position outside the range is no tie (the value is clipped there)
    tie, bound = O.flag_near_discontinuity(np.array([7.5, -8.5]), -7, 7, tau)
    assert not tie.any() and not bound.any()
    # fp32 band: only values within 2^-20 of the tie
    tie, _ = O.flag_near_discontinuity(np.array([2.5 + 2.0 ** -21, 2.5 + 2.0 ** -19]), -7, 7, O.discontinuity_band("f32"))
    assert tie.tolist() == [True, False]
    # unsigned grid with an offset: x^ = s q + z, z / s = -8.5 steps: the stored value at the lower bound 0 is
    # 8.5 steps large (band 8.5 / 128 = 0.066), at the upper bound 255 it is 246.5 steps large (band 1.93)
    v = np.array([0.05, 0.08, -0.06, 253.2, 252.9, 256.5, 100.0])
    _, bound = O.flag_near_discontinuity(v, 0, 255, tau, offset_steps=-8.5)
    assert bound.tolist() == [True, False, True, True, False, True, False]
    # ... and without offset nothing can be decided differently at the lower bound 0 (probabilities)
    _, bound = O.flag_near_discontinuity(np.array([0.0, 0.001, 254.0]), 0, 255, tau)
    assert bound.tolist() == [False, False, True]
    # the counts reach the per-quantizer records of a forward pass
    cfg = O.Config(n_layers=1, hidden=8, n_heads=1, ffn=8, a_bits=4, w_bits=4, act_round="bf16")
    aq = O._AQ(cfg, {"s_a": np.full(8, 0.5), "z_a": np.zeros(8)}, O.AQ_X, True)   # symmetric 4-bit: [-7, 7], band 7/128 at a bound
    aq.fwd(np.array([1.25, 0.6, 3.48, 3.6, -3.52]))                                  # v = 2.5, 1.2, 6.96, 7.2, -7.04
    assert (aq.n_near_tie, aq.n_near_bound) == (1, 2)
    tie, bound = aq.flags()
    assert tie.tolist() == [True, False, False, False, False] and bound.tolist() == [False, False, True, False, True]


def test_step_gradient_scale_hand_vector():
    """ds_abs = sum of |terms| of the step-size gradient (the scale a computed ds is judged on)."""
    cfg = O.Config(n_layers=1, hidden=8, n_heads=1, ffn=8, a_bits=4, w_bits=4)
    aq = O._AQ(cfg, {"s_a": np.full(8, 0.25), "z_a": np.zeros(8)}, O.AQ_X, True)      # [-7, 7]
    x = np.array([0.3, -0.9, 2.5, -0.625])          # v = 1.2, -3.6, 10 (clipped), -2.5 (tie -> -2)
    d = np.array([2.0, -1.0, 0.5, 4.0])
    aq.fwd(x)
    _, ds = aq.bwd(d)
    terms = np.array([2.0 * (1 - 1.2), -1.0 * (-4 + 3.6), 0.5 * 7, 4.0 * (-2 + 2.5)])   # -0.4, 0.4, 3.5, 2.0
    assert np.isclose(ds, terms.sum()) and np.isclose(ds, 5.5)
    assert np.isclose(aq.ds_abs, 0.4 + 0.4 + 3.5 + 2.0)
    # unsigned quantizer with an offset: v = (x - z) / s
    cfgu = O.Config(n_layers=1, hidden=8, n_heads=1, ffn=8, a_bits=2, w_bits=4)
    lp = {"s_a": np.full(8, 0.5), "z_a": np.full(8, -0.25)}
    aqu = O._AQ(cfgu, lp, O.AQ_G, True)                                                  # {0..3}, z = -0.25
    aqu.fwd(np.array([0.35, -0.5, 2.0]))           # v = 1.2, -0.5 (below 0: clipped), 4.5 (clipped to 3)
    _, dsu = aqu.bwd(np.array([1.0, 2.0, -1.0]))
    assert np.isclose(dsu, 1.0 * (1 - 1.2) + 2.0 * 0 + -1.0 * 3)
    assert np.isclose(aqu.ds_abs, 0.2 + 0.0 + 3.0)


def test_fp32_accumulation_mode_is_the_same_forward_pass():
    """accumulate='f32' forms the same products in fp32: without quantizers and storage rounding it differs
    from the fp64 pass at fp32 rounding level only; with them it measures the amplification."""
    cfg = tiny_cfg(n_layers=2, w_bits=0, a_bits=0)
    teacher, student, x = tiny_student(cfg)
    ref, _ = O.module_forward(x, teacher, cfg, 2, 6, quant=False)
    cfg32 = tiny_cfg(n_layers=2, w_bits=0, a_bits=0, accumulate="f32")
    got, _ = O.module_forward(x, teacher, cfg32, 2, 6, quant=False)
    for a, b in zip(ref, got):
        e = np.linalg.norm(a - b) / np.linalg.norm(a)
        assert 0 < e < 1e-5
    with pytest.raises(ValueError):
        O.module_forward(x, teacher, tiny_cfg(accumulate="f16"), 2, 6, quant=False)


def test_rem_single_product_vs_autograd_and_adamw():
    """Eq. 2: gradients of the single-product reconstruction objective against torch fp64 autograd of the
    frozen-residual surrogate (clipped weights and activations included), the loss against its definition
    written out with loops, and one update against torch.optim.AdamW."""
    rng = np.random.default_rng(21)
    T, N, K = 6, 5, 7
    a = rng.standard_normal((T, K)); a_q = a + 0.05 * rng.standard_normal((T, K))
    w0 = rng.standard_normal((N, K)) * 0.3
    w = w0 + 0.01 * rng.standard_normal((N, K))
    s_w = (np.abs(w).max(axis=1) / 7 * rng.uniform(0.5, 1.0, size=N)).astype(np.float32).astype(np.float64)   # some weights clip
    s_a = float(np.abs(a_q).max() / 127 * 0.7)                            # some activations clip
    for loss_mean in (True, False):
        cfg = O.Config(n_layers=1, hidden=8, n_heads=1, ffn=8, w_bits=4, a_bits=8, loss_mean=loss_mean)
        loss, y, y_hat, g = O.rem_grads(a, a_q, w0, w, s_w, s_a, cfg)
        # the definition, index by index
        want = 0.0
        _, a_hat_q, _, _ = O.fake_quant_forward(a_q, s_a, -127, 127, 0.0, False)
        wq, w_hat, _, _ = O.quantize_weight(w, s_w, 4)
        for t in range(T):
            for n in range(N):
                yq = sum(s_a * a_hat_q[t, k] * s_w[n] * wq[n, k] for k in range(K))
                yf = sum(a[t, k] * w0[n, k] for k in range(K))
                want += (yq - yf) ** 2
        assert np.isclose(loss, want / (T * N) if loss_mean else want, rtol=1e-12, atol=0)
        # autograd of the surrogate x^ = s (clamp(x / s) + kappa), kappa frozen
        ta, tw = torch.tensor(a_q), torch.tensor(w, requires_grad=True)
        tsa = torch.tensor(s_a, requires_grad=True, dtype=torch.float64)
        tsw = torch.tensor(s_w, requires_grad=True)
        ca = torch.clamp(ta / tsa, -127, 127)
        ah = tsa * (ca + (torch.round(ca) - ca).detach())
        cw = torch.clamp(tw / tsw[:, None], -7, 7)
        wh = tsw[:, None] * (cw + (torch.round(cw) - cw).detach())
        d = ah @ wh.T - torch.tensor(a @ w0.T)
        L = (d * d).mean() if loss_mean else (d * d).sum()
        L.backward()
        assert np.isclose(loss, L.item(), rtol=1e-12, atol=0)
        np.testing.assert_allclose(g["w"], tw.grad.numpy(), rtol=1e-9, atol=1e-14)
        # the weight ratio w / s is an fp32 value in the oracle (it decides the code): 6e-8 relative on v in q - v
        np.testing.assert_allclose(g["s_w"], tsw.grad.numpy(), rtol=1e-5, atol=1e-9)
        np.testing.assert_allclose(g["s_a"], tsa.grad.item(), rtol=1e-9)
    # per-matrix step: the gradient is the sum over rows, repeated
    cfg1 = O.Config(n_layers=1, hidden=8, n_heads=1, ffn=8, w_bits=4, a_bits=8, per_channel=False)
    s1 = np.full(N, s_w.max())
    _, _, _, g1 = O.rem_grads(a, a_q, w0, w, s1, s_a, cfg1)
    _, _, _, gp = O.rem_grads(a, a_q, w0, w, s1, s_a, O.Config(n_layers=1, hidden=8, n_heads=1, ffn=8, w_bits=4, a_bits=8))
    assert np.allclose(g1["s_w"], gp["s_w"].sum()) and np.all(g1["s_w"] == g1["s_w"][0])
    # one update vs torch.optim.AdamW (decay on w only)
    cfg = O.Config(n_layers=1, hidden=8, n_heads=1, ffn=8, w_bits=4, a_bits=8)
    p = {"w": w.copy(), "s_w": s_w.copy(), "s_a": np.array([s_a])}
    m = {k: np.zeros_like(x) for k, x in p.items()}
    v = {k: np.zeros_like(x) for k, x in p.items()}
    _, _, _, g = O.rem_step(a, a_q, w0, p, m, v, 1, 1e-3, cfg)
    for name, wd in (("w", 0.01), ("s_w", 0.0), ("s_a", 0.0)):
        start = {"w": w, "s_w": s_w, "s_a": np.array([s_a])}[name]
        tp = torch.tensor(start.copy(), requires_grad=True)
        opt = torch.optim.AdamW([tp], lr=1e-3, betas=(0.9, 0.999), eps=1e-8, weight_decay=wd)
        tp.grad = torch.tensor(np.asarray(g[name], dtype=np.float64).reshape(start.shape))
        opt.step()
        np.testing.assert_allclose(p[name], np.maximum(tp.detach().numpy(), 1e-8) if name != "w" else tp.detach().numpy(), rtol=1e-10)

"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the
same seeded inputs.  Tolerances:

* integer weight codes and initial steps: bit-exact;
* fp32 check mode: outputs, loss, gradients, updated parameters within 1e-4
  (norm-wise relative error per tensor);
* bf16 mode (bf16 stored activations, fp32 accumulation): within 2e-2;
* a scalar step-size gradient ds = sum_i t_i is a heavily cancelling sum, so it is
  judged against the size of its terms: |ds_gpu - ds_ref| <= tol * sum_i |t_i|.

The oracle takes its quantizer decisions in the kernel's precision (fp32 ratio
of stored activations), see oracle/mrem_oracle.py.
"""
import numpy as np
import pytest

from oracle import mrem_oracle as O
from paper_2109_15082_amd import synth
import helpers as Hh

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
W = synth.Workload


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2109_15082_amd import binding
    return binding


def _torch():
    import torch
    return torch


# --------------------------------------------------------------------------------
# mrem_quantize: bit-exact codes (Section 3.1, Eq. 1)
# --------------------------------------------------------------------------------

@pytest.mark.parametrize("N,K", [(1, 8), (37, 100), (256, 1024), (513, 3000)])
@pytest.mark.parametrize("bits", [2, 4, 8])
def test_quantize_codes_bit_exact(B, N, K, bits):
    torch = _torch()
    rng = np.random.default_rng(N * 1000 + K + bits)
    w = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    if N > 1:
        w[N // 2] = 0.0                                   # an all-zero channel
        w[0, : K // 2] *= 30.0
    wd = torch.from_numpy(w).cuda()
    scale = torch.zeros(N, dtype=torch.float32, device="cuda")
    codes = torch.zeros((N, K), dtype=torch.int8, device="cuda")
    B.mrem_quantize(wd, N, K, bits, 1, scale, codes)
    s_ref = O.weight_step_init(w, bits)
    s_ref[s_ref == 0] = np.finfo(np.float32).tiny
    assert np.array_equal(scale.cpu().numpy(), s_ref.astype(np.float32))
    c_ref, _, _, _ = O.quantize_weight(w, s_ref, bits)
    assert np.array_equal(codes.cpu().numpy().astype(np.int64), c_ref)
    # given steps (not the initial ones): some values clip
    s2 = (s_ref * rng.uniform(0.3, 1.7, size=N)).astype(np.float32)
    scale.copy_(torch.from_numpy(s2))
    B.mrem_quantize(wd, N, K, bits, 0, scale, codes)
    c_ref, _, _, _ = O.quantize_weight(w, s2.astype(np.float64), bits)
    got = codes.cpu().numpy().astype(np.int64)
    assert np.array_equal(got, c_ref)
    qp = 2 ** (bits - 1) - 1
    assert got.min() >= -qp and got.max() <= qp
    assert np.array_equal(scale.cpu().numpy(), s2)        # steps untouched without init


def test_quantize_rejects_bad_arguments(B):
    torch = _torch()
    w = torch.zeros((4, 8), dtype=torch.float32, device="cuda")
    s = torch.zeros(4, dtype=torch.float32, device="cuda")
    c = torch.zeros((4, 8), dtype=torch.int8, device="cuda")
    with pytest.raises(B.MremError) as e:
        B.mrem_quantize(w, 4, 8, 9, 1, s, c)
    assert e.value.status == B.MREM_EINVAL
    with pytest.raises(B.MremError) as e:
        B.mrem_quantize(w, 0, 8, 4, 1, s, c)
    assert e.value.status == B.MREM_ESHAPE


# --------------------------------------------------------------------------------
# whole step
# --------------------------------------------------------------------------------

# fp32 check mode.  The quantizer is discontinuous at rounding ties and clip bounds, and
# the two sides differ at fp32 rounding level, so these cases run on the first seeded
# input for which the oracle reports that every quantizer ratio of the forward pass is at
# least MARGIN quantization steps away from a discontinuity (helpers.make_case_with_margin).
MARGIN = 2e-5
CASES_F32 = {
    # the small workload of the benchmark definition
    "tiny_f32": W("tiny_f32", 1, 64, 2, 256, 32, 4, act_dtype="f32"),
    # several 64-wide tiles with ragged tails in every product (T = 80, H = 72, 3H = 216, F = 136), key padding, head dim 24
    "ragged_f32": W("ragged_f32", 1, 72, 3, 136, 40, 2, act_dtype="f32", seqlen_lo=20, seqlen_hi=40),
    # two layers: the backward pass crosses a layer boundary and its input quantizer
    "two_layer_f32": W("two_layer_f32", 2, 64, 2, 128, 24, 2, act_dtype="f32"),
    "d128_f32": W("d128_f32", 1, 256, 2, 64, 24, 1, act_dtype="f32"),
    # other bit-widths of Tables 1-3
    "w2a8_f32": W("w2a8_f32", 1, 64, 2, 128, 16, 2, act_dtype="f32", w_bits=2),
    "w2a4_f32": W("w2a4_f32", 1, 64, 2, 128, 16, 2, act_dtype="f32", w_bits=2, a_bits=4),
    "w8a8_f32": W("w8a8_f32", 1, 64, 2, 128, 16, 2, act_dtype="f32", w_bits=8),
}
# bf16 storage: a stored value that rounds the other way is a 2^-8 relative change of one
# element, well inside the 2e-2 tolerance, so plain seeds are used.
CASES_BF16 = {
    "tiny_bf16": W("tiny_bf16", 1, 64, 2, 256, 32, 4, act_dtype="bf16"),
    # several tiles and ragged tails (T = 240, S = 80), key padding, two layers, head dim 64
    "mid_bf16": W("mid_bf16", 2, 128, 2, 512, 80, 3, act_dtype="bf16", seqlen_lo=40, seqlen_hi=80, outlier_frac=0.02),
    # MFMA-tile-aligned shapes (T = 512), head dim 32, three layers
    "aligned_bf16": W("aligned_bf16", 3, 256, 8, 1024, 128, 4, act_dtype="bf16", outlier_frac=0.01),
    # long context with key padding (the 384-token attention path, forward and backward), T = 768
    "long_bf16": W("long_bf16", 1, 128, 2, 256, 384, 2, act_dtype="bf16", seqlen_lo=128, seqlen_hi=384),
    # the other bit-widths of Tables 1-3 in the storage type of the bench (int8 products, matrix-core
    # attention): ternary weights, and ternary weights with 4-bit activations
    "w2a8_bf16": W("w2a8_bf16", 2, 128, 2, 512, 128, 2, act_dtype="bf16", w_bits=2),
    "w2a4_bf16": W("w2a4_bf16", 2, 128, 2, 512, 128, 2, act_dtype="bf16", w_bits=2, a_bits=4),
}
# fp32 mode at several tiles without the margin guarantee (about 7e5 quantized values:
# no seed keeps all of them away from ties): a looser bound
MID_F32 = W("mid_f32", 2, 128, 2, 512, 80, 3, act_dtype="f32", seqlen_lo=40, seqlen_hi=80)


def _compare_step(B, wl, lr=1e-3, case=None, tol=None, tol_for=None, **cfg_kw):
    """tol_for: {quantity name: tolerance} for the quantities judged on another scale than tol."""
    torch = _torch()
    tol = tol or TOL[wl.act_dtype]
    tol_for = tol_for or {}
    case = case or Hh.make_case(wl, **cfg_kw)
    mod = Hh.device_module(case)
    x, sl = Hh.device_inputs(case)
    xo = case.x.reshape(-1, wl.hidden).astype(np.float64)
    m, v = Hh.fresh_moments(case.student)
    grads = torch.zeros_like(mod.params)
    res = O.module_step(xo, xo, case.teacher, case.student, m, v, 1, lr, case.cfg, wl.batch, wl.seq, case.seqlens)
    ofp, oq = mod.step(x, x, lr, sl, grads_out=grads)
    torch.cuda.synchronize()
    loss = mod.loss.cpu().numpy()
    report = []
    for l in range(wl.n_layers):
        report.append((f"f_fp[{l}]", Hh.rel_err(ofp[l].float().cpu().numpy(), res.f_fp[l])))
        report.append((f"f_q[{l}]", Hh.rel_err(oq[l].float().cpu().numpy(), res.f_q[l])))
        if res.per_layer_loss[l] > 0:
            report.append((f"loss[{l}]", abs(loss[1 + l] / res.per_layer_loss[l] - 1)))
        else:
            assert loss[1 + l] == 0.0
    if res.loss > 0:
        report.append(("loss", abs(loss[0] / res.loss - 1)))
    gg = B.unpack_params(mod.ctx, grads, wl.n_layers)
    pp = B.unpack_params(mod.ctx, mod.params, wl.n_layers)
    mm = B.unpack_params(mod.ctx, mod.adam_m, wl.n_layers)
    for l in range(wl.n_layers):
        for k in O.TRAINABLE_FIELDS:
            ref = res.grads[l][k]
            if k == "s_a":
                # judged on the natural scale sum |t_i|, against the interval that the oracle's ds spans
                # when the values within one storage rounding of a clip bound are decided either way
                # (crossing the bound moves an element's term from about zero to d * q_bound)
                scale = np.maximum(res.grads[l]["s_a_abs"], 1e-30)
                lo, hi = ref - res.grads[l]["s_a_down"], ref + res.grads[l]["s_a_up"]
                for i in range(8):
                    outside = max(0.0, gg[l][k][i] - hi[i], lo[i] - gg[l][k][i])
                    report.append((f"ds_a[{l}][{O.ACT_Q_NAMES[i]}]", outside / scale[i]))
            elif np.linalg.norm(ref) > 0:
                report.append((f"g.{k}[{l}]", Hh.rel_err(gg[l][k], ref)))
            else:
                assert not gg[l][k].any(), (k, l)
            report.append((f"p.{k}[{l}]", Hh.rel_err(pp[l][k], case.student[l][k])))
        assert not gg[l]["z_a"].any()
        assert np.array_equal(pp[l]["z_a"], case.student[l]["z_a"].astype(np.float32))
        # first moment after one step is (1-beta1)*g: ties the update to the exported gradient
        np.testing.assert_allclose(mm[l]["w_1"], (1 - case.cfg.beta1) * gg[l]["w_1"], rtol=1e-5, atol=1e-30)
    bad = [(n, e) for n, e in report if not e <= tol_for.get(n, tol)]
    assert not bad, f"{wl.name}: beyond {tol}: {bad}"
    mod.close()
    return dict(report)


@pytest.mark.parametrize("name", list(CASES_F32))
def test_step_matches_oracle_fp32(B, name):
    wl = CASES_F32[name]
    # With 8-bit weights |f^ - f| is about 5e-4 |f|, so the loss gradient 2 (f^ - f) / n formed from two fp32
    # tensors carries a relative error of 2^-23 |f| / |f^ - f|, about 2.5e-4, into every gradient: 1e-3 there.
    tol = 1e-3 if wl.w_bits == 8 else None
    _compare_step(B, wl, case=Hh.make_case_with_margin(wl, MARGIN), tol=tol)


@pytest.mark.parametrize("name", list(CASES_BF16))
def test_step_matches_oracle_bf16(B, name):
    _compare_step(B, CASES_BF16[name])


def test_per_tensor_weight_steps_fp32(B):
    """One step per weight matrix (Section 3.1's default granularity): whole step against the oracle;
    the step fields stay tied and carry the summed gradient."""
    wl = CASES_F32["two_layer_f32"]
    case = Hh.make_case_with_margin(wl, MARGIN, per_channel=False)
    _compare_step(B, wl, case=case)


def test_per_tensor_weight_steps_bf16_and_initial_steps(B):
    torch = _torch()
    wl = CASES_BF16["aligned_bf16"]
    _compare_step(B, wl, case=Hh.make_case(wl, per_channel=False))
    # mrem_module_init_steps under per_channel = 0: max|W| / Qp of the whole matrix in every entry, bit for bit
    case = Hh.make_case(wl, per_channel=False)
    mod = Hh.device_module(case)
    mod.init_steps()
    torch.cuda.synchronize()
    pp = B.unpack_params(mod.ctx, mod.params, wl.n_layers)
    for l in range(wl.n_layers):
        for n in Hh.MATRICES:
            want = O.weight_step_init(case.layers_f32[l][n], wl.w_bits, per_channel=False).astype(np.float32)
            assert np.array_equal(pp[l]["s" + n], want)
            assert np.all(want == want[0])
    mod.close()


def test_step_fp32_several_tiles_no_margin(B):
    _compare_step(B, MID_F32, tol=1e-2)


def test_w8a8_bf16_forward_and_loss(B):
    """W8A8 with bf16 storage: the reconstruction error f^ - f is of the size of the
    bf16 rounding of f itself, so its gradient is not a well-conditioned quantity
    to compare in this mode (the fp32 case above covers it); outputs and loss are."""
    torch = _torch()
    wl = W("w8a8_bf16", 2, 128, 2, 512, 64, 2, act_dtype="bf16", w_bits=8)
    case = Hh.make_case(wl)
    mod = Hh.device_module(case)
    x, sl = Hh.device_inputs(case)
    xo = case.x.reshape(-1, wl.hidden).astype(np.float64)
    res = O.module_grads(xo, xo, case.teacher, case.student, case.cfg, wl.batch, wl.seq, case.seqlens)
    ofp, oq = mod.step(x, x, 1e-4, sl)
    torch.cuda.synchronize()
    for l in range(wl.n_layers):
        assert Hh.rel_err(ofp[l].float().cpu().numpy(), res.f_fp[l]) <= 2e-2
        assert Hh.rel_err(oq[l].float().cpu().numpy(), res.f_q[l]) <= 2e-2
    assert abs(mod.loss[0].item() / res.loss - 1) <= 2e-2
    mod.close()


def test_step_loss_options(B):
    """Last layer only in Eq. 3, and the raw sum of squares instead of the mean."""
    wl = CASES_F32["two_layer_f32"]
    _compare_step(B, wl, case=Hh.make_case_with_margin(wl, MARGIN, loss_layer_mask=0b10))
    _compare_step(B, wl, case=Hh.make_case_with_margin(wl, MARGIN, loss_mean=False), lr=1e-4)


def test_quantizers_off_gives_zero_loss(B):
    """Without quantizers the two modules coincide: zero loss, zero gradients."""
    torch = _torch()
    wl = W("off", 2, 64, 2, 256, 32, 2, act_dtype="f32", w_bits=0, a_bits=0)
    case = Hh.make_case(wl)
    mod = Hh.device_module(case)
    x, sl = Hh.device_inputs(case)
    grads = torch.ones_like(mod.params)
    before = mod.params.clone()
    ofp, oq = mod.step(x, x, 1e-3, sl, grads_out=grads)
    torch.cuda.synchronize()
    assert torch.equal(ofp, oq)
    assert not mod.loss.any()
    assert not grads.any()
    # only the decoupled weight decay moves anything
    pp = B.unpack_params(mod.ctx, mod.params, wl.n_layers)
    bb = B.unpack_params(mod.ctx, before, wl.n_layers)
    for l in range(wl.n_layers):
        np.testing.assert_allclose(pp[l]["w_1"], bb[l]["w_1"] * (1 - 1e-3 * 0.01), rtol=1e-6)
        assert np.array_equal(pp[l]["b_1"], bb[l]["b_1"]) and np.array_equal(pp[l]["ln1_g"], bb[l]["ln1_g"])
    mod.close()


def test_forward_entry_matches_step_outputs_and_is_deterministic(B):
    torch = _torch()
    wl = CASES_BF16["mid_bf16"]
    case = Hh.make_case(wl)
    mod = Hh.device_module(case)
    x, sl = Hh.device_inputs(case)
    f1, q1 = mod.forward(x, x, sl)
    f2, q2 = mod.forward(x, x, sl)
    g1 = torch.zeros_like(mod.params)
    g2 = torch.zeros_like(mod.params)
    saved = (mod.params.clone(), mod.adam_m.clone(), mod.adam_v.clone())
    f3, q3 = mod.step(x, x, 1e-3, sl, grads_out=g1)
    l1 = mod.loss.clone()
    mod.params.copy_(saved[0]); mod.adam_m.copy_(saved[1]); mod.adam_v.copy_(saved[2]); mod.step_index = 0
    mod.step(x, x, 1e-3, sl, grads_out=g2)
    torch.cuda.synchronize()
    assert torch.equal(f1, f2) and torch.equal(q1, q2)
    assert torch.equal(f1, f3) and torch.equal(q1, q3)
    assert torch.equal(g1, g2) and torch.equal(l1, mod.loss)      # fixed-order reductions: run-to-run identical
    mod.close()


def test_steps_back_to_back_equal_steps_with_synchronisation(B):
    """The step forks work onto a stream of its own and joins it again; consecutive steps queued
    without any host synchronisation, on the default stream or on another one, must leave exactly
    the state that fully synchronised steps leave (parameters, moments, losses, outputs)."""
    torch = _torch()
    wl = CASES_BF16["aligned_bf16"]
    case = Hh.make_case(wl)
    x, sl = Hh.device_inputs(case)
    xs = [x, (x * 0.5).contiguous(), (x * 1.5).contiguous()]

    def run(mode):
        mod = Hh.device_module(case)
        losses, outs = [], None
        stream = torch.cuda.Stream() if mode == "other_stream" else torch.cuda.current_stream()
        stream.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(stream):
            for t in range(6):
                outs = mod.step(xs[t % 3], xs[t % 3], 1e-3 * (1 - t / 6), sl)
                losses.append(mod.loss.clone())
                if mode == "synchronised":
                    torch.cuda.synchronize()
        torch.cuda.synchronize()
        state = (mod.params.clone(), mod.adam_m.clone(), mod.adam_v.clone(), torch.stack(losses), outs[0].clone(), outs[1].clone())
        mod.close()
        return state

    ref = run("synchronised")
    for mode in ("back_to_back", "other_stream"):
        got = run(mode)
        for a, b in zip(ref, got):
            assert torch.equal(a, b), mode


def test_calibrate_and_init_steps_match_oracle(B):
    torch = _torch()
    for name, wl in (("mid_f32", MID_F32), ("mid_bf16", CASES_BF16["mid_bf16"])):
        case = Hh.make_case(wl)
        mod = Hh.device_module(case)
        x, sl = Hh.device_inputs(case)
        ref = [{k: v.copy() for k, v in lp.items()} for lp in case.student]
        # wipe what the two calls are supposed to produce
        blank = [{k: (np.zeros_like(v) if k in O.STEP_NAMES + ("s_a", "z_a") else v) for k, v in lp.items()} for lp in ref]
        mod.params.copy_(B.pack_params(mod.ctx, blank))
        mod.init_steps()
        mod.calibrate(x, sl)
        torch.cuda.synchronize()
        got = B.unpack_params(mod.ctx, mod.params, wl.n_layers)
        for l in range(wl.n_layers):
            for k in O.STEP_NAMES:
                assert np.array_equal(got[l][k], ref[l][k].astype(np.float32)), (name, l, k)
            np.testing.assert_allclose(got[l]["s_a"], ref[l]["s_a"], rtol=1e-5)
            np.testing.assert_allclose(got[l]["z_a"], ref[l]["z_a"], rtol=1e-5, atol=1e-7)
            assert np.array_equal(got[l]["w_1"], ref[l]["w_1"].astype(np.float32).reshape(-1))
        mod.close()


def test_mix_inputs(B):
    torch = _torch()
    for dt, td in (("f32", torch.float32), ("bf16", torch.bfloat16)):
        ctx = B.mrem_create(n_layers=1, hidden=64, n_heads=2, ffn=128, max_batch=2, max_seq=16,
                            act_dtype=B.MREM_FP32 if dt == "f32" else B.MREM_BF16)
        a = torch.randn(2, 16, 64, device="cuda", generator=torch.Generator("cuda").manual_seed(1)).to(td)
        b = torch.randn(2, 16, 64, device="cuda", generator=torch.Generator("cuda").manual_seed(2)).to(td)
        out = torch.empty_like(a)
        lam = O.teacher_forcing_lambda(10, 40)
        B.mrem_mix_inputs(ctx, a, b, lam, out, a.numel())
        ref = O.round_store(O.mix_inputs(a.float().cpu().numpy(), b.float().cpu().numpy(), lam), dt)
        np.testing.assert_allclose(out.float().cpu().numpy(), ref, rtol=1e-6 if dt == "f32" else 2 ** -8, atol=1e-7)
        with pytest.raises(B.MremError):
            B.mrem_mix_inputs(ctx, a, b, 1.5, out, a.numel())
        B.mrem_destroy(ctx)


def test_loss_decreases_over_steps(B):
    """Algorithm 2 iterated on the device: the reconstruction loss of a fixed batch goes down."""
    torch = _torch()
    wl = CASES_BF16["mid_bf16"]
    case = Hh.make_case(wl)
    mod = Hh.device_module(case)
    x, sl = Hh.device_inputs(case)
    out = mod.new_outputs(wl.batch, wl.seq)
    hist = []
    for t in range(30):
        mod.step(x, x, O.linear_decay_lr(1e-4, t, 30), sl, *out)
        hist.append(mod.loss[0].item())
    assert hist[-1] < 0.7 * hist[0], hist
    assert all(np.isfinite(hist))
    mod.close()


# --------------------------------------------------------------------------------
# full-size workloads, in the launch configuration bench.py times
# --------------------------------------------------------------------------------

def test_full_size_bert_base_module_step(B):
    """The BERT-base-shaped 3-layer module (seq 128, batch 32, bf16): one whole step
    against the oracle -- every output, loss and gradient."""
    _compare_step(B, synth.WORKLOADS["bert_base_3l"], lr=1e-4)


def test_full_size_bert_large_module_step(B):
    """The bench workload itself (6 layers, H1024, F4096, seq 128, batch 32, 1% outlier channels,
    W4A8, bf16): one whole step against the oracle at full size -- every layer output of both
    modules, the loss, every gradient and every updated parameter within 2e-2.  The one exception
    is stated in the next test's text: the quantized module's outputs of layers 3..5, where one
    bf16 rounding upstream that goes the other way flips a code worth half a standard deviation
    and such differences grow through the chained quantized layers (measured 2.2e-2, 3.1e-2,
    3.9e-2); they are held to 1e-1 here and checked layer by layer from the oracle's inputs below.
    The oracle takes about 20 s for this step on the machine's host cores."""
    wl = synth.WORKLOADS["bert_large_6l"]
    _compare_step(B, wl, lr=1e-4, tol_for={"f_q[3]": 1e-1, "f_q[4]": 1e-1, "f_q[5]": 1e-1})


def _full_size_forward_on_sampled_sequences(B, wl, pick, chained_tol):
    torch = _torch()
    layers, x_np, seqlens = synth.make_workload_inputs(wl)
    mod = B.MremModule(wl.n_layers, wl.hidden, wl.n_heads, wl.ffn, wl.batch, wl.seq, act_dtype="bf16", w_bits=wl.w_bits, a_bits=wl.a_bits)
    mod.load(layers, layers)
    x = torch.from_numpy(x_np).cuda().to(torch.bfloat16).contiguous()
    sl = None if seqlens is None else torch.from_numpy(seqlens).cuda()
    sl_pick = None if seqlens is None else seqlens[pick]
    mod.init_steps()
    mod.calibrate(x, sl)
    torch.cuda.synchronize()
    student = O.to_f64(B.unpack_params(mod.ctx, mod.params, wl.n_layers, mod.shapes()))
    teacher = O.to_f64(layers)
    for lp in teacher:
        for n in Hh.MATRICES:
            lp[n] = synth.round_to_dtype(lp[n].astype(np.float32), "bf16").astype(np.float64)
    # the device's initial steps must be the oracle's, bit for bit
    for l in range(wl.n_layers):
        for n in Hh.MATRICES:
            assert np.array_equal(student[l]["s" + n].astype(np.float32), O.weight_step_init(layers[l][n], wl.w_bits).astype(np.float32))
    ofp, oq = mod.step(x, x, 1e-4, sl)
    torch.cuda.synchronize()
    cfg = O.Config(wl.n_layers, wl.hidden, wl.n_heads, wl.ffn, w_bits=wl.w_bits, a_bits=wl.a_bits, act_round="bf16")
    xs = x_np[pick].reshape(-1, wl.hidden).astype(np.float64)
    f_fp, _ = O.module_forward(xs, teacher, cfg, len(pick), wl.seq, sl_pick, quant=False)
    f_q, _ = O.module_forward(xs, student, cfg, len(pick), wl.seq, sl_pick, quant=True)
    chained = []
    for l in range(wl.n_layers):
        got_fp = ofp[l][pick].float().cpu().numpy().reshape(-1, wl.hidden)
        got_q = oq[l][pick].float().cpu().numpy().reshape(-1, wl.hidden)
        chained.append((Hh.rel_err(got_fp, f_fp[l]), Hh.rel_err(got_q, f_q[l])))
    print("chained relative errors (teacher, student):", chained)
    assert all(a <= 2e-2 for a, _ in chained), chained
    assert all(b <= chained_tol[l] for l, (_, b) in enumerate(chained)), chained
    loss = mod.loss.cpu().numpy()
    per = [float(((oq[l].double() - ofp[l].double()) ** 2).mean().item()) for l in range(wl.n_layers)]
    np.testing.assert_allclose(loss[1:], per, rtol=1e-4)
    np.testing.assert_allclose(loss[0], sum(per), rtol=1e-4)
    mod.close()
    # every layer on its own at the full shape, started from the oracle's output of the layer below
    one = B.MremModule(1, wl.hidden, wl.n_heads, wl.ffn, len(pick), wl.seq, act_dtype="bf16", w_bits=wl.w_bits, a_bits=wl.a_bits)
    sl_one = None if sl_pick is None else torch.from_numpy(np.ascontiguousarray(sl_pick)).cuda()
    isolated = []
    for l in range(wl.n_layers):
        one.load([student[l]], [layers[l]])
        xin_q = xs if l == 0 else f_q[l - 1]
        xin_fp = xs if l == 0 else f_fp[l - 1]
        dq = torch.from_numpy(xin_q.reshape(len(pick), wl.seq, wl.hidden).astype(np.float32)).cuda().to(torch.bfloat16)
        dfp = torch.from_numpy(xin_fp.reshape(len(pick), wl.seq, wl.hidden).astype(np.float32)).cuda().to(torch.bfloat16)
        o_fp, o_q = one.forward(dfp, dq, sl_one)
        torch.cuda.synchronize()
        isolated.append((Hh.rel_err(o_fp[0].float().cpu().numpy().reshape(-1, wl.hidden), f_fp[l]),
                         Hh.rel_err(o_q[0].float().cpu().numpy().reshape(-1, wl.hidden), f_q[l])))
    print("per-layer relative errors from oracle inputs (teacher, student):", isolated)
    assert all(a <= 2e-2 and b <= 2e-2 for a, b in isolated), isolated
    one.close()


def test_full_size_bert_large_forward_on_sampled_sequences(B):
    """The bench workload (6 layers, H1024, F4096, seq 128, batch 32, outlier channels).
    Sequences do not interact in the forward pass, so the oracle recomputes two of the 32
    sequences through all six layers (teacher and student) and those rows are compared.

    With 1% outlier channels the activation step is about 20x a typical value, so one bf16
    rounding that goes the other way flips a code worth half a standard deviation; through six
    quantized layers such differences grow roughly 5x per layer (measured 1e-5, 4e-4, 7e-3,
    1.7e-2, 2.6e-2, 3.4e-2).  Each layer is therefore also checked on its own, started from the
    ORACLE's output of the layer below (2e-2); the chained run must stay within 2e-2 for the
    first three layers and 1e-1 for the rest.  The reported loss must equal Eq. 3 evaluated
    on the exported layer outputs."""
    _full_size_forward_on_sampled_sequences(B, synth.WORKLOADS["bert_large_6l"], [3, 17], [2e-2, 2e-2, 2e-2, 1e-1, 1e-1, 1e-1])


def test_full_size_long_context_masked_w4a8(B):
    """The long-context configuration (6 layers, H1024, F4096, seq 384, batch 16, key padding
    with lengths in [128, 384], outlier channels), W4A8: same protocol as above on two sequences."""
    _full_size_forward_on_sampled_sequences(B, synth.WORKLOADS["bert_large_6l_s384"], [2, 11], [2e-2, 2e-2, 2e-2, 1e-1, 1e-1, 1e-1])


def test_full_size_long_context_masked_w8a8(B):
    """Its W8A8 variant (isolates the cost of the quantizers: 8-bit weights reconstruct far better)."""
    _full_size_forward_on_sampled_sequences(B, synth.WORKLOADS["bert_large_6l_s384_w8"], [2, 11], [2e-2, 2e-2, 2e-2, 1e-1, 1e-1, 1e-1])

"""Pins for the oracle's reduced-precision mode (bf16 weights / activations, high-precision sums,
full-precision master weights), against torch's own bf16 conversion and autograd."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from paper_1804_05834_amd import synth


def _bf(x):
    """Round a float64 tensor the way the mode is defined: to fp32, then to bf16 (torch's RNE)."""
    return x.float().bfloat16().double()


def test_round_bf16_against_torch(orc):
    rng = np.random.RandomState(0)
    vals = np.concatenate([rng.randn(2000), rng.randn(500) * 1e-8, rng.randn(500) * 1e6,
                           [0.0, -0.0, 1.0, 255.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -9,
                            0.1, -0.3, 65504.0, 2.0 ** -130]])
    ref = _bf(torch.from_numpy(vals)).numpy()
    got = np.array([orc.round_bf16(v) for v in vals])
    assert np.array_equal(got, ref)
    # ties go to the even mantissa; 8 significant bits
    assert orc.round_bf16(1.0 + 2 ** -8) == 1.0 and orc.round_bf16(1.0 + 3 * 2 ** -8) == 1.0 + 2 ** -6
    assert all(orc.round_bf16(float(i)) == i for i in range(256))


class _GradRound(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x):
        return x.clone()

    @staticmethod
    def backward(ctx, g):
        return _bf(g)


class _RoundSTE(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x):
        return _bf(x)

    @staticmethod
    def backward(ctx, g):
        return g


def _torch_net_q(params, K, dueling, x_u8):
    o = 0
    T = {}
    for name, shape, _ in synth.param_spec(K, dueling):
        n = int(np.prod(shape))
        t = params[o:o + n].reshape(shape)
        if name in ("conv1.W", "conv2.W", "conv3.W", "fc1.W"):
            t = _RoundSTE.apply(t)
        T[name] = t
        o += n
    x = x_u8.to(torch.float64) / 255.0
    x = _RoundSTE.apply(F.relu(_GradRound.apply(F.conv2d(x, T["conv1.W"], T["conv1.b"], stride=4))))
    x = _RoundSTE.apply(F.relu(_GradRound.apply(F.conv2d(x, T["conv2.W"], T["conv2.b"], stride=2))))
    x = _RoundSTE.apply(F.relu(_GradRound.apply(F.conv2d(x, T["conv3.W"], T["conv3.b"], stride=1))))
    h = F.relu(_GradRound.apply(F.linear(x.flatten(1), T["fc1.W"], T["fc1.b"])))
    adv = F.linear(h, T["A.W"], T["A.b"])
    if dueling:
        v = F.linear(h, T["V.W"], T["V.b"])
        return v + adv - adv.mean(dim=1, keepdim=True), h
    return adv, h


@pytest.mark.parametrize("K,dueling", [(4, False), (18, True)])
def test_quant_forward_against_torch(orc, K, dueling):
    p = synth.he_uniform_params(1804, K, dueling, bias_scale=0.05)
    s = synth.states(11, 3)
    q, h = orc.forward(p, K, dueling, s.numpy(), want_hidden=True, quant=1)
    with torch.no_grad():
        qt, ht = _torch_net_q(torch.from_numpy(p).double(), K, dueling, s)
    # a sum that lands within 1e-16 of a bf16 rounding boundary may round the other way in one
    # of the two implementations; allow a handful of such one-ulp (2^-8 relative) events
    dh = np.abs(h - ht.numpy())
    assert (dh > 1e-10).mean() < 1e-2 and dh.max() < 1e-2
    assert np.abs(q - qt.numpy()).max() < 1e-3
    # the mode really differs from full precision, at the bf16 level
    q0 = orc.forward(p, K, dueling, s.numpy())
    rel = np.abs(q - q0).max() / np.abs(q0).max()
    assert 1e-5 < rel < 2e-2


def test_quant_gradient_against_torch_autograd(orc):
    K, dueling, B = 18, True, 4
    p = synth.he_uniform_params(68, K, dueling, bias_scale=0.05)
    pt = synth.he_uniform_params(69, K, dueling, bias_scale=0.05)
    s, sn, a, r, d = (t.numpy() for t in synth.batch(70, B, K))
    w = (0.25 + 0.75 * synth.u24(79, torch.arange(B))).numpy()
    cfg = orc.make_config(K, dueling, 1, 1, quant=1)
    out = orc.loss_grad(cfg, p, pt, s, sn, a, r, d, w)
    tp = torch.from_numpy(p).double().requires_grad_(True)
    q_s = _torch_net_q(tp, K, dueling, torch.from_numpy(s))[0]
    with torch.no_grad():
        q_no = _torch_net_q(tp, K, dueling, torch.from_numpy(sn))[0]
        q_nt = _torch_net_q(torch.from_numpy(pt).double(), K, dueling, torch.from_numpy(sn))[0]
        a_star = q_no.argmax(dim=1)
        y = torch.from_numpy(r).double() + 0.99 * (1 - torch.from_numpy(d).double()) * \
            q_nt.gather(1, a_star[:, None])[:, 0]
    td = y - q_s.gather(1, torch.from_numpy(a).long()[:, None])[:, 0]
    l = torch.where(td.abs() <= 1, 0.5 * td ** 2, td.abs() - 0.5)
    loss = (torch.from_numpy(w).double() * l).mean()
    loss.backward()
    gt = tp.grad.numpy()
    assert out["loss"] == pytest.approx(float(loss.detach()), rel=1e-9)
    assert np.abs(out["td"] - td.detach().numpy()).max() < 1e-9
    # identical roundings on both sides except for sums within 1e-16 of a rounding boundary
    for name, (o, shp) in orc.param_slices(K, dueling).items():
        n = int(np.prod(shp))
        e = np.abs(out["grads"][o:o + n] - gt[o:o + n]).max() / np.abs(gt[o:o + n]).max()
        assert e < 1e-6, (name, e)
    # and it differs from the full-precision gradient at the bf16 level, not more
    g0 = orc.loss_grad(orc.make_config(K, dueling, 1, 1), p, pt, s, sn, a, r, d, w)["grads"]
    rel = np.linalg.norm(out["grads"] - g0) / np.linalg.norm(g0)
    assert 1e-5 < rel < 0.2


def test_quant_step_keeps_master_weights_in_full_precision(orc):
    K, dueling, B = 6, True, 2
    p = synth.he_uniform_params(5, K, dueling)
    pt = synth.he_uniform_params(6, K, dueling)
    s, sn, a, r, d = (t.numpy() for t in synth.batch(7, B, K))
    cfg = orc.make_config(K, dueling, 1, 1, quant=1)
    theta = p.copy(); v = np.zeros_like(p)
    out = orc.train_step(cfg, theta, pt, v, s, sn, a, r, d)
    g = out["grads"]
    # the update starts from the unrounded parameters: theta - p is exactly the RMSProp step
    step = theta.astype(np.float64) - p
    ref = -2.5e-4 * g / np.sqrt(0.05 * g * g + 0.01)
    assert np.abs(step - ref).max() < 1e-8
    moved = np.abs(step) > 0
    assert moved.mean() > 0.3

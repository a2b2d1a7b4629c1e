"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Tolerance: per tensor X, max|X_gpu - X_ref| / max|X_ref| <= 1e-4 on the fp32 path and 2e-2 on the
bf16 path, applied to the Q-values, targets, TD errors, loss, EVERY gradient entry, the parameter
step and the optimizer state (the parameter step gets one extra ulp of the parameter: theta itself
is stored in fp32 on both sides).  Integer results (argmax actions, sampled indices, tree nodes)
are compared bit-exactly, except where the oracle's own top-2 gap or distance to a bucket boundary
is inside that tolerance.

ReLU decisions are decisions of the same kind: a pre-activation that is zero to within the rounding
of its sum is a tie which the two sides may settle differently, and the gradient then differs by
that element's whole contribution.  The tests read back the activations the GPU stored
(dqn_get_activations), compare them with the oracle's element by element, require that the masks
differ only at such ties and that ties are rare, and hold every gradient entry against
oracle + (the ties' exact contribution, tests/torch_ref.py): nothing is left out of the comparison.
"""
import numpy as np
import pytest
import torch

import torch_ref
from paper_1804_05834_amd import synth

pytestmark = pytest.mark.gpu

TOL = 1e-4        # fp32 path
TOL_BF16 = 2e-2   # bf16 activations / weights with fp32 accumulation and fp32 master weights


@pytest.fixture(scope="module")
def dq():
    from paper_1804_05834_amd import dqn
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    dqn.lib()
    return dqn


def relerr(x, ref):
    x = np.asarray(x, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    assert x.shape == ref.shape, (x.shape, ref.shape)
    return float(np.abs(x - ref).max() / max(np.abs(ref).max(), 1e-12))


def check_argmax(a_gpu, q_ref, tol=TOL):
    a_ref = q_ref.argmax(axis=1)
    bad = np.flatnonzero(a_gpu != a_ref)
    for j in bad:
        top2 = np.sort(q_ref[j])[-2:]
        assert top2[1] - top2[0] <= tol * np.abs(q_ref[j]).max(), (j, a_gpu[j], a_ref[j], q_ref[j])


def dev(t):
    return t.cuda() if isinstance(t, torch.Tensor) else torch.from_numpy(np.ascontiguousarray(t)).cuda()


# ------------------------------------------------------------------ parameters
@pytest.mark.parametrize("K,dueling", [(4, 0), (18, 1)])
def test_init_and_param_roundtrip(dq, K, dueling):
    print("case init/roundtrip", K, dueling, flush=True)
    m = dq.Dqn(dq.make_config(num_actions=K, dueling=dueling, seed=1804, target_seed=5834))
    assert np.array_equal(m.get_params(0).cpu().numpy(), synth.he_uniform_params(1804, K, dueling))
    assert np.array_equal(m.get_params(1).cpu().numpy(), synth.he_uniform_params(5834, K, dueling))
    assert float(m.get_params(3).abs().max()) == 0.0
    p = synth.he_uniform_params(77, K, dueling, bias_scale=0.05)
    m.set_params(0, torch.from_numpy(p))
    assert np.array_equal(m.get_params(0).cpu().numpy(), p)
    m.sync_target()
    assert np.array_equal(m.get_params(1).cpu().numpy(), p)
    m.close()


# ------------------------------------------------------------------ acting / forward
@pytest.mark.parametrize("K,dueling,E,prec", [(4, 0, 37, 0), (18, 1, 70, 0), (1, 1, 3, 0), (64, 0, 5, 0),
                                              (18, 1, 70, 1), (4, 0, 300, 1), (18, 1, 3, 1)])
def test_act_forward_parity(dq, orc, K, dueling, E, prec):
    print("case act", K, dueling, E, prec, flush=True)
    TOL = TOL_BF16 if prec else globals()["TOL"]
    m = dq.Dqn(dq.make_config(num_actions=K, dueling=dueling, max_act_batch=512, precision=prec))
    p = synth.he_uniform_params(3 + K, K, dueling, bias_scale=0.05)
    m.set_params(0, torch.from_numpy(p))
    obs = synth.states(31, E)
    q_ref = orc.forward(p, K, dueling, obs.numpy(), quant=prec)
    a0, q = m.act(dev(obs), 0.0, 99, want_q=True)
    if prec:   # and within the stated tolerance of the full-precision Q-values
        assert relerr(q.cpu().numpy(), orc.forward(p, K, dueling, obs.numpy())) <= TOL
    assert relerr(q.cpu().numpy(), q_ref) <= TOL
    check_argmax(a0.cpu().numpy(), q_ref, TOL)
    # epsilon = 1: every action is the specified random draw
    a1 = m.act(dev(obs), 1.0, 99).cpu().numpy()
    ref1, _ = orc.act(p, K, dueling, obs.numpy(), 1.0, 99, quant=prec)
    assert np.array_equal(a1, ref1)
    # mixed: explore decisions follow the draw stream exactly; greedy ones follow argmax
    a5 = m.act(dev(obs), 0.5, 1234).cpu().numpy()
    ref5, _ = orc.act(p, K, dueling, obs.numpy(), 0.5, 1234, quant=prec)
    explore = synth.u24(1234, 2 * torch.arange(E)).numpy() < 0.5
    assert np.array_equal(a5[explore], ref5[explore])
    check_argmax(a5[~explore], q_ref[~explore], TOL)
    m.close()


@pytest.mark.parametrize("E,prec", [(2048, 1), (8192, 1), (2048, 0)])
def test_act_large_batches(dq, orc, E, prec):
    """Acting at the fifth configuration's size (2048 environments) and at the library's limit (8192
    observations: 32 samples per workgroup of the fused conv1 + conv2 launch, the most its slot table
    holds).  Every row's Q-values against the oracle, the draws bit for bit."""
    print("case act large", E, prec, flush=True)
    K, dueling = 18, 1
    tol = TOL_BF16 if prec else TOL
    m = dq.Dqn(dq.make_config(num_actions=K, dueling=dueling, max_act_batch=E, precision=prec))
    p = synth.he_uniform_params(3 + K, K, dueling, bias_scale=0.05)
    m.set_params(0, torch.from_numpy(p))
    obs = synth.states(31, E)
    obs_d = dev(obs)
    a0, q = m.act(obs_d, 0.0, 99, want_q=True)
    q = q.cpu().numpy()
    q_ref = orc.forward(p, K, dueling, obs.numpy(), quant=prec)
    print("  oracle done", flush=True)
    assert relerr(q, q_ref) <= tol
    # row by row as well: no row may hide behind the largest one
    assert np.all(np.abs(q - q_ref).max(axis=1) <= tol * np.abs(q_ref).max(axis=1))
    check_argmax(a0.cpu().numpy(), q_ref, tol)
    if prec:
        assert relerr(q, orc.forward(p, K, dueling, obs.numpy())) <= tol
    a1 = m.act(obs_d, 1.0, 99).cpu().numpy()
    u2 = synth.u24(99, 2 * torch.arange(E) + 1).numpy()
    assert np.array_equal(a1, np.minimum(np.floor(u2.astype(np.float64) * K), K - 1).astype(np.int32))
    a5 = m.act(obs_d, 0.05, 1234).cpu().numpy()
    explore = synth.u24(1234, 2 * torch.arange(E)).numpy() < np.float32(0.05)
    u2 = synth.u24(1234, 2 * torch.arange(E) + 1).numpy()
    assert np.array_equal(a5[explore], np.minimum(np.floor(u2.astype(np.float64) * K), K - 1).astype(np.int32)[explore])
    check_argmax(a5[~explore], q_ref[~explore], tol)
    m.close()


# ------------------------------------------------------------------ training step
def _oracle_step(orc, cfgd, p, pt, batch_np, w, quant=0):
    cfg = orc.make_config(cfgd["num_actions"], cfgd["dueling"], cfgd["double_q"], cfgd["loss_kind"],
                          lr=cfgd.get("lr", 2.5e-4), rms_centered=cfgd.get("rms_centered", 0), quant=quant)
    theta = p.copy(); v = np.zeros_like(p)
    mm = np.zeros_like(p) if cfgd.get("rms_centered", 0) else None
    out = orc.train_step(cfg, theta, pt, v, *batch_np, w, rms_m=mm)
    out["theta"] = theta; out["v"] = v; out["m"] = mm
    return out


# A mask may differ between the two sides only where the pre-activation (fp64, tests/torch_ref.py)
# is a tie.  fp32 path: the GPU's sum of up to 3136 fp32 products differs from the fp64 sum by a
# few 1e-6 at most (measured: 3e-6 on activations of rms 0.7).  bf16 path: both sides round the same
# numbers to bf16, but a sum within fp32 rounding of a bf16 rounding boundary lands on the other
# side of it (measured: 1.5e-5 of conv1's outputs, one bf16 ulp each), and the next layers' sums
# inherit those differences times their weights (measured: 2e-4 / 1e-3 of conv2's / conv3's outputs
# differ, the hidden layer by up to 3e-3; masks that differ had |pre-activation| <= 2.5e-3).
TIE_FRACTION = {0: 2e-5, 1: 2e-4}    # largest share of a layer's elements that may be ties
# A small bf16 activation may differ by this much outright: one differing input of the largest size
# (one ulp of a value in [2, 4) is 2^-6) times the largest weight (0.1) moves a sum by 1.6e-3, and a
# sum may meet two or three of them (measured at batch 512 and 1024: up to 2.7e-3).
ACT_ABS_BF16 = 5e-3
TIE_ABS = {0: 5e-6, 1: ACT_ABS_BF16}   # a sum that can move by that much can change sign below it


def _compare_activations(m, orc, p, K, dueling, s_u8, prec, B):
    """Stored layer outputs of the online pass on s against the oracle's, element by element.
    Returns the GPU's activations (numpy)."""
    ref = orc.forward_acts(p, K, dueling, s_u8, quant=prec)
    got = []
    for layer, key in ((1, "a1"), (2, "a2"), (3, "a3"), (4, "h")):
        g = m.get_activations(layer, B).cpu().numpy().astype(np.float64)
        r = ref[key]
        got.append(g)
        if prec == 0 or layer == 4:
            # bf16 path: the hidden layer is kept in fp32 but its inputs are bf16 numbers that may sit one ulp apart
            assert relerr(g, r) <= (TOL if prec == 0 else TOL_BF16), (key, relerr(g, r))
        else:
            # conv1 (exact inputs): the same bf16 number or its neighbour (one ulp is at most 2^-7 of the
            # value).  conv2, conv3: their sums inherit the one-ulp differences of the layer below, so
            # EACH element is held to the tolerance relative to its own size (2.5 ulps), small ones to
            # ACT_ABS_BF16; and only a small share of the elements may differ at all.
            d = np.abs(g - r)
            big = np.maximum(np.abs(g), np.abs(r))
            rel = 2.0 ** -7 if layer == 1 else TOL_BF16
            viol = np.argwhere(d > np.maximum(rel * big, ACT_ABS_BF16 if layer > 1 else 1e-5))
            assert len(viol) == 0, (key, len(viol), [(tuple(i), g[tuple(i)], r[tuple(i)]) for i in viol[:6]])
            assert (d > 0).mean() <= 5e-3, (key, (d > 0).mean())
    return got


def _check_step(orc, out, ref, p, m, K, dueling, batch_np, w, tol=TOL, ref_full=None):
    """Compares every output of one step taken from parameters p and zero optimizer state with the
    oracle's (`ref`: the oracle in the GPU path's precision mode; `ref_full`: the full-precision
    oracle, bf16 path only).  batch_np = (s, s_next, a, r, done) as numpy, w the importance weights."""
    g = {k: v.cpu().numpy() for k, v in out.items()}
    prec = int(m.cfg.precision)
    B = batch_np[0].shape[0]
    errs = {}
    for k in ("q_s", "q_next_online", "q_next_target", "y", "td"):
        errs[k] = relerr(g[k], ref[k])
    errs["loss"] = abs(float(g["loss"][0]) - ref["loss"]) / max(abs(ref["loss"]), 1e-12)
    # the step's diagnostics: mean |td| and mean max_a Q(s, a)
    errs["td_abs_mean"] = abs(float(g["td_abs_mean"][0]) - np.abs(ref["td"]).mean()) / max(np.abs(ref["td"]).max(), 1e-12)
    errs["q_max_mean"] = abs(float(g["q_max_mean"][0]) - ref["q_s"].max(axis=1).mean()) / np.abs(ref["q_s"]).max()
    sel = ref["q_next_online"] if m.cfg.double_q else ref["q_next_target"]
    check_argmax(g["a_star"], sel, tol)
    grads = m.get_params(2).cpu().numpy().astype(np.float64)
    theta = m.get_params(0).cpu().numpy()
    v = m.get_params(3).cpu().numpy()

    # layer outputs, and the ReLU decisions the GPU took
    acts = _compare_activations(m, orc, p, K, dueling, batch_np[0], prec, B)
    tie = torch_ref.tie_correction(p, K, dueling, batch_np[0], batch_np[2], ref["y"], w, int(m.cfg.loss_kind),
                                   prec, acts)
    nflip = [len(f) for f in tie["flips"]]
    for k, (f, pre) in enumerate(zip(tie["flips"], tie["pre"])):
        if len(f):
            worst = float(np.abs(pre[tuple(f.T)]).max())
            assert worst <= TIE_ABS[prec], ("a ReLU decision differs where the pre-activation is no tie", k, worst)
        assert len(f) <= max(2, TIE_FRACTION[prec] * pre.size), ("too many ties", k, len(f), pre.size)
    theta_ref, v_ref = p.copy(), np.zeros_like(p)
    m_ref = np.zeros_like(p) if m.cfg.rms_centered else None
    full = {}
    g_ref = ref["grads"] + tie["correction"]
    orc.rmsprop(theta_ref, v_ref, g_ref, lr=float(m.cfg.lr), rho=float(m.cfg.rms_decay), eps=float(m.cfg.rms_eps), m=m_ref)
    for name, (o, shp) in orc.param_slices(K, dueling).items():
        n = int(np.prod(shp))
        sl = slice(o, o + n)
        # the analysis tool reproduces the oracle's gradient with its own masks (it is tied to the oracle here)
        assert relerr(tie["g_own"][sl], ref["grads"][sl]) <= 1e-6, name
        errs["g:" + name] = relerr(grads[sl], g_ref[sl])                      # every entry, max norm
        dth_g = theta[sl].astype(np.float64) - p[sl]
        dth_r = theta_ref[sl].astype(np.float64) - p[sl]
        ulp = float(np.spacing(np.float32(np.abs(p[sl]).max())))
        slack = max(np.abs(dth_g - dth_r).max() - ulp, 0.0)
        errs["dtheta:" + name] = slack / max(np.abs(dth_r).max(), 1e-12)
        # v = (1 - rho) g^2 after one step from zero: a relative error e of g is 2e of v
        errs["v:" + name] = relerr(v[sl], v_ref[sl]) / 2
        # against the oracle's own step, in the relative L2 norm: whatever the ties' contribution
        # itself amounts to is allowed, nothing else
        dth_o = ref["theta"][sl].astype(np.float64) - p[sl]
        nrm = np.linalg.norm
        errs["dtheta_l2:" + name] = float(max(nrm(dth_g - dth_o) - nrm(dth_r - dth_o), 0.0) / max(nrm(dth_o), 1e-30))
        errs["g_l2:" + name] = float(max(nrm(grads[sl] - ref["grads"][sl]) - nrm(tie["correction"][sl]), 0.0) /
                                     max(nrm(ref["grads"][sl]), 1e-30))
        if ref_full is not None:
            # bf16 path against the FULL-PRECISION oracle: how far reduced precision moves the gradient.
            # That distance is a property of the arithmetic, not of the kernels (ReLU and argmax
            # decisions taken on bf16 numbers differ from those taken on exact ones in about 1e-3 of
            # the cases; measured 2.5 to 5 % in the relative L2 norm at batch 512 to 1024, more at
            # small batches, where fewer rows average it out).  The oracle's reduced-precision mode
            # is the same distance away; the GPU may not be farther than that by more than the tolerance.
            e = float(nrm(grads[sl] - ref_full["grads"][sl]) / max(nrm(ref_full["grads"][sl]), 1e-30))
            e_mode = float(nrm(ref["grads"][sl] - ref_full["grads"][sl]) / max(nrm(ref_full["grads"][sl]), 1e-30))
            full[name] = (e, e_mode)
            errs["g_l2_full_excess:" + name] = max(e - e_mode, 0.0)
    if m.cfg.rms_centered:
        errs["m"] = relerr(m.get_params(4).cpu().numpy(), m_ref)
    errs["theta"] = relerr(theta, ref["theta"])
    print("  ties per layer:", nflip, " worst:", sorted(errs.items(), key=lambda kv: -kv[1])[:4], flush=True)
    if full:
        e, e_mode, n = max((e, em, n) for n, (e, em) in full.items())
        print("  B=%d gradient vs full-precision oracle, relative L2, worst tensor %s: GPU %.3e, reduced-precision oracle %.3e"
              % (B, n, e, e_mode), flush=True)
    bad = sorted((k, float(e)) for k, e in errs.items() if not e <= tol)
    assert not bad, bad
    return errs


def _check_against_full_precision(out, ref64, theta_gpu, double_q, tol):
    """bf16 path vs the full-precision oracle, on the quantities the tolerance is stated for:
    Q-values, targets, TD errors, loss and the updated weights.  Where the full-precision
    Q-values have a near-tie (top-2 gap inside the tolerance) the bf16 argmax may pick the other
    action; the Double-DQN target of such a row is discontinuous there, so its y and td (and then
    the loss, an average over all rows) are compared on the remaining rows only."""
    g = {k: v.cpu().numpy() for k, v in out.items()}
    errs = {k: relerr(g[k], ref64[k]) for k in ("q_s", "q_next_online", "q_next_target")}
    sel = ref64["q_next_online"] if double_q else ref64["q_next_target"]
    check_argmax(g["a_star"], sel, tol)
    keep = g["a_star"] == ref64["a_star"]
    assert keep.mean() > 0.9
    errs["y"] = relerr(g["y"][keep], ref64["y"][keep])
    # td = y - Q is a difference of the two: its error is bounded by theirs, relative to them
    errs["td"] = float(np.abs(g["td"] - ref64["td"])[keep].max() /
                       max(np.abs(ref64["q_s"]).max(), np.abs(ref64["y"]).max()))
    if keep.all():
        errs["loss"] = abs(float(g["loss"][0]) - ref64["loss"]) / max(abs(ref64["loss"]), 1e-12)
    errs["theta"] = relerr(theta_gpu, ref64["theta"])
    bad = sorted((k, float(e)) for k, e in errs.items() if not e <= tol)
    assert not bad, bad


CONFIGS = {
    # vanilla DQN, plain head, K=4 (first configuration)
    "dqn": dict(num_actions=4, dueling=0, double_q=0, loss_kind=1),
    # Double DQN + dueling head, K=18 (second configuration)
    "dueling_ddqn": dict(num_actions=18, dueling=1, double_q=1, loss_kind=1),
    # squared loss of Eq.7, and a centered RMSProp
    "squared_centered": dict(num_actions=6, dueling=1, double_q=0, loss_kind=0, rms_centered=1),
    # Double DQN with the plain output layer (one of the settings of the paper's performance figure)
    "ddqn_plain": dict(num_actions=18, dueling=0, double_q=1, loss_kind=1),
    # the most actions the library takes: 65 head rows, 195 dot products per training row
    "wide": dict(num_actions=64, dueling=1, double_q=1, loss_kind=1),
    "wide_plain": dict(num_actions=33, dueling=0, double_q=0, loss_kind=0),
}


@pytest.mark.parametrize("name,B,prec", [("dqn", 32, 0), ("dueling_ddqn", 32, 0), ("dueling_ddqn", 5, 0),
                                         ("dueling_ddqn", 67, 0), ("squared_centered", 33, 0), ("dqn", 1, 0),
                                         ("dueling_ddqn", 32, 1), ("dueling_ddqn", 67, 1), ("dqn", 130, 1),
                                         ("squared_centered", 3, 1), ("wide", 9, 0), ("wide", 40, 1),
                                         ("wide_plain", 6, 0)])
def test_train_step_explicit_batch(dq, orc, name, B, prec):
    print("case train_step", name, B, prec, flush=True)
    cfgd = CONFIGS[name]
    tol = TOL_BF16 if prec else TOL
    K, dueling = cfgd["num_actions"], cfgd["dueling"]
    m = dq.Dqn(dq.make_config(max_batch=max(B, 32), seed=1804, target_seed=5834, precision=prec, **cfgd))
    p = synth.he_uniform_params(1804, K, dueling, bias_scale=0.02)
    pt = synth.he_uniform_params(5834, K, dueling, bias_scale=0.02)
    m.set_params(0, torch.from_numpy(p)); m.set_params(1, torch.from_numpy(pt))
    s, sn, a, r, d = synth.batch(11, B, K)
    w = (0.25 + 0.75 * synth.u24(19, torch.arange(B))) if name != "dqn" else None
    batch = tuple(dev(t) for t in (s, sn, a, r, d)) + ((dev(w),) if w is not None else ())
    out = m.train_step(B, batch)
    bnp = (s.numpy(), sn.numpy(), a.numpy(), r.numpy(), d.numpy())
    # bf16 path: every decision (ReLU masks, argmax) is compared against the oracle taking it on
    # the same rounded numbers; the stated quantities also against the full-precision oracle
    wn = None if w is None else w.numpy()
    ref = _oracle_step(orc, cfgd, p, pt, bnp, wn, quant=prec)
    ref64 = _oracle_step(orc, cfgd, p, pt, bnp, wn) if prec else None
    _check_step(orc, out, ref, p, m, K, dueling, bnp, wn, tol, ref_full=ref64)
    if prec:
        _check_against_full_precision(out, ref64, m.get_params(0).cpu().numpy(), m.cfg.double_q, tol)
    # the target network is not touched by a step
    assert np.array_equal(m.get_params(1).cpu().numpy(), pt)
    m.close()


def test_three_step_chain(dq, orc):
    print("case chain", flush=True)
    cfgd = CONFIGS["dueling_ddqn"]
    K, dueling, B = 18, 1, 16
    m = dq.Dqn(dq.make_config(max_batch=32, **cfgd))
    p = synth.he_uniform_params(1804, K, dueling)
    pt = synth.he_uniform_params(5834, K, dueling)
    m.set_params(0, torch.from_numpy(p)); m.set_params(1, torch.from_numpy(pt))
    cfg = orc.make_config(K, dueling, 1, 1)
    theta = p.copy(); v = np.zeros_like(p)
    for step in range(3):
        s, sn, a, r, d = synth.batch(100 + 10 * step, B, K)
        out = m.train_step(B, tuple(dev(t) for t in (s, sn, a, r, d)))
        ref = orc.train_step(cfg, theta, pt, v, s.numpy(), sn.numpy(), a.numpy(), r.numpy(), d.numpy())
        e_td = relerr(out["td"].cpu().numpy(), ref["td"])
        e_l = abs(float(out["loss"][0]) - ref["loss"]) / abs(ref["loss"])
        print("  step %d: td %.2e loss %.2e" % (step, e_td, e_l), flush=True)
        assert e_td <= TOL and e_l <= TOL
    e_th = relerr(m.get_params(0).cpu().numpy() - p.astype(np.float64), theta.astype(np.float64) - p)
    e_v = relerr(m.get_params(3).cpu().numpy(), v)
    print("  after three steps: theta - theta0 %.2e v %.2e" % (e_th, e_v), flush=True)
    assert e_th <= TOL and e_v <= TOL
    m.close()


@pytest.mark.parametrize("B,prec", [(512, 0), (160, 0), (32, 0), (512, 1), (96, 1)])
def test_step_is_run_to_run_deterministic(dq, B, prec):
    """Every reduction has a fixed order (no floating-point atomics): the same step from the same
    state gives the same bits, whichever tile shapes the batch size selects."""
    print("case determinism", B, prec, flush=True)
    cfgd = CONFIGS["dueling_ddqn"]
    m = dq.Dqn(dq.make_config(max_batch=512, precision=prec, **cfgd))
    p = torch.from_numpy(synth.he_uniform_params(1804, 18, 1))
    pt = torch.from_numpy(synth.he_uniform_params(5834, 18, 1))
    batch = tuple(dev(t) for t in synth.batch(11, B, 18))
    runs = []
    for rep in range(3):
        m.set_params(0, p); m.set_params(1, pt); m.set_params(3, torch.zeros_like(p))
        out = m.train_step(B, batch)
        runs.append([m.get_params(2).cpu().numpy(), m.get_params(0).cpu().numpy(), out["td"].cpu().numpy()])
    for rep in (1, 2):
        for x, y in zip(runs[0], runs[rep]):
            assert np.array_equal(x, y)
    m.close()


# ------------------------------------------------------------------ prioritized replay
def _fill_replay(m, cap, seed_frames=21, seed_meta=40, K=18, chunk=20000):
    for s0 in range(0, cap, chunk):
        n = min(chunk, cap - s0)
        fr = synth.frames(seed_frames, torch.arange(s0, s0 + n, device="cuda"), device="cuda")
        a = synth.actions(seed_meta, n, K, "cuda", first=s0)
        r = synth.rewards(seed_meta + 1, n, "cuda", first=s0)
        d = synth.dones(seed_meta + 2, n, 0.01, "cuda", first=s0)
        m.replay_write(s0, fr, a, r, d)
    torch.cuda.synchronize()


def _check_indices(orc, idx_gpu, tree_ref, size, B, beta, seed, stratified=False):
    idx_ref, w_ref, z = orc.per_sample(tree_ref, size, B, beta, seed, stratified)
    bad = np.flatnonzero(idx_gpu != idx_ref)
    if bad.size:
        _, dist = orc.per_sample_cumsum(tree_ref, size, z)
        assert np.all(dist[bad] <= TOL * tree_ref[1]), (bad, dist[bad])
    return idx_ref, w_ref


@pytest.mark.parametrize("cap,n,B,strat", [(1000, 1000, 32, 0), (1000, 613, 512, 0), (5000, 5000, 64, 1),
                                           (37, 37, 1024, 0), (5, 1, 7, 0),
                                           # 8, 14 and 19 tree levels: the walk's first round takes 8, 8 and 7 of them
                                           (200, 200, 64, 0), (10000, 10000, 64, 1), (300000, 300000, 128, 0)])
def test_tree_fill_sample_update(dq, orc, cap, n, B, strat):
    print("case tree", cap, n, B, strat, flush=True)
    alpha, eps = np.float32(0.6), np.float32(1e-6)
    m = dq.Dqn(dq.make_config(replay_capacity=cap, per_stratified=strat, max_batch=32))
    p = synth.exp_priorities(9, n)
    m.per_fill(dev(p))
    L = m.L
    tree_ref = orc.tree_build(p.numpy(), L, float(alpha))
    assert np.array_equal(m.tree.cpu().numpy()[1:], tree_ref[1:])           # every node, bit for bit
    idx, w = m.per_sample(B, 0.4, 4242)
    idx = idx.cpu().numpy(); w = w.cpu().numpy()
    idx_ref, w_ref = _check_indices(orc, idx, tree_ref, n, B, 0.4, 4242, bool(strat))
    same = idx == idx_ref
    assert same.mean() > 0.99
    assert relerr(w[same], w_ref[same]) <= TOL and idx.min() >= 0 and idx.max() < n
    # priority update with repeated indices (last one wins) and an out-of-range entry (skipped)
    nu = min(B, 40)
    uidx = idx[:nu].copy()
    if nu > 3:
        uidx[3] = uidx[0]
    td = (synth.u24(5, torch.arange(nu)) * 3).numpy()
    m.per_update(dev(uidx.astype(np.int32)), dev(td.astype(np.float32)))
    mp = orc.per_update(tree_ref, n, uidx.astype(np.int32), td.astype(np.float32), float(alpha), float(eps), 1.0)
    assert np.array_equal(m.tree.cpu().numpy()[1:], tree_ref[1:])
    assert float(m.max_priority) == np.float32(mp)
    m.close()


def test_per_update_skips_non_finite_errors(dq, orc):
    """A NaN or infinite TD error must not reach the tree: the entry is skipped on both sides."""
    print("case per_update non-finite", flush=True)
    cap, n = 1000, 64
    m = dq.Dqn(dq.make_config(replay_capacity=cap, max_batch=n))
    pri = synth.exp_priorities(9, cap)
    m.per_fill(dev(pri))
    tree_ref = orc.tree_build(pri.numpy(), m.L, float(np.float32(0.6)))
    idx = torch.arange(0, 2 * n, 2, dtype=torch.int32)
    td = (0.1 + synth.u24(5, torch.arange(n))).float()
    td[7] = float("nan"); td[20] = float("inf"); td[21] = -float("inf")
    m.per_update(dev(idx), dev(td))
    mp = orc.per_update(tree_ref, cap, idx.numpy(), td.numpy(), float(np.float32(0.6)), float(np.float32(1e-6)), 1.0)
    tree = m.tree.cpu().numpy()
    assert np.all(np.isfinite(tree)) and np.array_equal(tree[1:], tree_ref[1:])
    assert float(m.max_priority) == np.float32(mp) and np.isfinite(mp)
    m.close()


def test_replay_gather(dq, orc):
    print("case gather", flush=True)
    cap, K = 300, 18
    m = dq.Dqn(dq.make_config(replay_capacity=cap, max_batch=64))
    _fill_replay(m, cap, K=K)
    idx = np.array([0, 1, 2, 3, 150, 298, 299, 77], np.int32)
    s, sn, a, r, d = m.replay_gather(dev(idx))
    fr = synth.frames(21, torch.arange(cap)).numpy()
    s_ref, sn_ref = orc.gather(fr, idx)
    assert np.array_equal(s.cpu().numpy(), s_ref) and np.array_equal(sn.cpu().numpy(), sn_ref)
    assert np.array_equal(a.cpu().numpy(), synth.actions(40, cap, K).numpy()[idx])
    assert np.array_equal(r.cpu().numpy(), synth.rewards(41, cap).numpy()[idx])
    assert np.array_equal(d.cpu().numpy(), synth.dones(42, cap).numpy()[idx])
    m.close()


def _replay_step_case(dq, orc, cap, B, m=None, draw_seed=7, tol=TOL, cfgd=None, alpha=0.6, strat=0, prec=0):
    """Third configuration: PER sample + gather + (dueling) Double-DQN step + priority update."""
    cfgd = cfgd or CONFIGS["dueling_ddqn"]
    K, dueling = cfgd["num_actions"], cfgd["dueling"]
    alpha = float(np.float32(alpha))
    own = m is None
    if own:
        m = dq.Dqn(dq.make_config(replay_capacity=cap, max_batch=B, per_alpha=alpha, per_stratified=strat,
                                  precision=prec, **cfgd))
        _fill_replay(m, cap, K=K)
    strat = int(m.cfg.per_stratified)
    p = synth.he_uniform_params(1804, K, dueling)
    pt = synth.he_uniform_params(5834, K, dueling)
    m.set_params(0, torch.from_numpy(p)); m.set_params(1, torch.from_numpy(pt))
    m.set_params(3, torch.zeros(p.size))
    pri = synth.exp_priorities(9, cap, "cuda")
    m.per_fill(pri)
    tree_ref = orc.tree_build(pri.cpu().numpy(), m.L, alpha)
    out = m.train_step(B, None, beta=0.4, draw_seed=draw_seed)
    idx = out["idx"].cpu().numpy()
    idx_ref, w_ref = _check_indices(orc, idx, tree_ref, cap, B, 0.4, draw_seed, bool(strat))
    assert np.array_equal(idx, idx_ref), "a draw fell on a bucket boundary; pick another draw_seed"
    assert relerr(out["is_w"].cpu().numpy(), w_ref) <= TOL
    if alpha == 0.0:   # uniform replay (Eq.10 with exponent 0): every stored slot alike, every weight 1
        assert np.all(out["is_w"].cpu().numpy() == 1.0) and np.all(w_ref == 1.0)
    # the oracle regenerates only the frames it needs
    slots = (idx_ref[:, None].astype(np.int64) - 3 + np.arange(5)[None, :]) % cap
    fr = synth.frames(21, torch.from_numpy(slots.reshape(-1))).numpy().reshape(B, 5, 84, 84)
    s, sn = fr[:, :4], fr[:, 1:]
    ii = torch.from_numpy(idx_ref.astype(np.int64))
    a = synth.u24(40, ii); a = torch.clamp((a * K).floor().to(torch.int32), max=K - 1).numpy()
    r = (torch.clamp((synth.u24(41, ii) * 3).floor(), max=2.0) - 1.0).numpy()
    d = (synth.u24(42, ii) < 0.01).to(torch.uint8).numpy()
    bnp = (np.ascontiguousarray(s), np.ascontiguousarray(sn), a, r, d)
    prec = int(m.cfg.precision)
    ref = _oracle_step(orc, cfgd, p, pt, bnp, w_ref, quant=prec)
    ref64 = _oracle_step(orc, cfgd, p, pt, bnp, w_ref) if prec else None
    errs = _check_step(orc, out, ref, p, m, K, dueling, bnp, w_ref, tol, ref_full=ref64)
    if prec:
        _check_against_full_precision(out, ref64, m.get_params(0).cpu().numpy(), m.cfg.double_q, tol)
    # priorities written back from |td|
    td_abs = np.abs(out["td"].cpu().numpy()).astype(np.float32)
    orc.per_update(tree_ref, cap, idx_ref, td_abs, alpha, float(np.float32(1e-6)), 1.0)
    tree_gpu = m.tree.cpu().numpy()
    leaves_same = tree_gpu[m.L + idx_ref] == tree_ref[m.L + idx_ref]
    # |td| itself carries the fp32 tolerance, so leaves agree to that tolerance and the rest of
    # the tree must be consistent with its own leaves bit for bit
    assert relerr(tree_gpu[m.L + idx_ref], tree_ref[m.L + idx_ref]) <= tol, leaves_same.mean()
    lv = tree_gpu[m.L:2 * m.L].copy()
    chk = orc.tree_build(np.ones(0, np.float32), m.L, 1.0)
    chk[m.L:] = lv
    for i in range(m.L - 1, 0, -1):
        chk[i] = chk[2 * i] + chk[2 * i + 1]
    assert np.array_equal(tree_gpu[1:], chk[1:])
    if own:
        m.close()
    return errs


def test_replay_train_step_small_ring(dq, orc):
    print("case replay step small", flush=True)
    _replay_step_case(dq, orc, cap=4096, B=32)


@pytest.mark.parametrize("name,B,prec,alpha,strat", [
    ("dueling_ddqn", 32, 0, 0.0, 0), ("dueling_ddqn", 64, 1, 0.0, 0),     # uniform replay (exponent 0)
    ("ddqn_plain", 32, 0, 0.6, 0), ("ddqn_plain", 32, 0, 0.0, 0),          # plain head + Double DQN
    ("dueling_ddqn", 32, 0, 0.6, 1), ("dueling_ddqn", 512, 1, 0.6, 1),     # one draw per stratum, drawn in the forward kernel
    ("dueling_ddqn", 512, 0, 0.6, 1)])
def test_replay_step_settings(dq, orc, name, B, prec, alpha, strat):
    """The model settings of the paper's performance figure (Double DQN with a plain or a dueling
    head, uniform or prioritized replay) and stratified sampling, each as a whole replay-mode step:
    indices bit-exact, weights, every output, every gradient entry, the repaired tree."""
    print("case replay settings", name, B, prec, alpha, strat, flush=True)
    for seed in (7, 8, 9):
        try:
            _replay_step_case(dq, orc, cap=20000, B=B, draw_seed=seed, tol=TOL_BF16 if prec else TOL,
                              cfgd=CONFIGS[name], alpha=alpha, strat=strat, prec=prec)
            break
        except AssertionError as err:   # a draw on a bucket boundary: another seed
            if "bucket boundary" not in str(err):
                raise
    else:
        raise AssertionError("three draw seeds in a row hit a bucket boundary")


@pytest.mark.parametrize("prec,B,n", [(0, 32, 20000), (1, 512, 20000), (0, 7, 777)])
def test_uniform_replay_without_the_tree(dq, orc, prec, B, n):
    """Priority exponent 0 (the settings without prioritized replay of the paper's performance
    figure) over a bulk-filled tree: sampling reads no tree node and the priority update writes none.
    The result must be what the walk over the tree of ones gives, bit for bit: the same slots and
    weights from standalone sampling, the same parameters, the same tree and running maximum
    priority after training steps (DQN_NO_UNIFORM_FAST_PATH=1 sends the same context through the
    tree).  After the store path, which leaves zero leaves behind, the tree is walked again."""
    import os
    print("case uniform replay", prec, B, n, flush=True)
    K = 18
    ms = []
    for _ in range(2):
        m = dq.Dqn(dq.make_config(replay_capacity=n + 100, max_batch=B, per_alpha=0.0, precision=prec, **CONFIGS["dueling_ddqn"]))
        _fill_replay(m, n + 100, K=K, chunk=n + 100)
        m.per_fill(synth.exp_priorities(9, n, "cuda"))
        ms.append(m)
    tree_ref = orc.tree_build(synth.exp_priorities(9, n).numpy(), ms[0].L, 0.0)
    for strat_seed in (3, 4):
        idx_ref, w_ref, _ = orc.per_sample(tree_ref, n, B, 0.4, strat_seed)
        idx, w = ms[0].per_sample(B, 0.4, strat_seed)
        assert np.array_equal(idx.cpu().numpy(), idx_ref) and np.all(w.cpu().numpy() == 1.0) and np.all(w_ref == 1.0)
    try:
        for step in range(3):
            os.environ.pop("DQN_NO_UNIFORM_FAST_PATH", None)
            o0 = ms[0].train_step(B, None, beta=0.5, draw_seed=40 + step)
            os.environ["DQN_NO_UNIFORM_FAST_PATH"] = "1"
            o1 = ms[1].train_step(B, None, beta=0.5, draw_seed=40 + step)
            for k in o0:
                assert torch.equal(o0[k], o1[k]), (step, k)
            assert torch.equal(ms[0].get_params(0), ms[1].get_params(0)) and torch.equal(ms[0].tree, ms[1].tree)
            assert float(ms[0].max_priority) == float(ms[1].max_priority) >= 1.0
    finally:
        os.environ.pop("DQN_NO_UNIFORM_FAST_PATH", None)
    # the store path: slots without a whole transition get leaf 0 and must not be drawn
    m = ms[0]
    ref = orc.ReplayState(n + 100, 0.0)
    m2 = dq.Dqn(dq.make_config(replay_capacity=n + 100, max_batch=B, per_alpha=0.0, precision=prec, **CONFIGS["dueling_ddqn"]))
    pos = 0
    for cnt in (200, 300):
        fr = synth.frames(21, torch.arange(pos, pos + cnt, device="cuda"), device="cuda")
        d = synth.dones(42, cnt, 0.1, "cuda", first=pos)
        m2.replay_store(fr, synth.actions(40, cnt, K, "cuda", first=pos), synth.rewards(41, cnt, "cuda", first=pos), d)
        ref.store(d.cpu().numpy())
        pos += cnt
    assert np.array_equal(m2.tree.cpu().numpy()[1:], ref.tree[1:])
    idx_ref, w_ref, _ = orc.per_sample(ref.tree, ref.stored, B, 0.4, 9)
    idx, w = m2.per_sample(B, 0.4, 9)
    assert np.array_equal(idx.cpu().numpy(), idx_ref) and ref.tree[ref.L + idx_ref].min() == 1.0
    assert relerr(w.cpu().numpy(), w_ref) <= TOL
    out = m2.train_step(B, None, beta=0.4, draw_seed=9)
    assert np.array_equal(out["idx"].cpu().numpy(), idx_ref)
    for mm in ms + [m2]:
        mm.close()


def _seed_for_draw(u_index, ctr=0):
    """A draw seed whose draw number `ctr` is u = u_index * 2^-24: the mixer is a bijection of the
    64-bit word seed + (ctr + 1) * gamma, so it is inverted step by step."""
    M = (1 << 64) - 1
    z = (u_index << 40) | 0x5555555555
    z ^= z >> 31; z ^= z >> 62
    z = (z * pow(0x94D049BB133111EB, -1, 1 << 64)) & M
    z ^= z >> 27; z ^= z >> 54
    z = (z * pow(0xBF58476D1CE4E5B9, -1, 1 << 64)) & M
    z ^= z >> 30; z ^= z >> 60
    return (z - (ctr + 1) * 0x9E3779B97F4A7C15) & M


def test_draw_never_returns_a_zero_leaf(dq, orc):
    """Eq.10: a slot with leaf 0 has probability zero.  The tree and the draw u = 6410600 * 2^-24 are
    the case of tests/test_oracle_replay.py in which the textbook descent overshoots an inner node
    and ends on a zero leaf; the seed is built so that draw 0 (and, in a second seed, draw 5) is that
    u.  Standalone sampling and the draw inside the first forward kernel must both return the
    oracle's slot, a stored transition with a finite weight."""
    print("case zero leaf", flush=True)
    n, K = 3000, 18
    pr = synth.exp_priorities(13, n)
    pr[1::2] = 0.0
    tree_ref = orc.tree_build(pr.numpy(), 4096, float(np.float32(0.6)))
    assert synth.u24(_seed_for_draw(6410600), torch.arange(1)).item() == np.float32(6410600 * 2.0 ** -24)
    for prec in (0, 1):
        m = dq.Dqn(dq.make_config(replay_capacity=n, max_batch=16, precision=prec, **CONFIGS["dueling_ddqn"]))
        _fill_replay(m, n, K=K, chunk=n)
        for ctr, B in ((0, 1), (5, 16), (3, 7)):
            seed = _seed_for_draw(6410600, ctr)
            m.per_fill(dev(pr))
            assert np.array_equal(m.tree.cpu().numpy()[1:], tree_ref[1:])
            idx_ref, w_ref, z = orc.per_sample(tree_ref, n, B, 0.4, seed)
            assert tree_ref[4096 + idx_ref].min() > 0
            idx, w = m.per_sample(B, 0.4, seed)
            assert np.array_equal(idx.cpu().numpy(), idx_ref) and relerr(w.cpu().numpy(), w_ref) <= TOL
            out = m.train_step(B, None, beta=0.4, draw_seed=seed)
            assert np.array_equal(out["idx"].cpu().numpy(), idx_ref)
            assert relerr(out["is_w"].cpu().numpy(), w_ref) <= TOL and np.isfinite(float(out["loss"][0]))
            assert torch.isfinite(m.get_params(0)).all() and torch.isfinite(m.tree).all()
        m.close()


def test_tree_without_mass_trains_on_nothing(dq):
    """Four time steps through the store path complete no transition: the count of stored steps is 4
    but every leaf is 0.  Nothing can be drawn: weights 0, parameters, optimizer state and tree
    untouched, nothing NaN."""
    print("case tree without mass", flush=True)
    K = 18
    for prec in (0, 1):
        m = dq.Dqn(dq.make_config(replay_capacity=64, max_batch=8, precision=prec, **CONFIGS["dueling_ddqn"]))
        fr = synth.frames(21, torch.arange(4, device="cuda"), device="cuda")
        m.replay_store(fr, synth.actions(40, 4, K, "cuda"), synth.rewards(41, 4, "cuda"), torch.zeros(4, dtype=torch.uint8, device="cuda"))
        assert float(m.tree[1]) == 0.0 and m.replay_state()[1] == 4
        before, tree0 = m.get_params(0).clone(), m.tree.clone()
        idx, w = m.per_sample(8, 0.4, 1)
        assert torch.equal(w.cpu(), torch.zeros(8))
        out = m.train_step(8, None, beta=0.4, draw_seed=2)
        assert torch.equal(out["is_w"].cpu(), torch.zeros(8)) and float(out["loss"][0]) == 0.0
        assert torch.equal(m.get_params(0), before) and float(m.get_params(3).abs().max()) == 0.0
        assert torch.equal(m.tree, tree0)
        m.close()


@pytest.mark.parametrize("B", [5, 33, 512])
def test_fused_and_separate_conv_launches_agree(dq, B):
    """bf16: conv1 and conv2 of the forward pass run as one launch (conv1's output handed over in
    LDS) from a handful of samples on, and as two launches below that or when
    DQN_CONV12_MIN_SAMPLES says so.  Both do the same arithmetic in the same order: two contexts over
    identical state, one on each path, must agree bit for bit -- in replay mode (the first forward
    kernel draws the transitions), on an explicit batch, and when acting.  B = 5: workgroups with a
    single sample; 33: ragged shares; 512: six or seven samples per workgroup."""
    import os
    print("case fused conv1+conv2", B, flush=True)
    cap = 3000
    cfgd = dict(CONFIGS["dueling_ddqn"], max_batch=B, max_act_batch=max(B, 8), precision=1, replay_capacity=cap)
    ms = []
    for least in ("1", "1000000000"):
        os.environ["DQN_CONV12_MIN_SAMPLES"] = least
        try:
            m = dq.Dqn(dq.make_config(**cfgd))
        finally:
            os.environ.pop("DQN_CONV12_MIN_SAMPLES", None)
        _fill_replay(m, cap)
        m.per_fill(synth.exp_priorities(9, cap, "cuda"))
        ms.append(m)
    batch = tuple(dev(t) for t in synth.batch(17, B, 18))
    obs = batch[0]
    for step in range(3):
        outs = [m.train_step(B, None, beta=0.5, draw_seed=70 + step) for m in ms]
        for k in ("idx", "td", "loss", "q_s"):
            assert torch.equal(outs[0][k], outs[1][k]), (step, k)
        assert torch.equal(ms[0].get_params(0), ms[1].get_params(0)), step
    outs = [m.train_step(B, batch) for m in ms]
    assert torch.equal(outs[0]["td"], outs[1]["td"])
    assert torch.equal(ms[0].get_params(2), ms[1].get_params(2))
    acts = [m.act(obs, 0.0, 3, want_q=True) for m in ms]
    assert torch.equal(acts[0][1], acts[1][1]) and torch.equal(acts[0][0], acts[1][0])
    for m in ms:
        m.close()


@pytest.mark.parametrize("B", [5, 33, 300, 512, 1024])
def test_fused_and_separate_conv1_weight_gradient_agree(dq, B):
    """bf16: conv1's weight gradient runs inside the per-sample workgroups of conv2's backward launch
    (conv1's dY never leaves the CU), or as a launch of its own when DQN_FUSED_BWD=0 says so.  A workgroup
    takes the same samples in the same order as a sample split of the separate kernel, so two contexts over
    identical state, one on each path, must agree bit for bit: in replay mode (frames read from the ring,
    wrapping windows included) and on an explicit batch.  B = 5, 33: one sample per workgroup; 300: one or
    two; 512, 1024: two and four."""
    import os
    print("case fused conv2 dgrad + conv1 wgrad", B, flush=True)
    cap = 3000
    cfgd = dict(CONFIGS["dueling_ddqn"], max_batch=B, max_act_batch=8, precision=1, replay_capacity=cap)
    ms = []
    for fused in ("1", "0"):
        os.environ["DQN_FUSED_BWD"] = fused
        try:
            m = dq.Dqn(dq.make_config(**cfgd))
        finally:
            os.environ.pop("DQN_FUSED_BWD", None)
        _fill_replay(m, cap)
        m.per_fill(synth.exp_priorities(9, cap, "cuda"))
        ms.append(m)
    batch = tuple(dev(t) for t in synth.batch(23, B, 18))
    for step in range(3):
        outs = [m.train_step(B, None, beta=0.5, draw_seed=170 + step) for m in ms]
        for k in ("idx", "td", "loss"):
            assert torch.equal(outs[0][k], outs[1][k]), (step, k)
        for which in (0, 2, 3):   # theta, v, the gradient of the step
            assert torch.equal(ms[0].get_params(which), ms[1].get_params(which)), (step, which)
    outs = [m.train_step(B, batch) for m in ms]
    assert torch.equal(outs[0]["td"], outs[1]["td"])
    for which in (0, 2, 3):
        assert torch.equal(ms[0].get_params(which), ms[1].get_params(which)), which
    for m in ms:
        m.close()


@pytest.mark.parametrize("prec,B", [(0, 32), (1, 64), (1, 6), (1, 1024)])
def test_recorded_step_replays_match_plain_launches(dq, prec, B):
    """With DQN_GRAPH=1 the replay-mode step is recorded into a HIP graph and replayed.  Two
    contexts over identical state, one on the graph and one on plain launches, must agree
    bit for bit on every replay: enqueued back to back, with other work and synchronisations
    between the replays, with the outputs requested and not requested, after a change of batch
    size and after the number of stored transitions has changed.

    In bf16 the two also differ in who draws the transitions: the graph path runs the sampling
    kernel in front of the graph, the plain path lets the first forward kernel walk the tree
    (one sample per working wave at B = 6 and 3, three samples per wave at B = 1024)."""
    import os
    print("case graph replays", prec, B, flush=True)
    cap = 6000
    cfgd = dict(CONFIGS["dueling_ddqn"], max_batch=B, precision=prec, replay_capacity=cap)
    ms = []
    for graph in ("1", "0"):
        os.environ["DQN_GRAPH"] = graph
        try:
            m = dq.Dqn(dq.make_config(**cfgd))
        finally:
            os.environ.pop("DQN_GRAPH", None)
        _fill_replay(m, cap)
        m.per_fill(synth.exp_priorities(9, cap, "cuda"))
        ms.append(m)
    # a run of steps enqueued back to back, nothing waited for in between
    for m in ms:
        for step in range(5):
            m.train_step(B, None, beta=0.3 + 0.1 * step, draw_seed=500 + step, outputs=False)
    for which in (0, 3):
        assert torch.equal(ms[0].get_params(which), ms[1].get_params(which)), which
    assert torch.equal(ms[0].tree, ms[1].tree)
    for step in range(6):
        beta, seed = 0.4 + 0.1 * step, 1000 + step
        outs = [m.train_step(B, None, beta=beta, draw_seed=seed, outputs=(step % 3 == 2)) for m in ms]
        torch.cuda.synchronize()
        if step % 3 == 2:
            for k in outs[0]:
                assert torch.equal(outs[0][k], outs[1][k]), (step, k)
        # unrelated work between replays: sampling on its own, acting, a parameter read
        for m in ms:
            m.per_sample(B, 0.5, 77 + step)
            m.act(dev(synth.states(5, 3)), 0.0, 1)
        for which in (0, 3):
            assert torch.equal(ms[0].get_params(which), ms[1].get_params(which)), (step, which)
        assert torch.equal(ms[0].tree, ms[1].tree), step
    # a different batch size (a new recording) and a different number of stored transitions
    B2 = B // 2
    for m in ms:
        m.train_step(B2, None, beta=0.7, draw_seed=5)
        m.per_fill(synth.exp_priorities(10, cap - 100, "cuda"))
        m.train_step(B2, None, beta=0.7, draw_seed=6, outputs=False)
    torch.cuda.synchronize()
    assert torch.equal(ms[0].get_params(0), ms[1].get_params(0))
    assert torch.equal(ms[0].tree, ms[1].tree)
    for m in ms:
        m.close()


def test_replay_train_step_full_size(dq, orc):
    """The throughput configuration as bench.py launches it: 1,000,000-frame ring, batch 512,
    then batch 32 on the same context; every output of the step is compared."""
    print("case replay step full size", flush=True)
    cap = 1_000_000
    m = dq.Dqn(dq.make_config(replay_capacity=cap, max_batch=512, **CONFIGS["dueling_ddqn"]))
    _fill_replay(m, cap, K=18, chunk=25000)
    print("  ring filled", flush=True)
    e512 = _replay_step_case(dq, orc, cap, 512, m=m, draw_seed=11)
    print("  B=512 worst:", max(e512.items(), key=lambda kv: kv[1]), flush=True)
    e32 = _replay_step_case(dq, orc, cap, 32, m=m, draw_seed=12)
    print("  B=32 worst:", max(e32.items(), key=lambda kv: kv[1]), flush=True)
    m.close()


def test_replay_train_step_full_size_bf16(dq, orc):
    """The bf16 throughput configuration (fourth configuration): batch 512 from the 1M ring."""
    print("case replay step full size bf16", flush=True)
    cap = 1_000_000
    m = dq.Dqn(dq.make_config(replay_capacity=cap, max_batch=512, precision=1, **CONFIGS["dueling_ddqn"]))
    _fill_replay(m, cap, K=18, chunk=25000)
    e = _replay_step_case(dq, orc, cap, 512, m=m, draw_seed=11, tol=TOL_BF16)
    print("  bf16 B=512 worst:", sorted(e.items(), key=lambda kv: -kv[1])[:4], flush=True)
    e = _replay_step_case(dq, orc, cap, 256, m=m, draw_seed=13, tol=TOL_BF16)
    print("  bf16 B=256 worst:", sorted(e.items(), key=lambda kv: -kv[1])[:4], flush=True)
    m.close()


@pytest.mark.parametrize("B", [100, 320, 448, 480])
def test_replay_train_step_fp32_schedules(dq, orc, B):
    """fp32 replay step at batch sizes on both sides of the library's schedule switch: up to 448 the
    step stays on one stream (one backward launch per layer; the priority update, one workgroup of
    256 threads, takes two entries per thread from 257 entries on), above it the weight gradients
    run on side streams.  Every output and the repaired tree are held against the oracle.  At these
    sizes the batch holds millions of ReLU inputs and a handful of them are ties (|x| of a few 1e-7
    against an rms of 0.8); _check_step finds them in the GPU's stored activations and accounts for
    each one's contribution, so one fixed seed serves and no gradient entry is left out."""
    print("case replay step fp32 schedules B=%d" % B, flush=True)
    _replay_step_case(dq, orc, cap=30000, B=B, draw_seed=41)


def test_replay_train_step_wrapping_ring_bf16(dq, orc):
    """bf16 step over a 40-slot ring with batch 96: most slots are drawn, so the four-frame windows
    of s and s' that straddle the end (and the start) of the ring are read by the conv1 kernels'
    non-contiguous path, next to windows that are contiguous."""
    print("case replay step wrapping ring bf16", flush=True)
    cap = 40
    m = dq.Dqn(dq.make_config(replay_capacity=cap, max_batch=96, precision=1, **CONFIGS["dueling_ddqn"]))
    _fill_replay(m, cap, K=18, chunk=cap)
    for seed in (21, 22, 23):
        try:
            e = _replay_step_case(dq, orc, cap, 96, m=m, draw_seed=seed, tol=TOL_BF16)
            break
        except AssertionError as err:   # a draw on a bucket boundary: another seed
            if "bucket boundary" not in str(err):
                raise
    else:
        raise AssertionError("three draw seeds in a row hit a bucket boundary")
    m.per_fill(synth.exp_priorities(9, cap, "cuda"))         # the tree the step drew from
    idx = m.per_sample(96, 0.4, seed)[0].cpu().numpy()       # same tree, same seed: the step's draw
    assert (idx < 3).any() and (idx == cap - 1).any(), "the draw must include wrapping windows"
    print("  worst:", sorted(e.items(), key=lambda kv: -kv[1])[:4], flush=True)
    m.close()


def test_replay_train_step_bf16_maximum_batch(dq, orc):
    """bf16 replay step at B = 1024, the library's limit: a wave's units of conv1 work span three
    samples, the most its draw table is sized for.  (Very small bf16 batches are held against the
    oracle with explicit batches, and their in-kernel draws against the sampling kernel bit for
    bit in the recorded-step test: at B = 3 a single ReLU mask that flips on a bf16 rounding
    boundary moves a third of a gradient entry, which no tolerance on the gradients survives.)"""
    print("case replay step bf16 maximum batch", flush=True)
    cap = 20000
    m = dq.Dqn(dq.make_config(replay_capacity=cap, max_batch=1024, precision=1, **CONFIGS["dueling_ddqn"]))
    _fill_replay(m, cap, K=18, chunk=cap)
    e = _replay_step_case(dq, orc, cap, 1024, m=m, draw_seed=32, tol=TOL_BF16)
    print("  B=1024 worst:", sorted(e.items(), key=lambda kv: -kv[1])[:3], flush=True)
    m.close()


# ------------------------------------------------------------------ error paths
def test_store_path_parity(dq, orc):
    """Alg.2 store line: chunks of time steps appended at the cursor, every tree node compared
    bit for bit with the oracle's one-step-at-a-time store, across a ring wrap, episode ends and
    priority updates that raise the maximal priority; then the stored data drive a train step."""
    print("case store path", flush=True)
    cap, K, B = 3000, 18, 64
    m = dq.Dqn(dq.make_config(max_batch=B, replay_capacity=cap, **CONFIGS["dueling_ddqn"]))
    ref = orc.ReplayState(cap, float(np.float32(0.6)))
    assert ref.L == m.L
    pos = 0
    rng = np.random.default_rng(3)

    def store(n):
        nonlocal pos
        fr = synth.frames(21, torch.arange(pos, pos + n, device="cuda"), device="cuda")
        a = synth.actions(40, n, K, "cuda", first=pos)
        r = synth.rewards(41, n, "cuda", first=pos)
        d = synth.dones(42, n, 0.05, "cuda", first=pos)
        m.replay_store(fr, a, r, d)
        ref.store(d.cpu().numpy())
        pos += n
        assert np.array_equal(m.tree.cpu().numpy()[1:], ref.tree[1:]), pos
        assert m.replay_state() == (pos % cap, min(pos, cap), pos)

    for n in (1, 1, 2, 5, 64, 1020, 333):
        store(n)
    # updates with known |delta| raise the maximal priority; later stores must use it
    idx, _ = m.per_sample(B, 0.4, 17)
    td = (0.5 + 3.0 * synth.u24(77, torch.arange(B))).cuda()
    m.per_update(idx, td)
    ref.max_p = orc.per_update(ref.tree, ref.stored, idx.cpu().numpy(), td.cpu().numpy(), ref.alpha,
                               float(np.float32(1e-6)), ref.max_p)
    assert float(m.max_priority) == np.float32(ref.max_p)
    for n in (3, 1020, 1020, 17, 600):      # wraps the 3000-slot ring
        store(n)
    assert pos > cap
    # what is drawn is whole, and reads back as the frames that were stored
    idx, w = m.per_sample(B, 0.4, 5)
    idx_ref, _ = _check_indices(orc, idx.cpu().numpy(), ref.tree, ref.stored, B, 0.4, 5)
    s, sn, a, r, d = m.replay_gather(idx)
    base = pos - cap
    q = (idx_ref.astype(np.int64) - base % cap) % cap + base      # stream position held by each drawn slot
    assert np.all(q + 1 < pos) and np.all(q - 3 >= base)
    want = synth.frames(21, torch.from_numpy((q[:, None] - 3 + np.arange(5)[None, :]).reshape(-1))).reshape(B, 5, 84, 84)
    assert torch.equal(s.cpu(), want[:, :4]) and torch.equal(sn.cpu(), want[:, 1:])
    dn = synth.dones(42, pos, 0.05, "cpu").numpy()
    assert not any(dn[qq - 3:qq].any() for qq in q)
    out = m.train_step(B, None, beta=0.5, draw_seed=8)
    assert np.isfinite(float(out["loss"][0]))
    # error paths: too many steps in one call, NULL metadata
    fr = synth.frames(21, torch.arange(4, device="cuda"), device="cuda")
    with pytest.raises(dq.DqnError):
        m.replay_store(fr, None, None, None)
    m.close()


@pytest.mark.parametrize("prec,E,C,steps", [(0, 37, 40, 100), (1, 64, 16, 45), (1, 2048, 24, 30)])
def test_store_path_many_environment_streams(dq, orc, prec, E, C, steps):
    """Alg.1's store line with one emulator per stream: E sub-rings of C slots, one time step per
    stream and call.  The oracle's one-stream store runs once per stream on a ring of C slots; the
    leaves of stream e are slots eC .. eC+C-1 of the library's tree, whose every node is compared bit
    for bit (node = left + right).  Draws return whole transitions of one stream (the five frames
    read back are the ones that stream stored, also where the window wraps inside its sub-ring),
    N of Eq.12 is the number of stored transitions, and a training step on the stored data is held
    against the oracle like any other."""
    print("case store many streams", prec, E, C, steps, flush=True)
    K, B = 18, 48
    cap = E * C + 7                      # the last 7 slots belong to no stream
    cfgd = CONFIGS["dueling_ddqn"]
    alpha = float(np.float32(0.6))
    m = dq.Dqn(dq.make_config(replay_capacity=cap, max_batch=B, precision=prec, **cfgd))
    refs = [orc.ReplayState(C, alpha) for _ in range(E)]
    L = m.L
    ee = torch.arange(E)

    def frame_id(e, t):
        return e * 4096 + t

    def ref_tree():
        t = np.zeros(2 * L, np.float32)
        for e, r in enumerate(refs):
            t[L + e * C:L + (e + 1) * C] = r.tree[r.L:r.L + C]
        for i in range(L - 1, 0, -1):
            t[i] = t[2 * i] + t[2 * i + 1]
        return t

    max_p = 1.0
    for t in range(steps):
        fr = synth.frames(21, (frame_id(ee, t)).cuda(), device="cuda")
        a = synth.actions(40, E, K, "cuda", first=t * E)
        r = synth.rewards(41, E, "cuda", first=t * E)
        d = synth.dones(42, E, 0.07, "cuda", first=t * E)
        m.replay_store_envs(fr, a, r, d)
        dn = d.cpu().numpy()
        for e, rf in enumerate(refs):
            rf.max_p = max_p
            rf.store(dn[e:e + 1])
        if t in (0, 3, 4, 5, C - 1, C, C + 3, steps // 2, steps - 1):
            assert np.array_equal(m.tree.cpu().numpy()[1:], ref_tree()[1:]), t
        if t == steps // 2:   # priorities move; later stores enter with the raised maximum
            tr = ref_tree()
            n_st = E * min(t + 1, C)
            idx_ref, w_ref, _ = orc.per_sample(tr, n_st, B, 0.4, 17, limit=E * C)
            idx, w = m.per_sample(B, 0.4, 17)
            assert np.array_equal(idx.cpu().numpy(), idx_ref) and relerr(w.cpu().numpy(), w_ref) <= TOL
            td = (0.5 + 3.0 * synth.u24(77, torch.arange(B))).cuda()
            m.per_update(idx, td)
            max_p = orc.per_update(tr, E * C, idx_ref, td.cpu().numpy(), alpha, float(np.float32(1e-6)), max_p)
            assert float(m.max_priority) == np.float32(max_p)
            for e, rf in enumerate(refs):
                rf.tree[rf.L:rf.L + C] = tr[L + e * C:L + (e + 1) * C]
                for i in range(rf.L - 1, 0, -1):
                    rf.tree[i] = rf.tree[2 * i] + rf.tree[2 * i + 1]
    assert m.replay_state()[1] == E * min(steps, C) and m.replay_state()[2] == steps
    # a training step on what was stored, drawn by the step itself
    p = synth.he_uniform_params(1804, K, 1); pt = synth.he_uniform_params(5834, K, 1)
    m.set_params(0, torch.from_numpy(p)); m.set_params(1, torch.from_numpy(pt)); m.set_params(3, torch.zeros(p.size))
    tr = ref_tree()
    n_st = E * min(steps, C)
    for seed in (5, 6, 7):
        idx_ref, w_ref, z = orc.per_sample(tr, n_st, B, 0.4, seed, limit=E * C)
        _, dist = orc.per_sample_cumsum(tr, E * C, z)
        if np.all(dist > TOL * tr[1]):
            break
    out = m.train_step(B, None, beta=0.4, draw_seed=seed)
    assert np.array_equal(out["idx"].cpu().numpy(), idx_ref) and relerr(out["is_w"].cpu().numpy(), w_ref) <= TOL
    # the stream position each drawn slot holds, and the frames its window must read
    e_of, l_of = idx_ref // C, idx_ref % C
    q = l_of + ((steps - 1 - l_of) // C) * C            # latest time step written to local slot l
    assert np.all(q + 1 <= steps - 1) and np.all(q - 3 >= max(0, steps - C))
    ids = (e_of[:, None].astype(np.int64) * 4096 + (q[:, None] - 3 + np.arange(5)[None, :])).reshape(-1)
    want = synth.frames(21, torch.from_numpy(ids)).reshape(B, 5, 84, 84)
    s_g, sn_g, a_g, r_g, d_g = m.replay_gather(out["idx"])
    assert torch.equal(s_g.cpu(), want[:, :4]) and torch.equal(sn_g.cpu(), want[:, 1:])
    assert (l_of < 3).any() or C > 30, "no drawn window wraps inside its sub-ring: lengthen the run"
    bnp = (want[:, :4].contiguous().numpy(), want[:, 1:].contiguous().numpy(), a_g.cpu().numpy(), r_g.cpu().numpy(), d_g.cpu().numpy())
    tol = TOL_BF16 if prec else TOL
    ref = _oracle_step(orc, cfgd, p, pt, bnp, w_ref, quant=prec)
    ref64 = _oracle_step(orc, cfgd, p, pt, bnp, w_ref) if prec else None
    _check_step(orc, out, ref, p, m, K, 1, bnp, w_ref, tol, ref_full=ref64)
    with pytest.raises(dq.DqnError):
        m.replay_store_envs(fr[:E - 1], a, r, d)         # the number of streams is fixed
    m.close()


@pytest.mark.parametrize("H,W,use_lut", [(210, 160, True), (84, 84, False), (100, 333, True)])
def test_preprocess_parity(dq, orc, H, W, use_lut):
    """Sec.3 preprocessing: bytes equal the oracle's, except where the oracle's unrounded value
    lies within 1e-3 of a rounding boundary (the kernel blends in fp32), where one level is allowed."""
    print("case preprocess", H, W, use_lut, flush=True)
    n = 5
    raw = (synth.u24(61, torch.arange(n * H * W)) * 256).floor().clamp(max=255).to(torch.uint8).reshape(n, H, W)
    lut = (255.0 * synth.u24(62, torch.arange(256))).float() if use_lut else None
    out = dq.preprocess(raw.cuda(), None if lut is None else lut.cuda()).cpu().numpy()
    ref, val = orc.preprocess(raw.numpy(), None if lut is None else lut.numpy())
    diff = out.astype(np.int32) - ref.astype(np.int32)
    near = np.abs(val - np.floor(val) - 0.5) <= 1e-3
    assert np.all(diff[~near] == 0) and np.all(np.abs(diff) <= 1), (np.abs(diff).max(), (diff != 0).sum())
    with pytest.raises(dq.DqnError):
        dq.preprocess(torch.zeros(0, H, W, dtype=torch.uint8, device="cuda"))


# ------------------------------------------------------------------ degenerate and maximal cases
@pytest.mark.parametrize("prec", [0, 1])
def test_degenerate_batches(dq, orc, prec):
    """Every transition terminal (y = r, Alg.1 terminal line), every importance weight zero (no
    gradient: the parameters must not move at all), a single action (argmax trivial)."""
    print("case degenerate", prec, flush=True)
    tol = TOL_BF16 if prec else TOL
    cfgd = CONFIGS["dueling_ddqn"]
    K, B = 18, 40
    m = dq.Dqn(dq.make_config(max_batch=64, precision=prec, **cfgd))
    p = synth.he_uniform_params(1804, K, 1, bias_scale=0.02); pt = synth.he_uniform_params(5834, K, 1, bias_scale=0.02)
    s, sn, a, r, d = synth.batch(11, B, K)
    # all terminal
    m.set_params(0, torch.from_numpy(p)); m.set_params(1, torch.from_numpy(pt))
    ones = torch.ones_like(d)
    out = m.train_step(B, tuple(dev(t) for t in (s, sn, a, r, ones)))
    assert torch.equal(out["y"].cpu(), r)
    ref = _oracle_step(orc, cfgd, p, pt, (s.numpy(), sn.numpy(), a.numpy(), r.numpy(), ones.numpy()), None, quant=prec)
    assert relerr(out["td"].cpu().numpy(), ref["td"]) <= tol
    # all weights zero: loss 0, gradient 0, parameters and optimizer state untouched bit for bit
    m.set_params(0, torch.from_numpy(p)); m.set_params(3, torch.zeros(p.size))
    before = m.get_params(0).clone()
    out = m.train_step(B, tuple(dev(t) for t in (s, sn, a, r, d, torch.zeros(B))))
    assert float(out["loss"][0]) == 0.0
    assert float(m.get_params(2).abs().max()) == 0.0
    assert torch.equal(m.get_params(0), before) and float(m.get_params(3).abs().max()) == 0.0
    m.close()
    # one action
    m1 = dq.Dqn(dq.make_config(num_actions=1, dueling=1, double_q=1, loss_kind=1, max_batch=8, precision=prec))
    p1 = synth.he_uniform_params(7, 1, 1, bias_scale=0.02)
    m1.set_params(0, torch.from_numpy(p1)); m1.sync_target()
    s, sn, a, r, d = synth.batch(12, 8, 1)
    out = m1.train_step(8, tuple(dev(t) for t in (s, sn, a, r, d)))
    assert int(out["a_star"].abs().max()) == 0
    ref = _oracle_step(orc, dict(num_actions=1, dueling=1, double_q=1, loss_kind=1), p1, p1,
                       (s.numpy(), sn.numpy(), a.numpy(), r.numpy(), d.numpy()), None, quant=prec)
    assert relerr(out["q_s"].cpu().numpy(), ref["q_s"]) <= tol and relerr(out["td"].cpu().numpy(), ref["td"]) <= tol
    m1.close()


def test_smallest_ring_and_single_stored_transition(dq, orc):
    """A ring of the minimum capacity (5 slots) and a tree with one non-zero leaf: every draw
    returns that slot with weight 1."""
    print("case tiny ring", flush=True)
    m = dq.Dqn(dq.make_config(replay_capacity=5, max_batch=8, **CONFIGS["dueling_ddqn"]))
    _fill_replay(m, 5, chunk=5)
    m.per_fill(dev(np.array([0.7], np.float32)))
    idx, w = m.per_sample(8, 0.4, 3)
    assert int(idx.abs().max()) == 0 and torch.equal(w.cpu(), torch.ones(8))
    m.per_fill(dev(np.array([1e-3, 0.5, 2.0, 1.0, 0.25], np.float32)))
    tree_ref = orc.tree_build(np.array([1e-3, 0.5, 2.0, 1.0, 0.25], np.float32), m.L, float(np.float32(0.6)))
    idx, w = m.per_sample(8, 0.4, 4)
    _check_indices(orc, idx.cpu().numpy(), tree_ref, 5, 8, 0.4, 4)
    out = m.train_step(8, None, beta=0.4, draw_seed=4)        # stacks wrap around the 5-slot ring
    s, sn, _, _, _ = m.replay_gather(out["idx"])
    fr = synth.frames(21, torch.arange(5)).numpy()
    slots = (out["idx"].cpu().numpy()[:, None].astype(np.int64) - 3 + np.arange(5)[None, :]) % 5
    assert np.array_equal(s.cpu().numpy(), fr[slots[:, :4]]) and np.array_equal(sn.cpu().numpy(), fr[slots[:, 1:]])
    assert np.isfinite(float(out["loss"][0]))
    m.close()


def test_maximum_batch(dq, orc):
    """max_batch = 1024 (the library's limit), fp32: the whole step against the oracle run on all
    1024 rows, every output and every gradient entry.  And a property that holds at any size: the
    loss is a mean over rows, so the gradient of the step is the mean of the gradients of its two
    512-row halves."""
    print("case max batch", flush=True)
    cfgd = CONFIGS["dueling_ddqn"]
    K, B = 18, 1024
    m = dq.Dqn(dq.make_config(max_batch=B, **cfgd))
    p = synth.he_uniform_params(1804, K, 1, bias_scale=0.02); pt = synth.he_uniform_params(5834, K, 1, bias_scale=0.02)
    s, sn, a, r, d = synth.batch(11, B, K)
    full = tuple(dev(t) for t in (s, sn, a, r, d))

    def step(rows):
        m.set_params(0, torch.from_numpy(p)); m.set_params(1, torch.from_numpy(pt)); m.set_params(3, torch.zeros(p.size))
        out = m.train_step(rows.stop - rows.start, tuple(t[rows] for t in full))
        return out, m.get_params(2).cpu().numpy().astype(np.float64)

    _, g_lo = step(slice(0, 512))
    _, g_hi = step(slice(512, B))
    out, g_all = step(slice(0, B))
    assert relerr(g_all, 0.5 * (g_lo + g_hi)) <= TOL
    bnp = (s.numpy(), sn.numpy(), a.numpy(), r.numpy(), d.numpy())
    ref = _oracle_step(orc, cfgd, p, pt, bnp, None)
    print("  oracle done", flush=True)
    _check_step(orc, out, ref, p, m, K, 1, bnp, None, TOL)
    m.close()


def test_rows_with_an_action_out_of_range_are_not_trained_on(dq, orc):
    """An action outside [0, K) names no output of the network.  Such a row enters the step with
    weight 0 (the same loss, gradient and update as the oracle gives with that row's weight set to
    0) and its TD error is reported as NaN; the other rows are untouched."""
    print("case invalid action", flush=True)
    cfgd = CONFIGS["dueling_ddqn"]
    K, B = 18, 12
    for prec in (0, 1):
        tol = TOL_BF16 if prec else TOL
        m = dq.Dqn(dq.make_config(max_batch=16, precision=prec, **cfgd))
        p = synth.he_uniform_params(1804, K, 1, bias_scale=0.02); pt = synth.he_uniform_params(5834, K, 1, bias_scale=0.02)
        m.set_params(0, torch.from_numpy(p)); m.set_params(1, torch.from_numpy(pt))
        s, sn, a, r, d = synth.batch(11, B, K)
        a_bad = a.clone(); a_bad[3] = K + 5; a_bad[7] = -1
        out = m.train_step(B, tuple(dev(t) for t in (s, sn, a_bad, r, d)))
        td = out["td"].cpu().numpy()
        assert np.isnan(td[[3, 7]]).all() and np.isfinite(np.delete(td, [3, 7])).all()
        w0 = np.ones(B, np.float32); w0[[3, 7]] = 0.0
        ref = _oracle_step(orc, cfgd, p, pt, (s.numpy(), sn.numpy(), a.numpy(), r.numpy(), d.numpy()), w0, quant=prec)
        keep = np.delete(np.arange(B), [3, 7])
        assert relerr(td[keep], ref["td"][keep]) <= tol
        assert abs(float(out["loss"][0]) - ref["loss"]) <= tol * abs(ref["loss"])
        g = m.get_params(2).cpu().numpy()
        for name, (o, shp) in orc.param_slices(K, 1).items():
            sl = slice(o, o + int(np.prod(shp)))
            e = np.linalg.norm(g[sl] - ref["grads"][sl]) / np.linalg.norm(ref["grads"][sl])
            assert e <= tol, (name, e)
        assert torch.isfinite(m.get_params(0)).all()
        m.close()


def test_error_paths_on_device(dq):
    print("case errors", flush=True)
    m = dq.Dqn(dq.make_config(replay_capacity=100, max_batch=8, max_act_batch=8))
    with pytest.raises(dq.DqnError) as e:
        m.per_sample(4, 0.4, 1)                      # nothing stored yet
    assert e.value.code == dq.ERR_STATE
    with pytest.raises(dq.DqnError) as e:
        m.train_step(4, None)
    assert e.value.code == dq.ERR_STATE
    with pytest.raises(dq.DqnError) as e:
        m.train_step(9, tuple(dev(t) for t in synth.batch(1, 9, 18)))
    assert e.value.code == dq.ERR_INVALID_ARG
    with pytest.raises(dq.DqnError) as e:
        m.act(dev(synth.states(1, 9)), 0.0, 1)
    assert e.value.code == dq.ERR_INVALID_ARG
    with pytest.raises(dq.DqnError) as e:
        m.act(dev(synth.states(1, 2)), 1.5, 1)
    assert e.value.code == dq.ERR_INVALID_ARG
    with pytest.raises(dq.DqnError) as e:
        m.per_fill(dev(synth.exp_priorities(1, 101)))
    assert e.value.code == dq.ERR_INVALID_ARG
    with pytest.raises(dq.DqnError):
        m.get_params(4)                              # not centered
    m2 = dq.Dqn(dq.make_config())
    with pytest.raises(dq.DqnError) as e:
        m2.per_fill(dev(synth.exp_priorities(1, 4)))  # context without replay
    assert e.value.code == dq.ERR_STATE
    m.close(); m2.close()

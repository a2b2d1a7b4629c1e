"""dqn_act_static, the acting entry point that allocates nothing (its scratch is a static device
array inside the library), against dqn_act on the same inputs: two calls in a row, the second with
a smaller input, both precisions.  The two entry points run the same kernels in the same launch
shapes, so the results must agree bit for bit (well inside the 1e-4 / 2e-2 tolerance of the other
parity tests); the Q-values are also held against the oracle."""
import numpy as np
import pytest
import torch

from paper_1804_05834_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("prec", [0, 1])
def test_act_static_matches_act(orc, prec):
    from paper_1804_05834_amd import dqn
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    print("case act static", prec, flush=True)
    K, dueling = 18, 1
    m = dqn.Dqn(dqn.make_config(num_actions=K, dueling=dueling, max_act_batch=64, precision=prec))
    p = synth.he_uniform_params(21, K, dueling, bias_scale=0.05)
    m.set_params(0, torch.from_numpy(p))
    tol = 2e-2 if prec else 1e-4
    # outputs allocated up front: nothing is allocated between the two static calls
    outs = [(torch.full((E,), -7, dtype=torch.int32, device="cuda"), torch.full((E, K), -7.0, device="cuda"))
            for E in (32, 5)]
    obs = [synth.states(31, 32).cuda(), synth.states(32, 5).cuda()]
    torch.cuda.synchronize()
    for (acts, q), o in zip(outs, obs):                  # two calls in a row, the second smaller
        m.act(o, 0.25, 77, static=True, out=(acts, q))
    torch.cuda.synchronize()
    for (acts, q), o in zip(outs, obs):
        a_ref, q_ref = m.act(o, 0.25, 77, want_q=True)
        assert torch.equal(acts, a_ref) and torch.equal(q, q_ref)
        q_orc = orc.forward(p, K, dueling, o.cpu().numpy(), quant=prec)
        err = np.abs(q.cpu().numpy() - q_orc).max() / np.abs(q_orc).max()
        assert err <= tol, err
    # a size beyond the static array is refused with a clear error, and nothing is written
    big = synth.states(33, 33).cuda()
    guard = torch.full((33,), -7, dtype=torch.int32, device="cuda")
    with pytest.raises(dqn.DqnError) as e:
        m.act(big, 0.0, 1, static=True, out=(guard, None))
    assert e.value.code == dqn.ERR_INVALID_ARG and "DQN_ACT_STATIC_MAX" in str(e.value)
    assert int((guard != -7).sum()) == 0
    m.close()

"""Does the step learn?  The agent loop of Alg.1 / Alg.2 (act, store with maximal priority,
prioritized sampling, dueling Double-DQN step, target copies, Table 1-style ramps) around a toy
"catch" environment that stands in for the Atari emulator the paper uses.  A random policy
catches about one ball in four (mean reward about -0.5); after 60,000 environment steps the
near-greedy policy must catch clearly more than half."""
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("precision", [0, 1])
def test_catch_is_learned(precision):
    from paper_1804_05834_amd import dqn, toy_catch
    assert torch.cuda.is_available()
    dqn.lib()
    print("case learning, precision", precision, flush=True)
    final, early = toy_catch.run(60000, seed=0, precision=precision, update_period=1, target_period=1000,
                                 log=lambda s: print("  " + s, flush=True))
    print("  evaluation %.2f, first 100 training episodes %.2f" % (final, early), flush=True)
    assert early < 0.0
    assert final >= 0.5


def test_every_model_setting_runs_the_agent_loop():
    """The four settings of the paper's comparison (plain / dueling head, uniform / prioritized
    replay) through the whole loop, store path included (with exponent 0 the store path's zero
    leaves send the draws through the tree): a short run each, finite and above the floor."""
    from paper_1804_05834_amd import dqn, toy_catch
    dqn.lib()
    for name, dueling, alpha in toy_catch.SETTINGS:
        final, early = toy_catch.run(4000, seed=3, dueling=dueling, per_alpha=alpha, update_period=1,
                                     target_period=500, eval_episodes=30)
        print("  %s: evaluation %.2f" % (name, final), flush=True)
        assert -1.0 <= final <= 1.0 and -1.0 <= early <= 1.0

"""A toy environment and the agent loop of Alg.1 / Alg.2 around the library.

The paper evaluates on Atari Breakout through the ALE emulator, which is not available here.
This module stands in with "catch": an 8x8 ball falls 4 pixels per step from a random column of an
84x84 frame, a 16x4 paddle on the bottom row moves 8 pixels left / stays / moves right; the episode
ends when the ball reaches the paddle's row with reward +1 if it is caught and -1 otherwise.  The
loop is the paper's: epsilon-greedy acting, storing every time step with the maximal priority,
prioritized sampling, a dueling Double-DQN step every `update_period` environment steps, a target
copy every `target_period` steps, with epsilon and beta on linear ramps.

Everything the method computes runs in the library's kernels; this file only moves the ball.
"""
import torch

from . import dqn

K = 3  # left, stay, right


class Catch:
    def __init__(self, seed, device="cuda"):
        self.g = torch.Generator().manual_seed(seed)
        self.device = device
        self.reset()

    def reset(self):
        self.ball_x = int(torch.randint(0, 77, (1,), generator=self.g))   # left edge of the 8x8 ball
        self.ball_y = 0
        self.pad_x = int(torch.randint(0, 9, (1,), generator=self.g)) * 8   # left edge of the 16x4 paddle
        return self.frame()

    def frame(self):
        f = torch.zeros(84, 84, dtype=torch.uint8, device=self.device)
        f[self.ball_y:self.ball_y + 8, self.ball_x:self.ball_x + 8] = 255
        f[80:84, self.pad_x:self.pad_x + 16] = 160
        return f

    def step(self, action):
        """-> (reward, done); the next frame is frame() (after reset() when done)."""
        self.pad_x = min(max(self.pad_x + 8 * (action - 1), 0), 68)
        self.ball_y += 4
        if self.ball_y + 8 >= 80:
            caught = self.ball_x + 8 > self.pad_x and self.ball_x < self.pad_x + 16
            return (1.0 if caught else -1.0), True
        return 0.0, False


def run(env_steps, seed=0, capacity=20000, batch=32, precision=0, learning_start=1000, update_period=2,
        target_period=500, eps_steps=15000, lr=2.5e-4, eval_episodes=100, log=None, dueling=1, per_alpha=0.6,
        curve=None):
    """Trains for env_steps environment steps; returns (mean reward per episode of a near-greedy
    evaluation with Table 1's test epsilon 0.001, mean reward of the first 100 training episodes).
    dueling / per_alpha select the model setting (Sec.4: plain or dueling head, uniform replay =
    exponent 0 or prioritized replay).  curve: a list that receives the reward of every training episode."""
    m = dqn.Dqn(dqn.make_config(num_actions=K, dueling=dueling, double_q=1, precision=precision, loss_kind=1,
                                lr=lr, max_batch=batch, max_act_batch=1, replay_capacity=capacity,
                                per_alpha=per_alpha, per_eps=1e-3, seed=1804 + seed, target_seed=5834 + seed))
    m.sync_target()
    sc = dqn.schedule_default()
    sc.learning_start, sc.update_period, sc.target_period = learning_start, update_period, target_period
    sc.eps_steps, sc.beta_steps = eps_steps, env_steps
    env = Catch(seed)
    dev = "cuda"
    obs = env.reset().repeat(4, 1, 1).unsqueeze(0).contiguous()           # [1][4][84][84]
    rew_t = torch.zeros(1, device=dev); done_t = torch.zeros(1, dtype=torch.uint8, device=dev)
    returns = []
    for t in range(1, env_steps + 1):
        eps, beta, train, sync = dqn.schedule_at(sc, t)
        act = m.act(obs, eps, t)
        r, done = env.step(int(act[0]))
        rew_t.fill_(r); done_t.fill_(int(done))
        # the time step (x_t = newest frame of the state acted on, a_t, r_t, done_t)
        m.replay_store(obs[0, 3:4], act, rew_t, done_t)
        if done:
            returns.append(r)
            obs = env.reset().repeat(4, 1, 1).unsqueeze(0).contiguous()
        else:
            obs = torch.cat([obs[:, 1:], env.frame()[None, None]], dim=1).contiguous()
        if train:
            m.train_step(batch, None, beta=beta, draw_seed=t, outputs=False)
        if sync:
            m.sync_target()
        if log and t % 5000 == 0:
            log("step %d: eps %.2f, mean reward of the last 100 episodes %.2f" % (t, eps, sum(returns[-100:]) / max(1, len(returns[-100:]))))
    # evaluation, near-greedy
    ev = Catch(seed + 1000)
    obs = ev.reset().repeat(4, 1, 1).unsqueeze(0).contiguous()
    total, t = 0.0, 0
    for ep in range(eval_episodes):
        while True:
            t += 1
            act = m.act(obs, 0.001, 10_000_000 + t)
            r, done = ev.step(int(act[0]))
            if done:
                total += r
                obs = ev.reset().repeat(4, 1, 1).unsqueeze(0).contiguous()
                break
            obs = torch.cat([obs[:, 1:], ev.frame()[None, None]], dim=1).contiguous()
    m.close()
    if curve is not None:
        curve.extend(returns)
    early = sum(returns[:100]) / max(1, len(returns[:100]))
    return total / eval_episodes, early


SETTINGS = (("double DQN", 0, 0.0), ("dueling double DQN", 1, 0.0),
            ("double DQN with prioritized replay", 0, 0.6),
            ("dueling double DQN with prioritized replay", 1, 0.6))


def sweep(env_steps=20000, seeds=(0, 1, 2), log=print):
    """The four model settings of the paper's performance comparison (Sec.4) on the toy environment:
    per setting and seed the near-greedy evaluation reward after env_steps steps and the mean reward
    over all training episodes (the area under the learning curve, which separates settings that all
    end near the ceiling)."""
    table = []
    for name, dueling, alpha in SETTINGS:
        finals, areas = [], []
        for seed in seeds:
            curve = []
            final, _ = run(env_steps, seed=seed, update_period=1, target_period=1000, dueling=dueling,
                           per_alpha=alpha, curve=curve)
            finals.append(final)
            areas.append(sum(curve) / max(1, len(curve)))
            log("%-44s seed %d: evaluation %.2f, mean training reward %.3f" % (name, seed, final, areas[-1]))
        table.append((name, sum(finals) / len(finals), sum(areas) / len(areas), finals, areas))
    log("setting | mean evaluation reward | mean training reward (area under the curve)")
    for name, f, a, _, _ in table:
        log("%-44s | %.3f | %.3f" % (name, f, a))
    return table


if __name__ == "__main__":
    import sys
    if len(sys.argv) > 1 and sys.argv[1] == "sweep":
        sweep(int(sys.argv[2]) if len(sys.argv) > 2 else 20000)
    else:
        steps = int(sys.argv[1]) if len(sys.argv) > 1 else 30000
        final, early = run(steps, log=lambda s: print(s, flush=True))
        print("evaluation: mean reward per episode %.2f (first 100 training episodes: %.2f)" % (final, early))

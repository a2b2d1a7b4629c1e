"""Pins for the counter-based draws and the synthetic-input generators."""
import numpy as np
import torch

from paper_1804_05834_amd import synth


def _mix_py(seed, ctr):
    """The mixer written out with Python integers (independent of both C and torch)."""
    M = (1 << 64) - 1
    z = (seed + (ctr + 1) * 0x9E3779B97F4A7C15) & M
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M
    return z ^ (z >> 31)


def test_mixer_three_ways(orc):
    for seed in (0, 1, 21, 1804, 2**63 + 12345, 2**64 - 1):
        ctrs = [0, 1, 2, 881, 882, 10**6, 2**40 + 7, 2**63 - 2]
        t = synth.mix64(seed, torch.tensor(ctrs, dtype=torch.int64))
        for c, tv in zip(ctrs, t.tolist()):
            ref = _mix_py(seed, c)
            assert orc.mix64(seed, c) == ref
            assert (tv & ((1 << 64) - 1)) == ref


def test_splitmix64_published_sequence(orc):
    # With seed 0 and counter k the mixer is the (k+1)-th output of SplitMix64 seeded with 0;
    # its first outputs are widely published test vectors.
    assert orc.mix64(0, 0) == 0xE220A8397B1DCDAF
    assert orc.mix64(0, 1) == 0x6E789E6AA1B965F4
    assert orc.mix64(0, 2) == 0x06C45D188009454F


def test_u24_range_and_exactness(orc):
    u = synth.u24(5, torch.arange(100000, dtype=torch.int64))
    assert u.dtype == torch.float32 and float(u.min()) >= 0.0 and float(u.max()) < 1.0
    assert torch.all(u * 16777216.0 == torch.floor(u * 16777216.0))
    for c in (0, 17, 99999):
        assert orc.draw_u24(5, c) == float(u[c])
    # roughly uniform
    assert abs(float(u.mean()) - 0.5) < 5e-3


def test_frames_are_pure_functions_of_slot():
    a = synth.frames(21, [5, 6, 7, 999999])
    b = synth.frames(21, [999999, 6])
    assert a.shape == (4, 84, 84) and a.dtype == torch.uint8
    assert torch.equal(a[3], b[0]) and torch.equal(a[1], b[1])
    w = _mix_py(21, 6 * 882 + 3)
    assert int(a[1].reshape(-1)[3 * 8 + 2]) == (w >> 16) & 0xFF
    # bytes are spread over the whole range
    h = torch.bincount(synth.frames(21, list(range(64))).reshape(-1).long(), minlength=256)
    assert h.min() > 0.8 * h.float().mean()


def test_batch_recipe_value_ranges():
    s, sn, a, r, d = synth.batch(11, 64, 18)
    assert s.shape == (64, 4, 84, 84) and sn.shape == s.shape and not torch.equal(s, sn)
    assert int(a.min()) >= 0 and int(a.max()) <= 17
    assert set(r.tolist()) <= {-1.0, 0.0, 1.0}
    assert set(d.tolist()) <= {0, 1}
    dd = synth.dones(4, 200000, 0.01)
    assert abs(float(dd.float().mean()) - 0.01) < 2e-3


def test_he_uniform_bounds():
    for K, due in ((4, False), (18, True)):
        p = synth.he_uniform_params(1804, K, due)
        assert p.dtype == np.float32 and p.size == synth.param_count(K, due)
        o = 0
        for name, shape, fan_in in synth.param_spec(K, due):
            n = int(np.prod(shape))
            blk = p[o:o + n]
            if fan_in:
                b = np.sqrt(6.0 / fan_in)
                assert np.abs(blk).max() <= b * (1 + 1e-6) and np.abs(blk).max() > 0.9 * b
                assert abs(blk.mean()) < 0.05 * b
            else:
                assert np.all(blk == 0)
            o += n
    assert synth.param_count(4, False) == 1686180 and synth.param_count(18, True) == 1693875


def test_exp_priorities_distribution():
    p = synth.exp_priorities(9, 400000).double()
    assert float(p.min()) > 0
    assert abs(float(p.mean()) - 1.0) < 1e-2 and abs(float(p.var()) - 1.0) < 3e-2

"""Seeded synthetic inputs with the shapes of the paper's Atari workload.

This module holds input generators only (no arithmetic of the method): frames,
actions, rewards, terminal flags, raw priorities and initial weights, all pure
functions of (seed, counter) through one 64-bit counter mixer, so any subset can
be regenerated anywhere (CPU for the checker, GPU for filling the replay ring)
without storing the rest.  It imports nothing else from this package.

Mixer: z = seed + (ctr+1)*0x9E3779B97F4A7C15; z = (z ^ z>>30)*0xBF58476D1CE4E5B9;
z = (z ^ z>>27)*0x94D049BB133111EB; z ^= z>>31  (64-bit wrap-around; the
SplitMix64 output function).  A uniform in [0,1) is (z >> 40) * 2^-24.
"""
import math

import numpy as np
import torch

FRAME = 84 * 84            # bytes per frame
WORDS_PER_FRAME = FRAME // 8   # 882 64-bit draws per frame

_M64 = (1 << 64) - 1


def _s64(c):
    """Python int (mod 2^64) -> the signed value with the same 64-bit pattern."""
    c &= _M64
    return c - (1 << 64) if c >= (1 << 63) else c


_GAMMA = _s64(0x9E3779B97F4A7C15)
_C1 = _s64(0xBF58476D1CE4E5B9)
_C2 = _s64(0x94D049BB133111EB)


def _lsr(x, s):
    return (x >> s) & ((1 << (64 - s)) - 1)


def mix64(seed, ctr):
    """ctr: int64 tensor of counters -> int64 tensor holding the 64-bit pattern."""
    z = (ctr + 1) * _GAMMA + _s64(seed)
    z = (z ^ _lsr(z, 30)) * _C1
    z = (z ^ _lsr(z, 27)) * _C2
    return z ^ _lsr(z, 31)


def u24(seed, ctr):
    """Uniform draws in [0,1) with 24 bits, exact in float32."""
    return _lsr(mix64(seed, ctr), 40).to(torch.float32) * (1.0 / 16777216.0)


def _arange(n, device, start=0):
    return torch.arange(start, start + n, dtype=torch.int64, device=device)


def frames(seed, slots, device="cpu"):
    """uint8 [len(slots)][84][84]: byte k of slot i is byte (k%8) of mix64(seed, i*882 + k//8)."""
    slots = torch.as_tensor(slots, dtype=torch.int64, device=device).reshape(-1)
    ctr = slots[:, None] * WORDS_PER_FRAME + _arange(WORDS_PER_FRAME, device)[None, :]
    words = mix64(seed, ctr)                                   # [n][882]
    shifts = (_arange(8, device) * 8)[None, None, :]
    b = (words[:, :, None] >> shifts) & 0xFF
    return b.to(torch.uint8).reshape(-1, 84, 84)


def states(seed, n, device="cpu", first=0):
    """uint8 [n][4][84][84], i.i.d. uniform bytes: state j is frames 4j..4j+3 of the stream."""
    return frames(seed, _arange(4 * n, device, 4 * first), device).reshape(n, 4, 84, 84)


def actions(seed, n, K, device="cpu", first=0):
    u = u24(seed, _arange(n, device, first))
    return torch.clamp((u * K).floor().to(torch.int32), max=K - 1)


def rewards(seed, n, device="cpu", first=0):
    """uniform over {-1, 0, 1}"""
    u = u24(seed, _arange(n, device, first))
    return torch.clamp((u * 3).floor(), max=2.0) - 1.0


def dones(seed, n, p=0.01, device="cpu", first=0):
    return (u24(seed, _arange(n, device, first)) < p).to(torch.uint8)


def exp_priorities(seed, n, device="cpu", first=0):
    """raw priorities p_i = -ln(1 - u_i)  (Exp(1)), computed in double, stored as float32;
    u = 0 would give p = 0, which a priority may not be, so it is lifted to 2^-25."""
    u = u24(seed, _arange(n, device, first)).to(torch.float64)
    u = torch.clamp(u, min=2.0 ** -25)
    return (-torch.log1p(-u)).to(torch.float32)


# canonical parameter blob: name, shape, fan_in
def param_spec(K, dueling):
    spec = [("conv1.W", (32, 4, 8, 8), 256), ("conv1.b", (32,), 0),
            ("conv2.W", (64, 32, 4, 4), 512), ("conv2.b", (64,), 0),
            ("conv3.W", (64, 64, 3, 3), 576), ("conv3.b", (64,), 0),
            ("fc1.W", (512, 3136), 3136), ("fc1.b", (512,), 0)]
    if dueling:
        spec += [("V.W", (1, 512), 512), ("V.b", (1,), 0)]
    spec += [("A.W", (K, 512), 512), ("A.b", (K,), 0)]
    return spec


def param_count(K, dueling):
    return sum(int(np.prod(s)) for _, s, _ in param_spec(K, dueling))


def he_uniform_params(seed, K, dueling, bias_scale=0.0):
    """Canonical fp32 blob: weights U(-b, b), b = fp32(sqrt(6/fan_in)), element e of the blob
    drawn as fp32((2*u24(seed, e) - 1) * b); biases 0 (or, for tests that need non-zero biases,
    U(-bias_scale, bias_scale) from the same stream)."""
    n = param_count(K, dueling)
    u = u24(seed, _arange(n, "cpu"))
    centred = 2.0 * u - 1.0          # exact in fp32
    out = torch.zeros(n, dtype=torch.float32)
    o = 0
    for _, shape, fan_in in param_spec(K, dueling):
        cnt = int(np.prod(shape))
        if fan_in:
            bound = torch.tensor(math.sqrt(6.0 / fan_in), dtype=torch.float32)
            out[o:o + cnt] = centred[o:o + cnt] * bound
        elif bias_scale:
            out[o:o + cnt] = centred[o:o + cnt] * torch.tensor(bias_scale, dtype=torch.float32)
        o += cnt
    return out.numpy()


def batch(seed, B, K, device="cpu"):
    """An explicit minibatch (s, s_next, a, r, done) with the recipe of the fixed-batch configs."""
    s = states(seed, B, device)
    s_next = states(seed + 1, B, device)
    a = actions(seed + 2, B, K, device)
    r = rewards(seed + 3, B, device)
    d = dones(seed + 4, B, 0.01, device)
    return s, s_next, a, r, d

"""CPU-side checks of the C-ABI boundary: the library loads, exports every symbol the header
declares, and its host-only entry points validate their arguments (no GPU call is made)."""
import ctypes as C
import os
import re

import pytest

from paper_1804_05834_amd import dqn

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(dqn.LIB_PATH):
        dqn.build()
    return dqn.lib()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "dqn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b((?:dqn|per)_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = _declared_functions()
    assert {"dqn_init", "dqn_act", "dqn_train_step", "per_sample", "per_update"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(dqn.EXPORTS) == names


def test_query_sizes_and_param_counts(lib):
    sz = dqn.query_sizes(dqn.make_config(num_actions=4, dueling=0, double_q=0))
    assert sz.param_count == 1686180 and sz.replay_frames == 0 and sz.tree == 0 and sz.shadow_bf16 == 0
    sz = dqn.query_sizes(dqn.make_config(num_actions=18, dueling=1, replay_capacity=1_000_000,
                                         max_batch=512, precision=1))
    assert sz.param_count == 1693875
    assert sz.replay_frames == 1_000_000 * 84 * 84
    assert sz.tree_leaves == 1 << 20 and sz.tree == (2 * (1 << 20) + 64) * 4
    assert sz.shadow_bf16 >= 2 * 2 * sz.param_count
    assert sz.workspace % 256 == 0 and sz.params % 256 == 0


@pytest.mark.parametrize("field,value", [("num_actions", 0), ("num_actions", 65), ("max_batch", 0),
                                         ("max_batch", 2000), ("precision", 2), ("gamma", 1.5),
                                         ("rms_eps", 0.0), ("replay_capacity", 3), ("loss_kind", 7),
                                         ("huber_delta", 0.0), ("max_act_batch", 100000)])
def test_query_sizes_rejects_bad_config(lib, field, value):
    cfg = dqn.make_config()
    setattr(cfg, field, value)
    sz = dqn.DqnSizes()
    assert lib.dqn_query_sizes(C.byref(cfg), C.byref(sz)) == dqn.ERR_INVALID_ARG
    assert len(lib.dqn_last_error(None)) > 0


def test_null_arguments_are_errors_not_crashes(lib):
    assert lib.dqn_query_sizes(None, None) == dqn.ERR_INVALID_ARG
    h = C.c_void_p()
    assert lib.dqn_init(C.byref(h), None, None, None) == dqn.ERR_INVALID_ARG
    cfg = dqn.make_config()
    bufs = dqn.DqnBuffers()          # all NULL
    assert lib.dqn_init(C.byref(h), C.byref(cfg), C.byref(bufs), None) == dqn.ERR_INVALID_ARG
    assert not h.value
    for fn, args in (("dqn_act", (None, None, 1, 0.0, 0, None, None, None)),
                     ("dqn_train_step", (None, 1, None, 0.4, 0, None, None)),
                     ("per_sample", (None, 1, 0.4, 0, None, None, None)),
                     ("per_update", (None, None, None, 1, None)),
                     ("per_fill", (None, None, 0, None)),
                     ("dqn_sync_target", (None, None)),
                     ("dqn_get_params", (None, 0, None, None))):
        assert getattr(lib, fn)(*args) == dqn.ERR_INVALID_ARG
    assert lib.dqn_destroy(None) == dqn.OK


def test_product_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_1804_05834_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip", ".cpp", "Makefile")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), (dirpath, f)


def test_fused_conv_ring_schedule_never_overwrites_an_unread_image(lib):
    """The fused conv1 + conv2 forward launch (bf16) hands conv1's output to the conv2 waves through
    a ring of LDS images with one barrier per interval.  The library replays that schedule on the
    host with the same functions its kernel loops call (which strip belongs to which sample, which
    image holds a sample, in which interval a sample is consumed, how many intervals a run takes),
    for every run length a workgroup can get: a sample is complete before it is read, it is read
    exactly once, and no strip is written into an image that still holds an unread sample."""
    for ns in range(1, 33):
        assert lib.dqn_selftest_fused_conv_schedule(ns) == 0, ns
    assert lib.dqn_selftest_fused_conv_schedule(0) != 0 and lib.dqn_selftest_fused_conv_schedule(33) != 0

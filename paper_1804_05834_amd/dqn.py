"""Thin ctypes binding of libdqn.so (include/dqn.h).

Argument marshalling only: every step of the training path runs in the HIP kernels of the
library.  torch is used to allocate device memory and to provide the stream.  There is no
CPU fallback: if the library is missing or no GPU is present, calls fail loudly.
"""
import ctypes as C
import os
import subprocess

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdqn.so")

OK, ERR_INVALID_ARG, ERR_OOM, ERR_HIP, ERR_STATE, ERR_UNSUPPORTED = 0, -1, -2, -3, -4, -5

EXPORTS = ["dqn_query_sizes", "dqn_init", "dqn_act", "dqn_train_step", "per_sample", "per_update",
           "per_fill", "dqn_replay_write", "dqn_replay_gather", "dqn_sync_target", "dqn_get_params",
           "dqn_set_params", "dqn_profile_begin", "dqn_profile_end", "dqn_last_error", "dqn_destroy",
           "dqn_replay_store", "dqn_replay_state", "dqn_schedule_default", "dqn_schedule_at", "dqn_preprocess",
           "dqn_get_activations", "dqn_act_static", "dqn_selftest_fused_conv_schedule", "dqn_replay_store_envs"]


class DqnConfig(C.Structure):
    _fields_ = [
        ("num_actions", C.c_int32), ("dueling", C.c_int32), ("double_q", C.c_int32),
        ("precision", C.c_int32), ("loss_kind", C.c_int32),
        ("huber_delta", C.c_float), ("gamma", C.c_float), ("lr", C.c_float),
        ("rms_decay", C.c_float), ("rms_eps", C.c_float),
        ("rms_centered", C.c_int32), ("max_batch", C.c_int32), ("max_act_batch", C.c_int32),
        ("per_stratified", C.c_int32),
        ("replay_capacity", C.c_int64),
        ("per_alpha", C.c_float), ("per_eps", C.c_float),
        ("seed", C.c_uint64), ("target_seed", C.c_uint64),
    ]


class DqnSizes(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("params", "opt_state", "shadow_bf16", "grads",
                                          "replay_frames", "replay_meta", "tree", "workspace")] + \
               [("param_count", C.c_int64), ("tree_leaves", C.c_int64)]


class DqnBuffers(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("online", "target", "opt_state", "shadow_bf16", "grads",
                                          "replay_frames", "replay_meta", "tree", "workspace")]


class DqnBatch(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("s", "s_next", "a", "r", "done", "w")]


class DqnStepOut(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("loss", "q_s", "q_next_online", "q_next_target", "y", "td",
                                          "a_star", "idx", "is_w", "td_abs_mean", "q_max_mean")]


class DqnSchedule(C.Structure):
    _fields_ = [("learning_start", C.c_int64), ("update_period", C.c_int64), ("target_period", C.c_int64),
                ("eps_steps", C.c_int64), ("beta_steps", C.c_int64), ("eps_start", C.c_float),
                ("eps_end", C.c_float), ("beta_start", C.c_float), ("beta_end", C.c_float)]


class DqnSchedulePoint(C.Structure):
    _fields_ = [("epsilon", C.c_float), ("beta", C.c_float), ("train", C.c_int32), ("sync_target", C.c_int32)]


class DqnError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("libdqn error %d: %s" % (code, msg))
        self.code = code


def build(force=True):
    """Compile libdqn.so for gfx950 with hipcc (cross-compiles without a GPU)."""
    args = ["make", "-C", os.path.join(_HERE, "csrc")]
    if force:
        args.insert(1, "-B")
    subprocess.check_call(args, stdout=subprocess.DEVNULL)
    return LIB_PATH


_lib = None


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libdqn.so is not built: run __graft_entry__.build() "
                               "(make -C paper_1804_05834_amd/csrc)")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, u64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_float
        sig = {
            "dqn_query_sizes": [C.POINTER(DqnConfig), C.POINTER(DqnSizes)],
            "dqn_init": [C.POINTER(vp), C.POINTER(DqnConfig), C.POINTER(DqnBuffers), vp],
            "dqn_act": [vp, vp, i32, f32, u64, vp, vp, vp],
            "dqn_act_static": [vp, vp, i32, f32, u64, vp, vp, vp],
            "dqn_train_step": [vp, i32, C.POINTER(DqnBatch), f32, u64, C.POINTER(DqnStepOut), vp],
            "per_sample": [vp, i32, f32, u64, vp, vp, vp],
            "per_update": [vp, vp, vp, i32, vp],
            "per_fill": [vp, vp, i64, vp],
            "dqn_replay_write": [vp, i64, i64, vp, vp, vp, vp, vp],
            "dqn_replay_gather": [vp, vp, i32, vp, vp, vp, vp, vp, vp],
            "dqn_replay_store": [vp, i64, vp, vp, vp, vp, vp],
            "dqn_replay_store_envs": [vp, i32, vp, vp, vp, vp, vp],
            "dqn_replay_state": [vp, C.POINTER(i64), C.POINTER(i64), C.POINTER(i64)],
            "dqn_preprocess": [vp, i64, i32, i32, vp, vp, vp],
            "dqn_schedule_default": [C.POINTER(DqnSchedule)],
            "dqn_schedule_at": [C.POINTER(DqnSchedule), i64, C.POINTER(DqnSchedulePoint)],
            "dqn_sync_target": [vp, vp],
            "dqn_get_params": [vp, i32, vp, vp],
            "dqn_set_params": [vp, i32, vp, vp],
            "dqn_get_activations": [vp, i32, i32, vp, vp],
            "dqn_selftest_fused_conv_schedule": [i32],
            "dqn_profile_begin": [vp],
            "dqn_profile_end": [vp, i32, C.POINTER(C.c_char_p), C.POINTER(i64), C.POINTER(C.c_double)],
            "dqn_destroy": [vp],
        }
        for name, argtypes in sig.items():
            fn = getattr(L, name)
            fn.argtypes = argtypes
            fn.restype = i32
        L.dqn_last_error.argtypes = [vp]
        L.dqn_last_error.restype = C.c_char_p
        _lib = L
    return _lib


def make_config(num_actions=18, dueling=1, double_q=1, precision=0, loss_kind=1, huber_delta=1.0,
                gamma=0.99, lr=2.5e-4, rms_decay=0.95, rms_eps=0.01, rms_centered=0, max_batch=32,
                max_act_batch=32, per_stratified=0, replay_capacity=0, per_alpha=0.6, per_eps=1e-6,
                seed=1804, target_seed=5834):
    return DqnConfig(num_actions, int(dueling), int(double_q), precision, loss_kind, huber_delta,
                     gamma, lr, rms_decay, rms_eps, rms_centered, max_batch, max_act_batch,
                     per_stratified, replay_capacity, per_alpha, per_eps, seed, target_seed)


def query_sizes(cfg):
    sz = DqnSizes()
    rc = lib().dqn_query_sizes(C.byref(cfg), C.byref(sz))
    if rc:
        raise DqnError(rc, lib().dqn_last_error(None).decode())
    return sz


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class Dqn:
    """One library context over torch-allocated device buffers."""

    def __init__(self, cfg, device="cuda:0"):
        if not torch.cuda.is_available():
            raise RuntimeError("libdqn needs a GPU (no CPU path exists)")
        self.cfg = cfg
        self.device = torch.device(device)
        self.sizes = query_sizes(cfg)
        sz = self.sizes
        self._bufs = {}
        b = DqnBuffers()
        for name, nbytes in (("online", sz.params), ("target", sz.params), ("opt_state", sz.opt_state),
                             ("shadow_bf16", sz.shadow_bf16), ("grads", sz.grads),
                             ("replay_frames", sz.replay_frames), ("replay_meta", sz.replay_meta),
                             ("tree", sz.tree), ("workspace", sz.workspace)):
            if nbytes:
                t = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
                assert t.data_ptr() % 256 == 0
                self._bufs[name] = t
                setattr(b, name, t.data_ptr())
        self.K = cfg.num_actions
        self.n = int(sz.param_count)
        self.L = int(sz.tree_leaves)
        h = C.c_void_p()
        with torch.cuda.device(self.device):
            rc = lib().dqn_init(C.byref(h), C.byref(cfg), C.byref(b), _stream())
        if rc:
            raise DqnError(rc, lib().dqn_last_error(None).decode())
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            torch.cuda.synchronize(self.device)
            lib().dqn_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc):
        if rc < 0:
            raise DqnError(rc, lib().dqn_last_error(self._h).decode())
        return rc

    # -- views of caller-owned state ------------------------------------------------
    @property
    def tree(self):
        """float32 view of the sum-tree heap: [0] unused, [1] root, leaves at [L, 2L)."""
        return self._bufs["tree"].view(torch.float32)[:2 * self.L]

    @property
    def max_priority(self):
        return self._bufs["tree"].view(torch.float32)[2 * self.L]

    # -- the five calls ----------------------------------------------------------------
    def act(self, obs, epsilon, draw_seed, want_q=False, static=False, out=None):
        """static: through dqn_act_static (scratch in the library's static device array).
        out: (actions, q) tensors to write into instead of new ones."""
        E = obs.shape[0]
        if out is not None:
            actions, q = out
        else:
            actions = torch.empty(E, dtype=torch.int32, device=self.device)
            q = torch.empty(E, self.K, dtype=torch.float32, device=self.device) if want_q else None
        fn = lib().dqn_act_static if static else lib().dqn_act
        self._check(fn(self._h, _ptr(obs), E, epsilon, draw_seed, _ptr(actions), _ptr(q), _stream()))
        return (actions, q) if (want_q or out is not None) else actions

    def train_step(self, B, batch=None, beta=0.4, draw_seed=0, outputs=True):
        """batch: None (replay mode) or a tuple (s, s_next, a, r, done[, w]) of device tensors.
        Returns a dict of output tensors (empty if outputs is False)."""
        out = {}
        so = None
        if outputs:
            dev = self.device
            out = dict(loss=torch.empty(1, device=dev), q_s=torch.empty(B, self.K, device=dev),
                       q_next_online=torch.empty(B, self.K, device=dev),
                       q_next_target=torch.empty(B, self.K, device=dev), y=torch.empty(B, device=dev),
                       td=torch.empty(B, device=dev),
                       a_star=torch.empty(B, dtype=torch.int32, device=dev),
                       is_w=torch.empty(B, device=dev), td_abs_mean=torch.empty(1, device=dev),
                       q_max_mean=torch.empty(1, device=dev))
            if batch is None:
                out["idx"] = torch.empty(B, dtype=torch.int32, device=dev)
            so = DqnStepOut(**{k: v.data_ptr() for k, v in out.items()})
        bb = None
        if batch is not None:
            s, sn, a, r, d = batch[:5]
            w = batch[5] if len(batch) > 5 else None
            bb = DqnBatch(s.data_ptr(), sn.data_ptr(), a.data_ptr(), r.data_ptr(), d.data_ptr(),
                          None if w is None else w.data_ptr())
        self._check(lib().dqn_train_step(self._h, B, None if bb is None else C.byref(bb), beta,
                                         draw_seed, None if so is None else C.byref(so), _stream()))
        return out

    def per_sample(self, B, beta, draw_seed):
        idx = torch.empty(B, dtype=torch.int32, device=self.device)
        w = torch.empty(B, dtype=torch.float32, device=self.device)
        self._check(lib().per_sample(self._h, B, beta, draw_seed, _ptr(idx), _ptr(w), _stream()))
        return idx, w

    def per_update(self, idx, td_abs):
        self._check(lib().per_update(self._h, _ptr(idx), _ptr(td_abs), idx.numel(), _stream()))

    # -- auxiliary ---------------------------------------------------------------------
    def per_fill(self, priorities):
        self._check(lib().per_fill(self._h, _ptr(priorities), priorities.numel(), _stream()))

    def replay_write(self, slot0, frames, a=None, r=None, done=None):
        self._check(lib().dqn_replay_write(self._h, slot0, frames.shape[0], _ptr(frames), _ptr(a),
                                           _ptr(r), _ptr(done), _stream()))

    def replay_store(self, frames, a, r, done):
        self._check(lib().dqn_replay_store(self._h, frames.shape[0], _ptr(frames), _ptr(a), _ptr(r), _ptr(done),
                                           _stream()))

    def replay_store_envs(self, frames, a, r, done):
        """One time step for each of frames.shape[0] environment streams."""
        self._check(lib().dqn_replay_store_envs(self._h, frames.shape[0], _ptr(frames), _ptr(a), _ptr(r), _ptr(done),
                                                _stream()))

    def replay_state(self):
        """(next slot, stored count, time steps stored so far)"""
        cur, st, n = C.c_int64(), C.c_int64(), C.c_int64()
        self._check(lib().dqn_replay_state(self._h, C.byref(cur), C.byref(st), C.byref(n)))
        return cur.value, st.value, n.value

    def replay_gather(self, idx):
        n, dev = idx.numel(), self.device
        s = torch.empty(n, 4, 84, 84, dtype=torch.uint8, device=dev)
        sn = torch.empty_like(s)
        a = torch.empty(n, dtype=torch.int32, device=dev)
        r = torch.empty(n, dtype=torch.float32, device=dev)
        d = torch.empty(n, dtype=torch.uint8, device=dev)
        self._check(lib().dqn_replay_gather(self._h, _ptr(idx), n, _ptr(s), _ptr(sn), _ptr(a), _ptr(r),
                                            _ptr(d), _stream()))
        return s, sn, a, r, d

    def sync_target(self):
        self._check(lib().dqn_sync_target(self._h, _stream()))

    def get_params(self, which=0):
        dst = torch.empty(self.n, dtype=torch.float32, device=self.device)
        self._check(lib().dqn_get_params(self._h, which, _ptr(dst), _stream()))
        return dst

    def set_params(self, which, src):
        src = src.to(device=self.device, dtype=torch.float32).contiguous()
        assert src.numel() == self.n
        self._check(lib().dqn_set_params(self._h, which, _ptr(src), _stream()))
        torch.cuda.current_stream().synchronize()   # src may be a temporary

    def get_activations(self, layer, n):
        """Stored outputs of layer 1..4 for the first n training rows of the last step (fp32, canonical order)."""
        shape = {1: (n, 32, 20, 20), 2: (n, 64, 9, 9), 3: (n, 64, 7, 7), 4: (n, 512)}[layer]
        dst = torch.empty(shape, dtype=torch.float32, device=self.device)
        self._check(lib().dqn_get_activations(self._h, layer, n, _ptr(dst), _stream()))
        return dst

    def profile_begin(self):
        self._check(lib().dqn_profile_begin(self._h))

    def profile_end(self, cap=64):
        names = (C.c_char_p * cap)()
        counts = (C.c_int64 * cap)()
        ms = (C.c_double * cap)()
        n = self._check(lib().dqn_profile_end(self._h, cap, names, counts, ms))
        return {names[i].decode(): (int(counts[i]), float(ms[i])) for i in range(min(n, cap))}


def schedule_default():
    sc = DqnSchedule()
    rc = lib().dqn_schedule_default(C.byref(sc))
    if rc != 0:
        raise DqnError(rc, "dqn_schedule_default")
    return sc


def schedule_at(sc, step):
    """(epsilon, beta, train, sync_target) at environment step `step` (host only)."""
    pt = DqnSchedulePoint()
    rc = lib().dqn_schedule_at(C.byref(sc), int(step), C.byref(pt))
    if rc != 0:
        raise DqnError(rc, "dqn_schedule_at")
    return pt.epsilon, pt.beta, pt.train, pt.sync_target


def preprocess(raw, grey_lut=None):
    """raw uint8 device tensor [n][H][W] -> uint8 [n][84][84] (grey levels through grey_lut if given)."""
    n, H, W = raw.shape
    out = torch.empty(n, 84, 84, dtype=torch.uint8, device=raw.device)
    rc = lib().dqn_preprocess(_ptr(raw), n, H, W, _ptr(grey_lut), _ptr(out), _stream())
    if rc != 0:
        raise DqnError(rc, (lib().dqn_last_error(None) or b"").decode())
    return out

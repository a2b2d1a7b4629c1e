"""ctypes binding of the CPU oracle (oracle/dqn_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  The product package never imports this module and
this module never imports the product package.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")


def build(force=False):
    """Compile liboracle.so with gcc (make -C oracle)."""
    src = os.path.join(_HERE, "dqn_oracle.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["make", "-B", "-C", _HERE, "liboracle.so"], stdout=subprocess.DEVNULL)
    return _LIB_PATH


class OrcConfig(C.Structure):
    _fields_ = [
        ("num_actions", C.c_int32), ("dueling", C.c_int32), ("double_q", C.c_int32),
        ("loss_kind", C.c_int32),
        ("huber_delta", C.c_double), ("gamma", C.c_double), ("lr", C.c_double),
        ("rms_decay", C.c_double), ("rms_eps", C.c_double),
        ("rms_centered", C.c_int32), ("quant", C.c_int32),
    ]


class OrcSchedule(C.Structure):
    _fields_ = [("learning_start", C.c_int64), ("update_period", C.c_int64), ("target_period", C.c_int64),
                ("eps_steps", C.c_int64), ("beta_steps", C.c_int64), ("eps_start", C.c_double),
                ("eps_end", C.c_double), ("beta_start", C.c_double), ("beta_end", C.c_double)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB_PATH)
        L.orc_mix64.restype = C.c_uint64
        L.orc_mix64.argtypes = [C.c_uint64, C.c_uint64]
        L.orc_draw_u24.restype = C.c_float
        L.orc_draw_u24.argtypes = [C.c_uint64, C.c_uint64]
        L.orc_discounted_return.restype = C.c_double
        L.orc_discounted_return.argtypes = [C.c_void_p, C.c_int64, C.c_double]
        L.orc_param_count.restype = C.c_int64
        L.orc_param_count.argtypes = [C.c_int32, C.c_int32]
        L.orc_param_offsets.restype = None
        L.orc_param_offsets.argtypes = [C.c_int32, C.c_int32, C.c_void_p]
        L.orc_forward_q.restype = C.c_int32
        L.orc_forward_q.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_int64,
                                    C.c_void_p, C.c_void_p]
        L.orc_forward_acts.restype = C.c_int32
        L.orc_forward_acts.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_int64,
                                       C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_round_bf16.restype = C.c_double
        L.orc_round_bf16.argtypes = [C.c_double]
        L.orc_target_loss.restype = C.c_int32
        L.orc_target_loss.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_double,
                                      C.c_double] + [C.c_void_p] * 12
        L.orc_rmsprop.restype = None
        L.orc_rmsprop.argtypes = [C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                  C.c_double, C.c_double, C.c_double, C.c_int32]
        L.orc_loss_grad.restype = C.c_int32
        L.orc_loss_grad.argtypes = [C.POINTER(OrcConfig), C.c_int32] + [C.c_void_p] * 16
        L.orc_train_step.restype = C.c_int32
        L.orc_train_step.argtypes = [C.POINTER(OrcConfig), C.c_int32] + [C.c_void_p] * 18
        L.orc_act.restype = C.c_int32
        L.orc_act.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_int64,
                              C.c_double, C.c_uint64, C.c_void_p, C.c_void_p]
        L.orc_tree_build.restype = None
        L.orc_tree_build.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_double, C.c_void_p]
        L.orc_per_sample.restype = C.c_int32
        L.orc_per_sample.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int32, C.c_double,
                                     C.c_uint64, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_per_sample_n.restype = C.c_int32
        L.orc_per_sample_n.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int32, C.c_double,
                                       C.c_uint64, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_tree_descend.restype = None
        L.orc_tree_descend.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.c_void_p]
        L.orc_per_sample_cumsum.restype = None
        L.orc_per_sample_cumsum.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p,
                                            C.c_int32, C.c_void_p, C.c_void_p]
        L.orc_per_update.restype = C.c_int32
        L.orc_per_update.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p,
                                     C.c_int32, C.c_double, C.c_double, C.c_void_p]
        L.orc_replay_store.restype = None
        L.orc_replay_store.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_int64, C.c_double, C.c_float]
        L.orc_schedule_at.restype = None
        L.orc_schedule_at.argtypes = [C.POINTER(OrcSchedule), C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_void_p]
        L.orc_preprocess.restype = None
        L.orc_preprocess.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_gather.restype = None
        L.orc_gather.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.c_void_p,
                                 C.c_void_p]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


# ---------------------------------------------------------------- draws
def mix64(seed, ctr):
    return int(lib().orc_mix64(C.c_uint64(seed & (2**64 - 1)), C.c_uint64(ctr & (2**64 - 1))))


def draw_u24(seed, ctr):
    return float(lib().orc_draw_u24(C.c_uint64(seed & (2**64 - 1)), C.c_uint64(ctr & (2**64 - 1))))


def discounted_return(r, gamma):
    r = _chk(r, np.float64)
    return float(lib().orc_discounted_return(_p(r), r.size, gamma))


# -------------------------------------------------------------- network
def param_count(K, dueling):
    return int(lib().orc_param_count(K, int(dueling)))


PARAM_NAMES = ["conv1.W", "conv1.b", "conv2.W", "conv2.b", "conv3.W", "conv3.b", "fc1.W", "fc1.b",
               "V.W", "V.b", "A.W", "A.b"]
PARAM_SHAPES = {"conv1.W": (32, 4, 8, 8), "conv1.b": (32,), "conv2.W": (64, 32, 4, 4),
                "conv2.b": (64,), "conv3.W": (64, 64, 3, 3), "conv3.b": (64,),
                "fc1.W": (512, 3136), "fc1.b": (512,), "V.W": (1, 512), "V.b": (1,)}


def param_slices(K, dueling):
    """name -> (offset, shape) into the canonical blob ('A.*' is the plain output layer when
    not dueling)."""
    offs = np.zeros(12, dtype=np.int64)
    lib().orc_param_offsets(K, int(dueling), _p(offs))
    out = {}
    for name, o in zip(PARAM_NAMES, offs):
        if o < 0:
            continue
        shape = PARAM_SHAPES.get(name) or ((K, 512) if name == "A.W" else (K,))
        out[name] = (int(o), shape)
    return out


def round_bf16(x):
    return float(lib().orc_round_bf16(float(x)))


def forward(params, K, dueling, states, want_hidden=False, quant=0):
    params = _chk(params, np.float32)
    states = _chk(states, np.uint8)
    n = states.shape[0]
    assert states.shape[1:] == (4, 84, 84) and params.size == param_count(K, dueling)
    q = np.zeros((n, K), dtype=np.float64)
    h = np.zeros((n, 512), dtype=np.float64) if want_hidden else None
    rc = lib().orc_forward_q(_p(params), K, int(dueling), int(quant), _p(states), n, _p(q), _p(h))
    assert rc == 0, rc
    return (q, h) if want_hidden else q


def forward_acts(params, K, dueling, states, quant=0):
    """Layer outputs after ReLU: dict a1 [n,32,20,20], a2 [n,64,9,9], a3 [n,64,7,7], h [n,512]."""
    params = _chk(params, np.float32)
    states = _chk(states, np.uint8)
    n = states.shape[0]
    assert states.shape[1:] == (4, 84, 84) and params.size == param_count(K, dueling)
    out = dict(a1=np.zeros((n, 32, 20, 20)), a2=np.zeros((n, 64, 9, 9)), a3=np.zeros((n, 64, 7, 7)),
               h=np.zeros((n, 512)))
    rc = lib().orc_forward_acts(_p(params), K, int(dueling), int(quant), _p(states), n, _p(out["a1"]),
                                _p(out["a2"]), _p(out["a3"]), _p(out["h"]))
    assert rc == 0, rc
    return out


def target_loss(q_s, q_no, q_nt, a, r, done, w=None, *, double_q, loss_kind, kappa=1.0, gamma=0.99):
    q_s = _chk(q_s, np.float64); q_no = _chk(q_no, np.float64); q_nt = _chk(q_nt, np.float64)
    B, K = q_s.shape
    a = _chk(a, np.int32); r = _chk(r, np.float32); done = _chk(done, np.uint8)
    w = None if w is None else _chk(w, np.float32)
    a_star = np.zeros(B, np.int32); y = np.zeros(B); td = np.zeros(B)
    loss = np.zeros(1); dq = np.zeros((B, K))
    rc = lib().orc_target_loss(B, K, int(double_q), int(loss_kind), kappa, gamma, _p(q_s), _p(q_no),
                               _p(q_nt), _p(a), _p(r), _p(done), _p(w), _p(a_star), _p(y), _p(td),
                               _p(loss), _p(dq))
    assert rc == 0, rc
    return dict(a_star=a_star, y=y, td=td, loss=float(loss[0]), dq=dq)


def rmsprop(theta, v, g, *, lr, rho, eps, m=None):
    """In-place on theta, v (and m if centered)."""
    assert theta.dtype == np.float32 and v.dtype == np.float32 and theta.flags.c_contiguous
    g = _chk(g, np.float64)
    lib().orc_rmsprop(theta.size, _p(theta), _p(v), _p(m), _p(g), lr, rho, eps, 0 if m is None else 1)


def make_config(K, dueling, double_q, loss_kind=1, huber_delta=1.0, gamma=0.99, lr=2.5e-4,
                rms_decay=0.95, rms_eps=0.01, rms_centered=0, quant=0):
    """quant=1: the reduced-precision mode (bf16 weights / activations, see dqn_oracle.c)."""
    return OrcConfig(K, int(dueling), int(double_q), int(loss_kind), huber_delta, gamma, lr,
                     rms_decay, rms_eps, int(rms_centered), int(quant))


def _batch(s, s_next, a, r, done, w):
    s = _chk(s, np.uint8); s_next = _chk(s_next, np.uint8)
    a = _chk(a, np.int32); r = _chk(r, np.float32); done = _chk(done, np.uint8)
    w = None if w is None else _chk(w, np.float32)
    assert s.shape == s_next.shape and s.shape[1:] == (4, 84, 84)
    return s, s_next, a, r, done, w


def loss_grad(cfg, theta, theta_target, s, s_next, a, r, done, w=None, want_grads=True):
    theta = _chk(theta, np.float32); theta_target = _chk(theta_target, np.float32)
    s, s_next, a, r, done, w = _batch(s, s_next, a, r, done, w)
    B, K = s.shape[0], cfg.num_actions
    n = param_count(K, cfg.dueling)
    assert theta.size == n and theta_target.size == n
    out = dict(q_s=np.zeros((B, K)), q_next_online=np.zeros((B, K)), q_next_target=np.zeros((B, K)),
               a_star=np.zeros(B, np.int32), y=np.zeros(B), td=np.zeros(B), loss=np.zeros(1),
               grads=np.zeros(n) if want_grads else None)
    rc = lib().orc_loss_grad(C.byref(cfg), B, _p(theta), _p(theta_target), _p(s), _p(s_next), _p(a),
                             _p(r), _p(done), _p(w), _p(out["q_s"]), _p(out["q_next_online"]),
                             _p(out["q_next_target"]), _p(out["a_star"]), _p(out["y"]),
                             _p(out["td"]), _p(out["loss"]), _p(out["grads"]))
    assert rc == 0, rc
    out["loss"] = float(out["loss"][0])
    return out


def train_step(cfg, theta, theta_target, rms_v, s, s_next, a, r, done, w=None, rms_m=None):
    """theta, rms_v (and rms_m) are updated in place (float32 arrays)."""
    assert theta.dtype == np.float32 and rms_v.dtype == np.float32
    theta_target = _chk(theta_target, np.float32)
    s, s_next, a, r, done, w = _batch(s, s_next, a, r, done, w)
    B, K = s.shape[0], cfg.num_actions
    n = param_count(K, cfg.dueling)
    out = dict(q_s=np.zeros((B, K)), q_next_online=np.zeros((B, K)), q_next_target=np.zeros((B, K)),
               a_star=np.zeros(B, np.int32), y=np.zeros(B), td=np.zeros(B), loss=np.zeros(1),
               grads=np.zeros(n))
    rc = lib().orc_train_step(C.byref(cfg), B, _p(theta), _p(theta_target), _p(rms_v), _p(rms_m),
                              _p(s), _p(s_next), _p(a), _p(r), _p(done), _p(w), _p(out["q_s"]),
                              _p(out["q_next_online"]), _p(out["q_next_target"]), _p(out["a_star"]),
                              _p(out["y"]), _p(out["td"]), _p(out["loss"]), _p(out["grads"]))
    assert rc == 0, rc
    out["loss"] = float(out["loss"][0])
    return out


def act(params, K, dueling, obs, epsilon, draw_seed, quant=0):
    params = _chk(params, np.float32); obs = _chk(obs, np.uint8)
    E = obs.shape[0]
    actions = np.zeros(E, np.int32); q = np.zeros((E, K))
    rc = lib().orc_act(_p(params), K, int(dueling), int(quant), _p(obs), E, epsilon,
                       C.c_uint64(draw_seed), _p(actions), _p(q))
    assert rc == 0, rc
    return actions, q


# ---------------------------------------------------- prioritized replay
def tree_build(raw_p, L, alpha):
    raw_p = _chk(raw_p, np.float32)
    tree = np.zeros(2 * L, dtype=np.float32)
    lib().orc_tree_build(_p(raw_p), raw_p.size, L, alpha, _p(tree))
    return tree


def per_sample(tree, size, B, beta, draw_seed, stratified=False, limit=None):
    """size: stored transitions (N of Eq.12).  limit: slots [0, limit) may hold a transition
    (default: size, one stream written from slot 0)."""
    L = tree.size // 2
    idx = np.zeros(B, np.int32); w = np.zeros(B, np.float32); z = np.zeros(B, np.float32)
    rc = lib().orc_per_sample_n(_p(tree), L, size if limit is None else limit, size, B, beta,
                                C.c_uint64(draw_seed), int(stratified), _p(idx), _p(w), _p(z))
    if rc != 0:
        raise ValueError("orc_per_sample rc=%d" % rc)
    return idx, w, z


def tree_descend(tree, z):
    z = _chk(z, np.float32)
    idx = np.zeros(z.size, np.int32)
    lib().orc_tree_descend(_p(tree), tree.size // 2, _p(z), z.size, _p(idx))
    return idx


def per_sample_cumsum(tree, size, z):
    L = tree.size // 2
    z = _chk(z, np.float32)
    idx = np.zeros(z.size, np.int32); dist = np.zeros(z.size)
    lib().orc_per_sample_cumsum(_p(tree), L, size, _p(z), z.size, _p(idx), _p(dist))
    return idx, dist


def per_update(tree, size, idx, td_abs, alpha, eps, max_p=1.0):
    """In place on tree; returns the new max priority."""
    assert tree.dtype == np.float32 and tree.flags.c_contiguous
    L = tree.size // 2
    idx = _chk(idx, np.int32); td_abs = _chk(td_abs, np.float32)
    mp = np.array([max_p], dtype=np.float32)
    rc = lib().orc_per_update(_p(tree), L, size, _p(idx), _p(td_abs), idx.size, alpha, eps, _p(mp))
    if rc != 0:
        raise ValueError("orc_per_update rc=%d" % rc)
    return float(mp[0])


class ReplayState:
    """Host-side picture of the store path: sum-tree, done flags, write cursor, stream length."""

    def __init__(self, capacity, alpha):
        self.capacity = int(capacity)
        self.alpha = float(alpha)
        L = 1
        while L < capacity:
            L *= 2
        self.L = L
        self.tree = np.zeros(2 * L, np.float32)
        self.done = np.zeros(capacity, np.uint8)
        self.cursor = np.zeros(1, np.int64)
        self.seq = np.zeros(1, np.int64)
        self.max_p = 1.0

    @property
    def stored(self):
        return int(min(self.seq[0], self.capacity))

    def store(self, done_new):
        done_new = _chk(done_new, np.uint8)
        lib().orc_replay_store(_p(self.tree), self.L, self.capacity, _p(self.cursor), _p(self.seq),
                               _p(self.done), _p(done_new), done_new.size, self.alpha,
                               C.c_float(self.max_p))


def schedule_at(t, learning_start=50000, update_period=4, target_period=30000, eps_steps=5000000,
                beta_steps=100000000, eps_start=1.0, eps_end=0.1, beta_start=0.4, beta_end=1.0):
    """(epsilon, beta, train, sync_target) at environment step t (Table 1 defaults)."""
    sc = OrcSchedule(learning_start, update_period, target_period, eps_steps, beta_steps,
                     eps_start, eps_end, beta_start, beta_end)
    e = np.zeros(1); b = np.zeros(1); tr = np.zeros(1, np.int32); sy = np.zeros(1, np.int32)
    lib().orc_schedule_at(C.byref(sc), int(t), _p(e), _p(b), _p(tr), _p(sy))
    return float(e[0]), float(b[0]), int(tr[0]), int(sy[0])


def preprocess(raw, lut=None):
    """raw uint8 [n][H][W] -> (uint8 [n][84][84], unrounded float64 values)."""
    raw = _chk(raw, np.uint8)
    n, H, W = raw.shape
    if lut is not None:
        lut = _chk(lut, np.float32)
        assert lut.size == 256
    out = np.zeros((n, 84, 84), np.uint8); val = np.zeros((n, 84, 84), np.float64)
    lib().orc_preprocess(_p(raw), n, H, W, None if lut is None else _p(lut), _p(out), _p(val))
    return out, val


def gather(frames, idx):
    frames = _chk(frames, np.uint8)
    idx = _chk(idx, np.int32)
    cap = frames.shape[0]
    B = idx.size
    s = np.zeros((B, 4, 84, 84), np.uint8); sn = np.zeros((B, 4, 84, 84), np.uint8)
    lib().orc_gather(_p(frames), cap, _p(idx), B, _p(s), _p(sn))
    return s, sn

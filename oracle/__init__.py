"""ctypes access to the CPU oracle (TEST INFRASTRUCTURE ONLY).

Only tests, the smoke check and the benchmark's cpu_baseline leg import this
package.  It knows nothing about the GPU library and shares no code with it.
The arithmetic lives in replay_oracle.c; this file only marshals numpy arrays.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libreplay_oracle.so")

F32, BF16, U8 = 0, 1, 2
PAIR, CHAIN = 0, 1
HUBER, MSE = 0, 1
SGD, ADAM = 0, 1

_NP_STATE = {F32: np.float32, BF16: np.uint16, U8: np.uint8}


def build(force=True):
    """Compile replay_oracle.c with gcc into libreplay_oracle.so."""
    if not force and os.path.exists(LIB_PATH):
        return LIB_PATH
    cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-Wall", "-Wextra", "-o", LIB_PATH, os.path.join(_HERE, "replay_oracle.c"), "-lm"]
    subprocess.run(cmd, check=True)
    return LIB_PATH


class TrainCfg(C.Structure):
    _fields_ = [("state_dim", C.c_uint32), ("hidden", C.c_uint32), ("num_actions", C.c_uint32),
                ("batch", C.c_uint32), ("loss", C.c_uint32), ("opt", C.c_uint32),
                ("bf16", C.c_uint32), ("dueling", C.c_uint32), ("lr", C.c_double),
                ("gamma", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double),
                ("eps", C.c_double), ("hidden2", C.c_uint32), ("pad_", C.c_uint32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            build()
        L = C.CDLL(LIB_PATH)
        vp, u32, u64, i32p = C.c_void_p, C.c_uint32, C.c_uint64, C.c_void_p
        L.oracle_set_threads.argtypes = [C.c_int]
        L.oracle_get_threads.restype = C.c_int
        L.oracle_philox4x32_10.argtypes = [vp, vp, vp]
        L.oracle_uniform_index.argtypes = [u64, u64, u32, u64]
        L.oracle_uniform_index.restype = u32
        L.oracle_uniform_indices.argtypes = [u64, u64, u64, u32, u64, vp]
        L.oracle_distinct_index.argtypes = [u64, u64, u32, u64]
        L.oracle_distinct_index.restype = u32
        L.oracle_ring_sample_mode.argtypes = [vp, u64, u64, u32, C.c_int, vp]
        L.oracle_ring_create.argtypes = [u64, u32, u32, u32, u64]
        L.oracle_ring_create.restype = vp
        L.oracle_ring_destroy.argtypes = [vp]
        L.oracle_ring_append.argtypes = [vp, u64, vp, vp, i32p, vp, vp]
        L.oracle_ring_state.argtypes = [vp, vp, vp, vp]
        L.oracle_ring_read.argtypes = [vp, u64, u64, vp, vp, vp, vp, vp]
        L.oracle_ring_sample.argtypes = [vp, u64, u64, u32, vp]
        L.oracle_ring_gather.argtypes = [vp, vp, u32, vp, vp, vp, vp, vp]
        L.oracle_round_bf16.argtypes = [C.c_double]
        L.oracle_round_bf16.restype = C.c_double
        L.oracle_bf16_bits.argtypes = [C.c_float]
        L.oracle_bf16_bits.restype = C.c_uint16
        L.oracle_param_count.argtypes = [u32, u32, u32]
        L.oracle_param_count.restype = C.c_size_t
        L.oracle_param_count2.argtypes = [u32, u32, u32, u32]
        L.oracle_param_count2.restype = C.c_size_t
        L.oracle_mlp_forward.argtypes = [vp, vp, vp, u32, vp, vp, vp]
        L.oracle_loss_fixed_targets.argtypes = [vp, vp, vp, vp, vp]
        L.oracle_loss_fixed_targets.restype = C.c_double
        L.oracle_train_step.argtypes = [vp] * 16
        L.oracle_opt_apply.argtypes = [vp, C.c_size_t, vp, vp, vp, vp, vp]
        L.oracle_train_step_target.argtypes = [vp] * 17
        _lib = L
    return _lib


def _p(arr):
    return None if arr is None else arr.ctypes.data_as(C.c_void_p)


def _c(arr, dtype):
    return np.ascontiguousarray(arr, dtype=dtype)


def set_threads(n):
    lib().oracle_set_threads(int(n))


def get_threads():
    return int(lib().oracle_get_threads())


def philox4x32_10(ctr, key):
    ctr = _c(ctr, np.uint32)
    key = _c(key, np.uint32)
    out = np.empty(4, np.uint32)
    lib().oracle_philox4x32_10(_p(ctr), _p(key), _p(out))
    return out


def uniform_index(seed, step, i, n_choices):
    return int(lib().oracle_uniform_index(seed, step, i, n_choices))


def distinct_index(seed, step, i, n_choices):
    return int(lib().oracle_distinct_index(seed, step, i, n_choices))


def distinct_indices(seed, step, batch, n_choices):
    """The first `batch` members of the step's sample without duplicates."""
    f = lib().oracle_distinct_index
    return np.array([f(seed, step, i, n_choices) for i in range(batch)], np.uint32)


def uniform_indices(seed, step0, nsteps, batch, n_choices):
    out = np.empty((nsteps, batch), np.uint32)
    lib().oracle_uniform_indices(seed, step0, nsteps, batch, n_choices, _p(out))
    return out


def round_bf16(x):
    return float(lib().oracle_round_bf16(float(x)))


def bf16_bits(x):
    return int(lib().oracle_bf16_bits(float(x)))


class Ring:
    """The FIFO replay of the paper's Methods section, on the host."""

    def __init__(self, capacity, state_dim, state_dtype=F32, layout=PAIR, burn_in=0):
        self.capacity, self.state_dim = int(capacity), int(state_dim)
        self.state_dtype, self.layout, self.burn_in = state_dtype, layout, int(burn_in)
        self._h = lib().oracle_ring_create(self.capacity, self.state_dim, state_dtype, layout,
                                           self.burn_in)
        if not self._h:
            raise ValueError("oracle_ring_create rejected the configuration")
        self._destroy = lib().oracle_ring_destroy

    def __del__(self):
        if getattr(self, "_h", None):
            self._destroy(self._h)
            self._h = None

    @property
    def np_state(self):
        return _NP_STATE[self.state_dtype]

    @property
    def np_out(self):
        return np.float32 if self.state_dtype == U8 else self.np_state

    def append(self, s, s_next, a, r, term):
        a = _c(a, np.int32)
        n = a.shape[0]
        s = _c(s, self.np_state)
        s_next = None if s_next is None else _c(s_next, self.np_state)
        rc = lib().oracle_ring_append(self._h, n, _p(s), _p(s_next), _p(a), _p(_c(r, np.float32)),
                                      _p(_c(term, np.uint8)))
        if rc != 0:
            raise ValueError("oracle_ring_append rejected the arguments")

    def state(self):
        h, s, t = C.c_uint64(), C.c_uint64(), C.c_uint64()
        lib().oracle_ring_state(self._h, C.byref(h), C.byref(s), C.byref(t))
        return h.value, s.value, t.value

    def read(self, first_slot, n):
        s = np.empty((n, self.state_dim), self.np_state)
        sn = np.empty((n, self.state_dim), self.np_state) if self.layout == PAIR else None
        a = np.empty(n, np.int32)
        r = np.empty(n, np.float32)
        term = np.empty(n, np.uint8)
        rc = lib().oracle_ring_read(self._h, first_slot, n, _p(s), _p(sn), _p(a), _p(r), _p(term))
        if rc != 0:
            raise ValueError("oracle_ring_read rejected the arguments")
        return s, sn, a, r, term

    def sample(self, seed, step, batch, distinct=False):
        """Slot numbers of one sample, or None while sampling is refused."""
        idx = np.empty(batch, np.uint32)
        rc = lib().oracle_ring_sample_mode(self._h, seed, step, batch, int(distinct), _p(idx))
        if rc < 0:
            raise ValueError("oracle_ring_sample rejected the arguments")
        return None if rc == 1 else idx

    def gather(self, idx):
        idx = _c(idx, np.uint32)
        b = idx.shape[0]
        s = np.empty((b, self.state_dim), self.np_out)
        sn = np.empty((b, self.state_dim), self.np_out)
        a = np.empty(b, np.int32)
        r = np.empty(b, np.float32)
        term = np.empty(b, np.uint8)
        rc = lib().oracle_ring_gather(self._h, _p(idx), b, _p(s), _p(sn), _p(a), _p(r), _p(term))
        if rc != 0:
            raise ValueError("oracle_ring_gather rejected the arguments")
        return s, sn, a, r, term


def make_cfg(state_dim, hidden, num_actions, batch, loss=HUBER, opt=SGD, bf16=0, lr=1e-3,
             gamma=0.99, beta1=0.9, beta2=0.999, eps=1e-8, dueling=0, hidden2=0):
    return TrainCfg(state_dim, hidden, num_actions, batch, loss, opt, bf16, dueling, lr, gamma, beta1,
                    beta2, eps, hidden2, 0)


def cfg_hidden2(cfg):
    return cfg.hidden2 or cfg.hidden


def cfg_param_count(cfg):
    """Parameters of the network a configuration describes (the dueling head has one more output)."""
    return param_count(cfg.state_dim, cfg.hidden, cfg.num_actions + (1 if cfg.dueling else 0),
                       cfg_hidden2(cfg))


def param_count(D, H, A, H2=None):
    return int(lib().oracle_param_count2(D, H, H if H2 is None else H2, A))


def mlp_forward(cfg, params, X, want_hidden=False):
    params = _c(params, np.float64)
    X = _c(X, np.float64)
    n = X.shape[0]
    Q = np.empty((n, cfg.num_actions), np.float64)
    h1 = np.empty((n, cfg.hidden), np.float64) if want_hidden else None
    h2 = np.empty((n, cfg_hidden2(cfg)), np.float64) if want_hidden else None
    lib().oracle_mlp_forward(C.byref(cfg), _p(params), _p(X), n, _p(h1), _p(h2), _p(Q))
    return (Q, h1, h2) if want_hidden else Q


def loss_fixed_targets(cfg, params, S, a, y):
    return float(lib().oracle_loss_fixed_targets(
        C.byref(cfg), _p(_c(params, np.float64)), _p(_c(S, np.float64)), _p(_c(a, np.int32)),
        _p(_c(y, np.float64))))


def target_after_step(target, new_params, updates_applied, sync_every):
    """The frozen target network after a train step (Deep Q-Network Model: overwritten with the
    trained weights every `sync_every` steps): the new weights when the number of updates applied
    so far is a multiple of sync_every, else unchanged."""
    if sync_every and updates_applied % sync_every == 0:
        return np.array(new_params, np.float64)
    return np.array(target, np.float64)


def opt_apply(cfg, params, m, v, t, grads):
    """The parameter update alone from a given gradient, on copies; returns (params, m, v, t) in
    float64 (m, v None and t unchanged for SGD)."""
    p = np.array(params, np.float64, order="C")
    g = _c(grads, np.float64)
    assert g.shape == p.shape
    tt = C.c_uint64(int(t))
    if cfg.opt == SGD:
        lib().oracle_opt_apply(C.byref(cfg), p.shape[0], _p(p), None, None, C.byref(tt), _p(g))
        return p, None, None, tt.value
    mm = np.array(m, np.float64, order="C")
    vv = np.array(v, np.float64, order="C")
    assert mm.shape == p.shape and vv.shape == p.shape
    lib().oracle_opt_apply(C.byref(cfg), p.shape[0], _p(p), _p(mm), _p(vv), C.byref(tt), _p(g))
    return p, mm, vv, tt.value


class StepResult:
    __slots__ = ("params", "m", "v", "t", "Q", "Qn", "y", "delta", "loss", "grads")


def train_step(cfg, params, m, v, t, S, S_next, a, r, term, target=None):
    """One step on copies of (params, m, v, t); returns a StepResult in float64.
    target: parameters of the frozen target network used for Q(s', .) (None = the trained one)."""
    out = StepResult()
    out.params = np.array(params, np.float64, order="C")
    n = out.params.shape[0]
    out.m = np.zeros(n) if m is None else np.array(m, np.float64, order="C")
    out.v = np.zeros(n) if v is None else np.array(v, np.float64, order="C")
    tt = C.c_uint64(int(t))
    B, A = cfg.batch, cfg.num_actions
    out.Q = np.empty((B, A))
    out.Qn = np.empty((B, A))
    out.y = np.empty(B)
    out.delta = np.empty(B)
    out.grads = np.empty(n)
    loss = C.c_double()
    S = _c(S, np.float64)
    S_next = _c(S_next, np.float64)
    a = _c(a, np.int32)
    r = _c(r, np.float64)
    term = _c(term, np.uint8)
    assert S.shape == (B, cfg.state_dim) and S_next.shape == S.shape
    assert a.shape == (B,) and r.shape == (B,) and term.shape == (B,)
    assert n == cfg_param_count(cfg)
    tgt = None if target is None else _c(target, np.float64)
    assert tgt is None or tgt.shape == (n,)
    lib().oracle_train_step_target(C.byref(cfg), _p(out.params), _p(tgt), _p(out.m), _p(out.v),
                                   C.byref(tt), _p(S), _p(S_next), _p(a), _p(r), _p(term),
                                   _p(out.Q), _p(out.Qn), _p(out.y), _p(out.delta), C.byref(loss),
                                   _p(out.grads))
    out.t = tt.value
    out.loss = loss.value
    return out

"""Thin ctypes binding of libingpu_replay.so (include/ingpu_replay.h).

Argument marshalling only: every step of the replay and of the train step runs
in the library's HIP kernels.  PyTorch is used here for device memory and
streams, nothing else.  If the library is missing or cannot be loaded this
module raises; there is no fallback path.
"""
import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libingpu_replay.so")

RP_OK, RP_SKIPPED_BURN_IN = 0, 1
RP_EINVAL, RP_ENOMEM, RP_EHIP, RP_ESTATE = -1, -2, -3, -4
RP_F32, RP_BF16, RP_U8 = 0, 1, 2
RP_PAIR, RP_CHAIN = 0, 1
RP_HUBER, RP_MSE = 0, 1
RP_SGD, RP_ADAM = 0, 1
RP_TRAIN_GRAPH, RP_TRAIN_LAYERED = 1, 2
RP_WITH_REPLACEMENT, RP_DISTINCT = 0, 1
RP_HEAD_PLAIN, RP_HEAD_DUELING = 0, 1

_NP_STATE = {RP_F32: np.float32, RP_BF16: np.uint16, RP_U8: np.uint8}
_TORCH_OUT = {RP_F32: torch.float32, RP_BF16: torch.bfloat16, RP_U8: torch.float32}


class ReplayError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"ingpu_replay status {status}: {message}")
        self.status = status


class ReplayConfig(C.Structure):
    _fields_ = [("capacity", C.c_uint64), ("state_dim", C.c_uint32), ("state_dtype", C.c_uint32),
                ("layout", C.c_uint32), ("max_append", C.c_uint32), ("burn_in", C.c_uint64),
                ("seed", C.c_uint64), ("sampling", C.c_uint32), ("reserved", C.c_uint32)]


class TrainConfig(C.Structure):
    _fields_ = [("state_dim", C.c_uint32), ("hidden", C.c_uint32), ("num_actions", C.c_uint32),
                ("batch", C.c_uint32), ("param_dtype", C.c_uint32), ("loss", C.c_uint32),
                ("opt", C.c_uint32), ("appends_per_step", C.c_uint32), ("lr", C.c_float),
                ("gamma", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("flags", C.c_uint32), ("target_sync", C.c_uint32),
                ("head", C.c_uint32), ("hidden2", C.c_uint32)]


# every symbol include/ingpu_replay.h declares: name -> (restype, argtypes)
_vp, _u32, _u64, _int = C.c_void_p, C.c_uint32, C.c_uint64, C.c_int
SYMBOLS = {
    "replay_storage_bytes": (C.c_size_t, [_vp]),
    "replay_row_bytes": (C.c_size_t, [_vp]),
    "replay_create": (_int, [_vp, _vp, C.c_size_t, _vp]),
    "replay_destroy": (_int, [_vp]),
    "replay_append": (_int, [_vp, _u64, _vp, _vp, _vp, _vp, _vp, _int, _vp]),
    "replay_sample_gather": (_int, [_vp, _u64, _u32, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "replay_sample_gather_static": (_int, [_vp, _u64, _u32, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "replay_get_state": (_int, [_vp, _vp, _vp, _vp]),
    "replay_read_rows": (_int, [_vp, _u64, _u64, _vp, _vp, _vp, _vp, _vp]),
    "train_param_count": (C.c_size_t, [_vp]),
    "train_workspace_bytes": (C.c_size_t, [_vp]),
    "train_create": (_int, [_vp, _vp, _vp, C.c_size_t, _vp, _vp]),
    "train_destroy": (_int, [_vp]),
    "train_step": (_int, [_vp, _vp, _vp, _vp, _vp, _vp, _int, _vp]),
    "train_steps": (_int, [_vp, _u64, _vp, _vp, _vp, _vp, _vp, _int, _vp, _vp]),
    "train_step_batch": (_int, [_vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "inram_device_bytes": (C.c_size_t, [_u32, _u32]),
    "inram_create": (_int, [_u64, _u32, _u64, _u64, _u32, _vp, C.c_size_t, _vp]),
    "inram_destroy": (_int, [_vp]),
    "inram_append": (_int, [_vp, _u64, _vp, _vp, _vp, _vp, _vp]),
    "inram_train_step": (_int, [_vp, _vp, _vp]),
    "inram_train_steps": (_int, [_vp, _vp, _u64, _u32, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "inram_get_state": (_int, [_vp, _vp, _vp, _vp, _vp]),
    "train_get_params": (_int, [_vp, _vp]),
    "train_get_grads": (_int, [_vp, _vp]),
    "train_get_opt_state": (_int, [_vp, _vp, _vp, _vp, _vp]),
    "train_set_state": (_int, [_vp, _vp, _vp, _vp, _u64, _u64]),
    "train_get_last": (_int, [_vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "train_get_target": (_int, [_vp, _vp]),
    "train_set_target": (_int, [_vp, _vp]),
    "train_kernels_per_step": (_int, [_vp, _vp]),
    "train_set_handoff_wait": (_int, [_vp, _u64, _int]),
    "train_get_target_source": (_int, [_vp, _vp]),
    "rp_last_error": (C.c_char_p, []),
    "rp_version": (C.c_char_p, []),
}

_lib = None


def lib():
    """Load the HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_1801_03138_amd.build` "
                              "(or __graft_entry__.build()) first; there is no fallback path")
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in SYMBOLS.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def _check(status):
    if status < 0:
        raise ReplayError(status, lib().rp_last_error().decode())
    return status


def _stream_ptr(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _dev(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _host(arr):
    return None if arr is None else arr.ctypes.data_as(C.c_void_p)


# torch dtypes a device array of each state type may have (bf16 bits also travel as 16-bit ints)
_TORCH_STATE = {RP_F32: (torch.float32,), RP_BF16: (torch.bfloat16, torch.int16, torch.uint16),
                RP_U8: (torch.uint8,)}
_TORCH_I32 = (torch.int32, torch.uint32)


def check_device_array(t, dtypes, numel, device, what):
    """The C interface carries no lengths: a device array handed to the library must be a
    contiguous tensor on the replay's device with the expected element type and count, or the
    kernels would read or write out of bounds.  Raises ValueError otherwise; returns t."""
    if not isinstance(t, torch.Tensor):
        raise ValueError(f"{what}: expected a torch tensor on {device}, got {type(t).__name__}")
    dev = torch.device(device)
    if t.device.type != dev.type or (dev.index is not None and t.device.index != dev.index):
        raise ValueError(f"{what}: tensor is on {t.device}, the replay is on {dev}")
    if t.dtype not in dtypes:
        raise ValueError(f"{what}: dtype {t.dtype}, expected one of {tuple(str(d) for d in dtypes)}")
    if not t.is_contiguous():
        raise ValueError(f"{what}: tensor is not contiguous")
    if t.numel() != numel:
        raise ValueError(f"{what}: {t.numel()} elements, expected {numel}")
    return t


def check_device_experiences(cfg, device, n, s, s_next, a, r, term, what):
    """n experiences as device arrays, structure of arrays (s_next is ignored for RP_CHAIN)."""
    D, st = cfg.state_dim, _TORCH_STATE[cfg.state_dtype]
    check_device_array(s, st, n * D, device, what + ": s")
    if cfg.layout == RP_PAIR:
        check_device_array(s_next, st, n * D, device, what + ": s_next")
    check_device_array(a, _TORCH_I32, n, device, what + ": a")
    check_device_array(r, (torch.float32,), n, device, what + ": r")
    check_device_array(term, (torch.uint8, torch.bool), n, device, what + ": term")


def check_host_experiences(cfg, n, s, s_next, a, r, term, what):
    """n experiences as host arrays (already converted to the field types): element counts."""
    D = cfg.state_dim
    fields = [("s", s, n * D), ("a", a, n), ("r", r, n), ("term", term, n)]
    if cfg.layout == RP_PAIR:
        fields.append(("s_next", s_next, n * D))
    for name, arr, want in fields:
        if arr is None or arr.size != want:
            raise ValueError(f"{what}: {name} has {None if arr is None else arr.size} elements, expected {want}")


def check_batch_out(cfg, device, batch, out, what):
    """The six output tensors of sample_gather for `batch` experiences."""
    if len(out) != 6:
        raise ValueError(f"{what}: expected (s, s_next, a, r, term, idx)")
    s, s_next, a, r, term, idx = out
    D, dt = cfg.state_dim, _TORCH_OUT[cfg.state_dtype]
    st = (dt,) if dt != torch.bfloat16 else _TORCH_STATE[RP_BF16]
    check_device_array(s, st, batch * D, device, what + ": s")
    check_device_array(s_next, st, batch * D, device, what + ": s_next")
    check_device_array(a, _TORCH_I32, batch, device, what + ": a")
    check_device_array(r, (torch.float32,), batch, device, what + ": r")
    check_device_array(term, (torch.uint8,), batch, device, what + ": term")
    if idx is not None:
        check_device_array(idx, _TORCH_I32, batch, device, what + ": idx")


def _alloc_bytes(nbytes, device):
    # torch's caching allocator hands out blocks aligned to at least 256 bytes
    buf = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
    assert buf.data_ptr() % 256 == 0
    return buf


def storage_bytes(cfg):
    return int(lib().replay_storage_bytes(C.byref(cfg)))


def row_bytes(cfg):
    return int(lib().replay_row_bytes(C.byref(cfg)))


class Replay:
    """The experience replay of the paper's Methods section, resident in HBM."""

    def __init__(self, capacity, state_dim, state_dtype=RP_F32, layout=RP_PAIR, burn_in=0, seed=0,
                 max_append=4096, device="cuda:0", distinct=False):
        self.cfg = ReplayConfig(capacity, state_dim, state_dtype, layout, max_append, burn_in, seed,
                                RP_DISTINCT if distinct else RP_WITH_REPLACEMENT, 0)
        nbytes = storage_bytes(self.cfg)
        if nbytes == 0:
            raise ReplayError(RP_EINVAL, "invalid replay configuration")
        self.device = torch.device(device)
        self.storage = _alloc_bytes(nbytes, self.device)
        h = C.c_void_p()
        with torch.cuda.device(self.device):
            _check(lib().replay_create(C.byref(self.cfg), _dev(self.storage), nbytes, C.byref(h)))
        self._h = h
        self._destroy = lib().replay_destroy

    def close(self):
        if getattr(self, "_h", None):
            self._destroy(self._h)
            self._h = None

    __del__ = close

    @property
    def np_state(self):
        return _NP_STATE[self.cfg.state_dtype]

    def append(self, s, s_next, a, r, term, stream=None):
        """Append experiences given as numpy arrays (host) or torch CUDA tensors (device)."""
        on_dev = isinstance(a, torch.Tensor)
        n = len(a)
        if on_dev:
            check_device_experiences(self.cfg, self.device, n, s, s_next, a, r, term, "append")
            if self.cfg.layout != RP_PAIR:
                s_next = None
            args = [_dev(s), _dev(s_next), _dev(a), _dev(r), _dev(term)]
            keep = None
        else:
            keep = [np.ascontiguousarray(s, self.np_state),
                    None if s_next is None else np.ascontiguousarray(s_next, self.np_state),
                    np.ascontiguousarray(a, np.int32), np.ascontiguousarray(r, np.float32),
                    np.ascontiguousarray(term, np.uint8)]
            check_host_experiences(self.cfg, n, *keep, "append")
            args = [_host(x) for x in keep]
        return _check(lib().replay_append(self._h, n, *args, 1 if on_dev else 0,
                                          _stream_ptr(stream)))

    def alloc_batch(self, batch):
        """Output tensors for sample_gather: (s, s_next, a, r, term, idx)."""
        D, dt, dev = self.cfg.state_dim, _TORCH_OUT[self.cfg.state_dtype], self.device
        return (torch.empty((batch, D), dtype=dt, device=dev),
                torch.empty((batch, D), dtype=dt, device=dev),
                torch.empty(batch, dtype=torch.int32, device=dev),
                torch.empty(batch, dtype=torch.float32, device=dev),
                torch.empty(batch, dtype=torch.uint8, device=dev),
                torch.empty(batch, dtype=torch.int32, device=dev))

    def sample_gather(self, step, batch, out=None, stream=None):
        """Returns (status, (s, s_next, a, r, term, idx)); status 1 = refused during burn-in."""
        out = self.alloc_batch(batch) if out is None else out
        check_batch_out(self.cfg, self.device, batch, out, "sample_gather")
        st = _check(lib().replay_sample_gather(self._h, step, batch, *[_dev(t) for t in out],
                                               _stream_ptr(stream)))
        return st, out

    def sample_gather_static(self, step, batch, out, stream=None):
        """sample_gather through the entry point that allocates nothing (its scratch is a fixed
        array inside the library); `out` must be given, e.g. from alloc_batch."""
        check_batch_out(self.cfg, self.device, batch, out, "sample_gather_static")
        st = _check(lib().replay_sample_gather_static(self._h, step, batch, *[_dev(t) for t in out],
                                                      _stream_ptr(stream)))
        return st, out

    def state(self):
        h, s, t = C.c_uint64(), C.c_uint64(), C.c_uint64()
        _check(lib().replay_get_state(self._h, C.byref(h), C.byref(s), C.byref(t)))
        return h.value, s.value, t.value

    def read_rows(self, first_slot, n):
        D = self.cfg.state_dim
        s = np.empty((n, D), self.np_state)
        sn = np.empty((n, D), self.np_state) if self.cfg.layout == RP_PAIR else None
        a, r, term = np.empty(n, np.int32), np.empty(n, np.float32), np.empty(n, np.uint8)
        _check(lib().replay_read_rows(self._h, first_slot, n, _host(s), _host(sn), _host(a),
                                      _host(r), _host(term)))
        return s, sn, a, r, term


class Trainer:
    """The Q-learning train step on top of a Replay; all state lives in HBM."""

    def __init__(self, replay, hidden, num_actions, batch, param_dtype=RP_F32, loss=RP_HUBER,
                 opt=RP_ADAM, appends_per_step=1, lr=1e-4, gamma=0.99, beta1=0.9, beta2=0.999,
                 eps=1e-8, use_graph=True, layered=False, target_sync=0, dueling=False, init_params=None,
                 hidden2=0):
        self.replay = replay
        self.cfg = TrainConfig(replay.cfg.state_dim, hidden, num_actions, batch, param_dtype, loss,
                               opt, appends_per_step, lr, gamma, beta1, beta2, eps,
                               (RP_TRAIN_GRAPH if use_graph else 0) | (RP_TRAIN_LAYERED if layered else 0),
                               target_sync, RP_HEAD_DUELING if dueling else RP_HEAD_PLAIN, hidden2)
        nbytes = int(lib().train_workspace_bytes(C.byref(self.cfg)))
        if nbytes == 0:
            raise ReplayError(RP_EINVAL, "invalid train configuration")
        self.n_params = int(lib().train_param_count(C.byref(self.cfg)))
        init = np.ascontiguousarray(init_params, np.float32)
        if init.shape != (self.n_params,):
            raise ValueError(f"init_params must have {self.n_params} entries")
        self.workspace = _alloc_bytes(nbytes, replay.device)
        h = C.c_void_p()
        with torch.cuda.device(replay.device):
            _check(lib().train_create(C.byref(self.cfg), replay._h, _dev(self.workspace), nbytes,
                                      _host(init), C.byref(h)))
        self._h = h
        self._destroy = lib().train_destroy

    def close(self):
        if getattr(self, "_h", None):
            self._destroy(self._h)
            self._h = None

    __del__ = close

    def _payload(self, n, s, s_next, a, r, term, what):
        """Marshal n new experiences (numpy arrays or CUDA tensors; none when n = 0): returns
        (pointer arguments, src_is_device, arrays to keep alive)."""
        if n == 0:
            return [None] * 5, 0, None
        if a is None:
            raise ValueError(f"{what}: this trainer appends {self.cfg.appends_per_step} experiences per "
                             "step; the arrays are missing")
        rc = self.replay.cfg
        if isinstance(a, torch.Tensor):
            check_device_experiences(rc, self.replay.device, n, s, s_next, a, r, term, what)
            return [_dev(s), _dev(s_next), _dev(a), _dev(r), _dev(term)], 1, None
        st = self.replay.np_state
        keep = [np.ascontiguousarray(s, st), np.ascontiguousarray(s_next, st),
                np.ascontiguousarray(a, np.int32), np.ascontiguousarray(r, np.float32),
                np.ascontiguousarray(term, np.uint8)]
        # the library reads exactly n experiences; longer arrays are allowed (steps() slices them)
        for name, arr, want in (("s", keep[0], n * rc.state_dim), ("s_next", keep[1], n * rc.state_dim),
                                ("a", keep[2], n), ("r", keep[3], n), ("term", keep[4], n)):
            if arr.size < want:
                raise ValueError(f"{what}: {name} has {arr.size} elements, needs {want}")
        return [_host(x) for x in keep], 0, keep

    def step(self, s=None, s_next=None, a=None, r=None, term=None, stream=None):
        """One train step; the arrays are the appends_per_step new experiences (numpy or CUDA tensors)."""
        args, on_dev, keep = self._payload(self.cfg.appends_per_step, s, s_next, a, r, term, "step")
        return _check(lib().train_step(self._h, *args, on_dev, _stream_ptr(stream)))

    def steps(self, count, s=None, s_next=None, a=None, r=None, term=None, stream=None):
        """`count` train steps in one call; the arrays hold count*appends_per_step experiences.
        Returns the number of steps that trained (the others only appended, during burn-in)."""
        args, on_dev, keep = self._payload(int(count) * self.cfg.appends_per_step, s, s_next, a, r,
                                           term, "steps")
        done = C.c_uint64()
        _check(lib().train_steps(self._h, count, *args, on_dev, _stream_ptr(stream),
                                 C.byref(done)))
        return done.value

    def step_batch(self, s, s_next, a, r, term, stream=None):
        """One train step on the given batch (torch CUDA tensors, as sample_gather returns them)."""
        check_device_experiences(self.replay.cfg, self.replay.device, self.cfg.batch, s, s_next, a,
                                 r, term, "step_batch")
        return _check(lib().train_step_batch(self._h, _dev(s), _dev(s_next), _dev(a), _dev(r),
                                             _dev(term), _stream_ptr(stream)))

    def params(self):
        p = np.empty(self.n_params, np.float32)
        _check(lib().train_get_params(self._h, _host(p)))
        return p

    def target(self):
        p = np.empty(self.n_params, np.float32)
        _check(lib().train_get_target(self._h, _host(p)))
        return p

    def set_target(self, params):
        p = np.ascontiguousarray(params, np.float32)
        _check(lib().train_set_target(self._h, _host(p)))

    def grads(self):
        g = np.empty(self.n_params, np.float32)
        _check(lib().train_get_grads(self._h, _host(g)))
        return g

    def opt_state(self):
        m, v = np.empty(self.n_params, np.float32), np.empty(self.n_params, np.float32)
        t, step = C.c_uint64(), C.c_uint64()
        _check(lib().train_get_opt_state(self._h, _host(m), _host(v), C.byref(t), C.byref(step)))
        return m, v, t.value, step.value

    def set_state(self, params, m, v, t, step):
        p = np.ascontiguousarray(params, np.float32)
        m = None if m is None else np.ascontiguousarray(m, np.float32)
        v = None if v is None else np.ascontiguousarray(v, np.float32)
        _check(lib().train_set_state(self._h, _host(p), _host(m), _host(v), int(t), int(step)))

    def last(self):
        B, A = self.cfg.batch, self.cfg.num_actions
        q, qn = np.empty((B, A), np.float32), np.empty((B, A), np.float32)
        y, d = np.empty(B, np.float32), np.empty(B, np.float32)
        loss, idx = np.empty(1, np.float32), np.empty(B, np.uint32)
        _check(lib().train_get_last(self._h, _host(q), _host(qn), _host(y), _host(d), _host(loss),
                                    _host(idx)))
        return {"Q": q, "Qn": qn, "y": y, "delta": d, "loss": float(loss[0]), "idx": idx}

    def set_handoff_wait(self, ticks=0, break_pairing=False):
        _check(lib().train_set_handoff_wait(self._h, int(ticks), int(bool(break_pairing))))

    def target_from_table(self):
        n = C.c_uint32()
        _check(lib().train_get_target_source(self._h, C.byref(n)))
        return bool(n.value)

    def kernels_per_step(self):
        n = C.c_uint32()
        _check(lib().train_kernels_per_step(self._h, C.byref(n)))
        return n.value


class InRamReplay:
    """The paper's comparison system: replay in host RAM, per-step host sampling and H2D copy."""

    def __init__(self, capacity, state_dim, batch, burn_in=0, seed=0, device="cuda:0"):
        self.D, self.batch = state_dim, batch
        nbytes = int(lib().inram_device_bytes(state_dim, batch))
        if nbytes == 0:
            raise ReplayError(RP_EINVAL, "invalid in-RAM replay configuration")
        self.dev_batch = _alloc_bytes(nbytes, torch.device(device))
        h = C.c_void_p()
        with torch.cuda.device(torch.device(device)):
            _check(lib().inram_create(capacity, state_dim, burn_in, seed, batch, _dev(self.dev_batch),
                                      nbytes, C.byref(h)))
        self._h = h
        self._destroy = lib().inram_destroy

    def close(self):
        if getattr(self, "_h", None):
            self._destroy(self._h)
            self._h = None

    __del__ = close

    @staticmethod
    def _fields(s, s_next, a, r, term):
        return [np.ascontiguousarray(s, np.float32), np.ascontiguousarray(s_next, np.float32),
                np.ascontiguousarray(a, np.int32), np.ascontiguousarray(r, np.float32),
                np.ascontiguousarray(term, np.uint8)]

    def append(self, s, s_next, a, r, term):
        keep = self._fields(s, s_next, a, r, term)
        return _check(lib().inram_append(self._h, len(keep[2]), *[_host(x) for x in keep]))

    def train_step(self, trainer, stream=None):
        return _check(lib().inram_train_step(self._h, trainer._h, _stream_ptr(stream)))

    def train_steps(self, trainer, count, appends_per_step, s, s_next, a, r, term, stream=None):
        keep = self._fields(s, s_next, a, r, term)
        if len(keep[2]) < count * appends_per_step:
            raise ValueError("not enough experiences for that many steps")
        done = C.c_uint64()
        _check(lib().inram_train_steps(self._h, trainer._h, count, appends_per_step,
                                       *[_host(x) for x in keep], _stream_ptr(stream), C.byref(done)))
        return done.value

    def state(self):
        v = [C.c_uint64() for _ in range(4)]
        _check(lib().inram_get_state(self._h, *[C.byref(x) for x in v]))
        return tuple(x.value for x in v)

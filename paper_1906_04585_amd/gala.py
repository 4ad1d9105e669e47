"""ctypes binding of libgala.so -- argument marshalling only.

Every function maps 1:1 to an entry point of include/gala.h.  Device buffers are
torch CUDA tensors (torch is used for device memory and streams, nothing else); the
library raises if the HIP extension is missing -- there is no CPU fallback."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("GALA_LIBRARY", os.path.join(_PKG, "libgala.so"))

EXPORTS = [
    "gala_create", "gala_destroy", "gala_param_count", "gala_last_error",
    "gala_set_params", "gala_get_params", "gala_set_opt_state", "gala_get_opt_state",
    "gala_learner_step", "gala_gossip", "gala_round", "gala_a2c_allreduce_step", "gala_get_mean_grad", "gala_act", "gala_grad_cosine", "gala_update_norm", "gala_prop1_bound", "gala_get_grads", "gala_get_step_stats",
    "gala_get_outputs", "gala_consensus_distance", "gala_consensus_distance_noalloc", "gala_get_head_grads",
    "gala_get_peer_table",
    "gala_set_profiling", "gala_get_phase_times", "gala_get_activations",
]

TOPOLOGY = {"ring": 0, "exp": 1, "explicit": 2, "exp_reverse": 3}


class GalaError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"gala error {code}: {text}")
        self.code = code


class _NetDims(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("in_c", "in_h", "in_w", "c1", "c2", "c3", "fc", "n_actions")]


class _HParams(C.Structure):
    _fields_ = [("T", C.c_int), ("B", C.c_int), ("gamma", C.c_float), ("vf_coef", C.c_float),
                ("ent_coef", C.c_float), ("lr", C.c_float), ("rms_alpha", C.c_float),
                ("rms_eps", C.c_float), ("max_grad_norm", C.c_float), ("compute_dtype", C.c_int)]


class _Topology(C.Structure):
    _fields_ = [("kind", C.c_int), ("max_delay", C.c_int), ("delay_seed", C.c_uint64),
                ("peers", C.c_void_p), ("weights", C.c_void_p), ("n_phases", C.c_int), ("max_in", C.c_int)]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load the built library; fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: run `python -m paper_1906_04585_amd.build` "
                              "(or __graft_entry__.build()) first; there is no fallback path")
        L = C.CDLL(_LIB_PATH)
        L.gala_create.argtypes = [C.POINTER(C.c_void_p), C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.gala_destroy.argtypes = [C.c_void_p]
        L.gala_param_count.argtypes = [C.c_void_p]
        L.gala_param_count.restype = C.c_size_t
        L.gala_last_error.argtypes = [C.c_void_p]
        L.gala_last_error.restype = C.c_char_p
        for name in ("gala_set_params", "gala_get_params", "gala_set_opt_state", "gala_get_opt_state",
                     "gala_get_grads"):
            getattr(L, name).argtypes = [C.c_void_p, C.c_void_p, C.c_int]
        L.gala_learner_step.argtypes = [C.c_void_p] * 6
        L.gala_gossip.argtypes = [C.c_void_p, C.c_int64]
        L.gala_round.argtypes = [C.c_void_p] * 6 + [C.c_int64]
        L.gala_a2c_allreduce_step.argtypes = [C.c_void_p] * 6
        L.gala_get_mean_grad.argtypes = [C.c_void_p, C.c_void_p, C.c_int]
        L.gala_grad_cosine.argtypes = [C.c_void_p, C.c_void_p]
        L.gala_update_norm.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.gala_prop1_bound.argtypes = [C.c_double, C.c_void_p, C.c_int, C.c_void_p]
        L.gala_act.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
        L.gala_get_step_stats.argtypes = [C.c_void_p, C.c_void_p]
        L.gala_get_outputs.argtypes = [C.c_void_p] * 5
        L.gala_consensus_distance.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.gala_consensus_distance_noalloc.argtypes = [C.c_void_p, C.c_void_p]
        L.gala_get_head_grads.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.gala_get_peer_table.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        L.gala_set_profiling.argtypes = [C.c_void_p, C.c_int]
        L.gala_get_activations.argtypes = [C.c_void_p, C.c_int, C.c_void_p]
        L.gala_get_phase_times.argtypes = [C.c_void_p, C.c_char_p, C.c_size_t, C.c_void_p, C.c_int, C.c_void_p]
        _lib = L
    return _lib


def _dev_ptr(t, dtype, numel=None):
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise TypeError(f"expected a contiguous CUDA tensor of {dtype}")
    if numel is not None and t.numel() != numel:
        raise ValueError(f"expected {numel} elements, got {t.numel()}")
    return C.c_void_p(t.data_ptr())


class Gala:
    """N A2C actor-learners on one GPU (gala_create / gala_destroy)."""

    def __init__(self, n_agents: int, n_actions: int, T: int, B: int, hparams: dict, topology: str = "ring",
                 max_delay: int = 0, delay_seed: int = 0, peers=None, weights=None, stream=None,
                 net_dims: dict | None = None):
        import torch
        self._lib = load_library()
        self._h = C.c_void_p()
        nd = dict(in_c=4, in_h=84, in_w=84, c1=32, c2=64, c3=64, fc=512)
        if net_dims:
            nd.update(net_dims)
        net = _NetDims(nd["in_c"], nd["in_h"], nd["in_w"], nd["c1"], nd["c2"], nd["c3"], nd["fc"], n_actions)
        hp = _HParams(T, B, hparams["gamma"], hparams["vf_coef"], hparams["ent_coef"], hparams["lr"],
                      hparams["rms_alpha"], hparams["rms_eps"], hparams["max_grad_norm"],
                      int(hparams.get("compute_dtype", 0)))
        topo = _Topology()
        topo.kind = TOPOLOGY[topology]
        topo.max_delay, topo.delay_seed = max_delay, delay_seed
        self._keep = []
        if topology == "explicit":
            p = np.ascontiguousarray(peers, dtype=np.int32)
            w = np.ascontiguousarray(weights, dtype=np.float32)
            self._keep += [p, w]
            topo.peers, topo.weights = p.ctypes.data, w.ctypes.data
            topo.n_phases, topo.max_in = p.shape[0], p.shape[2]
        self.max_in = topo.max_in if topology == "explicit" else 1
        if stream is None:
            stream = torch.cuda.current_stream()
        self._stream = stream
        rc = self._lib.gala_create(C.byref(self._h), n_agents, C.byref(topo), C.byref(net), C.byref(hp),
                                   C.c_void_p(stream.cuda_stream))
        if rc != 0:
            self._h = C.c_void_p()
            raise GalaError(rc, self._lib.gala_last_error(None).decode())
        self.N, self.A, self.T, self.B = n_agents, n_actions, T, B
        self.d = int(self._lib.gala_param_count(self._h))

    # -- helpers --------------------------------------------------------------------------
    def _check(self, rc: int):
        if rc != 0:
            raise GalaError(rc, self._lib.gala_last_error(self._h).decode())

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            self._lib.gala_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _put(self, fn, arr):
        import torch
        if isinstance(arr, torch.Tensor) and arr.is_cuda:
            self._check(fn(self._h, _dev_ptr(arr, torch.float32, self.N * self.d), 1))
        else:
            a = np.ascontiguousarray(arr, dtype=np.float32)
            if a.size != self.N * self.d:
                raise ValueError(f"expected {self.N * self.d} elements, got {a.size}")
            self._check(fn(self._h, a.ctypes.data_as(C.c_void_p), 0))

    def _get(self, fn, out=None):
        import torch
        if isinstance(out, torch.Tensor) and out.is_cuda:
            self._check(fn(self._h, _dev_ptr(out, torch.float32, self.N * self.d), 1))
            return out
        a = np.empty((self.N, self.d), dtype=np.float32)
        self._check(fn(self._h, a.ctypes.data_as(C.c_void_p), 0))
        return a

    # -- the ABI, one method per entry point -------------------------------------------------
    def param_count(self) -> int:
        return self.d

    def set_params(self, x):
        self._put(self._lib.gala_set_params, x)

    def get_params(self, out=None):
        return self._get(self._lib.gala_get_params, out)

    def set_opt_state(self, v):
        self._put(self._lib.gala_set_opt_state, v)

    def get_opt_state(self, out=None):
        return self._get(self._lib.gala_get_opt_state, out)

    def get_grads(self, out=None):
        return self._get(self._lib.gala_get_grads, out)

    def _rollout_ptrs(self, obs_u8, actions, rewards, dones, bootstrap_obs):
        import torch
        N, T, B = self.N, self.T, self.B
        fr = 4 * 84 * 84
        return (_dev_ptr(obs_u8, torch.uint8, N * T * B * fr), _dev_ptr(actions, torch.int32, N * T * B),
                _dev_ptr(rewards, torch.float32, N * T * B), _dev_ptr(dones, torch.uint8, N * T * B),
                _dev_ptr(bootstrap_obs, torch.uint8, N * B * fr))

    def learner_step(self, obs_u8, actions, rewards, dones, bootstrap_obs):
        self._check(self._lib.gala_learner_step(
            self._h, *self._rollout_ptrs(obs_u8, actions, rewards, dones, bootstrap_obs)))

    def round(self, obs_u8, actions, rewards, dones, bootstrap_obs, rnd: int):
        self._check(self._lib.gala_round(
            self._h, *self._rollout_ptrs(obs_u8, actions, rewards, dones, bootstrap_obs), int(rnd)))

    def a2c_allreduce_step(self, obs_u8, actions, rewards, dones, bootstrap_obs):
        self._check(self._lib.gala_a2c_allreduce_step(
            self._h, *self._rollout_ptrs(obs_u8, actions, rewards, dones, bootstrap_obs)))

    def get_mean_grad(self) -> np.ndarray:
        a = np.empty(self.d, dtype=np.float32)
        self._check(self._lib.gala_get_mean_grad(self._h, a.ctypes.data_as(C.c_void_p), 0))
        return a

    def act(self, obs_u8, seed: int, step: int, actions, values=None, logp=None):
        """actions int32 [N][B] (and optionally values, logp float32 [N][B]) are CUDA tensors written in place."""
        import torch
        n = self.N * self.B
        self._check(self._lib.gala_act(
            self._h, _dev_ptr(obs_u8, torch.uint8, n * 4 * 84 * 84), C.c_uint64(seed % 2 ** 64), int(step),
            _dev_ptr(actions, torch.int32, n),
            None if values is None else _dev_ptr(values, torch.float32, n),
            None if logp is None else _dev_ptr(logp, torch.float32, n)))

    def grad_cosine(self) -> np.ndarray:
        a = np.empty((self.N, self.N), dtype=np.float32)
        self._check(self._lib.gala_grad_cosine(self._h, a.ctypes.data_as(C.c_void_p)))
        return a

    def update_norm(self):
        rows = np.empty(self.N, dtype=np.float32)
        fr = C.c_float()
        self._check(self._lib.gala_update_norm(self._h, rows.ctypes.data_as(C.c_void_p), C.byref(fr)))
        return float(fr.value), rows

    def gossip(self, rnd: int):
        self._check(self._lib.gala_gossip(self._h, int(rnd)))

    def get_step_stats(self) -> np.ndarray:
        a = np.empty((self.N, 5), dtype=np.float32)
        self._check(self._lib.gala_get_step_stats(self._h, a.ctypes.data_as(C.c_void_p)))
        return a

    def get_outputs(self) -> dict:
        N, M, B, A = self.N, self.T * self.B, self.B, self.A
        out = dict(logits=np.empty((N, M, A), np.float32), values=np.empty((N, M + B), np.float32),
                   returns=np.empty((N, M), np.float32), advantages=np.empty((N, M), np.float32))
        self._check(self._lib.gala_get_outputs(self._h, *[out[k].ctypes.data_as(C.c_void_p) for k in
                                                          ("logits", "values", "returns", "advantages")]))
        return out

    def consensus_distance(self):
        mx, fr = C.c_float(0.0), C.c_float(0.0)
        self._check(self._lib.gala_consensus_distance(self._h, C.byref(mx), C.byref(fr)))
        return float(mx.value), float(fr.value)

    def consensus_distance_noalloc(self, result):
        """result: float32 CUDA tensor of (at least) 2 elements, written in stream order (no synchronisation)."""
        import torch
        if result.numel() < 2:
            raise ValueError("result needs two elements")
        self._check(self._lib.gala_consensus_distance_noalloc(self._h, _dev_ptr(result, torch.float32)))

    def get_head_grads(self):
        """(dlogits [N, T*B, A], dvalues [N, T*B]) as the loss kernel of the last learner step wrote them."""
        M = self.T * self.B
        dl = np.empty((self.N, M, self.A), np.float32)
        dv = np.empty((self.N, M), np.float32)
        self._check(self._lib.gala_get_head_grads(self._h, dl.ctypes.data_as(C.c_void_p), dv.ctypes.data_as(C.c_void_p)))
        return dl, dv

    def get_peer_table(self, rnd: int):
        peer = np.empty((self.N, self.max_in), dtype=np.int32)
        delay = np.empty((self.N, self.max_in), dtype=np.int32)
        self._check(self._lib.gala_get_peer_table(self._h, int(rnd), peer.ctypes.data_as(C.c_void_p),
                                                  delay.ctypes.data_as(C.c_void_p)))
        return peer, delay

    def set_profiling(self, enabled: bool):
        self._check(self._lib.gala_set_profiling(self._h, int(bool(enabled))))

    def get_phase_times(self) -> dict:
        """{phase name: milliseconds} of the phases recorded since the last learner step began."""
        names = C.create_string_buffer(2048)
        ms = (C.c_float * 64)()
        n = C.c_int(0)
        self._check(self._lib.gala_get_phase_times(self._h, names, 2048, ms, 64, C.byref(n)))
        keys = names.value.decode().split(";")[:n.value]
        out = {}
        for k, v in zip(keys, list(ms)[:n.value]):
            out[k] = out.get(k, 0.0) + float(v)
        return out

    _ACT_SHAPES = {1: (20, 20, 32), 2: (9, 9, 64), 3: (7, 7, 64), 4: (512,)}

    def get_activations(self, layer: int) -> np.ndarray:
        """[N, F, H, W, C] (layer 1..3) or [N, F, 512] (layer 4), channels-last, after ReLU."""
        F = self.T * self.B + self.B
        a = np.empty((self.N, F) + self._ACT_SHAPES[layer], dtype=np.float32)
        self._check(self._lib.gala_get_activations(self._h, layer, a.ctypes.data_as(C.c_void_p)))
        return a


def prop1_bound(beta: float, update_norms) -> float:
    u = np.ascontiguousarray(update_norms, dtype=np.float64)
    out = C.c_double()
    rc = load_library().gala_prop1_bound(float(beta), u.ctypes.data_as(C.c_void_p), int(u.size), C.byref(out))
    if rc != 0:
        raise GalaError(rc, load_library().gala_last_error(None).decode())
    return float(out.value)

"""ctypes binding of libgco.so: argument marshalling only.

Every method of ``Context`` is one call of the C ABI declared in include/gco.h
and carries the same name without the ``gco_`` prefix.  Host arrays are numpy
arrays; PyTorch supplies the HIP stream and, optionally, device memory (through
the allocator hooks of ``gco_config``).  There is no fallback: if the library
is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgco.so")

OK, EINVAL, ENOMEM, ESTATE, EDEVICE, ERANGE = 0, -1, -2, -3, -4, -5
PROBLEM = {"mis": 0, "maxcut": 1}
NORM = {"sym": 0, "mean": 1}
STORAGE = {"fp32": 0, "bf16": 1}
REPAIR = {"none": 0, "local": 1, "all": 2}
SCALAR_FORM = {"auto": 0, "streams": 1, "staged": 2, "one_launch": 3}

ALLOC_FN = C.CFUNCTYPE(C.c_void_p, C.c_size_t, C.c_void_p)
FREE_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_void_p)


class Config(C.Structure):
    _fields_ = [
        ("problem", C.c_int32), ("num_layers", C.c_int32), ("dim", C.c_int32),
        ("norm", C.c_int32), ("storage", C.c_int32), ("weight_sharing", C.c_int32),
        ("train_embed", C.c_int32), ("alpha", C.c_float), ("beta", C.c_float),
        ("lr", C.c_float), ("adam_b1", C.c_float), ("adam_b2", C.c_float),
        ("adam_eps", C.c_float), ("stream", C.c_void_p), ("dev_alloc", ALLOC_FN),
        ("dev_free", FREE_FN), ("alloc_user", C.c_void_p),
    ]


class RLConfig(C.Structure):
    _fields_ = [("rounds", C.c_int32), ("epochs_per_round", C.c_int32), ("lam", C.c_float),
                ("q_lr", C.c_float), ("q_gamma", C.c_float), ("epsilon", C.c_float)]


class GcoError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"gco error {code}: {message}")
        self.code = code


_lib = None

# name -> (restype, argtypes); the list mirrors include/gco.h one to one
_PROTOTYPES = {
    "gco_default_config": (C.c_int, [C.POINTER(Config)]),
    "gco_create": (C.c_int, [C.POINTER(Config), C.POINTER(C.c_void_p)]),
    "gco_destroy": (C.c_int, [C.c_void_p]),
    "gco_get_config": (C.c_int, [C.c_void_p, C.POINTER(Config)]),
    "gco_apportion": (C.c_int, [C.POINTER(C.c_double), C.c_int32, C.c_int64, C.POINTER(C.c_int32),
                                C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "gco_set_scalar_layer_form": (C.c_int, [C.c_void_p, C.c_int]),
    "gco_get_scalar_layer_form": (C.c_int, [C.c_void_p, C.POINTER(C.c_int)]),
    "gco_last_error": (C.c_char_p, [C.c_void_p]),
    "gco_upload_graph": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32]),
    "gco_graph_info": (C.c_int, [C.c_void_p] + [C.POINTER(C.c_int64)] * 4),
    "gco_set_params": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p)]),
    "gco_set_params_gumbel": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.POINTER(C.c_void_p)]),
    "gco_get_params": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p)]),
    "gco_get_opt_state": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p),
                                    C.POINTER(C.c_void_p), C.POINTER(C.c_int64)]),
    "gco_set_opt_state": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p),
                                    C.POINTER(C.c_void_p), C.c_int64]),
    "gco_set_linear_penalty": (C.c_int, [C.c_void_p, C.c_void_p]),
    "gco_train": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p]),
    "gco_train_subset": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p]),
    "gco_get_steps": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "gco_set_steps": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "gco_keep_best": (C.c_int, [C.c_void_p, C.c_int32]),
    "gco_get_best_loss": (C.c_int, [C.c_void_p, C.c_void_p]),
    "gco_restore_best": (C.c_int, [C.c_void_p]),
    "gco_forward": (C.c_int, [C.c_void_p]),
    "gco_get_probs": (C.c_int, [C.c_void_p, C.c_void_p]),
    "gco_loss": (C.c_int, [C.c_void_p, C.POINTER(C.c_double), C.c_void_p]),
    "gco_get_grads": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p)]),
    "gco_get_hidden": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p]),
    "gco_round_repair": (C.c_int, [C.c_void_p, C.c_float, C.c_int32, C.c_void_p] + [C.POINTER(C.c_int64)] * 3),
    "gco_round_repair_static": (C.c_int, [C.c_void_p, C.c_float, C.c_int32, C.c_void_p] + [C.POINTER(C.c_int64)] * 3),
    "gco_cut_edges": (C.c_int, [C.c_void_p, C.POINTER(C.c_int64), C.c_void_p, C.c_void_p]),
    "gco_cross_mask": (C.c_int, [C.c_void_p, C.c_void_p]),
    "gco_conflict_edges": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(C.c_int64), C.c_void_p, C.c_void_p]),
    "gco_coordinate": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(RLConfig), C.c_void_p, C.c_void_p,
                                 C.POINTER(C.c_double), C.c_void_p, C.c_void_p, C.c_void_p,
                                 C.POINTER(C.c_int32)]),
    "gco_stream_probe": (C.c_int, [C.c_int32, C.c_size_t, C.c_int32, C.POINTER(C.c_double)]),
    "gco_louvain": (C.c_int, [C.c_int64, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                              C.POINTER(C.c_int32), C.POINTER(C.c_double)]),
    "gco_pack_parts": (C.c_int, [C.c_int64, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.POINTER(C.c_int32)]),
    "gco_sync": (C.c_int, [C.c_void_p]),
    "gco_set_profiling": (C.c_int, [C.c_void_p, C.c_int32, C.c_uint64]),
    "gco_num_kernel_kinds": (C.c_int, []),
    "gco_kernel_kind_name": (C.c_char_p, [C.c_int32]),
    "gco_get_timing": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_double),
                                 C.POINTER(C.c_double)]),
    "gco_reset_timing": (C.c_int, [C.c_void_p]),
}


def load():
    """Load libgco.so (raises OSError if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise OSError(f"{LIB_PATH} is missing: run `python -m paper_2511_09261_amd.build`")
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in _PROTOTYPES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def exported_symbols():
    return list(_PROTOTYPES)


def _ptr(a):
    return None if a is None else a.ctypes.data


def stream_probe(kind, bytes_per_array=1 << 30, repeats=10):
    """gco_stream_probe: GB/s of a plain streaming kernel ("read", "copy" or "update")."""
    lib = load()
    out = C.c_double()
    rc = lib.gco_stream_probe({"read": 0, "copy": 1, "update": 2}[kind], bytes_per_array, repeats, C.byref(out))
    if rc != 0:
        raise GcoError(rc, "gco_stream_probe failed")
    return out.value


def apportion(work, target, lo, hi):
    """gco_apportion: shares of `target` workgroups in proportion to work, within [lo, hi].  Host only."""
    lib = load()
    work = np.ascontiguousarray(work, dtype=np.float64)
    lo = np.ascontiguousarray(lo, dtype=np.int32)
    hi = np.ascontiguousarray(hi, dtype=np.int32)
    share = np.empty(work.shape[0], dtype=np.int32)
    as_p = lambda a, t: a.ctypes.data_as(C.POINTER(t))
    rc = lib.gco_apportion(as_p(work, C.c_double), work.shape[0], int(target), as_p(lo, C.c_int32),
                           as_p(hi, C.c_int32), as_p(share, C.c_int32))
    if rc != 0:
        raise GcoError(rc, "gco_apportion failed (bad bounds or sizes)")
    return share


def louvain(n, rowptr, col, max_levels=32):
    """gco_louvain: (part_id int32[n], number of communities, modularity).  Host only."""
    lib = load()
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    col = np.ascontiguousarray(col, dtype=np.int32)
    part = np.empty(n, dtype=np.int32)
    P, q = C.c_int32(), C.c_double()
    rc = lib.gco_louvain(n, _ptr(rowptr), _ptr(col), max_levels, _ptr(part), C.byref(P), C.byref(q))
    if rc != 0:
        raise GcoError(rc, "gco_louvain failed (malformed graph or size out of range)")
    return part, P.value, q.value


def pack_parts(part, num_parts, max_parts):
    """gco_pack_parts: (group of every node int32[n], number of groups).  Host only."""
    lib = load()
    part = np.ascontiguousarray(part, dtype=np.int32)
    out = np.empty_like(part)
    P = C.c_int32()
    rc = lib.gco_pack_parts(part.shape[0], _ptr(part), num_parts, max_parts, _ptr(out), C.byref(P))
    if rc != 0:
        raise GcoError(rc, "gco_pack_parts failed (bad ids or counts)")
    return out, P.value


def _f32(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.float32)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {shape}, got {a.shape}")
    return a


class TorchAllocator:
    """Device memory from PyTorch's caching allocator, handed to the library
    through the dev_alloc / dev_free hooks."""

    def __init__(self):
        import torch
        self.torch = torch
        self.live = {}
        self.alloc_cb = ALLOC_FN(self._alloc)
        self.free_cb = FREE_FN(self._free)

    def _alloc(self, nbytes, _user):
        try:
            t = self.torch.empty(int(nbytes), dtype=self.torch.uint8, device="cuda")
        except Exception:  # out of memory: report NULL, the library returns GCO_ENOMEM
            return None
        self.live[t.data_ptr()] = t
        return t.data_ptr()

    def _free(self, ptr, _user):
        self.live.pop(ptr, None)


class Context:
    """One gco_ctx.  See include/gco.h for the meaning of every call."""

    def __init__(self, problem="mis", num_layers=2, dim=16, norm="sym", storage="fp32",
                 weight_sharing=False, train_embed=True, alpha=2.0, beta=1.0, lr=1e-2,
                 adam_b1=0.9, adam_b2=0.999, adam_eps=1e-8, use_torch=True):
        self.lib = load()
        cfg = Config()
        self._check(self.lib.gco_default_config(C.byref(cfg)), None)
        cfg.problem, cfg.num_layers, cfg.dim = PROBLEM[problem], num_layers, dim
        cfg.norm, cfg.storage = NORM[norm], STORAGE[storage]
        cfg.weight_sharing, cfg.train_embed = int(weight_sharing), int(train_embed)
        cfg.alpha, cfg.beta, cfg.lr = alpha, beta, lr
        cfg.adam_b1, cfg.adam_b2, cfg.adam_eps = adam_b1, adam_b2, adam_eps
        self._allocator = None
        self._stream = None
        if use_torch:
            import torch
            torch.cuda.init()
            self._stream = torch.cuda.current_stream()
            cfg.stream = self._stream.cuda_stream
            self._allocator = TorchAllocator()
            cfg.dev_alloc = self._allocator.alloc_cb
            cfg.dev_free = self._allocator.free_cb
        self.cfg = cfg
        self.num_layers, self.dim = num_layers, dim
        self.weight_sharing = bool(weight_sharing)
        self.n = 0
        self.num_parts = 1
        h = C.c_void_p()
        rc = self.lib.gco_create(C.byref(cfg), C.byref(h))
        if rc != OK:
            raise GcoError(rc, "gco_create failed")
        self.h = h

    # -- plumbing --
    def _check(self, rc, h="self"):
        if rc != OK:
            msg = self.lib.gco_last_error(self.h).decode() if h == "self" else "call failed"
            raise GcoError(rc, msg)

    def _w_shapes(self):
        pw = 1 if self.weight_sharing else self.num_parts
        return [(pw, self.dim, self.dim if l < self.num_layers else 1)
                for l in range(1, self.num_layers + 1)]

    def _ptr_array(self, arrays):
        arr = (C.c_void_p * len(arrays))()
        for i, a in enumerate(arrays):
            arr[i] = _ptr(a)
        return arr

    # -- the ABI --
    def set_scalar_layer_form(self, form):
        """form: "auto", "streams", "staged" or "one_launch"; before upload_graph."""
        self._check(self.lib.gco_set_scalar_layer_form(self.h, SCALAR_FORM[form]))

    def get_scalar_layer_form(self):
        out = C.c_int(0)
        self._check(self.lib.gco_get_scalar_layer_form(self.h, C.byref(out)))
        return {v: k for k, v in SCALAR_FORM.items()}[out.value]

    def destroy(self):
        if self.h:
            self.lib.gco_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def last_error(self):
        return self.lib.gco_last_error(self.h).decode()

    def upload_graph(self, n, rowptr, col, part_id=None, num_parts=1):
        rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
        col = np.ascontiguousarray(col, dtype=np.int32)
        if rowptr.shape[0] != n + 1:
            raise ValueError("rowptr must have n + 1 entries")
        if n >= 1 and col.shape[0] != rowptr[-1]:
            raise ValueError("col must have rowptr[n] entries")
        part = None if part_id is None else np.ascontiguousarray(part_id, dtype=np.int32)
        if part is not None and part.shape[0] != n:
            raise ValueError("part_id must have n entries")
        self._check(self.lib.gco_upload_graph(self.h, n, _ptr(rowptr), _ptr(col), _ptr(part), num_parts))
        self.n, self.num_parts = n, (num_parts if part is not None else 1)

    def graph_info(self):
        v = [C.c_int64() for _ in range(4)]
        self._check(self.lib.gco_graph_info(self.h, *[C.byref(x) for x in v]))
        return dict(zip(("n", "m", "m_local", "m_cut"), (x.value for x in v)))

    def set_params(self, E, Ws):
        E = _f32(E, (self.n, self.dim))
        Ws = [_f32(W, s) for W, s in zip(Ws, self._w_shapes())]
        if len(Ws) != self.num_layers:
            raise ValueError("one weight array per layer expected")
        self._check(self.lib.gco_set_params(self.h, _ptr(E), self._ptr_array(Ws)))

    def set_params_gumbel(self, E, U, tau, Ws):
        E = _f32(E, (self.n, self.dim))
        U = _f32(U, (self.n, self.dim))
        Ws = [_f32(W, s) for W, s in zip(Ws, self._w_shapes())]
        if len(Ws) != self.num_layers:
            raise ValueError("one weight array per layer expected")
        self._check(self.lib.gco_set_params_gumbel(self.h, _ptr(E), _ptr(U), tau, self._ptr_array(Ws)))

    def get_params(self):
        E = np.empty((self.n, self.dim), dtype=np.float32)
        Ws = [np.empty(s, dtype=np.float32) for s in self._w_shapes()]
        self._check(self.lib.gco_get_params(self.h, _ptr(E), self._ptr_array(Ws)))
        return E, Ws

    def get_opt_state(self):
        mE = np.empty((self.n, self.dim), dtype=np.float32)
        vE = np.empty_like(mE)
        mW = [np.empty(s, dtype=np.float32) for s in self._w_shapes()]
        vW = [np.empty(s, dtype=np.float32) for s in self._w_shapes()]
        step = C.c_int64()
        self._check(self.lib.gco_get_opt_state(self.h, _ptr(mE), _ptr(vE), self._ptr_array(mW),
                                               self._ptr_array(vW), C.byref(step)))
        return mE, vE, mW, vW, step.value

    def set_opt_state(self, mE, vE, mW, vW, step):
        mE, vE = _f32(mE, (self.n, self.dim)), _f32(vE, (self.n, self.dim))
        mW = [_f32(W, s) for W, s in zip(mW, self._w_shapes())]
        vW = [_f32(W, s) for W, s in zip(vW, self._w_shapes())]
        self._check(self.lib.gco_set_opt_state(self.h, _ptr(mE), _ptr(vE), self._ptr_array(mW),
                                               self._ptr_array(vW), int(step)))

    def set_linear_penalty(self, extra):
        extra = None if extra is None else _f32(extra, (self.n,))
        self._check(self.lib.gco_set_linear_penalty(self.h, _ptr(extra)))

    def train(self, epochs, return_loss=True):
        out = np.empty(epochs, dtype=np.float64) if return_loss else None
        self._check(self.lib.gco_train(self.h, epochs, _ptr(out)))
        return out

    @property
    def num_weight_sets(self):
        return 1 if self.weight_sharing else self.num_parts

    def train_subset(self, epochs, parts, return_loss=True):
        parts = np.ascontiguousarray(parts, dtype=np.int32)
        out = np.empty(epochs, dtype=np.float64) if return_loss else None
        self._check(self.lib.gco_train_subset(self.h, epochs, _ptr(parts), parts.shape[0], _ptr(out)))
        return out

    def get_steps(self):
        se = np.empty(self.num_parts, dtype=np.int64)
        sw = np.empty(self.num_weight_sets, dtype=np.int64)
        self._check(self.lib.gco_get_steps(self.h, _ptr(se), _ptr(sw)))
        return se, sw

    def set_steps(self, steps_embed, steps_weights):
        se = np.ascontiguousarray(steps_embed, dtype=np.int64)
        sw = np.ascontiguousarray(steps_weights, dtype=np.int64)
        assert se.shape[0] == self.num_parts and sw.shape[0] == self.num_weight_sets
        self._check(self.lib.gco_set_steps(self.h, _ptr(se), _ptr(sw)))

    def keep_best(self, enable=True):
        self._check(self.lib.gco_keep_best(self.h, 1 if enable else 0))

    def get_best_loss(self):
        best = np.empty(self.num_weight_sets, dtype=np.float64)
        self._check(self.lib.gco_get_best_loss(self.h, _ptr(best)))
        return best

    def restore_best(self):
        self._check(self.lib.gco_restore_best(self.h))

    def forward(self):
        self._check(self.lib.gco_forward(self.h))

    def get_probs(self):
        p = np.empty(self.n, dtype=np.float32)
        self._check(self.lib.gco_get_probs(self.h, _ptr(p)))
        return p

    def loss(self):
        tot = C.c_double()
        per = np.empty(self.num_parts, dtype=np.float64)
        self._check(self.lib.gco_loss(self.h, C.byref(tot), _ptr(per)))
        return tot.value, per

    def get_grads(self):
        gE = np.empty((self.n, self.dim), dtype=np.float32)
        gWs = [np.empty(s, dtype=np.float32) for s in self._w_shapes()]
        self._check(self.lib.gco_get_grads(self.h, _ptr(gE), self._ptr_array(gWs)))
        return gE, gWs

    def get_hidden(self, layer):
        H = np.empty((self.n, self.dim), dtype=np.float32)
        self._check(self.lib.gco_get_hidden(self.h, layer, _ptr(H)))
        return H

    def round_repair(self, thr=0.5, repair_scope="local"):
        x = np.empty(self.n, dtype=np.uint8)
        obj, cb, ca = C.c_int64(), C.c_int64(), C.c_int64()
        self._check(self.lib.gco_round_repair(self.h, thr, REPAIR[repair_scope], _ptr(x),
                                              C.byref(obj), C.byref(cb), C.byref(ca)))
        return x, obj.value, cb.value, ca.value

    def round_repair_static(self, thr=0.5, repair_scope="local"):
        """gco_round_repair_static: the same, inside the library's fixed work area (no allocation)."""
        x = np.empty(self.n, dtype=np.uint8)
        obj, cb, ca = C.c_int64(), C.c_int64(), C.c_int64()
        self._check(self.lib.gco_round_repair_static(self.h, thr, REPAIR[repair_scope], _ptr(x),
                                                     C.byref(obj), C.byref(cb), C.byref(ca)))
        return x, obj.value, cb.value, ca.value

    def coordinate(self, part, uniforms, rounds, epochs_per_round, lam=1.0, q_lr=0.5, q_gamma=0.9,
                   epsilon=0.2):
        """gco_coordinate: dict with x_best, score_best, actions, scores, conflicts (of the
        rounds that ran)."""
        part = None if part is None else np.ascontiguousarray(part, dtype=np.int32)
        uniforms = np.ascontiguousarray(uniforms, dtype=np.float64).reshape(-1)
        if uniforms.shape[0] < 2 * rounds:
            raise ValueError("two uniforms per round are needed")
        cfg = RLConfig(rounds, epochs_per_round, lam, q_lr, q_gamma, epsilon)
        x = np.empty(self.n, dtype=np.uint8)
        best, ran = C.c_double(), C.c_int32()
        actions = np.empty(max(rounds, 1), dtype=np.int32)
        scores = np.empty(rounds + 1, dtype=np.float64)
        conflicts = np.empty(rounds + 1, dtype=np.int64)
        self._check(self.lib.gco_coordinate(self.h, _ptr(part), C.byref(cfg), _ptr(uniforms), _ptr(x),
                                            C.byref(best), _ptr(actions), _ptr(scores), _ptr(conflicts),
                                            C.byref(ran)))
        r = ran.value
        return {"x_best": x, "score_best": best.value, "actions": actions[:r].tolist(),
                "scores": scores[:r + 1].tolist(), "conflicts": conflicts[:r + 1].tolist()}

    def cut_edges(self):
        cnt = C.c_int64()
        self._check(self.lib.gco_cut_edges(self.h, C.byref(cnt), None, None))
        u = np.empty(cnt.value, dtype=np.int32)
        v = np.empty(cnt.value, dtype=np.int32)
        if cnt.value:
            self._check(self.lib.gco_cut_edges(self.h, C.byref(cnt), _ptr(u), _ptr(v)))
        return u, v

    def cross_mask(self):
        c = np.empty(self.n, dtype=np.uint8)
        self._check(self.lib.gco_cross_mask(self.h, _ptr(c)))
        return c

    def conflict_edges(self, x):
        x = np.ascontiguousarray(x, dtype=np.uint8)
        if x.shape[0] != self.n:
            raise ValueError("x must have n entries")
        cnt = C.c_int64()
        self._check(self.lib.gco_conflict_edges(self.h, _ptr(x), C.byref(cnt), None, None))
        u = np.empty(cnt.value, dtype=np.int32)
        v = np.empty(cnt.value, dtype=np.int32)
        if cnt.value:
            self._check(self.lib.gco_conflict_edges(self.h, _ptr(x), C.byref(cnt), _ptr(u), _ptr(v)))
        return u, v

    def sync(self):
        self._check(self.lib.gco_sync(self.h))

    def set_profiling(self, mode, kinds=None):
        mask = 0xFFFFFFFFFFFFFFFF
        if kinds is not None:
            names = self.kernel_kind_names()
            mask = 0
            for k in kinds:
                mask |= 1 << names.index(k)
        self._check(self.lib.gco_set_profiling(self.h, mode, mask))

    def kernel_kind_names(self):
        return [self.lib.gco_kernel_kind_name(i).decode() for i in range(self.lib.gco_num_kernel_kinds())]

    def get_timing(self):
        out = {}
        for i, name in enumerate(self.kernel_kind_names()):
            ln, ms, by = C.c_int64(), C.c_double(), C.c_double()
            self._check(self.lib.gco_get_timing(self.h, i, C.byref(ln), C.byref(ms), C.byref(by)))
            out[name] = {"launches": ln.value, "total_ms": ms.value, "bytes_per_launch": by.value}
        return out

    def reset_timing(self):
        self._check(self.lib.gco_reset_timing(self.h))

"""ctypes loader for the C oracle (oracle/nt_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import this.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nt_oracle.c")
_LIB = os.path.join(_HERE, "libnt_oracle.so")


def build(force: bool = True) -> str:
    """Compile the oracle with gcc.  AVX2 is used when the host has it."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    flags = ["-O3", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-Wall"]
    try:
        with open("/proc/cpuinfo") as f:
            info = f.read()
        if " avx2 " in info and " fma " in info:
            flags += ["-mavx2", "-mfma"]
    except OSError:
        pass
    tmp = _LIB + f".tmp{os.getpid()}"
    subprocess.check_call(["gcc", *flags, "-o", tmp, _SRC, "-lm"])
    os.replace(tmp, _LIB)
    return _LIB


class _Cfg(C.Structure):
    _fields_ = [(k, C.c_int32) for k in ("n_enc", "n_dec", "d_model", "n_heads", "d_ffn", "vocab",
                                         "max_len", "rpr_clip", "tie_output", "bos_id",
                                         "dec_n_heads", "dec_d_ffn", "ln_l1", "q8_output")] + [("ln_eps", C.c_double)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        L = C.CDLL(_LIB)
        p, i32, i64, dbl = C.c_void_p, C.c_int32, C.c_int64, C.c_double
        L.ora_param_count.restype = i64
        L.ora_param_count.argtypes = [C.POINTER(_Cfg)]
        L.ora_half_to_float.restype = C.c_float
        L.ora_half_to_float.argtypes = [C.c_uint16]
        L.ora_n_steps.restype = i32
        L.ora_n_steps.argtypes = [i32]
        L.ora_load.restype = p
        L.ora_load.argtypes = [C.POINTER(_Cfg), p, i64]
        L.ora_free.restype = None
        L.ora_free.argtypes = [p]
        L.ora_pe.restype = None
        L.ora_pe.argtypes = [i32, i32, p]
        L.ora_layer_norm.restype = None
        L.ora_layer_norm.argtypes = [p, p, p, i32, dbl, p]
        L.ora_layer_norm_l1.restype = None
        L.ora_layer_norm_l1.argtypes = [p, p, p, i32, dbl, p]
        L.ora_linear.restype = None
        L.ora_linear.argtypes = [p, p, p, i32, i32, p]
        L.ora_softmax.restype = None
        L.ora_softmax.argtypes = [p, i32]
        L.ora_attend.restype = None
        L.ora_attend.argtypes = [p, p, p, i32, i32, i32, p, i32, i32, p, p]
        L.ora_encode.restype = i32
        L.ora_encode.argtypes = [p, p, i32, p]
        L.ora_greedy.restype = i32
        L.ora_greedy.argtypes = [p, p, i32, i32, p, p]
        L.ora_greedy_eos.restype = i32
        L.ora_greedy_eos.argtypes = [p, p, i32, i32, i32, p, p]
        L.ora_translate_eos.restype = i32
        L.ora_translate_eos.argtypes = [p, p, p, i64, i32, i32, p, p, p, i32]
        L.ora_q8_weight_row.restype = None
        L.ora_q8_weight_row.argtypes = [p, i32, p, p, p]
        L.ora_q8_activation_row.restype = None
        L.ora_q8_activation_row.argtypes = [p, i32, p, p, p]
        L.ora_q8_output_layer.restype = i32
        L.ora_q8_output_layer.argtypes = [p, p, i32, p, p]
        L.ora_q8_weights.restype = i32
        L.ora_q8_weights.argtypes = [p, i32, p, p, p]
        L.ora_teacher_forced.restype = i32
        L.ora_teacher_forced.argtypes = [p, p, i32, p, i32, p]
        L.ora_translate.restype = i32
        L.ora_translate.argtypes = [p, p, p, i64, p, p, i32]
        _lib = L
    return _lib


def _cfg(cfg: dict) -> _Cfg:
    c = _Cfg()
    for k, _ in _Cfg._fields_:
        setattr(c, k, cfg.get(k, 0) if k.startswith("dec_") or k in ("ln_l1", "q8_output") else cfg[k])
    return c


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def param_count(cfg: dict) -> int:
    c = _cfg(cfg)
    return int(lib().ora_param_count(C.byref(c)))


def n_steps(length: int) -> int:
    return int(lib().ora_n_steps(int(length)))


# ---- primitives ----
def pe(pos: int, d: int) -> np.ndarray:
    out = np.empty(d)
    lib().ora_pe(pos, d, _ptr(out))
    return out


def layer_norm(x, g, b, eps) -> np.ndarray:
    x, g, b = _f64(x), _f32(g), _f32(b)
    y = np.empty_like(x)
    lib().ora_layer_norm(_ptr(x), _ptr(g), _ptr(b), x.size, eps, _ptr(y))
    return y


def layer_norm_l1(x, g, b, eps) -> np.ndarray:
    x, g, b = _f64(x), _f32(g), _f32(b)
    y = np.empty_like(x)
    lib().ora_layer_norm_l1(_ptr(x), _ptr(g), _ptr(b), x.size, eps, _ptr(y))
    return y


def linear(x, W, b) -> np.ndarray:
    x, W = _f64(x), _f32(W)
    y = np.empty(W.shape[1])
    bb = _f32(b) if b is not None else None
    lib().ora_linear(_ptr(x), _ptr(W), _ptr(bb) if bb is not None else None, W.shape[0], W.shape[1], _ptr(y))
    return y


def softmax(s) -> np.ndarray:
    s = _f64(s).copy()
    lib().ora_softmax(_ptr(s), s.size)
    return s


def attend(q, K, V, heads=1, rk=None, clip=0, qpos=0):
    """Returns (context [d], probs [heads, n_keys])."""
    q, K, V = _f64(q), _f64(K), _f64(V)
    n, d = K.shape
    c = np.empty(d)
    probs = np.empty((heads, n))
    r = _f32(rk) if rk is not None else None
    lib().ora_attend(_ptr(q), _ptr(K), _ptr(V), n, d, heads, _ptr(r) if r is not None else None, clip, qpos,
                     _ptr(c), _ptr(probs))
    return c, probs


def q8_weight_row(w):
    """Eq. 3, 4 for one vocabulary entry: (codes int8 [d], scale float32, zero point int)."""
    w = _f32(w)
    q = np.empty(w.size, dtype=np.int8)
    sc, z = C.c_float(), C.c_int32()
    lib().ora_q8_weight_row(_ptr(w), w.size, _ptr(q), C.byref(sc), C.byref(z))
    return q, np.float32(sc.value), int(z.value)


def q8_activation_row(h):
    """Eq. 5, 6 for one row, in fp32: (codes uint8 [d], scale float32, zero point int)."""
    h = _f32(h)
    u = np.empty(h.size, dtype=np.uint8)
    sc, z = C.c_float(), C.c_int32()
    lib().ora_q8_activation_row(_ptr(h), h.size, _ptr(u), C.byref(sc), C.byref(z))
    return u, np.float32(sc.value), int(z.value)


class Model:
    def __init__(self, cfg: dict, blob: np.ndarray):
        assert blob.dtype == np.float16
        self.cfg = dict(cfg)
        blob = np.ascontiguousarray(blob)
        c = _cfg(cfg)
        self._h = lib().ora_load(C.byref(c), _ptr(blob), blob.size)
        if not self._h:
            raise ValueError("oracle: bad config or blob size")

    def close(self):
        if self._h:
            lib().ora_free(self._h)
            self._h = None

    def __del__(self):
        self.close()

    def encode(self, src) -> np.ndarray:
        src = _i32(src)
        out = np.empty((src.size, self.cfg["d_model"]))
        if lib().ora_encode(self._h, _ptr(src), src.size, _ptr(out)):
            raise ValueError("oracle: invalid source sentence")
        return out

    def greedy(self, src, steps: int | None = None):
        """Returns (tokens [steps] int32, margins [steps] = top-1 minus top-2 logit)."""
        src = _i32(src)
        steps = n_steps(src.size) if steps is None else steps
        out = np.empty(steps, dtype=np.int32)
        margin = np.empty(steps)
        rc = lib().ora_greedy(self._h, _ptr(src), src.size, steps, _ptr(out), _ptr(margin))
        if rc:
            raise ValueError(f"oracle: greedy failed ({rc})")
        return out, margin

    def greedy_eos(self, src, eos_id: int, max_steps: int | None = None):
        """EOS-terminated greedy search: (tokens [n] int32 ending with EOS unless the cap cut it, margins [n])."""
        src = _i32(src)
        cap = n_steps(src.size) if max_steps is None else max_steps
        out = np.empty(max(cap, 1), dtype=np.int32)
        margin = np.empty(max(cap, 1))
        n = lib().ora_greedy_eos(self._h, _ptr(src), src.size, cap, eos_id, _ptr(out), _ptr(margin))
        if n < 0:
            raise ValueError(f"oracle: greedy failed ({n})")
        return out[:n].copy(), margin[:n].copy()

    def q8_output_layer(self, h):
        """8-bit output layer on fp32 rows h [R, d]: (logits float32 [R, V], argmax int32 [R])."""
        h = np.ascontiguousarray(h, dtype=np.float32)
        R = h.shape[0]
        logits = np.empty((R, self.cfg["vocab"]), dtype=np.float32)
        am = np.empty(R, dtype=np.int32)
        if lib().ora_q8_output_layer(self._h, _ptr(h), R, _ptr(logits), _ptr(am)):
            raise ValueError("oracle: model has no 8-bit output layer")
        return logits, am

    def q8_weights(self, v: int):
        q = np.empty(self.cfg["d_model"], dtype=np.int8)
        sc, z = C.c_float(), C.c_int32()
        if lib().ora_q8_weights(self._h, v, _ptr(q), C.byref(sc), C.byref(z)):
            raise ValueError("oracle: no 8-bit weights")
        return q, np.float32(sc.value), int(z.value)

    def teacher_forced(self, src, tgt_in) -> np.ndarray:
        src, tgt_in = _i32(src), _i32(tgt_in)
        out = np.empty((tgt_in.size, self.cfg["vocab"]))
        if lib().ora_teacher_forced(self._h, _ptr(src), src.size, _ptr(tgt_in), tgt_in.size, _ptr(out)):
            raise ValueError("oracle: invalid input")
        return out

    def translate(self, tokens, offsets, n_threads: int = 0):
        """Returns (out tokens int32, out offsets int64, threads used)."""
        tokens = _i32(tokens)
        offsets = np.ascontiguousarray(offsets, dtype=np.int64)
        N = offsets.size - 1
        lens = np.diff(offsets)
        total = int(sum(n_steps(int(l)) for l in lens if l > 0))
        out = np.empty(max(total, 1), dtype=np.int32)
        oo = np.empty(N + 1, dtype=np.int64)
        used = lib().ora_translate(self._h, _ptr(tokens), _ptr(offsets), N, _ptr(out), _ptr(oo), n_threads)
        if used < 0:
            raise ValueError(f"oracle: translate failed ({used})")
        return out[:total], oo, used

    def translate_eos(self, tokens, offsets, eos_id: int, n_threads: int = 0):
        """EOS-terminated translate.  Returns (out int32 in the fixed-length layout, padded after each
        sentence's end; out offsets int64; out lengths int32; threads used)."""
        tokens = _i32(tokens)
        offsets = np.ascontiguousarray(offsets, dtype=np.int64)
        N = offsets.size - 1
        lens = np.diff(offsets)
        total = int(sum(n_steps(int(l)) for l in lens if l > 0))
        out = np.empty(max(total, 1), dtype=np.int32)
        oo = np.empty(N + 1, dtype=np.int64)
        ol = np.zeros(max(N, 1), dtype=np.int32)
        used = lib().ora_translate_eos(self._h, _ptr(tokens), _ptr(offsets), N, eos_id, self.cfg["pad_id"], _ptr(out),
                                       _ptr(oo), _ptr(ol), n_threads)
        if used < 0:
            raise ValueError(f"oracle: translate failed ({used})")
        return out[:total], oo, ol[:N], used

"""ctypes binding for libnt.so: argument marshalling only, same names as include/nt.h.

Device buffers are torch tensors (torch is used for device memory and streams only).  There is
no fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnt.so")

EXPORTS = ["nt_param_count", "nt_n_steps", "nt_load_weights", "nt_free", "nt_encode", "nt_decode_greedy",
           "nt_translate_batch", "nt_plan_batches", "nt_debug_encoder_out", "nt_debug_teacher_forced_logits",
           "nt_check_device_flags", "nt_device_bytes", "nt_last_error", "nt_debug_timing_enable",
           "nt_debug_timing_count", "nt_debug_timing_name", "nt_debug_timing_read", "nt_pipeline_lanes",
           "nt_pipeline_lane", "nt_lane_stream", "nt_decode_greedy_eos", "nt_translate_batch_eos",
           "nt_debug_q8_output_layer", "nt_debug_q8_quantize_row", "nt_output_slots", "nt_debug_set_vocab_tiled",
           "nt_debug_set_cert_distrust", "nt_q8_output_layer_static", "nt_debug_set_encoder_tails", "nt_debug_probe_peaks"]


class NtConfig(C.Structure):
    _fields_ = [("struct_size", C.c_uint32)] + [(k, C.c_int32) for k in (
        "n_enc", "n_dec", "d_model", "n_heads", "d_ffn", "vocab", "max_len", "rpr_clip", "tie_output", "bos_id",
        "pad_id")] + [("ln_eps", C.c_float), ("max_batch_rows", C.c_int32), ("max_batch_tokens", C.c_int64),
                                ("pipeline_lanes", C.c_int32), ("dec_n_heads", C.c_int32),
                                ("dec_d_ffn", C.c_int32), ("ln_l1", C.c_int32), ("q8_output", C.c_int32)]


class NtError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libnt error {code}: {msg}")
        self.code = code


_lib = None


def load_library() -> C.CDLL:
    """Load libnt.so and declare the signatures; raises if the library is not built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is not built: run python -m paper_2109_08003_amd.build")
    # torch ships its own HIP runtime (same soname); import it first so that libnt.so binds to
    # that copy instead of bringing a second runtime into the process
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    p, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    cfgp = C.POINTER(NtConfig)
    sig = {
        "nt_param_count": (i64, [cfgp]),
        "nt_n_steps": (i32, [i32]),
        "nt_load_weights": (C.c_int, [cfgp, p, C.c_size_t, p, C.POINTER(p)]),
        "nt_free": (None, [p]),
        "nt_encode": (C.c_int, [p, p, p, i32, i32, p]),
        "nt_decode_greedy": (C.c_int, [p, i32, i32, p, p, p]),
        "nt_translate_batch": (C.c_int, [p, p, p, i64, i64, i32, p, p, p]),
        "nt_decode_greedy_eos": (C.c_int, [p, i32, i32, p, i32, p, p, p]),
        "nt_debug_q8_output_layer": (C.c_int, [p, p, i32, p, p, p]),
        "nt_debug_q8_quantize_row": (C.c_int, [p, i32, p, p, p]),
        "nt_q8_output_layer_static": (C.c_int, [p, p, i32, p, p, p]),
        "nt_translate_batch_eos": (C.c_int, [p, p, p, i64, i64, i32, i32, p, p, p, p]),
        "nt_plan_batches": (C.c_int, [p, i64, i64, i32, p, p, C.POINTER(i64)]),
        "nt_output_slots": (C.c_int, [p, i64, C.POINTER(i64)]),
        "nt_debug_set_vocab_tiled": (C.c_int, [p, C.c_int]),
        "nt_debug_set_cert_distrust": (C.c_int, [p, C.c_int]),
        "nt_debug_set_encoder_tails": (C.c_int, [p, C.c_uint32]),
        "nt_debug_encoder_out": (C.c_int, [p, p, p]),
        "nt_debug_teacher_forced_logits": (C.c_int, [p, p, i32, i32, p, p]),
        "nt_check_device_flags": (C.c_int, [p, p]),
        "nt_device_bytes": (i64, [p]),
        "nt_last_error": (C.c_char_p, []),
        "nt_pipeline_lanes": (C.c_int, [p]),
        "nt_pipeline_lane": (p, [p, C.c_int]),
        "nt_lane_stream": (C.c_void_p, [p]),
        "nt_debug_timing_enable": (C.c_int, [p, C.c_uint64]),
        "nt_debug_probe_peaks": (C.c_int, [p] + [C.POINTER(C.c_double)] * 4 + [p]),
        "nt_debug_timing_count": (C.c_int, []),
        "nt_debug_timing_name": (C.c_char_p, [C.c_int]),
        "nt_debug_timing_read": (C.c_int, [p, C.c_int, C.POINTER(C.c_double), C.POINTER(i64), C.POINTER(C.c_double),
                                           C.POINTER(C.c_double), p]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    _lib = L
    return L


def lib() -> C.CDLL:
    return load_library()


def _check(rc: int):
    if rc != 0:
        raise NtError(rc, lib().nt_last_error().decode())


def make_config(cfg: dict, max_batch_tokens: int, max_batch_rows: int = 0, pipeline_lanes: int = 0) -> NtConfig:
    c = NtConfig()
    c.struct_size = C.sizeof(NtConfig)
    for k in ("n_enc", "n_dec", "d_model", "n_heads", "d_ffn", "vocab", "max_len", "rpr_clip", "tie_output", "bos_id",
              "pad_id"):
        setattr(c, k, int(cfg[k]))
    c.ln_eps = float(cfg["ln_eps"])
    c.max_batch_tokens = int(max_batch_tokens)
    c.max_batch_rows = int(max_batch_rows)
    c.pipeline_lanes = int(pipeline_lanes)
    c.dec_n_heads = int(cfg.get("dec_n_heads", 0))
    c.dec_d_ffn = int(cfg.get("dec_d_ffn", 0))
    c.ln_l1 = int(cfg.get("ln_l1", 0))
    c.q8_output = int(cfg.get("q8_output", 0))
    return c


def q8_quantize_row(w):
    """Weight side of the 8-bit output layer for one fp16 row (host only): (codes int8, scale float32, zero int)."""
    w = np.ascontiguousarray(w, dtype=np.float16)
    q = np.empty(w.size, dtype=np.int8)
    sc, z = C.c_float(), C.c_int32()
    _check(lib().nt_debug_q8_quantize_row(w.ctypes.data_as(C.c_void_p), w.size, q.ctypes.data_as(C.c_void_p),
                                          C.byref(sc), C.byref(z)))
    return q, np.float32(sc.value), int(z.value)


def param_count(cfg: dict) -> int:
    c = make_config(cfg, 1)
    return int(lib().nt_param_count(C.byref(c)))


def n_steps(length: int) -> int:
    return int(lib().nt_n_steps(int(length)))


def output_slots(offsets) -> int:
    """Number of output ids the translate calls write for these sentences (nt_output_slots)."""
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    total = C.c_int64(0)
    _check(lib().nt_output_slots(offsets.ctypes.data_as(C.c_void_p), offsets.size - 1, C.byref(total)))
    return int(total.value)


def plan_batches(lengths, budget: int, max_rows: int = 0):
    """Returns (order int64 [N], batch_starts int64 [n_batches+1])."""
    lengths = np.ascontiguousarray(lengths, dtype=np.int32)
    N = lengths.size
    order = np.empty(max(N, 1), dtype=np.int64)
    starts = np.empty(N + 1, dtype=np.int64)
    nb = C.c_int64(0)
    _check(lib().nt_plan_batches(lengths.ctypes.data_as(C.c_void_p), N, int(budget), int(max_rows),
                                 order.ctypes.data_as(C.c_void_p), starts.ctypes.data_as(C.c_void_p), C.byref(nb)))
    return order[:N], starts[: nb.value + 1]


def kernel_names() -> list:
    L = lib()
    return [L.nt_debug_timing_name(i).decode() for i in range(L.nt_debug_timing_count())]


def _stream_ptr(stream) -> int:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


class Model:
    """Owns one nt_model.  Methods mirror the C entry points."""

    def __init__(self, cfg: dict, blob: np.ndarray, max_batch_tokens: int, max_batch_rows: int = 0, stream=None,
                 pipeline_lanes: int = 0):
        assert blob.dtype == np.float16
        blob = np.ascontiguousarray(blob)
        self.cfg = dict(cfg)
        c = make_config(cfg, max_batch_tokens, max_batch_rows, pipeline_lanes)
        h = C.c_void_p()
        _check(lib().nt_load_weights(C.byref(c), blob.ctypes.data_as(C.c_void_p), blob.nbytes, _stream_ptr(stream),
                                     C.byref(h)))
        self._h = h

    def close(self):
        if getattr(self, "_h", None) and getattr(self, "_owner", None) is None:
            lib().nt_free(self._h)
        self._h = None

    def n_lanes(self) -> int:
        return int(lib().nt_pipeline_lanes(self._h))

    def lane(self, i: int) -> "Model":
        """Lane i as a Model that shares this model's weights (lane 0 is the model itself)."""
        if i == 0:
            return self
        h = lib().nt_pipeline_lane(self._h, i)
        if not h:
            raise IndexError(i)
        ln = object.__new__(Model)
        ln.cfg, ln._h, ln._owner = self.cfg, C.c_void_p(h), self   # the owner frees the lanes
        return ln

    def own_stream(self):
        """The lane's own HIP stream as a torch.cuda.ExternalStream (owned by the model)."""
        import torch
        ptr = lib().nt_lane_stream(self._h)
        if not ptr:
            raise RuntimeError("no lane stream")
        return torch.cuda.ExternalStream(int(ptr))

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def device_bytes(self) -> int:
        return int(lib().nt_device_bytes(self._h))

    def encode(self, d_src, d_len, stream=None):
        """d_src int32 cuda tensor [B,S], d_len int32 cuda tensor [B]."""
        B, S = d_src.shape
        assert d_src.is_cuda and d_len.is_cuda and d_src.is_contiguous() and d_len.is_contiguous()
        _check(lib().nt_encode(self._h, d_src.data_ptr(), d_len.data_ptr(), B, S, _stream_ptr(stream)))

    def decode_greedy(self, B: int, steps: int, d_out, row_steps=None, stream=None):
        """d_out int32 cuda tensor [B, steps]; row_steps optional host int32 array [B]."""
        assert d_out.is_cuda and d_out.is_contiguous() and d_out.numel() >= B * steps
        rs = None
        if row_steps is not None:
            rs = np.ascontiguousarray(row_steps, dtype=np.int32)
        _check(lib().nt_decode_greedy(self._h, B, steps, rs.ctypes.data_as(C.c_void_p) if rs is not None else None,
                                      d_out.data_ptr(), _stream_ptr(stream)))

    def decode_greedy_eos(self, B: int, steps: int, eos_id: int, d_out, d_out_len, row_steps=None, stream=None):
        """EOS-terminated greedy decoding: d_out int32 cuda [B, steps], d_out_len int32 cuda [B]."""
        assert d_out.is_cuda and d_out.is_contiguous() and d_out.numel() >= B * steps
        assert d_out_len.is_cuda and d_out_len.is_contiguous() and d_out_len.numel() >= B
        rs = None
        if row_steps is not None:
            rs = np.ascontiguousarray(row_steps, dtype=np.int32)
        _check(lib().nt_decode_greedy_eos(self._h, B, steps, rs.ctypes.data_as(C.c_void_p) if rs is not None else None,
                                          int(eos_id), d_out.data_ptr(), d_out_len.data_ptr(), _stream_ptr(stream)))

    def debug_q8_output_layer(self, d_h, d_argmax=None, d_logits=None, stream=None):
        """The 8-bit output layer alone on fp32 rows d_h [R, d] (cuda): arg-max int32 [R] and/or logits fp32 [R, V]."""
        assert d_h.is_cuda and d_h.is_contiguous()
        _check(lib().nt_debug_q8_output_layer(self._h, d_h.data_ptr(), d_h.shape[0],
                                              d_argmax.data_ptr() if d_argmax is not None else None,
                                              d_logits.data_ptr() if d_logits is not None else None, _stream_ptr(stream)))

    def q8_output_layer_static(self, d_h, d_argmax=None, d_logits=None, stream=None):
        """debug_q8_output_layer through the entry point that allocates nothing (at most NT_STATIC_MAX_ROWS rows)."""
        assert d_h.is_cuda and d_h.is_contiguous()
        _check(lib().nt_q8_output_layer_static(self._h, d_h.data_ptr(), d_h.shape[0],
                                               d_argmax.data_ptr() if d_argmax is not None else None,
                                               d_logits.data_ptr() if d_logits is not None else None, _stream_ptr(stream)))

    def debug_encoder_out(self, d_out, stream=None):
        _check(lib().nt_debug_encoder_out(self._h, d_out.data_ptr(), _stream_ptr(stream)))

    def debug_teacher_forced_logits(self, d_tgt_in, d_logits, stream=None):
        B, T = d_tgt_in.shape
        assert d_tgt_in.is_contiguous() and d_logits.is_contiguous()
        _check(lib().nt_debug_teacher_forced_logits(self._h, d_tgt_in.data_ptr(), B, T, d_logits.data_ptr(),
                                                    _stream_ptr(stream)))

    def debug_set_vocab_tiled(self, on: bool):
        _check(lib().nt_debug_set_vocab_tiled(self._h, int(bool(on))))

    def debug_set_cert_distrust(self, on: bool):
        _check(lib().nt_debug_set_cert_distrust(self._h, int(bool(on))))

    def debug_set_encoder_tails(self, mask: int):
        _check(lib().nt_debug_set_encoder_tails(self._h, int(mask)))

    def check_device_flags(self, stream=None):
        _check(lib().nt_check_device_flags(self._h, _stream_ptr(stream)))

    def probe_peaks(self, stream=None) -> dict:
        """Measured peaks of this GPU (nt_debug_probe_peaks): fp16 MFMA rate on changing random operands and on
        constant operands (TFLOP/s), streaming read and in-place copy (GB/s, the copy counting bytes read + written)."""
        a, c, b, d = C.c_double(), C.c_double(), C.c_double(), C.c_double()
        _check(lib().nt_debug_probe_peaks(self._h, C.byref(a), C.byref(c), C.byref(b), C.byref(d), _stream_ptr(stream)))
        return {"mfma_f16_tflops": a.value, "mfma_f16_tflops_constant_operands": c.value, "hbm_read_gbs": b.value,
                "hbm_copy_gbs": d.value}

    def timing_enable(self, kernels="all"):
        """kernels: "all", None/() to switch off, or an iterable of family names."""
        names = kernel_names()
        if kernels == "all":
            mask = (1 << len(names)) - 1
        else:
            mask = 0
            for k in kernels or ():
                mask |= 1 << names.index(k)
        _check(lib().nt_debug_timing_enable(self._h, mask))

    def timing_read(self, stream=None) -> dict:
        """name -> dict(ms, launches, bytes, flops) for every family with at least one launch."""
        res = {}
        for i, name in enumerate(kernel_names()):
            ms, n, by, fl = C.c_double(), C.c_int64(), C.c_double(), C.c_double()
            _check(lib().nt_debug_timing_read(self._h, i, C.byref(ms), C.byref(n), C.byref(by), C.byref(fl),
                                              _stream_ptr(stream)))
            if n.value:
                res[name] = dict(ms=ms.value, launches=n.value, bytes=by.value, flops=fl.value)
        return res

    def translate_batch(self, tokens, offsets, token_budget: int, max_rows: int = 0, stream=None):
        """Host arrays in, host arrays out: returns (out int32, out_offsets int64)."""
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        offsets = np.ascontiguousarray(offsets, dtype=np.int64)
        N = offsets.size - 1
        total = output_slots(offsets) if N > 0 else 0
        out = np.empty(max(total, 1), dtype=np.int32)
        oo = np.empty(N + 1, dtype=np.int64)
        _check(lib().nt_translate_batch(self._h, tokens.ctypes.data_as(C.c_void_p), offsets.ctypes.data_as(C.c_void_p),
                                        N, int(token_budget), int(max_rows), out.ctypes.data_as(C.c_void_p),
                                        oo.ctypes.data_as(C.c_void_p), _stream_ptr(stream)))
        return out[:total], oo

    def translate_batch_eos(self, tokens, offsets, token_budget: int, eos_id: int, max_rows: int = 0, stream=None):
        """EOS-terminated translate: returns (out int32 in the fixed-length slots, padded after each sentence's
        end; out_offsets int64; out_len int32)."""
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        offsets = np.ascontiguousarray(offsets, dtype=np.int64)
        N = offsets.size - 1
        total = output_slots(offsets) if N > 0 else 0
        out = np.empty(max(total, 1), dtype=np.int32)
        oo = np.empty(N + 1, dtype=np.int64)
        ol = np.zeros(max(N, 1), dtype=np.int32)
        _check(lib().nt_translate_batch_eos(self._h, tokens.ctypes.data_as(C.c_void_p),
                                            offsets.ctypes.data_as(C.c_void_p), N, int(token_budget), int(max_rows),
                                            int(eos_id), out.ctypes.data_as(C.c_void_p), oo.ctypes.data_as(C.c_void_p),
                                            ol.ctypes.data_as(C.c_void_p), _stream_ptr(stream)))
        return out[:total], oo, ol[:N]

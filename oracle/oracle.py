"""ctypes front end of the CPU oracle (oracle/specbound_oracle.c).

TEST INFRASTRUCTURE ONLY.  Argument marshalling; all arithmetic is in the C file.
"""
import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

from . import build as _build

EXITED, WIDTH_BOUND, DEPTH_BOUND = 1, 2, 3
PH_DRAFT, PH_ALIGN, PH_VERIFY, PH_PREFILL = 0, 1, 2, 3
MAX_W = 16

_libs: Dict[int, C.CDLL] = {}


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads",
                                          "head_dim", "d_ffn", "vocab")] + \
               [("rms_eps", C.c_float), ("rope_base", C.c_float)] + \
               [(n, C.c_int32) for n in ("weight_dtype", "kv_dtype", "n_exit_heads", "max_seq")]


class _Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("attn_norm", C.POINTER(C.c_void_p)), ("w_qkv", C.POINTER(C.c_void_p)),
                ("w_o", C.POINTER(C.c_void_p)), ("ffn_norm", C.POINTER(C.c_void_p)),
                ("w_gate_up", C.POINTER(C.c_void_p)), ("w_down", C.POINTER(C.c_void_p)),
                ("exit_norm", C.POINTER(C.c_void_p)), ("exit_head", C.POINTER(C.c_void_p))]


class _Params(C.Structure):
    _fields_ = [("d_max", C.c_int32), ("w_max", C.c_int32), ("T", C.POINTER(C.c_float)),
                ("threshold", C.c_float), ("eos_id", C.c_int32),
                ("forced_exit", C.POINTER(C.c_int32)), ("forced_draft", C.POINTER(C.c_int32)),
                ("n_forced", C.c_int64), ("head_mask", C.c_uint32),
                ("sample_temperature", C.c_float), ("top_p", C.c_float),
                ("sample_u", C.POINTER(C.c_float)), ("n_sample_u", C.c_int64)]


class _DraftResult(C.Structure):
    _fields_ = [("token", C.c_int32), ("exit_layer", C.c_int32), ("status", C.c_int32),
                ("confidence", C.c_float)]


class _VerifyResult(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_rows", "n_drafts", "n_matched", "n_emit",
                                          "align_layer")] + [("tokens", C.c_int32 * MAX_W)]


class _TraceEntry(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("phase", "layer", "first_slot", "n_rows")]


class _Stats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("rounds", "draft_steps", "drafts", "emitted",
                                          "layer_sweeps", "row_layers", "head_evals",
                                          "final_head_rows")] + \
               [("accept_hist", C.c_int64 * (MAX_W + 1)), ("exit_hist", C.c_int64 * 65)]


def load_lib(bits: int = 64) -> C.CDLL:
    if bits not in _libs:
        path = _build.lib_path(bits)
        if not os.path.exists(path):
            _build.build(force=False)
        lib = C.CDLL(path)
        assert lib.orc_real_bytes() == bits // 8
        lib.orc_round_time.restype = C.c_double
        lib.orc_expected_accept.restype = C.c_double
        lib.orc_speedup.restype = C.c_double
        lib.orc_round_time.argtypes = [C.c_int32] * 3
        lib.orc_expected_accept.argtypes = [C.c_double, C.c_int32]
        lib.orc_speedup.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_double]
        lib.orc_temperature_schedule.argtypes = [C.c_double, C.c_int32, C.c_int32, C.c_void_p]
        lib.orc_trace_read.restype = C.c_int64
        lib.orc_trace_read.argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
        lib.orc_trace_enable.argtypes = [C.c_void_p, C.c_int64]
        for name in ("orc_session_free", "orc_model_free", "orc_session_reset"):
            getattr(lib, name).restype = None
            getattr(lib, name).argtypes = [C.c_void_p]
        _libs[bits] = lib
    return _libs[bits]


def num_threads() -> int:
    return load_lib(64).orc_num_threads()


def _real(bits: int):
    return np.float64 if bits == 64 else np.float32


def _ptr(a: np.ndarray) -> C.c_void_p:
    return C.c_void_p(a.ctypes.data)


# ------------------------------------------------------------------ primitives

def matvec(W: np.ndarray, x: np.ndarray, bits: int = 64) -> np.ndarray:
    """W is float32 or uint16 (bf16 bits), [N, K]."""
    lib = load_lib(bits)
    W = np.ascontiguousarray(W)
    dtype = 1 if W.dtype == np.uint16 else 0
    assert W.dtype in (np.uint16, np.float32)
    x = np.ascontiguousarray(x, dtype=_real(bits))
    N, K = W.shape
    assert x.shape == (K,)
    y = np.empty(N, dtype=_real(bits))
    lib.orc_matvec(_ptr(W), C.c_int32(dtype), C.c_int32(N), C.c_int32(K), _ptr(x), _ptr(y))
    return y


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float, bits: int = 64) -> np.ndarray:
    lib = load_lib(bits)
    x = np.ascontiguousarray(x, dtype=_real(bits))
    g = np.ascontiguousarray(g, dtype=np.float32)
    out = np.empty_like(x)
    lib.orc_rmsnorm(_ptr(x), _ptr(g), C.c_int32(x.size), C.c_float(eps), _ptr(out))
    return out


def swiglu(gu: np.ndarray, bits: int = 64) -> np.ndarray:
    """gu = f gate values, then f up values -> silu(gate) * up."""
    lib = load_lib(bits)
    gu = np.ascontiguousarray(gu, dtype=_real(bits))
    f = gu.size // 2
    out = np.empty(f, dtype=_real(bits))
    lib.orc_swiglu(_ptr(gu), C.c_int32(f), _ptr(out))
    return out


def act(z: np.ndarray, T: float, bits: int = 64):
    """(argmax, confidence) of Eq. 2."""
    lib = load_lib(bits)
    z = np.ascontiguousarray(z, dtype=_real(bits))
    am = C.c_int32()
    conf = (C.c_double if bits == 64 else C.c_float)()
    Tc = (C.c_double if bits == 64 else C.c_float)(T)
    lib.orc_act(_ptr(z), C.c_int32(z.size), Tc, C.byref(am), C.byref(conf))
    return am.value, conf.value


def sample_dist(z: np.ndarray, temp: float, top_p: float = 1.0, bits: int = 64) -> np.ndarray:
    """The distribution sampling-mode decoding draws from (temperature, top-p nucleus)."""
    lib = load_lib(bits)
    z = np.ascontiguousarray(z, dtype=_real(bits))
    p = np.empty_like(z)
    tmp = np.empty_like(z)
    R = C.c_double if bits == 64 else C.c_float
    lib.orc_sample_dist(_ptr(z), C.c_int32(z.size), R(temp), R(top_p), _ptr(p), _ptr(tmp))
    return p


def sample_token(p: np.ndarray, u: float, exclude: int = -1, bits: int = 64) -> int:
    lib = load_lib(bits)
    p = np.ascontiguousarray(p, dtype=_real(bits))
    R = C.c_double if bits == 64 else C.c_float
    return lib.orc_sample_token(_ptr(p), C.c_int32(p.size), R(u), C.c_int32(exclude))


def rope_angles(pos: int, hd: int, base: float):
    lib = load_lib(64)
    c = np.empty(hd // 2, dtype=np.float32)
    s = np.empty(hd // 2, dtype=np.float32)
    lib.orc_rope_angles(C.c_int32(pos), C.c_int32(hd), C.c_float(base), _ptr(c), _ptr(s))
    return c, s


def rope_apply(v: np.ndarray, pos: int, base: float, bits: int = 64) -> np.ndarray:
    lib = load_lib(bits)
    v = np.array(v, dtype=_real(bits))
    c, s = rope_angles(pos, v.size, base)
    lib.orc_rope_apply(_ptr(v), C.c_int32(v.size), _ptr(c), _ptr(s))
    return v


def attention_head(q: np.ndarray, K: np.ndarray, V: np.ndarray, bits: int = 64) -> np.ndarray:
    """q [hd]; K, V float32 [n_keys, hd] (contiguous)."""
    lib = load_lib(bits)
    q = np.ascontiguousarray(q, dtype=_real(bits))
    K = np.ascontiguousarray(K, dtype=np.float32)
    V = np.ascontiguousarray(V, dtype=np.float32)
    n, hd = K.shape
    sc = np.empty(n, dtype=_real(bits))
    out = np.empty(hd, dtype=_real(bits))
    lib.orc_attention_head(_ptr(q), _ptr(K), _ptr(V), C.c_int32(n), C.c_int32(hd),
                           C.c_size_t(hd), _ptr(sc), _ptr(out))
    return out


def temperature_schedule(alpha: float, L: int, n: int) -> np.ndarray:
    T = np.empty(n, dtype=np.float32)
    load_lib(64).orc_temperature_schedule(alpha, L, n, _ptr(T))
    return T


def expected_accept(a: float, w: int) -> float:
    return load_lib(64).orc_expected_accept(a, w)


def round_time(L: int, d_max: int, w: int) -> float:
    return load_lib(64).orc_round_time(L, d_max, w)


def speedup(L: int, d_max: int, w: int, a: float) -> float:
    return load_lib(64).orc_speedup(L, d_max, w, a)


# ------------------------------------------------------------------ model / session

class OrcParams:
    """Speculation parameters; keeps the numpy arrays alive."""

    def __init__(self, d_max: int, w_max: int, T: Sequence[float], threshold: float,
                 forced_exit: Optional[Sequence[int]] = None,
                 forced_draft: Optional[Sequence[int]] = None, eos_id: int = -1, head_mask: int = 0,
                 sample_temperature: float = 0.0, top_p: float = 1.0, sample_u=None):
        self.T = np.ascontiguousarray(T, dtype=np.float32)
        assert len(self.T) >= d_max
        self.su = None if sample_u is None else np.ascontiguousarray(sample_u, dtype=np.float32)
        self.fe = None if forced_exit is None else np.ascontiguousarray(forced_exit, dtype=np.int32)
        self.fd = None if forced_draft is None else np.ascontiguousarray(forced_draft, dtype=np.int32)
        n_forced = 0
        if self.fe is not None:
            n_forced = len(self.fe)
        if self.fd is not None:
            n_forced = len(self.fd) if self.fe is None else min(n_forced, len(self.fd))
        self.c = _Params(d_max, w_max,
                         self.T.ctypes.data_as(C.POINTER(C.c_float)), threshold, eos_id,
                         None if self.fe is None else self.fe.ctypes.data_as(C.POINTER(C.c_int32)),
                         None if self.fd is None else self.fd.ctypes.data_as(C.POINTER(C.c_int32)),
                         n_forced, head_mask, sample_temperature, top_p,
                         None if self.su is None else self.su.ctypes.data_as(C.POINTER(C.c_float)),
                         0 if self.su is None else len(self.su))


class Oracle:
    """A model: config + borrowed weight arrays (numpy, kept alive here)."""

    def __init__(self, shape, weights: Dict[str, np.ndarray], max_seq: int, bits: int = 64):
        self.bits = bits
        self.lib = load_lib(bits)
        self.shape = shape
        self.max_seq = max_seq
        self.weights = {k: np.ascontiguousarray(v) for k, v in weights.items()}
        w = self.weights
        L, E = shape.n_layers, shape.n_exit_heads
        want = np.uint16 if shape.weight_dtype == 1 else np.float32
        for k, v in w.items():
            if "norm" in k:
                assert v.dtype == np.float32, k
            else:
                assert v.dtype == want, (k, v.dtype)

        def arr(prefix, n):
            a = (C.c_void_p * max(n, 1))()
            for i in range(n):
                a[i] = w[f"{prefix}.{i}"].ctypes.data
            return a

        self._arrs = [arr(p, L) for p in ("attn_norm", "w_qkv", "w_o", "ffn_norm", "w_gate_up", "w_down")]
        self._arrs += [arr("exit_norm", E), arr("exit_head", E)]
        self.cw = _Weights(w["embed"].ctypes.data, w["lm_head"].ctypes.data, w["final_norm"].ctypes.data,
                           *[C.cast(a, C.POINTER(C.c_void_p)) for a in self._arrs])
        self.cfg = _Config(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads,
                           shape.head_dim, shape.d_ffn, shape.vocab, shape.rms_eps, shape.rope_base,
                           shape.weight_dtype, shape.kv_dtype, shape.n_exit_heads, max_seq)
        self.h = C.c_void_p()
        rc = self.lib.orc_model_new(C.byref(self.cfg), C.byref(self.cw), C.byref(self.h))
        if rc != 0:
            raise RuntimeError(f"orc_model_new failed: {rc}")

    def session(self) -> "OracleSession":
        return OracleSession(self)

    def greedy_nocache(self, prompt: Sequence[int], max_new: int, want_logits: bool = False):
        prompt = np.ascontiguousarray(prompt, dtype=np.int32)
        out = np.empty(max_new, dtype=np.int32)
        logits = np.empty(self.shape.vocab, dtype=np.float64) if want_logits else None
        rc = self.lib.orc_greedy_nocache(self.h, _ptr(prompt), C.c_int32(len(prompt)),
                                         C.c_int32(max_new), _ptr(out),
                                         _ptr(logits) if want_logits else None)
        if rc != 0:
            raise RuntimeError(f"orc_greedy_nocache failed: {rc}")
        return (out, logits) if want_logits else out

    def __del__(self):
        try:
            self.lib.orc_model_free(self.h)
        except Exception:
            pass


class OracleSession:
    def __init__(self, model: Oracle):
        self.model = model
        self.lib = model.lib
        self.h = C.c_void_p()
        rc = self.lib.orc_session_new(model.h, C.byref(self.h))
        if rc != 0:
            raise RuntimeError(f"orc_session_new failed: {rc}")

    def __del__(self):
        try:
            self.lib.orc_session_free(self.h)
        except Exception:
            pass

    # --- calls mirroring the algorithm
    def prefill(self, prompt) -> int:
        prompt = np.ascontiguousarray(prompt, dtype=np.int32)
        t = C.c_int32()
        rc = self.lib.orc_prefill(self.h, _ptr(prompt), C.c_int32(len(prompt)), C.byref(t))
        if rc != 0:
            raise RuntimeError(f"orc_prefill failed: {rc}")
        return t.value

    def draft_step(self, p: OrcParams, check: bool = True):
        r = _DraftResult()
        rc = self.lib.orc_draft_step(self.h, C.byref(p.c), C.byref(r))
        if rc != 0:
            if check:
                raise RuntimeError(f"orc_draft_step failed: {rc}")
            return rc
        return dict(token=r.token, exit_layer=r.exit_layer, status=r.status, confidence=r.confidence)

    def verify(self, p: OrcParams, check: bool = True):
        r = _VerifyResult()
        rc = self.lib.orc_verify(self.h, C.byref(p.c), C.byref(r))
        if rc != 0:
            if check:
                raise RuntimeError(f"orc_verify failed: {rc}")
            return rc
        return dict(n_rows=r.n_rows, n_drafts=r.n_drafts, n_matched=r.n_matched, n_emit=r.n_emit,
                    align_layer=r.align_layer, tokens=list(r.tokens)[:r.n_rows])

    def generate(self, prompt, max_new: int, p: OrcParams) -> np.ndarray:
        prompt = np.ascontiguousarray(prompt, dtype=np.int32)
        out = np.empty(max_new, dtype=np.int32)
        n = C.c_int32()
        rc = self.lib.orc_generate(self.h, _ptr(prompt), C.c_int32(len(prompt)), C.c_int32(max_new),
                                   C.byref(p.c), _ptr(out), C.c_int32(max_new), C.byref(n))
        if rc != 0:
            raise RuntimeError(f"orc_generate failed: {rc}")
        return out[:n.value].copy()

    def step(self, tok: int, want_logits: bool = True):
        """Teacher-forced step: feed tok at the next position; returns (argmax, logits)."""
        logits = np.empty(self.model.shape.vocab, dtype=np.float64) if want_logits else None
        am = C.c_int32()
        rc = self.lib.orc_step(self.h, C.c_int32(int(tok)), _ptr(logits) if want_logits else None,
                               C.byref(am))
        if rc != 0:
            raise RuntimeError(f"orc_step failed: {rc}")
        return am.value, logits

    # --- taps
    def set_eager_align(self, on: bool):
        self.lib.orc_set_eager_align(self.h, C.c_int32(int(on)))

    def trace_enable(self, cap: int = 1 << 16):
        self.lib.orc_trace_enable(self.h, cap)

    def trace(self) -> List[tuple]:
        cap = 1 << 16
        buf = (_TraceEntry * cap)()
        n = self.lib.orc_trace_read(self.h, buf, cap)
        return [(buf[i].phase, buf[i].layer, buf[i].first_slot, buf[i].n_rows) for i in range(min(n, cap))]

    def stats(self) -> dict:
        st = _Stats()
        self.lib.orc_get_stats(self.h, C.byref(st))
        d = {n: getattr(st, n) for n, _ in _Stats._fields_[:8]}
        d["accept_hist"] = list(st.accept_hist)
        d["exit_hist"] = list(st.exit_hist)
        return d

    def committed_len(self) -> int:
        return self.lib.orc_committed_len(self.h)

    def open_slots(self) -> int:
        return self.lib.orc_open_slots(self.h)

    def slot_reached(self, i: int) -> int:
        return self.lib.orc_slot_reached(self.h, C.c_int32(i))

    def slot_hidden(self, i: int) -> np.ndarray:
        out = np.empty(self.model.shape.d_model, dtype=np.float64)
        self.lib.orc_slot_hidden(self.h, C.c_int32(i), _ptr(out))
        return out

    def head_logits(self) -> np.ndarray:
        out = np.empty(self.model.shape.vocab, dtype=np.float64)
        self.lib.orc_head_logits(self.h, _ptr(out))
        return out

    def verify_logits(self, row: int) -> np.ndarray:
        out = np.empty(self.model.shape.vocab, dtype=np.float64)
        self.lib.orc_verify_logits(self.h, C.c_int32(row), _ptr(out))
        return out

    def verify_dist(self, row: int) -> np.ndarray:
        out = np.empty(self.model.shape.vocab, dtype=np.float64)
        self.lib.orc_verify_dist(self.h, C.c_int32(row), _ptr(out))
        return out

    def rewind(self, n_keep: int, pending: int):
        rc = self.lib.orc_rewind(self.h, C.c_int32(n_keep), C.c_int32(pending))
        if rc != 0:
            raise RuntimeError(f"orc_rewind failed: {rc}")

    def kv_read(self, layer: int, pos: int):
        s = self.model.shape
        k = np.empty(s.n_kv_heads * s.head_dim, dtype=np.float32)
        v = np.empty_like(k)
        self.lib.orc_kv_read(self.h, C.c_int32(layer), C.c_int32(pos), _ptr(k), _ptr(v))
        return k, v

"""Thin ctypes binding of libspecbound.so (include/specbound.h).

Argument marshalling only: every step of the decode path runs in the library's
HIP kernels.  PyTorch is used for device memory and the stream handle.  There is
no fallback: if the shared library is missing, importing this module fails.
"""
import ctypes as C
import os
from typing import Dict, Optional, Sequence

import numpy as np

from . import build as _build

SB_MAX_W = 8
SB_KV_BLOCK = 16
SB_MAX_EXIT_LAYERS = 64
OK, EINVAL, ENOMEM, ECAPACITY, ESTATE, EDEVICE = 0, -1, -2, -3, -4, -5
FP32, BF16 = 0, 1
EXITED, WIDTH_BOUND, DEPTH_BOUND = 1, 2, 3
PROJ_AUTO, PROJ_VALU, PROJ_MFMA, PROJ_MFMA_PACKED = 0, 1, 2, 3


class SbError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libspecbound error {code}: {msg}")
        self.code = code


class sb_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim",
                                          "d_ffn", "vocab")] + \
               [("rms_eps", C.c_float), ("rope_base", C.c_float)] + \
               [(n, C.c_int32) for n in ("weight_dtype", "kv_dtype", "n_exit_heads", "max_seq",
                                          "proj_kernel", "kv_block", "max_w")]


class sb_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p),
                ("attn_norm", C.POINTER(C.c_void_p)), ("w_qkv", C.POINTER(C.c_void_p)),
                ("w_o", C.POINTER(C.c_void_p)), ("ffn_norm", C.POINTER(C.c_void_p)),
                ("w_gate_up", C.POINTER(C.c_void_p)), ("w_down", C.POINTER(C.c_void_p)),
                ("exit_norm", C.POINTER(C.c_void_p)), ("exit_head", C.POINTER(C.c_void_p)),
                ("packed", C.c_void_p), ("packed_bytes", C.c_size_t)]


class sb_params(C.Structure):
    _fields_ = [("d_max", C.c_int32), ("w_max", C.c_int32), ("T", C.POINTER(C.c_float)),
                ("threshold", C.c_float), ("eos_id", C.c_int32),
                ("forced_exit", C.POINTER(C.c_int32)), ("forced_draft", C.POINTER(C.c_int32)),
                ("n_forced", C.c_int64), ("head_mask", C.c_uint32),
                ("sample_temperature", C.c_float), ("top_p", C.c_float),
                ("sample_u", C.POINTER(C.c_float)), ("n_sample_u", C.c_int64), ("exit_readback", C.c_int32)]


class sb_draft_result(C.Structure):
    _fields_ = [("token", C.c_int32), ("exit_layer", C.c_int32), ("status", C.c_int32),
                ("confidence", C.c_float)]


class sb_verify_result(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_rows", "n_drafts", "n_matched", "n_emit", "align_layer")] + \
               [("tokens", C.c_int32 * SB_MAX_W), ("accept_prob", C.c_float * SB_MAX_W)]


class sb_stats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("rounds", "draft_steps", "drafts", "emitted", "layer_sweeps",
                                          "row_layers", "head_evals", "final_head_sweeps")] + \
               [("accept_hist", C.c_int64 * (SB_MAX_W + 1)),
                ("exit_hist", C.c_int64 * (SB_MAX_EXIT_LAYERS + 1)),
                ("weight_bytes", C.c_int64), ("kv_bytes", C.c_int64),
                ("prefill_ms", C.c_double), ("decode_ms", C.c_double)] + \
               [(n, C.c_double) for n in ("host_draft_ms", "host_verify_ms", "host_wait_ms", "gpu_draft_ms",
                                          "gpu_align_ms", "gpu_verify_ms", "gpu_readback_ms")] + \
               [(n, C.c_int64) for n in ("draft_bytes", "align_bytes", "verify_bytes")]


class sb_sizes(C.Structure):
    _fields_ = [("kv_pool_bytes", C.c_size_t), ("workspace_bytes", C.c_size_t),
                ("packed_weight_bytes", C.c_size_t)]


# every symbol include/specbound.h declares
SYMBOLS = ["sb_last_error", "sb_temperature_schedule", "sb_query_sizes", "sb_load_model", "sb_free_model",
           "sb_new_session", "sb_free_session", "sb_prefill", "sb_draft_step", "sb_verify", "sb_generate",
           "sb_get_stats", "sb_committed_len", "sb_debug_enable", "sb_debug_logits", "sb_debug_hidden",
           "sb_debug_kv", "sb_op_rmsnorm", "sb_op_gemv", "sb_op_gemv_scratch_bytes", "sb_op_gate_up", "sb_op_head",
           "sb_op_head_scratch_bytes", "sb_rope_table_host", "sb_op_attention",
           "sb_op_attention_scratch_bytes", "sb_op_prompt_attention", "sb_decode", "sb_rewind", "sb_profile_begin", "sb_profile_end", "sb_op_copy",
           "sb_op_read", "sb_op_repack", "sb_op_gemm", "sb_op_gemm_scratch_bytes", "sb_op_head_static", "sb_phase_timing", "sb_debug_fail_launch", "sb_open_rows", "sb_new_batch", "sb_free_batch",
           "sb_batch_decode"]

KERNEL_CLASSES = ["rmsnorm", "qkv", "attention", "wo", "gate_up", "down", "exit_head",
                  "final_head"]

_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    """Load libspecbound.so (building it first only if no built library exists)."""
    global _lib
    if _lib is None:
        path = os.environ.get("SPECBOUND_LIB") or _build.lib_path()
        if not os.path.exists(path):
            _build.build()
        L = C.CDLL(path)
        vp, i32, f32, sz = C.c_void_p, C.c_int32, C.c_float, C.c_size_t
        L.sb_last_error.restype = C.c_char_p
        L.sb_last_error.argtypes = []
        L.sb_temperature_schedule.argtypes = [C.c_double, i32, i32, vp]
        L.sb_query_sizes.argtypes = [C.POINTER(sb_config), C.POINTER(sb_sizes)]
        L.sb_load_model.argtypes = [C.POINTER(sb_config), C.POINTER(sb_weights), vp, C.POINTER(vp)]
        L.sb_free_model.argtypes = [vp]
        L.sb_free_model.restype = None
        L.sb_new_session.argtypes = [vp, vp, sz, vp, sz, vp, C.POINTER(vp)]
        L.sb_free_session.argtypes = [vp]
        L.sb_free_session.restype = None
        L.sb_prefill.argtypes = [vp, vp, i32, C.POINTER(i32)]
        L.sb_draft_step.argtypes = [vp, C.POINTER(sb_params), C.POINTER(sb_draft_result)]
        L.sb_verify.argtypes = [vp, C.POINTER(sb_params), C.POINTER(sb_verify_result)]
        L.sb_generate.argtypes = [vp, vp, i32, i32, C.POINTER(sb_params), vp, i32, C.POINTER(i32),
                                  C.POINTER(sb_stats)]
        L.sb_decode.argtypes = [vp, i32, C.POINTER(sb_params), vp, i32, C.POINTER(i32), C.POINTER(sb_stats)]
        L.sb_rewind.argtypes = [vp, i32, i32, C.c_int64]
        L.sb_profile_begin.argtypes = [vp, C.c_uint32, i32, i32]
        L.sb_profile_end.argtypes = [vp, vp, vp, vp, C.POINTER(C.c_double)]
        L.sb_get_stats.argtypes = [vp, C.POINTER(sb_stats)]
        L.sb_phase_timing.argtypes = [vp, i32]
        L.sb_debug_fail_launch.argtypes = [vp, i32]
        L.sb_open_rows.argtypes = [vp]
        L.sb_new_batch.argtypes = [C.POINTER(vp), i32, C.POINTER(vp)]
        L.sb_free_batch.argtypes = [vp]
        L.sb_free_batch.restype = None
        L.sb_batch_decode.argtypes = [vp, i32, C.POINTER(C.POINTER(sb_params)), C.POINTER(vp), C.POINTER(i32)]
        L.sb_committed_len.argtypes = [vp]
        L.sb_debug_enable.argtypes = [vp, i32]
        L.sb_debug_logits.argtypes = [vp, i32, i32, vp, i32]
        L.sb_debug_hidden.argtypes = [vp, i32, vp, i32]
        L.sb_debug_kv.argtypes = [vp, i32, i32, vp, vp, i32]
        L.sb_op_rmsnorm.argtypes = [vp, vp, vp, i32, i32, f32, vp]
        L.sb_op_gemv.argtypes = [vp, i32, i32, i32, vp, vp, i32, i32, vp, vp]
        L.sb_op_gemv_scratch_bytes.argtypes = [i32, i32]
        L.sb_op_gate_up.argtypes = [vp, i32, i32, i32, vp, vp, i32, i32, vp, vp]
        L.sb_op_gemv_scratch_bytes.restype = sz
        L.sb_op_head.argtypes = [vp, i32, i32, i32, vp, i32, f32, i32, vp, vp, vp, vp, vp]
        L.sb_op_head_static.argtypes = [vp, i32, i32, i32, vp, i32, f32, i32, vp, vp, vp]
        L.sb_op_head_scratch_bytes.argtypes = [i32, i32, i32]
        L.sb_op_head_scratch_bytes.restype = sz
        L.sb_op_repack.argtypes = [vp, i32, i32, vp, vp]
        L.sb_op_gemm.argtypes = [vp, i32, i32, vp, vp, i32, vp, vp]
        L.sb_op_gemm_scratch_bytes.argtypes = [i32, i32]
        L.sb_op_gemm_scratch_bytes.restype = sz
        L.sb_op_copy.argtypes = [vp, vp, sz, vp]
        L.sb_op_read.argtypes = [vp, sz, vp, vp]
        L.sb_rope_table_host.argtypes = [i32, f32, i32, vp, vp]
        L.sb_op_attention.argtypes = [vp, i32, i32, i32, i32, vp, vp, i32, i32, vp, vp, i32, i32, vp, vp, vp]
        L.sb_op_attention_scratch_bytes.argtypes = [i32, i32, i32, i32]
        L.sb_op_prompt_attention.argtypes = [vp, i32, i32, i32, vp, vp, i32, i32, vp, vp, i32, i32, vp, vp]
        L.sb_op_attention_scratch_bytes.restype = sz
        _lib = L
    return _lib


def check(rc: int) -> None:
    if rc != 0:
        raise SbError(rc, lib().sb_last_error().decode())


def make_config(shape, max_seq: int, proj_kernel: int = PROJ_AUTO, max_w: int = 0) -> sb_config:
    """shape: any object with the fields of sb_config (e.g. sb_inputs.ModelShape)."""
    return sb_config(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim,
                     shape.d_ffn, shape.vocab, shape.rms_eps, shape.rope_base, shape.weight_dtype,
                     shape.kv_dtype, shape.n_exit_heads, max_seq, proj_kernel, SB_KV_BLOCK, max_w)


def query_sizes(cfg: sb_config):
    out = sb_sizes()
    check(lib().sb_query_sizes(C.byref(cfg), C.byref(out)))
    return out.kv_pool_bytes, out.workspace_bytes


def packed_weight_bytes(cfg: sb_config) -> int:
    out = sb_sizes()
    check(lib().sb_query_sizes(C.byref(cfg), C.byref(out)))
    return out.packed_weight_bytes


def temperature_schedule(alpha: float, L: int, n: int) -> np.ndarray:
    T = np.empty(n, dtype=np.float32)
    check(lib().sb_temperature_schedule(alpha, L, n, T.ctypes.data))
    return T


class Params:
    """sb_params with the host arrays kept alive."""

    def __init__(self, d_max: int, w_max: int, T: Sequence[float], threshold: float,
                 forced_exit: Optional[Sequence[int]] = None, forced_draft: Optional[Sequence[int]] = None,
                 eos_id: int = -1, head_mask: int = 0, sample_temperature: float = 0.0, top_p: float = 1.0,
                 sample_u=None, exit_readback: bool = False):
        self.T = np.ascontiguousarray(T, dtype=np.float32)
        self.su = None if sample_u is None else np.ascontiguousarray(sample_u, dtype=np.float32)
        self.fe = None if forced_exit is None else np.ascontiguousarray(forced_exit, dtype=np.int32)
        self.fd = None if forced_draft is None else np.ascontiguousarray(forced_draft, dtype=np.int32)
        n_forced = 0
        if self.fe is not None:
            n_forced = len(self.fe)
        if self.fd is not None:
            n_forced = len(self.fd) if self.fe is None else min(n_forced, len(self.fd))
        self.c = sb_params(d_max, w_max,
                           self.T.ctypes.data_as(C.POINTER(C.c_float)) if len(self.T) else None,
                           threshold, eos_id,
                           None if self.fe is None else self.fe.ctypes.data_as(C.POINTER(C.c_int32)),
                           None if self.fd is None else self.fd.ctypes.data_as(C.POINTER(C.c_int32)),
                           n_forced, head_mask, sample_temperature, top_p,
                           None if self.su is None else self.su.ctypes.data_as(C.POINTER(C.c_float)),
                           0 if self.su is None else len(self.su), 1 if exit_readback else 0)


def _stats_dict(st: sb_stats) -> dict:
    d = {n: getattr(st, n) for n, _ in sb_stats._fields_ if n not in ("accept_hist", "exit_hist")}
    d["accept_hist"] = list(st.accept_hist)
    d["exit_hist"] = list(st.exit_hist)
    return d


class Model:
    """Device-resident weights + an sb_model handle.

    weights: {name: numpy array} as produced by sb_inputs.make_weights (uint16 bf16
    bits or float32 matrices, float32 norm gains); they are copied to `device`.
    """

    def __init__(self, shape, weights: Dict[str, np.ndarray], max_seq: int, device: str = "cuda:0",
                 proj_kernel: int = PROJ_AUTO, stream=None, own_packed: bool = True):
        """own_packed: this object allocates the buffer of the tile-packed projections and hands it
        to the library (and drops its row-major projection tensors after the load); False leaves
        that allocation to the library."""
        import torch
        self.torch = torch
        self.device = torch.device(device)
        self.shape = shape
        self.max_seq = max_seq
        self.cfg = make_config(shape, max_seq, proj_kernel)
        self.tensors = {}
        with torch.cuda.device(self.device):
            for k, v in weights.items():
                a = np.ascontiguousarray(v)
                if a.dtype == np.uint16:
                    a = a.view(np.int16)
                self.tensors[k] = torch.from_numpy(a).to(self.device)
        L, E = shape.n_layers, shape.n_exit_heads
        t = self.tensors

        def arr(prefix, n):
            a = (C.c_void_p * max(n, 1))()
            for i in range(n):
                a[i] = t[f"{prefix}.{i}"].data_ptr()
            return a

        self._arrs = {p: arr(p, L) for p in ("attn_norm", "w_qkv", "w_o", "ffn_norm", "w_gate_up", "w_down")}
        self._arrs["exit_norm"] = arr("exit_norm", E)
        self._arrs["exit_head"] = arr("exit_head", E)
        cast = lambda a: C.cast(a, C.POINTER(C.c_void_p))
        self.w = sb_weights(t["embed"].data_ptr(), t["final_norm"].data_ptr(), t["lm_head"].data_ptr(),
                            cast(self._arrs["attn_norm"]), cast(self._arrs["w_qkv"]), cast(self._arrs["w_o"]),
                            cast(self._arrs["ffn_norm"]), cast(self._arrs["w_gate_up"]),
                            cast(self._arrs["w_down"]), cast(self._arrs["exit_norm"]),
                            cast(self._arrs["exit_head"]), None, 0)
        self.packed = None
        pbytes = packed_weight_bytes(self.cfg)
        if own_packed and pbytes:
            with torch.cuda.device(self.device):
                self.packed = torch.empty(pbytes, dtype=torch.uint8, device=self.device)
            self.w.packed, self.w.packed_bytes = self.packed.data_ptr(), pbytes
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        self.h = C.c_void_p()
        with torch.cuda.device(self.device):
            check(lib().sb_load_model(C.byref(self.cfg), C.byref(self.w), C.c_void_p(self.stream.cuda_stream),
                                      C.byref(self.h)))
        if pbytes:   # the row-major projections are not read after the load
            for k in [k for k in t if k.split(".")[0] in ("w_qkv", "w_o", "w_gate_up", "w_down", "exit_head", "lm_head")]:
                del t[k]

    def session(self, page_order: Optional[Sequence[int]] = None) -> "Session":
        return Session(self, page_order)

    def close(self):
        if self.h:
            lib().sb_free_model(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Session:
    def __init__(self, model: Model, page_order: Optional[Sequence[int]] = None):
        torch = model.torch
        self.model = model
        kv_bytes, ws_bytes = query_sizes(model.cfg)
        with torch.cuda.device(model.device):
            self.kv_pool = torch.empty(kv_bytes, dtype=torch.uint8, device=model.device)
            self.workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=model.device)
        po = None
        if page_order is not None:
            self._po = np.ascontiguousarray(page_order, dtype=np.int32)
            po = self._po.ctypes.data
        self.h = C.c_void_p()
        with torch.cuda.device(model.device):
            check(lib().sb_new_session(model.h, self.kv_pool.data_ptr(), kv_bytes, self.workspace.data_ptr(),
                                       ws_bytes, po, C.byref(self.h)))

    def close(self):
        if self.h:
            lib().sb_free_session(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def prefill(self, prompt) -> int:
        prompt = np.ascontiguousarray(prompt, dtype=np.int32)
        t = C.c_int32()
        check(lib().sb_prefill(self.h, prompt.ctypes.data, len(prompt), C.byref(t)))
        return t.value

    def draft_step(self, p: Params) -> dict:
        r = sb_draft_result()
        check(lib().sb_draft_step(self.h, C.byref(p.c), C.byref(r)))
        return dict(token=r.token, exit_layer=r.exit_layer, status=r.status, confidence=r.confidence)

    def verify(self, p: Params) -> dict:
        r = sb_verify_result()
        check(lib().sb_verify(self.h, C.byref(p.c), C.byref(r)))
        return dict(n_rows=r.n_rows, n_drafts=r.n_drafts, n_matched=r.n_matched, n_emit=r.n_emit,
                    align_layer=r.align_layer, tokens=list(r.tokens)[:r.n_rows],
                    accept_prob=list(r.accept_prob)[:r.n_rows])

    def generate(self, prompt, max_new: int, p: Params):
        """Returns (tokens, stats dict)."""
        prompt = np.ascontiguousarray(prompt, dtype=np.int32)
        out = np.empty(max_new, dtype=np.int32)
        n = C.c_int32()
        st = sb_stats()
        check(lib().sb_generate(self.h, prompt.ctypes.data, len(prompt), max_new, C.byref(p.c),
                                out.ctypes.data, max_new, C.byref(n), C.byref(st)))
        return out[:n.value].copy(), _stats_dict(st)

    def decode(self, max_new: int, p: Params):
        """Continue from the current state; returns (tokens, stats dict)."""
        out = np.empty(max_new, dtype=np.int32)
        n = C.c_int32()
        st = sb_stats()
        check(lib().sb_decode(self.h, max_new, C.byref(p.c), out.ctypes.data, max_new, C.byref(n), C.byref(st)))
        return out[:n.value].copy(), _stats_dict(st)

    def rewind(self, n_keep: int, pending_token: int, draft_counter: int = 0):
        check(lib().sb_rewind(self.h, n_keep, int(pending_token), draft_counter))

    def profile_begin(self, classes=None, max_launches: int = 1 << 16, sample_every: int = 1):
        mask = 0
        for name in (classes or KERNEL_CLASSES):
            mask |= 1 << KERNEL_CLASSES.index(name)
        check(lib().sb_profile_begin(self.h, mask, max_launches, sample_every))

    def profile_end(self) -> dict:
        n = len(KERNEL_CLASSES)
        launches = np.zeros(n, dtype=np.int64)
        ms = np.zeros(n, dtype=np.float64)
        nbytes = np.zeros(n, dtype=np.int64)
        empty = C.c_double()
        check(lib().sb_profile_end(self.h, launches.ctypes.data, ms.ctypes.data, nbytes.ctypes.data,
                                   C.byref(empty)))
        self.empty_pair_ms = empty.value
        return {k: dict(launches=int(launches[i]), total_ms=float(ms[i]), bytes=int(nbytes[i]))
                for i, k in enumerate(KERNEL_CLASSES) if launches[i]}

    def phase_timing(self, on: bool = True):
        check(lib().sb_phase_timing(self.h, int(on)))

    def debug_fail_launch(self, n: int):
        check(lib().sb_debug_fail_launch(self.h, n))

    def open_rows(self) -> int:
        return lib().sb_open_rows(self.h)

    def stats(self) -> dict:
        st = sb_stats()
        check(lib().sb_get_stats(self.h, C.byref(st)))
        return _stats_dict(st)

    def committed_len(self) -> int:
        return lib().sb_committed_len(self.h)

    def debug_enable(self, on: bool = True):
        check(lib().sb_debug_enable(self.h, int(on)))

    def debug_logits(self, layer: int, row: int = 0) -> np.ndarray:
        out = np.empty(self.model.shape.vocab, dtype=np.float32)
        check(lib().sb_debug_logits(self.h, layer, row, out.ctypes.data, out.size))
        return out

    def debug_hidden(self, slot: int) -> np.ndarray:
        out = np.empty(self.model.shape.d_model, dtype=np.float32)
        check(lib().sb_debug_hidden(self.h, slot, out.ctypes.data, out.size))
        return out

    def debug_kv(self, layer: int, pos: int):
        s = self.model.shape
        k = np.empty(s.n_kv_heads * s.head_dim, dtype=np.float32)
        v = np.empty_like(k)
        check(lib().sb_debug_kv(self.h, layer, pos, k.ctypes.data, v.ctypes.data, k.size))
        return k, v


# ---------------------------------------------------------------- single kernels
class Batch:
    """Several sessions of one model decoded together (sb_new_batch / sb_batch_decode)."""

    def __init__(self, sessions: Sequence[Session]):
        self.sessions = list(sessions)
        arr = (C.c_void_p * len(self.sessions))(*[s.h for s in self.sessions])
        self.h = C.c_void_p()
        check(lib().sb_new_batch(arr, len(self.sessions), C.byref(self.h)))

    def decode(self, max_new: int, params: Sequence[Params]):
        """Returns a list of token arrays, one per sequence."""
        B = len(self.sessions)
        assert len(params) == B
        outs = [np.empty(max_new, dtype=np.int32) for _ in range(B)]
        pp = (C.POINTER(sb_params) * B)(*[C.pointer(p.c) for p in params])
        op = (C.c_void_p * B)(*[o.ctypes.data for o in outs])
        n = (C.c_int32 * B)()
        check(lib().sb_batch_decode(self.h, max_new, pp, op, n))
        return [outs[b][: n[b]].copy() for b in range(B)]

    def close(self):
        if self.h:
            lib().sb_free_batch(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _stream_ptr(torch, device):
    return C.c_void_p(torch.cuda.current_stream(device).cuda_stream)


def op_rmsnorm(x, gain, eps: float):
    """x [M, d] float32 cuda tensor, gain [d] float32 cuda tensor -> [M, d]."""
    import torch
    out = torch.empty_like(x)
    check(lib().sb_op_rmsnorm(x.data_ptr(), gain.data_ptr(), out.data_ptr(), x.shape[0], x.shape[1], eps,
                              _stream_ptr(torch, x.device)))
    return out


def _wdtype(W):
    import torch
    if W.dtype == torch.float32:
        return FP32
    if W.dtype in (torch.int16, torch.bfloat16):
        return BF16
    raise TypeError(f"weights must be float32, or bf16 bits as int16 / bfloat16, not {W.dtype}")


def op_repack(W):
    """Tile-packed copy of a bf16 matrix (int16 / bfloat16 tensor [N, K]) for PROJ_MFMA_PACKED."""
    import torch
    N, K = W.shape
    P = torch.empty_like(W)
    check(lib().sb_op_repack(W.data_ptr(), N, K, P.data_ptr(), _stream_ptr(torch, W.device)))
    return P


def op_gemm(Wp, x, scratch=None):
    """Prompt-pass projection: Wp = op_repack(W) of a bf16 W [N, K], x [M <= 128, K] float32 -> y [M, N]."""
    import torch
    N, K = Wp.shape
    M = x.shape[0]
    y = torch.empty((M, N), dtype=torch.float32, device=x.device)
    if scratch is None:
        scratch = torch.empty(max(lib().sb_op_gemm_scratch_bytes(N, K), 256), dtype=torch.uint8, device=x.device)
    check(lib().sb_op_gemm(Wp.data_ptr(), N, K, x.data_ptr(), y.data_ptr(), M, scratch.data_ptr(),
                           _stream_ptr(torch, x.device)))
    return y


def op_gemv(W, x, kernel: int = PROJ_VALU):
    """W [N, K] (float32, or bf16 as int16/bfloat16), x [M, K] float32 -> y [M, N] float32.
    For PROJ_MFMA_PACKED, W is the output of op_repack."""
    import torch
    N, K = W.shape
    M = x.shape[0]
    y = torch.empty((M, N), dtype=torch.float32, device=x.device)
    nbytes = lib().sb_op_gemv_scratch_bytes(M, K)
    scratch = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=x.device)
    check(lib().sb_op_gemv(W.data_ptr(), _wdtype(W), N, K, x.data_ptr(), y.data_ptr(), M, kernel,
                           scratch.data_ptr(), _stream_ptr(torch, x.device)))
    return y


def op_gate_up(W, x, kernel: int = PROJ_VALU):
    """W [2N, K] (gate rows, then up rows; op_repack of it for PROJ_MFMA_PACKED), x [M, K] float32 ->
    u [M, N] float32 = silu(gate) * up."""
    import torch
    N, K = W.shape[0] // 2, W.shape[1]
    M = x.shape[0]
    u = torch.empty((M, N), dtype=torch.float32, device=x.device)
    scratch = torch.empty(max(lib().sb_op_gemv_scratch_bytes(M, K), 256), dtype=torch.uint8, device=x.device)
    check(lib().sb_op_gate_up(W.data_ptr(), _wdtype(W), N, K, x.data_ptr(), u.data_ptr(), M, kernel,
                              scratch.data_ptr(), _stream_ptr(torch, x.device)))
    return u


def op_head(W, x, T: float, kernel: int = PROJ_VALU, want_logits: bool = False):
    """Exit-head evaluation on normalised rows: returns (argmax [M] int32, conf [M] float32, logits|None)."""
    import torch
    N, K = W.shape
    M = x.shape[0]
    am = torch.empty(M, dtype=torch.int32, device=x.device)
    cf = torch.empty(M, dtype=torch.float32, device=x.device)
    logits = torch.empty((M, N), dtype=torch.float32, device=x.device) if want_logits else None
    scratch = torch.zeros(lib().sb_op_head_scratch_bytes(M, N, K), dtype=torch.uint8, device=x.device)
    check(lib().sb_op_head(W.data_ptr(), _wdtype(W), N, K, x.data_ptr(), M, T, kernel, am.data_ptr(),
                           cf.data_ptr(), logits.data_ptr() if want_logits else None, scratch.data_ptr(),
                           _stream_ptr(torch, x.device)))
    return am, cf, logits


def op_head_static(W, x, T: float, kernel: int, am, cf):
    """op_head without a scratch buffer (the library's static device array): writes into the
    caller's am [M] int32 and cf [M] float32 tensors; allocates nothing."""
    import torch
    N, K = W.shape
    check(lib().sb_op_head_static(W.data_ptr(), _wdtype(W), N, K, x.data_ptr(), x.shape[0], T, kernel,
                                  am.data_ptr(), cf.data_ptr(), _stream_ptr(torch, x.device)))


def rope_table(head_dim: int, base: float, n_pos: int):
    c = np.empty((n_pos, head_dim // 2), dtype=np.float32)
    s = np.empty_like(c)
    check(lib().sb_rope_table_host(head_dim, base, n_pos, c.ctypes.data, s.ctypes.data))
    return c, s


def op_attention(qkv, n_heads, n_kv_heads, head_dim, kv_dtype, pool, table, layer, rope_cos, rope_sin, pos0,
                 scratch=None):
    """RoPE + KV append + causal attention of the rows in qkv [M, (Hq+2Hkv)*hd] (raw projections)."""
    import torch
    M = qkv.shape[0]
    out = torch.empty((M, n_heads * head_dim), dtype=torch.float32, device=qkv.device)
    if scratch is None:
        scratch = torch.empty(lib().sb_op_attention_scratch_bytes(n_heads, head_dim, kv_dtype, table.numel()),
                              dtype=torch.uint8, device=qkv.device)
    check(lib().sb_op_attention(qkv.data_ptr(), n_heads, n_kv_heads, head_dim, kv_dtype, pool.data_ptr(),
                                table.data_ptr(), table.numel(), layer, rope_cos.data_ptr(), rope_sin.data_ptr(),
                                pos0, M, out.data_ptr(), scratch.data_ptr(), _stream_ptr(torch, qkv.device)))
    return out


def op_prompt_attention(qkv, n_heads, n_kv_heads, head_dim, pool, table, layer, rope_cos, rope_sin, pos0):
    """op_attention in the prompt's form: any number of rows, bf16 pool, running soft-max per query."""
    import torch
    M = qkv.shape[0]
    out = torch.empty((M, n_heads * head_dim), dtype=torch.float32, device=qkv.device)
    check(lib().sb_op_prompt_attention(qkv.data_ptr(), n_heads, n_kv_heads, head_dim, pool.data_ptr(),
                                       table.data_ptr(), table.numel(), layer, rope_cos.data_ptr(),
                                       rope_sin.data_ptr(), pos0, M, out.data_ptr(), _stream_ptr(torch, qkv.device)))
    return out


def op_copy(dst, src):
    """Plain copy kernel between two equally sized cuda tensors (bandwidth yardstick)."""
    import torch
    n = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == n
    check(lib().sb_op_copy(dst.data_ptr(), src.data_ptr(), n, _stream_ptr(torch, src.device)))


def op_read(src, sink):
    import torch
    check(lib().sb_op_read(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(),
                           _stream_ptr(torch, src.device)))

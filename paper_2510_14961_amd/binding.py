"""ctypes binding of librdlm.so: same names as the C ABI (include/rdlm.h), marshalling only.

PyTorch appears here for device memory and the stream; every step of the path runs in the
library's kernels.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Iterable, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

EXPORTED_SYMBOLS = [
    "rdlm_num_weights", "rdlm_create", "rdlm_destroy", "rdlm_strerror", "rdlm_last_hip_error",
    "rdlm_device_bytes", "rdlm_set_tokens", "rdlm_prefill", "rdlm_init_state", "rdlm_prelude",
    "rdlm_core_step", "rdlm_coda_decode", "rdlm_sampler_begin", "rdlm_sampler_join", "rdlm_sample_step", "rdlm_generate",
    "rdlm_read_tokens", "rdlm_read_states", "rdlm_read_counts", "rdlm_read_deltas", "rdlm_read_kv",
    "rdlm_linear", "rdlm_time_linear", "rdlm_time_core_step", "rdlm_profile_gemm_begin",
    "rdlm_profile_gemm_read", "rdlm_workspace_bytes", "rdlm_create_ws", "rdlm_core_step_static",
    "rdlm_core_step_static_bytes", "rdlm_sampler_status", "rdlm_set_tuning", "rdlm_read_prev_states",
    "rdlm_read_window", "rdlm_time_stream_read", "rdlm_time_mfma_loop",
    "rdlm_create_paged", "rdlm_kv_blocks", "rdlm_seq_release", "rdlm_seq_evict_bytes", "rdlm_seq_evict",
    "rdlm_seq_admit", "rdlm_read_frozen",
]

STATUS = {"OK": 0, "EINVAL": -1, "ECAPACITY": -2, "ENOMEM": -3, "EHIP": -4, "ESTATE": -5, "ENUMERIC": -6}
STATIC_SCRATCH_BYTES = 40 << 20


class RdlmError(RuntimeError):
    def __init__(self, msg, status=None):
        super().__init__(msg)
        self.status = status


class _Model(C.Structure):
    _fields_ = [("vocab", C.c_int32), ("hidden", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32),
                ("mlp", C.c_int32), ("n_prelude", C.c_int32), ("n_core", C.c_int32), ("n_coda", C.c_int32),
                ("rope_base", C.c_float), ("rms_eps", C.c_float), ("emb_scale", C.c_float), ("dtype", C.c_int32)]


class _Sampler(C.Structure):
    _fields_ = [("n_new", C.c_int32), ("r_inner", C.c_int32), ("r_total", C.c_int32), ("w_max", C.c_int32),
                ("headway", C.c_int32), ("adaptive", C.c_int32), ("eps", C.c_float), ("alpha", C.c_float),
                ("temperature", C.c_float), ("pad_token", C.c_int32), ("beta", C.c_float), ("eta", C.c_float),
                ("top_p", C.c_float), ("init_mode", C.c_int32), ("seed", C.c_uint64)]


def library_path() -> str:
    return os.path.join(_HERE, "librdlm.so")


def load_library():
    """Load librdlm.so; raises if it has not been built (there is no fallback path)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    # PyTorch ships its own HIP runtime; it has to be in the process before librdlm.so is loaded so
    # that both resolve to one runtime (two runtimes in one process do not share the device).
    import torch  # noqa: F401
    path = library_path()
    if not os.path.exists(path):
        raise RdlmError(f"{path} is missing: build it first (python -m paper_2510_14961_amd.build)")
    lib = C.CDLL(path)
    vp, i32, u64, f32 = C.c_void_p, C.c_int32, C.c_uint64, C.c_float
    pi32 = C.POINTER(C.c_int32)
    sig = {
        "rdlm_num_weights": (i32, [C.POINTER(_Model)]),
        "rdlm_create": (C.c_int, [C.POINTER(_Model), C.POINTER(vp), i32, i32, i32, vp, C.POINTER(vp)]),
        "rdlm_destroy": (C.c_int, [vp]),
        "rdlm_strerror": (C.c_char_p, [C.c_int]),
        "rdlm_last_hip_error": (C.c_int, [vp]),
        "rdlm_device_bytes": (C.c_size_t, [vp]),
        "rdlm_set_tokens": (C.c_int, [vp, i32, pi32, i32]),
        "rdlm_prefill": (C.c_int, [vp, i32, i32, i32, f32, u64]),
        "rdlm_init_state": (C.c_int, [vp, i32, i32, i32, f32, u64, vp]),
        "rdlm_prelude": (C.c_int, [vp, i32, pi32, pi32, pi32, vp, vp]),
        "rdlm_core_step": (C.c_int, [vp, i32, pi32, pi32, pi32, vp, vp, i32, vp]),
        "rdlm_coda_decode": (C.c_int, [vp, i32, pi32, pi32, pi32, vp, f32, u64, i32, vp, vp, f32]),
        "rdlm_sampler_begin": (C.c_int, [vp, C.POINTER(_Sampler), i32]),
        "rdlm_sampler_join": (C.c_int, [vp, i32]),
        "rdlm_sample_step": (C.c_int, [vp]),
        "rdlm_generate": (C.c_int, [vp, i32, pi32]),
        "rdlm_read_tokens": (C.c_int, [vp, i32, pi32, i32, pi32]),
        "rdlm_read_frozen": (C.c_int, [vp, i32, pi32, i32, pi32]),
        "rdlm_read_states": (C.c_int, [vp, i32, i32, i32, C.POINTER(C.c_float)]),
        "rdlm_read_counts": (C.c_int, [vp, i32, i32, i32, pi32]),
        "rdlm_read_deltas": (C.c_int, [vp, i32, C.POINTER(C.c_float), i32, pi32]),
        "rdlm_read_kv": (C.c_int, [vp, i32, i32, i32, i32, C.POINTER(C.c_float), C.POINTER(C.c_float)]),
        "rdlm_linear": (C.c_int, [vp, i32, vp, i32, vp]),
        "rdlm_time_linear": (C.c_int, [vp, i32, i32, i32, C.POINTER(C.c_float)]),
        "rdlm_time_core_step": (C.c_int, [vp, i32, i32, i32, i32, C.POINTER(C.c_float)]),
        "rdlm_profile_gemm_begin": (C.c_int, [vp, i32, i32, i32]),
        "rdlm_profile_gemm_read": (C.c_int, [vp, C.POINTER(C.c_float), pi32]),
        "rdlm_workspace_bytes": (C.c_size_t, [C.POINTER(_Model), i32, i32]),
        "rdlm_create_ws": (C.c_int, [C.POINTER(_Model), C.POINTER(vp), i32, i32, i32, vp, vp, C.c_size_t,
                                     C.POINTER(vp)]),
        "rdlm_create_paged": (C.c_int, [C.POINTER(_Model), C.POINTER(vp), i32, i32, i32, i32, vp, C.POINTER(vp)]),
        "rdlm_kv_blocks": (C.c_int, [vp, pi32, pi32]),
        "rdlm_seq_release": (C.c_int, [vp, i32]),
        "rdlm_seq_evict_bytes": (C.c_size_t, [vp, i32]),
        "rdlm_seq_evict": (C.c_int, [vp, i32, vp, C.c_size_t]),
        "rdlm_seq_admit": (C.c_int, [vp, i32, vp, C.c_size_t]),
        "rdlm_core_step_static": (C.c_int, [vp, i32, pi32, pi32, pi32, vp, vp, i32, vp]),
        "rdlm_core_step_static_bytes": (C.c_size_t, [vp, i32]),
        "rdlm_sampler_status": (C.c_int, [vp, pi32, pi32]),
        "rdlm_set_tuning": (C.c_int, [vp, C.c_char_p, C.c_char_p]),
        "rdlm_read_prev_states": (C.c_int, [vp, i32, i32, i32, C.POINTER(C.c_float)]),
        "rdlm_read_window": (C.c_int, [vp, i32, pi32, pi32, pi32]),
        "rdlm_time_stream_read": (C.c_int, [vp, i32, i32, i32, i32, C.POINTER(C.c_float), C.POINTER(C.c_size_t)]),
        "rdlm_time_mfma_loop": (C.c_int, [vp, i32, i32, i32, C.POINTER(C.c_float), C.POINTER(C.c_double)]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _LIB = lib
    return lib


def _model_struct(shape) -> "_Model":
    return _Model(shape.vocab, shape.hidden, shape.n_heads, shape.head_dim, shape.mlp, shape.n_prelude,
                  shape.n_core, shape.n_coda, shape.rope_base, shape.rms_eps, shape.emb_scale,
                  0 if shape.dtype == "f32" else 1)


def workspace_bytes(shape, max_seqs: int, max_rows: int) -> int:
    """rdlm_workspace_bytes: size of the step workspace a context of these limits needs (host only)."""
    m = _model_struct(shape)
    return int(load_library().rdlm_workspace_bytes(C.byref(m), max_seqs, max_rows))


def weight_names(shape) -> List[str]:
    """Order in which rdlm_create expects the tensors (see include/rdlm.h)."""
    out = ["emb"]
    for blk, n in (("P", shape.n_prelude), ("R", shape.n_core), ("C", shape.n_coda)):
        for i in range(n):
            out += [f"{blk}{i}.{t}" for t in ("g1", "wqkv", "wo", "g2", "wg", "wu", "wd")]
    return out + ["wa", "gf", "gout"]


def upload_weights(shape, weights: Iterable, device="cuda"):
    """Copy (name, float32 numpy array) pairs to the device in the model dtype.  bf16 models get
    bf16 tensors (the inputs are already bf16-exact); gains stay float32."""
    import torch
    out = {}
    for name, arr in (weights.items() if isinstance(weights, dict) else weights):
        t = torch.from_numpy(np.ascontiguousarray(arr))
        if arr.ndim == 2 and shape.dtype == "bf16":
            t = t.to(torch.bfloat16)
        out[name] = t.to(device)
    return out


def _iptr(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


class Context:
    """One rdlm_ctx.  Methods carry the names of the C functions without the prefix."""

    def __init__(self, shape, dev_weights: Dict[str, "object"], max_seqs: int, max_positions: int,
                 max_rows: int, stream=None, workspace=None, kv_pool_positions=None):
        """workspace: None (the library allocates its step workspace) or a CUDA uint8 tensor of at
        least workspace_bytes(shape, max_seqs, max_rows) bytes that the caller keeps alive.
        kv_pool_positions: None (every slot can reach max_positions) or the total number of cached
        positions all slots share (rdlm_create_paged)."""
        import torch
        self.lib = load_library()
        self.shape = shape
        self.h, self.V = shape.hidden, shape.vocab
        self.model = _model_struct(shape)
        names = weight_names(shape)
        assert self.lib.rdlm_num_weights(C.byref(self.model)) == len(names)
        want = torch.float32 if shape.dtype == "f32" else torch.bfloat16
        ptrs = (C.c_void_p * len(names))()
        for i, n in enumerate(names):
            t = dev_weights[n]
            assert t.is_cuda and t.is_contiguous(), n
            assert t.dtype == (want if t.dim() == 2 else torch.float32), (n, t.dtype)
            ptrs[i] = t.data_ptr()
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        handle = C.c_void_p()
        if kv_pool_positions is not None:
            assert workspace is None
            rc = self.lib.rdlm_create_paged(C.byref(self.model), ptrs, max_seqs, max_positions, max_rows,
                                            int(kv_pool_positions), C.c_void_p(self.stream.cuda_stream),
                                            C.byref(handle))
        elif workspace is None:
            rc = self.lib.rdlm_create(C.byref(self.model), ptrs, max_seqs, max_positions, max_rows,
                                      C.c_void_p(self.stream.cuda_stream), C.byref(handle))
        else:
            assert workspace.is_cuda and workspace.is_contiguous() and workspace.element_size() == 1
            self._workspace = workspace                 # keep it alive as long as the context
            rc = self.lib.rdlm_create_ws(C.byref(self.model), ptrs, max_seqs, max_positions, max_rows,
                                         C.c_void_p(self.stream.cuda_stream), C.c_void_p(workspace.data_ptr()),
                                         workspace.numel(), C.byref(handle))
        if rc != 0:
            raise RdlmError(f"rdlm_create: {self.lib.rdlm_strerror(rc).decode()} ({rc})", rc)
        self.ctx = handle
        self.max_positions = max_positions

    # -- helpers ---------------------------------------------------------------------------
    def _chk(self, rc: int, what: str):
        if rc != 0:
            hip = self.lib.rdlm_last_hip_error(self.ctx)
            raise RdlmError(f"{what}: {self.lib.rdlm_strerror(rc).decode()} ({rc}), hip={hip}", rc)

    @staticmethod
    def _rows(seq_ids, pos0, n_rows):
        a = [np.ascontiguousarray(np.asarray(v, dtype=np.int32)).reshape(-1) for v in (seq_ids, pos0, n_rows)]
        assert len(a[0]) == len(a[1]) == len(a[2])
        return a

    def close(self):
        if getattr(self, "ctx", None):
            self.lib.rdlm_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def device_bytes(self) -> int:
        return int(self.lib.rdlm_device_bytes(self.ctx))

    # -- ABI calls --------------------------------------------------------------------------
    def set_tokens(self, seq: int, tokens):
        t = np.ascontiguousarray(np.asarray(tokens, dtype=np.int32))
        self._chk(self.lib.rdlm_set_tokens(self.ctx, seq, _iptr(t), len(t)), "rdlm_set_tokens")

    def prefill(self, seq: int, n: int, r: int, alpha: float, seed: int):
        self._chk(self.lib.rdlm_prefill(self.ctx, seq, n, r, alpha, seed), "rdlm_prefill")

    def init_state(self, seq: int, pos0: int, n: int, alpha: float, seed: int, z_out):
        assert z_out.is_cuda and z_out.is_contiguous() and z_out.numel() >= n * self.h
        self._chk(self.lib.rdlm_init_state(self.ctx, seq, pos0, n, alpha, seed, C.c_void_p(z_out.data_ptr())),
                  "rdlm_init_state")

    def prelude(self, seq_ids, pos0, n_rows, tokens_dev, e_out):
        s, p, n = self._rows(seq_ids, pos0, n_rows)
        self._chk(self.lib.rdlm_prelude(self.ctx, len(s), _iptr(s), _iptr(p), _iptr(n),
                                        C.c_void_p(tokens_dev.data_ptr()), C.c_void_p(e_out.data_ptr())),
                  "rdlm_prelude")

    def core_step(self, seq_ids, pos0, n_rows, e, z_inout, r_inner: int = 1, delta_out=None):
        s, p, n = self._rows(seq_ids, pos0, n_rows)
        d = C.c_void_p(delta_out.data_ptr()) if delta_out is not None else C.c_void_p()
        self._chk(self.lib.rdlm_core_step(self.ctx, len(s), _iptr(s), _iptr(p), _iptr(n), C.c_void_p(e.data_ptr()),
                                          C.c_void_p(z_inout.data_ptr()), r_inner, d), "rdlm_core_step")

    def core_step_static(self, seq_ids, pos0, n_rows, e, z_inout, r_inner: int = 1, delta_out=None):
        s, p, n = self._rows(seq_ids, pos0, n_rows)
        d = C.c_void_p(delta_out.data_ptr()) if delta_out is not None else C.c_void_p()
        self._chk(self.lib.rdlm_core_step_static(self.ctx, len(s), _iptr(s), _iptr(p), _iptr(n),
                                                 C.c_void_p(e.data_ptr()), C.c_void_p(z_inout.data_ptr()), r_inner, d),
                  "rdlm_core_step_static")

    def core_step_static_bytes(self, n_tiles: int) -> int:
        return int(self.lib.rdlm_core_step_static_bytes(self.ctx, n_tiles))

    def set_tuning(self, name: str, value: str):
        self._chk(self.lib.rdlm_set_tuning(self.ctx, name.encode(), str(value).encode()), "rdlm_set_tuning")

    def sampler_status(self):
        a, nf = C.c_int32(0), C.c_int32(0)
        self._chk(self.lib.rdlm_sampler_status(self.ctx, C.byref(a), C.byref(nf)), "rdlm_sampler_status")
        return a.value, bool(nf.value)

    def coda_decode(self, seq_ids, pos0, n_rows, z, temperature: float, seed: int, step: int, tokens_out,
                    logits_out=None, top_p: float = 0.0):
        s, p, n = self._rows(seq_ids, pos0, n_rows)
        lo = C.c_void_p(logits_out.data_ptr()) if logits_out is not None else C.c_void_p()
        self._chk(self.lib.rdlm_coda_decode(self.ctx, len(s), _iptr(s), _iptr(p), _iptr(n), C.c_void_p(z.data_ptr()),
                                            temperature, seed, step, C.c_void_p(tokens_out.data_ptr()), lo, top_p),
                  "rdlm_coda_decode")

    def sampler_begin(self, n_seqs: int, *, n_new: int, r_inner: int, r_total: int, w_max: int = 0,
                      headway: int = 1, adaptive: bool = False, eps: float = 0.0, alpha: float = 1.0,
                      temperature: float = 0.0, pad_token: int = 0, seed: int = 1, beta: float = 0.0,
                      eta: float = 0.0, top_p: float = 0.0, continuous_compute: bool = False):
        s = _Sampler(n_new, r_inner, r_total, w_max, headway, int(adaptive), eps, alpha, temperature, pad_token,
                     beta, eta, top_p, int(continuous_compute), seed)
        self._chk(self.lib.rdlm_sampler_begin(self.ctx, C.byref(s), n_seqs), "rdlm_sampler_begin")

    def sampler_join(self, seq: int):
        self._chk(self.lib.rdlm_sampler_join(self.ctx, seq), "rdlm_sampler_join")

    def kv_blocks(self):
        """(blocks of 32 positions in the KV pool, blocks no slot owns)"""
        t, f = C.c_int32(0), C.c_int32(0)
        self._chk(self.lib.rdlm_kv_blocks(self.ctx, C.byref(t), C.byref(f)), "rdlm_kv_blocks")
        return t.value, f.value

    def seq_release(self, seq: int):
        self._chk(self.lib.rdlm_seq_release(self.ctx, seq), "rdlm_seq_release")

    def seq_evict(self, seq: int) -> np.ndarray:
        """Evict slot seq; returns the host record rdlm_seq_admit takes."""
        n = self.lib.rdlm_seq_evict_bytes(self.ctx, seq)
        buf = np.empty(n, np.uint8)
        self._chk(self.lib.rdlm_seq_evict(self.ctx, seq, buf.ctypes.data_as(C.c_void_p), n), "rdlm_seq_evict")
        return buf

    def seq_admit(self, seq: int, record: np.ndarray):
        record = np.ascontiguousarray(record, dtype=np.uint8)
        self._chk(self.lib.rdlm_seq_admit(self.ctx, seq, record.ctypes.data_as(C.c_void_p), record.size),
                  "rdlm_seq_admit")

    def sample_step(self):
        self._chk(self.lib.rdlm_sample_step(self.ctx), "rdlm_sample_step")

    def generate(self, max_steps: int) -> int:
        steps = C.c_int32(0)
        self._chk(self.lib.rdlm_generate(self.ctx, max_steps, C.byref(steps)), "rdlm_generate")
        return steps.value

    def read_tokens(self, seq: int, cap: Optional[int] = None):
        cap = self.max_positions if cap is None else cap
        buf = np.zeros(cap, dtype=np.int32)
        nf = C.c_int32(0)
        self._chk(self.lib.rdlm_read_tokens(self.ctx, seq, _iptr(buf), cap, C.byref(nf)), "rdlm_read_tokens")
        return buf, nf.value

    def read_states(self, seq: int, pos0: int, n: int) -> np.ndarray:
        buf = np.zeros((n, self.h), dtype=np.float32)
        self._chk(self.lib.rdlm_read_states(self.ctx, seq, pos0, n, buf.ctypes.data_as(C.POINTER(C.c_float))),
                  "rdlm_read_states")
        return buf

    def read_prev_states(self, seq: int, pos0: int, n: int) -> np.ndarray:
        buf = np.zeros((n, self.h), dtype=np.float32)
        self._chk(self.lib.rdlm_read_prev_states(self.ctx, seq, pos0, n, buf.ctypes.data_as(C.POINTER(C.c_float))),
                  "rdlm_read_prev_states")
        return buf

    def read_frozen(self, seq: int):
        """the frozen text: prompt + tokens made final so far"""
        buf = np.zeros(self.max_positions, np.int32)
        n = C.c_int32(0)
        self._chk(self.lib.rdlm_read_frozen(self.ctx, seq, _iptr(buf), len(buf), C.byref(n)), "rdlm_read_frozen")
        return buf[: n.value].copy()

    def read_window(self, seq: int):
        """(position of the oldest in-flight state, number of in-flight states, finished)"""
        p, n, d = C.c_int32(0), C.c_int32(0), C.c_int32(0)
        self._chk(self.lib.rdlm_read_window(self.ctx, seq, C.byref(p), C.byref(n), C.byref(d)), "rdlm_read_window")
        return p.value, n.value, bool(d.value)

    def read_counts(self, seq: int, pos0: int, n: int) -> np.ndarray:
        buf = np.zeros(n, dtype=np.int32)
        self._chk(self.lib.rdlm_read_counts(self.ctx, seq, pos0, n, _iptr(buf)), "rdlm_read_counts")
        return buf

    def read_deltas(self, seq: int, cap: int = 4096) -> np.ndarray:
        buf = np.zeros(cap, dtype=np.float32)
        n = C.c_int32(0)
        self._chk(self.lib.rdlm_read_deltas(self.ctx, seq, buf.ctypes.data_as(C.POINTER(C.c_float)), cap, C.byref(n)),
                  "rdlm_read_deltas")
        return buf[: min(cap, n.value)]

    def read_kv(self, layer: int, seq: int, pos0: int, n: int):
        H, d = self.shape.n_heads, self.shape.head_dim
        k = np.zeros((n, H, d), dtype=np.float32)
        v = np.zeros((n, H, d), dtype=np.float32)
        fp = C.POINTER(C.c_float)
        self._chk(self.lib.rdlm_read_kv(self.ctx, layer, seq, pos0, n, k.ctypes.data_as(fp), v.ctypes.data_as(fp)),
                  "rdlm_read_kv")
        return k, v

    def linear(self, w_index: int, x, m: int, y):
        self._chk(self.lib.rdlm_linear(self.ctx, w_index, C.c_void_p(x.data_ptr()), m, C.c_void_p(y.data_ptr())),
                  "rdlm_linear")

    def time_linear(self, w_index: int, m: int, iters: int) -> float:
        ms = C.c_float(0)
        self._chk(self.lib.rdlm_time_linear(self.ctx, w_index, m, iters, C.byref(ms)), "rdlm_time_linear")
        return ms.value

    def time_core_step(self, seq: int, pos0: int, n: int, iters: int) -> float:
        ms = C.c_float(0)
        self._chk(self.lib.rdlm_time_core_step(self.ctx, seq, pos0, n, iters, C.byref(ms)), "rdlm_time_core_step")
        return ms.value

    def time_stream_read(self, w_index: int, workgroups: int, waves: int, iters: int):
        """(ms per launch, bytes read per launch)"""
        ms, nb = C.c_float(0), C.c_size_t(0)
        self._chk(self.lib.rdlm_time_stream_read(self.ctx, w_index, workgroups, waves, iters, C.byref(ms), C.byref(nb)),
                  "rdlm_time_stream_read")
        return ms.value, nb.value

    def time_mfma_loop(self, workgroups: int, inner_iters: int, launches: int):
        """(ms per launch, flops per launch)"""
        ms, fl = C.c_float(0), C.c_double(0)
        self._chk(self.lib.rdlm_time_mfma_loop(self.ctx, workgroups, inner_iters, launches, C.byref(ms), C.byref(fl)),
                  "rdlm_time_mfma_loop")
        return ms.value, fl.value

    def profile_gemm_begin(self, n_out: int, k_in: int, max_launches: int):
        self._chk(self.lib.rdlm_profile_gemm_begin(self.ctx, n_out, k_in, max_launches), "rdlm_profile_gemm_begin")

    def profile_gemm_read(self):
        ms, n = C.c_float(0), C.c_int32(0)
        self._chk(self.lib.rdlm_profile_gemm_read(self.ctx, C.byref(ms), C.byref(n)), "rdlm_profile_gemm_read")
        return ms.value, n.value

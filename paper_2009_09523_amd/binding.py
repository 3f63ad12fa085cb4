"""ctypes binding of include/vf.h.  Names follow the C ABI; no arithmetic happens here."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

VF_OK, VF_EINVAL, VF_ENOMEM, VF_EDEVICE, VF_ESTATE = 0, -1, -2, -3, -4
VF_MLP, VF_ENCODER, VF_CONV = 0, 1, 2
VF_F32, VF_BF16 = 0, 1
VF_SGDM, VF_ADAM = 0, 1
VF_MAX_DIMS = 16
VF_FLAG_FUSED_ACCUMULATE = 1
VF_FLAG_NO_GRAPH = 2
VF_FLAG_OVERLAP = 4
VF_FLAG_ORDERED_FOLD = 8

_HERE = os.path.dirname(os.path.abspath(__file__))


def lib_path() -> str:
    return os.path.join(_HERE, "libvf.so")


class VfError(RuntimeError):
    def __init__(self, code: int, where: str, detail: str = ""):
        self.code = code
        super().__init__(f"{where}: error {code}" + (f" ({detail})" if detail else ""))


VF_STATE_MAGIC = 0x3145544154534656
VF_STATE_HEADER_BYTES = 64


class VfDeviceProfile(C.Structure):
    _fields_ = [("n_devices", C.c_int32), ("n_points", C.c_int32),
                ("batch", C.POINTER(C.c_int32)), ("step_time", C.POINTER(C.c_double))]


class VfConfig(C.Structure):
    _fields_ = [
        ("model_kind", C.c_int32), ("n_dims", C.c_int32), ("dims", C.c_int32 * VF_MAX_DIMS),
        ("batchnorm", C.c_int32),
        ("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
        ("d_ffn", C.c_int32), ("seq_len", C.c_int32), ("vocab", C.c_int32), ("n_masked", C.c_int32),
        ("img", C.c_int32), ("in_ch", C.c_int32), ("width", C.c_int32), ("n_blocks", C.c_int32),
        ("classes", C.c_int32),
        ("dtype", C.c_int32), ("optimizer", C.c_int32),
        ("lr", C.c_float), ("momentum", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
        ("adam_eps", C.c_float), ("bn_eps", C.c_float), ("ln_eps", C.c_float),
        ("bn_momentum", C.c_float),
        ("max_batch", C.c_int32), ("max_node_size", C.c_int32), ("max_nodes", C.c_int32),
        ("fold_window", C.c_int32),
        ("node_group", C.c_int32),
        ("flags", C.c_uint32), ("stream", C.c_void_p),
    ]


_SIGNATURES = {
    "vf_partition": (C.c_int, [C.POINTER(C.c_int32), C.c_int32, C.c_int32, C.POINTER(C.c_int32),
                               C.POINTER(C.c_float)]),
    "vf_init": (C.c_int, [C.POINTER(VfConfig), C.POINTER(C.c_void_p)]),
    "vf_step": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                          C.POINTER(C.c_int32)]),
    "vf_prefetch": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32]),
    "vf_step_prefetched": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(C.c_int32)]),
    "vf_grads": (C.c_int, [C.c_void_p, C.c_void_p]),
    "vf_loss": (C.c_int, [C.c_void_p, C.POINTER(C.c_float)]),
    "vf_node_losses": (C.c_int, [C.c_void_p, C.POINTER(C.c_float), C.c_int32]),
    "vf_opt_state": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p]),
    "vf_profile_start": (C.c_int, [C.c_void_p]),
    "vf_profile_stop": (C.c_int, [C.c_void_p, C.c_char_p, C.c_size_t]),
    "vf_step_count": (C.c_int64, [C.c_void_p]),
    "vf_fold_window": (C.c_int32, [C.c_void_p]),
    "vf_streams": (C.c_int32, [C.c_void_p]),
    "vf_num_params": (C.c_int64, [C.c_void_p]),
    "vf_workspace_bytes": (C.c_size_t, [C.c_void_p]),
    "vf_destroy": (None, [C.c_void_p]),
    "vf_strerror": (C.c_char_p, [C.c_int]),
    "vf_last_error": (C.c_char_p, []),
    "vf_accumulate": (C.c_int, [C.c_void_p, C.c_void_p, C.c_float, C.c_int64, C.c_int32, C.c_void_p]),
    "vf_sgdm_update": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_float, C.c_int64,
                                 C.c_void_p]),
    "vf_adam_update": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_float,
                                 C.c_float, C.c_float, C.c_int64, C.c_int64, C.c_void_p]),
    "vf_gemm": (C.c_int, [C.c_int32, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                          C.c_int32, C.c_int32, C.c_int32, C.c_float, C.c_int32, C.c_int32, C.c_void_p]),
    "vf_gemm_noalloc": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int32,
                                  C.c_int32, C.c_int32, C.c_float, C.c_int32, C.c_int32, C.c_void_p]),
    "vf_state_bytes": (C.c_int64, [C.c_void_p]),
    "vf_state_export": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64]),
    "vf_state_import": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64]),
    "vf_solve_split": (C.c_int, [C.POINTER(VfDeviceProfile), C.c_int32, C.c_int32, C.c_double,
                                 C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_double)]),
}


def exported_symbols():
    """Names the header declares (and this binding expects)."""
    return sorted(_SIGNATURES)


_lib = None


def lib() -> C.CDLL:
    """Loads libvf.so; raises if it has not been built (there is no fallback)."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise ImportError(f"{path} is missing: run `python -m paper_2009_09523_amd.build`")
        L = C.CDLL(path)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def _check(rc: int, where: str):
    if rc != VF_OK:
        L = lib()
        detail = L.vf_strerror(rc).decode()
        last = L.vf_last_error().decode()
        raise VfError(rc, where, detail + (": " + last if last and rc == VF_EDEVICE else ""))


def vf_partition(node_sizes: Sequence[int], batch: int):
    """(off int32 [V+1], w float32 [V]) computed by the library (host only)."""
    V = len(node_sizes)
    sizes = (C.c_int32 * max(V, 1))(*[int(b) for b in node_sizes])
    off = (C.c_int32 * (V + 1))()
    w = (C.c_float * max(V, 1))()
    _check(lib().vf_partition(sizes, V, int(batch), off, w), "vf_partition")
    return np.array(off[: V + 1], dtype=np.int32), np.array(w[:V], dtype=np.float32)


def _ptr(t) -> int:
    return int(t.data_ptr())


def _stream_handle(stream) -> int:
    return 0 if stream is None else int(stream.cuda_stream)


def vf_accumulate(buf, g, w: float, first: bool, stream=None):
    n = buf.numel()
    assert g.numel() == n and buf.dtype == g.dtype and str(buf.dtype) == "torch.float32"
    _check(lib().vf_accumulate(_ptr(buf), _ptr(g), float(w), n, int(bool(first)),
                               _stream_handle(stream)), "vf_accumulate")


def vf_sgdm_update(theta, v, G, lr: float, momentum: float, stream=None):
    _check(lib().vf_sgdm_update(_ptr(theta), _ptr(v), _ptr(G), float(lr), float(momentum),
                                theta.numel(), _stream_handle(stream)), "vf_sgdm_update")


def vf_adam_update(theta, m, u, G, lr, beta1, beta2, eps, t: int, stream=None):
    _check(lib().vf_adam_update(_ptr(theta), _ptr(m), _ptr(u), _ptr(G), float(lr), float(beta1),
                                float(beta2), float(eps), int(t), theta.numel(),
                                _stream_handle(stream)), "vf_adam_update")


def vf_gemm(A, B, Cout, M: int, N: int, K: int, alpha: float = 1.0, accumulate: bool = False,
            nsplit: int = 1, stream=None):
    """Cout[M,N] (fp32) = alpha * A[M,K] B[N,K]^T (+ Cout).  A, B: 2-D torch tensors (bf16 or
    fp32), unit stride along the contraction.  With nsplit > 1 Cout is [nsplit, M, ldc]
    (contiguous slabs) and receives the partial products of the contraction slices."""
    import torch
    dtype = VF_BF16 if A.dtype == torch.bfloat16 else VF_F32
    assert A.dtype == B.dtype and A.stride(-1) == 1 and B.stride(-1) == 1 and Cout.stride(-1) == 1
    ldc = Cout.stride(-2)
    if nsplit > 1:
        assert Cout.dim() == 3 and Cout.stride(0) == M * ldc
    _check(lib().vf_gemm(dtype, _ptr(A), A.stride(0), _ptr(B), B.stride(0), _ptr(Cout), ldc,
                         M, N, K, float(alpha), int(bool(accumulate)), int(nsplit),
                         _stream_handle(stream)), "vf_gemm")


VF_NOALLOC_SCRATCH_BYTES = 32 * 1024 * 1024


def vf_gemm_noalloc(A, B, Cout, M: int, N: int, K: int, alpha: float = 1.0, accumulate: bool = False,
                    nsplit: int = 1, stream=None):
    """Cout[M,N] (fp32, dense) = alpha * A[M,K] B[N,K]^T (+ Cout), contraction in nsplit slices whose
    partial products stay in the library's static device scratch.  Returns the status code."""
    import torch
    assert A.dtype == torch.bfloat16 and B.dtype == torch.bfloat16 and Cout.dtype == torch.float32
    assert A.stride(-1) == 1 and B.stride(-1) == 1 and Cout.is_contiguous()
    return lib().vf_gemm_noalloc(_ptr(A), A.stride(0), _ptr(B), B.stride(0), _ptr(Cout), M, N, K,
                                 float(alpha), int(bool(accumulate)), int(nsplit), _stream_handle(stream))


def parse_state(payload: np.ndarray) -> dict:
    """Splits a host payload of vf_state_export into its parts (views, no arithmetic)."""
    header = payload[:VF_STATE_HEADER_BYTES].view(np.int64)
    if int(header[0]) != VF_STATE_MAGIC:
        raise VfError("not a state payload")
    P, n_opt, S, steps = (int(v) for v in header[1:5])
    body = payload[VF_STATE_HEADER_BYTES:VF_STATE_HEADER_BYTES + 4 * (P + n_opt * P + 2 * S)].view(np.float32)
    out = {"P": P, "steps": steps, "optimizer": int(header[5]), "theta": body[:P],
           "opt": [body[P * (1 + k):P * (2 + k)] for k in range(n_opt)]}
    tail = body[P * (1 + n_opt):]
    out["bn_mean"], out["bn_var"] = tail[:S], tail[S:2 * S]
    return out


def vf_solve_split(types, B: int, comm: float = 0.0):
    """types: sequence of (n_devices, batches, step_times).  Returns (b list, v list, step time)."""
    n = len(types)
    arr = (VfDeviceProfile * max(n, 1))()
    keep = []
    for i, (nd, batches, times) in enumerate(types):
        bs = (C.c_int32 * max(len(batches), 1))(*[int(b) for b in batches])
        ts = (C.c_double * max(len(times), 1))(*[float(t) for t in times])
        keep += [bs, ts]
        arr[i].n_devices, arr[i].n_points = int(nd), len(batches)
        arr[i].batch, arr[i].step_time = bs, ts
    b = (C.c_int32 * max(n, 1))()
    v = (C.c_int32 * max(n, 1))()
    t = C.c_double()
    _check(lib().vf_solve_split(arr, n, int(B), float(comm), b, v, C.byref(t)), "vf_solve_split")
    return list(b[:n]), list(v[:n]), float(t.value)


def config_from_workload(wl, max_batch: Optional[int] = None, max_node_size: Optional[int] = None,
                         max_nodes: Optional[int] = None, flags: int = 0, stream=None,
                         fold_window: int = 0, node_group: int = 0) -> VfConfig:
    """Fills a vf_config from a workload description (an object with the attributes of
    vf_inputs.Workload)."""
    cfg = VfConfig()
    cfg.model_kind = {"mlp": VF_MLP, "encoder": VF_ENCODER, "conv": VF_CONV}[wl.kind]
    if wl.kind == "conv":
        cfg.img, cfg.in_ch, cfg.width, cfg.n_blocks, cfg.classes = wl.img, wl.in_ch, wl.width, wl.n_blocks, wl.classes
    elif wl.kind == "mlp":
        cfg.n_dims = len(wl.dims)
        for i, d in enumerate(wl.dims):
            cfg.dims[i] = int(d)
        cfg.batchnorm = int(bool(wl.batchnorm))
    else:
        cfg.n_layers, cfg.d_model, cfg.n_heads = wl.n_layers, wl.d_model, wl.n_heads
        cfg.d_ffn, cfg.seq_len, cfg.vocab, cfg.n_masked = wl.d_ffn, wl.seq_len, wl.vocab, wl.n_masked
    cfg.dtype = {"f32": VF_F32, "bf16": VF_BF16}[wl.dtype]
    cfg.optimizer = {"sgdm": VF_SGDM, "adam": VF_ADAM}[wl.optimizer]
    cfg.lr, cfg.momentum, cfg.beta1, cfg.beta2 = wl.lr, wl.momentum, wl.beta1, wl.beta2
    cfg.adam_eps, cfg.bn_eps, cfg.ln_eps = wl.adam_eps, wl.bn_eps, wl.ln_eps
    cfg.bn_momentum = wl.bn_momentum
    cfg.max_batch = int(max_batch if max_batch is not None else wl.batch)
    cfg.max_node_size = int(max_node_size if max_node_size is not None else max(wl.node_sizes))
    cfg.max_nodes = int(max_nodes if max_nodes is not None else len(wl.node_sizes))
    cfg.flags = int(flags)
    cfg.fold_window = int(fold_window)
    cfg.node_group = int(node_group)
    cfg.stream = _stream_handle(stream)
    return cfg


class VirtualNodeStep:
    """Owns one vf_ctx.  Tensors are torch device tensors used as plain memory."""

    def __init__(self, cfg: VfConfig):
        self._h = C.c_void_p()
        self._cfg = cfg
        _check(lib().vf_init(C.byref(cfg), C.byref(self._h)), "vf_init")

    @classmethod
    def for_workload(cls, wl, **kw) -> "VirtualNodeStep":
        return cls(config_from_workload(wl, **kw))

    def close(self):
        if self._h:
            lib().vf_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def num_params(self) -> int:
        return int(lib().vf_num_params(self._h))

    @property
    def workspace_bytes(self) -> int:
        return int(lib().vf_workspace_bytes(self._h))

    @property
    def fold_window(self) -> int:
        return int(lib().vf_fold_window(self._h))

    @property
    def streams(self) -> int:
        return int(lib().vf_streams(self._h))

    @property
    def step_count(self) -> int:
        return int(lib().vf_step_count(self._h))

    def step(self, params, batch_x, batch_y, node_sizes: Sequence[int]):
        """vf_step: params fp32 [P] (updated in place), batch_x, batch_y device tensors."""
        V = len(node_sizes)
        sizes = (C.c_int32 * max(V, 1))(*[int(b) for b in node_sizes])
        B = int(batch_x.shape[0])
        rc = lib().vf_step(self._h, _ptr(params), _ptr(batch_x), _ptr(batch_y), B, V, sizes)
        _check(rc, "vf_step")

    def prefetch(self, host_x, host_y):
        """vf_prefetch: host_x, host_y are (pinned) host tensors laid out like step's batch."""
        rc = lib().vf_prefetch(self._h, _ptr(host_x), _ptr(host_y), int(host_x.shape[0]))
        _check(rc, "vf_prefetch")

    def step_prefetched(self, params, node_sizes: Sequence[int]):
        V = len(node_sizes)
        sizes = (C.c_int32 * max(V, 1))(*[int(b) for b in node_sizes])
        _check(lib().vf_step_prefetched(self._h, _ptr(params), V, sizes), "vf_step_prefetched")

    def step_raw(self, params_ptr: int, x_ptr: int, y_ptr: int, B: int, V: int, node_sizes) -> int:
        """vf_step with raw pointers and sizes; returns the status code (for error tests)."""
        n = len(node_sizes) if node_sizes is not None else 0
        sizes = (C.c_int32 * max(n, 1))(*[int(b) for b in (node_sizes or [])]) if node_sizes is not None else None
        return int(lib().vf_step(self._h, params_ptr, x_ptr, y_ptr, int(B), int(V), sizes))

    def profile_start(self):
        _check(lib().vf_profile_start(self._h), "vf_profile_start")

    def profile_stop(self) -> dict:
        import json
        buf = C.create_string_buffer(1 << 16)
        _check(lib().vf_profile_stop(self._h, buf, len(buf)), "vf_profile_stop")
        return json.loads(buf.value.decode())

    def grads(self, out):
        _check(lib().vf_grads(self._h, _ptr(out)), "vf_grads")
        return out

    def loss(self) -> float:
        v = C.c_float()
        _check(lib().vf_loss(self._h, C.byref(v)), "vf_loss")
        return float(v.value)

    def node_losses(self, V: int) -> np.ndarray:
        buf = (C.c_float * V)()
        _check(lib().vf_node_losses(self._h, buf, V), "vf_node_losses")
        return np.array(buf[:V], dtype=np.float32)

    @property
    def state_bytes(self) -> int:
        return int(lib().vf_state_bytes(self._h))

    def state_export(self, params, out=None):
        """vf_state_export into `out` (a uint8 torch tensor on the device or the host, or None for
        a new host numpy buffer).  Returns `out`."""
        n = self.state_bytes
        if out is None:
            out = np.empty(n, dtype=np.uint8)
        ptr = out.ctypes.data if isinstance(out, np.ndarray) else _ptr(out)
        size = out.nbytes if isinstance(out, np.ndarray) else out.numel() * out.element_size()
        _check(lib().vf_state_export(self._h, _ptr(params), ptr, size), "vf_state_export")
        return out

    def state_import(self, params, payload):
        ptr = payload.ctypes.data if isinstance(payload, np.ndarray) else _ptr(payload)
        size = payload.nbytes if isinstance(payload, np.ndarray) else payload.numel() * payload.element_size()
        _check(lib().vf_state_import(self._h, _ptr(params), ptr, size), "vf_state_import")

    def opt_state(self, which: int, out):
        _check(lib().vf_opt_state(self._h, which, _ptr(out)), "vf_opt_state")
        return out

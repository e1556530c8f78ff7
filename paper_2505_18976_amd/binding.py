"""ctypes binding of libgrass.so: argument marshalling only.

Every function mirrors one C entry point of include/grass.h with the same
name.  Tensors are torch CUDA (ROCm) tensors used purely as device memory;
their `data_ptr()` and the current HIP stream are handed to the library.  No
step of the compression path runs in Python or in torch ops, and there is no
fallback: if the library is missing, loading fails loudly.
"""
from __future__ import annotations

import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libgrass.so")

GRASS_OK, GRASS_EINVAL, GRASS_EWORKSPACE, GRASS_EHIP, GRASS_EUNSUPPORTED, GRASS_ETOOLARGE = range(6)
GRASS_NOALLOC_SCRATCH_BYTES = 32 << 20
GRASS_MAX_K = 32768
GRASS_MAX_FACTOR = 128

_u64, _u32, _sz, _vp, _int = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int

class FactgrassLayer(ctypes.Structure):
    """Mirror of `factgrass_layer` in include/grass.h."""
    _fields_ = [("x", _vp), ("gout", _vp), ("idx_in", _vp), ("idx_out", _vp),
                ("d_in", _u32), ("d_out", _u32), ("stream_id", _u64), ("out", _vp)]


class GrassTuning(ctypes.Structure):
    """Mirror of `grass_tuning` in include/grass.h (launch-shape overrides of one call; 0 = heuristic)."""
    _fields_ = [("sjlt_rows_per_block", _int), ("sjlt_column_chunks", _int), ("sjlt_threads", _int),
                ("sjlt_accumulator", _int), ("factgrass_tokens_per_block", _int)]


_tun = ctypes.POINTER(GrassTuning)

# name -> (restype, argtypes); the list the ABI test checks against the header.
SIGNATURES = {
    "grass_strerror": (ctypes.c_char_p, [_int]),
    "grass_version": (_int, []),
    "grass_mask_indices_workspace_bytes": (_int, [_u64, _u32, ctypes.POINTER(_sz)]),
    "grass_mask_indices": (_int, [_u64, _u64, _u64, _u32, _vp, _vp, _sz, _vp]),
    "grass_check_indices": (_int, [_vp, _u32, _u64, ctypes.POINTER(_int), _vp]),
    "grass_mask": (_int, [_vp, _u64, _u64, _u64, _vp, _u32, _vp, _u64, _vp]),
    "grass_sjlt_tables": (_int, [_u64, _u64, _u64, _u32, _u32, _vp, _vp, _vp]),
    "grass_sjlt_workspace_bytes": (_int, [_u64, _u64, _u32, _u32, _u32, _tun, ctypes.POINTER(_sz)]),
    "grass_sjlt": (_int, [_vp, _u64, _u64, _u64, _vp, _u32, _u32, _u32, _u64, _u64, _vp, _u64, _vp, _sz, _tun, _vp]),
    "grass_sjlt_bf16": (_int, [_vp, _u64, _u64, _u64, _vp, _u32, _u32, _u32, _u64, _u64, _vp, _u64, _vp, _sz, _tun,
                               _vp]),
    "grass_sjlt_describe": (_int, [_vp, _int, _u64, _u64, _u64, _u32, _u32, _u32, _int, _tun, ctypes.c_char_p, _sz]),
    "grass_sjlt_noalloc": (_int, [_vp, _u64, _u64, _u64, _vp, _u32, _u32, _u32, _u64, _u64, _vp, _u64, _vp]),
    "factgrass_linear_workspace_bytes": (_int, [_u64, _u64, _u32, _u32, _u32, _u32, _tun, ctypes.POINTER(_sz)]),
    "factgrass_linear": (_int, [_vp, _vp, _u64, _u64, _u32, _u32, _vp, _u32, _vp, _u32, _u32, _u32, _u64, _u64,
                                _vp, _u64, _vp, _sz, _tun, _vp]),
    "factgrass_layers_workspace_bytes": (_int, [_u32, _u64, _u64, _u32, _u32, _u32, _u32, _tun, ctypes.POINTER(_sz)]),
    "factgrass_layers": (_int, [ctypes.POINTER(FactgrassLayer), _u32, _u64, _u64, _u32, _u32, _u32, _u32, _u64, _u64,
                                _vp, _sz, _tun, _vp]),
    "logra_linear_workspace_bytes": (_int, [_u64, _u64, _u32, _u32, ctypes.POINTER(_sz)]),
    "logra_linear": (_int, [_vp, _vp, _u64, _u64, _u32, _u32, _vp, _u32, _vp, _u32, _vp, _u64, _vp, _sz, _vp]),
    "grass_score_workspace_bytes": (_int, [_u64, _u64, _u64, _int, ctypes.POINTER(_sz)]),
    "grass_score": (_int, [_vp, _vp, _int, _u64, _u64, _u64, _u64, _u64, _vp, _u64, _vp, _sz, _vp]),
    "grass_to_bf16": (_int, [_vp, _u64, _u64, _u64, _vp, _u64, _vp]),
    "grass_score_bf16": (_int, [_vp, _vp, _u64, _u64, _u64, _u64, _u64, _vp, _u64, _vp]),
    "grass_gauss_matrix": (_int, [_u64, _u64, _u64, _u32, _u64, _u64, _vp, _u64, _vp]),
    "grass_gauss_project_workspace_bytes": (_int, [_u64, _u64, _u32, _u64, ctypes.POINTER(_sz)]),
    "grass_gauss_project": (_int, [_vp, _u64, _u64, _u64, _u32, _u64, _u64, _u64, _int, _vp, _u64, _vp, _sz, _vp]),
    "grass_fim_workspace_bytes": (_int, [_u64, _u32, ctypes.POINTER(_sz)]),
    "grass_fim": (_int, [_vp, _u64, _u32, _u64, _vp, _u64, _vp, _sz, _vp]),
    "grass_fim_inverse_workspace_bytes": (_int, [_u32, ctypes.POINTER(_sz)]),
    "grass_fim_inverse": (_int, [_vp, _u32, _u64, ctypes.c_double, _vp, _u64, _vp, _vp, _sz, _vp]),
    "grass_ifvp": (_int, [_vp, _u64, _u32, _u64, _vp, _u64, _vp, _u64, _vp]),
    "grass_selective_mask_grad_workspace_bytes": (_int, [_u64, _u64, _u64, ctypes.POINTER(_sz)]),
    "grass_selective_mask_grad": (_int, [_vp, _u64, _u64, _vp, _u64, _u64, _u64, _vp, _u64, _vp, ctypes.c_double,
                                         ctypes.c_double, _vp, _vp, _vp, _sz, _vp]),
    "grass_selective_mask_train_workspace_bytes": (_int, [_u64, _u64, _u64, ctypes.POINTER(_sz)]),
    "grass_selective_mask_train": (_int, [_vp, _u64, _u64, _vp, _u64, _u64, _u64, _vp, _u64, _vp, ctypes.c_double,
                                          ctypes.c_double, ctypes.POINTER(ctypes.c_double), _u32, _vp, _vp, _sz, _vp]),
    "grass_score_correlation_workspace_bytes": (_int, [_u64, ctypes.POINTER(_sz)]),
    "grass_score_correlation": (_int, [_vp, _u64, _vp, _u64, _u64, _u64, _vp, _vp, _sz, _vp]),
    "grass_selective_mask_grad_factorized_workspace_bytes": (_int, [_u64, _u64, _u64, _u64, ctypes.POINTER(_sz)]),
    "grass_selective_mask_grad_factorized": (_int, [_vp, _vp, _u64, _u64, _u64, _vp, _vp, _u64, _u64, _u64, _u64, _u64,
                                                    _vp, _u64, _vp, _vp, ctypes.c_double, ctypes.c_double, _vp, _vp, _vp,
                                                    _vp, _sz, _vp]),
    "grass_graddot_factorized_workspace_bytes": (_int, [_u64, _u64, _u64, _u64, _u64, _u64, ctypes.POINTER(_sz)]),
    "grass_graddot_factorized": (_int, [_vp, _vp, _u64, _u64, _u64, _u64, _vp, _vp, _u64, _u64, _u64, _u64, _u64, _u64,
                                        _vp, _u64, _vp, _sz, _vp]),
    "grass_selective_mask_grad_factorized_seq_workspace_bytes": (_int, [_u64, _u64, _u64, _u64, _u64, _u64,
                                                                        ctypes.POINTER(_sz)]),
    "grass_selective_mask_grad_factorized_seq": (_int, [_vp, _vp, _u64, _u64, _u64, _u64, _vp, _vp, _u64, _u64, _u64, _u64,
                                                        _u64, _u64, _vp, _u64, _vp, _vp, ctypes.c_double, ctypes.c_double,
                                                        _vp, _vp, _vp, _vp, _sz, _vp]),
    "grass_selective_mask_train_factorized_workspace_bytes": (_int, [_u64, _u64, _u64, _u64, ctypes.POINTER(_sz)]),
    "grass_selective_mask_train_factorized": (_int, [_vp, _vp, _u64, _u64, _u64, _vp, _vp, _u64, _u64, _u64, _u64, _u64,
                                                     _vp, _u64, _vp, _vp, ctypes.c_double, ctypes.c_double,
                                                     ctypes.POINTER(ctypes.c_double), _u32, _vp, _vp, _sz, _vp]),
    "grass_selective_mask_train_factorized_seq_workspace_bytes": (_int, [_u64, _u64, _u64, _u64, _u64, _u64,
                                                                         ctypes.POINTER(_sz)]),
    "grass_selective_mask_train_factorized_seq": (_int, [_vp, _vp, _u64, _u64, _u64, _u64, _vp, _vp, _u64, _u64, _u64, _u64,
                                                         _u64, _u64, _vp, _u64, _vp, _vp, ctypes.c_double, ctypes.c_double,
                                                         ctypes.POINTER(ctypes.c_double), _u32, _vp, _vp, _sz, _vp]),
    "grass_selective_mask_indices_workspace_bytes": (_int, [_u64, ctypes.POINTER(_sz)]),
    "grass_selective_mask_indices": (_int, [_vp, _u64, _u32, _vp, _vp, _vp, _sz, _vp]),
    "factmask_linear_workspace_bytes": (_int, [_u64, _u64, _u32, _u32, ctypes.POINTER(_sz)]),
    "factmask_linear": (_int, [_vp, _vp, _u64, _u64, _u32, _u32, _vp, _u32, _vp, _u32, _vp, _u64, _vp, _sz, _vp]),
    "grass_projection_matrix": (_int, [_u64, _u64, _u64, _vp, _u32, _u32, _u32, _vp, _u64, _vp]),
    "grass_probe_line_reads": (_int, [_vp, _u64, _vp, _u64, _int, _u64, _u32, _vp]),
}

_lib = None


class GrassError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


def load_library() -> ctypes.CDLL:
    """Loads libgrass.so from the package directory.  Raises if it was not built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2505_18976_amd.build` "
            "(there is no fallback implementation)")
    lib = ctypes.CDLL(LIB_PATH)
    for name, (res, args) in SIGNATURES.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def strerror(status: int) -> str:
    return load_library().grass_strerror(int(status)).decode()


def _check(status: int, where: str):
    if status != GRASS_OK:
        raise GrassError(status, where)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _ld(t: torch.Tensor) -> int:
    assert t.dim() == 2 and t.stride(1) == 1, "row-major matrix expected"
    return t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])


def _tuning(tuning):
    """None, a GrassTuning, or a dict of its fields -> pointer argument."""
    if tuning is None:
        return None
    if isinstance(tuning, dict):
        tuning = GrassTuning(**tuning)
    return ctypes.byref(tuning)


def _workspace(nbytes: int, device) -> torch.Tensor | None:
    if nbytes == 0:
        return None
    return torch.empty(nbytes, dtype=torch.uint8, device=device)   # torch allocations are >= 256-byte aligned


def grass_version() -> int:
    return load_library().grass_version()


def grass_mask_indices_workspace_bytes(p: int, kprime: int) -> int:
    out = _sz(0)
    _check(load_library().grass_mask_indices_workspace_bytes(p, kprime, ctypes.byref(out)),
           "grass_mask_indices_workspace_bytes")
    return out.value


def grass_mask_indices(seed: int, stream_id: int, p: int, kprime: int, device="cuda") -> torch.Tensor:
    ws = _workspace(grass_mask_indices_workspace_bytes(p, kprime), device)
    idx = torch.empty(kprime, dtype=torch.int32, device=device)
    _check(load_library().grass_mask_indices(seed, stream_id, p, kprime, _ptr(idx), _ptr(ws),
                                             0 if ws is None else ws.numel(), _stream()), "grass_mask_indices")
    return idx


def grass_check_indices(idx: torch.Tensor, p: int) -> bool:
    ok = _int(0)
    _check(load_library().grass_check_indices(_ptr(idx), idx.numel(), p, ctypes.byref(ok), _stream()),
           "grass_check_indices")
    return bool(ok.value)


def grass_mask(g: torch.Tensor, idx: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    assert g.dtype == torch.float32 and idx.dtype == torch.int32
    n, p = g.shape
    kprime = idx.numel()
    if out is None:
        out = torch.empty((n, kprime), dtype=torch.float32, device=g.device)
    _check(load_library().grass_mask(_ptr(g), n, p, _ld(g), _ptr(idx), kprime, _ptr(out), _ld(out), _stream()),
           "grass_mask")
    return out


def grass_sjlt_tables(seed: int, stream_id: int, d: int, k: int, s: int, device="cuda"):
    bucket = torch.empty((d, s), dtype=torch.int32, device=device)     # uint32 payload
    sign = torch.empty((d, s), dtype=torch.int8, device=device)
    _check(load_library().grass_sjlt_tables(seed, stream_id, d, k, s, _ptr(bucket), _ptr(sign), _stream()),
           "grass_sjlt_tables")
    return bucket, sign


def grass_sjlt_workspace_bytes(n: int, p: int, kprime_or_0: int, k: int, s: int, tuning=None) -> int:
    out = _sz(0)
    _check(load_library().grass_sjlt_workspace_bytes(n, p, kprime_or_0, k, s, _tuning(tuning), ctypes.byref(out)),
           "grass_sjlt_workspace_bytes")
    return out.value


def grass_sjlt(g: torch.Tensor, k: int, s: int, seed: int, stream_id: int = 1, idx: torch.Tensor | None = None,
               out: torch.Tensor | None = None, ws: torch.Tensor | None = None, tuning=None) -> torch.Tensor:
    """SJLT_k of the rows of g, or fused GraSS when idx is given."""
    assert g.dtype == torch.float32
    n, p = g.shape
    kprime = 0 if idx is None else idx.numel()
    if out is None:
        out = torch.empty((n, k), dtype=torch.float32, device=g.device)
    if ws is None:
        ws = _workspace(grass_sjlt_workspace_bytes(n, p, kprime, k, s, tuning), g.device)
    _check(load_library().grass_sjlt(_ptr(g), n, p, _ld(g), _ptr(idx), kprime, k, s, seed, stream_id,
                                     _ptr(out), _ld(out), _ptr(ws), 0 if ws is None else ws.numel(), _tuning(tuning),
                                     _stream()),
           "grass_sjlt")
    return out


def grass_sjlt_bf16(g: torch.Tensor, k: int, s: int, seed: int, stream_id: int = 1, idx: torch.Tensor | None = None,
                    out: torch.Tensor | None = None, ws: torch.Tensor | None = None, tuning=None) -> torch.Tensor:
    """grass_sjlt on gradients stored as bf16 (fp32 accumulation and output)."""
    assert g.dtype == torch.bfloat16
    n, p = g.shape
    kprime = 0 if idx is None else idx.numel()
    if out is None:
        out = torch.empty((n, k), dtype=torch.float32, device=g.device)
    if ws is None:
        ws = _workspace(grass_sjlt_workspace_bytes(n, p, kprime, k, s, tuning), g.device)
    _check(load_library().grass_sjlt_bf16(_ptr(g), n, p, _ld(g), _ptr(idx), kprime, k, s, seed, stream_id,
                                          _ptr(out), _ld(out), _ptr(ws), 0 if ws is None else ws.numel(),
                                          _tuning(tuning), _stream()),
           "grass_sjlt_bf16")
    return out


def grass_sjlt_describe(n: int, p: int, ldg: int, kprime_or_0: int, k: int, s: int, g: torch.Tensor | None = None,
                        bf16: bool = False, with_workspace: bool = True, tuning=None) -> str:
    """Kernel instantiation and launch shape grass_sjlt would use (host only, launches nothing)."""
    buf = ctypes.create_string_buffer(256)
    _check(load_library().grass_sjlt_describe(_ptr(g), int(bf16), n, p, ldg, kprime_or_0, k, s, int(with_workspace),
                                              _tuning(tuning), buf, 256), "grass_sjlt_describe")
    return buf.value.decode()


def grass_sjlt_noalloc(g: torch.Tensor, k: int, s: int, seed: int, stream_id: int, out: torch.Tensor,
                       idx: torch.Tensor | None = None) -> torch.Tensor:
    """grass_sjlt without a workspace (the library's own fixed scratch buffer); `out` is the caller's."""
    assert g.dtype == torch.float32 and out.dtype == torch.float32
    n, p = g.shape
    kprime = 0 if idx is None else idx.numel()
    _check(load_library().grass_sjlt_noalloc(_ptr(g), n, p, _ld(g), _ptr(idx), kprime, k, s, seed, stream_id,
                                             _ptr(out), _ld(out), _stream()), "grass_sjlt_noalloc")
    return out


def factgrass_linear_workspace_bytes(n: int, T: int, kin_p: int, kout_p: int, k: int, s: int, tuning=None) -> int:
    out = _sz(0)
    _check(load_library().factgrass_linear_workspace_bytes(n, T, kin_p, kout_p, k, s, _tuning(tuning),
                                                           ctypes.byref(out)),
           "factgrass_linear_workspace_bytes")
    return out.value


def factgrass_linear(x: torch.Tensor, gout: torch.Tensor, idx_in: torch.Tensor, idx_out: torch.Tensor,
                     k: int, s: int, seed: int, stream_id: int, out: torch.Tensor | None = None,
                     ws: torch.Tensor | None = None, tuning=None) -> torch.Tensor:
    assert x.dtype == torch.bfloat16 and gout.dtype == torch.bfloat16
    assert x.is_contiguous() and gout.is_contiguous()
    n, T, d_in = x.shape
    d_out = gout.shape[2]
    assert gout.shape[0] == n and gout.shape[1] == T
    if out is None:
        out = torch.empty((n, k), dtype=torch.float32, device=x.device)
    if ws is None:
        ws = _workspace(factgrass_linear_workspace_bytes(n, T, idx_in.numel(), idx_out.numel(), k, s, tuning),
                        x.device)
    _check(load_library().factgrass_linear(_ptr(x), _ptr(gout), n, T, d_in, d_out, _ptr(idx_in), idx_in.numel(),
                                           _ptr(idx_out), idx_out.numel(), k, s, seed, stream_id, _ptr(out),
                                           _ld(out), _ptr(ws), 0 if ws is None else ws.numel(), _tuning(tuning),
                                           _stream()),
           "factgrass_linear")
    return out


def factgrass_layers_workspace_bytes(n_layers: int, n: int, T: int, kin_p: int, kout_p: int, k: int, s: int,
                                     tuning=None) -> int:
    out = _sz(0)
    _check(load_library().factgrass_layers_workspace_bytes(n_layers, n, T, kin_p, kout_p, k, s, _tuning(tuning),
                                                           ctypes.byref(out)),
           "factgrass_layers_workspace_bytes")
    return out.value


def factgrass_layers(layers, k: int, s: int, seed: int, out: torch.Tensor, ws: torch.Tensor | None = None,
                     tuning=None):
    """layers: list of (x, gout, idx_in, idx_out, stream_id); layer l is written to out[:, l*k:(l+1)*k]."""
    n, T = layers[0][0].shape[0], layers[0][0].shape[1]
    kin_p, kout_p = layers[0][2].numel(), layers[0][3].numel()
    assert out.dtype == torch.float32 and out.shape[0] == n and out.shape[1] >= k * len(layers)
    table = (FactgrassLayer * len(layers))()
    for l, (x, g, ii, io, stream_id) in enumerate(layers):
        assert x.dtype == torch.bfloat16 and g.dtype == torch.bfloat16 and x.is_contiguous() and g.is_contiguous()
        assert x.shape[:2] == (n, T) and g.shape[:2] == (n, T) and ii.numel() == kin_p and io.numel() == kout_p
        table[l] = FactgrassLayer(x.data_ptr(), g.data_ptr(), ii.data_ptr(), io.data_ptr(), x.shape[2], g.shape[2],
                                  stream_id, out.data_ptr() + 4 * l * k)
    if ws is None:
        ws = _workspace(factgrass_layers_workspace_bytes(len(layers), n, T, kin_p, kout_p, k, s, tuning), out.device)
    _check(load_library().factgrass_layers(table, len(layers), n, T, kin_p, kout_p, k, s, seed, _ld(out), _ptr(ws),
                                           0 if ws is None else ws.numel(), _tuning(tuning), _stream()),
           "factgrass_layers")
    return out


def logra_linear_workspace_bytes(n: int, T: int, k_in: int, k_out: int) -> int:
    out = _sz(0)
    _check(load_library().logra_linear_workspace_bytes(n, T, k_in, k_out, ctypes.byref(out)),
           "logra_linear_workspace_bytes")
    return out.value


def logra_linear(x: torch.Tensor, gout: torch.Tensor, P_in: torch.Tensor, P_out: torch.Tensor,
                 out: torch.Tensor | None = None, ws: torch.Tensor | None = None) -> torch.Tensor:
    for t in (x, gout, P_in, P_out):
        assert t.dtype == torch.bfloat16 and t.is_contiguous()
    n, T, d_in = x.shape
    d_out = gout.shape[2]
    k_in, k_out = P_in.shape[0], P_out.shape[0]
    assert P_in.shape[1] == d_in and P_out.shape[1] == d_out and gout.shape[:2] == (n, T)
    if out is None:
        out = torch.empty((n, k_in * k_out), dtype=torch.float32, device=x.device)
    if ws is None:
        ws = _workspace(logra_linear_workspace_bytes(n, T, k_in, k_out), x.device)
    _check(load_library().logra_linear(_ptr(x), _ptr(gout), n, T, d_in, d_out, _ptr(P_in), k_in, _ptr(P_out), k_out,
                                       _ptr(out), _ld(out), _ptr(ws), 0 if ws is None else ws.numel(), _stream()),
           "logra_linear")
    return out


def grass_score_workspace_bytes(N: int, M: int, K: int, compute_mode: int) -> int:
    out = _sz(0)
    _check(load_library().grass_score_workspace_bytes(N, M, K, compute_mode, ctypes.byref(out)),
           "grass_score_workspace_bytes")
    return out.value


def grass_score(train: torch.Tensor, test: torch.Tensor, compute_mode: int = 0,
                out: torch.Tensor | None = None, ws: torch.Tensor | None | bool = True) -> torch.Tensor:
    """scores[m, i] = <test_m, train_i>.  ws: True allocates the optional workspace, None runs without one."""
    assert train.dtype == torch.float32 and test.dtype == torch.float32
    N, K = train.shape
    M = test.shape[0]
    assert test.shape[1] == K
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=train.device)
    if ws is True:
        ws = _workspace(grass_score_workspace_bytes(N, M, K, compute_mode), train.device)
    _check(load_library().grass_score(_ptr(train), _ptr(test), compute_mode, N, M, K, _ld(train), _ld(test),
                                      _ptr(out), _ld(out), _ptr(ws), 0 if ws is None else ws.numel(), _stream()),
           "grass_score")
    return out


def grass_to_bf16(src: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    assert src.dtype == torch.float32
    rows, cols = src.shape
    if out is None:
        out = torch.empty((rows, cols), dtype=torch.bfloat16, device=src.device)
    _check(load_library().grass_to_bf16(_ptr(src), rows, cols, _ld(src), _ptr(out), _ld(out), _stream()),
           "grass_to_bf16")
    return out


def grass_score_bf16(train: torch.Tensor, test: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    assert train.dtype == torch.bfloat16 and test.dtype == torch.bfloat16
    N, K = train.shape
    M = test.shape[0]
    assert test.shape[1] == K
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=train.device)
    _check(load_library().grass_score_bf16(_ptr(train), _ptr(test), N, M, K, _ld(train), _ld(test), _ptr(out),
                                           _ld(out), _stream()), "grass_score_bf16")
    return out


def grass_gauss_matrix(seed: int, stream_id: int, p: int, k: int, p0: int, pc: int, device="cuda") -> torch.Tensor:
    P = torch.empty((k, pc), dtype=torch.float32, device=device)
    _check(load_library().grass_gauss_matrix(seed, stream_id, p, k, p0, pc, _ptr(P), _ld(P), _stream()),
           "grass_gauss_matrix")
    return P


def grass_gauss_project_workspace_bytes(n: int, p: int, k: int, p_chunk: int) -> int:
    out = _sz(0)
    _check(load_library().grass_gauss_project_workspace_bytes(n, p, k, p_chunk, ctypes.byref(out)),
           "grass_gauss_project_workspace_bytes")
    return out.value


def grass_gauss_project(g: torch.Tensor, k: int, seed: int, stream_id: int, p_chunk: int, compute_mode: int = 0,
                        out: torch.Tensor | None = None, ws: torch.Tensor | None = None) -> torch.Tensor:
    assert g.dtype == torch.float32
    n, p = g.shape
    if out is None:
        out = torch.empty((n, k), dtype=torch.float32, device=g.device)
    if ws is None:
        ws = _workspace(grass_gauss_project_workspace_bytes(n, p, k, p_chunk), g.device)
    _check(load_library().grass_gauss_project(_ptr(g), n, p, _ld(g), k, seed, stream_id, p_chunk, compute_mode,
                                              _ptr(out), _ld(out), _ptr(ws), 0 if ws is None else ws.numel(),
                                              _stream()), "grass_gauss_project")
    return out


def grass_fim_workspace_bytes(N: int, k: int) -> int:
    out = _sz(0)
    _check(load_library().grass_fim_workspace_bytes(N, k, ctypes.byref(out)), "grass_fim_workspace_bytes")
    return out.value


def grass_fim(G: torch.Tensor, out: torch.Tensor | None = None, ws: torch.Tensor | None = None) -> torch.Tensor:
    """F = (1/N) G^T G for the rows of G (N x k fp32)."""
    assert G.dtype == torch.float32
    N, k = G.shape
    if out is None:
        out = torch.empty((k, k), dtype=torch.float32, device=G.device)
    if ws is None:
        ws = _workspace(grass_fim_workspace_bytes(N, k), G.device)
    _check(load_library().grass_fim(_ptr(G), N, k, _ld(G), _ptr(out), _ld(out), _ptr(ws),
                                    0 if ws is None else ws.numel(), _stream()), "grass_fim")
    return out


def grass_fim_inverse_workspace_bytes(k: int) -> int:
    out = _sz(0)
    _check(load_library().grass_fim_inverse_workspace_bytes(k, ctypes.byref(out)), "grass_fim_inverse_workspace_bytes")
    return out.value


def grass_fim_inverse(F: torch.Tensor, lam: float, out: torch.Tensor | None = None, info: torch.Tensor | None = None,
                      ws: torch.Tensor | None = None) -> torch.Tensor:
    """W = (F + lam*I)^{-1}; `info` (int32 device tensor of one element) receives the pivot status if given."""
    assert F.dtype == torch.float32 and F.shape[0] == F.shape[1]
    k = F.shape[0]
    if out is None:
        out = torch.empty((k, k), dtype=torch.float32, device=F.device)
    if ws is None:
        ws = _workspace(grass_fim_inverse_workspace_bytes(k), F.device)
    assert info is None or (info.dtype == torch.int32 and info.numel() >= 1)
    _check(load_library().grass_fim_inverse(_ptr(F), k, _ld(F), float(lam), _ptr(out), _ld(out), _ptr(info), _ptr(ws),
                                            0 if ws is None else ws.numel(), _stream()), "grass_fim_inverse")
    return out


def grass_ifvp(G: torch.Tensor, W: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """Row i of the result is W g_i (W symmetric, from grass_fim_inverse)."""
    assert G.dtype == torch.float32 and W.dtype == torch.float32
    N, k = G.shape
    assert W.shape == (k, k)
    if out is None:
        out = torch.empty((N, k), dtype=torch.float32, device=G.device)
    _check(load_library().grass_ifvp(_ptr(G), N, k, _ld(G), _ptr(W), _ld(W), _ptr(out), _ld(out), _stream()),
           "grass_ifvp")
    return out


def grass_selective_mask_grad_workspace_bytes(n: int, m: int, p: int) -> int:
    out = _sz(0)
    _check(load_library().grass_selective_mask_grad_workspace_bytes(n, m, p, ctypes.byref(out)),
           "grass_selective_mask_grad_workspace_bytes")
    return out.value


def grass_selective_mask_grad(G: torch.Tensor, Gt: torch.Tensor, A: torch.Tensor, S: torch.Tensor, lam: float,
                              temperature: float = 1.0, grad: torch.Tensor | None = None,
                              objective: torch.Tensor | None = None, ws: torch.Tensor | None = None):
    """Objective of the Selective Mask problem and its gradient with respect to the logits S.
    A = grass_score(G, Gt) holds the exact scores.  Returns (grad fp32 [p], objective float64 [1])."""
    assert G.dtype == Gt.dtype == A.dtype == S.dtype == torch.float32 and S.is_contiguous()
    n, p = G.shape
    m = Gt.shape[0]
    assert Gt.shape[1] == p and A.shape == (m, n) and S.numel() == p
    if grad is None:
        grad = torch.empty(p, dtype=torch.float32, device=G.device)
    if objective is None:
        objective = torch.empty(1, dtype=torch.float64, device=G.device)
    if ws is None:
        ws = _workspace(grass_selective_mask_grad_workspace_bytes(n, m, p), G.device)
    _check(load_library().grass_selective_mask_grad(_ptr(G), n, _ld(G), _ptr(Gt), m, _ld(Gt), p, _ptr(A), _ld(A), _ptr(S),
                                                    float(lam), float(temperature), _ptr(grad), _ptr(objective), _ptr(ws),
                                                    0 if ws is None else ws.numel(), _stream()),
           "grass_selective_mask_grad")
    return grad, objective


def grass_selective_mask_train_workspace_bytes(n: int, m: int, p: int) -> int:
    out = _sz(0)
    _check(load_library().grass_selective_mask_train_workspace_bytes(n, m, p, ctypes.byref(out)),
           "grass_selective_mask_train_workspace_bytes")
    return out.value


def grass_selective_mask_train(G: torch.Tensor, Gt: torch.Tensor, A: torch.Tensor, S: torch.Tensor, lam: float, lr: float,
                               temperatures, objectives: torch.Tensor | None = None, ws: torch.Tensor | None = None):
    """len(temperatures) gradient-ascent steps on the logits S (updated in place), step i at temperatures[i].
    Returns (S, objectives float64 [steps]: the objective before each step)."""
    assert G.dtype == Gt.dtype == A.dtype == S.dtype == torch.float32 and S.is_contiguous()
    n, p = G.shape
    m = Gt.shape[0]
    assert Gt.shape[1] == p and A.shape == (m, n) and S.numel() == p
    steps = len(temperatures)
    sched = (ctypes.c_double * max(steps, 1))(*[float(t) for t in temperatures])
    if objectives is None:
        objectives = torch.empty(max(steps, 1), dtype=torch.float64, device=G.device)
    if ws is None:
        ws = _workspace(grass_selective_mask_train_workspace_bytes(n, m, p), G.device)
    _check(load_library().grass_selective_mask_train(_ptr(G), n, _ld(G), _ptr(Gt), m, _ld(Gt), p, _ptr(A), _ld(A), _ptr(S),
                                                     float(lam), float(lr), sched, steps, _ptr(objectives), _ptr(ws),
                                                     ws.numel(), _stream()), "grass_selective_mask_train")
    return S, objectives[:steps]


def grass_score_correlation(X: torch.Tensor, Y: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """Mean over rows of the Pearson correlation between matching rows of two m x n score matrices (float64 [1])."""
    assert X.dtype == Y.dtype == torch.float32 and X.shape == Y.shape
    m, n = X.shape
    if out is None:
        out = torch.empty(1, dtype=torch.float64, device=X.device)
    nbytes = _sz(0)
    _check(load_library().grass_score_correlation_workspace_bytes(m, ctypes.byref(nbytes)),
           "grass_score_correlation_workspace_bytes")
    ws = _workspace(nbytes.value, X.device)
    _check(load_library().grass_score_correlation(_ptr(X), _ld(X), _ptr(Y), _ld(Y), m, n, _ptr(out), _ptr(ws), ws.numel(),
                                                  _stream()), "grass_score_correlation")
    return out


def grass_selective_mask_grad_factorized(Z_in, Z_out, Zt_in, Zt_out, A, S_in, S_out, lam: float, temperature: float = 1.0):
    """Factorised Selective Mask step of a linear layer.  Returns (grad_in, grad_out, objective float64 [1])."""
    for t in (Z_in, Z_out, Zt_in, Zt_out, A, S_in, S_out):
        assert t.dtype == torch.float32
    n, d_in = Z_in.shape
    d_out = Z_out.shape[1]
    m = Zt_in.shape[0]
    assert Z_out.shape[0] == n and Zt_in.shape[1] == d_in and Zt_out.shape == (m, d_out) and A.shape == (m, n)
    assert S_in.is_contiguous() and S_out.is_contiguous() and S_in.numel() == d_in and S_out.numel() == d_out
    grad_in = torch.empty(d_in, dtype=torch.float32, device=Z_in.device)
    grad_out = torch.empty(d_out, dtype=torch.float32, device=Z_in.device)
    objective = torch.empty(1, dtype=torch.float64, device=Z_in.device)
    nbytes = _sz(0)
    _check(load_library().grass_selective_mask_grad_factorized_workspace_bytes(n, m, d_in, d_out, ctypes.byref(nbytes)),
           "grass_selective_mask_grad_factorized_workspace_bytes")
    ws = _workspace(nbytes.value, Z_in.device)
    _check(load_library().grass_selective_mask_grad_factorized(
        _ptr(Z_in), _ptr(Z_out), n, _ld(Z_in), _ld(Z_out), _ptr(Zt_in), _ptr(Zt_out), m, _ld(Zt_in), _ld(Zt_out), d_in, d_out,
        _ptr(A), _ld(A), _ptr(S_in), _ptr(S_out), float(lam), float(temperature), _ptr(grad_in), _ptr(grad_out),
        _ptr(objective), _ptr(ws), ws.numel(), _stream()), "grass_selective_mask_grad_factorized")
    return grad_in, grad_out, objective


def _seq_shapes(Z_in, Z_out, Zt_in, Zt_out):
    """(n, T, d) token tensors, contiguous over (sample, token): returns the flattened (n*T, d) views and the sizes."""
    for t in (Z_in, Z_out, Zt_in, Zt_out):
        assert t.dtype == torch.float32 and t.dim() == 3
    n, T, d_in = Z_in.shape
    m, Tt, d_out = Zt_out.shape
    assert Z_out.shape[:2] == (n, T) and Z_out.shape[2] == d_out and Zt_in.shape == (m, Tt, d_in)
    flat = [t.reshape(t.shape[0] * t.shape[1], t.shape[2]) for t in (Z_in, Z_out, Zt_in, Zt_out)]
    return flat, n, T, m, Tt, d_in, d_out


def grass_graddot_factorized(Z_in, Z_out, Zt_in, Zt_out, out: torch.Tensor | None = None) -> torch.Tensor:
    """Exact GradDot scores (m x n) of a linear layer on sequences: Z_* are (samples, tokens, features) tensors."""
    (zi, zo, zti, zto), n, T, m, Tt, d_in, d_out = _seq_shapes(Z_in, Z_out, Zt_in, Zt_out)
    if out is None:
        out = torch.empty((m, n), dtype=torch.float32, device=Z_in.device)
    nbytes = _sz(0)
    _check(load_library().grass_graddot_factorized_workspace_bytes(n, T, m, Tt, d_in, d_out, ctypes.byref(nbytes)),
           "grass_graddot_factorized_workspace_bytes")
    ws = _workspace(nbytes.value, Z_in.device)
    _check(load_library().grass_graddot_factorized(_ptr(zi), _ptr(zo), n, T, _ld(zi), _ld(zo), _ptr(zti), _ptr(zto), m, Tt,
                                                   _ld(zti), _ld(zto), d_in, d_out, _ptr(out), _ld(out), _ptr(ws),
                                                   ws.numel(), _stream()), "grass_graddot_factorized")
    return out


def grass_selective_mask_grad_factorized_seq(Z_in, Z_out, Zt_in, Zt_out, A, S_in, S_out, lam: float,
                                             temperature: float = 1.0):
    """Factorised Selective Mask step of a linear layer on sequences ((samples, tokens, features) tensors).
    Returns (grad_in, grad_out, objective float64 [1])."""
    (zi, zo, zti, zto), n, T, m, Tt, d_in, d_out = _seq_shapes(Z_in, Z_out, Zt_in, Zt_out)
    assert A.dtype == S_in.dtype == S_out.dtype == torch.float32 and A.shape == (m, n)
    assert S_in.is_contiguous() and S_out.is_contiguous() and S_in.numel() == d_in and S_out.numel() == d_out
    grad_in = torch.empty(d_in, dtype=torch.float32, device=Z_in.device)
    grad_out = torch.empty(d_out, dtype=torch.float32, device=Z_in.device)
    objective = torch.empty(1, dtype=torch.float64, device=Z_in.device)
    nbytes = _sz(0)
    _check(load_library().grass_selective_mask_grad_factorized_seq_workspace_bytes(n, T, m, Tt, d_in, d_out,
                                                                                   ctypes.byref(nbytes)),
           "grass_selective_mask_grad_factorized_seq_workspace_bytes")
    ws = _workspace(nbytes.value, Z_in.device)
    _check(load_library().grass_selective_mask_grad_factorized_seq(
        _ptr(zi), _ptr(zo), n, T, _ld(zi), _ld(zo), _ptr(zti), _ptr(zto), m, Tt, _ld(zti), _ld(zto), d_in, d_out,
        _ptr(A), _ld(A), _ptr(S_in), _ptr(S_out), float(lam), float(temperature), _ptr(grad_in), _ptr(grad_out),
        _ptr(objective), _ptr(ws), ws.numel(), _stream()), "grass_selective_mask_grad_factorized_seq")
    return grad_in, grad_out, objective


def grass_selective_mask_train_factorized(Z_in, Z_out, Zt_in, Zt_out, A, S_in, S_out, lam: float, lr: float, temperatures,
                                          objectives: torch.Tensor | None = None):
    """len(temperatures) gradient-ascent steps on both logit vectors of a linear layer's factorised mask (updated in
    place), step i at temperatures[i].  Returns (S_in, S_out, objectives float64 [steps])."""
    for t in (Z_in, Z_out, Zt_in, Zt_out, A, S_in, S_out):
        assert t.dtype == torch.float32
    n, d_in = Z_in.shape
    d_out = Z_out.shape[1]
    m = Zt_in.shape[0]
    assert Z_out.shape[0] == n and Zt_in.shape[1] == d_in and Zt_out.shape == (m, d_out) and A.shape == (m, n)
    assert S_in.is_contiguous() and S_out.is_contiguous() and S_in.numel() == d_in and S_out.numel() == d_out
    steps = len(temperatures)
    sched = (ctypes.c_double * max(steps, 1))(*[float(t) for t in temperatures])
    if objectives is None:
        objectives = torch.empty(max(steps, 1), dtype=torch.float64, device=Z_in.device)
    nbytes = _sz(0)
    _check(load_library().grass_selective_mask_train_factorized_workspace_bytes(n, m, d_in, d_out, ctypes.byref(nbytes)),
           "grass_selective_mask_train_factorized_workspace_bytes")
    ws = _workspace(nbytes.value, Z_in.device)
    _check(load_library().grass_selective_mask_train_factorized(
        _ptr(Z_in), _ptr(Z_out), n, _ld(Z_in), _ld(Z_out), _ptr(Zt_in), _ptr(Zt_out), m, _ld(Zt_in), _ld(Zt_out), d_in, d_out,
        _ptr(A), _ld(A), _ptr(S_in), _ptr(S_out), float(lam), float(lr), sched, steps, _ptr(objectives), _ptr(ws),
        ws.numel(), _stream()), "grass_selective_mask_train_factorized")
    return S_in, S_out, objectives[:steps]


def grass_selective_mask_train_factorized_seq(Z_in, Z_out, Zt_in, Zt_out, A, S_in, S_out, lam: float, lr: float,
                                              temperatures, objectives: torch.Tensor | None = None):
    """grass_selective_mask_train_factorized on sequences ((samples, tokens, features) tensors).
    Returns (S_in, S_out, objectives float64 [steps])."""
    (zi, zo, zti, zto), n, T, m, Tt, d_in, d_out = _seq_shapes(Z_in, Z_out, Zt_in, Zt_out)
    assert A.dtype == S_in.dtype == S_out.dtype == torch.float32 and A.shape == (m, n)
    assert S_in.is_contiguous() and S_out.is_contiguous() and S_in.numel() == d_in and S_out.numel() == d_out
    steps = len(temperatures)
    sched = (ctypes.c_double * max(steps, 1))(*[float(t) for t in temperatures])
    if objectives is None:
        objectives = torch.empty(max(steps, 1), dtype=torch.float64, device=Z_in.device)
    nbytes = _sz(0)
    _check(load_library().grass_selective_mask_train_factorized_seq_workspace_bytes(n, T, m, Tt, d_in, d_out,
                                                                                    ctypes.byref(nbytes)),
           "grass_selective_mask_train_factorized_seq_workspace_bytes")
    ws = _workspace(nbytes.value, Z_in.device)
    _check(load_library().grass_selective_mask_train_factorized_seq(
        _ptr(zi), _ptr(zo), n, T, _ld(zi), _ld(zo), _ptr(zti), _ptr(zto), m, Tt, _ld(zti), _ld(zto), d_in, d_out,
        _ptr(A), _ld(A), _ptr(S_in), _ptr(S_out), float(lam), float(lr), sched, steps, _ptr(objectives), _ptr(ws),
        ws.numel(), _stream()), "grass_selective_mask_train_factorized_seq")
    return S_in, S_out, objectives[:steps]


def grass_selective_mask_indices_workspace_bytes(p: int) -> int:
    out = _sz(0)
    _check(load_library().grass_selective_mask_indices_workspace_bytes(p, ctypes.byref(out)),
           "grass_selective_mask_indices_workspace_bytes")
    return out.value


def grass_selective_mask_indices(S: torch.Tensor, k: int = 0) -> torch.Tensor:
    """k == 0: every j with sigmoid(S_j) >= 1/2, ascending (reads the count back, which synchronises);
    k > 0: the k largest logits, ascending."""
    assert S.dtype == torch.float32 and S.is_contiguous()
    p = S.numel()
    idx = torch.empty(p if k == 0 else k, dtype=torch.int32, device=S.device)
    count = torch.zeros(1, dtype=torch.int32, device=S.device)
    ws = _workspace(grass_selective_mask_indices_workspace_bytes(p), S.device)
    _check(load_library().grass_selective_mask_indices(_ptr(S), p, k, _ptr(idx), _ptr(count), _ptr(ws), ws.numel(),
                                                       _stream()), "grass_selective_mask_indices")
    return idx[: int(count.item())] if k == 0 else idx


def factmask_linear_workspace_bytes(n: int, T: int, kin_p: int, kout_p: int) -> int:
    out = _sz(0)
    _check(load_library().factmask_linear_workspace_bytes(n, T, kin_p, kout_p, ctypes.byref(out)),
           "factmask_linear_workspace_bytes")
    return out.value


def factmask_linear(x: torch.Tensor, gout: torch.Tensor, idx_in: torch.Tensor, idx_out: torch.Tensor,
                    out: torch.Tensor | None = None, ws: torch.Tensor | None = None) -> torch.Tensor:
    """Mask_{k_in x k_out}: sum_t x_t[idx_in] (x) g_t[idx_out], flat index a*k_out' + b."""
    assert x.dtype == torch.bfloat16 and gout.dtype == torch.bfloat16
    assert x.is_contiguous() and gout.is_contiguous()
    n, T, d_in = x.shape
    d_out = gout.shape[2]
    ka, kb = idx_in.numel(), idx_out.numel()
    if out is None:
        out = torch.empty((n, ka * kb), dtype=torch.float32, device=x.device)
    if ws is None:
        ws = _workspace(factmask_linear_workspace_bytes(n, T, ka, kb), x.device)
    _check(load_library().factmask_linear(_ptr(x), _ptr(gout), n, T, d_in, d_out, _ptr(idx_in), ka, _ptr(idx_out), kb,
                                          _ptr(out), _ld(out), _ptr(ws), 0 if ws is None else ws.numel(), _stream()),
           "factmask_linear")
    return out


def grass_projection_matrix(seed: int, stream_id: int, p: int, k: int, s: int, idx: torch.Tensor | None = None,
                            device="cuda") -> torch.Tensor:
    """The SJLT (idx None) or GraSS (idx given) compressor as a dense k x p fp32 matrix."""
    P = torch.empty((k, p), dtype=torch.float32, device=device)
    kprime = 0 if idx is None else idx.numel()
    _check(load_library().grass_projection_matrix(seed, stream_id, p, _ptr(idx), kprime, k, s, _ptr(P), _ld(P), _stream()),
           "grass_projection_matrix")
    return P


def grass_probe_line_reads(src: torch.Tensor, dst: torch.Tensor, mode: int, salt: int, blocks: int) -> None:
    """Measurement aid: blocks * 256 * 16 pseudo-random line reads of src (fp32), see include/grass.h."""
    assert src.dtype == dst.dtype == torch.float32 and src.is_contiguous() and dst.is_contiguous()
    _check(load_library().grass_probe_line_reads(_ptr(src), src.numel(), _ptr(dst), dst.numel(), int(mode), int(salt),
                                                 int(blocks), _stream()), "grass_probe_line_reads")

"""ctypes binding of libapproxifer.so: same names as the C ABI, argument marshalling only.

Tensors are torch CUDA (ROCm) tensors used purely as device buffers; every step of the
coding layer runs inside the library's HIP kernels.  There is no CPU fallback: if the
library is missing the loader raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libapproxifer.so")

MAX_K = 64
MAX_N = 128
MAX_AVAIL_BYZ = 64
SIGN_WORKER_INDEX = 0
SIGN_SURVIVOR_RANK = 1
S_FROM_MASK = -1

EXPORTS = (
    "approxifer_version",
    "approxifer_wait_mask",
    "approxifer_strerror",
    "approxifer_chebyshev_nodes",
    "approxifer_encode",
    "approxifer_decode",
    "approxifer_decode_top1",
    "approxifer_decode_byzantine",
    "approxifer_decode_byzantine_homogeneous",
    "approxifer_workspace_bytes",
    "approxifer_decode_byzantine_static",
    "approxifer_decode_rational",
    "approxifer_group_count",
    "approxifer_pad_last_group",
    "approxifer_top1",
)

_lib = None


class ApproxiferError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("approxifer error %d: %s" % (code, text))
        self.code = code


def load() -> ctypes.CDLL:
    """Load the HIP library built in-tree.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            "%s is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'). "
            "There is no fallback path." % LIB_PATH
        )
    lib = ctypes.CDLL(LIB_PATH)
    c_dp = ctypes.POINTER(ctypes.c_double)
    vp = ctypes.c_void_p
    lib.approxifer_version.restype = ctypes.c_int
    lib.approxifer_version.argtypes = []
    lib.approxifer_strerror.restype = ctypes.c_char_p
    lib.approxifer_strerror.argtypes = [ctypes.c_int]
    lib.approxifer_chebyshev_nodes.restype = ctypes.c_int
    lib.approxifer_chebyshev_nodes.argtypes = [ctypes.c_int, ctypes.c_int, c_dp, c_dp]
    lib.approxifer_encode.restype = ctypes.c_int
    lib.approxifer_encode.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int64, c_dp, c_dp, vp]
    lib.approxifer_decode.restype = ctypes.c_int
    lib.approxifer_decode.argtypes = [vp, vp, vp, vp, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                      ctypes.c_int64, c_dp, c_dp, ctypes.c_int, vp]
    lib.approxifer_decode_top1.restype = ctypes.c_int
    lib.approxifer_decode_top1.argtypes = [vp, vp, vp, vp, vp, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                           ctypes.c_int64, c_dp, c_dp, ctypes.c_int, vp]
    lib.approxifer_decode_byzantine.restype = ctypes.c_int
    lib.approxifer_decode_byzantine.argtypes = [vp, vp, vp, vp, vp, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                                ctypes.c_int, ctypes.c_int, ctypes.c_int64, c_dp, c_dp, ctypes.c_int,
                                                vp, ctypes.c_size_t, vp]
    lib.approxifer_workspace_bytes.restype = ctypes.c_size_t
    lib.approxifer_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                               ctypes.c_int64]
    lib.approxifer_decode_byzantine_static.restype = ctypes.c_int
    lib.approxifer_decode_byzantine_static.argtypes = [vp, vp, vp, vp, vp, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                                       ctypes.c_int, ctypes.c_int, ctypes.c_int64, c_dp, c_dp,
                                                       ctypes.c_int, vp]
    lib.approxifer_group_count.restype = ctypes.c_int64
    lib.approxifer_group_count.argtypes = [ctypes.c_int64, ctypes.c_int]
    lib.approxifer_pad_last_group.restype = ctypes.c_int
    lib.approxifer_pad_last_group.argtypes = [vp, ctypes.c_int64, ctypes.c_int, ctypes.c_int64, vp]
    lib.approxifer_top1.restype = ctypes.c_int
    lib.approxifer_top1.argtypes = [vp, vp, vp, ctypes.c_int64, ctypes.c_int64, vp]
    lib.approxifer_decode_rational.restype = ctypes.c_int
    lib.approxifer_decode_rational.argtypes = [vp, vp, vp, vp, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                               ctypes.c_int, ctypes.c_int64, c_dp, c_dp, vp]
    lib.approxifer_decode_byzantine_homogeneous.restype = ctypes.c_int
    lib.approxifer_decode_byzantine_homogeneous.argtypes = lib.approxifer_decode_byzantine.argtypes
    lib.approxifer_wait_mask.restype = ctypes.c_int
    lib.approxifer_wait_mask.argtypes = [vp, vp, vp, ctypes.c_int64, ctypes.c_int, ctypes.c_int, vp]
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load().approxifer_strerror(int(code)).decode()


def _check(code: int) -> None:
    if code != 0:
        raise ApproxiferError(code, strerror(code))


def _nodes(a) -> tuple:
    arr = np.ascontiguousarray(a, dtype=np.float64)
    return arr, arr.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _stream_handle(stream) -> int:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _dev(t, dtype, shape=None):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("expected a tensor in device memory")
    if t.dtype != dtype or not t.is_contiguous():
        raise TypeError("expected a contiguous %s tensor, got %s" % (dtype, t.dtype))
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("expected shape %s, got %s" % (tuple(shape), tuple(t.shape)))
    return ctypes.c_void_p(t.data_ptr())


def approxifer_chebyshev_nodes(K: int, N: int):
    """(alpha[K], beta[N]) float64 numpy arrays from the library's own node generator."""
    alpha = np.empty(max(K, 0), dtype=np.float64)
    beta = np.empty(max(N, 0), dtype=np.float64)
    _check(load().approxifer_chebyshev_nodes(int(K), int(N),
                                             alpha.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                                             beta.ctypes.data_as(ctypes.POINTER(ctypes.c_double))))
    return alpha, beta


def approxifer_group_count(Q: int, K: int) -> int:
    """Number of groups of K consecutive queries that a stream of Q queries forms."""
    return int(load().approxifer_group_count(int(Q), int(K)))


def approxifer_pad_last_group(buffer, Q, K, stream=None):
    """buffer: [rows, D] float32 device tensor with rows >= ceil(Q / K) * K whose first Q rows hold the stream;
    rows Q .. ceil(Q / K) * K - 1 become copies of row Q - 1.  Returns the buffer's first G * K rows as [G, K, D]."""
    import torch
    rows, D = buffer.shape
    G = approxifer_group_count(Q, K)
    if G < 0 or rows < G * K:
        raise ValueError("the buffer must hold ceil(Q / K) * K rows")
    _check(load().approxifer_pad_last_group(_dev(buffer, torch.float32), int(Q), int(K), int(D),
                                            ctypes.c_void_p(_stream_handle(stream))))
    return buffer[: G * K].view(G, K, D)


def approxifer_encode(queries, alpha, beta, coded=None, stream=None):
    """queries [G, K, D] float32 device tensor -> coded [G, N, D]; K = len(alpha), N = len(beta)."""
    import torch
    a, ap = _nodes(alpha)
    b, bp = _nodes(beta)
    G, K, D = queries.shape
    N = b.size
    if K != a.size:
        raise ValueError("queries.shape[1] must equal len(alpha)")
    if coded is None:
        coded = torch.empty((G, N, D), dtype=torch.float32, device=queries.device)
    _check(load().approxifer_encode(_dev(queries, torch.float32), _dev(coded, torch.float32, (G, N, D)),
                                    G, K, N, D, ap, bp, ctypes.c_void_p(_stream_handle(stream))))
    return coded


def approxifer_decode(preds, mask, alpha, beta, S, sign_mode=SIGN_WORKER_INDEX, out=None, status=None, stream=None):
    """preds [G, N, C] float32, mask [G, N] uint8 -> (out [G, K, C] float32, status [G] int32)."""
    import torch
    a, ap = _nodes(alpha)
    b, bp = _nodes(beta)
    G, N, C = preds.shape
    K = a.size
    if N != b.size:
        raise ValueError("preds.shape[1] must equal len(beta)")
    if out is None:
        out = torch.zeros((G, K, C), dtype=torch.float32, device=preds.device)
    if status is None:
        status = torch.full((G,), -1, dtype=torch.int32, device=preds.device)
    _check(load().approxifer_decode(_dev(preds, torch.float32), _dev(mask, torch.uint8, (G, N)),
                                    _dev(out, torch.float32, (G, K, C)), _dev(status, torch.int32, (G,)),
                                    G, K, N, int(S), C, ap, bp, int(sign_mode),
                                    ctypes.c_void_p(_stream_handle(stream))))
    return out, status


def approxifer_decode_top1(preds, mask, alpha, beta, S, sign_mode=SIGN_WORKER_INDEX, top1=None, score=None, status=None,
                           stream=None, want_score=True):
    """Fused decode + argmax over classes: (top1 [G, K] int32, score [G, K] float32 or None, status [G] int32)."""
    import torch
    a, ap = _nodes(alpha)
    b, bp = _nodes(beta)
    G, N, C = preds.shape
    K = a.size
    if N != b.size:
        raise ValueError("preds.shape[1] must equal len(beta)")
    if top1 is None:
        top1 = torch.full((G, K), -1, dtype=torch.int32, device=preds.device)
    if score is None and want_score:
        score = torch.zeros((G, K), dtype=torch.float32, device=preds.device)
    if status is None:
        status = torch.full((G,), -1, dtype=torch.int32, device=preds.device)
    _check(load().approxifer_decode_top1(_dev(preds, torch.float32), _dev(mask, torch.uint8, (G, N)),
                                         _dev(top1, torch.int32, (G, K)),
                                         _dev(score, torch.float32, (G, K)) if score is not None else None,
                                         _dev(status, torch.int32, (G,)), G, K, N, int(S), C, ap, bp, int(sign_mode),
                                         ctypes.c_void_p(_stream_handle(stream))))
    return top1, score, status


def approxifer_workspace_bytes(G: int, K: int, N: int, S: int, A: int, C: int) -> int:
    """Bytes of device scratch memory with which the Byzantine decoders run fastest at this shape (0: none needed)."""
    return int(load().approxifer_workspace_bytes(int(G), int(K), int(N), int(S), int(A), int(C)))


NO_WORKSPACE = object()


def _decode_byzantine(entry, preds, mask, alpha, beta, S, A, sign_mode, out, adv, status, stream, workspace):
    import torch
    a, ap = _nodes(alpha)
    b, bp = _nodes(beta)
    G, N, C = preds.shape
    K = a.size
    if N != b.size:
        raise ValueError("preds.shape[1] must equal len(beta)")
    if out is None:
        out = torch.zeros((G, K, C), dtype=torch.float32, device=preds.device)
    if adv is None:
        adv = torch.full((G, max(int(A), 0)), -1, dtype=torch.int32, device=preds.device)
    if status is None:
        status = torch.full((G,), -1, dtype=torch.int32, device=preds.device)
    if workspace is None:
        # the caller left the workspace to the binding: a buffer of the size the library asks for
        need = approxifer_workspace_bytes(G, K, N, S, A, C)
        workspace = torch.empty((need,), dtype=torch.uint8, device=preds.device) if need else NO_WORKSPACE
    if workspace is NO_WORKSPACE:
        ws_ptr, ws_bytes = None, 0
    else:
        if not isinstance(workspace, torch.Tensor) or not workspace.is_cuda or not workspace.is_contiguous():
            raise TypeError("workspace must be a contiguous tensor in device memory")
        ws_ptr, ws_bytes = ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size()
    _check(getattr(load(), entry)(_dev(preds, torch.float32), _dev(mask, torch.uint8, (G, N)),
                                  _dev(out, torch.float32, (G, K, C)), _dev(adv, torch.int32, (G, int(A))),
                                  _dev(status, torch.int32, (G,)), G, K, N, int(S), int(A), C, ap, bp,
                                  int(sign_mode), ws_ptr, ctypes.c_size_t(ws_bytes),
                                  ctypes.c_void_p(_stream_handle(stream))))
    return out, adv, status


def approxifer_decode_byzantine(preds, mask, alpha, beta, S, A, sign_mode=SIGN_WORKER_INDEX, out=None, adv=None,
                                status=None, stream=None, workspace=None):
    """As approxifer_decode, after locating and dropping A adversaries per group.
    Returns (out [G, K, C] float32, adv [G, A] int32 ascending, status [G] int32).
    workspace: a device tensor (any dtype) passed as the C ABI's d_workspace / workspace_bytes; None allocates
    approxifer_workspace_bytes() bytes for this call; NO_WORKSPACE passes NULL / 0."""
    return _decode_byzantine("approxifer_decode_byzantine", preds, mask, alpha, beta, S, A, sign_mode, out, adv,
                             status, stream, workspace)


def approxifer_decode_byzantine_homogeneous(preds, mask, alpha, beta, S, A, sign_mode=SIGN_WORKER_INDEX, out=None,
                                            adv=None, status=None, stream=None, workspace=None):
    """As approxifer_decode_byzantine, with Algorithm 1's homogeneous fit as the per-class locator."""
    return _decode_byzantine("approxifer_decode_byzantine_homogeneous", preds, mask, alpha, beta, S, A, sign_mode,
                             out, adv, status, stream, workspace)


def approxifer_decode_rational(preds, mask, alpha, beta, S, A, out=None, status=None, stream=None):
    """Algorithm 3: out[g, j, c] = P(alpha_j) / Q(alpha_j) with (P, Q) Algorithm 2's fit per class.
    Returns (out [G, K, C] float32, status [G] int32)."""
    import torch
    a, ap = _nodes(alpha)
    b, bp = _nodes(beta)
    G, N, C = preds.shape
    K = a.size
    if N != b.size:
        raise ValueError("preds.shape[1] must equal len(beta)")
    if out is None:
        out = torch.zeros((G, K, C), dtype=torch.float32, device=preds.device)
    if status is None:
        status = torch.full((G,), -1, dtype=torch.int32, device=preds.device)
    _check(load().approxifer_decode_rational(_dev(preds, torch.float32), _dev(mask, torch.uint8, (G, N)),
                                             _dev(out, torch.float32, (G, K, C)), _dev(status, torch.int32, (G,)),
                                             G, K, N, int(S), int(A), C, ap, bp, ctypes.c_void_p(_stream_handle(stream))))
    return out, status


def approxifer_top1(values, top1=None, score=None, stream=None, want_score=True):
    """values [..., C] float32 device tensor -> (top1 [...] int32, score [...] float32 or None)."""
    import torch
    C = values.shape[-1]
    lead = tuple(values.shape[:-1])
    rows = int(np.prod(lead)) if lead else 1
    if top1 is None:
        top1 = torch.full(lead, -1, dtype=torch.int32, device=values.device)
    if score is None and want_score:
        score = torch.zeros(lead, dtype=torch.float32, device=values.device)
    _check(load().approxifer_top1(_dev(values, torch.float32), _dev(top1, torch.int32, lead),
                                  _dev(score, torch.float32, lead) if score is not None else None, rows, C,
                                  ctypes.c_void_p(_stream_handle(stream))))
    return top1, score


STATIC_WORKSPACE_BYTES = 65536


def approxifer_decode_byzantine_static(preds, mask, alpha, beta, S, A, out, adv, status, sign_mode=SIGN_WORKER_INDEX,
                                       stream=None):
    """approxifer_decode_byzantine on the library's built-in workspace.  Allocates nothing: every output is the
    caller's.  Raises ApproxiferError(-8) for shapes whose workspace exceeds STATIC_WORKSPACE_BYTES."""
    import torch
    a, ap = _nodes(alpha)
    b, bp = _nodes(beta)
    G, N, C = preds.shape
    K = a.size
    if N != b.size:
        raise ValueError("preds.shape[1] must equal len(beta)")
    _check(load().approxifer_decode_byzantine_static(_dev(preds, torch.float32), _dev(mask, torch.uint8, (G, N)),
                                                     _dev(out, torch.float32, (G, K, C)),
                                                     _dev(adv, torch.int32, (G, int(A))),
                                                     _dev(status, torch.int32, (G,)), G, K, N, int(S), int(A), C, ap, bp,
                                                     int(sign_mode), ctypes.c_void_p(_stream_handle(stream))))
    return out, adv, status


def approxifer_wait_mask(arrival, wait_for, mask=None, count=None, stream=None):
    """arrival [G, N] float32 device tensor -> (mask [G, N] uint8, count [G] int32): the wait_for fastest workers."""
    import torch
    G, N = arrival.shape
    if mask is None:
        mask = torch.zeros((G, N), dtype=torch.uint8, device=arrival.device)
    if count is None:
        count = torch.full((G,), -1, dtype=torch.int32, device=arrival.device)
    _check(load().approxifer_wait_mask(_dev(arrival, torch.float32), _dev(mask, torch.uint8, (G, N)),
                                       _dev(count, torch.int32, (G,)), G, N, int(wait_for),
                                       ctypes.c_void_p(_stream_handle(stream))))
    return mask, count

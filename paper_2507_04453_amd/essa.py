"""ctypes binding of include/essa.h.  Function names mirror the C entry points; arguments are torch
tensors living on the GPU (device memory) or numpy arrays (host memory), exactly as essa.h says."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

__all__ = [
    "EssaError", "lib", "LIB_PATH", "Context", "Graph", "Projection", "CmaState",
    "F32", "BF16", "QUANT_INT8_PERCH", "QUANT_INT4_G128", "COMPUTE_W8A8", "LORA_ONLY", "BASE_ONLY", "COMPUTE_BF16",
    "essa_create", "essa_proj_create", "essa_cma_create", "essa_sample_candidates", "essa_philox_words",
    "essa_theta_to_sigma", "essa_svdlora_forward", "essa_svdlora_forward_group", "essa_w8a8_accumulators",
    "essa_reward_accumulate", "essa_reward_accumulate_group", "essa_cmaes_update", "essa_rank_rewards", "essa_version", "EXPORTED_SYMBOLS",
    "ForwardGroup", "REWARD_BLOCK", "essa_svdlora_forward_reward_group", "essa_reward_finish",
    "essa_cma_create_opt", "OPT_CMA", "OPT_ACTIVE_CMA", "OPT_SEP_CMA", "OPT_ES", "OPT_ARS",
    "VALIDATE", "essa_svdlora_forward_noalloc", "NOALLOC_SCRATCH_BYTES",
]

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libessa.so")

F32, BF16 = 0, 1
QUANT_INT8_PERCH, QUANT_INT4_G128 = 0, 1
COMPUTE_W8A8, LORA_ONLY, BASE_ONLY, COMPUTE_BF16, VALIDATE = 1, 2, 4, 8, 16
NOALLOC_SCRATCH_BYTES = 8 << 20
MAX_GROUP = 8
REWARD_BLOCK = 128
OPT_CMA, OPT_ACTIVE_CMA, OPT_SEP_CMA, OPT_ES, OPT_ARS = 0, 1, 2, 3, 4

EXPORTED_SYMBOLS = [
    "essa_create", "essa_destroy", "essa_last_error", "essa_version", "essa_synchronize",
    "essa_profile_enable", "essa_profile_read",
    "essa_proj_create", "essa_proj_destroy", "essa_proj_spectrum",
    "essa_cma_create", "essa_cma_destroy", "essa_cma_set_basis", "essa_cma_export", "essa_cma_import",
    "essa_sample_candidates", "essa_philox_words", "essa_theta_to_sigma",
    "essa_svdlora_forward", "essa_svdlora_forward_group", "essa_w8a8_accumulators",
    "essa_reward_accumulate", "essa_reward_accumulate_group", "essa_cmaes_update", "essa_rank_rewards",
    "essa_svdlora_forward_reward_group", "essa_reward_finish",
    "essa_graph_begin", "essa_graph_end", "essa_graph_launch", "essa_graph_destroy", "essa_cma_refresh_basis",
    "essa_cma_create_opt", "essa_cma_kind", "essa_svdlora_forward_noalloc",
]


class EssaError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("essa status %d: %s" % (code, msg))
        self.code = code


class _ProjDesc(C.Structure):
    _fields_ = [("d_in", C.c_int32), ("d_out", C.c_int32), ("r", C.c_int32), ("quant", C.c_int32),
                ("Wq", C.c_void_p), ("scales", C.c_void_p), ("zeros", C.c_void_p),
                ("lora_A", C.c_void_p), ("lora_B", C.c_void_p)]


class _OptDesc(C.Structure):
    _fields_ = [("kind", C.c_int), ("ars_alpha", C.c_float), ("ars_top", C.c_int)]


class _FwdItem(C.Structure):
    _fields_ = [("proj", C.c_void_p), ("X", C.c_void_p), ("row2cand", C.c_void_p), ("sigmaA", C.c_void_p),
                ("sigmaB", C.c_void_p), ("Y", C.c_void_p), ("sigma_stride", C.c_int64), ("R", C.c_int32),
                ("K", C.c_int32)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError("libessa.so is not built (%s); run `python -m paper_2507_04453_amd.build`. "
                          "There is no fallback path." % LIB_PATH)
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, u32, f32 = C.c_void_p, C.c_int, C.c_int64, C.c_uint32, C.c_float
    sig = {
        "essa_create": (i32, [C.POINTER(vp), i32, vp]),
        "essa_destroy": (None, [vp]),
        "essa_last_error": (C.c_char_p, []),
        "essa_version": (C.c_char_p, []),
        "essa_synchronize": (i32, [vp]),
        "essa_profile_enable": (i32, [vp, i32]),
        "essa_profile_read": (i32, [vp, C.POINTER(C.c_double), C.POINTER(i32)]),
        "essa_proj_create": (i32, [vp, C.POINTER(_ProjDesc), C.POINTER(vp)]),
        "essa_cma_refresh_basis": (i32, [vp, vp, i32, f32, C.POINTER(i32), C.POINTER(f32)]),
        "essa_graph_begin": (i32, [vp]),
        "essa_graph_end": (i32, [vp, C.POINTER(vp)]),
        "essa_graph_launch": (i32, [vp]),
        "essa_graph_destroy": (None, [vp]),
        "essa_proj_destroy": (None, [vp]),
        "essa_proj_spectrum": (i32, [vp, vp, vp]),
        "essa_cma_create": (i32, [vp, i32, f32, vp, C.POINTER(vp)]),
        "essa_cma_create_opt": (i32, [vp, i32, f32, vp, C.POINTER(_OptDesc), C.POINTER(vp)]),
        "essa_cma_kind": (i32, [vp]),
        "essa_cma_destroy": (None, [vp]),
        "essa_cma_set_basis": (i32, [vp, vp, vp]),
        "essa_cma_export": (i32, [vp, vp, C.POINTER(C.c_size_t)]),
        "essa_cma_import": (i32, [vp, vp, C.c_size_t]),
        "essa_sample_candidates": (i32, [vp, vp, vp, i32, vp, vp]),
        "essa_philox_words": (i32, [vp, vp, i32, i32, vp]),
        "essa_theta_to_sigma": (i32, [vp, i32, i32, i32, vp, vp, vp, i32, vp, vp]),
        "essa_svdlora_forward": (i32, [vp, vp, vp, i32, i32, vp, vp, vp, i64, i32, vp, i32, u32]),
        "essa_svdlora_forward_noalloc": (i32, [vp, vp, vp, i32, i32, vp, vp, vp, i64, i32, vp, i32, u32]),
        "essa_svdlora_forward_group": (i32, [vp, C.POINTER(_FwdItem), i32, i32, i32, u32]),
        "essa_svdlora_forward_reward_group": (i32, [vp, C.POINTER(_FwdItem), i32, i32, i32, u32, C.POINTER(vp), vp, i64, i64]),
        "essa_reward_finish": (i32, [vp, vp, i64, i32, vp, i32, vp]),
        "essa_w8a8_accumulators": (i32, [vp, vp, vp, i32, i32, vp, vp, vp]),
        "essa_reward_accumulate": (i32, [vp, vp, i32, i32, i32, vp, vp, i32, vp]),
        "essa_reward_accumulate_group": (i32, [vp, i32, C.POINTER(vp), C.POINTER(i32), C.POINTER(vp), i32, i32, vp, i32, vp]),
        "essa_cmaes_update": (i32, [vp, vp, vp, vp, i32, vp]),
        "essa_rank_rewards": (i32, [vp, vp, i32, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    return L


lib = _load()


def _check(code):
    if code != 0:
        raise EssaError(code, lib.essa_last_error().decode("utf-8", "replace"))


def essa_version() -> str:
    return lib.essa_version().decode()


def _dev(t, dtype=None, name="tensor"):
    """Device pointer of a contiguous CUDA/HIP tensor (None -> NULL)."""
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a torch tensor on the GPU" % name)
    if dtype is not None and t.dtype != dtype:
        raise TypeError("%s must have dtype %s, got %s" % (name, dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    return C.c_void_p(t.data_ptr())


def _host(a, dtype, name="array"):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, C.c_void_p(a.ctypes.data)


def _xdtype(t):
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("activations must be float32 or bfloat16, got %s" % t.dtype)


class Graph:
    """essa_graph: a recorded launch sequence; launch() queues one replay on the stream it was recorded on."""

    def __init__(self, handle):
        self._h = handle

    def launch(self):
        _check(lib.essa_graph_launch(self._h))

    def close(self):
        if self._h:
            lib.essa_graph_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Context:
    """essa_ctx: one GPU, one stream (the current torch stream at creation unless given)."""

    def __init__(self, device: int = 0, stream: "torch.cuda.Stream | None" = None):
        self._h = C.c_void_p()
        self.device = device
        torch.cuda.set_device(device)
        self.stream = stream
        sp = C.c_void_p(stream.cuda_stream) if stream is not None else None
        _check(lib.essa_create(C.byref(self._h), device, sp))

    def synchronize(self):
        _check(lib.essa_synchronize(self._h))

    def profile_enable(self, on: bool):
        _check(lib.essa_profile_enable(self._h, 1 if on else 0))

    def profile_read(self):
        """(summed GEMM-kernel milliseconds, launches) since the last read."""
        ms, cnt = C.c_double(0), C.c_int(0)
        _check(lib.essa_profile_read(self._h, C.byref(ms), C.byref(cnt)))
        return ms.value, cnt.value

    def graph_begin(self):
        """Start recording the calls on this context (and anything else put on its stream) instead of running them."""
        _check(lib.essa_graph_begin(self._h))

    def graph_end(self) -> "Graph":
        h = C.c_void_p()
        _check(lib.essa_graph_end(self._h, C.byref(h)))
        return Graph(h)

    def close(self):
        if self._h:
            lib.essa_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def essa_create(device: int = 0, stream=None) -> Context:
    return Context(device, stream)


class Projection:
    """essa_proj: built from HOST arrays (quantised weight, scales, zeros, raw LoRA factors)."""

    def __init__(self, ctx: Context, Wq, scales, zeros, lora_A, lora_B, quant: int):
        self.ctx = ctx
        lora_A = np.ascontiguousarray(lora_A, np.float32)
        lora_B = np.ascontiguousarray(lora_B, np.float32)
        r, d_in = lora_A.shape
        d_out = lora_B.shape[0]
        if lora_B.shape[1] != r:
            raise ValueError("lora_B must be [d_out, r]")
        keep = [lora_A, lora_B]
        if quant == QUANT_INT8_PERCH:
            Wq = np.ascontiguousarray(Wq, np.int8)
            scales = np.ascontiguousarray(scales, np.float32)
            if Wq.shape != (d_out, d_in) or scales.shape != (d_out,):
                raise ValueError("int8: Wq [d_out,d_in], scales [d_out]")
            zp = None
        elif quant == QUANT_INT4_G128:
            Wq = np.ascontiguousarray(Wq, np.uint8)
            scales = np.ascontiguousarray(scales, np.float16)
            zeros = np.ascontiguousarray(zeros, np.float16)
            if Wq.shape != (d_out, d_in // 2) or scales.shape != (d_out, d_in // 128) or zeros.shape != scales.shape:
                raise ValueError("int4: Wq [d_out,d_in/2], scales/zeros [d_out,d_in/128]")
            zp = C.c_void_p(zeros.ctypes.data)
            keep.append(zeros)
        else:
            raise ValueError("unknown quant")
        keep += [Wq, scales]
        d = _ProjDesc(d_in, d_out, r, quant, C.c_void_p(Wq.ctypes.data), C.c_void_p(scales.ctypes.data), zp,
                      C.c_void_p(lora_A.ctypes.data), C.c_void_p(lora_B.ctypes.data))
        self._h = C.c_void_p()
        _check(lib.essa_proj_create(ctx._h, C.byref(d), C.byref(self._h)))
        self.d_in, self.d_out, self.r, self.quant = d_in, d_out, r, quant

    def spectrum(self):
        """(S_A[r], S_B[r]): the factors' own singular values, descending (host float32)."""
        sA, sB = np.empty(self.r, np.float32), np.empty(self.r, np.float32)
        _check(lib.essa_proj_spectrum(self._h, C.c_void_p(sA.ctypes.data), C.c_void_p(sB.ctypes.data)))
        return sA, sB

    def close(self):
        if self._h:
            lib.essa_proj_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def essa_proj_create(ctx, Wq, scales, zeros, lora_A, lora_B, quant) -> Projection:
    return Projection(ctx, Wq, scales, zeros, lora_A, lora_B, quant)


_BLOB_HEADER = np.dtype([("magic", "<u4"), ("version", "<u4"), ("n", "<i4"), ("t", "<i4"), ("sigma", "<f4"), ("reserved", "<u4")])


class CmaState:
    """essa_cma: the search distribution on the device."""

    def __init__(self, ctx: Context, n: int, sigma0: float, m0=None, kind: int = OPT_CMA, ars_alpha: float = 0.0, ars_top: int = 0):
        self.ctx, self.n, self.kind = ctx, n, kind
        self._h = C.c_void_p()
        if m0 is not None:
            m0, mp = _host(m0, np.float32)
            if m0.shape != (n,):
                raise ValueError("m0 must be [n]")
        else:
            mp = None
        if kind == OPT_CMA:
            _check(lib.essa_cma_create(ctx._h, n, C.c_float(sigma0), mp, C.byref(self._h)))
        else:
            desc = _OptDesc(kind, ars_alpha, ars_top)
            _check(lib.essa_cma_create_opt(ctx._h, n, C.c_float(sigma0), mp, C.byref(desc), C.byref(self._h)))

    def set_basis(self, B: torch.Tensor, D: torch.Tensor):
        if tuple(B.shape) != (self.n, self.n) or tuple(D.shape) != (self.n,):
            raise ValueError("B [n,n], D [n]")
        _check(lib.essa_cma_set_basis(self._h, _dev(B, torch.float32, "B"), _dev(D, torch.float32, "D")))

    def refresh_basis(self, ctx: "Context", max_sweeps: int = 30, tol: float = 1e-7):
        """C -> (B, D) on the device; returns (sweeps, last off-diagonal measure)."""
        sw, off = C.c_int(0), C.c_float(0)
        _check(lib.essa_cma_refresh_basis(ctx._h, self._h, max_sweeps, tol, C.byref(sw), C.byref(off)))
        return sw.value, off.value

    def export_blob(self) -> bytes:
        size = C.c_size_t(0)
        _check(lib.essa_cma_export(self._h, None, C.byref(size)))
        buf = (C.c_char * size.value)()
        _check(lib.essa_cma_export(self._h, C.cast(buf, C.c_void_p), C.byref(size)))
        return bytes(buf)

    def import_blob(self, blob: bytes):
        buf = (C.c_char * len(blob)).from_buffer_copy(blob)
        _check(lib.essa_cma_import(self._h, C.cast(buf, C.c_void_p), len(blob)))

    def export(self) -> dict:
        """The blob parsed into numpy arrays (t, sigma, m, p_sigma, p_c, D, then C, B or, for kinds without a matrix, c_diag)."""
        blob = self.export_blob()
        h = np.frombuffer(blob, _BLOB_HEADER, 1)[0]
        n = int(h["n"])
        body = np.frombuffer(blob, np.float32, offset=_BLOB_HEADER.itemsize)
        out = dict(n=n, t=int(h["t"]), sigma=float(h["sigma"]), kind=int(h["reserved"]))
        off = 0
        for name in ("m", "p_sigma", "p_c", "D"):
            out[name] = body[off:off + n].copy()
            off += n
        if out["kind"] in (OPT_CMA, OPT_ACTIVE_CMA):
            out["C"] = body[off:off + n * n].reshape(n, n).copy()
            off += n * n
            out["B"] = body[off:off + n * n].reshape(n, n).copy()
        else:
            out["c_diag"] = body[off:off + n].copy()
        return out

    @staticmethod
    def pack_blob(n, t, sigma, m, p_sigma, p_c, D, Cm, B=None, kind: int = OPT_CMA) -> bytes:
        """Cm: the covariance matrix [n, n] followed by B, or (kinds without a matrix, B = None) its diagonal [n]."""
        h = np.zeros(1, _BLOB_HEADER)
        h["magic"], h["version"], h["n"], h["t"], h["sigma"], h["reserved"] = 0x41535345, 1, n, t, sigma, kind
        arrays = (m, p_sigma, p_c, D, Cm) if B is None else (m, p_sigma, p_c, D, Cm, B)
        parts = [h.tobytes()] + [np.ascontiguousarray(a, np.float32).tobytes() for a in arrays]
        return b"".join(parts)

    def close(self):
        if self._h:
            lib.essa_cma_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def essa_cma_create(ctx, n, sigma0, m0=None) -> CmaState:
    return CmaState(ctx, n, sigma0, m0)


def essa_cma_create_opt(ctx, n, sigma0, m0=None, kind: int = OPT_CMA, ars_alpha: float = 0.0, ars_top: int = 0) -> CmaState:
    return CmaState(ctx, n, sigma0, m0, kind, ars_alpha, ars_top)


def essa_sample_candidates(ctx: Context, cma: CmaState, seeds: torch.Tensor, theta_out: torch.Tensor, z_out: torch.Tensor | None = None):
    K = seeds.numel() * (2 if cma.kind == OPT_ARS else 1)
    if tuple(theta_out.shape) != (K, cma.n) or (z_out is not None and tuple(z_out.shape) != (K, cma.n)):
        raise ValueError("theta_out / z_out must be [K, n]")
    _check(lib.essa_sample_candidates(ctx._h, cma._h, _dev(seeds, torch.int32, "seeds"), K, _dev(theta_out, torch.float32, "theta_out"),
                                      _dev(z_out, torch.float32, "z_out")))


def essa_philox_words(ctx: Context, seeds: torch.Tensor, n_blocks: int, words_out: torch.Tensor):
    K = seeds.numel()
    if words_out.numel() != K * n_blocks * 4:
        raise ValueError("words_out must hold K*n_blocks*4 words")
    _check(lib.essa_philox_words(ctx._h, _dev(seeds, torch.int32, "seeds"), K, n_blocks, _dev(words_out, torch.int32, "words_out")))


def essa_theta_to_sigma(ctx: Context, n_top: int, sft_A: torch.Tensor, sft_B: torch.Tensor, theta: torch.Tensor,
                        sigmaA: torch.Tensor, sigmaB: torch.Tensor):
    P, r = sft_A.shape
    K = theta.shape[0]
    if n_top >= 1 and theta.shape[1] != P * 2 * n_top:
        raise ValueError("theta must be [K, P*2*n_top]")
    if tuple(sigmaA.shape) != (K, P, r) or tuple(sigmaB.shape) != (K, P, r) or tuple(sft_B.shape) != (P, r):
        raise ValueError("sigma outputs must be [K,P,r], spectra [P,r]")
    _check(lib.essa_theta_to_sigma(ctx._h, P, r, n_top, _dev(sft_A, torch.float32), _dev(sft_B, torch.float32),
                                   _dev(theta, torch.float32), K, _dev(sigmaA, torch.float32), _dev(sigmaB, torch.float32)))


def _ydtype(t):
    return _xdtype(t)


def _sigma_args(proj, sigmaA, sigmaB, K):
    if sigmaA.dtype != torch.float32 or sigmaB.dtype != torch.float32 or not sigmaA.is_cuda or not sigmaB.is_cuda:
        raise TypeError("sigmaA/sigmaB must be float32 GPU tensors")
    if sigmaA.shape != sigmaB.shape or sigmaA.dim() != 2 or sigmaA.shape[0] != K or sigmaA.shape[1] != proj.r:
        raise ValueError("sigmaA/sigmaB must be [K, r] views")
    if sigmaA.stride(1) != 1 or sigmaB.stride(1) != 1 or sigmaA.stride(0) != sigmaB.stride(0):
        raise ValueError("sigmaA/sigmaB must have unit inner stride and equal candidate stride")
    return C.c_void_p(sigmaA.data_ptr()), C.c_void_p(sigmaB.data_ptr()), int(sigmaA.stride(0))


def essa_svdlora_forward(ctx: Context, proj: Projection, X: torch.Tensor, row2cand: torch.Tensor, sigmaA: torch.Tensor,
                         sigmaB: torch.Tensor, Y: torch.Tensor, flags: int = 0):
    """sigmaA/sigmaB: [K, r] float32 views (any candidate stride, unit inner stride)."""
    R = X.shape[0]
    K = sigmaA.shape[0]
    if X.dim() != 2 or X.shape[1] != proj.d_in or tuple(Y.shape) != (R, proj.d_out) or row2cand.numel() != R:
        raise ValueError("X [R,d_in], Y [R,d_out], row2cand [R]")
    pa, pb, stride = _sigma_args(proj, sigmaA, sigmaB, K)
    _check(lib.essa_svdlora_forward(ctx._h, proj._h, _dev(X, None, "X"), _xdtype(X), R, _dev(row2cand, torch.int32, "row2cand"),
                                    pa, pb, stride, K, _dev(Y, None, "Y"), _ydtype(Y), flags))


def essa_svdlora_forward_noalloc(ctx: Context, proj: Projection, X: torch.Tensor, row2cand: torch.Tensor, sigmaA: torch.Tensor,
                                 sigmaB: torch.Tensor, Y: torch.Tensor, flags: int = 0):
    """essa_svdlora_forward on the library's fixed scratch array: no device allocation of any kind."""
    R = X.shape[0]
    K = sigmaA.shape[0]
    if X.dim() != 2 or X.shape[1] != proj.d_in or tuple(Y.shape) != (R, proj.d_out) or row2cand.numel() != R:
        raise ValueError("X [R,d_in], Y [R,d_out], row2cand [R]")
    pa, pb, stride = _sigma_args(proj, sigmaA, sigmaB, K)
    _check(lib.essa_svdlora_forward_noalloc(ctx._h, proj._h, _dev(X, None, "X"), _xdtype(X), R, _dev(row2cand, torch.int32, "row2cand"),
                                            pa, pb, stride, K, _dev(Y, None, "Y"), _ydtype(Y), flags))


class ForwardGroup:
    """The marshalled argument block of a grouped forward: build it once for a fixed set of tensors and pass it to
    essa_svdlora_forward_group / essa_svdlora_forward_reward_group in place of the list, so that a call in a tight
    loop costs one foreign call.  Holds references to the tensors it points at.

    items: list of (proj, X, row2cand, sigmaA, sigmaB, Y); all X share a dtype and all Y share a dtype.
    vs: optional list of reward vectors [d_out_g] (float32), one per item."""

    def __init__(self, items, vs=None):
        if not 1 <= len(items) <= MAX_GROUP:
            raise ValueError("1..%d items" % MAX_GROUP)
        self.n = len(items)
        self.arr = (_FwdItem * self.n)()
        self.xd = self.yd = None
        for i, (proj, X, row2cand, sigmaA, sigmaB, Y) in enumerate(items):
            R, K = X.shape[0], sigmaA.shape[0]
            if X.dim() != 2 or X.shape[1] != proj.d_in or tuple(Y.shape) != (R, proj.d_out) or row2cand.numel() != R:
                raise ValueError("item %d: X [R,d_in], Y [R,d_out], row2cand [R]" % i)
            pa, pb, stride = _sigma_args(proj, sigmaA, sigmaB, K)
            if self.xd is None:
                self.xd, self.yd = _xdtype(X), _ydtype(Y)
            elif self.xd != _xdtype(X) or self.yd != _ydtype(Y):
                raise TypeError("all items of a group share the activation and output dtypes")
            self.arr[i] = _FwdItem(proj._h, _dev(X, None, "X"), _dev(row2cand, torch.int32, "row2cand"), pa, pb, _dev(Y, None, "Y"), stride, R, K)
        self.R = items[0][1].shape[0]
        self.blocks = sum((it[0].d_out + REWARD_BLOCK - 1) // REWARD_BLOCK for it in items)
        self.vp = None
        if vs is not None:
            if len(vs) != self.n:
                raise ValueError("one reward vector per item")
            self.vp = (C.c_void_p * self.n)()
            for g, (v, it) in enumerate(zip(vs, items)):
                if v.numel() != it[0].d_out or it[1].shape[0] != self.R:
                    raise ValueError("v_g has d_out_g entries; all items share the rows")
                self.vp[g] = _dev(v, torch.float32, "v").value
        self._keep = (list(items), list(vs) if vs is not None else None)


def essa_svdlora_forward_group(ctx: Context, items, flags: int = 0):
    """items: a ForwardGroup, or a list of (proj, X, row2cand, sigmaA, sigmaB, Y)."""
    g = items if isinstance(items, ForwardGroup) else ForwardGroup(items)
    _check(lib.essa_svdlora_forward_group(ctx._h, g.arr, g.n, g.xd, g.yd, flags))


def essa_svdlora_forward_reward_group(ctx: Context, items, vs, rowpart: torch.Tensor, block0: int = 0, flags: int = 0):
    """Forward of the group plus rowpart[block0 + b, i] = <Y[i, 128 b ..], v[128 b ..]> for the blocks of every item in turn.
    items: a ForwardGroup built with vs (then pass vs=None), or a list plus the list of reward vectors.
    rowpart: float32 [blocks, R].  Returns the first block after the ones written."""
    g = items if isinstance(items, ForwardGroup) else ForwardGroup(items, vs)
    if g.vp is None:
        raise ValueError("the group carries no reward vectors")
    if rowpart.dtype != torch.float32 or rowpart.dim() != 2 or rowpart.shape[1] != g.R:
        raise ValueError("rowpart must be float32 [blocks, R]")
    _check(lib.essa_svdlora_forward_reward_group(ctx._h, g.arr, g.n, g.xd, g.yd, flags, g.vp, _dev(rowpart, torch.float32, "rowpart"),
                                                 rowpart.shape[0], block0))
    return block0 + g.blocks


def essa_reward_finish(ctx: Context, rowpart: torch.Tensor, n_blocks: int, row2cand: torch.Tensor, F: torch.Tensor):
    """F[k] += mean over candidate k's rows of the sum of the first n_blocks rows of rowpart."""
    R = row2cand.numel()
    if rowpart.dtype != torch.float32 or rowpart.dim() != 2 or rowpart.shape[1] != R or not 1 <= n_blocks <= rowpart.shape[0]:
        raise ValueError("rowpart must be float32 [>= n_blocks, R]")
    _check(lib.essa_reward_finish(ctx._h, _dev(rowpart, torch.float32, "rowpart"), n_blocks, R, _dev(row2cand, torch.int32, "row2cand"),
                                  F.numel(), _dev(F, torch.float32, "F")))


def essa_w8a8_accumulators(ctx: Context, proj: Projection, X: torch.Tensor, xq_out: torch.Tensor, xscale_out: torch.Tensor,
                           acc_out: torch.Tensor):
    R = X.shape[0]
    if tuple(xq_out.shape) != (R, proj.d_in) or xscale_out.numel() != R or tuple(acc_out.shape) != (R, proj.d_out):
        raise ValueError("xq_out [R,d_in], xscale_out [R], acc_out [R,d_out]")
    _check(lib.essa_w8a8_accumulators(ctx._h, proj._h, _dev(X, None, "X"), _xdtype(X), R, _dev(xq_out, torch.int8), _dev(xscale_out, torch.float32),
                                      _dev(acc_out, torch.int32)))


def essa_reward_accumulate(ctx: Context, Y: torch.Tensor, v: torch.Tensor, row2cand: torch.Tensor, F: torch.Tensor):
    R, d_out = Y.shape
    _check(lib.essa_reward_accumulate(ctx._h, _dev(Y, None, "Y"), _ydtype(Y), R, d_out, _dev(v, torch.float32, "v"),
                                      _dev(row2cand, torch.int32, "row2cand"), F.numel(), _dev(F, torch.float32, "F")))


def essa_reward_accumulate_group(ctx: Context, Ys, vs, row2cand: torch.Tensor, F: torch.Tensor):
    """Ys, vs: lists of outputs [R, d_out_g] (one dtype) and reward vectors [d_out_g]."""
    n = len(Ys)
    if not 1 <= n <= MAX_GROUP or len(vs) != n:
        raise ValueError("1..%d outputs with one vector each" % MAX_GROUP)
    R = Ys[0].shape[0]
    yd = _ydtype(Ys[0])
    yp, vp_, dd = (C.c_void_p * n)(), (C.c_void_p * n)(), (C.c_int * n)()
    for g, (Y, v) in enumerate(zip(Ys, vs)):
        if Y.shape[0] != R or _ydtype(Y) != yd or v.numel() != Y.shape[1]:
            raise ValueError("outputs share rows and dtype; v_g has d_out_g entries")
        yp[g], vp_[g], dd[g] = _dev(Y, None, "Y").value, _dev(v, torch.float32, "v").value, Y.shape[1]
    _check(lib.essa_reward_accumulate_group(ctx._h, n, yp, dd, vp_, yd, R, _dev(row2cand, torch.int32, "row2cand"), F.numel(),
                                            _dev(F, torch.float32, "F")))


def essa_cmaes_update(ctx: Context, cma: CmaState, seeds: torch.Tensor, rewards: torch.Tensor, order_out: torch.Tensor | None = None):
    K = rewards.numel()
    per_seed = 2 if cma.kind == OPT_ARS else 1
    if seeds.numel() * per_seed != K or (order_out is not None and order_out.numel() != seeds.numel()):
        raise ValueError("seeds and order_out must hold one entry per candidate (ARS: per pair of candidates)")
    _check(lib.essa_cmaes_update(ctx._h, cma._h, _dev(seeds, torch.int32, "seeds"), _dev(rewards, torch.float32, "rewards"), K,
                                 _dev(order_out, torch.int32, "order_out")))


def essa_rank_rewards(ctx: Context, rewards: torch.Tensor, order: torch.Tensor):
    K = rewards.numel()
    if order.numel() != K:
        raise ValueError("order must hold K entries")
    _check(lib.essa_rank_rewards(ctx._h, _dev(rewards, torch.float32, "rewards"), K, _dev(order, torch.int32, "order")))

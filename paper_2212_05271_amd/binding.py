"""Thin ctypes binding over libgss.so: argument marshalling only.

Every function here has the name and the arguments of the C entry point in include/gss.h; tensors are
torch CUDA (HIP) tensors used purely as device memory, and the current torch stream is passed down as
the HIP stream.  No step of the method is computed in Python.  If the shared library is missing the
import of this module fails loudly; there is no fallback path.
"""

from __future__ import annotations

import ctypes as C
import os

import numpy as np
# torch first: it ships its own HIP runtime, and the tensors this binding takes live in that runtime.
# Loading libgss.so before torch would bring in the system's copy of the runtime as well, and a process with
# two HIP runtimes does not work (the library's calls and torch's would talk to different ones).
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgss.so")

GSS_OK, GSS_EINVAL, GSS_EUNSUPPORTED, GSS_ENOMEM, GSS_EHIP, GSS_ETOOBIG = 0, -1, -2, -3, -4, -5
GSS_STATIC_SCRATCH_BYTES = 64 << 20
GSS_OPT_EM_WHOLE_MIN_PROBLEMS = 1
GSS_REF_PER_SEGMENT, GSS_REF_PER_FREQUENCY = 0, 1
GSS_MAX_D, GSS_MAX_K = 32, 8
# bits of the status word (Context.get_status)
(GSS_STATUS_NONPD_B, GSS_STATUS_NONPD_PHI, GSS_STATUS_BAD_TARGET, GSS_STATUS_NONPD_WPE, GSS_STATUS_ZERO_FRAME,
 GSS_STATUS_BAD_REF) = 1, 2, 4, 8, 16, 32

EXPORTS = (
    "gss_create", "gss_destroy", "gss_strerror", "gss_version", "gss_get_status", "gss_scratch_bytes",
    "gss_profile_enable", "gss_profile_get", "gss_set_option",
    "gss_stft", "gss_wpe", "gss_cacgmm_em", "gss_cacgmm_em_noalloc", "gss_cacgmm_em_frames", "gss_mvdr",
    "gss_mvdr_frames", "gss_mvdr_ex", "gss_istft", "gss_frames_from_segments", "gss_frame_activity",
)


class GssError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        super().__init__(f"{what}: {strerror(code)} ({code})")


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2212_05271_amd.build` "
            "(there is no fallback implementation)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int, C.c_int64
    lib.gss_create.argtypes = [C.POINTER(vp), i32]
    lib.gss_create.restype = i32
    lib.gss_destroy.argtypes = [vp]
    lib.gss_destroy.restype = None
    lib.gss_strerror.argtypes = [i32]
    lib.gss_strerror.restype = C.c_char_p
    lib.gss_version.argtypes = []
    lib.gss_version.restype = C.c_char_p
    lib.gss_get_status.argtypes = [vp, C.POINTER(C.c_uint32), vp]
    lib.gss_get_status.restype = i32
    lib.gss_scratch_bytes.argtypes = [vp]
    lib.gss_scratch_bytes.restype = i64
    lib.gss_set_option.argtypes = [vp, i32, i64]
    lib.gss_set_option.restype = i32
    lib.gss_profile_enable.argtypes = [vp, i32]
    lib.gss_profile_enable.restype = i32
    lib.gss_profile_get.argtypes = [vp, i32, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    lib.gss_profile_get.restype = i32
    lib.gss_stft.argtypes = [vp, vp, i32, i32, i64, i32, i32, vp, i32, vp]
    lib.gss_stft.restype = i32
    lib.gss_cacgmm_em.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, vp]
    lib.gss_cacgmm_em.restype = i32
    lib.gss_cacgmm_em_noalloc.argtypes = lib.gss_cacgmm_em.argtypes
    lib.gss_cacgmm_em_noalloc.restype = i32
    lib.gss_cacgmm_em_frames.argtypes = [vp, vp, i64, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, vp]
    lib.gss_cacgmm_em_frames.restype = i32
    lib.gss_mvdr_frames.argtypes = [vp, vp, i64, vp, vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp]
    lib.gss_mvdr_frames.restype = i32
    lib.gss_mvdr_ex.argtypes = [vp, vp, i64, vp, vp, vp, i32, i32, i32, i32, i32, vp, i32, vp, vp, vp]
    lib.gss_mvdr_ex.restype = i32
    lib.gss_wpe.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, vp]
    lib.gss_wpe.restype = i32
    lib.gss_mvdr.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp]
    lib.gss_mvdr.restype = i32
    lib.gss_istft.argtypes = [vp, vp, i32, i32, i32, i32, vp, i64, vp]
    lib.gss_istft.restype = i32
    lib.gss_frames_from_segments.argtypes = [vp, vp, i32, i64, i64, i64, i32, vp, vp, vp, vp, vp, vp]
    lib.gss_frames_from_segments.restype = i32
    lib.gss_frame_activity.argtypes = [vp, i32, i64, i64, C.c_int32, i32, vp]
    lib.gss_frame_activity.restype = i32
    return lib


_lib = _load()


def strerror(code):
    return _lib.gss_strerror(int(code)).decode()


def version():
    return _lib.gss_version().decode()


def _check(rc, what):
    if rc != GSS_OK:
        raise GssError(rc, what)


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t, dtype=None, name="tensor"):
    """Device pointer of a contiguous CUDA tensor (None -> NULL)."""
    if t is None:
        return C.c_void_p(0)
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a CUDA tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must have dtype {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


class Context:
    """Owns a gss_ctx (the library's scratch memory and status word) on one device."""

    def __init__(self, device_id=0):
        h = C.c_void_p()
        _check(_lib.gss_create(C.byref(h), int(device_id)), "gss_create")
        self._h = h
        self.device_id = int(device_id)

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            _lib.gss_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    @property
    def handle(self):
        if self._h is None:
            raise RuntimeError("context is closed")
        return self._h

    def get_status(self):
        out = C.c_uint32(0)
        _check(_lib.gss_get_status(self.handle, C.byref(out), _stream()), "gss_get_status")
        return int(out.value)

    def set_option(self, option, value):
        _check(_lib.gss_set_option(self.handle, int(option), int(value)), "gss_set_option")

    def scratch_bytes(self):
        return int(_lib.gss_scratch_bytes(self.handle))

    def profile_enable(self, on=True):
        _check(_lib.gss_profile_enable(self.handle, 1 if on else 0), "gss_profile_enable")

    def profile_get(self, which=0):
        """(total milliseconds, launches) of kernel `which` since the last call."""
        ms, n = C.c_double(0.0), C.c_int64(0)
        _check(_lib.gss_profile_get(self.handle, int(which), C.byref(ms), C.byref(n)), "gss_profile_get")
        return float(ms.value), int(n.value)


def gss_stft(ctx, x, n_fft=1024, hop=256, out=None):
    """x[S,D,N] float32 -> Y[S,F,T,D] complex64."""
    import torch
    S, D, N = x.shape
    T = -(-N // hop) + 3
    F = n_fft // 2 + 1
    if out is None:
        out = torch.empty((S, F, T, D), dtype=torch.complex64, device=x.device)
    _check(_lib.gss_stft(ctx.handle, _ptr(x, torch.float32, "x"), S, D, N, n_fft, hop,
                         _ptr(out, torch.complex64, "Y"), T, _stream()), "gss_stft")
    return out


def gss_cacgmm_em(ctx, Y, activity, T_len=None, iters=20, weight_mode=1, out=None, _entry="gss_cacgmm_em"):
    """Y[S,F,Tmax,D] complex64, activity[S,K,Tmax] uint8, T_len[S] int32|None -> gamma[S,K,F,Tmax] float32."""
    import torch
    S, F, Tmax, D = Y.shape
    K = activity.shape[1]
    if tuple(activity.shape) != (S, K, Tmax):
        raise ValueError("activity must be [S,K,Tmax]")
    if T_len is not None and tuple(T_len.shape) != (S,):
        raise ValueError("T_len must be [S]")
    if out is None:
        out = torch.empty((S, K, F, Tmax), dtype=torch.float32, device=Y.device)
    _check(getattr(_lib, _entry)(ctx.handle, _ptr(Y, torch.complex64, "Y"), _ptr(activity, torch.uint8, "activity"),
                                 _ptr(T_len, torch.int32, "T_len"), S, F, Tmax, D, K, int(iters), int(weight_mode),
                                 _ptr(out, torch.float32, "gamma"), _stream()), _entry)
    return out


def gss_cacgmm_em_noalloc(ctx, Y, activity, T_len=None, iters=20, weight_mode=1, *, out):
    """gss_cacgmm_em with the library's static scratch array as working memory (no device allocation inside the
    call; `out` must be supplied by the caller for the same reason).  Raises GssError(GSS_ETOOBIG) when the problem
    does not fit GSS_STATIC_SCRATCH_BYTES."""
    return gss_cacgmm_em(ctx, Y, activity, T_len, iters, weight_mode, out=out, _entry="gss_cacgmm_em_noalloc")


def gss_cacgmm_em_frames(ctx, Yrec, frame0, activity, T_len, iters=20, weight_mode=1, out=None):
    """Yrec[F,Trec,D] complex64 (the recording's STFT), frame0[S] int64, activity[S,K,Tmax] uint8, T_len[S] int32
    -> gamma[S,K,F,Tmax] float32; segment s is frames frame0[s] .. frame0[s] + T_len[s] - 1 of the recording."""
    import torch
    F, Trec, D = Yrec.shape
    S, K, Tmax = activity.shape
    if tuple(frame0.shape) != (S,) or (T_len is not None and tuple(T_len.shape) != (S,)):
        raise ValueError("frame0 and T_len must be [S]")
    if out is None:
        out = torch.empty((S, K, F, Tmax), dtype=torch.float32, device=Yrec.device)
    _check(_lib.gss_cacgmm_em_frames(ctx.handle, _ptr(Yrec, torch.complex64, "Yrec"), Trec, _ptr(frame0, torch.int64, "frame0"),
                                     _ptr(activity, torch.uint8, "activity"), _ptr(T_len, torch.int32, "T_len"),
                                     S, F, Tmax, D, K, int(iters), int(weight_mode),
                                     _ptr(out, torch.float32, "gamma"), _stream()), "gss_cacgmm_em_frames")
    return out


def gss_mvdr_frames(ctx, Yrec, frame0, gamma, target, ref, T_len, out=None):
    """Yrec[F,Trec,D], frame0[S] int64, gamma[S,K,F,Tmax], target[S], ref[S] (in/out), T_len[S] -> X[S,F,Tmax]."""
    import torch
    F, Trec, D = Yrec.shape
    S, K, F2, Tmax = gamma.shape
    if F2 != F:
        raise ValueError("gamma must be [S,K,F,Tmax]")
    if tuple(frame0.shape) != (S,) or tuple(target.shape) != (S,) or tuple(ref.shape) != (S,):
        raise ValueError("frame0, target and ref must be [S]")
    if out is None:
        out = torch.empty((S, F, Tmax), dtype=torch.complex64, device=Yrec.device)
    _check(_lib.gss_mvdr_frames(ctx.handle, _ptr(Yrec, torch.complex64, "Yrec"), Trec, _ptr(frame0, torch.int64, "frame0"),
                                _ptr(gamma, torch.float32, "gamma"), _ptr(T_len, torch.int32, "T_len"), S, F, Tmax, D, K,
                                _ptr(target, torch.int32, "target"), _ptr(ref, torch.int32, "ref"),
                                _ptr(out, torch.complex64, "X"), _stream()), "gss_mvdr_frames")
    return out


def gss_mvdr_ex(ctx, Y, gamma, target, ref, T_len=None, frame0=None, ref_mode=GSS_REF_PER_SEGMENT, out=None):
    """The general beamformer call.  frame0 None: Y[S,F,Tmax,D] dense batch; frame0[S] int64: Y[F,Trec,D] is a
    recording's STFT.  ref_mode GSS_REF_PER_SEGMENT: ref[S]; GSS_REF_PER_FREQUENCY: ref[S,F] (in/out)."""
    import torch
    S, K, F, Tmax = gamma.shape
    if frame0 is None:
        if tuple(Y.shape[:3]) != (S, F, Tmax):
            raise ValueError("Y must be [S,F,Tmax,D]")
        D, Trec = Y.shape[3], 0
    else:
        if Y.dim() != 3 or Y.shape[0] != F or tuple(frame0.shape) != (S,):
            raise ValueError("Y must be [F,Trec,D] and frame0 [S]")
        Trec, D = Y.shape[1], Y.shape[2]
    want = (S, F) if ref_mode == GSS_REF_PER_FREQUENCY else (S,)
    if tuple(ref.shape) != want or tuple(target.shape) != (S,):
        raise ValueError(f"ref must be {want} and target [S]")
    if out is None:
        out = torch.empty((S, F, Tmax), dtype=torch.complex64, device=Y.device)
    _check(_lib.gss_mvdr_ex(ctx.handle, _ptr(Y, torch.complex64, "Y"), Trec, _ptr(frame0, torch.int64, "frame0"),
                            _ptr(gamma, torch.float32, "gamma"), _ptr(T_len, torch.int32, "T_len"), S, F, Tmax, D, K,
                            _ptr(target, torch.int32, "target"), int(ref_mode), _ptr(ref, torch.int32, "ref"),
                            _ptr(out, torch.complex64, "X"), _stream()), "gss_mvdr_ex")
    return out


def gss_wpe(ctx, Y, T_len=None, taps=10, delay=2, iters=3, out=None):
    """Y[S,F,Tmax,D] complex64 -> dereverberated X[S,F,Tmax,D] complex64 (a new tensor unless `out` is given)."""
    import torch
    S, F, Tmax, D = Y.shape
    if out is None:
        out = torch.empty((S, F, Tmax, D), dtype=torch.complex64, device=Y.device)
    if tuple(out.shape) != (S, F, Tmax, D):
        raise ValueError("out must be [S,F,Tmax,D]")
    _check(_lib.gss_wpe(ctx.handle, _ptr(Y, torch.complex64, "Y"), _ptr(T_len, torch.int32, "T_len"), S, F, Tmax, D,
                        int(taps), int(delay), int(iters), _ptr(out, torch.complex64, "X"), _stream()), "gss_wpe")
    return out


def gss_mvdr(ctx, Y, gamma, target, ref, T_len=None, out=None):
    """Y[S,F,Tmax,D], gamma[S,K,F,Tmax], target[S] int32, ref[S] int32 (in/out) -> X[S,F,Tmax] complex64."""
    import torch
    S, F, Tmax, D = Y.shape
    K = gamma.shape[1]
    if tuple(gamma.shape) != (S, K, F, Tmax):
        raise ValueError("gamma must be [S,K,F,Tmax]")
    if tuple(target.shape) != (S,) or tuple(ref.shape) != (S,):
        raise ValueError("target and ref must be [S]")
    if out is None:
        out = torch.empty((S, F, Tmax), dtype=torch.complex64, device=Y.device)
    _check(_lib.gss_mvdr(ctx.handle, _ptr(Y, torch.complex64, "Y"), _ptr(gamma, torch.float32, "gamma"),
                         _ptr(T_len, torch.int32, "T_len"), S, F, Tmax, D, K,
                         _ptr(target, torch.int32, "target"), _ptr(ref, torch.int32, "ref"),
                         _ptr(out, torch.complex64, "X"), _stream()), "gss_mvdr")
    return out


def gss_istft(ctx, X, N, n_fft=1024, hop=256, out=None):
    """X[S,F,T] complex64 -> x[S,N] float32."""
    import torch
    S, F, T = X.shape
    if out is None:
        out = torch.empty((S, N), dtype=torch.float32, device=X.device)
    _check(_lib.gss_istft(ctx.handle, _ptr(X, torch.complex64, "X"), S, T, n_fft, hop,
                          _ptr(out, torch.float32, "x"), int(N), _stream()), "gss_istft")
    return out


def _np_ptr(a):
    return C.c_void_p(a.ctypes.data) if a is not None else C.c_void_p(0)


def gss_frames_from_segments(seg_start, seg_end, n_samples, ctx_left, ctx_right, hop=256):
    """Host integer helper; returns a dict of numpy arrays (ext_start, ext_end, frame0, n_frames, cut_start, cut_end)."""
    s = np.ascontiguousarray(seg_start, dtype=np.int64)
    e = np.ascontiguousarray(seg_end, dtype=np.int64)
    n = int(s.shape[0])
    out = {k: np.zeros(n, dtype=np.int64) for k in ("ext_start", "ext_end", "frame0", "cut_start", "cut_end")}
    out["n_frames"] = np.zeros(n, dtype=np.int32)
    _check(_lib.gss_frames_from_segments(_np_ptr(s), _np_ptr(e), n, int(n_samples), int(ctx_left), int(ctx_right),
                                         int(hop), _np_ptr(out["ext_start"]), _np_ptr(out["ext_end"]),
                                         _np_ptr(out["frame0"]), _np_ptr(out["n_frames"]),
                                         _np_ptr(out["cut_start"]), _np_ptr(out["cut_end"])),
           "gss_frames_from_segments")
    return out


def gss_frame_activity(act_samples, frame0, n_frames, hop=256):
    """Host integer helper: act_samples[K,N] uint8 -> [K,n_frames] uint8."""
    a = np.ascontiguousarray(act_samples, dtype=np.uint8)
    K, N = a.shape
    out = np.zeros((K, int(n_frames)), dtype=np.uint8)
    _check(_lib.gss_frame_activity(_np_ptr(a), K, N, int(frame0), int(n_frames), int(hop), _np_ptr(out)),
           "gss_frame_activity")
    return out

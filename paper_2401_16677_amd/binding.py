"""Thin ctypes binding of libt3.so (the C ABI of include/t3.h).

Argument marshalling only: every step of the path runs in the library's kernels.
PyTorch tensors are used as device memory (data_ptr) and for the current stream.
There is no fallback: if the library is missing, loading fails.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libt3.so")

T3_OK = 0
T3_ERR_NULL, T3_ERR_BAD_SHAPE, T3_ERR_BAD_TILE, T3_ERR_ALIGN, T3_ERR_UNSUPPORTED, T3_ERR_HIP = \
    1, 2, 3, 4, 5, 6
T3_B_NK, T3_B_KN = 0, 1
T3_A_MK, T3_A_KM = 0, 1
T3_FLAG_STEP0_STORE_ONLY = 1
T3_FLAG_FWD_DIRECT = 2
T3_FLAG_TWO_WRITERS = 4
T3_FLAG_FWD_BF16 = 8
T3_STATIC_MAX_TP = 64
T3_TIMELINE_ITEMS = 16

EXPORTS = ["t3_chunk_order", "t3_default_tile", "t3_tiles_per_chunk", "t3_tile_of",
           "t3_track_words", "t3_track_reset", "t3_gemm_rs_fused", "t3_gemm", "t3_rs_reduce",
           "t3_upstream_update", "t3_release_chunks", "t3_gemm_rs_fused_static", "t3_ag_step",
           "t3_timeline", "t3_status_string", "t3_last_hip_error"]


class T3Problem(ctypes.Structure):
    _fields_ = [("M", ctypes.c_int32), ("N", ctypes.c_int32), ("K", ctypes.c_int32),
                ("tp", ctypes.c_int32), ("rank", ctypes.c_int32),
                ("tile_m", ctypes.c_int32), ("tile_n", ctypes.c_int32),
                ("b_layout", ctypes.c_int32),
                ("lda", ctypes.c_int64), ("ldb", ctypes.c_int64),
                ("ldr", ctypes.c_int64), ("ldc", ctypes.c_int64),
                ("tile_limit", ctypes.c_int64), ("flags", ctypes.c_uint32),
                ("tile_begin", ctypes.c_int64), ("split_k", ctypes.c_int32),
                ("upstream_agents", ctypes.c_int32), ("a_layout", ctypes.c_int32),
                ("reserved", ctypes.c_int32)]


class T3Error(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} (t3_status {status})")


_lib = None


def lib():
    """Load libt3.so (built in-tree by paper_2401_16677_amd.build).  Raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is not built: run `python -m paper_2401_16677_amd.build`")
        # The library must bind to the HIP runtime that owns the caller's device memory and
        # streams.  PyTorch ships its own copy, so it is loaded first and libt3.so's
        # dependency on libamdhip64 resolves to that one.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        pp = ctypes.POINTER(T3Problem)
        L.t3_chunk_order.argtypes = [i32, i32, vp, vp]
        L.t3_default_tile.argtypes = [pp, vp, vp]
        L.t3_tiles_per_chunk.argtypes = [pp, vp]
        L.t3_tile_of.argtypes = [pp, i64, vp, vp, vp, vp]
        L.t3_track_words.argtypes = [i32]
        L.t3_track_words.restype = i64
        L.t3_track_reset.argtypes = [i32, vp, vp]
        L.t3_gemm_rs_fused.argtypes = [pp, vp, vp, vp, vp, vp, vp]
        L.t3_gemm_rs_fused_static.argtypes = [pp, vp, vp, vp, vp, vp, vp]
        L.t3_ag_step.argtypes = [pp, i32, vp, i64, vp, vp]
        L.t3_timeline.argtypes = [vp, i64]
        L.t3_gemm.argtypes = [pp, vp, vp, vp, vp]
        L.t3_rs_reduce.argtypes = [pp, vp, vp, vp, vp, vp]
        L.t3_upstream_update.argtypes = [pp, vp, vp, vp, vp]
        L.t3_release_chunks.argtypes = [pp, vp, vp, vp, vp]
        L.t3_status_string.argtypes = [ctypes.c_int]
        L.t3_status_string.restype = ctypes.c_char_p
        L.t3_last_hip_error.restype = i32
        for f in ("t3_chunk_order", "t3_default_tile", "t3_tiles_per_chunk", "t3_tile_of",
                  "t3_track_reset", "t3_gemm_rs_fused", "t3_gemm", "t3_rs_reduce",
                  "t3_upstream_update", "t3_release_chunks", "t3_gemm_rs_fused_static",
                  "t3_ag_step", "t3_timeline"):
            getattr(L, f).restype = ctypes.c_int
        _lib = L
    return _lib


def status_string(status):
    return lib().t3_status_string(int(status)).decode()


def _check(status, what):
    if status != T3_OK:
        raise T3Error(status, what)


def problem(M, N, K, tp, rank, tile_m=0, tile_n=0, b_layout=T3_B_NK, lda=None, ldb=None,
            ldr=None, ldc=None, tile_limit=-1, flags=0, tile_begin=0, split_k=0,
            upstream_agents=0, a_layout=T3_A_MK):
    return T3Problem(M, N, K, tp, rank, tile_m, tile_n, b_layout,
                     (K if a_layout == T3_A_MK else M) if lda is None else lda,
                     (K if b_layout == T3_B_NK else N) if ldb is None else ldb,
                     N if ldr is None else ldr, N if ldc is None else ldc, tile_limit, flags,
                     tile_begin, split_k, upstream_agents, a_layout, 0)


def _dptr(t):
    """Device (or NULL) pointer of a torch tensor / raw int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


# ------------------------------------------------------------------ host-only entry points

def t3_chunk_order(tp, rank):
    order = (ctypes.c_int32 * max(tp, 1))()
    own = ctypes.c_int32(-1)
    _check(lib().t3_chunk_order(tp, rank, ctypes.cast(order, ctypes.c_void_p),
                                ctypes.cast(ctypes.pointer(own), ctypes.c_void_p)),
           "t3_chunk_order")
    return list(order)[:tp], own.value


def t3_default_tile(p):
    tm, tn = ctypes.c_int32(), ctypes.c_int32()
    _check(lib().t3_default_tile(ctypes.byref(p), ctypes.cast(ctypes.pointer(tm), ctypes.c_void_p),
                                 ctypes.cast(ctypes.pointer(tn), ctypes.c_void_p)),
           "t3_default_tile")
    return tm.value, tn.value


def t3_tiles_per_chunk(p):
    v = ctypes.c_int64()
    _check(lib().t3_tiles_per_chunk(ctypes.byref(p),
                                    ctypes.cast(ctypes.pointer(v), ctypes.c_void_p)),
           "t3_tiles_per_chunk")
    return v.value


def t3_tile_of(p, t):
    out = [ctypes.c_int32() for _ in range(4)]
    _check(lib().t3_tile_of(ctypes.byref(p), t,
                            *[ctypes.cast(ctypes.pointer(o), ctypes.c_void_p) for o in out]),
           "t3_tile_of")
    return tuple(o.value for o in out)


def t3_track_words(tp):
    return int(lib().t3_track_words(tp))


# ------------------------------------------------------------------ device entry points

def t3_track_reset(tp, track, stream=None):
    _check(lib().t3_track_reset(tp, _dptr(track), _stream(stream)), "t3_track_reset")


def t3_gemm_rs_fused(p, A, B, R, fwd, track, stream=None):
    _check(lib().t3_gemm_rs_fused(ctypes.byref(p), _dptr(A), _dptr(B), _dptr(R), _dptr(fwd),
                                  _dptr(track), _stream(stream)), "t3_gemm_rs_fused")


def t3_gemm_rs_fused_static(p, A, B, R, fwd, track_copy=None, stream=None):
    _check(lib().t3_gemm_rs_fused_static(ctypes.byref(p), _dptr(A), _dptr(B), _dptr(R), _dptr(fwd),
                                         _dptr(track_copy), _stream(stream)),
           "t3_gemm_rs_fused_static")


def t3_ag_step(p, step, upstream_R, R, ld_up=None, stream=None):
    _check(lib().t3_ag_step(ctypes.byref(p), step, _dptr(upstream_R), p.ldr if ld_up is None else ld_up,
                            _dptr(R), _stream(stream)), "t3_ag_step")


def t3_timeline(stamps):
    """stamps: an int64 device tensor (or None to switch recording off)."""
    if stamps is None:
        _check(lib().t3_timeline(None, 0), "t3_timeline")
    else:
        _check(lib().t3_timeline(_dptr(stamps), stamps.numel()), "t3_timeline")


def t3_gemm(p, A, B, C, stream=None):
    _check(lib().t3_gemm(ctypes.byref(p), _dptr(A), _dptr(B), _dptr(C), _stream(stream)),
           "t3_gemm")


def t3_rs_reduce(p, C, R, fwd, track, stream=None):
    _check(lib().t3_rs_reduce(ctypes.byref(p), _dptr(C), _dptr(R), _dptr(fwd), _dptr(track),
                              _stream(stream)), "t3_rs_reduce")


def t3_upstream_update(p, incoming, R, track, stream=None):
    _check(lib().t3_upstream_update(ctypes.byref(p), _dptr(incoming), _dptr(R), _dptr(track),
                                    _stream(stream)), "t3_upstream_update")


def t3_release_chunks(p, R, fwd, track, stream=None):
    _check(lib().t3_release_chunks(ctypes.byref(p), _dptr(R), _dptr(fwd), _dptr(track),
                                   _stream(stream)), "t3_release_chunks")


def read_track(track, tp):
    """Results of the launch that last completed, from a tracker-state tensor (synchronises):
    counter, ready, queue (numpy uint32), queue_len, done, gen, error."""
    import numpy as np
    w = track.detach().cpu().numpy().view(np.uint32)
    bank_words = 3 * tp + 2
    gen, error = int(w[2 * bank_words]), int(w[2 * bank_words + 1])
    b = w[((gen - 1) & 1) * bank_words:][:bank_words]
    return {"counter": b[0:tp].copy(), "ready": b[tp:2 * tp].copy(),
            "queue": b[2 * tp:3 * tp].copy(), "queue_len": int(b[3 * tp]),
            "done": int(b[3 * tp + 1]), "gen": gen, "error": error}

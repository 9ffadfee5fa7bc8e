"""ctypes front end of the CPU oracle (oracle/t3_oracle.c) plus the composition of
its steps into the whole fused path.

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by the smoke check and by the
CPU-baseline leg of the benchmark; never by the product package.  It imports
nothing from the product package either: inputs arrive as numpy arrays.

What the path computes (T3, arXiv 2401.16677): rank r of a P-way tensor-parallel
group multiplies its K-slice (Sec. 2.4), the M x N partial output is cut into P
column chunks that are produced in the staggered ring order (Sec. 4.1, 4.4),
each element is added to the partial received from upstream (Sec. 2.3), all
chunks but the last produced are handed on to the downstream neighbour once a
tracker has seen every update of the chunk (Sec. 4.2), and the last chunk stays
on the rank fully reduced.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libt3_oracle.so")
_lib = None

B_NK = 0  # B stored N x K, K contiguous
B_KN = 1  # B stored K x N, N contiguous
A_MK = 0  # A stored M x K, K contiguous
A_KM = 1  # A stored K x M, M contiguous (the transposed operand of the backward-pass GEMMs, Sec. 5.2)

_c_i32 = ctypes.c_int32
_c_i64 = ctypes.c_int64
_p = ctypes.c_void_p


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _build
            _build.build()
        L = ctypes.CDLL(_LIB_PATH)
        L.t3o_num_threads.restype = _c_i32
        L.t3o_chunk_order.argtypes = [_c_i32, _c_i32, _p, _p]
        L.t3o_gemm_rows.argtypes = [_c_i32, _c_i32, _c_i32, _p, _c_i64, _p, _c_i64, _c_i32,
                                    _p, _c_i32, _p]
        L.t3o_reduce_rows.argtypes = [_c_i32, _c_i32, _c_i32, _p, _p, _c_i64, _p, _c_i32,
                                      _p, _c_i64]
        L.t3o_tile_of.argtypes = [_c_i32, _c_i32, _c_i32, _c_i32, _c_i32, _c_i32, _c_i64,
                                  _p, _p, _p, _p]
        L.t3o_track.argtypes = [_c_i32, _c_i32, _c_i32, _c_i32, _c_i32, _c_i32, _p, _c_i64,
                                _p, _p, _p, _p]
        L.t3o_track_upd.argtypes = [_c_i32, _c_i32, _c_i32, _c_i32, _c_i32, _c_i32, _p, _p,
                                    _c_i64, _p, _p, _p, _p]
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(_p)


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what}: bad argument (rc={rc})")


def num_threads():
    return int(lib().t3o_num_threads())


def chunk_order(P, r):
    """Ring order of rank r and the chunk it keeps (Sec. 4.1, Sec. 4.4)."""
    order = np.zeros(max(P, 1), dtype=np.int32)
    own = _c_i32(-1)
    _check(lib().t3o_chunk_order(P, r, _ptr(order), ctypes.byref(own)), "chunk_order")
    return order[:P].copy(), int(own.value)


def gemm_rows(A_bits, B_bits, b_layout=B_NK, rows=None, a_layout=A_MK):
    """fp64 sliced GEMM (Sec. 2.4) for all rows or the listed rows.

    A_bits: uint16 (M, K) bf16 bit patterns for A_MK, (K, M) for A_KM (element (m, k) of the
    operand is then A_bits[k, m]: it is put back into (M, K) order first, which changes no
    value); B_bits: uint16 (N, K) for B_NK or (K, N) for B_KN.  Returns float64 (nrows, N).
    """
    if a_layout == A_KM:
        A_bits = np.asarray(A_bits, dtype=np.uint16).T
    elif a_layout != A_MK:
        raise ValueError("unknown a_layout")
    A_bits = np.ascontiguousarray(A_bits, dtype=np.uint16)
    B_bits = np.ascontiguousarray(B_bits, dtype=np.uint16)
    M, K = A_bits.shape
    if b_layout == B_NK:
        N, Kb = B_bits.shape
    else:
        Kb, N = B_bits.shape
    if Kb != K:
        raise ValueError("A and B disagree on K")
    if rows is None:
        rows_arr, nrows = None, M
    else:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int32)
        nrows = rows_arr.shape[0]
    C = np.empty((nrows, N), dtype=np.float64)
    _check(lib().t3o_gemm_rows(M, N, K, _ptr(A_bits), A_bits.shape[1], _ptr(B_bits),
                               B_bits.shape[1], int(b_layout), _ptr(rows_arr), nrows, _ptr(C)),
           "gemm_rows")
    return C


def reduce_rows(C, incoming, P, skip_chunk=-1, rows=None):
    """S = fl32(incoming + C) on all or the listed rows (Sec. 2.3)."""
    C = np.ascontiguousarray(C, dtype=np.float64)
    incoming = np.ascontiguousarray(incoming, dtype=np.float32)
    nrows, N = C.shape
    rows_arr = None if rows is None else np.ascontiguousarray(rows, dtype=np.int32)
    if rows_arr is None and incoming.shape[0] != nrows:
        raise ValueError("incoming and C disagree on rows")
    S = np.empty((nrows, N), dtype=np.float32)
    _check(lib().t3o_reduce_rows(N, P, skip_chunk, _ptr(C), _ptr(incoming), incoming.shape[1],
                                 _ptr(rows_arr), nrows, _ptr(S), N), "reduce_rows")
    return S


def tile_of(M, N, P, r, tile_m, tile_n, t):
    """Issue index t -> (stage s, chunk c, tile row mi, tile column nj inside the chunk)."""
    s, c, mi, nj = _c_i32(), _c_i32(), _c_i32(), _c_i32()
    _check(lib().t3o_tile_of(M, N, P, r, tile_m, tile_n, t, ctypes.byref(s), ctypes.byref(c),
                             ctypes.byref(mi), ctypes.byref(nj)), "tile_of")
    return int(s.value), int(c.value), int(mi.value), int(nj.value)


def tiles_per_chunk(M, N, P, tile_m, tile_n):
    W = N // P
    return -(-M // tile_m) * -(-W // tile_n)


def track(M, N, P, r, tile_m, tile_n, landed, updates=None):
    """Replay tile landings (issue indices, in landing order) through the tracker (Sec. 4.2).
    updates: per chunk, the updates expected per element (threshold = tiles per chunk x that;
    Sec. 4.2.1: 2 for a ring reduce-scatter chunk that also receives the upstream update)."""
    landed = np.ascontiguousarray(landed, dtype=np.int64)
    upd = None if updates is None else np.ascontiguousarray(updates, dtype=np.int32)
    counter = np.zeros(P, dtype=np.uint32)
    ready = np.zeros(P, dtype=np.uint32)
    queue = np.zeros(P, dtype=np.uint32)
    qlen = ctypes.c_uint32(0)
    _check(lib().t3o_track_upd(M, N, P, r, tile_m, tile_n, _ptr(upd), _ptr(landed),
                               landed.shape[0], _ptr(counter), _ptr(ready), _ptr(queue),
                               ctypes.byref(qlen)), "track")
    return {"counter": counter, "ready": ready, "queue": queue, "queue_len": int(qlen.value)}


def executed_mask(M, N, P, r, tile_m, tile_n, tile_limit, tile_begin=0):
    """Boolean (M, N): element lies in one of the tiles [tile_begin, tile_limit) of the issue
    order; also returns the clipped range end and start."""
    W = N // P
    T = P * tiles_per_chunk(M, N, P, tile_m, tile_n)
    L = T if tile_limit < 0 else min(tile_limit, T)
    B0 = min(max(tile_begin, 0), L)
    mask = np.zeros((M, N), dtype=bool)
    for t in range(B0, L):
        _, c, mi, nj = tile_of(M, N, P, r, tile_m, tile_n, t)
        m0, n0 = mi * tile_m, c * W + nj * tile_n
        mask[m0:min(m0 + tile_m, M), n0:min(n0 + tile_n, (c + 1) * W)] = True
    return mask, L, B0


def to_bf16_bits(x):
    """fp32 -> bfloat16 bit patterns (uint16), round to nearest, ties to even: the 16-bit
    format activations travel in under mixed precision (Sec. 5.2).  bfloat16 is the upper half
    of an fp32 word, so rounding adds half an ulp of the kept part (less one when the kept part
    is even) and truncates.  A NaN gives a quiet NaN of the same sign."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    kept_is_odd = (u >> np.uint64(16)) & np.uint64(1)
    rounded = (u + np.uint64(0x7FFF) + kept_is_odd) >> np.uint64(16)
    is_nan = (u & np.uint64(0x7FFFFFFF)) > np.uint64(0x7F800000)
    quiet = ((u >> np.uint64(16)) & np.uint64(0x8000)) | np.uint64(0x7FC0)
    return np.where(is_nan, quiet, rounded).astype(np.uint16)


def from_bf16_bits(b):
    """bfloat16 bit patterns -> the fp32 values they denote (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _new_fwd(P, M, W, fwd_init, fwd_bf16):
    dt = np.uint16 if fwd_bf16 else np.float32
    if fwd_init is None:
        return np.zeros((max(P - 1, 0), M, W), dtype=dt)
    if np.asarray(fwd_init).dtype != dt:
        raise ValueError("fwd_init must be %s" % np.dtype(dt).name)
    return np.array(fwd_init, dtype=dt, copy=True)


def fused_path(A_bits, B_bits, incoming, P, r, tile_m, tile_n, *, b_layout=B_NK, a_layout=A_MK,
               tile_limit=-1, tile_begin=0, step0_store_only=False, fwd_direct=False,
               fwd_init=None, two_writers=False, R_init=None, split_k=1, fwd_bf16=False):
    """The whole path for one rank, by the definition.

    Returns a dict with
      R        (M, N) fp32   local buffer after the call
      fwd      (P-1, M, W)   forward slots, slot s holds chunk order[s]
      owned    (M, W)        the chunk the rank keeps = R[:, own*W:(own+1)*W]
      order, own, counter, ready, queue (in issue order), queue_len, tiles_per_chunk
    Default release mode: every executed tile is added in place into R and a chunk
    is copied to its forward slot once complete.  fwd_direct: sums of forwarded
    chunks go straight to the forward slot and R keeps the incoming data there.
    fwd_bf16: the forward slots hold bfloat16 bit patterns (uint16; fwd_init likewise): what
    is written there is the fp32 sum rounded by to_bf16_bits; R stays fp32.
    Only the tiles [tile_begin, tile_limit) of the issue order are executed (a ring step s is
    the range [s*tpc, (s+1)*tpc), Sec. 4.1); elements outside executed tiles keep their
    initial contents, and a chunk is complete only if all of its tiles were executed.
    """
    incoming = np.ascontiguousarray(incoming, dtype=np.float32)
    M, N = incoming.shape
    if N % P:
        raise ValueError("N must be a multiple of P")
    W = N // P
    order, own = chunk_order(P, r)
    C = gemm_rows(A_bits, B_bits, b_layout, a_layout=a_layout)
    S = reduce_rows(C, incoming, P, skip_chunk=int(order[0]) if step0_store_only else -1)
    mask, L, B0 = executed_mask(M, N, P, r, tile_m, tile_n, tile_limit, tile_begin)
    if two_writers:
        return _two_writers(A_bits, B_bits, incoming, P, r, tile_m, tile_n, S, mask, L, B0,
                            order, own, step0_store_only, fwd_init, R_init, split_k, fwd_bf16)
    trk = track(M, N, P, r, tile_m, tile_n, np.arange(B0, L, dtype=np.int64))

    fwd = _new_fwd(P, M, W, fwd_init, fwd_bf16)
    sent = to_bf16_bits if fwd_bf16 else (lambda x: x)      # what a forward slot receives
    R = incoming.copy()
    for s in range(P):
        c = int(order[s])
        cols = slice(c * W, (c + 1) * W)
        if c == own or not fwd_direct:
            R[:, cols] = np.where(mask[:, cols], S[:, cols], incoming[:, cols])
        if c != own:
            if fwd_direct:
                fwd[s] = np.where(mask[:, cols], sent(S[:, cols]), fwd[s])
            elif trk["ready"][c]:
                fwd[s] = sent(S[:, cols])
    out = dict(trk)
    out.update(R=R, fwd=fwd, owned=R[:, own * W:(own + 1) * W].copy(), order=order, own=own,
               tiles_per_chunk=tiles_per_chunk(M, N, P, tile_m, tile_n), executed=L - B0)
    return out


def _two_writers(A_bits, B_bits, incoming, P, r, tile_m, tile_n, S, mask, L, B0, order, own,
                 step0_store_only, fwd_init, R_init, split_k=1, fwd_bf16=False):
    """Both writers add into R over the tiles [B0, L).  R_init must be zero on executed tiles:
    then 0 + x is exact and the second add rounds once, whichever writer comes first, so the
    result is S = fl32(incoming + C) either way (the sums of reduce_rows)."""
    M, N = incoming.shape
    W = N // P
    R = np.zeros((M, N), np.float32) if R_init is None else np.array(R_init, np.float32, copy=True)
    if np.any(R[mask] != 0):
        raise ValueError("two-writer oracle needs R_init == 0 on the executed tiles")
    R[mask] = S[mask]
    if split_k < 1:
        raise ValueError("split_k must be >= 1")
    # (with split_k > 1 the value is still S: the parts' sum is the same product, formed in fp64
    # here; on hardware the order of the fp32 adds is free, which the tolerance covers)
    upd = np.full(P, split_k + 1, dtype=np.int32)
    landed = list(range(B0, L)) * split_k             # the local GEMM's tile updates
    tpc = tiles_per_chunk(M, N, P, tile_m, tile_n)
    if step0_store_only:
        upd[order[0]] = split_k
        landed += [t for t in range(B0, L) if t >= tpc]   # upstream skips the first chunk
    else:
        landed += list(range(B0, L))
    trk = track(M, N, P, r, tile_m, tile_n, np.array(landed, dtype=np.int64), updates=upd)
    fwd = _new_fwd(P, M, W, fwd_init, fwd_bf16)
    out = dict(trk)
    out.update(R=R, fwd=fwd, owned=R[:, own * W:(own + 1) * W].copy(), order=order, own=own,
               tiles_per_chunk=tpc, executed=L - B0, updates=upd)
    return out


def release_ready(R, fwd, ready, P, r, fwd_bf16=False):
    """The triggered transfers (Sec. 4.2.2): every forwarded chunk whose ready flag is set is
    copied from R into its forward slot (rounded to bfloat16 bit patterns if fwd_bf16).
    Returns the new fwd."""
    order, own = chunk_order(P, r)
    W = R.shape[1] // P
    fwd = _new_fwd(P, R.shape[0], W, fwd, fwd_bf16)
    for s in range(P - 1):
        c = int(order[s])
        if ready[c]:
            chunk = R[:, c * W:(c + 1) * W]
            fwd[s] = to_bf16_bits(chunk) if fwd_bf16 else chunk
    return fwd


def all_gather_chunk(P, r, g):
    """Chunk that rank r receives at step g = 0 .. P-2 of the ring all-gather that follows the
    reduce-scatter (Sec. 2.3: like the reduce-scatter but without reductions, N-1 steps until
    every device has all the reduced chunks; same ring, Sec. 4.1: rank r receives from rank
    r+1).  At step 0 rank r+1 passes on the chunk it owns, ((r+1) - 1) mod P = r; at step g it
    passes on what it received at step g-1, so rank r receives chunk (r + g) mod P."""
    if not (0 <= r < P and 0 <= g < P - 1):
        raise ValueError("all-gather: rank or step out of range")
    return (r + g) % P


def all_gather_step(R_upstream, R, P, r, g):
    """One step of the ring all-gather on rank r: the chunk all_gather_chunk(P, r, g) is copied,
    unchanged, from the upstream neighbour's buffer into the same columns of this rank's.
    Returns the new R (M, N) fp32."""
    R_upstream = np.asarray(R_upstream, dtype=np.float32)
    out = np.array(R, dtype=np.float32, copy=True)
    if R_upstream.shape != out.shape or out.shape[1] % P:
        raise ValueError("all-gather: shapes")
    W = out.shape[1] // P
    c = all_gather_chunk(P, r, g)
    out[:, c * W:(c + 1) * W] = R_upstream[:, c * W:(c + 1) * W]
    return out

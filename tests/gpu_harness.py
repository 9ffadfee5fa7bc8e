"""Helpers of the GPU parity tests: put seeded host inputs on the device, call the C ABI
through the binding, bring results back as numpy arrays."""
import numpy as np
import torch

from paper_2401_16677_amd import binding as t3

SENTINEL = -7.0
SENTINEL_BF16 = 0xABCD          # bit pattern a bfloat16 forward slot is filled with beforehand


def to_dev_bits(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()


def run_gpu(a_bits, b_bits, inc, tp, rank, tile, *, flags=0, tile_limit=-1, unfused=False,
            ldr_pad=0, lda_pad=0, tile_begin=0, b_kn=False, a_km=False, launches_before=0):
    """One call of the fused path (or the unfused GEMM-then-reduce pair).  Returns a dict
    with R, fwd (uint16 bit patterns under T3_FLAG_FWD_BF16), counter, ready, queue, queue_len
    (numpy) and, for unfused, C.  launches_before: the same call is made that many times first,
    on the same tracker state without a reset in between, and the buffers are put back."""
    M, K = a_bits.shape
    N = b_bits.shape[0]
    W = N // tp
    dev = torch.device("cuda:0")
    if lda_pad:
        a_host = np.zeros((M, K + lda_pad), dtype=np.uint16)
        a_host[:, :K] = a_bits
        b_host = np.zeros((N, K + lda_pad), dtype=np.uint16)
        b_host[:, :K] = b_bits
    else:
        a_host, b_host = a_bits, b_bits
    ldb = K + lda_pad
    if b_kn:                       # the same B, stored K x N (N contiguous), rows padded by lda_pad
        ldb = N + lda_pad
        b_host = np.zeros((K, ldb), dtype=np.uint16)
        b_host[:, :N] = np.ascontiguousarray(b_bits.T)
    lda = K + lda_pad
    if a_km:                       # the same A, stored K x M (M contiguous), rows padded by lda_pad
        lda = M + lda_pad
        a_host = np.zeros((K, lda), dtype=np.uint16)
        a_host[:, :M] = np.ascontiguousarray(a_bits.T)
    A, B = to_dev_bits(a_host), to_dev_bits(b_host)
    ldr = N + ldr_pad
    R = torch.full((max(M, 1), ldr), 123.0, dtype=torch.float32, device=dev)
    if M:
        R[:M, :N] = torch.from_numpy(inc).to(dev)
    bf16 = bool(flags & t3.T3_FLAG_FWD_BF16)
    if bf16:      # int16 holding the sentinel's bit pattern
        fwd = torch.full((max(tp - 1, 1), max(M, 1), max(W, 1)), SENTINEL_BF16 - 65536,
                         dtype=torch.int16, device=dev)
    else:
        fwd = torch.full((max(tp - 1, 1), max(M, 1), max(W, 1)), SENTINEL, dtype=torch.float32,
                         device=dev)
    track = torch.full((t3.t3_track_words(tp),), 0x5A5A5A5A, dtype=torch.int32, device=dev)
    p = t3.problem(M, N, K, tp, rank, tile[0], tile[1], lda=lda, ldb=ldb,
                   b_layout=t3.T3_B_KN if b_kn else t3.T3_B_NK,
                   a_layout=t3.T3_A_KM if a_km else t3.T3_A_MK,
                   ldr=ldr, ldc=N, tile_limit=tile_limit, flags=flags, tile_begin=tile_begin)
    t3.t3_track_reset(tp, track)
    out = {}
    R0, fwd0 = (R.clone(), fwd.clone()) if launches_before else (None, None)
    for left in range(launches_before, -1, -1):
        if unfused:
            C = torch.full((max(M, 1), N), 55.0, dtype=torch.float32, device=dev)
            t3.t3_gemm(p, A, B, C)
            t3.t3_rs_reduce(p, C, R, fwd, track)
            torch.cuda.synchronize()
            out["C"] = C.cpu().numpy()[:M]
        else:
            t3.t3_gemm_rs_fused(p, A, B, R, fwd, track)
            torch.cuda.synchronize()
        if left:
            R.copy_(R0)
            fwd.copy_(fwd0)
    Rh = R.cpu().numpy()
    out["R"] = Rh[:M, :N]
    out["R_pad"] = Rh[:M, N:]
    out["fwd"] = fwd.cpu().numpy()[:max(tp - 1, 0), :M, :W]
    if bf16:
        out["fwd"] = out["fwd"].view(np.uint16)
    tr = t3.read_track(track, tp)
    out.update(counter=tr["counter"], ready=tr["ready"], queue=tr["queue"],
               queue_len=tr["queue_len"], error=tr["error"], gen=tr["gen"])
    return out


def rel_err(got, want):
    want = np.asarray(want, dtype=np.float64)
    d = np.linalg.norm(np.asarray(got, dtype=np.float64) - want)
    n = np.linalg.norm(want)
    return d / n if n > 0 else d

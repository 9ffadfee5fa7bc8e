"""Pins of the CPU oracle against things other than itself (CPU only).

The paper (T3, arXiv 2401.16677) prints no numeric worked example, so the pins are:
exact rational brute force, integer-exact cases against integer arithmetic, a library fp64
matmul, the invariants of the method, closure of an emulated P-rank ring onto the unsliced
GEMM (textbook reduce-scatter, Sec. 2.3), the paper's 4-GPU walk-through (Sec. 4.1, 4.4;
tests/golden/ring4_gpu0_map.txt) and closed forms for the tracker (Sec. 4.2).
"""
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2401_16677_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _small(seed, M, N, K, P):
    w = wl.make_shape("s", M, N, K, P, 0, 4, 4)
    return wl.make_inputs(w, seed=seed)


def _frac(bits):
    return [[Fraction(float(v)) for v in row] for row in wl.bf16_bits_to_f32(bits)]


# ---------------------------------------------------------------- GEMM + reduce numerics

def test_gemm_matches_exact_rational_bruteforce(oracle):
    M, N, K, P = 6, 8, 12, 2
    a, b, inc = _small(7, M, N, K, P)
    C = oracle.gemm_rows(a, b)
    S = oracle.reduce_rows(C, inc, P)
    fa, fb = _frac(a), _frac(b)
    for m in range(M):
        for n in range(N):
            exact = sum(fa[m][k] * fb[n][k] for k in range(K))
            assert C[m, n] == float(exact)          # fp64 sum of these few terms is exact
            want = np.float32(float(exact + Fraction(float(inc[m, n]))))
            assert S[m, n] == want


def test_gemm_row_subset_and_kn_layout(oracle):
    M, N, K, P = 9, 8, 16, 2
    a, b, _ = _small(3, M, N, K, P)
    full = oracle.gemm_rows(a, b)
    rows = np.array([8, 0, 5, 5], dtype=np.int32)
    assert np.array_equal(oracle.gemm_rows(a, b, rows=rows), full[rows])
    bt = np.ascontiguousarray(b.T)                    # K x N storage of the same operand
    assert np.array_equal(oracle.gemm_rows(a, bt, b_layout=oracle.B_KN), full)
    # a transposed *operand* is a different product: B must not be read as its transpose
    sq_a, sq_b, _ = _small(4, 8, 8, 8, 2)
    assert not np.array_equal(oracle.gemm_rows(sq_a, sq_b),
                              oracle.gemm_rows(sq_a, np.ascontiguousarray(sq_b.T)))


def test_gemm_a_stored_k_by_m(oracle):
    """A stored K x M (the transposed operand of the backward-pass GEMMs, Sec. 5.2): the same
    product as with the M x K storage of the same operand, checked against an exact integer
    matmul written on the K x M array itself; and not the product of the transposed operand."""
    M, N, K, P = 12, 8, 16, 2
    a, b, inc = _small(5, M, N, K, P)
    at = np.ascontiguousarray(a.T)                    # (K, M) storage
    full = oracle.gemm_rows(a, b)
    assert np.array_equal(oracle.gemm_rows(at, b, a_layout=oracle.A_KM), full)
    ai = wl.bf16_bits_to_f32(at).astype(np.float64)   # exact small values
    bi = wl.bf16_bits_to_f32(b).astype(np.float64)
    brute = np.array([[sum(ai[k, m] * bi[n, k] for k in range(K)) for n in range(N)] for m in range(M)])
    assert np.allclose(oracle.gemm_rows(at, b, a_layout=oracle.A_KM), brute, rtol=0, atol=1e-12)
    rows = np.array([11, 0, 3], dtype=np.int32)
    assert np.array_equal(oracle.gemm_rows(at, b, rows=rows, a_layout=oracle.A_KM), full[rows])
    bt = np.ascontiguousarray(b.T)
    assert np.array_equal(oracle.gemm_rows(at, bt, b_layout=oracle.B_KN, a_layout=oracle.A_KM), full)
    sq_a, sq_b, _ = _small(6, 8, 8, 8, 2)             # square: a wrong reading would go unnoticed by shape
    assert not np.array_equal(oracle.gemm_rows(sq_a, sq_b), oracle.gemm_rows(sq_a, sq_b, a_layout=oracle.A_KM))
    want = oracle.fused_path(a, b, inc, P, 1, 4, 4)
    got = oracle.fused_path(at, b, inc, P, 1, 4, 4, a_layout=oracle.A_KM)
    assert np.array_equal(got["R"], want["R"]) and np.array_equal(got["fwd"], want["fwd"])
    with pytest.raises(ValueError):
        oracle.gemm_rows(a, b, a_layout=7)


def test_gemm_integer_exact_against_int64(oracle):
    M, N, K = 33, 40, 200
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=5)
    ai = wl.bf16_bits_to_f32(a).astype(np.int64)
    bi = wl.bf16_bits_to_f32(b).astype(np.int64)
    C = oracle.gemm_rows(a, b)
    want = ai @ bi.T
    assert np.array_equal(C, want.astype(np.float64))
    S = oracle.reduce_rows(C, inc, 4)
    assert np.array_equal(S, (want + inc.astype(np.int64)).astype(np.float32))


def test_gemm_against_library_matmul(oracle):
    w = wl.make_shape("lib", 64, 96, 512, 4, 1, 32, 8)
    a, b, _ = wl.make_inputs(w, seed=11)
    C = oracle.gemm_rows(a, b)
    ref = wl.bf16_bits_to_f32(a).astype(np.float64) @ wl.bf16_bits_to_f32(b).astype(np.float64).T
    assert np.linalg.norm(C - ref) <= 1e-13 * np.linalg.norm(ref)
    # the drawn scale: Var(C) is about 1 by construction of the inputs
    assert 0.8 < C.std() < 1.2


def test_reduce_rounds_once_from_fp64(oracle):
    # inc + c is a tie in fp32 only if c is first rounded to fp32: one rounding must win
    c = np.array([[1.0 + 2.0 ** -24 + 2.0 ** -40, -1.0]], dtype=np.float64)
    inc = np.array([[0.0, 1.0 + 2.0 ** -23]], dtype=np.float32)
    S = oracle.reduce_rows(c, inc, 1)
    assert S[0, 0] == np.float32(1.0 + 2.0 ** -23)
    assert S[0, 1] == np.float32(2.0 ** -23)


def test_reduce_skip_chunk_is_pure_store(oracle):
    C = np.arange(24, dtype=np.float64).reshape(2, 12)
    inc = np.full((2, 12), 100.0, dtype=np.float32)
    S = oracle.reduce_rows(C, inc, 3, skip_chunk=1)
    want = C + 100.0
    want[:, 4:8] = C[:, 4:8]
    assert np.array_equal(S, want.astype(np.float32))


# ---------------------------------------------------------------- invariants of the method

def test_zero_incoming_is_plain_gemm_repartitioned(oracle):
    w = wl.make_shape("z", 16, 24, 32, 3, 2, 8, 4)
    a, b, inc = wl.make_inputs(w, seed=2)
    out = oracle.fused_path(a, b, np.zeros_like(inc), 3, 2, 8, 4)
    C32 = oracle.gemm_rows(a, b).astype(np.float32)
    W = w.W
    for s in range(2):
        c = out["order"][s]
        assert np.array_equal(out["fwd"][s], C32[:, c * W:(c + 1) * W])
    assert np.array_equal(out["owned"], C32[:, out["own"] * W:(out["own"] + 1) * W])
    assert np.array_equal(out["R"], C32)


def test_slices_sum_to_unsliced_gemm(oracle):
    P, M, N, Kfull = 4, 12, 16, 64
    a, b, _ = wl.make_integer_inputs(M, N, Kfull, seed=9)
    whole = oracle.gemm_rows(a, b)
    ks = Kfull // P
    parts = [oracle.gemm_rows(np.ascontiguousarray(a[:, r * ks:(r + 1) * ks]),
                              np.ascontiguousarray(b[:, r * ks:(r + 1) * ks])) for r in range(P)]
    assert np.array_equal(sum(parts), whole)
    w = wl.make_shape("f", M, N, Kfull, P, 0, 4, 4)
    af, bf, _ = wl.make_inputs(w, seed=10)
    whole = oracle.gemm_rows(af, bf)
    parts = [oracle.gemm_rows(np.ascontiguousarray(af[:, r * ks:(r + 1) * ks]),
                              np.ascontiguousarray(bf[:, r * ks:(r + 1) * ks])) for r in range(P)]
    assert np.abs(sum(parts) - whole).max() <= 1e-12 * np.abs(whole).max()


def test_linearity_in_incoming(oracle):
    M, N, K, P = 8, 12, 40, 3
    a, b, inc1 = wl.make_integer_inputs(M, N, K, seed=21)
    _, _, inc2 = wl.make_integer_inputs(M, N, K, seed=22)
    s1 = oracle.fused_path(a, b, inc1, P, 1, 4, 4)
    s12 = oracle.fused_path(a, b, inc1 + inc2, P, 1, 4, 4)
    assert np.array_equal(s12["R"] - s1["R"], inc2)
    assert np.array_equal(s12["fwd"] - s1["fwd"],
                          np.stack([inc2[:, c * 4:(c + 1) * 4] for c in s1["order"][:P - 1]]))


# ---------------------------------------------------------------- ring order and closure

def _golden_map():
    kv = {}
    with open(os.path.join(GOLDEN, "ring4_gpu0_map.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                k, v = line.split()
                kv[k] = v
    return kv


def test_paper_four_gpu_example(oracle):
    g = _golden_map()
    P = int(g["devices"])
    order0, own0 = oracle.chunk_order(P, 0)
    order1, _ = oracle.chunk_order(P, 1)
    # stage i (1-based) of GPU-0 produces chunk order0[i-1]; its fate on GPU-0:
    fate = {}
    for i in range(1, P + 1):
        c = order0[i - 1]
        fate[i] = "keep" if c == own0 else ("remote" if i == 1 else "dma")
    for i in range(1, P + 1):
        assert fate[i] == g[f"gpu0_stage{i}"]
    assert sum(v == "dma" for v in fate.values()) == int(g["steady_state_steps"]) == P - 2
    assert int(g["ring_steps"]) == P - 1
    # stagger: chunks are the stages of the un-staggered GPU-0; GPU-1 starts one later
    assert order0[0] + 1 == int(g["step1_gpu0_stage"])
    assert order1[0] + 1 == int(g["step1_gpu1_stage"])
    # what GPU-0 forwards in slot s is what GPU-3 (its downstream) produces at step s+1,
    # and what it receives for step s>=1 comes from GPU-1 (its upstream)
    down, up = int(g["gpu0_sends_to"]), int(g["gpu0_receives_from"])
    order_down, _ = oracle.chunk_order(P, down)
    order_up, _ = oracle.chunk_order(P, up)
    for s in range(P - 1):
        assert order0[s] == order_down[s + 1]
        assert order_up[s] == order0[s + 1]


@pytest.mark.parametrize("P", [1, 2, 3, 4, 8])
def test_owned_chunks_partition_the_output(oracle, P):
    owns = [oracle.chunk_order(P, r)[1] for r in range(P)]
    assert sorted(owns) == list(range(P))
    for r in range(P):
        order, own = oracle.chunk_order(P, r)
        assert sorted(order) == list(range(P)) and order[0] == r and own == (r - 1) % P


@pytest.mark.parametrize("P", [2, 4, 5])
def test_emulated_ring_closes_on_unsliced_gemm(oracle, P):
    """Textbook reduce-scatter: chain the ranks through their forward slots; every rank must
    end up owning the unsliced GEMM's columns of its chunk (exact: integer inputs)."""
    M, W, ks = 8, 6, 16
    N, Kfull = P * W, P * ks
    a, b, _ = wl.make_integer_inputs(M, N, Kfull, seed=31 + P)
    whole = (wl.bf16_bits_to_f32(a).astype(np.int64) @ wl.bf16_bits_to_f32(b).astype(np.int64).T)
    A_r = [np.ascontiguousarray(a[:, r * ks:(r + 1) * ks]) for r in range(P)]
    B_r = [np.ascontiguousarray(b[:, r * ks:(r + 1) * ks]) for r in range(P)]
    inc = [np.zeros((M, N), dtype=np.float32) for _ in range(P)]
    out = [None] * P
    for step in range(P):
        out = [oracle.fused_path(A_r[r], B_r[r], inc[r], P, r, 4, 3) for r in range(P)]
        for r in range(P):           # hand slot `step` of the upstream rank to rank r
            if step < P - 1:
                up = (r + 1) % P
                c = int(out[r]["order"][step + 1])
                assert c == out[up]["order"][step]
                inc[r][:, c * W:(c + 1) * W] = out[up]["fwd"][step]
    for r in range(P):
        own = out[r]["own"]
        assert np.array_equal(out[r]["owned"], whole[:, own * W:(own + 1) * W].astype(np.float32))


@pytest.mark.parametrize("P", [2, 4, 5])
def test_all_gather_after_the_ring_gives_every_rank_the_unsliced_gemm(oracle, P):
    """Sec. 2.3: reduce-scatter, then an all-gather of N-1 steps without reductions, is an
    all-reduce: every rank ends up with the whole sum.  The sums are those of the emulated ring
    above; the all-gather schedule is pinned by (a) the chunk a rank receives first being the one
    its upstream neighbour owns, (b) each later one being what that neighbour received a step
    earlier, (c) a rank receiving every chunk but its own exactly once, and (d) the result."""
    M, W, ks = 8, 6, 16
    N, Kfull = P * W, P * ks
    a, b, _ = wl.make_integer_inputs(M, N, Kfull, seed=77 + P)
    whole = (wl.bf16_bits_to_f32(a).astype(np.int64) @ wl.bf16_bits_to_f32(b).astype(np.int64).T
             ).astype(np.float32)
    for r in range(P):
        own = oracle.chunk_order(P, r)[1]
        up_own = oracle.chunk_order(P, (r + 1) % P)[1]
        got = [oracle.all_gather_chunk(P, r, g) for g in range(P - 1)]
        assert got[0] == up_own                                                  # (a)
        assert all(got[g] == oracle.all_gather_chunk(P, (r + 1) % P, g - 1) for g in range(1, P - 1))  # (b)
        assert sorted(got + [own]) == list(range(P))                             # (c)
    with pytest.raises(ValueError):
        oracle.all_gather_chunk(P, 0, P - 1)
    # rank r's buffer after the reduce-scatter: its own chunk reduced, garbage elsewhere
    R = []
    for r in range(P):
        own = oracle.chunk_order(P, r)[1]
        buf = np.full((M, N), -1000.0 - r, dtype=np.float32)
        buf[:, own * W:(own + 1) * W] = whole[:, own * W:(own + 1) * W]
        R.append(buf)
    for g in range(P - 1):
        R = [oracle.all_gather_step(R[(r + 1) % P], R[r], P, r, g) for r in range(P)]   # all ranks at once
    for r in range(P):
        assert np.array_equal(R[r], whole)                                       # (d)


@pytest.mark.parametrize("P", [3, 4])
def test_ring_steps_as_tile_ranges_compose_to_the_whole_path(oracle, P):
    """One ring step is the range [s*tpc, (s+1)*tpc) of the issue order (Sec. 4.1).  Running the
    steps one by one, each on what the previous left, must give what one full run gives; and
    the step-by-step ring of P ranks (first chunk stored, not added) closes on the unsliced GEMM."""
    M, W, ks, tm, tn = 8, 6, 16, 4, 3
    N, Kfull = P * W, P * ks
    a, b, inc0 = wl.make_integer_inputs(M, N, Kfull, seed=77 + P)
    tpc = oracle.tiles_per_chunk(M, N, P, tm, tn)
    # (1) composition on one rank, in-place release mode
    r = 1
    A1, B1 = np.ascontiguousarray(a[:, :ks]), np.ascontiguousarray(b[:, :ks])
    full = oracle.fused_path(A1, B1, inc0, P, r, tm, tn)
    R, fwd = inc0.copy(), np.zeros((P - 1, M, W), np.float32)
    ready = np.zeros(P, np.uint32)
    for s in range(P):
        out = oracle.fused_path(A1, B1, R, P, r, tm, tn, tile_begin=s * tpc,
                                tile_limit=(s + 1) * tpc, fwd_init=fwd)
        assert out["executed"] == tpc and out["ready"].sum() == 1
        assert out["queue_len"] == (1 if s < P - 1 else 0)
        R, fwd, ready = out["R"], out["fwd"], ready + out["ready"]
    assert np.array_equal(R, full["R"]) and np.array_equal(fwd, full["fwd"])
    assert np.all(ready == 1)
    # (2) the ring, step by step over all ranks
    whole = (wl.bf16_bits_to_f32(a).astype(np.int64) @ wl.bf16_bits_to_f32(b).astype(np.int64).T)
    A_r = [np.ascontiguousarray(a[:, q * ks:(q + 1) * ks]) for q in range(P)]
    B_r = [np.ascontiguousarray(b[:, q * ks:(q + 1) * ks]) for q in range(P)]
    Rr = [np.full((M, N), 99.0, np.float32) for _ in range(P)]      # garbage: step 0 must not read it
    Fr = [np.zeros((P - 1, M, W), np.float32) for _ in range(P)]
    for s in range(P):
        outs = [oracle.fused_path(A_r[q], B_r[q], Rr[q], P, q, tm, tn, tile_begin=s * tpc,
                                  tile_limit=(s + 1) * tpc, step0_store_only=True,
                                  fwd_direct=True, fwd_init=Fr[q]) for q in range(P)]
        for q in range(P):
            Rr[q], Fr[q] = outs[q]["R"], outs[q]["fwd"]
        if s < P - 1:
            for q in range(P):           # rank q's slot s is what rank q-1 receives for its step s+1
                c = int(outs[q]["order"][s])
                Rr[(q - 1) % P][:, c * W:(c + 1) * W] = Fr[q][s]
    for q in range(P):
        own = (q - 1) % P
        assert np.array_equal(Rr[q][:, own * W:(own + 1) * W],
                              whole[:, own * W:(own + 1) * W].astype(np.float32))


def test_two_writers_threshold_and_order_invariance(oracle):
    """Sec. 4.2.1: a ring reduce-scatter chunk expects 2 updates per element (local GEMM +
    upstream DMA), so its threshold is 2 x tiles-per-chunk (the paper's figure, from the golden
    map); the trigger fires on the LAST of them, whichever writer it is and however the two
    interleave; with the first chunk stored only, that chunk expects 1."""
    M, N, K, P, r, tm, tn = 10, 12, 16, 3, 1, 4, 2
    upe = int(_golden_map()["updates_per_element_ring_rs"])
    assert upe == 2
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=91)
    tpc = oracle.tiles_per_chunk(M, N, P, tm, tn)
    T = P * tpc
    one = oracle.fused_path(a, b, inc, P, r, tm, tn)
    two = oracle.fused_path(a, b, inc, P, r, tm, tn, two_writers=True)
    assert np.array_equal(two["R"], one["R"])            # same sums, whichever writer is first
    assert np.all(two["counter"] == upe * tpc) and np.all(two["ready"] == 1)
    assert two["queue_len"] == P - 1 and np.all(two["fwd"] == 0)
    # only one writer's tiles: nothing is ready
    half = oracle.track(M, N, P, r, tm, tn, np.arange(T), updates=[upe] * P)
    assert np.all(half["counter"] == tpc) and not half["ready"].any() and half["queue_len"] == 0
    # random interleavings of the two writers: same final state, and the trigger position is
    # exactly where the chunk's last update lands
    rng = np.random.default_rng(5)
    for _ in range(20):
        landed = rng.permutation(np.concatenate([np.arange(T), np.arange(T)]))
        full = oracle.track(M, N, P, r, tm, tn, landed, updates=[upe] * P)
        assert np.array_equal(full["counter"], two["counter"]) and np.all(full["ready"] == 1)
        assert set(full["queue"][:P - 1]) == set(two["queue"][:P - 1])
        c0 = int(full["queue"][0])                       # first chunk to trigger
        s0 = (c0 - r) % P
        last = max(i for i, t in enumerate(landed) if t // tpc == s0)
        before = oracle.track(M, N, P, r, tm, tn, landed[:last], updates=[upe] * P)
        assert before["ready"][c0] == 0
        assert oracle.track(M, N, P, r, tm, tn, landed[:last + 1], updates=[upe] * P)["ready"][c0] == 1
    # first chunk stored only: one update there, the upstream writer skips it
    st = oracle.fused_path(a, b, inc, P, r, tm, tn, two_writers=True, step0_store_only=True)
    ref = oracle.fused_path(a, b, inc, P, r, tm, tn, step0_store_only=True)
    assert np.array_equal(st["R"], ref["R"])
    assert st["counter"][r] == tpc and np.all(np.delete(st["counter"], r) == 2 * tpc)
    assert np.all(st["ready"] == 1)
    # split-K (Sec. 7.7): updates per element = split degree (+ the upstream update)
    sk = oracle.fused_path(a, b, inc, P, r, tm, tn, two_writers=True, split_k=3)
    assert np.array_equal(sk["R"], one["R"]) and np.all(sk["counter"] == (3 + 1) * tpc)
    assert np.all(sk["ready"] == 1) and list(sk["updates"]) == [4] * P
    sk0 = oracle.fused_path(a, b, inc, P, r, tm, tn, two_writers=True, split_k=3, step0_store_only=True)
    assert sk0["counter"][r] == 3 * tpc and np.all(sk0["ready"] == 1)
    # the triggered transfers
    fwd = oracle.release_ready(two["R"], two["fwd"], two["ready"], P, r)
    assert np.array_equal(fwd, one["fwd"])


# ---------------------------------------------------------------- tiles, tracker, prefixes

@pytest.mark.parametrize("M,N,P,r,tm,tn", [(8, 12, 3, 1, 4, 2), (10, 12, 2, 0, 4, 4),
                                           (256, 1024, 4, 0, 128, 128), (7, 5, 1, 0, 3, 2)])
def test_tile_map_is_chunk_major_bijection(oracle, M, N, P, r, tm, tn):
    W = N // P
    Mt, Wt = -(-M // tm), -(-W // tn)
    tpc = oracle.tiles_per_chunk(M, N, P, tm, tn)
    assert tpc == Mt * Wt
    order, _ = oracle.chunk_order(P, r)
    seen = set()
    for t in range(P * tpc):
        s, c, mi, nj = oracle.tile_of(M, N, P, r, tm, tn, t)
        assert s == t // tpc and c == order[s]
        assert 0 <= mi < Mt and 0 <= nj < Wt
        if t % tpc:                       # rows advance fastest inside a chunk
            ps, pc, pmi, pnj = oracle.tile_of(M, N, P, r, tm, tn, t - 1)
            assert (mi, nj) == ((pmi + 1) % Mt, pnj + (pmi + 1) // Mt)
        seen.add((c, mi, nj))
    assert len(seen) == P * tpc
    with pytest.raises(ValueError):
        oracle.tile_of(M, N, P, r, tm, tn, P * tpc)


def test_tracker_closed_forms_and_prefixes(oracle):
    M, N, P, r, tm, tn = 16, 24, 4, 2, 4, 3
    tpc = oracle.tiles_per_chunk(M, N, P, tm, tn)
    T = P * tpc
    order, own = oracle.chunk_order(P, r)
    for L in [0, 1, tpc - 1, tpc, tpc + 1, 2 * tpc, T - 1, T]:
        trk = oracle.track(M, N, P, r, tm, tn, np.arange(L))
        assert trk["counter"].sum() == L
        assert trk["ready"].sum() == L // tpc
        assert trk["queue_len"] == min(L // tpc, P - 1)
        assert list(trk["queue"][:trk["queue_len"]]) == list(order[:trk["queue_len"]])
        assert all(q == 0xFFFFFFFF for q in trk["queue"][trk["queue_len"]:])
    full = oracle.track(M, N, P, r, tm, tn, np.arange(T))
    assert list(full["counter"]) == [tpc] * P and list(full["ready"]) == [1] * P
    assert own not in set(full["queue"][:P - 1]) and set(full["queue"][:P - 1]) | {own} == set(range(P))


def test_tracker_is_order_invariant(oracle):
    M, N, P, r, tm, tn = 12, 20, 5, 3, 4, 2
    T = P * oracle.tiles_per_chunk(M, N, P, tm, tn)
    base = oracle.track(M, N, P, r, tm, tn, np.arange(T))
    rng = np.random.default_rng(0)
    for _ in range(20):
        trk = oracle.track(M, N, P, r, tm, tn, rng.permutation(T))
        assert np.array_equal(trk["counter"], base["counter"])
        assert np.array_equal(trk["ready"], base["ready"])
        assert trk["queue_len"] == base["queue_len"]
        assert set(trk["queue"][:P - 1]) == set(base["queue"][:P - 1])


@pytest.mark.parametrize("direct", [False, True])
def test_prefix_leaves_unexecuted_tiles_untouched(oracle, direct):
    M, N, K, P, r, tm, tn = 10, 12, 24, 3, 1, 4, 2     # ragged last tile row
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=41)
    W = N // P
    tpc = oracle.tiles_per_chunk(M, N, P, tm, tn)
    sentinel = np.full((P - 1, M, W), -7.0, dtype=np.float32)
    full = oracle.fused_path(a, b, inc, P, r, tm, tn, fwd_direct=direct, fwd_init=sentinel)
    L = tpc + 2
    part = oracle.fused_path(a, b, inc, P, r, tm, tn, tile_limit=L, fwd_direct=direct,
                             fwd_init=sentinel)
    mask, nexec, _ = oracle.executed_mask(M, N, P, r, tm, tn, L)
    assert nexec == L and mask.sum() == sum(
        (min(tm, M - mi * tm)) * tn for mi in [oracle.tile_of(M, N, P, r, tm, tn, t)[2]
                                               for t in range(L)])
    order, own = part["order"], part["own"]
    assert np.array_equal(part["fwd"][0], full["fwd"][0])          # first chunk complete
    c1 = order[1]
    if direct:
        m1 = mask[:, c1 * W:(c1 + 1) * W]
        assert np.array_equal(part["fwd"][1][m1], full["fwd"][1][m1])
        assert np.all(part["fwd"][1][~m1] == -7.0)
        assert np.array_equal(part["R"][:, order[0] * W:(order[0] + 1) * W],
                              inc[:, order[0] * W:(order[0] + 1) * W])
    else:
        assert np.all(part["fwd"][1] == -7.0)                      # not triggered yet
        assert np.array_equal(part["R"][mask], full["R"][mask])
        assert np.array_equal(part["R"][~mask], inc[~mask])
    assert np.array_equal(part["owned"], inc[:, own * W:(own + 1) * W])
    assert list(part["ready"]) == [1 if c == order[0] else 0 for c in range(P)]


def test_rejects_bad_arguments(oracle):
    with pytest.raises(ValueError):
        oracle.chunk_order(4, 4)
    with pytest.raises(ValueError):
        oracle.reduce_rows(np.zeros((2, 6)), np.zeros((2, 6), np.float32), 4)
    with pytest.raises(ValueError):
        oracle.track(8, 8, 2, 0, 4, 4, np.array([99]))


# ---------------------------------------------------------------- bfloat16 forward slots (Sec. 5.2)

def test_bf16_rounding_against_library_and_closed_forms(oracle):
    import torch
    rng = np.random.default_rng(5)
    # random bit patterns over the whole fp32 range (NaNs taken out), plus every kind of edge
    u = rng.integers(0, 2 ** 32, size=200000, dtype=np.uint64).astype(np.uint32)
    u = u[(u & 0x7FFFFFFF) <= 0x7F800000]
    edge = np.array([0x00000000, 0x80000000, 0x00000001, 0x00008000, 0x00018000, 0x7F7FFFFF,
                     0xFF7FFFFF, 0x7F800000, 0xFF800000, 0x3F800000, 0x3F808000, 0x3F818000,
                     0x3F807FFF, 0x3F808001, 0x3F817FFF, 0x3F818001], dtype=np.uint32)
    u = np.concatenate([u, edge])
    x = u.view(np.float32)
    got = oracle.to_bf16_bits(x)
    lib = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, lib)                      # the library's fp32 -> bf16 conversion
    # closed forms: a tie goes to the even neighbour, anything past it goes up, below it down
    def one(bits):
        return int(oracle.to_bf16_bits(np.array([bits], dtype=np.uint32).view(np.float32))[0])
    assert one(0x3F808000) == 0x3F80 and one(0x3F818000) == 0x3F82       # ties: down / up to even
    assert one(0x3F808001) == 0x3F81 and one(0x3F807FFF) == 0x3F80
    assert one(0x7F7FFFFF) == 0x7F80 and one(0xFF7FFFFF) == 0xFF80       # largest finite -> inf
    assert one(0x00008000) == 0x0000 and one(0x00018000) == 0x0002       # subnormal ties
    # values that fit are unchanged, and the round trip through from_bf16_bits is the identity
    k = rng.integers(0, 2 ** 16, size=5000, dtype=np.uint64).astype(np.uint16)
    k = k[(k & 0x7FFF) <= 0x7F80]
    assert np.array_equal(oracle.to_bf16_bits(oracle.from_bf16_bits(k)), k)
    assert np.array_equal(oracle.from_bf16_bits(k).view(np.uint32), k.astype(np.uint32) << 16)
    # error bound of round-to-nearest: half an ulp of the 8-bit significand, at most 2^-8 relative
    y = (rng.standard_normal(20000) * 10.0 ** rng.uniform(-20, 20, 20000)).astype(np.float32)
    err = np.abs(oracle.from_bf16_bits(oracle.to_bf16_bits(y)).astype(np.float64) - y)
    assert np.all(err <= np.abs(y.astype(np.float64)) * 2.0 ** -8)
    nan = oracle.to_bf16_bits(np.array([np.nan, -np.nan], dtype=np.float32))
    assert np.all((nan & 0x7FFF) > 0x7F80)


@pytest.mark.parametrize("direct", [False, True])
def test_bf16_forward_slots_are_the_rounded_fp32_ones(oracle, direct):
    """Only the forward slots change format: same tiles written, each value the fp32 one
    rounded once; R, the owned chunk and the tracker are those of the fp32 path."""
    M, N, K, P, r, tm, tn = 10, 24, 24, 3, 1, 4, 4
    a, b, inc = wl.make_inputs(wl.make_shape("s", M, N, K, P, r, tm, tn), seed=77)
    W = N // P
    tpc = oracle.tiles_per_chunk(M, N, P, tm, tn)
    for limit in (-1, tpc + 3):
        f32 = oracle.fused_path(a, b, inc, P, r, tm, tn, fwd_direct=direct, tile_limit=limit,
                                fwd_init=np.full((P - 1, M, W), -7.0, np.float32))
        b16 = oracle.fused_path(a, b, inc, P, r, tm, tn, fwd_direct=direct, tile_limit=limit,
                                fwd_init=np.full((P - 1, M, W), 0xABCD, np.uint16), fwd_bf16=True)
        written = f32["fwd"] != -7.0
        assert b16["fwd"].dtype == np.uint16
        assert np.array_equal(b16["fwd"][written], oracle.to_bf16_bits(f32["fwd"][written]))
        assert np.all(b16["fwd"][~written] == 0xABCD)
        assert np.array_equal(b16["R"], f32["R"]) and np.array_equal(b16["owned"], f32["owned"])
        for key in ("counter", "ready", "queue"):
            assert np.array_equal(b16[key], f32[key])
        # a forwarded value is within half a bf16 ulp of the exact sum it stands for
        S = oracle.reduce_rows(oracle.gemm_rows(a, b), inc, P)
        for s in range(P - 1):
            c = int(f32["order"][s])
            w_ = written[s]
            exact = S[:, c * W:(c + 1) * W][w_].astype(np.float64)
            assert np.all(np.abs(oracle.from_bf16_bits(b16["fwd"][s][w_]) - exact)
                          <= np.abs(exact) * 2.0 ** -8 + 1e-30)
    # the triggered transfers of two-writer mode round the same way
    tw = oracle.fused_path(a, b, inc, P, r, tm, tn, two_writers=True)
    rel = oracle.release_ready(tw["R"], np.zeros((P - 1, M, W), np.uint16), tw["ready"], P, r,
                               fwd_bf16=True)
    full = oracle.fused_path(a, b, inc, P, r, tm, tn, fwd_bf16=True)
    assert np.array_equal(rel, full["fwd"])

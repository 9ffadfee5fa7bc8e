"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element,
on the same seeded inputs.  Integers (counters, ready flags, queue as a set, owned / forward
partition) must be bit-exact; fp32 outputs must be within a normwise relative error of 5e-3
(bf16 inputs, fp32 accumulation), and bit-exact on small-integer inputs where fp32
accumulation is exact in any order."""
import numpy as np
import pytest

from paper_2401_16677_amd import binding as t3
from paper_2401_16677_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = 5e-3          # contract
EXPECT = 1e-4       # what fp32 accumulation should actually achieve


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "needs a GPU"
    from tests import gpu_harness
    return gpu_harness


def _check_ints(got, want, tp, own):
    assert np.array_equal(got["counter"], want["counter"])
    assert np.array_equal(got["ready"], want["ready"])
    assert got["queue_len"] == want["queue_len"]
    n = want["queue_len"]
    assert set(got["queue"][:n].tolist()) == set(want["queue"][:n].tolist())
    assert len(set(got["queue"][:n].tolist())) == n and own not in got["queue"][:n]
    assert np.all(got["queue"][n:] == 0xFFFFFFFF)
    assert got["error"] == 0


def _flags(step0, direct):
    return (t3.T3_FLAG_STEP0_STORE_ONLY if step0 else 0) | (t3.T3_FLAG_FWD_DIRECT if direct else 0)


# several tiles per chunk, ragged M / W / K tails, every tile shape, both release modes
EXACT_CASES = [
    # M,   N,    K,   tp, rank, tile
    (256, 1024, 256, 4, 0, (128, 128)),
    (300, 800, 200, 4, 2, (128, 128)),
    (520, 1056, 72, 2, 1, (256, 128)),
    (260, 1200, 136, 3, 0, (128, 256)),
    (512, 512, 64, 1, 0, (128, 128)),
    (100, 64, 8, 8, 5, (128, 128)),
    (600, 1280, 104, 2, 0, (256, 256)),
    (512, 2048, 160, 4, 3, (256, 256)),
    # long K (11 to 64 slabs of 64), full and ragged tiles
    (512, 1024, 1216, 2, 1, (256, 256)),
    (600, 1280, 1160, 2, 0, (256, 256)),
    (300, 800, 712, 4, 2, (128, 128)),
    (512, 1024, 4096, 2, 0, (256, 256)),
]


@pytest.mark.parametrize("direct", [False, True])
@pytest.mark.parametrize("step0", [False, True])
@pytest.mark.parametrize("case", EXACT_CASES)
def test_integer_inputs_bit_exact(gpu, oracle, case, step0, direct):
    M, N, K, tp, rank, tile = case
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=100 + M)
    print(f"case={case} step0={step0} direct={direct}", flush=True)
    want = oracle.fused_path(a, b, inc, tp, rank, *tile, step0_store_only=step0,
                             fwd_direct=direct,
                             fwd_init=np.full((tp - 1, M, N // tp), gpu.SENTINEL, np.float32))
    got = gpu.run_gpu(a, b, inc, tp, rank, tile, flags=_flags(step0, direct), ldr_pad=4,
                      lda_pad=8)
    assert np.array_equal(got["R"], want["R"])
    assert np.array_equal(got["fwd"], want["fwd"])
    assert np.all(got["R_pad"] == 123.0)           # nothing written outside the M x N view
    W = N // tp
    assert np.array_equal(got["R"][:, want["own"] * W:(want["own"] + 1) * W], want["owned"])
    _check_ints(got, want, tp, want["own"])


KN_CASES = [
    # M,   N,    K,   tp, rank, tile          (K a multiple of 64, W a multiple of 8)
    (256, 1024, 256, 4, 0, (128, 128)),
    (300, 832, 192, 4, 2, (128, 128)),
    (520, 1072, 128, 2, 1, (256, 128)),
    (260, 1200, 320, 3, 0, (128, 256)),
    (600, 1296, 1216, 2, 0, (256, 256)),
    (512, 2048, 64, 4, 3, (256, 256)),
]


@pytest.mark.parametrize("direct", [False, True])
@pytest.mark.parametrize("unfused", [False, True])
@pytest.mark.parametrize("case", KN_CASES)
def test_b_stored_k_by_n_bit_exact(gpu, oracle, case, unfused, direct):
    """B stored K x N, N contiguous (the backward-pass GEMMs' layout): same results as with the
    N x K storage, every tile shape, ragged M and W, padded leading dimensions."""
    M, N, K, tp, rank, tile = case
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=700 + M)
    print(f"case={case} unfused={unfused} direct={direct}", flush=True)
    want = oracle.fused_path(a, np.ascontiguousarray(b.T), inc, tp, rank, *tile, b_layout=oracle.B_KN,
                             fwd_direct=direct,
                             fwd_init=np.full((tp - 1, M, N // tp), gpu.SENTINEL, np.float32))
    got = gpu.run_gpu(a, b, inc, tp, rank, tile, flags=_flags(False, direct), unfused=unfused,
                      lda_pad=8, b_kn=True)
    assert np.array_equal(got["R"], want["R"])
    assert np.array_equal(got["fwd"], want["fwd"])
    _check_ints(got, want, tp, want["own"])
    if unfused:
        assert np.array_equal(got["C"], oracle.gemm_rows(a, b).astype(np.float32))


KM_CASES = [
    # M,   N,    K,   tp, rank, tile          (K a multiple of 64, M a multiple of 8)
    (256, 1024, 256, 4, 0, (128, 128)),
    (304, 832, 192, 4, 2, (128, 128)),
    (520, 1072, 128, 2, 1, (256, 128)),
    (264, 1200, 320, 3, 0, (128, 256)),
    (600, 1296, 1216, 2, 0, (256, 256)),
    (512, 2048, 64, 4, 3, (256, 256)),
]


@pytest.mark.parametrize("b_kn", [False, True])
@pytest.mark.parametrize("mode", ["fused_direct", "fused_copy", "unfused_direct"])
@pytest.mark.parametrize("case", KM_CASES)
def test_a_stored_k_by_m_bit_exact(gpu, oracle, case, mode, b_kn):
    """A stored K x M, M contiguous (the transposed operand of the backward-pass GEMMs, Sec. 5.2),
    with B in either layout: same results as with the M x K storage, every tile shape, ragged M
    and W, padded leading dimensions."""
    M, N, K, tp, rank, tile = case
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=1700 + M)
    direct, unfused = mode.endswith("direct"), mode.startswith("unfused")
    print(f"case={case} mode={mode} b_kn={b_kn}", flush=True)
    want = oracle.fused_path(np.ascontiguousarray(a.T), np.ascontiguousarray(b.T) if b_kn else b, inc, tp, rank,
                             *tile, a_layout=oracle.A_KM, b_layout=oracle.B_KN if b_kn else oracle.B_NK,
                             fwd_direct=direct,
                             fwd_init=np.full((tp - 1, M, N // tp), gpu.SENTINEL, np.float32))
    got = gpu.run_gpu(a, b, inc, tp, rank, tile, flags=_flags(False, direct), unfused=unfused,
                      lda_pad=8, b_kn=b_kn, a_km=True)
    assert np.array_equal(got["R"], want["R"])
    assert np.array_equal(got["fwd"], want["fwd"])
    _check_ints(got, want, tp, want["own"])
    if unfused:
        assert np.array_equal(got["C"], oracle.gemm_rows(a, b).astype(np.float32))


@pytest.mark.parametrize("direct", [False, True])
@pytest.mark.parametrize("case", EXACT_CASES[:4])
def test_unfused_baseline_bit_exact(gpu, oracle, case, direct):
    M, N, K, tp, rank, tile = case
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=200 + M)
    print(f"case={case} direct={direct}", flush=True)
    want = oracle.fused_path(a, b, inc, tp, rank, *tile, fwd_direct=direct,
                             fwd_init=np.full((tp - 1, M, N // tp), gpu.SENTINEL, np.float32))
    got = gpu.run_gpu(a, b, inc, tp, rank, tile, flags=_flags(False, direct), unfused=True)
    assert np.array_equal(got["C"], oracle.gemm_rows(a, b).astype(np.float32))
    assert np.array_equal(got["R"], want["R"])
    assert np.array_equal(got["fwd"], want["fwd"])
    _check_ints(got, want, tp, want["own"])


@pytest.mark.parametrize("direct", [False, True])
@pytest.mark.parametrize("limit_kind", ["zero", "one", "mid_chunk", "one_chunk", "chunk_plus",
                                        "all_but_one"])
def test_tile_limit_prefix_bit_exact(gpu, oracle, limit_kind, direct):
    M, N, K, tp, rank, tile = 300, 1536, 128, 3, 1, (128, 128)
    tpc = oracle.tiles_per_chunk(M, N, tp, *tile)
    L = {"zero": 0, "one": 1, "mid_chunk": tpc // 2, "one_chunk": tpc, "chunk_plus": tpc + 5,
         "all_but_one": 3 * tpc - 1}[limit_kind]
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=300)
    print(f"limit={L} of {3 * tpc} direct={direct}", flush=True)
    want = oracle.fused_path(a, b, inc, tp, rank, *tile, tile_limit=L, fwd_direct=direct,
                             fwd_init=np.full((tp - 1, M, N // tp), gpu.SENTINEL, np.float32))
    got = gpu.run_gpu(a, b, inc, tp, rank, tile, flags=_flags(False, direct), tile_limit=L)
    assert np.array_equal(got["R"], want["R"])
    assert np.array_equal(got["fwd"], want["fwd"])
    _check_ints(got, want, tp, want["own"])


@pytest.mark.parametrize("direct", [False, True])
@pytest.mark.parametrize("unfused", [False, True])
@pytest.mark.parametrize("rng_kind", ["step1", "step_last", "straddle", "inside", "empty"])
def test_tile_range_bit_exact(gpu, oracle, rng_kind, unfused, direct):
    """[tile_begin, tile_limit): one ring step, ranges cutting through chunks, an empty range."""
    M, N, K, tp, rank, tile = 300, 1536, 72, 3, 2, (128, 128)
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=58)
    tpc = oracle.tiles_per_chunk(M, N, tp, *tile)
    begin, limit = {"step1": (tpc, 2 * tpc), "step_last": (2 * tpc, 3 * tpc),
                    "straddle": (tpc - 2, 2 * tpc + 1), "inside": (tpc + 1, tpc + 3),
                    "empty": (5, 5)}[rng_kind]
    print(f"range=[{begin},{limit}) unfused={unfused} direct={direct}", flush=True)
    sent = np.full((tp - 1, M, N // tp), gpu.SENTINEL, np.float32)
    want = oracle.fused_path(a, b, inc, tp, rank, *tile, tile_begin=begin, tile_limit=limit,
                             fwd_direct=direct, fwd_init=sent)
    got = gpu.run_gpu(a, b, inc, tp, rank, tile, flags=_flags(False, direct), tile_begin=begin,
                      tile_limit=limit, unfused=unfused)
    assert np.array_equal(got["R"], want["R"])
    assert np.array_equal(got["fwd"], want["fwd"])
    if rng_kind == "empty":
        assert got["gen"] == 0          # nothing was launched
    else:
        _check_ints(got, want, tp, want["own"])


@pytest.mark.parametrize("kind", ["integer", "normal"])
def test_ring_of_virtual_ranks_closes_on_unsliced_gemm(gpu, oracle, kind):
    """Whole ring reduce-scatter on one GPU (Sec. 2.3, Sec. 4.1): P virtual ranks, each with its own
    K-slice, run ring step by ring step through the C ABI; after every step rank q's forward
    slot is handed to rank q-1 as the incoming partial of its next chunk.  At the end every
    rank must own the UNSLICED GEMM's columns of its chunk."""
    import torch
    P, M, W, ks, tile = 4, 512, 512, 192, (256, 256)
    N, Kfull = P * W, P * ks
    if kind == "integer":
        a, b, _ = wl.make_integer_inputs(M, N, Kfull, seed=404)
    else:
        w = wl.make_shape("ring", M, N, Kfull, P, 0, *tile)
        a, b, _ = wl.make_inputs(w, seed=405)
    whole = oracle.gemm_rows(a, b)                       # fp64, all of K
    dev = torch.device("cuda:0")
    A_r = [gpu.to_dev_bits(np.ascontiguousarray(a[:, q * ks:(q + 1) * ks])) for q in range(P)]
    B_r = [gpu.to_dev_bits(np.ascontiguousarray(b[:, q * ks:(q + 1) * ks])) for q in range(P)]
    R_r = [torch.full((M, N), 99.0, dtype=torch.float32, device=dev) for _ in range(P)]
    F_r = [torch.full((P - 1, M, W), gpu.SENTINEL, dtype=torch.float32, device=dev) for _ in range(P)]
    T_r = [torch.zeros(t3.t3_track_words(P), dtype=torch.int32, device=dev) for _ in range(P)]
    for q in range(P):
        t3.t3_track_reset(P, T_r[q])
    flags = t3.T3_FLAG_FWD_DIRECT | t3.T3_FLAG_STEP0_STORE_ONLY
    tpc = oracle.tiles_per_chunk(M, N, P, *tile)
    for s in range(P):
        for q in range(P):
            p = t3.problem(M, N, ks, P, q, *tile, flags=flags, tile_begin=s * tpc,
                           tile_limit=(s + 1) * tpc)
            t3.t3_gemm_rs_fused(p, A_r[q], B_r[q], R_r[q], F_r[q], T_r[q])
        torch.cuda.synchronize()
        for q in range(P):
            tr = t3.read_track(T_r[q], P)
            c = (q + s) % P
            assert tr["gen"] == s + 1 and tr["error"] == 0
            assert tr["counter"][c] == tpc and tr["ready"][c] == 1 and tr["counter"].sum() == tpc
            assert tr["queue_len"] == (1 if s < P - 1 else 0)
            if s < P - 1:                # the triggered chunk travels to the downstream neighbour
                assert tr["queue"][0] == c
                R_r[(q - 1) % P][:, c * W:(c + 1) * W] = F_r[q][s]
    print(f"ring of {P} ranks, {kind} inputs", flush=True)
    for q in range(P):
        own = (q - 1) % P
        got = R_r[q][:, own * W:(own + 1) * W].cpu().numpy()
        want = whole[:, own * W:(own + 1) * W]
        if kind == "integer":
            assert np.array_equal(got, want.astype(np.float32))
        else:
            e = gpu.rel_err(got, want)
            print(f"rank {q} owns chunk {own}: normwise error {e:.2e}", flush=True)
            assert e <= EXPECT
    # The sequential all-gather that follows (Sec. 2.3, Sec. 5.3): P-1 steps of t3_ag_step, every
    # rank pulling from its upstream neighbour's buffer; all ranks move together, so a step reads
    # what the neighbour held BEFORE the step (snapshots stand in for the simultaneous transfers).
    owned = [R_r[q][:, ((q - 1) % P) * W:(((q - 1) % P) + 1) * W].clone() for q in range(P)]
    for g in range(P - 1):
        snap = [r.clone() for r in R_r]
        for q in range(P):
            t3.t3_ag_step(t3.problem(M, N, ks, P, q), g, snap[(q + 1) % P], R_r[q])
        torch.cuda.synchronize()
    full = np.concatenate([owned[(c + 1) % P].cpu().numpy() for c in range(P)], axis=1)   # chunk c is rank c+1's
    for q in range(P):
        got = R_r[q].cpu().numpy()
        assert np.array_equal(got, full)              # copies: bit for bit what the owners reduced
        if kind == "integer":
            assert np.array_equal(got, whole.astype(np.float32))
        else:
            assert gpu.rel_err(got, whole) <= EXPECT


def test_all_gather_step_shapes_and_refusals(gpu, oracle):
    """t3_ag_step on a ragged shape with padded leading dimensions: only the chunk's columns
    change, bit for bit the oracle's step; bad steps and misaligned widths are refused."""
    import torch
    M, N, P, r = 301, 5 * 52, 5, 3
    rng = np.random.default_rng(9)
    up = rng.standard_normal((M, N + 8)).astype(np.float32)
    mine = rng.standard_normal((M, N + 4)).astype(np.float32)
    dev = torch.device("cuda:0")
    for g in range(P - 1):
        U, R = torch.from_numpy(up).to(dev), torch.from_numpy(mine).to(dev)
        p = t3.problem(M, N, 64, P, r, ldr=N + 4)
        t3.t3_ag_step(p, g, U, R, ld_up=N + 8)
        torch.cuda.synchronize()
        want = oracle.all_gather_step(up[:, :N], mine[:, :N], P, r, g)
        got = R.cpu().numpy()
        assert np.array_equal(got[:, :N], want) and np.array_equal(got[:, N:], mine[:, N:])
    for bad in (-1, P - 1):
        with pytest.raises(t3.T3Error) as e:
            t3.t3_ag_step(t3.problem(M, N, 64, P, r, ldr=N + 4), bad, U, R, ld_up=N + 8)
        assert e.value.status == t3.T3_ERR_BAD_SHAPE
    with pytest.raises(t3.T3Error) as e:
        t3.t3_ag_step(t3.problem(M, 5 * 50, 64, P, r, ldr=N + 4), 0, U, R, ld_up=N + 8)
    assert e.value.status == t3.T3_ERR_ALIGN


def _run_two_writers(gpu, a, b, inc, tp, rank, tile, *, order, step0=False, tile_begin=0, tile_limit=-1,
                     split_k=0, upstream_agents=0):
    """Two-writer mode through the C ABI: the fused call and the upstream update, one after the
    other in either order or on two streams at once, then the triggered transfers."""
    import torch
    M, K = a.shape
    N = b.shape[0]
    W = N // tp
    dev = torch.device("cuda:0")
    A, B = gpu.to_dev_bits(a), gpu.to_dev_bits(b)
    INC = torch.from_numpy(inc).to(dev)
    R = torch.zeros((M, N), dtype=torch.float32, device=dev)
    fwd = torch.full((tp - 1, M, W), gpu.SENTINEL, dtype=torch.float32, device=dev)
    track = torch.full((t3.t3_track_words(tp),), 0x5A5A5A5A, dtype=torch.int32, device=dev)
    flags = t3.T3_FLAG_TWO_WRITERS | (t3.T3_FLAG_STEP0_STORE_ONLY if step0 else 0)
    p = t3.problem(M, N, K, tp, rank, *tile, ldc=N, flags=flags, tile_begin=tile_begin,
                   tile_limit=tile_limit, split_k=split_k, upstream_agents=upstream_agents)
    t3.t3_track_reset(tp, track)
    torch.cuda.synchronize()
    if order == "local_first":
        t3.t3_gemm_rs_fused(p, A, B, R, None, track)
        t3.t3_upstream_update(p, INC, R, track)
    elif order == "upstream_first":
        t3.t3_upstream_update(p, INC, R, track)
        t3.t3_gemm_rs_fused(p, A, B, R, None, track)
    else:                                   # at the same time, on two streams
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        with torch.cuda.stream(s1):
            t3.t3_gemm_rs_fused(p, A, B, R, None, track)
        with torch.cuda.stream(s2):
            t3.t3_upstream_update(p, INC, R, track)
    torch.cuda.synchronize()
    tr = t3.read_track(track, tp)
    t3.t3_release_chunks(p, R, fwd, track)
    torch.cuda.synchronize()
    return R.cpu().numpy(), fwd.cpu().numpy(), tr


@pytest.mark.parametrize("order", ["local_first", "upstream_first", "concurrent"])
@pytest.mark.parametrize("step0", [False, True])
@pytest.mark.parametrize("case", [(300, 800, 200, 4, 2, (128, 128)), (600, 1280, 1160, 2, 0, (256, 256)),
                                  (1024, 4096, 512, 4, 1, (256, 256)), (520, 1056, 72, 2, 1, (256, 128))])
def test_two_writers_bit_exact(gpu, oracle, case, step0, order):
    """Sec. 4.1 / 4.2.1: the local GEMM's tiles and the upstream update are both added into R with
    atomics; every element gets two updates, a chunk triggers after both writers' tiles."""
    M, N, K, tp, rank, tile = case
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=300 + M)
    print(f"case={case} step0={step0} order={order}", flush=True)
    sent = np.full((tp - 1, M, N // tp), gpu.SENTINEL, np.float32)
    want = oracle.fused_path(a, b, inc, tp, rank, *tile, two_writers=True, step0_store_only=step0,
                             fwd_init=sent)
    R, fwd, tr = _run_two_writers(gpu, a, b, inc, tp, rank, tile, order=order, step0=step0)
    assert np.array_equal(R, want["R"])
    assert np.array_equal(tr["counter"], want["counter"]) and np.array_equal(tr["ready"], want["ready"])
    assert tr["queue_len"] == want["queue_len"] == tp - 1 and tr["error"] == 0 and tr["gen"] == 1
    assert set(tr["queue"][:tp - 1].tolist()) == set(want["queue"][:tp - 1].tolist())
    assert np.array_equal(fwd, oracle.release_ready(want["R"], sent, want["ready"], tp, rank))


@pytest.mark.parametrize("agents", [1, 3, 1000])
@pytest.mark.parametrize("case", [(300, 800, 200, 4, 2, (128, 128)), (1024, 4096, 512, 4, 1, (256, 256))])
def test_two_writers_throttled_upstream_bit_exact(gpu, oracle, case, agents):
    """The upstream writer held to a few workgroups that walk the tiles (the software stand-in for
    the arbitration of Sec. 4.5) changes when its updates land, not what is computed."""
    M, N, K, tp, rank, tile = case
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=700 + M)
    print(f"case={case} agents={agents}", flush=True)
    sent = np.full((tp - 1, M, N // tp), gpu.SENTINEL, np.float32)
    want = oracle.fused_path(a, b, inc, tp, rank, *tile, two_writers=True, fwd_init=sent)
    R, fwd, tr = _run_two_writers(gpu, a, b, inc, tp, rank, tile, order="concurrent",
                                  upstream_agents=agents)
    assert np.array_equal(R, want["R"])
    assert np.array_equal(tr["counter"], want["counter"]) and np.all(tr["ready"] == 1)
    assert tr["queue_len"] == tp - 1 and tr["error"] == 0 and tr["gen"] == 1
    assert np.array_equal(fwd, oracle.release_ready(want["R"], sent, want["ready"], tp, rank))


@pytest.mark.parametrize("step0", [False, True])
@pytest.mark.parametrize("case", [(300, 800, 200, 4, 2, (128, 128), 3), (600, 1280, 1160, 2, 0, (256, 256), 4),
                                  (512, 1024, 136, 2, 1, (256, 128), 2)])
def test_split_k_bit_exact(gpu, oracle, case, step0):
    """Sec. 7.7: split-K producer, updates per element = split degree (+ 1 for the upstream update)."""
    M, N, K, tp, rank, tile, S = case
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=500 + M)
    print(f"case={case} step0={step0}", flush=True)
    sent = np.full((tp - 1, M, N // tp), gpu.SENTINEL, np.float32)
    want = oracle.fused_path(a, b, inc, tp, rank, *tile, two_writers=True, step0_store_only=step0,
                             fwd_init=sent, split_k=S)
    R, fwd, tr = _run_two_writers(gpu, a, b, inc, tp, rank, tile, order="concurrent", step0=step0,
                                  split_k=S)
    assert np.array_equal(R, want["R"])
    assert np.array_equal(tr["counter"], want["counter"]) and np.all(tr["ready"] == 1)
    assert tr["queue_len"] == tp - 1 and tr["error"] == 0 and tr["gen"] == 1
    assert np.array_equal(fwd, oracle.release_ready(want["R"], sent, want["ready"], tp, rank))


def test_two_writers_one_ring_step_and_float(gpu, oracle):
    """A tile range (ring step 1) with two writers: only that chunk triggers; and normal inputs
    within the floating-point bar."""
    M, N, K, tp, rank, tile = 512, 2048, 320, 4, 3, (256, 256)
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=17)
    tpc = oracle.tiles_per_chunk(M, N, tp, *tile)
    sent = np.full((tp - 1, M, N // tp), gpu.SENTINEL, np.float32)
    want = oracle.fused_path(a, b, inc, tp, rank, *tile, two_writers=True, tile_begin=tpc,
                             tile_limit=2 * tpc, fwd_init=sent)
    R, fwd, tr = _run_two_writers(gpu, a, b, inc, tp, rank, tile, order="concurrent",
                                  tile_begin=tpc, tile_limit=2 * tpc)
    assert np.array_equal(R, want["R"])
    assert np.array_equal(tr["counter"], want["counter"]) and np.array_equal(tr["ready"], want["ready"])
    assert tr["queue_len"] == 1 and tr["ready"].sum() == 1
    assert np.array_equal(fwd, oracle.release_ready(want["R"], sent, want["ready"], tp, rank))
    w = wl.make_shape("two", 1024, 4096, 1024, 4, 1, 256, 256)
    a, b, inc = wl.make_inputs(w, seed=18)
    want = oracle.fused_path(a, b, inc, 4, 1, 256, 256, two_writers=True)
    R, fwd, tr = _run_two_writers(gpu, a, b, inc, 4, 1, (256, 256), order="concurrent")
    e = gpu.rel_err(R, want["R"])
    print(f"two writers, normal inputs: normwise error {e:.2e}", flush=True)
    assert e <= EXPECT and np.all(tr["ready"] == 1)


def test_tiny_outproj_config_float_parity(gpu, oracle):
    w = wl.WORKLOADS["tiny_outproj"]
    a, b, inc = wl.make_inputs(w)
    want = oracle.fused_path(a, b, inc, w.tp, w.rank, w.tile_m, w.tile_n)
    for flags in (0, t3.T3_FLAG_FWD_DIRECT):
        got = gpu.run_gpu(a, b, inc, w.tp, w.rank, (w.tile_m, w.tile_n), flags=flags)
        errs = [gpu.rel_err(got["fwd"][s], want["fwd"][s]) for s in range(w.tp - 1)]
        own = want["own"]
        errs.append(gpu.rel_err(got["R"][:, own * w.W:(own + 1) * w.W], want["owned"]))
        print(f"flags={flags} normwise errors {errs}", flush=True)
        assert max(errs) <= TOL and max(errs) <= EXPECT
        _check_ints(got, want, w.tp, own)


@pytest.mark.parametrize("tile", [(256, 256), (256, 128), (128, 256), (128, 128)])
def test_float_multi_tile_ragged(gpu, oracle, tile):
    M, N, K, tp, rank = 700, 2080, 328, 4, 3
    w = wl.make_shape("ragged", M, N, K, tp, rank, *tile)
    a, b, inc = wl.make_inputs(w, seed=77)
    want = oracle.fused_path(a, b, inc, tp, rank, *tile)
    got = gpu.run_gpu(a, b, inc, tp, rank, tile)
    assert gpu.rel_err(got["R"], want["R"]) <= EXPECT
    assert gpu.rel_err(got["fwd"], want["fwd"]) <= EXPECT
    assert np.abs(got["R"] - want["R"]).max() <= 1e-4 * np.abs(want["R"]).max()
    _check_ints(got, want, tp, want["own"])


# ---------------------------------------------------------------- bfloat16 forward slots

@pytest.mark.parametrize("mode", ["fused_direct", "fused_copy", "unfused_direct", "unfused_copy"])
@pytest.mark.parametrize("step0", [False, True])
@pytest.mark.parametrize("case", EXACT_CASES)
def test_bf16_forward_slots_bit_exact(gpu, oracle, case, step0, mode):
    """T3_FLAG_FWD_BF16: what is forwarded is the fp32 sum rounded to nearest even (Sec. 5.2's
    16-bit activations); with integer inputs the fp32 sums are exact, so every bit is fixed."""
    M, N, K, tp, rank, tile = case
    assert (N // tp) % 8 == 0
    direct, unfused = mode.endswith("direct"), mode.startswith("unfused")
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=900 + M)
    inc = inc * np.float32(257.0)      # sums well past 256: most need rounding to 8 bits
    print(f"case={case} step0={step0} mode={mode}", flush=True)
    want = oracle.fused_path(a, b, inc, tp, rank, *tile, step0_store_only=step0, fwd_direct=direct,
                             fwd_bf16=True,
                             fwd_init=np.full((tp - 1, M, N // tp), gpu.SENTINEL_BF16, np.uint16))
    got = gpu.run_gpu(a, b, inc, tp, rank, tile, unfused=unfused, ldr_pad=4, lda_pad=8,
                      flags=_flags(step0, direct) | t3.T3_FLAG_FWD_BF16)
    assert got["fwd"].dtype == np.uint16 and np.array_equal(got["fwd"], want["fwd"])
    assert np.array_equal(got["R"], want["R"]) and np.all(got["R_pad"] == 123.0)
    _check_ints(got, want, tp, want["own"])
    if tp > 1 and not step0:      # the case does exercise rounding (a stored-only first chunk
        # holds the small integers of C alone)
        exact = oracle.fused_path(a, b, inc, tp, rank, *tile, step0_store_only=step0,
                                  fwd_direct=direct)["fwd"]
        assert np.any(oracle.from_bf16_bits(want["fwd"]) != exact)


@pytest.mark.parametrize("direct", [False, True])
def test_bf16_forward_slots_partial_range_and_float(gpu, oracle, direct):
    """A tile range leaves the other elements of the bfloat16 slots untouched; float inputs agree
    to the fp32 path's tolerance plus one rounding to 8 bits."""
    M, N, K, tp, rank, tile = 700, 2080, 328, 4, 3, (256, 128)
    w = wl.make_shape("ragged", M, N, K, tp, rank, *tile)
    a, b, inc = wl.make_inputs(w, seed=78)
    W = N // tp
    tpc = oracle.tiles_per_chunk(M, N, tp, *tile)
    sent = np.full((tp - 1, M, W), gpu.SENTINEL_BF16, np.uint16)
    for begin, limit in ((0, -1), (0, tpc + 5), (2, tpc + 5)):
        want = oracle.fused_path(a, b, inc, tp, rank, *tile, fwd_direct=direct, fwd_bf16=True,
                                 tile_begin=begin, tile_limit=limit, fwd_init=sent)
        got = gpu.run_gpu(a, b, inc, tp, rank, tile, tile_begin=begin, tile_limit=limit,
                          flags=_flags(False, direct) | t3.T3_FLAG_FWD_BF16)
        written = want["fwd"] != gpu.SENTINEL_BF16
        assert np.array_equal(got["fwd"] != gpu.SENTINEL_BF16, written)
        assert gpu.rel_err(got["R"], want["R"]) <= EXPECT
        _check_ints(got, want, tp, want["own"])
        if not written.any():      # (a range that completes no chunk releases nothing by copy)
            assert not direct and begin > 0
            continue
        g, x = oracle.from_bf16_bits(got["fwd"][written]), oracle.from_bf16_bits(want["fwd"][written])
        # fp32 sums that differ in their last places (by up to 1e-4 of the largest sum where
        # terms cancel) may round to neighbouring bfloat16 values
        assert np.all(np.abs(g.astype(np.float64) - x)
                      <= np.abs(x) * 2.0 ** -7 + 1e-4 * np.abs(x).max())
        assert np.mean(got["fwd"][written] == want["fwd"][written]) > 0.99
        assert gpu.rel_err(g, x) <= EXPECT + 2.0 ** -9


def test_bf16_forward_slots_two_writer_release(gpu, oracle):
    """The triggered transfers of two-writer mode (t3_release_chunks) round the same way."""
    import torch
    M, N, K, tp, rank, tile = 300, 800, 200, 4, 2, (128, 128)
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=950)
    inc = inc * np.float32(257.0)
    W = N // tp
    dev = torch.device("cuda:0")
    A, B = gpu.to_dev_bits(a), gpu.to_dev_bits(b)
    INC = torch.from_numpy(inc).to(dev)
    R = torch.zeros((M, N), dtype=torch.float32, device=dev)
    fwd = torch.full((tp - 1, M, W), gpu.SENTINEL_BF16 - 65536, dtype=torch.int16, device=dev)
    track = torch.zeros(t3.t3_track_words(tp), dtype=torch.int32, device=dev)
    p = t3.problem(M, N, K, tp, rank, *tile, ldc=N,
                   flags=t3.T3_FLAG_TWO_WRITERS | t3.T3_FLAG_FWD_BF16)
    t3.t3_track_reset(tp, track)
    t3.t3_gemm_rs_fused(p, A, B, R, None, track)
    t3.t3_upstream_update(p, INC, R, track)
    t3.t3_release_chunks(p, R, fwd, track)
    torch.cuda.synchronize()
    want = oracle.fused_path(a, b, inc, tp, rank, *tile, two_writers=True)
    rel = oracle.release_ready(want["R"], np.full((tp - 1, M, W), gpu.SENTINEL_BF16, np.uint16),
                               want["ready"], tp, rank, fwd_bf16=True)
    assert np.array_equal(R.cpu().numpy(), want["R"])
    assert np.array_equal(fwd.cpu().numpy().view(np.uint16), rel)


EXTREME_CASES = [
    # M, N,   K,  tp, rank, tile          what is extreme
    (1, 256, 8, 64, 63, (128, 128)),      # one row, 64 chunks of 4 columns, K = one 16-byte piece
    (1, 8, 64, 1, 0, (256, 256)),         # a single ragged tile, no ring
    (257, 1032, 64, 3, 2, (256, 256)),    # one full tile row + one row; W = 344 = 256 + 88
    (129, 520, 72, 1, 0, (128, 256)),     # K = one slab + 8
    (640, 4096, 8, 32, 17, (256, 128)),   # 32 chunks, K below a slab: register path only
    (2049, 768, 128, 2, 1, (256, 256)),   # 9 tile rows, last one a single row
    (512, 12288, 64, 48, 47, (128, 128)), # 48 chunks, last rank
]


@pytest.mark.parametrize("direct", [False, True])
@pytest.mark.parametrize("case", EXTREME_CASES)
def test_extreme_shapes_bit_exact(gpu, oracle, case, direct):
    M, N, K, tp, rank, tile = case
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=1300 + M + tp)
    print(f"case={case} direct={direct}", flush=True)
    sent = np.full((tp - 1, M, N // tp), gpu.SENTINEL, np.float32)
    for unfused in (False, True):
        want = oracle.fused_path(a, b, inc, tp, rank, *tile, fwd_direct=direct, fwd_init=sent)
        got = gpu.run_gpu(a, b, inc, tp, rank, tile, flags=_flags(False, direct), unfused=unfused,
                          ldr_pad=8)
        assert np.array_equal(got["R"], want["R"]) and np.all(got["R_pad"] == 123.0)
        assert np.array_equal(got["fwd"], want["fwd"])
        _check_ints(got, want, tp, want["own"])


def _random_case(rng):
    tp = int(rng.integers(1, 7))
    tile = [(128, 128), (256, 128), (128, 256), (256, 256)][int(rng.integers(0, 4))]
    bf16 = bool(rng.integers(0, 2))
    kn = bool(rng.integers(0, 2))
    w_unit = 8 if (bf16 or kn) else 4
    W = w_unit * int(rng.integers(1, 1 + 600 // w_unit))
    M = int(rng.integers(1, 700))
    K = 64 * int(rng.integers(1, 8)) if kn else 8 * int(rng.integers(1, 60))
    return dict(M=M, N=W * tp, K=K, tp=tp, rank=int(rng.integers(0, tp)), tile=tile, bf16=bf16, kn=kn,
                direct=bool(rng.integers(0, 2)), step0=bool(rng.integers(0, 2)),
                unfused=bool(rng.integers(0, 4) == 0), ldr_pad=4 * int(rng.integers(0, 3)),
                lda_pad=8 * int(rng.integers(0, 3)))


@pytest.mark.parametrize("seed", range(32))
def test_random_shapes_and_modes_bit_exact(gpu, oracle, seed):
    """Seeded random shapes (ragged everywhere), tile shapes, layouts, release modes and forward
    formats, within the documented limits; integer inputs, so everything is fixed to the bit."""
    c = _random_case(np.random.default_rng(4000 + seed))
    print(f"seed={seed} case={c}", flush=True)
    M, N, K, tp, rank, tile = c["M"], c["N"], c["K"], c["tp"], c["rank"], c["tile"]
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=5000 + seed)
    inc = inc * np.float32(33.0)
    sent = (np.full((tp - 1, M, N // tp), gpu.SENTINEL_BF16, np.uint16) if c["bf16"]
            else np.full((tp - 1, M, N // tp), gpu.SENTINEL, np.float32))
    want = oracle.fused_path(a, np.ascontiguousarray(b.T) if c["kn"] else b, inc, tp, rank, *tile,
                             b_layout=oracle.B_KN if c["kn"] else oracle.B_NK,
                             step0_store_only=c["step0"], fwd_direct=c["direct"],
                             fwd_bf16=c["bf16"], fwd_init=sent)
    flags = _flags(c["step0"], c["direct"]) | (t3.T3_FLAG_FWD_BF16 if c["bf16"] else 0)
    got = gpu.run_gpu(a, b, inc, tp, rank, tile, flags=flags, unfused=c["unfused"],
                      ldr_pad=c["ldr_pad"], lda_pad=c["lda_pad"], b_kn=c["kn"])
    assert np.array_equal(got["R"], want["R"]) and np.all(got["R_pad"] == 123.0)
    assert np.array_equal(got["fwd"], want["fwd"])
    _check_ints(got, want, tp, want["own"])


def test_default_tile_and_k_zero_and_empty(gpu, oracle):
    # K = 0: C is zero, the path degenerates to the partition of the incoming data
    M, N, tp, rank = 128, 512, 4, 1
    inc = np.arange(M * N, dtype=np.float32).reshape(M, N)
    a = np.zeros((M, 0), dtype=np.uint16)
    b = np.zeros((N, 0), dtype=np.uint16)
    a_pad, b_pad = np.zeros((M, 8), np.uint16), np.zeros((N, 8), np.uint16)
    import torch
    from tests.gpu_harness import to_dev_bits
    A, B = to_dev_bits(a_pad), to_dev_bits(b_pad)
    R = torch.from_numpy(inc).cuda()
    fwd = torch.zeros((tp - 1, M, N // tp), dtype=torch.float32, device="cuda")
    track = torch.zeros(t3.t3_track_words(tp), dtype=torch.int32, device="cuda")
    p = t3.problem(M, N, 0, tp, rank, lda=8, ldb=8)          # default tile
    t3.t3_track_reset(tp, track)
    t3.t3_gemm_rs_fused(p, A, B, R, fwd, track)
    torch.cuda.synchronize()
    want = oracle.fused_path(a, b, inc, tp, rank, *t3.t3_default_tile(p))
    assert np.array_equal(R.cpu().numpy(), want["R"])
    assert np.array_equal(fwd.cpu().numpy(), want["fwd"])
    # M = 0: nothing runs, tracker stays clear
    p0 = t3.problem(0, N, 64, tp, rank)
    t3.t3_track_reset(tp, track)
    t3.t3_gemm_rs_fused(p0, A, B, R, fwd, track)
    torch.cuda.synchronize()
    tr = t3.read_track(track, tp)
    assert np.all(tr["counter"] == 0) and np.all(tr["ready"] == 0) and tr["queue_len"] == 0
    assert tr["gen"] == 0


def test_integer_state_repeats(gpu, oracle):
    M, N, K, tp, rank, tile = 512, 2048, 64, 8, 6, (128, 128)
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=5)
    want = oracle.fused_path(a, b, inc, tp, rank, *tile)
    for _ in range(3):
        got = gpu.run_gpu(a, b, inc, tp, rank, tile)
        assert np.array_equal(got["R"], want["R"]) and np.array_equal(got["fwd"], want["fwd"])
        _check_ints(got, want, tp, want["own"])


# ---------------------------------------------------------------- full-size configurations
# The launch configuration bench.py times, every element against the oracle (the full fp64
# GEMM + reduction takes the host cores a few seconds per configuration; it is computed once
# per workload and shared by the two release modes).
FULL = ["gpt3_outproj", "gpt3_fc2", "wide_fc2", "hightp_outproj"]
_full_cache = {}


def _full_oracle(oracle, name):
    if name not in _full_cache:
        _full_cache.clear()                       # one workload's arrays at a time
        w = wl.WORKLOADS[name]
        a, b, inc = wl.make_inputs(w)
        _full_cache[name] = (a, b, inc, oracle.reduce_rows(oracle.gemm_rows(a, b), inc, w.tp))
    return _full_cache[name]


@pytest.mark.parametrize("direct", [True, False])
@pytest.mark.parametrize("name", FULL)
def test_full_size_every_element(gpu, oracle, name, direct):
    import torch
    w = wl.WORKLOADS[name]
    print(f"workload={name} direct={direct} tile={w.tile_m}x{w.tile_n}", flush=True)
    a, b, inc, S = _full_oracle(oracle, name)     # S: (M, N) fp32 sums

    dev = torch.device("cuda:0")
    A, B = gpu.to_dev_bits(a), gpu.to_dev_bits(b)
    R = torch.from_numpy(inc).to(dev)
    fwd = torch.full((w.tp - 1, w.M, w.W), gpu.SENTINEL, dtype=torch.float32, device=dev)
    track = torch.zeros(t3.t3_track_words(w.tp), dtype=torch.int32, device=dev)
    p = t3.problem(w.M, w.N, w.K, w.tp, w.rank, w.tile_m, w.tile_n,
                   flags=t3.T3_FLAG_FWD_DIRECT if direct else 0)
    t3.t3_track_reset(w.tp, track)
    t3.t3_gemm_rs_fused(p, A, B, R, fwd, track)
    torch.cuda.synchronize()

    order, own = oracle.chunk_order(w.tp, w.rank)
    tpc = oracle.tiles_per_chunk(w.M, w.N, w.tp, w.tile_m, w.tile_n)
    tr = t3.read_track(track, w.tp)
    assert np.all(tr["counter"] == tpc) and np.all(tr["ready"] == 1)
    assert tr["queue_len"] == w.tp - 1 and tr["error"] == 0 and tr["gen"] == 1
    assert sorted(tr["queue"][:w.tp - 1].tolist()) == sorted(c for c in range(w.tp) if c != own)

    Rg = R.cpu().numpy()
    fg = fwd.cpu().numpy()
    W = w.W
    scale = float(np.abs(S).max())
    errs, worst = [], 0.0
    for s in range(w.tp):
        c = int(order[s])
        cols = slice(c * W, (c + 1) * W)
        want = S[:, cols]
        got = Rg[:, cols] if c == own else fg[s]
        errs.append(gpu.rel_err(got, want))
        worst = max(worst, float(np.abs(got.astype(np.float64) - want).max()))
        if c != own:
            if direct:      # R keeps the incoming data on forwarded chunks
                assert np.array_equal(Rg[:, cols], inc[:, cols])
            else:           # the slot is a copy of what was reduced in place
                assert np.array_equal(Rg[:, cols], fg[s])
    print(f"max normwise error over chunks {max(errs):.3e}; max |diff| over all {w.M * w.N} "
          f"elements {worst:.3e} = {worst / scale:.2e} of the largest sum", flush=True)
    assert max(errs) <= TOL and max(errs) <= EXPECT
    assert worst <= 1e-4 * scale                  # element by element: no tile, row or block is off


@pytest.mark.parametrize("name", sorted(wl.PAPER_SHAPES))
def test_paper_table2_shapes_sampled_rows(gpu, oracle, name):
    """Sub-layer shapes of the paper's Table 2 models with the library's default tile, direct
    release: sampled rows against the oracle (ragged chunk widths, TP up to 32)."""
    import torch
    w = wl.WORKLOADS[name]
    a, b, inc = wl.make_inputs(w)
    p = t3.problem(w.M, w.N, w.K, w.tp, w.rank, flags=t3.T3_FLAG_FWD_DIRECT)
    tm, tn = t3.t3_default_tile(p)
    print(f"workload={name} default tile={tm}x{tn} W={w.W}", flush=True)
    rng = np.random.default_rng(w.seed)
    rows = np.array(sorted({0, w.M - 1} | set(rng.integers(0, w.M, 24).tolist())), dtype=np.int32)
    S = oracle.reduce_rows(oracle.gemm_rows(a, b, rows=rows), inc, w.tp, rows=rows)
    dev = torch.device("cuda:0")
    A, B = gpu.to_dev_bits(a), gpu.to_dev_bits(b)
    R = torch.from_numpy(inc).to(dev)
    fwd = torch.full((w.tp - 1, w.M, w.W), gpu.SENTINEL, dtype=torch.float32, device=dev)
    track = torch.zeros(t3.t3_track_words(w.tp), dtype=torch.int32, device=dev)
    t3.t3_track_reset(w.tp, track)
    t3.t3_gemm_rs_fused(p, A, B, R, fwd, track)
    torch.cuda.synchronize()
    order, own = oracle.chunk_order(w.tp, w.rank)
    tr = t3.read_track(track, w.tp)
    assert np.all(tr["counter"] == oracle.tiles_per_chunk(w.M, w.N, w.tp, tm, tn))
    assert np.all(tr["ready"] == 1) and tr["queue_len"] == w.tp - 1 and tr["error"] == 0
    idx = torch.from_numpy(rows.astype(np.int64)).to(dev)
    Rg = R.index_select(0, idx).cpu().numpy()
    fg = fwd.index_select(1, idx).cpu().numpy()
    W = w.W
    errs = []
    for s in range(w.tp):
        c = int(order[s])
        want = S[:, c * W:(c + 1) * W]
        errs.append(gpu.rel_err(Rg[:, c * W:(c + 1) * W] if c == own else fg[s], want))
    print(f"max normwise error over chunks {max(errs):.3e}", flush=True)
    assert max(errs) <= EXPECT
    assert not bool((fwd == gpu.SENTINEL).all(dim=2).any())


def test_full_size_b_stored_k_by_n(gpu, oracle):
    """gpt3_outproj at full size with B stored K x N, direct release: sampled rows."""
    import torch
    w = wl.WORKLOADS["gpt3_outproj"]
    a, b, inc = wl.make_inputs(w)
    rng = np.random.default_rng(w.seed + 1)
    rows = np.array(sorted({0, w.M - 1} | set(rng.integers(0, w.M, 16).tolist())), dtype=np.int32)
    S = oracle.reduce_rows(oracle.gemm_rows(a, b, rows=rows), inc, w.tp, rows=rows)
    dev = torch.device("cuda:0")
    A, B = gpu.to_dev_bits(a), gpu.to_dev_bits(np.ascontiguousarray(b.T))
    R = torch.from_numpy(inc).to(dev)
    fwd = torch.full((w.tp - 1, w.M, w.W), gpu.SENTINEL, dtype=torch.float32, device=dev)
    track = torch.zeros(t3.t3_track_words(w.tp), dtype=torch.int32, device=dev)
    p = t3.problem(w.M, w.N, w.K, w.tp, w.rank, w.tile_m, w.tile_n, b_layout=t3.T3_B_KN,
                   flags=t3.T3_FLAG_FWD_DIRECT)
    t3.t3_track_reset(w.tp, track)
    t3.t3_gemm_rs_fused(p, A, B, R, fwd, track)
    torch.cuda.synchronize()
    order, own = oracle.chunk_order(w.tp, w.rank)
    tr = t3.read_track(track, w.tp)
    assert np.all(tr["ready"] == 1) and tr["queue_len"] == w.tp - 1 and tr["error"] == 0
    idx = torch.from_numpy(rows.astype(np.int64)).to(dev)
    Rg = R.index_select(0, idx).cpu().numpy()
    fg = fwd.index_select(1, idx).cpu().numpy()
    W = w.W
    errs = [gpu.rel_err(Rg[:, c * W:(c + 1) * W] if c == own else fg[s], S[:, c * W:(c + 1) * W])
            for s, c in enumerate(int(x) for x in order)]
    print(f"max normwise error over chunks {max(errs):.3e}", flush=True)
    assert max(errs) <= EXPECT


@pytest.mark.parametrize("b_kn", [False, True])
def test_full_size_a_stored_k_by_m(gpu, oracle, b_kn):
    """gpt3_outproj at full size with A stored K x M (and B in either layout), direct release:
    every element against the oracle."""
    import torch
    w = wl.WORKLOADS["gpt3_outproj"]
    a, b, inc, S = _full_oracle(oracle, "gpt3_outproj")
    dev = torch.device("cuda:0")
    A = gpu.to_dev_bits(np.ascontiguousarray(a.T))
    B = gpu.to_dev_bits(np.ascontiguousarray(b.T) if b_kn else b)
    R = torch.from_numpy(inc).to(dev)
    fwd = torch.full((w.tp - 1, w.M, w.W), gpu.SENTINEL, dtype=torch.float32, device=dev)
    track = torch.zeros(t3.t3_track_words(w.tp), dtype=torch.int32, device=dev)
    p = t3.problem(w.M, w.N, w.K, w.tp, w.rank, w.tile_m, w.tile_n, a_layout=t3.T3_A_KM,
                   b_layout=t3.T3_B_KN if b_kn else t3.T3_B_NK, flags=t3.T3_FLAG_FWD_DIRECT)
    t3.t3_track_reset(w.tp, track)
    t3.t3_gemm_rs_fused(p, A, B, R, fwd, track)
    torch.cuda.synchronize()
    order, own = oracle.chunk_order(w.tp, w.rank)
    tr = t3.read_track(track, w.tp)
    assert np.all(tr["ready"] == 1) and tr["queue_len"] == w.tp - 1 and tr["error"] == 0
    Rg, fg, W = R.cpu().numpy(), fwd.cpu().numpy(), w.W
    scale = float(np.abs(S).max())
    for s_, c in enumerate(int(x) for x in order):
        got = Rg[:, c * W:(c + 1) * W] if c == own else fg[s_]
        want = S[:, c * W:(c + 1) * W]
        assert gpu.rel_err(got, want) <= EXPECT
        assert float(np.abs(got.astype(np.float64) - want).max()) <= 1e-4 * scale


@pytest.mark.parametrize("direct", [True, False])
def test_full_size_bf16_forward_slots(gpu, oracle, direct):
    """gpt3_outproj at full size with bfloat16 forward slots: sampled rows.  The slots hold the
    rounding of what the fp32 path would have forwarded: within one bfloat16 step of the oracle's
    rounding of its own sum, equal on nearly every element; the owned chunk stays fp32."""
    import torch
    w = wl.WORKLOADS["gpt3_outproj"]
    a, b, inc = wl.make_inputs(w)
    rng = np.random.default_rng(w.seed + 2)
    rows = np.array(sorted({0, w.M - 1} | set(rng.integers(0, w.M, 16).tolist())), dtype=np.int32)
    S = oracle.reduce_rows(oracle.gemm_rows(a, b, rows=rows), inc, w.tp, rows=rows)
    dev = torch.device("cuda:0")
    A, B = gpu.to_dev_bits(a), gpu.to_dev_bits(b)
    R = torch.from_numpy(inc).to(dev)
    fwd = torch.full((w.tp - 1, w.M, w.W), gpu.SENTINEL_BF16 - 65536, dtype=torch.int16, device=dev)
    track = torch.zeros(t3.t3_track_words(w.tp), dtype=torch.int32, device=dev)
    p = t3.problem(w.M, w.N, w.K, w.tp, w.rank, w.tile_m, w.tile_n,
                   flags=t3.T3_FLAG_FWD_BF16 | (t3.T3_FLAG_FWD_DIRECT if direct else 0))
    t3.t3_track_reset(w.tp, track)
    t3.t3_gemm_rs_fused(p, A, B, R, fwd, track)
    torch.cuda.synchronize()
    order, own = oracle.chunk_order(w.tp, w.rank)
    tr = t3.read_track(track, w.tp)
    assert np.all(tr["ready"] == 1) and tr["queue_len"] == w.tp - 1 and tr["error"] == 0
    idx = torch.from_numpy(rows.astype(np.int64)).to(dev)
    Rg = R.index_select(0, idx).cpu().numpy()
    fg = fwd.index_select(1, idx).cpu().numpy().view(np.uint16)
    W = w.W
    same = []
    for s, c in enumerate(int(x) for x in order):
        want = S[:, c * W:(c + 1) * W]
        if c == own:
            assert gpu.rel_err(Rg[:, c * W:(c + 1) * W], want) <= EXPECT
            continue
        bits = oracle.to_bf16_bits(want)
        got = fg[s]
        same.append(np.mean(got == bits))
        x = oracle.from_bf16_bits(bits).astype(np.float64)
        assert np.all(np.abs(oracle.from_bf16_bits(got) - x) <= np.abs(x) * 2.0 ** -7 + 1e-4 * np.abs(x).max())
        assert gpu.rel_err(oracle.from_bf16_bits(got), want) <= EXPECT + 2.0 ** -9
    print(f"direct={direct}: fraction of identical bfloat16 values per slot {min(same):.5f}..{max(same):.5f}",
          flush=True)
    assert min(same) > 0.99
    assert not bool((fwd == gpu.SENTINEL_BF16 - 65536).all(dim=2).any())


@pytest.mark.parametrize("flags", [0, 2, 3])
def test_plain_c_client_of_the_abi(gpu, flags):
    """tests/c_abi_client.c: a C11 program that includes include/t3.h, links the library and the
    HIP runtime, and checks every output word itself.  Run as a child process."""
    import subprocess
    from paper_2401_16677_amd import build as hip_build
    exe = hip_build.build_c_client(force=False)
    r = subprocess.run([exe, str(flags)], capture_output=True, text=True, timeout=100)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0 and " 0 mismatches" in r.stdout


def test_largest_supported_buffers(gpu, oracle):
    """R, C and the forward slot just below the documented 4 GiB limit (the kernels address them
    with 32-bit byte offsets): M = 32768, N = 32760, so the last element sits at byte offset
    4,293,918,716.  Integer inputs given by a formula; rows sampled from both ends and the
    middle are compared bit for bit, fused and unfused, and the size one step further is refused."""
    import torch
    M, N, K, tp, rank, tile = 32768, 32760, 64, 2, 1, (256, 256)
    assert M * N * 4 < 2 ** 32 < (M + 16) * N * 4
    W = N // tp
    a = wl.make_integer_inputs(M, 8, K, seed=1700)[0]          # (the generator's own incoming
    b = wl.make_integer_inputs(8, N, K, seed=1701)[1]          # array would be 4 GiB: not drawn)
    rows = np.array([0, 1, 255, 256, 16383, 16384, 21000, 32511, 32512, 32766, 32767], dtype=np.int64)
    cols = np.arange(N, dtype=np.int64)
    inc_rows = ((rows[:, None] * 131 + cols[None, :] * 7) % 2001 - 1000).astype(np.float32)
    S = oracle.reduce_rows(oracle.gemm_rows(a, b, rows=rows.astype(np.int32)), inc_rows, tp)
    dev = torch.device("cuda:0")

    def fresh_R():
        r = torch.arange(M, dtype=torch.int32, device=dev)[:, None] * 131
        r = r + torch.arange(N, dtype=torch.int32, device=dev)[None, :] * 7
        return (r.remainder_(2001) - 1000).to(torch.float32)

    A, B = gpu.to_dev_bits(a), gpu.to_dev_bits(b)
    fwd = torch.full((tp - 1, M, W), gpu.SENTINEL, dtype=torch.float32, device=dev)
    track = torch.zeros(t3.t3_track_words(tp), dtype=torch.int32, device=dev)
    p = t3.problem(M, N, K, tp, rank, *tile, flags=t3.T3_FLAG_FWD_DIRECT)
    order, own = oracle.chunk_order(tp, rank)
    idx = torch.from_numpy(rows).to(dev)
    t3.t3_track_reset(tp, track)
    for unfused in (False, True):
        print(f"unfused={unfused}", flush=True)
        R = fresh_R()
        fwd.fill_(gpu.SENTINEL)
        if unfused:
            C = torch.empty((M, N), dtype=torch.float32, device=dev)
            t3.t3_gemm(p, A, B, C)
            t3.t3_rs_reduce(p, C, R, fwd, track)
        else:
            t3.t3_gemm_rs_fused(p, A, B, R, fwd, track)
        torch.cuda.synchronize()
        tr = t3.read_track(track, tp)
        assert np.all(tr["ready"] == 1) and tr["error"] == 0 and tr["queue_len"] == tp - 1
        Rg = R.index_select(0, idx).cpu().numpy()
        fg = fwd.index_select(1, idx).cpu().numpy()
        for s_, c in enumerate(int(x) for x in order):
            want = S[:, c * W:(c + 1) * W]
            if c == own:
                assert np.array_equal(Rg[:, c * W:(c + 1) * W], want)
            else:
                assert np.array_equal(fg[s_], want)
                assert np.array_equal(Rg[:, c * W:(c + 1) * W], inc_rows[:, c * W:(c + 1) * W])
        assert not bool((fwd == gpu.SENTINEL).all(dim=2).any())
        del R
        if unfused:
            del C
    too_big = t3.problem(M + 16, N, K, tp, rank, *tile, flags=t3.T3_FLAG_FWD_DIRECT)
    with pytest.raises(RuntimeError):
        t3.t3_gemm_rs_fused(too_big, A, B, fwd, fwd, track)      # refused before any launch


def test_largest_supported_operand(gpu, oracle):
    """A just below the documented 2^31-element limit (the kernels address A and B with 32-bit
    offsets): M = 32768 rows of K = lda = 65528 (1023 K-slabs and a tail of 56).  Integer inputs,
    A given by a formula; sampled rows bit for bit."""
    import torch
    M, N, K, tp, rank, tile = 32768, 256, 65528, 2, 0, (256, 128)
    assert M * K < 2 ** 31 < (M + 8) * K
    W = N // tp
    b = wl.make_integer_inputs(8, N, K, seed=1800, amax=1)[1]
    rows = np.array([0, 255, 256, 16384, 32767], dtype=np.int64)
    a_rows = ((rows[:, None] * 7 + np.arange(K, dtype=np.int64)[None, :] * 13) % 3 - 1).astype(np.float32)
    inc_rows = ((rows[:, None] * 5 + np.arange(N, dtype=np.int64)[None, :] * 3) % 201 - 100).astype(np.float32)
    S = oracle.reduce_rows(oracle.gemm_rows(wl.f32_to_bf16_bits(a_rows), b), inc_rows, tp)
    dev = torch.device("cuda:0")
    am = torch.arange(M, dtype=torch.int32, device=dev)[:, None] * 7
    am = (am + torch.arange(K, dtype=torch.int32, device=dev)[None, :] * 13).remainder_(3) - 1
    A = am.to(torch.float32).to(torch.bfloat16)
    del am
    B = gpu.to_dev_bits(b)
    r = torch.arange(M, dtype=torch.int32, device=dev)[:, None] * 5
    R = ((r + torch.arange(N, dtype=torch.int32, device=dev)[None, :] * 3).remainder_(201) - 100).to(torch.float32)
    fwd = torch.full((tp - 1, M, W), gpu.SENTINEL, dtype=torch.float32, device=dev)
    track = torch.zeros(t3.t3_track_words(tp), dtype=torch.int32, device=dev)
    p = t3.problem(M, N, K, tp, rank, *tile, flags=t3.T3_FLAG_FWD_DIRECT)
    t3.t3_track_reset(tp, track)
    t3.t3_gemm_rs_fused(p, A, B, R, fwd, track)
    torch.cuda.synchronize()
    tr = t3.read_track(track, tp)
    assert np.all(tr["ready"] == 1) and tr["error"] == 0
    order, own = oracle.chunk_order(tp, rank)
    idx = torch.from_numpy(rows).to(dev)
    Rg = R.index_select(0, idx).cpu().numpy()
    fg = fwd.index_select(1, idx).cpu().numpy()
    for s_, c in enumerate(int(x) for x in order):
        got = Rg[:, c * W:(c + 1) * W] if c == own else fg[s_]
        assert np.array_equal(got, S[:, c * W:(c + 1) * W])
    with pytest.raises(RuntimeError):      # one step further is refused before any launch
        t3.t3_gemm_rs_fused(t3.problem(M + 8, N, K, tp, rank, *tile, flags=t3.T3_FLAG_FWD_DIRECT),
                            A, B, R, fwd, track)


def test_graph_replays_match_eager(gpu, oracle):
    """The step bench.py times (tracker reset + fused call) captured in a HIP graph: every
    replay, with eager work and synchronisation in between, must reproduce the eager result."""
    import torch
    M, N, K, tp, rank, tile = 512, 2048, 192, 4, 1, (256, 256)
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=77)
    want = oracle.fused_path(a, b, inc, tp, rank, *tile, fwd_direct=True,
                             fwd_init=np.zeros((tp - 1, M, N // tp), np.float32))
    dev = torch.device("cuda:0")
    A, B = gpu.to_dev_bits(a), gpu.to_dev_bits(b)
    inc_dev = torch.from_numpy(inc).to(dev)
    R = inc_dev.clone()
    fwd = torch.zeros((tp - 1, M, N // tp), dtype=torch.float32, device=dev)
    track = torch.zeros(t3.t3_track_words(tp), dtype=torch.int32, device=dev)
    p = t3.problem(M, N, K, tp, rank, *tile, flags=t3.T3_FLAG_FWD_DIRECT)

    def step():
        t3.t3_track_reset(tp, track)
        t3.t3_gemm_rs_fused(p, A, B, R, fwd, track)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        step()
    for rep in range(4):
        R.copy_(inc_dev)                 # eager work between replays
        fwd.zero_()
        track.fill_(0x5A5A5A5A)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        own = want["own"]
        W = N // tp
        assert np.array_equal(fwd.cpu().numpy(), want["fwd"]), rep
        assert np.array_equal(R.cpu().numpy()[:, own * W:(own + 1) * W], want["owned"]), rep
        tr = t3.read_track(track, tp)
        assert np.array_equal(tr["counter"], want["counter"]) and tr["queue_len"] == tp - 1, rep
        assert tr["gen"] == 1, rep


def test_consecutive_launches_need_no_reset(gpu, oracle):
    """One reset, then several launches on the same tracker state: each finds a clean bank and
    leaves its own results behind; gen counts the launches (also partial ones)."""
    import torch
    M, N, K, tp, rank, tile = 384, 1536, 64, 3, 2, (128, 128)
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=91)
    dev = torch.device("cuda:0")
    A, B = gpu.to_dev_bits(a), gpu.to_dev_bits(b)
    inc_dev = torch.from_numpy(inc).to(dev)
    R = inc_dev.clone()
    W = N // tp
    fwd = torch.zeros((tp - 1, M, W), dtype=torch.float32, device=dev)
    track = torch.full((t3.t3_track_words(tp),), 0x5A5A5A5A, dtype=torch.int32, device=dev)
    t3.t3_track_reset(tp, track)
    tpc = oracle.tiles_per_chunk(M, N, tp, *tile)
    launches = [(-1, 0), (tpc + 3, 0), (-1, t3.T3_FLAG_FWD_DIRECT), (-1, 0), (2 * tpc, 0)]
    for n, (limit, flags) in enumerate(launches, start=1):
        R.copy_(inc_dev)
        fwd.fill_(gpu.SENTINEL)
        p = t3.problem(M, N, K, tp, rank, *tile, tile_limit=limit, flags=flags)
        t3.t3_gemm_rs_fused(p, A, B, R, fwd, track)
        torch.cuda.synchronize()
        want = oracle.fused_path(a, b, inc, tp, rank, *tile, tile_limit=limit,
                                 fwd_direct=bool(flags & t3.T3_FLAG_FWD_DIRECT),
                                 fwd_init=np.full((tp - 1, M, W), gpu.SENTINEL, np.float32))
        tr = t3.read_track(track, tp)
        print(f"launch {n}: limit={limit} flags={flags} gen={tr['gen']}", flush=True)
        assert tr["gen"] == n and tr["error"] == 0
        assert np.array_equal(tr["counter"], want["counter"])
        assert np.array_equal(tr["ready"], want["ready"])
        assert tr["queue_len"] == want["queue_len"]
        assert set(tr["queue"][:tr["queue_len"]].tolist()) == set(want["queue"][:want["queue_len"]].tolist())
        assert np.array_equal(R.cpu().numpy(), want["R"])
        assert np.array_equal(fwd.cpu().numpy(), want["fwd"])

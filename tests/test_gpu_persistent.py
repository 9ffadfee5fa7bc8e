"""GPU parity of the launch shape the benchmark times: persistent workgroups that each walk
three or more tiles (LDS reused from tile to tile, the count of a tile deferred into the next
tile's main loop), every element compared with the CPU oracle.

Small-integer inputs make fp32 accumulation exact in any order, so R, the forward slots and C
must equal the fp64 oracle bit for bit; the shapes have at least three tiles per resident
workgroup for each of the four tile shapes (256 compute units hold 256 workgroups, 512 of the
128 x 128 tile), a ragged last tile row and a K that ends in a partial slab."""
import numpy as np
import pytest

from paper_2401_16677_amd import binding as t3
from paper_2401_16677_amd import workloads as wl

pytestmark = pytest.mark.gpu

CUS = 256      # compute units of the device these shapes are sized for

# M, N, K, tp, rank, tile: tiles = ceil(M/tm) * ceil(N/tp/tn) * tp
MULTI = {
    (256, 256): (4090, 12288, 136, 8, 3),     # 16 x 6 x 8 = 768 tiles = 3 per workgroup
    (256, 128): (4090, 8192, 136, 8, 5),      # 16 x 8 x 8 = 1024 = 4
    (128, 256): (2040, 12288, 136, 8, 7),     # 16 x 6 x 8 = 768 = 3
    (128, 128): (2040, 12288, 136, 8, 0),     # 16 x 12 x 8 = 1536 = 3 (two workgroups per unit)
}


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "needs a GPU"
    from tests import gpu_harness
    return gpu_harness


def _tiles_per_workgroup(M, N, tp, tile):
    resident = CUS * (2 if tile == (128, 128) else 1)
    return (-(-M // tile[0])) * (-(-(N // tp) // tile[1])) * tp / resident


def _check_ints(got, want, own):
    assert np.array_equal(got["counter"], want["counter"])
    assert np.array_equal(got["ready"], want["ready"])
    n = want["queue_len"]
    assert got["queue_len"] == n
    assert set(got["queue"][:n].tolist()) == set(want["queue"][:n].tolist())
    assert len(set(got["queue"][:n].tolist())) == n and own not in got["queue"][:n]
    assert np.all(got["queue"][n:] == 0xFFFFFFFF)
    assert got["error"] == 0


def _first_mismatch(got, want):
    bad = np.argwhere(got != want)
    return "equal" if bad.size == 0 else f"{bad.shape[0]} mismatches, first at {tuple(bad[0])}"


@pytest.mark.parametrize("mode", ["fused_direct", "fused_copy", "unfused_direct", "fused_direct_step0"])
@pytest.mark.parametrize("tile", sorted(MULTI))
def test_three_tiles_per_workgroup_every_element(gpu, oracle, tile, mode):
    M, N, K, tp, rank = MULTI[tile]
    assert _tiles_per_workgroup(M, N, tp, tile) >= 3
    direct = "direct" in mode
    step0 = mode.endswith("step0")
    print(f"tile={tile} shape={(M, N, K, tp, rank)} mode={mode}", flush=True)
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=900 + tile[0] + tile[1] // 2)
    want = oracle.fused_path(a, b, inc, tp, rank, *tile, fwd_direct=direct, step0_store_only=step0,
                             fwd_init=np.full((tp - 1, M, N // tp), gpu.SENTINEL, np.float32))
    flags = (t3.T3_FLAG_FWD_DIRECT if direct else 0) | (t3.T3_FLAG_STEP0_STORE_ONLY if step0 else 0)
    got = gpu.run_gpu(a, b, inc, tp, rank, tile, flags=flags, unfused=mode.startswith("unfused"),
                      ldr_pad=4, lda_pad=8)
    assert np.array_equal(got["R"], want["R"]), _first_mismatch(got["R"], want["R"])
    assert np.array_equal(got["fwd"], want["fwd"]), _first_mismatch(got["fwd"], want["fwd"])
    assert np.all(got["R_pad"] == 123.0)
    if mode.startswith("unfused"):
        assert np.array_equal(got["C"], oracle.gemm_rows(a, b).astype(np.float32))
    _check_ints(got, want, want["own"])


@pytest.mark.parametrize("tile", [(256, 256), (128, 128)])
def test_three_tiles_per_workgroup_b_stored_k_by_n(gpu, oracle, tile):
    M, N, _, tp, rank = MULTI[tile]
    K = 192                                   # whole slabs only in this layout
    print(f"tile={tile} shape={(M, N, K, tp, rank)} B stored K x N", flush=True)
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=940 + tile[0])
    want = oracle.fused_path(a, np.ascontiguousarray(b.T), inc, tp, rank, *tile, b_layout=oracle.B_KN,
                             fwd_direct=True,
                             fwd_init=np.full((tp - 1, M, N // tp), gpu.SENTINEL, np.float32))
    got = gpu.run_gpu(a, b, inc, tp, rank, tile, flags=t3.T3_FLAG_FWD_DIRECT, b_kn=True, lda_pad=8)
    assert np.array_equal(got["R"], want["R"]), _first_mismatch(got["R"], want["R"])
    assert np.array_equal(got["fwd"], want["fwd"]), _first_mismatch(got["fwd"], want["fwd"])
    _check_ints(got, want, want["own"])


@pytest.mark.parametrize("direct", [True, False])
@pytest.mark.parametrize("tile", [(256, 256), (256, 128)])
def test_three_tiles_per_workgroup_bf16_slots(gpu, oracle, tile, direct):
    M, N, K, tp, rank = MULTI[tile]
    print(f"tile={tile} shape={(M, N, K, tp, rank)} bfloat16 forward slots direct={direct}", flush=True)
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=960 + tile[1])
    want = oracle.fused_path(a, b, inc, tp, rank, *tile, fwd_direct=direct, fwd_bf16=True,
                             fwd_init=np.full((tp - 1, M, N // tp), gpu.SENTINEL_BF16, np.uint16))
    got = gpu.run_gpu(a, b, inc, tp, rank, tile,
                      flags=t3.T3_FLAG_FWD_BF16 | (t3.T3_FLAG_FWD_DIRECT if direct else 0))
    assert np.array_equal(got["R"], want["R"]), _first_mismatch(got["R"], want["R"])
    assert np.array_equal(got["fwd"], want["fwd"]), _first_mismatch(got["fwd"], want["fwd"])
    _check_ints(got, want, want["own"])


@pytest.mark.parametrize("unfused", [False, True])
@pytest.mark.parametrize("tile", [(256, 256), (128, 256)])
def test_tile_range_cutting_a_persistent_wave(gpu, oracle, tile, unfused):
    """A range of the issue order that starts inside the first wave of workgroups and ends inside
    the third: workgroups find their first and last grid positions outside the range, chunks at
    both ends stay incomplete."""
    M, N, K, tp, rank = MULTI[tile]
    tpc = oracle.tiles_per_chunk(M, N, tp, *tile)
    begin, limit = 100, 2 * CUS + 77
    assert 0 < begin < CUS and 2 * CUS < limit < 3 * CUS and limit % tpc and begin % tpc
    print(f"tile={tile} range=[{begin},{limit}) of {tp * tpc} unfused={unfused}", flush=True)
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=980 + tile[0])
    sent = np.full((tp - 1, M, N // tp), gpu.SENTINEL, np.float32)
    want = oracle.fused_path(a, b, inc, tp, rank, *tile, tile_begin=begin, tile_limit=limit,
                             fwd_direct=True, fwd_init=sent)
    got = gpu.run_gpu(a, b, inc, tp, rank, tile, flags=t3.T3_FLAG_FWD_DIRECT, tile_begin=begin,
                      tile_limit=limit, unfused=unfused)
    assert np.array_equal(got["R"], want["R"]), _first_mismatch(got["R"], want["R"])
    assert np.array_equal(got["fwd"], want["fwd"]), _first_mismatch(got["fwd"], want["fwd"])
    _check_ints(got, want, want["own"])


@pytest.mark.parametrize("tile", [(256, 256), (128, 128)])
def test_three_tiles_per_workgroup_float_every_element(gpu, oracle, tile):
    """The same launch shape on normally distributed inputs: every element within 1e-4 of the
    largest sum (fp32 accumulation of K = 136 products), and the norm far inside the 5e-3 bound."""
    M, N, K, tp, rank = MULTI[tile]
    w = wl.make_shape("multi", M, N, K, tp, rank, *tile, index=70 + tile[0] // 128)
    a, b, inc = wl.make_inputs(w)
    want = oracle.fused_path(a, b, inc, tp, rank, *tile, fwd_direct=True,
                             fwd_init=np.full((tp - 1, M, N // tp), gpu.SENTINEL, np.float32))
    got = gpu.run_gpu(a, b, inc, tp, rank, tile, flags=t3.T3_FLAG_FWD_DIRECT)
    scale = float(np.abs(want["fwd"]).max())
    for name in ("R", "fwd"):
        d = np.abs(got[name].astype(np.float64) - want[name])
        print(f"tile={tile} {name}: max |diff| {d.max():.3e} (scale {scale:.3e}), "
              f"normwise {gpu.rel_err(got[name], want[name]):.3e}", flush=True)
        assert d.max() <= 1e-4 * scale
        assert gpu.rel_err(got[name], want[name]) <= 1e-5
    _check_ints(got, want, want["own"])


@pytest.mark.parametrize("unfused", [False, True])
@pytest.mark.parametrize("direct", [True, False])
@pytest.mark.parametrize("rng_kind", ["all", "step1", "steps12", "cut"])
def test_tracked_tiles_of_128_rows_computed_in_pairs(gpu, oracle, rng_kind, direct, unfused):
    """128 x 256 tracked tiles: over ranges of whole ring steps the tile kernel computes two of
    them as one 256 x 256 workgroup tile and counts both (the last tile row, here the 19th of a
    column, stands alone); a range that cuts a step falls back to one workgroup per tracked
    tile.  Counters, flags, queue and every element must not care."""
    M, N, K, tp, rank, tile = 2330, 3 * 1304, 200, 3, 1, (128, 256)
    tpc = oracle.tiles_per_chunk(M, N, tp, *tile)
    assert tpc == 19 * 6
    begin, limit = {"all": (0, -1), "step1": (tpc, 2 * tpc), "steps12": (tpc, 3 * tpc),
                    "cut": (tpc + 1, 2 * tpc + 7)}[rng_kind]
    print(f"range=[{begin},{limit}) of {tp * tpc} direct={direct} unfused={unfused}", flush=True)
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=1234)
    sent = np.full((tp - 1, M, N // tp), gpu.SENTINEL, np.float32)
    want = oracle.fused_path(a, b, inc, tp, rank, *tile, tile_begin=begin, tile_limit=limit,
                             fwd_direct=direct, fwd_init=sent)
    got = gpu.run_gpu(a, b, inc, tp, rank, tile, flags=t3.T3_FLAG_FWD_DIRECT if direct else 0,
                      tile_begin=begin, tile_limit=limit, unfused=unfused, ldr_pad=8)
    assert np.array_equal(got["R"], want["R"]), _first_mismatch(got["R"], want["R"])
    assert np.array_equal(got["fwd"], want["fwd"]), _first_mismatch(got["fwd"], want["fwd"])
    _check_ints(got, want, want["own"])


def test_incoming_partial_survives_a_busy_lds_queue(gpu, oracle):
    """The 128 x 128 tile runs two workgroups per compute unit, so the LDS unit is busy while a
    workgroup turns its incoming partial into the accumulator layout in the stage that the main
    loop refills next; those LDS accesses must be complete before the refill is requested.  The
    launch is repeated: what is checked depends on timing."""
    tile, (M, N, K, tp, rank) = (128, 128), (2040, 9728, 520, 4, 3)
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=77)
    want = oracle.fused_path(a, b, inc, tp, rank, *tile, fwd_direct=True,
                             fwd_init=np.full((tp - 1, M, N // tp), gpu.SENTINEL, np.float32))
    for rep in range(12):
        print(f"tile={tile} shape={(M, N, K, tp, rank)} repetition {rep}", flush=True)
        got = gpu.run_gpu(a, b, inc, tp, rank, tile, flags=t3.T3_FLAG_FWD_DIRECT, ldr_pad=4, lda_pad=8)
        assert np.array_equal(got["R"], want["R"]), _first_mismatch(got["R"], want["R"])
        assert np.array_equal(got["fwd"], want["fwd"]), _first_mismatch(got["fwd"], want["fwd"])
    _check_ints(got, want, want["own"])


# Balanced tail: the tiles do not fill a whole number of rounds of the resident workgroups and
# the last round would fill at most half of them, so each of its tiles is computed as two
# halves of K by two workgroups, the partial sums passing through the tile's destination.
# M, N, K, tp, rank: tiles = q * resident + r, 0 < r <= resident / 2; K has a ragged last slab.
TAIL = {
    (256, 256): (2040, 20480, 520, 5, 2),     # 8 x 16 x 5 = 640 = 2 x 256 + 128
    (256, 128): (2040, 10240, 584, 5, 4),     # 8 x 16 x 5 = 640
    (128, 256): (2040, 20480, 520, 5, 0),     # computed in pairs: 8 x 16 x 5 = 640 workgroup tiles
    (128, 128): (2040, 9728, 520, 4, 3),      # 16 x 19 x 4 = 1216 = 2 x 512 + 192
}


def _workgroup_tiles(M, N, tp, tile):
    tm = 256 if tile == (128, 256) else tile[0]
    return (-(-M // tm)) * (-(-(N // tp) // tile[1])) * tp


@pytest.mark.parametrize("mode", ["fused_direct", "unfused_direct", "fused_direct_step0"])
@pytest.mark.parametrize("tile", sorted(TAIL))
def test_balanced_tail_every_element(gpu, oracle, tile, mode):
    M, N, K, tp, rank = TAIL[tile]
    resident = CUS * (2 if tile == (128, 128) else 1)
    T = _workgroup_tiles(M, N, tp, tile)
    assert T > resident and 0 < T % resident <= resident // 2 and K // 64 >= 8
    step0 = mode.endswith("step0")
    print(f"tile={tile} shape={(M, N, K, tp, rank)} mode={mode} tiles={T}", flush=True)
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=1300 + tile[0] + tile[1] // 2)
    want = oracle.fused_path(a, b, inc, tp, rank, *tile, fwd_direct=True, step0_store_only=step0,
                             fwd_init=np.full((tp - 1, M, N // tp), gpu.SENTINEL, np.float32))
    flags = t3.T3_FLAG_FWD_DIRECT | (t3.T3_FLAG_STEP0_STORE_ONLY if step0 else 0)
    # two launches before the one that is checked: the flags of the split tiles must be back
    # to zero after every launch
    got = gpu.run_gpu(a, b, inc, tp, rank, tile, flags=flags, unfused=mode.startswith("unfused"),
                      ldr_pad=4, lda_pad=8, launches_before=2)
    assert np.array_equal(got["R"], want["R"]), _first_mismatch(got["R"], want["R"])
    assert np.array_equal(got["fwd"], want["fwd"]), _first_mismatch(got["fwd"], want["fwd"])
    assert np.all(got["R_pad"] == 123.0)
    if mode.startswith("unfused"):
        assert np.array_equal(got["C"], oracle.gemm_rows(a, b).astype(np.float32))
    _check_ints(got, want, want["own"])


def test_balanced_tail_of_one_tile(gpu, oracle):
    """513 tiles on 256 workgroups: one tile is split between two workgroups."""
    tile, (M, N, K, tp, rank) = (256, 256), (6900, 4864, 520, 19, 7)
    assert _workgroup_tiles(M, N, tp, tile) == 2 * CUS + 1
    print(f"tile={tile} shape={(M, N, K, tp, rank)}", flush=True)
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=1500)
    want = oracle.fused_path(a, b, inc, tp, rank, *tile, fwd_direct=True,
                             fwd_init=np.full((tp - 1, M, N // tp), gpu.SENTINEL, np.float32))
    got = gpu.run_gpu(a, b, inc, tp, rank, tile, flags=t3.T3_FLAG_FWD_DIRECT, launches_before=1)
    assert np.array_equal(got["R"], want["R"]), _first_mismatch(got["R"], want["R"])
    assert np.array_equal(got["fwd"], want["fwd"]), _first_mismatch(got["fwd"], want["fwd"])
    _check_ints(got, want, want["own"])


def test_balanced_tail_float_every_element(gpu, oracle):
    """Normally distributed inputs through a split tile: the two halves of K are summed in fp32
    one after the other, as the unsplit K loop does."""
    tile = (256, 256)
    M, N, K, tp, rank = TAIL[tile]
    w = wl.make_shape("tail", M, N, K, tp, rank, *tile, index=77)
    a, b, inc = wl.make_inputs(w)
    want = oracle.fused_path(a, b, inc, tp, rank, *tile, fwd_direct=True,
                             fwd_init=np.full((tp - 1, M, N // tp), gpu.SENTINEL, np.float32))
    got = gpu.run_gpu(a, b, inc, tp, rank, tile, flags=t3.T3_FLAG_FWD_DIRECT)
    scale = float(np.abs(want["fwd"]).max())
    for name in ("R", "fwd"):
        d = np.abs(got[name].astype(np.float64) - want[name])
        print(f"{name}: max |diff| {d.max():.3e} (scale {scale:.3e}), normwise {gpu.rel_err(got[name], want[name]):.3e}",
              flush=True)
        assert d.max() <= 1e-4 * scale
        assert gpu.rel_err(got[name], want[name]) <= 1e-5
    _check_ints(got, want, want["own"])


def test_ready_flag_publishes_a_chunk_while_the_launch_runs(gpu):
    """The publication contract of the tracker in the persistent direct mode: once ready[c] has
    been observed, chunk c's forward slot holds its final contents, although the launch that
    produces the other chunks is still running.  The host watches the tracker from a second
    stream while a long launch runs; whenever a chunk has become ready its slot is copied aside
    (device to device, behind the observation), and afterwards every copy must equal the slot
    as the finished launch left it."""
    import torch
    M, N, K, tp, rank, tile = 4096, 12288, 16384, 8, 3, (256, 256)
    W = N // tp
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(5)
    A = (torch.randn((M, K), device=dev, generator=g) * K ** -0.25).to(torch.bfloat16)
    B = (torch.randn((N, K), device=dev, generator=g) * K ** -0.25).to(torch.bfloat16)
    R = torch.randn((M, N), device=dev, generator=g)
    words = t3.t3_track_words(tp)
    p = t3.problem(M, N, K, tp, rank, *tile, flags=t3.T3_FLAG_FWD_DIRECT)
    main, side = torch.cuda.Stream(), torch.cuda.Stream()
    host = torch.zeros(words, dtype=torch.int32).pin_memory()
    order = [(rank + s) % tp for s in range(tp)]
    seen_early = 0
    for attempt in range(3):
        fwd = torch.full((tp - 1, M, W), gpu.SENTINEL, dtype=torch.float32, device=dev)
        snap = torch.zeros_like(fwd)
        track = torch.zeros(words, dtype=torch.int32, device=dev)
        t3.t3_track_reset(tp, track)
        torch.cuda.synchronize()
        done = torch.cuda.Event()
        t3.t3_gemm_rs_fused(p, A, B, R.clone(), fwd, track, stream=main)
        done.record(main)
        taken, early = set(), set()
        for _ in range(20000):
            finished = done.query()                 # before the observation: "early" is certain
            with torch.cuda.stream(side):
                host.copy_(track, non_blocking=True)
            side.synchronize()
            ready = host[tp:2 * tp].tolist()        # bank 0: the launch after a reset works there
            for s in range(tp - 1):
                if ready[order[s]] == 1 and s not in taken:
                    with torch.cuda.stream(side):
                        snap[s].copy_(fwd[s], non_blocking=True)
                    taken.add(s)
                    if not finished:
                        early.add(s)
            if finished:
                break
        torch.cuda.synchronize()
        tr = t3.read_track(track, tp)
        assert tr["error"] == 0 and tr["queue_len"] == tp - 1
        print(f"attempt {attempt}: slots copied {sorted(taken)}, of them while the launch ran {sorted(early)}",
              flush=True)
        for s in sorted(taken):
            assert torch.equal(snap[s], fwd[s]), f"slot {s} changed after its chunk was announced ready"
        assert not bool((fwd == gpu.SENTINEL).all(dim=(1, 2)).any())
        seen_early = max(seen_early, len(early))
        if seen_early:
            break
    assert seen_early >= 1, "the host never caught a chunk ready before the launch ended"


def test_timeline_records_every_piece_and_changes_nothing(gpu, oracle):
    """t3_timeline: with recording on, every workgroup leaves four non-decreasing clock readings
    per piece of work (here 3 tiles per workgroup), the results are what they are without it,
    and after switching it off nothing more is written."""
    import torch
    tile = (256, 256)
    M, N, K, tp, rank = MULTI[tile]
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=1600)
    want = oracle.fused_path(a, b, inc, tp, rank, *tile, fwd_direct=True,
                             fwd_init=np.full((tp - 1, M, N // tp), gpu.SENTINEL, np.float32))
    items = t3.T3_TIMELINE_ITEMS
    st = torch.zeros(CUS * items * 4, dtype=torch.int64, device="cuda:0")
    t3.t3_timeline(st)
    try:
        got = gpu.run_gpu(a, b, inc, tp, rank, tile, flags=t3.T3_FLAG_FWD_DIRECT)
    finally:
        t3.t3_timeline(None)
    assert np.array_equal(got["R"], want["R"]) and np.array_equal(got["fwd"], want["fwd"])
    _check_ints(got, want, want["own"])
    s = st.cpu().numpy().reshape(CUS, items, 4)
    pieces = (s[:, :, 0] > 0).sum(axis=1)
    assert np.all(pieces == 3), pieces                       # 768 tiles on 256 workgroups
    rec = s[:, :3, :]
    assert np.all(rec > 0) and np.all(np.diff(rec, axis=2) >= 0)
    assert np.all(rec[:, 1:, 0] >= rec[:, :-1, 3])           # a piece starts after the one before it
    assert np.all(s[:, 3:, :] == 0)
    before = st.clone()
    got = gpu.run_gpu(a, b, inc, tp, rank, tile, flags=t3.T3_FLAG_FWD_DIRECT)
    assert torch.equal(st, before)
    assert np.array_equal(got["fwd"], want["fwd"])


@pytest.mark.parametrize("unfused", [False, True])
def test_balanced_tail_in_a_captured_graph(gpu, oracle, unfused):
    """A problem with a balanced tail captured in a HIP graph and replayed: the fused call keeps
    the flags between the halves of a tile in the tracker state, which the graph carries; the
    plain GEMM of the unfused pair has none of its own and runs without a balanced tail while its
    stream is being captured.  Every replay must reproduce the oracle, with eager launches of the
    same calls (which do balance the tail) in between."""
    import torch
    tile = (256, 256)
    M, N, K, tp, rank = TAIL[tile]
    W = N // tp
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=1700)
    want = oracle.fused_path(a, b, inc, tp, rank, *tile, fwd_direct=True,
                             fwd_init=np.zeros((tp - 1, M, W), np.float32))
    dev = torch.device("cuda:0")
    A, B = gpu.to_dev_bits(a), gpu.to_dev_bits(b)
    inc_dev = torch.from_numpy(inc).to(dev)
    R = inc_dev.clone()
    C = torch.zeros((M, N), dtype=torch.float32, device=dev)
    fwd = torch.zeros((tp - 1, M, W), dtype=torch.float32, device=dev)
    track = torch.zeros(t3.t3_track_words(tp), dtype=torch.int32, device=dev)
    p = t3.problem(M, N, K, tp, rank, *tile, flags=t3.T3_FLAG_FWD_DIRECT)

    def step():
        t3.t3_track_reset(tp, track)
        if unfused:
            t3.t3_gemm(p, A, B, C)
            t3.t3_rs_reduce(p, C, R, fwd, track)
        else:
            t3.t3_gemm_rs_fused(p, A, B, R, fwd, track)

    def check(what):
        torch.cuda.synchronize()
        own = want["own"]
        assert np.array_equal(fwd.cpu().numpy(), want["fwd"]), what
        assert np.array_equal(R.cpu().numpy()[:, own * W:(own + 1) * W], want["owned"]), what
        tr = t3.read_track(track, tp)
        assert np.array_equal(tr["counter"], want["counter"]) and tr["queue_len"] == tp - 1, what
        assert tr["error"] == 0, what

    def restore():
        R.copy_(inc_dev)
        fwd.zero_()
        C.fill_(3.0)
        torch.cuda.synchronize()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    check("eager, before capture")
    restore()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        step()
    for rep in range(3):
        restore()
        g.replay()
        check(f"replay {rep}")
        restore()
        step()
        check(f"eager after replay {rep}")


@pytest.mark.parametrize("direct", [False, True])
def test_balanced_tail_single_rank_in_place(gpu, oracle, direct):
    """tp = 1: one chunk, the rank's own, reduced in place in R (no release work in either mode,
    so the launch is persistent and balances its tail); the partial sums of the split tiles pass
    through the very place the incoming partial was read from."""
    tile, (M, N, K, tp, rank) = (256, 256), (4090, 10240, 520, 1, 0)
    assert _workgroup_tiles(M, N, tp, tile) == 2 * CUS + 128
    print(f"tile={tile} shape={(M, N, K, tp, rank)} direct={direct}", flush=True)
    a, b, inc = wl.make_integer_inputs(M, N, K, seed=1800)
    want = oracle.fused_path(a, b, inc, tp, rank, *tile, fwd_direct=direct,
                             fwd_init=np.full((0, M, N), gpu.SENTINEL, np.float32))
    got = gpu.run_gpu(a, b, inc, tp, rank, tile, flags=t3.T3_FLAG_FWD_DIRECT if direct else 0,
                      ldr_pad=4, launches_before=1)
    assert np.array_equal(got["R"], want["R"]), _first_mismatch(got["R"], want["R"])
    assert np.all(got["R_pad"] == 123.0)
    _check_ints(got, want, want["own"])

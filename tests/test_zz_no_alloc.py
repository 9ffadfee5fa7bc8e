"""The entry point that allocates nothing (t3_gemm_rs_fused_static: tracker state in a fixed
array inside the library) against t3_gemm_rs_fused, through the C ABI: same R, same forward
slots, same tracker results, bit for bit, on two calls in a row, the second on a smaller
problem (so the array still holds the first call's state when the second starts)."""
import numpy as np
import pytest

from paper_2401_16677_amd import binding as t3
from paper_2401_16677_amd import workloads as wl

pytestmark = pytest.mark.gpu

SENTINEL = -7.0


def _run(case, flags, static, torch):
    M, N, K, tp, rank, tile, seed = case
    a, b, inc = wl.make_inputs(wl.make_shape("na", M, N, K, tp, rank, *tile, index=seed))
    dev = torch.device("cuda:0")
    A = torch.from_numpy(a.view(np.int16)).to(dev)
    B = torch.from_numpy(b.view(np.int16)).to(dev)
    R = torch.from_numpy(inc).to(dev)
    fwd = torch.full((tp - 1, M, N // tp), SENTINEL, dtype=torch.float32, device=dev)
    track = torch.full((t3.t3_track_words(tp),), 0x5A5A5A5A, dtype=torch.int32, device=dev)
    p = t3.problem(M, N, K, tp, rank, *tile, flags=flags)
    if static:
        free0 = torch.cuda.mem_get_info()[0]
        t3.t3_gemm_rs_fused_static(p, A, B, R, fwd, track)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free0          # no device memory was taken
    else:
        t3.t3_track_reset(tp, track)
        t3.t3_gemm_rs_fused(p, A, B, R, fwd, track)
        torch.cuda.synchronize()
    return R.cpu().numpy(), fwd.cpu().numpy(), t3.read_track(track, tp)


@pytest.mark.parametrize("flags", [0, t3.T3_FLAG_FWD_DIRECT])
def test_static_tracker_entry_matches_the_caller_tracker_entry(flags):
    import torch
    assert torch.cuda.is_available(), "needs a GPU"
    # first a problem whose last round of tiles is split in halves of K (the flags between the
    # halves live in the static array too), then one with many tiles per workgroup and 8 chunks,
    # then a smaller one with 4
    cases = [(2040, 20480, 520, 5, 2, (256, 256), 40), (2040, 12288, 200, 8, 3, (256, 256), 41),
             (300, 1024, 136, 4, 1, (128, 128), 42)]
    for case in cases:
        print(f"case={case} flags={flags}", flush=True)
        R0, f0, tr0 = _run(case, flags, False, torch)
        R1, f1, tr1 = _run(case, flags, True, torch)
        assert np.array_equal(R0, R1) and np.array_equal(f0, f1)
        tp = case[3]
        assert np.array_equal(tr0["counter"], tr1["counter"]) and np.all(tr1["ready"] == 1)
        assert tr1["queue_len"] == tr0["queue_len"] == tp - 1
        assert set(tr1["queue"][:tp - 1].tolist()) == set(tr0["queue"][:tp - 1].tolist())
        assert np.all(tr1["queue"][tp - 1:] == 0xFFFFFFFF)
        assert tr1["error"] == 0 and tr1["gen"] == 1 and tr1["done"] == tr0["done"]


def test_static_tracker_entry_limits():
    import torch
    assert torch.cuda.is_available(), "needs a GPU"
    dev = torch.device("cuda:0")
    x = torch.zeros(1 << 16, dtype=torch.float32, device=dev)
    tp = t3.T3_STATIC_MAX_TP * 2
    p = t3.problem(128, 8 * tp, 64, tp, 0, 128, 128)
    with pytest.raises(t3.T3Error) as e:
        t3.t3_gemm_rs_fused_static(p, x, x, x, x)
    assert e.value.status == t3.T3_ERR_UNSUPPORTED
    p = t3.problem(128, 512, 64, 4, 0, 128, 128, flags=t3.T3_FLAG_TWO_WRITERS)
    with pytest.raises(t3.T3Error) as e:
        t3.t3_gemm_rs_fused_static(p, x, x, x, x)
    assert e.value.status == t3.T3_ERR_UNSUPPORTED

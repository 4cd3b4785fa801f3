"""The automatic kernel choice against every forced choice, timed on the GPU on a small grid of
mid-size shapes (where tile shape, K split and kernel family all matter): the automatic pick must be
within 15 % of the best forced pick.  Times are minima over flushed replays of a captured graph after
a clock warm-up, the protocol of bench.py; one microsecond of slack absorbs timer granularity."""
import pytest
import torch

import bench
from paper_2406_09904_amd import binding as qqq
from paper_2406_09904_amd import synth

pytestmark = pytest.mark.gpu

GRID = [(64, 11008, 4096, "perchannel"), (128, 5120, 13824, "perchannel"), (512, 5120, 13824, "perchannel"),
        (256, 8192, 28672, "perchannel"), (1024, 4096, 4096, "perchannel"), (256, 8192, 28672, "pergroup")]


@pytest.fixture(autouse=True)
def _reset():
    yield
    qqq.set_prefill_tuning(0)
    qqq.set_prefill_ksplit(0)
    qqq.set_kernel_override(0)


@pytest.mark.parametrize("M,K,N,variant", GRID)
def test_automatic_pick_is_close_to_the_best_forced_pick(M, K, N, variant):
    wl = synth.Workload("dispatch", variant, M, K, N, seed=700 + M)
    case = bench.Case(wl, torch, qqq, rotate_bytes=1 << 28)

    def us():
        case.gemm(0)
        route = qqq.last_route()
        t, _ = bench.timed(torch, case.gemm, 20, 3, True, replays=4)
        return t["min"] * 1e3, route

    auto_us, auto_route = us()
    forced = {}
    picks = [(2, 10, 1), (2, 15, 1), (2, 16, 1), (2, 17, 1), (2, 13, 0)]
    if M <= 512:
        picks += [(2, t, s) for t in (15, 16, 17) for s in (2, 4)]
    if M <= 64:
        picks.append((1, 0, 0))
    for family, tune, ksplit in picks:
        qqq.set_kernel_override(family)
        qqq.set_prefill_tuning(tune)
        qqq.set_prefill_ksplit(ksplit)
        forced[(family, tune, ksplit)] = us()
    best = min(forced, key=lambda k: forced[k][0])
    print("M=%d K=%d N=%d %s: automatic %.1f us (%s); best forced %.1f us (%s)" % (
        M, K, N, variant, auto_us, auto_route, forced[best][0], forced[best][1]), flush=True)
    assert auto_us <= 1.15 * forced[best][0] + 1.0, (auto_route, forced[best])

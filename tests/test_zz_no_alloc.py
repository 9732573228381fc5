"""The entry point that allocates nothing (sparbit_allgather_static): its output against the entry point it is a
variant of (sparbit_allgather_steps over the whole range) and against the CPU oracle, bit-exact, on two calls in a
row, the second with a smaller input; its size limit; and a check that it really does not allocate device memory."""
import numpy as np
import pytest

import oracle
import paper_2109_08751_amd as sb
from paper_2109_08751_amd import workloads

pytestmark = pytest.mark.gpu

POISON = workloads.POISON


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available()
    return t


def _one_case(torch, p, B, in_place, stream):
    print("[case] static", p, B, in_place, flush=True)
    dev = torch.device("cuda:0")
    send = workloads.make_send_raw(p, B, seed=p + B)
    d_send = torch.from_numpy(send).to(dev)
    got = torch.full((p, p, B), POISON, dtype=torch.uint8, device=dev)
    ref = torch.full((p, p, B), POISON, dtype=torch.uint8, device=dev)
    if in_place:
        for r in range(p):
            got[r, r] = d_send[r]
            ref[r, r] = d_send[r]
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    sb.sparbit_allgather_static(None if in_place else d_send, got, p, B, stream)
    free_after = torch.cuda.mem_get_info()[0]
    nsteps = sb.Plan(p).num_steps
    sb.sparbit_allgather_steps(None if in_place else d_send, ref, p, B, sb.SPARBIT, -1, nsteps - 1, stream)
    torch.cuda.synchronize()
    assert torch.equal(got, ref), (p, B, in_place)
    want = np.full((p, p, B), POISON, dtype=np.uint8)
    if in_place:
        for r in range(p):
            want[r, r] = send[r]
    oracle.allgather(oracle.SPARBIT, p, B, None if in_place else send, want)
    assert np.array_equal(got.cpu().numpy(), want), (p, B, in_place)
    return free_before - free_after


def test_two_calls_in_a_row_the_second_smaller(torch):
    st = torch.cuda.Stream()
    _one_case(torch, 6, 1024, False, st)  # first use on the device: looks up the array's address
    grew = [_one_case(torch, 96, 4096, False, st), _one_case(torch, 21, 1040, False, st),
            _one_case(torch, 257, 4100, True, st), _one_case(torch, 5, 17, False, st),
            _one_case(torch, 512, 64, False, st), _one_case(torch, 64, 65536, False, st)]
    assert all(g <= 0 for g in grew), grew  # no device memory was taken by any of the calls


def test_back_to_back_without_synchronising(torch):
    """Calls in stream order share the table safely: each call's table kernel runs after the previous call's steps."""
    dev = torch.device("cuda:0")
    st = torch.cuda.Stream()
    jobs = []
    for p, B in ((96, 4096), (33, 2048), (128, 512), (7, 16)):
        send = workloads.make_send_raw(p, B, seed=p)
        jobs.append((p, B, send, torch.from_numpy(send).to(dev),
                     torch.full((p, p, B), POISON, dtype=torch.uint8, device=dev)))
    torch.cuda.synchronize()
    for _ in range(3):
        for p, B, _, d_send, d_recv in jobs:
            sb.sparbit_allgather_static(d_send, d_recv, p, B, st)
    torch.cuda.synchronize()
    for p, B, send, _, d_recv in jobs:
        want = np.full((p, p, B), POISON, dtype=np.uint8)
        oracle.allgather(oracle.SPARBIT, p, B, send, want)
        assert np.array_equal(d_recv.cpu().numpy(), want), (p, B)


def test_limit_and_argument_checks(torch):
    d = torch.full((1 << 20,), POISON, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(sb.SparbitError) as e:
        sb.sparbit_allgather_static(d[:513], d[4096:], 513, 1)
    assert e.value.code == -7
    with pytest.raises(sb.SparbitError) as e:
        sb.sparbit_allgather_static(d[:64], d[32:], 4, 16)  # overlapping buffers
    assert e.value.code == -2
    sb.sparbit_allgather_static(d[:64], d[4096:], 4, 0)  # zero-size blocks: nothing to do
    torch.cuda.synchronize()
    assert bool((d == POISON).all())

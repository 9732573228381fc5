"""GPU parity: the HIP path, called through the C-ABI binding, against the CPU
oracle on the same seeded payloads.  Everything is bytes, so the bar is
bit-exact equality (np.array_equal / torch.equal on uint8)."""
import numpy as np
import pytest

import oracle
import paper_2109_08751_amd as sb
from paper_2109_08751_amd import workloads

pytestmark = pytest.mark.gpu

POISON = workloads.POISON
MODES = {"per_step": sb.MODE_PER_STEP, "persistent": sb.MODE_PERSISTENT, "auto": sb.MODE_AUTO,
         "dataflow": sb.MODE_DATAFLOW, "tree": sb.MODE_TREE}
ORACLE_ALGO = {sb.SPARBIT: oracle.SPARBIT, sb.RING: oracle.RING,
               sb.RECURSIVE_DOUBLING: oracle.RECURSIVE_DOUBLING, sb.BRUCK: oracle.BRUCK,
               sb.DIRECT: oracle.NAIVE}


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available()
    return t


def announce(*what):
    print("[case]", *what, flush=True)


def oracle_result(algo, p, B, send, max_steps=-1, in_place=False):
    recv = np.full((p, p, B), POISON, dtype=np.uint8)
    if in_place:
        for r in range(p):
            recv[r, r] = send[r]
    if algo == sb.DIRECT:
        oracle.naive_allgather(p, B, send, recv)
    else:
        oracle.allgather(ORACLE_ALGO[algo], p, B, None if in_place else send, recv, max_steps)
    return recv


def gpu_buffers(torch, p, B, send, in_place=False, misalign=0, send_misalign=None):
    """Device send / poison-filled recv; `misalign` shifts both base addresses (`send_misalign`: the send
    buffer's own shift)."""
    dev = torch.device("cuda:0")
    sraw = torch.empty(p * B + 256, dtype=torch.uint8, device=dev)
    rraw = torch.full((p * p * B + 256,), POISON, dtype=torch.uint8, device=dev)
    ms = misalign if send_misalign is None else send_misalign
    assert 0 <= misalign <= 256 and 0 <= ms <= 256  # the views below must lie inside the allocations
    d_send = sraw[ms:ms + p * B]
    d_recv = rraw[misalign:misalign + p * p * B]
    d_send.copy_(torch.from_numpy(send.reshape(-1)))
    if in_place:
        v = d_recv.view(p, p, B)
        for r in range(p):
            v[r, r] = d_send.view(p, B)[r]
    return d_send, d_recv, (sraw, rraw)


def gpu_result(torch, algo, p, B, send, mode, in_place=False, misalign=0, send_misalign=None):
    d_send, d_recv, keep = gpu_buffers(torch, p, B, send, in_place, misalign, send_misalign)
    sb.sparbit_allgather_mode(None if in_place else d_send.data_ptr(), d_recv.data_ptr(), p, B, algo, mode)
    torch.cuda.synchronize()
    assert sb.sparbit_barrier_timeouts() == 0
    # nothing outside the receive buffer was touched
    assert bool((keep[1][:misalign] == POISON).all()) and bool((keep[1][misalign + p * p * B:] == POISON).all())
    return d_recv.cpu().numpy().reshape(p, p, B)


# ------------------------------------------------------------------ the configs
@pytest.mark.parametrize("mode", ["per_step", "persistent", "dataflow", "tree", "auto"])
@pytest.mark.parametrize("cfg", ["cfg1", "cfg3", "cfg2"])
def test_config_matches_oracle_element_by_element(torch, cfg, mode):
    w = workloads.WORKLOADS[cfg]
    announce(cfg, mode, w.p, w.block_bytes)
    send = workloads.make_send(w)
    want = oracle_result(sb.SPARBIT, w.p, w.block_bytes, send)
    got = gpu_result(torch, sb.SPARBIT, w.p, w.block_bytes, send, MODES[mode])
    assert np.array_equal(got, want)


@pytest.mark.parametrize("cfg", ["cfg1", "cfg3"])
def test_every_step_boundary_matches_oracle(torch, cfg):
    """The state after each Waitall of Algorithm 1 is unique; slots not yet
    received must still hold the poison the test put there."""
    w = workloads.WORKLOADS[cfg]
    p, B = w.p, w.block_bytes
    send = workloads.make_send(w, seed=workloads.DEFAULT_SEED + 1)
    d_send, d_recv, _ = gpu_buffers(torch, p, B, send)
    nsteps = sb.Plan(p).num_steps
    for last in range(-1, nsteps):
        announce(cfg, "steps up to", last)
        sb.sparbit_allgather_steps(d_send, d_recv, p, B, sb.SPARBIT, last, last)  # one more step
        torch.cuda.synchronize()
        want = oracle_result(sb.SPARBIT, p, B, send, max_steps=last + 1)
        assert np.array_equal(d_recv.cpu().numpy().reshape(p, p, B), want), last


# ------------------------------------------------------------------ sweeps
@pytest.mark.parametrize("mode", ["per_step", "persistent", "dataflow", "tree"])
def test_every_p_up_to_33_and_ragged_block_sizes(torch, mode):
    for p in list(range(1, 34)) + [63, 65, 100]:
        for B in (1, 3, 20, 100, 4096 + 16):
            if p > 33 and B not in (20, 4096 + 16):
                continue
            announce("sweep", mode, p, B)
            send = workloads.make_send_raw(p, B, seed=p * 1000 + B)
            want = oracle_result(sb.SPARBIT, p, B, send)
            got = gpu_result(torch, sb.SPARBIT, p, B, send, MODES[mode])
            assert np.array_equal(got, want), (p, B)


@pytest.mark.parametrize("mode", ["per_step", "persistent", "dataflow", "tree"])
@pytest.mark.parametrize("misalign", [1, 4, 16])
def test_misaligned_base_pointers(torch, mode, misalign):
    for p, B in ((6, 1024), (21, 48), (5, 70000), (33, 4100)):
        announce("misaligned", mode, misalign, p, B)
        send = workloads.make_send_raw(p, B, seed=misalign)
        want = oracle_result(sb.SPARBIT, p, B, send)
        got = gpu_result(torch, sb.SPARBIT, p, B, send, MODES[mode], misalign=misalign)
        assert np.array_equal(got, want), (p, B)


@pytest.mark.parametrize("algo", [sb.SPARBIT, sb.RING, sb.BRUCK, sb.DIRECT])
def test_blocks_off_the_16_byte_grid(torch, algo):
    """Blocks whose ends fall between 16-byte boundaries, source and destination shifted against each other:
    aligned body, byte-wise head and tail.  The bytes around the receive buffer must stay untouched."""
    cases = ((5, 513, 0, 0), (7, 1000, 3, 9), (8, 4099, 1, 0), (3, 70001, 15, 2), (12, (1 << 20) + 7, 5, 11),
             (16, 515, 0, 4), (9, 4100, 4, 8), (2, 1 << 16, 7, 7),
             # on the 16-byte grid but off the 128-byte one: long blocks take the same kernel
             (6, (1 << 16) + 16, 0, 0), (4, (1 << 18) + 64, 16, 32), (5, 1 << 17, 0, 48))
    for p, B, ms, mr in cases:
        send = workloads.make_send_raw(p, B, seed=B)
        for in_place in (False, True):
            if in_place and algo == sb.BRUCK:
                continue
            announce("off grid", algo, p, B, ms, mr, in_place)
            want = oracle_result(algo, p, B, send, in_place=in_place)
            got = gpu_result(torch, algo, p, B, send, sb.MODE_PER_STEP, in_place=in_place, misalign=mr,
                             send_misalign=ms)
            assert np.array_equal(got, want), (p, B, ms, mr, in_place)


def test_realigning_kernel_on_tiny_blocks(torch):
    """The same kernel forced onto blocks of 16..600 bytes: heads that reach the end of the block, bodies of zero
    or one vector, every relative shift of source and destination."""
    sb.sparbit_tune("realign_min_bytes", 16)
    try:
        for B in (17, 18, 23, 31, 33, 47, 63, 100, 255, 257, 600):
            for p, ms, mr in ((5, 0, 1), (6, 13, 0), (9, 2, 15)):
                announce("tiny realign", p, B, ms, mr)
                send = workloads.make_send_raw(p, B, seed=B + p)
                want = oracle_result(sb.SPARBIT, p, B, send)
                got = gpu_result(torch, sb.SPARBIT, p, B, send, sb.MODE_PER_STEP, misalign=mr, send_misalign=ms)
                assert np.array_equal(got, want), (p, B, ms, mr)
    finally:
        sb.sparbit_tune("realign_min_bytes", 512)


@pytest.mark.parametrize("mode", ["per_step", "persistent", "dataflow", "tree"])
def test_in_place(torch, mode):
    for p, B in ((1, 64), (6, 1024), (21, 48), (64, 4096), (257, 16)):
        announce("in place", mode, p, B)
        send = workloads.make_send_raw(p, B, seed=3)
        want = oracle_result(sb.SPARBIT, p, B, send, in_place=True)
        got = gpu_result(torch, sb.SPARBIT, p, B, send, MODES[mode], in_place=True)
        assert np.array_equal(got, want), (p, B)


def test_large_rank_count(torch):
    p, B = 1000, 16
    announce("p=1000")
    send = workloads.make_send_raw(p, B, seed=5)
    want = np.broadcast_to(send[None], (p, p, B))  # oracle pinned to this at p=1000 in the CPU tests
    for mode in ("per_step", "persistent", "dataflow", "tree"):
        got = gpu_result(torch, sb.SPARBIT, p, B, send, MODES[mode])
        assert np.array_equal(got, want)


def test_zero_size_blocks_and_single_rank(torch):
    d = torch.full((64,), POISON, dtype=torch.uint8, device="cuda:0")
    sb.sparbit_allgather(d[:16], d[32:], 4, 0)
    torch.cuda.synchronize()
    assert bool((d == POISON).all())
    send = workloads.make_send_raw(1, 48, seed=1)
    got = gpu_result(torch, sb.SPARBIT, 1, 48, send, sb.MODE_AUTO)
    assert np.array_equal(got, send[None])


@pytest.mark.parametrize("mode", ["persistent", "dataflow"])
def test_repeated_calls_on_two_streams(torch, mode):
    """Back-to-back single-launch calls reuse the per-stream barrier / flag state
    (also across different p and block sizes on one stream)."""
    w = workloads.WORKLOADS["cfg3"]
    send = workloads.make_send(w)
    want = oracle_result(sb.SPARBIT, w.p, w.block_bytes, send)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    bufs = [gpu_buffers(torch, w.p, w.block_bytes, send) for _ in range(2)]
    torch.cuda.synchronize()
    small = gpu_buffers(torch, 21, 48, workloads.make_send_raw(21, 48, seed=2))
    for it in range(5):
        for st, (d_send, d_recv, _) in zip((s1, s2), bufs):
            sb.sparbit_allgather_mode(d_send, d_recv, w.p, w.block_bytes, sb.SPARBIT, MODES[mode], st)
            sb.sparbit_allgather_mode(small[0], small[1], 21, 48, sb.SPARBIT, MODES[mode], st)
    torch.cuda.synchronize()
    assert bool((small[1].view(21, 21, 48) == small[0].view(1, 21, 48)).all())
    assert sb.sparbit_barrier_timeouts(s1) == 0 and sb.sparbit_barrier_timeouts(s2) == 0
    for _, d_recv, _ in bufs:
        assert np.array_equal(d_recv.cpu().numpy().reshape(want.shape), want)


# ------------------------------------------------------------------ context schedules
@pytest.mark.parametrize("mode", ["per_step", "persistent", "dataflow"])
@pytest.mark.parametrize("algo", [sb.RING, sb.RECURSIVE_DOUBLING, sb.BRUCK, sb.DIRECT])
def test_context_schedules_match_oracle(torch, algo, mode):
    for p, B in ((1, 32), (6, 1024), (8, 100), (64, 4096), (96, 4096), (33, 20)):
        if algo == sb.RECURSIVE_DOUBLING and p & (p - 1):
            continue
        announce("context", algo, mode, p, B)
        send = workloads.make_send_raw(p, B, seed=11)
        want = oracle_result(algo, p, B, send)
        got = gpu_result(torch, algo, p, B, send, MODES[mode])
        assert np.array_equal(got, want), (algo, p, B)


# ------------------------------------------------------------------ full size
def expected_origins(p, max_steps=-1):
    """The oracle run on 4-byte rank tags: which rank's block each slot holds
    after `max_steps` steps (-1 = never written)."""
    send = np.arange(p, dtype=np.int32).view(np.uint8).reshape(p, 4)
    recv = np.full((p, p), -1, dtype=np.int32)
    oracle.allgather(oracle.SPARBIT, p, 4, send, recv.view(np.uint8).reshape(p, p, 4), max_steps)
    return recv


@pytest.mark.parametrize("cfg,mode", [("cfg4", "auto"), ("cfg4", "per_step"), ("cfg5", "auto"), ("cfg5", "per_step"),
                                      ("cfg5", "dataflow"), ("cfg5", "persistent")])
def test_full_size_configs(torch, cfg, mode):
    """16 GiB receive buffers, in the launch configuration the benchmark times (AUTO: the tree kernel), as one
    launch per step, and, on the largest configuration, in the two self-waiting forms, which are accepted at any
    size (dataflow: one workgroup per 16 KiB piece, over a million of them; persistent: a cooperative launch).
    Every slot is compared on the device with the block the oracle says it must
    hold (oracle run on rank tags), after the last-but-one step (unreceived
    slots still poison) and at the end; sampled slots are also copied back and
    compared on the host."""
    w = workloads.WORKLOADS[cfg]
    p, B = w.p, w.block_bytes
    announce(cfg, "generating payload")
    send = workloads.make_send(w)
    dev = torch.device("cuda:0")
    d_send = torch.from_numpy(send).to(dev)
    d_recv = torch.full((p, p, B), POISON, dtype=torch.uint8, device=dev)
    nsteps = sb.Plan(p).num_steps

    announce(cfg, "steps -1 ..", nsteps - 2)
    sb.sparbit_allgather_steps(d_send, d_recv, p, B, sb.SPARBIT, -1, nsteps - 2)
    torch.cuda.synchronize()
    origin = expected_origins(p, nsteps - 1)
    poison_row = torch.full((B,), POISON, dtype=torch.uint8, device=dev)
    for r in range(p):
        have = torch.from_numpy(origin[r] >= 0).to(dev)
        idx = torch.from_numpy(np.where(origin[r] >= 0, origin[r], 0).astype(np.int64)).to(dev)
        want = torch.where(have[:, None], d_send[idx], poison_row[None, :])
        assert torch.equal(d_recv[r], want), (cfg, "intermediate", r)
        del want

    announce(cfg, "whole call,", mode)
    d_recv.fill_(POISON)
    if mode == "auto":
        sb.sparbit_allgather(d_send, d_recv, p, B)
        name = sb.sparbit_last_launch_info()[0]
        # the largest calls: runs of 8 with every forwarder read back at once, write-through for the other stores
        assert "tree_kernel" in name and ", 8, 4, true, " in name and name.endswith(", false, 8>"), name  # ... in gangs of 8
    else:
        sb.sparbit_allgather_mode(d_send, d_recv, p, B, sb.SPARBIT, MODES[mode])
    torch.cuda.synchronize()
    assert sb.sparbit_barrier_timeouts() == 0
    origin = expected_origins(p)
    assert (origin == np.arange(p)[None, :]).all()
    for r in range(p):
        assert torch.equal(d_recv[r], d_send), (cfg, "final", r)
    rng = np.random.default_rng(7)
    for r, k in zip(rng.integers(0, p, 24), rng.integers(0, p, 24)):
        assert np.array_equal(d_recv[r, k].cpu().numpy(), send[origin[r, k]])

    # With enough host memory: the oracle itself at full size, every byte compared.
    avail = 0
    for line in open("/proc/meminfo"):
        if line.startswith("MemAvailable:"):
            avail = int(line.split()[1]) * 1024
    if mode != "auto":
        return  # the byte-for-byte oracle run once per configuration is enough
    if avail < 3 * w.recv_bytes:
        print("[case]", cfg, "full-size oracle run skipped: host memory", avail >> 30, "GiB", flush=True)
        return
    announce(cfg, "oracle at full size")
    want = np.full((p, p, B), POISON, dtype=np.uint8)
    oracle.allgather(oracle.SPARBIT, p, B, send, want)
    for r in range(p):
        assert np.array_equal(d_recv[r].cpu().numpy(), want[r]), (cfg, "oracle row", r)


# ------------------------------------------------------------------ library life cycle
def test_finalize_then_reuse(torch):
    """sparbit_finalize drops every cache; the next call rebuilds them."""
    w = workloads.WORKLOADS["cfg1"]
    send = workloads.make_send(w)
    want = oracle_result(sb.SPARBIT, w.p, w.block_bytes, send)
    for _ in range(2):
        for mode in ("per_step", "persistent", "dataflow"):
            assert np.array_equal(gpu_result(torch, sb.SPARBIT, w.p, w.block_bytes, send, MODES[mode]), want)
        torch.cuda.synchronize()
        sb.sparbit_finalize()


def test_two_host_threads(torch):
    """Two host threads, each with its own stream and buffers, call concurrently."""
    import threading
    w = workloads.WORKLOADS["cfg3"]
    send = workloads.make_send(w)
    want = oracle_result(sb.SPARBIT, w.p, w.block_bytes, send)
    results, errors = {}, []

    def worker(i):
        try:
            st = torch.cuda.Stream()
            d_send, d_recv, _ = gpu_buffers(torch, w.p, w.block_bytes, send)
            torch.cuda.synchronize()
            for _ in range(20):
                sb.sparbit_allgather_mode(d_send, d_recv, w.p, w.block_bytes, sb.SPARBIT, sb.MODE_PER_STEP, st)
            st.synchronize()
            results[i] = d_recv.cpu().numpy().reshape(want.shape)
        except Exception as e:  # pragma: no cover
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors
    for i in range(2):
        assert np.array_equal(results[i], want)


@pytest.mark.parametrize("tree_auto", [0, 1])
def test_auto_calls_on_eight_streams_beside_a_heavy_kernel(torch, tree_auto):
    """With the tree kernel switched off AUTO sends small jobs and the leading steps of larger ones through grids
    that wait on ready flags (as it does for the other schedules); with it on, every call is one tree launch.  Eight
    streams issue such calls at once while another stream keeps the whole GPU busy with writes: every result must
    match the oracle and no bounded wait may expire."""
    sb.sparbit_tune("tree_auto", tree_auto)
    try:
        _eight_streams(torch)
    finally:
        sb.sparbit_tune("tree_auto", 1)


def _eight_streams(torch):
    dev = torch.device("cuda:0")
    cases = [(96, 4096), (64, 16384), (125, 512), (32, 65536), (12, 1024), (6, 1024), (256, 64), (16, 262144)]
    streams = [torch.cuda.Stream() for _ in cases]
    background = torch.cuda.Stream()
    big = torch.empty(2 << 30, dtype=torch.uint8, device=dev)
    jobs = []
    for i, (p, B) in enumerate(cases):
        send = workloads.make_send_raw(p, B, seed=40 + i)
        want = torch.from_numpy(oracle_result(sb.SPARBIT, p, B, send)).to(dev)
        d_send, d_recv, keep = gpu_buffers(torch, p, B, send)
        jobs.append((p, B, d_send, d_recv, want, keep))
    for rnd in range(6):
        announce("eight streams, round", rnd)
        for job in jobs:
            job[3].fill_(POISON)
        torch.cuda.synchronize()
        with torch.cuda.stream(background):
            for _ in range(4):
                big.fill_(rnd)
        for rep in range(10):
            for st, (p, B, d_send, d_recv, _, _) in zip(streams, jobs):
                sb.sparbit_allgather(d_send, d_recv, p, B, st)
        torch.cuda.synchronize()
        for p, B, _, d_recv, want, _ in jobs:
            assert torch.equal(d_recv.view(p, p, B), want), (rnd, p, B)
    assert sum(sb.sparbit_barrier_timeouts(st) for st in streams) == 0
    del big
    torch.cuda.empty_cache()


def _calls_until_quiet(call, limit=8):
    """Issues `call` until it neither raises nor leaves anything to report; returns how many times the library
    answered SPARBIT_ERR_TIMEOUT (-6)."""
    reports = 0
    for _ in range(limit):
        try:
            call()
            return reports
        except sb.SparbitError as e:
            assert e.code == -6, e
            reports += 1
    raise AssertionError("the stream never became quiet")


@pytest.mark.parametrize("mode", ["persistent", "dataflow"])
def test_expired_waits_are_reported_and_the_next_call_is_clean(torch, mode):
    """The waits of the self-waiting kernels are bounded.  With the bound set to zero a wait that does not find its
    condition met at the first look gives up: the launch still ends normally (every workgroup leaves), the per-stream
    counter moves, the next call on that stream answers SPARBIT_ERR_TIMEOUT once and enqueues nothing, and the call
    after that, with the normal bound, is correct again."""
    p, B = 64, 4096
    send = workloads.make_send_raw(p, B, seed=11)
    want = oracle_result(sb.SPARBIT, p, B, send)
    d_send, d_recv, _ = gpu_buffers(torch, p, B, send)
    st = torch.cuda.Stream()
    call = lambda: sb.sparbit_allgather_mode(d_send, d_recv, p, B, sb.SPARBIT, MODES[mode], st)
    call()  # allocates the stream's state with the normal bound
    before = sb.sparbit_barrier_timeouts(st)
    sb.sparbit_tune("spin_limit_ms", 0)
    reports = 0
    try:
        for _ in range(5):
            try:
                call()
            except sb.SparbitError as e:  # an earlier one of the five already ended with an expired wait
                assert e.code == -6
                reports += 1
        expired = sb.sparbit_barrier_timeouts(st) - before  # synchronises the stream: all launches ended
    finally:
        sb.sparbit_tune("spin_limit_ms", 2000)
    announce("expired waits", mode, expired, "reported while issuing", reports)
    assert 0 <= expired <= 5
    d_recv.fill_(POISON)
    torch.cuda.synchronize()
    # Every launch has ended, so whatever expired is visible to the host now: reported by the next call (one report
    # covers all launches since the last one), which enqueues nothing.
    try:
        call()
        assert expired == 0 or reports > 0
    except sb.SparbitError as e:
        assert e.code == -6 and expired > 0
        torch.cuda.synchronize()
        assert bool((d_recv == POISON).all())  # nothing was enqueued
        call()
    assert sb.sparbit_barrier_timeouts(st) - before == expired  # the clean call adds none
    assert np.array_equal(d_recv.cpu().numpy().reshape(p, p, B), want)
    # other entry points on that stream are quiet as well
    sb.sparbit_allgather(d_send, d_recv, p, B, st)
    st.synchronize()


def test_call_numbers_go_on_when_the_flag_array_grows(torch):
    """An expired wait leaves its call's number in the stream's abort word.  When a later, larger call makes the
    library allocate a bigger flag array, the numbers must not start over: the call that would get that number again
    would take every unsatisfied wait for aborted and return incomplete results without any error."""
    st = torch.cuda.Stream()
    small = (12, 4096)
    large = (64, 4096)
    bufs = {}
    for p, B in (small, large):
        send = workloads.make_send_raw(p, B, seed=p)
        bufs[(p, B)] = (send, *gpu_buffers(torch, p, B, send)[:2])
    def call(pb):
        p, B = pb
        sb.sparbit_allgather_mode(bufs[pb][1], bufs[pb][2], p, B, sb.SPARBIT, sb.MODE_DATAFLOW, st)
    call(small)  # call number 1 of this stream
    st.synchronize()
    sb.sparbit_tune("spin_limit_ms", 0)
    try:
        for _ in range(3):  # numbers 2 .. 4; whichever expire leave their number behind
            try:
                call(small)
            except sb.SparbitError as e:
                assert e.code == -6
        st.synchronize()
    finally:
        sb.sparbit_tune("spin_limit_ms", 2000)
    expired = sb.sparbit_barrier_timeouts(st)
    announce("expired before the growth", expired)
    _calls_until_quiet(lambda: call(small))
    for k in range(6):  # the first of these grows the flag array; none may reuse a number from above
        p, B = large
        bufs[large][2].fill_(POISON)
        torch.cuda.synchronize()
        call(large)
        st.synchronize()
        want = oracle_result(sb.SPARBIT, p, B, bufs[large][0])
        assert np.array_equal(bufs[large][2].cpu().numpy().reshape(p, p, B), want), k
    assert sb.sparbit_barrier_timeouts(st) == expired


def test_dataflow_call_counter_wraps(torch):
    """Ready flags hold the 32-bit number of the call that set them.  When the counter wraps, the flags are cleared
    before the numbers start over, so stale flags of 2^32 calls ago cannot pass for fresh ones."""
    p, B = 12, 4096
    send = workloads.make_send_raw(p, B, seed=21)
    want = oracle_result(sb.SPARBIT, p, B, send)
    d_send, d_recv, _ = gpu_buffers(torch, p, B, send)
    st = torch.cuda.Stream()
    for _ in range(3):  # calls 1..3 on this stream: flags now hold 1, 2 or 3
        sb.sparbit_allgather_mode(d_send, d_recv, p, B, sb.SPARBIT, sb.MODE_DATAFLOW, st)
    st.synchronize()
    import ctypes
    hook = sb.lib.sparbit_test_set_flow_call_number  # exported for this test only, not declared in sparbit.h
    hook.argtypes, hook.restype = [ctypes.c_longlong], ctypes.c_int
    assert hook(2) == -1  # only forward: numbers already handed out may still sit in ready flags
    assert hook(0xfffffffe) == 0
    for k in range(5):  # numbers 0xffffffff, then 1 (after the clearing), 2, 3, 4
        announce("call counter wrap", k)
        d_recv.fill_(POISON)
        torch.cuda.synchronize()
        sb.sparbit_allgather_mode(d_send, d_recv, p, B, sb.SPARBIT, sb.MODE_DATAFLOW, st)
        st.synchronize()
        assert np.array_equal(d_recv.cpu().numpy().reshape(p, p, B), want), k
    assert sb.sparbit_barrier_timeouts(st) == 0


def test_capture_in_a_hip_graph(torch):
    """Once the tables of (schedule, p) are cached a per-step call allocates
    nothing and enqueues only kernels, so it can be captured; every replay must
    reproduce the eager result, with eager work and synchronisation in between."""
    w = workloads.WORKLOADS["cfg3"]
    p, B = w.p, w.block_bytes
    send = workloads.make_send(w)
    want = oracle_result(sb.SPARBIT, p, B, send)
    d_send, d_recv, _ = gpu_buffers(torch, p, B, send)
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        sb.sparbit_allgather_mode(d_send, d_recv, p, B, sb.SPARBIT, sb.MODE_PER_STEP, st)  # builds the tables
        st.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            sb.sparbit_allgather_mode(d_send, d_recv, p, B, sb.SPARBIT, sb.MODE_PER_STEP, torch.cuda.current_stream())
    for rep in range(3):
        d_recv.fill_(POISON)          # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(d_recv.cpu().numpy().reshape(p, p, B), want), rep


def test_capture_of_an_auto_call_records_the_per_step_form(torch):
    """With the tree kernel switched off (AUTO as it is for the other schedules), a small AUTO call runs the
    dataflow kernel when issued eagerly; that kernel's call number is a launch
    argument, so a replay would find every ready flag already set.  On a capturing stream AUTO therefore records
    the per-step launches, the self-waiting modes are refused, and so is a call whose tables do not exist yet;
    the refused calls record nothing, so the graph still replays correctly."""
    sb.sparbit_tune("tree_auto", 0)
    try:
        _capture_of_an_auto_call(torch)
    finally:
        sb.sparbit_tune("tree_auto", 1)


def _capture_of_an_auto_call(torch):
    w = workloads.WORKLOADS["cfg1"]
    p, B = w.p, w.block_bytes
    send = workloads.make_send(w)
    want = oracle_result(sb.SPARBIT, p, B, send)
    d_send, d_recv, _ = gpu_buffers(torch, p, B, send)
    st = torch.cuda.Stream()
    refused = []
    sb.sparbit_finalize()  # drop every cached table, so that (Ring, 7) below is certainly absent
    with torch.cuda.stream(st):
        sb.sparbit_allgather(d_send, d_recv, p, B, st)  # eager: builds the tables
        st.synchronize()
        assert np.array_equal(d_recv.cpu().numpy().reshape(p, p, B), want)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            cur = torch.cuda.current_stream()
            for mode in (sb.MODE_DATAFLOW, sb.MODE_PERSISTENT):
                try:
                    sb.sparbit_allgather_mode(d_send, d_recv, p, B, sb.SPARBIT, mode, cur)
                except sb.SparbitError as e:
                    refused.append(e.code)
            try:
                sb.sparbit_allgather_algo(d_send, d_recv, 7, 16, sb.RING, cur)  # (Ring, 7) was never built
            except sb.SparbitError as e:
                refused.append(e.code)
            sb.sparbit_allgather(d_send, d_recv, p, B, cur)
    assert refused == [-3, -3, -3]
    for rep in range(3):
        d_recv.fill_(POISON)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(d_recv.cpu().numpy().reshape(p, p, B), want), rep
    assert sb.sparbit_barrier_timeouts(st) == 0


def test_auto_merges_leading_steps_into_one_dataflow_launch(torch):
    """AUTO sends the first small steps of a larger call through one dataflow launch and the rest as one launch
    per step; the split point moves with the item limit (0 = never merge)."""
    cases = ((sb.SPARBIT, 125, 512, False), (sb.SPARBIT, 64, 16384, False), (sb.SPARBIT, 33, 40000, True),
             (sb.RING, 40, 4096, False), (sb.RING, 17, 70000, True), (sb.BRUCK, 96, 4096, False),
             (sb.RECURSIVE_DOUBLING, 32, 65536, False), (sb.SPARBIT, 257, 1040, False), (sb.SPARBIT, 21, 4100, False))
    sb.sparbit_tune("tree_auto", 0)  # Sparbit too goes the way of the other schedules here
    try:
        for limit in (0, 64, 300, 1024):
            sb.sparbit_tune("hybrid_max_items", limit)
            for algo, p, B, in_place in cases:
                announce("hybrid", limit, algo, p, B, in_place)
                send = workloads.make_send_raw(p, B, seed=limit + p)
                want = oracle_result(algo, p, B, send, in_place=in_place)
                got = gpu_result(torch, algo, p, B, send, sb.MODE_AUTO, in_place=in_place,
                                 misalign=4 if B == 4100 else 0)
                assert np.array_equal(got, want), (limit, algo, p, B, in_place)
    finally:
        sb.sparbit_tune("hybrid_max_items", 512)
        sb.sparbit_tune("tree_auto", 1)


def test_maximum_rank_count(torch):
    """p = SPARBIT_MAX_P (4096): 16.7 million block copies in 12 steps."""
    p, B = 4096, 16
    announce("p=4096")
    send = workloads.make_send_raw(p, B, seed=8)
    want = oracle_result(sb.SPARBIT, p, B, send)
    assert np.array_equal(want, np.broadcast_to(send[None], (p, p, B)))
    got = gpu_result(torch, sb.SPARBIT, p, B, send, sb.MODE_PER_STEP)
    assert np.array_equal(got, want)
    sb.sparbit_finalize()  # drop the 134 MB table
    got = gpu_result(torch, sb.SPARBIT, p, B, send, sb.MODE_TREE)  # needs no table
    assert np.array_equal(got, want)


@pytest.mark.parametrize("mode", ["per_step", "tree"])
@pytest.mark.parametrize("extra,in_place", [(4112, False), (4112, True), (4, False)])
def test_blocks_larger_than_4_gib(torch, extra, in_place, mode):
    """Offsets inside one block beyond 32 bits: p = 2 with blocks of 4 GiB + a ragged tail
    (16-byte path, and a size that is only a multiple of 4: the realigning kernel).  The expected
    state is the oracle's, taken from its run on rank tags."""
    p, B = 2, (4 << 30) + extra
    announce("huge blocks", B, in_place)
    dev = torch.device("cuda:0")
    origin = expected_origins(p)
    assert (origin == np.arange(p)[None, :]).all()
    d_send = torch.randint(0, 256, (p, B), dtype=torch.uint8, device=dev)
    d_recv = torch.full((p, p, B), POISON, dtype=torch.uint8, device=dev)
    if in_place:
        for r in range(p):
            d_recv[r, r] = d_send[r]
    if mode == "tree" and extra % 16:
        # 2^30 four-byte elements per block are more pieces than one grid holds: the tree form says so
        with pytest.raises(sb.SparbitError) as e:
            sb.sparbit_allgather_mode(d_send, d_recv, p, B, sb.SPARBIT, MODES[mode])
        assert e.value.code == -3
        torch.cuda.synchronize()
        assert bool((d_recv[0, 0, :4096] == POISON).all())
        del d_send, d_recv
        torch.cuda.empty_cache()
        return
    sb.sparbit_allgather_mode(None if in_place else d_send, d_recv, p, B, sb.SPARBIT, MODES[mode])
    torch.cuda.synchronize()
    for r in range(p):
        for k in range(p):
            assert torch.equal(d_recv[r, k], d_send[origin[r, k]]), (r, k)
    del d_send, d_recv
    torch.cuda.empty_cache()


def _fill_aperiodic(torch, t, seed):
    """Fill a flat uint8 device tensor from a random piece whose length shares no factor with any tile, grid or
    block size, so that data copied from a wrong offset cannot look right."""
    g = torch.Generator(device=t.device)
    g.manual_seed(seed)
    piece = torch.randint(0, 256, ((1 << 28) + 12347,), dtype=torch.uint8, device=t.device, generator=g)
    for at in range(0, t.numel(), piece.numel()):
        n = min(piece.numel(), t.numel() - at)
        t[at:at + n] = piece[:n]


@pytest.mark.parametrize("shift", [0, 4])
def test_blocks_with_more_tiles_than_the_grid_holds(torch, shift):
    """Nine copies of 4 GiB + 4112-byte blocks in one launch (DIRECT, p = 3): one tile per workgroup would need
    more than 2^31 lanes along x, so the kernels take several trips (the aligned tile kernel, and with the base
    addresses shifted by 4 bytes the realigning one).  Expected state: the Allgather definition (Section II),
    which is what the oracle's DIRECT schedule is pinned to; compared on the device."""
    p, B = 3, (4 << 30) + 4112
    announce("more tiles than the grid", shift)
    dev = torch.device("cuda:0")
    sraw = torch.empty(p * B + 16, dtype=torch.uint8, device=dev)
    rraw = torch.full((p * p * B + 16,), POISON, dtype=torch.uint8, device=dev)
    d_send, d_recv = sraw[shift:shift + p * B], rraw[shift:shift + p * p * B]
    _fill_aperiodic(torch, d_send, 77 + shift)
    sb.sparbit_allgather_mode(d_send.data_ptr(), d_recv.data_ptr(), p, B, sb.DIRECT, sb.MODE_PER_STEP)
    torch.cuda.synchronize()
    for r in range(p):
        assert torch.equal(d_recv[r * p * B:(r + 1) * p * B], d_send), r
    assert bool((rraw[:shift] == POISON).all()) and bool((rraw[shift + p * p * B:] == POISON).all())
    del d_send, d_recv, sraw, rraw
    torch.cuda.empty_cache()


def test_randomized_cases(torch):
    """400 seeded random (schedule, p, block size, mode, in-place, misalignment, AUTO limits, tree-kernel
    settings) cases against the oracle."""
    rng = np.random.default_rng(20210908)
    algos = [sb.SPARBIT, sb.SPARBIT, sb.SPARBIT, sb.RING, sb.RECURSIVE_DOUBLING, sb.BRUCK, sb.DIRECT]
    modes = ["per_step", "persistent", "dataflow", "auto"]
    sizes = [1, 2, 3, 4, 7, 8, 12, 16, 20, 31, 32, 48, 64, 100, 128, 256, 500, 1024, 1040, 4096, 4100, 8192, 20000,
             65536, 70000, 513, 2049, 16400, 65552, 65600, 131072 + 64, 262144 + 16, 100003]
    done = 0
    while done < 400:
        algo = algos[rng.integers(len(algos))]
        p = int(rng.integers(1, 81))
        if algo == sb.RECURSIVE_DOUBLING:
            p = 1 << int(rng.integers(0, 7))
        B = sizes[rng.integers(len(sizes))]
        if p * p * B > (64 << 20):
            continue
        mode = modes[rng.integers(len(modes))]
        if algo in (sb.SPARBIT, sb.RECURSIVE_DOUBLING, sb.RING) and rng.integers(0, 3) == 0:
            mode = "tree"
            sb.sparbit_tune("tree_run_log2", int(rng.integers(0, 8)))
            sb.sparbit_tune("tree_small_bytes", [0, 96 << 20][rng.integers(2)])
            sb.sparbit_tune("tree_unroll", [1, 2][rng.integers(2)])
            sb.sparbit_tune("tree_store", [0, 2, 3][rng.integers(3)])
            sb.sparbit_tune("tree_prefetch", int(rng.integers(0, 2)))
        in_place = bool(rng.integers(0, 4) == 0) and algo != sb.BRUCK
        misalign = [0, 0, 0, 1, 4, 8, 16][rng.integers(7)]
        sb.sparbit_tune("hybrid_max_items", [0, 64, 1024, 1024][rng.integers(4)])
        sb.sparbit_tune("dataflow_max_items", [0, 256, 256, 2000][rng.integers(4)])
        announce("random", done, algo, p, B, mode, in_place, misalign)
        send = workloads.make_send_raw(p, B, seed=done)
        want = oracle_result(algo, p, B, send, in_place=in_place)
        try:
            got = gpu_result(torch, algo, p, B, send, MODES[mode], in_place=in_place, misalign=misalign)
        finally:
            sb.sparbit_tune("hybrid_max_items", 512)
            sb.sparbit_tune("dataflow_max_items", 256)
            sb.sparbit_tune("tree_run_log2", -1)
            sb.sparbit_tune("tree_small_bytes", 96 << 20)
            sb.sparbit_tune("tree_unroll", 1)
            sb.sparbit_tune("tree_store", 2)
            sb.sparbit_tune("tree_prefetch", 1)
        assert np.array_equal(got, want), (algo, p, B, mode, in_place, misalign)
        done += 1


def test_ring_with_256_steps(torch):
    """Ring at p = 257: 256 dependent launches (or barrier phases) per call."""
    p, B = 257, 64
    send = workloads.make_send_raw(p, B, seed=6)
    want = oracle_result(sb.RING, p, B, send)
    for mode in ("per_step", "persistent", "dataflow"):
        announce("ring 257", mode)
        assert np.array_equal(gpu_result(torch, sb.RING, p, B, send, MODES[mode]), want)

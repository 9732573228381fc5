"""Allgatherv (blocks of different sizes; the extension named in the paper's
conclusion): oracle pins on the CPU, host-side argument checks of the C-ABI,
and GPU parity against the oracle."""
import numpy as np
import pytest

import oracle
import paper_2109_08751_amd as sb
from paper_2109_08751_amd import binding, workloads

POISON = workloads.POISON


def geometry(p, seed, align=1, max_len=40, gaps=True, shuffle=True):
    """Random block sizes (some zero), displacements with gaps and in shuffled order."""
    rng = np.random.default_rng(seed)
    counts = rng.integers(0, max_len // align + 1, p) * align
    if p > 2:
        counts[rng.integers(0, p)] = 0
    order = rng.permutation(p) if shuffle else np.arange(p)
    displs = np.zeros(p, dtype=np.int64)
    at = 0
    for k in order:
        at += int(rng.integers(0, 3)) * align if gaps else 0
        displs[k] = at
        at += int(counts[k])
    row = at + (align * int(rng.integers(0, 3)) if gaps else 0)
    row = max(row, align)
    return counts.astype(np.uint64), displs.astype(np.uint64), int(row)


def payload(row, seed):
    return workloads.make_send_raw(1, row, seed).reshape(row)


def definition(p, counts, displs, row, send):
    """MPI_Allgatherv by definition: block k of the send layout lands at
    displs[k] of every receive buffer; everything else is untouched."""
    want = np.full((p, row), POISON, dtype=np.uint8)
    for r in range(p):
        for k in range(p):
            d, c = int(displs[k]), int(counts[k])
            want[r, d:d + c] = send[d:d + c]
    return want


@pytest.mark.parametrize("p", list(range(1, 34)) + [64, 96, 257])
def test_oracle_allgatherv_equals_definition(p):
    for algo in (oracle.SPARBIT, oracle.RING, oracle.NAIVE):
        counts, displs, row = geometry(p, seed=p * 3 + algo)
        send = payload(row, p)
        recv = np.full((p, row), POISON, dtype=np.uint8)
        oracle.allgatherv(algo, p, counts, displs, row, send, recv)
        assert np.array_equal(recv, definition(p, counts, displs, row, send)), (algo, p)


@pytest.mark.parametrize("p", [1, 2, 5, 6, 21, 64, 96])
def test_oracle_allgatherv_with_equal_blocks_is_allgather(p):
    """Same schedule, same messages: with counts = B and displs = k*B the
    result, every step boundary and the message log equal the Allgather run."""
    B = 6
    counts = np.full(p, B, dtype=np.uint64)
    displs = np.arange(p, dtype=np.uint64) * B
    send = workloads.make_send_raw(p, B, seed=p)
    for steps in range(-1, oracle.num_steps(oracle.SPARBIT, p) + 1):
        a = np.full((p, p, B), POISON, dtype=np.uint8)
        b = np.full((p, p * B), POISON, dtype=np.uint8)
        ra = oracle.allgather(oracle.SPARBIT, p, B, send, a, steps, want_trace=True)
        rb = oracle.allgatherv(oracle.SPARBIT, p, counts, displs, p * B, send.reshape(-1), b, steps, want_trace=True)
        assert np.array_equal(a.reshape(p, p * B), b)
        assert np.array_equal(ra.trace, rb.trace) and np.array_equal(ra.step_info, rb.step_info)


@pytest.mark.parametrize("p", [2, 5, 21, 33])
def test_oracle_allgatherv_message_log_does_not_depend_on_sizes(p):
    counts, displs, row = geometry(p, seed=p)
    recv = np.full((p, row), POISON, dtype=np.uint8)
    rv = oracle.allgatherv(oracle.SPARBIT, p, counts, displs, row, payload(row, 1), recv, want_trace=True)
    ru = oracle.allgather(oracle.SPARBIT, p, 1, np.zeros((p, 1), np.uint8), np.zeros((p, p, 1), np.uint8),
                          want_trace=True)
    assert np.array_equal(rv.trace, ru.trace)
    assert (rv.sent_per_rank == p - 1).all()


def test_oracle_allgatherv_in_place_and_rejections():
    p = 7
    counts, displs, row = geometry(p, seed=11)
    send = payload(row, 2)
    recv = np.full((p, row), POISON, dtype=np.uint8)
    for r in range(p):
        d, c = int(displs[r]), int(counts[r])
        recv[r, d:d + c] = send[d:d + c]
    oracle.allgatherv(oracle.SPARBIT, p, counts, displs, row, None, recv)
    assert np.array_equal(recv, definition(p, counts, displs, row, send))
    with pytest.raises(oracle.OracleError):  # Bruck's rotated buffer needs equal blocks
        oracle.allgatherv(oracle.BRUCK, p, counts, displs, row, send, recv)
    bad = counts.copy()
    bad[0] = row + 1
    with pytest.raises(oracle.OracleError):
        oracle.allgatherv(oracle.SPARBIT, p, bad, displs, row, send, recv)


def test_allgatherv_arguments_are_checked_on_the_host():
    L = binding.lib
    import ctypes
    def call(p, counts, displs, row, algo=0, send=0x1000, recv=0x100000):
        c = (ctypes.c_size_t * len(counts))(*counts)
        d = (ctypes.c_size_t * len(displs))(*displs)
        return L.sparbit_allgatherv(send, recv, p, c, d, row, algo, None)
    assert call(0, [1], [0], 8) == -1
    assert call(2, [4, 5], [0, 4], 8) == -1           # block 1 runs past the row
    assert call(2, [4, 4], [0, 2], 8) == -1           # blocks overlap
    assert call(3, [4, 4, 4], [0, 4, 8], 12, algo=sb.BRUCK) == -3
    assert call(3, [4, 4, 4], [0, 4, 8], 12, algo=sb.RECURSIVE_DOUBLING) == -3
    assert call(2, [4, 4], [0, 4], 8, send=0x100004) == -2   # send overlaps the receive buffers
    assert call(2, [0, 0], [0, 0], 8) == 0            # nothing to move
    assert call(2, [4, 4], [0, 4], 1 << 39, send=1 << 44, recv=1 << 45) == -1   # p * row_bytes reaches 2^40
    assert L.sparbit_allgatherv(0x1000, 0x100000, 2, None, None, 8, 0, None) == -1


# ------------------------------------------------------------------ GPU parity
import contextlib


@contextlib.contextmanager
def without_tree_kernel():
    """Sparbit as the other schedules go: dataflow launches for small calls and leading steps, else per step."""
    sb.sparbit_tune("tree_auto", 0)
    try:
        yield
    finally:
        sb.sparbit_tune("tree_auto", 1)


@contextlib.contextmanager
def launch_per_step_only():
    """AUTO without the tree kernel and without the dataflow launches: one launch per step and size class."""
    sb.sparbit_tune("tree_auto", 0)
    sb.sparbit_tune("hybrid_max_items", 0)
    sb.sparbit_tune("dataflow_max_items", 0)
    try:
        yield
    finally:
        sb.sparbit_tune("tree_auto", 1)
        sb.sparbit_tune("hybrid_max_items", 512)
        sb.sparbit_tune("dataflow_max_items", 256)


def gpu_allgatherv(torch, algo, p, counts, displs, row, send, in_place=False, misalign=0):
    dev = torch.device("cuda:0")
    assert 0 <= misalign <= 64  # the views below must lie inside the allocations
    sraw = torch.empty(row + 64, dtype=torch.uint8, device=dev)
    rraw = torch.full((p * row + 64,), POISON, dtype=torch.uint8, device=dev)
    d_send = sraw[misalign:misalign + row]
    d_recv = rraw[misalign:misalign + p * row]
    d_send.copy_(torch.from_numpy(send))
    if in_place:
        v = d_recv.view(p, row)
        for r in range(p):
            d, c = int(displs[r]), int(counts[r])
            v[r, d:d + c] = d_send[d:d + c]
    sb.sparbit_allgatherv(None if in_place else d_send, d_recv, p, counts, displs, row, algo)
    torch.cuda.synchronize()
    assert bool((rraw[:misalign] == POISON).all()) and bool((rraw[misalign + p * row:] == POISON).all())
    return d_recv.cpu().numpy().reshape(p, row)


@pytest.mark.gpu
def test_gpu_allgatherv_matches_oracle():
    import torch
    algos = {sb.SPARBIT: oracle.SPARBIT, sb.RING: oracle.RING, sb.RECURSIVE_DOUBLING: oracle.RECURSIVE_DOUBLING,
             sb.DIRECT: oracle.NAIVE}
    for p in list(range(1, 18)) + [21, 32, 33, 64, 96, 257]:
        for align, max_len in ((1, 40), (4, 400), (16, 9000)):
            counts, displs, row = geometry(p, seed=p * 10 + align, align=align, max_len=max_len)
            send = payload(row, p)
            for algo, oalgo in algos.items():
                if algo == sb.RECURSIVE_DOUBLING and p & (p - 1):
                    continue
                if algo == sb.RING and p > 64:
                    continue
                print("[case] allgatherv", p, align, algo, flush=True)
                want = np.full((p, row), POISON, dtype=np.uint8)
                oracle.allgatherv(oalgo, p, counts, displs, row, send, want)
                got = gpu_allgatherv(torch, algo, p, counts, displs, row, send)
                assert np.array_equal(got, want), (p, align, algo)
                with launch_per_step_only():  # the same call without the tree and dataflow launches
                    got = gpu_allgatherv(torch, algo, p, counts, displs, row, send)
                assert np.array_equal(got, want), (p, align, algo, "per step")
                if algo == sb.SPARBIT:
                    with without_tree_kernel():  # and as the other schedules go
                        got = gpu_allgatherv(torch, algo, p, counts, displs, row, send)
                    assert np.array_equal(got, want), (p, align, algo, "without the tree kernel")


@pytest.mark.gpu
def test_gpu_allgatherv_in_place_misaligned_and_cached_geometries():
    import torch
    for rep in range(2):  # the second pass hits the geometry cache, then evicts through it
        for p in (5, 6, 21, 33, 64, 7, 9, 11, 13, 15):
            counts, displs, row = geometry(p, seed=p, align=4, max_len=600)
            send = payload(row, p + rep)
            want = np.full((p, row), POISON, dtype=np.uint8)
            for r in range(p):
                d, c = int(displs[r]), int(counts[r])
                want[r, d:d + c] = send[d:d + c]
            oracle.allgatherv(oracle.SPARBIT, p, counts, displs, row, None, want)
            got = gpu_allgatherv(torch, sb.SPARBIT, p, counts, displs, row, send, in_place=True, misalign=4 * rep)
            assert np.array_equal(got, want), (rep, p)


@pytest.mark.gpu
def test_gpu_allgatherv_large_unequal_blocks():
    """Blocks from 0 bytes to 3 MiB in one call (several tiles, ragged tails)."""
    import torch
    p = 12
    rng = np.random.default_rng(5)
    counts = (rng.integers(0, 200000, p) * 16).astype(np.uint64)
    counts[3] = 0
    counts[7] = 16
    displs = np.concatenate([[0], np.cumsum(counts[:-1] + 32)]).astype(np.uint64)
    row = int(displs[-1] + counts[-1] + 48)
    send = np.tile(workloads.make_send_raw(1, 65536, 9).reshape(-1), row // 65536 + 1)[:row].copy()
    want = np.full((p, row), POISON, dtype=np.uint8)
    oracle.allgatherv(oracle.SPARBIT, p, counts, displs, row, send, want)
    got = gpu_allgatherv(torch, sb.SPARBIT, p, counts, displs, row, send)
    assert np.array_equal(got, want)


@pytest.mark.gpu
def test_gpu_allgatherv_skewed_sizes():
    """One 40 MiB block among blocks of 0 B .. 100 KiB: copies of one step go out in
    launches per size class."""
    import torch
    p = 9
    counts = np.array([16, 0, 40 << 20, 100 << 10, 48, 4096, 0, 33 << 10, 16], dtype=np.uint64)
    displs = np.concatenate([[0], np.cumsum(counts[:-1] + 16)]).astype(np.uint64)
    row = int(displs[-1] + counts[-1])
    send = np.tile(workloads.make_send_raw(1, 65536, 4).reshape(-1), row // 65536 + 1)[:row].copy()
    for algo, oalgo in ((sb.SPARBIT, oracle.SPARBIT), (sb.RING, oracle.RING), (sb.DIRECT, oracle.NAIVE)):
        print("[case] skewed allgatherv", algo, flush=True)
        want = np.full((p, row), POISON, dtype=np.uint8)
        oracle.allgatherv(oalgo, p, counts, displs, row, send, want)
        got = gpu_allgatherv(torch, algo, p, counts, displs, row, send)
        assert np.array_equal(got, want)


@pytest.mark.gpu
def test_gpu_allgatherv_blocks_off_the_16_byte_grid():
    """Byte-granular counts and displacements with blocks from 0 bytes to ~300 KiB: the body of every copy moves
    in 16-byte vectors, its ends byte-wise; gaps between blocks keep their poison."""
    import torch
    for p, seed, mis in ((5, 1, 0), (12, 2, 3), (33, 3, 8), (64, 4, 1)):
        rng = np.random.default_rng(seed)
        counts = rng.integers(0, 300000 // (1 + p // 16), p).astype(np.uint64)
        counts[rng.integers(0, p)] = 0
        counts[rng.integers(0, p)] = 1
        counts[rng.integers(0, p)] = 513
        gaps = rng.integers(0, 40, p).astype(np.uint64)
        displs = (np.concatenate([[0], np.cumsum(counts[:-1] + gaps[:-1])]) + 5).astype(np.uint64)
        # Rows as long as the blocks need, and rounded up to whole 128-byte lines (every rank's slot then lies the
        # same way relative to the lines).  Both go out as one launch of the any-alignment tree form, the first with
        # plain stores and only up to a total size; beyond it (limit 0 here) as one launch per step.
        tight = int(displs[-1] + counts[-1] + 9)
        for row, limit in ((tight, 512 << 20), (tight, 0), ((tight + 127) // 128 * 128, 512 << 20)):
            sb.sparbit_tune("tree_part_line_max_bytes", limit)
            send = np.tile(workloads.make_send_raw(1, 65536, seed).reshape(-1), row // 65536 + 1)[:row].copy()
            try:
                for in_place in (False, True):
                    print("[case] off-grid allgatherv", p, mis, row % 128, limit, in_place, flush=True)
                    want = np.full((p, row), POISON, dtype=np.uint8)
                    if in_place:
                        for r in range(p):
                            d, c = int(displs[r]), int(counts[r])
                            want[r, d:d + c] = send[d:d + c]
                    oracle.allgatherv(oracle.SPARBIT, p, counts, displs, row, None if in_place else send, want)
                    got = gpu_allgatherv(torch, sb.SPARBIT, p, counts, displs, row, send, in_place=in_place, misalign=mis)
                    name, launches = sb.sparbit_last_launch_info()
                    if limit:
                        store = 2 if row % 128 == 0 else 0
                        # store form 1: forwarders read back at once, AUTO's choice for calls of this size
                        assert "tree_kernel" in name and (f", 8, {store}, " in name or ", 8, 1, " in name), name
                        assert name.rstrip(">").split(", ")[5:8] == ["true", "true", "0"] and launches == 1, name
                    else:
                        assert "tree_kernel" not in name, name
                    assert np.array_equal(got, want), (p, row, limit, in_place)
            finally:
                sb.sparbit_tune("tree_part_line_max_bytes", 512 << 20)


@pytest.mark.gpu
def test_gpu_allgatherv_forwarders_read_back_at_once():
    """The tree kernel's form with plain stores and forwarders read back at once (what AUTO takes for calls the caches
    hold a good part of), forced onto small geometries with per-slot sizes: blocks of 0 .. 4 KiB on whole lines, gaps,
    shuffled displacements, in place."""
    import torch
    sb.sparbit_tune("tree_hot", 1)
    try:
        for p in (1, 2, 5, 8, 9, 12, 17, 33, 64, 96):
            counts, displs, row = geometry(p, seed=p + 40, align=128, max_len=4096)
            send = payload(row, p)
            for in_place in (False, True):
                print("[case] allgatherv read back at once", p, row, in_place, flush=True)
                want = np.full((p, row), POISON, dtype=np.uint8)
                if in_place:
                    for r in range(p):
                        d, c = int(displs[r]), int(counts[r])
                        want[r, d:d + c] = send[d:d + c]
                oracle.allgatherv(oracle.SPARBIT, p, counts, displs, row, None if in_place else send, want)
                got = gpu_allgatherv(torch, sb.SPARBIT, p, counts, displs, row, send, in_place=in_place)
                name = sb.sparbit_last_launch_info()[0]
                if counts.any() and not (p == 1 and in_place):
                    assert ", 8, 1, true, true, " in name, name
                assert np.array_equal(got, want), (p, in_place)
    finally:
        sb.sparbit_tune("tree_hot", -1)


@pytest.mark.gpu
@pytest.mark.parametrize("algo", ["sparbit", "recursive_doubling"])
def test_gpu_allgatherv_long_blocks_of_any_size_in_rows_a_multiple_of_64_kib(algo):
    """Per-slot sizes at 1-byte granularity, blocks of 0.5-1 MiB, some hundred MiB per call: in rows that are a multiple
    of 64 KiB apart AUTO runs the any-alignment form in gangs whose pieces are counted from the boundaries of the
    address grid (places ahead of a block's first piece and past its last one stay empty); in rows rounded up to 1 KiB
    only, as independent wavefronts.  From a base on a 64 KiB boundary and from one 48 bytes past it, in place."""
    import torch
    a, oa, p = (sb.SPARBIT, oracle.SPARBIT, 24) if algo == "sparbit" else (sb.RECURSIVE_DOUBLING, oracle.RECURSIVE_DOUBLING, 32)
    rng = np.random.default_rng(7)
    counts = rng.integers(512 << 10, (1 << 20) + 1, p).astype(np.uint64)
    counts[3] = 0
    counts[5] = 700
    displs = np.concatenate([[0], np.cumsum(counts[:-1])]).astype(np.uint64)
    for row_grain, misalign, in_place, gangs in ((65536, 0, False, True), (65536, 48, True, True), (1024, 0, False, False)):
        row = (int(counts.sum()) + row_grain - 1) // row_grain * row_grain
        assert p * row > (336 << 20)
        send = payload(row, p)
        print("[case] allgatherv, any sizes, long blocks", algo, p, row, misalign, in_place, flush=True)
        want = np.full((p, row), POISON, dtype=np.uint8)
        if in_place:
            for r in range(p):
                d, c = int(displs[r]), int(counts[r])
                want[r, d:d + c] = send[d:d + c]
        oracle.allgatherv(oa, p, counts, displs, row, None if in_place else send, want)
        got = gpu_allgatherv(torch, a, p, counts, displs, row, send, in_place=in_place, misalign=misalign)
        name = sb.sparbit_last_launch_info()[0]
        args = name.rstrip(">").split(", ")  # access type, U, NB, store, look-ahead, sizes, any, walk, team, gang
        assert "tree_kernel" in name and args[5] == "true" and args[6] == "true", name
        assert (args[9] == "4" and args[3] == "4") == gangs, name
        assert np.array_equal(got, want), (algo, row_grain, misalign, in_place)


@pytest.mark.gpu
def test_gpu_allgatherv_block_with_more_tiles_than_the_grid_holds():
    """Eight copies of a block of 4 GiB + 48 B in one launch (DIRECT, p = 8, the other blocks tiny): the looping
    kernel takes over.  Expected state: every receive buffer equals the send layout inside the blocks (the
    Allgatherv definition the oracle is pinned to) and keeps its poison in the gaps; compared on the device."""
    import torch
    p = 8
    counts = np.array([16, 48, (4 << 30) + 48, 0, 4096, 16, 1024, 32], dtype=np.uint64)
    displs = np.concatenate([[0], np.cumsum(counts[:-1] + 16)]).astype(np.uint64)
    row = int(displs[-1] + counts[-1] + 16)
    dev = torch.device("cuda:0")
    print("[case] allgatherv, more tiles than the grid", flush=True)
    d_send = torch.empty(row, dtype=torch.uint8, device=dev)
    g = torch.Generator(device=dev)
    g.manual_seed(5)
    piece = torch.randint(0, 256, ((1 << 28) + 12347,), dtype=torch.uint8, device=dev, generator=g)
    for at in range(0, row, piece.numel()):
        n = min(piece.numel(), row - at)
        d_send[at:at + n] = piece[:n]
    want = torch.full((row,), POISON, dtype=torch.uint8, device=dev)
    for k in range(p):
        d, c = int(displs[k]), int(counts[k])
        want[d:d + c] = d_send[d:d + c]
    d_recv = torch.full((p * row,), POISON, dtype=torch.uint8, device=dev)
    sb.sparbit_allgatherv(d_send, d_recv, p, counts, displs, row, sb.DIRECT)
    torch.cuda.synchronize()
    for r in range(p):
        assert torch.equal(d_recv[r * row:(r + 1) * row], want), r
    del d_send, d_recv, want, piece
    torch.cuda.empty_cache()


@pytest.mark.gpu
def test_gpu_allgatherv_with_packed_equal_blocks_is_the_allgather():
    """Equal counts packed back to back are handed to the equal-block path; same result as the oracle's Allgatherv."""
    import torch
    for p, B, algo, oalgo in ((6, 1024, sb.SPARBIT, oracle.SPARBIT), (33, 4100, sb.SPARBIT, oracle.SPARBIT),
                              (16, 70000, sb.RING, oracle.RING), (8, 48, sb.RECURSIVE_DOUBLING, oracle.RECURSIVE_DOUBLING)):
        counts = np.full(p, B, dtype=np.uint64)
        displs = (np.arange(p) * B).astype(np.uint64)
        row = p * B
        send = payload(row, p)
        for in_place in (False, True):
            print("[case] packed allgatherv", p, B, algo, in_place, flush=True)
            want = np.full((p, row), POISON, dtype=np.uint8)
            if in_place:
                for r in range(p):
                    want[r, r * B:(r + 1) * B] = send[r * B:(r + 1) * B]
            oracle.allgatherv(oalgo, p, counts, displs, row, None if in_place else send, want)
            got = gpu_allgatherv(torch, algo, p, counts, displs, row, send, in_place=in_place)
            assert np.array_equal(got, want), (p, B, algo, in_place)


@pytest.mark.gpu
def test_gpu_allgatherv_randomized_geometries():
    """300 seeded random geometries: schedule, p, size scale (40 B .. 2.4 MB), granularity (1, 4, 16, 128 bytes),
    empty blocks, one outsized block, shuffled displacements with gaps, in place, shifted base addresses."""
    import torch
    rng = np.random.default_rng(20210908)
    algos = [(sb.SPARBIT, oracle.SPARBIT), (sb.SPARBIT, oracle.SPARBIT), (sb.RING, oracle.RING),
             (sb.RECURSIVE_DOUBLING, oracle.RECURSIVE_DOUBLING), (sb.DIRECT, oracle.NAIVE)]
    done = 0
    while done < 300:
        algo, oalgo = algos[rng.integers(len(algos))]
        p = int(rng.integers(1, 70))
        if algo == sb.RECURSIVE_DOUBLING:
            p = 1 << int(rng.integers(0, 7))
        grain = int(rng.choice([1, 4, 16, 128]))
        scale = int(rng.choice([40, 600, 5000, 70000, 300000]))
        counts = (rng.integers(0, scale // grain + 1, p) * grain).astype(np.uint64)
        if rng.integers(3) == 0:
            counts[rng.integers(0, p)] = 0
        if rng.integers(4) == 0:
            counts[rng.integers(0, p)] = np.uint64(scale * 8 // grain * grain)
        gaps = (rng.integers(0, 5, p) * grain).astype(np.uint64)
        displs = np.zeros(p, dtype=np.uint64)
        at = int(rng.integers(0, 3)) * grain
        for k in rng.permutation(p):
            displs[k] = at
            at += int(counts[k]) + int(gaps[k])
        row = max(at + int(rng.integers(0, 3)) * grain, grain)
        if p * row > (48 << 20):
            continue
        in_place = bool(rng.integers(0, 4) == 0)
        mis = int(rng.choice([0, 0, 1, 4, 16, 64]))
        if grain >= 16 and mis % 16:
            mis = 0
        print("[case] random allgatherv", done, algo, p, grain, scale, row, in_place, mis, flush=True)
        send = payload(row, done)
        want = np.full((p, row), POISON, dtype=np.uint8)
        if in_place:
            for r in range(p):
                d, c = int(displs[r]), int(counts[r])
                want[r, d:d + c] = send[d:d + c]
        # the plain all-to-all definition needs the send buffer; in place it yields the same state
        oracle.allgatherv(oalgo, p, counts, displs, row, None if (in_place and algo != sb.DIRECT) else send, want)
        form = rng.integers(4)
        if form == 0:
            with launch_per_step_only():
                got = gpu_allgatherv(torch, algo, p, counts, displs, row, send, in_place=in_place, misalign=mis)
        elif form == 1:
            with without_tree_kernel():
                got = gpu_allgatherv(torch, algo, p, counts, displs, row, send, in_place=in_place, misalign=mis)
        else:
            got = gpu_allgatherv(torch, algo, p, counts, displs, row, send, in_place=in_place, misalign=mis)
        assert np.array_equal(got, want), (done, algo, p, grain, scale, in_place, mis)
        done += 1


@pytest.mark.gpu
def test_gpu_allgatherv_capture_in_a_hip_graph():
    """A geometry that was used once outside a capture can be recorded (per-step launches only, although the same
    call issued eagerly takes the dataflow launch) and replayed; a new geometry is refused with nothing recorded."""
    import torch
    sb.sparbit_tune("tree_auto", 0)
    try:
        _capture_without_the_tree_kernel(torch)
    finally:
        sb.sparbit_tune("tree_auto", 1)


def _capture_without_the_tree_kernel(torch):
    p = 6
    counts, displs, row = geometry(p, seed=77, align=16, max_len=2000)
    send = payload(row, 3)
    want = np.full((p, row), POISON, dtype=np.uint8)
    oracle.allgatherv(oracle.SPARBIT, p, counts, displs, row, send, want)
    dev = torch.device("cuda:0")
    d_send = torch.from_numpy(send).to(dev)
    d_recv = torch.full((p * row,), POISON, dtype=torch.uint8, device=dev)
    st = torch.cuda.Stream()
    refused = []
    with torch.cuda.stream(st):
        sb.sparbit_allgatherv(d_send, d_recv, p, counts, displs, row, sb.SPARBIT, st)
        st.synchronize()
        assert np.array_equal(d_recv.cpu().numpy().reshape(p, row), want)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            cur = torch.cuda.current_stream()
            try:
                sb.sparbit_allgatherv(d_send, d_recv, p, counts, displs, row + 16, sb.SPARBIT, cur)  # never seen
            except sb.SparbitError as e:
                refused.append(e.code)
            sb.sparbit_allgatherv(d_send, d_recv, p, counts, displs, row, sb.SPARBIT, cur)
    assert refused == [-3]
    for rep in range(3):
        d_recv.fill_(POISON)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(d_recv.cpu().numpy().reshape(p, row), want), rep


@pytest.mark.gpu
def test_gpu_allgatherv_expired_waits_are_reported_and_the_next_call_is_clean():
    """Same bounded waits in the Allgatherv dataflow launch: a zero bound makes them give up, the launches end and
    are counted, the next call on the stream answers SPARBIT_ERR_TIMEOUT once, and the call after it, with the
    normal bound, is correct."""
    import torch
    sb.sparbit_tune("tree_auto", 0)  # the tree kernel has no wait that can expire for lack of residency
    try:
        _expired_waits(torch)
    finally:
        sb.sparbit_tune("tree_auto", 1)


def _expired_waits(torch):
    p = 12
    counts, displs, row = geometry(p, seed=5, align=16, max_len=3000)
    send = payload(row, 8)
    want = np.full((p, row), POISON, dtype=np.uint8)
    oracle.allgatherv(oracle.SPARBIT, p, counts, displs, row, send, want)
    dev = torch.device("cuda:0")
    d_send = torch.from_numpy(send).to(dev)
    d_recv = torch.full((p * row,), POISON, dtype=torch.uint8, device=dev)
    st = torch.cuda.Stream()
    call = lambda: sb.sparbit_allgatherv(d_send, d_recv, p, counts, displs, row, sb.SPARBIT, st)
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
        expired = sb.sparbit_barrier_timeouts(st) - before
    finally:
        sb.sparbit_tune("spin_limit_ms", 2000)
    print("[case] allgatherv expired waits", expired, "reported while issuing", reports, flush=True)
    assert 0 <= expired <= 5
    d_recv.fill_(POISON)
    torch.cuda.synchronize()
    try:
        call()
        assert expired == 0 or reports > 0
    except sb.SparbitError as e:
        assert e.code == -6 and expired > 0
        call()
    assert sb.sparbit_barrier_timeouts(st) - before == expired
    assert np.array_equal(d_recv.cpu().numpy().reshape(p, row), want)


@pytest.mark.gpu
def test_gpu_allgatherv_equal_blocks_in_padded_rows():
    """Equal blocks at their packed positions in rows longer than p blocks: the equal-block tree kernel with the row
    length as its stride (no table), for power-of-two rank counts where padding the rows is the remedy for the
    stripe pattern meeting the address interleaving.  Also in place, and with the padding not a multiple of 16."""
    import torch
    for p, B, pad in ((8, 1024, 128), (64, 4096, 128), (128, 4096, 256), (16, 48, 16), (32, 1040, 4), (5, 4100, 7)):
        for in_place in (False, True):
            row = p * B + pad
            counts = np.full(p, B, dtype=np.uint64)
            displs = np.arange(p, dtype=np.uint64) * B
            send = payload(row, p)
            print("[case] padded rows", p, B, pad, in_place, flush=True)
            want = np.full((p, row), POISON, dtype=np.uint8)
            if in_place:
                for r in range(p):
                    want[r, r * B:(r + 1) * B] = send[r * B:(r + 1) * B]
            oracle.allgatherv(oracle.SPARBIT, p, counts, displs, row, None if in_place else send, want)
            got = gpu_allgatherv(torch, sb.SPARBIT, p, counts, displs, row, send, in_place=in_place)
            assert np.array_equal(got, want), (p, B, pad, in_place)
            if row % 16 == 0 or B < 512:  # else the blocks are off the 16-byte grid: realigning per-step kernels
                assert "tree_kernel" in sb.sparbit_last_launch_info()[0]


@pytest.mark.gpu
def test_gpu_allgatherv_capture_of_the_tree_kernel():
    """With the tree kernel a Sparbit Allgatherv call is one launch that reads the geometry's device copy; once the
    geometry is cached the call can be recorded and replayed."""
    import torch
    p = 21
    counts, displs, row = geometry(p, seed=78, align=16, max_len=5000)
    send = payload(row, 3)
    want = np.full((p, row), POISON, dtype=np.uint8)
    oracle.allgatherv(oracle.SPARBIT, p, counts, displs, row, send, want)
    dev = torch.device("cuda:0")
    d_send = torch.from_numpy(send).to(dev)
    d_recv = torch.full((p * row,), POISON, dtype=torch.uint8, device=dev)
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        sb.sparbit_allgatherv(d_send, d_recv, p, counts, displs, row, sb.SPARBIT, st)
        st.synchronize()
        assert np.array_equal(d_recv.cpu().numpy().reshape(p, row), want)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            sb.sparbit_allgatherv(d_send, d_recv, p, counts, displs, row, sb.SPARBIT, torch.cuda.current_stream())
    for rep in range(3):
        d_recv.fill_(POISON)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(d_recv.cpu().numpy().reshape(p, row), want), rep

"""GPU parity of the tree form (SPARBIT_MODE_TREE) beyond what the mode-parametrised tests of
test_gpu_parity.py cover: every traversal order, piece size and store form of the kernel, the refusals, and
recording into a HIP graph.  Bit-exact against the CPU oracle."""
import numpy as np
import pytest

import oracle
import paper_2109_08751_amd as sb
from paper_2109_08751_amd import workloads

from test_gpu_parity import POISON, announce, gpu_buffers, gpu_result, oracle_result

pytestmark = pytest.mark.gpu

DEFAULTS = {"tree_run_log2": -1, "tree_small_bytes": 96 << 20, "tree_unroll": 1, "tree_store": 2, "tree_prefetch": 1,
            "tree_lds_bytes": -1, "tree_any_align": 1, "realign_min_bytes": 512,
            "tree_part_line_max_bytes": 512 << 20, "tree_team_log2": -1, "tree_hot": -1, "tree_gang": -1,
            "tree_gang_apart_log2": -1}


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available()
    return t


@pytest.fixture(autouse=True)
def default_knobs():
    yield
    for k, v in DEFAULTS.items():
        sb.sparbit_tune(k, v)


@pytest.mark.parametrize("prefetch", [0, 1])
@pytest.mark.parametrize("run_log2", [0, 1, 2, 3, 4, 5, 7, 12])
def test_every_traversal_order(torch, run_log2, prefetch):
    """Runs of 1, 2, 4, ... relative ranks up to the whole tree (= step order), for rank counts around every
    power of two and the paper's examples (5, 21), with ragged pieces."""
    sb.sparbit_tune("tree_small_bytes", 0)  # the run length under test applies to every size
    sb.sparbit_tune("tree_run_log2", run_log2)
    sb.sparbit_tune("tree_prefetch", prefetch)
    sb.sparbit_tune("tree_store", 3 if prefetch else 2)
    for p in (1, 2, 3, 5, 6, 7, 8, 9, 15, 16, 17, 21, 31, 32, 33, 63, 64, 65, 96, 100, 127, 129, 257):
        for B in (16, 1040, 4096 + 16) if p <= 65 else (1040,):
            announce("tree order", run_log2, p, B)
            send = workloads.make_send_raw(p, B, seed=p * 7 + run_log2)
            want = oracle_result(sb.SPARBIT, p, B, send)
            got = gpu_result(torch, sb.SPARBIT, p, B, send, sb.MODE_TREE)
            assert np.array_equal(got, want), (run_log2, p, B)


@pytest.mark.parametrize("unroll", [1, 2])
@pytest.mark.parametrize("store", [0, 1, 2, 3, 4])
def test_piece_sizes_and_store_forms(torch, unroll, store):
    sb.sparbit_tune("tree_unroll", unroll)
    sb.sparbit_tune("tree_store", store)
    sb.sparbit_tune("tree_lds_bytes", 10240 if store == 2 else 0)
    for small in (0, 96 << 20):
        sb.sparbit_tune("tree_small_bytes", small)
        for p, B, in_place in ((6, 1024, False), (21, 5008, False), (33, 2048 + 1024 * unroll + 16, True),
                               (96, 4096, False), (64, 65536, False), (257, 48, True), (13, 1 << 18, False)):
            announce("tree pieces", unroll, store, small, p, B, in_place)
            send = workloads.make_send_raw(p, B, seed=B % 1000 + unroll)
            want = oracle_result(sb.SPARBIT, p, B, send, in_place=in_place)
            got = gpu_result(torch, sb.SPARBIT, p, B, send, sb.MODE_TREE, in_place=in_place)
            assert np.array_equal(got, want), (unroll, store, p, B, in_place)


def test_narrow_accesses(torch):
    """Blocks or base addresses off the 16-byte grid: the same kernel with 4- and 1-byte elements."""
    for p, B, mis in ((5, 20, 0), (9, 4100, 4), (6, 1023, 0), (33, 100, 1), (17, 70001, 3), (64, 4096, 8)):
        for in_place in (False, True):
            announce("tree narrow", p, B, mis, in_place)
            send = workloads.make_send_raw(p, B, seed=B)
            want = oracle_result(sb.SPARBIT, p, B, send, in_place=in_place)
            got = gpu_result(torch, sb.SPARBIT, p, B, send, sb.MODE_TREE, in_place=in_place, misalign=mis)
            assert np.array_equal(got, want), (p, B, mis, in_place)


def launched_any_alignment_form():
    name = sb.sparbit_last_launch_info()[0]
    return "tree_kernel" in name and name.rstrip(">").split(", ")[6] == "true"


@pytest.mark.parametrize("knobs", [{}, {"tree_small_bytes": 0, "tree_run_log2": 0, "tree_prefetch": 0},
                                   {"tree_small_bytes": 0, "tree_run_log2": 3, "tree_store": 0},
                                   {"tree_small_bytes": 0, "tree_run_log2": 2, "tree_lds_bytes": 14336}])
def test_any_alignment_form(torch, knobs):
    """Blocks of 512 bytes and more that do not start and end on 128-byte lines, in rows that are a multiple of 128
    bytes apart: pieces cut relative to the lines, 16-byte chunks plus single bytes at a block's two ends.  Block
    lengths and base addresses at 1-, 4- and 16-byte granularity, a first piece of 0 .. 127 bytes (0 .. 1023 in rows
    that are a multiple of 1 KiB apart), in place, and what AUTO does with such a call."""
    for k, v in knobs.items():
        sb.sparbit_tune(k, v)
    cases = ((128, 513, 0, 0), (128, 1028, 0, 0), (64, 4100, 0, 0), (32, 1000, 0, 0), (8, 65552, 0, 0), (16, 2072, 3, 5),
             (64, 4096, 1, 0), (64, 4096, 127, 13), (256, 600, 0, 0), (96, 4100, 0, 8), (257, 1280, 4, 0), (24, 70000, 0, 0),
             (8, 3 * 1024 + 16, 112, 0), (8, 2048, 16, 0), (40, 16 * 77, 15, 1),
             (64, 4112, 0, 0), (256, 1028, 0, 3), (128, 5 * 1024 + 8, 250, 0))  # rows a multiple of 1 KiB: pieces cut on 1 KiB boundaries
    for p, B, mis, smis in cases:
        assert p * B % 128 == 0
        for mode, in_place in ((sb.MODE_TREE, False), (sb.MODE_AUTO, False), (sb.MODE_TREE, True)):
            announce("tree any alignment", knobs, p, B, mis, smis, mode, in_place)
            send = workloads.make_send_raw(p, B, seed=B + p)
            want = oracle_result(sb.SPARBIT, p, B, send, in_place=in_place)
            got = gpu_result(torch, sb.SPARBIT, p, B, send, mode, in_place=in_place, misalign=mis, send_misalign=smis)
            assert launched_any_alignment_form(), sb.sparbit_last_launch_info()
            assert np.array_equal(got, want), (p, B, mis, smis, mode, in_place)


def test_any_alignment_form_on_tiny_blocks(torch):
    """The same form forced onto blocks of 16 .. 300 bytes: blocks that end before the first line boundary, pieces
    of single bytes only, a last piece of one byte."""
    sb.sparbit_tune("realign_min_bytes", 16)
    for p, B, mis in ((128, 16, 1), (128, 16, 120), (128, 17, 100), (128, 33, 1), (64, 50, 0), (128, 127, 1), (128, 129, 127),
                      (128, 300, 120), (128, 16, 8), (128, 31, 113), (128, 145, 0), (64, 256 + 2, 126)):
        assert p * B % 128 == 0
        for in_place in (False, True):
            announce("tree any alignment, tiny", p, B, mis, in_place)
            send = workloads.make_send_raw(p, B, seed=B + mis)
            want = oracle_result(sb.SPARBIT, p, B, send, in_place=in_place)
            got = gpu_result(torch, sb.SPARBIT, p, B, send, sb.MODE_TREE, in_place=in_place, misalign=mis)
            assert launched_any_alignment_form() or (B % 128 == 0 and mis == 0), sb.sparbit_last_launch_info()
            assert np.array_equal(got, want), (p, B, mis, in_place)


def test_rows_off_the_lines(torch):
    """Rows that are not a multiple of 128 bytes apart: the any-alignment form's stores then cover part-lines, so it
    stores plainly, and AUTO uses it only up to a total size; beyond that AUTO launches per step and the explicit
    mode runs narrow elements.  All match the oracle."""
    for p, B in ((125, 4100), (33, 1000), (61, 65552), (13, (1 << 18) + 1)):
        for limit in (512 << 20, 0):
            sb.sparbit_tune("tree_part_line_max_bytes", limit)
            for mode in (sb.MODE_AUTO, sb.MODE_TREE):
                announce("tree rows off lines", p, B, limit, mode)
                send = workloads.make_send_raw(p, B, seed=B)
                want = oracle_result(sb.SPARBIT, p, B, send)
                got = gpu_result(torch, sb.SPARBIT, p, B, send, mode)
                name = sb.sparbit_last_launch_info()[0]
                if limit:
                    # plain stores: form 0, or form 1 (forwarders read back at once) where AUTO's size rule picks it
                    assert launched_any_alignment_form() and (", 8, 0, " in name or ", 8, 1, " in name), name
                else:
                    assert not launched_any_alignment_form(), name
                    assert ("tree_kernel" in name) == (mode == sb.MODE_TREE or B % 16 == 0 and B < 65536), name
                assert np.array_equal(got, want), (p, B, limit, mode)


@pytest.mark.parametrize("extra", [4, 1])
def test_any_alignment_form_at_full_size(torch, extra):
    """128 ranks with blocks of 1 MiB + 4 bytes and 1 MiB + 1 byte (16 GiB of receive buffers), as AUTO launches
    them and as the benchmark times them: every slot of every rank is compared on the device with the block the
    oracle says it must hold (oracle run on rank tags), sampled slots on the host, and the bytes behind the
    receive buffers must be untouched."""
    from test_gpu_parity import expected_origins
    p, B = 128, (1 << 20) + extra
    announce("any alignment at full size", p, B)
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(workloads.DEFAULT_SEED + extra)
    d_send = torch.randint(0, 256, (p, B), dtype=torch.uint8, device=dev, generator=gen)
    raw = torch.full((p * p * B + 256,), POISON, dtype=torch.uint8, device=dev)
    d_recv = raw[:p * p * B].view(p, p, B)
    sb.sparbit_allgather(d_send, d_recv, p, B)
    torch.cuda.synchronize()
    assert launched_any_alignment_form(), sb.sparbit_last_launch_info()
    origin = expected_origins(p)
    for r in range(p):
        idx = torch.from_numpy(origin[r].astype(np.int64)).to(dev)
        assert torch.equal(d_recv[r], d_send[idx]), ("final", r)
    assert bool((raw[p * p * B:] == POISON).all())
    send = d_send.cpu().numpy()
    rng = np.random.default_rng(11)
    for r, k in zip(rng.integers(0, p, 16), rng.integers(0, p, 16)):
        assert np.array_equal(d_recv[r, k].cpu().numpy(), send[origin[r, k]])


@pytest.mark.parametrize("team_log2", [1, 2, 3, 4])
def test_teams_of_wavefronts(torch, team_log2):
    """Small calls: 2, 4, 8 or 16 wavefronts of one workgroup walk one run of a tree each and hand a run's first
    rank over through a flag in LDS.  Rank counts around every power of two (runs that do not exist, runs whose first
    rank has nothing to forward, a last run of one rank), all access widths, the any-alignment form, in place, with
    plain and write-through stores; and what AUTO does by itself (teams from 33 ranks on in calls up to 96 MiB)."""
    sb.sparbit_tune("tree_team_log2", team_log2)
    for p in (1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 21, 31, 32, 33, 47, 48, 49, 63, 64, 65, 96, 97, 127, 128, 129, 255, 256, 257):
        for B, mis in ((16, 0), (1040, 0), (100, 0), (333, 1), (4100, 0)) if p <= 65 else ((1040, 0), (513, 0)):
            in_place = (p + B) % 3 == 0
            sb.sparbit_tune("tree_store", 0 if (p + B) % 2 else 2)
            announce("tree team", team_log2, p, B, mis, in_place)
            send = workloads.make_send_raw(p, B, seed=p * 3 + team_log2)
            want = oracle_result(sb.SPARBIT, p, B, send, in_place=in_place)
            got = gpu_result(torch, sb.SPARBIT, p, B, send, sb.MODE_TREE, in_place=in_place, misalign=mis)
            name = sb.sparbit_last_launch_info()[0]
            if p > 2 and not (p == 1 and in_place):
                assert name.endswith(", true, 1>"), name  # a team
            assert np.array_equal(got, want), (team_log2, p, B, mis, in_place)


def test_auto_forms_teams_for_small_calls_of_many_ranks(torch):
    for p, B, team in ((32, 4096, False), (33, 4096, True), (96, 4096, True), (256, 1024, True), (257, 48, True),
                       (128, 16384, False)):  # the last one is 256 MiB: past the size limit of the step-order walk
        announce("tree team by itself", p, B)
        send = workloads.make_send_raw(p, B, seed=p)
        want = oracle_result(sb.SPARBIT, p, B, send)
        got = gpu_result(torch, sb.SPARBIT, p, B, send, sb.MODE_AUTO)
        name = sb.sparbit_last_launch_info()[0]
        assert "tree_kernel" in name and name.endswith(", true, 1>") == team, name
        assert np.array_equal(got, want), (p, B)


def test_forwarders_read_back_at_once(torch):
    """The form for calls that the caches hold a good part of: plain stores, runs of 8, every forwarder read back
    right after it was stored and kept in registers until its turn.  Forced onto every rank count around the run
    length, the powers of two and the multiples of 16, 32 and 64 (last runs of 1 .. 8 ranks, trees shorter than a run,
    runs whose first rank was kept in registers since it was stored 8, 16 or 32 ranks earlier, or is loaded), in place;
    and AUTO's own choice of it.  (Per-slot sizes: test_allgatherv.py.)"""
    sb.sparbit_tune("tree_hot", 1)
    for p in (1, 2, 3, 5, 7, 8, 9, 10, 15, 16, 17, 21, 23, 24, 25, 31, 32, 33, 40, 41, 47, 48, 49, 56, 57, 63, 64, 65, 72, 73,
              81, 96, 97, 113, 127, 129, 145, 193, 200, 257):
        for B in (16, 1024, 4096 + 128) if p <= 65 else (1024,):  # whole vectors on whole lines, or short blocks
            in_place = (p + B) % 3 == 0
            announce("tree read back at once", p, B, in_place)
            send = workloads.make_send_raw(p, B, seed=p * 5 + 1)
            want = oracle_result(sb.SPARBIT, p, B, send, in_place=in_place)
            got = gpu_result(torch, sb.SPARBIT, p, B, send, sb.MODE_TREE, in_place=in_place)
            name = sb.sparbit_last_launch_info()[0]
            if not (p == 1 and in_place):
                assert ", 8, 1, true, " in name, name
            assert np.array_equal(got, want), (p, B, in_place)
    sb.sparbit_tune("tree_hot", -1)
    for p, B, hot in ((64, 16384, True), (16, 262144, True), (64, 4096, False), (128, 8192, True), (128, 4096, False)):
        announce("tree read back at once, by itself", p, B)
        send = workloads.make_send_raw(p, B, seed=p)
        want = oracle_result(sb.SPARBIT, p, B, send)
        got = gpu_result(torch, sb.SPARBIT, p, B, send, sb.MODE_AUTO)
        name = sb.sparbit_last_launch_info()[0]
        assert "tree_kernel" in name and (", 8, 1, true, " in name) == hot, name
        assert np.array_equal(got, want), (p, B)


@pytest.mark.parametrize("algo,p,B", [
    ("sparbit", 61, 131072),   # 465 MiB, 7808 wavefronts: 16 resident per unit
    ("sparbit", 125, 33792),   # 504 MiB, 4125 wavefronts: a cap of 4096 would leave a round of 29, so another or none
    ("sparbit", 33, 393216),   # 408 MiB on few ranks
    ("sparbit", 16, 2 << 20),  # 512 MiB on fewer ranks than a capped grid used to need
    ("sparbit", 64, 131072 + 4),   # the any-alignment form in rows on the lines
    ("sparbit", 96, 57344),    # 504 MiB, 5376 wavefronts
    ("ring", 64, 131072), ("recursive_doubling", 64, 131072)])
def test_calls_of_some_hundred_mib(torch, algo, p, B):
    """Between the calls the caches hold and the 16 GiB ones AUTO picks store form 4 on a grid capped by size, rank
    count and the fill of its last round (Ring and Recursive Doubling: their own caps): every byte against the
    oracle, and the form that ran."""
    a = {"sparbit": sb.SPARBIT, "ring": sb.RING, "recursive_doubling": sb.RECURSIVE_DOUBLING}[algo]
    announce("some hundred MiB", algo, p, B)
    send = workloads.make_send_raw(p, B, seed=p + 3)
    want = oracle_result(a, p, B, send)
    got = gpu_result(torch, a, p, B, send, sb.MODE_AUTO)
    name = sb.sparbit_last_launch_info()[0]
    assert "tree_kernel" in name, name
    if algo == "sparbit":
        assert ", 8, 4, true, " in name, name
        assert launched_any_alignment_form() == (B % 16 != 0)
    assert np.array_equal(got, want), (algo, p, B)


def launched_gangs():
    """Wavefronts per gang in the last launch (4 or 8); 0 if it was not the tree kernel in gangs."""
    name = sb.sparbit_last_launch_info()[0]
    for size in (4, 8):
        if "tree_kernel" in name and name.endswith(", false, %d>" % size):
            return size
    return 0


@pytest.mark.parametrize("algo,p,B,store,gang", [
    ("sparbit", 16, 1 << 20, 1, 4),            # 256 MiB, forwarders read back at once: gangs from 240 MiB on
    ("sparbit", 48, 128 << 10, 1, 4),          # 288 MiB
    ("sparbit", 29, 256 << 10, 1, 0),          # 210 MiB: none
    ("sparbit", 40, 160 << 10, 1, 0),          # 250 MiB, blocks under 512 KiB off the 64 KiB boundaries: none
    ("recursive_doubling", 16, 1 << 20, 1, 4),
    ("ring", 16, 1 << 20, 0, 4),
    ("ring", 29, 256 << 10, 0, 0),
    ("sparbit", 64, 128 << 10, 4, 8),          # 512 MiB, blocks a multiple of 128 KiB, 48 ranks and more: one gang of 8 per unit
    ("sparbit", 64, 192 << 10, 4, 4),          # blocks a multiple of 64 KiB only
    ("sparbit", 32, 512 << 10, 4, 4),          # fewer than 48 ranks
    ("recursive_doubling", 64, 128 << 10, 4, 8),
    ("ring", 64, 128 << 10, 0, 8),
])
def test_where_auto_forms_gangs(torch, algo, p, B, store, gang):
    """AUTO's choice of the gang form by call size, block length and rank count (store form 1 from 240 MiB on with
    blocks of 128 KiB and more, store form 4 beyond 336 MiB, Ring's chain by the same sizes; gangs of 8 from 48 ranks
    on for blocks that are a multiple of 128 KiB), every byte against the oracle."""
    a = {"sparbit": sb.SPARBIT, "ring": sb.RING, "recursive_doubling": sb.RECURSIVE_DOUBLING}[algo]
    announce("where AUTO forms gangs", algo, p, B)
    send = workloads.make_send_raw(p, B, seed=p + 5)
    want = oracle_result(a, p, B, send)
    got = gpu_result(torch, a, p, B, send, sb.MODE_AUTO)
    name = sb.sparbit_last_launch_info()[0]
    assert "tree_kernel" in name and name.rstrip(">").split(", ")[3] == str(store), name
    assert launched_gangs() == gang, name
    assert np.array_equal(got, want), (algo, p, B)


@pytest.mark.parametrize("algo", ["sparbit", "recursive_doubling", "ring"])
def test_long_blocks_off_the_64_kib_boundaries_are_cut_by_the_address_grid(torch, algo):
    """Blocks on the lines whose length is not a multiple of 64 KiB, in rows that are: AUTO cuts them by the 1 KiB grid
    of addresses (the any-alignment form) and counts a gang's pieces from the grid's 64 KiB boundaries, so the groups
    at a block's two ends are part empty.  Ring keeps the cut from the block's start.  Every byte against the oracle."""
    a = {"sparbit": sb.SPARBIT, "ring": sb.RING, "recursive_doubling": sb.RECURSIVE_DOUBLING}[algo]
    p = 32 if algo == "recursive_doubling" else 24
    B = (1 << 20) + (8 << 10)
    assert p * B % 65536 == 0 and B % 65536 != 0
    announce("cut by the address grid", algo, p, B)
    send = workloads.make_send_raw(p, B, seed=p + 6)
    want = oracle_result(a, p, B, send)
    got = gpu_result(torch, a, p, B, send, sb.MODE_AUTO)
    name = sb.sparbit_last_launch_info()[0]
    assert launched_gangs() == 4, name
    assert launched_any_alignment_form() == (algo != "ring"), name
    assert np.array_equal(got, want), (algo, p, B)


@pytest.mark.parametrize("gang", [1, 8])
@pytest.mark.parametrize("store", [1, 4])
def test_gangs_of_wavefronts(torch, store, gang):
    """Workgroups of 4 wavefronts whose pieces lie 32 KiB apart and that meet at a barrier before every run: forced
    onto blocks of less than one group of 128 pieces (wavefronts without a piece), of whole groups, of groups and a
    ragged rest, with a last piece of a few bytes; rank counts around the run length, in place, Recursive Doubling,
    the any-alignment form, Ring's chain, and where the form does not allow gangs (teams, narrow accesses, Ring off
    the lines).  The same with gangs of 8 asked for, which exist for equal blocks of whole vectors in store form 4
    and for the chain (elsewhere gangs of 4 run), with the pieces 4, 16 and 32 KiB apart."""
    sb.sparbit_tune("tree_gang", gang)
    sb.sparbit_tune("tree_store", store)
    sb.sparbit_tune("tree_small_bytes", 0)
    size = 8 if gang == 8 and store == 4 else 4
    if gang == 8:
        for apart_log2, p, B in ((2, 5, 32 * 1024), (2, 19, 33 * 1024 + 128), (4, 10, 128 * 1024), (4, 65, 129 * 1024), (5, 3, 256 * 1024)):
            sb.sparbit_tune("tree_gang_apart_log2", apart_log2)
            announce("gangs of 8, apart", store, apart_log2, p, B)
            send = workloads.make_send_raw(p, B, seed=p + apart_log2)
            want = oracle_result(sb.SPARBIT, p, B, send)
            got = gpu_result(torch, sb.SPARBIT, p, B, send, sb.MODE_TREE)
            assert launched_gangs() == size, sb.sparbit_last_launch_info()
            assert np.array_equal(got, want), (apart_log2, p, B)
        sb.sparbit_tune("tree_gang_apart_log2", -1)
    for p, B in ((1, 4096), (2, 16), (3, 1024 + 128), (5, 33 * 1024), (7, 128 * 1024), (8, 160 * 1024 + 384), (9, 64 * 1024),
                 (16, 256 * 1024), (17, 100 * 1024 + 128), (21, 31 * 1024 + 256), (33, 130 * 1024), (64, 96 * 1024),
                 (65, 32 * 1024 + 128), (96, 1024), (129, 4096), (257, 2048 + 128)):  # whole lines, or under 512 bytes
        for in_place in (False, True):
            announce("gangs", store, p, B, in_place)
            send = workloads.make_send_raw(p, B, seed=p + B % 97)
            want = oracle_result(sb.SPARBIT, p, B, send, in_place=in_place)
            got = gpu_result(torch, sb.SPARBIT, p, B, send, sb.MODE_TREE, in_place=in_place)
            if not (p == 1 and in_place):
                assert launched_gangs() == size, sb.sparbit_last_launch_info()
            assert np.array_equal(got, want), (p, B, in_place)
    for p, B in ((4, 64 * 1024), (32, 40 * 1024 + 128), (128, 1024)):
        announce("gangs, doubling", store, p, B)
        send = workloads.make_send_raw(p, B, seed=p)
        want = oracle_result(sb.RECURSIVE_DOUBLING, p, B, send)
        got = gpu_result(torch, sb.RECURSIVE_DOUBLING, p, B, send, sb.MODE_TREE)
        assert launched_gangs() == size and launched_doubling_form(), sb.sparbit_last_launch_info()
        assert np.array_equal(got, want), (p, B)
    for p, B, mis in ((9, 4100, 0), (3, 1040, 0), (7, 33 * 1024 + 1, 0), (32, 70 * 1024 + 4, 0), (33, 40 * 1024 + 16, 3), (64, 512, 1),
                      (128, 3 * 1024 + 1, 0), (16, 200 * 1024 + 8, 0),
                      # rows a multiple of 1 KiB: a gang's pieces counted from a boundary of the address grid
                      (32, 70 * 1024 + 32, 0), (16, 200 * 1024 + 64, 5), (128, 3 * 1024 + 8, 3), (64, 64 * 1024 + 16, 200), (8, 128 + 1024 * 1024, 64)):
        announce("gangs, any alignment", store, p, B, mis)
        send = workloads.make_send_raw(p, B, seed=p + 1)
        want = oracle_result(sb.SPARBIT, p, B, send)
        got = gpu_result(torch, sb.SPARBIT, p, B, send, sb.MODE_TREE, misalign=mis)
        # rows off the lines store plain, which form 4 does not do: form 0 then, one wavefront per workgroup
        assert launched_gangs() == (4 if store == 1 or p * B % 128 == 0 else 0) and launched_any_alignment_form(), sb.sparbit_last_launch_info()
        assert np.array_equal(got, want), (p, B, mis)
    for p, B, in_place in ((2, 1024, False), (9, 4096, False), (17, 33 * 1024, True), (40, 130 * 1024 + 128, False), (131, 2048, False)):
        announce("gangs, ring", store, p, B, in_place)
        send = workloads.make_send_raw(p, B, seed=p + 2)
        want = oracle_result(sb.RING, p, B, send, in_place=in_place)
        got = gpu_result(torch, sb.RING, p, B, send, sb.MODE_TREE, in_place=in_place)
        name = sb.sparbit_last_launch_info()[0]
        assert launched_gangs() == (8 if gang == 8 else 4) and name.rstrip(">").split(", ")[7] == "2", name
        assert np.array_equal(got, want), (p, B, in_place)
    for algo, p, B, knobs in ((sb.SPARBIT, 9, 20, {}), (sb.SPARBIT, 9, 500, {}), (sb.RING, 9, 4100, {}),
                              (sb.SPARBIT, 64, 1024, {"tree_team_log2": 2, "tree_store": 2})):
        for k, v in knobs.items():
            sb.sparbit_tune(k, v)
        announce("no gangs here", algo, p, B)
        send = workloads.make_send_raw(p, B, seed=p)
        want = oracle_result(algo, p, B, send)
        got = gpu_result(torch, algo, p, B, send, sb.MODE_TREE)
        assert not launched_gangs(), sb.sparbit_last_launch_info()
        assert np.array_equal(got, want), (algo, p, B)


def launched_doubling_form():
    name = sb.sparbit_last_launch_info()[0]
    args = name.rstrip(">").split(", ")
    return "tree_kernel" in name and args[7] == "1"  # access type, U, NB, store, look-ahead, sizes, any, walk, team, gang


@pytest.mark.parametrize("knobs", [{}, {"tree_store": 0, "tree_lds_bytes": 0}, {"tree_team_log2": 0}, {"tree_team_log2": 1},
                                   {"tree_team_log2": 2, "tree_store": 0}, {"tree_team_log2": 4}, {"tree_hot": 1},
                                   {"tree_store": 4, "tree_small_bytes": 0}])
def test_recursive_doubling_in_the_tree_form(torch, knobs):
    """Recursive Doubling seen by block is a binomial tree as well (relative rank = rank xor origin, a rank forwards
    in every step after the one it received in); the same one-launch form walks it in step order, or, in store forms
    1 and 4, like Sparbit's tree with the bits of the relative rank reversed.  Every power of
    two up to 256, blocks on and off the grids, in place, explicit mode and AUTO; one wavefront per piece and teams of
    2 .. 16 (the tree split by the low bits of the relative rank)."""
    for k, v in knobs.items():
        sb.sparbit_tune(k, v)
    for p in (1, 2, 4, 8, 16, 32, 64, 128, 256):
        for B, mis in ((16, 0), (1040, 0), (20, 0), (333, 1), (4100, 0), (4096, 4), (65552, 0)) if p <= 64 else ((1040, 0), (516, 0)):
            for mode, in_place in ((sb.MODE_TREE, False), (sb.MODE_AUTO, False), (sb.MODE_TREE, True)):
                announce("doubling tree", knobs, p, B, mis, mode, in_place)
                send = workloads.make_send_raw(p, B, seed=p + B)
                want = oracle_result(sb.RECURSIVE_DOUBLING, p, B, send, in_place=in_place)
                got = gpu_result(torch, sb.RECURSIVE_DOUBLING, p, B, send, mode, in_place=in_place, misalign=mis)
                if not (p == 1 and in_place):  # one rank in place: nothing moves, nothing is launched
                    assert launched_doubling_form(), sb.sparbit_last_launch_info()
                assert np.array_equal(got, want), (p, B, mis, mode, in_place)
    with pytest.raises(sb.SparbitError) as e:  # not a power of two: no such schedule, in any form
        d = torch.full((8192,), POISON, dtype=torch.uint8, device="cuda:0")
        sb.sparbit_allgather_mode(d[:96], d[1024:], 6, 16, sb.RECURSIVE_DOUBLING, sb.MODE_TREE)
    assert e.value.code == -3


def test_recursive_doubling_in_the_tree_form_at_full_size(torch):
    """cfg4's shape (128 ranks x 1 MiB, 16 GiB of receive buffers) as AUTO issues Recursive Doubling: every rank's
    receive buffer is compared on the device with the Allgather definition (the final state the oracle's Recursive
    Doubling is pinned to), sampled slots on the host."""
    w = workloads.WORKLOADS["cfg4"]
    p, B = w.p, w.block_bytes
    announce("doubling tree at full size", p, B)
    send = workloads.make_send(w)
    dev = torch.device("cuda:0")
    d_send = torch.from_numpy(send).to(dev)
    d_recv = torch.full((p, p, B), POISON, dtype=torch.uint8, device=dev)
    sb.sparbit_allgather_mode(d_send, d_recv, p, B, sb.RECURSIVE_DOUBLING, sb.MODE_AUTO)
    torch.cuda.synchronize()
    assert launched_doubling_form(), sb.sparbit_last_launch_info()
    assert ", 8, 4, true, " in sb.sparbit_last_launch_info()[0]  # walked like Sparbit's tree, bits reversed
    for r in range(p):
        assert torch.equal(d_recv[r], d_send), r
    small = workloads.make_send_raw(p, 4, seed=3)
    want = oracle_result(sb.RECURSIVE_DOUBLING, p, 4, small)  # slot k of every rank holds rank k's block
    assert all(np.array_equal(want[r], small) for r in range(p))
    rng = np.random.default_rng(5)
    for r, k in zip(rng.integers(0, p, 16), rng.integers(0, p, 16)):
        assert np.array_equal(d_recv[r, k].cpu().numpy(), send.reshape(p, B)[k])


def test_ring_in_the_tree_form(torch):
    """Ring seen by block is a chain (relative rank rho forwards to rho + 1): the same one-launch form stores a rank
    and reads it back, p - 1 times, with plain stores whatever the store setting.  Explicit mode and AUTO, blocks on
    and off the grids, in place."""
    for p in (1, 2, 3, 5, 8, 21, 33, 64, 96, 257):
        for B, mis in ((16, 0), (1040, 0), (100, 0), (333, 1), (4100, 0), (4096, 4)) if p <= 64 else ((1040, 0), (516, 0)):
            for mode, in_place in ((sb.MODE_TREE, False), (sb.MODE_AUTO, False), (sb.MODE_TREE, True)):
                announce("ring chain", p, B, mis, mode, in_place)
                send = workloads.make_send_raw(p, B, seed=p + B)
                want = oracle_result(sb.RING, p, B, send, in_place=in_place)
                got = gpu_result(torch, sb.RING, p, B, send, mode, in_place=in_place, misalign=mis)
                name = sb.sparbit_last_launch_info()[0]
                if not (p == 1 and in_place):
                    assert "tree_kernel" in name and name.rstrip(">").split(", ")[7] == "2" and ", 8, 0, " in name, name
                assert np.array_equal(got, want), (p, B, mis, mode, in_place)


def test_refusals(torch):
    """The tree form exists for the schedules whose messages, seen by block, form a tree that ends in the block's own
    slot at every rank: Sparbit, Recursive Doubling and Ring.  Bruck (rotated working buffer), DIRECT, and step ranges
    are refused."""
    d = torch.full((4096,), POISON, dtype=torch.uint8, device="cuda:0")
    for algo in (sb.BRUCK, sb.DIRECT):
        with pytest.raises(sb.SparbitError) as e:
            sb.sparbit_allgather_mode(d[:64], d[1024:], 4, 16, algo, sb.MODE_TREE)
        assert e.value.code == -3
    torch.cuda.synchronize()
    assert bool((d == POISON).all())


def test_capture_records_the_tree_launch_and_needs_no_tables(torch):
    """The tree kernel has no table, flag or state, so an AUTO call can be recorded into a HIP graph even when
    the library has never seen its (schedule, p); every replay must reproduce the oracle's result, with eager
    work and synchronisation in between."""
    w = workloads.WORKLOADS["cfg3"]
    p, B = w.p, w.block_bytes
    send = workloads.make_send(w)
    want = oracle_result(sb.SPARBIT, p, B, send)
    d_send, d_recv, _ = gpu_buffers(torch, p, B, send)
    sb.sparbit_finalize()  # no cached tables at all
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            sb.sparbit_allgather(d_send, d_recv, p, B, torch.cuda.current_stream())
    for rep in range(3):
        d_recv.fill_(POISON)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(d_recv.cpu().numpy().reshape(p, p, B), want), rep


def test_capture_of_a_call_in_gangs_of_8(torch):
    """A gang of 8 reserves more LDS than a kernel may ask for by default; the limit is raised outside the stream, so
    such a launch can be recorded too, and every replay reproduces the oracle's result."""
    p, B = 64, 128 << 10
    send = workloads.make_send_raw(p, B, seed=8)
    want = oracle_result(sb.SPARBIT, p, B, send)
    d_send, d_recv, _ = gpu_buffers(torch, p, B, send)
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            sb.sparbit_allgather(d_send, d_recv, p, B, torch.cuda.current_stream())
    assert launched_gangs() == 8, sb.sparbit_last_launch_info()
    for rep in range(3):
        d_recv.fill_(POISON)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(d_recv.cpu().numpy().reshape(p, p, B), want), rep


def test_many_streams_at_once(torch):
    """Nothing in the tree form waits for another workgroup, so any number of calls may run side by side."""
    cases = [(96, 4096), (64, 16384), (125, 512), (32, 65536), (12, 1024), (257, 1040)]
    streams = [torch.cuda.Stream() for _ in cases]
    jobs = []
    for i, (p, B) in enumerate(cases):
        send = workloads.make_send_raw(p, B, seed=90 + i)
        want = torch.from_numpy(oracle_result(sb.SPARBIT, p, B, send)).to("cuda:0")
        jobs.append((p, B, *gpu_buffers(torch, p, B, send), want))
    torch.cuda.synchronize()
    for rep in range(5):
        for st, (p, B, d_send, d_recv, _, _) in zip(streams, jobs):
            sb.sparbit_allgather_mode(d_send, d_recv, p, B, sb.SPARBIT, sb.MODE_TREE, st)
    torch.cuda.synchronize()
    for p, B, _, d_recv, _, want in jobs:
        assert torch.equal(d_recv.view(p, p, B), want), (p, B)

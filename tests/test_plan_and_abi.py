"""Host-side tests of the C-ABI library: it loads, exports every symbol the
header declares, rejects bad arguments without touching a GPU, and its schedule
tables reproduce the message log of the CPU oracle (two independent
derivations: the library builds tables from the stripe/comb closed form, the
oracle runs Algorithm 1's bit-mask loop per rank)."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2109_08751_amd as sb
from paper_2109_08751_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "sparbit.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sparbit_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert {"sparbit_allgather", "sparbit_allgather_algo", "sparbit_allgather_steps",
            "sparbit_plan_create", "sparbit_finalize", "sparbit_strerror"} <= set(names)
    L = ctypes.CDLL(sb.lib_path())
    for n in names:
        assert hasattr(L, n), n


def test_binding_names_match_header():
    for n in declared_symbols():
        if n.startswith("sparbit_plan_") or n == "sparbit_last_hip_error":
            continue  # wrapped by binding.Plan / SparbitError
        assert hasattr(binding, n), n


def test_bad_arguments_are_rejected_on_the_host():
    """None of these reaches a HIP call, so they run without a GPU."""
    L = binding.lib
    fake_send, fake_recv = 0x1000, 0x100000
    assert L.sparbit_allgather(fake_send, fake_recv, 0, 16, None) == -1
    assert L.sparbit_allgather(fake_send, fake_recv, 4, 0, None) == 0  # zero count: nothing to do
    assert L.sparbit_allgather_steps(fake_send, fake_recv, 4, 0, 0, 0, 5, None) == -1
    assert L.sparbit_allgather(fake_send, None, 4, 16, None) == -1
    assert L.sparbit_allgather(fake_send, fake_recv, 40000, 16, None) == -1
    assert L.sparbit_allgather_algo(fake_send, fake_recv, 4, 16, 9, None) == -1
    assert L.sparbit_allgather_mode(fake_send, fake_recv, 4, 16, 0, 7, None) == -1
    # overlapping send / recv ranges
    assert L.sparbit_allgather(fake_recv + 32, fake_recv, 4, 16, None) == -2
    assert L.sparbit_allgather(fake_recv - 16, fake_recv, 4, 16, None) == -2
    # Recursive Doubling needs a power of two; Bruck has no in-place form
    assert L.sparbit_allgather_algo(fake_send, fake_recv, 6, 16, sb.RECURSIVE_DOUBLING, None) == -3
    assert L.sparbit_allgather_algo(None, fake_recv, 6, 16, sb.BRUCK, None) == -3
    # p * p * block_bytes must not overflow
    assert L.sparbit_allgather(fake_send, fake_recv, 4096, 1 << 62, None) == -1
    for code in (0, -1, -2, -3, -4, -5, -99):
        assert sb.sparbit_strerror(code)
    with pytest.raises(sb.SparbitError):
        sb.Plan(0)
    with pytest.raises(sb.SparbitError):
        sb.Plan(12, sb.RECURSIVE_DOUBLING)
    with pytest.raises(sb.SparbitError):
        sb.sparbit_tune("no_such_knob", 1)
    with pytest.raises(sb.SparbitError):
        sb.sparbit_tune("wg_threads", 1000)
    for value in (2, 3, 5, 16, -2):  # wavefronts per gang: 4 or 8 (1: 4; 0: none; -1: by the call)
        with pytest.raises(sb.SparbitError):
            sb.sparbit_tune("tree_gang", value)
    for value in (0, 1, 4, 8, -1):
        sb.sparbit_tune("tree_gang", value)


ORACLE_ALGO = {sb.SPARBIT: oracle.SPARBIT, sb.RING: oracle.RING,
               sb.RECURSIVE_DOUBLING: oracle.RECURSIVE_DOUBLING, sb.BRUCK: oracle.BRUCK}


def oracle_trace(algo, p):
    send = np.arange(p, dtype=np.int32).view(np.uint8).reshape(p, 4)
    recv = np.full((p, p, 4), 0xA5, dtype=np.uint8)
    return oracle.allgather(ORACLE_ALGO[algo], p, 4, send, recv, -1, want_trace=True)


def check_plan_against_oracle(algo, p):
    run = oracle_trace(algo, p)
    plan = sb.Plan(p, algo)
    assert plan.num_steps == run.steps_run == oracle.num_steps(ORACLE_ALGO[algo], p)
    for s in range(plan.num_steps):
        st = plan.step(s)
        t = run.trace[run.trace[:, 0] == s]
        d, ign, n = run.step_info[s]
        assert (st["distance"], st["nblocks"]) == (d, n)
        if algo == sb.SPARBIT:
            assert st["ignore"] == ign
        assert len(t) == p * n
        # the library's messages as (src, dst, src_slot, dst_slot), j-th send -> j-th receive
        r = np.repeat(np.arange(p, dtype=np.int32), n)
        dst = st["dst"][r]
        j = np.tile(np.arange(n), p)
        mine = np.stack([r, dst, st["send_slot"].reshape(-1), st["recv_slot"][dst, j]], axis=1)
        theirs = t[:, 1:5]
        key = lambda a: a[np.lexsort((a[:, 3], a[:, 2], a[:, 1], a[:, 0]))]
        assert np.array_equal(key(mine), key(theirs)), (algo, p, s)
        assert np.array_equal(st["src"][st["dst"]], np.arange(p))
    plan.close()


@pytest.mark.parametrize("p", list(range(1, 70)) + [96, 127, 128, 129, 200, 255, 256, 257, 300])
def test_sparbit_plan_reproduces_oracle_message_log(p):
    check_plan_against_oracle(sb.SPARBIT, p)


@pytest.mark.parametrize("p", [1, 2, 3, 6, 17, 64, 96, 257])
def test_context_plans_reproduce_oracle_message_log(p):
    check_plan_against_oracle(sb.RING, p)
    check_plan_against_oracle(sb.BRUCK, p)
    if p & (p - 1) == 0:
        check_plan_against_oracle(sb.RECURSIVE_DOUBLING, p)


@pytest.mark.parametrize("p,want", [
    (6, [1, 1, 3]), (64, [1, 2, 4, 8, 16, 32]), (96, [1, 1, 3, 6, 12, 24, 48]),
    (128, [1, 2, 4, 8, 16, 32, 64]), (257, [1, 1, 2, 4, 8, 16, 32, 64, 128])])
def test_blocks_per_step_of_the_five_configs(p, want):
    """Regression values; each list sums to p - 1 (the bandwidth-optimal volume
    of the cost formula in Section III-B) and has ceil(log2 p) entries."""
    plan = sb.Plan(p)
    got = [plan.step(s)["nblocks"] for s in range(plan.num_steps)]
    assert got == want and sum(got) == p - 1 and len(got) == (p - 1).bit_length()
    # and the oracle agrees
    assert oracle_trace(sb.SPARBIT, p).step_info[:, 2].tolist() == want


def test_direct_plan_has_no_steps():
    assert sb.Plan(7, sb.DIRECT).num_steps == 0


def test_plan_at_the_maximum_rank_count():
    """p = SPARBIT_MAX_P: 12 steps, blocks per step from the comb closed form, p - 1 in total;
    one more rank is refused."""
    plan = sb.Plan(4096)
    got = [plan.step(s)["nblocks"] for s in range(plan.num_steps)]
    assert got == [2 ** s for s in range(12)] and sum(got) == 4095
    last = plan.step(11)
    assert last["distance"] == 1 and last["send_slot"].shape == (4096, 2048)
    assert np.array_equal(last["send_slot"][5, :3], [5, 3, 1])
    plan.close()
    with pytest.raises(sb.SparbitError):
        sb.Plan(4097)


def test_every_tuning_key_is_documented_in_the_header():
    """The keys sparbit_tune accepts (read off the source) and the keys the header lists are the same set, and an
    unknown key is an argument error."""
    import re
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    api = open(os.path.join(root, "paper_2109_08751_amd", "csrc", "api.hip")).read()
    hdr = open(os.path.join(root, "include", "sparbit.h")).read()
    accepted = set(re.findall(r'std::strcmp\(key, "([a-z0-9_]+)"\)', api))
    documented = set(re.findall(r'^ \*   "([a-z0-9_]+)"', hdr, re.M))
    assert accepted and accepted == documented, (sorted(accepted - documented), sorted(documented - accepted))
    with pytest.raises(sb.SparbitError) as e:
        sb.sparbit_tune("no_such_key", 1)
    assert e.value.code == -1

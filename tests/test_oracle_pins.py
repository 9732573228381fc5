"""Pins for the CPU oracle against what the paper and the mathematics fix.

None of these retypes the oracle's formulas: they use the Allgather definition
(Section II), the worked examples printed in Section III-B, the closed forms of
Section II-A / III-B, an independent simulation of the paper's *conceptual*
definition (p rank-shifted binomial trees, Section III-A/B) and planted
mistakes that the pins must catch.
"""
import os
import subprocess
import sys

import numpy as np
import pytest

import oracle
from paper_2109_08751_amd import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
POISON = workloads.POISON


def ceil_log2(p):
    return (p - 1).bit_length()


def run(algo, p, B, max_steps=-1, seed=1, in_place=False, want_trace=False, lib=oracle):
    send = workloads.make_send_raw(p, B, seed)
    recv = np.full((p, p, B), POISON, dtype=np.uint8)
    if in_place:
        for r in range(p):
            recv[r, r] = send[r]
    info = lib.allgather(algo, p, B, None if in_place else send, recv, max_steps, want_trace)
    return send, recv, info


def tagged_state(algo, p, max_steps=-1):
    """Which block sits in which slot: blocks are 4-byte rank tags, -1 = never written."""
    send = np.arange(p, dtype=np.int32).view(np.uint8).reshape(p, 4)
    recv = np.full((p, p), -1, dtype=np.int32)
    info = oracle.allgather(algo, p, 4, send, recv.view(np.uint8).reshape(p, p, 4), max_steps)
    return recv, info


# ---------------------------------------------------------------- definition
ALL_P = list(range(1, 34)) + [64, 96, 128, 257]


@pytest.mark.parametrize("p", ALL_P)
def test_sparbit_equals_allgather_definition(p):
    """Section II: block j ends in slot j of every receive buffer -- brute force
    against the plain all-to-all copy for every p in 1..33 and the config sizes."""
    for B in (1, 3, 16):
        send, recv, info = run(oracle.SPARBIT, p, B, seed=p * 7 + B)
        want = np.empty_like(recv)
        oracle.naive_allgather(p, B, send, want)
        assert np.array_equal(want, np.broadcast_to(send[None], (p, p, B)))  # definition itself
        assert np.array_equal(recv, want)
        assert info.steps_run == ceil_log2(p)


@pytest.mark.parametrize("p", [1, 2, 5, 6, 21, 64])
def test_sparbit_in_place(p):
    send, recv, _ = run(oracle.SPARBIT, p, 8, in_place=True)
    assert np.array_equal(recv, np.broadcast_to(send[None], (p, p, 8)))


@pytest.mark.parametrize("p", [1000, 2049])
def test_sparbit_large_p(p):
    recv, info = tagged_state(oracle.SPARBIT, p)
    assert np.array_equal(recv, np.broadcast_to(np.arange(p, dtype=np.int32)[None], (p, p)))
    assert info.steps_run == ceil_log2(p)
    assert (info.sent_per_rank == p - 1).all()


# ---------------------------------------------------------------- cost model
@pytest.mark.parametrize("p", ALL_P)
def test_sparbit_cost_terms(p):
    """C = ceil(log2 p) alpha + (p-1)(m/p) beta (Section III-B): step count and
    exactly p-1 blocks sent and received by every rank."""
    _, _, info = run(oracle.SPARBIT, p, 2, want_trace=True)
    assert info.steps_run == ceil_log2(p) == oracle.num_steps(oracle.SPARBIT, p)
    assert (info.sent_per_rank == p - 1).all()
    if p > 1:
        recvd = np.bincount(info.trace[:, 2], minlength=p)
        assert (recvd == p - 1).all()
        # every one of the p*p slots written exactly once: p own + p(p-1) deliveries
        keys = info.trace[:, 2].astype(np.int64) * p + info.trace[:, 4]
        assert len(np.unique(keys)) == p * (p - 1)
        assert not (info.trace[:, 2] == info.trace[:, 4]).any()  # own slot never overwritten


@pytest.mark.parametrize("p", [2, 4, 8, 16, 32, 64, 128, 256])
def test_power_of_two_closed_form(p):
    """Section III-B: with p a power of two, on step s every process sends and
    receives 2^s blocks to/from peers 2^(log2 p - (s+1)) away."""
    _, _, info = run(oracle.SPARBIT, p, 1, want_trace=True)
    L = ceil_log2(p)
    for s in range(L):
        d, ign, n = info.step_info[s]
        assert (d, ign, n) == (2 ** (L - (s + 1)), 0, 2 ** s)
        t = info.trace[info.trace[:, 0] == s]
        assert ((t[:, 2] - t[:, 1]) % p == d).all()
        assert (np.bincount(t[:, 1], minlength=p) == 2 ** s).all()
        assert (np.bincount(t[:, 2], minlength=p) == 2 ** s).all()


# ---------------------------------------------------------------- worked examples
def _read_fig3():
    steps, never = [], None
    for line in open(os.path.join(GOLDEN, "fig3_p5.txt")):
        tok = line.split()
        if not tok or tok[0].startswith("#"):
            continue
        if tok[0] == "p":
            p = int(tok[1])
        elif tok[0] == "step":
            steps.append((int(tok[1]), int(tok[3]), int(tok[5]), [int(x) for x in tok[7:]]))
        elif tok[0] == "never_forwarded":
            never = int(tok[1])
    return p, steps, never


def test_worked_example_five_processes():
    """Figure 3 and its walk-through (Section III-B)."""
    p, steps, never = _read_fig3()
    assert oracle.num_steps(oracle.SPARBIT, p) == len(steps)
    for s, d, sent, held in steps:
        recv, info = tagged_state(oracle.SPARBIT, p, max_steps=s + 1)
        assert tuple(info.step_info[s][[0, 2]]) == (d, sent)
        for r in range(p):
            want = np.full(p, -1, dtype=np.int32)
            for off in held:
                want[(r + off) % p] = (r + off) % p
            assert np.array_equal(recv[r], want), (s, r)
    _, _, info = run(oracle.SPARBIT, p, 1, want_trace=True)
    for r in range(p):
        mine = info.trace[info.trace[:, 1] == r]
        assert (r + never) % p not in set(mine[:, 3])
        # step 0 sends the original block to r+4; it arrives from r-4
        first = mine[mine[:, 0] == 0]
        assert first[:, 2].tolist() == [(r + 4) % p] and first[:, 3].tolist() == [r]


def _read_subtrees():
    out = []
    for line in open(os.path.join(GOLDEN, "subtrees.txt")):
        tok = line.split()
        if not tok or tok[0].startswith("#"):
            continue
        i_sub, i_all, i_ign = tok.index("subtrees"), tok.index("all"), tok.index("ignore")
        out.append((int(tok[1]), [int(x) for x in tok[i_sub + 1:i_all]],
                    [int(x) for x in tok[i_all + 1:i_ign]], [int(x) for x in tok[i_ign + 1:]]))
    return out


@pytest.mark.parametrize("p,subtrees,send_all,ignore", _read_subtrees())
def test_subtree_examples(p, subtrees, send_all, ignore):
    assert sum(subtrees) == p
    _check_expansion_rule(p, set(send_all), set(ignore))


def _check_expansion_rule(p, send_all, ignore):
    """On a send-all step a process sends every block it holds, on an ignore
    step all but one (Section III-B, tree expansion)."""
    L = ceil_log2(p)
    assert send_all | ignore == {2 ** i for i in range(L)}
    for s in range(L):
        before, _ = tagged_state(oracle.SPARBIT, p, max_steps=s)
        _, info = tagged_state(oracle.SPARBIT, p, max_steps=s + 1)
        d, ign, n = info.step_info[s]
        held = (before >= 0).sum(axis=1)
        assert (held == held[0]).all()
        if d in send_all:
            assert ign == 0 and n == held[0]
        else:
            assert d in ignore and ign == 1 and n == held[0] - 1


@pytest.mark.parametrize("p", list(range(2, 70)) + [96, 100, 257, 320])
def test_expansion_rule_from_binary_representation(p):
    """Section III-B prose: sub-tree sizes are the powers of two composing p;
    expansions (send everything) happen on all of them but the smallest, and on
    every distance below the smallest; all other steps ignore a block."""
    L = ceil_log2(p)
    bits = [2 ** i for i in range(p.bit_length()) if p >> i & 1]
    smallest = min(bits)
    send_all = {b for b in bits if b != smallest} | {2 ** i for i in range(L) if 2 ** i < smallest}
    send_all &= {2 ** i for i in range(L)}
    ignore = {2 ** i for i in range(L)} - send_all
    _check_expansion_rule(p, send_all, ignore)


# ---------------------------------------------------------------- binomial trees
def binomial_tree_holders(p):
    """Section III-A: broadcast over relative ranks 0..p-1 that mimics the tree
    of size 2^ceil(log2 p) and drops sends to relative ranks >= p.  Returns, per
    step, the set of relative ranks that hold the root's block afterwards."""
    have, out = {0}, []
    d = 2 ** (ceil_log2(p) - 1) if p > 1 else 0
    while d >= 1:
        have = have | {h + d for h in have if h + d < p}
        out.append(set(have))
        d //= 2
    return out


@pytest.mark.parametrize("p", list(range(2, 34)) + [63, 64, 65, 96, 257])
def test_matches_stripe_parallel_binomial_trees(p):
    """Section III-B: Sparbit = p binomial trees, tree of root t shifted by t
    with wrap-around, all advancing one level per step.  After each step rank
    (t + rel) mod p holds block t iff rel is reached in the tree -- and nothing
    else (unwritten slots stay poison)."""
    per_step = binomial_tree_holders(p)
    for s, rels in enumerate(per_step):
        recv, _ = tagged_state(oracle.SPARBIT, p, max_steps=s + 1)
        want = np.full((p, p), -1, dtype=np.int32)
        for t in range(p):
            for rel in rels:
                want[(t + rel) % p, t] = t
        assert np.array_equal(recv, want), (p, s)
    assert per_step[-1] == set(range(p))


# ---------------------------------------------------------------- context schedules
@pytest.mark.parametrize("p", list(range(1, 34)) + [64, 96, 257])
def test_ring_and_bruck(p):
    """Section II-A: Ring takes p-1 steps of one block; Bruck ceil(log2 p)
    steps, 2^s blocks on step s < floor(log2 p) and p - 2^floor(log2 p) on the
    extra one; both satisfy the Allgather definition."""
    for algo in (oracle.RING, oracle.BRUCK):
        send, recv, info = run(algo, p, 5, seed=p)
        assert np.array_equal(recv, np.broadcast_to(send[None], (p, p, 5)))
        assert (info.sent_per_rank == p - 1).all()
    _, _, ring = run(oracle.RING, p, 1, want_trace=True)
    assert ring.steps_run == p - 1
    assert (ring.step_info[:, 2] == 1).all()
    if p > 1:
        assert ((ring.trace[:, 2] - ring.trace[:, 1]) % p == 1).all()
    _, _, bruck = run(oracle.BRUCK, p, 1, want_trace=True)
    assert bruck.steps_run == ceil_log2(p)
    fl = p.bit_length() - 1
    want = [2 ** s for s in range(fl)] + ([p - 2 ** fl] if p != 2 ** fl else [])
    assert bruck.step_info[:, 2].tolist() == want
    for s in range(bruck.steps_run):
        t = bruck.trace[bruck.trace[:, 0] == s]
        assert ((t[:, 1] - t[:, 2]) % p == 2 ** s % p).all()  # r sends to r - 2^s


@pytest.mark.parametrize("p", [1, 2, 4, 8, 16, 32, 64, 128])
def test_recursive_doubling(p):
    """Section II-A: log2 p steps, pairwise with r xor 2^s, data doubling."""
    send, recv, info = run(oracle.RECURSIVE_DOUBLING, p, 3, want_trace=True)
    assert np.array_equal(recv, np.broadcast_to(send[None], (p, p, 3)))
    assert info.steps_run == ceil_log2(p)
    assert info.step_info[:, 2].tolist() == [2 ** s for s in range(info.steps_run)]
    for s in range(info.steps_run):
        t = info.trace[info.trace[:, 0] == s]
        assert ((t[:, 1] ^ t[:, 2]) == 2 ** s).all()


def test_recursive_doubling_rejects_non_power_of_two():
    assert oracle.num_steps(oracle.RECURSIVE_DOUBLING, 6) == -1
    with pytest.raises(oracle.OracleError):
        run(oracle.RECURSIVE_DOUBLING, 6, 1)


def test_bad_arguments():
    recv = np.zeros(4, dtype=np.uint8)
    with pytest.raises(oracle.OracleError):
        oracle.allgather(oracle.SPARBIT, 0, 1, None, recv)
    with pytest.raises(ValueError):
        oracle.allgather(oracle.SPARBIT, 2, 2, None, recv)


# ---------------------------------------------------------------- payload generator
def test_splitmix64_reference_values():
    """SplitMix64 (Steele, Lea, Flood 2014): outputs of the generator seeded
    with 0 -- its first three published test values."""
    g = 0x9E3779B97F4A7C15
    states = np.array([0, g, (2 * g) % 2 ** 64], dtype=np.uint64)
    got = workloads.splitmix64(states)
    assert [int(x) for x in got] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_workload_shapes():
    for name, w in workloads.WORKLOADS.items():
        blk = workloads.make_block(w.kind, 3, min(w.block_bytes, 4096))
        assert blk.dtype == np.uint8 and blk.size == min(w.block_bytes, 4096)
    u = workloads.make_block("f32_uniform", 1, 4096).view(np.float32)
    assert (u >= -1).all() and (u < 1).all()
    n = workloads.make_block("f32_normal", 1, 1 << 16).view(np.float32)
    assert np.isfinite(n).all() and abs(float(n.mean())) < 0.05 and abs(float(n.std()) - 1) < 0.05
    assert workloads.WORKLOADS["cfg4"].recv_bytes == 16 << 30


# ---------------------------------------------------------------- planted mistakes
MUTATIONS = [
    ("never keep a block back", "sparbit_forwards_everything(p, d) ? 0 : 1;", "sparbit_forwards_everything(p, d) ? 0 : 0;"),
    ("send slot sign", "origin = (long long)rank - 2LL * j * d;", "origin = (long long)rank + 2LL * j * d;"),
    ("recv slot off by d", "(int)mod_ll(origin - d, p));", "(int)mod_ll(origin - 2LL * d, p));"),
    ("send peer direction", "ahead = (int)mod_ll((long long)rank + d, p);", "ahead = (int)mod_ll((long long)rank - d, p);"),
    ("held blocks overcounted", "stripes = blocks_held(s, rank) - keep_back;", "stripes = blocks_held(s, rank) + 1 - keep_back;"),
    ("smallest sub-tree expands", "    if (d == smallest_subtree)\n        return 0;", "    if (d == smallest_subtree)\n        return 1;"),
    ("missing sub-tree expands", "    return (p & d) != 0;", "    return 1;"),
    ("keeps back below the smallest sub-tree", "    if (d < smallest_subtree)\n        return 1;", "    if (d < smallest_subtree)\n        return 0;"),
    ("distance starts one level low", "sparbit_d = 1 << (nsteps - 1);", "sparbit_d = 1 << (nsteps - 2);"),
    ("distance does not halve", "        sparbit_d /= 2;", "        sparbit_d /= 1;"),
]


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_pins_catch_planted_mistake(tmp_path, name, old, new):
    """A mistake planted in a copy of the oracle's source must trip the
    definition pin (wrong bytes) or the oracle's own protocol checks."""
    src = open(os.path.join(os.path.dirname(oracle.__file__), "sparbit_oracle.c")).read()
    assert src.count(old) == 1, name
    c = tmp_path / "mutant.c"
    so = tmp_path / "mutant.so"
    c.write_text(src.replace(old, new))
    subprocess.check_call(["gcc", "-std=c11", "-O1", "-fPIC", "-shared", str(c), "-o", str(so)])
    code = f"""
import ctypes, sys, numpy as np
lib = ctypes.CDLL({str(so)!r})
lib.oracle_allgather.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_size_t] + [ctypes.c_void_p] * 2 + \
    [ctypes.c_int] + [ctypes.c_void_p] * 3 + [ctypes.c_size_t, ctypes.c_void_p]
bad = 0
for p in range(2, 34):
    send = (np.arange(p * 2, dtype=np.uint8) * 7 + 1).reshape(p, 2)
    recv = np.full((p, p, 2), {POISON}, dtype=np.uint8)
    rc = lib.oracle_allgather(0, p, 2, send.ctypes.data, recv.ctypes.data, -1, None, None, None, 0, None)
    if rc != 0 or not np.array_equal(recv, np.broadcast_to(send[None], (p, p, 2))):
        bad += 1
print(bad)
"""
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=120)
    # a mutant may also crash outright (e.g. a negative shift): that counts as caught
    caught = out.returncode != 0 or int(out.stdout.strip() or 0) > 0
    assert caught, name

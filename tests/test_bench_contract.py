"""bench.py's command-line contract that can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    out = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert out.returncode != 0
    assert "one GPU" in out.stderr and out.stdout.strip() == ""


def test_help_lists_the_contract_flags():
    out = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--help"],
                         capture_output=True, text=True, timeout=120)
    assert out.returncode == 0
    for flag in ("--gpus", "--steps", "--warmup", "--sweep", "--calibrate-copy"):
        assert flag in out.stdout


def _bench():
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_algorithmic_bytes_per_form():
    """One launch per step moves every delivered byte twice, the tree form once plus the send buffer, Recursive
    Doubling's tree form additionally reads every forwarder below p/2 from memory."""
    b = _bench()
    p, B = 128, 1 << 20
    assert b.algorithmic_bytes("per_step", p, B) == 2 * p * p * B
    assert b.algorithmic_bytes("tree", p, B) == p * p * B + p * B
    assert b.algorithmic_bytes("direct", p, B) == p * p * B + p * B
    assert b.algorithmic_bytes("tree_doubling", p, B) == p * p * B + p * B + (p // 2 - 1) * p * B


def test_forms_are_read_off_the_kernel_name():
    b = _bench()
    tree = "sparbit::tree_kernel<unsigned int __vector(4), 1, 8, 2, true, false, false, 0, false, 1>"
    anyal = "sparbit::tree_kernel<unsigned int __vector(4), 1, 8, 2, true, false, true, 0, false, 1>"
    doubling = "sparbit::tree_kernel<unsigned int __vector(4), 1, 8, 2, false, false, false, 1, true, 1>"
    chain = "sparbit::tree_kernel<unsigned int __vector(4), 1, 8, 0, false, false, false, 2, false, 1>"
    assert b.form_of(tree) == "tree" and b.form_of(anyal) == "tree" and b.form_of(doubling) == "tree_doubling"
    assert b.form_of(chain) == "tree"  # a chain's re-reads follow their writes at once: the tree form's byte count
    assert b.tree_kernel_flags(anyal) == {"store": 2, "any_alignment": True, "walk": "sparbit", "team": False, "gang": 1}
    assert b.tree_kernel_flags(doubling) == {"store": 2, "any_alignment": False, "walk": "doubling", "team": True, "gang": 1}
    # Recursive Doubling in store forms 1 and 4 is walked like Sparbit's tree: read back at once
    reversed_bits = "sparbit::tree_kernel<unsigned int __vector(4), 1, 8, 4, true, false, false, 1, false, 1>"
    assert b.form_of(reversed_bits) == "tree" and b.tree_kernel_flags(reversed_bits)["store"] == 4
    assert b.form_of("sparbit::copy_tiles_kernel<unsigned int __vector(4), unsigned int, 64, 1, true, false, true>") == "per_step"
    assert b.form_of("anything", "direct") == "direct" and b.form_of("anything", "memcpy_d2d") == "copy"
    for key in b.MEASURED_TRAFFIC:  # the table's kernel names parse, and name the tree kernel without teams
        assert b.form_of(key[1]) == "tree" and not b.tree_kernel_flags(key[1])["team"]


def test_sweep_summary_from_a_small_file(tmp_path):
    import json
    b = _bench()
    rows = []
    for p in (8, 5):
        for B in (1024, 4096):
            for algo, us in (("sparbit", 10.0), ("sparbit_per_step", 20.0), ("ring", 30.0), ("bruck", 15.0),
                             ("recursive_doubling", 12.0), ("recursive_doubling_per_step", 16.0), ("direct", 9.0)):
                if algo.startswith("recursive") and p & (p - 1):
                    continue
                rows.append({"p": p, "block_bytes": B, "algo": algo, "ok": True, "avg_us": us, "min_us": us, "max_us": us,
                             "effective_GBps": p * p * B / us / 1e3})
    name = "sparbit::tree_kernel<unsigned int __vector(4), 1, 8, 0, false, false, true, 0, true, 1>"
    for algo, us in (("sparbit", 11.0), ("sparbit_per_step", 22.0), ("bruck", 16.0)):
        rows.append({"p": 5, "block_bytes": 1025, "algo": algo, "ok": True, "avg_us": us, "min_us": us, "max_us": us,
                     "effective_GBps": 1.0, "off_grid": True, "kernel": name, "rows_on_lines": False})
    path = tmp_path / "ladder.jsonl"
    path.write_text("".join(json.dumps(r) + "\n" for r in rows))
    text = b.sweep_summary(str(path))
    assert f"Cases: {len(rows)}" in text
    assert "Cells won: sparbit 4, ring 0, recursive_doubling 0, bruck 0 of 4." in text
    assert "| 8 | 0.83 | 0.83 |" in text  # Sparbit / Recursive Doubling
    assert "| 8 | 0.75 | 0.75 |" in text  # Recursive Doubling AUTO / per step
    assert "| 5 | 1K+1 | no | tree* | 11 | 22 | 0.50 |  |  | 16 |" in text
    assert "| 8 | 0.33 | 0.33 |" in text  # Sparbit / Ring
    rows[0]["ok"] = False
    path.write_text("".join(json.dumps(r) + "\n" for r in rows))
    try:
        b.sweep_summary(str(path))
        raise RuntimeError("a failed case must not be summarised")
    except AssertionError:
        pass

"""Host-only checks of bench.py's bookkeeping (no GPU): the HBM-traffic figures it reports come from the counter
records under profiles/, and are withheld when the kernel sources differ from the ones the counters were read with."""
import importlib.util
import os
import shutil

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def load_bench():
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_traffic_records_parse_and_are_plausible():
    b = load_bench()
    for op, wl, algorithmic in (("sa_fwd", "qwen3_8b_prefill_32k", 675.4e6), ("sa_bwd", "pretrain_fwdbwd_8k", 539e6)):
        nbytes, source = b.measured_traffic(op, wl)
        # either the record matches the sources in this tree (a figure at or above the algorithmic bytes), or it is
        # withheld with the reason
        assert nbytes is None or algorithmic <= nbytes <= 3 * algorithmic, (op, nbytes)
        assert source


def test_traffic_is_withheld_when_a_kernel_source_changes(tmp_path):
    b = load_bench()
    shutil.copytree(b.CSRC, tmp_path / "csrc", ignore=shutil.ignore_patterns("*.o", "*.tmp"))
    b.CSRC = str(tmp_path / "csrc")
    before, _ = b.measured_traffic("sa_fwd", "qwen3_8b_prefill_32k")
    with open(tmp_path / "csrc" / "sa_fwd_mfma.hip", "a") as f:
        f.write("// edited\n")
    after, why = b.measured_traffic("sa_fwd", "qwen3_8b_prefill_32k")
    assert after is None and "changed" in why
    assert b.measured_traffic("no_such_op", "nowhere")[0] is None
    # (before is a number in a tree whose sources match the record, None otherwise: both are legitimate states)
    assert before is None or before > 0


def test_multi_gpu_request_is_refused():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "ONE GPU" in r.stderr

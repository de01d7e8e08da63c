"""Host-side checks of bench.py that need no GPU: the one-GPU rule and the bookkeeping that ties
stored HBM-traffic figures to the kernel sources they were measured on."""
import importlib.util
import json
import os
import subprocess
import sys


def load_bench(repo_root):
    spec = importlib.util.spec_from_file_location("bench", os.path.join(repo_root, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_more_than_one_gpu_is_refused(repo_root):
    r = subprocess.run([sys.executable, os.path.join(repo_root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_kernel_source_hash_covers_existing_files(repo_root):
    b = load_bench(repo_root)
    csrc = os.path.join(repo_root, "paper_2604_19906_amd", "csrc")
    for op, files in b.KERNEL_SOURCES.items():
        for f in files:
            assert os.path.exists(os.path.join(csrc, f)), (op, f)
        assert len(b.kernel_source_hash(op)) == 16
    assert b.kernel_source_hash("ihelm") != b.kernel_source_hash("convection")


def test_stored_traffic_needs_a_matching_hash(repo_root):
    b = load_bench(repo_root)
    table = json.load(open(os.path.join(repo_root, "profiles", "traffic.json")))
    assert b.stored_traffic("no such workload", "pencil") is None
    for key, ent in table.items():
        op = "convection" if ":convection" in key else "ihelm"
        workload, variant = key.rsplit(":", 1)
        got = b.stored_traffic(workload, variant, op)
        if ent["source_hash"] == b.kernel_source_hash(op):
            assert got == ent["hbm_bytes_per_launch"]
        else:
            assert got is None
        assert os.path.exists(os.path.join(repo_root, ent["summary"]))


def test_kernel_source_hash_follows_code_not_comments(repo_root, tmp_path):
    """A comment or layout change keeps the hash (the kernel is the same), a code change does not."""
    import shutil

    b = load_bench(repo_root)
    want = b.kernel_source_hash("aniso")
    shutil.copytree(os.path.join(repo_root, "paper_2604_19906_amd", "csrc"),
                    tmp_path / "paper_2604_19906_amd" / "csrc")
    b.ROOT = str(tmp_path)
    assert b.kernel_source_hash("aniso") == want
    src = tmp_path / "paper_2604_19906_amd" / "csrc" / "tpo_generic.hip"
    text = src.read_text()
    src.write_text("// another comment\n/* and a\n   block */\n" + text.replace("\n", "\n\n    ", 3))
    assert b.kernel_source_hash("aniso") == want
    src.write_text(text.replace("ANISO_MAX_NT = 256", "ANISO_MAX_NT = 128"))
    assert b.kernel_source_hash("aniso") != want

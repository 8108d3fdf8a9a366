"""Host-side checks of bench.py and the entry script that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: --gpus N > 1 must exit with a message that says so, before touching a device."""
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr and "--gpus 2" in res.stderr
    assert not res.stdout.strip()


def test_binding_fails_loudly_without_the_library(tmp_path):
    """The product has no CPU fallback: importing the binding where the built library is absent raises."""
    pkg = tmp_path / "paper_2511_11062_amd"
    pkg.mkdir()
    for name in ("__init__.py", "lite_attn.py"):
        (pkg / name).write_text(open(os.path.join(ROOT, "paper_2511_11062_amd", name)).read())
    code = "import sys; sys.path.insert(0, %r)\nimport paper_2511_11062_amd.lite_attn" % str(tmp_path)
    res = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=120)
    assert res.returncode != 0 and "ImportError" in res.stderr


def test_product_sources_never_import_the_oracle():
    """Only tests, the smoke check and bench.py's cpu_baseline leg may touch oracle/."""
    import re
    for name in os.listdir(os.path.join(ROOT, "paper_2511_11062_amd")):
        if name.endswith(".py"):
            text = open(os.path.join(ROOT, "paper_2511_11062_amd", name)).read()
            assert not re.search(r"^\s*(from|import)\s+oracle\b", text, flags=re.M), name
    for name in os.listdir(os.path.join(ROOT, "paper_2511_11062_amd", "csrc")):
        text = open(os.path.join(ROOT, "paper_2511_11062_amd", "csrc", name)).read()
        assert "oracle" not in text.lower(), name
    bench = open(os.path.join(ROOT, "bench.py")).read()
    uses = [m.start() for m in re.finditer(r"from oracle import|import oracle", bench)]
    assert uses, "bench.py times the oracle for cpu_baseline"
    for pos in uses:                                   # every import sits inside the cpu_baseline leg
        head = bench[:pos]
        assert head.rfind("def cpu_baseline") > head.rfind("\ndef main") or "rows = args.cpu_rows" in head[head.rfind("\ndef main"):]

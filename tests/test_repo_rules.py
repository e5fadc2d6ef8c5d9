"""Host-side checks of how the pieces are allowed to depend on each other (no GPU needed)."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2402_15678_amd")


def _sources(top, exts):
    for base, dirs, files in os.walk(top):
        dirs[:] = [d for d in dirs if d not in ("__pycache__", "_build")]
        for f in files:
            if f.endswith(exts):
                yield os.path.join(base, f)


def test_bench_refuses_more_than_one_gpu():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert p.returncode != 0
    assert "one GPU" in p.stderr and p.stdout.strip() == ""


def test_product_path_never_touches_the_oracle():
    # the oracle is test infrastructure: the package (binding, harness, input generators, kernels) neither imports
    # nor names it, and the oracle does not import the package's HIP side either
    for path in _sources(PKG, (".py", ".hip", ".h", ".cpp")):
        text = open(path).read()
        assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), path
        assert "minions_oracle" not in text, path
    for path in _sources(os.path.join(ROOT, "oracle"), (".py", ".c", ".h")):
        text = open(path).read()
        assert "binding" not in text and "harness" not in text and "libminions_verify" not in text, path


def test_only_tests_smoke_and_the_cpu_baseline_import_the_oracle():
    bench = open(os.path.join(ROOT, "bench.py")).read()
    # one import, inside cpu_baseline
    assert len(re.findall(r"^\s*from oracle import|^\s*import oracle", bench, re.M)) == 1
    head = bench[:bench.index("def cpu_baseline")]
    assert "oracle import" not in head
    body = bench[bench.index("def cpu_baseline"):]
    nxt = re.search(r"^def ", body[4:], re.M)
    assert "from oracle import" in body[:nxt.start() + 4]


def test_nothing_committed_reads_the_reference_or_the_scratch_folder():
    tops = [PKG, os.path.join(ROOT, "tests"), os.path.join(ROOT, "oracle"), os.path.join(ROOT, "include")]
    files = [p for t in tops for p in _sources(t, (".py", ".hip", ".h", ".cpp", ".c"))]
    files += [os.path.join(ROOT, "bench.py"), os.path.join(ROOT, "__graft_entry__.py")]
    me = os.path.abspath(__file__)
    for path in files:
        if os.path.abspath(path) == me:
            continue
        text = open(path).read()
        assert "/root/reference" not in text, path
        assert "_work/" not in text and "_work\"" not in text, path


def test_profiles_are_short_text_summaries_with_their_command():
    prof = os.path.join(ROOT, "profiles")
    names = sorted(os.listdir(prof))
    assert names, "no profile summaries"
    for n in names:
        path = os.path.join(prof, n)
        assert n.endswith((".txt", ".md")), n
        assert "round" not in n.lower(), n                      # named for kernel and workload, not for a build round
        assert os.path.getsize(path) < 64 * 1024, n
        text = open(path).read()
        assert "rocprofv3" in text and "bench.py" in text, n   # the full command, which runs committed files only
        assert "_work" not in text and "gpurun" not in text, n

"""Host-side checks of the repository's contracts: the benchmark refuses more than one GPU,
the product package never touches the oracle, and nothing that ships reads scratch folders."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2008_02002_amd")


def _sources(top, exts):
    for base, dirs, files in os.walk(top):
        dirs[:] = [x for x in dirs if not x.startswith(("_", "."))]
        for f in files:
            if f.endswith(exts):
                yield os.path.join(base, f)


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""


def test_product_package_never_uses_the_oracle():
    for path in _sources(PKG, (".py", ".hip", ".h")):
        text = open(path).read()
        assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), path
        assert "xfbq_oracle" not in text, path


def test_oracle_never_uses_the_product_kernels():
    for path in _sources(os.path.join(ROOT, "oracle"), (".py", ".c", ".h")):
        text = open(path).read()
        assert "libxbq" not in text and "csrc" not in text, path
        assert not re.search(r"paper_2008_02002_amd\.(xbq|build)\b", text), path


def test_nothing_shipped_reads_scratch_or_reference_folders():
    tops = [PKG, os.path.join(ROOT, "oracle"), os.path.join(ROOT, "include")]
    files = [p for t in tops for p in _sources(t, (".py", ".hip", ".h", ".c"))]
    files += [os.path.join(ROOT, "bench.py"), os.path.join(ROOT, "__graft_entry__.py")]
    files += [p for p in _sources(os.path.join(ROOT, "tests"), (".py",)) if not p.endswith("test_repo_contract.py")]
    for path in files:
        text = open(path).read()
        assert not re.search(r"(^|[\"'/ ])_work/", text), path
        assert "/root/reference" not in text, path


def test_header_cites_the_paper_for_every_compute_entry_point():
    text = open(os.path.join(ROOT, "include", "xbq.h")).read()
    for name in ("xbq_encode", "xbq_search", "xbq_search_asym", "xbq_search_refine", "xbq_k_select"):
        decl = text.index(name + "(")
        block = text[max(0, decl - 3000):decl]
        assert re.search(r"Section|Algorithm|Eq\.", block), name


def test_equation_citations_use_the_papers_running_numbers():
    """The paper numbers its displayed equations 1..11 across sections.  Every citation in the
    sources must be one of the numbers this build uses, each with one meaning: 1 sigma, 2 the
    product/XOR identity, 5 the scalar product identity, 6 the vector operator, 7 the vector
    score relation, 8 the per-coordinate XOR form, 9 the bit-plane reconstruction, 10 the POPCNT
    form.  Section-relative numbers ("Eq. 6 of Section 3.3") are ambiguous and rejected."""
    tops = [PKG, os.path.join(ROOT, "oracle"), os.path.join(ROOT, "include"), os.path.join(ROOT, "tests")]
    meaning = {"1", "2", "5", "6", "7", "8", "9", "10"}
    for path in [p for t in tops for p in _sources(t, (".py", ".hip", ".h", ".c", ".cpp"))]:
        if path.endswith("test_repo_contract.py"):
            continue
        text = open(path).read()
        for num in re.findall(r"Eq\. (\d+)", text):
            assert num in meaning, (path, num)
        assert not re.search(r"Eq\. (5|6) of Section 3\.3|Eq\. 2 of Section 3\.3|Eq\. 6 \(Section 3\.[23]\)", text), path
    header = open(os.path.join(ROOT, "include", "xbq.h")).read()
    assert "Eq. 10" in header and "Eq. 9" in header and "Eq. 7" in header

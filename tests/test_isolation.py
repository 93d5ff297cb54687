"""The oracle is test infrastructure and shares nothing with the HIP path: these checks read the
source tree and fail if the product package ever imports the oracle (a CPU fallback would void
every parity claim), if the oracle imports the product or includes its headers, or if anything
committed depends on a working folder."""
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2603_21331_amd")


def sources(top, suffixes):
    for folder, _, names in os.walk(top):
        if "__pycache__" in folder:
            continue
        for name in names:
            if name.endswith(suffixes):
                yield os.path.join(folder, name)


def test_product_package_never_touches_the_oracle():
    for path in sources(PKG, (".py", ".h", ".hip", ".cpp")):
        text = open(path).read()
        assert not re.search(r"^\s*(import|from)\s+oracle\b", text, flags=re.M), path
        assert not re.search(r'#include\s*[<"][^>"]*oracle', text), path
        assert "liboracle" not in text and "_oracle.so" not in text, path


def test_oracle_never_touches_the_product():
    for path in sources(os.path.join(ROOT, "oracle"), (".py", ".cpp", ".h", ".c")):
        text = open(path).read()
        assert "paper_2603_21331_amd" not in text, path
        for inc in re.findall(r'#include\s*[<"]([^>"]+)[>"]', text):
            assert "/" not in inc and not inc.endswith((".h", ".hip")), f"{path} includes {inc}"
        assert not re.search(r"hip/|hipcc|__global__|__device__|\.hip\b", text), path


def test_only_the_allowed_entry_points_import_the_oracle():
    """tests/, bench.py's CPU-baseline leg and __graft_entry__.smoke() may; bench.py must import it
    inside the baseline branch, so that the timed GPU path cannot reach it."""
    for name in os.listdir(ROOT):
        if name.endswith(".py") and name not in ("bench.py", "__graft_entry__.py"):
            assert not re.search(r"^\s*(import|from)\s+oracle\b", open(os.path.join(ROOT, name)).read(), flags=re.M), name
    bench = open(os.path.join(ROOT, "bench.py")).read()
    assert not re.search(r"^(import|from)\s+oracle\b", bench, flags=re.M), "bench.py imports the oracle at module level"
    for m in re.finditer(r"^(\s+)import oracle\b", bench, flags=re.M):
        before = bench[:m.start()].rstrip().splitlines()[-1]
        assert "no_cpu_baseline" in before or before.lstrip().startswith(("import", "def ", '"""', "(")) or \
            before.strip().endswith(('"""', ":")), f"import oracle after: {before!r}"
    entry = open(os.path.join(ROOT, "__graft_entry__.py")).read()
    assert not re.search(r"^(import|from)\s+oracle\b", entry, flags=re.M), "__graft_entry__ imports the oracle at module level"


def test_nothing_committed_depends_on_a_working_folder():
    for top in (PKG, os.path.join(ROOT, "oracle"), os.path.join(ROOT, "tests")):
        for path in sources(top, (".py", ".h", ".hip", ".cpp")):
            if path.endswith("test_isolation.py"):
                continue
            text = open(path).read()
            assert "_work/" not in text and "gpurun_out" not in text, path
    for name in ("bench.py", "__graft_entry__.py"):
        text = open(os.path.join(ROOT, name)).read()
        assert "_work/" not in text, name

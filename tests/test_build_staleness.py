"""A built library that no longer matches its sources must not be loaded silently: every
library carries a hash of the files it was built from, the build script compares it with the
present files, and the bindings go through that check before they load.  No GPU needed."""
import os
import shutil

import pytest

from paper_2603_21331_amd import build

NAMES = sorted(build.LIBRARIES)


def test_every_library_is_listed_with_its_own_sources_and_public_header():
    assert NAMES == ["crossentropy", "layernorm", "measure", "rmsnorm", "rowsum", "softmax"]
    for name in NAMES:
        deps = build.dependencies(name)
        for d in deps:
            assert os.path.exists(d), d
        base = [os.path.basename(d) for d in deps]
        assert f"{name}_api.hip" in base and f"{name}.h" in base
        if name != "measure":
            assert f"{name}_kernels.h" in base
        # every csrc header the source includes, directly or through its kernels header, is a dependency
        included = set()
        for d in deps:
            if d.startswith(build.CSRC):
                for line in open(d):
                    line = line.strip()
                    if line.startswith('#include "') and "/" not in line.split('"')[1]:
                        included.add(line.split('"')[1])
        assert included <= set(base), (name, included - set(base))


@pytest.mark.parametrize("name", NAMES)
def test_a_built_library_carries_the_id_of_the_present_sources(name):
    build.ensure(name)
    assert build.built_id(name) == build.source_id(name)
    assert not build.is_stale(name)


@pytest.mark.parametrize("name", NAMES)
def test_changing_any_dependency_makes_the_library_stale(name, tmp_path, monkeypatch):
    """A copy of the tree's sources with one byte more in one file: the id of the sources
    changes, so the built library (which carries the old id) reads as stale.  A changed
    modification time alone does not: the id is a hash of contents."""
    build.ensure(name)
    csrc, include = tmp_path / "csrc", tmp_path / "include"
    shutil.copytree(build.CSRC, csrc)
    shutil.copytree(build.INCLUDE, include)
    monkeypatch.setattr(build, "CSRC", str(csrc))
    monkeypatch.setattr(build, "INCLUDE", str(include))
    assert not build.is_stale(name)
    for dep in build.dependencies(name):
        os.utime(dep, (1, 1))
    assert not build.is_stale(name)
    for dep in build.dependencies(name):
        original = open(dep, "rb").read()
        with open(dep, "ab") as f:
            f.write(b"\n// touched\n")
        assert build.is_stale(name), f"{name}: a change in {os.path.basename(dep)} went unnoticed"
        with open(dep, "wb") as f:
            f.write(original)
        assert not build.is_stale(name)


def test_changed_flags_make_every_library_stale(monkeypatch):
    monkeypatch.setattr(build, "HIPCC_FLAGS", build.HIPCC_FLAGS + ["-DSOMETHING_ELSE"])
    for name in NAMES:
        assert build.is_stale(name)


def test_without_hipcc_a_stale_library_is_an_error_that_names_the_file(tmp_path, monkeypatch):
    include = tmp_path / "include"
    shutil.copytree(build.INCLUDE, include)
    monkeypatch.setattr(build, "INCLUDE", str(include))
    with open(include / "rowsum.h", "ab") as f:
        f.write(b"\n/* touched */\n")
    monkeypatch.setattr(build, "hipcc", lambda: None)
    with pytest.raises(RuntimeError) as e:
        build.ensure("rowsum")
    assert "librowsum_hip.so" in str(e.value) and "stale" in str(e.value)
    assert build.ensure("softmax") == build.lib_path("softmax")      # an up-to-date one still loads


def test_a_missing_library_reads_as_stale(monkeypatch, tmp_path):
    monkeypatch.setitem(build.LIBRARIES, "rowsum", ("libnot_there.so",) + build.LIBRARIES["rowsum"][1:])
    assert build.built_id("rowsum") is None and build.is_stale("rowsum")
    monkeypatch.setattr(build, "hipcc", lambda: None)
    with pytest.raises(RuntimeError) as e:
        build.ensure("rowsum")
    assert "libnot_there.so" in str(e.value) and "missing" in str(e.value)

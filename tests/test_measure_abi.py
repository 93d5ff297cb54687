"""Host-side checks of the measurement library's C ABI (include/measure.h): it loads, exports
what the header declares, and rejects bad arguments before touching the device."""
import os
import re

from paper_2603_21331_amd import measure

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "measure.h")
P = 0x10000


def test_library_exports_every_declared_symbol_and_the_binding_has_the_same_names():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(measure_[a-z0-9_]+)\s*\(", text)))
    assert names == ["measure_copy", "measure_staged_copy", "measure_status_string"]
    lib = measure.load()
    for name in names + ["measure_build_id"]:
        assert hasattr(lib, name), name
    for name in names:
        assert hasattr(measure, name), name
    for name, value in re.findall(r"\b(MEASURE_[A-Z0-9_]+)\s*=\s*(-?\d+)", open(HEADER).read()):
        assert getattr(measure, name) == int(value)


def test_argument_checks():
    lib = measure.load()
    for copy in (lib.measure_copy, lib.measure_staged_copy):
        assert copy(P, P + 4096, 0, None) == measure.MEASURE_OK
        assert copy(None, None, 0, None) == measure.MEASURE_OK
        assert copy(P, P + 4096, 24, None) == measure.MEASURE_ERR_INVALID_ARG
        assert copy(P, P + 4096, -16, None) == measure.MEASURE_ERR_INVALID_ARG
        assert copy(P + 4, P + 4096, 32, None) == measure.MEASURE_ERR_INVALID_ARG
        assert copy(P, P + 4096 + 8, 32, None) == measure.MEASURE_ERR_INVALID_ARG
        assert copy(None, P, 32, None) == measure.MEASURE_ERR_INVALID_ARG
        assert copy(P, None, 32, None) == measure.MEASURE_ERR_INVALID_ARG
    assert measure.measure_status_string(0) == "ok"
    for s in (-1, -3, 5):
        assert measure.measure_status_string(s)

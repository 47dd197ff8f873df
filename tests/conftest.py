import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def json_oracle():
    from oracle import Oracle
    from workloads import grammars
    return Oracle(grammars.JSON)


@pytest.fixture(autouse=True)
def no_walk_stopped_at_an_internal_guard(request, monkeypatch):
    """Every GPU test ends with the device fault counter of each handle it compiled at 0: a walk
    that a kernel stopped at one of its internal guards would otherwise pass as "not allowed"."""
    if request.node.get_closest_marker("gpu") is None:
        yield
        return
    import weakref
    from paper_2506_03887_amd import binding
    made = []
    init = binding.Pre3.__init__

    def recording_init(self, *a, **kw):
        init(self, *a, **kw)
        if not kw.get("host_only", False):
            made.append(weakref.ref(self))

    monkeypatch.setattr(binding.Pre3, "__init__", recording_init)
    yield
    for ref in made:
        lib = ref()
        if lib is not None and getattr(lib, "_h", None):
            assert lib.fault_count() == 0, "a kernel stopped a token walk at an internal guard"

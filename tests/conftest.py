import os
import re
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")


# GPU tests whose names match run once per rank walk of the reduce-scatter
# kernels: the library's own choice (wide at test sizes) and the deep and the
# half-chunk walk forced, so that those kernels see the ragged, misaligned,
# split-W, hybrid, accumulate and unscale cases at small sizes too.
_WALK_TESTS = re.compile(r"reduce|fused|hybrid|accumul|unscale|scaler|whole_path|graph|prefetch|fig3")


def pytest_generate_tests(metafunc):
    if metafunc.definition.get_closest_marker("gpu") is None and not any(
            m.name == "gpu" for m in getattr(metafunc.module, "pytestmark", []) or []):
        return
    if "_reduce_walk" in metafunc.fixturenames and _WALK_TESTS.search(metafunc.function.__name__):
        metafunc.parametrize("_reduce_walk", ["auto", "deep", "half"], indirect=True)


@pytest.fixture(autouse=True)
def _reduce_walk(request, monkeypatch):
    """The rank walk is a per-layout hint (fsdp_layout_init_ex): under the
    "deep" and "half" parameters every layout the test creates through the
    package asks for that walk.  Only this test's view of the binding is patched."""
    walk = getattr(request, "param", None)
    if walk not in ("deep", "half"):
        yield
        return
    import functools
    import paper_2304_11277_amd as F
    hint = F.FSDP_WALK_DEEP if walk == "deep" else F.FSDP_WALK_HALF
    monkeypatch.setattr(F, "fsdp_layout_init", functools.partial(F.binding.fsdp_layout_init, reduce_walk=hint))
    yield

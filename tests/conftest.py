import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GUARD_BYTES = 64 * 1024


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(autouse=True)
def guard_bands_around_every_cache(request):
    """GPU tests only: every Cache a test creates gets 64 KiB of 0xFF on either side of the
    device buffer it hands to the library (0xFF.. is NaN as bf16 and fp32), and after the test
    all of those bands must be untouched: a kernel that writes outside the library's own
    buffer fails the test that ran it."""
    if request.node.get_closest_marker("gpu") is None:
        yield
        return
    import paper_2604_16734_amd as K
    created = []
    real_init = K.Cache.__init__

    def tracking_init(self, *args, **kwargs):
        real_init(self, *args, **kwargs)
        created.append(self)

    K.Cache.default_guard_bytes = GUARD_BYTES
    K.Cache.__init__ = tracking_init
    try:
        yield
        import torch
        torch.cuda.synchronize()
        for cache in created:
            assert cache.guard == GUARD_BYTES
            assert cache.guards_intact(), "a kernel wrote outside the cache's device buffer"
    finally:
        K.Cache.__init__ = real_init
        K.Cache.default_guard_bytes = 0
        created.clear()

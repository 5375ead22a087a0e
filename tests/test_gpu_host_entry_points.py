"""The host-only entry points (scheduling arithmetic of Sec. 4.2 / 4.3, lifecycle of Sec. 6.2, residency index)
against the oracle once more, in the process and on the machine that runs the GPU tests: the same test
functions as in the CPU selection, collected here under the gpu marker."""
import pytest

import test_index_parity as _index_tests
import test_policy_parity as _policy_tests
from test_index_parity import index  # noqa: F401  (fixture used by the index tests)

pytestmark = pytest.mark.gpu

for _mod, _tag in ((_policy_tests, "policy"), (_index_tests, "index")):
    for _name in dir(_mod):
        if _name.startswith("test_"):
            globals()["test_%s_%s" % (_tag, _name[5:])] = getattr(_mod, _name)

"""Host-side checks of the channel-mixing linear (no GPU): exports against include/el.h and
argument errors."""
import os
import re

import pytest

el = pytest.importorskip("paper_2504_10700_amd.el_binding")

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "el.h")).read()
    declared = set(re.findall(r"^(?:sc_status|int32_t)\s+(el_\w+)\s*\(", header, flags=re.M))
    assert declared == set(el.EXPORTS)
    for name in declared:
        assert getattr(el.lib, name) is not None


def test_argument_errors_and_workspace():
    cfg = el.make_config(128, 128, 3)
    small, big = el.el_workspace_bytes(cfg, 100), el.el_workspace_bytes(cfg, 100_000)
    assert 256 <= small <= big
    assert el.el_workspace_bytes(el.make_config(96, 40, 1), 1000) == 256     # plain kernels need none
    for bad in (el.make_config(0, 128, 3), el.make_config(128, 128, 4), el.make_config(128, 128, 3, dtype=7)):
        with pytest.raises(el.ScError):
            el.el_workspace_bytes(bad, 10)
    with pytest.raises(el.ScError) as e:
        el.el_forward(cfg, 10, None, None, None, stream=0)
    assert e.value.status == 1

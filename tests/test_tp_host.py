"""Host-side checks of the channelwise tensor product part of the library (no GPU): exports
against include/tp.h, paths and sparse terms against the oracle's independent derivation."""
import os
import re

import numpy as np
import pytest

from oracle import channelwise_tp as otp
from oracle import coupling as oc

tp = pytest.importorskip("paper_2504_10700_amd.tp_binding")

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "tp.h")).read()
    declared = set(re.findall(r"^sc_status\s+(tp_\w+)\s*\(", header, flags=re.M))
    assert declared == set(tp.EXPORTS)
    for name in declared:
        assert getattr(tp.lib, name) is not None


@pytest.mark.parametrize("l_Y,l_h,L_max", [(3, 1, 3), (3, 0, 3), (1, 1, 1), (2, 3, 1), (3, 3, 3), (0, 0, 0)])
def test_paths_and_terms_match_the_oracle(l_Y, l_h, L_max):
    plan = tp.tp_plan_create(64, l_Y, l_h, L_max, tp.SC_F64, 0, tp.SC_PLAN_HOST_ONLY)
    cfg = otp.TPConfig(64, l_Y, l_h, L_max)
    paths = [tuple(r) for r in tp.tp_plan_paths(plan).tolist()]
    assert paths == otp.enumerate_paths(cfg)
    info = tp.tp_plan_info(plan)
    assert (info.n_Y, info.n_h, info.n_out, info.num_paths) == (cfg.n_Y, cfg.n_h, cfg.n_out, len(paths))
    p, a, b, c, coef = tp.tp_plan_terms(plan)
    dense = np.zeros((len(paths), cfg.n_Y, cfg.n_h, cfg.n_out))
    np.add.at(dense, (p, a, b, c), coef)
    for i, (l1, l2, l3) in enumerate(paths):
        want = np.zeros((cfg.n_Y, cfg.n_h, cfg.n_out))
        want[l1 * l1:(l1 + 1) ** 2, l2 * l2:(l2 + 1) ** 2, l3 * l3:(l3 + 1) ** 2] = oc.coupling_tensor(l1, l2, l3)
        assert np.abs(dense[i] - want).max() < 1e-13
    # every listed term is a genuine non-zero, listed once
    assert np.all(np.abs(coef) > 1e-14)
    assert len(set(zip(p.tolist(), a.tolist(), b.tolist(), c.tolist()))) == len(coef)
    tp.tp_plan_destroy(plan)


def test_argument_errors_on_the_host():
    with pytest.raises(tp.ScError) as e:
        tp.tp_plan_create(64, 4, 1, 3, tp.SC_F32, 0, tp.SC_PLAN_HOST_ONLY)
    assert e.value.status == 2
    with pytest.raises(tp.ScError) as e:
        tp.tp_plan_create(0, 3, 1, 3, tp.SC_F32, 0, tp.SC_PLAN_HOST_ONLY)
    assert e.value.status == 1
    plan = tp.tp_plan_create(64, 3, 1, 3, tp.SC_F32, 0, tp.SC_PLAN_HOST_ONLY)
    with pytest.raises(tp.ScError) as e:        # compute calls fail on a host-only plan
        tp.tp_forward(plan, 1, 1, 0, None, None, None, None, None, None, stream=0)
    assert e.value.status == 2
    assert tp.tp_workspace_bytes(plan, 1000) >= 1000 * 16 * 4
    tp.tp_plan_destroy(plan)

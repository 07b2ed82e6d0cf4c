"""The committed straight-line kernel sources (csrc/generated/*.inc) are exactly what the
generators write from the library's own tables: a hand edit or a stale file fails here, on
the CPU, before any GPU run.  Needs the built library (host-side table builder only)."""
import os

import pytest

from paper_2504_10700_amd.codegen import generate, generate_tp
from paper_2504_10700_amd.codegen.tables import HOST_LIB

pytestmark = pytest.mark.skipif(not os.path.exists(HOST_LIB), reason="library not built")


def test_contraction_kernels_match_the_generator(capsys):
    assert generate.main(["--check"]) == 0, capsys.readouterr().err


def test_tensor_product_kernels_match_the_generator(capsys):
    assert generate_tp.main(["--check"]) == 0, capsys.readouterr().err


def test_every_generated_file_has_a_generator():
    have = {f for f in os.listdir(generate.OUT_DIR) if f.endswith(".inc")}
    want = {f"sc_gen_{t}.inc" for t in generate.SPECS} | {f"tp_gen_{t}.inc" for t in generate_tp.SPECS}
    assert have == want

"""ficoco_v_step called from a compiled C program written against include/ficoco.h (no ctypes
marshalling between the caller and the library): tests/c_abi/step_check.c runs one tiny step
whose result has a closed form, checks that an aliased output is refused, and returns 0."""
import ctypes as C
import os

import pytest

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))


def test_step_called_from_c_matches_closed_form():
    so = os.path.join(HERE, "c_abi", "libstep_check.so")
    assert os.path.exists(so), "tests/c_abi/libstep_check.so is not built: run `python -m paper_2411_17686_amd.build`"
    lib = C.CDLL(so)
    assert lib.ficoco_c_step_check() == 0

"""Host side of the resident kernels compiled for one network (no GPU): the description the library writes
for a network compiles with the library's own kernel source into a code object that holds the kernel and its
plan.  (The compile needs hipcc, not a GPU; the objects it leaves under paper_1102_0183_amd/_spec/ are the ones
the GPU tests load.)"""
import os
import subprocess

import pytest

from paper_1102_0183_amd import binding, specialize
from tests.resident_code_cases import CASES


@pytest.mark.parametrize("name", sorted(CASES))
def test_the_description_of_a_network_compiles(name):
    arch, fan = CASES[name]
    text = binding.resident_spec_source_for(arch, fan)
    assert "StaticSpec<FLOW_SPECIAL_ID>" in text and "flow_plan(Z, 0, 0, 256)" in text
    path = specialize.code_object_for(text)
    assert os.path.getsize(path) > 10000
    # the same description gives the same file; another network another one
    assert specialize.code_object_for(text) == path
    other = binding.resident_spec_source_for(arch.replace("150N", "151N").replace("80N", "81N").replace("300N", "301N"), fan)
    assert specialize._digest(other) != specialize._digest(text)


def test_what_the_description_holds():
    text = binding.resident_spec_source_for("1x29x29-20C4-MP2-40C5-MP3-150N-10N", 8, 40, 1)
    for line in ("Z.n_conv = 2;", "Z.conv[1].Mi = 20;", "Z.conv[1].K = 5;", "Z.conv[1].max_conn = 8;", "Z.conv[1].max_back = 16;",
                 "Z.conv[1].full_table = 0;", "Z.fc[0].n_in = 360;", "Z.fc[1].is_output = 1;", "flow_plan(Z, 40, 1, 256);"):
        assert line in text, line
    with pytest.raises(binding.CnnError):       # a network the resident mode cannot run has no description
        binding.resident_spec_source_for("3x32x32-300C3-MP2-300C2-MP2-300C4-MP2-300N-10N")


def test_a_broken_description_is_reported():
    with pytest.raises(RuntimeError, match="hipcc failed"):
        specialize.code_object_for("this is not C++;\n")

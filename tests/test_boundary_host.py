"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and its architecture grammar / shape inference agree with the oracle's."""
import os
import re

import pytest

import oracle
from oracle.binding import OracleError
from paper_1102_0183_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "cnn355.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cnn_[a-z_0-9]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    L = binding.lib()
    names = _declared()
    assert len(names) >= 25
    for n in names:
        assert hasattr(L, n), n
    assert sorted(binding.EXPORTS) == names


@pytest.mark.parametrize("name", sorted(synth.WORKLOADS))
def test_shapes_agree_with_the_oracle(name):
    arch = synth.WORKLOADS[name].arch
    info = binding.arch_info(arch)
    o = oracle.Oracle(arch)
    assert len(info) == o.num_layers
    for l, i in enumerate(info):
        assert i == o.layer_info(l), (l, i)
    assert binding.workspace_bytes(arch) > 8 * o.num_weights


BAD = ["", "1x29", "1x29x29", "1x29x29-20C4", "1x29x29-20C4-MP2", "1x29x29-20Q4-10N", "1x29x29-MP2-10N",
       "1x29x29-10N-20C4-10N", "1x29x29-20C4-MP2-MP2-10N", "1x29x29-20C4-MP4-10N", "1x4x4-20C5-10N",
       "0x4x4-10N", "1x29x29-0C4-10N", "1x29x29-20C4-MP0-10N", "1x29x29--10N", "1x29x29-20C4S-10N",
       "1x29x29-20C4-10N-", "1x29x29-20C4x-10N", "x29x29-10N", "1x29x29-20C4-10N10", "1x29x29-20C-10N",
       "1x29x29-20C4x0-10N", "1x29x29-20C4-MP2x-10N", "1x29x29-20C4-MP2x3-10N", "1x29x29-20C4x30-10N",
       "1x29x29-20C4S1x-10N"]


@pytest.mark.parametrize("arch", BAD)
def test_rejected_architectures_agree_with_the_oracle(arch):
    with pytest.raises(binding.CnnError) as e:
        binding.arch_info(arch)
    with pytest.raises(OracleError) as eo:
        oracle.Oracle(arch)
    assert e.value.code == eo.value.code
    assert str(e.value)
    with pytest.raises(binding.CnnError):
        binding.workspace_bytes(arch)


def test_extra_grammar_cases():
    info = binding.arch_info("2x12x12-4C5S1-MP2-3C2-3N")
    assert [(i["maps"], i["h"], i["w"]) for i in info] == [(2, 12, 12), (4, 4, 4), (4, 2, 2), (3, 1, 1), (3, 1, 1)]
    assert info[1]["S"] == 1 and info[1]["K"] == 5 and info[2]["K"] == 2
    assert info[1]["Sx"] == 1 and info[1]["Kx"] == 5 and info[2]["Kx"] == 2
    # x and y values of their own (rows first): Eq. 1 axis by axis; the 6-number call reports the y values
    arch = "2x14x11-3C4x2S1x0-MP2x5-4C1x2-5N-3N"
    info = binding.arch_info(arch)
    assert [(i["maps"], i["h"], i["w"]) for i in info] == [(2, 14, 11), (3, 6, 10), (3, 3, 2), (4, 3, 1), (5, 1, 1), (3, 1, 1)]
    assert (info[1]["K"], info[1]["Kx"], info[1]["S"], info[1]["Sx"]) == (4, 2, 1, 0)
    assert (info[2]["K"], info[2]["Kx"]) == (2, 5)
    import ctypes as C
    import numpy as np
    n = C.c_int32()
    six = np.zeros((6, 6), dtype=np.int32)
    assert binding.lib().cnn_arch_info(arch.encode(), C.addressof(n), six.ctypes.data, 6) == 0
    assert n.value == 6 and six[1].tolist() == [1, 3, 6, 10, 4, 1] and six[2].tolist()[4] == 2

"""The networks whose resident kernel the tests load as a code object compiled for them alone: the examples the
package's build step compiles (paper_1102_0183_amd/specialize.py), and the connection table that goes with a fan-in."""
from paper_1102_0183_amd import synth
from paper_1102_0183_amd.specialize import EXAMPLES as CASES  # noqa: F401


def table_for(maps_out, maps_in, fan_in):
    """Output map j reads the input maps j .. j + fan_in - 1 (mod maps_in); fan_in = -d: maps_in / d of them."""
    return synth.regular_table(maps_out, maps_in, fan_in)

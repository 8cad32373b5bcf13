"""The networks whose resident kernel the tests load as a code object compiled for them alone: the examples the
package's build step compiles (paper_1102_0183_amd/specialize.py), and the connection table that goes with a fan-in."""
import numpy as np

from paper_1102_0183_amd.specialize import EXAMPLES as CASES  # noqa: F401


def table_for(maps_out, maps_in, fan_in):
    """Output map j reads the input maps j .. j + fan_in - 1 (mod maps_in)."""
    t = np.zeros((maps_out, maps_in), dtype=np.uint8)
    for j in range(maps_out):
        for k in range(fan_in):
            t[j, (j + k) % maps_in] = 1
    return t

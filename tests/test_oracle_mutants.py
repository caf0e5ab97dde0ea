"""Each planted mistake in the oracle (built as a separate, deliberately wrong library on the CPU)
must fail at least one pin. This shows the pins are sharp enough to notice a dropped term, a wrong
head mapping, swapped planes, a transposed layout, a missing normalisation, a stale newest token,
a wrong allocation order, broken migration bookkeeping, a worst-fit choice, a release that
retains nothing, an unmap with the wrong bound or without the release, and activation chunks that
never become idle again."""
import os

import pytest

import oracle
from oracle import build
from tests import oracle_pins as P

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

MUTANTS = {
    1: "q head -> kv head by modulo instead of contiguous groups",
    2: "softmax scale dropped",
    3: "K and V planes swapped",
    4: "weights not normalised",
    5: "newest token ignored",
    6: "chunk layout plane-major instead of head-major",
    7: "last dim dropped from the dot product",
    8: "pool picks the highest free chunk",
    9: "offload does not free the device chunk",
    10: "fetch does not copy the bytes back",
    11: "acquire takes the largest fitting available tensor instead of the smallest",
    12: "release unmaps everything instead of keeping the mapping",
    13: "SLO window counts every iteration since the last change instead of the last five",
    14: "unmap treats a partly filled slot as empty",
    15: "unmap clears the table entry but leaves the chunk (and host slot) taken",
    16: "busy = 0 leaves the activation chunks busy",
    17: "pre-mapping ahead also maps the slot after the last token it looks at",
}


@pytest.mark.parametrize("m", sorted(MUTANTS), ids=lambda m: f"mutant{m}")
def test_mutant_is_caught(tmp_path, m):
    lib = oracle.load(build.build(force=True, defines=(f"ORC_MUTANT={m}",), out=str(tmp_path / f"mut{m}.so")))
    failed = []
    pins = list(P.ALL_PINS) + [lambda l: P.pin_inflation_walkthrough(l, os.path.join(GOLDEN, "inflation_walkthrough.txt")),
                               lambda l: P.pin_slo_buffer_trace(l, os.path.join(GOLDEN, "slo_buffer_trace.txt"))]
    for pin in pins:
        try:
            pin(lib)
        except AssertionError:
            failed.append(getattr(pin, "__name__", "walkthrough"))
    assert failed, f"no pin noticed: {MUTANTS[m]}"

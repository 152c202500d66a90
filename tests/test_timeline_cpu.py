"""The timeline module turns the decode kernel's phase comments into time stamps; the
comments and the module must stay in step (no GPU, no compiler needed)."""
import os

from paper_2311_18677_amd import build as sw_build
from paper_2311_18677_amd import timeline


def test_every_phase_comment_exists_exactly_once():
    src = open(os.path.join(sw_build.CSRC, "sw_decode_split.hip")).read()
    for name, _ in timeline.STAMPS:
        assert src.count("// -- phase: " + name) == 1, name
    # nothing in the kernel is a phase the module does not know
    known = {name for name, _ in timeline.STAMPS}
    for line in src.splitlines():
        if "// -- phase: " in line:
            assert line.split("// -- phase: ", 1)[1].strip() in known, line


def test_stamp_slots_fit_the_table_and_the_report():
    slots = []
    for _, code in timeline.STAMPS:
        for part in code.split("SW_STAMP")[1:]:
            slots.append(int(part.split("(", 1)[1].split(")", 1)[0]))
    assert sorted(set(slots)) == list(range(len(timeline.COLUMNS)))
    assert max(slots) < timeline.SLOTS


def test_the_product_library_is_not_built_from_the_instrumented_source():
    assert "timeline" not in " ".join(sw_build.SOURCES)
    assert os.path.basename(timeline.LIB) != os.path.basename(sw_build.LIB)

"""What the compiler reports for every kernel instance of the library (no GPU needed): no kernel may
use scratch memory or spill registers -- a private copy of a kernel's argument block, which is what a
run-time index into a narrow array of it or too many inlined bodies produce, costs an order of
magnitude in step time -- and none may fall below half occupancy."""
from paper_1711_00705_amd import resource_usage as ru


def test_no_kernel_uses_scratch_or_spills():
    sources, per_source = ru.collect()
    seen = 0
    for src, rows in zip(sources, per_source):
        assert rows, f"{src}: no kernel found"
        for r in rows:
            seen += 1
            assert int(r["ScratchSize [bytes/lane]"]) == 0, (src, r["name"], r["ScratchSize [bytes/lane]"])
            # (a few scalar registers parked in lanes of a vector register are harmless)
            assert int(r["VGPRs Spill"]) == 0 and int(r["SGPRs Spill"]) <= 32, (src, r["name"])
            assert int(r["Occupancy [waves/SIMD]"]) >= 4, (src, r["name"], r["Occupancy [waves/SIMD]"])
    assert seen >= 100

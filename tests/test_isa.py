"""The hand-scheduled kernels rely on the compiler leaving in-flight registers alone; check the
generated ISA (CPU only: hipcc cross-compiles)."""

import shutil

import pytest

import isa_check


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
@pytest.mark.parametrize("source", ["lookup_mfma.hip"])
def test_no_instruction_touches_a_fragment_register_in_flight(source):
    asm = isa_check.device_asm(source)
    ks = isa_check.kernels(asm)
    checked = 0
    for name, lines in ks.items():
        reads = [l for l in lines if l.startswith("ds_read_b128") and ("hand-scheduled" in l or "hand-placed" in l)]
        if not reads:
            continue
        high = isa_check.fixed_fragment_users_not_hand_placed(lines)
        assert not high, f"{name}: compiler-placed use of the hand-placed fragment registers: {high[:3]}"
        bad = isa_check.inflight_violations(lines)
        assert not bad, f"{name}: {bad[:3]}"
        stray = isa_check.agpr_users_not_hand_placed(lines)
        assert not stray, f"{name}: compiler-placed AGPR use next to hand-placed accumulators: {stray[:3]}"
        early = isa_check.early_accumulator_reads(lines)
        assert not early, f"{name}: accumulator read too close behind its MFMA: {early[:3]}"
        checked += 1
    assert checked >= 3


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_the_mfma_kernels_keep_everything_in_registers():
    """A counter or an accumulator that ends up in per-lane scratch memory costs a memory round trip in
    every slab of the pipelined kernels: no kernel of the file may have a private segment."""
    sizes = isa_check.private_segment_sizes(isa_check.device_asm("lookup_mfma.hip"))
    pipe = [k for k in sizes if "k_lookup_pipe" in k]
    assert len(pipe) >= 10 and any("k_lookup_wide" in k for k in sizes)
    spilled = {k: v for k, v in sizes.items() if v}
    assert not spilled, spilled

"""The hot kernels keep their accumulators and operand sets in registers (no GPU needed: the compiler's own
resource remarks).  A slot-program kernel whose register arrays fall into scratch memory still computes the right
results, thirty times slower, so parity tests would not notice; the same holds, at 15 %, for a build that moves the
matrix instructions out of the slots they are written in."""
import functools

from paper_2605_01255_amd import build


@functools.lru_cache(maxsize=None)
def resources():
    return build.kernel_resources()


def test_hot_kernels_use_no_scratch_memory():
    res = resources()
    hot = {n: r for n, r in res.items()
           if any(k in n for k in ("gemm16_persist_kernel", "gemm8_persist_kernel", "gemm16_smallk_kernel",
                                   "sketch8_kernel", "gemm_bf16_kernel"))}
    assert len(hot) >= 10, sorted(res)
    bad = {n: r for n, r in hot.items() if r.get("scratch", -1) != 0 or r.get("vgpr_spill", -1) != 0}
    assert not bad, bad


def test_slot_programs_hold_one_matrix_instruction_per_slot():
    """Between two scheduling fences of the persistent GEMM kernels there is at most one matrix instruction, and every
    K-tile variant is there in full (bf16: three variants of 128 slots; 8-bit: three of 64)."""
    res = resources()
    for key, slots in (("gemm16_persist_kernel", 3 * 128), ("gemm8_persist_kernel", 3 * 64)):
        kernels = {n: r["mfma_regions"] for n, r in res.items() if key in n}
        assert kernels, key
        for name, regions in kernels.items():
            assert set(regions) <= {0, 1}, (name, regions)
            assert regions.get(1, 0) == slots, (name, regions)


def test_transfers_read_no_scalar_register_a_vector_instruction_just_wrote():
    """A kernel with more scalar values than registers had its transfers' offsets restored from vector lanes right
    in front of the hand-written transfer: it moved the wrong rows.  No kernel of the library may do that."""
    res = resources()
    assert any(r.get("stale_transfer_operands") is not None for r in res.values())
    bad = {n: r["stale_transfer_operands"] for n, r in res.items() if r.get("stale_transfer_operands")}
    assert not bad, bad


def test_the_assembly_scan_sees_a_planted_stale_operand_and_a_crowded_slot():
    text = """
kern_a: ; @kern_a
	; sched_barrier mask(0x00000000)
	v_mfma_f32_16x16x32_bf16 a[0:3], v[0:3], v[4:7], a[0:3]
	v_readlane_b32 vcc_lo, v254, 6
	buffer_store_dwordx2 v[156:157], v212, s[24:27], 64 offen
	buffer_load_dwordx4 v253, s[48:51], vcc_lo offen lds
	; sched_barrier mask(0x00000000)
	v_mfma_f32_16x16x32_bf16 a[4:7], v[0:3], v[4:7], a[4:7]
	v_mfma_f32_16x16x32_bf16 a[8:11], v[0:3], v[4:7], a[8:11]
	v_readlane_b32 s50, v254, 7
	s_nop 4
	buffer_load_dwordx4 v253, s[48:51], s7 offen lds
	; sched_barrier mask(0x00000000)
	v_readlane_b32 s9, v254, 8
	s_nop 0
	s_nop 0
	s_nop 0
	s_nop 0
	s_nop 0
	buffer_load_dwordx4 v253, s[48:51], s9 offen lds
	s_endpgm
kern_b: ; @kern_b
	v_readlane_b32 s9, v254, 8
	buffer_load_dwordx4 v253, s[48:51], s9 offen
	s_endpgm
"""
    found = build.scan_assembly(text.splitlines(keepends=True), {"kern_a", "kern_b"})
    assert found["kern_a"]["stale_transfer_operands"] == 2       # vcc_lo two before; s50 of the resource two before
    assert found["kern_a"]["mfma_regions"] == {0: 1, 1: 1, 2: 1}
    assert found["kern_b"] == {"mfma_regions": {}, "stale_transfer_operands": 0}  # an ordinary load: the compiler's job

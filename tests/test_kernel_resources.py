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

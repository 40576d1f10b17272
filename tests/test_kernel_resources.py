"""The hot kernels keep their accumulators and operand sets in registers (no GPU needed: the compiler's own
resource remarks).  A slot-program kernel whose register arrays fall into scratch memory still computes the right
results, thirty times slower, so parity tests would not notice."""
from paper_2605_01255_amd import build


def test_hot_kernels_use_no_scratch_memory():
    res = build.kernel_resources()
    hot = {n: r for n, r in res.items()
           if any(k in n for k in ("gemm16_persist_kernel", "gemm8_persist_kernel", "gemm16_smallk_kernel",
                                   "sketch8_kernel", "gemm_bf16_kernel"))}
    assert len(hot) >= 10, sorted(res)
    bad = {n: r for n, r in hot.items() if r.get("scratch", -1) != 0 or r.get("vgpr_spill", -1) != 0}
    assert not bad, bad

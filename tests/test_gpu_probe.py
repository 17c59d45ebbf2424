"""The matrix-instruction-only probe kernel (a measurement aid of bench.py): it must run to completion and, on its
constant operands, leave the sums that the instruction count implies."""
import pytest
import torch

import paper_2409_15097_amd as bbm

pytestmark = pytest.mark.gpu


def test_probe_accumulates_what_its_instruction_count_implies():
    iters = 10
    sink = bbm.bbm_probe_mfma_bf16(False, iters)
    torch.cuda.synchronize()
    # every operand element: a = 1, b = 0.5; one instruction adds 16 * 0.5 = 8 to each of a lane's 16 accumulator values;
    # 16 instructions per iteration over four accumulators; the lane writes the sum of its 64 values
    assert torch.all(sink == 16 * 8.0 * 16 * iters)
    again = bbm.bbm_probe_mfma_bf16(True, iters)
    torch.cuda.synchronize()
    assert torch.isfinite(again).all() and again.abs().max() > 0
    assert bbm.bbm_probe_mfma_bf16_flop(iters) == 256 * 4 * 16 * iters * 32768

"""CPU oracle for the Binary Block Masking attention path (forward, and the backward pass that widens it).  TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 numpy definitions of (a) masked softmax attention and its gradients and (b) the block matrix / run index /
sparse block list / packed mask bits that the GPU preprocessing must reproduce bit-exactly.  Nothing here is
imported by the product path; only the tests, the smoke check and the benchmark's cpu_baseline leg use it.
It shares no code with the GPU library or its Python binding.
"""
from .attention import bf16_bits_to_f64, masked_attention, masked_attention_rows  # noqa: F401
from .attention_bwd import (masked_attention_bwd, masked_attention_bwd_rows, masked_attention_bwd_cols,  # noqa: F401
                            masked_attention_bwd_magnitudes)
from .reorder import cuthill_mckee_order, reverse_cuthill_mckee, permute_mask, bandwidth  # noqa: F401
from .brute import brute_attention, brute_block_counts, brute_bwd_magnitudes  # noqa: F401
from .blocks import (block_counts, block_class, bin_blk_mat, run_index, sparse_index, packed_bits,  # noqa: F401
                     block_index, schedule, column_index, column_schedule)

"""Bounds shared by the GPU parity tests (bf16 forward outputs against the fp64 oracle).

max-abs <= 2e-2 and pooled relative L2 <= 1e-2 are the task's bounds.  Outputs shrink like 1/sqrt(keys), so at
the paper's sizes max-abs cannot fail; the pooled norm cannot see one wrong row among thousands.  Hence two
internal bars: pooled relative L2 <= 5e-3, and a relative L2 bound on EVERY query row.
"""
import numpy as np

BF16_MAX_ABS, BF16_REL_L2, FP32_MAX_ABS = 2e-2, 1e-2, 1e-4
BF16_REL_L2_INTERNAL = 5e-3
# |g_i - o_i|_2 / |o_i|_2 for every query row i; about three times the worst row measured over all GPU tests
BF16_ROW_REL_L2 = 2.5e-2  # worst row measured: 8.6e-3 (16-frame training form, 12 heads), 7.6e-3 (c2 at full size)


def row_errors(got, ref):
    """Relative L2 error of every query row (last axis = features)."""
    num = np.sqrt(np.sum((got - ref) ** 2, axis=-1))
    den = np.sqrt(np.sum(ref ** 2, axis=-1))
    return num / np.maximum(den, 1e-30)


def worst_row(got, ref):
    r = row_errors(got, ref)
    i = int(r.argmax())
    return float(r.reshape(-1)[i]), np.unravel_index(i, r.shape)

# Log-sum-exp written by the forward of the training pair (absolute, natural units): fp32 sums of fp32 exponentials
# of scores accumulated exactly from the bf16 inputs; measured < 1e-5.
BF16_LSE_ABS = 2e-4

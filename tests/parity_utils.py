"""Helpers of the GPU <-> oracle parity tests (teacher-forced verification of the walk)."""
import numpy as np
import torch

MARGIN = 1e-4      # decisions whose |u_j - p_j| is below this may legitimately differ (counted, reported)


def to_f64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of fp32 / bf16 device data to float64 on the host."""
    return t.detach().to("cpu", torch.float32).numpy().astype(np.float64)


def f32(x: float) -> float:
    """The value the C ABI receives when x is passed as a float."""
    return float(np.float32(x))


def verify_halving(oracle, K_blocks, u, gpu_signs, *, log_c, center, r_key=0.0, V_blocks=None, r_value=0.0):
    """Feed the GPU's signs to the oracle (teacher forcing) and classify every decision.

    Decision j is a hard mismatch if the oracle's rule (u_j < p_j), evaluated on the GPU's own
    prefix of signs, disagrees with the GPU and |u_j - p_j| >= MARGIN; a margin case if it
    disagrees with a smaller margin.  V_blocks: the value rows, when the weights carry the value factor.
    Returns dict(hard, margin, n, res).
    """
    res = oracle.softmax_balance_batch(K_blocks, V_blocks, u=u, log_c=log_c, r_key=r_key, r_value=r_value, center=center,
                                       forced=gpu_signs)
    differ = res["dec"] != gpu_signs
    marg = np.abs(u - res["p"])
    hard = int(np.count_nonzero(differ & (marg >= MARGIN)))
    soft = int(np.count_nonzero(differ & (marg < MARGIN)))
    return dict(hard=hard, margin=soft, n=int(gpu_signs.size), res=res, near=int(np.count_nonzero(marg < MARGIN)))


def expected_survivors(oracle, gpu_signs):
    """The integer function of the output step applied to the GPU's own signs, per instance."""
    return np.stack([oracle.select_half(s, strict=True) for s in gpu_signs])


def rel_l2(a: np.ndarray, b: np.ndarray) -> float:
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))

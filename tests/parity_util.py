"""Helpers shared by the GPU parity tests: run the numpy oracle per head on the same
tensors that went to the HIP library, and compare under the stated tolerances."""
import numpy as np
import torch

from oracle import basa_oracle as o

# A block is "don't care" when the oracle's m' lies within this relative distance of the row's
# selection threshold (smallest kept m'): fp32 logits on the GPU may order such a pair differently.
MASK_REL_BAND = 1e-5
# fp32 path: max-abs against the fp64 oracle; bf16 path: max-abs and relative L2
TOL_F32_MAXABS = 1e-4
TOL_BF16_MAXABS = 2e-2
TOL_BF16_RELL2 = 5e-3


def np64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def unpack_mask(mask_bits: torch.Tensor, n_k: int) -> np.ndarray:
    """[.., N_q, words] int32 -> bool [.., N_q, n_k]"""
    w = mask_bits.detach().cpu().numpy().view(np.uint32)
    bits = ((w[..., :, None] >> np.arange(32, dtype=np.uint32)) & 1).astype(bool)
    return bits.reshape(*w.shape[:-1], -1)[..., :n_k]


def oracle_select(Q, K, hq, block, sparsity, beta, sort, window=0):
    """Oracle selection for query head hq of [1, H, L, d] tensors."""
    group = Q.shape[1] // K.shape[1]
    return o.select(np64(Q[0, hq]), np64(K[0, hq // group]), block, sparsity, beta, sort, window)


def mask_report(gpu_mask: np.ndarray, sel: dict):
    """Return (n_mismatch_outside_band, n_dontcare) for one head."""
    m, theta = sel["m"], sel["theta"][:, None]
    dontcare = np.abs(m - theta) <= MASK_REL_BAND * theta
    diff = gpu_mask != sel["mask"]
    return int((diff & ~dontcare).sum()), int(dontcare.sum())


def check_output(got: np.ndarray, want: np.ndarray, bf16: bool, what=""):
    err = np.abs(got - want)
    if bf16:
        rel = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-30)
        assert err.max() <= TOL_BF16_MAXABS, f"{what}: max-abs {err.max():.3e} > {TOL_BF16_MAXABS}"
        assert rel <= TOL_BF16_RELL2, f"{what}: rel-L2 {rel:.3e} > {TOL_BF16_RELL2}"
        return err.max(), rel
    assert err.max() <= TOL_F32_MAXABS, f"{what}: max-abs {err.max():.3e} > {TOL_F32_MAXABS}"
    return err.max(), 0.0

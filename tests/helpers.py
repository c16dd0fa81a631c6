"""Plumbing shared by the GPU parity tests: numpy bit patterns <-> torch device tensors, and a
small state object that runs the oracle's prefill-side quantiser once and mirrors it on the GPU."""
import numpy as np
import torch

import sik_workloads as W

TORCH_DT = {"fp16": torch.float16, "bf16": torch.bfloat16}


def dev(bits: np.ndarray, dtype: str) -> torch.Tensor:
    """uint16 bit patterns -> contiguous device tensor of the 16-bit float type (bit-identical)."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16).copy())
    return t.view(TORCH_DT[dtype]).cuda()


def bits_of_tensor(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def f64(bits, dtype):
    return W.from_bits(bits, dtype).astype(np.float64)


def topk_sets_agree(idx_gpu_row, idx_ref_row, s_ref_row, L, k, rel=1e-5):
    """North-star rule: |S| = min(k, L), no duplicates, all < L; every index in the symmetric
    difference has a reference score within rel * |k-th reference score| of the k-th score."""
    kk = min(k, L)
    g = [int(i) for i in idx_gpu_row if i >= 0]
    assert len(g) == kk, (len(g), kk)
    assert sum(1 for i in idx_gpu_row if i < 0) == k - kk
    assert len(set(g)) == kk, "duplicate indices"
    assert all(0 <= i < L for i in g)
    r = [int(i) for i in idx_ref_row if i >= 0]
    diff = set(g) ^ set(r)
    if not diff:
        return 0
    kth = np.sort(s_ref_row[:L])[::-1][kk - 1]
    tol = rel * abs(kth)
    for i in diff:
        assert abs(s_ref_row[i] - kth) <= tol, (i, s_ref_row[i], kth, tol)
    return len(diff)

"""CPU oracle for low-rank (LoRA) adapters served beside compressed deltas -- TEST INFRASTRUCTURE ONLY.

The engine also serves requests whose model is the base plus a low-rank adapter (paper Section 3.2:
adapters can be registered next to deltas; Section 6.4 compares the two).  For a linear layer with
base weight W [N][K] an adapter m is a pair A_m [r][K], B_m [N][r] and stands for the dense update
B_m . A_m, so for request t with adapter index m = Idx[t]

    y[t] = B_m . (A_m . x[t])                (the adapter term; zero if Idx[t] is outside [0, D))

which is the selective batched product of Section 5.2 with a low-rank matrix in place of a
compressed delta.  This file is the definition written out with library matrix products, in fp64
(operands are fp16, so every product is exact and only the sums round).  It shares no code with the
GPU library.  Pins: tests/test_oracle_lora.py (a pure-Python triple loop, the rank-1 closed form, a
zero adapter, and agreement with the dense-delta oracle on Delta = B . A).
"""
from __future__ import annotations

import numpy as np


def lora_sbmm(x, A_list, B_list, token_to_adapter, dtype=np.float64) -> np.ndarray:
    """y[t] = B_m (A_m x[t]) with m = token_to_adapter[t]; rows with m outside [0, D) are zero.
    x f16 [T][K]; A_list[m] f16 [r][K]; B_list[m] f16 [N][r].  Returns `dtype` [T][N]."""
    T, K = x.shape
    D = len(A_list)
    N = B_list[0].shape[0] if D else 0
    y = np.zeros((T, N), dtype)
    xf = x.astype(dtype)
    for t in range(T):
        m = int(token_to_adapter[t])
        if 0 <= m < D:
            u = A_list[m].astype(dtype) @ xf[t]          # [r]
            y[t] = B_list[m].astype(dtype) @ u           # [N]
    return y


def dense_update(A, B, dtype=np.float64) -> np.ndarray:
    """The dense matrix an adapter stands for: B . A, [N][K]."""
    return B.astype(dtype) @ A.astype(dtype)

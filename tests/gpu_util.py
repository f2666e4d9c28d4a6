"""Helpers shared by the GPU parity tests (marshalling and error metrics only)."""
import numpy as np
import torch

from paper_1511_04348_amd import binding as tg
from paper_1511_04348_amd import inputs


def rel_fro(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got - ref))


def run_incore(ctx, A, B, C, T, dtype=tg.TGEMM_F32):
    M, K = A.shape
    N = B.shape[1]
    torch.cuda.synchronize()      # the library's streams do not wait for torch's stream
    tg.tgemm_run(ctx, A, B, C, M, N, K, T, dtype, 0)
    torch.cuda.synchronize()
    return C


def announce(*a):
    print("[case]", *a, flush=True)

"""The allocation-free variant of the normalisation backward (pq_rmsnorm_bwd_static) against pq_rmsnorm_bwd:
same kernels, the partial rows of dgain in the library's static device array instead of a caller workspace, so
dX and dgain must agree bit for bit -- on two calls in a row, the second with a smaller input (the array keeps
the first call's partial rows)."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2602_22592_amd import binding as pq
from paper_2602_22592_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _case(seed, T, K, bf16):
    rng = np.random.default_rng(seed)
    X = wl.activations(rng, T, K, outlier_frac=0.01, outlier_scale=20.0, bf16=bf16)
    dXn = wl.normal(rng, (T, K), 1.0, bf16)
    gain = (1.0 + wl.normal(rng, (K,), 0.1, bf16)).astype(np.float32)
    dt = torch.bfloat16 if bf16 else torch.float32
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda().to(dt)
    return to(X), to(dXn), to(gain)


@pytest.mark.parametrize("bf16", [True, False])
def test_rmsnorm_bwd_static_matches_workspace_variant(bf16):
    K = 2048
    for seed, T in ((1, 1100), (2, 37)):               # the second call is smaller: stale partial rows stay behind it
        print(f"rmsnorm_bwd_static T={T} K={K} bf16={bf16}", flush=True)
        X, dXn, gain = _case(seed, T, K, bf16)
        _, _, _, _, rstd = pq.rmsnorm_quant_fwd(X, gain, 1e-6, want_xn=False, want_xt=False)
        dX_ref, dg_ref = pq.rmsnorm_bwd(dXn, X, gain, rstd)
        dX = torch.empty_like(X)
        dg = torch.empty((K,), dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        pq.rmsnorm_bwd_static_into(dXn, X, gain, rstd, dX, dg)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(dX, dX_ref)
        assert torch.equal(dg, dg_ref)
        assert torch.isfinite(dg).all()


def test_rmsnorm_bwd_static_rejects_sizes_beyond_its_scratch():
    lim = pq.rmsnorm_bwd_static_max_bytes()
    assert lim == 4 << 20
    fake = C.c_void_p(0x1000)                           # never dereferenced: validation fails first
    T, K = 16384, 2048                                  # 1024 partial rows of 8 KiB = 8 MiB
    rc = pq.lib().pq_rmsnorm_bwd_static(fake, fake, fake, fake, pq.PQ_BF16, T, K, fake, fake, None)
    assert rc == -4 and b"static scratch" in pq.lib().pq_last_error_string()

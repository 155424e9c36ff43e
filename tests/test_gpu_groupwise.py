"""Parity of the group-wise(64) contrast of the 1-bit forward (Sec. 4.6 ablation) against the CPU oracle.

Bars: the group partial sums are exact integers and the group scales are decided in the same precision on both sides
(exact fp64 mean -> fp32 -> fp16), so what differs is the fp32 accumulation over the groups and the two fp32 roundings
of the epilogue against the oracle's fp64: max|a-b| / max|b| <= 2e-6 for up to 172 groups (K = 11008), and per element
|a-b| <= 2e-6 * sum_g |lambda_g part_g| * beta / gamma.  The per-tensor form in the same kernel (group = 0) has an exact
int32 accumulator and is held to 1e-6.
"""
import numpy as np
import pytest
import torch

from oracle import pquant_oracle as po
from paper_2602_22592_amd import binding as pq
from paper_2602_22592_amd import workloads as wl

pytestmark = pytest.mark.gpu


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda().to(torch.bfloat16)


def say(msg):
    print(msg, flush=True)


def _case(seed, T, K, N, vary=True):
    rng = np.random.default_rng(seed)
    X = wl.activations(rng, T, K, outlier_frac=0.01, outlier_scale=20.0, bf16=True)
    W = wl.normal(rng, (N, K), 0.02, True)
    if vary:   # magnitudes that differ from group to group along a row, which is what group scales are for
        W = (W * np.repeat(np.exp2(rng.integers(-2, 3, size=(N, K // 64))), 64, axis=1)).astype(np.float32)
    return X, W


SHAPES = [(64, 128, 128), (300, 896, 352), (1, 64, 32), (129, 2048, 160), (77, 4096, 1024), (33, 11008, 96)]


@pytest.mark.parametrize("T,K,N", SHAPES)
def test_groupwise_forward_matches_oracle(T, K, N):
    say(f"groupwise fwd T={T} K={K} N={N}")
    X, W = _case(3100 + T, T, K, N)
    beta = 1.25
    Y = pq.groupwise_fwd(dev(X), dev(W), beta, group=64)
    torch.cuda.synchronize()
    ref = po.groupwise_fwd(X, W, beta, group=64)
    got = Y.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    assert np.abs(got - ref["Y"]).max() <= 2e-6 * np.abs(ref["Y"]).max()
    # element-wise: against the sum of the magnitudes of the terms each output adds up
    S = po.binarise(W, ref["mu"]).astype(np.int64)
    q = ref["q"].astype(np.int64)
    G = K // 64
    mag = np.zeros((T, N))
    for g in range(G):
        part = q[:, g * 64:(g + 1) * 64] @ S[:, g * 64:(g + 1) * 64].T
        mag += np.abs(part) * ref["lam_group"].astype(np.float64)[None, :, g]
    mag = beta * mag / ref["gamma"].astype(np.float64)[:, None]
    assert np.all(np.abs(got - ref["Y"]) <= 2e-6 * mag + 1e-30)


@pytest.mark.parametrize("T,K,N", SHAPES[:4])
def test_per_tensor_form_in_the_same_kernel_matches_oracle(T, K, N):
    say(f"groupwise kernel, per-tensor scale T={T} K={K} N={N}")
    X, W = _case(3200 + T, T, K, N, vary=False)
    Y = pq.groupwise_fwd(dev(X), dev(W), 0.75, group=0)
    torch.cuda.synchronize()
    ref = po.groupwise_fwd(X, W, 0.75, group=0)
    got = Y.cpu().numpy().astype(np.float64)
    assert np.abs(got - ref["Y"]).max() <= 1e-6 * np.abs(ref["Y"]).max()


def test_groupwise_config2_shape_sampled_rows():
    """Full width of the bench's workload (2048 x 2048) at 8192 tokens, oracle on sampled token rows."""
    T, K, N = 8192, 2048, 2048
    say(f"groupwise fwd full size T={T} K={K} N={N}")
    X, W = _case(3300, T, K, N)
    Y = pq.groupwise_fwd(dev(X), dev(W), 1.0, group=64)
    torch.cuda.synchronize()
    rows = np.array([0, 1, 127, 128, 4095, 6001, 8191])
    ref = po.groupwise_fwd(X[rows], W, 1.0, group=64)
    got = Y[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    assert np.abs(got - ref["Y"]).max() <= 2e-6 * np.abs(ref["Y"]).max()


def test_groupwise_rejects_what_it_does_not_run():
    X = torch.zeros((4, 96), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((32, 96), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(pq.PQError):
        pq.groupwise_fwd(X, W, 1.0, group=64)          # d_in not a multiple of 64
    X = torch.zeros((4, 128), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((32, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(pq.PQError):
        pq.groupwise_fwd(X, W, 1.0, group=32)          # only groups of 64
    Y = pq.groupwise_fwd(X[:0], W, 1.0, group=64)      # no tokens: nothing to do
    assert Y.shape == (0, 32)

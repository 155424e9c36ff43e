"""Parity of the decoupled FFN at inference on packed weights (Sec. 3.2 FFN equation, Sec. 3.3, App. A) against the
CPU oracle: the int32 accumulators of the up and gate products bit-exact, the bf16 output within 2e-2 (max-norm
relative).  The gated unit runs in fp32 on the GPU and in fp64 in the oracle, so a code of Hd may differ by one
step where silu(G) * U falls on a rounding boundary; the output tolerance covers that."""
import numpy as np
import pytest
import torch

from oracle import pquant_oracle as po
from paper_2602_22592_amd import binding as pq
from paper_2602_22592_amd import workloads as wl

pytestmark = pytest.mark.gpu


def dev(x, bf16=False):
    t = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    return t.to(torch.bfloat16) if bf16 else t


def relerr(a, b):
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    return float(np.abs(a - b).max() / max(np.abs(b).max(), 1e-30))


def _case(seed, L, D, F, E, r, B=1):
    rng = np.random.default_rng(seed)
    return dict(X=wl.activations(rng, L * B, D, bf16=True).reshape(L, B, D), Wu=wl.normal(rng, (L, F, D), 0.02, True),
                Wg=wl.normal(rng, (L, F, D), 0.02, True), Wd=wl.normal(rng, (L, D, F), 0.02, True),
                Up=wl.normal(rng, (L, E, r, D), 0.02, True), Gate=wl.normal(rng, (L, E, r, D), 0.02, True),
                Down=wl.normal(rng, (L, E, D, r), 0.02, True), Wr=wl.normal(rng, (L, E, D), 0.02, True))


def check(L, D, F, E, r, k, alpha=1.5, beta=0.4, seed=0, B=1):
    """B tokens per layer: every token of a layer is checked against the oracle's per-token FFN on that layer's weights."""
    c = _case(300 + D + F + seed + B, L, D, F, E, r, B)
    pu, pd, su, sd, lams = [], [], [], [], []
    for l in range(L):                                   # offline: binarise, pack, re-tile, fold the scalars to fp16
        Pu, _, mlu = pq.pack_sign(dev(c["Wu"][l], True))
        Pg, _, mlg = pq.pack_sign(dev(c["Wg"][l], True))
        Pd, _, mld = pq.pack_sign(dev(c["Wd"][l], True))
        lu, lg, ld = (float(m.cpu().numpy()[1]) for m in (mlu, mlg, mld))
        lams.append((np.float32(lu), np.float32(lg), np.float32(ld)))
        pu.append(torch.stack([pq.pack_retile64(Pu, D), pq.pack_retile64(Pg, D)]))
        pd.append(pq.pack_retile64(Pd, F))
        su.append([np.float16(np.float32(lu)), np.float16(np.float32(lg))])
        sd.append(np.float16(np.float32(beta) * np.float32(ld)))
    packed_ug = torch.stack(pu).contiguous()
    packed_d = torch.stack(pd).contiguous()
    scale_ug = dev(np.array(su, np.float16).view(np.int16))
    scale_d = dev(np.array(sd, np.float16).view(np.int16))
    desc = pq.DecodeFFNDesc(D, F, r, E, k, L, alpha, B)
    ws = pq.decode_ffn_workspace(desc)
    UpGate = dev(np.concatenate([c["Up"], c["Gate"]], axis=2), True)      # [L][E][2r][D]
    Y = torch.empty((L, B, D), dtype=torch.bfloat16, device="cuda")
    acc = torch.empty((L, 2, B, F), dtype=torch.int32, device="cuda")
    pq.decode_ffn(desc, dev(c["X"], True), packed_ug, scale_ug, packed_d, scale_d, UpGate, dev(c["Down"], True),
                  dev(c["Wr"], True), Y, ws, acc_upgate=acc)
    torch.cuda.synchronize()
    Y = Y.float().cpu().numpy(); acc = acc.cpu().numpy()
    worst = 0.0
    for l in range(L):
        refs = []
        for W in (c["Wu"][l], c["Wg"][l], c["Wd"][l]):
            mu, lam = po.weight_stats(W)
            refs.append((po.pack_sign(po.binarise(W, mu)), lam))
        assert tuple(np.float32(x[1]) for x in refs) == lams[l]
        f = po.decode_ffn(c["X"][l], refs[0][0], refs[1][0], refs[2][0], refs[0][1], refs[1][1], refs[2][1],
                          c["Up"][l], c["Gate"][l], c["Down"][l], c["Wr"][l], alpha, beta, top_k=k)
        assert np.array_equal(acc[l, 0].astype(np.int64), f["acc_u"]), f"layer {l}: up accumulators differ"
        assert np.array_equal(acc[l, 1].astype(np.int64), f["acc_g"]), f"layer {l}: gate accumulators differ"
        for b in range(B):
            worst = max(worst, relerr(Y[l, b], f["Y"][b]))
    print(f"  decode FFN max-norm relative error {worst:.2e}", flush=True)
    assert worst <= 2e-2


@pytest.mark.parametrize("L,D,F,E,r,k", [(1, 256, 384, 4, 16, 2), (3, 640, 1152, 8, 8, 3), (2, 2048, 5504, 8, 32, 1),
                                         (1, 128, 128, 1, 8, 1)])
def test_decode_ffn(L, D, F, E, r, k):
    print(f"decode FFN: L={L} D={D} F={F} E={E} r={r} k={k}", flush=True)
    check(L, D, F, E, r, k)


@pytest.mark.parametrize("L,B,D,F,E,r,k", [(2, 2, 256, 384, 4, 32, 2), (1, 8, 640, 1152, 8, 32, 3), (2, 5, 2048, 5504, 8, 32, 1),
                                           (1, 16, 512, 640, 2, 64, 1), (1, 11, 384, 256, 4, 32, 2),
                                           # 16 tokens x 11008 codes are more than the LDS: the down product walks them in blocks
                                           (1, 16, 256, 11008, 2, 64, 1)])
def test_decode_ffn_small_batch(L, B, D, F, E, r, k):
    """Several tokens per layer (App. A, small-batch decoding): the accumulators of the up and gate products bit-exact
    per token, every token's output within 2e-2 of the oracle's per-token FFN."""
    print(f"decode FFN batch: L={L} B={B} D={D} F={F} E={E} r={r} k={k}", flush=True)
    check(L, D, F, E, r, k, B=B)


def test_decode_ffn_config4_shape_batch8():
    print("decode FFN 4096 -> 11008 -> 4096, E=8 top-2 r=64, 8 tokens, two layers", flush=True)
    check(2, 4096, 11008, 8, 64, 2, B=8)


def test_decode_ffn_batch_limits():
    with pytest.raises(pq.PQError):
        pq.decode_ffn_workspace(pq.DecodeFFNDesc(256, 256, 16, 4, 2, 1, 1.0, 4))    # batch > 1 needs r % 32 == 0
    with pytest.raises(pq.PQError):
        pq.decode_ffn_workspace(pq.DecodeFFNDesc(256, 256, 32, 4, 2, 1, 1.0, 17))   # at most 16 tokens


def test_decode_ffn_config4_shape():
    print("decode FFN 4096 -> 11008 -> 4096, E=8 top-2 r=64, two layers", flush=True)
    check(2, 4096, 11008, 8, 64, 2)


def test_decode_ffn_expert_term_alone_and_limits():
    check(1, 256, 256, 4, 16, 2, alpha=2.0, beta=0.0, seed=5)      # beta = 0: only the experts reach the output
    check(1, 256, 256, 4, 16, 2, alpha=0.0, beta=1.0, seed=6)      # alpha = 0: only the 1-bit FFN
    with pytest.raises(pq.PQError):
        pq.decode_ffn_workspace(pq.DecodeFFNDesc(200, 256, 16, 4, 2, 1, 1.0))
    with pytest.raises(pq.PQError):
        pq.decode_ffn_workspace(pq.DecodeFFNDesc(256, 256, 0, 4, 2, 1, 1.0))


def test_decode_ffn_largest_d_ffn():
    print("decode FFN d_ffn = 16384", flush=True)
    check(1, 128, 16384, 2, 8, 1)
    print("decode FFN d_ffn = 16384, 16 tokens", flush=True)
    check(1, 128, 16384, 2, 64, 1, B=16)

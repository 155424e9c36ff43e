"""Writes tests/golden/full_size_<case>.npz: gradients that depend on EVERY token of a full-size workload
(weight gradients, scalar gradients), computed by the CPU oracle alone on the seeded inputs of
paper_2602_22592_amd/workloads.py and stored for sampled output channels.  The GPU parity tests compare the
library's results at the bench's launch configuration with these values; nothing here touches the HIP path.

    python tests/golden/make_full_size_expected.py config2      # ~1 min   (T=8192, 2048x2048, r=128)
    python tests/golden/make_full_size_expected.py config3      # ~6 min   (T=8192, d=2048, F=5504, E=8 x 32)
    python tests/golden/make_full_size_expected.py stack        # ~30 min  (2 layers at T=16384, config-5 layer shape)
    python tests/golden/make_full_size_expected.py stack1       # ~15 min  (1 layer at T=16384: the bar of a single layer applies)

The integer products of the oracle run through NumPy's int64 matmul (no BLAS), hence the run times."""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import pquant_oracle as po                    # noqa: E402
from paper_2602_22592_amd import workloads as wl         # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))
F32 = np.float32


def rss(x):
    return float(np.sqrt((np.asarray(x, np.float64) ** 2).sum()))


def config2():
    c = wl.config2()
    f = po.linear_fwd(c["X"], c["W"], 2.0, 0.2, A=c["A"], B=c["B"])
    g = po.linear_bwd(c["dY"], c["X"], c["W"], 2.0, 0.2, f, A=c["A"], B=c["B"])
    rng = np.random.default_rng(20)
    ch = np.sort(rng.choice(c["d_out"], 32, replace=False))
    dY = c["dY"].astype(np.float64)
    np.savez_compressed(os.path.join(HERE, "full_size_config2.npz"), ch=ch, dW=g["dW"][ch].astype(F32), dB=g["dB"][ch].astype(F32),
                        dA=g["dA"].astype(F32), dalpha=g["dalpha"], dbeta=g["dbeta"],
                        dalpha_scale=rss(dY * f["Yhp"]), dbeta_scale=rss(dY * f["Y1_nobeta"]))


def config3():
    c = wl.config3()
    f = po.ffn_fwd(c["X"], c["W_up"], c["W_gate"], c["W_down"], c["Up"], c["Gate"], c["Down"], c["Wr"], 2.0, 0.2, top_k=1, bf16=True)
    g = po.ffn_bwd(c["dY"], c["X"], c["Up"], c["Gate"], c["Down"], c["Wr"], 2.0, 0.2, f)
    rng = np.random.default_rng(30)
    chF = np.sort(rng.choice(c["d_ffn"], 32, replace=False))
    chD = np.sort(rng.choice(c["d_model"], 32, replace=False))
    rr = np.sort(rng.choice(c["hp_rank"], 8, replace=False))
    dY = c["dY"].astype(np.float64)
    np.savez_compressed(os.path.join(HERE, "full_size_config3.npz"), chF=chF, chD=chD, rr=rr,
                        dW_up=g["dW_up"][chF].astype(F32), dW_gate=g["dW_gate"][chF].astype(F32),
                        dW_down=g["dW_down"][chD].astype(F32), dUp=g["dUp"][:, rr].astype(F32),
                        dGate=g["dGate"][:, rr].astype(F32), dDown=g["dDown"][:, chD].astype(F32), dWr=g["dWr"].astype(F32),
                        dalpha=g["dalpha"], dbeta=g["dbeta"], dalpha_scale=rss(dY * f["Yhp"]), dbeta_scale=rss(dY * f["Y1"]),
                        counts=np.bincount(f["idx"][:, 0], minlength=c["n_experts"]))


def stack():
    L, T, D, F, E, r = 2, 16384, 2048, 5504, 8, 32
    c = wl.stack_case(11, L, T, D, F, E, r, vocab=4096)
    h0 = c["table"][c["ids"]]
    y, saved = po.stack_fwd(h0, c["layers"], top_k=1)
    d, grads = po.stack_bwd(c["dY"], c["layers"], saved)
    rng = np.random.default_rng(50)
    ch = np.sort(rng.choice(D, 16, replace=False))
    np.savez_compressed(os.path.join(HERE, "full_size_stack.npz"), ch=ch, Wq0=grads[0]["Wq"][ch].astype(F32),
                        W_down1=grads[L - 1]["W_down"][ch].astype(F32), Wo1=grads[L - 1]["Wo"][ch].astype(F32),
                        Wr0=grads[0]["Wr"].astype(F32), Wr1=grads[L - 1]["Wr"].astype(F32),
                        idx0=saved[0]["ff"]["idx"][:, 0].astype(np.int8), idx1=saved[L - 1]["ff"]["idx"][:, 0].astype(np.int8),
                        gap1=np.diff(np.sort(saved[L - 1]["ff"]["logits"], axis=1)[:, -2:], axis=1)[:, 0].astype(F32))


def stack1():
    L, T, D, F, E, r = 1, 16384, 2048, 5504, 8, 32
    c = wl.stack_case(12, L, T, D, F, E, r, vocab=4096)
    h0 = c["table"][c["ids"]]
    y, saved = po.stack_fwd(h0, c["layers"], top_k=1)
    d, grads = po.stack_bwd(c["dY"], c["layers"], saved)
    rng = np.random.default_rng(51)
    ch = np.sort(rng.choice(D, 16, replace=False))
    chF = np.sort(rng.choice(F, 16, replace=False))
    g = grads[0]
    np.savez_compressed(os.path.join(HERE, "full_size_stack1.npz"), ch=ch, chF=chF, Wq=g["Wq"][ch].astype(F32), Wk=g["Wk"][ch].astype(F32),
                        Wo=g["Wo"][ch].astype(F32), W_up=g["W_up"][chF].astype(F32), W_gate=g["W_gate"][chF].astype(F32),
                        W_down=g["W_down"][ch].astype(F32), Wr=g["Wr"].astype(F32), Up=g["Up"][:, :8].astype(F32),
                        Down=g["Down"][:, ch].astype(F32))


if __name__ == "__main__":
    for name in sys.argv[1:]:
        t = time.time()
        {"config2": config2, "config3": config3, "stack": stack, "stack1": stack1}[name]()
        print(f"{name}: {time.time() - t:.0f} s", flush=True)

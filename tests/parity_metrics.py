"""Error measures shared by the GPU parity tests (no method arithmetic here).

max-norm relative error   max|a - b| / max|b|          -- the bar the tolerances are stated in;
relative L2 error         ||a - b||_2 / ||b||_2        -- reported and asserted next to it;
per-channel max-norm      the max-norm error of every input channel (last axis) against that channel's own
                          maximum: with a few activation channels scaled up, the whole-tensor maximum of a
                          weight gradient sits in those columns and would hide errors everywhere else."""
import numpy as np


def relerr(a, b):
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    return float(np.abs(a - b).max() / max(np.abs(b).max(), 1e-30)) if b.size else 0.0


def rel_l2(a, b):
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    return float(np.sqrt(((a - b) ** 2).sum()) / max(np.sqrt((b ** 2).sum()), 1e-30)) if b.size else 0.0


def channel_relerr(a, b):
    """Worst input channel: max over the last axis of (max|a - b| over the other axes / max|b| over the other axes)."""
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    if not b.size:
        return 0.0
    a2 = a.reshape(-1, a.shape[-1]); b2 = b.reshape(-1, b.shape[-1])
    num = np.abs(a2 - b2).max(axis=0)
    den = np.maximum(np.abs(b2).max(axis=0), 1e-30 + 1e-12 * np.abs(b2).max())
    return float((num / den).max())


def report(name, a, b, per_channel=False):
    """dict of the error measures of one tensor, for printing and asserting."""
    out = {name: relerr(a, b), name + ".l2": rel_l2(a, b)}
    if per_channel:
        out[name + ".chan"] = channel_relerr(a, b)
    return out

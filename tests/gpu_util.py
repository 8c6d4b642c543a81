"""Helpers for the GPU parity tests: move the seeded inputs to the device in
their storage dtype and run the library's calls through the binding."""
import numpy as np
import torch

TOL = {"bf16": 1e-2, "f32": 1e-5}      # relative Frobenius error, from the benchmark spec
# Per-row guard beside it: max over tokens of ||dY_t|| / ||Y_t||.  The Frobenius bar alone would let
# a few garbage rows (or one bad column chunk of a few rows) through among thousands of good ones.
# Bars: the observed per-row maximum is 1.2-1.6 x the whole-tensor figure (the per-row errors of
# 2048..5120 roundings concentrate), so 2 x the Frobenius bar leaves the same margin.
ROW_TOL = {"bf16": 2e-2, "f32": 2e-5}
TDT = {"bf16": torch.bfloat16, "f32": torch.float32}


def dev(a, dtype):
    if a is None:
        return None
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda", dtype=TDT[dtype])


def host(t):
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def relf(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a - b))


OBSERVED = []      # (dtype, what, rel-Frobenius, worst row) of every comparison, for the run's summary


def row_err(a, b):
    """max_t ||a_t - b_t|| / max(||b_t||, 0.5 * rms_t ||b_t||): the worst token.  The floor: a row
    much smaller than the typical row is a cancellation among contributions of typical size (with
    a single heavy neuron, a pre-activation near zero), and the rounding errors of those
    contributions do not shrink with it (observed: 5 % of its own norm for a row at 9 % of the
    rms norm, from bf16-rounded weights, every row exact to 0.5 % of the rms norm).  A garbage
    row still scores about 1 or more."""
    a = np.asarray(a, np.float64).reshape(len(a), -1)
    b = np.asarray(b, np.float64).reshape(len(b), -1)
    if a.shape[0] == 0:
        return 0.0
    nb = np.linalg.norm(b, axis=1)
    floor = 0.5 * float(np.sqrt(np.mean(nb * nb)))
    den = np.maximum(nb, floor)
    num = np.linalg.norm(a - b, axis=1)
    if not (den > 0).all():
        return float(num.max())
    return float((num / den).max())


def assert_close(got, want, dtype, what=""):
    """Both bars of a floating-point output: relative Frobenius error over the whole tensor and
    the worst row."""
    e, r = relf(got, want), row_err(got, want)
    OBSERVED.append((dtype, what, e, r))
    assert np.isfinite(np.asarray(got)).all(), (what, "non-finite output")
    assert e < TOL[dtype], (what, "rel-Frobenius", e)
    assert r < ROW_TOL[dtype], (what, "worst row", r)
    return e, r


def elem_err(a, b):
    """max_j |a_j - b_j| / max(|b_j|, 1e-3 * max|b|): the worst entry of a score vector."""
    a = np.asarray(a, np.float64).ravel()
    b = np.asarray(b, np.float64).ravel()
    if a.size == 0:
        return 0.0
    den = np.maximum(np.abs(b), 1e-3 * float(np.abs(b).max()))
    if not (den > 0).all():
        return float(np.abs(a - b).max())
    return float((np.abs(a - b) / den).max())


def assert_scores_close(got, want, dtype, what=""):
    """Neuron scores: relative Frobenius error over the vector and the worst neuron (same bars
    as for the outputs: a score is a sum over tokens of squares of the same activations)."""
    e, r = relf(got, want), elem_err(got, want)
    OBSERVED.append((dtype, "scores " + what, e, r))
    assert np.isfinite(np.asarray(got)).all(), (what, "non-finite score")
    assert e < TOL[dtype], (what, "rel-Frobenius", e)
    assert r < ROW_TOL[dtype], (what, "worst neuron", r)
    return e, r


def desc_for(ff, cfg, rem_kind=None, k=None, rank=None):
    rk = cfg.rem_kind if rem_kind is None else rem_kind
    return ff.make_desc(cfg.d_model, cfg.d_ff, cfg.act, cfg.dtype, cfg.k if k is None else k, rk,
                        (cfg.rank if rank is None else rank) if rk == "lowrank" else 0,
                        (cfg.group or 128) if rk in ("int4", "w3h8") else 0)


def layer_to_dev(L, dtype):
    return {nm: dev(L[nm], dtype) for nm in ("W1", "W2", "Wg")}


def gpu_scores(ff, desc, Ld, Xd_batches, kind=0, reuse_tiled=False):
    """reuse_tiled: one workspace for the whole run, batches after the first reuse the re-tiled
    copy of the up projection that the first one left in it."""
    d_ff = desc.d_ff
    acc = torch.zeros(2 * d_ff, dtype=torch.float32, device="cuda")
    scores = torch.empty(d_ff, dtype=torch.float32, device="cuda")
    tt = 0
    ws = None
    if reuse_tiled:
        n = max(ff.workspace_bytes(desc, ff.WS_SCORE, x.shape[0]) for x in Xd_batches)
        ws = torch.empty(n, dtype=torch.uint8, device="cuda")
    for i, Xd in enumerate(Xd_batches):
        last = i == len(Xd_batches) - 1
        flag = ff.SCORE_REUSE_TILED if (reuse_tiled and i > 0) else 0
        tt = ff.score_neurons(desc, Xd, Ld["W1"], Ld["Wg"], Ld["W2"], acc, tt, scores if last else None, kind | flag, ws)
    torch.cuda.synchronize()
    return scores, acc, tt


GUARD = 1 << 20   # bytes of sentinel on either side of the workspace


def guarded_forward(ff, desc, split, X, want_parts=False):
    """ffsplit_forward with a workspace of exactly the size the library asks for, placed between
    two sentinel regions: any write outside the workspace (a scratch buffer sized too small for a
    launch) shows up as a changed sentinel byte even where it would not fault."""
    n = ff.workspace_bytes(desc, ff.WS_FORWARD, X.shape[0])
    buf = torch.full((n + 2 * GUARD,), 0xA5, dtype=torch.uint8, device=X.device)
    out = ff.forward(desc, split, X, None, want_parts, buf[GUARD:GUARD + n])
    torch.cuda.synchronize()
    assert bool((buf[:GUARD] == 0xA5).all()), "write below the workspace"
    assert bool((buf[GUARD + n:] == 0xA5).all()), "write beyond the workspace"
    return out


class Guarded:
    """A device buffer of exactly n bytes between two sentinel regions (256-byte aligned start)."""

    def __init__(self, n, device="cuda"):
        self.n = int(n)
        self.buf = torch.full((self.n + 2 * GUARD,), 0xA5, dtype=torch.uint8, device=device)
        self.view = self.buf[GUARD:GUARD + self.n]

    def check(self, what):
        torch.cuda.synchronize()
        assert bool((self.buf[:GUARD] == 0xA5).all()), f"{what}: write below the buffer"
        assert bool((self.buf[GUARD + self.n:] == 0xA5).all()), f"{what}: write beyond the buffer"

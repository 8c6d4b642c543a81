"""Seeded generators.  Everything is drawn in fp32 from numpy's counter-based
Philox generator, then rounded (round-to-nearest-even) to the storage dtype and
handed out as fp32 arrays whose values are exactly representable in that dtype,
so the oracle (upcasting to fp64) and the GPU path (converting to bf16/fp16
tensors) start from bit-identical numbers."""
import numpy as np

from .configs import FFNConfig

# stream ids that enter the seed
S_WEIGHTS, S_PLANTED, S_EVAL, S_CALIB, S_FACTORS = 0, 1, 2, 3, 4


def seed_for(cfg: FFNConfig, stream: int, layer: int = 0) -> int:
    """seed = 1000*config + stream + 10*layer; the BERT-shaped config keeps the
    literal seeds 0 (weights), 1 (planted set), 2 (eval tokens) it is stated with."""
    if cfg.index == 1 and layer == 0:
        return stream
    return 1000 * cfg.index + stream + 10 * layer


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=seed))


def bf16_round(a, inplace: bool = False) -> np.ndarray:
    """fp32 -> nearest bf16 (ties to even) -> fp32.  NaN/Inf pass through.
    Works through the array in blocks with small scratch buffers (the matrices of the large
    layers hold 10^8 entries, and fresh pages are the expensive part); inplace=True overwrites
    a contiguous fp32 array instead of returning a copy."""
    src = np.ascontiguousarray(a, dtype=np.float32)
    dst = src if (inplace and src is a) else np.empty_like(src)
    u = src.reshape(-1).view(np.uint32)
    o = dst.reshape(-1).view(np.uint32)
    blk = 1 << 20
    r = np.empty(blk, np.uint32)
    e = np.empty(blk, np.uint32)
    for lo in range(0, u.size, blk):
        ub = u[lo:lo + blk]
        n = ub.size
        rb, eb = r[:n], e[:n]
        np.right_shift(ub, np.uint32(16), out=rb)
        rb &= np.uint32(1)
        rb += np.uint32(0x7FFF)
        rb += ub
        rb &= np.uint32(0xFFFF0000)
        np.bitwise_and(ub, np.uint32(0x7F800000), out=eb)
        nonfinite = eb == np.uint32(0x7F800000)
        if nonfinite.any():
            rb[nonfinite] = ub[nonfinite]
        o[lo:lo + n] = rb
    return dst.reshape(src.shape)


def fp16_round(a) -> np.ndarray:
    return np.asarray(a, dtype=np.float32).astype(np.float16).astype(np.float32)


def storage_round(a, dtype: str, inplace: bool = False) -> np.ndarray:
    if dtype == "bf16":
        return bf16_round(a, inplace)
    if dtype == "f16":
        return fp16_round(a)
    return np.ascontiguousarray(a, dtype=np.float32)


def planted_set(cfg: FFNConfig, layer: int = 0) -> np.ndarray:
    """The k planted heavy neurons: first k entries of a seeded permutation, sorted."""
    perm = _rng(seed_for(cfg, S_PLANTED, layer)).permutation(cfg.d_ff)
    return np.sort(perm[: cfg.k]).astype(np.int32)


def make_layer(cfg: FFNConfig, layer: int = 0) -> dict:
    """Dense weights W1 [d, d_ff], W2 [d_ff, d] (and Wg [d, d_ff] for SwiGLU):
    i.i.d. N(0, weight_std^2); the planted neurons' W1/Wg column and W2 row are
    multiplied by heavy_scale; then rounded to the storage dtype."""
    rng = _rng(seed_for(cfg, S_WEIGHTS, layer))
    d, f = cfg.d_model, cfg.d_ff
    planted = planted_set(cfg, layer)
    out = {"planted": planted}
    names = ["W1", "W2"] + (["Wg"] if cfg.act == "swiglu" else [])
    for nm in names:
        shape = (f, d) if nm == "W2" else (d, f)
        w = rng.standard_normal(shape, dtype=np.float32)
        w *= np.float32(cfg.weight_std)
        if nm == "W2":
            w[planted, :] *= np.float32(cfg.heavy_scale)
        else:
            w[:, planted] *= np.float32(cfg.heavy_scale)
        out[nm] = storage_round(w, cfg.dtype, inplace=True)
    if "Wg" not in out:
        out["Wg"] = None
    return out


def make_tokens(cfg: FFNConfig, T: int, stream: int = S_EVAL, layer: int = 0) -> np.ndarray:
    """T tokens x ~ N(0, 1) of width d_model, rounded to the storage dtype."""
    rng = _rng(seed_for(cfg, stream, layer) + 100000)
    x = rng.standard_normal((T, cfg.d_model), dtype=np.float32)
    return storage_round(x, cfg.dtype, inplace=True)


def remainder_order(idx, d_ff: int) -> np.ndarray:
    """Indices not in idx, ascending: the neuron order the factor inputs refer to."""
    mask = np.ones(d_ff, dtype=bool)
    mask[np.asarray(idx, dtype=np.int64)] = False
    return np.nonzero(mask)[0].astype(np.int32)


def truncated_factors(W: np.ndarray, r: int):
    """Best rank-r factors of W [p, q] (fp64): W ~= P @ Q, P [p, r], Q [r, q],
    from the eigen-decomposition of the Gram matrix on W's smaller side.  The
    singular values are shared evenly (sqrt each) between P and Q."""
    W = np.ascontiguousarray(W, dtype=np.float64)
    p, q = W.shape
    if p <= q:
        lam, L = np.linalg.eigh(W @ W.T)            # ascending
        L = np.ascontiguousarray(L[:, ::-1][:, :r])
        s = np.sqrt(np.maximum(lam[::-1][:r], 0.0))
        Rt = (L.T @ W) / np.where(s > 0, s, 1.0)[:, None]
    else:
        lam, R = np.linalg.eigh(W.T @ W)
        R = np.ascontiguousarray(R[:, ::-1][:, :r])
        s = np.sqrt(np.maximum(lam[::-1][:r], 0.0))
        Rt = R.T
        L = (W @ R) / np.where(s > 0, s, 1.0)[None, :]
    rs = np.sqrt(s)
    return L * rs[None, :], rs[:, None] * Rt


def gaussian_factors(p: int, q: int, r: int, std: float, rng: np.random.Generator):
    """Stand-in factors of the right shape whose product has entries of std `std`."""
    a = np.sqrt(std / np.sqrt(r))
    P = rng.standard_normal((p, r), dtype=np.float32)
    P *= np.float32(a)
    Q = rng.standard_normal((r, q), dtype=np.float32)
    Q *= np.float32(a)
    return P, Q


def make_factors(cfg: FFNConfig, layer_w: dict, idx, layer: int = 0, rank: int = None) -> dict:
    """Factor inputs of the low-rank remainder, each remainder matrix factored on
    its own at the same rank: W1[:, rest] ~= P1 Q1, Wg[:, rest] ~= Pg Qg,
    W2[rest, :] ~= P2 Q2 with rest = remainder_order(idx).  Rounded to storage dtype."""
    r = cfg.rank if rank is None else rank
    rest = remainder_order(idx, cfg.d_ff)
    rng = _rng(seed_for(cfg, S_FACTORS, layer))
    out = {}
    for tag, nm in (("1", "W1"), ("g", "Wg"), ("2", "W2")):
        W = layer_w.get(nm)
        if W is None:
            out["P" + tag] = out["Q" + tag] = None
            continue
        Wr = W[rest, :] if nm == "W2" else W[:, rest]
        if cfg.exact_svd:
            P, Q = truncated_factors(Wr, r)
        else:
            P, Q = gaussian_factors(Wr.shape[0], Wr.shape[1], r, cfg.weight_std, rng)
        out["P" + tag] = storage_round(P, cfg.dtype)
        out["Q" + tag] = storage_round(Q, cfg.dtype)
    return out

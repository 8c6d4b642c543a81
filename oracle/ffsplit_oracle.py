"""CPU oracle for the split feed-forward path (FFSplit, arXiv 2401.04044).

TEST INFRASTRUCTURE ONLY.  Plain numpy in fp64, written from the paper's
equations; it shares no code with the HIP library and never imports it.  Only
the tests, the smoke check and the benchmark's cpu_baseline leg may call it.

Every function names the passage it follows.  All floating-point work is fp64
with no intermediate rounding, except the group-wise quantiser, whose decisions
(scale, integer code) are taken in fp32/fp16 exactly as specified there so that
a GPU implementation can agree bit for bit.

Pins (tests/test_oracle_pins.py): dense special cases (heavy = all neurons,
full-rank factors), Y = Y1 + Y2, the neuron-removal identity of Sec. 4.1 by
brute force, exhaustive ranking for top-k, enumeration of the levels of the 3-,
4- and 8-bit quantiser,
closed-form identities of GeLU/SiLU, the parameter-count figure of Sec. 5.1.1;
the biased layer and the residual against pure-Python loops, the unbiased case and
a permutation of the neurons together with their biases;
the randomised factorisation against exact recovery, the projector identities,
Eckart-Young from below and the published expected-error bound from above.
Forward outputs at the full workload shapes have no pin beyond those identities
holding at full shape: parity unpinned there (the oracle is the definition).

Notation: the paper's U (d x d_ff) is W1 here, its V (d_ff x d) is W2; Wg is
the SwiGLU gate.  h2 = heavy set, k = |h2|, m = d_ff - k.
"""
import math

import numpy as np
from scipy.special import erf as _erf

F64 = np.float64

# ---------------------------------------------------------------- activations


def gelu(z):
    """GeLU in its exact form z * Phi(z) (the activation Sec. 2 cites)."""
    z = np.asarray(z, dtype=F64)
    return 0.5 * z * (1.0 + _erf(z / math.sqrt(2.0)))


def silu(z):
    """SiLU z * sigmoid(z), the gate non-linearity of SwiGLU (Sec. 2 cites it)."""
    z = np.asarray(z, dtype=F64)
    with np.errstate(over="ignore"):
        return z / (1.0 + np.exp(-z))


def neuron_activations(X, W1, Wg=None, act="gelu"):
    """H[t, j] = sigma(X U[:, j]) of Sec. 2's first equation; for SwiGLU neuron
    j's activation is silu(X Wg[:, j]) * (X W1[:, j])."""
    X = np.asarray(X, F64)
    Z = X @ np.asarray(W1, F64)
    if act == "gelu":
        return gelu(Z)
    if act == "swiglu":
        return silu(X @ np.asarray(Wg, F64)) * Z
    raise ValueError(act)


def dense_ffn(X, W1, W2, Wg=None, act="gelu"):
    """FFN(X) = sigma(X U) V  (Sec. 2, first equation)."""
    return neuron_activations(X, W1, Wg, act) @ np.asarray(W2, F64)


def dense_ffn_rank_one(X, W1, W2, Wg=None, act="gelu"):
    """Eq. 1: the same FFN as a sum of d_ff rank-one terms (slow, tiny inputs)."""
    X = np.asarray(X, F64)
    Y = np.zeros((X.shape[0], np.asarray(W2).shape[1]), F64)
    for j in range(np.asarray(W1).shape[1]):
        Y += rank_one_term(X, W1, W2, j, Wg, act)
    return Y


def rank_one_term(X, W1, W2, j, Wg=None, act="gelu"):
    """sigma(X U[:, j]) V[j, :] : neuron j's contribution in Eq. 1."""
    X = np.asarray(X, F64)
    wg = None if Wg is None else np.asarray(Wg, F64)[:, j:j + 1]
    h = neuron_activations(X, np.asarray(W1, F64)[:, j:j + 1], wg, act)
    return h @ np.asarray(W2, F64)[j:j + 1, :]


# ---------------------------------------------------------------- calibration

SCORE_SUMSQ, SCORE_MEAN_L2, SCORE_ACT_ONLY = 0, 1, 2


def new_accumulator(d_ff):
    """Running per-neuron sums over calibration tokens: S2 = sum_t H^2,
    S1 = sum_t |H|, and the token count."""
    return {"S2": np.zeros(d_ff, F64), "S1": np.zeros(d_ff, F64), "T": 0}


def score_accumulate(acc, X, W1, Wg=None, act="gelu"):
    """One calibration batch (Sec. 4.2, first step): add this batch's tokens to
    ||sigma(X U[:, j])||_F^2 (and to the L1 sum) for every neuron j."""
    H = neuron_activations(X, W1, Wg, act)
    acc["S2"] += np.sum(H * H, axis=0)
    acc["S1"] += np.sum(np.abs(H), axis=0)
    acc["T"] += H.shape[0]
    return acc


def row_sqnorms(W2):
    """||V[j, :]||_F^2, the second factor of Eq. 3."""
    W2 = np.asarray(W2, F64)
    return np.sum(W2 * W2, axis=1)


def neuron_scores(acc, W2, kind=SCORE_SUMSQ):
    """Importance score of every neuron.
    SUMSQ    : Eq. 3's last line, ||sigma(X U[:, j])||_F^2 * ||V[j, :]||_F^2.
    MEAN_L2  : mean over tokens of ||sigma(x U[:, j]) V[j, :]||_2
               = (S1 / T) * ||V[j, :]||_2 (the per-token-norm wording).
    ACT_ONLY : ||sigma(X U[:, j])||_F^2 alone (Sec. 2's definition of a heavy hitter).
    """
    n2 = row_sqnorms(W2)
    if kind == SCORE_SUMSQ:
        s = acc["S2"] * n2
    elif kind == SCORE_MEAN_L2:
        s = (acc["S1"] / max(acc["T"], 1)) * np.sqrt(n2)
    elif kind == SCORE_ACT_ONLY:
        s = acc["S2"].copy()
    else:
        raise ValueError(kind)
    return s + 0.0  # -0 -> +0


def select_heavy(scores, k):
    """Indices of the k highest scores (Sec. 4.1/5.1.1: neurons with the highest
    score are the heavy hitters), ordered by score descending; equal scores are
    ordered by the lower index first.  NaN scores are an error."""
    s = np.asarray(scores)
    if np.isnan(s).any():
        raise ValueError("NaN score")
    if not 0 <= k <= s.shape[0]:
        raise ValueError("k out of range")
    order = np.lexsort((np.arange(s.shape[0]), -s.astype(F64)))
    return order[:k].astype(np.int32)


# ---------------------------------------------------------------- split

def neuron_permutation(idx, d_ff):
    """[h2 in the given order ; all other neurons ascending] (Eq. 2's partition)."""
    idx = np.asarray(idx, dtype=np.int64)
    mask = np.ones(d_ff, dtype=bool)
    mask[idx] = False
    if mask.sum() != d_ff - idx.shape[0]:
        raise ValueError("duplicate heavy index")
    return np.concatenate([idx, np.nonzero(mask)[0]]).astype(np.int32)


def split_weights(W1, W2, Wg, idx):
    """Fig. 3's caption: U1 = U[:, h2], V1 = V[h2, :]; U2, V2 the rest."""
    d_ff = np.asarray(W1).shape[1]
    perm = neuron_permutation(idx, d_ff)
    k = len(idx)
    h, r = perm[:k], perm[k:]
    out = {"perm": perm,
           "W1h": np.asarray(W1, F64)[:, h], "W2h": np.asarray(W2, F64)[h, :],
           "W1r": np.asarray(W1, F64)[:, r], "W2r": np.asarray(W2, F64)[r, :],
           "Wgh": None, "Wgr": None}
    if Wg is not None:
        out["Wgh"] = np.asarray(Wg, F64)[:, h]
        out["Wgr"] = np.asarray(Wg, F64)[:, r]
    return out


# ---------------------------------------------------------------- int4 remainder

def quantize_rtn(V, group, bits=4):
    """Round-to-nearest, symmetric, group-wise quantisation (Sec. 5.2: RTN with
    group size 128) of each row of V [n, d] in groups of `group` along d.
    All decisions in fp32, the scale stored as fp16:
        a = max |w| over the group;  s = fp16(a / qmax), qmax = 2^(bits-1) - 1;
        s == 0 -> q = 0;  else q = clamp(rint(w / float(s)), -qmax-1, qmax)
    with rint = round-half-to-even and IEEE fp32 division.
    Returns q int8 [n, d] and s fp16 [n, d/group]."""
    V = np.ascontiguousarray(V, dtype=np.float32)
    n, d = V.shape
    if d % group:
        raise ValueError("group must divide the row length")
    qmax = np.float32((1 << (bits - 1)) - 1)
    g = V.reshape(n, d // group, group)
    a = np.max(np.abs(g), axis=2)
    with np.errstate(over="ignore"):
        s16 = (a / qmax).astype(np.float32).astype(np.float16)
    s32 = s16.astype(np.float32)
    safe = np.where(s32 > 0, s32, np.float32(1.0))
    q = np.rint((g / safe[:, :, None]).astype(np.float32))
    q = np.clip(q, -qmax - 1, qmax)
    q = np.where((s32 > 0)[:, :, None], q, 0.0)
    return q.astype(np.int8).reshape(n, d), s16


def dequantize(q, s, group):
    """w^ = float(s) * q, exact in fp64."""
    n, d = q.shape
    return (q.reshape(n, d // group, group).astype(F64)
            * s.astype(F64)[:, :, None]).reshape(n, d)


# ---------------------------------------------------------------- forward

def _act_pair(Z, G, act):
    if act == "gelu":
        return gelu(Z)
    return silu(G) * Z


def forward_heavy(X, sw, act):
    """FFN_1 of Eq. 2: the heavy neurons, weights untouched (Sec. 4.2)."""
    X = np.asarray(X, F64)
    G = None if sw["Wgh"] is None else X @ sw["Wgh"]
    return _act_pair(X @ sw["W1h"], G, act) @ sw["W2h"]


def forward_remainder_dense(X, sw, act):
    """FFN_2 of Eq. 2 with the remainder left uncompressed."""
    X = np.asarray(X, F64)
    G = None if sw["Wgr"] is None else X @ sw["Wgr"]
    return _act_pair(X @ sw["W1r"], G, act) @ sw["W2r"]


def forward_remainder_lowrank(X, fac, act):
    """FFN_2 with U2 ~= P1 Q1 (and the gate ~= Pg Qg) and V2 ~= P2 Q2, each
    remainder matrix factored on its own (Sec. 4.2 / 5.1.1), evaluated as
    written: sigma((X P1) Q1) P2 Q2."""
    X = np.asarray(X, F64)
    Z = (X @ np.asarray(fac["P1"], F64)) @ np.asarray(fac["Q1"], F64)
    G = None
    if act == "swiglu":
        G = (X @ np.asarray(fac["Pg"], F64)) @ np.asarray(fac["Qg"], F64)
    H = _act_pair(Z, G, act)
    return (H @ np.asarray(fac["P2"], F64)) @ np.asarray(fac["Q2"], F64)


def quantize_remainder(sw, group, bits=4):
    """Quantise every remainder neuron's up column, gate column and down row in
    groups along d_model.  Returns {name: (q [m, d], s [m, d/group])}."""
    out = {"W1r": quantize_rtn(sw["W1r"].T, group, bits),
           "W2r": quantize_rtn(sw["W2r"], group, bits)}
    if sw["Wgr"] is not None:
        out["Wgr"] = quantize_rtn(sw["Wgr"].T, group, bits)
    return out


def forward_remainder_int4(X, qw, group, act):
    """FFN_2 with the remainder's weights replaced by their dequantised values."""
    X = np.asarray(X, F64)
    Z = X @ dequantize(*qw["W1r"], group).T
    G = None
    if act == "swiglu":
        G = X @ dequantize(*qw["Wgr"], group).T
    return _act_pair(Z, G, act) @ dequantize(*qw["W2r"], group)


def quantize_heavy(sw, group, bits=8):
    """Sec. 5.2, the LLM setting: the heavy neurons are quantised too, at a
    higher bit width (8 bits, group 128), each neuron's up column, gate column
    and down row in groups along d_model like the remainder's.
    Returns {name: (q [k, d], s [k, d/group])}."""
    out = {"W1h": quantize_rtn(sw["W1h"].T, group, bits),
           "W2h": quantize_rtn(sw["W2h"], group, bits)}
    if sw["Wgh"] is not None:
        out["Wgh"] = quantize_rtn(sw["Wgh"].T, group, bits)
    return out


def forward_heavy_quant(X, qh, group, act):
    """FFN_1 with the heavy neurons' weights replaced by their dequantised values."""
    X = np.asarray(X, F64)
    Z = X @ dequantize(*qh["W1h"], group).T
    G = None
    if act == "swiglu":
        G = X @ dequantize(*qh["Wgh"], group).T
    return _act_pair(Z, G, act) @ dequantize(*qh["W2h"], group)


def forward_split(X, W1, W2, Wg, idx, act, rem_kind, factors=None, group=128, bits=4, heavy_bits=8):
    """Eq. 2: Y = FFN_1(X) + FFN_2~(X).  rem_kind: "none" (FFN_2 dropped),
    "dense", "lowrank" (factors refer to the remainder in ascending index
    order), "int4" (remainder at `bits`, heavy untouched), "w3h8" (Sec. 5.2's
    pairing for the LLMs: heavy at heavy_bits = 8, remainder at 3 bits, both
    round-to-nearest with the same group length).  Returns (Y, Y1, Y2)."""
    sw = split_weights(W1, W2, Wg, idx)
    if rem_kind == "w3h8":
        k, m = sw["W1h"].shape[1], sw["W1r"].shape[1]
        X64 = np.asarray(X, F64)
        zero = np.zeros((X64.shape[0], np.asarray(W2).shape[1]), F64)
        Y1 = forward_heavy_quant(X, quantize_heavy(sw, group, heavy_bits), group, act) if k else zero
        Y2 = forward_remainder_int4(X, quantize_remainder(sw, group, 3), group, act) if m else zero
        return Y1 + Y2, Y1, Y2
    Y1 = forward_heavy(X, sw, act)
    if rem_kind == "none" or sw["W1r"].shape[1] == 0:
        Y2 = np.zeros_like(Y1)
    elif rem_kind == "dense":
        Y2 = forward_remainder_dense(X, sw, act)
    elif rem_kind == "lowrank":
        Y2 = forward_remainder_lowrank(X, factors, act)
    elif rem_kind == "int4":
        Y2 = forward_remainder_int4(X, quantize_remainder(sw, group, bits), group, act)
    else:
        raise ValueError(rem_kind)
    return Y1 + Y2, Y1, Y2


# ---------------------------------------------------------------- biases and the residual connection

def dense_ffn_biased(X, W1, W2, b1=None, b2=None):
    """The feed-forward layer as the models of Sec. 5.1 / 5.2 (BERT, OPT) define it, biases
    included: gelu(X U + b1) V + b2.  Sec. 2's first equation is the case b1 = b2 = 0."""
    X = np.asarray(X, F64)
    Z = X @ np.asarray(W1, F64)
    if b1 is not None:
        Z = Z + np.asarray(b1, F64)[None, :]
    Y = gelu(Z) @ np.asarray(W2, F64)
    if b2 is not None:
        Y = Y + np.asarray(b2, F64)[None, :]
    return Y


def forward_split_biased(X, W1, W2, idx, rem_kind, factors=None, b1=None, b2=None, residual=None):
    """Eq. 2 for a GeLU layer with biases and, optionally, the residual connection around it.
    A neuron's bias belongs to the neuron (it is the constant term of its pre-activation), so
    it moves with it in the partition: FFN_1 uses b1[h2]; the remainder, whose up projection is
    compressed, adds b1[rest] to the compressed pre-activation: gelu((X P1) Q1 + b1[rest]).
    b2 is not a neuron's: it is added once to the sum.  residual [T, d]: the layer's input
    stream, Y = residual + FFN_1 + FFN_2 + b2 (Sec. 4.1 applies the split at each layer of a
    model whose layers are wrapped this way).  Returns (Y, Y1, Y2), Y1 and Y2 without b2 and
    without the residual."""
    X = np.asarray(X, F64)
    sw = split_weights(W1, W2, None, idx)
    k = len(idx)
    perm = sw["perm"]
    b1 = np.zeros(np.asarray(W1).shape[1], F64) if b1 is None else np.asarray(b1, F64)
    bh, br = b1[perm[:k]], b1[perm[k:]]
    Y1 = gelu(X @ sw["W1h"] + bh[None, :]) @ sw["W2h"]
    if rem_kind == "none" or sw["W1r"].shape[1] == 0:
        Y2 = np.zeros_like(Y1)
    elif rem_kind == "dense":
        Y2 = gelu(X @ sw["W1r"] + br[None, :]) @ sw["W2r"]
    elif rem_kind == "lowrank":
        Z = (X @ np.asarray(factors["P1"], F64)) @ np.asarray(factors["Q1"], F64) + br[None, :]
        Y2 = (gelu(Z) @ np.asarray(factors["P2"], F64)) @ np.asarray(factors["Q2"], F64)
    else:
        raise ValueError(rem_kind)
    Y = Y1 + Y2
    if b2 is not None:
        Y = Y + np.asarray(b2, F64)[None, :]
    if residual is not None:
        Y = np.asarray(residual, F64) + Y
    return Y, Y1, Y2


# ---------------------------------------------------------------- remainder factorisation on the device's plan

def _fmix32(h):
    """Finaliser of the public MurmurHash3 (32-bit), on uint64 arrays holding 32-bit values."""
    m = np.uint64(0xFFFFFFFF)
    h = h & m
    h ^= h >> np.uint64(16)
    h = (h * np.uint64(0x85EBCA6B)) & m
    h ^= h >> np.uint64(13)
    h = (h * np.uint64(0xC2B2AE35)) & m
    h ^= h >> np.uint64(16)
    return h


def rademacher(seed, stream, n_rows, n_cols):
    """Test matrix of the randomised range finder: entry (i, j) = +1 / -1 from the top bit of
    fmix32(index * 0x9E3779B1 + fmix32(seed + 0x9E3779B9 * stream)), index = i * n_cols + j.
    A counter-based generator, so that the device draws exactly the same signs."""
    m = np.uint64(0xFFFFFFFF)
    key = _fmix32(np.array([(int(seed) + 0x9E3779B9 * int(stream)) & 0xFFFFFFFF], np.uint64))[0]
    idx = np.arange(n_rows * n_cols, dtype=np.uint64)
    h = _fmix32(((idx * np.uint64(0x9E3779B1)) & m) + key)
    return np.where((h >> np.uint64(31)) & np.uint64(1), -1.0, 1.0).reshape(n_rows, n_cols)


def range_finder(Z, r, seed, stream):
    """Randomised range finder (Halko, Martinsson, Tropp 2011, Alg. 4.1) for Z [d, m], m
    columns: Y = Z Omega^T with a Rademacher test matrix Omega [r, m], B = an orthonormal basis
    of range(Y) [d, r]; the rank-r approximation is B (B^T Z).  Stands in for the SVD of
    Sec. 5.1.1 where the split is built on the device.  Returns (B, B^T Z)."""
    Z = np.asarray(Z, F64)
    Om = rademacher(seed, stream, r, Z.shape[1])
    B, _ = np.linalg.qr(Z @ Om.T)
    return B, B.T @ Z


def factorize_remainder(W1, W2, Wg, idx, r, seed):
    """Rank-r factors of each remainder matrix on its own (Sec. 4.2 / 5.1.1), by the range
    finder above on the d_model side of every matrix: streams 0 (W1), 1 (Wg), 2 (W2).
    Same conventions as the factors forward_remainder_lowrank takes."""
    sw = split_weights(W1, W2, Wg, idx)
    out = {}
    B, C = range_finder(sw["W1r"], r, seed, 0)
    out["P1"], out["Q1"] = B, C
    if sw["Wgr"] is not None:
        B, C = range_finder(sw["Wgr"], r, seed, 1)
        out["Pg"], out["Qg"] = B, C
    B, C = range_finder(sw["W2r"].T, r, seed, 2)
    out["P2"], out["Q2"] = C.T, B.T
    return out


# ---------------------------------------------------------------- layer stack

def token_rms_normalise(x, eps=1e-6):
    """n(x) = x / sqrt(mean(x^2) + eps) per token, no learned scale: the pre-norm
    that keeps a 40-layer residual stack of these synthetic layers finite."""
    x = np.asarray(x, F64)
    return x / np.sqrt(np.mean(x * x, axis=1, keepdims=True) + eps)


def stack_calibrate_layer(x, layer_w, act, acc):
    """One layer of the calibration pass: heavy hitters are identified on the
    unmodified model (Sec. 4.2), so the residual stream moves through the dense
    layer: x <- x + FFN(n(x)); scores accumulate on n(x)."""
    xn = token_rms_normalise(x)
    score_accumulate(acc, xn, layer_w["W1"], layer_w["Wg"], act)
    return x + dense_ffn(xn, layer_w["W1"], layer_w["W2"], layer_w["Wg"], act), xn


def stack_forward_layer(x, layer_w, idx, act, rem_kind, factors=None, group=128):
    """One layer of inference through the split model: x <- x + FFN_split(n(x))."""
    xn = token_rms_normalise(x)
    Y, _, _ = forward_split(xn, layer_w["W1"], layer_w["W2"], layer_w["Wg"], idx, act,
                            rem_kind, factors, group)
    return x + Y, xn


# ---------------------------------------------------------------- bookkeeping

def split_param_count(d, d_ff, k, r):
    """Parameters of one split GeLU FFN with both remainder matrices factored at
    rank r: 2 d k heavy + 2 r (d + m) factors."""
    return 2 * d * k + 2 * r * (d + (d_ff - k))


def rel_frobenius(a, b):
    a = np.asarray(a, F64)
    b = np.asarray(b, F64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a - b))

"""ctypes binding: same names as the C ABI, argument marshalling only."""
import ctypes
import os

import torch

ACT_GELU, ACT_SWIGLU = 0, 1
F32, BF16 = 0, 1
REM_NONE, REM_DENSE, REM_LOWRANK, REM_INT4, REM_W3H8 = 0, 1, 2, 3, 4
SCORE_SUMSQ, SCORE_MEAN_L2, SCORE_ACT_ONLY = 0, 1, 2
SCORE_REUSE_TILED = 0x100
WS_SCORE, WS_SELECT, WS_BUILD, WS_FORWARD, WS_FACTORIZE, WS_STACK = 0, 1, 2, 3, 4, 5
E_NONFINITE = -7

_HERE = os.path.dirname(os.path.abspath(__file__))


def lib_path() -> str:
    return os.path.join(_HERE, "libffsplit.so")


class FFSplitError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {status_string(code)} ({code})")


class Epilogue(ctypes.Structure):
    _fields_ = [("b1_packed", ctypes.c_void_p), ("b2", ctypes.c_void_p), ("residual", ctypes.c_void_p),
                ("y_f32", ctypes.c_int32)]


class Desc(ctypes.Structure):
    _fields_ = [("d_model", ctypes.c_int32), ("d_ff", ctypes.c_int32), ("act", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("k", ctypes.c_int32), ("rem_kind", ctypes.c_int32),
                ("rank", ctypes.c_int32), ("group", ctypes.c_int32)]


def _load():
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    L = ctypes.CDLL(path)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    dp = ctypes.POINTER(Desc)
    L.ffsplit_status_string.restype = ctypes.c_char_p
    L.ffsplit_status_string.argtypes = [ctypes.c_int]
    L.ffsplit_workspace_bytes.restype = sz
    L.ffsplit_workspace_bytes.argtypes = [dp, i32, i64]
    L.ffsplit_split_bytes.restype = sz
    L.ffsplit_split_bytes.argtypes = [dp]
    L.ffsplit_score_neurons.restype = ctypes.c_int
    L.ffsplit_score_neurons.argtypes = [dp, vp, i64, vp, vp, vp, vp, ctypes.POINTER(i64), vp, i32, vp, sz, vp]
    L.ffsplit_select_heavy.restype = ctypes.c_int
    L.ffsplit_select_heavy.argtypes = [vp, i32, i32, vp, vp, vp, vp, sz, vp]
    L.ffsplit_select_heavy_static.restype = ctypes.c_int
    L.ffsplit_select_heavy_static.argtypes = [vp, i32, i32, vp, vp, vp, vp]
    L.ffsplit_build_split.restype = ctypes.c_int
    L.ffsplit_build_split.argtypes = [dp, vp, vp, vp, vp, ctypes.POINTER(vp), vp, vp, sz, vp]
    L.ffsplit_forward.restype = ctypes.c_int
    L.ffsplit_forward.argtypes = [dp, vp, vp, i64, vp, vp, vp, vp, sz, vp]
    L.ffsplit_forward_ex.restype = ctypes.c_int
    L.ffsplit_forward_ex.argtypes = [dp, vp, vp, i64, vp, vp, vp, ctypes.POINTER(Epilogue), vp, sz, vp]
    L.ffsplit_neuron_bias_floats.restype = sz
    L.ffsplit_neuron_bias_floats.argtypes = [dp]
    L.ffsplit_pack_neuron_bias.restype = ctypes.c_int
    L.ffsplit_pack_neuron_bias.argtypes = [dp, vp, vp, vp, vp, sz, vp]
    L.ffsplit_token_rmsnorm.restype = ctypes.c_int
    L.ffsplit_token_rmsnorm.argtypes = [vp, i64, i32, ctypes.c_float, i32, vp, vp]
    L.ffsplit_stack_forward.restype = ctypes.c_int
    L.ffsplit_stack_forward.argtypes = [dp, i32, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), vp, i64,
                                        ctypes.c_float, vp, sz, vp]
    L.ffsplit_probe_mfma.restype = ctypes.c_int
    L.ffsplit_probe_mfma.argtypes = [i32, i32, vp, ctypes.POINTER(ctypes.c_double), vp]
    L.ffsplit_probe_stream_read.restype = ctypes.c_int
    L.ffsplit_probe_stream_read.argtypes = [vp, sz, i32, vp, vp]
    L.ffsplit_factorize_remainder.restype = ctypes.c_int
    L.ffsplit_factorize_remainder.argtypes = [dp, vp, vp, vp, vp, ctypes.c_uint32, ctypes.POINTER(vp), vp, sz, vp]
    L.ffsplit_split_export.restype = ctypes.c_int
    L.ffsplit_split_export.argtypes = [dp, vp, i32, vp, vp, vp]
    return L


lib = _load()


def status_string(code: int) -> str:
    return lib.ffsplit_status_string(int(code)).decode()


def make_desc(d_model, d_ff, act="gelu", dtype="bf16", k=0, rem_kind="none", rank=0, group=0) -> Desc:
    acts = {"gelu": ACT_GELU, "swiglu": ACT_SWIGLU}
    dts = {"f32": F32, "bf16": BF16}
    rems = {"none": REM_NONE, "dense": REM_DENSE, "lowrank": REM_LOWRANK, "int4": REM_INT4, "w3h8": REM_W3H8}
    return Desc(d_model, d_ff, acts.get(act, act), dts.get(dtype, dtype), k, rems.get(rem_kind, rem_kind),
                rank, group)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(code, where):
    if code != 0:
        raise FFSplitError(code, where)


def workspace_bytes(desc: Desc, call_id: int, T: int = 0) -> int:
    return int(lib.ffsplit_workspace_bytes(ctypes.byref(desc), call_id, T))


def split_bytes(desc: Desc) -> int:
    return int(lib.ffsplit_split_bytes(ctypes.byref(desc)))


def _ws(nbytes, workspace, device):
    if workspace is not None:
        return workspace
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def score_neurons(desc, X, W1, Wg, W2, acc, T_total, scores=None, score_kind=SCORE_SUMSQ, workspace=None):
    """One calibration batch.  Returns the updated token count."""
    T = 0 if X is None else X.shape[0]
    ws = _ws(workspace_bytes(desc, WS_SCORE, T), workspace, acc.device)
    tt = ctypes.c_int64(int(T_total))
    rc = lib.ffsplit_score_neurons(ctypes.byref(desc), _ptr(X), T, _ptr(W1), _ptr(Wg), _ptr(W2), _ptr(acc),
                                   ctypes.byref(tt), _ptr(scores), score_kind, _ptr(ws), ws.numel(), _stream())
    _check(rc, "ffsplit_score_neurons")
    return tt.value


def select_heavy(scores, k, want_perm=False, workspace=None):
    """Returns (idx [k] int32, perm [d_ff] int32 or None, nan_flag [1] int32), all on the device."""
    d_ff = scores.numel()
    dev = scores.device
    idx = torch.empty(max(k, 1), dtype=torch.int32, device=dev)[:k]
    perm = torch.empty(d_ff, dtype=torch.int32, device=dev) if want_perm else None
    flag = torch.zeros(1, dtype=torch.int32, device=dev)
    ws = _ws(int(lib.ffsplit_workspace_bytes(ctypes.byref(make_desc(8, d_ff)), WS_SELECT, 0)), workspace, dev)
    rc = lib.ffsplit_select_heavy(_ptr(scores), d_ff, k, _ptr(idx) if k > 0 else None, _ptr(perm), _ptr(flag),
                                  _ptr(ws), ws.numel(), _stream())
    _check(rc, "ffsplit_select_heavy")
    return idx, perm, flag


SELECT_STATIC_MAX_DFF = 65536


def select_heavy_static(scores, k, idx, perm=None, flag=None):
    """ffsplit_select_heavy_static: every buffer is the caller's, nothing is allocated here."""
    rc = lib.ffsplit_select_heavy_static(_ptr(scores), scores.numel(), k, _ptr(idx) if k > 0 else None, _ptr(perm),
                                         _ptr(flag), _stream())
    _check(rc, "ffsplit_select_heavy_static")


def build_split(desc, W1, Wg, W2, idx, factors=None, split=None, workspace=None):
    """factors: dict with P1, Q1, Pg, Qg, P2, Q2 (device tensors or None).  Returns the packed split."""
    dev = W1.device
    nbytes = split_bytes(desc)
    if nbytes == 0:
        _check(-2, "ffsplit_split_bytes")
    if split is None:
        split = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    ws = _ws(workspace_bytes(desc, WS_BUILD, 0), workspace, dev)
    fac = None
    if factors is not None:
        arr = (ctypes.c_void_p * 6)()
        for i, nm in enumerate(("P1", "Q1", "Pg", "Qg", "P2", "Q2")):
            t = factors.get(nm)
            arr[i] = None if t is None else t.data_ptr()
        fac = arr
    rc = lib.ffsplit_build_split(ctypes.byref(desc), _ptr(W1), _ptr(Wg), _ptr(W2),
                                 _ptr(idx) if idx is not None and idx.numel() > 0 else None, fac, _ptr(split),
                                 _ptr(ws), ws.numel(), _stream())
    _check(rc, "ffsplit_build_split")
    return split


def factorize_remainder(desc, W1, Wg, W2, idx, seed=0, workspace=None):
    """Rank-r factors of the remainder on the device: dict P1, Q1, Pg, Qg, P2, Q2 (device tensors)."""
    dev = W1.device
    d, m, r = desc.d_model, desc.d_ff - desc.k, desc.rank
    glu = Wg is not None
    shapes = {"P1": (d, r), "Q1": (r, m), "Pg": (d, r), "Qg": (r, m), "P2": (m, r), "Q2": (r, d)}
    out = {nm: (torch.empty(sh, dtype=W1.dtype, device=dev) if (glu or nm not in ("Pg", "Qg")) else None)
           for nm, sh in shapes.items()}
    arr = (ctypes.c_void_p * 6)()
    for i, nm in enumerate(("P1", "Q1", "Pg", "Qg", "P2", "Q2")):
        arr[i] = None if out[nm] is None else out[nm].data_ptr()
    ws = _ws(workspace_bytes(desc, WS_FACTORIZE, 0), workspace, dev)
    rc = lib.ffsplit_factorize_remainder(ctypes.byref(desc), _ptr(W1), _ptr(Wg), _ptr(W2),
                                         _ptr(idx) if idx is not None and idx.numel() > 0 else None,
                                         ctypes.c_uint32(seed), arr, _ptr(ws), ws.numel(), _stream())
    _check(rc, "ffsplit_factorize_remainder")
    return out


def forward(desc, split, X, Y=None, want_parts=False, workspace=None):
    """Returns Y, or (Y, Y_heavy, Y_rem) with want_parts."""
    T = X.shape[0]
    if Y is None:
        Y = torch.empty((T, desc.d_model), dtype=X.dtype, device=X.device)
    Yh = torch.empty_like(Y) if want_parts else None
    Yr = torch.empty_like(Y) if want_parts else None
    ws = _ws(workspace_bytes(desc, WS_FORWARD, T), workspace, X.device)
    rc = lib.ffsplit_forward(ctypes.byref(desc), _ptr(split), _ptr(X), T, _ptr(Y), _ptr(Yh), _ptr(Yr), _ptr(ws),
                             ws.numel(), _stream())
    _check(rc, "ffsplit_forward")
    return (Y, Yh, Yr) if want_parts else Y


def forward_ex(desc, split, X, Y=None, b1_packed=None, b2=None, residual=None, y_f32=False, want_parts=False,
               workspace=None):
    """ffsplit_forward_ex: Y = [residual +] FFN_split(X) [+ b2], neuron biases in packed order.
    Returns Y, or (Y, Y_heavy, Y_rem) with want_parts."""
    T = X.shape[0]
    if Y is None:
        Y = torch.empty((T, desc.d_model), dtype=torch.float32 if y_f32 else X.dtype, device=X.device)
    Yh = torch.empty((T, desc.d_model), dtype=X.dtype, device=X.device) if want_parts else None
    Yr = torch.empty((T, desc.d_model), dtype=X.dtype, device=X.device) if want_parts else None
    ws = _ws(workspace_bytes(desc, WS_FORWARD, T), workspace, X.device)
    e = Epilogue(None if b1_packed is None else b1_packed.data_ptr(), None if b2 is None else b2.data_ptr(),
                 None if residual is None else residual.data_ptr(), 1 if y_f32 else 0)
    rc = lib.ffsplit_forward_ex(ctypes.byref(desc), _ptr(split), _ptr(X), T, _ptr(Y), _ptr(Yh), _ptr(Yr),
                                ctypes.byref(e), _ptr(ws), ws.numel(), _stream())
    _check(rc, "ffsplit_forward_ex")
    return (Y, Yh, Yr) if want_parts else Y


def pack_neuron_bias(desc, b1, idx, workspace=None):
    """b1 [d_ff] in the layer's dtype -> fp32 vector in the packed split's neuron order."""
    n = int(lib.ffsplit_neuron_bias_floats(ctypes.byref(desc)))
    out = torch.empty(max(n, 1), dtype=torch.float32, device=b1.device)
    ws = _ws(workspace_bytes(desc, WS_BUILD, 0), workspace, b1.device)
    rc = lib.ffsplit_pack_neuron_bias(ctypes.byref(desc), _ptr(b1), _ptr(idx) if idx is not None and idx.numel() > 0
                                      else None, _ptr(out), _ptr(ws), ws.numel(), _stream())
    _check(rc, "ffsplit_pack_neuron_bias")
    return out


def token_rmsnorm(x, dtype=BF16, eps=1e-6, out=None):
    """n(x) = x / sqrt(mean(x^2) + eps) per token; x fp32 [T, d]."""
    T, d = x.shape
    if out is None:
        out = torch.empty((T, d), dtype=torch.bfloat16 if dtype == BF16 else torch.float32, device=x.device)
    rc = lib.ffsplit_token_rmsnorm(_ptr(x), T, d, ctypes.c_float(eps), dtype, _ptr(out), _stream())
    _check(rc, "ffsplit_token_rmsnorm")
    return out


def stack_forward(desc, splits, x, b1_packed=None, b2=None, eps=1e-6, workspace=None):
    """x <- x + FFN_split_l(n(x)) [+ b2_l] for every layer, in place on the fp32 stream x [T, d]."""
    n, T = len(splits), x.shape[0]

    def arr(ts):
        if ts is None:
            return None
        a = (ctypes.c_void_p * n)()
        for i, t in enumerate(ts):
            a[i] = None if t is None else t.data_ptr()
        return a

    ws = _ws(workspace_bytes(desc, WS_STACK, T), workspace, x.device)
    rc = lib.ffsplit_stack_forward(ctypes.byref(desc), n, arr(splits), arr(b1_packed), arr(b2), _ptr(x), T,
                                   ctypes.c_float(eps), _ptr(ws), ws.numel(), _stream())
    _check(rc, "ffsplit_stack_forward")
    return x


def probe_mfma(workgroups, iters, scratch):
    """Enqueue the pure matrix-core loop; returns its flop count."""
    fl = ctypes.c_double(0.0)
    _check(lib.ffsplit_probe_mfma(workgroups, iters, _ptr(scratch), ctypes.byref(fl), _stream()), "ffsplit_probe_mfma")
    return fl.value


def probe_stream_read(buf, workgroups, scratch):
    """Enqueue one streaming read of buf (a uint8 tensor whose size is a multiple of 16)."""
    _check(lib.ffsplit_probe_stream_read(_ptr(buf), buf.numel() * buf.element_size(), workgroups, _ptr(scratch), _stream()),
           "ffsplit_probe_stream_read")


def split_export(desc, split, what):
    """Test hook of the quantised kinds: (q int8 [n, d_model], scale bits uint16 as int16 tensor
    [n, d_model/group]); what 0..2 = remainder W1 / Wg / W2 (n = m), 3..5 = heavy (W3H8 only, n = k)."""
    n = desc.k if what >= 3 else desc.d_ff - desc.k
    q = torch.empty((n, desc.d_model), dtype=torch.int8, device=split.device)
    s = torch.empty((n, desc.d_model // desc.group), dtype=torch.int16, device=split.device)
    rc = lib.ffsplit_split_export(ctypes.byref(desc), _ptr(split), what, _ptr(q), _ptr(s), _stream())
    _check(rc, "ffsplit_split_export")
    return q, s

"""ctypes binding of liblime_hip.so: argument marshalling only.

Every function here has the name and the meaning of the C entry point it calls
(see include/lime.h); tensors are torch CUDA tensors whose device pointers are
handed through, work goes onto torch's current stream.  There is no fallback:
if the library has not been built, or a call returns a non-zero status, an
exception is raised.
"""

from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblime_hip.so")

LIME_F32, LIME_BF16 = 0, 1
(OP_LINK_HISTORY, OP_XOR_HISTORY, OP_SCORE_CANDIDATES, OP_MHA_TARGET, OP_BUILD_QK_CACHE, OP_SCORE_CACHED,
 OP_XOR_LAYERS, OP_REQUEST_PREPARED, OP_REQUEST, OP_XOR_BACKWARD) = range(10)
STATUS_NAMES = {0: "LIME_OK", 1: "LIME_INVALID_ARG", 2: "LIME_UNSUPPORTED", 3: "LIME_WORKSPACE_TOO_SMALL",
                4: "LIME_LAUNCH_FAILED"}

_c = ctypes
_vp, _i32, _i64, _f32, _sz = _c.c_void_p, _c.c_int32, _c.c_int64, _c.c_float, _c.c_size_t

SIGNATURES = {
    "lime_link_history": (_i32, [_vp, _vp, _vp, _i64, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _f32, _i32,
                                 _vp, _sz, _vp]),
    "lime_xor_history": (_i32, [_vp, _vp, _vp, _i64, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _f32,
                                _i32, _vp, _sz, _vp]),
    "lime_xor_layers": (_i32, [_vp, _vp, _vp, _i64, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _i32, _i32, _i32, _i32, _i32,
                               _f32, _i32, _vp, _sz, _vp]),
    "lime_score_candidates": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _f32, _i32,
                                     _vp, _sz, _vp]),
    "mha_target_attention": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _f32, _i32,
                                    _vp, _sz, _vp]),
    "lime_build_qk_cache": (_i32, [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _f32, _i32, _vp, _sz, _vp]),
    "lime_score_candidates_cached": (_i32, [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _sz, _vp]),
    "lime_prepared_bytes": (_sz, [_i32, _i32, _i32, _i32]),
    "lime_prepare": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _f32, _f32, _vp, _sz, _i32, _i32, _i32, _i32, _vp]),
    "lime_link_history_prepared": (_i32, [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _f32, _i32, _i32, _vp, _sz,
                                          _vp]),
    "lime_score_candidates_prepared": (_i32, [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _f32, _i32, _vp,
                                              _sz, _vp]),
    "lime_request_prepared": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _i32, _f32, _f32,
                                     _i32, _i32, _vp, _sz, _vp]),
    "lime_request": (_i32, [_vp, _vp, _vp, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32,
                            _i32, _i32, _f32, _f32, _i32, _i32, _vp, _sz, _vp]),
    "lime_request_static": (_i32, [_vp, _vp, _vp, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32,
                                   _i32, _i32, _i32, _f32, _f32, _i32, _i32, _vp]),
    "lime_request_static_capacity": (_sz, []),
    "lime_request_many": (_i32, [_vp, _i32, _vp, _i32]),
    "lime_xor_backward": (_i32, [_vp] * 15 + [_i32] * 5 + [_f32, _i32, _vp, _sz, _vp]),
    "lime_score_candidates_gathered": (_i32, [_vp, _vp, _i32, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _sz,
                                              _vp]),
    "lime_workspace_bytes": (_sz, [_i32] * 9),
    "lime_probe_copy": (_i32, [_vp, _vp, _sz, _vp]),
    "lime_probe_mfma_out_bytes": (_sz, []),
    "lime_probe_mfma": (_c.c_double, [_vp, _i32, _vp]),
    "lime_profile_enable": (None, [_i32]),
    "lime_profile_collect": (_i32, [_i32, _c.POINTER(_c.c_float), _i32]),
    "lime_last_error": (_c.c_char_p, []),
    "lime_version": (_c.c_char_p, []),
}



class ScoringModel(_c.Structure):
    """lime_scoring_model of include/lime.h (a host struct of device pointers and sizes)."""
    _fields_ = [("d", _i32), ("h", _i32), ("m", _i32), ("dc", _i32), ("dhid", _i32), ("L", _vp),
                ("ctx_W1", _vp), ("ctx_b1", _vp), ("ctx_W2", _vp), ("ctx_b2", _vp),
                ("hist_Wq", _vp), ("hist_Wk", _vp), ("hist_Wv", _vp), ("cand_Wq", _vp), ("cand_Wk", _vp), ("cand_Wv", _vp),
                ("ln_hist_q", _vp * 2), ("ln_hist_kv", _vp * 2), ("ln_cand_q", _vp * 2), ("ln_cand_k", _vp * 2),
                ("ln_cand_v", _vp * 2), ("n_mlp", _i32), ("mlp_width", _i32 * 4), ("mlp_W", _vp * 4), ("mlp_b", _vp * 4),
                ("scale_hist", _f32), ("scale_cand", _f32), ("ln_eps", _f32)]


SIGNATURES.update({
    "lime_layer_norm": (_i32, [_vp, _vp, _vp, _f32, _vp, _i64, _i32, _i32, _vp]),
    "lime_contextualize_links": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _sz, _vp]),
    "lime_interaction_mlp_workspace_bytes": (_sz, [_i64, _i32, _c.POINTER(_i32), _i32, _i32]),
    "lime_interaction_mlp": (_i32, [_vp, _c.POINTER(_vp), _c.POINTER(_vp), _c.POINTER(_i32), _i32, _vp, _i64, _i32, _i32, _vp, _sz,
                                    _vp]),
    "lime_scores_workspace_bytes": (_sz, [_c.POINTER(ScoringModel), _i32, _i32, _i32, _i32]),
    "lime_scores": (_i32, [_c.POINTER(ScoringModel), _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _vp, _sz, _vp]),
})

_lib = None


class LimeError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {text}")
        self.status = status


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built (python -c 'import __graft_entry__ as g; g.build()')."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first (python paper_2510_18239_amd/build.py); "
                               "there is no CPU fallback")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def last_error() -> str:
    return lib().lime_last_error().decode()


def version() -> str:
    return lib().lime_version().decode()


def profile_enable(on: bool) -> None:
    lib().lime_profile_enable(1 if on else 0)


def profile_collect(kernel: int, capacity: int = 65536) -> list[float]:
    """Durations (ms) of the recorded launches of one kernel id since the last collect."""
    buf = (_c.c_float * capacity)()
    n = lib().lime_profile_collect(kernel, buf, capacity)
    return [float(buf[i]) for i in range(n)]


KERNEL_PROBE_COPY, KERNEL_PROBE_MFMA = 5, 6


def probe_copy(src: torch.Tensor, dst: torch.Tensor, stream=None) -> None:
    """A plain device copy of src into dst (same byte size, a multiple of 16) by the library's streaming-copy probe."""
    nbytes = src.numel() * src.element_size()
    assert nbytes == dst.numel() * dst.element_size() and src.is_contiguous() and dst.is_contiguous()
    with torch.cuda.device(src.device):
        _raise(lib().lime_probe_copy(_ptr(src), _ptr(dst), nbytes, _stream(stream)))


def probe_mfma(iters: int, stream=None) -> float:
    """Runs the register-resident matrix-instruction loop; returns the floating-point operations it executes."""
    out = get_workspace(lib().lime_probe_mfma_out_bytes(), torch.device("cuda", torch.cuda.current_device()), stream)
    with torch.cuda.device(out.device):
        flops = lib().lime_probe_mfma(_ptr(out), int(iters), _stream(stream))
    if flops <= 0:
        raise LimeError(4, "lime_probe_mfma failed")
    return float(flops)


def workspace_bytes(op: int, B=1, N=1, C=1, d=1, h=1, m=1, dtype=LIME_BF16, flags=0) -> int:
    return int(lib().lime_workspace_bytes(op, B, N, C, d, h, m, dtype, flags))


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return LIME_F32
    if t.dtype == torch.bfloat16:
        return LIME_BF16
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _ptr(t):
    return None if t is None else t.data_ptr()


def _check(*tensors):
    first = next(t for t in tensors if t is not None)
    for t in tensors:
        if t is None:
            continue
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("tensors must be contiguous CUDA tensors")
        if t.dtype != first.dtype or t.device != first.device:
            raise ValueError("tensors must share dtype and device")
    return first


_workspaces: dict = {}
_outgrown: list = []


def _stream(stream):
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def get_workspace(nbytes: int, device, stream=None) -> torch.Tensor:
    """A grow-only scratch buffer per (device, stream): caller-owned memory as far as the C ABI is concerned.
    Calls on different streams may run at the same time, so they must not share scratch memory; calls on one
    stream are ordered and may.  A buffer that is outgrown is replaced by one at least twice its size and kept
    until the process ends (work already queued on the stream may still use it)."""
    if not isinstance(device, torch.device):
        device = torch.device(device)
    # (this runs on every call of every wrapper: no device context, one stream query)
    key = (device.index, stream.cuda_stream if stream is not None else torch.cuda.current_stream(device).cuda_stream)
    ws = _workspaces.get(key)
    if ws is None or ws.numel() < nbytes:
        if ws is not None:
            _outgrown.append(ws)
            nbytes = max(nbytes, 2 * ws.numel())
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
        _workspaces[key] = ws
    return ws


def _raise(status):
    if status != 0:
        raise LimeError(status, last_error())


def _lens_arg(lens, B, device):
    if lens is None:
        return None
    if lens.dtype != torch.int32 or not lens.is_cuda or lens.numel() != B or not lens.is_contiguous():
        raise ValueError("lens must be a contiguous CUDA int32 tensor of B entries")
    return lens


def _history(fn_name, op, E, lens, LC, Wq, Wk, Wv, h, scale, LP, OS, workspace, stream, want_os):
    first = _check(E, LC, Wq, Wk, Wv, LP, OS)
    B, N, d = E.shape
    if LC.dim() == 2:
        m, stride = LC.shape[0], 0
    else:
        if LC.shape[0] != B:
            raise ValueError("per-user links must be [B, m, d]")
        m, stride = LC.shape[1], LC.shape[1] * LC.shape[2]
    lens = _lens_arg(lens, B, E.device)
    code = _dtype_code(first)
    if LP is None:
        LP = torch.empty((B, m, d), dtype=E.dtype, device=E.device)
    if want_os and OS is None:
        OS = torch.empty((B, N, d), dtype=E.dtype, device=E.device)
    need = workspace_bytes(op, B=B, N=N, d=d, h=h, m=m, dtype=code, flags=1 if want_os else 0)
    ws = workspace if workspace is not None else get_workspace(need, E.device, stream)
    fn = getattr(lib(), fn_name)
    with torch.cuda.device(E.device):
        if op == OP_LINK_HISTORY:
            st = fn(_ptr(E), _ptr(lens), _ptr(LC), stride, _ptr(Wq), _ptr(Wk), _ptr(Wv), _ptr(LP), B, N, d, h, m,
                    float(scale), code, _ptr(ws), ws.numel(), _stream(stream))
        else:
            st = fn(_ptr(E), _ptr(lens), _ptr(LC), stride, _ptr(Wq), _ptr(Wk), _ptr(Wv), _ptr(LP), _ptr(OS), B, N, d,
                    h, m, float(scale), code, _ptr(ws), ws.numel(), _stream(stream))
    _raise(st)
    return LP, OS


def lime_link_history(E, lens, LC, Wq, Wk, Wv, h, scale, LP=None, workspace=None, stream=None):
    """LP[B, m, d] = MHA(LC, E, E) per user, softmax over the valid history rows (Eq. 3)."""
    return _history("lime_link_history", OP_LINK_HISTORY, E, lens, LC, Wq, Wk, Wv, h, scale, LP, None, workspace,
                    stream, False)[0]


def lime_xor_history(E, lens, LC, Wq, Wk, Wv, h, scale=1.0, want_os=False, LP=None, OS=None, workspace=None,
                     stream=None):
    """One XORA layer (Eq. 6-7): returns (O[T] = link states [B, m, d], O[S] [B, N, d] or None)."""
    return _history("lime_xor_history", OP_XOR_HISTORY, E, lens, LC, Wq, Wk, Wv, h, scale, LP, OS, workspace, stream,
                    want_os or OS is not None)


def lime_xor_layers(E, lens, LC, Wq, Wk, Wv, Wu, Wo, h, scale=1.0, LP=None, workspace=None, stream=None):
    """LP[B, m, d] of LIME-XOR with Wu.shape[0] stacked XOR layers (Eq. 8); Wu, Wo [n, d, d] are the gated blocks' weights."""
    first = _check(E, LC, Wq, Wk, Wv, Wu, Wo, LP)
    B, N, d = E.shape
    if LC.dim() == 2:
        m, stride = LC.shape[0], 0
    else:
        if LC.shape[0] != B:
            raise ValueError("per-user links must be [B, m, d]")
        m, stride = LC.shape[1], LC.shape[1] * LC.shape[2]
    if Wu.dim() != 3 or Wu.shape != Wo.shape or tuple(Wu.shape[1:]) != (d, d):
        raise ValueError("Wu and Wo must both be [n_layers, d, d]")
    lens = _lens_arg(lens, B, E.device)
    code = _dtype_code(first)
    if LP is None:
        LP = torch.empty((B, m, d), dtype=E.dtype, device=E.device)
    need = workspace_bytes(OP_XOR_LAYERS, B=B, N=N, d=d, h=h, m=m, dtype=code)
    ws = workspace if workspace is not None else get_workspace(need, E.device, stream)
    with torch.cuda.device(E.device):
        st = lib().lime_xor_layers(_ptr(E), _ptr(lens), _ptr(LC), stride, _ptr(Wq), _ptr(Wk), _ptr(Wv), _ptr(Wu), _ptr(Wo),
                                   int(Wu.shape[0]), _ptr(LP), B, N, d, h, m, float(scale), code, _ptr(ws), ws.numel(),
                                   _stream(stream))
    _raise(st)
    return LP


def lime_score_candidates(T, L, LP, Wq, Wk, Wv, h, scale, O=None, workspace=None, stream=None):
    """O[B, C, d] = MHA(T, L, LP) per user, softmax over the m links (Eq. 4); W* may be None (identity)."""
    first = _check(T, L, LP, Wq, Wk, Wv, O)
    B, C, d = T.shape
    m = L.shape[0]
    code = _dtype_code(first)
    if O is None:
        O = torch.empty_like(T)
    need = workspace_bytes(OP_SCORE_CANDIDATES, B=B, C=C, d=d, h=h, m=m, dtype=code)
    ws = workspace if workspace is not None else get_workspace(need, T.device, stream)
    with torch.cuda.device(T.device):
        st = lib().lime_score_candidates(_ptr(T), _ptr(L), _ptr(LP), _ptr(Wq), _ptr(Wk), _ptr(Wv), _ptr(O), B, C, d,
                                         h, m, float(scale), code, _ptr(ws), ws.numel(), _stream(stream))
    _raise(st)
    return O


def mha_target_attention(T, E, lens, Wq, Wk, Wv, h, scale, O=None, workspace=None, stream=None):
    """O[B, C, d] = MHA(T, E, E) per user over the valid history rows (Eq. 1; the baseline)."""
    first = _check(T, E, Wq, Wk, Wv, O)
    B, C, d = T.shape
    N = E.shape[1]
    lens = _lens_arg(lens, B, E.device)
    code = _dtype_code(first)
    if O is None:
        O = torch.empty_like(T)
    need = workspace_bytes(OP_MHA_TARGET, B=B, N=N, C=C, d=d, h=h, dtype=code)
    ws = workspace if workspace is not None else get_workspace(need, T.device, stream)
    with torch.cuda.device(T.device):
        st = lib().mha_target_attention(_ptr(T), _ptr(E), _ptr(lens), _ptr(Wq), _ptr(Wk), _ptr(Wv), _ptr(O), B, C, N,
                                        d, h, float(scale), code, _ptr(ws), ws.numel(), _stream(stream))
    _raise(st)
    return O


def lime_build_qk_cache(T, L, Wq, Wk, h, scale, W=None, workspace=None, stream=None):
    """W[B, C, h, m] = softmax over the links of the scaled candidate-link logits (Section 3.3, offline side)."""
    first = _check(T, L, Wq, Wk, W)
    B, C, d = T.shape
    m = L.shape[0]
    code = _dtype_code(first)
    if W is None:
        W = torch.empty((B, C, h, m), dtype=T.dtype, device=T.device)
    need = workspace_bytes(OP_BUILD_QK_CACHE, B=B, C=C, d=d, h=h, m=m, dtype=code)
    ws = workspace if workspace is not None else get_workspace(need, T.device, stream)
    with torch.cuda.device(T.device):
        st = lib().lime_build_qk_cache(_ptr(T), _ptr(L), _ptr(Wq), _ptr(Wk), _ptr(W), B, C, d, h, m, float(scale), code,
                                       _ptr(ws), ws.numel(), _stream(stream))
    _raise(st)
    return W


def lime_score_candidates_cached(W, LP, Wv, O=None, workspace=None, stream=None):
    """O[B, C, d] = cached weights W[B, C, h, m] times the projected link states (Section 3.3, online side)."""
    first = _check(W, LP, Wv, O)
    B, C, h, m = W.shape
    d = LP.shape[2]
    code = _dtype_code(first)
    if O is None:
        O = torch.empty((B, C, d), dtype=W.dtype, device=W.device)
    need = workspace_bytes(OP_SCORE_CACHED, B=B, C=C, d=d, h=h, m=m, dtype=code)
    ws = workspace if workspace is not None else get_workspace(need, W.device, stream)
    with torch.cuda.device(W.device):
        st = lib().lime_score_candidates_cached(_ptr(W), _ptr(LP), _ptr(Wv), _ptr(O), B, C, d, h, m, code, _ptr(ws),
                                                ws.numel(), _stream(stream))
    _raise(st)
    return O


def lime_score_candidates_gathered(Wtable, ids, LP, Wv, O=None, workspace=None, stream=None):
    """O[B, C, d] from a corpus-wide table of cached weights Wtable[n_items, h, m] and candidate ids [B, C] (int32):
    row ids[b, c] of the table times the projected link states of user b; ids outside the table give zero rows."""
    first = _check(Wtable, LP, Wv, O)
    assert ids.dtype == torch.int32 and ids.is_contiguous() and ids.device == Wtable.device, "ids: contiguous int32 on the device"
    n_items, h, m = Wtable.shape
    B, C = ids.shape
    d = LP.shape[2]
    code = _dtype_code(first)
    if O is None:
        O = torch.empty((B, C, d), dtype=Wtable.dtype, device=Wtable.device)
    need = workspace_bytes(OP_SCORE_CACHED, B=B, C=C, d=d, h=h, m=m, dtype=code)
    ws = workspace if workspace is not None else get_workspace(need, Wtable.device, stream)
    with torch.cuda.device(Wtable.device):
        st = lib().lime_score_candidates_gathered(_ptr(Wtable), _ptr(ids), n_items, _ptr(LP), _ptr(Wv), _ptr(O), B, C, d,
                                                  h, m, code, _ptr(ws), ws.numel(), _stream(stream))
    _raise(st)
    return O


def lime_prepare(LC, L, Wq_hist, Wk_hist, Wv_hist, Wq_cand, Wk_cand, h, scale_hist, scale_cand, stream=None):
    """Packs what depends on the model only (weights, shared links [m, d]) once; returns the prepared buffer."""
    first = _check(LC, L, Wq_hist, Wk_hist, Wv_hist, Wq_cand, Wk_cand)
    m, d = LC.shape
    code = _dtype_code(first)
    need = lib().lime_prepared_bytes(d, h, m, code)
    if need == 0:
        raise LimeError(2, "lime_prepare: shape or dtype without prepared operands")
    prepared = torch.empty(need, dtype=torch.uint8, device=LC.device)
    with torch.cuda.device(LC.device):
        st = lib().lime_prepare(_ptr(LC), _ptr(L), _ptr(Wq_hist), _ptr(Wk_hist), _ptr(Wv_hist), _ptr(Wq_cand),
                                _ptr(Wk_cand), float(scale_hist), float(scale_cand), _ptr(prepared), need, d, h, m, code,
                                _stream(stream))
    _raise(st)
    return prepared


def lime_link_history_prepared(E, lens, prepared, h, m, scale, xor_attention=False, LP=None, workspace=None, stream=None):
    """lime_link_history (or the link states of lime_xor_history) on operands prepared by lime_prepare."""
    first = _check(E, LP)
    B, N, d = E.shape
    code = _dtype_code(first)
    if LP is None:
        LP = torch.empty((B, m, d), dtype=E.dtype, device=E.device)
    need = workspace_bytes(OP_LINK_HISTORY, B=B, N=N, d=d, h=h, m=m, dtype=code)
    ws = workspace if workspace is not None else get_workspace(need, E.device, stream)
    with torch.cuda.device(E.device):
        st = lib().lime_link_history_prepared(_ptr(E), _ptr(lens), _ptr(prepared), _ptr(LP), B, N, d, h, m, float(scale),
                                              int(bool(xor_attention)), code, _ptr(ws), ws.numel(), _stream(stream))
    _raise(st)
    return LP


def lime_score_candidates_prepared(T, LP, Wv, prepared, h, scale, O=None, workspace=None, stream=None):
    """lime_score_candidates on operands prepared by lime_prepare (the user's link states LP are projected per call)."""
    first = _check(T, LP, Wv, O)
    B, C, d = T.shape
    m = LP.shape[1]
    code = _dtype_code(first)
    if O is None:
        O = torch.empty_like(T)
    need = workspace_bytes(OP_SCORE_CANDIDATES, B=B, C=C, d=d, h=h, m=m, dtype=code)
    ws = workspace if workspace is not None else get_workspace(need, T.device, stream)
    with torch.cuda.device(T.device):
        st = lib().lime_score_candidates_prepared(_ptr(T), _ptr(LP), _ptr(Wv), _ptr(prepared), _ptr(O), B, C, d, h, m,
                                                  float(scale), code, _ptr(ws), ws.numel(), _stream(stream))
    _raise(st)
    return O


def lime_xor_backward(QS, KS, VS, QT, KT, VT, dOT, dOS, lens, h, scale=1.0, workspace=None, stream=None):
    """Gradients of one XORA layer w.r.t. its projected inputs (Appendix H.2): returns (dQS, dKS, dVS, dQT, dKT, dVT)."""
    first = _check(QS, KS, VS, QT, KT, VT, dOT, dOS)
    B, N, d = QS.shape
    m = QT.shape[1]
    if QT.dim() != 3 or QT.shape[0] != B:
        raise ValueError("the projected links must be per user: [B, m, d]")
    code = _dtype_code(first)
    lens = _lens_arg(lens, B, QS.device)
    outs = [torch.empty_like(QS) for _ in range(3)] + [torch.empty_like(QT) for _ in range(3)]
    need = workspace_bytes(OP_XOR_BACKWARD, B=B, N=N, d=d, h=h, m=m, dtype=code)
    ws = workspace if workspace is not None else get_workspace(need, QS.device, stream)
    with torch.cuda.device(QS.device):
        st = lib().lime_xor_backward(_ptr(QS), _ptr(KS), _ptr(VS), _ptr(QT), _ptr(KT), _ptr(VT), _ptr(dOT), _ptr(dOS),
                                     _ptr(lens), *[_ptr(o) for o in outs], B, N, m, d, h, float(scale), code, _ptr(ws),
                                     ws.numel(), _stream(stream))
    _raise(st)
    return tuple(outs)


def lime_request(E, lens, LC, Wq_hist, Wk_hist, Wv_hist, T, L, Wq_cand, Wk_cand, Wv_cand, h, scale_hist, scale_cand,
                 xor_attention=False, LP=None, O=None, workspace=None, stream=None):
    """lime_link_history (or the link states of lime_xor_history) followed by lime_score_candidates, as one call; returns (LP, O)."""
    first = _check(E, LC, Wq_hist, Wk_hist, Wv_hist, T, L, Wq_cand, Wk_cand, Wv_cand, LP, O)
    B, N, d = E.shape
    C = T.shape[1]
    if LC.dim() == 2:
        m, stride = LC.shape[0], 0
    else:
        if LC.shape[0] != B:
            raise ValueError("per-user links must be [B, m, d]")
        m, stride = LC.shape[1], LC.shape[1] * LC.shape[2]
    code = _dtype_code(first)
    lens = _lens_arg(lens, B, E.device)
    if LP is None:
        LP = torch.empty((B, m, d), dtype=E.dtype, device=E.device)
    if O is None:
        O = torch.empty_like(T)
    need = workspace_bytes(OP_REQUEST, B=B, N=N, C=C, d=d, h=h, m=m, dtype=code)
    ws = workspace if workspace is not None else get_workspace(need, E.device, stream)
    with torch.cuda.device(E.device):
        st = lib().lime_request(_ptr(E), _ptr(lens), _ptr(LC), stride, _ptr(Wq_hist), _ptr(Wk_hist), _ptr(Wv_hist), _ptr(T),
                                _ptr(L), _ptr(Wq_cand), _ptr(Wk_cand), _ptr(Wv_cand), _ptr(LP), _ptr(O), B, N, C, d, h, m,
                                float(scale_hist), float(scale_cand), int(bool(xor_attention)), code, _ptr(ws), ws.numel(),
                                _stream(stream))
    _raise(st)
    return LP, O


class RequestArgs(ctypes.Structure):
    """lime_request_args of include/lime.h: the arguments of lime_request, one request of a batch."""
    _fields_ = [("E", _vp), ("lens", _vp), ("LC", _vp), ("lc_user_stride", _i64), ("Wq_hist", _vp), ("Wk_hist", _vp),
                ("Wv_hist", _vp), ("T", _vp), ("L", _vp), ("Wq_cand", _vp), ("Wk_cand", _vp), ("Wv_cand", _vp), ("LP", _vp),
                ("O", _vp), ("B", _i32), ("N", _i32), ("C", _i32), ("d", _i32), ("h", _i32), ("m", _i32),
                ("scale_hist", _f32), ("scale_cand", _f32), ("xor_attention", _i32), ("dtype", _i32), ("workspace", _vp),
                ("ws_bytes", _sz)]


def request_args(E, lens, LC, Wq_hist, Wk_hist, Wv_hist, T, L, Wq_cand, Wk_cand, Wv_cand, h, scale_hist, scale_cand, LP, O,
                 workspace, xor_attention=False) -> RequestArgs:
    """One entry of the array lime_request_many takes (shapes as lime_request; LP, O and workspace are required: requests
    in flight at the same time must not share them).  The tensors must stay alive until the GPU has passed the request."""
    first = _check(E, LC, Wq_hist, Wk_hist, Wv_hist, T, L, Wq_cand, Wk_cand, Wv_cand, LP, O)
    B, N, d = E.shape
    C = T.shape[1]
    m, stride = (LC.shape[0], 0) if LC.dim() == 2 else (LC.shape[1], LC.shape[1] * LC.shape[2])
    lens = _lens_arg(lens, B, E.device)
    r = RequestArgs(_ptr(E), _ptr(lens), _ptr(LC), stride, _ptr(Wq_hist), _ptr(Wk_hist), _ptr(Wv_hist), _ptr(T), _ptr(L),
                    _ptr(Wq_cand), _ptr(Wk_cand), _ptr(Wv_cand), _ptr(LP), _ptr(O), B, N, C, d, h, m, float(scale_hist),
                    float(scale_cand), 1 if xor_attention else 0, _dtype_code(first), _ptr(workspace), workspace.numel())
    r._keep = (lens,)
    return r


def lime_request_many(requests, streams) -> None:
    """Submits the requests (a list of RequestArgs) over the streams (torch streams or raw handles), request i on
    streams[i % len(streams)], from one host thread per stream; returns when everything is enqueued."""
    arr = (RequestArgs * len(requests))(*requests)
    handles = (_vp * len(streams))(*[s.cuda_stream if hasattr(s, "cuda_stream") else s for s in streams])
    _raise(lib().lime_request_many(ctypes.cast(arr, _vp), len(requests), ctypes.cast(handles, _vp), len(streams)))


def lime_request_static(E, lens, LC, Wq_hist, Wk_hist, Wv_hist, T, L, Wq_cand, Wk_cand, Wv_cand, h, scale_hist, scale_cand,
                        xor_attention=False, LP=None, O=None, stream=None):
    """lime_request on the library's own fixed scratch array instead of a workspace; returns (LP, O).  Calls on one
    GPU must not overlap."""
    first = _check(E, LC, Wq_hist, Wk_hist, Wv_hist, T, L, Wq_cand, Wk_cand, Wv_cand, LP, O)
    B, N, d = E.shape
    C = T.shape[1]
    if LC.dim() == 2:
        m, stride = LC.shape[0], 0
    else:
        if LC.shape[0] != B:
            raise ValueError("per-user links must be [B, m, d]")
        m, stride = LC.shape[1], LC.shape[1] * LC.shape[2]
    code = _dtype_code(first)
    lens = _lens_arg(lens, B, E.device)
    if LP is None:
        LP = torch.empty((B, m, d), dtype=E.dtype, device=E.device)
    if O is None:
        O = torch.empty_like(T)
    with torch.cuda.device(E.device):
        st = lib().lime_request_static(_ptr(E), _ptr(lens), _ptr(LC), stride, _ptr(Wq_hist), _ptr(Wk_hist), _ptr(Wv_hist),
                                       _ptr(T), _ptr(L), _ptr(Wq_cand), _ptr(Wk_cand), _ptr(Wv_cand), _ptr(LP), _ptr(O), B, N,
                                       C, d, h, m, float(scale_hist), float(scale_cand), int(bool(xor_attention)), code,
                                       _stream(stream))
    _raise(st)
    return LP, O


def lime_request_prepared(E, lens, T, Wv, prepared, h, m, scale_hist, scale_cand, xor_attention=False, LP=None, O=None,
                          workspace=None, stream=None):
    """lime_link_history_prepared + lime_score_candidates_prepared as one call of three kernels; returns (LP, O)."""
    first = _check(E, T, Wv, LP, O)
    B, N, d = E.shape
    C = T.shape[1]
    code = _dtype_code(first)
    lens = _lens_arg(lens, B, E.device)
    if LP is None:
        LP = torch.empty((B, m, d), dtype=E.dtype, device=E.device)
    if O is None:
        O = torch.empty_like(T)
    need = workspace_bytes(OP_REQUEST_PREPARED, B=B, N=N, C=C, d=d, h=h, m=m, dtype=code)
    ws = workspace if workspace is not None else get_workspace(need, E.device, stream)
    with torch.cuda.device(E.device):
        st = lib().lime_request_prepared(_ptr(E), _ptr(lens), _ptr(T), _ptr(Wv), _ptr(prepared), _ptr(LP), _ptr(O), B, N, C,
                                         d, h, m, float(scale_hist), float(scale_cand), int(bool(xor_attention)), code,
                                         _ptr(ws), ws.numel(), _stream(stream))
    _raise(st)
    return LP, O


def lime_layer_norm(X, gamma, beta, eps=1e-5, Y=None, stream=None):
    """Y = LayerNorm(X; gamma, beta, eps) over the last axis (Appendix C); gamma, beta [d] or None."""
    first = _check(X, gamma, beta, Y)
    d = X.shape[-1]
    if Y is None:
        Y = torch.empty_like(X)
    with torch.cuda.device(X.device):
        st = lib().lime_layer_norm(_ptr(X), _ptr(gamma), _ptr(beta), float(eps), _ptr(Y), X.numel() // d, d, _dtype_code(first),
                                   _stream(stream))
    _raise(st)
    return Y


def lime_contextualize_links(L, EC, W1, b1, W2, b2, LC=None, workspace=None, stream=None):
    """LC[B, m, d] = ReLU([L | EC_b] W1 + b1) W2 + b2 per user (Eq. 2)."""
    first = _check(L, EC, W1, b1, W2, b2, LC)
    m, d = L.shape
    B, dc = EC.shape
    dhid = W1.shape[1]
    if W1.shape[0] != d + dc or tuple(W2.shape) != (dhid, d):
        raise ValueError("W1 must be [d + dc, dhid] and W2 [dhid, d]")
    if LC is None:
        LC = torch.empty((B, m, d), dtype=L.dtype, device=L.device)
    need = (B * m * dhid * 4 + 255) // 256 * 256
    ws = workspace if workspace is not None else get_workspace(need, L.device, stream)
    with torch.cuda.device(L.device):
        st = lib().lime_contextualize_links(_ptr(L), _ptr(EC), _ptr(W1), _ptr(b1), _ptr(W2), _ptr(b2), _ptr(LC), B, m, d, dc, dhid,
                                            _dtype_code(first), _ptr(ws), ws.numel(), _stream(stream))
    _raise(st)
    return LC


def _mlp_arrays(weights, biases):
    n = len(weights)
    W = (_vp * n)(*[_ptr(w) for w in weights])
    b = (_vp * n)(*[_ptr(x) for x in biases])
    widths = (_i32 * n)(*[int(w.shape[1]) for w in weights])
    return n, W, b, widths


def lime_interaction_mlp(O, weights, biases, scores=None, workspace=None, stream=None):
    """scores[...] (fp32) of the interaction network (Section 3.3) on the rows of O[..., d]: weights[i] [d_in, d_out] with
    ReLU after all but the last map, whose d_out is 1; biases[i] [d_out] or None."""
    first = _check(O, *weights, *biases)
    d = O.shape[-1]
    rows = O.numel() // d
    n, W, b, widths = _mlp_arrays(weights, biases)
    code = _dtype_code(first)
    if scores is None:
        scores = torch.empty(O.shape[:-1], dtype=torch.float32, device=O.device)
    need = int(lib().lime_interaction_mlp_workspace_bytes(rows, d, widths, n, code))
    ws = workspace if workspace is not None else get_workspace(need, O.device, stream)
    with torch.cuda.device(O.device):
        st = lib().lime_interaction_mlp(_ptr(O), W, b, widths, n, _ptr(scores), rows, d, code, _ptr(ws), ws.numel(), _stream(stream))
    _raise(st)
    return scores


def scoring_model(L, ctx, hist, cand, ln_hist_q, ln_hist_kv, ln_cand_q, ln_cand_k, ln_cand_v, mlp, h, scale_hist, scale_cand,
                  ln_eps=1e-5) -> ScoringModel:
    """The host struct lime_scores takes: ctx = (W1, b1, W2, b2); hist, cand = (Wq, Wk, Wv); ln_* = (gamma, beta) or
    (None, None); mlp = (weights, biases).  The tensors must stay alive while the struct is used."""
    M = ScoringModel()
    M.m, M.d = L.shape
    M.h, M.dc, M.dhid = h, ctx[0].shape[0] - L.shape[1], ctx[0].shape[1]
    M.L = _ptr(L)
    M.ctx_W1, M.ctx_b1, M.ctx_W2, M.ctx_b2 = (_ptr(x) for x in ctx)
    M.hist_Wq, M.hist_Wk, M.hist_Wv = (_ptr(x) for x in hist)
    M.cand_Wq, M.cand_Wk, M.cand_Wv = (_ptr(x) for x in cand)
    for name, gb in (("ln_hist_q", ln_hist_q), ("ln_hist_kv", ln_hist_kv), ("ln_cand_q", ln_cand_q), ("ln_cand_k", ln_cand_k),
                     ("ln_cand_v", ln_cand_v)):
        setattr(M, name, (_vp * 2)(_ptr(gb[0]), _ptr(gb[1])))
    weights, biases = mlp
    M.n_mlp = len(weights)
    for i, (w, bias) in enumerate(zip(weights, biases)):
        M.mlp_width[i], M.mlp_W[i], M.mlp_b[i] = int(w.shape[1]), _ptr(w), _ptr(bias)
    M.scale_hist, M.scale_cand, M.ln_eps = float(scale_hist), float(scale_cand), float(ln_eps)
    return M


def lime_scores(model: ScoringModel, E, lens, EC, T, want_intermediates=False, workspace=None, stream=None):
    """One LIME-MHA request from embeddings to scores (Eq. 2 -> LN -> Eq. 3 -> LN -> Eq. 4 -> interaction network).
    Returns scores [B, C] (fp32), and with want_intermediates also (LC, LP, O)."""
    first = _check(E, EC, T)
    B, N, d = E.shape
    C = T.shape[1]
    code = _dtype_code(first)
    lens = _lens_arg(lens, B, E.device)
    scores = torch.empty((B, C), dtype=torch.float32, device=E.device)
    LC = LP = O = None
    if want_intermediates:
        LC = torch.empty((B, model.m, d), dtype=E.dtype, device=E.device)
        LP = torch.empty_like(LC)
        O = torch.empty_like(T)
    need = int(lib().lime_scores_workspace_bytes(_c.byref(model), B, N, C, code))
    if need == 0:
        raise LimeError(1, "lime_scores: the model or the sizes are not valid")
    ws = workspace if workspace is not None else get_workspace(need, E.device, stream)
    with torch.cuda.device(E.device):
        st = lib().lime_scores(_c.byref(model), _ptr(E), _ptr(lens), _ptr(EC), _ptr(T), _ptr(LC), _ptr(LP), _ptr(O), _ptr(scores), B, N,
                               C, code, _ptr(ws), ws.numel(), _stream(stream))
    _raise(st)
    return (scores, LC, LP, O) if want_intermediates else scores

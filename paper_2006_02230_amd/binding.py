"""ctypes binding of libpolydl.so: same names as the C entry points, argument marshalling only."""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpolydl.so")

if not os.path.exists(LIB_PATH):
    raise ImportError("libpolydl.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                      "(or python paper_2006_02230_amd/build.py) first; there is no fallback path")

# PyTorch ships its own copy of the HIP runtime (same soname as the system one) and owns the
# device memory and streams handed to this library, so it must be the copy this library binds to:
# load torch first, then the dynamic linker resolves libamdhip64 to the one already in the process.
import torch  # noqa: E402,F401

lib = ctypes.CDLL(LIB_PATH)

ACT = {None: 0, "none": 0, "relu": 1, "relu6": 2, 0: 0, 1: 1, 2: 2, False: 0, True: 1}


class PolydlError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        extra = ""
        if status == -4:
            lib.polydl_last_hip_error.restype = ctypes.c_int
            extra = ", hipError_t %d" % lib.polydl_last_hip_error()
        super().__init__("%s: %s (%d%s)" % (where, status_string(status), status, extra))


class TileCfg(ctypes.Structure):
    """Mirror of polydl_tile_cfg."""
    _fields_ = [(n, ctypes.c_int) for n in ("bm", "bn", "bk", "wm", "wn", "split_k", "layout", "raster",
                                            "algo", "cb")]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}

    def __repr__(self):
        return "TileCfg(%s)" % ", ".join("%s=%d" % kv for kv in self.as_dict().items())


class ModelReport(ctypes.Structure):
    """Mirror of polydl_model_report."""
    _fields_ = [("predicted_us", ctypes.c_double), ("mfma_us", ctypes.c_double), ("mem_us", ctypes.c_double),
                ("fixed_us", ctypes.c_double), ("ws", ctypes.c_double * 8), ("n_ws", ctypes.c_int),
                ("level_bytes", ctypes.c_double * 4), ("mem_bytes", ctypes.c_double),
                ("eq1_cost", ctypes.c_double), ("workgroups", ctypes.c_int), ("simd_load", ctypes.c_double),
                ("ws_level", ctypes.c_int * 8), ("ws_traffic", ctypes.c_double * 8)]

    def as_dict(self):
        return {"predicted_us": self.predicted_us, "mfma_us": self.mfma_us, "mem_us": self.mem_us,
                "fixed_us": self.fixed_us, "ws": list(self.ws)[:self.n_ws], "level_bytes": list(self.level_bytes),
                "mem_bytes": self.mem_bytes, "eq1_cost": self.eq1_cost, "workgroups": self.workgroups,
                "simd_load": self.simd_load, "ws_level": list(self.ws_level)[:self.n_ws],
                "ws_traffic": list(self.ws_traffic)[:self.n_ws]}


_i, _p = ctypes.c_int, ctypes.c_void_p
lib.polydl_conv2d_fwd.argtypes = [_i] * 9 + [_p, _p, _p, _p, _i, _p]
lib.polydl_conv2d_fwd_act.argtypes = [_i] * 9 + [_p, _p, _p, _p, _i, _p]
lib.polydl_conv2d_fwd_pre_act.argtypes = [_i] * 9 + [_p, _p, _p, _p, _i, _i, _p]
lib.polydl_conv2d_fwd_pre_act.restype = _i
lib.polydl_conv2d_fwd_noalloc.argtypes = [_i] * 9 + [_p, _p, _p, _p, _i, _p]
lib.polydl_conv2d_fwd_noalloc.restype = _i
lib.polydl_conv2d_fwd_tap.argtypes = [_i] * 9 + [_p, _p, _p, _p, _p, _i, _p]
lib.polydl_conv2d_fwd_tap.restype = _i
lib.polydl_sgemm.argtypes = [_i, _i, _i, _p, _p, _p, _p]
lib.polydl_sgemm_ex.argtypes = [_i, _i, _i, ctypes.c_float, _p, _p, ctypes.c_float, _p, _p]
lib.polydl_sgemm_ex.restype = _i
lib.polydl_model_conv2d_bf16.argtypes = [_i] * 9 + [ctypes.POINTER(TileCfg), ctypes.POINTER(ctypes.c_double)]
lib.polydl_pick_conv2d_bf16.argtypes = [_i] * 9 + [ctypes.POINTER(TileCfg), ctypes.POINTER(ctypes.c_double)]
lib.polydl_model_conv2d_bf16.restype = _i
lib.polydl_pick_conv2d_bf16.restype = _i
_dp, _ip = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int)
lib.polydl_ranker_num_params.argtypes = []
lib.polydl_ranker_set_params.argtypes = [_dp, _i]
lib.polydl_ranker_stats_conv2d.argtypes = [_i] * 9 + [ctypes.POINTER(TileCfg), _dp]
lib.polydl_ranker_play.argtypes = [_dp, _dp, ctypes.c_double, _dp, _ip]
lib.polydl_ranker_tournament.argtypes = [_i, _dp, ctypes.c_double, _ip, _ip]
lib.polydl_pick_conv2d_learned.argtypes = [_i] * 9 + [ctypes.c_double, ctypes.POINTER(TileCfg),
                                                      ctypes.POINTER(ModelReport), _ip, _ip]
for _f in (lib.polydl_ranker_num_params, lib.polydl_ranker_set_params, lib.polydl_ranker_stats_conv2d,
           lib.polydl_ranker_play, lib.polydl_ranker_tournament, lib.polydl_pick_conv2d_learned):
    _f.restype = _i
lib.polydl_nchw_to_nchwc.argtypes = [_i] * 5 + [_p, _p, _p]
lib.polydl_nchwc_to_nchw.argtypes = [_i] * 5 + [_p, _p, _p]
lib.polydl_kcrs_to_kcrsck.argtypes = [_i] * 6 + [_p, _p, _p]
lib.polydl_bias_add.argtypes = [_i] * 4 + [_p, _p, _p]
lib.polydl_activation.argtypes = [ctypes.c_int64, _p, _i, _p]
lib.polydl_bnorm_fwd.argtypes = [_i] * 4 + [_p] * 5 + [ctypes.c_float, _p, _i, _p]
lib.polydl_bnorm_fwd.restype = _i
for _f in (lib.polydl_nchw_to_nchwc, lib.polydl_nchwc_to_nchw, lib.polydl_kcrs_to_kcrsck,
           lib.polydl_bias_add, lib.polydl_activation):
    _f.restype = _i
_d = ctypes.c_double
_pd = ctypes.POINTER(ctypes.c_double)
lib.polydl_reuse_bucket.argtypes = [_i, _pd, _i, _pd, _pd, _pd]
lib.polydl_reuse_bucket.restype = _i
lib.polydl_reuse_cost.argtypes = [_i, _pd, _d, _pd, _d]
lib.polydl_reuse_cost.restype = _d
lib.polydl_model_conv2d.argtypes = [_i] * 9 + [ctypes.POINTER(TileCfg), ctypes.POINTER(ModelReport)]
lib.polydl_model_sgemm.argtypes = [_i] * 3 + [ctypes.POINTER(TileCfg), ctypes.POINTER(ModelReport)]
lib.polydl_pick_conv2d.argtypes = [_i] * 9 + [ctypes.POINTER(TileCfg), ctypes.POINTER(ModelReport)]
lib.polydl_pick_sgemm.argtypes = [_i] * 3 + [ctypes.POINTER(TileCfg), ctypes.POINTER(ModelReport)]
for _f in (lib.polydl_model_conv2d, lib.polydl_model_sgemm, lib.polydl_pick_conv2d, lib.polydl_pick_sgemm):
    _f.restype = _i
lib.polydl_nchw_to_nchwc_bf16.argtypes = [_i] * 5 + [_p, _p, _p]
lib.polydl_kcrs_to_kcrsck_bf16.argtypes = [_i] * 6 + [_p, _p, _p]
lib.polydl_conv2d_fwd_bf16_blocked.argtypes = [_i] * 9 + [_p, _p, _p, _p, _i, _p]
lib.polydl_conv2d_bf16_workspace_bytes.argtypes = [_i] * 7
lib.polydl_conv2d_bf16_workspace_bytes.restype = ctypes.c_size_t
lib.polydl_conv2d_fwd_bf16.argtypes = [_i] * 9 + [_p, _p, _p, _p, _i, _p, ctypes.c_size_t, _p]
for _f in (lib.polydl_nchw_to_nchwc_bf16, lib.polydl_kcrs_to_kcrsck_bf16, lib.polydl_conv2d_fwd_bf16_blocked,
           lib.polydl_conv2d_fwd_bf16):
    _f.restype = _i
lib.polydl_set_tile_override.argtypes = [ctypes.POINTER(TileCfg)]
lib.polydl_get_last_tile.argtypes = [ctypes.POINTER(TileCfg)]
lib.polydl_num_variants.argtypes = [_i]
lib.polydl_get_variant.argtypes = [_i, _i, ctypes.POINTER(TileCfg)]
lib.polydl_status_string.argtypes = [_i]
lib.polydl_status_string.restype = ctypes.c_char_p
for _f in (lib.polydl_conv2d_fwd, lib.polydl_conv2d_fwd_act, lib.polydl_sgemm,
           lib.polydl_set_tile_override, lib.polydl_get_last_tile, lib.polydl_num_variants,
           lib.polydl_get_variant):
    _f.restype = _i


def status_string(status):
    return lib.polydl_status_string(int(status)).decode()


def _check(status, where):
    if status != 0:
        raise PolydlError(status, where)


def _stream_ptr(stream=None):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _dev(t, name):
    """Device pointer of a contiguous float32 CUDA/HIP tensor (None passes NULL)."""
    if t is None:
        return None
    if not (t.is_cuda and t.is_contiguous() and t.dtype.is_floating_point and t.element_size() == 4):
        raise TypeError("%s must be a contiguous float32 tensor in device memory" % name)
    return ctypes.c_void_p(t.data_ptr())


def _dev16(t, name):
    """Device pointer of a contiguous 2-byte-element tensor holding bfloat16 bit patterns."""
    if not (t.is_cuda and t.is_contiguous() and t.element_size() == 2):
        raise TypeError("%s must be a contiguous 16-bit tensor in device memory" % name)
    return ctypes.c_void_p(t.data_ptr())


def nchw_to_nchwc_bf16(x, b=8, stream=None, out=None):
    """polydl_nchw_to_nchwc_bf16 on a 16-bit NCHW tensor: returns [N][ceil(C/b)][H][W][b]."""
    import torch
    N, C, H, W = x.shape
    if out is None:
        out = torch.empty((N, -(-C // b), H, W, b), dtype=x.dtype, device=x.device)
    elif tuple(out.shape) != (N, -(-C // b), H, W, b) or out.dtype != x.dtype:
        raise ValueError("out must be a [N][ceil(C/b)][H][W][b] tensor of the input's type")
    _check(lib.polydl_nchw_to_nchwc_bf16(N, C, H, W, b, _dev16(x, "x"), _dev16(out, "out"), _stream_ptr(stream)),
           "polydl_nchw_to_nchwc_bf16")
    return out


def kcrs_to_kcrsck_bf16(w, bc=8, bk=1, stream=None, out=None):
    """polydl_kcrs_to_kcrsck_bf16: returns [ceil(K/bk)][ceil(C/bc)][R][S][bc][bk] (16-bit elements)."""
    import torch
    K, C, R, S = w.shape
    if out is None:
        out = torch.empty((-(-K // bk), -(-C // bc), R, S, bc, bk), dtype=w.dtype, device=w.device)
    elif tuple(out.shape) != (-(-K // bk), -(-C // bc), R, S, bc, bk) or out.dtype != w.dtype:
        raise ValueError("out must be a [ceil(K/bk)][ceil(C/bc)][R][S][bc][bk] tensor of the input's type")
    _check(lib.polydl_kcrs_to_kcrsck_bf16(K, C, R, S, bc, bk, _dev16(w, "w"), _dev16(out, "out"),
                                          _stream_ptr(stream)), "polydl_kcrs_to_kcrsck_bf16")
    return out


def conv2d_fwd_bf16_blocked(x8c, w8c, C, bias=None, out=None, stride=1, pad=0, act=None, stream=None):
    """polydl_conv2d_fwd_bf16_blocked: x8c [N][C/8][H][W][8], w8c [K][C/8][R][S][8][1] bf16 bits."""
    import torch
    N, _, H, W, _ = x8c.shape
    K, _, R, S = w8c.shape[:4]
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    if out is None:
        out = torch.empty((N, K, max(P, 0), max(Q, 0)), dtype=torch.float32, device=x8c.device)
    st = lib.polydl_conv2d_fwd_bf16_blocked(N, C, H, W, K, R, S, stride, pad, _dev16(x8c, "x8c"),
                                            _dev16(w8c, "w8c"), _dev(bias, "bias"), _dev(out, "out"), ACT[act],
                                            _stream_ptr(stream))
    _check(st, "polydl_conv2d_fwd_bf16_blocked")
    return out


def conv2d_fwd_bf16(x, w, bias=None, out=None, stride=1, pad=0, act=None, workspace=None, stream=None):
    """polydl_conv2d_fwd_bf16 on 16-bit NCHW / KCRS tensors; allocates the workspace when not given."""
    import torch
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    need = lib.polydl_conv2d_bf16_workspace_bytes(N, C, H, W, K, R, S)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    if out is None:
        out = torch.empty((N, K, max(P, 0), max(Q, 0)), dtype=torch.float32, device=x.device)
    st = lib.polydl_conv2d_fwd_bf16(N, C, H, W, K, R, S, stride, pad, _dev16(x, "x"), _dev16(w, "w"),
                                    _dev(bias, "bias"), _dev(out, "out"), ACT[act],
                                    ctypes.c_void_p(workspace.data_ptr()), workspace.numel(), _stream_ptr(stream))
    _check(st, "polydl_conv2d_fwd_bf16")
    return out


def filter_tap_copy(w, stream=None, out=None):
    """The [K][R][S][C] copy of a KCRS filter that conv2d_fwd(..., w_tap=) takes: polydl_kcrs_to_kcrsck
    with bc = C, bk = 1."""
    K, C, R, S = w.shape
    return kcrs_to_kcrsck(w, C, 1, stream=stream, out=out).view(K, R, S, C)


def conv2d_fwd(x, w, bias=None, out=None, stride=1, pad=0, act=None, stream=None, pre_act=None, w_tap=None):
    """polydl_conv2d_fwd_act on torch device tensors x (NCHW), w (KCRS); returns out (NKPQ).
    With pre_act given, polydl_conv2d_fwd_pre_act: the convolution of pre_act(x).
    With w_tap given (filter_tap_copy(w)), polydl_conv2d_fwd_tap."""
    import torch
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    if C2 != C:
        raise ValueError("channel mismatch")
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    if out is None:
        out = torch.empty((N, K, max(P, 0), max(Q, 0)), dtype=torch.float32, device=x.device)
    if w_tap is not None:
        if pre_act is not None:
            raise ValueError("w_tap and pre_act do not combine")
        if tuple(w_tap.shape) != (K, R, S, C):
            raise ValueError("w_tap must be [K][R][S][C]")
        st = lib.polydl_conv2d_fwd_tap(N, C, H, W, K, R, S, stride, pad, _dev(x, "x"), _dev(w, "w"),
                                       _dev(w_tap, "w_tap"), _dev(bias, "bias"), _dev(out, "out"), ACT[act],
                                       _stream_ptr(stream))
    elif pre_act is None:
        st = lib.polydl_conv2d_fwd_act(N, C, H, W, K, R, S, stride, pad, _dev(x, "x"), _dev(w, "w"),
                                       _dev(bias, "bias"), _dev(out, "out"), ACT[act], _stream_ptr(stream))
    else:
        st = lib.polydl_conv2d_fwd_pre_act(N, C, H, W, K, R, S, stride, pad, _dev(x, "x"), _dev(w, "w"),
                                           _dev(bias, "bias"), _dev(out, "out"), ACT[pre_act], ACT[act],
                                           _stream_ptr(stream))
    _check(st, "polydl_conv2d_fwd")
    return out


def conv2d_fwd_noalloc(x, w, bias, out, stride=1, pad=0, act=None, stream=None):
    """polydl_conv2d_fwd_noalloc: as conv2d_fwd into a caller-provided out, scratch memory from the
    library's fixed array (the call allocates nothing)."""
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    if C2 != C:
        raise ValueError("channel mismatch")
    st = lib.polydl_conv2d_fwd_noalloc(N, C, H, W, K, R, S, stride, pad, _dev(x, "x"), _dev(w, "w"),
                                       _dev(bias, "bias"), _dev(out, "out"), ACT[act], _stream_ptr(stream))
    _check(st, "polydl_conv2d_fwd_noalloc")
    return out


def sgemm(A, B, C, stream=None, alpha=None, beta=None):
    """polydl_sgemm: C += A @ B in place on torch device tensors (row-major); with alpha or beta
    given, polydl_sgemm_ex: C = beta*C + alpha*A@B."""
    M, K = A.shape
    K2, N = B.shape
    if K2 != K or tuple(C.shape) != (M, N):
        raise ValueError("shape mismatch")
    if alpha is None and beta is None:
        st = lib.polydl_sgemm(M, N, K, _dev(A, "A"), _dev(B, "B"), _dev(C, "C"), _stream_ptr(stream))
        _check(st, "polydl_sgemm")
        return C
    st = lib.polydl_sgemm_ex(M, N, K, ctypes.c_float(1.0 if alpha is None else alpha), _dev(A, "A"), _dev(B, "B"),
                             ctypes.c_float(1.0 if beta is None else beta), _dev(C, "C"), _stream_ptr(stream))
    _check(st, "polydl_sgemm_ex")
    return C


def nchw_to_nchwc(x, b, stream=None, out=None):
    """polydl_nchw_to_nchwc: returns the [N][ceil(C/b)][H][W][b] tensor (written into out if given)."""
    import torch
    N, C, H, W = x.shape
    if out is None:
        out = torch.empty((N, -(-C // b), H, W, b), dtype=torch.float32, device=x.device)
    _check(lib.polydl_nchw_to_nchwc(N, C, H, W, b, _dev(x, "x"), _dev(out, "out"), _stream_ptr(stream)),
           "polydl_nchw_to_nchwc")
    return out


def nchwc_to_nchw(xb, C, stream=None, out=None):
    """polydl_nchwc_to_nchw: returns the [N][C][H][W] tensor (written into out if given)."""
    import torch
    N, Cb, H, W, b = xb.shape
    if out is None:
        out = torch.empty((N, C, H, W), dtype=torch.float32, device=xb.device)
    _check(lib.polydl_nchwc_to_nchw(N, C, H, W, b, _dev(xb, "xb"), _dev(out, "out"), _stream_ptr(stream)),
           "polydl_nchwc_to_nchw")
    return out


def kcrs_to_kcrsck(w, bc, bk, stream=None, out=None):
    """polydl_kcrs_to_kcrsck: returns the [ceil(K/bk)][ceil(C/bc)][R][S][bc][bk] tensor (out if given)."""
    import torch
    K, C, R, S = w.shape
    if out is None:
        out = torch.empty((-(-K // bk), -(-C // bc), R, S, bc, bk), dtype=torch.float32, device=w.device)
    _check(lib.polydl_kcrs_to_kcrsck(K, C, R, S, bc, bk, _dev(w, "w"), _dev(out, "out"), _stream_ptr(stream)),
           "polydl_kcrs_to_kcrsck")
    return out


def bias_add(y, bias, stream=None):
    """polydl_bias_add, in place on an NKPQ tensor."""
    N, K, P, Q = y.shape
    _check(lib.polydl_bias_add(N, K, P, Q, _dev(y, "y"), _dev(bias, "bias"), _stream_ptr(stream)), "polydl_bias_add")
    return y


def bnorm_fwd(x, gamma, beta, mean, var, eps=1e-5, out=None, act=None, stream=None):
    """polydl_bnorm_fwd on an NKPQ tensor; out defaults to a new tensor (pass out=x for in place)."""
    import torch
    N, K, P, Q = x.shape
    if out is None:
        out = torch.empty_like(x)
    st = lib.polydl_bnorm_fwd(N, K, P, Q, _dev(x, "x"), _dev(gamma, "gamma"), _dev(beta, "beta"), _dev(mean, "mean"),
                              _dev(var, "var"), ctypes.c_float(eps), _dev(out, "out"), ACT[act], _stream_ptr(stream))
    _check(st, "polydl_bnorm_fwd")
    return out


def activation(y, act="relu", stream=None):
    """polydl_activation, in place."""
    _check(lib.polydl_activation(y.numel(), _dev(y, "y"), ACT[act], _stream_ptr(stream)), "polydl_activation")
    return y


def reuse_bucket(ws, sizes):
    """polydl_reuse_bucket on Python sequences: returns (per-level sums, memory sum)."""
    n, m = len(ws), len(sizes)
    a = (ctypes.c_double * max(n, 1))(*ws)
    b = (ctypes.c_double * max(m, 1))(*sizes)
    lv = (ctypes.c_double * max(m, 1))()
    mem = ctypes.c_double()
    _check(lib.polydl_reuse_bucket(n, a, m, b, lv, ctypes.byref(mem)), "polydl_reuse_bucket")
    return list(lv)[:m], mem.value


def reuse_cost(levels, mem, weights, mem_weight):
    """polydl_reuse_cost on Python sequences."""
    m = len(levels)
    return lib.polydl_reuse_cost(m, (ctypes.c_double * max(m, 1))(*levels), mem,
                                 (ctypes.c_double * max(m, 1))(*weights), mem_weight)


lib.polydl_model_get_levels.argtypes = [_pd, _pd, _pd]
lib.polydl_model_set_levels.argtypes = [_pd, _pd, _d]
lib.polydl_model_get_levels.restype = _i
lib.polydl_model_set_levels.restype = _i


def model_get_levels():
    """polydl_model_get_levels: (capacities in bytes, rates in GB/s, memory rate in GB/s)."""
    cap, rate, mem = (ctypes.c_double * 4)(), (ctypes.c_double * 4)(), ctypes.c_double()
    _check(lib.polydl_model_get_levels(cap, rate, ctypes.byref(mem)), "polydl_model_get_levels")
    return list(cap), list(rate), mem.value


def model_set_levels(capacity, rate, mem_rate):
    """polydl_model_set_levels: replace the model's memory-hierarchy table (process-wide)."""
    _check(lib.polydl_model_set_levels((ctypes.c_double * 4)(*capacity), (ctypes.c_double * 4)(*rate), mem_rate),
           "polydl_model_set_levels")


def model_conv2d(shape, cfg):
    """polydl_model_conv2d for a synth.ConvShape-like tuple (N, C, H, W, K, R, S, stride, pad)."""
    rep = ModelReport()
    _check(lib.polydl_model_conv2d(*[int(v) for v in shape], ctypes.byref(cfg), ctypes.byref(rep)),
           "polydl_model_conv2d")
    return rep


def model_sgemm(M, N, K, cfg):
    rep = ModelReport()
    _check(lib.polydl_model_sgemm(M, N, K, ctypes.byref(cfg), ctypes.byref(rep)), "polydl_model_sgemm")
    return rep


def pick_conv2d(shape):
    """polydl_pick_conv2d: (TileCfg, ModelReport) of the variant the reuse model ranks first."""
    cfg, rep = TileCfg(), ModelReport()
    _check(lib.polydl_pick_conv2d(*[int(v) for v in shape], ctypes.byref(cfg), ctypes.byref(rep)),
           "polydl_pick_conv2d")
    return cfg, rep


REUSE_MAX_LOOPS = 8


class LoopRef(ctypes.Structure):
    """Mirror of polydl_loop_ref."""
    _fields_ = [("array", ctypes.c_int), ("rank", ctypes.c_int), ("coef", (ctypes.c_int * REUSE_MAX_LOOPS) * 4),
                ("offset", ctypes.c_int * 4)]


class ReuseDep(ctypes.Structure):
    """Mirror of polydl_reuse_dep."""
    _fields_ = [("src_ref", ctypes.c_int), ("tgt_ref", ctypes.c_int), ("n_pairs", ctypes.c_int),
                ("parallel", ctypes.c_int), ("n_ws", ctypes.c_int), ("ws", ctypes.c_double * 2),
                ("source", ctypes.c_int * REUSE_MAX_LOOPS), ("min_target", ctypes.c_int * REUSE_MAX_LOOPS),
                ("max_target", ctypes.c_int * REUSE_MAX_LOOPS)]


lib.polydl_reuse_analyse.argtypes = [_i, _ip, _ip, _i, ctypes.POINTER(LoopRef), _i, ctypes.POINTER(ReuseDep), _ip]
lib.polydl_reuse_analyse.restype = _i


def reuse_analyse(extents, refs, parallel=None, max_deps=64):
    """polydl_reuse_analyse.  refs: [(array id, [[coefficient per loop] per subscript], [offset per subscript])];
    parallel: one flag per loop.  Returns a list of dicts (one per dependence)."""
    n = len(extents)
    ext = (ctypes.c_int * n)(*[int(e) for e in extents])
    par = None if parallel is None else (ctypes.c_int * n)(*[int(bool(f)) for f in parallel])
    arr = (LoopRef * len(refs))()
    for r, (array, coef, offset) in enumerate(refs):
        arr[r].array, arr[r].rank = int(array), len(coef)
        for d, row in enumerate(coef):
            for l, c in enumerate(row):
                arr[r].coef[d][l] = int(c)
            arr[r].offset[d] = int(offset[d])
    deps, nd = (ReuseDep * max_deps)(), ctypes.c_int(0)
    _check(lib.polydl_reuse_analyse(n, ext, par, len(refs), arr, max_deps, deps, ctypes.byref(nd)),
           "polydl_reuse_analyse")
    out = []
    for d in deps[:min(nd.value, max_deps)]:
        out.append({"src_ref": d.src_ref, "tgt_ref": d.tgt_ref, "n_pairs": d.n_pairs, "parallel": bool(d.parallel),
                    "ws": [int(v) for v in list(d.ws)[:d.n_ws]], "source": tuple(d.source[:n]),
                    "min_target": None if d.parallel else tuple(d.min_target[:n]),
                    "max_target": None if d.parallel else tuple(d.max_target[:n])})
    return out


RANKER_STATS = 8
RANKER_PARAMS_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "ranker_params.txt")


def _doubles(values, count=None):
    values = [float(v) for v in values]
    if count is not None and len(values) != count:
        raise ValueError("expected %d values, got %d" % (count, len(values)))
    return (ctypes.c_double * len(values))(*values)


def ranker_num_params():
    return lib.polydl_ranker_num_params()


def ranker_set_params(params):
    """polydl_ranker_set_params: load the pairwise network's parameters (flat sequence of floats)."""
    buf = _doubles(params)
    _check(lib.polydl_ranker_set_params(buf, len(buf)), "polydl_ranker_set_params")


def ranker_load(path=None):
    """Read a parameter file (one number per line, '#' comments) and load it into the library."""
    vals = []
    with open(path or RANKER_PARAMS_PATH) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                vals.append(float(line))
    ranker_set_params(vals)


def ranker_stats_conv2d(shape, cfg):
    """polydl_ranker_stats_conv2d: the statistics of one variant the network is fed."""
    out = (ctypes.c_double * RANKER_STATS)()
    _check(lib.polydl_ranker_stats_conv2d(*[int(v) for v in shape], ctypes.byref(cfg), out),
           "polydl_ranker_stats_conv2d")
    return list(out)


def ranker_play(stats1, stats2, theta=0.6):
    """polydl_ranker_play: (winner, [p1, p2]); winner 1, 2 or 0 for a draw."""
    probs, winner = (ctypes.c_double * 2)(), ctypes.c_int(-1)
    _check(lib.polydl_ranker_play(_doubles(stats1, RANKER_STATS), _doubles(stats2, RANKER_STATS), theta, probs,
                                  ctypes.byref(winner)), "polydl_ranker_play")
    return winner.value, list(probs)


def ranker_tournament(stats, theta=0.6):
    """polydl_ranker_tournament over a list of statistics vectors: (wins, order)."""
    n = len(stats)
    flat = _doubles([v for s in stats for v in s], n * RANKER_STATS)
    wins, order = (ctypes.c_int * max(n, 1))(), (ctypes.c_int * max(n, 1))()
    _check(lib.polydl_ranker_tournament(n, flat, theta, wins, order), "polydl_ranker_tournament")
    return list(wins)[:n], list(order)[:n]


def pick_conv2d_learned(shape, theta=0.6):
    """polydl_pick_conv2d_learned: (TileCfg, ModelReport, games won, games played) of the tournament's winner."""
    cfg, rep, wins, games = TileCfg(), ModelReport(), ctypes.c_int(0), ctypes.c_int(0)
    _check(lib.polydl_pick_conv2d_learned(*[int(v) for v in shape], theta, ctypes.byref(cfg), ctypes.byref(rep),
                                          ctypes.byref(wins), ctypes.byref(games)), "polydl_pick_conv2d_learned")
    return cfg, rep, wins.value, games.value


def model_conv2d_bf16(shape, cfg):
    """polydl_model_conv2d_bf16: predicted microseconds of one bfloat16 variant (algo 1, cb and split_k set)."""
    us = ctypes.c_double(0.0)
    _check(lib.polydl_model_conv2d_bf16(*[int(v) for v in shape], ctypes.byref(cfg), ctypes.byref(us)),
           "polydl_model_conv2d_bf16")
    return us.value


def pick_conv2d_bf16(shape):
    """polydl_pick_conv2d_bf16: (TileCfg, predicted microseconds) of the bfloat16 variant ranked first."""
    cfg, us = TileCfg(), ctypes.c_double(0.0)
    _check(lib.polydl_pick_conv2d_bf16(*[int(v) for v in shape], ctypes.byref(cfg), ctypes.byref(us)),
           "polydl_pick_conv2d_bf16")
    return cfg, us.value


def pick_sgemm(M, N, K):
    cfg, rep = TileCfg(), ModelReport()
    _check(lib.polydl_pick_sgemm(M, N, K, ctypes.byref(cfg), ctypes.byref(rep)), "polydl_pick_sgemm")
    return cfg, rep


lib.polydl_conv2d_candidates.argtypes = [_i] * 11 + [ctypes.POINTER(TileCfg), _ip]
lib.polydl_sgemm_candidates.argtypes = [_i] * 4 + [ctypes.POINTER(TileCfg), _ip]
lib.polydl_conv2d_candidates.restype = _i
lib.polydl_sgemm_candidates.restype = _i


def _candidates(call, where):
    n = ctypes.c_int(0)
    _check(call(0, None, ctypes.byref(n)), where)
    arr = (TileCfg * max(n.value, 1))()
    _check(call(n.value, arr, ctypes.byref(n)), where)
    return [TileCfg(*[getattr(arr[i], f) for f, _ in TileCfg._fields_]) for i in range(n.value)]


def conv_candidates(shape, tap=False):
    """polydl_conv2d_candidates, kind 0: every variant polydl_pick_conv2d ranks for this problem;
    tap=True, kind 3: the variants ranked when the filter's [K][R][S][C] copy is given."""
    dims = [int(v) for v in shape]
    kind = 3 if tap else 0
    return _candidates(lambda m, a, n: lib.polydl_conv2d_candidates(*dims, kind, m, a, n), "polydl_conv2d_candidates")


def sgemm_candidates(M, N, K):
    """polydl_sgemm_candidates: every variant polydl_pick_sgemm ranks."""
    return _candidates(lambda m, a, n: lib.polydl_sgemm_candidates(M, N, K, m, a, n), "polydl_sgemm_candidates")


def conv_candidates_bf16(shape):
    """polydl_conv2d_candidates, kind 2: every variant polydl_pick_conv2d_bf16 ranks."""
    dims = [int(v) for v in shape]
    return _candidates(lambda m, a, n: lib.polydl_conv2d_candidates(*dims, 2, m, a, n), "polydl_conv2d_candidates")


def set_tile_override(cfg=None, **kw):
    """Force a variant (TileCfg or keyword fields) for later calls; None returns to the picker."""
    if cfg is None and not kw:
        _check(lib.polydl_set_tile_override(None), "polydl_set_tile_override")
        return
    if cfg is None:
        cfg = TileCfg(kw["bm"], kw["bn"], kw.get("bk", 0), kw["wm"], kw["wn"], kw.get("split_k", 1),
                      kw.get("layout", 0), kw.get("raster", 0), kw.get("algo", 0), kw.get("cb", 0))
    _check(lib.polydl_set_tile_override(ctypes.byref(cfg)), "polydl_set_tile_override")


def get_last_tile():
    cfg = TileCfg()
    _check(lib.polydl_get_last_tile(ctypes.byref(cfg)), "polydl_get_last_tile")
    return cfg


def variants(kind=0):
    """The compiled variant family (kind 0 = convolution, 1 = sgemm, 2 = bfloat16 convolution) as a list of TileCfg."""
    n = lib.polydl_num_variants(kind)
    if n < 0:
        raise PolydlError(n, "polydl_num_variants")
    out = []
    for i in range(n):
        c = TileCfg()
        _check(lib.polydl_get_variant(kind, i, ctypes.byref(c)), "polydl_get_variant")
        out.append(c)
    return out

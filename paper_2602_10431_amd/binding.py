"""ctypes binding of libqtale.so: same names as the C ABI (include/qtale.h), argument marshalling only.

torch tensors are used as device-memory holders; their data pointers and the current HIP stream are
handed to the library.  Every step of the path runs in the library's kernels.  There is no fallback:
if the library is missing or a call fails, an exception is raised.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqtale.so")

QTALE_ACT_FP16, QTALE_ACT_BF16 = 0, 1
QTALE_MODE_RATIO, QTALE_MODE_THRESHOLD = 0, 1
QTALE_PROF_CLASSES = 10
PROF_NAMES = ["router", "select", "norm1", "qkv_gemm", "rope_append", "attention", "o_gemm", "norm2",
              "gate_up_gemm", "down_gemm"]
ERRORS = {-1: "INVALID_ARG", -2: "SHAPE", -3: "UNSUPPORTED", -4: "WORKSPACE_TOO_SMALL", -5: "HIP"}

EXPORTS = ["qtale_strerror", "qtale_create", "qtale_destroy", "qtale_set_exec_ratio", "qtale_set_threshold",
           "qtale_get_control", "qtale_prepacked_bytes", "qtale_quantize", "qtale_prepack",
           "qtale_workspace_bytes", "qtale_layer_forward", "qtale_stack_forward", "qtale_router_select",
           "qtale_linear_w4a16", "qtale_swiglu_w4a16", "qtale_profile_enable", "qtale_profile_read",
           "qtale_calibration_scratch_bytes", "qtale_calibrate_threshold_from_scores", "qtale_calibrate_threshold",
           "qtale_graph_capture_stack", "qtale_graph_launch", "qtale_graph_destroy", "qtale_router_mlp_scores",
           "qtale_static_scratch_bytes", "qtale_layer_forward_static"]
QTALE_THETA_GRID = 50


class QtaleError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__("%s failed: %s (%d)" % (where, ERRORS.get(code, "?"), code))


class qtale_layer_cfg(C.Structure):
    _fields_ = [("hidden", C.c_int), ("n_heads", C.c_int), ("n_kv_heads", C.c_int), ("head_dim", C.c_int),
                ("inter", C.c_int), ("bits", C.c_int), ("group", C.c_int), ("act_dtype", C.c_int),
                ("rms_eps", C.c_float), ("rope_base", C.c_float)]


class qtale_qlinear(C.Structure):
    _fields_ = [("codes", C.c_void_p), ("scales", C.c_void_p), ("zeros", C.c_void_p), ("prepacked", C.c_void_p),
                ("N", C.c_int), ("K", C.c_int)]


class qtale_layer_weights(C.Structure):
    _fields_ = [("q", qtale_qlinear), ("k", qtale_qlinear), ("v", qtale_qlinear), ("o", qtale_qlinear),
                ("gate", qtale_qlinear), ("up", qtale_qlinear), ("down", qtale_qlinear),
                ("norm1", C.c_void_p), ("norm2", C.c_void_p), ("router_w", C.c_void_p), ("router_b", C.c_float),
                ("router_hidden", C.c_int), ("router_w1", C.c_void_p), ("router_b1", C.c_void_p),
                ("router_w2", C.c_void_p), ("router_b2", C.c_void_p), ("bits", C.c_int)]


class qtale_kv(C.Structure):
    _fields_ = [("k_cache", C.c_void_p), ("v_cache", C.c_void_p), ("kv_len", C.c_void_p), ("cap", C.c_int)]


_lib = None


def load_library():
    """Loads libqtale.so (built in-tree by paper_2602_10431_amd/build.py).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError("%s not found: run `python -c 'import __graft_entry__ as g; g.build()'`" % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    vp, i, f, sz = C.c_void_p, C.c_int, C.c_float, C.c_size_t
    lib.qtale_strerror.restype = C.c_char_p
    lib.qtale_strerror.argtypes = [i]
    lib.qtale_create.argtypes = [C.POINTER(vp)]
    lib.qtale_destroy.argtypes = [vp]
    lib.qtale_set_exec_ratio.argtypes = [vp, f]
    lib.qtale_set_threshold.argtypes = [vp, f]
    lib.qtale_get_control.argtypes = [vp, C.POINTER(i), C.POINTER(f)]
    lib.qtale_prepacked_bytes.restype = sz
    lib.qtale_prepacked_bytes.argtypes = [i, i, i, i]
    lib.qtale_quantize.argtypes = [vp, i, i, i, i, vp, vp, vp, vp, vp]
    lib.qtale_prepack.argtypes = [vp, vp, vp, i, i, i, i, vp, vp]
    lib.qtale_workspace_bytes.restype = sz
    lib.qtale_workspace_bytes.argtypes = [C.POINTER(qtale_layer_cfg), i, i]
    lib.qtale_layer_forward.argtypes = [vp, C.POINTER(qtale_layer_cfg), C.POINTER(qtale_layer_weights), vp, i, vp, i,
                                        vp, C.POINTER(qtale_kv), vp, vp, vp, vp, sz, vp]
    lib.qtale_static_scratch_bytes.restype = sz
    lib.qtale_static_scratch_bytes.argtypes = []
    lib.qtale_layer_forward_static.argtypes = [vp, C.POINTER(qtale_layer_cfg), C.POINTER(qtale_layer_weights), vp, i, vp,
                                               i, vp, C.POINTER(qtale_kv), vp, vp, vp, vp]
    lib.qtale_stack_forward.argtypes = [vp, C.POINTER(qtale_layer_cfg), C.POINTER(qtale_layer_weights), i, vp, i, vp,
                                        i, vp, C.POINTER(qtale_kv), vp, vp, vp, vp, vp, sz, vp]
    lib.qtale_router_select.argtypes = [vp, i, vp, i, i, vp, f, vp, i, vp, vp, vp, vp, vp]
    lib.qtale_linear_w4a16.argtypes = [C.POINTER(qtale_qlinear), i, i, vp, i, vp, vp]
    lib.qtale_swiglu_w4a16.argtypes = [C.POINTER(qtale_qlinear), C.POINTER(qtale_qlinear), i, i, vp, i, vp, vp]
    fp = C.POINTER(C.c_float)
    lib.qtale_calibration_scratch_bytes.argtypes = [i]
    lib.qtale_calibration_scratch_bytes.restype = C.c_size_t
    lib.qtale_calibrate_threshold_from_scores.argtypes = [vp, vp, C.c_int64, C.c_float, vp, fp, fp, fp, vp]
    lib.qtale_calibrate_threshold.argtypes = [vp, C.POINTER(qtale_layer_cfg), C.POINTER(qtale_layer_weights), i, vp, vp,
                                              i, vp, i, vp, C.c_float, vp, vp, C.c_size_t, fp, fp, fp, vp]
    lib.qtale_graph_capture_stack.argtypes = [vp, C.POINTER(qtale_layer_cfg), C.POINTER(qtale_layer_weights), i, vp, i, vp,
                                              i, vp, C.POINTER(qtale_kv), vp, vp, vp, vp, C.c_size_t, C.POINTER(vp)]
    lib.qtale_router_mlp_scores.argtypes = [i, vp, i, i, vp, vp, vp, vp, i, vp, vp]
    lib.qtale_graph_launch.argtypes = [vp, vp]
    lib.qtale_graph_destroy.argtypes = [vp]
    lib.qtale_graph_destroy.restype = None
    lib.qtale_profile_enable.argtypes = [vp, i]
    lib.qtale_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    for name in EXPORTS:
        if name not in ("qtale_strerror", "qtale_prepacked_bytes", "qtale_workspace_bytes",
                        "qtale_calibration_scratch_bytes", "qtale_graph_destroy", "qtale_static_scratch_bytes"):
            getattr(lib, name).restype = i
    _lib = lib
    return lib


def _check(code, where):
    if code != 0:
        raise QtaleError(code, where)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _act_code(dtype):
    return {torch.float16: QTALE_ACT_FP16, torch.bfloat16: QTALE_ACT_BF16}[dtype]


def make_cfg(hidden, n_heads, n_kv_heads, head_dim, inter, bits=4, group=128, act_dtype="bf16",
             rms_eps=1e-5, rope_base=10000.0):
    code = {"fp16": QTALE_ACT_FP16, "bf16": QTALE_ACT_BF16}[act_dtype]
    return qtale_layer_cfg(hidden, n_heads, n_kv_heads, head_dim, inter, bits, group, code, rms_eps, rope_base)


class Context:
    """Owns a qtale_ctx (the runtime control state)."""

    def __init__(self):
        self._h = C.c_void_p()
        _check(load_library().qtale_create(C.byref(self._h)), "qtale_create")

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.qtale_destroy(self._h)
            self._h = None


def qtale_set_exec_ratio(ctx, r):
    _check(load_library().qtale_set_exec_ratio(ctx._h, float(r)), "qtale_set_exec_ratio")


def qtale_set_threshold(ctx, theta):
    _check(load_library().qtale_set_threshold(ctx._h, float(theta)), "qtale_set_threshold")


def qtale_get_control(ctx):
    m, v = C.c_int(), C.c_float()
    _check(load_library().qtale_get_control(ctx._h, C.byref(m), C.byref(v)), "qtale_get_control")
    return m.value, v.value


def qtale_prepacked_bytes(N, K, bits=4, group=128):
    return load_library().qtale_prepacked_bytes(N, K, bits, group)


class QuantLinear:
    """Device buffers of one quantized linear: canonical codes/scales/zeros and the prepacked copy."""

    def __init__(self, N, K, bits, group, codes, scales, zeros, prepacked):
        self.N, self.K, self.bits, self.group = N, K, bits, group
        self.codes, self.scales, self.zeros, self.prepacked = codes, scales, zeros, prepacked

    def c_struct(self):
        return qtale_qlinear(self.codes.data_ptr() if self.codes is not None else None,
                             self.scales.data_ptr() if self.scales is not None else None,
                             self.zeros.data_ptr() if self.zeros is not None else None,
                             self.prepacked.data_ptr(), self.N, self.K)


def canonical_words(K, bits):
    """uint32 words per row of the canonical code array."""
    return 3 * ((K + 31) // 32) if bits == 3 else (K + 15) // 16 if bits == 2 else (K + 7) // 8


def qtale_quantize(W, bits=4, group=128, keep_canonical=True):
    """W: fp32 [N, K] CUDA tensor.  Returns a QuantLinear whose buffers were written by the library."""
    assert W.is_cuda and W.dtype == torch.float32 and W.is_contiguous()
    N, K = W.shape
    ng = (K + group - 1) // group
    codes = torch.empty((N, canonical_words(K, bits)), dtype=torch.int32, device=W.device)
    scales = torch.empty((N, ng), dtype=torch.float16, device=W.device)
    zeros = torch.empty((N, ng), dtype=torch.float16, device=W.device)
    nbytes = qtale_prepacked_bytes(N, K, bits, group)
    if nbytes == 0:
        raise QtaleError(-3, "qtale_prepacked_bytes")
    pre = torch.empty(nbytes, dtype=torch.uint8, device=W.device)
    _check(load_library().qtale_quantize(_ptr(W), N, K, bits, group, _ptr(codes), _ptr(scales), _ptr(zeros),
                                         _ptr(pre), _stream()), "qtale_quantize")
    if not keep_canonical:
        torch.cuda.current_stream().synchronize()
        return QuantLinear(N, K, bits, group, None, None, None, pre)
    return QuantLinear(N, K, bits, group, codes, scales, zeros, pre)


def qtale_prepack(codes, scales, zeros, N, K, bits=4, group=128):
    nbytes = qtale_prepacked_bytes(N, K, bits, group)
    pre = torch.empty(nbytes, dtype=torch.uint8, device=codes.device)
    _check(load_library().qtale_prepack(_ptr(codes), _ptr(scales), _ptr(zeros), N, K, bits, group, _ptr(pre),
                                        _stream()), "qtale_prepack")
    return QuantLinear(N, K, bits, group, codes, scales, zeros, pre)


class LayerWeights:
    """Holds the device tensors of one layer and the matching C struct."""

    def __init__(self, q, k, v, o, gate, up, down, norm1, norm2, router_w, router_b=0.0, router_mlp=None):
        """router_mlp: None (linear router) or (W1 [R,H], b1 [R], W2 [2,R], b2 [2]) fp32 CUDA tensors."""
        self.lin = dict(q=q, k=k, v=v, o=o, gate=gate, up=up, down=down)
        self.norm1, self.norm2, self.router_w, self.router_b = norm1, norm2, router_w, float(router_b)
        self.router_mlp = router_mlp
        if router_mlp is not None:
            W1, b1, W2, b2 = router_mlp
            for t in router_mlp:
                assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
            assert W2.shape == (2, W1.shape[0]) and b1.shape == (W1.shape[0],) and b2.shape == (2,)

    def c_struct(self):
        l = self.lin
        return qtale_layer_weights(l["q"].c_struct(), l["k"].c_struct(), l["v"].c_struct(), l["o"].c_struct(),
                                   l["gate"].c_struct(), l["up"].c_struct(), l["down"].c_struct(),
                                   self.norm1.data_ptr(), self.norm2.data_ptr(),
                                   self.router_w.data_ptr() if self.router_w is not None else None, self.router_b,
                                   *((0, None, None, None, None) if self.router_mlp is None else
                                     (self.router_mlp[0].shape[0],) + tuple(t.data_ptr() for t in self.router_mlp)),
                                   l["q"].bits)


class KVCache:
    def __init__(self, k_cache, v_cache, kv_len):
        # k_cache / v_cache: [B, n_kv_heads, cap, head_dim] fp16, contiguous
        assert k_cache.dtype == torch.float16 and v_cache.dtype == torch.float16 and kv_len.dtype == torch.int32
        assert k_cache.dim() == 4 and k_cache.shape == v_cache.shape and k_cache.is_contiguous() and v_cache.is_contiguous()
        self.k, self.v, self.kv_len = k_cache, v_cache, kv_len
        self.cap = k_cache.shape[2]

    @classmethod
    def from_token_major(cls, k, v, kv_len, n_kv_heads):
        """k, v: [B, cap, n_kv_heads * head_dim] (one row per cached token) -> the library's layout."""
        B, cap, W = k.shape
        d = W // n_kv_heads
        conv = lambda t: t.view(B, cap, n_kv_heads, d).permute(0, 2, 1, 3).contiguous()
        return cls(conv(k), conv(v), kv_len)

    def k_token_major(self):
        B, nkv, cap, d = self.k.shape
        return self.k.permute(0, 2, 1, 3).reshape(B, cap, nkv * d)

    def v_token_major(self):
        B, nkv, cap, d = self.v.shape
        return self.v.permute(0, 2, 1, 3).reshape(B, cap, nkv * d)

    def c_struct(self):
        return qtale_kv(self.k.data_ptr(), self.v.data_ptr(), self.kv_len.data_ptr(), self.cap)


def qtale_workspace_bytes(cfg, max_tokens, max_seqs):
    return load_library().qtale_workspace_bytes(C.byref(cfg), max_tokens, max_seqs)


def alloc_workspace(cfg, max_tokens, max_seqs, device="cuda"):
    n = qtale_workspace_bytes(cfg, max_tokens, max_seqs)
    if n == 0 and max_tokens > 0:
        raise QtaleError(-1, "qtale_workspace_bytes")
    return torch.empty(max(n, 256), dtype=torch.uint8, device=device)


def qtale_layer_forward(ctx, cfg, weights, x, seq_offsets, positions, kv=None, sel_idx=None, sel_count=None,
                        scores=None, workspace=None):
    T = x.shape[0]
    B = seq_offsets.numel() - 1
    if workspace is None:
        workspace = alloc_workspace(cfg, T, B, x.device)
    w = weights.c_struct()
    kvs = kv.c_struct() if kv is not None else None
    _check(load_library().qtale_layer_forward(
        ctx._h, C.byref(cfg), C.byref(w), _ptr(x), T, _ptr(seq_offsets), B, _ptr(positions),
        C.byref(kvs) if kvs is not None else None, _ptr(sel_idx), _ptr(sel_count), _ptr(scores),
        _ptr(workspace), workspace.numel(), _stream()), "qtale_layer_forward")


def qtale_static_scratch_bytes():
    return load_library().qtale_static_scratch_bytes()


def qtale_layer_forward_static(ctx, cfg, weights, x, seq_offsets, positions, kv=None, sel_idx=None, sel_count=None,
                               scores=None):
    """qtale_layer_forward on the library's own scratch array: the call allocates nothing."""
    T = x.shape[0]
    B = seq_offsets.numel() - 1
    w = weights.c_struct()
    kvs = kv.c_struct() if kv is not None else None
    _check(load_library().qtale_layer_forward_static(
        ctx._h, C.byref(cfg), C.byref(w), _ptr(x), T, _ptr(seq_offsets), B, _ptr(positions),
        C.byref(kvs) if kvs is not None else None, _ptr(sel_idx), _ptr(sel_count), _ptr(scores), _stream()),
        "qtale_layer_forward_static")


class Stack:
    """Pre-marshalled arguments of qtale_stack_forward for a fixed set of layers (and caches)."""

    def __init__(self, cfg, layers, kvs=None):
        self.cfg, self.layers, self.kvs = cfg, layers, kvs
        self.n = len(layers)
        self._w = (qtale_layer_weights * self.n)(*[l.c_struct() for l in layers])
        self._kv = (qtale_kv * self.n)(*[k.c_struct() for k in kvs]) if kvs is not None else None


def qtale_stack_forward(ctx, stack, x, seq_offsets, positions, sel_idx=None, sel_count=None, scores=None,
                        dbg_hidden=None, workspace=None):
    T = x.shape[0]
    B = seq_offsets.numel() - 1
    if workspace is None:
        workspace = alloc_workspace(stack.cfg, T, B, x.device)
    _check(load_library().qtale_stack_forward(
        ctx._h, C.byref(stack.cfg), stack._w, stack.n, _ptr(x), T, _ptr(seq_offsets), B, _ptr(positions),
        stack._kv, _ptr(sel_idx), _ptr(sel_count), _ptr(scores), _ptr(dbg_hidden), _ptr(workspace),
        workspace.numel(), _stream()), "qtale_stack_forward")


def _calibration_result(theta, ratio, table):
    seen = {n + 1: float(table[n]) for n in range(QTALE_THETA_GRID) if table[n] == table[n]}   # NaN = not evaluated
    return float(theta.value), float(ratio.value), seen


def qtale_calibrate_threshold_from_scores(ctx, scores, target_ratio):
    """scores: fp32 CUDA tensor (any shape).  Returns (theta, R_avg, {n: R_avg of theta = n/100}); ctx is left
    in threshold mode at theta."""
    assert scores.is_cuda and scores.dtype == torch.float32 and scores.is_contiguous()
    lib = load_library()
    scratch = torch.empty(lib.qtale_calibration_scratch_bytes(0), dtype=torch.uint8, device=scores.device)
    theta, ratio, table = C.c_float(), C.c_float(), (C.c_float * QTALE_THETA_GRID)()
    _check(lib.qtale_calibrate_threshold_from_scores(ctx._h, _ptr(scores), scores.numel(), float(target_ratio),
                                                     _ptr(scratch), C.byref(theta), C.byref(ratio), table, _stream()),
           "qtale_calibrate_threshold_from_scores")
    return _calibration_result(theta, ratio, table)


def qtale_calibrate_threshold(ctx, stack, x_calib, seq_offsets, positions, target_ratio, workspace=None):
    """Runs the stack in threshold mode on the calibration batch for every candidate theta.  x_calib is not
    modified.  Returns (theta, R_avg, {n: R_avg}); ctx is left in threshold mode at theta."""
    T = x_calib.shape[0]
    B = seq_offsets.numel() - 1
    lib = load_library()
    if workspace is None:
        workspace = alloc_workspace(stack.cfg, T, B, x_calib.device)
    scratch = torch.empty(lib.qtale_calibration_scratch_bytes(stack.n), dtype=torch.uint8, device=x_calib.device)
    x_work = torch.empty_like(x_calib)
    theta, ratio, table = C.c_float(), C.c_float(), (C.c_float * QTALE_THETA_GRID)()
    _check(lib.qtale_calibrate_threshold(ctx._h, C.byref(stack.cfg), stack._w, stack.n, _ptr(x_calib), _ptr(x_work), T,
                                         _ptr(seq_offsets), B, _ptr(positions), float(target_ratio), _ptr(scratch),
                                         _ptr(workspace), workspace.numel(), C.byref(theta), C.byref(ratio), table,
                                         _stream()), "qtale_calibrate_threshold")
    return _calibration_result(theta, ratio, table)


def qtale_router_mlp_scores(x, W1, b1, W2, b2):
    T, H = x.shape
    scores = torch.empty(T, dtype=torch.float32, device=x.device)
    _check(load_library().qtale_router_mlp_scores(_act_code(x.dtype), _ptr(x), T, H, _ptr(W1), _ptr(b1), _ptr(W2),
                                                  _ptr(b2), W1.shape[0], _ptr(scores), _stream()),
           "qtale_router_mlp_scores")
    return scores


class StackGraph:
    """HIP graph of one qtale_stack_forward call; holds references to every baked-in tensor."""

    def __init__(self, ctx, stack, x, seq_offsets, positions, sel_idx=None, sel_count=None, scores=None, workspace=None):
        T = x.shape[0]
        B = seq_offsets.numel() - 1
        if workspace is None:
            workspace = alloc_workspace(stack.cfg, T, B, x.device)
        self._keep = (ctx, stack, x, seq_offsets, positions, sel_idx, sel_count, scores, workspace)
        h = C.c_void_p()
        _check(load_library().qtale_graph_capture_stack(
            ctx._h, C.byref(stack.cfg), stack._w, stack.n, _ptr(x), T, _ptr(seq_offsets), B, _ptr(positions),
            stack._kv, _ptr(sel_idx), _ptr(sel_count), _ptr(scores), _ptr(workspace), workspace.numel(),
            C.byref(h)), "qtale_graph_capture_stack")
        self._h = h

    def launch(self):
        _check(load_library().qtale_graph_launch(self._h, _stream()), "qtale_graph_launch")

    def __del__(self):
        if getattr(self, "_h", None):
            load_library().qtale_graph_destroy(self._h)
            self._h = None


def qtale_router_select(ctx, x, router_w, router_b=0.0, seq_offsets=None):
    """Returns (scores fp32 [T], idx int32 [T], count int32 [1], cu_exec int32 [B+1] or None)."""
    T, H = x.shape
    dev = x.device
    scores = torch.empty(T, dtype=torch.float32, device=dev)
    idx = torch.full((T,), -1, dtype=torch.int32, device=dev)
    count = torch.zeros(1, dtype=torch.int32, device=dev)
    B = 0 if seq_offsets is None else seq_offsets.numel() - 1
    cu = None if seq_offsets is None else torch.empty(B + 1, dtype=torch.int32, device=dev)
    _check(load_library().qtale_router_select(ctx._h, _act_code(x.dtype), _ptr(x), T, H, _ptr(router_w),
                                              float(router_b), _ptr(seq_offsets), B, _ptr(scores), _ptr(idx),
                                              _ptr(count), _ptr(cu), _stream()), "qtale_router_select")
    return scores, idx, count, cu


def qtale_linear_w4a16(qlin, A, out=None):
    M = A.shape[0]
    assert A.dtype == torch.float16 and A.is_contiguous() and A.shape[1] == qlin.K
    if out is None:
        out = torch.empty((M, qlin.N), dtype=torch.float16, device=A.device)
    s = qlin.c_struct()
    _check(load_library().qtale_linear_w4a16(C.byref(s), qlin.bits, qlin.group, _ptr(A), M, _ptr(out), _stream()),
           "qtale_linear_w4a16")
    return out


def qtale_swiglu_w4a16(gate, up, A, out=None):
    M = A.shape[0]
    assert A.dtype == torch.float16 and A.is_contiguous() and A.shape[1] == gate.K
    if out is None:
        out = torch.empty((M, gate.N), dtype=torch.float16, device=A.device)
    g, u = gate.c_struct(), up.c_struct()
    _check(load_library().qtale_swiglu_w4a16(C.byref(g), C.byref(u), gate.bits, gate.group, _ptr(A), M, _ptr(out), _stream()),
           "qtale_swiglu_w4a16")
    return out


def qtale_profile_enable(ctx, on):
    _check(load_library().qtale_profile_enable(ctx._h, int(bool(on))), "qtale_profile_enable")


def qtale_profile_read(ctx):
    ms = (C.c_double * QTALE_PROF_CLASSES)()
    n = (C.c_int64 * QTALE_PROF_CLASSES)()
    _check(load_library().qtale_profile_read(ctx._h, ms, n), "qtale_profile_read")
    return {PROF_NAMES[i]: (ms[i], n[i]) for i in range(QTALE_PROF_CLASSES)}

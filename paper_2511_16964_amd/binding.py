"""ctypes binding of libfle (see include/fle.h).  Argument marshalling only: every
step of fused_linear_epilogue runs in the library's HIP kernels.  PyTorch provides
device memory and the stream, nothing else.  There is no fallback path: if the
library is missing or refuses a problem, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfle.so")

F32, BF16, F16, F8E4M3 = 0, 1, 2, 3
OP_KINDS = {"bias": 0, "scale": 1, "relu": 2, "gelu_erf": 3, "gelu_tanh": 4, "residual": 5,
            "layernorm": 6, "softmax": 7, "logsumexp": 8, "store": 9, "mxscale": 10, "layernorm_pre": 11}
MAX_OPS = 8
STATIC_SCRATCH_BYTES = 16 << 20
VARIANTS = {"auto": 0, "general": 1, "tiled": 2, "skinny": 3, "tiled256": 4, "tiled128": 5, "skinny128": 6, "skinny256": 7, "skinnyseq": 8, "thin": 9}
EXPORTS = ["fle_validate", "fle_workspace_size", "fle_run", "fle_run_static", "fle_run_with", "fle_workspace_size_with", "fle_status_string", "fle_last_error",
           "fle_last_plan", "fle_force_variant", "fle_force_split", "fle_version",
           "fle_validate_grouped", "fle_workspace_size_grouped", "fle_run_grouped",
           "fle_attention_validate", "fle_attention_run", "fle_attention_block_validate",
           "fle_attention_block_workspace_size", "fle_attention_block_run",
           "fle_chain_validate", "fle_chain_workspace_size", "fle_chain_run"]


class FleOp(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("alpha", ctypes.c_float), ("p0", ctypes.c_void_p),
                ("p1", ctypes.c_void_p), ("ld", ctypes.c_int64)]


class FleProblem(ctypes.Structure):
    _fields_ = [("M", ctypes.c_int64), ("N", ctypes.c_int64), ("K", ctypes.c_int64),
                ("dtype", ctypes.c_int32),
                ("x", ctypes.c_void_p), ("ldx", ctypes.c_int64),
                ("w", ctypes.c_void_p), ("ldw", ctypes.c_int64),
                ("b", ctypes.c_void_p),
                ("out", ctypes.c_void_p), ("ldo", ctypes.c_int64),
                ("ops", ctypes.POINTER(FleOp)), ("n_ops", ctypes.c_int32),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
                ("stream", ctypes.c_void_p)]


class FlePlanChoice(ctypes.Structure):
    _fields_ = [("variant", ctypes.c_int32), ("split", ctypes.c_int32)]


class FleGroups(ctypes.Structure):
    _fields_ = [("n_groups", ctypes.c_int32), ("row_offsets", ctypes.c_void_p),
                ("w_group_stride", ctypes.c_int64), ("b_group_stride", ctypes.c_int64)]


class FleAttention(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("causal", ctypes.c_int32),
                ("B", ctypes.c_int64), ("H", ctypes.c_int64), ("T", ctypes.c_int64), ("D", ctypes.c_int64),
                ("q", ctypes.c_void_p), ("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("ldq", ctypes.c_int64), ("ldk", ctypes.c_int64), ("ldv", ctypes.c_int64),
                ("o", ctypes.c_void_p), ("ldo", ctypes.c_int64), ("scale", ctypes.c_float),
                ("stream", ctypes.c_void_p), ("Tk", ctypes.c_int64),
                ("sbq", ctypes.c_int64), ("sbk", ctypes.c_int64), ("sbv", ctypes.c_int64), ("sbo", ctypes.c_int64)]


class FleAttentionBlock(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("causal", ctypes.c_int32),
                ("B", ctypes.c_int64), ("T", ctypes.c_int64), ("C", ctypes.c_int64), ("H", ctypes.c_int64),
                ("x", ctypes.c_void_p), ("w_qkv", ctypes.c_void_p), ("b_qkv", ctypes.c_void_p),
                ("w_o", ctypes.c_void_p), ("b_o", ctypes.c_void_p), ("residual", ctypes.c_void_p),
                ("out", ctypes.c_void_p), ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
                ("stream", ctypes.c_void_p)]


class FleChainLayer(ctypes.Structure):
    _fields_ = [("w", ctypes.c_void_p), ("b", ctypes.c_void_p), ("n", ctypes.c_int64), ("k", ctypes.c_int64),
                ("act", ctypes.c_int32)]


class FleChain(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("n_layers", ctypes.c_int32), ("layers", ctypes.POINTER(FleChainLayer)),
                ("x", ctypes.c_void_p), ("out", ctypes.c_void_p), ("workspace", ctypes.c_void_p),
                ("workspace_bytes", ctypes.c_size_t), ("stream", ctypes.c_void_p), ("w_dtype", ctypes.c_int32)]


class FleError(RuntimeError):
    def __init__(self, status: int, name: str, detail: str):
        super().__init__("libfle: %s (status %d): %s" % (name, status, detail))
        self.status = status


_lib = None


def lib():
    """Load libfle.so (built in-tree by ``__graft_entry__.build()``); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                LIB_PATH + " is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`")
        L = ctypes.CDLL(LIB_PATH)
        for name in ("fle_validate", "fle_run", "fle_run_static"):
            getattr(L, name).restype = ctypes.c_int
            getattr(L, name).argtypes = [ctypes.POINTER(FleProblem)]
        L.fle_workspace_size.restype = ctypes.c_int
        L.fle_workspace_size.argtypes = [ctypes.POINTER(FleProblem), ctypes.POINTER(ctypes.c_size_t)]
        L.fle_run_with.restype = ctypes.c_int
        L.fle_run_with.argtypes = [ctypes.POINTER(FleProblem), ctypes.POINTER(FlePlanChoice)]
        L.fle_workspace_size_with.restype = ctypes.c_int
        L.fle_workspace_size_with.argtypes = [ctypes.POINTER(FleProblem), ctypes.POINTER(FlePlanChoice), ctypes.POINTER(ctypes.c_size_t)]
        for name in ("fle_validate_grouped", "fle_run_grouped"):
            getattr(L, name).restype = ctypes.c_int
            getattr(L, name).argtypes = [ctypes.POINTER(FleProblem), ctypes.POINTER(FleGroups)]
        L.fle_workspace_size_grouped.restype = ctypes.c_int
        L.fle_workspace_size_grouped.argtypes = [ctypes.POINTER(FleProblem), ctypes.POINTER(FleGroups), ctypes.POINTER(ctypes.c_size_t)]
        for name in ("fle_attention_validate", "fle_attention_run"):
            getattr(L, name).restype = ctypes.c_int
            getattr(L, name).argtypes = [ctypes.POINTER(FleAttention)]
        for name in ("fle_attention_block_validate", "fle_attention_block_run"):
            getattr(L, name).restype = ctypes.c_int
            getattr(L, name).argtypes = [ctypes.POINTER(FleAttentionBlock)]
        L.fle_attention_block_workspace_size.restype = ctypes.c_int
        L.fle_attention_block_workspace_size.argtypes = [ctypes.POINTER(FleAttentionBlock), ctypes.POINTER(ctypes.c_size_t)]
        for name in ("fle_chain_validate", "fle_chain_run"):
            getattr(L, name).restype = ctypes.c_int
            getattr(L, name).argtypes = [ctypes.POINTER(FleChain)]
        L.fle_chain_workspace_size.restype = ctypes.c_int
        L.fle_chain_workspace_size.argtypes = [ctypes.POINTER(FleChain), ctypes.POINTER(ctypes.c_size_t)]
        L.fle_status_string.restype = ctypes.c_char_p
        L.fle_status_string.argtypes = [ctypes.c_int]
        L.fle_last_error.restype = ctypes.c_char_p
        L.fle_last_plan.restype = ctypes.c_int
        L.fle_last_plan.argtypes = [ctypes.c_char_p, ctypes.c_size_t]
        L.fle_force_variant.restype = None
        L.fle_force_variant.argtypes = [ctypes.c_int]
        L.fle_force_split.restype = None
        L.fle_force_split.argtypes = [ctypes.c_int]
        L.fle_version.restype = ctypes.c_int
        _lib = L
    return _lib


def _check(status: int):
    if status != 0:
        L = lib()
        raise FleError(status, L.fle_status_string(status).decode(), L.fle_last_error().decode())


def _dtype_code(dt: torch.dtype) -> int:
    if dt == torch.float32:
        return F32
    if dt == torch.bfloat16:
        return BF16
    if dt == torch.float16:
        return F16
    if dt == torch.float8_e4m3fn:
        return F8E4M3
    raise TypeError("fused_linear_epilogue supports float32, bfloat16, float16 and float8_e4m3fn (x and W only), got %s" % dt)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _raw_stream(device_index: int) -> int:
    try:
        return torch._C._cuda_getCurrentRawStream(device_index)   # several times cheaper than building a Stream object
    except AttributeError:
        return torch.cuda.current_stream(device_index).cuda_stream


class Call:
    """A marshalled fle_problem bound to its tensors: ``run()`` enqueues it on the
    current stream.  Keeps every tensor alive; reusable (the benchmark times ``run``)."""

    def __init__(self, x, w, b, epilogue, out=None, workspace=None, variant="auto", split=0, offsets=None, table=None):
        grouped = offsets is not None
        if x.dim() != 2 or w.dim() != (3 if grouped else 2) or x.shape[1] != w.shape[-1]:
            raise ValueError("x must be [M,K] and w [N,K] (grouped: [G,N,K])")
        if x.stride(1) != 1 and x.shape[1] > 1 or w.stride(-1) != 1 and w.shape[-1] > 1:
            raise ValueError("x and w must be row-major (unit stride along K)")
        self.variant = VARIANTS[variant]
        self.split = int(split)  # 0: automatic split of K; S >= 1 forces S workgroups per tile
        M, K = x.shape
        N = w.shape[-2]
        dt = x.dtype
        io = torch.bfloat16 if dt == torch.float8_e4m3fn else dt   # dtype of everything but x and W
        if w.dtype != dt:
            raise TypeError("x and w must share one dtype")
        tensors = [x, w, b]
        if b is not None and not grouped and (b.dim() != 1 or b.shape[0] != N or (N > 1 and b.stride(0) != 1)):
            raise ValueError("b must be a contiguous vector of N = %d elements" % N)
        if b is not None and grouped and b.dim() == 1 and (b.shape[0] != N or (N > 1 and b.stride(0) != 1)):
            raise ValueError("a shared b must be a contiguous vector of N = %d elements" % N)
        self._groups = None
        if grouped:
            G = w.shape[0]
            if offsets.dtype != torch.int64 or offsets.dim() != 1 or offsets.numel() != G + 1 or not offsets.is_contiguous() or offsets.device != x.device:
                raise ValueError("offsets must be a contiguous int64 tensor of G + 1 entries on x's device")
            if b is not None and b.dim() == 2 and (b.shape != (G, N) or (b.stride(1) != 1 and N > 1)):
                raise ValueError("grouped b must be [G,N] (or [N], shared by all groups)")
            g = FleGroups()
            g.n_groups, g.row_offsets = G, offsets.data_ptr()
            g.w_group_stride = w.stride(0) if G > 1 else 0
            g.b_group_stride = b.stride(0) if (b is not None and b.dim() == 2 and G > 1) else 0
            self._groups, self._gref = g, ctypes.byref(g)
            tensors.append(offsets)
            offsets = None
        if len(epilogue) > MAX_OPS:
            raise ValueError("at most %d epilogue ops" % MAX_OPS)
        ops = (FleOp * max(1, len(epilogue)))()
        for i, e in enumerate(epilogue):
            kind = OP_KINDS[e[0]]
            ops[i].kind = kind
            if e[0] == "scale":
                ops[i].alpha = float(e[1])
            elif e[0] == "residual":
                r = e[1]
                if r.shape != (M, N) or (r.stride(1) != 1 and N > 1):
                    raise ValueError("residual must be [M,N] with unit column stride")
                tensors.append(r)
                ops[i].p0 = r.data_ptr()
                ops[i].ld = r.stride(0) if M > 1 else max(N, r.stride(0))
            elif e[0] == "store":
                t = e[1]
                if t.shape != (M, N) or (t.stride(1) != 1 and N > 1):
                    raise ValueError("store target must be [M,N] with unit column stride")
                tensors.append(t)
                ops[i].p0 = t.data_ptr()
                ops[i].ld = t.stride(0) if M > 1 else max(N, t.stride(0))
            elif e[0] == "mxscale":   # block scales of fp8 operands: uint8 [M, K/32] and [N, K/32]
                sx, sw = e[1], e[2]
                for name, t, rows in (("x", sx, M), ("w", sw, N)):
                    if t.dtype != torch.uint8 or tuple(t.shape) != (rows, K // 32) or not t.is_contiguous() or t.device != x.device:
                        raise ValueError("block scales of %s must be a contiguous uint8 tensor [%d, K/32 = %d] on x's device" % (name, rows, K // 32))
                self._scales = (sx, sw)   # (kept alive; uint8, so outside the dtype check below)
                ops[i].p0, ops[i].p1 = sx.data_ptr(), sw.data_ptr()
            elif e[0] in ("layernorm", "layernorm_pre"):   # over the N outputs / over the K inputs of every row of x
                g, be, eps = e[1], e[2], e[3]
                n_aff = K if e[0] == "layernorm_pre" else N
                for name, t in (("gamma", g), ("beta", be)):
                    if t is not None and (t.dim() != 1 or t.shape[0] != n_aff or (n_aff > 1 and t.stride(0) != 1)):
                        raise ValueError("%s %s must be a contiguous vector of %d elements" % (e[0], name, n_aff))
                tensors += [g, be]
                ops[i].p0 = None if g is None else g.data_ptr()
                ops[i].p1 = None if be is None else be.data_ptr()
                ops[i].alpha = float(eps)
        for i, t in enumerate(tensors):
            if t is not None and t.dtype != torch.int64 and (t.dtype != (dt if i < 2 else io) or t.device != x.device):
                raise TypeError("all operands must be on x's device; b, residual and store operands, gamma and beta must have x's dtype (bfloat16 for fp8 problems)")
        lse = bool(epilogue) and epilogue[-1][0] == "logsumexp"
        if out is None:
            out = torch.empty((M,) if lse else (M, N), dtype=io, device=x.device)
        else:   # the kernels write through a raw pointer and a row stride: everything they assume is checked here
            if out.dtype != io or out.device != x.device:
                raise TypeError("out must have x's dtype (bfloat16 for fp8 problems) and device")
            if lse:
                if tuple(out.shape) != (M,) or (M > 1 and out.stride(0) != 1):
                    raise ValueError("out must be a contiguous vector of M = %d elements (the list ends in logsumexp)" % M)
            elif tuple(out.shape) != (M, N) or (N > 1 and out.stride(1) != 1) or (M > 1 and out.stride(0) < N):
                raise ValueError("out must be [M,N] = [%d,%d] with unit column stride and a row stride of at least N" % (M, N))
        self.out = out
        p = FleProblem()
        p.M, p.N, p.K, p.dtype = M, N, K, _dtype_code(dt)
        p.x, p.ldx = x.data_ptr(), (x.stride(0) if M > 1 else max(K, x.stride(0)))
        p.w, p.ldw = w.data_ptr(), (w.stride(-2) if N > 1 else max(K, w.stride(-2)))
        p.b = None if b is None else b.data_ptr()
        p.out = out.data_ptr()
        p.ldo = 0 if lse else (out.stride(0) if M > 1 else max(N, out.stride(0)))
        p.ops, p.n_ops = ops, len(epilogue)
        self._p, self._ops, self._tensors = p, ops, tensors
        self._dev = x.device.index   # (None: resolved when the call is enqueued)
        L = lib()
        if table is not None and not grouped and self.variant == 0 and self.split == 0:   # a tuned plan, where the table has one
            hit = table.lookup(p.dtype, M, N, K, epilogue)
            if hit is not None:
                self.variant, self.split = VARIANTS[hit[0]], int(hit[1])
        need = ctypes.c_size_t(0)
        if self._groups is None:   # plain problems: the plan choice travels with the call, the library keeps no state
            self._choice = FlePlanChoice(self.variant, self.split)
            _check(L.fle_workspace_size_with(ctypes.byref(p), ctypes.byref(self._choice), ctypes.byref(need)))
        else:
            L.fle_force_variant(self.variant)
            L.fle_force_split(self.split)
            try:
                _check(L.fle_workspace_size_grouped(ctypes.byref(p), self._gref, ctypes.byref(need)))
            finally:
                L.fle_force_variant(0)
                L.fle_force_split(0)
        if workspace is None and need.value:
            workspace = torch.empty(need.value, dtype=torch.uint8, device=x.device)
        self.workspace = workspace
        if workspace is not None:
            p.workspace, p.workspace_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
        self.workspace_needed = need.value
        self._pref = ctypes.byref(p)

    def run(self, stream=None):
        """Enqueue on ``stream`` (default: torch's current stream) and return ``out`` without synchronising."""
        L = lib()
        if self._dev is None:
            self._dev = torch.cuda.current_device()
        # the HIP stream handle: torch's current stream on the operands' device unless one is given
        self._p.stream = _raw_stream(self._dev) if stream is None else stream.cuda_stream
        if self.variant == 0 and self.split == 0:
            status = L.fle_run(self._pref) if self._groups is None else L.fle_run_grouped(self._pref, self._gref)
        elif self._groups is None:
            status = L.fle_run_with(self._pref, ctypes.byref(self._choice))
        else:   # (grouped problems have no per-call form: the thread's test knobs, set back at once)
            L.fle_force_variant(self.variant)
            L.fle_force_split(self.split)
            try:
                status = L.fle_run_grouped(self._pref, self._gref)
            finally:
                L.fle_force_variant(0)
                L.fle_force_split(0)
        if status != 0:
            _check(status)
        return self.out

    def run_static(self, stream=None):
        """As ``run`` through ``fle_run_static``: the library's static scratch array stands in for the
        workspace (plain problems up to FLE_STATIC_SCRATCH_BYTES of scratch; calls must not overlap on one GPU)."""
        if self._groups is not None:
            raise ValueError("fle_run_static takes plain problems only")
        L = lib()
        if self._dev is None:
            self._dev = torch.cuda.current_device()
        self._p.stream = _raw_stream(self._dev) if stream is None else stream.cuda_stream
        L.fle_force_variant(self.variant)
        L.fle_force_split(self.split)
        try:
            status = L.fle_run_static(self._pref)
        finally:
            L.fle_force_variant(0)
            L.fle_force_split(0)
        if status != 0:
            _check(status)
        return self.out

    def plan(self) -> str:
        buf = ctypes.create_string_buffer(256)
        lib().fle_last_plan(buf, 256)
        return buf.value.decode()


class TileTable:
    """Plans found by an offline tuning run (``python -m paper_2511_16964_amd.autotune``): for a class of problems
    (dtype, whether the list holds a row reduction, M, N, K each rounded to the nearest power of two) the kernel
    variant and split of K that measured fastest on the GPU the table was made on.  ``Call(..., table=t)`` uses
    the entry of its problem's class if there is one and the library's own cost model otherwise."""

    DEFAULT_PATH = os.path.join(_HERE, "tile_table.json")

    def __init__(self, entries=None, meta=None):
        self.entries, self.meta = dict(entries or {}), dict(meta or {})

    @staticmethod
    def bucket(v: int) -> int:
        v = max(1, int(v))
        b = v.bit_length() - 1
        return b + 1 if v * v > (1 << (2 * b + 1)) else b      # round log2(v) to the nearest integer

    @classmethod
    def key(cls, dtype_code, M, N, K, epilogue) -> str:
        row = int(any(e[0] in ("layernorm", "softmax", "logsumexp") for e in epilogue))
        return "%d:%d:%d:%d:%d" % (dtype_code, row, cls.bucket(M), cls.bucket(N), cls.bucket(K))

    def lookup(self, dtype_code, M, N, K, epilogue):
        e = self.entries.get(self.key(dtype_code, M, N, K, epilogue))
        return None if e is None else (e["variant"], e["split"])

    @classmethod
    def load(cls, path=None):
        import json
        d = json.load(open(path or cls.DEFAULT_PATH))
        return cls(d.get("entries"), {k: v for k, v in d.items() if k != "entries"})

    def save(self, path):
        import json
        with open(path, "w") as f:
            json.dump(dict(self.meta, entries=self.entries), f, indent=1, sort_keys=True)
            f.write("\n")


def grouped_fused_linear_epilogue(x, w, b, offsets, epilogue, out=None, workspace=None, variant="auto"):
    """Grouped form: rows offsets[g] .. offsets[g+1]-1 of x go through w[g] (and b[g]), one launch.

    x [M,K]; w [G,N,K]; b [G,N], [N] (shared) or None; offsets: int64 tensor [G+1] on the device,
    non-decreasing from 0 to M (read by the kernel only, no host synchronisation); epilogue as in
    ``fused_linear_epilogue`` with residual operands [M,N].  Returns [M,N] (or [M] for logsumexp).
    """
    if not x.is_cuda:
        raise RuntimeError("grouped_fused_linear_epilogue runs on the GPU only; there is no CPU path")
    return Call(x, w, b, epilogue, out=out, workspace=workspace, variant=variant, offsets=offsets).run()


def fused_linear_epilogue(x, w, b, epilogue, out=None, workspace=None, variant="auto", split=0, table=None):
    """out = epilogue(x @ w.T) in one fused library call.

    x [M,K], w [N,K], b [N] or None: CUDA(HIP) tensors of one dtype (float32, bfloat16 or float16), or x and w in
    float8_e4m3fn with b and everything else in bfloat16.
    epilogue: ordered list of ("bias",) ("scale", a) ("relu",) ("gelu_erf",) ("gelu_tanh",)
    ("residual", r[M,N]) ("layernorm", gamma|None, beta|None, eps) ("softmax",) ("logsumexp",), at most two of the
    last three;
    ("store", t[M,N]): t receives a copy of the values at that point of the list (before the first row op only);
    as the first entry only: ("mxscale", sx[M,K/32], sw[N,K/32]): the fp8 operands are block-scaled, one uint8 E8M0
    scale per 32 consecutive k (K a multiple of 128); ("layernorm_pre", gamma[K]|None, beta[K]|None, eps): LayerNorm
    over K of every row of x in front of the multiplication.
    table: a ``TileTable`` of tuned plans (default: the library's cost model decides).
    Returns a tensor of x's dtype (bfloat16 for fp8 operands): [M,N], or [M] when the list ends in logsumexp.
    """
    if not x.is_cuda:
        raise RuntimeError("fused_linear_epilogue runs on the GPU only; there is no CPU path")
    return Call(x, w, b, epilogue, out=out, workspace=workspace, variant=variant, split=split, table=table).run()


def _strides(t):
    """(token stride, sequence stride) of a [B,T,H,D] view whose (h, d) axes are packed."""
    B, T, H, D = t.shape
    if (D > 1 and t.stride(3) != 1) or (H > 1 and t.stride(2) != D):
        raise ValueError("q, k, v, o must be [B,T,H,D] views with unit stride along D and stride D along H")
    return t.stride(1) if T > 1 else H * D, t.stride(0) if B > 1 else 0


class AttentionCall:
    """A marshalled fle_attention bound to its tensors; ``run()`` enqueues it on the current stream."""

    def __init__(self, q, k, v, causal, scale=None, out=None):
        if q.dim() != 4 or k.dim() != 4 or k.shape != v.shape or q.shape[0] != k.shape[0] or q.shape[2:] != k.shape[2:]:
            raise ValueError("q must be [B,T,H,D] and k, v [B,Tk,H,D]")
        if not (q.is_cuda and k.is_cuda and v.is_cuda):
            raise RuntimeError("attention runs on the GPU only; there is no CPU path")
        if k.dtype != q.dtype or v.dtype != q.dtype:
            raise TypeError("q, k, v must share one dtype")
        B, T, H, D = q.shape
        if out is None:
            out = torch.empty((B, T, H, D), device=q.device, dtype=q.dtype)
        p = FleAttention()
        p.dtype, p.causal = _dtype_code(q.dtype), int(causal)
        p.B, p.H, p.T, p.D, p.Tk = B, H, T, D, k.shape[1]
        p.q, p.k, p.v, p.o = q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr()
        (p.ldq, p.sbq), (p.ldk, p.sbk), (p.ldv, p.sbv), (p.ldo, p.sbo) = (_strides(t) for t in (q, k, v, out))
        p.scale = 0.0 if scale is None else float(scale)
        self._keep = (q, k, v)
        self.out, self._p, self._pref, self._dev = out, p, ctypes.byref(p), q.device.index
        _check(lib().fle_attention_validate(self._pref))

    def run(self, stream=None):
        self._p.stream = _raw_stream(self._dev) if stream is None else stream.cuda_stream
        status = lib().fle_attention_run(self._pref)
        if status != 0:
            _check(status)
        return self.out


def attention(q, k, v, causal, scale=None, out=None):
    """Scaled dot-product attention over [B,T,H,D] queries and [B,Tk,H,D] keys / values (bf16 or fp16, D = 32 .. 256).

    q, k, v may be views into one fused projection output (``qkv.view(B,T,3,H,D)[:, :, i]``) or views of
    sequence-first tensors (``x.view(T,B,H,D).transpose(0,1)``): any token and sequence strides; nothing is
    copied or transposed.  causal: False / 0 no mask, True / 1 query t sees keys 0..t, G > 1 the same over
    groups of G tokens (keys below (t // G + 1) * G).  scale defaults to 1/sqrt(D).
    """
    return AttentionCall(q, k, v, causal, scale, out).run()


class TransformerLayerCall:
    """One pre-norm transformer layer as five fused calls bound to their tensors (no arithmetic here: every
    step is a library call; the store op hands each residual sum over together with its LayerNorm):
        qkv = n W_qkv^T + b_qkv;  o = attention(qkv, in place);
        h, m = store / LayerNorm_mid of (o W_o^T + b_o + x);  u = gelu_erf(m W1^T + b1);
        x', n' = store / LayerNorm_out of (u W2^T + b2 + h).
    ``run()`` returns (x', n'), the residual stream and its normalised form for the next layer."""

    def __init__(self, x, n, w_qkv, b_qkv, w_o, b_o, heads, causal, ln_mid, w1, b1, w2, b2, ln_out):
        if x.dim() != 3 or n.shape != x.shape:
            raise ValueError("x and n must be [B,T,C]")
        if not x.is_cuda:
            raise RuntimeError("transformer_layer runs on the GPU only; there is no CPU path")
        B, T, C = x.shape
        if C % heads:
            raise ValueError("C must be a multiple of heads")
        D, M, Fh = C // heads, B * T, w1.shape[0]
        new = lambda *shape: torch.empty(shape, device=x.device, dtype=x.dtype)
        x2, n2 = x.reshape(M, C), n.reshape(M, C)
        self.qkv, self.o, self.h, self.m, self.u = new(M, 3 * C), new(M, C), new(M, C), new(M, C), new(M, Fh)
        self.x_out, self.n_out = new(B, T, C), new(B, T, C)
        q5 = self.qkv.view(B, T, 3, heads, D)
        self.calls = [
            Call(n2, w_qkv, b_qkv, [("bias",)] if b_qkv is not None else [], out=self.qkv),
            AttentionCall(q5[:, :, 0], q5[:, :, 1], q5[:, :, 2], causal, out=self.o.view(B, T, heads, D)),
            Call(self.o, w_o, b_o, ([("bias",)] if b_o is not None else []) + [("residual", x2), ("store", self.h), ("layernorm", ln_mid[0], ln_mid[1], ln_mid[2])], out=self.m),
            Call(self.m, w1, b1, [("bias",), ("gelu_erf",)], out=self.u),
            Call(self.u, w2, b2, [("bias",), ("residual", self.h), ("store", self.x_out.view(M, C)), ("layernorm", ln_out[0], ln_out[1], ln_out[2])], out=self.n_out.view(M, C)),
        ]
        self.out = self.x_out

    def run(self, stream=None):
        for c in self.calls:
            c.run(stream)
        return self.x_out, self.n_out

    def plan(self) -> str:
        return "transformer layer: five fused calls (qkv projection, attention, output projection + residual + store + LayerNorm, perceptron up + GELU, perceptron down + residual + store + LayerNorm)"


def transformer_layer(x, n, w_qkv, b_qkv, w_o, b_o, heads, causal, ln_mid, w1, b1, w2, b2, ln_out):
    """One pre-norm transformer layer from its normalised input on; see ``TransformerLayerCall``.
    x, n [B,T,C]; ln_mid, ln_out = (gamma, beta, eps).  Returns (x', n')."""
    return TransformerLayerCall(x, n, w_qkv, b_qkv, w_o, b_o, heads, causal, ln_mid, w1, b1, w2, b2, ln_out).run()


class AttentionBlockCall:
    """A marshalled fle_attention_block (QKV projection, attention, output projection) bound to its tensors."""

    def __init__(self, x, w_qkv, b_qkv, w_o, b_o, heads, causal, residual=None, out=None, workspace=None):
        if x.dim() != 3:
            raise ValueError("x must be [B,T,C]")
        if not x.is_cuda:
            raise RuntimeError("attention_block runs on the GPU only; there is no CPU path")
        B, T, C = x.shape
        for name, t, shape in (("w_qkv", w_qkv, (3 * C, C)), ("b_qkv", b_qkv, (3 * C,)), ("w_o", w_o, (C, C)),
                               ("b_o", b_o, (C,)), ("residual", residual, (B, T, C)), ("out", out, (B, T, C))):
            if t is None:
                continue
            if tuple(t.shape) != shape or not t.is_contiguous() or t.dtype != x.dtype or t.device != x.device:
                raise ValueError("%s must be a contiguous %s tensor of x's dtype and device" % (name, list(shape)))
        if not x.is_contiguous():
            raise ValueError("x must be contiguous")
        if out is None:
            out = torch.empty_like(x)
        p = FleAttentionBlock()
        p.dtype, p.causal = _dtype_code(x.dtype), int(causal)
        p.B, p.T, p.C, p.H = B, T, C, int(heads)
        p.x, p.w_qkv, p.w_o, p.out = x.data_ptr(), w_qkv.data_ptr(), w_o.data_ptr(), out.data_ptr()
        p.b_qkv = None if b_qkv is None else b_qkv.data_ptr()
        p.b_o = None if b_o is None else b_o.data_ptr()
        p.residual = None if residual is None else residual.data_ptr()
        need = ctypes.c_size_t(0)
        _check(lib().fle_attention_block_workspace_size(ctypes.byref(p), ctypes.byref(need)))
        if workspace is None:
            workspace = torch.empty(max(need.value, 256), device=x.device, dtype=torch.uint8)
        p.workspace, p.workspace_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
        self.workspace_needed = need.value
        self._keep = (x, w_qkv, b_qkv, w_o, b_o, residual, workspace)
        self.out, self._p, self._pref, self._dev = out, p, ctypes.byref(p), x.device.index

    def run(self, stream=None):
        self._p.stream = _raw_stream(self._dev) if stream is None else stream.cuda_stream
        status = lib().fle_attention_block_run(self._pref)
        if status != 0:
            _check(status)
        return self.out

    def plan(self) -> str:
        """Plan text of the block's output projection (the last stage enqueued)."""
        buf = ctypes.create_string_buffer(256)
        lib().fle_last_plan(buf, 256)
        return buf.value.decode()


def attention_block(x, w_qkv, b_qkv, w_o, b_o, heads, causal, residual=None, out=None, workspace=None):
    """out = (attention over `heads` heads of (x w_qkv^T + b_qkv)) w_o^T + b_o (+ residual), three fused launches.

    x [B,T,C]; w_qkv [3C,C] with output columns q | k | v; C / heads must be 64 or 128; bf16 or fp16.
    """
    return AttentionBlockCall(x, w_qkv, b_qkv, w_o, b_o, heads, causal, residual, out, workspace).run()


_ACTS = {None: -1, "none": -1, "relu": 2, "gelu_erf": 3, "gelu_tanh": 4}


class ChainCall:
    """A marshalled fle_chain (a perceptron at batch 1 in one persistent launch) bound to its tensors."""

    def __init__(self, x, weights, biases, activations, out=None, workspace=None):
        if not x.is_cuda:
            raise RuntimeError("mlp_chain runs on the GPU only; there is no CPU path")
        if x.numel() != weights[0].shape[1] or (x.dim() == 2 and x.shape[0] != 1) or x.dim() > 2:
            raise ValueError("x must be one row of weights[0].shape[1] elements")
        n = len(weights)
        if len(biases) != n or len(activations) != n:
            raise ValueError("one bias (or None) and one activation per layer")
        arr = (FleChainLayer * n)()
        for i, (w, b, act) in enumerate(zip(weights, biases, activations)):
            if w.dtype != weights[0].dtype or (b is not None and b.dtype != x.dtype):
                raise ValueError("all weights share one dtype; biases have x's dtype")
            for t in (w, b):
                if t is not None and (t.device != x.device or not t.is_contiguous()):
                    raise ValueError("weights and biases must be contiguous tensors on x's device")
            if w.dim() != 2 or (b is not None and tuple(b.shape) != (w.shape[0],)):
                raise ValueError("layer %d: w must be [n,k] and b [n]" % i)
            arr[i].w, arr[i].b = w.data_ptr(), (None if b is None else b.data_ptr())
            arr[i].n, arr[i].k, arr[i].act = w.shape[0], w.shape[1], _ACTS[act]
        if out is None:
            out = torch.empty((1, weights[-1].shape[0]) if x.dim() == 2 else (weights[-1].shape[0],), device=x.device, dtype=x.dtype)
        p = FleChain()
        p.dtype, p.n_layers, p.layers = _dtype_code(x.dtype), n, arr
        p.w_dtype = _dtype_code(weights[0].dtype)
        p.x, p.out = x.data_ptr(), out.data_ptr()
        need = ctypes.c_size_t(0)
        _check(lib().fle_chain_workspace_size(ctypes.byref(p), ctypes.byref(need)))
        if workspace is None:
            workspace = torch.zeros(max(need.value, 256), device=x.device, dtype=torch.uint8)   # the barrier words start at zero
        p.workspace, p.workspace_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
        self.workspace_needed = need.value
        self.workspace = workspace
        self._keep = (x, list(weights), list(biases), workspace, arr)
        self.out, self._p, self._pref, self._dev = out, p, ctypes.byref(p), x.device.index

    def run(self, stream=None):
        self._p.stream = _raw_stream(self._dev) if stream is None else stream.cuda_stream
        status = lib().fle_chain_run(self._pref)
        if status != 0:
            _check(status)
        return self.out

    def barrier_error(self) -> bool:
        """True if a barrier wait ran out in some call since the workspace was zeroed (synchronises)."""
        return bool(self.workspace[256:260].view(torch.int32).item())

    def run_checked(self, stream=None):
        """``run``, then wait for the result and raise if a barrier wait was given up (the workgroups were not all
        resident: out holds NaN in the shares of those that gave up).  The barrier state is zeroed again so that
        the workspace can be reused."""
        out = self.run(stream)
        torch.cuda.synchronize(self._dev)
        if self.barrier_error():
            self.workspace[:2560].zero_()
            raise RuntimeError("mlp_chain: a grid barrier wait was given up; the result is not valid")
        return out

    def plan(self) -> str:
        return "mlp_chain: %d layers in one launch" % self._p.n_layers


def mlp_chain(x, weights, biases, activations, out=None, workspace=None):
    """out = act_L(W_L ... act_1(W_1 x + b_1) ... + b_L) for one input row, every layer in one persistent launch.

    x: [k] or [1,k]; weights[i]: [n_i, k_i] with k_{i+1} = n_i; biases[i]: [n_i] or None;
    activations[i]: None, "relu", "gelu_erf" or "gelu_tanh".  float32, bfloat16 or float16; with a float32 x the
    weights may be bfloat16 or float16 (biases, activations and the result stay float32).
    """
    return ChainCall(x, weights, biases, activations, out, workspace).run()


def mlp_chain_checked(x, weights, biases, activations, out=None, workspace=None):
    """As ``mlp_chain``, synchronising and raising if a grid barrier wait was given up."""
    return ChainCall(x, weights, biases, activations, out, workspace).run_checked()

"""Host-side tests of the C-ABI library that need no GPU: the library loads, exports
every function include/fle.h declares, and rejects invalid problems before any HIP call."""
import ctypes
import os
import re

import pytest

from paper_2511_16964_amd import binding
from paper_2511_16964_amd.binding import FleOp, FleProblem

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, E_NULL, E_SHAPE, E_ALIGN, E_OP, E_UNSUP, E_WS, E_HIP = range(8)


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return binding.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "fle.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fle_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(L):
    names = declared_functions()
    assert sorted(names) == sorted(binding.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_version_and_status_strings(L):
    assert L.fle_version() >= 100
    seen = {L.fle_status_string(i) for i in range(8)}
    assert len(seen) == 8 and all(s for s in seen)


G = 1 << 32   # fake buffers sit 4 GiB apart so that large shapes never overlap


def problem(M=64, N=64, K=64, dtype=binding.BF16, ops=(), b=5 * G, base=G):
    """A problem with fake (never dereferenced) device addresses; validation is host-only."""
    p = FleProblem()
    p.M, p.N, p.K, p.dtype = M, N, K, dtype
    p.x, p.ldx = base, K
    p.w, p.ldw = base + G, K
    p.b = b
    p.out, p.ldo = base + 2 * G, N
    arr = (FleOp * max(1, len(ops)))()
    for i, (kind, alpha, p0, p1, ld) in enumerate(ops):
        arr[i].kind, arr[i].alpha, arr[i].p0, arr[i].p1, arr[i].ld = kind, alpha, p0, p1, ld
    p.ops, p.n_ops = arr, len(ops)
    p._keep = arr
    return p


def op(kind, alpha=0.0, p0=None, p1=None, ld=0):
    return (binding.OP_KINDS[kind], alpha, p0, p1, ld)


def validate(L, p):
    return L.fle_validate(ctypes.byref(p))


def test_accepts_all_benchmark_chains(L):
    res = 6 * G
    chains = [
        [op("bias"), op("gelu_erf")],
        [op("bias"), op("relu"), op("scale", 0.5), op("residual", p0=res, ld=64)],
        [op("bias"), op("gelu_tanh"), op("layernorm", 1e-5, 7 * G, 8 * G)],
        [op("softmax")],
        [op("bias"), op("residual", p0=res, ld=64), op("layernorm", 1e-5, 7 * G, 8 * G)],
        [op("scale", 2.0), op("logsumexp")],
        [op("layernorm", 1e-5), op("gelu_erf"), op("residual", p0=res, ld=64)],
        [],
    ]
    for ch in chains:
        for dt in (binding.F32, binding.BF16):
            assert validate(L, problem(ops=ch, dtype=dt)) == OK, L.fle_last_error()


def test_null_pointers(L):
    assert L.fle_validate(None) == E_NULL
    p = problem(); p.x = None
    assert validate(L, p) == E_NULL
    p = problem(); p.out = None
    assert validate(L, p) == E_NULL
    assert validate(L, problem(ops=[op("bias")], b=None)) == E_NULL
    assert b"bias" in L.fle_last_error()
    assert validate(L, problem(ops=[op("residual", p0=None, ld=64)])) == E_NULL
    p = problem(); p.n_ops = 2; p.ops = None
    assert validate(L, p) == E_NULL
    assert L.fle_workspace_size(ctypes.byref(problem()), None) == E_NULL


def test_shapes(L):
    assert validate(L, problem(M=-1)) == E_SHAPE
    assert validate(L, problem(N=0)) == E_SHAPE
    assert validate(L, problem(K=-3)) == E_SHAPE
    p = problem(); p.ldx = 63
    assert validate(L, p) == E_SHAPE
    p = problem(); p.ldw = 8
    assert validate(L, p) == E_SHAPE
    p = problem(); p.ldo = 63
    assert validate(L, p) == E_SHAPE
    assert validate(L, problem(ops=[op("residual", p0=6 * G, ld=63)])) == E_SHAPE
    # M == 0 is a valid no-op, even with NULL buffers
    p = problem(M=0); p.x = None; p.out = None
    assert validate(L, p) == OK
    assert L.fle_run(ctypes.byref(p)) == OK          # returns before any HIP call


def test_ops_and_grammar(L):
    assert validate(L, problem(ops=[(42, 0.0, None, None, 0)])) == E_OP
    assert validate(L, problem(ops=[op("scale", float("nan"))])) == E_OP
    assert validate(L, problem(ops=[op("layernorm", -1.0)])) == E_OP
    p = problem(); p.n_ops = 9
    assert validate(L, p) == E_OP
    p = problem(); p.dtype = 7
    assert validate(L, p) == E_OP
    # two row reductions in one list are accepted (a third one is not): fp32 [M,N] more workspace for the values between them
    need = ctypes.c_size_t(0)
    one = problem(M=64, N=64, K=64, ops=[op("softmax")])
    assert L.fle_workspace_size(ctypes.byref(one), ctypes.byref(need)) == OK
    base = need.value
    two = problem(M=64, N=64, K=64, ops=[op("softmax"), op("relu"), op("layernorm", 1e-5), op("scale", 2.0)])
    assert L.fle_workspace_size(ctypes.byref(two), ctypes.byref(need)) == OK and need.value == base + 64 * 64 * 4
    assert validate(L, problem(ops=[op("layernorm", 1e-5), op("bias"), op("logsumexp")])) == OK
    assert validate(L, problem(ops=[op("softmax"), op("layernorm", 1e-5), op("softmax")])) == E_UNSUP
    assert validate(L, problem(ops=[op("layernorm", 1e-5), op("logsumexp"), op("relu")])) == E_UNSUP
    assert validate(L, problem(ops=[op("logsumexp"), op("relu")])) == E_UNSUP
    assert b"logsumexp" in L.fle_last_error()


def test_alignment_and_aliasing(L):
    p = problem(); p.x = G + 1
    assert validate(L, p) == E_ALIGN                  # not even element-aligned
    p = problem(); p.out = p.x
    assert validate(L, p) == E_UNSUP                  # out overlaps x
    out = problem().out
    assert validate(L, problem(ops=[op("residual", p0=out, ld=64)])) == OK        # exact alias allowed
    assert validate(L, problem(ops=[op("residual", p0=out + 2, ld=64)])) == E_UNSUP  # partial overlap


def test_workspace_sizes_and_plan_text(L):
    need = ctypes.c_size_t(99)
    assert L.fle_workspace_size(ctypes.byref(problem(ops=[op("bias"), op("relu")])), ctypes.byref(need)) == OK
    assert need.value == 0
    # LayerNorm, bf16, staged in out: only partials [M][np][2] floats
    p = problem(M=512, N=1024, K=256, ops=[op("layernorm", 1e-5)])
    assert L.fle_workspace_size(ctypes.byref(p), ctypes.byref(need)) == OK
    buf = ctypes.create_string_buffer(256)
    L.fle_last_plan(buf, 256)
    text = buf.value.decode()
    assert "tiled_bf16_mfma" in text and "staging=out" in text
    np_ = int(re.search(r"np=(\d+)", text).group(1))
    assert need.value == 512 * np_ * 8
    # bf16 softmax also stages in out (relative to the partial maxima): partials only ...
    p = problem(M=512, N=1024, K=256, ops=[op("softmax")])
    assert L.fle_workspace_size(ctypes.byref(p), ctypes.byref(need)) == OK
    L.fle_last_plan(buf, 256)
    assert "staging=out" in buf.value.decode() and need.value < 512 * 1024
    # ... unless a trailing residual aliases out: then the values are staged as fp32 in the workspace
    p = problem(M=512, N=1024, K=256, ops=[op("softmax"), op("residual", p0=G + 2 * G, ld=1024)])
    assert L.fle_workspace_size(ctypes.byref(p), ctypes.byref(need)) == OK
    L.fle_last_plan(buf, 256)
    assert "staging=workspace_f32" in buf.value.decode() and need.value >= 512 * 1024 * 4
    # run without workspace fails before any HIP call
    assert L.fle_run(ctypes.byref(p)) == E_WS
    p.workspace, p.workspace_bytes = 9 * G, 16
    assert L.fle_run(ctypes.byref(p)) == E_WS


def test_variant_selection(L):
    def plan_of(p):
        need = ctypes.c_size_t(0)
        assert L.fle_workspace_size(ctypes.byref(p), ctypes.byref(need)) == OK
        buf = ctypes.create_string_buffer(256)
        L.fle_last_plan(buf, 256)
        return buf.value.decode()
    assert "tile=256x256" in plan_of(problem(M=4096, N=4096, K=4096))
    assert "tile=128x128" in plan_of(problem(M=1024, N=1024, K=512))
    assert "general" in plan_of(problem(M=256, N=256, K=256)) and "tile=16x16" in plan_of(problem(M=256, N=256, K=256))   # tiny: many small tiles
    assert "tiled" in plan_of(problem(M=128, N=256, K=4096))                                                              # few tiles, long K: split K
    assert "general" in plan_of(problem(M=64, N=256, K=256, dtype=binding.F32))   # tiny: launch-bound, many small tiles win
    assert "tiled_f32_mfma tile=128x128x32" in plan_of(problem(M=2048, N=2048, K=2048, dtype=binding.F32))
    assert "tiled_f32_mfma" in plan_of(problem(M=4096, N=4096, K=4096, dtype=binding.F32))
    assert "general" in plan_of(problem(M=2048, N=2048, K=2046, dtype=binding.F32))
    assert "general" in plan_of(problem(M=512, N=512, K=500))      # K not a multiple of 64
    p = problem(M=512, N=512, K=512); p.x = p.x + 2                # misaligned x
    assert "general" in plan_of(p)
    L.fle_force_variant(2)
    try:
        assert validate(L, problem(M=64, N=256, K=254, dtype=binding.F32)) == E_UNSUP   # rows are not whole 16-byte chunks
        assert validate(L, problem(M=64, N=256, K=256, dtype=binding.F32)) == OK
    finally:
        L.fle_force_variant(0)


def test_thin_kernel_selection(L):
    def plan_of(p):
        need = ctypes.c_size_t(0)
        assert L.fle_workspace_size(ctypes.byref(p), ctypes.byref(need)) == OK
        buf = ctypes.create_string_buffer(256)
        L.fle_last_plan(buf, 256)
        text = buf.value.decode()
        assert need.value == 0 or "thin" not in text   # the thin kernels never need a workspace without a row op
        return text
    F32, BF16, F16 = binding.F32, binding.BF16, binding.F16
    # a perceptron layer at batch 1: the dot-product form (8-row plan), one launch, no split of K
    for dt in (F32, BF16, F16):
        text = plan_of(problem(M=1, N=4096, K=4096, dtype=dt))
        assert "thin_" in text and "tile=8x16" in text and "split_k=1" in text, text
    assert "thin_f32_dot tile=8x16" in plan_of(problem(M=8, N=1024, K=32768, dtype=F32))     # fp32: up to 8 rows, any size
    assert "thin_f32_dot tile=8x16" in plan_of(problem(M=1, N=32768, K=8192, dtype=F32))
    assert "thin" not in plan_of(problem(M=9, N=4096, K=4096, dtype=F32))                      # more rows in fp32: general / tiled
    assert "thin" not in plan_of(problem(M=1, N=256, K=256, dtype=F32))                        # tiny: the general kernel
    assert "thin_bf16_dot tile=8x16" in plan_of(problem(M=4, N=2048, K=2048))
    assert "thin_bf16_dot tile=8x16x1 " in plan_of(problem(M=1, N=32768, K=8192))              # one row, many long rows of W: one W row per wave
    assert "thin_bf16_dot tile=8x16x4 " in plan_of(problem(M=1, N=2048, K=2048))
    assert "skinny" in plan_of(problem(M=2, N=32768, K=8192))                                  # more rows on large weights in 2 bytes: the skinny kernel
    assert "skinny" in plan_of(problem(M=4, N=32768, K=1024))                                  # short rows
    # 5 .. 32 rows of a 2-byte dtype on mid-sized weights: the MFMA form, 16- or 32-row plan
    assert "thin_bf16_mfma tile=16x16x32" in plan_of(problem(M=16, N=2048, K=2048))
    assert "thin_f16_mfma tile=32x16x32" in plan_of(problem(M=32, N=1024, K=2048, dtype=F16))
    assert "skinny" in plan_of(problem(M=16, N=4096, K=4096))
    assert "thin" not in plan_of(problem(M=33, N=2048, K=2048))
    # x or W rows that are not whole 16-byte chunks: not eligible
    assert "general" in plan_of(problem(M=1, N=4096, K=4092, dtype=BF16))
    L.fle_force_variant(9)
    try:
        assert validate(L, problem(M=32, N=64, K=64)) == OK
        assert validate(L, problem(M=33, N=64, K=64)) == E_UNSUP
        assert validate(L, problem(M=4, N=64, K=62)) == E_UNSUP
        L.fle_force_split(2)
        assert validate(L, problem(M=4, N=64, K=64)) == E_UNSUP
    finally:
        L.fle_force_variant(0)
        L.fle_force_split(0)


def test_fp32_skinny_selection(L):
    def plan_of(p):
        need = ctypes.c_size_t(0)
        assert L.fle_workspace_size(ctypes.byref(p), ctypes.byref(need)) == OK
        buf = ctypes.create_string_buffer(256)
        L.fle_last_plan(buf, 256)
        return buf.value.decode()
    F32 = binding.F32
    assert "skinny_f32_mfma tile=32x128x128" in plan_of(problem(M=16, N=8192, K=8192, dtype=F32))   # 512 bytes of a row per K step
    assert "skinny_f32_mfma tile=32x128x128" in plan_of(problem(M=48, N=4096, K=4096, dtype=F32))   # two row blocks of 32
    assert "skinny_f32_mfma tile=32x128x64" in plan_of(problem(M=32, N=8192, K=8256, dtype=F32))    # K not a multiple of 128 elements
    assert "skinny" not in plan_of(problem(M=16, N=4096, K=4096, dtype=F32))                          # the general kernel is as fast there
    assert "skinny" not in plan_of(problem(M=65, N=8192, K=8192, dtype=F32))
    assert "thin_f32_dot" in plan_of(problem(M=8, N=8192, K=8192, dtype=F32))                        # up to 8 rows: dot products
    L.fle_force_variant(7)
    try:
        assert "skinny_f32_mfma tile=32x128x128" in plan_of(problem(M=100, N=260, K=128, dtype=F32))
        assert validate(L, problem(M=32, N=256, K=48, dtype=F32)) == E_UNSUP                          # a K step is at least 128 bytes
    finally:
        L.fle_force_variant(0)


def test_split_k_planning(L):
    def plan_of(p):
        need = ctypes.c_size_t(0)
        assert L.fle_workspace_size(ctypes.byref(p), ctypes.byref(need)) == OK
        buf = ctypes.create_string_buffer(256)
        L.fle_last_plan(buf, 256)
        return buf.value.decode(), need.value
    split = lambda text: int(re.search(r"split_k=(\d+)", text).group(1))
    # the large benchmark shapes fill the chip by themselves: 256 tile, no split, no workspace
    for M, N, K in ((4096, 4096, 4096), (8192, 4096, 4096), (16384, 16384, 4096), (16384, 4096, 16384)):
        text, need = plan_of(problem(M=M, N=N, K=K))
        assert "tile=256x256" in text and split(text) == 1 and need == 0, text
    # one tile row and a long K: split, and the slabs are counted in the workspace
    text, need = plan_of(problem(M=192, N=4096, K=4096))
    s = split(text)
    assert "tiled" in text and s > 1 and need == s * 192 * 4096 * 4, text
    # 65 .. 128 rows of a 2-byte dtype: the streaming kernel, 64 rows at once on a 128-wide K step (fp32: still tiled)
    text, need = plan_of(problem(M=128, N=4096, K=4096))
    s = split(text)
    assert "skinny" in text and "tile=64x128x128" in text and s > 1 and need == s * 128 * 4096 * 4, text
    text, need = plan_of(problem(M=128, N=4096, K=4096, dtype=binding.F32))
    assert "tiled" in text, text
    text, need = plan_of(problem(M=16, N=4096, K=4096))
    assert "skinny" in text and split(text) > 1 and need == split(text) * 16 * 4096 * 4, text
    # a long K and too few 256 tiles for the chip: the 256 tile with K split until the workgroups fill it (measured ahead of the 128 tile)
    for M, sp in ((768, 4), (1024, 4), (1536, 2), (2048, 2)):
        text, need = plan_of(problem(M=M, N=4096, K=16384))
        assert "tile=256x256" in text and split(text) == sp and need == sp * M * 4096 * 4, text
    # many small tiles and a short K: the 128 tile without a split
    text, need = plan_of(problem(M=512, N=16384, K=1024))
    assert "tile=128x128" in text and split(text) == 1 and need == 0, text
    # the slabs come after the row-op partials
    text, need = plan_of(problem(M=128, N=4096, K=4096, ops=[op("softmax")]))
    s, np_ = split(text), int(re.search(r"np=(\d+)", text).group(1))
    assert s > 1 and np_ == 4096 // 256 and need == 128 * np_ * 8 + s * 128 * 4096 * 4, text
    L.fle_force_split(3)
    try:
        text, need = plan_of(problem(M=300, N=520, K=576))
        assert split(text) == 3 and need == -(-3 * 300 * 520 * 4 // 256) * 256, text
        text, need = plan_of(problem(M=300, N=520, K=72))        # two K steps only
        assert split(text) == 2, text
        text, need = plan_of(problem(M=64, N=256, K=254, dtype=binding.F32))   # rows are not whole chunks: general kernel, no split
        assert "general" in text and split(text) == 1 and need == 0, text
    finally:
        L.fle_force_split(0)
    text, _ = plan_of(problem(M=300, N=520, K=576))
    assert split(text) == 1, text


def test_store_validation_and_planning(L):
    """The store op: a second output [M,N] that takes a copy of the values at its place in the list."""
    t = 6 * G
    pre_norm = [op("bias"), op("residual", p0=G, ld=64), op("store", p0=t, ld=64), op("layernorm", 1e-5, 7 * G, 8 * G)]
    p = problem(ops=pre_norm); p.x = 3 * G + G // 2                     # the residual is not x here
    assert validate(L, p) == OK
    assert validate(L, problem(ops=[op("store", p0=t, ld=64), op("store", p0=t + G // 2, ld=80)])) == OK
    assert validate(L, problem(ops=[op("store", p0=None, ld=64)])) == E_NULL
    assert validate(L, problem(ops=[op("store", p0=t, ld=63)])) == E_SHAPE
    assert validate(L, problem(ops=[op("store", p0=t + 1, ld=64)])) == E_ALIGN
    # only before the row op
    assert validate(L, problem(ops=[op("softmax"), op("store", p0=t, ld=64)])) == E_UNSUP
    assert b"store" in L.fle_last_error()
    assert validate(L, problem(ops=[op("store", p0=t, ld=64), op("logsumexp")])) == OK
    # the target overlaps nothing else the call reads or writes
    q = problem()
    for other in (q.x, q.w, q.b, q.out, q.out + 2):
        assert validate(L, problem(ops=[op("store", p0=other, ld=64)])) == E_UNSUP, hex(other)
    assert validate(L, problem(ops=[op("residual", p0=t, ld=64), op("store", p0=t, ld=64)])) == E_UNSUP
    assert validate(L, problem(ops=[op("store", p0=t, ld=64), op("relu"), op("store", p0=t + 64, ld=64)])) == E_UNSUP
    assert validate(L, problem(ops=[op("store", p0=7 * G, ld=64), op("layernorm", 1e-5, 7 * G, 8 * G)])) == E_UNSUP
    p = problem(M=128, N=4096, K=4096, ops=[op("softmax")]); p.workspace, p.workspace_bytes = t, 1 << 26
    assert validate(L, p) == OK
    p = problem(M=128, N=4096, K=4096, ops=[op("store", p0=t + 4096, ld=4096), op("softmax")]); p.workspace, p.workspace_bytes = t, 1 << 26
    assert validate(L, p) == E_UNSUP
    # a split along K keeps the op: the reduction pass writes the copy
    need = ctypes.c_size_t(0)
    buf = ctypes.create_string_buffer(256)
    p = problem(M=128, N=4096, K=4096, ops=[op("store", p0=t, ld=4096)])
    assert L.fle_workspace_size(ctypes.byref(p), ctypes.byref(need)) == OK
    L.fle_last_plan(buf, 256)
    sp = int(re.search(r"split_k=(\d+)", buf.value.decode()).group(1))
    assert sp > 1 and need.value == sp * 128 * 4096 * 4, buf.value
    # every kernel family takes the op; an unaligned target or leading dimension falls back to element stores
    for shape, name in (((4096, 4096, 4096), "tiled"), ((16, 2048, 2048), "thin"), ((64, 4096, 4096), "skinny"), ((64, 63, 64), "general")):
        M, N, K = shape
        p = problem(M=M, N=N, K=K, ops=[op("bias"), op("store", p0=t, ld=N)])
        assert L.fle_workspace_size(ctypes.byref(p), ctypes.byref(need)) == OK
        L.fle_last_plan(buf, 256)
        assert name in buf.value.decode(), (shape, buf.value)
    p = problem(M=4096, N=4096, K=4096, ops=[op("store", p0=t + 2, ld=4098)])
    assert L.fle_workspace_size(ctypes.byref(p), ctypes.byref(need)) == OK
    L.fle_last_plan(buf, 256)
    assert "edge" in buf.value.decode() or "general" in buf.value.decode(), buf.value


# ---------------------------------------------------------------- grouped problems
def groups(n=8, offs=9 * G, w_stride=None, b_stride=None, N=1024, K=512):
    g = binding.FleGroups()
    g.n_groups, g.row_offsets = n, offs
    g.w_group_stride = N * K if w_stride is None else w_stride
    g.b_group_stride = N if b_stride is None else b_stride
    return g


def test_grouped_validation_and_planning(L):
    def plan_of(p, g):
        need = ctypes.c_size_t(0)
        assert L.fle_workspace_size_grouped(ctypes.byref(p), ctypes.byref(g), ctypes.byref(need)) == OK, L.fle_last_error()
        buf = ctypes.create_string_buffer(256)
        L.fle_last_plan(buf, 256)
        return buf.value.decode(), need.value
    tiles = lambda text: tuple(int(v) for v in re.search(r"tiles=(\d+)x(\d+)", text).groups())
    p = problem(M=4096, N=1024, K=512, ops=[op("bias"), op("gelu_tanh")])
    text, need = plan_of(problem(M=32768, N=1024, K=512, ops=[op("bias"), op("gelu_tanh")]), groups(8))
    # 4096 rows per group and more tiles than the chip holds at once: the 256 tile; at most one partly filled tile row per group
    assert "grouped_tiled_bf16_mfma tile=256x256" in text and tiles(text) == (32768 // 256 + 8, 4) and "split_k=1" in text and need == 0, text
    text, _ = plan_of(p, groups(64))
    assert "tile=128x128" in text and tiles(text) == (4096 // 128 + 64, 8), text       # 64 rows per group: the small tile
    assert "+wstream" in text and "+wstream" not in plan_of(problem(M=8192, N=1024, K=512), groups(64))[0]   # W panels read once: streamed
    text, _ = plan_of(problem(M=40, N=1024, K=512), groups(64))
    assert tiles(text)[0] == 40, text                                                     # never more tile rows than rows
    # row ops work as in the plain form: partials per row, staged in out
    text, need = plan_of(problem(M=4096, N=1024, K=512, ops=[op("bias"), op("layernorm", 1e-5, 7 * G, 8 * G)]), groups(8))
    np_ = int(re.search(r"np=(\d+)", text).group(1))
    assert "staging=out" in text and need == 4096 * np_ * 8, text
    # ragged N or a bias stride that breaks 4-column groups: element-wise epilogue
    text, _ = plan_of(problem(M=4096, N=1022, K=512), groups(8, N=1022))
    assert "+edge" in text, text
    text, _ = plan_of(p, groups(8, b_stride=1026))
    assert "+edge" in text, text
    text, _ = plan_of(p, groups(8, b_stride=0))
    assert "+edge" not in text, text
    # fp32 and fp16 operands
    assert "grouped_tiled_f32_mfma" in plan_of(problem(M=4096, N=1024, K=512, dtype=binding.F32), groups(8))[0]
    assert "grouped_tiled_f16_mfma" in plan_of(problem(M=4096, N=1024, K=512, dtype=binding.F16), groups(8))[0]
    # forced tiles
    for code, want in ((4, "tile=256x256"), (5, "tile=128x128")):
        L.fle_force_variant(code)
        try:
            assert want in plan_of(p, groups(8))[0]
        finally:
            L.fle_force_variant(0)

    bad = lambda p_, g_: L.fle_validate_grouped(ctypes.byref(p_), ctypes.byref(g_))
    assert L.fle_validate_grouped(ctypes.byref(p), None) == E_NULL
    assert bad(p, groups(0)) == E_SHAPE
    assert bad(p, groups(1 << 20)) == E_SHAPE
    assert bad(p, groups(8, offs=None)) == E_NULL
    assert bad(p, groups(8, offs=9 * G + 4)) == E_ALIGN
    assert bad(p, groups(8, w_stride=-1)) == E_SHAPE
    assert bad(p, groups(8, w_stride=1024 * 512 + 4)) == E_UNSUP          # W_g would not be 16-byte aligned
    assert bad(problem(M=4096, N=1024, K=500), groups(8, K=500)) == E_UNSUP   # no general-kernel path for groups
    assert b"grouped" in L.fle_last_error()
    assert bad(p, groups(8, offs=p.out + 64)) == E_UNSUP                  # out overlaps the offsets
    g_big = groups(8, w_stride=G // 8)                                      # W_7 would reach into out
    assert bad(p, g_big) == E_UNSUP
    for code in (1, 3, 6, 7, 8):
        L.fle_force_variant(code)
        try:
            assert bad(p, groups(8)) == E_UNSUP
        finally:
            L.fle_force_variant(0)
    L.fle_force_split(2)
    try:
        assert bad(p, groups(8)) == E_UNSUP
    finally:
        L.fle_force_split(0)
    # M == 0: nothing to do, no HIP call
    p0 = problem(M=0, N=1024, K=512); p0.x = None; p0.out = None
    assert L.fle_run_grouped(ctypes.byref(p0), ctypes.byref(groups(8, offs=None))) == OK
    # a workspace that is needed but missing is reported before any launch
    pl = problem(M=4096, N=1024, K=512, ops=[op("softmax")])
    assert L.fle_run_grouped(ctypes.byref(pl), ctypes.byref(groups(8))) == E_WS


def test_every_variant_plans_every_kind_of_epilogue(L):
    """Planning is pure host arithmetic: every kernel variant must produce a complete plan (partials per
    row, staging, workspace) for every kind of epilogue, for each dtype it supports."""
    chains = [[], [op("bias")], [op("softmax")], [op("scale", 2.0), op("logsumexp")],
              [op("bias"), op("residual", p0=6 * G, ld=2048), op("layernorm", 1e-5, 7 * G, 8 * G)],
              [op("bias"), op("store", p0=10 * G, ld=2048), op("gelu_erf")],
              [op("bias"), op("residual", p0=6 * G, ld=2048), op("store", p0=10 * G, ld=2048), op("layernorm", 1e-5, 7 * G, 8 * G)]]
    shapes = {"general": (70, 2048, 83), "tiled": (200, 2048, 128), "tiled256": (300, 2048, 256), "tiled128": (64, 2048, 64),
              "skinny": (32, 2048, 256), "skinny128": (40, 2048, 640), "skinny256": (32, 2048, 1024), "skinnyseq": (100, 2048, 512),
              "thin": (1, 2048, 1024), "auto": (1, 2048, 2048)}
    buf = ctypes.create_string_buffer(256)
    for name, (M, N, K) in shapes.items():
        for dt in (binding.F32, binding.BF16, binding.F16):
            if name.startswith("skinny") and dt == binding.F32:
                continue
            for rows in ((M,) if name != "thin" else (1, 3, 8, 16, 32)):
                for ch in chains:
                    p = problem(M=rows, N=N, K=K, dtype=dt, ops=ch)
                    need = ctypes.c_size_t(0)
                    L.fle_force_variant(binding.VARIANTS[name])
                    try:
                        assert L.fle_workspace_size(ctypes.byref(p), ctypes.byref(need)) == OK, (name, dt, rows, L.fle_last_error())
                    finally:
                        L.fle_force_variant(0)
                    L.fle_last_plan(buf, 256)
                    text = buf.value.decode()
                    np_ = int(re.search(r"np=(\d+)", text).group(1))
                    has_row = any(6 <= o[0] <= 8 for o in ch)
                    assert (np_ > 0) == has_row and (need.value >= rows * np_ * 8) and ("row_op=-1" in text) == (not has_row), text


# ------------------------------------------------------------------ attention (host-side validation only)
def attention(B=2, H=4, T=100, D=64, dtype=binding.BF16, causal=1, base=G, ld=None, scale=0.0, o=None, ldo=None):
    p = binding.FleAttention()
    HD = H * D
    ld = 3 * HD if ld is None else ld
    p.dtype, p.causal, p.B, p.H, p.T, p.D = dtype, causal, B, H, T, D
    p.q, p.k, p.v = base, base + 2 * HD, base + 4 * HD          # the three thirds of one [B*T, 3*H*D] matrix
    p.ldq = p.ldk = p.ldv = ld
    p.o = 64 * G if o is None else o
    p.ldo = HD if ldo is None else ldo
    p.scale = scale
    return p


def test_attention_validation(L):
    v = lambda p: L.fle_attention_validate(ctypes.byref(p))
    assert v(attention()) == OK
    assert v(attention(D=128, dtype=binding.F16, causal=0, scale=0.25)) == OK
    assert v(attention(B=0)) == OK                                   # empty batch: a no-op
    assert v(attention(causal=0)) == OK and v(attention(causal=37)) == OK and v(attention(causal=-1)) == E_OP
    assert v(attention(dtype=binding.F32)) == E_UNSUP
    assert v(attention(D=16)) == E_UNSUP and v(attention(D=96)) == E_UNSUP and v(attention(D=512)) == E_UNSUP
    assert v(attention(D=32)) == OK and v(attention(D=256, H=2)) == OK
    assert v(attention(T=0)) == E_SHAPE and v(attention(H=0)) == E_SHAPE and v(attention(B=-1)) == E_SHAPE
    assert v(attention(ld=4 * 64 - 8)) == E_SHAPE                    # token stride below H*D
    assert v(attention(ld=3 * 256 + 4)) == E_ALIGN                   # not a multiple of 8 elements
    assert v(attention(base=G + 8)) == E_ALIGN
    assert v(attention(ldo=4 * 64 + 2)) == E_ALIGN
    assert v(attention(scale=-1.0)) == E_OP and v(attention(scale=float("inf"))) == E_OP and v(attention(scale=float("nan"))) == E_OP
    assert v(attention(o=G + 64)) == E_UNSUP                         # o inside q
    p = attention(); p.k = None
    assert v(p) == E_NULL
    assert v(attention(T=1 << 20, H=64, D=128)) == E_SHAPE           # a sequence's K spans more than 2 GiB
    assert b"2 GiB" in L.fle_last_error()
    assert L.fle_attention_validate(None) == E_NULL
    # different numbers of queries and keys; sequence strides
    p = attention(T=10); p.Tk = 300
    assert v(p) == OK
    p = attention(T=300, causal=1); p.Tk = 10
    assert v(p) == E_SHAPE                                           # causal needs Tk >= T
    p = attention(T=300, causal=0); p.Tk = 10
    assert v(p) == OK
    p = attention(B=3, H=2, T=50, D=64, ld=3 * 3 * 128); p.sbq = p.sbk = p.sbv = 3 * 128   # sequence-first: tokens interleave
    p.ldo, p.sbo = 3 * 128, 128
    assert v(p) == OK
    p.sbo = 64
    assert v(p) == E_SHAPE                                           # output sequences would collide
    p.sbo = 130
    assert v(p) == E_ALIGN


def attention_block(B=2, T=100, C=256, H=4, dtype=binding.BF16, residual=True, ws=None, ws_bytes=0):
    p = binding.FleAttentionBlock()
    p.dtype, p.causal, p.B, p.T, p.C, p.H = dtype, 1, B, T, C, H
    p.x, p.w_qkv, p.b_qkv, p.w_o, p.b_o, p.out = G, 2 * G, 3 * G, 4 * G, 5 * G, 6 * G
    p.residual = G if residual else None                             # the block's input
    p.workspace, p.workspace_bytes = ws, ws_bytes
    return p


def test_attention_block_validation_and_workspace(L):
    v = lambda p: L.fle_attention_block_validate(ctypes.byref(p))
    assert v(attention_block()) == OK
    assert v(attention_block(C=250)) == E_SHAPE                      # C not a multiple of H
    assert v(attention_block(C=64, H=4)) == E_UNSUP                  # head dimension 16
    assert v(attention_block(dtype=binding.F32)) == E_UNSUP
    p = attention_block(); p.w_o = None
    assert v(p) == E_NULL
    p = attention_block(); p.out = 2 * G                             # out on top of w_qkv
    assert v(p) == E_UNSUP
    need = ctypes.c_size_t(0)
    p = attention_block(B=2, T=100, C=256)
    assert L.fle_attention_block_workspace_size(ctypes.byref(p), ctypes.byref(need)) == OK
    rows = 200
    assert need.value >= rows * 3 * 256 * 2 + rows * 256 * 2 and need.value % 256 == 0
    # run refuses a missing or short workspace before anything is enqueued (no HIP call is made)
    assert L.fle_attention_block_run(ctypes.byref(p)) == E_WS
    p = attention_block(ws=8 * G, ws_bytes=need.value - 256)
    assert L.fle_attention_block_run(ctypes.byref(p)) == E_WS
    p = attention_block(ws=8 * G + 16, ws_bytes=need.value)
    assert L.fle_attention_block_run(ctypes.byref(p)) == E_ALIGN
    p = attention_block(B=0)
    assert L.fle_attention_block_run(ctypes.byref(p)) == OK          # empty batch


# ------------------------------------------------------------------ perceptron chain (host-side validation only)
def chain(widths=(256, 512, 128), dtype=binding.F32, act=2, ws=7 * G, ws_bytes=1 << 20, w_dtype=None):
    n = len(widths) - 1
    arr = (binding.FleChainLayer * n)()
    for i in range(n):
        arr[i].w, arr[i].b, arr[i].n, arr[i].k, arr[i].act = (10 + i) * G, (30 + i) * G, widths[i + 1], widths[i], act
    p = binding.FleChain()
    p.dtype, p.n_layers, p.layers, p.x, p.out = dtype, n, arr, G, 2 * G
    p.w_dtype = dtype if w_dtype is None else w_dtype
    p.workspace, p.workspace_bytes = ws, ws_bytes
    p._keep = arr
    return p


def test_chain_validation_and_workspace(L):
    v = lambda p: L.fle_chain_validate(ctypes.byref(p))
    assert v(chain()) == OK
    assert v(chain(dtype=binding.BF16, act=-1)) == OK and v(chain(act=4)) == OK
    assert v(chain(act=7)) == E_OP                                   # softmax is not an activation of the chain
    assert v(chain(w_dtype=binding.BF16)) == OK and v(chain(w_dtype=binding.F16)) == OK   # 2-byte weights under fp32
    assert v(chain(dtype=binding.BF16, w_dtype=binding.F32)) == E_UNSUP and v(chain(dtype=binding.BF16, w_dtype=binding.F16)) == E_UNSUP
    assert v(chain(widths=(260, 512, 128), w_dtype=binding.BF16)) == E_ALIGN   # 260 bf16 weights: 520 bytes per row
    assert v(chain(widths=(250, 512, 128))) == E_ALIGN               # 250 floats: not a multiple of 16 bytes
    assert v(chain(widths=(256,))) == E_SHAPE                        # no layer
    p = chain(); p.layers[1].k = 640
    assert v(p) == E_SHAPE                                           # layer 1 does not take what layer 0 gives
    p = chain(); p.layers[0].w = None
    assert v(p) == E_NULL
    p = chain(); p.out = 10 * G
    assert v(p) == E_UNSUP                                           # out on top of the first weight matrix
    need = ctypes.c_size_t(0)
    assert L.fle_chain_workspace_size(ctypes.byref(chain()), ctypes.byref(need)) == OK
    assert need.value == 2560 + 1 * 512 * 4                          # barrier state + one buffer (of the widest hidden layer) per layer boundary
    assert L.fle_chain_run(ctypes.byref(chain(ws=None))) == E_WS
    assert L.fle_chain_run(ctypes.byref(chain(ws_bytes=1000))) == E_WS
    assert L.fle_chain_run(ctypes.byref(chain(ws=7 * G + 64))) == E_ALIGN


def test_run_static_refuses_on_the_host_what_it_cannot_take(L):
    """fle_run_static decides everything except the launch on the host: an invalid problem and a problem whose
    scratch exceeds the static array come back as errors before any HIP call."""
    assert L.fle_run_static(None) == E_NULL
    p = problem(ops=[op("softmax"), op("softmax"), op("softmax")])
    assert L.fle_run_static(ctypes.byref(p)) == E_UNSUP
    out = 2 * G
    p = problem(M=4096, N=8192, K=64, ops=[op("layernorm", 1e-5), op("residual", p0=G + out, ld=8192)])
    p.workspace, p.workspace_bytes = 9 * G, 1 << 30     # ignored: the static array is what counts
    need = ctypes.c_size_t(0)
    assert L.fle_workspace_size(ctypes.byref(p), ctypes.byref(need)) == OK and need.value > binding.STATIC_SCRATCH_BYTES
    assert L.fle_run_static(ctypes.byref(p)) == E_WS
    assert b"static array" in L.fle_last_error()
    text = open(os.path.join(ROOT, "include", "fle.h")).read()
    assert "#define FLE_STATIC_SCRATCH_BYTES (16u << 20)" in text and binding.STATIC_SCRATCH_BYTES == 16 << 20


def test_binding_checks_every_tensor_a_kernel_would_touch(L):
    """The kernels get raw pointers and strides: the binding refuses, before the call, an out / b / gamma / beta
    whose shape, dtype, device or stride is not what the kernels assume (host tensors suffice: nothing runs)."""
    import torch
    M, N, K = 8, 16, 32
    bf = torch.bfloat16
    x, w, b = torch.zeros(M, K, dtype=bf), torch.zeros(N, K, dtype=bf), torch.zeros(N, dtype=bf)
    g = torch.ones(N, dtype=bf)
    ok = binding.Call(x, w, b, [("bias",), ("layernorm", g, g, 1e-5)], out=torch.zeros(M, N, dtype=bf))
    assert ok.out.shape == (M, N)
    view = torch.zeros(M, 2 * N, dtype=bf)[:, :N]                     # a row stride larger than N is fine
    assert binding.Call(x, w, b, [("bias",)], out=view).out is view
    bad_outs = [torch.zeros(M, N - 1, dtype=bf), torch.zeros(M - 1, N, dtype=bf), torch.zeros(M, N, dtype=torch.float32),
                torch.zeros(N, M, dtype=bf).t(), torch.zeros(M * N, dtype=bf)]
    for out in bad_outs:
        with pytest.raises((ValueError, TypeError)):
            binding.Call(x, w, b, [("bias",)], out=out)
    with pytest.raises(ValueError):
        binding.Call(x, w, None, [("logsumexp",)], out=torch.zeros(M, 1, dtype=bf))
    assert binding.Call(x, w, None, [("logsumexp",)], out=torch.zeros(M, dtype=bf)).out.shape == (M,)
    for bad_b in (torch.zeros(N - 1, dtype=bf), torch.zeros(2 * N, dtype=bf)[::2], torch.zeros(1, N, dtype=bf)):
        with pytest.raises(ValueError):
            binding.Call(x, w, bad_b, [("bias",)])
    for bad in (torch.ones(N + 1, dtype=bf), torch.ones(2 * N, dtype=bf)[::2]):
        with pytest.raises(ValueError):
            binding.Call(x, w, b, [("layernorm", bad, g, 1e-5)])
        with pytest.raises(ValueError):
            binding.Call(x, w, b, [("layernorm", g, bad, 1e-5)])
    with pytest.raises(TypeError):
        binding.Call(x, w, b, [("layernorm", g.float(), g, 1e-5)])


def test_fp8_problems_validate_and_plan_on_the_tiled_kernels_only(L):
    F8 = binding.F8E4M3
    res = 6 * G
    p = problem(M=4096, N=4096, K=4096, dtype=F8, ops=[op("scale", 0.01), op("bias"), op("relu"), op("residual", p0=res, ld=4096)])
    assert validate(L, p) == OK
    need = ctypes.c_size_t(0)
    assert L.fle_workspace_size(ctypes.byref(p), ctypes.byref(need)) == OK and need.value == 0
    buf = ctypes.create_string_buffer(256)
    L.fle_last_plan(buf, 256)
    assert b"tiled_f8_mfma" in buf.value and b"tile=256x256x128" in buf.value, buf.value
    # a K step is 128 fp8 values; rows must be whole 16-byte chunks: K and the strides multiples of 16 elements
    assert validate(L, problem(M=64, N=64, K=48, dtype=F8)) == OK
    assert validate(L, problem(M=64, N=64, K=40, dtype=F8)) == E_UNSUP
    assert validate(L, problem(M=64, N=64, K=8, dtype=F8)) == E_UNSUP
    q = problem(M=64, N=64, K=64, dtype=F8)
    q.x = G + 8
    assert validate(L, q) == E_UNSUP
    # out / b / residual are bf16: 2-byte alignment and spans
    q = problem(M=64, N=64, K=64, dtype=F8)
    q.out = 3 * G + 1
    assert validate(L, q) == E_ALIGN
    # row ops and the split of K work as for the other dtypes; every other kernel family refuses fp8
    p = problem(M=8192, N=4096, K=4096, dtype=F8, ops=[op("bias"), op("gelu_tanh"), op("layernorm", 1e-5, 7 * G, 8 * G)])
    assert L.fle_workspace_size(ctypes.byref(p), ctypes.byref(need)) == OK and need.value == 8192 * 32 * 2 * 4   # one partial per row and 128 columns
    for forced in (1, 3, 6, 7, 8, 9):
        L.fle_force_variant(forced)
        try:
            assert validate(L, problem(M=32, N=256, K=256, dtype=F8)) == E_UNSUP, forced
        finally:
            L.fle_force_variant(0)
    L.fle_force_split(4)
    try:
        p = problem(M=64, N=128, K=4096, dtype=F8, ops=[op("bias")])
        assert L.fle_workspace_size(ctypes.byref(p), ctypes.byref(need)) == OK and need.value == 4 * 64 * 128 * 4
    finally:
        L.fle_force_split(0)
    assert validate(L, problem(dtype=4)) == E_OP


def test_per_call_plan_choice_is_stateless_and_validated(L):
    """fle_workspace_size_with / fle_run_with take the plan choice as an argument: the same plans as the thread's
    knobs give, nothing left set afterwards, bad choices refused on the host."""
    from paper_2511_16964_amd.binding import FlePlanChoice

    def plan_with(p, variant, split):
        need = ctypes.c_size_t(0)
        c = FlePlanChoice(variant, split)
        st = L.fle_workspace_size_with(ctypes.byref(p), ctypes.byref(c), ctypes.byref(need))
        buf = ctypes.create_string_buffer(256)
        L.fle_last_plan(buf, 256)
        return st, need.value, buf.value.decode()

    def plan_auto(p):
        need = ctypes.c_size_t(0)
        assert L.fle_workspace_size(ctypes.byref(p), ctypes.byref(need)) == OK
        buf = ctypes.create_string_buffer(256)
        L.fle_last_plan(buf, 256)
        return need.value, buf.value.decode()

    p = problem(M=4096, N=4096, K=4096)
    auto = plan_auto(p)
    st, need, text = plan_with(p, binding.VARIANTS["tiled128"], 4)
    assert st == OK and "tile=128x128" in text and "split_k=4" in text and need > 0
    assert plan_auto(p) == auto                                   # nothing stays set
    L.fle_force_variant(binding.VARIANTS["tiled128"]); L.fle_force_split(4)
    try:
        assert plan_auto(p) == (need, text)                       # the knobs reach the same plan
        st2, need2, text2 = plan_with(p, binding.VARIANTS["tiled256"], 1)   # the argument wins over the knobs
        assert st2 == OK and "tile=256x256" in text2 and "split_k=1 " in text2
    finally:
        L.fle_force_variant(0); L.fle_force_split(0)
    assert plan_with(p, 0, 0)[1:] == auto                          # {0, 0} is the library's own choice
    assert L.fle_workspace_size_with(ctypes.byref(p), None, ctypes.byref(ctypes.c_size_t(0))) == E_NULL
    assert plan_with(p, 10, 0)[0] == E_OP and plan_with(p, -1, 0)[0] == E_OP
    assert plan_with(p, 0, 65)[0] == E_OP and plan_with(p, 0, -2)[0] == E_OP
    assert plan_with(problem(M=512, N=512, K=500), binding.VARIANTS["tiled256"], 1)[0] == E_UNSUP    # a plan the problem cannot take
    assert L.fle_run_with(None, None) == E_NULL and L.fle_run_with(ctypes.byref(p), None) == E_NULL
    p = problem(M=512, N=1024, K=256, ops=[op("layernorm", 1e-5)])                                  # needs a workspace: refused on the host
    assert L.fle_run_with(ctypes.byref(p), ctypes.byref(FlePlanChoice(binding.VARIANTS["tiled128"], 1))) == E_WS


def test_tile_table_lookup_and_round_trip(tmp_path):
    T = binding.TileTable
    assert [T.bucket(v) for v in (0, 1, 2, 3, 4, 5, 6, 11, 12, 4096, 5792, 5793, 8192)] == [0, 0, 1, 2, 2, 2, 3, 3, 4, 12, 12, 13, 13]
    plain, row = [("bias",), ("relu",)], [("bias",), ("softmax",)]
    t = T(meta={"device": "x"})
    t.entries[T.key(binding.BF16, 4096, 4096, 4096, plain)] = {"variant": "tiled128", "split": 2, "us": 1.0, "auto_us": 2.0}
    assert t.lookup(binding.BF16, 4000, 4500, 3000, plain) == ("tiled128", 2)
    assert t.lookup(binding.BF16, 4096, 4096, 4096, row) is None           # row reductions are a class of their own
    assert t.lookup(binding.F16, 4096, 4096, 4096, plain) is None and t.lookup(binding.BF16, 2048, 4096, 4096, plain) is None
    t.save(tmp_path / "t.json")
    u = T.load(tmp_path / "t.json")
    assert u.entries == t.entries and u.meta["device"] == "x"
    shipped = T.load()                                                       # the table in the package parses and names real plans
    assert shipped.entries and all(e["variant"] in binding.VARIANTS and 0 <= e["split"] <= 64 for e in shipped.entries.values())
    assert all(re.fullmatch(r"\d:[01]:\d+:\d+:\d+", k) for k in shipped.entries)


def test_block_scaled_fp8_problems_validate_and_plan(L):
    """FLE_MXSCALE: first entry only, fp8 operands only, K a multiple of 128, both scale pointers, no grouped form;
    the plan names the block-scaled kernel."""
    def mx(**kw):
        return op("mxscale", p0=kw.pop("p0", 20 * G), p1=kw.pop("p1", 21 * G))
    p = problem(M=512, N=512, K=512, dtype=binding.F8E4M3, ops=[mx(), op("bias"), op("relu")])
    need = ctypes.c_size_t(0)
    assert L.fle_workspace_size(ctypes.byref(p), ctypes.byref(need)) == OK
    buf = ctypes.create_string_buffer(256)
    L.fle_last_plan(buf, 256)
    assert "tiled_f8mx_mfma" in buf.value.decode(), buf.value
    assert validate(L, problem(M=512, N=512, K=512, dtype=binding.F8E4M3, ops=[op("bias"), mx()])) == E_UNSUP        # not first
    assert validate(L, problem(M=512, N=512, K=512, dtype=binding.BF16, ops=[mx()])) == E_UNSUP                      # bf16 operands
    assert validate(L, problem(M=512, N=512, K=448, dtype=binding.F8E4M3, ops=[mx()])) == E_UNSUP                    # K not a multiple of 128
    assert validate(L, problem(M=512, N=512, K=512, dtype=binding.F8E4M3, ops=[op("mxscale", p0=20 * G, p1=0)])) == E_NULL
    assert validate(L, problem(M=512, N=512, K=512, dtype=binding.F8E4M3, ops=[op("mxscale", p0=20 * G + 2, p1=21 * G)])) == E_ALIGN
    p = problem(M=512, N=512, K=512, dtype=binding.F8E4M3, ops=[mx()])
    assert validate(L, p) == OK
    p = problem(M=512, N=512, K=512, dtype=binding.F8E4M3, ops=[op("mxscale", p0=3 * G + 64, p1=21 * G)])             # scales inside out
    assert validate(L, p) == E_UNSUP
    p = problem(M=512, N=512, K=1024, dtype=binding.F8E4M3, ops=[mx(), op("layernorm", 1e-5)])
    from paper_2511_16964_amd.binding import FlePlanChoice
    c = FlePlanChoice(binding.VARIANTS["tiled128"], 2)
    assert L.fle_workspace_size_with(ctypes.byref(p), ctypes.byref(c), ctypes.byref(need)) == OK and need.value > 0  # split K keeps the scales


def test_layernorm_in_front_of_the_multiplication_validates_and_plans(L):
    """FLE_LAYERNORM_PRE: first entry only, no fp8 and no grouped form; a few rows plan the fused dot-product kernel
    without workspace, other shapes a pass with M * K elements of workspace more than the same list without it."""
    def plan_of(p):
        need = ctypes.c_size_t(0)
        st = L.fle_workspace_size(ctypes.byref(p), ctypes.byref(need))
        buf = ctypes.create_string_buffer(256)
        L.fle_last_plan(buf, 256)
        return st, need.value, buf.value.decode()
    lnp = op("layernorm_pre", 1e-5, 20 * G, 21 * G)
    st, need, text = plan_of(problem(M=2, N=4096, K=4096, ops=[lnp, op("bias"), op("gelu_erf")]))
    assert st == OK and need == 0 and "thin_bf16_dot" in text and "ln_pre=fused" in text
    st, need, text = plan_of(problem(M=4, N=4096, K=4096, dtype=binding.F32, ops=[lnp]))
    assert st == OK and need == 0 and "ln_pre=fused" in text
    st, need, text = plan_of(problem(M=8, N=4096, K=4096, dtype=binding.F32, ops=[lnp]))
    assert st == OK and need == 8 * 4096 * 4 and "thin_f32_dot" in text and "ln_pre=pass" in text   # more than 4 rows: the pass, then the same kernel
    st, need, text = plan_of(problem(M=4096, N=4096, K=4096, ops=[lnp, op("bias")]))
    assert st == OK and need == 4096 * 4096 * 2 and "tile=256x256" in text and "ln_pre=pass" in text
    st0, need0, _ = plan_of(problem(M=512, N=1024, K=256, ops=[op("layernorm", 1e-5)]))
    st, need, text = plan_of(problem(M=512, N=1024, K=256, ops=[lnp, op("layernorm", 1e-5)]))
    assert st == OK and need == need0 + 512 * 256 * 2 and "ln_pre=pass" in text
    p = problem(M=1024, N=1024, K=1024, ops=[lnp]); p.x = p.x + 2; p.ldx = 1027          # misaligned x: the copy is what the kernels read
    st, need, text = plan_of(p)
    assert st == OK and "tiled" in text and "ln_pre=pass" in text
    assert validate(L, problem(M=64, N=64, K=64, ops=[op("bias"), lnp])) == E_UNSUP         # not first
    assert validate(L, problem(M=512, N=512, K=512, dtype=binding.F8E4M3, ops=[lnp])) == E_UNSUP
    assert validate(L, problem(M=64, N=64, K=64, ops=[op("layernorm_pre", float("nan"), 20 * G, 21 * G)])) == E_OP
    assert validate(L, problem(M=64, N=64, K=64, ops=[op("layernorm_pre", 1e-5, 20 * G + 1, 21 * G)])) == E_ALIGN
    assert validate(L, problem(M=64, N=64, K=64, ops=[op("layernorm_pre", 1e-5, 3 * G + 8, 21 * G)])) == E_UNSUP   # gamma inside out
    assert validate(L, problem(M=64, N=64, K=64, ops=[op("layernorm_pre", 1e-5)])) == OK    # gamma and beta absent
    p = problem(M=4096, N=4096, K=4096, ops=[lnp])
    assert L.fle_run(ctypes.byref(p)) == E_WS                                               # the pass needs its workspace
    # grouped problems refuse it
    from paper_2511_16964_amd.binding import FleGroups
    g = FleGroups(); g.n_groups, g.row_offsets, g.w_group_stride, g.b_group_stride = 2, 30 * G, 64 * 64, 64
    assert L.fle_validate_grouped(ctypes.byref(problem(M=64, N=64, K=64, ops=[lnp])), ctypes.byref(g)) == E_UNSUP

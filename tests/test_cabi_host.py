"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol the header declares, and rejects bad arguments before enqueueing
anything (every error path returns its documented code)."""
import ctypes
import os
import re

import pytest

import paper_2411_17116_amd as sa
from paper_2411_17116_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "star_attn.h")

# status codes as the header defines them
ERR = dict(INVALID_SHAPE=-1, NULL_POINTER=-2, UNSUPPORTED_HEAD_DIM=-3, UNSUPPORTED_DTYPE=-4,
           ANCHOR_GT_BLOCK=-5, CACHE_OVERFLOW=-6, WORKSPACE_TOO_SMALL=-7, LAUNCH_FAILED=-8,
           MISALIGNED=-9, INVALID_MODE=-10, BUSY=-11)


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(sa.lib_path()):
        from paper_2411_17116_amd import build
        build.build(verbose=False)
    return sa.load_library()


def good_shape(**kw):
    base = dict(dtype="bf16", batch=1, n_q_heads=8, n_kv_heads=2, head_dim=128, ctx_len=1024,
                block=256, anchor=256, cache_capacity=1024 + 64)
    base.update(kw)
    return sa.StarShape.make(**base)


def test_header_symbols_are_exported(lib):
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(star_attn_[a-z0-9_]+)\s*\(", text)
    assert set(names) >= {"star_attn_phase1", "star_attn_phase2", "star_attn_workspace_bytes",
                          "star_attn_status_string", "star_attn_kernel_path",
                          "star_attn_phase1_anchor", "star_attn_phase1_workspace_bytes",
                          "star_attn_phase1_rope", "star_attn_phase2_rope", "star_attn_rope",
                          "star_attn_phase2_partial", "star_attn_merge", "star_attn_phase2_plan",
                          "star_attn_phase2_static"}
    for n in set(names):
        assert hasattr(lib, n), f"{n} declared in the header but not exported"


def test_header_status_codes_match(lib):
    text = open(HEADER).read()
    for name, code in ERR.items():
        m = re.search(rf"STAR_ATTN_ERR_{name}\s*=\s*(-?\d+)", text)
        assert m and int(m.group(1)) == code
        assert sa.status_string(code) != "unknown status"
    assert sa.status_string(0) == "ok"
    assert sa.status_string(-1234) == "unknown status"


def test_shape_struct_layout_matches_header():
    # 6 x int32, 4 x int64, 2 x float = 24 + 32 + 8 bytes, no padding surprises
    assert ctypes.sizeof(binding.StarShape) == 64
    assert binding.StarShape.ctx_len.offset == 24
    assert binding.StarShape.softmax_scale.offset == 56


# Placeholder pointers: aligned, non-NULL, never dereferenced because every call
# below is rejected by the host-side validation.
def _p1(lib, shape, Q=0x1000, K=0x1000, V=0x1000, O=0x1000, LSE=None, Kc=0x1000, Vc=0x1000):
    return lib.star_attn_phase1(ctypes.byref(shape) if shape is not None else None,
                                Q, K, V, O, LSE, Kc, Vc, None, 0, None)


def _p1a(lib, shape, mode, Q=0x1000, K=0x1000, V=0x1000, Ka=0x1000, Va=0x1000, O=0x1000, LSE=None,
         Kc=0x1000, Vc=0x1000, ws=0x1000, ws_bytes=0):
    return lib.star_attn_phase1_anchor(ctypes.byref(shape), mode, Q, K, V, Ka, Va, O, LSE, Kc, Vc,
                                       ws, ws_bytes, None)


def _p2(lib, shape, cache_len, q_len, Qq=0x1000, Kq=0x1000, Vq=0x1000, Kc=0x1000, Vc=0x1000,
        Op=None, Lp=None, O=0x1000, ws=0x1000, ws_bytes=1 << 40):
    return lib.star_attn_phase2(ctypes.byref(shape), cache_len, q_len, Qq, Kq, Vq, Kc, Vc, Op, Lp,
                                O, ws, ws_bytes, None)


@pytest.mark.parametrize("kw,code", [
    (dict(dtype=7), "UNSUPPORTED_DTYPE"),
    (dict(batch=0), "INVALID_SHAPE"),
    (dict(n_q_heads=6, n_kv_heads=4), "INVALID_SHAPE"),
    (dict(ctx_len=0), "INVALID_SHAPE"),
    (dict(block=0), "INVALID_SHAPE"),
    (dict(head_dim=96), "UNSUPPORTED_HEAD_DIM"),
    (dict(head_dim=64), "UNSUPPORTED_HEAD_DIM"),          # bf16 path is d = 128 only
    (dict(dtype="fp32", head_dim=32), "UNSUPPORTED_HEAD_DIM"),
    (dict(anchor=257), "ANCHOR_GT_BLOCK"),
    (dict(anchor=-1), "ANCHOR_GT_BLOCK"),
    (dict(cache_capacity=1000), "CACHE_OVERFLOW"),
    (dict(softmax_scale=-1.0), "INVALID_SHAPE"),
    (dict(cache_capacity=1 << 31), "INVALID_SHAPE"),       # tokens are indexed with 32 bits
    (dict(block=1 << 32, anchor=0), "INVALID_SHAPE"),
])
def test_bad_shapes_are_rejected_by_both_entry_points(lib, kw, code):
    shape = good_shape(**kw)
    assert _p1(lib, shape) == ERR[code]
    assert _p2(lib, shape, shape.ctx_len, 1) == ERR[code]
    assert sa.workspace_bytes(shape, 8) == 0
    assert sa.kernel_path(shape) is None


def test_null_and_misaligned_pointers(lib):
    shape = good_shape()
    assert _p1(lib, None) == ERR["NULL_POINTER"]
    for arg in ("Q", "K", "V", "O", "Kc", "Vc"):
        assert _p1(lib, shape, **{arg: None}) == ERR["NULL_POINTER"]
        assert _p1(lib, shape, **{arg: 0x1008}) == ERR["MISALIGNED"]
    L = shape.ctx_len
    for arg in ("Qq", "Kq", "Vq", "Kc", "Vc", "O", "ws"):
        assert _p2(lib, shape, L, 1, **{arg: None}) == ERR["NULL_POINTER"]
    assert _p2(lib, shape, L, 1, Op=0x1000, Lp=None) == ERR["NULL_POINTER"]   # parts come in pairs
    assert _p2(lib, shape, L, 1, Op=None, Lp=0x1000) == ERR["NULL_POINTER"]
    assert _p2(lib, shape, L, 1, Qq=0x1004) == ERR["MISALIGNED"]
    assert _p2(lib, shape, L, 1, ws=0x1010) == ERR["MISALIGNED"]             # workspace: 256 bytes


def test_phase2_call_arguments(lib):
    shape = good_shape()
    L, cap = shape.ctx_len, shape.cache_capacity
    assert _p2(lib, shape, L, 0) == ERR["INVALID_SHAPE"]
    assert _p2(lib, shape, L - 1, 1) == ERR["INVALID_SHAPE"]          # cache_len below the context
    assert _p2(lib, shape, cap, 1) == ERR["CACHE_OVERFLOW"]
    assert _p2(lib, shape, cap - 3, 4) == ERR["CACHE_OVERFLOW"]
    need = sa.workspace_bytes(shape, 16)
    assert need > 0 and need % 256 == 0
    # (every call in this file carries at least one invalid argument, so nothing
    # is ever enqueued with the placeholder pointers)
    assert _p2(lib, shape, L, 16, ws_bytes=64) == ERR["WORKSPACE_TOO_SMALL"]
    assert _p2(lib, shape, L, 1, ws_bytes=64) == ERR["WORKSPACE_TOO_SMALL"]
    assert _p2(lib, shape, L, 16, Op=0x1000, Lp=0x1000, ws_bytes=64) == ERR["WORKSPACE_TOO_SMALL"]


def test_workspace_query_covers_every_call_size(lib):
    """The size reported for max_q_len covers every smaller call: it never
    shrinks as max_q_len grows."""
    for shape in (good_shape(), good_shape(dtype="fp32", head_dim=64, n_q_heads=1, n_kv_heads=1),
                  good_shape(ctx_len=100000, block=8192, anchor=2048, cache_capacity=100500,
                             n_q_heads=64, n_kv_heads=8, batch=2)):
        sizes = [sa.workspace_bytes(shape, q) for q in (1, 2, 3, 4, 5, 16, 17, 64, 65, 200, 256)]
        assert all(s > 0 for s in sizes)
        assert sizes == sorted(sizes), "requirement must not shrink as max_q_len grows"


def test_plan_query(lib):
    """star_attn_phase2_plan answers on the host: decode-sized calls stream the
    cache, flat only without per-part outputs; caches beyond 192 MiB of K + V are
    read with non-temporal loads, two steps per batch."""
    small = good_shape()
    p = sa.phase2_plan(small, small.ctx_len, 1)
    assert (p.decode, p.flat, p.non_temporal, p.steps_per_batch) == (1, 1, 0, 1)
    assert p.workspace_bytes <= sa.workspace_bytes(small, 1)
    p = sa.phase2_plan(small, small.ctx_len, 1, want_parts=True)
    assert (p.decode, p.flat) == (1, 0) and p.n_splits >= 5          # 4 blocks + the tail
    p = sa.phase2_plan(small, small.ctx_len, 64)
    assert (p.decode, p.flat, p.steps_per_batch) == (0, 0, 0)
    c3 = good_shape(n_q_heads=32, n_kv_heads=8, ctx_len=131072, block=16384, anchor=16384,
                    cache_capacity=131072 + 384)
    p = sa.phase2_plan(c3, 131072 + 256, 1)
    assert (p.decode, p.flat, p.non_temporal, p.steps_per_batch) == (1, 1, 1, 2)
    assert p.n_splits == 96                                           # 256 CUs x 3 over 8 KV heads
    p = sa.phase2_plan(c3, 131072 + 256, 1, want_parts=True)
    assert (p.decode, p.flat, p.non_temporal) == (1, 0, 1)
    f32 = good_shape(dtype="fp32", head_dim=64)
    assert sa.phase2_plan(f32, f32.ctx_len, 1).decode == 0
    info = binding.PlanInfo()
    call = lib.star_attn_phase2_plan
    assert call(ctypes.byref(small), small.ctx_len, 0, 0, ctypes.byref(info)) == ERR["INVALID_SHAPE"]
    assert call(ctypes.byref(small), small.cache_capacity, 1, 0, ctypes.byref(info)) == ERR["CACHE_OVERFLOW"]
    assert call(ctypes.byref(small), small.ctx_len, 1, 0, None) == ERR["NULL_POINTER"]


def test_static_scratch_entry_point_arguments(lib):
    """star_attn_phase2_static validates like star_attn_phase2 and refuses a call
    whose per-split pairs do not fit its static scratch."""
    shape = good_shape()
    L, cap = shape.ctx_len, shape.cache_capacity

    def st(sh=shape, cache_len=L, q_len=1, Qq=0x1000, Kq=0x1000, Vq=0x1000, Kc=0x1000, Vc=0x1000,
           O=0x1000):
        return lib.star_attn_phase2_static(ctypes.byref(sh), cache_len, q_len, Qq, Kq, Vq, Kc, Vc, O,
                                           None)

    assert st(q_len=0) == ERR["INVALID_SHAPE"]
    assert st(cache_len=cap) == ERR["CACHE_OVERFLOW"]
    for arg in ("Qq", "Kq", "Vq", "Kc", "Vc", "O"):
        assert st(**{arg: None}) == ERR["NULL_POINTER"]
    assert st(O=0x1008) == ERR["MISALIGNED"]
    assert st(sh=good_shape(head_dim=96)) == ERR["UNSUPPORTED_HEAD_DIM"]
    m = re.search(r"#define\s+STAR_ATTN_STATIC_SCRATCH_BYTES\s+\((\d+)u\s*<<\s*(\d+)\)", open(HEADER).read())
    assert m and int(m.group(1)) << int(m.group(2)) == binding.STATIC_SCRATCH_BYTES
    # query encoding at the 128K shape: 38 MB of per-split pairs, more than the scratch
    c3 = good_shape(n_q_heads=32, n_kv_heads=8, ctx_len=131072, block=16384, anchor=16384,
                    cache_capacity=131072 + 384)
    assert sa.phase2_plan(c3, 131072, 256).workspace_bytes > binding.STATIC_SCRATCH_BYTES
    assert st(sh=c3, cache_len=131072, q_len=256) == ERR["WORKSPACE_TOO_SMALL"]
    # every decode-sized call fits
    for sh in (c3, good_shape(n_q_heads=64, n_kv_heads=8, batch=4, ctx_len=131072, block=8192,
                              anchor=2048, cache_capacity=131072 + 192)):
        for q in (1, 2):
            assert sa.phase2_plan(sh, sh.ctx_len, q).workspace_bytes <= binding.STATIC_SCRATCH_BYTES


def test_kernel_path_names(lib):
    assert sa.kernel_path(good_shape()) == "bf16-mfma"
    assert sa.kernel_path(good_shape(dtype="fp32", head_dim=64)) == "f32-valu"


def test_binding_refuses_to_run_without_the_library(monkeypatch, tmp_path):
    """No CPU fallback: a missing library is an error, not a silent slow path."""
    monkeypatch.setattr(binding, "_LIB", None)
    monkeypatch.setattr(binding, "_HERE", str(tmp_path))
    with pytest.raises(FileNotFoundError):
        binding.load_library()


def test_phase1_anchor_variant_arguments(lib):
    shape = good_shape()
    EXT = binding.ANCHOR_EXTERNAL
    for mode in (-1, 5, 99):
        assert _p1a(lib, shape, mode) == ERR["INVALID_MODE"]
    assert _p1a(lib, good_shape(anchor=300), binding.ANCHOR_PREVIOUS) == ERR["ANCHOR_GT_BLOCK"]
    for mode in (binding.ANCHOR_FIRST, binding.ANCHOR_PREVIOUS, EXT):
        assert _p1a(lib, shape, mode, Q=None) == ERR["NULL_POINTER"]
        assert _p1a(lib, shape, mode, Kc=0x1004) == ERR["MISALIGNED"]
    # the external anchor needs its tensors; the fp32 path also needs a workspace
    # for their head-major copy (the bf16 kernel reads the tensors where they are:
    # its workspace is the launch's work-queue counters in every mode)
    assert sa.binding.phase1_workspace_bytes(shape, EXT) == 256
    assert sa.binding.phase1_workspace_bytes(shape, binding.ANCHOR_FIRST) == 256
    assert _p1a(lib, shape, EXT, ws=0x1008, ws_bytes=256) == ERR["MISALIGNED"]
    assert _p1a(lib, shape, EXT, ws_bytes=64) == ERR["WORKSPACE_TOO_SMALL"]
    assert _p1a(lib, shape, EXT, Ka=None) == ERR["NULL_POINTER"]
    assert _p1a(lib, shape, EXT, Va=None) == ERR["NULL_POINTER"]
    assert _p1a(lib, shape, EXT, Ka=0x1008) == ERR["MISALIGNED"]
    f32 = good_shape(dtype="fp32", head_dim=64)
    need = sa.binding.phase1_workspace_bytes(f32, EXT)
    assert need == 2 * 1 * 2 * 256 * 64 * 4 and need % 256 == 0
    assert sa.binding.phase1_workspace_bytes(f32, binding.ANCHOR_FIRST) == 0
    assert sa.binding.phase1_workspace_bytes(f32, binding.ANCHOR_PREVIOUS) == 0
    assert sa.binding.phase1_workspace_bytes(good_shape(batch=0), EXT) == 0
    # one anchor per block: n = 4 of them
    assert sa.binding.phase1_workspace_bytes(f32, binding.ANCHOR_PER_BLOCK) == 4 * need
    assert sa.binding.phase1_workspace_bytes(shape, binding.ANCHOR_PER_BLOCK) == 256
    assert _p1a(lib, shape, binding.ANCHOR_PER_BLOCK, Ka=None) == ERR["NULL_POINTER"]
    assert _p1a(lib, f32, binding.ANCHOR_PER_BLOCK, ws_bytes=need) == ERR["WORKSPACE_TOO_SMALL"]
    assert _p1a(lib, f32, EXT, Ka=None, ws_bytes=need) == ERR["NULL_POINTER"]
    assert _p1a(lib, f32, EXT, ws=None, ws_bytes=need) == ERR["NULL_POINTER"]
    assert _p1a(lib, f32, EXT, ws=0x1010, ws_bytes=need) == ERR["MISALIGNED"]
    assert _p1a(lib, f32, EXT, ws_bytes=need - 1) == ERR["WORKSPACE_TOO_SMALL"]
    # a host's share takes one anchor, like EXTERNAL
    ALL = binding.ANCHOR_ALL_BLOCKS
    assert sa.binding.phase1_workspace_bytes(f32, ALL) == need
    assert sa.binding.phase1_workspace_bytes(shape, ALL) == 256
    assert _p1a(lib, shape, ALL, Ka=None) == ERR["NULL_POINTER"]
    assert _p1a(lib, shape, ALL, Va=0x1008) == ERR["MISALIGNED"]
    assert _p1a(lib, f32, ALL, ws_bytes=need - 1) == ERR["WORKSPACE_TOO_SMALL"]


def test_host_share_entry_point_arguments(lib):
    """star_attn_phase2_partial and star_attn_merge validate on the host."""
    shape = good_shape()
    L, cap = shape.ctx_len, shape.cache_capacity

    def part(cache_len=L, q_len=1, Qq=0x1000, Kq=None, Vq=None, Kc=0x1000, Vc=0x1000, A=0x1000,
             LSE=0x1000, ws=0x1000, ws_bytes=64):
        return lib.star_attn_phase2_partial(ctypes.byref(shape), cache_len, q_len, Qq, Kq, Vq, Kc, Vc,
                                            A, LSE, ws, ws_bytes, None)

    assert part() == ERR["WORKSPACE_TOO_SMALL"]                     # valid up to the workspace
    assert part(Kq=0x1000, Vq=0x1000) == ERR["WORKSPACE_TOO_SMALL"]
    assert part(Kq=0x1000) == ERR["NULL_POINTER"]                   # K without V
    assert part(Vq=0x1000) == ERR["NULL_POINTER"]
    assert part(A=None) == ERR["NULL_POINTER"]
    assert part(LSE=None) == ERR["NULL_POINTER"]
    assert part(Qq=None) == ERR["NULL_POINTER"]
    assert part(A=0x1004) == ERR["MISALIGNED"]
    assert part(LSE=0x1002) == ERR["MISALIGNED"]
    assert part(q_len=0) == ERR["INVALID_SHAPE"]
    assert part(cache_len=L - 1) == ERR["INVALID_SHAPE"]
    # a context host may read a full cache; the query host needs room to append
    assert part(cache_len=cap) == ERR["WORKSPACE_TOO_SMALL"]
    assert part(cache_len=cap + 1) == ERR["CACHE_OVERFLOW"]
    assert part(cache_len=cap, Kq=0x1000, Vq=0x1000) == ERR["CACHE_OVERFLOW"]

    def mrg(n_parts=3, q_len=2, Ap=0x1000, Lp=0x1000, O=0x1000, A=None, LSE=None, sh=shape):
        return lib.star_attn_merge(ctypes.byref(sh), n_parts, q_len, Ap, Lp, O, A, LSE, None)

    assert mrg(n_parts=0) == ERR["INVALID_SHAPE"]
    assert mrg(q_len=0) == ERR["INVALID_SHAPE"]
    assert mrg(n_parts=(1 << 20) + 1) == ERR["INVALID_SHAPE"]
    assert mrg(Ap=None) == ERR["NULL_POINTER"]
    assert mrg(Lp=None) == ERR["NULL_POINTER"]
    assert mrg(O=None) == ERR["NULL_POINTER"]                       # neither O nor A
    assert mrg(Ap=0x1004) == ERR["MISALIGNED"]
    assert mrg(O=0x1008) == ERR["MISALIGNED"]
    assert mrg(O=None, A=0x1008) == ERR["MISALIGNED"]
    assert mrg(LSE=0x1001) == ERR["MISALIGNED"]
    assert mrg(sh=good_shape(head_dim=96)) == ERR["UNSUPPORTED_HEAD_DIM"]


def test_rope_entry_point_arguments(lib):
    shape = good_shape()
    L = shape.ctx_len
    d = ctypes.c_double

    def p1r(theta=10000.0, pos0=0, Q=0x1000, K=0x1000):
        return lib.star_attn_phase1_rope(ctypes.byref(shape), d(theta), pos0, Q, K, 0x1000, 0x1000,
                                         None, 0x1000, 0x1000, None, 0, None)

    def p2r(theta=10000.0, pos0=0, Qq=0x1000, ws_bytes=64):
        return lib.star_attn_phase2_rope(ctypes.byref(shape), d(theta), pos0, L, 1, Qq, 0x1000,
                                         0x1000, 0x1000, 0x1000, None, None, 0x1000, 0x1000,
                                         ws_bytes, None)

    def rot(theta=10000.0, pos0=0, heads=8, tokens=4, X=0x1000, Y=0x1000):
        return lib.star_attn_rope(ctypes.byref(shape), heads, tokens, pos0, d(theta), X, Y, None)

    for bad_theta in (0.0, 1.0, -5.0, float("inf"), float("nan")):
        assert p1r(theta=bad_theta) == ERR["INVALID_SHAPE"]
        assert p2r(theta=bad_theta) == ERR["INVALID_SHAPE"]
        assert rot(theta=bad_theta) == ERR["INVALID_SHAPE"]
    assert p1r(pos0=-1) == ERR["INVALID_SHAPE"]
    assert p2r(pos0=-1) == ERR["INVALID_SHAPE"]
    assert rot(pos0=-1) == ERR["INVALID_SHAPE"]
    assert p1r(Q=None) == ERR["NULL_POINTER"]
    assert p1r(K=0x1004) == ERR["MISALIGNED"]
    assert p2r(Qq=None) == ERR["NULL_POINTER"]
    assert p2r() == ERR["WORKSPACE_TOO_SMALL"]
    assert rot(heads=0) == ERR["INVALID_SHAPE"]
    assert rot(tokens=0) == ERR["INVALID_SHAPE"]
    assert rot(X=None) == ERR["NULL_POINTER"]
    assert rot(Y=0x1002) == ERR["MISALIGNED"]


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 on its own, and a
    C caller must link against the library by the declared names."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_header.c"
    src.write_text(
        '#include "star_attn.h"\n'
        "int main(void) {\n"
        "  star_attn_shape s = {0};\n"
        "  s.dtype = STAR_ATTN_BF16; s.batch = 0;\n"
        "  /* every call below is rejected by validation: nothing is enqueued */\n"
        "  int rc = star_attn_phase1(&s, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0);\n"
        "  rc |= star_attn_phase2(&s, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0);\n"
        "  rc |= star_attn_phase1_anchor(&s, STAR_ATTN_ANCHOR_PER_BLOCK, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0);\n"
        "  rc |= star_attn_phase1_rope(&s, 10000.0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0);\n"
        "  rc |= star_attn_phase2_rope(&s, 10000.0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0);\n"
        "  rc |= star_attn_rope(&s, 1, 1, 0, 10000.0, 0, 0, 0);\n"
        "  rc |= star_attn_phase2_partial(&s, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0);\n"
        "  rc |= star_attn_merge(&s, 1, 1, 0, 0, 0, 0, 0, 0);\n"
        "  { star_attn_plan_info pi; rc |= star_attn_phase2_plan(&s, 0, 1, 0, &pi); }\n"
        "  rc |= star_attn_phase2_static(&s, 0, 0, 0, 0, 0, 0, 0, 0, 0);\n"
        "  return (rc != 0 && star_attn_workspace_bytes(&s, 1) == 0 &&\n"
        "          star_attn_phase1_workspace_bytes(&s, 0) == 0 &&\n"
        "          star_attn_status_string(rc) != 0 && star_attn_kernel_path(&s) == 0) ? 0 : 1;\n"
        "}\n")
    inc = os.path.join(ROOT, "include")
    subprocess.run([gcc, "-std=c99", "-Wall", "-Werror", "-pedantic", "-fsyntax-only", f"-I{inc}", str(src)],
                   check=True)
    if not os.path.exists(sa.lib_path()):
        pytest.skip("library not built")
    exe = tmp_path / "use_header"
    libdir = os.path.dirname(sa.lib_path())
    r = subprocess.run([gcc, "-std=c99", f"-I{inc}", str(src), "-o", str(exe), f"-L{libdir}", "-lstarattn",
                        f"-Wl,-rpath,{libdir}"], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    assert subprocess.run([str(exe)]).returncode == 0

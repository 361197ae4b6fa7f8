"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every function the public header declares, the host helpers compute, and
argument errors are reported before anything is launched."""
import ctypes as C
import os
import re

import pytest

from oracle import fastvar_oracle as O
from paper_2503_23367_amd import binding as fb
from paper_2503_23367_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    src = open(os.path.join(ROOT, "include", "fastvar.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(fastvar_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    L = fb.lib()
    names = _declared_functions()
    assert len(names) >= 11
    for n in names:
        assert hasattr(L, n), f"{n} declared in include/fastvar.h but not exported"
    assert set(names) == set(fb.EXPORTS)


def test_version_and_strerror():
    assert fb.fastvar_version() == 100
    assert fb.strerror(0) == "ok"
    for code in (-1, -2, -3, -4, -5):
        assert fb.strerror(code) not in ("ok", "unknown error")
    assert fb.strerror(-99) == "unknown error"


def test_keep_count_agrees_with_oracle_reading():
    for N in (0, 1, 7, 256, 576, 1024, 4096, 9216, 16384):
        for r in (0.0, 0.1, 0.25, 0.3, 0.4, 0.5, 0.6, 0.75, 1.0, 1.5, -0.5):
            assert fb.fastvar_keep_count(N, r) == O.keep_count(N, r), (N, r)
    for w in synth.WORKLOADS.values():
        assert fb.fastvar_keep_count(w.N, w.keep_ratio) == w.k
    assert fb.fastvar_keep_count(-1, 0.5) == fb.FASTVAR_EINVAL


def test_schedule_plan_agrees_with_oracle_and_rejects_bad_schedules():
    sides = (1, 2, 4, 6, 8, 12, 16, 20, 24, 32, 40, 48, 64)
    cases = [(sides, sides, (0.4, 0.5, 1.0, 1.0)), (sides, sides, (0.5, 0.75)), (sides, sides, ()),
             ((1, 2, 4, 8, 16), (1, 3, 6, 12, 24), (0.5, 0.75)), ((5, 5), (5, 5), (0.5,)),
             ((3, 7, 9, 11), (2, 5, 9, 13), (0.0, 0.33, 0.999))]
    for hs, ws, pr in cases:
        keep, cached = fb.fastvar_schedule_plan(hs, ws, pr)
        want_keep, _, want_cached = O.schedule_plan(list(zip(hs, ws)), pr)
        assert keep == want_keep and cached == want_cached, (hs, ws, pr)
    # the paper's thirteen-step setting: the cached step is the 24x24 one, the last two steps are skipped
    keep, cached = fb.fastvar_schedule_plan(sides, sides, (0.4, 0.5, 1.0, 1.0))
    assert cached == 8 and keep[9:] == [614, 800, 0, 0]
    for hs, ws, pr in [((2, 4), (2, 4), (0.5, 0.5)),          # every step pruned: nothing left to cache
                       ((2, 0), (2, 4), (0.5,)), ((2, 4), (2, 4), (1.5,)), ((2, 4), (2, 4), (-0.1,)),
                       ((2, 400), (2, 400), (0.5,))]:          # 160000 tokens: beyond the maximum
        with pytest.raises(fb.FastvarError) as e:
            fb.fastvar_schedule_plan(hs, ws, pr)
        assert e.value.code == fb.FASTVAR_EINVAL


def test_workspace_sizes_cover_the_stages():
    d = fb.make_dims(2048, 16, 128, 8192)
    s = fb.fastvar_select_workspace_bytes(1, 4096, 2048)
    b = fb.fastvar_block_workspace_bytes(d, 1, 2048)
    r = fb.fastvar_restore_workspace_bytes(1, 4096)
    assert s > 0 and b >= 2048 * (3 * 2048 + 8192) * 2 and r >= 4096 * 4
    assert fb.fastvar_step_workspace_bytes(d, 1, 4096, 2048) == s + b + r
    assert fb.fastvar_block_workspace_bytes(d, 1, 0) == 0
    # (not monotone in the row count: the shapes that split work between workgroups add scratch for partial
    # results; far enough up the activations dominate)
    assert fb.fastvar_block_workspace_bytes(d, 8, 2048) > b
    assert fb.fastvar_select_workspace_bytes(0, 16, 64) == 0


def test_sublayer_workspace_covers_both_halves_whatever_their_kept_counts():
    """The block scratch is not monotone in the kept count (k = 2560 needs more than k = 3072 at the large
    model's widths), so the sub-layer step's size must be the larger of the two halves' layouts, not the
    layout of the larger count: exactly what the entry point's own argument check asks for."""
    d = fb.make_dims(2048, 16, 128, 8192)
    B, N = 1, 4096
    fixed = fb.fastvar_select_workspace_bytes(B, N, 2048) + fb.fastvar_restore_workspace_bytes(B, N)
    ks = (0, 1, 64, 410, 1024, 1638, 2048, 2458, 2560, 3072, 4096)
    sizes = {k: fb.fastvar_block_workspace_bytes(d, B, k) for k in ks}
    assert any(sizes[a] > sizes[b] for a in ks for b in ks if a < b), "expected a non-monotone pair"
    for ka in ks:
        for kf in ks:
            got = fb.fastvar_step_sublayer_workspace_bytes(d, B, N, ka, kf)
            assert got == fixed + max(sizes[ka], sizes[kf]), (ka, kf)


def test_argument_errors_are_reported_before_any_launch():
    """Fake (never dereferenced) pointers: every call must fail validation on the host."""
    L = fb.lib()
    P = 0x10000  # 16-byte aligned, not a real allocation
    big = 1 << 40
    # selection
    assert L.fastvar_select_pivotal(None, 1, 4, 4, 64, 4, P, None, None, P, big, None) == fb.FASTVAR_EINVAL
    assert L.fastvar_select_pivotal(P, 0, 4, 4, 64, 4, P, None, None, P, big, None) == fb.FASTVAR_EINVAL
    assert L.fastvar_select_pivotal(P, 1, 4, 4, 64, 17, P, None, None, P, big, None) == fb.FASTVAR_EINVAL
    assert L.fastvar_select_pivotal(P, 1, 4, 4, 64, 4, None, None, None, P, big, None) == fb.FASTVAR_EINVAL
    assert L.fastvar_select_pivotal(P, 1, 4, 4, 64, 4, P, None, None, P, 8, None) == fb.FASTVAR_EWORKSPACE
    assert L.fastvar_select_pivotal(P, 1, 4, 4, 64, 4, P, None, None, None, 0, None) == fb.FASTVAR_EWORKSPACE
    assert L.fastvar_select_pivotal(P + 4, 1, 4, 4, 64, 4, P, None, None, P, big, None) == fb.FASTVAR_EALIGN
    assert L.fastvar_select_pivotal(P, 1, 4, 4, 63, 4, P, None, None, P, big, None) == fb.FASTVAR_EALIGN
    assert L.fastvar_select_pivotal(P, 1, 200, 200, 64, 4, P, None, None, P, big, None) == fb.FASTVAR_ECAPACITY
    # block
    d = fb.make_dims(128, 2, 64, 256)
    w = fb.BlockWeights(*([P] * 12))
    args = lambda **o: [o.get("x", P), o.get("N", 16), o.get("idx", P), o.get("B", 1), o.get("k", 4),
                        C.byref(o.get("d", d)), C.byref(o.get("w", w)), o.get("kc", P), o.get("vc", P),
                        o.get("L0", 8), o.get("L_cap", 16), o.get("y", P), o.get("ws", P),
                        o.get("nb", big), None]
    f = L.fastvar_block_forward_pruned
    assert f(*args(L0=13)) == fb.FASTVAR_ECAPACITY
    assert f(*args(k=17)) == fb.FASTVAR_EINVAL
    assert f(*args(kc=None)) == fb.FASTVAR_EINVAL
    assert f(*args(d=fb.make_dims(128, 3, 64, 256))) == fb.FASTVAR_EINVAL
    assert f(*args(d=fb.make_dims(128, 4, 32, 256))) == fb.FASTVAR_EALIGN
    assert f(*args(d=fb.make_dims(128, 2, 64, 250))) == fb.FASTVAR_EALIGN
    assert f(*args(d=fb.Dims(128, 2, 64, 256, 1e-6, 0.0))) == fb.FASTVAR_EINVAL
    assert f(*args(L_cap=12, L0=4)) == fb.FASTVAR_EALIGN
    assert f(*args(nb=64)) == fb.FASTVAR_EWORKSPACE
    wn = fb.BlockWeights(*([P] * 12))
    wn.w_fc1 = None
    assert f(*args(w=wn)) == fb.FASTVAR_EINVAL
    assert f(*args(k=0)) == fb.FASTVAR_OK      # empty kept set: nothing to do, nothing launched
    # restore
    g = L.fastvar_restore
    assert g(None, None, None, 1, 0, None, 2, 2, 4, 4, 64, P, None, 0, None) == fb.FASTVAR_EINVAL
    assert g(None, None, None, 1, 2, P, 2, 2, 4, 4, 64, P + 4096, None, 0, None) == fb.FASTVAR_EINVAL
    assert g(None, None, None, 1, 0, P, 2, 2, 4, 4, 64, P, None, 0, None) == fb.FASTVAR_EINVAL   # aliasing
    assert g(None, None, None, 1, 0, P, 2, 2, 4, 4, 62, P + 4096, None, 0, None) == fb.FASTVAR_EALIGN
    assert g(P, P, None, 1, 2, P + 4096, 2, 2, 4, 4, 64, P + 8192, None, 0, None) == fb.FASTVAR_EWORKSPACE
    # step
    sh = (C.c_int32 * 3)(2, 4, 8)
    kv = C.c_int32(20)
    h = L.fastvar_step
    base = lambda **o: [P, sh, sh, 3, o.get("step", 2), o.get("cstep", 1), 1, o.get("k", 8), C.byref(d),
                        C.byref(w), P, P, C.byref(kv), o.get("L_cap", 64), P + 4096, o.get("y", P + 8192), P,
                        o.get("ws", P), o.get("nb", big), None]
    assert h(*base(step=3)) == fb.FASTVAR_EINVAL
    assert h(*base(cstep=2)) == fb.FASTVAR_EINVAL
    assert h(*base(k=65)) == fb.FASTVAR_EINVAL
    assert h(*base(L_cap=24)) == fb.FASTVAR_ECAPACITY
    assert h(*base(nb=1024)) == fb.FASTVAR_EWORKSPACE
    assert h(*base(y=P)) == fb.FASTVAR_EINVAL
    assert kv.value == 20                      # cache length untouched on error


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(fb, "_lib", None)
    monkeypatch.setattr(fb, "LIB_PATH", "/nonexistent/libfastvar.so")
    with pytest.raises(RuntimeError, match="no CPU or PyTorch fallback"):
        fb.lib()

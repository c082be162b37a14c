"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and turns invalid arguments into status codes before anything is launched."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "jp_obrs.h")

obrs = pytest.importorskip("paper_2602_06107_amd.obrs", reason="HIP library not built")


def _declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(jp_[a-z_0-9]+)\s*\(", src)))


def test_every_declared_symbol_is_exported():
    names = _declared_functions()
    assert {"jp_obrs_forward", "jp_obrs_rows", "jp_obrs_finalize", "jp_obrs_workspace_bytes",
            "jp_obrs_forward_lmhead", "jp_obrs_lmhead_workspace_bytes",
            "jp_status_string", "jp_obrs_abi_version"} <= set(names)
    lib = obrs.raw()
    for n in names:
        assert hasattr(lib, n), n
    assert set(obrs.EXPORTS) == set(names)
    assert obrs.jp_obrs_abi_version() == 9


def test_struct_layouts_match_header():
    assert C.sizeof(obrs.Params) == 32
    assert C.sizeof(obrs.Stats) == 72
    assert C.sizeof(obrs.Outputs) == 16 * C.sizeof(C.c_void_p)


def test_workspace_bytes():
    f = obrs.jp_obrs_workspace_bytes
    assert f(0, 1024, 4, obrs.JP_F32) > 0
    assert f(8192, 151936, 64, obrs.JP_BF16) >= 8192 * (7 * 4 + 2 * 8 + 2)
    assert f(8192, 151936, 64, obrs.JP_BF16) < 8192 * 64
    assert f(-1, 10, 1, obrs.JP_F32) == 0 and f(4, 0, 1, obrs.JP_F32) == 0 and f(4, 10, 1, 7) == 0


A0, P0, X0 = 0x10000, 0x20000, 0x30000


def _call(actor=0x10000, policy=0x20000, T=4, V=1024, stride=1024, dt=None, ids=0x30000, uni=0x40000,
          ref=None, lam=1.0, k=8, c1=3.0, c2=3.0, flags=0, ws=0x100000, ws_bytes=1 << 20, out=None,
          prm_null=False, f_mode=0, f_lo=0.0, f_hi=0.0):
    """Calls jp_obrs_forward with fake (never dereferenced) device addresses: every case below must
    be rejected by host-side validation, so nothing is launched."""
    lib = obrs.raw()
    dt = obrs.JP_F32 if dt is None else dt
    prm = obrs.Params(lam, k, c1, c2, flags, f_mode, f_lo, f_hi)
    o = obrs.Outputs() if out is None else out
    return lib.jp_obrs_forward(actor, policy, T, V, stride, dt, ids, uni, ref,
                               None if prm_null else C.byref(prm), C.byref(o), ws, ws_bytes, None)


@pytest.mark.parametrize("kw,want", [
    (dict(actor=None), obrs.JP_ERR_NULL),
    (dict(policy=None), obrs.JP_ERR_NULL),
    (dict(ids=None), obrs.JP_ERR_NULL),
    (dict(prm_null=True), obrs.JP_ERR_NULL),
    (dict(T=-1), obrs.JP_ERR_SHAPE),
    (dict(V=0), obrs.JP_ERR_SHAPE),
    (dict(stride=1000), obrs.JP_ERR_SHAPE),
    (dict(T=1 << 31), obrs.JP_ERR_SHAPE),
    (dict(dt=5), obrs.JP_ERR_UNSUPPORTED),
    (dict(flags=64), obrs.JP_ERR_UNSUPPORTED),
    (dict(lam=0.0), obrs.JP_ERR_PARAM),
    (dict(lam=-1.0), obrs.JP_ERR_PARAM),
    (dict(lam=float("nan")), obrs.JP_ERR_PARAM),
    (dict(lam=float("inf")), obrs.JP_ERR_PARAM),
    (dict(c1=0.0), obrs.JP_ERR_PARAM),
    (dict(c2=float("nan")), obrs.JP_ERR_PARAM),
    (dict(f_mode=3), obrs.JP_ERR_UNSUPPORTED),
    (dict(f_mode=2, f_lo=2.0, f_hi=1.0), obrs.JP_ERR_PARAM),
    (dict(f_mode=2, f_lo=-1.0, f_hi=1.0), obrs.JP_ERR_PARAM),
    (dict(k=0), obrs.JP_ERR_PARAM),
    (dict(k=2000), obrs.JP_ERR_PARAM),             # k > V
    (dict(k=257), obrs.JP_ERR_UNSUPPORTED),        # k > JP_K_MAX
    (dict(actor=0x10004), obrs.JP_ERR_ALIGN),
    (dict(policy=0x20008), obrs.JP_ERR_ALIGN),
    (dict(V=1022, stride=1022), obrs.JP_ERR_ALIGN),   # fp32 row pitch 4088 B
    (dict(dt=1, V=1020, stride=1020), obrs.JP_ERR_ALIGN),  # bf16 row pitch 2040 B
    (dict(ws=None), obrs.JP_ERR_WORKSPACE),
    (dict(ws_bytes=16), obrs.JP_ERR_WORKSPACE),
    (dict(ws=0x100010), obrs.JP_ERR_ALIGN),
])
def test_invalid_arguments_are_rejected_before_launch(kw, want):
    assert _call(**kw) == want


def _call_static(actor=A0, policy=P0, T=4, V=1024, stride=1024, dt=0, ids=X0, lam=1.0, k=8, prm_null=False):
    lib = obrs.raw()
    prm = obrs.Params(lam, k, 3.0, 3.0, 0, 0, 0.0, 0.0)
    o = obrs.Outputs()
    return lib.jp_obrs_forward_static(actor, policy, T, V, stride, dt, ids, None, None,
                                      None if prm_null else C.byref(prm), C.byref(o), None)


@pytest.mark.parametrize("kw,want", [
    (dict(T=obrs.JP_STATIC_MAX_T + 1), obrs.JP_ERR_TOO_LARGE),      # beyond the static scratch: a status of its own
    (dict(T=1 << 40), obrs.JP_ERR_TOO_LARGE),
    (dict(T=-1), obrs.JP_ERR_SHAPE),
    (dict(prm_null=True), obrs.JP_ERR_NULL),
    (dict(actor=None), obrs.JP_ERR_NULL),
    (dict(V=0), obrs.JP_ERR_SHAPE),
    (dict(k=0), obrs.JP_ERR_PARAM),
    (dict(k=257), obrs.JP_ERR_UNSUPPORTED),
    (dict(lam=0.0), obrs.JP_ERR_PARAM),
    (dict(policy=0x20008), obrs.JP_ERR_ALIGN),
    (dict(dt=1, V=1020, stride=1020), obrs.JP_ERR_ALIGN),
])
def test_static_scratch_entry_point_rejects_before_touching_the_gpu(kw, want):
    """Every argument error of jp_obrs_forward_static comes back before its scratch is looked up,
    so these calls work (and launch nothing) on a machine without a GPU."""
    assert _call_static(**kw) == want
    assert "static scratch" in obrs.jp_status_string(obrs.JP_ERR_TOO_LARGE)


def test_status_strings():
    seen = set()
    for s in range(9):
        msg = obrs.jp_status_string(s)
        assert msg and msg not in seen
        seen.add(msg)
    assert obrs.jp_status_string(99) == "unknown status"


# ---- the other entry points: everything below is rejected by host-side validation (fake device
# addresses, never dereferenced), so nothing is launched ------------------------------------------------

A_, P_, X_, U_, O_, W_ = 0x10000, 0x20000, 0x30000, 0x40000, 0x50000, 0x100000


def test_workspace_queries_of_the_other_entry_points():
    base = obrs.jp_obrs_workspace_bytes(64, 1024, 8, obrs.JP_F32)
    assert obrs.jp_obrs_forward3_workspace_bytes(64, 1024, 8, obrs.JP_F32) == base + 256
    assert obrs.jp_obrs_forward3_workspace_bytes(-1, 1024, 8, obrs.JP_F32) == 0
    assert obrs.raw().jp_obrs_budget_scratch_bytes() >= 1088
    lm = obrs.jp_obrs_lmhead_workspace_bytes
    assert lm(256, 8192, 128, 256, 8, 4096) > base
    assert lm(256, 8192, 128, 256, 8, 4096) >= 2 * 256 * 8192 * 4          # two logit buffers of two chunks
    assert lm(256, 8192, 100, 256, 8, 4096) == 0                            # d not a multiple of 64
    assert lm(256, 8192, 128, 256, 0, 4096) == 0


@pytest.mark.parametrize("kw,want", [
    (dict(), None),                                          # baseline of this table: only the workspace is wrong
    (dict(tail=3), obrs.JP_ERR_PARAM),
    (dict(flags=obrs.JP_FLAG_EXACT_Z), obrs.JP_ERR_UNSUPPORTED),
    (dict(flags=obrs.JP_FLAG_DISTILL_KL), obrs.JP_ERR_UNSUPPORTED),
    (dict(ids_q=None), obrs.JP_ERR_NULL),
    (dict(policy=P_ + 2), obrs.JP_ERR_ALIGN),
    (dict(k=0), obrs.JP_ERR_PARAM),
])
def test_forward_stored_rejections(kw, want):
    a = dict(policy=P_, ids_q=0x60000, lq=0x70000, lqx=0x80000, k=8, flags=0, tail=1, ws_bytes=1 << 20)
    a.update(kw)
    prm = obrs.Params(1.0, a["k"], 3.0, 3.0, a["flags"])
    out = obrs.Outputs()
    st = obrs.raw().jp_obrs_forward_stored(a["policy"], 4, 1024, 1024, obrs.JP_F32, a["ids_q"], a["lq"], a["lqx"],
                                           X_, U_, None, C.byref(prm), a["tail"], C.byref(out), W_,
                                           16 if want is None else a["ws_bytes"], None)
    assert st == (obrs.JP_ERR_WORKSPACE if want is None else want)


def test_distill_grad_token_logprob_and_budget_rejections():
    lib = obrs.raw()
    g = lambda **k: lib.jp_obrs_distill_grad(k.get("actor", A_), P_, 4, 1024, 1024, obrs.JP_F32, None,
                                             C.c_float(k.get("scale", 1.0)), k.get("grad", O_), k.get("gs", 1024),
                                             k.get("gdt", obrs.JP_BF16), W_, k.get("wsb", 16), None)
    assert g() == obrs.JP_ERR_WORKSPACE
    assert g(grad=None) == obrs.JP_ERR_NULL
    assert g(grad=O_ + 8) == obrs.JP_ERR_ALIGN
    assert g(gs=1000) == obrs.JP_ERR_SHAPE
    assert g(gdt=4) == obrs.JP_ERR_UNSUPPORTED
    assert g(scale=float("inf")) == obrs.JP_ERR_PARAM
    t = lambda **k: lib.jp_obrs_token_logprob(k.get("logits", P_), k.get("T", 4), k.get("V", 1024), k.get("stride", 1024),
                                              k.get("dt", obrs.JP_F32), k.get("ids", X_), k.get("out", O_), None)
    assert t(T=0) == obrs.JP_OK                               # nothing to do, nothing launched
    assert t(out=None) == obrs.JP_ERR_NULL
    assert t(logits=P_ + 4) == obrs.JP_ERR_ALIGN
    assert t(stride=1000) == obrs.JP_ERR_SHAPE
    assert t(dt=3) == obrs.JP_ERR_UNSUPPORTED
    b = lambda **k: lib.jp_obrs_lambda_for_budget(A_, P_, 4, 1024, 1024, obrs.JP_F32, k.get("rt", None),
                                                  C.c_float(k.get("target", 0.5)), k.get("out", O_), W_,
                                                  k.get("wsb", 16), None)
    assert b() == obrs.JP_ERR_WORKSPACE
    assert b(target=0.0) == obrs.JP_ERR_PARAM and b(target=1.5) == obrs.JP_ERR_PARAM
    assert b(target=0.0, rt=0x90000) == obrs.JP_ERR_WORKSPACE  # per-row budgets are checked on the device
    assert b(out=None) == obrs.JP_ERR_NULL
    bb = lambda **k: lib.jp_obrs_lambda_for_budget_batch(A_, P_, 4, 1024, 1024, obrs.JP_F32, C.c_float(k.get("target", 0.5)),
                                                         k.get("out", O_), W_, k.get("wsb", 1 << 20),
                                                         k.get("scratch", 0xA0000), k.get("sb", 16), None)
    assert bb() == obrs.JP_ERR_WORKSPACE                      # scratch too small
    assert bb(out=None) == obrs.JP_ERR_NULL
    assert bb(target=2.0) == obrs.JP_ERR_PARAM
    assert bb(scratch=None, sb=4096) == obrs.JP_ERR_WORKSPACE


def test_forward3_rejections():
    lib = obrs.raw()
    prm = obrs.Params(1.0, 8, 3.0, 3.0, 0)
    out = obrs.Outputs()
    f = lambda **k: lib.jp_obrs_forward3(A_, k.get("new", P_), k.get("ref", 0x60000), k.get("tir", 0), 4, 1024, 1024,
                                         obrs.JP_F32, X_, U_, C.byref(prm), C.byref(out), W_, k.get("wsb", 16), None)
    assert f() == obrs.JP_ERR_WORKSPACE
    assert f(ref=None) == obrs.JP_ERR_NULL
    assert f(new=None, wsb=1 << 20) == obrs.JP_ERR_NULL       # the new policy is needed when it is the target
    assert f(tir=1, new=None) == obrs.JP_ERR_WORKSPACE        # ... and is not read when p_ref is the target


def test_lmhead_stored_rejections_need_no_gpu():
    """jp_obrs_forward_lmhead_stored with fake (never dereferenced) device addresses: rejected by
    host-side validation, nothing is launched."""
    lib = obrs.raw()
    need = obrs.jp_obrs_lmhead_stored_workspace_bytes(4, 1024, 64, 8, 0)
    assert need > obrs.jp_obrs_workspace_bytes(4, 1024, 8, obrs.JP_F32)
    assert need < obrs.jp_obrs_lmhead_workspace_bytes(4, 1024, 64, 64, 8, 0)      # one head, one logit buffer
    assert obrs.jp_obrs_lmhead_stored_workspace_bytes(4, 1024, 60, 8, 0) == 0     # d not a multiple of 64
    assert obrs.jp_obrs_lmhead_workspace_bytes(4, 1024, 0, 64, 8, 0) == 0          # the two-head form needs both heads

    def call(H=0x10000, d=64, W=0x20000, T=4, V=1024, ids=0x30000, lq=0x40000, lqx=0x50000, x=0x60000, k=8,
             lam=1.0, flags=0, rule=1, ws=0x100000, ws_bytes=need):
        prm = obrs.Params(lam, k, 3.0, 3.0, flags, 0, 0.0, 0.0)
        o = obrs.Outputs()
        return lib.jp_obrs_forward_lmhead_stored(H, d, W, T, V, 0, ids, lq, lqx, x, None, None, C.byref(prm), rule,
                                                 C.byref(o), ws, ws_bytes, None)

    assert call(H=None) == obrs.JP_ERR_NULL
    assert call(ids=None) == obrs.JP_ERR_NULL
    assert call(lqx=None) == obrs.JP_ERR_NULL
    assert call(d=60) == obrs.JP_ERR_SHAPE
    assert call(V=0) == obrs.JP_ERR_SHAPE
    assert call(k=0) == obrs.JP_ERR_PARAM
    assert call(k=2000) == obrs.JP_ERR_PARAM                   # k > V
    assert call(lam=0.0) == obrs.JP_ERR_PARAM
    assert call(rule=5) == obrs.JP_ERR_PARAM
    assert call(flags=obrs.JP_FLAG_EXACT_Z) == obrs.JP_ERR_UNSUPPORTED
    assert call(flags=obrs.JP_FLAG_DISTILL_KL) == obrs.JP_ERR_UNSUPPORTED
    assert call(H=0x10008) == obrs.JP_ERR_ALIGN
    assert call(W=0x20001) == obrs.JP_ERR_ALIGN
    assert call(W=0x20008, flags=obrs.JP_FLAG_W_VOCAB_MAJOR) == obrs.JP_ERR_ALIGN
    assert call(ws_bytes=need - 1) == obrs.JP_ERR_WORKSPACE
    assert call(ws=0x100010) == obrs.JP_ERR_ALIGN

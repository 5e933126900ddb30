"""CPU-side checks of the C ABI: the library loads, exports what include/pskv.h declares,
and rejects bad problems on the host before anything could be launched."""
import ctypes
import os
import re

import pytest

from paper_2603_13420_amd import binding as pk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "pskv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pskv_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = pk.load()
    names = declared_functions()
    assert set(names) == set(pk.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n
    assert pk.pskv_version() >= 100
    for s in range(5):
        assert pk.pskv_status_str(s) not in ("", "unknown status")


def test_params_struct_matches_header_layout():
    # 10 four-byte fields then 11 eight-byte strides, no padding surprises
    assert ctypes.sizeof(pk.pskv_attn_params) == 10 * 4 + 11 * 8
    assert pk.pskv_attn_params.q_stride_b.offset == 40


def ok(**kw):
    base = dict(B=8, S=16, P=48, Hq=4, Hkv=4, D=64, dtype="f32")
    base.update(kw)
    return pk.make_params(**base)


def test_valid_problems_pass_on_host():
    assert pk.pskv_attn_validate(ok()) == pk.PSKV_OK
    assert pk.pskv_attn_fwd_workspace_bytes(ok()) == 0
    assert pk.pskv_attn_validate(ok(P=0)) == pk.PSKV_OK
    assert pk.pskv_attn_validate(ok(B=1024, S=24, P=256, Hq=32, Hkv=8, D=128, dtype="bf16")) == pk.PSKV_OK
    assert pk.pskv_attn_validate(ok(Hq=28, Hkv=4, D=128, dtype="bf16")) == pk.PSKV_OK
    assert pk.pskv_attn_validate(ok(D=128, dtype="bf16", impl="mfma")) == pk.PSKV_OK


@pytest.mark.parametrize("kw,status,needle", [
    (dict(B=0), pk.PSKV_ERR_INVALID_ARG, "sizes"),
    (dict(S=0), pk.PSKV_ERR_INVALID_ARG, "sizes"),
    (dict(P=-1), pk.PSKV_ERR_INVALID_ARG, "sizes"),
    (dict(Hq=6, Hkv=4), pk.PSKV_ERR_INVALID_ARG, "multiple"),
    (dict(D=66), pk.PSKV_ERR_UNSUPPORTED, "16-byte"),
    (dict(D=512), pk.PSKV_ERR_UNSUPPORTED, "maximum"),
    (dict(q_stride_h=-64), pk.PSKV_ERR_INVALID_ARG, "negative"),
    (dict(q_stride_h=66), pk.PSKV_ERR_INVALID_ARG, "16 bytes"),
    (dict(o_stride_s=32), pk.PSKV_ERR_INVALID_ARG, "overlap"),
    (dict(scale=float("nan")), pk.PSKV_ERR_INVALID_ARG, "finite"),
    (dict(impl="mfma"), pk.PSKV_ERR_UNSUPPORTED, "MFMA"),              # f32 has no MFMA path
    (dict(D=64, dtype="bf16", impl="mfma"), pk.PSKV_ERR_UNSUPPORTED, "MFMA"),
    (dict(P=40000, impl="simple"), pk.PSKV_ERR_UNSUPPORTED, "LDS"),
])
def test_bad_problems_are_refused_with_a_reason(kw, status, needle):
    p = ok(**kw)
    assert pk.pskv_attn_validate(p) == status
    assert needle in pk.pskv_last_error()
    with pytest.raises(pk.PskvError):
        pk.pskv_attn_fwd_workspace_bytes(p)


def test_unknown_enums_and_reserved():
    p = ok()
    p.dtype = 7
    assert pk.pskv_attn_validate(p) == pk.PSKV_ERR_INVALID_ARG
    p = ok()
    p.impl = 9
    assert pk.pskv_attn_validate(p) == pk.PSKV_ERR_INVALID_ARG
    p = ok()
    p.reserved = 1
    assert pk.pskv_attn_validate(p) == pk.PSKV_ERR_INVALID_ARG
    assert pk.load().pskv_attn_validate(None) == pk.PSKV_ERR_INVALID_ARG


def test_fwd_refuses_null_and_misaligned_pointers_before_any_launch():
    """Pointer checks run on the host before the first HIP call, so they are testable here."""
    lib = pk.load()
    p = ok()
    null = ctypes.c_void_p(0)
    a = ctypes.c_void_p(0x1000)
    rc = lib.pskv_attn_fwd(ctypes.byref(p), null, a, a, a, a, None, a, None, None, 0, None)
    assert rc == pk.PSKV_ERR_INVALID_ARG and "NULL" in pk.pskv_last_error()
    rc = lib.pskv_attn_fwd(ctypes.byref(p), a, a, a, null, a, None, ctypes.c_void_p(0x2000), None, None, 0, None)
    assert rc == pk.PSKV_ERR_INVALID_ARG and "k_pre" in pk.pskv_last_error()
    rc = lib.pskv_attn_fwd(ctypes.byref(p), ctypes.c_void_p(0x1008), a, a, a, a, None,
                           ctypes.c_void_p(0x2000), None, None, 0, None)
    assert rc == pk.PSKV_ERR_INVALID_ARG and "aligned" in pk.pskv_last_error()
    rc = lib.pskv_attn_fwd(ctypes.byref(p), a, a, a, a, a, None, a, None, None, 0, None)
    assert rc == pk.PSKV_ERR_INVALID_ARG and "alias" in pk.pskv_last_error()
    # overlap is judged on address ranges, not on first bytes: out starting inside q, q starting inside out
    big = 1 << 40
    q_bytes = p.B * p.S * p.Hq * p.D * 4
    for q_at, out_at in ((big, big + 256), (big + q_bytes - 16, big)):
        rc = lib.pskv_attn_fwd(ctypes.byref(p), ctypes.c_void_p(q_at), a, a, a, a, None, ctypes.c_void_p(out_at), None,
                               None, 0, None)
        assert rc == pk.PSKV_ERR_INVALID_ARG and "out overlaps q" in pk.pskv_last_error()
    # lse inside an input
    rc = lib.pskv_attn_fwd(ctypes.byref(p), ctypes.c_void_p(big), a, a, a, a, None, ctypes.c_void_p(2 * big),
                           ctypes.c_void_p(big + 64), None, 0, None)
    assert rc == pk.PSKV_ERR_INVALID_ARG and "lse overlaps q" in pk.pskv_last_error()


def test_bwd_refuses_bad_pointers_before_any_launch():
    """Both backward entry points check their pointers on the host before the first HIP call."""
    lib = pk.load()
    p = ok(dtype="bf16", D=128)
    a, b, c, d_ = (ctypes.c_void_p(x) for x in (0x1000, 0x2000, 0x3000, 0x4000))
    out, lse, dout = ctypes.c_void_p(0x5000), ctypes.c_void_p(0x6000), ctypes.c_void_p(0x7000)
    # lse is required
    rc = lib.pskv_attn_bwd(ctypes.byref(p), a, a, a, a, a, None, out, None, dout, b, c, d_, None, 0, None)
    assert rc == pk.PSKV_ERR_INVALID_ARG and "NULL" in pk.pskv_last_error()
    # a gradient output may not be an input, nor another gradient output
    rc = lib.pskv_attn_bwd(ctypes.byref(p), a, a, a, a, a, None, out, lse, dout, a, c, d_, None, 0, None)
    assert rc == pk.PSKV_ERR_INVALID_ARG and "alias" in pk.pskv_last_error()
    rc = lib.pskv_attn_bwd(ctypes.byref(p), a, a, a, a, a, None, out, lse, dout, b, b, d_, None, 0, None)
    assert rc == pk.PSKV_ERR_INVALID_ARG and "alias" in pk.pskv_last_error()
    rc = lib.pskv_attn_bwd(ctypes.byref(p), a, a, a, a, a, None, out, lse, ctypes.c_void_p(0x7004), b, c, d_, None, 0,
                           None)
    assert rc == pk.PSKV_ERR_INVALID_ARG and "aligned" in pk.pskv_last_error()
    m = pk.pskv_multi_params()
    m.base = p
    m.Np = 2
    m.reserved = 0
    m.kp_stride_n = 0
    rc = lib.pskv_attn_bwd_multi(ctypes.byref(m), a, a, a, a, a, None, None, out, None, dout, b, c, d_, None, 0, None)
    assert rc == pk.PSKV_ERR_INVALID_ARG and "NULL" in pk.pskv_last_error()
    m.reserved = 1
    rc = lib.pskv_attn_bwd_multi(ctypes.byref(m), a, a, a, a, a, None, None, out, lse, dout, b, c, d_, None, 0, None)
    assert rc == pk.PSKV_ERR_INVALID_ARG and "reserved" in pk.pskv_last_error()
    rc = lib.pskv_attn_bwd_multi(None, a, a, a, a, a, None, None, out, lse, dout, b, c, d_, None, 0, None)
    assert rc == pk.PSKV_ERR_INVALID_ARG


def test_bwd_refuses_a_workspace_inside_a_tensor_and_noalloc_refuses_what_its_scratch_cannot_hold():
    lib = pk.load()
    p = ok(dtype="bf16", D=128)
    g = 1 << 36
    q, ks, vs, kp, vp, out, lse, dout, dq, dk, dv = (ctypes.c_void_p(g * i) for i in range(1, 12))
    need = lib.pskv_attn_bwd_workspace_bytes(ctypes.byref(p))
    rc = lib.pskv_attn_bwd(ctypes.byref(p), q, ks, vs, kp, vp, None, out, lse, dout, dq, dk, dv,
                           ctypes.c_void_p(g * 11 + 4096), need, None)       # inside dv
    assert rc == pk.PSKV_ERR_WORKSPACE and "workspace overlaps dv_suf" in pk.pskv_last_error()
    rc = lib.pskv_attn_bwd(ctypes.byref(p), q, ks, vs, kp, vp, None, out, lse, dout, dq, dk, dv,
                           ctypes.c_void_p(g * 12 + 8), need, None)
    assert rc == pk.PSKV_ERR_WORKSPACE and "aligned" in pk.pskv_last_error()
    # column slices of one fused [B,S,(Hq+2Hkv),D] gradient buffer interleave without sharing a byte and are
    # accepted (GPU tests run them); slices whose per-token spans run into each other are not
    fused = ok(dtype="bf16", D=128, Hq=4, Hkv=2, q_stride_s=8 * 128, q_stride_b=16 * 8 * 128,
               ks_stride_s=8 * 128, ks_stride_b=16 * 8 * 128)
    base = 13 * g
    dq_f, dk_f, dv_f = (ctypes.c_void_p(base + off * 128 * 2) for off in (0, 3, 6))   # dk starts inside dq's 4 heads
    rc = lib.pskv_attn_bwd(ctypes.byref(fused), q, ks, vs, kp, vp, None, out, lse, dout, dq_f, dk_f, dv_f, None, 0, None)
    assert rc == pk.PSKV_ERR_INVALID_ARG and "dq overlaps dk_suf" in pk.pskv_last_error()
    # the entry point that allocates nothing: B*Hq*S*4 beyond its built-in scratch is refused on the host
    huge = ok(B=4096, S=64, P=512, Hq=40, Hkv=40, D=128, dtype="bf16")
    assert 4096 * 40 * 64 * 4 > pk.PSKV_NOALLOC_SCRATCH_BYTES
    rc = lib.pskv_attn_bwd_noalloc(ctypes.byref(huge), q, ks, vs, kp, vp, None, out, lse, dout, dq, dk, dv, None)
    assert rc == pk.PSKV_ERR_WORKSPACE and "exceed" in pk.pskv_last_error()
    rc = lib.pskv_attn_bwd_noalloc(None, q, ks, vs, kp, vp, None, out, lse, dout, dq, dk, dv, None)
    assert rc == pk.PSKV_ERR_INVALID_ARG
    header = open(os.path.join(ROOT, "include", "pskv.h")).read()
    assert "#define PSKV_NOALLOC_SCRATCH_BYTES (8u << 20)" in header


def test_binding_refuses_expanded_views():
    """The ABI reads stride 0 as "contiguous": a broadcast view must be refused, not read as dense."""
    import torch
    q = torch.zeros(4, 8, 4, 128, dtype=torch.bfloat16)
    ks = torch.zeros(4, 8, 2, 128, dtype=torch.bfloat16)
    kp = torch.zeros(16, 2, 128, dtype=torch.bfloat16)
    pk._params_from_tensors(q, ks, kp, q.clone(), "auto", 0.0)              # dense tensors are fine
    with pytest.raises(ValueError, match="stride 0"):
        pk._params_from_tensors(q[:1].expand(4, 8, 4, 128), ks, kp, q.clone(), "auto", 0.0)
    with pytest.raises(ValueError, match="stride 0"):
        pk._params_from_tensors(q, ks[:1].expand(4, 8, 2, 128), kp, q.clone(), "auto", 0.0)
    with pytest.raises(ValueError, match="stride 0"):                       # one prefix broadcast over the instructions
        kpm = kp[None].expand(2, 16, 2, 128)
        pk.make_multi_params(pk._params_from_tensors(q, ks, kpm[0], q.clone(), "auto", 0.0), 2, pk._stride(kpm, 0, "k_pre"))
    # a dimension of size 1 has no stride to speak of: whatever torch reports for it is not passed on
    one = pk._params_from_tensors(q[:1], ks[:1], kp, q[:1].clone(), "auto", 0.0)
    assert one.q_stride_b == 0 and one.B == 1


def test_bwd_workspace_size():
    lib = pk.load()
    p = ok(B=7, S=24, Hq=32, Hkv=8, D=128, dtype="bf16")
    assert lib.pskv_attn_bwd_workspace_bytes(ctypes.byref(p)) == 7 * 32 * 24 * 4
    p.D = 0
    assert lib.pskv_attn_bwd_workspace_bytes(ctypes.byref(p)) == ctypes.c_size_t(-1).value


def test_multi_params_layout_and_host_validation():
    """The multi-instruction struct is the single-prefix struct plus three fields; its rules are
    checked on the host: B a multiple of Np, Np >= 1, reserved 0, a prefix stride that holds a prefix."""
    assert ctypes.sizeof(pk.pskv_multi_params) == ctypes.sizeof(pk.pskv_attn_params) + 16
    assert pk.pskv_multi_params.Np.offset == ctypes.sizeof(pk.pskv_attn_params)
    base = ok(B=8, dtype="bf16", D=128)
    assert pk.pskv_attn_multi_validate(pk.make_multi_params(base, 4)) == pk.PSKV_OK
    assert pk.pskv_attn_multi_validate(pk.make_multi_params(base, 1)) == pk.PSKV_OK
    for np_, stride, needle in ((3, 0, "multiple of Np"), (0, 0, "at least 1"), (-2, 0, "at least 1"),
                                (2, 48 * 4 * 128 - 8, "smaller than one prefix"), (2, 12345, "16 bytes"),
                                (2, -8, "negative")):
        st = pk.pskv_attn_multi_validate(pk.make_multi_params(base, np_, stride))
        assert st == pk.PSKV_ERR_INVALID_ARG and needle in pk.pskv_last_error(), (np_, stride, pk.pskv_last_error())
    p = pk.make_multi_params(base, 2, 48 * 4 * 128 + 64)
    assert pk.pskv_attn_multi_validate(p) == pk.PSKV_OK
    p.reserved = 1
    assert pk.pskv_attn_multi_validate(p) == pk.PSKV_ERR_INVALID_ARG
    # a forward call with bad arguments is refused before anything could be launched
    lib = pk.load()
    rc = lib.pskv_attn_fwd_multi(ctypes.byref(pk.make_multi_params(base, 4)), None, None, None, None, None, None,
                                 None, None, None, None, 0, None)
    assert rc == pk.PSKV_ERR_INVALID_ARG and "must not be NULL" in pk.pskv_last_error()
    rc = lib.pskv_attn_fwd_multi(None, None, None, None, None, None, None, None, None, None, None, 0, None)
    assert rc == pk.PSKV_ERR_INVALID_ARG


def test_product_path_does_not_import_the_oracle():
    """No file of the package imports, links or loads anything of the CPU oracle."""
    pkg = os.path.join(ROOT, "paper_2603_13420_amd")
    pat = re.compile(r"(import\s+oracle|from\s+oracle|pskv_oracle|oracle/|oracle\.)")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert not pat.search(src), f

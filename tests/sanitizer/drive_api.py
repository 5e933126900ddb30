"""Run inside a process that has the AddressSanitizer runtime preloaded: loads the sanitizer build of
the C ABI's host side and walks through its validation paths (good and bad params, null, misaligned
and overlapping pointers, the multi-instruction and backward entry points, the error strings).  Any
finding of the sanitizers aborts the process."""
import ctypes
import sys

sys.path.insert(0, sys.argv[2])
from paper_2603_13420_amd import binding as pk  # noqa: E402  (struct layouts only; its library is not loaded)

lib = ctypes.CDLL(sys.argv[1])
lib.pskv_last_error.restype = ctypes.c_char_p
lib.pskv_status_str.restype = ctypes.c_char_p
lib.pskv_attn_fwd_workspace_bytes.restype = ctypes.c_size_t
lib.pskv_attn_bwd_workspace_bytes.restype = ctypes.c_size_t
vp = ctypes.c_void_p
P = ctypes.POINTER(pk.pskv_attn_params)
PM = ctypes.POINTER(pk.pskv_multi_params)
lib.pskv_attn_validate.argtypes = [P]
lib.pskv_attn_fwd_workspace_bytes.argtypes = [P]
lib.pskv_attn_bwd_workspace_bytes.argtypes = [P]
lib.pskv_attn_multi_validate.argtypes = [PM]
lib.pskv_attn_fwd.argtypes = [P] + [vp] * 9 + [ctypes.c_size_t, vp]
lib.pskv_attn_fwd_multi.argtypes = [PM] + [vp] * 10 + [ctypes.c_size_t, vp]
lib.pskv_attn_bwd.argtypes = [P] + [vp] * 13 + [ctypes.c_size_t, vp]
lib.pskv_attn_bwd_multi.argtypes = [PM] + [vp] * 14 + [ctypes.c_size_t, vp]
lib.pskv_attn_bwd_noalloc.argtypes = [P] + [vp] * 13

calls = 0
g = 1 << 36
ptrs = [vp(g * i) for i in range(1, 13)]
for kw in (dict(), dict(P=0), dict(B=0), dict(S=-3), dict(Hq=6, Hkv=4), dict(D=66), dict(D=512), dict(q_stride_h=-64),
           dict(q_stride_h=66), dict(o_stride_s=32), dict(scale=float("nan")), dict(impl="mfma"),
           dict(D=128, dtype="bf16"), dict(D=128, dtype="bf16", impl="mfma"), dict(P=40000, impl="simple"),
           dict(B=2 ** 20, S=2 ** 10, Hq=64, Hkv=64, D=128, dtype="bf16"),
           dict(B=1024, S=24, P=256, Hq=32, Hkv=8, D=128, dtype="bf16", q_stride_s=48 * 128, q_stride_b=24 * 48 * 128)):
    base = dict(B=8, S=16, P=48, Hq=4, Hkv=4, D=64, dtype="f32")
    base.update(kw)
    p = pk.make_params(**base)
    lib.pskv_attn_validate(ctypes.byref(p))
    lib.pskv_last_error()
    lib.pskv_attn_fwd_workspace_bytes(ctypes.byref(p))
    lib.pskv_attn_bwd_workspace_bytes(ctypes.byref(p))
    q, ks, vs, kp, vpre, out, lse, dout, dq, dk, dv, ws = ptrs
    for args in ((q, ks, vs, kp, vpre, None, out, lse), (None, ks, vs, kp, vpre, None, out, None),
                 (q, ks, vs, kp, vpre, None, q, None), (q, ks, vs, kp, vpre, None, vp(g + 256), None),
                 (vp(g + 8), ks, vs, kp, vpre, None, out, None), (q, ks, vs, None, None, vp(6), out, vp(g * 6 + 2))):
        lib.pskv_attn_fwd(ctypes.byref(p), *args, None, 0, None)
        calls += 1
    for np_, stride in ((1, 0), (2, 0), (3, 0), (0, 0), (2, 12345), (2, -8), (4, 1 << 40)):
        m = pk.make_multi_params(p, np_, stride)
        lib.pskv_attn_multi_validate(ctypes.byref(m))
        lib.pskv_attn_fwd_multi(ctypes.byref(m), q, ks, vs, kp, vpre, None, None, out, lse, None, 0, None)
        lib.pskv_attn_bwd_multi(ctypes.byref(m), q, ks, vs, kp, vpre, None, None, out, lse, dout, dq, dk, dv, ws, 1 << 30, None)
        calls += 2
    for grads, wsp, wsb in (((dq, dk, dv), None, 0), ((dq, dk, dv), ws, 1 << 30), ((q, dk, dv), None, 0), ((dq, dq, dv), None, 0),
                            ((dq, dk, dv), vp(g * 11 + 4096), 1 << 30), ((dq, dk, dv), vp(g * 12 + 8), 1 << 30),
                            ((vp(g * 9), vp(g * 9 + 3 * 256), vp(g * 9 + 6 * 256)), None, 0)):
        lib.pskv_attn_bwd(ctypes.byref(p), q, ks, vs, kp, vpre, None, out, lse, dout, *grads, wsp, wsb, None)
        lib.pskv_attn_bwd_noalloc(ctypes.byref(p), q, ks, vs, kp, vpre, None, out, lse, dout, *grads, None)
        calls += 2
lib.pskv_attn_validate(None)
lib.pskv_attn_multi_validate(None)
lib.pskv_attn_fwd(None, *([None] * 9), 0, None)
for s in range(-1, 7):
    lib.pskv_status_str(s)
print("sanitizer walk done:", calls, "calls")

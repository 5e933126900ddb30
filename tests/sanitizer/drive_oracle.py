"""Run inside a process that has gcc's AddressSanitizer runtime preloaded: loads the sanitizer build of
the C oracle and runs every entry point on small ragged problems (empty candidates, no prefix,
grouped heads, NaN-poisoned padding, lse and weights requested).  Any finding aborts the process."""
import ctypes
import sys

import numpy as np

sys.path.insert(0, sys.argv[2])
import oracle.pskv_oracle as orc  # noqa: E402

orc._LIB = sys.argv[1]
orc.build = lambda force=False: orc._LIB      # the sanitizer build stands in for the regular one
rng = np.random.default_rng(5)
n = 0
for B, P, S, Hq, Hkv, D in ((3, 5, 4, 2, 1, 8), (2, 0, 6, 4, 2, 16), (4, 33, 9, 6, 3, 64), (1, 70, 1, 1, 1, 128)):
    for dtype in ("f64", "f32", "bf16"):
        def draw(*shape):
            a = rng.standard_normal(shape)
            if dtype == "f32":
                return a.astype(np.float32)
            if dtype == "bf16":
                return (a.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
            return a
        q, ks, vs, kp, vpre = draw(B, S, Hq, D), draw(B, S, Hkv, D), draw(B, S, Hkv, D), draw(P, Hkv, D), draw(P, Hkv, D)
        sl = rng.integers(0, S + 1, size=B).astype(np.int32)
        out, lse, probs = orc.attn(q, ks, vs, kp, vpre, sl, 0.3, dtype, want_lse=True, want_probs=True)
        assert np.isfinite(out).all()
        orc.attn(q, ks, vs, kp, vpre, None, 0.3, dtype, nthreads=3)
        do = rng.standard_normal((B, S, Hq, D))
        orc.attn_bwd(q, ks, vs, kp, vpre, sl, do, 0.3, dtype)
        if P > 0:
            kpm, vpm = np.stack([kp, kp]), np.stack([vpre, vpre])
            pl = np.array([P, P // 2], dtype=np.int32)
            q2, ks2, vs2 = np.concatenate([q, q]), np.concatenate([ks, ks]), np.concatenate([vs, vs])
            sl2 = np.concatenate([sl, sl])
            orc.attn_multi(q2, ks2, vs2, kpm, vpm, pl, sl2, 0.3, dtype, want_lse=True, want_probs=True)
            orc.attn_bwd_multi(q2, ks2, vs2, kpm, vpm, pl, sl2, np.concatenate([do, do]), 0.3, dtype)
        n += 1
print("sanitizer walk done:", n, "problems")

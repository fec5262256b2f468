"""The allocation-free entry point (moska_decode_step_static) against moska_decode_step: same
kernels, the workspace in the library's static device array instead of a caller's buffer."""
import pytest
import torch

import paper_2511_06010_amd as moska
from moska_inputs import Problem, generate

pytestmark = pytest.mark.gpu


def _both(p, seed):
    inp = generate(p, seed=seed, unique_len="ragged").to("cuda")
    out = []
    for static in (False, True):
        buf = moska.Buffers(p)
        buf.part_O.fill_(float("nan"))
        buf.part_LSE.fill_(float("nan"))
        args = (p, inp.Q, inp.E, inp.Ks, inp.Vs, inp.scale_k, inp.scale_v, inp.Ku, inp.Vu, inp.unique_len, buf.ids,
                buf.bucket_off, buf.bucket_items, buf.part_O, buf.part_LSE, buf.O, buf.LSE)
        if static:
            moska.decode_step_static(*args)
        else:
            moska.decode_step(*args, buf.ws)
        torch.cuda.synchronize()
        out.append(buf)
    return out


def test_static_scratch_entry_point_matches_decode_step():
    # two calls in a row on the same GPU (they share the static array, which keeps the first call's
    # contents), the second with a smaller problem of another shape and store dtype; the same kernels
    # run, so every output must carry the bits of the existing entry point
    big = Problem(B=48, Hq=16, Hkv=4, D=128, C=24, L=700, k=4, U=500, name="static-first")
    small = Problem(B=5, Hq=8, Hkv=2, D=128, C=6, L=100, k=2, U=40, kv_dtype="fp8", name="static-second")
    assert moska.workspace_bytes(small) < moska.workspace_bytes(big) <= moska.STATIC_SCRATCH_BYTES
    for p, seed in ((big, 51), (small, 52)):
        print(f"case {p.name}: {p}", flush=True)
        want, got = _both(p, seed)
        for name in ("ids", "bucket_off", "bucket_items", "part_O", "part_LSE", "O", "LSE"):
            x, y = getattr(want, name), getattr(got, name)
            assert torch.equal(x.view(torch.uint8), y.view(torch.uint8)), (p.name, name)
        assert torch.isfinite(got.O.float()).all()


def test_static_scratch_entry_point_rejects_large_problems():
    from moska_inputs import config
    p = config(3)                                   # needs 65 MiB of workspace
    assert moska.workspace_bytes(p) > moska.STATIC_SCRATCH_BYTES
    with pytest.raises(moska.MoskaError, match="static scratch"):
        z = torch.zeros(1, device="cuda")
        cp = moska.problem_t(p)
        import ctypes
        ptr = ctypes.c_void_p(z.data_ptr())
        rc = moska.load_library().moska_decode_step_static(ctypes.byref(cp), *([ptr] * 16), None)
        if rc != 0:
            raise moska.MoskaError(moska.load_library().moska_status_string(rc).decode())
